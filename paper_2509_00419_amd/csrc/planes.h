// Token planes ([B, N, row] tensors that share the token axis) as the kernels see them, and the 16 / 4 /
// 2-byte "unit" a thread moves or accumulates.
#pragma once

#include "common.h"

namespace lvlm {

inline int elem_bytes(int dtype) { return dtype == LVLM_BF16 ? 2 : 4; }

struct PlaneDev {
    const char *src;
    char *dst;
    long long src_stride_b, dst_stride_b;   // bytes
    int row_bytes;
    int row_elems;
    int dtype;
    int rule;
    int unit_bytes;   // 16, 4 or 2
    int tpr_log2;     // threads per row (power of two, <= 256)
    int col_blocks;   // blocks of 256 units across a row
    int n_sub;        // row sub-chunks (partial sums) of this plane
};

// Device view of one caller plane: strides in bytes, the widest unit its rows and strides allow, and how
// many threads cover one row.
inline PlaneDev make_plane_dev(const lvlm_plane &pl) {
    PlaneDev p{};
    const int es = elem_bytes(pl.dtype);
    p.src = static_cast<const char *>(pl.src);
    p.dst = static_cast<char *>(pl.dst);
    p.src_stride_b = pl.src_stride_b * es;
    p.dst_stride_b = pl.dst_stride_b * es;
    p.row_elems = pl.row_elems;
    p.row_bytes = pl.row_elems * es;
    p.dtype = pl.dtype;
    p.rule = pl.merge_rule;
    const bool vec = p.row_bytes % 16 == 0 && p.src_stride_b % 16 == 0 && p.dst_stride_b % 16 == 0;
    p.unit_bytes = vec ? 16 : (p.row_bytes % 4 == 0 && p.src_stride_b % 4 == 0 && p.dst_stride_b % 4 == 0 ? 4 : 2);
    const int row_units = p.row_bytes / p.unit_bytes;
    int tl = 0;
    while ((1 << tl) < row_units && tl < 8) ++tl;
    p.tpr_log2 = tl;
    p.col_blocks = (row_units + 255) / 256;
    p.n_sub = 0;
    return p;
}

#if defined(__HIPCC__)
template <int UB>
struct Unit;
template <>
struct Unit<16> { using type = uint4; };
template <>
struct Unit<4> { using type = uint32_t; };
template <>
struct Unit<2> { using type = uint16_t; };

template <int DT, int UB>
struct Acc {
    static constexpr int NE = UB / (DT == LVLM_BF16 ? 2 : 4);
    float v[NE > 0 ? NE : 1];
};

template <int DT, int UB>
__device__ __forceinline__ void accumulate(Acc<DT, UB> &acc, const typename Unit<UB>::type &u, float w) {
    if constexpr (DT == LVLM_BF16 && UB == 16) {
        const uint32_t d[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            acc.v[2 * i] = fmaf(w, __uint_as_float(d[i] << 16), acc.v[2 * i]);
            acc.v[2 * i + 1] = fmaf(w, __uint_as_float(d[i] & 0xffff0000u), acc.v[2 * i + 1]);
        }
    } else if constexpr (DT == LVLM_BF16 && UB == 4) {
        acc.v[0] = fmaf(w, __uint_as_float(u << 16), acc.v[0]);
        acc.v[1] = fmaf(w, __uint_as_float(u & 0xffff0000u), acc.v[1]);
    } else if constexpr (DT == LVLM_BF16 && UB == 2) {
        acc.v[0] = fmaf(w, bf16_to_f32(u), acc.v[0]);
    } else if constexpr (DT == LVLM_F32 && UB == 16) {
        acc.v[0] = fmaf(w, __uint_as_float(u.x), acc.v[0]);
        acc.v[1] = fmaf(w, __uint_as_float(u.y), acc.v[1]);
        acc.v[2] = fmaf(w, __uint_as_float(u.z), acc.v[2]);
        acc.v[3] = fmaf(w, __uint_as_float(u.w), acc.v[3]);
    } else if constexpr (DT == LVLM_F32 && UB == 4) {
        acc.v[0] = fmaf(w, __uint_as_float(u), acc.v[0]);
    }
}

#endif

}  // namespace lvlm
