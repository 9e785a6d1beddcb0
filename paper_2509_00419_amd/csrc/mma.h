// Matrix-core helpers shared by the kernels: operand fragments for the 32x32 MFMA tiles and the
// register <-> (row, column) map of their accumulators.
#pragma once

#include "common.h"

namespace lvlm {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

template <int DT>
__host__ __device__ constexpr int esize() {
    return DT == LVLM_BF16 ? 2 : 4;
}

// The HD/2 contiguous elements one lane contributes to a 32 x 32 x HD product: lane = (row l32 of the
// operand, half hf of the contraction range).  The contraction index of an MFMA is a dummy index, so
// both operands simply use the same split and every lane reads plain 16-byte words.
template <int DT, int HD>
struct HalfRow {
    static constexpr int NV = (HD / 2) * esize<DT>() / 16;
    uint4 v[NV];
};

// acc[32x32] += A[32 x HD] * B[32 x HD]^T ; rows of A map to rows of acc, rows of B to its columns.
template <int DT, int HD>
__device__ __forceinline__ void mma_tile(f32x16 &acc, const HalfRow<DT, HD> &a, const HalfRow<DT, HD> &b) {
    constexpr int NV = HalfRow<DT, HD>::NV;
    if constexpr (DT == LVLM_BF16) {
#pragma unroll
        for (int i = 0; i < NV; ++i)
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a.v[i]),
                                                          __builtin_bit_cast(bf16x8, b.v[i]), acc, 0, 0, 0);
    } else {
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.v[i].x), __uint_as_float(b.v[i].x), acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.v[i].y), __uint_as_float(b.v[i].y), acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.v[i].z), __uint_as_float(b.v[i].z), acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.v[i].w), __uint_as_float(b.v[i].w), acc, 0, 0, 0);
        }
    }
}

// One matrix instruction of such a product: 16-byte words a, b of the two operands (bf16: the whole word,
// contraction length 16; fp32: component comp of the word, contraction length 2).
template <int DT>
__device__ __forceinline__ void mfma_one(f32x16 &acc, const uint4 &a, const uint4 &b, int comp) {
    if constexpr (DT == LVLM_BF16) {
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), acc,
                                                      0, 0, 0);
    } else {
        const unsigned aw = comp == 0 ? a.x : comp == 1 ? a.y : comp == 2 ? a.z : a.w;
        const unsigned bw = comp == 0 ? b.x : comp == 1 ? b.y : comp == 2 ? b.z : b.w;
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(aw), __uint_as_float(bw), acc, 0, 0, 0);
    }
}

// Exchanges with the other half-wave and with the neighbouring 16-lane row (common.h: lane-swap instructions).
__device__ __forceinline__ float other_half(float x) { return swap_halves(x); }
__device__ __forceinline__ float other_row(float x) { return swap_rows(x); }

// Row of the 32x32 accumulator held in register r of a lane in half hf (its column is lane % 32).
__device__ __forceinline__ int acc_row(int r, int hf) { return 8 * (r >> 2) + 4 * hf + (r & 3); }

}  // namespace lvlm
