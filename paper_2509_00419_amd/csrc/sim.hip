// Step 3b -- similarity merge (named by the benchmark spec; the paper itself merges by rank weights and
// avoids clustering, Sec. 3.2.1 par. 3).  The dominant tokens are the n_keep highest-scoring ones; every
// other token joins the dominant token it is most similar to (cosine of the rows of plane 0) and each
// dominant token becomes the size-weighted mean of its cluster.
//
//   rank_kernel (merge.hip)  ranks by score                     -> dominant = rank < n_keep
//   sim_index_kernel         positions of dominant tokens, list of the others (both ascending)
//   sim_norm_kernel          1 / |row| of every image token
//   sim_gemm_kernel          the one dense contraction of the path: (dominant x others) dot products on
//                            the matrix cores, 128 x 128 tile per workgroup, with the arg-max over the
//                            dominant axis taken in the epilogue (nothing of the similarity matrix is stored)
//   sim_assign_kernel        folds the per-block arg-maxima; emits the assignment and a sort key
//   rank_kernel + sim_order_kernel   tokens ordered by (assignment, index): each cluster is a contiguous,
//                            index-ordered segment, so the sums below run in a fixed order
//   sim_merge_kernel         one workgroup per dominant token and column block: size-weighted mean
//   sim_copy_kernel          rows outside the image span
#include <limits.h>

#include "common.h"
#include "mma.h"
#include "planes.h"

namespace lvlm {
namespace {

struct SimArgs {
    PlaneDev plane[LVLM_MAX_PLANES];
    const float *score;
    const float *size_in;   // [B, n] or null (all ones)
    float *size_out;        // [B, n_keep] or null
    int32_t *rank;          // [B, n]
    int32_t *dom_of;        // [B, n]  p >= 0: dominant position; -(q+1): q-th other token
    int32_t *keep_idx;      // [B, n_keep]
    int32_t *rest_idx;      // [B, r]
    float *inv_norm;        // [B, n]
    float *pbest_val;       // [B, NB, r]
    int32_t *pbest_idx;     // [B, NB, r]
    int32_t *assign;        // [B, n]
    float *key;             // [B, n]
    int32_t *rank2;         // [B, n]
    int32_t *order;         // [B, n]
    int B, N, img_begin, n, n_keep, r, NB, n_planes;
};

// ---- dominant positions and the list of the other tokens, both in ascending index ----
__global__ __launch_bounds__(1024) void sim_index_kernel(SimArgs a) {
    __shared__ int wave_cnt[16];
    __shared__ int base_s;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int b = blockIdx.x;
    const int32_t *rank = a.rank + (long long)b * a.n;
    if (tid == 0) base_s = 0;
    __syncthreads();
    for (int j0 = 0; j0 < a.n; j0 += 1024) {
        const int j = j0 + tid;
        const bool dom = j < a.n && rank[j] < a.n_keep;
        const unsigned long long bal = __ballot(dom);
        if (lane == 0) wave_cnt[wave] = __popcll(bal);
        __syncthreads();
        int p = base_s + __popcll(bal & ((1ull << lane) - 1ull));
        int tot = 0;
        for (int w = 0; w < 16; ++w) {
            p += w < wave ? wave_cnt[w] : 0;
            tot += wave_cnt[w];
        }
        if (j < a.n) {
            if (dom) {
                a.dom_of[(long long)b * a.n + j] = p;
                a.keep_idx[(long long)b * a.n_keep + p] = j;
            } else {
                const int q = j - p;              // tokens before j that are not dominant
                a.dom_of[(long long)b * a.n + j] = -(q + 1);
                a.rest_idx[(long long)b * a.r + q] = j;
            }
        }
        __syncthreads();
        if (tid == 0) base_s += tot;
        __syncthreads();
    }
}

// ---- 1 / |row| of every image token of plane 0 (one wave per token) ----
template <int DT>
__global__ __launch_bounds__(256) void sim_norm_kernel(SimArgs a) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int j = blockIdx.x * 4 + wave, b = blockIdx.y;
    if (j >= a.n) return;
    const PlaneDev &p = a.plane[0];
    const char *row = p.src + (long long)b * p.src_stride_b + (long long)(a.img_begin + j) * p.row_bytes;
    float s = 0.f;
    for (int u = lane; u < p.row_bytes / 16; u += 64) {
        const uint4 v = *reinterpret_cast<const uint4 *>(row + 16 * u);
        const uint32_t d[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if constexpr (DT == LVLM_BF16) {
                const float lo = __uint_as_float(d[i] << 16), hi = __uint_as_float(d[i] & 0xffff0000u);
                s = fmaf(lo, lo, s);
                s = fmaf(hi, hi, s);
            } else {
                const float x = __uint_as_float(d[i]);
                s = fmaf(x, x, s);
            }
        }
    }
    s = wave_sum(s);
    if (lane == 0) a.inv_norm[(long long)b * a.n + j] = s > 0.f ? 1.0f / sqrtf(s) : 1.0f;
}

// ---- dot products dominant x others on the matrix cores, arg-max over the dominant axis ----
// Workgroup tile: TM dominant rows x TN other rows, NWN x NWM waves, each owning TR x TC tiles of 32 x 32.
// Two shapes are built: 256 x 256 with eight waves of 128 x 64 (large problems: per tile product it moves
// a third less through LDS than the small shape, and half as much from L2) and 128 x 128 with four waves of
// 64 x 64 (more workgroups when the problem is small).  Rows are gathered by index; the contraction runs
// over 128-byte slices of the rows, double buffered in LDS with the next slice's global loads in flight
// (named scalars: they are carried around the loop).  One slice is eight 16-byte units per row and every
// thread stages four units of the dominant and four of the other rows.
//
// Tiles are numbered block by block (blocks of GN x GM tiles, ragged at the edges, batch rows one after the
// other) and handed out in runs of GN * GM consecutive numbers, run j to XCD j % 8 (workgroups reach the
// XCDs round-robin by id).  The workgroups resident on an XCD at the same time are then neighbours that
// sweep the contraction axis together: a row slice fetched into that XCD's L2 serves up to GM (dominant
// rows) or GN (other rows) of them, and every XCD gets the same number of tiles to within one run.
constexpr int kSimGN = 8, kSimGM = 4;

template <int DT, int NWN, int NWM, int TR, int TC, bool RAGGED>
__global__ __launch_bounds__(64 * NWN * NWM) void sim_gemm_kernel(SimArgs a) {
    constexpr int NT = 64 * NWN * NWM;
    constexpr int TM = NWN * TR * 32, TN = NWM * TC * 32;
    constexpr int SB = 128;              // bytes of one slice of a row
    constexpr int PITCH = SB + 16;       // slice + 16 bytes: spreads the rows over the LDS banks
    constexpr int RPI = NT / 8;          // rows one load instruction of the workgroup covers
    constexpr int UA = TM / RPI, UB = TN / RPI;      // staging units per thread: rows srow + RPI j of each operand
    __shared__ __attribute__((aligned(16))) char a_lds[2][TM * PITCH];
    __shared__ __attribute__((aligned(16))) char b_lds[2][TN * PITCH];
    __shared__ float invn[TM];
    __shared__ float bv[NWN][TN];
    __shared__ int bi[NWN][TN];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int hf = lane >> 5, l32 = lane & 31;
    const int wn = wave % NWN, wm = wave / NWN;
    // tile of this workgroup
    const int NBt = (a.n_keep + TM - 1) / TM, MBt = (a.r + TN - 1) / TN;
    constexpr int RUN = kSimGN * kSimGM;
    const int xcd = blockIdx.x & 7, seq = blockIdx.x >> 3;
    int t = ((seq / RUN) * 8 + xcd) * RUN + seq % RUN;
    if (t >= a.B * NBt * MBt) return;
    const int b = t / (NBt * MBt);
    t -= b * NBt * MBt;
    const int gm = (MBt + kSimGM - 1) / kSimGM, gn = (NBt + kSimGN - 1) / kSimGN;
    const int bj = min(t / (NBt * kSimGM), gm - 1);              // row of blocks; its height (the last may be lower)
    t -= bj * NBt * kSimGM;
    const int bh = min(kSimGM, MBt - bj * kSimGM);
    const int bi_ = min(t / (kSimGN * bh), gn - 1);              // block in that row; its width
    t -= bi_ * kSimGN * bh;
    const int bw = min(kSimGN, NBt - bi_ * kSimGN);
    const int nb = bi_ * kSimGN + t % bw, mb = bj * kSimGM + t / bw;

    const PlaneDev &p = a.plane[0];
    const int32_t *keep = a.keep_idx + (long long)b * a.n_keep;
    const int32_t *rest = a.rest_idx + (long long)b * a.r;
    const int srow = tid >> 3, su = tid & 7;        // staging: rows srow + RPI j (j < 4), unit su of the slice
    // Addresses are a uniform base (batch row, slice) plus a per-thread 32-bit byte offset (row, unit) that
    // never changes: the slice loop then needs no vector instruction per load -- on this chip matrix and
    // vector instructions do not overlap, so every one of them is time taken from the matrix cores.  The
    // offsets fit: the image rows of one batch row span less than 2 GiB (checked on the host).
    const char *img = p.src + (long long)b * p.src_stride_b + (long long)a.img_begin * p.row_bytes;
    // (named scalars below, not arrays: values carried around the slice loop must stay in registers)
    static_assert(UA <= 8 && UB <= 8, "staging registers are written out for up to eight units");
#define LVLM_SIM8(M) M(0) M(1) M(2) M(3) M(4) M(5) M(6) M(7)
#define LVLM_DECL(j)                                                                                        \
    const unsigned oa##j = j < UA ? keep[min(nb * TM + srow + RPI * j, a.n_keep - 1)] * p.row_bytes + 16 * su : 0; \
    const unsigned ob##j = j < UB ? rest[min(mb * TN + srow + RPI * j, a.r - 1)] * p.row_bytes + 16 * su : 0;      \
    uint4 sa##j, sb##j;      /* written by load before store reads them */
    LVLM_SIM8(LVLM_DECL)
#undef LVLM_DECL
    for (int i = tid; i < TM; i += NT) invn[i] = a.inv_norm[(long long)b * a.n + keep[min(nb * TM + i, a.n_keep - 1)]];
    const int nk = (p.row_bytes + SB - 1) / SB;      // the last slice may be partial: zero-filled

    // RAGGED: rows that are not a whole number of slices; units of the last slice beyond the row read as zero
    auto load = [&](int k) {
        const char *base = img + SB * k;             // uniform
        const bool in = !RAGGED || p.row_bytes - SB * k - 16 * su >= 16;
        const uint4 z = make_uint4(0, 0, 0, 0);
#define LVLM_LD(j)                                                                              \
        if constexpr (j < UA) sa##j = in ? *reinterpret_cast<const uint4 *>(base + oa##j) : z;  \
        if constexpr (j < UB) sb##j = in ? *reinterpret_cast<const uint4 *>(base + ob##j) : z;
        LVLM_SIM8(LVLM_LD)
#undef LVLM_LD
    };
    auto store = [&](int buf) {
        char *da = &a_lds[buf][srow * PITCH + 16 * su], *db = &b_lds[buf][srow * PITCH + 16 * su];
#define LVLM_ST(j)                                                                      \
        if constexpr (j < UA) *reinterpret_cast<uint4 *>(da + j * RPI * PITCH) = sa##j;  \
        if constexpr (j < UB) *reinterpret_cast<uint4 *>(db + j * RPI * PITCH) = sb##j;
        LVLM_SIM8(LVLM_ST)
#undef LVLM_ST
    };

    f32x16 acc[TR][TC];
#pragma unroll
    for (int nd = 0; nd < TR; ++nd)
#pragma unroll
        for (int nr = 0; nr < TC; ++nr)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[nd][nr][r] = 0.f;

    load(0);
    store(0);
    load(min(1, nk - 1));
    __syncthreads();
    for (int k = 0; k < nk; ++k) {
        store((k + 1) & 1);                      // slice k+1 (a harmless repeat after the last one)
        load(min(k + 2, nk - 1));
        const int buf = k & 1;
        const char *ar = &a_lds[buf][(wn * TR * 32 + l32) * PITCH + (SB / 2) * hf];
        const char *br = &b_lds[buf][(wm * TC * 32 + l32) * PITCH + (SB / 2) * hf];
        // one contraction step (16 bytes per lane and tile row) at a time: TR + TC operand words, TR x TC products
#pragma unroll
        for (int i = 0; i < SB / 32; ++i) {
            uint4 fa[TR], fb[TC];
#pragma unroll
            for (int t = 0; t < TR; ++t) fa[t] = *reinterpret_cast<const uint4 *>(ar + t * 32 * PITCH + 16 * i);
#pragma unroll
            for (int t = 0; t < TC; ++t) fb[t] = *reinterpret_cast<const uint4 *>(br + t * 32 * PITCH + 16 * i);
#pragma unroll
            for (int nd = 0; nd < TR; ++nd)
#pragma unroll
                for (int nr = 0; nr < TC; ++nr) {
                    if constexpr (DT == LVLM_BF16) {
                        mfma_one<DT>(acc[nd][nr], fa[nd], fb[nr], 0);      // rows = dominant, cols = others
                    } else {
#pragma unroll
                        for (int cpt = 0; cpt < 4; ++cpt) mfma_one<DT>(acc[nd][nr], fa[nd], fb[nr], cpt);
                    }
                }
        }
        __syncthreads();
    }

    // arg-max over the dominant rows: lane-local over its TR x 16 registers, then the other lane half, then
    // the NWN waves that share the columns.  Larger cosine wins; equal cosines go to the lower position.
#pragma unroll
    for (int nr = 0; nr < TC; ++nr) {
        float best_v = -INFINITY;
        int best_i = INT_MAX;
#pragma unroll
        for (int nd = 0; nd < TR; ++nd) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int il = wn * TR * 32 + nd * 32 + acc_row(r, hf);
                const int gi = nb * TM + il;
                const float v = acc[nd][nr][r] * invn[il];
                if (gi < a.n_keep && (v > best_v || (v == best_v && gi < best_i))) {
                    best_v = v;
                    best_i = gi;
                }
            }
        }
        const float ov = __shfl_xor(best_v, 32);
        const int oi = __shfl_xor(best_i, 32);
        if (ov > best_v || (ov == best_v && oi < best_i)) {
            best_v = ov;
            best_i = oi;
        }
        if (hf == 0) {
            bv[wn][wm * TC * 32 + nr * 32 + l32] = best_v;
            bi[wn][wm * TC * 32 + nr * 32 + l32] = best_i;
        }
    }
    __syncthreads();
    for (int i = tid; i < TN; i += NT) {
        const int q = mb * TN + i;
        if (q < a.r) {
            float v = bv[0][i];
            int ix = bi[0][i];
#pragma unroll
            for (int w = 1; w < NWN; ++w)
                if (bv[w][i] > v || (bv[w][i] == v && bi[w][i] < ix)) {
                    v = bv[w][i];
                    ix = bi[w][i];
                }
            const long long o = ((long long)b * a.NB + nb) * a.r + q;
            a.pbest_val[o] = v;
            a.pbest_idx[o] = ix;
        }
    }
#undef LVLM_SIM8
}

// ---- fold the dominant blocks; assignment of every token and the key that sorts tokens by it ----
__global__ __launch_bounds__(256) void sim_assign_kernel(SimArgs a) {
    const int j = blockIdx.x * 256 + threadIdx.x, b = blockIdx.y;
    if (j >= a.n) return;
    const int d = a.dom_of[(long long)b * a.n + j];
    int pos;
    float key;
    if (d >= 0) {
        pos = d;
        key = -1.0e9f;          // dominant tokens sort behind every cluster member
    } else {
        const int q = -d - 1;
        float best_v = -INFINITY;
        pos = INT_MAX;
        for (int nb = 0; nb < a.NB; ++nb) {
            const long long o = ((long long)b * a.NB + nb) * a.r + q;
            const float v = a.pbest_val[o];
            const int i = a.pbest_idx[o];
            if (v > best_v || (v == best_v && i < pos)) {
                best_v = v;
                pos = i;
            }
        }
        if (pos == INT_MAX) pos = 0;
        key = -(float)pos;      // exact: positions are far below 2^24
    }
    a.assign[(long long)b * a.n + j] = pos;
    a.key[(long long)b * a.n + j] = key;
}

__global__ __launch_bounds__(256) void sim_order_kernel(SimArgs a) {
    const int j = blockIdx.x * 256 + threadIdx.x, b = blockIdx.y;
    if (j < a.n) a.order[(long long)b * a.n + a.rank2[(long long)b * a.n + j]] = j;
}

// ---- size-weighted mean of each cluster ----
template <int DT, int UB>
__device__ __forceinline__ void store_mean(char *dst, const Acc<DT, UB> &acc, float inv_tot) {
    if constexpr (DT == LVLM_BF16 && UB == 16) {
        uint4 u;
        u.x = (uint32_t)f32_to_bf16(acc.v[0] * inv_tot) | ((uint32_t)f32_to_bf16(acc.v[1] * inv_tot) << 16);
        u.y = (uint32_t)f32_to_bf16(acc.v[2] * inv_tot) | ((uint32_t)f32_to_bf16(acc.v[3] * inv_tot) << 16);
        u.z = (uint32_t)f32_to_bf16(acc.v[4] * inv_tot) | ((uint32_t)f32_to_bf16(acc.v[5] * inv_tot) << 16);
        u.w = (uint32_t)f32_to_bf16(acc.v[6] * inv_tot) | ((uint32_t)f32_to_bf16(acc.v[7] * inv_tot) << 16);
        *reinterpret_cast<uint4 *>(dst) = u;
    } else if constexpr (DT == LVLM_BF16 && UB == 4) {
        *reinterpret_cast<uint32_t *>(dst) =
            (uint32_t)f32_to_bf16(acc.v[0] * inv_tot) | ((uint32_t)f32_to_bf16(acc.v[1] * inv_tot) << 16);
    } else if constexpr (DT == LVLM_BF16 && UB == 2) {
        *reinterpret_cast<uint16_t *>(dst) = f32_to_bf16(acc.v[0] * inv_tot);
    } else if constexpr (DT == LVLM_F32 && UB == 16) {
        *reinterpret_cast<float4 *>(dst) =
            make_float4(acc.v[0] * inv_tot, acc.v[1] * inv_tot, acc.v[2] * inv_tot, acc.v[3] * inv_tot);
    } else if constexpr (DT == LVLM_F32 && UB == 4) {
        *reinterpret_cast<float *>(dst) = acc.v[0] * inv_tot;
    }
}

template <int DT, int UB>
__device__ __forceinline__ void merge_plane(const SimArgs &a, const PlaneDev &p, int b, int i, int lo, int hi) {
    using U = typename Unit<UB>::type;
    const int unit = blockIdx.y * 256 + threadIdx.x;
    if (unit >= p.row_bytes / UB) return;
    const char *img = p.src + (long long)b * p.src_stride_b + (long long)a.img_begin * p.row_bytes + (long long)unit * UB;
    char *dst = p.dst + (long long)b * p.dst_stride_b + (long long)(a.img_begin + i) * p.row_bytes + (long long)unit * UB;
    const int ji = a.keep_idx[(long long)b * a.n_keep + i];
    const U own = *reinterpret_cast<const U *>(img + (long long)ji * p.row_bytes);
    if (p.rule != LVLM_RULE_WEIGHTED || DT == LVLM_I32) {
        *reinterpret_cast<U *>(dst) = own;
        return;
    }
    if constexpr (DT != LVLM_I32) {
        const float *size = a.size_in ? a.size_in + (long long)b * a.n : nullptr;
        const int32_t *order = a.order + (long long)b * a.n;
        Acc<DT, UB> acc;
#pragma unroll
        for (int e = 0; e < Acc<DT, UB>::NE; ++e) acc.v[e] = 0.f;
        float tot = size ? size[ji] : 1.0f;
        accumulate<DT, UB>(acc, own, tot);
        for (int s = lo; s < hi; ++s) {          // cluster members in ascending index
            const int t = order[s];
            const float st = size ? size[t] : 1.0f;
            accumulate<DT, UB>(acc, *reinterpret_cast<const U *>(img + (long long)t * p.row_bytes), st);
            tot += st;
        }
        store_mean<DT, UB>(dst, acc, 1.0f / tot);
        if (size && blockIdx.y == 0 && threadIdx.x == 0 && (int)blockIdx.z < a.B && a.size_out)
            a.size_out[(long long)b * a.n_keep + i] = tot;
    }
}

__global__ __launch_bounds__(256) void sim_merge_kernel(SimArgs a) {
    __shared__ int s_lo, s_hi;
    const int i = blockIdx.x;
    const int pi = blockIdx.z / a.B, b = blockIdx.z % a.B;
    const PlaneDev &p = a.plane[pi];
    if ((int)blockIdx.y >= p.col_blocks) return;
    if (threadIdx.x == 0) {
        // the tokens assigned to dominant position i form the segment [lo, hi) of the sorted order
        const int32_t *order = a.order + (long long)b * a.n;
        const int32_t *assign = a.assign + (long long)b * a.n;
        int lo = 0, hi = a.r;
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (assign[order[mid]] >= i) hi = mid; else lo = mid + 1;
        }
        s_lo = lo;
        hi = a.r;
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (assign[order[mid]] >= i + 1) hi = mid; else lo = mid + 1;
        }
        s_hi = lo;
        // sizes of all-ones clusters are written here (the weighted path writes them when sizes are given)
        if (pi == 0 && blockIdx.y == 0 && a.size_out && a.size_in == nullptr)
            a.size_out[(long long)b * a.n_keep + i] = (float)(1 + s_hi - s_lo);
    }
    __syncthreads();
    const int lo = s_lo, hi = s_hi;
    if (p.dtype == LVLM_BF16) {
        if (p.unit_bytes == 16) merge_plane<LVLM_BF16, 16>(a, p, b, i, lo, hi);
        else if (p.unit_bytes == 4) merge_plane<LVLM_BF16, 4>(a, p, b, i, lo, hi);
        else merge_plane<LVLM_BF16, 2>(a, p, b, i, lo, hi);
    } else if (p.dtype == LVLM_F32) {
        if (p.unit_bytes == 16) merge_plane<LVLM_F32, 16>(a, p, b, i, lo, hi);
        else merge_plane<LVLM_F32, 4>(a, p, b, i, lo, hi);
    } else {
        if (p.unit_bytes == 16) merge_plane<LVLM_I32, 16>(a, p, b, i, lo, hi);
        else merge_plane<LVLM_I32, 4>(a, p, b, i, lo, hi);
    }
}

// ---- rows outside the image span (or every row when nothing is removed) ----
struct CopyArgs {
    PlaneDev plane[LVLM_MAX_PLANES];
    int B, n_rows, split, src_shift, dst_shift;   // row ro >= split reads ro + src_shift, writes ro + dst_shift
};

__global__ __launch_bounds__(256) void sim_copy_kernel(CopyArgs a) {
    const int pi = blockIdx.z / a.B, b = blockIdx.z % a.B;
    const PlaneDev &p = a.plane[pi];
    const long long byte = ((long long)blockIdx.y * 256 + threadIdx.x) * p.unit_bytes;
    if (byte >= p.row_bytes) return;
    for (int ro = blockIdx.x; ro < a.n_rows; ro += gridDim.x) {
        const int rs = ro < a.split ? ro : ro + a.src_shift;
        const int rd = ro < a.split ? ro : ro + a.dst_shift;
        const char *s = p.src + (long long)b * p.src_stride_b + (long long)rs * p.row_bytes + byte;
        char *d = p.dst + (long long)b * p.dst_stride_b + (long long)rd * p.row_bytes + byte;
        if (p.unit_bytes == 16) *reinterpret_cast<uint4 *>(d) = *reinterpret_cast<const uint4 *>(s);
        else if (p.unit_bytes == 4) *reinterpret_cast<uint32_t *>(d) = *reinterpret_cast<const uint32_t *>(s);
        else *reinterpret_cast<uint16_t *>(d) = *reinterpret_cast<const uint16_t *>(s);
    }
}

// nothing removed: every token is its own cluster
__global__ __launch_bounds__(256) void sim_identity_kernel(SimArgs a) {
    const int j = blockIdx.x * 256 + threadIdx.x, b = blockIdx.y;
    if (j >= a.n) return;
    if (a.keep_idx) a.keep_idx[(long long)b * a.n + j] = j;
    if (a.assign) a.assign[(long long)b * a.n + j] = j;
    if (a.size_out) a.size_out[(long long)b * a.n + j] = a.size_in ? a.size_in[(long long)b * a.n + j] : 1.0f;
}

}  // namespace

SimWs sim_ws(const lvlm_merge_desc &d) {
    SimWs w{};
    const size_t n = (size_t)d.B * d.n_img;
    const int r = d.n_img - d.n_keep;
    // the large tile shape once it still gives every CU two workgroups
    w.tile = ((long long)d.B * ((d.n_keep + 255) / 256) * ((r + 255) / 256) >= 512) ? 256 : 128;
    w.NB = (d.n_keep + w.tile - 1) / w.tile;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        const size_t at = off;
        off = align_up(off + bytes, 256);
        return at;
    };
    w.rank = take(n * 4);
    w.dom_of = take(n * 4);
    w.keep_idx = take((size_t)d.B * d.n_keep * 4);
    w.rest_idx = take((size_t)d.B * (r > 0 ? r : 1) * 4);
    w.inv_norm = take(n * 4);
    w.pbest_val = take((size_t)d.B * w.NB * (r > 0 ? r : 1) * 4);
    w.pbest_idx = take((size_t)d.B * w.NB * (r > 0 ? r : 1) * 4);
    w.assign = take(n * 4);
    w.key = take(n * 4);
    w.rank2 = take(n * 4);
    w.order = take(n * 4);
    w.sorted = take(rank_scratch_bytes(d.n_img, d.B));     // sorted blocks of the two rankings, used in turn
    w.total = off;
    return w;
}

hipError_t launch_merge_similar(const Prof &prof, const lvlm_merge_desc &d, const SimWs &w, char *ws,
                                const float *score_mean, const lvlm_plane *planes, const float *size_in,
                                float *size_out, int32_t *keep_idx, int32_t *assign) {
    hipStream_t stream = prof.stream;
    const int r = d.n_img - d.n_keep;
    SimArgs a{};
    CopyArgs c{};
    int col_blocks = 1;
    for (int i = 0; i < d.n_planes; ++i) {
        a.plane[i] = make_plane_dev(planes[i]);
        c.plane[i] = a.plane[i];
        if (a.plane[i].col_blocks > col_blocks) col_blocks = a.plane[i].col_blocks;
    }
    a.score = score_mean;
    a.size_in = size_in;
    a.size_out = size_out;
    a.rank = reinterpret_cast<int32_t *>(ws + w.rank);
    a.dom_of = reinterpret_cast<int32_t *>(ws + w.dom_of);
    a.keep_idx = keep_idx ? keep_idx : reinterpret_cast<int32_t *>(ws + w.keep_idx);
    a.rest_idx = reinterpret_cast<int32_t *>(ws + w.rest_idx);
    a.inv_norm = reinterpret_cast<float *>(ws + w.inv_norm);
    a.pbest_val = reinterpret_cast<float *>(ws + w.pbest_val);
    a.pbest_idx = reinterpret_cast<int32_t *>(ws + w.pbest_idx);
    a.assign = assign ? assign : reinterpret_cast<int32_t *>(ws + w.assign);
    a.key = reinterpret_cast<float *>(ws + w.key);
    a.rank2 = reinterpret_cast<int32_t *>(ws + w.rank2);
    a.order = reinterpret_cast<int32_t *>(ws + w.order);
    a.B = d.B; a.N = d.N; a.img_begin = d.img_begin; a.n = d.n_img; a.n_keep = d.n_keep; a.r = r; a.NB = w.NB;
    a.n_planes = d.n_planes;
    c.B = d.B;

    if (r == 0) {
        a.keep_idx = keep_idx;
        a.assign = assign;
        c.n_rows = d.N; c.split = d.N; c.src_shift = 0; c.dst_shift = 0;
        prof.begin("sim_copy");
        LVLM_LAUNCH(prof, sim_copy_kernel, dim3(d.N < 2048 ? d.N : 2048, col_blocks, d.B * d.n_planes), dim3(256), 0,
                           stream, c);
        prof.end();
        if (keep_idx || assign || size_out)
            LVLM_LAUNCH(prof, sim_identity_kernel, dim3((d.n_img + 255) / 256, d.B), dim3(256), 0, stream, a);
        return hipGetLastError();
    }

    const dim3 per_token((d.n_img + 255) / 256, d.B);
    prof.begin("sim_rank");
    launch_rank(prof, score_mean, a.rank, d.n_img, d.B, ws + w.sorted);
    prof.end();
    prof.begin("sim_index");
    LVLM_LAUNCH(prof, sim_index_kernel, dim3(d.B), dim3(1024), 0, stream, a);
    prof.end();
    prof.begin("sim_norm");
    if (planes[0].dtype == LVLM_BF16)
        LVLM_LAUNCH(prof, sim_norm_kernel<LVLM_BF16>, dim3((d.n_img + 3) / 4, d.B), dim3(256), 0, stream, a);
    else
        LVLM_LAUNCH(prof, sim_norm_kernel<LVLM_F32>, dim3((d.n_img + 3) / 4, d.B), dim3(256), 0, stream, a);
    prof.end();
    prof.begin("sim_gemm");
    {
        const long long tiles = (long long)d.B * w.NB * ((r + w.tile - 1) / w.tile);
        constexpr int run = kSimGN * kSimGM;
        const dim3 ggrid((unsigned)(((tiles + run - 1) / run + 7) / 8 * 8 * run));
        const bool bf = planes[0].dtype == LVLM_BF16;
        const bool ragged = (planes[0].row_elems * (bf ? 2 : 4)) % 128 != 0;
#define LVLM_GEMM(DT, NWN, NWM, TR, TC)                                                                              \
    if (ragged)                                                                                                      \
        LVLM_LAUNCH(prof, (sim_gemm_kernel<DT, NWN, NWM, TR, TC, true>), ggrid, dim3(64 * NWN * NWM), 0, stream, a);  \
    else                                                                                                             \
        LVLM_LAUNCH(prof, (sim_gemm_kernel<DT, NWN, NWM, TR, TC, false>), ggrid, dim3(64 * NWN * NWM), 0, stream, a)
        if (w.tile == 256) {
            if (bf) { LVLM_GEMM(LVLM_BF16, 2, 4, 4, 2); } else { LVLM_GEMM(LVLM_F32, 2, 4, 4, 2); }
        } else {
            if (bf) { LVLM_GEMM(LVLM_BF16, 2, 2, 2, 2); } else { LVLM_GEMM(LVLM_F32, 2, 2, 2, 2); }
        }
#undef LVLM_GEMM
    }
    prof.end();
    prof.begin("sim_assign");
    LVLM_LAUNCH(prof, sim_assign_kernel, per_token, dim3(256), 0, stream, a);
    prof.end();
    prof.begin("sim_rank2");
    launch_rank(prof, a.key, a.rank2, d.n_img, d.B, ws + w.sorted);
    prof.end();
    prof.begin("sim_order");
    LVLM_LAUNCH(prof, sim_order_kernel, per_token, dim3(256), 0, stream, a);
    prof.end();
    prof.begin("sim_merge");
    LVLM_LAUNCH(prof, sim_merge_kernel, dim3(d.n_keep, col_blocks, d.B * d.n_planes), dim3(256), 0, stream, a);
    prof.end();
    const int outside = d.N - d.n_img;
    if (outside > 0) {
        c.n_rows = outside; c.split = d.img_begin; c.src_shift = d.n_img; c.dst_shift = d.n_keep;
        prof.begin("sim_copy");
        LVLM_LAUNCH(prof, sim_copy_kernel, dim3(outside < 2048 ? outside : 2048, col_blocks, d.B * d.n_planes),
                           dim3(256), 0, stream, c);
        prof.end();
    }
    return hipGetLastError();
}

}  // namespace lvlm
