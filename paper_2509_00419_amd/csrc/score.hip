// Step 1 -- token importance = attention received (Sec. 3.2.1).
//
// For one (batch, KV head) the G*T query rows of the head group meet a block
// of keys as a dense tile product on the matrix cores.  The softmax needs
// each row's normaliser over ALL visible keys before a column sum can be
// taken, so the work is two passes over the same tiling:
//   pass 0  keys x queries tiles  -> per-row (max, sum-exp) of every key block,
//           then a small kernel folds the blocks into log2-domain LSE per row;
//   pass 1  queries x keys tiles over the image span only ->
//           p = exp2(logit - lse), summed down the rows of the tile.
// When the caller already has the row LSE (an attention kernel produces it),
// pass 0 is skipped.  The N x N probability matrix is never stored.
//
// Tiling (wave64, MFMA 32x32): a workgroup of 4 waves owns 4*KPW*32 keys; each
// wave keeps its KPW 32-key operand tiles in registers for the whole kernel and
// streams 32-row query chunks through LDS (double buffered, one barrier per
// chunk).  The reduction index of the MFMA is a dummy index, so each lane feeds
// one contiguous half of a head vector (lane/32 selects the half) -- global and
// LDS reads are then plain 16-byte vectors.
#include <limits.h>

#include "common.h"

namespace lvlm {
namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

struct ScoreArgs {
    const char *q;
    const char *k;
    const float *row_lse;
    float *part_m;
    float *part_l;
    float *lse2;
    float *score_head;
    float *score_mean;
    int B, N, T, q_pos0, Hq, Hkv, G, img_begin, n_img, causal, nkb;
    float scale_log2;
    long long qsb, qst, qsh, ksb, ksn, ksh, shb, shh;
};

template <int DT>
__host__ __device__ constexpr int esize() {
    return DT == LVLM_BF16 ? 2 : 4;
}

// The HD/2 contiguous elements one lane contributes to a 32 x 32 x HD product.
template <int DT, int HD>
struct HalfRow {
    static constexpr int NV = (HD / 2) * esize<DT>() / 16;
    uint4 v[NV];
};

// acc[32x32] += A[32 x HD] * B[32 x HD]^T ; rows of A map to rows of acc.
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

// Row of the 32x32 accumulator held in register r of a lane in half `hf`.
__device__ __forceinline__ int acc_row(int r, int hf) { return 8 * (r >> 2) + 4 * hf + (r & 3); }

template <int DT, int HD, int KPW, int PASS>
__global__ __launch_bounds__(256) void score_pass_kernel(ScoreArgs a) {
    constexpr int ES = esize<DT>();
    constexpr int ROWB = HD * ES;
    constexpr int PITCH = ROWB + 16;        // odd multiple of 16 B: conflict-free 128-bit LDS reads
    constexpr int UPR = ROWB / 16;          // 16-byte units per row
    constexpr int UPT = 32 * UPR / 256;     // units each thread stages per chunk
    constexpr int BN = 4 * KPW * 32;
    constexpr int NV = HalfRow<DT, HD>::NV;
    static_assert(UPT >= 1, "chunk smaller than the workgroup");

    __shared__ __attribute__((aligned(16))) char q_lds[2][32 * PITCH];
    __shared__ __attribute__((aligned(16))) int pos_lds[2][32];
    __shared__ __attribute__((aligned(16))) float lse_lds[2][32];
    __shared__ float red_m[2][4][32];
    __shared__ float red_l[2][4][32];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int hf = lane >> 5, l32 = lane & 31;
    const int kb = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
    const int GT = a.G * a.T;
    const int n_chunks = (GT + 31) >> 5;
    const int key_lo = PASS == 0 ? 0 : a.img_begin;
    const int key_hi = PASS == 0 ? a.N : a.img_begin + a.n_img;
    const int jbase = key_lo + kb * BN + wave * (KPW * 32);

    // this wave's key tiles, resident for the whole kernel
    HalfRow<DT, HD> kf[KPW];
#pragma unroll
    for (int s = 0; s < KPW; ++s) {
        const int j = jbase + 32 * s + l32;
        if (j < key_hi) {
            const char *src = a.k + ((long long)b * a.ksb + (long long)j * a.ksn + (long long)g * a.ksh) * ES +
                              hf * (ROWB / 2);
#pragma unroll
            for (int i = 0; i < NV; ++i) kf[s].v[i] = *reinterpret_cast<const uint4 *>(src + 16 * i);
        } else {
#pragma unroll
            for (int i = 0; i < NV; ++i) kf[s].v[i] = make_uint4(0, 0, 0, 0);
        }
    }

    uint4 stage[UPT];
    int stage_pos = -1;
    float stage_lse = 0.f;

    auto load_chunk = [&](int c) {
#pragma unroll
        for (int x = 0; x < UPT; ++x) {
            const int u = tid + 256 * x;
            const int row = u / UPR, cu = u % UPR;
            const int rho = c * 32 + row;
            if (rho < GT) {
                const int hl = rho / a.T, i = rho - hl * a.T;
                const char *src = a.q + ((long long)b * a.qsb + (long long)i * a.qst +
                                         (long long)(g * a.G + hl) * a.qsh) * ES + 16 * cu;
                stage[x] = *reinterpret_cast<const uint4 *>(src);
            } else {
                stage[x] = make_uint4(0, 0, 0, 0);
            }
        }
        if (tid < 32) {
            const int rho = c * 32 + tid;
            stage_pos = -1;          // padding row: sees no key
            stage_lse = 0.f;
            if (rho < GT) {
                const int hl = rho / a.T, i = rho - hl * a.T;
                stage_pos = a.causal ? a.q_pos0 + i : INT_MAX;
                if (PASS == 1) {
                    const long long ridx = ((long long)b * a.Hq + g * a.G + hl) * a.T + i;
                    stage_lse = a.row_lse ? a.row_lse[ridx] * kLog2e : a.lse2[ridx];
                }
            }
        }
    };
    auto store_chunk = [&](int buf) {
#pragma unroll
        for (int x = 0; x < UPT; ++x) {
            const int u = tid + 256 * x;
            const int row = u / UPR, cu = u % UPR;
            *reinterpret_cast<uint4 *>(&q_lds[buf][row * PITCH + 16 * cu]) = stage[x];
        }
        if (tid < 32) {
            pos_lds[buf][tid] = stage_pos;
            lse_lds[buf][tid] = stage_lse;
        }
    };
    // pass 0: fold the four waves' (max, sum) of chunk c and write the block's partial
    auto flush_partial = [&](int c) {
        if (tid < 32) {
            const int rho = c * 32 + tid;
            if (rho < GT) {
                const int buf = c & 1;
                float m = red_m[buf][0][tid];
#pragma unroll
                for (int w = 1; w < 4; ++w) m = fmaxf(m, red_m[buf][w][tid]);
                const float ms = (m == -INFINITY) ? 0.f : m;
                float l = 0.f;
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    const float mw = red_m[buf][w][tid];
                    l += (mw == -INFINITY) ? 0.f : red_l[buf][w][tid] * __builtin_amdgcn_exp2f(mw - ms);
                }
                const int hl = rho / a.T, i = rho - hl * a.T;
                const long long ridx = ((long long)b * a.Hq + g * a.G + hl) * a.T + i;
                const long long rows = (long long)a.B * a.Hq * a.T;
                a.part_m[kb * rows + ridx] = m;      // [key block][row]: coalesced here and in the fold
                a.part_l[kb * rows + ridx] = l;
            }
        }
    };

    float colsum[KPW];
#pragma unroll
    for (int s = 0; s < KPW; ++s) colsum[s] = 0.f;

    load_chunk(0);
    store_chunk(0);
    __syncthreads();

    for (int c = 0; c < n_chunks; ++c) {
        const int buf = c & 1;
        if (c + 1 < n_chunks) load_chunk(c + 1);
        if (PASS == 0 && c > 0) flush_partial(c - 1);

        HalfRow<DT, HD> qa;
        {
            const char *src = &q_lds[buf][l32 * PITCH + hf * (ROWB / 2)];
#pragma unroll
            for (int i = 0; i < NV; ++i) qa.v[i] = *reinterpret_cast<const uint4 *>(src + 16 * i);
        }
        f32x16 acc[KPW];
#pragma unroll
        for (int s = 0; s < KPW; ++s) {
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[s][r] = 0.f;
            if (PASS == 0)
                mma_tile<DT, HD>(acc[s], kf[s], qa);   // rows = keys, cols = queries
            else
                mma_tile<DT, HD>(acc[s], qa, kf[s]);   // rows = queries, cols = keys
        }

        if (PASS == 0) {
            // this lane: query l32 of the chunk, 16 keys per tile
            const int pos = pos_lds[buf][l32];
            float m = -INFINITY;
#pragma unroll
            for (int s = 0; s < KPW; ++s) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int j = jbase + 32 * s + acc_row(r, hf);
                    float t = acc[s][r] * a.scale_log2;
                    t = (j <= pos && j < key_hi) ? t : -INFINITY;
                    acc[s][r] = t;
                    m = fmaxf(m, t);
                }
            }
            m = fmaxf(m, __shfl_xor(m, 32));
            const float ms = (m == -INFINITY) ? 0.f : m;
            float l = 0.f;
#pragma unroll
            for (int s = 0; s < KPW; ++s) {
#pragma unroll
                for (int r = 0; r < 16; ++r) l += __builtin_amdgcn_exp2f(acc[s][r] - ms);   // exp2(-inf) = 0
            }
            l += __shfl_xor(l, 32);
            if (hf == 0) {
                red_m[buf][wave][l32] = m;
                red_l[buf][wave][l32] = l;
            }
        } else {
            // this lane: key l32 of each tile, 16 query rows of the chunk
#pragma unroll
            for (int qd = 0; qd < 4; ++qd) {
                const int4 pos4 = *reinterpret_cast<const int4 *>(&pos_lds[buf][8 * qd + 4 * hf]);
                const float4 lse4 = *reinterpret_cast<const float4 *>(&lse_lds[buf][8 * qd + 4 * hf]);
                const int pos[4] = {pos4.x, pos4.y, pos4.z, pos4.w};
                const float lse[4] = {lse4.x, lse4.y, lse4.z, lse4.w};
#pragma unroll
                for (int s = 0; s < KPW; ++s) {
                    const int j = jbase + 32 * s + l32;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float p = __builtin_amdgcn_exp2f(acc[s][4 * qd + e] * a.scale_log2 - lse[e]);
                        colsum[s] += (j <= pos[e]) ? p : 0.f;
                    }
                }
            }
        }

        if (c + 1 < n_chunks) store_chunk(buf ^ 1);
        __syncthreads();
    }

    if (PASS == 0) {
        flush_partial(n_chunks - 1);
    } else {
        const float inv_g = 1.0f / (float)a.G;
#pragma unroll
        for (int s = 0; s < KPW; ++s) {
            const float tot = colsum[s] + __shfl_xor(colsum[s], 32);
            const int j = jbase + 32 * s + l32;
            if (hf == 0 && j < key_hi)
                a.score_head[(long long)b * a.shb + (long long)g * a.shh + (j - a.img_begin)] = tot * inv_g;
        }
    }
}

// Fold the per-block (max, sum) pairs of each row into a log2-domain LSE (online, in block order).
__global__ __launch_bounds__(256) void score_lse_kernel(const float *part_m, const float *part_l, float *lse2,
                                                        int rows, int nkb) {
    const int row = blockIdx.x * 256 + threadIdx.x;
    if (row >= rows) return;
    float m = -INFINITY, l = 0.f;
#pragma unroll 8
    for (int i = 0; i < nkb; ++i) {
        const float mi = part_m[(long long)i * rows + row];
        const float li = part_l[(long long)i * rows + row];
        const float mn = fmaxf(m, mi);
        const float ms = (mn == -INFINITY) ? 0.f : mn;
        l = l * exp2f(m - ms) + li * exp2f(mi - ms);      // exp2(-inf) = 0 covers empty blocks
        m = mn;
    }
    lse2[row] = (l > 0.f) ? m + log2f(l) : INFINITY;   // a row that sees no key contributes nothing
}

// score_mean[b][j] = mean over KV heads, summed in head order.
__global__ __launch_bounds__(256) void score_mean_kernel(const float *score_head, float *score_mean, int Hkv,
                                                         int n_img, long long shb, long long shh) {
    const int j = blockIdx.x * 256 + threadIdx.x;
    const int b = blockIdx.y;
    if (j >= n_img) return;
    float s = 0.f;
    for (int g = 0; g < Hkv; ++g) s += score_head[(long long)b * shb + (long long)g * shh + j];
    score_mean[(long long)b * n_img + j] = s / (float)Hkv;
}

template <int DT, int HD, int KPW>
void launch_passes(const Prof &prof, const ScoreArgs &a, bool need_lse) {
    hipStream_t stream = prof.stream;
    constexpr int BN = 4 * KPW * 32;
    if (need_lse) {
        dim3 grid0((a.N + BN - 1) / BN, a.Hkv, a.B);
        prof.begin("score_pass0");
        hipLaunchKernelGGL((score_pass_kernel<DT, HD, KPW, 0>), grid0, dim3(256), 0, stream, a);
        prof.end();
        const int rows = a.B * a.Hq * a.T;
        prof.begin("score_lse");
        hipLaunchKernelGGL(score_lse_kernel, dim3((rows + 255) / 256), dim3(256), 0, stream, a.part_m, a.part_l,
                           a.lse2, rows, a.nkb);
        prof.end();
    }
    dim3 grid1((a.n_img + BN - 1) / BN, a.Hkv, a.B);
    prof.begin("score_pass1");
    hipLaunchKernelGGL((score_pass_kernel<DT, HD, KPW, 1>), grid1, dim3(256), 0, stream, a);
    prof.end();
    prof.begin("score_mean");
    hipLaunchKernelGGL(score_mean_kernel, dim3((a.n_img + 255) / 256, a.B), dim3(256), 0, stream, a.score_head,
                       a.score_mean, a.Hkv, a.n_img, a.shb, a.shh);
    prof.end();
}

}  // namespace

ScoreWs score_ws(const lvlm_score_desc &d) {
    ScoreWs w{};
    // Wide key blocks (2 tiles per wave) once they still give every CU two workgroups.
    const long long wide = (long long)d.B * d.Hkv * ((d.N + 255) / 256);
    w.block_keys = (d.dtype == LVLM_BF16 && wide >= 512) ? 256 : 128;
    w.nkb = (d.N + w.block_keys - 1) / w.block_keys;
    const size_t rows = (size_t)d.B * d.Hq * d.T;
    w.part_m = 0;
    w.part_l = align_up(w.part_m + rows * w.nkb * sizeof(float), 256);
    w.lse2 = align_up(w.part_l + rows * w.nkb * sizeof(float), 256);
    w.total = align_up(w.lse2 + rows * sizeof(float), 256);
    return w;
}

hipError_t launch_score(const Prof &prof, const lvlm_score_desc &d, const ScoreWs &w, char *ws, const void *q,
                        const void *k, const float *row_lse, float *score_head, float *score_mean) {
    ScoreArgs a{};
    a.q = static_cast<const char *>(q);
    a.k = static_cast<const char *>(k);
    a.row_lse = row_lse;
    a.part_m = reinterpret_cast<float *>(ws + w.part_m);
    a.part_l = reinterpret_cast<float *>(ws + w.part_l);
    a.lse2 = reinterpret_cast<float *>(ws + w.lse2);
    a.score_head = score_head;
    a.score_mean = score_mean;
    a.B = d.B; a.N = d.N; a.T = d.T; a.q_pos0 = d.q_pos0; a.Hq = d.Hq; a.Hkv = d.Hkv; a.G = d.Hq / d.Hkv;
    a.img_begin = d.img_begin; a.n_img = d.n_img; a.causal = d.causal; a.nkb = w.nkb;
    a.scale_log2 = d.scale * kLog2e;
    a.qsb = d.q_stride_b; a.qst = d.q_stride_t; a.qsh = d.q_stride_h;
    a.ksb = d.k_stride_b; a.ksn = d.k_stride_n; a.ksh = d.k_stride_h;
    const bool dense = d.sh_stride_b == 0 && d.sh_stride_h == 0;
    a.shh = dense ? d.n_img : d.sh_stride_h;
    a.shb = dense ? (long long)d.Hkv * d.n_img : d.sh_stride_b;
    const bool need_lse = row_lse == nullptr;
    const bool wide = w.block_keys == 256;
    if (d.dtype == LVLM_BF16 && d.hd == 128) {
        if (wide) launch_passes<LVLM_BF16, 128, 2>(prof, a, need_lse);
        else launch_passes<LVLM_BF16, 128, 1>(prof, a, need_lse);
    } else if (d.dtype == LVLM_BF16 && d.hd == 64) {
        if (wide) launch_passes<LVLM_BF16, 64, 2>(prof, a, need_lse);
        else launch_passes<LVLM_BF16, 64, 1>(prof, a, need_lse);
    } else if (d.dtype == LVLM_F32 && d.hd == 128) {
        launch_passes<LVLM_F32, 128, 1>(prof, a, need_lse);
    } else {
        launch_passes<LVLM_F32, 64, 1>(prof, a, need_lse);
    }
    return hipGetLastError();
}

}  // namespace lvlm
