// The layer's own prefill attention, leaving the row normalisers the token scores are computed from
// (Sec. 3.2.1: the scores are a by-product of the attention of the layer; Sec. 3.2.2: of its statistics).
//
// out[b,i,h,:] = sum_j softmax_j(scale q[b,i,h].k[b,j,g]) v[b,j,g,:], g = h / G, over the keys row i may
// see; row_lse[b,h,i] = natural-log sum-exp of the row's scaled logits.  The last T rows' normalisers are
// also left densely packed for the column-sum pass of the score kernels, which then needs no normaliser
// pass of its own.
#include "mma.h"

#include <climits>
#include <type_traits>

namespace lvlm {
namespace {

struct PrefillArgs {
    const char *q, *k, *v;
    char *out;
    float *row_lse;     // [B][Hq][N]
    float *lse_t;       // [B][Hq][T] or null: the last T rows again
    int *redo;          // [grid]: workgroups the FAST kernel gave up, for the SAFE kernel
    int B, N, Hq, Hkv, G, causal, T;
    int nqb;            // query blocks per head
    int heads_per_xcd;  // ceil(B * Hq / 8)
    float scale, scale_log2;
    long long qsb, qsn, qsh, ksb, ksn, ksh, vsb, vsn, vsh, osb, osn, osh;   // bytes
};

constexpr float kLazy = 8.f;    // SAFE sweep: log2 of how far the row maximum may run ahead of the reference before a rescale
constexpr float kRisk = 64.f;   // FAST sweep: ... before the workgroup falls back to the SAFE sweep

// max of a value and the one held by the lane 32 places away (the other half-wave): one lane-swap instruction
// instead of a trip through the LDS permute unit.  The swap exchanges lanes 32..63 of its first operand with
// lanes 0..31 of its second; with the same value in both, every lane ends up with the two halves' values.
__device__ __forceinline__ float half_max(float x) {
    typedef unsigned u2 __attribute__((ext_vector_type(2)));
    const u2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r.x), __uint_as_float(r.y));
}

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
    typedef __bf16 bf2 __attribute__((ext_vector_type(2)));
    typedef float f2 __attribute__((ext_vector_type(2)));
    const bf2 r = __builtin_convertvector(f2{lo, hi}, bf2);
    return __builtin_bit_cast(uint32_t, r);
}

// bf16, matrix cores.  A workgroup of two waves owns 128 query rows of one head, 64 per wave as two 32-row
// blocks held in registers as MFMA operands.  Keys and values go by in tiles of 32: the 128 threads fetch
// the next tile while the current one is multiplied, K into LDS as it is (rows = keys), V turned around
// (rows = channels, 32 keys each) in registers on the way in; one barrier per tile.  Per tile and block:
// S^T = K Q^T (rows = keys, columns = queries), so a lane owns ONE query row and 16 of its logits -- the
// online max and sum are lane-local but for one exchange with the other half-wave -- and the 16
// probabilities, rounded to bf16, are already laid out as the second operand of O^T += V^T P^T when the
// keys inside V^T's rows are stored in the order the accumulator registers hold them.  Both blocks of a wave
// use each K and V^T fragment read from LDS, which is what keeps LDS bandwidth (about 64 bytes a clock per
// CU, measured) from bounding the kernel: one fragment read feeds two matrix instructions.
//
// The kernel exists twice.  The FAST one fixes each row's reference maximum at the first tile (every row sees
// key 0 there) and never rescales: probabilities are exp2 of the distance to that reference, possibly far
// above 1, which fp32 sums and bf16 operands carry at unchanged relative precision, and no vector instruction
// touches the output accumulators inside the loop, so they stay in the accumulation registers (with the
// rescaling branch in the loop the compiler copied all of them to vector registers and back on every tile).
// Should a logit rise more than 2^kRisk above its row's reference, the wave writes nothing and the workgroup
// marks itself in `redo`; the SAFE
// kernel, launched right after over the same grid, does the marked workgroups again with the textbook online
// softmax, whose reference follows the running maximum (lazily, in steps of 2^kLazy) and rescales sums and
// accumulators when it moves.  Unmarked workgroups of the SAFE launch exit at once.
template <int HD, bool SAFE>
__global__ __launch_bounds__(128, 1) void prefill_attn_bf16_kernel(PrefillArgs a) {
    constexpr int ROWB = HD * 2;
    constexpr int KP = ROWB + 16;           // K tile pitch: odd multiple of 16 bytes
    constexpr int VP = 80;                  // V^T row: 32 keys x 2 bytes + 16
    constexpr int NV = HD / 16;             // 16-byte words a lane holds of a row half
    constexpr int NCB = HD / 32;            // blocks of 32 channels
    constexpr int UPR = ROWB / 16;          // 16-byte units per row
    constexpr int KUPT = 32 * UPR / 128;    // K units per thread and tile
    constexpr int KTPR = UPR / KUPT;        // threads per K row
    __shared__ __attribute__((aligned(16))) char k_lds[2][32 * KP];
    __shared__ __attribute__((aligned(16))) char v_lds[2][HD * VP];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);     // uniform: conditions on it are scalar branches
    const int hf = lane >> 5, l32 = lane & 31;
    // Workgroup id -> (batch, head, query block).  Ids with the same remainder modulo 8 run on one XCD.  The
    // B * Hq heads, in memory order (heads of one KV head next to each other), are dealt to the 8 XCDs in
    // contiguous runs of equal length (+-1): heads that read the same keys and values mostly share an L2, and
    // every XCD gets the same load whatever the head counts.  Within an XCD the longest blocks (latest rows)
    // come first.
    const int xcd = blockIdx.x & 7, seq = blockIdx.x >> 3;
    const int NH = a.B * a.Hq;
    const int qb = a.nqb - 1 - seq / a.heads_per_xcd;
    const int head_first = (xcd * NH + 7) >> 3, head_end = ((xcd + 1) * NH + 7) >> 3;
    const int bh = head_first + seq % a.heads_per_xcd;
    if (bh >= head_end) return;
    if constexpr (SAFE) {
        if (a.redo[blockIdx.x] == 0) return;
    }
    const int b = bh / a.Hq, h = bh % a.Hq, g = h / a.G;
    const int q0 = qb * 128;
    const int wrow0 = q0 + 64 * wave;                 // this wave's first row
    const int kmax = a.causal ? min(a.N, q0 + 128) : a.N;
    const int n_tiles = (kmax + 31) >> 5;

    // staging.  K: thread -> row krow, units kcu + KTPR x.  V: thread -> four keys 4 vkg .. 4 vkg + 3 of one
    // 16-byte unit vcu (8 channels); HD = 64 needs only half the threads for V.
    const int krow = tid / KTPR, kcu = tid % KTPR;
    const char *kbase = a.k + (long long)b * a.ksb + (long long)g * a.ksh + 16 * kcu;
    const int vkg = tid & 7, vcu = tid >> 3;
    const bool v_on = vcu < UPR;
    const char *vbase = a.v + (long long)b * a.vsb + (long long)g * a.vsh + 16 * (v_on ? vcu : 0);
    // Named registers, not arrays (an indexed array that lives across the tile's arithmetic goes to scratch), and
    // written on EVERY tile (the last one fetches itself again): a value that may survive from the previous
    // tile is carried around the loop, and the compiler parks it in accumulation registers and copies it back.
    uint4 ks0 = make_uint4(0, 0, 0, 0), ks1 = ks0, ks2 = ks0, ks3 = ks0, vs0 = ks0, vs1 = ks0, vs2 = ks0, vs3 = ks0;
    const char *kthr = kbase + (long long)krow * a.ksn;           // this thread's row of tile 0
    const char *vthr = vbase + (long long)(4 * vkg) * a.vsn;
    auto fetch = [&](int j0) {
        if (j0 + 32 <= a.N) {                                     // whole tile: uniform offsets only
            const uint4 *src = reinterpret_cast<const uint4 *>(kthr + (long long)j0 * a.ksn);
            ks0 = src[0];
            if constexpr (KUPT > 1) ks1 = src[KTPR];
            if constexpr (KUPT > 2) ks2 = src[2 * KTPR];
            if constexpr (KUPT > 3) ks3 = src[3 * KTPR];
            if (v_on) {
                const char *vp = vthr + (long long)j0 * a.vsn;
                vs0 = *reinterpret_cast<const uint4 *>(vp);
                vs1 = *reinterpret_cast<const uint4 *>(vp + a.vsn);
                vs2 = *reinterpret_cast<const uint4 *>(vp + 2 * a.vsn);
                vs3 = *reinterpret_cast<const uint4 *>(vp + 3 * a.vsn);
            }
            return;
        }
        // the ragged last tile: rows past the end repeat the last row (masked later)
        const uint4 *src = reinterpret_cast<const uint4 *>(kbase + (long long)min(j0 + krow, a.N - 1) * a.ksn);
        ks0 = src[0];
        if constexpr (KUPT > 1) ks1 = src[KTPR];
        if constexpr (KUPT > 2) ks2 = src[2 * KTPR];
        if constexpr (KUPT > 3) ks3 = src[3 * KTPR];
        if (v_on) {
            const int jv = j0 + 4 * vkg;
            vs0 = *reinterpret_cast<const uint4 *>(vbase + (long long)min(jv + 0, a.N - 1) * a.vsn);
            vs1 = *reinterpret_cast<const uint4 *>(vbase + (long long)min(jv + 1, a.N - 1) * a.vsn);
            vs2 = *reinterpret_cast<const uint4 *>(vbase + (long long)min(jv + 2, a.N - 1) * a.vsn);
            vs3 = *reinterpret_cast<const uint4 *>(vbase + (long long)min(jv + 3, a.N - 1) * a.vsn);
        }
    };
    // Position of key kk of a tile inside a V^T row: accumulator register r of half hf holds key
    // 8 (r / 4) + 4 hf + r % 4 of a 32-key tile, and the second product wants the 8 keys of registers
    // 8 t .. 8 t + 7 in one 16-byte word: word index 2 t + hf, inside it 4 (r / 4 % 2) + r % 4.  Four keys
    // 4 vkg .. 4 vkg + 3 stay together: they go to byte 32 (vkg / 4) + 16 (vkg % 2) + 8 (vkg / 2 % 2).
    const int v_off = 32 * (vkg >> 2) + 16 * (vkg & 1) + 8 * ((vkg >> 1) & 1);
    // channels 2m (low halves of word m) and 2m + 1 (high halves) of the unit, four keys each
#define LVLM_VT(m, c)                                                                    \
    {                                                                                    \
        uint2 lo, hi;                                                                    \
        lo.x = __builtin_amdgcn_perm(vs1.c, vs0.c, 0x05040100u);                         \
        lo.y = __builtin_amdgcn_perm(vs3.c, vs2.c, 0x05040100u);                         \
        hi.x = __builtin_amdgcn_perm(vs1.c, vs0.c, 0x07060302u);                         \
        hi.y = __builtin_amdgcn_perm(vs3.c, vs2.c, 0x07060302u);                         \
        *reinterpret_cast<uint2 *>(vd + (2 * m) * VP) = lo;                              \
        *reinterpret_cast<uint2 *>(vd + (2 * m + 1) * VP) = hi;                          \
    }
    auto stash = [&](int buf) {
        uint4 *dst = reinterpret_cast<uint4 *>(&k_lds[buf][krow * KP + 16 * kcu]);
        dst[0] = ks0;
        if constexpr (KUPT > 1) dst[KTPR] = ks1;
        if constexpr (KUPT > 2) dst[2 * KTPR] = ks2;
        if constexpr (KUPT > 3) dst[3 * KTPR] = ks3;
        if (v_on) {
            char *vd = &v_lds[buf][(8 * vcu) * VP + v_off];
            LVLM_VT(0, x) LVLM_VT(1, y) LVLM_VT(2, z) LVLM_VT(3, w)
        }
    };
#undef LVLM_VT

    __shared__ int bail_s[2];
    float m_run[2], l_run[2];
    f32x16 oacc[2][NCB];
    bool risky = false;                     // FAST: some logit ran too far ahead of its row's reference (uniform per wave)
    (void)risky;
#pragma unroll
    for (int x = 0; x < 2; ++x) {
        m_run[x] = -INFINITY;
        l_run[x] = 0.f;
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[x][cb][r] = 0.f;
    }
    fetch(0);
    // The operand loads go out after the first tile's: loads return in order, and the tile (mostly in L2) would
    // otherwise wait behind the operand rows (from memory) before it can go to LDS.
    // Query operands: lane (row l32 of block x, half hf) holds bytes 16 hf + 32 i of its row
    uint4 qf[2][NV];
#pragma unroll
    for (int x = 0; x < 2; ++x) {
        const int row = wrow0 + 32 * x + l32;
        const char *src = a.q + (long long)b * a.qsb + (long long)min(row, a.N - 1) * a.qsn + (long long)h * a.qsh + 16 * hf;
#pragma unroll
        for (int i = 0; i < NV; ++i) qf[x][i] = *reinterpret_cast<const uint4 *>(src + 32 * i);
    }

    stash(0);
    __syncthreads();
    // One tile.  EDGE = false: every row of the workgroup sees the whole tile -- no masks, both blocks.  EDGE = true
    // (the up to four tiles around the diagonal, and a ragged last tile): per block the tile is seen whole, cut by
    // the diagonal (one fixed lane pattern, blocks and tiles being aligned alike), cut by the end of the sequence,
    // or not seen at all; a block that does not see it skips the logits and the softmax and multiplies zeros
    // into its accumulators (no branch around the instructions that update them: such a branch makes the
    // compiler copy all accumulators where its paths join).
    const int diag_lim = l32 - 4 * hf;       // register r of this lane holds a key past the diagonal iff 8 (r / 4) + r % 4 > diag_lim
    auto step = [&](int t, auto edge_tag) {
        constexpr bool EDGE = decltype(edge_tag)::value;
        const int j0 = t << 5, buf = t & 1;
        fetch(min(j0 + 32, (n_tiles - 1) << 5));
        // the output accumulators stay where the matrix instructions keep them
#pragma unroll
        for (int x = 0; x < 2; ++x)
#pragma unroll
            for (int cb = 0; cb < NCB; ++cb) asm volatile("" : "+a"(oacc[x][cb]));
        uint4 pf[2][2];
        auto softmax = [&](int x, f32x16 &s) {
            // Key j0 is visible to every row of a block the tile reaches, so the first tile sets a finite reference.
            auto row_max = [&]() {
                float mx = s[0];
#pragma unroll
                for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s[r]);
                return half_max(mx);
            };
            if constexpr (!SAFE) {
                // the reference is the first tile's maximum; later tiles need no maximum at all: a logit
                // far above the reference shows in the row sum (checked once, after the sweep)
                if (t == 0) m_run[x] = row_max();
            } else if (const float mx = row_max(); __builtin_amdgcn_ballot_w64((mx - m_run[x]) * a.scale_log2 > kLazy) != 0ull) {
                const float m_new = fmaxf(m_run[x], mx);
                const float alpha = __builtin_amdgcn_exp2f((m_run[x] - m_new) * a.scale_log2);   // first tile: 0
                l_run[x] *= alpha;
#pragma unroll
                for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
                    for (int r = 0; r < 16; ++r) oacc[x][cb][r] *= alpha;
                m_run[x] = m_new;
            }
            const float mb = m_run[x] * a.scale_log2;
            float sum = 0.f;
            float p[16];
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                p[r] = __builtin_amdgcn_exp2f(fmaf(s[r], a.scale_log2, -mb));
                sum += p[r];
            }
            l_run[x] += sum;
#pragma unroll
            for (int t2 = 0; t2 < 2; ++t2) {
                pf[x][t2].x = pack_bf16(p[8 * t2 + 0], p[8 * t2 + 1]);
                pf[x][t2].y = pack_bf16(p[8 * t2 + 2], p[8 * t2 + 3]);
                pf[x][t2].z = pack_bf16(p[8 * t2 + 4], p[8 * t2 + 5]);
                pf[x][t2].w = pack_bf16(p[8 * t2 + 6], p[8 * t2 + 7]);
            }
        };
        const char *ksrc = &k_lds[buf][l32 * KP + 16 * hf];
        if constexpr (!EDGE) {
            f32x16 s0, s1;
#pragma unroll
            for (int r = 0; r < 16; ++r) s0[r] = 0.f, s1[r] = 0.f;
#pragma unroll
            for (int i = 0; i < NV; ++i) {
                const uint4 kf = *reinterpret_cast<const uint4 *>(ksrc + 32 * i);
                const bf16x8 kb = __builtin_bit_cast(bf16x8, kf);
                s0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kb, __builtin_bit_cast(bf16x8, qf[0][i]), s0, 0, 0, 0);
                s1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kb, __builtin_bit_cast(bf16x8, qf[1][i]), s1, 0, 0, 0);
            }
            softmax(0, s0);
            softmax(1, s1);
        } else {
#pragma unroll
            for (int x = 0; x < 2; ++x) {
                const int blk0 = wrow0 + 32 * x;             // first row of the block
                if (a.causal && j0 > blk0) {                 // not seen at all
                    pf[x][0] = pf[x][1] = make_uint4(0, 0, 0, 0);
                    continue;
                }
                f32x16 s;
#pragma unroll
                for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
                for (int i = 0; i < NV; ++i) {
                    const uint4 kf = *reinterpret_cast<const uint4 *>(ksrc + 32 * i);
                    s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kf),
                                                                __builtin_bit_cast(bf16x8, qf[x][i]), s, 0, 0, 0);
                }
                if (j0 + 32 > a.N) {                         // the ragged last tile: by key index
                    const int row = blk0 + l32;
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int j = j0 + acc_row(r, hf);
                        if ((a.causal && j > row) || j >= a.N) s[r] = -INFINITY;
                    }
                } else if (a.causal && j0 == blk0) {         // the diagonal tile: a fixed pattern
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        if (8 * (r >> 2) + (r & 3) > diag_lim) s[r] = -INFINITY;
                }
                softmax(x, s);
            }
        }
        {
            const char *src = &v_lds[buf][l32 * VP + 16 * hf];
#pragma unroll
            for (int cb = 0; cb < NCB; ++cb) {
#pragma unroll
                for (int t2 = 0; t2 < 2; ++t2) {
                    const uint4 vf = *reinterpret_cast<const uint4 *>(src + (32 * cb) * VP + 32 * t2);
                    const bf16x8 vb = __builtin_bit_cast(bf16x8, vf);
                    oacc[0][cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vb, __builtin_bit_cast(bf16x8, pf[0][t2]),
                                                                         oacc[0][cb], 0, 0, 0);
                    oacc[1][cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vb, __builtin_bit_cast(bf16x8, pf[1][t2]),
                                                                         oacc[1][cb], 0, 0, 0);
                }
            }
        }
        if (t + 1 < n_tiles) stash(buf ^ 1);
        __syncthreads();
    };
    // tiles [0, t_whole) are seen whole by every row of the workgroup
    const int t_whole = a.causal ? min(q0, a.N) >> 5 : a.N >> 5;
    for (int t = 0; t < t_whole; ++t) step(t, std::false_type{});
    for (int t = t_whole; t < n_tiles; ++t) step(t, std::true_type{});
    // The FAST sweep runs to its end even when it has become useless (an exit from inside the loop makes the
    // compiler copy the accumulators on every tile); a wave that saw the risk writes nothing, and the mark
    // makes the SAFE kernel do the whole workgroup again.
    if constexpr (!SAFE) {
        // sums stay below 2^kRisk times the row length unless some probability went beyond 2^kRisk (or to inf / NaN)
        const float limit = __builtin_amdgcn_exp2f(kRisk) * 65536.f;
        risky = __builtin_amdgcn_ballot_w64(!(l_run[0] < limit) || !(l_run[1] < limit)) != 0ull;
        if (lane == 0) bail_s[wave] = risky;
        __syncthreads();
        if (tid == 0) a.redo[blockIdx.x] = bail_s[0] | bail_s[1];
        if (risky) return;
    }

    // normalise and write: lane (query l32, half hf) holds channels 32 cb + 8 (r / 4) + 4 hf + r % 4
#pragma unroll
    for (int x = 0; x < 2; ++x) {
        const int row = wrow0 + 32 * x + l32;
        const float l_tot = l_run[x] + __shfl_xor(l_run[x], 32);
        if (row >= a.N) continue;
        const float inv = 1.f / l_tot;
        char *dst = a.out + (long long)b * a.osb + (long long)row * a.osn + (long long)h * a.osh + 8 * hf;
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                uint2 w;
                w.x = pack_bf16(oacc[x][cb][4 * r4 + 0] * inv, oacc[x][cb][4 * r4 + 1] * inv);
                w.y = pack_bf16(oacc[x][cb][4 * r4 + 2] * inv, oacc[x][cb][4 * r4 + 3] * inv);
                *reinterpret_cast<uint2 *>(dst + 64 * cb + 16 * r4) = w;
            }
        if (hf == 0) {
            const float lse = m_run[x] * a.scale + __logf(l_tot);
            a.row_lse[((long long)b * a.Hq + h) * a.N + row] = lse;
            if (a.lse_t && row >= a.N - a.T) a.lse_t[((long long)b * a.Hq + h) * a.T + (row - (a.N - a.T))] = lse;
        }
    }
}

// fp32 (the small fp32 configuration), on the fp32 matrix instruction (32 x 32 x 2, exact fp32 products, fp32 sums).
// A workgroup of four waves owns 128 query rows of one head, one 32-row block per wave, its rows held as an MFMA
// operand.  K and V tiles of 32 keys go through LDS as they are (rows = keys), fetched one tile ahead by the 256
// threads, one barrier per tile.  S^T = K Q^T (rows = keys, columns = queries): a lane owns one query row and 16
// of its logits; the textbook online softmax (the reference follows the running maximum, sums and accumulators
// are rescaled when it moves).  For O^T += V^T P^T the contraction of one instruction is two keys, one per
// half-wave: exactly the two keys the two halves hold in the same accumulator register, so register r of the
// probabilities is the second operand as it stands and the first is V[that key][channel] read from the tile.
template <int HD>
__global__ __launch_bounds__(256, 1) void prefill_attn_f32_kernel(PrefillArgs a) {
    constexpr int ROWB = HD * 4;
    constexpr int KP = ROWB + 16;           // tile pitch: odd multiple of 16 bytes
    constexpr int NV = HalfRow<LVLM_F32, HD>::NV;
    constexpr int NCB = HD / 32;
    constexpr int UPR = ROWB / 16;          // 16-byte units per row
    constexpr int UPT = 32 * UPR / 256;     // units per thread and tile (2 or 4)
    constexpr int TPR = UPR / UPT;          // threads per row
    __shared__ __attribute__((aligned(16))) char k_lds[2][32 * KP];
    __shared__ __attribute__((aligned(16))) char v_lds[2][32 * KP];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int hf = lane >> 5, l32 = lane & 31;
    const int qb = gridDim.x - 1 - blockIdx.x, h = blockIdx.y, b = blockIdx.z;      // longest blocks first
    const int g = h / a.G;
    const int q0 = qb * 128, blk0 = q0 + 32 * wave;
    const int row = blk0 + l32;
    const int kmax = a.causal ? min(a.N, q0 + 128) : a.N;
    const int n_tiles = (kmax + 31) >> 5;

    HalfRow<LVLM_F32, HD> qa;               // lane (row l32, half hf): bytes 16 hf + 32 i of its row
    {
        const char *src = a.q + (long long)b * a.qsb + (long long)min(row, a.N - 1) * a.qsn + (long long)h * a.qsh + 16 * hf;
#pragma unroll
        for (int i = 0; i < NV; ++i) qa.v[i] = *reinterpret_cast<const uint4 *>(src + 32 * i);
    }
    const int srow = tid / TPR, scu = tid % TPR;
    const char *kbase = a.k + (long long)b * a.ksb + (long long)g * a.ksh + 16 * scu;
    const char *vbase = a.v + (long long)b * a.vsb + (long long)g * a.vsh + 16 * scu;
    uint4 ks0 = make_uint4(0, 0, 0, 0), ks1 = ks0, ks2 = ks0, ks3 = ks0, vs0 = ks0, vs1 = ks0, vs2 = ks0, vs3 = ks0;
    auto fetch = [&](int j0) {              // rows past the end repeat the last row (masked later)
        const long long r = min(j0 + srow, a.N - 1);
        const uint4 *ksrc = reinterpret_cast<const uint4 *>(kbase + r * a.ksn);
        const uint4 *vsrc = reinterpret_cast<const uint4 *>(vbase + r * a.vsn);
        ks0 = ksrc[0], vs0 = vsrc[0];
        ks1 = ksrc[TPR], vs1 = vsrc[TPR];
        if constexpr (UPT > 2) {
            ks2 = ksrc[2 * TPR], vs2 = vsrc[2 * TPR];
            ks3 = ksrc[3 * TPR], vs3 = vsrc[3 * TPR];
        }
    };
    auto stash = [&](int buf) {
        uint4 *kd = reinterpret_cast<uint4 *>(&k_lds[buf][srow * KP + 16 * scu]);
        uint4 *vd = reinterpret_cast<uint4 *>(&v_lds[buf][srow * KP + 16 * scu]);
        kd[0] = ks0, vd[0] = vs0;
        kd[TPR] = ks1, vd[TPR] = vs1;
        if constexpr (UPT > 2) {
            kd[2 * TPR] = ks2, vd[2 * TPR] = vs2;
            kd[3 * TPR] = ks3, vd[3 * TPR] = vs3;
        }
    };

    float m_run = -INFINITY, l_run = 0.f;
    f32x16 oacc[NCB];
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[cb][r] = 0.f;

    fetch(0);
    stash(0);
    __syncthreads();
    for (int t = 0; t < n_tiles; ++t) {
        const int j0 = t << 5, buf = t & 1;
        fetch(min(j0 + 32, (n_tiles - 1) << 5));
        if (!a.causal || j0 <= blk0 + 31) {                       // the block sees some key of the tile
            HalfRow<LVLM_F32, HD> kf;
            {
                const char *src = &k_lds[buf][l32 * KP + 16 * hf];
#pragma unroll
                for (int i = 0; i < NV; ++i) kf.v[i] = *reinterpret_cast<const uint4 *>(src + 32 * i);
            }
            f32x16 s;
#pragma unroll
            for (int r = 0; r < 16; ++r) s[r] = 0.f;
            mma_tile<LVLM_F32, HD>(s, kf, qa);                    // rows = keys, columns = queries
            if ((a.causal && j0 + 31 > blk0) || j0 + 32 > a.N) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int j = j0 + acc_row(r, hf);
                    if ((a.causal && j > row) || j >= a.N) s[r] = -INFINITY;
                }
            }
            float mx = s[0];
#pragma unroll
            for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s[r]);
            mx = fmaxf(mx, other_half(mx));                       // finite: key j0 <= blk0 is visible to every row
            const float m_new = fmaxf(m_run, mx);
            const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * a.scale_log2);   // first tile: 0
            const float mb = m_new * a.scale_log2;
            float p[16], sum = 0.f;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                p[r] = __builtin_amdgcn_exp2f(fmaf(s[r], a.scale_log2, -mb));
                sum += p[r];
            }
            l_run = l_run * alpha + sum;
            m_run = m_new;
#pragma unroll
            for (int cb = 0; cb < NCB; ++cb) {
#pragma unroll
                for (int r = 0; r < 16; ++r) oacc[cb][r] *= alpha;
                // register r of the two half-waves: keys acc_row(r, 0) and acc_row(r, 1) -- the two keys one
                // instruction contracts
                const char *vsrc = &v_lds[buf][4 * (32 * cb + l32)];
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float vv = *reinterpret_cast<const float *>(vsrc + acc_row(r, hf) * KP);
                    oacc[cb] = __builtin_amdgcn_mfma_f32_32x32x2f32(vv, p[r], oacc[cb], 0, 0, 0);
                }
            }
        }
        if (t + 1 < n_tiles) stash(buf ^ 1);
        __syncthreads();
    }

    const float l_tot = l_run + other_half(l_run);
    if (row >= a.N) return;
    const float inv = 1.f / l_tot;
    // lane (query l32, half hf) holds channels 32 cb + 8 (r / 4) + 4 hf + r % 4
    float *dst = reinterpret_cast<float *>(a.out + (long long)b * a.osb + (long long)row * a.osn + (long long)h * a.osh) + 4 * hf;
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4)
            *reinterpret_cast<float4 *>(dst + 32 * cb + 8 * r4) =
                make_float4(oacc[cb][4 * r4 + 0] * inv, oacc[cb][4 * r4 + 1] * inv, oacc[cb][4 * r4 + 2] * inv,
                            oacc[cb][4 * r4 + 3] * inv);
    if (hf == 0) {
        const float lse = m_run * a.scale + __logf(l_tot);
        a.row_lse[((long long)b * a.Hq + h) * a.N + row] = lse;
        if (a.lse_t && row >= a.N - a.T) a.lse_t[((long long)b * a.Hq + h) * a.T + (row - (a.N - a.T))] = lse;
    }
}

}  // namespace

PrefillWs prefill_ws(const lvlm_prefill_desc &d) {
    PrefillWs w{};
    w.lse_t = 0;
    w.redo = align_up((size_t)d.B * d.Hq * (d.T > 0 ? d.T : 0) * sizeof(float), 256);
    const size_t grid = (size_t)((d.B * d.Hq + 7) / 8) * 8 * ((d.N + 127) / 128);
    w.score = align_up(w.redo + grid * sizeof(int), 256);
    w.total = w.score;
    if (d.T > 0) w.total += align_up(score_ws(prefill_score_desc(d)).total, 256);
    return w;
}

lvlm_score_desc prefill_score_desc(const lvlm_prefill_desc &d) {
    lvlm_score_desc s{};
    s.dtype = d.dtype; s.B = d.B; s.N = d.N; s.T = d.T; s.q_pos0 = d.N - d.T; s.Hq = d.Hq; s.Hkv = d.Hkv; s.hd = d.hd;
    s.img_begin = d.img_begin; s.n_img = d.n_img; s.causal = d.causal; s.scale = d.scale;
    s.q_stride_b = d.q_stride_b; s.q_stride_t = d.q_stride_n; s.q_stride_h = d.q_stride_h;
    s.k_stride_b = d.k_stride_b; s.k_stride_n = d.k_stride_n; s.k_stride_h = d.k_stride_h;
    s.sh_stride_b = d.sh_stride_b; s.sh_stride_h = d.sh_stride_h;
    return s;
}

hipError_t launch_prefill_attn(const Prof &prof, const lvlm_prefill_desc &d, const PrefillWs &w, char *ws, const void *q,
                               const void *k, const void *v, void *out, float *row_lse, float *score_head,
                               float *score_mean) {
    hipStream_t stream = prof.stream;
    const int es = d.dtype == LVLM_BF16 ? 2 : 4;
    PrefillArgs a{};
    a.q = static_cast<const char *>(q); a.k = static_cast<const char *>(k); a.v = static_cast<const char *>(v);
    a.out = static_cast<char *>(out);
    a.row_lse = row_lse;
    a.lse_t = d.T > 0 ? reinterpret_cast<float *>(ws + w.lse_t) : nullptr;
    a.redo = reinterpret_cast<int *>(ws + w.redo);
    a.B = d.B; a.N = d.N; a.Hq = d.Hq; a.Hkv = d.Hkv; a.G = d.Hq / d.Hkv; a.causal = d.causal; a.T = d.T;
    a.nqb = (d.N + 127) / 128;
    a.heads_per_xcd = (d.B * d.Hq + 7) / 8;
    a.scale = d.scale; a.scale_log2 = d.scale * kLog2e;
    a.qsb = d.q_stride_b * es; a.qsn = d.q_stride_n * es; a.qsh = d.q_stride_h * es;
    a.ksb = d.k_stride_b * es; a.ksn = d.k_stride_n * es; a.ksh = d.k_stride_h * es;
    a.vsb = d.v_stride_b * es; a.vsn = d.v_stride_n * es; a.vsh = d.v_stride_h * es;
    a.osb = d.o_stride_b * es; a.osn = d.o_stride_n * es; a.osh = d.o_stride_h * es;
    prof.begin("prefill_attn");
    if (d.dtype == LVLM_BF16) {
        const long long grid = (long long)a.heads_per_xcd * 8 * a.nqb;
        if (d.hd == 128) {
            LVLM_LAUNCH(prof, (prefill_attn_bf16_kernel<128, false>), dim3((unsigned)grid), dim3(128), 0, stream, a);
            LVLM_LAUNCH(prof, (prefill_attn_bf16_kernel<128, true>), dim3((unsigned)grid), dim3(128), 0, stream, a);
        } else {
            LVLM_LAUNCH(prof, (prefill_attn_bf16_kernel<64, false>), dim3((unsigned)grid), dim3(128), 0, stream, a);
            LVLM_LAUNCH(prof, (prefill_attn_bf16_kernel<64, true>), dim3((unsigned)grid), dim3(128), 0, stream, a);
        }
    } else {
        const dim3 grid((unsigned)a.nqb, (unsigned)d.Hq, (unsigned)d.B);
        if (d.hd == 128) LVLM_LAUNCH(prof, (prefill_attn_f32_kernel<128>), grid, dim3(256), 0, stream, a);
        else LVLM_LAUNCH(prof, (prefill_attn_f32_kernel<64>), grid, dim3(256), 0, stream, a);
    }
    prof.end();
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || d.T <= 0) return e;
    // the scores of the last T rows from the normalisers just written: the column-sum pass alone
    const lvlm_score_desc sd = prefill_score_desc(d);
    const char *q_t = static_cast<const char *>(q) + (long long)(d.N - d.T) * d.q_stride_n * es;
    return launch_score(prof, sd, score_ws(sd), ws + w.score, q_t, k, a.lse_t, score_head, score_mean);
}

}  // namespace lvlm
