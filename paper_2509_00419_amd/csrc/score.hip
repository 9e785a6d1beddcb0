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
// chunk).  The reduction index of the MFMA is a dummy index, so step i of lane
// half lane/32 simply takes bytes [32 i + 16 (lane/32), +16) of a head vector --
// global and LDS reads are then plain 16-byte vectors.
#include <limits.h>

#include "common.h"
#include "mma.h"

#include <type_traits>

namespace lvlm {
namespace {


struct ScoreArgs {
    const char *q;
    const char *k;
    const float *row_lse;
    float *part_m;      // [nkb * 4][rows]   per key block and wave: row max (log2 domain)
    float *part_l;      // [nkb * 4][rows]   ... and sum of exp2(logit - max)
    float *lse2;        // [rows]
    float *colpart;     // [RS][B][Hkv][n_img]  column sums of each row split
    float *score_head;
    float *score_mean;
    int B, N, T, q_pos0, Hq, Hkv, G, img_begin, n_img, causal, nkb;
    int rs;             // row splits: workgroups that share a key block and take different query chunks
    int cps;            // chunks per split
    int n_seg;          // shared-tile form: runs the keys are cut into (1 = both sweeps in one launch)
    unsigned t_magic;   // floor(2^32 / T) + 1: rho / T == umulhi(rho, t_magic) for rho, T < 65536
    float scale_log2;
    long long qsb, qst, qsh, ksb, ksn, ksh, shb, shh;
};


template <int DT, int HD, int KPW, int PASS>
__global__ __launch_bounds__(256, 3) void score_pass_kernel(ScoreArgs a) {
    constexpr int ES = esize<DT>();
    constexpr int ROWB = HD * ES;
    constexpr int PITCH = ROWB + 16;        // odd multiple of 16 B: conflict-free 128-bit LDS reads
    constexpr int UPR = ROWB / 16;          // 16-byte units per row
    constexpr int UPT = 32 * UPR / 256;     // units each thread stages per chunk
    constexpr int BN = 4 * KPW * 32;
    constexpr int NV = HalfRow<DT, HD>::NV;
    constexpr int NBUF = 3;
    static_assert(UPT >= 1 && UPT <= 4, "staging covers 1..4 units per thread");

    __shared__ __attribute__((aligned(16))) char q_lds[NBUF][32 * PITCH];
    __shared__ __attribute__((aligned(16))) int pos_lds[NBUF][32];
    __shared__ __attribute__((aligned(16))) float lse_lds[NBUF][32];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int hf = lane >> 5, l32 = lane & 31;
    // Workgroups are handed to the 8 XCDs round-robin by linear id, and grid.x is a multiple of 8, so
    // blockIdx.x % 8 names the XCD (and its private L2).  The row splits of one key block are placed on
    // the same XCD: they read the same keys.
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    // The normaliser pass takes its key blocks from the last one down: the blocks at the end of the sequence are the
    // ones that need the mask (the slow path), and a slow workgroup started last would run on after all the others.
    const int kslot = PASS == 0 ? (int)(gridDim.x / (8 * a.rs)) - 1 - slot / a.rs : slot / a.rs;
    const int kb = kslot * 8 + xcd, rs = slot % a.rs;
    const int g = blockIdx.y, b = blockIdx.z;
    if (kb * BN >= (PASS == 0 ? a.N : a.n_img)) return;      // padding of the key-block count to a multiple of 8
    const int GT = a.G * a.T;
    const int n_chunks = (GT + 31) >> 5;
    const int c_lo = rs * a.cps, c_hi = min(n_chunks, c_lo + a.cps);
    const int key_lo = PASS == 0 ? 0 : a.img_begin;
    const int key_hi = PASS == 0 ? a.N : a.img_begin + a.n_img;
    const int jbase = key_lo + kb * BN + wave * (KPW * 32);
    const long long rowbase = ((long long)b * a.Hq + (long long)g * a.G) * a.T;   // row index of chunk row rho: rowbase + rho
    const long long rows_total = (long long)a.B * a.Hq * a.T;

    // rho / T without a hardware divide (exact for rho, T < 65536; T == 1 has no 32-bit magic number)
    auto div_t = [&](int rho) -> int { return a.T == 1 ? rho : (int)__umulhi((unsigned)rho, a.t_magic); };

    // this wave's key tiles, resident for the whole kernel
    HalfRow<DT, HD> kf[KPW];
#pragma unroll
    for (int s = 0; s < KPW; ++s) {
        // Contraction step i of lane half hf takes bytes [32 i + 16 hf, +16) of a row (both operands).  The
        // load puts a lane PAIR on 32 contiguous bytes of one row -- the memory pipeline serves one request
        // per lane when every lane of a quad reads another row -- and a lane permute then moves each piece
        // to the lane (row l32, half hf) the MFMA wants it in.
        const int j = jbase + 32 * s + (lane >> 1);
        uint4 raw[NV];
#pragma unroll
        for (int i = 0; i < NV; ++i) raw[i] = make_uint4(0, 0, 0, 0);
        if (j < key_hi) {
            const char *src = a.k + ((long long)b * a.ksb + (long long)j * a.ksn + (long long)g * a.ksh) * ES +
                              16 * (lane & 1);
#pragma unroll
            for (int i = 0; i < NV; ++i) raw[i] = *reinterpret_cast<const uint4 *>(src + 32 * i);
        }
        const int from = 4 * (2 * l32 + hf);
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            kf[s].v[i].x = __builtin_amdgcn_ds_bpermute(from, raw[i].x);
            kf[s].v[i].y = __builtin_amdgcn_ds_bpermute(from, raw[i].y);
            kf[s].v[i].z = __builtin_amdgcn_ds_bpermute(from, raw[i].z);
            kf[s].v[i].w = __builtin_amdgcn_ds_bpermute(from, raw[i].w);
        }
    }

    // Two chunks of 32 query rows are on their way from global memory to LDS at any time (stages A and
    // B).  Named scalars, not arrays or structs: the values are carried around the chunk loop and must
    // stay in registers.
    uint4 stA0 = make_uint4(0, 0, 0, 0), stA1 = stA0, stA2 = stA0, stA3 = stA0;
    uint4 stB0 = stA0, stB1 = stA0, stB2 = stA0, stB3 = stA0;
    int stA_pos = -1, stB_pos = -1;
    float stA_lse = 0.f, stB_lse = 0.f;
    // A thread stages UPT 16-byte units of ONE row of every chunk.  Its source address is
    // carried from load to load (a stage takes every second chunk: 64 rows further down, stepping over to
    // the next head when the rows of one are used up), so the chunk loop holds no address multiplies.
    constexpr int TPR = UPR / UPT;       // threads per row: neighbouring lanes read neighbouring 16-byte units
    const int srow = tid / TPR, scu = tid % TPR;       // units scu + TPR x, x < UPT
    const long long q_step = 64 * a.qst * ES;                            // 64 rows further in the same head
    const long long q_wrap = (a.qsh - (long long)a.T * a.qst) * ES;      // from row T of a head to row 0 of the next
    const char *q_grp0 = a.q + ((long long)b * a.qsb + (long long)g * a.G * a.qsh) * ES;    // uniform
    const char *q_grp = q_grp0 + 16 * scu;
    // padding rows (beyond the last row of the group, in its last chunk only) repeat the last row; they are
    // masked in compute.  Its address is formed where it is used, from uniform values: a register pair
    // held around the loop would push a staging register out to scratch memory.
    const char *q_last0 = q_grp0 + ((long long)(a.G - 1) * a.qsh + (long long)(a.T - 1) * a.qst) * ES;
    auto chunk_row = [&](int c, const char *ptr) -> const uint4 * {
        if (c == n_chunks - 1) {
            int off = 16 * scu;
            asm volatile("" : "+v"(off));            // keeps the sum below inside this branch
            if (c * 32 + srow >= GT) ptr = q_last0 + off;
        }
        return reinterpret_cast<const uint4 *>(ptr);
    };
    auto row_ptr = [&](int c, int &i) -> const char * {
        const int rho = c * 32 + srow;
        const int hl = div_t(rho);
        i = rho - hl * a.T;
        return q_grp + ((long long)hl * a.qsh + (long long)i * a.qst) * ES;
    };
    int iA = 0, iB = 0;
    const char *pA = row_ptr(c_lo, iA), *pB = row_ptr(c_lo + 1, iB);
    auto advance = [&](const char *&ptr, int &i) {
        i += 64;
        ptr += q_step;
        if (a.T >= 64) {
            const bool over = i >= a.T;
            i -= over ? a.T : 0;
            ptr += over ? q_wrap : 0;
        } else {
            while (i >= a.T) {
                i -= a.T;
                ptr += q_wrap;
            }
        }
    };
    auto chunk_dst = [&](int buf, int x) -> uint4 * {
        return reinterpret_cast<uint4 *>(&q_lds[buf][srow * PITCH + 16 * (scu + TPR * x)]);
    };
    auto row_meta = [&](int c, int &pos, float &lse) {
        pos = -1;             // padding row: sees no key
        lse = 0.f;
        if (tid < 32) {
            const int rho = c * 32 + tid;
            if (rho < GT) {
                pos = a.causal ? a.q_pos0 + (rho - div_t(rho) * a.T) : INT_MAX;
                // (as loaded: the change of base waits for store time -- a use right here would stall the wave on the
                // load, with the chunk's own loads just issued in front of it)
                if (PASS == 1) lse = a.row_lse ? a.row_lse[rowbase + rho] : a.lse2[rowbase + rho];
            }
        }
    };
#define LVLM_STAGE_FUNCS(S)                                              \
    auto load_##S = [&](int kk) {           /* chunk c_lo + kk; nothing to fetch past the last chunk */ \
        const int c = c_lo + kk;                                         \
        if (c < c_hi) {                                                  \
            const uint4 *src = chunk_row(c, p##S);                      \
            st##S##0 = src[0];                                           \
            if constexpr (UPT > 1) st##S##1 = src[TPR];                  \
            if constexpr (UPT > 2) st##S##2 = src[2 * TPR];              \
            if constexpr (UPT > 3) st##S##3 = src[3 * TPR];              \
            row_meta(c, st##S##_pos, st##S##_lse);                       \
        }                                                                \
        advance(p##S, i##S);                                             \
    };                                                                   \
    auto store_##S = [&](int buf) {                                      \
        *chunk_dst(buf, 0) = st##S##0;                                   \
        if constexpr (UPT > 1) *chunk_dst(buf, 1) = st##S##1;            \
        if constexpr (UPT > 2) *chunk_dst(buf, 2) = st##S##2;            \
        if constexpr (UPT > 3) *chunk_dst(buf, 3) = st##S##3;            \
        if (tid < 32) {                                                  \
            pos_lds[buf][tid] = st##S##_pos;                             \
            lse_lds[buf][tid] = a.row_lse ? st##S##_lse * kLog2e : st##S##_lse;   /* a caller's are natural logarithms */ \
        }                                                                \
    };
    LVLM_STAGE_FUNCS(A)
    LVLM_STAGE_FUNCS(B)
#undef LVLM_STAGE_FUNCS

    float colsum[KPW];
#pragma unroll
    for (int s = 0; s < KPW; ++s) colsum[s] = 0.f;

    auto compute = [&](int c, int buf) {
        // Positions of the chunk's rows (uniform): a chunk inside one head covers rows i0 .. i0 + 31 of it, one
        // that straddles two heads anything from 0 to T - 1.
        const int rho0 = c * 32, rho1 = min(rho0 + 31, GT - 1);
        const int h0 = div_t(rho0), h1 = div_t(rho1);
        const int min_i = (h0 != h1) ? 0 : rho0 - h0 * a.T;
        const int max_i = (h0 != h1) ? a.T - 1 : rho1 - h1 * a.T;
        // Every key of this wave lies ahead of every row of the chunk (query rows inside the key range, as when
        // all rows of the sequence are scored): nothing to multiply.
        if (a.causal && jbase > a.q_pos0 + max_i) {
            if (PASS == 0) {
                const int rho = rho0 + l32;
                if (hf == 0 && rho < GT) {
                    const long long pidx = ((long long)kb * 4 + wave) * rows_total + rowbase + rho;
                    a.part_m[pidx] = -INFINITY;
                    a.part_l[pidx] = 0.f;
                }
            }
            return;
        }
        HalfRow<DT, HD> qa;
        {
            const char *src = &q_lds[buf][l32 * PITCH + 16 * hf];
#pragma unroll
            for (int i = 0; i < NV; ++i) qa.v[i] = *reinterpret_cast<const uint4 *>(src + 32 * i);
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
        // Is any element of this 32 x (KPW*32) block masked?  Uniform over the workgroup's wave:
        // keys beyond the range, padding rows, or a key ahead of the earliest query position of the chunk.
        const bool masked = jbase + KPW * 32 > key_hi || rho0 + 32 > GT ||
                            (a.causal && jbase + KPW * 32 - 1 > a.q_pos0 + min_i);

        if (PASS == 0) {
            // this lane: query l32 of the chunk, 16 keys per tile
            float m = -INFINITY, l = 0.f;
            if (!masked) {
#pragma unroll
                for (int s = 0; s < KPW; ++s)
#pragma unroll
                    for (int r = 0; r < 16; ++r) m = fmaxf(m, acc[s][r]);
                m = fmaxf(m, other_half(m)) * a.scale_log2;      // scale >= 0 (checked on the host)
#pragma unroll
                for (int s = 0; s < KPW; ++s)
#pragma unroll
                    for (int r = 0; r < 16; ++r) l += __builtin_amdgcn_exp2f(fmaf(acc[s][r], a.scale_log2, -m));
            } else {
                const int pos = pos_lds[buf][l32];
#pragma unroll
                for (int s = 0; s < KPW; ++s) {
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int j = jbase + 32 * s + acc_row(r, hf);
                        const float t = (j <= pos && j < key_hi) ? acc[s][r] * a.scale_log2 : -INFINITY;
                        acc[s][r] = t;
                        m = fmaxf(m, t);
                    }
                }
                m = fmaxf(m, other_half(m));
                const float ms = (m == -INFINITY) ? 0.f : m;
#pragma unroll
                for (int s = 0; s < KPW; ++s)
#pragma unroll
                    for (int r = 0; r < 16; ++r) l += __builtin_amdgcn_exp2f(acc[s][r] - ms);   // exp2(-inf) = 0
            }
            l += other_half(l);
            const int rho = rho0 + l32;
            if (hf == 0 && rho < GT) {
                const long long pidx = ((long long)kb * 4 + wave) * rows_total + rowbase + rho;
                a.part_m[pidx] = m;
                a.part_l[pidx] = l;
            }
        } else {
            // this lane: key l32 of each tile, 16 query rows of the chunk
#pragma unroll
            for (int qd = 0; qd < 4; ++qd) {
                const float4 lse4 = *reinterpret_cast<const float4 *>(&lse_lds[buf][8 * qd + 4 * hf]);
                const float lse[4] = {lse4.x, lse4.y, lse4.z, lse4.w};
                if (!masked) {
#pragma unroll
                    for (int s = 0; s < KPW; ++s)
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            colsum[s] += __builtin_amdgcn_exp2f(fmaf(acc[s][4 * qd + e], a.scale_log2, -lse[e]));
                } else {
                    const int4 pos4 = *reinterpret_cast<const int4 *>(&pos_lds[buf][8 * qd + 4 * hf]);
                    const int pos[4] = {pos4.x, pos4.y, pos4.z, pos4.w};
#pragma unroll
                    for (int s = 0; s < KPW; ++s) {
                        const int j = jbase + 32 * s + l32;
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const float p = __builtin_amdgcn_exp2f(fmaf(acc[s][4 * qd + e], a.scale_log2, -lse[e]));
                            colsum[s] += (j <= pos[e]) ? p : 0.f;
                        }
                    }
                }
            }
        }
    };

    // Pipeline over the chunks k = 0 .. nc-1 of this workgroup: chunk k is loaded from global memory into
    // a register stage two iterations before it is computed (even chunks in A, odd ones in B), copied
    // into one of three LDS buffers one iteration before, and one barrier per chunk publishes the copy.
    // Past the last chunk nothing is loaded; the copies then repeat stale registers that nothing reads.
    const int nc = c_hi - c_lo;
    load_A(0);
    store_A(0);
    load_B(1);
    load_A(2);
    __syncthreads();
    for (int k = 0; k < nc; k += 2) {
        store_B((k + 1) % NBUF);          // chunk k+1
        load_B(k + 3);
        compute(c_lo + k, k % NBUF);
        __syncthreads();
        if (k + 1 >= nc) break;
        store_A((k + 2) % NBUF);          // chunk k+2
        load_A(k + 4);
        compute(c_lo + k + 1, (k + 1) % NBUF);
        __syncthreads();
    }

    if (PASS == 1) {
#pragma unroll
        for (int s = 0; s < KPW; ++s) {
            const float tot = colsum[s] + other_half(colsum[s]);
            const int j = jbase + 32 * s + l32;
            if (hf == 0 && j < key_hi)
                a.colpart[(((long long)rs * a.B + b) * a.Hkv + g) * a.n_img + (j - a.img_begin)] = tot;
        }
    }
}

// ---- short sequences: both passes in one launch ---------------------------------------------------------
// A workgroup owns ONE chunk of 32 query rows (held in registers as an MFMA operand by all four waves) and
// sweeps over all keys twice: first for the row normalisers (online max / sum per row, folded over the
// waves through LDS), then again over the image keys for the column sums.  Nothing but the final column
// sums of the chunk leaves the workgroup, so the normaliser partials, their fold kernel and the second
// launch disappear; the price is that every chunk streams the keys from L2 itself, which only pays while
// the sequence is short (the launch decides by the bytes that re-streaming costs).  Wave w of NW takes the key
// tiles 32 (w + NW k) .. +32; a tile's rows go straight from global memory into operand registers, the next
// tile's loads are in flight while the current one is used (two named register sets).
#define LVLM_K16(M) M(0) M(1) M(2) M(3) M(4) M(5) M(6) M(7) M(8) M(9) M(10) M(11) M(12) M(13) M(14) M(15)

template <int DT, int HD, int NW>
__global__ __launch_bounds__(64 * NW, (DT == LVLM_F32 && HD == 128) ? 2 : 3) void score_small_kernel(ScoreArgs a) {
    constexpr int ES = esize<DT>();
    constexpr int NV = HalfRow<DT, HD>::NV;
    constexpr int SW = 32 * NW;             // keys all waves take per sweep step
    static_assert(NV <= 16, "operand registers are written out for up to 16 words");
    __shared__ float wm[NW][32], wl[NW][32];
    __shared__ float lse_s[32];
    __shared__ int pos_s[32];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int hf = lane >> 5, l32 = lane & 31;
    // Workgroups reach the 8 XCDs round-robin by id: all chunks of one (batch, KV head) pair are given ids
    // with the same remainder, so that the pair's keys are fetched into one L2 only
    const int xcd = blockIdx.x & 7, seq = blockIdx.x >> 3;
    const int pair = (seq / a.rs) * 8 + xcd, c = seq % a.rs;
    if (pair >= a.B * a.Hkv) return;
    const int b = pair / a.Hkv, g = pair % a.Hkv;
    const int GT = a.G * a.T;
    const long long rowbase = ((long long)b * a.Hq + (long long)g * a.G) * a.T;
    auto div_t = [&](int rho) -> int { return a.T == 1 ? rho : (int)__umulhi((unsigned)rho, a.t_magic); };

    // this lane's query row (padding rows repeat the last row and get an infinite LSE)
    const int rho = c * 32 + l32;
    const int rc = min(rho, GT - 1);
    const int hl = div_t(rc), qi = rc - hl * a.T;
    const int pos = a.causal ? a.q_pos0 + qi : INT_MAX;
    HalfRow<DT, HD> qa;
    {
        // contraction step i of lane half hf takes bytes [32 i + 16 hf, +16) of the row (the contraction index
        // is a dummy index: any split works as long as both operands use it): the two halves of one load
        // instruction then read 32 contiguous bytes of a row, half as many cache lines as with a half row each
        const char *src = a.q + ((long long)b * a.qsb + (long long)qi * a.qst + (long long)(g * a.G + hl) * a.qsh) * ES +
                          16 * hf;
#pragma unroll
        for (int i = 0; i < NV; ++i) qa.v[i] = *reinterpret_cast<const uint4 *>(src + 32 * i);
    }
    if (tid < 32) pos_s[tid] = pos;

    // loads: lane pair (2 r, 2 r + 1) reads 32 contiguous bytes of row r (half as many memory requests as one
    // row per lane); LVLM_PACK moves each piece to the lane (row l32, half hf) the MFMA wants it in
    const char *kbase = a.k + ((long long)b * a.ksb + (long long)g * a.ksh) * ES + 16 * (lane & 1);
    const int k_src = 4 * (2 * l32 + hf);
#define LVLM_DECL(x) uint4 kA##x = make_uint4(0, 0, 0, 0), kB##x = make_uint4(0, 0, 0, 0), kC##x = make_uint4(0, 0, 0, 0);
    LVLM_K16(LVLM_DECL)
#undef LVLM_DECL
#define LVLM_LD(S, x) if (x < NV) S##x = *reinterpret_cast<const uint4 *>(kp_ + 32 * x);
#define LVLM_LOADK(S, j0, jmax)                                                              \
    {                                                                                        \
        const char *kp_ = kbase + (long long)min((j0) + (lane >> 1), (jmax) - 1) * a.ksn * ES; \
        LVLM_LD(S, 0) LVLM_LD(S, 1) LVLM_LD(S, 2) LVLM_LD(S, 3) LVLM_LD(S, 4) LVLM_LD(S, 5) LVLM_LD(S, 6) LVLM_LD(S, 7) \
        LVLM_LD(S, 8) LVLM_LD(S, 9) LVLM_LD(S, 10) LVLM_LD(S, 11) LVLM_LD(S, 12) LVLM_LD(S, 13) LVLM_LD(S, 14) LVLM_LD(S, 15) \
    }
#define LVLM_PACK(S, kf)                                                                     \
    {                                                                                        \
        const uint4 w_[16] = {S##0, S##1, S##2, S##3, S##4, S##5, S##6, S##7, S##8, S##9, S##10, S##11, S##12, S##13, S##14, S##15}; \
        _Pragma("unroll") for (int i = 0; i < NV; ++i) {                                     \
            kf.v[i].x = __builtin_amdgcn_ds_bpermute(k_src, w_[i].x);                         \
            kf.v[i].y = __builtin_amdgcn_ds_bpermute(k_src, w_[i].y);                         \
            kf.v[i].z = __builtin_amdgcn_ds_bpermute(k_src, w_[i].z);                         \
            kf.v[i].w = __builtin_amdgcn_ds_bpermute(k_src, w_[i].w);                         \
        }                                                                                    \
    }

    // the first tile of the second sweep is fetched now: its latency hides behind the first sweep (where
    // the operand registers allow a third set)
    constexpr bool kEarly = NV <= 8;
    const int key_lo = a.img_begin, key_hi = a.img_begin + a.n_img;
    const int j2_first = key_lo + 32 * wave;
    if (kEarly && j2_first < key_hi) LVLM_LOADK(kC, j2_first, key_hi)

    // A tile whose keys all lie in range and at or before the earliest query position of the chunk needs no
    // per-element mask (uniform test): that is every image key for instruction rows.
    const int rho_last = min(c * 32 + 31, GT - 1);
    const int hc0 = div_t(c * 32), hc1 = div_t(rho_last);
    const int pos_min = a.causal ? a.q_pos0 + ((hc0 != hc1) ? 0 : c * 32 - hc0 * a.T) : INT_MAX;

    // ---- sweep 1: row normalisers over all keys (rows = keys, columns = queries: the row's statistics are
    // lane-local over 16 registers)
    if (a.row_lse == nullptr) {
        float m = -INFINITY, l = 0.f;
        auto stats = [&](int j0, const HalfRow<DT, HD> &kf) {
            f32x16 acc;
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[r] = 0.f;
            mma_tile<DT, HD>(acc, kf, qa);
            if (j0 + 32 <= a.N && j0 + 31 <= pos_min) {
                float tmax = acc[0];
#pragma unroll
                for (int r = 1; r < 16; ++r) tmax = fmaxf(tmax, acc[r]);
                const float mn = fmaxf(m, tmax * a.scale_log2);      // finite; scale >= 0 (checked on the host)
                float sum = 0.f;
#pragma unroll
                for (int r = 0; r < 16; ++r) sum += __builtin_amdgcn_exp2f(fmaf(acc[r], a.scale_log2, -mn));
                l = l * __builtin_amdgcn_exp2f(m - mn) + sum;
                m = mn;
                return;
            }
            float t[16];
            float tmax = -INFINITY;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int j = j0 + acc_row(r, hf);
                t[r] = (j <= pos && j < a.N) ? acc[r] * a.scale_log2 : -INFINITY;
                tmax = fmaxf(tmax, t[r]);
            }
            const float mn = fmaxf(m, tmax);
            const float ms = (mn == -INFINITY) ? 0.f : mn;
            float sum = 0.f;
#pragma unroll
            for (int r = 0; r < 16; ++r) sum += __builtin_amdgcn_exp2f(t[r] - ms);   // exp2(-inf) = 0
            l = l * __builtin_amdgcn_exp2f(m - ms) + sum;
            m = mn;
        };
        const int j_first = 32 * wave;
        if (j_first < a.N) LVLM_LOADK(kA, j_first, a.N)
        for (int j0 = j_first; j0 < a.N; j0 += 2 * SW) {
            HalfRow<DT, HD> kf;
            if (j0 + SW < a.N) LVLM_LOADK(kB, j0 + SW, a.N)
            LVLM_PACK(kA, kf)
            stats(j0, kf);
            if (j0 + SW >= a.N) break;
            if (j0 + 2 * SW < a.N) LVLM_LOADK(kA, j0 + 2 * SW, a.N)
            LVLM_PACK(kB, kf)
            stats(j0 + SW, kf);
        }
        // the two lane halves, then the four waves
        {
            const float mo = other_half(m), lo = other_half(l);
            const float mn = fmaxf(m, mo);
            const float ms = (mn == -INFINITY) ? 0.f : mn;
            l = l * __builtin_amdgcn_exp2f(m - ms) + lo * __builtin_amdgcn_exp2f(mo - ms);
            m = mn;
        }
        if (hf == 0) {
            wm[wave][l32] = m;
            wl[wave][l32] = l;
        }
        __syncthreads();
        if (tid < 32) {
            float mx = -INFINITY;
#pragma unroll
            for (int w = 0; w < NW; ++w) mx = fmaxf(mx, wm[w][tid]);
            const float ms = (mx == -INFINITY) ? 0.f : mx;
            float tot = 0.f;
#pragma unroll
            for (int w = 0; w < NW; ++w) tot += wl[w][tid] * exp2f(wm[w][tid] - ms);
            // no visible key, or a padding row: contributes nothing
            lse_s[tid] = (tot > 0.f && rho < GT) ? mx + log2f(tot) : INFINITY;
        }
    } else if (tid < 32) {
        lse_s[tid] = rho < GT ? a.row_lse[rowbase + rho] * kLog2e : INFINITY;
    }
    __syncthreads();

    // ---- sweep 2: column sums over the image keys (rows = queries, columns = keys: a key's sum is lane-local)
    float *out = a.colpart + (((long long)c * a.B + b) * a.Hkv + g) * a.n_img;
    auto colsum = [&](int j0, const HalfRow<DT, HD> &kf) {
        f32x16 acc;
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] = 0.f;
        mma_tile<DT, HD>(acc, qa, kf);
        const int j = j0 + l32;
        float sum = 0.f;
        if (j0 + 31 <= pos_min) {
#pragma unroll
            for (int r = 0; r < 16; ++r)
                sum += __builtin_amdgcn_exp2f(fmaf(acc[r], a.scale_log2, -lse_s[acc_row(r, hf)]));
        } else {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = acc_row(r, hf);
                const float p = __builtin_amdgcn_exp2f(fmaf(acc[r], a.scale_log2, -lse_s[row]));
                sum += (j <= pos_s[row]) ? p : 0.f;
            }
        }
        sum += other_half(sum);
        if (hf == 0 && j < key_hi) out[j - key_lo] = sum;
    };
    if (j2_first < key_hi) {
        HalfRow<DT, HD> kf;
        if (!kEarly) LVLM_LOADK(kC, j2_first, key_hi)
        if (j2_first + SW < key_hi) LVLM_LOADK(kB, j2_first + SW, key_hi)
        LVLM_PACK(kC, kf)
        colsum(j2_first, kf);
        for (int j0 = j2_first + SW; j0 < key_hi; j0 += 2 * SW) {      // tile j0 is in set B
            if (j0 + SW < key_hi) LVLM_LOADK(kA, j0 + SW, key_hi)
            LVLM_PACK(kB, kf)
            colsum(j0, kf);
            if (j0 + SW >= key_hi) break;
            if (j0 + 2 * SW < key_hi) LVLM_LOADK(kB, j0 + 2 * SW, key_hi)
            LVLM_PACK(kA, kf)
            colsum(j0 + SW, kf);
        }
    }
#undef LVLM_LD
#undef LVLM_LOADK
#undef LVLM_PACK
}
#undef LVLM_K16

// ---- short sequences, several query chunks per KV head: one launch, key tiles shared through LDS -------
// A workgroup owns FOUR chunks of 32 query rows of one (batch, KV head) pair, one per wave, each held in
// registers as an MFMA operand.  The keys are swept twice, tile by tile (32 keys): the 256 threads fetch a
// tile with fully coalesced 16-byte loads (16 lanes per row) two tiles ahead, copy it into one of two LDS
// buffers one tile ahead, and after one barrier per tile every wave reads it as its other operand -- the
// keys cross the memory pipeline once per workgroup instead of once per wave, and in whole 64-byte requests.
// Sweep 1 (rows = keys, columns = queries) leaves each lane the online (max, sum) of its own query row: no
// fold across waves; sweep 2 (rows = queries, columns = keys) over the image keys leaves each lane the
// column sum of its key for this wave's chunk, which is that chunk's part of the result.
// MODE 0: both sweeps in this launch.  MODE 1 / 2: the keys are cut into a.n_seg runs of whole tiles and a workgroup takes ONE
// run -- MODE 1 the normaliser sweep over it, leaving each row's (max, sum) of the run for score_lse_kernel to fold, MODE 2
// the column-sum sweep over it with the folded (or the caller's) normalisers.  A wave's unit of work is then a chunk over a
// run instead of a chunk over all keys twice, which is what lets a launch of few workgroups load every SIMD evenly.
template <int DT, int HD, int MODE>
__global__ __launch_bounds__(256, (DT == LVLM_F32 && HD == 128) ? 2 : 4) void score_chunks_kernel(ScoreArgs a) {
    constexpr int ES = esize<DT>();
    constexpr int ROWB = HD * ES;
    constexpr int PITCH = ROWB + 16;
    constexpr int NV = HalfRow<DT, HD>::NV;
    constexpr int UPR = ROWB / 16;          // 16-byte units per row
    constexpr int UPT = 32 * UPR / 256;     // units each thread stages per tile
    constexpr int TPR = UPR / UPT;          // threads per row
    static_assert(UPT >= 1 && UPT <= 4, "staging covers 1..4 units per thread");
    __shared__ __attribute__((aligned(16))) char k_lds[2][32 * PITCH];
    __shared__ float lse_s[4][32];
    __shared__ int pos_s[4][32];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int hf = lane >> 5, l32 = lane & 31;
    // all workgroups of one (batch, KV head) pair on one XCD (ids with the same remainder modulo 8)
    const int wpp = (a.rs + 3) >> 2;                      // workgroups per pair
    const int xcd = blockIdx.x & 7;
    const int seg = MODE == 0 ? 0 : (int)(blockIdx.x >> 3) % a.n_seg;      // this workgroup's run of keys
    const int seq = MODE == 0 ? (int)(blockIdx.x >> 3) : (int)(blockIdx.x >> 3) / a.n_seg;
    const int pair = (seq / wpp) * 8 + xcd;
    if (pair >= a.B * a.Hkv) return;
    const int b = pair / a.Hkv, g = pair % a.Hkv;
    const int c = (seq % wpp) * 4 + wave;                 // this wave's chunk
    const bool live = c < a.rs;                           // a wave without a chunk only helps to move tiles
    const int GT = a.G * a.T;
    const long long rowbase = ((long long)b * a.Hq + (long long)g * a.G) * a.T;
    auto div_t = [&](int rho) -> int { return a.T == 1 ? rho : (int)__umulhi((unsigned)rho, a.t_magic); };

    // this lane's query row (padding rows repeat the last row and get an infinite LSE)
    const int rho = c * 32 + l32;
    const int rc = min(rho, GT - 1);
    const int hl = div_t(rc), qi = rc - hl * a.T;
    const int pos = a.causal ? a.q_pos0 + qi : INT_MAX;
    HalfRow<DT, HD> qa;
    {
        const char *src = a.q + ((long long)b * a.qsb + (long long)qi * a.qst + (long long)(g * a.G + hl) * a.qsh) * ES +
                          16 * hf;
#pragma unroll
        for (int i = 0; i < NV; ++i) qa.v[i] = *reinterpret_cast<const uint4 *>(src + 32 * i);
    }
    if (hf == 0) pos_s[wave][l32] = pos;
    // earliest position of the chunk's rows (uniform per wave): tiles at or before it need no mask
    const int rho_last = min(c * 32 + 31, GT - 1);
    const int hc0 = div_t(min(c * 32, GT - 1)), hc1 = div_t(rho_last);
    const int pos_min = a.causal ? a.q_pos0 + ((hc0 != hc1) ? 0 : min(c * 32, GT - 1) - hc0 * a.T) : INT_MAX;

    // staging: thread -> row srow of the tile, units scu + TPR x
    const int srow = tid / TPR, scu = tid % TPR;
    const char *kbase = a.k + ((long long)b * a.ksb + (long long)g * a.ksh) * ES + 16 * scu;
    uint4 st0 = make_uint4(0, 0, 0, 0), st1 = st0, st2 = st0, st3 = st0;
    auto fetch = [&](int j0, int j_end) {                 // tile rows j0 .. j0+31, clamped to the range
        const uint4 *src = reinterpret_cast<const uint4 *>(kbase + (long long)min(j0 + srow, j_end - 1) * a.ksn * ES);
        st0 = src[0];
        if constexpr (UPT > 1) st1 = src[TPR];
        if constexpr (UPT > 2) st2 = src[2 * TPR];
        if constexpr (UPT > 3) st3 = src[3 * TPR];
    };
    auto stash = [&](int buf) {
        uint4 *dst = reinterpret_cast<uint4 *>(&k_lds[buf][srow * PITCH + 16 * scu]);
        dst[0] = st0;
        if constexpr (UPT > 1) dst[TPR] = st1;
        if constexpr (UPT > 2) dst[2 * TPR] = st2;
        if constexpr (UPT > 3) dst[3 * TPR] = st3;
    };
    auto tile_operand = [&](int buf, HalfRow<DT, HD> &kf) {
        const char *src = &k_lds[buf][l32 * PITCH + 16 * hf];
#pragma unroll
        for (int i = 0; i < NV; ++i) kf.v[i] = *reinterpret_cast<const uint4 *>(src + 32 * i);
    };

    // ---- sweep 1: this lane's row normaliser over all keys
    float m = -INFINITY, l = 0.f;
    // SAFE = false: after the first whole tile has set a finite reference m, later whole tiles take it as it is --
    // no maximum, no rescaling; a logit far above it shows as an overflowing sum, checked after the sweep, and the
    // workgroup then repeats the sweep with SAFE = true (the reference follows the running maximum on every tile).
    auto stats = [&](int j0, bool first, const HalfRow<DT, HD> &kf, auto safe_tag) {
        constexpr bool SAFE = decltype(safe_tag)::value;
        f32x16 acc;
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] = 0.f;
        mma_tile<DT, HD>(acc, kf, qa);                    // rows = keys, columns = queries
        if (j0 + 32 <= a.N && j0 + 31 <= pos_min) {
            if (!SAFE && !first) {                        // the sweep's first tile was whole too (tiles ascend): m is finite
                float sum = 0.f;
#pragma unroll
                for (int r = 0; r < 16; ++r) sum += __builtin_amdgcn_exp2f(fmaf(acc[r], a.scale_log2, -m));
                l += sum;
                return;
            }
            float tmax = acc[0];
#pragma unroll
            for (int r = 1; r < 16; ++r) tmax = fmaxf(tmax, acc[r]);
            const float mn = fmaxf(m, tmax * a.scale_log2);      // finite; scale >= 0 (checked on the host)
            float sum = 0.f;
#pragma unroll
            for (int r = 0; r < 16; ++r) sum += __builtin_amdgcn_exp2f(fmaf(acc[r], a.scale_log2, -mn));
            l = l * __builtin_amdgcn_exp2f(m - mn) + sum;
            m = mn;
            return;
        }
        float t[16];
        float tmax = -INFINITY;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int j = j0 + acc_row(r, hf);
            t[r] = (j <= pos && j < a.N) ? acc[r] * a.scale_log2 : -INFINITY;
            tmax = fmaxf(tmax, t[r]);
        }
        const float mn = fmaxf(m, tmax);
        const float ms = (mn == -INFINITY) ? 0.f : mn;
        float sum = 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) sum += __builtin_amdgcn_exp2f(t[r] - ms);   // exp2(-inf) = 0
        l = l * __builtin_amdgcn_exp2f(m - ms) + sum;
        m = mn;
    };
    // ---- sweep 2: column sums of the image keys for this wave's chunk
    const int key_lo = a.img_begin, key_hi = a.img_begin + a.n_img;
    float *out = a.colpart + (((long long)min(c, a.rs - 1) * a.B + b) * a.Hkv + g) * a.n_img;
    float lse_r[16];                                      // the normalisers of this lane's 16 accumulator rows
    auto colsum = [&](int j0, const HalfRow<DT, HD> &kf) {
        f32x16 acc;
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] = 0.f;
        mma_tile<DT, HD>(acc, qa, kf);                    // rows = queries, columns = keys
        const int j = j0 + l32;
        float sum = 0.f;
        if (j0 + 31 <= pos_min) {
#pragma unroll
            for (int r = 0; r < 16; ++r) sum += __builtin_amdgcn_exp2f(fmaf(acc[r], a.scale_log2, -lse_r[r]));
        } else {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float p = __builtin_amdgcn_exp2f(fmaf(acc[r], a.scale_log2, -lse_r[r]));
                sum += (j <= pos_s[wave][acc_row(r, hf)]) ? p : 0.f;
            }
        }
        sum += other_half(sum);
        if (hf == 0 && j < key_hi) out[j - key_lo] = sum;
    };

    // One sweep: tile t is fetched in iteration t-2, copied to LDS in iteration t-1 and used in iteration t
    // (one barrier per tile publishes the copy; fetches past the last tile repeat its last row).
    auto sweep = [&](int j_begin, int j_end, bool second, auto safe_tag) {
        const int nt = (j_end - j_begin + 31) >> 5;
        fetch(j_begin, j_end);
        stash(0);
        fetch(j_begin + 32, j_end);
        __syncthreads();
        for (int t = 0; t < nt; ++t) {
            stash((t + 1) & 1);                           // tile t+1
            fetch(j_begin + 32 * (t + 2), j_end);
            if (live) {
                HalfRow<DT, HD> kf;
                tile_operand(t & 1, kf);
                if (second) colsum(j_begin + 32 * t, kf);
                else stats(j_begin + 32 * t, t == 0, kf, safe_tag);
            }
            __syncthreads();
        }
    };

    // the tiles of [lo, hi) this workgroup takes: all of them, or its run (equal shares of whole tiles)
    auto run_of = [&](int lo, int hi, int &jb, int &je) {
        jb = lo, je = hi;
        if (MODE != 0) {
            const long long nt = (hi - lo + 31) >> 5;
            jb = lo + 32 * (int)(nt * seg / a.n_seg);
            je = min(hi, lo + 32 * (int)(nt * (seg + 1) / a.n_seg));
        }
    };
    if (MODE == 1 || (MODE == 0 && a.row_lse == nullptr)) {
        int jb, je;
        run_of(0, a.N, jb, je);
        if (jb < je) {
            sweep(jb, je, false, std::false_type{});
            if (__syncthreads_or(!(l < 1.0e30f))) {       // some sum ran away (or is not a number): the careful sweep
                m = -INFINITY, l = 0.f;
                sweep(jb, je, false, std::true_type{});
            }
        }
        {
            const float mo = other_half(m), lo = other_half(l);
            const float mn = fmaxf(m, mo);
            const float ms = (mn == -INFINITY) ? 0.f : mn;
            l = l * __builtin_amdgcn_exp2f(m - ms) + lo * __builtin_amdgcn_exp2f(mo - ms);
            m = mn;
        }
        if (MODE == 1) {                                  // this run's share of the rows' normalisers
            if (hf == 0 && live && rho < GT) {
                const long long pidx = (long long)seg * a.B * a.Hq * a.T + rowbase + rho;
                a.part_m[pidx] = m;
                a.part_l[pidx] = l;
            }
            return;
        }
        // no visible key, or a padding row: contributes nothing
        if (hf == 0) lse_s[wave][l32] = (l > 0.f && rho < GT) ? m + log2f(l) : INFINITY;
    } else if (hf == 0) {
        const bool real = live && rho < GT;
        lse_s[wave][l32] = !real ? INFINITY : (a.row_lse ? a.row_lse[rowbase + rho] * kLog2e : a.lse2[rowbase + rho]);
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < 16; ++r) lse_r[r] = lse_s[wave][acc_row(r, hf)];
    int jb, je;
    run_of(key_lo, key_hi, jb, je);
    if (jb < je) sweep(jb, je, true, std::true_type{});
}

// Fold the per-block, per-wave (max, sum) pairs of each row into a log2-domain LSE.  Eight lanes share a
// row: each folds every eighth pair online, then the eight partial (max, sum) states are merged.
__global__ __launch_bounds__(256) void score_lse_kernel(const float *part_m, const float *part_l, float *lse2,
                                                        int rows, int nparts) {
    const int t = blockIdx.x * 256 + threadIdx.x;
    const int row = t >> 3, sub = t & 7;
    float m = -INFINITY, l = 0.f;
    if (row < rows) {
#pragma unroll 4
        for (int i = sub; i < nparts; i += 8) {
            const float mi = part_m[(long long)i * rows + row];
            const float li = part_l[(long long)i * rows + row];
            const float mn = fmaxf(m, mi);
            const float ms = (mn == -INFINITY) ? 0.f : mn;
            l = l * exp2f(m - ms) + li * exp2f(mi - ms);      // exp2(-inf) = 0 covers empty blocks
            m = mn;
        }
    }
#pragma unroll
    for (int o = 1; o < 8; o <<= 1) {
        const float mo = __shfl_xor(m, o), lo = __shfl_xor(l, o);
        const float mn = fmaxf(m, mo);
        const float ms = (mn == -INFINITY) ? 0.f : mn;
        l = l * exp2f(m - ms) + lo * exp2f(mo - ms);
        m = mn;
    }
    if (row < rows && sub == 0) lse2[row] = (l > 0.f) ? m + log2f(l) : INFINITY;   // no visible key: contributes nothing
}

// score_head[b][g][j] = (sum over row splits of the column sums) / G;  score_mean[b][j] = mean over g.
// Four heads x eight splits are loaded together so that the loads overlap; more splits take more rounds
// (a fixed summation order either way).
constexpr int kMaxRowSplit = 8;

__global__ __launch_bounds__(256) void score_finalize_kernel(ScoreArgs a) {
    const int j = blockIdx.x * 256 + threadIdx.x;
    const int b = blockIdx.y;
    if (j >= a.n_img) return;
    const float inv_g = 1.0f / (float)a.G;
    const long long split_stride = (long long)a.B * a.Hkv * a.n_img;
    float mean = 0.f;
    for (int g0 = 0; g0 < a.Hkv; g0 += 4) {
        float tot[4] = {0.f, 0.f, 0.f, 0.f};
        for (int r0 = 0; r0 < a.rs; r0 += kMaxRowSplit) {
            float v[4][kMaxRowSplit];
#pragma unroll
            for (int gg = 0; gg < 4; ++gg)
#pragma unroll
                for (int r = 0; r < kMaxRowSplit; ++r) {
                    const bool on = g0 + gg < a.Hkv && r0 + r < a.rs;
                    const int gc = min(g0 + gg, a.Hkv - 1), rc = min(r0 + r, a.rs - 1);
                    const float x = a.colpart[rc * split_stride + ((long long)b * a.Hkv + gc) * a.n_img + j];
                    v[gg][r] = on ? x : 0.f;
                }
#pragma unroll
            for (int gg = 0; gg < 4; ++gg) {
                float s = 0.f;
#pragma unroll
                for (int r = 0; r < kMaxRowSplit; ++r) s += v[gg][r];
                tot[gg] += s;
            }
        }
#pragma unroll
        for (int gg = 0; gg < 4; ++gg) {
            if (g0 + gg >= a.Hkv) break;
            float s = tot[gg];
            s *= inv_g;
            a.score_head[(long long)b * a.shb + (long long)(g0 + gg) * a.shh + j] = s;
            mean += s;
        }
    }
    a.score_mean[(long long)b * a.n_img + j] = mean / (float)a.Hkv;
}

// ---- scores from probabilities the caller already holds ---------------------------------------------
// Workgroup (column block, row group c): thread j sums probs[b][g*G + hl][i][img_begin + j] over the 32
// rows rho = hl*T + i of group c (neighbouring threads read neighbouring columns), all 32 loads in flight;
// the per-group sums go through the same finalize kernel as the column sums of the passes.
struct ProbsArgs {
    const char *p;
    float *colpart;
    int B, T, Hkv, G, img_begin, n_img;
    unsigned t_magic;
    long long psb, psh, pst;
};

template <int DT>
__global__ __launch_bounds__(256) void probs_colsum_kernel(ProbsArgs a, int n_col_blocks) {
    constexpr int ES = esize<DT>();
    const int cb = blockIdx.x % n_col_blocks, c = blockIdx.x / n_col_blocks;
    const int g = blockIdx.y, b = blockIdx.z;
    const int j = cb * 256 + threadIdx.x;
    if (j >= a.n_img) return;
    const int GT = a.G * a.T;
    const int r0 = c * 32, r1 = min(GT, r0 + 32);
    const char *base = a.p + ((long long)b * a.psb + (long long)g * a.G * a.psh + a.img_begin + j) * ES;
    auto at = [&](int rho) -> float {
        const int hl = a.T == 1 ? rho : (int)__umulhi((unsigned)rho, a.t_magic), i = rho - hl * a.T;
        const char *q = base + ((long long)hl * a.psh + (long long)i * a.pst) * ES;
        if constexpr (DT == LVLM_BF16) return bf16_to_f32(*reinterpret_cast<const uint16_t *>(q));
        else return *reinterpret_cast<const float *>(q);
    };
    // all 32 loads of the group are issued before the first is used
    float v[32];
#pragma unroll
    for (int u = 0; u < 32; ++u) v[u] = r0 + u < r1 ? at(r0 + u) : 0.f;
    float sum = 0.f;
#pragma unroll
    for (int u = 0; u < 32; ++u) sum += v[u];
    a.colpart[(((long long)c * a.B + b) * a.Hkv + g) * a.n_img + j] = sum;
}

// The same with 16-byte loads, for probabilities whose rows and image span start on 16-byte boundaries and
// whose image span is a whole number of 16-byte words: thread (sub, cj) sums 8 rows (group c, rows 8 sub ..)
// of the 16 / ES columns of word cj; the four row subsets are folded through LDS.
template <int DT>
__global__ __launch_bounds__(256) void probs_colsum_vec_kernel(ProbsArgs a, int n_col_blocks) {
    constexpr int ES = esize<DT>();
    constexpr int CPT = 16 / ES;              // columns per thread
    constexpr int WC = 64 * CPT;              // columns per workgroup
    __shared__ float part[4][WC];
    const int cb = blockIdx.x % n_col_blocks, c = blockIdx.x / n_col_blocks;
    const int g = blockIdx.y, b = blockIdx.z;
    const int sub = threadIdx.x >> 6, cj = threadIdx.x & 63;
    const int j0 = cb * WC + cj * CPT;
    const int GT = a.G * a.T;
    const int r0 = c * 32 + 8 * sub, r1 = min(GT, r0 + 8);
    float acc[CPT];
#pragma unroll
    for (int e = 0; e < CPT; ++e) acc[e] = 0.f;
    if (j0 < a.n_img) {
        const char *base = a.p + ((long long)b * a.psb + (long long)g * a.G * a.psh + a.img_begin + j0) * ES;
        uint4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int rho = min(r0 + u, GT - 1);
            const int hl = a.T == 1 ? rho : (int)__umulhi((unsigned)rho, a.t_magic), i = rho - hl * a.T;
            v[u] = *reinterpret_cast<const uint4 *>(base + ((long long)hl * a.psh + (long long)i * a.pst) * ES);
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            if (r0 + u >= r1) continue;
            const uint32_t w[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                if constexpr (DT == LVLM_BF16) {
                    acc[2 * q] += __uint_as_float(w[q] << 16);
                    acc[2 * q + 1] += __uint_as_float(w[q] & 0xffff0000u);
                } else {
                    acc[q] += __uint_as_float(w[q]);
                }
            }
        }
    }
#pragma unroll
    for (int e = 0; e < CPT; ++e) part[sub][cj * CPT + e] = acc[e];
    __syncthreads();
    for (int x = threadIdx.x; x < WC; x += 256) {
        const int j = cb * WC + x;
        if (j < a.n_img)
            a.colpart[(((long long)c * a.B + b) * a.Hkv + g) * a.n_img + j] =
                (part[0][x] + part[1][x]) + (part[2][x] + part[3][x]);
    }
}

template <int DT, int HD, int KPW>
void launch_passes(const Prof &prof, const ScoreArgs &a, bool need_lse, bool single, bool shared_tiles) {
    hipStream_t stream = prof.stream;
    constexpr int BN = 4 * KPW * 32;
    if (single) {
        prof.begin("score_single");
        if (shared_tiles && a.n_seg > 1) {
            // the keys in runs: the normaliser sweep, the fold of the runs' partials, then the column-sum sweep
            const dim3 grid((a.B * a.Hkv + 7) / 8 * 8 * ((a.rs + 3) / 4) * a.n_seg);
            if (need_lse) {
                LVLM_LAUNCH(prof, (score_chunks_kernel<DT, HD, 1>), grid, dim3(256), 0, stream, a);
                prof.end();
                const int rows = a.B * a.Hq * a.T;
                prof.begin("score_lse");
                LVLM_LAUNCH(prof, score_lse_kernel, dim3((rows * 8 + 255) / 256), dim3(256), 0, stream, a.part_m, a.part_l,
                                   a.lse2, rows, a.n_seg);
                prof.end();
                prof.begin("score_single");
            }
            LVLM_LAUNCH(prof, (score_chunks_kernel<DT, HD, 2>), grid, dim3(256), 0, stream, a);
        } else if (shared_tiles)
            LVLM_LAUNCH(prof, (score_chunks_kernel<DT, HD, 0>), dim3((a.B * a.Hkv + 7) / 8 * 8 * ((a.rs + 3) / 4)), dim3(256), 0,
                               stream, a);
        else
            LVLM_LAUNCH(prof, (score_small_kernel<DT, HD, 4>), dim3((a.B * a.Hkv + 7) / 8 * 8 * a.rs), dim3(256), 0, stream,
                               a);
        prof.end();
        prof.begin("score_finalize");
        LVLM_LAUNCH(prof, score_finalize_kernel, dim3((a.n_img + 255) / 256, a.B), dim3(256), 0, stream, a);
        prof.end();
        return;
    }
    if (need_lse) {
        dim3 grid0(((a.N + BN - 1) / BN + 7) / 8 * 8 * a.rs, a.Hkv, a.B);
        prof.begin("score_pass0");
        LVLM_LAUNCH(prof, (score_pass_kernel<DT, HD, KPW, 0>), grid0, dim3(256), 0, stream, a);
        prof.end();
        const int rows = a.B * a.Hq * a.T;
        prof.begin("score_lse");
        LVLM_LAUNCH(prof, score_lse_kernel, dim3((rows * 8 + 255) / 256), dim3(256), 0, stream, a.part_m, a.part_l,
                           a.lse2, rows, a.nkb * 4);
        prof.end();
    }
    dim3 grid1(((a.n_img + BN - 1) / BN + 7) / 8 * 8 * a.rs, a.Hkv, a.B);
    prof.begin("score_pass1");
    LVLM_LAUNCH(prof, (score_pass_kernel<DT, HD, KPW, 1>), grid1, dim3(256), 0, stream, a);
    prof.end();
    prof.begin("score_finalize");
    LVLM_LAUNCH(prof, score_finalize_kernel, dim3((a.n_img + 255) / 256, a.B), dim3(256), 0, stream, a);
    prof.end();
}

}  // namespace

constexpr int kRowSplitWgs = 1536;      // workgroups the two-pass kernels aim for
constexpr int kSingleMaxChunks = 32;
constexpr int kSharedMinWgs = 192;       // workgroups of four chunks from which the shared-tile form is taken
constexpr int kSingleMaxRows = 1100;      // in 256-byte key rows, one chunk per workgroup
constexpr int kSharedMaxRows = 8192;      // ... four chunks per workgroup sharing the key tiles

ProbsWs probs_ws(const lvlm_probs_desc &d) {
    ProbsWs w{};
    w.rs = (d.Hq / d.Hkv * d.T + 31) / 32;
    w.colpart = 0;
    w.total = align_up((size_t)w.rs * d.B * d.Hkv * d.n_img * sizeof(float), 256);
    return w;
}

hipError_t launch_score_probs(const Prof &prof, const lvlm_probs_desc &d, const ProbsWs &w, char *ws, const void *probs,
                              float *score_head, float *score_mean) {
    ProbsArgs pa{};
    pa.p = static_cast<const char *>(probs);
    pa.colpart = reinterpret_cast<float *>(ws + w.colpart);
    pa.B = d.B; pa.T = d.T; pa.Hkv = d.Hkv; pa.G = d.Hq / d.Hkv; pa.img_begin = d.img_begin; pa.n_img = d.n_img;
    pa.t_magic = (unsigned)(0x100000000ull / (unsigned long long)d.T) + 1u;
    pa.psb = d.p_stride_b; pa.psh = d.p_stride_h; pa.pst = d.p_stride_t;
    const int es = d.dtype == LVLM_BF16 ? 2 : 4, cpt = 16 / es;
    const bool vec = (d.p_stride_b * es) % 16 == 0 && (d.p_stride_h * es) % 16 == 0 && (d.p_stride_t * es) % 16 == 0 &&
                     (d.img_begin * es) % 16 == 0 && d.n_img % cpt == 0;      // the base pointer is 16-byte aligned
    prof.begin("score_probs");
    if (vec) {
        const int ncb = (d.n_img + 64 * cpt - 1) / (64 * cpt);
        const dim3 grid(ncb * w.rs, d.Hkv, d.B);
        if (d.dtype == LVLM_BF16)
            LVLM_LAUNCH(prof, probs_colsum_vec_kernel<LVLM_BF16>, grid, dim3(256), 0, prof.stream, pa, ncb);
        else
            LVLM_LAUNCH(prof, probs_colsum_vec_kernel<LVLM_F32>, grid, dim3(256), 0, prof.stream, pa, ncb);
    } else {
        const int ncb = (d.n_img + 255) / 256;
        const dim3 grid(ncb * w.rs, d.Hkv, d.B);
        if (d.dtype == LVLM_BF16)
            LVLM_LAUNCH(prof, probs_colsum_kernel<LVLM_BF16>, grid, dim3(256), 0, prof.stream, pa, ncb);
        else
            LVLM_LAUNCH(prof, probs_colsum_kernel<LVLM_F32>, grid, dim3(256), 0, prof.stream, pa, ncb);
    }
    prof.end();
    ScoreArgs a{};
    a.colpart = pa.colpart;
    a.rs = w.rs;
    a.score_head = score_head;
    a.score_mean = score_mean;
    a.B = d.B; a.Hkv = d.Hkv; a.G = pa.G; a.n_img = d.n_img;
    const bool dense = d.sh_stride_b == 0 && d.sh_stride_h == 0;
    a.shh = dense ? d.n_img : d.sh_stride_h;
    a.shb = dense ? (long long)d.Hkv * d.n_img : d.sh_stride_b;
    prof.begin("score_finalize");
    LVLM_LAUNCH(prof, score_finalize_kernel, dim3((d.n_img + 255) / 256, d.B), dim3(256), 0, prof.stream, a);
    prof.end();
    return hipGetLastError();
}

ScoreWs score_ws(const lvlm_score_desc &d) {
    ScoreWs w{};
    // Wide key blocks (2 tiles per wave) once they still give every CU two workgroups.
    const long long wide = (long long)d.B * d.Hkv * ((d.N + 255) / 256);
    w.block_keys = (d.dtype == LVLM_BF16 && wide >= 512) ? 256 : 128;
    w.nkb = (d.N + w.block_keys - 1) / w.block_keys;
    // Few workgroups: split the query chunks of a key block over several workgroups (>= 2 chunks each), up to six
    // workgroups per compute unit (measured on 16512 keys of one sequence: 110 us for both passes with 520
    // workgroups, 98 us with 1560).
    const int n_chunks = (d.Hq / d.Hkv * d.T + 31) / 32;
    const long long wgs = (long long)d.B * d.Hkv * w.nkb;
    int rs = (int)((kRowSplitWgs + wgs - 1) / wgs);
    if (rs > (n_chunks + 1) / 2) rs = (n_chunks + 1) / 2;
    if (rs > 8) rs = 8;            // kMaxRowSplit of the finalize kernel
    if (rs < 1) rs = 1;
    w.cps = (n_chunks + rs - 1) / rs;
    w.rs = (n_chunks + w.cps - 1) / w.cps;
    // Short sequences: both passes in ONE launch (the column sums then come in one part per chunk).  Two
    // shapes: four chunks per workgroup that share the key tiles through LDS, when that still fills the
    // chip -- measured faster than the two-pass kernels up to several thousand keys (it saves the partials,
    // their fold and a launch) -- else one chunk per workgroup whose waves split the keys and fetch them
    // themselves, which pays up to the length where the three launches it replaces cost the same.
    const long long sweep_rows = (long long)d.N * (d.hd * (d.dtype == LVLM_BF16 ? 2 : 4)) / 256;
    w.shared_tiles = n_chunks >= 3 && n_chunks <= kSingleMaxChunks && (long long)d.B * d.Hkv * ((n_chunks + 3) / 4) >= kSharedMinWgs &&
                     sweep_rows <= kSharedMaxRows;
    w.single = w.shared_tiles || (n_chunks <= kSingleMaxChunks && sweep_rows <= kSingleMaxRows);
    // The shared-tile kernel with the keys in runs.  A wave's unit of work is a chunk over ALL keys, twice: a launch of
    // 2.25 workgroups per compute unit takes the time of three, one of 0.75 the time of one whose lone wave per SIMD hides
    // nothing, and one long sequence has too few workgroups for the form at all.  Cutting the keys into runs (a launch
    // per sweep, a workgroup per four chunks and run, the runs' normaliser partials folded in between) makes the units
    // small and many; it costs each workgroup its start-up (about three tiles' time) per run and the call two more
    // launches.  Taken when the estimate below says it saves more than 12 us over the form chosen so far.
    w.key_segs = 1;
    if (n_chunks >= 3 && n_chunks <= kSingleMaxChunks && (w.shared_tiles || !w.single)) {
        const long long wgs = (long long)d.B * d.Hkv * ((n_chunks + 3) / 4);
        const double tiles = (d.N + 31) / 32 + (d.n_img + 31) / 32;          // both sweeps
        // (measured, in us per tile sweep of a workgroup, with k = 1..5 workgroups resident on every compute unit: a lone
        // wave per SIMD hides nothing, from three on the SIMDs are saturated; five are resident at most, a launch of more
        // runs in turns of 1280 workgroups plus the rest)
        auto launch_us = [](long long n_wg, double tiles_per_wg) {
            static const double per_tile[6] = {0.0, 0.53, 0.73, 0.95, 1.25, 1.5};
            const long long turns = n_wg / 1280, rest = n_wg % 1280;
            return tiles_per_wg * (1.5 * (double)turns + per_tile[(rest + 255) / 256]);
        };
        // the form chosen so far: one launch of this kernel, or the two-pass kernels (0.53 PFLOP/s measured on one
        // sequence of 16512 keys: 0.002 us per workgroup-tile of this kernel's size) with their fold
        const double so_far = w.shared_tiles ? launch_us(wgs, tiles) : 0.002 * (double)wgs * tiles + 12.0;
        double best = so_far - 12.0;
        for (int s = 2; s <= 32 && (wgs <= 1280 || !w.shared_tiles); s *= 2) {
            if (tiles / 2 / s < 12) break;                                    // runs of at least 12 tiles
            if (wgs * s < kSharedMinWgs || sweep_rows / s > kSharedMaxRows) continue;
            const double cut = launch_us(wgs * s, tiles / s + 2 * 3) + 10.0;
            if (cut < best) best = cut, w.key_segs = s;
        }
        if (w.key_segs > 1) w.shared_tiles = w.single = true;
    }
    if (w.single) {
        w.rs = n_chunks;
        w.cps = 1;
    }
    const size_t rows = (size_t)d.B * d.Hq * d.T;
    w.part_m = 0;
    const size_t n_part = (size_t)w.nkb * 4 > (size_t)w.key_segs ? (size_t)w.nkb * 4 : (size_t)w.key_segs;
    w.part_l = align_up(w.part_m + rows * n_part * sizeof(float), 256);
    w.lse2 = align_up(w.part_l + rows * n_part * sizeof(float), 256);
    w.colpart = align_up(w.lse2 + rows * sizeof(float), 256);
    w.total = align_up(w.colpart + (size_t)w.rs * d.B * d.Hkv * d.n_img * sizeof(float), 256);
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
    a.colpart = reinterpret_cast<float *>(ws + w.colpart);
    a.rs = w.rs;
    a.cps = w.cps;
    a.n_seg = w.key_segs;
    a.t_magic = (unsigned)(0x100000000ull / (unsigned long long)d.T) + 1u;
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
        if (wide) launch_passes<LVLM_BF16, 128, 2>(prof, a, need_lse, w.single, w.shared_tiles);
        else launch_passes<LVLM_BF16, 128, 1>(prof, a, need_lse, w.single, w.shared_tiles);
    } else if (d.dtype == LVLM_BF16 && d.hd == 64) {
        if (wide) launch_passes<LVLM_BF16, 64, 2>(prof, a, need_lse, w.single, w.shared_tiles);
        else launch_passes<LVLM_BF16, 64, 1>(prof, a, need_lse, w.single, w.shared_tiles);
    } else if (d.dtype == LVLM_F32 && d.hd == 128) {
        launch_passes<LVLM_F32, 128, 1>(prof, a, need_lse, w.single, w.shared_tiles);
    } else {
        launch_passes<LVLM_F32, 64, 1>(prof, a, need_lse, w.single, w.shared_tiles);
    }
    return hipGetLastError();
}

}  // namespace lvlm
