// Step 6 -- one decode step of grouped-query attention over the retained,
// per-head ragged KV cache (Sec. 3.2.2), with the optional importance update
// that continues the received-attention score of Sec. 3.2.1 into decoding.
//
// The step streams K and V of every retained entry once; everything else is
// arranged around that stream:
//   attn_partial_kernel  grid (split, KV head, batch).  A wave takes 32 entries
//       at a time.  K rows go straight from global memory into the A operand of
//       a 32x32 MFMA (rows = entries, columns = the G query heads of the group,
//       padded), V rows are loaded in their natural, fully coalesced layout.
//       Softmax is online (fp32, log2 domain); the 32 x G probabilities pass
//       through a wave-private LDS tile so that P.V can run on the vector ALUs
//       against the natural V layout.  Each workgroup leaves (max, sum, o) of
//       its split and, if importance is tracked, the raw logits of its entries.
//       The entry being appended is taken from k_new / v_new instead of the
//       cache, so no workgroup depends on another one's write.
//   attn_combine_kernel  folds the splits, writes the output rows, turns the
//       logits into normalised probabilities for the importance update and
//       publishes the new length.
#include <type_traits>

#include "common.h"
#include "mma.h"

namespace lvlm {
namespace {


// What a head's first workgroup tells the fold kernel besides the attended length.
constexpr int kAppended = 1;    // the new entry went into the cache: the length is to be published
constexpr int kTruncated = 2;   // the head is longer than the caller's bound: only its first `bound` entries were
                                // attended to; its length is left alone and nothing is evicted

// The entries a head attends to.  A head with room below the caller's bound (len_bound, at most Lmax) takes the new
// entry; a full head does not (the entry is dropped, nothing is overwritten); a head already longer than the bound
// is read up to the bound only.  Every index derived from L therefore stays below the bound the workspace and the
// grids were sized for.
struct HeadLen {
    int L, new_slot, flags;
};
__device__ __forceinline__ HeadLen head_len(int len0, int bound, int append) {
    HeadLen h;
    const bool app = append && len0 < bound;
    h.L = min(len0, bound) + (app ? 1 : 0);
    h.new_slot = app ? h.L - 1 : -1;
    h.flags = (app ? kAppended : 0) | (len0 > bound ? kTruncated : 0);
    return h;
}

struct AttnArgs {
    const char *q;
    const char *k_new;
    const char *v_new;
    char *k;
    char *v;
    float *score;
    uint8_t *kind;
    int32_t *pos;
    int32_t *len;
    char *out;
    float *part_ml;     // [B*Hkv][n_split][GP][2]
    float *part_o;      // [B*Hkv][n_split][GP][HD]
    float *logits;      // [B*Hkv][GP][Lcap]  log2-domain logits of every head and entry (Lcap: whole tiles)
    int32_t *cur_len;   // [B*Hkv][2]  entries attended to; flags (kAppended, kTruncated)
    int Hq, Hkv, G, Lmax, Lcap, bound, n_split, split_len, append, new_kind, new_pos, update_score;
    int evict_budget, evict_recent;
    int tail_entry;     // the last split's wave 0 also takes the single entry at slot n_split * split_len
    float scale_log2, decay;
};


// One operand fragment of the P.V product: 8 probabilities as bf16 (round-to-nearest-even, the packed conversion
// instruction of this chip: one instruction per pair).
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2_t{lo, hi}, bf16x2_t));
}
__device__ __forceinline__ bf16x8 pack_bf16x8(const float *p) {
    uint4 u;
    u.x = pack_bf16x2(p[0], p[1]);
    u.y = pack_bf16x2(p[2], p[3]);
    u.z = pack_bf16x2(p[4], p[5]);
    u.w = pack_bf16x2(p[6], p[7]);
    return __builtin_bit_cast(bf16x8, u);
}

template <int DT, int HD>
struct TileRegs {
    static constexpr int ROWB = HD * esize<DT>();
    static constexpr int UPR = ROWB / 16;
    static constexpr int KSUB = 64 / UPR;
    static constexpr int VPL = 32 / KSUB;
    HalfRow<DT, HD> kf;   // K rows as the MFMA A operand: lane = (entry l32, half hf)
    uint4 vv[VPL];        // V rows in natural layout: lane = (unit lane % UPR, entry lane / UPR + KSUB * i)
};

template <int DT, int HD, int GP>
__global__ __launch_bounds__(256) void attn_partial_kernel(AttnArgs a) {
    constexpr int ES = esize<DT>();
    constexpr int ROWB = HD * ES;
    constexpr int NV = HalfRow<DT, HD>::NV;
    constexpr int UPR = ROWB / 16;        // 16-byte units per row
    constexpr int KSUB = 64 / UPR;        // rows a wave covers with one load instruction
    constexpr int VPL = 32 / KSUB;        // V units per lane per 32-entry tile
    constexpr int NB = HD / 32;           // 32-row blocks of the transposed output
    constexpr int VPITCH = ROWB + 16;     // LDS row pitch of the V tile: the two lane halves hit different banks
    static_assert(UPR <= 64 && KSUB >= 1, "row too long for one wave");

    __shared__ __attribute__((aligned(16))) char v_lds[4][32 * VPITCH];
    __shared__ float wm[4][GP], wl[4][GP];
    __shared__ __attribute__((aligned(16))) float wo[4][GP][HD];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int hf = lane >> 5, l32 = lane & 31;
    const int split = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
    const int hg = b * a.Hkv + g;
    const long long cbase = (long long)hg * a.Lmax;
    const char *kc = a.k + cbase * ROWB;
    const char *vc = a.v + cbase * ROWB;
    const int vunit = lane % UPR, vsub = lane / UPR;
    const int s_lo = split * a.split_len;

    // Loads do not wait for the length: any slot below Lmax is readable, stale rows are masked later.
    auto load_tile = [&](int j0, TileRegs<DT, HD> &t) {
        const int jk = min(j0 + l32, a.Lmax - 1);
        const char *ks = kc + (long long)jk * ROWB + hf * (ROWB / 2);
#pragma unroll
        for (int i = 0; i < NV; ++i) t.kf.v[i] = *reinterpret_cast<const uint4 *>(ks + 16 * i);
#pragma unroll
        for (int i = 0; i < VPL; ++i) {
            const int jv = min(j0 + vsub + KSUB * i, a.Lmax - 1);
            t.vv[i] = *reinterpret_cast<const uint4 *>(vc + (long long)jv * ROWB + 16 * vunit);
        }
    };
    TileRegs<DT, HD> cur;
    const int j_first = s_lo + 32 * wave;
    if (j_first < a.Lmax) load_tile(j_first, cur);

    // query operand: column l32 of the product is head l32 of the group (zero beyond G)
    HalfRow<DT, HD> qf;
    if (l32 < a.G) {
        const char *src = a.q + ((long long)b * a.Hq + g * a.G + l32) * ROWB + hf * (ROWB / 2);
#pragma unroll
        for (int i = 0; i < NV; ++i) qf.v[i] = *reinterpret_cast<const uint4 *>(src + 16 * i);
    } else {
#pragma unroll
        for (int i = 0; i < NV; ++i) qf.v[i] = make_uint4(0, 0, 0, 0);
    }
    // the entry being appended, in both operand layouts (split 0 also stores it into the cache)
    HalfRow<DT, HD> kn_f;
    uint4 vn_u = make_uint4(0, 0, 0, 0);
    if (a.append) {
        const char *kn = a.k_new + (long long)hg * ROWB;
        const char *vn = a.v_new + (long long)hg * ROWB;
#pragma unroll
        for (int i = 0; i < NV; ++i) kn_f.v[i] = *reinterpret_cast<const uint4 *>(kn + hf * (ROWB / 2) + 16 * i);
        vn_u = *reinterpret_cast<const uint4 *>(vn + 16 * vunit);
    }

    const HeadLen hl = head_len(a.len[hg], a.bound, a.append);
    const int L = hl.L, new_slot = hl.new_slot;
    const int s_hi = split == a.n_split - 1 ? L : min(L, s_lo + a.split_len);   // the last split takes the remainder
    if (split == 0) {
        if (new_slot >= 0) {
            if (tid < UPR)
                *reinterpret_cast<uint4 *>(a.k + (cbase + new_slot) * ROWB + 16 * tid) =
                    *reinterpret_cast<const uint4 *>(a.k_new + (long long)hg * ROWB + 16 * tid);
            else if (tid < 2 * UPR)
                *reinterpret_cast<uint4 *>(a.v + (cbase + new_slot) * ROWB + 16 * (tid - UPR)) =
                    *reinterpret_cast<const uint4 *>(a.v_new + (long long)hg * ROWB + 16 * (tid - UPR));
            else if (tid == 2 * UPR) {
                a.kind[cbase + new_slot] = (uint8_t)a.new_kind;
                a.pos[cbase + new_slot] = a.new_pos;
            }
        }
        if (tid == 0) {
            a.cur_len[2 * hg] = L;
            a.cur_len[2 * hg + 1] = hl.flags;
        }
    }

    float m_run = -INFINITY, l_run = 0.f;   // of head l32 (both lane halves hold the same value)
    f32x16 oacc[NB];                        // O^T: rows = output channels of block nb, column = head l32
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[nb][r] = 0.f;

    char *vt = &v_lds[wave][0];
    for (int j0 = j_first; j0 < s_hi; j0 += 128) {
        TileRegs<DT, HD> nxt = cur;     // always defined (a conditionally written local would live in scratch)
        const bool more = j0 + 128 < s_hi;
        if (more) load_tile(j0 + 128, nxt);

        // substitute the appended entry, zero the rows beyond the range (their V must not reach the MFMA)
        if (j0 + 32 > s_hi || (new_slot >= j0 && new_slot < j0 + 32)) {
            if (j0 + l32 == new_slot) cur.kf = kn_f;
#pragma unroll
            for (int i = 0; i < VPL; ++i) {
                const int j = j0 + vsub + KSUB * i;
                if (j == new_slot) cur.vv[i] = vn_u;
                if (j >= s_hi) cur.vv[i] = make_uint4(0, 0, 0, 0);
            }
        }
        // V tile to LDS in natural layout
#pragma unroll
        for (int i = 0; i < VPL; ++i)
            *reinterpret_cast<uint4 *>(vt + (vsub + KSUB * i) * VPITCH + 16 * vunit) = cur.vv[i];

        // logits: rows = entries, columns = heads
        f32x16 acc;
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] = 0.f;
        mma_tile<DT, HD>(acc, cur.kf, qf);

        float tmax = -INFINITY;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int j = j0 + acc_row(r, hf);
            const float t = (j < s_hi) ? acc[r] * a.scale_log2 : -INFINITY;
            acc[r] = t;
            tmax = fmaxf(tmax, t);
        }
        tmax = fmaxf(tmax, other_half(tmax));
        const float m_new = fmaxf(m_run, tmax);          // finite: the tile holds at least one entry
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
        // (rows of a tile beyond the range lie beyond the head's length, and the logit rows are whole tiles
        // long: the four consecutive entries of a register quad go out as one 16-byte word, masked or not)
        if (a.update_score && l32 < a.G) {
            float *lg = a.logits + ((long long)hg * GP + l32) * a.Lcap + j0 + 4 * hf;
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4)
                *reinterpret_cast<float4 *>(lg + 8 * r4) =
                    make_float4(acc[4 * r4], acc[4 * r4 + 1], acc[4 * r4 + 2], acc[4 * r4 + 3]);
        }
        float p[16];
        float psum = 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            p[r] = __builtin_amdgcn_exp2f(acc[r] - m_new);
            psum += p[r];
        }
        psum += other_half(psum);
        l_run = l_run * alpha + psum;
        m_run = m_new;
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[nb][r] *= alpha;

        // the V tile is private to this wave: order the LDS traffic, no workgroup barrier
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

        // O^T += V^T P^T on the matrix cores.  The contraction index is free, so it is numbered the way
        // the probabilities already sit in this lane's registers: step s, slot i <-> entry
        // 16 s + 8 (i/4) + 4 hf + i%4 (bf16) or entry acc_row(s, hf) (fp32).  V is read transposed from LDS.
        if constexpr (DT == LVLM_BF16) {
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2) {
                const bf16x8 pb = pack_bf16x8(&p[8 * s2]);
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    uint32_t w[4];
#pragma unroll
                    for (int i2 = 0; i2 < 4; ++i2) {
                        const int e0 = 16 * s2 + 8 * ((2 * i2) >> 2) + 4 * hf + ((2 * i2) & 3);
                        const uint32_t lo = *reinterpret_cast<const uint16_t *>(vt + e0 * VPITCH + 2 * (32 * nb + l32));
                        const uint32_t hi =
                            *reinterpret_cast<const uint16_t *>(vt + (e0 + 1) * VPITCH + 2 * (32 * nb + l32));
                        w[i2] = lo | (hi << 16);
                    }
                    const bf16x8 va = __builtin_bit_cast(bf16x8, make_uint4(w[0], w[1], w[2], w[3]));
                    oacc[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, pb, oacc[nb], 0, 0, 0);
                }
            }
        } else {
#pragma unroll
            for (int s2 = 0; s2 < 16; ++s2) {
                const int e0 = acc_row(s2, hf);
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    const float va = *reinterpret_cast<const float *>(vt + e0 * VPITCH + 4 * (32 * nb + l32));
                    oacc[nb] = __builtin_amdgcn_mfma_f32_32x32x2f32(va, p[s2], oacc[nb], 0, 0, 0);
                }
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        if (more) cur = nxt;
    }

    // ---- fold the four waves: lane (head l32 < G, half hf) holds 16 channels of every block
    if (l32 < GP) {
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int r = 0; r < 16; ++r) wo[wave][l32][32 * nb + acc_row(r, hf)] = oacc[nb][r];
        if (hf == 0) {
            wm[wave][l32] = m_run;
            wl[wave][l32] = l_run;
        }
    }
    __syncthreads();
    float *po = a.part_o + ((long long)hg * a.n_split + split) * GP * HD;
    for (int idx = tid; idx < GP * HD; idx += 256) {
        const int h = idx / HD, e = idx % HD;
        float mx = wm[0][h];
#pragma unroll
        for (int w = 1; w < 4; ++w) mx = fmaxf(mx, wm[w][h]);
        const float ms = (mx == -INFINITY) ? 0.f : mx;
        float sacc = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) sacc += wo[w][h][e] * __builtin_amdgcn_exp2f(wm[w][h] - ms);
        po[idx] = sacc;
    }
    if (tid < GP) {
        float mx = wm[0][tid];
#pragma unroll
        for (int w = 1; w < 4; ++w) mx = fmaxf(mx, wm[w][tid]);
        const float ms = (mx == -INFINITY) ? 0.f : mx;
        float sacc = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) sacc += wl[w][tid] * __builtin_amdgcn_exp2f(wm[w][tid] - ms);
        float *pml = a.part_ml + (((long long)hg * a.n_split + split) * GP + tid) * 2;
        pml[0] = mx;
        pml[1] = sacc;
    }
}


// bf16 variant on 16x16x32 MFMA tiles: a group has at most 8 query heads, so a 16-wide head axis wastes
// half as much as a 32-wide one, and the accumulators (32 + 8 registers) leave room for three waves per
// SIMD.  Lane = (l16, kg): for Q.K^T the A operand row is entry l16 of a 16-entry block and kg selects
// which 16 bytes of every 64-byte piece of the head vector the lane contracts (the contraction index is
// free, and this numbering lets one load instruction read whole 64-byte pieces); the result holds
// head l16 in column position and entries 4 kg + r in its 4 registers.  Those 8 probabilities per lane
// (two blocks) are exactly one B operand of the P.V product when the contraction slot i of lane group kg
// is numbered entry 16 (i/4) + 4 kg + i%4.  V never passes through LDS: lane (l16, kg) loads, for each of
// those same 8 entries, the CPL = HD/16 consecutive channels [CPL l16, +CPL) -- 16 lanes read one whole
// row, so the loads are as coalesced as a row copy -- and turns its 8 x CPL block around in registers
// (byte permutes) into the CPL operands "8 entries of one channel".  Output block nb, row l16 is then
// channel CPL l16 + nb.
// The queries are requested first, then K, then V: loads come back in the order they went out, so the
// logits and the softmax of a tile run while its V rows are still on the way.
// MULTI: a wave may have several tiles (splits longer than 128 entries) and requests the next one while it
// works on the current one; with one tile per wave there is no running maximum to rescale by.
// TAIL: whole 128-entry splits plus exactly one more entry (steady-state decode: a cache at its budget
// plus the entry just appended).  That entry is not worth a tile pass of every workgroup: wave 0 of the last
// split takes it by itself after its tile -- its K row fills every row of one more A operand, so each lane
// has the logit of its head, and its V row is accumulated on the vector ALU.
// With 128 channels the kernel is built for two workgroups per CU: squeezed into the register budget of
// three it spills and measured slower.
template <int HD, int GP, bool MULTI, bool TAIL>
__global__ __launch_bounds__(256, HD == 128 ? 2 : 3) void attn_partial_bf16_kernel(AttnArgs a) {
    constexpr int ROWB = HD * 2;
    constexpr int UPR = ROWB / 16;
    constexpr int QV = HD / 32;           // 16-byte words of a quarter row
    constexpr int NB = HD / 16;           // output blocks = channels per lane (CPL)
    constexpr int VW = NB / 2;            // 32-bit words of V per lane and entry
    using vrow_t = typename std::conditional<VW == 4, uint4, uint2>::type;
    static_assert(!(MULTI && TAIL), "the single extra entry goes with one-tile waves");

    __shared__ float wm[4][GP], wl[4][GP];
    __shared__ __attribute__((aligned(16))) float wo[4][GP][HD + 4];     // rows 16 bytes apart in the banks: the
                                                                         // heads' 16-byte stores do not collide

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l16 = lane & 15, kg = lane >> 4;
    const int split = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
    const int hg = b * a.Hkv + g;
    const long long cbase = (long long)hg * a.Lmax;
    const char *kc = a.k + cbase * ROWB;
    const char *vc = a.v + cbase * ROWB + 2 * NB * l16;
    const int s_lo = split * a.split_len;
    const int j_first = s_lo + 32 * wave;
    auto v_entry = [&](int s) { return 16 * (s >> 2) + 4 * kg + (s & 3); };   // entry (within the tile) of slot s

    uint4 qf[QV];
    if (l16 < a.G) {
        const char *src = a.q + ((long long)b * a.Hq + g * a.G + l16) * ROWB + 16 * kg;
#pragma unroll
        for (int i = 0; i < QV; ++i) qf[i] = *reinterpret_cast<const uint4 *>(src + 64 * i);
    } else {
#pragma unroll
        for (int i = 0; i < QV; ++i) qf[i] = make_uint4(0, 0, 0, 0);
    }

    uint4 kf[2][QV];
    vrow_t vv[8];
    // Loads do not wait for the length: any slot below Lmax is readable, stale rows are masked later.
    auto load_tile = [&](int j0) {
#pragma unroll
        for (int blk = 0; blk < 2; ++blk) {
            const int jk = min(j0 + 16 * blk + l16, a.Lmax - 1);
            // contraction step i of lane group kg covers bytes [64 i + 16 kg, +16) of the row: the four lane
            // groups of one load instruction read one contiguous 64-byte piece of each row
            const char *ks = kc + (long long)jk * ROWB + 16 * kg;
#pragma unroll
            for (int i = 0; i < QV; ++i) kf[blk][i] = *reinterpret_cast<const uint4 *>(ks + 64 * i);
        }
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            const int jv = min(j0 + v_entry(s), a.Lmax - 1);
            vv[s] = *reinterpret_cast<const vrow_t *>(vc + (long long)jv * ROWB);
        }
    };
    if (j_first < a.Lmax) load_tile(j_first);

    const HeadLen hl = head_len(a.len[hg], a.bound, a.append);
    const int L = hl.L, new_slot = hl.new_slot;
    // the last split takes the remainder (only the form whose waves fetch a second tile can)
    const int s_hi = (MULTI && split == a.n_split - 1) ? L : min(L, s_lo + a.split_len);

    // TAIL: the operands of the one entry beyond the whole splits, from the cache or, if it is the entry
    // being appended, from k_new / v_new (the length is known by now; these loads queue behind the tile's)
    const int jt = a.n_split * a.split_len;
    const bool tail = TAIL && split == a.n_split - 1 && wave == 0 && jt < L;
    uint4 kt[QV], tv[NB / 2];
    if (tail) {
        const bool fresh = jt == new_slot;
        const char *ks = (fresh ? a.k_new + (long long)hg * ROWB : kc + (long long)jt * ROWB) + 16 * kg;
        const char *vs = (fresh ? a.v_new + (long long)hg * ROWB : a.v + (cbase + jt) * ROWB) + 8 * NB * kg;
#pragma unroll
        for (int i = 0; i < QV; ++i) kt[i] = *reinterpret_cast<const uint4 *>(ks + 64 * i);
#pragma unroll
        for (int i = 0; i < NB / 2; ++i) tv[i] = *reinterpret_cast<const uint4 *>(vs + 16 * i);
    }

    if (split == 0) {
        // the appended entry goes into the cache here; every reader below takes it from k_new / v_new
        if (new_slot >= 0) {
            if (tid < UPR)
                *reinterpret_cast<uint4 *>(a.k + (cbase + new_slot) * ROWB + 16 * tid) =
                    *reinterpret_cast<const uint4 *>(a.k_new + (long long)hg * ROWB + 16 * tid);
            else if (tid < 2 * UPR)
                *reinterpret_cast<uint4 *>(a.v + (cbase + new_slot) * ROWB + 16 * (tid - UPR)) =
                    *reinterpret_cast<const uint4 *>(a.v_new + (long long)hg * ROWB + 16 * (tid - UPR));
            else if (tid == 2 * UPR) {
                a.kind[cbase + new_slot] = (uint8_t)a.new_kind;
                a.pos[cbase + new_slot] = a.new_pos;
            }
        }
        if (tid == 0) {
            a.cur_len[2 * hg] = L;
            a.cur_len[2 * hg + 1] = hl.flags;
        }
    }

    float m_run = -INFINITY, l_run = 0.f;   // of head l16 (all four lane groups hold the same value)
    f32x4 oacc[NB];                         // O^T block nb: channels NB (4 kg + r) + nb, head l16
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) oacc[nb] = f32x4{0.f, 0.f, 0.f, 0.f};
    float *lg = a.logits + ((long long)hg * GP + l16) * a.Lcap;      // this lane's head, one float per entry

    // one tile (a branch, so that the first product starts from a constant zero) or a loop over the wave's tiles
    for (int j0 = j_first; j0 < s_hi; j0 = MULTI ? j0 + 128 : s_hi) {
        const bool whole = j0 + 32 <= s_hi;
        // the appended entry comes from k_new / v_new; rows beyond the range must not reach the MFMA
        if (!whole || (new_slot >= j0 && new_slot < j0 + 32)) {
#pragma unroll
            for (int blk = 0; blk < 2; ++blk) {
                if (j0 + 16 * blk + l16 == new_slot) {
                    const char *kn = a.k_new + (long long)hg * ROWB + 16 * kg;
#pragma unroll
                    for (int i = 0; i < QV; ++i) kf[blk][i] = *reinterpret_cast<const uint4 *>(kn + 64 * i);
                }
            }
#pragma unroll
            for (int s = 0; s < 8; ++s) {
                const int j = j0 + v_entry(s);
                if (j == new_slot) vv[s] = *reinterpret_cast<const vrow_t *>(a.v_new + (long long)hg * ROWB + 2 * NB * l16);
                if (j >= s_hi) vv[s] = vrow_t{};
            }
        }
        // this tile's V block, turned around: vt[nb][m] = channel nb of entries 2m and 2m+1.  With several
        // tiles per wave it is done now, before the next tile's loads overwrite vv; with one tile it waits
        // until the logits are done (the V rows arrive last).
        uint32_t vt[NB][4];
        auto turn = [&]() {
#pragma unroll
            for (int m = 0; m < 4; ++m) {
                const uint32_t *ea = reinterpret_cast<const uint32_t *>(&vv[2 * m]);
                const uint32_t *eb = reinterpret_cast<const uint32_t *>(&vv[2 * m + 1]);
#pragma unroll
                for (int w2 = 0; w2 < VW; ++w2) {
                    vt[2 * w2][m] = __builtin_amdgcn_perm(eb[w2], ea[w2], 0x05040100u);       // low halves
                    vt[2 * w2 + 1][m] = __builtin_amdgcn_perm(eb[w2], ea[w2], 0x07060302u);   // high halves
                }
            }
        };
        if (MULTI) turn();

        f32x4 acc[2];
#pragma unroll
        for (int blk = 0; blk < 2; ++blk) {
            acc[blk] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int i = 0; i < QV; ++i)
                acc[blk] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kf[blk][i]),
                                                                   __builtin_bit_cast(bf16x8, qf[i]), acc[blk], 0, 0, 0);
        }
        // next tile's loads go out while this one is reduced (registers are free again)
        if (MULTI && j0 + 128 < s_hi) load_tile(j0 + 128);

        float t[8];
        float tmax = -INFINITY;
        if (whole) {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                t[i] = acc[i >> 2][i & 3] * a.scale_log2;
                tmax = fmaxf(tmax, t[i]);
            }
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int j = j0 + 16 * (i >> 2) + 4 * kg + (i & 3);
                t[i] = (j < s_hi) ? acc[i >> 2][i & 3] * a.scale_log2 : -INFINITY;
                tmax = fmaxf(tmax, t[i]);
            }
        }
        tmax = fmaxf(tmax, other_row(tmax));
        tmax = fmaxf(tmax, other_half(tmax));
        // a tile's rows beyond the range lie beyond the head's length, and the logit rows are whole tiles long:
        // the four entries of a block a lane holds go out as one 16-byte word, masked or not
        if (a.update_score && l16 < a.G) {
#pragma unroll
            for (int blk = 0; blk < 2; ++blk)
                *reinterpret_cast<float4 *>(lg + j0 + 16 * blk + 4 * kg) =
                    make_float4(t[4 * blk], t[4 * blk + 1], t[4 * blk + 2], t[4 * blk + 3]);
        }
        const float m_new = MULTI ? fmaxf(m_run, tmax) : tmax;    // finite: the tile holds at least one entry
        float p[8];
        float psum = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            p[i] = __builtin_amdgcn_exp2f(t[i] - m_new);
            psum += p[i];
        }
        psum += other_row(psum);
        psum += other_half(psum);
        if (MULTI) {
            const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
            l_run = l_run * alpha + psum;
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) oacc[nb] *= alpha;
        } else {
            l_run = psum;
        }
        m_run = m_new;
        const bf16x8 pb = pack_bf16x8(p);

        if (!MULTI) turn();
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            const bf16x8 va = __builtin_bit_cast(bf16x8, make_uint4(vt[nb][0], vt[nb][1], vt[nb][2], vt[nb][3]));
            oacc[nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va, pb, oacc[nb], 0, 0, 0);
        }
    }

    if (TAIL && tail) {
        f32x4 at = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int i = 0; i < QV; ++i)
            at = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kt[i]), __builtin_bit_cast(bf16x8, qf[i]),
                                                         at, 0, 0, 0);
        const float t = at[0] * a.scale_log2;        // every row of the operand was the same entry
        if (a.update_score && l16 < a.G && kg == 0) lg[jt] = t;
        const float m_new = fmaxf(m_run, t);
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
        const float p = __builtin_amdgcn_exp2f(t - m_new);
        l_run = l_run * alpha + p;
        m_run = m_new;
        // the lane's channels NB (4 kg + r) + nb are the 4 NB consecutive ones from 4 NB kg on
        const uint32_t *tw = reinterpret_cast<const uint32_t *>(tv);
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                const uint32_t w2 = tw[(NB * r + nb) >> 1];
                const float v = __uint_as_float((nb & 1) ? (w2 & 0xffff0000u) : (w2 << 16));
                oacc[nb][r] = fmaf(p, v, oacc[nb][r] * alpha);
            }
    }

    // ---- fold the four waves
    if (l16 < GP) {
        // register r of block nb is channel NB (4 kg + r) + nb: for one r the NB blocks are neighbours
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int q4 = 0; q4 < NB / 4; ++q4)
                *reinterpret_cast<float4 *>(&wo[wave][l16][NB * (4 * kg + r) + 4 * q4]) =
                    make_float4(oacc[4 * q4][r], oacc[4 * q4 + 1][r], oacc[4 * q4 + 2][r], oacc[4 * q4 + 3][r]);
        if (kg == 0) {
            wm[wave][l16] = m_run;
            wl[wave][l16] = l_run;
        }
    }
    __syncthreads();
    float *po = a.part_o + ((long long)hg * a.n_split + split) * GP * HD;
    for (int i4 = tid; i4 < GP * HD / 4; i4 += 256) {                  // four channels of one head per thread
        const int h = i4 / (HD / 4), e = 4 * (i4 % (HD / 4));
        float mx = wm[0][h];
#pragma unroll
        for (int w = 1; w < 4; ++w) mx = fmaxf(mx, wm[w][h]);
        const float ms = (mx == -INFINITY) ? 0.f : mx;
        float4 sacc = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const float wgt = __builtin_amdgcn_exp2f(wm[w][h] - ms);
            const float4 x = *reinterpret_cast<const float4 *>(&wo[w][h][e]);
            sacc.x += x.x * wgt; sacc.y += x.y * wgt; sacc.z += x.z * wgt; sacc.w += x.w * wgt;
        }
        *reinterpret_cast<float4 *>(po + 4 * i4) = sacc;
    }
    if (tid < GP) {
        float mx = wm[0][tid];
#pragma unroll
        for (int w = 1; w < 4; ++w) mx = fmaxf(mx, wm[w][tid]);
        const float ms = (mx == -INFINITY) ? 0.f : mx;
        float sacc = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) sacc += wl[w][tid] * __builtin_amdgcn_exp2f(wm[w][tid] - ms);
        float *pml = a.part_ml + (((long long)hg * a.n_split + split) * GP + tid) * 2;
        pml[0] = mx;
        pml[1] = sacc;
    }
}

constexpr int kMaxSplit = 64;   // splits one combine workgroup can fold (checked on the host)

template <int GP>
struct CombineLds {
    float pm[kMaxSplit][GP];    // per split: running max of each head
    float pl[kMaxSplit][GP];    // per split: sum, then the split's weight exp2(m_s - M)
    float m[GP], inv[GP];       // per head: max over the splits, 1 / normaliser
};

// The fold kernels are chains of memory latencies, so each of them requests everything it will read --
// the splits' (max, sum) pairs and partial outputs, the logits, importance and kind of its entries --
// before it waits for anything; indices are clamped into the arrays instead of tested against the length,
// which is itself still on its way.

// (max, sum) pair `tid` of the head's n_split x GP pairs.
template <int GP>
__device__ __forceinline__ float2 load_pair(const AttnArgs &a, int hg) {
    const int tid = threadIdx.x;
    const float *pml = a.part_ml + (long long)hg * a.n_split * GP * 2;
    return tid < a.n_split * GP ? *reinterpret_cast<const float2 *>(pml + 2 * tid) : make_float2(0.f, 0.f);
}

// Rebuilds the per-head normalisers of one (batch, KV head) from the splits' (max, sum) pairs.
template <int GP, int NT>
__device__ __forceinline__ void fold_normalisers(const AttnArgs &a, CombineLds<GP> &c, float2 ml) {
    const int tid = threadIdx.x;
    static_assert(NT >= kMaxSplit * GP, "one pair per thread");
    if (tid < a.n_split * GP) {
        c.pm[tid / GP][tid % GP] = ml.x;
        c.pl[tid / GP][tid % GP] = ml.y;
    }
    __syncthreads();
    // Few splits: one thread per head walks them.  Many (up to 64): one wave per head, one lane per split, two wave
    // reductions instead of two serial loops (measured: config 5's 16 splits gain 0.9 us per launch, 8 splits lose).
    static_assert(NT >= 64 * GP, "one wave per head");
    const int wave = tid >> 6, lane = tid & 63;
    if (a.n_split <= 8) {
        if (tid < GP) {
            float mx = -INFINITY;
            for (int s = 0; s < a.n_split; ++s) mx = fmaxf(mx, c.pm[s][tid]);
            const float ms = (mx == -INFINITY) ? 0.f : mx;
            float l = 0.f;
            for (int s = 0; s < a.n_split; ++s) {
                const float wgt = exp2f(c.pm[s][tid] - ms);
                l += c.pl[s][tid] * wgt;
                c.pl[s][tid] = wgt;                      // reused below as the split's weight
            }
            c.m[tid] = ms;
            c.inv[tid] = l > 0.f ? 1.0f / l : 0.f;
        }
    } else if (wave < GP) {
        const bool on = lane < a.n_split;
        const float m_s = on ? c.pm[lane][wave] : -INFINITY;
        const float mx = wave_max(m_s);
        const float ms = (mx == -INFINITY) ? 0.f : mx;
        const float wgt = on ? exp2f(m_s - ms) : 0.f;
        const float l = wave_sum(on ? c.pl[lane][wave] * wgt : 0.f);
        if (on) c.pl[lane][wave] = wgt;              // reused below as the split's weight
        if (lane == 0) {
            c.m[wave] = ms;
            c.inv[wave] = l > 0.f ? 1.0f / l : 0.f;
        }
    }
    __syncthreads();
}

// Output element idx0 + tid (head idx / HD, channel idx % HD) of the head group: the first 16 splits' partial values.
constexpr int kOutRegs = 16;
template <int HD, int GP>
__device__ __forceinline__ void load_output(const AttnArgs &a, int hg, int idx0, float (&v)[kOutRegs]) {
    const int idx = min(idx0 + (int)threadIdx.x, a.G * HD - 1);
    const int h = idx / HD, e = idx % HD;
    const float *po = a.part_o + (long long)hg * a.n_split * GP * HD + (long long)h * HD + e;
#pragma unroll
    for (int u = 0; u < kOutRegs; ++u) v[u] = u < a.n_split ? po[(long long)u * GP * HD] : 0.f;
}

// Folds the splits' partial outputs into output elements [idx0, idx1) of the head group (one per thread).
template <int DT, int HD, int GP, int NT>
__device__ __forceinline__ void write_output(const AttnArgs &a, const CombineLds<GP> &c, int b, int g, int hg, int idx0,
                                             int idx1, const float (&v)[kOutRegs]) {
    static_assert(NT >= 8 * HD, "one output element per thread");
    const int idx = idx0 + threadIdx.x;
    if (idx >= idx1) return;
    const int h = idx / HD, e = idx % HD;
    float acc = 0.f;
#pragma unroll
    for (int u = 0; u < kOutRegs; ++u) acc = u < a.n_split ? fmaf(v[u], c.pl[u][h], acc) : acc;
    const float *po = a.part_o + (long long)hg * a.n_split * GP * HD + (long long)h * HD + e;
    for (int s0 = kOutRegs; s0 < a.n_split; s0 += kOutRegs) {           // long caches: further rounds of 16 loads
        float x[kOutRegs];
#pragma unroll
        for (int u = 0; u < kOutRegs; ++u) x[u] = s0 + u < a.n_split ? po[(long long)(s0 + u) * GP * HD] : 0.f;
#pragma unroll
        for (int u = 0; u < kOutRegs; ++u) acc = s0 + u < a.n_split ? fmaf(x[u], c.pl[s0 + u][h], acc) : acc;
    }
    acc *= c.inv[h];
    const long long oi = ((long long)b * a.Hq + g * a.G + h) * HD + e;
    if constexpr (DT == LVLM_BF16)
        reinterpret_cast<uint16_t *>(a.out)[oi] = f32_to_bf16(acc);
    else
        reinterpret_cast<float *>(a.out)[oi] = acc;
}

// What the importance update reads of one entry.
template <int GP>
struct EntryRegs {
    float old;
    float lv[GP];
    uint8_t kd;
};

template <int GP, bool EVICT>
__device__ __forceinline__ void load_entry(const AttnArgs &a, int hg, int j, EntryRegs<GP> &r) {
    const long long cbase = (long long)hg * a.Lmax;
    const int jl = min(j, a.Lcap - 1), jc = min(j, a.Lmax - 1);
    const float *lg = a.logits + (long long)hg * GP * a.Lcap + jl;
#pragma unroll
    for (int h = 0; h < GP; ++h) r.lv[h] = h < a.G ? lg[(long long)h * a.Lcap] : 0.f;
    r.old = a.score[cbase + jc];
    r.kd = EVICT ? a.kind[cbase + jc] : (uint8_t)0;
}

// The stored logits become normalised probabilities.  With EVICT the least important evictable entry seen
// so far is tracked in `best` (importance key in the high half, inverted slot in the low half: the minimum
// is the lowest score, highest slot among equals).
template <int GP, bool EVICT>
__device__ __forceinline__ void apply_entry(const AttnArgs &a, const CombineLds<GP> &c, int hg, int L, bool appended,
                                            int j, const EntryRegs<GP> &r, int recent_lo, unsigned long long &best,
                                            float *last_ns = nullptr) {
    if (j >= L) return;
    const long long cbase = (long long)hg * a.Lmax;
    // (every product-sum is an explicit fused multiply-add: the two fold kernels must give the same bits)
    float pm = 0.f;
#pragma unroll
    for (int h = 0; h < GP; ++h)
        if (h < a.G) pm = fmaf(exp2f(r.lv[h] - c.m[h]), c.inv[h], pm);
    const float old = (appended && j == L - 1) ? 0.f : r.old;        // the new entry starts from nothing
    const float ns = fmaf(a.decay, old, pm * (1.0f / (float)a.G));
    a.score[cbase + j] = ns;
    if (EVICT && j == L - 1) *last_ns = ns;          // the entry that fills the victim's slot
    if (EVICT && r.kd != LVLM_KIND_PROTECTED && j < recent_lo) {
        const unsigned long long cand =
            ((unsigned long long)score_key(ns) << 32) | (unsigned long long)(0xffffffffu - (uint32_t)j);
        best = cand < best ? cand : best;
    }
}

// Workgroup x = 0 folds the splits into the output rows; workgroups x >= 1 each update the importance of
// 1024 entries.  All of them first rebuild the per-head normalisers.
template <int DT, int HD, int GP>
__global__ __launch_bounds__(1024) void attn_combine_kernel(AttnArgs a) {
    constexpr int NT = 1024;      // one entry or output element per thread: the kernel is a chain of latencies
    __shared__ CombineLds<GP> c;
    const int g = blockIdx.y, b = blockIdx.z;
    const int hg = b * a.Hkv + g;
    const float2 ml = load_pair<GP>(a, hg);
    if (blockIdx.x == 0) {
        float v[kOutRegs];
        load_output<HD, GP>(a, hg, 0, v);
        const int L = a.cur_len[2 * hg];
        const bool appended = a.cur_len[2 * hg + 1] & kAppended;
        fold_normalisers<GP, NT>(a, c, ml);
        write_output<DT, HD, GP, NT>(a, c, b, g, hg, 0, a.G * HD, v);
        if (threadIdx.x == 0 && appended) a.len[hg] = L;
        return;
    }
    const int j = (blockIdx.x - 1) * NT + threadIdx.x;
    EntryRegs<GP> r;
    load_entry<GP, false>(a, hg, j, r);
    const int L = a.cur_len[2 * hg];
    const bool appended = a.cur_len[2 * hg + 1] & kAppended;
    fold_normalisers<GP, NT>(a, c, ml);
    unsigned long long unused = ~0ull;
    apply_entry<GP, false>(a, c, hg, L, appended, j, r, 0, unused);
}

// Per-step cache compression in the same launch as the fold (Sec. 3.2.2, steady state).  One compute unit
// fetches the 4-byte words this kernel reads at some tens of GB/s only, so what a (batch, KV head) pair has to
// read is spread over several workgroups: n_out of them fold the splits' partial outputs into the output rows (a share of
// the group's heads each), one more updates every entry's importance and, if the head is now longer than
// evict_budget, evicts its least important evictable entry (not protected, not among the last evict_recent
// slots): the last entry takes its slot, as LVLM_ORDER_FILL does.
// NCH > 0: the head has at most 1024 NCH entries (the caller's bound) and a thread keeps its NCH entries in
// registers, requested at the very start; NCH == 0: any length, 1024 entries at a time.
template <int DT, int HD, int GP, int NCH>
__global__ __launch_bounds__(1024) void attn_combine_evict_kernel(AttnArgs a, int n_out) {
    constexpr int ROWB = HD * esize<DT>();
    constexpr int NT = 1024;
    constexpr int NR = NCH > 0 ? NCH : 1;
    __shared__ CombineLds<GP> c;
    __shared__ unsigned long long w_best[NT / 64];
    __shared__ float last_ns;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int g = blockIdx.y, b = blockIdx.z;
    const int hg = b * a.Hkv + g;
    const float2 ml = load_pair<GP>(a, hg);
    if ((int)blockIdx.x < n_out) {
        // output elements [idx0, idx1): whole channels-of-a-head runs, at most 1024
        const int per = (a.G * HD + n_out - 1) / n_out;
        const int idx0 = blockIdx.x * per, idx1 = min(a.G * HD, idx0 + per);
        float v[kOutRegs];
        load_output<HD, GP>(a, hg, idx0, v);
        fold_normalisers<GP, NT>(a, c, ml);
        write_output<DT, HD, GP, NT>(a, c, b, g, hg, idx0, idx1, v);
        return;
    }
    EntryRegs<GP> er[NR];
#pragma unroll
    for (int x = 0; x < NR; ++x) load_entry<GP, true>(a, hg, NT * x + tid, er[x]);

    const int L = a.cur_len[2 * hg];
    const int flags = a.cur_len[2 * hg + 1];
    const bool appended = flags & kAppended;
    const bool evict = L > a.evict_budget && !(flags & kTruncated);
    // The entry that will fill the victim's slot is known before the victim is: its K and V rows, kind and
    // position are fetched now (nothing in this kernel changes them), its new importance comes through LDS,
    // so the move at the end is stores only.
    constexpr int UPR = ROWB / 16;
    const long long cbase = (long long)hg * a.Lmax;
    uint4 last_row = make_uint4(0, 0, 0, 0);
    uint8_t last_kind = 0;
    int32_t last_pos = 0;
    if (evict) {
        const long long last = cbase + L - 1;
        if (tid < UPR) last_row = *reinterpret_cast<const uint4 *>(a.k + last * ROWB + 16 * tid);
        else if (tid < 2 * UPR) last_row = *reinterpret_cast<const uint4 *>(a.v + last * ROWB + 16 * (tid - UPR));
        else if (tid == 2 * UPR) {
            last_kind = a.kind[last];
            last_pos = a.pos[last];
        }
    }
    fold_normalisers<GP, NT>(a, c, ml);
    const int recent_lo = evict ? L - a.evict_recent : 0;      // nothing is a candidate when nothing is evicted
    unsigned long long best = ~0ull;
#pragma unroll
    for (int x = 0; x < NR; ++x) apply_entry<GP, true>(a, c, hg, L, appended, NT * x + tid, er[x], recent_lo, best, &last_ns);
    if (NCH == 0) {
        for (int j = NT + tid; j - tid < L; j += NT) {
            EntryRegs<GP> r;
            load_entry<GP, true>(a, hg, j, r);
            apply_entry<GP, true>(a, c, hg, L, appended, j, r, recent_lo, best, &last_ns);
        }
    }
    int new_len = L;
    if (evict) {
        best = wave_min_u64(best);
        if (lane == 0) w_best[wave] = best;
        __syncthreads();                                   // also orders the score stores above before the move below
        best = w_best[0];
#pragma unroll
        for (int w = 1; w < NT / 64; ++w) best = w_best[w] < best ? w_best[w] : best;
        if (best != ~0ull) {
            const int victim = (int)(0xffffffffu - (uint32_t)(best & 0xffffffffull));
            const int last = L - 1;
            new_len = last;
            if (victim != last) {
                if (tid < UPR)
                    *reinterpret_cast<uint4 *>(a.k + (cbase + victim) * ROWB + 16 * tid) = last_row;
                else if (tid < 2 * UPR)
                    *reinterpret_cast<uint4 *>(a.v + (cbase + victim) * ROWB + 16 * (tid - UPR)) = last_row;
                else if (tid == 2 * UPR) {
                    a.score[cbase + victim] = last_ns;
                    a.kind[cbase + victim] = last_kind;
                    a.pos[cbase + victim] = last_pos;
                }
            }
        }
    }
    if (tid == 0 && (appended || new_len != L)) a.len[hg] = new_len;
}

template <int DT, int HD, int GP>
void launch_both(const Prof &prof, const AttnArgs &a, int B, int len_bound) {
    hipStream_t stream = prof.stream;
    prof.begin("attn_partial");
    if constexpr (DT == LVLM_BF16)
    {
        const dim3 grid(a.n_split, a.Hkv, B);
        if (a.tail_entry)
            LVLM_LAUNCH(prof, (attn_partial_bf16_kernel<HD, GP, false, true>), grid, dim3(256), 0, stream, a);
        else if (a.split_len > 128 || a.n_split * a.split_len < len_bound)      // some wave has a second tile
            LVLM_LAUNCH(prof, (attn_partial_bf16_kernel<HD, GP, true, false>), grid, dim3(256), 0, stream, a);
        else
            LVLM_LAUNCH(prof, (attn_partial_bf16_kernel<HD, GP, false, false>), grid, dim3(256), 0, stream, a);
    }
    else
        LVLM_LAUNCH(prof, (attn_partial_kernel<DT, HD, GP>), dim3(a.n_split, a.Hkv, B), dim3(256), 0, stream, a);
    prof.end();
    if (a.evict_budget > 0) {
        prof.begin("attn_combine_evict");
        // output workgroups per head: as many as keep the launch within one round of the chip, at most one per
        // query head of the group
        int n_out = 256 / (a.Hkv * B) - 1;
        n_out = n_out < 1 ? 1 : (n_out > a.G ? a.G : n_out);
        const dim3 grid(n_out + 1, a.Hkv, B);
        if (len_bound <= 1024) LVLM_LAUNCH(prof, (attn_combine_evict_kernel<DT, HD, GP, 1>), grid, dim3(1024), 0, stream, a, n_out);
        else if (len_bound <= 2048) LVLM_LAUNCH(prof, (attn_combine_evict_kernel<DT, HD, GP, 2>), grid, dim3(1024), 0, stream, a, n_out);
        else if (len_bound <= 3072) LVLM_LAUNCH(prof, (attn_combine_evict_kernel<DT, HD, GP, 3>), grid, dim3(1024), 0, stream, a, n_out);
        else LVLM_LAUNCH(prof, (attn_combine_evict_kernel<DT, HD, GP, 0>), grid, dim3(1024), 0, stream, a, n_out);
        prof.end();
        return;
    }
    const int chunks = a.update_score ? (len_bound + 1023) / 1024 : 0;
    prof.begin("attn_combine");
    LVLM_LAUNCH(prof, (attn_combine_kernel<DT, HD, GP>), dim3(1 + chunks, a.Hkv, B), dim3(1024), 0, stream, a);
    prof.end();
}

template <int DT, int HD>
void launch_gp(const Prof &prof, const AttnArgs &a, int B, int len_bound, int gp) {
    switch (gp) {
        case 1: launch_both<DT, HD, 1>(prof, a, B, len_bound); break;
        case 2: launch_both<DT, HD, 2>(prof, a, B, len_bound); break;
        case 4: launch_both<DT, HD, 4>(prof, a, B, len_bound); break;
        default: launch_both<DT, HD, 8>(prof, a, B, len_bound); break;
    }
}

int group_pad(int G) { return G <= 1 ? 1 : (G <= 2 ? 2 : (G <= 4 ? 4 : 8)); }

}  // namespace

AttnWs attn_ws(const lvlm_attn_desc &d) {
    AttnWs w{};
    const int bound = d.len_bound > 0 ? d.len_bound : d.Lmax;
    const long long heads = (long long)d.B * d.Hkv;
    // As many splits as fit the chip in one round (two workgroups on each of 256 compute units), each at
    // least one pass of the four waves (128 entries) and a whole number of 32-entry tiles; measured: a
    // second, partly filled round costs more than longer splits do.
    const int max_split = (bound + 127) / 128;
    const long long want_round = 512 / heads;
    long long want = want_round;
    // The bf16 kernel whose waves take ONE tile is lean enough for four workgroups per compute unit (122 registers):
    // where splits of 128 entries are still one round that way (at most 1024 workgroups), they beat half as many
    // splits of two tiles per wave by a little (64 heads: 15.3 against 15.9 us at 1889 entries, 11.4 against 12.0 us
    // at 1360).
    if (d.dtype == LVLM_BF16 && heads * max_split <= 1024 && max_split > want) want = max_split;
    int n_split = (int)(want < 1 ? 1 : (want > max_split ? max_split : want));
    if (n_split > 64) n_split = 64;               // kMaxSplit of the combine kernel
    int split_len = ((bound + n_split - 1) / n_split + 31) / 32 * 32;
    if (split_len < 128) split_len = 128;
    n_split = (bound + split_len - 1) / split_len;
    // A remainder of at most one tile beyond whole 128-entry splits (steady-state decode: budget + 1 entries)
    // does not lengthen every split by a tile: a single extra entry is taken by one wave of the last split on
    // its own (tail_entry), a longer remainder goes to the last split as one extra tile of one wave.
    const int full = bound / 128;
    w.tail_entry = 0;
    if (full >= 1 && want_round >= full && bound - 128 * full <= 32 && full <= 64) {
        n_split = full;
        split_len = 128;
        w.tail_entry = d.dtype == LVLM_BF16 && bound - 128 * full == 1;
    }
    if (n_split < 1) n_split = 1;
    w.n_split = n_split;
    w.split_len = split_len;
    const int G = d.Hq / d.Hkv, gp = group_pad(G);
    const int lcap = (bound + 31) / 32 * 32;       // whole tiles: a tile's logits are stored without a bound test
    w.part_ml = 0;
    w.part_o = align_up(w.part_ml + (size_t)heads * n_split * gp * 2 * sizeof(float), 256);
    w.logits = align_up(w.part_o + (size_t)heads * n_split * gp * d.hd * sizeof(float), 256);
    w.lcap = lcap;
    w.cur_len = align_up(w.logits + (size_t)heads * gp * lcap * sizeof(float), 256);
    w.total = align_up(w.cur_len + (size_t)heads * 2 * sizeof(int32_t), 256);
    return w;
}

hipError_t launch_decode_attn(const Prof &prof, const lvlm_attn_desc &d, const AttnWs &w, char *ws, const void *q,
                              const void *k_new, const void *v_new, void *k_cache, void *v_cache, float *score,
                              uint8_t *kind, int32_t *orig_pos, int32_t *len, void *out) {
    const int bound = d.len_bound > 0 ? d.len_bound : d.Lmax;
    const int G = d.Hq / d.Hkv;
    AttnArgs a{};
    a.q = static_cast<const char *>(q);
    a.k_new = static_cast<const char *>(k_new);
    a.v_new = static_cast<const char *>(v_new);
    a.k = static_cast<char *>(k_cache);
    a.v = static_cast<char *>(v_cache);
    a.score = score; a.kind = kind; a.pos = orig_pos; a.len = len;
    a.out = static_cast<char *>(out);
    a.part_ml = reinterpret_cast<float *>(ws + w.part_ml);
    a.part_o = reinterpret_cast<float *>(ws + w.part_o);
    a.logits = reinterpret_cast<float *>(ws + w.logits);
    a.cur_len = reinterpret_cast<int32_t *>(ws + w.cur_len);
    a.Hq = d.Hq; a.Hkv = d.Hkv; a.G = G; a.Lmax = d.Lmax; a.Lcap = w.lcap; a.bound = bound;
    a.n_split = w.n_split; a.split_len = w.split_len; a.tail_entry = w.tail_entry;
    a.append = k_new != nullptr;
    a.new_kind = d.new_kind; a.new_pos = d.new_pos;
    a.update_score = score != nullptr;
    a.evict_budget = d.evict_budget;
    a.evict_recent = d.evict_recent;
    a.scale_log2 = d.scale * kLog2e;
    a.decay = d.score_decay;
    const int gp = group_pad(G);
    if (d.dtype == LVLM_BF16 && d.hd == 128) launch_gp<LVLM_BF16, 128>(prof, a, d.B, bound, gp);
    else if (d.dtype == LVLM_BF16 && d.hd == 64) launch_gp<LVLM_BF16, 64>(prof, a, d.B, bound, gp);
    else if (d.dtype == LVLM_F32 && d.hd == 128) launch_gp<LVLM_F32, 128>(prof, a, d.B, bound, gp);
    else launch_gp<LVLM_F32, 64>(prof, a, d.B, bound, gp);
    return hipGetLastError();
}

}  // namespace lvlm
