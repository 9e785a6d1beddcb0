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
#include "common.h"

namespace lvlm {
namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

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
    float *logits;      // [B*Hkv][G][Lcap]
    int32_t *cur_len;   // [B*Hkv]
    int Hq, Hkv, G, Lmax, Lcap, n_split, split_len, append, new_kind, new_pos, update_score;
    float scale_log2, decay;
};

template <int DT>
__host__ __device__ constexpr int esize() {
    return DT == LVLM_BF16 ? 2 : 4;
}

template <int DT, int HD>
struct HalfRow {
    static constexpr int NV = (HD / 2) * esize<DT>() / 16;
    uint4 v[NV];
};

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

__device__ __forceinline__ int acc_row(int r, int hf) { return 8 * (r >> 2) + 4 * hf + (r & 3); }

// Elements of one 16-byte unit as floats.
template <int DT>
__device__ __forceinline__ void unpack(const uint4 &u, float (&f)[16 / esize<DT>()]) {
    if constexpr (DT == LVLM_BF16) {
        const uint32_t d[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            f[2 * i] = __uint_as_float(d[i] << 16);
            f[2 * i + 1] = __uint_as_float(d[i] & 0xffff0000u);
        }
    } else {
        f[0] = __uint_as_float(u.x);
        f[1] = __uint_as_float(u.y);
        f[2] = __uint_as_float(u.z);
        f[3] = __uint_as_float(u.w);
    }
}

template <int DT, int HD, int GP>
__global__ __launch_bounds__(256) void attn_partial_kernel(AttnArgs a) {
    constexpr int ES = esize<DT>();
    constexpr int ROWB = HD * ES;
    constexpr int NV = HalfRow<DT, HD>::NV;
    constexpr int UPR = ROWB / 16;        // 16-byte units per row
    constexpr int KSUB = 64 / UPR;        // rows a wave covers with one load instruction
    constexpr int VPL = 32 / KSUB;        // V units per lane per 32-entry tile
    constexpr int EPU = 16 / ES;          // elements per unit
    static_assert(UPR <= 64 && KSUB >= 1, "row too long for one wave");

    __shared__ __attribute__((aligned(16))) float p_lds[4][32][GP];
    __shared__ __attribute__((aligned(16))) float alpha_lds[4][GP];
    __shared__ float wm[4][GP], wl[4][GP];
    __shared__ __attribute__((aligned(16))) float wo[4][GP][HD];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int hf = lane >> 5, l32 = lane & 31;
    const int split = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
    const int hg = b * a.Hkv + g;
    const long long cbase = (long long)hg * a.Lmax;
    const int L = min(a.len[hg] + (a.append ? 1 : 0), a.Lmax);
    const int new_slot = a.append ? L - 1 : -1;
    const char *kc = a.k + cbase * ROWB;
    const char *vc = a.v + cbase * ROWB;
    const char *kn = a.k_new ? a.k_new + (long long)hg * ROWB : nullptr;
    const char *vn = a.v_new ? a.v_new + (long long)hg * ROWB : nullptr;

    // the appended entry is stored by split 0; nobody reads that slot from the cache in this kernel
    if (split == 0 && a.append) {
        if (tid < UPR)
            *reinterpret_cast<uint4 *>(a.k + (cbase + new_slot) * ROWB + 16 * tid) =
                *reinterpret_cast<const uint4 *>(kn + 16 * tid);
        else if (tid < 2 * UPR)
            *reinterpret_cast<uint4 *>(a.v + (cbase + new_slot) * ROWB + 16 * (tid - UPR)) =
                *reinterpret_cast<const uint4 *>(vn + 16 * (tid - UPR));
        else if (tid == 2 * UPR) {
            a.kind[cbase + new_slot] = (uint8_t)a.new_kind;
            a.pos[cbase + new_slot] = a.new_pos;
        }
    }
    if (split == 0 && tid == 0) a.cur_len[hg] = L;

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

    const int s_lo = split * a.split_len;
    const int s_hi = min(L, s_lo + a.split_len);
    const int vunit = lane % UPR, vsub = lane / UPR;

    float m_run = -INFINITY, l_run = 0.f;   // of head l32 (both halves hold the same value)
    float o[GP][EPU];
#pragma unroll
    for (int h = 0; h < GP; ++h)
#pragma unroll
        for (int e = 0; e < EPU; ++e) o[h][e] = 0.f;

    for (int j0 = s_lo + 32 * wave; j0 < s_hi; j0 += 128) {
        // ---- loads: K as MFMA operand (lane = entry), V in natural layout
        HalfRow<DT, HD> kf;
        {
            const int j = j0 + l32;
            if (j < s_hi) {
                const char *src = (j == new_slot ? kn : kc + (long long)j * ROWB) + hf * (ROWB / 2);
#pragma unroll
                for (int i = 0; i < NV; ++i) kf.v[i] = *reinterpret_cast<const uint4 *>(src + 16 * i);
            } else {
#pragma unroll
                for (int i = 0; i < NV; ++i) kf.v[i] = make_uint4(0, 0, 0, 0);
            }
        }
        uint4 vv[VPL];
#pragma unroll
        for (int i = 0; i < VPL; ++i) {
            const int j = j0 + vsub + KSUB * i;
            if (j < s_hi) {
                const char *src = (j == new_slot ? vn : vc + (long long)j * ROWB) + 16 * vunit;
                vv[i] = *reinterpret_cast<const uint4 *>(src);
            } else {
                vv[i] = make_uint4(0, 0, 0, 0);
            }
        }

        // ---- logits: rows = entries, columns = heads
        f32x16 acc;
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] = 0.f;
        mma_tile<DT, HD>(acc, kf, qf);

        float tmax = -INFINITY;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int j = j0 + acc_row(r, hf);
            const float t = (j < s_hi) ? acc[r] * a.scale_log2 : -INFINITY;
            acc[r] = t;
            tmax = fmaxf(tmax, t);
        }
        tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
        const float m_new = fmaxf(m_run, tmax);          // finite: the tile holds at least one entry
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
        float psum = 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const float p = __builtin_amdgcn_exp2f(acc[r] - m_new);
            psum += p;
            if (l32 < GP) p_lds[wave][acc_row(r, hf)][l32] = p;
        }
        psum += __shfl_xor(psum, 32);
        l_run = l_run * alpha + psum;
        m_run = m_new;
        if (lane < GP) alpha_lds[wave][lane] = alpha;
        if (a.update_score && l32 < a.G) {
            float *lg = a.logits + ((long long)hg * a.G + l32) * a.Lcap;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int j = j0 + acc_row(r, hf);
                if (j < s_hi) lg[j] = acc[r];
            }
        }
        // the tile is private to this wave: order the LDS traffic, no workgroup barrier
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

        // ---- o = o * alpha + P^T V on the vector ALUs
        float al[GP];
#pragma unroll
        for (int h = 0; h < GP; ++h) al[h] = alpha_lds[wave][h];
#pragma unroll
        for (int h = 0; h < GP; ++h)
#pragma unroll
            for (int e = 0; e < EPU; ++e) o[h][e] *= al[h];
#pragma unroll
        for (int i = 0; i < VPL; ++i) {
            float vf[EPU];
            unpack<DT>(vv[i], vf);
            const float *pr = &p_lds[wave][vsub + KSUB * i][0];
#pragma unroll
            for (int h = 0; h < GP; ++h) {
                const float p = pr[h];
#pragma unroll
                for (int e = 0; e < EPU; ++e) o[h][e] = fmaf(p, vf[e], o[h][e]);
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }

    // ---- fold the lanes that hold the same V unit, then the four waves
#pragma unroll
    for (int h = 0; h < GP; ++h)
#pragma unroll
        for (int e = 0; e < EPU; ++e) {
            float x = o[h][e];
#pragma unroll
            for (int off = UPR; off < 64; off <<= 1) x += __shfl_xor(x, off);
            o[h][e] = x;
        }
    if (vsub == 0) {
#pragma unroll
        for (int h = 0; h < GP; ++h)
#pragma unroll
            for (int e = 0; e < EPU; ++e) wo[wave][h][vunit * EPU + e] = o[h][e];
    }
    if (lane < GP) {
        wm[wave][lane] = m_run;
        wl[wave][lane] = l_run;
    }
    __syncthreads();
    float *po = a.part_o + ((long long)hg * a.n_split + split) * GP * HD;
    for (int idx = tid; idx < GP * HD; idx += 256) {
        const int h = idx / HD, e = idx % HD;
        float mx = wm[0][h];
#pragma unroll
        for (int w = 1; w < 4; ++w) mx = fmaxf(mx, wm[w][h]);
        const float ms = (mx == -INFINITY) ? 0.f : mx;
        float s = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) s += wo[w][h][e] * __builtin_amdgcn_exp2f(wm[w][h] - ms);
        po[idx] = s;
    }
    if (tid < GP) {
        float mx = wm[0][tid];
#pragma unroll
        for (int w = 1; w < 4; ++w) mx = fmaxf(mx, wm[w][tid]);
        const float ms = (mx == -INFINITY) ? 0.f : mx;
        float s = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) s += wl[w][tid] * __builtin_amdgcn_exp2f(wm[w][tid] - ms);
        float *pml = a.part_ml + (((long long)hg * a.n_split + split) * GP + tid) * 2;
        pml[0] = mx;
        pml[1] = s;
    }
}

template <int DT, int HD, int GP>
__global__ __launch_bounds__(256) void attn_combine_kernel(AttnArgs a) {
    __shared__ float s_m[GP], s_inv[GP];
    const int tid = threadIdx.x;
    const int chunk = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
    const int hg = b * a.Hkv + g;
    const int L = a.cur_len[hg];
    const float *pml = a.part_ml + (long long)hg * a.n_split * GP * 2;
    if (tid < GP) {
        float mx = -INFINITY;
        for (int s = 0; s < a.n_split; ++s) mx = fmaxf(mx, pml[(s * GP + tid) * 2]);
        const float ms = (mx == -INFINITY) ? 0.f : mx;
        float l = 0.f;
        for (int s = 0; s < a.n_split; ++s)
            l += pml[(s * GP + tid) * 2 + 1] * exp2f(pml[(s * GP + tid) * 2] - ms);
        s_m[tid] = ms;
        s_inv[tid] = l > 0.f ? 1.0f / l : 0.f;
    }
    __syncthreads();

    if (chunk == 0) {
        const float *po = a.part_o + (long long)hg * a.n_split * GP * HD;
        for (int idx = tid; idx < a.G * HD; idx += 256) {
            const int h = idx / HD, e = idx % HD;
            float acc = 0.f;
            for (int s = 0; s < a.n_split; ++s)
                acc += po[((long long)s * GP + h) * HD + e] * exp2f(pml[(s * GP + h) * 2] - s_m[h]);
            acc *= s_inv[h];
            const long long oi = ((long long)b * a.Hq + g * a.G + h) * HD + e;
            if constexpr (DT == LVLM_BF16)
                reinterpret_cast<uint16_t *>(a.out)[oi] = f32_to_bf16(acc);
            else
                reinterpret_cast<float *>(a.out)[oi] = acc;
        }
        if (tid == 0 && a.append) a.len[hg] = L;
    }

    if (a.update_score) {
        const long long cbase = (long long)hg * a.Lmax;
        const float inv_g = 1.0f / (float)a.G;
        for (int j = chunk * 1024 + tid; j < min(L, (chunk + 1) * 1024); j += 256) {
            float pm = 0.f;
            for (int h = 0; h < a.G; ++h)
                pm += exp2f(a.logits[((long long)hg * a.G + h) * a.Lcap + j] - s_m[h]) * s_inv[h];
            const float old = (a.append && j == L - 1) ? 0.f : a.score[cbase + j];
            a.score[cbase + j] = a.decay * old + pm * inv_g;
        }
    }
}

template <int DT, int HD, int GP>
void launch_both(const Prof &prof, const AttnArgs &a, int B, int len_bound) {
    hipStream_t stream = prof.stream;
    prof.begin("attn_partial");
    hipLaunchKernelGGL((attn_partial_kernel<DT, HD, GP>), dim3(a.n_split, a.Hkv, B), dim3(256), 0, stream, a);
    prof.end();
    const int chunks = a.update_score ? (len_bound + 1023) / 1024 : 1;
    prof.begin("attn_combine");
    hipLaunchKernelGGL((attn_combine_kernel<DT, HD, GP>), dim3(chunks < 1 ? 1 : chunks, a.Hkv, B), dim3(256), 0,
                       stream, a);
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
    const int max_split = (bound + 127) / 128;
    long long want = (1024 + heads - 1) / heads;
    int n_split = (int)(want < 1 ? 1 : (want > max_split ? max_split : want));
    if (n_split < 1) n_split = 1;
    int split_len = ((bound + n_split - 1) / n_split + 127) / 128 * 128;
    n_split = (bound + split_len - 1) / split_len;
    if (n_split < 1) n_split = 1;
    w.n_split = n_split;
    w.split_len = split_len;
    const int G = d.Hq / d.Hkv, gp = group_pad(G);
    const int lcap = (bound + 3) / 4 * 4;
    w.part_ml = 0;
    w.part_o = align_up(w.part_ml + (size_t)heads * n_split * gp * 2 * sizeof(float), 256);
    w.logits = align_up(w.part_o + (size_t)heads * n_split * gp * d.hd * sizeof(float), 256);
    const size_t cur_len = align_up(w.logits + (size_t)heads * G * lcap * sizeof(float), 256);
    w.total = align_up(cur_len + (size_t)heads * sizeof(int32_t), 256);
    return w;
}

hipError_t launch_decode_attn(const Prof &prof, const lvlm_attn_desc &d, const AttnWs &w, char *ws, const void *q,
                              const void *k_new, const void *v_new, void *k_cache, void *v_cache, float *score,
                              uint8_t *kind, int32_t *orig_pos, int32_t *len, void *out) {
    const int bound = d.len_bound > 0 ? d.len_bound : d.Lmax;
    const long long heads = (long long)d.B * d.Hkv;
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
    const int lcap = (bound + 3) / 4 * 4;
    a.cur_len = reinterpret_cast<int32_t *>(ws + align_up(w.logits + (size_t)heads * G * lcap * sizeof(float), 256));
    a.Hq = d.Hq; a.Hkv = d.Hkv; a.G = G; a.Lmax = d.Lmax; a.Lcap = lcap;
    a.n_split = w.n_split; a.split_len = w.split_len;
    a.append = k_new != nullptr;
    a.new_kind = d.new_kind; a.new_pos = d.new_pos;
    a.update_score = score != nullptr;
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
