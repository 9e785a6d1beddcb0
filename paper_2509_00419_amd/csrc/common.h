// Shared declarations of the library's translation units: the context, the
// per-op launch entry points (host side) and a few device helpers.
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>
#include <stdio.h>

#include "../../include/lvlm.h"

struct lvlm_ctx {
    int device;
    void *ws;
    size_t ws_bytes;
    char err[256];
    // optional per-kernel timing (eager launches only): one event pair per bracket of launches
    bool prof_on;
    bool prof_open, prof_first;  // a bracket is open / it has launched nothing yet
    int prof_n, prof_cap;
    hipEvent_t *prof_ev;        // 2 * prof_cap events
    const char **prof_name;     // prof_cap static strings
};

namespace lvlm {

constexpr int kWave = 64;
constexpr float kLog2e = 1.4426950408889634f;

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// ---- workspace layouts (host arithmetic shared by the size query and the launch) ----
struct ScoreWs {
    size_t part_m, part_l, lse2, colpart, total;
    int nkb;       // key blocks of the normaliser pass
    int block_keys;
    int rs, cps;   // row splits per key block, query chunks per split
    bool single;   // short sequence: both passes in one launch, one part of column sums per query chunk
    bool shared_tiles;   // ... with four query chunks per workgroup sharing the key tiles through LDS
    int key_segs;        // ... and the keys cut into this many runs, a launch per sweep (1 = one launch)
};
ScoreWs score_ws(const lvlm_score_desc &d);

struct ProbsWs {
    size_t colpart, total;
    int rs;        // row groups of 32 rows (heads of a group x query rows) that are summed separately
};
ProbsWs probs_ws(const lvlm_probs_desc &d);

struct PrefillWs {
    size_t lse_t, redo, score, total;   // normalisers of the last T rows, redo marks per workgroup, the score pass's workspace
};
PrefillWs prefill_ws(const lvlm_prefill_desc &d);
lvlm_score_desc prefill_score_desc(const lvlm_prefill_desc &d);   // the score call the last T rows amount to

struct MergeWs {
    size_t rank_part, dst_of, wgt, partial, sorted, total;
    int n_split;   // always 1: the rank kernel leaves complete ranks
    int n_chunk;   // source-row chunks of the gather kernel (partial sums per chunk)
    int rows_per_chunk;
    int max_row_elems;
};
MergeWs merge_ws(const lvlm_merge_desc &d, const lvlm_plane *planes);

struct SimWs {
    size_t rank, dom_of, keep_idx, rest_idx, inv_norm, pbest_val, pbest_idx, assign, key, rank2, order, sorted, total;
    int tile;      // rows of dominant (and of other) tokens per workgroup tile of the similarity product
    int NB;        // blocks of `tile` dominant tokens
};
SimWs sim_ws(const lvlm_merge_desc &d);

struct KvWs {
    size_t src, total;
};
KvWs kv_ws(const lvlm_kv_desc &d);

struct AttnWs {
    size_t part_ml, part_o, logits, cur_len, total;
    int n_split, split_len, lcap, tail_entry;
};
AttnWs attn_ws(const lvlm_attn_desc &d);

// Names the kernel launches between begin() and end() for the optional timing.  The events are bound to the
// kernels themselves (the start event to the first launch of the bracket, the stop event to its last), so what
// is read back is the time from that kernel's first wave to its last -- the duration a kernel trace reports --
// without the dispatch gaps that events recorded around a launch would add.
struct Prof {
    lvlm_ctx *ctx;
    hipStream_t stream;
    void begin(const char *name) const {
        if (!ctx->prof_on || ctx->prof_n >= ctx->prof_cap) return;
        ctx->prof_name[ctx->prof_n] = name;
        ctx->prof_open = ctx->prof_first = true;
    }
    void end() const {
        if (!ctx->prof_open) return;
        ctx->prof_open = false;
        if (!ctx->prof_first) ++ctx->prof_n;     // a bracket without a launch leaves no entry
    }
    // the events the next launch carries (null: none), or false when no bracket is open
    bool events(hipEvent_t *start, hipEvent_t *stop) const {
        if (!ctx->prof_open) return false;
        *start = ctx->prof_first ? ctx->prof_ev[2 * ctx->prof_n] : nullptr;
        *stop = ctx->prof_ev[2 * ctx->prof_n + 1];
        ctx->prof_first = false;
        return true;
    }
};

// hipLaunchKernelGGL with a Prof in front: the same launch, carrying the open bracket's events if there is one.
#define LVLM_LAUNCH(prof, kernel, grid, block, lds_bytes, stream_, ...)                                      \
    do {                                                                                                     \
        hipEvent_t lvlm_ev0_, lvlm_ev1_;                                                                     \
        if ((prof).events(&lvlm_ev0_, &lvlm_ev1_))                                                           \
            hipExtLaunchKernelGGL(kernel, grid, block, lds_bytes, stream_, lvlm_ev0_, lvlm_ev1_, 0, __VA_ARGS__); \
        else                                                                                                 \
            hipLaunchKernelGGL(kernel, grid, block, lds_bytes, stream_, __VA_ARGS__);                        \
    } while (0)

// ---- launches (defined in the .hip files; all asynchronous on `stream`) ----
// scratch: rank_scratch_bytes(n, B) bytes for the sorted blocks of long sequences, or null (counting at any length)
size_t rank_scratch_bytes(int n, int B);
void launch_rank(const Prof &prof, const float *score, int32_t *rank, int n, int B, void *scratch);
hipError_t launch_score(const Prof &prof, const lvlm_score_desc &d, const ScoreWs &w, char *ws,
                        const void *q, const void *k, const float *row_lse, float *score_head,
                        float *score_mean);
hipError_t launch_score_probs(const Prof &prof, const lvlm_probs_desc &d, const ProbsWs &w, char *ws, const void *probs,
                              float *score_head, float *score_mean);
hipError_t launch_prefill_attn(const Prof &prof, const lvlm_prefill_desc &d, const PrefillWs &w, char *ws, const void *q,
                               const void *k, const void *v, void *out, float *row_lse, float *score_head,
                               float *score_mean);
hipError_t launch_merge(const Prof &prof, const lvlm_merge_desc &d, const MergeWs &w, char *ws,
                        const float *score_mean, const float *wtab, const lvlm_plane *planes,
                        int32_t *keep_idx, int32_t *merged_idx);
hipError_t launch_merge_similar(const Prof &prof, const lvlm_merge_desc &d, const SimWs &w, char *ws,
                                const float *score_mean, const lvlm_plane *planes, const float *size_in,
                                float *size_out, int32_t *keep_idx, int32_t *assign);
hipError_t launch_kv_compress(const Prof &prof, const lvlm_kv_desc &d, const KvWs &w, char *ws,
                              void *k_cache, void *v_cache, float *score, uint8_t *kind,
                              int32_t *orig_pos, int32_t *len, int32_t *n_evicted);
hipError_t launch_decode_attn(const Prof &prof, const lvlm_attn_desc &d, const AttnWs &w, char *ws,
                              const void *q, const void *k_new, const void *v_new, void *k_cache,
                              void *v_cache, float *score, uint8_t *kind, int32_t *orig_pos,
                              int32_t *len, void *out);

hipError_t launch_stream_probe(const Prof &prof, const void *src, size_t bytes, int n_workgroups, unsigned int *sink);

// Device address and size of the fixed scratch array that lvlm_decode_attn_static uses on the current device
// (looked up once per device; no allocation).
hipError_t attn_static_scratch(int device, char **ptr, size_t *bytes);

#if defined(__HIPCC__)
// ---- device helpers ----
__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

// round-to-nearest-even; NaN stays NaN
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return 0x7fc0;
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// Order-preserving map float -> u32: a < b  <=>  key(a) < key(b); -0 == +0;
// NaN maps to 0, below -inf.  Descending importance = descending key.
__device__ __forceinline__ uint32_t score_key(float x) {
    if (x != x) return 0u;
    x += 0.0f;
    uint32_t b = __float_as_uint(x);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

// Exact fixed-point image of a score used for cumulative thresholds:
// floor(clamp(score, 0, 2^16) * 2^32); NaN and negatives give 0.
// Computed as two 32-bit halves (integer part, then the fraction scaled by 2^32: both conversions
// truncate and both products are exact), which is much cheaper than a float -> u64 conversion.
__device__ __forceinline__ unsigned long long score_fixed(float s) {
    if (!(s > 0.0f)) return 0ull;
    s = fminf(s, 65536.0f);
    const unsigned int hi = (unsigned int)s;
    const unsigned int lo = (unsigned int)((s - (float)hi) * 4294967296.0f);
    return ((unsigned long long)hi << 32) | lo;
}

// Wave reductions that leave the result in every lane, without the LDS permute unit: inside a row of 16 lanes by
// data-parallel-primitive moves (swap neighbours, swap pairs, mirror the halves of 8, mirror the row), across the
// rows and the two half-waves by the lane-swap instructions.
__device__ __forceinline__ float dpp_quad1(float v) { return __int_as_float(__hip_move_dpp(__float_as_int(v), 0xB1, 0xF, 0xF, true)); }   // lanes 1,0,3,2
__device__ __forceinline__ float dpp_quad2(float v) { return __int_as_float(__hip_move_dpp(__float_as_int(v), 0x4E, 0xF, 0xF, true)); }   // lanes 2,3,0,1
__device__ __forceinline__ float dpp_half_mirror(float v) { return __int_as_float(__hip_move_dpp(__float_as_int(v), 0x141, 0xF, 0xF, true)); }
__device__ __forceinline__ float dpp_row_mirror(float v) { return __int_as_float(__hip_move_dpp(__float_as_int(v), 0x140, 0xF, 0xF, true)); }
__device__ __forceinline__ float swap_rows(float x) {          // the value of the lane 16 places away
    typedef unsigned u2 __attribute__((ext_vector_type(2)));
    const u2 r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float((threadIdx.x & 16) ? r.x : r.y);
}
__device__ __forceinline__ float swap_halves(float x) {        // the value of the lane 32 places away
    typedef unsigned u2 __attribute__((ext_vector_type(2)));
    const u2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float((threadIdx.x & 32) ? r.x : r.y);
}
__device__ __forceinline__ float wave_max(float v) {
    v = fmaxf(v, dpp_quad1(v));
    v = fmaxf(v, dpp_quad2(v));
    v = fmaxf(v, dpp_half_mirror(v));
    v = fmaxf(v, dpp_row_mirror(v));
    v = fmaxf(v, swap_rows(v));
    return fmaxf(v, swap_halves(v));
}
__device__ __forceinline__ float wave_sum(float v) {
    v += dpp_quad1(v);
    v += dpp_quad2(v);
    v += dpp_half_mirror(v);
    v += dpp_row_mirror(v);
    v += swap_rows(v);
    return v + swap_halves(v);
}
// Minimum of a 64-bit key over the wave, in every lane (the moves are bitwise: the halves travel as floats).
__device__ __forceinline__ unsigned long long wave_min_u64(unsigned long long v) {
#define LVLM_MIN_STEP(MOVE)                                                                          \
    {                                                                                                \
        const unsigned ph = __float_as_uint(MOVE(__uint_as_float((unsigned)(v >> 32))));             \
        const unsigned pl = __float_as_uint(MOVE(__uint_as_float((unsigned)v)));                     \
        const unsigned long long o = ((unsigned long long)ph << 32) | pl;                            \
        v = o < v ? o : v;                                                                           \
    }
    LVLM_MIN_STEP(dpp_quad1)
    LVLM_MIN_STEP(dpp_quad2)
    LVLM_MIN_STEP(dpp_half_mirror)
    LVLM_MIN_STEP(dpp_row_mirror)
    LVLM_MIN_STEP(swap_rows)
    LVLM_MIN_STEP(swap_halves)
#undef LVLM_MIN_STEP
    return v;
}
// Any associative, commutative OP over the wave's 32-bit or 64-bit values, in every lane, by the same moves.
template <class OP>
__device__ __forceinline__ uint32_t wave_reduce_u32(uint32_t v, OP op) {
#define LVLM_RED_STEP(MOVE) v = op(v, __float_as_uint(MOVE(__uint_as_float(v))));
    LVLM_RED_STEP(dpp_quad1)
    LVLM_RED_STEP(dpp_quad2)
    LVLM_RED_STEP(dpp_half_mirror)
    LVLM_RED_STEP(dpp_row_mirror)
    LVLM_RED_STEP(swap_rows)
    LVLM_RED_STEP(swap_halves)
#undef LVLM_RED_STEP
    return v;
}
template <class OP>
__device__ __forceinline__ unsigned long long wave_reduce_u64(unsigned long long v, OP op) {
#define LVLM_RED_STEP(MOVE)                                                                          \
    {                                                                                                \
        const unsigned ph = __float_as_uint(MOVE(__uint_as_float((unsigned)(v >> 32))));             \
        const unsigned pl = __float_as_uint(MOVE(__uint_as_float((unsigned)v)));                     \
        v = op(v, ((unsigned long long)ph << 32) | pl);                                              \
    }
    LVLM_RED_STEP(dpp_quad1)
    LVLM_RED_STEP(dpp_quad2)
    LVLM_RED_STEP(dpp_half_mirror)
    LVLM_RED_STEP(dpp_row_mirror)
    LVLM_RED_STEP(swap_rows)
    LVLM_RED_STEP(swap_halves)
#undef LVLM_RED_STEP
    return v;
}
#endif

}  // namespace lvlm
