// Steps 2-4 -- partition by importance, merge P_merged into one token, compact
// every plane that shares the token axis (Sec. 3.2.1, par. 4).
//
//   rank_kernel      rank[j] = number of image tokens that precede j in
//                    descending score order (ties: lower index first).  It is
//                    the counting definition itself, spread over the chip:
//                    64 tokens per workgroup, the keys staged in LDS and split
//                    over the 16 waves.  Nothing iterative or data dependent.
//                    Long sequences: rank_block_kernel + rank_search_kernel
//                    (blocks of 1024 tokens sorted by counting, then one
//                    binary search per token and block).
//   index_kernel     one workgroup per 4096 tokens: counts the kept tokens in
//                    front of its chunk, prefix-scans its own "kept" flags
//                    in index order and emits
//                    keep_idx (ascending), merged_idx (rank order) and, per
//                    source token, where it goes (row of P_unmerged or its
//                    rank inside P_merged).
//   gather_kernel    one streaming pass over every source row of every plane:
//                    a kept row is copied to its new place with 128-bit loads
//                    and stores, a merged row is multiplied by its rank weight
//                    and accumulated in fp32 registers; each row chunk leaves
//                    one partial sum.
//   finalize_kernel  adds the partial sums in chunk order, rounds once and
//                    writes P_new behind P_unmerged.
#include "common.h"
#include "planes.h"

namespace lvlm {
namespace {

constexpr int kGatherWgs = 1536;   // workgroups the gather launch aims for (six per compute unit)


constexpr int kRankTile = 8192;   // keys staged in LDS per step of the rank kernel (32 KB)
constexpr int kRankBlock = 64;    // tokens ranked by one workgroup (one per lane; the 16 waves split the keys)

struct RankArgs {
    const float *score;   // [B, n]
    int32_t *rank;        // [B, n]
    int n;
};

// rank[j] = #{i : key_i > key_j, or key_i == key_j and i < j}.  A workgroup ranks 64 tokens: every wave
// holds the same 64 tokens (one per lane) and counts over its own sixteenth of the staged keys, read
// from LDS as broadcast 128-bit words; the sixteen counts are added through LDS.
__global__ __launch_bounds__(1024) void rank_kernel(RankArgs a) {
    __shared__ __attribute__((aligned(16))) uint32_t keys[kRankTile];
    __shared__ int cnt_lds[16][kRankBlock];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int b = blockIdx.y;
    const int j0 = blockIdx.x * kRankBlock;
    const int j = j0 + lane;
    const float *score = a.score + (long long)b * a.n;
    const uint32_t kj = j < a.n ? score_key(score[j]) : 0u;
    int cnt = 0;
    for (int t0 = 0; t0 < a.n; t0 += kRankTile) {
        const int tile_n = min(kRankTile, a.n - t0);
        const int share = ((tile_n + 15) / 16 + 3) & ~3;          // keys per wave, a multiple of 4
        __syncthreads();
        for (int x = tid; x < 16 * share && x < kRankTile; x += 1024) {
            const int i = t0 + x;
            // Padding sits above every real index, so it only ever meets the ">" rule (or the full
            // rule with i > j): the lowest key can never precede anything.
            keys[x] = i < a.n ? score_key(score[i]) : 0u;
        }
        __syncthreads();
        const int x_lo = wave * share, x_hi = min(kRankTile, x_lo + share);
        // Groups of four keys: entirely below the block (i < j: ">=" precedes), entirely above
        // (i > j: only ">" precedes), or overlapping the block's own indices (full rule).
        const int below_end = min(x_hi, max(x_lo, (j0 - t0) & ~3));
        const int above_beg = max(x_lo, min(x_hi, (j0 + kRankBlock - t0 + 3) & ~3));
#pragma unroll 8
        for (int x = x_lo; x < below_end; x += 4) {
            const uint4 k4 = *reinterpret_cast<const uint4 *>(&keys[x]);
            cnt += (k4.x >= kj) + (k4.y >= kj) + (k4.z >= kj) + (k4.w >= kj);
        }
#pragma unroll 4
        for (int x = below_end; x < above_beg; x += 4) {
            const uint4 k4 = *reinterpret_cast<const uint4 *>(&keys[x]);
            const int i = t0 + x;
            cnt += ((k4.x > kj) | ((k4.x == kj) & (i < j))) + ((k4.y > kj) | ((k4.y == kj) & (i + 1 < j))) +
                   ((k4.z > kj) | ((k4.z == kj) & (i + 2 < j))) + ((k4.w > kj) | ((k4.w == kj) & (i + 3 < j)));
        }
#pragma unroll 8
        for (int x = above_beg; x < x_hi; x += 4) {
            const uint4 k4 = *reinterpret_cast<const uint4 *>(&keys[x]);
            cnt += (k4.x > kj) + (k4.y > kj) + (k4.z > kj) + (k4.w > kj);
        }
    }
    cnt_lds[wave][lane] = cnt;
    __syncthreads();
    if (wave == 0 && j < a.n) {
        int tot = 0;
#pragma unroll
        for (int w = 0; w < 16; ++w) tot += cnt_lds[w][lane];
        a.rank[(long long)b * a.n + j] = tot;
    }
}

// ---- ranks of long sequences: sorted blocks + binary searches ------------------------------------
// Counting costs n^2 comparisons; from kSortMinTokens tokens on the ranks come in two launches instead.
// A token's place in the order is told by one 64-bit word, key in the high half and inverted index in the low
// half: i precedes j  <=>  word_i > word_j (higher key, or the same key and the lower index).
//   rank_block_kernel   every block of 1024 tokens is sorted by counting WITHIN the block (1024 comparisons per
//                       token, spread over all workgroups): a token's word goes to its place in the block's
//                       descending order; places past the last token of a partly filled block hold 0 (below every word)
//   rank_search_kernel  a token's rank = over all sorted blocks, the number of words above its own, each found by
//                       a binary search (11 probes) in LDS; a workgroup stages eight blocks and searches them for
//                       256 tokens, the groups of eight add their counts into the rank
constexpr int kSortBlock = 1024;
constexpr int kSortMinTokens = 4096;
constexpr int kSortStage = 8;        // sorted blocks held in LDS at a time (64 KB)

__device__ __forceinline__ unsigned long long order_word(float score, int idx) {
    return ((unsigned long long)score_key(score) << 32) | (unsigned long long)(0xffffffffu - (uint32_t)idx);
}

struct SortArgs {
    const float *score;             // [B, n]
    unsigned long long *sorted;     // [B, n_blocks, 1024]
    int32_t *rank;                  // [B, n]
    int n, n_blocks;
};

// 64 tokens per workgroup (one per lane, the same in all 16 waves); wave w counts over words 64 w .. 64 w + 63 of
// the tokens' own block, read from LDS as broadcast 128-bit pairs.
__global__ __launch_bounds__(1024) void rank_block_kernel(SortArgs a) {
    __shared__ __attribute__((aligned(16))) unsigned long long words[kSortBlock];
    __shared__ int cnt_lds[16][64];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int b = blockIdx.y;
    const int j0 = blockIdx.x * 64, j = j0 + lane;
    const int blk = j0 / kSortBlock, r0 = blk * kSortBlock;
    const float *score = a.score + (long long)b * a.n;
    unsigned long long *out = a.sorted + ((long long)b * a.n_blocks + blk) * kSortBlock;
    if (j0 >= a.n) {                              // nothing but padding here (uniform over the workgroup)
        if (wave == 0) out[j - r0] = 0ull;
        return;
    }
    {
        const int i = r0 + tid;
        words[tid] = i < a.n ? order_word(score[i], i) : 0ull;
    }
    const unsigned long long mine = j < a.n ? order_word(score[j], j) : 0ull;
    __syncthreads();
    int cnt = 0;
#pragma unroll 8
    for (int x = 64 * wave; x < 64 * wave + 64; x += 2) {
        const ulonglong2 w2 = *reinterpret_cast<const ulonglong2 *>(&words[x]);
        cnt += (w2.x > mine) + (w2.y > mine);
    }
    cnt_lds[wave][lane] = cnt;
    __syncthreads();
    if (wave == 0) {
        int place = 0;
#pragma unroll
        for (int w = 0; w < 16; ++w) place += cnt_lds[w][lane];
        // tokens past the end fill the places past the last token (the real ones take 0 .. count-1 between them)
        if (j < a.n) {
            out[place] = mine;
            a.rank[(long long)b * a.n + j] = 0;          // the searches add to it
        } else {
            out[j - r0] = 0ull;
        }
    }
}

__global__ __launch_bounds__(256) void rank_search_kernel(SortArgs a) {
    __shared__ __attribute__((aligned(16))) unsigned long long words[kSortStage * kSortBlock];
    const int tid = threadIdx.x;
    const int b = blockIdx.y;
    const int j = blockIdx.x * 256 + tid;
    const unsigned long long mine = j < a.n ? order_word(a.score[(long long)b * a.n + j], j) : ~0ull;
    const uint4 *src = reinterpret_cast<const uint4 *>(a.sorted + (long long)b * a.n_blocks * kSortBlock);
    int rank = 0;
    {
        // one group of eight sorted blocks per workgroup (blockIdx.z): the groups' counts meet in rank[j], which
        // rank_block_kernel has set to 0, by an atomic add -- a CU streams too slowly to stage them all in turn
        const int g0 = blockIdx.z * kSortStage;
        const int nb = min(kSortStage, a.n_blocks - g0);
        const int units = nb * (kSortBlock / 2);                       // 16-byte units to stage
        constexpr int kUnits = kSortStage * (kSortBlock / 2), kPer = kUnits / 256;
        uint4 v[kPer];                                                 // all of a thread's loads in flight together
#pragma unroll
        for (int x = 0; x < kPer; ++x) v[x] = src[(long long)g0 * (kSortBlock / 2) + min(256 * x + tid, units - 1)];
#pragma unroll
        for (int x = 0; x < kPer; ++x)                                 // blocks past the last one: words of 0
            reinterpret_cast<uint4 *>(words)[256 * x + tid] = 256 * x + tid < units ? v[x] : make_uint4(0, 0, 0, 0);
        __syncthreads();
        // words above `mine` in each staged block: the blocks descend, so that is the first place whose word is
        // not above it.  Branch-free bisections, the eight blocks' side by side: their probes are independent.
        int pos[kSortStage];
#pragma unroll
        for (int bb = 0; bb < kSortStage; ++bb) pos[bb] = 0;
#pragma unroll
        for (int step = kSortBlock / 2; step >= 1; step >>= 1) {
#pragma unroll
            for (int bb = 0; bb < kSortStage; ++bb) pos[bb] += words[bb * kSortBlock + pos[bb] + step - 1] > mine ? step : 0;
        }
#pragma unroll
        for (int bb = 0; bb < kSortStage; ++bb) rank += pos[bb] + (words[bb * kSortBlock + pos[bb]] > mine ? 1 : 0);   // place 1023 itself
    }
    if (j < a.n) {
        if (gridDim.z == 1) a.rank[(long long)b * a.n + j] = rank;
        else atomicAdd(&a.rank[(long long)b * a.n + j], rank);
    }
}

struct IndexArgs {
    const int32_t *rank;
    int32_t *dst_of;       // [B, n]: >= 0 row inside the new image span; -1: most important merged token;
                           //         -2: any other merged token
    float *wgt;            // [B, n]: merge weight of the token (0 for kept tokens)
    int32_t *keep_idx;     // [B, n_keep-1] or null
    int32_t *merged_idx;   // [B, r+1] or null
    const float *w;        // rank -> weight table, or null for the linear table
    float lin_scale;       // 1 / (m (m+1) / 2)
    int n, n_keep;
};

// One workgroup per 4096 tokens of a sequence (thread t holds tokens 4t..4t+3 of its chunk).  The workgroup
// first counts the kept tokens in front of its chunk -- a pass over the ranks before it, all loads in flight
// together -- so the chunks need nothing from each other; one block-wide scan then gives every kept token its
// row in P_unmerged.  Then keep_idx (ascending), merged_idx (by rank) and the per-token destination are written.
constexpr int kIndexChunk = 4096;
__global__ __launch_bounds__(1024) void index_kernel(IndexArgs a) {
    __shared__ int wave_tot[16], wave_before[16];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int b = blockIdx.y;
    const int s0 = blockIdx.x * kIndexChunk;
    const int n_unmerged = a.n_keep - 1;
    const int32_t *rank = a.rank + (long long)b * a.n;
    int32_t *dst_of = a.dst_of + (long long)b * a.n;
    float *wgt = a.wgt + (long long)b * a.n;
    const int m = a.n - n_unmerged;

    // this chunk's ranks
    int rk[4];
    const int j0 = s0 + 4 * tid;
    if (j0 + 3 < a.n && (a.n & 3) == 0) {
        const int4 v = *reinterpret_cast<const int4 *>(rank + j0);
        rk[0] = v.x; rk[1] = v.y; rk[2] = v.z; rk[3] = v.w;
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) rk[e] = j0 + e < a.n ? rank[j0 + e] : 0x7fffffff;
    }
    // kept tokens before the chunk (s0 is a multiple of 4096: whole 16-byte words when the rows are aligned)
    int before = 0;
    if ((a.n & 3) == 0) {
        for (int i = 4 * tid; i < s0; i += 4 * 1024) {
            const int4 v = *reinterpret_cast<const int4 *>(rank + i);
            before += (v.x < n_unmerged) + (v.y < n_unmerged) + (v.z < n_unmerged) + (v.w < n_unmerged);
        }
    } else {
        for (int i = tid; i < s0; i += 1024) before += rank[i] < n_unmerged;
    }
    int cnt = 0;
#pragma unroll
    for (int e = 0; e < 4; ++e) cnt += rk[e] < n_unmerged;
    int incl = cnt;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int t = __shfl_up(incl, o);
        if (lane >= o) incl += t;
        before += __shfl_xor(before, o);
    }
    if (lane == 63) wave_tot[wave] = incl;
    if (lane == 0) wave_before[wave] = before;
    __syncthreads();
    int p = incl - cnt;
#pragma unroll
    for (int w = 0; w < 16; ++w) p += wave_before[w] + (w < wave ? wave_tot[w] : 0);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int j = j0 + e;
        if (j >= a.n) continue;
        if (rk[e] < n_unmerged) {
            dst_of[j] = p;
            wgt[j] = 0.f;
            if (a.keep_idx) a.keep_idx[(long long)b * n_unmerged + p] = j;
            ++p;
        } else {
            const int k = rk[e] - n_unmerged;
            dst_of[j] = k == 0 ? -1 : -2;
            wgt[j] = a.w ? a.w[k] : (float)(m - k) * a.lin_scale;
            if (a.merged_idx) a.merged_idx[(long long)b * m + k] = j;
        }
    }
}

// ---- gather -----------------------------------------------------------------

struct GatherArgs {
    PlaneDev plane[LVLM_MAX_PLANES];
    const int32_t *dst_of;   // null: identity (nothing removed)
    const float *wgt;        // per-token merge weight
    float *partial;          // [B][n_planes][n_sub_max][max_row_elems]
    int B, N, img_begin, n_img, n_keep, n_planes;
    int rows_per_sub, n_sub_max, max_row_elems;
};

// One thread group walks `rows_per_sub` consecutive source rows of one plane, one unit column per thread.
// The loop is free of data-dependent branches before its stores: row data, destination code and weight
// of a batch of RB rows are loaded unconditionally (indices clamped into range), so the loads of many
// rows are in flight at once; then kept rows are stored and every row is multiplied by its weight (zero
// unless it is merged) and accumulated.
template <int DT, int UB>
__device__ __forceinline__ void gather_plane(const GatherArgs &a, const PlaneDev &p, int pi, int b) {
    using U = typename Unit<UB>::type;
    constexpr int RB = 8;   // rows per batch (all of a batch's loads are in flight together)
    const int tid = threadIdx.x;
    const int tpr = 1 << p.tpr_log2;
    const int group = tid >> p.tpr_log2;
    const int groups = 256 >> p.tpr_log2;
    const int sub = blockIdx.x * groups + group;
    const int row_units = p.row_bytes / UB;
    if (sub >= p.n_sub || (int)blockIdx.y >= p.col_blocks) return;
    const int unit_raw = blockIdx.y * 256 + (tid & (tpr - 1));
    const bool active = unit_raw < row_units;
    const int unit = active ? unit_raw : row_units - 1;
    const int r = a.n_img - a.n_keep;
    const char *src = p.src + (long long)b * p.src_stride_b + (long long)unit * UB;
    char *dst = p.dst + (long long)b * p.dst_stride_b + (long long)unit * UB;
    const int n_lo = sub * a.rows_per_sub;
    const int n_hi = min(a.N, n_lo + a.rows_per_sub);
    if (a.dst_of == nullptr) {
        // nothing is removed (kernel-uniform case): plain row copy
        if (active) {
#pragma unroll 4
            for (int n = n_lo; n < n_hi; ++n)
                *reinterpret_cast<U *>(dst + (long long)n * p.row_bytes) =
                    *reinterpret_cast<const U *>(src + (long long)n * p.row_bytes);
        }
        return;
    }
    const int32_t *dst_of = a.dst_of + (long long)b * a.n_img;
    const float *wgt = a.wgt + (long long)b * a.n_img;
    const bool weighted = p.rule == LVLM_RULE_WEIGHTED;             // uniform per plane
    const int new_row = a.img_begin + a.n_keep - 1;

    Acc<DT, UB> acc;
#pragma unroll
    for (int i = 0; i < Acc<DT, UB>::NE; ++i) acc.v[i] = 0.f;

    for (int n0 = n_lo; n0 < n_hi; n0 += RB) {
        // all loads of the batch first (clamped row / token indices keep every address valid) ...
        U val[RB];
        int code[RB];
        float wk[RB];
#pragma unroll
        for (int x = 0; x < RB; ++x) {
            const int n = min(n0 + x, n_hi - 1);
            const int j = min(max(n - a.img_begin, 0), a.n_img - 1);
            val[x] = *reinterpret_cast<const U *>(src + (long long)n * p.row_bytes);
            code[x] = dst_of[j];
            wk[x] = wgt[j];
        }
        // ... then the stores and the weighted accumulation
#pragma unroll
        for (int x = 0; x < RB; ++x) {
            const int n = n0 + x;
            const bool valid = active && n < n_hi;
            const bool in_img = n >= a.img_begin && n < a.img_begin + a.n_img;
            int dest = n < a.img_begin ? n : n - r;                  // rows outside the image span
            if (in_img) dest = code[x] >= 0 ? a.img_begin + code[x] : (code[x] == -1 && !weighted ? new_row : -1);
            if (valid && dest >= 0) *reinterpret_cast<U *>(dst + (long long)dest * p.row_bytes) = val[x];
            // Only the rows of P_merged enter the sum (a kept or text row must not, whatever it holds: 0 * inf
            // would poison the merged token).  A row is shared by whole waves for all but the narrowest planes,
            // so the test is uniform there.
            if constexpr (DT != LVLM_I32) {
                if (weighted && valid && in_img && code[x] < 0) accumulate<DT, UB>(acc, val[x], wk[x]);
            }
        }
    }
    if constexpr (DT != LVLM_I32) {
        if (weighted && active) {
            constexpr int NE = Acc<DT, UB>::NE;
            float *out = a.partial + (((long long)b * a.n_planes + pi) * a.n_sub_max + sub) * a.max_row_elems +
                         (long long)unit * NE;
#pragma unroll
            for (int i = 0; i < NE; ++i) out[i] = acc.v[i];
        }
    }
}

__global__ __launch_bounds__(256) void gather_kernel(GatherArgs a) {
    const int pi = blockIdx.z / a.B, b = blockIdx.z % a.B;
    // (selected by comparison: indexing the argument array with a run-time value would copy it to scratch)
    PlaneDev p = a.plane[0];
#pragma unroll
    for (int i = 1; i < LVLM_MAX_PLANES; ++i)
        if (pi == i) p = a.plane[i];
    if (p.dtype == LVLM_BF16) {
        if (p.unit_bytes == 16) gather_plane<LVLM_BF16, 16>(a, p, pi, b);
        else if (p.unit_bytes == 4) gather_plane<LVLM_BF16, 4>(a, p, pi, b);
        else gather_plane<LVLM_BF16, 2>(a, p, pi, b);
    } else if (p.dtype == LVLM_F32) {
        if (p.unit_bytes == 16) gather_plane<LVLM_F32, 16>(a, p, pi, b);
        else gather_plane<LVLM_F32, 4>(a, p, pi, b);
    } else {
        if (p.unit_bytes == 16) gather_plane<LVLM_I32, 16>(a, p, pi, b);
        else gather_plane<LVLM_I32, 4>(a, p, pi, b);
    }
}

// P_new[c] = sum of the chunks' partial sums, rounded once.  A workgroup owns 16 columns; its 16 thread
// rows each add a contiguous share of the chunks (independent loads, unrolled), then the shares are
// added in order -- a fixed summation tree, so the result is reproducible.
__global__ __launch_bounds__(256) void finalize_kernel(GatherArgs a) {
    __shared__ float share[16][17];
    const int pi = blockIdx.y / a.B, b = blockIdx.y % a.B;
    const PlaneDev &p = a.plane[pi];
    if (p.rule != LVLM_RULE_WEIGHTED) return;
    const int col = threadIdx.x & 15, grp = threadIdx.x >> 4;
    const int c = blockIdx.x * 16 + col;
    if ((int)blockIdx.x * 16 >= p.row_elems) return;
    const int per = (p.n_sub + 15) / 16;
    const int i_lo = grp * per, i_hi = min(p.n_sub, i_lo + per);
    float s = 0.f;
    if (c < p.row_elems) {
        const float *part = a.partial + ((long long)b * a.n_planes + pi) * a.n_sub_max * a.max_row_elems + c;
#pragma unroll 8
        for (int i = i_lo; i < i_hi; ++i) s += part[(long long)i * a.max_row_elems];
    }
    share[grp][col] = s;
    __syncthreads();
    if (grp == 0 && c < p.row_elems) {
        float t = 0.f;
#pragma unroll
        for (int g2 = 0; g2 < 16; ++g2) t += share[g2][col];
        char *dst = p.dst + (long long)b * p.dst_stride_b + (long long)(a.img_begin + a.n_keep - 1) * p.row_bytes;
        if (p.dtype == LVLM_BF16)
            reinterpret_cast<uint16_t *>(dst)[c] = f32_to_bf16(t);
        else
            reinterpret_cast<float *>(dst)[c] = t;
    }
}

}  // namespace

size_t rank_scratch_bytes(int n, int B) {
    if (n < kSortMinTokens) return 0;
    return (size_t)B * ((n + kSortBlock - 1) / kSortBlock) * kSortBlock * sizeof(unsigned long long);
}

void launch_rank(const Prof &prof, const float *score, int32_t *rank, int n, int B, void *scratch) {
    hipStream_t stream = prof.stream;
    if (scratch && n >= kSortMinTokens) {
        SortArgs sa{};
        sa.score = score;
        sa.sorted = static_cast<unsigned long long *>(scratch);
        sa.rank = rank;
        sa.n = n;
        sa.n_blocks = (n + kSortBlock - 1) / kSortBlock;
        LVLM_LAUNCH(prof, rank_block_kernel, dim3(sa.n_blocks * (kSortBlock / 64), B), dim3(1024), 0, stream, sa);
        LVLM_LAUNCH(prof, rank_search_kernel, dim3((n + 255) / 256, B, (sa.n_blocks + kSortStage - 1) / kSortStage), dim3(256), 0,
                    stream, sa);
        return;
    }
    RankArgs ra{};
    ra.score = score;
    ra.rank = rank;
    ra.n = n;
    LVLM_LAUNCH(prof, rank_kernel, dim3((n + kRankBlock - 1) / kRankBlock, B), dim3(1024), 0, stream, ra);
}

MergeWs merge_ws(const lvlm_merge_desc &d, const lvlm_plane *planes) {
    MergeWs w{};
    w.n_split = 1;
    // gather kernel: rows per partial sum
    int max_elems = 1;
    long long units = 0;
    for (int i = 0; i < d.n_planes; ++i) {
        if (planes[i].row_elems > max_elems) max_elems = planes[i].row_elems;
        units += ((long long)planes[i].row_elems * elem_bytes(planes[i].dtype) + 4095) / 4096;
    }
    // about six workgroups per CU (a workgroup waits out the memory latency of every batch of rows, so the
    // overlap comes from its neighbours); longer chunks would mean fewer partial sums to write and re-read
    long long rows = (long long)d.N * d.B * (units ? units : 1) / kGatherWgs;
    rows = rows / 4 * 4;
    w.rows_per_chunk = (int)(rows < 8 ? 8 : (rows > 128 ? 128 : rows));
    w.n_chunk = (d.N + w.rows_per_chunk - 1) / w.rows_per_chunk;
    w.max_row_elems = max_elems;
    w.rank_part = 0;
    w.dst_of = align_up(w.rank_part + (size_t)d.B * w.n_split * d.n_img * sizeof(int32_t), 256);
    w.wgt = align_up(w.dst_of + (size_t)d.B * d.n_img * sizeof(int32_t), 256);
    w.partial = align_up(w.wgt + (size_t)d.B * d.n_img * sizeof(float), 256);
    w.sorted = align_up(w.partial + (size_t)d.B * d.n_planes * w.n_chunk * max_elems * sizeof(float), 256);
    w.total = align_up(w.sorted + rank_scratch_bytes(d.n_img, d.B), 256);
    return w;
}

hipError_t launch_merge(const Prof &prof, const lvlm_merge_desc &d, const MergeWs &w, char *ws,
                        const float *score_mean, const float *wtab, const lvlm_plane *planes, int32_t *keep_idx,
                        int32_t *merged_idx) {
    hipStream_t stream = prof.stream;
    const int r = d.n_img - d.n_keep;
    GatherArgs g{};
    g.B = d.B; g.N = d.N; g.img_begin = d.img_begin; g.n_img = d.n_img; g.n_keep = d.n_keep;
    g.n_planes = d.n_planes;
    g.rows_per_sub = w.rows_per_chunk;
    g.n_sub_max = w.n_chunk;
    g.max_row_elems = w.max_row_elems;
    g.partial = reinterpret_cast<float *>(ws + w.partial);
    const double m = (double)r + 1.0;
    g.dst_of = r > 0 ? reinterpret_cast<const int32_t *>(ws + w.dst_of) : nullptr;
    g.wgt = reinterpret_cast<const float *>(ws + w.wgt);

    int grid_x = 1, grid_y = 1;
    bool any_weighted = false;
    for (int i = 0; i < d.n_planes; ++i) {
        PlaneDev &p = g.plane[i];
        p = make_plane_dev(planes[i]);
        p.n_sub = w.n_chunk;
        const int groups = 256 >> p.tpr_log2;
        const int gx = (p.n_sub + groups - 1) / groups;
        if (gx > grid_x) grid_x = gx;
        if (p.col_blocks > grid_y) grid_y = p.col_blocks;
        any_weighted |= p.rule == LVLM_RULE_WEIGHTED;
    }

    if (r > 0) {
        int32_t *rank = reinterpret_cast<int32_t *>(ws + w.rank_part);
        prof.begin("merge_rank");
        launch_rank(prof, score_mean, rank, d.n_img, d.B, ws + w.sorted);
        prof.end();
        IndexArgs ia{};
        ia.rank = rank;
        ia.dst_of = reinterpret_cast<int32_t *>(ws + w.dst_of);
        ia.wgt = reinterpret_cast<float *>(ws + w.wgt);
        ia.w = wtab;
        ia.lin_scale = (float)(1.0 / (m * (m + 1.0) / 2.0));
        ia.keep_idx = keep_idx;
        ia.merged_idx = merged_idx;
        ia.n = d.n_img; ia.n_keep = d.n_keep;
        prof.begin("merge_index");
        LVLM_LAUNCH(prof, index_kernel, dim3((d.n_img + kIndexChunk - 1) / kIndexChunk, d.B), dim3(1024), 0, stream, ia);
        prof.end();
    }
    prof.begin("merge_gather");
    LVLM_LAUNCH(prof, gather_kernel, dim3(grid_x, grid_y, d.B * d.n_planes), dim3(256), 0, stream, g);
    prof.end();
    if (r > 0 && any_weighted) {
        prof.begin("merge_finalize");
        LVLM_LAUNCH(prof, finalize_kernel, dim3((w.max_row_elems + 15) / 16, d.B * d.n_planes), dim3(256), 0,
                           stream, g);
        prof.end();
    }
    return hipGetLastError();
}

}  // namespace lvlm
