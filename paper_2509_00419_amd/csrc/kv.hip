// Step 5 -- KV-cache compression, independently per (batch, KV head) (Sec. 3.2.2).
//
// Neither rule needs a sort.  Both ask for "the best entries until a quota is
// met", where the quota is a number of entries (fixed budget) or an amount of
// score mass (threshold beta).  A most-significant-digit radix descent over the
// order-preserving 32-bit image of the score finds, in at most four histogram passes,
// the key K* at which the quota is met: entries above K* stay, entries below go,
// and among the entries equal to K* the lowest slots stay.  Score mass is summed
// as exact integers, so the result does not depend on summation order.  (Digits of
// 9 bits over the bits in which the head's keys differ: at most four histogram passes.)
//
//   kv_select_kernel  one workgroup per head: totals, radix descent, then one
//                     pass in slot order that numbers survivors / holes.  With
//                     LVLM_ORDER_FILL it also performs the (few, disjoint)
//                     moves itself.
//   kv_fill_kernel    LVLM_ORDER_FILL with many moves per head (bulk eviction): the
//                     disjoint moves, spread over the chip.
//   kv_move_kernel    LVLM_ORDER_STABLE: survivors slide down in place.  A move
//                     never goes up and sources are ascending, so processing
//                     destination slots in ascending steps, each step reading
//                     everything before writing anything, is safe; column
//                     slices of the rows are independent and go to different
//                     workgroups.
#include "common.h"

namespace lvlm {
namespace {

struct KvArgs {
    char *k;
    char *v;
    float *score;
    uint8_t *kind;
    int32_t *pos;
    int32_t *len;
    int32_t *n_evicted;
    int32_t *list_a;   // [B*Hkv, Lmax]  STABLE: source slot of each new slot; FILL: holes
    int32_t *list_b;   // [B*Hkv, Lmax]  FILL: survivors beyond the new length
    int32_t *meta;     // [B*Hkv, 2]     STABLE: {new length, first destination slot that moves}
    int Hkv, Lmax, bound, row_bytes, mode, order, budget, n_recent;   // bound: the caller's len_bound (<= Lmax)
    double beta;
    int fill_external;   // FILL order: the moves are left to kv_fill_kernel (meta[1] = their number)
};

constexpr int kDigitBits = 9;     // radix digit width: three passes cover 27 differing key bits
constexpr int kBins = 1 << kDigitBits;
constexpr int kSub = 2;           // copies of every histogram bin (lane % kSub picks one): scores of one head
                                  // may crowd into few digits, and LDS atomics on one address go one at a time
constexpr int kChunkMax = 17;     // most chunks (one slot per thread each) numbered per round of the slot-order pass

// Exact fixed-point mass of a candidate, from its order-preserving key alone: keys with the top bit set
// are the non-negative scores (bit pattern = key without that bit); negative scores and NaN weigh 0.
__device__ __forceinline__ unsigned long long key_mass(uint32_t key) {
    return (key & 0x80000000u) ? score_fixed(__uint_as_float(key & 0x7fffffffu)) : 0ull;
}

// Where digit d sits in a histogram: lane l of the wave that scans it owns digits 8 l .. 8 l + 7 and reads
// them in eight steps; with digit d at row (d % 8) 64 + d / 8 the lanes of one step read neighbouring rows
// (with the digits in order they would all meet in one LDS bank).
static_assert(kBins == 512, "eight digits per lane");
__device__ __forceinline__ uint32_t digit_row(uint32_t d) { return ((d & 7u) << 6) | (d >> 3); }

struct SelectShared {
    unsigned long long hist_m[2][kBins][kSub];   // two histograms: one is cleared while the other is in use;
    unsigned int hist_c[2][kBins][kSub];         // rows by digit_row()
    unsigned long long need_next, last_m;
    unsigned int cabove, digit, last_c;
    int first_hole;
    unsigned long long w_best[16];   // per-wave partial results of the block reductions
    unsigned long long w_mass[16];
    uint32_t w_min[16], w_max[16];
    int w_cnt[16];
    int cnt[2][kChunkMax * 16 + 1];  // slot-order pass: per (chunk, wave) counts of two flags, then their
                                     // exclusive prefixes in (chunk, wave) order; last element: the total
};

// Wave 0, after a histogram pass: suffix sums over the digits give the mass (and count) above each
// digit; the digit in which the quota `need` (> 0, at most the mass in the histogram) is met becomes the
// next digit of the key.
__device__ __forceinline__ void pick_digit(SelectShared &sh, int cur, unsigned long long need, bool count_only) {
    const int lane = threadIdx.x & 63;
    constexpr int PER = kBins / 64;     // lane owns PER consecutive digits
    unsigned long long loc_m = 0ull;
    unsigned int loc_c = 0u;
    unsigned long long hm[PER];
    unsigned int hc[PER];
#pragma unroll
    for (int i = 0; i < PER; ++i) {
        hm[i] = 0ull;
        hc[i] = 0u;
        static_assert(kSub == 2, "two copies are added here");
        static_assert(PER == 8, "digit_row() places eight digits per lane");
        const int row = 64 * i + lane;              // = digit_row(PER * lane + i)
        if (!count_only) hm[i] = sh.hist_m[cur][row][0] + sh.hist_m[cur][row][1];
        hc[i] = sh.hist_c[cur][row][0] + sh.hist_c[cur][row][1];
        if (count_only) hm[i] = hc[i];
        loc_m += hm[i];
        loc_c += hc[i];
    }
    unsigned long long inc_m = loc_m;
    unsigned int inc_c = loc_c;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const unsigned long long tm = __shfl_down(inc_m, o);
        const unsigned int tc = __shfl_down(inc_c, o);
        if (lane + o < 64) {
            inc_m += tm;
            inc_c += tc;
        }
    }
    unsigned long long above_m = inc_m - loc_m;
    unsigned int above_c = inc_c - loc_c;
#pragma unroll
    for (int i = PER - 1; i >= 0; --i) {
        if (above_m < need && need <= above_m + hm[i]) {
            sh.digit = (unsigned int)(PER * lane + i);
            sh.need_next = need - above_m;
            sh.cabove += above_c;     // exactly one lane and one digit take this branch
            sh.last_m = hm[i];
            sh.last_c = hc[i];
        }
        above_m += hm[i];
        above_c += hc[i];
    }
}

// Slot-order numbering of two flags over NCH chunks of NT slots (thread t holds slot NT c + t of
// chunk c; bit c of f0 / f1 is its flag).  Returns in e0[c] / e1[c] the number of flagged slots before
// the thread's slot of chunk c within this round (packed: flag 0 in the low, flag 1 in the high 16 bits;
// a round has fewer than 2^16 slots), and the round totals.  Every wave files its ballots'
// counts, waves 0 and 1 turn the two NCH x NT/64 tables into exclusive prefixes, every thread adds the lanes below it.
// Two barriers; the table may be reused after one more barrier.
template <int NCH, int NT>
__device__ __forceinline__ void chunk_scan2(SelectShared &sh, uint32_t f0, uint32_t f1, uint32_t (&e)[NCH], int &t0,
                                            int &t1) {
    static_assert(NCH * NT < 65536, "packed counts need 16 bits");
    constexpr int NW = NT / 64;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const unsigned long long below = (1ull << lane) - 1ull;
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        const unsigned long long b0 = __ballot((f0 >> c) & 1u), b1 = __ballot((f1 >> c) & 1u);
        e[c] = (uint32_t)__popcll(b0 & below) | ((uint32_t)__popcll(b1 & below) << 16);
        if (lane == 0) {
            sh.cnt[0][NW * c + wave] = __popcll(b0);
            sh.cnt[1][NW * c + wave] = __popcll(b1);
        }
    }
    __syncthreads();
    if (wave < 2) {
        // wave k scans table k: lane owns PER consecutive entries
        constexpr int N = NCH * NW;
        constexpr int PER = (N + 63) / 64;
        int *tab = sh.cnt[wave];
        int v[PER];
        int sum = 0;
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int idx = PER * lane + i;
            v[i] = idx < N ? tab[idx] : 0;
            sum += v[i];
        }
        int inc = sum;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int u = __shfl_up(inc, o);
            if (lane >= o) inc += u;
        }
        int run = inc - sum;
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int idx = PER * lane + i;
            if (idx < N) tab[idx] = run;
            run += v[i];
        }
        if (lane == 63) tab[N] = inc;
    }
    __syncthreads();
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        e[c] += (uint32_t)sh.cnt[0][NW * c + wave] | ((uint32_t)sh.cnt[1][NW * c + wave] << 16);
    }
    t0 = sh.cnt[0][NCH * NW];
    t1 = sh.cnt[1][NCH * NW];
}

// NT threads per head.  KPT > 0: every thread keeps the keys of its KPT slots (slot = NT i + thread) in
// registers, so the scores are read once, with all loads in flight together; heads longer than NT KPT are not accepted
// by the launch.  KPT == 0: any length, scores re-read from memory in every pass.
template <int KPT, int NT>
__global__ __launch_bounds__(NT) void kv_select_kernel(KvArgs a) {
    constexpr int NW = NT / 64;
    __shared__ SelectShared sh;
    constexpr int NREG = KPT > 0 ? KPT : 1;
    // slots per thread in one round of the slot-order pass: register-resident keys go in one round, or in two
    // when there are many (the numbering state of a round is live across its barriers)
    constexpr int CH = KPT > 8 ? (KPT + 1) / 2 : KPT > 0 ? KPT : 16;
    constexpr int NROUND = KPT > 0 ? (KPT + CH - 1) / CH : 1;
    static_assert(CH <= kChunkMax, "count table too small");

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int hg = blockIdx.x;
    const long long base = (long long)hg * a.Lmax;
    const float *score = a.score + base;
    const uint8_t *kind = a.kind + base;
    // The launch (keys per thread, list sizes) was sized for heads of at most `bound` entries.  A head that is
    // longer than the caller said is left exactly as it is: nothing evicted, length untouched.
    const int len0 = a.len[hg];
    const int L = len0 > a.bound ? 0 : len0;
    const bool budget_mode = a.mode == LVLM_KV_BUDGET;

    auto nothing_to_do = [&]() {
        if (tid == 0) {
            if (a.n_evicted) a.n_evicted[hg] = 0;
            a.meta[2 * hg] = L;
            a.meta[2 * hg + 1] = a.fill_external ? 0 : L;
        }
    };
    if ((budget_mode && L <= a.budget) || (!budget_mode && !(a.beta < 1.0)) || L <= 0) {
        nothing_to_do();
        return;
    }
    const int recent_lo = L - a.n_recent;
    auto is_cand = [&](int slot, uint8_t kd) -> bool {
        return budget_mode ? (kd != LVLM_KIND_PROTECTED && slot < recent_lo) : (kd == LVLM_KIND_IMAGE);
    };

    // register-resident keys; bit i of `candm` marks slot NT i + tid as a candidate
    uint32_t key[NREG];
    uint32_t candm = 0u;
    if constexpr (KPT > 0) {
        float sc[NREG];
        uint8_t kd[NREG];
#pragma unroll
        for (int i = 0; i < NREG; ++i) {
            const int sl = min(NT * i + tid, L - 1);     // clamped: every load is issued, none depends on another
            sc[i] = score[sl];
            kd[i] = kind[sl];
        }
#pragma unroll
        for (int i = 0; i < NREG; ++i) {
            const int slot = NT * i + tid;
            key[i] = score_key(sc[i]);
            if (slot < L && is_cand(slot, kd[i])) candm |= 1u << i;
        }
    } else {
        key[0] = 0u;
    }

    // ---- steady-state decode: the head is exactly one entry over budget and holes are filled from
    // the tail.  One pass finds the candidate that is last in importance order (lowest key, highest
    // slot among equals); the entry in the last slot takes its place.
    if (budget_mode && a.order == LVLM_ORDER_FILL && L - a.budget == 1) {
        unsigned long long best = ~0ull;
        int cnt = 0;
        if constexpr (KPT > 0) {
#pragma unroll
            for (int i = 0; i < NREG; ++i) {
                if (candm & (1u << i)) {
                    ++cnt;
                    const unsigned long long c =
                        ((unsigned long long)key[i] << 32) | (unsigned long long)(0xffffffffu - (uint32_t)(NT * i + tid));
                    best = c < best ? c : best;
                }
            }
        } else {
            for (int slot = tid; slot < L; slot += NT) {
                if (is_cand(slot, kind[slot])) {
                    ++cnt;
                    const unsigned long long c = ((unsigned long long)score_key(score[slot]) << 32) |
                                                 (unsigned long long)(0xffffffffu - (uint32_t)slot);
                    best = c < best ? c : best;
                }
            }
        }
        best = wave_min_u64(best);
        cnt = (int)wave_reduce_u32((uint32_t)cnt, [](uint32_t x, uint32_t y) { return x + y; });
        if (lane == 0) {
            sh.w_best[wave] = best;
            sh.w_cnt[wave] = cnt;
        }
        __syncthreads();
        best = sh.w_best[0];
        cnt = sh.w_cnt[0];
#pragma unroll
        for (int w = 1; w < NW; ++w) {
            best = sh.w_best[w] < best ? sh.w_best[w] : best;
            cnt += sh.w_cnt[w];
        }
        if (a.budget - (L - cnt) > 0) {           // room for all but one candidate
            const int victim = (int)(0xffffffffu - (uint32_t)(best & 0xffffffffull));
            const int last = L - 1;
            if (victim != last) {
                const int units = a.row_bytes / 16;
                char *kc = a.k + base * a.row_bytes;
                char *vc = a.v + base * a.row_bytes;
                if (tid < units)
                    *reinterpret_cast<uint4 *>(kc + (long long)victim * a.row_bytes + 16 * tid) =
                        *reinterpret_cast<const uint4 *>(kc + (long long)last * a.row_bytes + 16 * tid);
                else if (tid < 2 * units)
                    *reinterpret_cast<uint4 *>(vc + (long long)victim * a.row_bytes + 16 * (tid - units)) =
                        *reinterpret_cast<const uint4 *>(vc + (long long)last * a.row_bytes + 16 * (tid - units));
                else if (tid == 2 * units) {
                    a.score[base + victim] = a.score[base + last];
                    a.kind[base + victim] = a.kind[base + last];
                    a.pos[base + victim] = a.pos[base + last];
                }
            }
            if (tid == 0) {
                a.meta[2 * hg] = last;
                a.meta[2 * hg + 1] = a.fill_external ? 0 : last;
                a.len[hg] = last;
                if (a.n_evicted) a.n_evicted[hg] = 1;
            }
            return;
        }
        __syncthreads();     // protected entries alone exceed the budget: general path below
    }

    // ---- totals and the key range of the candidates (one block reduction)
    {
        unsigned long long mass = 0ull;
        int cnt = 0;
        uint32_t kmin = 0xffffffffu, kmax = 0u;
        auto see = [&](uint32_t k) {
            ++cnt;
            mass += budget_mode ? 1ull : key_mass(k);
            kmin = min(kmin, k);
            kmax = max(kmax, k);
        };
        if constexpr (KPT > 0) {
#pragma unroll
            for (int i = 0; i < NREG; ++i)
                if (candm & (1u << i)) see(key[i]);
        } else {
            for (int slot = tid; slot < L; slot += NT)
                if (is_cand(slot, kind[slot])) see(score_key(score[slot]));
        }
        mass = wave_reduce_u64(mass, [](unsigned long long x, unsigned long long y) { return x + y; });
        cnt = (int)wave_reduce_u32((uint32_t)cnt, [](uint32_t x, uint32_t y) { return x + y; });
        kmin = wave_reduce_u32(kmin, [](uint32_t x, uint32_t y) { return x < y ? x : y; });
        kmax = wave_reduce_u32(kmax, [](uint32_t x, uint32_t y) { return x > y ? x : y; });
        if (lane == 0) {
            sh.w_mass[wave] = mass;
            sh.w_cnt[wave] = cnt;
            sh.w_min[wave] = kmin;
            sh.w_max[wave] = kmax;
        }
        if (tid == 0) {
            sh.cabove = 0u;
            sh.first_hole = L;
        }
        for (int i = tid; i < kBins * kSub; i += NT) {
            (&sh.hist_m[0][0][0])[i] = 0ull;
            (&sh.hist_c[0][0][0])[i] = 0u;
        }
        __syncthreads();
    }
    unsigned long long total = 0ull;
    int ncand = 0;
    uint32_t kmin = 0xffffffffu, kmax = 0u;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
        total += sh.w_mass[w];
        ncand += sh.w_cnt[w];
        kmin = min(kmin, sh.w_min[w]);
        kmax = max(kmax, sh.w_max[w]);
    }
    const int n_fixed = L - ncand;                 // entries that are never candidates
    bool evict_all_cand = false;
    unsigned long long need;                       // quota still to be met among the keys that match `prefix`
    if (budget_mode) {
        const int room = a.budget - n_fixed;
        evict_all_cand = room <= 0;
        need = room > 0 ? (unsigned long long)room : 0ull;
    } else {
        if (ncand == 0 || total == 0ull) {
            nothing_to_do();
            return;
        }
        const double target = ceil(a.beta * (double)total);
        need = target >= 1.0 ? (unsigned long long)target : 1ull;
        if (need > total) need = total;
    }

    // ---- radix descent over the bits in which the candidates' keys differ, most significant digit
    // first (scores of one head share their leading bits, so the digits that are looked at spread over
    // the histogram instead of piling up in a few bins)
    const int hb = 32 - __clz((int)(kmin ^ kmax));     // bits below the common prefix (0: all keys equal)
    const int n_pass = evict_all_cand ? 0 : (hb + kDigitBits - 1) / kDigitBits;
    uint32_t prefix = hb >= 32 ? 0u : (kmin >> hb) << hb;
    unsigned long long last_m = total;
    unsigned int last_c = (unsigned int)ncand;
    for (int pass = 0; pass < n_pass; ++pass) {
        const int top = hb - kDigitBits * pass;        // bits still undecided
        const int width = top < kDigitBits ? top : kDigitBits;
        const int shift = top - width;
        const uint32_t dmask = (1u << width) - 1u;
        const int cur = pass & 1;
        // the other histogram was last read before the barrier that ended the previous pass
        for (int i = tid; i < kBins * kSub; i += NT) {
            (&sh.hist_m[cur ^ 1][0][0])[i] = 0ull;
            (&sh.hist_c[cur ^ 1][0][0])[i] = 0u;
        }
        {
            const int sub = lane & (kSub - 1);
            auto add = [&](uint32_t k) {
                const uint32_t row = digit_row((k >> shift) & dmask);
                if (!budget_mode) atomicAdd(&sh.hist_m[cur][row][sub], key_mass(k));   // budget: mass = count
                atomicAdd(&sh.hist_c[cur][row][sub], 1u);
            };
            // keys that agree with the prefix in every bit above the current digit
            auto matches = [&](uint32_t k) { return pass == 0 || ((k ^ prefix) >> top) == 0u; };
            if constexpr (KPT > 0) {
#pragma unroll
                for (int i = 0; i < NREG; ++i)
                    if ((candm & (1u << i)) && matches(key[i])) add(key[i]);
            } else {
                for (int slot = tid; slot < L; slot += NT) {
                    if (!is_cand(slot, kind[slot])) continue;
                    const uint32_t k = score_key(score[slot]);
                    if (matches(k)) add(k);
                }
            }
        }
        __syncthreads();
        if (wave == 0) pick_digit(sh, cur, need, budget_mode);
        __syncthreads();
        prefix |= sh.digit << shift;
        need = sh.need_next;
        last_m = sh.last_m;
        last_c = sh.last_c;
    }
    uint32_t kstar = 0xffffffffu;
    unsigned long long tie_keep = 0ull;
    if (!evict_all_cand) {
        kstar = prefix;
        if (budget_mode) {
            tie_keep = need;
        } else {
            const unsigned long long u = last_m / (last_c ? last_c : 1u);   // equal keys have equal mass
            tie_keep = u ? (need + u - 1ull) / u : (unsigned long long)last_c;
        }
    }
    const int n_keep_cand = evict_all_cand ? 0 : (int)(sh.cabove + (unsigned int)tie_keep);
    const int n_new = n_fixed + n_keep_cand;
    const int n_evict = L - n_new;
    if (n_evict <= 0) {
        nothing_to_do();
        return;
    }

    // ---- one pass in slot order: number the survivors (STABLE) or holes / tail survivors (FILL).
    // A round covers CH chunks of NT slots (all of them when the keys sit in registers); lanes hold
    // neighbouring slots, so the list entries they write are neighbours too.
    int32_t *list_a = a.list_a + base;
    int32_t *list_b = a.list_b + base;
    const bool stable = a.order == LVLM_ORDER_STABLE;
    int first_hole = L;                  // lowest new slot whose entry moves (STABLE)
    int base_tie = 0, base_keep = 0, base_hole = 0, base_tail = 0;
    const bool ties_all_kept = evict_all_cand || tie_keep >= (unsigned long long)last_c;
    auto number_round = [&](int s0, auto round_tag) {
        constexpr int R0 = decltype(round_tag)::value * CH;   // first register-resident key of the round
        uint32_t tiem = 0u, keepm = 0u;              // bit c: the thread's slot of chunk c is a tie / a sure survivor
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            const int slot = s0 + NT * c + tid;
            if (slot < L) {
                uint32_t k;
                bool cand;
                if constexpr (KPT > 0) {
                    k = key[R0 + c < NREG ? R0 + c : 0];
                    cand = (candm >> (R0 + c)) & 1u;
                } else {
                    cand = is_cand(slot, kind[slot]);
                    k = score_key(score[slot]);
                }
                if (!cand || k > kstar) keepm |= 1u << c;
                else if (k == kstar) tiem |= 1u << c;
            }
        }
        uint32_t before[CH];                         // ties (low half) and sure survivors (high half) before the slot
        int tot_tie = 0, tot_keep = 0;
        uint32_t keptm = keepm | tiem;
        // FILL order with every entry of the cut's key kept (the usual case: scores are distinct) needs no
        // numbering of ties or survivors; uniform over the workgroup
        if (stable || !ties_all_kept) {
            chunk_scan2<CH, NT>(sh, tiem, keepm, before, tot_tie, tot_keep);
            keptm = 0u;
#pragma unroll
            for (int c = 0; c < CH; ++c) {
                const unsigned long long tb = (unsigned long long)(base_tie + (int)(before[c] & 0xffffu));
                if (((keepm >> c) & 1u) || (((tiem >> c) & 1u) && tb < tie_keep)) keptm |= 1u << c;
            }
            if (!stable) __syncthreads();            // the count table is reused
        }
        if (stable) {
#pragma unroll
            for (int c = 0; c < CH; ++c) {
                const int slot = s0 + NT * c + tid;
                if (slot >= L) continue;
                // survivors before a slot = sure survivors before it + kept ties before it
                const unsigned long long tb = (unsigned long long)(base_tie + (int)(before[c] & 0xffffu));
                const int p = base_keep + (int)(before[c] >> 16) + (int)min(tb, tie_keep);
                if ((keptm >> c) & 1u) list_a[p] = slot;
                else first_hole = min(first_hole, p);
            }
        } else {
            // holes (evicted, below the new length) and tail survivors (kept, at or beyond it) are
            // numbered by a second scan
            uint32_t holem = 0u, tailm = 0u;
#pragma unroll
            for (int c = 0; c < CH; ++c) {
                const int slot = s0 + NT * c + tid;
                if (slot >= L) continue;
                const bool kept = (keptm >> c) & 1u;
                if (!kept && slot < n_new) holem |= 1u << c;
                if (kept && slot >= n_new) tailm |= 1u << c;
            }
            int tot_hole, tot_tail;
            chunk_scan2<CH, NT>(sh, holem, tailm, before, tot_hole, tot_tail);
#pragma unroll
            for (int c = 0; c < CH; ++c) {
                const int slot = s0 + NT * c + tid;
                if ((holem >> c) & 1u) list_a[base_hole + (int)(before[c] & 0xffffu)] = slot;
                if ((tailm >> c) & 1u) list_b[base_tail + (int)(before[c] >> 16)] = slot;
            }
            base_hole += tot_hole;
            base_tail += tot_tail;
        }
        base_tie += tot_tie;
        base_keep += tot_keep;
        __syncthreads();                             // the count table is reused by the next round
    };
    if constexpr (KPT > 0) {
        number_round(0, std::integral_constant<int, 0>{});
        if constexpr (NROUND > 1) {
            if (NT * CH < L) number_round(NT * CH, std::integral_constant<int, 1>{});
        }
        static_assert(NROUND <= 2, "two rounds cover the register-resident keys");
    } else {
        for (int s0 = 0; s0 < L; s0 += NT * CH) number_round(s0, std::integral_constant<int, 0>{});
    }
    if (stable) {
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) first_hole = min(first_hole, __shfl_xor(first_hole, o));
        if (lane == 0) atomicMin(&sh.first_hole, first_hole);
    }
    __syncthreads();

    if (stable) {
        if (tid == 0) {
            a.meta[2 * hg] = n_new;
            a.meta[2 * hg + 1] = sh.first_hole;
            a.len[hg] = n_new;
            if (a.n_evicted) a.n_evicted[hg] = n_evict;
        }
        return;
    }

    // ---- FILL: sources (>= n_new) and destinations (< n_new) are disjoint
    const int n_moves = base_hole;           // = base_tail: as many holes as tail survivors
    if (a.fill_external) {
        if (tid == 0) {
            a.meta[2 * hg] = n_new;
            a.meta[2 * hg + 1] = n_moves;
            a.len[hg] = n_new;
            if (a.n_evicted) a.n_evicted[hg] = n_evict;
        }
        return;
    }
    const int units = a.row_bytes / 16;
    char *kc = a.k + base * a.row_bytes;
    char *vc = a.v + base * a.row_bytes;
    for (int idx = tid; idx < n_moves * units; idx += NT) {
        const int i = idx / units, u = idx - i * units;
        const long long src = (long long)list_b[i] * a.row_bytes + 16 * u;
        const long long dst = (long long)list_a[i] * a.row_bytes + 16 * u;
        *reinterpret_cast<uint4 *>(kc + dst) = *reinterpret_cast<const uint4 *>(kc + src);
        *reinterpret_cast<uint4 *>(vc + dst) = *reinterpret_cast<const uint4 *>(vc + src);
    }
    for (int i = tid; i < n_moves; i += NT) {
        const int src = list_b[i], dst = list_a[i];
        a.score[base + dst] = a.score[base + src];
        a.kind[base + dst] = a.kind[base + src];
        a.pos[base + dst] = a.pos[base + src];
    }
    if (tid == 0) {
        a.meta[2 * hg] = n_new;
        a.meta[2 * hg + 1] = n_new;
        a.len[hg] = n_new;
        if (a.n_evicted) a.n_evicted[hg] = n_evict;
    }
}

constexpr int kFillInKernel = 64;  // most FILL moves per head that the selection kernel performs itself
constexpr int kFillRows = 32;      // moves per batch of kv_fill_kernel (at most 4 row units per thread)
constexpr int kFillWgs = 16384;    // workgroups the fill launch aims for

// LVLM_ORDER_FILL with many moves per head: entry list_b[i] (at or beyond the new length) goes to hole
// list_a[i] (below it).  Sources and destinations are disjoint, so the moves are independent.
__global__ __launch_bounds__(256) void kv_fill_kernel(KvArgs a) {
    const int tid = threadIdx.x;
    const int hg = blockIdx.y;
    const int n_moves = a.meta[2 * hg + 1];
    const long long base = (long long)hg * a.Lmax;
    const int units = a.row_bytes / 16;
    char *kc = a.k + base * a.row_bytes;
    char *vc = a.v + base * a.row_bytes;
    // The head's workgroups take batches of 32 moves in turn (how many moves a head has is known only on the
    // device: a grid sized for the most there can be would start tens of thousands of workgroups that find nothing).
    for (int i0 = blockIdx.x * kFillRows; i0 < n_moves; i0 += gridDim.x * kFillRows) {
    const int cnt = min(kFillRows, n_moves - i0);
    const int32_t *holes = a.list_a + base + i0;
    const int32_t *tails = a.list_b + base + i0;
    // rows have at most 32 units (fp32, 128 channels): 32 rows are at most 4 units per thread
    const int n_units = cnt * units;
    uint4 kv0, kv1, kv2, kv3, vv0, vv1, vv2, vv3;
    long long d0, d1, d2, d3;
#define LVLM_FILL_LOAD(x)                                                            \
    {                                                                                \
        const int idx = min(256 * x + tid, n_units - 1);                             \
        const int i = idx / units, u = idx - i * units;                              \
        const long long src = (long long)tails[i] * a.row_bytes + 16 * u;            \
        d##x = (long long)holes[i] * a.row_bytes + 16 * u;                           \
        kv##x = *reinterpret_cast<const uint4 *>(kc + src);                          \
        vv##x = *reinterpret_cast<const uint4 *>(vc + src);                          \
    }
#define LVLM_FILL_STORE(x)                                    \
    if (256 * x + tid < n_units) {                            \
        *reinterpret_cast<uint4 *>(kc + d##x) = kv##x;        \
        *reinterpret_cast<uint4 *>(vc + d##x) = vv##x;        \
    }
    LVLM_FILL_LOAD(0) LVLM_FILL_LOAD(1) LVLM_FILL_LOAD(2) LVLM_FILL_LOAD(3)
    LVLM_FILL_STORE(0) LVLM_FILL_STORE(1) LVLM_FILL_STORE(2) LVLM_FILL_STORE(3)
#undef LVLM_FILL_LOAD
#undef LVLM_FILL_STORE
    if (tid < cnt) {
        const int src = tails[tid], dst = holes[tid];
        a.score[base + dst] = a.score[base + src];
        a.kind[base + dst] = a.kind[base + src];
        a.pos[base + dst] = a.pos[base + src];
    }
    }
}

constexpr int kMoveUpt = 8;       // 16-byte units per thread per step (two such sets are in flight)

// NT threads move one SLICE-byte column slice of NT / (SLICE / 16) * kMoveUpt rows per step.  A step's
// sources all lie at or above its first destination, and above every destination of earlier steps, so
// the only ordering that matters is inside a step: all of its loads go before any of its stores (the
// barrier; a compute unit performs the vector memory operations of its waves in issue order).  The
// loads of step s + 1 are issued before the stores of step s, so that reads and writes overlap.  With few heads the launch uses 1024-thread workgroups and narrower slices, so that
// the few workgroups there are keep enough bytes in flight.
template <int NT, int SLICE>
__global__ __launch_bounds__(NT) void kv_move_kernel(KvArgs a) {
    constexpr int TPR = SLICE / 16;              // threads per row slice
    constexpr int RPS = NT / TPR;                // rows per load instruction of the workgroup
    const int tid = threadIdx.x;
    const int hg = blockIdx.y;
    const int n_new = a.meta[2 * hg], first = a.meta[2 * hg + 1];
    if (first >= n_new) return;
    const long long base = (long long)hg * a.Lmax;
    const int32_t *src_of = a.list_a + base;
    const int slices = a.row_bytes / SLICE;
    const int sl = blockIdx.x;
    if (sl < 2 * slices) {
        char *cache = (sl < slices ? a.k : a.v) + base * a.row_bytes + (sl % slices) * SLICE + 16 * (tid % TPR);
        constexpr int ROWS = RPS * kMoveUpt;
        static_assert(kMoveUpt == 8, "the register sets below are written out for 8 units");
        const int row = tid / TPR;
        // Two register sets with named members: arrays carried around the loop would be placed in
        // scratch memory.
#define LVLM_MV_EACH(M) M(0) M(1) M(2) M(3) M(4) M(5) M(6) M(7)
#define LVLM_MV_DECL(x) uint4 c##x, n##x;
#define LVLM_MV_LOAD_C(x) \
    c##x = *reinterpret_cast<const uint4 *>(cache + (long long)src_of[min(first + RPS * x + row, n_new - 1)] * a.row_bytes);
#define LVLM_MV_LOAD_N(x)                                                                                        \
    n##x = c##x;                                                                                                 \
    if (more)                                                                                                    \
        n##x = *reinterpret_cast<const uint4 *>(cache +                                                          \
                                                (long long)src_of[min(p0 + ROWS + RPS * x + row, n_new - 1)] * a.row_bytes);
#define LVLM_MV_STORE(x)                                                                      \
    if (p0 + RPS * x + row < n_new)                                                           \
        *reinterpret_cast<uint4 *>(cache + (long long)(p0 + RPS * x + row) * a.row_bytes) = c##x;
#define LVLM_MV_NEXT(x) c##x = n##x;
        LVLM_MV_EACH(LVLM_MV_DECL)
        LVLM_MV_EACH(LVLM_MV_LOAD_C)
        for (int p0 = first; p0 < n_new; p0 += ROWS) {
            __syncthreads();                     // every load of this step was issued before any of its stores
            const bool more = p0 + ROWS < n_new;
            LVLM_MV_EACH(LVLM_MV_LOAD_N)
            LVLM_MV_EACH(LVLM_MV_STORE)
            LVLM_MV_EACH(LVLM_MV_NEXT)
        }
#undef LVLM_MV_EACH
#undef LVLM_MV_DECL
#undef LVLM_MV_LOAD_C
#undef LVLM_MV_LOAD_N
#undef LVLM_MV_STORE
#undef LVLM_MV_NEXT
    } else {
        constexpr int ROWS = NT * kMoveUpt;
        for (int p0 = first; p0 < n_new; p0 += ROWS) {
            float sc[kMoveUpt];
            uint8_t kd[kMoveUpt];
            int32_t ps[kMoveUpt];
#pragma unroll
            for (int x = 0; x < kMoveUpt; ++x) {
                const int s = src_of[min(p0 + NT * x + tid, n_new - 1)];
                sc[x] = a.score[base + s];
                kd[x] = a.kind[base + s];
                ps[x] = a.pos[base + s];
            }
            __syncthreads();
#pragma unroll
            for (int x = 0; x < kMoveUpt; ++x) {
                const int p = p0 + NT * x + tid;
                if (p < n_new) {
                    a.score[base + p] = sc[x];
                    a.kind[base + p] = kd[x];
                    a.pos[base + p] = ps[x];
                }
            }
        }
    }
}

}  // namespace

KvWs kv_ws(const lvlm_kv_desc &d) {
    KvWs w{};
    const size_t heads = (size_t)d.B * d.Hkv;
    w.src = 0;
    // two slot lists per head, then two ints of bookkeeping per head
    w.total = align_up(2 * heads * d.Lmax * sizeof(int32_t), 256) + align_up(heads * 2 * sizeof(int32_t), 256);
    return w;
}

hipError_t launch_kv_compress(const Prof &prof, const lvlm_kv_desc &d, const KvWs &w, char *ws, void *k_cache,
                              void *v_cache, float *score, uint8_t *kind, int32_t *orig_pos, int32_t *len,
                              int32_t *n_evicted) {
    const size_t heads = (size_t)d.B * d.Hkv;
    KvArgs a{};
    a.k = static_cast<char *>(k_cache);
    a.v = static_cast<char *>(v_cache);
    a.score = score; a.kind = kind; a.pos = orig_pos; a.len = len; a.n_evicted = n_evicted;
    a.list_a = reinterpret_cast<int32_t *>(ws + w.src);
    a.list_b = a.list_a + heads * d.Lmax;
    a.meta = reinterpret_cast<int32_t *>(ws + align_up(2 * heads * d.Lmax * sizeof(int32_t), 256));
    a.Hkv = d.Hkv; a.Lmax = d.Lmax;
    a.bound = d.len_bound > 0 ? d.len_bound : d.Lmax;
    a.row_bytes = d.hd * (d.dtype == LVLM_BF16 ? 2 : 4);
    a.mode = d.mode; a.order = d.order; a.budget = d.budget; a.n_recent = d.n_recent; a.beta = d.beta;
    hipStream_t stream = prof.stream;
    const int bound = d.len_bound > 0 ? d.len_bound : d.Lmax;
    // FILL moves at most min(new length, evicted entries) entries per head
    const int max_moves = d.mode == LVLM_KV_BUDGET ? (bound - d.budget < bound / 2 ? bound - d.budget : bound / 2) : bound / 2;
    a.fill_external = d.order == LVLM_ORDER_FILL && max_moves > kFillInKernel;
    prof.begin("kv_select");
    // Much of the selection is one wave's chain of latencies, so with more heads than the chip holds workgroups of
    // 1024 threads, short heads go to workgroups of 256 threads: more heads are in flight at once.
    if (bound <= 2048 && heads > 512) LVLM_LAUNCH(prof, (kv_select_kernel<8, 256>), dim3((unsigned)heads), dim3(256), 0, stream, a);
    else if (bound <= 2048) LVLM_LAUNCH(prof, (kv_select_kernel<2, 1024>), dim3((unsigned)heads), dim3(1024), 0, stream, a);
    else if (bound <= 4096) LVLM_LAUNCH(prof, (kv_select_kernel<4, 1024>), dim3((unsigned)heads), dim3(1024), 0, stream, a);
    else if (bound <= 8192) LVLM_LAUNCH(prof, (kv_select_kernel<8, 1024>), dim3((unsigned)heads), dim3(1024), 0, stream, a);
    else if (bound <= 17408) LVLM_LAUNCH(prof, (kv_select_kernel<17, 1024>), dim3((unsigned)heads), dim3(1024), 0, stream, a);
    else LVLM_LAUNCH(prof, (kv_select_kernel<0, 1024>), dim3((unsigned)heads), dim3(1024), 0, stream, a);
    prof.end();
    if (d.order == LVLM_ORDER_STABLE) {
        prof.begin("kv_move");
        const int s64 = a.row_bytes / 64;
        if (heads * (2 * s64 + 1) >= 1024)
            LVLM_LAUNCH(prof, (kv_move_kernel<256, 64>), dim3(2 * s64 + 1, (unsigned)heads), dim3(256), 0, stream, a);
        else if (heads * (2 * s64 + 1) >= 256)
            LVLM_LAUNCH(prof, (kv_move_kernel<1024, 64>), dim3(2 * s64 + 1, (unsigned)heads), dim3(1024), 0, stream, a);
        else
            LVLM_LAUNCH(prof, (kv_move_kernel<1024, 32>), dim3(4 * s64 + 1, (unsigned)heads), dim3(1024), 0, stream, a);
        prof.end();
    } else if (a.fill_external) {
        prof.begin("kv_fill");
        // about 16384 workgroups in all, at most one per batch of moves the longest head can have
        const long long most = (max_moves + kFillRows - 1) / kFillRows;
        long long per_head = (kFillWgs + (long long)heads - 1) / (long long)heads;
        per_head = per_head < 1 ? 1 : (per_head > most ? most : per_head);
        LVLM_LAUNCH(prof, kv_fill_kernel, dim3((unsigned)per_head, (unsigned)heads), dim3(256), 0, stream, a);
        prof.end();
    }
    return hipGetLastError();
}

}  // namespace lvlm
