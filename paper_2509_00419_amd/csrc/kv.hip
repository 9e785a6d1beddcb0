// Step 5 -- KV-cache compression, independently per (batch, KV head) (Sec. 3.2.2).
//
// Neither rule needs a sort.  Both ask for "the best entries until a quota is
// met", where the quota is a number of entries (fixed budget) or an amount of
// score mass (threshold beta).  A most-significant-digit radix descent over the
// order-preserving 32-bit image of the score finds, in four histogram passes,
// the key K* at which the quota is met: entries above K* stay, entries below go,
// and among the entries equal to K* the lowest slots stay.  Score mass is summed
// as exact integers, so the result does not depend on summation order.  (Four
// 8-bit digits: four histogram passes over the scores; the first also gives the totals.)
//
//   kv_select_kernel  one workgroup per head: totals, radix descent, then one
//                     pass in slot order that numbers survivors / holes.  With
//                     LVLM_ORDER_FILL it also performs the (few, disjoint)
//                     moves itself.
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
    int Hkv, Lmax, row_bytes, mode, order, budget, n_recent;
    double beta;
};

constexpr int kScanChunks = 4;    // 1024-slot chunks numbered per barrier round in the slot-order pass
constexpr int kBins = 256;        // radix: four 8-bit digits of the 32-bit key

struct ScanState {
    int wave_cnt[3][kScanChunks][16];   // per-wave counts, turned into exclusive prefixes in place
    int tot[3][kScanChunks];
    int base[3];
};

// Exclusive prefix counts, in slot order, of three flags over kScanChunks consecutive 1024-slot chunks
// (thread t holds slot c * 1024 + t of chunk c).  `base` carries the totals to the next round.
__device__ __forceinline__ void block_scan3(ScanState &s, const bool (&f0)[kScanChunks], const bool (&f1)[kScanChunks],
                                            const bool (&f2)[kScanChunks], int (&p0)[kScanChunks],
                                            int (&p1)[kScanChunks], int (&p2)[kScanChunks]) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const unsigned long long below = (1ull << lane) - 1ull;
#pragma unroll
    for (int c = 0; c < kScanChunks; ++c) {
        const unsigned long long b0 = __ballot(f0[c]), b1 = __ballot(f1[c]), b2 = __ballot(f2[c]);
        p0[c] = __popcll(b0 & below);
        p1[c] = __popcll(b1 & below);
        p2[c] = __popcll(b2 & below);
        if (lane == 0) {
            s.wave_cnt[0][c][wave] = __popcll(b0);
            s.wave_cnt[1][c][wave] = __popcll(b1);
            s.wave_cnt[2][c][wave] = __popcll(b2);
        }
    }
    __syncthreads();
    if (tid < 3 * kScanChunks) {
        const int k = tid / kScanChunks, c = tid % kScanChunks;
        int run = 0;
        for (int w = 0; w < 16; ++w) {
            const int v = s.wave_cnt[k][c][w];
            s.wave_cnt[k][c][w] = run;
            run += v;
        }
        s.tot[k][c] = run;
    }
    __syncthreads();
    int run0 = s.base[0], run1 = s.base[1], run2 = s.base[2];
#pragma unroll
    for (int c = 0; c < kScanChunks; ++c) {
        p0[c] += run0 + s.wave_cnt[0][c][wave];
        p1[c] += run1 + s.wave_cnt[1][c][wave];
        p2[c] += run2 + s.wave_cnt[2][c][wave];
        run0 += s.tot[0][c];
        run1 += s.tot[1][c];
        run2 += s.tot[2][c];
    }
    __syncthreads();
    if (tid == 0) {
        s.base[0] = run0;
        s.base[1] = run1;
        s.base[2] = run2;
    }
    __syncthreads();
}

// Exact fixed-point mass of a candidate, from its order-preserving key alone: keys with the top bit set
// are the non-negative scores (bit pattern = key without that bit); negative scores and NaN weigh 0.
__device__ __forceinline__ unsigned long long key_mass(uint32_t key) {
    return (key & 0x80000000u) ? score_fixed(__uint_as_float(key & 0x7fffffffu)) : 0ull;
}

struct SelectShared {
    unsigned long long hist_m[kBins];
    unsigned int hist_c[kBins];
    unsigned long long total, need, need_next;
    unsigned int ncand, cabove, digit;
    int first_hole;
    ScanState scan;
    unsigned long long w_best[16];   // per-wave partial results of the block reductions
    unsigned long long w_mass[16];
    uint32_t w_min[16], w_max[16];
    int w_cnt[16];
};

// Wave 0, after a histogram pass: suffix sums over the digits give the mass (and count) above each
// digit; the digit in which the quota `need` (> 0, at most the mass in the histogram) is met becomes the
// next digit of the key.
__device__ __forceinline__ void pick_digit(SelectShared &sh, unsigned long long need) {
    const int lane = threadIdx.x & 63;
    constexpr int PER = kBins / 64;     // lane owns 4 consecutive digits
    unsigned long long loc_m = 0ull;
    unsigned int loc_c = 0u;
    unsigned long long hm[PER];
    unsigned int hc[PER];
#pragma unroll
    for (int i = 0; i < PER; ++i) {
        hm[i] = sh.hist_m[PER * lane + i];
        hc[i] = sh.hist_c[PER * lane + i];
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
        }
        above_m += hm[i];
        above_c += hc[i];
    }
}

// One round of the slot-order pass over kScanChunks chunks of 1024 slots: numbers the survivors (STABLE)
// or the holes and the tail survivors (FILL) and writes the slot lists.
__device__ __forceinline__ void number_round(SelectShared &sh, bool stable, const bool (&tie)[kScanChunks],
                                             const bool (&keep)[kScanChunks], const bool (&inside)[kScanChunks],
                                             const int (&slot)[kScanChunks], unsigned long long tie_keep, int n_new,
                                             int32_t *list_a, int32_t *list_b, int &first_hole) {
    bool none[kScanChunks];
#pragma unroll
    for (int c = 0; c < kScanChunks; ++c) none[c] = false;
    int tie_before[kScanChunks], p1[kScanChunks], p2[kScanChunks];
    if (stable) {
        // survivors before a slot = sure survivors before it + kept ties before it
        block_scan3(sh.scan, tie, keep, none, tie_before, p1, p2);
#pragma unroll
        for (int c = 0; c < kScanChunks; ++c) {
            if (!inside[c]) continue;
            const bool kept = keep[c] || (tie[c] && (unsigned long long)tie_before[c] < tie_keep);
            const int p = p1[c] + (int)min((unsigned long long)tie_before[c], tie_keep);
            if (kept) list_a[p] = slot[c];
            else first_hole = min(first_hole, p);      // folded over the workgroup once, after the last round
        }
    } else {
        block_scan3(sh.scan, tie, none, none, tie_before, p1, p2);
        bool hole[kScanChunks], tail[kScanChunks];
#pragma unroll
        for (int c = 0; c < kScanChunks; ++c) {
            const bool kept = keep[c] || (tie[c] && (unsigned long long)tie_before[c] < tie_keep);
            hole[c] = inside[c] && !kept && slot[c] < n_new;
            tail[c] = inside[c] && kept && slot[c] >= n_new;
        }
        int dummy[kScanChunks], hi[kScanChunks], ti[kScanChunks];
        // a second scan numbers holes and tail survivors (counter 0 keeps counting ties)
        block_scan3(sh.scan, none, hole, tail, dummy, hi, ti);
#pragma unroll
        for (int c = 0; c < kScanChunks; ++c) {
            if (hole[c]) list_a[hi[c]] = slot[c];
            if (tail[c]) list_b[ti[c]] = slot[c];
        }
    }
}

// KPT > 0: every thread keeps the keys of its KPT slots (slot = 1024 i + thread) in registers, so the
// scores are read once, with all loads in flight together; heads longer than 1024 KPT are not accepted
// by the launch.  KPT == 0: any length, scores re-read from memory in every pass.
template <int KPT>
__global__ __launch_bounds__(1024) void kv_select_kernel(KvArgs a) {
    __shared__ SelectShared sh;
    constexpr int NREG = KPT > 0 ? KPT : 1;
    constexpr int NROUND = (NREG + kScanChunks - 1) / kScanChunks;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int hg = blockIdx.x;
    const long long base = (long long)hg * a.Lmax;
    const float *score = a.score + base;
    const uint8_t *kind = a.kind + base;
    int L = min(a.len[hg], a.Lmax);
    if (KPT > 0) L = min(L, 1024 * KPT);
    const bool budget_mode = a.mode == LVLM_KV_BUDGET;

    auto nothing_to_do = [&]() {
        if (tid == 0) {
            if (a.n_evicted) a.n_evicted[hg] = 0;
            a.meta[2 * hg] = L;
            a.meta[2 * hg + 1] = L;
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

    // register-resident keys; bit i of `candm` marks slot 1024 i + tid as a candidate
    uint32_t key[NREG];
    uint32_t candm = 0u;
    if constexpr (KPT > 0) {
        float sc[NREG];
        uint8_t kd[NREG];
#pragma unroll
        for (int i = 0; i < NREG; ++i) {
            const int sl = min(1024 * i + tid, L - 1);     // clamped: every load is issued, none depends on another
            sc[i] = score[sl];
            kd[i] = kind[sl];
        }
#pragma unroll
        for (int i = 0; i < NREG; ++i) {
            const int slot = 1024 * i + tid;
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
                        ((unsigned long long)key[i] << 32) | (unsigned long long)(0xffffffffu - (uint32_t)(1024 * i + tid));
                    best = c < best ? c : best;
                }
            }
        } else {
            for (int slot = tid; slot < L; slot += 1024) {
                if (is_cand(slot, kind[slot])) {
                    ++cnt;
                    const unsigned long long c = ((unsigned long long)score_key(score[slot]) << 32) |
                                                 (unsigned long long)(0xffffffffu - (uint32_t)slot);
                    best = c < best ? c : best;
                }
            }
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            const unsigned long long ob = __shfl_xor(best, o);
            best = ob < best ? ob : best;
            cnt += __shfl_xor(cnt, o);
        }
        if (lane == 0) {
            sh.w_best[wave] = best;
            sh.w_cnt[wave] = cnt;
        }
        __syncthreads();
        best = sh.w_best[0];
        cnt = sh.w_cnt[0];
#pragma unroll
        for (int w = 1; w < 16; ++w) {
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
                a.meta[2 * hg + 1] = last;
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
            for (int slot = tid; slot < L; slot += 1024)
                if (is_cand(slot, kind[slot])) see(score_key(score[slot]));
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            mass += __shfl_xor(mass, o);
            cnt += __shfl_xor(cnt, o);
            kmin = min(kmin, (uint32_t)__shfl_xor((int)kmin, o));
            kmax = max(kmax, (uint32_t)__shfl_xor((int)kmax, o));
        }
        if (lane == 0) {
            sh.w_mass[wave] = mass;
            sh.w_cnt[wave] = cnt;
            sh.w_min[wave] = kmin;
            sh.w_max[wave] = kmax;
        }
        if (tid == 0) {
            sh.cabove = 0u;
            sh.first_hole = L;
            sh.scan.base[0] = sh.scan.base[1] = sh.scan.base[2] = 0;
        }
        __syncthreads();
    }
    unsigned long long total = 0ull;
    int ncand = 0;
    uint32_t kmin = 0xffffffffu, kmax = 0u;
#pragma unroll
    for (int w = 0; w < 16; ++w) {
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
    const int n_pass = evict_all_cand ? 0 : (hb + 7) / 8;
    uint32_t prefix = hb >= 32 ? 0u : (kmin >> hb) << hb;
    unsigned long long last_m = total;
    unsigned int last_c = (unsigned int)ncand;
    for (int pass = 0; pass < n_pass; ++pass) {
        const int top = hb - 8 * pass;                 // bits still undecided
        const int width = top < 8 ? top : 8;
        const int shift = top - width;
        const uint32_t dmask = (1u << width) - 1u;
        for (int i = tid; i < kBins; i += 1024) {
            sh.hist_m[i] = 0ull;
            sh.hist_c[i] = 0u;
        }
        __syncthreads();
        {
            // a thread first adds up runs of equal digits in registers and only then touches the shared
            // histogram (fewer colliding LDS atomics)
            uint32_t run_d = 0xffffffffu;
            unsigned long long run_m = 0ull;
            unsigned int run_c = 0u;
            auto add = [&](uint32_t k) {
                const uint32_t dgt = (k >> shift) & dmask;
                if (dgt != run_d) {
                    if (run_c) {
                        atomicAdd(&sh.hist_m[run_d], run_m);
                        atomicAdd(&sh.hist_c[run_d], run_c);
                    }
                    run_d = dgt;
                    run_m = 0ull;
                    run_c = 0u;
                }
                run_m += budget_mode ? 1ull : key_mass(k);
                ++run_c;
            };
            // keys that agree with the prefix in every bit above the current digit
            auto matches = [&](uint32_t k) { return pass == 0 || ((k ^ prefix) >> top) == 0u; };
            if constexpr (KPT > 0) {
#pragma unroll
                for (int i = 0; i < NREG; ++i)
                    if ((candm & (1u << i)) && matches(key[i])) add(key[i]);
            } else {
                for (int slot = tid; slot < L; slot += 1024) {
                    if (!is_cand(slot, kind[slot])) continue;
                    const uint32_t k = score_key(score[slot]);
                    if (matches(k)) add(k);
                }
            }
            if (run_c) {
                atomicAdd(&sh.hist_m[run_d], run_m);
                atomicAdd(&sh.hist_c[run_d], run_c);
            }
        }
        __syncthreads();
        if (wave == 0) pick_digit(sh, need);
        __syncthreads();
        prefix |= sh.digit << shift;
        need = sh.need_next;
        if (pass == n_pass - 1) {
            last_m = sh.hist_m[sh.digit];
            last_c = sh.hist_c[sh.digit];
        }
        __syncthreads();
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

    // ---- one pass in slot order: number the survivors (STABLE) or holes / tail survivors (FILL)
    int32_t *list_a = a.list_a + base;
    int32_t *list_b = a.list_b + base;
    const bool stable = a.order == LVLM_ORDER_STABLE;
    int first_hole = L;                  // lowest new slot whose entry moves (STABLE)
    if constexpr (KPT > 0) {
#pragma unroll
        for (int r = 0; r < NROUND; ++r) {
            if (r * kScanChunks * 1024 >= L) break;
            bool tie[kScanChunks], keep[kScanChunks], inside[kScanChunks];
            int slot[kScanChunks];
#pragma unroll
            for (int c = 0; c < kScanChunks; ++c) {
                const int i = r * kScanChunks + c;
                slot[c] = 1024 * i + tid;
                inside[c] = slot[c] < L;
                tie[c] = keep[c] = false;
                if (i < NREG && inside[c]) {
                    const uint32_t k = key[i < NREG ? i : 0];
                    if (!(candm & (1u << i))) {
                        keep[c] = true;
                    } else {
                        tie[c] = k == kstar;
                        keep[c] = k > kstar;
                    }
                }
            }
            number_round(sh, stable, tie, keep, inside, slot, tie_keep, n_new, list_a, list_b, first_hole);
        }
    } else {
        for (int s0 = 0; s0 < L; s0 += kScanChunks * 1024) {
            bool tie[kScanChunks], keep[kScanChunks], inside[kScanChunks];
            int slot[kScanChunks];
#pragma unroll
            for (int c = 0; c < kScanChunks; ++c) {
                slot[c] = s0 + c * 1024 + tid;
                inside[c] = slot[c] < L;
                tie[c] = keep[c] = false;
                if (inside[c]) {
                    if (!is_cand(slot[c], kind[slot[c]])) {
                        keep[c] = true;
                    } else {
                        const uint32_t k = score_key(score[slot[c]]);
                        tie[c] = k == kstar;
                        keep[c] = k > kstar;
                    }
                }
            }
            number_round(sh, stable, tie, keep, inside, slot, tie_keep, n_new, list_a, list_b, first_hole);
        }
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
    const int n_moves = sh.scan.base[1];
    const int units = a.row_bytes / 16;
    char *kc = a.k + base * a.row_bytes;
    char *vc = a.v + base * a.row_bytes;
    for (int idx = tid; idx < n_moves * units; idx += 1024) {
        const int i = idx / units, u = idx - i * units;
        const long long src = (long long)list_b[i] * a.row_bytes + 16 * u;
        const long long dst = (long long)list_a[i] * a.row_bytes + 16 * u;
        *reinterpret_cast<uint4 *>(kc + dst) = *reinterpret_cast<const uint4 *>(kc + src);
        *reinterpret_cast<uint4 *>(vc + dst) = *reinterpret_cast<const uint4 *>(vc + src);
    }
    for (int i = tid; i < n_moves; i += 1024) {
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
    a.row_bytes = d.hd * (d.dtype == LVLM_BF16 ? 2 : 4);
    a.mode = d.mode; a.order = d.order; a.budget = d.budget; a.n_recent = d.n_recent; a.beta = d.beta;
    hipStream_t stream = prof.stream;
    prof.begin("kv_select");
    const int bound = d.len_bound > 0 ? d.len_bound : d.Lmax;
    if (bound <= 2048) hipLaunchKernelGGL(kv_select_kernel<2>, dim3((unsigned)heads), dim3(1024), 0, stream, a);
    else if (bound <= 4096) hipLaunchKernelGGL(kv_select_kernel<4>, dim3((unsigned)heads), dim3(1024), 0, stream, a);
    else if (bound <= 8192) hipLaunchKernelGGL(kv_select_kernel<8>, dim3((unsigned)heads), dim3(1024), 0, stream, a);
    else if (bound <= 17408) hipLaunchKernelGGL(kv_select_kernel<17>, dim3((unsigned)heads), dim3(1024), 0, stream, a);
    else hipLaunchKernelGGL(kv_select_kernel<0>, dim3((unsigned)heads), dim3(1024), 0, stream, a);
    prof.end();
    if (d.order == LVLM_ORDER_STABLE) {
        prof.begin("kv_move");
        const int s64 = a.row_bytes / 64;
        if (heads * (2 * s64 + 1) >= 1024)
            hipLaunchKernelGGL((kv_move_kernel<256, 64>), dim3(2 * s64 + 1, (unsigned)heads), dim3(256), 0, stream, a);
        else if (heads * (2 * s64 + 1) >= 256)
            hipLaunchKernelGGL((kv_move_kernel<1024, 64>), dim3(2 * s64 + 1, (unsigned)heads), dim3(1024), 0, stream, a);
        else
            hipLaunchKernelGGL((kv_move_kernel<1024, 32>), dim3(4 * s64 + 1, (unsigned)heads), dim3(1024), 0, stream, a);
        prof.end();
    }
    return hipGetLastError();
}

}  // namespace lvlm
