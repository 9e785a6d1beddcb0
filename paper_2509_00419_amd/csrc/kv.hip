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

__global__ __launch_bounds__(1024) void kv_select_kernel(KvArgs a) {
    __shared__ unsigned long long hist_m[kBins];
    __shared__ unsigned int hist_c[kBins];
    __shared__ unsigned long long s_total, s_need, s_need_next;
    __shared__ unsigned int s_ncand, s_cabove, s_digit;
    __shared__ int s_first_hole;
    __shared__ ScanState scan;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int hg = blockIdx.x;
    const long long base = (long long)hg * a.Lmax;
    const float *score = a.score + base;
    const uint8_t *kind = a.kind + base;
    const int L = min(a.len[hg], a.Lmax);
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

    // ---- steady-state decode: the head is exactly one entry over budget and holes are filled from
    // the tail.  One pass finds the candidate that is last in importance order (lowest key, highest
    // slot among equals); the entry in the last slot takes its place.
    if (budget_mode && a.order == LVLM_ORDER_FILL && L - a.budget == 1) {
        __shared__ unsigned long long w_best[16];
        __shared__ int w_cnt[16];
        unsigned long long best = ~0ull;
        int cnt = 0;
        for (int slot = tid; slot < L; slot += 1024) {
            if (is_cand(slot, kind[slot])) {
                ++cnt;
                const unsigned long long c =
                    ((unsigned long long)score_key(score[slot]) << 32) | (unsigned long long)(0xffffffffu - (uint32_t)slot);
                best = c < best ? c : best;
            }
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            const unsigned long long ob = __shfl_xor(best, o);
            best = ob < best ? ob : best;
            cnt += __shfl_xor(cnt, o);
        }
        if (lane == 0) {
            w_best[wave] = best;
            w_cnt[wave] = cnt;
        }
        __syncthreads();
        best = w_best[0];
        cnt = w_cnt[0];
#pragma unroll
        for (int w = 1; w < 16; ++w) {
            best = w_best[w] < best ? w_best[w] : best;
            cnt += w_cnt[w];
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

    // ---- radix descent, most significant digit first.  The first histogram also yields the totals.
    if (tid == 0) {
        s_cabove = 0u;
        s_first_hole = L;
        scan.base[0] = scan.base[1] = scan.base[2] = 0;
    }
    unsigned long long need = 0ull;      // quota still to be met inside the current bin
    int n_fixed = 0;                     // entries that are never candidates
    bool evict_all_cand = false;
    uint32_t prefix = 0u;
    unsigned long long last_m = 0ull;
    unsigned int last_c = 1u;
    for (int pass = 0; pass < 4; ++pass) {
        const int shift = 24 - 8 * pass;
        for (int i = tid; i < kBins; i += 1024) {
            hist_m[i] = 0ull;
            hist_c[i] = 0u;
        }
        __syncthreads();
        {
            // Scores cluster in few digits, so a thread first adds up runs of equal digits in registers
            // and only then touches the shared histogram (far fewer colliding LDS atomics).
            uint32_t run_d = 0xffffffffu;
            unsigned long long run_m = 0ull;
            unsigned int run_c = 0u;
            for (int slot = tid; slot < L; slot += 1024) {
                if (!is_cand(slot, kind[slot])) continue;
                const float sc = score[slot];
                const uint32_t key = score_key(sc);
                if (pass > 0 && (key >> (shift + 8)) != (prefix >> (shift + 8))) continue;
                const uint32_t dgt = (key >> shift) & 255u;
                if (dgt != run_d) {
                    if (run_c) {
                        atomicAdd(&hist_m[run_d], run_m);
                        atomicAdd(&hist_c[run_d], run_c);
                    }
                    run_d = dgt;
                    run_m = 0ull;
                    run_c = 0u;
                }
                run_m += budget_mode ? 1ull : score_fixed(sc);
                ++run_c;
            }
            if (run_c) {
                atomicAdd(&hist_m[run_d], run_m);
                atomicAdd(&hist_c[run_d], run_c);
            }
        }
        __syncthreads();
        if (wave == 0) {
            // lane owns 4 consecutive digits; suffix sums give the mass above each digit
            constexpr int PER = kBins / 64;
            unsigned long long loc_m = 0ull;
            unsigned int loc_c = 0u;
            for (int i = 0; i < PER; ++i) {
                loc_m += hist_m[PER * lane + i];
                loc_c += hist_c[PER * lane + i];
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
            if (pass == 0) {
                // totals over all candidates (lane 0 holds the full suffix sum) fix the quota
                const unsigned long long total = __shfl(inc_m, 0);
                const unsigned int ncand = __shfl(inc_c, 0);
                if (lane == 0) {
                    s_total = total;
                    s_ncand = ncand;
                    unsigned long long nd;
                    if (budget_mode) {
                        const int room = a.budget - (L - (int)ncand);
                        nd = room > 0 ? (unsigned long long)room : 0ull;
                    } else {
                        const double target = ceil(a.beta * (double)total);
                        nd = target >= 1.0 ? (unsigned long long)target : 1ull;
                        if (nd > total) nd = total;
                    }
                    s_need = nd;
                }
            }
            // every lane needs the quota of this pass
            unsigned long long nd = pass == 0 ? 0ull : need;
            if (pass == 0) {
                nd = __shfl(lane == 0 ? s_need : 0ull, 0);
            }
            unsigned long long above_m = inc_m - loc_m;
            unsigned int above_c = inc_c - loc_c;
            if (nd > 0ull) {
                for (int i = PER - 1; i >= 0; --i) {
                    const unsigned long long hm = hist_m[PER * lane + i];
                    if (above_m < nd && nd <= above_m + hm) {
                        s_digit = (unsigned int)(PER * lane + i);
                        s_need_next = nd - above_m;
                        s_cabove += above_c;     // exactly one lane and one digit take this branch
                    }
                    above_m += hm;
                    above_c += hist_c[PER * lane + i];
                }
            }
        }
        __syncthreads();
        if (pass == 0) {
            const unsigned int ncand = s_ncand;
            n_fixed = L - (int)ncand;
            if (budget_mode) {
                evict_all_cand = a.budget - n_fixed <= 0;
            } else if (ncand == 0u || s_total == 0ull) {
                nothing_to_do();
                return;
            }
            if (evict_all_cand) break;
        }
        prefix |= s_digit << shift;
        need = s_need_next;
        if (pass == 3) {
            last_m = hist_m[s_digit];
            last_c = hist_c[s_digit];
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
    const int n_keep_cand = evict_all_cand ? 0 : (int)(s_cabove + (unsigned int)tie_keep);
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
    for (int s0 = 0; s0 < L; s0 += kScanChunks * 1024) {
        bool tie[kScanChunks], keep[kScanChunks], inside[kScanChunks], none[kScanChunks];
        int slot[kScanChunks];
#pragma unroll
        for (int c = 0; c < kScanChunks; ++c) {
            slot[c] = s0 + c * 1024 + tid;
            inside[c] = slot[c] < L;
            tie[c] = keep[c] = none[c] = false;
            if (inside[c]) {
                if (!is_cand(slot[c], kind[slot[c]])) {
                    keep[c] = true;
                } else {
                    const uint32_t key = score_key(score[slot[c]]);
                    tie[c] = key == kstar;
                    keep[c] = key > kstar;
                }
            }
        }
        int tie_before[kScanChunks], p1[kScanChunks], p2[kScanChunks];
        if (stable) {
            // survivors before a slot = sure survivors before it + kept ties before it
            block_scan3(scan, tie, keep, none, tie_before, p1, p2);
#pragma unroll
            for (int c = 0; c < kScanChunks; ++c) {
                if (!inside[c]) continue;
                const bool kept = keep[c] || (tie[c] && (unsigned long long)tie_before[c] < tie_keep);
                const int p = p1[c] + (int)min((unsigned long long)tie_before[c], tie_keep);
                if (kept) list_a[p] = slot[c];
                else atomicMin(&s_first_hole, p);
            }
        } else {
            block_scan3(scan, tie, none, none, tie_before, p1, p2);
            bool hole[kScanChunks], tail[kScanChunks];
#pragma unroll
            for (int c = 0; c < kScanChunks; ++c) {
                const bool kept = keep[c] || (tie[c] && (unsigned long long)tie_before[c] < tie_keep);
                hole[c] = inside[c] && !kept && slot[c] < n_new;
                tail[c] = inside[c] && kept && slot[c] >= n_new;
            }
            int dummy[kScanChunks], hi[kScanChunks], ti[kScanChunks];
            // a second scan numbers holes and tail survivors (counter 0 keeps counting ties)
            block_scan3(scan, none, hole, tail, dummy, hi, ti);
#pragma unroll
            for (int c = 0; c < kScanChunks; ++c) {
                if (hole[c]) list_a[hi[c]] = slot[c];
                if (tail[c]) list_b[ti[c]] = slot[c];
            }
        }
    }
    __syncthreads();

    if (stable) {
        if (tid == 0) {
            a.meta[2 * hg] = n_new;
            a.meta[2 * hg + 1] = s_first_hole;
            a.len[hg] = n_new;
            if (a.n_evicted) a.n_evicted[hg] = n_evict;
        }
        return;
    }

    // ---- FILL: sources (>= n_new) and destinations (< n_new) are disjoint
    const int n_moves = scan.base[1];
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

constexpr int kSliceBytes = 64;   // column slice of a K or V row handled by one workgroup
constexpr int kMoveUpt = 16;      // units per thread per step (1024 rows of a 64-byte slice)

__global__ __launch_bounds__(256) void kv_move_kernel(KvArgs a) {
    const int tid = threadIdx.x;
    const int hg = blockIdx.y;
    const int n_new = a.meta[2 * hg], first = a.meta[2 * hg + 1];
    if (first >= n_new) return;
    const long long base = (long long)hg * a.Lmax;
    const int32_t *src_of = a.list_a + base;
    const int slices = a.row_bytes / kSliceBytes;
    const int sl = blockIdx.x;
    if (sl < 2 * slices) {
        char *cache = (sl < slices ? a.k : a.v) + base * a.row_bytes + (sl % slices) * kSliceBytes + 16 * (tid & 3);
        constexpr int ROWS = 64 * kMoveUpt;
        for (int p0 = first; p0 < n_new; p0 += ROWS) {
            uint4 val[kMoveUpt];
#pragma unroll
            for (int x = 0; x < kMoveUpt; ++x) {
                const int p = p0 + 64 * x + (tid >> 2);
                val[x] = make_uint4(0, 0, 0, 0);   // always defined, or the array is placed in scratch memory
                if (p < n_new) val[x] = *reinterpret_cast<const uint4 *>(cache + (long long)src_of[p] * a.row_bytes);
            }
            __syncthreads();
#pragma unroll
            for (int x = 0; x < kMoveUpt; ++x) {
                const int p = p0 + 64 * x + (tid >> 2);
                if (p < n_new) *reinterpret_cast<uint4 *>(cache + (long long)p * a.row_bytes) = val[x];
            }
        }
    } else {
        constexpr int ROWS = 256 * kMoveUpt;
        for (int p0 = first; p0 < n_new; p0 += ROWS) {
            float sc[kMoveUpt];
            uint8_t kd[kMoveUpt];
            int32_t ps[kMoveUpt];
#pragma unroll
            for (int x = 0; x < kMoveUpt; ++x) {
                const int p = p0 + 256 * x + tid;
                sc[x] = 0.f;
                kd[x] = 0;
                ps[x] = 0;
                if (p < n_new) {
                    const int s = src_of[p];
                    sc[x] = a.score[base + s];
                    kd[x] = a.kind[base + s];
                    ps[x] = a.pos[base + s];
                }
            }
            __syncthreads();
#pragma unroll
            for (int x = 0; x < kMoveUpt; ++x) {
                const int p = p0 + 256 * x + tid;
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
    hipLaunchKernelGGL(kv_select_kernel, dim3((unsigned)heads), dim3(1024), 0, stream, a);
    prof.end();
    if (d.order == LVLM_ORDER_STABLE) {
        const int slices = a.row_bytes / kSliceBytes;
        prof.begin("kv_move");
        hipLaunchKernelGGL(kv_move_kernel, dim3(2 * slices + 1, (unsigned)heads), dim3(256), 0, stream, a);
        prof.end();
    }
    return hipGetLastError();
}

}  // namespace lvlm
