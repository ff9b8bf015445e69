// Split-chain path of the ECRM update (Sec. 3.3.1 on an entry that receives many updates in one call): entries
// with more than kLongRun updates are not walked by one wavefront inside the apply kernel.  For a run g_1..g_m
// on one parameter, G_t = G_0 + sum_{s<=t} g_s^2 is a prefix sum and the entry moves by
// -lr * sum_t g_t / sqrt(G_t + eps).  Runs of moderate length are walked by one workgroup each, with one read of
// their gradients (mid_chain_kernel); longer ones are cut into pieces: (1) each piece sums its g^2, (2) a scan over
// the pieces gives every piece its starting accumulator, (3) each piece sums its steps, (4) the pieces' sums are
// added in order.  Either way long_res[slot] receives the run's totals, which the apply kernel takes from there.
#include "rows.h"

namespace ecrm {

// ================================================================================================
// split-chain path
// ================================================================================================

// Marks the heads of rows with more than kLongRun updates and gives each a slot.  Only every (kLongRun/2)-th
// sorted position is looked at: a run of more than kLongRun positions contains two such positions in a row, q and
// q + kLongRun/2, and exactly one q whose predecessor q - kLongRun/2 lies outside the run; the thread of that q finds
// the run's head (binary search over the kLongRun/2 positions before q) and checks its length.  So the kernel reads
// three keys per kLongRun/2 positions instead of three per position.
__global__ __launch_bounds__(256) void long_find_kernel(const uint32_t *sk, uint32_t n, Header *hdr,
                                                        uint32_t *long_slot, uint32_t *long_head,
                                                        uint32_t max_slots)
{
    static_assert(kLongRun % 2 == 0 && kLongRun >= 2, "the probe distance is half the threshold");
    constexpr uint32_t H = kLongRun / 2;
    if (hdr->batch_bad) return;
    n = min(n, hdr->n_valid);
    const uint32_t threads = gridDim.x * blockDim.x;
    for (uint32_t t = blockIdx.x * blockDim.x + threadIdx.x; t < n / H; t += threads) {
        const uint32_t q = t * H;                    // q + H <= n
        if (q + H >= n) break;
        const uint32_t x = sk[q];
        if (sk[q + H] != x) continue;
        if (q >= H && sk[q - H] == x) continue;      // not the first probed position inside its run
        // the head lies in (q - H, q], or in [0, q] at the start of the batch: the first position whose key is x
        uint32_t lo = q >= H ? q - H : 0xFFFFFFFFu, hi = q;      // sk[lo] != x (lo = -1: before the batch), sk[hi] == x
        while (hi - lo > 1u) {                       // unsigned wrap-around makes -1 work: hi - lo = hi + 1
            const uint32_t mid = lo + (hi - lo) / 2u;
            if (sk[mid] == x) hi = mid; else lo = mid;
        }
        const uint32_t p = hi;
        if (p + kLongRun < n && sk[p + kLongRun] == x) {
            const uint32_t slot = atomicAdd(&hdr->n_long, 1u);
            if (slot < max_slots) {          // always true: at most n / (kLongRun+1) such rows exist
                long_head[slot] = p;
                long_slot[p] = slot;
            }
        }
    }
}

// Length of each long run (binary search for its end) and its cut into pieces.  One wave per run.
// A run of at most mid_max updates gets no pieces: its slot goes on the list of its length class
// (mid_chain_kernel) -- provided the batch has at least mid_min_rows long rows.
constexpr int kPlanWaves = 16;      // runs a block of the plan kernel looks at together

__global__ __launch_bounds__(kPlanWaves * kWave) void long_plan_kernel(
    const uint32_t *sk, uint32_t n, Header *hdr, const uint32_t *long_head, uint32_t *long_len, uint32_t *long_piece,
    uint32_t *long_count, uint32_t *long_base, uint32_t *piece_slot, uint32_t *mid_list, uint32_t mid_max,
    uint32_t mid_min_rows, uint32_t piece_waves, uint32_t max_slots, uint32_t max_pieces)
{
    // what each wave found, and where its run's pieces (or its place in a list) begin
    __shared__ uint32_t s_pieces[kPlanWaves], s_len[kPlanWaves], s_class[kPlanWaves], s_start[kPlanWaves];
    constexpr uint32_t kNoClass = 0xFFFFFFFFu;
    if (hdr->batch_bad) return;
    n = min(n, hdr->n_valid);
    const uint32_t nl = min(hdr->n_long, max_slots);
    if (nl < mid_min_rows) mid_max = 0;
    // Smallest piece: a piece costs its wave a few memory latencies before the first gradient arrives, so pieces
    // should be as long as the work allows while there are still several per wave of the piece kernels.  How much
    // work there is is not known yet; the number of long rows is, and such a row has kLongRowGuess updates on
    // average in the skewed batches this path exists for (measured optimum: 256-512 with 420 long rows in 2^24
    // updates, >= 2048 with 3801 in 2^26).
    const uint32_t piece_min = min(kPieceMinCap, max(kPieceMin, (uint32_t)((unsigned long long)nl * kLongRowGuess / piece_waves)));
    const uint32_t lane = lane_id(), w = uniform(threadIdx.x / kWave);
    for (uint32_t slot0 = blockIdx.x * kPlanWaves; slot0 < nl; slot0 += gridDim.x * kPlanWaves) {
        const uint32_t slot = slot0 + w;
        uint32_t L = 0, C = 0, P = 0, cls = kNoClass;
        if (slot < nl) {
            const uint32_t p = uniform(long_head[slot]);
            const uint32_t x = uniform(sk[p]);
            // the run's end, by a 64-ary search: the lanes probe 64 evenly spaced positions of (lo, hi] at once, and
            // the probes that still carry x are a prefix of them (the keys are sorted)
            uint32_t lo = p + kLongRun, hi = n;            // sk[lo] == x, sk[hi] != x (hi == n: past the end)
            while (hi - lo > 1) {
                const uint32_t step = (hi - lo + kWave - 1) / kWave;                 // >= 1
                const uint32_t probe = lo + (lane + 1u) * step;                      // <= lo + 64 * step < 2^32: n <= 2^31
                const uint32_t inside = (uint32_t)__popcll(__ballot(probe < hi && sk[probe] == x));
                const uint32_t first_out = lo + (inside + 1u) * step;                // the first probe that is not x, if any
                lo += inside * step;
                if (inside < (uint32_t)kWave && first_out < hi) hi = first_out;
            }
            L = hi - p;
            if (L <= mid_max) {
                cls = 0;
                while (cls + 1 < kMidClasses && ((L - 1) / kLongRun) >> (cls + 1)) ++cls;
            } else {
                C = (L + kPieceMaxCount - 1) / kPieceMaxCount;
                if (C < piece_min) C = piece_min;
                P = (L + C - 1) / C;
            }
        }
        if (lane == 0) {
            s_pieces[w] = P;
            s_len[w] = L;
            s_class[w] = cls;
        }
        __syncthreads();
        // One thread reserves for the whole block: the counters are updated once per kPlanWaves runs (one update
        // per run kept this kernel at the pace of the counters: 11 000 updates of three addresses, 94 us).
        if (threadIdx.x == 0) {
            uint32_t pieces = 0, in_class[kMidClasses];
            unsigned long long items = 0;
#pragma unroll
            for (uint32_t c = 0; c < kMidClasses; ++c) in_class[c] = 0;
#pragma unroll
            for (int v = 0; v < kPlanWaves; ++v) {
                pieces += s_pieces[v];
                items += s_len[v];
#pragma unroll
                for (uint32_t c = 0; c < kMidClasses; ++c) in_class[c] += s_class[v] == c ? 1u : 0u;
            }
            uint32_t piece_at = pieces ? atomicAdd(&hdr->n_pieces, pieces) : 0u;
            if (items) atomicAdd(&hdr->n_long_items, items);
            uint32_t class_at[kMidClasses];
#pragma unroll
            for (uint32_t c = 0; c < kMidClasses; ++c) class_at[c] = in_class[c] ? atomicAdd(&hdr->n_mid[c], in_class[c]) : 0u;
#pragma unroll
            for (int v = 0; v < kPlanWaves; ++v) {
                uint32_t start = piece_at;
                piece_at += s_pieces[v];
#pragma unroll
                for (uint32_t c = 0; c < kMidClasses; ++c) {
                    if (s_class[v] == c) start = class_at[c]++;
                }
                s_start[v] = start;
            }
        }
        __syncthreads();
        const uint32_t start = s_start[w];
        __syncthreads();                                   // s_* are free for the next round
        if (slot >= nl) continue;
        if (lane == 0) {
            long_len[slot] = L;
            long_piece[slot] = C;                          // 0: no pieces, one workgroup walks the run
            long_count[slot] = P;
            long_base[slot] = P ? start : 0u;
            if (cls != kNoClass && start < max_slots) mid_list[(size_t)cls * max_slots + start] = slot;   // always true: at most n_long such rows
        }
        for (uint32_t j = lane; j < P; j += kWave)
            if (start + j < max_pieces) piece_slot[start + j] = slot;   // always true by the bound on pieces
    }
}

// Phase 1 (STEPS == false): partial[piece] = the piece's summary started from zero (Adagrad: sum of
//                           g^2; momentum: the velocity it builds; combined rules: sum of g).
//                           Momentum also gets partial2[piece] = the sum of the velocities the piece
//                           goes through when started from zero: its rule is linear, so the steps of
//                           a piece started from velocity v are lr * (c * v + that sum) with
//                           c = mu + mu^2 + ... + mu^len, and the gradients need no second read.
// Phase 3 (STEPS == true):  partial[piece] holds the piece's starting state on entry and the sum of
//                           its steps on exit (sequential rules only).
// One wave per piece; the item indices of 64 positions are fetched with one coalesced load and
// handed out lane by lane, and U gradient rows are in flight at a time.
template <int NC, bool STEPS, int MODE>
__global__ __launch_bounds__(256) void long_piece_kernel(const uint32_t *si, const float *grads, Header *hdr,
                                                         const uint32_t *long_head, const uint32_t *long_len,
                                                         const uint32_t *long_piece, const uint32_t *long_base,
                                                         const uint32_t *piece_slot, double *partial,
                                                         double *partial2, uint32_t max_pieces, Geometry geo)
{
    constexpr bool kVelSum = !STEPS && MODE == kMomentumSeq;
    if (hdr->batch_bad) return;
    const uint32_t np = min(hdr->n_pieces, max_pieces);
    const uint32_t D = geo.D, lane = lane_id();
    const RuleParams rp = rule_params(geo);
    constexpr int U = 16;
    for (uint32_t pc = wave_id(); pc < np; pc += wave_count()) {
        const uint32_t slot = uniform(piece_slot[pc]);
        const uint32_t j = pc - uniform(long_base[slot]);
        const uint32_t head = uniform(long_head[slot]), L = uniform(long_len[slot]), C = uniform(long_piece[slot]);
        const uint32_t start = head + j * C;
        const uint32_t end = min(start + C, head + L);
        for (uint32_t cb = 0; cb < geo.ncb; ++cb) {
            const uint32_t col0 = cb * NC * 128u;
            const rsrc_t part = row_f64(partial, pc, D, col0);
            D2 G[NC], acc[NC], vs[NC];
#pragma unroll
            for (int i = 0; i < NC; ++i) {
                acc[i] = vs[i] = D2{0, 0};
                G[i] = STEPS ? ldd2(part, i) : D2{0, 0};
            }
            uint32_t widx = start + lane < end ? si[start + lane] : 0u;
            for (uint32_t base = start; base < end; base += kWave) {
                const uint32_t cnt = min((uint32_t)kWave, end - base);
                const uint32_t cur_idx = widx;
                if (base + kWave < end)            // next window in flight while this one is consumed
                    widx = base + kWave + lane < end ? si[base + kWave + lane] : 0u;
                for (uint32_t u0 = 0; u0 < cnt; u0 += U) {
                    float2 g[U][NC];
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        // lanes past the end of the piece re-read its last item; their values are not used
                        const uint32_t idx = from_lane(cur_idx, min(u0 + u, cnt - 1));
                        const rsrc_t r = row_f32(grads, idx, D, col0);
#pragma unroll
                        for (int i = 0; i < NC; ++i) g[u][i] = ldg2(r, i);
                    }
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        if (u0 + u < cnt) {
#pragma unroll
                            for (int i = 0; i < NC; ++i) {
                                if (STEPS) item2<MODE>(G[i], acc[i], g[u][i], rp);
                                else summary2<MODE>(acc[i], g[u][i], rp);
                                if (kVelSum) {
                                    vs[i].x += acc[i].x;
                                    vs[i].y += acc[i].y;
                                }
                            }
                        }
                    }
                }
            }
#pragma unroll
            for (int i = 0; i < NC; ++i) std2(part, i, acc[i]);
            if (kVelSum) {
                const rsrc_t part2 = row_f64(partial2, pc, D, col0);
#pragma unroll
                for (int i = 0; i < NC; ++i) std2(part2, i, vs[i]);
            }
        }
    }
}

constexpr int kRowWaves = 16;      // waves that share one long row in the scan and reduce kernels

// Phase 2: exclusive scan of the pieces' summaries, seeded with the stored state, so that every
// piece knows the state it starts from: Adagrad adds the sums of squares; momentum composes
// v -> mu^len * v + V_piece.  long_res[slot][1] receives the state after the whole run.
// Adagrad: partial[piece] leaves as the piece's starting state (the steps need a second pass over
// its gradients); momentum: it leaves as the sum of the piece's steps, from partial2 (see above).
// One block of 16 waves per long row: every wave folds a contiguous range of pieces, the ranges'
// results are exchanged through LDS, and every wave then rewrites its range with the prefixes.
template <int NC, int MODE>
__global__ __launch_bounds__(kRowWaves * kWave) void long_scan_kernel(
    const uint32_t *sk, const float *A, Header *hdr, const uint32_t *long_head, const uint32_t *long_count,
    const uint32_t *long_base, const uint32_t *long_len, const uint32_t *long_piece, double *partial,
    const double *partial2, double *long_res, uint32_t max_slots, Geometry geo)
{
    __shared__ double s_fold[kRowWaves][NC][2][kWave];
    if (hdr->batch_bad) return;
    const uint32_t nl = min(hdr->n_long, max_slots);
    const uint32_t D = geo.D, lane = lane_id(), w = threadIdx.x / kWave;
    constexpr uint32_t U = 8;
    for (uint32_t slot = blockIdx.x; slot < nl; slot += gridDim.x) {
        const uint32_t x = uniform(sk[long_head[slot]]);
        const uint32_t P = uniform(long_count[slot]), base = uniform(long_base[slot]);
        if (P == 0) continue;                                        // walked by one workgroup: no pieces to scan
        const uint32_t C = uniform(long_piece[slot]), L = uniform(long_len[slot]);
        const uint32_t Q = (P + kRowWaves - 1) / kRowWaves;          // pieces per wave
        const uint32_t j_lo = min(w * Q, P), j_hi = min(j_lo + Q, P);
        // momentum: decay over one full piece, over the run's (shorter) last piece
        const double mu = (double)geo.mu;
        const double decay_full = MODE == kMomentumSeq ? pow(mu, (double)C) : 1.0;
        const double decay_last = MODE == kMomentumSeq ? pow(mu, (double)(L - (P - 1) * C)) : 1.0;
        // mu + mu^2 + ... + mu^len for a full piece and for the last one
        const double geo_full = mu * (1.0 - decay_full) / (1.0 - mu), geo_last = mu * (1.0 - decay_last) / (1.0 - mu);
        const double lr = (double)geo.lr;
        for (uint32_t cb = 0; cb < geo.ncb; ++cb) {
            const uint32_t col0 = cb * NC * 128u;
            // (a) fold of this wave's range, started from zero
            D2 f[NC];
#pragma unroll
            for (int i = 0; i < NC; ++i) f[i] = D2{0, 0};
            for (uint32_t j0 = j_lo; j0 < j_hi; j0 += U) {
                D2 t[U][NC];
#pragma unroll
                for (uint32_t u = 0; u < U; ++u) {
                    const rsrc_t r = row_f64(partial, base + min(j0 + u, j_hi - 1), D, col0);
#pragma unroll
                    for (int i = 0; i < NC; ++i) t[u][i] = ldd2(r, i);
                }
#pragma unroll
                for (uint32_t u = 0; u < U; ++u) {
                    if (j0 + u < j_hi) {
                        const double dec = j0 + u + 1 == P ? decay_last : decay_full;
#pragma unroll
                        for (int i = 0; i < NC; ++i) {
                            if (MODE == kMomentumSeq) {
                                f[i].x = fma(dec, f[i].x, t[u][i].x);
                                f[i].y = fma(dec, f[i].y, t[u][i].y);
                            } else {
                                f[i].x += t[u][i].x;
                                f[i].y += t[u][i].y;
                            }
                        }
                    }
                }
            }
            __syncthreads();                                         // previous column block's reads are done
#pragma unroll
            for (int i = 0; i < NC; ++i) {
                s_fold[w][i][0][lane] = f[i].x;
                s_fold[w][i][1][lane] = f[i].y;
            }
            __syncthreads();
            // (b) state at the start of this wave's range (and, for wave 0, after the whole run)
            const rsrc_t arow = row_f32(A, x, D, col0);
            D2 G[NC], total[NC];
#pragma unroll
            for (int i = 0; i < NC; ++i) {
                G[i] = widen2(ld2(arow, i));
                total[i] = G[i];
            }
            for (uint32_t u = 0; u < (uint32_t)kRowWaves; ++u) {
                const uint32_t u_lo = min(u * Q, P), u_hi = min(u_lo + Q, P);
                if (u_lo == u_hi) break;
                double dec = 1.0;
                if (MODE == kMomentumSeq) {
                    const uint32_t items = u_hi == P ? L - u_lo * C : (u_hi - u_lo) * C;
                    dec = pow(mu, (double)items);
                }
#pragma unroll
                for (int i = 0; i < NC; ++i) {
                    const double fx = s_fold[u][i][0][lane], fy = s_fold[u][i][1][lane];
                    if (u < w) {
                        G[i].x = MODE == kMomentumSeq ? fma(dec, G[i].x, fx) : G[i].x + fx;
                        G[i].y = MODE == kMomentumSeq ? fma(dec, G[i].y, fy) : G[i].y + fy;
                    }
                    total[i].x = MODE == kMomentumSeq ? fma(dec, total[i].x, fx) : total[i].x + fx;
                    total[i].y = MODE == kMomentumSeq ? fma(dec, total[i].y, fy) : total[i].y + fy;
                }
            }
            // (c) rewrite this wave's range with the prefixes
            for (uint32_t j0 = j_lo; j0 < j_hi; j0 += U) {
                D2 t[U][NC], t2[U][NC];
#pragma unroll
                for (uint32_t u = 0; u < U; ++u) {
                    const rsrc_t r = row_f64(partial, base + min(j0 + u, j_hi - 1), D, col0);
#pragma unroll
                    for (int i = 0; i < NC; ++i) t[u][i] = ldd2(r, i);
                    if (MODE == kMomentumSeq) {
                        const rsrc_t r2 = row_f64(partial2, base + min(j0 + u, j_hi - 1), D, col0);
#pragma unroll
                        for (int i = 0; i < NC; ++i) t2[u][i] = ldd2(r2, i);
                    }
                }
#pragma unroll
                for (uint32_t u = 0; u < U; ++u) {
                    if (j0 + u < j_hi) {
                        const rsrc_t r = row_f64(partial, base + j0 + u, D, col0);
                        const bool is_last = j0 + u + 1 == P;
                        const double dec = is_last ? decay_last : decay_full;
#pragma unroll
                        for (int i = 0; i < NC; ++i) {
                            if (MODE == kMomentumSeq) {          // the piece's steps, from its starting velocity
                                const double c = is_last ? geo_last : geo_full;
                                std2(r, i, D2{lr * fma(c, G[i].x, t2[u][i].x), lr * fma(c, G[i].y, t2[u][i].y)});
                            } else {
                                std2(r, i, G[i]);
                            }
                            if (MODE == kMomentumSeq) {
                                G[i].x = fma(dec, G[i].x, t[u][i].x);
                                G[i].y = fma(dec, G[i].y, t[u][i].y);
                            } else {
                                G[i].x += t[u][i].x;
                                G[i].y += t[u][i].y;
                            }
                        }
                    }
                }
            }
            if (w == 0) {
                const rsrc_t res = row_f64(long_res, (size_t)slot * 2 + 1, D, col0);
#pragma unroll
                for (int i = 0; i < NC; ++i) std2(res, i, total[i]);
            }
        }
    }
}

// Phase 4: long_res[slot][0] = sum over the pieces of their step sums (16 waves per long row: ranges
// of pieces are summed in order, then the ranges' sums in order).
template <int NC>
__global__ __launch_bounds__(kRowWaves * kWave) void long_reduce_kernel(Header *hdr, const uint32_t *long_count,
                                                                        const uint32_t *long_base, const double *partial,
                                                                        double *long_res, uint32_t max_slots, Geometry geo)
{
    __shared__ double s_fold[kRowWaves][NC][2][kWave];
    if (hdr->batch_bad) return;
    const uint32_t nl = min(hdr->n_long, max_slots);
    const uint32_t D = geo.D, lane = lane_id(), w = threadIdx.x / kWave;
    constexpr uint32_t U = 8;
    for (uint32_t slot = blockIdx.x; slot < nl; slot += gridDim.x) {
        const uint32_t P = uniform(long_count[slot]), base = uniform(long_base[slot]);
        if (P == 0) continue;                                        // its totals are there already
        const uint32_t Q = (P + kRowWaves - 1) / kRowWaves;
        const uint32_t j_lo = min(w * Q, P), j_hi = min(j_lo + Q, P);
        for (uint32_t cb = 0; cb < geo.ncb; ++cb) {
            const uint32_t col0 = cb * NC * 128u;
            D2 s[NC];
#pragma unroll
            for (int i = 0; i < NC; ++i) s[i] = D2{0, 0};
            for (uint32_t j0 = j_lo; j0 < j_hi; j0 += U) {
                D2 t[U][NC];
#pragma unroll
                for (uint32_t u = 0; u < U; ++u) {
                    const rsrc_t r = row_f64(partial, base + min(j0 + u, j_hi - 1), D, col0);
#pragma unroll
                    for (int i = 0; i < NC; ++i) t[u][i] = ldd2(r, i);
                }
#pragma unroll
                for (uint32_t u = 0; u < U; ++u) {
                    if (j0 + u < j_hi) {
#pragma unroll
                        for (int i = 0; i < NC; ++i) {
                            s[i].x += t[u][i].x;
                            s[i].y += t[u][i].y;
                        }
                    }
                }
            }
            __syncthreads();
#pragma unroll
            for (int i = 0; i < NC; ++i) {
                s_fold[w][i][0][lane] = s[i].x;
                s_fold[w][i][1][lane] = s[i].y;
            }
            __syncthreads();
            if (w == 0) {
                const rsrc_t res = row_f64(long_res, (size_t)slot * 2 + 0, D, col0);
#pragma unroll
                for (int i = 0; i < NC; ++i) {
                    D2 tot = D2{0, 0};
                    for (int u = 0; u < kRowWaves; ++u) {
                        tot.x += s_fold[u][i][0][lane];
                        tot.y += s_fold[u][i][1][lane];
                    }
                    std2(res, i, tot);
                }
            }
        }
    }
}

// A run of moderate length on the Adagrad rule, walked by one workgroup with one read of its gradients.
// Per round every wave takes T consecutive updates of the run and keeps their gradient rows in registers:
// it sums their squares, the waves exchange these sums through LDS -- so that each knows the accumulator
// its updates start from -- and it then takes its steps from the registers.  The accumulator is carried
// from round to round; the waves' step sums are added up once, at the end of the run.  Runs are taken
// longest first (the lists are by length class), so that the longest one does not end the kernel alone.
// long_res[slot] receives what the pieces' kernels would have left there: the sum of the steps and the
// accumulator after the run.
template <int NC>
__global__ __launch_bounds__(kMidWaves * kWave, 4) void mid_chain_kernel(
    const uint32_t *sk, const uint32_t *si, const float *grads, const float *A, Header *hdr, const uint32_t *long_head,
    const uint32_t *long_len, const uint32_t *mid_list, double *long_res, uint32_t max_slots, Geometry geo)
{
    constexpr int T = 32 / NC;                               // gradient rows a wave holds
    constexpr uint32_t R = kMidWaves * T;                    // updates per round
    __shared__ double s_part[2][kMidWaves][NC][2][kWave];
    __shared__ uint32_t s_ticket;
    if (hdr->batch_bad) return;
    uint32_t in_class[kMidClasses], total = 0;
#pragma unroll
    for (uint32_t c = 0; c < kMidClasses; ++c) {
        in_class[c] = min(hdr->n_mid[c], max_slots);
        total += in_class[c];
    }
    const uint32_t D = geo.D, lane = lane_id(), w = uniform(threadIdx.x / kWave);
    const RuleParams rp = rule_params(geo);
    for (;;) {
        if (threadIdx.x == 0) s_ticket = atomicAdd(&hdr->mid_ticket, 1u);
        __syncthreads();
        uint32_t t = uniform(s_ticket);
        __syncthreads();                                     // everyone has read the ticket before the next one is written
        if (t >= total) break;
        uint32_t c = kMidClasses - 1;
        while (t >= in_class[c]) {                           // ends: t < total
            t -= in_class[c];
            --c;
        }
        const uint32_t slot = uniform(mid_list[(size_t)c * max_slots + t]);
        const uint32_t head = uniform(long_head[slot]), L = uniform(long_len[slot]), x = uniform(sk[head]);
        for (uint32_t cb = 0; cb < geo.ncb; ++cb) {
            const uint32_t col0 = cb * NC * 128u;
            const rsrc_t arow = row_f32(A, x, D, col0);
            D2 G[NC], acc[NC];
#pragma unroll
            for (int i = 0; i < NC; ++i) {
                G[i] = widen2(ld2(arow, i));
                acc[i] = D2{0, 0};
            }
            uint32_t buf = 0;
            for (uint32_t r0 = 0; r0 < L; r0 += R, buf ^= 1u) {
                const uint32_t off = r0 + w * T;             // this wave's first update, counted from the head
                const uint32_t cnt = off < L ? min((uint32_t)T, L - off) : 0u;
                // positions past the end of the run re-read its last update; their values are not used
                const uint32_t my_idx = si[head + min(off + lane, L - 1u)];
                float2 g[T][NC];
#pragma unroll
                for (int u = 0; u < T; ++u) {
                    const rsrc_t r = row_f32(grads, from_lane(my_idx, u), D, col0);
#pragma unroll
                    for (int i = 0; i < NC; ++i) g[u][i] = ldg2(r, i);
                }
                D2 s[NC];
#pragma unroll
                for (int i = 0; i < NC; ++i) s[i] = D2{0, 0};
#pragma unroll
                for (int u = 0; u < T; ++u) {
                    if ((uint32_t)u < cnt) {
#pragma unroll
                        for (int i = 0; i < NC; ++i) summary2<kAdagradSeq>(s[i], g[u][i], rp);
                    }
                }
                // the rows stay in registers as the floats they are (otherwise the compiler keeps the
                // widened copies it made for the squares alive until the steps: three times the registers)
#pragma unroll
                for (int u = 0; u < T; ++u) {
#pragma unroll
                    for (int i = 0; i < NC; ++i) asm volatile("" : "+v"(g[u][i].x), "+v"(g[u][i].y));
                }
#pragma unroll
                for (int i = 0; i < NC; ++i) {
                    s_part[buf][w][i][0][lane] = s[i].x;
                    s_part[buf][w][i][1][lane] = s[i].y;
                }
                // One barrier per round is enough: the next round writes the other half of s_part, and a wave
                // that writes this half again (two rounds on) has passed the next round's barrier, which every
                // wave reaches only after reading this half.
                __syncthreads();
                D2 Gs[NC];
#pragma unroll
                for (int i = 0; i < NC; ++i) Gs[i] = G[i];
#pragma unroll
                for (int v = 0; v < kMidWaves; ++v) {
#pragma unroll
                    for (int i = 0; i < NC; ++i) {
                        if ((uint32_t)v == w) Gs[i] = G[i];  // accumulator before this wave's first update
                        G[i].x += s_part[buf][v][i][0][lane];
                        G[i].y += s_part[buf][v][i][1][lane];
                    }
                }
#pragma unroll
                for (int u = 0; u < T; ++u) {
                    if ((uint32_t)u < cnt) {
#pragma unroll
                        for (int i = 0; i < NC; ++i) item2<kAdagradSeq>(Gs[i], acc[i], g[u][i], rp);
                    }
                }
            }
            // the waves' step sums, added in the order of the waves
#pragma unroll
            for (int i = 0; i < NC; ++i) {
                s_part[buf][w][i][0][lane] = acc[i].x;
                s_part[buf][w][i][1][lane] = acc[i].y;
            }
            __syncthreads();
            if (w == 0) {
                const rsrc_t r0 = row_f64(long_res, (size_t)slot * 2 + 0, D, col0);
                const rsrc_t r1 = row_f64(long_res, (size_t)slot * 2 + 1, D, col0);
#pragma unroll
                for (int i = 0; i < NC; ++i) {
                    D2 tot = D2{0, 0};
#pragma unroll
                    for (int v = 0; v < kMidWaves; ++v) {
                        tot.x += s_part[buf][v][i][0][lane];
                        tot.y += s_part[buf][v][i][1][lane];
                    }
                    std2(r0, i, tot);
                    std2(r1, i, G[i]);
                }
            }
            __syncthreads();                                 // s_part is free for the next run
        }
    }
}

// ================================================================================================
// host side
// ================================================================================================

template <int NC, int MODE>
static bool chain_grids_for(int cus, LaunchGrids *out)
{
    out->p1 = resident_grid(long_piece_kernel<NC, false, MODE>, cus);
    out->p3 = resident_grid(long_piece_kernel<NC, true, MODE>, cus);
    out->mid = resident_grid(mid_chain_kernel<NC>, cus, kMidWaves * kWave);
    out->mid_min_rows = kMidMinRowsPerBlock * (uint32_t)(out->mid > 0 ? out->mid : 0);
    return out->p1 > 0 && out->p3 > 0 && out->mid > 0;
}

template <int NC, int MODE>
static void chains_for(const Scratch &s, const Geometry &g, const LaunchGrids &lg, const float *A, const float *grads,
                       const uint32_t *sk, const uint32_t *si, uint32_t n, uint32_t max_slots,
                       uint32_t max_pieces, int cus, hipStream_t st)
{
    const dim3 grid(cus * 8), block(256);
    hipLaunchKernelGGL(long_find_kernel, grid, block, 0, st, sk, n, s.hdr, s.long_slot, s.long_head, max_slots);
    const uint32_t mid_max = MODE == kAdagradSeq ? kMidMax : 0u;     // the other rules read a long run once anyway
    hipLaunchKernelGGL(long_plan_kernel, dim3(cus * 2), dim3(kPlanWaves * kWave), 0, st, sk, n, s.hdr, s.long_head, s.long_len,
                       s.long_piece, s.long_count, s.long_base, s.piece_slot, s.mid_list, mid_max, lg.mid_min_rows,
                       (uint32_t)lg.p1 * (256u / kWave), max_slots, max_pieces);
    if (mid_max > kLongRun && n / (kLongRun + 1u) >= lg.mid_min_rows)       // else the plan kernel lists no such run
        hipLaunchKernelGGL((mid_chain_kernel<NC>), dim3(lg.mid), dim3(kMidWaves * kWave), 0, st, sk, si, grads, A, s.hdr,
                           s.long_head, s.long_len, s.mid_list, s.long_res, max_slots, g);
    hipLaunchKernelGGL((long_piece_kernel<NC, false, MODE>), dim3(lg.p1), block, 0, st, si, grads, s.hdr, s.long_head,
                       s.long_len, s.long_piece, s.long_base, s.piece_slot, s.partial, s.partial2, max_pieces, g);
    if (!Rule<MODE>::combine) {
        hipLaunchKernelGGL((long_scan_kernel<NC, MODE>), dim3(cus * 2), dim3(kRowWaves * kWave), 0, st, sk, A, s.hdr, s.long_head, s.long_count,
                           s.long_base, s.long_len, s.long_piece, s.partial, s.partial2, s.long_res, max_slots, g);
        if (MODE != kMomentumSeq)        // momentum's steps came out of the scan: no second pass over the gradients
            hipLaunchKernelGGL((long_piece_kernel<NC, true, MODE>), dim3(lg.p3), block, 0, st, si, grads, s.hdr,
                               s.long_head, s.long_len, s.long_piece, s.long_base, s.piece_slot, s.partial, s.partial2,
                               max_pieces, g);
    }
    hipLaunchKernelGGL((long_reduce_kernel<NC>), dim3(cus * 2), dim3(kRowWaves * kWave), 0, st, s.hdr, s.long_count, s.long_base, s.partial,
                       s.long_res, max_slots, g);
}

bool query_chain_grids(const Geometry &g, int cus, LaunchGrids *out)
{
    bool ok = false;
    ECRM_DISPATCH(ok = chain_grids_for, cus, out);
    return ok;
}

void launch_chains(const Scratch &s, const Geometry &g, const LaunchGrids &lg, const float *A, const float *grads,
                   const uint32_t *sk, const uint32_t *si, uint32_t n, uint32_t max_slots,
                   uint32_t max_pieces, int cus, hipStream_t st)
{
    if (n <= kLongRun) return;    // no row can have more than kLongRun updates
    ECRM_DISPATCH(chains_for, s, g, lg, A, grads, sk, si, n, max_slots, max_pieces, cus, st);
}

}  // namespace ecrm
