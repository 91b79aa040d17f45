// Moves on a placement schedule: incremental cost change, the annealing loop
// (one wavefront per chain) and the best-so-far reduction.  gfx950 only.
//
// A move edits the timeline of one (layer, page) bit inside a window of at most
// 64 token steps, so the 64 lanes of a wavefront each own one step of the
// window: lane i <-> step base + i.  Which steps flip is decided with ballots;
// the cost change is the 64-wide tree sum over the lanes of (t' - t), i.e. the
// same summation tree as the total latency uses.
#include <math.h>
#include <string.h>

#include <vector>

#include "kvp_internal.h"

#define LOG_WORDS 10   // layer, page, layer2, page2, base, flip1 lo/hi, flip2 lo/hi, spare
#define CALIB_MOVES 256

struct ChainState {
    double t_cur, t_best, c0, c;
    uint64_t accepted, uphill, null_moves, clipped, improved, log_len, moves_done;
    uint32_t level, log_overflow;
    uint32_t best_saved, pad_;   // the best schedule is the chain's snapshot (the log does not lead to it and is not kept)
};

struct SAParams {
    uint32_t seed_lo, seed_hi;
    uint64_t th0, th1;          // operator thresholds on a 32-bit draw
    uint64_t mpl;               // moves per temperature level
    uint32_t n_levels, max_len;
    double alpha, neg_ln_p0;
};

struct MoveEval {
    int verdict;        // uniform
    double dT;          // uniform
    int base;           // uniform: first step of the window
    uint64_t flip1, flip2;
    bool second;        // victim on another layer
    // per lane
    int n;              // step of this lane, -1 if outside the trace
    bool f1, f2, touch1, touch2, xnew;
    uint4 c1, c2;       // counters after the move of rows (layer, n) and (layer2, n)
    uint32_t xw1, xw2;  // the schedule words of the page and of the victim at step n, as loaded
    uint32_t oc;        // pages in HBM at step n, as loaded
};

__device__ __forceinline__ uint64_t ballot64(bool p) { return (uint64_t)__ballot(p); }
__device__ __forceinline__ int ctz64(uint64_t v) { return __ffsll((unsigned long long)v) - 1; }
__device__ __forceinline__ int msb64(uint64_t v) { return 63 - __clzll((long long)v); }

// Everything a lane needs to know about one (layer, page) at its step, gathered with
// independent loads that are all issued together: one memory round trip per move.
struct PageBits {
    bool v, pm, wm, x, xprev;   // exists, persists, written, in HBM now, in HBM one step earlier
    int au;                     // read units the page accounts for at this step (sum of its planes' weights)
};

// The words that hold one (layer, page) at a lane's step: requested together, looked at later.
// NP: weight planes looked at (>= q.pn; the surplus repeats the last plane with weight 0), so that
// the loads are a fixed, branch-free set.
template <int NP>
struct PageWords {
    uint32_t vw, pw, ww, xw, vpw, xpw, aw[NP];
};

template <int NP>
__device__ __forceinline__ PageWords<NP> request_page(const DevProblem &q, const uint32_t *X, uint32_t l, uint32_t n,
                                                      uint32_t w) {
    const size_t o = (size_t)n * q.Wd + w, op = (size_t)(n > 0 ? n - 1 : 0) * q.Wd + w;
    const uint32_t *Xl = X + (size_t)l * q.N * q.Wd;
    PageWords<NP> r;
    r.vw = q.V[o]; r.pw = q.Pm[o]; r.ww = q.Wm[o]; r.xw = Xl[o]; r.vpw = q.V[op]; r.xpw = Xl[op];
    const uint32_t *a = q.pl + ((size_t)l * q.N + n) * q.pn * q.Wd + w;
#pragma unroll
    for (int j = 0; j < NP; j++) r.aw[j] = a[(size_t)min((uint32_t)j, q.pn - 1) * q.Wd];
    return r;
}

// Makes the compiler treat the words as used here, unconditionally: without it the loads of words
// that only matter under a condition sink into branches and wait there one after the other.
template <int NP>
__device__ __forceinline__ void arrive(PageWords<NP> &r) {
    asm volatile("" : "+v"(r.vw), "+v"(r.pw), "+v"(r.ww), "+v"(r.xw), "+v"(r.vpw), "+v"(r.xpw));
#pragma unroll
    for (int j = 0; j < NP; j++) asm volatile("" : "+v"(r.aw[j]));
}

template <int NP>
__device__ __forceinline__ PageBits page_bits(const DevProblem &q, const PageWords<NP> &g, uint32_t n, bool ok,
                                              uint32_t b) {
    int au = 0;
#pragma unroll
    for (int j = 0; j < NP; j++) au += (int)(q.pw[j] * ((g.aw[j] >> b) & 1u));
    PageBits r;
    r.v = ok && ((g.vw >> b) & 1u);
    r.pm = ok && ((g.pw >> b) & 1u);
    r.wm = ok && ((g.ww >> b) & 1u);
    r.x = r.v && ((g.xw >> b) & 1u);
    r.xprev = ok && n > 0 && ((g.vpw >> b) & 1u) && ((g.xpw >> b) & 1u);
    r.au = au;
    return r;
}

// Effect on a step's counters of one page whose bit goes x -> x_new here and
// xprev -> xp_new one step earlier.
__device__ __forceinline__ void page_effect(const PageBits &g, bool x_new, bool xp_new, int &hr, int &hw, int &mi,
                                            int &mo) {
    if (g.x != x_new) {
        const int s = x_new ? 1 : -1;
        hr += s * g.au;
        hw += s * (int)g.wm;
    }
    if (g.pm) {
        mi += (int)(x_new && !xp_new) - (int)(g.x && !g.xprev);
        mo += (int)(!x_new && xp_new) - (int)(!g.x && g.xprev);
    }
}

// The first round trip of a move: every word, counter row and occupancy that pricing it may look
// at, requested together.  Fields of a malformed record are clamped so that the requests are valid
// and unconditional; `ok` tells.
template <int NP>
struct MoveLoads {
    bool ok;                        // uniform: the record is well formed
    PageWords<NP> gp, gq;           // the page, and the victim (a SET or SHIFT looks at the page itself again)
    uint32_t oc, acc1, acc2, wr;
    uint4 C1, C2;
};

// OCC_LATE: the occupancy is not requested here; finish_move reads it when it starts (from a copy
// that is cheap to read and may change until then).
template <int NP, bool OCC_LATE = false>
__device__ __forceinline__ MoveLoads<NP> issue_move(const DevProblem &q, const uint32_t *X, const uint32_t *cnt,
                                                    const uint32_t *occ, const kvp_move &m, int lane) {
    MoveLoads<NP> Ld;
    const uint32_t L = q.L, N = q.N;
    Ld.ok = !(m.op > 2 || m.layer >= L || m.page >= q.P || m.n1 >= N || m.len < 1 || m.len > KVP_MAX_LEN ||
              m.layer2 >= L || m.page2 >= q.P);
    const uint32_t l = min(m.layer, L - 1), l2 = min(m.layer2, L - 1);
    const uint32_t wp = min(m.page, q.P - 1) >> 5, wq = min(m.page2, q.P - 1) >> 5;
    const bool swap = m.op == KVP_OP_SWAP;
    // lane <-> step n1 + lane; steps past the trace shadow the last one
    const uint32_t nc = min(min(m.n1, N - 1) + (uint32_t)lane, N - 1);
    const uint32_t lv = swap ? l2 : l, wv = swap ? wq : wp;
    Ld.gp = request_page<NP>(q, X, l, nc, wp);
    Ld.gq = request_page<NP>(q, X, lv, nc, wv);
    Ld.oc = OCC_LATE ? 0u : occ[nc];
    Ld.C1 = *(const uint4 *)(cnt + ((size_t)l * N + nc) * 4);
    Ld.C2 = *(const uint4 *)(cnt + ((size_t)lv * N + nc) * 4);
    Ld.acc1 = q.acc[(size_t)l * N + nc];
    Ld.acc2 = q.acc[(size_t)lv * N + nc];
    Ld.wr = q.wr[nc];
    return Ld;
}

// Resolve a raw move against the schedule X (with its counters and occupancy)
// and price it, from the words that issue_move requested.  All 64 lanes of the
// wavefront must call this together.
// SLOT: the capacity holds at every inference step (n, l), not only once per token step: slot is
// the chain's table [L][N] of the pool after every slot, and a step may take the page if no slot of
// the two token steps that the bit reaches ends above the capacity: the bit of (l, p) at step n is
// part of the pool in the slots (n, l' >= l) and, if the page persists, (n + 1, l' < l), where layer l
// still holds its placement of step n.  An evicted victim (l2, q) leaves the slots (n, l' >= l2) and,
// if it persists, (n + 1, l' < l2).  Every step is judged against the schedule before the move: two
// steps of one run add to different slots, so no slot gains more than the one page it was judged for.
template <int NP, bool OCC_LATE = false, bool SLOT = false>
__device__ __forceinline__ MoveEval finish_move(const DevProblem &q, const uint32_t *X, const uint32_t *cnt,
                                                const uint32_t *occ, const kvp_move &m, int lane, MoveLoads<NP> &Ld,
                                                const uint32_t *slot = nullptr) {
    MoveEval R;
    R.verdict = KVP_MOVE_NULL; R.dT = 0.0; R.base = 0; R.flip1 = R.flip2 = 0; R.second = false;
    R.n = -1; R.f1 = R.f2 = R.touch1 = R.touch2 = R.xnew = false;
    R.c1 = make_uint4(0, 0, 0, 0); R.c2 = R.c1;
    R.xw1 = R.xw2 = R.oc = 0;
    const uint32_t L = q.L, N = q.N, cap = q.cap;
    (void)L;
    PageWords<NP> gp = Ld.gp, gq = Ld.gq;
    uint32_t oc = Ld.oc, acc1 = Ld.acc1, acc2 = Ld.acc2, wr = Ld.wr;
    uint4 C1 = Ld.C1, C2 = Ld.C2;
    // everything counts as used here, whether the move turns out to need it or not: otherwise the
    // loads of words that matter only under a condition sink into branches and wait there in turn
    arrive(gp); arrive(gq);
    asm volatile("" : "+v"(oc), "+v"(C1.x), "+v"(C1.y), "+v"(C1.z), "+v"(C1.w), "+v"(C2.x), "+v"(C2.y), "+v"(C2.z),
                 "+v"(C2.w), "+v"(acc1), "+v"(acc2), "+v"(wr));
    if (!Ld.ok) return R;
    const uint32_t l = m.layer, n1 = m.n1, len = m.len, l2 = m.layer2;
    const uint32_t wp = m.page >> 5, bp = m.page & 31, bq = m.page2 & 31;
    const bool swap = m.op == KVP_OP_SWAP;
    const bool same_layer = l2 == l;
    int n = (int)n1 + lane;
    bool inb = n < (int)N;
    uint32_t nc = inb ? (uint32_t)n : N - 1;
    if (OCC_LATE) oc = occ[nc];
    // may this lane's step take the page: as it is (room), or with the victim leaving (evict_fit)
    bool room = false, evict_fit = true;
    auto judge = [&]() {
        if (!SLOT) { room = oc < cap; return; }
        // largest pool over the slots that gain the page: a1, a2 of step nc (layers below l2, from l2 on),
        // b1, b2 of step nc + 1 (layers from l2 on, below l2); -1: no such slot
        int a1 = -1, a2 = -1, b1 = -1, b2 = -1;
        const bool nxt = inb && nc + 1 < N;
        const uint32_t nn = nxt ? nc + 1 : nc;
        for (uint32_t lp = 0; lp < L; lp++) {
            const int a = (int)slot[(size_t)lp * N + nc], b = (int)slot[(size_t)lp * N + nn];
            if (lp >= l) { if (lp >= l2) a2 = max(a2, a); else a1 = max(a1, a); }
            else { if (lp < l2) b2 = max(b2, b); else b1 = max(b1, b); }
        }
        const bool pers_p = nxt && ((q.Pm[(size_t)nn * q.Wd + wp] >> bp) & 1u);
        const bool pers_q = nxt && ((q.Pm[(size_t)nn * q.Wd + (m.page2 >> 5)] >> bq) & 1u);
        const int64_t c = (int64_t)cap;
        room = (int64_t)max(a1, a2) + 1 <= c && (!pers_p || (int64_t)max(b1, b2) + 1 <= c);
        evict_fit = (int64_t)a1 + 1 <= c && (int64_t)a2 <= c &&
                    (!pers_p || ((int64_t)b1 + 1 <= c && (int64_t)b2 + (pers_q ? 0 : 1) <= c));
    };
    PageBits P = page_bits<NP>(q, gp, nc, inb, bp);
    PageBits Q = swap ? page_bits<NP>(q, gq, nc, inb, bq) : P;
    if (!(ballot64(P.v) & 1ull)) return R;                 // the page does not exist at n1
    const uint64_t xmask = ballot64(P.x);
    const bool x1 = xmask & 1ull;
    bool f1 = false, f2 = false, clipped = false;
    int base = (int)n1;

    if (m.op != KVP_OP_SHIFT) {
        judge();
        const bool cont = lane == 0 || (inb && (uint32_t)lane < len && P.pm);
        const uint64_t bad = ballot64(!cont);
        const int e = bad ? ctz64(bad) : 64;
        const bool in_span = lane < e;
        if (m.op == KVP_OP_SET || x1) {
            const bool v = !x1;
            const bool differ = in_span && (P.x != v);
            if (v) {
                const uint64_t stop = ballot64(differ && !room);
                const int fs = stop ? ctz64(stop) : 64;
                f1 = differ && lane < fs;
                clipped = stop != 0;
            } else {
                f1 = differ;
            }
        } else {
            const bool victim_ok = !(same_layer && m.page2 == m.page);
            const bool cand = in_span && !P.x;
            const bool evict = cand && !room && victim_ok && Q.x && evict_fit;
            f1 = cand && (room || evict);
            f2 = evict;
            clipped = ballot64(cand && !room && !evict) != 0;
        }
    } else {
        const bool cont = lane == 0 || (inb && (uint32_t)lane <= len && P.pm);
        const uint64_t bad = ballot64(!cont);
        const int e = bad ? ctz64(bad) : 64;
        const bool xprev = lane > 0 && ((xmask >> (lane - 1)) & 1ull);
        const uint64_t tm = ballot64(lane >= 1 && lane < e && P.x != xprev);
        if (!tm) return R;                                  // constant timeline: nothing to shift
        const int it = ctz64(tm);
        const int nt = (int)n1 + it;
        const bool a = (xmask >> (it - 1)) & 1ull;
        const int d = (m.dsel & 2u) ? (int)(m.dsel & 1u) + 1 : (int)(m.dsel & 1u) - 2;   // -2,-1,+1,+2
        base = nt - 2;
        // re-map the lanes onto the five steps around the edge: lane k takes step nt - 2 + k
        n = base + lane;
        inb = lane < 5 && n >= 0 && n < (int)N;
        nc = inb ? (uint32_t)n : 0u;
        if (it <= 61) {
            // those steps are lanes it - 2 .. it + 2 of the window just loaded: a cross-lane move of
            // what they hold.  (For it = 1 lane 0 would be the step before the window; it is then neither
            // a target nor the neighbour of one, so what it gets is never looked at.)
            const int src = min(max(it - 2 + lane, 0), 63);
            auto take = [&](uint32_t &v) { v = (uint32_t)__shfl((int)v, src, KVP_WAVE); };
            take(gp.vw); take(gp.pw); take(gp.ww); take(gp.xw); take(gp.vpw); take(gp.xpw);
#pragma unroll
            for (int j = 0; j < NP; j++) take(gp.aw[j]);
            take(oc); take(C1.x); take(C1.y); take(C1.z); take(C1.w); take(acc1); take(wr);
        } else {
            // an edge at the far end of a long span: a second round trip
            gp = request_page<NP>(q, X, l, nc, wp);
            oc = occ[nc];
            C1 = *(const uint4 *)(cnt + ((size_t)l * N + nc) * 4);
            acc1 = q.acc[(size_t)l * N + nc];
            wr = q.wr[nc];
            arrive(gp);
        }
        P = page_bits<NP>(q, gp, nc, inb, bp);
        judge();
        if (d < 0) {
            const bool target = lane == 1 || (lane == 0 && d == -2 && it >= 2);   // steps hold a, take not(a)
            if (!a) {
                const uint64_t full = ballot64(target && !room);
                const int hs = full ? msb64(full) : -1;
                f1 = target && lane > hs;
                clipped = full != 0;
            } else {
                f1 = target;
            }
        } else {
            const bool target = lane == 2 || (lane == 3 && d == 2 && inb && P.pm);
            const bool differ = target && (P.x != a);
            if (a) {
                const uint64_t stop = ballot64(differ && !room);
                const int fs = stop ? ctz64(stop) : 64;
                f1 = differ && lane < fs;
                clipped = stop != 0;
            } else {
                f1 = differ;
            }
        }
    }
    const uint64_t flip1 = ballot64(f1), flip2 = ballot64(f2);
    if (!flip1) return R;

    // ---- cost change over the window [base, base + 64): all from registers -----
    const bool fp1 = lane > 0 && ((flip1 >> (lane - 1)) & 1ull);
    const bool fp2 = lane > 0 && ((flip2 >> (lane - 1)) & 1ull);
    double dd = 0.0;
    const bool touch1 = inb && (f1 || fp1 || (same_layer && (f2 || fp2)));
    if (touch1) {
        const double t_old = step_time(q, C1.x, C1.y, C1.z, C1.w, acc1, wr);
        int hr = (int)C1.x, hw = (int)C1.y, mi = (int)C1.z, mo = (int)C1.w;
        page_effect(P, P.x != f1, P.xprev != fp1, hr, hw, mi, mo);
        if (same_layer && (f2 || fp2)) page_effect(Q, Q.x != f2, Q.xprev != fp2, hr, hw, mi, mo);
        R.c1 = make_uint4((uint32_t)hr, (uint32_t)hw, (uint32_t)mi, (uint32_t)mo);
        dd = step_time(q, R.c1.x, R.c1.y, R.c1.z, R.c1.w, acc1, wr) - t_old;
    }
    double dT = wave_tree_sum_f64(dd);
    const bool second = flip2 != 0 && !same_layer;
    bool touch2 = false;
    if (second) {
        dd = 0.0;
        touch2 = inb && (f2 || fp2);
        if (touch2) {
            const double t_old = step_time(q, C2.x, C2.y, C2.z, C2.w, acc2, wr);
            int hr = (int)C2.x, hw = (int)C2.y, mi = (int)C2.z, mo = (int)C2.w;
            page_effect(Q, Q.x != f2, Q.xprev != fp2, hr, hw, mi, mo);
            R.c2 = make_uint4((uint32_t)hr, (uint32_t)hw, (uint32_t)mi, (uint32_t)mo);
            dd = step_time(q, R.c2.x, R.c2.y, R.c2.z, R.c2.w, acc2, wr) - t_old;
        }
        dT = dT + wave_tree_sum_f64(dd);
    }
    R.verdict = clipped ? KVP_MOVE_CLIPPED : KVP_MOVE_OK;
    R.dT = dT; R.base = base; R.flip1 = flip1; R.flip2 = flip2; R.second = second;
    R.n = inb ? n : -1; R.f1 = f1; R.f2 = f2; R.touch1 = touch1; R.touch2 = touch2; R.xnew = P.x != f1;
    R.xw1 = gp.xw; R.xw2 = gq.xw; R.oc = oc;
    return R;
}

// Both halves in one go.  `meanwhile` is run once, after the move's loads have been issued and
// before anything waits for them: work that does not depend on the schedule (drawing the next
// proposal) then costs no time of its own.
template <int NP, class F>
__device__ __forceinline__ MoveEval eval_move(const DevProblem &q, const uint32_t *X, const uint32_t *cnt,
                                              const uint32_t *occ, const kvp_move &m, int lane, F meanwhile) {
    MoveLoads<NP> Ld = issue_move<NP>(q, X, cnt, occ, m, lane);
    meanwhile();
    return finish_move<NP>(q, X, cnt, occ, m, lane, Ld);
}

// ---- kvp_delta_score -----------------------------------------------------------
template <int NP>
__global__ __launch_bounds__(256) void delta_kernel(DevProblem q, const uint32_t *__restrict__ X, uint32_t S,
                                                    const kvp_move *__restrict__ moves,
                                                    const uint32_t *__restrict__ cnt,
                                                    const uint32_t *__restrict__ occ, double *__restrict__ delta,
                                                    int32_t *__restrict__ verdict) {
    const uint32_t s = blockIdx.x * (blockDim.x / KVP_WAVE) + threadIdx.x / KVP_WAVE;
    if (s >= S) return;                                    // whole wavefronts leave together
    const int lane = lane_id();
    const size_t rows = (size_t)q.L * q.N;
    kvp_move m = moves[s];
    const MoveEval R = eval_move<NP>(q, X + (size_t)s * rows * q.Wd, cnt + (size_t)s * rows * 4,
                                 occ + (size_t)s * q.N, m, lane, [] {});
    if (lane == 0) { delta[s] = R.dT; verdict[s] = R.verdict; }
}

extern "C" int kvp_delta_score(kvp_ctx *ctx, const uint32_t *d_placements, uint32_t S, const kvp_move *d_moves,
                               const uint32_t *d_counters, const uint32_t *d_occ, double *d_delta,
                               int32_t *d_verdict) {
    if (!ctx) return KVP_EINVAL;
    if (!ctx->has_trace) return KVP_ENOTRACE;
    if (S == 0) return KVP_OK;
    if (!d_placements || !d_moves || !d_delta || !d_verdict) return KVP_EINVAL;
    if (((uintptr_t)d_placements & 15u) || ((uintptr_t)d_counters & 15u) || ((uintptr_t)d_moves & 3u) ||
        ((uintptr_t)d_delta & 7u) || ((uintptr_t)d_verdict & 3u) || ((uintptr_t)d_occ & 3u))
        return KVP_EINVAL;
    KVP_HIP(hipSetDevice(ctx->device));
    const DevProblem &q = ctx->dp;
    if (!d_counters || !d_occ) {
        // no counters from the caller: one scoring pass produces them
        int rc;
        const size_t rows = (size_t)q.L * q.N;
        if ((rc = kvp_ensure(ctx, (void **)&ctx->d_cnt_tmp, &ctx->cnt_tmp_cap, (size_t)S * rows * 16 + (size_t)S * 16))) return rc;
        if ((rc = kvp_ensure(ctx, (void **)&ctx->d_occ_tmp, &ctx->occ_tmp_cap, (size_t)S * q.N * 4))) return rc;
        // cost/excess of that pass are not wanted: park them behind the counters
        double *junk_cost = (double *)(ctx->d_cnt_tmp + (size_t)S * rows * 4);
        uint32_t *junk_ex = (uint32_t *)(junk_cost + S);
        if ((rc = kvp_score_launch(ctx, d_placements, S, junk_cost, junk_ex, ctx->d_cnt_tmp, ctx->d_occ_tmp))) return rc;
        d_counters = ctx->d_cnt_tmp; d_occ = ctx->d_occ_tmp;
    }
    const dim3 grid((S + 3) / 4), block(256);
    if (q.pn == 1) delta_kernel<1><<<grid, block, 0, ctx->stream>>>(q, d_placements, S, d_moves, d_counters, d_occ, d_delta, d_verdict);
    else if (q.pn <= 4) delta_kernel<4><<<grid, block, 0, ctx->stream>>>(q, d_placements, S, d_moves, d_counters, d_occ, d_delta, d_verdict);
    else delta_kernel<KVP_MAX_PLANES><<<grid, block, 0, ctx->stream>>>(q, d_placements, S, d_moves, d_counters, d_occ, d_delta, d_verdict);
    KVP_HIP(hipGetLastError());
    return KVP_OK;
}

// ---- Philox4x32-10 (Salmon et al., SC'11), counter-based ----------------------
__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0,
                                              uint32_t k1, uint32_t out[4]) {
#pragma unroll
    for (int r = 0; r < 10; r++) {
        const uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
        const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
        const uint32_t t0 = hi1 ^ c1 ^ k0, t2 = hi0 ^ c3 ^ k1;
        c0 = t0; c1 = lo1; c2 = t2; c3 = lo0;
        k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// Proposal number `mi` of chain `chain` is made of three Philox blocks on counters
// (mi, chain, stream0 + {0,1,2}).  A wavefront computes the blocks of sixteen consecutive proposals
// at once, lane 4 j + t the block t of proposal first + j (the fourth lane of a group idles), and a
// proposal is then read out of the three lanes that hold it: the generator costs one pass of ten
// rounds per sixteen proposals instead of three per proposal.
constexpr uint32_t DRAW_BATCH = 16;

struct DrawBatch {
    uint32_t o0, o1, o2, o3;    // per lane: the four words of its block
    uint64_t first;             // uniform: the proposal of lanes 0..3
};

__device__ __forceinline__ void fill_draws(const SAParams &sp, uint32_t chain, uint64_t first, uint32_t stream0,
                                           int lane, DrawBatch &B) {
    const uint64_t mi = first + (uint32_t)(lane >> 2);
    uint32_t out[4];
    philox4x32_10((uint32_t)mi, (uint32_t)(mi >> 32), chain, stream0 + ((uint32_t)lane & 3u), sp.seed_lo, sp.seed_hi, out);
    B.o0 = out[0]; B.o1 = out[1]; B.o2 = out[2]; B.o3 = out[3];
    B.first = first;
}

// u is uniform on (0,1) with 52 random bits.  mi must lie in [B.first, B.first + DRAW_BATCH).
__device__ __forceinline__ void take_move(const DevProblem &q, const SAParams &sp, const DrawBatch &B, uint64_t mi,
                                          kvp_move &m, double &u) {
    const int j = (int)(uint32_t)(mi - B.first) * 4;
    auto word = [&](uint32_t v, int at) { return (uint32_t)__builtin_amdgcn_readlane((int)v, at); };
    const uint32_t a0 = word(B.o0, j), a1 = word(B.o1, j), a2 = word(B.o2, j), a3 = word(B.o3, j);
    const uint32_t b0 = word(B.o0, j + 1), b1 = word(B.o1, j + 1), b2 = word(B.o2, j + 1), b3 = word(B.o3, j + 1);
    const uint32_t c0 = word(B.o0, j + 2), c1 = word(B.o1, j + 2);
    m.op = ((uint64_t)a0 < sp.th0) ? KVP_OP_SET : ((uint64_t)a0 < sp.th1) ? KVP_OP_SWAP : KVP_OP_SHIFT;
    m.layer = __umulhi(a1, q.L);
    m.page = __umulhi(a2, q.P);
    m.n1 = __umulhi(a3, q.N);
    m.len = 1 + __umulhi(b0, sp.max_len);
    m.layer2 = __umulhi(b1, q.L);
    m.page2 = __umulhi(b2, q.P);
    m.dsel = b3 >> 30;
    const uint64_t bits = ((uint64_t)c0 << 20) | (uint64_t)(c1 >> 12);
    u = ((double)bits + 0.5) * (1.0 / 4503599627370496.0);
    // The draw is complete HERE: it keeps its place among the other pinned statements (the point
    // where a move's loads are waited for), instead of drifting behind that wait.
    asm volatile("" : "+s"(m.op), "+s"(m.layer), "+s"(m.page), "+s"(m.n1), "+s"(m.len), "+s"(m.layer2), "+s"(m.page2),
                 "+s"(m.dsel), "+v"(u));
}

// proposal mi, refilling the batch when mi has run past it
__device__ __forceinline__ void next_move(const DevProblem &q, const SAParams &sp, uint32_t chain, uint32_t stream0,
                                          int lane, DrawBatch &B, uint64_t mi, kvp_move &m, double &u) {
    if (mi - B.first >= DRAW_BATCH) fill_draws(sp, chain, mi, stream0, lane, B);
    take_move(q, sp, B, mi, m, u);
}

// Write an accepted move into the chain's schedule, counters and occupancy.  Every lane owns one
// step of the window, so no two lanes write the same word; the new words are made from the ones the
// move was priced on, so nothing is read back from memory here.
template <bool SLOT = false>
__device__ __forceinline__ void apply_move(const DevProblem &q, uint32_t *X, uint32_t *cnt, uint32_t *occ,
                                           const kvp_move &m, const MoveEval &R, uint32_t *slot = nullptr) {
    const bool same_word = m.layer == m.layer2 && (m.page >> 5) == (m.page2 >> 5);
    uint32_t w1 = R.xw1, w2 = R.xw2;
    if (R.f1) w1 ^= 1u << (m.page & 31);
    if (R.f2) { if (same_word) w1 ^= 1u << (m.page2 & 31); else w2 ^= 1u << (m.page2 & 31); }
    if (R.f1 || (R.f2 && same_word)) X[((size_t)m.layer * q.N + R.n) * q.Wd + (m.page >> 5)] = w1;
    if (R.f2 && !same_word) X[((size_t)m.layer2 * q.N + R.n) * q.Wd + (m.page2 >> 5)] = w2;
    if (R.touch1) *(uint4 *)(cnt + ((size_t)m.layer * q.N + R.n) * 4) = R.c1;
    if (R.touch2) *(uint4 *)(cnt + ((size_t)m.layer2 * q.N + R.n) * 4) = R.c2;
    if (R.f1 && !R.f2) occ[R.n] = R.oc + (R.xnew ? 1u : 0xFFFFFFFFu);
    if (SLOT) {
        // the table of the pool after every slot: a lane's step n gains or loses the page in the slots
        // l' >= layer from its own flip and in the slots l' < layer from the flip of the step before
        // (the bit of step n - 1 is still held there if the page persists into n); the same for the victim.
        const int lane = lane_id();
        const uint64_t xn = ballot64(R.xnew);
        const bool fp1 = lane > 0 && ((R.flip1 >> (lane - 1)) & 1ull), fp2 = lane > 0 && ((R.flip2 >> (lane - 1)) & 1ull);
        if (R.n >= 0 && (R.f1 || R.f2 || fp1 || fp2)) {
            const uint32_t n = (uint32_t)R.n;
            const bool pers_p = (q.Pm[(size_t)n * q.Wd + (m.page >> 5)] >> (m.page & 31)) & 1u;
            const bool pers_q = (q.Pm[(size_t)n * q.Wd + (m.page2 >> 5)] >> (m.page2 & 31)) & 1u;
            const int own1 = R.f1 ? (R.xnew ? 1 : -1) : 0, own2 = R.f2 ? -1 : 0;
            const int prev1 = fp1 && pers_p ? (((xn >> (lane - 1)) & 1ull) ? 1 : -1) : 0, prev2 = fp2 && pers_q ? -1 : 0;
            for (uint32_t lp = 0; lp < q.L; lp++) {
                const int dl = (lp >= m.layer ? own1 : prev1) + (lp >= m.layer2 ? own2 : prev2);
                if (dl) slot[(size_t)lp * q.N + n] += (uint32_t)dl;
            }
        }
    }
}

// ---- the annealing loop: one wavefront per chain --------------------------------
template <int NP, bool SLOT = false>
__global__ __launch_bounds__(KVP_WAVE) void anneal_kernel(DevProblem q, SAParams sp, uint32_t *__restrict__ Xall,
                                                          uint32_t *__restrict__ cnt_all,
                                                          uint32_t *__restrict__ occ_all,
                                                          ChainState *__restrict__ states,
                                                          uint32_t *__restrict__ log_all, uint64_t log_cap,
                                                          uint64_t move_begin, uint64_t move_end, int calibrate,
                                                          uint32_t *slot_all = nullptr) {
    const uint32_t chain = blockIdx.x;
    uint32_t *slot = SLOT ? slot_all + (size_t)chain * q.L * q.N : nullptr;
    const int lane = (int)threadIdx.x;
    const size_t rows = (size_t)q.L * q.N;
    uint32_t *X = Xall + (size_t)chain * rows * q.Wd;
    uint32_t *cnt = cnt_all + (size_t)chain * rows * 4;
    uint32_t *occ = occ_all + (size_t)chain * q.N;
    uint32_t *log = log_all + (size_t)chain * log_cap * LOG_WORDS;
    ChainState st = states[chain];
    // values that only ever enter vector arithmetic or per-lane addresses are moved to vector registers:
    // the scalar file is the scarce one here, and what does not fit in it is spilled and re-read every move
    asm volatile("" : "+v"(q.unit_b), "+v"(q.page_b), "+v"(q.token_b), "+v"(q.inv_bh), "+v"(q.inv_bk), "+v"(q.inv_bd),
                 "+v"(q.inv_min));
    asm volatile("" : "+v"(q.V), "+v"(q.Pm), "+v"(q.Wm), "+v"(q.acc), "+v"(q.wr), "+v"(q.pl), "+v"(X), "+v"(cnt), "+v"(occ));
    asm volatile("" : "+v"(st.t_cur), "+v"(st.t_best), "+v"(st.c), "+v"(st.c0), "+v"(sp.alpha));
    asm volatile("" : "+v"(st.accepted), "+v"(st.uphill), "+v"(st.null_moves), "+v"(st.clipped), "+v"(st.improved),
                 "+v"(st.moves_done), "+v"(log));

    if (calibrate) {
        // initial temperature from the target acceptance p0 of uphill moves:
        // C0 = mean(dT | dT > 0) / (-ln p0) over proposals that are not applied
        double sum = 0.0;
        uint32_t k = 0;
        kvp_move m, mn; double u, un;
        DrawBatch B;
        fill_draws(sp, chain, 0, 8, lane, B);
        take_move(q, sp, B, 0, m, u);
        for (uint64_t j = 0; j < CALIB_MOVES; j++) {
            MoveLoads<NP> Ld = issue_move<NP>(q, X, cnt, occ, m, lane);
            next_move(q, sp, chain, 8, lane, B, j + 1, mn, un);
            const MoveEval R = finish_move<NP, false, SLOT>(q, X, cnt, occ, m, lane, Ld, slot);
            m = mn;
            if (R.verdict != KVP_MOVE_NULL && R.dT > 0.0) { sum = sum + R.dT; k++; }
        }
        st.c0 = k ? (sum / (double)k) / sp.neg_ln_p0 : 0.0;
        st.c = st.c0;
        st.level = 0;
    }

    // Two proposals are in the pipeline: while move mi is priced from words that were requested one
    // iteration ago, the words of move mi + 1 are already on their way (proposals depend on the move
    // number, chain and seed only, never on the schedule).  When move mi is accepted and what it
    // writes may be among the words requested for mi + 1, they are requested again after the writes.
    kvp_move m_cur, m_nxt;
    double u_cur, u_nxt;
    DrawBatch B;
    fill_draws(sp, chain, move_begin, 0, lane, B);
    take_move(q, sp, B, move_begin, m_cur, u_cur);
    MoveLoads<NP> Lc = issue_move<NP>(q, X, cnt, occ, m_cur, lane);
    for (uint64_t mi = move_begin; mi < move_end; mi++) {
        uint64_t lvl = mi / sp.mpl;
        if (lvl > sp.n_levels - 1) lvl = sp.n_levels - 1;
        while (st.level < lvl) { st.c = st.c * sp.alpha; st.level++; }      // geometric cooling
        next_move(q, sp, chain, 0, lane, B, mi + 1, m_nxt, u_nxt);
        MoveLoads<NP> Ln = issue_move<NP>(q, X, cnt, occ, m_nxt, lane);
        const kvp_move m = m_cur;
        const double u = u_cur;
        const MoveEval R = finish_move<NP, false, SLOT>(q, X, cnt, occ, m, lane, Lc, slot);
        st.moves_done++;
        bool accept = false;
        if (R.verdict == KVP_MOVE_NULL) {
            st.null_moves++;
        } else {
            if (R.verdict == KVP_MOVE_CLIPPED) st.clipped++;
            accept = (R.dT <= 0.0) || (st.c > 0.0 && u < exp(-R.dT / st.c));   // Metropolis
        }
        if (accept) {
            st.accepted++;
            if (R.dT > 0.0) st.uphill++;
            apply_move<SLOT>(q, X, cnt, occ, m, R, slot);
            st.t_cur = st.t_cur + R.dT;
            // edits since the best schedule, so that it can be rebuilt by undoing them (not while the best
            // schedule is held as a snapshot: then nothing leads back to it but the snapshot itself)
            if (st.best_saved) {
            } else if (st.log_len < log_cap) {
                if (lane < LOG_WORDS) {
                    uint32_t w;
                    switch (lane) {
                        case 0: w = m.layer; break;
                        case 1: w = m.page; break;
                        case 2: w = m.layer2; break;
                        case 3: w = m.page2; break;
                        case 4: w = (uint32_t)R.base; break;
                        case 5: w = (uint32_t)R.flip1; break;
                        case 6: w = (uint32_t)(R.flip1 >> 32); break;
                        case 7: w = (uint32_t)R.flip2; break;
                        case 8: w = (uint32_t)(R.flip2 >> 32); break;
                        default: w = 0; break;
                    }
                    log[st.log_len * LOG_WORDS + lane] = w;
                }
                st.log_len++;
            } else {
                st.log_overflow = 1;
            }
            if (st.t_cur < st.t_best) { st.t_best = st.t_cur; st.improved++; st.log_len = 0; st.best_saved = 0; }
            // Later proposals read, from other lanes, what this one wrote.  The chain is one wavefront:
            // its memory instructions reach the cache in program order, so a fence of wavefront scope
            // (no wait; it only keeps the compiler from moving accesses across) is all that is needed.
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            // Written: schedule words and counter rows of the move's layers, and the occupancy, at
            // steps [base + first flip, base + last flip + 1].  Requested for the next move: rows
            // n1 - 1 .. n1 + 63 of its layers and the occupancy of those steps.
            const uint64_t fl = R.flip1 | R.flip2;
            const int w_lo = R.base + ctz64(fl), w_hi = R.base + msb64(fl) + 1;
            const int r_lo = (int)m_nxt.n1 - 1, r_hi = (int)m_nxt.n1 + 63;
            if (w_lo <= r_hi && w_hi >= r_lo) Ln = issue_move<NP>(q, X, cnt, occ, m_nxt, lane);
        }
        Lc = Ln;
        m_cur = m_nxt; u_cur = u_nxt;
    }
    if (lane == 0) states[chain] = st;
}

// ---- the annealing loop, several proposals per round ---------------------------------
// A chain is a serial walk, but its proposals are known in advance (they depend on the move number,
// the chain and the seed only) and most are rejected.  SPEC wavefronts therefore price the next SPEC
// proposals against the same schedule at once; the walk then takes them in order up to and including
// the first one that is accepted (everything before it was rejected, so it was priced on the right
// schedule), that wavefront applies its move, and the next round starts behind it.  The walk is the
// serial one, move for move; a round costs one memory round trip and one pricing for 1/a proposals or
// so at acceptance rate a.  Every wavefront keeps a copy of the chain's running state and updates it
// alike from what the round's wavefronts publish in LDS.

__device__ __forceinline__ int uniform_i32(int v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ double uniform_f64(double v) {
    return __hiloint2double(__builtin_amdgcn_readfirstlane(__double2hiint(v)),
                            __builtin_amdgcn_readfirstlane(__double2loint(v)));
}

template <int NP, int SPEC>
__global__ __launch_bounds__(SPEC * KVP_WAVE) void anneal_rounds_kernel(
    DevProblem q, SAParams sp, uint32_t *__restrict__ Xall, uint32_t *__restrict__ cnt_all,
    uint32_t *__restrict__ occ_all, ChainState *__restrict__ states, uint32_t *__restrict__ log_all, uint64_t log_cap,
    uint64_t move_begin, uint64_t move_end) {
    // The chain's occupancy per token step lives in LDS for the launch: every accepted move changes it
    // over its span, so it is the one thing that proposals requested ahead would nearly always find
    // changed; from LDS it is read when a proposal is priced, not when its words are requested.
    extern __shared__ uint32_t s_occ[];
    // what the round's wavefronts publish, in two sets used in turn (a set is still being read when
    // the next round's is written)
    __shared__ double s_dT[2][SPEC];
    __shared__ int s_verdict[2][SPEC], s_accept[2][SPEC], s_wlo[2][SPEC], s_whi[2][SPEC], s_l1[2][SPEC], s_l2[2][SPEC];
    const uint32_t chain = blockIdx.x;
    const int lane = lane_id();
    const int w = uniform_i32((int)(threadIdx.x / KVP_WAVE));
    const size_t rows = (size_t)q.L * q.N;
    uint32_t *X = Xall + (size_t)chain * rows * q.Wd;
    uint32_t *cnt = cnt_all + (size_t)chain * rows * 4;
    uint32_t *occ = occ_all + (size_t)chain * q.N;
    uint32_t *log = log_all + (size_t)chain * log_cap * LOG_WORDS;
    ChainState st = states[chain];
    // values that only ever enter vector arithmetic or per-lane addresses are moved to vector registers:
    // the scalar file is the scarce one here, and what does not fit in it is spilled and re-read every move
    asm volatile("" : "+v"(q.unit_b), "+v"(q.page_b), "+v"(q.token_b), "+v"(q.inv_bh), "+v"(q.inv_bk), "+v"(q.inv_bd),
                 "+v"(q.inv_min));
    asm volatile("" : "+v"(q.V), "+v"(q.Pm), "+v"(q.Wm), "+v"(q.acc), "+v"(q.wr), "+v"(q.pl), "+v"(X), "+v"(cnt));
    asm volatile("" : "+v"(st.t_cur), "+v"(st.t_best), "+v"(st.c), "+v"(st.c0), "+v"(sp.alpha));
    asm volatile("" : "+v"(st.accepted), "+v"(st.uphill), "+v"(st.null_moves), "+v"(st.clipped), "+v"(st.improved),
                 "+v"(st.moves_done), "+v"(log));
    for (uint32_t i = threadIdx.x; i < q.N; i += SPEC * KVP_WAVE) s_occ[i] = occ[i];
    __syncthreads();
    DrawBatch B;
    B.first = ~0ull - DRAW_BATCH;                                      // empty: the first proposal fills it
    B.o0 = B.o1 = B.o2 = B.o3 = 0;
    auto level_of = [&](uint64_t mi) {
        const uint64_t lvl = mi / sp.mpl;
        return (uint32_t)(lvl > sp.n_levels - 1 ? sp.n_levels - 1 : lvl);
    };
    uint64_t mi = move_begin;
    kvp_move m; double u;
    m.op = m.layer = m.page = m.n1 = m.layer2 = m.page2 = m.dsel = 0; m.len = 1; u = 0.5;
    MoveLoads<NP> Ld;
    if (mi < move_end) {
        next_move(q, sp, chain, 0, lane, B, mi + (uint32_t)w < move_end ? mi + (uint32_t)w : mi, m, u);
        Ld = issue_move<NP, true>(q, X, cnt, nullptr, m, lane);
    }
    uint32_t set = 0;
    while (mi < move_end) {                                            // the same trip count in every wavefront
        const uint64_t my = mi + (uint32_t)w;
        const bool valid = my < move_end;
        // temperature of this proposal: geometric cooling, continued from the chain's state
        double c = st.c;
        for (uint32_t lev = st.level, to = level_of(my); lev < to; lev++) c = c * sp.alpha;
        const MoveEval R = finish_move<NP, true>(q, X, cnt, s_occ, m, lane, Ld);
        bool accept = false;
        if (valid && R.verdict != KVP_MOVE_NULL) accept = (R.dT <= 0.0) || (c > 0.0 && u < exp(-R.dT / c));   // Metropolis
        if (lane == 0) {
            s_dT[set][w] = R.dT; s_verdict[set][w] = valid ? R.verdict : -1; s_accept[set][w] = accept ? 1 : 0;
            // what the move writes if it is the one applied: schedule words and counter rows of its
            // layers at steps [base + first flip, base + last flip + 1]
            const uint64_t fl = R.flip1 | R.flip2;
            s_wlo[set][w] = fl ? R.base + ctz64(fl) : 0;
            s_whi[set][w] = fl ? R.base + msb64(fl) + 1 : -1;
            s_l1[set][w] = (int)m.layer;
            s_l2[set][w] = R.flip2 ? (int)m.layer2 : (int)m.layer;
        }
        __syncthreads();
        // the proposals of this round that the walk reaches
        int f = SPEC;
        uint32_t reached = 0;
#pragma unroll
        for (int k = 0; k < SPEC; k++) {
            const int v = uniform_i32(s_verdict[set][k]), acc = uniform_i32(s_accept[set][k]);
            if (f == SPEC && v >= 0 && reached == (uint32_t)k) {
                reached++;
                st.moves_done++;
                if (v == KVP_MOVE_NULL) st.null_moves++;
                else {
                    if (v == KVP_MOVE_CLIPPED) st.clipped++;
                    if (acc) f = k;
                }
            }
        }
        if (f < SPEC) {
            const double dT = uniform_f64(s_dT[set][f]);
            st.accepted++;
            if (dT > 0.0) st.uphill++;
            if (w == f) {
                apply_move(q, X, cnt, s_occ, m, R);
                // edits since the best schedule, so that it can be rebuilt by undoing them
                if (!st.best_saved && st.log_len < log_cap && lane < LOG_WORDS) {
                    uint32_t e;
                    switch (lane) {
                        case 0: e = m.layer; break;
                        case 1: e = m.page; break;
                        case 2: e = m.layer2; break;
                        case 3: e = m.page2; break;
                        case 4: e = (uint32_t)R.base; break;
                        case 5: e = (uint32_t)R.flip1; break;
                        case 6: e = (uint32_t)(R.flip1 >> 32); break;
                        case 7: e = (uint32_t)R.flip2; break;
                        case 8: e = (uint32_t)(R.flip2 >> 32); break;
                        default: e = 0; break;
                    }
                    log[st.log_len * LOG_WORDS + lane] = e;
                }
            }
            st.t_cur = st.t_cur + dT;
            if (st.best_saved) {}
            else if (st.log_len < log_cap) st.log_len++;
            else st.log_overflow = 1;
            if (st.t_cur < st.t_best) { st.t_best = st.t_cur; st.improved++; st.log_len = 0; st.best_saved = 0; }
        }
        // the cooling state as the last proposal reached leaves it
        for (const uint32_t to = level_of(mi + reached - 1); st.level < to; st.level++) st.c = st.c * sp.alpha;
        mi += reached;
        // The next round's proposal and its words, requested while the accepted move is on its way to
        // memory: the two round trips overlap.
        const bool more = mi < move_end;
        if (more) {
            next_move(q, sp, chain, 0, lane, B, mi + (uint32_t)w < move_end ? mi + (uint32_t)w : mi, m, u);
            Ld = issue_move<NP, true>(q, X, cnt, nullptr, m, lane);
        }
        __syncthreads();        // this round's writes are in memory (and the occupancy in LDS) for every wavefront
        // words requested before an accepted move that writes among them are requested again
        if (more && f < SPEC && w != f) {
            const int w_lo = uniform_i32(s_wlo[set][f]), w_hi = uniform_i32(s_whi[set][f]);
            const int a1 = uniform_i32(s_l1[set][f]), a2 = uniform_i32(s_l2[set][f]);
            const int r_lo = (int)m.n1 - 1, r_hi = (int)m.n1 + 63;
            const int b1 = (int)m.layer, b2 = m.op == KVP_OP_SWAP ? (int)m.layer2 : (int)m.layer;
            if (w_lo <= r_hi && w_hi >= r_lo && (b1 == a1 || b1 == a2 || b2 == a1 || b2 == a2))
                Ld = issue_move<NP, true>(q, X, cnt, nullptr, m, lane);
        }
        set ^= 1u;
    }
    __syncthreads();
    for (uint32_t i = threadIdx.x; i < q.N; i += SPEC * KVP_WAVE) occ[i] = s_occ[i];
    if (threadIdx.x == 0) states[chain] = st;
}

// Apply (or, applied twice, undo) every logged edit of every chain: XOR commutes,
// so one wavefront per log entry and atomics on the words are enough.
// Only chains whose log holds more than `longer_than` entries take part.
__global__ __launch_bounds__(256) void log_xor_kernel(DevProblem q, uint32_t *__restrict__ Xall,
                                                      const ChainState *__restrict__ states,
                                                      const uint32_t *__restrict__ log_all, uint64_t log_cap,
                                                      uint32_t chain0, uint64_t longer_than) {
    const uint32_t chain = chain0 + blockIdx.y;
    const int lane = lane_id();
    const uint64_t n_entries = states[chain].log_len;
    if (n_entries <= longer_than) return;
    const size_t rows = (size_t)q.L * q.N;
    uint32_t *X = Xall + (size_t)chain * rows * q.Wd;
    const uint32_t *log = log_all + (size_t)chain * log_cap * LOG_WORDS;
    const uint64_t wave0 = (uint64_t)blockIdx.x * (blockDim.x / KVP_WAVE) + threadIdx.x / KVP_WAVE;
    const uint64_t nwaves = (uint64_t)gridDim.x * (blockDim.x / KVP_WAVE);
    for (uint64_t e = wave0; e < n_entries; e += nwaves) {
        const uint32_t *r = log + e * LOG_WORDS;
        const uint32_t l = r[0], p = r[1], l2 = r[2], pq = r[3];
        const int n = (int)r[4] + lane;
        const uint64_t f1 = (uint64_t)r[5] | ((uint64_t)r[6] << 32), f2 = (uint64_t)r[7] | ((uint64_t)r[8] << 32);
        if (n < 0 || n >= (int)q.N) continue;
        if ((f1 >> lane) & 1ull) atomicXor(&X[((size_t)l * q.N + n) * q.Wd + (p >> 5)], 1u << (p & 31));
        if ((f2 >> lane) & 1ull) atomicXor(&X[((size_t)l2 * q.N + n) * q.Wd + (pq >> 5)], 1u << (pq & 31));
    }
}

// Bounding the log: a chain whose log has grown beyond `soft` entries gets its best schedule written out
// (a copy of the current one, the logged edits undone by log_xor_kernel) and starts its log afresh.
__global__ __launch_bounds__(256) void snapshot_copy_kernel(const uint32_t *__restrict__ Xall, uint32_t *__restrict__ Xbest,
                                                            const ChainState *__restrict__ states, size_t per,
                                                            uint64_t soft) {
    const uint32_t chain = blockIdx.y;
    if (states[chain].log_len <= soft) return;
    const uint32_t *src = Xall + (size_t)chain * per;
    uint32_t *dst = Xbest + (size_t)chain * per;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < per; i += (size_t)gridDim.x * 256) dst[i] = src[i];
}
__global__ void snapshot_commit_kernel(ChainState *states, uint32_t C, uint64_t soft) {
    const uint32_t c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= C || states[c].log_len <= soft) return;
    states[c].log_len = 0;
    states[c].best_saved = 1;
}
// Chains whose best schedule is a snapshot: exchange it with the current one (applied twice: back again).
__global__ __launch_bounds__(256) void snapshot_swap_kernel(uint32_t *__restrict__ Xall, uint32_t *__restrict__ Xbest,
                                                            const ChainState *__restrict__ states, size_t per,
                                                            uint32_t chain0) {
    const uint32_t chain = chain0 + blockIdx.y;
    if (!states[chain].best_saved) return;
    uint32_t *a = Xall + (size_t)chain * per, *b = Xbest + (size_t)chain * per;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < per; i += (size_t)gridDim.x * 256) {
        const uint32_t t = a[i]; a[i] = b[i]; b[i] = t;
    }
}

__global__ void init_states_kernel(ChainState *states, const double *cost, uint32_t C) {
    const uint32_t c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= C) return;
    ChainState s;
    memset(&s, 0, sizeof s);
    s.t_cur = cost[c]; s.t_best = cost[c];
    states[c] = s;
}

// Starting schedules: copy (one per chain, or one for all) and keep existing pages only.
__global__ __launch_bounds__(256) void init_copy_kernel(DevProblem q, uint32_t *__restrict__ X,
                                                        const uint32_t *__restrict__ src, uint32_t C, int broadcast) {
    const size_t per = (size_t)q.L * q.N * q.Wd;
    const size_t total = per * C;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
        const size_t j = i % per;
        const size_t nw = j % ((size_t)q.N * q.Wd);
        X[i] = src[broadcast ? j : i] & q.V[nw];
    }
}

// Lowest cost, ties to the lowest chain id.  One workgroup.
__global__ __launch_bounds__(256) void argmin_kernel(const double *__restrict__ cost, uint32_t C,
                                                     uint32_t *__restrict__ out) {
    __shared__ double sv[256];
    __shared__ uint32_t si[256];
    double bv = INFINITY; uint32_t bi = 0xFFFFFFFFu;
    for (uint32_t c = threadIdx.x; c < C; c += blockDim.x) {
        const double v = cost[c];
        if (v < bv || (v == bv && c < bi)) { bv = v; bi = c; }
    }
    sv[threadIdx.x] = bv; si[threadIdx.x] = bi;
    __syncthreads();
    for (uint32_t h = 128; h >= 1; h >>= 1) {
        if (threadIdx.x < h) {
            const double v = sv[threadIdx.x + h]; const uint32_t i = si[threadIdx.x + h];
            if (v < sv[threadIdx.x] || (v == sv[threadIdx.x] && i < si[threadIdx.x])) { sv[threadIdx.x] = v; si[threadIdx.x] = i; }
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) out[0] = si[0] == 0xFFFFFFFFu ? 0u : si[0];
}

static bool same_schedule(const kvp_anneal_params &a, const kvp_anneal_params &b) {
    return a.n_chains == b.n_chains && a.n_levels == b.n_levels && a.seed == b.seed &&
           a.total_moves == b.total_moves && a.max_len == b.max_len && a.p0 == b.p0 && a.alpha == b.alpha &&
           a.op_prob[0] == b.op_prob[0] && a.op_prob[1] == b.op_prob[1] && a.op_prob[2] == b.op_prob[2];
}

// current <-> best-so-far schedules of the chains [chain0, chain0 + nchains): the logged edits are XOR-ed in
// (or out again), and a chain whose best schedule is a snapshot exchanges the two
static int launch_log_xor(kvp_ctx *ctx, uint32_t chain0, uint32_t nchains) {
    const size_t per = (size_t)ctx->dp.L * ctx->dp.N * ctx->dp.Wd;
    if (ctx->d_Xbest) {
        snapshot_swap_kernel<<<dim3(64, nchains), dim3(256), 0, ctx->stream>>>(ctx->d_X, ctx->d_Xbest, ctx->d_state, per, chain0);
        KVP_HIP(hipGetLastError());
    }
    log_xor_kernel<<<dim3(64, nchains), dim3(256), 0, ctx->stream>>>(ctx->dp, ctx->d_X, ctx->d_state, ctx->d_log,
                                                                    ctx->log_cap, chain0, 0);
    KVP_HIP(hipGetLastError());
    return KVP_OK;
}

// Bounded log: after a launch, chains whose log has passed the soft limit write their best schedule out.
static int compact_logs(kvp_ctx *ctx, uint32_t C) {
    const size_t per = (size_t)ctx->dp.L * ctx->dp.N * ctx->dp.Wd;
    snapshot_copy_kernel<<<dim3(64, C), dim3(256), 0, ctx->stream>>>(ctx->d_X, ctx->d_Xbest, ctx->d_state, per, ctx->log_soft);
    KVP_HIP(hipGetLastError());
    log_xor_kernel<<<dim3(64, C), dim3(256), 0, ctx->stream>>>(ctx->dp, ctx->d_Xbest, ctx->d_state, ctx->d_log, ctx->log_cap, 0,
                                                              ctx->log_soft);
    KVP_HIP(hipGetLastError());
    snapshot_commit_kernel<<<dim3((C + 255) / 256), dim3(256), 0, ctx->stream>>>(ctx->d_state, C, ctx->log_soft);
    KVP_HIP(hipGetLastError());
    return KVP_OK;
}

extern "C" int kvp_anneal(kvp_ctx *ctx, const kvp_anneal_params *p, const uint32_t *d_init) {
    if (!ctx || !p) return KVP_EINVAL;
    if (!ctx->has_trace) return KVP_ENOTRACE;
    if (p->n_chains > 65535u) return KVP_ESHAPE;             // one grid row per chain when the best schedules are rebuilt
    if (p->n_chains == 0 || p->n_levels == 0 || p->max_len < 1 ||
        p->max_len > KVP_MAX_LEN || !(p->p0 > 0.0 && p->p0 < 1.0) || !(p->alpha > 0.0 && p->alpha <= 1.0) ||
        p->init_mode > KVP_INIT_CONTINUE || p->total_moves == 0)
        return KVP_EINVAL;
    double ps = 0.0;
    for (int i = 0; i < 3; i++) { if (!(p->op_prob[i] >= 0.0)) return KVP_EINVAL; ps += p->op_prob[i]; }
    if (!(ps > 0.0 && ps <= 1.0 + 1e-9)) return KVP_EINVAL;
    if ((p->init_mode == KVP_INIT_GIVEN || p->init_mode == KVP_INIT_BROADCAST) &&
        (!d_init || ((uintptr_t)d_init & 15u)))
        return KVP_EINVAL;
    KVP_HIP(hipSetDevice(ctx->device));
    const DevProblem &q = ctx->dp;
    const uint32_t C = p->n_chains;
    const size_t rows = (size_t)q.L * q.N, per = rows * q.Wd;

    if (p->init_mode == KVP_INIT_CONTINUE) {
        if (!ctx->has_chains) return KVP_ENOCHAINS;
        if (!same_schedule(*p, ctx->sa)) return KVP_EINVAL;
        if (ctx->capacity_mode != ctx->chains_mode) return KVP_EINVAL;   // the chains walk on under the reading they started with
        if (ctx->moves_done + p->moves > p->total_moves) return KVP_EINVAL;
    } else {
        if (p->moves > p->total_moves) return KVP_EINVAL;            // before the previous chains are given up
        KVP_HIP(hipStreamSynchronize(ctx->stream));
        kvp_free_chains(ctx);
        // The log of accepted edits: one entry per move at most, so total_moves entries always suffice.  When
        // that is more than twice what a schedule takes, the log is bounded instead: launches are cut to `soft`
        // moves, and a chain whose log has passed `soft` entries after a launch writes its best schedule out
        // and starts afresh, so 2 * soft entries and one more schedule per chain do, however long the run.
        const uint64_t sched_entries = (uint64_t)(per * 4 / (LOG_WORDS * 4));
        uint64_t soft = ctx->log_entries ? ctx->log_entries : (sched_entries > 16384 ? sched_entries : 16384);
        if (!ctx->log_entries && p->total_moves <= 2 * soft) soft = 0;
        if (soft >= p->total_moves) soft = 0;
        ctx->log_soft = soft;
        ctx->log_cap = soft ? 2 * soft : p->total_moves;
        const struct { void **p; size_t bytes; } want[] = {
            {(void **)&ctx->d_Xbest, soft ? per * C * 4 : 0},
            {(void **)&ctx->d_X, per * C * 4}, {(void **)&ctx->d_cnt, rows * C * 16}, {(void **)&ctx->d_occ, (size_t)q.N * C * 4},
            {(void **)&ctx->d_state, sizeof(ChainState) * C}, {(void **)&ctx->d_log, (size_t)ctx->log_cap * C * LOG_WORDS * 4},
            {(void **)&ctx->d_cost, sizeof(double) * C}, {(void **)&ctx->d_excess, 4 * (size_t)C}, {(void **)&ctx->d_argmin, 16}};
        for (const auto &w : want) {
            if (!w.bytes) continue;
            const hipError_t e = hipMalloc(w.p, w.bytes);
            if (e != hipSuccess) {
                kvp_tls_hip_error = (int)e; kvp_tls_hip_line = __LINE__;
                (void)hipGetLastError();
                kvp_free_chains(ctx);                                    // nothing half-allocated stays behind
                return e == hipErrorOutOfMemory ? KVP_ENOMEM : KVP_EHIP;
            }
        }
        if (p->init_mode == KVP_INIT_EMPTY) {
            KVP_HIP(hipMemsetAsync(ctx->d_X, 0, per * C * 4, ctx->stream));
        } else {
            init_copy_kernel<<<dim3(2048), dim3(256), 0, ctx->stream>>>(q, ctx->d_X, d_init, C,
                                                                       p->init_mode == KVP_INIT_BROADCAST);
            KVP_HIP(hipGetLastError());
        }
        int rc = kvp_score_launch(ctx, ctx->d_X, C, ctx->d_cost, ctx->d_excess, ctx->d_cnt, ctx->d_occ);
        if (rc) { kvp_free_chains(ctx); return rc; }
        uint32_t *hex = (uint32_t *)malloc(4 * (size_t)C);
        if (!hex) { kvp_free_chains(ctx); return KVP_ENOMEM; }
        hipError_t e = hipMemcpyAsync(hex, ctx->d_excess, 4 * (size_t)C, hipMemcpyDeviceToHost, ctx->stream);
        if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
        bool bad = false;
        for (uint32_t c = 0; c < C && e == hipSuccess; c++) bad = bad || (hex[c] & 0x7FFFFFFFu) != 0;
        free(hex);
        if (e != hipSuccess) { kvp_free_chains(ctx); return KVP_EHIP; }
        if (bad) { kvp_free_chains(ctx); return KVP_EINFEASIBLE; }
        if (ctx->capacity_mode == KVP_CAPACITY_PER_SLOT) {
            // the pool after every slot of every chain; a start that overfills a slot is refused
            const hipError_t ea = hipMalloc((void **)&ctx->d_slot, rows * C * 4);
            if (ea != hipSuccess) {
                kvp_tls_hip_error = (int)ea; kvp_tls_hip_line = __LINE__;
                (void)hipGetLastError();
                kvp_free_chains(ctx);
                return ea == hipErrorOutOfMemory ? KVP_ENOMEM : KVP_EHIP;
            }
            rc = kvp_slot_occupancy_launch(ctx, ctx->d_X, C, ctx->d_excess, ctx->d_slot);
            if (rc) { kvp_free_chains(ctx); return rc; }
            hex = (uint32_t *)malloc(4 * (size_t)C);
            if (!hex) { kvp_free_chains(ctx); return KVP_ENOMEM; }
            e = hipMemcpyAsync(hex, ctx->d_excess, 4 * (size_t)C, hipMemcpyDeviceToHost, ctx->stream);
            if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
            for (uint32_t c = 0; c < C && e == hipSuccess; c++) bad = bad || hex[c] != 0;
            free(hex);
            if (e != hipSuccess) { kvp_free_chains(ctx); return KVP_EHIP; }
            if (bad) { kvp_free_chains(ctx); return KVP_EINFEASIBLE; }
        }
        ctx->chains_mode = ctx->capacity_mode;
        init_states_kernel<<<dim3((C + 255) / 256), dim3(256), 0, ctx->stream>>>(ctx->d_state, ctx->d_cost, C);
        KVP_HIP(hipGetLastError());
        ctx->sa = *p;
        ctx->moves_done = 0;
        ctx->has_chains = true;
    }
    SAParams sp;
    sp.seed_lo = (uint32_t)p->seed; sp.seed_hi = (uint32_t)(p->seed >> 32);
    sp.th0 = (uint64_t)(p->op_prob[0] * 4294967296.0);
    sp.th1 = (uint64_t)((p->op_prob[0] + p->op_prob[1]) * 4294967296.0);
    sp.mpl = p->total_moves / p->n_levels; if (sp.mpl < 1) sp.mpl = 1;
    sp.n_levels = p->n_levels; sp.max_len = p->max_len;
    sp.alpha = p->alpha; sp.neg_ln_p0 = -log(p->p0);
    // bounded launches: every wavefront runs a fixed number of moves and exits
    const uint64_t chunk = ctx->log_soft && ctx->log_soft < 16384 ? ctx->log_soft : 16384;
    uint64_t m0 = ctx->moves_done;
    const uint64_t m_end = m0 + p->moves;
    bool first = ctx->moves_done == 0;
    const bool per_slot = ctx->chains_mode == KVP_CAPACITY_PER_SLOT;
    auto launch = [&](uint64_t b, uint64_t e, int calibrate) {
        const dim3 grid(C), block(KVP_WAVE);
        if (per_slot) {
            if (q.pn == 1)
                anneal_kernel<1, true><<<grid, block, 0, ctx->stream>>>(q, sp, ctx->d_X, ctx->d_cnt, ctx->d_occ, ctx->d_state,
                                                                       ctx->d_log, ctx->log_cap, b, e, calibrate, ctx->d_slot);
            else if (q.pn <= 4)
                anneal_kernel<4, true><<<grid, block, 0, ctx->stream>>>(q, sp, ctx->d_X, ctx->d_cnt, ctx->d_occ, ctx->d_state,
                                                                       ctx->d_log, ctx->log_cap, b, e, calibrate, ctx->d_slot);
            else
                anneal_kernel<KVP_MAX_PLANES, true><<<grid, block, 0, ctx->stream>>>(
                    q, sp, ctx->d_X, ctx->d_cnt, ctx->d_occ, ctx->d_state, ctx->d_log, ctx->log_cap, b, e, calibrate, ctx->d_slot);
            return;
        }
        if (q.pn == 1)
            anneal_kernel<1><<<grid, block, 0, ctx->stream>>>(q, sp, ctx->d_X, ctx->d_cnt, ctx->d_occ, ctx->d_state,
                                                             ctx->d_log, ctx->log_cap, b, e, calibrate);
        else if (q.pn <= 4)
            anneal_kernel<4><<<grid, block, 0, ctx->stream>>>(q, sp, ctx->d_X, ctx->d_cnt, ctx->d_occ, ctx->d_state,
                                                             ctx->d_log, ctx->log_cap, b, e, calibrate);
        else
            anneal_kernel<KVP_MAX_PLANES><<<grid, block, 0, ctx->stream>>>(
                q, sp, ctx->d_X, ctx->d_cnt, ctx->d_occ, ctx->d_state, ctx->d_log, ctx->log_cap, b, e, calibrate);
    };
    // Proposals priced per round: four, each by a wavefront of its own, while that leaves every
    // wavefront a SIMD to itself (four SIMDs per compute unit) and while the chains' state stays in
    // the 256 MB last-level cache.  Otherwise the serial loop, one wavefront per chain, is the faster
    // one: with more wavefronts they share SIMDs, and with the state out in HBM a round waits for
    // the slowest of four sets of scattered loads (measured: 512 and 1024 chains; 256 chains of 32 MB).
    int spec = ctx->anneal_lookahead;
    if (spec == 0) {
        const uint64_t state = (uint64_t)C * ((uint64_t)q.L * q.N * ((uint64_t)q.Wd * 4 + 16) + (uint64_t)q.N * 4);
        spec = (uint64_t)C * 4 <= 4ull * ctx->compute_units && state <= (256ull << 20) ? 4 : 1;
    }
    if ((size_t)q.N * 4 > 48 * 1024) spec = 1;                         // the rounds keep the occupancy of all steps in LDS
    if (per_slot) spec = 1;                                            // the per-slot walk is the serial one
    auto launch_rounds = [&](uint64_t b, uint64_t e) {
        const dim3 grid(C), block(4 * KVP_WAVE);
        const size_t lds = (size_t)q.N * 4;                            // the chain's occupancy
        if (q.pn == 1)
            anneal_rounds_kernel<1, 4><<<grid, block, lds, ctx->stream>>>(q, sp, ctx->d_X, ctx->d_cnt, ctx->d_occ, ctx->d_state,
                                                                       ctx->d_log, ctx->log_cap, b, e);
        else if (q.pn <= 4)
            anneal_rounds_kernel<4, 4><<<grid, block, lds, ctx->stream>>>(q, sp, ctx->d_X, ctx->d_cnt, ctx->d_occ, ctx->d_state,
                                                                       ctx->d_log, ctx->log_cap, b, e);
        else
            anneal_rounds_kernel<KVP_MAX_PLANES, 4><<<grid, block, lds, ctx->stream>>>(
                q, sp, ctx->d_X, ctx->d_cnt, ctx->d_occ, ctx->d_state, ctx->d_log, ctx->log_cap, b, e);
    };
    const bool rounds = spec == 4;
    if (first) {                                                       // the initial temperature, once per chain
        launch(0, 0, 1);
        KVP_HIP(hipGetLastError());
    }
    while (m0 < m_end) {
        const uint64_t m1 = m0 + chunk < m_end ? m0 + chunk : m_end;
        if (rounds) launch_rounds(m0, m1);
        else launch(m0, m1, 0);
        KVP_HIP(hipGetLastError());
        if (ctx->log_soft) { const int rcc = compact_logs(ctx, C); if (rcc) return rcc; }
        m0 = m1;
    }
    ctx->moves_done = m_end;
    return KVP_OK;
}

// ---- annealing over the inference steps in which pages migrate (kvp_slots.hip has the scoring) ----
// One wavefront per chain; the placement X is the same for all chains and does not change, so the pages
// that migrate are known: `list` holds them, M entries (l*N + n)*P + p in ascending order.  A proposal is
// one Philox block: an entry of the list, a new Y, the acceptance draw; a wavefront computes the blocks
// of 64 consecutive proposals at once, one per lane.  Null if Y stays.  The move takes the page out of
// |M^i| or |M^o| of the old step and into the new one's: two step latencies change, dT = (t' - t) at the
// old step + (t' - t) at the new one.  A page that enters HBM earlier or leaves it later is in the pool
// during the steps in between: the lanes look at those (at most L - 1) and the proposal is dropped if
// one is full.  Control flow is the same for all lanes.
namespace {

__global__ __launch_bounds__(KVP_WAVE) void refine_slots_kernel(DevProblem q, SAParams sp, const uint32_t *__restrict__ X,
                                                                const uint32_t *__restrict__ cnt,
                                                                const uint32_t *__restrict__ list, uint32_t M, uint8_t *Yall,
                                                                uint32_t *mig_all, uint32_t *pool_all,
                                                                ChainState *__restrict__ states, uint64_t move_begin,
                                                                uint64_t move_end, int calibrate) {
    const uint32_t chain = blockIdx.x;
    const int lane = (int)threadIdx.x;
    const uint32_t L = q.L, N = q.N, Wd = q.Wd;
    const size_t G = (size_t)L * N;
    uint8_t *Y = Yall + (size_t)chain * G * q.P;
    uint32_t *mig = mig_all + (size_t)chain * G * 2, *pool = pool_all + (size_t)chain * G;
    ChainState st = states[chain];
    const uint32_t stream = calibrate ? 40u : 32u;
    double sum = 0.0;
    uint32_t npos = 0;
    uint32_t o0 = 0, o1 = 0, o2 = 0, o3 = 0;      // the block of proposal `first + lane`
    uint64_t first = move_begin;
    auto refill = [&](uint64_t from) {
        uint32_t out[4];
        const uint64_t mine = from + (uint32_t)lane;
        philox4x32_10((uint32_t)mine, (uint32_t)(mine >> 32), chain, stream, sp.seed_lo, sp.seed_hi, out);
        o0 = out[0]; o1 = out[1]; o2 = out[2]; o3 = out[3];
        first = from;
    };
    refill(move_begin);
    for (uint64_t mi = move_begin; mi < move_end; mi++) {
        if (!calibrate) {
            uint64_t lvl = mi / sp.mpl;
            if (lvl > sp.n_levels - 1) lvl = sp.n_levels - 1;
            while (st.level < lvl) { st.c = st.c * sp.alpha; st.level++; }  // geometric cooling
            st.moves_done++;
        }
        if (mi - first >= KVP_WAVE) refill(mi);
        const int at = (int)(uint32_t)(mi - first);
        const uint32_t r0 = (uint32_t)__builtin_amdgcn_readlane((int)o0, at), r1 = (uint32_t)__builtin_amdgcn_readlane((int)o1, at);
        const uint32_t r2 = (uint32_t)__builtin_amdgcn_readlane((int)o2, at), r3 = (uint32_t)__builtin_amdgcn_readlane((int)o3, at);
        const double u = ((double)(((uint64_t)r2 << 20) | (r3 >> 12)) + 0.5) * (1.0 / 4503599627370496.0);
        if (M == 0) { if (!calibrate) st.null_moves++; continue; }
        const uint32_t entry = list[__umulhi(r0, M)], ynew = __umulhi(r1, L);
        const uint32_t row = entry / q.P, p = entry - row * q.P, l = row / N, n = row - l * N, w = p >> 5, b = p & 31u;
        const int c = ((X[((size_t)l * N + n) * Wd + w] & q.V[(size_t)n * Wd + w]) >> b) & 1u ? 1 : -1;   // comes in, or goes out
        const size_t iy = entry;
        const uint32_t yold = Y[iy];
        if (ynew == yold) { if (!calibrate) st.null_moves++; continue; }
        const uint32_t g_own = n * L + l, g_old = g_own - yold, g_new = g_own - ynew;
        // the steps during which the page is in the pool only after the move
        uint32_t lo = 0, hi = 0;
        if (c > 0 && g_new < g_old) { lo = g_new; hi = g_old; }
        if (c < 0 && g_new > g_old) { lo = g_old; hi = g_new; }
        bool full = false;
        for (uint32_t g = lo + (uint32_t)lane; g < hi; g += KVP_WAVE) full = full || pool[g] + 1u > q.cap;
        if (ballot64(full)) { if (!calibrate) { st.null_moves++; st.clipped++; } continue; }
        const uint32_t no = g_old / L, lo_ = g_old - no * L, nn = g_new / L, ln = g_new - nn * L;
        const uint32_t *co = cnt + ((size_t)lo_ * N + no) * 4, *cn = cnt + ((size_t)ln * N + nn) * 4;
        const uint32_t mio = mig[(size_t)g_old * 2], moo = mig[(size_t)g_old * 2 + 1];
        const uint32_t min_ = mig[(size_t)g_new * 2], mon = mig[(size_t)g_new * 2 + 1];
        const uint32_t acco = q.acc[(size_t)lo_ * N + no], accn = q.acc[(size_t)ln * N + nn], wro = q.wr[no], wrn = q.wr[nn];
        const uint32_t di = c > 0 ? 1u : 0u, dout = c > 0 ? 0u : 1u;
        const double t_old = step_time(q, co[0], co[1], mio, moo, acco, wro);
        const double t_old2 = step_time(q, co[0], co[1], mio - di, moo - dout, acco, wro);
        const double t_new = step_time(q, cn[0], cn[1], min_, mon, accn, wrn);
        const double t_new2 = step_time(q, cn[0], cn[1], min_ + di, mon + dout, accn, wrn);
        const double dT = (t_old2 - t_old) + (t_new2 - t_new);
        if (calibrate) {
            if (dT > 0.0) { sum = sum + dT; npos++; }
            continue;
        }
        const bool accept = (dT <= 0.0) || (st.c > 0.0 && u < exp(-dT / st.c));   // Metropolis
        if (!accept) continue;
        st.accepted++;
        if (dT > 0.0) st.uphill++;
        if (lane == 0) {
            Y[iy] = (uint8_t)ynew;
            mig[(size_t)g_old * 2] = mio - di; mig[(size_t)g_old * 2 + 1] = moo - dout;
            mig[(size_t)g_new * 2] = min_ + di; mig[(size_t)g_new * 2 + 1] = mon + dout;
        }
        // in the pool from the new step to the old one (or the other way round) where it was not, or no longer
        const uint32_t a = min(g_old, g_new), e = max(g_old, g_new);
        const uint32_t delta = ((c > 0) == (g_new < g_old)) ? 1u : 0xFFFFFFFFu;
        for (uint32_t g = a + (uint32_t)lane; g < e; g += KVP_WAVE) pool[g] += delta;
        st.t_cur = st.t_cur + dT;
        if (st.t_cur < st.t_best) { st.t_best = st.t_cur; st.improved++; }
        // later proposals read, from other lanes, what this one wrote: one wavefront, program order
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
    if (calibrate) {
        st.c0 = npos ? (sum / (double)npos) / sp.neg_ln_p0 : 0.0;
        st.c = st.c0;
        st.level = 0;
    }
    if (lane == 0) states[chain] = st;
}

}  // namespace

extern "C" int kvp_refine_slots(kvp_ctx *ctx, const kvp_anneal_params *p, const uint32_t *d_placement, uint8_t *d_slots,
                                kvp_chain_stats_t *h_stats) {
    if (!ctx || !p || !d_placement || !d_slots || ((uintptr_t)d_placement & 15u)) return KVP_EINVAL;
    if (!ctx->has_trace) return KVP_ENOTRACE;
    if (p->n_chains == 0 || p->n_chains > 65535u || p->n_levels == 0 || !(p->p0 > 0.0 && p->p0 < 1.0) ||
        !(p->alpha > 0.0 && p->alpha <= 1.0) || p->total_moves == 0 || p->moves > p->total_moves ||
        (p->init_mode != KVP_INIT_EMPTY && p->init_mode != KVP_INIT_GIVEN))
        return KVP_EINVAL;
    KVP_HIP(hipSetDevice(ctx->device));
    const DevProblem &q = ctx->dp;
    const uint32_t C = p->n_chains;
    const size_t G = (size_t)q.L * q.N;
    if (p->init_mode == KVP_INIT_EMPTY) KVP_HIP(hipMemsetAsync(d_slots, 0, (size_t)C * G * q.P, ctx->stream));
    double *d_cost = nullptr;
    uint32_t *d_excess = nullptr;
    ChainState *d_state = nullptr;
    auto cleanup = [&]() {
        if (d_cost) (void)hipFree(d_cost);
        if (d_excess) (void)hipFree(d_excess);
        if (d_state) (void)hipFree(d_state);
    };
    if (hipMalloc((void **)&d_cost, sizeof(double) * C) != hipSuccess || hipMalloc((void **)&d_excess, 4 * (size_t)C) != hipSuccess ||
        hipMalloc((void **)&d_state, sizeof(ChainState) * C) != hipSuccess) {
        (void)hipGetLastError();
        cleanup();
        return KVP_ENOMEM;
    }
    uint32_t *cnt = nullptr, *mig = nullptr, *pool = nullptr, *list = nullptr, M = 0;
    int rc = kvp_slots_state_launch(ctx, d_placement, true, d_slots, C, d_cost, d_excess, &cnt, &mig, &pool);
    if (!rc) rc = kvp_slot_list_build(ctx, d_placement, &list, &M);
    if (rc) { cleanup(); return rc; }
    std::vector<uint32_t> hex(C);
    hipError_t e = hipMemcpyAsync(hex.data(), d_excess, 4 * (size_t)C, hipMemcpyDeviceToHost, ctx->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
    if (e != hipSuccess) { (void)hipGetLastError(); cleanup(); return KVP_EHIP; }
    for (uint32_t c = 0; c < C; c++)
        if (hex[c] & 0x7FFFFFFFu) { cleanup(); return KVP_EINFEASIBLE; }   // a step overfilled, or a Y out of range
    init_states_kernel<<<dim3((C + 255) / 256), dim3(256), 0, ctx->stream>>>(d_state, d_cost, C);
    SAParams sp;
    sp.seed_lo = (uint32_t)p->seed; sp.seed_hi = (uint32_t)(p->seed >> 32);
    sp.th0 = (uint64_t)(0.4 * 4294967296.0); sp.th1 = (uint64_t)(0.8 * 4294967296.0);   // the operator field is not used
    sp.mpl = p->total_moves / p->n_levels; if (sp.mpl < 1) sp.mpl = 1;
    sp.n_levels = p->n_levels; sp.max_len = 1;
    sp.alpha = p->alpha; sp.neg_ln_p0 = -log(p->p0);
    refine_slots_kernel<<<dim3(C), dim3(KVP_WAVE), 0, ctx->stream>>>(q, sp, d_placement, cnt, list, M, d_slots, mig, pool, d_state,
                                                                     0, CALIB_MOVES, 1);
    for (uint64_t m0 = 0; m0 < p->moves; m0 += 16384) {                // bounded launches: every wavefront exits after a fixed count
        const uint64_t m1 = m0 + 16384 < p->moves ? m0 + 16384 : p->moves;
        refine_slots_kernel<<<dim3(C), dim3(KVP_WAVE), 0, ctx->stream>>>(q, sp, d_placement, cnt, list, M, d_slots, mig, pool,
                                                                         d_state, m0, m1, 0);
    }
    e = hipGetLastError();
    std::vector<ChainState> hs(C);
    if (e == hipSuccess) e = hipMemcpyAsync(hs.data(), d_state, sizeof(ChainState) * C, hipMemcpyDeviceToHost, ctx->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
    cleanup();
    if (e != hipSuccess) { kvp_tls_hip_error = (int)e; kvp_tls_hip_line = __LINE__; (void)hipGetLastError(); return KVP_EHIP; }
    if (h_stats)
        for (uint32_t c = 0; c < C; c++) {
            h_stats[c].t_cur = hs[c].t_cur; h_stats[c].t_best = hs[c].t_best; h_stats[c].c0 = hs[c].c0; h_stats[c].c = hs[c].c;
            h_stats[c].moves_done = hs[c].moves_done; h_stats[c].accepted = hs[c].accepted; h_stats[c].uphill = hs[c].uphill;
            h_stats[c].null_moves = hs[c].null_moves; h_stats[c].clipped = hs[c].clipped; h_stats[c].improved = hs[c].improved;
        }
    return KVP_OK;
}

// ---- parallel tempering: the chains' temperatures spread over a ladder and traded between slices ----

namespace {

__global__ __launch_bounds__(256) void temper_kernel(ChainState *__restrict__ st, const double *__restrict__ factor,
                                                     uint32_t C) {
    const uint32_t c = blockIdx.x * 256 + threadIdx.x;
    if (c >= C) return;
    st[c].c0 = st[c].c0 * factor[c];
    st[c].c = st[c].c * factor[c];
}

// One workgroup walks the pairs (a, a + 1), a = round mod 2, + 2, ...: the pairs of a round are
// disjoint, so every thread owns both chains of its pairs.  out[0] = pairs that traded.
__global__ __launch_bounds__(256) void exchange_kernel(ChainState *__restrict__ st, uint32_t C, uint32_t seed_lo,
                                                       uint32_t seed_hi, uint64_t round, uint32_t *__restrict__ out) {
    __shared__ uint32_t traded;
    if (threadIdx.x == 0) traded = 0;
    __syncthreads();
    uint32_t mine = 0;
    for (uint64_t a64 = (round & 1u) + 2ull * threadIdx.x; a64 + 1 < C; a64 += 512) {
        const uint32_t a = (uint32_t)a64, b = a + 1;
        const double ca = st[a].c, cb = st[b].c;
        if (!(ca > 0.0) || !(cb > 0.0)) continue;
        uint32_t r[4];
        philox4x32_10((uint32_t)round, (uint32_t)(round >> 32), a, 16u, seed_lo, seed_hi, r);
        const uint64_t bits = ((uint64_t)r[0] << 20) | (uint64_t)(r[1] >> 12);
        const double u = ((double)bits + 0.5) * (1.0 / 4503599627370496.0);
        const double d = (1.0 / ca - 1.0 / cb) * (st[a].t_cur - st[b].t_cur);
        if (d >= 0.0 || u < exp(d)) {
            const double c0a = st[a].c0, c0b = st[b].c0;
            st[a].c = cb; st[b].c = ca;
            st[a].c0 = c0b; st[b].c0 = c0a;
            mine++;
        }
    }
    if (mine) atomicAdd(&traded, mine);
    __syncthreads();
    if (threadIdx.x == 0) out[0] = traded;
}

}  // namespace

extern "C" int kvp_temper(kvp_ctx *ctx, const double *h_factor) {
    if (!ctx || !h_factor) return KVP_EINVAL;
    if (!ctx->has_chains) return KVP_ENOCHAINS;
    if (ctx->moves_done == 0) return KVP_EINVAL;                       // the next slice would calibrate anew
    const uint32_t C = ctx->sa.n_chains;
    for (uint32_t c = 0; c < C; c++)
        if (!(h_factor[c] > 0.0) || !(h_factor[c] <= 1.7976931348623157e308)) return KVP_EINVAL;
    KVP_HIP(hipSetDevice(ctx->device));
    int rc = kvp_ensure(ctx, (void **)&ctx->d_cnt_tmp, &ctx->cnt_tmp_cap, sizeof(double) * (size_t)C);
    if (rc) return rc;
    double *d_factor = (double *)ctx->d_cnt_tmp;
    KVP_HIP(hipMemcpyAsync(d_factor, h_factor, sizeof(double) * (size_t)C, hipMemcpyHostToDevice, ctx->stream));
    temper_kernel<<<dim3((C + 255) / 256), dim3(256), 0, ctx->stream>>>(ctx->d_state, d_factor, C);
    KVP_HIP(hipGetLastError());
    KVP_HIP(hipStreamSynchronize(ctx->stream));                        // h_factor may be pageable: it is free again
    return KVP_OK;
}

extern "C" int kvp_exchange(kvp_ctx *ctx, uint64_t round, uint32_t *h_traded) {
    if (!ctx) return KVP_EINVAL;
    if (!ctx->has_chains) return KVP_ENOCHAINS;
    KVP_HIP(hipSetDevice(ctx->device));
    exchange_kernel<<<dim3(1), dim3(256), 0, ctx->stream>>>(ctx->d_state, ctx->sa.n_chains, (uint32_t)ctx->sa.seed,
                                                            (uint32_t)(ctx->sa.seed >> 32), round, ctx->d_argmin + 2);
    KVP_HIP(hipGetLastError());
    if (h_traded) {
        KVP_HIP(hipMemcpyAsync(h_traded, ctx->d_argmin + 2, 4, hipMemcpyDeviceToHost, ctx->stream));
        KVP_HIP(hipStreamSynchronize(ctx->stream));
    }
    return KVP_OK;
}

extern "C" int kvp_best(kvp_ctx *ctx, double *h_cost, uint32_t *h_chain, uint32_t *h_placement,
                        double *h_chain_costs) {
    if (!ctx || !h_cost || !h_chain) return KVP_EINVAL;
    if (!ctx->has_trace) return KVP_ENOTRACE;
    if (!ctx->has_chains) return KVP_ENOCHAINS;
    KVP_HIP(hipSetDevice(ctx->device));
    const DevProblem &q = ctx->dp;
    const uint32_t C = ctx->sa.n_chains;
    const size_t per = (size_t)q.L * q.N * q.Wd;
    int rc;
    if ((rc = launch_log_xor(ctx, 0, C))) return rc;                       // current -> best-so-far schedules
    rc = kvp_score_launch(ctx, ctx->d_X, C, ctx->d_cost, ctx->d_excess, nullptr, nullptr);   // exact re-score
    if (!rc) {
        argmin_kernel<<<dim3(1), dim3(256), 0, ctx->stream>>>(ctx->d_cost, C, ctx->d_argmin);
        if (hipGetLastError() != hipSuccess) rc = KVP_EHIP;
    }
    uint32_t win = 0;
    if (!rc && hipMemcpyAsync(&win, ctx->d_argmin, 4, hipMemcpyDeviceToHost, ctx->stream) != hipSuccess) rc = KVP_EHIP;
    if (!rc && hipStreamSynchronize(ctx->stream) != hipSuccess) rc = KVP_EHIP;
    if (!rc && hipMemcpyAsync(h_cost, ctx->d_cost + win, 8, hipMemcpyDeviceToHost, ctx->stream) != hipSuccess) rc = KVP_EHIP;
    if (!rc && h_placement &&
        hipMemcpyAsync(h_placement, ctx->d_X + (size_t)win * per, per * 4, hipMemcpyDeviceToHost, ctx->stream) != hipSuccess)
        rc = KVP_EHIP;
    if (!rc && h_chain_costs &&
        hipMemcpyAsync(h_chain_costs, ctx->d_cost, 8 * (size_t)C, hipMemcpyDeviceToHost, ctx->stream) != hipSuccess)
        rc = KVP_EHIP;
    const int rc2 = launch_log_xor(ctx, 0, C);                             // back to the current schedules
    if (hipStreamSynchronize(ctx->stream) != hipSuccess && !rc) rc = KVP_EHIP;
    if (!rc && !rc2) *h_chain = win;
    return rc ? rc : rc2;
}

extern "C" int kvp_chain_placement(kvp_ctx *ctx, uint32_t chain, int best, uint32_t *h_placement) {
    if (!ctx || !h_placement) return KVP_EINVAL;
    if (!ctx->has_chains) return KVP_ENOCHAINS;
    if (chain >= ctx->sa.n_chains) return KVP_EINVAL;
    KVP_HIP(hipSetDevice(ctx->device));
    const DevProblem &q = ctx->dp;
    const size_t per = (size_t)q.L * q.N * q.Wd;
    int rc = KVP_OK;
    if (best && (rc = launch_log_xor(ctx, chain, 1))) return rc;
    if (hipMemcpyAsync(h_placement, ctx->d_X + (size_t)chain * per, per * 4, hipMemcpyDeviceToHost, ctx->stream) != hipSuccess)
        rc = KVP_EHIP;
    int rc2 = KVP_OK;
    if (best) rc2 = launch_log_xor(ctx, chain, 1);
    if (hipStreamSynchronize(ctx->stream) != hipSuccess && !rc) rc = KVP_EHIP;
    return rc ? rc : rc2;
}

extern "C" int kvp_chain_stats(kvp_ctx *ctx, kvp_chain_stats_t *h_stats) {
    if (!ctx || !h_stats) return KVP_EINVAL;
    if (!ctx->has_chains) return KVP_ENOCHAINS;
    KVP_HIP(hipSetDevice(ctx->device));
    const uint32_t C = ctx->sa.n_chains;
    ChainState *h = (ChainState *)malloc(sizeof(ChainState) * C);
    if (!h) return KVP_ENOMEM;
    hipError_t e = hipMemcpyAsync(h, ctx->d_state, sizeof(ChainState) * C, hipMemcpyDeviceToHost, ctx->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
    if (e != hipSuccess) { free(h); (void)hipGetLastError(); return KVP_EHIP; }
    for (uint32_t c = 0; c < C; c++) {
        h_stats[c].t_cur = h[c].t_cur; h_stats[c].t_best = h[c].t_best; h_stats[c].c0 = h[c].c0; h_stats[c].c = h[c].c;
        h_stats[c].moves_done = h[c].moves_done; h_stats[c].accepted = h[c].accepted; h_stats[c].uphill = h[c].uphill;
        h_stats[c].null_moves = h[c].null_moves; h_stats[c].clipped = h[c].clipped; h_stats[c].improved = h[c].improved;
    }
    free(h);
    return KVP_OK;
}
