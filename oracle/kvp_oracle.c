/*
 * CPU oracle for the KV-cache placement problem of "Accelerating LLM Inference
 * via Dynamic KV Cache Placement in Heterogeneous Memory System" (Sec. III).
 *
 * TEST INFRASTRUCTURE ONLY.  Plain, single-threaded, slow on purpose.  It works
 * on one byte per (layer, step, page) boolean and shares no code, table or
 * header with the GPU library; only the tests, the smoke check and the
 * benchmark's cpu_baseline leg may call it.
 *
 * Part (i), the objective, is the definition of Eqs. 1-5 written out.
 * Part (ii), the annealer, takes the Metropolis / cooling skeleton of
 * Sec. III-B step by step; its move set on the placement schedule itself is
 * this project's own design (the paper anneals two policy scalars), so its
 * effectiveness is "parity unpinned" by the paper: it is pinned only by
 * exhaustive search on tiny instances and by its invariants.  The exchange of
 * temperatures between chains (orc_exchange, parallel tempering) is an
 * extension of the same standing: pinned by hand-worked pairs, by the
 * acceptance frequency 1/e of a pair with exponent -1 and by its invariants.
 * Part (iii), at the end, is the paper's own search: a look-ahead policy with the
 * two scalars W and R, and the annealing over them.  The paper states the
 * policy in two sentences; the reading taken is written out step by step above
 * orc_wr_policy and pinned by hand-worked instances ("parity unpinned" by the
 * paper beyond that: it prints no worked example).
 *
 * Build: gcc -O2 -ffp-contract=off -fno-fast-math -shared -fPIC
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    int32_t L, N, P, K;
    const uint8_t *access;   /* [L][N][K][P] page p is read by plane k at step (n,l) */
    const uint8_t *alive;    /* [N][P] page holds data at step n                    */
    const uint8_t *persist;  /* [N][P] same data as at step n-1                     */
    const uint8_t *written;  /* [N][P] page receives the token generated at step n  */
    uint64_t plane_bytes[8]; /* bytes read per accessed page of plane k             */
    uint64_t page_bytes;     /* bytes moved when a page changes tier                */
    uint64_t token_bytes;    /* bytes of new KV written per written page and layer  */
    double bw_hbm, bw_link, bw_dram;   /* B_h, B_k, B_d in bytes/s                  */
    uint64_t cap_pages;      /* HBM pool, pages, shared by all layers               */
} orc_problem;

typedef struct { uint32_t op, layer, page, n1, len, layer2, page2, dsel; } orc_move;

enum { ORC_SET = 0, ORC_SWAP = 1, ORC_SHIFT = 2 };
enum { ORC_OK = 0, ORC_CLIPPED = 1, ORC_NULL = 2 };
#define ORC_MAX_LEN 63
#define ORC_WIN 64

/* ---- indexing helpers ---------------------------------------------------- */
static inline size_t ix_x(const orc_problem *q, int l, int n, int p) {
    return ((size_t)l * q->N + n) * q->P + p;
}
static inline int a_bit(const orc_problem *q, int l, int n, int k, int p) {
    return q->access[(((size_t)l * q->N + n) * q->K + k) * q->P + p] != 0;
}
static inline int v_bit(const orc_problem *q, int n, int p) { return q->alive[(size_t)n * q->P + p] != 0; }
static inline int pm_bit(const orc_problem *q, int n, int p) { return q->persist[(size_t)n * q->P + p] != 0; }
static inline int wm_bit(const orc_problem *q, int n, int p) { return q->written[(size_t)n * q->P + p] != 0; }
/* a page is in HBM at step (n,l) iff its bit is set and the page exists */
static inline int x_bit(const orc_problem *q, const uint8_t *X, int l, int n, int p) {
    return X[ix_x(q, l, n, p)] != 0 && v_bit(q, n, p);
}

/* ---- canonical sum (order of Eq. 1) --------------------------------------
 * Pad to a multiple of 64 with +0.0; inside each block of 64 fold the upper
 * half onto the lower half (32, 16, ..., 1); add the block sums in order. */
double orc_csum(const double *v, size_t m) {
    double total = 0.0;
    for (size_t b = 0; b < m; b += 64) {
        double blk[64];
        for (int i = 0; i < 64; i++) blk[i] = (b + i < m) ? v[b + i] : 0.0;
        for (int h = 32; h >= 1; h >>= 1)
            for (int i = 0; i < h; i++) blk[i] = blk[i] + blk[i + h];
        total = (b == 0) ? blk[0] : total + blk[0];
    }
    return total;
}

/* ---- per-step data volumes (Sec. III-A, the sets of Eqs. 3-4) ------------
 * out = {|H^r|, |E^r|, |H^w|, |E^w|, |M^i|, |M^o|} in bytes for step (n,l).
 * Reads and the new token's write see the placement of this step; the change
 * from the previous step's placement of the same layer is this step's
 * migration.  Pages that did not hold the same data one step earlier (n = 0,
 * a page just born, a slot re-used by a new sequence) migrate nothing. */
void orc_step_bytes(const orc_problem *q, const uint8_t *X, int l, int n, uint64_t out[6]) {
    uint64_t hr = 0, er = 0, hw = 0, ew = 0, mi = 0, mo = 0;
    for (int p = 0; p < q->P; p++) {
        int x = x_bit(q, X, l, n, p);
        for (int k = 0; k < q->K; k++)
            if (a_bit(q, l, n, k, p)) { if (x) hr += q->plane_bytes[k]; else er += q->plane_bytes[k]; }
        if (wm_bit(q, n, p)) { if (x) hw += q->token_bytes; else ew += q->token_bytes; }
        if (n > 0 && pm_bit(q, n, p)) {
            int xp = x_bit(q, X, l, n - 1, p);
            if (x && !xp) mi += q->page_bytes;
            if (!x && xp) mo += q->page_bytes;
        }
    }
    out[0] = hr; out[1] = er; out[2] = hw; out[3] = ew; out[4] = mi; out[5] = mo;
}

static inline double dmax(double a, double b) { return a > b ? a : b; }

/* ---- step latency (Eqs. 2-4) ----------------------------------------------
 * Divisions are written as products with reciprocals formed once in fp64. */
double orc_step_time(const orc_problem *q, const uint64_t b[6]) {
    double inv_bh = 1.0 / q->bw_hbm, inv_bk = 1.0 / q->bw_link, inv_bd = 1.0 / q->bw_dram;
    double inv_min = 1.0 / (q->bw_link < q->bw_dram ? q->bw_link : q->bw_dram);
    uint64_t hr = b[0], er = b[1], hw = b[2], ew = b[3], mi = b[4], mo = b[5];
    double t_h = (double)(hr + hw + mi + mo) * inv_bh;                         /* Eq. 3 */
    double link_out = (double)(ew + mo) * inv_bk;
    double link_in = (double)mi * inv_bk;
    double chan = (double)(ew + mi + mo) * inv_bd;
    double t_e = (double)er * inv_min + dmax(dmax(link_out, link_in), chan);   /* Eq. 4 */
    return dmax(t_h, t_e);                                                     /* Eq. 2 */
}

static double step_time_at(const orc_problem *q, const uint8_t *X, int l, int n) {
    uint64_t b[6];
    orc_step_bytes(q, X, l, n, b);
    return orc_step_time(q, b);
}

/* occupancy of the HBM pool while token step n runs (Eq. 5, per token step) */
void orc_occupancy(const orc_problem *q, const uint8_t *X, uint32_t *occ) {
    for (int n = 0; n < q->N; n++) {
        uint32_t c = 0;
        for (int l = 0; l < q->L; l++)
            for (int p = 0; p < q->P; p++) c += (uint32_t)x_bit(q, X, l, n, p);
        occ[n] = c;
    }
}

/* ---- total latency and feasibility (Eqs. 1, 5) ---------------------------
 * Steps are summed in execution order g = n*L + l.  excess = largest overshoot
 * of the capacity over all token steps (0: feasible); bit 31 flags bits set on
 * pages that do not exist (they are ignored).  Optional outputs:
 * step_bytes [L][N][6], step_t [L][N], occ [N]. */
double orc_score(const orc_problem *q, const uint8_t *X, uint32_t *excess,
                 uint64_t *step_bytes, double *step_t, uint32_t *occ_out) {
    int L = q->L, N = q->N;
    double *t = (double *)malloc(sizeof(double) * (size_t)L * N);
    uint32_t *occ = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)N);
    for (int n = 0; n < N; n++)
        for (int l = 0; l < L; l++) {
            uint64_t b[6];
            orc_step_bytes(q, X, l, n, b);
            double tt = orc_step_time(q, b);
            t[(size_t)n * L + l] = tt;
            if (step_bytes) memcpy(step_bytes + ((size_t)l * N + n) * 6, b, sizeof b);
            if (step_t) step_t[(size_t)l * N + n] = tt;
        }
    double T = orc_csum(t, (size_t)L * N);
    orc_occupancy(q, X, occ);
    uint64_t ex = 0;
    for (int n = 0; n < N; n++)
        if ((uint64_t)occ[n] > q->cap_pages && occ[n] - q->cap_pages > ex) ex = occ[n] - q->cap_pages;
    uint32_t flag = 0;
    for (int l = 0; l < L && !flag; l++)
        for (int n = 0; n < N && !flag; n++)
            for (int p = 0; p < q->P; p++)
                if (X[ix_x(q, l, n, p)] && !v_bit(q, n, p)) { flag = 0x80000000u; break; }
    if (excess) *excess = (uint32_t)ex | flag;
    if (occ_out) memcpy(occ_out, occ, sizeof(uint32_t) * (size_t)N);
    free(t); free(occ);
    return T;
}

/* ---- Philox4x32-10 (Salmon, Moraes, Dror, Shaw; SC'11) ------------------- */
void orc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3], k0 = key[0], k1 = key[1];
    for (int r = 0; r < 10; r++) {
        uint64_t m0 = (uint64_t)0xD2511F53u * c0;
        uint64_t m1 = (uint64_t)0xCD9E8D57u * c2;
        uint32_t n0 = (uint32_t)(m1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)m1;
        uint32_t n2 = (uint32_t)(m0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)m0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* ---- moves -----------------------------------------------------------------
 * A move edits the timeline of one (layer, page) bit, and for SWAP also of a
 * victim (layer2, page2).  orc_resolve turns the raw record into per-step flip
 * flags f1 (for layer,page) and f2 (for layer2,page2), both of length N, and
 * the first step `base` of the 64-step window over which the cost change is
 * summed.  `occ` is the occupancy of the current schedule, which must be
 * feasible.  No move ever raises a step's occupancy above the capacity.
 *
 *  span   steps n1 <= n < e, e = first n > n1 with n-n1 == len, n == N, or the
 *         page not persisting into n.  The page must exist at n1.
 *  SET    target value v = not(bit at n1).  Ascending over the span, give the
 *         bit value v; when v = 1 stop at the first step that is full and whose
 *         bit is clear.
 *  SWAP   if the bit at n1 is set: as SET (v = 0).  Otherwise, at every step of
 *         the span whose bit is clear: set it if the step is below capacity;
 *         else, if the victim's bit is set there, clear the victim and set it;
 *         else leave the step alone.
 *  SHIFT  first step nt in (n1, n1+len] (while the page persists) whose bit
 *         differs from the step before.  With a = bit before nt and d in
 *         {-2,-1,+1,+2}: d < 0 moves the transition earlier (steps nt-1 down to
 *         max(nt+d, n1) take the value not(a)), d > 0 later (steps nt up to
 *         nt+d-1, while the page persists, take a); setting stops at a full
 *         step.  base = nt - 2.
 */
static const int SHIFT_D[4] = {-2, -1, 1, 2};

/* May the bit of (l, p) be set at token step n?  `evict`: the victim (l2, pq), which is set at n,
 * is cleared at the same step.
 * tab == NULL, Eq. 5 once per token step: yes if the step is below capacity; with a victim always
 * (the pool of step n gains one page and loses one).
 * tab != NULL, Eq. 5 at every inference step (n, l'): tab[n][l'] is the pool after layer l' of step
 * n has taken its placement (orc_slot_occupancy).  Setting (l, p) at n adds the page to the slots
 * (n, l' >= l) and, if the page persists into n + 1, to the slots (n + 1, l' < l), where layer l
 * still holds its placement of step n; clearing the victim takes one page off (n, l' >= l2) and,
 * if it persists, off (n + 1, l' < l2).  Yes if no slot of the two steps ends above the capacity.
 * Every step of a move is judged against the schedule as it is before the move: two steps of one
 * page's run add to different slots (l' >= l of a step from its own bit, l' < l from the bit of
 * the step before), so each slot gains one page at most and what was judged stays true. */
static int fits(const orc_problem *q, const uint32_t *occ, const uint32_t *tab, int l, int p, int n,
                int evict, int l2, int pq) {
    uint64_t cap = q->cap_pages;
    if (!tab) return evict ? 1 : (uint64_t)occ[n] < cap;
    int L = q->L, N = q->N;
    for (int lp = 0; lp < L; lp++) {
        int64_t v = (int64_t)tab[(size_t)n * L + lp] + (lp >= l) - (evict && lp >= l2);
        if (v > (int64_t)cap) return 0;
    }
    if (n + 1 < N) {
        int pp = pm_bit(q, n + 1, p), pv = evict && pm_bit(q, n + 1, pq);
        for (int lp = 0; lp < L; lp++) {
            int64_t v = (int64_t)tab[(size_t)(n + 1) * L + lp] + (pp && lp < l) - (pv && lp < l2);
            if (v > (int64_t)cap) return 0;
        }
    }
    return 1;
}

static int resolve_move(const orc_problem *q, const uint8_t *X, const uint32_t *occ, const uint32_t *tab,
                        const orc_move *m, uint8_t *f1, uint8_t *f2, int *base) {
    int L = q->L, N = q->N, P = q->P;
    memset(f1, 0, (size_t)N); memset(f2, 0, (size_t)N);
    *base = 0;
    if (m->op > 2 || m->layer >= (uint32_t)L || m->page >= (uint32_t)P || m->n1 >= (uint32_t)N ||
        m->len < 1 || m->len > ORC_MAX_LEN || m->layer2 >= (uint32_t)L || m->page2 >= (uint32_t)P)
        return ORC_NULL;
    int l = (int)m->layer, p = (int)m->page, n1 = (int)m->n1, len = (int)m->len;
    int l2 = (int)m->layer2, pq = (int)m->page2;
    *base = n1;
    if (!v_bit(q, n1, p)) return ORC_NULL;
    int e = n1 + 1;
    while (e < N && e - n1 < len && pm_bit(q, e, p)) e++;
    int clipped = 0, flips = 0;
    int x1 = x_bit(q, X, l, n1, p);
    if (m->op == ORC_SET || (m->op == ORC_SWAP && x1)) {
        int v = !x1;
        for (int n = n1; n < e; n++) {
            if (x_bit(q, X, l, n, p) == v) continue;
            if (v && !fits(q, occ, tab, l, p, n, 0, 0, 0)) { clipped = 1; break; }
            f1[n] = 1; flips++;
        }
    } else if (m->op == ORC_SWAP) {
        int victim_ok = !(l2 == l && pq == p);
        for (int n = n1; n < e; n++) {
            if (x_bit(q, X, l, n, p)) continue;
            if (fits(q, occ, tab, l, p, n, 0, 0, 0)) { f1[n] = 1; flips++; }
            else if (victim_ok && x_bit(q, X, l2, n, pq) && fits(q, occ, tab, l, p, n, 1, l2, pq)) { f1[n] = 1; f2[n] = 1; flips++; }
            else clipped = 1;
        }
    } else { /* SHIFT */
        int nt = -1;
        for (int n = n1 + 1; n < N && n - n1 <= len && pm_bit(q, n, p); n++)
            if (x_bit(q, X, l, n, p) != x_bit(q, X, l, n - 1, p)) { nt = n; break; }
        if (nt < 0) return ORC_NULL;
        int a = x_bit(q, X, l, nt - 1, p);
        int d = SHIFT_D[m->dsel & 3];
        *base = nt - 2;
        if (d < 0) {
            int lo = nt + d > n1 ? nt + d : n1;
            for (int n = nt - 1; n >= lo; n--) {          /* these steps hold a, give them not(a) */
                if (!a && !fits(q, occ, tab, l, p, n, 0, 0, 0)) { clipped = 1; break; }
                f1[n] = 1; flips++;
            }
        } else {
            for (int n = nt; n < nt + d && n < N && (n == nt || pm_bit(q, n, p)); n++) {
                if (x_bit(q, X, l, n, p) == a) continue;
                if (a && !fits(q, occ, tab, l, p, n, 0, 0, 0)) { clipped = 1; break; }
                f1[n] = 1; flips++;
            }
        }
    }
    if (!flips) return ORC_NULL;
    return clipped ? ORC_CLIPPED : ORC_OK;
}

int orc_resolve(const orc_problem *q, const uint8_t *X, const uint32_t *occ, const orc_move *m,
                uint8_t *f1, uint8_t *f2, int *base) {
    return resolve_move(q, X, occ, NULL, m, f1, f2, base);
}

/* The same moves under Eq. 5 read at every inference step: `tab` is orc_slot_occupancy of X, which
 * must not exceed the capacity in any slot.  No move ever raises a slot above the capacity. */
int orc_resolve_strict(const orc_problem *q, const uint8_t *X, const uint32_t *tab, const orc_move *m,
                       uint8_t *f1, uint8_t *f2, int *base) {
    return resolve_move(q, X, NULL, tab, m, f1, f2, base);
}

static void apply_flips(const orc_problem *q, uint8_t *X, uint32_t *occ, const orc_move *m,
                        const uint8_t *f1, const uint8_t *f2, int lo, int hi) {
    for (int n = lo; n < hi; n++) {
        if (f1[n]) {
            size_t i = ix_x(q, (int)m->layer, n, (int)m->page);
            int was = x_bit(q, X, (int)m->layer, n, (int)m->page);
            X[i] = (uint8_t)!was;
            if (occ) occ[n] += was ? (uint32_t)-1 : 1u;
        }
        if (f2[n]) {
            size_t i = ix_x(q, (int)m->layer2, n, (int)m->page2);
            int was = x_bit(q, X, (int)m->layer2, n, (int)m->page2);
            X[i] = (uint8_t)!was;
            if (occ) occ[n] += was ? (uint32_t)-1 : 1u;
        }
    }
}

static int has_second_layer(const orc_problem *q, const orc_move *m, const uint8_t *f2) {
    if (m->layer2 == m->layer) return 0;
    for (int n = 0; n < q->N; n++) if (f2[n]) return 1;
    return 0;
}

/* ---- cost change of a move, the slow way -----------------------------------
 * dT = csum over the 64-step window [base, base+64) of (t' - t) on the move's
 * layer, plus the same on layer2 when the victim lives on another layer.  Both
 * schedules are scored in full here; steps the move does not touch contribute
 * an exact 0.0.  Returns the verdict; *delta = 0 for a null move. */
int orc_delta(const orc_problem *q, const uint8_t *X, const orc_move *m, double *delta, int *base_out,
              uint8_t *f1_out, uint8_t *f2_out) {
    int L = q->L, N = q->N;
    size_t sz = (size_t)L * N * q->P;
    uint32_t *occ = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)N);
    uint8_t *f1 = (uint8_t *)malloc((size_t)N), *f2 = (uint8_t *)malloc((size_t)N);
    orc_occupancy(q, X, occ);
    int base;
    int verdict = orc_resolve(q, X, occ, m, f1, f2, &base);
    *delta = 0.0;
    if (verdict != ORC_NULL) {
        uint8_t *Y = (uint8_t *)malloc(sz);
        memcpy(Y, X, sz);
        apply_flips(q, Y, NULL, m, f1, f2, 0, N);
        double *t0 = (double *)malloc(sizeof(double) * (size_t)L * N);
        double *t1 = (double *)malloc(sizeof(double) * (size_t)L * N);
        orc_score(q, X, NULL, NULL, t0, NULL);
        orc_score(q, Y, NULL, NULL, t1, NULL);
        double d[ORC_WIN];
        int l = (int)m->layer;
        for (int i = 0; i < ORC_WIN; i++) {
            int n = base + i;
            d[i] = (n >= 0 && n < N) ? t1[(size_t)l * N + n] - t0[(size_t)l * N + n] : 0.0;
        }
        double dT = orc_csum(d, ORC_WIN);
        if (has_second_layer(q, m, f2)) {
            int l2 = (int)m->layer2;
            for (int i = 0; i < ORC_WIN; i++) {
                int n = base + i;
                d[i] = (n >= 0 && n < N) ? t1[(size_t)l2 * N + n] - t0[(size_t)l2 * N + n] : 0.0;
            }
            dT = dT + orc_csum(d, ORC_WIN);
        }
        *delta = dT;
        free(Y); free(t0); free(t1);
    }
    if (base_out) *base_out = base;
    if (f1_out) memcpy(f1_out, f1, (size_t)N);
    if (f2_out) memcpy(f2_out, f2, (size_t)N);
    free(occ); free(f1); free(f2);
    return verdict;
}

/* Occupancy slot by slot (Eq. 5 read strictly): the layers of a token step change
 * their placement one after the other, each at its own step (n, l), so between
 * two layers of step n the pool holds the new placement of the layers done and
 * still the old one of the layers to come.  Simulated as it happens: at the start
 * of step n the pages that do not persist into it are gone; then layer after layer
 * takes its placement of step n, and the pool is counted after each.  Returns the
 * largest overshoot of cap_pages over all (n, l); never less than the overshoot
 * counted once per token step. */
uint32_t orc_strict_excess(const orc_problem *q, const uint8_t *X) {
    int L = q->L, N = q->N, P = q->P;
    uint8_t *cur = (uint8_t *)calloc((size_t)L * P ? (size_t)L * P : 1, 1);
    uint64_t worst = 0;
    for (int n = 0; n < N; n++) {
        for (int l = 0; l < L; l++)
            for (int p = 0; p < P; p++)
                if (!(n > 0 && pm_bit(q, n, p))) cur[(size_t)l * P + p] = 0;
        for (int l = 0; l < L; l++) {
            for (int p = 0; p < P; p++) cur[(size_t)l * P + p] = (uint8_t)(x_bit(q, X, l, n, p) && v_bit(q, n, p));
            uint64_t occ = 0;
            for (size_t i = 0; i < (size_t)L * P; i++) occ += cur[i];
            if (occ > q->cap_pages && occ - q->cap_pages > worst) worst = occ - q->cap_pages;
        }
    }
    free(cur);
    return (uint32_t)(worst > 0x7FFFFFFFull ? 0x7FFFFFFFull : worst);
}

/* The pool after every slot, tab[n][l], by the same simulation (the count is carried along: a
 * layer that takes its placement swaps its old pages for its new ones). */
void orc_slot_occupancy(const orc_problem *q, const uint8_t *X, uint32_t *tab) {
    int L = q->L, N = q->N, P = q->P;
    uint8_t *cur = (uint8_t *)calloc((size_t)L * P ? (size_t)L * P : 1, 1);
    uint32_t occ = 0;
    for (int n = 0; n < N; n++) {
        for (int l = 0; l < L; l++)
            for (int p = 0; p < P; p++)
                if (!(n > 0 && pm_bit(q, n, p)) && cur[(size_t)l * P + p]) { cur[(size_t)l * P + p] = 0; occ--; }
        for (int l = 0; l < L; l++) {
            for (int p = 0; p < P; p++) {
                uint8_t now = (uint8_t)(x_bit(q, X, l, n, p) && v_bit(q, n, p));
                occ += now; occ -= cur[(size_t)l * P + p];
                cur[(size_t)l * P + p] = now;
            }
            tab[(size_t)n * L + l] = occ;
        }
    }
    free(cur);
}

/* ---- starting schedules (the paper's non-migrating and reactive baselines,
 * Sec. IV-A, restated for a pool shared by all layers) ---------------------- */

typedef struct { int64_t key; size_t idx; } rank_item;
/* larger key first; equal keys: lower index first */
static int rank_cmp(const void *a, const void *b) {
    const rank_item *x = (const rank_item *)a, *y = (const rank_item *)b;
    if (x->key != y->key) return x->key > y->key ? -1 : 1;
    return x->idx < y->idx ? -1 : (x->idx > y->idx);
}

/* Static by frequency: the cap_pages (layer,page) pairs read most often over the
 * whole trace stay in HBM whenever they exist; nothing ever migrates.
 * Ties go to the lower l*P+p. */
void orc_init_static_frequency(const orc_problem *q, uint8_t *X) {
    int L = q->L, N = q->N, P = q->P;
    size_t M = (size_t)L * P;
    rank_item *it = (rank_item *)malloc(M * sizeof(rank_item));
    uint8_t *chosen = (uint8_t *)calloc(M, 1);
    for (size_t i = 0; i < M; i++) { it[i].key = 0; it[i].idx = i; }
    for (int l = 0; l < L; l++)
        for (int n = 0; n < N; n++)
            for (int k = 0; k < q->K; k++)
                for (int p = 0; p < P; p++) it[(size_t)l * P + p].key += a_bit(q, l, n, k, p);
    qsort(it, M, sizeof(rank_item), rank_cmp);
    for (size_t c = 0; c < M && (uint64_t)c < q->cap_pages; c++) chosen[it[c].idx] = 1;
    for (int l = 0; l < L; l++)
        for (int n = 0; n < N; n++)
            for (int p = 0; p < P; p++)
                X[ix_x(q, l, n, p)] = (uint8_t)(chosen[(size_t)l * P + p] && v_bit(q, n, p));
    free(it); free(chosen);
}

/* Recency: at step n the pool holds the cap_pages existing (layer,page) pairs
 * read most recently before n (never read: oldest).  Ties go to the lower
 * l*P+p.  A page that stops persisting forgets its history. */
void orc_init_recency(const orc_problem *q, uint8_t *X) {
    int L = q->L, N = q->N, P = q->P;
    size_t M = (size_t)L * P;
    int32_t *last = (int32_t *)malloc(M * sizeof(int32_t));
    rank_item *it = (rank_item *)malloc(M * sizeof(rank_item));
    for (size_t i = 0; i < M; i++) last[i] = -1;
    for (int n = 0; n < N; n++) {
        if (n > 0)
            for (int l = 0; l < L; l++)
                for (int p = 0; p < P; p++) {
                    size_t i = (size_t)l * P + p;
                    if (!pm_bit(q, n, p)) { last[i] = -1; continue; }
                    for (int k = 0; k < q->K; k++)
                        if (a_bit(q, l, n - 1, k, p)) last[i] = n - 1;
                }
        size_t cnt = 0;
        for (size_t i = 0; i < M; i++)
            if (v_bit(q, n, (int)(i % (size_t)P))) { it[cnt].key = last[i]; it[cnt].idx = i; cnt++; }
        qsort(it, cnt, sizeof(rank_item), rank_cmp);
        for (int l = 0; l < L; l++)
            for (int p = 0; p < P; p++) X[ix_x(q, l, n, p)] = 0;
        for (size_t c = 0; c < cnt && (uint64_t)c < q->cap_pages; c++) {
            size_t i = it[c].idx;
            X[ix_x(q, (int)(i / (size_t)P), n, (int)(i % (size_t)P))] = 1;
        }
    }
    free(last); free(it);
}

/* Static fill (the paper's "Static Placement", Sec. IV-A): an entry is placed
 * when it is first written and never moves; HBM is taken while there is room.
 * Reading for a pool shared by all layers and for slots that are re-used: step
 * by step, pages that stop persisting give their place back; then the pages new
 * at this step (existing, not persisting) take the free places in the order of
 * l*P+p (layer after layer, as a prefill writes them), the rest stay outside
 * for as long as they live. */
void orc_init_static_fill(const orc_problem *q, uint8_t *X) {
    int L = q->L, N = q->N, P = q->P;
    size_t M = (size_t)L * P;
    uint8_t *in = (uint8_t *)calloc(M ? M : 1, 1);
    uint64_t occ = 0;
    for (int n = 0; n < N; n++) {
        for (size_t i = 0; i < M; i++)
            if (in[i] && !(n > 0 && pm_bit(q, n, (int)(i % (size_t)P)))) { in[i] = 0; occ--; }
        for (size_t i = 0; i < M; i++) {
            int p = (int)(i % (size_t)P);
            int is_new = v_bit(q, n, p) && !(n > 0 && pm_bit(q, n, p));
            if (is_new && occ < q->cap_pages) { in[i] = 1; occ++; }
        }
        for (int l = 0; l < L; l++)
            for (int p = 0; p < P; p++) X[ix_x(q, l, n, p)] = in[(size_t)l * P + p];
    }
    free(in);
}

/* ---- exhaustive optimum (tiny instances only) ------------------------------
 * Enumerates every assignment of the existing (layer, step, page) bits; returns
 * the cheapest capacity-feasible schedule (first one found on ties). */
int orc_bruteforce(const orc_problem *q, double *best_cost, uint8_t *best_X, uint64_t *n_feasible) {
    int L = q->L, N = q->N, P = q->P;
    size_t sz = (size_t)L * N * P, pos[32];
    int m = 0;
    for (int l = 0; l < L; l++)
        for (int n = 0; n < N; n++)
            for (int p = 0; p < P; p++)
                if (v_bit(q, n, p)) { if (m >= 26) return -1; pos[m++] = ix_x(q, l, n, p); }
    uint8_t *X = (uint8_t *)calloc(sz ? sz : 1, 1);
    double best = INFINITY; uint64_t feas = 0;
    for (uint64_t code = 0; code < (1ull << m); code++) {
        for (int i = 0; i < m; i++) X[pos[i]] = (uint8_t)((code >> i) & 1);
        uint32_t ex;
        double T = orc_score(q, X, &ex, NULL, NULL, NULL);
        if (ex != 0) continue;
        feas++;
        if (T < best) { best = T; if (best_X) memcpy(best_X, X, sz); }
    }
    *best_cost = best; *n_feasible = feas;
    free(X);
    return 0;
}

/* ---- simulated annealing over the schedule (Sec. III-B skeleton) ---------- */
typedef struct {
    uint64_t seed;
    uint64_t total_moves;     /* length of the whole cooling schedule          */
    uint64_t move_begin, move_end;   /* this call runs moves [begin, end)      */
    uint32_t n_levels;        /* temperature levels, equal length              */
    uint32_t max_len;         /* longest span of a move, 1..63                  */
    double p0, alpha;         /* initial acceptance of uphill moves; cooling    */
    double op_prob[3];        /* SET, SWAP, SHIFT                               */
    uint32_t per_slot;        /* 0: Eq. 5 once per token step; 1: at every inference step (n, l) */
} orc_sa_params;

typedef struct {
    double T_cur, T_best, C0, C;
    uint32_t level;
    uint64_t accepted, uphill, null_moves, clipped, improved, uphill_seen;
} orc_sa_state;

#define ORC_CALIB 256

/* Proposal `mi` of chain `chain`: three Philox blocks, counter (mi lo, mi hi, chain, stream0 + 0..2)
 * under the seed.  Block 0: operator (word 0 against the cumulative shares of op_prob: the
 * three-operator mixture of Sec. III-B), layer, page, first step; block 1: span 1..max_len, victim
 * layer and page, direction of a SHIFT; block 2: the 52 bits of the acceptance draw u in (0, 1).
 * An index in 0..n-1 is the high word of (32 random bits) x n.  Exported for the pins. */
void orc_draw_move(const orc_problem *q, const orc_sa_params *sp, uint32_t chain, uint64_t mi,
                   uint32_t stream0, orc_move *m, double *u) {
    uint32_t key[2] = {(uint32_t)sp->seed, (uint32_t)(sp->seed >> 32)};
    uint32_t ctr[4] = {(uint32_t)mi, (uint32_t)(mi >> 32), chain, stream0};
    uint32_t a[4], b[4], c[4];
    orc_philox4x32_10(ctr, key, a);
    ctr[3] = stream0 + 1; orc_philox4x32_10(ctr, key, b);
    ctr[3] = stream0 + 2; orc_philox4x32_10(ctr, key, c);
    uint64_t th0 = (uint64_t)(sp->op_prob[0] * 4294967296.0);
    uint64_t th1 = (uint64_t)((sp->op_prob[0] + sp->op_prob[1]) * 4294967296.0);
    m->op = (a[0] < th0) ? ORC_SET : (a[0] < th1) ? ORC_SWAP : ORC_SHIFT;
    m->layer = (uint32_t)(((uint64_t)a[1] * (uint32_t)q->L) >> 32);
    m->page = (uint32_t)(((uint64_t)a[2] * (uint32_t)q->P) >> 32);
    m->n1 = (uint32_t)(((uint64_t)a[3] * (uint32_t)q->N) >> 32);
    m->len = 1 + (uint32_t)(((uint64_t)b[0] * sp->max_len) >> 32);
    m->layer2 = (uint32_t)(((uint64_t)b[1] * (uint32_t)q->L) >> 32);
    m->page2 = (uint32_t)(((uint64_t)b[2] * (uint32_t)q->P) >> 32);
    m->dsel = b[3] >> 30;
    uint64_t bits = ((uint64_t)c[0] << 20) | (c[1] >> 12);        /* 52 random bits */
    *u = ((double)bits + 0.5) * (1.0 / 4503599627370496.0);       /* (bits + 1/2) 2^-52 */
}

/* cost change over the window, recomputing only the rows of the move's
 * layer(s) inside the window; X is left modified iff `keep`. */
static double window_delta(const orc_problem *q, uint8_t *X, const orc_move *m, const uint8_t *f1,
                           const uint8_t *f2, int base, const double *tcur, double *tnew1, double *tnew2,
                           int *second) {
    int N = q->N;
    int lo = base < 0 ? 0 : base, hi = base + ORC_WIN < N ? base + ORC_WIN : N;
    apply_flips(q, X, NULL, m, f1, f2, lo, hi);
    double d[ORC_WIN];
    int l = (int)m->layer, l2 = (int)m->layer2;
    for (int i = 0; i < ORC_WIN; i++) {
        int n = base + i;
        if (n < 0 || n >= N) { d[i] = 0.0; continue; }
        tnew1[i] = step_time_at(q, X, l, n);
        d[i] = tnew1[i] - tcur[(size_t)l * N + n];
    }
    double dT = orc_csum(d, ORC_WIN);
    *second = has_second_layer(q, m, f2);
    if (*second) {
        for (int i = 0; i < ORC_WIN; i++) {
            int n = base + i;
            if (n < 0 || n >= N) { d[i] = 0.0; continue; }
            tnew2[i] = step_time_at(q, X, l2, n);
            d[i] = tnew2[i] - tcur[(size_t)l2 * N + n];
        }
        dT = dT + orc_csum(d, ORC_WIN);
    }
    apply_flips(q, X, NULL, m, f1, f2, lo, hi);   /* undo */
    return dT;
}

/* One chain.  X: current schedule (in/out, must be feasible).  best_X: best
 * schedule seen (in/out when resuming: st->T_best must match it).  On the first
 * call (move_begin == 0) the state is initialised and the temperature calibrated
 * from 256 proposals that are not applied: C0 = mean(dT | dT > 0) / (-ln p0). */
int orc_anneal_chain(const orc_problem *q, const orc_sa_params *sp, uint32_t chain, uint8_t *X,
                     uint8_t *best_X, orc_sa_state *st) {
    int L = q->L, N = q->N;
    size_t sz = (size_t)L * N * q->P;
    if (sp->max_len < 1 || sp->max_len > ORC_MAX_LEN || sp->n_levels < 1) return -1;
    double *tcur = (double *)malloc(sizeof(double) * (size_t)L * N);
    uint32_t *occ = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)N);
    uint8_t *f1 = (uint8_t *)malloc((size_t)N), *f2 = (uint8_t *)malloc((size_t)N);
    double tn1[ORC_WIN], tn2[ORC_WIN];
    uint32_t ex;
    double T0 = orc_score(q, X, &ex, NULL, tcur, occ);
    uint32_t *tab = NULL;                     /* per-slot capacity: the pool after every (n, l) */
    if (sp->per_slot && ex == 0) {
        tab = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)L * N);
        orc_slot_occupancy(q, X, tab);
        if (orc_strict_excess(q, X) != 0) ex = 1;
    }
    if (ex != 0) { free(tcur); free(occ); free(f1); free(f2); free(tab); return -2; }
    uint64_t mpl = sp->total_moves / sp->n_levels; if (mpl < 1) mpl = 1;

    if (sp->move_begin == 0) {
        memset(st, 0, sizeof *st);
        st->T_cur = T0; st->T_best = T0;
        memcpy(best_X, X, sz);
        double sum = 0.0; uint32_t cnt = 0;
        for (uint64_t j = 0; j < ORC_CALIB; j++) {
            orc_move m; double u; int base, second;
            orc_draw_move(q, sp, chain, j, 8, &m, &u);
            if (resolve_move(q, X, occ, tab, &m, f1, f2, &base) == ORC_NULL) continue;
            double dT = window_delta(q, X, &m, f1, f2, base, tcur, tn1, tn2, &second);
            if (dT > 0.0) { sum = sum + dT; cnt++; }
        }
        st->C0 = cnt ? (sum / (double)cnt) / (-log(sp->p0)) : 0.0;
        st->C = st->C0; st->level = 0;
    }

    for (uint64_t mi = sp->move_begin; mi < sp->move_end; mi++) {
        uint64_t lvl = mi / mpl; if (lvl > sp->n_levels - 1) lvl = sp->n_levels - 1;
        while (st->level < lvl) { st->C = st->C * sp->alpha; st->level++; }
        orc_move m; double u; int base, second;
        orc_draw_move(q, sp, chain, mi, 0, &m, &u);
        int verdict = resolve_move(q, X, occ, tab, &m, f1, f2, &base);
        if (verdict == ORC_NULL) { st->null_moves++; continue; }
        if (verdict == ORC_CLIPPED) st->clipped++;
        double dT = window_delta(q, X, &m, f1, f2, base, tcur, tn1, tn2, &second);
        if (dT > 0.0) st->uphill_seen++;
        int accept = (dT <= 0.0) || (st->C > 0.0 && u < exp(-dT / st->C));   /* Metropolis */
        if (!accept) continue;
        st->accepted++; if (dT > 0.0) st->uphill++;
        int lo = base < 0 ? 0 : base, hi = base + ORC_WIN < N ? base + ORC_WIN : N;
        apply_flips(q, X, occ, &m, f1, f2, lo, hi);
        if (tab) orc_slot_occupancy(q, X, tab);
        for (int i = 0; i < ORC_WIN; i++) {
            int n = base + i;
            if (n < 0 || n >= N) continue;
            tcur[(size_t)m.layer * N + n] = tn1[i];
            if (second) tcur[(size_t)m.layer2 * N + n] = tn2[i];
        }
        st->T_cur = st->T_cur + dT;
        if (st->T_cur < st->T_best) { st->T_best = st->T_cur; st->improved++; memcpy(best_X, X, sz); }
    }
    free(tcur); free(occ); free(f1); free(f2); free(tab);
    return 0;
}

/* ---- migration in any inference step (Sec. III-A: the decision S(n, l) places all KV data) ----
 * In orc_score a page of layer l changes tier only in its own step (n, l).  Here the step is chosen:
 * a page (l, p) whose placement differs between its steps n-1 and n, and which persists into n,
 * migrates in the inference step
 *     g = n*L + l - Y[l][n][p],   Y in 0 .. L-1,
 * any step after the page's use at (n-1, l) up to its use at (n, l); the bytes are charged to that
 * step (|M^i|, |M^o| of Eqs. 3-4 at g).  Reads and the new token's write are as before: at (n, l) the
 * page is where X[l][n] says.  Y is looked at only where a page migrates; Y = 0 everywhere is the
 * schedule of orc_score.  A value above L-1 on a migrating page counts as 0 and sets bit 30 of the
 * excess. */
static int slot_change(const orc_problem *q, const uint8_t *X, int l, int n, int p) {
    if (n < 1 || !pm_bit(q, n, p)) return 0;
    int x = x_bit(q, X, l, n, p), xp = x_bit(q, X, l, n - 1, p);
    return x == xp ? 0 : (x ? 1 : -1);
}

static int slot_of(const orc_problem *q, const uint8_t *Y, int l, int n, int p) {
    int y = Y[ix_x(q, l, n, p)];
    if (y > q->L - 1) y = 0;
    return n * q->L + l - y;
}

/* the volumes of inference step g = n*L + l, migration from whichever layers' pages move there */
void orc_slot_bytes(const orc_problem *q, const uint8_t *X, const uint8_t *Y, int g, uint64_t out[6]) {
    int L = q->L, N = q->N, n0 = g / L, l0 = g % L;
    orc_step_bytes(q, X, l0, n0, out);
    uint64_t mi = 0, mo = 0;
    for (int l = 0; l < L; l++)
        for (int n = n0; n <= n0 + 1 && n < N; n++)          /* a page of step n moves in ((n-1)L + l, nL + l] */
            for (int p = 0; p < q->P; p++) {
                int c = slot_change(q, X, l, n, p);
                if (!c || slot_of(q, Y, l, n, p) != g) continue;
                if (c > 0) mi += q->page_bytes; else mo += q->page_bytes;
            }
    out[4] = mi; out[5] = mo;
}

/* Total latency (Eq. 1 over the inference steps in execution order) and the pool after every
 * inference step (Eq. 5), simulated as it happens: at the start of token step n the pages that do
 * not persist into it are gone; in step g the pages that migrate there change tier, and the layer
 * whose step it is takes its placement (which places its new pages; its migrating pages have moved
 * by now or move here).  excess = largest overshoot of the pool over all steps; bit 31: bits on
 * pages that do not exist; bit 30: a Y out of range.  Optional: slot_t [N*L], pool [N*L]. */
double orc_score_slots(const orc_problem *q, const uint8_t *X, const uint8_t *Y, uint32_t *excess,
                       double *slot_t, uint32_t *pool_out) {
    int L = q->L, N = q->N, P = q->P;
    size_t G = (size_t)L * N;
    double *t = (double *)malloc(sizeof(double) * (G ? G : 1));
    for (size_t g = 0; g < G; g++) {
        uint64_t b[6];
        orc_slot_bytes(q, X, Y, (int)g, b);
        t[g] = orc_step_time(q, b);
    }
    double T = orc_csum(t, G);
    uint8_t *cur = (uint8_t *)calloc((size_t)L * P ? (size_t)L * P : 1, 1);
    uint64_t worst = 0;
    uint32_t flag = 0;
    for (int n = 0; n < N; n++) {
        for (int l = 0; l < L; l++)
            for (int p = 0; p < P; p++)
                if (!(n > 0 && pm_bit(q, n, p))) cur[(size_t)l * P + p] = 0;
        for (int l0 = 0; l0 < L; l0++) {
            int g = n * L + l0;
            for (int l = 0; l < L; l++)
                for (int m = n; m <= n + 1 && m < N; m++)
                    for (int p = 0; p < P; p++)
                        if (slot_change(q, X, l, m, p) && slot_of(q, Y, l, m, p) == g)
                            cur[(size_t)l * P + p] = (uint8_t)x_bit(q, X, l, m, p);
            for (int p = 0; p < P; p++) cur[(size_t)l0 * P + p] = (uint8_t)x_bit(q, X, l0, n, p);
            uint64_t occ = 0;
            for (size_t i = 0; i < (size_t)L * P; i++) occ += cur[i];
            if (pool_out) pool_out[g] = (uint32_t)occ;
            if (occ > q->cap_pages && occ - q->cap_pages > worst) worst = occ - q->cap_pages;
        }
    }
    for (int l = 0; l < L; l++)
        for (int n = 0; n < N; n++)
            for (int p = 0; p < P; p++) {
                if (X[ix_x(q, l, n, p)] && !v_bit(q, n, p)) flag |= 0x80000000u;
                if (slot_change(q, X, l, n, p) && Y[ix_x(q, l, n, p)] > L - 1) flag |= 0x40000000u;
            }
    if (excess) *excess = (uint32_t)(worst > 0x3FFFFFFFull ? 0x3FFFFFFFull : worst) | flag;
    if (slot_t) memcpy(slot_t, t, sizeof(double) * G);
    free(t); free(cur);
    return T;
}

/* Proposal mi of a chain in the annealing over migration steps: ONE Philox block, counter (mi lo,
 * mi hi, chain, stream) under the seed.  Word 0 picks one of the M migrating pages (an index in
 * 0 .. M-1 is the high word of 32 random bits x M), word 1 the new Y in 0 .. L-1, words 2 and 3 give
 * the 52 bits of the acceptance draw u in (0, 1), as in orc_draw_move.  Exported for the pins. */
void orc_draw_slot_move(uint64_t seed, uint32_t chain, uint64_t mi, uint32_t stream, uint32_t M, uint32_t L,
                        uint32_t *idx, uint32_t *ynew, double *u) {
    uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    uint32_t ctr[4] = {(uint32_t)mi, (uint32_t)(mi >> 32), chain, stream}, r[4];
    orc_philox4x32_10(ctr, key, r);
    *idx = (uint32_t)(((uint64_t)r[0] * M) >> 32);
    *ynew = (uint32_t)(((uint64_t)r[1] * L) >> 32);
    uint64_t bits = ((uint64_t)r[2] << 20) | (r[3] >> 12);
    *u = ((double)bits + 0.5) * (1.0 / 4503599627370496.0);
}

/* Annealing over the migration steps Y of a fixed placement X (the Metropolis skeleton of
 * Sec. III-B: acceptance exp(-dT/C), C0 from p0 over 256 proposals that are not applied, cooling by
 * alpha per level).  The pages that migrate are those of X: they are listed once, in the order
 * (layer, step, page), and a proposal (orc_draw_slot_move, stream 32; 40 for the calibration) names
 * one of them and a new Y.  Null if Y stays (or nothing migrates at all).  A page that enters HBM
 * earlier, or leaves it later, is in the pool during the steps between the old and the new one: if
 * one of them is full the proposal is dropped (counted as null and as clipped).
 * dT = (t' - t) at the old step + (t' - t) at the new step, in that order.
 * X must be feasible with Y at every inference step (-2 otherwise). */
int orc_refine_slots(const orc_problem *q, const orc_sa_params *sp, uint32_t chain, const uint8_t *X,
                     uint8_t *Y, orc_sa_state *st) {
    int L = q->L, N = q->N, P = q->P;
    size_t G = (size_t)L * N;
    if (sp->n_levels < 1 || L > 256 || (uint64_t)G * P >= (1ull << 32)) return -1;
    double *t = (double *)malloc(sizeof(double) * (G ? G : 1));
    uint32_t *pool = (uint32_t *)malloc(sizeof(uint32_t) * (G ? G : 1));
    uint64_t (*vol)[6] = (uint64_t (*)[6])malloc(sizeof(uint64_t[6]) * (G ? G : 1));
    uint32_t ex;
    double T0 = orc_score_slots(q, X, Y, &ex, t, pool);
    if (ex != 0) { free(t); free(pool); free(vol); return -2; }
    for (size_t g = 0; g < G; g++) orc_slot_bytes(q, X, Y, (int)g, vol[g]);
    /* the migrating pages, in the order (l, n, p) */
    uint32_t M = 0;
    for (int l = 0; l < L; l++) for (int n = 0; n < N; n++) for (int p = 0; p < P; p++) M += slot_change(q, X, l, n, p) != 0;
    uint32_t *list = (uint32_t *)malloc(sizeof(uint32_t) * (M ? M : 1));
    M = 0;
    for (int l = 0; l < L; l++) for (int n = 0; n < N; n++) for (int p = 0; p < P; p++)
        if (slot_change(q, X, l, n, p)) list[M++] = (uint32_t)ix_x(q, l, n, p);
    uint64_t mpl = sp->total_moves / sp->n_levels; if (mpl < 1) mpl = 1;
    if (sp->move_begin == 0) {
        memset(st, 0, sizeof *st);
        st->T_cur = T0; st->T_best = T0;
    }
    for (int phase = (sp->move_begin == 0 ? 0 : 1); phase < 2; phase++) {
        uint64_t first = phase == 0 ? 0 : sp->move_begin, last = phase == 0 ? ORC_CALIB : sp->move_end;
        double sum = 0.0; uint32_t cnt = 0;
        for (uint64_t mi = first; mi < last; mi++) {
            if (phase == 1) {
                uint64_t lvl = mi / mpl; if (lvl > sp->n_levels - 1) lvl = sp->n_levels - 1;
                while (st->level < lvl) { st->C = st->C * sp->alpha; st->level++; }
            }
            uint32_t idx, ydraw; double u;
            orc_draw_slot_move(sp->seed, chain, mi, phase == 0 ? 40 : 32, M, (uint32_t)L, &idx, &ydraw, &u);
            if (M == 0) { if (phase == 1) st->null_moves++; continue; }
            size_t iy = list[idx];
            int p = (int)(iy % (size_t)P), n = (int)((iy / (size_t)P) % (size_t)N), l = (int)(iy / ((size_t)P * N));
            int ynew = (int)ydraw, yold = Y[iy];
            int c = slot_change(q, X, l, n, p);
            if (ynew == yold) { if (phase == 1) st->null_moves++; continue; }
            int g_old = n * L + l - yold, g_new = n * L + l - ynew;
            /* the steps during which the page is in the pool only after the move */
            int lo = 0, hi = 0;
            if (c > 0 && g_new < g_old) { lo = g_new; hi = g_old; }
            if (c < 0 && g_new > g_old) { lo = g_old; hi = g_new; }
            int blocked = 0;
            for (int g = lo; g < hi; g++) if ((uint64_t)pool[g] + 1 > q->cap_pages) blocked = 1;
            if (blocked) { if (phase == 1) { st->null_moves++; st->clipped++; } continue; }
            uint64_t bo[6], bn[6];
            memcpy(bo, vol[g_old], sizeof bo); memcpy(bn, vol[g_new], sizeof bn);
            int k = c > 0 ? 4 : 5;
            bo[k] -= q->page_bytes; bn[k] += q->page_bytes;
            double to = orc_step_time(q, bo), tn = orc_step_time(q, bn);
            double dT = (to - t[g_old]) + (tn - t[g_new]);
            if (phase == 0) { if (dT > 0.0) { sum = sum + dT; cnt++; } continue; }
            if (dT > 0.0) st->uphill_seen++;
            int accept = (dT <= 0.0) || (st->C > 0.0 && u < exp(-dT / st->C));
            if (!accept) continue;
            st->accepted++; if (dT > 0.0) st->uphill++;
            Y[iy] = (uint8_t)ynew;
            memcpy(vol[g_old], bo, sizeof bo); memcpy(vol[g_new], bn, sizeof bn);
            t[g_old] = to; t[g_new] = tn;
            if (c > 0) { for (int g = g_new; g < g_old; g++) pool[g]++; for (int g = g_old; g < g_new; g++) pool[g]--; }
            else { for (int g = g_old; g < g_new; g++) pool[g]++; for (int g = g_new; g < g_old; g++) pool[g]--; }
            st->T_cur = st->T_cur + dT;
            if (st->T_cur < st->T_best) { st->T_best = st->T_cur; st->improved++; }
        }
        if (phase == 0) {
            st->C0 = cnt ? (sum / (double)cnt) / (-log(sp->p0)) : 0.0;
            st->C = st->C0; st->level = 0;
        }
    }
    free(t); free(pool); free(vol); free(list);
    return 0;
}

/* ---- replica exchange between the chains (parallel tempering) ---------------
 * Not in the paper (its search is one annealing run): the standard exchange
 * step of parallel tempering (Swendsen & Wang 1986; Geyer 1991), offered
 * between two slices of the annealing.  Chains that stand next to each other in
 * the chain order, (a, a+1) with a = round mod 2, round mod 2 + 2, ..., trade
 * their temperatures (the current one C and the initial one C0; each chain goes
 * on cooling from what it holds) with the Metropolis probability of the pair,
 *     min(1, exp((1/C_a - 1/C_b) (T_a - T_b))),   T = the chain's current cost,
 * so the better schedule tends to end up at the lower temperature.  One uniform
 * number per pair and round: Philox counter (round, a, 16), the mapping to (0,1)
 * that the acceptance test of a move uses.  A pair with a temperature that is
 * not positive is left alone.  Returns the number of pairs that traded. */
uint32_t orc_exchange(uint64_t seed, uint64_t round, uint32_t n, const double *T, double *C, double *C0) {
    uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    uint32_t traded = 0;
    for (uint32_t a = (uint32_t)(round & 1u); a + 1 < n; a += 2) {
        uint32_t b = a + 1;
        if (!(C[a] > 0.0) || !(C[b] > 0.0)) continue;
        uint32_t ctr[4] = {(uint32_t)round, (uint32_t)(round >> 32), a, 16u}, r[4];
        orc_philox4x32_10(ctr, key, r);
        uint64_t bits = ((uint64_t)r[0] << 20) | (r[1] >> 12);
        double u = ((double)bits + 0.5) * (1.0 / 4503599627370496.0);
        double d = (1.0 / C[a] - 1.0 / C[b]) * (T[a] - T[b]);
        if (d >= 0.0 || u < exp(d)) {
            double t = C[a]; C[a] = C[b]; C[b] = t;
            t = C0[a]; C0[a] = C0[b]; C0[b] = t;
            traded++;
        }
    }
    return traded;
}

/* ---- the (W, R) look-ahead policy and its search (Sec. III-B) ---------------
 * The paper anneals two scalars of a placement policy: W, how many coming
 * token steps are looked at, and R, the share of the pages "qualified for
 * migration" that really migrate.  It gives the policy in two sentences; this
 * is the reading taken here, step by step, once per token step n (one decision
 * for all layers, on the shared pool of cap_pages):
 *   1. pages that do not hold the same data as one step earlier leave the pool
 *      (a page born at n starts outside, like every page at n = 0);
 *   2. collect the existing pages that are read in steps n .. n+W-1, with their
 *      read frequency f there (summed over the planes);
 *   3. rank them, f descending, ties to the lower l*P+p ("priority queue"); the
 *      first cap_pages of the ranking are the wanted set;
 *   4. qualified for migration: the wanted pages that are not in the pool, in
 *      rank order; the first m = round(R * their number) of them migrate in,
 *      R = r10 / 10 and m = (r10 * number + 5) div 10;
 *   5. if the pool would overflow, as many pool pages that are not wanted leave,
 *      least-read-in-the-window first, ties to the lower l*P+p;
 *   6. the pool is the placement of step n in every layer's row.
 * The schedule is then scored like any other (Eqs. 1-5): T(W, R). */
void orc_wr_policy(const orc_problem *q, uint32_t W, uint32_t r10, uint8_t *X) {
    int L = q->L, N = q->N, P = q->P;
    size_t M = (size_t)L * P;
    uint8_t *pool = (uint8_t *)calloc(M, 1), *wanted = (uint8_t *)malloc(M);
    int64_t *f = (int64_t *)malloc(M * sizeof(int64_t));
    rank_item *it = (rank_item *)malloc(M * sizeof(rank_item));
    for (int n = 0; n < N; n++) {
        /* 1 */
        for (int l = 0; l < L; l++)
            for (int p = 0; p < P; p++)
                if (!pm_bit(q, n, p)) pool[(size_t)l * P + p] = 0;
        /* 2 */
        int end = (uint64_t)n + W < (uint64_t)N ? n + (int)W : N;
        size_t cnt = 0;
        for (int l = 0; l < L; l++)
            for (int p = 0; p < P; p++) {
                size_t i = (size_t)l * P + p;
                f[i] = 0;
                wanted[i] = 0;
                if (!v_bit(q, n, p)) continue;
                for (int m = n; m < end; m++)
                    for (int k = 0; k < q->K; k++) f[i] += a_bit(q, l, m, k, p);
                if (f[i] > 0) { it[cnt].key = f[i]; it[cnt].idx = i; cnt++; }
            }
        /* 3 */
        qsort(it, cnt, sizeof(rank_item), rank_cmp);
        size_t nw = cnt < q->cap_pages ? cnt : (size_t)q->cap_pages;
        for (size_t c = 0; c < nw; c++) wanted[it[c].idx] = 1;
        /* 4 */
        size_t nq = 0;
        for (size_t c = 0; c < nw; c++)
            if (!pool[it[c].idx]) nq++;
        size_t m_in = (size_t)(((uint64_t)r10 * nq + 5) / 10);
        size_t in_pool = 0;
        for (size_t i = 0; i < M; i++) in_pool += pool[i];
        /* 5 */
        if (in_pool + m_in > q->cap_pages) {
            size_t need = in_pool + m_in - (size_t)q->cap_pages, ne = 0;
            rank_item *ev = (rank_item *)malloc(M * sizeof(rank_item));
            for (size_t i = 0; i < M; i++)
                if (pool[i] && !wanted[i]) { ev[ne].key = -f[i]; ev[ne].idx = i; ne++; }
            qsort(ev, ne, sizeof(rank_item), rank_cmp);          /* -f descending = f ascending */
            for (size_t c = 0; c < need && c < ne; c++) pool[ev[c].idx] = 0;
            free(ev);
        }
        /* 4, carried out */
        size_t taken = 0;
        for (size_t c = 0; c < nw && taken < m_in; c++)
            if (!pool[it[c].idx]) { pool[it[c].idx] = 1; taken++; }
        /* 6 */
        for (int l = 0; l < L; l++)
            for (int p = 0; p < P; p++) X[ix_x(q, l, n, p)] = pool[(size_t)l * P + p];
    }
    free(pool); free(wanted); free(f); free(it);
}

/* The annealing over (W, R), Sec. III-B: proposals are a window move (W by
 * -2, -1, +1 or +2), a ratio move (R by -0.1 or +0.1) or both at once, with
 * probabilities op_prob[0..2] (the paper: 0.4, 0.4, 0.2); Metropolis acceptance;
 * the temperature starts where an average uphill proposal from the start state
 * is accepted with probability p0 and is multiplied by alpha after every level
 * of total_moves / n_levels proposals; the search ends when the budget is spent,
 * when the best cost improved by less than stop_rel (the paper: 0.1 %) over a
 * level, or when the temperature falls below c_min_frac times its start value.
 * Proposals that leave 1 <= W <= w_max or 0 <= R <= 1 are counted and skipped.
 * Proposal i uses Philox block (i, 0, 0, 16) under the seed: word 0 picks the
 * operator, the top two bits of word 1 the window step, the top bit of word 2 the
 * ratio step, u = (word 3 + 0.5) / 2^32; the 32 calibration proposals use
 * stream 24.  table: [w_max][11] costs T(W, r10) (W from 1), < 0 where not yet
 * evaluated; filled on demand.  Returns the number of proposals made. */
typedef struct {
    uint32_t w_max, w0, r10_0, n_levels;
    uint64_t seed, total_moves;
    double p0, alpha, op_prob[3], stop_rel, c_min_frac;
} orc_wr_params;

typedef struct {
    uint32_t best_w, best_r10, cur_w, cur_r10, levels_done, stop_reason;   /* 0 budget, 1 stalled, 2 cold */
    uint64_t proposals, accepted, out_of_range, evaluated;
    double best_T, cur_T, c0;
} orc_wr_result;

static double wr_cost(const orc_problem *q, uint32_t w_max, double *table, uint32_t w, uint32_t r10, uint8_t *X,
                      uint64_t *evaluated) {
    double *slot = &table[(size_t)(w - 1) * 11 + r10];
    (void)w_max;
    if (*slot < 0.0) {
        orc_wr_policy(q, w, r10, X);
        *slot = orc_score(q, X, NULL, NULL, NULL, NULL);
        (*evaluated)++;
    }
    return *slot;
}

/* Proposal i from state (w, r10): returns 0 if it leaves the grid.  Exported for the pins. */
int orc_wr_propose(const orc_wr_params *sp, uint64_t i, uint32_t stream, uint32_t w, uint32_t r10, uint32_t *w2,
                   uint32_t *r2, double *u) {
    uint32_t ctr[4] = {(uint32_t)i, (uint32_t)(i >> 32), 0, stream};
    uint32_t key[2] = {(uint32_t)sp->seed, (uint32_t)(sp->seed >> 32)}, a[4];
    orc_philox4x32_10(ctr, key, a);
    uint64_t th0 = (uint64_t)(sp->op_prob[0] * 4294967296.0);
    uint64_t th1 = (uint64_t)((sp->op_prob[0] + sp->op_prob[1]) * 4294967296.0);
    int op = (uint64_t)a[0] < th0 ? 0 : (uint64_t)a[0] < th1 ? 1 : 2;
    static const int dws[4] = {-2, -1, 1, 2};
    int dw = op != 1 ? dws[a[1] >> 30] : 0;
    int dr = op != 0 ? ((a[2] >> 31) ? 1 : -1) : 0;
    *u = ((double)a[3] + 0.5) * (1.0 / 4294967296.0);
    int64_t nw = (int64_t)w + dw, nr = (int64_t)r10 + dr;
    if (nw < 1 || nw > (int64_t)sp->w_max || nr < 0 || nr > 10) return 0;
    *w2 = (uint32_t)nw; *r2 = (uint32_t)nr;
    return 1;
}

uint64_t orc_wr_search(const orc_problem *q, const orc_wr_params *sp, double *table, orc_wr_result *res) {
    uint8_t *X = (uint8_t *)malloc((size_t)q->L * q->N * q->P);
    memset(res, 0, sizeof *res);
    uint32_t w = sp->w0, r10 = sp->r10_0;
    double T = wr_cost(q, sp->w_max, table, w, r10, X, &res->evaluated);
    res->best_w = w; res->best_r10 = r10; res->best_T = T;
    double sum = 0.0; uint32_t cnt = 0;
    for (uint64_t j = 0; j < 32; j++) {
        uint32_t w2, r2; double u;
        if (!orc_wr_propose(sp, j, 24, w, r10, &w2, &r2, &u)) continue;
        double dT = wr_cost(q, sp->w_max, table, w2, r2, X, &res->evaluated) - T;
        if (dT > 0.0) { sum = sum + dT; cnt++; }
    }
    res->c0 = cnt ? (sum / (double)cnt) / (-log(sp->p0)) : 0.0;
    double C = res->c0, best_at_level_start = res->best_T;
    uint64_t mpl = sp->total_moves / sp->n_levels; if (mpl < 1) mpl = 1;
    uint64_t i = 0;
    res->stop_reason = 0;
    for (; i < sp->total_moves; i++) {
        if (i > 0 && i % mpl == 0) {                              /* a level ends */
            res->levels_done++;
            if (best_at_level_start - res->best_T < sp->stop_rel * best_at_level_start) { res->stop_reason = 1; break; }
            best_at_level_start = res->best_T;
            C = C * sp->alpha;
            if (C < sp->c_min_frac * res->c0) { res->stop_reason = 2; break; }
        }
        uint32_t w2, r2; double u;
        res->proposals++;
        if (!orc_wr_propose(sp, i, 16, w, r10, &w2, &r2, &u)) { res->out_of_range++; continue; }
        double T2 = wr_cost(q, sp->w_max, table, w2, r2, X, &res->evaluated);
        double dT = T2 - T;
        int accept = (dT <= 0.0) || (C > 0.0 && u < exp(-dT / C));    /* Metropolis */
        if (!accept) continue;
        res->accepted++;
        w = w2; r10 = r2; T = T2;
        if (T < res->best_T) { res->best_T = T; res->best_w = w; res->best_r10 = r10; }
    }
    res->cur_w = w; res->cur_r10 = r10; res->cur_T = T;
    free(X);
    return res->proposals;
}
