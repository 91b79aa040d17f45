// Scorer for rows of more than 68 words under the conditions of the rowblock scorer (a single
// decoding sequence, one page written per step: on every 64-step tile the words of a row are a
// FULL prefix, a few words that need masks and then words in which no page exists yet).
//
// The row is walked in G = ceil(Wd / 64) segments of equal width, the least of 40, 48, 56 and 64
// words that covers it (the width is a template parameter: every loop over a segment has a fixed
// trip count); a (layer, pass of 32 token steps, segment) is one unit, handled the way the
// rowblock scorer handles a pass: a wavefront fetches the 33 row pieces of its schedule as 16-byte
// vectors (a piece is up to 256 contiguous bytes), parks them in LDS with a row stride of 66
// words, and two lanes share a row, one on the even words and one on the odd.  The trace words of
// a unit (binary digit planes of the read weights) are fetched once per workgroup of four
// schedules into a double-buffered LDS slot, one unit ahead; the row pieces two units ahead.
// Counters stay in registers over the segments of a pass; Eqs. 2-4 and the summation tree run
// once per layer.
//
// The last segment ends at the end of the row: it overlaps its neighbour when the segments do not
// tile the row exactly and owns only the words that its neighbour does not reach.  Masked words,
// the word that receives the step's token and the words past the sequence's end are handled by
// the segment that owns them.
#include "kvp_internal.h"

namespace {

typedef uint32_t s4u __attribute__((ext_vector_type(4), aligned(4)));   // rows are only 4-byte aligned

constexpr int SQ = 4;           // schedules (= wavefronts) per workgroup
constexpr int SR = 32;          // token steps per pass (two lanes per step)
constexpr int SEG = 64;         // most words per segment
constexpr int SRS = SEG + 2;    // LDS row stride, 2 (mod 4): the 32 lanes served together hit 32 banks
constexpr int STW = 6;          // words at the end of a row that may need masks
constexpr int STPL = SR * SRS;  // words of one digit plane in a slot

__device__ __forceinline__ void seg_put4(uint32_t *p, s4u v) { p[0] = v.x; p[1] = v.y; p[2] = v.z; p[3] = v.w; }
__device__ __forceinline__ uint32_t seg_pair_sum(uint32_t v) {        // v + the other lane of the row
    return v + (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xf, 0xf, false);   // quad_perm [1,0,3,2]
}

// KB: digit planes (1 or 2); POW2: L is a power of two >= 2 (the summation tree is kept on chip:
// layers in bit-reversed order, binary counter of partial sums), else step latencies go to [S][L][N];
// SPP: 16-byte parts of a row piece (a segment has 4 SPP words).
template <int KB, bool POW2, int SPP>
__global__ __launch_bounds__(SQ * 64) void score_rowseg_kernel(
    DevProblem q, const uint32_t *__restrict__ Aw, const uint32_t *__restrict__ X, uint32_t S, uint32_t tiles,
    uint32_t nb_total, uint32_t log2L, double *__restrict__ blocksum, double *__restrict__ tglobal,
    uint32_t *__restrict__ tileflag, uint32_t *__restrict__ counters, uint32_t *__restrict__ occ_out) {
    extern __shared__ double smem_d[];
    constexpr int SXV = ((SR + 1) * SPP + 63) / 64;                    // row vectors per lane and unit (<= 9)
    constexpr int TV = (KB * SR * SPP + SQ * 64 - 1) / (SQ * 64);      // trace vectors per thread and unit (<= 2 KB)
    const uint32_t L = q.L, N = q.N, Wd = q.Wd;
    const uint32_t G = (Wd + SEG - 1) / SEG;                           // segments of a row (>= 2)
    constexpr uint32_t spp = SPP, segw = 4 * SPP;                      // G * segw >= Wd (the host's choice of SPP)
    const uint32_t tid = threadIdx.x;
    const int lane = lane_id();
    const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane((int)(tid / KVP_WAVE));
    uint32_t tile, group;                                             // see xcd_pair for the placement
    if (!xcd_pair(tiles, (S + SQ - 1) / SQ, tile, group)) return;
    const uint32_t s = group * SQ + wave;
    const bool has_s = s < S;
    const uint32_t sc = has_s ? s : S - 1;                            // spare wavefronts shadow the last schedule
    const uint32_t n0 = tile * 64;
    const uint32_t rows = min(64u, N - n0);
    uint32_t *xbuf = (uint32_t *)smem_d + (size_t)wave * (SR + 1) * SRS;
    uint32_t *tbuf = (uint32_t *)smem_d + (size_t)SQ * (SR + 1) * SRS; // two slots of KB * STPL words
    const uint32_t r = (uint32_t)lane >> 1, h2 = (uint32_t)lane & 1u;
    // The words of a row on this tile: [0, pfw2) FULL at every step (no masks needed), [pfw2, wend) with
    // masks (at most STW: the host checks), [wend, Wd) without a page at any step (only stray bits).
    const uint32_t pfw2 = q.tile_pfw[tile] & ~1u, wend = q.tile_end[tile];
    const uint32_t tw = wend - pfw2;

    // What a segment covers: words [start, start + segw) are loaded; it OWNS the words [own_lo, own_hi)
    // (the last segment ends at the end of the row and owns what the one before it does not reach).
    auto seg_start = [&](uint32_t g) { return g + 1 < G ? g * segw : Wd - segw; };
    auto seg_own_lo = [&](uint32_t g) { return g * segw; };
    auto seg_own_hi = [&](uint32_t g) { return g + 1 < G ? (g + 1) * segw : Wd; };

    // the lane's own step
    const uint32_t rho = h2 * SR + r;
    const bool active = rho < rows;
    const uint32_t n = n0 + (active ? rho : rows - 1);                // idle lanes shadow the last row
    const uint32_t wr_n = q.wr[n], wsel = q.wsel[n];
    const uint32_t wmw = q.Wm[(size_t)n * Wd + wsel];
    uint32_t vt[STW], pt[STW];
#pragma unroll
    for (int t = 0; t < STW; t++) {
        const uint32_t w = min(pfw2 + t, Wd - 1);
        vt[t] = q.V[(size_t)n * Wd + w];
        pt[t] = q.Pm[(size_t)n * Wd + w];
    }
    // vector slots of the lane: byte offsets from the first row piece of a unit, word offsets in LDS
    uint32_t xrel[SXV], xlds[SXV], trel[TV], tlds[TV];
#pragma unroll
    for (int jv = 0; jv < SXV; jv++) {
        const uint32_t vi = min((uint32_t)lane + 64u * jv, (SR + 1) * spp - 1);   // spare lanes repeat the last vector
        const uint32_t row = vi / spp, part = vi - row * spp;
        xrel[jv] = 4 * (row * Wd + 4 * part);
        xlds[jv] = row * SRS + 4 * part;
    }
#pragma unroll
    for (int jt = 0; jt < TV; jt++) {
        const uint32_t ti = min(tid + 256u * jt, KB * SR * spp - 1);   // spare threads repeat the last vector
        const uint32_t k = ti / (SR * spp), rem = ti - k * (SR * spp);
        const uint32_t row = rem / spp, part = rem - row * spp;
        trel[jt] = 4 * ((row * KB + k) * Wd + 4 * part);
        tlds[jt] = k * STPL + row * SRS + 4 * part;
    }
    const uint32_t sched_words = L * N * Wd;                           // < 2^29 (checked by the host)

    struct Stage { s4u x[SXV]; };
    Stage st0, st1;
    s4u tr[TV];
    auto layer_of = [&](uint32_t i) { return POW2 ? (__brev(i) >> (32 - log2L)) : i; };
    // unit v of a layer: pass v / G, segment v % G; the units of all layers follow each other
    auto next_unit = [&](uint32_t &i, uint32_t &v) {
        v++;
        if (v == 2 * G) { v = 0; i = min(i + 1, L - 1); }             // past the last layer: its units again (never used)
    };
    // Addresses are a wavefront-uniform base plus a 32-bit byte offset per lane.  A unit whose 33 row
    // pieces all lie inside the schedule (no step before step 0, none past the trace) needs no clamping;
    // clamped requests fetch words that are never looked at.
    const char *Xs = (const char *)(X + (size_t)sc * sched_words);
    const bool edge_tile = rows < 64;
    auto issue_x = [&](Stage &st, uint32_t i, uint32_t v) __attribute__((always_inline)) {
        const uint32_t p = v >= G ? 1u : 0u, g = v - p * G;
        const uint32_t l = layer_of(i);
        const int rowbase = 4 * ((int)((l * N + n0 + SR * p) * Wd) - (int)Wd);   // the step before the pass; < 0 at step 0
        const int before = rowbase + 4 * (int)seg_start(g);
        if (rowbase >= 0 && !edge_tile) {
#pragma unroll
            for (int jv = 0; jv < SXV; jv++) st.x[jv] = *(const s4u *)(Xs + ((uint32_t)before + xrel[jv]));
        } else {
            const int hi = 4 * ((int)sched_words - 4);
#pragma unroll
            for (int jv = 0; jv < SXV; jv++) st.x[jv] = *(const s4u *)(Xs + (uint32_t)min(max(before + (int)xrel[jv], 0), hi));
        }
    };
    auto issue_t = [&](uint32_t i, uint32_t v) __attribute__((always_inline)) {
        const uint32_t p = v >= G ? 1u : 0u, g = v - p * G;
        const uint32_t first = 4 * ((layer_of(i) * N + n0 + SR * p) * KB * Wd + seg_start(g));
        const char *Ab = (const char *)Aw;
        if (!edge_tile) {
#pragma unroll
            for (int jt = 0; jt < TV; jt++) tr[jt] = *(const s4u *)(Ab + (first + trel[jt]));
        } else {
            const uint32_t hi = 4 * (L * N * KB * Wd - 4);
#pragma unroll
            for (int jt = 0; jt < TV; jt++) tr[jt] = *(const s4u *)(Ab + min(first + trel[jt], hi));
        }
    };
    auto commit_t = [&](uint32_t slot) __attribute__((always_inline)) {
        uint32_t *dst = tbuf + slot * KB * STPL;
#pragma unroll
        for (int jt = 0; jt < TV; jt++) seg_put4(dst + tlds[jt], tr[jt]);
    };

    const uint32_t row_off = r * SRS;
    const bool very_first = n0 == 0 && r == 0;                         // the lane's row in pass 0 is step 0
    uint32_t fl_acc = 0, occ_acc = 0;
    double stk[6] = {0.0, 0.0, 0.0, 0.0, 0.0, 0.0}, total = 0.0;
    uint32_t hr = 0, hw = 0, oc = 0, mi = 0, mg = 0;                   // the lane's own step, this layer
    // counters of the lane's half row over the segments of a pass
    uint32_t hrk[KB], c_oc = 0, c_mi = 0, c_mg = 0, c_hw = 0;
#pragma unroll
    for (int k = 0; k < KB; k++) hrk[k] = 0;

    // one unit: stage st holds the row pieces of (layer i-th in visiting order, unit v); its trace
    // words are in slot `slot`
    auto unit = [&](Stage &st, const uint32_t slot, uint32_t i, uint32_t v) __attribute__((always_inline)) {
        const uint32_t p = v >= G ? 1u : 0u, g = v - p * G;
#pragma unroll
        for (int jv = 0; jv < SXV; jv++) seg_put4(xbuf + xlds[jv], st.x[jv]);
        uint32_t i1 = i, v1 = v;
        next_unit(i1, v1);
        issue_t(i1, v1);                                               // trace words of the next unit
        next_unit(i1, v1);
        issue_x(st, i1, v1);                                           // row pieces of two units ahead
        __syncthreads();                                               // this unit's trace slot is complete
        // (addresses below are rebuilt in every unit from these two copies: kept across the loops they
        // would occupy dozens of registers)
        uint32_t ro = row_off, hv = h2;
        asm volatile("" : "+v"(ro), "+v"(hv));
        const uint32_t *cur = xbuf + SRS + ro, *prv = xbuf + ((p == 0 && very_first) ? (uint32_t)SRS : ro);
        const uint32_t *ts = tbuf + slot * KB * STPL + ro;
        const uint32_t start = seg_start(g), own_lo = seg_own_lo(g), own_hi = seg_own_hi(g);
        // the unmasked words among the owned ones, relative to start: the word loop counts [lo, hi)
        const uint32_t lo = own_lo - start, hi = min(own_hi, max(pfw2, own_lo)) - start;
        auto word = [&](uint32_t w) __attribute__((always_inline)) {
            const uint32_t raw = cur[w], d = raw ^ prv[w];
#pragma unroll
            for (int k = 0; k < KB; k++) hrk[k] += __popc(raw & ts[k * STPL + w]);
            c_oc += __popc(raw);
            c_mi += __popc(d & raw);
            c_mg += __popc(d);
        };
        if (lo == 0 && hi == segw) {                                   // a whole segment of unmasked words
#pragma unroll 8
            for (uint32_t j = 0; j < segw / 2; j++) word(2 * j + hv);
        } else if (hi > lo) {                                          // the lane's words 2 j + hv in [lo, hi)
            const uint32_t j_lo = (lo + 1 - hv) >> 1, j_hi = (hi + 1 - hv) >> 1;
            for (uint32_t j = j_lo; j < j_hi; j++) word(2 * j + hv);
        }
        const bool own = hv == p;
        if (pfw2 < own_hi && wend > own_lo) {
            // the masked words that this segment owns, taken by the lane that owns the row
            uint32_t flt = 0;
#pragma unroll
            for (int t = 0; t < STW; t++) {
                if ((uint32_t)t < tw && pfw2 + t >= own_lo && pfw2 + t < own_hi) {
                    const uint32_t w = pfw2 + t - start;
                    const uint32_t vv = own ? vt[t] : 0u, pp = own ? pt[t] : 0u;
                    const uint32_t raw = cur[w], x = raw & vv;
                    flt |= raw & ~vv;
                    const uint32_t d = (x ^ prv[w]) & pp;
#pragma unroll
                    for (int k = 0; k < KB; k++) hrk[k] += __popc(x & ts[k * STPL + w]);
                    c_oc += __popc(x);
                    c_mi += __popc(d & x);
                    c_mg += __popc(d);
                }
            }
            fl_acc |= (own && active) ? flt : 0u;
        }
        if (wend < own_hi) {                                           // bits where no page exists: the row's lanes take turns
            uint32_t fdead = 0;
            const uint32_t first = max(wend, own_lo) - start;
            for (uint32_t w = first + ((first ^ hv) & 1u); w < own_hi - start; w += 2) fdead |= cur[w];
            fl_acc |= (SR * p + r < rows) ? fdead : 0u;
        }
        // the word that receives the step's token, in the segment that counts it (written pages exist:
        // no alive mask needed); every lane looks, the row's owner keeps it
        {
            const bool here = wsel >= own_lo && wsel < own_hi;
            const uint32_t col = here ? wsel - start : 0u;
            c_hw += here ? (uint32_t)__popc(cur[col] & wmw) : 0u;
        }
        if (g + 1 == G) {                                              // the pass is complete
            uint32_t c_hr = 0;
#pragma unroll
            for (int k = 0; k < KB; k++) { c_hr += hrk[k] << k; hrk[k] = 0; }
            c_hr = seg_pair_sum(c_hr); c_oc = seg_pair_sum(c_oc); c_mi = seg_pair_sum(c_mi); c_mg = seg_pair_sum(c_mg);
            if (p == 0 || h2) { hr = c_hr; oc = c_oc; mi = c_mi; mg = c_mg; hw = c_hw; }
            c_oc = c_mi = c_mg = c_hw = 0;
        }
        commit_t(slot ^ 1u);                                           // arrived while this unit was scored
    };
    // once per layer, after both passes: Eqs. 2-4 and the layer's place in the summation tree
    auto layer_end = [&](uint32_t i, uint32_t acc_n) __attribute__((always_inline)) {
        const uint32_t l = layer_of(i);
        const uint32_t mo = mg - mi;
        double t = step_time(q, hr, hw, mi, mo, acc_n, wr_n);
        t = active ? t : 0.0;                                          // rows past the end of the trace pad with +0.0
        occ_acc += oc;
        if (counters && has_s && active)
            *(uint4 *)(counters + (((size_t)s * L + l) * N + n) * 4) = make_uint4(hr, hw, mi, mo);
        if (POW2) {
            // folds of the summation tree that join the steps of one block (steps are two lanes apart)
            for (uint32_t m = (64u >> log2L) >> 1; m >= 1; m >>= 1) t = fold_xor_f64(t, 2 * m);
            // folds that join layers: binary counter over the bit-reversed visiting order
            double carry = t;
            bool parked = false;
#pragma unroll
            for (int j = 0; j < 6; j++) {
                if (!parked && (uint32_t)j < log2L) {
                    if (((i >> j) & 1u) == 0) { stk[j] = carry; parked = true; }
                    else carry = stk[j] + carry;
                }
            }
            if (!parked) total = carry;                                // only at the last layer
        } else if (has_s && active) {
            tglobal[((size_t)s * L + l) * N + n] = t;
        }
    };
    {
        uint32_t i1 = 0, v1 = 0;
        issue_t(0, 0);
        issue_x(st0, 0, 0);
        next_unit(i1, v1);
        issue_x(st1, i1, v1);
        commit_t(0);
    }
    uint32_t acc_nx = q.acc[(size_t)layer_of(0) * N + n];              // read units of the lane's step
    for (uint32_t i = 0; i < L; i++) {
        const uint32_t acc_n = acc_nx;
        acc_nx = q.acc[(size_t)layer_of(min(i + 1, L - 1)) * N + n];
        for (uint32_t v = 0; v < 2 * G; v += 2) {
            unit(st0, 0, i, v);
            unit(st1, 1, i, v + 1);
        }
        layer_end(i, acc_n);
    }
    if (!has_s) return;
    if (POW2) {
        const uint32_t bpl = 64u >> log2L;                             // block b of the tile: steps [b*bpl, (b+1)*bpl)
        if ((r & (bpl - 1)) == 0 && rho < rows) blocksum[(size_t)s * nb_total + (size_t)tile * L + rho / bpl] = total;
    }
    uint32_t ex = 0;
    if (active) {
        if (occ_out) occ_out[(size_t)s * N + n] = occ_acc;            // Eq. 5 per token step
        ex = occ_acc > q.cap ? occ_acc - q.cap : 0;
    }
    ex = wave_max_u32(ex);
    const uint32_t fl = wave_or_u32(fl_acc);
    if (lane == 0) tileflag[(size_t)s * tiles + tile] = ex | (fl ? 0x80000000u : 0u);
}

}  // namespace

int kvp_blocksum_from_t_launch(kvp_ctx *ctx, uint32_t S, uint32_t nb_total);

// Returns KVP_OK if launched, 1 if this kernel does not cover the shape, <0 on error.
int kvp_score_rowseg_launch(kvp_ctx *ctx, const uint32_t *X, uint32_t S, uint32_t tiles, uint32_t nb_total,
                            uint32_t *counters, uint32_t *occ) {
    const DevProblem &q = ctx->dp;
    if (!ctx->aw || !q.single_write || q.Wd <= 68) return 1;
    const uint32_t KB = ctx->kb;
    if (ctx->max_tail > STW || KB > 2) return 1;
    // 32-bit (signed) byte offsets inside the digit planes and inside a schedule, the rows that a
    // ragged last tile asks for past the end included (they are clamped after the addition)
    if (((size_t)q.L * q.N + 64) * KB * q.Wd >= (1ull << 29)) return 1;
    uint32_t log2L = 0;
    while ((1u << log2L) < q.L) log2L++;
    const bool pow2 = q.L >= 2 && q.L <= 64 && (1u << log2L) == q.L;
    const size_t lds = ((size_t)SQ * (SR + 1) * SRS + 2 * (size_t)KB * SR * SRS) * 4;
    const uint64_t nwg = xcd_grid(tiles, (S + SQ - 1) / SQ);
    if (nwg > 0x7FFFFFFFull) return 1;
    if (!pow2) {
        int rc = kvp_ensure(ctx, (void **)&ctx->d_tglobal, &ctx->tglobal_cap, (size_t)S * q.L * q.N * sizeof(double));
        if (rc) return rc;
    }
    dim3 grid((uint32_t)nwg), block(SQ * 64);
    const uint32_t G = (q.Wd + SEG - 1) / SEG, need = (q.Wd + G - 1) / G;   // words a segment has to cover: 33..64
#define KVP_GO(KK, PP, SS)                                                                                         \
    do {                                                                                                           \
        KVP_HIP(hipFuncSetAttribute((const void *)score_rowseg_kernel<KK, PP, SS>,                                 \
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));                       \
        score_rowseg_kernel<KK, PP, SS><<<grid, block, lds, ctx->stream>>>(q, ctx->aw, X, S, tiles, nb_total,      \
                                                                           log2L, ctx->d_blocksum,                 \
                                                                           ctx->d_tglobal, ctx->d_tileflag,        \
                                                                           counters, occ);                         \
    } while (0)
#define KVP_W(KK, PP)                                                                                              \
    do {                                                                                                           \
        if (need <= 40) KVP_GO(KK, PP, 10);                                                                        \
        else if (need <= 48) KVP_GO(KK, PP, 12);                                                                   \
        else if (need <= 56) KVP_GO(KK, PP, 14);                                                                   \
        else KVP_GO(KK, PP, 16);                                                                                   \
    } while (0)
    if (KB == 1) { if (pow2) KVP_W(1, true); else KVP_W(1, false); }
    else { if (pow2) KVP_W(2, true); else KVP_W(2, false); }
#undef KVP_W
#undef KVP_GO
    KVP_HIP(hipGetLastError());
    ctx->last_kernel = KVP_SCORE_ROWSEG;
    if (!pow2) return kvp_blocksum_from_t_launch(ctx, S, nb_total);
    return KVP_OK;
}
