// Host side of libkvp: context, trace upload, argument checks.  gfx950 only.
#include <math.h>
#include <new>
#include <stdlib.h>
#include <string.h>

#include "kvp_internal.h"

int kvp_trace_totals_launch(kvp_ctx *ctx, uint32_t *acc, uint32_t *wr, uint32_t *wsel);

thread_local int kvp_tls_hip_error = 0;
thread_local int kvp_tls_hip_line = 0;

extern "C" int kvp_last_hip_error(int *line) {
    if (line) *line = kvp_tls_hip_line;
    return kvp_tls_hip_error;
}

int kvp_ensure(kvp_ctx *ctx, void **p, size_t *cap, size_t bytes) {
    if (bytes <= *cap && *p) return KVP_OK;
    if (ctx->no_alloc) return KVP_ESHAPE;             // the caller cannot allocate and what it brought is too small
    if (*p) {
        KVP_HIP(hipStreamSynchronize(ctx->stream));   // earlier work may still read the old buffer
        KVP_HIP(hipFree(*p));
        *p = nullptr; *cap = 0;
    }
    if (bytes == 0) bytes = 16;
    KVP_HIP(hipMalloc(p, bytes));
    *cap = bytes;
    return KVP_OK;
}

static void free_dev(void *p) { if (p) (void)hipFree(p); }

void kvp_free_chains(kvp_ctx *ctx) {
    free_dev(ctx->d_X); free_dev(ctx->d_cnt); free_dev(ctx->d_occ); free_dev(ctx->d_state);
    free_dev(ctx->d_log); free_dev(ctx->d_cost); free_dev(ctx->d_excess); free_dev(ctx->d_argmin); free_dev(ctx->d_slot);
    free_dev(ctx->d_Xbest);
    ctx->d_X = ctx->d_cnt = ctx->d_occ = ctx->d_log = ctx->d_excess = ctx->d_argmin = ctx->d_slot = ctx->d_Xbest = nullptr;
    ctx->d_state = nullptr; ctx->d_cost = nullptr;
    ctx->log_cap = 0; ctx->has_chains = false; ctx->moves_done = 0;
}

extern "C" int kvp_create(kvp_ctx **out, int device, void *hip_stream) {
    if (!out) return KVP_EINVAL;
    *out = nullptr;
    int ndev = 0;
    KVP_HIP(hipGetDeviceCount(&ndev));
    if (device < 0 || device >= ndev) return KVP_EINVAL;
    KVP_HIP(hipSetDevice(device));
    {
        const int rc = kvp_static_scratch_init(device);
        if (rc) return rc;
    }
    kvp_ctx *c = new (std::nothrow) kvp_ctx();
    if (!c) return KVP_ENOMEM;
    c->device = device;
    c->stream = (hipStream_t)hip_stream;
    int cus = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess || cus < 1) cus = 1;
    c->compute_units = (uint32_t)cus;
    *out = c;
    return KVP_OK;
}

extern "C" void kvp_destroy(kvp_ctx *ctx) {
    if (!ctx) return;
    (void)hipSetDevice(ctx->device);
    (void)hipStreamSynchronize(ctx->stream);
    kvp_free_chains(ctx);
    free_dev(ctx->d_trace); free_dev(ctx->d_blocksum); free_dev(ctx->d_tileflag);
    free_dev(ctx->d_cnt_tmp); free_dev(ctx->d_occ_tmp); free_dev(ctx->d_tglobal); free_dev(ctx->d_chunkfull);
    free_dev(ctx->d_aw); free_dev(ctx->d_policy_work); free_dev(ctx->d_policy_x);
    free_dev(ctx->d_tl); free_dev(ctx->d_sparse); free_dev(ctx->d_sel_keys); free_dev(ctx->d_slots_work);
    free_dev(ctx->d_slots_cw); free_dev(ctx->d_slots_list);
    delete ctx;
}

extern "C" const char *kvp_strerror(int code) {
    switch (code) {
        case KVP_OK: return "ok";
        case KVP_EINVAL: return "invalid argument";
        case KVP_ENOTRACE: return "no trace uploaded";
        case KVP_ENOMEM: return "out of memory";
        case KVP_EHIP: return "HIP call failed";
        case KVP_ESHAPE: return "inconsistent or unsupported sizes";
        case KVP_ETRACE: return "trace masks contradict each other";
        case KVP_ENOCHAINS: return "no annealing state";
        case KVP_EINFEASIBLE: return "starting schedule exceeds the HBM capacity";
        default: return "unknown error";
    }
}

extern "C" int kvp_set_generator_batch_bytes(kvp_ctx *ctx, uint64_t bytes) {
    if (!ctx) return KVP_EINVAL;
    ctx->gen_batch_bytes = bytes;
    return KVP_OK;
}

extern "C" int kvp_set_anneal_log_entries(kvp_ctx *ctx, uint64_t entries) {
    if (!ctx) return KVP_EINVAL;
    ctx->log_entries = entries;
    return KVP_OK;
}

extern "C" int kvp_set_capacity_mode(kvp_ctx *ctx, int mode) {
    if (!ctx || (mode != KVP_CAPACITY_PER_STEP && mode != KVP_CAPACITY_PER_SLOT)) return KVP_EINVAL;
    ctx->capacity_mode = mode;
    return KVP_OK;
}

extern "C" int kvp_set_anneal_lookahead(kvp_ctx *ctx, int proposals_per_round) {
    if (!ctx || (proposals_per_round != 0 && proposals_per_round != 1 && proposals_per_round != 4)) return KVP_EINVAL;
    ctx->anneal_lookahead = proposals_per_round;
    return KVP_OK;
}

extern "C" int kvp_set_score_kernel(kvp_ctx *ctx, int which) {
    switch (which) {
        case KVP_SCORE_AUTO: case KVP_SCORE_ROWS: case KVP_SCORE_LANES: case KVP_SCORE_QUAD: case KVP_SCORE_CHUNK:
        case KVP_SCORE_ROWBLOCK: case KVP_SCORE_LINE: case KVP_SCORE_ROWSEG: case KVP_SCORE_ROWLANE: break;
        default: return KVP_EINVAL;
    }
    if (!ctx) return KVP_EINVAL;
    ctx->score_kernel = which;
    return KVP_OK;
}

extern "C" int kvp_score_kernel_used(const kvp_ctx *ctx) { return ctx ? ctx->last_kernel : 0; }

extern "C" uint64_t kvp_plane_unit(const kvp_ctx *ctx) { return ctx && ctx->has_trace ? ctx->unit : 0; }

static uint64_t gcd_u64(uint64_t a, uint64_t b) { while (b) { uint64_t t = a % b; a = b; b = t; } return a; }
static bool good_bw(double b) { return isfinite(b) && b > 0.0; }

extern "C" int kvp_trace_upload(kvp_ctx *ctx, const kvp_problem *pr, const uint32_t *h_access,
                                const uint32_t *h_alive, const uint32_t *h_persist,
                                const uint32_t *h_written) {
    if (!ctx || !pr || !h_access || !h_alive || !h_persist || !h_written) return KVP_EINVAL;
    const uint64_t L = pr->n_layers, N = pr->n_steps, P = pr->n_pages, Wd = pr->n_words, K = pr->n_planes;
    if (K < 1 || K > KVP_MAX_PLANES) return KVP_EINVAL;
    if (!good_bw(pr->bw_hbm) || !good_bw(pr->bw_link) || !good_bw(pr->bw_dram)) return KVP_EINVAL;
    if (L == 0 || N == 0 || P == 0 || Wd != (P + 31) / 32) return KVP_ESHAPE;
    if (L * P >= (1ull << 31) || L * N >= (1ull << 31) || N * Wd >= (1ull << 31)) return KVP_ESHAPE;
    uint64_t unit = 0, sum_pb = 0;
    for (uint64_t k = 0; k < K; k++) {
        if (pr->plane_bytes[k] == 0) return KVP_EINVAL;
        if (pr->plane_bytes[k] >= (1ull << 53)) return KVP_ESHAPE;
        unit = gcd_u64(unit, pr->plane_bytes[k]);
        sum_pb += pr->plane_bytes[k];
    }
    // every byte count of a step must stay an exact integer in fp64
    const long double lim = 9007199254740992.0L;
    if ((long double)P * ((long double)sum_pb + (long double)pr->page_bytes + (long double)pr->token_bytes) >= lim)
        return KVP_ESHAPE;
    if ((long double)P * ((long double)sum_pb / (long double)unit) >= 4294967296.0L) return KVP_ESHAPE;
    const uint32_t tile_unit = 64 / (uint32_t)gcd_u64(L, 64);
    if (L * tile_unit * sizeof(double) > 48 * 1024) return KVP_ESHAPE;   // one summation tile must fit LDS

    // consistency of the masks
    const uint32_t tail = (P % 32) ? ~((1u << (P % 32)) - 1u) : 0u;
    for (uint64_t n = 0; n < N; n++) {
        const uint32_t *v = h_alive + n * Wd, *pm = h_persist + n * Wd, *wm = h_written + n * Wd;
        const uint32_t *vp = n ? h_alive + (n - 1) * Wd : nullptr;
        if (tail && ((v[Wd - 1] | pm[Wd - 1] | wm[Wd - 1]) & tail)) return KVP_ETRACE;
        for (uint64_t w = 0; w < Wd; w++) {
            if (wm[w] & ~v[w]) return KVP_ETRACE;
            if (pm[w] & ~v[w]) return KVP_ETRACE;
            if (n == 0 ? pm[w] != 0 : (pm[w] & ~vp[w]) != 0) return KVP_ETRACE;
        }
    }
    for (uint64_t l = 0; l < L; l++)
        for (uint64_t n = 0; n < N; n++) {
            const uint32_t *v = h_alive + n * Wd;
            for (uint64_t k = 0; k < K; k++) {
                const uint32_t *a = h_access + ((l * N + n) * K + k) * Wd;
                for (uint64_t w = 0; w < Wd; w++)
                    if (a[w] & ~v[w]) return KVP_ETRACE;
            }
        }

    KVP_HIP(hipSetDevice(ctx->device));
    KVP_HIP(hipStreamSynchronize(ctx->stream));
    kvp_free_chains(ctx);
    free_dev(ctx->d_trace); ctx->d_trace = nullptr; ctx->has_trace = false;
    free_dev(ctx->d_chunkfull); ctx->d_chunkfull = nullptr; ctx->cf_words = 0;
    free_dev(ctx->d_aw); ctx->d_aw = nullptr; ctx->aw = nullptr; ctx->kb = 0;
    free_dev(ctx->d_tl); ctx->d_tl = nullptr; ctx->kd = 0;
    free_dev(ctx->d_sparse); ctx->d_sparse = nullptr;

    const size_t nA = (size_t)(L * N * K * Wd), nM = (size_t)(N * Wd);
    auto up4 = [](size_t x) { return (x + 3) & ~(size_t)3; };          // keep every array 16-byte aligned
    const size_t oV = up4(nA), oPm = oV + up4(nM), oWm = oPm + up4(nM), oAcc = oWm + up4(nM);
    const size_t oWr = oAcc + up4((size_t)(L * N)), oSel = oWr + up4((size_t)N);
    const size_t T64 = (size_t)((N + 63) / 64), oCls = oSel + up4((size_t)N), oTile = oCls + up4(4 * T64), total = oTile + up4(2 * T64);
    KVP_HIP(hipMalloc((void **)&ctx->d_trace, total * sizeof(uint32_t)));
    uint32_t *d = ctx->d_trace;
    KVP_HIP(hipMemcpyAsync(d, h_access, nA * 4, hipMemcpyHostToDevice, ctx->stream));
    KVP_HIP(hipMemcpyAsync(d + oV, h_alive, nM * 4, hipMemcpyHostToDevice, ctx->stream));
    KVP_HIP(hipMemcpyAsync(d + oPm, h_persist, nM * 4, hipMemcpyHostToDevice, ctx->stream));
    KVP_HIP(hipMemcpyAsync(d + oWm, h_written, nM * 4, hipMemcpyHostToDevice, ctx->stream));

    ctx->prob = *pr;
    ctx->unit = unit;
    DevProblem &q = ctx->dp;
    q = DevProblem{};
    q.L = (uint32_t)L; q.N = (uint32_t)N; q.P = (uint32_t)P; q.Wd = (uint32_t)Wd; q.K = (uint32_t)K;
    q.cap = pr->cap_pages > 0x7FFFFFFFull ? 0x7FFFFFFFu : (uint32_t)pr->cap_pages;
    q.A = d; q.V = d + oV; q.Pm = d + oPm; q.Wm = d + oWm; q.acc = d + oAcc; q.wr = d + oWr; q.wsel = d + oSel; q.tilecls = d + oCls;
    q.fullmask16 = d + oCls + T64; q.fullmask64 = d + oCls + 2 * T64; q.fullmask256 = d + oCls + 3 * T64;
    q.tile_pfw = d + oTile; q.tile_end = d + oTile + T64;
    for (uint64_t k = 0; k < K; k++) q.wt[k] = (uint32_t)(pr->plane_bytes[k] / unit);
    q.unit_b = (double)unit; q.page_b = (double)pr->page_bytes; q.token_b = (double)pr->token_bytes;
    q.inv_bh = 1.0 / pr->bw_hbm; q.inv_bk = 1.0 / pr->bw_link; q.inv_bd = 1.0 / pr->bw_dram;
    q.inv_min = 1.0 / (pr->bw_link < pr->bw_dram ? pr->bw_link : pr->bw_dram);
    q.dram_bound = q.inv_bd >= q.inv_bk;
    {   // class of every mask word over each tile of 64 steps, and groups of words that are all FULL
        uint32_t *cls = (uint32_t *)calloc(4 * (T64 ? T64 : 1), 4);
        uint32_t *tpe = (uint32_t *)calloc(2 * (T64 ? T64 : 1), 4);   // tile_pfw, tile_end
        uint8_t *fullw = (uint8_t *)malloc((size_t)Wd);
        const uint64_t NCH = (Wd + 15) / 16, CFW = (NCH + 31) / 32;
        uint32_t *cfull = (uint32_t *)calloc((size_t)(T64 * CFW ? T64 * CFW : 1), 4);
        if (!cls || !tpe || !fullw || !cfull) { free(cls); free(tpe); free(fullw); free(cfull); return KVP_ENOMEM; }
        uint32_t *m16 = cls + T64, *m64 = cls + 2 * T64, *m256 = cls + 3 * T64;
        ctx->prefix_full = Wd >= 2 && Wd <= 16;
        ctx->pfw = (uint32_t)Wd;
        ctx->max_tail = 0;
        for (size_t t = 0; t < T64; t++) {
            const uint64_t n0 = t * 64, n1 = n0 + 64 < N ? n0 + 64 : N;
            uint32_t t_pfw = (uint32_t)Wd, t_end = 0;
            for (uint64_t w = 0; w < Wd; w++) {
                bool full = true, empty = true;
                for (uint64_t n = n0 ? n0 - 1 : 0; n < n1; n++) {
                    const uint32_t v = h_alive[n * Wd + w];
                    if (v != 0xFFFFFFFFu) full = false;
                    if (n >= n0 && v != 0) empty = false;
                    if (n >= n0 && n >= 1 && h_persist[n * Wd + w] != 0xFFFFFFFFu) full = false;
                }
                fullw[w] = full;
                if (Wd <= 16)
                    cls[t] |= (uint32_t)(full ? KVP_WORD_FULL : empty ? KVP_WORD_EMPTY : KVP_WORD_MIXED) << (2 * w);
                if (w + 1 < Wd && !full) ctx->prefix_full = false;
                if (!full && w < ctx->pfw) ctx->pfw = (uint32_t)w;
                if (!full && w < t_pfw) t_pfw = (uint32_t)w;
                if (!empty) t_end = (uint32_t)w + 1;
            }
            if (t_end < t_pfw) t_end = t_pfw;                            // (cannot happen: a FULL word is not empty)
            tpe[t] = t_pfw; tpe[T64 + t] = t_end;
            if (t_end - (t_pfw & ~1u) > ctx->max_tail) ctx->max_tail = t_end - (t_pfw & ~1u);
            for (uint64_t c = 0; c < NCH; c++) {
                bool all = true;
                for (uint64_t w = c * 16; w < (c + 1) * 16 && w < Wd; w++) all = all && fullw[w];
                if (all) cfull[t * CFW + c / 32] |= 1u << (c % 32);
            }
            const uint64_t G[3] = {16, 64, 256};
            uint32_t *M[3] = {m16, m64, m256};
            for (int k = 0; k < 3; k++)
                for (uint64_t i = 0; i < 16 && i * G[k] < Wd; i++) {
                    bool all = true;                     // slots past the last word hold zeros: as good as full
                    for (uint64_t w = i * G[k]; w < (i + 1) * G[k] && w < Wd; w++) all = all && fullw[w];
                    if (all) M[k][t] |= 1u << i;
                }
        }
        hipError_t ec = hipMemcpyAsync(d + oCls, cls, 4 * T64 * 4, hipMemcpyHostToDevice, ctx->stream);
        if (ec == hipSuccess) ec = hipMemcpyAsync(d + oTile, tpe, 2 * T64 * 4, hipMemcpyHostToDevice, ctx->stream);
        if (ec == hipSuccess) ec = hipMalloc((void **)&ctx->d_chunkfull, (size_t)T64 * CFW * 4);
        if (ec == hipSuccess)
            ec = hipMemcpyAsync(ctx->d_chunkfull, cfull, (size_t)T64 * CFW * 4, hipMemcpyHostToDevice, ctx->stream);
        if (ec == hipSuccess) ec = hipStreamSynchronize(ctx->stream);
        ctx->cf_words = (uint32_t)CFW;
        free(cls); free(tpe); free(fullw); free(cfull);
        KVP_HIP(ec);
    }
    int rc = kvp_trace_totals_launch(ctx, d + oAcc, d + oWr, d + oSel);
    if (rc) return rc;
    uint32_t *hsel = (uint32_t *)malloc((size_t)N * 4);
    if (!hsel) return KVP_ENOMEM;
    hipError_t e = hipMemcpyAsync(hsel, d + oSel, (size_t)N * 4, hipMemcpyDeviceToHost, ctx->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
    q.single_write = 1;
    for (uint64_t n = 0; n < N && e == hipSuccess; n++)
        if (hsel[n] == 0xFFFFFFFFu) q.single_write = 0;
    free(hsel);
    KVP_HIP(e);
    if ((rc = kvp_bitslice_build(ctx))) return rc;
    ctx->has_trace = true;
    return KVP_OK;
}

static bool aligned16(const void *p) { return ((uintptr_t)p & 15u) == 0; }

extern "C" int kvp_score(kvp_ctx *ctx, const uint32_t *d_placements, uint32_t S, double *d_cost,
                         uint32_t *d_excess, uint32_t *d_counters, uint32_t *d_occ) {
    if (!ctx) return KVP_EINVAL;
    if (!ctx->has_trace) return KVP_ENOTRACE;
    if (S == 0) return KVP_OK;
    if (!d_placements || !d_cost || !d_excess) return KVP_EINVAL;
    if (!aligned16(d_placements) || !aligned16(d_counters) || ((uintptr_t)d_cost & 7u) ||
        ((uintptr_t)d_excess & 3u) || ((uintptr_t)d_occ & 3u))
        return KVP_EINVAL;
    KVP_HIP(hipSetDevice(ctx->device));
    return kvp_score_launch(ctx, d_placements, S, d_cost, d_excess, d_counters, d_occ);
}

int kvp_score_static_launch(kvp_ctx *ctx, const uint32_t *d_placements, uint32_t S, double *d_cost, uint32_t *d_excess);

extern "C" int kvp_score_static(kvp_ctx *ctx, const uint32_t *d_placements, uint32_t S, double *d_cost,
                                uint32_t *d_excess) {
    if (!ctx) return KVP_EINVAL;
    if (!ctx->has_trace) return KVP_ENOTRACE;
    if (S == 0) return KVP_OK;
    if (!d_placements || !d_cost || !d_excess) return KVP_EINVAL;
    if (!aligned16(d_placements) || ((uintptr_t)d_cost & 7u) || ((uintptr_t)d_excess & 3u)) return KVP_EINVAL;
    KVP_HIP(hipSetDevice(ctx->device));
    return kvp_score_static_launch(ctx, d_placements, S, d_cost, d_excess);
}
