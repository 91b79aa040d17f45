// Scoring of placement schedules: per-step tier bytes, migration traffic, the
// step-latency model (Eqs. 2-4), the ordered total (Eq. 1) and the capacity
// check (Eq. 5).  gfx950 only.
#include "kvp_internal.h"

// One pass over the trace: read units per step and written pages per token step.
__global__ __launch_bounds__(256) void trace_totals_kernel(DevProblem q, uint32_t *acc, uint32_t *wr, uint32_t *wsel) {
    const int lane = lane_id();
    const uint32_t row = blockIdx.x * 4 + threadIdx.x / KVP_WAVE;
    const uint32_t rows = q.L * q.N;
    if (row < rows) {
        const uint32_t *a = q.A + (size_t)row * q.K * q.Wd;
        uint32_t u = 0;
        for (uint32_t k = 0; k < q.K; k++)
            for (uint32_t w = lane; w < q.Wd; w += KVP_WAVE) u += q.wt[k] * __popc(a[(size_t)k * q.Wd + w]);
        u = wave_sum_u32(u);
        if (lane == 0) acc[row] = u;
    } else if (row < rows + q.N) {
        const uint32_t n = row - rows;
        uint32_t c = 0, nz = 0, last = 0;
        for (uint32_t w = lane; w < q.Wd; w += KVP_WAVE) {
            const uint32_t m = q.Wm[(size_t)n * q.Wd + w];
            c += __popc(m);
            if (m) { nz++; last = w; }
        }
        c = wave_sum_u32(c); nz = wave_sum_u32(nz); last = wave_max_u32(last);
        if (lane == 0) { wr[n] = c; wsel[n] = nz <= 1 ? last : 0xFFFFFFFFu; }
    }
}

int kvp_trace_totals_launch(kvp_ctx *ctx, uint32_t *acc, uint32_t *wr, uint32_t *wsel) {
    const DevProblem &q = ctx->dp;
    uint32_t rows = q.L * q.N + q.N;
    trace_totals_kernel<<<dim3((rows + 3) / 4), dim3(256), 0, ctx->stream>>>(q, acc, wr, wsel);
    KVP_HIP(hipGetLastError());
    return KVP_OK;
}

// ---- general scorer: one wavefront per (layer, step) row, lanes across words --
//
// A workgroup owns one schedule s and a tile of Tn token steps, for all layers.
// Tn*L is a multiple of 64, so the tile's step latencies fill whole blocks of the
// 64-wide summation tree; they are staged in LDS in execution order n*L+l
// together with the tile's occupancy counts.
template <bool WT1>
__global__ __launch_bounds__(256) void score_rows_kernel(DevProblem q, const uint32_t *__restrict__ X,
                                                         uint32_t Tn, uint32_t tiles, uint32_t nb_total,
                                                         double *__restrict__ blocksum,
                                                         uint32_t *__restrict__ tileflag,
                                                         uint32_t *__restrict__ counters,
                                                         uint32_t *__restrict__ occ_out) {
    extern __shared__ double smem[];
    const uint32_t s = blockIdx.x, tile = blockIdx.y;
    const uint32_t n0 = tile * Tn;
    const uint32_t rows = min(Tn, q.N - n0);
    double *tb = smem;
    uint32_t *occ_l = (uint32_t *)(tb + (size_t)Tn * q.L);
    uint32_t *misc = occ_l + Tn;        // [0] flag of stray bits, [1] max excess
    for (uint32_t i = threadIdx.x; i < Tn; i += blockDim.x) occ_l[i] = 0;
    if (threadIdx.x < 2) misc[threadIdx.x] = 0;
    __syncthreads();

    const int lane = lane_id();
    const uint32_t wave = threadIdx.x / KVP_WAVE, nwaves = blockDim.x / KVP_WAVE;
    const uint32_t Wd = q.Wd, K = q.K;
    for (uint32_t l = wave; l < q.L; l += nwaves) {
        const uint32_t *Xl = X + ((size_t)s * q.L + l) * q.N * Wd;
        for (uint32_t r = 0; r < rows; r++) {
            const uint32_t n = n0 + r;
            const uint32_t *xr = Xl + (size_t)n * Wd;
            const uint32_t *a = q.A + ((size_t)l * q.N + n) * K * Wd;
            const uint32_t *v = q.V + (size_t)n * Wd, *pm = q.Pm + (size_t)n * Wd, *wm = q.Wm + (size_t)n * Wd;
            uint32_t hr = 0, hw = 0, mi = 0, mo = 0, oc = 0, fl = 0;
            for (uint32_t w = lane; w < Wd; w += KVP_WAVE) {
                const uint32_t raw = xr[w], vv = v[w];
                const uint32_t x = raw & vv;
                fl |= raw & ~vv;
                if (WT1) {
                    for (uint32_t k = 0; k < K; k++) hr += __popc(x & a[(size_t)k * Wd + w]);
                } else {
                    for (uint32_t k = 0; k < K; k++) hr += q.wt[k] * __popc(x & a[(size_t)k * Wd + w]);
                }
                hw += __popc(x & wm[w]);
                oc += __popc(x);
                if (n > 0) {
                    const uint32_t xp = xr[(ptrdiff_t)w - (ptrdiff_t)Wd];
                    const uint32_t d = (x ^ xp) & pm[w];
                    mi += __popc(d & x);
                    mo += __popc(d & xp);
                }
            }
            hr = wave_sum_u32(hr); hw = wave_sum_u32(hw); mi = wave_sum_u32(mi); mo = wave_sum_u32(mo);
            oc = wave_sum_u32(oc); fl = wave_or_u32(fl);
            if (lane == 0) {
                const size_t row = (size_t)l * q.N + n;
                tb[(size_t)r * q.L + l] = step_time(q, hr, hw, mi, mo, q.acc[row], q.wr[n]);
                atomicAdd(&occ_l[r], oc);
                if (fl) atomicOr(&misc[0], 1u);
                if (counters) {
                    uint4 c = make_uint4(hr, hw, mi, mo);
                    *(uint4 *)(counters + ((size_t)s * q.L * q.N + row) * 4) = c;
                }
            }
        }
    }
    __syncthreads();

    // Eq. 1 inside the tile: whole 64-blocks of the execution order.
    const uint32_t nvalid = rows * q.L;
    const uint32_t nblk = (nvalid + 63) / 64;
    const size_t blk0 = ((size_t)n0 * q.L) / 64;
    for (uint32_t b = wave; b < nblk; b += nwaves) {
        const uint32_t i = b * 64 + lane;
        double t = i < nvalid ? tb[i] : 0.0;
        t = wave_tree_sum_f64(t);
        if (lane == 0) blocksum[(size_t)s * nb_total + blk0 + b] = t;
    }
    // Eq. 5 per token step.
    uint32_t ex = 0;
    for (uint32_t r = threadIdx.x; r < rows; r += blockDim.x) {
        const uint32_t o = occ_l[r];
        if (occ_out) occ_out[(size_t)s * q.N + n0 + r] = o;
        const uint32_t e = o > q.cap ? o - q.cap : 0;
        ex = e > ex ? e : ex;
    }
    ex = wave_max_u32(ex);
    if (lane == 0 && ex) atomicMax(&misc[1], ex);
    __syncthreads();
    if (threadIdx.x == 0) tileflag[(size_t)s * tiles + tile] = misc[1] | (misc[0] ? 0x80000000u : 0u);
}

// Block sums are added in order from block 0 (the sequential part of the
// summation order), tile verdicts are merged.  One wavefront per schedule: 64
// block sums are fetched at a time, one per lane, and added one after the other
// through lane broadcasts; every lane carries the same running total.
__global__ __launch_bounds__(256) void score_finalize_kernel(uint32_t S, uint32_t nb_total, uint32_t tiles,
                                                             const double *__restrict__ blocksum,
                                                             const uint32_t *__restrict__ tileflag,
                                                             double *__restrict__ cost,
                                                             uint32_t *__restrict__ excess) {
    const uint32_t s = blockIdx.x * 4 + threadIdx.x / KVP_WAVE;
    if (s >= S) return;
    const uint32_t lane = (uint32_t)lane_id();
    const double *b = blocksum + (size_t)s * nb_total;
    double T = 0.0;
    double v = lane < nb_total ? b[lane] : 0.0;
    for (uint32_t i0 = 0; i0 < nb_total; i0 += 64) {
        const double cur = v;
        const uint32_t nx = i0 + 64 + lane;
        v = nx < nb_total ? b[nx] : 0.0;                               // next 64 while these are added
        const uint32_t cnt = min(64u, nb_total - i0);
        if (cnt == 64) {
            // lane j's value through the scalar unit: a few cycles, where a cross-lane shuffle would
            // put an LDS round trip into every link of this chain of additions
            const int lo = __double2loint(cur), hi = __double2hiint(cur);
#pragma unroll
            for (int j = 0; j < 64; j++) {
                const double bj = __hiloint2double(__builtin_amdgcn_readlane(hi, j), __builtin_amdgcn_readlane(lo, j));
                T = (i0 == 0 && j == 0) ? bj : T + bj;
            }
        } else {
            for (uint32_t j = 0; j < cnt; j++) {
                const double bj = __shfl(cur, (int)j, KVP_WAVE);
                T = (i0 == 0 && j == 0) ? bj : T + bj;
            }
        }
    }
    uint32_t ex = 0, fl = 0;
    for (uint32_t t = lane; t < tiles; t += 64) {
        const uint32_t f = tileflag[(size_t)s * tiles + t];
        fl |= f & 0x80000000u;
        const uint32_t e = f & 0x7FFFFFFFu;
        ex = e > ex ? e : ex;
    }
    ex = wave_max_u32(ex);
    fl = wave_or_u32(fl);
    if (lane == 0) {
        cost[s] = T;
        excess[s] = ex | fl;
    }
}

static uint32_t gcd_u32(uint32_t a, uint32_t b) { while (b) { uint32_t t = a % b; a = b; b = t; } return a; }

int kvp_score_tile_launch(kvp_ctx *ctx, const uint32_t *X, uint32_t S, uint32_t tiles, uint32_t nb_total,
                          uint32_t *counters, uint32_t *occ);
int kvp_score_chunk_launch(kvp_ctx *ctx, const uint32_t *X, uint32_t S, uint32_t tiles, uint32_t nb_total,
                           uint32_t *counters, uint32_t *occ);
int kvp_score_quad_launch(kvp_ctx *ctx, const uint32_t *X, uint32_t S, uint32_t tiles, uint32_t nb_total,
                          uint32_t *counters, uint32_t *occ);
int kvp_score_rowblock_launch(kvp_ctx *ctx, const uint32_t *X, uint32_t S, uint32_t tiles, uint32_t nb_total,
                              uint32_t *counters, uint32_t *occ);
int kvp_score_rowlane_launch(kvp_ctx *ctx, const uint32_t *X, uint32_t S, uint32_t tiles, uint32_t nb_total,
                             uint32_t *counters, uint32_t *occ);
int kvp_score_rowseg_launch(kvp_ctx *ctx, const uint32_t *X, uint32_t S, uint32_t tiles, uint32_t nb_total,
                            uint32_t *counters, uint32_t *occ);
int kvp_score_line_launch(kvp_ctx *ctx, const uint32_t *X, uint32_t S, uint32_t tiles, uint32_t nb_total,
                          uint32_t *counters, uint32_t *occ);

int kvp_score_launch(kvp_ctx *ctx, const uint32_t *d_placements, uint32_t S, double *d_cost,
                     uint32_t *d_excess, uint32_t *d_counters, uint32_t *d_occ) {
    const DevProblem &q = ctx->dp;
    if (S == 0) return KVP_OK;
    int rc;
    const uint32_t nb_total = (uint32_t)(((uint64_t)q.L * q.N + 63) / 64);
    const int forced = ctx->score_kernel;                  // KVP_SCORE_AUTO or the scorer to try first
    if (forced != KVP_SCORE_ROWS) {
        // scorers with one lane per token step: tiles of 64 steps
        const uint32_t tiles64 = (q.N + 63) / 64;
        if ((rc = kvp_ensure(ctx, (void **)&ctx->d_blocksum, &ctx->blocksum_cap, (size_t)S * nb_total * sizeof(double)))) return rc;
        if ((rc = kvp_ensure(ctx, (void **)&ctx->d_tileflag, &ctx->tileflag_cap, (size_t)S * tiles64 * sizeof(uint32_t)))) return rc;
        typedef int (*launch_fn)(kvp_ctx *, const uint32_t *, uint32_t, uint32_t, uint32_t, uint32_t *, uint32_t *);
        // the order AUTO tries them in: narrow rows first, then by how close each comes to the HBM rate
        struct { int id; launch_fn fn; bool narrow; } const order[] = {
            {KVP_SCORE_QUAD, kvp_score_quad_launch, true},     {KVP_SCORE_LANES, kvp_score_tile_launch, true},
            {KVP_SCORE_ROWLANE, kvp_score_rowlane_launch, false},
            {KVP_SCORE_ROWBLOCK, kvp_score_rowblock_launch, false}, {KVP_SCORE_ROWSEG, kvp_score_rowseg_launch, false},
            {KVP_SCORE_LINE, kvp_score_line_launch, false},
            {KVP_SCORE_CHUNK, kvp_score_chunk_launch, false},
        };
        const int family = forced;
        rc = 1;
        for (const auto &o : order)                            // the forced scorer, wherever it is in the order
            if (rc == 1 && o.id == family) rc = o.fn(ctx, d_placements, S, tiles64, nb_total, d_counters, d_occ);
        for (const auto &o : order)                            // then (or under AUTO) the first that covers the shape
            if (rc == 1 && o.id != family && o.narrow == (q.Wd <= 16))
                rc = o.fn(ctx, d_placements, S, tiles64, nb_total, d_counters, d_occ);
        if (rc < 0) return rc;
        if (rc == KVP_OK) {
            score_finalize_kernel<<<dim3((S + 3) / 4), dim3(256), 0, ctx->stream>>>(
                S, nb_total, tiles64, ctx->d_blocksum, ctx->d_tileflag, d_cost, d_excess);
            KVP_HIP(hipGetLastError());
            return KVP_OK;
        }
    }
    // tile: a multiple of `unit` token steps so that Tn*L is a multiple of 64
    const uint32_t unit = 64 / gcd_u32(q.L, 64);
    uint32_t tn_max = (4096 / (q.L * unit)) * unit;        // <= 32 KB of step latencies in LDS
    if (tn_max < unit) tn_max = unit;
    uint32_t want_tiles = (2048 + S - 1) / S;              // enough workgroups to fill the chip
    uint32_t Tn = (q.N / want_tiles) / unit * unit;
    if (Tn < unit) Tn = unit;
    if (Tn > tn_max) Tn = tn_max;
    const uint32_t tiles = (q.N + Tn - 1) / Tn;
    if (tiles > 65535) return KVP_ESHAPE;
    if ((rc = kvp_ensure(ctx, (void **)&ctx->d_blocksum, &ctx->blocksum_cap, (size_t)S * nb_total * sizeof(double)))) return rc;
    if ((rc = kvp_ensure(ctx, (void **)&ctx->d_tileflag, &ctx->tileflag_cap, (size_t)S * tiles * sizeof(uint32_t)))) return rc;
    const size_t lds = (size_t)Tn * q.L * sizeof(double) + (size_t)Tn * sizeof(uint32_t) + 16;
    if (lds > 64 * 1024) return KVP_ESHAPE;
    bool wt1 = true;
    for (uint32_t k = 0; k < q.K; k++) wt1 = wt1 && q.wt[k] == 1;
    dim3 grid(S, tiles), block(256);
    if (wt1)
        score_rows_kernel<true><<<grid, block, lds, ctx->stream>>>(q, d_placements, Tn, tiles, nb_total,
                                                                  ctx->d_blocksum, ctx->d_tileflag, d_counters, d_occ);
    else
        score_rows_kernel<false><<<grid, block, lds, ctx->stream>>>(q, d_placements, Tn, tiles, nb_total,
                                                                   ctx->d_blocksum, ctx->d_tileflag, d_counters, d_occ);
    KVP_HIP(hipGetLastError());
    ctx->last_kernel = KVP_SCORE_ROWS;
    score_finalize_kernel<<<dim3((S + 3) / 4), dim3(256), 0, ctx->stream>>>(S, nb_total, tiles, ctx->d_blocksum,
                                                                               ctx->d_tileflag, d_cost, d_excess);
    KVP_HIP(hipGetLastError());
    return KVP_OK;
}

// ---- scoring for callers that cannot allocate ------------------------------------------------
// The block sums, the tile verdicts and (for the layer counts whose summation tree is not kept on
// chip) the step latencies of a launch live in device memory beyond the caller's inputs and
// outputs.  kvp_score keeps them in buffers that it allocates and grows; kvp_score_static keeps
// them in this array instead, which every GPU the library runs on holds from load to exit.
static __device__ __align__(256) unsigned char scratch[KVP_STATIC_SCRATCH_BYTES];

// The array's name is a host-side handle, not a device address: each device has its own copy at
// its own address, resolved once per device (with that device current) and kept here.
#define KVP_MAX_DEVICES 64
static unsigned char *scratch_ptr[KVP_MAX_DEVICES];

int kvp_static_scratch_init(int device) {
    if (device < 0 || device >= KVP_MAX_DEVICES) return KVP_EINVAL;
    if (scratch_ptr[device]) return KVP_OK;
    void *p = nullptr;
    KVP_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p || ((uintptr_t)p & 255u)) return KVP_EHIP;
    scratch_ptr[device] = (unsigned char *)p;
    return KVP_OK;
}

int kvp_score_static_launch(kvp_ctx *ctx, const uint32_t *d_placements, uint32_t S, double *d_cost, uint32_t *d_excess) {
    const DevProblem &q = ctx->dp;
    unsigned char *base = scratch_ptr[ctx->device];
    if (!base) return KVP_EHIP;                                // kvp_create resolves it; never null after that
    const uint64_t nb_total = ((uint64_t)q.L * q.N + 63) / 64;
    auto up = [](uint64_t x) { return (x + 255) & ~(uint64_t)255; };
    // the general scorer may cut the steps into more tiles than the others' 64-step tiles; N bounds both
    const uint64_t need_bs = up((uint64_t)S * nb_total * sizeof(double)), need_tf = up((uint64_t)S * q.N * sizeof(uint32_t));
    if (need_bs + need_tf > KVP_STATIC_SCRATCH_BYTES) return KVP_ESHAPE;
    // swap the context's own buffers for parts of the static array for the length of this call
    struct Saved { double *bs; size_t bsc; uint32_t *tf; size_t tfc; double *tg; size_t tgc; } const old = {
        ctx->d_blocksum, ctx->blocksum_cap, ctx->d_tileflag, ctx->tileflag_cap, ctx->d_tglobal, ctx->tglobal_cap};
    ctx->d_blocksum = (double *)base;                      ctx->blocksum_cap = (size_t)need_bs;
    ctx->d_tileflag = (uint32_t *)(base + need_bs);        ctx->tileflag_cap = (size_t)need_tf;
    ctx->d_tglobal = (double *)(base + need_bs + need_tf); ctx->tglobal_cap = (size_t)(KVP_STATIC_SCRATCH_BYTES - need_bs - need_tf);
    ctx->no_alloc = true;                                  // a scorer that needs more gets KVP_ESHAPE from kvp_ensure
    const int rc = kvp_score_launch(ctx, d_placements, S, d_cost, d_excess, nullptr, nullptr);
    ctx->no_alloc = false;
    ctx->d_blocksum = old.bs; ctx->blocksum_cap = old.bsc; ctx->d_tileflag = old.tf; ctx->tileflag_cap = old.tfc;
    ctx->d_tglobal = old.tg; ctx->tglobal_cap = old.tgc;
    return rc;
}
