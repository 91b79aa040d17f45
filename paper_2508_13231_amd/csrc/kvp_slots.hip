// Placements whose pages migrate in any inference step between their uses (Sec. III-A: the decision
// S(n, l) places all KV data, not only layer l's).
//
// In kvp_score a page of layer l changes tier in its own step (n, l).  Here a second plane Y names the
// step: a page (l, p) whose placement differs between its steps n-1 and n, and which persists into n,
// moves in the inference step g = n*L + l - Y[l][n][p], Y in 0 .. L-1 (any step after its use at
// (n-1, l) up to its use at (n, l)), and its bytes are charged there.  Reads and the new token's write
// do not depend on Y, so the scorer of kvp_score supplies them (its per-step counters); what this file
// adds is
//   scatter  every migrating page adds itself to |M^i| or |M^o| of its step (which is also where it enters
//            or leaves the pool); pages that are born in HBM enter the pool in their own step, pages that
//            do not persist leave it at the start of the token step (atomics on [S][N*L] arrays);
//   time     Eqs. 2-4 per inference step from the two sets of counters; Eq. 1 through the same
//            64-wide summation tree as everywhere (block sums, then added in order);
//   pool     a prefix sum over the steps gives the pool after every step (Eq. 5) and its largest
//            overshoot.
// The same arrays are the state of the chains that anneal Y (kvp_refine_slots in kvp_moves.hip), which
// draw their proposals from a list of the migrating pages that is also made here.
// gfx950 only.
#include "kvp_internal.h"
#include "kvp_select.h"

namespace {

// thread per schedule word: grid (words of a layer, L, S)
__global__ __launch_bounds__(256) void slot_scatter_kernel(DevProblem q, RowDiv rd, const uint32_t *__restrict__ X, size_t x_stride,
                                                           const uint8_t *__restrict__ Y, uint32_t S,
                                                           uint32_t *__restrict__ mig, int32_t *__restrict__ dpool,
                                                           uint32_t *__restrict__ flag) {
    const uint32_t L = q.L, N = q.N, Wd = q.Wd;
    const uint32_t i = blockIdx.x * 256 + threadIdx.x, l = blockIdx.y, s = blockIdx.z;
    if (i >= N * Wd) return;
    const uint32_t n = rd.quot(i), w = i - n * Wd;
    const uint32_t *Xs = X + (size_t)s * x_stride;
    const size_t G = (size_t)L * N;
    const uint32_t x = Xs[((size_t)l * N + n) * Wd + w] & q.V[(size_t)n * Wd + w];
    uint32_t xp = 0, pm = 0;
    if (n > 0) {
        xp = Xs[((size_t)l * N + n - 1) * Wd + w] & q.V[(size_t)(n - 1) * Wd + w];
        pm = q.Pm[(size_t)n * Wd + w];
    }
    const uint32_t born = x & ~pm, dying = xp & ~pm;
    const uint32_t cin = x & ~xp & pm, cout = ~x & xp & pm;
    const size_t g_own = (size_t)n * L + l;
    if (born) atomicAdd(&dpool[(size_t)s * G + g_own], (int32_t)__popc(born));
    if (dying) atomicAdd(&dpool[(size_t)s * G + (size_t)n * L], -(int32_t)__popc(dying));
    const uint8_t *Ys = Y + (((size_t)s * L + l) * N + n) * q.P + (size_t)w * 32;
    for (uint32_t m = cin | cout; m; m &= m - 1) {
        const uint32_t b = __ffs(m) - 1;
        uint32_t y = Ys[b];
        if (y > L - 1) { y = 0; atomicOr(&flag[s], 0x40000000u); }
        const size_t g = g_own - y;
        const bool in = (cin >> b) & 1u;
        atomicAdd(&mig[((size_t)s * G + g) * 2 + (in ? 0 : 1)], 1u);       // the pool kernel adds these to the pool's changes
    }
}

// thread per inference step (s, g): Eqs. 2-4 from the step's read / write counters and the pages that move there
__global__ __launch_bounds__(256) void slot_time_kernel(DevProblem q, const uint32_t *__restrict__ cnt, size_t cnt_stride,
                                                        const uint32_t *__restrict__ mig, uint32_t S,
                                                        double *__restrict__ tglobal) {
    const uint32_t L = q.L, N = q.N;
    const uint64_t G = (uint64_t)L * N, i = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= G * S) return;
    const uint32_t s = (uint32_t)(i / G);
    const uint64_t g = i - (uint64_t)s * G;
    const uint32_t n = (uint32_t)(g / L), l = (uint32_t)(g - (uint64_t)n * L);
    const uint32_t *c = cnt + (size_t)s * cnt_stride + ((size_t)l * N + n) * 4;
    const uint32_t *m = mig + ((size_t)s * G + g) * 2;
    tglobal[((size_t)s * L + l) * N + n] = step_time(q, c[0], c[1], m[0], m[1], q.acc[(size_t)l * N + n], q.wr[n]);
}

// One workgroup per schedule: the pool after every inference step is the running sum of the changes; the
// changes are replaced by the pool, and the largest overshoot joins the flags into the excess word.
__global__ __launch_bounds__(256) void slot_pool_kernel(DevProblem q, int32_t *__restrict__ dpool, const uint32_t *__restrict__ mig,
                                                        const uint32_t *__restrict__ flag, uint32_t *__restrict__ excess) {
    __shared__ int32_t part[256];
    __shared__ int32_t carry_s;
    const uint32_t s = blockIdx.x, tid = threadIdx.x;
    const size_t G = (size_t)q.L * q.N;
    int32_t *d = dpool + (size_t)s * G;
    if (tid == 0) carry_s = 0;
    __syncthreads();
    int32_t worst = 0;
    for (size_t g0 = 0; g0 < G; g0 += 256) {
        const size_t g = g0 + tid;
        int32_t v = 0;                                                 // pages born or gone, pages moving in, pages moving out
        if (g < G) v = d[g] + (int32_t)mig[((size_t)s * G + g) * 2] - (int32_t)mig[((size_t)s * G + g) * 2 + 1];
        part[tid] = v;
        __syncthreads();
        for (uint32_t o = 1; o < 256; o <<= 1) {                       // inclusive scan of the 256 changes
            const int32_t add = tid >= o ? part[tid - o] : 0;
            __syncthreads();
            part[tid] += add;
            __syncthreads();
        }
        const int32_t pool = carry_s + part[tid];
        if (g < G) { d[g] = pool; worst = max(worst, pool); }
        __syncthreads();
        if (tid == 255) carry_s = pool;
        __syncthreads();
    }
    part[tid] = worst;
    __syncthreads();
    for (uint32_t o = 128; o >= 1; o >>= 1) {
        if (tid < o) part[tid] = max(part[tid], part[tid + o]);
        __syncthreads();
    }
    if (tid == 0) {
        const uint32_t top = (uint32_t)part[0];
        const uint32_t over = top > q.cap ? min(top - q.cap, 0x3FFFFFFFu) : 0u;
        excess[s] = over | (excess[s] & 0x80000000u) | (flag[s] & 0x40000000u);
    }
}

// block sums in order from block 0: one wavefront per schedule
__global__ __launch_bounds__(256) void slot_cost_kernel(uint32_t S, uint32_t nb_total, const double *__restrict__ blocksum,
                                                        double *__restrict__ cost) {
    const uint32_t s = blockIdx.x * 4 + threadIdx.x / KVP_WAVE;
    if (s >= S) return;
    const uint32_t lane = (uint32_t)lane_id();
    const double *b = blocksum + (size_t)s * nb_total;
    double T = 0.0;
    for (uint32_t i0 = 0; i0 < nb_total; i0 += 64) {
        const double cur = i0 + lane < nb_total ? b[i0 + lane] : 0.0;
        const uint32_t cnt = min(64u, nb_total - i0);
        for (uint32_t j = 0; j < cnt; j++) {
            const double bj = __shfl(cur, (int)j, KVP_WAVE);
            T = (i0 == 0 && j == 0) ? bj : T + bj;
        }
    }
    if (lane == 0) cost[s] = T;
}

// ---- the migrating pages of one placement, listed in the order (layer, step, page) ----
// count: migrating pages per schedule word; an exclusive prefix sum over the words (blocks of 1024, the block
// totals by one workgroup, then added back); fill: every word writes its pages at its offset.
__device__ __forceinline__ uint32_t migrating_bits(const DevProblem &q, const uint32_t *X, uint32_t l, uint32_t n, uint32_t w) {
    if (n == 0) return 0;
    const uint32_t x = X[((size_t)l * q.N + n) * q.Wd + w] & q.V[(size_t)n * q.Wd + w];
    const uint32_t xp = X[((size_t)l * q.N + n - 1) * q.Wd + w] & q.V[(size_t)(n - 1) * q.Wd + w];
    return (x ^ xp) & q.Pm[(size_t)n * q.Wd + w];
}

__global__ __launch_bounds__(256) void slot_list_count_kernel(DevProblem q, RowDiv rd, const uint32_t *__restrict__ X,
                                                              uint32_t *__restrict__ cw) {
    const uint32_t i = blockIdx.x * 256 + threadIdx.x, l = blockIdx.y;
    if (i >= q.N * q.Wd) return;
    const uint32_t n = rd.quot(i), w = i - n * q.Wd;
    cw[(size_t)l * q.N * q.Wd + i] = __popc(migrating_bits(q, X, l, n, w));
}

// in place: v[i] becomes the sum of the elements before it inside its block of 1024; the block's total goes to bsum
__global__ __launch_bounds__(256) void scan_blocks_kernel(uint32_t *__restrict__ v, uint64_t count, uint32_t *__restrict__ bsum) {
    __shared__ uint32_t part[256];
    const uint64_t base = (uint64_t)blockIdx.x * 1024 + (uint64_t)threadIdx.x * 4;
    uint32_t a[4], sum = 0;
#pragma unroll
    for (int j = 0; j < 4; j++) { a[j] = base + j < count ? v[base + j] : 0u; sum += a[j]; }
    part[threadIdx.x] = sum;
    __syncthreads();
    for (uint32_t o = 1; o < 256; o <<= 1) {
        const uint32_t add = threadIdx.x >= o ? part[threadIdx.x - o] : 0;
        __syncthreads();
        part[threadIdx.x] += add;
        __syncthreads();
    }
    uint32_t run = part[threadIdx.x] - sum;
#pragma unroll
    for (int j = 0; j < 4; j++) { if (base + j < count) v[base + j] = run; run += a[j]; }
    if (threadIdx.x == 255) bsum[blockIdx.x] = part[255];
}
// one workgroup: bsum[b] becomes the sum of the totals before block b; total[0] the sum of all
__global__ __launch_bounds__(256) void scan_totals_kernel(uint32_t *__restrict__ bsum, uint32_t nblocks, uint32_t *__restrict__ total) {
    __shared__ uint32_t part[256];
    __shared__ uint32_t carry;
    if (threadIdx.x == 0) carry = 0;
    __syncthreads();
    for (uint32_t b0 = 0; b0 < nblocks; b0 += 256) {
        const uint32_t b = b0 + threadIdx.x, mine = b < nblocks ? bsum[b] : 0u;
        part[threadIdx.x] = mine;
        __syncthreads();
        for (uint32_t o = 1; o < 256; o <<= 1) {
            const uint32_t add = threadIdx.x >= o ? part[threadIdx.x - o] : 0;
            __syncthreads();
            part[threadIdx.x] += add;
            __syncthreads();
        }
        if (b < nblocks) bsum[b] = carry + part[threadIdx.x] - mine;
        __syncthreads();
        if (threadIdx.x == 255) carry += part[255];
        __syncthreads();
    }
    if (threadIdx.x == 0) total[0] = carry;
}

__global__ __launch_bounds__(256) void slot_list_fill_kernel(DevProblem q, RowDiv rd, const uint32_t *__restrict__ X,
                                                             const uint32_t *__restrict__ cw, const uint32_t *__restrict__ bsum,
                                                             uint32_t *__restrict__ list) {
    const uint32_t i = blockIdx.x * 256 + threadIdx.x, l = blockIdx.y;
    if (i >= q.N * q.Wd) return;
    const uint32_t n = rd.quot(i), w = i - n * q.Wd;
    const uint64_t word = (uint64_t)l * q.N * q.Wd + i;
    uint32_t at = cw[word] + bsum[word >> 10];
    for (uint32_t m = migrating_bits(q, X, l, n, w); m; m &= m - 1)
        list[at++] = (l * q.N + n) * q.P + w * 32 + (uint32_t)(__ffs(m) - 1);
}

size_t up64(size_t v) { return (v + 63) & ~(size_t)63; }

}  // namespace

// The pages of the placement X (one schedule) that migrate, as entries (l*N + n)*P + p in ascending order: *list_out
// (device memory of the context, valid until the next call) and their number.  Arguments checked by the caller.
int kvp_slot_list_build(kvp_ctx *ctx, const uint32_t *X, uint32_t **list_out, uint32_t *count_out) {
    const DevProblem &q = ctx->dp;
    const uint64_t row_words = (uint64_t)q.N * q.Wd, words = row_words * q.L;
    if (row_words >= (1ull << 31) || q.L > 65535u || (uint64_t)q.L * q.N * q.P >= (1ull << 32)) return KVP_ESHAPE;
    const uint64_t nblocks = (words + 1023) / 1024;
    if (nblocks >= (1ull << 31)) return KVP_ESHAPE;
    int rc = kvp_ensure(ctx, (void **)&ctx->d_slots_cw, &ctx->slots_cw_cap, (size_t)(words + nblocks + 4) * 4);
    if (rc) return rc;
    uint32_t *cw = ctx->d_slots_cw, *bsum = cw + words, *total = bsum + nblocks;
    const RowDiv rd(q.Wd, row_words);
    const dim3 grid((uint32_t)((row_words + 255) / 256), q.L);
    slot_list_count_kernel<<<grid, dim3(256), 0, ctx->stream>>>(q, rd, X, cw);
    KVP_HIP(hipGetLastError());
    scan_blocks_kernel<<<dim3((uint32_t)nblocks), dim3(256), 0, ctx->stream>>>(cw, words, bsum);
    KVP_HIP(hipGetLastError());
    scan_totals_kernel<<<dim3(1), dim3(256), 0, ctx->stream>>>(bsum, (uint32_t)nblocks, total);
    KVP_HIP(hipGetLastError());
    uint32_t M = 0;
    KVP_HIP(hipMemcpyAsync(&M, total, 4, hipMemcpyDeviceToHost, ctx->stream));
    KVP_HIP(hipStreamSynchronize(ctx->stream));
    if ((rc = kvp_ensure(ctx, (void **)&ctx->d_slots_list, &ctx->slots_list_cap, ((size_t)M + 1) * 4))) return rc;
    slot_list_fill_kernel<<<grid, dim3(256), 0, ctx->stream>>>(q, rd, X, cw, bsum, ctx->d_slots_list);
    KVP_HIP(hipGetLastError());
    *list_out = ctx->d_slots_list;
    *count_out = M;
    return KVP_OK;
}

// The state of S schedules (X[s], or the one X for all if broadcast_x; Y[s]): cost and excess as
// kvp_score_slots returns them, and the arrays they were made from, which stay valid in the context's
// buffer until the next call: cnt [L][N][4] per schedule of X (kvp_score's counters), mig [S][N*L][2]
// (pages that move in / out at a step), pool [S][N*L].  Arguments checked by the caller.
int kvp_slots_state_launch(kvp_ctx *ctx, const uint32_t *X, bool broadcast_x, const uint8_t *Y, uint32_t S, double *d_cost,
                           uint32_t *d_excess, uint32_t **cnt_out, uint32_t **mig_out, uint32_t **pool_out) {
    const DevProblem &q = ctx->dp;
    const size_t G = (size_t)q.L * q.N, per = G * q.Wd;
    const uint32_t Sx = broadcast_x ? 1u : S;
    if (q.L > 256) return KVP_ESHAPE;                                  // Y is a byte
    if ((uint64_t)per * S > (1ull << 39) || G * S > (1ull << 39)) return KVP_ESHAPE;
    const size_t o_cnt = 0, o_occ = o_cnt + up64((size_t)Sx * G * 16), o_mig = o_occ + up64((size_t)Sx * q.N * 4);
    const size_t o_pool = o_mig + up64((size_t)S * G * 8), o_flag = o_pool + up64((size_t)S * G * 4);
    const size_t o_c1 = o_flag + up64((size_t)S * 4), o_e1 = o_c1 + up64((size_t)Sx * 8), total = o_e1 + up64((size_t)Sx * 4);
    int rc = kvp_ensure(ctx, (void **)&ctx->d_slots_work, &ctx->slots_work_cap, total);
    if (rc) return rc;
    unsigned char *base = (unsigned char *)ctx->d_slots_work;
    uint32_t *cnt = (uint32_t *)(base + o_cnt), *occ = (uint32_t *)(base + o_occ), *mig = (uint32_t *)(base + o_mig);
    int32_t *dpool = (int32_t *)(base + o_pool);
    uint32_t *flag = (uint32_t *)(base + o_flag), *e1 = (uint32_t *)(base + o_e1);
    double *c1 = (double *)(base + o_c1);
    // reads and writes per step, and the flag for bits on pages that do not exist
    if ((rc = kvp_score_launch(ctx, X, Sx, broadcast_x ? c1 : d_cost, broadcast_x ? e1 : d_excess, cnt, occ))) return rc;
    KVP_HIP(hipMemsetAsync(base + o_mig, 0, o_c1 - o_mig, ctx->stream));
    const uint64_t steps = (uint64_t)G * S, row_words = (uint64_t)q.N * q.Wd;
    if (row_words >= (1ull << 31) || S > 65535u || q.L > 65535u) return KVP_ESHAPE;
    const RowDiv rd(q.Wd, row_words);
    slot_scatter_kernel<<<dim3((uint32_t)((row_words + 255) / 256), q.L, S), dim3(256), 0, ctx->stream>>>(
        q, rd, X, broadcast_x ? 0 : per, Y, S, mig, dpool, flag);
    KVP_HIP(hipGetLastError());
    if ((rc = kvp_ensure(ctx, (void **)&ctx->d_tglobal, &ctx->tglobal_cap, (size_t)S * G * sizeof(double)))) return rc;
    const uint32_t nb_total = (uint32_t)((G + 63) / 64);
    if ((rc = kvp_ensure(ctx, (void **)&ctx->d_blocksum, &ctx->blocksum_cap, (size_t)S * nb_total * sizeof(double)))) return rc;
    slot_time_kernel<<<dim3((uint32_t)((steps + 255) / 256)), dim3(256), 0, ctx->stream>>>(q, cnt, broadcast_x ? 0 : G * 4, mig, S,
                                                                                         ctx->d_tglobal);
    KVP_HIP(hipGetLastError());
    if ((rc = kvp_blocksum_from_t_launch(ctx, S, nb_total))) return rc;
    slot_cost_kernel<<<dim3((S + 3) / 4), dim3(256), 0, ctx->stream>>>(S, nb_total, ctx->d_blocksum, d_cost);
    KVP_HIP(hipGetLastError());
    if (broadcast_x) {                                                 // every schedule carries the one placement's flag
        KVP_HIP(hipMemsetAsync(d_excess, 0, (size_t)S * 4, ctx->stream));
        uint32_t h = 0;
        KVP_HIP(hipMemcpyAsync(&h, e1, 4, hipMemcpyDeviceToHost, ctx->stream));
        KVP_HIP(hipStreamSynchronize(ctx->stream));
        if (h & 0x80000000u) KVP_HIP(hipMemsetD32Async((hipDeviceptr_t)d_excess, 0x80000000u, S, ctx->stream));
    }
    slot_pool_kernel<<<dim3(S), dim3(256), 0, ctx->stream>>>(q, dpool, mig, flag, d_excess);
    KVP_HIP(hipGetLastError());
    if (cnt_out) *cnt_out = cnt;
    if (mig_out) *mig_out = mig;
    if (pool_out) *pool_out = (uint32_t *)dpool;
    return KVP_OK;
}

extern "C" int kvp_score_slots(kvp_ctx *ctx, const uint32_t *d_placements, const uint8_t *d_slots, uint32_t S, double *d_cost,
                               uint32_t *d_excess) {
    if (!ctx) return KVP_EINVAL;
    if (!ctx->has_trace) return KVP_ENOTRACE;
    if (S == 0) return KVP_OK;
    if (!d_placements || !d_slots || !d_cost || !d_excess || ((uintptr_t)d_placements & 15u) || ((uintptr_t)d_cost & 7u) ||
        ((uintptr_t)d_excess & 3u))
        return KVP_EINVAL;
    KVP_HIP(hipSetDevice(ctx->device));
    return kvp_slots_state_launch(ctx, d_placements, false, d_slots, S, d_cost, d_excess, nullptr, nullptr, nullptr);
}
