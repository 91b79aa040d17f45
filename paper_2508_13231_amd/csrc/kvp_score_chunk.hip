// Scorer for wide rows (n_words >= 16), any layer count, any number of planes.
//
// The narrow-row scheme (a lane per (layer, step) row, four schedules per
// workgroup sharing the trace, two stages in flight in registers) carried over
// to rows of any width by walking a row in CHUNKS of 16 words:
//
//   * one iteration = (layer l, chunk c): the wavefront fetches words
//     [w0, w0+16) of its 65 rows (the 64 steps of the tile and the step before)
//     as 16-byte vectors, four per row, parks them in its LDS slice with a row
//     stride of 17 words (odd: lane-per-row reads hit 64 different banks) and
//     each lane adds its row's 16 words to the row's counters, which live in
//     registers until the row's last chunk;
//   * the trace words of the chunk (planes, alive, persist, written) are the same
//     for the four schedules: fetched once per workgroup, one vector per thread
//     and array, into a double-buffered LDS slot; a chunk whose words are FULL on
//     the tile needs no alive / persist words at all;
//   * the last chunk of a row is shifted left to end at the row's end, so that no
//     load ever leaves the row; the words it shares with the chunk before are
//     zeroed after the load;
//   * step latencies go to a [S][L][N] array in HBM (16 bytes of traffic per row
//     of >= 64 bytes) and a second kernel sums them in execution order with the
//     64-wide tree.
#include <type_traits>

#include "kvp_internal.h"
#include "kvp_lane_common.h"

namespace {

typedef uint32_t c4u __attribute__((ext_vector_type(4), aligned(4)));   // rows are only 4-byte aligned

constexpr int CQ = 4;          // schedules (= wavefronts) per workgroup
constexpr int CW = 16;         // words per chunk
constexpr int RS = 17;         // LDS row stride in words
constexpr int XROWS = TILE_N + 1;
constexpr int XSLICE = XROWS * RS + 3;          // words of a wavefront's slice
constexpr int XVEC = (XROWS * (CW / 4) + 63) / 64;   // vectors per lane: 65 rows x 4 vectors / 64 lanes -> 5
constexpr int TPLANE = TILE_N * RS;             // words of one trace array in a slot

__device__ __forceinline__ void put4(uint32_t *p, c4u v) { p[0] = v.x; p[1] = v.y; p[2] = v.z; p[3] = v.w; }

// KT = number of access planes (compile time: the trace vectors of a chunk sit in registers).
// No load inside the loop is consumed in the iteration that issues it: the schedule rows are
// requested two iterations ahead, the trace words one iteration ahead, and everything is
// unconditional, so the hardware counters tell exactly what has arrived.
template <bool W1, int KT>
__global__ __launch_bounds__(CQ * 64) void score_chunk_kernel(
    DevProblem q, const uint32_t *__restrict__ X, uint32_t S, uint32_t tiles, const uint32_t *__restrict__ chunkfull,
    uint32_t cf_words, double *__restrict__ tglobal, uint32_t *__restrict__ tileflag,
    uint32_t *__restrict__ counters, uint32_t *__restrict__ occ_out) {
    extern __shared__ double smem_d[];
    constexpr int NT = KT + 2 + (W1 ? 0 : 1);                        // planes, alive, persist(, written)
    const uint32_t L = q.L, N = q.N, Wd = q.Wd;
    const uint32_t NCH = (Wd + CW - 1) / CW;
    const uint32_t tid = threadIdx.x;
    const int lane = lane_id();
    const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane((int)(tid / KVP_WAVE));
    uint32_t tile, group;                                             // see xcd_pair for the placement
    if (!xcd_pair(tiles, (S + CQ - 1) / CQ, tile, group)) return;
    const uint32_t s = group * CQ + wave;
    const bool has_s = s < S;
    const uint32_t sc = has_s ? s : S - 1;
    const uint32_t n0 = tile * TILE_N;
    const uint32_t rows = min((uint32_t)TILE_N, N - n0);
    uint32_t *xbuf = (uint32_t *)smem_d + (size_t)wave * XSLICE;
    uint32_t *tbuf = (uint32_t *)smem_d + (size_t)CQ * XSLICE;        // two slots of NT * TPLANE words

    const bool active = (uint32_t)lane < rows;
    const uint32_t lc = active ? (uint32_t)lane : rows - 1;
    const uint32_t n = n0 + lc;
    const uint32_t wr_n = q.wr[n];
    const uint32_t wsel = W1 ? q.wsel[n] : 0u;
    const uint32_t wmw = W1 ? q.Wm[(size_t)n * Wd + wsel] : 0u;
    // X vectors of this lane: vector vi covers row vi/4 of the 65 (row 0 = the step before the tile,
    // step 0 itself for the first tile: then nothing differs and nothing migrates) and part vi%4
    uint32_t xoff[XVEC];
#pragma unroll
    for (int jv = 0; jv < XVEC; jv++) {
        const uint32_t vi = min((uint32_t)lane + 64u * jv, (uint32_t)(XROWS * 4 - 1));
        const uint32_t nn = n0 + (vi >> 2);                            // step + 1
        xoff[jv] = min(nn > 0 ? nn - 1 : 0u, N - 1) * Wd + 4 * (vi & 3u);
    }
    // trace vector of this thread: row tid/4 of the 64, part tid%4
    const uint32_t trow = min(n0 + (tid >> 2), N - 1), tpart = tid & 3u;
    const uint32_t toff = trow * Wd + 4 * tpart, tlds = (tid >> 2) * RS + 4 * tpart;

    struct Stage {
        c4u x[XVEC];
        uint32_t acc;
    };
    Stage st0, st1;
    c4u tr[NT];
    const uint32_t iters = L * NCH;
    // iteration it = (layer it / NCH, chunk it % NCH); kept incrementally for the three streams
    auto advance = [&](uint32_t &l, uint32_t &c) __attribute__((always_inline)) {
        if (++c == NCH) { c = 0; if (l + 1 < L) l++; else c = NCH - 1; }   // past the end: stay on the last chunk
    };
    auto issue_x = [&](Stage &st, uint32_t l, uint32_t c) __attribute__((always_inline)) {
        const uint32_t w0 = min(c * CW, Wd - CW);
        const uint32_t *Xl = X + ((size_t)sc * L + l) * N * Wd + w0;
#pragma unroll
        for (int jv = 0; jv < XVEC; jv++) st.x[jv] = *(const c4u *)(Xl + xoff[jv]);
        st.acc = q.acc[(size_t)l * N + n];
    };
    auto issue_t = [&](uint32_t l, uint32_t c) __attribute__((always_inline)) {
        const uint32_t w0 = min(c * CW, Wd - CW);
        const uint32_t *Ap = q.A + ((size_t)l * N + trow) * KT * Wd + w0 + 4 * tpart;
#pragma unroll
        for (int k = 0; k < KT; k++) tr[k] = *(const c4u *)(Ap + (size_t)k * Wd);
        tr[KT] = *(const c4u *)(q.V + toff + w0);
        tr[KT + 1] = *(const c4u *)(q.Pm + toff + w0);
        if (!W1) tr[NT - 1] = *(const c4u *)(q.Wm + toff + w0);
    };
    auto commit_t = [&](uint32_t it) __attribute__((always_inline)) {
        uint32_t *slot = tbuf + (it & 1u) * NT * TPLANE + tlds;
#pragma unroll
        for (int k = 0; k < NT; k++) put4(slot + k * TPLANE, tr[k]);
    };

    uint32_t hr = 0, hw = 0, mi = 0, mg = 0, oc = 0, fl_acc = 0, occ_acc = 0;
    uint32_t l0 = 0, c0 = 0;                 // iteration being scored
    uint32_t lt = 0, ct = 0;                 // iteration whose trace words are requested next
    uint32_t lx = 0, cx = 0;                 // iteration whose rows are requested next
    auto body = [&](Stage &st, uint32_t it) __attribute__((always_inline)) {
        const uint32_t l = l0, c = c0;
        const uint32_t w0 = min(c * CW, Wd - CW);
        const uint32_t skip = c * CW - w0;                           // leading words already counted (last chunk only)
        const bool full = (chunkfull[(size_t)tile * cf_words + (c >> 5)] >> (c & 31u)) & 1u;
        const uint32_t *slot = tbuf + (it & 1u) * NT * TPLANE;
        // park the rows (zeroing words that the chunk before has counted)
#pragma unroll
        for (int jv = 0; jv < XVEC; jv++) {
            c4u v = st.x[jv];
            const uint32_t vi = (uint32_t)lane + 64u * jv;
            if (skip) {
                const uint32_t b = 4 * (vi & 3u);
                v.x = b + 0 < skip ? 0u : v.x; v.y = b + 1 < skip ? 0u : v.y;
                v.z = b + 2 < skip ? 0u : v.z; v.w = b + 3 < skip ? 0u : v.w;
            }
            if (vi < XROWS * 4) put4(xbuf + (vi >> 2) * RS + 4 * (vi & 3u), v);
        }
        const uint32_t acc_n = st.acc;
        issue_t(lt, ct); advance(lt, ct);                            // trace words of the next iteration
        issue_x(st, lx, cx); advance(lx, cx);                        // rows of two iterations ahead
        __syncthreads();                                             // this iteration's trace slot is complete
        const uint32_t *cur = xbuf + (lc + 1) * RS, *prv = xbuf + lc * RS;
        const uint32_t *ts = slot + lc * RS;
        // two copies of the word loop, chosen once per chunk: with and without the alive / persist masks
        auto words = [&](auto fc) __attribute__((always_inline)) {
            constexpr bool FULLC = decltype(fc)::value;
#pragma unroll
            for (int i = 0; i < CW; i++) {
                const uint32_t raw = cur[i], xp = prv[i];
                uint32_t x, d;
                if (FULLC) {
                    x = raw;
                    d = raw ^ xp;
                } else {
                    const uint32_t vv = ts[KT * TPLANE + i], pmw = ts[(KT + 1) * TPLANE + i];
                    x = raw & vv;
                    fl_acc |= raw & ~vv;
                    d = (x ^ xp) & pmw;
                }
                if (KT == 1) {
                    hr += __popc(x & ts[i]);
                } else {
#pragma unroll
                    for (int k = 0; k < KT; k++) hr += q.wt[k] * __popc(x & ts[k * TPLANE + i]);
                }
                if (!W1) hw += __popc(x & ts[(NT - 1) * TPLANE + i]);
                oc += __popc(x);
                mi += __popc(d & x);
                mg += __popc(d);
            }
        };
        if (full) words(std::true_type{}); else words(std::false_type{});
        if (W1) {
            // the word that holds the written page passes through this chunk or another
            const uint32_t ci = wsel - w0;
            if (ci < CW && ci >= skip) hw = __popc(cur[ci] & wmw);   // written pages exist: no alive mask needed
        }
        if (c == NCH - 1) {
            // the row is complete: Eqs. 2-4
            const uint32_t mo = mg - mi;
            const size_t row = (size_t)l * N + n;
            const double t = step_time(q, hr, hw, mi, mo, acc_n, wr_n);
            if (has_s && active) {
                tglobal[(size_t)s * L * N + row] = t;
                if (counters) *(uint4 *)(counters + ((size_t)s * L * N + row) * 4) = make_uint4(hr, hw, mi, mo);
            }
            occ_acc += oc;
            hr = hw = mi = mg = oc = 0;
        }
        advance(l0, c0);
        commit_t(it + 1);                                            // arrived while this iteration was scored
    };
    issue_t(lt, ct); advance(lt, ct);
    issue_x(st0, lx, cx); advance(lx, cx);
    issue_x(st1, lx, cx); advance(lx, cx);
    commit_t(0);
    for (uint32_t it = 0; it < iters; it += 2) {
        body(st0, it);
        if (it + 1 < iters) body(st1, it + 1);
    }
    if (!has_s) return;
    uint32_t ex = 0;
    if (active) {
        if (occ_out) occ_out[(size_t)s * N + n] = occ_acc;
        ex = occ_acc > q.cap ? occ_acc - q.cap : 0;
    }
    ex = wave_max_u32(ex);
    const uint32_t fl = wave_or_u32(active ? fl_acc : 0u);
    if (lane == 0) tileflag[(size_t)s * tiles + tile] = ex | (fl ? 0x80000000u : 0u);
}

// Eq. 1 from the step latencies in HBM.  A workgroup takes 64 token steps of one
// schedule: the L rows of 64 latencies are read as they lie in memory, turned in
// LDS, and each wavefront folds every fourth of the tile's 64-blocks of the
// execution order g = n*L + l.
__global__ __launch_bounds__(256) void blocksum_from_t_kernel(uint32_t L, uint32_t N, uint32_t tiles, uint32_t nb_total,
                                                              const double *__restrict__ tglobal,
                                                              double *__restrict__ blocksum) {
    extern __shared__ double tb[];                                     // [L][65]
    const uint32_t s = blockIdx.x / tiles, tile = blockIdx.x % tiles;
    const uint32_t n0 = tile * 64, rows = min(64u, N - n0);
    const uint32_t wave = threadIdx.x / KVP_WAVE, lane = (uint32_t)lane_id();
    const double *ts = tglobal + (size_t)s * L * N + n0 + min(lane, rows - 1);
    for (uint32_t l0 = wave; l0 < L; l0 += 32) {                       // eight rows in flight per wavefront
        double v[8];
#pragma unroll
        for (int u = 0; u < 8; u++) v[u] = ts[(size_t)min(l0 + 4 * u, L - 1) * N];
#pragma unroll
        for (int u = 0; u < 8; u++)
            if (l0 + 4 * u < L) tb[(l0 + 4 * u) * 65 + lane] = lane < rows ? v[u] : 0.0;
    }
    __syncthreads();
    const uint32_t nvalid = rows * L, nblk = (nvalid + 63) / 64;
    for (uint32_t b = wave; b < nblk; b += 4) {
        const uint32_t g = b * 64 + lane;
        const uint32_t r = g / L, l = g - r * L;
        double t = g < nvalid ? tb[l * 65 + r] : 0.0;
        t = wave_tree_sum_f64(t);
        if (lane == 0) blocksum[(size_t)s * nb_total + (size_t)tile * L + b] = t;
    }
}

// The same for layer counts whose tile does not fit LDS: one wavefront per 64-block gathers its
// latencies straight from memory.
__global__ __launch_bounds__(256) void blocksum_gather_kernel(uint32_t S, uint32_t L, uint32_t N, uint32_t nb_total,
                                                              const double *__restrict__ tglobal,
                                                              double *__restrict__ blocksum) {
    const uint64_t wv = (uint64_t)blockIdx.x * 4 + threadIdx.x / KVP_WAVE;
    if (wv >= (uint64_t)S * nb_total) return;
    const uint32_t s = (uint32_t)(wv / nb_total), b = (uint32_t)(wv % nb_total);
    const uint64_t g = (uint64_t)b * 64 + lane_id();
    double t = 0.0;
    if (g < (uint64_t)L * N) {
        const uint32_t n = (uint32_t)(g / L), l = (uint32_t)(g % L);
        t = tglobal[((size_t)s * L + l) * N + n];
    }
    t = wave_tree_sum_f64(t);
    if (lane_id() == 0) blocksum[(size_t)s * nb_total + b] = t;
}

}  // namespace

// Block sums of Eq. 1 from the step latencies in ctx->d_tglobal ([S][L][N]).
int kvp_blocksum_from_t_launch(kvp_ctx *ctx, uint32_t S, uint32_t nb_total) {
    const DevProblem &q = ctx->dp;
    const uint32_t tiles = (q.N + 63) / 64;
    const size_t lds = (size_t)q.L * 65 * sizeof(double);
    if (lds > 160 * 1024 || (uint64_t)S * tiles > 0x7FFFFFFFull) {
        const uint64_t nwv = (uint64_t)S * nb_total;
        if ((nwv + 3) / 4 > 0x7FFFFFFFull) return KVP_ESHAPE;
        blocksum_gather_kernel<<<dim3((uint32_t)((nwv + 3) / 4)), dim3(256), 0, ctx->stream>>>(
            S, q.L, q.N, nb_total, ctx->d_tglobal, ctx->d_blocksum);
        KVP_HIP(hipGetLastError());
        return KVP_OK;
    }
    if (lds > 48 * 1024)
        KVP_HIP(hipFuncSetAttribute((const void *)blocksum_from_t_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                    (int)lds));
    blocksum_from_t_kernel<<<dim3(S * tiles), dim3(256), lds, ctx->stream>>>(q.L, q.N, tiles, nb_total, ctx->d_tglobal,
                                                                             ctx->d_blocksum);
    KVP_HIP(hipGetLastError());
    return KVP_OK;
}

// Returns KVP_OK if launched, 1 if this kernel does not cover the shape, <0 on error.
int kvp_score_chunk_launch(kvp_ctx *ctx, const uint32_t *X, uint32_t S, uint32_t tiles, uint32_t nb_total,
                           uint32_t *counters, uint32_t *occ) {
    const DevProblem &q = ctx->dp;
    if (q.Wd < CW || !ctx->d_chunkfull) return 1;
    const bool w1 = q.single_write != 0;
    const size_t nt = q.K + 2 + (w1 ? 0 : 1);
    const size_t lds = ((size_t)CQ * XSLICE + 2 * nt * TPLANE) * 4;
    if (lds > 160 * 1024) return 1;
    const uint64_t nwg = xcd_grid(tiles, (S + CQ - 1) / CQ);
    if (nwg > 0x7FFFFFFFull) return 1;
    int rc = kvp_ensure(ctx, (void **)&ctx->d_tglobal, &ctx->tglobal_cap, (size_t)S * q.L * q.N * sizeof(double));
    if (rc) return rc;
    dim3 grid((uint32_t)nwg), block(CQ * 64);
#define KVP_GO(WW, KK)                                                                                        \
    do {                                                                                                      \
        if (lds > 48 * 1024)                                                                                  \
            KVP_HIP(hipFuncSetAttribute((const void *)score_chunk_kernel<WW, KK>,                             \
                                        hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));              \
        score_chunk_kernel<WW, KK><<<grid, block, lds, ctx->stream>>>(q, X, S, tiles, ctx->d_chunkfull,        \
                                                                      ctx->cf_words, ctx->d_tglobal,          \
                                                                      ctx->d_tileflag, counters, occ);        \
    } while (0)
#define KVP_K(KK) case KK: if (w1) KVP_GO(true, KK); else KVP_GO(false, KK); break;
    switch (q.K) {
        KVP_K(1) KVP_K(2) KVP_K(3) KVP_K(4) KVP_K(5) KVP_K(6) KVP_K(7) KVP_K(8)
        default: return 1;
    }
#undef KVP_K
#undef KVP_GO
    KVP_HIP(hipGetLastError());
    ctx->last_kernel = KVP_SCORE_CHUNK;
    return kvp_blocksum_from_t_launch(ctx, S, nb_total);
}
