// Scorer for narrow rows (n_words <= 16): one LANE per (layer, step) row.
//
// A row of the schedule is only a few words (9 for a 4352-token context in
// 16-token pages), far less than a wavefront, so here each lane owns a whole
// row: lane i of a wavefront scores token step n0 + i of one layer, and the
// wavefront walks over the layers.  Nothing has to be reduced across lanes.
//
//   * The 64 rows of (schedule s, layer l, steps n0-1 .. n0+63) are contiguous in
//     HBM.  The wavefront fetches them with 16-byte loads, lane after lane
//     (perfectly coalesced), parks them in its private slice of LDS and reads
//     them back row-wise (stride n_words: no bank conflict when that is odd).
//     The previous step's row, needed for the migration term, is the
//     neighbouring row of the same staged chunk: no second pass over HBM.
//   * The loads for the next layer are issued before the current one is scored.
//   * alive / persist / written words of a step are the same for every layer:
//     they stay in registers for the whole walk.
//   * Step latencies go to LDS (padded rows), and are summed afterwards in
//     execution order n*L+l by the 64-wide tree, as whole blocks.
#include "kvp_internal.h"
#include "kvp_lane_common.h"

namespace {

// WD = n_words, NW = wavefronts per workgroup, K1: exactly one access plane of
// weight 1, W1: the pages written at a step all sit in one word of the row.
template <int WD, int NW, bool K1, bool W1>
__global__ __launch_bounds__(NW * 64) void score_lane_rows_kernel(
    DevProblem q, const uint32_t *__restrict__ X, size_t x_total, size_t a_total, uint32_t tiles,
    uint32_t nb_total, double *__restrict__ blocksum, uint32_t *__restrict__ tileflag,
    uint32_t *__restrict__ counters, uint32_t *__restrict__ occ_out) {
    extern __shared__ double smem_d[];
    constexpr int XW = ((TILE_N + 1) * WD + 3 + 3) / 4 * 4;     // staged words of X per wavefront
    constexpr int XV = vecs_per_lane((TILE_N + 1) * WD);
    constexpr int AV1 = vecs_per_lane(TILE_N * WD);
    constexpr int WREG = W1 ? 1 : WD;
    // the read weights come as weight planes: the access planes themselves, or (fewer) the binary digits
    // of the pages' read weights
    const uint32_t L = q.L, N = q.N, K = q.pn;
    const uint32_t AW = (TILE_N * K * WD + 3 + 3) / 4 * 4;
    const uint32_t s = blockIdx.x, tile = blockIdx.y;
    const uint32_t n0 = tile * TILE_N;
    const uint32_t rows = min((uint32_t)TILE_N, N - n0);
    const int lane = lane_id();
    // wavefront index as a scalar: everything derived from it stays in scalar registers
    const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane((int)(threadIdx.x / KVP_WAVE));

    // LDS: per-wavefront staging slices (16-byte aligned), then the shared latency buffer
    uint32_t *xbuf = (uint32_t *)smem_d + (size_t)wave * (XW + AW);
    uint32_t *abuf = xbuf + XW;
    double *tb = (double *)((uint32_t *)smem_d + (size_t)NW * (XW + AW));   // [L][TB_STRIDE]
    uint32_t *occ_l = (uint32_t *)(tb + (size_t)L * TB_STRIDE);  // [64]
    uint32_t *misc = occ_l + TILE_N;                             // [0] stray-bit flag
    if (threadIdx.x < TILE_N) occ_l[threadIdx.x] = 0;
    if (threadIdx.x < 4) misc[threadIdx.x] = 0;
    __syncthreads();

    const uint32_t n = n0 + lane;
    const bool active = (uint32_t)lane < rows;
    uint32_t vv[WD], pm[WD], wm[WREG];
#pragma unroll
    for (int w = 0; w < WD; w++) {
        vv[w] = active ? q.V[(size_t)n * WD + w] : 0u;
        pm[w] = active ? q.Pm[(size_t)n * WD + w] : 0u;
    }
    uint32_t wsel = 0;
    if (W1) {
        wsel = active ? q.wsel[n] : 0u;
        wm[0] = active ? q.Wm[(size_t)n * WD + wsel] : 0u;
    } else {
#pragma unroll
        for (int w = 0; w < WREG; w++) wm[w] = active ? q.Wm[(size_t)n * WD + w] : 0u;
    }
    const uint32_t wr_n = active ? q.wr[n] : 0u;
    const uint32_t halo = n0 > 0 ? WD : 0;
    uint32_t occ_acc = 0, fl_acc = 0;

    Staged<XV> sx;
    Staged<AV1> sa;
    uint32_t xshift = 0, xnvec = 0, ashift = 0, anvec = 0;
    auto chunk_x = [&](uint32_t l) { return ((size_t)(s * (size_t)L + l) * N + n0) * WD - halo; };
    auto chunk_a = [&](uint32_t l) { return ((size_t)l * N + n0) * K * WD; };
    if (wave < L) {
        stage_load<XV>(sx, X, chunk_x(wave), rows * WD + halo, x_total, lane, xshift, xnvec);
        if (K1) stage_load<AV1>(sa, q.pl, chunk_a(wave), rows * WD, a_total, lane, ashift, anvec);
    }
    for (uint32_t l = wave; l < L; l += NW) {
        stage_commit<XV>(sx, xbuf, xnvec, lane);
        const uint32_t xs = xshift;
        uint32_t as;
        if (K1) {
            stage_commit<AV1>(sa, abuf, anvec, lane);
            as = ashift;
        } else {
            // several planes: stream the trace chunk straight into LDS
            const size_t start = chunk_a(l), a0 = start & ~(size_t)3;
            as = (uint32_t)(start - a0);
            const uint32_t nv = (as + rows * K * WD + 3) >> 2;
            const uint32_t *p = q.pl + a0;
            const uint32_t left = (uint32_t)min((size_t)0xFFFFFFFFu, a_total - a0);
            for (uint32_t vi = lane; vi < nv; vi += 64) {
                uint4 r = make_uint4(0, 0, 0, 0);
                if (4 * vi + 4 <= left) r = *(const uint4 *)(p + 4 * vi);
                else {
                    if (4 * vi + 0 < left) r.x = p[4 * vi + 0];
                    if (4 * vi + 1 < left) r.y = p[4 * vi + 1];
                    if (4 * vi + 2 < left) r.z = p[4 * vi + 2];
                }
                *(uint4 *)(abuf + 4 * vi) = r;
            }
        }
        if (l + NW < L) {                                       // next layer's rows are in flight meanwhile
            stage_load<XV>(sx, X, chunk_x(l + NW), rows * WD + halo, x_total, lane, xshift, xnvec);
            if (K1) stage_load<AV1>(sa, q.pl, chunk_a(l + NW), rows * WD, a_total, lane, ashift, anvec);
        }
        // the wavefront's LDS writes are complete and visible to all its lanes
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        if (active) {
            const uint32_t *cur = xbuf + xs + halo + (uint32_t)lane * WD;
            const uint32_t *prv = n > 0 ? cur - WD : cur;       // step 0 migrates nothing (persist is empty)
            const uint32_t *ar = abuf + as + (uint32_t)lane * K * WD;
            uint32_t hr = 0, hw = 0, mi = 0, mg = 0, oc = 0;
#pragma unroll
            for (int w = 0; w < WD; w++) {
                const uint32_t raw = cur[w], xp = prv[w];
                const uint32_t x = raw & vv[w];
                fl_acc |= raw & ~vv[w];
                if (K1) {
                    hr += __popc(x & ar[w]);
                } else {
                    for (uint32_t k = 0; k < K; k++) hr += q.pw[k] * __popc(x & ar[k * WD + w]);
                }
                if (!W1) hw += __popc(x & wm[w]);
                oc += __popc(x);
                const uint32_t d = (x ^ xp) & pm[w];
                mi += __popc(d & x);
                mg += __popc(d);
            }
            if (W1) hw = __popc(cur[wsel] & wm[0]);            // written pages exist, so raw & wm == x & wm
            const uint32_t mo = mg - mi;
            const size_t row = (size_t)l * N + n;
            tb[(size_t)l * TB_STRIDE + lane] = step_time(q, hr, hw, mi, mo, q.acc[row], wr_n);
            occ_acc += oc;
            if (counters) *(uint4 *)(counters + ((size_t)s * L * N + row) * 4) = make_uint4(hr, hw, mi, mo);
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }
    if (active && occ_acc) atomicAdd(&occ_l[lane], occ_acc);
    if (fl_acc) atomicOr(&misc[0], 1u);
    __syncthreads();

    // Eq. 1 inside the tile: element g = r*L + l of the execution order lives at tb[l][r]
    const uint32_t nvalid = rows * L;
    const uint32_t nblk = (nvalid + 63) / 64;
    uint32_t g = wave * 64 + lane;
    uint32_t r = g / L, l = g - r * L;
    const uint32_t dr = (NW * 64) / L, dl = (NW * 64) - dr * L;
    for (uint32_t b = wave; b < nblk; b += NW) {
        double t = g < nvalid ? tb[(size_t)l * TB_STRIDE + r] : 0.0;
        t = wave_tree_sum_f64(t);
        if (lane == 0) blocksum[(size_t)s * nb_total + (size_t)tile * L + b] = t;
        g += NW * 64; r += dr; l += dl;
        if (l >= L) { l -= L; r++; }
    }
    // Eq. 5 per token step
    if (threadIdx.x < TILE_N) {
        uint32_t ex = 0;
        if (threadIdx.x < rows) {
            const uint32_t o = occ_l[threadIdx.x];
            if (occ_out) occ_out[(size_t)s * N + n0 + threadIdx.x] = o;
            ex = o > q.cap ? o - q.cap : 0;
        }
        ex = wave_max_u32(ex);
        if (threadIdx.x == 0) tileflag[(size_t)s * tiles + tile] = ex | (misc[0] ? 0x80000000u : 0u);
    }
}

template <int WD, int NW>
int launch_wd_nw(kvp_ctx *ctx, const uint32_t *X, uint32_t S, uint32_t tiles, uint32_t nb_total,
                 uint32_t *counters, uint32_t *occ) {
    const DevProblem &q = ctx->dp;
    const size_t XW = ((TILE_N + 1) * WD + 3 + 3) / 4 * 4, AW = ((size_t)TILE_N * q.pn * WD + 3 + 3) / 4 * 4;
    const size_t lds = (size_t)q.L * TB_STRIDE * 8 + (TILE_N + 4) * 4 + NW * (XW + AW) * 4;
    if (lds > 160 * 1024) return 1;
    const size_t x_total = (size_t)S * q.L * q.N * WD, a_total = (size_t)q.L * q.N * q.pn * WD;
    const bool k1 = q.pn == 1 && q.pw[0] == 1, w1 = q.single_write != 0;
    dim3 grid(S, tiles), block(NW * 64);
#define KVP_GO(KK, WW)                                                                                  \
    do {                                                                                                \
        if (lds > 48 * 1024)                                                                            \
            KVP_HIP(hipFuncSetAttribute((const void *)score_lane_rows_kernel<WD, NW, KK, WW>,           \
                                        hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));         \
        score_lane_rows_kernel<WD, NW, KK, WW><<<grid, block, lds, ctx->stream>>>(                      \
            q, X, x_total, a_total, tiles, nb_total, ctx->d_blocksum, ctx->d_tileflag, counters, occ);  \
    } while (0)
    if (k1 && w1) KVP_GO(true, true);
    else if (k1) KVP_GO(true, false);
    else if (w1) KVP_GO(false, true);
    else KVP_GO(false, false);
#undef KVP_GO
    KVP_HIP(hipGetLastError());
    return KVP_OK;
}

template <int WD>
int launch_wd(kvp_ctx *ctx, const uint32_t *X, uint32_t S, uint32_t tiles, uint32_t nb_total,
              uint32_t *counters, uint32_t *occ) {
    const int rc = launch_wd_nw<WD, 4>(ctx, X, S, tiles, nb_total, counters, occ);
    if (rc == KVP_OK) ctx->last_kernel = KVP_SCORE_LANES;
    return rc;
}

}  // namespace
// Returns KVP_OK if launched, 1 if this kernel does not cover the shape, <0 on error.
// blocksum/tileflag must already hold S*nb_total doubles and S*tiles words.
int kvp_score_tile_launch(kvp_ctx *ctx, const uint32_t *X, uint32_t S, uint32_t tiles, uint32_t nb_total,
                          uint32_t *counters, uint32_t *occ) {
    switch (ctx->dp.Wd) {
#define KVP_CASE(W) case W: return launch_wd<W>(ctx, X, S, tiles, nb_total, counters, occ);
        KVP_CASE(1) KVP_CASE(2) KVP_CASE(3) KVP_CASE(4) KVP_CASE(5) KVP_CASE(6) KVP_CASE(7) KVP_CASE(8)
        KVP_CASE(9) KVP_CASE(10) KVP_CASE(11) KVP_CASE(12) KVP_CASE(13) KVP_CASE(14) KVP_CASE(15) KVP_CASE(16)
#undef KVP_CASE
        default: return 1;
    }
}
