// Scorer for wide rows (n_words >= 16): R lanes share a (layer, step) row.
//
// A workgroup owns one schedule and a tile of 64 token steps, for all layers;
// its wavefronts split the layers (as in the narrow-row scorer).  A wavefront
// walks the 64 rows of its layer in passes of 64/R rows:
//
//   count   lane j of a row's group loads words j, j+R, ... (R = 16) or vectors of
//           four words (R = 64) straight from memory: every load instruction
//           reads whole contiguous segments, nothing is staged.  The rows of the
//           next pass are requested before the current ones are counted.  The
//           previous step's row is the row of the group 16 lanes below (one
//           cross-lane move per word; the last group's rows are carried over from
//           the pass before), or simply the previous pass when R = 64.
//           Where the trace says that all pages of the words of an iteration
//           exist and persist on the whole tile, the alive / persist masks are
//           neither loaded nor applied.
//   reduce  the R partial counters of a row are summed across its lanes and
//           parked in LDS, one slot per row of the tile;
//   time    after the 64 rows, lane i takes row i: written pages, Eqs. 2-4, the
//           step latency into the tile's latency buffer.  The buffer is summed in
//           execution order by the 64-wide tree exactly as in the other scorers.
#include "kvp_internal.h"
#include "kvp_lane_common.h"

namespace {

typedef uint32_t w4u __attribute__((ext_vector_type(4)));

// R lanes per row; VEC words per load; NI load iterations per row (R * VEC * NI >= n_words).
template <int R, int VEC, int NI, bool W1>
__global__ __launch_bounds__(256) void score_wide_kernel(
    DevProblem q, const uint32_t *__restrict__ X, const uint32_t *__restrict__ fullmask, uint32_t tiles,
    uint32_t nb_total, double *__restrict__ blocksum, uint32_t *__restrict__ tileflag,
    uint32_t *__restrict__ counters, uint32_t *__restrict__ occ_out) {
    static_assert((R == 16 && VEC == 1) || (R == 64 && (VEC == 1 || VEC == 4)), "supported shapes");
    constexpr int NWV = 4;                     // wavefronts per workgroup
    constexpr int RPP = 64 / R;                // rows per pass
    constexpr int NPASS = TILE_N / RPP;
    constexpr int NW_ = NI * VEC;              // words per lane and row
    extern __shared__ double smem_d[];
    const uint32_t L = q.L, N = q.N, K = q.K, Wd = q.Wd;
    const uint32_t s = blockIdx.x, tile = blockIdx.y;
    const uint32_t n0 = tile * TILE_N;
    const uint32_t rows = min((uint32_t)TILE_N, N - n0);
    const int lane = lane_id();
    const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane((int)(threadIdx.x / KVP_WAVE));
    const uint32_t j = (uint32_t)lane % R, grp = (uint32_t)lane / R;

    uint32_t *rowcnt = (uint32_t *)smem_d + (size_t)wave * TILE_N * 8;     // per wavefront [64][8], 16-byte aligned
    double *tb = (double *)((uint32_t *)smem_d + (size_t)NWV * TILE_N * 8);   // [L][TB_STRIDE]
    uint32_t *occ_l = (uint32_t *)(tb + (size_t)L * TB_STRIDE);     // [64]
    uint32_t *misc = occ_l + TILE_N;                                // [0] stray-bit flag
    if (threadIdx.x < TILE_N) occ_l[threadIdx.x] = 0;
    if (threadIdx.x < 4) misc[threadIdx.x] = 0;
    __syncthreads();

    const uint32_t fmask = fullmask[tile];     // bit i: iteration i needs no masks on this tile
    // word index of this lane in iteration i, and whether it exists
    uint32_t widx[NI];
    bool wok[NI];
#pragma unroll
    for (int i = 0; i < NI; i++) {
        widx[i] = ((uint32_t)i * R + j) * VEC;
        wok[i] = widx[i] < Wd;                 // VEC == 4 needs n_words % 4 == 0: whole vectors exist or not
        if (!wok[i]) widx[i] = 0;              // in bounds; the value is zeroed after the load
    }
    uint32_t occ_acc = 0, fl_acc = 0;          // meaningful in lane i for row i (phase "time")

    auto load_words = [&](const uint32_t *__restrict__ rowp, uint32_t (&dst)[NW_]) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < NI; i++) {
            if (VEC == 4) {
                const w4u v = *(const w4u *)(rowp + widx[i]);
                dst[4 * i] = v.x; dst[4 * i + 1] = v.y; dst[4 * i + 2] = v.z; dst[4 * i + 3] = v.w;
            } else {
                dst[i] = rowp[widx[i]];
            }
        }
    };
    auto zero_missing = [&](uint32_t (&dst)[NW_]) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < NI; i++)
#pragma unroll
            for (int v = 0; v < VEC; v++) dst[VEC * i + v] = wok[i] ? dst[VEC * i + v] : 0u;
    };

    for (uint32_t l = wave; l < L; l += NWV) {
        const uint32_t *Xl = X + ((size_t)s * L + l) * N * Wd;
        const uint32_t *Al = q.A + (size_t)l * N * K * Wd;
        uint32_t cur[NW_], nxt[NW_], old[NW_];
        // the step before the tile: it is the "previous pass" of the first pass
        {
            const uint32_t np = n0 > 0 ? n0 - 1 : 0;          // step 0 has no predecessor: persist is empty there
            load_words(Xl + (size_t)np * Wd, old);
            zero_missing(old);
            const uint32_t nf = min(n0 + grp, N - 1);
            load_words(Xl + (size_t)nf * Wd, nxt);
        }
        for (int p = 0; p < NPASS; p++) {
            const uint32_t r = (uint32_t)p * RPP + grp;        // row of this lane's group within the tile
            const bool rok = r < rows;
            const uint32_t n = n0 + (rok ? r : rows - 1);      // rows past the end shadow the last row
#pragma unroll
            for (int w = 0; w < NW_; w++) cur[w] = nxt[w];
            zero_missing(cur);
            if (p + 1 < NPASS) {
                const uint32_t rn = (uint32_t)(p + 1) * RPP + grp;
                load_words(Xl + (size_t)(n0 + min(rn, rows - 1)) * Wd, nxt);
            }
            const uint32_t *Ar = Al + (size_t)n * K * Wd;
            const uint32_t *Vr = q.V + (size_t)n * Wd, *Pr = q.Pm + (size_t)n * Wd, *Wr = q.Wm + (size_t)n * Wd;
            uint32_t hr = 0, hw = 0, mi = 0, mg = 0, oc = 0, fl = 0;
#pragma unroll
            for (int i = 0; i < NI; i++) {
                const bool full = (fmask >> i) & 1u;           // wavefront-uniform
#pragma unroll
                for (int v = 0; v < VEC; v++) {
                    const int w = VEC * i + v;
                    const uint32_t raw = cur[w];
                    uint32_t xp;
                    if (R == 64) {
                        xp = old[w];
                    } else {
                        // row above: same word, 16 lanes below; the first group takes the last group's
                        // row of the previous pass
                        const uint32_t src = lane >= 64 - R ? old[w] : raw;
                        xp = (uint32_t)__builtin_amdgcn_ds_bpermute(((lane - R) & 63) << 2, (int)src);
                    }
                    uint32_t x, d;
                    if (full) {
                        x = raw;
                        d = raw ^ xp;
                    } else {
                        const uint32_t vv = wok[i] ? Vr[widx[i] + v] : 0u;
                        const uint32_t pmw = wok[i] ? Pr[widx[i] + v] : 0u;
                        x = raw & vv;
                        fl |= raw & ~vv;
                        d = (x ^ xp) & pmw;
                    }
                    // (at step 0 the "row above" is the row itself: nothing migrates)
                    for (uint32_t k = 0; k < K; k++)
                        hr += q.wt[k] * __popc(x & Ar[(size_t)k * Wd + widx[i] + v]);
                    if (!W1) hw += __popc(x & Wr[widx[i] + v]);
                    oc += __popc(x);
                    mi += __popc(d & x);
                    mg += __popc(d);
                }
            }
#pragma unroll
            for (int w = 0; w < NW_; w++) old[w] = cur[w];
            // sum over the R lanes of the row
#pragma unroll
            for (int o = R / 2; o >= 1; o >>= 1) {
                hr += __shfl_xor(hr, o, KVP_WAVE); hw += __shfl_xor(hw, o, KVP_WAVE);
                mi += __shfl_xor(mi, o, KVP_WAVE); mg += __shfl_xor(mg, o, KVP_WAVE);
                oc += __shfl_xor(oc, o, KVP_WAVE); fl |= __shfl_xor(fl, o, KVP_WAVE);
            }
            if (j == 0 && rok) {
                uint32_t *c = rowcnt + r * 8;
                *(uint4 *)c = make_uint4(hr, hw, mi, mg);
                *(uint2 *)(c + 4) = make_uint2(oc, fl);
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        // lane i finishes row i
        if ((uint32_t)lane < rows) {
            const uint32_t n = n0 + lane;
            const uint32_t *c = rowcnt + (uint32_t)lane * 8;
            const uint4 c4 = *(const uint4 *)c;
            const uint2 c2 = *(const uint2 *)(c + 4);
            uint32_t hw = c4.y;
            if (W1) {
                const uint32_t ws = q.wsel[n];
                hw = __popc(Xl[(size_t)n * Wd + ws] & q.Wm[(size_t)n * Wd + ws]);   // written pages exist
            }
            const uint32_t mi = c4.z, mo = c4.w - c4.z;
            const size_t row = (size_t)l * N + n;
            tb[(size_t)l * TB_STRIDE + lane] = step_time(q, c4.x, hw, mi, mo, q.acc[row], q.wr[n]);
            occ_acc += c2.x;
            fl_acc |= c2.y;
            if (counters) *(uint4 *)(counters + ((size_t)s * L * N + row) * 4) = make_uint4(c4.x, hw, mi, mo);
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }
    if ((uint32_t)lane < rows && occ_acc) atomicAdd(&occ_l[lane], occ_acc);
    if (fl_acc) atomicOr(&misc[0], 1u);
    __syncthreads();

    // Eq. 1 inside the tile: element g = r*L + l of the execution order lives at tb[l][r]
    const uint32_t nvalid = rows * L;
    const uint32_t nblk = (nvalid + 63) / 64;
    uint32_t g = wave * 64 + lane;
    uint32_t r = g / L, l = g - r * L;
    const uint32_t dr = (NWV * 64) / L, dl = (NWV * 64) - dr * L;
    for (uint32_t b = wave; b < nblk; b += NWV) {
        double t = g < nvalid ? tb[(size_t)l * TB_STRIDE + r] : 0.0;
        t = wave_tree_sum_f64(t);
        if (lane == 0) blocksum[(size_t)s * nb_total + (size_t)tile * L + b] = t;
        g += NWV * 64; r += dr; l += dl;
        if (l >= L) { l -= L; r++; }
    }
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

template <int R, int VEC, int NI>
int launch_wide(kvp_ctx *ctx, const uint32_t *X, uint32_t S, uint32_t tiles, uint32_t nb_total,
                const uint32_t *fullmask, uint32_t *counters, uint32_t *occ) {
    const DevProblem &q = ctx->dp;
    const size_t lds = (size_t)q.L * TB_STRIDE * 8 + (TILE_N + 4) * 4 + 4 * TILE_N * 8 * 4;
    if (lds > 64 * 1024 || tiles > 65535) return 1;
    dim3 grid(S, tiles), block(256);
    if (q.single_write)
        score_wide_kernel<R, VEC, NI, true><<<grid, block, lds, ctx->stream>>>(
            q, X, fullmask, tiles, nb_total, ctx->d_blocksum, ctx->d_tileflag, counters, occ);
    else
        score_wide_kernel<R, VEC, NI, false><<<grid, block, lds, ctx->stream>>>(
            q, X, fullmask, tiles, nb_total, ctx->d_blocksum, ctx->d_tileflag, counters, occ);
    KVP_HIP(hipGetLastError());
    ctx->last_kernel = KVP_SCORE_WIDE;
    return KVP_OK;
}

template <int R, int VEC>
int launch_wide_ni(kvp_ctx *ctx, uint32_t ni, const uint32_t *X, uint32_t S, uint32_t tiles, uint32_t nb_total,
                   const uint32_t *fullmask, uint32_t *counters, uint32_t *occ) {
    switch (ni) {
#define KVP_CASE(I) case I: return launch_wide<R, VEC, I>(ctx, X, S, tiles, nb_total, fullmask, counters, occ);
        KVP_CASE(1) KVP_CASE(2) KVP_CASE(3) KVP_CASE(4) KVP_CASE(5) KVP_CASE(6) KVP_CASE(7) KVP_CASE(8)
        KVP_CASE(9) KVP_CASE(10) KVP_CASE(11) KVP_CASE(12) KVP_CASE(13) KVP_CASE(14) KVP_CASE(15) KVP_CASE(16)
#undef KVP_CASE
        default: return 1;
    }
}

}  // namespace

// Returns KVP_OK if launched, 1 if this kernel does not cover the shape, <0 on error.
int kvp_score_wide_launch(kvp_ctx *ctx, const uint32_t *X, uint32_t S, uint32_t tiles, uint32_t nb_total,
                          uint32_t *counters, uint32_t *occ) {
    const DevProblem &q = ctx->dp;
    const uint32_t Wd = q.Wd;
    if (Wd <= 256)        // 16 lanes per row, one word per load
        return launch_wide_ni<16, 1>(ctx, (Wd + 15) / 16, X, S, tiles, nb_total, q.fullmask16, counters, occ);
    if (Wd % 4 == 0 && Wd <= 4096)   // a wavefront per row, four words per load
        return launch_wide_ni<64, 4>(ctx, (Wd + 255) / 256, X, S, tiles, nb_total, q.fullmask256, counters, occ);
    if (Wd <= 1024)       // a wavefront per row, one word per load
        return launch_wide_ni<64, 1>(ctx, (Wd + 63) / 64, X, S, tiles, nb_total, q.fullmask64, counters, occ);
    return 1;
}
