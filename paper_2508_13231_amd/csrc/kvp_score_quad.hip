// Fastest scorer for narrow rows: n_words <= 15, one access plane, and a layer
// count L that is a power of two (<= 64).
//
// As in the other narrow-row scorer one LANE owns a (layer, step) row and a
// wavefront walks over the layers of 64 consecutive token steps.  Three things
// are different:
//
//  * A workgroup is four wavefronts that score the same 64 steps of FOUR
//    different schedules.  The access-trace chunk of a layer is the same for all
//    of them, so it is fetched once (each thread one 16-byte vector) into a
//    double-buffered LDS slot instead of once per schedule.  One barrier per
//    layer keeps the four in step.
//  * The schedule rows of TWO layers ahead are in flight in registers while the
//    current layer is scored from LDS: enough bytes outstanding to cover HBM
//    latency at a few wavefronts per SIMD.
//  * No latency buffer.  With L = 2^k a block of the 64-wide summation tree is
//    64/L consecutive steps x L layers; its folds first join the steps (lanes:
//    a few cross-lane adds), then the layers (l, l + L/2), (l, l + L/4), ...
//    Visiting the layers in bit-reversed order turns those layer folds into a
//    binary counter of partial sums held in k registers per lane, exactly the
//    tree of the definition, with no LDS traffic at all.
#include <type_traits>

#include "kvp_internal.h"
#include "kvp_lane_common.h"

namespace {

typedef uint32_t v4u __attribute__((ext_vector_type(4)));   // native vector: stays in registers

// acc += popcount(v) as the one instruction the hardware has for it (left to itself the compiler
// counts into fresh registers and adds them up three at a time)
__device__ __forceinline__ void count(uint32_t &acc, uint32_t v) {
    asm("v_bcnt_u32_b32 %0, %1, %0" : "+v"(acc) : "v"(v));
}

constexpr int QUAD = 4;              // schedules (= wavefronts) per workgroup
constexpr int A_SLOT = QUAD * 64 * 4;   // words of one trace slot: one 16-byte vector per thread

// Every load below is unconditional and its index clamped instead of predicated:
// straight-line code lets the hardware counters tell exactly which stage has
// arrived, so two stages really stay in flight.  The host guarantees that whole
// 16-byte vectors can be read up to three words past any chunk (kvp_score_quad_launch).
// WD = n_words; W1: the pages written at a step sit in one word; PF: on every tile
// all words but the last are FULL (kvp_internal.h), so only the last word needs
// the alive / persist masks; NS: register stages (layers in flight), L % NS == 0.
template <int WD, bool W1, bool PF, int NS>
__global__ __launch_bounds__(QUAD * 64) void score_quad_kernel(
    DevProblem q, const uint32_t *__restrict__ X, uint32_t S, uint32_t tiles, uint32_t nb_total, uint32_t log2L,
    double *__restrict__ blocksum, uint32_t *__restrict__ tileflag, uint32_t *__restrict__ counters,
    uint32_t *__restrict__ occ_out) {
    extern __shared__ double smem_d[];
    static_assert(NS == 2 || NS == 4, "two or four register stages");
    constexpr int XV = vecs_per_lane((TILE_N + 1) * WD);
    constexpr int XW = XV * 64 * 4;                               // a full vector slot per lane and round
    constexpr int W0 = PF ? WD - 1 : 0;                           // first word that needs the masks
    constexpr int MREG = WD - W0, WREG = W1 ? 1 : WD;
    const uint32_t L = 1u << log2L, N = q.N;
    const uint32_t tid = threadIdx.x;
    const int lane = lane_id();
    const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane((int)(tid / KVP_WAVE));
    // consecutive workgroups take the consecutive tiles of the same four schedules, so the rows of
    // one (schedule, layer), contiguous in memory, are fetched at about the same time
    const uint32_t tile = blockIdx.x % tiles;
    const uint32_t s = (blockIdx.x / tiles) * QUAD + wave;
    const bool has_s = s < S;
    const uint32_t sc = has_s ? s : S - 1;                        // spare wavefronts shadow the last schedule
    const uint32_t n0 = tile * TILE_N;
    const uint32_t rows = min((uint32_t)TILE_N, N - n0);
    uint32_t *xbuf = (uint32_t *)smem_d + (size_t)wave * XW;
    uint32_t *abuf = (uint32_t *)smem_d + (size_t)QUAD * XW;          // two slots of A_SLOT words

    const bool active = (uint32_t)lane < rows;
    const uint32_t lc = active ? (uint32_t)lane : rows - 1;           // idle lanes shadow the last row
    const uint32_t n = n0 + lc;
    uint32_t vv[MREG], pm[MREG], wm[WREG];
#pragma unroll
    for (int w = 0; w < MREG; w++) {
        vv[w] = q.V[(size_t)n * WD + W0 + w];
        pm[w] = q.Pm[(size_t)n * WD + W0 + w];
    }
    uint32_t wsel = 0;
    if (W1) {
        wsel = q.wsel[n];
        wm[0] = q.Wm[(size_t)n * WD + wsel];
    } else {
#pragma unroll
        for (int w = 0; w < WREG; w++) wm[w] = q.Wm[(size_t)n * WD + w];
    }
    const uint32_t wr_n = q.wr[n];
    const uint32_t halo = n0 > 0 ? WD : 0;
    const uint32_t xcnt = rows * WD + halo, acnt = rows * WD;
    const size_t lstride = (size_t)N * WD;
    const size_t xbase = ((size_t)sc * L * N + n0) * WD - halo;   // words; layer l adds l * lstride
    const size_t abase = (size_t)n0 * WD;

    // one register stage: the rows of one layer on their way from HBM to LDS
    struct Stage {
        v4u x[XV];
        v4u a;
        uint32_t acc, xshift, ashift;
    };
    Stage st0, st1, st2, st3;
    auto layer_of = [&](uint32_t it) { return log2L ? (__brev(it) >> (32 - log2L)) : 0u; };
    auto issue = [&](Stage &st, uint32_t it) __attribute__((always_inline)) {
        const uint32_t l = layer_of(it);
        const size_t xs = xbase + l * lstride, xa0 = xs & ~(size_t)3;
        st.xshift = (uint32_t)(xs - xa0);
        const uint32_t xlast = ((st.xshift + xcnt + 3) >> 2) - 1;
        const uint32_t *px = X + xa0;
#pragma unroll
        for (int j = 0; j < XV; j++) st.x[j] = *(const v4u *)(px + 4 * min((uint32_t)lane + 64u * j, xlast));
        const size_t as = abase + l * lstride, aa0 = as & ~(size_t)3;
        st.ashift = (uint32_t)(as - aa0);
        const uint32_t alast = ((st.ashift + acnt + 3) >> 2) - 1;
        st.a = *(const v4u *)(q.A + aa0 + 4 * min(tid, alast));
        st.acc = q.acc[(size_t)l * N + n];
    };

    double stk[6] = {0.0, 0.0, 0.0, 0.0, 0.0, 0.0}, total = 0.0;
    uint32_t occ_acc = 0, fl_acc = 0;
    auto body = [&](Stage &st, uint32_t it) __attribute__((always_inline)) {
        const uint32_t l = layer_of(it);
        uint32_t *aslot = abuf + (it & 1u) * A_SLOT;
#pragma unroll
        for (int j = 0; j < XV; j++) *(v4u *)(xbuf + 4 * ((uint32_t)lane + 64u * j)) = st.x[j];
        *(v4u *)(aslot + 4 * tid) = st.a;
        const uint32_t xs = st.xshift, as = st.ashift, acc_n = st.acc;
        issue(st, min(it + NS, L - 1));                         // rows of NS layers ahead are now in flight
                                                                // (past the end: a redundant, harmless reload)
        __syncthreads();                                        // this layer's trace slot is complete
        const uint32_t *cur = xbuf + xs + halo + lc * WD;
        const uint32_t *prv = n > 0 ? cur - WD : cur;           // step 0 migrates nothing (persist is empty)
        const uint32_t *ar = aslot + as + lc * WD;
        uint32_t hr = 0, hw = 0, mi = 0, mg = 0, oc = 0;
#pragma unroll
        for (int w = 0; w < WD; w++) {
            const uint32_t raw = cur[w], xp = prv[w];
            if (w < W0) {
                // all 32 pages exist and persist on every step of the tile: no masking needed
                // (at step 0 prv is cur, so nothing migrates there either)
                count(hr, raw & ar[w]);
                if (!W1) count(hw, raw & wm[w]);
                count(oc, raw);
                const uint32_t d = raw ^ xp;
                count(mi, d & raw);
                count(mg, d);
            } else {
                const uint32_t x = raw & vv[w - W0];
                fl_acc |= raw & ~vv[w - W0];
                count(hr, x & ar[w]);
                if (!W1) count(hw, x & wm[w]);
                count(oc, x);
                const uint32_t d = (x ^ xp) & pm[w - W0];
                count(mi, d & x);
                count(mg, d);
            }
        }
        if (W1) hw = __popc(cur[wsel] & wm[0]);                // written pages exist, so raw & wm == x & wm
        const uint32_t mo = mg - mi;
        double t = step_time(q, hr, hw, mi, mo, acc_n, wr_n);
        t = active ? t : 0.0;                                   // rows past the end of the trace pad with +0.0
        occ_acc += oc;
        if (counters && has_s && active)
            *(uint4 *)(counters + (((size_t)s * L + l) * N + n) * 4) = make_uint4(hr, hw, mi, mo);
        // folds of the summation tree that join the steps of one block (lanes)
        for (uint32_t m = (64u >> log2L) >> 1; m >= 1; m >>= 1) t = fold_xor_f64(t, m);
        // folds that join layers: binary counter over the bit-reversed visiting order
        double carry = t;
        bool parked = false;
#pragma unroll
        for (int j = 0; j < 6; j++) {
            if (!parked && (uint32_t)j < log2L) {
                if (((it >> j) & 1u) == 0) { stk[j] = carry; parked = true; }
                else carry = stk[j] + carry;
            }
        }
        if (!parked) total = carry;                             // only at the last layer
    };
    // NS layers per trip, one register stage each (L is a multiple of NS)
    issue(st0, 0);
    issue(st1, 1);
    if (NS == 4) { issue(st2, 2); issue(st3, 3); }
    for (uint32_t it = 0; it < L; it += NS) {
        body(st0, it);
        body(st1, it + 1);
        if (NS == 4) { body(st2, it + 2); body(st3, it + 3); }
    }
    if (!has_s) return;
    // block sums: lane (b * 64/L) holds block b of this tile
    const uint32_t bpl = 64u >> log2L;
    const uint32_t nblk = (rows + bpl - 1) / bpl;
    if (((uint32_t)lane & (bpl - 1)) == 0 && (uint32_t)lane / bpl < nblk)
        blocksum[(size_t)s * nb_total + (size_t)tile * L + (uint32_t)lane / bpl] = total;
    // Eq. 5 per token step, and the verdict of the tile
    uint32_t ex = 0;
    if (active) {
        if (occ_out) occ_out[(size_t)s * N + n] = occ_acc;
        ex = occ_acc > q.cap ? occ_acc - q.cap : 0;
    }
    ex = wave_max_u32(ex);
    const uint32_t fl = wave_or_u32(active ? fl_acc : 0u);
    if (lane == 0) tileflag[(size_t)s * tiles + tile] = ex | (fl ? 0x80000000u : 0u);
}

template <int WD>
int launch_quad(kvp_ctx *ctx, const uint32_t *X, uint32_t S, uint32_t tiles, uint32_t nb_total, uint32_t log2L,
                uint32_t *counters, uint32_t *occ) {
    const DevProblem &q = ctx->dp;
    constexpr size_t XW = (size_t)vecs_per_lane((TILE_N + 1) * WD) * 64 * 4;
    static_assert((TILE_N * WD + 3 + 3) / 4 <= QUAD * 64, "one vector per thread must cover a trace chunk");
    const size_t lds = (QUAD * XW + 2 * A_SLOT) * 4;
    const uint64_t nwg = (uint64_t)((S + QUAD - 1) / QUAD) * tiles;
    if (nwg > 0x7FFFFFFFull) return 1;
    dim3 grid((uint32_t)nwg), block(QUAD * 64);
    const bool pf = WD > 1 && ctx->prefix_full, w1 = q.single_write != 0;
#define KVP_GO(WW, PP, NN)                                                                             \
    score_quad_kernel<WD, WW, PP, NN><<<grid, block, lds, ctx->stream>>>(q, X, S, tiles, nb_total, log2L, \
                                                                        ctx->d_blocksum, ctx->d_tileflag, counters, occ)
    if (w1 && pf) KVP_GO(true, true, 2); else if (w1) KVP_GO(true, false, 2);
    else if (pf) KVP_GO(false, true, 2); else KVP_GO(false, false, 2);
#undef KVP_GO
    KVP_HIP(hipGetLastError());
    ctx->last_kernel = KVP_SCORE_QUAD;
    return KVP_OK;
}

}  // namespace

// Returns KVP_OK if launched, 1 if this kernel does not cover the shape, <0 on error.
int kvp_score_quad_launch(kvp_ctx *ctx, const uint32_t *X, uint32_t S, uint32_t tiles, uint32_t nb_total,
                          uint32_t *counters, uint32_t *occ) {
    const DevProblem &q = ctx->dp;
    if (q.K != 1 || q.wt[0] != 1 || q.L > 64 || q.L < 2 || (q.L & (q.L - 1)) != 0) return 1;
    // Chunks are fetched as whole 16-byte vectors, up to three words past their end.  Inside the
    // batch that is the next chunk; at the very end it is only safe if the batch ends on a vector
    // boundary.  (The trace array is followed by the other trace arrays in one allocation.)
    if (((size_t)S * q.L * q.N * q.Wd) % 4 != 0) return 1;
    uint32_t log2L = 0;
    while ((1u << log2L) < q.L) log2L++;
    switch (q.Wd) {
#define KVP_CASE(W) case W: return launch_quad<W>(ctx, X, S, tiles, nb_total, log2L, counters, occ);
        KVP_CASE(1) KVP_CASE(2) KVP_CASE(3) KVP_CASE(4) KVP_CASE(5) KVP_CASE(6) KVP_CASE(7) KVP_CASE(8)
        KVP_CASE(9) KVP_CASE(10) KVP_CASE(11) KVP_CASE(12) KVP_CASE(13) KVP_CASE(14) KVP_CASE(15)
#undef KVP_CASE
        default: return 1;
    }
}
