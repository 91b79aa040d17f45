// Scorer for rows of 16 to 68 words of a single decoding sequence (the prompt's
// pages are there at step 0, pages born later follow them in the row) where one
// page is written per step.
//
//   * A workgroup is four wavefronts scoring the same 64 token steps of four
//     schedules.  Per layer the tile is taken in two passes of 32 steps; in a pass
//     a wavefront fetches its 33 rows (32 steps and the step before) WHOLE, as
//     16-byte vectors that follow each other in memory, so every 128-byte line is
//     requested once and by one instruction group.  The vectors are parked in LDS
//     with a row stride of 2 (mod 4) words and two lanes share a row, one taking
//     the even words and one the odd: the 32 lanes that the LDS serves per cycle
//     hit its 32 banks once each.
//   * The access planes are replaced by the binary digits of each page's read
//     weight (sum over planes of plane_bytes/unit): K planes of equal size become
//     floor(log2 K) + 1 digit planes, and hr = sum_j 2^j popcount(x & digit_j).
//     The digit planes of a pass are fetched once per workgroup into a
//     double-buffered LDS slot, one pass ahead, and so are the rows, into registers
//     (two passes ahead cost 36 more registers and, on rows of 66 words, the third
//     wavefront per SIMD: 6 % slower).
//   * On a tile of 64 steps the words below the first one that is not FULL there need
//     no masks; the at most four words from there to the sequence's end use alive /
//     persist words that do not depend on the layer and stay in registers for the
//     whole kernel; the words past the end hold no page and are only checked for
//     stray bits.  The ranges are the tile's own, so the sequence may grow for long.
//   * Step latencies are summed on the fly when L is a power of two (bit-reversed
//     layer order, binary counter of partial sums: the 64-wide tree of the
//     definition) and when L = 2^k q with 3 <= k <= 5 and q in {3, 5, 7} (see
//     MIXED below); otherwise they go to a [S][L][N] array that a second kernel sums.
#include "kvp_internal.h"

namespace {

typedef uint32_t r4u __attribute__((ext_vector_type(4), aligned(4)));   // rows are only 4-byte aligned

constexpr int RQ = 4;          // schedules (= wavefronts) per workgroup
constexpr int RR = 32;         // token steps per pass (two lanes per step)
constexpr int TWMAX = 4;       // words at the end of a row that may need masks

typedef uint32_t a2u __attribute__((ext_vector_type(2)));               // 8-byte aligned LDS words

__device__ __forceinline__ void put4(uint32_t *p, r4u v) { p[0] = v.x; p[1] = v.y; p[2] = v.z; p[3] = v.w; }
// The same at an even word of LDS: two 8-byte writes.  (An LDS instruction costs some four cycles of the LDS
// pipeline whatever its width, and a 4-byte write at a lane stride of four words twice that.)
__device__ __forceinline__ void put22(uint32_t *p, r4u v) {
    *(a2u *)p = (a2u){v.x, v.y};
    *(a2u *)(p + 2) = (a2u){v.z, v.w};
}
__device__ __forceinline__ uint32_t pair_sum(uint32_t v) {            // v + the other lane of the row
    return v + (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xf, 0xf, false);   // quad_perm [1,0,3,2]
}

// binary digit planes of the read weights: Aw[l][n][j][w], j < KB
__global__ __launch_bounds__(256) void bitslice_kernel(DevProblem q, uint32_t KB, uint32_t *__restrict__ Aw) {
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;           // (l*N + n)*Wd + w
    const size_t total = (size_t)q.L * q.N * q.Wd;
    if (i >= total) return;
    const size_t row = i / q.Wd;
    const uint32_t w = (uint32_t)(i - row * q.Wd);
    uint32_t d[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    for (uint32_t k = 0; k < q.K; k++) {
        const uint32_t a = q.A[(row * q.K + k) * q.Wd + w];
        for (uint32_t b = 0; b < 8; b++) {
            if (!((q.wt[k] >> b) & 1u)) continue;
            uint32_t carry = a;                                        // add a * 2^b to the digit planes
#pragma unroll
            for (uint32_t j = 0; j < 8; j++) {
                if (j < b) continue;
                const uint32_t t = d[j] & carry;
                d[j] ^= carry;
                carry = t;
            }
        }
    }
    for (uint32_t j = 0; j < KB; j++) Aw[(row * KB + j) * q.Wd + w] = d[j];
}

// How the step latencies of a tile reach the 64-wide summation tree.
//   SPILL: written to a [S][L][N] array; a second kernel sums them.
//   POW2:  L = 2^k <= 64.  Position g = n L + l has the layer in its low k bits, so the tree first
//          joins the 64 / L steps of a block (cross-lane adds) and then layers that differ in bit
//          k-1, k-2, ...: with the layers visited in bit-reversed order that is a binary counter of
//          k partial sums per lane.
//   MIXED: L = 2^k q, q odd.  Write l = 2^k lh + ll; then g = 2^k (q n + lh) + ll, so for a fixed ll
//          the values m = q n + lh = 0, 1, 2, ... of a tile fall into the blocks c = 64 / 2^k at a
//          time (block m / c, upper tree bits m % c), and the 64 q values of a tile make exactly L
//          blocks.  Layers are visited ll-major (ll bit-reversed, lh = 0 .. q-1 inside): after the q
//          layers of one ll a wavefront has 64 q latencies in LDS, every lane adds the c values of
//          "its" blocks in tree order, and the partial block sums of the 2^k values of ll meet in a
//          binary counter as above, kept in LDS (k levels of L sums).
enum { SPILL = 0, POW2 = 1, MIXED = 2 };

// XV: 16-byte vectors per lane and pass (33 rows); KB: digit planes; MODE: see above.
// No load is consumed in the pass that issues it, and all are unconditional: offsets that would
// leave the schedule (or the planes) are clamped, and what they fetch is never used.
//
// Lane (r, h2), r = lane / 2, h2 = lane % 2: in pass p it counts the words w = h2 (mod 2) of step
// 32 p + r; the two lanes of a row then add their counters.  After pass 1 lane (r, h2) keeps the
// counters of step 32 h2 + r, "its own" step: Eqs. 2-4, the occupancy and the summation tree then
// run once per layer with all 64 lanes busy.  The masked words at the end of a row are taken by the
// lane that owns the row.
template <int XV, int KB, int MODE>
__global__ __launch_bounds__(RQ * 64) void score_rowblock_kernel(
    DevProblem q, const uint32_t *__restrict__ Aw, const uint32_t *__restrict__ X, uint32_t S, uint32_t tiles,
    uint32_t nb_total, uint32_t log2L, uint32_t qodd, double *__restrict__ blocksum, double *__restrict__ tglobal,
    uint32_t *__restrict__ tileflag, uint32_t *__restrict__ counters, uint32_t *__restrict__ occ_out) {
    extern __shared__ double smem_d[];
    constexpr int UN = (KB >= 2 && MODE != MIXED) ? 4 : 8;             // unroll of the word loop
    constexpr int TV = (KB * XV * 8 + 32) / 33;                        // trace vectors per thread and pass
    const uint32_t L = q.L, N = q.N, Wd = q.Wd;
    // LDS row stride = 2 (mod 4): the LDS serves 32 lanes per cycle from 32 banks, and lanes (r, h2),
    // r < 16, then read words 2r + h2 + const (mod 32) of their rows: all different
    const uint32_t RS = Wd + ((6 - (Wd & 3u)) & 3u), PPR = (Wd + 3) / 4;
    const uint32_t TPL = RR * RS;                                      // words of one digit plane in a slot
    const uint32_t tid = threadIdx.x;
    const int lane = lane_id();
    const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane((int)(tid / KVP_WAVE));
    uint32_t tile, group;                                             // see xcd_pair for the placement
    if (!xcd_pair(tiles, (S + RQ - 1) / RQ, tile, group)) return;
    const uint32_t s = group * RQ + wave;
    const bool has_s = s < S;
    const uint32_t sc = has_s ? s : S - 1;                            // spare wavefronts shadow the last schedule
    const uint32_t n0 = tile * 64;
    const uint32_t rows = min(64u, N - n0);
    uint32_t *xbuf = (uint32_t *)smem_d + (size_t)wave * (RR + 1) * RS;
    uint32_t *tbuf = (uint32_t *)smem_d + (size_t)RQ * (RR + 1) * RS;  // two slots of KB * TPL words
    // MIXED: the wavefront's 64 q latencies of one ll, then its k levels of L partial block sums
    double *stage = (double *)(tbuf + 2 * KB * TPL) + (size_t)wave * (64 * qodd + log2L * L);
    double *level = stage + 64 * qodd;
    const uint32_t r = (uint32_t)lane >> 1, h2 = (uint32_t)lane & 1u;
    // The words of a row on this tile: [0, pfw2) FULL at every step (no masks needed), [pfw2, wend) with
    // masks (at most TWMAX: the host checks), [wend, Wd) without a page at any step (only stray bits).
    const uint32_t pfw2 = q.tile_pfw[tile] & ~1u, wend = q.tile_end[tile];
    const uint32_t tw = wend - pfw2;

    // the lane's own step
    const uint32_t rho = h2 * RR + r;
    const bool active = rho < rows;
    const uint32_t n = n0 + (active ? rho : rows - 1);                // idle lanes shadow the last row
    const uint32_t wr_n = q.wr[n], wsel = q.wsel[n];
    const uint32_t wmw = q.Wm[(size_t)n * Wd + wsel];
    uint32_t vt[TWMAX], pt[TWMAX];
#pragma unroll
    for (int t = 0; t < TWMAX; t++) {
        const uint32_t w = min(pfw2 + t, Wd - 1);
        vt[t] = q.V[(size_t)n * Wd + w];
        pt[t] = q.Pm[(size_t)n * Wd + w];
    }
    // vector slots of the lane: word offsets from the first row of a pass, in memory and in LDS
    uint32_t xrel[XV], xlds[XV], trel[TV], tlds[TV];
#pragma unroll
    for (int jv = 0; jv < XV; jv++) {
        const uint32_t vi = min((uint32_t)lane + 64u * jv, (RR + 1) * PPR - 1);
        const uint32_t row = vi / PPR, part = vi - row * PPR;
        const uint32_t w0 = min(4 * part, Wd - 4);                     // a row's last vector ends at the row's end
        xrel[jv] = 4 * (row * Wd + w0);                                // bytes from the first row of a pass
        xlds[jv] = row * RS + w0;
    }
#pragma unroll
    for (int jt = 0; jt < TV; jt++) {
        const uint32_t ti = min(tid + 256u * jt, KB * RR * PPR - 1);
        const uint32_t k = ti / (RR * PPR), rem = ti - k * RR * PPR;
        const uint32_t row = rem / PPR, part = rem - row * PPR;
        const uint32_t w0 = min(4 * part, Wd - 4);
        trel[jt] = 4 * ((row * KB + k) * Wd + w0);
        tlds[jt] = k * TPL + row * RS + w0;
    }
    // Pass p of layer l starts at word ((l*N + n0 + 32p) - 1) * Wd of the schedule: the step before
    // comes first.  Step 0 has none: there the offsets are clamped from below and the lanes of step 0
    // use the step itself as its predecessor (nothing migrates at step 0).
    const uint32_t sched_words = L * N * Wd;                           // < 2^31 (checked by the host)

    struct Stage { r4u x[XV]; };
    Stage st0;
    uint32_t acc_nx = 0;                                               // read units of the lane's step, next layer
    r4u tr[TV];
    // i-th layer in visiting order (i / q by a multiplication: exact for i < 256, q <= 7; the host checks)
    const uint32_t qinv = 65536u / qodd + 1u;
    auto layer_of = [&](uint32_t i) {
        if (MODE == POW2) return __brev(i) >> (32 - log2L);
        if (MODE == MIXED) {
            const uint32_t vi = (i * qinv) >> 16, lh = i - vi * qodd;
            return (lh << log2L) + (__brev(vi) >> (32 - log2L));
        }
        return i;
    };
    // Addresses are a wavefront-uniform base plus a 32-bit byte offset per lane (the host checks
    // that a schedule and the digit planes stay below 4 GiB).  A pass whose 33 rows all lie inside the
    // schedule (no step before step 0, no steps past the trace) needs no clamping.
    const char *Xs = (const char *)(X + (size_t)sc * sched_words);
    const bool edge_tile = rows < 64;
    auto issue_x = [&](Stage &st, uint32_t p, uint32_t l) __attribute__((always_inline)) {
        const int before = 4 * ((int)((l * N + n0 + RR * p) * Wd) - (int)Wd);   // byte of the step before the pass; < 0 at step 0
        if (before >= 0 && !edge_tile) {
#pragma unroll
            for (int jv = 0; jv < XV; jv++) st.x[jv] = KVP_LOAD_X((const r4u *)(Xs + ((uint32_t)before + xrel[jv])));
        } else {
            const int hi = 4 * ((int)sched_words - 4);
#pragma unroll
            for (int jv = 0; jv < XV; jv++) st.x[jv] = KVP_LOAD_X((const r4u *)(Xs + (uint32_t)min(max(before + (int)xrel[jv], 0), hi)));
        }
    };
    auto issue_t = [&](uint32_t p, uint32_t l) __attribute__((always_inline)) {
        const uint32_t first = 4 * (l * N + n0 + RR * p) * KB * Wd;
        const char *Ab = (const char *)Aw;
        if (!edge_tile) {
#pragma unroll
            for (int jt = 0; jt < TV; jt++) tr[jt] = *(const r4u *)(Ab + (first + trel[jt]));
        } else {
            const uint32_t hi = 4 * (L * N * KB * Wd - 4);
#pragma unroll
            for (int jt = 0; jt < TV; jt++) tr[jt] = *(const r4u *)(Ab + min(first + trel[jt], hi));
        }
    };
    auto commit_t = [&](uint32_t slot) __attribute__((always_inline)) {
        uint32_t *dst = tbuf + slot * KB * TPL;
#pragma unroll
        for (int jt = 0; jt < TV; jt++) {
            if (Wd & 1u) put4(dst + tlds[jt], tr[jt]);
            else put22(dst + tlds[jt], tr[jt]);
        }
    };

    const uint32_t row_off = r * RS;
    const bool very_first = n0 == 0 && r == 0;                         // the lane's row in pass 0 is step 0
    uint32_t fl_acc = 0, occ_acc = 0;
    double stk[6] = {0.0, 0.0, 0.0, 0.0, 0.0, 0.0}, total = 0.0;
    const uint32_t nfull = pfw2 >> 1;                                  // unmasked words per lane
    uint32_t hr, hw, oc, mi, mg;                                       // the lane's own step, this layer
    // one pass: stage st holds the rows of (layer i-th in visiting order, pass p)
    auto pass = [&](Stage &st, const uint32_t p, uint32_t i) __attribute__((always_inline)) {
        const uint32_t lnext = layer_of(min(i + 1, L - 1));
        // rows of an even number of words: every vector starts at an even word of LDS (the row stride is even)
        if (Wd & 1u) {
#pragma unroll
            for (int jv = 0; jv < XV; jv++) put4(xbuf + xlds[jv], st.x[jv]);
        } else {
#pragma unroll
            for (int jv = 0; jv < XV; jv++) put22(xbuf + xlds[jv], st.x[jv]);
        }
        issue_t(p ^ 1u, p ? lnext : layer_of(i));                      // digit planes of the next pass
        issue_x(st, p ^ 1u, p ? lnext : layer_of(i));                  // rows of the next pass
        __syncthreads();                                               // this pass's trace slot is complete
        // (addresses and masks below are rebuilt in every pass from these two copies: kept across the
        // layer loop they would occupy some sixty registers)
        uint32_t ro = row_off, hv = h2;                                // ro: the row's offset in a parked pass, words
        asm volatile("" : "+v"(ro), "+v"(hv));
        const uint32_t *cur = xbuf + RS + ro, *prv = xbuf + ((p == 0 && very_first) ? RS : ro);
        const uint32_t *ts = tbuf + p * KB * TPL + ro;
        const bool own = hv == p;
        uint32_t hrk[KB], c_oc = 0, c_mi = 0, c_mg = 0;
#pragma unroll
        for (int k = 0; k < KB; k++) hrk[k] = 0;
        // (a deeper unroll keeps more LDS words in flight per wavefront; with several planes the
        // registers are better spent on a third wavefront per SIMD)
#pragma unroll UN
        for (uint32_t j = 0; j < nfull; j++) {
            const uint32_t w = 2 * j + hv;
            const uint32_t raw = cur[w], d = raw ^ prv[w];
#pragma unroll
            for (int k = 0; k < KB; k++) hrk[k] += __popc(raw & ts[k * TPL + w]);
            c_oc += __popc(raw);
            c_mi += __popc(d & raw);
            c_mg += __popc(d);
        }
        uint32_t flt = 0;
#pragma unroll
        for (int t = 0; t < TWMAX; t++) {
            if ((uint32_t)t < tw) {
                const uint32_t w = pfw2 + t;
                const uint32_t vv = own ? vt[t] : 0u, pp = own ? pt[t] : 0u;
                const uint32_t raw = cur[w], x = raw & vv;
                flt |= raw & ~vv;
                const uint32_t d = (x ^ prv[w]) & pp;
#pragma unroll
                for (int k = 0; k < KB; k++) hrk[k] += __popc(x & ts[k * TPL + w]);
                c_oc += __popc(x);
                c_mi += __popc(d & x);
                c_mg += __popc(d);
            }
        }
        fl_acc |= (own && active) ? flt : 0u;
        uint32_t fdead = 0;                                            // bits where no page exists: the row's lanes take turns
        for (uint32_t w = wend + ((wend ^ hv) & 1u); w < Wd; w += 2) fdead |= cur[w];
        fl_acc |= (RR * p + r < rows) ? fdead : 0u;
        uint32_t c_hr = 0;
#pragma unroll
        for (int k = 0; k < KB; k++) c_hr += hrk[k] << k;
        c_hr = pair_sum(c_hr); c_oc = pair_sum(c_oc); c_mi = pair_sum(c_mi); c_mg = pair_sum(c_mg);
        const uint32_t c_hw = __popc(cur[wsel] & wmw);                 // written pages exist: no alive mask needed
        if (p == 0) { hr = c_hr; oc = c_oc; mi = c_mi; mg = c_mg; hw = c_hw; }
        else if (h2) { hr = c_hr; oc = c_oc; mi = c_mi; mg = c_mg; hw = c_hw; }
        commit_t(p ^ 1u);                                              // arrived while this pass was scored
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
        if (MODE == POW2) {
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
        } else if (MODE == MIXED) {
            const uint32_t vi = (i * qinv) >> 16, lh = i - vi * qodd, c = 64u >> log2L;
            stage[qodd * rho + lh] = t;
            if (lh == qodd - 1) {                                      // the q layers of this ll are in
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
                for (uint32_t b = 0; b < 2; b++) {
                    const uint32_t B = (uint32_t)lane + 64u * b;       // block of the tile
                    if (B < L) {
                        double v[8];
#pragma unroll
                        for (uint32_t j = 0; j < 8; j++) v[j] = j < c ? stage[c * B + j] : 0.0;   // + 0.0 changes nothing
#pragma unroll
                        for (uint32_t h = 4; h >= 1; h >>= 1)
#pragma unroll
                            for (uint32_t j = 0; j < h; j++) v[j] = v[j] + v[j + h];
                        double carry = v[0];
                        bool parked = false;
#pragma unroll
                        for (uint32_t j = 0; j < 5; j++) {
                            if (!parked && j < log2L) {
                                if (((vi >> j) & 1u) == 0) { level[j * L + B] = carry; parked = true; }
                                else carry = level[j * L + B] + carry;
                            }
                        }
                        // only after the last ll; blocks past the end of the trace do not exist
                        if (!parked && has_s && 64u * B < rows * L) blocksum[(size_t)s * nb_total + (size_t)tile * L + B] = carry;
                    }
                }
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
            }
        } else if (has_s && active) {
            tglobal[((size_t)s * L + l) * N + n] = t;
        }
    };
    issue_t(0, layer_of(0));
    issue_x(st0, 0, layer_of(0));
    acc_nx = q.acc[(size_t)layer_of(0) * N + n];
    commit_t(0);
    for (uint32_t i = 0; i < L; i++) {
        const uint32_t acc_n = acc_nx;
        acc_nx = q.acc[(size_t)layer_of(min(i + 1, L - 1)) * N + n];
        pass(st0, 0, i);
        pass(st0, 1, i);
        layer_end(i, acc_n);
    }
    if (!has_s) return;
    if (MODE == POW2) {
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

// Digit planes of the read weights, built once per trace.  Leaves ctx->d_aw null (and the scorer
// above unavailable) when the weights need more than five digits (five: the tokens read in a page
// of 16, with reads priced per token).
int kvp_bitslice_build(kvp_ctx *ctx) {
    DevProblem &q = ctx->dp;
    ctx->aw = nullptr; ctx->kb = 0;
    q.pl = q.A; q.pn = q.K;
    for (uint32_t k = 0; k < KVP_MAX_PLANES; k++) q.pw[k] = k < q.K ? q.wt[k] : 0;
    uint64_t sum = 0;
    for (uint32_t k = 0; k < q.K; k++) sum += q.wt[k];
    uint32_t kb = 0;
    while ((sum >> kb) != 0) kb++;
    if (kb > 5) return KVP_OK;
    if (q.K == 1 && q.wt[0] == 1) { ctx->aw = q.A; ctx->kb = 1; return kvp_rowlane_build(ctx); }
    const size_t words = (size_t)q.L * q.N * kb * q.Wd;
    KVP_HIP(hipMalloc((void **)&ctx->d_aw, words * 4));
    const size_t cells = (size_t)q.L * q.N * q.Wd;
    bitslice_kernel<<<dim3((uint32_t)((cells + 255) / 256)), dim3(256), 0, ctx->stream>>>(q, kb, ctx->d_aw);
    KVP_HIP(hipGetLastError());
    KVP_HIP(hipStreamSynchronize(ctx->stream));
    ctx->aw = ctx->d_aw; ctx->kb = kb;
    q.pl = ctx->d_aw; q.pn = kb;
    for (uint32_t k = 0; k < KVP_MAX_PLANES; k++) q.pw[k] = k < kb ? 1u << k : 0;
    return kvp_rowlane_build(ctx);
}

// Returns KVP_OK if launched, 1 if this kernel does not cover the shape, <0 on error.
int kvp_score_rowblock_launch(kvp_ctx *ctx, const uint32_t *X, uint32_t S, uint32_t tiles, uint32_t nb_total,
                              uint32_t *counters, uint32_t *occ) {
    const DevProblem &q = ctx->dp;
    if (!ctx->aw || !q.single_write || q.Wd < 16 || q.Wd > 68) return 1;
    if (ctx->max_tail > TWMAX) return 1;
    const uint32_t PPR = (q.Wd + 3) / 4, RS = q.Wd + ((6 - (q.Wd & 3u)) & 3u), KB = ctx->kb;
    const uint32_t need = ((RR + 1) * PPR + 63) / 64;
    const int xv = need <= 5 ? 5 : 9;
    if (need > 9) return 1;
    if ((size_t)q.L * q.N * KB * q.Wd >= (1ull << 29)) return 1;      // 32-bit (signed) byte offsets inside the digit planes
    if ((size_t)q.L * q.N * q.Wd >= (1ull << 29)) return 1;           // and inside a schedule
    uint32_t log2L = 0;
    while ((1u << log2L) < q.L) log2L++;
    const bool pow2 = q.L >= 2 && q.L <= 64 && (1u << log2L) == q.L;
    // L = 2^k q with q odd: summed on chip for 3 <= k <= 5, q in {3, 5, 7}, L <= 128
    uint32_t k2 = 0;
    while (!((q.L >> k2) & 1u)) k2++;
    const uint32_t qodd = q.L >> k2;
    bool mixed = !pow2 && k2 >= 3 && k2 <= 5 && qodd >= 3 && qodd <= 7 && q.L <= 128;
    for (uint32_t i = 0; mixed && i < q.L; i++) mixed = ((i * (65536u / qodd + 1u)) >> 16) == i / qodd;
    size_t lds = ((size_t)RQ * (RR + 1) * RS + 2 * (size_t)KB * RR * RS) * 4;
    if (mixed) lds += (size_t)RQ * (64 * qodd + k2 * q.L) * sizeof(double);
    if (lds > 160 * 1024) return 1;
    const uint64_t nwg = xcd_grid(tiles, (S + RQ - 1) / RQ);
    if (nwg > 0x7FFFFFFFull) return 1;
    const int mode = pow2 ? POW2 : mixed ? MIXED : SPILL;
    if (mode == MIXED) log2L = k2;
    if (mode == SPILL) {
        int rc = kvp_ensure(ctx, (void **)&ctx->d_tglobal, &ctx->tglobal_cap, (size_t)S * q.L * q.N * sizeof(double));
        if (rc) return rc;
    }
    dim3 grid((uint32_t)nwg), block(RQ * 64);
#define KVP_GO(XX, KK, PP)                                                                                          \
    do {                                                                                                            \
        if (lds > 48 * 1024)                                                                                        \
            KVP_HIP(hipFuncSetAttribute((const void *)score_rowblock_kernel<XX, KK, PP>,                            \
                                        hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));                    \
        score_rowblock_kernel<XX, KK, PP><<<grid, block, lds, ctx->stream>>>(                                       \
            q, ctx->aw, X, S, tiles, nb_total, log2L, qodd, ctx->d_blocksum, ctx->d_tglobal, ctx->d_tileflag,      \
            counters, occ);                                                                                         \
    } while (0)
#define KVP_P(XX, KK)                                                                                               \
    do {                                                                                                            \
        if (mode == POW2) KVP_GO(XX, KK, POW2);                                                                     \
        else if (mode == MIXED) KVP_GO(XX, KK, MIXED);                                                              \
        else KVP_GO(XX, KK, SPILL);                                                                                 \
    } while (0)
#define KVP_K(KK) case KK: if (xv == 5) KVP_P(5, KK); else KVP_P(9, KK); break;
    switch (KB) {
        KVP_K(1) KVP_K(2) KVP_K(3) KVP_K(4) KVP_K(5)
        default: return 1;
    }
#undef KVP_K
#undef KVP_P
#undef KVP_GO
    KVP_HIP(hipGetLastError());
    ctx->last_kernel = KVP_SCORE_ROWBLOCK;
    if (mode == SPILL) return kvp_blocksum_from_t_launch(ctx, S, nb_total);
    return KVP_OK;
}
