// Scorer for rows of 29 to 36 words of a single decoding sequence (one page written per step, pages born
// during the decode follow the prompt's in the row): a LANE per token step, a whole layer of a 64-step
// tile per pass.
//
// What bounds such rows is the number of instructions a wavefront has to issue per byte of schedule, and
// next to it the bytes that travel from L2 to the compute units beside the schedule's own: so
//   * a wavefront takes the 65 rows of (schedule, layer, tile) whole, as 16-byte vectors that follow each
//     other in memory, and parks them in LDS with a row stride of 36 words; lane i then reads row i (and
//     the row above it) back with 16-byte LDS reads, which the 32 banks serve without conflicts at that
//     stride, and counts four words per read;
//   * the read weights come as one or two dense binary digit planes, laid out at upload per (layer,
//     tile) with the same row stride, so that the workgroup copies a layer's planes into an LDS slot with
//     aligned 16-byte moves, one layer ahead, once for all its schedules; digit planes above those are
//     almost empty where several access sets seldom meet on a page (one set per KV head) and come as a
//     list of their non-zero words per (layer, 32 steps): lane e looks up the word of entry e in the
//     parked rows and adds 2^digit * popcount(word & mask) to the row's extra read units in LDS;
//   * the words below the tile's first word that is not FULL, rounded down to a multiple of four, need no
//     masks; the at most seven words from there to the sequence's end use alive / persist words that stay
//     in registers; the words past the end hold no page and are only checked for stray bits;
//   * Eqs. 2-4 and the 64-wide summation tree run once per layer with one step per lane; the tree is kept
//     on chip for L = 2^k (binary counter over the bit-reversed layer order) and L = 2^k q, q in {3, 5, 7}
//     (the q latencies of a lane and the partial sums of its blocks wait in registers).
#include "kvp_internal.h"

namespace {

typedef uint32_t r4u __attribute__((ext_vector_type(4), aligned(4)));   // rows in memory are only 4-byte aligned
typedef uint32_t a4u __attribute__((ext_vector_type(4)));               // rows in LDS are 16-byte aligned

constexpr int LRS = 36;         // LDS row stride in words (a multiple of 4, and 4 (mod 32): no bank conflicts)
constexpr int LROWS = 65;       // rows parked per layer: the step before the tile and its 64 steps
constexpr int LXV = 10;         // 16-byte vectors per lane and layer: ceil(65 * 9 / 64)
constexpr int LGEN = 7;         // words between the unmasked groups of four and the sequence's end
constexpr int LQMAX = 7;        // largest odd factor of L whose tree stays on chip

// acc += popcount(v) as the one instruction the hardware has for it
__device__ __forceinline__ void count(uint32_t &acc, uint32_t v) {
    asm("v_bcnt_u32_b32 %0, %1, %0" : "+v"(acc) : "v"(v));
}

enum { SPILL = 0, POW2 = 1, MIXED = 2 };       // how the step latencies reach the summation tree: see kvp_score_rowblock.hip

// KB: dense digit planes (1 or 2); SP: a list of the digit planes above them; NW: wavefronts (= schedules)
// per workgroup.  Planes: [L][tiles][KB][64][LRS] words, zero past the row's and the trace's end.
template <int KB, int MODE, bool SP, int NW>
__global__ __launch_bounds__(NW * 64) void score_rowlane_kernel(
    DevProblem q, const uint32_t *__restrict__ TL, const uint2 *__restrict__ sparse, const uint32_t *__restrict__ X,
    uint32_t S, uint32_t tiles, uint32_t nb_total, uint32_t log2L, uint32_t qodd, double *__restrict__ blocksum,
    double *__restrict__ tglobal, uint32_t *__restrict__ tileflag, uint32_t *__restrict__ counters,
    uint32_t *__restrict__ occ_out) {
    extern __shared__ double smem_d[];
    constexpr uint32_t SLOT = KB * 64 * LRS;                           // words of a trace slot
    constexpr int TV = (KB * 64 * LRS / 4 + NW * 64 - 1) / (NW * 64);  // trace vectors per thread and layer
    const uint32_t L = q.L, N = q.N, Wd = q.Wd;
    const uint32_t PPR = (Wd + 3) / 4;
    const uint32_t tid = threadIdx.x;
    const int lane = lane_id();
    const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane((int)(tid / KVP_WAVE));
    uint32_t tile, group;                                             // see xcd_pair for the placement
    if (!xcd_pair(tiles, (S + NW - 1) / NW, tile, group)) return;
    const uint32_t s = group * NW + wave;
    const bool has_s = s < S;
    const uint32_t sc = has_s ? s : S - 1;                            // spare wavefronts shadow the last schedule
    const uint32_t n0 = tile * 64;
    const uint32_t rows = min(64u, N - n0);
    // LDS: the wavefronts' parked rows, two trace slots, (SP) the rows' extra read units
    uint32_t *xbuf = (uint32_t *)smem_d + (size_t)wave * LROWS * LRS;
    uint32_t *tbuf = (uint32_t *)smem_d + (size_t)NW * LROWS * LRS;
    uint32_t *hx = tbuf + 2 * SLOT + wave * 64;
    // The words of a row on this tile: [0, wg) FULL at every step (no masks needed), in groups of four;
    // [wg, wend) with masks (at most LGEN: the host checks); [wend, Wd) without a page at any step.
    const uint32_t nf4 = q.tile_pfw[tile] >> 2, wg = 4 * nf4, wend = q.tile_end[tile];

    // the lane's own step
    const bool active = (uint32_t)lane < rows;
    const uint32_t n = n0 + (active ? (uint32_t)lane : rows - 1);      // idle lanes shadow the last row
    const uint32_t wr_n = q.wr[n], wsel = q.wsel[n];
    const uint32_t wmw = q.Wm[(size_t)n * Wd + wsel];
    uint32_t vm[LGEN], pm[LGEN];
#pragma unroll
    for (int t = 0; t < LGEN; t++) {
        const uint32_t w = wg + t;
        vm[t] = w < wend ? q.V[(size_t)n * Wd + min(w, Wd - 1)] : 0u;
        pm[t] = w < wend ? q.Pm[(size_t)n * Wd + min(w, Wd - 1)] : 0u;
    }
    // vector slots of the lane: byte offsets from the first parked row in memory, word offsets in LDS
    uint32_t xrel[LXV], xlds[LXV];
#pragma unroll
    for (int jv = 0; jv < LXV; jv++) {
        const uint32_t vi = min((uint32_t)lane + 64u * jv, LROWS * PPR - 1);
        const uint32_t row = vi / PPR, part = vi - row * PPR;
        // Every vector starts at a multiple of four words of its row, so that it goes to LDS as one 16-byte
        // write (an LDS instruction costs some four cycles whatever its width, and four-byte writes at this
        // stride twice that).  A row's last vector then runs up to three words into the next row: they land in
        // the row's padding, which nobody reads.
        xrel[jv] = 4 * (row * Wd + 4 * part);
        xlds[jv] = row * LRS + 4 * part;
    }
    const uint32_t sched_words = L * N * Wd;                           // < 2^29 (checked by the host)
    const uint32_t qinv = 65536u / qodd + 1u;
    auto layer_of = [&](uint32_t i) {
        if (MODE == POW2) return __brev(i) >> (32 - log2L);
        if (MODE == MIXED) {
            const uint32_t vi = (i * qinv) >> 16, lh = i - vi * qodd;
            return (lh << log2L) + (__brev(vi) >> (32 - log2L));
        }
        return i;
    };
    struct Stage { r4u x[LXV]; };
    Stage st0;                                                         // rows of the layer to come
    r4u tr[TV];
    uint2 spe[2] = {make_uint2(0u, 0u), make_uint2(0u, 0u)};
    const char *Xs = (const char *)(X + (size_t)sc * sched_words);
    const bool edge_tile = rows < 64;
    const bool batch_end = sc == S - 1 && tile == tiles - 1;           // the tile's last row of the last layer ends the batch
    // The parked rows of layer l start at the step before the tile.  Step 0 has none: there the offsets are
    // clamped from below and lane 0 uses the step itself as its predecessor (nothing migrates at step 0).
    // Where the rows end with the schedule (the last layer of a tile that the trace does not fill, and the very
    // end of the batch), a vector that would run past the end is fetched from the schedule's last 16 bytes
    // instead and its words are moved down to where they belong.
    auto issue_x = [&](Stage &st, uint32_t l) __attribute__((always_inline)) {
        const int before = 4 * ((int)((l * N + n0) * Wd) - (int)Wd);
        if (before >= 0 && !edge_tile && !(batch_end && l == L - 1)) {
#pragma unroll
            for (int jv = 0; jv < LXV; jv++) st.x[jv] = KVP_LOAD_X((const r4u *)(Xs + ((uint32_t)before + xrel[jv])));
        } else {
            const int hi = 4 * ((int)sched_words - 4);
#pragma unroll
            for (int jv = 0; jv < LXV; jv++) {
                const int at = before + (int)xrel[jv];
                const r4u v = KVP_LOAD_X((const r4u *)(Xs + (uint32_t)min(max(at, 0), hi)));
                const int d = at > hi ? (at - hi) >> 2 : 0;            // words that the fetch was moved back by
                r4u w = v;
                w.x = d == 1 ? v.y : d == 2 ? v.z : d == 3 ? v.w : v.x;
                w.y = d == 1 ? v.z : d == 2 ? v.w : v.y;
                w.z = d == 1 ? v.w : v.z;
                st.x[jv] = w;
            }
        }
    };
    const char *Tt = (const char *)TL + (size_t)tile * SLOT * 4 + 16u * tid;
    auto issue_t = [&](uint32_t l) __attribute__((always_inline)) {
        const char *src = Tt + (size_t)l * tiles * SLOT * 4;
#pragma unroll
        for (int jt = 0; jt < TV; jt++) tr[jt] = *(const r4u *)(src + min((uint32_t)jt * NW * 1024u, SLOT * 4 - NW * 1024u));
        if (SP) {
            const uint32_t NB = (N + 31) / 32;
#pragma unroll
            for (uint32_t b = 0; b < 2; b++) {
                spe[b] = sparse[((size_t)l * NB + min(2 * tile + b, NB - 1)) * KVP_SPARSE_CAP + (uint32_t)lane];
                if (2 * tile + b >= NB) spe[b] = make_uint2(0u, 0u);
            }
        }
    };
    auto commit_t = [&](uint32_t slot) __attribute__((always_inline)) {
        uint32_t *dst = tbuf + slot * SLOT + 4 * tid;
#pragma unroll
        for (int jt = 0; jt < TV; jt++) *(a4u *)(dst + min((uint32_t)jt * NW * 256u, SLOT - NW * 256u)) = (a4u)tr[jt];
    };

    const bool very_first = n0 == 0 && lane == 0;                      // the lane's row is step 0
    uint32_t fl_acc = 0, occ_acc = 0;
    double stk[6] = {0.0, 0.0, 0.0, 0.0, 0.0, 0.0}, total = 0.0;
    double tq[LQMAX] = {0.0, 0.0, 0.0, 0.0, 0.0, 0.0, 0.0};           // MIXED: the lane's latencies of the q layers of one ll
    double lvl[2][5] = {{0.0, 0.0, 0.0, 0.0, 0.0}, {0.0, 0.0, 0.0, 0.0, 0.0}};   // ... and the levels of partial sums of its blocks
    uint32_t hr, hw, oc, mi, mg;
    // one layer: stage st holds its rows, trace slot i & 1 its digit planes
    auto layer = [&](Stage &st, uint32_t i) __attribute__((always_inline)) {
        const uint32_t lnext = layer_of(min(i + 1, L - 1));
#pragma unroll
        for (int jv = 0; jv < LXV; jv++) *(a4u *)(xbuf + xlds[jv]) = (a4u)st.x[jv];
        uint2 e0 = spe[0], e1 = spe[1];
        // (loads complete in the order of their issue: the digit planes, wanted at the end of this layer, go
        // first, so that waiting for them does not wait for the rows, which have until the next layer starts)
        issue_t(lnext);                                                // digit planes (and list) of the next layer
        issue_x(st, lnext);                                            // rows of the next layer
        __syncthreads();                                               // this layer's trace slot is complete
        if (SP) {
#pragma unroll
            for (uint32_t b = 0; b < 2; b++) {
                const uint2 e = b ? e1 : e0;
                if (e.y >> 31) {
                    const uint32_t row = (e.y & 31u) + 32u * b;
                    const uint32_t xw = xbuf[(row + 1u) * LRS + ((e.y >> 8) & 127u)];
                    atomicAdd(&hx[row], (uint32_t)__popc(xw & e.x) << ((e.y >> 16) & 7u));
                }
            }
        }
        uint32_t ro = (uint32_t)lane * LRS;                            // rebuilt per layer: keeps loop-invariant addresses out of registers
        asm volatile("" : "+v"(ro));
        const uint32_t *cur = xbuf + LRS + ro, *prv = very_first ? cur : xbuf + ro;
        const uint32_t *ts = tbuf + (i & 1u) * SLOT + ro;
        uint32_t hrk[KB];
#pragma unroll
        for (int k = 0; k < KB; k++) hrk[k] = 0;
        oc = 0; mi = 0; mg = 0;
#pragma unroll
        for (int j4 = 0; j4 < LRS / 4; j4++) {
            if ((uint32_t)j4 < nf4) {                                  // four words that need no masks
                const a4u xc = *(const a4u *)(cur + 4 * j4), xp = *(const a4u *)(prv + 4 * j4);
                a4u tk[KB];
#pragma unroll
                for (int k = 0; k < KB; k++) tk[k] = *(const a4u *)(ts + k * 64 * LRS + 4 * j4);
#pragma unroll
                for (int e = 0; e < 4; e++) {
                    const uint32_t raw = xc[e], d = raw ^ xp[e];
#pragma unroll
                    for (int k = 0; k < KB; k++) count(hrk[k], raw & tk[k][e]);
                    count(oc, raw);
                    count(mi, d & raw);
                    count(mg, d);
                }
            }
        }
        uint32_t flt = 0;
#pragma unroll
        for (int t = 0; t < LGEN; t++) {
            const uint32_t w = wg + t;
            if (w < wend) {
                const uint32_t raw = cur[w], x = raw & vm[t];
                flt |= raw & ~vm[t];
                const uint32_t d = (x ^ prv[w]) & pm[t];
#pragma unroll
                for (int k = 0; k < KB; k++) count(hrk[k], x & ts[k * 64 * LRS + w]);
                count(oc, x);
                count(mi, d & x);
                count(mg, d);
            }
        }
        for (uint32_t w = wend; w < Wd; w++) flt |= cur[w];           // bits where no page exists
        fl_acc |= active ? flt : 0u;
        hr = 0;
#pragma unroll
        for (int k = 0; k < KB; k++) hr += hrk[k] << k;
        if (SP) {                                                      // the list's share; the wavefront's LDS accesses complete in order
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            hr += hx[lane];
            hx[lane] = 0;
        }
        hw = __popc(cur[wsel] & wmw);                                  // written pages exist: no alive mask needed
        commit_t((i + 1u) & 1u);                                       // arrived while this layer was scored
    };
    // after a layer: Eqs. 2-4 and the layer's place in the summation tree
    auto layer_end = [&](uint32_t i, uint32_t acc_n) __attribute__((always_inline)) {
        const uint32_t l = layer_of(i);
        const uint32_t mo = mg - mi;
        double t = step_time(q, hr, hw, mi, mo, acc_n, wr_n);
        t = active ? t : 0.0;                                          // rows past the end of the trace pad with +0.0
        occ_acc += oc;
        if (counters && has_s && active)
            *(uint4 *)(counters + (((size_t)s * L + l) * N + n) * 4) = make_uint4(hr, hw, mi, mo);
        if (MODE == POW2) {
            // folds of the summation tree that join the steps of one block (lanes)
            for (uint32_t m = (64u >> log2L) >> 1; m >= 1; m >>= 1) t = fold_xor_f64(t, m);
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
#pragma unroll
            for (int j = 0; j < LQMAX; j++) tq[j] = (uint32_t)j == lh ? t : tq[j];
            if (lh == qodd - 1) {
                // The q layers of this ll are in: position m = q step + lh of the tile's 64 q values.  They pass
                // through the wavefront's parked rows (free until the next layer is parked there): every lane
                // then adds the c values of "its" blocks in tree order.
                double *stage = (double *)xbuf;
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
#pragma unroll
                for (int j = 0; j < LQMAX; j++)
                    if ((uint32_t)j < qodd) stage[qodd * (uint32_t)lane + j] = tq[j];
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
                                if (((vi >> j) & 1u) == 0) { lvl[b][j] = carry; parked = true; }
                                else carry = lvl[b][j] + carry;
                            }
                        }
                        // only after the last ll; blocks past the end of the trace do not exist
                        if (!parked && has_s && 64u * B < rows * L) blocksum[(size_t)s * nb_total + (size_t)tile * L + B] = carry;
                    }
                }
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");   // all reads of the stage precede the next parking
                __builtin_amdgcn_wave_barrier();
            }
        } else if (has_s && active) {
            tglobal[((size_t)s * L + l) * N + n] = t;
        }
    };
    if (SP) hx[lane] = 0;
    issue_t(layer_of(0));
    issue_x(st0, layer_of(0));
    uint32_t acc_nx = q.acc[(size_t)layer_of(0) * N + n];
    commit_t(0);
    // Two layers per trip, unconditionally (an odd last layer follows the loop): with the second one under
    // a condition the compiler has to assume the fewest loads in flight where the paths meet, and makes
    // every layer wait for the rows of the next.
    for (uint32_t i = 0; i + 1 < L; i += 2) {
        uint32_t acc_n = acc_nx;
        acc_nx = q.acc[(size_t)layer_of(i + 1) * N + n];
        layer(st0, i);
        layer_end(i, acc_n);
        acc_n = acc_nx;
        acc_nx = q.acc[(size_t)layer_of(min(i + 2, L - 1)) * N + n];
        layer(st0, i + 1);
        layer_end(i + 1, acc_n);
    }
    if (L & 1u) {
        layer(st0, L - 1);
        layer_end(L - 1, acc_nx);
    }
    if (!has_s) return;
    if (MODE == POW2) {
        const uint32_t bpl = 64u >> log2L;                             // block b of the tile: steps [b*bpl, (b+1)*bpl)
        if (((uint32_t)lane & (bpl - 1)) == 0 && (uint32_t)lane < rows)
            blocksum[(size_t)s * nb_total + (size_t)tile * L + (uint32_t)lane / bpl] = total;
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

// Non-zero words of every digit plane above plane 0, per (layer, block of 32 token steps):
// cnt[(j - 1) * L * NB + l * NB + b] for plane j.  One wavefront per block.
__global__ __launch_bounds__(64) void sparse_count_kernel(DevProblem q, uint32_t KB, const uint32_t *__restrict__ Aw,
                                                          uint32_t NB, uint32_t *__restrict__ cnt) {
    const uint32_t l = blockIdx.x / NB, b = blockIdx.x - l * NB, lane = threadIdx.x;
    const uint32_t n0 = b * 32, rows = min(32u, q.N - n0);
    for (uint32_t j = 1; j < KB; j++) {
        uint32_t c = 0;
        for (uint32_t i = lane; i < rows * q.Wd; i += 64) {
            const uint32_t row = i / q.Wd, w = i - row * q.Wd;
            c += Aw[(((size_t)l * q.N + n0 + row) * KB + j) * q.Wd + w] != 0;
        }
        c = wave_sum_u32(c);
        if (lane == 0) cnt[((size_t)(j - 1) * q.L + l) * NB + b] = c;
    }
}

// The list of a block: the non-zero words of planes KD..KB-1 in the order (row, plane, word) as
// {mask, row | word << 8 | plane << 16 | 1 << 31}, unused slots zero.  One wavefront per block; the
// host has checked that no block has more than KVP_SPARSE_CAP of them.
__global__ __launch_bounds__(64) void sparse_fill_kernel(DevProblem q, uint32_t KB, uint32_t KD,
                                                         const uint32_t *__restrict__ Aw, uint32_t NB,
                                                         uint2 *__restrict__ ent) {
    const uint32_t l = blockIdx.x / NB, b = blockIdx.x - l * NB, lane = threadIdx.x;
    const uint32_t n0 = b * 32, rows = min(32u, q.N - n0), per_row = (KB - KD) * q.Wd;
    uint2 *out = ent + (size_t)blockIdx.x * KVP_SPARSE_CAP;
    out[lane] = make_uint2(0u, 0u);
    __syncthreads();
    uint32_t base = 0;
    for (uint32_t i0 = 0; i0 < rows * per_row; i0 += 64) {
        const uint32_t i = i0 + lane;
        uint32_t m = 0, meta = 0;
        if (i < rows * per_row) {
            const uint32_t row = i / per_row, rem = i - row * per_row, j = KD + rem / q.Wd, w = rem % q.Wd;
            m = Aw[(((size_t)l * q.N + n0 + row) * KB + j) * q.Wd + w];
            meta = row | (w << 8) | (j << 16) | 0x80000000u;
        }
        const uint64_t nz = __ballot(m != 0);
        const uint32_t pos = base + (uint32_t)__popcll(nz & ((1ull << lane) - 1ull));
        if (m != 0 && pos < KVP_SPARSE_CAP) out[pos] = make_uint2(m, meta);
        base += (uint32_t)__popcll(nz);
    }
}

// The low KD planes per (layer, tile) with the LDS row stride: out[l][tile][k][64][LRS].
__global__ __launch_bounds__(256) void tile_planes_kernel(DevProblem q, uint32_t KB, uint32_t KD, uint32_t tiles,
                                                          const uint32_t *__restrict__ Aw, uint32_t *__restrict__ out) {
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    const size_t total = (size_t)q.L * tiles * KD * 64 * LRS;
    if (i >= total) return;
    const uint32_t w = (uint32_t)(i % LRS);
    size_t rest = i / LRS;
    const uint32_t row = (uint32_t)(rest & 63u); rest >>= 6;
    const uint32_t k = (uint32_t)(rest % KD); rest /= KD;
    const uint32_t tile = (uint32_t)(rest % tiles), l = (uint32_t)(rest / tiles);
    const uint32_t nn = tile * 64 + row;
    out[i] = (w < q.Wd && nn < q.N) ? Aw[(((size_t)l * q.N + nn) * KB + k) * q.Wd + w] : 0u;
}

}  // namespace

int kvp_blocksum_from_t_launch(kvp_ctx *ctx, uint32_t S, uint32_t nb_total);

// Whether the scorer above covers the trace's shape.
static bool rowlane_shape(const kvp_ctx *ctx) {
    const DevProblem &q = ctx->dp;
    return ctx->aw && q.single_write && q.Wd >= 29 && q.Wd <= LRS && ctx->max_tail <= 4;
}

// Built once per trace, after the digit planes: the low planes per tile and the list of the rest.  Takes
// the smallest number of dense planes (1 or 2) for which no (layer, 32 steps) block lists more than
// KVP_SPARSE_CAP words of the planes above them.  Leaves ctx->d_tl null where the scorer does not apply.
int kvp_rowlane_build(kvp_ctx *ctx) {
    const DevProblem &q = ctx->dp;
    if (!rowlane_shape(ctx)) return KVP_OK;
    const uint32_t KB = ctx->kb, NB = (q.N + 31) / 32, tiles = (q.N + 63) / 64;
    const size_t blocks = (size_t)q.L * NB;
    if (blocks > 0x7FFFFFFFull) return KVP_OK;
    uint32_t kd = KB <= 2 ? KB : 0;
    if (KB > 2) {
        uint32_t *d_cnt = nullptr;
        KVP_HIP(hipMalloc((void **)&d_cnt, (size_t)(KB - 1) * blocks * 4));
        sparse_count_kernel<<<dim3((uint32_t)blocks), dim3(64), 0, ctx->stream>>>(q, KB, ctx->aw, NB, d_cnt);
        hipError_t e = hipGetLastError();
        uint32_t *h = (uint32_t *)malloc((size_t)(KB - 1) * blocks * 4);
        if (e == hipSuccess && !h) { (void)hipFree(d_cnt); return KVP_ENOMEM; }
        if (e == hipSuccess) e = hipMemcpyAsync(h, d_cnt, (size_t)(KB - 1) * blocks * 4, hipMemcpyDeviceToHost, ctx->stream);
        if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
        (void)hipFree(d_cnt);
        if (e != hipSuccess) { free(h); KVP_HIP(e); }
        for (uint32_t cand = 1; cand <= 2 && !kd; cand++) {
            bool fits = true;
            for (size_t b = 0; b < blocks && fits; b++) {
                uint64_t c = 0;
                for (uint32_t j = cand; j < KB; j++) c += h[(size_t)(j - 1) * blocks + b];
                fits = c <= KVP_SPARSE_CAP;
            }
            if (fits) kd = cand;
        }
        free(h);
        if (!kd) return KVP_OK;
        KVP_HIP(hipMalloc((void **)&ctx->d_sparse, blocks * KVP_SPARSE_CAP * sizeof(uint2)));
        sparse_fill_kernel<<<dim3((uint32_t)blocks), dim3(64), 0, ctx->stream>>>(q, KB, kd, ctx->aw, NB, ctx->d_sparse);
        KVP_HIP(hipGetLastError());
    }
    const size_t words = (size_t)q.L * tiles * kd * 64 * LRS;
    KVP_HIP(hipMalloc((void **)&ctx->d_tl, words * 4));
    tile_planes_kernel<<<dim3((uint32_t)((words + 255) / 256)), dim3(256), 0, ctx->stream>>>(q, KB, kd, tiles, ctx->aw, ctx->d_tl);
    KVP_HIP(hipGetLastError());
    KVP_HIP(hipStreamSynchronize(ctx->stream));
    ctx->kd = kd;
    return KVP_OK;
}

// Returns KVP_OK if launched, 1 if this kernel does not cover the shape, <0 on error.
int kvp_score_rowlane_launch(kvp_ctx *ctx, const uint32_t *X, uint32_t S, uint32_t tiles, uint32_t nb_total,
                             uint32_t *counters, uint32_t *occ) {
    const DevProblem &q = ctx->dp;
    if (!ctx->d_tl || !rowlane_shape(ctx)) return 1;
    const uint32_t KB = ctx->kd;
    const bool sp = ctx->d_sparse != nullptr;
    if ((size_t)q.L * q.N * q.Wd >= (1ull << 29)) return 1;           // 32-bit (signed) byte offsets inside a schedule
    uint32_t log2L = 0;
    while ((1u << log2L) < q.L) log2L++;
    const bool pow2 = q.L >= 2 && q.L <= 64 && (1u << log2L) == q.L;
    // L = 2^k q with q odd: summed on chip for 3 <= k <= 5, q in {3, 5, 7}, L <= 128
    uint32_t k2 = 0;
    while (!((q.L >> k2) & 1u)) k2++;
    const uint32_t qodd = q.L >> k2;
    bool mixed = !pow2 && k2 >= 3 && k2 <= 5 && qodd >= 3 && qodd <= LQMAX && q.L <= 128;
    for (uint32_t i = 0; mixed && i < q.L; i++) mixed = ((i * (65536u / qodd + 1u)) >> 16) == i / qodd;
    if (mixed && (size_t)64 * qodd * sizeof(double) > (size_t)LROWS * LRS * 4) return 1;   // the stage borrows the parked rows' place
    // Four wavefronts per workgroup, two workgroups per compute unit: the workgroups' barriers fall at different
    // times, so one's arithmetic fills the other's waits (eight wavefronts in one workgroup: 6 % slower).
    constexpr int NW = 4;
    size_t lds = ((size_t)NW * LROWS * LRS + 2 * (size_t)KB * 64 * LRS + (sp ? NW * 64 : 0)) * 4;
    if (lds > 160 * 1024) return 1;
    const uint64_t nwg = xcd_grid(tiles, (S + NW - 1) / NW);
    if (nwg > 0x7FFFFFFFull) return 1;
    const int mode = pow2 ? POW2 : mixed ? MIXED : SPILL;
    if (mode == MIXED) log2L = k2;
    if (mode == SPILL) {
        int rc = kvp_ensure(ctx, (void **)&ctx->d_tglobal, &ctx->tglobal_cap, (size_t)S * q.L * q.N * sizeof(double));
        if (rc) return rc;
    }
    dim3 grid((uint32_t)nwg), block(NW * 64);
#define KVP_GO(KK, PP, SS)                                                                                          \
    do {                                                                                                            \
        if (lds > 48 * 1024)                                                                                        \
            KVP_HIP(hipFuncSetAttribute((const void *)score_rowlane_kernel<KK, PP, SS, NW>,                         \
                                        hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));                    \
        score_rowlane_kernel<KK, PP, SS, NW><<<grid, block, lds, ctx->stream>>>(                                    \
            q, ctx->d_tl, ctx->d_sparse, X, S, tiles, nb_total, log2L, qodd, ctx->d_blocksum, ctx->d_tglobal,       \
            ctx->d_tileflag, counters, occ);                                                                        \
    } while (0)
#define KVP_P(KK, SS)                                                                                               \
    do {                                                                                                            \
        if (mode == POW2) KVP_GO(KK, POW2, SS);                                                                     \
        else if (mode == MIXED) KVP_GO(KK, MIXED, SS);                                                              \
        else KVP_GO(KK, SPILL, SS);                                                                                 \
    } while (0)
    if (KB == 1 && sp) KVP_P(1, true);
    else if (KB == 1) KVP_P(1, false);
    else if (KB == 2 && sp) KVP_P(2, true);
    else if (KB == 2) KVP_P(2, false);
    else return 1;
#undef KVP_P
#undef KVP_GO
    KVP_HIP(hipGetLastError());
    ctx->last_kernel = KVP_SCORE_ROWLANE;
    if (mode == SPILL) return kvp_blocksum_from_t_launch(ctx, S, nb_total);
    return KVP_OK;
}
