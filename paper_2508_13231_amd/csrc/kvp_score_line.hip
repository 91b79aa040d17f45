// Scorer for wide rows (n_words >= 32): the schedule rows never touch LDS.
//
//   * A workgroup is eight wavefronts scoring the same 64 token steps of eight or
//     sixteen schedules.  A row is walked in chunks of 32 words = one 128-byte line when
//     rows are line-aligned.  Lane (g, p), g = lane / 8, p = lane % 8, takes the
//     16-byte part p of the chunk for the steps 8g .. 8g+7: eight loads per lane and
//     chunk, each wavefront instruction covering whole lines.  A lane scores its
//     parts straight from registers, the row above being the previous register (for
//     a lane's first step: the last register of the lane eight below, or, in the
//     first group, a ninth load of the step before the tile), and keeps five counters
//     per step until the row ends.
//   * The trace words of a chunk (binary digit planes of the read weights, alive,
//     persist, written) are the same for those schedules: fetched once per
//     workgroup, one chunk ahead, into a double-buffered LDS slot laid out in the
//     order the lanes read it (16 bytes per lane, consecutive lanes consecutive).
//     With sixteen schedules a wavefront scores the chunk for one schedule and then
//     for another from the same slot: the registers that the first one's rows leave
//     are refilled with the second one's, then with the first one's next chunk.
//   * The loop over the chunks has no branch around a load or around the counting: every
//     row vector is requested again, into the same registers, right after its last use.
//     (A branch that skips the counting for chunks without pages made the compiler keep
//     two sets of row registers and copy one to the other at the end of each iteration,
//     which waits for every load in flight: slower than counting zeros.)
//   * At the end of a row the eight lanes of a group add their counters and lane
//     (g, p) keeps step 8g + p: Eqs. 2-4 and the summation tree then run once per
//     layer with one step per lane, as in the other lane-per-step scorers.
//   * The last chunk of a row is shifted left to end at the row's end; the words
//     it shares with the chunk before count nothing: their alive and persist words are
//     zeroed on the way to LDS, and a lane mask takes them out of the chunk's stray bits.
#include "kvp_internal.h"

namespace {

typedef uint32_t l4u __attribute__((ext_vector_type(4), aligned(4)));    // rows may be only 4-byte aligned
typedef uint32_t a4u __attribute__((ext_vector_type(4)));                // LDS vectors are 16-byte aligned

constexpr int LCW = 32;         // words per chunk
constexpr int PLANE = 64 * LCW; // words of one trace array in a slot

__device__ __forceinline__ uint32_t oct_sum(uint32_t v) {               // sum over the 8 lanes of a group
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xf, 0xf, false);    // quad_perm [1,0,3,2]
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xf, 0xf, false);    // quad_perm [2,3,0,1]
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x141, 0xf, 0xf, false);   // row_half_mirror
    return v;
}
// acc += popcount(v) as the one instruction the hardware has for it (left to itself the compiler
// counts into fresh registers and adds them up afterwards)
__device__ __forceinline__ void count(uint32_t &acc, uint32_t v) {
    asm("v_bcnt_u32_b32 %0, %1, %0" : "+v"(acc) : "v"(v));
}

// KB: digit planes of the read weights; POW2: L is a power of two in 2..64; LQ: wavefronts per workgroup,
// 4 or 8 (8 is what the launcher takes); PS: schedules per wavefront, 1 or 2 (a wavefront then scores the chunk for one schedule after the
// other from the same trace slot).  No load is consumed in the iteration that issues it, and all are unconditional.
template <int KB, bool POW2, int LQ, int PS>
__global__ __launch_bounds__(LQ * 64) void score_line_kernel(
    DevProblem q, const uint32_t *__restrict__ Aw, const uint32_t *__restrict__ X, uint32_t s_first, uint32_t S,
    uint32_t tiles, uint32_t nb_total, uint32_t log2L,
    double *__restrict__ blocksum, double *__restrict__ tglobal, uint32_t *__restrict__ tileflag,
    uint32_t *__restrict__ counters, uint32_t *__restrict__ occ_out) {
    extern __shared__ double smem_d[];
    constexpr int NT = KB + 3;                                          // digit planes, alive, persist, written
    constexpr int TV = 8 / LQ;     // vectors of each trace array that a thread moves per chunk (64 rows x 8 parts)
    const uint32_t L = q.L, N = q.N, Wd = q.Wd;
    const uint32_t NCH = (Wd + LCW - 1) / LCW;
    const uint32_t tid = threadIdx.x;
    const int lane = lane_id();
    const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane((int)(tid / KVP_WAVE));
    uint32_t tile, group;                                             // see xcd_pair for the placement
    // the launch scores the schedules [s_first, S) of the batch
    if (!xcd_pair(tiles, (S - s_first + LQ * PS - 1) / (LQ * PS), tile, group)) return;
    const uint32_t s0 = s_first + (group * LQ + wave) * PS;            // the wavefront's schedules: s0 .. s0 + PS - 1
    const uint32_t n0 = tile * 64;
    const uint32_t rows = min(64u, N - n0);
    uint32_t *tbuf = (uint32_t *)smem_d;                               // two slots of NT * PLANE words
    const uint32_t g = (uint32_t)lane >> 3, p = (uint32_t)lane & 7u;

    // the lane's own step
    const bool active = (uint32_t)lane < rows;
    const uint32_t n = n0 + (active ? (uint32_t)lane : rows - 1);      // idle lanes shadow the last row
    const uint32_t wr_n = q.wr[n];
    // The lane's steps are 8g .. 8g+7 of the tile, kept inside the trace: steps past the end repeat the
    // last one, whose trace words the loader repeats too, and are never owned by an active lane.  Step 0
    // is its own predecessor (nothing differs, nothing migrates).
    const int step0 = (int)(n0 + 8 * g) - 1;
    const uint32_t sched_words = L * N * Wd;                           // < 2^31 (checked by the host)
    // trace vectors of this thread: rows tid/8 + 8 LQ v of the tile, part tid%8
    const uint32_t tpart = tid & 7u;
    uint32_t tl[TV], tb[TV], ta[TV];      // LDS word of (row, part): [a][row % 8][row / 8][part][4]; byte offsets in V, Pm, Wm; in the planes
#pragma unroll
    for (int v = 0; v < TV; v++) {
        const uint32_t r = (tid >> 3) + 8 * LQ * v, trow = min(n0 + r, N - 1);
        tl[v] = (((r & 7u) * 8 + (r >> 3)) * 8 + tpart) * 4;
        tb[v] = 4 * (trow * Wd + 4 * tpart);
        ta[v] = 4 * (trow * KB * Wd + 4 * tpart);
    }

    // The nine row vectors of the lane.  Vector j is reloaded for the next iteration as soon as the
    // current one has no more use for it, so one iteration's worth of rows is in flight all the time
    // and nothing needs a second set of registers.
    l4u x[9];
    auto layer_of = [&](uint32_t i) { return POW2 ? (__brev(i) >> (32 - log2L)) : i; };
    auto advance = [&](uint32_t &i, uint32_t &c) __attribute__((always_inline)) {
        if (++c == NCH) { c = 0; if (i + 1 < L) i++; else c = NCH - 1; }   // past the end: stay on the last chunk
    };
    // All addresses are a wavefront-uniform base plus a 32-bit byte offset (the host checks that a
    // schedule and the digit planes stay below 4 GiB).
    const char *Xs[PS];
#pragma unroll
    for (int u = 0; u < PS; u++)                                       // spare places shadow the last schedule
        Xs[u] = (const char *)(X + (size_t)min(s0 + u, S - 1) * sched_words);
    auto x_base = [&](uint32_t i, uint32_t c) { return 4 * (layer_of(i) * N * Wd + min(c * LCW, Wd - LCW) + 4 * p); };
    // Vector j >= 1 is the lane's step 8g + j - 1; vector 0 is the step before the TILE, the same 128 bytes for
    // every lane (one request), which only the first group of lanes uses: the step before the first of any other
    // group is the last step of the group below, taken from those lanes' registers.  (Requested by both groups,
    // an iteration apart, such a row came from memory twice more often than not: the rows are streamed through
    // L2 without being kept.)
    auto issue_x = [&](int j, const char *Xu, uint32_t base, int last_step) __attribute__((always_inline)) {
        const int row = j == 0 ? (int)(n0 ? n0 - 1 : 0) : min(step0 + j, last_step);
        x[j] = KVP_LOAD_X((const l4u *)(Xu + (base + (uint32_t)row * (4 * Wd))));
    };
    l4u tr[TV * NT];
    auto issue_t = [&](uint32_t i, uint32_t c) __attribute__((always_inline)) {
        const uint32_t w0b = 4 * min(c * LCW, Wd - LCW);
        const char *Al = (const char *)Aw + (size_t)layer_of(i) * N * KB * Wd * 4 + w0b;
        const char *Vb = (const char *)q.V + w0b, *Pb = (const char *)q.Pm + w0b, *Wb = (const char *)q.Wm + w0b;
#pragma unroll
        for (int v = 0; v < TV; v++) {
#pragma unroll
            for (int k = 0; k < KB; k++) tr[TV * k + v] = *(const l4u *)(Al + (ta[v] + 4 * k * Wd));
            tr[TV * KB + v] = *(const l4u *)(Vb + tb[v]);
            tr[TV * (KB + 1) + v] = *(const l4u *)(Pb + tb[v]);
            tr[TV * (KB + 2) + v] = *(const l4u *)(Wb + tb[v]);
        }
    };
    // `keep`: all ones, but zero for the words that the row's last chunk shares with the chunk before.  Their alive
    // and persist words go to the slot as zeros, so they count nothing a second time (a thread moves the same part
    // of a chunk as its lane scores: tid % 8 = lane % 8).
    auto commit_t = [&](uint32_t it, a4u keep) __attribute__((always_inline)) {
        uint32_t *slot = tbuf + (it & 1u) * NT * PLANE;
#pragma unroll
        for (int a = 0; a < NT; a++)
#pragma unroll
            for (int v = 0; v < TV; v++) {
                const a4u t = (a4u)tr[TV * a + v];
                *(a4u *)(slot + a * PLANE + tl[v]) = (a == KB || a == KB + 1) ? (t & keep) : t;
            }
    };

    uint32_t fl_acc[PS], occ_acc[PS];
    double total[PS];
#pragma unroll
    for (int u = 0; u < PS; u++) { fl_acc[u] = 0; occ_acc[u] = 0; total[u] = 0.0; }
    // partial sums of the binary counter: touched once per layer, so they live in LDS ([schedule][level][thread])
    double *stk = smem_d + (size_t)NT * PLANE + tid;
    uint32_t it_ = 0, ct = 0;                // iteration whose trace words are requested next
    uint32_t ix = 0, cx = 0;                 // the iteration after the one being scored
    uint32_t it = 0;                         // iterations done: (layer, chunk) pairs in order

    issue_t(it_, ct); advance(it_, ct);
    uint32_t cbase = x_base(0, 0);           // where the chunk being scored starts in a schedule
#pragma unroll
    for (int j = 8; j >= 0; j--) issue_x(j, Xs[0], cbase, (int)N - 1);
    advance(ix, cx);
    commit_t(0, (a4u){~0u, ~0u, ~0u, ~0u});
    for (uint32_t i = 0; i < L; i++) {
        const uint32_t l = layer_of(i);
        const uint32_t acc_n = q.acc[(size_t)l * N + n];               // used when the row ends
        // counters of the steps 8g .. 8g+7 on this layer, this lane's parts only
        uint32_t chr[PS][8][KB], chw[PS][8], coc[PS][8], cmi[PS][8], cmg[PS][8];
#pragma unroll
        for (int u = 0; u < PS; u++)
#pragma unroll
            for (int j = 0; j < 8; j++) {
#pragma unroll
                for (int k = 0; k < KB; k++) chr[u][j][k] = 0;
                chw[u][j] = coc[u][j] = cmi[u][j] = cmg[u][j] = 0;
            }
        for (uint32_t c = 0; c < NCH; c++, it++) {
            const uint32_t w0 = min(c * LCW, Wd - LCW);
            const uint32_t skip = c * LCW - w0;                       // leading words already counted (last chunk only)
            // `kp` is all ones but for those words.  The row vectors themselves are left alone (cleared under a
            // condition, every one of them would be waited for at the top of the iteration; cleared always, that is 36
            // instructions per chunk): the shared words count nothing because their alive and persist words are zero
            // in the slot, and `kp` takes them out of the chunk's stray bits at its end.
            const a4u kp = {4 * p + 0 < skip ? 0u : ~0u, 4 * p + 1 < skip ? 0u : ~0u, 4 * p + 2 < skip ? 0u : ~0u,
                            4 * p + 3 < skip ? 0u : ~0u};
            const uint32_t nbase = x_base(ix, cx);
            advance(ix, cx);
            int last_step = (int)N - 1;
            asm volatile("" : "+s"(last_step));                        // keeps the nine row offsets out of registers
            // This iteration's trace words, requested one iteration ago, go to their slot only now, just before
            // the rows requested during that iteration are needed anyway: loads complete in the order of their
            // issue, and waiting for the trace words at the end of an iteration would also wait for the rows
            // requested last, a memory round trip per chunk.  (Nobody reads the slot before the barrier below,
            // and its last readers have passed the barrier of the iteration before.)
            if (it > 0) commit_t(it, kp);
            issue_t(it_, ct); advance(it_, ct);                        // trace words of the next iteration
            __syncthreads();                                           // this iteration's trace slot is complete
            const uint32_t *slot = tbuf + (it & 1u) * NT * PLANE + 4 * (uint32_t)lane;
            // The trace vectors of step j+1 are requested from LDS before step j is scored, and
            // the scheduler is kept from hoisting them any further: otherwise all eight steps'
            // vectors would be live at once.
            a4u tv[2][NT];
            auto fetch = [&](int j, a4u *dst) __attribute__((always_inline)) {
                const uint32_t *sj = slot + j * 256;               // [row % 8 = j][lane][4]
#pragma unroll
                for (int a = 0; a < NT; a++) dst[a] = *(const a4u *)(sj + a * PLANE);
            };
#pragma unroll
            for (int u = 0; u < PS; u++) {
                // the rows requested while this schedule is scored: the same chunk of the wavefront's next
                // schedule, or the next chunk of its first
                const char *Xn = u + 1 < PS ? Xs[u + 1 < PS ? u + 1 : 0] : Xs[0];
                const uint32_t bn = u + 1 < PS ? cbase : nbase;
                // The steps are taken from the lane's last to its first: the last step's row arrives first and
                // hands its words to the group above right away; the step before the tile is needed last.
                fetch(7, tv[1]);
                a4u fl_e = {0u, 0u, 0u, 0u};                           // stray bits of this chunk, per word of the lane's part
                a4u below;                                             // the last step of the group of lanes below
#pragma unroll
                for (int e = 0; e < 4; e++)
                    below[e] = (uint32_t)__builtin_amdgcn_ds_bpermute(4 * (lane - 8), (int)x[8][e]);
#pragma unroll
                for (int j = 7; j >= 0; j--) {
                    if (j > 0) fetch(j - 1, tv[(j - 1) & 1]);
                    const a4u *cv = tv[j & 1];
                    const a4u before = j > 0 ? (a4u)x[j] : (g == 0 ? (a4u)x[0] : below);
#pragma unroll
                    for (int e = 0; e < 4; e++) {
                        const uint32_t raw = x[j + 1][e], xp = before[e];
                        const uint32_t xx = raw & cv[KB][e];       // alive
                        fl_e[e] |= raw & ~cv[KB][e];
                        const uint32_t d = (xx ^ xp) & cv[KB + 1][e];  // persist
#pragma unroll
                        for (int k = 0; k < KB; k++) count(chr[u][j][k], xx & cv[k][e]);
                        count(chw[u][j], xx & cv[KB + 2][e]);      // written
                        count(coc[u][j], xx);
                        count(cmi[u][j], d & xx);
                        count(cmg[u][j], d);
                    }
                    issue_x(j + 1, Xn, bn, last_step);             // its last use was as this step's own row
                    if (j == 0) issue_x(0, Xn, bn, last_step);
                    __builtin_amdgcn_sched_barrier(0);
                }
                fl_acc[u] |= (fl_e.x & kp.x) | (fl_e.y & kp.y) | (fl_e.z & kp.z) | (fl_e.w & kp.w);
            }
            cbase = nbase;
        }
        // the rows are complete: the group's lanes add up, lane (g, p) keeps step 8g + p
#pragma unroll
        for (int u = 0; u < PS; u++) {
            const uint32_t s = s0 + u;
            const bool has_s = s < S;
            uint32_t hr = 0, hw = 0, oc = 0, mi = 0, mg = 0;
#pragma unroll
            for (int j = 0; j < 8; j++) {
                uint32_t h = 0;
#pragma unroll
                for (int k = 0; k < KB; k++) h += chr[u][j][k] << k;
                h = oct_sum(h);
                const uint32_t w = oct_sum(chw[u][j]), o = oct_sum(coc[u][j]), m1 = oct_sum(cmi[u][j]), m2 = oct_sum(cmg[u][j]);
                const bool mine = p == (uint32_t)j;
                hr = mine ? h : hr; hw = mine ? w : hw; oc = mine ? o : oc; mi = mine ? m1 : mi; mg = mine ? m2 : mg;
                __builtin_amdgcn_sched_barrier(0);                     // one step at a time: few temporaries
            }
            const uint32_t mo = mg - mi;
            double t = step_time(q, hr, hw, mi, mo, acc_n, wr_n);      // Eqs. 2-4
            t = active ? t : 0.0;                                      // rows past the end of the trace pad with +0.0
            occ_acc[u] += oc;
            if (counters && has_s && active)
                *(uint4 *)(counters + (((size_t)s * L + l) * N + n) * 4) = make_uint4(hr, hw, mi, mo);
            if (POW2) {
                // folds of the summation tree that join the steps of one block (lanes)
                for (uint32_t m = (64u >> log2L) >> 1; m >= 1; m >>= 1) t = fold_xor_f64(t, m);
                // folds that join layers: binary counter over the bit-reversed visiting order
                double *su = stk + (size_t)u * 6 * LQ * 64;
                double carry = t;
                bool parked = false;
#pragma unroll
                for (int j = 0; j < 6; j++) {
                    if (!parked && (uint32_t)j < log2L) {
                        if (((i >> j) & 1u) == 0) { su[j * LQ * 64] = carry; parked = true; }
                        else carry = su[j * LQ * 64] + carry;
                    }
                }
                if (!parked) total[u] = carry;                         // only at the last layer
            } else if (has_s && active) {
                tglobal[((size_t)s * L + l) * N + n] = t;
            }
        }
    }
#pragma unroll
    for (int u = 0; u < PS; u++) {
        const uint32_t s = s0 + u;
        // (every lane takes part in the two reductions; only the stores depend on the schedule being there)
        uint32_t ex = 0;
        if (active) ex = occ_acc[u] > q.cap ? occ_acc[u] - q.cap : 0;
        ex = wave_max_u32(ex);
        const uint32_t fl = wave_or_u32(fl_acc[u]);
        if (s >= S) continue;
        if (POW2) {
            const uint32_t bpl = 64u >> log2L;                         // block b of the tile: steps [b*bpl, (b+1)*bpl)
            if (((uint32_t)lane & (bpl - 1)) == 0 && (uint32_t)lane < rows)
                blocksum[(size_t)s * nb_total + (size_t)tile * L + (uint32_t)lane / bpl] = total[u];
        }
        if (active && occ_out) occ_out[(size_t)s * N + n] = occ_acc[u];   // Eq. 5 per token step
        if (lane == 0) tileflag[(size_t)s * tiles + tile] = ex | (fl ? 0x80000000u : 0u);
    }
}

}  // namespace

int kvp_blocksum_from_t_launch(kvp_ctx *ctx, uint32_t S, uint32_t nb_total);

namespace {

template <int LQ, int PS>
int launch_line(kvp_ctx *ctx, const uint32_t *X, uint32_t s_first, uint32_t S, uint32_t tiles, uint32_t nb_total, uint32_t log2L,
                bool pow2, uint32_t *counters, uint32_t *occ) {
    const DevProblem &q = ctx->dp;
    const uint32_t KB = ctx->kb;
    const size_t lds = 2 * (size_t)(KB + 3) * PLANE * 4 + (pow2 ? (size_t)6 * LQ * PS * 64 * 8 : 0);
    if (lds > 160 * 1024) return 1;
    const uint64_t nwg = xcd_grid(tiles, (S - s_first + LQ * PS - 1) / (LQ * PS));
    if (nwg > 0x7FFFFFFFull) return 1;
    dim3 grid((uint32_t)nwg), block(LQ * 64);
#define KVP_GO(KK, PP)                                                                                         \
    do {                                                                                                       \
        KVP_HIP(hipFuncSetAttribute((const void *)score_line_kernel<KK, PP, LQ, PS>,                             \
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));                   \
        score_line_kernel<KK, PP, LQ, PS><<<grid, block, lds, ctx->stream>>>(                                 \
            q, ctx->aw, X, s_first, S, tiles, nb_total, log2L, ctx->d_blocksum,                                        \
            ctx->d_tglobal, ctx->d_tileflag, counters, occ);                                                   \
    } while (0)
#define KVP_K(KK) case KK: if (pow2) KVP_GO(KK, true); else KVP_GO(KK, false); break;
    if constexpr (PS == 2) {                                           // registers: one digit plane only
        switch (KB) {
            KVP_K(1)
            default: return 1;
        }
    } else {
        switch (KB) {
            KVP_K(1) KVP_K(2) KVP_K(3) KVP_K(4)
            default: return 1;
        }
    }
#undef KVP_K
#undef KVP_GO
    KVP_HIP(hipGetLastError());
    return KVP_OK;
}

}  // namespace

// Returns KVP_OK if launched, 1 if this kernel does not cover the shape, <0 on error.
int kvp_score_line_launch(kvp_ctx *ctx, const uint32_t *X, uint32_t S, uint32_t tiles, uint32_t nb_total,
                          uint32_t *counters, uint32_t *occ) {
    const DevProblem &q = ctx->dp;
    if (!ctx->aw || q.Wd < LCW) return 1;
    const uint32_t KB = ctx->kb;
    if (KB > 4) return 1;                                             // registers: five counters per step and digit
    if ((size_t)q.L * q.N * q.Wd * KB >= (1ull << 30)) return 1;      // 32-bit byte offsets inside a schedule and the planes
    uint32_t log2L = 0;
    while ((1u << log2L) < q.L) log2L++;
    const bool pow2 = q.L >= 2 && q.L <= 64 && (1u << log2L) == q.L;
    if (!pow2) {
        int rc = kvp_ensure(ctx, (void **)&ctx->d_tglobal, &ctx->tglobal_cap, (size_t)S * q.L * q.N * sizeof(double));
        if (rc) return rc;
    }
    // The more schedules share each fetch of the trace, the fewer trace bytes cross from L2 to the compute
    // units (as many as schedule bytes with four schedules per workgroup, which ran at 0.69 of the memory's
    // peak): a workgroup is eight wavefronts, one workgroup per compute unit (0.80), and with one digit plane
    // (registers) a wavefront may take two schedules (0.85).  A workgroup then takes twice as long, and a launch
    // is over when its last round of workgroups is, however few they are.  So the schedules that fill whole
    // rounds of workgroups of sixteen go first, and the rest follow in workgroups of eight; a batch that does
    // not fill one such round takes sixteen only if rounds x group / rate is no larger that way.
    const uint64_t cus = ctx->compute_units;
    auto estimate = [&](uint32_t group, double rate) {
        const uint64_t wgs = (uint64_t)((S + group - 1) / group) * tiles;
        return (double)((wgs + cus - 1) / cus) * group / rate;
    };
    int rc;
    if (KB != 1) {
        rc = launch_line<8, 1>(ctx, X, 0, S, tiles, nb_total, log2L, pow2, counters, occ);
    } else {
        const uint64_t rounds = (uint64_t)(S / 16) * tiles / cus;      // whole rounds of workgroups of sixteen
        uint64_t groups = rounds * cus / tiles;
        uint32_t s_two = groups * 16 > S ? S : (uint32_t)(groups * 16);
        if (rounds == 0) s_two = estimate(16, 0.85) <= estimate(8, 0.80) ? S : 0;
        rc = s_two ? launch_line<8, 2>(ctx, X, 0, s_two, tiles, nb_total, log2L, pow2, counters, occ) : KVP_OK;
        if (!rc && s_two < S) rc = launch_line<8, 1>(ctx, X, s_two, S, tiles, nb_total, log2L, pow2, counters, occ);
    }
    if (rc) return rc;
    ctx->last_kernel = KVP_SCORE_LINE;
    if (!pow2) return kvp_blocksum_from_t_launch(ctx, S, nb_total);
    return KVP_OK;
}
