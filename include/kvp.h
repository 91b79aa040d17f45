/*
 * kvp.h -- C boundary of the MI355X KV-cache placement scorer and annealer.
 *
 * The library searches for the upper-bound dynamic placement of KV-cache pages
 * across HBM and off-package DRAM of "Accelerating LLM Inference via Dynamic KV
 * Cache Placement in Heterogeneous Memory System" (Sec. III).  A placement
 * schedule says, for every inference step (n, l) and every page, whether the
 * page sits in HBM while the step runs; its cost is the total decode latency of
 * Eqs. 1-4 and it is admissible when it respects the HBM capacity (Eq. 5).
 *
 * Conventions
 *   - Every function returns KVP_OK (0) or a negative KVP_E* code; nothing
 *     aborts, throws or prints.  kvp_strerror names a code.
 *   - Pointers named d_* are DEVICE memory on the context's GPU, allocated and
 *     owned by the caller, 16-byte aligned.  Pointers named h_* are HOST memory.
 *     The library copies what it keeps and retains no caller pointer.
 *   - kvp_score, kvp_delta_score, kvp_anneal, kvp_baseline, kvp_strict_excess
 *     and kvp_exchange (without a count) enqueue their work on the HIP stream
 *     given to kvp_create and return without waiting (they may allocate
 *     internal buffers first).  kvp_trace_upload, kvp_best, kvp_temper,
 *     kvp_chain_placement and kvp_chain_stats wait for the stream.
 *   - Bit masks: uint32 words, bit b of word w is page 32*w + b; bits at or
 *     above n_pages are zero.  A schedule is [n_layers][n_steps][n_words]
 *     words; a batch of S schedules is S of those back to back.
 *   - One context serves one host thread at a time.
 */
#ifndef KVP_H
#define KVP_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct kvp_ctx kvp_ctx;

enum {
    KVP_OK = 0,
    KVP_EINVAL = -1,      /* null pointer, misaligned pointer, value out of range        */
    KVP_ENOTRACE = -2,    /* no trace uploaded yet                                        */
    KVP_ENOMEM = -3,      /* device or host allocation failed                             */
    KVP_EHIP = -4,        /* a HIP call failed                                            */
    KVP_ESHAPE = -5,      /* sizes inconsistent with each other or beyond what is built   */
    KVP_ETRACE = -6,      /* trace masks contradict each other (see kvp_trace_upload)     */
    KVP_ENOCHAINS = -7,   /* no annealing state to continue or to read                    */
    KVP_EINFEASIBLE = -8  /* a starting schedule exceeds the HBM capacity                 */
};

#define KVP_MAX_PLANES 8
#define KVP_MAX_LEN 63     /* longest span of a move: its window fits one 64-lane wavefront */

/* The placement problem (Sec. III-A): access sets per step come with the trace;
 * this holds sizes, data volumes, the three bandwidths of Eqs. 3-4 and the
 * capacity of Eq. 5. */
typedef struct {
    uint32_t n_layers;    /* L: transformer layers                                        */
    uint32_t n_steps;     /* N: decode tokens; inference step (n,l) runs in order n*L+l   */
    uint32_t n_pages;     /* P: page slots per layer                                      */
    uint32_t n_words;     /* must equal ceil(P/32)                                        */
    uint32_t n_planes;    /* K in 1..8: access sets per step (e.g. one per KV head)       */
    uint32_t reserved;    /* 0                                                            */
    uint64_t plane_bytes[KVP_MAX_PLANES]; /* bytes read per accessed page of plane k, >0  */
    uint64_t page_bytes;  /* bytes moved when a page changes tier (|M^i|, |M^o| unit)     */
    uint64_t token_bytes; /* bytes of new KV written per written page and layer (H^w,E^w) */
    double bw_hbm;        /* B_h, bytes/s, finite and > 0                                 */
    double bw_link;       /* B_k, one direction of the full-duplex link                   */
    double bw_dram;       /* B_d, off-package DRAM channels                               */
    uint64_t cap_pages;   /* HBM pool in pages, shared by all layers (Eq. 5)              */
} kvp_problem;

/* A raw move on a schedule (before clipping to the capacity).  The move set is
 * this library's own; Sec. III-B of the paper fixes only the Metropolis rule,
 * the three-operator mixture and the cooling constants.
 *   op 0 SET    give the bit of (layer, page) the value opposite to the one it
 *               has at step n1, on steps n1 .. n1+len-1 (while the page lives)
 *   op 1 SWAP   as SET towards HBM, evicting (layer2, page2) on full steps
 *   op 2 SHIFT  move the first 0/1 edge of the page's timeline after n1 by
 *               {-2,-1,+1,+2}[dsel & 3] steps
 * A record with a field out of range (len outside 1..KVP_MAX_LEN) is a null move. */
typedef struct {
    uint32_t op, layer, page, n1, len, layer2, page2, dsel;
} kvp_move;

enum { KVP_OP_SET = 0, KVP_OP_SWAP = 1, KVP_OP_SHIFT = 2 };
enum { KVP_MOVE_OK = 0, KVP_MOVE_CLIPPED = 1, KVP_MOVE_NULL = 2 };

enum {
    KVP_INIT_EMPTY = 0,     /* every chain starts with nothing in HBM                     */
    KVP_INIT_GIVEN = 1,     /* start from d_init: one schedule per chain                  */
    KVP_INIT_BROADCAST = 2, /* start every chain from the single schedule d_init          */
    KVP_INIT_CONTINUE = 3   /* carry on the chains of the previous call                   */
};

/* Simulated annealing (Sec. III-B): Metropolis acceptance exp(-dT/C), initial
 * temperature from the target acceptance p0 of uphill moves, geometric cooling
 * by alpha over n_levels levels of equal length, fixed move budget. */
typedef struct {
    uint32_t n_chains;     /* independent chains (one to four wavefronts each)            */
    uint32_t n_levels;     /* temperature levels (>= 1), e.g. 100                          */
    uint64_t seed;         /* Philox4x32-10 key; the chain id is part of the counter      */
    uint64_t total_moves;  /* length of the whole cooling schedule, per chain             */
    uint64_t moves;        /* moves to run in this call, per chain (proposals, incl. null) */
    uint32_t max_len;      /* longest span, 1..KVP_MAX_LEN                                 */
    uint32_t init_mode;    /* KVP_INIT_*                                                   */
    double p0;             /* 0 < p0 < 1, the paper uses 0.8                               */
    double alpha;          /* 0 < alpha <= 1, the paper uses 0.9                           */
    double op_prob[3];     /* SET, SWAP, SHIFT; the paper's mixture is 0.4, 0.4, 0.2       */
} kvp_anneal_params;

typedef struct {
    double t_cur;          /* running cost of the current schedule (start + accepted dT)  */
    double t_best;         /* lowest running cost seen                                    */
    double c0, c;          /* initial and current temperature                             */
    uint64_t moves_done, accepted, uphill, null_moves, clipped, improved;
} kvp_chain_stats_t;

/* Create a context on GPU `device` whose work runs on `hip_stream` (a
 * hipStream_t, may be NULL for the default stream).  The caller keeps the
 * stream alive until kvp_destroy.  Errors: KVP_EINVAL, KVP_EHIP, KVP_ENOMEM. */
int kvp_create(kvp_ctx **out, int device, void *hip_stream);

/* Wait for the stream, free everything the context owns.  NULL is allowed. */
void kvp_destroy(kvp_ctx *ctx);

/* Sec. III-B (access patterns known a priori) and Sec. IV-A (recorded per
 * layer): hand over the access trace.  All four arrays are HOST memory:
 *   h_access  [L][N][K][Wd]  pages read by plane k at step (n,l)
 *   h_alive   [N][Wd]        pages that hold KV data while token step n runs
 *   h_persist [N][Wd]        pages holding the same data as at step n-1
 *   h_written [N][Wd]        pages that receive the token generated at step n
 * Required (else KVP_ETRACE): access and written inside alive; persist[n]
 * inside alive[n] and alive[n-1]; persist[0] empty; no bit at or above P.
 * KVP_ESHAPE if n_words != ceil(P/32), a dimension is 0, or a byte total could
 * reach 2^53; KVP_EINVAL for null pointers, non-finite or non-positive
 * bandwidths, K outside 1..8.  Copies everything to the GPU (replacing any
 * earlier trace and discarding annealing state) and waits for the copy. */
int kvp_trace_upload(kvp_ctx *ctx, const kvp_problem *problem, const uint32_t *h_access,
                     const uint32_t *h_alive, const uint32_t *h_persist, const uint32_t *h_written);

/* Eqs. 1-5: score S schedules at once.
 *   d_placements [S][L][N][Wd]  in
 *   d_cost       [S]            total latency T in seconds (Eq. 1: steps summed in
 *                               execution order by the fixed 64-wide tree)
 *   d_excess     [S]            largest overshoot of cap_pages over all token steps
 *                               (0 = admissible, Eq. 5); bit 31 set if the schedule
 *                               had bits on pages that do not exist (those are ignored)
 *   d_counters   [S][L][N][4]   nullable: per step {units read from HBM, written pages
 *                               in HBM, pages migrated in, pages migrated out}; one
 *                               read unit is kvp_plane_unit() bytes
 *   d_occ        [S][N]         nullable: pages in HBM per token step
 * An inadmissible schedule is not an error.  S = 0 is a no-op.  */
int kvp_score(kvp_ctx *ctx, const uint32_t *d_placements, uint32_t S, double *d_cost,
              uint32_t *d_excess, uint32_t *d_counters, uint32_t *d_occ);

/* kvp_score for callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments and results as kvp_score with
 * d_counters = d_occ = NULL, bit for bit, and the same kernels; what kvp_score keeps in buffers
 * that it allocates and grows (the partial sums of Eq. 1 per block of 64 inference steps, the
 * capacity verdict of every tile of token steps, and, for layer counts that are not 2^k or
 * 2^k * {3, 5, 7}, the step latencies) lives here in a static device array of
 * KVP_STATIC_SCRATCH_BYTES that every GPU on which the library is used holds until the process
 * ends.  The call makes no hipMalloc, hipFree or other allocating call.
 *   d_placements [S][L][N][Wd]  in, DEVICE, caller-owned, 16-byte aligned
 *   d_cost [S], d_excess [S]    out, DEVICE, caller-owned
 * Errors: as kvp_score, and KVP_ESHAPE when the batch needs more scratch than the array holds:
 * S * (ceil(L*N/64) * 8 + N * 4) bytes, each of the two terms rounded up to 256, must not exceed
 * KVP_STATIC_SCRATCH_BYTES (plus S*L*N*8 for the layer counts named above).  Nothing is launched
 * then.  All calls on one GPU share the one array, whatever their context: two such calls that
 * overlap in time on a GPU (different streams or threads) race; calls on one stream do not.
 * Nothing in the array needs to start at zero: every word that a launch reads it has written. */
#define KVP_STATIC_SCRATCH_BYTES (32u << 20)
int kvp_score_static(kvp_ctx *ctx, const uint32_t *d_placements, uint32_t S, double *d_cost,
                     uint32_t *d_excess);

/* Sec. III-B, dT = T_new - T_current of one proposed move per schedule, summed
 * over the 64-step window the move can touch, without re-scoring the rest.
 *   d_moves    [S]  raw moves
 *   d_counters, d_occ  as written by kvp_score for the same schedules; if either
 *                   is NULL the library computes both first (one scoring pass)
 *   d_delta    [S]  dT in seconds (0 for a null move)
 *   d_verdict  [S]  KVP_MOVE_OK, _CLIPPED (shortened by the capacity) or _NULL
 * Schedules must be admissible for the clipping to mean anything. */
int kvp_delta_score(kvp_ctx *ctx, const uint32_t *d_placements, uint32_t S, const kvp_move *d_moves,
                    const uint32_t *d_counters, const uint32_t *d_occ, double *d_delta,
                    int32_t *d_verdict);

/* Eq. 5 counted slot by slot.  kvp_score checks the capacity once per token step; here the layers of
 * a step change their placement one after the other, each at its own slot (n, l), so after slot
 * (n, l) the pool holds the step-n placement of layers 0..l and still the step-(n-1) placement of
 * the layers to come (less the pages that do not persist into step n).
 *   d_placements [S][L][N][Wd]  in (bits on pages that do not exist are ignored)
 *   d_excess     [S]            largest overshoot of cap_pages over all slots; never less than the
 *                               excess kvp_score reports, equal to it for a schedule that never migrates
 * Runs on the context's stream.  S = 0 is a no-op.  Errors: KVP_EINVAL (null or misaligned pointer),
 * KVP_ENOTRACE, KVP_ESHAPE (more than 2048 layers), KVP_EHIP. */
int kvp_strict_excess(kvp_ctx *ctx, const uint32_t *d_placements, uint32_t S, uint32_t *d_excess);

/* Sec. III-A: the placement decision at an inference step covers all KV data, so a page may change tier in
 * another layer's step and its bytes are charged there.  A schedule is then a placement X as above and
 * a second plane Y of bytes: a page (l, p) whose placement differs between its steps n-1 and n, and which
 * persists into n, migrates in the inference step
 *     g = n*L + l - Y[l][n][p],   Y in 0 .. L-1
 * (any step after its use at (n-1, l) up to its use at (n, l)); Y is not looked at elsewhere, and Y = 0
 * everywhere is the schedule that kvp_score prices.  Reads and the new token's write are those of X.
 *
 * kvp_score_slots: Eqs. 1-4 with |M^i|, |M^o| counted in the step where the pages move, and Eq. 5 after
 * every inference step (pages born in HBM enter the pool in their own step, pages that do not persist
 * leave it at the start of the token step).
 *   d_placements [S][L][N][Wd]  in, DEVICE, 16-byte aligned
 *   d_slots      [S][L][N][P]   in, DEVICE, one byte per page (P = n_pages)
 *   d_cost       [S]            out: T in seconds, summed in execution order by the tree of kvp_score
 *   d_excess     [S]            out: largest overshoot of cap_pages over all inference steps; bit 31: bits
 *                               on pages that do not exist; bit 30: a Y above L-1 on a migrating page
 *                               (taken as 0)
 * Runs on the context's stream; scratch of S*L*N*36 bytes is held by the context.  S = 0 is a no-op.
 * Errors: KVP_EINVAL (null or misaligned pointer), KVP_ENOTRACE, KVP_ESHAPE (more than 256 layers or 65535 schedules),
 * KVP_ENOMEM, KVP_EHIP.
 *
 * kvp_refine_slots: annealing over Y for ONE fixed placement (the Metropolis rule, start temperature
 * and cooling of Sec. III-B; the move is this library's): params->n_chains chains.  The M pages that
 * migrate are listed once in the order (layer, step, page).  Chain c draws proposal i from the Philox
 * block (i lo, i hi, c, 32) under params->seed (stream 40 for the 256 calibration proposals): word 0
 * picks the list entry (high word of word 0 x M), word 1 the new Y (high word of word 1 x L), words 2
 * and 3 the 52 bits of the acceptance draw.  Null if Y stays (or nothing migrates); dropped (counted
 * as null and as clipped) if the page would be in the pool during a step that is full; dT = the
 * change of the old step's latency + that of the new step's.  Runs moves [0, params->moves) of a
 * cooling schedule of params->total_moves; max_len and op_prob are not used; init_mode
 * KVP_INIT_EMPTY (every chain starts from Y = 0, written by the call) or KVP_INIT_GIVEN (from d_slots).
 *   d_placement  [L][N][Wd]      in, DEVICE, 16-byte aligned
 *   d_slots      [C][L][N][P]    in (GIVEN) / out, DEVICE: every chain's final Y
 *   h_stats      [C]             out, HOST, may be NULL: t_cur is the start's cost plus the accepted dT
 * The call waits for the stream.  Errors: KVP_EINVAL, KVP_ENOTRACE, KVP_ESHAPE, KVP_EINFEASIBLE (a start that
 * overfills an inference step or holds a Y out of range), KVP_ENOMEM, KVP_EHIP. */
int kvp_score_slots(kvp_ctx *ctx, const uint32_t *d_placements, const uint8_t *d_slots, uint32_t S, double *d_cost,
                    uint32_t *d_excess);
int kvp_refine_slots(kvp_ctx *ctx, const kvp_anneal_params *params, const uint32_t *d_placement, uint8_t *d_slots,
                     kvp_chain_stats_t *h_stats);

/* Parallel tempering across the chains of kvp_anneal: an extension, not in the paper, whose search
 * (Sec. III-B) is one annealing run; the exchange step is the standard one (Swendsen & Wang 1986,
 * Geyer 1991).  Used between slices of kvp_anneal (KVP_INIT_CONTINUE):
 *
 * kvp_temper multiplies the temperature of chain c (the current one and the initial one that
 * kvp_chain_stats reports) by h_factor[c], e.g. a geometric ladder; every chain goes on cooling by
 * alpha per level from what it holds.
 *   h_factor   host, [n_chains] doubles, finite and > 0; free again on return
 * Errors: KVP_EINVAL (null pointer, a factor that is not positive and finite, or no move made yet:
 * the slice that begins at move 0 sets the initial temperatures), KVP_ENOCHAINS, KVP_ENOMEM, KVP_EHIP.
 *
 * kvp_exchange lets neighbouring chains trade their temperatures: in round r the pairs (a, a+1),
 * a = r mod 2, r mod 2 + 2, ..., trade with probability min(1, exp((1/C_a - 1/C_b)(T_a - T_b))),
 * T the chain's current cost and C its temperature, so the better schedule tends to the lower
 * temperature.  One uniform number per pair: Philox4x32-10 with the seed of kvp_anneal as key and
 * counter (round lo, round hi, a, 16), mapped to (0,1) like the acceptance draw of a move.  Pairs
 * with a temperature that is not positive are left alone.
 *   round      any number; its parity picks the pairs, callers count it up
 *   h_traded   host, may be null: receives the number of pairs that traded (the call then waits
 *              for the stream; otherwise it only enqueues)
 * Errors: KVP_EINVAL (null ctx), KVP_ENOCHAINS, KVP_EHIP. */
int kvp_temper(kvp_ctx *ctx, const double *h_factor);
int kvp_exchange(kvp_ctx *ctx, uint64_t round, uint32_t *h_traded);

/* Tuning knob of kvp_anneal: how many consecutive proposals of a chain are priced at once, each
 * by a wavefront of its own (the walk takes them in order up to the first accepted one, so it is
 * the same walk whatever the number).  0 (default): chosen from the number of chains and the
 * size of the GPU; 1: one wavefront per chain prices one proposal after the other; 4: four per
 * round (traces of more than 12288 token steps are always walked the first way).  Other values:
 * KVP_EINVAL. */
int kvp_set_anneal_lookahead(kvp_ctx *ctx, int proposals_per_round);

/* Tuning knob of the placement generators (KVP_BASELINE_RECENCY, kvp_wr_policy, kvp_wr_search): they
 * work through the token steps in batches whose per-step keys, window counts and wanted sets fit this
 * many bytes of scratch (one step at least).  0 (default): one gigabyte (recency), two (policy).  The
 * results do not depend on it.  Errors: KVP_EINVAL (null ctx). */
int kvp_set_generator_batch_bytes(kvp_ctx *ctx, uint64_t bytes);

/* Tuning knob of kvp_anneal, read by its next fresh start: the number of logged edits after which a
 * chain writes its best schedule out and starts its log afresh (launches are cut to that many moves
 * per chain).  0 (default): chosen from the sizes, see kvp_anneal; a value of total_moves or more: the
 * log is not bounded.  The walk and its results do not depend on it.  Errors: KVP_EINVAL (null ctx). */
int kvp_set_anneal_log_entries(kvp_ctx *ctx, uint64_t entries);

/* Which reading of Eq. 5 the walks of kvp_anneal honour (Sec. III-A: a decision S(n, l) is made at
 * every inference step, layer l of token step n).
 *   KVP_CAPACITY_PER_STEP (default)  the pool is counted once per token step, when all layers have
 *       taken their placement of that step: what kvp_score's excess reports.
 *   KVP_CAPACITY_PER_SLOT            the pool is counted after every inference step: what
 *       kvp_strict_excess reports.  A move sets the bit of (l, p) at step n only if no slot
 *       (n, l' >= l) and, when the page persists into n + 1, no slot (n + 1, l' < l) (where layer l
 *       still holds its placement of step n) would exceed cap_pages; a SWAP's victim (l2, q) counts
 *       as gone from the slots (n, l' >= l2) and, if it persists, (n + 1, l' < l2).  Every step of a
 *       move is judged against the schedule before the move.  Starting schedules must fit every
 *       slot (KVP_EINFEASIBLE); every schedule the walk visits then does.  One wavefront per chain
 *       prices one proposal after the other (the lookahead knob is not used); per chain L*N*4
 *       more bytes of device memory.
 * The mode is read by the next fresh start of kvp_anneal; KVP_INIT_CONTINUE under another mode than
 * the chains were started with is KVP_EINVAL.  kvp_delta_score always clips per token step.
 * Errors: KVP_EINVAL (null ctx, unknown mode). */
enum { KVP_CAPACITY_PER_STEP = 0, KVP_CAPACITY_PER_SLOT = 1 };
int kvp_set_capacity_mode(kvp_ctx *ctx, int mode);

/* Sec. III-B: run params->moves annealing moves on every chain.  d_init is
 * [C][L][N][Wd] (KVP_INIT_GIVEN), [L][N][Wd] (KVP_INIT_BROADCAST) or NULL.
 * Starting schedules must be admissible (checked, KVP_EINFEASIBLE) and are
 * masked to existing pages.  KVP_INIT_CONTINUE needs the parameters of the
 * previous call except `moves` (else KVP_EINVAL; KVP_ENOCHAINS if none).
 * moves beyond what is left of total_moves: KVP_EINVAL, and the chains of an
 * earlier call stay as they are.  More than 65535 chains: KVP_ESHAPE.
 * Device memory per chain, held until the next trace or the next fresh start:
 * the schedule (L*N*Wd*4 bytes), its step counters (L*N*16), occupancy (N*4)
 * and the log of accepted edits since the chain's best schedule (40 bytes an
 * entry, one entry per move at most): total_moves entries, or, where that is
 * more than twice what a schedule takes, 2 * max(16384, schedule bytes / 40)
 * entries and one more schedule: a chain whose log has passed half of that
 * writes its best schedule out between two launches and starts its log afresh
 * (kvp_set_anneal_log_entries sets the half). */
int kvp_anneal(kvp_ctx *ctx, const kvp_anneal_params *params, const uint32_t *d_init);

/* Sec. III-B (the search returns the schedule of the best latency found).
 * Best schedule over all chains: each chain's best-so-far schedule is scored
 * again in full (never the running value), the lowest cost wins, ties go to the
 * lowest chain id.  h_placement [L][N][Wd] and h_chain_costs [C] are nullable.
 * Outputs are written on success only (h_placement and h_chain_costs may be
 * partly written when a copy fails). */
int kvp_best(kvp_ctx *ctx, double *h_cost, uint32_t *h_chain, uint32_t *h_placement,
             double *h_chain_costs);

/* Copy one chain's current (best = 0) or best-so-far (best = 1) schedule out. */
int kvp_chain_placement(kvp_ctx *ctx, uint32_t chain, int best, uint32_t *h_placement);

/* Per-chain counters, h_stats [C]. */
int kvp_chain_stats(kvp_ctx *ctx, kvp_chain_stats_t *h_stats);

/* Bytes per read unit of d_counters (gcd of plane_bytes); 0 without a trace. */
uint64_t kvp_plane_unit(const kvp_ctx *ctx);

/* Tuning knob: which scoring kernel kvp_score uses.  AUTO picks by the shape of the rows and of the
 * trace; a forced scorer that does not cover the shape is replaced by the next one that does.
 * Results are identical bit for bit whichever runs.  Values that name no scorer: KVP_EINVAL. */
enum { KVP_SCORE_AUTO = 0,
       KVP_SCORE_ROWS = 1,      /* any shape: a wavefront per (layer, step) row, lanes across words */
       KVP_SCORE_LANES = 2,     /* rows of <= 16 words: a lane per row, rows staged through LDS */
       KVP_SCORE_QUAD = 6,      /* rows of <= 15 words, one plane, 2^k layers: a lane per row, four
                                   schedules per workgroup share the trace chunk */
       KVP_SCORE_CHUNK = 9,     /* rows of >= 16 words, any masks: a lane per row, rows walked in chunks of
                                   16 words */
       KVP_SCORE_ROWBLOCK = 10, /* one decoding sequence, rows of 16..68 words: two lanes per row, whole rows
                                   staged at once, read weights as binary digit planes */
       KVP_SCORE_LINE = 11,     /* rows of >= 32 words, any masks: 128-byte chunks scored from registers,
                                   eight lanes per chunk (several sequences) */
       KVP_SCORE_ROWSEG = 12,   /* ROWBLOCK's scheme for rows of more than 68 words, walked in equal
                                   segments of 40..64 words */
       KVP_SCORE_ROWLANE = 13   /* one decoding sequence, rows of 29..36 words, one or two dense digit planes
                                   (further ones almost empty): a lane per step, a layer of a tile per pass */ };
int kvp_set_score_kernel(kvp_ctx *ctx, int which);

/* The scorer that the last kvp_score on ctx ran (a KVP_SCORE_* value other than
 * AUTO), 0 before the first call or for a null ctx.  A forced scorer that does
 * not cover the trace's shape is replaced by one that does: this tells which. */
int kvp_score_kernel_used(const kvp_ctx *ctx);

/* Three placements that need no search, to start one from or to compare it with
 * (the evaluation section of the paper sets its search against a static and a
 * reactive least-recently-used placement; these are their counterparts on this
 * problem's terms: a pool of cap_pages shared by the layers, whole pages, no
 * migration cost model of their own).
 *   KVP_BASELINE_STATIC:  the cap_pages (layer, page) pairs read most often over
 *     the whole trace (accesses summed over the planes) are in HBM at every step
 *     at which they exist; nothing ever migrates.
 *   KVP_BASELINE_RECENCY: at step n the pool holds the cap_pages existing pairs
 *     read most recently before n (never read: oldest); a page that stops
 *     persisting forgets its history.
 *   KVP_BASELINE_FILL:    the paper's "Static Placement": an entry is placed when
 *     it is first written and never moves, HBM first while there is room.  Step
 *     by step, pages that stop persisting give their place back, then the pages
 *     new at this step take the free places in the order of l * n_pages + p
 *     (layer after layer, as a prefill writes them); the rest stay outside for
 *     as long as they live.
 * Ties go to the lower l * n_pages + p in the first two.  d_placement: DEVICE, one
 * schedule [L][N][Wd] uint32, written in full; the caller owns it.  The result
 * never exceeds the capacity.  Runs on the context's stream.
 * Errors: KVP_EINVAL (null or misaligned pointer, unknown kind), KVP_ENOTRACE,
 * KVP_ESHAPE (STATIC, RECENCY: more than 32767 steps, or steps x planes above
 * 32767, for the histogram of the selection), KVP_ENOMEM, KVP_EHIP. */
enum { KVP_BASELINE_STATIC = 0, KVP_BASELINE_RECENCY = 1, KVP_BASELINE_FILL = 2 };
int kvp_baseline(kvp_ctx *ctx, int kind, uint32_t *d_placement);

/* ---- the paper's own search: a look-ahead policy with two scalars (Sec. III-B) ----
 * W >= 1: token steps looked ahead; R = r10 / 10, r10 in 0..10: share of the pages
 * qualified for migration that migrate.  The policy, once per token step n on the
 * pool of cap_pages shared by the layers (the paper states it in two sentences;
 * this is the reading taken, the same as the oracle's):
 *   1. pages that do not persist into n leave the pool;
 *   2. the existing pages read in steps n .. n+W-1 are collected with their read
 *      frequency f there (summed over the planes);
 *   3. ranked by f descending, ties to the lower l * n_pages + p; the first
 *      cap_pages of the ranking are wanted;
 *   4. wanted pages outside the pool are qualified; the first
 *      (r10 * their number + 5) div 10 of them, in rank order, come in;
 *   5. if the pool would overflow, as many unwanted pool pages leave, smallest f
 *      first, ties to the lower l * n_pages + p;
 *   6. the pool is the placement of step n in every layer.
 *
 * kvp_wr_policy: n candidates (h_w[i], h_r10[i]), HOST arrays, read before the
 * call returns; d_placements: DEVICE [n][L][N][Wd] uint32, written in full, owned
 * by the caller.  Steps 2 and 3 are computed once per distinct W, for all token
 * steps of a batch at once; steps 1 and 4 to 6 by one workgroup per candidate.  W
 * above n_steps acts as n_steps.  Scratch held by the context: up to 2 GiB for the
 * window counts and wanted sets of a batch of steps (at least one step's:
 * distinct W x L x Wd x (32 x count bytes + 4)), plus n x L x Wd x 4 bytes.
 * Errors: KVP_EINVAL (null pointer, W = 0, r10 > 10), KVP_ENOTRACE, KVP_ESHAPE
 * (W x planes above 16383), KVP_ENOMEM, KVP_EHIP. */
int kvp_wr_policy(kvp_ctx *ctx, uint32_t n, const uint32_t *h_w, const uint32_t *h_r10, uint32_t *d_placements);

/* The annealing over (W, R) as Sec. III-B describes it: window moves (W by -2, -1,
 * +1, +2), ratio moves (R by -0.1, +0.1) and diagonal moves (both), drawn with
 * probabilities op_prob[0..2] (the paper: 0.4, 0.4, 0.2); Metropolis acceptance;
 * the temperature starts where an average uphill proposal from the start state
 * is accepted with probability p0 (0.8) and is multiplied by alpha (0.9) after
 * each level of total_moves / n_levels proposals; the walk ends when the budget
 * is spent (stop_reason 0), when the best cost improved by less than stop_rel
 * (0.001) over a level (1), or when the temperature is below c_min_frac times its
 * start (2).  Proposals that leave 1 <= W <= w_max or 0 <= R <= 1 are counted and
 * skipped.  Proposal i uses Philox4x32-10 block (i, 0, 0, 16) under the seed
 * (word 0: operator; top two bits of word 1: window step; top bit of word 2:
 * ratio step; u = (word 3 + 0.5) / 2^32); the 32 proposals that set the start
 * temperature use stream 24.  Costs are those of kvp_score on the policy's
 * schedules, kept in h_table (HOST, [w_max][11] doubles, row W-1, column r10;
 * negative = not yet known; in/out, so that a table can be carried from one walk
 * to the next); unknown neighbours of the current state are evaluated together.
 * d_best_placement: DEVICE [L][N][Wd] or null; receives the best policy's schedule.
 * Errors: KVP_EINVAL, KVP_ENOTRACE, KVP_ESHAPE, KVP_ENOMEM, KVP_EHIP. */
typedef struct {
    uint32_t w_max, w0, r10_0, n_levels;
    uint64_t seed, total_moves;
    double p0, alpha, op_prob[3], stop_rel, c_min_frac;
} kvp_wr_params;
typedef struct {
    uint32_t best_w, best_r10, cur_w, cur_r10, levels_done, stop_reason;
    uint64_t proposals, accepted, out_of_range, evaluated;
    double best_T, cur_T, c0;
} kvp_wr_result;
int kvp_wr_search(kvp_ctx *ctx, const kvp_wr_params *params, double *h_table, kvp_wr_result *result,
                  uint32_t *d_best_placement);

const char *kvp_strerror(int code);

/* After a KVP_EHIP / KVP_ENOMEM return on this thread: the hipError_t value of
 * the failing HIP call (0 if none yet); *line (nullable) gets the library
 * source line, for bug reports. */
int kvp_last_hip_error(int *line);

#ifdef __cplusplus
}
#endif
#endif /* KVP_H */
