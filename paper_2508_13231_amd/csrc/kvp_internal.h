// Internal declarations shared by the translation units of libkvp.
// gfx950 (CDNA4) only: 64-lane wavefronts are assumed throughout.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kvp.h"

#define KVP_WAVE 64
#define KVP_SPARSE_CAP 64   // list entries per (layer, 32 token steps): one per lane of a wavefront

// Problem as the kernels see it.  Passed by value.
struct DevProblem {
    uint32_t L, N, P, Wd, K;
    uint32_t cap;                 // min(cap_pages, 2^31-1)
    const uint32_t *A;            // [L][N][K][Wd]
    const uint32_t *V;            // [N][Wd] alive
    const uint32_t *Pm;           // [N][Wd] persist
    const uint32_t *Wm;           // [N][Wd] written
    const uint32_t *acc;          // [L][N] read units of the step (all tiers)
    const uint32_t *wr;           // [N] pages written at the step
    const uint32_t *wsel;         // [N] index of the only word of Wm[n] with bits (0 if none), ~0 if several
    uint32_t single_write;        // every step's written pages sit in one word
    const uint32_t *tilecls;      // [ceil(N/64)] two bits per word (n_words <= 16): see KVP_WORD_*
    // [ceil(N/64)] bit i: words [i*G, (i+1)*G) are all FULL on the tile, G = 16, 64, 256 words
    const uint32_t *fullmask16, *fullmask64, *fullmask256;
    // per tile of 64 steps: leading words that are FULL on the tile; one past the last word in which a
    // page exists at some step of the tile (the words from there on hold no page: only stray bits)
    const uint32_t *tile_pfw, *tile_end;
    uint32_t wt[KVP_MAX_PLANES];  // plane_bytes[k] / unit
    // weight planes for single-page look-ups: the access planes with their weights, or (fewer) the
    // binary digit planes of the pages' read weights; pw[j] = 0 for j >= pn
    const uint32_t *pl;           // [L][N][pn][Wd]
    uint32_t pn;
    uint32_t pw[KVP_MAX_PLANES];
    double unit_b, page_b, token_b;          // bytes, exact integers held in fp64
    double inv_bh, inv_bk, inv_bd, inv_min;  // reciprocals of Eqs. 3-4's bandwidths
    uint32_t dram_bound;          // the DRAM channels are no faster than the link (inv_bd >= inv_bk)
};

// Class of a mask word over a tile of 64 token steps (and the step before it):
// FULL: all 32 pages exist at every one of those steps and persist into every
// step of the tile; EMPTY: none exists at any step of the tile; else MIXED.
enum { KVP_WORD_MIXED = 0, KVP_WORD_FULL = 1, KVP_WORD_EMPTY = 2 };

struct ChainState;   // kvp_moves.hip

struct kvp_ctx {
    int device = 0;
    hipStream_t stream = nullptr;
    bool has_trace = false;
    kvp_problem prob{};
    DevProblem dp{};
    uint64_t unit = 0;
    int score_kernel = 0;                // KVP_SCORE_AUTO, or the scorer kvp_score tries first
    uint32_t compute_units = 1;          // of the context's GPU
    int anneal_lookahead = 0;            // proposals per round in kvp_anneal: 0 auto, 1 or 4
    int capacity_mode = 0;               // KVP_CAPACITY_*: what the next fresh start of kvp_anneal walks under
    int chains_mode = 0;                 // what the present chains walk under
    unsigned char *d_slots_work = nullptr; size_t slots_work_cap = 0;   // migration steps: counters, moves per step, pool
    uint32_t *d_slots_cw = nullptr; size_t slots_cw_cap = 0;            // migrating pages per schedule word, scanned
    uint32_t *d_slots_list = nullptr; size_t slots_list_cap = 0;        // the migrating pages of a placement
    uint32_t *d_Xbest = nullptr;         // bounded log: [C][L][N][Wd], the best schedule of chains that have written it out
    uint64_t log_soft = 0;               // bounded log: entries after which a chain writes its best schedule out (0: not bounded)
    uint64_t log_entries = 0;            // kvp_set_anneal_log_entries: 0 = chosen from the sizes
    uint64_t gen_batch_bytes = 0;        // kvp_set_generator_batch_bytes: 0 = one / two gigabytes
    uint32_t *d_slot = nullptr;          // per-slot mode: [C][L][N], the pool after every slot of every chain
    bool no_alloc = false;               // set while kvp_score_static runs: kvp_ensure must not allocate
    int last_kernel = 0;                 // scorer that the last kvp_score ran (KVP_SCORE_*), 0 before the first
    bool prefix_full = false;            // on every 64-step tile all mask words but the last are FULL
    uint32_t pfw = 0;                    // leading mask words that are FULL on every 64-step tile
    uint32_t max_tail = 0;               // most words of a tile between its FULL prefix (rounded down to even) and tile_end
    const uint32_t *aw = nullptr;        // [L][N][kb][Wd] binary digits of the pages' read weights (may alias A)
    uint32_t kb = 0;                     // digit planes, 0 if the weights need more than five
    uint32_t *d_aw = nullptr;            // owned storage of aw when it is not A
    // For the row-per-lane scorer (rows of 29..36 words of one decoding sequence): the low `kd` digit planes
    // per (layer, tile of 64 steps) with a row stride of 36 words, [L][tiles][kd][64][36], and, when there
    // are more digit planes than kd, the non-zero words of those as a list per (layer, block of 32 steps):
    // [L][ceil(N/32)][KVP_SPARSE_CAP] entries {mask, row in the block | word << 8 | digit << 16 | 1 << 31}
    // (0: unused slot).  d_tl is null where that scorer does not apply.
    uint32_t *d_tl = nullptr; uint32_t kd = 0;
    uint2 *d_sparse = nullptr;
    uint32_t *d_trace = nullptr;         // one allocation: A, V, Pm, Wm, acc, wr
    // scoring scratch
    double *d_blocksum = nullptr;  size_t blocksum_cap = 0;   // [S][nb]
    uint32_t *d_tileflag = nullptr; size_t tileflag_cap = 0;  // [S][tiles]
    double *d_tglobal = nullptr; size_t tglobal_cap = 0;      // [S][L][N] step latencies (wide rows)
    uint32_t *d_chunkfull = nullptr; uint32_t cf_words = 0;   // [tiles][cf_words] bit c: chunk c of 16 words is FULL
    uint32_t *d_policy_work = nullptr; size_t policy_work_cap = 0;   // (W,R) policy: window counts, pool, wanted per candidate
    uint32_t *d_policy_x = nullptr; size_t policy_x_cap = 0;         // (W,R) search: schedules of a batch and their costs
    uint32_t *d_sel_keys = nullptr; size_t sel_keys_cap = 0;  // recency placement: 16-bit keys of a batch of steps
    uint32_t *d_cnt_tmp = nullptr; size_t cnt_tmp_cap = 0;    // delta: counters when not given
    uint32_t *d_occ_tmp = nullptr; size_t occ_tmp_cap = 0;
    // annealing state
    bool has_chains = false;
    kvp_anneal_params sa{};
    uint64_t moves_done = 0;
    uint32_t *d_X = nullptr;      // [C][L][N][Wd] current schedules
    uint32_t *d_cnt = nullptr;    // [C][L][N][4]
    uint32_t *d_occ = nullptr;    // [C][N]
    ChainState *d_state = nullptr;
    uint32_t *d_log = nullptr;    // [C][log_cap][LOG_WORDS] edits since the best schedule
    uint64_t log_cap = 0;
    double *d_cost = nullptr;     // [C]
    uint32_t *d_excess = nullptr; // [C]
    uint32_t *d_argmin = nullptr; // 1
};

// last failing HIP call of this thread: error code and source line, for kvp_last_hip_error()
extern thread_local int kvp_tls_hip_error;
extern thread_local int kvp_tls_hip_line;

#define KVP_HIP(call)                                   \
    do {                                                \
        hipError_t e_ = (call);                         \
        if (e_ != hipSuccess) {                         \
            kvp_tls_hip_error = (int)e_;                \
            kvp_tls_hip_line = __LINE__;                \
            (void)hipGetLastError();                    \
            return e_ == hipErrorOutOfMemory ? KVP_ENOMEM : KVP_EHIP; \
        }                                               \
    } while (0)

// ---- device helpers ---------------------------------------------------------
#if defined(__HIPCC__)

// Load of schedule words.  A launch reads them once, while the trace words are read again by every
// group of schedules: marked as streaming, they leave the trace its place in the L2.
#define KVP_LOAD_X(ptr) __builtin_nontemporal_load(ptr)

// Placement of workgroups that each take one (tile of token steps, group of schedules): the
// hardware hands consecutive workgroups to the eight XCDs in turn (blockIdx & 7), each XCD with an
// L2 of its own.  The pairs, tile-major, are cut into eight equal runs, one per XCD, and the
// workgroups of an XCD walk its run in order: the XCD works on one tile at a time (that tile's trace
// is fetched from HBM once and then served by its L2), and every XCD gets the same amount of work
// whatever the number of tiles.  Returns false for the few workgroups past the end of a run.
__device__ __forceinline__ bool xcd_pair(uint32_t tiles, uint32_t groups, uint32_t &tile, uint32_t &group) {
    const uint32_t pairs = tiles * groups, per = (pairs + 7) / 8;
    const uint32_t pair = (blockIdx.x & 7u) * per + (blockIdx.x >> 3);
    tile = pair / groups;
    group = pair - tile * groups;
    return (blockIdx.x >> 3) < per && pair < pairs;
}
// workgroups to launch for xcd_pair
static inline uint64_t xcd_grid(uint32_t tiles, uint32_t groups) { return ((uint64_t)tiles * groups + 7) / 8 * 8; }

__device__ __forceinline__ int lane_id() { return (int)(threadIdx.x & (KVP_WAVE - 1)); }

__device__ __forceinline__ uint32_t wave_sum_u32(uint32_t v) {
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o, KVP_WAVE);
    return v;
}
// Inclusive prefix sum over the 64 lanes without LDS: shifts inside the rows of 16 lanes, then the
// last lane of a row is broadcast into the next row (rows 1 and 3), then lane 31 into rows 2 and 3.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ uint32_t dpp_or_zero(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, ROW_MASK, 0xf, false);   // lanes without a source get 0
}
__device__ __forceinline__ uint32_t wave_incl_scan_u32(uint32_t v) {
    v += dpp_or_zero<0x111, 0xf>(v);     // row_shr:1
    v += dpp_or_zero<0x112, 0xf>(v);     // row_shr:2
    v += dpp_or_zero<0x114, 0xf>(v);     // row_shr:4
    v += dpp_or_zero<0x118, 0xf>(v);     // row_shr:8
    v += dpp_or_zero<0x142, 0xa>(v);     // row_bcast:15 into rows 1 and 3
    v += dpp_or_zero<0x143, 0xc>(v);     // row_bcast:31 into rows 2 and 3
    return v;
}

__device__ __forceinline__ uint32_t wave_or_u32(uint32_t v) {
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) v |= __shfl_xor(v, o, KVP_WAVE);
    return v;
}
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v) {
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) { uint32_t t = __shfl_xor(v, o, KVP_WAVE); v = t > v ? t : v; }
    return v;
}
// The 64-wide summation tree of the total latency: fold the upper half onto the
// lower half (32, 16, ..., 1).  Every lane ends with the same bits because
// a + b == b + a in IEEE arithmetic.  All 64 lanes must be active.
// Folds 32 and 16 use the gfx950 half / row swaps (v_permlane32_swap with both operands v leaves
// (low half, low half) and (high half, high half): their sum is v[i] + v[i ^ 32] in every lane;
// v_permlane16_swap does the same with the 16-lane rows).  Folds 8..1 rotate within rows of 16:
// after the folds before it the values repeat with period 2k, so the lane k places away holds
// the same bits as lane i ^ k.  No LDS round trips, unlike a cross-lane shuffle.
template <int CTRL>
__device__ __forceinline__ double dpp_f64(double v) {
    const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(v), CTRL, 0xf, 0xf, false);
    const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(v), CTRL, 0xf, 0xf, false);
    return __hiloint2double(hi, lo);
}
__device__ __forceinline__ double wave_tree_sum_f64(double v) {
    {
        const uint32_t lo = (uint32_t)__double2loint(v), hi = (uint32_t)__double2hiint(v);
        const auto a = __builtin_amdgcn_permlane32_swap(lo, lo, false, false);
        const auto b = __builtin_amdgcn_permlane32_swap(hi, hi, false, false);
        v = __hiloint2double((int)b[0], (int)a[0]) + __hiloint2double((int)b[1], (int)a[1]);
    }
    {
        const uint32_t lo = (uint32_t)__double2loint(v), hi = (uint32_t)__double2hiint(v);
        const auto a = __builtin_amdgcn_permlane16_swap(lo, lo, false, false);
        const auto b = __builtin_amdgcn_permlane16_swap(hi, hi, false, false);
        v = __hiloint2double((int)b[0], (int)a[0]) + __hiloint2double((int)b[1], (int)a[1]);
    }
    v = v + dpp_f64<0x128>(v);   // row_ror:8
    v = v + dpp_f64<0x124>(v);   // row_ror:4
    v = v + dpp_f64<0x122>(v);   // row_ror:2
    v = v + dpp_f64<0x121>(v);   // row_ror:1
    return v;
}

// v[i] + v[i ^ m] in every lane, m a power of two (the same for the whole wavefront), all lanes
// active: one fold of the summation tree across lanes, without LDS where the hardware allows.
__device__ __forceinline__ double fold_xor_f64(double v, uint32_t m) {
    switch (m) {
        case 1: return v + dpp_f64<0xB1>(v);    // quad_perm [1,0,3,2]
        case 2: return v + dpp_f64<0x4E>(v);    // quad_perm [2,3,0,1]
        case 8: return v + dpp_f64<0x128>(v);   // row_ror:8 is i ^ 8 within a row of 16
        case 16: {
            const uint32_t lo = (uint32_t)__double2loint(v), hi = (uint32_t)__double2hiint(v);
            const auto a = __builtin_amdgcn_permlane16_swap(lo, lo, false, false);
            const auto b = __builtin_amdgcn_permlane16_swap(hi, hi, false, false);
            return __hiloint2double((int)b[0], (int)a[0]) + __hiloint2double((int)b[1], (int)a[1]);
        }
        case 32: {
            const uint32_t lo = (uint32_t)__double2loint(v), hi = (uint32_t)__double2hiint(v);
            const auto a = __builtin_amdgcn_permlane32_swap(lo, lo, false, false);
            const auto b = __builtin_amdgcn_permlane32_swap(hi, hi, false, false);
            return __hiloint2double((int)b[0], (int)a[0]) + __hiloint2double((int)b[1], (int)a[1]);
        }
        default: return v + __shfl_xor(v, (int)m, KVP_WAVE);
    }
}

// Step latency, Eqs. 2-4, from the step's counters.  hr_u: read units served by
// HBM; hw: written pages in HBM; mi/mo: pages migrated in/out; acc_u, wr: the
// step's totals.  Every product below is an integer < 2^53, hence exact; the
// order of the floating-point operations is fixed (no contraction).
__device__ __forceinline__ double step_time(const DevProblem &q, uint32_t hr_u, uint32_t hw, uint32_t mi,
                                            uint32_t mo, uint32_t acc_u, uint32_t wr) {
    double hr_b = (double)hr_u * q.unit_b;
    double er_b = (double)(acc_u - hr_u) * q.unit_b;
    double hw_b = (double)hw * q.token_b;
    double ew_b = (double)(wr - hw) * q.token_b;
    double mi_b = (double)mi * q.page_b;
    double mo_b = (double)mo * q.page_b;
    double t_h = (((hr_b + hw_b) + mi_b) + mo_b) * q.inv_bh;                 // Eq. 3
    double chan = ((ew_b + mi_b) + mo_b) * q.inv_bd;
    double m = chan;
    if (!q.dram_bound) {
        // Otherwise the channel term is the largest of the three as it stands: its byte count (an
        // exact integer) is no smaller than the other two, its factor no smaller than theirs, and
        // rounding a product is monotonic.
        double link_out = (ew_b + mo_b) * q.inv_bk;
        double link_in = mi_b * q.inv_bk;
        // all operands are finite and >= +0: the hardware maximum picks the same value as a comparison
        m = __builtin_fmax(__builtin_fmax(link_out, link_in), chan);
    }
    double t_e = er_b * q.inv_min + m;                                       // Eq. 4
    return __builtin_fmax(t_h, t_e);                                         // Eq. 2
}

#endif  // __HIPCC__

// ---- entry points implemented across files -----------------------------------
int kvp_score_launch(kvp_ctx *ctx, const uint32_t *d_placements, uint32_t S, double *d_cost,
                     uint32_t *d_excess, uint32_t *d_counters, uint32_t *d_occ);
int kvp_ensure(kvp_ctx *ctx, void **p, size_t *cap, size_t bytes);
int kvp_static_scratch_init(int device);     // kvp_score.hip: resolves the device address of the static scratch
int kvp_bitslice_build(kvp_ctx *ctx);
int kvp_slots_state_launch(kvp_ctx *ctx, const uint32_t *X, bool broadcast_x, const uint8_t *Y, uint32_t S, double *d_cost,
                           uint32_t *d_excess, uint32_t **cnt_out, uint32_t **mig_out, uint32_t **pool_out);
int kvp_slot_list_build(kvp_ctx *ctx, const uint32_t *X, uint32_t **list_out, uint32_t *count_out);
int kvp_blocksum_from_t_launch(kvp_ctx *ctx, uint32_t S, uint32_t nb_total);
int kvp_slot_occupancy_launch(kvp_ctx *ctx, const uint32_t *d_placements, uint32_t S, uint32_t *d_excess, uint32_t *d_table);
int kvp_rowlane_build(kvp_ctx *ctx);          // kvp_score_rowlane.hip: called at the end of kvp_bitslice_build
void kvp_free_chains(kvp_ctx *ctx);
