// The paper's own search (Sec. III-B): a look-ahead placement policy with two
// scalars, the window W (token steps looked ahead) and the ratio R (share of the
// pages qualified for migration that really migrate), and the annealing over
// (W, R).  The reading of the policy, once per token step n, one pool of
// cap_pages for all layers:
//   1. pages that do not hold the same data as one step earlier leave the pool;
//   2. the existing pages read in steps n .. n+W-1 are collected with their read
//      frequency f there (summed over the planes);
//   3. ranked by f descending, ties to the lower l*P+p, the first cap_pages are
//      the wanted set;
//   4. the wanted pages outside the pool are qualified for migration; the first
//      m = (r10 * their number + 5) div 10 of them, in rank order, come in (R = r10/10);
//   5. if the pool would overflow, as many pool pages that are not wanted leave,
//      least-read-in-the-window first, ties to the lower l*P+p;
//   6. the pool is the placement of step n in every layer's row.
//
// kvp_wr_policy turns a batch of (W, R) candidates into schedules in three passes over a batch of
// token steps.  The window counts f and the wanted set (steps 2 and 3) follow from the trace and W
// alone, so they are computed once per distinct window, for all steps of the batch at once: a thread
// per pair slides its window count along the steps, then a workgroup per step selects the wanted
// pages by histogram threshold and index-ordered ties (kvp_select.h).  Only the pool carries from one
// step to the next: a workgroup per candidate walks the steps, and its two selections (steps 4 and 5)
// visit the set bits of the pool and wanted masks only.  kvp_wr_search is the annealing itself: a
// host loop over a memoised table T(W, R), filled by scoring whole neighbourhoods of candidates at
// once (generator + kvp_score), so the accelerator sees batches, not single points.
#include <math.h>

#include <vector>

#include "kvp_internal.h"
#include "kvp_select.h"

namespace {

// reads of (layer l, word w, bit b) at step m, summed over the planes
__device__ __forceinline__ uint32_t reads_at(const DevProblem &q, uint32_t l, uint32_t m, uint32_t w, uint32_t b) {
    const uint32_t *a = q.A + ((size_t)l * q.N + m) * q.K * q.Wd + w;
    uint32_t s = 0;
    for (uint32_t k = 0; k < q.K; k++) s += (a[(size_t)k * q.Wd] >> b) & 1u;
    return s;
}

// Window counts.  Thread (g, u) walks the steps [n_lo, n_hi) for pair g and distinct window u and
// writes f[u][n - n_lo][g]; fstate[u][g] carries the count into the next batch of steps.  FT is the
// narrowest type that holds W * K (a byte for one plane and any window up to 255 steps).
template <class FT>
__global__ __launch_bounds__(256) void wr_counts_kernel(DevProblem q, RowDiv rd, const uint32_t *__restrict__ uw,
                                                        uint32_t n_lo, uint32_t n_hi, uint32_t B, FT *__restrict__ fstate,
                                                        FT *__restrict__ fk) {
    const uint32_t G = q.L * q.Wd * 32, g = blockIdx.x * 256 + threadIdx.x, u = blockIdx.y;
    if (g >= G) return;
    const uint32_t wi = g >> 5, b = g & 31u, l = rd.quot(wi), w = wi - l * q.Wd;
    const uint32_t W = min(uw[u], q.N);
    uint32_t s = 0;
    if (n_lo == 0)
        for (uint32_t m = 0; m < W; m++) s += reads_at(q, l, m, w, b);
    else
        s = (uint32_t)fstate[(size_t)u * G + g];
    FT *out = fk + (size_t)u * B * G + g;
    for (uint32_t n = n_lo; n < n_hi; n++) {
        if (n > 0) {                                                   // the window slides: step n-1 leaves, n+W-1 enters
            s -= reads_at(q, l, n - 1, w, b);
            if (n + W - 1 < q.N) s += reads_at(q, l, n + W - 1, w, b);
        }
        out[(size_t)(n - n_lo) * G] = (FT)s;
    }
    fstate[(size_t)u * G + g] = (FT)s;
}

// Steps 2 and 3 for step n_lo + blockIdx.x and distinct window blockIdx.y: the wanted set as mask words.
template <class FT>
__global__ __launch_bounds__(BT) void wr_wanted_kernel(DevProblem q, RowDiv rd, uint64_t cap, const uint32_t *__restrict__ uw,
                                                       uint32_t n_lo, uint32_t B, const FT *__restrict__ fk,
                                                       uint32_t *__restrict__ wanted_all) {
    extern __shared__ uint32_t lds_u[];
    __shared__ SelectShared sh;
    const uint32_t LW = q.L * q.Wd, G = LW * 32, u = blockIdx.y, n = n_lo + blockIdx.x;
    const uint32_t W = min(uw[u], q.N);
    const FT *f = fk + ((size_t)u * B + blockIdx.x) * G;
    uint32_t *wanted = wanted_all + ((size_t)u * B + blockIdx.x) * LW;
    auto key_want = [&](uint32_t g) {
        const uint32_t w = rd.rem(g >> 5), b = g & 31u;
        const uint32_t vw = q.V[(size_t)n * q.Wd + w];
        uint32_t fv = (uint32_t)f[g];
        asm volatile("" : "+v"(fv));                                   // loaded whether the page exists or not
        return ((vw >> b) & 1u) && fv > 0 ? fv : NOT_A_CANDIDATE;
    };
    block_select(G, W * q.K + 1, cap, lds_u, sh, key_want, key_want, [&](uint32_t word, uint32_t bits) { wanted[word] = bits; });
}

// Steps 1 and 4 to 6 for candidate blockIdx.x over the steps [n_lo, n_hi): pools[candidate][LW] carries
// the pool from one batch of steps to the next.  Per step three passes over the L * Wd mask words, every
// wavefront on its own run of 64-word chunks (lane = word, CU chunks in flight):
//   pass 0  pool &= persist; how many wanted pages are outside, how many pages are in the pool: that
//           fixes how many come in (m_in) and how many must leave (need);
//   pass 1  both selections at once.  Who leaves is chosen among pool & ~wanted by key fmax - f, who comes
//           among wanted & ~pool by key f; the second set does not depend on the outcome of the first, so
//           one pass fills both histograms (and one per wavefront each, for the ties);
//   pass 2  the two thresholds and the index-ordered ties decide every candidate; the new pool word is
//           stored and written to the schedule rows of step n.
// Only the set bits of a word are visited (a handful per word), their keys picked out of the word's 32,
// which were fetched as whole vectors.
// LDS: [2][nbins] histograms, then [2][BW][nbins] per wavefront if wave_bins.
template <class FT>
__global__ __launch_bounds__(BT) void wr_pool_kernel(DevProblem q, RowDiv rd, uint64_t cap, const uint32_t *__restrict__ cand_w,
                                                     const uint32_t *__restrict__ cand_r10, const uint32_t *__restrict__ cand_u,
                                                     uint32_t n_lo, uint32_t n_hi, uint32_t B, uint32_t *pools,
                                                     const uint32_t *__restrict__ wanted_all, const FT *__restrict__ fk,
                                                     uint32_t *Xall, int wave_bins) {
    extern __shared__ __align__(16) uint32_t lds_w[];
    __shared__ SelectShared sh_out, sh_in;
    __shared__ uint32_t counts[2];
    const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const uint32_t LW = q.L * q.Wd, G = LW * 32;
    const uint32_t W = min(cand_w[blockIdx.x], q.N), r10 = cand_r10[blockIdx.x], u = cand_u[blockIdx.x];
    uint32_t *pool = pools + (size_t)blockIdx.x * LW;
    uint32_t *X = Xall + (size_t)blockIdx.x * q.L * q.N * q.Wd;
    const uint32_t fmax = W * q.K, nbins = fmax + 1;
    uint32_t *hist_out = lds_w, *hist_in = lds_w + nbins;
    uint32_t *mine_out = wave_bins ? lds_w + (size_t)(2 + wave) * nbins : nullptr;
    uint32_t *mine_in = wave_bins ? lds_w + (size_t)(2 + BW + wave) * nbins : nullptr;
    const uint32_t nchunks = (LW + 63) / 64, cpw = (nchunks + BW - 1) / BW;     // chunks of 64 words per wavefront
    const uint32_t c_lo = min(wave * cpw, nchunks), c_hi = min(c_lo + cpw, nchunks);
    constexpr int KU = sizeof(FT) == 1 ? CU : sizeof(FT) == 2 ? CU / 2 : 1;    // chunks whose keys are in flight together
    if (n_lo == 0)
        for (uint32_t wi = tid; wi < LW; wi += BT) pool[wi] = 0;
    __syncthreads();
    for (uint32_t n = n_lo; n < n_hi; n++) {
        const uint32_t *wanted = wanted_all + ((size_t)u * B + (n - n_lo)) * LW;
        const FT *f = fk + ((size_t)u * B + (n - n_lo)) * G;
        if (tid < 2) counts[tid] = 0;
        for (uint32_t k = tid; k < (wave_bins ? (2 + 2 * BW) * nbins : 2 * nbins); k += BT) lds_w[k] = 0;
        // ---- pass 0
        uint32_t nq = 0, np = 0;
        for (uint32_t c0 = c_lo; c0 < c_hi; c0 += CU) {
            uint32_t pw[CU], ww[CU], pm[CU];
#pragma unroll
            for (int j = 0; j < CU; j++) {
                const uint32_t wi = min((c0 + j) * 64 + lane, LW - 1);
                pw[j] = pool[wi]; ww[j] = wanted[wi]; pm[j] = q.Pm[(size_t)n * q.Wd + rd.rem(wi)];
            }
#pragma unroll
            for (int j = 0; j < CU; j++) {
                const uint32_t wi = (c0 + j) * 64 + lane;
                if (c0 + j >= c_hi || wi >= LW) continue;
                const uint32_t keep = pw[j] & pm[j];                   // step 1
                if (keep != pw[j]) pool[wi] = keep;
                nq += __popc(ww[j] & ~keep);
                np += __popc(keep);
            }
        }
        nq = wave_sum_u32(nq); np = wave_sum_u32(np);
        __syncthreads();                                               // counts and histograms are clear
        if (lane == 0) { atomicAdd(&counts[0], nq); atomicAdd(&counts[1], np); }
        __syncthreads();
        const uint64_t m_in = ((uint64_t)r10 * counts[0] + 5) / 10;    // step 4
        const uint64_t in_pool = counts[1];
        const uint64_t need = in_pool + m_in > cap ? in_pool + m_in - cap : 0;   // step 5
        const bool do_out = need > 0, do_in = m_in > 0;
        // ---- pass 1
        if (do_out || do_in)
            for (uint32_t c0 = c_lo; c0 < c_hi; c0 += KU) {
                uint32_t mo[KU], mi[KU];
                WordKeys<FT> kw[KU];
                // every load of the group is issued whether its word holds a candidate or not: loads under
                // conditions would each wait for the ones before
#pragma unroll
                for (int j = 0; j < KU; j++) {
                    const uint32_t wi = (c0 + j) * 64 + lane;
                    const bool in = c0 + j < c_hi && wi < LW;
                    const uint32_t wc = in ? wi : LW - 1;
                    const uint32_t pw = pool[wc], ww = wanted[wc];
                    kw[j].load(f, wc);
                    mo[j] = do_out && in ? pw & ~ww : 0u;
                    mi[j] = do_in && in ? ww & ~pw : 0u;
                }
#pragma unroll
                for (int j = 0; j < KU; j++)
                    for (uint32_t m = mo[j] | mi[j]; m; m &= m - 1) {
                        const uint32_t b = __ffs(m) - 1, fv = kw[j].get(b);
                        // a wavefront counts into its own histograms where it has them: sixteen wavefronts
                        // adding to the same few counters of one histogram take four times as long
                        if ((mo[j] >> b) & 1u) atomicAdd(mine_out ? &mine_out[fmax - fv] : &hist_out[fmax - fv], 1u);
                        else atomicAdd(mine_in ? &mine_in[fv] : &hist_in[fv], 1u);
                    }
            }
        __syncthreads();
        if (wave_bins) {                                               // the workgroup's histograms: the sums
            for (uint32_t k = tid; k < 2 * nbins; k += BT) {
                const uint32_t *src = lds_w + (k < nbins ? (size_t)2 * nbins + k : (size_t)(2 + BW) * nbins + (k - nbins));
                uint32_t sum = 0;
                for (int w = 0; w < BW; w++) sum += src[(size_t)w * nbins];
                lds_w[k] = sum;
            }
            __syncthreads();
        }
        if (do_out) select_threshold(nbins, need, hist_out, sh_out);
        if (do_in) select_threshold(nbins, m_in, hist_in, sh_in);
        const uint32_t T_out = sh_out.threshold, r_out = sh_out.take_ties, T_in = sh_in.threshold, r_in = sh_in.take_ties;
        const bool all_out = sh_out.take_all != 0, all_in = sh_in.take_all != 0;
        // the ties of every wavefront's words, so that they can be numbered in index order
        uint32_t t_out = 0, t_in = 0;
        if (wave_bins) {
            t_out = do_out && !all_out && T_out < nbins ? mine_out[T_out] : 0u;
            t_in = do_in && !all_in && T_in < nbins ? mine_in[T_in] : 0u;
        } else if ((do_out && !all_out) || (do_in && !all_in)) {
            for (uint32_t c = c_lo; c < c_hi; c++) {
                const uint32_t wi = c * 64 + lane;
                const uint32_t pw = wi < LW ? pool[wi] : 0u, ww = wi < LW ? wanted[wi] : 0u;
                const uint32_t o = do_out ? pw & ~ww : 0u, i = do_in ? ww & ~pw : 0u;
                if (!__ballot((o | i) != 0)) continue;
                WordKeys<FT> kw;
                if (o | i) kw.load(f, wi);
                for (uint32_t m = o | i; m; m &= m - 1) {
                    const uint32_t b = __ffs(m) - 1, fv = kw.get(b);
                    if ((o >> b) & 1u) t_out += fmax - fv == T_out;
                    else t_in += fv == T_in;
                }
            }
            t_out = wave_sum_u32(t_out); t_in = wave_sum_u32(t_in);
        }
        if (lane == 0) { sh_out.wave_ties[wave] = t_out; sh_in.wave_ties[wave] = t_in; }
        __syncthreads();
        uint32_t rank_out = 0, rank_in = 0;
        for (uint32_t w = 0; w < wave; w++) { rank_out += sh_out.wave_ties[w]; rank_in += sh_in.wave_ties[w]; }
        // ---- pass 2
        // which of a chunk's ties (bits of `tie`, lane = word) are among the first r in index order, rank0
        // of them lying before the chunk: all lanes together
        auto number_ties = [&](uint32_t tie, uint32_t &rank0, uint32_t r) -> uint32_t {
            if (rank0 >= r || !__ballot(tie != 0)) return 0u;         // the same for the whole wavefront
            const uint32_t tc = __popc(tie);
            const uint32_t incl = wave_incl_scan_u32(tc);              // ties in this and the lower lanes
            uint32_t rank = rank0 + incl - tc;                         // rank of this word's first tie
            rank0 += (uint32_t)__builtin_amdgcn_readlane((int)incl, 63);
            if (rank + tc <= r) return tie;                            // all of the word's
            uint32_t take = 0;
            for (uint32_t t = tie; t; t &= t - 1, rank++)              // ties below rank r are taken
                if (rank < r) take |= t & (0u - t);
            return take;
        };
        for (uint32_t c0 = c_lo; c0 < c_hi; c0 += KU) {
            uint32_t pw[KU], mo[KU], mi[KU];
            WordKeys<FT> kw[KU];
#pragma unroll
            for (int j = 0; j < KU; j++) {
                const uint32_t wi = (c0 + j) * 64 + lane;
                const bool in = c0 + j < c_hi && wi < LW;
                const uint32_t wc = in ? wi : LW - 1;
                const uint32_t ww = wanted[wc];
                pw[j] = pool[wc];
                kw[j].load(f, wc);
                mo[j] = do_out && in ? pw[j] & ~ww : 0u;
                mi[j] = do_in && in ? ww & ~pw[j] : 0u;
            }
            const bool keys_out = do_out && !all_out, keys_in = do_in && !all_in;
#pragma unroll
            for (int j = 0; j < KU; j++) {
                if (c0 + j >= c_hi) break;                             // the same for the whole wavefront
                uint32_t out = all_out ? mo[j] : 0u, in = all_in ? mi[j] : 0u, tie_o = 0, tie_i = 0;
                for (uint32_t m = (keys_out ? mo[j] : 0u) | (keys_in ? mi[j] : 0u); m; m &= m - 1) {
                    const uint32_t b = __ffs(m) - 1, fv = kw[j].get(b), bit = 1u << b;
                    if (mo[j] & bit) {
                        const uint32_t k = fmax - fv;
                        out |= k > T_out ? bit : 0u;
                        tie_o |= k == T_out ? bit : 0u;
                    } else {
                        in |= fv > T_in ? bit : 0u;
                        tie_i |= fv == T_in ? bit : 0u;
                    }
                }
                out |= number_ties(tie_o, rank_out, r_out);
                in |= number_ties(tie_i, rank_in, r_in);
                const uint32_t wi = (c0 + j) * 64 + lane;
                if (wi < LW) {
                    const uint32_t now = (pw[j] & ~out) | in;
                    if (now != pw[j]) pool[wi] = now;
                    const uint32_t l = rd.quot(wi), w = wi - l * q.Wd;
                    X[((size_t)l * q.N + n) * q.Wd + w] = now;         // step 6
                }
            }
        }
        __syncthreads();
    }
}

}  // namespace

extern "C" int kvp_wr_policy(kvp_ctx *ctx, uint32_t n, const uint32_t *h_w, const uint32_t *h_r10,
                             uint32_t *d_placements) {
    if (!ctx) return KVP_EINVAL;
    if (!ctx->has_trace) return KVP_ENOTRACE;
    if (n == 0) return KVP_OK;
    if (!h_w || !h_r10 || !d_placements || ((uintptr_t)d_placements & 3u)) return KVP_EINVAL;
    const DevProblem &q = ctx->dp;
    uint32_t wmax = 0;
    for (uint32_t i = 0; i < n; i++) {
        if (h_w[i] < 1 || h_r10[i] > 10) return KVP_EINVAL;
        const uint32_t w = h_w[i] < q.N ? h_w[i] : q.N;
        wmax = w > wmax ? w : wmax;
    }
    const uint64_t G64 = (uint64_t)q.L * q.Wd * 32;
    if (G64 >= (1ull << 31)) return KVP_ESHAPE;
    const size_t lds = ((size_t)wmax * q.K + 1) * 4;
    if (lds > 64 * 1024) return KVP_ESHAPE;                            // the pool walk keeps two such histograms in LDS
    KVP_HIP(hipSetDevice(ctx->device));
    const RowDiv rd(q.Wd, (uint64_t)q.L * q.Wd);
    const uint64_t fmax = (uint64_t)wmax * q.K;
    const size_t fbytes = fmax <= 0xFF ? 1 : fmax <= 0xFFFF ? 2 : 4;
    // the distinct windows of the batch, and which of them each candidate uses
    std::vector<uint32_t> host(3 * (size_t)n), uw;
    for (uint32_t i = 0; i < n; i++) {
        const uint32_t w = h_w[i] < q.N ? h_w[i] : q.N;
        uint32_t u = 0;
        while (u < uw.size() && uw[u] != w) u++;
        if (u == uw.size()) uw.push_back(w);
        host[i] = w; host[(size_t)n + i] = h_r10[i]; host[2 * (size_t)n + i] = u;
    }
    const uint32_t nu = (uint32_t)uw.size();
    host.insert(host.end(), uw.begin(), uw.end());
    // steps per batch: the counts and wanted masks of a batch take two gigabytes at most, or what
    // kvp_set_generator_batch_bytes says (one step at least)
    const size_t LW = (size_t)q.L * q.Wd, G = (size_t)G64;
    const size_t per_step = (size_t)nu * (G * fbytes + LW * 4);
    const size_t budget = ctx->gen_batch_bytes ? (size_t)ctx->gen_batch_bytes : ((size_t)2 << 30);
    const uint32_t B = (uint32_t)(per_step >= budget ? 1 : budget / per_step < q.N ? budget / per_step : q.N);
    // layout, in words: candidate table | pools | wanted masks | count state | counts
    const size_t o_pool = (host.size() + 3) & ~(size_t)3, o_want = o_pool + (size_t)n * LW, o_state = o_want + (size_t)nu * B * LW;
    const size_t o_f = (o_state + ((size_t)nu * G * fbytes + 3) / 4 + 31) & ~(size_t)31;   // a word's 32 counts: whole 16-byte vectors
    const size_t total = o_f + ((size_t)nu * B * G * fbytes + 3) / 4;
    // the pool walk keeps two histograms, and two per wavefront beside them when all 34 fit 64 KB
    const int wave_bins = lds * (2 + 2 * BW) <= 64 * 1024;
    const size_t lds_pool = wave_bins ? lds * (2 + 2 * BW) : lds * 2;
    int rc = kvp_ensure(ctx, (void **)&ctx->d_policy_work, &ctx->policy_work_cap, total * 4);
    if (rc) return rc;
    uint32_t *wk = ctx->d_policy_work;
    const uint32_t *d_w = wk, *d_r = wk + n, *d_u = wk + 2 * (size_t)n, *d_uw = wk + 3 * (size_t)n;
    KVP_HIP(hipMemcpyAsync(wk, host.data(), host.size() * 4, hipMemcpyHostToDevice, ctx->stream));
    KVP_HIP(hipStreamSynchronize(ctx->stream));                        // the host arrays go away after the call
    const uint64_t cap = ctx->prob.cap_pages;
#define KVP_POLICY(FT)                                                                                              \
    do {                                                                                                            \
        if (lds > 48 * 1024) {                                                                                      \
            KVP_HIP(hipFuncSetAttribute((const void *)wr_wanted_kernel<FT>, hipFuncAttributeMaxDynamicSharedMemorySize, \
                                        (int)lds));                                                                 \
        }                                                                                                           \
        if (lds_pool > 48 * 1024)                                                                                   \
            KVP_HIP(hipFuncSetAttribute((const void *)wr_pool_kernel<FT>, hipFuncAttributeMaxDynamicSharedMemorySize, \
                                        (int)lds_pool));                                                            \
        FT *fstate = (FT *)(wk + o_state), *fk = (FT *)(wk + o_f);                                                  \
        for (uint32_t n_lo = 0; n_lo < q.N; n_lo += B) {                                                            \
            const uint32_t n_hi = n_lo + B < q.N ? n_lo + B : q.N;                                                  \
            wr_counts_kernel<FT><<<dim3((uint32_t)((G + 255) / 256), nu), dim3(256), 0, ctx->stream>>>(             \
                q, rd, d_uw, n_lo, n_hi, B, fstate, fk);                                                            \
            wr_wanted_kernel<FT><<<dim3(n_hi - n_lo, nu), dim3(BT), lds, ctx->stream>>>(q, rd, cap, d_uw, n_lo, B, fk, \
                                                                                       wk + o_want);                \
            wr_pool_kernel<FT><<<dim3(n), dim3(BT), lds_pool, ctx->stream>>>(                                       \
                q, rd, cap, d_w, d_r, d_u, n_lo, n_hi, B, wk + o_pool, wk + o_want, fk, d_placements, wave_bins);   \
        }                                                                                                           \
    } while (0)
    if (fbytes == 1) KVP_POLICY(uint8_t);
    else if (fbytes == 2) KVP_POLICY(uint16_t);
    else KVP_POLICY(uint32_t);
#undef KVP_POLICY
    KVP_HIP(hipGetLastError());
    return KVP_OK;
}

namespace {

// proposal i of the walk: Philox4x32-10 block (i, 0, 0, stream) under the seed
void philox_host(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0, uint32_t k1, uint32_t out[4]) {
    for (int r = 0; r < 10; r++) {
        const uint64_t m0 = (uint64_t)0xD2511F53u * c0, m1 = (uint64_t)0xCD9E8D57u * c2;
        const uint32_t n0 = (uint32_t)(m1 >> 32) ^ c1 ^ k0, n2 = (uint32_t)(m0 >> 32) ^ c3 ^ k1;
        c0 = n0; c1 = (uint32_t)m1; c2 = n2; c3 = (uint32_t)m0;
        k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

bool propose(const kvp_wr_params &sp, uint64_t i, uint32_t stream, uint32_t w, uint32_t r10, uint32_t &w2, uint32_t &r2,
             double &u) {
    uint32_t a[4];
    philox_host((uint32_t)i, (uint32_t)(i >> 32), 0, stream, (uint32_t)sp.seed, (uint32_t)(sp.seed >> 32), a);
    const uint64_t th0 = (uint64_t)(sp.op_prob[0] * 4294967296.0);
    const uint64_t th1 = (uint64_t)((sp.op_prob[0] + sp.op_prob[1]) * 4294967296.0);
    const int op = (uint64_t)a[0] < th0 ? 0 : (uint64_t)a[0] < th1 ? 1 : 2;   // window, ratio, both
    static const int steps[4] = {-2, -1, 1, 2};
    const int dw = op != 1 ? steps[a[1] >> 30] : 0;
    const int dr = op != 0 ? ((a[2] >> 31) ? 1 : -1) : 0;
    u = ((double)a[3] + 0.5) * (1.0 / 4294967296.0);
    const int64_t nw = (int64_t)w + dw, nr = (int64_t)r10 + dr;
    if (nw < 1 || nw > (int64_t)sp.w_max || nr < 0 || nr > 10) return false;
    w2 = (uint32_t)nw; r2 = (uint32_t)nr;
    return true;
}

}  // namespace

extern "C" int kvp_wr_search(kvp_ctx *ctx, const kvp_wr_params *sp, double *h_table, kvp_wr_result *res,
                             uint32_t *d_best_placement) {
    if (!ctx || !sp || !h_table || !res) return KVP_EINVAL;
    if (!ctx->has_trace) return KVP_ENOTRACE;
    if (sp->w_max < 1 || sp->w0 < 1 || sp->w0 > sp->w_max || sp->r10_0 > 10 || sp->n_levels < 1 || !(sp->p0 > 0.0) ||
        !(sp->p0 < 1.0))
        return KVP_EINVAL;
    const DevProblem &q = ctx->dp;
    const size_t words = (size_t)q.L * q.N * q.Wd;
    KVP_HIP(hipSetDevice(ctx->device));
    *res = kvp_wr_result{};
    // T(w, r10).  An unknown cost is never evaluated alone: the states nearest to the current one
    // (cw, cr) that are still unknown go with it, in one batch for the generator (a workgroup per
    // state: a batch should have a few hundred to fill the GPU) and the scorer.  The batch takes up
    // to a third of the free device memory, at least 4 GiB and at least the 14 states one proposal away.
    int err = KVP_OK;
    size_t mem_free = 0, mem_total = 0;
    KVP_HIP(hipMemGetInfo(&mem_free, &mem_total));
    const size_t budget = mem_free / 3 > ((size_t)4 << 30) ? mem_free / 3 : ((size_t)4 << 30);
    const size_t fit = budget / (words * 4);
    const size_t batch_max = fit > 15 ? fit : 15;
    auto cost = [&](uint32_t w, uint32_t r10, uint32_t cw, uint32_t cr) -> double {
        double &slot = h_table[(size_t)(w - 1) * 11 + r10];
        if (slot >= 0.0 || err) return slot;
        std::vector<uint32_t> ws{w}, rs{r10};
        for (uint32_t ring = 1; ring <= sp->w_max + 10 && ws.size() < batch_max; ring++)
            for (int64_t nw = (int64_t)cw - ring; nw <= (int64_t)cw + ring && ws.size() < batch_max; nw++)
                for (int64_t nr = (int64_t)cr - ring; nr <= (int64_t)cr + ring && ws.size() < batch_max; nr++) {
                    const int64_t dw = nw > (int64_t)cw ? nw - cw : (int64_t)cw - nw, dr = nr > (int64_t)cr ? nr - cr : (int64_t)cr - nr;
                    if ((dw > dr ? dw : dr) != (int64_t)ring) continue;             // only the ring itself
                    if (nw < 1 || nw > (int64_t)sp->w_max || nr < 0 || nr > 10) continue;
                    if (h_table[(size_t)(nw - 1) * 11 + nr] >= 0.0 || ((uint32_t)nw == w && (uint32_t)nr == r10)) continue;
                    ws.push_back((uint32_t)nw); rs.push_back((uint32_t)nr);
                }
        const uint32_t nb = (uint32_t)ws.size();
        const size_t xwords = ((size_t)nb * words + 3) & ~(size_t)3;     // results start 16-byte aligned
        if ((err = kvp_ensure(ctx, (void **)&ctx->d_policy_x, &ctx->policy_x_cap, xwords * 4 + (size_t)nb * 16)))
            return slot;
        double *d_cost = (double *)(ctx->d_policy_x + xwords);
        uint32_t *d_ex = (uint32_t *)(d_cost + nb);
        if ((err = kvp_wr_policy(ctx, nb, ws.data(), rs.data(), ctx->d_policy_x))) return slot;
        if ((err = kvp_score_launch(ctx, ctx->d_policy_x, nb, d_cost, d_ex, nullptr, nullptr))) return slot;
        std::vector<double> hc(nb);
        hipError_t e = hipMemcpyAsync(hc.data(), d_cost, (size_t)nb * 8, hipMemcpyDeviceToHost, ctx->stream);
        if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
        if (e != hipSuccess) { err = KVP_EHIP; return slot; }
        for (uint32_t j = 0; j < nb; j++) h_table[(size_t)(ws[j] - 1) * 11 + rs[j]] = hc[j];
        res->evaluated += nb;
        return slot;
    };
    uint32_t w = sp->w0, r10 = sp->r10_0;
    double T = cost(w, r10, w, r10);
    if (err) return err;
    res->best_w = w; res->best_r10 = r10; res->best_T = T;
    double sum = 0.0;
    uint32_t cnt = 0;
    for (uint64_t j = 0; j < 32; j++) {                                // start temperature from p0
        uint32_t w2, r2; double u;
        if (!propose(*sp, j, 24, w, r10, w2, r2, u)) continue;
        const double dT = cost(w2, r2, w, r10) - T;
        if (err) return err;
        if (dT > 0.0) { sum = sum + dT; cnt++; }
    }
    res->c0 = cnt ? (sum / (double)cnt) / (-log(sp->p0)) : 0.0;
    double C = res->c0, best_at_level_start = res->best_T;
    uint64_t mpl = sp->total_moves / sp->n_levels;
    if (mpl < 1) mpl = 1;
    res->stop_reason = 0;
    for (uint64_t i = 0; i < sp->total_moves; i++) {
        if (i > 0 && i % mpl == 0) {                                   // a level ends
            res->levels_done++;
            if (best_at_level_start - res->best_T < sp->stop_rel * best_at_level_start) { res->stop_reason = 1; break; }
            best_at_level_start = res->best_T;
            C = C * sp->alpha;
            if (C < sp->c_min_frac * res->c0) { res->stop_reason = 2; break; }
        }
        uint32_t w2, r2; double u;
        res->proposals++;
        if (!propose(*sp, i, 16, w, r10, w2, r2, u)) { res->out_of_range++; continue; }
        const double T2 = cost(w2, r2, w, r10);
        if (err) return err;
        const double dT = T2 - T;
        const bool accept = dT <= 0.0 || (C > 0.0 && u < exp(-dT / C));   // Metropolis
        if (!accept) continue;
        res->accepted++;
        w = w2; r10 = r2; T = T2;
        if (T < res->best_T) { res->best_T = T; res->best_w = w; res->best_r10 = r10; }
    }
    res->cur_w = w; res->cur_r10 = r10; res->cur_T = T;
    if (d_best_placement) {
        if (((uintptr_t)d_best_placement & 3u)) return KVP_EINVAL;
        if ((err = kvp_wr_policy(ctx, 1, &res->best_w, &res->best_r10, d_best_placement))) return err;
        KVP_HIP(hipStreamSynchronize(ctx->stream));
    }
    return KVP_OK;
}
