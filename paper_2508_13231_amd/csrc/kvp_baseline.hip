// Foresight-free placements to start a search from or to compare it with: a
// static one (the pages read most often over the whole trace stay in HBM for
// as long as they exist; nothing migrates), a recency one (at every token step
// the pool holds the existing pages read most recently, LRU order) and a fill
// one (pages take HBM in the order in which they are written while there is
// room, and never move: the "Static Placement" of the paper's evaluation; see
// fill_kernel).  The first two are
// "the cap_pages (layer, page) pairs with the largest key, ties to the lower
// l * P + p", once for the static placement and once per token step for the
// recency placement; the evaluation section of the paper compares its search with
// a static and a reactive LRU placement of this kind.
//
// The recency keys of a step follow from the trace alone, so all steps are selected at once, a
// workgroup each, from keys written by a pass with a thread per pair.
// One workgroup of 1024 threads makes a selection: a histogram of the keys in
// LDS gives the threshold key and how many of the pairs AT the threshold still
// fit; a second sweep numbers those in index order (wavefront ballots and a scan
// over the 16 wavefronts) and emits the chosen pairs as 32-bit mask words.
// Pairs are walked in the padded order (layer, word, bit), which is the order of
// l * P + p with the unused bits of each layer's last word skipped.
#include "kvp_internal.h"
#include "kvp_select.h"

namespace {

// how often each (layer, page) is read over the trace, summed over the planes: [L][Wd][32]
__global__ __launch_bounds__(256) void read_counts_kernel(DevProblem q, RowDiv rd, uint32_t *__restrict__ freq) {
    const uint32_t g = blockIdx.x * 256 + threadIdx.x;
    if (g >= q.L * q.Wd * 32) return;
    const uint32_t wi = g >> 5, b = g & 31u, l = rd.quot(wi), w = wi - l * q.Wd;
    uint32_t f = 0;
    for (uint32_t n = 0; n < q.N; n++)
        for (uint32_t k = 0; k < q.K; k++) f += (q.A[(((size_t)l * q.N + n) * q.K + k) * q.Wd + w] >> b) & 1u;
    freq[g] = f;
}

__global__ __launch_bounds__(BT) void static_select_kernel(DevProblem q, RowDiv rd, uint64_t cap, uint32_t nbins,
                                                           const uint32_t *__restrict__ freq,
                                                           uint32_t *__restrict__ chosen) {
    extern __shared__ uint32_t lds_u[];
    __shared__ SelectShared sh;
    const uint32_t G = q.L * q.Wd * 32;
    auto key = [&](uint32_t g) {
        const uint32_t w = rd.rem(g >> 5), p = 32 * w + (g & 31u);
        return p < q.P ? freq[g] : NOT_A_CANDIDATE;                    // every pair competes, existing or not
    };
    block_select(G, nbins, cap, lds_u, sh, key, key, [&](uint32_t word, uint32_t bits) { chosen[word] = bits; });
}

__global__ __launch_bounds__(256) void static_fill_kernel(DevProblem q, const uint32_t *__restrict__ chosen,
                                                          uint32_t *__restrict__ X) {
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;           // (l * N + n) * Wd + w
    if (i >= (size_t)q.L * q.N * q.Wd) return;
    const uint32_t w = (uint32_t)(i % q.Wd);
    const size_t ln = i / q.Wd;
    const uint32_t n = (uint32_t)(ln % q.N), l = (uint32_t)(ln / q.N);
    X[i] = chosen[l * q.Wd + w] & q.V[(size_t)n * q.Wd + w];
}

// The recency placement in two passes.  A pair's key at step n (the last step before n at which it was
// read since it last (re)started to persist, plus one; 0 if never) depends on the trace alone, so a thread
// per pair walks the steps [n_lo, n_hi) and writes the keys of all of them, [n - n_lo][G] 16-bit words
// (0xFFFF: the page does not exist at that step); `last` carries the walk from one batch of steps to the
// next.  The selections of the steps are then independent: a workgroup per step.
constexpr uint32_t KEY16_NONE = 0xFFFFu;

__global__ __launch_bounds__(256) void recency_keys_kernel(DevProblem q, RowDiv rd, uint32_t n_lo, uint32_t n_hi,
                                                           int32_t *__restrict__ last, uint16_t *__restrict__ keys) {
    const uint32_t G = q.L * q.Wd * 32;
    const uint32_t g = blockIdx.x * 256 + threadIdx.x;
    if (g >= G) return;
    const uint32_t wi = g >> 5, b = g & 31u, l = rd.quot(wi), w = wi - l * q.Wd;
    int32_t lv = n_lo ? last[g] : -1;
    for (uint32_t n = n_lo; n < n_hi; n++) {
        if (n > 0) {
            if (!((q.Pm[(size_t)n * q.Wd + w] >> b) & 1u)) {
                lv = -1;                                               // a page that stops persisting forgets its history
            } else {
                uint32_t any = 0;
                for (uint32_t k = 0; k < q.K; k++) any |= q.A[(((size_t)l * q.N + (n - 1)) * q.K + k) * q.Wd + w];
                if ((any >> b) & 1u) lv = (int32_t)(n - 1);
            }
        }
        const bool alive = (q.V[(size_t)n * q.Wd + w] >> b) & 1u;      // dead bits of the last word are never alive
        keys[(size_t)(n - n_lo) * G + g] = alive ? (uint16_t)(lv + 1) : (uint16_t)KEY16_NONE;
    }
    last[g] = lv;
}

__global__ __launch_bounds__(BT) void recency_select_kernel(DevProblem q, uint64_t cap, uint32_t n_lo,
                                                            const uint16_t *__restrict__ keys, uint32_t *__restrict__ X) {
    extern __shared__ uint32_t lds_u[];
    __shared__ SelectShared sh;
    const uint32_t G = q.L * q.Wd * 32, n = n_lo + blockIdx.x;
    const uint16_t *kn = keys + (size_t)blockIdx.x * G;
    auto key = [&](uint32_t g) {
        const uint32_t k = kn[g];
        return k == KEY16_NONE ? NOT_A_CANDIDATE : k;
    };
    block_select(G, n + 1, cap, lds_u, sh, key, key, [&](uint32_t word, uint32_t bits) {
        const uint32_t l = word / q.Wd, w = word - l * q.Wd;
        X[((size_t)l * q.N + n) * q.Wd + w] = bits;
    });
}

// Static fill, step after step, in one workgroup.  The state is one mask word per (layer, word):
// the pages now in HBM.  Per step: entries that stop persisting leave (AND with the persist word),
// the survivors are counted, and the pages new at this step take the free places in the order of
// l * P + p: a running count over the words, in chunks of BT words, finds the word at which the room
// ends.  Thread t owns the words t, t + BT, ... in every pass, so the state needs no barrier of its own.
__global__ __launch_bounds__(BT) void fill_kernel(DevProblem q, uint64_t cap, uint32_t *__restrict__ in,
                                                  uint32_t *__restrict__ X) {
    __shared__ uint32_t wave_sum[BW];
    const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const uint32_t NW = q.L * q.Wd;
    // sum over the workgroup (every thread gets it) and, optionally, the sum over the threads before this one
    auto block_scan = [&](uint32_t v, uint32_t *before) {
        uint32_t inc = v;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const uint32_t o = __shfl_up(inc, d, 64);
            if ((int)lane >= d) inc += o;
        }
        __syncthreads();                                               // wave_sum of the previous call is read
        if (lane == 63) wave_sum[wave] = inc;
        __syncthreads();
        uint32_t total = 0, pre = 0;
        for (uint32_t w = 0; w < (uint32_t)BW; w++) {
            const uint32_t x = wave_sum[w];
            if (w < wave) pre += x;
            total += x;
        }
        if (before) *before = pre + inc - v;
        return total;
    };
    for (uint32_t i = tid; i < NW; i += BT) in[i] = 0;
    for (uint32_t n = 0; n < q.N; n++) {
        uint32_t mine = 0;
        for (uint32_t i = tid; i < NW; i += BT) {
            const uint32_t w = i % q.Wd;
            const uint32_t v = n ? in[i] & q.Pm[(size_t)n * q.Wd + w] : 0u;
            in[i] = v;
            mine += __popc(v);
        }
        const uint32_t occ = block_scan(mine, nullptr);
        uint64_t room = cap > occ ? cap - occ : 0;
        for (uint32_t base = 0; base < NW; base += BT) {               // same trip count for every thread
            const uint32_t i = base + tid;
            const bool has = i < NW;
            const uint32_t l = has ? i / q.Wd : 0, w = has ? i - l * q.Wd : 0;
            uint32_t v = has ? in[i] : 0u;
            if (room != 0) {                                           // uniform
                const uint32_t fresh = has ? q.V[(size_t)n * q.Wd + w] & ~(n ? q.Pm[(size_t)n * q.Wd + w] : 0u) : 0u;
                uint32_t before;
                const uint32_t total = block_scan(__popc(fresh), &before);
                uint32_t take = 0;
                if (before + __popc(fresh) <= room) {
                    take = fresh;
                } else if (before < room) {                            // the word at which the room ends
                    uint32_t rest = fresh;
                    for (uint64_t c = room - before; c != 0; c--) { const uint32_t b = rest & (0u - rest); take |= b; rest ^= b; }
                }
                v |= take;
                room -= room < total ? room : total;
            }
            if (has) {
                in[i] = v;
                X[((size_t)l * q.N + n) * q.Wd + w] = v;
            }
        }
    }
}

}  // namespace

extern "C" int kvp_baseline(kvp_ctx *ctx, int kind, uint32_t *d_placement) {
    if (!ctx) return KVP_EINVAL;
    if (!ctx->has_trace) return KVP_ENOTRACE;
    if (!d_placement || ((uintptr_t)d_placement & 3u)) return KVP_EINVAL;
    if (kind != KVP_BASELINE_STATIC && kind != KVP_BASELINE_RECENCY && kind != KVP_BASELINE_FILL) return KVP_EINVAL;
    KVP_HIP(hipSetDevice(ctx->device));
    const DevProblem &q = ctx->dp;
    const uint64_t G64 = (uint64_t)q.L * q.Wd * 32;
    if (G64 >= (1ull << 31)) return KVP_ESHAPE;
    const uint32_t G = (uint32_t)G64;
    const uint64_t cap = ctx->prob.cap_pages;
    const RowDiv rd(q.Wd, (uint64_t)q.L * q.Wd);
    const uint32_t nbins = kind == KVP_BASELINE_STATIC ? q.N * q.K + 1 : kind == KVP_BASELINE_RECENCY ? q.N + 1 : 0;
    const size_t lds = (size_t)nbins * 4;
    if (lds > 128 * 1024) return KVP_ESHAPE;
    int rc = kvp_ensure(ctx, (void **)&ctx->d_cnt_tmp, &ctx->cnt_tmp_cap, (size_t)G * 4 + (size_t)q.L * q.Wd * 4);
    if (rc) return rc;
    uint32_t *work = ctx->d_cnt_tmp;                                   // [G] keys, then [L][Wd] chosen words
    if (kind == KVP_BASELINE_STATIC) {
        uint32_t *chosen = work + G;
        read_counts_kernel<<<dim3((G + 255) / 256), dim3(256), 0, ctx->stream>>>(q, rd, work);
        KVP_HIP(hipGetLastError());
        if (lds > 48 * 1024)
            KVP_HIP(hipFuncSetAttribute((const void *)static_select_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        static_select_kernel<<<dim3(1), dim3(BT), lds, ctx->stream>>>(q, rd, cap, nbins, work, chosen);
        KVP_HIP(hipGetLastError());
        const size_t words = (size_t)q.L * q.N * q.Wd;
        static_fill_kernel<<<dim3((uint32_t)((words + 255) / 256)), dim3(256), 0, ctx->stream>>>(q, chosen, d_placement);
        KVP_HIP(hipGetLastError());
    } else if (kind == KVP_BASELINE_FILL) {
        fill_kernel<<<dim3(1), dim3(BT), 0, ctx->stream>>>(q, cap, work, d_placement);
        KVP_HIP(hipGetLastError());
    } else {
        // batches of steps whose keys fit a gigabyte, or what kvp_set_generator_batch_bytes says (at least one step)
        const uint64_t per_step = (uint64_t)G * sizeof(uint16_t);
        const uint64_t budget = ctx->gen_batch_bytes ? ctx->gen_batch_bytes : (1ull << 30);
        const uint32_t batch = (uint32_t)(per_step >= budget ? 1 : budget / per_step < q.N ? budget / per_step : q.N);
        rc = kvp_ensure(ctx, (void **)&ctx->d_sel_keys, &ctx->sel_keys_cap, (size_t)batch * per_step);
        if (rc) return rc;
        if (lds > 48 * 1024)
            KVP_HIP(hipFuncSetAttribute((const void *)recency_select_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        for (uint32_t n_lo = 0; n_lo < q.N; n_lo += batch) {
            const uint32_t n_hi = n_lo + batch < q.N ? n_lo + batch : q.N;
            recency_keys_kernel<<<dim3((G + 255) / 256), dim3(256), 0, ctx->stream>>>(q, rd, n_lo, n_hi, (int32_t *)work,
                                                                                      (uint16_t *)ctx->d_sel_keys);
            KVP_HIP(hipGetLastError());
            recency_select_kernel<<<dim3(n_hi - n_lo), dim3(BT), lds, ctx->stream>>>(q, cap, n_lo, (const uint16_t *)ctx->d_sel_keys,
                                                                                   d_placement);
            KVP_HIP(hipGetLastError());
        }
    }
    return KVP_OK;
}
