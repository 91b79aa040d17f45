// Two foresight-free placements to start a search from or to compare it with:
// a static one (the pages read most often over the whole trace stay in HBM for
// as long as they exist; nothing migrates) and a recency one (at every token step
// the pool holds the existing pages read most recently, LRU order).  Both are
// "the cap_pages (layer, page) pairs with the largest key, ties to the lower
// l * P + p", once for the static placement and once per token step for the
// recency placement; the evaluation section of the paper compares its search with
// a static and a reactive LRU placement of this kind.
//
// One workgroup of 1024 threads makes a selection: a histogram of the keys in
// LDS gives the threshold key and how many of the pairs AT the threshold still
// fit; a second sweep numbers those in index order (wavefront ballots and a scan
// over the 16 wavefronts) and emits the chosen pairs as 32-bit mask words.
// Pairs are walked in the padded order (layer, word, bit), which is the order of
// l * P + p with the unused bits of each layer's last word skipped.
#include "kvp_internal.h"

namespace {

constexpr int BT = 1024;                 // threads of the selecting workgroup
constexpr int BW = BT / KVP_WAVE;        // its wavefronts
constexpr uint32_t NOT_A_CANDIDATE = 0xFFFFFFFFu;

struct SelectShared {
    uint32_t part[BT];                   // partial sums of the histogram scan
    uint32_t wave_ties[BW];
    uint32_t threshold, take_ties, take_all;
};

// Among the items g in [0, G) whose key(g) is not NOT_A_CANDIDATE, choose the `cap` with the
// largest keys (keys < nbins; ties: lower g first).  first_key(g) is called once per item before
// anything else (it may update state and returns the key); key(g) afterwards, twice.  Every 32
// consecutive items form a word: emit(word, bits) is called once per word by one lane.
// All BT threads must call this together; hist holds nbins words of LDS.
template <class FirstKey, class Key, class Emit>
__device__ __forceinline__ void block_select(uint32_t G, uint32_t nbins, uint64_t cap, uint32_t *hist, SelectShared &sh,
                                             FirstKey first_key, Key key, Emit emit) {
    const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const uint32_t nchunks = (G + 63) / 64, cpw = (nchunks + BW - 1) / BW;     // chunks of 64 items per wavefront
    const uint32_t c_lo = min(wave * cpw, nchunks), c_hi = min(c_lo + cpw, nchunks);
    for (uint32_t k = tid; k < nbins; k += BT) hist[k] = 0;
    __syncthreads();
    // keys into the histogram; the two most crowded bins (0 and the last) are counted with ballots.
    // Four chunks at a time, so that four sets of loads are in flight per wavefront.
    uint32_t n0 = 0, nl = 0;
    for (uint32_t c = c_lo; c < c_hi; c += 4) {
        uint32_t k[4];
#pragma unroll
        for (int u = 0; u < 4; u++) {
            const uint32_t g = (c + u) * 64 + lane;
            k[u] = (c + u < c_hi && g < G) ? first_key(g) : NOT_A_CANDIDATE;
        }
#pragma unroll
        for (int u = 0; u < 4; u++) {
            n0 += __popcll(__ballot(k[u] == 0));
            nl += __popcll(__ballot(k[u] == nbins - 1 && k[u] != 0));
            if (k[u] != NOT_A_CANDIDATE && k[u] != 0 && k[u] != nbins - 1) atomicAdd(&hist[k[u]], 1u);
        }
    }
    if (lane == 0) {
        if (n0) atomicAdd(&hist[0], n0);
        if (nl) atomicAdd(&hist[nbins - 1], nl);
    }
    __syncthreads();
    // suffix sums over the bins: thread t owns bins [t * bpt, (t + 1) * bpt)
    const uint32_t bpt = (nbins + BT - 1) / BT;
    const uint32_t b_lo = min(tid * bpt, nbins), b_hi = min(b_lo + bpt, nbins);
    uint32_t mine = 0;
    for (uint32_t k = b_lo; k < b_hi; k++) mine += hist[k];
    sh.part[tid] = mine;
    __syncthreads();
    for (uint32_t d = 1; d < BT; d <<= 1) {                            // inclusive scan from the top
        const uint32_t add = tid + d < BT ? sh.part[tid + d] : 0;
        __syncthreads();
        sh.part[tid] += add;
        __syncthreads();
    }
    if (tid == 0) {
        sh.take_all = (uint64_t)sh.part[0] <= cap;                     // everything that exists fits
        if (cap == 0) { sh.threshold = nbins; sh.take_ties = 0; }     // nothing is chosen
    }
    const uint32_t above_me = tid + 1 < BT ? sh.part[tid + 1] : 0;     // items in bins above this thread's
    if (cap > 0 && (uint64_t)sh.part[tid] >= cap && (uint64_t)above_me < cap) {
        uint32_t acc = above_me;                                       // the threshold lies in this thread's bins
        for (uint32_t k = b_hi; k-- > b_lo;) {
            if ((uint64_t)acc + hist[k] >= cap) { sh.threshold = k; sh.take_ties = (uint32_t)(cap - acc); break; }
            acc += hist[k];
        }
    }
    __syncthreads();
    const uint32_t T = sh.threshold, r = sh.take_ties;
    const bool all = sh.take_all != 0;
    // items at the threshold, counted per wavefront, then numbered in index order
    uint32_t ties = 0;
    if (!all)
        for (uint32_t c = c_lo; c < c_hi; c += 4) {
            uint32_t k[4];
#pragma unroll
            for (int u = 0; u < 4; u++) {
                const uint32_t g = (c + u) * 64 + lane;
                k[u] = (c + u < c_hi && g < G) ? key(g) : NOT_A_CANDIDATE;
            }
#pragma unroll
            for (int u = 0; u < 4; u++) ties += __popcll(__ballot(k[u] == T));
        }
    if (lane == 0) sh.wave_ties[wave] = ties;
    __syncthreads();
    uint32_t rank0 = 0;
    for (uint32_t w = 0; w < wave; w++) rank0 += sh.wave_ties[w];
    for (uint32_t c0 = c_lo; c0 < c_hi; c0 += 4) {
        uint32_t kk[4];
#pragma unroll
        for (int u = 0; u < 4; u++) {
            const uint32_t g = (c0 + u) * 64 + lane;
            kk[u] = (c0 + u < c_hi && g < G) ? key(g) : NOT_A_CANDIDATE;
        }
#pragma unroll
        for (int u = 0; u < 4; u++) {
            const uint32_t c = c0 + u, k = kk[u];
            if (c >= c_hi) break;                                      // the same for the whole wavefront
            const uint64_t tie = __ballot(k == T);
            const uint32_t rank = rank0 + __popcll(tie & ((1ull << lane) - 1ull));
            const bool chosen = k != NOT_A_CANDIDATE && (all || k > T || (k == T && rank < r));
            rank0 += __popcll(tie);
            const uint64_t bits = __ballot(chosen);
            if (lane == 0) emit(2 * c, (uint32_t)bits);
            if (lane == 32 && (2 * c + 1) * 32 < G) emit(2 * c + 1, (uint32_t)(bits >> 32));
        }
    }
    __syncthreads();
}

// how often each (layer, page) is read over the trace, summed over the planes: [L][Wd][32]
__global__ __launch_bounds__(256) void read_counts_kernel(DevProblem q, uint32_t *__restrict__ freq) {
    const uint32_t g = blockIdx.x * 256 + threadIdx.x;
    if (g >= q.L * q.Wd * 32) return;
    const uint32_t wi = g >> 5, b = g & 31u, l = wi / q.Wd, w = wi - l * q.Wd;
    uint32_t f = 0;
    for (uint32_t n = 0; n < q.N; n++)
        for (uint32_t k = 0; k < q.K; k++) f += (q.A[(((size_t)l * q.N + n) * q.K + k) * q.Wd + w] >> b) & 1u;
    freq[g] = f;
}

__global__ __launch_bounds__(BT) void static_select_kernel(DevProblem q, uint64_t cap, uint32_t nbins,
                                                           const uint32_t *__restrict__ freq,
                                                           uint32_t *__restrict__ chosen) {
    extern __shared__ uint32_t lds_u[];
    __shared__ SelectShared sh;
    const uint32_t G = q.L * q.Wd * 32;
    auto key = [&](uint32_t g) {
        const uint32_t w = (g >> 5) % q.Wd, p = 32 * w + (g & 31u);
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

// the whole recency placement, step after step, in one workgroup: last[g] = last step at which the
// pair was read since it last (re)started to persist, -1 if never
__global__ __launch_bounds__(BT) void recency_kernel(DevProblem q, uint64_t cap, int32_t *__restrict__ last,
                                                     uint32_t *__restrict__ X) {
    extern __shared__ uint32_t lds_u[];
    __shared__ SelectShared sh;
    const uint32_t G = q.L * q.Wd * 32;
    for (uint32_t g = threadIdx.x; g < G; g += BT) last[g] = -1;
    __syncthreads();
    for (uint32_t n = 0; n < q.N; n++) {
        auto key = [&](uint32_t g) {
            const uint32_t w = (g >> 5) % q.Wd, b = g & 31u;
            const uint32_t vw = q.V[(size_t)n * q.Wd + w];             // dead bits of the last word are never alive
            int32_t lv = last[g];
            asm volatile("" : "+v"(lv));                               // loaded whether alive or not: no branch, loads overlap
            return ((vw >> b) & 1u) ? (uint32_t)(lv + 1) : NOT_A_CANDIDATE;
        };
        auto first_key = [&](uint32_t g) {
            if (n > 0) {
                const uint32_t wi = g >> 5, b = g & 31u, l = wi / q.Wd, w = wi - l * q.Wd;
                if (!((q.Pm[(size_t)n * q.Wd + w] >> b) & 1u)) {
                    last[g] = -1;                                      // a page that stops persisting forgets its history
                } else {
                    uint32_t any = 0;
                    for (uint32_t k = 0; k < q.K; k++) any |= q.A[(((size_t)l * q.N + (n - 1)) * q.K + k) * q.Wd + w];
                    if ((any >> b) & 1u) last[g] = (int32_t)(n - 1);
                }
            }
            return key(g);
        };
        block_select(G, n + 1, cap, lds_u, sh, first_key, key, [&](uint32_t word, uint32_t bits) {
            const uint32_t l = word / q.Wd, w = word - l * q.Wd;
            X[((size_t)l * q.N + n) * q.Wd + w] = bits;
        });
    }
}

}  // namespace

extern "C" int kvp_baseline(kvp_ctx *ctx, int kind, uint32_t *d_placement) {
    if (!ctx) return KVP_EINVAL;
    if (!ctx->has_trace) return KVP_ENOTRACE;
    if (!d_placement || ((uintptr_t)d_placement & 3u)) return KVP_EINVAL;
    if (kind != KVP_BASELINE_STATIC && kind != KVP_BASELINE_RECENCY) return KVP_EINVAL;
    KVP_HIP(hipSetDevice(ctx->device));
    const DevProblem &q = ctx->dp;
    const uint64_t G64 = (uint64_t)q.L * q.Wd * 32;
    if (G64 >= (1ull << 31)) return KVP_ESHAPE;
    const uint32_t G = (uint32_t)G64;
    const uint64_t cap = ctx->prob.cap_pages;
    const uint32_t nbins = kind == KVP_BASELINE_STATIC ? q.N * q.K + 1 : q.N + 1;
    const size_t lds = (size_t)nbins * 4;
    if (lds > 128 * 1024) return KVP_ESHAPE;
    int rc = kvp_ensure(ctx, (void **)&ctx->d_cnt_tmp, &ctx->cnt_tmp_cap, (size_t)G * 4 + (size_t)q.L * q.Wd * 4);
    if (rc) return rc;
    uint32_t *work = ctx->d_cnt_tmp;                                   // [G] keys, then [L][Wd] chosen words
    if (kind == KVP_BASELINE_STATIC) {
        uint32_t *chosen = work + G;
        read_counts_kernel<<<dim3((G + 255) / 256), dim3(256), 0, ctx->stream>>>(q, work);
        KVP_HIP(hipGetLastError());
        if (lds > 48 * 1024)
            KVP_HIP(hipFuncSetAttribute((const void *)static_select_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        static_select_kernel<<<dim3(1), dim3(BT), lds, ctx->stream>>>(q, cap, nbins, work, chosen);
        KVP_HIP(hipGetLastError());
        const size_t words = (size_t)q.L * q.N * q.Wd;
        static_fill_kernel<<<dim3((uint32_t)((words + 255) / 256)), dim3(256), 0, ctx->stream>>>(q, chosen, d_placement);
        KVP_HIP(hipGetLastError());
    } else {
        if (lds > 48 * 1024)
            KVP_HIP(hipFuncSetAttribute((const void *)recency_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        recency_kernel<<<dim3(1), dim3(BT), lds, ctx->stream>>>(q, cap, (int32_t *)work, d_placement);
        KVP_HIP(hipGetLastError());
    }
    return KVP_OK;
}
