// Selection of the cap items with the largest keys by one workgroup of 1024
// threads (shared by the placement generators).  gfx950 only.
#pragma once

#include "kvp_internal.h"

namespace {

// Division of a word index by the row width without the integer-division sequence: one multiply.
// m = ceil(2^32 / d) gives floor(x / d) = mulhi(x, m) for every x with x * d < 2^32 (the error term
// m * d - 2^32 is below d); wider problems keep m = 0 and divide.
struct RowDiv {
    uint32_t d, m;
    __host__ __device__ RowDiv() : d(1), m(0) {}
    __host__ RowDiv(uint32_t width, uint64_t largest_x) : d(width), m(0) {
        if (width > 1 && largest_x * width < (1ull << 32)) m = (uint32_t)(((1ull << 32) + width - 1) / width);
    }
#ifdef __HIPCC__
    __device__ __forceinline__ uint32_t quot(uint32_t x) const { return m ? __umulhi(x, m) : x / d; }
    __device__ __forceinline__ uint32_t rem(uint32_t x) const { return x - quot(x) * d; }
#endif
};

constexpr int BT = 1024;                 // threads of the selecting workgroup
constexpr int BW = BT / KVP_WAVE;        // its wavefronts
constexpr uint32_t NOT_A_CANDIDATE = 0xFFFFFFFFu;
constexpr int CU = 8;                    // chunks of 64 items whose loads a wavefront keeps in flight

struct SelectShared {
    uint32_t part[BT];                   // partial sums of the histogram scan
    uint32_t wave_ties[BW];
    uint32_t threshold, take_ties, take_all;
};

// From the histogram of the keys to the selection rule: sh.threshold is the smallest key chosen,
// sh.take_ties how many of the items with that key are chosen, sh.take_all whether every item is.
// All BT threads call this together, after a barrier that completes the histogram.
__device__ __forceinline__ void select_threshold(uint32_t nbins, uint64_t cap, const uint32_t *hist, SelectShared &sh) {
    const uint32_t tid = threadIdx.x;
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
}

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
    // CU chunks at a time, so that as many sets of loads are in flight per wavefront (the passes
    // are bound by memory latency: one workgroup has a whole problem's pairs to walk).
    uint32_t n0 = 0, nl = 0;
    for (uint32_t c = c_lo; c < c_hi; c += CU) {
        uint32_t k[CU];
#pragma unroll
        for (int u = 0; u < CU; u++) {
            const uint32_t g = (c + u) * 64 + lane;
            k[u] = (c + u < c_hi && g < G) ? first_key(g) : NOT_A_CANDIDATE;
        }
#pragma unroll
        for (int u = 0; u < CU; u++) {
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
    select_threshold(nbins, cap, hist, sh);
    const uint32_t T = sh.threshold, r = sh.take_ties;
    const bool all = sh.take_all != 0;
    // items at the threshold, counted per wavefront, then numbered in index order
    uint32_t ties = 0;
    if (!all)
        for (uint32_t c = c_lo; c < c_hi; c += CU) {
            uint32_t k[CU];
#pragma unroll
            for (int u = 0; u < CU; u++) {
                const uint32_t g = (c + u) * 64 + lane;
                k[u] = (c + u < c_hi && g < G) ? key(g) : NOT_A_CANDIDATE;
            }
#pragma unroll
            for (int u = 0; u < CU; u++) ties += __popcll(__ballot(k[u] == T));
        }
    if (lane == 0) sh.wave_ties[wave] = ties;
    __syncthreads();
    uint32_t rank0 = 0;
    for (uint32_t w = 0; w < wave; w++) rank0 += sh.wave_ties[w];
    for (uint32_t c0 = c_lo; c0 < c_hi; c0 += CU) {
        uint32_t kk[CU];
#pragma unroll
        for (int u = 0; u < CU; u++) {
            const uint32_t g = (c0 + u) * 64 + lane;
            kk[u] = (c0 + u < c_hi && g < G) ? key(g) : NOT_A_CANDIDATE;
        }
#pragma unroll
        for (int u = 0; u < CU; u++) {
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

// The same selection among the set bits of mask words: item g = 32 * wi + b is a candidate when bit
// b of cand(wi) is set, wi in [0, LW).  key(g) is called for candidates only (three times);
// emit(wi, bits) once per word in which something is chosen, by the lane that owns the word.
// The cost follows the number of candidates, not the number of items.
template <class Cand, class Key, class Emit>
__device__ __forceinline__ void mask_select(uint32_t LW, uint32_t nbins, uint64_t cap, uint32_t *hist, SelectShared &sh,
                                            Cand cand, Key key, Emit emit) {
    const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const uint32_t nchunks = (LW + 63) / 64, cpw = (nchunks + BW - 1) / BW;     // chunks of 64 words per wavefront
    const uint32_t c_lo = min(wave * cpw, nchunks), c_hi = min(c_lo + cpw, nchunks);
    for (uint32_t k = tid; k < nbins; k += BT) hist[k] = 0;
    __syncthreads();
    for (uint32_t c = c_lo; c < c_hi; c++) {
        const uint32_t wi = c * 64 + lane;
        uint32_t m = wi < LW ? cand(wi) : 0;
        while (m) {
            const uint32_t b = __ffs(m) - 1;
            m &= m - 1;
            atomicAdd(&hist[key(wi * 32 + b)], 1u);
        }
    }
    __syncthreads();
    select_threshold(nbins, cap, hist, sh);
    const uint32_t T = sh.threshold, r = sh.take_ties;
    const bool all = sh.take_all != 0;
    uint32_t ties = 0;
    if (!all)
        for (uint32_t c = c_lo; c < c_hi; c++) {
            const uint32_t wi = c * 64 + lane;
            uint32_t m = wi < LW ? cand(wi) : 0;
            while (m) {
                const uint32_t b = __ffs(m) - 1;
                m &= m - 1;
                ties += key(wi * 32 + b) == T;
            }
        }
    ties = wave_sum_u32(ties);
    if (lane == 0) sh.wave_ties[wave] = ties;
    __syncthreads();
    uint32_t rank0 = 0;
    for (uint32_t w = 0; w < wave; w++) rank0 += sh.wave_ties[w];
    for (uint32_t c = c_lo; c < c_hi; c++) {
        const uint32_t wi = c * 64 + lane;
        const uint32_t m0 = wi < LW ? cand(wi) : 0;
        uint32_t chosen = m0;
        if (!all) {
            uint32_t above = 0, tie = 0;
            for (uint32_t m = m0; m;) {
                const uint32_t b = __ffs(m) - 1;
                m &= m - 1;
                const uint32_t k = key(wi * 32 + b);
                above |= (uint32_t)(k > T) << b;
                tie |= (uint32_t)(k == T) << b;
            }
            chosen = above;
            if (__ballot(tie != 0)) {                                  // the same for the whole wavefront
                const uint32_t tc = __popc(tie);
                uint32_t incl = tc;                                    // ties in this and the lower lanes
                for (uint32_t d = 1; d < 64; d <<= 1) {
                    const uint32_t up = __shfl_up(incl, d, KVP_WAVE);
                    if (lane >= d) incl += up;
                }
                uint32_t rank = rank0 + incl - tc;                     // rank of this word's first tie
                for (uint32_t m = tie; m; m &= m - 1, rank++)          // ties below rank r are chosen
                    if (rank < r) chosen |= m & (0u - m);
                rank0 += __shfl(incl, 63, KVP_WAVE);
            }
        }
        if (chosen) emit(wi, chosen);
    }
    __syncthreads();
}

}  // namespace
