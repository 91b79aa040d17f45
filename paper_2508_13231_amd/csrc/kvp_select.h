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

// The 32 keys of a mask word, fetched as whole 16-byte vectors (the key of item g is f[g], so a word's
// keys are 32 consecutive elements; f + 32 * wi must be 16-byte aligned).
template <class FT>
struct WordKeys {
    static constexpr int NV = (int)sizeof(FT) * 2;      // vectors
    uint4 v[NV];
    __device__ __forceinline__ void load(const FT *f, uint32_t wi) {
        const uint4 *p = (const uint4 *)(f + (size_t)wi * 32);
#pragma unroll
        for (int j = 0; j < NV; j++) v[j] = p[j];
    }
    // key of bit b, b different from lane to lane: the vectors are halved log2(2 NV) times by selects on
    // the bits of the key's byte offset (no register indexing), then one 64-bit shift picks the key
    __device__ __forceinline__ uint32_t get(uint32_t b) const {
        constexpr int NP = NV * 2;                          // 64-bit pieces
        uint64_t p[NP];
#pragma unroll
        for (int j = 0; j < NV; j++) {
            p[2 * j] = ((uint64_t)v[j].y << 32) | v[j].x;
            p[2 * j + 1] = ((uint64_t)v[j].w << 32) | v[j].z;
        }
        const uint32_t byte = b * (uint32_t)sizeof(FT);
#pragma unroll
        for (int half = NP / 2, bit = 8; half >= 1; half >>= 1, bit <<= 1) {
            const bool hi = byte & (uint32_t)bit;           // pieces are interleaved: piece i covers bytes 8i .. 8i+7
#pragma unroll
            for (int i = 0; i < half; i++) p[i] = hi ? p[2 * i + 1] : p[2 * i];
        }
        const uint64_t s = p[0] >> ((byte & 7u) * 8u);
        return sizeof(FT) == 4 ? (uint32_t)s : (uint32_t)s & ((1u << (8 * (sizeof(FT) % 4))) - 1u);
    }
};

}  // namespace
