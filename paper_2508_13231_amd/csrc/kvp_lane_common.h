// Pieces shared by the narrow-row scorers (one lane per row): tile shape and the
// staging of contiguous row chunks through registers into LDS.  gfx950 only.
#pragma once

#include "kvp_internal.h"

namespace {

constexpr int TILE_N = 64;     // token steps per tile = lanes per wavefront
constexpr int TB_STRIDE = 65;  // doubles per layer in the latency buffer (odd: spreads LDS banks)

template <int NV>
struct Staged { uint4 v[NV]; };

// Issue the loads of `cnt` words starting at base[start] as whole 16-byte vectors
// from the aligned address below `start` (all arguments wavefront-uniform).
// If the last vector would cross `total`, the end of the array, the chunk is
// fetched word by word instead: that only ever happens for the array's last chunk.
template <int NV>
__device__ __forceinline__ void stage_load(Staged<NV> &st, const uint32_t *__restrict__ base, size_t start,
                                           uint32_t cnt, size_t total, int lane, uint32_t &shift, uint32_t &nvec) {
    const size_t a0 = start & ~(size_t)3;
    shift = (uint32_t)(start - a0);
    nvec = (shift + cnt + 3) >> 2;
    const uint32_t *p = base + a0;
    if (a0 + 4 * (size_t)nvec <= total) {
#pragma unroll
        for (int j = 0; j < NV; j++) {
            const uint32_t vi = (uint32_t)lane + 64u * j;
            if (vi < nvec) st.v[j] = *(const uint4 *)(p + 4 * vi);
        }
    } else {
        const uint32_t left = (uint32_t)(total - a0);
#pragma unroll
        for (int j = 0; j < NV; j++) {
            const uint32_t w = 4 * ((uint32_t)lane + 64u * j);
            uint4 r = make_uint4(0, 0, 0, 0);
            if (w + 0 < left) r.x = p[w + 0];
            if (w + 1 < left) r.y = p[w + 1];
            if (w + 2 < left) r.z = p[w + 2];
            if (w + 3 < left) r.w = p[w + 3];
            st.v[j] = r;
        }
    }
}

template <int NV>
__device__ __forceinline__ void stage_commit(const Staged<NV> &st, uint32_t *lds, uint32_t nvec, int lane) {
#pragma unroll
    for (int j = 0; j < NV; j++) {
        const uint32_t vi = (uint32_t)lane + 64u * j;
        if (vi < nvec) *(uint4 *)(lds + 4 * vi) = st.v[j];
    }
}

constexpr int vecs_per_lane(int words) { return ((words + 3 + 3) / 4 + 63) / 64; }


}  // namespace
