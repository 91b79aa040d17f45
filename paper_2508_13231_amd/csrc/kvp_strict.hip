// Occupancy counted after every (token step, layer) slot (Eq. 5 read strictly).
//
// The layers of a token step change their placement one after the other, each at its own slot
// (n, l).  After slot (n, l) the pool holds the step-n placement of layers 0..l and still the
// step-(n-1) placement of layers l+1..L-1, less the pages that do not persist into step n:
//
//     occ(n, l) = sum_{l' <= l} |X[l'][n] & alive[n]|  +  sum_{l' > l} |X[l'][n-1] & persist[n]|
//
// One wavefront per (schedule, token step): the lanes walk the L * Wd words of the two steps,
// per-layer counts are gathered in LDS, and a prefix sum over the layers (new placements) against
// a suffix sum (old ones) gives every slot's occupancy; the largest overshoot of a schedule is
// merged with an atomic maximum.  gfx950 only.
#include "kvp_internal.h"

namespace {

constexpr int SW = 4;          // wavefronts (= (schedule, step) pairs) per workgroup

__global__ __launch_bounds__(256) void fill_u32_kernel(uint32_t *p, uint32_t n, uint32_t v) {
    const uint32_t i = blockIdx.x * 256 + threadIdx.x;
    if (i < n) p[i] = v;
}

// table (may be null): [S][L][N], the pool after every slot
__global__ __launch_bounds__(SW * KVP_WAVE) void strict_excess_kernel(DevProblem q, const uint32_t *__restrict__ X,
                                                                      uint32_t S, uint32_t *__restrict__ excess,
                                                                      uint32_t *__restrict__ table) {
    extern __shared__ uint32_t lds_u[];                                // [SW][2][L]
    const int lane = lane_id();
    const uint32_t wave = threadIdx.x / KVP_WAVE;
    const uint64_t pair = (uint64_t)blockIdx.x * SW + wave;            // (s, n)
    if (pair >= (uint64_t)S * q.N) return;                             // whole wavefronts leave; no workgroup barrier below
    const uint32_t s = (uint32_t)(pair / q.N), n = (uint32_t)(pair - (uint64_t)s * q.N);
    const uint32_t L = q.L, Wd = q.Wd;
    uint32_t *cnt_new = lds_u + (size_t)wave * 2 * L, *cnt_old = cnt_new + L;
    for (uint32_t l = lane; l < L; l += KVP_WAVE) { cnt_new[l] = 0; cnt_old[l] = 0; }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    const uint32_t *Xs = X + (size_t)s * L * q.N * Wd;
    for (uint32_t i = lane; i < L * Wd; i += KVP_WAVE) {
        const uint32_t l = i / Wd, w = i - l * Wd;
        const size_t o = ((size_t)l * q.N + n) * Wd + w;
        const uint32_t now = Xs[o] & q.V[(size_t)n * Wd + w];
        const uint32_t before = n ? Xs[o - Wd] & q.Pm[(size_t)n * Wd + w] : 0u;   // the old placement of what persists
        if (now) atomicAdd(&cnt_new[l], (uint32_t)__popc(now));
        if (before) atomicAdd(&cnt_old[l], (uint32_t)__popc(before));
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    uint32_t old_total = 0;
    for (uint32_t l = lane; l < L; l += KVP_WAVE) old_total += cnt_old[l];
    old_total = wave_sum_u32(old_total);
    uint32_t worst = 0, new_before = 0, old_before = 0;               // sums over the layers of earlier chunks
    for (uint32_t base = 0; base < L; base += KVP_WAVE) {
        const uint32_t l = base + (uint32_t)lane;
        const uint32_t a = l < L ? cnt_new[l] : 0u, b = l < L ? cnt_old[l] : 0u;
        const uint32_t a_in = wave_incl_scan_u32(a) + new_before, b_in = wave_incl_scan_u32(b) + old_before;
        if (l < L) {
            const uint32_t o = a_in + (old_total - b_in);               // slot (n, l)
            worst = max(worst, o);
            if (table) table[((size_t)s * L + l) * q.N + n] = o;
        }
        new_before = (uint32_t)__builtin_amdgcn_readlane((int)a_in, 63);
        old_before = (uint32_t)__builtin_amdgcn_readlane((int)b_in, 63);
    }
    worst = wave_max_u32(worst);
    const uint32_t over = worst > q.cap ? worst - q.cap : 0u;
    if (lane == 0 && over) atomicMax(&excess[s], over);
}

}  // namespace

// d_excess [S] and, if not null, d_table [S][L][N]; arguments checked by the caller
int kvp_slot_occupancy_launch(kvp_ctx *ctx, const uint32_t *d_placements, uint32_t S, uint32_t *d_excess, uint32_t *d_table) {
    const DevProblem &q = ctx->dp;
    const size_t lds = (size_t)SW * 2 * q.L * 4;
    if (lds > 64 * 1024 || (uint64_t)q.L * q.Wd >= (1ull << 31)) return KVP_ESHAPE;
    const uint64_t pairs = (uint64_t)S * q.N, nwg = (pairs + SW - 1) / SW;
    if (nwg > 0x7FFFFFFFull) return KVP_ESHAPE;
    fill_u32_kernel<<<dim3((S + 255) / 256), dim3(256), 0, ctx->stream>>>(d_excess, S, 0u);
    KVP_HIP(hipGetLastError());
    if (lds > 48 * 1024)
        KVP_HIP(hipFuncSetAttribute((const void *)strict_excess_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    strict_excess_kernel<<<dim3((uint32_t)nwg), dim3(SW * KVP_WAVE), lds, ctx->stream>>>(q, d_placements, S, d_excess, d_table);
    KVP_HIP(hipGetLastError());
    return KVP_OK;
}

extern "C" int kvp_strict_excess(kvp_ctx *ctx, const uint32_t *d_placements, uint32_t S, uint32_t *d_excess) {
    if (!ctx) return KVP_EINVAL;
    if (!ctx->has_trace) return KVP_ENOTRACE;
    if (S == 0) return KVP_OK;
    if (!d_placements || !d_excess || ((uintptr_t)d_placements & 3u) || ((uintptr_t)d_excess & 3u)) return KVP_EINVAL;
    KVP_HIP(hipSetDevice(ctx->device));
    return kvp_slot_occupancy_launch(ctx, d_placements, S, d_excess, nullptr);
}
