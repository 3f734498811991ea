// Token permutation that groups routed rows by expert (the per-expert inputs of paper
// Section 3.1): a stable counting sort of flat ids i = t*k + s by expert, built from
// per-wavefront histograms, one scan, and an in-wavefront stable rank. Integer only and
// bit-exact; no atomic operation decides a position.
//
// A wavefront owns 256 consecutive ids ("segment"), visited in 4 rounds of 64; lane e keeps the
// running count of expert e (E <= 64).
//   1. hist   : seg_hist[g][e] = ids of segment g routed to e          (ballot + popcount)
//   2. scan   : counts, offsets, and seg_base[g][e] = offsets[e] + sum_{g'<g} seg_hist[g'][e]
//   3. scatter: position = seg_base[g][e] + rank of the id among equal experts in the segment
// Ids whose expert index is outside [0,E) are dropped (inv_perm = -1).
#include "common.h"

namespace moe {
namespace {

constexpr int kSegIds = 256;                 // ids per wavefront segment
constexpr int kRounds = kSegIds / kWave;     // 4
constexpr int kBlockWaves = 4;

__device__ __forceinline__ uint64_t lanemask_lt(int lane) { return (1ull << lane) - 1ull; }

__global__ __launch_bounds__(kBlockWaves* kWave) void hist_kernel(
    const int32_t* __restrict__ topk_idx, int R, int E, int32_t* __restrict__ seg_hist) {
    const int lane = threadIdx.x & (kWave - 1);
    const int seg = blockIdx.x * kBlockWaves + (threadIdx.x / kWave);
    const int64_t base = static_cast<int64_t>(seg) * kSegIds;
    if (base >= R) return;
    int cnt = 0;
    for (int r = 0; r < kRounds; ++r) {
        const int64_t i = base + r * kWave + lane;
        const int my = (i < R) ? topk_idx[i] : -1;
        for (int e = 0; e < E; ++e) {
            const uint64_t b = __ballot(my == e);
            if (lane == e) cnt += __popcll(b);
        }
    }
    if (lane < E) seg_hist[static_cast<size_t>(seg) * E + lane] = cnt;
}

// One block of 1024 threads (16 wavefronts). Wavefront w scans the columns e = w, w+16, ...
__global__ __launch_bounds__(1024) void scan_kernel(const int32_t* __restrict__ seg_hist,
                                                    int nseg, int E, int32_t* __restrict__ counts,
                                                    int32_t* __restrict__ offsets,
                                                    int32_t* __restrict__ seg_base) {
    __shared__ int32_t tot[kMaxExperts];
    __shared__ int32_t off[kMaxExperts + 1];
    const int lane = threadIdx.x & (kWave - 1);
    const int w = threadIdx.x / kWave;
    for (int e = w; e < E; e += 16) {
        int sum = 0;
        for (int g = lane; g < nseg; g += kWave) sum += seg_hist[static_cast<size_t>(g) * E + e];
        for (int s = 32; s >= 1; s >>= 1) sum += __shfl_xor(sum, s, kWave);
        if (lane == 0) tot[e] = sum;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        int run = 0;
        for (int e = 0; e < E; ++e) {
            off[e] = run;
            counts[e] = tot[e];
            offsets[e] = run;
            run += tot[e];
        }
        off[E] = run;
        offsets[E] = run;
    }
    __syncthreads();
    for (int e = w; e < E; e += 16) {
        int carry = off[e];
        for (int g0 = 0; g0 < nseg; g0 += kWave) {
            const int g = g0 + lane;
            const int v = (g < nseg) ? seg_hist[static_cast<size_t>(g) * E + e] : 0;
            int incl = v;                                  // inclusive prefix over the 64 lanes
            for (int s = 1; s < kWave; s <<= 1) {
                const int up = __shfl_up(incl, s, kWave);
                if (lane >= s) incl += up;
            }
            if (g < nseg) seg_base[static_cast<size_t>(g) * E + e] = carry + incl - v;
            carry += __shfl(incl, kWave - 1, kWave);
        }
    }
}

__global__ __launch_bounds__(kBlockWaves* kWave) void scatter_kernel(
    const int32_t* __restrict__ topk_idx, int R, int E, const int32_t* __restrict__ seg_base,
    int32_t* __restrict__ perm, int32_t* __restrict__ inv_perm) {
    const int lane = threadIdx.x & (kWave - 1);
    const int seg = blockIdx.x * kBlockWaves + (threadIdx.x / kWave);
    const int64_t base = static_cast<int64_t>(seg) * kSegIds;
    if (base >= R) return;
    int run = (lane < E) ? seg_base[static_cast<size_t>(seg) * E + lane] : 0;
    for (int r = 0; r < kRounds; ++r) {
        const int64_t i = base + r * kWave + lane;
        const int my = (i < R) ? topk_idx[i] : -1;
        int pos = -1;
        for (int e = 0; e < E; ++e) {
            const uint64_t b = __ballot(my == e);
            const int base_e = __shfl(run, e, kWave);
            if (my == e) pos = base_e + __popcll(b & lanemask_lt(lane));
            if (lane == e) run += __popcll(b);
        }
        if (i < R) {
            inv_perm[i] = pos;
            if (pos >= 0) perm[pos] = static_cast<int32_t>(i);
        }
    }
}

// One block per permuted row: x_perm[p,:] = x[perm[p] / k, :], 16 bytes per lane per step.
// Rows at or past *n_grouped (ids dropped for an out-of-range expert index) are zero-filled.
__global__ __launch_bounds__(256) void gather_kernel(const uint16_t* __restrict__ x,
                                                     const int32_t* __restrict__ perm,
                                                     const int32_t* __restrict__ n_grouped, int d,
                                                     int k, uint16_t* __restrict__ x_perm) {
    const int p = blockIdx.x;
    uint4* dst = reinterpret_cast<uint4*>(x_perm + static_cast<size_t>(p) * d);
    if (p >= *n_grouped) {
        for (int c = threadIdx.x; c < d / 8; c += blockDim.x) dst[c] = make_uint4(0, 0, 0, 0);
        return;
    }
    const int t = perm[p] / k;
    const uint4* src = reinterpret_cast<const uint4*>(x + static_cast<size_t>(t) * d);
    for (int c = threadIdx.x; c < d / 8; c += blockDim.x) dst[c] = src[c];
}

}  // namespace

size_t permute_scratch_ints(int R_max, int E) {
    const size_t nseg = (static_cast<size_t>(R_max) + kSegIds - 1) / kSegIds;
    return 2 * nseg * static_cast<size_t>(E);           // seg_hist + seg_base
}

int launch_permute(const int32_t* topk_idx, int R, int E, int32_t* counts, int32_t* offsets,
                   int32_t* perm, int32_t* inv_perm, int32_t* scratch, hipStream_t s) {
    const int nseg = (R + kSegIds - 1) / kSegIds;
    int32_t* seg_hist = scratch;
    int32_t* seg_base = scratch + static_cast<size_t>(nseg) * E;
    const int blocks = (nseg + kBlockWaves - 1) / kBlockWaves;
    if (nseg > 0)
        hipLaunchKernelGGL(hist_kernel, dim3(blocks), dim3(kBlockWaves * kWave), 0, s, topk_idx, R,
                           E, seg_hist);
    hipLaunchKernelGGL(scan_kernel, dim3(1), dim3(1024), 0, s, seg_hist, nseg, E, counts, offsets,
                       seg_base);
    if (nseg > 0)
        hipLaunchKernelGGL(scatter_kernel, dim3(blocks), dim3(kBlockWaves * kWave), 0, s, topk_idx,
                           R, E, seg_base, perm, inv_perm);
    return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

int launch_gather(const moe_bf16* x, const int32_t* perm, const int32_t* offsets, int R, int d,
                  int k, int E, moe_bf16* x_perm, hipStream_t s) {
    if (R == 0) return MOE_OK;
    hipLaunchKernelGGL(gather_kernel, dim3(R), dim3(256), 0, s, x, perm, offsets + E, d, k, x_perm);
    return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

}  // namespace moe
