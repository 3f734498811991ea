// Token permutation that groups routed rows by expert (the per-expert inputs of paper
// Section 3.1): a stable counting sort of flat ids i = t*k + s by expert, built from
// per-wavefront histograms, one scan, and an in-wavefront stable rank. Integer only and
// bit-exact; no atomic operation decides a position.
//
// A wavefront owns 256 consecutive ids ("segment"), visited in 4 rounds of 64; lane l keeps the
// running counts of experts l, l+64, l+128, l+192 (E <= 256).
//   1. hist   : seg_hist[g][e] = ids of segment g routed to e          (ballot + popcount)
//   2. scan   : counts, offsets, and seg_base[g][e] = offsets[e] + sum_{g'<g} seg_hist[g'][e]
//               (one block; experts across lanes, slices of the segment range side by side)
//   3. scatter: position = seg_base[g][e] + rank of the id among equal experts in the segment
// Ids whose expert index is outside [0,E) are dropped (inv_perm = -1).
// Up to 4096 ids the three steps run in one workgroup (permute_small_kernel).
#include <mutex>

#include "common.h"

// Segment tables of moe_permute_static(): device memory that exists from load time, so that the
// call allocates nothing. 2 * kStaticTableInts ints (histograms, then start positions).
constexpr size_t kStaticTableInts = 65536;
static __device__ __align__(256) int32_t scratch[2 * kStaticTableInts];

namespace moe {
namespace {

constexpr int kSegIds = 256;                 // ids per wavefront segment
constexpr int kRounds = kSegIds / kWave;     // 4
constexpr int kBlockWaves = 4;
constexpr int kExpertWords = kMaxExperts / kWave;   // experts per lane: 4

__device__ __forceinline__ uint64_t lanemask_lt(int lane) { return (1ull << lane) - 1ull; }

// Lanes of the wavefront that hold the same value as this lane (values in [0, 256), or -1 for
// "none", which matches nothing): one ballot per bit of the value instead of one per expert.
__device__ __forceinline__ uint64_t same_value_lanes(int my) {
    uint64_t m = __ballot(my >= 0);
#pragma unroll
    for (int b = 0; b < 8; ++b) {
        const uint64_t bit = __ballot((my >> b) & 1);
        m &= ((my >> b) & 1) ? bit : ~bit;
    }
    return my >= 0 ? m : 0ull;
}

// The same histogram for many experts (E > 16): every round finds the lanes that share an
// expert with 8 ballots, and the first lane of each such set adds the set's size to a
// wavefront-private table in LDS (one writer per expert and round: no atomics needed).
__global__ __launch_bounds__(kBlockWaves* kWave) void hist_many_kernel(
    const int32_t* __restrict__ topk_idx, int R, int E, int32_t* __restrict__ seg_hist) {
    __shared__ int32_t table[kBlockWaves][kMaxExperts];
    const int lane = threadIdx.x & (kWave - 1);
    const int wv = threadIdx.x / kWave;
    const int seg = blockIdx.x * kBlockWaves + wv;
    const int64_t base = static_cast<int64_t>(seg) * kSegIds;
    if (base >= R) return;
    volatile int32_t* cnt = table[wv];      // read and written across lanes: never cached
    for (int e = lane; e < E; e += kWave) cnt[e] = 0;
    for (int r = 0; r < kRounds; ++r) {
        const int64_t i = base + r * kWave + lane;
        int my = (i < R) ? topk_idx[i] : -1;
        if (my < 0 || my >= E) my = -1;
        const uint64_t same = same_value_lanes(my);
        if (my >= 0 && (same & lanemask_lt(lane)) == 0) cnt[my] += __popcll(same);
        __builtin_amdgcn_wave_barrier();    // rounds stay in order for the compiler too
    }
    for (int e = lane; e < E; e += kWave) seg_hist[static_cast<size_t>(seg) * E + e] = cnt[e];
}

__global__ __launch_bounds__(kBlockWaves* kWave) void hist_kernel(
    const int32_t* __restrict__ topk_idx, int R, int E, int32_t* __restrict__ seg_hist) {
    const int lane = threadIdx.x & (kWave - 1);
    const int seg = blockIdx.x * kBlockWaves + (threadIdx.x / kWave);
    const int64_t base = static_cast<int64_t>(seg) * kSegIds;
    if (base >= R) return;
    int cnt[kExpertWords] = {0, 0, 0, 0};
    for (int r = 0; r < kRounds; ++r) {
        const int64_t i = base + r * kWave + lane;
        const int my = (i < R) ? topk_idx[i] : -1;
#pragma unroll
        for (int w = 0; w < kExpertWords; ++w) {
            if (w * kWave >= E) break;
            const int e_end = min(E - w * kWave, kWave);
            for (int el = 0; el < e_end; ++el) {
                const uint64_t b = __ballot(my == w * kWave + el);
                if (lane == el) cnt[w] += __popcll(b);
            }
        }
    }
#pragma unroll
    for (int w = 0; w < kExpertWords; ++w)
        if (w * kWave + lane < E) seg_hist[static_cast<size_t>(seg) * E + w * kWave + lane] = cnt[w];
}

// One block of 1024 threads. Thread (q, e) = (tid / E, tid % E) walks the segments of slice q
// of the segment range for expert e, so consecutive lanes read consecutive experts of a row of
// seg_hist (coalesced) and the 1024 / E slices run side by side; the slices' sums are then
// prefix-summed per expert, the experts' totals across experts, and a second walk writes
// seg_base. All integer: any summation order gives the same bits.
__global__ __launch_bounds__(1024) void scan_kernel(const int32_t* __restrict__ seg_hist,
                                                    int nseg, int E, int32_t* __restrict__ counts,
                                                    int32_t* __restrict__ offsets,
                                                    int32_t* __restrict__ seg_base) {
    __shared__ int32_t part[1024];              // [slice][expert]: sum, then exclusive prefix
    __shared__ int32_t tot[kMaxExperts];
    __shared__ int32_t off[kMaxExperts + 1];
    const int tid = threadIdx.x;
    const int slices = min(1024 / E, 32);       // >= 4 because E <= 256; 32 bound the serial
                                                // pass over the slices below
    const int e = tid % E, q = tid / E;
    const bool active = q < slices;
    const int per = (nseg + slices - 1) / slices;
    const int g0 = min(nseg, q * per), g1 = min(nseg, g0 + per);
    if (active) {
        int sum = 0;
#pragma unroll 8
        for (int g = g0; g < g1; ++g) sum += seg_hist[static_cast<size_t>(g) * E + e];
        part[q * E + e] = sum;
    }
    __syncthreads();
    if (tid < E) {                              // slices of one expert, in order
        int run = 0;
        for (int i = 0; i < slices; ++i) {
            const int v = part[i * E + tid];
            part[i * E + tid] = run;
            run += v;
        }
        tot[tid] = run;
    }
    __syncthreads();
    if (tid < kWave) {                          // exclusive prefix over the experts, 4 per lane
        int mine[kExpertWords], sum = 0;
#pragma unroll
        for (int w = 0; w < kExpertWords; ++w) {
            const int x = tid * kExpertWords + w;
            mine[w] = x < E ? tot[x] : 0;
            sum += mine[w];
        }
        int incl = sum;
        for (int s = 1; s < kWave; s <<= 1) {
            const int up = __shfl_up(incl, s, kWave);
            if (tid >= s) incl += up;
        }
        int run = incl - sum;
#pragma unroll
        for (int w = 0; w < kExpertWords; ++w) {
            const int x = tid * kExpertWords + w;
            if (x < E) off[x] = run;
            run += mine[w];
        }
        if (tid == kWave - 1) off[E] = incl;
    }
    __syncthreads();
    if (tid < E) {
        counts[tid] = tot[tid];
        offsets[tid] = off[tid];
    }
    if (tid == 0) offsets[E] = off[E];
    if (active) {
        int run = off[e] + part[q * E + e];
#pragma unroll 8
        for (int g = g0; g < g1; ++g) {
            const int v = seg_hist[static_cast<size_t>(g) * E + e];
            seg_base[static_cast<size_t>(g) * E + e] = run;
            run += v;
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
    int run[kExpertWords];
#pragma unroll
    for (int w = 0; w < kExpertWords; ++w)
        run[w] = (w * kWave + lane < E) ? seg_base[static_cast<size_t>(seg) * E + w * kWave + lane] : 0;
    for (int r = 0; r < kRounds; ++r) {
        const int64_t i = base + r * kWave + lane;
        const int my = (i < R) ? topk_idx[i] : -1;
        int pos = -1;
#pragma unroll
        for (int w = 0; w < kExpertWords; ++w) {
            if (w * kWave >= E) break;
            const int e_end = min(E - w * kWave, kWave);
            for (int el = 0; el < e_end; ++el) {
                const int e = w * kWave + el;
                const uint64_t b = __ballot(my == e);
                const int base_e = __shfl(run[w], el, kWave);
                if (my == e) pos = base_e + __popcll(b & lanemask_lt(lane));
                if (lane == el) run[w] += __popcll(b);
            }
        }
        if (i < R) {
            inv_perm[i] = pos;
            if (pos >= 0) perm[pos] = static_cast<int32_t>(i);
        }
    }
}

// Scatter for many experts: running positions per expert in a wavefront-private LDS table; the
// rank of an id inside a round is its position among the lanes with the same expert, and the
// first of those lanes advances the table (rounds are in id order, so the sort stays stable).
__global__ __launch_bounds__(kBlockWaves* kWave) void scatter_many_kernel(
    const int32_t* __restrict__ topk_idx, int R, int E, const int32_t* __restrict__ seg_base,
    int32_t* __restrict__ perm, int32_t* __restrict__ inv_perm) {
    __shared__ int32_t table[kBlockWaves][kMaxExperts];
    const int lane = threadIdx.x & (kWave - 1);
    const int wv = threadIdx.x / kWave;
    const int seg = blockIdx.x * kBlockWaves + wv;
    const int64_t base = static_cast<int64_t>(seg) * kSegIds;
    if (base >= R) return;
    volatile int32_t* run = table[wv];      // read and written across lanes: never cached
    for (int e = lane; e < E; e += kWave) run[e] = seg_base[static_cast<size_t>(seg) * E + e];
    for (int r = 0; r < kRounds; ++r) {
        const int64_t i = base + r * kWave + lane;
        int my = (i < R) ? topk_idx[i] : -1;
        if (my < 0 || my >= E) my = -1;
        const uint64_t same = same_value_lanes(my);
        int pos = -1;
        if (my >= 0) {
            const int start = run[my];                  // every lane of the set reads first ...
            pos = start + __popcll(same & lanemask_lt(lane));
        }
        // ... then its first lane writes (a wavefront executes the two steps in lockstep, and
        // LDS operations of one wavefront complete in order; the fence keeps the compiler from
        // moving the read below the write)
        __builtin_amdgcn_wave_barrier();
        if (my >= 0 && (same & lanemask_lt(lane)) == 0) run[my] = pos + __popcll(same);
        __builtin_amdgcn_wave_barrier();
        if (i < R) {
            inv_perm[i] = pos;
            if (pos >= 0) perm[pos] = static_cast<int32_t>(i);
        }
    }
}

// All three steps in one workgroup of 16 wavefronts for up to 16 segments (R <= 4096: decode
// batches), with the per-segment tables in LDS instead of global memory: one launch, not three.
constexpr int kSmallWaves = 16;
__global__ __launch_bounds__(kSmallWaves* kWave) void permute_small_kernel(
    const int32_t* __restrict__ topk_idx, int R, int E, int32_t* __restrict__ counts,
    int32_t* __restrict__ offsets, int32_t* __restrict__ perm, int32_t* __restrict__ inv_perm) {
    __shared__ int32_t table[kSmallWaves][kMaxExperts];   // per segment: count, then start position
    __shared__ int32_t tot[kMaxExperts];
    __shared__ int32_t off[kMaxExperts + 1];
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wv = tid / kWave;
    const int64_t base = static_cast<int64_t>(wv) * kSegIds;
    volatile int32_t* mine = table[wv];       // read and written across lanes: never cached
    int my[kRounds];
    uint64_t same[kRounds];
    for (int e = lane; e < E; e += kWave) mine[e] = 0;
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
        const int64_t i = base + r * kWave + lane;
        my[r] = (i < R) ? topk_idx[i] : -1;
        if (my[r] < 0 || my[r] >= E) my[r] = -1;
        same[r] = same_value_lanes(my[r]);
        if (my[r] >= 0 && (same[r] & lanemask_lt(lane)) == 0) mine[my[r]] += __popcll(same[r]);
        __builtin_amdgcn_wave_barrier();
    }
    __syncthreads();
    if (tid < E) {                            // segments of one expert, in order
        int run = 0;
        for (int g = 0; g < kSmallWaves; ++g) {
            const int v = table[g][tid];
            table[g][tid] = run;
            run += v;
        }
        tot[tid] = run;
    }
    __syncthreads();
    if (tid < kWave) {                        // exclusive prefix over the experts, 4 per lane
        int part[kExpertWords], sum = 0;
#pragma unroll
        for (int w = 0; w < kExpertWords; ++w) {
            const int x = tid * kExpertWords + w;
            part[w] = x < E ? tot[x] : 0;
            sum += part[w];
        }
        int incl = sum;
        for (int s = 1; s < kWave; s <<= 1) {
            const int up = __shfl_up(incl, s, kWave);
            if (tid >= s) incl += up;
        }
        int run = incl - sum;
#pragma unroll
        for (int w = 0; w < kExpertWords; ++w) {
            const int x = tid * kExpertWords + w;
            if (x < E) off[x] = run;
            run += part[w];
        }
        if (tid == kWave - 1) off[E] = incl;
    }
    __syncthreads();
    if (tid < E) {
        counts[tid] = tot[tid];
        offsets[tid] = off[tid];
    }
    if (tid == 0) offsets[E] = off[E];
    for (int e = lane; e < E; e += kWave) mine[e] += off[e];   // start positions of this segment
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
        const int64_t i = base + r * kWave + lane;
        int pos = -1;
        if (my[r] >= 0) pos = mine[my[r]] + __popcll(same[r] & lanemask_lt(lane));
        __builtin_amdgcn_wave_barrier();      // every lane of a set has read before its first lane writes
        if (my[r] >= 0 && (same[r] & lanemask_lt(lane)) == 0) mine[my[r]] = pos + __popcll(same[r]);
        __builtin_amdgcn_wave_barrier();
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

int permute_launches(int R) { return (R + kSegIds - 1) / kSegIds <= kSmallWaves ? 1 : 3; }

int launch_permute(const int32_t* topk_idx, int R, int E, int32_t* counts, int32_t* offsets,
                   int32_t* perm, int32_t* inv_perm, int32_t* seg_tables, hipStream_t s) {
    const int nseg = (R + kSegIds - 1) / kSegIds;
    if (nseg <= kSmallWaves) {
        hipLaunchKernelGGL(permute_small_kernel, dim3(1), dim3(kSmallWaves * kWave), 0, s, topk_idx,
                           R, E, counts, offsets, perm, inv_perm);
        return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
    }
    int32_t* seg_hist = seg_tables;
    int32_t* seg_base = seg_tables + static_cast<size_t>(nseg) * E;
    const int blocks = (nseg + kBlockWaves - 1) / kBlockWaves;
    const bool many = E > 16;            // one ballot per expert below, 9 per round above
    if (nseg > 0)
        hipLaunchKernelGGL(many ? hist_many_kernel : hist_kernel, dim3(blocks),
                           dim3(kBlockWaves * kWave), 0, s, topk_idx, R, E, seg_hist);
    hipLaunchKernelGGL(scan_kernel, dim3(1), dim3(1024), 0, s, seg_hist, nseg, E, counts, offsets,
                       seg_base);
    if (nseg > 0)
        hipLaunchKernelGGL(many ? scatter_many_kernel : scatter_kernel, dim3(blocks),
                           dim3(kBlockWaves * kWave), 0, s, topk_idx, R, E, seg_base, perm, inv_perm);
    return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

int launch_gather(const moe_bf16* x, const int32_t* perm, const int32_t* offsets, int R, int d,
                  int k, int E, moe_bf16* x_perm, hipStream_t s) {
    if (R == 0) return MOE_OK;
    hipLaunchKernelGGL(gather_kernel, dim3(R), dim3(256), 0, s, x, perm, offsets + E, d, k, x_perm);
    return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

}  // namespace moe

// ---- the permutation without a context and without any allocation -------------------------
namespace {

constexpr int kMaxDevices = 64;
std::mutex g_static_mutex;
int32_t* g_static_tables[kMaxDevices] = {};   // per device: address of that GPU's copy of `scratch`

// Address of the current device's copy of the static array (looked up once per device, with
// that device current). Host code never uses the array's name as a pointer.
int static_tables(int32_t** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return MOE_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_static_mutex);
    if (g_static_tables[dev] == nullptr) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) {
            (void)hipGetLastError();
            return MOE_ERR_HIP;
        }
        g_static_tables[dev] = static_cast<int32_t*>(p);
    }
    *out = g_static_tables[dev];
    return MOE_OK;
}

}  // namespace

extern "C" int moe_permute_static(const int32_t* topk_idx, int32_t T, int32_t k, int32_t E,
                                  int32_t* counts, int32_t* offsets, int32_t* perm,
                                  int32_t* inv_perm, void* stream) {
    if (T < 0 || k < 1 || E < 1 || E > moe::kMaxExperts || k > E || k > moe::kWave)
        return MOE_ERR_INVALID_ARG;
    if (static_cast<long long>(T) * k >= (1LL << 31)) return MOE_ERR_INVALID_ARG;
    if (!counts || !offsets) return MOE_ERR_INVALID_ARG;
    if (T > 0 && (!topk_idx || !perm || !inv_perm)) return MOE_ERR_INVALID_ARG;
    const int R = T * k;
    if (moe::permute_scratch_ints(R, E) > 2 * kStaticTableInts) return MOE_ERR_UNSUPPORTED_SHAPE;
    int32_t* tables = nullptr;
    const int rc = static_tables(&tables);
    if (rc != MOE_OK) return rc;
    // Every table entry that a kernel reads is written earlier in the same call (the histogram
    // kernel stores all E counts of every segment), so nothing has to be cleared.
    return moe::launch_permute(topk_idx, R, E, counts, offsets, perm, inv_perm, tables,
                               static_cast<hipStream_t>(stream));
}
