// Router: logits, top-k selection and gates (paper Section 2.1: a routing function sends each
// token to the top-k of the experts). One wavefront owns TOK consecutive tokens.
//
// The fp32 summation order of a logit is fixed so that the selected indices are reproducible
// bit for bit: lane l of the wavefront owns elements i = 512*j + 8*l + v (one 16-byte vector
// of x per 512-element chunk) and accumulates acc = fma(x_i, w_i, acc) for j ascending, then
// v ascending; the 64 lane partials combine by the xor butterfly s = 32,16,8,4,2,1; the bias
// is added last. Several tokens share one pass over W_r (it is re-read from L2, not HBM) but
// each (token, expert) accumulator sees exactly that order.
//
// HBM traffic per token: 2*d_model bytes of x read, 8*k bytes written.
#include "common.h"

namespace moe {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// Selection + gates for one token whose E logits sit in registers (static indexing only).
// Slot s takes the largest remaining logit; ties go to the lower index because the scan is
// ascending with a strict '>'. NaN ranks below every number. Gates: softmax over the
// selected logits, exp(l_s - l_0) / sum.
template <int EP>
__device__ __forceinline__ void select_and_gate(const float (&l)[EP], int E, int k,
                                                int32_t* idx_out, float* w_out) {
    uint64_t taken = 0;
    float top = 0.f, den = 0.f;
    for (int s = 0; s < k; ++s) {
        int best = -1;
        float bestv = 0.f;
#pragma unroll
        for (int e = 0; e < EP; ++e) {
            if (e < E && !((taken >> e) & 1ull)) {
                float v = (l[e] != l[e]) ? -INFINITY : l[e];
                if (best < 0 || v > bestv) { best = e; bestv = v; }
            }
        }
        taken |= 1ull << best;
        if (s == 0) top = bestv;
        // the raw (non-NaN-mapped) logit difference; NaN inputs are unsupported beyond ordering
        float w = expf(bestv - top);
        den += w;
        idx_out[s] = best;
        w_out[s] = w;
    }
    for (int s = 0; s < k; ++s) w_out[s] = w_out[s] / den;
}

template <int EP, int TOK>
__global__ __launch_bounds__(256) void route_kernel(const uint16_t* __restrict__ x,
                                                    const float* __restrict__ wr,
                                                    const float* __restrict__ bias, int T, int d,
                                                    int E, int k, int32_t* __restrict__ topk_idx,
                                                    float* __restrict__ topk_w,
                                                    float* __restrict__ logits_out) {
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = (blockIdx.x * blockDim.x + threadIdx.x) / kWave;
    const int t0 = wave * TOK;
    if (t0 >= T) return;

    float acc[TOK][EP];
#pragma unroll
    for (int q = 0; q < TOK; ++q)
#pragma unroll
        for (int e = 0; e < EP; ++e) acc[q][e] = 0.f;

    const int chunks = d / 512;
    for (int j = 0; j < chunks; ++j) {
        const int i0 = 512 * j + 8 * lane;
        u32x4 xv[TOK];
#pragma unroll
        for (int q = 0; q < TOK; ++q) {
            const int t = min(t0 + q, T - 1);   // clamp: the duplicate result is never stored
            xv[q] = *reinterpret_cast<const u32x4*>(x + static_cast<size_t>(t) * d + i0);
        }
#pragma unroll
        for (int v = 0; v < 8; ++v) {
            float w[EP];
            const float* wrow = wr + static_cast<size_t>(i0 + v) * E;
#pragma unroll
            for (int e = 0; e < EP; ++e) w[e] = (e < E) ? wrow[e] : 0.f;
#pragma unroll
            for (int q = 0; q < TOK; ++q) {
                const uint32_t word = xv[q][v >> 1];
                const float xf = __uint_as_float((v & 1) ? (word & 0xffff0000u) : (word << 16));
#pragma unroll
                for (int e = 0; e < EP; ++e) acc[q][e] = fmaf(xf, w[e], acc[q][e]);
            }
        }
    }

#pragma unroll
    for (int s = 32; s >= 1; s >>= 1)
#pragma unroll
        for (int q = 0; q < TOK; ++q)
#pragma unroll
            for (int e = 0; e < EP; ++e) acc[q][e] = acc[q][e] + __shfl_xor(acc[q][e], s, kWave);

    if (bias != nullptr) {
#pragma unroll
        for (int e = 0; e < EP; ++e) {
            const float b = (e < E) ? bias[e] : 0.f;
#pragma unroll
            for (int q = 0; q < TOK; ++q) acc[q][e] = acc[q][e] + b;
        }
    }

    // Every lane now holds all logits; lane q finishes token t0+q.
#pragma unroll
    for (int q = 0; q < TOK; ++q) {
        const int t = t0 + q;
        if (t < T && lane == q) {
            if (logits_out != nullptr) {
#pragma unroll
                for (int e = 0; e < EP; ++e)
                    if (e < E) logits_out[static_cast<size_t>(t) * E + e] = acc[q][e];
            }
            select_and_gate<EP>(acc[q], E, k, topk_idx + static_cast<size_t>(t) * k,
                                topk_w + static_cast<size_t>(t) * k);
        }
    }
}

// Fast path for E in {8, 16}: the same arithmetic, but the 512 x E slice of W_r that a chunk
// needs is staged once per workgroup in LDS (coalesced 16-byte global reads) and every lane
// then pulls its own 8 x E weights with 16-byte LDS reads. Lane l's 8*E floats sit at byte
// offset l * (32*E + 16): the 16-byte pad spreads 16 consecutive lanes over all 64 banks.
template <int E_, int TOK>
__global__ __launch_bounds__(256) void route_kernel_lds(const uint16_t* __restrict__ x,
                                                        const float* __restrict__ wr,
                                                        const float* __restrict__ bias, int T,
                                                        int d, int k,
                                                        int32_t* __restrict__ topk_idx,
                                                        float* __restrict__ topk_w,
                                                        float* __restrict__ logits_out) {
    constexpr int E = E_;
    constexpr int LANE_BYTES = 32 * E + 16;             // padded per-lane slice
    constexpr int CHUNK_BYTES = 512 * E * 4;            // W_r bytes per 512-element chunk
    constexpr int VEC_PER_THREAD = CHUNK_BYTES / 16 / 256;
    __shared__ __attribute__((aligned(16))) unsigned char wlds[2][64 * LANE_BYTES];

    const int lane = threadIdx.x & (kWave - 1);
    const int wave_in_block = threadIdx.x / kWave;
    const int t0 = (blockIdx.x * 4 + wave_in_block) * TOK;

    float acc[TOK][E];
#pragma unroll
    for (int q = 0; q < TOK; ++q)
#pragma unroll
        for (int e = 0; e < E; ++e) acc[q][e] = 0.f;

    const int chunks = d / 512;
    u32x4 stage[VEC_PER_THREAD];
    auto load_w = [&](int j) {
        const u32x4* src = reinterpret_cast<const u32x4*>(wr + static_cast<size_t>(j) * 512 * E);
#pragma unroll
        for (int i = 0; i < VEC_PER_THREAD; ++i) stage[i] = src[threadIdx.x + i * 256];
    };
    auto store_w = [&](int buf) {
#pragma unroll
        for (int i = 0; i < VEC_PER_THREAD; ++i) {
            const int byte = (threadIdx.x + i * 256) * 16;          // offset inside the chunk
            const int l = byte / (32 * E), within = byte % (32 * E);
            *reinterpret_cast<u32x4*>(&wlds[buf][l * LANE_BYTES + within]) = stage[i];
        }
    };
    load_w(0);
    store_w(0);
    __syncthreads();
    for (int j = 0; j < chunks; ++j) {
        const int buf = j & 1;
        if (j + 1 < chunks) load_w(j + 1);
        const int i0 = 512 * j + 8 * lane;
        u32x4 xv[TOK];
#pragma unroll
        for (int q = 0; q < TOK; ++q) {
            const int t = min(t0 + q, T - 1);   // clamp: the duplicate result is never stored
            xv[q] = *reinterpret_cast<const u32x4*>(x + static_cast<size_t>(t) * d + i0);
        }
        const unsigned char* mine = &wlds[buf][lane * LANE_BYTES];
#pragma unroll
        for (int v = 0; v < 8; ++v) {
            float w[E];
#pragma unroll
            for (int c = 0; c < E / 4; ++c) {
                const f32x4 f = *reinterpret_cast<const f32x4*>(mine + (v * E + c * 4) * 4);
                w[c * 4 + 0] = f[0]; w[c * 4 + 1] = f[1]; w[c * 4 + 2] = f[2]; w[c * 4 + 3] = f[3];
            }
#pragma unroll
            for (int q = 0; q < TOK; ++q) {
                const uint32_t word = xv[q][v >> 1];
                const float xf = __uint_as_float((v & 1) ? (word & 0xffff0000u) : (word << 16));
#pragma unroll
                for (int e = 0; e < E; ++e) acc[q][e] = fmaf(xf, w[e], acc[q][e]);
            }
        }
        if (j + 1 < chunks) store_w(buf ^ 1);
        __syncthreads();
    }

#pragma unroll
    for (int s = 32; s >= 1; s >>= 1)
#pragma unroll
        for (int q = 0; q < TOK; ++q)
#pragma unroll
            for (int e = 0; e < E; ++e) acc[q][e] = acc[q][e] + __shfl_xor(acc[q][e], s, kWave);

    if (bias != nullptr) {
#pragma unroll
        for (int e = 0; e < E; ++e) {
            const float b = bias[e];
#pragma unroll
            for (int q = 0; q < TOK; ++q) acc[q][e] = acc[q][e] + b;
        }
    }
#pragma unroll
    for (int q = 0; q < TOK; ++q) {
        const int t = t0 + q;
        if (t < T && lane == q) {
            if (logits_out != nullptr) {
#pragma unroll
                for (int e = 0; e < E; ++e) logits_out[static_cast<size_t>(t) * E + e] = acc[q][e];
            }
            select_and_gate<E>(acc[q], E, k, topk_idx + static_cast<size_t>(t) * k,
                               topk_w + static_cast<size_t>(t) * k);
        }
    }
}

template <int E_, int TOK>
int launch_route_lds(const moe_bf16* x, const float* wr, const float* bias, int T, int d, int k,
                     int32_t* idx, float* w, float* logits_out, hipStream_t s) {
    const int blocks = (T + 4 * TOK - 1) / (4 * TOK);
    hipLaunchKernelGGL((route_kernel_lds<E_, TOK>), dim3(blocks), dim3(256), 0, s, x, wr, bias, T, d,
                       k, idx, w, logits_out);
    return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

// One thread per token, logits read from memory.
template <int EP>
__global__ __launch_bounds__(256) void route_from_logits_kernel(const float* __restrict__ logits,
                                                                int T, int E, int k,
                                                                int32_t* __restrict__ topk_idx,
                                                                float* __restrict__ topk_w) {
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= T) return;
    float l[EP];
#pragma unroll
    for (int e = 0; e < EP; ++e) l[e] = (e < E) ? logits[static_cast<size_t>(t) * E + e] : 0.f;
    select_and_gate<EP>(l, E, k, topk_idx + static_cast<size_t>(t) * k,
                        topk_w + static_cast<size_t>(t) * k);
}

template <int EP, int TOK>
int launch_route_t(const moe_bf16* x, const float* wr, const float* bias, int T, int d, int E,
                   int k, int32_t* idx, float* w, float* logits_out, hipStream_t s) {
    const int waves = (T + TOK - 1) / TOK;
    const int blocks = (waves + 3) / 4;
    hipLaunchKernelGGL((route_kernel<EP, TOK>), dim3(blocks), dim3(256), 0, s, x, wr, bias, T, d,
                       E, k, idx, w, logits_out);
    return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

}  // namespace

int launch_route(const moe_bf16* x, const float* w_router, const float* bias, int T, int d, int E,
                 int k, int32_t* topk_idx, float* topk_w, float* logits_out, hipStream_t s) {
    if (T == 0) return MOE_OK;
    if (E == 8) return launch_route_lds<8, 2>(x, w_router, bias, T, d, k, topk_idx, topk_w, logits_out, s);
    if (E == 16) return launch_route_lds<16, 2>(x, w_router, bias, T, d, k, topk_idx, topk_w, logits_out, s);
    if (E <= 8) return launch_route_t<8, 4>(x, w_router, bias, T, d, E, k, topk_idx, topk_w, logits_out, s);
    if (E <= 16) return launch_route_t<16, 2>(x, w_router, bias, T, d, E, k, topk_idx, topk_w, logits_out, s);
    if (E <= 32) return launch_route_t<32, 1>(x, w_router, bias, T, d, E, k, topk_idx, topk_w, logits_out, s);
    return launch_route_t<64, 1>(x, w_router, bias, T, d, E, k, topk_idx, topk_w, logits_out, s);
}

int launch_route_from_logits(const float* logits, int T, int E, int k, int32_t* topk_idx,
                             float* topk_w, hipStream_t s) {
    if (T == 0) return MOE_OK;
    const int blocks = (T + 255) / 256;
#define MOE_RFL(EP)                                                                              \
    hipLaunchKernelGGL((route_from_logits_kernel<EP>), dim3(blocks), dim3(256), 0, s, logits, T, \
                       E, k, topk_idx, topk_w)
    if (E <= 8) MOE_RFL(8);
    else if (E <= 16) MOE_RFL(16);
    else if (E <= 32) MOE_RFL(32);
    else MOE_RFL(64);
#undef MOE_RFL
    return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

}  // namespace moe
