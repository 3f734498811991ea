// Router: logits, top-k selection and gates (paper Section 2.1: a routing function sends each
// token to the top-k of the experts). In the vector-unit kernels one wavefront owns TOK
// consecutive tokens; the matrix-core kernel (many experts, many tokens) gives a wavefront a
// tile of 16 tokens x 16 experts.
//
// The fp32 summation order of a logit is fixed so that the selected indices are reproducible
// bit for bit: lane l of the wavefront owns elements i = 512*j + 8*l + v (one 16-byte vector
// of x per 512-element chunk) and accumulates acc = fma(x_i, w_i, acc) for j ascending, then
// v ascending; the 64 lane partials combine by the xor butterfly s = 32,16,8,4,2,1; the bias
// is added last. Several tokens share one pass over W_r (it is re-read from L2, not HBM) but
// each (token, expert) accumulator sees exactly that order.
//
// HBM traffic per token: 2*d_model bytes of x read, 8*k bytes written.
#include <algorithm>
#include <atomic>
#include <type_traits>

#include "common.h"

namespace moe {
namespace {

// Sum of N per-lane values over the 64 lanes in the order of the xor butterfly (partner
// distances 32, 16, ..., 1), without keeping every sum in every lane: while more than one value
// is left, the two partners split them (the lane with the distance bit clear keeps the lower
// half) and each adds its partner's half, so a step moves half as many values as the one
// before. a + b == b + a bitwise, hence v[0] of lane l equals what the full butterfly would
// leave everywhere for value l >> (6 - log2 N). N - 1 + (6 - log2 N) shuffles instead of 6N.
template <int N, int LEFT, int S>
__device__ __forceinline__ void halving_step(float (&v)[N], int lane) {
    if constexpr (S >= 1) {
        if constexpr (LEFT > 1) {
            constexpr int H = LEFT / 2;
            const bool upper = (lane & S) != 0;
#pragma unroll
            for (int n = 0; n < H; ++n) {
                const float send = upper ? v[n] : v[n + H];
                const float keep = upper ? v[n + H] : v[n];
                v[n] = keep + __shfl_xor(send, S, kWave);
            }
            halving_step<N, H, S / 2>(v, lane);
        } else {
            v[0] = v[0] + __shfl_xor(v[0], S, kWave);
            halving_step<N, 1, S / 2>(v, lane);
        }
    }
}
template <int N>
__device__ __forceinline__ void halving_reduce(float (&v)[N], int lane) {
    static_assert(N >= 1 && N <= kWave && (N & (N - 1)) == 0, "power of two up to 64");
    halving_step<N, N, 32>(v, lane);
}


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

// Up to 16 experts, any count: W_r is read from global memory (L2) by every wavefront.
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

// Selection and gates for more than 16 experts: 16 lanes per token (four tokens per wavefront),
// lane g of a token's group holds the logits of experts g, g+16, g+32, ... (EW of them). Each of
// the k rounds takes the largest remaining logit of the group (ties -> lower expert index, NaN
// below every number): first inside the lane, ascending, then by four exchange steps of
// (value, index) pairs over the 16 lanes; "larger value, then lower index" is a total order, so
// the result does not depend on how the lanes are paired. The gates are the softmax over the selected logits,
// accumulated in slot order like select_and_gate().
template <int EW>
__global__ __launch_bounds__(256) void route_select_kernel(const float* __restrict__ logits, int T,
                                                           int E, int k,
                                                           int32_t* __restrict__ topk_idx,
                                                           float* __restrict__ topk_w) {
    constexpr int G = 16;
    const int g = threadIdx.x & (G - 1);
    const int t = (blockIdx.x * blockDim.x + threadIdx.x) / G;
    const bool live = t < T;                              // whole groups; shuffles stay in a group
    float v[EW];
#pragma unroll
    for (int w = 0; w < EW; ++w) {
        const int e = w * G + g;
        const float l = (live && e < E) ? logits[static_cast<size_t>(t) * E + e] : -INFINITY;
        v[w] = (l != l) ? -INFINITY : l;
    }
    unsigned taken = 0;                                   // bit w: expert w*16+g is selected
    float top = 0.f, den = 0.f;
    float my_w[4] = {0.f, 0.f, 0.f, 0.f};                 // lane g keeps slots g, g+16, g+32, g+48
    int my_idx[4] = {0, 0, 0, 0};
    for (int s = 0; s < k; ++s) {
        // best of this lane: ascending expert index, strict '>' keeps the lower index on ties
        float bv = 0.f;
        int be = -1;
#pragma unroll
        for (int w = 0; w < EW; ++w) {
            const int e = w * G + g;
            if (e < E && !((taken >> w) & 1u) && (be < 0 || v[w] > bv)) { bv = v[w]; be = e; }
        }
        // best of the group: larger value, then lower index; lanes without a candidate lose
        // (data-parallel-primitive moves inside a row of 16 lanes: rotate by 8, by 4, then swap
        // inside quads at distance 2 and 1; after the four steps every lane has seen all 16)
        auto take = [&](float ov, int oe) {
            const bool other = oe >= 0 && (be < 0 || ov > bv || (ov == bv && oe < be));
            if (other) { bv = ov; be = oe; }
        };
#define MOE_DPP_STEP(CTRL)                                                                        \
        take(__int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(bv), CTRL, 0xf, 0xf, false)), \
             __builtin_amdgcn_update_dpp(0, be, CTRL, 0xf, 0xf, false))
        MOE_DPP_STEP(0x128);      // row_ror:8
        MOE_DPP_STEP(0x124);      // row_ror:4
        MOE_DPP_STEP(0x4e);       // quad_perm:[2,3,0,1]
        MOE_DPP_STEP(0xb1);       // quad_perm:[1,0,3,2]
#undef MOE_DPP_STEP
        if ((be & (G - 1)) == g) taken |= 1u << (be >> 4);    // be >= 0 because k <= E
        if (s == 0) top = bv;
        const float w = expf(bv - top);
        den += w;
        if ((s & (G - 1)) == g) {
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if ((s >> 4) == j) { my_w[j] = w; my_idx[j] = be; }
        }
    }
    if (!live) return;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int s = j * G + g;
        if (s < k) {
            topk_idx[static_cast<size_t>(t) * k + s] = my_idx[j];
            topk_w[static_cast<size_t>(t) * k + s] = my_w[j] / den;
        }
    }
}

// Fast path for E in {8, 16}: the same arithmetic, but the 512 x E slice of W_r that a chunk
// needs is staged once per workgroup in LDS (coalesced 16-byte global reads) and every lane
// then pulls its own 8 x E weights with 16-byte LDS reads. Lane l's 8*E floats sit at byte
// offset l * (32*E + 16): the 16-byte pad spreads 16 consecutive lanes over all 64 banks.
template <int E_, int TOK, int WAVES>
__global__ __launch_bounds__(WAVES * 64) void route_kernel_lds(const uint16_t* __restrict__ x,
                                                        const float* __restrict__ wr,
                                                        const float* __restrict__ bias, int T,
                                                        int d, int k,
                                                        int32_t* __restrict__ topk_idx,
                                                        float* __restrict__ topk_w,
                                                        float* __restrict__ logits_out) {
    constexpr int E = E_;
    constexpr int LANE_BYTES = 32 * E + 16;             // padded per-lane slice
    constexpr int CHUNK_BYTES = 512 * E * 4;            // W_r bytes per 512-element chunk
    constexpr int NTHR = WAVES * 64;
    constexpr int VEC_PER_THREAD = CHUNK_BYTES / 16 / NTHR;
    static_assert(VEC_PER_THREAD >= 1 && VEC_PER_THREAD * NTHR * 16 == CHUNK_BYTES, "staging split");
    __shared__ __attribute__((aligned(16))) unsigned char wlds[2][64 * LANE_BYTES];

    const int lane = threadIdx.x & (kWave - 1);
    const int wave_in_block = threadIdx.x / kWave;
    const int t0 = (blockIdx.x * WAVES + wave_in_block) * TOK;

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
        for (int i = 0; i < VEC_PER_THREAD; ++i) stage[i] = src[threadIdx.x + i * NTHR];
    };
    auto store_w = [&](int buf) {
#pragma unroll
        for (int i = 0; i < VEC_PER_THREAD; ++i) {
            const int byte = (threadIdx.x + i * NTHR) * 16;          // offset inside the chunk
            const int l = byte / (32 * E), within = byte % (32 * E);
            *reinterpret_cast<u32x4*>(&wlds[buf][l * LANE_BYTES + within]) = stage[i];
        }
    };
    u32x4 xnext[TOK];
    auto load_x = [&](int j) {
#pragma unroll
        for (int q = 0; q < TOK; ++q) {
            const int t = min(t0 + q, T - 1);   // clamp: the duplicate result is never stored
            xnext[q] = *reinterpret_cast<const u32x4*>(x + static_cast<size_t>(t) * d + 512 * j +
                                                       8 * lane);
        }
    };
    load_w(0);
    load_x(0);
    store_w(0);
    __syncthreads();
    // One chunk; MORE is a compile-time flag (last chunk: nothing further to fetch) so that the
    // steady loop has no branch for the compiler to move the multiply-adds across.
    auto chunk = [&](int j, auto more) {
        constexpr bool MORE = decltype(more)::value;
        const int buf = j & 1;
        u32x4 xv[TOK];
#pragma unroll
        for (int q = 0; q < TOK; ++q) xv[q] = xnext[q];
        if constexpr (MORE) {                   // the next chunk's operands fly during this one
            load_w(j + 1);
            load_x(j + 1);
        }
        const unsigned char* mine = &wlds[buf][lane * LANE_BYTES];
        // Rows are read one ahead of the multiply-adds that use them; the fences keep the
        // compiler from hoisting all eight rows' reads (128 registers) to the top.
        f32x4 wrow[2][E / 4];
#pragma unroll
        for (int c = 0; c < E / 4; ++c) wrow[0][c] = *reinterpret_cast<const f32x4*>(mine + c * 16);
#pragma unroll
        for (int v = 0; v < 8; ++v) {
            if (v + 1 < 8) {
#pragma unroll
                for (int c = 0; c < E / 4; ++c)
                    wrow[(v + 1) & 1][c] =
                        *reinterpret_cast<const f32x4*>(mine + ((v + 1) * E + c * 4) * 4);
            }
#pragma unroll
            for (int q = 0; q < TOK; ++q) {
                const uint32_t word = xv[q][v >> 1];
                const float xf = __uint_as_float((v & 1) ? (word & 0xffff0000u) : (word << 16));
#pragma unroll
                for (int e = 0; e < E; ++e)
                    acc[q][e] = fmaf(xf, wrow[v & 1][e >> 2][e & 3], acc[q][e]);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        if constexpr (MORE) store_w(buf ^ 1);
        __syncthreads();
    };
    for (int j = 0; j + 1 < chunks; ++j) chunk(j, std::true_type{});
    chunk(chunks - 1, std::false_type{});

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

// Logits for more than 16 experts: the experts are cut into groups of 16, one workgroup takes
// 4*TOK tokens and one group, and stages that group's 512 x 16 slice of W_r per chunk in LDS
// exactly like route_kernel_lds (rows of W_r are E floats apart here). Every (token, expert)
// accumulator still sees the canonical order. Only the logits are stored; the selection runs
// afterwards (route_select_kernel).
template <int TOK, bool VEC>
__global__ __launch_bounds__(256, 2) void route_logits_group_kernel(const uint16_t* __restrict__ x,
                                                                 const float* __restrict__ wr,
                                                                 const float* __restrict__ bias,
                                                                 int T, int d, int E,
                                                                 float* __restrict__ logits_out) {
    constexpr int EG = 16;                              // experts per group
    constexpr int LANE_BYTES = 32 * EG + 16;            // padded per-lane slice (8 rows x 16 floats)
    constexpr int VEC_PER_THREAD = 512 * EG * 4 / 16 / 256;   // 8
    __shared__ __attribute__((aligned(16))) unsigned char wlds[2][64 * LANE_BYTES];

    const int lane = threadIdx.x & (kWave - 1);
    const int wave_in_block = threadIdx.x / kWave;
    const int t0 = (blockIdx.x * 4 + wave_in_block) * TOK;
    const int e0 = blockIdx.y * EG;

    float acc[TOK * EG];                                // [token][expert of the group]
#pragma unroll
    for (int n = 0; n < TOK * EG; ++n) acc[n] = 0.f;

    const int chunks = d / 512;
    f32x4 stage[VEC_PER_THREAD];
    auto load_w = [&](int j) {
#pragma unroll
        for (int i = 0; i < VEC_PER_THREAD; ++i) {
            const int vi = threadIdx.x + i * 256;        // vector index inside the 512 x 16 slice
            const int r = vi >> 2, c4 = (vi & 3) * 4;
            const float* src = wr + static_cast<size_t>(512 * j + r) * E + e0 + c4;
            if (VEC) {                                    // 16-byte loads aligned and inside
                stage[i] = *reinterpret_cast<const f32x4*>(src);
            } else {
#pragma unroll
                for (int c = 0; c < 4; ++c) stage[i][c] = (e0 + c4 + c < E) ? src[c] : 0.f;
            }
        }
    };
    auto store_w = [&](int buf) {
#pragma unroll
        for (int i = 0; i < VEC_PER_THREAD; ++i) {
            const int vi = threadIdx.x + i * 256;
            const int r = vi >> 2, c4 = (vi & 3) * 4;
            *reinterpret_cast<f32x4*>(&wlds[buf][(r >> 3) * LANE_BYTES + ((r & 7) * EG + c4) * 4]) = stage[i];
        }
    };
    u32x4 xnext[TOK];
    auto load_x = [&](int j) {
#pragma unroll
        for (int q = 0; q < TOK; ++q) {
            const int t = min(t0 + q, T - 1);   // clamp: the duplicate result is never stored
            xnext[q] = *reinterpret_cast<const u32x4*>(x + static_cast<size_t>(t) * d + 512 * j +
                                                       8 * lane);
        }
    };
    load_w(0);
    load_x(0);
    store_w(0);
    __syncthreads();
    // One chunk; MORE is a compile-time flag (last chunk: nothing further to fetch) so that the
    // steady loop has no branch for the compiler to move the multiply-adds across.
    auto chunk = [&](int j, auto more) {
        constexpr bool MORE = decltype(more)::value;
        const int buf = j & 1;
        u32x4 xv[TOK];
#pragma unroll
        for (int q = 0; q < TOK; ++q) xv[q] = xnext[q];
        if constexpr (MORE) {                   // the next chunk's operands fly during this one
            load_w(j + 1);
            load_x(j + 1);
        }
        const unsigned char* mine = &wlds[buf][lane * LANE_BYTES];
        // Rows are read one ahead of the multiply-adds that use them; the fences keep the
        // compiler from hoisting all eight rows' reads (128 registers) to the top.
        f32x4 wrow[2][EG / 4];
#pragma unroll
        for (int c = 0; c < EG / 4; ++c) wrow[0][c] = *reinterpret_cast<const f32x4*>(mine + c * 16);
#pragma unroll
        for (int v = 0; v < 8; ++v) {
            if (v + 1 < 8) {
#pragma unroll
                for (int c = 0; c < EG / 4; ++c)
                    wrow[(v + 1) & 1][c] =
                        *reinterpret_cast<const f32x4*>(mine + ((v + 1) * EG + c * 4) * 4);
            }
#pragma unroll
            for (int q = 0; q < TOK; ++q) {
                const uint32_t word = xv[q][v >> 1];
                const float xf = __uint_as_float((v & 1) ? (word & 0xffff0000u) : (word << 16));
#pragma unroll
                for (int e = 0; e < EG; ++e)
                    acc[q * EG + e] = fmaf(xf, wrow[v & 1][e >> 2][e & 3], acc[q * EG + e]);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        if constexpr (MORE) store_w(buf ^ 1);
        __syncthreads();
    };
    for (int j = 0; j + 1 < chunks; ++j) chunk(j, std::true_type{});
    chunk(chunks - 1, std::false_type{});

    // Lane 16*q + e ends with the logit of token t0+q and expert e0+e.
    halving_reduce<TOK * EG>(acc, lane);
    static_assert(TOK * EG == kWave, "one result per lane");
    const int q = lane / EG, e = lane % EG, t = t0 + q;
    if (t < T && e0 + e < E)
        logits_out[static_cast<size_t>(t) * E + e0 + e] =
            bias != nullptr ? acc[0] + bias[e0 + e] : acc[0];
}

// Logits of 16 tokens x 16 experts per wavefront on the matrix cores, for E a multiple of 16.
//
// v_mfma_f32_16x16x1_4b_f32 performs four independent rank-1 updates D_b = a_b * b_b^T + C_b of
// 16x16 tiles, each element one fused multiply-add, round to nearest even, denormals kept: the
// same operation as the fmaf of the definition above, at twice the rate of the vector unit.
// Block b of instruction slot q carries partial sum l = 4*q + b of every (token, expert) pair of
// the tile, so the 16 slots x 4 blocks hold all 64 partial chains (256 accumulator registers),
// and the updates of one chain are issued in the defined order (chunk j ascending, then
// v ascending). The 64 partials of a pair end in ONE lane, where the butterfly
// s = 32, ..., 1 becomes a tree of plain additions p[l] + p[l + s] (a + b == b + a bitwise).
//
// Operands: lane (b, i) = (lane / 16, lane % 16) supplies x[token i][512 j + 8 (4 q + b) + v]
// as the A value of slot q, step v, and lane (b, n) supplies W_r[512 j + 8 (4 q + b) + v][e0 + n]
// as the B value. Both come through LDS by direct-to-LDS loads of whole cache lines, half a
// chunk (256 elements = slots 8 hh .. 8 hh + 7) per stage, three stages in a ring, the loads of
// half-chunk h + 2 issued between the matrix instructions of half-chunk h:
//   * W_r: the 256 x 16 slice of a stage is shared by the four wavefronts (four token groups,
//     one expert group), stored as [slot][step v][lane] so that an operand fetch is one
//     conflict-free 4-byte read per lane; wavefront w brings in slots 2w, 2w+1;
//   * x: every wavefront brings in its own 16 token rows, two rows per load, 16-byte pieces of
//     the two rows interleaved and 32 bytes of padding after each pair, which makes the 16-byte
//     operand reads (row i, piece 4 q' + b) conflict-free.
typedef float f32x16 __attribute__((ext_vector_type(16)));

struct RouteMfma {
    static constexpr int W_BYTES = 8 * 8 * 64 * 4;          // 16 KB: W_r slice of half a chunk
    static constexpr int X_PAIR = 1024 + 32;                // two token rows of 512 bytes + padding
    static constexpr int X_WAVE = 8 * X_PAIR;               // 16 token rows of one wavefront
    static constexpr int STAGE = W_BYTES + 4 * X_WAVE;      // 50176 bytes
    static constexpr int NSTAGE = 3;
    static constexpr int SMEM = NSTAGE * STAGE;             // 150528 bytes
    static constexpr int LOADS = 12;                        // per wavefront and stage: 8 of x, 4 of W_r
};

// no "memory" clobber: ordinary LDS reads may move across these loads; the barriers and the
// counter waits around the stages (which do clobber memory) order what must be ordered
__device__ __forceinline__ void dma16_to_lds(const void* sbase, uint32_t voff, uint32_t lds_off) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(lds_off), "v"(voff), "s"(sbase) : "m0");
}

__global__ __launch_bounds__(256) void route_logits_mfma_kernel(const uint16_t* __restrict__ x,
                                                                const float* __restrict__ wr,
                                                                const float* __restrict__ bias,
                                                                int T, int d, int E,
                                                                float* __restrict__ logits_out) {
    using R = RouteMfma;
    extern __shared__ __attribute__((aligned(1024))) unsigned char rsm[];

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int groups = E / 16, halves = d / 256;
    // A tile is one 64-token block x one group of 16 experts. Tiles are numbered so that the
    // E/16 groups of one token block are consecutive tiles of ONE XCD (workgroups are dealt to
    // the 8 XCDs in turn): the block's token rows come from HBM once and from that XCD's L2 for
    // the other groups. A workgroup takes tiles blockIdx.x, blockIdx.x + gridDim.x, ... (the
    // grid is a multiple of 8, so it stays on its XCD's tiles); a token block past T ends its
    // list, since every later tile of the list has a higher token block.
    auto decode = [&](int id, int& tb, int& e0) {
        const int in_xcd = id / kXcds;
        tb = (in_xcd / groups) * kXcds + id % kXcds;
        e0 = (in_xcd % groups) * 16;
    };
    int tile = blockIdx.x, tb, e0;
    decode(tile, tb, e0);
    if (tb * 64 >= T) return;                             // uniform for the workgroup

    // Loads of the tile that the ring is being filled for (the "target"): x load m covers token
    // rows 2m, 2m+1 of the wavefront (rows past T read the last row; never stored), lane -> row
    // 2m + lane%2, 16-byte piece lane/2 of the half-chunk; offsets are relative to the token
    // block's first row, which goes into the scalar base. W_r load mm covers (slot, step) pairs
    // 4*(4*wave + mm) .. +3, one per 16 lanes; inside a pair lane%16 = 4*b + (16-byte piece of
    // the 16 experts); the group's first expert goes into the scalar base.
    uint32_t x_voff[8], w_voff[4];
    const uint16_t* x_base;
    const float* w_base;
    auto set_target = [&](int ttb, int te0) {
#pragma unroll
        for (int m = 0; m < 8; ++m) {
            const int row = min(ttb * 64 + wave * 16 + 2 * m + (lane & 1), T - 1) - ttb * 64;
            x_voff[m] = static_cast<uint32_t>(row) * d * 2u + 16u * (lane >> 1);
        }
        x_base = x + static_cast<size_t>(ttb) * 64 * d;
        w_base = wr + te0;
    };
#pragma unroll
    for (int mm = 0; mm < 4; ++mm) {
        const int pair = 4 * (4 * wave + mm) + (lane >> 4), q = pair >> 3, v = pair & 7, b = (lane & 15) >> 2;
        w_voff[mm] = (static_cast<uint32_t>(8 * (4 * q + b) + v) * E + 4 * (lane & 3)) * 4u;
    }
    const uint32_t lds0 = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(rsm));
    // load n (0..11) of the target's half-chunk h into stage st
    auto issue = [&](int n, int h, int st) {
        const uint32_t sb = lds0 + st * R::STAGE;
        if (n < 8)
            dma16_to_lds(x_base + 256 * h, x_voff[n], sb + R::W_BYTES + wave * R::X_WAVE + n * R::X_PAIR);
        else
            dma16_to_lds(w_base + static_cast<size_t>(256 * h) * E, w_voff[n - 8],
                         sb + (4 * wave + n - 8) * 1024);
    };
    set_target(tb, e0);
#pragma unroll
    for (int n = 0; n < R::LOADS; ++n) issue(n, 0, 0);
#pragma unroll
    for (int n = 0; n < R::LOADS; ++n) issue(n, 1, 1);

    // operand addresses of this lane inside a stage
    const int ab = lane >> 4, ai = lane & 15;
    const uint32_t x_off = R::W_BYTES + wave * R::X_WAVE + (ai >> 1) * R::X_PAIR + 32 * ab + 16 * (ai & 1);
    const uint32_t w_off = lane * 4;

    f32x16 acc[16];
    // One half-chunk (slots 8*(h%2) .. +7, steps v = 0..7) from stage st, while the 12 loads of
    // the target's half-chunk th go to stage stn between the matrix instructions. A turn always
    // issues 12 loads (past the end of the work: the last half-chunk again, into a stage nobody
    // reads), so the counter wait at its top is the same on every turn. The results stored
    // between two turns may complete before older loads: 12 outstanding operations or fewer
    // still means that the 12 oldest loads, the stage about to be read, have landed.
    auto turn = [&](int st, int th, int stn, auto odd) {
        constexpr int Q0 = decltype(odd)::value ? 8 : 0;
        asm volatile("s_waitcnt vmcnt(%0)" :: "n"(R::LOADS) : "memory");   // this stage has landed
        __syncthreads();                     // ... for everyone; nobody still reads the stage before
        const unsigned char* sb = rsm + st * R::STAGE;
        u32x4 xv[8];
#pragma unroll
        for (int ql = 0; ql < 8; ++ql) xv[ql] = *reinterpret_cast<const u32x4*>(sb + x_off + 128 * ql);
        float wv[16][4];
        auto read_w = [&](int sidx) {
#pragma unroll
            for (int qq = 0; qq < 4; ++qq)
                wv[sidx][qq] = *reinterpret_cast<const float*>(
                    sb + w_off + ((4 * (sidx / 8) + qq) * 8 + sidx % 8) * 256);
        };
        // The bf16 -> fp32 widening of a step's four token values is done a step ahead, into
        // registers of its own: a matrix instruction whose operand was written just before it
        // (or whose operand register the next conversion wants) would wait for the vector unit,
        // and with one wavefront per SIMD nothing else fills that time.
        float xf[16][4];
        auto widen = [&](int sidx) {
            const int v = sidx % 8;
#pragma unroll
            for (int qq = 0; qq < 4; ++qq) {
                const uint32_t word = xv[4 * (sidx / 8) + qq][v >> 1];
                xf[sidx][qq] = __uint_as_float((v & 1) ? (word & 0xffff0000u) : (word << 16));
            }
        };
        read_w(0);
        read_w(1);
        widen(0);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int sidx = 0; sidx < 16; ++sidx) {          // (slot group, step) = (sidx / 8, sidx % 8)
            if (sidx + 2 < 16) read_w(sidx + 2);         // operands two steps ahead
            if (sidx + 1 < 16) widen(sidx + 1);
#pragma unroll
            for (int qq = 0; qq < 4; ++qq) {
                const int ql = 4 * (sidx / 8) + qq;
                acc[Q0 + ql] = __builtin_amdgcn_mfma_f32_16x16x1f32(xf[sidx][qq], wv[sidx][qq], acc[Q0 + ql], 0, 0, 0);
            }
            if (sidx < R::LOADS) issue(sidx, th, stn);
            // order inside the step: operand reads, the widenings for the next step, then the
            // four matrix instructions (whose operands were all produced a step ago)
            __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
            __builtin_amdgcn_sched_group_barrier(0x002, 4, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    int st = 0;                                           // stage of the next turn
    for (;;) {
        int ntb, ne0;
        decode(tile + gridDim.x, ntb, ne0);
        const bool has_next = ntb * 64 < T;
#pragma unroll
        for (int q = 0; q < 16; ++q)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[q][r] = 0.f;
        for (int h = 0; h < halves; h += 2) {
            const bool last = h + 2 == halves;
            if (last && has_next) set_target(ntb, ne0);  // the ring moves on to the next tile
            const int th0 = !last ? h + 2 : has_next ? 0 : halves - 1;
            const int th1 = !last ? h + 3 : has_next ? 1 : halves - 1;
            const int st1 = st == 2 ? 0 : st + 1, st2 = st1 == 2 ? 0 : st1 + 1;
            turn(st, th0, st2, std::false_type{});
            turn(st1, th1, st, std::true_type{});
            st = st2;
        }
        // Register 4*b + r of slot q: partial l = 4*q + b of token 4*(lane/16) + r, expert lane%16.
        // Straight-line code, one token after the other (64 partials in registers at a time).
        float res[4];
        float prev = 0.f;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            // An empty statement that "uses" the previous token's result and "redefines" the
            // accumulators: the compiler cannot start this token's 64 register reads before
            // the previous token's tree is done (all four at once need more registers than
            // there are).
            asm volatile("" : "+a"(acc[0]), "+a"(acc[1]), "+a"(acc[2]), "+a"(acc[3]), "+a"(acc[4]),
                              "+a"(acc[5]), "+a"(acc[6]), "+a"(acc[7]), "+a"(acc[8]), "+a"(acc[9]),
                              "+a"(acc[10]), "+a"(acc[11]), "+a"(acc[12]), "+a"(acc[13]),
                              "+a"(acc[14]), "+a"(acc[15]) : "v"(prev));
            float p[64];
#pragma unroll
            for (int q = 0; q < 16; ++q)
#pragma unroll
                for (int b = 0; b < 4; ++b) p[4 * q + b] = acc[q][4 * b + r];
#pragma unroll
            for (int s = 32; s >= 1; s >>= 1)
#pragma unroll
                for (int l = 0; l < s; ++l) p[l] = p[l] + p[l + s];
            res[r] = p[0];
            prev = p[0];
        }
        const int e = e0 + (lane & 15);
        const float be = bias != nullptr ? bias[e] : 0.f;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int t = tb * 64 + wave * 16 + 4 * (lane >> 4) + r;
            if (t < T) logits_out[static_cast<size_t>(t) * E + e] = bias != nullptr ? res[r] + be : res[r];
        }
        if (!has_next) break;
        tile += gridDim.x;
        tb = ntb;
        e0 = ne0;
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // no load may still target LDS at the end
}

template <int E_, int TOK, int WAVES>
int launch_route_lds(const moe_bf16* x, const float* wr, const float* bias, int T, int d, int k,
                     int32_t* idx, float* w, float* logits_out, hipStream_t s) {
    const int blocks = (T + WAVES * TOK - 1) / (WAVES * TOK);
    hipLaunchKernelGGL((route_kernel_lds<E_, TOK, WAVES>), dim3(blocks), dim3(WAVES * 64), 0, s, x, wr, bias, T, d,
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

int launch_select_groups(const float* logits, int T, int E, int k, int32_t* idx, float* w,
                         hipStream_t s) {
    const int blocks = (T + 15) / 16;                     // 16 lanes per token, 16 tokens per block
#define MOE_SEL(EW)                                                                              \
    hipLaunchKernelGGL((route_select_kernel<EW>), dim3(blocks), dim3(256), 0, s, logits, T, E, k, \
                       idx, w)
    if (E <= 32) MOE_SEL(2);
    else if (E <= 64) MOE_SEL(4);
    else if (E <= 128) MOE_SEL(8);
    else MOE_SEL(16);
#undef MOE_SEL
    return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

}  // namespace

// `logits_scratch` [T, E] fp32 is only used for more than 16 experts, and only if the caller
// does not ask for the logits anyway.
int launch_route(const moe_bf16* x, const float* w_router, const float* bias, int T, int d, int E,
                 int k, int32_t* topk_idx, float* topk_w, float* logits_out,
                 float* logits_scratch, hipStream_t s) {
    if (T == 0) return MOE_OK;
    if (E > 16) {
        // logits by expert groups of 16 with W_r staged in LDS, then the selection
        float* logits = logits_out ? logits_out : logits_scratch;
        if (!logits) return MOE_ERR_INVALID_ARG;
        constexpr int TOK = 4;
        const dim3 grid((T + 4 * TOK - 1) / (4 * TOK), (E + 15) / 16);
        // Full groups and at least 128 tiles of 64 tokens x 16 experts: the matrix-core form. One
        // tile takes it about as long as 130 k (token, expert) pairs take the vector-unit
        // kernel, whatever the number of tiles up to one per compute unit (measured crossover).
        if (E % 16 == 0 && static_cast<long long>((T + 63) / 64) * (E / 16) >= 128) {
            int device = 0;
            if (hipGetDevice(&device) != hipSuccess || device < 0 || device >= 64) return MOE_ERR_HIP;
            static std::atomic<uint64_t> attr_set{0};     // one bit per device, as for the GEMM kernels
            if (!(attr_set.load(std::memory_order_acquire) & (1ull << device))) {
                if (hipFuncSetAttribute(reinterpret_cast<const void*>(route_logits_mfma_kernel),
                                        hipFuncAttributeMaxDynamicSharedMemorySize,
                                        RouteMfma::SMEM) != hipSuccess)
                    return MOE_ERR_HIP;
                attr_set.fetch_or(1ull << device, std::memory_order_release);
            }
            // one workgroup per compute unit (LDS and registers allow no more), each working
            // through its share of the tiles with the operand ring running across tile borders
            const long long tiles = static_cast<long long>(((T + 63) / 64 + kXcds - 1) / kXcds) * kXcds * (E / 16);
            static std::atomic<int> cus_of[64];           // compute units per device, asked once
            int cus = cus_of[device].load(std::memory_order_relaxed);
            if (cus == 0) {
                if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess ||
                    cus <= 0)
                    return MOE_ERR_HIP;
                cus_of[device].store(cus, std::memory_order_relaxed);
            }
            const long long grid = std::min<long long>(tiles, std::max(kXcds, cus / kXcds * kXcds));
            hipLaunchKernelGGL(route_logits_mfma_kernel, dim3(static_cast<unsigned>(grid)),
                               dim3(256), RouteMfma::SMEM, s, x, w_router, bias, T, d, E, logits);
        }
        else if (E % 16 == 0)     // every group full and 16-byte aligned: vector loads of W_r
            hipLaunchKernelGGL((route_logits_group_kernel<TOK, true>), grid, dim3(256), 0, s, x,
                               w_router, bias, T, d, E, logits);
        else
            hipLaunchKernelGGL((route_logits_group_kernel<TOK, false>), grid, dim3(256), 0, s, x,
                               w_router, bias, T, d, E, logits);
        if (hipGetLastError() != hipSuccess) return MOE_ERR_HIP;
        return launch_route_from_logits(logits, T, E, k, topk_idx, topk_w, s);
    }
    // 8 wavefronts share one staged slice of W_r: half the staging work per token of 4-wave blocks
    if (E == 8) return launch_route_lds<8, 2, 8>(x, w_router, bias, T, d, k, topk_idx, topk_w, logits_out, s);
    if (E == 16) return launch_route_lds<16, 2, 8>(x, w_router, bias, T, d, k, topk_idx, topk_w, logits_out, s);
    if (E <= 8) return launch_route_t<8, 4>(x, w_router, bias, T, d, E, k, topk_idx, topk_w, logits_out, s);
    return launch_route_t<16, 2>(x, w_router, bias, T, d, E, k, topk_idx, topk_w, logits_out, s);
}

int launch_route_from_logits(const float* logits, int T, int E, int k, int32_t* topk_idx,
                             float* topk_w, hipStream_t s) {
    if (T == 0) return MOE_OK;
    if (E > 16) return launch_select_groups(logits, T, E, k, topk_idx, topk_w, s);
    const int blocks = (T + 255) / 256;
#define MOE_RFL(EP)                                                                              \
    hipLaunchKernelGGL((route_from_logits_kernel<EP>), dim3(blocks), dim3(256), 0, s, logits, T, \
                       E, k, topk_idx, topk_w)
    if (E <= 8) MOE_RFL(8);
    else MOE_RFL(16);
#undef MOE_RFL
    return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

}  // namespace moe
