// Internal helpers shared by the HIP translation units of libmoe (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "moe.h"

namespace moe {

constexpr int kWave = 64;        // CDNA wavefront width
constexpr int kMaxExperts = 256; // four experts per lane in the permutation and routing kernels
constexpr int kXcds = 8;         // workgroups are dealt round-robin to the 8 XCDs (own L2 each)

__device__ __forceinline__ float bf16_to_f32(uint16_t b) {
    return __uint_as_float(static_cast<uint32_t>(b) << 16);
}

// fp32 -> bf16, round to nearest even; NaN stays a quiet NaN.
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return static_cast<uint16_t>((u >> 16) | 0x0040u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return static_cast<uint16_t>(u >> 16);
}

#define MOE_HIP_TRY(expr)                         \
    do {                                          \
        hipError_t e__ = (expr);                  \
        if (e__ != hipSuccess) return MOE_ERR_HIP; \
    } while (0)

// Launch wrappers (defined in the .hip files). Each returns a moe_status and only enqueues.
int launch_route(const moe_bf16* x, const float* w_router, const float* bias, int T, int d, int E,
                 int k, int32_t* topk_idx, float* topk_w, float* logits_out,
                 float* logits_scratch, hipStream_t s);
int launch_route_from_logits(const float* logits, int T, int E, int k, int32_t* topk_idx,
                             float* topk_w, hipStream_t s);
size_t permute_scratch_ints(int R_max, int E);
int permute_launches(int R);     // kernels that launch_permute enqueues for R ids
int launch_permute(const int32_t* topk_idx, int R, int E, int32_t* counts, int32_t* offsets,
                   int32_t* perm, int32_t* inv_perm, int32_t* scratch, hipStream_t s);
int launch_gather(const moe_bf16* x, const int32_t* perm, const int32_t* offsets, int R, int d,
                  int k, int E, moe_bf16* x_perm, hipStream_t s);
// Where and how a context launches its expert GEMMs: its device and the tuning knobs of
// moe_set_gemm_config (all settings give identical bits).
struct GemmEnv {
    int device = 0;
    int forced_config = -1;           // -1: automatic; 0..3: force a tile configuration
    int stream_mode = -1;             // -1: automatic; 0: weights never non-temporal; 1: always
    bool materialise_gather = false;  // layer calls write x_perm instead of fusing the gather
    bool split_last_round = true;     // large tiles: halve the tiles of a last round under half full
    int large_tile_waves = 0;         // 0: automatic; 4 / 8: wavefronts of the 256 x 256 tile
};
int launch_gateup(const GemmEnv& env, const moe_bf16* a, const int32_t* row_index, int index_div,
                  const int32_t* offsets, int R, int R_hint, int d, int f, int E,
                  const moe_bf16* W1, const moe_bf16* W3, moe_bf16* H, hipStream_t s);
int launch_down(const GemmEnv& env, const moe_bf16* H, const int32_t* offsets, int R, int R_hint,
                int d, int f, int E, const moe_bf16* W2, void* y_perm, bool y_f32, hipStream_t s);
int launch_combine(const void* y_perm, bool y_f32, const int32_t* inv_perm, const float* topk_w, int T,
                   int d, int k, moe_bf16* y, hipStream_t s);

}  // namespace moe
