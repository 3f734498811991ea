// Grouped expert GEMMs on the gfx950 matrix cores (paper Table 1 row 3: per expert three
// d_h x d_e bf16 matrices, 6*rows*d_h*d_e FLOPs; Section 4.1: each expert is a gated FFN).
//
//   gate/up : H[p, j]  = bf16( SiLU(sum_i Xp[p,i] W1_e[j,i]) * (sum_i Xp[p,i] W3_e[j,i]) )
//   down    : Yp[p, c] = bf16( sum_j H[p,j] W2_e[c,j] )
// for every row p of expert e's group, offsets[e] <= p < offsets[e+1].
//
// A workgroup owns a BM x BN output tile of ONE expert; tiles are enumerated on the device
// from `offsets` (no host synchronisation, variable rows per expert, empty experts produce no
// tile). Every output element is one accumulator chain over k = 0,16,32,... with the same
// MFMA instruction in every tile configuration, so results do not depend on how many rows an
// expert has or which configuration is picked (coalesced == micro-batched, bit for bit).
#include <atomic>
#include <cmath>

#include "expert_gemm_kernel.h"

namespace moe {
namespace {

using gemm::Config;
template <bool F32, class Cfg>
using Out = std::conditional_t<F32, gemm::F32Out<Cfg>, Cfg>;


// Compute units of a device (rounds of the pipelined kernel are that many tiles long).
int compute_units(int device) {
    static std::atomic<int> cached[64];
    int n = cached[device].load(std::memory_order_relaxed);
    if (n == 0) {
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess || n <= 0) {
            (void)hipGetLastError();
            n = 256;
        }
        cached[device].store(n, std::memory_order_relaxed);
    }
    return n;
}

template <class Kernel, class... Args>
int launch_tiles(const GemmEnv& env, std::atomic<uint64_t>& attr_set, Kernel kern, int smem,
                 int threads, long long grid, hipStream_t s, Args... args) {
    // The attribute belongs to the kernel's code object on ONE device: one bit per device, set
    // by whichever thread launches this kernel there first (setting it twice is harmless).
    if (env.device < 0 || env.device >= 64) return MOE_ERR_INVALID_ARG;
    const uint64_t bit = 1ull << env.device;
    if (!(attr_set.load(std::memory_order_acquire) & bit)) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                hipFuncAttributeMaxDynamicSharedMemorySize, smem) != hipSuccess)
            return MOE_ERR_HIP;
        attr_set.fetch_or(bit, std::memory_order_release);
    }
    grid = (grid + kXcds - 1) / kXcds * kXcds;
    if (grid > 0x7fffffffLL) return MOE_ERR_UNSUPPORTED_SHAPE;
    hipLaunchKernelGGL(kern, dim3(static_cast<unsigned>(grid)), dim3(threads), smem, s, args...);
    return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

// The generic kernel with Cfg::NSTAGE stages.
template <class Cfg>
int launch_grouped(const GemmEnv& env, const moe_bf16* A, const moe_bf16* B0, const moe_bf16* B1, moe_bf16* C,
                   const int32_t* offsets, const int32_t* row_index, int index_div, int R, int E,
                   int N, int K, hipStream_t s) {
    if (N % Cfg::BN_OUT != 0 || K % Cfg::BK != 0) return MOE_ERR_UNSUPPORTED_SHAPE;
    static std::atomic<uint64_t> attr_set{0};
    const long long max_mt = R / Cfg::BM + E;                  // >= sum_e ceil(M_e / BM)
    return launch_tiles(env, attr_set, gemm::grouped_gemm_kernel<Cfg>, Cfg::SMEM, Cfg::NTHREADS,
                        max_mt * (N / Cfg::BN_OUT), s, A, B0, B1, C, offsets, row_index, index_div,
                        E, N, K);
}

// The pipelined kernel with operand rings of NA and NB stages; tiles of at most HalfCfg::BM rows
// and the tiles of a last round that is less than half full run at half height.
template <class Cfg, class HalfCfg, int NA, int NB>
int launch_ring(const GemmEnv& env, const moe_bf16* A, const moe_bf16* B0, const moe_bf16* B1, moe_bf16* C,
                const int32_t* offsets, const int32_t* row_index, int index_div, int R, int E,
                int N, int K, hipStream_t s) {
    if (N % Cfg::BN_OUT != 0 || K % Cfg::BK != 0) return MOE_ERR_UNSUPPORTED_SHAPE;
    if (K / Cfg::BK < (NA > NB ? NA : NB)) return MOE_ERR_UNSUPPORTED_SHAPE;
    static std::atomic<uint64_t> attr_set{0};
    const int cus = env.split_last_round ? compute_units(env.device) : 0;
    const long long max_mt = R / Cfg::BM + E;                  // >= sum_e ceil(M_e / BM)
    // split tiles take two slots each: at most ceil(cus / 2 / 8) more slots in every XCD's range
    const long long grid = max_mt * (N / Cfg::BN_OUT) + kXcds * ((cus / 2 + kXcds - 1) / kXcds + 1);
    return launch_tiles(env, attr_set, gemm::grouped_gemm_ring_kernel<Cfg, HalfCfg, NA, NB>,
                        gemm::RingCfg<Cfg, NA, NB>::SMEM, Cfg::NTHREADS, grid, s, A, B0, B1, C,
                        offsets, row_index, index_div, E, N, K, cus);
}

// Tile configuration by average rows per expert. All configurations give identical bits.
int pick_config(const GemmEnv& env, int R, int E, int nt_large, int nt_mid) {
    if (env.forced_config >= 0) return env.forced_config;
    // 0: pipelined 256-row tiles (with half-height tails). 1: 128-row tiles (generic kernel).
    // 2: a few dozen rows per expert (64-row tiles). 3: a handful (32-row tiles, deep weight
    // ring). 4: 96-row tiles of four wavefronts side by side (groups of 33 to 96 rows: a quarter
    // fewer matrix instructions and fragment reads per k-step than the 128-row tile, and room
    // for a deeper weight ring in the down projection). Per-expert counts are not known on the
    // host, so the choice prices a uniform routing: the average group and its standard deviation.
    const double avg = static_cast<double>(R) / (E > 0 ? E : 1);
    const double sigma = std::sqrt(avg);
    const double upper = avg + 2.0 * sigma;
    if (upper <= 32.0) return 3;
    if (avg <= 32.0) return 2;
    if (upper <= 96.0) return 4;
    if (upper <= 256.0) {
        // one row tile per expert either way: the padded rows decide, the large tiles priced at
        // 0.8 of the time per padded row of the 128-row ones (measured on micro-batches of 64 to
        // 512 tokens at the 8x22B shape)
        const double padded_mid = std::ceil(upper / 128.0) * 128.0;
        return 256.0 * 0.8 <= padded_mid ? 0 : 1;
    }
    // Several row tiles per expert. Launch time in units of one full 256-row tile, for groups
    // one standard deviation below and above the mean: a large tile costs 1, a tail of at most
    // 128 rows 0.55 (half-height tile), a 128-row tile of the generic kernel 0.8. A launch of
    // many rounds of tiles (one workgroup per compute unit) costs its tiles; one of fewer than
    // four rounds costs whole rounds, a last round under half full 0.55 with the large tiles
    // (it is split), and the large tiles 1.25 times their count then (fewer, longer tiles
    // balance worse). Measured on micro-batches of 1024 and 2048 tokens at the 8x22B shape,
    // where the two GEMMs of one call want different answers.
    const int cus = compute_units(env.device);
    double units0 = 0.0, tiles0 = 0.0, tiles1 = 0.0;
    for (const double m : {std::max(1.0, avg - sigma), avg + sigma}) {
        const double full = std::floor(m / 256.0), tail = m - full * 256.0;
        units0 += 0.5 * (full + (tail <= 0.0 ? 0.0 : tail <= 128.0 ? 0.55 : 1.0));
        tiles0 += 0.5 * std::ceil(m / 256.0);
        tiles1 += 0.5 * std::ceil(m / 128.0);
    }
    const double scale0 = static_cast<double>(E) * nt_large, scale1 = static_cast<double>(E) * nt_mid;
    units0 *= scale0;
    tiles0 *= scale0;
    tiles1 *= scale1;
    double t0, t1;
    if (tiles0 >= 4.0 * cus) {
        t0 = units0 / cus;
    } else {
        const double whole = std::floor(tiles0 / cus), rem = tiles0 - whole * cus;
        t0 = 1.25 * (whole + (rem <= 0.0 ? 0.0 : rem <= 0.5 * cus ? 0.55 : 1.0));
    }
    t1 = 0.8 * (tiles1 >= 4.0 * cus ? tiles1 / cus : std::ceil(tiles1 / cus));
    return t0 <= t1 ? 0 : 1;
}

// Large tiles: four wavefronts of 128 x 128 outputs (one per SIMD) or eight of 128 x 64. The
// four-wavefront form addresses a weight row by a 32-bit byte offset from the expert's matrix.
bool use_one_wave_per_simd(const GemmEnv& env, int N, int K) {
    if (static_cast<unsigned long long>(N) * K * 2ull >= (1ull << 32)) return false;
    if (K % 128 != 0) return false;       // its k-loop takes two 64-wide steps per trip
    if (env.large_tile_waves != 0) return env.large_tile_waves == 4;
    return true;     // faster at every shape measured (reductions of 768 to 16384)
}

// Weights may be loaded as non-temporal when (almost) every expert has a single m-tile: then no
// other tile asks for the same weight bytes and keeping them cached only displaces the rows.
bool single_m_tile(const GemmEnv& env, int R, int E, int BM) {
    if (env.stream_mode >= 0) return env.stream_mode != 0;
    const double avg = static_cast<double>(R) / (E > 0 ? E : 1);
    return avg + 2.0 * std::sqrt(avg) <= BM;
}

//                      BM   BN  BK WM WN NSTAGE DUAL [STREAM_B]
using GateUpLarge = Config<256, 256, 64, 2, 4, 2, true>;
// one wavefront per SIMD: 2 x 2 wavefronts of 128 x 128 outputs, or of 64 x 128 at half height
using GateUpLarge1W = Config<256, 256, 64, 2, 2, 2, true>;
using GateUpHalf1W  = Config<128, 256, 64, 2, 2, 3, true>;
using DownLarge1W   = Config<256, 256, 64, 2, 2, 2, false>;
using DownHalf1W    = Config<128, 256, 64, 2, 2, 3, false>;
using GateUpMid   = Config<128, 256, 64, 2, 4, 3, true>;   // also the half-height tile of GateUpLarge
using GateUpSmall = Config<64, 128, 64, 1, 2, 4, true>;
using DownLarge   = Config<256, 256, 64, 2, 4, 2, false>;
using DownMid     = Config<128, 128, 64, 2, 2, 4, false>;
using DownMidWide = Config<128, 256, 64, 2, 4, 3, false>;
using DownSmall   = Config<64, 64, 64, 1, 2, 4, false>;
using GateUpMidS   = Config<128, 256, 64, 2, 4, 3, true, true>;
using GateUpSmallS = Config<64, 128, 64, 1, 2, 4, true, true>;
using DownMidS     = Config<128, 128, 64, 2, 2, 4, false, true>;
using DownMidWideS = Config<128, 256, 64, 2, 4, 3, false, true>;
using DownSmallS   = Config<64, 64, 64, 1, 2, 4, false, true>;
// a handful of rows per expert (decode): 32-row tiles leave LDS for seven 16 KB weight stages
using GateUpMid96  = Config<96, 256, 64, 1, 4, 3, true>;
using GateUpMid96S = Config<96, 256, 64, 1, 4, 3, true, true>;
using DownMid96      = Config<96, 128, 64, 1, 4, 5, false>;
using DownMid96S     = Config<96, 128, 64, 1, 4, 5, false, true>;
using DownMid96Wide  = Config<96, 256, 64, 1, 4, 3, false>;
using DownMid96WideS = Config<96, 256, 64, 1, 4, 3, false, true>;
using GateUpTiny   = Config<32, 128, 64, 1, 2, 7, true>;
using GateUpTinyS  = Config<32, 128, 64, 1, 2, 7, true, true>;
using DownTiny     = Config<32, 128, 64, 1, 2, 7, false>;
using DownTinyS    = Config<32, 128, 64, 1, 2, 7, false, true>;
using DownTinyNarrowS = Config<32, 64, 64, 1, 2, 11, false, true>;   // more, narrower tiles

}  // namespace

// `a` is the grouped activation matrix [R, d] when row_index is NULL; otherwise it is the
// token matrix [T, d] and grouped row p reads token row_index[p] / index_div (the caller makes
// sure that T * d * 2 bytes fit a 32-bit offset). R bounds the rows of the E launched experts
// (it sizes the grid); R_hint is how many rows they are expected to hold together (it picks the
// tile configuration): the two differ when a call covers a subset of a layer's experts.
int launch_gateup(const GemmEnv& env, const moe_bf16* a, const int32_t* row_index, int index_div,
                  const int32_t* offsets, int R, int R_hint, int d, int f, int E,
                  const moe_bf16* W1, const moe_bf16* W3, moe_bf16* H, hipStream_t s) {
    if (R == 0) return MOE_OK;
    const moe_bf16* x_perm = a;
    int config = pick_config(env, R_hint, E, f / 128, f / 128);
    if (config == 0 && d / 64 < 3) config = 1;     // the pipelined kernel needs three k-steps
    switch (config) {
        case 0:
            if (use_one_wave_per_simd(env, f, d))
                return launch_ring<GateUpLarge1W, GateUpHalf1W, 2, 3>(env, x_perm, W1, W3, H, offsets, row_index, index_div, R, E, f, d, s);
            return launch_ring<GateUpLarge, GateUpMid, 2, 3>(env, x_perm, W1, W3, H, offsets, row_index, index_div, R, E, f, d, s);
        case 1:
            if (single_m_tile(env, R_hint, E, 128))
                return launch_grouped<GateUpMidS>(env, x_perm, W1, W3, H, offsets, row_index, index_div, R, E, f, d, s);
            return launch_grouped<GateUpMid>(env, x_perm, W1, W3, H, offsets, row_index, index_div, R, E, f, d, s);
        case 4:
            if (single_m_tile(env, R_hint, E, 96))
                return launch_grouped<GateUpMid96S>(env, x_perm, W1, W3, H, offsets, row_index, index_div, R, E, f, d, s);
            return launch_grouped<GateUpMid96>(env, x_perm, W1, W3, H, offsets, row_index, index_div, R, E, f, d, s);
        case 3:
            if (single_m_tile(env, R_hint, E, 32))
                return launch_grouped<GateUpTinyS>(env, x_perm, W1, W3, H, offsets, row_index, index_div, R, E, f, d, s);
            return launch_grouped<GateUpTiny>(env, x_perm, W1, W3, H, offsets, row_index, index_div, R, E, f, d, s);
        default:
            if (single_m_tile(env, R_hint, E, 64))
                return launch_grouped<GateUpSmallS>(env, x_perm, W1, W3, H, offsets, row_index, index_div, R, E, f, d, s);
            return launch_grouped<GateUpSmall>(env, x_perm, W1, W3, H, offsets, row_index, index_div, R, E, f, d, s);
    }
}

namespace {

// F32: the same tilings with a float output matrix (gemm::F32Out).
template <bool F32>
int launch_down_as(const GemmEnv& env, const moe_bf16* H, const int32_t* offsets, int R, int R_hint,
                   int d, int f, int E, const moe_bf16* W2, moe_bf16* y_perm, hipStream_t s) {
    if (R == 0) return MOE_OK;
    const bool wide_mid = static_cast<long long>(E) * (d / 256) >= 160 && d % 256 == 0;
    int config = pick_config(env, R_hint, E, d / 256, wide_mid ? d / 256 : d / 128);
    if (config == 0 && f / 64 < 3) config = 1;     // the pipelined kernel needs three k-steps
    switch (config) {
        case 0:
            if (use_one_wave_per_simd(env, d, f))
                return launch_ring<Out<F32, DownLarge1W>, Out<F32, DownHalf1W>, 2, 3>(env, H, W2, nullptr, y_perm, offsets, nullptr, 1, R, E, d, f, s);
            return launch_ring<Out<F32, DownLarge>, Out<F32, DownMidWide>, 2, 3>(env, H, W2, nullptr, y_perm, offsets, nullptr, 1, R, E, d, f, s);
        case 1:
            // HBM-bound: wide tiles stream more bytes per workgroup, but only if there are
            // enough of them to occupy the 256 compute units (about one m-tile per expert).
            if (wide_mid) {
                if (single_m_tile(env, R_hint, E, 128))
                    return launch_grouped<Out<F32, DownMidWideS>>(env, H, W2, nullptr, y_perm, offsets, nullptr, 1, R, E, d, f, s);
                return launch_grouped<Out<F32, DownMidWide>>(env, H, W2, nullptr, y_perm, offsets, nullptr, 1, R, E, d, f, s);
            }
            if (single_m_tile(env, R_hint, E, 128))
                return launch_grouped<Out<F32, DownMidS>>(env, H, W2, nullptr, y_perm, offsets, nullptr, 1, R, E, d, f, s);
            return launch_grouped<Out<F32, DownMid>>(env, H, W2, nullptr, y_perm, offsets, nullptr, 1, R, E, d, f, s);
        case 4:
            // wide tiles where there are enough of them for the 256 compute units, as for case 1
            if (wide_mid) {
                if (single_m_tile(env, R_hint, E, 96))
                    return launch_grouped<Out<F32, DownMid96WideS>>(env, H, W2, nullptr, y_perm, offsets, nullptr, 1, R, E, d, f, s);
                return launch_grouped<Out<F32, DownMid96Wide>>(env, H, W2, nullptr, y_perm, offsets, nullptr, 1, R, E, d, f, s);
            }
            if (single_m_tile(env, R_hint, E, 96))
                return launch_grouped<Out<F32, DownMid96S>>(env, H, W2, nullptr, y_perm, offsets, nullptr, 1, R, E, d, f, s);
            return launch_grouped<Out<F32, DownMid96>>(env, H, W2, nullptr, y_perm, offsets, nullptr, 1, R, E, d, f, s);
        case 3:
            // with fewer routed rows than experts only about R experts have a tile: narrower
            // tiles so that their weights still stream through most compute units
            if (static_cast<long long>(R_hint < E ? R_hint : E) * (d / 128) < 192 && single_m_tile(env, R_hint, E, 32))
                return launch_grouped<Out<F32, DownTinyNarrowS>>(env, H, W2, nullptr, y_perm, offsets, nullptr, 1, R, E, d, f, s);
            if (d % 128 == 0) {
                if (single_m_tile(env, R_hint, E, 32))
                    return launch_grouped<Out<F32, DownTinyS>>(env, H, W2, nullptr, y_perm, offsets, nullptr, 1, R, E, d, f, s);
                return launch_grouped<Out<F32, DownTiny>>(env, H, W2, nullptr, y_perm, offsets, nullptr, 1, R, E, d, f, s);
            }
            [[fallthrough]];
        default:
            if (single_m_tile(env, R_hint, E, 64))
                return launch_grouped<Out<F32, DownSmallS>>(env, H, W2, nullptr, y_perm, offsets, nullptr, 1, R, E, d, f, s);
            return launch_grouped<Out<F32, DownSmall>>(env, H, W2, nullptr, y_perm, offsets, nullptr, 1, R, E, d, f, s);
    }
}

}  // namespace

// y_perm is [R, d] bf16, or [R, d] fp32 when y_f32 is set.
int launch_down(const GemmEnv& env, const moe_bf16* H, const int32_t* offsets, int R, int R_hint,
                int d, int f, int E, const moe_bf16* W2, void* y_perm, bool y_f32, hipStream_t s) {
    moe_bf16* out = static_cast<moe_bf16*>(y_perm);
    return y_f32 ? launch_down_as<true>(env, H, offsets, R, R_hint, d, f, E, W2, out, s)
                 : launch_down_as<false>(env, H, offsets, R, R_hint, d, f, E, W2, out, s);
}

}  // namespace moe
