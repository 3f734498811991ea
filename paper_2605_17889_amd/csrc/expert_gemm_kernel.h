// Grouped expert GEMM kernel for gfx950 (device code; included by expert_gemm.hip).
//
//   C[p, n] = sum_k A[p, k] * B_e[n, k]           for the rows p of expert e's group,
// both operands contiguous along k ("NT"), bf16 in, fp32 accumulation on
// v_mfma_f32_32x32x16_bf16, bf16 out. With DUAL, a tile carries BN/2 rows of W1 and the
// matching BN/2 rows of W3 (interleaved in blocks of 32) and stores SiLU(gate)*up.
//
// Data path: global memory -> LDS by direct-to-LDS loads (no VGPR staging), a ring of LDS
// stages, one workgroup barrier per k-step; LDS -> VGPR by 16-byte reads of a swizzled
// layout; MFMA. Tiles are enumerated on the device from `offsets`.
//
// Two kernels share the tile mapping, the LDS layout, the MFMA loop and the epilogue:
//   grouped_gemm_kernel     every wavefront loads its share of a stage and then computes
//                           (small tiles: decode and micro-batch sized expert groups);
//   grouped_gemm_ws_kernel  wavefront-specialised: 8 consumer wavefronts only read LDS and
//                           issue MFMAs, 2 producer wavefronts only issue the direct-to-LDS
//                           loads (the texture-address unit accepts one 1 KB wavefront load
//                           per ~25 cycles, which would otherwise stall the MFMA issue of the
//                           wavefront that waits for it), and 1 wavefront touches the lines of
//                           a later k-step so that the loads find them in L2.
#pragma once
#include "common.h"

namespace moe {
namespace gemm {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kXcds = 8;     // workgroups are dealt round-robin to the 8 XCDs (own L2 each)
constexpr int kGroupM = 8;   // m-tiles that sweep the n-tiles together (share weight tiles)

struct TileCoord {
    int expert;      // -1: no tile for this workgroup
    int row0;        // first row (in the permuted matrix) of the tile
    int rows;        // valid rows in the tile (1..BM)
    int nt;          // n-tile index
    int mi;          // m-tile index inside its group
    int gm;          // m-tiles in that group
};

// Map a workgroup to its tile. Logical tile order: expert by expert; inside an expert, groups
// of kGroupM m-tiles; inside a group the n-tiles, each visited by all m-tiles of the group in
// turn. XCD x is handed the x-th contiguous eighth of that order, so the workgroups resident
// together on one XCD share A rows and weight tiles in its L2.
template <int BM>
__device__ __forceinline__ TileCoord locate_tile(const int32_t* __restrict__ offsets, int E,
                                                 int NT) {
    TileCoord tc{-1, 0, 0, 0, 0, 1};
    int total = 0;
    for (int e = 0; e < E; ++e) total += ((offsets[e + 1] - offsets[e] + BM - 1) / BM) * NT;
    const int per = (total + kXcds - 1) / kXcds;
    const int xcd = blockIdx.x % kXcds;
    const int slot = blockIdx.x / kXcds;
    const int L = xcd * per + slot;
    if (slot >= per || L >= total) return tc;
    int start = 0;
    for (int e = 0; e < E; ++e) {
        const int m_e = offsets[e + 1] - offsets[e];
        const int mt = (m_e + BM - 1) / BM;
        const int n_tiles = mt * NT;
        if (L < start + n_tiles) {
            const int local = L - start;
            const int g = local / (kGroupM * NT);
            const int first = g * kGroupM;
            const int gm = min(kGroupM, mt - first);
            const int in = local - g * (kGroupM * NT);
            const int mi = first + in % gm;
            tc.expert = e;
            tc.mi = in % gm;
            tc.gm = gm;
            tc.nt = in / gm;
            tc.row0 = offsets[e] + mi * BM;
            tc.rows = min(BM, m_e - mi * BM);
            return tc;
        }
        start += n_tiles;
    }
    return tc;
}

// LDS tile layout: rows of BK bf16 in 16-byte chunks; logical chunk c of row r is stored at
// chunk position c ^ swz(r). LDS has 64 four-byte banks and a 16-byte read is served 16 lanes
// at a time, so the swizzle makes any 16 consecutive rows at one logical chunk hit 16 distinct
// 16-byte slots of a 256-byte bank window.
template <int BK>
__device__ __forceinline__ int swz(int row) {
    if (BK == 64) return (row >> 1) & 7;     // 128-byte rows: 2 rows per bank window
    return (row >> 2) & 3;                   // 64-byte rows: 4 rows per bank window
}

// One direct-to-LDS load: every lane fetches 16 bytes from sbase + voff and the wavefront's
// 64 x 16 bytes land contiguously at LDS byte offset lds_off (wave-uniform, passed in M0).
// The compiler is not told that this is a memory operation with a counter: the kernel places
// its own s_waitcnt vmcnt(n) before the barrier that publishes a stage.
__device__ __forceinline__ void dma16(const void* sbase, uint32_t voff, uint32_t lds_off) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(lds_off), "v"(voff), "s"(sbase) : "memory", "m0");
}

template <int N> __device__ __forceinline__ void wait_vmcnt() {
    static_assert(N >= 0 && N < 64, "vmcnt range");
    asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory");
}

__device__ __forceinline__ float silu(float a) { return a / (1.0f + __expf(-a)); }

__device__ __forceinline__ uint16_t to_bf16(float v) {
    __bf16 h = static_cast<__bf16>(v);       // v_cvt_pk_bf16_f32: round to nearest even
    return *reinterpret_cast<uint16_t*>(&h);
}

template <int BM_, int BN_, int BK_, int WM_, int WN_, int NSTAGE_, bool DUAL_>
struct Config {
    static constexpr int BM = BM_, BN = BN_, BK = BK_, WM = WM_, WN = WN_, NSTAGE = NSTAGE_;
    static constexpr bool DUAL = DUAL_;
    static constexpr int NW = WM * WN, NTHREADS = NW * 64;
    static constexpr int WTM = BM / WM, WTN = BN / WN, TM = WTM / 32, TN = WTN / 32;
    static constexpr int CPR = BK / 8;                     // 16-byte chunks per row
    static constexpr int RPI = 64 / CPR;                   // rows one wavefront load covers
    static constexpr int A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2;
    static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
    static constexpr int SMEM = NSTAGE * STAGE_BYTES;
    static constexpr int NIA = BM / RPI, NIB = BN / RPI;   // wavefront loads per stage
    static constexpr int LPW = (NIA + NIB) / NW;           // ... per wavefront
    static constexpr int BN_OUT = DUAL ? BN / 2 : BN;      // output columns per tile
    static_assert(BK == 64 || BK == 32, "BK");
    static_assert(BM % (WM * 32) == 0 && BN % (WN * 32) == 0, "wave tile");
    static_assert(!DUAL || TN % 2 == 0, "gate/up pairs must live in one wave");
    static_assert(NIA % NW == 0 && NIB % NW == 0, "loads must split evenly over wavefronts");
    static_assert(NSTAGE >= 2 && SMEM <= 160 * 1024, "LDS budget");
};

// ---- pieces shared by both kernels -------------------------------------------------------

// Per-lane LDS byte offsets (inside a stage) of the MFMA operand fragments of k-substep 0 and
// the swizzle term that the other substeps xor in.
template <class Cfg>
struct FragPlan {
    int a_off[Cfg::TM], a_sw[Cfg::TM], b_off[Cfg::TN], b_sw[Cfg::TN];
    int frag_row, frag_half;
    __device__ __forceinline__ void init(int lane, int wm, int wn) {
        frag_row = lane & 31;      // operand row inside a 32-row MFMA tile
        frag_half = lane >> 5;     // which 8 of the 16 k this lane feeds
#pragma unroll
        for (int i = 0; i < Cfg::TM; ++i) {
            const int r = wm * Cfg::WTM + i * 32 + frag_row;
            a_off[i] = r * (Cfg::BK * 2);
            a_sw[i] = swz<Cfg::BK>(r);
        }
#pragma unroll
        for (int j = 0; j < Cfg::TN; ++j) {
            const int r = wn * Cfg::WTN + j * 32 + frag_row;
            b_off[j] = Cfg::A_BYTES + r * (Cfg::BK * 2);
            b_sw[j] = swz<Cfg::BK>(r);
        }
    }
};

// All k-substeps of one stage: acc[i][j] += A_i * B_j, k ascending.
template <class Cfg>
__device__ __forceinline__ void mma_stage(const unsigned char* s, const FragPlan<Cfg>& fp,
                                          f32x16 (&acc)[Cfg::TM][Cfg::TN]) {
#pragma unroll
    for (int kk = 0; kk < Cfg::BK / 16; ++kk) {
        bf16x8 af[Cfg::TM], bfr[Cfg::TN];
        const int c = kk * 2 + fp.frag_half;
#pragma unroll
        for (int i = 0; i < Cfg::TM; ++i)
            af[i] = *reinterpret_cast<const bf16x8*>(s + fp.a_off[i] + ((c ^ fp.a_sw[i]) << 4));
#pragma unroll
        for (int j = 0; j < Cfg::TN; ++j)
            bfr[j] = *reinterpret_cast<const bf16x8*>(s + fp.b_off[j] + ((c ^ fp.b_sw[j]) << 4));
#pragma unroll
        for (int i = 0; i < Cfg::TM; ++i)
#pragma unroll
            for (int j = 0; j < Cfg::TN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
    }
}

// Epilogue. MFMA 32x32 result layout: lane holds column (lane & 31); register 4*q + r is row
// 8*q + 4*(lane >> 5) + r. With DUAL, accumulator tiles 2j / 2j+1 are gate / up of the same
// output columns and SiLU(gate)*up is applied in registers.
template <class Cfg>
__device__ __forceinline__ void store_tile(const f32x16 (&acc)[Cfg::TM][Cfg::TN], const TileCoord& tc,
                                           const FragPlan<Cfg>& fp, int wm, int wn,
                                           uint16_t* __restrict__ C, int ldc) {
    constexpr bool DUAL = Cfg::DUAL;
#pragma unroll
    for (int i = 0; i < Cfg::TM; ++i) {
#pragma unroll
        for (int j = 0; j < Cfg::TN; j += (DUAL ? 2 : 1)) {
            int col;
            if (DUAL) {
                const int b32 = (wn * Cfg::WTN) / 32 + j;
                col = tc.nt * Cfg::BN_OUT + (b32 >> 1) * 32 + fp.frag_row;
            } else {
                col = tc.nt * Cfg::BN_OUT + wn * Cfg::WTN + j * 32 + fp.frag_row;
            }
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int row = wm * Cfg::WTM + i * 32 + 8 * q + 4 * fp.frag_half + r;
                    if (row < tc.rows) {
                        float v;
                        if (DUAL) v = silu(acc[i][j][4 * q + r]) * acc[i][j + (DUAL ? 1 : 0)][4 * q + r];
                        else v = acc[i][j][4 * q + r];
                        C[static_cast<size_t>(tc.row0 + row) * ldc + col] = to_bf16(v);
                    }
                }
        }
    }
}

// Weight row (and matrix) that tile row r0 of the B tile comes from. With DUAL the tile rows
// alternate between W1 and W3 in blocks of 32.
template <class Cfg>
__device__ __forceinline__ const uint16_t* weight_row_ptr(const TileCoord& tc, int r0,
                                                          const uint16_t* B0, const uint16_t* B1,
                                                          int N, int K) {
    int col0;
    const uint16_t* base;
    if (Cfg::DUAL) {
        const int b32 = r0 >> 5;
        col0 = tc.nt * Cfg::BN_OUT + (b32 >> 1) * 32 + (r0 & 31);
        base = (b32 & 1) ? B1 : B0;
    } else {
        col0 = tc.nt * Cfg::BN_OUT + r0;
        base = B0;
    }
    return base + (static_cast<size_t>(tc.expert) * N + col0) * K;
}

// Row of A, relative to a_origin(), that feeds row r of the tile. Without an index the A
// matrix is already grouped: the origin is the tile's first row and the answer is r. With one,
// A holds one row per token, the origin is A itself and grouped row p reads the token
// row_index[p] / index_div (the permutation's flat id t*k+s divided by k) — the row gather
// fused into the operand load. Offsets from the origin are 32-bit: the caller guarantees
// that the token matrix is smaller than 4 GiB when it passes an index.
__device__ __forceinline__ int source_row(const TileCoord& tc, int r,
                                          const int32_t* __restrict__ row_index, int index_div) {
    return row_index ? row_index[tc.row0 + r] / index_div : r;
}
__device__ __forceinline__ const uint16_t* a_origin(const uint16_t* A, const TileCoord& tc,
                                                    const int32_t* row_index, int K) {
    return row_index ? A : A + static_cast<size_t>(tc.row0) * K;
}

// ---- kernel 1: every wavefront loads and computes ------------------------------------------
template <class Cfg>
__global__ __launch_bounds__(Cfg::NTHREADS) void grouped_gemm_kernel(
    const uint16_t* __restrict__ A, const uint16_t* __restrict__ B0,
    const uint16_t* __restrict__ B1, uint16_t* __restrict__ C,
    const int32_t* __restrict__ offsets, const int32_t* __restrict__ row_index, int index_div,
    int E, int N, int K) {
    constexpr int BM = Cfg::BM, BK = Cfg::BK, WN = Cfg::WN, NW = Cfg::NW;
    constexpr int TM = Cfg::TM, TN = Cfg::TN;
    constexpr int CPR = Cfg::CPR, RPI = Cfg::RPI, NIA = Cfg::NIA, NIB = Cfg::NIB;
    constexpr int LA = NIA / NW, LB = NIB / NW, LPW = Cfg::LPW, NSTAGE = Cfg::NSTAGE;
    static_assert(NIA % NW == 0 && NIB % NW == 0, "loads must split evenly over wavefronts");

    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];

    const TileCoord tc = locate_tile<BM>(offsets, E, N / Cfg::BN_OUT);
    if (tc.expert < 0) return;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;

    // ---- direct-to-LDS load plan. Wavefront load q of a stage covers tile rows
    //      [q*RPI, (q+1)*RPI); lane l lands at row q*RPI + l/CPR, chunk position l%CPR, so it
    //      must fetch logical chunk (l%CPR) ^ swz(row). A rows past the group's end are
    //      clamped to its last row (always in bounds; masked at the store).
    const int lrow = lane / CPR, lpos = lane % CPR;
    const uint16_t* a_base = a_origin(A, tc, row_index, K);
    uint32_t a_voff[LA], a_lds[LA];
#pragma unroll
    for (int i = 0; i < LA; ++i) {
        const int q = wave * LA + i;
        const int r = q * RPI + lrow;
        const int src = source_row(tc, min(r, tc.rows - 1), row_index, index_div);
        a_voff[i] = (static_cast<uint32_t>(src) * K + ((lpos ^ swz<BK>(r)) * 8)) * 2u;
        a_lds[i] = q * 1024;
    }
    const uint16_t* b_base[LB];
    uint32_t b_voff[LB], b_lds[LB];
#pragma unroll
    for (int i = 0; i < LB; ++i) {
        const int q = wave * LB + i;
        const int r = q * RPI + lrow;
        b_base[i] = weight_row_ptr<Cfg>(tc, q * RPI, B0, B1, N, K);
        b_voff[i] = (static_cast<uint32_t>(lrow) * K + ((lpos ^ swz<BK>(r)) * 8)) * 2u;
        b_lds[i] = Cfg::A_BYTES + q * 1024;
    }
    auto issue = [&](int stage, int kt) {
        const uint32_t sbase = stage * Cfg::STAGE_BYTES;
        const size_t koff = static_cast<size_t>(kt) * BK;
#pragma unroll
        for (int i = 0; i < LA; ++i) dma16(a_base + koff, a_voff[i], sbase + a_lds[i]);
#pragma unroll
        for (int i = 0; i < LB; ++i) dma16(b_base[i] + koff, b_voff[i], sbase + b_lds[i]);
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int q = 0; q < 16; ++q) acc[i][j][q] = 0.f;
    FragPlan<Cfg> fp;
    fp.init(lane, wm, wn);

    // ---- main loop: ring of NSTAGE stages, NSTAGE-1 k-steps of loads in flight.
    const int KT = K / BK;
#pragma unroll
    for (int s = 0; s < NSTAGE - 1; ++s)
        if (s < KT) issue(s, s);
    int stage = 0;
    for (int kt = 0; kt < KT; ++kt) {
        // The loads of k-step kt are the oldest in flight; up to NSTAGE-2 newer steps may stay
        // pending. Near the tail fewer are in flight, so wait for everything.
        if (kt + NSTAGE - 2 < KT) wait_vmcnt<(NSTAGE - 2) * LPW>(); else wait_vmcnt<0>();
        __builtin_amdgcn_s_barrier();          // stage `stage` is complete for every wavefront
                                               // and stage (stage-1) is no longer being read
        const int nk = kt + NSTAGE - 1;
        if (nk < KT) issue(stage == 0 ? NSTAGE - 1 : stage - 1, nk);
        mma_stage<Cfg>(smem + stage * Cfg::STAGE_BYTES, fp, acc);
        stage = (stage + 1 == NSTAGE) ? 0 : stage + 1;
    }
    store_tile<Cfg>(acc, tc, fp, wm, wn, C, N);
}

// ---- kernel 2: wavefront-specialised, two LDS stages ---------------------------------------
// Wavefronts 0..NW-1 compute; NW loads the A tile, NW+1 the B tile, NW+2 prefetches into L2.
// All of them meet at one barrier per k-step: after barrier kt the stage of k-step kt is
// complete (the producers waited for their loads before arriving) and the other stage is free
// (the consumers finished reading it before arriving), so the producers refill it with k-step
// kt+1 while the consumers work on kt.
constexpr int kWsExtraWaves = 3;
constexpr int kPrefetchDist = 2;   // k-steps between the L2 touch and the direct-to-LDS load

template <class Cfg>
__global__ __launch_bounds__(Cfg::NTHREADS + kWsExtraWaves * 64) void grouped_gemm_ws_kernel(
    const uint16_t* __restrict__ A, const uint16_t* __restrict__ B0,
    const uint16_t* __restrict__ B1, uint16_t* __restrict__ C,
    const int32_t* __restrict__ offsets, const int32_t* __restrict__ row_index, int index_div,
    int E, int N, int K) {
    constexpr int BM = Cfg::BM, BN = Cfg::BN, BK = Cfg::BK, WN = Cfg::WN, NW = Cfg::NW;
    constexpr int TM = Cfg::TM, TN = Cfg::TN;
    constexpr int CPR = Cfg::CPR, RPI = Cfg::RPI, NIA = Cfg::NIA, NIB = Cfg::NIB;
    static_assert(Cfg::NSTAGE == 2, "the specialised kernel uses two stages");
    static_assert(NIA <= 32 && NIB <= 32, "producer load count must fit the load counter");

    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];

    const TileCoord tc = locate_tile<BM>(offsets, E, N / Cfg::BN_OUT);
    if (tc.expert < 0) return;                       // uniform for the whole workgroup

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int KT = K / BK;

    if (wave == NW + 2) {
        // ---------------- L2 prefetch wavefront. The workgroups resident together on an XCD
        // share every A row among the n-tiles of a group and every weight row among its gm
        // m-tiles; each one touches its slice of those lines kPrefetchDist k-steps ahead with
        // 4-byte loads whose results are never used (the counter is only bounded).
        const int n_share = max(1, 32 / tc.gm);                // n-tiles resident per m-group
        const int a_rows = (BM + n_share - 1) / n_share;       // <= BM
        const int b_rows = (BN + tc.gm - 1) / tc.gm;           // <= BN
        const int a0 = (tc.nt % n_share) * a_rows, b0 = tc.mi * b_rows;
        uint32_t sink = 0;
        for (int kt = 0; kt < KT; ++kt) {
            __builtin_amdgcn_s_barrier();
            const size_t ko = static_cast<size_t>(min(kt + kPrefetchDist, KT - 1)) * BK;
            for (int r = 0; r < a_rows; r += 64) {
                const int row = min(min(a0 + r + lane, a0 + a_rows - 1), tc.rows - 1);
                const uint16_t* p = a_origin(A, tc, row_index, K) +
                                    static_cast<size_t>(source_row(tc, row, row_index, index_div)) * K + ko;
                asm volatile("global_load_dword %0, %1, off" : "+v"(sink) : "v"(p) : "memory");
            }
            for (int r = 0; r < b_rows; r += 64) {
                const int row = min(min(b0 + r + lane, b0 + b_rows - 1), BN - 1);
                const uint16_t* p = weight_row_ptr<Cfg>(tc, row, B0, B1, N, K) + ko;
                asm volatile("global_load_dword %0, %1, off" : "+v"(sink) : "v"(p) : "memory");
            }
            wait_vmcnt<24>();
        }
        wait_vmcnt<0>();
        asm volatile("" :: "v"(sink));
        return;
    }

    if (wave >= NW) {
        // ---------------- producer wavefronts. Load q of a tile covers tile rows
        // [q*RPI, (q+1)*RPI); lane l lands at row q*RPI + l/CPR, chunk position l%CPR, so it
        // fetches logical chunk (l%CPR) ^ swz(row). A rows past the group's end are clamped to
        // its last row (always in bounds; masked at the store).
        const bool is_b = (wave == NW + 1);
        constexpr int NI = (NIA > NIB) ? NIA : NIB;
        const int ni = is_b ? NIB : NIA;
        const int lrow = lane / CPR, lpos = lane % CPR;
        uint32_t voff[NI];
#pragma unroll
        for (int q = 0; q < NI; ++q) {
            const int r = q * RPI + lrow;
            const int rr = is_b ? lrow
                                : source_row(tc, min(r, tc.rows - 1), row_index, index_div);
            voff[q] = (static_cast<uint32_t>(rr) * K + ((lpos ^ swz<BK>(r)) * 8)) * 2u;
        }
        const uint16_t* a_base = a_origin(A, tc, row_index, K);
        auto issue = [&](int stage, int kt) {
            const uint32_t sbase = stage * Cfg::STAGE_BYTES + (is_b ? Cfg::A_BYTES : 0);
            const size_t koff = static_cast<size_t>(kt) * BK;
#pragma unroll
            for (int q = 0; q < NI; ++q)
                if (q < ni) {
                    const uint16_t* base = is_b ? weight_row_ptr<Cfg>(tc, q * RPI, B0, B1, N, K) : a_base;
                    dma16(base + koff, voff[q], sbase + q * 1024);
                }
        };
        issue(0, 0);
        for (int kt = 0; kt < KT; ++kt) {
            wait_vmcnt<0>();                       // this wavefront's loads of k-step kt landed
            __builtin_amdgcn_s_barrier();
            if (kt + 1 < KT) issue((kt + 1) & 1, kt + 1);
        }
        return;                                    // nothing in flight: the last wait was total
    }

    // ---------------- consumer wavefronts
    const int wm = wave / WN, wn = wave % WN;
    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int q = 0; q < 16; ++q) acc[i][j][q] = 0.f;
    FragPlan<Cfg> fp;
    fp.init(lane, wm, wn);
    for (int kt = 0; kt < KT; ++kt) {
        __builtin_amdgcn_s_barrier();
        mma_stage<Cfg>(smem + (kt & 1) * Cfg::STAGE_BYTES, fp, acc);
    }
    store_tile<Cfg>(acc, tc, fp, wm, wn, C, N);
}

}  // namespace gemm
}  // namespace moe
