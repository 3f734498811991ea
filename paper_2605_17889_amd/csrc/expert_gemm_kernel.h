// Grouped expert GEMM kernels for gfx950 (device code; included by expert_gemm.hip).
//
//   C[p, n] = sum_k A[p, k] * B_e[n, k]           for the rows p of expert e's group,
// both operands contiguous along k ("NT"), bf16 in, fp32 accumulation on
// v_mfma_f32_16x16x32_bf16, bf16 out. With DUAL, a tile carries BN/2 rows of W1 and the
// matching BN/2 rows of W3 (interleaved in blocks of 32) and stores SiLU(gate)*up.
//
// Data path: global memory -> LDS by direct-to-LDS loads (no VGPR staging); LDS -> VGPR by
// 16-byte reads of a swizzled layout; MFMA. Tiles are enumerated on the device from `offsets`.
//
// The 16x16x32 instruction is used instead of 32x32x16 because it does the same work per cycle
// with half the accumulator updates per multiply-add: under the board's power limit a loop of
// it sustains ~13 % more FLOP/s on random operands. The weight fragment is the first MFMA
// operand, so a lane ends up with four consecutive output columns of one row (one 8-byte store).
//
// Two kernels share the tile mapping, the LDS layout, the fragment plan and the epilogue:
//   grouped_gemm_kernel       ring of NSTAGE LDS stages, compiler-scheduled k-step (small tiles:
//                           decode and micro-batch sized expert groups, HBM-bound);
//   grouped_gemm_ring_kernel  hand-placed software pipeline for the large compute-bound tiles:
//                           the fragments of the next half k-step are read from LDS while the
//                           MFMAs of the current one issue, the workgroup barrier sits in the
//                           middle of a k-step so that MFMAs are ready on both sides of it, the
//                           direct-to-LDS loads are spread between the MFMAs, and the two
//                           operands have LDS rings of different depth.
#pragma once
#include <type_traits>

#include "common.h"

namespace moe {
namespace gemm {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kGroupM = 8;   // at most this many m-tiles that sweep the n-tiles together (share weight tiles)

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
//
// Every wavefront works the map out by itself, without LDS: lane l takes experts l, l+64, ...
// (one vector load of their offsets), the tile counts are prefix-summed across the lanes, and
// the lane whose range holds the tile number broadcasts its expert. The cost does not grow
// with the number of experts (a scalar loop over 128 experts would cost more than a tile of a
// small expert).
//
// split_cus > 0 (the pipelined kernel passes the number of compute units): a launch of `total`
// tiles runs in rounds of split_cus tiles, one per compute unit; when the last round is less
// than half full, each of its tiles is handed to two workgroups as an upper and a lower half
// of BM/2 rows, so that the round ends after a half-height tile instead of a full one. The
// halves are the highest slots of every XCD's range, hence the last workgroups dispatched.
//
// The tile is named by (xcd, slot): slot-th entry of XCD xcd's range; the kernels take both from
// the workgroup index. Result: expert >= 0: a tile; kNoTile: the range is exhausted (every later
// slot is too); kEmptySlot: this slot holds nothing (the lower half of a tile that has none).
constexpr int kNoTile = -1, kEmptySlot = -2;

// The same map for exactly 8 experts, on the scalar unit: the nine offsets are wavefront-uniform
// reads of memory that the kernel never writes, so they come through the scalar cache (a hit
// for every workgroup of a compute unit after the first) and the search is a handful of scalar
// instructions instead of vector loads, a prefix scan by shuffles and a ballot.
template <int BM>
__device__ __forceinline__ TileCoord locate_tile_scalar8(const int32_t* __restrict__ offsets, int NT,
                                                         int split_cus, int xcd, int slot) {
    TileCoord tc{kNoTile, 0, 0, 0, 0, 1};
    int off[9];
#pragma unroll
    for (int e = 0; e < 9; ++e) off[e] = offsets[e];
    int incl[8];
    int total = 0;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        total += ((off[e + 1] - off[e] + BM - 1) / BM) * NT;
        incl[e] = total;
    }
    const int per = (total + kXcds - 1) / kXcds;
    const int len = max(0, min(per, total - xcd * per));
    int halved = 0;
    if (split_cus > 0) {
        const int rem = total % split_cus;
        if (rem > 0 && 2 * rem <= split_cus) halved = min(len, (rem + kXcds - 1) / kXcds);
    }
    int tile_slot = slot, half = -1;
    if (slot >= len - halved) {
        const int j = slot - (len - halved);
        if (j >= 2 * halved) return tc;
        tile_slot = len - halved + (j >> 1);
        half = j & 1;
    }
    const int L = xcd * per + tile_slot;
    if (L >= total) return tc;
    int e = 0;
#pragma unroll
    for (int i = 0; i < 7; ++i) e += (L >= incl[i]) ? 1 : 0;      // first expert whose range holds L
    int start = 0, m_e = 0, row_e = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i)
        if (i == e) {
            start = i == 0 ? 0 : incl[i - 1];
            m_e = off[i + 1] - off[i];
            row_e = off[i];
        }
    const int mt = (m_e + BM - 1) / BM;
    const int ngroups = (mt + kGroupM - 1) / kGroupM;
    const int base = mt / ngroups, extra = mt - base * ngroups;
    const int local = L - start;
    const int big = extra * (base + 1) * NT;
    int gm, head, in;
    if (local < big) {
        gm = base + 1;
        const int g = local / (gm * NT);
        head = g * gm;
        in = local - g * (gm * NT);
    } else {
        gm = base;
        const int g = (local - big) / (gm * NT);
        head = extra * (base + 1) + g * gm;
        in = local - big - g * (gm * NT);
    }
    const int mi = head + in % gm;
    int row0 = row_e + mi * BM, nrows = min(BM, m_e - mi * BM);
    if (half >= 0) {
        const int h0 = half * (BM / 2);
        if (nrows <= h0) {
            tc.expert = kEmptySlot;
            return tc;
        }
        row0 += h0;
        nrows = min(BM / 2, nrows - h0);
    }
    tc.expert = e;
    tc.mi = in % gm;
    tc.gm = gm;
    tc.nt = in / gm;
    tc.row0 = row0;
    tc.rows = nrows;
    return tc;
}

template <int BM>
__device__ __forceinline__ TileCoord locate_tile_at(const int32_t* __restrict__ offsets, int E,
                                                    int NT, int split_cus, int xcd, int slot) {
    constexpr int EW = kMaxExperts / kWave;
    TileCoord tc{kNoTile, 0, 0, 0, 0, 1};
    if (E == 8) return locate_tile_scalar8<BM>(offsets, NT, split_cus, xcd, slot);
    const int lane = threadIdx.x & (kWave - 1);
    int rows[EW], first[EW], tiles[EW], incl[EW];     // per expert of this lane; incl: prefix sum
    int carry = 0;
#pragma unroll
    for (int w = 0; w < EW; ++w) {
        const int e = w * kWave + lane;
        rows[w] = first[w] = tiles[w] = incl[w] = 0;
        if (w * kWave >= E) continue;                  // uniform
        if (e < E) {
            first[w] = offsets[e];
            rows[w] = offsets[e + 1] - first[w];
            tiles[w] = ((rows[w] + BM - 1) / BM) * NT;
        }
        int sum = tiles[w];
#pragma unroll
        for (int s = 1; s < kWave; s <<= 1) {
            const int up = __shfl_up(sum, s, kWave);
            if (lane >= s) sum += up;
        }
        incl[w] = carry + sum;
        carry += __shfl(sum, kWave - 1, kWave);
    }
    const int total = __builtin_amdgcn_readfirstlane(carry);
    const int per = (total + kXcds - 1) / kXcds;
    const int len = max(0, min(per, total - xcd * per));   // tiles in this XCD's range
    int halved = 0;                                        // of those, the last `halved` are split
    if (split_cus > 0) {
        const int rem = total % split_cus;
        if (rem > 0 && 2 * rem <= split_cus) halved = min(len, (rem + kXcds - 1) / kXcds);
    }
    int tile_slot = slot, half = -1;
    if (slot >= len - halved) {
        const int j = slot - (len - halved);
        if (j >= 2 * halved) return tc;
        tile_slot = len - halved + (j >> 1);
        half = j & 1;
    }
    const int L = xcd * per + tile_slot;
#pragma unroll
    for (int w = 0; w < EW; ++w) {
        if (w * kWave >= E) continue;
        const uint64_t hit = __ballot(tiles[w] > 0 && L >= incl[w] - tiles[w] && L < incl[w]);
        if (hit == 0) continue;                        // uniform
        const int src = __builtin_ctzll(hit);
        const int start = __builtin_amdgcn_readfirstlane(__shfl(incl[w] - tiles[w], src, kWave));
        const int m_e = __builtin_amdgcn_readfirstlane(__shfl(rows[w], src, kWave));
        const int row_e = __builtin_amdgcn_readfirstlane(__shfl(first[w], src, kWave));
        // The expert's mt m-tiles form ceil(mt / kGroupM) groups of nearly equal height (the
        // first `extra` groups hold one tile more), so that a short tail tile sweeps the n-tiles
        // together with full tiles of its expert and finds the weight tiles in L2.
        const int mt = (m_e + BM - 1) / BM;
        const int ngroups = (mt + kGroupM - 1) / kGroupM;
        const int base = mt / ngroups, extra = mt - base * ngroups;
        const int local = L - start;
        const int big = extra * (base + 1) * NT;       // tiles in the taller groups
        int gm, head, in;
        if (local < big) {
            gm = base + 1;
            const int g = local / (gm * NT);
            head = g * gm;
            in = local - g * (gm * NT);
        } else {
            gm = base;
            const int g = (local - big) / (gm * NT);
            head = extra * (base + 1) + g * gm;
            in = local - big - g * (gm * NT);
        }
        const int mi = head + in % gm;
        int row0 = row_e + mi * BM, nrows = min(BM, m_e - mi * BM);
        if (half >= 0) {
            const int h0 = half * (BM / 2);
            if (nrows <= h0) {                         // the tile has no lower half
                tc.expert = kEmptySlot;
                return tc;
            }
            row0 += h0;
            nrows = min(BM / 2, nrows - h0);
        }
        tc.expert = w * kWave + src;
        tc.mi = in % gm;
        tc.gm = gm;
        tc.nt = in / gm;
        tc.row0 = row0;
        tc.rows = nrows;
        return tc;
    }
    return tc;
}

template <int BM>
__device__ __forceinline__ TileCoord locate_tile(const int32_t* __restrict__ offsets, int E,
                                                 int NT, int split_cus = 0) {
    return locate_tile_at<BM>(offsets, E, NT, split_cus, blockIdx.x % kXcds, blockIdx.x / kXcds);
}

// LDS tile layout: rows of BK bf16 in 16-byte chunks; logical chunk c of row r is stored at
// chunk position c ^ swz(r). LDS has 64 four-byte banks and a 16-byte read is served 16 lanes
// at a time; the 16 lanes of a fragment read the same logical chunk of 16 consecutive rows,
// which the swizzle spreads over 16 distinct 16-byte slots of a 256-byte bank window.
template <int BK>
__device__ __forceinline__ int swz(int row) {
    if (BK == 64) return (row >> 1) & 7;     // 128-byte rows: 2 rows per bank window
    return (row >> 2) & 3;                   // 64-byte rows: 4 rows per bank window
}

// One direct-to-LDS load: every lane fetches 16 bytes from sbase + voff and the wavefront's
// 64 x 16 bytes land contiguously at LDS byte offset lds_off (wave-uniform, passed in M0).
// The compiler is not told that this is a memory operation with a counter: the kernels place
// their own s_waitcnt vmcnt(n) before the barrier that publishes a stage.
// STREAM marks the line non-temporal: for operand bytes that no other tile will ask for again
// (weights when every expert has a single m-tile), so that they do not displace reusable lines.
template <bool STREAM = false>
__device__ __forceinline__ void dma16(const void* sbase, uint32_t voff, uint32_t lds_off) {
    if constexpr (STREAM)
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2 nt"
                     :: "s"(lds_off), "v"(voff), "s"(sbase) : "memory", "m0");
    else
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                     :: "s"(lds_off), "v"(voff), "s"(sbase) : "memory", "m0");
}

template <int N> __device__ __forceinline__ void wait_vmcnt() {
    static_assert(N >= 0 && N < 64, "vmcnt range");
    asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory");
}

// SiLU with the hardware exponential and reciprocal (about 1 ulp each): the result is rounded
// to bf16 right away, and the exact division costs three times as many instructions in the
// epilogue of every gate/up tile.
__device__ __forceinline__ float silu(float a) { return a * __builtin_amdgcn_rcpf(1.0f + __expf(-a)); }

template <int BM_, int BN_, int BK_, int WM_, int WN_, int NSTAGE_, bool DUAL_,
          bool STREAM_B_ = false>
struct Config {
    static constexpr int BM = BM_, BN = BN_, BK = BK_, WM = WM_, WN = WN_, NSTAGE = NSTAGE_;
    static constexpr bool DUAL = DUAL_;
    static constexpr bool STREAM_B = STREAM_B_;            // weights loaded as non-temporal
    static constexpr int NW = WM * WN, NTHREADS = NW * 64;
    static constexpr int WTM = BM / WM, WTN = BN / WN, TM = WTM / 16, TN = WTN / 16;
    static constexpr int KSUB = BK / 32;                   // MFMA k-substeps per stage
    static constexpr int ROW_BYTES = BK * 2;
    static constexpr int CPR = BK / 8;                     // 16-byte chunks per row
    static constexpr int RPI = 64 / CPR;                   // rows one wavefront load covers
    static constexpr int TILE_STEP = 16 * ROW_BYTES;       // LDS bytes between 16-row tiles
    static constexpr int A_BYTES = BM * ROW_BYTES, B_BYTES = BN * ROW_BYTES;
    static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
    static constexpr int SMEM = NSTAGE * STAGE_BYTES;
    static constexpr int NIA = BM / RPI, NIB = BN / RPI;   // wavefront loads per stage
    static constexpr int LPW = (NIA + NIB) / NW;           // ... per wavefront
    static constexpr int BN_OUT = DUAL ? BN / 2 : BN;      // output columns per tile
    static_assert(BK == 64 || BK == 32, "LDS rows of 128 or 64 bytes");
    static_assert(BM % (WM * 16) == 0 && BN % (WN * 16) == 0, "wave tile");
    static_assert(!DUAL || WTN % 64 == 0, "gate/up blocks of 32+32 rows must live in one wave");
    static_assert(NIA % NW == 0 && NIB % NW == 0, "loads must split evenly over wavefronts");
    static_assert(NSTAGE >= 2 && SMEM <= 160 * 1024, "LDS budget");
};

// The same tiling with fp32 outputs: C is then a float matrix. Used for the down projection
// when the layer keeps the expert outputs in fp32 until the gate-weighted sum (one bf16
// rounding fewer per output element); the accumulation is identical.
template <class Cfg>
struct F32Out : Cfg {
    static constexpr bool OUT_F32 = true;
    static_assert(!Cfg::DUAL, "the gate/up intermediate stays bf16");
};
template <class Cfg, class = void>
struct out_is_f32 : std::false_type {};
template <class Cfg>
struct out_is_f32<Cfg, std::void_t<decltype(Cfg::OUT_F32)>> : std::bool_constant<Cfg::OUT_F32> {};

// ---- pieces shared by the kernels ---------------------------------------------------------

// MFMA 16x16x32 operand fragment: lane l supplies 8 consecutive k (k-group l >> 4) of operand
// row l & 15. Per-lane LDS byte offsets inside a stage of the fragment of this wavefront's
// first A / B tile at each k-substep; tile i of the wave is 16 rows (TILE_STEP bytes) further on
// (the swizzle only depends on row & 15, so it is the same for every tile).
template <class Cfg>
struct FragPlan {
    uint32_t a_off[Cfg::KSUB], b_off[Cfg::KSUB];
    int frag_row, frag_kg;
    __device__ __forceinline__ void init(int lane, int wm, int wn) {
        frag_row = lane & 15;
        frag_kg = lane >> 4;
#pragma unroll
        for (int kk = 0; kk < Cfg::KSUB; ++kk) {
            const uint32_t chunk =
                static_cast<uint32_t>(((kk * 4 + frag_kg) ^ swz<Cfg::BK>(frag_row)) << 4);
            a_off[kk] = (wm * Cfg::WTM + frag_row) * Cfg::ROW_BYTES + chunk;
            b_off[kk] = Cfg::A_BYTES + (wn * Cfg::WTN + frag_row) * Cfg::ROW_BYTES + chunk;
        }
    }
};

__device__ __forceinline__ bf16x8 lds16(const unsigned char* p) {
    return *reinterpret_cast<const bf16x8*>(p);
}

// acc (16x16, transposed: rows = weight rows, columns = activation rows) += W_frag * X_frag
__device__ __forceinline__ f32x4 mma16(const bf16x8& w, const bf16x8& x, const f32x4& acc) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(w, x, acc, 0, 0, 0);
}

// The same instruction with the accumulator pinned to the accumulation registers (AGPRs). The
// pipelined kernel uses it so that its 128 or 256 accumulator registers never compete with the
// fragment registers (left to itself the register allocator shuffles accumulators between the
// two register classes inside the k-loop). The compiler does not know that this is an MFMA:
// it still waits for the LDS reads that feed it, but the kernel must pad by hand before
// anything other than an MFMA touches the accumulators (see mfma_drain()).
__device__ __forceinline__ void mma16_agpr(const bf16x8& w, const bf16x8& x, f32x4& acc) {
    asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(w), "v"(x));
}
// Wait states between the last MFMA and the first ordinary read of its result.
__device__ __forceinline__ void mfma_drain() {
    asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
}

// All k-substeps of one stage: acc[i][j] += A_i * B_j, k ascending.
template <class Cfg>
__device__ __forceinline__ void mma_stage(const unsigned char* s, const FragPlan<Cfg>& fp,
                                          f32x4 (&acc)[Cfg::TM][Cfg::TN]) {
#pragma unroll
    for (int kk = 0; kk < Cfg::KSUB; ++kk) {
        bf16x8 af[Cfg::TM], bfr[Cfg::TN];
#pragma unroll
        for (int i = 0; i < Cfg::TM; ++i) af[i] = lds16(s + fp.a_off[kk] + i * Cfg::TILE_STEP);
#pragma unroll
        for (int j = 0; j < Cfg::TN; ++j) bfr[j] = lds16(s + fp.b_off[kk] + j * Cfg::TILE_STEP);
#pragma unroll
        for (int i = 0; i < Cfg::TM; ++i)
#pragma unroll
            for (int j = 0; j < Cfg::TN; ++j) acc[i][j] = mma16(bfr[j], af[i], acc[i][j]);
    }
}

// Epilogue. Result layout of the transposed 16x16 tile: lane holds activation row (lane & 15)
// and the four output columns 4 * (lane >> 4) + r in registers r = 0..3. With DUAL, B-tile rows
// come in blocks of 32 W1 rows followed by the 32 W3 rows of the same output columns, so
// accumulator tiles j and j + 2 (j & 2 == 0) are gate and up of the same columns.
template <class Cfg>
__device__ __forceinline__ void store_tile(const f32x4 (&acc)[Cfg::TM][Cfg::TN], const TileCoord& tc,
                                           const FragPlan<Cfg>& fp, int wm, int wn,
                                           uint16_t* __restrict__ C, int ldc) {
    constexpr bool DUAL = Cfg::DUAL;
#pragma unroll
    for (int i = 0; i < Cfg::TM; ++i) {
        const int row = wm * Cfg::WTM + i * 16 + fp.frag_row;
        if (row >= tc.rows) continue;
        uint16_t* crow = C + static_cast<size_t>(tc.row0 + row) * ldc + tc.nt * Cfg::BN_OUT + 4 * fp.frag_kg;
#pragma unroll
        for (int j = 0; j < Cfg::TN; ++j) {
            if (DUAL && (j & 2)) continue;
            const int r0 = wn * Cfg::WTN + j * 16;                 // first B-tile row of tile j
            const int col = DUAL ? (r0 >> 6) * 32 + (r0 & 31) : r0;
            if constexpr (out_is_f32<Cfg>::value) {
                float* frow = reinterpret_cast<float*>(C) + static_cast<size_t>(tc.row0 + row) * ldc +
                              tc.nt * Cfg::BN_OUT + 4 * fp.frag_kg;
                *reinterpret_cast<f32x4*>(frow + col) = acc[i][j];
                continue;
            }
            bf16x4 o;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float v = DUAL ? silu(acc[i][j][r]) * acc[i][DUAL ? j + 2 : j][r] : acc[i][j][r];
                o[r] = static_cast<__bf16>(v);                     // round to nearest even
            }
            *reinterpret_cast<bf16x4*>(crow + col) = o;
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

// Direct-to-LDS load plan of one wavefront. Wavefront load q of a stage covers tile rows
// [q*RPI, (q+1)*RPI); lane l lands at row q*RPI + l/CPR, chunk position l%CPR, so it must
// fetch logical chunk (l%CPR) ^ swz(row). A rows past the group's end are clamped to its last
// row (always in bounds; masked at the store).
template <class Cfg>
struct LoadPlan {
    static constexpr int LA = Cfg::NIA / Cfg::NW, LB = Cfg::NIB / Cfg::NW;
    const uint16_t* a_base;
    const uint16_t* b_base[LB];
    uint32_t a_voff[LA], a_lds[LA], b_voff[LB], b_lds[LB];
    bool a_on[LA];      // false: every row of this A load lies past the end of the group
    __device__ __forceinline__ void init(const TileCoord& tc, int wave, int lane, const uint16_t* A,
                                         const uint16_t* B0, const uint16_t* B1,
                                         const int32_t* row_index, int index_div, int N, int K) {
        const int lrow = lane / Cfg::CPR, lpos = lane % Cfg::CPR;
        a_base = a_origin(A, tc, row_index, K);
#pragma unroll
        for (int i = 0; i < LA; ++i) {
            const int q = wave * LA + i;
            const int r = q * Cfg::RPI + lrow;
            const int src = source_row(tc, min(r, tc.rows - 1), row_index, index_div);
            a_voff[i] = (static_cast<uint32_t>(src) * K + ((lpos ^ swz<Cfg::BK>(r)) * 8)) * 2u;
            a_lds[i] = q * 1024;
            a_on[i] = q * Cfg::RPI < tc.rows;
        }
#pragma unroll
        for (int i = 0; i < LB; ++i) {
            const int q = wave * LB + i;
            const int r = q * Cfg::RPI + lrow;
            b_base[i] = weight_row_ptr<Cfg>(tc, q * Cfg::RPI, B0, B1, N, K);
            b_voff[i] = (static_cast<uint32_t>(lrow) * K + ((lpos ^ swz<Cfg::BK>(r)) * 8)) * 2u;
            b_lds[i] = Cfg::A_BYTES + q * 1024;
        }
    }
    // load number n (0 <= n < LA + LB) of k-step kt into the stage at LDS byte offset sbase
    __device__ __forceinline__ void issue_one(int n, uint32_t sbase, size_t koff) const {
        if (n < LA) dma16(a_base + koff, a_voff[n], sbase + a_lds[n]);
        else dma16<Cfg::STREAM_B>(b_base[n - LA] + koff, b_voff[n - LA], sbase + b_lds[n - LA]);
    }
    // single loads with explicit LDS region bases (operand rings of different depth)
    __device__ __forceinline__ void issue_a(int i, uint32_t region, size_t koff) const {
        dma16(a_base + koff, a_voff[i], region + a_lds[i]);
    }
    __device__ __forceinline__ void issue_b(int i, uint32_t region, size_t koff) const {
        dma16(b_base[i] + koff, b_voff[i], region + (b_lds[i] - Cfg::A_BYTES));
    }
    __device__ __forceinline__ void issue_all(uint32_t sbase, size_t koff) const {
#pragma unroll
        for (int n = 0; n < LA + LB; ++n) issue_one(n, sbase, koff);
    }
};

// ---- kernel 1: ring of stages, every wavefront loads and computes ---------------------------
template <class Cfg>
__global__ __launch_bounds__(Cfg::NTHREADS) void grouped_gemm_kernel(
    const uint16_t* __restrict__ A, const uint16_t* __restrict__ B0,
    const uint16_t* __restrict__ B1, uint16_t* __restrict__ C,
    const int32_t* __restrict__ offsets, const int32_t* __restrict__ row_index, int index_div,
    int E, int N, int K) {
    constexpr int BM = Cfg::BM, BK = Cfg::BK, WN = Cfg::WN;
    constexpr int TM = Cfg::TM, TN = Cfg::TN, LPW = Cfg::LPW, NSTAGE = Cfg::NSTAGE;

    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];

    const TileCoord tc = locate_tile<BM>(offsets, E, N / Cfg::BN_OUT);
    if (tc.expert < 0) return;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;

    LoadPlan<Cfg> lp;
    lp.init(tc, wave, lane, A, B0, B1, row_index, index_div, N, K);

    f32x4 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
    FragPlan<Cfg> fp;
    fp.init(lane, wm, wn);

    // ---- main loop: ring of NSTAGE stages, NSTAGE-1 k-steps of loads in flight.
    const int KT = K / BK;
#pragma unroll
    for (int s = 0; s < NSTAGE - 1; ++s)
        if (s < KT) lp.issue_all(s * Cfg::STAGE_BYTES, static_cast<size_t>(s) * BK);
    int stage = 0;
    for (int kt = 0; kt < KT; ++kt) {
        // The loads of k-step kt are the oldest in flight; up to NSTAGE-2 newer steps may stay
        // pending. Near the tail fewer are in flight, so wait for everything.
        if (kt + NSTAGE - 2 < KT) wait_vmcnt<(NSTAGE - 2) * LPW>(); else wait_vmcnt<0>();
        __builtin_amdgcn_s_barrier();          // stage `stage` is complete for every wavefront
                                               // and stage (stage-1) is no longer being read
        const int nk = kt + NSTAGE - 1;
        if (nk < KT)
            lp.issue_all((stage == 0 ? NSTAGE - 1 : stage - 1) * Cfg::STAGE_BYTES,
                         static_cast<size_t>(nk) * BK);
        mma_stage<Cfg>(smem + stage * Cfg::STAGE_BYTES, fp, acc);
        stage = (stage + 1 == NSTAGE) ? 0 : stage + 1;
    }
    store_tile<Cfg>(acc, tc, fp, wm, wn, C, N);
}

// ---- kernel 2: operand rings of different depth, hand-placed software pipeline ---------------
// A k-step (64 k) is two half-steps of one MFMA k-substep each. While the MFMAs of a half-step
// issue, the fragments of the next half-step are read from LDS into the registers that the
// MFMAs just consumed. The barrier of k-step kt sits between its two half-steps: when a
// wavefront arrives it has read all of k-step kt (the fragments of the second half are in
// registers) and its loads of k-step kt+1 have landed, so after the barrier the stages of
// k-step kt may be refilled and k-step kt+1 may be read, and the MFMAs of the second half-step
// are ready to issue at once. Scheduling fences keep each group of MFMAs, LDS reads and
// direct-to-LDS loads where it is written.
//
// LDS holds NA stages of the A tile and NB stages of the B tile (BM or BN rows of 64 k each;
// for 256 x 256 tiles NA + NB = 5 stages of 32 KB fill the 160 KB). After the barrier of k-step
// kt the A stage is refilled with k-step kt+NA and the B stage with k-step kt+NB, so the
// operand with the deeper ring has NB-1 (or NA-1) k-steps to arrive: with two stages each the
// kernel waits about a third of every k-step for the slowest cache line of the next one. The
// operand with the shallower ring is issued first within a k-step: loads complete in order, so
// the wait for it then leaves only the newest loads of the deeper operand pending.
#define MOE_FENCE() __builtin_amdgcn_sched_barrier(0)

template <class Cfg, int NA, int NB>
struct RingCfg {
    static constexpr int A_RING = NA * Cfg::A_BYTES, SMEM = NA * Cfg::A_BYTES + NB * Cfg::B_BYTES;
    static constexpr bool A_FIRST = NA <= NB;                 // issue order inside a k-step
    static constexpr int LA = Cfg::NIA / Cfg::NW, LB = Cfg::NIB / Cfg::NW;
    // loads that may stay pending when k-step kt+1 must have landed
    static constexpr int PENDING = (NA == NB) ? 0 : (NA < NB ? (NB - NA) * LB : (NA - NB) * LA);
    static_assert(SMEM <= 160 * 1024 && NA >= 2 && NB >= 2, "LDS budget");
    static_assert(NA - NB <= 1 && NB - NA <= 1, "pending count assumes rings that differ by one");
    static_assert(NA * LA + NB * LB < 64, "loads in flight must fit the 6-bit load counter");
};

// One k-step of one wavefront.
//   COMPUTE  false for a wavefront whose rows all lie past the end of a partial tile: it only
//            issues its loads and meets the others at the barrier.
//   PARTIAL  the tile has fewer than BM rows: A loads whose rows all lie past the end are
//            skipped (what the MFMAs read there only reaches output rows that are never stored).
//   RUNTIME  tail of the k-loop: dma_a / dma_b say whether k-steps kt+NA / kt+NB exist,
//            read_next whether kt+1 does, and the wait for loads is total.
//
// Fragment registers: A tile i of the next half-step replaces fa[i] right after the MFMAs that
// consumed it, except the last tile, which alternates between fa[TM-1] (first half-steps) and
// fx (second half-steps) so that it can be read at the start of the half-step: no LDS read is
// issued in the last chunk and the wait for all reads before the barrier costs nothing. B
// fragments alternate between fb0 and fb1 and are read in the first chunks.
template <class Cfg, int NA, int NB, bool COMPUTE, bool PARTIAL, bool RUNTIME>
__device__ __forceinline__ void ring_kstep(f32x4 (&acc)[Cfg::TM][Cfg::TN], bf16x8 (&fa)[Cfg::TM],
                                           bf16x8& fx, bf16x8 (&fb0)[Cfg::TN],
                                           bf16x8 (&fb1)[Cfg::TN], const unsigned char* pa_h1,
                                           const unsigned char* pb_h1, const unsigned char* pa_n0,
                                           const unsigned char* pb_n0, const LoadPlan<Cfg>& lp,
                                           uint32_t a_region, uint32_t b_region, size_t a_koff,
                                           size_t b_koff, bool dma_a, bool dma_b, bool read_next) {
    using R = RingCfg<Cfg, NA, NB>;
    constexpr int TM = Cfg::TM, TN = Cfg::TN, LA = R::LA, LB = R::LB, LPW = LA + LB;
    constexpr int BPC = (TN + TM / 2 - 1) / (TM / 2);      // B reads per chunk (first chunks)
    static_assert(TN <= TM, "interleave plan");
    static_assert(!PARTIAL || R::A_FIRST, "skipping A loads needs the B loads to be the newest");
    // ---- first half: MFMAs on (fa, fb0); read the second-half fragments of this k-step
    if (COMPUTE) {
#pragma unroll
        for (int i = 0; i < TM; ++i) {
#pragma unroll
            for (int j = 0; j < TN; ++j) mma16_agpr(fb0[j], fa[i], acc[i][j]);
            MOE_FENCE();    // the reads below reuse the registers of fa[i]: after its MFMAs
            if (i == 0) fx = lds16(pa_h1 + (TM - 1) * Cfg::TILE_STEP);
            if (i < TM - 1) fa[i] = lds16(pa_h1 + i * Cfg::TILE_STEP);
#pragma unroll
            for (int b = i * BPC; b < (i + 1) * BPC && b < TN; ++b)
                fb1[b] = lds16(pb_h1 + b * Cfg::TILE_STEP);
            MOE_FENCE();
        }
    }
    if (RUNTIME) asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
    else asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" :: "n"(R::PENDING) : "memory");
    __builtin_amdgcn_s_barrier();      // k-step kt+1 complete in LDS; this k-step's stages are free
    MOE_FENCE();
    // ---- second half: MFMAs on (fa[0..TM-2], fx, fb1); read the first-half fragments of k-step
    //      kt+1; refill the freed stages
    auto issue = [&](int n) {          // n-th load of this k-step in issue order
        const bool is_a = R::A_FIRST ? (n < LA) : (n >= LB);
        const int idx = R::A_FIRST ? (is_a ? n : n - LA) : (is_a ? n - LB : n);
        if (is_a) {
            if ((!RUNTIME || dma_a) && (!PARTIAL || lp.a_on[idx])) lp.issue_a(idx, a_region, a_koff);
        } else {
            if (!RUNTIME || dma_b) lp.issue_b(idx, b_region, b_koff);
        }
    };
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        if (COMPUTE) {
#pragma unroll
            for (int j = 0; j < TN; ++j) mma16_agpr(fb1[j], i == TM - 1 ? fx : fa[i], acc[i][j]);
            MOE_FENCE();
            if (!RUNTIME || read_next) {
                if (i == 0) fa[TM - 1] = lds16(pa_n0 + (TM - 1) * Cfg::TILE_STEP);
                if (i < TM - 1) fa[i] = lds16(pa_n0 + i * Cfg::TILE_STEP);
#pragma unroll
                for (int b = i * BPC; b < (i + 1) * BPC && b < TN; ++b)
                    fb0[b] = lds16(pb_n0 + b * Cfg::TILE_STEP);
            }
        }
        // the LPW loads of the k-step are spread evenly over the TM chunks
#pragma unroll
        for (int n = (i * LPW + TM - 1) / TM; n < ((i + 1) * LPW + TM - 1) / TM; ++n) issue(n);
        MOE_FENCE();
    }
}

// One tile of the pipelined kernel (all wavefronts of the workgroup call it together).
template <class Cfg, int NA, int NB>
__device__ __forceinline__ void ring_tile(const TileCoord& tc, unsigned char* smem,
                                          const uint16_t* __restrict__ A,
                                          const uint16_t* __restrict__ B0,
                                          const uint16_t* __restrict__ B1, uint16_t* __restrict__ C,
                                          const int32_t* __restrict__ row_index, int index_div,
                                          int N, int K) {
    using R = RingCfg<Cfg, NA, NB>;
    constexpr int BM = Cfg::BM, BK = Cfg::BK, WN = Cfg::WN, TM = Cfg::TM, TN = Cfg::TN;
    constexpr int LA = R::LA, LB = R::LB, AB = Cfg::A_BYTES, BB = Cfg::B_BYTES;
    static_assert(BK == 64, "64-k stages");

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;

    LoadPlan<Cfg> lp;
    lp.init(tc, wave, lane, A, B0, B1, row_index, index_div, N, K);
    FragPlan<Cfg> fp;
    fp.init(lane, wm, wn);
    // fragment addresses of the two k-halves inside stage 0 of each ring
    const unsigned char* pa[2] = {smem + fp.a_off[0], smem + fp.a_off[1]};
    const unsigned char* pb[2] = {smem + R::A_RING + (fp.b_off[0] - AB), smem + R::A_RING + (fp.b_off[1] - AB)};

    f32x4 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
    mfma_drain();                                    // accumulator writes settle before MFMAs

    const int KT = K / BK;                           // >= max(NA, NB) (checked by the launcher)
    constexpr int NMAX = NA < NB ? NB : NA;

    auto run = [&](auto compute_tag, auto partial_tag) {
        constexpr bool COMPUTE = decltype(compute_tag)::value, PARTIAL = decltype(partial_tag)::value;
        // prologue: fill both rings in the order the k-loop would have issued them
#pragma unroll
        for (int s = 0; s < NMAX; ++s) {
            const size_t koff = static_cast<size_t>(s) * BK;
            if (R::A_FIRST) {
                if (s < NA) for (int i = 0; i < LA; ++i) if (!PARTIAL || lp.a_on[i]) lp.issue_a(i, s * AB, koff);
                if (s < NB) for (int i = 0; i < LB; ++i) lp.issue_b(i, R::A_RING + s * BB, koff);
            } else {
                if (s < NB) for (int i = 0; i < LB; ++i) lp.issue_b(i, R::A_RING + s * BB, koff);
                if (s < NA) for (int i = 0; i < LA; ++i) lp.issue_a(i, s * AB, koff);
            }
        }
        constexpr int TOTAL = NA * LA + NB * LB;
        if (PARTIAL) wait_vmcnt<0>();                // fewer loads than TOTAL were issued
        else wait_vmcnt<TOTAL - (LA + LB)>();        // k-step 0 landed
        __builtin_amdgcn_s_barrier();
        bf16x8 fa[TM], fx, fb0[TN], fb1[TN];
        if (COMPUTE) {
#pragma unroll
            for (int i = 0; i < TM; ++i) fa[i] = lds16(pa[0] + i * Cfg::TILE_STEP);
#pragma unroll
            for (int j = 0; j < TN; ++j) fb0[j] = lds16(pb[0] + j * Cfg::TILE_STEP);
            fx = fa[TM - 1];
        }
        MOE_FENCE();

        int ra = 0, rb = 0;                          // ring positions of k-step kt
        auto step = [&](auto runtime_tag, int kt) {
            constexpr bool RT = decltype(runtime_tag)::value;
            const int ra1 = (ra + 1 == NA) ? 0 : ra + 1, rb1 = (rb + 1 == NB) ? 0 : rb + 1;
            ring_kstep<Cfg, NA, NB, COMPUTE, PARTIAL, RT>(
                acc, fa, fx, fb0, fb1, pa[1] + ra * AB, pb[1] + rb * BB, pa[0] + ra1 * AB,
                pb[0] + rb1 * BB, lp, ra * AB, R::A_RING + rb * BB,
                static_cast<size_t>(kt + NA) * BK, static_cast<size_t>(kt + NB) * BK, kt + NA < KT,
                kt + NB < KT, kt + 1 < KT);
            ra = ra1; rb = rb1;
        };
        int kt = 0;
        for (; kt + NMAX < KT; ++kt) step(std::false_type{}, kt);
        for (; kt < KT; ++kt) step(std::true_type{}, kt);
    };
    using T = std::true_type;
    using F = std::false_type;
    if (tc.rows == BM) {
        run(T{}, F{});
    } else if (wm * Cfg::WTM < tc.rows) {
        run(T{}, T{});
    } else {
        run(F{}, T{});                               // no row of this wavefront is in the tile
        return;
    }
    mfma_drain();
    store_tile<Cfg>(acc, tc, fp, wm, wn, C, N);
}

// Epilogue of the one-wavefront-per-SIMD tile: the outputs go through LDS so that global memory
// sees whole cache lines. In the accumulator layout a lane holds four consecutive columns of one
// row per fragment, so a direct store writes sixteen separate 32-byte pieces; 256 compute units
// finishing their tiles together then queue at the L2 for thousands of cycles. Here a wavefront
// writes the sixteen rows of fragment row i into a small region of its own in the now idle
// operand stages and reads them back 16 bytes per lane, whole rows at a time, so that each store
// instruction covers full 128-byte lines; the region is reused for the next fragment row. LDS
// serves a wavefront's requests in order, so neither the read after the write nor the next
// write after the read needs a wait. The 16-byte chunks of a row are XOR-swizzled by the row so
// that both the writes (16 rows at one column) and the reads (whole rows) spread over all banks.
template <class Cfg>
__device__ __forceinline__ void store_tile_via_lds(const f32x4 (&acc)[Cfg::TM][8], const TileCoord& tc,
                                                   const FragPlan<Cfg>& fp, int wave, int lane,
                                                   unsigned char* smem, uint16_t* __restrict__ C,
                                                   int ldc) {
    constexpr bool DUAL = Cfg::DUAL, F32 = out_is_f32<Cfg>::value;
    constexpr int TM = Cfg::TM, WN = Cfg::WN;
    constexpr int COLS = DUAL ? 64 : 128;            // output columns of this wavefront
    constexpr int ESZ = F32 ? 4 : 2;                 // bytes per output element
    constexpr int ROWB = COLS * ESZ;                 // bytes of one output row of this wavefront
    constexpr int CP = ROWB / 16;                    // 16-byte chunks per row
    constexpr int RSH = CP == 8 ? 1 : 0;             // log2 of the rows that share 256 bytes of LDS
    constexpr int SWM = (CP < 16 ? CP : 16) - 1;     // the swizzle permutes chunks inside 256 bytes
    constexpr int NJ = DUAL ? 4 : 8;                 // output fragments per fragment row
    constexpr int RPI = 64 / CP;                     // rows per store instruction
    static_assert(Cfg::TN == 8 && Cfg::NW * 16 * ROWB <= 2 * Cfg::A_BYTES, "fits the A ring");
    const int wm = wave / WN, wn = wave % WN;
    unsigned char* stage = smem + wave * (16 * ROWB);
    const uint32_t wswz = (fp.frag_row >> RSH) & SWM;
    unsigned char* wbase = stage + fp.frag_row * ROWB;
    const int rrow = lane / CP, rchunk = lane % CP;
    const size_t row_bytes = static_cast<size_t>(ldc) * ESZ;
    unsigned char* cbase = reinterpret_cast<unsigned char*>(C) +
                           static_cast<size_t>(tc.row0 + wm * Cfg::WTM) * row_bytes +
                           static_cast<size_t>(tc.nt * Cfg::BN_OUT + wn * COLS) * ESZ + rchunk * 16;
    const int rows_here = tc.rows - wm * Cfg::WTM;   // rows of this wavefront inside the tile
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int jj = 0; jj < NJ; ++jj) {
            const int j = DUAL ? (jj & 1) + (jj >> 1) * 4 : jj;     // gate fragments; up = j + 2
            if constexpr (F32) {
                const uint32_t chunk = (static_cast<uint32_t>(jj * 4 + fp.frag_kg) ^ wswz) * 16;
                *reinterpret_cast<f32x4*>(wbase + chunk) = acc[i][j];
            } else {
                bf16x4 o;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float v = DUAL ? silu(acc[i][j][r]) * acc[i][DUAL ? j + 2 : j][r] : acc[i][j][r];
                    o[r] = static_cast<__bf16>(v);                 // round to nearest even
                }
                const uint32_t chunk = (static_cast<uint32_t>(jj * 2 + (fp.frag_kg >> 1)) ^ wswz) * 16;
                *reinterpret_cast<bf16x4*>(wbase + chunk + (fp.frag_kg & 1) * 8) = o;
            }
        }
#pragma unroll
        for (int q = 0; q < 16 / RPI; ++q) {
            const int rl = q * RPI + rrow;                          // row inside the fragment row
            const uint32_t chunk = (static_cast<uint32_t>(rchunk) ^ ((rl >> RSH) & SWM)) * 16;
            const bf16x8 v = *reinterpret_cast<const bf16x8*>(stage + rl * ROWB + chunk);
            const int r = i * 16 + rl;
            if (r < rows_here) *reinterpret_cast<bf16x8*>(cbase + static_cast<size_t>(r) * row_bytes) = v;
        }
        MOE_FENCE();                                 // one fragment row's registers at a time
    }
}

// f(integral_constant<int, 0>) ... f(integral_constant<int, N - 1>) in order
template <int N, int I = 0, class F>
__device__ __forceinline__ void static_for(F&& f) {
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<N, I + 1>(f);
    }
}

// ---- the full tile with ONE wavefront per SIMD (4 wavefronts, 128 x 128 outputs each) --------
// Four wavefronts read 128 KB of fragments from LDS per k-step where eight read 192 KB, and hold
// all 256 accumulator registers of a lane's SIMD, so every fragment set can be double-buffered
// in the other 256 registers. With a single wavefront per SIMD nothing covers for it: a wavefront
// issues one instruction every four cycles, an MFMA occupies the matrix pipe for sixteen, so at
// most three other instructions fit between two MFMAs before the pipe runs dry. The k-step below
// therefore places every LDS read, every direct-to-LDS load and every scalar update behind an
// MFMA of its own: per half-step of 64 MFMAs, 16 fragment reads (after every fourth MFMA), 8
// loads (in every group of eight MFMAs: M0 is written before one MFMA and the load issued after
// it, the MFMA serving as the wait state that a write to M0 needs) and the pointer updates.
// The A loads of k-step kt+NA go out in the second half of k-step kt, the B loads of k-step
// kt+NB in the first half of k-step kt+1, so the texture-address unit sees one load per SIMD
// every 128 cycles throughout instead of all sixteen within one half.
template <class Cfg>
struct LoadPlan1W {
    static constexpr int LA = Cfg::NIA / Cfg::NW, LB = Cfg::NIB / Cfg::NW;
    const uint16_t* a_ptr;          // A origin + current k offset of the A loads
    const uint16_t* b_ptr[2];       // expert's W (and W3 with DUAL) + current k offset of the B loads
    uint32_t a_voff[LA], b_voff[LB];
    uint32_t a_lds, b_lds;          // this wavefront's first load inside an A / B stage
    __device__ __forceinline__ void init(const TileCoord& tc, int wave, int lane, const uint16_t* A,
                                         const uint16_t* B0, const uint16_t* B1,
                                         const int32_t* row_index, int index_div, int N, int K) {
        const int lrow = lane / Cfg::CPR, lpos = lane % Cfg::CPR;
        a_ptr = a_origin(A, tc, row_index, K);
        const size_t expert_off = static_cast<size_t>(tc.expert) * N * K;
        b_ptr[0] = B0 + expert_off;
        b_ptr[1] = Cfg::DUAL ? B1 + expert_off : b_ptr[0];
#pragma unroll
        for (int i = 0; i < LA; ++i) {
            const int r = (wave * LA + i) * Cfg::RPI + lrow;
            const int src = source_row(tc, min(r, tc.rows - 1), row_index, index_div);
            a_voff[i] = (static_cast<uint32_t>(src) * K + ((lpos ^ swz<Cfg::BK>(r)) * 8)) * 2u;
        }
#pragma unroll
        for (int i = 0; i < LB; ++i) {
            const int r0 = (wave * LB + i) * Cfg::RPI;          // first tile row of the load
            const int col0 = tc.nt * Cfg::BN_OUT + (Cfg::DUAL ? (r0 >> 6) * 32 + (r0 & 31) : r0);
            b_voff[i] = (static_cast<uint32_t>(col0 + lrow) * K + ((lpos ^ swz<Cfg::BK>(r0 + lrow)) * 8)) * 2u;
        }
        a_lds = wave * LA * 1024;
        b_lds = wave * LB * 1024;
    }
    // weight matrix of B load i (W1 and W3 rows alternate in blocks of 32 tile rows)
    __device__ __forceinline__ const uint16_t* b_src(int wave, int i) const {
        return b_ptr[Cfg::DUAL ? (((wave * LB + i) * Cfg::RPI) >> 5) & 1 : 0];
    }
};

// acc += W_frag * X_frag with the accumulator pinned to AGPRs; then one direct-to-LDS load whose
// LDS address (lds_base + LDS_OFF) was put into M0 before the MFMA.
template <int LDS_OFF>
__device__ __forceinline__ void mma16_then_dma(const bf16x8& w, const bf16x8& x, f32x4& acc,
                                               uint32_t lds_base, uint32_t voff, const void* sbase) {
    asm volatile("s_add_u32 m0, %3, %4\n\t"
                 "v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0\n\t"
                 "global_load_lds_dwordx4 %5, %6"
                 : "+a"(acc)
                 : "v"(w), "v"(x), "s"(lds_base), "n"(LDS_OFF), "v"(voff), "s"(sbase)
                 : "memory", "m0", "scc");
}

// One k-step of one wavefront. On entry f[0] holds the first-half fragments of this k-step.
// Every k-step runs exactly this code, without a branch: the accumulators are operands of inline
// assembly, which the compiler does not know to be MFMAs, so it must never find a reason (a join
// of two paths, a second loop) to move them between registers next to one. The first half issues
// the B loads of k-step kt-1+NB, the second half the A loads of k-step kt+NA. Past the end of the
// reduction the pointers stop advancing: the loads of the last k-steps fetch the last 64 k again
// into stages that nobody reads any more, which keeps the number of loads in flight, and with it
// the load-counter value to wait for, the same in every k-step. Likewise the last k-step reads
// "next" fragments from a stage that holds nothing new; they are never used.
// LDS addresses of one k-step: fragment pointers of this k-step's second half (h1) and of the
// next k-step's first half (n0), the stages that this k-step's loads refill, and the ring
// positions (as byte offsets) they derive from.
struct RingState1W {
    const unsigned char *pa_h1, *pb_h1, *pa_n0, *pb_n0;
    uint32_t a_region, b_region;    // M0 bases of the A loads (stage kt) / B loads (stage kt-1)
    uint32_t sa, sb;                // byte offsets of k-step kt's stages inside the A / B ring
};

// MFMA number m of a half-step with its load, if it has one: load n = m / STRIDE goes out behind
// MFMA m when m % STRIDE == 3 and n < NLOADS.
template <int M, int STRIDE, int NLOADS>
__device__ __forceinline__ void mma16_slot(const bf16x8& w, const bf16x8& x, f32x4& acc,
                                           uint32_t lds_base, const uint32_t* voff,
                                           const void* sbase) {
    if constexpr (M % STRIDE == 3 && M / STRIDE < NLOADS)
        mma16_then_dma<(M / STRIDE) * 1024>(w, x, acc, lds_base, voff[M / STRIDE], sbase);
    else
        mma16_agpr(w, x, acc);
}

template <class Cfg, int NA, int NB>
__device__ __forceinline__ void kstep_1w(f32x4 (&acc)[Cfg::TM][8], bf16x8 (&fa)[2][Cfg::TM],
                                         bf16x8 (&fb)[2][8], RingState1W& rs, LoadPlan1W<Cfg>& lp,
                                         int wave, const unsigned char* pa0, const unsigned char* pa1,
                                         const unsigned char* pb0, const unsigned char* pb1, int kt,
                                         int KT) {
    using R = RingCfg<Cfg, NA, NB>;
    constexpr int TM = Cfg::TM, NM = TM * 8, NR = TM + 8;      // MFMAs and fragment reads per half
    constexpr int LA = LoadPlan1W<Cfg>::LA, LB = LoadPlan1W<Cfg>::LB;
    constexpr uint32_t AB = Cfg::A_BYTES, BB = Cfg::B_BYTES;
    static_assert((TM == 8 || TM == 4) && Cfg::TN == 8 && LA == TM && LB == 8 && NA == 2,
                  "128 or 64 rows x 128 columns per wavefront");
    const uint32_t a_region = rs.a_region, b_region = rs.b_region;
    const unsigned char *pa_h1 = rs.pa_h1, *pb_h1 = rs.pb_h1, *pa_n0 = rs.pa_n0, *pb_n0 = rs.pb_n0;
    // fragment read r of a half goes out behind MFMA r * SPAN / NR: B fragments first (every MFMA
    // row needs all of them), then the A fragments in the order the MFMA rows use them. The reads
    // of the first half must all have returned at the barrier in the middle of the k-step, so
    // they are spread over the first three quarters of it only; those of the second half have
    // until their MFMA in the next k-step and are spread over the whole half.
    constexpr int SPAN1 = (3 * NR <= NM) ? 3 * NR : 2 * NR;
    auto read_behind = [&](auto mtag, auto spantag, bf16x8 (&dfb)[8], bf16x8 (&dfa)[TM],
                           const unsigned char* pbq, const unsigned char* paq) {
        constexpr int m = decltype(mtag)::value, SPAN = decltype(spantag)::value;
        constexpr int r = (m * NR + SPAN - 1) / SPAN;           // first read index with r * SPAN / NR >= m
        if constexpr (r < NR && (r * SPAN) / NR == m) {
            if constexpr (r < 8) dfb[r] = lds16(pbq + r * Cfg::TILE_STEP);
            else dfa[r - 8] = lds16(paq + (r - 8) * Cfg::TILE_STEP);
            MOE_FENCE();
        }
    };
    // ---- first half: MFMAs on f[0]; read f[1] (second half of this k-step); the eight B loads
    //      (with DUAL: four loads of W1 rows, then four of W3 rows)
    auto first = [&](auto mtag) {
        constexpr int m = decltype(mtag)::value, i = m >> 3, j = m & 7, n = m / (NM / 8);
        const void* src = lp.b_src(wave, n < 8 ? n : 0);
        mma16_slot<m, NM / 8, 8>(fb[0][j], fa[0][i], acc[i][j], b_region, lp.b_voff, src);
        MOE_FENCE();
        read_behind(mtag, std::integral_constant<int, SPAN1>{}, fb[1], fa[1], pb_h1, pa_h1);
        // the B pointers move on behind the last B load (MFMA 7 * NM / 8 + 3) while a later k-step exists
        constexpr int after_loads = 7 * (NM / 8) + 4;
        if constexpr (m == (after_loads < NM ? after_loads + 1 : NM - 1)) {
            lp.b_ptr[0] += (kt + NB < KT) ? Cfg::BK : 0;
            if (Cfg::DUAL) lp.b_ptr[1] += (kt + NB < KT) ? Cfg::BK : 0;
            MOE_FENCE();
        }
    };
    // ---- second half: MFMAs on f[1]; read f[0] of k-step kt+1; the A loads; the next k-step's
    //      ring addresses, one small step behind an MFMA at a time
    uint32_t sb1 = 0, sb2 = 0, sa1 = 0;
    RingState1W nx;
    auto second = [&](auto mtag) {
        constexpr int m = decltype(mtag)::value, i = m >> 3, j = m & 7;
        mma16_slot<m, 8, LA>(fb[1][j], fa[1][i], acc[i][j], a_region, lp.a_voff, lp.a_ptr);
        MOE_FENCE();
        read_behind(mtag, std::integral_constant<int, NM>{}, fb[0], fa[0], pb_n0, pa_n0);
        if constexpr (m == 1) { sb1 = rs.sb + BB; MOE_FENCE(); }
        if constexpr (m == 2) { sb1 = (sb1 == NB * BB) ? 0u : sb1; MOE_FENCE(); }        // stage of k-step kt+1
        if constexpr (m == 5) { sb2 = sb1 + BB; MOE_FENCE(); }
        if constexpr (m == 6) { sb2 = (sb2 == NB * BB) ? 0u : sb2; MOE_FENCE(); }        // ... of kt+2
        if constexpr (m == 9) { sa1 = rs.sa ^ AB; MOE_FENCE(); }                         // two A stages
        if constexpr (m == 10) { nx.pa_h1 = pa1 + sa1; MOE_FENCE(); }
        if constexpr (m == 13) { nx.pb_h1 = pb1 + sb1; MOE_FENCE(); }
        if constexpr (m == 14) { nx.pa_n0 = pa0 + rs.sa; MOE_FENCE(); }
        if constexpr (m == 17) { nx.pb_n0 = pb0 + sb2; MOE_FENCE(); }
        if constexpr (m == 18) { nx.a_region = sa1 + lp.a_lds; MOE_FENCE(); }
        if constexpr (m == 21) { nx.b_region = R::A_RING + rs.sb + lp.b_lds; MOE_FENCE(); }
        if constexpr (m == NM - 3) { lp.a_ptr += (kt + NA + 1 < KT) ? Cfg::BK : 0; MOE_FENCE(); }
    };
    static_for<NM>(first);
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" :: "n"(LB) : "memory");
    __builtin_amdgcn_s_barrier();      // k-step kt+1 complete in LDS; this k-step's stages are free
    MOE_FENCE();
    static_for<NM>(second);
    nx.sa = sa1;
    nx.sb = sb1;
    rs = nx;
}

// The first loads of a tile: A stages 0..NA-1 and B stages 0..NB-2, in the order the k-loop
// issues them; the first half of k-step 0 adds B stage NB-1 like any other k-step.
template <class Cfg, int NA, int NB>
__device__ __forceinline__ void prologue_1w(const TileCoord& tc, LoadPlan1W<Cfg>& lp, int wave, int lane,
                                            const uint16_t* __restrict__ A,
                                            const uint16_t* __restrict__ B0,
                                            const uint16_t* __restrict__ B1,
                                            const int32_t* __restrict__ row_index, int index_div,
                                            int N, int K) {
    using R = RingCfg<Cfg, NA, NB>;
    constexpr int BK = Cfg::BK, LA = R::LA, LB = R::LB, AB = Cfg::A_BYTES, BB = Cfg::B_BYTES;
    static_assert(NB - 1 == NA, "prologue order");
    lp.init(tc, wave, lane, A, B0, B1, row_index, index_div, N, K);
#pragma unroll
    for (int s = 0; s < NA; ++s) {
#pragma unroll
        for (int i = 0; i < LA; ++i) dma16(lp.a_ptr, lp.a_voff[i], s * AB + lp.a_lds + i * 1024);
        lp.a_ptr += BK;
        if (s < NB - 1) {
#pragma unroll
            for (int i = 0; i < LB; ++i)
                dma16(lp.b_src(wave, i), lp.b_voff[i], R::A_RING + s * BB + lp.b_lds + i * 1024);
            lp.b_ptr[0] += BK;
            if (Cfg::DUAL) lp.b_ptr[1] += BK;
        }
    }
}

// From the landing of k-step 0 to the last MFMA: on return every load has landed, every
// wavefront has passed the closing barrier (nobody reads a stage any more) and the accumulators
// hold the tile.
template <class Cfg, int NA, int NB>
__device__ __forceinline__ void mainloop_1w(f32x4 (&acc)[Cfg::TM][8], LoadPlan1W<Cfg>& lp,
                                            const FragPlan<Cfg>& fp, unsigned char* smem, int wave,
                                            int K) {
    using R = RingCfg<Cfg, NA, NB>;
    constexpr int BK = Cfg::BK, TM = Cfg::TM, TN = Cfg::TN;
    constexpr int LA = R::LA, LB = R::LB, AB = Cfg::A_BYTES, BB = Cfg::B_BYTES;
    static_assert(BK == 64 && NA == 2 && NB == 3 && TN == 8, "rings of 2 + 3 stages of 64 k");
    const unsigned char* pa[2] = {smem + fp.a_off[0], smem + fp.a_off[1]};
    const unsigned char* pb[2] = {smem + R::A_RING + (fp.b_off[0] - AB), smem + R::A_RING + (fp.b_off[1] - AB)};
    // The accumulators start as the result of an MFMA, 0 * 0 + 0, not as ordinary register
    // writes: the compiler may sink those to just in front of the k-loop, and it cannot know
    // that the inline assembly there is an MFMA that needs wait states after them (it did
    // exactly that once the zeroing stood after the first loads, and a few fragments came out
    // wrong). MFMA after MFMA on the same registers needs nothing.
    {
        const bf16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
        asm volatile("s_nop 4" :: "v"(zero));
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %1, 0" : "=a"(acc[i][j]) : "v"(zero));
    }

    const int KT = K / BK;                           // >= NB (checked by the launcher)
    wait_vmcnt<(NA - 1) * (LA + LB)>();              // k-step 0 landed
    __builtin_amdgcn_s_barrier();
    bf16x8 fa[2][TM], fb[2][TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) fb[0][j] = lds16(pb[0] + j * Cfg::TILE_STEP);
#pragma unroll
    for (int i = 0; i < TM; ++i) fa[0][i] = lds16(pa[0] + i * Cfg::TILE_STEP);
    MOE_FENCE();

    // k-step 0: stages 0; its B loads refill the stage "before" it, NB-1, which is still empty
    RingState1W rs{pa[1], pb[1], pa[0] + AB, pb[0] + BB, lp.a_lds,
                   R::A_RING + (NB - 1) * BB + lp.b_lds, 0u, 0u};
    // two k-steps per trip (K is a multiple of 128 for every supported shape): the loop's own
    // compare-and-branch then falls between MFMAs half as often
    for (int kt = 0; kt < KT; kt += 2) {
        kstep_1w<Cfg, NA, NB>(acc, fa, fb, rs, lp, wave, pa[0], pa[1], pb[0], pb[1], kt, KT);
        kstep_1w<Cfg, NA, NB>(acc, fa, fb, rs, lp, wave, pa[0], pa[1], pb[0], pb[1], kt + 1, KT);
    }
    wait_vmcnt<0>();                                 // the refills of the last k-steps, never read
    __builtin_amdgcn_s_barrier();                    // ... have all landed; nobody reads a stage any more
    mfma_drain();                                    // before anything else touches the accumulators
}

template <class Cfg, int NA, int NB>
__device__ __forceinline__ void ring_tile_1w(const TileCoord& tc, unsigned char* smem,
                                             const uint16_t* __restrict__ A,
                                             const uint16_t* __restrict__ B0,
                                             const uint16_t* __restrict__ B1, uint16_t* __restrict__ C,
                                             const int32_t* __restrict__ row_index, int index_div,
                                             int N, int K) {
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    LoadPlan1W<Cfg> lp;
    prologue_1w<Cfg, NA, NB>(tc, lp, wave, lane, A, B0, B1, row_index, index_div, N, K);
    FragPlan<Cfg> fp;
    fp.init(lane, wave / Cfg::WN, wave % Cfg::WN);
    f32x4 acc[Cfg::TM][Cfg::TN];
    mainloop_1w<Cfg, NA, NB>(acc, lp, fp, smem, wave, K);
    store_tile_via_lds<Cfg>(acc, tc, fp, wave, lane, smem, C, N);
}

// Tiles are enumerated at Cfg::BM rows. A tile that holds at most HalfCfg::BM = Cfg::BM / 2 rows
// (an expert's short tail, or a half of a tile of the last, partial round: see locate_tile) runs
// the same pipeline at half height: it issues half the MFMAs and A loads, and takes about 0.6 of
// the time of a full tile. Every output element is still one accumulator chain over k, so the
// bits do not depend on which height computed it.
template <class Cfg, class HalfCfg, int NA, int NB>
__global__ __launch_bounds__(Cfg::NTHREADS) void grouped_gemm_ring_kernel(
    const uint16_t* __restrict__ A, const uint16_t* __restrict__ B0,
    const uint16_t* __restrict__ B1, uint16_t* __restrict__ C,
    const int32_t* __restrict__ offsets, const int32_t* __restrict__ row_index, int index_div,
    int E, int N, int K, int split_cus) {
    static_assert(HalfCfg::BM * 2 == Cfg::BM && HalfCfg::BN == Cfg::BN && HalfCfg::BK == Cfg::BK &&
                  HalfCfg::NTHREADS == Cfg::NTHREADS && HalfCfg::DUAL == Cfg::DUAL, "same n-tiling");
    static_assert(RingCfg<HalfCfg, NA, NB>::SMEM <= RingCfg<Cfg, NA, NB>::SMEM, "LDS of the full tile");
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];

    const TileCoord tc = locate_tile<Cfg::BM>(offsets, E, N / Cfg::BN_OUT, split_cus);
    if (tc.expert < 0) return;                       // uniform for the whole workgroup
    // four wavefronts of (128 or 64) x 128 outputs run the one-wavefront-per-SIMD pipeline
    if (tc.rows <= HalfCfg::BM) {
        if constexpr (HalfCfg::NW == 4 && HalfCfg::TN == 8)
            ring_tile_1w<HalfCfg, NA, NB>(tc, smem, A, B0, B1, C, row_index, index_div, N, K);
        else
            ring_tile<HalfCfg, NA, NB>(tc, smem, A, B0, B1, C, row_index, index_div, N, K);
    } else {
        if constexpr (Cfg::NW == 4 && Cfg::TN == 8)
            ring_tile_1w<Cfg, NA, NB>(tc, smem, A, B0, B1, C, row_index, index_div, N, K);
        else
            ring_tile<Cfg, NA, NB>(tc, smem, A, B0, B1, C, row_index, index_div, N, K);
    }
}

}  // namespace gemm
}  // namespace moe
