// Grouped expert GEMMs on the gfx950 matrix cores (paper Table 1 row 3: per expert three
// d_h x d_e bf16 matrices, 6*rows*d_h*d_e FLOPs; Section 4.1: "gated FFN execution per expert").
//
//   gate/up : H[p, j]  = bf16( SiLU(sum_i Xp[p,i] W1_e[j,i]) * (sum_i Xp[p,i] W3_e[j,i]) )
//   down    : Yp[p, c] = bf16( sum_j H[p,j] W2_e[c,j] )
// for every row p of expert e's group, offsets[e] <= p < offsets[e+1].
//
// Both are "NT" contractions: the activation row and the weight row are contiguous along the
// reduction axis, which is exactly the operand shape v_mfma_f32_32x32x16_bf16 wants (each lane
// feeds 8 consecutive k). A workgroup owns a BM x BN output tile of ONE expert; tiles are
// enumerated on the device from `offsets` (no host synchronisation, variable rows per expert,
// empty experts produce no tile). Operand tiles are staged through LDS, double buffered.
// In the gate/up kernel a workgroup's BN weight rows are BN/2 rows of W1 and the matching
// BN/2 rows of W3, interleaved in blocks of 32, so that gate and up accumulators of the same
// H element sit in the same lane and register slot and SiLU(a)*b is applied in registers.
//
// Every output element is one accumulator chain over k = 0,16,32,... with the same MFMA
// instruction in every tile configuration, so results do not depend on how many rows an
// expert has or which configuration is picked (coalesced == micro-batched, bit for bit).
#include "common.h"

namespace moe {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kXcds = 8;     // workgroups are dealt round-robin to the 8 XCDs (own L2 each)
constexpr int kGroupM = 8;   // m-tiles that sweep the n-tiles together (share weight tiles)

struct TileCoord {
    int expert;      // -1: no tile for this workgroup
    int row0;        // first row (in the permuted matrix) of the tile
    int rows;        // valid rows in the tile (1..BM)
    int nt;          // n-tile index
};

// Map a workgroup to its tile. Logical tile order: expert by expert; inside an expert groups
// of kGroupM m-tiles; inside a group the n-tiles, each visited by all m-tiles of the group in
// turn. XCD x is handed the x-th contiguous eighth of that order, so the workgroups that are
// resident together on one XCD share A rows and weight tiles in its L2.
template <int BM>
__device__ __forceinline__ TileCoord locate_tile(const int32_t* __restrict__ offsets, int E,
                                                 int NT) {
    TileCoord tc{-1, 0, 0, 0};
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
            tc.nt = in / gm;
            tc.row0 = offsets[e] + mi * BM;
            tc.rows = min(BM, m_e - mi * BM);
            return tc;
        }
        start += n_tiles;
    }
    return tc;
}

// LDS tile: ROWS rows of BK bf16 (BK*2 bytes), stored in 16-byte chunks; chunk c of row r sits
// at chunk position c ^ (r & 7) so that the 32 lanes of an MFMA operand read (same logical
// chunk, consecutive rows) spread over the banks.
template <int BK>
__device__ __forceinline__ int lds_chunk_offset(int row, int chunk) {
    constexpr int kChunksPerRow = BK / 8;
    return (row * kChunksPerRow + (chunk ^ (row & (kChunksPerRow - 1) & 7))) * 16;
}

__device__ __forceinline__ float silu(float a) { return a / (1.0f + __expf(-a)); }

template <int BM, int BN, int BK, int WM, int WN, bool DUAL>
__global__ __launch_bounds__(WM* WN * 64) void grouped_gemm_kernel(
    const uint16_t* __restrict__ A, const uint16_t* __restrict__ B0,
    const uint16_t* __restrict__ B1, uint16_t* __restrict__ C,
    const int32_t* __restrict__ offsets, int E, int N, int K) {
    constexpr int NTHREADS = WM * WN * 64;
    constexpr int WTM = BM / WM, WTN = BN / WN;       // wave tile
    constexpr int TM = WTM / 32, TN = WTN / 32;       // 32x32 MFMA tiles per wave
    constexpr int CPR = BK / 8;                       // 16-byte chunks per tile row
    constexpr int LA = BM * CPR / NTHREADS;           // chunks each thread moves, A tile
    constexpr int LB = BN * CPR / NTHREADS;           // ... B tile
    constexpr int BN_OUT = DUAL ? BN / 2 : BN;        // output columns per tile
    static_assert(BM % (WM * 32) == 0 && BN % (WN * 32) == 0, "wave tile");
    static_assert(!DUAL || TN % 2 == 0, "gate/up pairs must live in one wave");
    static_assert((BM * CPR) % NTHREADS == 0 && (BN * CPR) % NTHREADS == 0, "loader");
    static_assert(BK % 16 == 0 && CPR >= 8, "BK");

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    constexpr int A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2;
    // layout: [A buf0][A buf1][B buf0][B buf1]

    const TileCoord tc = locate_tile<BM>(offsets, E, N / BN_OUT);
    if (tc.expert < 0) return;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;

    // ---- global source pointers of this thread's chunks (rows past the group's end are
    //      clamped to its last row: always in bounds, results masked at the store)
    const uint16_t* a_src[LA];
    int a_dst[LA];
#pragma unroll
    for (int it = 0; it < LA; ++it) {
        const int c = tid + it * NTHREADS;
        const int r = c / CPR, ch = c % CPR;
        const int rr = min(r, tc.rows - 1);
        a_src[it] = A + static_cast<size_t>(tc.row0 + rr) * K + ch * 8;
        a_dst[it] = lds_chunk_offset<BK>(r, ch);
    }
    const uint16_t* b_src[LB];
    int b_dst[LB];
#pragma unroll
    for (int it = 0; it < LB; ++it) {
        const int c = tid + it * NTHREADS;
        const int r = c / CPR, ch = c % CPR;
        const uint16_t* base;
        int col;
        if (DUAL) {
            const int b32 = r >> 5;
            col = tc.nt * BN_OUT + (b32 >> 1) * 32 + (r & 31);
            base = (b32 & 1) ? B1 : B0;
        } else {
            col = tc.nt * BN_OUT + r;
            base = B0;
        }
        b_src[it] = base + (static_cast<size_t>(tc.expert) * N + col) * K + ch * 8;
        b_dst[it] = lds_chunk_offset<BK>(r, ch);
    }

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int q = 0; q < 16; ++q) acc[i][j][q] = 0.f;

    uint4 a_reg[LA], b_reg[LB];
    auto load_global = [&](int kt) {
#pragma unroll
        for (int it = 0; it < LA; ++it)
            a_reg[it] = *reinterpret_cast<const uint4*>(a_src[it] + static_cast<size_t>(kt) * BK);
#pragma unroll
        for (int it = 0; it < LB; ++it)
            b_reg[it] = *reinterpret_cast<const uint4*>(b_src[it] + static_cast<size_t>(kt) * BK);
    };
    auto store_lds = [&](int buf) {
        unsigned char* sa = smem + buf * A_BYTES;
        unsigned char* sb = smem + 2 * A_BYTES + buf * B_BYTES;
#pragma unroll
        for (int it = 0; it < LA; ++it) *reinterpret_cast<uint4*>(sa + a_dst[it]) = a_reg[it];
#pragma unroll
        for (int it = 0; it < LB; ++it) *reinterpret_cast<uint4*>(sb + b_dst[it]) = b_reg[it];
    };

    const int KT = K / BK;
    load_global(0);
    store_lds(0);
    __syncthreads();

    const int frag_row = lane & 31;      // operand row inside a 32-row MFMA tile
    const int frag_half = lane >> 5;     // which 8 of the 16 k this lane feeds

    for (int kt = 0; kt < KT; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < KT) load_global(kt + 1);
        const unsigned char* sa = smem + buf * A_BYTES;
        const unsigned char* sb = smem + 2 * A_BYTES + buf * B_BYTES;
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            bf16x8 af[TM], bfr[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i)
                af[i] = *reinterpret_cast<const bf16x8*>(
                    sa + lds_chunk_offset<BK>(wm * WTM + i * 32 + frag_row, kk * 2 + frag_half));
#pragma unroll
            for (int j = 0; j < TN; ++j)
                bfr[j] = *reinterpret_cast<const bf16x8*>(
                    sb + lds_chunk_offset<BK>(wn * WTN + j * 32 + frag_row, kk * 2 + frag_half));
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < KT) store_lds(buf ^ 1);
        __syncthreads();
    }

    // ---- epilogue. MFMA 32x32 result layout: lane holds column (lane & 31); register 4*q + r
    //      is row 8*q + 4*(lane >> 5) + r.
    const int ldc = N;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int j = 0; j < TN; j += (DUAL ? 2 : 1)) {
            int col;
            if (DUAL) {
                const int b32 = (wn * WTN) / 32 + j;
                col = tc.nt * BN_OUT + (b32 >> 1) * 32 + frag_row;
            } else {
                col = tc.nt * BN_OUT + wn * WTN + j * 32 + frag_row;
            }
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int row = wm * WTM + i * 32 + 8 * q + 4 * frag_half + r;
                    if (row < tc.rows) {
                        float v;
                        if (DUAL) v = silu(acc[i][j][4 * q + r]) * acc[i][j + 1][4 * q + r];
                        else v = acc[i][j][4 * q + r];
                        C[static_cast<size_t>(tc.row0 + row) * ldc + col] = f32_to_bf16(v);
                    }
                }
        }
    }
}

template <int BM, int BN, int BK, int WM, int WN, bool DUAL>
int launch_grouped(const moe_bf16* A, const moe_bf16* B0, const moe_bf16* B1, moe_bf16* C,
                   const int32_t* offsets, int R, int E, int N, int K, hipStream_t s) {
    constexpr int BN_OUT = DUAL ? BN / 2 : BN;
    constexpr int SMEM = 2 * (BM + BN) * BK * 2;
    if (N % BN_OUT != 0 || K % BK != 0) return MOE_ERR_UNSUPPORTED_SHAPE;
    auto kern = grouped_gemm_kernel<BM, BN, BK, WM, WN, DUAL>;
    static bool attr_set = false;
    if (!attr_set) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                hipFuncAttributeMaxDynamicSharedMemorySize, SMEM) != hipSuccess)
            return MOE_ERR_HIP;
        attr_set = true;
    }
    const long long max_mt = R / BM + E;                       // >= sum_e ceil(M_e / BM)
    long long grid = max_mt * (N / BN_OUT);
    grid = (grid + kXcds - 1) / kXcds * kXcds;
    if (grid > 0x7fffffffLL) return MOE_ERR_UNSUPPORTED_SHAPE;
    hipLaunchKernelGGL(kern, dim3(static_cast<unsigned>(grid)), dim3(WM * WN * 64), SMEM, s, A, B0,
                       B1, C, offsets, E, N, K);
    return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

// Tile configuration by average rows per expert. All configurations give identical bits.
int g_forced_config = -1;   // -1: automatic; 0,1,2: force (tests / tuning)

int pick_config(int R, int E) {
    if (g_forced_config >= 0) return g_forced_config;
    const int avg = R / (E > 0 ? E : 1);
    if (avg >= 192) return 0;
    if (avg >= 96) return 1;
    return 2;
}

}  // namespace

void set_gemm_config(int cfg) { g_forced_config = cfg; }

int launch_gateup(const moe_bf16* x_perm, const int32_t* offsets, int R, int d, int f, int E,
                  const moe_bf16* W1, const moe_bf16* W3, moe_bf16* H, hipStream_t s) {
    if (R == 0) return MOE_OK;
    switch (pick_config(R, E)) {
        case 0: return launch_grouped<256, 256, 64, 2, 4, true>(x_perm, W1, W3, H, offsets, R, E, f, d, s);
        case 1: return launch_grouped<128, 128, 64, 2, 2, true>(x_perm, W1, W3, H, offsets, R, E, f, d, s);
        default: return launch_grouped<64, 128, 64, 1, 2, true>(x_perm, W1, W3, H, offsets, R, E, f, d, s);
    }
}

int launch_down(const moe_bf16* H, const int32_t* offsets, int R, int d, int f, int E,
                const moe_bf16* W2, moe_bf16* y_perm, hipStream_t s) {
    if (R == 0) return MOE_OK;
    switch (pick_config(R, E)) {
        case 0: return launch_grouped<256, 256, 64, 2, 4, false>(H, W2, nullptr, y_perm, offsets, R, E, d, f, s);
        case 1: return launch_grouped<128, 128, 64, 2, 2, false>(H, W2, nullptr, y_perm, offsets, R, E, d, f, s);
        default: return launch_grouped<64, 64, 64, 1, 2, false>(H, W2, nullptr, y_perm, offsets, R, E, d, f, s);
    }
}

}  // namespace moe
