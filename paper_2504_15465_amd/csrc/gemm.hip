// Atom-aware bf16 GEMM for gfx950: C = op(A) op(B) [+bias][GELU][+residual].
//
// Two kernel families:
//  * gemm_tile_kernel  - MFMA (v_mfma_f32_32x32x16_bf16) on LDS-staged tiles of
//    64x64, 128x128 or 256x256 outputs, BK = 64, 4 wavefronts per workgroup;
//  * gemm_skinny_kernel - M <= 32 rows (bf16 or fp32 activations) against a
//    [N,K] bf16 weight matrix: HBM-bound, the weights are streamed exactly
//    once with 16-byte loads.  The products still go through MFMA 16x16x32
//    (weights as the row operand, activations padded to 16 rows): on a 64-CU
//    partition the plain vector ALUs would need longer for the 2*M*N*K flops
//    than HBM needs for the weights.
//
// Every workgroup computes the output tile named by its LOGICAL block index
// (LithOS Section 4.4), so a launch of any sub-range of blocks writes exactly
// what the full launch writes for those tiles.  No split-K, no atomics: each
// tile's arithmetic depends only on its logical index.
#include "common.hpp"
#include <math.h>

namespace lithos {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

struct GemmArgs {
    const uint16_t* A;
    const uint16_t* B;
    void* C;
    const float* bias;
    const float* resid;
    int M, N, K;
    int64_t lda, ldb, ldc, ldr;
    uint32_t flags;
    uint32_t tiles_m, tiles_n;
    int64_t a_plane;     // SPLIT_A: elements between the hi and the lo plane of A
    int64_t c_plane;     // OUT_SPLIT: elements between the hi and the lo plane of C
};

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);  // quiet NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

__device__ __forceinline__ float gelu_erf(float u)
{
    return 0.5f * u * (1.0f + erff(u * 0.70710678118654752440f));
}

// Compile-time loop: the body sees its index as a constant, so register
// arrays indexed with it never become memory.
template <typename F, int... Is>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, Is...>)
{
    (f(std::integral_constant<int, Is>{}), ...);
}
template <int N, typename F>
__device__ __forceinline__ void static_for(F&& f)
{
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}

__device__ __forceinline__ void epilogue_store(const GemmArgs& g, int m, int n, float v)
{
    if (m >= g.M || n >= g.N) return;
    if (g.flags & LITHOS_F_BIAS) v += g.bias[n];
    if (g.flags & LITHOS_F_GELU) v = gelu_erf(v);
    if (g.flags & LITHOS_F_RESIDUAL) v += g.resid[(int64_t)m * g.ldr + n];
    if (g.flags & LITHOS_F_OUT_F32) {
        reinterpret_cast<float*>(g.C)[(int64_t)m * g.ldc + n] = v;
    } else {
        uint16_t hi = f32_to_bf16_rne(v);
        reinterpret_cast<uint16_t*>(g.C)[(int64_t)m * g.ldc + n] = hi;
        if (g.flags & LITHOS_F_OUT_SPLIT)       // second bf16 carries what the first one dropped
            reinterpret_cast<uint16_t*>(g.C)[g.c_plane + (int64_t)m * g.ldc + n] =
                f32_to_bf16_rne(v - __uint_as_float((uint32_t)hi << 16));
    }
}

// LDS tiles are [rows][64] bf16 (128-byte rows of eight 16-byte chunks).
// Chunk kc of row r lives in slot kc ^ swz(r); both the row-wise MFMA operand
// reads (32 consecutive rows, one chunk) and the transposing stores (rows 8
// apart, one chunk) then touch distinct banks within every 8-lane group.
__device__ __forceinline__ int swz(int row) { return (row ^ (row >> 3)) & 7; }
__device__ __forceinline__ int lds_index(int row, int kc) { return row * 64 + ((kc ^ swz(row)) << 3); }

// ---- global -> register -> LDS staging of one [R x 64] operand tile ------
// KSTRIDED = false: the operand is k-contiguous in memory (A[m][k], or B given
// as [N,K]); a thread moves 16-byte chunks.
// KSTRIDED = true: the operand is stored [k][row] (row-contiguous: A given as
// [K,M], or B as [K,N]); a thread loads a KB x 8 block and writes it
// transposed, so LDS always holds k-contiguous rows.
template <int R, int T, bool KSTRIDED>
struct TileStage {
    static constexpr int NCH = R * 8 / T;                       // 16-byte registers per thread
    static constexpr int KB = KSTRIDED ? (R >= T ? 8 : 8 * R / T) : 8;
    static constexpr int NB = KSTRIDED ? (R >= T ? R / T : 1) : NCH;
    static_assert(!KSTRIDED || KB >= 2, "tile too small for this workgroup size");
    uint4 r[NCH];

    __device__ __forceinline__ void load(const uint16_t* base, int64_t ld, int row0, int rows_total,
                                         int k0, int K, int tid)
    {
        if constexpr (!KSTRIDED) {
#pragma unroll
            for (int i = 0; i < NCH; ++i) {
                int c = tid + i * T;
                int row = c >> 3, kc = c & 7;
                int gr = min(row0 + row, rows_total - 1);
                int k = k0 + kc * 8;
                uint4 v = make_uint4(0, 0, 0, 0);
                if (k < K) v = *reinterpret_cast<const uint4*>(base + (int64_t)gr * ld + k);
                r[i] = v;
            }
        } else {
#pragma unroll
            for (int i = 0; i < NB; ++i) {
                int c = tid + i * T;
                int nb = c % (R / 8), kb = c / (R / 8);
                int gr = min(row0 + nb * 8, rows_total - 8);
#pragma unroll
                for (int q = 0; q < KB; ++q) {
                    int k = k0 + kb * KB + q;
                    uint4 v = make_uint4(0, 0, 0, 0);
                    if (k < K) v = *reinterpret_cast<const uint4*>(base + (int64_t)k * ld + gr);
                    r[i * KB + q] = v;
                }
            }
        }
    }

    __device__ __forceinline__ void store(uint16_t* lds, int tid) const
    {
        if constexpr (!KSTRIDED) {
#pragma unroll
            for (int i = 0; i < NCH; ++i) {
                int c = tid + i * T;
                int row = c >> 3, kc = c & 7;
                *reinterpret_cast<uint4*>(lds + lds_index(row, kc)) = r[i];
            }
        } else {
#pragma unroll
            for (int i = 0; i < NB; ++i) {
                int c = tid + i * T;
                int nb = c % (R / 8), kb = c / (R / 8);
                int kbase = kb * KB;
#pragma unroll
                for (int j = 0; j < 8; ++j) {           // j-th row of the 8-row block
                    int row = nb * 8 + j;
                    uint32_t w[KB / 2];
#pragma unroll
                    for (int p = 0; p < KB / 2; ++p) {  // pack k = 2p, 2p+1 of row j
                        const uint4& lo4 = r[i * KB + 2 * p];
                        const uint4& hi4 = r[i * KB + 2 * p + 1];
                        uint32_t lo = (j < 2) ? lo4.x : (j < 4) ? lo4.y : (j < 6) ? lo4.z : lo4.w;
                        uint32_t hi = (j < 2) ? hi4.x : (j < 4) ? hi4.y : (j < 6) ? hi4.z : hi4.w;
                        if (j & 1) w[p] = (lo >> 16) | (hi & 0xffff0000u);
                        else       w[p] = (lo & 0xffffu) | (hi << 16);
                    }
                    uint16_t* dst = lds + lds_index(row, kbase >> 3) + (kbase & 7);
                    if constexpr (KB == 8)
                        *reinterpret_cast<uint4*>(dst) = make_uint4(w[0], w[1], w[2], w[3]);
                    else if constexpr (KB == 4)
                        *reinterpret_cast<uint2*>(dst) = make_uint2(w[0], w[1]);
                    else
                        *reinterpret_cast<uint32_t*>(dst) = w[0];
                }
            }
        }
    }
};

// Tile order inside the logical grid: groups of GM tile-rows are walked
// column-major, so 32 neighbouring logical blocks form a GM x (32/GM) patch
// that shares A and B panels in one die's L2.
__device__ __forceinline__ void tile_of_block(uint32_t lin, uint32_t tiles_m, uint32_t tiles_n,
                                              uint32_t& tm, uint32_t& tn)
{
    constexpr uint32_t GM = 4;
    uint32_t per_group = GM * tiles_n;
    uint32_t grp = lin / per_group, rem = lin % per_group;
    uint32_t first = grp * GM;
    uint32_t gm = min(tiles_m - first, GM);
    tm = first + rem % gm;
    tn = rem / gm;
}

// SPLIT: A is a pair of bf16 planes (hi, lo) whose sum carries ~16 significant
// bits of the activation; both planes are multiplied with the same B operand.
template <int BM, int BN, int WGM, int WGN, bool TA, bool TB, bool SPLIT>
__global__ __launch_bounds__(WGM * WGN * 64)
void gemm_tile_kernel(GemmArgs g, AtomArgs atom)
{
    constexpr int T = WGM * WGN * 64, BK = 64;
    constexpr int WM = BM / WGM, WN = BN / WGN, MI = WM / 32, NI = WN / 32;
    __shared__ __attribute__((aligned(16))) uint16_t As[BM * BK];
    __shared__ __attribute__((aligned(16))) uint16_t As2[SPLIT ? BM * BK : 8];
    __shared__ __attribute__((aligned(16))) uint16_t Bs[BN * BK];

    const uint32_t L = atom_logical_block(atom);
    const Block3 blk = atom_delinearize(L, atom);
    uint32_t tm, tn;
    tile_of_block((blk.z * atom.gy + blk.y) * atom.gx + blk.x, g.tiles_m, g.tiles_n, tm, tn);
    const int m0 = tm * BM, n0 = tn * BN;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WGN, wn = wave % WGN;

    f32x16 acc[MI][NI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    TileStage<BM, T, TA> sa;        // A is k-strided in memory when transposed
    TileStage<SPLIT ? BM : T / 8, T, TA && SPLIT> sa2;   // lo plane of A (a dummy 32-row stage when unused)
    TileStage<BN, T, !TB> sb;       // B is k-strided in memory when NOT transposed

    const int KT = (g.K + BK - 1) / BK;
    sa.load(g.A, g.lda, m0, g.M, 0, g.K, tid);
    if constexpr (SPLIT) sa2.load(g.A + g.a_plane, g.lda, m0, g.M, 0, g.K, tid);
    sb.load(g.B, g.ldb, n0, g.N, 0, g.K, tid);
    sa.store(As, tid);
    if constexpr (SPLIT) sa2.store(As2, tid);
    sb.store(Bs, tid);
    __syncthreads();

    for (int kt = 0; kt < KT; ++kt) {
        if (kt + 1 < KT) {          // next tile's global loads fly during the MFMAs
            sa.load(g.A, g.lda, m0, g.M, (kt + 1) * BK, g.K, tid);
            if constexpr (SPLIT) sa2.load(g.A + g.a_plane, g.lda, m0, g.M, (kt + 1) * BK, g.K, tid);
            sb.load(g.B, g.ldb, n0, g.N, (kt + 1) * BK, g.K, tid);
        }
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            const int kc = kk * 2 + (lane >> 5);
            bf16x8 af[MI], af2[MI], bfr[NI];
#pragma unroll
            for (int i = 0; i < MI; ++i) {
                int row = wm * WM + i * 32 + (lane & 31);
                af[i] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(As + lds_index(row, kc)));
                if constexpr (SPLIT)
                    af2[i] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(As2 + lds_index(row, kc)));
            }
#pragma unroll
            for (int j = 0; j < NI; ++j) {
                int row = wn * WN + j * 32 + (lane & 31);
                bfr[j] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(Bs + lds_index(row, kc)));
            }
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < NI; ++j) {
                    if constexpr (SPLIT)    // small term first
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af2[i], bfr[j], acc[i][j], 0, 0, 0);
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
                }
        }
        __syncthreads();            // every wave is done reading this tile
        if (kt + 1 < KT) {
            sa.store(As, tid);
            if constexpr (SPLIT) sa2.store(As2, tid);
            sb.store(Bs, tid);
            __syncthreads();
        }
    }

    // 32x32 accumulator block: lane holds column (lane & 31); element e is
    // row 8*(e/4) + 4*(lane/32) + e%4.
    static_for<MI * NI>([&](auto ij) {
        constexpr int i = decltype(ij)::value / NI, j = decltype(ij)::value % NI;
        const int n = n0 + wn * WN + j * 32 + (lane & 31);
        const int mb = m0 + wm * WM + i * 32 + 4 * (lane >> 5);
        static_for<16>([&](auto ee) {
            constexpr int e = decltype(ee)::value;
            epilogue_store(g, mb + 8 * (e >> 2) + (e & 3), n, acc[i][j][e]);
        });
    });
}

// ---- 256x256 tile, both operands k-contiguous, global -> LDS without registers ---
// C = A B^T with A [M,K] and B [N,K] (TRANS_B), K a multiple of 64.  The k-tiles go
// from global memory straight into LDS (global_load_lds_dwordx4: the 64 lanes of a
// wavefront fill 1 KB of LDS in lane order, so each lane fetches the 16-byte chunk
// that the swizzled layout wants at its position).  That frees the 32 staging
// registers of the general kernel, which pay for a second set of operand fragments:
// the LDS reads of step kk+1 are issued before the MFMAs of step kk.
typedef const __attribute__((address_space(1))) void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

template <int WGM, int WGN>
__global__ __launch_bounds__(WGM * WGN * 64)
void gemm_nt256_kernel(GemmArgs g, AtomArgs atom)
{
    constexpr int BM = 256, BN = 256, BK = 64, WM = BM / WGM, WN = BN / WGN, MI = WM / 32, NI = WN / 32;
    constexpr int NBLK = 32 / (WGM * WGN);          // 1 KB blocks of each operand that a wavefront fetches
    // four separate arrays, each addressed statically: the compiler can then tell that the
    // LDS reads of one stage do not depend on the loads in flight into the other
    __shared__ __attribute__((aligned(1024))) uint16_t A0[BM * BK];
    __shared__ __attribute__((aligned(1024))) uint16_t A1[BM * BK];
    __shared__ __attribute__((aligned(1024))) uint16_t B0[BN * BK];
    __shared__ __attribute__((aligned(1024))) uint16_t B1[BN * BK];

    const uint32_t L = atom_logical_block(atom);
    const Block3 blk = atom_delinearize(L, atom);
    uint32_t tm, tn;
    tile_of_block((blk.z * atom.gy + blk.y) * atom.gx + blk.x, g.tiles_m, g.tiles_n, tm, tn);
    const int m0 = tm * BM, n0 = tn * BN;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WGN, wn = wave % WGN;

    f32x16 acc[MI][NI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    // Wavefront w fills LDS blocks 4w..4w+3 of each operand; a block is 8 rows x 8 chunks
    // of 16 bytes, and lane l lands on row l/8, stored chunk l%8, which holds the logical
    // chunk (l%8) ^ swizzle(row).  Rows beyond the matrix re-read its last row.
    const uint16_t* ga[NBLK];
    const uint16_t* gb[NBLK];
#pragma unroll
    for (int i = 0; i < NBLK; ++i) {
        const int row = (wave * NBLK + i) * 8 + (lane >> 3);
        const int kc = (lane & 7) ^ ((row ^ (row >> 3)) & 7);
        ga[i] = g.A + (int64_t)min(m0 + row, g.M - 1) * g.lda + kc * 8;
        gb[i] = g.B + (int64_t)min(n0 + row, g.N - 1) * g.ldb + kc * 8;
    }
    auto fetch1 = [&](uint16_t* Ad, uint16_t* Bd, int k0, int i) {
        __builtin_amdgcn_global_load_lds((gptr_t)(ga[i] + k0), (lptr_t)(Ad + (wave * NBLK + i) * 512), 16, 0, 0);
        __builtin_amdgcn_global_load_lds((gptr_t)(gb[i] + k0), (lptr_t)(Bd + (wave * NBLK + i) * 512), 16, 0, 0);
    };
    auto fetch = [&](uint16_t* Ad, uint16_t* Bd, int k0) {
#pragma unroll
        for (int i = 0; i < NBLK; ++i) fetch1(Ad, Bd, k0, i);
    };

    const int KT = g.K / BK;
    // Operand fragments: set 0 and set 1 alternate between the four 16-wide k-steps of a tile.
    bf16x8 af[2][MI], bfr[2][NI];
    auto read_frags = [&](const uint16_t* Ac, const uint16_t* Bc, int kk, bf16x8 (&a)[MI], bf16x8 (&b)[NI]) {
        const int kc = kk * 2 + (lane >> 5);
#pragma unroll
        for (int i = 0; i < MI; ++i)
            a[i] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(Ac + lds_index(wm * WM + i * 32 + (lane & 31), kc)));
#pragma unroll
        for (int j = 0; j < NI; ++j)
            b[j] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(Bc + lds_index(wn * WN + j * 32 + (lane & 31), kc)));
    };
    // the MFMAs of one step; the LDS reads of the next step are issued after the first NI of
    // them, so that the wait in front of a step only covers reads that are a step old
    auto mfmas = [&](const bf16x8 (&a)[MI], const bf16x8 (&b)[NI], int i0, int i1) {
#pragma unroll
        for (int i = i0; i < i1; ++i)
#pragma unroll
            for (int j = 0; j < NI; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    };
    // One k-tile.  On entry set 0 holds step 0 of this tile (read after the previous barrier).
    // The next tile lands in stage (An, Bn), last read before the previous barrier, while
    // this one is multiplied; the reads of a step precede most MFMAs of the step before it,
    // also across the barrier: the last step's MFMAs cover the first reads of the next
    // tile, which all wavefronts issue at once when the barrier opens.
    auto tile_step = [&](const uint16_t* Ac, const uint16_t* Bc, uint16_t* An, uint16_t* Bn, int kt) {
        const bool more = kt + 1 < KT;
        if (more) fetch(An, Bn, (kt + 1) * BK);
        __builtin_amdgcn_sched_barrier(0);
        mfmas(af[0], bfr[0], 0, 1);
        __builtin_amdgcn_sched_barrier(0);
        read_frags(Ac, Bc, 1, af[1], bfr[1]);
        __builtin_amdgcn_sched_barrier(0);
        mfmas(af[0], bfr[0], 1, MI);
        mfmas(af[1], bfr[1], 0, 1);
        __builtin_amdgcn_sched_barrier(0);
        read_frags(Ac, Bc, 2, af[0], bfr[0]);
        __builtin_amdgcn_sched_barrier(0);
        mfmas(af[1], bfr[1], 1, MI);
        mfmas(af[0], bfr[0], 0, 1);
        __builtin_amdgcn_sched_barrier(0);
        read_frags(Ac, Bc, 3, af[1], bfr[1]);
        __builtin_amdgcn_sched_barrier(0);
        mfmas(af[0], bfr[0], 1, MI);
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0): the next tile's chunks of this wavefront have landed
        __syncthreads();                      // ... and everybody's; everybody is done reading this tile
        __builtin_amdgcn_sched_barrier(0);
        mfmas(af[1], bfr[1], 0, 1);
        __builtin_amdgcn_sched_barrier(0);
        if (more) read_frags(An, Bn, 0, af[0], bfr[0]);
        __builtin_amdgcn_sched_barrier(0);
        mfmas(af[1], bfr[1], 1, MI);
        __builtin_amdgcn_sched_barrier(0);
    };

    fetch(A0, B0, 0);
    __builtin_amdgcn_s_waitcnt(0x0f70);
    __syncthreads();
    read_frags(A0, B0, 0, af[0], bfr[0]);
    for (int kt = 0; kt < KT; kt += 2) {
        tile_step(A0, B0, A1, B1, kt);
        if (kt + 1 < KT) tile_step(A1, B1, A0, B0, kt + 1);
    }

    static_for<MI * NI>([&](auto ij) {
        constexpr int i = decltype(ij)::value / NI, j = decltype(ij)::value % NI;
        const int n = n0 + wn * WN + j * 32 + (lane & 31);
        const int mb = m0 + wm * WM + i * 32 + 4 * (lane >> 5);
        static_for<16>([&](auto ee) {
            constexpr int e = decltype(ee)::value;
            epilogue_store(g, mb + 8 * (e >> 2) + (e & 3), n, acc[i][j][e]);
        });
    });
}

// ---- skinny: M <= 32 rows, B stored [N,K] -----------------------------------
// out[m][n] = sum_k x[m][k] W[n][k] on MFMA 16x16x32 with the WEIGHTS as the
// row operand: D[n][m] += W[n][k..k+31] x[m][k..k+31].  A workgroup owns 16*NB
// output columns; its eight wavefronts split K in equal slices and their partial
// tiles are added in wave order through LDS.  Every lane streams 16 bytes of
// one weight row per step (64 contiguous bytes per row and step, rows walked
// sequentially), so the weight matrix is read from HBM exactly once.
// fp32 activations are fed exactly: x = hi + mid + lo with three bf16 values
// (8 + 8 + 8 significant bits), three MFMAs per weight operand.
typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ bf16x8 pack_hi16(const float (&v)[8])
{
    // keep the upper 16 bits of each fp32 (truncation): a bf16 value
    uint32_t w[4];
#pragma unroll
    for (int p = 0; p < 4; ++p)
        w[p] = (__float_as_uint(v[2 * p]) >> 16) | (__float_as_uint(v[2 * p + 1]) & 0xffff0000u);
    return __builtin_bit_cast(bf16x8, make_uint4(w[0], w[1], w[2], w[3]));
}

// One register buffer of the skinny kernel: U k-steps of weights and activations.
template <int MB, int NB, bool A32, int U>
struct SkinnyBuf {
    uint4 wv[U][NB];
    uint4 xv[U][MB][A32 ? 2 : 1];

    // step = index of the first of U consecutive 32-wide k-steps; the slice is walked
    // cyclically from a per-workgroup rotation so that the workgroups, whose weight rows
    // are a power-of-two stride apart, do not all address the same memory channels.
    __device__ __forceinline__ void load(const GemmArgs& g, const uint16_t* const (&wrow)[NB], const bool (&mlive)[MB],
                                         int step, int nsteps, int rot, int kbeg, int kend, int r16, int kg)
    {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            // Loads are unconditional (addresses clamped into the matrix) and dead lanes are
            // zeroed afterwards: straight-line loads let the hardware keep both register
            // buffers' requests in flight, which branches around loads would prevent.
            const int st = step + u;
            const int k = kbeg + ((st + rot) % nsteps) * 32 + kg * 8;
            const bool klive = st < nsteps && k < kend;
            const int kc = min(k, g.K - 8);
            const uint4 zero = make_uint4(0, 0, 0, 0);
#pragma unroll
            for (int j = 0; j < NB; ++j) {
                const uint4 v = *reinterpret_cast<const uint4*>(wrow[j] + kc);
                wv[u][j] = klive ? v : zero;
            }
#pragma unroll
            for (int i = 0; i < MB; ++i) {
                const int64_t row = min(i * 16 + r16, g.M - 1);
                const bool live = klive && mlive[i];
                if constexpr (A32) {
                    const float* xp = reinterpret_cast<const float*>(g.A) + row * g.lda + kc;
                    const uint4 v0 = *reinterpret_cast<const uint4*>(xp);
                    const uint4 v1 = *reinterpret_cast<const uint4*>(xp + 4);
                    xv[u][i][0] = live ? v0 : zero;
                    xv[u][i][1] = live ? v1 : zero;
                } else {
                    const uint4 v0 = *reinterpret_cast<const uint4*>(g.A + row * g.lda + kc);
                    xv[u][i][0] = live ? v0 : zero;
                }
            }
        }
    }

    __device__ __forceinline__ void compute(f32x4 (&acc)[MB][NB]) const
    {
#pragma unroll
        for (int u = 0; u < U; ++u) {
#pragma unroll
            for (int i = 0; i < MB; ++i) {
                if constexpr (A32) {
                    float x[8], r1[8], r2[8];
                    const uint4 a = xv[u][i][0], b = xv[u][i][1];
                    const uint32_t raw[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        x[e] = __uint_as_float(raw[e]);
                        r1[e] = x[e] - __uint_as_float(raw[e] & 0xffff0000u);               // exact
                        r2[e] = r1[e] - __uint_as_float(__float_as_uint(r1[e]) & 0xffff0000u);  // exact, <= 8 bits
                    }
                    const bf16x8 xh = pack_hi16(x), xm = pack_hi16(r1), xl = pack_hi16(r2);
#pragma unroll
                    for (int j = 0; j < NB; ++j) {
                        const bf16x8 wf = __builtin_bit_cast(bf16x8, wv[u][j]);
                        acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf, xl, acc[i][j], 0, 0, 0);
                        acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf, xm, acc[i][j], 0, 0, 0);
                        acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf, xh, acc[i][j], 0, 0, 0);
                    }
                } else {
                    const bf16x8 xf = __builtin_bit_cast(bf16x8, xv[u][i][0]);
#pragma unroll
                    for (int j = 0; j < NB; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wv[u][j]), xf,
                                                                             acc[i][j], 0, 0, 0);
                }
            }
        }
    }
};

constexpr int SKINNY_WAVES = 8;     // wavefronts per workgroup, each owning one slice of K

template <int MB, int NB, bool A32>
__global__ __launch_bounds__(SKINNY_WAVES * 64)
void gemm_skinny_kernel(GemmArgs g, AtomArgs atom)
{
    constexpr int U = 2, KW = SKINNY_WAVES;     // two register buffers of U k-steps each
    __shared__ __attribute__((aligned(16))) float red[KW][MB][NB][64][4];

    const uint32_t L = atom_logical_block(atom);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r16 = lane & 15, kg = lane >> 4;
    const int n0 = (int)L * 16 * NB;
    // this wavefront's K range: equal slices rounded to whole 32-wide steps
    const int kq = ((g.K + 32 * KW - 1) / (32 * KW)) * 32;
    const int kbeg = wave * kq, kend = min(g.K, kbeg + kq);

    f32x4 acc[MB][NB];
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

    const uint16_t* wrow[NB];
#pragma unroll
    for (int j = 0; j < NB; ++j) wrow[j] = g.B + (int64_t)min(n0 + j * 16 + r16, g.N - 1) * g.ldb;
    bool mlive[MB];
#pragma unroll
    for (int i = 0; i < MB; ++i) mlive[i] = (i * 16 + r16) < g.M;

    // software pipeline: the other buffer's loads are in flight while one is multiplied
    const int nsteps = max(1, (kend - kbeg + 31) / 32);
    const int rot = (int)((L * 7u + (uint32_t)wave * 3u) % (uint32_t)nsteps);
    SkinnyBuf<MB, NB, A32, U> b0, b1;
    b0.load(g, wrow, mlive, 0, nsteps, rot, kbeg, kend, r16, kg);
    for (int st = 0; st < nsteps; st += 2 * U) {
        b1.load(g, wrow, mlive, st + U, nsteps, rot, kbeg, kend, r16, kg);
        b0.compute(acc);
        b0.load(g, wrow, mlive, st + 2 * U, nsteps, rot, kbeg, kend, r16, kg);
        b1.compute(acc);
    }

#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j)
            *reinterpret_cast<f32x4*>(&red[wave][i][j][lane][0]) = acc[i][j];
    __syncthreads();
    if (wave == 0) {
        // accumulator element e of a lane is D[n = 4*kg + e][m = r16]; slices are added in wave order
#pragma unroll
        for (int i = 0; i < MB; ++i)
#pragma unroll
            for (int j = 0; j < NB; ++j)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    float v = red[0][i][j][lane][e];
#pragma unroll
                    for (int w = 1; w < KW; ++w) v += red[w][i][j][lane][e];
                    epilogue_store(g, i * 16 + r16, n0 + j * 16 + 4 * kg + e, v);
                }
    }
}

// ---- skinny GEMM, fp32 activations of at most 16 rows -------------------------
// The kernel above loads activations straight into the MFMA operand layout,
// which pads them to 16 rows: with 8 (or 4) live rows half (three quarters) of
// those loads, and of the work of splitting fp32 into three bf16 values, is
// spent on padding, and the padded activation loads take as many vector-memory
// cycles as the weights.  Here a wavefront loads only the live rows of its
// next K chunk (coalesced), splits them once and keeps the three bf16 planes in
// its own piece of LDS, from which the operands are read; rows beyond MR read
// one shared row of zeros.  Weights go global -> registers -> MFMA as before.
__device__ __forceinline__ void wave_lds_sync()
{
    // LDS operations of one wavefront complete in order; this only stops the compiler
    // from moving reads of other lanes' data across the writes
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <int MR, int NB, int CH, bool A32>
struct SkinnyChunk {
    static constexpr int KC = CH * 32;              // k per chunk
    static constexpr int EPL = A32 ? 4 : 8;         // activation elements per lane and 16-byte load
    static constexpr int NX = MR * KC / (64 * EPL); // 16-byte loads per lane
    static_assert(MR * KC % (64 * EPL) == 0, "a chunk of activations must fill whole 64-lane 16-byte loads");
    uint4 wv[CH][NB];
    uint4 xv[NX];

    // kc0 = first k of the chunk; dead = chunk index beyond the slice
    __device__ __forceinline__ void load(const GemmArgs& g, const uint16_t* const (&wrow)[NB], int kc0, int kend, bool dead,
                                         int lane, int kg)
    {
        const uint4 zero = make_uint4(0, 0, 0, 0);
#pragma unroll
        for (int u = 0; u < CH; ++u) {
            const int k = kc0 + u * 32 + kg * 8;
            const bool klive = !dead && k < kend;
            const int kc = min(k, g.K - 8);
#pragma unroll
            for (int j = 0; j < NB; ++j) {
                const uint4 v = *reinterpret_cast<const uint4*>(wrow[j] + kc);
                wv[u][j] = klive ? v : zero;
            }
        }
#pragma unroll
        for (int i = 0; i < NX; ++i) {
            const int f = (i * 64 + lane) * EPL;
            const int row = f / KC, k = kc0 + f % KC;
            const bool live = !dead && row < g.M && k < kend;
            const int64_t at = (int64_t)min(row, g.M - 1) * g.lda + min(k, g.K - EPL);
            uint4 v;
            if constexpr (A32) v = *reinterpret_cast<const uint4*>(reinterpret_cast<const float*>(g.A) + at);
            else v = *reinterpret_cast<const uint4*>(g.A + at);
            xv[i] = live ? v : zero;
        }
    }

    // x = hi + mid + lo exactly, each a bf16 value (upper 16 bits kept); planes are PL elements apart
    template <int ROW, int PL>
    __device__ __forceinline__ void stage(uint16_t* xs, int lane) const
    {
#pragma unroll
        for (int i = 0; i < NX; ++i) {
            const int f = (i * 64 + lane) * EPL;
            uint16_t* dst = xs + (f / KC) * ROW + f % KC;
            if constexpr (!A32) {
                *reinterpret_cast<uint4*>(dst) = xv[i];
                continue;
            }
            const float x[4] = {__uint_as_float(xv[i].x), __uint_as_float(xv[i].y), __uint_as_float(xv[i].z), __uint_as_float(xv[i].w)};
            uint32_t h[4], m[4], l[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                h[e] = __float_as_uint(x[e]) & 0xffff0000u;
                const float r1 = x[e] - __uint_as_float(h[e]);                 // exact
                m[e] = __float_as_uint(r1) & 0xffff0000u;
                const float r2 = r1 - __uint_as_float(m[e]);                   // exact, at most 8 bits
                l[e] = __float_as_uint(r2) & 0xffff0000u;
            }
            *reinterpret_cast<uint2*>(dst) = make_uint2((h[0] >> 16) | h[1], (h[2] >> 16) | h[3]);
            *reinterpret_cast<uint2*>(dst + PL) = make_uint2((m[0] >> 16) | m[1], (m[2] >> 16) | m[3]);
            *reinterpret_cast<uint2*>(dst + 2 * PL) = make_uint2((l[0] >> 16) | l[1], (l[2] >> 16) | l[3]);
        }
    }

    template <int ROW, int PL>
    __device__ __forceinline__ void compute(const uint16_t* xrow, int kg, f32x4 (&acc)[NB]) const
    {
#pragma unroll
        for (int u = 0; u < CH; ++u) {
            const uint16_t* xp = xrow + u * 32 + kg * 8;
            const bf16x8 xh = *reinterpret_cast<const bf16x8*>(xp);
            if constexpr (A32) {
                const bf16x8 xm = *reinterpret_cast<const bf16x8*>(xp + PL);
                const bf16x8 xl = *reinterpret_cast<const bf16x8*>(xp + 2 * PL);
#pragma unroll
                for (int j = 0; j < NB; ++j) {
                    const bf16x8 wf = __builtin_bit_cast(bf16x8, wv[u][j]);
                    acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf, xl, acc[j], 0, 0, 0);
                    acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf, xm, acc[j], 0, 0, 0);
                    acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf, xh, acc[j], 0, 0, 0);
                }
            } else {
#pragma unroll
                for (int j = 0; j < NB; ++j)
                    acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wv[u][j]), xh, acc[j], 0, 0, 0);
            }
        }
    }
};

template <int MR, int NB, int CH, bool A32>
__global__ __launch_bounds__(SKINNY_WAVES * 64)
void gemm_skinny_lds_kernel(GemmArgs g, AtomArgs atom)
{
    constexpr int KW = SKINNY_WAVES;
    constexpr int KC = CH * 32;
    constexpr int ROW = KC + 8;                      // padded row: 16 rows read 16 B each without bank conflicts
    constexpr int PL = (MR + 1) * ROW;               // one plane: MR rows and the row of zeros
    constexpr int NPL = A32 ? 3 : 1;                 // bf16 activations need no splitting
    constexpr int XBYTES = KW * NPL * PL * 2;
    constexpr int RBYTES = KW * NB * 64 * 16;
    __shared__ __attribute__((aligned(16))) unsigned char smem[XBYTES > RBYTES ? XBYTES : RBYTES];

    const uint32_t L = atom_logical_block(atom);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r16 = lane & 15, kg = lane >> 4;
    const int n0 = (int)L * 16 * NB;
    const int kq = ((g.K + 32 * KW - 1) / (32 * KW)) * 32;
    const int kbeg = wave * kq, kend = min(g.K, kbeg + kq);

    uint16_t* xs = reinterpret_cast<uint16_t*>(smem) + wave * NPL * PL;
    for (int t = lane; t < NPL * (ROW / 4); t += 64) // the row of zeros of each plane
        *reinterpret_cast<uint2*>(xs + (t / (ROW / 4)) * PL + MR * ROW + (t % (ROW / 4)) * 4) = make_uint2(0, 0);
    const uint16_t* xrow = xs + min(r16, MR) * ROW;

    f32x4 acc[NB];
#pragma unroll
    for (int j = 0; j < NB; ++j) acc[j] = f32x4{0.f, 0.f, 0.f, 0.f};
    const uint16_t* wrow[NB];
#pragma unroll
    for (int j = 0; j < NB; ++j) wrow[j] = g.B + (int64_t)min(n0 + j * 16 + r16, g.N - 1) * g.ldb + 0;

    // chunks are walked cyclically from a per-workgroup start so that workgroups, whose weight
    // rows are a power-of-two stride apart, do not address the same memory channels together
    const int nch = max(1, (kend - kbeg + KC - 1) / KC);
    int ci = (int)((L * 7u + (uint32_t)wave * 3u) % (uint32_t)nch);
    auto next_chunk = [&](int& kc0) { kc0 = kbeg + ci * KC; ci = ci + 1 == nch ? 0 : ci + 1; };

    SkinnyChunk<MR, NB, CH, A32> c0, c1;
    int kc0;
    next_chunk(kc0);
    c0.load(g, wrow, kc0, kend, false, lane, kg);
    c0.template stage<ROW, PL>(xs, lane);
    wave_lds_sync();
    for (int c = 0; c < nch; c += 2) {
        next_chunk(kc0);
        c1.load(g, wrow, kc0, kend, c + 1 >= nch, lane, kg);
        c0.template compute<ROW, PL>(xrow, kg, acc);
        wave_lds_sync();
        c1.template stage<ROW, PL>(xs, lane);
        wave_lds_sync();
        next_chunk(kc0);
        c0.load(g, wrow, kc0, kend, c + 2 >= nch, lane, kg);
        c1.template compute<ROW, PL>(xrow, kg, acc);
        wave_lds_sync();
        c0.template stage<ROW, PL>(xs, lane);
        wave_lds_sync();
    }

    __syncthreads();                                  // the reduction buffer overlays the activations
    float (*red)[NB][64][4] = reinterpret_cast<float (*)[NB][64][4]>(smem);
#pragma unroll
    for (int j = 0; j < NB; ++j) *reinterpret_cast<f32x4*>(&red[wave][j][lane][0]) = acc[j];
    __syncthreads();
    if (wave == 0) {
        // accumulator element e of a lane is D[n = 4*kg + e][m = r16]; slices are added in wave order
#pragma unroll
        for (int j = 0; j < NB; ++j)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float v = red[0][j][lane][e];
#pragma unroll
                for (int w = 1; w < KW; ++w) v += red[w][j][lane][e];
                epilogue_store(g, r16, n0 + j * 16 + 4 * kg + e, v);
            }
    }
}

// ---- host side -------------------------------------------------------------

constexpr int SKINNY_NB = 2;        // 16-column blocks per workgroup of the skinny kernels

enum { V_SKINNY32 = 3, V_TILE64 = 10, V_TILE128 = 20, V_TILE256 = 30, V_NT256 = 31,
       V_SKL4 = 40, V_SKL8 = 41, V_SKL16 = 42 };   // LDS-staged activations of at most 4 / 8 / 16 rows

typedef void (*gemm_fn)(GemmArgs, AtomArgs);

static gemm_fn tile_fn(int tile, bool ta, bool tb, bool split)
{
#define PICK(BMN, WGM, WGN)                                                                     \
    (ta ? (tb ? (gemm_fn)gemm_tile_kernel<BMN, BMN, WGM, WGN, true, true, false>                \
              : (gemm_fn)gemm_tile_kernel<BMN, BMN, WGM, WGN, true, false, false>)              \
        : (tb ? (gemm_fn)gemm_tile_kernel<BMN, BMN, WGM, WGN, false, true, false>               \
              : (gemm_fn)gemm_tile_kernel<BMN, BMN, WGM, WGN, false, false, false>))
#define PICKS(BMN)                                                                              \
    (tb ? (gemm_fn)gemm_tile_kernel<BMN, BMN, 2, 2, false, true, true>                          \
        : (gemm_fn)gemm_tile_kernel<BMN, BMN, 2, 2, false, false, true>)
    if (split) return tile == 64 ? PICKS(64) : PICKS(128);
    switch (tile) {
    case 64: return PICK(64, 2, 2);
    case 128: return PICK(128, 2, 2);
    default: return PICK(256, 2, 4);
    }
#undef PICK
#undef PICKS
}

static int tile_threads(int variant) { return (variant == 30 || variant == 31) ? 512 : (variant < 10 || variant >= 40) ? SKINNY_WAVES * 64 : 256; }

static gemm_fn variant_fn(int variant, bool ta, bool tb, bool a32, bool split)
{
    switch (variant) {
    case V_SKINNY32: return a32 ? (gemm_fn)gemm_skinny_kernel<2, SKINNY_NB, true> : (gemm_fn)gemm_skinny_kernel<2, SKINNY_NB, false>;
    case V_SKL4: return a32 ? (gemm_fn)gemm_skinny_lds_kernel<4, 2, 4, true> : (gemm_fn)gemm_skinny_lds_kernel<4, 2, 4, false>;
    case V_SKL8: return a32 ? (gemm_fn)gemm_skinny_lds_kernel<8, 2, 4, true> : (gemm_fn)gemm_skinny_lds_kernel<8, 2, 4, false>;
    case V_SKL16: return a32 ? (gemm_fn)gemm_skinny_lds_kernel<16, 2, 2, true> : (gemm_fn)gemm_skinny_lds_kernel<16, 2, 2, false>;
    case V_NT256: return (gemm_fn)gemm_nt256_kernel<2, 4>;
    case V_TILE64: return tile_fn(64, ta, tb, split);
    case V_TILE128: return tile_fn(128, ta, tb, split);
    default: return tile_fn(256, ta, tb, split);
    }
}

int gemm_plan(const lithos_op_t& op, OpPlan* plan)
{
    const int64_t M = op.dim[0], N = op.dim[1], K = op.dim[2];
    const bool ta = op.flags & LITHOS_F_TRANS_A, tb = op.flags & LITHOS_F_TRANS_B, a32 = op.flags & LITHOS_F_IN_F32;
    const bool split = op.flags & LITHOS_F_SPLIT_A, out_split = op.flags & LITHOS_F_OUT_SPLIT;
    if (M <= 0 || N <= 0 || K <= 0 || M > (1 << 30) || N > (1 << 30) || K > (1 << 30))
        return fail(LITHOS_EINVAL, "gemm: M,N,K must be positive (got %lld,%lld,%lld)", (long long)M, (long long)N, (long long)K);
    if (K % 8) return fail(LITHOS_EINVAL, "gemm: K must be a multiple of 8 (got %lld)", (long long)K);
    const int64_t lda = op.ld[0], ldb = op.ld[1], ldc = op.ld[2], ldr = op.ld[3];
    if (lda % 8 || ldb % 8) return fail(LITHOS_EINVAL, "gemm: lda and ldb must be multiples of 8");
    if (lda < (ta ? M : K) || ldb < (tb ? K : N) || ldc < N)
        return fail(LITHOS_EINVAL, "gemm: leading dimension smaller than the row length");
    if (ta && (M % 8)) return fail(LITHOS_EINVAL, "gemm: a transposed A needs M %% 8 == 0");
    if (!tb && (N % 8)) return fail(LITHOS_EINVAL, "gemm: a non-transposed B needs N %% 8 == 0");
    if (!op.in[0] || !op.in[1] || !op.out[0]) return fail(LITHOS_EINVAL, "gemm: null operand");
    if (!aligned16(op.in[0]) || !aligned16(op.in[1])) return fail(LITHOS_EINVAL, "gemm: A and B must be 16-byte aligned");
    if ((op.flags & LITHOS_F_BIAS) && !op.in[2]) return fail(LITHOS_EINVAL, "gemm: BIAS set but in[2] is null");
    if (op.flags & LITHOS_F_RESIDUAL) {
        if (!op.in[3]) return fail(LITHOS_EINVAL, "gemm: RESIDUAL set but in[3] is null");
        if (ldr < N) return fail(LITHOS_EINVAL, "gemm: ldr smaller than N");
    }
    if (split && (ta || a32 || op.dim[3] <= 0 || op.dim[3] % 8))
        return fail(LITHOS_EINVAL, "gemm: SPLIT_A needs bf16 A, no TRANS_A and a plane stride (dim[3]) that is a positive multiple of 8");
    if (out_split && ((op.flags & LITHOS_F_OUT_F32) || op.dim[4] <= 0))
        return fail(LITHOS_EINVAL, "gemm: OUT_SPLIT needs a bf16 output and a positive plane stride (dim[4])");
    int tile = op.tile;
    if (a32 && !(M <= 32 && tb && !ta && (tile == 0 || tile == LITHOS_TILE_SKINNY)))
        return fail(LITHOS_EINVAL, "gemm: fp32 activations (IN_F32) are only taken by the skinny kernel (M <= 32, TRANS_B)");
    if (tile == 0) {
        if (M <= 32 && tb && !ta) tile = LITHOS_TILE_SKINNY;
        else if (!split && ((M + 255) / 256) * ((N + 255) / 256) >= 256) tile = 256;
        else if (((M + 127) / 128) * ((N + 127) / 128) >= 128) tile = 128;
        else tile = 64;
    }
    int variant;
    if (tile == LITHOS_TILE_SKINNY) {
        if (split) return fail(LITHOS_EINVAL, "gemm: the skinny kernel takes fp32 activations instead of SPLIT_A");
        if (M > 32 || !tb || ta) return fail(LITHOS_EINVAL, "gemm: the skinny kernel needs M <= 32, TRANS_B and no TRANS_A");
        if (a32 && (lda % 4)) return fail(LITHOS_EINVAL, "gemm: fp32 activations need lda %% 4 == 0");
        variant = V_SKINNY32;
        if (M <= 16) variant = M <= 4 ? V_SKL4 : M <= 8 ? V_SKL8 : V_SKL16;
        plan->grid = {(uint32_t)((N + 16 * SKINNY_NB - 1) / (16 * SKINNY_NB)), 1, 1};
    } else if (tile == 64 || tile == 128 || tile == 256) {
        if (split && tile == 256) return fail(LITHOS_EINVAL, "gemm: SPLIT_A is built for the 64 and 128 tiles only");
        variant = tile == 64 ? V_TILE64 : tile == 128 ? V_TILE128 : V_TILE256;
        if (tile == 256 && !ta && tb && K % 64 == 0) variant = V_NT256;
        plan->grid = {(uint32_t)((N + tile - 1) / tile), (uint32_t)((M + tile - 1) / tile), 1};
    } else {
        return fail(LITHOS_EINVAL, "gemm: unknown tile selector %d", tile);
    }
    plan->total = plan->grid.x * plan->grid.y;
    plan->threads = tile_threads(variant);
    plan->variant = variant;
    int occ = 0;
    hipError_t e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ, (const void*)variant_fn(variant, ta, tb, a32, split), tile_threads(variant), 0);
    plan->wg_per_cu = (e == hipSuccess && occ > 0) ? (uint32_t)occ : 1u;
    if (e != hipSuccess) (void)hipGetLastError();
    return LITHOS_OK;
}

int gemm_launch(const lithos_op_t& op, const OpPlan& plan, const AtomArgs& atom, hipStream_t s)
{
    GemmArgs g;
    g.A = (const uint16_t*)op.in[0];
    g.B = (const uint16_t*)op.in[1];
    g.C = op.out[0];
    g.bias = (const float*)op.in[2];
    g.resid = (const float*)op.in[3];
    g.M = (int)op.dim[0]; g.N = (int)op.dim[1]; g.K = (int)op.dim[2];
    g.lda = op.ld[0]; g.ldb = op.ld[1]; g.ldc = op.ld[2]; g.ldr = op.ld[3];
    g.flags = op.flags;
    g.tiles_m = plan.grid.y; g.tiles_n = plan.grid.x;
    g.a_plane = op.dim[3]; g.c_plane = op.dim[4];
    gemm_fn fn = variant_fn(plan.variant, op.flags & LITHOS_F_TRANS_A, op.flags & LITHOS_F_TRANS_B, op.flags & LITHOS_F_IN_F32,
                            op.flags & LITHOS_F_SPLIT_A);
    LITHOS_HIP(launch_kernel(fn, dim3(atom.n), dim3(plan.threads), s, g, atom));
    return LITHOS_OK;
}

} // namespace lithos
