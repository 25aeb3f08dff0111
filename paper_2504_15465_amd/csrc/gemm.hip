// Atom-aware bf16 GEMM for gfx950: C = op(A) op(B) [+bias][GELU][+residual].
//
// Two kernel families:
//  * gemm_tile_kernel  - MFMA (v_mfma_f32_32x32x16_bf16) on LDS-staged tiles of
//    64x64, 128x128 or 256x256 outputs, BK = 64, 4 wavefronts per workgroup;
//  * gemm_skinny_kernel - M <= 32 rows (bf16 or fp32 activations) against a
//    [N,K] bf16 weight matrix: the weights are streamed once from HBM with
//    16-byte loads and multiplied on the vector ALUs (the op is HBM-bound;
//    reshaping it for MFMA buys nothing).
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
template <int BM, int BN, bool TA, bool TB, bool SPLIT>
__global__ __launch_bounds__(256)
void gemm_tile_kernel(GemmArgs g, AtomArgs atom)
{
    constexpr int T = 256, BK = 64, WGM = 2, WGN = 2;
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
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j) {
            int n = n0 + wn * WN + j * 32 + (lane & 31);
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                int m = m0 + wm * WM + i * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
                epilogue_store(g, m, n, acc[i][j][e]);
            }
        }
}

// ---- skinny: M <= MT rows, B stored [N,K] ---------------------------------
// A workgroup owns 16 output columns (4 per wavefront) and walks K in stages
// of KC.  The activations x[:, stage] are staged in LDS (fp32 when the op
// gives fp32 activations, else bf16); each lane multiplies eight consecutive k
// of four weight rows with the same eight k of every x row, and a butterfly
// over the 64 lanes finishes each dot product.  The next stage's x and
// weights are already in flight (in registers) while the current one is
// computed.  Lane order and stage order are fixed, so the result is a pure
// function of the logical block index.
template <int MT, bool A32>
struct SkinnyStage {
    static constexpr int KC0 = (A32 ? 8192 : 16384) / MT;     // 32 KB of x per stage ...
    static constexpr int KC = KC0 < 512 ? 512 : KC0;          // ... but at least one k-step per lane
    static constexpr int LDS_BYTES = MT * KC * (A32 ? 4 : 2);
    static constexpr int XV = LDS_BYTES / 16 / 256;           // 16-byte x registers per thread
    static constexpr int IT = KC / 512;                       // k-steps per lane per stage
    static constexpr int NC = 4;
    uint4 x[XV];
    uint4 w[IT][NC];

    __device__ __forceinline__ void load(const GemmArgs& g, const uint16_t* const (&wrow)[NC], int k0, int tid, int lane)
    {
#pragma unroll
        for (int it = 0; it < IT; ++it) {
            int k = k0 + it * 512 + lane * 8;
#pragma unroll
            for (int c = 0; c < NC; ++c) {
                uint4 v = make_uint4(0, 0, 0, 0);
                if (k < g.K) v = *reinterpret_cast<const uint4*>(wrow[c] + k);
                w[it][c] = v;
            }
        }
        constexpr int EPV = A32 ? 4 : 8;                      // elements per 16-byte register
#pragma unroll
        for (int i = 0; i < XV; ++i) {
            int c = tid + i * 256;
            int m = c / (KC / EPV), kk = (c % (KC / EPV)) * EPV;
            uint4 v = make_uint4(0, 0, 0, 0);
            if (m < g.M && k0 + kk < g.K) {
                if constexpr (A32) v = *reinterpret_cast<const uint4*>(reinterpret_cast<const float*>(g.A) + (int64_t)m * g.lda + k0 + kk);
                else v = *reinterpret_cast<const uint4*>(g.A + (int64_t)m * g.lda + k0 + kk);
            }
            x[i] = v;
        }
    }

    // fp32 layout in LDS: the two halves (k%8 < 4, k%8 >= 4) of every 8-group
    // live in separate planes, so the 64 lanes read consecutive 16-byte slots.
    __device__ __forceinline__ void store(void* lds, int tid) const
    {
        constexpr int EPV = A32 ? 4 : 8;
#pragma unroll
        for (int i = 0; i < XV; ++i) {
            int c = tid + i * 256;
            int m = c / (KC / EPV), kk = (c % (KC / EPV)) * EPV;
            if constexpr (A32) {
                int grp = kk >> 3, half = (kk >> 2) & 1;
                reinterpret_cast<uint4*>(lds)[(m * KC + half * (KC / 2)) / 4 + grp] = x[i];
            } else {
                reinterpret_cast<uint4*>(lds)[(m * KC + kk) / 8] = x[i];
            }
        }
    }
};

template <int MT, bool A32>
__global__ __launch_bounds__(256)
void gemm_skinny_kernel(GemmArgs g, AtomArgs atom)
{
    using Stage = SkinnyStage<MT, A32>;
    constexpr int KC = Stage::KC, NC = Stage::NC, IT = Stage::IT;
    __shared__ __attribute__((aligned(16))) unsigned char xs_raw[Stage::LDS_BYTES];

    const uint32_t L = atom_logical_block(atom);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nbase = (int)L * 16 + wave * NC;

    float acc[MT][NC];
#pragma unroll
    for (int m = 0; m < MT; ++m)
#pragma unroll
        for (int c = 0; c < NC; ++c) acc[m][c] = 0.0f;

    const uint16_t* wrow[NC];
#pragma unroll
    for (int c = 0; c < NC; ++c) wrow[c] = g.B + (int64_t)min(nbase + c, g.N - 1) * g.ldb;

    Stage cur, nxt;
    cur.load(g, wrow, 0, tid, lane);
    for (int k0 = 0; k0 < g.K; k0 += KC) {
        cur.store(xs_raw, tid);
        __syncthreads();
        if (k0 + KC < g.K) nxt.load(g, wrow, k0 + KC, tid, lane);
#pragma unroll
        for (int it = 0; it < IT; ++it) {
            const int kk = it * 512 + lane * 8;          // offset inside the stage
            float wf[NC][8];
#pragma unroll
            for (int c = 0; c < NC; ++c) {
                const uint4 v = cur.w[it][c];
                const uint32_t u[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                for (int p = 0; p < 4; ++p) {
                    wf[c][2 * p] = __uint_as_float(u[p] << 16);
                    wf[c][2 * p + 1] = __uint_as_float(u[p] & 0xffff0000u);
                }
            }
#pragma unroll
            for (int m = 0; m < MT; ++m) {
                float xf[8];
                if constexpr (A32) {
                    const float* xl = reinterpret_cast<const float*>(xs_raw);
                    const float4 lo = *reinterpret_cast<const float4*>(xl + m * KC + (kk >> 3) * 4);
                    const float4 hi = *reinterpret_cast<const float4*>(xl + m * KC + KC / 2 + (kk >> 3) * 4);
                    xf[0] = lo.x; xf[1] = lo.y; xf[2] = lo.z; xf[3] = lo.w;
                    xf[4] = hi.x; xf[5] = hi.y; xf[6] = hi.z; xf[7] = hi.w;
                } else {
                    const uint4 v = *reinterpret_cast<const uint4*>(reinterpret_cast<const uint16_t*>(xs_raw) + m * KC + kk);
                    const uint32_t u[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                    for (int p = 0; p < 4; ++p) {
                        xf[2 * p] = __uint_as_float(u[p] << 16);
                        xf[2 * p + 1] = __uint_as_float(u[p] & 0xffff0000u);
                    }
                }
#pragma unroll
                for (int c = 0; c < NC; ++c)
#pragma unroll
                    for (int e = 0; e < 8; ++e) acc[m][c] = fmaf(xf[e], wf[c][e], acc[m][c]);
            }
        }
        __syncthreads();
        cur = nxt;
    }

#pragma unroll
    for (int m = 0; m < MT; ++m)
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            float v = acc[m][c];
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
            if (lane == ((m * NC + c) & 63)) epilogue_store(g, m, nbase + c, v);
        }
}

// ---- host side -------------------------------------------------------------

enum { V_SKINNY8 = 1, V_SKINNY16 = 2, V_SKINNY32 = 3, V_TILE64 = 10, V_TILE128 = 20, V_TILE256 = 30 };

typedef void (*gemm_fn)(GemmArgs, AtomArgs);

static gemm_fn tile_fn(int tile, bool ta, bool tb, bool split)
{
#define PICK(BMN)                                                                          \
    (ta ? (tb ? (gemm_fn)gemm_tile_kernel<BMN, BMN, true, true, false>                     \
              : (gemm_fn)gemm_tile_kernel<BMN, BMN, true, false, false>)                   \
        : (tb ? (gemm_fn)gemm_tile_kernel<BMN, BMN, false, true, false>                    \
              : (gemm_fn)gemm_tile_kernel<BMN, BMN, false, false, false>))
#define PICKS(BMN)                                                                         \
    (tb ? (gemm_fn)gemm_tile_kernel<BMN, BMN, false, true, true>                           \
        : (gemm_fn)gemm_tile_kernel<BMN, BMN, false, false, true>)
    if (split) return tile == 64 ? PICKS(64) : PICKS(128);
    switch (tile) {
    case 64: return PICK(64);
    case 128: return PICK(128);
    default: return PICK(256);
    }
#undef PICK
#undef PICKS
}

static gemm_fn variant_fn(int variant, bool ta, bool tb, bool a32, bool split)
{
    switch (variant) {
    case V_SKINNY8: return a32 ? (gemm_fn)gemm_skinny_kernel<8, true> : (gemm_fn)gemm_skinny_kernel<8, false>;
    case V_SKINNY16: return a32 ? (gemm_fn)gemm_skinny_kernel<16, true> : (gemm_fn)gemm_skinny_kernel<16, false>;
    case V_SKINNY32: return a32 ? (gemm_fn)gemm_skinny_kernel<32, true> : (gemm_fn)gemm_skinny_kernel<32, false>;
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
        variant = M <= 8 ? V_SKINNY8 : M <= 16 ? V_SKINNY16 : V_SKINNY32;
        plan->grid = {(uint32_t)((N + 15) / 16), 1, 1};
    } else if (tile == 64 || tile == 128 || tile == 256) {
        if (split && tile == 256) return fail(LITHOS_EINVAL, "gemm: SPLIT_A is built for the 64 and 128 tiles only");
        variant = tile == 64 ? V_TILE64 : tile == 128 ? V_TILE128 : V_TILE256;
        plan->grid = {(uint32_t)((N + tile - 1) / tile), (uint32_t)((M + tile - 1) / tile), 1};
    } else {
        return fail(LITHOS_EINVAL, "gemm: unknown tile selector %d", tile);
    }
    plan->total = plan->grid.x * plan->grid.y;
    plan->threads = 256;
    plan->variant = variant;
    int occ = 0;
    hipError_t e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ, (const void*)variant_fn(variant, ta, tb, a32, split), 256, 0);
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
    LITHOS_HIP(launch_kernel(fn, dim3(atom.n), dim3(256), s, g, atom));
    return LITHOS_OK;
}

} // namespace lithos
