// Shared device helpers of the atom-aware bf16 GEMM kernels for gfx950:
// argument block, epilogue (bias, GELU, residual, bf16 rounding; element-wise or
// through LDS), LDS tile layout, logical-block -> tile order.
#pragma once
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
    int k_slices;        // > 1: logical block z computes k-tiles [z*KT/S, (z+1)*KT/S) into fp32 plane z of C
    int64_t c_slice;     // elements between the planes of consecutive K slices
    const float* gamma;  // NORM_LN / NORM_RMS: per-k scale of the normalised rows of A
    const float* colsum; // NORM_LN: [2, ldcs] = the rows gamma and beta multiplied with op(B)
    int64_t ldcs;
    float eps;
};

// K slices (the logical grid's z axis): slice z of S owns the k-tiles [z*KT/S, (z+1)*KT/S),
// a balanced cut that depends on nothing but z, so a slice's sum is the same in every launch.
__device__ __forceinline__ void slice_ktiles(const GemmArgs& g, uint32_t z, int KT, int& kt0, int& kt1)
{
    if (g.k_slices <= 1) { kt0 = 0; kt1 = KT; return; }
    kt0 = (int)(((int64_t)z * KT) / g.k_slices);
    kt1 = (int)(((int64_t)(z + 1) * KT) / g.k_slices);
}

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

// The same value without the store, for the epilogue that goes through LDS (m, n in range).
__device__ __forceinline__ uint16_t epilogue_bf16(const GemmArgs& g, int m, int n, float v)
{
    if (g.flags & LITHOS_F_BIAS) v += g.bias[n];
    if (g.flags & LITHOS_F_GELU) v = gelu_erf(v);
    if (g.flags & LITHOS_F_RESIDUAL) v += g.resid[(int64_t)m * g.ldr + n];
    return f32_to_bf16_rne(v);
}

// ---- epilogue of a full bf16 tile through LDS ---------------------------------
// Storing accumulators one element at a time costs a 2-byte global store per
// element (1024 wavefront-wide stores for a 256x256 tile, ~25 us: as long as 14
// k-tiles of the main loop).  Kernels built with ST = true therefore feed the
// MFMA with the operands exchanged, so that a lane holds four CONSECUTIVE
// columns of one output row per accumulator quad, write those 8 bytes into the
// (now idle) operand buffers as a row-major bf16 tile, and then store whole
// 512-byte rows with 16 bytes per lane.  Row r keeps its 16-byte piece p at
// piece p ^ (r mod pieces-per-row): the 32 lanes that write one piece of 32
// different rows then fall into different banks, and a row read back is a
// permutation of its pieces.  The values (and their rounding) are those of
// epilogue_store, so which path a tile takes never changes a bit of C.
template <int BN>
__device__ __forceinline__ int stage_index(int r, int p)
{
    constexpr int PPR = BN / 8;
    return r * BN + ((p ^ (r & (PPR - 1))) << 3);
}

// accumulator block with exchanged operands: lane holds output row (lane & 31) of the
// block and columns 8*q + 4*(lane >> 5) + t, q = 0..3, t = 0..3

// bias, GELU and residual applied in place (a no-op without those flags)
__device__ __forceinline__ void epilogue_block_swapped(const GemmArgs& g, int m, int n_glob, f32x16& acc, int lane)
{
    if (!(g.flags & (LITHOS_F_BIAS | LITHOS_F_GELU | LITHOS_F_RESIDUAL))) return;   // uniform
    static_for<16>([&](auto ee) {
        constexpr int e = decltype(ee)::value;
        const int n = n_glob + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
        float v = acc[e];
        if (g.flags & LITHOS_F_BIAS) v += g.bias[n];
        if (g.flags & LITHOS_F_GELU) v = gelu_erf(v);
        if (g.flags & LITHOS_F_RESIDUAL) v += g.resid[(int64_t)m * g.ldr + n];
        acc[e] = v;
    });
}

// the block's values rounded to bf16 into the staged tile; LO: what the first rounding dropped,
// bf16(v - bf16(v)), the second plane of a split-bf16 output
template <int BN, bool LO>
__device__ __forceinline__ void stage_block_values(uint16_t* st, int r, int n_tile, const f32x16& acc, int lane)
{
    static_for<4>([&](auto qq) {
        constexpr int q = decltype(qq)::value;
        const int nl = n_tile + 8 * q + 4 * (lane >> 5);
        uint16_t h[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const float v = acc[4 * q + t];
            h[t] = f32_to_bf16_rne(v);
            if constexpr (LO) h[t] = f32_to_bf16_rne(v - __uint_as_float((uint32_t)h[t] << 16));
        }
        *reinterpret_cast<uint2*>(st + stage_index<BN>(r, nl >> 3) + (nl & 4)) =
            make_uint2(h[0] | ((uint32_t)h[1] << 16), h[2] | ((uint32_t)h[3] << 16));
    });
}

template <int BN>
__device__ __forceinline__ void stage_block(const GemmArgs& g, uint16_t* st, int r, int m, int n_tile, int n_glob,
                                            const f32x16& acc, int lane)
{
    f32x16 v = acc;
    epilogue_block_swapped(g, m, n_glob, v, lane);
    stage_block_values<BN, false>(st, r, n_tile, v, lane);
}

// the same block of a full fp32 tile: 16 bytes (four columns) per lane and store
__device__ __forceinline__ void store_block_swapped_f32(const GemmArgs& g, float* C, int m, int n_glob, const f32x16& acc, int lane)
{
    const bool plain = !(g.flags & (LITHOS_F_BIAS | LITHOS_F_GELU | LITHOS_F_RESIDUAL));   // uniform
    static_for<4>([&](auto qq) {
        constexpr int q = decltype(qq)::value;
        const int n = n_glob + 8 * q + 4 * (lane >> 5);
        float v[4] = {acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]};
        if (!plain) {
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                if (g.flags & LITHOS_F_BIAS) v[t] += g.bias[n + t];
                if (g.flags & LITHOS_F_GELU) v[t] = gelu_erf(v[t]);
                if (g.flags & LITHOS_F_RESIDUAL) v[t] += g.resid[(int64_t)m * g.ldr + n + t];
            }
        }
        *reinterpret_cast<float4*>(C + (int64_t)m * g.ldc + n) = make_float4(v[0], v[1], v[2], v[3]);
    });
}

// the same block stored element by element (edge tiles)
__device__ __forceinline__ void store_block_swapped(const GemmArgs& g, int m, int n_glob, const f32x16& acc, int lane)
{
    static_for<16>([&](auto ee) {
        constexpr int e = decltype(ee)::value;
        epilogue_store(g, m, n_glob + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3), acc[e]);
    });
}

// LDS tiles are [rows][64] bf16 (128-byte rows of eight 16-byte chunks).
// Chunk kc of row r lives in slot kc ^ swz(r); both the row-wise MFMA operand
// reads (32 consecutive rows, one chunk) and the transposing stores (rows 8
// apart, one chunk) then touch distinct banks within every 8-lane group.
__device__ __forceinline__ int swz(int row) { return (row ^ (row >> 3)) & 7; }
__device__ __forceinline__ int lds_index(int row, int kc) { return row * 64 + ((kc ^ swz(row)) << 3); }

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

typedef void (*gemm_fn)(GemmArgs, AtomArgs);

// kernel tables, one translation unit per family
gemm_fn gemm_tile64_fn(bool ta, bool tb, bool split, bool st);
gemm_fn gemm_tile128_fn(bool ta, bool tb, bool split, bool st);
gemm_fn gemm_tile256_wide_fn(bool ta, bool tb);
gemm_fn gemm_tile256_elem_fn(bool ta, bool tb);
gemm_fn gemm_lds256_wide_fn(bool ta, bool tb);
gemm_fn gemm_lds256_elem_fn(bool ta, bool tb);
gemm_fn gemm_skinny_fn(int variant, bool a32, int norm);

constexpr int SKINNY_WAVES = 8;     // wavefronts per workgroup of the skinny kernels, each owning one slice of K
constexpr int SKINNY_NB = 2;        // 16-column blocks per workgroup of the skinny kernels

enum { V_SKINNY32 = 3, V_TILE64 = 10, V_TILE128 = 20, V_TILE256 = 30, V_LDS256 = 31,
       V_SKL4 = 40, V_SKL8 = 41, V_SKL16 = 42 };   // LDS-staged activations of at most 4 / 8 / 16 rows

} // namespace lithos
