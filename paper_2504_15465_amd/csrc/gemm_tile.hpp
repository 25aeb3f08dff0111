// LDS-staged MFMA tile GEMM (v_mfma_f32_32x32x16_bf16) for any operand layout:
// 64x64, 128x128 or 256x256 output tiles, BK = 64.  Every workgroup computes the
// tile named by its LOGICAL block index (LithOS Section 4.4).
#pragma once
#include "gemm_common.hpp"

namespace lithos {

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

// SPLIT: A is a pair of bf16 planes (hi, lo) whose sum carries ~16 significant
// bits of the activation; both planes are multiplied with the same B operand.
// ST: full bf16 tiles leave through LDS (operands exchanged in the MFMA, see stage_block).
// Registers are capped so that 256x256 tiles keep two wavefronts per SIMD (one 8-wave workgroup
// per CU), 128x128 tiles three workgroups and 64x64 tiles four: left alone, the compiler spends
// the whole register file on hoisted epilogue addresses and halves the occupancy.
template <int BM, int BN, int WGM, int WGN, bool TA, bool TB, bool SPLIT, bool ST>
__global__ __launch_bounds__(WGM * WGN * 64, BM >= 256 ? 2 : BM >= 128 ? 3 : 4)
void gemm_tile_kernel(GemmArgs g, AtomArgs atom)
{
    constexpr int T = WGM * WGN * 64, BK = 64;
    constexpr int WM = BM / WGM, WN = BN / WGN, MI = WM / 32, NI = WN / 32;
    // operand buffers; a staged epilogue needs room for the whole bf16 output tile
    constexpr int OPERAND_ELEMS = (BM + BN) * BK + (SPLIT ? BM * BK : 0);
    __shared__ __attribute__((aligned(16))) uint16_t smem[ST && BM * BN > OPERAND_ELEMS ? BM * BN : OPERAND_ELEMS];
    uint16_t* const As = smem;
    uint16_t* const Bs = smem + BM * BK;
    uint16_t* const As2 = smem + (BM + BN) * BK;

    const uint32_t L = atom_logical_block(atom);
    const Block3 blk = atom_delinearize(L, atom);
    uint32_t tm, tn;
    tile_of_block(blk.y * atom.gx + blk.x, g.tiles_m, g.tiles_n, tm, tn);   // blk.z is the K slice
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

    TileStage<BM, T, TA> sa;        // A is k-strided in memory when transposed
    TileStage<SPLIT ? BM : T / 8, T, TA && SPLIT> sa2;   // lo plane of A (a dummy 32-row stage when unused)
    TileStage<BN, T, !TB> sb;       // B is k-strided in memory when NOT transposed

    int kt0, kt1;
    slice_ktiles(g, blk.z, (g.K + BK - 1) / BK, kt0, kt1);
    const int KT = kt1;
    if (g.k_slices > 1) g.C = reinterpret_cast<float*>(g.C) + (int64_t)blk.z * g.c_slice;
    if (kt0 < kt1) {
        sa.load(g.A, g.lda, m0, g.M, kt0 * BK, g.K, tid);
        if constexpr (SPLIT) sa2.load(g.A + g.a_plane, g.lda, m0, g.M, kt0 * BK, g.K, tid);
        sb.load(g.B, g.ldb, n0, g.N, kt0 * BK, g.K, tid);
        sa.store(As, tid);
        if constexpr (SPLIT) sa2.store(As2, tid);
        sb.store(Bs, tid);
    }
    __syncthreads();

    for (int kt = kt0; kt < KT; ++kt) {
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
                    if constexpr (SPLIT && ST)    // small term first
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[j], af2[i], acc[i][j], 0, 0, 0);
                    else if constexpr (SPLIT)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af2[i], bfr[j], acc[i][j], 0, 0, 0);
                    if constexpr (ST)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[j], af[i], acc[i][j], 0, 0, 0);
                    else
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

    if constexpr (ST) {
        // the operand buffers are free after the loop's last barrier
        constexpr int PPR = BN / 8;
        if (m0 + BM <= g.M && n0 + BN <= g.N && (g.flags & LITHOS_F_OUT_F32)) {
            static_for<MI * NI>([&](auto ij) {
                constexpr int i = decltype(ij)::value / NI, j = decltype(ij)::value % NI;
                store_block_swapped_f32(g, reinterpret_cast<float*>(g.C), m0 + wm * WM + i * 32 + (lane & 31),
                                        n0 + wn * WN + j * 32, acc[i][j], lane);
            });
        } else if (m0 + BM <= g.M && n0 + BN <= g.N) {
            uint16_t* const C = reinterpret_cast<uint16_t*>(g.C);
            static_for<MI * NI>([&](auto ij) {
                constexpr int i = decltype(ij)::value / NI, j = decltype(ij)::value % NI;
                const int rb = wm * WM + i * 32;
                epilogue_block_swapped(g, m0 + rb + (lane & 31), n0 + wn * WN + j * 32, acc[i][j], lane);
                stage_block_values<BN, false>(smem, rb + (lane & 31), wn * WN + j * 32, acc[i][j], lane);
            });
            auto store_tile = [&](uint16_t* dst) {
                __syncthreads();
#pragma unroll 4
                for (int c = tid; c < BM * PPR; c += T) {
                    const int r = c / PPR, p = c % PPR;
                    const uint4 v = *reinterpret_cast<const uint4*>(smem + stage_index<BN>(r, p));
                    *reinterpret_cast<uint4*>(dst + (int64_t)(m0 + r) * g.ldc + n0 + p * 8) = v;
                }
            };
            store_tile(C);
            if (g.flags & LITHOS_F_OUT_SPLIT) {          // second plane: what the bf16 rounding dropped
                __syncthreads();
                static_for<MI * NI>([&](auto ij) {
                    constexpr int i = decltype(ij)::value / NI, j = decltype(ij)::value % NI;
                    stage_block_values<BN, true>(smem, wm * WM + i * 32 + (lane & 31), wn * WN + j * 32, acc[i][j], lane);
                });
                store_tile(C + g.c_plane);
            }
        } else {
            static_for<MI * NI>([&](auto ij) {
                constexpr int i = decltype(ij)::value / NI, j = decltype(ij)::value % NI;
                store_block_swapped(g, m0 + wm * WM + i * 32 + (lane & 31), n0 + wn * WN + j * 32, acc[i][j], lane);
            });
        }
        return;
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

#define LITHOS_TILE_PICK4(BMN, WGM, WGN, ST)                                                    \
    (ta ? (tb ? (gemm_fn)gemm_tile_kernel<BMN, BMN, WGM, WGN, true, true, false, ST>            \
              : (gemm_fn)gemm_tile_kernel<BMN, BMN, WGM, WGN, true, false, false, ST>)          \
        : (tb ? (gemm_fn)gemm_tile_kernel<BMN, BMN, WGM, WGN, false, true, false, ST>           \
              : (gemm_fn)gemm_tile_kernel<BMN, BMN, WGM, WGN, false, false, false, ST>))
#define LITHOS_TILE_PICK(BMN, WGM, WGN) (st ? LITHOS_TILE_PICK4(BMN, WGM, WGN, true) : LITHOS_TILE_PICK4(BMN, WGM, WGN, false))
#define LITHOS_TILE_PICK_SPLIT4(BMN, ST)                                                        \
    (tb ? (gemm_fn)gemm_tile_kernel<BMN, BMN, 2, 2, false, true, true, ST>                      \
        : (gemm_fn)gemm_tile_kernel<BMN, BMN, 2, 2, false, false, true, ST>)
#define LITHOS_TILE_PICK_SPLIT(BMN) (st ? LITHOS_TILE_PICK_SPLIT4(BMN, true) : LITHOS_TILE_PICK_SPLIT4(BMN, false))

} // namespace lithos
