#pragma once
#include "gemm_common.hpp"

namespace lithos {

// ---- 256x256 tile, K a multiple of 64, global -> LDS without registers -------------
// The k-tiles go from global memory straight into LDS (global_load_lds_dwordx4: the 64
// lanes of a wavefront fill 1 KB of LDS in lane order, so each lane fetches the 16-byte
// chunk that the swizzled layout wants at its position).  That frees the 32 staging
// registers of the general kernel, which pay for a second set of operand fragments:
// the LDS reads of step kk+1 are issued before the MFMAs of step kk.
//
// An operand that is k-contiguous in memory (A [M,K]; B given as [N,K]) lies in LDS as
// [row][64 k] and a lane reads its 8 consecutive k with one 16-byte load.  An operand that
// is k-strided in memory (KSA: A given as [K,M]; KSB: B given as [K,N]) lies in LDS as it
// lies in memory, [64 k][256 rows], and is read with the transposing LDS load
// (ds_read_b64_tr_b16): within 16 lanes, source lane s supplies 4 consecutive rows of
// k-row s/4, and lane l receives row l of the four k-rows: 4 consecutive k of one row,
// which is the MFMA operand layout.  Two such loads make a fragment; nothing is
// transposed in registers.
typedef const __attribute__((address_space(1))) void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

// [64 k][256 rows] tile: 16-byte chunk c of k-row k is stored at chunk c ^ ((k & 3) << 2), so
// the four k-rows that one transposing load touches fall into different banks.
__device__ __forceinline__ int ks_index(int k, int row) { return k * 256 + ((((row >> 3) ^ ((k & 3) << 2))) << 3) + (row & 7); }

template <int WGM, int WGN, bool ST, bool KSA, bool KSB>
__global__ __launch_bounds__(WGM * WGN * 64)
void gemm_lds256_kernel(GemmArgs g, AtomArgs atom)
{
    static_assert(!ST || (WGM == 2 && WGN == 4), "the staged epilogue maps 32-row blocks to the four 64-row buffers");
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

    // Wavefront w fills LDS blocks 4w..4w+3 of each operand.  k-contiguous operand: a block is
    // 8 rows x 8 chunks of 16 bytes, and lane l lands on row l/8, stored chunk l%8, which holds
    // the logical chunk (l%8) ^ swizzle(row); rows beyond the matrix re-read its last row.
    // k-strided operand: a block is 2 k-rows x 32 chunks, lane l lands on k-row l/32, stored
    // chunk l%32; chunks beyond the matrix re-read the row's last chunk.
    auto lane_ptr = [&](auto ks, const uint16_t* base, int64_t ld, int r0, int rows, int blkno) {
        if constexpr (decltype(ks)::value) {
            const int k = blkno * 2 + (lane >> 5);
            const int c = (lane & 31) ^ ((k & 3) << 2);
            return base + (int64_t)k * ld + min(r0 + c * 8, rows - 8);
        } else {
            const int row = blkno * 8 + (lane >> 3);
            const int kc = (lane & 7) ^ ((row ^ (row >> 3)) & 7);
            return base + (int64_t)min(r0 + row, rows - 1) * ld + kc * 8;
        }
    };
    const uint16_t* ga[NBLK];
    const uint16_t* gb[NBLK];
#pragma unroll
    for (int i = 0; i < NBLK; ++i) {
        ga[i] = lane_ptr(std::bool_constant<KSA>{}, g.A, g.lda, m0, g.M, wave * NBLK + i);
        gb[i] = lane_ptr(std::bool_constant<KSB>{}, g.B, g.ldb, n0, g.N, wave * NBLK + i);
    }
    const int64_t a_kstep = KSA ? g.lda : 1, b_kstep = KSB ? g.ldb : 1;    // elements per unit of k
    auto fetch = [&](uint16_t* Ad, uint16_t* Bd, int k0) {
#pragma unroll
        for (int i = 0; i < NBLK; ++i) {
            __builtin_amdgcn_global_load_lds((gptr_t)(ga[i] + k0 * a_kstep), (lptr_t)(Ad + (wave * NBLK + i) * 512), 16, 0, 0);
            __builtin_amdgcn_global_load_lds((gptr_t)(gb[i] + k0 * b_kstep), (lptr_t)(Bd + (wave * NBLK + i) * 512), 16, 0, 0);
        }
    };

    int kt0, KT;                                    // this block's k-tiles are [kt0, KT)
    slice_ktiles(g, blk.z, g.K / BK, kt0, KT);
    if (g.k_slices > 1) g.C = reinterpret_cast<float*>(g.C) + (int64_t)blk.z * g.c_slice;
    // Operand fragments: set 0 and set 1 alternate between the four 16-wide k-steps of a tile.
    bf16x8 af[2][MI], bfr[2][NI];
    // one 32-row fragment of k-step kk: rows r0 .. r0+31 of the tile, this lane's 8 k
    auto read_frag = [&](auto ks, const uint16_t* T, int r0, int kk) -> bf16x8 {
        if constexpr (decltype(ks)::value) {
            // source lane s of a 16-lane group addresses k-row s/4, rows 4*(s%4)..+3 of the group's 16
            const int grp = lane >> 4, s = lane & 15;
            const int k = kk * 16 + 8 * (grp >> 1) + (s >> 2);
            const int row = r0 + 16 * (grp & 1) + 4 * (s & 3);
            const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(T + ks_index(k, row)));
            const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(T + ks_index(k + 4, row)));
            return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
        } else {
            return __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(T + lds_index(r0 + (lane & 31), kk * 2 + (lane >> 5))));
        }
    };
    auto read_frags = [&](const uint16_t* Ac, const uint16_t* Bc, int kk, bf16x8 (&a)[MI], bf16x8 (&b)[NI]) {
#pragma unroll
        for (int i = 0; i < MI; ++i) a[i] = read_frag(std::bool_constant<KSA>{}, Ac, wm * WM + i * 32, kk);
#pragma unroll
        for (int j = 0; j < NI; ++j) b[j] = read_frag(std::bool_constant<KSB>{}, Bc, wn * WN + j * 32, kk);
    };
    // the MFMAs of one step; the LDS reads of the next step are issued after the first NI of
    // them, so that the wait in front of a step only covers reads that are a step old
    auto mfmas = [&](const bf16x8 (&a)[MI], const bf16x8 (&b)[NI], int i0, int i1) {
#pragma unroll
        for (int i = i0; i < i1; ++i)
#pragma unroll
            for (int j = 0; j < NI; ++j) {
                if constexpr (ST) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[j], a[i], acc[i][j], 0, 0, 0);
                else acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
            }
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

    if (kt0 < KT) fetch(A0, B0, kt0 * BK);
    __builtin_amdgcn_s_waitcnt(0x0f70);
    __syncthreads();
    if (kt0 < KT) read_frags(A0, B0, 0, af[0], bfr[0]);
    for (int kt = kt0; kt < KT; kt += 2) {
        tile_step(A0, B0, A1, B1, kt);
        if (kt + 1 < KT) tile_step(A1, B1, A0, B0, kt + 1);
    }

    if constexpr (ST) {
        // the four 32 KB buffers hold rows 0-63, 64-127, 128-191, 192-255 of the bf16 tile
        if (m0 + BM <= g.M && n0 + BN <= g.N && (g.flags & LITHOS_F_OUT_F32)) {
            static_for<MI * NI>([&](auto ij) {
                constexpr int i = decltype(ij)::value / NI, j = decltype(ij)::value % NI;
                store_block_swapped_f32(g, reinterpret_cast<float*>(g.C), m0 + wm * WM + i * 32 + (lane & 31),
                                        n0 + wn * WN + j * 32, acc[i][j], lane);
            });
        } else if (m0 + BM <= g.M && n0 + BN <= g.N && !(g.flags & LITHOS_F_OUT_SPLIT)) {
            __syncthreads();
            static_for<MI * NI>([&](auto ij) {
                constexpr int i = decltype(ij)::value / NI, j = decltype(ij)::value % NI;
                uint16_t* const st = wm == 0 ? (i < 2 ? A0 : A1) : (i < 2 ? B0 : B1);
                stage_block<BN>(g, st, (i & 1) * 32 + (lane & 31), m0 + wm * WM + i * 32 + (lane & 31), wn * WN + j * 32,
                                n0 + wn * WN + j * 32, acc[i][j], lane);
            });
            __syncthreads();
            uint16_t* const C = reinterpret_cast<uint16_t*>(g.C);
            const uint16_t* const src = wave < 2 ? A0 : wave < 4 ? A1 : wave < 6 ? B0 : B1;
#pragma unroll 4
            for (int it = 0; it < 16; ++it) {            // wavefront w stores rows 32w .. 32w+31, two per step
                const int r = (wave & 1) * 32 + it * 2 + (lane >> 5), p = lane & 31;
                const uint4 v = *reinterpret_cast<const uint4*>(src + stage_index<BN>(r, p));
                *reinterpret_cast<uint4*>(C + (int64_t)(m0 + (wave >> 1) * 64 + r) * g.ldc + n0 + p * 8) = v;
            }
        } else {
            static_for<MI * NI>([&](auto ij) {
                constexpr int i = decltype(ij)::value / NI, j = decltype(ij)::value % NI;
                store_block_swapped(g, m0 + wm * WM + i * 32 + (lane & 31), n0 + wn * WN + j * 32, acc[i][j], lane);
            });
        }
        return;
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

#define LITHOS_LDS256_PICK(ST)                                                                                              \
    (ta ? (tb ? (gemm_fn)gemm_lds256_kernel<2, 4, ST, true, false> : (gemm_fn)gemm_lds256_kernel<2, 4, ST, true, true>)    \
        : (tb ? (gemm_fn)gemm_lds256_kernel<2, 4, ST, false, false> : (gemm_fn)gemm_lds256_kernel<2, 4, ST, false, true>))

} // namespace lithos
