// Atom-aware bf16 GEMM for gfx950: C = op(A) op(B) [+bias][GELU][+residual].
// This file validates a GEMM descriptor, picks the kernel and launches one atom.
//
// Kernel families (one translation unit each):
//  * gemm_lds256_kernel (gemm_lds256.hpp, gemm_lds256_{wide,elem}.hip) - 256x256 tiles, K % 64 == 0, any operand
//    layout: global memory straight into LDS, k-strided operands read with the
//    transposing LDS load; the best-effort and training-shaped GEMMs;
//  * gemm_tile_kernel (gemm_tile.hpp, gemm_tile{64,128}.hip, gemm_tile256_{wide,elem}.hip) - 64/128/256
//    tiles through registers, ragged K, split-bf16 A;
//  * gemm_skinny_*_kernel (gemm_skinny.hip) - M <= 32 rows (bf16 or fp32
//    activations) against a [N,K] bf16 weight matrix: HBM-bound, the weights are
//    streamed exactly once.  The products still go through MFMA 16x16x32
//    (weights as the row operand): on a 64-CU partition the plain vector ALUs
//    would need longer for the 2*M*N*K flops than HBM needs for the weights.
//
// Every workgroup computes the output tile named by its LOGICAL block index
// (LithOS Section 4.4), so a launch of any sub-range of blocks writes exactly
// what the full launch writes for those tiles.  No atomics; a K that is cut
// into slices (dim[5]) puts the slice on the logical grid's z axis and writes
// one fp32 plane per slice, which SUM_SLICES adds in slice order: each block's
// arithmetic depends only on its logical index.
#include "gemm_common.hpp"

namespace lithos {

// ---- host side -------------------------------------------------------------

static int tile_threads(int variant) { return (variant == 30 || variant == 31) ? 512 : (variant < 10 || variant >= 40) ? SKINNY_WAVES * 64 : 256; }

// full bf16 tiles can leave through LDS when whole 16-byte pieces of C rows are addressable
// (fp32 tiles of the same kernels are stored from registers, 16 bytes per lane)
static bool staged_epilogue(const lithos_op_t& op)
{
    if ((op.flags & LITHOS_F_OUT_SPLIT) && op.dim[4] % 8) return false;
    if (op.flags & LITHOS_F_OUT_F32) return op.ld[2] % 4 == 0 && op.dim[6] % 4 == 0 && aligned16(op.out[0]);
    return op.ld[2] % 8 == 0 && aligned16(op.out[0]);
}

static int norm_of(uint32_t flags) { return (flags & LITHOS_F_NORM_LN) ? 1 : (flags & LITHOS_F_NORM_RMS) ? 2 : 0; }

static gemm_fn variant_fn(int variant, bool ta, bool tb, bool a32, bool split, bool st, int norm)
{
    switch (variant) {
    case V_LDS256: return st ? gemm_lds256_wide_fn(ta, tb) : gemm_lds256_elem_fn(ta, tb);
    case V_TILE64: return gemm_tile64_fn(ta, tb, split, st);
    case V_TILE128: return gemm_tile128_fn(ta, tb, split, st);
    case V_TILE256: return st ? gemm_tile256_wide_fn(ta, tb) : gemm_tile256_elem_fn(ta, tb);
    default: return gemm_skinny_fn(variant, a32, norm);
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
    const int64_t slices = op.dim[5];
    if (slices < 0 || slices > LITHOS_GEMM_MAX_SLICES) return fail(LITHOS_EINVAL, "gemm: K slices (dim[5]) must be in [0, %d]", LITHOS_GEMM_MAX_SLICES);
    if (slices > 1) {
        if (!(op.flags & LITHOS_F_OUT_F32) || (op.flags & (LITHOS_F_BIAS | LITHOS_F_GELU | LITHOS_F_RESIDUAL | LITHOS_F_OUT_SPLIT | LITHOS_F_IN_F32)))
            return fail(LITHOS_EINVAL, "gemm: K slices write plain fp32 partial planes (OUT_F32, no epilogue flags); SUM_SLICES applies the epilogue");
        if (op.dim[6] < M * ldc) return fail(LITHOS_EINVAL, "gemm: slice plane stride (dim[6]) smaller than M*ldc");
        if (slices > (K + 63) / 64) return fail(LITHOS_EINVAL, "gemm: more K slices than 64-wide k-tiles");
    }
    const int norm = norm_of(op.flags);
    const bool glu = op.flags & LITHOS_F_GLU, fused = norm || glu;
    int tile = op.tile;
    if (a32 && !(M <= 32 && tb && !ta && (tile == 0 || tile == LITHOS_TILE_SKINNY)))
        return fail(LITHOS_EINVAL, "gemm: fp32 activations (IN_F32) are only taken by the skinny kernel (M <= 32, TRANS_B)");
    if (tile == 0) {
        if (M <= 32 && tb && !ta && slices <= 1) tile = LITHOS_TILE_SKINNY;
        else if (!split && ((M + 255) / 256) * ((N + 255) / 256) >= 256) tile = 256;
        else if (((M + 127) / 128) * ((N + 127) / 128) >= 128) tile = 128;
        else tile = 64;
    }
    int variant;
    if (tile == LITHOS_TILE_SKINNY) {
        if (split) return fail(LITHOS_EINVAL, "gemm: the skinny kernel takes fp32 activations instead of SPLIT_A");
        if (slices > 1) return fail(LITHOS_EINVAL, "gemm: the skinny kernel splits K inside the workgroup; K slices need a tile kernel");
        if (M > 32 || !tb || ta) return fail(LITHOS_EINVAL, "gemm: the skinny kernel needs M <= 32, TRANS_B and no TRANS_A");
        if (N * ldb * 2 >= (1ll << 32)) return fail(LITHOS_EINVAL, "gemm: the skinny kernel addresses weight rows with 32-bit byte offsets (N*ldb*2 < 4 GiB)");
        if (a32 && (lda % 4)) return fail(LITHOS_EINVAL, "gemm: fp32 activations need lda %% 4 == 0");
        variant = V_SKINNY32;
        if (M <= 16) variant = M <= 4 ? V_SKL4 : M <= 8 ? V_SKL8 : V_SKL16;
        if (fused && M > 16) return fail(LITHOS_EINVAL, "gemm: NORM_LN, NORM_RMS and GLU need M <= 16");
        if (norm) {
            if ((op.flags & LITHOS_F_NORM_LN) && (op.flags & LITHOS_F_NORM_RMS)) return fail(LITHOS_EINVAL, "gemm: NORM_LN and NORM_RMS exclude each other");
            if (!a32) return fail(LITHOS_EINVAL, "gemm: NORM_LN / NORM_RMS need fp32 activations (IN_F32)");
            if (!op.in[4] || ((op.flags & LITHOS_F_NORM_LN) && !op.in[5])) return fail(LITHOS_EINVAL, "gemm: NORM_* set but gamma (in[4]) or the column sums (in[5]) are null");
            if ((op.flags & LITHOS_F_NORM_LN) && op.dim[7] < (glu ? 2 * N : N)) return fail(LITHOS_EINVAL, "gemm: NORM_LN needs the row stride of the column sums (dim[7]) >= the rows of B");
            if (!(op.fparam[0] >= 0.0f)) return fail(LITHOS_EINVAL, "gemm: NORM_* needs eps (fparam0) >= 0");
        }
        if (glu) {
            if (op.flags & (LITHOS_F_BIAS | LITHOS_F_GELU | LITHOS_F_RESIDUAL | LITHOS_F_OUT_SPLIT)) return fail(LITHOS_EINVAL, "gemm: GLU takes no BIAS, GELU, RESIDUAL or OUT_SPLIT");
            if (2 * N * ldb * 2 >= (1ll << 32)) return fail(LITHOS_EINVAL, "gemm: the skinny kernel addresses weight rows with 32-bit byte offsets (2N*ldb*2 < 4 GiB with GLU)");
        }
        plan->grid = {(uint32_t)(glu ? (N + 15) / 16 : (N + 16 * SKINNY_NB - 1) / (16 * SKINNY_NB)), 1, 1};
    } else if (tile == 64 || tile == 128 || tile == 256) {
        if (fused) return fail(LITHOS_EINVAL, "gemm: NORM_LN, NORM_RMS and GLU are built into the weight-streaming kernel only (TRANS_B, M <= 16)");
        if (split && tile == 256) return fail(LITHOS_EINVAL, "gemm: SPLIT_A is built for the 64 and 128 tiles only");
        variant = tile == 64 ? V_TILE64 : tile == 128 ? V_TILE128 : V_TILE256;
        if (tile == 256 && K % 64 == 0) variant = V_LDS256;
        plan->grid = {(uint32_t)((N + tile - 1) / tile), (uint32_t)((M + tile - 1) / tile), (uint32_t)(slices > 1 ? slices : 1)};
    } else {
        return fail(LITHOS_EINVAL, "gemm: unknown tile selector %d", tile);
    }
    plan->total = plan->grid.x * plan->grid.y * plan->grid.z;
    plan->threads = tile_threads(variant);
    plan->variant = variant;
    plan->wg_per_cu = cached_occupancy((const void*)variant_fn(variant, ta, tb, a32, split, staged_epilogue(op), norm), tile_threads(variant), 1);
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
    g.k_slices = (int)op.dim[5]; g.c_slice = op.dim[6];
    g.gamma = (const float*)op.in[4]; g.colsum = (const float*)op.in[5]; g.ldcs = op.dim[7]; g.eps = op.fparam[0];
    gemm_fn fn = variant_fn(plan.variant, op.flags & LITHOS_F_TRANS_A, op.flags & LITHOS_F_TRANS_B, op.flags & LITHOS_F_IN_F32,
                            op.flags & LITHOS_F_SPLIT_A, staged_epilogue(op), norm_of(op.flags));
    LITHOS_HIP(launch_kernel(fn, dim3(LITHOS_ATOM_LAUNCH_BLOCKS(atom)), dim3(plan.threads), s, g, atom));
    return LITHOS_OK;
}

} // namespace lithos
