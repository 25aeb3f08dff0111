#include "gemm_common.hpp"

namespace lithos {

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
// one shared row of zeros.
// Weights: a load instruction fetches whole 128-byte pieces of 8 weight rows (lane l:
// row l/8, 16-byte chunk l%8) rather than the operand layout's 64-byte pieces of 16
// rows - on a 64-CU partition the short pieces stream at 1.2 TB/s, these at up to 3.6 -
// and a 16-row block changes layout through the wavefront's own LDS piece (write as
// loaded, read back as MFMA fragments) before it is multiplied.  (256-byte pieces of 4
// rows, chunks of 128 k, stream no faster and their two register buffers leave no room
// under the 128 registers that two workgroups per CU allow: 64-wide chunks it is.)
// On a 64-CU partition a large weight matrix streams at that partition's read ceiling and
// the vector ALUs are the next limit, so the loop is kept lean: nothing is masked but the
// activations, and no load sits under a condition.
__device__ __forceinline__ void wave_lds_sync()
{
    // LDS operations of one wavefront complete in order; this only stops the compiler
    // from moving reads of other lanes' data across the writes
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// NORM: 0 = activations as stored; NORM_RMS / NORM_LN = the GEMM of the normalised rows, without a
// pass over the rows before the first chunk.  A row's statistics scale and shift whole output rows,
// so they can wait for the epilogue:
//   RMSNorm    sum_k (x r g)_k W_nk = r * sum_k (x g)_k W_nk,                   r = 1/sqrt(mean x^2 + eps);
//   LayerNorm  sum_k ((x - mu) r g + b)_k W_nk
//                = r * (sum_k ((x - c) g)_k W_nk - (mu - c) * sum_k g_k W_nk) + sum_k b_k W_nk
//              with c = the row's first element (sums of x - c and (x - c)^2 lose nothing to
//              cancellation when c lies among the data).
// The loop multiplies by gamma while it splits the activations into planes and keeps sum x^2 (and
// sum (x - c)) per lane; LayerNorm's two column vectors sum_k g_k W_nk and sum_k b_k W_nk depend on the
// weights alone and come in as an input (this kernel's own product of the rows gamma and beta).
constexpr int NORM_LN = 1, NORM_RMS = 2;

template <int NX, int NORM>
struct RowStats {
    float s1[NX], s2[NX], c[NX];      // per 16-byte load of a lane: sum (x - c), sum (x - c)^2, the shift (0 for RMSNorm)
};

template <int MR, int NB, int CH, bool A32, int NORM>
struct SkinnyChunk {
    static constexpr int KC = CH * 32;              // k per chunk
    static constexpr int EPL = A32 ? 4 : 8;         // activation elements per lane and 16-byte load
    static constexpr int NX = MR * KC / (64 * EPL); // 16-byte loads per lane
    static_assert(MR * KC % (64 * EPL) == 0, "a chunk of activations must fill whole 64-lane 16-byte loads");
    uint4 wv[CH][NB];
    uint4 xv[NX];
    float4 gv;              // NORM: gamma of this lane's four k (the same k in every one of its loads), as loaded
    static_assert((64 * EPL) % KC == 0, "a lane keeps one k offset in every one of its activation loads");
    static_assert(NORM == 0 || A32, "normalised activations are fp32");

    static constexpr int CPRW = CH * 4;             // 16-byte chunks of a weight row per chunk of K
    static constexpr int RPI = 64 / CPRW;           // weight rows per load instruction

    bool xlive;             // this lane's k of the activation loads (the same in each) lie inside the wavefront's slice

    // kc0 = first k of the chunk; dead = chunk index beyond the slice.  woff[u][j] = byte offset of
    // the weight row that instruction u of 16-row block j reads for this lane (row u*RPI + lane/CPRW).
    // Loads are unconditional, their addresses clamped into the operands.  Outside the slice the
    // ACTIVATIONS are zeroed when they are staged; the weights are used as they come: a clamped
    // address stays in its weight row, whose other elements enter the same outputs anyway, and
    // finite values times zero add nothing.  Rows beyond M repeat row M - 1: they only reach output
    // rows that are never stored.
    __device__ __forceinline__ void load(const GemmArgs& g, const uint32_t (&woff)[CH][NB], int kc0, int kend, bool dead, int lane)
    {
        const int k = kc0 + (lane % CPRW) * 8;
        const int kx = kc0 + (lane * EPL) % KC;
        xlive = !dead && kx < kend;
        const char* wk = reinterpret_cast<const char*>(g.B) + (size_t)min(k, g.K - 8) * 2;
#pragma unroll
        for (int u = 0; u < CH; ++u)
#pragma unroll
            for (int j = 0; j < NB; ++j) wv[u][j] = *reinterpret_cast<const uint4*>(wk + woff[u][j]);
#pragma unroll
        for (int i = 0; i < NX; ++i) {
            const int row = (i * 64 + lane) * EPL / KC;
            const int64_t at = (int64_t)min(row, g.M - 1) * g.lda + min(kx, g.K - EPL);
            if constexpr (A32) xv[i] = *reinterpret_cast<const uint4*>(reinterpret_cast<const float*>(g.A) + at);
            else xv[i] = *reinterpret_cast<const uint4*>(g.A + at);
        }
        if constexpr (NORM != 0) gv = *reinterpret_cast<const float4*>(g.gamma + min(kx, g.K - 4));
        // The normalising forms pin every load of the chunk here, before the other chunk's MFMAs: left
        // alone, the instruction scheduler sinks the gamma load to its first use, behind the wait for the
        // weights, which puts an L2 round trip into every chunk.  The plain form is left to the scheduler,
        // which measured faster there (66 against 73 us on a 235 MB matrix, repeated launches on 64 CUs).
        if constexpr (NORM != 0) __builtin_amdgcn_sched_barrier(0);
    }

    // Loaded layout (instruction u: rows u*RPI + lane/CPRW, chunk lane%CPRW) -> MFMA layout (fragment u:
    // row lane%16, chunk 4u + lane/16) through `scr` (16 rows x CPRW chunks, chunk c of row r at c ^ (r % CPRW)).
    __device__ __forceinline__ void to_fragments(uint16_t* scr, int lane)
    {
        const int cc = lane % CPRW, rr0 = lane / CPRW, r16 = lane & 15, kg = lane >> 4;
#pragma unroll
        for (int j = 0; j < NB; ++j) {
#pragma unroll
            for (int u = 0; u < CH; ++u) {
                const int rr = u * RPI + rr0;
                *reinterpret_cast<uint4*>(scr + (rr * CPRW + (cc ^ (rr % CPRW))) * 8) = wv[u][j];
            }
            wave_lds_sync();
#pragma unroll
            for (int u = 0; u < CH; ++u)
                wv[u][j] = *reinterpret_cast<const uint4*>(scr + (r16 * CPRW + ((4 * u + kg) ^ (r16 % CPRW))) * 8);
            wave_lds_sync();
        }
    }

    // x = hi + mid + lo exactly, each a bf16 value (upper 16 bits kept); planes are PL elements apart
    // NORM: the activations are multiplied by gamma and their sums kept in `rs`; elements outside the
    // slice stay out of the sums.
    template <int ROW, int PL>
    __device__ __forceinline__ void stage(uint16_t* xs, int lane, RowStats<NX, NORM>& rs) const
    {
        float gm[4] = {0.f, 0.f, 0.f, 0.f};
        if constexpr (NORM != 0) {
            const float ge[4] = {gv.x, gv.y, gv.z, gv.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) gm[e] = xlive ? ge[e] : 0.0f;
        }
#pragma unroll
        for (int i = 0; i < NX; ++i) {
            const int f = (i * 64 + lane) * EPL;
            uint16_t* dst = xs + (f / KC) * ROW + f % KC;
            const uint4 xm = xlive ? xv[i] : make_uint4(0, 0, 0, 0);
            if constexpr (!A32) {
                *reinterpret_cast<uint4*>(dst) = xm;
                continue;
            }
            float x[4] = {__uint_as_float(xm.x), __uint_as_float(xm.y), __uint_as_float(xm.z), __uint_as_float(xm.w)};
            if constexpr (NORM != 0) {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float d = NORM == NORM_RMS ? x[e] : (xlive ? x[e] - rs.c[i] : 0.0f);
                    if constexpr (NORM == NORM_LN) rs.s1[i] += d;
                    rs.s2[i] += d * d;
                    x[e] = d * gm[e];
                }
            }
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

// GLU (a flag, NB = 2): the weight matrix holds N gate rows followed by N up rows; a workgroup owns 16
// output columns, its first 16-row block takes their gate rows and its second their up rows, and it
// stores silu(gate) * up.
template <int MR, int NB, int CH, bool A32, int NORM>
__global__ __launch_bounds__(SKINNY_WAVES * 64, 4)      // 128 registers: two workgroups per CU
void gemm_skinny_lds_kernel(GemmArgs g, AtomArgs atom)
{
    constexpr int KW = SKINNY_WAVES;
    constexpr int KC = CH * 32;
    constexpr int ROW = KC + 8;                      // padded row: 16 rows read 16 B each without bank conflicts
    constexpr int PL = (MR + 1) * ROW;               // one plane: MR rows and the row of zeros
    constexpr int NPL = A32 ? 3 : 1;                 // bf16 activations need no splitting
    constexpr int XW = NPL * PL * 2 > CH * 1024 ? NPL * PL * 2 : CH * 1024;   // a wavefront's piece: activation planes, or one
    constexpr int XBYTES = KW * XW;                                           // 16-row weight block while it changes layout
    constexpr int RBYTES = KW * NB * 64 * 16;
    __shared__ __attribute__((aligned(16))) unsigned char smem[XBYTES > RBYTES ? XBYTES : RBYTES];
    __shared__ float2 stat_part[NORM ? KW : 1][MR];   // per wavefront and row: sum (x - c), sum (x - c)^2 over its K slice

    const uint32_t L = atom_logical_block(atom);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r16 = lane & 15, kg = lane >> 4;
    const bool glu = NB == 2 && (g.flags & LITHOS_F_GLU);
    const int n0 = glu ? (int)L * 16 : (int)L * 16 * NB;
    const int kq = ((g.K + 32 * KW - 1) / (32 * KW)) * 32;
    const int kbeg = wave * kq, kend = min(g.K, kbeg + kq);

    uint16_t* xs = reinterpret_cast<uint16_t*>(smem + wave * XW);
    auto zero_rows = [&]() {                         // the row of zeros of each plane (the weight blocks pass over it)
        for (int t = lane; t < NPL * (ROW / 4); t += 64)
            *reinterpret_cast<uint2*>(xs + (t / (ROW / 4)) * PL + MR * ROW + (t % (ROW / 4)) * 4) = make_uint2(0, 0);
    };
    const uint16_t* xrow = xs + min(r16, MR) * ROW;

    f32x4 acc[NB];
#pragma unroll
    for (int j = 0; j < NB; ++j) acc[j] = f32x4{0.f, 0.f, 0.f, 0.f};
    typedef SkinnyChunk<MR, NB, CH, A32, NORM> Chunk;
    uint32_t woff[CH][NB];
#pragma unroll
    for (int u = 0; u < CH; ++u)
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            const int r = min(n0 + (glu ? 0 : j * 16) + u * Chunk::RPI + lane / Chunk::CPRW, g.N - 1) + (glu ? j * g.N : 0);
            woff[u][j] = (uint32_t)((int64_t)r * g.ldb * 2);
        }

    // chunks are walked cyclically from a per-workgroup start so that workgroups, whose weight
    // rows are a power-of-two stride apart, do not address the same memory channels together
    const int nch = max(1, (kend - kbeg + KC - 1) / KC);
    int ci = (int)((L * 7u + (uint32_t)wave * 3u) % (uint32_t)nch);
    auto next_chunk = [&](int& kc0) { kc0 = kbeg + ci * KC; ci = ci + 1 == nch ? 0 : ci + 1; };

    Chunk c0, c1;
    // a chunk's weights change layout in the piece of LDS that its activations then occupy
    RowStats<Chunk::NX, NORM> rs;
#pragma unroll
    for (int i = 0; i < Chunk::NX; ++i) {
        rs.s1[i] = rs.s2[i] = rs.c[i] = 0.0f;
        if constexpr (NORM == NORM_LN) {
            const int row = (i * 64 + lane) * 4 / KC;
            if (row < g.M) rs.c[i] = reinterpret_cast<const float*>(g.A)[(int64_t)row * g.lda];
        }
    }
    auto settle = [&](Chunk& c) {
        c.to_fragments(xs, lane);
        zero_rows();
        c.template stage<ROW, PL>(xs, lane, rs);
        wave_lds_sync();
    };
    int kc0;
    next_chunk(kc0);
    c0.load(g, woff, kc0, kend, false, lane);
    settle(c0);
    for (int c = 0; c < nch; c += 2) {
        next_chunk(kc0);
        c1.load(g, woff, kc0, kend, c + 1 >= nch, lane);
        c0.template compute<ROW, PL>(xrow, kg, acc);
        wave_lds_sync();
        settle(c1);
        next_chunk(kc0);
        c0.load(g, woff, kc0, kend, c + 2 >= nch, lane);
        c1.template compute<ROW, PL>(xrow, kg, acc);
        wave_lds_sync();
        settle(c0);
    }

    if constexpr (NORM != 0) {
        // the lanes that loaded one row (KC / 4 neighbours) add up their sums; slices are added in wave order below
#pragma unroll
        for (int i = 0; i < Chunk::NX; ++i) {
#pragma unroll
            for (int o = KC / 8; o >= 1; o >>= 1) { rs.s1[i] += __shfl_xor(rs.s1[i], o); rs.s2[i] += __shfl_xor(rs.s2[i], o); }
            const int row = (i * 64 + lane) * 4 / KC;
            if (lane % (KC / 4) == 0 && row < MR) stat_part[wave][row] = make_float2(rs.s1[i], rs.s2[i]);
        }
    }
    __syncthreads();                                  // the reduction buffer overlays the activations
    float (*red)[NB][64][4] = reinterpret_cast<float (*)[NB][64][4]>(smem);
#pragma unroll
    for (int j = 0; j < NB; ++j) *reinterpret_cast<f32x4*>(&red[wave][j][lane][0]) = acc[j];
    __syncthreads();
    if (wave == 0) {
        // accumulator element e of a lane is D[n = 4*kg + e][m = r16]; slices are added in wave order
        float v[NB][4];
#pragma unroll
        for (int j = 0; j < NB; ++j)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                v[j][e] = red[0][j][lane][e];
#pragma unroll
                for (int w = 1; w < KW; ++w) v[j][e] += red[w][j][lane][e];
            }
        if constexpr (NORM != 0) {
            // this lane's row statistics, then the scale (and shift) that the loop left out
            float s1 = 0.0f, s2 = 0.0f;
            if (r16 < MR)
                for (int w = 0; w < KW; ++w) { s1 += stat_part[w][r16].x; s2 += stat_part[w][r16].y; }
            const float inv_k = 1.0f / (float)g.K;
            if constexpr (NORM == NORM_RMS) {
                const float rinv = 1.0f / sqrtf(s2 * inv_k + g.eps);
#pragma unroll
                for (int j = 0; j < NB; ++j)
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[j][e] *= rinv;
            } else {
                const float dm = s1 * inv_k;                                  // mean - c
                const float rstd = 1.0f / sqrtf(fmaxf(s2 * inv_k - dm * dm, 0.0f) + g.eps);
#pragma unroll
                for (int j = 0; j < NB; ++j)
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        // g.colsum: row 0 = sum_k gamma_k W_nk, row 1 = sum_k beta_k W_nk (ldcs apart)
                        const int n = min(n0 + (glu ? 0 : j * 16) + 4 * kg + e, g.N - 1) + (glu ? j * g.N : 0);
                        v[j][e] = rstd * (v[j][e] - dm * g.colsum[n]) + g.colsum[g.ldcs + n];
                    }
            }
        }
        if (glu) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float gt = v[0][e], up = v[NB - 1][e];
                epilogue_store(g, r16, n0 + 4 * kg + e, gt / (1.0f + expf(-gt)) * up);
            }
        } else {
#pragma unroll
            for (int j = 0; j < NB; ++j)
#pragma unroll
                for (int e = 0; e < 4; ++e) epilogue_store(g, r16, n0 + j * 16 + 4 * kg + e, v[j][e]);
        }
    }
}

// Chunks are 64 k wide (a load instruction fetches 128-byte pieces of 8 weight rows): with 128-wide
// chunks two buffers in flight do not fit the 128 registers that two workgroups per CU leave a lane.
template <int MR>
static gemm_fn skinny_lds_fn(bool a32, int norm)
{
    // bf16 activations fill whole 16-byte loads from 8 rows on
    if (!a32) return (gemm_fn)gemm_skinny_lds_kernel<(MR < 8 ? 8 : MR), 2, 2, false, 0>;
    if (norm == NORM_LN) return (gemm_fn)gemm_skinny_lds_kernel<MR, 2, 2, true, NORM_LN>;
    if (norm == NORM_RMS) return (gemm_fn)gemm_skinny_lds_kernel<MR, 2, 2, true, NORM_RMS>;
    return (gemm_fn)gemm_skinny_lds_kernel<MR, 2, 2, true, 0>;
}

// norm: 0, NORM_LN or NORM_RMS (fp32 activations of at most 16 rows only)
gemm_fn gemm_skinny_fn(int variant, bool a32, int norm)
{
    switch (variant) {
    case V_SKL4: return skinny_lds_fn<4>(a32, norm);
    case V_SKL8: return skinny_lds_fn<8>(a32, norm);
    case V_SKL16: return skinny_lds_fn<16>(a32, norm);
    default: return a32 ? (gemm_fn)gemm_skinny_kernel<2, SKINNY_NB, true> : (gemm_fn)gemm_skinny_kernel<2, SKINNY_NB, false>;
    }
}

} // namespace lithos
