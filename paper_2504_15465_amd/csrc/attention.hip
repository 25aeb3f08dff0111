// Atom-aware attention kernels for gfx950.
//
//  * attn_enc_kernel - full (unmasked) multi-head attention on a packed
//    [tokens, 3*heads*d] bf16 qkv tensor, d = 64, sequence 64/128/256.  One
//    workgroup per (batch, head); each of its wavefronts owns 32 queries and
//    runs both products on MFMA (v_mfma_f32_32x32x16_bf16):
//      S^T = K Q^T   (keys x queries: a lane then holds ONE query's scores, so
//                     the softmax needs a single cross-lane step)
//      O^T = V^T P^T (P^T is fed to the MFMA straight from the accumulator
//                     registers; only V is transposed, through LDS)
//  * attn_dec_kernel - one query token per sequence against a bf16 key/value
//    cache with grouped-query sharing (HBM-bound: the cache is streamed once).
//    One workgroup per (sequence, key/value head); its wavefronts split the
//    keys, each handling all query heads of the group with an online softmax;
//    the partial results are merged in a fixed order.
//
// Every workgroup works on the (batch, head) named by its LOGICAL block index
// (LithOS Section 4.4), so any sub-range of blocks is a valid atom.
#include "common.hpp"
#include <math.h>

namespace lithos {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

struct AttnArgs {
    const void* q;          // enc: packed qkv (bf16); dec: q rows (bf16 or fp32)
    const uint16_t* k;      // dec: key cache
    const uint16_t* v;      // dec: value cache
    void* o;
    int batch, n_q, n_kv, d, seq, cap;
    int64_t ldq;
    float scale;
    uint32_t flags;
    int splits;             // dec: key ranges per (sequence, key/value head)
    float* ws;              // dec with splits > 1: partial softmaxes
};

__device__ __forceinline__ uint16_t attn_f32_to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

__device__ __forceinline__ float attn_bf16_to_f32(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }

// ---- encoder -------------------------------------------------------------------
// NKB = seq / 32 key blocks, D = 64.  4 wavefronts when seq >= 128, else seq/32.
template <int NKB>
__global__ __launch_bounds__(256) void attn_enc_kernel(AttnArgs a, AtomArgs atom)
{
    constexpr int D = 64, SEQ = NKB * 32, VT_LD = SEQ + 4;       // padded V^T rows
    constexpr int WAVES = 4;
    __shared__ __attribute__((aligned(16))) uint16_t vt[D * VT_LD];

    const uint32_t L = atom_logical_block(atom);
    const int b = L / a.n_q, h = L % a.n_q;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int half = lane >> 5, l32 = lane & 31;
    const int64_t row_stride = 3 * (int64_t)a.n_q * D;           // elements per token
    const uint16_t* base = reinterpret_cast<const uint16_t*>(a.q) + (int64_t)b * SEQ * row_stride + h * D;
    const uint16_t* qp = base;
    const uint16_t* kp = base + (int64_t)a.n_q * D;
    const uint16_t* vp = base + 2 * (int64_t)a.n_q * D;

    // V -> LDS, transposed: vt[d][key]
    for (int c = tid; c < SEQ * D / 8; c += 256) {
        int key = c >> 3, d0 = (c & 7) * 8;
        uint4 v = *reinterpret_cast<const uint4*>(vp + key * row_stride + d0);
        uint32_t u[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int j = 0; j < 8; ++j) vt[(d0 + j) * VT_LD + key] = (uint16_t)(u[j >> 1] >> ((j & 1) * 16));
    }
    __syncthreads();

    // Sequences longer than 128 give a wavefront several 32-query groups.
    for (int qg = wave; qg < NKB; qg += WAVES) {
        const int q0 = qg * 32;
        // S^T[key][query] = sum_d K[key][d] Q[query][d]
        f32x16 s[NKB];
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
            for (int e = 0; e < 16; ++e) s[kb][e] = 0.0f;
#pragma unroll
        for (int ds = 0; ds < D / 16; ++ds) {
            const int d0 = ds * 16 + half * 8;
            bf16x8 qf = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(qp + (q0 + l32) * row_stride + d0));
#pragma unroll
            for (int kb = 0; kb < NKB; ++kb) {
                bf16x8 kf = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(kp + (kb * 32 + l32) * row_stride + d0));
                s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf, s[kb], 0, 0, 0);
            }
        }
        // softmax over keys for this lane's query (the other half-wave holds the other keys)
        float mx = -INFINITY;
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
            for (int e = 0; e < 16; ++e) { s[kb][e] *= a.scale; mx = fmaxf(mx, s[kb][e]); }
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        float sum = 0.0f;
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
            for (int e = 0; e < 16; ++e) { s[kb][e] = expf(s[kb][e] - mx); sum += s[kb][e]; }
        sum += __shfl_xor(sum, 32, 64);
        const float inv = 1.0f / sum;

        // O^T[d][query] = sum_key V^T[d][key] P^T[key][query]
        // accumulator element e of block kb is key 32 kb + 8 (e/4) + 4 half + e%4, so
        // MFMA k-slot j of step (kb, gp) is key 32 kb + 16 gp + 8 (j/4) + 4 half + j%4
        // = accumulator element 8 gp + j: eight consecutive registers.
        f32x16 o[D / 32];
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
            for (int e = 0; e < 16; ++e) o[db][e] = 0.0f;
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
            for (int gp = 0; gp < 2; ++gp) {
                uint32_t pw[4];
#pragma unroll
                for (int p = 0; p < 4; ++p) {
                    uint32_t lo = attn_f32_to_bf16(s[kb][8 * gp + 2 * p] * inv);
                    uint32_t hi = attn_f32_to_bf16(s[kb][8 * gp + 2 * p + 1] * inv);
                    pw[p] = lo | (hi << 16);
                }
                bf16x8 pf = __builtin_bit_cast(bf16x8, make_uint4(pw[0], pw[1], pw[2], pw[3]));
                const int key0 = kb * 32 + gp * 16 + half * 4;
#pragma unroll
                for (int db = 0; db < D / 32; ++db) {
                    const uint16_t* vrow = vt + (db * 32 + l32) * VT_LD + key0;
                    uint2 v0 = *reinterpret_cast<const uint2*>(vrow);
                    uint2 v1 = *reinterpret_cast<const uint2*>(vrow + 8);
                    bf16x8 vf = __builtin_bit_cast(bf16x8, make_uint4(v0.x, v0.y, v1.x, v1.y));
                    o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf, o[db], 0, 0, 0);
                }
            }
        // o[db][e] is d = 32 db + 8 (e/4) + 4 half + e%4 of query q0 + l32
        uint16_t* op = reinterpret_cast<uint16_t*>(a.o) + ((int64_t)b * SEQ + q0 + l32) * ((int64_t)a.n_q * D) + h * D;
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                uint16_t hi[4], lo[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    hi[e] = attn_f32_to_bf16(o[db][4 * g + e]);
                    lo[e] = attn_f32_to_bf16(o[db][4 * g + e] - attn_bf16_to_f32(hi[e]));
                }
                *reinterpret_cast<uint2*>(op + db * 32 + 8 * g + 4 * half) =
                    make_uint2(hi[0] | ((uint32_t)hi[1] << 16), hi[2] | ((uint32_t)hi[3] << 16));
                if (a.flags & LITHOS_F_OUT_SPLIT)
                    *reinterpret_cast<uint2*>(op + (int64_t)a.batch * SEQ * a.n_q * D + db * 32 + 8 * g + 4 * half) =
                        make_uint2(lo[0] | ((uint32_t)lo[1] << 16), lo[2] | ((uint32_t)lo[3] << 16));
            }
    }
}

// ---- decode, grouped-query -------------------------------------------------------
// G = query heads per key/value head (1, 2 or 4), D = 128.  The keys of one
// (sequence, key/value head) are cut into `splits` contiguous ranges of 32-key
// units, one workgroup each, so that a partition's CUs all stream the cache.
//
// Loads: the 16 lanes of a DPP row share one key; lane c of the row owns head
// dimensions 8c..8c+7, so a row reads one 256-byte cache row with 16-byte loads
// and four rows of a wavefront read four neighbouring tokens.
// Scores: on MFMA 16x16x32 with the KEYS as the row operand, S[key][head] = sum_d
// K[key][d] (scale q)[head][d].  A unit's keys pass through the wavefront's own
// piece of LDS to change from the loaded layout to operand fragments; scale*q is
// kept in LDS as three bf16 planes hi + mid + lo (exact), three MFMAs per key
// fragment, so a score is an fp32 sum of exact products as it was on the vector
// ALUs.  Two 16-key blocks per unit, block b row n = key 8(n/4) + 4b + n%4: a lane
// (head = lane%16, kg = lane/16) then holds the scores of keys 8kg..8kg+7 of ONE
// head, and the softmax costs one exp per key and head (a row sum left every lane
// of a row with the same score and the same exp to compute).
// Values: on the vector ALUs in the loaded layout (no exchange of values); the
// probabilities reach them through LDS as p[key][head].
// Every wavefront keeps one running softmax over its units; its four row groups
// hold partial value sums.  These 16 partial results per workgroup are merged in a
// fixed order, then the splits (attn_merge).
__device__ __forceinline__ void unpack_bf16x8(const uint4& u, float* f)
{
    f[0] = __uint_as_float(u.x << 16); f[1] = __uint_as_float(u.x & 0xffff0000u);
    f[2] = __uint_as_float(u.y << 16); f[3] = __uint_as_float(u.y & 0xffff0000u);
    f[4] = __uint_as_float(u.z << 16); f[5] = __uint_as_float(u.z & 0xffff0000u);
    f[6] = __uint_as_float(u.w << 16); f[7] = __uint_as_float(u.w & 0xffff0000u);
}

__device__ __forceinline__ void dec_wave_lds_sync()
{
    // LDS operations of one wavefront complete in order; this only stops the compiler
    // from moving reads of other lanes' data across the writes
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

typedef float f32x4 __attribute__((ext_vector_type(4)));

// 16-byte slot of chunk c of key row r in a wavefront's key tile: the 8 lanes that read one chunk
// column of rows {0-3, 8-11} + 4b (+16) fall into 8 different slots mod 8
__device__ __forceinline__ int dec_kslot(int r, int c) { return r * 16 + (c ^ ((r & 3) | ((r >> 1) & 4))); }

// Workspace of a split launch (floats): numerators [batch*n_kv][splits][G][D],
// then (max, denominator) pairs [batch*n_kv][splits][G][2].
template <int G, bool Q32, bool O32>
__global__ __launch_bounds__(256, 3) void attn_dec_kernel(AttnArgs a, AtomArgs atom)      // 168 registers: three workgroups per CU
{
    constexpr int D = 128, R = 8;                 // R keys per lane and step: 32 keys per wavefront step
    constexpr int QLD = D + 8;                    // padded rows: the G live rows are read without bank conflicts
    constexpr int KT_BYTES = 32 * 16 * 16;        // a wavefront's key tile: 32 keys x 16 chunks of 16 bytes
    constexpr int PO_BYTES = 16 * G * D * 4;
    // the partial value sums overlay the key tiles, which are dead by then
    __shared__ __attribute__((aligned(16))) unsigned char big[4 * KT_BYTES > PO_BYTES ? 4 * KT_BYTES : PO_BYTES];
    __shared__ __attribute__((aligned(16))) uint16_t qpl[3][G + 1][QLD];   // scale*q = hi + mid + lo, and a row of zeros
    __shared__ __attribute__((aligned(16))) float pbuf[4][32][4];           // per wavefront: p[key][head]
    __shared__ float cbuf[4][4];                                             // per wavefront: rescale factor per head
    __shared__ float part_m[16][G], part_l[16][G];

    const uint32_t L = atom_logical_block(atom);
    const int S = a.splits;
    const int sp = L % S, bg = L / S;
    const int b = bg / a.n_kv, g = bg % a.n_kv;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = lane & 15, rg = lane >> 4;      // loads and values: chunk of 8 head dimensions, row group
    const int r16 = c, kg = rg;                   // MFMA: key row / head, k group

    for (int i = tid; i < (G + 1) * D; i += 256) {
        const int h = i / D, d = i % D;
        float x = 0.0f;
        if (h < G) {
            const int64_t idx = (int64_t)b * a.ldq + (g * G + h) * D + d;
            if constexpr (Q32) x = reinterpret_cast<const float*>(a.q)[idx];
            else x = attn_bf16_to_f32(reinterpret_cast<const uint16_t*>(a.q)[idx]);
            x *= a.scale;
        }
        const uint32_t hi = __float_as_uint(x) & 0xffff0000u;
        const float r1 = x - __uint_as_float(hi);                         // exact
        const uint32_t mid = __float_as_uint(r1) & 0xffff0000u;
        const float r2 = r1 - __uint_as_float(mid);                       // exact, at most 8 bits
        qpl[0][h][d] = (uint16_t)(hi >> 16);
        qpl[1][h][d] = (uint16_t)(mid >> 16);
        qpl[2][h][d] = (uint16_t)(__float_as_uint(r2) >> 16);
    }
    __syncthreads();

    const int64_t tok_stride = (int64_t)a.n_kv * D;
    const uint16_t* kbase = a.k + ((int64_t)b * a.cap * a.n_kv + g) * D + 8 * c;
    const uint16_t* vbase = a.v + ((int64_t)b * a.cap * a.n_kv + g) * D + 8 * c;
    const int T = a.seq;
    const int U = (T + 31) / 32;                                   // 32-key units
    const int u0 = (int)((int64_t)sp * U / S), u1 = (int)((int64_t)(sp + 1) * U / S);

    uint4* kt = reinterpret_cast<uint4*>(big + wave * KT_BYTES);
    const uint16_t* qrow = &qpl[0][min(r16, G)][8 * kg];
    constexpr int QPLANE = (G + 1) * QLD;

    float m = -INFINITY, l = 0.0f;                // running softmax of head r16 (the same in its four kg lanes; l: this lane's keys)
    float acc[G][8];
#pragma unroll
    for (int h = 0; h < G; ++h)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[h][e] = 0.0f;

    for (int u = u0 + wave; u < u1; u += 4) {
        uint4 kx[R], vx[R];
#pragma unroll
        for (int i = 0; i < R; ++i) {
            const int t = 32 * u + 4 * i + rg;
            const int64_t off = (int64_t)min(t, T - 1) * tok_stride;    // dead keys read the last live row
            kx[i] = *reinterpret_cast<const uint4*>(kbase + off);
            vx[i] = *reinterpret_cast<const uint4*>(vbase + off);
        }
#pragma unroll
        for (int i = 0; i < R; ++i) kt[dec_kslot(4 * i + rg, c)] = kx[i];
        dec_wave_lds_sync();

        float s8[8];
#pragma unroll
        for (int blk = 0; blk < 2; ++blk) {
            const int row = 8 * (r16 >> 2) + 4 * blk + (r16 & 3);
            f32x4 sc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int st = 0; st < 4; ++st) {
                const bf16x8 kf = __builtin_bit_cast(bf16x8, kt[dec_kslot(row, 4 * st + kg)]);
#pragma unroll
                for (int p = 2; p >= 0; --p) {
                    const bf16x8 qf = *reinterpret_cast<const bf16x8*>(qrow + p * QPLANE + 32 * st);
                    sc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf, qf, sc, 0, 0, 0);
                }
            }
            // element e: key 8*kg + 4*blk + e of the unit, head r16
#pragma unroll
            for (int e = 0; e < 4; ++e) s8[4 * blk + e] = 32 * u + 8 * kg + 4 * blk + e < T ? sc[e] : -INFINITY;
        }
        float bm = s8[0];
#pragma unroll
        for (int j = 1; j < 8; ++j) bm = fmaxf(bm, s8[j]);
        bm = fmaxf(bm, __shfl_xor(bm, 16));
        bm = fmaxf(bm, __shfl_xor(bm, 32));
        const float nm = fmaxf(m, bm);
        const float ref = nm == -INFINITY ? 0.0f : nm;             // a unit always holds a live key; kept for safety
        const float corr = expf(m - ref);                          // 0 while m = -inf
        float ls = 0.0f;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const float p = expf(s8[j] - ref);                     // 0 for a dead key
            ls += p;
            if (r16 < G) pbuf[wave][8 * kg + j][r16] = p;
        }
        l = l * corr + ls;
        m = nm;
        if (lane < G) cbuf[wave][lane] = corr;
        dec_wave_lds_sync();

        float cr[G];
#pragma unroll
        for (int h = 0; h < G; ++h) cr[h] = cbuf[wave][h];
#pragma unroll
        for (int h = 0; h < G; ++h)
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[h][e] *= cr[h];
#pragma unroll
        for (int i = 0; i < R; ++i) {
            float vf[8];
            unpack_bf16x8(vx[i], vf);
            const float4 p4 = *reinterpret_cast<const float4*>(&pbuf[wave][4 * i + rg][0]);
            const float ph[4] = {p4.x, p4.y, p4.z, p4.w};
#pragma unroll
            for (int h = 0; h < G; ++h)
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[h][e] += ph[h] * vf[e];
        }
        dec_wave_lds_sync();                                       // the next unit rewrites the tile and p
    }

    // merge the 16 partial softmaxes (wavefront-major, then row group) in that order: a wavefront's
    // four row groups share its running maximum, its denominator is booked on the first of them
    float lt = l + __shfl_xor(l, 16);
    lt = lt + __shfl_xor(lt, 32);
    __syncthreads();                                               // every wavefront is done with its key tile
    float (*part_o)[G][D] = reinterpret_cast<float (*)[G][D]>(big);
    const int slot = wave * 4 + rg;
#pragma unroll
    for (int h = 0; h < G; ++h) {
        *reinterpret_cast<float4*>(&part_o[slot][h][8 * c]) = make_float4(acc[h][0], acc[h][1], acc[h][2], acc[h][3]);
        *reinterpret_cast<float4*>(&part_o[slot][h][8 * c + 4]) = make_float4(acc[h][4], acc[h][5], acc[h][6], acc[h][7]);
    }
    if (lane < G) {
#pragma unroll
        for (int q = 0; q < 4; ++q) { part_m[wave * 4 + q][lane] = m; part_l[wave * 4 + q][lane] = q == 0 ? lt : 0.0f; }
    }
    __syncthreads();
    for (int i = tid; i < G * D; i += 256) {
        const int h = i / D, d = i % D;
        float gm = -INFINITY;
        for (int w = 0; w < 16; ++w) gm = fmaxf(gm, part_m[w][h]);
        const float ref = gm == -INFINITY ? 0.0f : gm;            // a split without keys: all partials empty
        float num = 0.0f, den = 0.0f;
        for (int w = 0; w < 16; ++w) {
            const float f = expf(part_m[w][h] - ref);             // 0 for a wavefront that saw no key
            num += part_o[w][h][d] * f;
            den += part_l[w][h] * f;
        }
        if (S == 1) {
            const float r = num / den;
            const int64_t idx = (int64_t)b * ((int64_t)a.n_q * D) + (g * G + h) * D + d;
            if constexpr (O32) reinterpret_cast<float*>(a.o)[idx] = r;
            else reinterpret_cast<uint16_t*>(a.o)[idx] = attn_f32_to_bf16(r);
        } else {
            float* ws = a.ws;
            const int64_t row = ((int64_t)bg * S + sp) * G + h;
            ws[row * D + d] = num;
            if (d == 0) {
                float* ml = ws + (int64_t)a.batch * a.n_kv * S * G * D;
                ml[row * 2] = gm;
                ml[row * 2 + 1] = den;
            }
        }
    }
}

// Merge of the splits' partial softmaxes, in split order.  One workgroup per
// (sequence, key/value head).
template <int G, bool O32>
__global__ __launch_bounds__(256) void attn_merge_kernel(AttnArgs a, AtomArgs atom)
{
    constexpr int D = 128;
    const uint32_t bg = atom_logical_block(atom);
    const int b = bg / a.n_kv, g = bg % a.n_kv, S = a.splits;
    const float* ws = a.ws;
    const float* ml = ws + (int64_t)a.batch * a.n_kv * S * G * D;
    for (int i = threadIdx.x; i < G * D; i += 256) {
        const int h = i / D, d = i % D;
        // eight splits at a time, their loads issued together (a split index beyond S re-reads the
        // last split and is given weight 0); the sums still run in split order
        const float2* mlr = reinterpret_cast<const float2*>(ml) + (int64_t)bg * S * G + h;     // split s at mlr[s * G]
        const float* wsr = ws + ((int64_t)bg * S * G + h) * D + d;                               // split s at wsr[s * G * D]
        float gm = -INFINITY;
        for (int s0 = 0; s0 < S; s0 += 8) {
            float m8[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) m8[u] = mlr[(int64_t)min(s0 + u, S - 1) * G].x;
#pragma unroll
            for (int u = 0; u < 8; ++u) gm = fmaxf(gm, m8[u]);
        }
        float num = 0.0f, den = 0.0f;
        for (int s0 = 0; s0 < S; s0 += 8) {
            float2 p8[8];
            float o8[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int64_t sc = min(s0 + u, S - 1);
                p8[u] = mlr[sc * G];
                o8[u] = wsr[sc * G * D];
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const float f = s0 + u < S ? expf(p8[u].x - gm) : 0.0f;     // 0 for a split without keys
                num += o8[u] * f;
                den += p8[u].y * f;
            }
        }
        const float r = num / den;
        const int64_t idx = (int64_t)b * ((int64_t)a.n_q * D) + (g * G + h) * D + d;
        if constexpr (O32) reinterpret_cast<float*>(a.o)[idx] = r;
        else reinterpret_cast<uint16_t*>(a.o)[idx] = attn_f32_to_bf16(r);
    }
}

// ---- host side ----------------------------------------------------------------------

typedef void (*attn_fn)(AttnArgs, AtomArgs);

static attn_fn dec_fn(int G, bool q32, bool o32)
{
#define PICKG(GG) (q32 ? (o32 ? (attn_fn)attn_dec_kernel<GG, true, true> : (attn_fn)attn_dec_kernel<GG, true, false>) \
                       : (o32 ? (attn_fn)attn_dec_kernel<GG, false, true> : (attn_fn)attn_dec_kernel<GG, false, false>))
    switch (G) {
    case 1: return PICKG(1);
    case 2: return PICKG(2);
    default: return PICKG(4);
    }
#undef PICKG
}

// the kernel that serves a (validated) descriptor
static attn_fn attn_kernel(const lithos_op_t& op)
{
    if (op.kind == LITHOS_OP_ATTN_ENC)
        return op.dim[2] == 64 ? (attn_fn)attn_enc_kernel<2> : op.dim[2] == 128 ? (attn_fn)attn_enc_kernel<4> : (attn_fn)attn_enc_kernel<8>;
    const int G = (int)(op.dim[1] / op.dim[2]);
    const bool o32 = op.flags & LITHOS_F_OUT_F32;
    if (op.kind == LITHOS_OP_ATTN_MERGE)
        return G == 1 ? (o32 ? (attn_fn)attn_merge_kernel<1, true> : (attn_fn)attn_merge_kernel<1, false>)
             : G == 2 ? (o32 ? (attn_fn)attn_merge_kernel<2, true> : (attn_fn)attn_merge_kernel<2, false>)
                      : (o32 ? (attn_fn)attn_merge_kernel<4, true> : (attn_fn)attn_merge_kernel<4, false>);
    return dec_fn(G, op.flags & LITHOS_F_IN_F32, o32);
}

// resident workgroups per CU, from the runtime (the constants are the fallback)
static void attn_occupancy(const lithos_op_t& op, OpPlan* plan)
{
    plan->wg_per_cu = cached_occupancy((const void*)attn_kernel(op), (int)plan->threads, plan->wg_per_cu);
}

int attn_plan(const lithos_op_t& op, OpPlan* plan)
{
    plan->threads = 256;
    plan->variant = 0;
    if (op.kind == LITHOS_OP_ATTN_ENC) {
        const int64_t batch = op.dim[0], heads = op.dim[1], seq = op.dim[2], d = op.dim[3];
        if (batch <= 0 || heads <= 0 || batch * heads > 0x7fffffff) return fail(LITHOS_EINVAL, "attn_enc: batch and heads must be positive");
        if (d != 64) return fail(LITHOS_EINVAL, "attn_enc: head width %lld is not built (64 only)", (long long)d);
        if (seq != 64 && seq != 128 && seq != 256) return fail(LITHOS_EINVAL, "attn_enc: sequence length %lld is not built (64, 128, 256)", (long long)seq);
        if (!op.in[0] || !op.out[0] || !aligned16(op.in[0]) || (reinterpret_cast<uintptr_t>(op.out[0]) & 7u))
            return fail(LITHOS_EINVAL, "attn_enc: null or misaligned qkv / output");
        plan->grid = {(uint32_t)heads, (uint32_t)batch, 1};
        plan->total = (uint32_t)(batch * heads);
        plan->wg_per_cu = 2;
        attn_occupancy(op, plan);
        return LITHOS_OK;
    }
    if (op.kind == LITHOS_OP_ATTN_MERGE) {
        // dim = batch, n_q, n_kv, d, splits
        const int64_t batch = op.dim[0], n_q = op.dim[1], n_kv = op.dim[2], d = op.dim[3], splits = op.dim[4];
        if (batch <= 0 || n_q <= 0 || n_kv <= 0 || n_q % n_kv || batch * n_kv > 0x7fffffff) return fail(LITHOS_EINVAL, "attn_merge: need batch > 0 and n_kv dividing n_q");
        const int64_t G = n_q / n_kv;
        if (G != 1 && G != 2 && G != 4) return fail(LITHOS_EINVAL, "attn_merge: group size %lld is not built (1, 2, 4)", (long long)G);
        if (d != 128) return fail(LITHOS_EINVAL, "attn_merge: head width %lld is not built (128 only)", (long long)d);
        if (splits < 1 || splits > LITHOS_ATTN_MAX_SPLITS) return fail(LITHOS_EINVAL, "attn_merge: splits %lld outside 1..%d", (long long)splits, LITHOS_ATTN_MAX_SPLITS);
        if (!op.in[0] || !op.out[0]) return fail(LITHOS_EINVAL, "attn_merge: null operand");
        plan->grid = {(uint32_t)n_kv, (uint32_t)batch, 1};
        plan->total = (uint32_t)(batch * n_kv);
        plan->wg_per_cu = 4;
        attn_occupancy(op, plan);
        return LITHOS_OK;
    }
    // decode: dim = batch, n_q, n_kv, d, keys, cap, splits
    const int64_t batch = op.dim[0], n_q = op.dim[1], n_kv = op.dim[2], d = op.dim[3], keys = op.dim[4], cap = op.dim[5];
    const int64_t splits = op.dim[6] > 0 ? op.dim[6] : 1;
    if (batch <= 0 || n_q <= 0 || n_kv <= 0 || n_q % n_kv) return fail(LITHOS_EINVAL, "attn_dec: need batch > 0 and n_kv dividing n_q");
    const int64_t G = n_q / n_kv;
    if (G != 1 && G != 2 && G != 4) return fail(LITHOS_EINVAL, "attn_dec: group size %lld is not built (1, 2, 4)", (long long)G);
    if (d != 128) return fail(LITHOS_EINVAL, "attn_dec: head width %lld is not built (128 only)", (long long)d);
    if (keys <= 0 || keys > cap) return fail(LITHOS_EINVAL, "attn_dec: need 0 < keys <= cap");
    if (op.ld[0] < n_q * d) return fail(LITHOS_EINVAL, "attn_dec: q row stride smaller than n_q*d");
    if (!op.in[0] || !op.in[1] || !op.in[2] || !op.out[0]) return fail(LITHOS_EINVAL, "attn_dec: null operand");
    if (!aligned16(op.in[1]) || !aligned16(op.in[2])) return fail(LITHOS_EINVAL, "attn_dec: caches must be 16-byte aligned");
    if (!aligned16(op.in[0]) || op.ld[0] % 8) return fail(LITHOS_EINVAL, "attn_dec: q must be 16-byte aligned with a row stride that is a multiple of 8");
    if (splits > LITHOS_ATTN_MAX_SPLITS) return fail(LITHOS_EINVAL, "attn_dec: splits %lld above %d", (long long)splits, LITHOS_ATTN_MAX_SPLITS);
    if (splits > 1 && (!op.in[3] || !aligned16(op.in[3]))) return fail(LITHOS_EINVAL, "attn_dec: a split launch needs a 16-byte aligned workspace in in[3]");
    if (batch * n_kv * splits > 0x7fffffff) return fail(LITHOS_EINVAL, "attn_dec: too many workgroups");
    plan->grid = {(uint32_t)(n_kv * splits), (uint32_t)batch, 1};
    plan->total = (uint32_t)(batch * n_kv * splits);
    plan->wg_per_cu = 2;
    attn_occupancy(op, plan);
    return LITHOS_OK;
}

int attn_launch(const lithos_op_t& op, const OpPlan& plan, const AtomArgs& atom, hipStream_t s)
{
    AttnArgs a{};
    a.q = op.in[0];
    a.o = op.out[0];
    a.scale = op.fparam[0];
    a.flags = op.flags;
    const dim3 grid(LITHOS_ATOM_LAUNCH_BLOCKS(atom)), block(256);
    if (op.kind == LITHOS_OP_ATTN_ENC) {
        a.batch = (int)op.dim[0]; a.n_q = (int)op.dim[1]; a.seq = (int)op.dim[2]; a.d = (int)op.dim[3];
        LITHOS_HIP(launch_kernel(attn_kernel(op), grid, block, s, a, atom));
        return LITHOS_OK;
    }
    if (op.kind == LITHOS_OP_ATTN_MERGE) {
        a.batch = (int)op.dim[0]; a.n_q = (int)op.dim[1]; a.n_kv = (int)op.dim[2]; a.d = (int)op.dim[3]; a.splits = (int)op.dim[4];
        a.ws = (float*)const_cast<void*>(op.in[0]);
        LITHOS_HIP(launch_kernel(attn_kernel(op), grid, block, s, a, atom));
        return LITHOS_OK;
    }
    a.k = (const uint16_t*)op.in[1];
    a.v = (const uint16_t*)op.in[2];
    a.splits = op.dim[6] > 0 ? (int)op.dim[6] : 1;
    a.ws = (float*)const_cast<void*>(op.in[3]);
    a.batch = (int)op.dim[0]; a.n_q = (int)op.dim[1]; a.n_kv = (int)op.dim[2]; a.d = (int)op.dim[3];
    a.seq = (int)op.dim[4]; a.cap = (int)op.dim[5];
    a.ldq = op.ld[0];
    LITHOS_HIP(launch_kernel(attn_kernel(op), grid, block, s, a, atom));
    return LITHOS_OK;
}

} // namespace lithos
