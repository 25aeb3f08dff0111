// Atom-aware causal attention over a long prompt (prefill), grouped-query, head width 128.
//
// One workgroup per (sequence, query head, PAIR of 128-query tiles: tile p from the end and tile p
// from the start of the prompt, which together see the same number of keys for every p); for each
// tile in turn, each of the four wavefronts
// owns 32 queries and walks the keys 0 .. last query of the tile in blocks of 64 with a running
// softmax (maximum, denominator and unnormalised output per query).  Both products run on MFMA
// (v_mfma_f32_32x32x16_bf16):
//   S^T = K Q^T   keys x queries: a lane holds ONE query's scores, so the running maximum and
//                 denominator are per-lane scalars and need a single exchange with the other
//                 half of the wavefront;
//   O^T = V^T P^T P^T goes from the accumulator registers into the second MFMA; V lies in LDS
//                 as it lies in memory, [key][d], and its fragments come out of the
//                 transposing LDS load (ds_read_b64_tr_b16), so nothing is transposed by hand.
// The key and value blocks are fetched into registers one block ahead and pass through LDS,
// where all four wavefronts read them.  Probabilities are rounded to bf16 for the second
// product; the normalisation is applied to the fp32 result.
//
// The tile a workgroup computes is named by its LOGICAL block index (LithOS Section 4.4), so
// any sub-range of blocks is a valid atom, and every block does the same amount of work.
#include "common.hpp"
#include <math.h>

namespace lithos {

typedef __bf16 pf_bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 pf_bf16x2 __attribute__((ext_vector_type(2)));
typedef float pf_f32x2 __attribute__((ext_vector_type(2)));
typedef float pf_f32x16 __attribute__((ext_vector_type(16)));
typedef short pf_s16x4 __attribute__((ext_vector_type(4)));

struct PrefillArgs {
    const uint16_t* q;      // [batch*T, ldq], head h at columns h*128
    const uint16_t* k;      // [batch, cap, n_kv, 128]
    const uint16_t* v;
    uint16_t* o;            // [batch*T, ldo]
    int batch, n_q, n_kv, T, cap;
    int64_t ldq, ldo;
    float scale_log2e;      // scale * log2(e): the softmax runs in base 2
};

constexpr int PF_D = 128, PF_QT = 128, PF_KB = 64;

// K block [64 keys][128 d]: 16-byte chunk c of key r at chunk c ^ (r & 15): the 16 lanes that
// read one chunk column of 16 consecutive keys then touch 16 different chunk slots.
__device__ __forceinline__ int pf_k_index(int key, int chunk) { return key * PF_D + ((chunk ^ (key & 15)) << 3); }
// V block [64 keys][128 d]: chunk c of key k at chunk c ^ ((k & 3) << 2), so the four keys that one
// transposing load touches fall into different banks.
__device__ __forceinline__ int pf_v_index(int key, int d) { return key * PF_D + ((((d >> 3) ^ ((key & 3) << 2))) << 3) + (d & 7); }

__device__ __forceinline__ uint32_t pf_pack_bf16(float lo, float hi)
{
    pf_f32x2 f = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, pf_bf16x2));   // round to nearest even
}

// One block of keys and values is 1024 chunks of 16 bytes per operand, four per thread, held in
// eight named registers between the fetch and the store to LDS one iteration later (an array
// that lives across the loop's back edge is placed in scratch memory by the compiler).
#define PF_FETCH(i, kb)                                                                        \
    {                                                                                          \
        const int c_ = tid + 256 * i, key_ = c_ >> 4, ch_ = c_ & 15;                           \
        const int64_t off_ = (int64_t)((kb) * PF_KB + key_) * tok + ch_ * 8;                   \
        kr##i = *reinterpret_cast<const uint4*>(kg + off_);                                    \
        vr##i = *reinterpret_cast<const uint4*>(vg + off_);                                    \
    }
#define PF_STASH(i)                                                                            \
    {                                                                                          \
        const int c_ = tid + 256 * i, key_ = c_ >> 4, ch_ = c_ & 15;                           \
        *reinterpret_cast<uint4*>(Ks + pf_k_index(key_, ch_)) = kr##i;                         \
        *reinterpret_cast<uint4*>(Vs + pf_v_index(key_, ch_ * 8)) = vr##i;                     \
    }

__global__ __launch_bounds__(256, 2) void attn_prefill_kernel(PrefillArgs a, AtomArgs atom)
{
    __shared__ __attribute__((aligned(16))) uint16_t Ks[PF_KB * PF_D];
    __shared__ __attribute__((aligned(16))) uint16_t Vs[PF_KB * PF_D];

    const uint32_t L = atom_logical_block(atom);
    // A block computes TWO query tiles, number p from the end of the prompt and number p from its
    // start: together they see T/128 + 1 tiles of keys whatever p is, so all blocks of the grid do the
    // same work (a causal tile alone sees between 1 and T/128 tiles).  Order of the logical blocks,
    // fastest first: the query heads of one key/value head, the pair p, key/value head, sequence:
    // neighbouring blocks stream the same keys and values through one die's L2.
    const int nqt = a.T / PF_QT, npair = nqt / 2, G = a.n_q / a.n_kv;
    uint32_t rest = L;
    const int hq = (int)(rest % G); rest /= G;
    const int pr = (int)(rest % npair); rest /= npair;
    const int g = (int)(rest % a.n_kv); rest /= a.n_kv;
    const int b = (int)rest;
    const int h = g * G + hq;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int half = lane >> 5, l32 = lane & 31;
    const int64_t tok = (int64_t)a.n_kv * PF_D;
    const uint16_t* kg = a.k + ((int64_t)b * a.cap * a.n_kv + g) * PF_D;
    const uint16_t* vg = a.v + ((int64_t)b * a.cap * a.n_kv + g) * PF_D;

  for (int pass = 0; pass < 2; ++pass) {
    const int qtile = pass == 0 ? nqt - 1 - pr : pr;        // the long tile first
    const int q0 = qtile * PF_QT + wave * 32;               // this wavefront's first query
    const int qi = q0 + l32;                                // this lane's query

    // Q fragments (B operand of S^T = K Q^T): query l32, 8 consecutive d per 16-wide step
    pf_bf16x8 qf[PF_D / 16];
    {
        const uint16_t* qp = a.q + ((int64_t)b * a.T + qi) * a.ldq + h * PF_D + half * 8;
#pragma unroll
        for (int ds = 0; ds < PF_D / 16; ++ds) qf[ds] = __builtin_bit_cast(pf_bf16x8, *reinterpret_cast<const uint4*>(qp + ds * 16));
    }

    uint4 kr0, kr1, kr2, kr3, vr0, vr1, vr2, vr3;
    pf_f32x16 o[PF_D / 32];
#pragma unroll
    for (int db = 0; db < PF_D / 32; ++db)
#pragma unroll
        for (int e = 0; e < 16; ++e) o[db][e] = 0.0f;
    float m_run = -INFINITY, l_run = 0.0f;

    const int nkb = (qtile + 1) * (PF_QT / PF_KB);          // key blocks up to the tile's last query
    PF_FETCH(0, 0) PF_FETCH(1, 0) PF_FETCH(2, 0) PF_FETCH(3, 0)
    for (int kb = 0; kb < nkb; ++kb) {
        __syncthreads();                                    // everybody is done reading the previous block
        PF_STASH(0) PF_STASH(1) PF_STASH(2) PF_STASH(3)
        __syncthreads();
        if (kb + 1 < nkb) { PF_FETCH(0, kb + 1) PF_FETCH(1, kb + 1) PF_FETCH(2, kb + 1) PF_FETCH(3, kb + 1) }

        const int key_base = kb * PF_KB;
        if (key_base > q0 + 31) continue;                   // every key of the block lies after this wavefront's queries
        pf_f32x16 s[2];
        bool live[2];
#pragma unroll
        for (int sub = 0; sub < 2; ++sub) {
            live[sub] = key_base + sub * 32 <= q0 + 31;      // uniform over the wavefront
#pragma unroll
            for (int e = 0; e < 16; ++e) s[sub][e] = 0.0f;
            if (live[sub]) {
#pragma unroll
                for (int ds = 0; ds < PF_D / 16; ++ds) {
                    const pf_bf16x8 kf = __builtin_bit_cast(pf_bf16x8, *reinterpret_cast<const uint4*>(Ks + pf_k_index(sub * 32 + l32, ds * 2 + half)));
                    s[sub] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ds], s[sub], 0, 0, 0);
                }
            }
        }
        // accumulator element e of sub-block `sub` is key key_base + 32 sub + 8 (e/4) + 4 half + e%4
        const bool diag = key_base + PF_KB - 1 > q0;        // some key of the block lies after some query
        // The running maximum is kept in raw score units; the scale (times log2 e) enters as the
        // factor of one fused multiply-add per score: p = 2^(s c - m c).
        const float c = a.scale_log2e;
        if (diag || !live[1]) {                             // uniform over the wavefront
#pragma unroll
            for (int sub = 0; sub < 2; ++sub)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int key = key_base + sub * 32 + 8 * (e >> 2) + 4 * half + (e & 3);
                    if (!live[sub] || key > qi) s[sub][e] = -INFINITY;
                }
        }
        float mloc = -INFINITY;
#pragma unroll
        for (int sub = 0; sub < 2; ++sub)
#pragma unroll
            for (int e = 0; e < 16; ++e) mloc = fmaxf(mloc, s[sub][e]);
        mloc = fmaxf(mloc, __shfl_xor(mloc, 32, 64));
        // key 0 is visible to every query and block 0 comes first, so m_new is finite from the start
        const float m_new = fmaxf(m_run, mloc);
        const float mc = m_new * c;
        float lsum = 0.0f;
#pragma unroll
        for (int sub = 0; sub < 2; ++sub)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const float p = __builtin_amdgcn_exp2f(fmaf(s[sub][e], c, -mc));    // 0 for a masked key
                s[sub][e] = p;
                lsum += p;
            }
        // Once a query has seen its largest score the maximum stays, and rescaling by exactly 1 would
        // change nothing: the 64 multiplications are skipped unless some lane's maximum moved.
        if (__any(m_new != m_run)) {
            const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * c);      // 1 where the maximum stayed, 0 at the start
            l_run *= alpha;
#pragma unroll
            for (int db = 0; db < PF_D / 32; ++db)
#pragma unroll
                for (int e = 0; e < 16; ++e) o[db][e] *= alpha;
            m_run = m_new;
        }
        l_run += lsum;

        // O^T[d][query] += V^T[d][key] P^T[key][query].  MFMA k-slot j of step (sub, gp) is key
        // 32 sub + 16 gp + 8 (j/4) + 4 half + j%4 = accumulator element 8 gp + j of s[sub]; the V
        // fragment of that step holds the same eight keys: two transposing loads, four keys each.
        const int grp = lane >> 4, sl = lane & 15;
#pragma unroll
        for (int sub = 0; sub < 2; ++sub) {
            if (!live[sub]) continue;
#pragma unroll
            for (int gp = 0; gp < 2; ++gp) {
                uint32_t pw[4];
#pragma unroll
                for (int p = 0; p < 4; ++p) pw[p] = pf_pack_bf16(s[sub][8 * gp + 2 * p], s[sub][8 * gp + 2 * p + 1]);
                const pf_bf16x8 pf = __builtin_bit_cast(pf_bf16x8, make_uint4(pw[0], pw[1], pw[2], pw[3]));
                // source lane sl of a 16-lane group supplies key krow, d-rows 4 (sl%4) .. +3 of the group's 16
                const int krow = sub * 32 + gp * 16 + 4 * (grp >> 1) + (sl >> 2);
#pragma unroll
                for (int db = 0; db < PF_D / 32; ++db) {
                    const int drow = db * 32 + 16 * (grp & 1) + 4 * (sl & 3);
                    const pf_s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) pf_s16x4*)(Vs + pf_v_index(krow, drow)));
                    const pf_s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) pf_s16x4*)(Vs + pf_v_index(krow + 8, drow)));
                    const pf_bf16x8 vf = __builtin_bit_cast(pf_bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
                    o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf, o[db], 0, 0, 0);
                }
            }
        }
    }

    // o[db][e] is d = 32 db + 8 (e/4) + 4 half + e%4 of query qi; both halves hold half of the denominator
    l_run += __shfl_xor(l_run, 32, 64);
    const float inv = 1.0f / l_run;
    uint16_t* op = a.o + ((int64_t)b * a.T + qi) * a.ldo + h * PF_D;
#pragma unroll
    for (int db = 0; db < PF_D / 32; ++db)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4)
            *reinterpret_cast<uint2*>(op + db * 32 + 8 * q4 + 4 * half) =
                make_uint2(pf_pack_bf16(o[db][4 * q4] * inv, o[db][4 * q4 + 1] * inv),
                           pf_pack_bf16(o[db][4 * q4 + 2] * inv, o[db][4 * q4 + 3] * inv));
  }
}

#undef PF_FETCH
#undef PF_STASH

// ---- host side ----------------------------------------------------------------------

// dim = batch, n_q, n_kv, d, T, cap; in = q, kcache, vcache; out = o; ld0 = q row stride, ld1 = o row stride
int attn_prefill_plan(const lithos_op_t& op, OpPlan* plan)
{
    const int64_t batch = op.dim[0], n_q = op.dim[1], n_kv = op.dim[2], d = op.dim[3], T = op.dim[4], cap = op.dim[5];
    if (batch <= 0 || n_q <= 0 || n_kv <= 0 || n_q % n_kv) return fail(LITHOS_EINVAL, "attn_prefill: need batch > 0 and n_kv dividing n_q");
    if (d != PF_D) return fail(LITHOS_EINVAL, "attn_prefill: head width %lld is not built (128 only)", (long long)d);
    if (T <= 0 || T % (2 * PF_QT)) return fail(LITHOS_EINVAL, "attn_prefill: prompt length %lld must be a positive multiple of %d", (long long)T, 2 * PF_QT);
    if (T > cap) return fail(LITHOS_EINVAL, "attn_prefill: prompt longer than the key/value buffers (cap)");
    if (op.ld[0] < n_q * d || op.ld[1] < n_q * d || op.ld[0] % 8 || op.ld[1] % 4)
        return fail(LITHOS_EINVAL, "attn_prefill: row strides of q (multiple of 8) and o (multiple of 4) must be at least n_q*d");
    if (!op.in[0] || !op.in[1] || !op.in[2] || !op.out[0]) return fail(LITHOS_EINVAL, "attn_prefill: null operand");
    if (!aligned16(op.in[0]) || !aligned16(op.in[1]) || !aligned16(op.in[2]) || (reinterpret_cast<uintptr_t>(op.out[0]) & 7u))
        return fail(LITHOS_EINVAL, "attn_prefill: q, k, v must be 16-byte aligned, o 8-byte aligned");
    if (op.flags & (LITHOS_F_IN_F32 | LITHOS_F_OUT_F32 | LITHOS_F_OUT_SPLIT)) return fail(LITHOS_EINVAL, "attn_prefill: bf16 in, bf16 out only");
    const int64_t total = batch * n_q * (T / PF_QT / 2);
    if (total > 0x7fffffff) return fail(LITHOS_EINVAL, "attn_prefill: too many workgroups");
    plan->grid = {(uint32_t)(n_q / n_kv * (T / PF_QT / 2)), (uint32_t)n_kv, (uint32_t)batch};
    plan->total = (uint32_t)total;
    plan->threads = 256;
    plan->variant = 0;
    plan->wg_per_cu = cached_occupancy((const void*)attn_prefill_kernel, 256, 2);
    return LITHOS_OK;
}

int attn_prefill_launch(const lithos_op_t& op, const OpPlan& plan, const AtomArgs& atom, hipStream_t s)
{
    PrefillArgs a{};
    a.q = (const uint16_t*)op.in[0];
    a.k = (const uint16_t*)op.in[1];
    a.v = (const uint16_t*)op.in[2];
    a.o = (uint16_t*)op.out[0];
    a.batch = (int)op.dim[0]; a.n_q = (int)op.dim[1]; a.n_kv = (int)op.dim[2]; a.T = (int)op.dim[4]; a.cap = (int)op.dim[5];
    a.ldq = op.ld[0]; a.ldo = op.ld[1];
    a.scale_log2e = op.fparam[0] * 1.44269504088896340736f;
    LITHOS_HIP(launch_kernel(attn_prefill_kernel, dim3(LITHOS_ATOM_LAUNCH_BLOCKS(atom)), dim3(plan.threads), s, a, atom));
    return LITHOS_OK;
}

} // namespace lithos
