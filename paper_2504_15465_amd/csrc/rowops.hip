// Atom-aware row and elementwise kernels for gfx950: bias+activation,
// LayerNorm, RMSNorm, softmax, SiLU-gate, rotary embedding + cache append,
// and a fixed-duration spin kernel for scheduler tests.
//
// All are HBM-bound (a few flops per byte): the design rule is coalesced
// access and wavefront reductions, fp32 arithmetic on bf16 or fp32 data.
// Each workgroup handles the rows / elements named by its LOGICAL block index
// (LithOS Section 4.4), so any sub-range of blocks is a valid atom.
#include "common.hpp"
#include <math.h>

namespace lithos {

struct RowArgs {
    const void* x;
    const float* p0;     // bias / gamma / weight
    const float* p1;     // beta
    void* y;
    void* y2;            // optional bf16 copy
    int64_t rows, cols;
    float f0;            // eps / scale / theta
    uint32_t flags;
    int64_t aux[5];
};

__device__ __forceinline__ float bf16_bits_to_f32(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }

__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

template <bool F32>
__device__ __forceinline__ float load_elem(const void* p, int64_t i)
{
    if constexpr (F32) return reinterpret_cast<const float*>(p)[i];
    else return bf16_bits_to_f32(reinterpret_cast<const uint16_t*>(p)[i]);
}

template <bool F32>
__device__ __forceinline__ void store_elem(void* p, int64_t i, float v)
{
    if constexpr (F32) reinterpret_cast<float*>(p)[i] = v;
    else reinterpret_cast<uint16_t*>(p)[i] = f32_to_bf16_bits(v);
}

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
    return v;
}

// Sum over the TPR threads that share a row (TPR = 64: one wavefront;
// TPR = 256: the whole workgroup through LDS).  Fixed order: deterministic.
template <int TPR>
__device__ __forceinline__ float row_sum(float v, float* red)
{
    v = wave_sum(v);
    if constexpr (TPR == 256) {
        __syncthreads();
        if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
        __syncthreads();
        v = red[0] + red[1] + red[2] + red[3];
    }
    return v;
}

template <int TPR>
__device__ __forceinline__ float row_max(float v, float* red)
{
    v = wave_max(v);
    if constexpr (TPR == 256) {
        __syncthreads();
        if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
        __syncthreads();
        v = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    }
    return v;
}

__device__ __forceinline__ float gelu_erf_f(float u)
{
    return 0.5f * u * (1.0f + erff(u * 0.70710678118654752440f));
}

// ---- y = act(x + bias): 2048 consecutive elements per block ---------------
template <bool IN32, bool OUT32>
__global__ __launch_bounds__(256) void bias_act_kernel(RowArgs a, AtomArgs atom)
{
    const uint32_t L = atom_logical_block(atom);
    const int64_t total = a.rows * a.cols;
    const int64_t base = (int64_t)L * 2048;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        int64_t idx = base + threadIdx.x + i * 256;
        if (idx < total) {
            float v = load_elem<IN32>(a.x, idx);
            if (a.flags & LITHOS_F_BIAS) v += a.p0[idx % a.cols];
            if (a.flags & LITHOS_F_GELU) v = gelu_erf_f(v);
            store_elem<OUT32>(a.y, idx, v);
            if (!OUT32 && (a.flags & LITHOS_F_OUT_SPLIT)) {      // lo plane follows the hi plane
                float hi = bf16_bits_to_f32(f32_to_bf16_bits(v));
                reinterpret_cast<uint16_t*>(a.y)[total + idx] = f32_to_bf16_bits(v - hi);
            }
        }
    }
}

// ---- y = act(sum_z plane_z + bias) + residual: 2048 consecutive elements per block ----
// The planes are the fp32 partial products of a K-sliced GEMM; they are added in
// slice order, starting from plane 0, so the sum is the same for every launch shape.
// VEC: four elements per thread and step (cols, strides and pointers permit 16-byte access).
template <bool OUT32, bool VEC>
__global__ __launch_bounds__(256) void sum_slices_kernel(RowArgs a, AtomArgs atom)
{
    const uint32_t L = atom_logical_block(atom);
    const int64_t total = a.rows * a.cols;
    const int64_t base = (int64_t)L * 2048;
    const float* planes = reinterpret_cast<const float*>(a.x);
    const int64_t S = a.aux[0], plane = a.aux[1], ldx = a.aux[2], ldy = a.aux[3];
    const int64_t ldr = a.aux[4];
    constexpr int W = VEC ? 4 : 1;
#pragma unroll
    for (int i = 0; i < 8 / W; ++i) {
        const int64_t idx = base + ((int64_t)threadIdx.x + i * 256) * W;
        if (idx >= total) continue;
        const int64_t r = idx / a.cols, c = idx % a.cols;
        float v[W];
        if constexpr (VEC) {
            float4 s = *reinterpret_cast<const float4*>(planes + r * ldx + c);
            for (int64_t z = 1; z < S; ++z) {
                const float4 t = *reinterpret_cast<const float4*>(planes + z * plane + r * ldx + c);
                s.x += t.x; s.y += t.y; s.z += t.z; s.w += t.w;
            }
            v[0] = s.x; v[1] = s.y; v[2] = s.z; v[3] = s.w;
        } else {
            float s = planes[r * ldx + c];
            for (int64_t z = 1; z < S; ++z) s += planes[z * plane + r * ldx + c];
            v[0] = s;
        }
#pragma unroll
        for (int t = 0; t < W; ++t) {
            if (a.flags & LITHOS_F_BIAS) v[t] += a.p0[c + t];
            if (a.flags & LITHOS_F_GELU) v[t] = gelu_erf_f(v[t]);
            if (a.flags & LITHOS_F_RESIDUAL) v[t] += a.p1[r * ldr + c + t];
        }
        if constexpr (VEC && OUT32) {
            *reinterpret_cast<float4*>(reinterpret_cast<float*>(a.y) + r * ldy + c) = make_float4(v[0], v[1], v[2], v[3]);
        } else if constexpr (VEC) {
            *reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(a.y) + r * ldy + c) =
                make_uint2(f32_to_bf16_bits(v[0]) | ((uint32_t)f32_to_bf16_bits(v[1]) << 16),
                           f32_to_bf16_bits(v[2]) | ((uint32_t)f32_to_bf16_bits(v[3]) << 16));
        } else {
            store_elem<OUT32>(a.y, r * ldy + c, v[0]);
        }
    }
}

// ---- y[r, :F] = silu(gu[r, :F]) * gu[r, F:2F] ------------------------------
template <bool IN32, bool OUT32>
__global__ __launch_bounds__(256) void silu_mul_kernel(RowArgs a, AtomArgs atom)
{
    const uint32_t L = atom_logical_block(atom);
    const int64_t F = a.cols, total = a.rows * F;
    const int64_t base = (int64_t)L * 2048;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        int64_t idx = base + threadIdx.x + i * 256;
        if (idx < total) {
            int64_t r = idx / F, c = idx % F;
            float g = load_elem<IN32>(a.x, r * 2 * F + c);
            float u = load_elem<IN32>(a.x, r * 2 * F + F + c);
            float v = g / (1.0f + expf(-g)) * u;
            store_elem<OUT32>(a.y, idx, v);
        }
    }
}

// ---- LayerNorm: two passes over the row (mean, then centred variance) ------
template <bool IN32, bool OUT32, int TPR>
__global__ __launch_bounds__(256) void layernorm_kernel(RowArgs a, AtomArgs atom)
{
    __shared__ float red[4];
    const uint32_t L = atom_logical_block(atom);
    constexpr int RPB = 256 / TPR;
    const int64_t row = (int64_t)L * RPB + threadIdx.x / TPR;
    const int t = threadIdx.x % TPR;
    const bool live = row < a.rows;
    const int64_t H = a.cols, off = row * H;
    float s = 0.0f;
    if (live) for (int64_t c = t; c < H; c += TPR) s += load_elem<IN32>(a.x, off + c);
    const float mean = row_sum<TPR>(s, red) / (float)H;
    float q = 0.0f;
    if (live) for (int64_t c = t; c < H; c += TPR) { float d = load_elem<IN32>(a.x, off + c) - mean; q += d * d; }
    const float var = row_sum<TPR>(q, red) / (float)H;
    const float rstd = 1.0f / sqrtf(var + a.f0);
    if (live) for (int64_t c = t; c < H; c += TPR) {
        float v = (load_elem<IN32>(a.x, off + c) - mean) * rstd * a.p0[c] + a.p1[c];
        store_elem<OUT32>(a.y, off + c, v);
        if (OUT32 && a.y2) {
            uint16_t hi = f32_to_bf16_bits(v);
            reinterpret_cast<uint16_t*>(a.y2)[off + c] = hi;
            if (a.flags & LITHOS_F_OUT_SPLIT)
                reinterpret_cast<uint16_t*>(a.y2)[a.rows * H + off + c] = f32_to_bf16_bits(v - bf16_bits_to_f32(hi));
        }
    }
}

// Register-resident variant: the row is read ONCE with 16-byte (fp32) or
// 8-byte (bf16) loads, four elements per thread and step, and stays in
// registers for the mean, the centred variance and the output.  Needs
// H % 4 == 0 and H <= 16 * TPR.
template <bool IN32, bool OUT32, int TPR>
__global__ __launch_bounds__(256) void layernorm_vec_kernel(RowArgs a, AtomArgs atom)
{
    __shared__ float red[4];
    constexpr int NV = 4;                                   // 4-element groups per thread
    const uint32_t L = atom_logical_block(atom);
    constexpr int RPB = 256 / TPR;
    const int64_t row = (int64_t)L * RPB + threadIdx.x / TPR;
    const int t = threadIdx.x % TPR;
    const bool live = row < a.rows;
    const int64_t H = a.cols, off = row * H;
    float v[NV][4];
    float s = 0.0f;
#pragma unroll
    for (int j = 0; j < NV; ++j) {
        const int64_t c = 4 * (t + (int64_t)j * TPR);
        v[j][0] = v[j][1] = v[j][2] = v[j][3] = 0.0f;
        if (live && c < H) {
            if constexpr (IN32) {
                const float4 f = *reinterpret_cast<const float4*>(reinterpret_cast<const float*>(a.x) + off + c);
                v[j][0] = f.x; v[j][1] = f.y; v[j][2] = f.z; v[j][3] = f.w;
            } else {
                const uint2 u = *reinterpret_cast<const uint2*>(reinterpret_cast<const uint16_t*>(a.x) + off + c);
                v[j][0] = __uint_as_float(u.x << 16); v[j][1] = __uint_as_float(u.x & 0xffff0000u);
                v[j][2] = __uint_as_float(u.y << 16); v[j][3] = __uint_as_float(u.y & 0xffff0000u);
            }
            s += (v[j][0] + v[j][1]) + (v[j][2] + v[j][3]);
        }
    }
    const float mean = row_sum<TPR>(s, red) / (float)H;
    float q = 0.0f;
#pragma unroll
    for (int j = 0; j < NV; ++j) {
        const int64_t c = 4 * (t + (int64_t)j * TPR);
        if (live && c < H)
#pragma unroll
            for (int e = 0; e < 4; ++e) { const float d = v[j][e] - mean; q += d * d; }
    }
    const float var = row_sum<TPR>(q, red) / (float)H;
    const float rstd = 1.0f / sqrtf(var + a.f0);
#pragma unroll
    for (int j = 0; j < NV; ++j) {
        const int64_t c = 4 * (t + (int64_t)j * TPR);
        if (live && c < H) {
            const float4 gm = *reinterpret_cast<const float4*>(a.p0 + c);
            const float4 bt = *reinterpret_cast<const float4*>(a.p1 + c);
            float y[4];
            y[0] = (v[j][0] - mean) * rstd * gm.x + bt.x;
            y[1] = (v[j][1] - mean) * rstd * gm.y + bt.y;
            y[2] = (v[j][2] - mean) * rstd * gm.z + bt.z;
            y[3] = (v[j][3] - mean) * rstd * gm.w + bt.w;
            uint16_t hi[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) hi[e] = f32_to_bf16_bits(y[e]);
            if constexpr (OUT32) {
                *reinterpret_cast<float4*>(reinterpret_cast<float*>(a.y) + off + c) = make_float4(y[0], y[1], y[2], y[3]);
                if (a.y2) {
                    uint16_t* y2 = reinterpret_cast<uint16_t*>(a.y2);
                    *reinterpret_cast<uint2*>(y2 + off + c) = make_uint2(hi[0] | ((uint32_t)hi[1] << 16), hi[2] | ((uint32_t)hi[3] << 16));
                    if (a.flags & LITHOS_F_OUT_SPLIT) {
                        uint16_t lo[4];
#pragma unroll
                        for (int e = 0; e < 4; ++e) lo[e] = f32_to_bf16_bits(y[e] - bf16_bits_to_f32(hi[e]));
                        *reinterpret_cast<uint2*>(y2 + a.rows * H + off + c) = make_uint2(lo[0] | ((uint32_t)lo[1] << 16), lo[2] | ((uint32_t)lo[3] << 16));
                    }
                }
            } else {
                *reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(a.y) + off + c) = make_uint2(hi[0] | ((uint32_t)hi[1] << 16), hi[2] | ((uint32_t)hi[3] << 16));
            }
        }
    }
}

// ---- RMSNorm ----------------------------------------------------------------
template <bool IN32, bool OUT32, int TPR>
__global__ __launch_bounds__(256) void rmsnorm_kernel(RowArgs a, AtomArgs atom)
{
    __shared__ float red[4];
    const uint32_t L = atom_logical_block(atom);
    constexpr int RPB = 256 / TPR;
    const int64_t row = (int64_t)L * RPB + threadIdx.x / TPR;
    const int t = threadIdx.x % TPR;
    const bool live = row < a.rows;
    const int64_t H = a.cols, off = row * H;
    float s = 0.0f;
    if (live) for (int64_t c = t; c < H; c += TPR) { float v = load_elem<IN32>(a.x, off + c); s += v * v; }
    const float ms = row_sum<TPR>(s, red) / (float)H;
    const float rinv = 1.0f / sqrtf(ms + a.f0);
    if (live) for (int64_t c = t; c < H; c += TPR)
        store_elem<OUT32>(a.y, off + c, load_elem<IN32>(a.x, off + c) * rinv * a.p0[c]);
}

// Register-resident variant (H % 4 == 0, H <= 16 * TPR): the row is read once with
// 16-byte (fp32) or 8-byte (bf16) loads that are all in flight together.
template <bool IN32, bool OUT32, int TPR>
__global__ __launch_bounds__(256) void rmsnorm_vec_kernel(RowArgs a, AtomArgs atom)
{
    __shared__ float red[4];
    constexpr int NV = 4;
    const uint32_t L = atom_logical_block(atom);
    constexpr int RPB = 256 / TPR;
    const int64_t row = (int64_t)L * RPB + threadIdx.x / TPR;
    const int t = threadIdx.x % TPR;
    const bool live = row < a.rows;
    const int64_t H = a.cols, off = row * H;
    float v[NV][4];
    float4 w[NV];
    float s = 0.0f;
#pragma unroll
    for (int j = 0; j < NV; ++j) {
        const int64_t c = 4 * (t + (int64_t)j * TPR);
        v[j][0] = v[j][1] = v[j][2] = v[j][3] = 0.0f;
        w[j] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (live && c < H) {
            if constexpr (IN32) {
                const float4 f = *reinterpret_cast<const float4*>(reinterpret_cast<const float*>(a.x) + off + c);
                v[j][0] = f.x; v[j][1] = f.y; v[j][2] = f.z; v[j][3] = f.w;
            } else {
                const uint2 u = *reinterpret_cast<const uint2*>(reinterpret_cast<const uint16_t*>(a.x) + off + c);
                v[j][0] = __uint_as_float(u.x << 16); v[j][1] = __uint_as_float(u.x & 0xffff0000u);
                v[j][2] = __uint_as_float(u.y << 16); v[j][3] = __uint_as_float(u.y & 0xffff0000u);
            }
            w[j] = *reinterpret_cast<const float4*>(a.p0 + c);
        }
    }
#pragma unroll
    for (int j = 0; j < NV; ++j)
#pragma unroll
        for (int e = 0; e < 4; ++e) s += v[j][e] * v[j][e];
    const float ms = row_sum<TPR>(s, red) / (float)H;
    const float rinv = 1.0f / sqrtf(ms + a.f0);
#pragma unroll
    for (int j = 0; j < NV; ++j) {
        const int64_t c = 4 * (t + (int64_t)j * TPR);
        if (live && c < H) {
            const float y[4] = {v[j][0] * rinv * w[j].x, v[j][1] * rinv * w[j].y, v[j][2] * rinv * w[j].z, v[j][3] * rinv * w[j].w};
            if constexpr (OUT32) {
                *reinterpret_cast<float4*>(reinterpret_cast<float*>(a.y) + off + c) = make_float4(y[0], y[1], y[2], y[3]);
            } else {
                uint16_t h[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) h[e] = f32_to_bf16_bits(y[e]);
                *reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(a.y) + off + c) =
                    make_uint2(h[0] | ((uint32_t)h[1] << 16), h[2] | ((uint32_t)h[3] << 16));
            }
        }
    }
}

// ---- softmax(scale * s) -----------------------------------------------------
template <bool IN32, bool OUT32, int TPR>
__global__ __launch_bounds__(256) void softmax_kernel(RowArgs a, AtomArgs atom)
{
    __shared__ float red[4];
    const uint32_t L = atom_logical_block(atom);
    constexpr int RPB = 256 / TPR;
    const int64_t row = (int64_t)L * RPB + threadIdx.x / TPR;
    const int t = threadIdx.x % TPR;
    const bool live = row < a.rows;
    const int64_t n = a.cols, off = row * n;
    float mx = -INFINITY;
    if (live) for (int64_t c = t; c < n; c += TPR) mx = fmaxf(mx, load_elem<IN32>(a.x, off + c) * a.f0);
    mx = row_max<TPR>(mx, red);
    float s = 0.0f;
    if (live) for (int64_t c = t; c < n; c += TPR) s += expf(load_elem<IN32>(a.x, off + c) * a.f0 - mx);
    const float den = row_sum<TPR>(s, red);
    if (live) for (int64_t c = t; c < n; c += TPR)
        store_elem<OUT32>(a.y, off + c, expf(load_elem<IN32>(a.x, off + c) * a.f0 - mx) / den);
}

// ---- rotary embedding of q and k heads in place + k,v appended to the cache --
// One wavefront per (row, head slot); slots 0..n_q-1 are query heads,
// n_q..n_q+n_kv-1 key heads, the rest value heads (copied to the cache only).
// aux = {n_q, n_kv, pos, cap}; cols = d.
template <bool F32>
__global__ __launch_bounds__(256) void rope_kv_kernel(RowArgs a, AtomArgs atom)
{
    const uint32_t L = atom_logical_block(atom);
    const int64_t n_q = a.aux[0], n_kv = a.aux[1], pos = a.aux[2], cap = a.aux[3], d = a.cols;
    const int64_t slots = n_q + 2 * n_kv;
    const int64_t unit = (int64_t)L * 4 + (threadIdx.x >> 6);
    if (unit >= a.rows * slots) return;
    const int lane = threadIdx.x & 63;
    const int64_t row = unit / slots, slot = unit % slots;
    void* head = const_cast<void*>(a.x);
    const int64_t hoff = row * slots * d + slot * d;
    uint16_t* kc = reinterpret_cast<uint16_t*>(a.y);
    uint16_t* vc = reinterpret_cast<uint16_t*>(a.y2);
    const int64_t half = d / 2;
    if (slot < n_q + n_kv) {
        uint16_t* dst = nullptr;
        if (slot >= n_q) dst = kc + ((row * cap + pos) * n_kv + (slot - n_q)) * d;
        for (int64_t e = lane; e < half; e += 64) {
            float inv = powf(a.f0, -2.0f * (float)e / (float)d);
            float sn, cs;
            sincosf((float)pos * inv, &sn, &cs);
            float x0 = load_elem<F32>(head, hoff + e), x1 = load_elem<F32>(head, hoff + e + half);
            float r0 = x0 * cs - x1 * sn, r1 = x1 * cs + x0 * sn;
            store_elem<F32>(head, hoff + e, r0);
            store_elem<F32>(head, hoff + e + half, r1);
            if (dst) { dst[e] = f32_to_bf16_bits(r0); dst[e + half] = f32_to_bf16_bits(r1); }
        }
    } else {
        uint16_t* dst = vc + ((row * cap + pos) * n_kv + (slot - n_q - n_kv)) * d;
        for (int64_t e = lane; e < d; e += 64) dst[e] = f32_to_bf16_bits(load_elem<F32>(head, hoff + e));
    }
}

// ---- spin: every block waits `ticks` of the constant 100 MHz counter -------
// 1024 threads and 64 KB of LDS per block: exactly two blocks fit on a CU, so
// the kernel's latency is ticks * ceil(blocks / (2 * CUs)) - a known scaling
// curve for scheduler and right-sizing tests.
__global__ __launch_bounds__(1024) void spin_kernel(uint64_t ticks, AtomArgs atom)
{
    __shared__ uint32_t pad[16384];
    const uint32_t L = atom_logical_block(atom);
    if (threadIdx.x == 0) reinterpret_cast<volatile uint32_t*>(pad)[L & 16383] = L;
    const uint64_t t0 = wall_clock64();
    while (wall_clock64() - t0 < ticks) __builtin_amdgcn_s_sleep(8);
}

// ---- host side ----------------------------------------------------------------

static RowArgs make_args(const lithos_op_t& op)
{
    RowArgs a{};
    a.x = op.in[0];
    a.p0 = (const float*)op.in[1];
    a.p1 = (const float*)op.in[2];
    a.y = op.out[0];
    a.y2 = op.out[1];
    a.rows = op.dim[0];
    a.cols = op.dim[1];
    a.f0 = op.fparam[0];
    a.flags = op.flags;
    return a;
}

static int tpr_for(int64_t cols) { return cols <= 1024 ? 64 : 256; }

// The kernel that serves a descriptor (everything but SPIN, whose kernel has its own signature).
typedef void (*row_fn)(RowArgs, AtomArgs);
#define PICK2(K) (in32 ? (out32 ? (row_fn)K<true, true> : (row_fn)K<true, false>) : (out32 ? (row_fn)K<false, true> : (row_fn)K<false, false>))
#define PICK3(K, T) (in32 ? (out32 ? (row_fn)K<true, true, T> : (row_fn)K<true, false, T>) : (out32 ? (row_fn)K<false, true, T> : (row_fn)K<false, false, T>))
static row_fn row_kernel(const lithos_op_t& op, int variant)
{
    const bool in32 = op.flags & LITHOS_F_IN_F32, out32 = op.flags & LITHOS_F_OUT_F32;
    const bool wide = tpr_for(op.dim[1]) == 256;
    switch (op.kind) {
    case LITHOS_OP_BIAS_ACT: return PICK2(bias_act_kernel);
    case LITHOS_OP_SILU_MUL: return PICK2(silu_mul_kernel);
    case LITHOS_OP_SUM_SLICES:
        return variant == 1 ? (out32 ? (row_fn)sum_slices_kernel<true, true> : (row_fn)sum_slices_kernel<false, true>)
                            : (out32 ? (row_fn)sum_slices_kernel<true, false> : (row_fn)sum_slices_kernel<false, false>);
    case LITHOS_OP_LAYERNORM:
        if (variant == 1) return wide ? PICK3(layernorm_vec_kernel, 256) : PICK3(layernorm_vec_kernel, 64);   // register-resident rows
        return wide ? PICK3(layernorm_kernel, 256) : PICK3(layernorm_kernel, 64);
    case LITHOS_OP_RMSNORM:
        if (variant == 1) return wide ? PICK3(rmsnorm_vec_kernel, 256) : PICK3(rmsnorm_vec_kernel, 64);
        return wide ? PICK3(rmsnorm_kernel, 256) : PICK3(rmsnorm_kernel, 64);
    case LITHOS_OP_SOFTMAX: return wide ? PICK3(softmax_kernel, 256) : PICK3(softmax_kernel, 64);
    case LITHOS_OP_ROPE_KV: return in32 ? (row_fn)rope_kv_kernel<true> : (row_fn)rope_kv_kernel<false>;
    default: return nullptr;
    }
}
#undef PICK2
#undef PICK3

int rowops_plan(const lithos_op_t& op, OpPlan* plan)
{
    const int64_t rows = op.dim[0], cols = op.dim[1];
    if (rows <= 0 || cols <= 0 || rows > (1ll << 31) || cols > (1ll << 24))
        return fail(LITHOS_EINVAL, "row op %d: rows and cols must be positive (got %lld, %lld)", op.kind, (long long)rows, (long long)cols);
    if (!op.in[0] && op.kind != LITHOS_OP_SPIN) return fail(LITHOS_EINVAL, "row op %d: null input", op.kind);
    plan->threads = 256;
    plan->variant = 0;
    plan->wg_per_cu = 8;
    uint64_t blocks = 0;
    switch (op.kind) {
    case LITHOS_OP_BIAS_ACT:
        if (!op.out[0]) return fail(LITHOS_EINVAL, "bias_act: null output");
        if ((op.flags & LITHOS_F_BIAS) && !op.in[1]) return fail(LITHOS_EINVAL, "bias_act: BIAS set but in[1] is null");
        blocks = ((uint64_t)rows * cols + 2047) / 2048;
        break;
    case LITHOS_OP_SILU_MUL:
        if (!op.out[0]) return fail(LITHOS_EINVAL, "silu_mul: null output");
        blocks = ((uint64_t)rows * cols + 2047) / 2048;
        break;
    case LITHOS_OP_SUM_SLICES: {
        // dim = rows, cols, slices, slice plane stride; ld = row strides of the planes, of y, of the residual
        const int64_t S = op.dim[2], plane = op.dim[3], ldx = op.ld[0], ldy = op.ld[1], ldr = op.ld[2];
        if (!op.out[0]) return fail(LITHOS_EINVAL, "sum_slices: null output");
        if (S < 1 || S > LITHOS_GEMM_MAX_SLICES) return fail(LITHOS_EINVAL, "sum_slices: slices must be in [1, %d]", LITHOS_GEMM_MAX_SLICES);
        if (ldx < cols || ldy < cols || plane < rows * ldx) return fail(LITHOS_EINVAL, "sum_slices: row or plane stride too small");
        if ((op.flags & LITHOS_F_BIAS) && !op.in[1]) return fail(LITHOS_EINVAL, "sum_slices: BIAS set but in[1] is null");
        if ((op.flags & LITHOS_F_RESIDUAL) && (!op.in[2] || ldr < cols)) return fail(LITHOS_EINVAL, "sum_slices: RESIDUAL needs in[2] and ld[2] >= cols");
        if (op.flags & (LITHOS_F_IN_F32 | LITHOS_F_OUT_SPLIT)) return fail(LITHOS_EINVAL, "sum_slices: the planes are always fp32; no split output");
        blocks = ((uint64_t)rows * cols + 2047) / 2048;
        if (cols % 4 == 0 && ldx % 4 == 0 && ldy % 4 == 0 && plane % 4 == 0 && aligned16(op.in[0]) && aligned16(op.out[0]) &&
            (!(op.flags & LITHOS_F_RESIDUAL) || ldr % 4 == 0))
            plan->variant = 1;
        break;
    }
    case LITHOS_OP_LAYERNORM:
        if (!op.in[1] || !op.in[2] || !op.out[0]) return fail(LITHOS_EINVAL, "layernorm: null gamma, beta or output");
        if (!(op.flags & LITHOS_F_OUT_F32) && op.out[1]) return fail(LITHOS_EINVAL, "layernorm: a bf16 copy needs OUT_F32");
        blocks = (rows + (256 / tpr_for(cols)) - 1) / (256 / tpr_for(cols));
        if (cols % 4 == 0 && cols <= 16 * tpr_for(cols) && aligned16(op.in[0]) && aligned16(op.in[1]) && aligned16(op.in[2]) &&
            aligned16(op.out[0]) && (!op.out[1] || aligned16(op.out[1])))
            plan->variant = 1;
        break;
    case LITHOS_OP_RMSNORM:
        if (!op.in[1] || !op.out[0]) return fail(LITHOS_EINVAL, "rmsnorm: null weight or output");
        blocks = (rows + (256 / tpr_for(cols)) - 1) / (256 / tpr_for(cols));
        if (cols % 4 == 0 && cols <= 16 * tpr_for(cols) && aligned16(op.in[0]) && aligned16(op.in[1]) && aligned16(op.out[0]))
            plan->variant = 1;
        break;
    case LITHOS_OP_SOFTMAX:
        if (!op.out[0]) return fail(LITHOS_EINVAL, "softmax: null output");
        blocks = (rows + (256 / tpr_for(cols)) - 1) / (256 / tpr_for(cols));
        break;
    case LITHOS_OP_ROPE_KV: {
        // dim = rows, n_q, n_kv, d, pos, cap
        const int64_t n_q = op.dim[1], n_kv = op.dim[2], d = op.dim[3], pos = op.dim[4], cap = op.dim[5];
        if (n_q <= 0 || n_kv <= 0 || d <= 0 || (d & 1) || pos < 0 || pos >= cap)
            return fail(LITHOS_EINVAL, "rope_kv: need n_q,n_kv,d > 0, d even, 0 <= pos < cap");
        if (!op.out[0] || !op.out[1]) return fail(LITHOS_EINVAL, "rope_kv: null cache pointer");
        blocks = ((uint64_t)rows * (n_q + 2 * n_kv) + 3) / 4;
        break;
    }
    case LITHOS_OP_SPIN:
        if (op.dim[1] < 0 || op.dim[1] > 100000000) return fail(LITHOS_EINVAL, "spin: ticks must be in [0, 1e8] (1 s)");
        blocks = rows;
        plan->threads = 1024;
        plan->wg_per_cu = 2;
        break;
    default:
        return fail(LITHOS_EINVAL, "unknown row op kind %d", op.kind);
    }
    if (blocks == 0 || blocks > 0x7fffffffull) return fail(LITHOS_EINVAL, "row op %d: grid out of range", op.kind);
    plan->grid = {(uint32_t)blocks, 1, 1};
    plan->total = (uint32_t)blocks;
    // resident workgroups per CU: asked of the runtime once per kernel (it feeds the atom quantum and
    // the occupancy filter of right-sizing); the constants above only serve if the query fails
    const void* fn = op.kind == LITHOS_OP_SPIN ? (const void*)spin_kernel : (const void*)row_kernel(op, plan->variant);
    plan->wg_per_cu = cached_occupancy(fn, (int)plan->threads, plan->wg_per_cu);
    return LITHOS_OK;
}

int rowops_launch(const lithos_op_t& op, const OpPlan& plan, const AtomArgs& atom, hipStream_t s)
{
    const dim3 grid(LITHOS_ATOM_LAUNCH_BLOCKS(atom)), block(plan.threads);
    if (op.kind == LITHOS_OP_SPIN) {
        LITHOS_HIP(launch_kernel(spin_kernel, grid, block, s, (uint64_t)op.dim[1], atom));
        return LITHOS_OK;
    }
    RowArgs a = make_args(op);
    if (op.kind == LITHOS_OP_SUM_SLICES) {
        a.aux[0] = op.dim[2]; a.aux[1] = op.dim[3]; a.aux[2] = op.ld[0]; a.aux[3] = op.ld[1];
        a.aux[4] = op.ld[2];
    } else if (op.kind == LITHOS_OP_ROPE_KV) {
        a.cols = op.dim[3];
        a.aux[0] = op.dim[1]; a.aux[1] = op.dim[2]; a.aux[2] = op.dim[4]; a.aux[3] = op.dim[5];
        a.p0 = nullptr; a.p1 = nullptr;
    }
    row_fn fn = row_kernel(op, plan.variant);
    if (!fn) return fail(LITHOS_EINVAL, "unknown row op kind %d", op.kind);
    LITHOS_HIP(launch_kernel(fn, grid, block, s, a, atom));
    return LITHOS_OK;
}

} // namespace lithos
