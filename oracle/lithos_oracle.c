/*
 * CPU oracle for the atomized operator kernels.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is a plain, slow, obviously-correct
 * implementation of what each operator computes.  It shares no code, header,
 * table or helper with the HIP path, and nothing in the product library may
 * call it.  All arithmetic is fp64; every loop follows the mathematical
 * definition of the operator in its textbook order (no blocking, no fusion).
 *
 * The paper (LithOS, Section 4.4) treats operator kernels as opaque: it only
 * requires that an atomized launch computes exactly what the single launch
 * computes.  The operator definitions below are therefore the standard ones
 * for the operator families the build targets (GEMM, bias+GELU, LayerNorm,
 * softmax, attention, RMSNorm, rotary embedding, SiLU-gate).
 *
 * Conventions: row-major; bf16 values travel as uint16_t bit patterns;
 * all fp64 buffers are caller-owned; functions return 0 or a negative code
 * for a bad argument.
 *
 * Parity pins live in tests/test_oracle_*.py (closed forms, identities,
 * brute-force triple loops, exactly representable data).
 */
#include <math.h>
#include <stdint.h>
#include <stddef.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* ---------------------------------------------------------------- bf16 --- */

/* bf16 = sign(1) exponent(8, bias 127) fraction(7): the upper half of an
 * IEEE-754 binary32 pattern.  Widening to fp64 is exact. */
double lo_bf16_to_f64(uint16_t h)
{
    uint32_t w = (uint32_t)h << 16;
    float f;
    memcpy(&f, &w, sizeof f);
    return (double)f;
}

/* Round an fp64 value to the nearest bf16, ties to the even significand.
 * Done on the value itself (not through an intermediate binary32), so there
 * is a single rounding.  NaN -> quiet NaN, +-Inf kept, overflow -> +-Inf,
 * results below 2^-126 land on the bf16 subnormal grid (step 2^-133). */
uint16_t lo_f64_to_bf16(double d)
{
    uint16_t sign = signbit(d) ? 0x8000u : 0u;
    if (isnan(d)) return (uint16_t)(sign | 0x7FC0u);
    double a = fabs(d);
    if (isinf(a)) return (uint16_t)(sign | 0x7F80u);
    if (a == 0.0) return sign;
    const double min_normal = ldexp(1.0, -126);
    if (a < min_normal) {
        /* subnormal grid: multiples of 2^-133; 128 steps reach 2^-126 */
        double q = nearbyint(ldexp(a, 133)); /* default mode: ties-to-even */
        return (uint16_t)(sign | (uint16_t)q);
    }
    int e;
    double m = frexp(a, &e);            /* a = m * 2^e, m in [0.5, 1)      */
    double scaled = ldexp(m, 8);        /* in [128, 256): 8 significant bits */
    double q = nearbyint(scaled);       /* exact RNE at the 8th bit         */
    int be = e - 1 + 127;               /* biased exponent of 1.xxx * 2^(e-1) */
    if (q == 256.0) { q = 128.0; be += 1; }
    if (be >= 255) return (uint16_t)(sign | 0x7F80u);
    return (uint16_t)(sign | ((uint16_t)be << 7) | ((uint16_t)q - 128u));
}

void lo_bf16_to_f64_array(const uint16_t *in, double *out, size_t n)
{
    for (size_t i = 0; i < n; ++i) out[i] = lo_bf16_to_f64(in[i]);
}

void lo_f64_to_bf16_array(const double *in, uint16_t *out, size_t n)
{
    for (size_t i = 0; i < n; ++i) out[i] = lo_f64_to_bf16(in[i]);
}

/* value-level rounding: out[i] = the bf16 nearest to in[i], held as fp64 */
void lo_round_bf16_array(const double *in, double *out, size_t n)
{
    for (size_t i = 0; i < n; ++i) out[i] = lo_bf16_to_f64(lo_f64_to_bf16(in[i]));
}

/* ---------------------------------------------------------------- GEMM --- */

/* C[i,j] = sum_{k=0}^{K-1} op(A)[i,k] * op(B)[k,j], k ascending, fp64.
 * op(A)[i,k] = ta ? A[k*lda+i] : A[i*lda+k]
 * op(B)[k,j] = tb ? B[j*ldb+k] : B[k*ldb+j]
 * B is bf16 bit patterns (the very bits the GPU kernel reads).  A is given as
 * fp64 values that are exactly the GPU's activations (widened bf16 bits, or
 * widened fp32 for kernels that read fp32 activations); a product of an fp32
 * and a bf16 value is exact in fp64, so the only rounding is the running sum.
 * Rows are independent and may run on separate threads. */
int lo_gemm(int ta, int tb, int64_t M, int64_t N, int64_t K,
            const double *A, int64_t lda,
            const uint16_t *B, int64_t ldb,
            double *C, int64_t ldc)
{
    if (M < 0 || N < 0 || K < 0 || ldc < N) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i) {
        for (int64_t j = 0; j < N; ++j) {
            double s = 0.0;
            for (int64_t k = 0; k < K; ++k) {
                double a = ta ? A[k * lda + i] : A[i * lda + k];
                double b = lo_bf16_to_f64(tb ? B[j * ldb + k] : B[k * ldb + j]);
                s += a * b;
            }
            C[i * ldc + j] = s;
        }
    }
    return 0;
}

/* Same sums, same ascending-k order per element, but the two inner loops are
 * swapped (i, k, j) so a row-major non-transposed B is read contiguously.
 * Every C[i,j] still receives its K products in ascending k, so the result
 * is bit-identical to lo_gemm; it exists only so full-size checks finish. */
int lo_gemm_rowsweep(int ta, int64_t M, int64_t N, int64_t K,
                     const double *A, int64_t lda,
                     const uint16_t *B, int64_t ldb,
                     double *C, int64_t ldc)
{
    if (M < 0 || N < 0 || K < 0 || ldc < N) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i) {
        double *c = C + i * ldc;
        for (int64_t j = 0; j < N; ++j) c[j] = 0.0;
        for (int64_t k = 0; k < K; ++k) {
            double a = ta ? A[k * lda + i] : A[i * lda + k];
            const uint16_t *b = B + k * ldb;
            for (int64_t j = 0; j < N; ++j) c[j] += a * lo_bf16_to_f64(b[j]);
        }
    }
    return 0;
}

/* K cut into ranges: C = sum_z A[:, K_z] B[K_z, :].  The planes hold the partial
 * products of the ranges; they are added in range order, plane 0 first. */
int lo_sum_slices(int64_t slices, int64_t n, const double *planes, double *out)
{
    if (slices < 1 || n < 0) return -1;
    for (int64_t i = 0; i < n; ++i) {
        double s = planes[i];
        for (int64_t z = 1; z < slices; ++z) s += planes[z * n + i];
        out[i] = s;
    }
    return 0;
}

/* -------------------------------------------------------- bias + GELU --- */

/* exact (erf) GELU: g(u) = u/2 * (1 + erf(u / sqrt 2)) */
double lo_gelu(double u) { return 0.5 * u * (1.0 + erf(u * M_SQRT1_2)); }

/* y[r,c] = g(x[r,c] + bias[c]); bias may be NULL (treated as 0);
 * gelu = 0 leaves the sum unactivated. */
int lo_bias_act(int64_t rows, int64_t cols, const double *x, const double *bias,
                int gelu, double *y)
{
    if (rows < 0 || cols < 0) return -1;
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t c = 0; c < cols; ++c) {
            double u = x[r * cols + c] + (bias ? bias[c] : 0.0);
            y[r * cols + c] = gelu ? lo_gelu(u) : u;
        }
    return 0;
}

/* ----------------------------------------------------------- LayerNorm --- */

/* per row: mu = mean(x); var = mean((x-mu)^2) (biased);
 * y = (x-mu)/sqrt(var+eps)*gamma + beta.  Two passes over the row. */
int lo_layernorm(int64_t rows, int64_t H, const double *x, const double *gamma,
                 const double *beta, double eps, double *y)
{
    if (rows < 0 || H <= 0) return -1;
    for (int64_t r = 0; r < rows; ++r) {
        const double *xr = x + r * H;
        double mu = 0.0;
        for (int64_t c = 0; c < H; ++c) mu += xr[c];
        mu /= (double)H;
        double var = 0.0;
        for (int64_t c = 0; c < H; ++c) var += (xr[c] - mu) * (xr[c] - mu);
        var /= (double)H;
        double rstd = 1.0 / sqrt(var + eps);
        for (int64_t c = 0; c < H; ++c)
            y[r * H + c] = (xr[c] - mu) * rstd * gamma[c] + beta[c];
    }
    return 0;
}

/* ------------------------------------------------------------- RMSNorm --- */

/* y = x / sqrt(mean(x^2) + eps) * w */
int lo_rmsnorm(int64_t rows, int64_t H, const double *x, const double *w,
               double eps, double *y)
{
    if (rows < 0 || H <= 0) return -1;
    for (int64_t r = 0; r < rows; ++r) {
        const double *xr = x + r * H;
        double ms = 0.0;
        for (int64_t c = 0; c < H; ++c) ms += xr[c] * xr[c];
        ms /= (double)H;
        double rinv = 1.0 / sqrt(ms + eps);
        for (int64_t c = 0; c < H; ++c) y[r * H + c] = xr[c] * rinv * w[c];
    }
    return 0;
}

/* ------------------------------------------------------------- softmax --- */

/* p_j = exp(s_j - max s) / sum_j exp(s_j - max s), per row */
int lo_softmax(int64_t rows, int64_t n, const double *s, double *p)
{
    if (rows < 0 || n <= 0) return -1;
    for (int64_t r = 0; r < rows; ++r) {
        const double *sr = s + r * n;
        double mx = sr[0];
        for (int64_t j = 1; j < n; ++j) if (sr[j] > mx) mx = sr[j];
        double den = 0.0;
        for (int64_t j = 0; j < n; ++j) den += exp(sr[j] - mx);
        for (int64_t j = 0; j < n; ++j) p[r * n + j] = exp(sr[j] - mx) / den;
    }
    return 0;
}

/* ----------------------------------------------------------- attention --- */

/* O[b,i,h,:] = sum_j softmax_j( Q[b,i,h,:] . K[b,j,g,:] * scale ) V[b,j,g,:]
 * with g = h / (Hq / Hkv) (grouped-query sharing; Hq == Hkv is plain
 * multi-head).  No mask: every query sees all Sk keys.
 * Element strides (in doubles): X[b,t,h,e] = X[b*xb + t*xt + h*xh + e]. */
int lo_attention(int64_t Bn, int64_t Hq, int64_t Hkv, int64_t Sq, int64_t Sk, int64_t d,
                 const double *Q, int64_t qb, int64_t qt, int64_t qh,
                 const double *Kx, int64_t kb, int64_t kt, int64_t kh,
                 const double *V, int64_t vb, int64_t vt, int64_t vh,
                 double scale,
                 double *O, int64_t ob, int64_t ot, int64_t oh)
{
    if (Hkv <= 0 || Hq % Hkv != 0 || Sk <= 0 || d <= 0) return -1;
    int64_t group = Hq / Hkv;
    int64_t work = Bn * Hq * Sq;
#pragma omp parallel
    {
        double *p = (double *)__builtin_malloc((size_t)Sk * sizeof(double));
#pragma omp for schedule(static)
        for (int64_t w = 0; w < work; ++w) {
            int64_t b = w / (Hq * Sq), h = (w / Sq) % Hq, i = w % Sq;
            int64_t g = h / group;
            const double *q = Q + b * qb + i * qt + h * qh;
            double mx = -INFINITY;
            for (int64_t j = 0; j < Sk; ++j) {
                const double *kk = Kx + b * kb + j * kt + g * kh;
                double s = 0.0;
                for (int64_t e = 0; e < d; ++e) s += q[e] * kk[e];
                p[j] = s * scale;
                if (p[j] > mx) mx = p[j];
            }
            double den = 0.0;
            for (int64_t j = 0; j < Sk; ++j) { p[j] = exp(p[j] - mx); den += p[j]; }
            double *o = O + b * ob + i * ot + h * oh;
            for (int64_t e = 0; e < d; ++e) {
                double acc = 0.0;
                for (int64_t j = 0; j < Sk; ++j)
                    acc += (p[j] / den) * V[b * vb + j * vt + g * vh + e];
                o[e] = acc;
            }
        }
        __builtin_free(p);
    }
    return 0;
}

/* Causal self-attention over a prompt: query i (0-based, Sq == Sk positions)
 * sees keys 0..i only:
 *   O[b,i,h,:] = sum_{j<=i} softmax_{j<=i}( Q[b,i,h,:] . K[b,j,g,:] * scale ) V[b,j,g,:]
 * Same layout and grouped-query rule as lo_attention. */
int lo_attention_causal(int64_t Bn, int64_t Hq, int64_t Hkv, int64_t S, int64_t d,
                        const double *Q, int64_t qb, int64_t qt, int64_t qh,
                        const double *Kx, int64_t kb, int64_t kt, int64_t kh,
                        const double *V, int64_t vb, int64_t vt, int64_t vh,
                        double scale,
                        double *O, int64_t ob, int64_t ot, int64_t oh)
{
    if (Hkv <= 0 || Hq % Hkv != 0 || S <= 0 || d <= 0) return -1;
    int64_t group = Hq / Hkv;
    int64_t work = Bn * Hq * S;
#pragma omp parallel
    {
        double *p = (double *)__builtin_malloc((size_t)S * sizeof(double));
#pragma omp for schedule(dynamic, 16)
        for (int64_t w = 0; w < work; ++w) {
            int64_t b = w / (Hq * S), h = (w / S) % Hq, i = w % S;
            int64_t g = h / group;
            const double *q = Q + b * qb + i * qt + h * qh;
            double mx = -INFINITY;
            for (int64_t j = 0; j <= i; ++j) {
                const double *kk = Kx + b * kb + j * kt + g * kh;
                double s = 0.0;
                for (int64_t e = 0; e < d; ++e) s += q[e] * kk[e];
                p[j] = s * scale;
                if (p[j] > mx) mx = p[j];
            }
            double den = 0.0;
            for (int64_t j = 0; j <= i; ++j) { p[j] = exp(p[j] - mx); den += p[j]; }
            double *o = O + b * ob + i * ot + h * oh;
            for (int64_t e = 0; e < d; ++e) {
                double acc = 0.0;
                for (int64_t j = 0; j <= i; ++j)
                    acc += (p[j] / den) * V[b * vb + j * vt + g * vh + e];
                o[e] = acc;
            }
        }
        __builtin_free(p);
    }
    return 0;
}

/* ---------------------------------------------------- rotary embedding --- */

/* Rotate-half pairing on a head of even width d: element e < d/2 is paired
 * with e + d/2; angle = pos * theta^(-2e/d).
 *   y[e]       = x[e] cos - x[e+d/2] sin
 *   y[e+d/2]   = x[e+d/2] cos + x[e] sin
 * x, y: [rows, heads, d] contiguous; pos[rows] integer positions. */
int lo_rope(int64_t rows, int64_t heads, int64_t d, const double *x,
            const int64_t *pos, double theta, double *y)
{
    if (d <= 0 || (d & 1)) return -1;
    int64_t half = d / 2;
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t h = 0; h < heads; ++h) {
            const double *xi = x + (r * heads + h) * d;
            double *yo = y + (r * heads + h) * d;
            for (int64_t e = 0; e < half; ++e) {
                double ang = (double)pos[r] * pow(theta, -2.0 * (double)e / (double)d);
                double c = cos(ang), s = sin(ang);
                double x0 = xi[e], x1 = xi[e + half];
                yo[e] = x0 * c - x1 * s;
                yo[e + half] = x1 * c + x0 * s;
            }
        }
    return 0;
}

/* ----------------------------------------------------------- SiLU gate --- */

/* y = silu(g) * u, silu(g) = g / (1 + exp(-g)) */
int lo_silu_mul(size_t n, const double *g, const double *u, double *y)
{
    for (size_t i = 0; i < n; ++i) y[i] = g[i] / (1.0 + exp(-g[i])) * u[i];
    return 0;
}

int lo_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
