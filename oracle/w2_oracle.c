/*
 * CPU oracle for the 2-bit-weight mixed-precision matmul
 *     Y[M,N] = X[M,K] . dequant(W2[K,N])
 *
 * THIS IS TEST INFRASTRUCTURE.  It is a plain, slow, loop-by-loop statement of
 * what the method computes, written from the paper's description, and it is
 * the thing the GPU library is checked against.  It shares no code, header,
 * table or helper with the HIP library and must never be called from the
 * product path; only the tests, the smoke check and the benchmark's
 * "cpu_baseline" leg use it.
 *
 * Naming follows the LLM convention (X = activations, M tokens; W = weights,
 * N output features).  The paper calls the weight matrix A (M x K there), the
 * activations B (N x K there) and the output C.
 *
 * What the paper fixes and where:
 *   - weights are 2-bit codes that are up-converted to int8 and multiplied
 *     with int8 activations into int32 accumulators       (Sec. II-A, II-C)
 *   - activations are quantised to int8 before the GEMM: abs-max per
 *     granularity gives the scale, entries are multiplied by the inverse of
 *     the scale and converted to int8                      (Sec. II-B, II-D)
 *   - the int32 result is converted to float, multiplied by the dequant
 *     scale = activation scale x weight scale, converted to bf16 (Sec. II-D)
 *   - one 16-bit scale per 128 weights along K (group-wise)  (Sec. III-F)
 *   - the 16-bit alternative leaves activations unquantised; the weight is
 *     code-value x group scale; fp32-or-better accumulate, no dequant step
 *                                  (Sec. II-D, "Alternative implementation")
 *
 * Readings where the paper is silent (each also listed in the design notes):
 *   - code -> value: int2 codec q = c - 2 (values -2,-1,0,1); ternary codec
 *     q = c - 1 (values -1,0,1), code 3 is illegal under the ternary codec
 *   - activation granularity: one scale per token (row of X) over all K
 *   - inv = 127/amax, t = x*inv, round half to even, clamp to [-127,127],
 *     sx = amax/127; all in IEEE binary32, each operation rounded once
 *   - an all-zero row gives inv = 0, sx = 0, xq = 0
 *   - per group: exact int32 sum; across groups: fp64 sum of
 *     scale x accumulator, g ascending; one rounding to bf16 (nearest even)
 *
 * Parity pins (tests/, not here): a hand-worked 2x8x4 example, numpy int64 /
 * fp64 matmuls of the dequantised operands, closed forms and invariants.
 *
 * Build: gcc -O2 -ffp-contract=off -fopenmp -shared -fPIC w2_oracle.c -lm
 * (-ffp-contract=off: the binary32 quantisation arithmetic must not be fused)
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define W2O_OK 0
#define W2O_ERR_ARG (-1)
#define W2O_ERR_BAD_CODE (-6)

/* ---- bf16 <-> wider formats ------------------------------------------ */

/* bf16 is the upper 16 bits of an IEEE binary32: widening is exact. */
float w2o_bf16_to_f32(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

/* Round a double to the nearest bf16 (ties to even) in ONE rounding.
 * bf16 has 8 significant bits (1 implicit + 7 stored) and binary32's exponent
 * range; below 2^-126 the spacing is fixed at 2^-133 (subnormals). */
uint16_t w2o_f64_to_bf16(double v)
{
    if (isnan(v)) return 0x7fc0;
    uint16_t sign = signbit(v) ? 0x8000 : 0;
    double a = fabs(v);
    if (isinf(a)) return sign | 0x7f80;
    if (a == 0.0) return sign;
    int e;                         /* a = f * 2^e, f in [0.5,1)  =>  a in [2^(e-1), 2^e) */
    (void)frexp(a, &e);
    int lsb = (e - 1) - 7;         /* exponent of the last kept bit */
    if (lsb < -133) lsb = -133;    /* subnormal range: fixed spacing */
    double q = ldexp(1.0, lsb);
    double r = nearbyint(a / q) * q;   /* both scalings by 2^lsb are exact; RNE */
    if (r >= ldexp(1.0, 128)) return sign | 0x7f80;
    float f = (float)r;            /* exact: r has at most 8 significant bits */
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    return sign | (uint16_t)(u >> 16);
}

void w2o_f64_to_bf16_array(const double* v, int64_t n, uint16_t* out)
{
    for (int64_t i = 0; i < n; ++i) out[i] = w2o_f64_to_bf16(v[i]);
}

/* ---- code -> value (reading: int2 q=c-2, ternary q=c-1) ---------------- */

static int zero_point(int codec) { return codec == 0 ? 2 : 1; }

/* Returns W2O_ERR_BAD_CODE if a code is out of range for the codec. */
int w2o_check_codes(const uint8_t* codes, int64_t K, int64_t N, int codec)
{
    if (codec != 0 && codec != 1) return W2O_ERR_ARG;
    uint8_t top = codec == 0 ? 3 : 2;
    for (int64_t i = 0; i < K * N; ++i)
        if (codes[i] > top) return W2O_ERR_BAD_CODE;
    return W2O_OK;
}

/* ---- activation quantisation (Sec. II-B, II-D) ------------------------- */

/* One scale per row.  X is row-major with row stride ldx (elements).
 * x_is_bf16 != 0: X holds bf16 bit patterns (uint16_t), widened exactly.
 * gs may be NULL; otherwise gs[m][g] = sum of xq over group g (int32). */
int w2o_quantize_rows(const void* X, int x_is_bf16, int64_t M, int64_t K, int64_t ldx,
                      int G, int8_t* xq, float* sx, int32_t* gs)
{
    if (M < 0 || K <= 0 || ldx < K || G <= 0 || K % G) return W2O_ERR_ARG;
    for (int64_t m = 0; m < M; ++m) {
        float amax = 0.0f;
        for (int64_t k = 0; k < K; ++k) {
            float x = x_is_bf16 ? w2o_bf16_to_f32(((const uint16_t*)X)[m * ldx + k])
                                : ((const float*)X)[m * ldx + k];
            float ax = fabsf(x);
            if (ax > amax) amax = ax;
        }
        float inv = 0.0f, s = 0.0f;
        if (amax > 0.0f) {
            inv = 127.0f / amax;       /* correctly rounded binary32 divide */
            s = amax / 127.0f;
        }
        sx[m] = s;
        for (int64_t k = 0; k < K; ++k) {
            float x = x_is_bf16 ? w2o_bf16_to_f32(((const uint16_t*)X)[m * ldx + k])
                                : ((const float*)X)[m * ldx + k];
            float t = x * inv;         /* one rounded binary32 multiply */
            float r = nearbyintf(t);   /* round half to even (default mode) */
            if (r > 127.0f) r = 127.0f;
            if (r < -127.0f) r = -127.0f;
            xq[m * K + k] = (int8_t)r;
        }
        if (gs) {
            for (int64_t g = 0; g < K / G; ++g) {
                int32_t s32 = 0;
                for (int64_t k = g * G; k < (g + 1) * G; ++k) s32 += xq[m * K + k];
                gs[m * (K / G) + g] = s32;
            }
        }
    }
    return W2O_OK;
}

/* ---- exact integer group accumulators (Sec. II-C) ---------------------- */

/* acc[m][g][n] = sum_{k in group g} xq[m][k] * (codes[k][n] - z), int32.
 * codes: one code per byte, row-major [K][N].  acc: [M][K/G][N]. */
int w2o_group_acc(const uint8_t* codes, int64_t K, int64_t N, int G, int codec,
                  const int8_t* xq, int64_t M, int32_t* acc)
{
    if (K <= 0 || N <= 0 || G <= 0 || K % G || M < 0) return W2O_ERR_ARG;
    int rc = w2o_check_codes(codes, K, N, codec);
    if (rc) return rc;
    const int z = zero_point(codec);
    const int64_t Kg = K / G;
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        for (int64_t g = 0; g < Kg; ++g) {
            int32_t* a = acc + (m * Kg + g) * N;
            for (int64_t n = 0; n < N; ++n) a[n] = 0;
            for (int64_t k = g * G; k < (g + 1) * G; ++k) {
                const int32_t x = xq[m * K + k];
                const uint8_t* c = codes + k * N;
                for (int64_t n = 0; n < N; ++n) a[n] += x * ((int32_t)c[n] - z);
            }
        }
    }
    return W2O_OK;
}

/* ---- w2a8: int8 activations, fused dequant (Sec. II-D) ----------------- */

/* y64[m][n] = sx[m] * sum_g sw[g][n] * acc[m][g][n]  (fp64, g ascending),
 * Y = bf16(y64).  scales: bf16 bit patterns [K/G][N].  Y: [M][N] bf16 bits.
 * y64_out may be NULL; if not, receives the unrounded fp64 values. */
int w2o_matmul_a8(const uint8_t* codes, const uint16_t* scales, int64_t K, int64_t N, int G,
                  int codec, const int8_t* xq, const float* sx, int64_t M,
                  uint16_t* Y, double* y64_out)
{
    if (K <= 0 || N <= 0 || G <= 0 || K % G || M < 0) return W2O_ERR_ARG;
    const int64_t Kg = K / G;
    int32_t* acc = (int32_t*)malloc((size_t)(M > 0 ? M : 1) * Kg * N * sizeof(int32_t));
    if (!acc) return W2O_ERR_ARG;
    int rc = w2o_group_acc(codes, K, N, G, codec, xq, M, acc);
    if (rc) { free(acc); return rc; }
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        for (int64_t n = 0; n < N; ++n) {
            double s = 0.0;
            for (int64_t g = 0; g < Kg; ++g)
                s += (double)w2o_bf16_to_f32(scales[g * N + n]) * (double)acc[(m * Kg + g) * N + n];
            double y = (double)sx[m] * s;
            if (y64_out) y64_out[m * N + n] = y;
            Y[m * N + n] = w2o_f64_to_bf16(y);
        }
    }
    free(acc);
    return W2O_OK;
}

/* Cancellation floor used by the parity tolerance:
 * mag[m][n] = |sx[m]| * sum_g |sw[g][n] * acc[m][g][n]|  (fp64). */
int w2o_a8_term_magnitude(const uint8_t* codes, const uint16_t* scales, int64_t K, int64_t N,
                          int G, int codec, const int8_t* xq, const float* sx, int64_t M,
                          double* mag)
{
    if (K <= 0 || N <= 0 || G <= 0 || K % G || M < 0) return W2O_ERR_ARG;
    const int64_t Kg = K / G;
    int32_t* acc = (int32_t*)malloc((size_t)(M > 0 ? M : 1) * Kg * N * sizeof(int32_t));
    if (!acc) return W2O_ERR_ARG;
    int rc = w2o_group_acc(codes, K, N, G, codec, xq, M, acc);
    if (rc) { free(acc); return rc; }
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            double s = 0.0;
            for (int64_t g = 0; g < Kg; ++g)
                s += fabs((double)w2o_bf16_to_f32(scales[g * N + n]) * (double)acc[(m * Kg + g) * N + n]);
            mag[m * N + n] = fabs((double)sx[m]) * s;
        }
    free(acc);
    return W2O_OK;
}

/* ---- w2a16: unquantised bf16 activations (Sec. II-D, alternative kernel) */

/* y64[m][n] = sum_k x[m][k] * (sw[k/G][n] * q[k][n]), k ascending, fp64.
 * This is dequantise-then-matmul written out.  mag_out (may be NULL) gets
 * sum_k |x * w| for the tolerance floor. */
int w2o_matmul_a16(const uint8_t* codes, const uint16_t* scales, int64_t K, int64_t N, int G,
                   int codec, const uint16_t* X, int64_t ldx, int64_t M,
                   uint16_t* Y, double* y64_out, double* mag_out)
{
    if (K <= 0 || N <= 0 || G <= 0 || K % G || M < 0 || ldx < K) return W2O_ERR_ARG;
    int rc = w2o_check_codes(codes, K, N, codec);
    if (rc) return rc;
    const int z = zero_point(codec);
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        double* y = (double*)calloc((size_t)N * 2, sizeof(double));
        double* mg = y + N;
        for (int64_t k = 0; k < K; ++k) {
            const double x = (double)w2o_bf16_to_f32(X[m * ldx + k]);
            const uint8_t* c = codes + k * N;
            const uint16_t* s = scales + (k / G) * N;
            for (int64_t n = 0; n < N; ++n) {
                double w = (double)w2o_bf16_to_f32(s[n]) * (double)((int)c[n] - z);
                y[n] += x * w;
                mg[n] += fabs(x * w);
            }
        }
        for (int64_t n = 0; n < N; ++n) {
            if (y64_out) y64_out[m * N + n] = y[n];
            if (mag_out) mag_out[m * N + n] = mg[n];
            Y[m * N + n] = w2o_f64_to_bf16(y[n]);
        }
        free(y);
    }
    return W2O_OK;
}

/* ---- brute-force cross-check of the w2a8 path (tiny shapes) ------------ */

/* Dequantise BOTH operands to fp64, then a plain triple loop:
 *   xd[m][k] = sx[m]*xq[m][k],  wd[k][n] = sw[k/G][n]*q[k][n],
 *   y[m][n] = sum_k xd*wd (k ascending).  Differs from w2o_matmul_a8 only by
 * fp64 association. */
int w2o_bruteforce_a8(const uint8_t* codes, const uint16_t* scales, int64_t K, int64_t N, int G,
                      int codec, const int8_t* xq, const float* sx, int64_t M, double* y64)
{
    if (K <= 0 || N <= 0 || G <= 0 || K % G || M < 0) return W2O_ERR_ARG;
    int rc = w2o_check_codes(codes, K, N, codec);
    if (rc) return rc;
    const int z = zero_point(codec);
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            double s = 0.0;
            for (int64_t k = 0; k < K; ++k) {
                double xd = (double)sx[m] * (double)xq[m * K + k];
                double wd = (double)w2o_bf16_to_f32(scales[(k / G) * N + n]) *
                            (double)((int)codes[k * N + n] - z);
                s += xd * wd;
            }
            y64[m * N + n] = s;
        }
    return W2O_OK;
}

/* ---- fused epilogue (Sec. II-D: bias addition and post-GEMM activation
 * functions applied to the result before it is stored) --------------------- */

/* z[m][n] = y64[m][n] + bias[n] (bias: bf16 bit patterns [N], may be NULL).
 * act 0: out = z.  act 1: out = z * sigmoid(z) (SiLU), sigmoid(z) = 1/(1+e^-z).
 * act 2, the gated form: the columns come in blocks of 16 that alternate gate,
 * up, gate, up, ...; out has N/2 columns,
 *   out[m][16 b + l] = silu(z[m][32 b + l]) * z[m][32 b + 16 + l].
 * Reading (the paper names the operations, not their layout): bias is added in
 * the wide precision before the activation; one rounding to bf16 at the end.
 * Y: bf16 bits, out64: unrounded, both [M][N_out] dense, N_out = N or N/2. */
int w2o_epilogue(const double* y64, int64_t M, int64_t N, const uint16_t* bias, int act,
                 uint16_t* Y, double* out64)
{
    if (M < 0 || N <= 0 || act < 0 || act > 2) return W2O_ERR_ARG;
    if (act == 2 && N % 32) return W2O_ERR_ARG;
    const int64_t n_out = act == 2 ? N / 2 : N;
    for (int64_t m = 0; m < M; ++m)
        for (int64_t no = 0; no < n_out; ++no) {
            double r;
            if (act == 2) {
                const int64_t ng = (no / 16) * 32 + no % 16, nu = ng + 16;
                double g = y64[m * N + ng], u = y64[m * N + nu];
                if (bias) {
                    g += (double)w2o_bf16_to_f32(bias[ng]);
                    u += (double)w2o_bf16_to_f32(bias[nu]);
                }
                r = g * (1.0 / (1.0 + exp(-g))) * u;
            } else {
                double z = y64[m * N + no];
                if (bias) z += (double)w2o_bf16_to_f32(bias[no]);
                r = act == 1 ? z * (1.0 / (1.0 + exp(-z))) : z;
            }
            if (out64) out64[m * n_out + no] = r;
            if (Y) Y[m * n_out + no] = w2o_f64_to_bf16(r);
        }
    return W2O_OK;
}

/* Number of OpenMP threads the timed baseline will use. */
int w2o_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp single
        n = omp_get_num_threads();
    }
#endif
    return n;
}
