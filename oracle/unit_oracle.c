/*
 * CPU oracle for mixed-precision conv2d / matmul (int8 x int8 -> int32 and
 * fp16 x fp16 -> fp32) and the int8 inference glue around them.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is the plain definition
 * written out as direct loops: no blocking, no packing, no intrinsics, no code
 * shared with the GPU library.  Only the tests, the smoke check and the
 * benchmark's cpu_baseline leg may call it.
 *
 * What is computed follows the paper's statement of the problem:
 *   - Matmul and Conv are series of multiply-accumulates: elementwise products
 *     of low-precision operands, accumulated "horizontally" into one
 *     higher-precision element (Section I; Section II-A).
 *   - conv index forms c[x,y,k] += a[x+r,y+s,rc] * b[r,s,k,rc] (Section III-C.2,
 *     the operand-generation example): cross-correlation, no kernel flip.
 *   - int8 products accumulate in int32 (Section III-A, the VNNI description:
 *     16 int32 lanes, each the sum of 4 byte products plus the addend);
 *     fp16 products accumulate in fp32 (Section III-A, the Tensor Core
 *     description: 16x16x16 matmul, fp16 in, fp32 accumulator).
 *
 * Readings where the paper is silent (all listed in the design notes):
 *   - zero padding, floor output size, dilation 1, groups 1;
 *   - both int8 operands signed;
 *   - fp32 accumulation order c -> r -> s (outer to inner), one rounding per add;
 *   - requantize: t = acc (+bias) (+residual) in int32; f = (float)t (IEEE
 *     round-to-nearest-even conversion); g = f * scale[k] (one fp32 multiply);
 *     i = round-half-to-even(g); ReLU; clamp to [-128,127].
 *
 * Pins (tests/test_oracle_*.py): brute force in pure Python on tiny shapes,
 * delta and identity kernels, the all-ones closed form, conv == im2col-matmul,
 * conv3d against a float64 library conv3d, a scatter-form brute force and its depth-1
 * reduction to conv2d,
 * float64 library conv/matmul on integer-valued tensors, the 16x4 VNNI lane
 * semantics, the 16x16x16 Tensor Core shape, Table I output sizes, the requant
 * tie/saturation table and an exhaustive 2^16 sweep against exact rational
 * rounding.  The chained network (unit_oracle has no function for it; the test
 * harness composes these functions) is pinned by composition only.
 *
 * The OpenMP pragmas only spread independent (n,k) / (m) iterations over
 * threads; each output element is still produced by one thread running the
 * plain loop, so results do not depend on the thread count.
 */
#include <stdint.h>
#include <stddef.h>
#include <string.h>
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void oracle_set_num_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* Output extent of one spatial dimension: floor((in + 2*pad - window)/stride) + 1. */
int oracle_out_dim(int in, int window, int stride, int pad)
{
    int span = in + 2 * pad - window;
    if (span < 0 || stride <= 0) return 0;
    return span / stride + 1;
}

/* IEEE binary16 bit pattern -> float, exact (every binary16 value is a float). */
float oracle_half_to_float(uint16_t h)
{
    uint32_t sign = (uint32_t)(h >> 15) & 1u;
    int      expo = (int)((h >> 10) & 0x1f);
    uint32_t frac = (uint32_t)h & 0x3ffu;
    float mag;
    if (expo == 0) {
        mag = ldexpf((float)frac, -24);               /* zero or subnormal: frac * 2^-24 */
    } else if (expo == 31) {
        mag = frac ? NAN : INFINITY;
    } else {
        mag = ldexpf((float)(frac | 0x400u), expo - 25); /* (1024+frac) * 2^(e-15-10) */
    }
    return sign ? -mag : mag;
}

/* ------------------------------------------------------------------ conv2d */

/*
 * y[n,k,p,q] = sum_{c,r,s} X(n,c,p*sh + r - ph, q*sw + s - pw) * w[k,c,r,s]
 * with X = 0 outside the image.  x: NCHW int8, w: KCRS int8, y: NKPQ int32.
 * Each factor is widened to int32 before the multiply.
 */
void oracle_conv2d_i8(int N, int C, int H, int W, int K, int R, int S,
                      int sh, int sw, int ph, int pw,
                      const int8_t *x, const int8_t *w, int32_t *y)
{
    const int P = oracle_out_dim(H, R, sh, ph);
    const int Q = oracle_out_dim(W, S, sw, pw);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int k = 0; k < K; ++k)
            for (int p = 0; p < P; ++p)
                for (int q = 0; q < Q; ++q) {
                    int32_t acc = 0;
                    for (int c = 0; c < C; ++c)
                        for (int r = 0; r < R; ++r)
                            for (int s = 0; s < S; ++s) {
                                int h  = p * sh + r - ph;
                                int ww = q * sw + s - pw;
                                if (h < 0 || h >= H || ww < 0 || ww >= W) continue;
                                int32_t a = (int32_t)x[(((size_t)n * C + c) * H + h) * W + ww];
                                int32_t b = (int32_t)w[(((size_t)k * C + c) * R + r) * S + s];
                                acc += a * b;
                            }
                    y[(((size_t)n * K + k) * P + p) * Q + q] = acc;
                }
}

/*
 * Same definition on binary16 bit patterns, fp32 accumulator.  The product of
 * two binary16 values is exact in fp32 (22 significant bits, exponent in range),
 * so each step is one rounding: acc = fl32(acc + a*b), in c -> r -> s order.
 */
void oracle_conv2d_f16(int N, int C, int H, int W, int K, int R, int S,
                       int sh, int sw, int ph, int pw,
                       const uint16_t *x, const uint16_t *w, float *y)
{
    const int P = oracle_out_dim(H, R, sh, ph);
    const int Q = oracle_out_dim(W, S, sw, pw);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int k = 0; k < K; ++k)
            for (int p = 0; p < P; ++p)
                for (int q = 0; q < Q; ++q) {
                    float acc = 0.0f;
                    for (int c = 0; c < C; ++c)
                        for (int r = 0; r < R; ++r)
                            for (int s = 0; s < S; ++s) {
                                int h  = p * sh + r - ph;
                                int ww = q * sw + s - pw;
                                if (h < 0 || h >= H || ww < 0 || ww >= W) continue;
                                float a = oracle_half_to_float(x[(((size_t)n * C + c) * H + h) * W + ww]);
                                float b = oracle_half_to_float(w[(((size_t)k * C + c) * R + r) * S + s]);
                                float prod = a * b;
                                acc = acc + prod;
                            }
                    y[(((size_t)n * K + k) * P + p) * Q + q] = acc;
                }
}

/*
 * The same sum accumulated in fp64 (products are exact there too), plus the
 * sum of |a*b| per output: "truth" and the scale of the a-priori error bound
 * gamma_K * sum|a||b| that any fp32 summation order must satisfy.
 */
void oracle_conv2d_f16_f64(int N, int C, int H, int W, int K, int R, int S,
                           int sh, int sw, int ph, int pw,
                           const uint16_t *x, const uint16_t *w,
                           double *y, double *yabs)
{
    const int P = oracle_out_dim(H, R, sh, ph);
    const int Q = oracle_out_dim(W, S, sw, pw);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int k = 0; k < K; ++k)
            for (int p = 0; p < P; ++p)
                for (int q = 0; q < Q; ++q) {
                    double acc = 0.0, aacc = 0.0;
                    for (int c = 0; c < C; ++c)
                        for (int r = 0; r < R; ++r)
                            for (int s = 0; s < S; ++s) {
                                int h  = p * sh + r - ph;
                                int ww = q * sw + s - pw;
                                if (h < 0 || h >= H || ww < 0 || ww >= W) continue;
                                double a = (double)oracle_half_to_float(x[(((size_t)n * C + c) * H + h) * W + ww]);
                                double b = (double)oracle_half_to_float(w[(((size_t)k * C + c) * R + r) * S + s]);
                                acc  += a * b;
                                aacc += fabs(a * b);
                            }
                    size_t o = (((size_t)n * K + k) * P + p) * Q + q;
                    y[o] = acc;
                    if (yabs) yabs[o] = aacc;
                }
}

/* ------------------------------------------------------------------ conv3d */

/*
 * The paper's extensibility experiment (Section VI-C, "3D Convolution") feeds the same
 * pipeline a conv3d: the 2-D definition with one more spatial axis.
 * x: [N,C,D,H,W], w: [K,C,T,R,S], y: [N,K,O,P,Q];  zero padding, no dilation.
 * stride = {sd,sh,sw}, pad = {pd,ph,pw}.
 */
void oracle_conv3d_i8(int N, int C, int D, int H, int W, int K, int T, int R, int S,
                      const int *stride, const int *pad,
                      const int8_t *x, const int8_t *w, int32_t *y)
{
    const int O = oracle_out_dim(D, T, stride[0], pad[0]);
    const int P = oracle_out_dim(H, R, stride[1], pad[1]);
    const int Q = oracle_out_dim(W, S, stride[2], pad[2]);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int k = 0; k < K; ++k)
            for (int o = 0; o < O; ++o)
                for (int p = 0; p < P; ++p)
                    for (int q = 0; q < Q; ++q) {
                        int32_t acc = 0;
                        for (int c = 0; c < C; ++c)
                            for (int t = 0; t < T; ++t)
                                for (int r = 0; r < R; ++r)
                                    for (int s = 0; s < S; ++s) {
                                        int d  = o * stride[0] + t - pad[0];
                                        int h  = p * stride[1] + r - pad[1];
                                        int ww = q * stride[2] + s - pad[2];
                                        if (d < 0 || d >= D || h < 0 || h >= H || ww < 0 || ww >= W) continue;
                                        int32_t a = (int32_t)x[((((size_t)n * C + c) * D + d) * H + h) * W + ww];
                                        int32_t b = (int32_t)w[((((size_t)k * C + c) * T + t) * R + r) * S + s];
                                        acc += a * b;
                                    }
                        y[((((size_t)n * K + k) * O + o) * P + p) * Q + q] = acc;
                    }
}

/* fp16 inputs, fp32 accumulation in c -> t -> r -> s order; y64/yabs (optional) receive the
 * fp64-accumulated value and the sum of |products|. */
void oracle_conv3d_f16(int N, int C, int D, int H, int W, int K, int T, int R, int S,
                       const int *stride, const int *pad,
                       const uint16_t *x, const uint16_t *w, float *y, double *y64, double *yabs)
{
    const int O = oracle_out_dim(D, T, stride[0], pad[0]);
    const int P = oracle_out_dim(H, R, stride[1], pad[1]);
    const int Q = oracle_out_dim(W, S, stride[2], pad[2]);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int k = 0; k < K; ++k)
            for (int o = 0; o < O; ++o)
                for (int p = 0; p < P; ++p)
                    for (int q = 0; q < Q; ++q) {
                        float acc = 0.0f;
                        double acc64 = 0.0, aabs = 0.0;
                        for (int c = 0; c < C; ++c)
                            for (int t = 0; t < T; ++t)
                                for (int r = 0; r < R; ++r)
                                    for (int s = 0; s < S; ++s) {
                                        int d  = o * stride[0] + t - pad[0];
                                        int h  = p * stride[1] + r - pad[1];
                                        int ww = q * stride[2] + s - pad[2];
                                        if (d < 0 || d >= D || h < 0 || h >= H || ww < 0 || ww >= W) continue;
                                        float a = oracle_half_to_float(x[((((size_t)n * C + c) * D + d) * H + h) * W + ww]);
                                        float b = oracle_half_to_float(w[((((size_t)k * C + c) * T + t) * R + r) * S + s]);
                                        float prod = a * b;
                                        acc = acc + prod;
                                        acc64 += (double)a * (double)b;
                                        aabs += fabs((double)a * (double)b);
                                    }
                        size_t idx = ((((size_t)n * K + k) * O + o) * P + p) * Q + q;
                        y[idx] = acc;
                        if (y64) y64[idx] = acc64;
                        if (yabs) yabs[idx] = aabs;
                    }
}

/* ------------------------------------------------------------------ matmul */

/*
 * C[m,n] = sum_k A[m,k] * B[k,n];  A row-major (A[m,k] at A[m*lda + k]),
 * B column-major (B[k,n] at B[n*ldb + k]),  C row-major (C[m*ldc + n]).
 */
void oracle_matmul_i8(int M, int N, int K,
                      const int8_t *A, long lda, const int8_t *B, long ldb,
                      int32_t *C, long ldc)
{
#pragma omp parallel for schedule(static)
    for (int m = 0; m < M; ++m)
        for (int n = 0; n < N; ++n) {
            int32_t acc = 0;
            for (int k = 0; k < K; ++k)
                acc += (int32_t)A[(size_t)m * lda + k] * (int32_t)B[(size_t)n * ldb + k];
            C[(size_t)m * ldc + n] = acc;
        }
}

void oracle_matmul_f16(int M, int N, int K,
                       const uint16_t *A, long lda, const uint16_t *B, long ldb,
                       float *C, long ldc)
{
#pragma omp parallel for schedule(static)
    for (int m = 0; m < M; ++m)
        for (int n = 0; n < N; ++n) {
            float acc = 0.0f;
            for (int k = 0; k < K; ++k) {
                float prod = oracle_half_to_float(A[(size_t)m * lda + k]) *
                             oracle_half_to_float(B[(size_t)n * ldb + k]);
                acc = acc + prod;
            }
            C[(size_t)m * ldc + n] = acc;
        }
}

void oracle_matmul_f16_f64(int M, int N, int K,
                           const uint16_t *A, long lda, const uint16_t *B, long ldb,
                           double *C, double *Cabs, long ldc)
{
#pragma omp parallel for schedule(static)
    for (int m = 0; m < M; ++m)
        for (int n = 0; n < N; ++n) {
            double acc = 0.0, aacc = 0.0;
            for (int k = 0; k < K; ++k) {
                double prod = (double)oracle_half_to_float(A[(size_t)m * lda + k]) *
                              (double)oracle_half_to_float(B[(size_t)n * ldb + k]);
                acc += prod;
                aacc += fabs(prod);
            }
            C[(size_t)m * ldc + n] = acc;
            if (Cabs) Cabs[(size_t)m * ldc + n] = aacc;
        }
}

/* ---------------------------------------------------------------- requantize */

/* One element: int32 -> int8 under the fixed rounding rule (default FP
 * environment: round-to-nearest-even for both the conversion and nearbyintf). */
int8_t oracle_requant_one(int32_t t, float scale, int relu)
{
    float f = (float)t;
    volatile float g = f * scale;          /* volatile: force one fp32 rounding */
    float i = nearbyintf(g);
    if (relu && i < 0.0f) i = 0.0f;
    if (i < -128.0f) i = -128.0f;
    if (i > 127.0f)  i = 127.0f;
    return (int8_t)i;
}

/*
 * acc, residual: [N,K,PQ] int32;  bias, scale: [K];  out: [N,K,PQ] int8.
 * bias and residual may be NULL.  The caller keeps |acc + bias + residual| < 2^31.
 */
void oracle_requant(int N, int K, int PQ,
                    const int32_t *acc, const int32_t *bias, const int32_t *residual,
                    const float *scale, int relu, int8_t *out)
{
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int k = 0; k < K; ++k)
            for (int i = 0; i < PQ; ++i) {
                size_t o = ((size_t)n * K + k) * PQ + i;
                int32_t t = acc[o];
                if (bias) t += bias[k];
                if (residual) t += residual[o];
                out[o] = oracle_requant_one(t, scale[k], relu);
            }
}

/* ------------------------------------------------------------ pooling glue */

/* int8 max over a window; padded positions are ignored (never win). NCHW. */
void oracle_maxpool_i8(int N, int C, int H, int W, int R, int S,
                       int sh, int sw, int ph, int pw,
                       const int8_t *x, int8_t *y)
{
    const int P = oracle_out_dim(H, R, sh, ph);
    const int Q = oracle_out_dim(W, S, sw, pw);
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c)
            for (int p = 0; p < P; ++p)
                for (int q = 0; q < Q; ++q) {
                    int best = -128;
                    for (int r = 0; r < R; ++r)
                        for (int s = 0; s < S; ++s) {
                            int h  = p * sh + r - ph;
                            int ww = q * sw + s - pw;
                            if (h < 0 || h >= H || ww < 0 || ww >= W) continue;
                            int v = x[(((size_t)n * C + c) * H + h) * W + ww];
                            if (v > best) best = v;
                        }
                    y[(((size_t)n * C + c) * P + p) * Q + q] = (int8_t)best;
                }
}

/* Global average pool as an integer sum over H*W followed by the requant rule
 * with a per-channel scale (the 1/(H*W) factor is folded into scale by the caller). */
void oracle_global_sumpool_requant_i8(int N, int C, int HW,
                                      const int8_t *x, const float *scale, int8_t *y)
{
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c) {
            int32_t sum = 0;
            for (int i = 0; i < HW; ++i) sum += (int32_t)x[((size_t)n * C + c) * HW + i];
            y[(size_t)n * C + c] = oracle_requant_one(sum, scale[c], 0);
        }
}

/* Widen int8 to int32 and multiply by an integer (identity-shortcut residual). */
void oracle_widen_scale_i8(size_t count, const int8_t *x, int32_t mult, int32_t *y)
{
    for (size_t i = 0; i < count; ++i) y[i] = (int32_t)x[i] * mult;
}

/* ------------------------------------------------- other operand types */

/*
 * The paper presents its method as open to further operand types (Section I;
 * Section III-A describes an unsigned-byte x signed-byte instruction).  Two more
 * pairs, same definitions as above with only the element decoding changed:
 *   u8 x i8 -> i32   (the x86 instruction's operand types: activations unsigned)
 *   bf16 x bf16 -> f32
 */

/* bfloat16 bit pattern -> float: the pattern is the upper half of the binary32 word. */
float oracle_bf16_to_float(uint16_t b)
{
    uint32_t word = (uint32_t)b << 16;
    float f;
    memcpy(&f, &word, sizeof f);
    return f;
}

void oracle_conv2d_u8i8(int N, int C, int H, int W, int K, int R, int S,
                        int sh, int sw, int ph, int pw,
                        const uint8_t *x, const int8_t *w, int32_t *y)
{
    const int P = oracle_out_dim(H, R, sh, ph);
    const int Q = oracle_out_dim(W, S, sw, pw);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int k = 0; k < K; ++k)
            for (int p = 0; p < P; ++p)
                for (int q = 0; q < Q; ++q) {
                    int32_t acc = 0;
                    for (int c = 0; c < C; ++c)
                        for (int r = 0; r < R; ++r)
                            for (int s = 0; s < S; ++s) {
                                int h  = p * sh + r - ph;
                                int ww = q * sw + s - pw;
                                if (h < 0 || h >= H || ww < 0 || ww >= W) continue;
                                int32_t a = (int32_t)x[(((size_t)n * C + c) * H + h) * W + ww];
                                int32_t b = (int32_t)w[(((size_t)k * C + c) * R + r) * S + s];
                                acc += a * b;
                            }
                    y[(((size_t)n * K + k) * P + p) * Q + q] = acc;
                }
}

void oracle_matmul_u8i8(int M, int N, int K,
                        const uint8_t *A, long lda, const int8_t *B, long ldb,
                        int32_t *C, long ldc)
{
#pragma omp parallel for schedule(static)
    for (int m = 0; m < M; ++m)
        for (int n = 0; n < N; ++n) {
            int32_t acc = 0;
            for (int k = 0; k < K; ++k)
                acc += (int32_t)A[(size_t)m * lda + k] * (int32_t)B[(size_t)n * ldb + k];
            C[(size_t)m * ldc + n] = acc;
        }
}

/* bf16: products of two 8-bit significands are exact in fp32 while the exponents stay in
 * range; y = sequential fp32 sum in c -> r -> s order, y64 / yabs as for binary16. */
void oracle_conv2d_bf16(int N, int C, int H, int W, int K, int R, int S,
                        int sh, int sw, int ph, int pw,
                        const uint16_t *x, const uint16_t *w,
                        float *y, double *y64, double *yabs)
{
    const int P = oracle_out_dim(H, R, sh, ph);
    const int Q = oracle_out_dim(W, S, sw, pw);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int k = 0; k < K; ++k)
            for (int p = 0; p < P; ++p)
                for (int q = 0; q < Q; ++q) {
                    float acc = 0.0f;
                    double acc64 = 0.0, aacc = 0.0;
                    for (int c = 0; c < C; ++c)
                        for (int r = 0; r < R; ++r)
                            for (int s = 0; s < S; ++s) {
                                int h  = p * sh + r - ph;
                                int ww = q * sw + s - pw;
                                if (h < 0 || h >= H || ww < 0 || ww >= W) continue;
                                float a = oracle_bf16_to_float(x[(((size_t)n * C + c) * H + h) * W + ww]);
                                float b = oracle_bf16_to_float(w[(((size_t)k * C + c) * R + r) * S + s]);
                                float prod = a * b;
                                acc = acc + prod;
                                acc64 += (double)a * (double)b;
                                aacc  += fabs((double)a * (double)b);
                            }
                    size_t o = (((size_t)n * K + k) * P + p) * Q + q;
                    y[o] = acc;
                    if (y64)  y64[o]  = acc64;
                    if (yabs) yabs[o] = aacc;
                }
}

void oracle_matmul_bf16(int M, int N, int K,
                        const uint16_t *A, long lda, const uint16_t *B, long ldb,
                        float *C, double *C64, double *Cabs, long ldc)
{
#pragma omp parallel for schedule(static)
    for (int m = 0; m < M; ++m)
        for (int n = 0; n < N; ++n) {
            float acc = 0.0f;
            double acc64 = 0.0, aacc = 0.0;
            for (int k = 0; k < K; ++k) {
                float a = oracle_bf16_to_float(A[(size_t)m * lda + k]);
                float b = oracle_bf16_to_float(B[(size_t)n * ldb + k]);
                float prod = a * b;
                acc = acc + prod;
                acc64 += (double)a * (double)b;
                aacc  += fabs((double)a * (double)b);
            }
            C[(size_t)m * ldc + n] = acc;
            if (C64)  C64[(size_t)m * ldc + n]  = acc64;
            if (Cabs) Cabs[(size_t)m * ldc + n] = aacc;
        }
}

/*
 * fp8 (OCP E4M3, the finite-only "fn" variant: 1 sign, 4 exponent bits with bias 7,
 * 3 fraction bits; no infinities; the single NaN pattern per sign is S.1111.111; largest
 * finite value 448; subnormals are multiples of 2^-9).  Every value is exact in fp32 and so
 * is every product of two of them.
 */
float oracle_fp8_e4m3_to_float(uint8_t b)
{
    int sign = (b >> 7) & 1;
    int expo = (b >> 3) & 0xf;
    int frac = b & 0x7;
    float mag;
    if (expo == 0xf && frac == 0x7) {
        mag = NAN;
    } else if (expo == 0) {
        mag = ldexpf((float)frac, -9);                 /* 0 or subnormal: frac/8 * 2^-6 */
    } else {
        mag = ldexpf((float)(8 + frac), expo - 10);    /* (1 + frac/8) * 2^(expo-7) */
    }
    return sign ? -mag : mag;
}

void oracle_conv2d_fp8(int N, int C, int H, int W, int K, int R, int S,
                       int sh, int sw, int ph, int pw,
                       const uint8_t *x, const uint8_t *w,
                       float *y, double *y64, double *yabs)
{
    const int P = oracle_out_dim(H, R, sh, ph);
    const int Q = oracle_out_dim(W, S, sw, pw);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int k = 0; k < K; ++k)
            for (int p = 0; p < P; ++p)
                for (int q = 0; q < Q; ++q) {
                    float acc = 0.0f;
                    double acc64 = 0.0, aacc = 0.0;
                    for (int c = 0; c < C; ++c)
                        for (int r = 0; r < R; ++r)
                            for (int s = 0; s < S; ++s) {
                                int h  = p * sh + r - ph;
                                int ww = q * sw + s - pw;
                                if (h < 0 || h >= H || ww < 0 || ww >= W) continue;
                                float a = oracle_fp8_e4m3_to_float(x[(((size_t)n * C + c) * H + h) * W + ww]);
                                float b = oracle_fp8_e4m3_to_float(w[(((size_t)k * C + c) * R + r) * S + s]);
                                float prod = a * b;
                                acc = acc + prod;
                                acc64 += (double)a * (double)b;
                                aacc  += fabs((double)a * (double)b);
                            }
                    size_t o = (((size_t)n * K + k) * P + p) * Q + q;
                    y[o] = acc;
                    if (y64)  y64[o]  = acc64;
                    if (yabs) yabs[o] = aacc;
                }
}

void oracle_matmul_fp8(int M, int N, int K,
                       const uint8_t *A, long lda, const uint8_t *B, long ldb,
                       float *C, double *C64, double *Cabs, long ldc)
{
#pragma omp parallel for schedule(static)
    for (int m = 0; m < M; ++m)
        for (int n = 0; n < N; ++n) {
            float acc = 0.0f;
            double acc64 = 0.0, aacc = 0.0;
            for (int k = 0; k < K; ++k) {
                float a = oracle_fp8_e4m3_to_float(A[(size_t)m * lda + k]);
                float b = oracle_fp8_e4m3_to_float(B[(size_t)n * ldb + k]);
                float prod = a * b;
                acc = acc + prod;
                acc64 += (double)a * (double)b;
                aacc  += fabs((double)a * (double)b);
            }
            C[(size_t)m * ldc + n] = acc;
            if (C64)  C64[(size_t)m * ldc + n]  = acc64;
            if (Cabs) Cabs[(size_t)m * ldc + n] = aacc;
        }
}
