/*
 * CPU oracle for the grouped dense forward  Y_g = act(s_g * X_g W_g + b_g).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the plain definition of what the GPU
 * library computes, written so that it can be checked against the mathematics by
 * eye: a naive triple loop in fp64, the closed-form activations, and the number
 * formats' published definitions (bfloat16 = upper half of IEEE binary32; OCP
 * FP8 E4M3 "fn": bias 7, 3 mantissa bits, no infinities, max finite 448,
 * S.1111.111 = NaN).  It shares no code, table or constant with the GPU path and
 * nothing in the product may call it.
 *
 * What is grouped and why (the paper, Sec. 3.1 "Allocation operators"): a batch
 * is the set of requests of ONE service (BS), several services run on one GPU at
 * the same time (MT), and a request may contribute several rows (MF).  The paper
 * gives no layer arithmetic; the formula is the textbook affine layer followed
 * by an activation.
 *
 * Build:  gcc -O2 -fopenmp -shared -fPIC dense_oracle.c -o liboracle.so -lm
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* Activation ids of the ORACLE (its own numbering; the Python wrapper maps names). */
enum { OR_NONE = 0, OR_RELU = 1, OR_GELU_ERF = 2, OR_GELU_TANH = 3, OR_SILU = 4 };

/* Closed forms:
 *   ReLU(z)      = max(z, 0)
 *   SiLU(z)      = z / (1 + exp(-z))
 *   GELU_erf(z)  = z/2 * (1 + erf(z / sqrt 2))
 *   GELU_tanh(z) = z/2 * (1 + tanh( sqrt(2/pi) * (z + 0.044715 z^3) ))            */
double oracle_act(double z, int act)
{
    switch (act) {
    case OR_NONE:      return z;
    case OR_RELU:      return z > 0.0 ? z : 0.0;
    case OR_GELU_ERF:  return 0.5 * z * (1.0 + erf(z / sqrt(2.0)));
    case OR_GELU_TANH: return 0.5 * z * (1.0 + tanh(sqrt(2.0 / M_PI) * (z + 0.044715 * z * z * z)));
    case OR_SILU:      return z / (1.0 + exp(-z));
    default:           return NAN;
    }
}

int oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* One group:  Y[i,j] = act( s * sum_k X[i,k] W[k,j] + b[j] ).
 * X is [M,K] row-major, W is the LOGICAL weight [K,N] row-major, b has N entries
 * or is NULL (no bias), Y is [M,N] row-major.  Rows are independent, so the only
 * parallelism is one OpenMP thread per row; the sum over k runs in increasing k. */
void oracle_dense_forward(const double* X, const double* W, const double* b,
                          int64_t M, int64_t K, int64_t N, double s, int act, double* Y)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i) {
        double* y = Y + i * N;
        for (int64_t j = 0; j < N; ++j) y[j] = 0.0;
        for (int64_t k = 0; k < K; ++k) {
            const double x = X[i * K + k];
            const double* w = W + k * N;
            for (int64_t j = 0; j < N; ++j) y[j] += x * w[j];
        }
        for (int64_t j = 0; j < N; ++j) {
            double z = s * y[j] + (b ? b[j] : 0.0);
            y[j] = oracle_act(z, act);
        }
    }
}

/* SwiGLU hidden:  H = SiLU(sg * X Wg) (.) (su * X Wu), all [M,F]; no biases. */
void oracle_swiglu_hidden(const double* X, const double* Wg, const double* Wu,
                          int64_t M, int64_t K, int64_t F, double sg, double su, double* H)
{
#pragma omp parallel
    {
        double* u = (double*)malloc((size_t)(F > 0 ? F : 1) * sizeof(double));
#pragma omp for schedule(static)
        for (int64_t i = 0; i < M; ++i) {
            double* g = H + i * F;                    /* gate sums live in the output row */
            for (int64_t j = 0; j < F; ++j) { g[j] = 0.0; u[j] = 0.0; }
            for (int64_t k = 0; k < K; ++k) {
                const double x = X[i * K + k];
                const double* wg = Wg + k * F;
                const double* wu = Wu + k * F;
                for (int64_t j = 0; j < F; ++j) { g[j] += x * wg[j]; u[j] += x * wu[j]; }
            }
            for (int64_t j = 0; j < F; ++j) g[j] = oracle_act(sg * g[j], OR_SILU) * (su * u[j]);
        }
        free(u);
    }
}

/* ---- number formats ------------------------------------------------------ */

/* bfloat16 -> double: the 16 bits are the high half of a binary32. */
void oracle_bf16_decode(const uint16_t* src, int64_t n, double* dst)
{
    for (int64_t i = 0; i < n; ++i) {
        uint32_t u = (uint32_t)src[i] << 16;
        float f;
        memcpy(&f, &u, 4);
        dst[i] = (double)f;
    }
}

/* binary32 -> bfloat16, round to nearest, ties to even (NaN stays NaN). */
void oracle_bf16_encode(const float* src, int64_t n, uint16_t* dst)
{
    for (int64_t i = 0; i < n; ++i) {
        uint32_t u;
        memcpy(&u, &src[i], 4);
        if ((u & 0x7fffffffu) > 0x7f800000u) { dst[i] = (uint16_t)((u >> 16) | 0x0040u); continue; }
        uint32_t lower = u & 0xffffu, upper = u >> 16;
        if (lower > 0x8000u || (lower == 0x8000u && (upper & 1u))) upper += 1u;
        dst[i] = (uint16_t)upper;
    }
}

/* E4M3fn code -> value.  exponent field e (4 bits), mantissa m (3 bits):
 *   e == 0        : (-1)^s * 2^-6 * (m/8)          subnormal, smallest 2^-9
 *   e == 15, m==7 : NaN
 *   otherwise     : (-1)^s * 2^(e-7) * (1 + m/8)   largest 2^8 * 1.75 = 448      */
double oracle_e4m3_value(uint8_t code)
{
    int s = code >> 7, e = (code >> 3) & 15, m = code & 7;
    double v;
    if (e == 15 && m == 7) return NAN;
    if (e == 0) v = ldexp((double)m / 8.0, -6);
    else        v = ldexp(1.0 + (double)m / 8.0, e - 7);
    return s ? -v : v;
}

void oracle_e4m3_decode(const uint8_t* src, int64_t n, double scale, double* dst)
{
    for (int64_t i = 0; i < n; ++i) dst[i] = scale * oracle_e4m3_value(src[i]);
}

/* value -> E4M3fn code: q = sat(RNE(x / scale)), saturating at +-448. */
uint8_t oracle_e4m3_code(double x, double scale)
{
    double a = x / scale;
    if (isnan(a)) return 0x7f;
    uint8_t sign = signbit(a) ? 0x80 : 0x00;
    a = fabs(a);
    if (a >= 448.0) return sign | 0x7e;               /* saturate (covers +-inf) */
    int e;
    (void)frexp(a, &e);                               /* a = f * 2^e, f in [0.5,1) */
    int ex = e - 1;                                   /* floor(log2 a) */
    if (ex < -6) ex = -6;                             /* subnormal spacing 2^-9 */
    double quantum = ldexp(1.0, ex - 3);
    double q = nearbyint(a / quantum) * quantum;      /* default mode: ties to even */
    if (q > 448.0) q = 448.0;
    if (q == 0.0) return sign;
    double f = frexp(q, &e);                          /* q = f*2^e */
    ex = e - 1;
    if (ex < -6) {                                    /* subnormal: q = m/8 * 2^-6 */
        int m = (int)(q * 512.0);
        return sign | (uint8_t)m;
    }
    int m = (int)((f * 2.0 - 1.0) * 8.0);
    return sign | (uint8_t)(((ex + 7) << 3) | m);
}

void oracle_e4m3_encode(const double* src, int64_t n, double scale, uint8_t* dst)
{
    for (int64_t i = 0; i < n; ++i) dst[i] = oracle_e4m3_code(src[i], scale);
}

/* Elementwise activation over an array (used to pin the closed forms). */
void oracle_act_array(const double* z, int64_t n, int act, double* out)
{
    for (int64_t i = 0; i < n; ++i) out[i] = oracle_act(z[i], act);
}
