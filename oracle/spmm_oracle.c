/*
 * CPU oracle for the structured-sparse INT8 SpMM with fused epilogue.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the checker the HIP library is
 * compared against; it is never linked into, imported by or called from the
 * product path, and it shares no code, header, table or helper with it.
 *
 * The method of the paper (Section 3.2, Algorithm 1) reaches *exactly* the
 * dense product of the weight matrix and the activations: pruning in 4x1
 * blocks and the compressed storage only decide which multiply-adds are
 * skipped because a factor is zero.  The oracle is therefore the textbook
 * definition written out on the dense-with-zeros weight matrix, followed by
 * the post-operator chain (Section 3.3, Figure 3: BiasAdd, GeLU, Quantize)
 * in a fully specified order of IEEE-754 binary32 operations, and the lookup
 * table of Algorithm 2 for the low-precision GELU->int8 chain.
 *
 * Axis names:  W int8 [N][K] (ldw),  X uint8 [K][M] (ldx),  out [N][M] (ldo).
 *
 * Arithmetic (everything the paper leaves open is a stated reading):
 *   acc[n][m] = sum_k  W[n][k] * (X[k][m] - x_zp)          int32, u8 x s8 -> s32
 *   s[n]      = w_scale[n] * x_scale                        one binary32 multiply
 *   y         = fmaf((float)acc, s[n], bias ? bias[n] : 0)  one fused binary32 op
 *   GELU, f32 out :  z = (float)(0.5 * y * erfc(-y / sqrt(2)))   evaluated in double
 *   GELU, int8 out:  t = sat_s8(rintf(y * (1.0f / mid_scale)));  q = lut[t + 128]
 *   TABLE, int8 out: the same look-up with a caller's table of any element-wise chain (Algorithm 2
 *                    is stated for a post-operator chain in general; GELU is the instance above)
 *   no post-op    :  z = y
 *   Sum (optional):  z = z + R[n][m]       one binary32 add of a second [N][M] tensor
 *                    (Figure 3 names Sum among the fused post-operators without a formula;
 *                    reading: the residual is added after BiasAdd / GeLU and before Quantize.
 *                    Not combined with the table chain, whose value is a function of one key.)
 *   Quantize      :  q = (int) min(hi, max(lo, rintf(z * (1.0f / out_scale)) + (float)out_zp))
 * rintf / rint round half to even (default rounding mode).
 *
 * Build:  gcc -O2 -fopenmp -ffp-contract=off -fno-fast-math -shared -fPIC
 */
#include <math.h>
#include <stdint.h>
#include <stddef.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_OUT_S32 = 0, ORACLE_OUT_F32 = 1, ORACLE_OUT_S8 = 2, ORACLE_OUT_U8 = 3 };
enum { ORACLE_POST_NONE = 0, ORACLE_POST_GELU = 1, ORACLE_POST_TABLE = 2 };

/* Exact (erf-based) GELU in double: x * Phi(x), Phi written with erfc so the
 * negative tail keeps its relative accuracy. */
double oracle_gelu(double x)
{
    return 0.5 * x * erfc(-x / sqrt(2.0));
}

/* acc = W * (X - x_zp): Section 3.2 (unsigned 8-bit times signed 8-bit, summed into 32-bit integers).
 * Plain triple loop n, k, m over the dense-with-zeros W.  acc is [N][M], ld = M. */
void oracle_acc_s32(const int8_t *W, int64_t ldw, const uint8_t *X, int64_t ldx,
                    int64_t N, int64_t K, int64_t M, int32_t x_zp, int32_t *acc)
{
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        int32_t *row = acc + n * M;
        for (int64_t m = 0; m < M; ++m)
            row[m] = 0;
        for (int64_t k = 0; k < K; ++k) {
            const int32_t w = (int32_t)W[n * ldw + k];
            const uint8_t *x = X + k * ldx;
            for (int64_t m = 0; m < M; ++m)
                row[m] += w * ((int32_t)x[m] - x_zp);
        }
    }
}

static inline float sat_round(float v, float lo, float hi)
{
    return fminf(hi, fmaxf(lo, v));
}

/* Algorithm 2: table over every int8 key of the chain
 * dequantise(mid_scale) -> GELU -> quantise(out_scale, out_zp), rounded half to even.
 * lut[i + 128] is the output code for key i in [-128, 127]; for a U8 output the
 * stored byte is the uint8 code. Returns 0, or -1 for a bad out_type. */
int oracle_gelu_lut(float mid_scale, float out_scale, int32_t out_zp, int out_type, int8_t *lut)
{
    double lo, hi;
    if (out_type == ORACLE_OUT_S8) { lo = -128.0; hi = 127.0; }
    else if (out_type == ORACLE_OUT_U8) { lo = 0.0; hi = 255.0; }
    else return -1;
    for (int i = -128; i <= 127; ++i) {
        double v = oracle_gelu((double)i * (double)mid_scale);
        double q = rint(v / (double)out_scale) + (double)out_zp;
        if (q < lo) q = lo;
        if (q > hi) q = hi;
        int iq = (int)q;
        lut[i + 128] = (int8_t)(uint8_t)(iq & 0xff);
    }
    return 0;
}

/* Post-operator chain on an int32 accumulator matrix acc [N][M] (ld = M).
 * out is [N][ldo] of the element type selected by out_type.
 * sum: optional second operand of the Sum post-operator, [N][ld_sum] binary32, or NULL.
 * Returns 0, or -1 for an invalid combination. */
int oracle_epilogue_sum(const int32_t *acc, int64_t N, int64_t M,
                        const float *w_scale, float x_scale, const float *bias,
                        int postop, const float *sum, int64_t ld_sum,
                        int out_type, float out_scale, int32_t out_zp,
                        float mid_scale, const int8_t *lut, void *out, int64_t ldo)
{
    if (out_type < ORACLE_OUT_S32 || out_type > ORACLE_OUT_U8) return -1;
    if (postop != ORACLE_POST_NONE && postop != ORACLE_POST_GELU && postop != ORACLE_POST_TABLE) return -1;
    const int quant = (out_type == ORACLE_OUT_S8 || out_type == ORACLE_OUT_U8);
    if (out_type != ORACLE_OUT_S32 && !w_scale) return -1;
    if (postop == ORACLE_POST_TABLE && !quant) return -1;
    const int table = quant && (postop == ORACLE_POST_GELU || postop == ORACLE_POST_TABLE);
    if (table && !lut) return -1;
    if (sum && (out_type == ORACLE_OUT_S32 || table)) return -1;

    const float lo = (out_type == ORACLE_OUT_U8) ? 0.0f : -128.0f;
    const float hi = (out_type == ORACLE_OUT_U8) ? 255.0f : 127.0f;
    const float inv_out = quant ? 1.0f / out_scale : 0.0f;
    const float inv_mid = table ? 1.0f / mid_scale : 0.0f;

#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        const float s = (out_type != ORACLE_OUT_S32) ? w_scale[n] * x_scale : 0.0f;
        const float b = bias ? bias[n] : 0.0f;
        for (int64_t m = 0; m < M; ++m) {
            const int32_t a = acc[n * M + m];
            if (out_type == ORACLE_OUT_S32) {
                ((int32_t *)out)[n * ldo + m] = a;
                continue;
            }
            const float y = fmaf((float)a, s, b);
            if (out_type == ORACLE_OUT_F32) {
                float z = y;
                if (postop == ORACLE_POST_GELU)
                    z = (float)oracle_gelu((double)y);
                if (sum)
                    z = z + sum[n * ld_sum + m];
                ((float *)out)[n * ldo + m] = z;
                continue;
            }
            int q;
            if (table) {
                const int t = (int)sat_round(rintf(y * inv_mid), -128.0f, 127.0f);
                q = (out_type == ORACLE_OUT_U8) ? (int)(uint8_t)lut[t + 128] : (int)lut[t + 128];
            } else {
                float z = y;
                if (sum)
                    z = z + sum[n * ld_sum + m];
                q = (int)sat_round(rintf(z * inv_out) + (float)out_zp, lo, hi);
            }
            if (out_type == ORACLE_OUT_S8)
                ((int8_t *)out)[n * ldo + m] = (int8_t)q;
            else
                ((uint8_t *)out)[n * ldo + m] = (uint8_t)q;
        }
    }
    return 0;
}

/* Threads an OpenMP parallel region of this library uses (reported beside timings). */
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
