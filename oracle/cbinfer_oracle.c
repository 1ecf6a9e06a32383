/*
 * CPU oracle for change-based convolution (CBinfer, arXiv 1704.04313).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference the HIP library is
 * compared against.  Nothing in the product path may call it; it shares no code, header,
 * table or helper with the HIP sources.  Only tests, the smoke check and the benchmark's
 * cpu_baseline leg load it.
 *
 * Conventions (all from Section 3 of the paper):
 *   - maps are planar  x[c][y][x]  (the X-matrix construction indexes x(k, j+y_o, i+x_o));
 *   - weights are  w[o][c][j][i], the row order of the filter matrix K;
 *   - the convolution is the cross-correlation that the X/K matrix construction spells out
 *     (eq. (1) is printed with mirrored offsets; the matrix form is what is multiplied),
 *     with zero padding applied while reading x and stride applied by skipping outputs;
 *   - every output value is accumulated in double in the order c, j, i starting from the
 *     bias, and rounded to float once (optionally then to bfloat16, round-to-nearest-even);
 *   - positions are linear indices  y*W + x.
 *
 * OpenMP only distributes independent output pixels over threads; it changes no result.
 */
#include <math.h>
#include <stdint.h>
#include <string.h>

static float round_to_bf16(float v)
{
    uint32_t u;
    memcpy(&u, &v, 4);
    if ((u & 0x7fffffffu) > 0x7f800000u) {          /* NaN stays NaN */
        u |= 0x00400000u;
        u &= 0xffff0000u;
    } else {
        uint32_t lsb = (u >> 16) & 1u;
        u += 0x7fffu + lsb;
        u &= 0xffff0000u;
    }
    memcpy(&v, &u, 4);
    return v;
}

/* One output value of the convolution layer, Section 3 eq. (1) in its matrix form
 * Y = K X:  b_o + sum over c, j, i of  w(o,c,j,i) * x(c, qy*s - p + j, qx*s - p + i). */
static float conv_value(const float *x, int C, int H, int W,
                        const float *w, const float *b, int kh, int kw, int s, int p,
                        int o, int qy, int qx, int relu, int bf16)
{
    double acc = b ? (double)b[o] : 0.0;
    for (int c = 0; c < C; ++c)
        for (int j = 0; j < kh; ++j) {
            int iy = qy * s - p + j;
            if (iy < 0 || iy >= H) continue;
            for (int i = 0; i < kw; ++i) {
                int ix = qx * s - p + i;
                if (ix < 0 || ix >= W) continue;
                acc += (double)w[(((int64_t)o * C + c) * kh + j) * kw + i] *
                       (double)x[((int64_t)c * H + iy) * W + ix];
            }
        }
    float r = (float)acc;
    if (bf16) r = round_to_bf16(r);
    if (relu && r < 0.0f) r = 0.0f;
    return r;
}

/* Dense per-frame convolution: every output position (the non-change-based layer). */
void orc_conv_dense(const float *x, int C, int H, int W, const float *w, const float *b,
                    int M, int kh, int kw, int s, int p, int relu, int bf16, float *y)
{
    int Ho = (H + 2 * p - kh) / s + 1, Wo = (W + 2 * p - kw) / s + 1;
#pragma omp parallel for collapse(2) schedule(static)
    for (int o = 0; o < M; ++o)
        for (int qy = 0; qy < Ho; ++qy)
            for (int qx = 0; qx < Wo; ++qx)
                y[((int64_t)o * Ho + qy) * Wo + qx] =
                    conv_value(x, C, H, W, w, b, kh, kw, s, p, o, qy, qx, relu, bf16);
}

/* Matrix multiplication restricted to the listed columns, followed by the output update
 * (Section 3.1, "Matrix Generation & Matrix Multiplication" and "Output Updating"):
 * for each listed output position all M channels are recomputed from the CURRENT input
 * and written over the stored value; every other position of y keeps what it held. */
void orc_conv_update(const float *x, int C, int H, int W, const float *w, const float *b,
                     int M, int kh, int kw, int s, int p, int relu, int bf16,
                     const int32_t *list, int64_t n, float *y)
{
    int Ho = (H + 2 * p - kh) / s + 1, Wo = (W + 2 * p - kw) / s + 1;
#pragma omp parallel for schedule(dynamic, 16)
    for (int64_t u = 0; u < n; ++u) {
        int q = list[u], qy = q / Wo, qx = q % Wo;
        for (int o = 0; o < M; ++o)
            y[((int64_t)o * Ho + qy) * Wo + qx] =
                conv_value(x, C, H, W, w, b, kh, kw, s, p, o, qy, qx, relu, bf16);
    }
}

/* k x k max-pooling with stride k (floor), planar. */
void orc_maxpool(const float *x, int C, int H, int W, int k, float *y)
{
    int Ho = H / k, Wo = W / k;
#pragma omp parallel for collapse(2) schedule(static)
    for (int c = 0; c < C; ++c)
        for (int py = 0; py < Ho; ++py)
            for (int px = 0; px < Wo; ++px) {
                float m = x[((int64_t)c * H + py * k) * W + px * k];
                for (int j = 0; j < k; ++j)
                    for (int i = 0; i < k; ++i) {
                        float v = x[((int64_t)c * H + py * k + j) * W + px * k + i];
                        if (v > m) m = v;
                    }
                y[((int64_t)c * Ho + py) * Wo + px] = m;
            }
}

/* Change detection, Section 3.1:  m(p) = OR over channels of |x(c,p) - ref(c,p)| > tau,
 * evaluated in float (one subtraction, one absolute value, one strict comparison).
 * Returns the number of flagged positions. */
int64_t orc_detect(const float *x, const float *ref, int C, int64_t N, float tau, uint8_t *flag)
{
    int64_t count = 0;
    for (int64_t p = 0; p < N; ++p) {
        uint8_t f = 0;
        for (int c = 0; c < C; ++c) {
            float d = x[(int64_t)c * N + p] - ref[(int64_t)c * N + p];
            if (fabsf(d) > tau) f = 1;
        }
        flag[p] = f;
        count += f;
    }
    return count;
}

/* The stored previous input after a frame.  mode 0: the previous frame's layer input at
 * every position (the x^(t-1) of the detection formula).  mode 1: only flagged positions
 * take the new value (all channels); unflagged ones keep the value they were last
 * recomputed against. */
void orc_update_ref(const float *x, float *ref, int C, int64_t N, const uint8_t *flag, int mode)
{
    for (int c = 0; c < C; ++c)
        for (int64_t p = 0; p < N; ++p)
            if (mode == 0 || flag[p]) ref[(int64_t)c * N + p] = x[(int64_t)c * N + p];
}

/* Which outputs must be recomputed, Section 3.1 second formula, in its gather form:
 * an output position is marked iff some tap of its filter support reads a flagged,
 * in-range input position.  Written for any kernel size, stride and padding. */
void orc_update_set(const uint8_t *flag, int H, int W, int kh, int kw, int s, int p,
                    uint8_t *upd)
{
    int Ho = (H + 2 * p - kh) / s + 1, Wo = (W + 2 * p - kw) / s + 1;
    for (int qy = 0; qy < Ho; ++qy)
        for (int qx = 0; qx < Wo; ++qx) {
            uint8_t m = 0;
            for (int j = 0; j < kh; ++j) {
                int iy = qy * s - p + j;
                if (iy < 0 || iy >= H) continue;
                for (int i = 0; i < kw; ++i) {
                    int ix = qx * s - p + i;
                    if (ix < 0 || ix >= W) continue;
                    if (flag[(int64_t)iy * W + ix]) m = 1;
                }
            }
            upd[(int64_t)qy * Wo + qx] = m;
        }
}

/* Change-index extraction, Section 3.1: the marked positions in ascending order and
 * their count. */
int64_t orc_extract(const uint8_t *map, int64_t n, int32_t *list)
{
    int64_t k = 0;
    for (int64_t p = 0; p < n; ++p)
        if (map[p]) list[k++] = (int32_t)p;
    return k;
}

/* Pooled positions whose window contains an updated position: unique (qy/k, qx/k),
 * as a map over the pooled grid (floor division; positions beyond the last full window
 * belong to no pooled output). */
void orc_pool_set(const uint8_t *upd, int H, int W, int k, uint8_t *pupd)
{
    int Ho = H / k, Wo = W / k;
    memset(pupd, 0, (size_t)Ho * Wo);
    for (int y = 0; y < Ho * k; ++y)
        for (int x = 0; x < Wo * k; ++x)
            if (upd[(int64_t)y * W + x]) pupd[(int64_t)(y / k) * Wo + x / k] = 1;
}

void orc_round_bf16(float *v, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) v[i] = round_to_bf16(v[i]);
}

int orc_max_threads(void)
{
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    return omp_get_max_threads();
#else
    return 1;
#endif
}
