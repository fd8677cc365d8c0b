/*
 * CPU oracle for DHQ (distribution-aware Hadamard quantization) inference of a
 * SIREN-style coordinate MLP.
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It is the slow, plain statement of what
 * the method computes, written from the paper, and exists only so that tests,
 * the smoke check and the benchmark's CPU-baseline leg can compare the GPU
 * library against it.  The GPU library shares no code with it and never calls
 * it.  Nothing here is blocked, fused or reordered: every step is a loop nest
 * a reader can check against the paper by eye.  Floating point is fp64 unless
 * the method fixes a narrower type (scales, biases, activations handed from
 * layer to layer and the final outputs are fp32 values).
 *
 * Steps and where the paper defines them
 *   - Hadamard matrix, Sylvester recursion, H^T H = n I ......... Sec. 3.2, Eq. 3
 *   - transform of a vector / two-sided transform of a matrix ... Sec. 3.2, Eq. 4-5
 *   - "a standard quantizer" after the transform ................ Sec. 3.2 (last
 *     paragraph) with the round() and bit width b of Eq. 1 (Sec. 2.2)
 *   - MAC array with adder tree, quantization module between
 *     layers, sine after every layer but the last ............... Sec. 3.3
 *   - wavelet activation of the second evaluated architecture ... Sec. 4.1, Table 1
 *     (formula from the publication the paper cites for it; see dhqo_activation)
 *
 * Readings taken where the paper is silent (all listed in the design notes):
 * rotation over the input-feature dimension of both operands (it cancels in
 * the product), orthonormal 1/sqrt(n) scaling per side as in Eq. 5, symmetric
 * per-tensor quantizer with zero point 0, scale absmax/qmax, qmax = 2^(b-1)-1,
 * round-half-to-even, codes clamped to [-qmax, qmax], an all-zero tensor gets
 * scale 1.
 *
 * Parity pins (tests marked "not gpu"): H H^T = n I and the popcount closed
 * form; rotation invariance and norm preservation; Eq. 4 against the element
 * form Eq. 5; quantizer brute force and tie table; int32 GEMM against int64;
 * the closed form of layer 1 on the [-1,1]^2 grid; the unquantized rotated
 * path against the plain MLP and against torch's linear+sin.
 * Two-sided variant: the un-rotated product against the plain product, the
 * integer un-rotation against an int64 matrix product with scipy's Hadamard
 * matrix, fan-out 1 against the one-sided path (bitwise), reconstruction
 * error bound of the de-rotated quantized weights.
 * Wavelet activation: the real part of numpy's complex exponential, the
 * zero-spread case against the sine network with shifted biases, evenness,
 * zeros and envelope.
 * Complex-valued wavelet layers (the WIRE architecture as published, see
 * dhqo_activation_complex): the activation against numpy's complex
 * exponential and against its expansion into real functions, the
 * real-valued matrices against numpy's complex matrix product, the whole
 * un-quantized network against a complex-valued numpy network, a purely
 * real pre-activation against the real wavelet.
 * Parity unpinned: absolute image quality (Table 1) -- it needs the paper's
 * images and trained weights.
 */
#include <complex.h>
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define DHQO_OK 0
#define DHQO_EINVAL (-1)
#define DHQO_ENOMEM (-2)
#define DHQO_EOVERFLOW (-3)

/* ---------------------------------------------------------------- helpers */

/* Smallest power of two >= k (k >= 1). */
int dhqo_next_pow2(int k)
{
    int p = 1;
    while (p < k) p *= 2;
    return p;
}

/* qmax = 2^(b-1) - 1 : the largest code of a symmetric b-bit quantizer. */
int dhqo_qmax(int bits)
{
    return (1 << (bits - 1)) - 1;
}

/*
 * Sec. 3.2, Eq. 3: H_1 = [1], H_2n = [[H_n, H_n], [H_n, -H_n]].
 * Writes the n x n matrix of +1/-1 (row-major, as doubles).  n must be a
 * power of two.
 */
int dhqo_hadamard(int n, double *H)
{
    if (n < 1 || (n & (n - 1)) != 0 || !H) return DHQO_EINVAL;
    H[0] = 1.0;
    for (int m = 1; m < n; m *= 2) {
        /* The m x m block in the top-left corner is H_m; fill the other three
         * blocks of H_2m.  Go through rows from the bottom up so that H_m is
         * not overwritten before it has been read (row stride is n). */
        for (int i = m - 1; i >= 0; --i) {
            for (int j = 0; j < m; ++j) {
                double h = H[(size_t)i * n + j];
                H[(size_t)i * n + (j + m)] = h;
                H[(size_t)(i + m) * n + j] = h;
                H[(size_t)(i + m) * n + (j + m)] = -h;
            }
        }
    }
    return DHQO_OK;
}

/*
 * Transform of row vectors (Sec. 3.2, the vector case of Eq. 4 with the
 * normalisation of Eq. 5): each of the `rows` rows of x (rows x K, fp64) is
 * zero-padded to Kp = next_pow2(K) and multiplied by H_Kp / sqrt(Kp).
 * xr is rows x Kp.
 */
int dhqo_rotate_rows(const double *x, int64_t rows, int K, double *xr)
{
    if (!x || !xr || rows < 0 || K < 1) return DHQO_EINVAL;
    int Kp = dhqo_next_pow2(K);
    double *H = (double *)malloc(sizeof(double) * (size_t)Kp * Kp);
    if (!H) return DHQO_ENOMEM;
    dhqo_hadamard(Kp, H);
    const double inv = 1.0 / sqrt((double)Kp);
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        const double *xi = x + r * K;
        double *yo = xr + r * Kp;
        for (int j = 0; j < Kp; ++j) {
            double s = 0.0;
            for (int k = 0; k < K; ++k) /* padded entries k >= K are zero */
                s += xi[k] * H[(size_t)k * Kp + j];
            yo[j] = s * inv;
        }
    }
    free(H);
    return DHQO_OK;
}

/*
 * Two-sided transform of a matrix, Eq. 4 with the 1/sqrt(mn) of Eq. 5:
 * W' = H_m W H_n / sqrt(m n); m and n powers of two.  Used by the pins only
 * (the inference path rotates the input-feature side).
 */
int dhqo_rotate_two_sided(const double *W, int m, int n, double *Wp)
{
    if (!W || !Wp) return DHQO_EINVAL;
    if (m < 1 || n < 1 || (m & (m - 1)) || (n & (n - 1))) return DHQO_EINVAL;
    double *Hm = (double *)malloc(sizeof(double) * (size_t)m * m);
    double *Hn = (double *)malloc(sizeof(double) * (size_t)n * n);
    double *T = (double *)malloc(sizeof(double) * (size_t)m * n);
    if (!Hm || !Hn || !T) { free(Hm); free(Hn); free(T); return DHQO_ENOMEM; }
    dhqo_hadamard(m, Hm);
    dhqo_hadamard(n, Hn);
    for (int i = 0; i < m; ++i)          /* T = H_m W */
        for (int l = 0; l < n; ++l) {
            double s = 0.0;
            for (int k = 0; k < m; ++k) s += Hm[(size_t)i * m + k] * W[(size_t)k * n + l];
            T[(size_t)i * n + l] = s;
        }
    const double inv = 1.0 / sqrt((double)m * (double)n);
    for (int i = 0; i < m; ++i)          /* W' = T H_n / sqrt(mn) */
        for (int j = 0; j < n; ++j) {
            double s = 0.0;
            for (int l = 0; l < n; ++l) s += T[(size_t)i * n + l] * Hn[(size_t)l * n + j];
            Wp[(size_t)i * n + j] = s * inv;
        }
    free(Hm); free(Hn); free(T);
    return DHQO_OK;
}

/*
 * Per-tensor scale of the symmetric quantizer: s = (float)(max|x| / qmax);
 * an all-zero tensor gets s = 1.
 */
float dhqo_absmax_scale(const double *x, int64_t count, int bits)
{
    double m = 0.0;
    for (int64_t i = 0; i < count; ++i) {
        double a = fabs(x[i]);
        if (a > m) m = a;
    }
    if (m == 0.0) return 1.0f;
    return (float)(m / (double)dhqo_qmax(bits));
}

/*
 * The quantizer: q = clamp(rne(x / s), -qmax, qmax).  nearbyint() rounds
 * half to even under the default rounding mode, which this file never
 * changes.
 */
int dhqo_quantize(const double *x, int64_t count, float s, int bits, int8_t *q)
{
    if (!x || !q || bits < 2 || bits > 8 || !(s > 0.0f) || !isfinite(s)) return DHQO_EINVAL;
    const double qmax = (double)dhqo_qmax(bits);
    const double sd = (double)s;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < count; ++i) {
        double r = nearbyint(x[i] / sd);
        if (r > qmax) r = qmax;
        if (r < -qmax) r = -qmax;
        q[i] = (int8_t)r;
    }
    return DHQO_OK;
}

/* Dequantizer of the same quantizer (used by the pins): x ~ q * s. */
void dhqo_dequantize(const int8_t *q, int64_t count, float s, double *x)
{
    for (int64_t i = 0; i < count; ++i) x[i] = (double)q[i] * (double)s;
}

/*
 * Integer GEMM of the MAC array (Sec. 3.3): acc[i][j] = sum_k q[i][k] w[j][k],
 * q is N x Kp, w is M x Kp, acc is N x M, all row-major.  Accumulates in
 * int32 and, beside it, in int64; returns DHQO_EOVERFLOW if they ever differ.
 */
int dhqo_igemm(const int8_t *q, const int8_t *w, int64_t N, int M, int Kp, int32_t *acc)
{
    if (!q || !w || !acc || N < 0 || M < 1 || Kp < 1) return DHQO_EINVAL;
    int bad = 0;
#pragma omp parallel for schedule(static) reduction(| : bad)
    for (int64_t i = 0; i < N; ++i) {
        const int8_t *qi = q + i * Kp;
        for (int j = 0; j < M; ++j) {
            const int8_t *wj = w + (size_t)j * Kp;
            int32_t a32 = 0;
            int64_t a64 = 0;
            for (int k = 0; k < Kp; ++k) {
                int32_t p = (int32_t)qi[k] * (int32_t)wj[k];
                a32 = (int32_t)((uint32_t)a32 + (uint32_t)p); /* wraps like hardware */
                a64 += p;
            }
            if ((int64_t)a32 != a64) bad |= 1;
            acc[i * M + j] = a32;
        }
    }
    return bad ? DHQO_EOVERFLOW : DHQO_OK;
}

/*
 * Activation functions (argument y = the layer's pre-activation, fp64).
 *   DHQO_ACT_NONE   y                                   the output layer (Sec. 3.3)
 *   DHQO_ACT_SINE   sin(omega0 y)                       SIREN (Sec. 3.1, 3.3)
 *   DHQO_ACT_GABOR  cos(omega0 y) exp(-(s0 y)^2)        wavelet activation: the real part of
 *                   the complex Gabor wavelet exp(j omega0 y - |s0 y|^2) of the WIRE
 *                   architecture that Sec. 4.1 / Table 1 evaluate.  Reading: the paper names
 *                   WIRE and cites its publication but prints neither the activation nor the
 *                   layer structure; the activation is taken from that publication, and the
 *                   network is kept real-valued (real weights, real part of the wavelet), so
 *                   that every other step of the quantized path is unchanged.
 */
#define DHQO_ACT_NONE 0
#define DHQO_ACT_SINE 1
#define DHQO_ACT_GABOR 2
#define DHQO_ACT_GABOR_COMPLEX 3

double dhqo_activation(double y, int act, double omega0, double s0)
{
    if (act == DHQO_ACT_SINE) return sin(omega0 * y);
    if (act == DHQO_ACT_GABOR) return cos(omega0 * y) * exp(-(s0 * y) * (s0 * y));
    return y;
}

/*
 * DHQO_ACT_GABOR_COMPLEX: the WIRE architecture as its publication has it (Sec. 4.1 / Table 1 name
 * it and cite that publication): hidden features are complex numbers, the weights of every
 * layer after the first are complex, the activation is the complex Gabor wavelet
 *     a = exp(j omega0 y - |s0 y|^2)          y = yr + j yi complex,
 * and the network's output is the real part of the last (linear) layer.  Written out with the
 * C library's complex exponential: this is the definition, not an expansion of it.
 * Reading (the paper says nothing about complex numbers): such a network is run as a real one
 * of twice the width -- feature 2m holds Re, feature 2m + 1 holds Im, a complex weight w
 * becomes the 2 x 2 block [[Re w, -Im w], [Im w, Re w]] (dhqo_complex_layer_to_real) -- so that
 * the rotation of Eq. 3-5, the quantizer and the integer product apply to it unchanged, and only
 * the activation acts on pairs of features.
 */
void dhqo_activation_complex(double yr, double yi, double omega0, double s0, double *ar, double *ai)
{
    const double complex y = yr + yi * I;
    const double mag = cabs(s0 * y);
    const double complex a = cexp(I * omega0 * y - mag * mag);
    *ar = creal(a);
    *ai = cimag(a);
}

/*
 * A layer with complex weights W = Wre + j Wim (M x K) and bias b = bre + j bim as the real layer
 * that computes the same thing on interleaved (Re, Im) features:
 *   in_complex  != 0: the input has K complex features = 2 K real ones (else K real ones);
 *   out_complex != 0: the output has M complex features = 2 M real ones; else the output is
 *                     the real part (the network's last layer), M real features.
 * Wim / bim may be NULL (a real-valued layer, e.g. the first one).  W gets
 * (out_complex ? 2 M : M) x (in_complex ? 2 K : K) floats, b as many as W has rows.
 *   Re (w x) = Re w Re x - Im w Im x        Im (w x) = Im w Re x + Re w Im x
 */
int dhqo_complex_layer_to_real(const float *Wre, const float *Wim, const float *bre, const float *bim, int M, int K,
                               int in_complex, int out_complex, float *W, float *b)
{
    if (!Wre || !bre || !W || !b || M < 1 || K < 1) return DHQO_EINVAL;
    const int cols = in_complex ? 2 * K : K;
    for (int m = 0; m < M; ++m) {
        float *row_re = W + (size_t)(out_complex ? 2 * m : m) * cols;
        float *row_im = out_complex ? row_re + cols : NULL;
        for (int k = 0; k < K; ++k) {
            const float wr = Wre[(size_t)m * K + k], wi = Wim ? Wim[(size_t)m * K + k] : 0.0f;
            if (in_complex) {
                row_re[2 * k] = wr;
                row_re[2 * k + 1] = -wi;
                if (row_im) { row_im[2 * k] = wi; row_im[2 * k + 1] = wr; }
            } else {
                row_re[k] = wr;
                if (row_im) row_im[k] = wi;
            }
        }
        if (out_complex) {
            b[2 * m] = bre[m];
            b[2 * m + 1] = bim ? bim[m] : 0.0f;
        } else {
            b[m] = bre[m];
        }
    }
    return DHQO_OK;
}

/*
 * Dequantize, add bias and (except in the output layer) apply the sine
 * or the wavelet (Sec. 3.3): y = acc * (s_a * s_w) + b;  a = activation(y),
 * rounded once to fp32;  the output layer (act = DHQO_ACT_NONE) returns (float) y.
 */
int dhqo_epilogue(const int32_t *acc, int64_t N, int M, float s_a, float s_w,
                  const float *b, int act, float omega0, float s0, float *out)
{
    if (!acc || !b || !out) return DHQO_EINVAL;
    const double sc = (double)s_a * (double)s_w;
    if (act == DHQO_ACT_GABOR_COMPLEX) {
        if (M % 2) return DHQO_EINVAL;
#pragma omp parallel for schedule(static)
        for (int64_t i = 0; i < N; ++i)
            for (int j = 0; j < M; j += 2) {
                double yr = (double)acc[i * M + j] * sc + (double)b[j];
                double yi = (double)acc[i * M + j + 1] * sc + (double)b[j + 1];
                double ar, ai;
                dhqo_activation_complex(yr, yi, (double)omega0, (double)s0, &ar, &ai);
                out[i * M + j] = (float)ar;
                out[i * M + j + 1] = (float)ai;
            }
        return DHQO_OK;
    }
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < N; ++i)
        for (int j = 0; j < M; ++j) {
            double y = (double)acc[i * M + j] * sc + (double)b[j];
            out[i * M + j] = (float)dhqo_activation(y, act, (double)omega0, (double)s0);
        }
    return DHQO_OK;
}

/*
 * Offline weight step: rotate each row of W (M x K, fp32) over the
 * input-feature dimension, take the per-tensor scale, quantize.
 * Wq is M x Kp.  If rot_out is not NULL it receives the rotated fp64 weights.
 */
int dhqo_quantize_weights(const float *W, int M, int K, int bits, int8_t *Wq, float *s_w,
                          double *rot_out)
{
    if (!W || !Wq || !s_w || M < 1 || K < 1 || bits < 2 || bits > 8) return DHQO_EINVAL;
    int Kp = dhqo_next_pow2(K);
    double *Wd = (double *)malloc(sizeof(double) * (size_t)M * K);
    double *Wr = (double *)malloc(sizeof(double) * (size_t)M * Kp);
    if (!Wd || !Wr) { free(Wd); free(Wr); return DHQO_ENOMEM; }
    for (size_t i = 0; i < (size_t)M * K; ++i) Wd[i] = (double)W[i];
    int rc = dhqo_rotate_rows(Wd, M, K, Wr);
    if (rc == DHQO_OK) {
        *s_w = dhqo_absmax_scale(Wr, (int64_t)M * Kp, bits);
        rc = dhqo_quantize(Wr, (int64_t)M * Kp, *s_w, bits, Wq);
        if (rot_out) memcpy(rot_out, Wr, sizeof(double) * (size_t)M * Kp);
    }
    free(Wd); free(Wr);
    return rc;
}

/*
 * One quantized layer on N rows.
 *   a_in   N x K fp32 (the previous layer's output, or the coordinates)
 *   Wq     M x Kp int8, s_w, bias[M]
 *   *s_a   activation scale; if calibrate != 0 it is computed here from the
 *          whole rotated N x Kp tensor (per-tensor absmax) and written back
 *   out    N x M fp32
 * Optional dumps (may be NULL): rot N x Kp fp64, codes N x Kp, acc N x M.
 */
int dhqo_layer(const float *a_in, int64_t N, int K, int M, const int8_t *Wq, float s_w,
               const float *bias, float *s_a, int calibrate, int bits_a, int act,
               float omega0, float s0, float *out, double *dump_rot, int8_t *dump_codes,
               int32_t *dump_acc)
{
    if (!a_in || !Wq || !bias || !s_a || !out || N < 0) return DHQO_EINVAL;
    int Kp = dhqo_next_pow2(K);
    int rc = DHQO_OK;
    double *ad = (double *)malloc(sizeof(double) * (size_t)(N * K + 1));
    double *rot = dump_rot ? dump_rot : (double *)malloc(sizeof(double) * (size_t)(N * Kp + 1));
    int8_t *codes = dump_codes ? dump_codes : (int8_t *)malloc((size_t)(N * Kp + 1));
    int32_t *acc = dump_acc ? dump_acc : (int32_t *)malloc(sizeof(int32_t) * (size_t)(N * M + 1));
    if (!ad || !rot || !codes || !acc) { rc = DHQO_ENOMEM; goto done; }
    for (int64_t i = 0; i < N * K; ++i) ad[i] = (double)a_in[i];
    rc = dhqo_rotate_rows(ad, N, K, rot);
    if (rc) goto done;
    if (calibrate) *s_a = dhqo_absmax_scale(rot, N * Kp, bits_a);
    rc = dhqo_quantize(rot, N * Kp, *s_a, bits_a, codes);
    if (rc) goto done;
    rc = dhqo_igemm(codes, Wq, N, M, Kp, acc);
    if (rc) goto done;
    rc = dhqo_epilogue(acc, N, M, *s_a, s_w, bias, act, omega0, s0, out);
done:
    free(ad);
    if (!dump_rot) free(rot);
    if (!dump_codes) free(codes);
    if (!dump_acc) free(acc);
    return rc;
}

/*
 * Whole quantized forward.  dims has n_layers+1 entries.  Wq[l] is
 * dims[l+1] x next_pow2(dims[l]); bias[l] has dims[l+1] entries.
 * s_a has n_layers entries: read when calibrate == 0, written when
 * calibrate != 0 (each layer's scale is then measured on the input that the
 * quantized layers before it produced).  The activation `act` (sine or wavelet) follows every layer except
 * the last.  Optional per-layer dumps: arrays of n_layers pointers, each
 * either NULL or a buffer of the size given in dhqo_layer.
 */
int dhqo_forward(int n_layers, const int32_t *dims, int act, float omega0, float s0, int bits_a,
                 const int8_t *const *Wq, const float *s_w, const float *const *bias,
                 float *s_a, int calibrate, const float *coords, int64_t N, float *out,
                 double *const *dump_rot, int8_t *const *dump_codes,
                 int32_t *const *dump_acc, float *const *dump_act)
{
    if (n_layers < 1 || !dims || !Wq || !s_w || !bias || !s_a || !coords || !out || N < 0)
        return DHQO_EINVAL;
    int rc = DHQO_OK;
    const float *cur = coords;
    float *owned = NULL;
    for (int l = 0; l < n_layers; ++l) {
        int K = dims[l], M = dims[l + 1];
        int last = (l == n_layers - 1);
        float *dst = last ? out : (float *)malloc(sizeof(float) * (size_t)(N * M + 1));
        if (!dst) { rc = DHQO_ENOMEM; break; }
        rc = dhqo_layer(cur, N, K, M, Wq[l], s_w[l], bias[l], &s_a[l], calibrate, bits_a,
                        last ? DHQO_ACT_NONE : act, omega0, s0, dst, dump_rot ? dump_rot[l] : NULL,
                        dump_codes ? dump_codes[l] : NULL, dump_acc ? dump_acc[l] : NULL);
        if (rc == DHQO_OK && dump_act && dump_act[l])
            memcpy(dump_act[l], dst, sizeof(float) * (size_t)(N * M));
        free(owned);
        owned = last ? NULL : dst;
        cur = dst;
        if (rc) break;
    }
    free(owned);
    return rc;
}

/* ------------------------------------------------------------------------
 * Two-sided variant: the weight transform exactly as Eq. 4-5 print it,
 * W' = H_m W H_n / sqrt(m n), over BOTH the output-feature side (m) and the
 * input-feature side (n).  The activations are rotated over the input
 * features as before, so the integer GEMM now yields the layer output in the
 * rotated output basis: acc' = q W'q^T ~ (a W^T) H_m / (s_a s_w sqrt(m)).
 * Because H_m H_m = m I the rotation is undone by one more multiplication by
 * H_m, which has entries +-1 and is therefore exact on the int32
 * accumulators; the factor 1/sqrt(m) joins the dequantization scale.
 * Fan-out M is zero-padded to Mp = next_pow2(M) (rows of zeros), the padded
 * outputs are dropped after the un-rotation.  Reading of the paper: it
 * prints only the weight transform; how the output side is undone is this
 * build's choice (listed in the design notes).
 * ---------------------------------------------------------------------- */

/*
 * Offline weight step, two-sided.  W is M x K fp32; Wq is Mp x Kp int8.
 * If rot_out is not NULL it receives the rotated fp64 weights (Mp x Kp).
 */
int dhqo_quantize_weights_two_sided(const float *W, int M, int K, int bits, int8_t *Wq,
                                    float *s_w, double *rot_out)
{
    if (!W || !Wq || !s_w || M < 1 || K < 1 || bits < 2 || bits > 8) return DHQO_EINVAL;
    int Kp = dhqo_next_pow2(K), Mp = dhqo_next_pow2(M);
    double *Wd = (double *)calloc((size_t)Mp * Kp, sizeof(double));
    double *Wr = (double *)malloc(sizeof(double) * (size_t)Mp * Kp);
    if (!Wd || !Wr) { free(Wd); free(Wr); return DHQO_ENOMEM; }
    for (int j = 0; j < M; ++j)
        for (int k = 0; k < K; ++k) Wd[(size_t)j * Kp + k] = (double)W[(size_t)j * K + k];
    int rc = dhqo_rotate_two_sided(Wd, Mp, Kp, Wr);
    if (rc == DHQO_OK) {
        *s_w = dhqo_absmax_scale(Wr, (int64_t)Mp * Kp, bits);
        rc = dhqo_quantize(Wr, (int64_t)Mp * Kp, *s_w, bits, Wq);
        if (rot_out) memcpy(rot_out, Wr, sizeof(double) * (size_t)Mp * Kp);
    }
    free(Wd); free(Wr);
    return rc;
}

/*
 * Un-rotation of the accumulators: z[i][j] = sum_j' acc[i][j'] H_Mp[j'][j],
 * acc and z are N x Mp int32.  Computed in int64; DHQO_EOVERFLOW if a result
 * does not fit int32.
 */
int dhqo_unrotate_acc(const int32_t *acc, int64_t N, int Mp, int32_t *z)
{
    if (!acc || !z || N < 0 || Mp < 1 || (Mp & (Mp - 1))) return DHQO_EINVAL;
    double *H = (double *)malloc(sizeof(double) * (size_t)Mp * Mp);
    if (!H) return DHQO_ENOMEM;
    dhqo_hadamard(Mp, H);
    int bad = 0;
#pragma omp parallel for schedule(static) reduction(| : bad)
    for (int64_t i = 0; i < N; ++i)
        for (int j = 0; j < Mp; ++j) {
            int64_t s = 0;
            for (int jp = 0; jp < Mp; ++jp)
                s += (H[(size_t)jp * Mp + j] > 0.0) ? (int64_t)acc[i * Mp + jp] : -(int64_t)acc[i * Mp + jp];
            if (s > INT32_MAX || s < INT32_MIN) bad |= 1;
            z[i * Mp + j] = (int32_t)s;
        }
    free(H);
    return bad ? DHQO_EOVERFLOW : DHQO_OK;
}

/*
 * One quantized layer, two-sided.  Same arguments as dhqo_layer except that
 * Wq is Mp x Kp.  Optional dumps: rot N x Kp fp64, codes N x Kp, acc N x Mp
 * (the rotated accumulators), unrot N x Mp (after the un-rotation).
 * y[j] = z[j] * (s_a s_w / sqrt(Mp)) + b[j] for j < M.
 */
int dhqo_layer_two_sided(const float *a_in, int64_t N, int K, int M, const int8_t *Wq, float s_w,
                         const float *bias, float *s_a, int calibrate, int bits_a, int act,
                         float omega0, float s0, float *out, double *dump_rot, int8_t *dump_codes,
                         int32_t *dump_acc, int32_t *dump_unrot)
{
    if (!a_in || !Wq || !bias || !s_a || !out || N < 0) return DHQO_EINVAL;
    int Kp = dhqo_next_pow2(K), Mp = dhqo_next_pow2(M);
    int rc = DHQO_OK;
    double *ad = (double *)malloc(sizeof(double) * (size_t)(N * K + 1));
    double *rot = dump_rot ? dump_rot : (double *)malloc(sizeof(double) * (size_t)(N * Kp + 1));
    int8_t *codes = dump_codes ? dump_codes : (int8_t *)malloc((size_t)(N * Kp + 1));
    int32_t *acc = dump_acc ? dump_acc : (int32_t *)malloc(sizeof(int32_t) * (size_t)(N * Mp + 1));
    int32_t *z = dump_unrot ? dump_unrot : (int32_t *)malloc(sizeof(int32_t) * (size_t)(N * Mp + 1));
    if (!ad || !rot || !codes || !acc || !z) { rc = DHQO_ENOMEM; goto done; }
    for (int64_t i = 0; i < N * K; ++i) ad[i] = (double)a_in[i];
    rc = dhqo_rotate_rows(ad, N, K, rot);
    if (rc) goto done;
    if (calibrate) *s_a = dhqo_absmax_scale(rot, N * Kp, bits_a);
    rc = dhqo_quantize(rot, N * Kp, *s_a, bits_a, codes);
    if (rc) goto done;
    rc = dhqo_igemm(codes, Wq, N, Mp, Kp, acc);
    if (rc) goto done;
    rc = dhqo_unrotate_acc(acc, N, Mp, z);
    if (rc) goto done;
    {
        const double sc = (double)*s_a * (double)s_w / sqrt((double)Mp);
        if (act == DHQO_ACT_GABOR_COMPLEX && M % 2) { rc = DHQO_EINVAL; goto done; }
#pragma omp parallel for schedule(static)
        for (int64_t i = 0; i < N; ++i)
            for (int j = 0; j < M; ++j) {
                double y = (double)z[i * Mp + j] * sc + (double)bias[j];
                if (act == DHQO_ACT_GABOR_COMPLEX) {
                    if (j % 2) continue;  /* the pair (j, j + 1) was taken at j */
                    double yi = (double)z[i * Mp + j + 1] * sc + (double)bias[j + 1], ar, ai;
                    dhqo_activation_complex(y, yi, (double)omega0, (double)s0, &ar, &ai);
                    out[i * M + j] = (float)ar;
                    out[i * M + j + 1] = (float)ai;
                } else {
                    out[i * M + j] = (float)dhqo_activation(y, act, (double)omega0, (double)s0);
                }
            }
    }
done:
    free(ad);
    if (!dump_rot) free(rot);
    if (!dump_codes) free(codes);
    if (!dump_acc) free(acc);
    if (!dump_unrot) free(z);
    return rc;
}

/* Whole quantized forward, two-sided; arguments as dhqo_forward (Wq[l] is Mp x Kp). */
int dhqo_forward_two_sided(int n_layers, const int32_t *dims, int act, float omega0, float s0, int bits_a,
                           const int8_t *const *Wq, const float *s_w, const float *const *bias,
                           float *s_a, int calibrate, const float *coords, int64_t N, float *out,
                           double *const *dump_rot, int8_t *const *dump_codes,
                           int32_t *const *dump_acc, float *const *dump_act)
{
    if (n_layers < 1 || !dims || !Wq || !s_w || !bias || !s_a || !coords || !out || N < 0)
        return DHQO_EINVAL;
    int rc = DHQO_OK;
    const float *cur = coords;
    float *owned = NULL;
    for (int l = 0; l < n_layers; ++l) {
        int K = dims[l], M = dims[l + 1];
        int last = (l == n_layers - 1);
        float *dst = last ? out : (float *)malloc(sizeof(float) * (size_t)(N * M + 1));
        if (!dst) { rc = DHQO_ENOMEM; break; }
        rc = dhqo_layer_two_sided(cur, N, K, M, Wq[l], s_w[l], bias[l], &s_a[l], calibrate, bits_a,
                                  last ? DHQO_ACT_NONE : act, omega0, s0, dst, dump_rot ? dump_rot[l] : NULL,
                                  dump_codes ? dump_codes[l] : NULL, dump_acc ? dump_acc[l] : NULL, NULL);
        if (rc == DHQO_OK && dump_act && dump_act[l])
            memcpy(dump_act[l], dst, sizeof(float) * (size_t)(N * M));
        free(owned);
        owned = last ? NULL : dst;
        cur = dst;
        if (rc) break;
    }
    free(owned);
    return rc;
}

/* ------------------------------------------------------------------------
 * Weight-only quantization, "W8A32" (Sec. 1, Fig. 1-2, Table 2): the weights
 * go through the same offline step (rotation over the input features,
 * per-tensor scale, quantizer) and are then used de-quantized, the
 * activations stay in floating point.  De-quantized weights in the original
 * basis: W~ = (s_w Wq) Hn (Hn is symmetric and orthonormal, so the rotation is
 * undone by applying it again), columns beyond K dropped, rounded to fp32.
 * The W8A32 network is the plain MLP (dhqo_mlp_float) run on W~; "W32A32" is
 * dhqo_mlp_float on the original weights.
 * ---------------------------------------------------------------------- */
int dhqo_dequantize_weights(const int8_t *Wq, float s_w, int M, int K, float *Wt)
{
    if (!Wq || !Wt || M < 1 || K < 1 || !(s_w > 0.0f)) return DHQO_EINVAL;
    int Kp = dhqo_next_pow2(K);
    double *d = (double *)malloc(sizeof(double) * (size_t)M * Kp);
    double *r = (double *)malloc(sizeof(double) * (size_t)M * Kp);
    if (!d || !r) { free(d); free(r); return DHQO_ENOMEM; }
    dhqo_dequantize(Wq, (int64_t)M * Kp, s_w, d);
    int rc = dhqo_rotate_rows(d, M, Kp, r);
    if (rc == DHQO_OK)
        for (int j = 0; j < M; ++j)
            for (int k = 0; k < K; ++k) Wt[(size_t)j * K + k] = (float)r[(size_t)j * Kp + k];
    free(d); free(r);
    return rc;
}

/*
 * Float reference: the plain MLP, neither rotated nor quantized, in fp64
 * (out64) and, if out32 is not NULL, a second pass in fp32 arithmetic.
 * y = W a + b per layer, the activation (sine or wavelet) after all but the last.
 */
int dhqo_mlp_float(int n_layers, const int32_t *dims, int act, float omega0, float s0, const float *const *W,
                   const float *const *bias, const float *coords, int64_t N, double *out64,
                   float *out32)
{
    if (n_layers < 1 || !dims || !W || !bias || !coords || N < 0) return DHQO_EINVAL;
    if (act == DHQO_ACT_GABOR_COMPLEX)
        for (int l = 1; l < n_layers; ++l) if (dims[l] % 2) return DHQO_EINVAL;
    int maxw = 0;
    for (int l = 0; l <= n_layers; ++l) if (dims[l] > maxw) maxw = dims[l];
    int fail = 0;
#pragma omp parallel
    {
        double *a = (double *)malloc(sizeof(double) * (size_t)maxw);
        double *y = (double *)malloc(sizeof(double) * (size_t)maxw);
        float *af = (float *)malloc(sizeof(float) * (size_t)maxw);
        float *yf = (float *)malloc(sizeof(float) * (size_t)maxw);
        if (!a || !y || !af || !yf) {
#pragma omp atomic write
            fail = 1;
        } else {
#pragma omp for schedule(static)
            for (int64_t i = 0; i < N; ++i) {
                for (int k = 0; k < dims[0]; ++k) {
                    a[k] = (double)coords[i * dims[0] + k];
                    af[k] = coords[i * dims[0] + k];
                }
                for (int l = 0; l < n_layers; ++l) {
                    int K = dims[l], M = dims[l + 1], last = (l == n_layers - 1);
                    for (int j = 0; j < M; ++j) {
                        double s = 0.0;
                        float sf = 0.0f;
                        for (int k = 0; k < K; ++k) {
                            s += (double)W[l][(size_t)j * K + k] * a[k];
                            sf += W[l][(size_t)j * K + k] * af[k];
                        }
                        s += (double)bias[l][j];
                        sf += bias[l][j];
                        y[j] = s;
                        yf[j] = sf;
                    }
                    if (!last && act == DHQO_ACT_GABOR_COMPLEX) {
                        /* pairs (2m, 2m + 1) = (Re, Im); an odd width is refused by the caller's check below */
                        for (int j = 0; j + 1 < M; j += 2) {
                            double ar, ai;
                            dhqo_activation_complex(y[j], y[j + 1], (double)omega0, (double)s0, &ar, &ai);
                            const float complex zf = yf[j] + yf[j + 1] * I;
                            const float mf = cabsf(s0 * zf);
                            const float complex af = cexpf(I * omega0 * zf - mf * mf);
                            y[j] = ar; y[j + 1] = ai;
                            yf[j] = crealf(af); yf[j + 1] = cimagf(af);
                        }
                    } else if (!last) {
                        for (int j = 0; j < M; ++j) {
                            const double s = y[j];
                            const float sf = yf[j];
                            y[j] = dhqo_activation(s, act, (double)omega0, (double)s0);
                            if (act == DHQO_ACT_GABOR) yf[j] = cosf(omega0 * sf) * expf(-(s0 * sf) * (s0 * sf));
                            else if (act == DHQO_ACT_SINE) yf[j] = sinf(omega0 * sf);
                        }
                    }
                    memcpy(a, y, sizeof(double) * (size_t)M);
                    memcpy(af, yf, sizeof(float) * (size_t)M);
                }
                int Mo = dims[n_layers];
                if (out64) for (int j = 0; j < Mo; ++j) out64[i * Mo + j] = a[j];
                if (out32) for (int j = 0; j < Mo; ++j) out32[i * Mo + j] = af[j];
            }
        }
        free(a); free(y); free(af); free(yf);
    }
    return fail ? DHQO_ENOMEM : DHQO_OK;
}

/*
 * The rotated but unquantized network in fp64: each layer computes
 * (pad(a) Hn)(pad(W) Hn)^T + b.  Because Hn Hn^T = I this equals the plain
 * MLP; the pin that compares the two checks the rotation's placement,
 * padding and normalisation.
 */
int dhqo_mlp_rotated_f64(int n_layers, const int32_t *dims, float omega0,
                         const float *const *W, const float *const *bias,
                         const float *coords, int64_t N, double *out64)
{
    if (n_layers < 1 || !dims || !W || !bias || !coords || !out64 || N < 0) return DHQO_EINVAL;
    int rc = DHQO_OK;
    double *cur = (double *)malloc(sizeof(double) * (size_t)(N * dims[0] + 1));
    if (!cur) return DHQO_ENOMEM;
    for (int64_t i = 0; i < N * dims[0]; ++i) cur[i] = (double)coords[i];
    for (int l = 0; l < n_layers && rc == DHQO_OK; ++l) {
        int K = dims[l], M = dims[l + 1], Kp = dhqo_next_pow2(K), last = (l == n_layers - 1);
        double *Wd = (double *)malloc(sizeof(double) * (size_t)M * K);
        double *Wr = (double *)malloc(sizeof(double) * (size_t)M * Kp);
        double *ar = (double *)malloc(sizeof(double) * (size_t)(N * Kp + 1));
        double *nxt = (double *)malloc(sizeof(double) * (size_t)(N * M + 1));
        if (!Wd || !Wr || !ar || !nxt) rc = DHQO_ENOMEM;
        if (rc == DHQO_OK) {
            for (size_t i = 0; i < (size_t)M * K; ++i) Wd[i] = (double)W[l][i];
            rc = dhqo_rotate_rows(Wd, M, K, Wr);
        }
        if (rc == DHQO_OK) rc = dhqo_rotate_rows(cur, N, K, ar);
        if (rc == DHQO_OK) {
#pragma omp parallel for schedule(static)
            for (int64_t i = 0; i < N; ++i)
                for (int j = 0; j < M; ++j) {
                    double s = 0.0;
                    for (int k = 0; k < Kp; ++k) s += ar[i * Kp + k] * Wr[(size_t)j * Kp + k];
                    s += (double)bias[l][j];
                    nxt[i * M + j] = last ? s : sin((double)omega0 * s);
                }
        }
        free(Wd); free(Wr); free(ar); free(cur);
        cur = nxt;
    }
    if (rc == DHQO_OK) memcpy(out64, cur, sizeof(double) * (size_t)(N * dims[n_layers]));
    free(cur);
    return rc;
}
