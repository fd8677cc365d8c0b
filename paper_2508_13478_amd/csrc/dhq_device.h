// Device-side helpers shared by the layer-by-layer kernels and the fused kernel.
#ifndef DHQ_DEVICE_H
#define DHQ_DEVICE_H

#include <hip/hip_runtime.h>
#include <stdint.h>

typedef int dhq_v4i __attribute__((ext_vector_type(4)));
typedef int dhq_v16i __attribute__((ext_vector_type(16)));

// 1.5 * 2^23: adding it to a float |v| < 2^22 leaves round-half-to-even(v) in the low
// mantissa bits, because the sum's unit in the last place is exactly 1.
#define DHQ_MAGIC_F 12582912.0f
#define DHQ_MAGIC_I 0x4B400000

// The quantizer of Sec. 3.2 (symmetric, round-half-to-even, clamp to +-qmax) on one value:
// returns an int whose low byte is the two's-complement code.
// One fused multiply-add rounds x*inv to an integer exactly once (no double rounding);
// float bit patterns of positive floats are ordered like integers and negative floats are
// negative integers, so one integer clamp also handles values far outside the range.
__device__ __forceinline__ int dhq_quant_bits(float x, float inv, int qmax)
{
    float t = __builtin_fmaf(x, inv, DHQ_MAGIC_F);
    int b = __float_as_int(t);
    return min(max(b, DHQ_MAGIC_I - qmax), DHQ_MAGIC_I + qmax);
}

// Packs the low bytes of four quantizer results into one dword (byte 0 = a).
__device__ __forceinline__ unsigned dhq_pack4(int a, int b, int c, int d)
{
    unsigned lo = __builtin_amdgcn_perm((unsigned)b, (unsigned)a, 0x0c0c0400u);
    unsigned hi = __builtin_amdgcn_perm((unsigned)d, (unsigned)c, 0x0c0c0400u);
    return __builtin_amdgcn_perm(hi, lo, 0x05040100u);
}

// sin(2 pi t): the hardware sine takes its argument in revolutions (defined for |t| <= 256).
__device__ __forceinline__ float dhq_sin_rev(float t)
{
    return __builtin_amdgcn_sinf(t);
}

// What follows a layer's affine part: nothing (the output layer), the sine of Sec. 3.3, or the
// wavelet cos(omega0 y) exp(-(s0 y)^2) (the real part of the complex Gabor wavelet of the WIRE
// architecture, Sec. 4.1).  c2 = 2 pi s0 sqrt(log2 e) / omega0 turns the argument in revolutions
// into the square root of the envelope's base-2 exponent.
#define DHQ_ACT_KIND_NONE 0
#define DHQ_ACT_KIND_SINE 1
#define DHQ_ACT_KIND_WAVELET 2
// the complex wavelet exp(j omega0 y - |s0 y|^2) on pairs of features (2m, 2m + 1) = (Re y, Im y): the
// WIRE architecture with complex-valued hidden layers, run as a real network of interleaved features
#define DHQ_ACT_KIND_WAVELET_COMPLEX 3
struct dhq_act {
    int kind;
    float c2;
};

// The activation on an argument t = omega0 y / (2 pi) in revolutions (the hardware sine and
// cosine take revolutions; the hardware exponential is base 2).
__device__ __forceinline__ float dhq_activate_rev(float t, dhq_act act)
{
    if (act.kind == DHQ_ACT_KIND_WAVELET) {
        const float g = t * act.c2;
        return __builtin_amdgcn_cosf(t) * __builtin_amdgcn_exp2f(-(g * g));
    }
    return dhq_sin_rev(t);
}

// The complex wavelet on a pair of arguments in revolutions, tr = omega0 Re y / 2 pi, ti = omega0 Im y / 2 pi:
//   exp(j omega0 y - |s0 y|^2) = exp(-omega0 Im y - s0^2 |y|^2) (cos(omega0 Re y) + j sin(omega0 Re y)),
// the envelope as a base-2 exponential: (c2 t)^2 = (s0 y)^2 log2 e as for the real wavelet, and
// omega0 Im y log2 e = 2 pi log2(e) ti.  ANY: take the fractional part of tr first (any finite argument).
template <bool ANY>
__device__ __forceinline__ void dhq_activate_pair_rev(float tr, float ti, float c2, float &ar, float &ai)
{
    const float gr = tr * c2, gi = ti * c2;
    const float e = __builtin_fmaf(gr, gr, __builtin_fmaf(gi, gi, ti * 9.0647202836543876f));
    const float mag = __builtin_amdgcn_exp2f(-e);
    const float f = ANY ? __builtin_amdgcn_fractf(tr) : tr;
    ar = __builtin_amdgcn_cosf(f) * mag;
    ai = __builtin_amdgcn_sinf(f) * mag;
}

// The same for any finite argument: the hardware sine and cosine are defined up to 256
// revolutions, so the fractional part is taken first (one more instruction; the kernels that
// are bound by memory traffic use this form, the whole-network kernels the one above on
// arguments the host has bounded).  The wavelet's envelope needs the whole argument.
__device__ __forceinline__ float dhq_activate_rev_any(float t, dhq_act act)
{
    const float f = __builtin_amdgcn_fractf(t);
    if (act.kind == DHQ_ACT_KIND_WAVELET) {
        const float g = t * act.c2;
        return __builtin_amdgcn_cosf(f) * __builtin_amdgcn_exp2f(-(g * g));
    }
    return __builtin_amdgcn_sinf(f);
}

// Dequantize + bias (+ activation), Sec. 3.3.  For layers with an activation c1 and bias are
// pre-multiplied by omega0 / (2 pi) on the host, so the fused multiply-add yields the argument in
// revolutions.
__device__ __forceinline__ float dhq_epilogue(int acc, float c1, float bias, dhq_act act)
{
    float y = __builtin_fmaf((float)acc, c1, bias);
    return act.kind == DHQ_ACT_KIND_NONE ? y : dhq_activate_rev_any(y, act);
}

// From max |un-normalised x^| of a layer input to the constants of the dynamic mode, in the same
// fp64 steps the host takes when it calibrates (so both give the same bits):
//   inv = 1 / (s_a sqrt(Kp))    the quantizer's multiplier
//   c1  = s_a * c1_over_sa      the epilogue's multiplier (c1_over_sa = s_w [omega0 / 2 pi] [/ sqrt(Mp)])
//   s_a = (float)(max|x^| / qmax), 1 for an all-zero tensor
__device__ __forceinline__ void dhq_dyn_constants(float mx, int Kp, int qmax, double c1_over_sa, float &inv, float &c1,
                                                  float &s_a)
{
    const double amax = (double)mx / sqrt((double)Kp);
    s_a = amax == 0.0 ? 1.0f : (float)(amax / (double)qmax);
    inv = (float)(1.0 / ((double)s_a * sqrt((double)Kp)));
    c1 = (float)((double)s_a * c1_over_sa);
}

#endif
