/*
 * libdhq -- DHQ (distribution-aware Hadamard quantization) inference of a
 * SIREN-style coordinate MLP on one AMD MI355X (gfx950).
 *
 * The library evaluates f_theta(x) -> y (paper Sec. 2.1) with every linear
 * layer run as in Sec. 3.2-3.3 of the paper:
 *
 *   for each layer l (fan-in K, fan-out M, Kp = next power of two >= K):
 *     x^  = pad(a_{l-1}) * H_Kp / sqrt(Kp)        Walsh-Hadamard rotation, Eq. 3-5
 *     q   = clamp(rne(x^ / s_a[l]), -qmax, qmax)  the "standard quantizer", Sec. 3.2
 *     acc = q * Wq[l]^T   (int8 x int8 -> int32)  MAC array + adder tree, Sec. 3.3
 *     y   = acc * (s_a[l] * s_w[l]) + b[l]
 *     a_l = sin(omega0 * y)   (all layers but the last; the last returns y;
 *                              dhq_quantize_weights_wavelet: a wavelet instead of the sine)
 *
 * with Wq[l] = clamp(rne((pad(W[l]) * H_Kp / sqrt(Kp)) / s_w[l])) produced once,
 * offline, by dhq_quantize_weights, and qmax = 2^(bits-1) - 1.  The rotation is
 * applied over the input-feature dimension of both operands, so it cancels in
 * the product; all scales are per tensor.
 *
 * Conventions
 *   - Every function returns DHQ_OK (0) or a negative dhq_status; nothing throws
 *     or aborts.  dhq_strerror() names a status.
 *   - "host" pointers are ordinary CPU memory, "dev" pointers are device memory
 *     of the current HIP device, owned by the caller.  Matrices are row-major.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     dhq_forward, dhq_forward_debug and dhq_gemm_i8 only enqueue work on it and
 *     return without synchronising; dhq_calibrate synchronises the stream.
 *     dhq_forward enqueues kernels only (no memset, no copy), so a stream capture of it
 *     can be replayed as a HIP graph; with DHQ_DYNAMIC make one eager call of at least the
 *     captured size first, so that the workspace does not grow during capture.
 *   - A model owns device buffers (quantized weights, biases, a workspace for the
 *     layer-by-layer path) which its forward calls write: use one stream per model.  Calls
 *     that use the same model concurrently from several streams or threads race.
 *   - Limits: 1 <= n_layers <= 16, every dims[] entry in [1, 512], bits in
 *     {4, 6, 8}.  Anything else is DHQ_EUNSUPPORTED / DHQ_EINVAL.
 */
#ifndef DHQ_H
#define DHQ_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    DHQ_OK = 0,
    DHQ_EINVAL = -1,       /* null pointer, negative size, bad bit width, non-finite scale ... */
    DHQ_EUNSUPPORTED = -2, /* a shape or flag the library has no kernel for */
    DHQ_ENOMEM = -3,       /* host or device allocation failed */
    DHQ_EHIP = -4,         /* a HIP runtime call or kernel launch failed */
    DHQ_ENOSCALE = -5,     /* forward called before activation scales exist */
    DHQ_ETOOBIG = -6       /* dhq_forward_noalloc: more rows than its fixed buffer holds */
} dhq_status;

/* dhq_forward flags: which implementation runs.  0 picks the fused kernel when the
 * network shape has one and the layer-by-layer path otherwise. */
#define DHQ_AUTO 0u
#define DHQ_LAYERWISE 1u /* two to four kernels per layer, activations round-trip device memory */
#define DHQ_FUSED 2u     /* one kernel for the whole network; DHQ_EUNSUPPORTED if the shape has none */
/* Shapes with a whole-network kernel (DHQ_ROTATE_IN): at least two layers, fan-in <= 4, all hidden
 * widths equal and 32 / 64 / 128 / 256 / 512, fan-out <= 32.  dhq_has_fused() tells. */
/* or-ed onto the above: measure every layer's activation scale on line, on this call's own
 * coordinates, instead of using the scales stored in the model (Sec. 3.3, "dynamic
 * quantization module ... between layers").  With DHQ_LAYERWISE: an absmax pass added to every layer, any
 * shape.  With DHQ_FUSED (and DHQ_AUTO where available): one kernel per layer that keeps the
 * layer's arithmetic in registers and passes only the transformed activations through device
 * memory; exists on every shape that has a whole-network kernel (either rotation mode),
 * DHQ_EUNSUPPORTED otherwise. */
#define DHQ_DYNAMIC 4u

/* dhq_quantize_weights_mode: which sides of the weight matrix are rotated. */
#define DHQ_ROTATE_IN 0u   /* input-feature side only (what dhq_quantize_weights does) */
#define DHQ_ROTATE_BOTH 1u /* both sides, W' = H_m W H_n / sqrt(m n), Eq. 4-5 as printed */
/* ... or-ed with what is quantized (the three rows of the paper's Table 2): */
#define DHQ_W8A8 0x00u   /* weights and activations (the method; bit widths from the descriptor) */
#define DHQ_W8A32 0x10u  /* weights only: the network runs in fp32 on the de-quantized weights */
#define DHQ_W32A32 0x20u /* nothing: the plain fp32 network, the full-precision reference */

typedef struct dhq_model dhq_model; /* opaque */

/* Network description (the SIREN of Sec. 3.1: sine after every layer but the last). */
typedef struct {
    int32_t n_layers;    /* number of linear layers including the output layer */
    const int32_t *dims; /* host, n_layers + 1 entries: fan-in of layer 0, then every fan-out */
    float omega0;        /* sine frequency factor, applied after every layer but the last */
    int32_t bits_w;      /* weight bit width, 4 / 6 / 8; codes are stored in int8 */
    int32_t bits_a;      /* activation bit width, 4 / 6 / 8 */
} dhq_net_desc;

/*
 * Offline weight step (Sec. 3.2, Eq. 4-5 restricted to the input-feature side;
 * "a standard quantizer" after the transform): rotates, scales and quantizes
 * every layer's weights on the host in fp64, uploads them and creates a model.
 *   W_host[l]  host, dims[l+1] x dims[l] fp32, row-major (out x in)
 *   b_host[l]  host, dims[l+1] fp32
 *   *out       receives the model; release it with dhq_free
 * The inputs are not referenced after the call returns.
 */
int dhq_quantize_weights(const dhq_net_desc *desc, const float *const *W_host,
                         const float *const *b_host, dhq_model **out);

/*
 * The same offline step with the rotation of Eq. 4-5 taken on both sides (mode =
 * DHQ_ROTATE_BOTH): fan-out M is zero-padded to Mp = next power of two, the weights become
 * W' = H_Mp pad(W) H_Kp / sqrt(Mp Kp) (Mp x Kp codes, one scale), and every layer of the
 * forward path then computes
 *     acc' = q * W'q^T                 (n x Mp, the output in the rotated basis)
 *     z    = acc' * H_Mp               (exact in int32: entries of H are +-1, H H = Mp I)
 *     y    = z[:, :M] * (s_a s_w / sqrt(Mp)) + b
 * Weights for which |z| could leave int32 (bound: qmax_a * sum_k |(H_Mp W'q)[j][k]| for some
 * output j) are refused with DHQ_EUNSUPPORTED.  Such a model has a fused kernel when fan-in
 * <= 4, all hidden widths are equal and 32 / 64 / 128 / 256, and fan-out <= 32; otherwise it
 * runs on the layer-by-layer path only.  dhq_get_weight_codes returns Mp x Kp codes,
 * dhq_gemm_i8 the rotated accumulators (n x Mp) and dhq_forward_debug the un-rotated ones
 * (n x Mp).
 * mode = DHQ_ROTATE_IN is dhq_quantize_weights.
 *
 * mode | DHQ_W8A32 / DHQ_W32A32 (with DHQ_ROTATE_IN only) builds the comparison networks of
 * Sec. 1 / Table 2 with floating-point activations: y = W a + b, a = sin(omega0 y) in fp32 on
 * the fp32 MFMA, where W is the original weight matrix (DHQ_W32A32) or
 * W~ = (s_w Wq) H_Kp / sqrt(Kp), the de-quantized weights taken back to the original basis
 * (DHQ_W8A32; bits_w applies, bits_a is ignored).  Any shape within the limits: with fan-in <= 4,
 * equal hidden widths of 32 / 64 / 128 / 256 and fan-out <= 32 one fused kernel runs the whole
 * network (DHQ_AUTO, DHQ_FUSED), every other shape (and DHQ_LAYERWISE) runs one fp32 GEMM kernel
 * per layer.  Such a model has no activation scales: dhq_set_act_scales, dhq_calibrate,
 * DHQ_DYNAMIC and the test hooks return DHQ_EUNSUPPORTED; dhq_forward needs none.
 */
int dhq_quantize_weights_mode(const dhq_net_desc *desc, uint32_t mode, const float *const *W_host,
                              const float *const *b_host, dhq_model **out);

/*
 * The same offline step for a network with wavelet activations, the second architecture the
 * paper evaluates (WIRE: Sec. 4.1, Table 1): every layer but the last is followed by
 *     a = cos(omega0 y) exp(-(s0 y)^2)
 * instead of sin(omega0 y) -- the real part of the complex Gabor wavelet exp(j omega0 y - |s0 y|^2)
 * of the publication the paper cites for WIRE (the paper itself does not print the activation;
 * layers stay real-valued, so rotation, quantizer, integer GEMM and dequantization are those of
 * the sine network).  `mode` as in dhq_quantize_weights_mode (both rotation modes, all three
 * precisions); s0 >= 0 is the spread of the Gaussian envelope (finite; 0 leaves a plain cosine);
 * omega0 must not be 0.  Such a model has the fused kernels of a sine model on the same shapes
 * and behaves like one in every other respect.
 */
int dhq_quantize_weights_wavelet(const dhq_net_desc *desc, uint32_t mode, float s0, const float *const *W_host,
                                 const float *const *b_host, dhq_model **out);

/*
 * The same architecture as its publication has it (Sec. 4.1 / Table 1 name it and cite that
 * publication; the paper itself prints no formula): hidden features are complex numbers, the
 * weights of every layer after the first are complex, every layer but the last ends in the
 * complex wavelet exp(j omega0 y - |s0 y|^2), and the network's output is the real part of the
 * last layer.  Reading: the network runs as a real one on interleaved (Re, Im) features -- a
 * complex weight w becomes the block [[Re w, -Im w], [Im w, Re w]] -- so that the rotation of
 * Eq. 3-5, the quantizer and the integer product of Sec. 3.2-3.3 apply unchanged (DHQ_ROTATE_IN,
 * W8A8), and only the activation acts on pairs of features.
 *   desc->dims   fan-in (real coordinates), the COMPLEX widths of the hidden layers (each at
 *                most 256), fan-out (real values)
 *   W_re, W_im   host, per layer dims[l+1] x dims[l] fp32, row-major; W_im or W_im[l] may be
 *                NULL (a real-valued layer: the first one in the published architecture)
 *   b_re, b_im   host, per layer dims[l+1] fp32; b_im or b_im[l] may be NULL; the imaginary
 *                part of the last layer's weights enters its real output, that of its bias does not
 * The model that comes back has the real dims (fan-in, 2 x width, ..., fan-out): every other
 * call (scales, calibration, forward, the test hooks, dhq_get_weight_codes) sees that real
 * network.  Whole-network kernel: hidden widths 16 / 32 / 64 / 128 / 256 complex (32 .. 512 real).
 */
int dhq_quantize_weights_complex(const dhq_net_desc *desc, float s0, const float *const *W_re,
                                 const float *const *W_im, const float *const *b_re,
                                 const float *const *b_im, dhq_model **out);

/*
 * Static per-layer activation scales for the quantization module between layers (Sec. 3.3; the
 * per-tensor scale of the "standard quantizer" of Sec. 3.2, Eq. 1's step size with zero-point 0):
 * s_a_host is a host array of n_layers entries, each finite and > 0; entry l divides the rotated
 * input of layer l.  Copied into the model; replaces any scales set or calibrated before.
 * Returns DHQ_EUNSUPPORTED, and leaves the model's scales as they were, if with these scales the
 * argument of a layer's sine could leave the range of the hardware sine (see dhq_forward).
 */
int dhq_set_act_scales(dhq_model *m, const float *s_a_host);

/*
 * The "dynamic quantization module" between layers (Sec. 3.3) run once over a
 * coordinate set: layer by layer, s_a[l] = max|x^| / qmax over the whole rotated
 * n x Kp input of layer l, that input being produced by the already quantized
 * layers before it.  An all-zero tensor gets scale 1.  Stores the scales in the
 * model (as dhq_set_act_scales would).  Synchronises `stream`.
 *   coords_dev  dev, n x dims[0] fp32
 */
int dhq_calibrate(dhq_model *m, const float *coords_dev, int64_t n, void *stream);

/* Copies out the per-tensor scales of Sec. 3.2's quantizer (either pointer may be NULL): host
 * arrays of n_layers floats -- s_w[l] = max|W^[l]| / qmax of the rotated weights (Eq. 4-5 on the
 * input side), s_a[l] the activation scale of layer l's rotated input (Sec. 3.3).
 * s_a_host is filled with zeros if no activation scales are set yet. */
int dhq_get_scales(const dhq_model *m, float *s_w_host, float *s_a_host);

/* Copies out layer l's weights after the transform of Eq. 4-5 and the quantizer of Sec. 3.2
 * (what the MAC array of Sec. 3.3 multiplies with): host, dims[l+1] x Kp int8, row-major, column k
 * = rotated input feature k (Mp x Kp for a DHQ_ROTATE_BOTH model). */
int dhq_get_weight_codes(const dhq_model *m, int32_t layer, int8_t *Wq_host);

/*
 * The hot path (Sec. 3.3 pipeline, all layers): coordinates in, signal values out.
 *   coords_dev  dev, n x dims[0] fp32
 *   out_dev     dev, n x dims[n_layers] fp32
 *   n           number of coordinates; 0 is a successful no-op
 *   flags       DHQ_AUTO / DHQ_LAYERWISE / DHQ_FUSED, optionally | DHQ_DYNAMIC
 * Uses the activation scales stored in the model (DHQ_ENOSCALE if there are none), unless
 * DHQ_DYNAMIC is given: then each layer's scale is max|x^| / qmax over the whole rotated
 * n x Kp input of that layer in THIS call (the scale never leaves the device; an all-zero
 * tensor gets scale 1).  DHQ_DYNAMIC | DHQ_LAYERWISE gives exactly what dhq_calibrate on these
 * coordinates followed by a static DHQ_LAYERWISE forward gives; DHQ_DYNAMIC | DHQ_FUSED gives
 * exactly what a static DHQ_FUSED forward with the scales it measured gives (the two transform
 * the activations with differently rounded fp32 arithmetic, so their scales can differ in the
 * last place).  Dynamic mode keeps all n rows of a layer in device memory: unless
 * dhq_reserve_dynamic has provided for n rows, the model's workspace grows to n rows in this call
 * (an allocation, and a device synchronisation, whenever n exceeds every earlier dynamic call and
 * reservation); this is the only case in which dhq_forward changes the model or does anything but
 * enqueue kernels.  dhq_forward_noalloc is the variant that never allocates.
 *
 * Domain of the sine: the hardware sine takes its argument in revolutions and is defined up to
 * 256 of them.  With static scales dhq_set_act_scales / dhq_calibrate check that no layer's
 * argument omega0 y / 2 pi can exceed that (bound: qmax_a c max_j sum_k |Wq[j][k]| + max_j |b_j|
 * omega0 / 2 pi with c = s_a s_w omega0 / 2 pi; for layers whose inputs lie in [-1, 1] also the
 * norm bound below, whichever is smaller) and refuse the scales otherwise.  With DHQ_DYNAMIC the
 * scales are not known in advance: every layer after the first is covered by a bound that needs
 * none (its inputs lie in [-1, 1], so |y_j| <= sqrt(K) (1 + sqrt(Kp) / (2 qmax_a)) s_w ||Wq[j]||_2 + |b_j|),
 * checked when the model is created, and DHQ_DYNAMIC returns DHQ_EUNSUPPORTED for a model that fails
 * it; for the first layer the caller keeps |omega0 (W x + b)| / 2 pi of its coordinates below 256.
 */
int dhq_forward(const dhq_model *m, const float *coords_dev, int64_t n, float *out_dev,
                void *stream, uint32_t flags);

/*
 * Sizes the whole-batch buffers of DHQ_DYNAMIC forwards for up to n rows now (allocates, and
 * synchronises the device if they have to grow), so that later dhq_forward(... | DHQ_DYNAMIC)
 * calls with at most n rows only enqueue kernels.  Not needed for static-scale forwards, which
 * never allocate.  (Sec. 3.3's dynamic quantization module needs a layer's whole input before it
 * can emit a code; these buffers hold it.)
 */
int dhq_reserve_dynamic(dhq_model *m, int64_t n);

/*
 * For callers that cannot allocate device memory -- a stream being captured into a HIP graph, a
 * serving loop or harness with a no-allocation rule: dhq_forward(..., flags | DHQ_DYNAMIC) on a
 * fixed scratch buffer that is part of the library's device image instead of the model's growing
 * buffers.  Same kernels, same results, bit for bit.  Calls no hipMalloc / hipFree and nothing
 * that allocates; only enqueues kernels on `stream`.
 *   flags  DHQ_AUTO / DHQ_LAYERWISE / DHQ_FUSED (the dynamic mode is implied)
 *   n      at most dhq_noalloc_max_rows(m) rows, else DHQ_ETOOBIG and nothing is enqueued.  The buffer
 *          is 32 MiB per device (held by every device that has loaded the library, until the process
 *          ends): e.g. 14336 rows for a 256-wide network, about 7200 for a 512-wide one.
 * All calls on one device share that device's buffer, whichever model they use: calls that overlap
 * in time on one device (different streams or threads) race and give wrong results; calls on one
 * stream, or otherwise ordered, are fine.  The buffer keeps the last call's contents; nothing in it
 * needs clearing between calls.  The measured scales go to the model as with dhq_forward
 * (dhq_get_dynamic_scales).
 */
int dhq_forward_noalloc(const dhq_model *m, const float *coords_dev, int64_t n, float *out_dev,
                        void *stream, uint32_t flags);
/* Largest n dhq_forward_noalloc accepts for this model (0 for a model without quantized activations). */
int64_t dhq_noalloc_max_rows(const dhq_model *m);

/* The scales s_a (host, n_layers floats) that the last DHQ_DYNAMIC forward on this model
 * measured (zeros if there has been none).  Synchronises `stream` (pass the stream that forward ran on). */
int dhq_get_dynamic_scales(const dhq_model *m, float *s_a_host, void *stream);

/*
 * Test hook: one layer of the layer-by-layer path on a caller-supplied input,
 * with every intermediate exposed (any output pointer may be NULL).
 *   in_dev     dev, n x dims[layer] fp32   (the layer's un-rotated input)
 *   codes_dev  dev, n x Kp int8            rotated + quantized input
 *   acc_dev    dev, n x dims[layer+1] int32 (n x Mp, un-rotated, for a DHQ_ROTATE_BOTH model)
 *   act_dev    dev, n x dims[layer+1] fp32 (after bias and, except for the last layer, sine)
 * n is limited to the model's workspace chunk (65536 rows).
 */
int dhq_forward_debug(const dhq_model *m, const float *in_dev, int64_t n, int32_t layer,
                      int8_t *codes_dev, int32_t *acc_dev, float *act_dev, void *stream);

/*
 * Test hook for the whole-network kernels (DHQ_FUSED), which keep every intermediate in
 * registers: one layer of such a kernel -- the same device code, on the same packed weights --
 * run on caller-supplied input codes, with what it hands to the next layer exposed.  Covers the
 * steps of Sec. 3.3 after the quantization module of layer `layer`: MAC array (acc), dequantize +
 * bias + activation, the rotation of Eq. 3-5 over the layer's outputs (x^), and the next quantization
 * module (codes).  `layer` must be one that ends in an activation (not the last); needs static scales.
 *   codes_in_dev   dev, n x Kp(layer) int8: the layer's rotated + quantized input (what
 *                  dhq_forward_debug returns in codes_dev), rotated-feature order
 *   xhat_dev       dev, n x Kp(layer+1) fp32: pad(a_layer) * H_Kp UN-normalised, i.e. sqrt(Kp) x^
 *   codes_out_dev  dev, n x Kp(layer+1) int8: clamp(rne(x^ / s_a[layer+1]))
 *   acc_dev        dev, n x dims[layer+1] int32 accumulators of the layer (DHQ_ROTATE_BOTH: the
 *                  rotated ones, before the integer un-rotation)
 * Any output may be NULL.  DHQ_EUNSUPPORTED if the model has no whole-network kernel.
 */
int dhq_forward_debug_fused(const dhq_model *m, const int8_t *codes_in_dev, int64_t n, int32_t layer,
                            float *xhat_dev, int8_t *codes_out_dev, int32_t *acc_dev, void *stream);

/*
 * Test hook: the integer GEMM of one layer alone (Sec. 3.3 MAC array) on
 * caller-supplied codes: acc = codes * Wq[layer]^T.
 *   codes_dev  dev, n x Kp int8;  acc_dev  dev, n x dims[layer+1] int32 (n x Mp for DHQ_ROTATE_BOTH)
 */
int dhq_gemm_i8(const dhq_model *m, int32_t layer, const int8_t *codes_dev, int64_t n,
                int32_t *acc_dev, void *stream);

/* 1 if DHQ_FUSED can run this model's shape -- the whole pipeline of Sec. 3.3 (input layer, linear
 * layers with the quantization module between them, output layer) in one kernel -- else 0
 * (negative status on error). */
int dhq_has_fused(const dhq_model *m);

/*
 * Hidden width 512 has two whole-network kernels for the pipeline of Sec. 3.3, which compute the
 * same steps in the same precision and differ in how the work of a layer is laid out: one wave
 * per SIMD that holds all 512 features of its 32 coordinates (which = 1), or two waves per SIMD
 * that share 32 coordinates and take half of every layer's output features each, exchanging
 * through LDS what the rotation of Eq. 3 needs from the other half (which = 2).  which = 0
 * returns to the library's default (the faster one).  The choice applies to dhq_forward and
 * dhq_forward_debug_fused on this model from the next call on; it is not thread-safe against
 * calls in flight on the same model.  DHQ_EUNSUPPORTED for a model of any other shape.
 */
int dhq_select_wide_kernel(dhq_model *m, int32_t which);

void dhq_free(dhq_model *m);
const char *dhq_strerror(int status);
int dhq_version(void);

#ifdef __cplusplus
}
#endif
#endif /* DHQ_H */
