// Internal declarations shared by the translation units of libdhq (not installed).
#ifndef DHQ_INTERNAL_H
#define DHQ_INTERNAL_H

#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include <vector>

#include "dhq.h"
#include "dhq_device.h"

#define DHQ_MAX_LAYERS 16
#define DHQ_MAX_DIM 512
#define DHQ_CHUNK 65536  // rows per pass of the layer-by-layer path (workspace size)
#define DHQ_MAX_DEVICES 64

// One linear layer as the kernels see it.
struct dhq_layer {
    int K = 0, M = 0;     // fan-in, fan-out
    int Kp = 0;           // next power of two >= K: length of the rotated input
    int Kb = 0;           // number of 32-wide K blocks of the MFMA operand (>= 1; K zero-padded)
    int Mp = 0;           // next power of two >= M (two-sided variant: rows of the rotated weights)
    int Mg = 0;           // rows of the quantized weight matrix = columns the GEMM produces: M, or Mp when two-sided
    int Mt = 0;           // number of 32-row tiles of those rows (zero-padded)
    float s_w = 0.f;      // weight scale
    float s_a = 0.f;      // activation scale (0 = unset)
    int8_t *wq_dev = nullptr;     // Mg x Kp, row-major (rotated index order)
    int8_t *wfrag_dev = nullptr;  // [Mt][Kb][64 lanes][16 B] MFMA A fragments, natural k order
    float *bias_dev = nullptr;    // M, fp32
    float *bias_rev_dev = nullptr;  // M, bias * omega0 / (2 pi): the sine argument in revolutions
    std::vector<int8_t> wq_host;  // copy of the codes for dhq_get_weight_codes
    std::vector<float> bias_host;      // M
    std::vector<float> bias_rev_host;  // M
    // for the range check of the sine's argument: over the outputs j < M of the integer matrix U the
    // epilogue's input is a product with (Wq, or H_Mp Wq when two-sided)
    int64_t sum_abs_max = 0;        // max_j sum_k |U[j][k]|
    double norm2_max = 0.0;         // max_j ||U[j]||_2
    double bias_rev_abs_max = 0.0;  // max_j |bias_rev[j]|
};

struct dhq_fused_plan;  // defined in dhq_fused.hip
struct dhq_wide_plan;   // defined in dhq_fused_wide.hip
struct dhq_float_plan;  // defined in dhq_float.hip
struct dhq_fused2_plan; // defined in dhq_fused_two_sided.hip
struct dhq_pair_plan;   // defined in dhq_fused_pair.hip

struct dhq_model {
    int n_layers = 0;
    int dims[DHQ_MAX_LAYERS + 1] = {0};
    float omega0 = 0.f;
    int act_kind = DHQ_ACT_KIND_SINE;  // what follows every layer but the last: sine or wavelet
    float wavelet_s0 = 0.f;            // spread of the wavelet's Gaussian envelope
    int bits_w = 8, bits_a = 8;
    int qmax_a = 127;
    bool have_scales = false;
    bool rot_out = false;  // two-sided variant: weights also rotated over the output features
    bool fused_sine_ok = true;  // with the current static scales (or fp32 weights) no sine argument can leave the hardware's range
    bool dyn_sine_ok = true;  // scales measured on line cannot push a sine argument out of the hardware's range
    uint32_t precision = 0;  // DHQ_W8A8 / DHQ_W8A32 / DHQ_W32A32
    dhq_layer layer[DHQ_MAX_LAYERS];
    // workspace of the layer-by-layer path: two activation buffers, one code buffer
    float *act0 = nullptr, *act1 = nullptr;  // DHQ_CHUNK x max dim, fp32
    int8_t *codes = nullptr;                 // DHQ_CHUNK x max Kp
    int32_t *acc_ws = nullptr;               // two-sided variant: DHQ_CHUNK x max Mg rotated accumulators
    unsigned *absmax_dev = nullptr;          // one word for calibration
    int max_dim = 0, max_kp = 0, max_mg = 0;
    // dynamic mode (scales measured on line): whole-batch buffers, grown on demand, and per
    // layer one absmax word and three floats {quantizer multiplier, epilogue multiplier, s_a}
    float *dyn_act0 = nullptr, *dyn_act1 = nullptr;
    int8_t *dyn_codes = nullptr;
    int32_t *dyn_acc = nullptr;
    int64_t dyn_rows = 0;
    unsigned *dyn_absmax = nullptr;  // DHQ_MAX_LAYERS absmax words, then 2 x DHQ_ABSMAX_PARTIALS floats of scratch
    float *dyn_params = nullptr;     // DHQ_MAX_LAYERS x 3
    dhq_fused_plan *fused = nullptr;  // hidden width 32..256; null if the shape has no such kernel
    dhq_wide_plan *wide = nullptr;    // hidden width 512, one wave per SIMD
    dhq_pair_plan *pair = nullptr;    // hidden width 512, two waves per SIMD that split the features
    int wide_kernel = 0;              // which of the two runs: 0 the default, 1 one wave, 2 two waves (dhq_select_wide_kernel)
    dhq_float_plan *flt = nullptr;    // floating-point activations (DHQ_W8A32 / DHQ_W32A32)
    dhq_fused2_plan *fused2 = nullptr;  // two-sided variant, hidden width 32..256, fan-out <= 4
    int device = 0;
    unsigned char *scratch = nullptr;  // this device's copy of the library's fixed scratch buffer (dhq_forward_noalloc)
};

// Raises a kernel's dynamic-LDS limit to `bytes` on `device`, once: the library remembers what it
// has already asked for per kernel and device, so after a kernel's first launch on a device the
// launch path makes no runtime call besides the launch itself (defined in dhq_api.hip).
hipError_t dhq_lds_limit_once_impl(const void *kern, size_t bytes, int device);
template <typename Kern>
static inline hipError_t dhq_lds_limit_once(Kern kern, size_t bytes, int device)
{
    return dhq_lds_limit_once_impl((const void *)kern, bytes, device);
}

// ---- launchers (defined in dhq_layerwise.hip) --------------------------------------------
// Rotate rows over K (zero-padded to Kp) and quantize: codes = clamp(rne(x^ * inv)).
// inv = 1 / (s_a * sqrt(Kp)) because the butterflies run un-normalised.
// Dynamic mode (fold != nullptr): inv is ignored; the kernel folds the `count` per-workgroup maxima that
// dhq_launch_wht_absmax_partials left in `partial` into max |x^| and derives the layer's constants from it,
// and stores dyn_out[0..2] = {1 / (s_a sqrt(Kp)), s_a * c1_over_sa, s_a} for the kernels that follow.
struct dhq_wht_fold {
    const float *partial;
    int count;
    double c1_over_sa;
    float *dyn_out;
};
hipError_t dhq_launch_wht_quant(const float *in, int64_t n, int K, int Kp, float inv, int qmax, int8_t *codes,
                                const dhq_wht_fold *fold, hipStream_t st);

// The same rotation, reduced to max |un-normalised x^| over all rows: *absmax_bits (float bits;
// cleared by the caller before the first of several calls that are to accumulate) is raised to
// that maximum.  `partial` is scratch for DHQ_ABSMAX_PARTIALS floats.  If dyn != nullptr, also
// dyn[0..2] = {1 / (s_a sqrt(Kp)), s_a * c1_over_sa, s_a} with s_a = (float)(max|x^| / qmax)
// (1 if the tensor is all zero).  Two launches.
#define DHQ_ABSMAX_PARTIALS 2048
hipError_t dhq_launch_wht_absmax(const float *in, int64_t n, int K, int Kp, unsigned *absmax_bits, float *partial,
                                 int qmax, double c1_over_sa, float *dyn, hipStream_t st);

// acc = codes * Wq^T.  Exactly one of acc_out / act_out is written:
//   acc_out  n x Mg int32
//   act_out  n x Mg fp32 = activation(acc * c1 + bias[f]) (sine or wavelet of an argument in revolutions, or none)
// If dyn != nullptr, c1 is read from dyn[1] on the device.
hipError_t dhq_launch_gemm(const dhq_layer &L, const int8_t *codes, int64_t n, int32_t *acc_out,
                           float *act_out, float c1, const float *bias, dhq_act act, const float *dyn, hipStream_t st);

// Two-sided variant: z = acc H_Mp (int32, n x Mp) and act[:, f < M] = epilogue(z, c1, bias).
// Either output may be null.  If dyn != nullptr, c1 is read from dyn[1].
hipError_t dhq_launch_unrotate(const int32_t *acc, int64_t n, int Mp, int M, float c1, const float *bias, dhq_act act,
                               const float *dyn, int32_t *z_out, float *act_out, hipStream_t st);

// Two-sided variant, static scales: un-rotation and epilogue of a layer (sine or wavelet) and, in the same lanes, the
// rotation and quantizer of the next layer (whose rotated length is Mp): codes = n x Mp int8.
hipError_t dhq_launch_unrotate_quant(const int32_t *acc, int64_t n, int Mp, int M, float c1, const float *bias, dhq_act act,
                                     float inv_next, int qmax, int8_t *codes, hipStream_t st);

// The first of the two launches of dhq_launch_wht_absmax only: partial[0 .. *count) holds the
// workgroups' maxima and the caller folds them.
hipError_t dhq_launch_wht_absmax_partials(const float *in, int64_t n, int K, int Kp, float *partial, int *count,
                                          hipStream_t st);

hipError_t dhq_launch_clear_words(unsigned *p, int n, hipStream_t st);

// Epilogue multiplier divided by the activation scale: s_w, times omega0 / (2 pi) in the sine
// layers (the sine takes revolutions), over sqrt(Mp) in the two-sided variant.
static inline double dhq_c1_over_sa(const dhq_model *m, int l)
{
    const dhq_layer &Ly = m->layer[l];
    double c = (double)Ly.s_w;
    if (l != m->n_layers - 1) c = c * (double)m->omega0 / 6.283185307179586476925286766559;
    if (m->rot_out) c = c / sqrt((double)Ly.Mp);
    return c;
}
// The activation after every layer but the last, and after layer l, as the kernels take it.
static inline dhq_act dhq_hidden_act(const dhq_model *m)
{
    dhq_act a;
    a.kind = m->act_kind;
    a.c2 = (a.kind == DHQ_ACT_KIND_WAVELET || a.kind == DHQ_ACT_KIND_WAVELET_COMPLEX)
               ? (float)(6.283185307179586476925286766559 * (double)m->wavelet_s0 * sqrt(1.4426950408889634074) / (double)m->omega0)
               : 0.f;
    return a;
}
static inline dhq_act dhq_layer_act(const dhq_model *m, int l)
{
    return (l == m->n_layers - 1) ? dhq_act{DHQ_ACT_KIND_NONE, 0.f} : dhq_hidden_act(m);
}
static inline float dhq_c1(const dhq_model *m, int l) { return (float)((double)m->layer[l].s_a * dhq_c1_over_sa(m, l)); }

// act_out = epilogue(acc) elementwise, same formula as above.
hipError_t dhq_launch_epilogue(const int32_t *acc, int64_t n, int M, float c1, const float *bias,
                               dhq_act act, float *act_out, hipStream_t st);

// The complex wavelet on the pairs (2p, 2p + 1) of every row of acc (n x M int32, M even): act_out = n x M fp32.
// If dyn != nullptr, c1 is read from dyn[1].
hipError_t dhq_launch_epilogue_pairs(const int32_t *acc, int64_t n, int M, float c1, const float *bias, dhq_act act,
                                     const float *dyn, float *act_out, hipStream_t st);

// ---- fused path (defined in dhq_fused.hip) -------------------------------------------------
// Builds the packed weights for the whole-network kernel if the shape is supported.
// Returns DHQ_OK with *plan == nullptr when it is not.
int dhq_fused_create(const dhq_model *m, dhq_fused_plan **plan);
void dhq_fused_destroy(dhq_fused_plan *plan);
// Refreshes the per-layer constants after the activation scales changed.
int dhq_fused_update_scales(const dhq_model *m, dhq_fused_plan *plan);
hipError_t dhq_fused_launch(const dhq_model *m, const float *coords, int64_t n, float *out,
                            hipStream_t st);
// Dynamic mode, one launch per layer with the transformed activations passing through ws0 / ws1
// (dhq_fused_dynamic_rows(n) x hidden width floats each); partial: 2 x DHQ_ABSMAX_PARTIALS floats of
// scratch; dyn: three floats per layer.
size_t dhq_fused_dynamic_rows(int64_t n);
hipError_t dhq_fused_dynamic_launch(const dhq_model *m, const float *coords, int64_t n, float *out, float *ws0, float *ws1,
                                    float *partial, float *dyn, hipStream_t st);


// Hidden width 512 (defined in dhq_fused_wide.hip); same contract as the functions above.
int dhq_wide_create(const dhq_model *m, dhq_wide_plan **plan);
void dhq_wide_destroy(dhq_wide_plan *plan);
int dhq_wide_update_scales(const dhq_model *m, dhq_wide_plan *plan);
hipError_t dhq_wide_launch(const dhq_wide_plan *plan, const float *coords, int64_t n, float *out, hipStream_t st);


// Hidden width 512 on two waves per SIMD (defined in dhq_fused_pair.hip); same contract.
int dhq_pair_create(const dhq_model *m, dhq_pair_plan **plan);
void dhq_pair_destroy(dhq_pair_plan *plan);
int dhq_pair_update_scales(const dhq_model *m, dhq_pair_plan *plan);
hipError_t dhq_pair_launch(const dhq_pair_plan *plan, const float *coords, int64_t n, float *out, hipStream_t st);
// Dynamic mode at this width, one launch per layer (same contract as dhq_fused_dynamic_launch; ws0 / ws1:
// dhq_pair_dynamic_rows(n) x 512 floats each).
size_t dhq_pair_dynamic_rows(int64_t n);
hipError_t dhq_pair_dynamic_launch(const dhq_model *m, const float *coords, int64_t n, float *out, float *ws0, float *ws1,
                                   float *partial, float *dyn, hipStream_t st);
// Which width-512 kernel a model runs at the moment.
#define DHQ_WIDE_DEFAULT_TWO_WAVES 1
static inline bool dhq_use_pair(const dhq_model *m)
{
    if (!m->pair) return false;
    if (!m->wide) return true;
    return m->wide_kernel == 2 || (m->wide_kernel == 0 && DHQ_WIDE_DEFAULT_TWO_WAVES);
}

// Two-sided variant, whole network in one kernel (defined in dhq_fused_two_sided.hip); same
// contract as the dhq_fused_* functions.
int dhq_fused2_create(const dhq_model *m, dhq_fused2_plan **plan);
void dhq_fused2_destroy(dhq_fused2_plan *plan);
int dhq_fused2_update_scales(const dhq_model *m, dhq_fused2_plan *plan);
hipError_t dhq_fused2_launch(const dhq_fused2_plan *plan, const float *coords, int64_t n, float *out, hipStream_t st);
size_t dhq_fused2_dynamic_rows(int64_t n);
hipError_t dhq_fused2_dynamic_launch(const dhq_model *m, const float *coords, int64_t n, float *out, float *ws0, float *ws1,
                                     float *partial, float *dyn, hipStream_t st);

// Test hooks: layer `layer` (one that ends in an activation) of a whole-network kernel on the
// caller's input codes (n x Kp int8, rotated-feature order).  Outputs, each n x hidden width,
// row-major in rotated-feature order, any may be null: the un-normalised transform x^ of the
// layer's output, the codes the next layer's quantizer makes of it, the layer's int32 accumulators
// (two-sided: the rotated ones).
hipError_t dhq_fused_debug_launch(const dhq_model *m, int layer, const int8_t *codes_in, int64_t n, float *xhat, int8_t *codes_out,
                                  int32_t *acc, hipStream_t st);
hipError_t dhq_wide_debug_launch(const dhq_model *m, int layer, const int8_t *codes_in, int64_t n, float *xhat, int8_t *codes_out,
                                 int32_t *acc, hipStream_t st);
hipError_t dhq_pair_debug_launch(const dhq_model *m, int layer, const int8_t *codes_in, int64_t n, float *xhat, int8_t *codes_out,
                                 int32_t *acc, hipStream_t st);
hipError_t dhq_fused2_debug_launch(const dhq_model *m, int layer, const int8_t *codes_in, int64_t n, float *xhat, int8_t *codes_out,
                                   int32_t *acc, hipStream_t st);

// Floating-point activations (defined in dhq_float.hip): the plain network (sine, or the wavelet `act`) on the given fp32
// weights W[l] (dims[l+1] x dims[l]) and biases.  Every shape has the layer-by-layer path
// (dhq_float_launch_layerwise); the shapes dhq_float_shape_ok accepts also have one kernel fused
// over all layers (dhq_float_launch; dhq_float_has_fused tells).
bool dhq_float_shape_ok(const int *dims, int n_layers);
int dhq_float_create(const int *dims, int n_layers, float omega0, dhq_act act, const std::vector<std::vector<float>> &W,
                     const std::vector<std::vector<float>> &b, int device, dhq_float_plan **plan);
void dhq_float_destroy(dhq_float_plan *plan);
hipError_t dhq_float_launch(const dhq_float_plan *plan, const float *coords, int64_t n, float *out, hipStream_t st);
bool dhq_float_has_fused(const dhq_float_plan *plan);
hipError_t dhq_float_launch_layerwise(const dhq_float_plan *plan, const float *coords, int64_t n, float *out, hipStream_t st);

#endif
