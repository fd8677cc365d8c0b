// Internal declarations shared by the translation units of libdhq (not installed).
#ifndef DHQ_INTERNAL_H
#define DHQ_INTERNAL_H

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <vector>

#include "dhq.h"

#define DHQ_MAX_LAYERS 16
#define DHQ_MAX_DIM 512
#define DHQ_CHUNK 65536  // rows per pass of the layer-by-layer path (workspace size)

// One linear layer as the kernels see it.
struct dhq_layer {
    int K = 0, M = 0;     // fan-in, fan-out
    int Kp = 0;           // next power of two >= K: length of the rotated input
    int Kb = 0;           // number of 32-wide K blocks of the MFMA operand (>= 1; K zero-padded)
    int Mt = 0;           // number of 32-row M tiles (rows zero-padded)
    float s_w = 0.f;      // weight scale
    float s_a = 0.f;      // activation scale (0 = unset)
    int8_t *wq_dev = nullptr;     // M x Kp, row-major (rotated index order)
    int8_t *wfrag_dev = nullptr;  // [Mt][Kb][64 lanes][16 B] MFMA A fragments, natural k order
    float *bias_dev = nullptr;    // M, fp32
    float *bias_rev_dev = nullptr;  // M, bias * omega0 / (2 pi): the sine argument in revolutions
    std::vector<int8_t> wq_host;  // copy of the codes for dhq_get_weight_codes
    std::vector<float> bias_host;      // M
    std::vector<float> bias_rev_host;  // M
};

struct dhq_fused_plan;  // defined in dhq_fused.hip
struct dhq_wide_plan;   // defined in dhq_fused_wide.hip

struct dhq_model {
    int n_layers = 0;
    int dims[DHQ_MAX_LAYERS + 1] = {0};
    float omega0 = 0.f;
    int bits_w = 8, bits_a = 8;
    int qmax_a = 127;
    bool have_scales = false;
    dhq_layer layer[DHQ_MAX_LAYERS];
    // workspace of the layer-by-layer path: two activation buffers, one code buffer
    float *act0 = nullptr, *act1 = nullptr;  // DHQ_CHUNK x max dim, fp32
    int8_t *codes = nullptr;                 // DHQ_CHUNK x max Kp
    unsigned *absmax_dev = nullptr;          // one word for calibration
    int max_dim = 0, max_kp = 0;
    dhq_fused_plan *fused = nullptr;  // hidden width 32..256; null if the shape has no such kernel
    dhq_wide_plan *wide = nullptr;    // hidden width 512
    int device = 0;
};

// ---- launchers (defined in dhq_layerwise.hip) --------------------------------------------
// Rotate rows over K (zero-padded to Kp) and quantize: codes = clamp(rne(x^ * inv)).
// inv = 1 / (s_a * sqrt(Kp)) because the butterflies run un-normalised.
// If absmax_bits != nullptr the kernel instead records max |un-normalised x^| (as float bits)
// with atomicMax and writes no codes.
hipError_t dhq_launch_wht_quant(const float *in, int64_t n, int K, int Kp, float inv, int qmax,
                                int8_t *codes, unsigned *absmax_bits, hipStream_t st);

// acc = codes * Wq^T.  Exactly one of acc_out / act_out is written:
//   acc_out  n x M int32
//   act_out  n x M fp32 = sine ? sin(2 pi (acc * c1 + bias[f])) : acc * c1 + bias[f]
hipError_t dhq_launch_gemm(const dhq_layer &L, const int8_t *codes, int64_t n, int32_t *acc_out,
                           float *act_out, float c1, const float *bias, bool sine, hipStream_t st);

// act = epilogue(acc) elementwise, same formula as above.
hipError_t dhq_launch_epilogue(const int32_t *acc, int64_t n, int M, float c1, const float *bias,
                               bool sine, float *act, hipStream_t st);

// ---- fused path (defined in dhq_fused.hip) -------------------------------------------------
// Builds the packed weights for the whole-network kernel if the shape is supported.
// Returns DHQ_OK with *plan == nullptr when it is not.
int dhq_fused_create(const dhq_model *m, dhq_fused_plan **plan);
void dhq_fused_destroy(dhq_fused_plan *plan);
// Refreshes the per-layer constants after the activation scales changed.
int dhq_fused_update_scales(const dhq_model *m, dhq_fused_plan *plan);
hipError_t dhq_fused_launch(const dhq_model *m, const float *coords, int64_t n, float *out,
                            hipStream_t st);


// Hidden width 512 (defined in dhq_fused_wide.hip); same contract as the functions above.
int dhq_wide_create(const dhq_model *m, dhq_wide_plan **plan);
void dhq_wide_destroy(dhq_wide_plan *plan);
int dhq_wide_update_scales(const dhq_model *m, dhq_wide_plan *plan);
hipError_t dhq_wide_launch(const dhq_wide_plan *plan, const float *coords, int64_t n, float *out, hipStream_t st);

#endif
