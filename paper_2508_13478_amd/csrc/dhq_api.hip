// Host side of libdhq: the C ABI of include/dhq.h.
//
//   dhq_quantize_weights  offline rotation (fast Walsh-Hadamard transform in fp64 over the
//   (_mode)               input-feature side, or over both sides as Eq. 4-5 print it) +
//                         per-tensor symmetric quantizer
//   dhq_calibrate         per-layer activation scales measured on a coordinate set
//   dhq_forward           layer-by-layer or fused whole-network evaluation; with DHQ_DYNAMIC
//                         the scales are measured on line, per call
//   dhq_forward_debug / dhq_gemm_i8   test hooks exposing one layer's intermediates
#include <math.h>
#include <string.h>

#include <new>
#include <vector>

#include "dhq_internal.h"

#define DHQ_VERSION_NUM 200
#define DHQ_SINE_MAX_REV 256.0  // the hardware sine and cosine are defined up to this many revolutions

// What dhq_lds_limit_once has already set: (kernel, device) -> bytes.  A fixed table searched
// linearly (the library has a few dozen kernel instances); when it is full the attribute is
// simply set again on every call.  Entries are only ever added, by whole-word stores, so
// concurrent callers at worst set an attribute twice.
#define DHQ_LDS_TABLE 256
static struct { const void *kern; int device; int bytes; } lds_table[DHQ_LDS_TABLE];
static int lds_table_used = 0;

hipError_t dhq_lds_limit_once_impl(const void *kern, size_t bytes, int device)
{
    const int used = lds_table_used;
    int slot = -1;
    for (int i = 0; i < used; ++i)
        if (lds_table[i].kern == kern && lds_table[i].device == device) {
            if ((size_t)lds_table[i].bytes >= bytes) return hipSuccess;
            slot = i;
            break;
        }
    const hipError_t e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e != hipSuccess) return e;
    if (slot < 0 && used < DHQ_LDS_TABLE) {
        slot = used;
        lds_table[slot].kern = kern;
        lds_table[slot].device = device;
        lds_table[slot].bytes = 0;
        lds_table_used = used + 1;
    }
    if (slot >= 0) lds_table[slot].bytes = (int)bytes;
    return hipSuccess;
}

// ---- the fixed scratch buffer of dhq_forward_noalloc ------------------------------------------
// dhq_forward with DHQ_DYNAMIC keeps whole-batch buffers in the model and grows them with
// hipMalloc when a call brings more rows than any before.  Callers that cannot allocate (a
// stream being captured into a graph, a serving loop with a no-allocation rule) get the same
// computation on a fixed buffer that is part of the library's device image: every device that
// loads the library holds DHQ_NOALLOC_SCRATCH_BYTES of it until the process ends.  In host code
// `scratch` is only a handle for the symbol; its device address is looked up once per device
// (scratch_on_device, called when a model is created on that device) and only that pointer is
// ever handed to kernels.
#define DHQ_NOALLOC_SCRATCH_BYTES ((size_t)32 << 20)
#define DHQ_NOALLOC_PARTIAL_BYTES ((size_t)2 * DHQ_ABSMAX_PARTIALS * sizeof(float))
static __device__ __align__(256) unsigned char scratch[DHQ_NOALLOC_SCRATCH_BYTES + DHQ_NOALLOC_PARTIAL_BYTES];
static unsigned char *scratch_dev_ptr[DHQ_MAX_DEVICES];

// The device address of `scratch` on `device`, which must be the current device.
static int scratch_on_device(int device, unsigned char **ptr)
{
    if (device < 0 || device >= DHQ_MAX_DEVICES) return DHQ_EUNSUPPORTED;
    if (!scratch_dev_ptr[device]) {
        unsigned char *p = nullptr;
        if (hipGetSymbolAddress((void **)&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return DHQ_EHIP;
        scratch_dev_ptr[device] = p;
    }
    *ptr = scratch_dev_ptr[device];
    return DHQ_OK;
}

static size_t round256(size_t b) { return (b + 255) / 256 * 256; }

static int next_pow2(int k)
{
    int p = 1;
    while (p < k) p <<= 1;
    return p;
}

static bool bits_ok(int b) { return b == 4 || b == 6 || b == 8; }

// In-place un-normalised fast Walsh-Hadamard transform of n = 2^k doubles
// (butterflies over the index bits from the lowest up).
static void fwht_f64(double *v, int n)
{
    for (int h = 1; h < n; h <<= 1)
        for (int i = 0; i < n; i += 2 * h)
            for (int j = i; j < i + h; ++j) {
                const double a = v[j], b = v[j + h];
                v[j] = a + b;
                v[j + h] = a - b;
            }
}

// The same transform down a column of a row-major matrix (stride = row length), on doubles
// or on 64-bit integers.
template <typename T>
static void fwht_strided(T *v, int n, size_t stride)
{
    for (int h = 1; h < n; h <<= 1)
        for (int i = 0; i < n; i += 2 * h)
            for (int j = i; j < i + h; ++j) {
                const T a = v[(size_t)j * stride], b = v[(size_t)(j + h) * stride];
                v[(size_t)j * stride] = a + b;
                v[(size_t)(j + h) * stride] = a - b;
            }
}

static void free_layer(dhq_layer &L)
{
    if (L.wq_dev) (void)hipFree(L.wq_dev);
    if (L.wfrag_dev) (void)hipFree(L.wfrag_dev);
    if (L.bias_dev) (void)hipFree(L.bias_dev);
    if (L.bias_rev_dev) (void)hipFree(L.bias_rev_dev);
    L.wq_dev = L.wfrag_dev = nullptr;
    L.bias_dev = L.bias_rev_dev = nullptr;
}

extern "C" void dhq_free(dhq_model *m)
{
    if (!m) return;
    for (int l = 0; l < m->n_layers; ++l) free_layer(m->layer[l]);
    if (m->act0) (void)hipFree(m->act0);
    if (m->act1) (void)hipFree(m->act1);
    if (m->codes) (void)hipFree(m->codes);
    if (m->absmax_dev) (void)hipFree(m->absmax_dev);
    if (m->acc_ws) (void)hipFree(m->acc_ws);
    if (m->dyn_act0) (void)hipFree(m->dyn_act0);
    if (m->dyn_act1) (void)hipFree(m->dyn_act1);
    if (m->dyn_codes) (void)hipFree(m->dyn_codes);
    if (m->dyn_acc) (void)hipFree(m->dyn_acc);
    if (m->dyn_absmax) (void)hipFree(m->dyn_absmax);
    if (m->dyn_params) (void)hipFree(m->dyn_params);
    dhq_fused_destroy(m->fused);
    dhq_wide_destroy(m->wide);
    dhq_pair_destroy(m->pair);
    dhq_float_destroy(m->flt);
    dhq_fused2_destroy(m->fused2);
    delete m;
}

extern "C" const char *dhq_strerror(int status)
{
    switch (status) {
        case DHQ_OK: return "ok";
        case DHQ_EINVAL: return "invalid argument";
        case DHQ_EUNSUPPORTED: return "unsupported shape or flag";
        case DHQ_ENOMEM: return "out of memory";
        case DHQ_EHIP: return "HIP runtime error";
        case DHQ_ENOSCALE: return "activation scales not set";
        case DHQ_ETOOBIG: return "input larger than the fixed buffer of the non-allocating entry point";
        default: return "unknown status";
    }
}

extern "C" int dhq_version(void) { return DHQ_VERSION_NUM; }

template <typename T>
static int upload(T **dst, const T *src, size_t count)
{
    if (hipMalloc((void **)dst, sizeof(T) * (count ? count : 1)) != hipSuccess) {
        *dst = nullptr;
        return DHQ_ENOMEM;
    }
    if (count && hipMemcpy(*dst, src, sizeof(T) * count, hipMemcpyHostToDevice) != hipSuccess) return DHQ_EHIP;
    return DHQ_OK;
}

// Host-only part of the offline step for one layer: rotation, scale, codes, overflow check.
static int quantize_layer_host(dhq_model *m, int l, const float *W, const float *b)
{
    dhq_layer &Ly = m->layer[l];
    Ly.K = m->dims[l];
    Ly.M = m->dims[l + 1];
    Ly.Kp = next_pow2(Ly.K);
    Ly.Kb = (Ly.Kp + 31) / 32;
    Ly.Mp = next_pow2(Ly.M);
    Ly.Mg = m->rot_out ? Ly.Mp : Ly.M;
    Ly.Mt = (Ly.Mg + 31) / 32;
    const int K = Ly.K, M = Ly.M, Kp = Ly.Kp, Mg = Ly.Mg;
    const double qmax_w = (double)((1 << (m->bits_w - 1)) - 1);
    // W^ = pad(W) H_Kp / sqrt(Kp) over the input features of every row; in the two-sided variant
    // also H_Mp / sqrt(Mp) over the (zero-padded) output features: W' = H_Mp pad(W) H_Kp / sqrt(Mp Kp)
    std::vector<double> rot((size_t)Mg * Kp, 0.0);
    for (int r = 0; r < M; ++r) {
        double *row = rot.data() + (size_t)r * Kp;
        for (int k = 0; k < K; ++k) {
            const float w = W[(size_t)r * K + k];
            if (!isfinite(w)) return DHQ_EINVAL;
            row[k] = (double)w;
        }
        fwht_f64(row, Kp);
    }
    if (m->rot_out)
        for (int k = 0; k < Kp; ++k) fwht_strided(rot.data() + k, Mg, (size_t)Kp);
    const double inv = m->rot_out ? 1.0 / sqrt((double)Mg * (double)Kp) : 1.0 / sqrt((double)Kp);
    double amax = 0.0;
    for (size_t i = 0; i < rot.size(); ++i) {
        rot[i] *= inv;
        const double a = fabs(rot[i]);
        if (a > amax) amax = a;
    }
    Ly.s_w = amax == 0.0 ? 1.0f : (float)(amax / qmax_w);
    // the quantizer: clamp(rne(w^ / s_w)); nearbyint rounds half to even
    Ly.wq_host.resize((size_t)Mg * Kp);
    const double sd = (double)Ly.s_w;
    for (size_t i = 0; i < rot.size(); ++i) {
        double q = nearbyint(rot[i] / sd);
        if (q > qmax_w) q = qmax_w;
        if (q < -qmax_w) q = -qmax_w;
        Ly.wq_host[i] = (int8_t)q;
    }
    // U = the integer matrix whose product with the codes is what the epilogue scales: Wq itself, or
    // in the two-sided variant H_Mp Wq (the un-rotation z = acc' H_Mp runs in int32 and
    // z[j] = sum_k q[k] U[j][k]).
    std::vector<int64_t> U(Ly.wq_host.begin(), Ly.wq_host.end());
    if (m->rot_out)
        for (int k = 0; k < Kp; ++k) fwht_strided(U.data() + k, Mg, (size_t)Kp);
    Ly.sum_abs_max = 0;
    Ly.norm2_max = 0.0;
    for (int j = 0; j < Mg; ++j) {
        int64_t sum = 0;
        double sq = 0.0;
        for (int k = 0; k < Kp; ++k) {
            const int64_t u = U[(size_t)j * Kp + k];
            sum += u < 0 ? -u : u;
            sq += (double)u * (double)u;
        }
        // |z[j]| <= qmax_a sum_k |U[j][k]|: refuse weights for which that bound leaves int32
        if (m->rot_out && sum * (int64_t)m->qmax_a > (int64_t)INT32_MAX) return DHQ_EUNSUPPORTED;
        if (j < M) {  // padded outputs are dropped before the activation
            if (sum > Ly.sum_abs_max) Ly.sum_abs_max = sum;
            if (sqrt(sq) > Ly.norm2_max) Ly.norm2_max = sqrt(sq);
        }
    }
    const double two_pi = 6.283185307179586476925286766559;
    Ly.bias_host.assign(b, b + M);
    Ly.bias_rev_host.resize(M);
    Ly.bias_rev_abs_max = 0.0;
    for (int j = 0; j < M; ++j) {
        if (!isfinite(b[j])) return DHQ_EINVAL;
        Ly.bias_rev_host[j] = (float)((double)b[j] * (double)m->omega0 / two_pi);
        if (fabs((double)Ly.bias_rev_host[j]) > Ly.bias_rev_abs_max) Ly.bias_rev_abs_max = fabs((double)Ly.bias_rev_host[j]);
    }
    if (M > m->max_dim) m->max_dim = M;
    if (K > m->max_dim) m->max_dim = K;
    if (Kp > m->max_kp) m->max_kp = Kp;
    if (Mg > m->max_mg) m->max_mg = Mg;
    return DHQ_OK;
}

// Device part: uploads the codes (row-major and as MFMA A fragments) and the biases.
static int upload_layer(dhq_layer &Ly)
{
    const int Kp = Ly.Kp, Mg = Ly.Mg;
    // MFMA A fragments, natural k order: lane (i, u) of (tile T, k block kb) holds
    // Wq[32T + i][32 kb + 16 u .. + 15]
    std::vector<int8_t> frag((size_t)Ly.Mt * Ly.Kb * 1024, 0);
    for (int T = 0; T < Ly.Mt; ++T)
        for (int kb = 0; kb < Ly.Kb; ++kb)
            for (int ln = 0; ln < 64; ++ln) {
                const int row = 32 * T + (ln & 31);
                if (row >= Mg) continue;
                for (int jj = 0; jj < 16; ++jj) {
                    const int k = 32 * kb + 16 * (ln >> 5) + jj;
                    if (k < Kp)
                        frag[((size_t)(T * Ly.Kb + kb) * 64 + ln) * 16 + jj] = Ly.wq_host[(size_t)row * Kp + k];
                }
            }
    int rc = upload(&Ly.wq_dev, Ly.wq_host.data(), Ly.wq_host.size());
    if (rc == DHQ_OK) rc = upload(&Ly.wfrag_dev, frag.data(), frag.size());
    if (rc == DHQ_OK) rc = upload(&Ly.bias_dev, Ly.bias_host.data(), (size_t)Ly.M);
    if (rc == DHQ_OK) rc = upload(&Ly.bias_rev_dev, Ly.bias_rev_host.data(), (size_t)Ly.M);
    return rc;
}

// The hardware sine and cosine take revolutions and are defined for |t| <= 256.  The layer-by-layer
// kernels reduce the argument first (they are bound by memory traffic, the extra instruction is
// free); the whole-network kernels, which are bound by vector instruction issue, do not, and run
// only when the argument provably stays in range.  Upper bounds of
// |t| = |acc c1 + b omega0 / 2 pi| of layer l (one that ends in an activation):
//   by magnitudes: |acc| <= qmax_a max_j sum_k |U[j][k]|;
//   by norms, for layers whose inputs lie in [-1, 1] (every layer after the first): the rotation is
//   orthonormal, so ||x^|| <= sqrt(K); rounding adds at most s_a sqrt(Kp) / 2 to the norm of the
//   de-quantized codes and clamping only shortens it, hence s_a |acc| <= (sqrt(K) + s_a sqrt(Kp) / 2) ||U[j]||.
static double sine_arg_bound(const dhq_model *m, int l, double s_a)
{
    const dhq_layer &Ly = m->layer[l];
    const double c_over = dhq_c1_over_sa(m, l);
    double bound = s_a * c_over * (double)m->qmax_a * (double)Ly.sum_abs_max;
    // (the complex wavelet's modulus exp(-omega0 Im y - |s0 y|^2) is not bounded by 1: magnitudes only)
    if (l >= 1 && m->act_kind != DHQ_ACT_KIND_WAVELET_COMPLEX) {
        const double by_norm = c_over * (sqrt((double)Ly.K) + s_a * sqrt((double)Ly.Kp) / 2.0) * Ly.norm2_max;
        if (by_norm < bound) bound = by_norm;
    }
    return bound + Ly.bias_rev_abs_max;
}
// Static scales: every layer with an activation.
static bool sine_range_ok_static(const dhq_model *m)
{
    for (int l = 0; l < m->n_layers - 1; ++l)
        if (!(sine_arg_bound(m, l, (double)m->layer[l].s_a) <= DHQ_SINE_MAX_REV)) return false;
    return true;
}
// Scales measured on line: s_a = max|x^| / qmax_a <= sqrt(K) / qmax_a for the layers after the first.
static bool sine_range_ok_dynamic(const dhq_model *m)
{
    if (m->act_kind == DHQ_ACT_KIND_WAVELET_COMPLEX && m->n_layers > 2) return false;  // no bound on a layer's input
    for (int l = 1; l < m->n_layers - 1; ++l)
        if (!(sine_arg_bound(m, l, sqrt((double)m->layer[l].K) / (double)m->qmax_a) <= DHQ_SINE_MAX_REV)) return false;
    return true;
}

// The offline step behind every dhq_quantize_weights* entry point; act_kind follows every layer but the last.
static int create_model(const dhq_net_desc *desc, uint32_t mode, int act_kind, float wavelet_s0, const float *const *W_host,
                        const float *const *b_host, dhq_model **out)
{
    if (!desc || !W_host || !b_host || !out || !desc->dims) return DHQ_EINVAL;
    *out = nullptr;
    const uint32_t rotate = mode & 0xfu, precision = mode & 0xf0u;
    if ((mode & ~0xffu) != 0 || (rotate != DHQ_ROTATE_IN && rotate != DHQ_ROTATE_BOTH)) return DHQ_EINVAL;
    if (precision != DHQ_W8A8 && precision != DHQ_W8A32 && precision != DHQ_W32A32) return DHQ_EINVAL;
    if (precision != DHQ_W8A8 && rotate != DHQ_ROTATE_IN) return DHQ_EUNSUPPORTED;
    const bool cplx = (act_kind == DHQ_ACT_KIND_WAVELET_COMPLEX);
    if (cplx && (precision != DHQ_W8A8 || rotate != DHQ_ROTATE_IN)) return DHQ_EUNSUPPORTED;
    const int L = desc->n_layers;
    if (L < 1) return DHQ_EINVAL;
    if (L > DHQ_MAX_LAYERS) return DHQ_EUNSUPPORTED;
    if (!bits_ok(desc->bits_w) || !bits_ok(desc->bits_a)) return DHQ_EINVAL;
    if (!isfinite(desc->omega0)) return DHQ_EINVAL;
    for (int l = 0; l <= L; ++l) {
        if (desc->dims[l] < 1) return DHQ_EINVAL;
        if (desc->dims[l] > DHQ_MAX_DIM) return DHQ_EUNSUPPORTED;
    }
    for (int l = 0; l < L; ++l)
        if (!W_host[l] || !b_host[l]) return DHQ_EINVAL;

    dhq_model *m = new (std::nothrow) dhq_model();
    if (!m) return DHQ_ENOMEM;
    m->n_layers = L;
    for (int l = 0; l <= L; ++l) m->dims[l] = desc->dims[l];
    m->omega0 = desc->omega0;
    m->act_kind = act_kind;
    m->wavelet_s0 = wavelet_s0;
    m->bits_w = desc->bits_w;
    m->bits_a = desc->bits_a;
    m->qmax_a = (1 << (desc->bits_a - 1)) - 1;
    m->rot_out = (rotate == DHQ_ROTATE_BOTH);
    m->precision = precision;
    int rc = DHQ_OK;
    // everything that can be refused is refused before the device is touched
    for (int l = 0; l < L && rc == DHQ_OK; ++l) rc = quantize_layer_host(m, l, W_host[l], b_host[l]);
    if (rc == DHQ_OK) m->dyn_sine_ok = sine_range_ok_dynamic(m);
    if (rc == DHQ_OK && hipGetDevice(&m->device) != hipSuccess) rc = DHQ_EHIP;
    if (rc == DHQ_OK && precision != DHQ_W8A8) {
        // floating-point activations: the network runs on the original weights (W32A32) or on the
        // de-quantized ones in the original basis, W~ = (s_w Wq) H_Kp / sqrt(Kp) (W8A32)
        std::vector<std::vector<float>> Wf(L), bf(L);
        for (int l = 0; l < L; ++l) {
            const dhq_layer &Ly = m->layer[l];
            Wf[l].resize((size_t)Ly.M * Ly.K);
            bf[l] = Ly.bias_host;
            if (precision == DHQ_W32A32) {
                memcpy(Wf[l].data(), W_host[l], sizeof(float) * Wf[l].size());
                continue;
            }
            std::vector<double> row(Ly.Kp);
            const double inv = 1.0 / sqrt((double)Ly.Kp);
            for (int r = 0; r < Ly.M; ++r) {
                for (int k = 0; k < Ly.Kp; ++k) row[k] = (double)Ly.wq_host[(size_t)r * Ly.Kp + k] * (double)Ly.s_w;
                fwht_f64(row.data(), Ly.Kp);
                for (int k = 0; k < Ly.K; ++k) Wf[l][(size_t)r * Ly.K + k] = (float)(row[k] * inv);
            }
        }
        // the sine's argument in revolutions, layers after the first (inputs in [-1, 1]):
        // |t_j| <= (sum_k |W[j][k]| + |b_j|) omega0 / 2 pi; beyond the hardware sine's range only the
        // layer-by-layer kernels (which reduce the argument) may run
        for (int l = 1; l < L - 1; ++l) {
            const dhq_layer &Ly = m->layer[l];
            for (int r = 0; r < Ly.M; ++r) {
                double sum = fabs((double)bf[l][r]);
                for (int k = 0; k < Ly.K; ++k) sum += fabs((double)Wf[l][(size_t)r * Ly.K + k]);
                if (!(sum * fabs((double)m->omega0) / 6.283185307179586476925286766559 <= DHQ_SINE_MAX_REV)) m->fused_sine_ok = false;
            }
        }
        rc = dhq_float_create(m->dims, L, m->omega0, dhq_hidden_act(m), Wf, bf, m->device, &m->flt);
        if (rc != DHQ_OK) {
            dhq_free(m);
            return rc;
        }
        *out = m;
        return DHQ_OK;
    }
    for (int l = 0; l < L && rc == DHQ_OK; ++l) rc = upload_layer(m->layer[l]);
    if (rc == DHQ_OK) {
        const size_t act_bytes = sizeof(float) * (size_t)DHQ_CHUNK * m->max_dim;
        if (hipMalloc((void **)&m->act0, act_bytes) != hipSuccess) rc = DHQ_ENOMEM;
        if (rc == DHQ_OK && hipMalloc((void **)&m->act1, act_bytes) != hipSuccess) rc = DHQ_ENOMEM;
        if (rc == DHQ_OK && hipMalloc((void **)&m->codes, (size_t)DHQ_CHUNK * m->max_kp) != hipSuccess) rc = DHQ_ENOMEM;
        if (rc == DHQ_OK && hipMalloc((void **)&m->absmax_dev, sizeof(unsigned)) != hipSuccess) rc = DHQ_ENOMEM;
        if (rc == DHQ_OK && (m->rot_out || cplx) &&
            hipMalloc((void **)&m->acc_ws, sizeof(int32_t) * (size_t)DHQ_CHUNK * m->max_mg) != hipSuccess)
            rc = DHQ_ENOMEM;
        if (rc == DHQ_OK && hipMalloc((void **)&m->dyn_absmax, sizeof(unsigned) * (DHQ_MAX_LAYERS + 2 * DHQ_ABSMAX_PARTIALS)) != hipSuccess) rc = DHQ_ENOMEM;
        if (rc == DHQ_OK && hipMalloc((void **)&m->dyn_params, sizeof(float) * 3 * DHQ_MAX_LAYERS) != hipSuccess) rc = DHQ_ENOMEM;
        // dhq_get_dynamic_scales before any dynamic forward reports zeros
        if (rc == DHQ_OK && hipMemset(m->dyn_params, 0, sizeof(float) * 3 * DHQ_MAX_LAYERS) != hipSuccess) rc = DHQ_EHIP;
    }
    if (rc == DHQ_OK) rc = scratch_on_device(m->device, &m->scratch);
    if (rc == DHQ_OK && !m->rot_out) rc = dhq_fused_create(m, &m->fused);
    if (rc == DHQ_OK && !m->rot_out && !cplx) rc = dhq_wide_create(m, &m->wide);
    if (rc == DHQ_OK && !m->rot_out) rc = dhq_pair_create(m, &m->pair);  // (also the complex wavelet, which the one-wave kernel does not have)
    if (rc == DHQ_OK && m->rot_out) rc = dhq_fused2_create(m, &m->fused2);
    if (rc != DHQ_OK) {
        dhq_free(m);
        return rc;
    }
    *out = m;
    return DHQ_OK;
}

extern "C" int dhq_quantize_weights_mode(const dhq_net_desc *desc, uint32_t mode, const float *const *W_host,
                                         const float *const *b_host, dhq_model **out)
{
    return create_model(desc, mode, DHQ_ACT_KIND_SINE, 0.f, W_host, b_host, out);
}

extern "C" int dhq_quantize_weights(const dhq_net_desc *desc, const float *const *W_host,
                                    const float *const *b_host, dhq_model **out)
{
    return create_model(desc, DHQ_ROTATE_IN, DHQ_ACT_KIND_SINE, 0.f, W_host, b_host, out);
}

extern "C" int dhq_quantize_weights_wavelet(const dhq_net_desc *desc, uint32_t mode, float s0, const float *const *W_host,
                                            const float *const *b_host, dhq_model **out)
{
    if (out) *out = nullptr;
    if (!isfinite(s0) || s0 < 0.0f) return DHQ_EINVAL;
    // the sine and cosine take omega0 y / 2 pi; the envelope's argument is recovered from it
    if (desc && !(fabsf(desc->omega0) > 0.0f)) return DHQ_EINVAL;
    return create_model(desc, mode, DHQ_ACT_KIND_WAVELET, s0, W_host, b_host, out);
}

// A layer with complex weights as the real layer on interleaved (Re, Im) features:
//   Re (w x) = Re w Re x - Im w Im x,   Im (w x) = Im w Re x + Re w Im x.
// in_c: the inputs are complex (2 K real columns); out_c: so are the outputs (2 M real rows), else the
// output is the real part (M rows).
static void complex_layer_rows(const float *Wre, const float *Wim, const float *bre, const float *bim, int M, int K, bool in_c,
                               bool out_c, std::vector<float> &W, std::vector<float> &b)
{
    const int cols = in_c ? 2 * K : K, rows = out_c ? 2 * M : M;
    W.assign((size_t)rows * cols, 0.f);
    b.assign((size_t)rows, 0.f);
    for (int m = 0; m < M; ++m) {
        const size_t r0 = (size_t)(out_c ? 2 * m : m) * cols, r1 = r0 + cols;
        for (int k = 0; k < K; ++k) {
            const float wr = Wre[(size_t)m * K + k], wi = Wim ? Wim[(size_t)m * K + k] : 0.f;
            const int c0 = in_c ? 2 * k : k;
            W[r0 + c0] = wr;
            if (in_c) W[r0 + c0 + 1] = -wi;
            if (out_c) {
                W[r1 + c0] = wi;
                if (in_c) W[r1 + c0 + 1] = wr;
            }
        }
        b[out_c ? 2 * m : m] = bre[m];
        if (out_c) b[2 * m + 1] = bim ? bim[m] : 0.f;
    }
}

extern "C" int dhq_quantize_weights_complex(const dhq_net_desc *desc, float s0, const float *const *W_re, const float *const *W_im,
                                            const float *const *b_re, const float *const *b_im, dhq_model **out)
{
    if (out) *out = nullptr;
    if (!desc || !desc->dims || !W_re || !b_re || !out) return DHQ_EINVAL;
    if (!isfinite(s0) || s0 < 0.0f || !(fabsf(desc->omega0) > 0.0f)) return DHQ_EINVAL;
    const int L = desc->n_layers;
    if (L < 2) return DHQ_EINVAL;  // without a hidden layer nothing is complex
    if (L > DHQ_MAX_LAYERS) return DHQ_EUNSUPPORTED;
    int32_t dims[DHQ_MAX_LAYERS + 1];
    for (int l = 0; l <= L; ++l) {
        if (desc->dims[l] < 1) return DHQ_EINVAL;
        dims[l] = (l == 0 || l == L) ? desc->dims[l] : 2 * desc->dims[l];
        if (dims[l] > DHQ_MAX_DIM) return DHQ_EUNSUPPORTED;
    }
    std::vector<std::vector<float>> W(L), b(L);
    std::vector<const float *> Wp(L), bp(L);
    for (int l = 0; l < L; ++l) {
        if (!W_re[l] || !b_re[l]) return DHQ_EINVAL;
        complex_layer_rows(W_re[l], W_im ? W_im[l] : nullptr, b_re[l], b_im ? b_im[l] : nullptr, desc->dims[l + 1], desc->dims[l],
                           l > 0, l < L - 1, W[l], b[l]);
        Wp[l] = W[l].data();
        bp[l] = b[l].data();
    }
    dhq_net_desc real = *desc;
    real.dims = dims;
    return create_model(&real, DHQ_ROTATE_IN, DHQ_ACT_KIND_WAVELET_COMPLEX, s0, Wp.data(), bp.data(), out);
}

static int update_fused_scales(dhq_model *m)
{
    m->fused_sine_ok = sine_range_ok_static(m);
    int rc = dhq_fused_update_scales(m, m->fused);
    if (rc == DHQ_OK) rc = dhq_wide_update_scales(m, m->wide);
    if (rc == DHQ_OK) rc = dhq_pair_update_scales(m, m->pair);
    if (rc == DHQ_OK) rc = dhq_fused2_update_scales(m, m->fused2);
    return rc;
}

extern "C" int dhq_set_act_scales(dhq_model *m, const float *s_a_host)
{
    if (!m || !s_a_host) return DHQ_EINVAL;
    if (m->flt) return DHQ_EUNSUPPORTED;  // activations are not quantized in this model
    for (int l = 0; l < m->n_layers; ++l)
        if (!(s_a_host[l] > 0.0f) || !isfinite(s_a_host[l])) return DHQ_EINVAL;
    for (int l = 0; l < m->n_layers; ++l) m->layer[l].s_a = s_a_host[l];
    m->have_scales = true;
    return update_fused_scales(m);
}

extern "C" int dhq_get_scales(const dhq_model *m, float *s_w_host, float *s_a_host)
{
    if (!m) return DHQ_EINVAL;
    for (int l = 0; l < m->n_layers; ++l) {
        if (s_w_host) s_w_host[l] = m->layer[l].s_w;
        if (s_a_host) s_a_host[l] = m->have_scales ? m->layer[l].s_a : 0.0f;
    }
    return DHQ_OK;
}

extern "C" int dhq_get_weight_codes(const dhq_model *m, int32_t layer, int8_t *Wq_host)
{
    if (!m || !Wq_host || layer < 0 || layer >= m->n_layers) return DHQ_EINVAL;
    if (m->precision == DHQ_W32A32) return DHQ_EUNSUPPORTED;
    const dhq_layer &Ly = m->layer[layer];
    memcpy(Wq_host, Ly.wq_host.data(), Ly.wq_host.size());
    return DHQ_OK;
}

extern "C" int dhq_has_fused(const dhq_model *m)
{
    if (!m) return DHQ_EINVAL;
    if (m->flt) return (dhq_float_has_fused(m->flt) && m->fused_sine_ok) ? 1 : 0;
    return ((m->fused || m->wide || m->pair || m->fused2) && (!m->have_scales || m->fused_sine_ok)) ? 1 : 0;
}

extern "C" int dhq_select_wide_kernel(dhq_model *m, int32_t which)
{
    if (!m || which < 0 || which > 2) return DHQ_EINVAL;
    if (!m->wide || !m->pair) return DHQ_EUNSUPPORTED;
    m->wide_kernel = which;
    return DHQ_OK;
}

// Per-layer constant of the quantizer kernel.
static float quant_inv(const dhq_layer &Ly) { return (float)(1.0 / ((double)Ly.s_a * sqrt((double)Ly.Kp))); }

// Buffers one pass of the layer-by-layer path works in.
struct layer_ws {
    float *act[2];
    int8_t *codes;
    int32_t *acc;  // two-sided variant only
};

// GEMM + epilogue of layer l from `codes` into dst (n x M fp32): one kernel, or in the two-sided
// variant the GEMM into the rotated accumulators followed by the un-rotation kernel.
// dyn = device constants of the dynamic mode, or null for the model's static scales.
static hipError_t gemm_epilogue(const dhq_model *m, int l, const int8_t *codes, int64_t rows, int32_t *acc_ws,
                                const float *dyn, float *dst, hipStream_t st)
{
    const dhq_layer &Ly = m->layer[l];
    const bool last = (l == m->n_layers - 1);
    const float c1 = dyn ? 0.0f : dhq_c1(m, l);
    const float *bias = last ? Ly.bias_dev : Ly.bias_rev_dev;
    if (!last && m->act_kind == DHQ_ACT_KIND_WAVELET_COMPLEX) {
        // the complex wavelet pairs neighbouring features, which the GEMM's lanes hold one each: raw
        // accumulators out, then one thread per pair
        hipError_t e = dhq_launch_gemm(Ly, codes, rows, acc_ws, nullptr, 0.0f, nullptr, dhq_act{DHQ_ACT_KIND_NONE, 0.f}, nullptr, st);
        if (e != hipSuccess) return e;
        return dhq_launch_epilogue_pairs(acc_ws, rows, Ly.M, c1, bias, dhq_layer_act(m, l), dyn, dst, st);
    }
    if (!m->rot_out) return dhq_launch_gemm(Ly, codes, rows, nullptr, dst, c1, bias, dhq_layer_act(m, l), dyn, st);
    hipError_t e = dhq_launch_gemm(Ly, codes, rows, acc_ws, nullptr, 0.0f, nullptr, dhq_act{DHQ_ACT_KIND_NONE, 0.f}, nullptr, st);
    if (e != hipSuccess) return e;
    return dhq_launch_unrotate(acc_ws, rows, Ly.Mp, Ly.M, c1, bias, dhq_layer_act(m, l), dyn, nullptr, dst, st);
}

// Runs layers [0, upto) of the layer-by-layer path on `rows` coordinates with the model's static
// scales.  The result of layer upto-1 lands in *result (one of the workspace buffers, or
// `final_out` for the network's last layer when it is given).
static hipError_t run_layers(const dhq_model *m, const layer_ws &ws, const float *in, int64_t rows, int upto,
                             float *final_out, const float **result, hipStream_t st)
{
    const float *cur = in;
    int which = 0;
    // Two-sided variant, whole network: a layer's un-rotation kernel goes on to rotate and quantize the next layer's
    // input in the same lanes, so between two layers only codes and rotated accumulators cross device memory.
    // (Not for a prefix of the network, whose last activations the caller wants, nor for the complex wavelet,
    // whose activation is a kernel of its own.)
    const bool chain = m->rot_out && upto == m->n_layers && m->act_kind != DHQ_ACT_KIND_WAVELET_COMPLEX;
    for (int l = 0; l < upto; ++l) {
        const dhq_layer &Ly = m->layer[l];
        const bool last = (l == m->n_layers - 1);
        hipError_t e = hipSuccess;
        if (!(chain && l > 0)) {
            e = dhq_launch_wht_quant(cur, rows, Ly.K, Ly.Kp, quant_inv(Ly), m->qmax_a, ws.codes, nullptr, st);
            if (e != hipSuccess) return e;
        }
        if (chain && !last) {
            e = dhq_launch_gemm(Ly, ws.codes, rows, ws.acc, nullptr, 0.0f, nullptr, dhq_act{DHQ_ACT_KIND_NONE, 0.f}, nullptr, st);
            if (e != hipSuccess) return e;
            e = dhq_launch_unrotate_quant(ws.acc, rows, Ly.Mp, Ly.M, dhq_c1(m, l), Ly.bias_rev_dev, dhq_layer_act(m, l),
                                          quant_inv(m->layer[l + 1]), m->qmax_a, ws.codes, st);
            if (e != hipSuccess) return e;
            continue;
        }
        float *dst = (last && final_out) ? final_out : ws.act[which];
        e = gemm_epilogue(m, l, ws.codes, rows, ws.acc, nullptr, dst, st);
        if (e != hipSuccess) return e;
        cur = dst;
        which ^= 1;
    }
    *result = cur;
    return hipSuccess;
}

static layer_ws chunk_ws(const dhq_model *m) { return layer_ws{{m->act0, m->act1}, m->codes, m->acc_ws}; }

extern "C" int dhq_calibrate(dhq_model *m, const float *coords_dev, int64_t n, void *stream)
{
    if (!m || n < 0 || (n > 0 && !coords_dev)) return DHQ_EINVAL;
    if (m->flt) return DHQ_EUNSUPPORTED;
    if (n == 0) return DHQ_EINVAL;  // a scale cannot be measured on nothing
    hipStream_t st = (hipStream_t)stream;
    const int K0 = m->dims[0];
    for (int l = 0; l < m->n_layers; ++l) {
        dhq_layer &Ly = m->layer[l];
        if (dhq_launch_clear_words(m->absmax_dev, 1, st) != hipSuccess) return DHQ_EHIP;
        for (int64_t off = 0; off < n; off += DHQ_CHUNK) {
            const int64_t rows = (n - off) < DHQ_CHUNK ? (n - off) : DHQ_CHUNK;
            const float *res = nullptr;
            // the input of layer l is the output of the already calibrated quantized layers before it
            if (run_layers(m, chunk_ws(m), coords_dev + off * K0, rows, l, nullptr, &res, st) != hipSuccess) return DHQ_EHIP;
            if (dhq_launch_wht_absmax(res, rows, Ly.K, Ly.Kp, m->absmax_dev, reinterpret_cast<float *>(m->dyn_absmax + DHQ_MAX_LAYERS),
                                      m->qmax_a, 0.0, nullptr, st) != hipSuccess)
                return DHQ_EHIP;
        }
        unsigned bits = 0;
        if (hipMemcpyAsync(&bits, m->absmax_dev, sizeof(unsigned), hipMemcpyDeviceToHost, st) != hipSuccess) return DHQ_EHIP;
        if (hipStreamSynchronize(st) != hipSuccess) return DHQ_EHIP;
        float mx;
        memcpy(&mx, &bits, sizeof(float));
        // the kernel's transform is un-normalised: max|x^| = mx / sqrt(Kp)
        const double amax = (double)mx / sqrt((double)Ly.Kp);
        Ly.s_a = amax == 0.0 ? 1.0f : (float)(amax / (double)m->qmax_a);
    }
    m->have_scales = true;
    return update_fused_scales(m);
}

// Buffers a dynamic forward works in: whole-batch activations (transformed activations for the
// per-layer fused kernels), codes, the two-sided variant's rotated accumulators, two sets of
// per-workgroup maxima, and the per-layer constants {quantizer multiplier, epilogue multiplier, s_a}.
struct dyn_ws {
    float *act0, *act1;
    int8_t *codes;
    int32_t *acc;
    float *partial;  // 2 x DHQ_ABSMAX_PARTIALS floats
    float *params;   // DHQ_MAX_LAYERS x 3
};

// Bytes of each whole-batch buffer for n rows.
struct dyn_sizes {
    size_t act, codes, acc;
};
static dyn_sizes dyn_buffer_sizes(const dhq_model *m, int64_t n)
{
    // the per-layer fused kernels store whole workgroup tiles
    const size_t rows = m->fused ? dhq_fused_dynamic_rows(n) : m->fused2 ? dhq_fused2_dynamic_rows(n) : m->pair ? dhq_pair_dynamic_rows(n) : (size_t)n;
    dyn_sizes z;
    z.act = sizeof(float) * rows * m->max_dim;
    z.codes = (size_t)n * m->max_kp;
    z.acc = (m->rot_out || m->act_kind == DHQ_ACT_KIND_WAVELET_COMPLEX) ? sizeof(int32_t) * (size_t)n * m->max_mg : 0;
    return z;
}

// Whole-batch buffers of the dynamic mode in the model, grown when a call brings more rows than any before.
static int ensure_dyn_workspace(dhq_model *m, int64_t n)
{
    if (n <= m->dyn_rows) return DHQ_OK;
    if (hipDeviceSynchronize() != hipSuccess) return DHQ_EHIP;  // nothing may still be using the old buffers
    if (m->dyn_act0) (void)hipFree(m->dyn_act0);
    if (m->dyn_act1) (void)hipFree(m->dyn_act1);
    if (m->dyn_codes) (void)hipFree(m->dyn_codes);
    if (m->dyn_acc) (void)hipFree(m->dyn_acc);
    m->dyn_act0 = m->dyn_act1 = nullptr;
    m->dyn_codes = nullptr;
    m->dyn_acc = nullptr;
    m->dyn_rows = 0;
    const dyn_sizes z = dyn_buffer_sizes(m, n);
    if (hipMalloc((void **)&m->dyn_act0, z.act) != hipSuccess) return DHQ_ENOMEM;
    if (hipMalloc((void **)&m->dyn_act1, z.act) != hipSuccess) return DHQ_ENOMEM;
    if (hipMalloc((void **)&m->dyn_codes, z.codes) != hipSuccess) return DHQ_ENOMEM;
    if (z.acc && hipMalloc((void **)&m->dyn_acc, z.acc) != hipSuccess) return DHQ_ENOMEM;
    m->dyn_rows = n;
    return DHQ_OK;
}

extern "C" int dhq_reserve_dynamic(dhq_model *m, int64_t n)
{
    if (!m || n < 0) return DHQ_EINVAL;
    if (m->flt) return DHQ_EUNSUPPORTED;
    return ensure_dyn_workspace(m, n);
}

// The dynamic quantization module between layers (Sec. 3.3) taken literally: every layer first
// reduces max|x^| over its whole rotated input (all n rows), a one-workgroup kernel turns the
// maximum into the layer's constants, then the quantizer and the GEMM read them from device
// memory.  Nothing returns to the host in between.
//
// Two realisations: layer by layer (absmax pass, quantizer, GEMM: three launches per layer, any
// shape), or -- where the whole-network fused kernel exists -- one launch per layer that keeps
// the layer's arithmetic in registers and passes only the transformed activations through
// device memory (dhq_fused_dynamic_launch).  Enqueues kernels only.
static int forward_dynamic(const dhq_model *m, const dyn_ws &ws, const float *coords_dev, int64_t n, float *out_dev,
                           bool per_layer_fused, hipStream_t st)
{
    const int L = m->n_layers;
    if (per_layer_fused) {
        const hipError_t e =
            m->fused2 ? dhq_fused2_dynamic_launch(m, coords_dev, n, out_dev, ws.act0, ws.act1, ws.partial, ws.params, st)
            : m->fused ? dhq_fused_dynamic_launch(m, coords_dev, n, out_dev, ws.act0, ws.act1, ws.partial, ws.params, st)
                       : dhq_pair_dynamic_launch(m, coords_dev, n, out_dev, ws.act0, ws.act1, ws.partial, ws.params, st);
        return e == hipSuccess ? DHQ_OK : DHQ_EHIP;
    }
    const float *cur = coords_dev;
    float *bufs[2] = {ws.act0, ws.act1};
    int which = 0;
    for (int l = 0; l < L; ++l) {
        const dhq_layer &Ly = m->layer[l];
        const bool last = (l == L - 1);
        float *dyn = ws.params + 3 * l;
        // pass 1 leaves one maximum of |x^| per workgroup; pass 2 folds them, quantizes and stores the constants
        int count = 0;
        if (dhq_launch_wht_absmax_partials(cur, n, Ly.K, Ly.Kp, ws.partial, &count, st) != hipSuccess) return DHQ_EHIP;
        const dhq_wht_fold fold = {ws.partial, count, dhq_c1_over_sa(m, l), dyn};
        if (dhq_launch_wht_quant(cur, n, Ly.K, Ly.Kp, 0.0f, m->qmax_a, ws.codes, &fold, st) != hipSuccess) return DHQ_EHIP;
        float *dst = last ? out_dev : bufs[which];
        if (gemm_epilogue(m, l, ws.codes, n, ws.acc, dyn, dst, st) != hipSuccess) return DHQ_EHIP;
        cur = dst;
        which ^= 1;
    }
    return DHQ_OK;
}

// Argument checks shared by the two entry points that run a dynamic forward.
static int check_dynamic_call(const dhq_model *m, int64_t n, uint32_t path, bool *per_layer_fused)
{
    if (!m || n < 0) return DHQ_EINVAL;
    if (path == 3u) return DHQ_EINVAL;
    const bool dyn_fused_ok = (m->fused || m->fused2 || m->pair) && m->dyn_sine_ok;  // per-layer fused kernels of the dynamic mode
    if (m->flt) return DHQ_EUNSUPPORTED;
    if (path == DHQ_FUSED && !dyn_fused_ok) return DHQ_EUNSUPPORTED;
    *per_layer_fused = path != DHQ_LAYERWISE && dyn_fused_ok;
    return DHQ_OK;
}

extern "C" int dhq_forward(const dhq_model *m, const float *coords_dev, int64_t n, float *out_dev, void *stream,
                           uint32_t flags)
{
    if (!m || n < 0) return DHQ_EINVAL;
    const uint32_t path = flags & 3u;
    const bool dynamic = (flags & DHQ_DYNAMIC) != 0;
    if ((flags & ~(3u | DHQ_DYNAMIC)) != 0 || path == 3u) return DHQ_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    if (m->flt) {
        // the whole-network fp32 kernel runs only where the sine's argument provably stays in range
        const bool fused_ok = dhq_float_has_fused(m->flt) && m->fused_sine_ok;
        if (dynamic || (path == DHQ_FUSED && !fused_ok)) return DHQ_EUNSUPPORTED;
        if (n == 0) return DHQ_OK;
        if (!coords_dev || !out_dev) return DHQ_EINVAL;
        const hipError_t e = (path != DHQ_LAYERWISE && fused_ok) ? dhq_float_launch(m->flt, coords_dev, n, out_dev, st)
                                                                 : dhq_float_launch_layerwise(m->flt, coords_dev, n, out_dev, st);
        return e == hipSuccess ? DHQ_OK : DHQ_EHIP;
    }
    if (dynamic) {
        bool per_layer_fused = false;
        int rc = check_dynamic_call(m, n, path, &per_layer_fused);
        if (rc != DHQ_OK) return rc;
        if (n == 0) return DHQ_OK;
        if (!coords_dev || !out_dev) return DHQ_EINVAL;
        // The whole-batch buffers are the one thing a forward call may change in the model: they grow
        // here when this call brings more rows than dhq_reserve_dynamic or any earlier call provided for.
        rc = ensure_dyn_workspace(const_cast<dhq_model *>(m), n);
        if (rc != DHQ_OK) return rc;
        const dyn_ws ws = {m->dyn_act0, m->dyn_act1, m->dyn_codes, m->dyn_acc,
                           reinterpret_cast<float *>(m->dyn_absmax + DHQ_MAX_LAYERS), m->dyn_params};
        return forward_dynamic(m, ws, coords_dev, n, out_dev, per_layer_fused, st);
    }
    // static scales; a whole-network kernel runs only where the sine's argument provably stays in range
    const bool fused_ok = (m->fused || m->wide || m->pair || m->fused2) && m->fused_sine_ok;
    if (path == DHQ_FUSED && !(m->fused || m->wide || m->pair || m->fused2)) return DHQ_EUNSUPPORTED;
    if (n == 0) return DHQ_OK;
    if (!coords_dev || !out_dev) return DHQ_EINVAL;
    if (!m->have_scales) return DHQ_ENOSCALE;
    if (path == DHQ_FUSED && !fused_ok) return DHQ_EUNSUPPORTED;
    if (path != DHQ_LAYERWISE && fused_ok) {
        const hipError_t e = m->fused2 ? dhq_fused2_launch(m->fused2, coords_dev, n, out_dev, st)
                             : m->fused ? dhq_fused_launch(m, coords_dev, n, out_dev, st)
                             : dhq_use_pair(m) ? dhq_pair_launch(m->pair, coords_dev, n, out_dev, st)
                                               : dhq_wide_launch(m->wide, coords_dev, n, out_dev, st);
        return e == hipSuccess ? DHQ_OK : DHQ_EHIP;
    }
    const int K0 = m->dims[0], Mo = m->dims[m->n_layers];
    for (int64_t off = 0; off < n; off += DHQ_CHUNK) {
        const int64_t rows = (n - off) < DHQ_CHUNK ? (n - off) : DHQ_CHUNK;
        const float *res = nullptr;
        if (run_layers(m, chunk_ws(m), coords_dev + off * K0, rows, m->n_layers, out_dev + off * Mo, &res, st) != hipSuccess)
            return DHQ_EHIP;
    }
    return DHQ_OK;
}

// ---- the entry point that allocates nothing (its buffer is declared near the top of this file) ----
extern "C" int64_t dhq_noalloc_max_rows(const dhq_model *m)
{
    if (!m || m->flt) return 0;
    // bytes per row: two activation buffers, the codes, the two-sided variant's accumulators; the
    // per-layer fused kernels round the rows up to a whole workgroup tile, hence the search
    int64_t lo = 0, hi = (int64_t)(DHQ_NOALLOC_SCRATCH_BYTES / 4);
    while (lo < hi) {
        const int64_t mid = lo + (hi - lo + 1) / 2;
        const dyn_sizes z = dyn_buffer_sizes(m, mid);
        if (2 * round256(z.act) + round256(z.codes) + round256(z.acc) <= DHQ_NOALLOC_SCRATCH_BYTES) lo = mid;
        else hi = mid - 1;
    }
    return lo;
}

extern "C" int dhq_forward_noalloc(const dhq_model *m, const float *coords_dev, int64_t n, float *out_dev, void *stream,
                                   uint32_t flags)
{
    bool per_layer_fused = false;
    if ((flags & ~3u) != 0) return DHQ_EINVAL;
    int rc = check_dynamic_call(m, n, flags & 3u, &per_layer_fused);
    if (rc != DHQ_OK) return rc;
    if (n == 0) return DHQ_OK;
    if (!coords_dev || !out_dev) return DHQ_EINVAL;
    const dyn_sizes z = dyn_buffer_sizes(m, n);
    if (2 * round256(z.act) + round256(z.codes) + round256(z.acc) > DHQ_NOALLOC_SCRATCH_BYTES) return DHQ_ETOOBIG;
    unsigned char *base = m->scratch;  // looked up when the model was created, with its device current
    if (!base) return DHQ_EHIP;
    dyn_ws ws;
    ws.partial = reinterpret_cast<float *>(base);
    base += DHQ_NOALLOC_PARTIAL_BYTES;
    ws.act0 = reinterpret_cast<float *>(base);
    base += round256(z.act);
    ws.act1 = reinterpret_cast<float *>(base);
    base += round256(z.act);
    ws.codes = reinterpret_cast<int8_t *>(base);
    base += round256(z.codes);
    ws.acc = z.acc ? reinterpret_cast<int32_t *>(base) : nullptr;
    // the per-layer constants are a result (dhq_get_dynamic_scales reads them), not scratch: they
    // stay in the model, whose buffer exists since dhq_quantize_weights
    ws.params = m->dyn_params;
    // Nothing in the scratch buffer has to start at zero: every kernel writes the part it hands to
    // the next one in full (per-workgroup maxima up to the count the host passes on, every row of
    // the activation and code buffers below n) before that kernel reads it.
    return forward_dynamic(m, ws, coords_dev, n, out_dev, per_layer_fused, (hipStream_t)stream);
}

extern "C" int dhq_get_dynamic_scales(const dhq_model *m, float *s_a_host, void *stream)
{
    if (!m || !s_a_host) return DHQ_EINVAL;
    if (m->flt) return DHQ_EUNSUPPORTED;
    float tmp[3 * DHQ_MAX_LAYERS];
    hipStream_t st = (hipStream_t)stream;
    if (hipMemcpyAsync(tmp, m->dyn_params, sizeof(float) * 3 * m->n_layers, hipMemcpyDeviceToHost, st) != hipSuccess) return DHQ_EHIP;
    if (hipStreamSynchronize(st) != hipSuccess) return DHQ_EHIP;
    for (int l = 0; l < m->n_layers; ++l) s_a_host[l] = tmp[3 * l + 2];
    return DHQ_OK;
}

extern "C" int dhq_forward_debug(const dhq_model *m, const float *in_dev, int64_t n, int32_t layer, int8_t *codes_dev,
                                 int32_t *acc_dev, float *act_dev, void *stream)
{
    if (!m || n < 0 || layer < 0 || layer >= m->n_layers) return DHQ_EINVAL;
    if (n > DHQ_CHUNK || m->flt) return DHQ_EUNSUPPORTED;
    if (n == 0) return DHQ_OK;
    if (!in_dev) return DHQ_EINVAL;
    if (!m->have_scales) return DHQ_ENOSCALE;
    hipStream_t st = (hipStream_t)stream;
    const dhq_layer &Ly = m->layer[layer];
    const bool last = (layer == m->n_layers - 1);
    const float *bias = last ? Ly.bias_dev : Ly.bias_rev_dev;
    int8_t *codes = codes_dev ? codes_dev : m->codes;
    if (dhq_launch_wht_quant(in_dev, n, Ly.K, Ly.Kp, quant_inv(Ly), m->qmax_a, codes, nullptr, st) != hipSuccess)
        return DHQ_EHIP;
    if (!acc_dev && !act_dev) return DHQ_OK;
    if (m->rot_out) {
        // rotated accumulators into the workspace, then un-rotated ones and the activation out
        if (dhq_launch_gemm(Ly, codes, n, m->acc_ws, nullptr, 0.0f, nullptr, dhq_act{DHQ_ACT_KIND_NONE, 0.f}, nullptr, st) != hipSuccess) return DHQ_EHIP;
        return dhq_launch_unrotate(m->acc_ws, n, Ly.Mp, Ly.M, dhq_c1(m, layer), bias, dhq_layer_act(m, layer), nullptr, acc_dev, act_dev, st) == hipSuccess
                   ? DHQ_OK
                   : DHQ_EHIP;
    }
    // the int32 accumulators go through the workspace when the caller does not want them
    int32_t *acc = acc_dev ? acc_dev : reinterpret_cast<int32_t *>(m->act0);
    if (dhq_launch_gemm(Ly, codes, n, acc, nullptr, 0.0f, nullptr, dhq_act{DHQ_ACT_KIND_NONE, 0.f}, nullptr, st) != hipSuccess) return DHQ_EHIP;
    if (act_dev && !last && m->act_kind == DHQ_ACT_KIND_WAVELET_COMPLEX)
        return dhq_launch_epilogue_pairs(acc, n, Ly.M, dhq_c1(m, layer), bias, dhq_layer_act(m, layer), nullptr, act_dev, st) == hipSuccess ? DHQ_OK : DHQ_EHIP;
    if (act_dev && dhq_launch_epilogue(acc, n, Ly.M, dhq_c1(m, layer), bias, dhq_layer_act(m, layer), act_dev, st) != hipSuccess) return DHQ_EHIP;
    return DHQ_OK;
}

extern "C" int dhq_forward_debug_fused(const dhq_model *m, const int8_t *codes_in_dev, int64_t n, int32_t layer, float *xhat_dev,
                                       int8_t *codes_out_dev, int32_t *acc_dev, void *stream)
{
    if (!m || n < 0 || layer < 0 || layer >= m->n_layers) return DHQ_EINVAL;
    if (m->flt || !(m->fused || m->wide || m->pair || m->fused2)) return DHQ_EUNSUPPORTED;
    if (layer >= m->n_layers - 1) return DHQ_EUNSUPPORTED;  // the output layer has no transform after it
    if (n == 0) return DHQ_OK;
    if (!codes_in_dev) return DHQ_EINVAL;
    if (!m->have_scales) return DHQ_ENOSCALE;
    if (!m->fused_sine_ok) return DHQ_EUNSUPPORTED;
    hipStream_t st = (hipStream_t)stream;
    const hipError_t e = m->fused2 ? dhq_fused2_debug_launch(m, layer, codes_in_dev, n, xhat_dev, codes_out_dev, acc_dev, st)
                         : m->fused ? dhq_fused_debug_launch(m, layer, codes_in_dev, n, xhat_dev, codes_out_dev, acc_dev, st)
                         : dhq_use_pair(m) ? dhq_pair_debug_launch(m, layer, codes_in_dev, n, xhat_dev, codes_out_dev, acc_dev, st)
                                           : dhq_wide_debug_launch(m, layer, codes_in_dev, n, xhat_dev, codes_out_dev, acc_dev, st);
    return e == hipSuccess ? DHQ_OK : DHQ_EHIP;
}

extern "C" int dhq_gemm_i8(const dhq_model *m, int32_t layer, const int8_t *codes_dev, int64_t n, int32_t *acc_dev,
                           void *stream)
{
    if (!m || n < 0 || layer < 0 || layer >= m->n_layers) return DHQ_EINVAL;
    if (m->flt) return DHQ_EUNSUPPORTED;
    if (n == 0) return DHQ_OK;
    if (!codes_dev || !acc_dev) return DHQ_EINVAL;
    return dhq_launch_gemm(m->layer[layer], codes_dev, n, acc_dev, nullptr, 0.0f, nullptr, dhq_act{DHQ_ACT_KIND_NONE, 0.f}, nullptr, (hipStream_t)stream) == hipSuccess
               ? DHQ_OK
               : DHQ_EHIP;
}
