// Whole-network fused forward with floating-point activations (gfx950): the "W32A32" and
// "W8A32" rows of the paper's comparison (Sec. 1, Fig. 1-2, Table 2).  W32A32 is the plain
// SIREN, y = W a + b, a = sin(omega0 y); W8A32 is the same network run on the weights after
// the offline step and de-quantization, W~ = (s_w Wq) Hn (the caller passes whichever
// weights apply; the kernel does not know the difference).  fp32 throughout, on the fp32
// MFMA (v_mfma_f32_32x32x2_f32: 32 features x 32 coordinates x 2 k per instruction).
//
// Layout: as in the int8 kernels the features are the MFMA M dimension and a wave carries
// 32 coordinates through all layers.  The D layout gives lane (c, h) rows 8g + 4h + e of
// every 32-row tile T, i.e. register R = 16T + 4g + e holds feature 32T + 8g + 4h + e.  The
// B operand of k step kk wants lane half h to hold "k = 2 kk + h" -- and since the order of k
// is free as long as the weights use the same one, k step kk simply takes register R = kk:
// the activations are consumed exactly where the previous layer's epilogue left them, and
// the weights are packed offline in that order.  Nothing is ever shuffled.
//
// The weights of a 256-wide layer are 256 KiB in fp32, more than LDS holds, and every MFMA
// needs only 256 B of them per wave: they are read straight from device memory (they stay
// in L2), one 16-byte load per lane and four MFMAs, eight groups (4096 matrix-unit clocks)
// ahead of use.  The kernel is bound by the matrix unit (64 clocks per instruction); the
// vector ALU only does one multiply-add and one sine per accumulator.
//
// Registers: one wave per SIMD.  The current activations (B operands, 128 per lane at width
// 256) live in accumulation registers a128..a255, addressed by number from inline assembly
// (the MFMA included: the builtin cannot take B from an accumulation register without a
// copy); the build checks on the compiler's assembly output that compiler-generated code never
// touches them.  Wait states the compiler can no longer see (accumulation-register write ->
// MFMA read, MFMA result -> vector ALU read) are covered by explicit s_nop.
//
// Every other shape (and DHQ_LAYERWISE on the shapes above) runs layer by layer through
// float_layer_kernel: one fp32 MFMA GEMM with the bias + sine epilogue per layer, activations
// in device memory between the layers, 65 536 rows at a time.
#include <math.h>
#include <string.h>

#include <new>
#include <utility>
#include <vector>

#include "dhq_device.h"
#include "dhq_internal.h"

#define FLT_WAVES 4
#define FLT_THREADS (FLT_WAVES * 64)
#define FLT_TILE (FLT_WAVES * 32)
#define FLT_AGPR_X 128   // first accumulation register of the activations
#define FLT_AHEAD 8      // weight groups (of four k steps) in flight

typedef float dhq_v16f __attribute__((ext_vector_type(16)));

struct float_layer_desc {
    uint32_t w_off;     // float offset of the layer's packed weights in the blob
    uint32_t b_off;     // float offset of its bias block [tile][h][16]
};

struct float_args {
    const float *coords;
    float *out;
    const float *blob;
    int64_t n;
    int n_layers;
    int k0;          // fan-in of the input layer (<= 4)
    int m_out;       // fan-out of the output layer (<= 32)
    float rev;       // omega0 / (2 pi): the sine takes revolutions
    float c2;        // wavelet activation: 2 pi s0 sqrt(log2 e) / omega0
    float_layer_desc layer[DHQ_MAX_LAYERS];
};

// One layer of the layer-by-layer path: weights as B fragments [M tile][k group J][quarter q][lane]
// float4, lane (c, kk) holding W[32 T + c][32 J + 16 kk + 4 q + e], e = 0..3 (zero beyond M and K);
// bias (times omega0 / 2 pi in the sine layers).
struct float_lw_layer {
    float *wfrag_dev = nullptr;
    float *bias_dev = nullptr;
    int K = 0, M = 0, NG = 0, Mt = 0;
};

struct dhq_float_plan {
    int nf = 0;              // hidden width of the fused kernel, 0 if the shape has none
    float *blob_dev = nullptr;
    size_t blob_floats = 0;
    float_args args;
    int n_cu = 0;
    int n_layers = 0;
    float rev = 0.f;
    dhq_act actf = {DHQ_ACT_KIND_SINE, 0.f};  // what follows every layer but the last
    float_lw_layer lw[DHQ_MAX_LAYERS];
    float *act[2] = {nullptr, nullptr};  // DHQ_CHUNK x widest layer, fp32
};

// ----------------------------------------------------------------------------- device code
template <int KK>
__device__ __forceinline__ void flt_x_write(float v)
{
    asm volatile("v_accvgpr_write_b32 a[%1], %0" : : "v"(v), "n"(FLT_AGPR_X + KK));
}
template <int KK>
__device__ __forceinline__ void flt_mfma_first(dhq_v16f &acc, float a)
{
    asm volatile("v_mfma_f32_32x32x2_f32 %0, %1, a[%2], 0" : "=&v"(acc) : "v"(a), "n"(FLT_AGPR_X + KK));
}
template <int KK>
__device__ __forceinline__ void flt_mfma_next(dhq_v16f &acc, float a)
{
    asm volatile("v_mfma_f32_32x32x2_f32 %0, %1, a[%2], %0" : "+v"(acc) : "v"(a), "n"(FLT_AGPR_X + KK));
}
// Idle issue slots that the readers of `acc` cannot be moved ahead of (16-pass MFMA -> vector ALU).
__device__ __forceinline__ void flt_settle(dhq_v16f &acc)
{
    asm volatile("s_nop 7\n\ts_nop 7\n\ts_nop 7" : "+v"(acc));
}

template <int... Ks>
__device__ __forceinline__ void flt_x_store(const float *y, std::integer_sequence<int, Ks...>)
{
    (flt_x_write<Ks>(y[Ks]), ...);
    asm volatile("s_nop 7" ::: "memory");  // accumulation-register write -> MFMA read
}

// One group of a hidden layer's GEMM: k steps 4q .. 4q+3 for the CHN tiles of pair P.
//   ring   weight groups in flight: ring[(g % FLT_AHEAD) * CHN + j] is the float4 of tile j
//   wl     this lane's pointer into the layer's packed weights: group g, tile j at wl[(g * CHN + j) * 64]
template <int NF, int CHN, int G>
__device__ __forceinline__ void flt_group(const float4 *__restrict__ wl, float4 (&ring)[FLT_AHEAD * CHN],
                                          dhq_v16f (&acc)[CHN])
{
    constexpr int NQ = NF / 8;           // groups per pair (k steps / 4)
    constexpr int NP = NF / 32 / CHN;    // pairs per layer
    constexpr int q = G % NQ;
    constexpr int pf = G + FLT_AHEAD;
    float4 cur[CHN];
#pragma unroll
    for (int j = 0; j < CHN; ++j) cur[j] = ring[(G % FLT_AHEAD) * CHN + j];
    if constexpr (pf < NP * NQ) {
#pragma unroll
        for (int j = 0; j < CHN; ++j) ring[(pf % FLT_AHEAD) * CHN + j] = wl[(pf * CHN + j) * 64];
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int j = 0; j < CHN; ++j) {
        if constexpr (q == 0)
            flt_mfma_first<4 * q + 0>(acc[j], cur[j].x);
        else
            flt_mfma_next<4 * q + 0>(acc[j], cur[j].x);
    }
#pragma unroll
    for (int j = 0; j < CHN; ++j) flt_mfma_next<4 * q + 1>(acc[j], cur[j].y);
#pragma unroll
    for (int j = 0; j < CHN; ++j) flt_mfma_next<4 * q + 2>(acc[j], cur[j].z);
#pragma unroll
    for (int j = 0; j < CHN; ++j) flt_mfma_next<4 * q + 3>(acc[j], cur[j].w);
    __builtin_amdgcn_sched_barrier(0);
}

// ACTK: the activation (sine, or the wavelet with envelope constant c2).
template <int NF, int CHN, int ACTK, int P, int... Qs>
__device__ __forceinline__ void flt_pair(const float4 *__restrict__ wl, const float4 *__restrict__ bl,
                                         float4 (&ring)[FLT_AHEAD * CHN], float rev, float c2, float (&y)[NF / 2],
                                         std::integer_sequence<int, Qs...>)
{
    constexpr int NQ = NF / 8;
    dhq_v16f acc[CHN];
    // the pair's biases, fetched while the matrix unit works
    float4 bq[CHN][4];
#pragma unroll
    for (int j = 0; j < CHN; ++j)
#pragma unroll
        for (int gg = 0; gg < 4; ++gg) bq[j][gg] = bl[(P * CHN + j) * 8 + gg];
    (flt_group<NF, CHN, P * NQ + Qs>(wl, ring, acc), ...);
#pragma unroll
    for (int j = 0; j < CHN; ++j) {
        flt_settle(acc[j]);
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const float4 bb = bq[j][v >> 2];
            const float bias = (v & 3) == 0 ? bb.x : (v & 3) == 1 ? bb.y : (v & 3) == 2 ? bb.z : bb.w;
            y[16 * (P * CHN + j) + v] = dhq_activate_rev(__builtin_fmaf(acc[j][v], rev, bias), dhq_act{ACTK, c2});
        }
    }
}

template <int NF, int CHN, int ACTK, int... Ps>
__device__ __forceinline__ void flt_hidden_layer(const float4 *__restrict__ wl, const float4 *__restrict__ bl, float rev, float c2,
                                                 float (&y)[NF / 2], std::integer_sequence<int, Ps...>)
{
    constexpr int NQ = NF / 8;
    constexpr int NG = (NF / 32 / CHN) * NQ;
    float4 ring[FLT_AHEAD * CHN];
#pragma unroll
    for (int g = 0; g < FLT_AHEAD; ++g)
        if (g < NG) {
#pragma unroll
            for (int j = 0; j < CHN; ++j) ring[g * CHN + j] = wl[(g * CHN + j) * 64];
        }
    (flt_pair<NF, CHN, ACTK, Ps>(wl, bl, ring, rev, c2, y, std::make_integer_sequence<int, NQ>{}), ...);
}

template <int NF, int... Qs>
__device__ __forceinline__ void flt_out_layer(const float4 *__restrict__ wl, dhq_v16f &acc, std::integer_sequence<int, Qs...>)
{
    // one tile, no look-ahead ring: the compiler's own scheduling of these loads is enough for 1/8 of a layer
    ((Qs == 0 ? flt_mfma_first<4 * Qs>(acc, wl[Qs * 64].x) : flt_mfma_next<4 * Qs>(acc, wl[Qs * 64].x),
      flt_mfma_next<4 * Qs + 1>(acc, wl[Qs * 64].y), flt_mfma_next<4 * Qs + 2>(acc, wl[Qs * 64].z),
      flt_mfma_next<4 * Qs + 3>(acc, wl[Qs * 64].w)),
     ...);
}

template <int NF, int ACTK>
__global__ __launch_bounds__(FLT_THREADS) void dhq_float_kernel(const float_args A)
{
    constexpr int NT = NF / 32;
    constexpr int NR = NF / 2;
    constexpr int CHN = NT >= 2 ? 2 : 1;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = lane & 31, h = lane >> 5;
    const int L = A.n_layers;
    const int64_t n_tiles = (A.n + FLT_TILE - 1) / FLT_TILE;
    // the registers addressed by number count towards the kernel's register allocation
    asm volatile("" ::: "a255");
    static_assert(FLT_AGPR_X + NR <= 256, "register map");

    for (int64_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const int64_t ci = tile * FLT_TILE + wave * 32 + c;
        const bool valid = ci < A.n;
        const int64_t cl = valid ? ci : A.n - 1;
        float y[NR];
        {
            // input layer: k step kk holds coordinate component 2 kk + h of this lane's coordinate
            const float x0 = (h < A.k0) ? A.coords[cl * A.k0 + h] : 0.0f;
            const float x1 = (2 + h < A.k0) ? A.coords[cl * A.k0 + 2 + h] : 0.0f;
            flt_x_write<0>(x0);
            flt_x_write<1>(x1);
            asm volatile("s_nop 7" ::: "memory");
            const float *w0 = A.blob + A.layer[0].w_off + lane;
            const float4 *b0 = reinterpret_cast<const float4 *>(A.blob + A.layer[0].b_off) + h * 4;
#pragma unroll
            for (int T = 0; T < NT; ++T) {
                dhq_v16f acc;
                flt_mfma_first<0>(acc, w0[(T * 2 + 0) * 64]);
                flt_mfma_next<1>(acc, w0[(T * 2 + 1) * 64]);
                float4 bq[4];
#pragma unroll
                for (int gg = 0; gg < 4; ++gg) bq[gg] = b0[T * 8 + gg];
                flt_settle(acc);
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const float4 bb = bq[v >> 2];
                    const float bias = (v & 3) == 0 ? bb.x : (v & 3) == 1 ? bb.y : (v & 3) == 2 ? bb.z : bb.w;
                    y[16 * T + v] = dhq_activate_rev(__builtin_fmaf(acc[v], A.rev, bias), dhq_act{ACTK, A.c2});
                }
            }
        }
        for (int l = 1; l < L - 1; ++l) {
            flt_x_store(y, std::make_integer_sequence<int, NR>{});
            const float4 *wl = reinterpret_cast<const float4 *>(A.blob + A.layer[l].w_off) + lane;
            const float4 *bl = reinterpret_cast<const float4 *>(A.blob + A.layer[l].b_off) + h * 4;
            flt_hidden_layer<NF, CHN, ACTK>(wl, bl, A.rev, A.c2, y, std::make_integer_sequence<int, NT / CHN>{});
        }
        {
            // output layer: one zero-padded tile, no sine
            flt_x_store(y, std::make_integer_sequence<int, NR>{});
            const float4 *wl = reinterpret_cast<const float4 *>(A.blob + A.layer[L - 1].w_off) + lane;
            const float *bo = A.blob + A.layer[L - 1].b_off + h * 16;
            dhq_v16f acc;
            flt_out_layer<NF>(wl, acc, std::make_integer_sequence<int, NR / 4>{});
            float bias[16];
#pragma unroll
            for (int v = 0; v < 16; ++v) bias[v] = bo[v];
            flt_settle(acc);
            if (valid) {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int row = 8 * (v >> 2) + 4 * h + (v & 3);
                    if (row < A.m_out) A.out[ci * A.m_out + row] = acc[v] + bias[v];
                }
            }
        }
    }
}

// ---------------------------------------------------------------- layer by layer, any shape
// out = epilogue(in W^T + b) for one layer: in n x K, out n x M, both row-major fp32.  Coordinates
// are the MFMA row dimension (A operand), features the columns (B operand: the packed weights),
// so the 32 lanes of a wave half store 128 contiguous bytes of one output row.  A wave takes 32
// rows and up to FLW_TILES column tiles; k runs in groups of 32: lane (r, kk) reads the sixteen
// inputs 32 J + 16 kk + i of its row (64 contiguous bytes, so that a row's cache line is fetched
// once) and feeds them to sixteen MFMAs per tile, MFMA i taking k = 32 J + i and 32 J + 16 + i.
#define FLW_WAVES 4
#define FLW_TILES 4

// NTT: column tiles per wave (NTT, or all of a layer with fewer: its few tiles then cost no more than their own MFMAs).
template <int ACT, int NTT>
__global__ __launch_bounds__(64 * FLW_WAVES) void float_layer_kernel(const float *__restrict__ in, int64_t n, int K, int NG,
                                                                     int vec, const float4 *__restrict__ wfrag, int M, int Mt,
                                                                     const float *__restrict__ bias, float rev, float c2,
                                                                     float *__restrict__ out)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = lane & 31, h = lane >> 5;
    // wave-uniform, so that the row part of every store address is scalar arithmetic
    const int64_t row0 = ((int64_t)blockIdx.x * FLW_WAVES + __builtin_amdgcn_readfirstlane(wave)) * 32;
    if (row0 >= n) return;  // no barrier below
    const int T0 = blockIdx.y * NTT;
    const int nt = (Mt - T0 < NTT) ? Mt - T0 : NTT;
    const int64_t arow = (row0 + c < n) ? row0 + c : n - 1;  // rows past the end repeat the last one and are not stored
    const float *ap = in + arow * K;
    dhq_v16f acc[NTT];
#pragma unroll
    for (int t = 0; t < NTT; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[t][v] = 0.f;
    // this lane's sixteen inputs of k group J (zero beyond K): 64 contiguous bytes of its row
    auto load_a = [&](int J, float4 (&a)[4]) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int k0 = 32 * J + 16 * h + 4 * q;
            if (vec && k0 + 3 < K) {
                a[q] = *reinterpret_cast<const float4 *>(ap + k0);
            } else {
                a[q].x = (k0 < K) ? ap[k0] : 0.f;
                a[q].y = (k0 + 1 < K) ? ap[k0 + 1] : 0.f;
                a[q].z = (k0 + 2 < K) ? ap[k0 + 2] : 0.f;
                a[q].w = (k0 + 3 < K) ? ap[k0 + 3] : 0.f;
            }
        }
    };
    // tiles past the layer's last one re-read the last one's weights; their results are dropped
    const float4 *wp[NTT];
#pragma unroll
    for (int t = 0; t < NTT; ++t) wp[t] = wfrag + (size_t)(T0 + (t < nt ? t : nt - 1)) * NG * 4 * 64 + lane;
    float4 a[4], w[NTT];
    load_a(0, a);
#pragma unroll
    for (int t = 0; t < NTT; ++t) w[t] = wp[t][0];
    for (int J = 0; J < NG; ++J) {
        // the next operands are fetched while the current MFMAs run (inputs one group of 32 k ahead, weights
        // one quarter group ahead); consecutive MFMAs go to different accumulators
        const int Jn = (J + 1 < NG) ? J + 1 : J;
        float4 an[4];
        load_a(Jn, an);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int nxt = (q < 3) ? 4 * J + q + 1 : 4 * Jn;
            float4 wn[NTT];
#pragma unroll
            for (int t = 0; t < NTT; ++t) wn[t] = wp[t][(size_t)nxt * 64];
#pragma unroll
            for (int t = 0; t < NTT; ++t) acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[q].x, w[t].x, acc[t], 0, 0, 0);
#pragma unroll
            for (int t = 0; t < NTT; ++t) acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[q].y, w[t].y, acc[t], 0, 0, 0);
#pragma unroll
            for (int t = 0; t < NTT; ++t) acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[q].z, w[t].z, acc[t], 0, 0, 0);
#pragma unroll
            for (int t = 0; t < NTT; ++t) acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[q].w, w[t].w, acc[t], 0, 0, 0);
#pragma unroll
            for (int t = 0; t < NTT; ++t) w[t] = wn[t];
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) a[q] = an[q];
    }
    // accumulator v of a lane: row row0 + 8 (v / 4) + 4 h + v % 4, feature 32 (T0 + t) + c; a store address is a
    // scalar base (row, tile) plus the lane's constant offset; whole 32-row blocks skip the row checks
    const int nrows = (n - row0 < 32) ? (int)(n - row0) : 32;
    const bool full = (nrows == 32);
    const unsigned loff = (unsigned)(4 * h * M + c);
    auto epi = [&](float a, float bf) {
        return ACT != DHQ_ACT_KIND_NONE ? dhq_activate_rev_any(__builtin_fmaf(a, rev, bf), dhq_act{ACT, c2}) : a + bf;
    };
#pragma unroll
    for (int t = 0; t < NTT; ++t) {
        if (t < nt) {
            const int f = 32 * (T0 + t) + c;
            if (f < M) {
                const float bf = bias[f];
                float *tile_out = out + (size_t)row0 * M + (size_t)(T0 + t) * 32;  // wave-uniform
                if (full) {
#pragma unroll
                    for (int v = 0; v < 16; ++v)
                        (tile_out + (size_t)(8 * (v >> 2) + (v & 3)) * M)[loff] = epi(acc[t][v], bf);
                } else {
#pragma unroll
                    for (int v = 0; v < 16; ++v)
                        if (8 * (v >> 2) + (v & 3) + 4 * h < nrows) (tile_out + (size_t)(8 * (v >> 2) + (v & 3)) * M)[loff] = epi(acc[t][v], bf);
                }
            }
        }
    }
}

// ------------------------------------------------------------------------------- host code
// Feature held by register kk of lane half h (the D layout of the 32 x 32 MFMA).
static int flt_feature(int kk, int h) { return 32 * (kk >> 4) + 8 * ((kk >> 2) & 3) + 4 * h + (kk & 3); }

bool dhq_float_shape_ok(const int *dims, int L)
{
    if (L < 2) return false;
    if (dims[0] > 4 || dims[L] > 32) return false;
    const int nf = dims[1];
    if (nf != 32 && nf != 64 && nf != 128 && nf != 256) return false;
    for (int l = 1; l < L; ++l)
        if (dims[l] != nf) return false;
    return true;
}

static int float_create_fused(dhq_float_plan *P, const int *dims, int L, double rev, const std::vector<std::vector<float>> &W,
                              const std::vector<std::vector<float>> &b);
static int float_create_layerwise(dhq_float_plan *P, const int *dims, int L, double rev, const std::vector<std::vector<float>> &W,
                                  const std::vector<std::vector<float>> &b);

// W[l]: dims[l+1] x dims[l] fp32 (the weights the network is to run on), b[l]: dims[l+1].
// `act` follows every layer but the last.
int dhq_float_create(const int *dims, int L, float omega0, dhq_act act, const std::vector<std::vector<float>> &W,
                     const std::vector<std::vector<float>> &b, int device, dhq_float_plan **plan_out)
{
    *plan_out = nullptr;
    dhq_float_plan *P = new (std::nothrow) dhq_float_plan();
    if (!P) return DHQ_ENOMEM;
    memset(&P->args, 0, sizeof(P->args));
    const double rev = (double)omega0 / 6.283185307179586476925286766559;
    P->n_layers = L;
    P->rev = (float)rev;
    P->actf = act;
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, device) != hipSuccess) {
        delete P;
        return DHQ_EHIP;
    }
    P->n_cu = prop.multiProcessorCount;
    int rc = float_create_layerwise(P, dims, L, rev, W, b);
    if (rc == DHQ_OK && dhq_float_shape_ok(dims, L)) rc = float_create_fused(P, dims, L, rev, W, b);
    if (rc != DHQ_OK) {
        dhq_float_destroy(P);
        return rc;
    }
    *plan_out = P;
    return DHQ_OK;
}

// The packed weights and biases of the whole-network kernel.
static int float_create_fused(dhq_float_plan *P, const int *dims, int L, double rev, const std::vector<std::vector<float>> &W,
                              const std::vector<std::vector<float>> &b)
{
    const int nf = dims[1], NT = nf / 32, NR = nf / 2, CHN = NT >= 2 ? 2 : 1;
    std::vector<float> blob;
    auto bias_block = [&](int l, int tiles, bool sine) {
        // [tile][h][16]: register v of lane half h holds feature 32 T + 8 (v / 4) + 4 h + v % 4
        const size_t off = blob.size();
        blob.resize(off + (size_t)tiles * 32, 0.0f);
        for (int T = 0; T < tiles; ++T)
            for (int h = 0; h < 2; ++h)
                for (int v = 0; v < 16; ++v) {
                    const int f = 32 * T + 8 * (v >> 2) + 4 * h + (v & 3);
                    if (f < dims[l + 1])
                        blob[off + (size_t)(T * 2 + h) * 16 + v] = sine ? (float)((double)b[l][f] * rev) : b[l][f];
                }
        return (uint32_t)off;
    };
    for (int l = 0; l < L; ++l) {
        const int K = dims[l], M = dims[l + 1];
        const size_t off = blob.size();
        if (l == 0) {
            // [T][kk0 = 0, 1][lane]: A[m][h] = W[32 T + m][2 kk0 + h]
            blob.resize(off + (size_t)NT * 2 * 64, 0.0f);
            for (int T = 0; T < NT; ++T)
                for (int kk = 0; kk < 2; ++kk)
                    for (int ln = 0; ln < 64; ++ln) {
                        const int row = 32 * T + (ln & 31), k = 2 * kk + (ln >> 5);
                        if (row < M && k < K) blob[off + (size_t)(T * 2 + kk) * 64 + ln] = W[l][(size_t)row * K + k];
                    }
        } else {
            // [group g = pair * NQ + q][tile j of the pair][lane][4 k steps]; the output layer is one tile
            const bool last = (l == L - 1);
            const int chn = last ? 1 : CHN, tiles = last ? 1 : NT, NQ = NR / 4;
            blob.resize(off + (size_t)tiles * NR * 64, 0.0f);
            for (int p = 0; p < tiles / chn; ++p)
                for (int q = 0; q < NQ; ++q)
                    for (int j = 0; j < chn; ++j)
                        for (int ln = 0; ln < 64; ++ln)
                            for (int i = 0; i < 4; ++i) {
                                const int row = 32 * (p * chn + j) + (ln & 31);
                                const int k = flt_feature(4 * q + i, ln >> 5);
                                if (row < M && k < K)
                                    blob[off + ((size_t)((p * NQ + q) * chn + j) * 64 + ln) * 4 + i] = W[l][(size_t)row * K + k];
                            }
        }
        P->args.layer[l].w_off = (uint32_t)off;
        P->args.layer[l].b_off = bias_block(l, l == L - 1 ? 1 : NT, l != L - 1);
    }
    P->blob_floats = blob.size();
    if (hipMalloc((void **)&P->blob_dev, sizeof(float) * blob.size()) != hipSuccess) return DHQ_ENOMEM;
    if (hipMemcpy(P->blob_dev, blob.data(), sizeof(float) * blob.size(), hipMemcpyHostToDevice) != hipSuccess) return DHQ_EHIP;
    P->args.blob = P->blob_dev;
    P->args.n_layers = L;
    P->args.k0 = dims[0];
    P->args.m_out = dims[L];
    P->args.rev = (float)rev;
    P->args.c2 = P->actf.c2;
    P->nf = nf;
    return DHQ_OK;
}

// Fragments, biases and the two activation buffers of the layer-by-layer path.
static int float_create_layerwise(dhq_float_plan *P, const int *dims, int L, double rev, const std::vector<std::vector<float>> &W,
                                  const std::vector<std::vector<float>> &b)
{
    int max_dim = 1;
    for (int l = 0; l <= L; ++l) max_dim = dims[l] > max_dim ? dims[l] : max_dim;
    for (int l = 0; l < L; ++l) {
        float_lw_layer &Ly = P->lw[l];
        Ly.K = dims[l];
        Ly.M = dims[l + 1];
        Ly.NG = (Ly.K + 31) / 32;
        Ly.Mt = (Ly.M + 31) / 32;
        std::vector<float> frag((size_t)Ly.Mt * Ly.NG * 4 * 64 * 4, 0.0f);
        for (int T = 0; T < Ly.Mt; ++T)
            for (int J = 0; J < Ly.NG; ++J)
                for (int q = 0; q < 4; ++q)
                    for (int ln = 0; ln < 64; ++ln)
                        for (int e = 0; e < 4; ++e) {
                            const int row = 32 * T + (ln & 31), k = 32 * J + 16 * (ln >> 5) + 4 * q + e;
                            if (row < Ly.M && k < Ly.K)
                                frag[((((size_t)T * Ly.NG + J) * 4 + q) * 64 + ln) * 4 + e] = W[l][(size_t)row * Ly.K + k];
                        }
        std::vector<float> bias(Ly.M);
        for (int f = 0; f < Ly.M; ++f) bias[f] = (l != L - 1) ? (float)((double)b[l][f] * rev) : b[l][f];
        if (hipMalloc((void **)&Ly.wfrag_dev, sizeof(float) * frag.size()) != hipSuccess) return DHQ_ENOMEM;
        if (hipMalloc((void **)&Ly.bias_dev, sizeof(float) * bias.size()) != hipSuccess) return DHQ_ENOMEM;
        if (hipMemcpy(Ly.wfrag_dev, frag.data(), sizeof(float) * frag.size(), hipMemcpyHostToDevice) != hipSuccess) return DHQ_EHIP;
        if (hipMemcpy(Ly.bias_dev, bias.data(), sizeof(float) * bias.size(), hipMemcpyHostToDevice) != hipSuccess) return DHQ_EHIP;
    }
    for (int i = 0; i < 2; ++i)
        if (hipMalloc((void **)&P->act[i], sizeof(float) * (size_t)DHQ_CHUNK * max_dim) != hipSuccess) return DHQ_ENOMEM;
    return DHQ_OK;
}

void dhq_float_destroy(dhq_float_plan *P)
{
    if (!P) return;
    if (P->blob_dev) (void)hipFree(P->blob_dev);
    for (int l = 0; l < DHQ_MAX_LAYERS; ++l) {
        if (P->lw[l].wfrag_dev) (void)hipFree(P->lw[l].wfrag_dev);
        if (P->lw[l].bias_dev) (void)hipFree(P->lw[l].bias_dev);
    }
    for (int i = 0; i < 2; ++i)
        if (P->act[i]) (void)hipFree(P->act[i]);
    delete P;
}

bool dhq_float_has_fused(const dhq_float_plan *P) { return P && P->nf != 0; }

template <int ACT>
static void float_layer_launch_act(int ntt, float c2, dim3 grid, hipStream_t st, const float *in, int64_t n, int K, int NG, int vec,
                                   const float4 *wf, int M, int Mt, const float *bias, float rev, float *out)
{
    switch (ntt) {
        case 1: float_layer_kernel<ACT, 1><<<grid, 64 * FLW_WAVES, 0, st>>>(in, n, K, NG, vec, wf, M, Mt, bias, rev, c2, out); break;
        case 2: float_layer_kernel<ACT, 2><<<grid, 64 * FLW_WAVES, 0, st>>>(in, n, K, NG, vec, wf, M, Mt, bias, rev, c2, out); break;
        case 3: float_layer_kernel<ACT, 3><<<grid, 64 * FLW_WAVES, 0, st>>>(in, n, K, NG, vec, wf, M, Mt, bias, rev, c2, out); break;
        default: float_layer_kernel<ACT, FLW_TILES><<<grid, 64 * FLW_WAVES, 0, st>>>(in, n, K, NG, vec, wf, M, Mt, bias, rev, c2, out); break;
    }
}
static void float_layer_launch(int ntt, dhq_act act, dim3 grid, hipStream_t st, const float *in, int64_t n, int K, int NG, int vec,
                               const float4 *wf, int M, int Mt, const float *bias, float rev, float *out)
{
    if (act.kind == DHQ_ACT_KIND_SINE) float_layer_launch_act<DHQ_ACT_KIND_SINE>(ntt, 0.f, grid, st, in, n, K, NG, vec, wf, M, Mt, bias, rev, out);
    else if (act.kind == DHQ_ACT_KIND_WAVELET) float_layer_launch_act<DHQ_ACT_KIND_WAVELET>(ntt, act.c2, grid, st, in, n, K, NG, vec, wf, M, Mt, bias, rev, out);
    else float_layer_launch_act<DHQ_ACT_KIND_NONE>(ntt, 0.f, grid, st, in, n, K, NG, vec, wf, M, Mt, bias, rev, out);
}

hipError_t dhq_float_launch_layerwise(const dhq_float_plan *P, const float *coords, int64_t n, float *out, hipStream_t st)
{
    if (!P) return hipErrorInvalidValue;
    const int L = P->n_layers;
    for (int64_t start = 0; start < n; start += DHQ_CHUNK) {
        const int64_t rows = (n - start < DHQ_CHUNK) ? n - start : DHQ_CHUNK;
        const float *cur = coords + start * P->lw[0].K;
        for (int l = 0; l < L; ++l) {
            const float_lw_layer &Ly = P->lw[l];
            float *dst = (l == L - 1) ? out + start * Ly.M : P->act[l & 1];
            const int ntt = Ly.Mt < FLW_TILES ? Ly.Mt : FLW_TILES;  // column tiles per wave
            const dim3 grid((unsigned)((rows + 32 * FLW_WAVES - 1) / (32 * FLW_WAVES)), (unsigned)((Ly.Mt + ntt - 1) / ntt));
            // one 16-byte load per lane needs rows that start on 16-byte boundaries
            const int vec = (Ly.K % 4 == 0 && ((uintptr_t)cur & 15) == 0) ? 1 : 0;
            const float4 *wf = reinterpret_cast<const float4 *>(Ly.wfrag_dev);
            const dhq_act act = (l == L - 1) ? dhq_act{DHQ_ACT_KIND_NONE, 0.f} : P->actf;
            float_layer_launch(ntt, act, grid, st, cur, rows, Ly.K, Ly.NG, vec, wf, Ly.M, Ly.Mt, Ly.bias_dev, P->rev, dst);
            const hipError_t e = hipGetLastError();
            if (e != hipSuccess) return e;
            cur = dst;
        }
    }
    return hipSuccess;
}

hipError_t dhq_float_launch(const dhq_float_plan *P, const float *coords, int64_t n, float *out, hipStream_t st)
{
    if (!P || P->nf == 0) return hipErrorInvalidValue;
    if (n <= 0) return hipSuccess;
    float_args a = P->args;
    a.coords = coords;
    a.out = out;
    a.n = n;
    const int64_t tiles = (n + FLT_TILE - 1) / FLT_TILE;
    const unsigned grid = (unsigned)(tiles < P->n_cu ? tiles : P->n_cu);
    const bool wav = (P->actf.kind == DHQ_ACT_KIND_WAVELET);
    switch (P->nf) {
        case 32:
            if (wav) dhq_float_kernel<32, DHQ_ACT_KIND_WAVELET><<<grid, FLT_THREADS, 0, st>>>(a);
            else dhq_float_kernel<32, DHQ_ACT_KIND_SINE><<<grid, FLT_THREADS, 0, st>>>(a);
            break;
        case 64:
            if (wav) dhq_float_kernel<64, DHQ_ACT_KIND_WAVELET><<<grid, FLT_THREADS, 0, st>>>(a);
            else dhq_float_kernel<64, DHQ_ACT_KIND_SINE><<<grid, FLT_THREADS, 0, st>>>(a);
            break;
        case 128:
            if (wav) dhq_float_kernel<128, DHQ_ACT_KIND_WAVELET><<<grid, FLT_THREADS, 0, st>>>(a);
            else dhq_float_kernel<128, DHQ_ACT_KIND_SINE><<<grid, FLT_THREADS, 0, st>>>(a);
            break;
        case 256:
            if (wav) dhq_float_kernel<256, DHQ_ACT_KIND_WAVELET><<<grid, FLT_THREADS, 0, st>>>(a);
            else dhq_float_kernel<256, DHQ_ACT_KIND_SINE><<<grid, FLT_THREADS, 0, st>>>(a);
            break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}
