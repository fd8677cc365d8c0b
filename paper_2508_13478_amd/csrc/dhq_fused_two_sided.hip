// Whole-network fused forward for the two-sided variant (weights rotated over input AND output
// features, Eq. 4-5 as printed), hidden widths 32 .. 256, gfx950.
//
// Same orientation as dhq_fused.hip: features are the MFMA M dimension, a wave carries 32
// coordinates through all layers in registers, lane (c, h) holds rows 8g + 4h + e of every
// 32-row tile T in registers R = 16T + 4g + e.  Per layer:
//   G   acc' = W'q q: all tiles accumulate straight into the lane's registers (as int32);
//   U   un-rotation z = H acc' over the output features, exactly in int32: butterflies over
//       the bits of R in place, then the stage over h with v_permlane32_swap on register pairs;
//   E   y = z c1 + b, a = sin(2 pi y) on every register;
//   W   the forward transform of the next layer's input (fp32): the 32-point factor inside
//       each tile as a product on the matrix unit, the stages over the tile index in
//       registers, then the quantizer.
// Index bookkeeping.  Call "location" (s, u) register s of lane half u.  Before U, location
// (R, h) holds rotated output m = 32T + 8g + 4h + e =: P0(R, h).  Butterflies over register
// bits are in place; the swap stage moves data: location (s, u) receives the h-butterfly of
// register (s & ~1) | u, output bit s & 1 -- i.e. the roles of bit 0 of s and of u are
// exchanged.  So after U, location (s, u) holds true feature f = P0((s & ~1) | u, s & 1)
// (= rot_index(s, u)); the biases are laid out accordingly.  W starts from that arrangement:
// the H_32 operand of its MFMAs is built for it, and an MFMA delivers its result in the
// accumulator layout, so after W location (s, u) holds rotated index P0(s, u) -- the natural
// accumulator order.  Hence the next layer's weights are packed with
// their k positions in P0 order, and again nothing is shuffled at run time.
//
// The output layer (fan-out padded to at most 32) is one tile whose rows are arranged so that its
// un-rotation is butterfly stages on the lane's sixteen accumulators plus, for 32 outputs, one
// exchange between the lane halves (f2_out_row).
#include <math.h>
#include <string.h>

#include <new>
#include <vector>

#include "dhq_device.h"
#include "dhq_fused_common.h"
#include "dhq_internal.h"

#define F2_WAVES 8
#define F2_THREADS (F2_WAVES * 64)
#define F2_TILE (F2_WAVES * 32)

struct f2_layer_desc {
    uint32_t blob_off;   // byte offset of the layer's block (A fragments, then 1 KiB of biases)
    uint32_t chunks;     // block size in KiB
    float c1;            // s_a s_w / sqrt(Mp) [omega0 / (2 pi) in sine layers]
    float inv_in;        // 1 / (s_a sqrt(Kp)) of this layer's input quantizer
};

struct f2_args {
    const float *coords;
    float *out;
    const unsigned char *blob;
    int64_t n;
    int n_layers;
    int k0, k0p;
    int m_out, m_out_p;  // fan-out of the output layer and its power-of-two padding (<= 32)
    int qmax;
    float c2;            // wavelet activation: 2 pi s0 sqrt(log2 e) / omega0
    f2_layer_desc layer[DHQ_MAX_LAYERS];
};

struct dhq_fused2_plan {
    int nf = 0;
    int act_kind = DHQ_ACT_KIND_SINE;  // the activation after every layer but the last
    unsigned char *blob_dev = nullptr;
    size_t blob_bytes = 0;
    f2_args args;
    size_t lds_bytes = 0;
    int n_cu = 0;
    int device = 0;
};

// ----------------------------------------------------------------------------- device code
// All tiles of one layer: x[16 T + v] = sum over k blocks.  Two tiles are accumulated
// alternately so that consecutive MFMAs do not depend on each other; A fragments are
// fetched from LDS PF MFMAs ahead.
template <int NT, int KB, int NCD>
__device__ __forceinline__ void f2_gemm(const dhq_v4i *__restrict__ wA, const dhq_v4i (&cd)[NCD], dhq_v16i (&acc)[NT], int lane)
{
    constexpr int NM = NT * KB;
    constexpr int PF = (NM >= 4) ? 4 : (NM >= 2 ? 2 : 1);
    constexpr int CH = (NT >= 2) ? 2 : 1;
    // MFMA number m -> (tile, k block): tiles in groups of CH, k blocks outer inside a group
    auto tile_of = [](int m) { return (m / (CH * KB)) * CH + (m % CH); };
    auto kb_of = [](int m) { return (m % (CH * KB)) / CH; };
    dhq_v4i fr[PF + 1];
#pragma unroll
    for (int m = 0; m < PF; ++m)
        if (m < NM) fr[m % (PF + 1)] = wA[(tile_of(m) * KB + kb_of(m)) * 64 + lane];
#pragma unroll
    for (int m = 0; m < NM; ++m) {
        const int T = tile_of(m), kb = kb_of(m);
        if (m + PF < NM) fr[(m + PF) % (PF + 1)] = wA[(tile_of(m + PF) * KB + kb_of(m + PF)) * 64 + lane];
        if (kb == 0) {
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[T][v] = 0;
        }
        acc[T] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fr[m % (PF + 1)], cd[kb], acc[T], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
    }
}

// A operand of the H_32 products of W: this lane supplies row c of H_32 at the contraction
// slots 8 h + j of block kk; slot j of lane half u carries the value at location (s, u),
// s % 16 = 8 kk + j, i.e. (after U) feature 8 ((s >> 2) & 3) + 4 (s & 1) + (s & 2) + u of its tile.
__device__ __forceinline__ void f2_h32_operand(int c, int h, dhq_v4i (&hA)[2])
{
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) {
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            const int v = 8 * kk + 2 * d;  // locations v (bit 0 clear) and v + 1
            const int i0 = 8 * (v >> 2) + (v & 2) + h;
            hA[kk][d] = (int)hm_h32_pair(c, i0, i0 + 4);
        }
    }
}

// Input layer: rotate the coordinate vector (fan-in <= 4) and quantize it; the four codes are
// bytes 0..3 of the first operand word.
__device__ __forceinline__ int f2_input_codes(const float *__restrict__ coords, int64_t cl, int k0, int k0p, float inv, int qmax)
{
    float v[4] = {0.f, 0.f, 0.f, 0.f};
    if (k0 == 2) {
        const float2 xy = *reinterpret_cast<const float2 *>(coords + cl * 2);
        v[0] = xy.x; v[1] = xy.y;
    } else {
        for (int k = 0; k < k0; ++k) v[k] = coords[cl * k0 + k];
    }
    if (k0p >= 2) {
        float a = v[0], b = v[1]; v[0] = a + b; v[1] = a - b;
        a = v[2]; b = v[3]; v[2] = a + b; v[3] = a - b;
    }
    if (k0p == 4) {
        float a = v[0], b = v[2]; v[0] = a + b; v[2] = a - b;
        a = v[1]; b = v[3]; v[1] = a + b; v[3] = a - b;
    }
    return (int)dhq_pack4(dhq_quant_bits(v[0], inv, qmax), dhq_quant_bits(v[1], inv, qmax), dhq_quant_bits(v[2], inv, qmax),
                          dhq_quant_bits(v[3], inv, qmax));
}

// One hidden layer, G to W: codes cd -> un-normalised transform xt of the layer's activations.
// wA: the layer's A fragments, wB: its biases in location order (both in LDS).
// ACTK: the activation (sine, or the wavelet with envelope constant c2).
template <int NT, int KB, int NCD, int ACTK>
__device__ __forceinline__ void f2_hidden_layer(const dhq_v4i *__restrict__ wA, const float4 *__restrict__ wB,
                                                const dhq_v4i (&cd)[NCD], float c1, const dhq_v4i (&hA)[2], dhq_v16f (&xt)[NT],
                                                int lane, int h, float c2)
{
    constexpr int NR = 16 * NT;
    // G: rotated accumulators of all output tiles
    dhq_v16i acc[NT];
    f2_gemm<NT, KB, NCD>(wA, cd, acc, lane);
    int z[NR];
#pragma unroll
    for (int T = 0; T < NT; ++T)
#pragma unroll
        for (int v = 0; v < 16; ++v) z[16 * T + v] = acc[T][v];
    // U: z = H acc' in int32 (wrapping adds; the host has checked that the results fit)
#pragma unroll
    for (int s = 1; s < NR; s <<= 1) {
#pragma unroll
        for (int i = 0; i < NR; ++i) {
            if ((i & s) == 0) {
                const unsigned a = (unsigned)z[i], b = (unsigned)z[i | s];
                z[i] = (int)(a + b);
                z[i | s] = (int)(a - b);
            }
        }
    }
    float x[NR];
    // the stage over the lane-half bit, then E: dequantize + bias + sine (biases in location order)
#pragma unroll
    for (int pr = 0; pr < NR / 2; ++pr) {
        const auto r = __builtin_amdgcn_permlane32_swap((unsigned)z[2 * pr], (unsigned)z[2 * pr + 1], false, false);
        const int z0 = (int)(r[0] + r[1]), z1 = (int)(r[0] - r[1]);
        const float4 bb = wB[(pr >> 1) * 2 + h];
        const float b0 = (pr & 1) ? bb.z : bb.x, b1 = (pr & 1) ? bb.w : bb.y;
        x[2 * pr] = dhq_activate_rev(__builtin_fmaf((float)z0, c1, b0), dhq_act{ACTK, c2});
        x[2 * pr + 1] = dhq_activate_rev(__builtin_fmaf((float)z1, c1, b1), dhq_act{ACTK, c2});
    }
    // W: forward transform of the next layer's input.  The factor H_32 over the 32 features of a
    // tile goes to the matrix unit as in dhq_fused.hip (activations split into two binary16
    // pieces, four MFMAs per tile); the stages over the tile index follow in registers.  The
    // MFMA's D layout is the natural accumulator order P0 again.
#pragma unroll
    for (int T = 0; T < NT; ++T) {
        unsigned hp[8], lp[8];
#pragma unroll
        for (int d = 0; d < 8; ++d) hm_split_pair(x[16 * T + 2 * d], x[16 * T + 2 * d + 1], hp[d], lp[d]);
        dhq_v16f acc_t;
#pragma unroll
        for (int v = 0; v < 16; ++v) acc_t[v] = 0.f;
#pragma unroll
        for (int k = 0; k < 4; ++k) {  // small pieces first: lo, hi of block 0, then of block 1
            const int blk = k >> 1;
            dhq_v4i b;
#pragma unroll
            for (int d = 0; d < 4; ++d) b[d] = (int)((k & 1) ? hp[4 * blk + d] : lp[4 * blk + d]);
            acc_t = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(dhq_v8h, hA[blk]), __builtin_bit_cast(dhq_v8h, b),
                                                           acc_t, 0, 0, 0);
        }
        xt[T] = acc_t;
    }
#pragma unroll
    for (int s = 1; s < NT; s <<= 1) {
#pragma unroll
        for (int T = 0; T < NT; ++T) {
            if ((T & s) == 0) {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const float a = xt[T][v], b = xt[T | s][v];
                    xt[T][v] = a + b;
                    xt[T | s][v] = a - b;
                }
            }
        }
    }
}

// Tile row that holds rotated output j (< 32) of the output layer: bits 0, 1 of j are the row-in-group e,
// bits 2, 3 the row group g and bit 4 the lane half, so that accumulator v = j % 16 of lane half j / 16
// holds it and the stages of the un-rotation over bits 0..3 of j never leave the lane.
static inline int f2_out_row(int j) { return 8 * ((j >> 2) & 3) + 4 * (j >> 4) + (j & 3); }

// Output layer: one zero-padded tile whose rows are arranged by f2_out_row; the (<= 32) rotated
// outputs are un-rotated by butterfly stages over the accumulator index and, for 32 of them, one
// exchange between the lane halves.  wB: the biases in plain order.
template <int NKB>
__device__ __forceinline__ void f2_output_layer(const dhq_v4i *__restrict__ wA, const float *__restrict__ wB,
                                                const dhq_v4i (&cd)[NKB], float c1, float *__restrict__ out, int64_t ci, bool valid,
                                                int m_out, int m_out_p, int lane, int h)
{
    dhq_v16i acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0;
#pragma unroll
    for (int kb = 0; kb < NKB; ++kb) {
        const dhq_v4i a = wA[kb * 64 + lane];
        acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, cd[kb], acc, 0, 0, 0);
    }
    unsigned z[16];
#pragma unroll
    for (int v = 0; v < 16; ++v) z[v] = (unsigned)acc[v];
#pragma unroll
    for (int s = 1; s < 16; s <<= 1) {
        if (m_out_p > s) {  // wave-uniform
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                if ((v & s) == 0) {
                    const unsigned a = z[v], b = z[v | s];
                    z[v] = a + b;
                    z[v | s] = a - b;
                }
            }
        }
    }
    if (m_out_p > 16) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const unsigned p = (unsigned)__shfl_xor((int)z[v], 32, 64);
            z[v] = h ? p - z[v] : z[v] + p;
        }
    }
    if (valid) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int j = 16 * h + v;
            if (j < m_out) out[ci * m_out + j] = __builtin_fmaf((float)(int)z[v], c1, wB[j]);
        }
    }
}

template <int NF, int ACTK>
__global__ __launch_bounds__(F2_THREADS) void dhq_fused2_kernel(const f2_args A)
{
    constexpr int NT = NF / 32;
    constexpr int NKB = NF / 32;
    constexpr int NR = NF / 2;
    constexpr int BLK = (NT * NKB + 1) * 1024;

    extern __shared__ __align__(16) unsigned char lds[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = lane & 31, h = lane >> 5;
    const int L = A.n_layers;
    const int64_t n_tiles = (A.n + F2_TILE - 1) / F2_TILE;
    const int qlo = DHQ_MAGIC_I - A.qmax, qhi = DHQ_MAGIC_I + A.qmax;

    dhq_v4i hA[2];
    f2_h32_operand(c, h, hA);

    int p = 0;
    if ((int64_t)blockIdx.x < n_tiles)
        fused_issue_copy(A.blob + A.layer[0].blob_off, lds, (int)A.layer[0].chunks, wave, lane, F2_WAVES);

    for (int64_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const int64_t ci = tile * F2_TILE + wave * 32 + c;
        const bool valid = ci < A.n;
        const int64_t cl = valid ? ci : A.n - 1;

        dhq_v4i cd[NKB];
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb) cd[kb] = dhq_v4i{0, 0, 0, 0};
        cd[0][0] = f2_input_codes(A.coords, cl, A.k0, A.k0p, A.layer[0].inv_in, A.qmax);

        for (int l = 0; l < L - 1; ++l) {
            // weights of layer l have landed; everyone is done with the other buffer
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();
            {
                const f2_layer_desc &nx = A.layer[l + 1];
                fused_issue_copy(A.blob + nx.blob_off, lds + (p ^ 1) * BLK, (int)nx.chunks, wave, lane, F2_WAVES);
            }
            const dhq_v4i *wA = reinterpret_cast<const dhq_v4i *>(lds + p * BLK);
            const int Kb = (l == 0) ? 1 : NKB;
            const float4 *wB = reinterpret_cast<const float4 *>(lds + p * BLK + NT * Kb * 1024);
            dhq_v16f xt[NT];
            if (l == 0)
                f2_hidden_layer<NT, 1, NKB, ACTK>(wA, wB, cd, A.layer[l].c1, hA, xt, lane, h, A.c2);
            else
                f2_hidden_layer<NT, NKB, NKB, ACTK>(wA, wB, cd, A.layer[l].c1, hA, xt, lane, h, A.c2);
            // the next layer's quantizer
            const float inv = A.layer[l + 1].inv_in;
#pragma unroll
            for (int w = 0; w < NR / 4; ++w) {
                const int v = 4 * (w & 3);
                cd[w / 4][w % 4] = (int)fused_quant4(xt[w >> 2][v], xt[w >> 2][v + 1], xt[w >> 2][v + 2], xt[w >> 2][v + 3], inv, qlo, qhi);
            }
            p ^= 1;
        }

        {
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();
            if (tile + gridDim.x < n_tiles)
                fused_issue_copy(A.blob + A.layer[0].blob_off, lds + (p ^ 1) * BLK, (int)A.layer[0].chunks, wave, lane, F2_WAVES);
            f2_output_layer<NKB>(reinterpret_cast<const dhq_v4i *>(lds + p * BLK), reinterpret_cast<const float *>(lds + p * BLK + NKB * 1024),
                                 cd, A.layer[L - 1].c1, A.out, ci, valid, A.m_out, A.m_out_p, lane, h);
            p ^= 1;
        }
    }
}

// With scales measured on line the network is cut at every quantizer, as in dhq_fused.hip: one
// launch per layer folds the per-workgroup maxima of its input into the layer's constants,
// quantizes, runs G, U, E and W of the layer and stores the transformed output x^ (fp32, in the
// lanes' register order: [wave tile][float4 q][lane]) plus each workgroup's max |x^|.
//   MODE 0  input layer: coordinates in, x^ out        MODE 1  hidden layer: x^ in, x^ out
//   MODE 2  output layer: x^ in, signal values out
struct f2l_args {
    const float *coords;       // MODE 0
    const float4 *xin;         // MODE 1, 2
    float4 *xout;              // MODE 0, 1
    float *out;                // MODE 2
    const unsigned char *blk;  // this layer's block of the packed weights (fragments, then biases)
    const float *partial_in;   // max |x^| of this layer's input, one float per workgroup of the launch before
    int partial_count;
    int kp;                    // length of this layer's rotated input
    double c1_over_sa;         // epilogue multiplier divided by the activation scale
    float *dyn;                // this layer's {1 / (s_a sqrt(Kp)), epilogue multiplier, s_a}: written by workgroup 0
    float *partial;            // MODE 0, 1: max |x^| of the output per workgroup (not the buffer partial_in points to)
    int64_t n;
    int chunks;                // block size in KiB
    int k0, k0p, m_out, m_out_p, qmax;
    float c2;                  // wavelet activation: 2 pi s0 sqrt(log2 e) / omega0
};

// ACTK: the activation after the layer (MODE 0, 1).
template <int NF, int MODE, int ACTK>
__global__ __launch_bounds__(F2_THREADS) void dhq_fused2_layer_kernel(const f2l_args A)
{
    constexpr int NT = NF / 32, NKB = NF / 32, NR = NF / 2;
    constexpr int KB = (MODE == 0) ? 1 : NKB;  // k blocks of this layer's GEMM
    constexpr int MT = (MODE == 2) ? 1 : NT;   // M tiles of this layer's GEMM
    extern __shared__ __align__(16) unsigned char lds[];
    __shared__ float red_in[F2_WAVES], red[F2_WAVES];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = lane & 31, h = lane >> 5;
    const int64_t n_tiles = (A.n + F2_TILE - 1) / F2_TILE;
    const int qlo = DHQ_MAGIC_I - A.qmax, qhi = DHQ_MAGIC_I + A.qmax;
    dhq_v4i hA[2];
    f2_h32_operand(c, h, hA);
    fused_issue_copy(A.blk, lds, A.chunks, wave, lane, F2_WAVES);
    // this layer's constants from the maxima of its input
    float inv, c1, s_a;
    {
        float mi = 0.f;
        for (int i = threadIdx.x; i < A.partial_count; i += F2_THREADS) mi = fmaxf(mi, A.partial_in[i]);
#pragma unroll
        for (int m = 1; m < 64; m *= 2) mi = fmaxf(mi, __shfl_xor(mi, m, 64));
        if (lane == 0) red_in[wave] = mi;
        __syncthreads();
        mi = red_in[0];
#pragma unroll
        for (int w = 1; w < F2_WAVES; ++w) mi = fmaxf(mi, red_in[w]);
        dhq_dyn_constants(mi, A.kp, A.qmax, A.c1_over_sa, inv, c1, s_a);
        if (blockIdx.x == 0 && threadIdx.x == 0) {
            A.dyn[0] = inv; A.dyn[1] = c1; A.dyn[2] = s_a;
        }
    }
    const dhq_v4i *wA = reinterpret_cast<const dhq_v4i *>(lds);
    float mx = 0.f;
    bool landed = false;
    for (int64_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const int64_t ci = tile * F2_TILE + wave * 32 + c;
        const bool valid = ci < A.n;
        const int64_t cl = valid ? ci : A.n - 1;  // lanes past the end repeat the last coordinate: no effect on the maximum
        const size_t slot = ((size_t)tile * F2_WAVES + wave) * (NR / 4) * 64 + lane;
        dhq_v4i cd[NKB];
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb) cd[kb] = dhq_v4i{0, 0, 0, 0};
        if constexpr (MODE == 0) {
            cd[0][0] = f2_input_codes(A.coords, cl, A.k0, A.k0p, inv, A.qmax);
        } else {
#pragma unroll
            for (int q = 0; q < NR / 4; ++q) {
                const float4 x = A.xin[slot + (size_t)q * 64];
                cd[q / 4][q % 4] = (int)fused_quant4(x.x, x.y, x.z, x.w, inv, qlo, qhi);
            }
        }
        if (!landed) {
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();  // the weights are in LDS
            landed = true;
        }
        if constexpr (MODE == 2) {
            f2_output_layer<NKB>(wA, reinterpret_cast<const float *>(lds + MT * KB * 1024), cd, c1, A.out, ci, valid, A.m_out,
                                 A.m_out_p, lane, h);
        } else {
            dhq_v16f xt[NT];
            f2_hidden_layer<NT, KB, NKB, ACTK>(wA, reinterpret_cast<const float4 *>(lds + MT * KB * 1024), cd, c1, hA, xt, lane, h, A.c2);
#pragma unroll
            for (int q = 0; q < NR / 4; ++q) {
                const float4 x = make_float4(xt[q >> 2][4 * (q & 3)], xt[q >> 2][4 * (q & 3) + 1], xt[q >> 2][4 * (q & 3) + 2],
                                             xt[q >> 2][4 * (q & 3) + 3]);
                mx = fmaxf(fmaxf(mx, fmaxf(fabsf(x.x), fabsf(x.y))), fmaxf(fabsf(x.z), fabsf(x.w)));
                A.xout[slot + (size_t)q * 64] = x;
            }
        }
    }
    if constexpr (MODE != 2) {
#pragma unroll
        for (int m = 1; m < 64; m *= 2) mx = fmaxf(mx, __shfl_xor(mx, m, 64));
        if (lane == 0) red[wave] = mx;
        __syncthreads();
        if (threadIdx.x == 0) {
            float r = red[0];
#pragma unroll
            for (int w = 1; w < F2_WAVES; ++w) r = fmaxf(r, red[w]);
            A.partial[blockIdx.x] = r;
        }
    }
}

// ---- test hook: one layer of the whole-network kernel on caller-supplied codes ---------------
// The layer body is f2_hidden_layer and the quantizer as dhq_fused2_kernel runs them, on the same
// packed weights; the codes come in from a row-major n x Kp array (rotated-feature order) and the
// un-normalised transform x^ of the layer's output, the next layer's codes and the rotated
// accumulators (from a second, plain MFMA loop) go out to row-major n x NF arrays.
struct f2d_args {
    const int8_t *codes_in;
    const unsigned char *blk;
    float *xhat;
    int8_t *codes_out;
    int32_t *acc;
    int64_t n;
    int chunks, kp_in, qmax;
    float c1, inv_next, c2;
};

template <int NF, bool FIRST, int ACTK>
__global__ __launch_bounds__(F2_THREADS) void dhq_fused2_debug_kernel(const f2d_args A)
{
    constexpr int NT = NF / 32, NKB = NF / 32, NR = NF / 2;
    constexpr int KB = FIRST ? 1 : NKB;
    extern __shared__ __align__(16) unsigned char lds[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = lane & 31, h = lane >> 5;
    const int qlo = DHQ_MAGIC_I - A.qmax, qhi = DHQ_MAGIC_I + A.qmax;
    dhq_v4i hA[2];
    f2_h32_operand(c, h, hA);
    fused_issue_copy(A.blk, lds, A.chunks, wave, lane, F2_WAVES);
    const int64_t ci = (int64_t)blockIdx.x * F2_TILE + wave * 32 + c;
    const bool valid = ci < A.n;
    const int64_t cl = valid ? ci : A.n - 1;
    dhq_v4i cd[NKB];
#pragma unroll
    for (int kb = 0; kb < NKB; ++kb) cd[kb] = dhq_v4i{0, 0, 0, 0};
    if constexpr (FIRST) {
        unsigned w = 0;
        for (int k = 0; k < A.kp_in; ++k) w |= (unsigned)(uint8_t)A.codes_in[cl * A.kp_in + k] << (8 * k);
        cd[0][0] = (int)w;
    } else {
#pragma unroll
        for (int s = 0; s < NR; ++s) {
            const int f = 32 * (s >> 4) + 8 * ((s >> 2) & 3) + 4 * h + (s & 3);  // rotated feature of register s
            const unsigned byte = (unsigned)(uint8_t)A.codes_in[cl * A.kp_in + f];
            cd[s >> 4][(s >> 2) & 3] |= (int)(byte << (8 * (s & 3)));
        }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    const dhq_v4i *wA = reinterpret_cast<const dhq_v4i *>(lds);
    if (A.acc) {
#pragma unroll
        for (int T = 0; T < NT; ++T) {
            dhq_v16i acc;
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[v] = 0;
#pragma unroll
            for (int kb = 0; kb < KB; ++kb) acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(wA[(T * KB + kb) * 64 + lane], cd[kb], acc, 0, 0, 0);
            if (valid) {
#pragma unroll
                for (int v = 0; v < 16; ++v) A.acc[ci * NF + 32 * T + 8 * (v >> 2) + 4 * h + (v & 3)] = acc[v];
            }
        }
    }
    dhq_v16f xt[NT];
    f2_hidden_layer<NT, KB, NKB, ACTK>(wA, reinterpret_cast<const float4 *>(lds + NT * KB * 1024), cd, A.c1, hA, xt, lane, h, A.c2);
#pragma unroll
    for (int w = 0; w < NR / 4; ++w) {
        const int v = 4 * (w & 3);
        cd[w / 4][w % 4] = (int)fused_quant4(xt[w >> 2][v], xt[w >> 2][v + 1], xt[w >> 2][v + 2], xt[w >> 2][v + 3], A.inv_next, qlo, qhi);
    }
    if (valid) {
#pragma unroll
        for (int s = 0; s < NR; ++s) {
            const int f = 32 * (s >> 4) + 8 * ((s >> 2) & 3) + 4 * h + (s & 3);
            if (A.xhat) A.xhat[ci * NF + f] = xt[s >> 4][s & 15];
            if (A.codes_out) A.codes_out[ci * NF + f] = (int8_t)(((unsigned)cd[s >> 4][(s >> 2) & 3] >> (8 * (s & 3))) & 0xffu);
        }
    }
}

// ------------------------------------------------------------------------------- host code
// Natural accumulator order: rotated index held by register s of lane half u.
static int p0_index(int s, int u) { return 32 * (s >> 4) + 8 * ((s >> 2) & 3) + 4 * u + (s & 3); }

static bool fused2_shape_ok(const dhq_model *m, int *nf_out)
{
    const int L = m->n_layers;
    if (!m->rot_out || L < 2) return false;
    if (m->dims[0] > 4 || m->dims[L] > 32) return false;
    const int nf = m->dims[1];
    if (nf != 32 && nf != 64 && nf != 128 && nf != 256) return false;
    for (int l = 1; l < L; ++l)
        if (m->dims[l] != nf) return false;
    *nf_out = nf;
    return true;
}

int dhq_fused2_create(const dhq_model *m, dhq_fused2_plan **plan_out)
{
    *plan_out = nullptr;
    int nf = 0;
    if (!fused2_shape_ok(m, &nf)) return DHQ_OK;
    const int L = m->n_layers;
    const int NT = nf / 32, NKB = nf / 32;
    dhq_fused2_plan *P = new (std::nothrow) dhq_fused2_plan();
    if (!P) return DHQ_ENOMEM;
    P->nf = nf;
    memset(&P->args, 0, sizeof(P->args));
    std::vector<unsigned char> blob;
    for (int l = 0; l < L; ++l) {
        const dhq_layer &Ly = m->layer[l];
        const int Mt = (l == L - 1) ? 1 : NT;
        const int Kb = (l == 0) ? 1 : NKB;
        const size_t off = blob.size();
        const size_t bytes = (size_t)(Mt * Kb + 1) * 1024;
        blob.resize(off + bytes, 0);
        int8_t *frag = reinterpret_cast<int8_t *>(blob.data() + off);
        const int8_t *wq = Ly.wq_host.data();  // Mp x Kp, rows = rotated output index
        for (int T = 0; T < Mt; ++T)
            for (int kb = 0; kb < Kb; ++kb)
                for (int ln = 0; ln < 64; ++ln) {
                    // rotated output index this lane's A row stands for: tile rows in natural order, except in the
                    // output layer, whose rows are arranged for the in-lane un-rotation (inverse of f2_out_row)
                    const int tr = ln & 31, u = ln >> 5;
                    const int row = (l == L - 1) ? ((tr & 3) | ((tr >> 3) << 2) | (((tr >> 2) & 1) << 4)) : 32 * T + tr;
                    for (int jj = 0; jj < 16; ++jj) {
                        int8_t val = 0;
                        if (row < Ly.Mg) {
                            if (l == 0) {
                                if (u == 0 && jj < Ly.Kp) val = wq[(size_t)row * Ly.Kp + jj];
                            } else {
                                val = wq[(size_t)row * Ly.Kp + p0_index(16 * kb + jj, u)];
                            }
                        }
                        frag[((size_t)(T * Kb + kb) * 64 + ln) * 16 + jj] = val;
                    }
                }
        // the bias part of the block.  Hidden layers: location (s, u) holds true feature
        // rot_index(s, u) after the un-rotation, and lane half u reads the biases of registers
        // s .. s+3 as one float4 at index (s / 4) * 2 + u.  Output layer: plain order.
        {
            float *blk = reinterpret_cast<float *>(blob.data() + off + (size_t)Mt * Kb * 1024);
            if (l == L - 1) {
                for (int f = 0; f < Ly.M; ++f) blk[f] = Ly.bias_host[f];
            } else {
                for (int s = 0; s < nf / 2; ++s)
                    for (int u = 0; u < 2; ++u) {
                        const int f = rot_index(s, u);
                        if (f < Ly.M) blk[((s >> 2) * 2 + u) * 4 + (s & 3)] = Ly.bias_rev_host[f];
                    }
            }
        }
        P->args.layer[l].blob_off = (uint32_t)off;
        P->args.layer[l].chunks = (uint32_t)(bytes / 1024);
    }
    P->blob_bytes = blob.size();
    if (hipMalloc((void **)&P->blob_dev, P->blob_bytes) != hipSuccess) {
        delete P;
        return DHQ_ENOMEM;
    }
    if (hipMemcpy(P->blob_dev, blob.data(), P->blob_bytes, hipMemcpyHostToDevice) != hipSuccess) {
        (void)hipFree(P->blob_dev);
        delete P;
        return DHQ_EHIP;
    }
    P->args.blob = P->blob_dev;
    P->args.n_layers = L;
    P->args.k0 = m->dims[0];
    P->args.k0p = m->layer[0].Kp;
    P->args.m_out = m->dims[L];
    P->args.m_out_p = m->layer[L - 1].Mp;
    P->args.qmax = m->qmax_a;
    P->args.c2 = dhq_hidden_act(m).c2;
    P->act_kind = m->act_kind;
    P->lds_bytes = (size_t)2 * (NT * NKB + 1) * 1024;
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, m->device) != hipSuccess) {
        (void)hipFree(P->blob_dev);
        delete P;
        return DHQ_EHIP;
    }
    P->n_cu = prop.multiProcessorCount;
    P->device = m->device;
    *plan_out = P;
    return DHQ_OK;
}

void dhq_fused2_destroy(dhq_fused2_plan *P)
{
    if (!P) return;
    if (P->blob_dev) (void)hipFree(P->blob_dev);
    delete P;
}

// Per-layer constants of the static path.
int dhq_fused2_update_scales(const dhq_model *m, dhq_fused2_plan *P)
{
    if (!P) return DHQ_OK;
    for (int l = 0; l < m->n_layers; ++l) {
        P->args.layer[l].c1 = dhq_c1(m, l);
        P->args.layer[l].inv_in = (float)(1.0 / ((double)m->layer[l].s_a * sqrt((double)m->layer[l].Kp)));
    }
    return DHQ_OK;
}

template <int NF, int ACTK>
static hipError_t fused2_launch_act(const dhq_fused2_plan *P, const f2_args &a, unsigned grid, hipStream_t st)
{
    auto kern = dhq_fused2_kernel<NF, ACTK>;
    hipError_t e = dhq_lds_limit_once(kern, P->lds_bytes, P->device);
    if (e != hipSuccess) return e;
    kern<<<grid, F2_THREADS, P->lds_bytes, st>>>(a);
    return hipGetLastError();
}
template <int NF>
static hipError_t fused2_launch_t(const dhq_fused2_plan *P, const f2_args &a, unsigned grid, hipStream_t st)
{
    return P->act_kind == DHQ_ACT_KIND_WAVELET ? fused2_launch_act<NF, DHQ_ACT_KIND_WAVELET>(P, a, grid, st)
                                               : fused2_launch_act<NF, DHQ_ACT_KIND_SINE>(P, a, grid, st);
}

hipError_t dhq_fused2_launch(const dhq_fused2_plan *P, const float *coords, int64_t n, float *out, hipStream_t st)
{
    if (!P) return hipErrorInvalidValue;
    if (n <= 0) return hipSuccess;
    f2_args a = P->args;
    a.coords = coords;
    a.out = out;
    a.n = n;
    const int64_t tiles = (n + F2_TILE - 1) / F2_TILE;
    const unsigned grid = (unsigned)(tiles < P->n_cu ? tiles : P->n_cu);
    switch (P->nf) {
        case 32: return fused2_launch_t<32>(P, a, grid, st);
        case 64: return fused2_launch_t<64>(P, a, grid, st);
        case 128: return fused2_launch_t<128>(P, a, grid, st);
        case 256: return fused2_launch_t<256>(P, a, grid, st);
        default: return hipErrorInvalidValue;
    }
}

// The dynamic mode on the per-layer kernels; arguments as for dhq_fused_dynamic_launch.
size_t dhq_fused2_dynamic_rows(int64_t n) { return (size_t)((n + F2_TILE - 1) / F2_TILE) * F2_TILE; }

template <int NF, int MODE, int ACTK>
static hipError_t f2l_launch_t(const f2l_args &a, unsigned grid, int device, hipStream_t st)
{
    auto kern = dhq_fused2_layer_kernel<NF, MODE, ACTK>;
    const size_t lds = (size_t)a.chunks * 1024;
    hipError_t e = dhq_lds_limit_once(kern, lds, device);
    if (e != hipSuccess) return e;
    kern<<<grid, F2_THREADS, lds, st>>>(a);
    return hipGetLastError();
}
template <int NF>
static hipError_t f2l_launch_mode(int mode, int act_kind, const f2l_args &a, unsigned grid, int device, hipStream_t st)
{
    const bool wav = (act_kind == DHQ_ACT_KIND_WAVELET);
    switch (mode) {
        case 0: return wav ? f2l_launch_t<NF, 0, DHQ_ACT_KIND_WAVELET>(a, grid, device, st) : f2l_launch_t<NF, 0, DHQ_ACT_KIND_SINE>(a, grid, device, st);
        case 1: return wav ? f2l_launch_t<NF, 1, DHQ_ACT_KIND_WAVELET>(a, grid, device, st) : f2l_launch_t<NF, 1, DHQ_ACT_KIND_SINE>(a, grid, device, st);
        default: return f2l_launch_t<NF, 2, DHQ_ACT_KIND_NONE>(a, grid, device, st);  // the output layer has no activation
    }
}

hipError_t dhq_fused2_dynamic_launch(const dhq_model *m, const float *coords, int64_t n, float *out, float *ws0, float *ws1,
                                     float *partial, float *dyn, hipStream_t st)
{
    const dhq_fused2_plan *P = m->fused2;
    if (!P) return hipErrorInvalidValue;
    if (n <= 0) return hipSuccess;
    const int L = m->n_layers;
    const int64_t tiles = (n + F2_TILE - 1) / F2_TILE;
    const unsigned grid = (unsigned)(tiles < P->n_cu ? tiles : P->n_cu);
    // the input layer's scale: max over the rotated coordinates, left as per-workgroup maxima
    float *pbuf[2] = {partial, partial + DHQ_ABSMAX_PARTIALS};
    int count = 0;
    hipError_t e = dhq_launch_wht_absmax_partials(coords, n, m->layer[0].K, m->layer[0].Kp, pbuf[0], &count, st);
    if (e != hipSuccess) return e;
    float *bufs[2] = {ws0, ws1};
    for (int l = 0; l < L; ++l) {
        f2l_args a;
        memset(&a, 0, sizeof(a));
        a.coords = coords;
        a.xin = reinterpret_cast<const float4 *>(bufs[(l + 1) & 1]);
        a.xout = reinterpret_cast<float4 *>(bufs[l & 1]);
        a.out = out;
        a.blk = P->blob_dev + P->args.layer[l].blob_off;
        a.chunks = (int)P->args.layer[l].chunks;
        a.partial_in = pbuf[l & 1];
        a.partial_count = count;
        a.kp = m->layer[l].Kp;
        a.c1_over_sa = dhq_c1_over_sa(m, l);
        a.dyn = dyn + 3 * l;
        a.partial = pbuf[(l + 1) & 1];
        a.n = n;
        a.k0 = P->args.k0; a.k0p = P->args.k0p; a.m_out = P->args.m_out; a.m_out_p = P->args.m_out_p; a.qmax = P->args.qmax;
        a.c2 = P->args.c2;
        const int mode = (l == 0) ? 0 : (l == L - 1 ? 2 : 1);
        switch (P->nf) {
            case 32: e = f2l_launch_mode<32>(mode, m->act_kind, a, grid, P->device, st); break;
            case 64: e = f2l_launch_mode<64>(mode, m->act_kind, a, grid, P->device, st); break;
            case 128: e = f2l_launch_mode<128>(mode, m->act_kind, a, grid, P->device, st); break;
            case 256: e = f2l_launch_mode<256>(mode, m->act_kind, a, grid, P->device, st); break;
            default: e = hipErrorInvalidValue;
        }
        if (e != hipSuccess) return e;
        count = (int)grid;
    }
    return hipSuccess;
}

// Test hook behind dhq_forward_debug_fused for the two-sided whole-network kernel.
template <int NF, bool FIRST, int ACTK>
static hipError_t f2d_launch_t(const f2d_args &a, unsigned grid, int device, hipStream_t st)
{
    auto kern = dhq_fused2_debug_kernel<NF, FIRST, ACTK>;
    const size_t lds = (size_t)a.chunks * 1024;
    hipError_t e = dhq_lds_limit_once(kern, lds, device);
    if (e != hipSuccess) return e;
    kern<<<grid, F2_THREADS, lds, st>>>(a);
    return hipGetLastError();
}
template <int NF>
static hipError_t f2d_launch_nf(bool first, int act_kind, const f2d_args &a, unsigned grid, int device, hipStream_t st)
{
    const bool wav = (act_kind == DHQ_ACT_KIND_WAVELET);
    if (first) return wav ? f2d_launch_t<NF, true, DHQ_ACT_KIND_WAVELET>(a, grid, device, st) : f2d_launch_t<NF, true, DHQ_ACT_KIND_SINE>(a, grid, device, st);
    return wav ? f2d_launch_t<NF, false, DHQ_ACT_KIND_WAVELET>(a, grid, device, st) : f2d_launch_t<NF, false, DHQ_ACT_KIND_SINE>(a, grid, device, st);
}

hipError_t dhq_fused2_debug_launch(const dhq_model *m, int layer, const int8_t *codes_in, int64_t n, float *xhat, int8_t *codes_out,
                                   int32_t *acc, hipStream_t st)
{
    const dhq_fused2_plan *P = m->fused2;
    if (!P || layer < 0 || layer >= m->n_layers - 1) return hipErrorInvalidValue;
    if (n <= 0) return hipSuccess;
    f2d_args a;
    memset(&a, 0, sizeof(a));
    a.codes_in = codes_in;
    a.blk = P->blob_dev + P->args.layer[layer].blob_off;
    a.chunks = (int)P->args.layer[layer].chunks;
    a.xhat = xhat;
    a.codes_out = codes_out;
    a.acc = acc;
    a.n = n;
    a.kp_in = m->layer[layer].Kp;
    a.qmax = P->args.qmax;
    a.c1 = P->args.layer[layer].c1;
    a.inv_next = P->args.layer[layer + 1].inv_in;
    a.c2 = P->args.c2;
    const unsigned grid = (unsigned)((n + F2_TILE - 1) / F2_TILE);
    switch (P->nf) {
        case 32: return f2d_launch_nf<32>(layer == 0, m->act_kind, a, grid, P->device, st);
        case 64: return f2d_launch_nf<64>(layer == 0, m->act_kind, a, grid, P->device, st);
        case 128: return f2d_launch_nf<128>(layer == 0, m->act_kind, a, grid, P->device, st);
        case 256: return f2d_launch_nf<256>(layer == 0, m->act_kind, a, grid, P->device, st);
        default: return hipErrorInvalidValue;
    }
}
