// Whole-network fused DHQ forward for gfx950 (paper Sec. 3.3 pipeline: input layer, linear
// layers with a quantization module between them, output layer -- here one kernel).
//
// Every wave owns 32 coordinates and carries them through all layers without their
// activations ever leaving registers; device-memory traffic is the coordinates in and the
// signal values out.  The only shared state is the current layer's weights in LDS.
//
// Data layout.  The GEMM runs "features x coordinates": the int8 weights are the A operand
// of v_mfma_i32_32x32x32_i8 (32 output features x 32 k), the activation codes the B operand
// (32 k x 32 coordinates).  With that orientation lane l of a wave holds, for coordinate
// l % 32, accumulator rows 8g + 4h + e (g = 0..3, h = l / 32, e = 0..3) of every 32-row
// tile T: half of the feature vector of one coordinate, in registers R = 16T + 4g + e.
// The Walsh-Hadamard transform over the feature index (Eq. 3) factors as H_NF = H_NT (x) H_32
// and is done in two parts:
//   - H_32 over the 32 rows of each tile on the matrix unit (see fused_gemm_sine_hm below):
//     the tile's activations are already laid out as an MFMA B operand, H_32 is the A operand;
//   - log2(NT) butterfly stages over the tile index, i.e. over bits 4.. of R: plain register
//     add/sub, no lane traffic.
// After the last stage register s of lane half u holds rotated feature j(s, u) (hm_index in
// dhq_fused_common.h); quantizing register s into byte s % 4 of dword s / 4 makes four consecutive dwords
// exactly the B operand of k block s / 16.  The contraction index of an MFMA can be enumerated
// in any order as long as both operands agree, so the weights are packed offline with their k
// positions permuted by j(s, u) and nothing is ever shuffled at run time.
//
// The first layer (fan-in <= 4) and the output layer (fan-out <= 32) use the same
// machinery with the k block / the M tile zero-padded.
//
// Weights: each layer's A fragments ([tile][k block][lane] x 16 B) followed by its biases
// form one contiguous block; while layer l computes, the block of layer l+1 is copied from
// device memory (L2-resident) straight into the other LDS buffer with 16-byte
// global->LDS loads, so the copy costs no registers and no VALU work.
#include <math.h>
#include <string.h>

#include <vector>

#include "dhq_device.h"
#include "dhq_fused_common.h"
#include "dhq_internal.h"

#define FUSED_WAVES 8            // waves per workgroup, two per SIMD
#define FUSED_THREADS (FUSED_WAVES * 64)
#define FUSED_TILE (FUSED_WAVES * 32)  // coordinates per workgroup pass

struct fused_layer_desc {
    uint32_t blob_off;   // byte offset of the layer's block in the packed weight blob
    uint32_t chunks;     // block size in KiB (1 KiB = what one wave copies per instruction)
    float c1;            // sine layers: s_a s_w omega0 / (2 pi); output layer: s_a s_w
    float inv_in;        // 1 / (s_a sqrt(Kp)) of this layer's input quantizer
};

struct fused_args {
    const float *coords;
    float *out;
    const unsigned char *blob;
    int64_t n;
    int n_layers;
    int k0, k0p;   // fan-in of the first layer and its power-of-two padding (<= 4)
    int m_out;     // fan-out of the output layer (<= 32)
    int qmax;
    float c2;      // wavelet activation: 2 pi s0 sqrt(log2 e) / omega0
    fused_layer_desc layer[DHQ_MAX_LAYERS];
};

struct dhq_fused_plan {
    int nf = 0;                      // hidden width
    unsigned char *blob_dev = nullptr;
    size_t blob_bytes = 0;
    fused_args args;
    size_t lds_bytes = 0;
    int n_cu = 0;
    int device = 0;
};

// ---- the in-tile part of the transform on the matrix unit ------------------------------------
// The 32 features of an M tile are one factor of the Sylvester matrix, H_NF = H_NT (x) H_32, so
// the five butterfly stages over the within-tile index (four over register bits, one over the
// lane half) are the product H_32 * (tile of activations): a 32 x 32 x 32 contraction whose B
// operand the lanes already hold.  The matrix unit has no fp32 input at a useful rate, so an
// activation a (|a| <= 1) is split into two binary16 pieces, hi = a rounded toward zero and
// lo = (a - hi) rounded toward zero (a - hi is exact in fp32), which carry a to within 2^-21 |a|
// (2^-24 absolute below 2^-10, where lo is subnormal; v_mfma_f32_32x32x16_f16 takes subnormal
// inputs as they are).  That is up to four units in the last place of a, still below the error
// of the sine that produced a, and the rotated activations come out with about the same error
// as from fp32 butterflies (1.3e-6 against 0.9e-6 rms at width 256, un-normalised).  The
// products with +-1 are exact and the sum is accumulated in fp32 like
// the butterflies' sums.  Per tile: 8 + 8 packed conversions, 16 mixed-precision subtractions
// and 4 MFMAs replace 80 add/sub and 8 lane swaps.  The three stages over the tile index stay
// on the vector ALU.  Afterwards register s of lane half u holds rotated feature hm_index(s, u).
template <int NT, int KB>
struct hm_sched {
    static constexpr bool STAGGER = (NT >= 2 && KB >= 2);
    static constexpr int STEPS = (STAGGER ? (NT / 2) * 2 * KB + KB + 1 : NT * KB) + KB + 6;
    static constexpr int NM = NT * KB;
    int tile[STEPS], kb[STEPS], seq[STEPS];   // GEMM MFMA issued at this step (tile -1: none)
    int drain[STEPS], drain_pos[STEPS];       // tile drained at this step and which slice of it
    int hm_n[STEPS], hm_tile[STEPS][4], hm_k[STEPS][4];  // transform MFMAs issued at this step
    int seq_tile[NM], seq_kb[NM];
    int last;                                 // last step with any work
    constexpr hm_sched()
        : tile(), kb(), seq(), drain(), drain_pos(), hm_n(), hm_tile(), hm_k(), seq_tile(), seq_kb(), last(0)
    {
        int done[NT > 0 ? NT : 1] = {};
        for (int g = 0; g < STEPS; ++g) { tile[g] = -1; kb[g] = 0; seq[g] = -1; drain[g] = -1; drain_pos[g] = 0; hm_n[g] = 0; }
        for (int t = 0; t < NT; ++t) {
            const int i = t / 2;
            const int base = (t & 1) ? 2 * KB * i + KB + 1 : 2 * KB * i;
            for (int k = 0; k < KB; ++k) {
                const int g = STAGGER ? base + 2 * k : t * KB + k;
                tile[g] = t; kb[g] = k; done[t] = g;
            }
        }
        int m = 0;
        for (int g = 0; g < STEPS; ++g)
            if (tile[g] >= 0) { seq[g] = m; seq_tile[m] = tile[g]; seq_kb[m] = kb[g]; ++m; }
        for (int t = 0; t < NT; ++t) {
            int at[KB + 3] = {};
            int g = done[t] + 1;
            for (int k = 0; k < KB; ++k) {
                while (drain[g] >= 0) ++g;
                drain[g] = t; drain_pos[g] = k; at[k] = g;
                ++g;
            }
            at[KB] = at[KB - 1] + 1; at[KB + 1] = at[KB - 1] + 2;
            // pieces of block 0 (accumulators 0..7) are complete after slice KB/2 - 1, of block 1 after the last
            int when[4] = {at[KB], at[KB], at[KB], at[KB]};
            if (KB >= 4) { when[0] = at[KB / 2]; when[1] = at[KB / 2 + 1]; when[2] = at[KB]; when[3] = at[KB + 1]; }
            for (int k = 0; k < 4; ++k) {
                const int w = when[k];
                hm_tile[w][hm_n[w]] = t; hm_k[w][hm_n[w]] = k; ++hm_n[w];
                if (w > last) last = w;
            }
        }
    }
};

// One layer's GEMM with the dequantize + bias + sine epilogue, the split into binary16 pieces and
// the H_32 products, software-pipelined by hand according to hm_sched.  On return xt[T][v]
// holds, for this lane's coordinate, row 8 (v / 4) + 4 h + v % 4 of H_32 * (activations of tile T).
// ACTK: the activation (sine, or the wavelet with envelope constant c2).
template <int NT, int KB, int NCD, int ACTK = DHQ_ACT_KIND_SINE>
__device__ __forceinline__ void fused_gemm_sine_hm(const dhq_v4i *__restrict__ wA, const float4 *__restrict__ wB,
                                                   const dhq_v4i (&cd)[NCD], float c1, dhq_v16f (&xt)[NT],
                                                   const dhq_v4i (&hA)[2], int lane, int h, float c2 = 0.f)
{
    constexpr hm_sched<NT, KB> S{};
    // the multiplier in a vector register: a multiply-add whose operands are all vector registers issues in about
    // 3 clocks per wave, one with a scalar operand in about 4.5 (measured with a register-only loop)
    asm volatile("" : "+v"(c1));
    constexpr int LAST = S.last;
    constexpr int NM = NT * KB;
    constexpr int EPS = 16 / KB;  // accumulators drained per step (KB <= 8: an even number)
    constexpr int PF = (NM >= 4) ? 4 : (NM >= 2 ? 2 : 1);  // LDS prefetch distance in MFMAs
    dhq_v4i fr[PF + 1];
    float4 bq[3][4];
    dhq_v16i acc[3];
    unsigned hp[2][8], lp[2][8];  // packed pieces of the tile being drained (and of the one before)
#pragma unroll
    for (int m = 0; m < PF; ++m)
        if (m < NM) fr[m % (PF + 1)] = wA[(S.seq_tile[m] * KB + S.seq_kb[m]) * 64 + lane];
    constexpr int GB = 8;
#pragma unroll
    for (int g0 = 0; g0 <= LAST; g0 += GB) {
#pragma unroll
      for (int g1 = 0; g1 < GB; ++g1) {
        const int g = g0 + g1;
        if (g > LAST) continue;
        const int T = S.tile[g];
        if (T >= 0) {
            const int m = S.seq[g], kb = S.kb[g];
            if (m + PF < NM) {
                fr[(m + PF) % (PF + 1)] = wA[(S.seq_tile[m + PF] * KB + S.seq_kb[m + PF]) * 64 + lane];
                __builtin_amdgcn_sched_barrier(0);  // keep the prefetch at the top of the step
            }
#pragma unroll
            for (int gg = 0; gg < 4; ++gg)
                if ((gg * KB) / 4 == kb) bq[T % 3][gg] = wB[(T * 4 + gg) * 2 + h];
            if (kb == 0) {
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[T % 3][v] = 0;
            }
            acc[T % 3] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fr[m % (PF + 1)], cd[kb], acc[T % 3], 0, 0, 0);
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if (q < S.hm_n[g]) {
                const int Th = S.hm_tile[g][q], k = S.hm_k[g][q];
                const int blk = k >> 1;
                dhq_v4i b;  // small pieces first
#pragma unroll
                for (int d = 0; d < 4; ++d) b[d] = (int)((k & 1) ? hp[Th & 1][4 * blk + d] : lp[Th & 1][4 * blk + d]);
                dhq_v16f d;
                if (k == 0) {
#pragma unroll
                    for (int v = 0; v < 16; ++v) d[v] = 0.f;
                } else {
                    d = xt[Th];
                }
                xt[Th] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(dhq_v8h, hA[blk]),
                                                                __builtin_bit_cast(dhq_v8h, b), d, 0, 0, 0);
            }
        }
        const int Td = S.drain[g];
        if (Td >= 0) {
#pragma unroll
            for (int j = 0; j < EPS; j += 2) {
                const int v = S.drain_pos[g] * EPS + j;
                const float4 bb = bq[Td % 3][v >> 2];
                const float bias0 = (v & 2) ? bb.z : bb.x, bias1 = (v & 2) ? bb.w : bb.y;
                // accumulators v, v + 1 (v even) are neighbouring features 2m, 2m + 1: the pair the complex wavelet takes
                const float t0 = __builtin_fmaf((float)acc[Td % 3][v], c1, bias0), t1 = __builtin_fmaf((float)acc[Td % 3][v + 1], c1, bias1);
                float a0, a1;
                if constexpr (ACTK == DHQ_ACT_KIND_WAVELET_COMPLEX) {
                    dhq_activate_pair_rev<false>(t0, t1, c2, a0, a1);
                } else {
                    a0 = dhq_activate_rev(t0, dhq_act{ACTK, c2});
                    a1 = dhq_activate_rev(t1, dhq_act{ACTK, c2});
                }
                hm_split_pair(a0, a1, hp[Td & 1][v >> 1], lp[Td & 1][v >> 1]);
            }
        }
        if (T >= 0 || Td >= 0 || S.hm_n[g] > 0) __builtin_amdgcn_sched_barrier(0);
      }
    }
}

// The stages of the transform over the tile index: plain register add/sub.
template <int NT>
__device__ __forceinline__ void fused_tile_stages(dhq_v16f (&xt)[NT])
{
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

// The quantizer: register s = 16 T + v becomes byte s % 4 of dword s / 4 of the codes.
template <int NT>
__device__ __forceinline__ void fused_quantize(const dhq_v16f (&xt)[NT], dhq_v4i (&cd)[NT], float inv, int qlo, int qhi)
{
    asm volatile("" : "+v"(inv));  // a vector-register multiplier, as in fused_gemm_sine_hm
#pragma unroll
    for (int w = 0; w < NT * 4; ++w) {
        const int v = 4 * (w & 3);
        cd[w / 4][w % 4] = (int)fused_quant4(xt[w >> 2][v], xt[w >> 2][v + 1], xt[w >> 2][v + 2], xt[w >> 2][v + 3], inv, qlo, qhi);
    }
}

// The output layer: one zero-padded M tile, no sine.
template <int NKB>
__device__ __forceinline__ void fused_output_layer(const dhq_v4i *__restrict__ wA, const float *__restrict__ wB,
                                                   const dhq_v4i (&cd)[NKB], float c1, float *__restrict__ out, int64_t ci,
                                                   bool valid, int m_out, int lane, int h)
{
    dhq_v16i acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0;
#pragma unroll
    for (int kb = 0; kb < NKB; ++kb) {
        const dhq_v4i a = wA[kb * 64 + lane];
        acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, cd[kb], acc, 0, 0, 0);
    }
    if (valid) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = 8 * (v >> 2) + 4 * h + (v & 3);
            if (row < m_out) out[ci * m_out + row] = __builtin_fmaf((float)acc[v], c1, wB[((v >> 2) * 2 + h) * 4 + (v & 3)]);
        }
    }
}

template <int NF, int ACTK>
__global__ __launch_bounds__(FUSED_THREADS) void dhq_fused_kernel(const fused_args A)
{
    constexpr int NT = NF / 32;   // M tiles of a hidden layer
    constexpr int NKB = NF / 32;  // k blocks of a hidden layer
    constexpr int BLK = (NT * NKB + 1) * 1024;  // LDS bytes per weight buffer

    extern __shared__ __align__(16) unsigned char lds[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = lane & 31, h = lane >> 5;
    const int L = A.n_layers;
    const int64_t n_tiles = (A.n + FUSED_TILE - 1) / FUSED_TILE;
    const int qlo = DHQ_MAGIC_I - A.qmax, qhi = DHQ_MAGIC_I + A.qmax;

    dhq_v4i hA[2];
    fused_h32_operand(c, h, hA);

    int p = 0;  // LDS buffer holding the layer about to run
    if ((int64_t)blockIdx.x < n_tiles)
        fused_issue_copy(A.blob + A.layer[0].blob_off, lds, (int)A.layer[0].chunks, wave, lane, FUSED_WAVES);

    for (int64_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const int64_t ci = tile * FUSED_TILE + wave * 32 + c;
        const bool valid = ci < A.n;
        const int64_t cl = valid ? ci : A.n - 1;

        dhq_v4i cd[NKB];  // activation codes: the B operands of the next GEMM
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb) cd[kb] = dhq_v4i{0, 0, 0, 0};
        cd[0][0] = fused_input_codes(A.coords, cl, A.k0, A.k0p, A.layer[0].inv_in, A.qmax);

        dhq_v16f xt[NT];
        for (int l = 0; l < L - 1; ++l) {
            // weights of layer l have landed; everyone is done with the other buffer
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();
            {
                const fused_layer_desc &nx = A.layer[l + 1];
                fused_issue_copy(A.blob + nx.blob_off, lds + (p ^ 1) * BLK, (int)nx.chunks, wave, lane, FUSED_WAVES);
            }
            const dhq_v4i *wA = reinterpret_cast<const dhq_v4i *>(lds + p * BLK);
            const float c1 = A.layer[l].c1;
            if (l == 0)
                fused_gemm_sine_hm<NT, 1, NKB, ACTK>(wA, reinterpret_cast<const float4 *>(lds + p * BLK + NT * 1024), cd, c1, xt,
                                                     hA, lane, h, A.c2);
            else
                fused_gemm_sine_hm<NT, NKB, NKB, ACTK>(wA, reinterpret_cast<const float4 *>(lds + p * BLK + NT * NKB * 1024), cd,
                                                       c1, xt, hA, lane, h, A.c2);
            // The two waves of a SIMD overlap well while both feed the matrix unit or both
            // do vector work, but a wave in its vector phase starves the MFMA chain of the
            // other; keep the phases aligned across the workgroup.
            __syncthreads();
            fused_tile_stages<NT>(xt);
            fused_quantize<NT>(xt, cd, A.layer[l + 1].inv_in, qlo, qhi);
            p ^= 1;
        }

        // output layer: one zero-padded M tile, no sine
        {
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();
            if (tile + gridDim.x < n_tiles)
                fused_issue_copy(A.blob + A.layer[0].blob_off, lds + (p ^ 1) * BLK, (int)A.layer[0].chunks, wave, lane, FUSED_WAVES);
            fused_output_layer<NKB>(reinterpret_cast<const dhq_v4i *>(lds + p * BLK),
                                    reinterpret_cast<const float *>(lds + p * BLK + NKB * 1024), cd, A.layer[L - 1].c1, A.out, ci,
                                    valid, A.m_out, lane, h);
            p ^= 1;
        }
    }
}

// ---- one layer per launch: the dynamic quantization module (Sec. 3.3) ------------------------
// With scales measured on line, a layer's quantizer needs max |x^| over the whole batch before
// it can emit a single code, so the network cannot stay in registers from end to end.  These
// kernels cut the fused kernel at exactly that point: a launch folds the maxima the previous
// launch's workgroups left into this layer's constants (every workgroup for itself: a few hundred
// floats and three fp64 operations cost less than a launch in between), quantizes its input
// with them, runs the layer (GEMM, epilogue, transform of the output) and writes the
// transformed output x^ (fp32) plus each workgroup's max |x^|.  Per hidden
// layer the activations cross device memory once in each direction, in the lanes' register order
// ([wave tile][float4 q][lane]: every 16-byte access of a wave is 1 KiB contiguous).
//   MODE 0  input layer: coordinates in, x^ out        MODE 1  hidden layer: x^ in, x^ out
//   MODE 2  output layer: x^ in, signal values out
struct fusedl_args {
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
    int k0, k0p, m_out, qmax;
    float c2;                  // wavelet activation: 2 pi s0 sqrt(log2 e) / omega0
};

// ACTK: the activation after the layer (MODE 0, 1).
template <int NF, int MODE, int ACTK>
__global__ __launch_bounds__(FUSED_THREADS) void dhq_fused_layer_kernel(const fusedl_args A)
{
    constexpr int NT = NF / 32, NKB = NF / 32, NR = NF / 2;
    constexpr int KB = (MODE == 0) ? 1 : NKB;      // k blocks of this layer's GEMM
    constexpr int MT = (MODE == 2) ? 1 : NT;       // M tiles of this layer's GEMM
    extern __shared__ __align__(16) unsigned char lds[];
    __shared__ float red_in[FUSED_WAVES], red[FUSED_WAVES];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = lane & 31, h = lane >> 5;
    const int64_t n_tiles = (A.n + FUSED_TILE - 1) / FUSED_TILE;
    const int qlo = DHQ_MAGIC_I - A.qmax, qhi = DHQ_MAGIC_I + A.qmax;
    dhq_v4i hA[2];
    fused_h32_operand(c, h, hA);
    fused_issue_copy(A.blk, lds, A.chunks, wave, lane, FUSED_WAVES);
    // this layer's constants from the maxima of its input
    float inv, c1, s_a;
    {
        float mi = 0.f;
        for (int i = threadIdx.x; i < A.partial_count; i += FUSED_THREADS) mi = fmaxf(mi, A.partial_in[i]);
#pragma unroll
        for (int m = 1; m < 64; m *= 2) mi = fmaxf(mi, __shfl_xor(mi, m, 64));
        if (lane == 0) red_in[wave] = mi;
        __syncthreads();
        mi = red_in[0];
#pragma unroll
        for (int w = 1; w < FUSED_WAVES; ++w) mi = fmaxf(mi, red_in[w]);
        dhq_dyn_constants(mi, A.kp, A.qmax, A.c1_over_sa, inv, c1, s_a);
        if (blockIdx.x == 0 && threadIdx.x == 0) {
            A.dyn[0] = inv; A.dyn[1] = c1; A.dyn[2] = s_a;
        }
    }
    const dhq_v4i *wA = reinterpret_cast<const dhq_v4i *>(lds);
    float mx = 0.f;
    bool landed = false;
    for (int64_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const int64_t ci = tile * FUSED_TILE + wave * 32 + c;
        const bool valid = ci < A.n;
        const int64_t cl = valid ? ci : A.n - 1;  // lanes past the end repeat the last coordinate: no effect on the maximum
        const size_t slot = ((size_t)tile * FUSED_WAVES + wave) * (NR / 4) * 64 + lane;
        dhq_v4i cd[NKB];
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb) cd[kb] = dhq_v4i{0, 0, 0, 0};
        if constexpr (MODE == 0) {
            cd[0][0] = fused_input_codes(A.coords, cl, A.k0, A.k0p, inv, A.qmax);
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
            fused_output_layer<NKB>(wA, reinterpret_cast<const float *>(lds + MT * KB * 1024), cd, c1, A.out, ci, valid, A.m_out,
                                    lane, h);
        } else {
            dhq_v16f xt[NT];
            fused_gemm_sine_hm<NT, KB, NKB, ACTK>(wA, reinterpret_cast<const float4 *>(lds + MT * KB * 1024), cd, c1, xt, hA, lane, h,
                                                  A.c2);
            fused_tile_stages<NT>(xt);
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
            for (int w = 1; w < FUSED_WAVES; ++w) r = fmaxf(r, red[w]);
            A.partial[blockIdx.x] = r;
        }
    }
}

// ---- test hook: one layer of the whole-network kernel on caller-supplied codes ---------------
// The layer body is the code dhq_fused_kernel runs (fused_gemm_sine_hm, fused_tile_stages,
// fused_quant4 on the same packed weights); only the way in and out differs: the input codes
// are gathered from a row-major n x Kp array into the lanes' register order, and the
// un-normalised transform x^ of the layer's output and the codes the next layer's quantizer
// makes of it are scattered back to row-major n x NF arrays in rotated-feature order.  The
// integer accumulators come from a second, plain MFMA loop over the same fragments and codes.
struct fusedd_args {
    const int8_t *codes_in;    // n x kp_in, rotated-feature order
    const unsigned char *blk;  // the layer's block of the packed weights
    float *xhat;               // n x NF or null
    int8_t *codes_out;         // n x NF or null
    int32_t *acc;              // n x NF or null
    int64_t n;
    int chunks, kp_in, qmax;
    float c1, inv_next, c2;
};

template <int NF, bool FIRST, int ACTK>
__global__ __launch_bounds__(FUSED_THREADS) void dhq_fused_debug_kernel(const fusedd_args A)
{
    constexpr int NT = NF / 32, NKB = NF / 32, NR = NF / 2;
    constexpr int KB = FIRST ? 1 : NKB;
    extern __shared__ __align__(16) unsigned char lds[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = lane & 31, h = lane >> 5;
    const int qlo = DHQ_MAGIC_I - A.qmax, qhi = DHQ_MAGIC_I + A.qmax;
    dhq_v4i hA[2];
    fused_h32_operand(c, h, hA);
    fused_issue_copy(A.blk, lds, A.chunks, wave, lane, FUSED_WAVES);
    const int64_t ci = (int64_t)blockIdx.x * FUSED_TILE + wave * 32 + c;
    const bool valid = ci < A.n;
    const int64_t cl = valid ? ci : A.n - 1;
    dhq_v4i cd[NKB];
#pragma unroll
    for (int kb = 0; kb < NKB; ++kb) cd[kb] = dhq_v4i{0, 0, 0, 0};
    if constexpr (FIRST) {
        // the input layer's (<= 4) codes sit in bytes 0.. of dword 0, whichever lane half
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
    fused_gemm_sine_hm<NT, KB, NKB, ACTK>(wA, reinterpret_cast<const float4 *>(lds + NT * KB * 1024), cd, A.c1, xt, hA, lane, h, A.c2);
    __syncthreads();
    fused_tile_stages<NT>(xt);
    fused_quantize<NT>(xt, cd, A.inv_next, qlo, qhi);
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
static bool fused_shape_ok(const dhq_model *m, int *nf_out)
{
    const int L = m->n_layers;
    if (L < 2) return false;
    if (m->dims[0] > 4 || m->dims[L] > 32) return false;
    const int nf = m->dims[1];
    if (nf != 32 && nf != 64 && nf != 128 && nf != 256) return false;
    for (int l = 1; l < L; ++l)
        if (m->dims[l] != nf) return false;
    *nf_out = nf;
    return true;
}

int dhq_fused_create(const dhq_model *m, dhq_fused_plan **plan_out)
{
    *plan_out = nullptr;
    int nf = 0;
    if (!fused_shape_ok(m, &nf)) return DHQ_OK;
    const int L = m->n_layers;
    const int NT = nf / 32, NKB = nf / 32;

    dhq_fused_plan *P = new (std::nothrow) dhq_fused_plan();
    if (!P) return DHQ_ENOMEM;
    P->nf = nf;
    memset(&P->args, 0, sizeof(P->args));

    // block sizes: fragments [Mt][Kb] KiB + one KiB of biases
    std::vector<unsigned char> blob;
    for (int l = 0; l < L; ++l) {
        const dhq_layer &Ly = m->layer[l];
        const int Mt = (l == L - 1) ? 1 : NT;
        const int Kb = (l == 0) ? 1 : NKB;
        const size_t off = blob.size();
        const size_t bytes = (size_t)(Mt * Kb + 1) * 1024;
        blob.resize(off + bytes, 0);
        int8_t *frag = reinterpret_cast<int8_t *>(blob.data() + off);
        const int8_t *wq = Ly.wq_host.data();  // M x Kp, rotated-index order
        for (int T = 0; T < Mt; ++T)
            for (int kb = 0; kb < Kb; ++kb)
                for (int ln = 0; ln < 64; ++ln) {
                    const int row = 32 * T + (ln & 31), u = ln >> 5;
                    for (int jj = 0; jj < 16; ++jj) {
                        int8_t val = 0;
                        if (row < Ly.M) {
                            if (l == 0) {
                                // un-permuted: the input layer's codes sit in bytes 0..Kp-1 of half 0
                                if (u == 0 && jj < Ly.Kp) val = wq[(size_t)row * Ly.Kp + jj];
                            } else {
                                const int k = hm_index(16 * kb + jj, u);
                                val = wq[(size_t)row * Ly.Kp + k];
                            }
                        }
                        frag[((size_t)(T * Kb + kb) * 64 + ln) * 16 + jj] = val;
                    }
                }
        // the bias block: [T][g][h][e], in revolutions for the sine layers
        {
            float *bias = reinterpret_cast<float *>(blob.data() + off + (size_t)Mt * Kb * 1024);
            const std::vector<float> &src = (l == L - 1) ? Ly.bias_host : Ly.bias_rev_host;
            for (int f = 0; f < Ly.M; ++f) bias[bias_slot(f)] = src[f];
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
    P->args.qmax = m->qmax_a;
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

void dhq_fused_destroy(dhq_fused_plan *plan)
{
    if (!plan) return;
    if (plan->blob_dev) (void)hipFree(plan->blob_dev);
    delete plan;
}

// Refreshes the per-layer constants after the activation scales changed.
int dhq_fused_update_scales(const dhq_model *m, dhq_fused_plan *P)
{
    if (!P) return DHQ_OK;
    for (int l = 0; l < m->n_layers; ++l) {
        const dhq_layer &Ly = m->layer[l];
        P->args.layer[l].c1 = dhq_c1(m, l);
        P->args.layer[l].inv_in = (float)(1.0 / ((double)Ly.s_a * sqrt((double)Ly.Kp)));
    }
    return DHQ_OK;
}

template <int NF, int ACTK>
static hipError_t fused_launch_act(const dhq_fused_plan *P, const fused_args &a, unsigned grid, hipStream_t st)
{
    auto kern = dhq_fused_kernel<NF, ACTK>;
    hipError_t e = dhq_lds_limit_once(kern, P->lds_bytes, P->device);
    if (e != hipSuccess) return e;
    kern<<<grid, FUSED_THREADS, P->lds_bytes, st>>>(a);
    return hipGetLastError();
}
template <int NF>
static hipError_t fused_launch_t(const dhq_fused_plan *P, const fused_args &a, int act_kind, unsigned grid, hipStream_t st)
{
    if (act_kind == DHQ_ACT_KIND_WAVELET_COMPLEX) return fused_launch_act<NF, DHQ_ACT_KIND_WAVELET_COMPLEX>(P, a, grid, st);
    return act_kind == DHQ_ACT_KIND_WAVELET ? fused_launch_act<NF, DHQ_ACT_KIND_WAVELET>(P, a, grid, st)
                                            : fused_launch_act<NF, DHQ_ACT_KIND_SINE>(P, a, grid, st);
}

hipError_t dhq_fused_launch(const dhq_model *m, const float *coords, int64_t n, float *out, hipStream_t st)
{
    const dhq_fused_plan *P = m->fused;
    if (!P) return hipErrorInvalidValue;
    if (n <= 0) return hipSuccess;
    fused_args a = P->args;
    a.coords = coords;
    a.out = out;
    a.n = n;
    a.c2 = dhq_hidden_act(m).c2;
    const int64_t tiles = (n + FUSED_TILE - 1) / FUSED_TILE;
    const unsigned grid = (unsigned)(tiles < P->n_cu ? tiles : P->n_cu);
    switch (P->nf) {
        case 32: return fused_launch_t<32>(P, a, m->act_kind, grid, st);
        case 64: return fused_launch_t<64>(P, a, m->act_kind, grid, st);
        case 128: return fused_launch_t<128>(P, a, m->act_kind, grid, st);
        case 256: return fused_launch_t<256>(P, a, m->act_kind, grid, st);
        default: return hipErrorInvalidValue;
    }
}

// The dynamic mode on the per-layer kernels above.  ws0 / ws1: two buffers of rows(n) x width
// floats (rows(n) = n rounded up to a whole workgroup tile); partial: room for 2 x
// DHQ_ABSMAX_PARTIALS floats (two sets of per-workgroup maxima, used alternately: a layer's
// slower workgroups still read one set while its faster ones already write the other);
// dyn: three floats per layer.
size_t dhq_fused_dynamic_rows(int64_t n) { return (size_t)((n + FUSED_TILE - 1) / FUSED_TILE) * FUSED_TILE; }

template <int NF, int MODE, int ACTK>
static hipError_t fusedl_launch_t(const fusedl_args &a, unsigned grid, int device, hipStream_t st)
{
    auto kern = dhq_fused_layer_kernel<NF, MODE, ACTK>;
    const size_t lds = (size_t)a.chunks * 1024;
    hipError_t e = dhq_lds_limit_once(kern, lds, device);
    if (e != hipSuccess) return e;
    kern<<<grid, FUSED_THREADS, lds, st>>>(a);
    return hipGetLastError();
}
template <int NF>
static hipError_t fusedl_launch_mode(int mode, int act_kind, const fusedl_args &a, unsigned grid, int device, hipStream_t st)
{
    const bool wav = (act_kind == DHQ_ACT_KIND_WAVELET);
    if (act_kind == DHQ_ACT_KIND_WAVELET_COMPLEX && mode < 2)
        return mode == 0 ? fusedl_launch_t<NF, 0, DHQ_ACT_KIND_WAVELET_COMPLEX>(a, grid, device, st)
                         : fusedl_launch_t<NF, 1, DHQ_ACT_KIND_WAVELET_COMPLEX>(a, grid, device, st);
    switch (mode) {
        case 0: return wav ? fusedl_launch_t<NF, 0, DHQ_ACT_KIND_WAVELET>(a, grid, device, st) : fusedl_launch_t<NF, 0, DHQ_ACT_KIND_SINE>(a, grid, device, st);
        case 1: return wav ? fusedl_launch_t<NF, 1, DHQ_ACT_KIND_WAVELET>(a, grid, device, st) : fusedl_launch_t<NF, 1, DHQ_ACT_KIND_SINE>(a, grid, device, st);
        default: return fusedl_launch_t<NF, 2, DHQ_ACT_KIND_NONE>(a, grid, device, st);  // the output layer has no activation
    }
}

hipError_t dhq_fused_dynamic_launch(const dhq_model *m, const float *coords, int64_t n, float *out, float *ws0, float *ws1,
                                    float *partial, float *dyn, hipStream_t st)
{
    const dhq_fused_plan *P = m->fused;
    if (!P) return hipErrorInvalidValue;
    if (n <= 0) return hipSuccess;
    const int L = m->n_layers;
    const int64_t tiles = (n + FUSED_TILE - 1) / FUSED_TILE;
    const unsigned grid = (unsigned)(tiles < P->n_cu ? tiles : P->n_cu);
    // the input layer's scale: max over the rotated coordinates, left as per-workgroup maxima
    float *pbuf[2] = {partial, partial + DHQ_ABSMAX_PARTIALS};
    int count = 0;
    hipError_t e = dhq_launch_wht_absmax_partials(coords, n, m->layer[0].K, m->layer[0].Kp, pbuf[0], &count, st);
    if (e != hipSuccess) return e;
    float *bufs[2] = {ws0, ws1};
    for (int l = 0; l < L; ++l) {
        fusedl_args a;
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
        a.k0 = P->args.k0; a.k0p = P->args.k0p; a.m_out = P->args.m_out; a.qmax = P->args.qmax;
        a.c2 = dhq_hidden_act(m).c2;
        const int mode = (l == 0) ? 0 : (l == L - 1 ? 2 : 1);
        switch (P->nf) {
            case 32: e = fusedl_launch_mode<32>(mode, m->act_kind, a, grid, P->device, st); break;
            case 64: e = fusedl_launch_mode<64>(mode, m->act_kind, a, grid, P->device, st); break;
            case 128: e = fusedl_launch_mode<128>(mode, m->act_kind, a, grid, P->device, st); break;
            case 256: e = fusedl_launch_mode<256>(mode, m->act_kind, a, grid, P->device, st); break;
            default: e = hipErrorInvalidValue;
        }
        if (e != hipSuccess) return e;
        count = (int)grid;
    }
    return hipSuccess;
}

// Test hook behind dhq_forward_debug_fused: layer `layer` (one that ends in an activation) of the
// whole-network kernel on the caller's codes.
template <int NF, bool FIRST, int ACTK>
static hipError_t fusedd_launch_t(const fusedd_args &a, unsigned grid, int device, hipStream_t st)
{
    auto kern = dhq_fused_debug_kernel<NF, FIRST, ACTK>;
    const size_t lds = (size_t)a.chunks * 1024;
    hipError_t e = dhq_lds_limit_once(kern, lds, device);
    if (e != hipSuccess) return e;
    kern<<<grid, FUSED_THREADS, lds, st>>>(a);
    return hipGetLastError();
}
template <int NF>
static hipError_t fusedd_launch_nf(bool first, int act_kind, const fusedd_args &a, unsigned grid, int device, hipStream_t st)
{
    const bool wav = (act_kind == DHQ_ACT_KIND_WAVELET);
    if (act_kind == DHQ_ACT_KIND_WAVELET_COMPLEX)
        return first ? fusedd_launch_t<NF, true, DHQ_ACT_KIND_WAVELET_COMPLEX>(a, grid, device, st)
                     : fusedd_launch_t<NF, false, DHQ_ACT_KIND_WAVELET_COMPLEX>(a, grid, device, st);
    if (first) return wav ? fusedd_launch_t<NF, true, DHQ_ACT_KIND_WAVELET>(a, grid, device, st) : fusedd_launch_t<NF, true, DHQ_ACT_KIND_SINE>(a, grid, device, st);
    return wav ? fusedd_launch_t<NF, false, DHQ_ACT_KIND_WAVELET>(a, grid, device, st) : fusedd_launch_t<NF, false, DHQ_ACT_KIND_SINE>(a, grid, device, st);
}

hipError_t dhq_fused_debug_launch(const dhq_model *m, int layer, const int8_t *codes_in, int64_t n, float *xhat, int8_t *codes_out,
                                  int32_t *acc, hipStream_t st)
{
    const dhq_fused_plan *P = m->fused;
    if (!P || layer < 0 || layer >= m->n_layers - 1) return hipErrorInvalidValue;
    if (n <= 0) return hipSuccess;
    fusedd_args a;
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
    a.c2 = dhq_hidden_act(m).c2;
    const unsigned grid = (unsigned)((n + FUSED_TILE - 1) / FUSED_TILE);
    switch (P->nf) {
        case 32: return fusedd_launch_nf<32>(layer == 0, m->act_kind, a, grid, P->device, st);
        case 64: return fusedd_launch_nf<64>(layer == 0, m->act_kind, a, grid, P->device, st);
        case 128: return fusedd_launch_nf<128>(layer == 0, m->act_kind, a, grid, P->device, st);
        case 256: return fusedd_launch_nf<256>(layer == 0, m->act_kind, a, grid, P->device, st);
        default: return hipErrorInvalidValue;
    }
}
