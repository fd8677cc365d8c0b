// Layer-by-layer kernels of the DHQ forward path (paper Sec. 3.2-3.3), gfx950.
//
//   wht_quant   rotation of every activation row by the Walsh-Hadamard transform (Eq. 3,
//               vector case) fused with the symmetric quantizer, or with the absmax reduction
//               that calibration needs
//   gemm_i8     int8 x int8 -> int32 on MFMA (the MAC array of Sec. 3.3), optionally with the
//               dequantize + bias + sine epilogue fused in
//   gemm_narrow the same contraction for fan-in < 32, on integer ALU ops
//   epilogue    dequantize + bias + sine from stored accumulators
//   unrotate    two-sided variant (Eq. 4-5 with both factors): multiplies the rotated
//               accumulators by H over the output features, exactly in int32, then the epilogue
//   unrotate_quant  the same, going on to the next layer's rotation and quantizer in the same lanes
//               (static scales: rotated accumulators in, the next layer's codes out)
//   dyn_scale   on-line per-tensor scale (the dynamic quantization module of Sec. 3.3): the per-workgroup
//               maxima of a layer input become the constants the kernels read -- folded by the quantizing
//               kernel itself in a forward pass, by a one-workgroup kernel during calibration
//
// Activations travel through device memory between these kernels; the fused whole-network
// kernel lives in dhq_fused.hip.
#include "dhq_device.h"
#include "dhq_internal.h"

// ------------------------------------------------------------------ rotation + quantizer
// Row-parallel transform.  A row of KP values is spread over LPR lanes holding EPL values
// each; butterflies over the index bits held inside a lane are plain add/sub, the others
// exchange between lanes.  The transform runs un-normalised (entries of H are +-1);
// 1/sqrt(KP) is folded into `inv`.
//   KP >= 64: 16 lanes per row (one DPP row), lane t holds values 64 j + 4 t + e (e = 0..3,
//             j = 0..KP/64-1): every 16-byte load of a row's 16 lanes covers 256 contiguous
//             bytes, and the four stages over t run as data-parallel-primitive moves (quad
//             permutes for t ^ 1 and t ^ 2, two bank-masked row shifts for t ^ 4, a row
//             rotation for t ^ 8) instead of going through the LDS crossbar;
//   KP <  64: EPL = min(4, KP) consecutive values per lane, wavefront shuffles between lanes.
template <int KP>
struct wht_shape {
    static constexpr bool ROW16 = KP >= 64;
    static constexpr int EPL = ROW16 ? KP / 16 : (KP >= 4 ? 4 : KP);
    static constexpr int LPR = KP / EPL;
    // index within the row of value i of lane t; values 4 g .. 4 g + 3 of a lane are consecutive
    static __device__ __forceinline__ constexpr int index(int t, int i)
    {
        return ROW16 ? 64 * (i / 4) + 4 * t + (i % 4) : t * EPL + i;
    }
};

// Value of lane (t ^ M) of the same 16-lane row, M = 1, 2, 4, 8.
template <int M>
__device__ __forceinline__ int wht_row16_xor(int x)
{
    static_assert(M == 1 || M == 2 || M == 4 || M == 8, "");
    if constexpr (M == 1) return __builtin_amdgcn_mov_dpp(x, 0xB1, 0xF, 0xF, true);   // quad_perm:[1,0,3,2]
    if constexpr (M == 2) return __builtin_amdgcn_mov_dpp(x, 0x4E, 0xF, 0xF, true);   // quad_perm:[2,3,0,1]
    if constexpr (M == 8) return __builtin_amdgcn_mov_dpp(x, 0x128, 0xF, 0xF, true);  // row_ror:8
    // lanes 0-3 and 8-11 of a row read four lanes up (row_shl:4), lanes 4-7 and 12-15 four lanes down (row_shr:4)
    const int up = __builtin_amdgcn_update_dpp(x, x, 0x104, 0xF, 0x5, false);
    return __builtin_amdgcn_update_dpp(up, x, 0x114, 0xF, 0xA, false);
}

// One butterfly stage over lane bit M: the lane with the bit clear keeps v + p, the other p - v
// (p = the partner lane's value).  Float: p + (v with its sign flipped in the upper lane), which
// lets the partner's value come in through the add's own data-parallel-primitive operand.
__device__ __forceinline__ int wht_add(int a, int b) { return (int)((unsigned)a + (unsigned)b); }
__device__ __forceinline__ int wht_sub(int a, int b) { return (int)((unsigned)a - (unsigned)b); }
__device__ __forceinline__ float wht_add(float a, float b) { return a + b; }
__device__ __forceinline__ float wht_sub(float a, float b) { return a - b; }

template <int KP, int M>
__device__ __forceinline__ void wht_lane_stage(float (&v)[wht_shape<KP>::EPL], int t)
{
    constexpr int EPL = wht_shape<KP>::EPL;
    if constexpr (wht_shape<KP>::ROW16) {
        const int flip = (t & M) ? (int)0x80000000 : 0;
#pragma unroll
        for (int e = 0; e < EPL; ++e) {
            const float p = __int_as_float(wht_row16_xor<M>(__float_as_int(v[e])));
            v[e] = p + __int_as_float(__float_as_int(v[e]) ^ flip);
        }
    } else {
        const bool upper = (t & M) != 0;
#pragma unroll
        for (int e = 0; e < EPL; ++e) {
            const float p = __shfl_xor(v[e], M, 64);
            v[e] = upper ? p - v[e] : v[e] + p;
        }
    }
}
template <int KP, int M>
__device__ __forceinline__ void wht_lane_stage(int (&v)[wht_shape<KP>::EPL], int t)
{
    constexpr int EPL = wht_shape<KP>::EPL;
    const bool upper = (t & M) != 0;
#pragma unroll
    for (int e = 0; e < EPL; ++e) {
        const int p = wht_shape<KP>::ROW16 ? wht_row16_xor<M>(v[e]) : __shfl_xor(v[e], M, 64);
        v[e] = upper ? wht_sub(p, v[e]) : wht_add(v[e], p);
    }
}

template <int KP, typename T>
__device__ __forceinline__ void wht_butterflies(T (&v)[wht_shape<KP>::EPL], int t)
{
    constexpr int EPL = wht_shape<KP>::EPL;
    constexpr int LPR = wht_shape<KP>::LPR;
#pragma unroll
    for (int h = 1; h < EPL; h *= 2) {
#pragma unroll
        for (int e = 0; e < EPL; ++e) {
            if ((e & h) == 0) {
                const T a = v[e], b = v[e | h];
                v[e] = wht_add(a, b);
                v[e | h] = wht_sub(a, b);
            }
        }
    }
    if constexpr (LPR > 1) wht_lane_stage<KP, 1>(v, t);
    if constexpr (LPR > 2) wht_lane_stage<KP, 2>(v, t);
    if constexpr (LPR > 4) wht_lane_stage<KP, 4>(v, t);
    if constexpr (LPR > 8) wht_lane_stage<KP, 8>(v, t);
    static_assert(LPR <= 16, "a row spans at most 16 lanes");
}

// Loads this lane's EPL values of one row (zero beyond K, zero for a dead row) and transforms the row.
template <int KP>
__device__ __forceinline__ void wht_row(const float *__restrict__ in, int64_t row, int t, bool live, int K,
                                        float (&v)[wht_shape<KP>::EPL])
{
    using S = wht_shape<KP>;
    constexpr int EPL = S::EPL;
    if (live && K == KP && EPL >= 4) {
#pragma unroll
        for (int g = 0; g < EPL / 4; ++g) {
            const float4 x = *reinterpret_cast<const float4 *>(in + row * KP + S::index(t, 4 * g));
            v[(4 * g) % EPL] = x.x; v[(4 * g + 1) % EPL] = x.y; v[(4 * g + 2) % EPL] = x.z; v[(4 * g + 3) % EPL] = x.w;
        }
    } else {
#pragma unroll
        for (int e = 0; e < EPL; ++e) {
            const int idx = S::index(t, e);
            v[e] = (live && idx < K) ? in[row * K + idx] : 0.0f;
        }
    }
    wht_butterflies<KP>(v, t);
}

template <int KP>
__global__ __launch_bounds__(256) void wht_quant_kernel(const float *__restrict__ in, int64_t n,
                                                        int K, float inv, int qmax,
                                                        int8_t *__restrict__ codes,
                                                        const float *__restrict__ fold_partial, int fold_count,
                                                        double c1_over_sa, float *__restrict__ dyn_out)
{
    if (fold_partial) {
        // dynamic mode: the scale is measured on the device.  Every workgroup folds the per-workgroup maxima
        // the absmax pass left (a few KiB from L2: cheaper than a one-workgroup launch in between) and turns
        // the maximum into the layer's constants; workgroup 0 also stores them for the kernels that follow.
        __shared__ float red[5];
        float mx = 0.0f;
        for (int i = threadIdx.x; i < fold_count; i += 256) mx = fmaxf(mx, fold_partial[i]);
#pragma unroll
        for (int m = 1; m < 64; m *= 2) mx = fmaxf(mx, __shfl_xor(mx, m, 64));
        if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = mx;
        __syncthreads();
        if (threadIdx.x == 0) {
            float c1, s_a;
            dhq_dyn_constants(fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3])), KP, qmax, c1_over_sa, inv, c1, s_a);
            red[4] = inv;
            if (blockIdx.x == 0) {
                dyn_out[0] = inv; dyn_out[1] = c1; dyn_out[2] = s_a;
            }
        }
        __syncthreads();
        inv = red[4];
    }
    constexpr int EPL = wht_shape<KP>::EPL;
    constexpr int LPR = wht_shape<KP>::LPR;
    const int64_t gtid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t row = gtid / LPR;
    const int t = (int)(gtid % LPR);
    const bool live = row < n;
    float v[EPL];
    wht_row<KP>(in, row, t, live, K, v);
    if (!live) return;
    if constexpr (EPL >= 4) {
#pragma unroll
        for (int e = 0; e < EPL; e += 4) {
            const unsigned w = dhq_pack4(dhq_quant_bits(v[e], inv, qmax), dhq_quant_bits(v[e + 1], inv, qmax),
                                         dhq_quant_bits(v[e + 2], inv, qmax), dhq_quant_bits(v[e + 3], inv, qmax));
            *reinterpret_cast<unsigned *>(codes + row * KP + wht_shape<KP>::index(t, e)) = w;
        }
    } else {
#pragma unroll
        for (int e = 0; e < EPL; ++e)
            codes[row * KP + wht_shape<KP>::index(t, e)] = (int8_t)(dhq_quant_bits(v[e], inv, qmax) & 0xff);
    }
}

// The constants of the dynamic mode (dhq_dyn_constants) for the absmax word of a layer input, stored
// as dyn[0..2] = {inv, c1, s_a}.
__device__ __forceinline__ void dyn_scale_write(unsigned absmax_bits, int Kp, int qmax, double c1_over_sa,
                                                float *__restrict__ dyn)
{
    dhq_dyn_constants(__uint_as_float(absmax_bits), Kp, qmax, c1_over_sa, dyn[0], dyn[1], dyn[2]);
}

// max |un-normalised x^| over all rows.  The grid is a few workgroups per CU, every workgroup
// strides over the rows keeping its maximum in registers and stores it to partial[blockIdx.x];
// a second, one-workgroup kernel folds the partial maxima into *absmax_bits (float bits:
// non-negative floats order like unsigned integers) and, in dynamic mode, into the layer's
// constants.  No atomics: one atomicMax per wave on a single word made this pass three times
// slower than the quantizing pass, one per workgroup still 1.7 times.
#define DHQ_ABSMAX_BLOCKS DHQ_ABSMAX_PARTIALS
template <int KP>
__global__ __launch_bounds__(256) void wht_absmax_kernel(const float *__restrict__ in, int64_t n, int K,
                                                         float *__restrict__ partial)
{
    constexpr int EPL = wht_shape<KP>::EPL;
    constexpr int LPR = wht_shape<KP>::LPR;
    constexpr int RPB = 256 / LPR;  // rows a workgroup transforms per pass
    __shared__ float red[4];
    const int t = threadIdx.x % LPR;
    float mx = 0.0f;
    // the loop bound is the same for the whole workgroup: every lane takes part in the shuffles
    for (int64_t base = (int64_t)blockIdx.x * RPB; base < n; base += (int64_t)gridDim.x * RPB) {
        const int64_t row = base + threadIdx.x / LPR;
        float v[EPL];
        wht_row<KP>(in, row, t, row < n, K, v);
#pragma unroll
        for (int e = 0; e < EPL; ++e) mx = fmaxf(mx, fabsf(v[e]));
    }
#pragma unroll
    for (int m = 1; m < 64; m *= 2) mx = fmaxf(mx, __shfl_xor(mx, m, 64));
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = mx;
    __syncthreads();
    if (threadIdx.x == 0) partial[blockIdx.x] = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
}

// One workgroup: *absmax_bits = max(*absmax_bits, partial[0 .. count)); then, if dyn is given,
// the constants of the dynamic mode for that maximum.
__global__ __launch_bounds__(256) void absmax_finish_kernel(const float *__restrict__ partial, int count,
                                                            unsigned *__restrict__ absmax_bits, int Kp, int qmax,
                                                            double c1_over_sa, float *__restrict__ dyn)
{
    __shared__ float red[4];
    float mx = 0.0f;
    for (int i = threadIdx.x; i < count; i += 256) mx = fmaxf(mx, partial[i]);
#pragma unroll
    for (int m = 1; m < 64; m *= 2) mx = fmaxf(mx, __shfl_xor(mx, m, 64));
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = mx;
    __syncthreads();
    if (threadIdx.x == 0) {
        mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
        unsigned bits = __float_as_uint(mx);
        if (*absmax_bits > bits) bits = *absmax_bits;
        *absmax_bits = bits;
        if (dyn) dyn_scale_write(bits, Kp, qmax, c1_over_sa, dyn);
    }
}

template <int KP>
static hipError_t launch_wht(const float *in, int64_t n, int K, float inv, int qmax, int8_t *codes,
                             const dhq_wht_fold *fold, hipStream_t st)
{
    constexpr int LPR = wht_shape<KP>::LPR;
    const int64_t threads = n * LPR;
    const unsigned blocks = (unsigned)((threads + 255) / 256);
    wht_quant_kernel<KP><<<blocks, 256, 0, st>>>(in, n, K, inv, qmax, codes, fold ? fold->partial : nullptr, fold ? fold->count : 0,
                                                 fold ? fold->c1_over_sa : 0.0, fold ? fold->dyn_out : nullptr);
    return hipGetLastError();
}

template <int KP>
static hipError_t launch_absmax(const float *in, int64_t n, int K, unsigned *absmax_bits, float *partial, int qmax,
                                double c1_over_sa, float *dyn, int *count_out, hipStream_t st)
{
    constexpr int LPR = wht_shape<KP>::LPR;
    const int64_t need = (n * LPR + 255) / 256;
    const unsigned blocks = (unsigned)(need < DHQ_ABSMAX_BLOCKS ? need : DHQ_ABSMAX_BLOCKS);  // 8 workgroups per CU
    wht_absmax_kernel<KP><<<blocks, 256, 0, st>>>(in, n, K, partial);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (count_out) {  // the caller folds the partial maxima itself
        *count_out = (int)blocks;
        return hipSuccess;
    }
    absmax_finish_kernel<<<1, 256, 0, st>>>(partial, (int)blocks, absmax_bits, KP, qmax, c1_over_sa, dyn);
    return hipGetLastError();
}

hipError_t dhq_launch_wht_quant(const float *in, int64_t n, int K, int Kp, float inv, int qmax,
                                int8_t *codes, const dhq_wht_fold *fold, hipStream_t st)
{
    if (n <= 0) return hipSuccess;
    if (fold && (!fold->partial || !fold->dyn_out || fold->count < 1 || fold->count > DHQ_ABSMAX_PARTIALS)) return hipErrorInvalidValue;
    switch (Kp) {
        case 1: return launch_wht<1>(in, n, K, inv, qmax, codes, fold, st);
        case 2: return launch_wht<2>(in, n, K, inv, qmax, codes, fold, st);
        case 4: return launch_wht<4>(in, n, K, inv, qmax, codes, fold, st);
        case 8: return launch_wht<8>(in, n, K, inv, qmax, codes, fold, st);
        case 16: return launch_wht<16>(in, n, K, inv, qmax, codes, fold, st);
        case 32: return launch_wht<32>(in, n, K, inv, qmax, codes, fold, st);
        case 64: return launch_wht<64>(in, n, K, inv, qmax, codes, fold, st);
        case 128: return launch_wht<128>(in, n, K, inv, qmax, codes, fold, st);
        case 256: return launch_wht<256>(in, n, K, inv, qmax, codes, fold, st);
        case 512: return launch_wht<512>(in, n, K, inv, qmax, codes, fold, st);
        default: return hipErrorInvalidValue;
    }
}

static hipError_t wht_absmax_dispatch(const float *in, int64_t n, int K, int Kp, unsigned *absmax_bits, float *partial,
                                      int qmax, double c1_over_sa, float *dyn, int *count_out, hipStream_t st)
{
    switch (Kp) {
        case 1: return launch_absmax<1>(in, n, K, absmax_bits, partial, qmax, c1_over_sa, dyn, count_out, st);
        case 2: return launch_absmax<2>(in, n, K, absmax_bits, partial, qmax, c1_over_sa, dyn, count_out, st);
        case 4: return launch_absmax<4>(in, n, K, absmax_bits, partial, qmax, c1_over_sa, dyn, count_out, st);
        case 8: return launch_absmax<8>(in, n, K, absmax_bits, partial, qmax, c1_over_sa, dyn, count_out, st);
        case 16: return launch_absmax<16>(in, n, K, absmax_bits, partial, qmax, c1_over_sa, dyn, count_out, st);
        case 32: return launch_absmax<32>(in, n, K, absmax_bits, partial, qmax, c1_over_sa, dyn, count_out, st);
        case 64: return launch_absmax<64>(in, n, K, absmax_bits, partial, qmax, c1_over_sa, dyn, count_out, st);
        case 128: return launch_absmax<128>(in, n, K, absmax_bits, partial, qmax, c1_over_sa, dyn, count_out, st);
        case 256: return launch_absmax<256>(in, n, K, absmax_bits, partial, qmax, c1_over_sa, dyn, count_out, st);
        case 512: return launch_absmax<512>(in, n, K, absmax_bits, partial, qmax, c1_over_sa, dyn, count_out, st);
        default: return hipErrorInvalidValue;
    }
}

hipError_t dhq_launch_wht_absmax(const float *in, int64_t n, int K, int Kp, unsigned *absmax_bits, float *partial,
                                 int qmax, double c1_over_sa, float *dyn, hipStream_t st)
{
    if (n <= 0) return hipSuccess;
    if (!partial || !absmax_bits) return hipErrorInvalidValue;
    return wht_absmax_dispatch(in, n, K, Kp, absmax_bits, partial, qmax, c1_over_sa, dyn, nullptr, st);
}

hipError_t dhq_launch_wht_absmax_partials(const float *in, int64_t n, int K, int Kp, float *partial, int *count,
                                          hipStream_t st)
{
    if (n <= 0 || !partial || !count) return hipErrorInvalidValue;
    return wht_absmax_dispatch(in, n, K, Kp, nullptr, partial, 0, 0.0, nullptr, count, st);
}

// ------------------------------------------------------------------------- int8 GEMM, MFMA
// D[coord][feature] = sum_k q[coord][k] * Wq[feature][k] with v_mfma_i32_32x32x32_i8: the
// codes are the A operand (32 coords x 32 k), the weights the B operand (32 k x 32 features).
// Lane l supplies row/column l % 32 and the 16 consecutive k of half l / 32 for both operands
// (so a weight fragment has the same bytes whichever operand it feeds); it receives D rows
// 8*(v/4) + 4*(l/32) + v%4 (v = 0..15) of column l % 32.  With coordinates as rows the 32
// lanes of a wave half write 32 consecutive features of one coordinate per store: whole
// 128-byte lines (the other orientation, which the fused kernels need for their in-register
// transform, would write 32-byte pieces of 32 different lines).
//
// A workgroup of GEMM_WAVES waves covers 32 coordinates per wave x up to 4 M tiles (128 features); the weight
// fragments of its tiles are copied once into LDS ([tile][k block][lane] x 16 B, the order
// they are stored in device memory) and read back conflict-free with one 16-byte LDS load
// per lane.  Codes are read straight from device memory.
#define GEMM_WAVES 8  // waves per workgroup: 32 coordinates each, sharing the staged weight fragments

// The tiles of one wave, one after the other: a tile's epilogue and stores follow its MFMAs directly, so
// the stores of one tile travel while the next one is multiplied.  Accumulator v of a lane: coordinate
// row0 + 8 (v / 4) + 4 h + v % 4, feature 32 (tile0 + t) + c.  KIND: the activation of the epilogue, or
// -1 for the raw accumulators; FULL: all 32 rows exist.
template <int NKB, bool FULL, int KIND>
__device__ __forceinline__ void gemm_tiles(const dhq_v4i *lds, const dhq_v4i (&b)[NKB], int tile0, int ntile, int M, int64_t row0,
                                           int nrows, int lane, int32_t *__restrict__ acc_out, float *__restrict__ act_out,
                                           float c1, const float *__restrict__ bias, float c2)
{
    const int c = lane & 31, h = lane >> 5;
    const unsigned loff = (unsigned)(4 * h * M + c);  // this lane's place within a tile's 32 x M block of the output
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        if (t >= ntile) break;
        dhq_v16i acc;
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[v] = 0;
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb) {
            const dhq_v4i w = lds[(t * NKB + kb) * 64 + lane];
            acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(b[kb], w, acc, 0, 0, 0);
        }
        const int f = (tile0 + t) * 32 + c;
        if (f >= M) continue;
        const size_t tile_off = (size_t)row0 * M + (size_t)(tile0 + t) * 32;  // wave-uniform
        const float bf = (KIND >= 0) ? bias[f] : 0.f;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int rl = 8 * (v >> 2) + (v & 3);  // row within the block, less the lane half's 4 h
            if (!FULL && rl + 4 * h >= nrows) continue;
            if constexpr (KIND >= 0)
                (act_out + tile_off + (size_t)rl * M)[loff] = dhq_epilogue(acc[v], c1, bf, dhq_act{KIND, c2});
            else
                (acc_out + tile_off + (size_t)rl * M)[loff] = acc[v];
        }
    }
}
template <int NKB, bool ACT>
__global__ __launch_bounds__(64 * GEMM_WAVES) void gemm_i8_mfma_kernel(const int8_t *__restrict__ codes, int64_t n,
                                                           const int8_t *__restrict__ wfrag, int M, int Mt,
                                                           int32_t *__restrict__ acc_out,
                                                           float *__restrict__ act_out, float c1,
                                                           const float *__restrict__ bias, dhq_act act,
                                                           const float *__restrict__ dyn)
{
    if (ACT && dyn) c1 = dyn[1];
    extern __shared__ __align__(16) unsigned char lds_raw[];
    dhq_v4i *lds = reinterpret_cast<dhq_v4i *>(lds_raw);
    constexpr int KP = NKB * 32;
    const int tile0 = blockIdx.y * 4;
    const int ntile = min(4, Mt - tile0);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = lane & 31, h = lane >> 5;
    const int64_t row = (int64_t)blockIdx.x * (32 * GEMM_WAVES) + wave * 32 + c;
    const int64_t rrow = row < n ? row : n - 1;  // tail lanes read a valid row, store nothing
    const dhq_v4i *brow = reinterpret_cast<const dhq_v4i *>(codes + rrow * KP + 16 * h);

    // this lane's codes (from device memory) are requested first, so that they travel while the
    // block's A fragments are staged: ntile * NKB * 64 vectors of 16 B
    dhq_v4i b[NKB];
#pragma unroll
    for (int kb = 0; kb < NKB; ++kb) b[kb] = brow[kb * 2];
    {
        const dhq_v4i *src = reinterpret_cast<const dhq_v4i *>(wfrag) + (size_t)tile0 * NKB * 64;
        const int total = ntile * NKB * 64;
        for (int i = threadIdx.x; i < total; i += 64 * GEMM_WAVES) lds[i] = src[i];
    }
    __syncthreads();

    // The 32 rows of a wave start at a wave-uniform row, so every store address is a scalar base (row and tile)
    // plus one 32-bit lane offset that never changes; whole 32-row blocks skip the row checks, and the
    // activation is chosen once per wave, not once per value.
    const int64_t row0 = (int64_t)blockIdx.x * (32 * GEMM_WAVES) + __builtin_amdgcn_readfirstlane(wave) * 32;
    if (row0 >= n) return;  // no barrier below
    const int nrows = (n - row0 < 32) ? (int)(n - row0) : 32;
    const int kind = ACT ? act.kind : -1;
    if (nrows == 32) {
        if (kind == DHQ_ACT_KIND_SINE) gemm_tiles<NKB, true, DHQ_ACT_KIND_SINE>(lds, b, tile0, ntile, M, row0, nrows, lane, acc_out, act_out, c1, bias, act.c2);
        else if (kind == DHQ_ACT_KIND_WAVELET) gemm_tiles<NKB, true, DHQ_ACT_KIND_WAVELET>(lds, b, tile0, ntile, M, row0, nrows, lane, acc_out, act_out, c1, bias, act.c2);
        else if (kind == DHQ_ACT_KIND_NONE) gemm_tiles<NKB, true, DHQ_ACT_KIND_NONE>(lds, b, tile0, ntile, M, row0, nrows, lane, acc_out, act_out, c1, bias, act.c2);
        else gemm_tiles<NKB, true, -1>(lds, b, tile0, ntile, M, row0, nrows, lane, acc_out, act_out, c1, bias, act.c2);
    } else {
        if (kind == DHQ_ACT_KIND_SINE) gemm_tiles<NKB, false, DHQ_ACT_KIND_SINE>(lds, b, tile0, ntile, M, row0, nrows, lane, acc_out, act_out, c1, bias, act.c2);
        else if (kind == DHQ_ACT_KIND_WAVELET) gemm_tiles<NKB, false, DHQ_ACT_KIND_WAVELET>(lds, b, tile0, ntile, M, row0, nrows, lane, acc_out, act_out, c1, bias, act.c2);
        else if (kind == DHQ_ACT_KIND_NONE) gemm_tiles<NKB, false, DHQ_ACT_KIND_NONE>(lds, b, tile0, ntile, M, row0, nrows, lane, acc_out, act_out, c1, bias, act.c2);
        else gemm_tiles<NKB, false, -1>(lds, b, tile0, ntile, M, row0, nrows, lane, acc_out, act_out, c1, bias, act.c2);
    }
}

// Fan-in below 32 (the input layer, K = 2): the contraction is a handful of integer
// multiply-adds and the kernel is bound by its output.  Workgroup = 64 feature groups x 4
// coordinates, so no thread needs an integer division to find its place; a thread keeps the
// weights of its VEC consecutive features (4 when the row length allows 16-byte stores) in
// registers and walks over NARROW_ROWS coordinates.  KP = 0 takes the fan-in at run time.
#define NARROW_ROWS 8
// KIND: the activation, fixed at compile time so that the epilogue has no branch per value.
template <bool ACT, int VEC, int KP, int KIND>
__device__ __forceinline__ void gemm_narrow_body(const int8_t *__restrict__ codes, int64_t n, int Kp_rt,
                                                          const int8_t *__restrict__ wq, int M,
                                                          int32_t *__restrict__ acc_out,
                                                          float *__restrict__ act_out, float c1,
                                                          const float *__restrict__ bias, float c2,
                                                          const float *__restrict__ dyn)
{
    const dhq_act act{KIND, c2};
    if (ACT && dyn) c1 = dyn[1];
    const int Kp = KP ? KP : Kp_rt;
    constexpr int KMAX = KP ? KP : 16;
    const int groups = M / VEC;
    const int64_t row0 = ((int64_t)blockIdx.x * 4 + threadIdx.y) * NARROW_ROWS;
    for (int g = threadIdx.x; g < groups; g += 64) {
        const int f0 = g * VEC;
        int w[VEC][KMAX];
        float bv[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
#pragma unroll
            for (int k = 0; k < KMAX; ++k) w[e][k] = k < Kp ? (int)wq[(f0 + e) * Kp + k] : 0;
            bv[e] = ACT ? bias[f0 + e] : 0.f;
        }
#pragma unroll 2
        for (int r = 0; r < NARROW_ROWS; ++r) {
            const int64_t row = row0 + r;
            if (row >= n) break;
            int acc[VEC];
#pragma unroll
            for (int e = 0; e < VEC; ++e) acc[e] = 0;
#pragma unroll
            for (int k = 0; k < KMAX; ++k) {
                const int q = k < Kp ? (int)codes[row * Kp + k] : 0;
#pragma unroll
                for (int e = 0; e < VEC; ++e) acc[e] += q * w[e][k];
            }
            if (ACT) {
                float o[VEC];
#pragma unroll
                for (int e = 0; e < VEC; ++e) o[e] = dhq_epilogue(acc[e], c1, bv[e], act);
                if constexpr (VEC == 4)
                    *reinterpret_cast<float4 *>(act_out + row * M + f0) = make_float4(o[0], o[1], o[2], o[3]);
                else
                    act_out[row * M + f0] = o[0];
            } else {
                if constexpr (VEC == 4)
                    *reinterpret_cast<int4 *>(acc_out + row * M + f0) = make_int4(acc[0], acc[1], acc[2], acc[3]);
                else
                    acc_out[row * M + f0] = acc[0];
            }
        }
    }
}

template <bool ACT, int VEC, int KP>
__global__ __launch_bounds__(256) void gemm_narrow_kernel(const int8_t *__restrict__ codes, int64_t n, int Kp_rt,
                                                          const int8_t *__restrict__ wq, int M,
                                                          int32_t *__restrict__ acc_out,
                                                          float *__restrict__ act_out, float c1,
                                                          const float *__restrict__ bias, dhq_act act,
                                                          const float *__restrict__ dyn)
{
    if (act.kind == DHQ_ACT_KIND_SINE) gemm_narrow_body<ACT, VEC, KP, DHQ_ACT_KIND_SINE>(codes, n, Kp_rt, wq, M, acc_out, act_out, c1, bias, act.c2, dyn);
    else if (act.kind == DHQ_ACT_KIND_WAVELET) gemm_narrow_body<ACT, VEC, KP, DHQ_ACT_KIND_WAVELET>(codes, n, Kp_rt, wq, M, acc_out, act_out, c1, bias, act.c2, dyn);
    else gemm_narrow_body<ACT, VEC, KP, DHQ_ACT_KIND_NONE>(codes, n, Kp_rt, wq, M, acc_out, act_out, c1, bias, act.c2, dyn);
}

template <bool ACT, int VEC>
static void launch_gemm_narrow_kp(const dhq_layer &L, const int8_t *codes, int64_t n, int32_t *acc_out, float *act_out,
                                  float c1, const float *bias, dhq_act act, const float *dyn, hipStream_t st)
{
    const unsigned blocks = (unsigned)((n + 4 * NARROW_ROWS - 1) / (4 * NARROW_ROWS));
    const dim3 block(64, 4);
    if (L.Kp == 2)
        gemm_narrow_kernel<ACT, VEC, 2><<<blocks, block, 0, st>>>(codes, n, L.Kp, L.wq_dev, L.Mg, acc_out, act_out, c1, bias, act, dyn);
    else if (L.Kp == 4)
        gemm_narrow_kernel<ACT, VEC, 4><<<blocks, block, 0, st>>>(codes, n, L.Kp, L.wq_dev, L.Mg, acc_out, act_out, c1, bias, act, dyn);
    else
        gemm_narrow_kernel<ACT, VEC, 0><<<blocks, block, 0, st>>>(codes, n, L.Kp, L.wq_dev, L.Mg, acc_out, act_out, c1, bias, act, dyn);
}

template <bool ACT>
static hipError_t launch_gemm_narrow(const dhq_layer &L, const int8_t *codes, int64_t n, int32_t *acc_out, float *act_out,
                                     float c1, const float *bias, dhq_act act, const float *dyn, hipStream_t st)
{
    if ((L.Mg & 3) == 0)
        launch_gemm_narrow_kp<ACT, 4>(L, codes, n, acc_out, act_out, c1, bias, act, dyn, st);
    else
        launch_gemm_narrow_kp<ACT, 1>(L, codes, n, acc_out, act_out, c1, bias, act, dyn, st);
    return hipGetLastError();
}

template <int NKB>
static hipError_t launch_gemm_mfma(const dhq_layer &L, const int8_t *codes, int64_t n, int32_t *acc_out,
                                   float *act_out, float c1, const float *bias, dhq_act act, const float *dyn,
                                   hipStream_t st)
{
    dim3 grid((unsigned)((n + 32 * GEMM_WAVES - 1) / (32 * GEMM_WAVES)), (unsigned)((L.Mt + 3) / 4));
    const size_t lds = (size_t)(L.Mt < 4 ? L.Mt : 4) * NKB * 1024;
    int device = -1;
    if (lds > 48 * 1024 && hipGetDevice(&device) != hipSuccess) return hipErrorInvalidDevice;
    if (act_out) {
        auto kern = gemm_i8_mfma_kernel<NKB, true>;
        if (lds > 48 * 1024) {
            hipError_t e = dhq_lds_limit_once(kern, lds, device);
            if (e != hipSuccess) return e;
        }
        kern<<<grid, 64 * GEMM_WAVES, lds, st>>>(codes, n, L.wfrag_dev, L.Mg, L.Mt, nullptr, act_out, c1, bias, act, dyn);
    } else {
        auto kern = gemm_i8_mfma_kernel<NKB, false>;
        if (lds > 48 * 1024) {
            hipError_t e = dhq_lds_limit_once(kern, lds, device);
            if (e != hipSuccess) return e;
        }
        kern<<<grid, 64 * GEMM_WAVES, lds, st>>>(codes, n, L.wfrag_dev, L.Mg, L.Mt, acc_out, nullptr, c1, bias, act, dyn);
    }
    return hipGetLastError();
}

hipError_t dhq_launch_gemm(const dhq_layer &L, const int8_t *codes, int64_t n, int32_t *acc_out,
                           float *act_out, float c1, const float *bias, dhq_act act, const float *dyn, hipStream_t st)
{
    if (n <= 0) return hipSuccess;
    if ((acc_out == nullptr) == (act_out == nullptr)) return hipErrorInvalidValue;
    if (L.Kp < 32)
        return act_out ? launch_gemm_narrow<true>(L, codes, n, nullptr, act_out, c1, bias, act, dyn, st)
                       : launch_gemm_narrow<false>(L, codes, n, acc_out, nullptr, c1, bias, act, dyn, st);
    switch (L.Kp / 32) {
        case 1: return launch_gemm_mfma<1>(L, codes, n, acc_out, act_out, c1, bias, act, dyn, st);
        case 2: return launch_gemm_mfma<2>(L, codes, n, acc_out, act_out, c1, bias, act, dyn, st);
        case 4: return launch_gemm_mfma<4>(L, codes, n, acc_out, act_out, c1, bias, act, dyn, st);
        case 8: return launch_gemm_mfma<8>(L, codes, n, acc_out, act_out, c1, bias, act, dyn, st);
        case 16: return launch_gemm_mfma<16>(L, codes, n, acc_out, act_out, c1, bias, act, dyn, st);
        default: return hipErrorInvalidValue;
    }
}

// -------------------------------------------------------------------------------- epilogue
__global__ __launch_bounds__(256) void epilogue_kernel(const int32_t *__restrict__ acc, int64_t total, int M,
                                                       float c1, const float *__restrict__ bias, dhq_act act,
                                                       float *__restrict__ act_out)
{
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    act_out[idx] = dhq_epilogue(acc[idx], c1, bias[idx % M], act);
}

hipError_t dhq_launch_epilogue(const int32_t *acc, int64_t n, int M, float c1, const float *bias, dhq_act act,
                               float *act_out, hipStream_t st)
{
    if (n <= 0) return hipSuccess;
    const int64_t total = n * M;
    epilogue_kernel<<<(unsigned)((total + 255) / 256), 256, 0, st>>>(acc, total, M, c1, bias, act, act_out);
    return hipGetLastError();
}

// The complex wavelet (DHQ_ACT_KIND_WAVELET_COMPLEX) acts on the pairs (2p, 2p + 1) of a row: one thread per pair.
__global__ __launch_bounds__(256) void epilogue_pairs_kernel(const int32_t *__restrict__ acc, int64_t total_pairs, int half_m,
                                                             float c1, const float *__restrict__ bias, float c2,
                                                             const float *__restrict__ dyn, float *__restrict__ act_out)
{
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total_pairs) return;
    if (dyn) c1 = dyn[1];
    const int p = (int)(idx % half_m);
    const int2 a = reinterpret_cast<const int2 *>(acc)[idx];
    const float2 b = reinterpret_cast<const float2 *>(bias)[p];
    float ar, ai;
    dhq_activate_pair_rev<true>(__builtin_fmaf((float)a.x, c1, b.x), __builtin_fmaf((float)a.y, c1, b.y), c2, ar, ai);
    reinterpret_cast<float2 *>(act_out)[idx] = make_float2(ar, ai);
}

hipError_t dhq_launch_epilogue_pairs(const int32_t *acc, int64_t n, int M, float c1, const float *bias, dhq_act act,
                                     const float *dyn, float *act_out, hipStream_t st)
{
    if (n <= 0) return hipSuccess;
    if (M % 2 || act.kind != DHQ_ACT_KIND_WAVELET_COMPLEX) return hipErrorInvalidValue;
    const int64_t total = n * (M / 2);
    epilogue_pairs_kernel<<<(unsigned)((total + 255) / 256), 256, 0, st>>>(acc, total, M / 2, c1, bias, act.c2, dyn, act_out);
    return hipGetLastError();
}

// ------------------------------------------------------------ two-sided variant: un-rotation
// z = acc' H_MP over the output features of every row, in int32 (H has entries +-1, and
// H H = MP I, so this undoes the output-side rotation of the weights up to the factor that
// c1 carries), then y = z c1 + bias (and the sine) for the first M features.  Same lane
// layout and the same butterfly network as the forward transform (wht_shape, wht_butterflies).
// Intermediate sums may wrap; the host has checked that the final ones fit.
// KIND: the activation, fixed at compile time so that the epilogue has no branch per value.
template <int MP, int KIND>
__device__ __forceinline__ void unrotate_epilogue_body(const int32_t *__restrict__ acc, int64_t n, int M, float c1,
                                                       const float *__restrict__ bias, float c2, const float *__restrict__ dyn,
                                                       int32_t *__restrict__ z_out, float *__restrict__ act_out)
{
    const dhq_act act{KIND, c2};
    if (dyn) c1 = dyn[1];
    constexpr int EPL = wht_shape<MP>::EPL;
    constexpr int LPR = wht_shape<MP>::LPR;
    const int64_t gtid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t row = gtid / LPR;
    const int t = (int)(gtid % LPR);
    const bool live = row < n;
    using S = wht_shape<MP>;
    int v[EPL];
    if (live && EPL >= 4) {
#pragma unroll
        for (int g = 0; g < EPL / 4; ++g) {
            const int4 x = *reinterpret_cast<const int4 *>(acc + row * MP + S::index(t, 4 * g));
            v[(4 * g) % EPL] = x.x; v[(4 * g + 1) % EPL] = x.y; v[(4 * g + 2) % EPL] = x.z; v[(4 * g + 3) % EPL] = x.w;
        }
    } else {
#pragma unroll
        for (int e = 0; e < EPL; ++e) v[e] = live ? acc[row * MP + S::index(t, e)] : 0;
    }
    wht_butterflies<MP>(v, t);
    if (!live) return;
    if constexpr (EPL >= 4) {
#pragma unroll
        for (int g = 0; g < EPL / 4; ++g) {
            const int f = S::index(t, 4 * g);  // first of four consecutive features
            if (z_out) *reinterpret_cast<int4 *>(z_out + row * MP + f) = make_int4(v[4 * g], v[4 * g + 1], v[4 * g + 2], v[4 * g + 3]);
            if (act_out && f < M) {
                if ((M & 3) == 0) {
                    *reinterpret_cast<float4 *>(act_out + row * M + f) =
                        make_float4(dhq_epilogue(v[4 * g], c1, bias[f], act), dhq_epilogue(v[4 * g + 1], c1, bias[f + 1], act),
                                    dhq_epilogue(v[4 * g + 2], c1, bias[f + 2], act), dhq_epilogue(v[4 * g + 3], c1, bias[f + 3], act));
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (f + e < M) act_out[row * M + f + e] = dhq_epilogue(v[4 * g + e], c1, bias[f + e], act);
                }
            }
        }
    } else {
#pragma unroll
        for (int e = 0; e < EPL; ++e) {
            const int f = S::index(t, e);
            if (z_out) z_out[row * MP + f] = v[e];
            if (act_out && f < M) act_out[row * M + f] = dhq_epilogue(v[e], c1, bias[f], act);
        }
    }
}

template <int MP>
__global__ __launch_bounds__(256) void unrotate_epilogue_kernel(const int32_t *__restrict__ acc, int64_t n, int M,
                                                                float c1, const float *__restrict__ bias, dhq_act act,
                                                                const float *__restrict__ dyn,
                                                                int32_t *__restrict__ z_out,
                                                                float *__restrict__ act_out)
{
    if (act.kind == DHQ_ACT_KIND_SINE) unrotate_epilogue_body<MP, DHQ_ACT_KIND_SINE>(acc, n, M, c1, bias, act.c2, dyn, z_out, act_out);
    else if (act.kind == DHQ_ACT_KIND_WAVELET) unrotate_epilogue_body<MP, DHQ_ACT_KIND_WAVELET>(acc, n, M, c1, bias, act.c2, dyn, z_out, act_out);
    else unrotate_epilogue_body<MP, DHQ_ACT_KIND_NONE>(acc, n, M, c1, bias, act.c2, dyn, z_out, act_out);
}

template <int MP>
static hipError_t launch_unrotate(const int32_t *acc, int64_t n, int M, float c1, const float *bias, dhq_act act,
                                  const float *dyn, int32_t *z_out, float *act_out, hipStream_t st)
{
    constexpr int LPR = wht_shape<MP>::LPR;
    const int64_t threads = n * LPR;
    unrotate_epilogue_kernel<MP><<<(unsigned)((threads + 255) / 256), 256, 0, st>>>(acc, n, M, c1, bias, act, dyn,
                                                                                   z_out, act_out);
    return hipGetLastError();
}

hipError_t dhq_launch_unrotate(const int32_t *acc, int64_t n, int Mp, int M, float c1, const float *bias, dhq_act act,
                               const float *dyn, int32_t *z_out, float *act_out, hipStream_t st)
{
    if (n <= 0) return hipSuccess;
    switch (Mp) {
        case 1: return launch_unrotate<1>(acc, n, M, c1, bias, act, dyn, z_out, act_out, st);
        case 2: return launch_unrotate<2>(acc, n, M, c1, bias, act, dyn, z_out, act_out, st);
        case 4: return launch_unrotate<4>(acc, n, M, c1, bias, act, dyn, z_out, act_out, st);
        case 8: return launch_unrotate<8>(acc, n, M, c1, bias, act, dyn, z_out, act_out, st);
        case 16: return launch_unrotate<16>(acc, n, M, c1, bias, act, dyn, z_out, act_out, st);
        case 32: return launch_unrotate<32>(acc, n, M, c1, bias, act, dyn, z_out, act_out, st);
        case 64: return launch_unrotate<64>(acc, n, M, c1, bias, act, dyn, z_out, act_out, st);
        case 128: return launch_unrotate<128>(acc, n, M, c1, bias, act, dyn, z_out, act_out, st);
        case 256: return launch_unrotate<256>(acc, n, M, c1, bias, act, dyn, z_out, act_out, st);
        case 512: return launch_unrotate<512>(acc, n, M, c1, bias, act, dyn, z_out, act_out, st);
        default: return hipErrorInvalidValue;
    }
}

// Two-sided variant, static scales: the un-rotation and epilogue of a layer fused with the rotation and
// quantizer of the next one.  Both are transforms of one row with the same lane layout (the next layer's
// rotated length is this layer's padded fan-out), so the layer's activations stay in the lanes' registers
// instead of crossing device memory as fp32: rotated accumulators in, the next layer's codes out.
// The arithmetic is that of unrotate_epilogue_kernel followed by wht_quant_kernel (same functions, same order).
template <int MP, int KIND>
__global__ __launch_bounds__(256) void unrotate_quant_kernel(const int32_t *__restrict__ acc, int64_t n, int M, float c1,
                                                             const float *__restrict__ bias, float c2, float inv_next, int qmax,
                                                             int8_t *__restrict__ codes)
{
    using S = wht_shape<MP>;
    constexpr int EPL = S::EPL;
    constexpr int LPR = S::LPR;
    const dhq_act act{KIND, c2};
    const int64_t gtid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t row = gtid / LPR;
    const int t = (int)(gtid % LPR);
    const bool live = row < n;
    int v[EPL];
    if (live && EPL >= 4) {
#pragma unroll
        for (int g = 0; g < EPL / 4; ++g) {
            const int4 x = *reinterpret_cast<const int4 *>(acc + row * MP + S::index(t, 4 * g));
            v[(4 * g) % EPL] = x.x; v[(4 * g + 1) % EPL] = x.y; v[(4 * g + 2) % EPL] = x.z; v[(4 * g + 3) % EPL] = x.w;
        }
    } else {
#pragma unroll
        for (int e = 0; e < EPL; ++e) v[e] = live ? acc[row * MP + S::index(t, e)] : 0;
    }
    wht_butterflies<MP>(v, t);
    // the layer's output: features beyond the fan-out are the zero padding of the next layer's input
    float a[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) {
        const int f = S::index(t, e);
        a[e] = (live && f < M) ? dhq_epilogue(v[e], c1, bias[f], act) : 0.0f;
    }
    wht_butterflies<MP>(a, t);
    if (!live) return;
    if constexpr (EPL >= 4) {
#pragma unroll
        for (int e = 0; e < EPL; e += 4) {
            const unsigned w = dhq_pack4(dhq_quant_bits(a[e], inv_next, qmax), dhq_quant_bits(a[e + 1], inv_next, qmax),
                                         dhq_quant_bits(a[e + 2], inv_next, qmax), dhq_quant_bits(a[e + 3], inv_next, qmax));
            *reinterpret_cast<unsigned *>(codes + row * MP + S::index(t, e)) = w;
        }
    } else {
#pragma unroll
        for (int e = 0; e < EPL; ++e) codes[row * MP + S::index(t, e)] = (int8_t)(dhq_quant_bits(a[e], inv_next, qmax) & 0xff);
    }
}

template <int MP>
static hipError_t launch_unrotate_quant(const int32_t *acc, int64_t n, int M, float c1, const float *bias, dhq_act act,
                                        float inv_next, int qmax, int8_t *codes, hipStream_t st)
{
    constexpr int LPR = wht_shape<MP>::LPR;
    const unsigned grid = (unsigned)((n * LPR + 255) / 256);
    if (act.kind == DHQ_ACT_KIND_SINE)
        unrotate_quant_kernel<MP, DHQ_ACT_KIND_SINE><<<grid, 256, 0, st>>>(acc, n, M, c1, bias, act.c2, inv_next, qmax, codes);
    else if (act.kind == DHQ_ACT_KIND_WAVELET)
        unrotate_quant_kernel<MP, DHQ_ACT_KIND_WAVELET><<<grid, 256, 0, st>>>(acc, n, M, c1, bias, act.c2, inv_next, qmax, codes);
    else
        return hipErrorInvalidValue;
    return hipGetLastError();
}

hipError_t dhq_launch_unrotate_quant(const int32_t *acc, int64_t n, int Mp, int M, float c1, const float *bias, dhq_act act,
                                     float inv_next, int qmax, int8_t *codes, hipStream_t st)
{
    if (n <= 0) return hipSuccess;
    switch (Mp) {
        case 1: return launch_unrotate_quant<1>(acc, n, M, c1, bias, act, inv_next, qmax, codes, st);
        case 2: return launch_unrotate_quant<2>(acc, n, M, c1, bias, act, inv_next, qmax, codes, st);
        case 4: return launch_unrotate_quant<4>(acc, n, M, c1, bias, act, inv_next, qmax, codes, st);
        case 8: return launch_unrotate_quant<8>(acc, n, M, c1, bias, act, inv_next, qmax, codes, st);
        case 16: return launch_unrotate_quant<16>(acc, n, M, c1, bias, act, inv_next, qmax, codes, st);
        case 32: return launch_unrotate_quant<32>(acc, n, M, c1, bias, act, inv_next, qmax, codes, st);
        case 64: return launch_unrotate_quant<64>(acc, n, M, c1, bias, act, inv_next, qmax, codes, st);
        case 128: return launch_unrotate_quant<128>(acc, n, M, c1, bias, act, inv_next, qmax, codes, st);
        case 256: return launch_unrotate_quant<256>(acc, n, M, c1, bias, act, inv_next, qmax, codes, st);
        case 512: return launch_unrotate_quant<512>(acc, n, M, c1, bias, act, inv_next, qmax, codes, st);
        default: return hipErrorInvalidValue;
    }
}

// Clears n words (a kernel rather than a memset so that callers may capture the stream).
__global__ void clear_words_kernel(unsigned *p, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0u;
}

hipError_t dhq_launch_clear_words(unsigned *p, int n, hipStream_t st)
{
    if (n <= 0) return hipSuccess;
    clear_words_kernel<<<(n + 63) / 64, 64, 0, st>>>(p, n);
    return hipGetLastError();
}
