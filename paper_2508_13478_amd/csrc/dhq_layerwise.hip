// Layer-by-layer kernels of the DHQ forward path (paper Sec. 3.2-3.3), gfx950.
//
//   wht_quant   rotation of every activation row by the Walsh-Hadamard transform (Eq. 3,
//               vector case) fused with the symmetric quantizer, or with the absmax reduction
//               that calibration needs
//   gemm_i8     int8 x int8 -> int32 on MFMA (the MAC array of Sec. 3.3), optionally with the
//               dequantize + bias + sine epilogue fused in
//   gemm_narrow the same contraction for fan-in < 32, on integer ALU ops
//   epilogue    dequantize + bias + sine from stored accumulators
//
// Activations travel through device memory between these kernels; the fused whole-network
// kernel lives in dhq_fused.hip.
#include "dhq_device.h"
#include "dhq_internal.h"

// ------------------------------------------------------------------ rotation + quantizer
// Row-parallel transform.  A row of KP values is spread over LPR lanes holding EPL
// consecutive values each; butterflies over the low index bits stay inside a lane, the
// others exchange through wavefront shuffles.  The transform runs un-normalised
// (entries of H are +-1); 1/sqrt(KP) is folded into `inv`.
template <int KP>
struct wht_shape {
    static constexpr int EPL = KP >= 256 ? KP / 64 : (KP >= 4 ? 4 : KP);
    static constexpr int LPR = KP / EPL;
};

template <int KP, bool ABSMAX>
__global__ __launch_bounds__(256) void wht_quant_kernel(const float *__restrict__ in, int64_t n,
                                                        int K, float inv, int qmax,
                                                        int8_t *__restrict__ codes,
                                                        unsigned *__restrict__ absmax_bits)
{
    constexpr int EPL = wht_shape<KP>::EPL;
    constexpr int LPR = wht_shape<KP>::LPR;
    const int64_t gtid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t row = gtid / LPR;
    const int t = (int)(gtid % LPR);
    const bool live = row < n;

    float v[EPL];
    if (live && K == KP && EPL == 4) {
        const float4 x = *reinterpret_cast<const float4 *>(in + row * KP + t * 4);
        v[0] = x.x; v[1 % EPL] = x.y; v[2 % EPL] = x.z; v[3 % EPL] = x.w;
    } else {
#pragma unroll
        for (int e = 0; e < EPL; ++e) {
            const int idx = t * EPL + e;
            v[e] = (live && idx < K) ? in[row * K + idx] : 0.0f;
        }
    }
    // butterflies over the index bits held inside the lane
#pragma unroll
    for (int h = 1; h < EPL; h *= 2) {
#pragma unroll
        for (int e = 0; e < EPL; ++e) {
            if ((e & h) == 0) {
                const float a = v[e], b = v[e | h];
                v[e] = a + b;
                v[e | h] = a - b;
            }
        }
    }
    // butterflies over the index bits that select the lane
#pragma unroll
    for (int m = 1; m < LPR; m *= 2) {
        const bool upper = (t & m) != 0;
#pragma unroll
        for (int e = 0; e < EPL; ++e) {
            const float p = __shfl_xor(v[e], m, 64);
            v[e] = upper ? p - v[e] : v[e] + p;
        }
    }

    if (ABSMAX) {
        float mx = 0.0f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) mx = fmaxf(mx, fabsf(v[e]));
#pragma unroll
        for (int m = 1; m < 64; m *= 2) mx = fmaxf(mx, __shfl_xor(mx, m, 64));
        // one word collects the maximum; a wave only pays for the atomic when it would raise it
        if ((threadIdx.x & 63) == 0) {
            const unsigned bits = __float_as_uint(mx);  // non-negative floats order like unsigned ints
            if (bits > __hip_atomic_load(absmax_bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))
                atomicMax(absmax_bits, bits);
        }
        return;
    }

    if (!live) return;
    int8_t *dst = codes + row * KP + t * EPL;
    if constexpr (EPL >= 4) {
#pragma unroll
        for (int e = 0; e < EPL; e += 4) {
            const unsigned w = dhq_pack4(dhq_quant_bits(v[e], inv, qmax), dhq_quant_bits(v[e + 1], inv, qmax),
                                         dhq_quant_bits(v[e + 2], inv, qmax), dhq_quant_bits(v[e + 3], inv, qmax));
            *reinterpret_cast<unsigned *>(dst + e) = w;
        }
    } else {
#pragma unroll
        for (int e = 0; e < EPL; ++e) dst[e] = (int8_t)(dhq_quant_bits(v[e], inv, qmax) & 0xff);
    }
}

template <int KP>
static hipError_t launch_wht(const float *in, int64_t n, int K, float inv, int qmax, int8_t *codes,
                             unsigned *absmax_bits, hipStream_t st)
{
    constexpr int LPR = wht_shape<KP>::LPR;
    const int64_t threads = n * LPR;
    const unsigned blocks = (unsigned)((threads + 255) / 256);
    if (absmax_bits)
        wht_quant_kernel<KP, true><<<blocks, 256, 0, st>>>(in, n, K, inv, qmax, codes, absmax_bits);
    else
        wht_quant_kernel<KP, false><<<blocks, 256, 0, st>>>(in, n, K, inv, qmax, codes, absmax_bits);
    return hipGetLastError();
}

hipError_t dhq_launch_wht_quant(const float *in, int64_t n, int K, int Kp, float inv, int qmax,
                                int8_t *codes, unsigned *absmax_bits, hipStream_t st)
{
    if (n <= 0) return hipSuccess;
    switch (Kp) {
        case 1: return launch_wht<1>(in, n, K, inv, qmax, codes, absmax_bits, st);
        case 2: return launch_wht<2>(in, n, K, inv, qmax, codes, absmax_bits, st);
        case 4: return launch_wht<4>(in, n, K, inv, qmax, codes, absmax_bits, st);
        case 8: return launch_wht<8>(in, n, K, inv, qmax, codes, absmax_bits, st);
        case 16: return launch_wht<16>(in, n, K, inv, qmax, codes, absmax_bits, st);
        case 32: return launch_wht<32>(in, n, K, inv, qmax, codes, absmax_bits, st);
        case 64: return launch_wht<64>(in, n, K, inv, qmax, codes, absmax_bits, st);
        case 128: return launch_wht<128>(in, n, K, inv, qmax, codes, absmax_bits, st);
        case 256: return launch_wht<256>(in, n, K, inv, qmax, codes, absmax_bits, st);
        case 512: return launch_wht<512>(in, n, K, inv, qmax, codes, absmax_bits, st);
        default: return hipErrorInvalidValue;
    }
}

// ------------------------------------------------------------------------- int8 GEMM, MFMA
// D[feature][coord] = sum_k Wq[feature][k] * q[coord][k] with v_mfma_i32_32x32x32_i8:
// the weights are the A operand (32 features x 32 k), the codes the B operand (32 k x 32
// coords).  Lane l supplies row/column l % 32 and the 16 consecutive k of half l / 32 for
// both operands; it receives D rows 8*(v/4) + 4*(l/32) + v%4 (v = 0..15) of column l % 32.
//
// A workgroup of 4 waves covers 128 coordinates x up to 4 M tiles (128 features); the A
// fragments of its tiles are copied once into LDS ([tile][k block][lane] x 16 B, the order
// they are stored in device memory) and read back conflict-free with one 16-byte LDS load
// per lane.  Codes are read straight from device memory.
template <int NKB, bool ACT>
__global__ __launch_bounds__(256) void gemm_i8_mfma_kernel(const int8_t *__restrict__ codes, int64_t n,
                                                           const int8_t *__restrict__ wfrag, int M, int Mt,
                                                           int32_t *__restrict__ acc_out,
                                                           float *__restrict__ act_out, float c1,
                                                           const float *__restrict__ bias, int sine)
{
    extern __shared__ __align__(16) unsigned char lds_raw[];
    dhq_v4i *lds = reinterpret_cast<dhq_v4i *>(lds_raw);
    constexpr int KP = NKB * 32;
    const int tile0 = blockIdx.y * 4;
    const int ntile = min(4, Mt - tile0);
    // stage this block's A fragments: ntile * NKB * 64 vectors of 16 B
    {
        const dhq_v4i *src = reinterpret_cast<const dhq_v4i *>(wfrag) + (size_t)tile0 * NKB * 64;
        const int total = ntile * NKB * 64;
        for (int i = threadIdx.x; i < total; i += 256) lds[i] = src[i];
    }
    __syncthreads();

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = lane & 31, h = lane >> 5;
    const int64_t row = (int64_t)blockIdx.x * 128 + wave * 32 + c;
    const int64_t rrow = row < n ? row : n - 1;  // tail lanes read a valid row, store nothing
    const dhq_v4i *brow = reinterpret_cast<const dhq_v4i *>(codes + rrow * KP + 16 * h);

    dhq_v4i b[NKB];
#pragma unroll
    for (int kb = 0; kb < NKB; ++kb) b[kb] = brow[kb * 2];

    dhq_v16i acc[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[t][v] = 0;
    }
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        if (t < ntile) {
#pragma unroll
            for (int kb = 0; kb < NKB; ++kb) {
                const dhq_v4i a = lds[(t * NKB + kb) * 64 + lane];
                acc[t] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b[kb], acc[t], 0, 0, 0);
            }
        }
    }
    if (row >= n) return;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        if (t >= ntile) break;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int f = (tile0 + t) * 32 + 8 * g + 4 * h;  // first of 4 consecutive features
            if (f >= M) continue;
            if (ACT) {
                float o[4];
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    o[e] = (f + e < M) ? dhq_epilogue(acc[t][4 * g + e], c1, bias[f + e], sine != 0) : 0.0f;
                float *dst = act_out + row * M + f;
                if ((M & 3) == 0) {
                    *reinterpret_cast<float4 *>(dst) = make_float4(o[0], o[1], o[2], o[3]);
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (f + e < M) dst[e] = o[e];
                }
            } else {
                int32_t *dst = acc_out + row * M + f;
                if ((M & 3) == 0) {
                    *reinterpret_cast<int4 *>(dst) =
                        make_int4(acc[t][4 * g], acc[t][4 * g + 1], acc[t][4 * g + 2], acc[t][4 * g + 3]);
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (f + e < M) dst[e] = acc[t][4 * g + e];
                }
            }
        }
    }
}

// Fan-in below 32 (the input layer, K = 2): one thread per (coordinate, feature); the
// contraction is a handful of integer multiply-adds and the kernel is bound by its output.
template <bool ACT>
__global__ __launch_bounds__(256) void gemm_narrow_kernel(const int8_t *__restrict__ codes, int64_t n, int Kp,
                                                          const int8_t *__restrict__ wq, int M,
                                                          int32_t *__restrict__ acc_out,
                                                          float *__restrict__ act_out, float c1,
                                                          const float *__restrict__ bias, int sine)
{
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= n * M) return;
    const int64_t row = idx / M;
    const int f = (int)(idx % M);
    int acc = 0;
    for (int k = 0; k < Kp; ++k) acc += (int)codes[row * Kp + k] * (int)wq[f * Kp + k];
    if (ACT)
        act_out[idx] = dhq_epilogue(acc, c1, bias[f], sine != 0);
    else
        acc_out[idx] = acc;
}

template <int NKB>
static hipError_t launch_gemm_mfma(const dhq_layer &L, const int8_t *codes, int64_t n, int32_t *acc_out,
                                   float *act_out, float c1, const float *bias, bool sine, hipStream_t st)
{
    dim3 grid((unsigned)((n + 127) / 128), (unsigned)((L.Mt + 3) / 4));
    const size_t lds = (size_t)(L.Mt < 4 ? L.Mt : 4) * NKB * 1024;
    if (act_out) {
        auto kern = gemm_i8_mfma_kernel<NKB, true>;
        if (lds > 48 * 1024) {
            hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
        }
        kern<<<grid, 256, lds, st>>>(codes, n, L.wfrag_dev, L.M, L.Mt, nullptr, act_out, c1, bias, sine ? 1 : 0);
    } else {
        auto kern = gemm_i8_mfma_kernel<NKB, false>;
        if (lds > 48 * 1024) {
            hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
        }
        kern<<<grid, 256, lds, st>>>(codes, n, L.wfrag_dev, L.M, L.Mt, acc_out, nullptr, c1, bias, sine ? 1 : 0);
    }
    return hipGetLastError();
}

hipError_t dhq_launch_gemm(const dhq_layer &L, const int8_t *codes, int64_t n, int32_t *acc_out,
                           float *act_out, float c1, const float *bias, bool sine, hipStream_t st)
{
    if (n <= 0) return hipSuccess;
    if ((acc_out == nullptr) == (act_out == nullptr)) return hipErrorInvalidValue;
    if (L.Kp < 32) {
        const int64_t total = n * L.M;
        const unsigned blocks = (unsigned)((total + 255) / 256);
        if (act_out)
            gemm_narrow_kernel<true><<<blocks, 256, 0, st>>>(codes, n, L.Kp, L.wq_dev, L.M, nullptr, act_out, c1, bias, sine ? 1 : 0);
        else
            gemm_narrow_kernel<false><<<blocks, 256, 0, st>>>(codes, n, L.Kp, L.wq_dev, L.M, acc_out, nullptr, c1, bias, sine ? 1 : 0);
        return hipGetLastError();
    }
    switch (L.Kp / 32) {
        case 1: return launch_gemm_mfma<1>(L, codes, n, acc_out, act_out, c1, bias, sine, st);
        case 2: return launch_gemm_mfma<2>(L, codes, n, acc_out, act_out, c1, bias, sine, st);
        case 4: return launch_gemm_mfma<4>(L, codes, n, acc_out, act_out, c1, bias, sine, st);
        case 8: return launch_gemm_mfma<8>(L, codes, n, acc_out, act_out, c1, bias, sine, st);
        case 16: return launch_gemm_mfma<16>(L, codes, n, acc_out, act_out, c1, bias, sine, st);
        default: return hipErrorInvalidValue;
    }
}

// -------------------------------------------------------------------------------- epilogue
__global__ __launch_bounds__(256) void epilogue_kernel(const int32_t *__restrict__ acc, int64_t total, int M,
                                                       float c1, const float *__restrict__ bias, int sine,
                                                       float *__restrict__ act)
{
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    act[idx] = dhq_epilogue(acc[idx], c1, bias[idx % M], sine != 0);
}

hipError_t dhq_launch_epilogue(const int32_t *acc, int64_t n, int M, float c1, const float *bias, bool sine,
                               float *act, hipStream_t st)
{
    if (n <= 0) return hipSuccess;
    const int64_t total = n * M;
    epilogue_kernel<<<(unsigned)((total + 255) / 256), 256, 0, st>>>(acc, total, M, c1, bias, sine ? 1 : 0, act);
    return hipGetLastError();
}
