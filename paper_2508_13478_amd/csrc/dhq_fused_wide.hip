// Whole-network fused DHQ forward for hidden width 512 (gfx950).
//
// Same data layout and the same arithmetic as dhq_fused.hip (features are the MFMA M
// dimension, a wave carries 32 coordinates through all layers in registers, the weights are
// packed offline in the k order the in-register Walsh-Hadamard transform produces), with
// what changes when a lane has to hold 256 activations instead of 128:
//
//   - one wave per SIMD (4 waves per workgroup, 128 coordinates per pass) so that a wave owns
//     the whole 512-entry register file; the matrix unit and the vector ALU overlap inside
//     the wave (every MFMA issues in the shadow of about eight vector instructions);
//   - the activations of a layer are kept as two halves (rows 0-7 / rows 8-15 of every
//     32-row tile).  The butterfly stages over the tile index never mix the halves, so the
//     second half waits in accumulation registers (which the vector ALU cannot compute on,
//     but which cost one move in and one move out) while the first is transformed and
//     quantized;
//   - a 512 x 512 layer is 256 KiB of int8, more than LDS holds: it is streamed in four
//     chunks of four M tiles (64 KiB of A fragments + their biases) through two LDS buffers,
//     each chunk copied global -> LDS while the previous one is being consumed.
#include <math.h>
#include <string.h>

#include <new>
#include <utility>
#include <vector>

#include "dhq_device.h"
#include "dhq_fused_common.h"
#include "dhq_internal.h"

#define WIDE_WAVES 4
#define WIDE_THREADS (WIDE_WAVES * 64)
#define WIDE_TILE (WIDE_WAVES * 32)  // coordinates per workgroup pass
#define WIDE_MAX_CHUNKS 64
#define WIDE_CH 4                    // M tiles per chunk of a hidden layer

struct wide_args {
    const float *coords;
    float *out;
    const unsigned char *blob;
    int64_t n;
    int n_layers;
    int k0, k0p;
    int m_out;
    int qmax;
    int n_chunks;                       // weight chunks per coordinate pass
    float c1[DHQ_MAX_LAYERS];           // sine layers: s_a s_w omega0 / (2 pi); output layer: s_a s_w
    float inv_in[DHQ_MAX_LAYERS];       // 1 / (s_a sqrt(Kp))
    uint32_t chunk_off[WIDE_MAX_CHUNKS];  // byte offset of each chunk in the blob
    uint32_t chunk_kib[WIDE_MAX_CHUNKS];  // its size in KiB
};

struct dhq_wide_plan {
    int nf = 0;
    unsigned char *blob_dev = nullptr;
    size_t blob_bytes = 0;
    wide_args args;
    size_t lds_bytes = 0;
    int n_cu = 0;
    std::vector<uint32_t> bias_off;  // per layer and tile: byte offset of the tile's 32 biases in the blob
};

// ----------------------------------------------------------------------------- device code
// State of the weight stream: `cc` counts the chunks this workgroup has entered so far;
// chunk j lives in LDS buffer j & 1.
struct wide_stream {
    const wide_args *A;
    unsigned char *lds;
    int blk;           // bytes per LDS buffer
    int total_chunks;  // chunks this workgroup will consume over all its coordinate passes
    int wave, lane;
};

// Entering chunk `cc`: all of its bytes have landed (every wave waits for its own loads, then
// the barrier), nobody reads chunk cc-1 any more, so chunk cc+1 may overwrite it.
__device__ __forceinline__ void wide_enter_chunk(const wide_stream &S, int cc)
{
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
    __syncthreads();
    const int j = cc + 1;
    if (j < S.total_chunks) {
        const int t = j % S.A->n_chunks;
        fused_issue_copy(S.A->blob + S.A->chunk_off[t], S.lds + (j & 1) * S.blk, (int)S.A->chunk_kib[t], S.wave, S.lane,
                         WIDE_WAVES);
    }
}

__device__ __forceinline__ int wide_park(float v)
{
    int a;
    asm volatile("v_accvgpr_write_b32 %0, %1" : "=a"(a) : "v"(v));
    return a;
}
__device__ __forceinline__ float wide_unpark(int a)
{
    float v;
    asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(v) : "a"(a));
    return v;
}

// One layer's GEMM + epilogue + in-tile butterflies, tiles one after the other:
//   step g            MFMA (tile g / KB, k block g % KB)
//   steps +KB .. +2KB  the tile's 16 accumulators are drained (dequantize + bias + sine)
//   steps +2KB .. +3KB the four butterfly stages over the tile's 16 values; then rows 0-7 go
//                      to xlo and rows 8-15 are parked in xhi (accumulation registers)
// A fragments are fetched from LDS PF MFMAs ahead; when that prefetch crosses into the next
// chunk of CH tiles the chunk is entered first (wide_enter_chunk).  Every step is its own
// template instance, so all register indices are compile-time constants.
template <int NT, int KB, int NCD>
struct wide_gemm_ctx {
    static constexpr int PF = (NT * KB >= 4) ? 4 : (NT * KB >= 2 ? 2 : 1);
    const wide_stream &S;
    const dhq_v4i (&cd)[NCD];
    float (&xlo)[NT * 8];
    int (&xhi)[NT * 8];
    const unsigned char *bufs[2];
    int cc;
    float c1;
    int h;
    dhq_v4i fr[PF + 1];
    float4 bq[2][4];
    dhq_v16i acc[2];
    float tv[2][16];
    __device__ __forceinline__ wide_gemm_ctx(const wide_stream &S_, const dhq_v4i (&cd_)[NCD], float (&xlo_)[NT * 8],
                                             int (&xhi_)[NT * 8])
        : S(S_), cd(cd_), xlo(xlo_), xhi(xhi_)
    {
    }
};

template <int NT, int KB, int CH, int NCD, int G>
__device__ __forceinline__ void wide_gemm_step(wide_gemm_ctx<NT, KB, NCD> &C)
{
    constexpr int NM = NT * KB;
    constexpr int CHM = CH * KB;  // MFMAs per chunk
    constexpr int EPS = 16 / KB;
    constexpr int BPS = 32 / KB;
    constexpr int PF = wide_gemm_ctx<NT, KB, NCD>::PF;
    if constexpr (G < NM) {
        constexpr int T = G / KB, kb = G % KB;
        constexpr int pf = G + PF;
        if constexpr (pf < NM) {
            if constexpr (pf % CHM == 0) wide_enter_chunk(C.S, C.cc + pf / CHM);
            C.fr[pf % (PF + 1)] =
                reinterpret_cast<const dhq_v4i *>(C.bufs[(pf / CHM) & 1])[(pf % CHM) * 64 + C.S.lane];
            __builtin_amdgcn_sched_barrier(0);
        }
        // the tile's four bias vectors, early in its k loop (well before the chunk is left)
#pragma unroll
        for (int gg = 0; gg < 4; ++gg)
            if ((KB >= 4) ? (gg == kb) : (kb == 0)) {
                const unsigned char *bb = C.bufs[(T / CH) & 1] + CHM * 1024;
                C.bq[T & 1][gg] = reinterpret_cast<const float4 *>(bb)[((T % CH) * 4 + gg) * 2 + C.h];
            }
        if constexpr (kb == 0) {
#pragma unroll
            for (int v = 0; v < 16; ++v) C.acc[T & 1][v] = 0;
        }
        C.acc[T & 1] = __builtin_amdgcn_mfma_i32_32x32x32_i8(C.fr[G % (PF + 1)], C.cd[kb], C.acc[T & 1], 0, 0, 0);
    }
    if constexpr (G >= KB && G < NM + KB) {
        constexpr int Td = (G - KB) / KB, pos = (G - KB) % KB;
#pragma unroll
        for (int j = 0; j < EPS; ++j) {
            const int v = pos * EPS + j;
            const float4 bb = C.bq[Td & 1][v >> 2];
            const float bias = (v & 3) == 0 ? bb.x : (v & 3) == 1 ? bb.y : (v & 3) == 2 ? bb.z : bb.w;
            C.tv[Td & 1][v] = dhq_sin_rev(__builtin_fmaf((float)C.acc[Td & 1][v], C.c1, bias));
        }
    }
    if constexpr (G >= 2 * KB) {
        constexpr int Tb = (G - 2 * KB) / KB, pos = (G - 2 * KB) % KB;
#pragma unroll
        for (int j = 0; j < BPS; ++j) {
            const int b = pos * BPS + j;
            const int st = b >> 3, q = b & 7;
            const int r = ((q >> st) << (st + 1)) | (q & ((1 << st) - 1));
            const float u = C.tv[Tb & 1][r], w = C.tv[Tb & 1][r | (1 << st)];
            C.tv[Tb & 1][r] = u + w;
            C.tv[Tb & 1][r | (1 << st)] = u - w;
        }
        if constexpr (pos == KB - 1) {
#pragma unroll
            for (int r = 0; r < 8; ++r) {
                C.xlo[8 * Tb + r] = C.tv[Tb & 1][r];
                C.xhi[8 * Tb + r] = wide_park(C.tv[Tb & 1][8 + r]);
            }
        }
    }
    __builtin_amdgcn_sched_barrier(0);
}

template <int NT, int KB, int CH, int NCD, int... Gs>
__device__ __forceinline__ void wide_gemm_steps(wide_gemm_ctx<NT, KB, NCD> &C, std::integer_sequence<int, Gs...>)
{
    (wide_gemm_step<NT, KB, CH, NCD, Gs>(C), ...);
}

// cc is the running chunk count on entry and is advanced by the chunks consumed.
template <int NT, int KB, int CH, int NCD>
__device__ __forceinline__ void wide_gemm_sine(const wide_stream &S, int &cc, const dhq_v4i (&cd)[NCD], float c1,
                                               float (&xlo)[NT * 8], int (&xhi)[NT * 8], int h)
{
    constexpr int NM = NT * KB;
    constexpr int PF = wide_gemm_ctx<NT, KB, NCD>::PF;
    static_assert(CH * KB >= PF, "a chunk must be longer than the prefetch distance");
    wide_gemm_ctx<NT, KB, NCD> C(S, cd, xlo, xhi);
    C.cc = cc;
    C.c1 = c1;
    C.h = h;
    wide_enter_chunk(S, cc);
    C.bufs[0] = S.lds + (cc & 1) * S.blk;
    C.bufs[1] = S.lds + ((cc + 1) & 1) * S.blk;
#pragma unroll
    for (int m = 0; m < PF; ++m)
        if (m < NM) C.fr[m % (PF + 1)] = reinterpret_cast<const dhq_v4i *>(C.bufs[0])[m * 64 + S.lane];
    wide_gemm_steps<NT, KB, CH, NCD>(C, std::make_integer_sequence<int, NM + 2 * KB>{});
    cc += NT / CH;
}

// Remaining transform stages and the quantizer on one half (128 values, index 8 T + r):
// the stages over the tile index, then per group of four registers the stage over the
// lane-half bit fused with the quantizer.  The codes of rows r..r+3 of tile T go to dword
// dw0 + r / 4 of k block T.
template <int NT, int NCD>
__device__ __forceinline__ void wide_transform_quant(float (&xv)[NT * 8], dhq_v4i (&cd)[NCD], int dw0, float inv, int qlo,
                                                     int qhi)
{
    constexpr int NV = NT * 8;
#pragma unroll
    for (int s = 8; s < NV; s <<= 1) {
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            if ((i & s) == 0) {
                const float a = xv[i], b = xv[i | s];
                xv[i] = a + b;
                xv[i | s] = a - b;
            }
        }
    }
#pragma unroll
    for (int w = 0; w < NV / 4; ++w) {
        unsigned packed = 0;
#pragma unroll
        for (int pr = 0; pr < 2; ++pr) {
            const int s0 = 4 * w + 2 * pr;
            const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(xv[s0]), __float_as_uint(xv[s0 + 1]), false,
                                                            false);
            const float r0 = __uint_as_float(r[0]), r1 = __uint_as_float(r[1]);
            fused_quant_byte(packed, r0 + r1, inv, qlo, qhi, 2 * pr);
            fused_quant_byte(packed, r0 - r1, inv, qlo, qhi, 2 * pr + 1);
        }
        cd[w / 2][dw0 + (w & 1)] = (int)packed;
    }
}

template <int NF>
__global__ __launch_bounds__(WIDE_THREADS) void dhq_fused_wide_kernel(const wide_args A)
{
    constexpr int NT = NF / 32;
    constexpr int NKB = NF / 32;
    constexpr int BLK = (WIDE_CH * NKB + 1) * 1024;

    extern __shared__ __align__(16) unsigned char lds[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = lane & 31, h = lane >> 5;
    const int L = A.n_layers;
    const int64_t n_tiles = (A.n + WIDE_TILE - 1) / WIDE_TILE;
    if ((int64_t)blockIdx.x >= n_tiles) return;
    const int my_tiles = (int)((n_tiles - 1 - blockIdx.x) / gridDim.x) + 1;
    const int qlo = DHQ_MAGIC_I - A.qmax, qhi = DHQ_MAGIC_I + A.qmax;

    wide_stream S;
    S.A = &A;
    S.lds = lds;
    S.blk = BLK;
    S.total_chunks = my_tiles * A.n_chunks;
    S.wave = wave;
    S.lane = lane;
    int cc = 0;
    fused_issue_copy(A.blob + A.chunk_off[0], lds, (int)A.chunk_kib[0], wave, lane, WIDE_WAVES);

    for (int it = 0; it < my_tiles; ++it) {
        const int64_t tile = (int64_t)blockIdx.x + (int64_t)it * gridDim.x;
        const int64_t ci = tile * WIDE_TILE + wave * 32 + c;
        const bool valid = ci < A.n;
        const int64_t cl = valid ? ci : A.n - 1;

        dhq_v4i cd[NKB];
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb) cd[kb] = dhq_v4i{0, 0, 0, 0};
        {
            // input layer: rotate the coordinate vector (fan-in <= 4) and quantize it
            float v[4] = {0.f, 0.f, 0.f, 0.f};
            if (A.k0 == 2) {
                const float2 xy = *reinterpret_cast<const float2 *>(A.coords + cl * 2);
                v[0] = xy.x; v[1] = xy.y;
            } else {
                for (int k = 0; k < A.k0; ++k) v[k] = A.coords[cl * A.k0 + k];
            }
            if (A.k0p >= 2) {
                float a = v[0], b = v[1]; v[0] = a + b; v[1] = a - b;
                a = v[2]; b = v[3]; v[2] = a + b; v[3] = a - b;
            }
            if (A.k0p == 4) {
                float a = v[0], b = v[2]; v[0] = a + b; v[2] = a - b;
                a = v[1]; b = v[3]; v[1] = a + b; v[3] = a - b;
            }
            const float inv = A.inv_in[0];
            cd[0][0] = (int)dhq_pack4(dhq_quant_bits(v[0], inv, A.qmax), dhq_quant_bits(v[1], inv, A.qmax),
                                      dhq_quant_bits(v[2], inv, A.qmax), dhq_quant_bits(v[3], inv, A.qmax));
        }

        float xlo[NT * 8];
        int xhi[NT * 8];
        for (int l = 0; l < L - 1; ++l) {
            if (l == 0)
                wide_gemm_sine<NT, 1, NT, NKB>(S, cc, cd, A.c1[0], xlo, xhi, h);
            else
                wide_gemm_sine<NT, NKB, WIDE_CH, NKB>(S, cc, cd, A.c1[l], xlo, xhi, h);
            const float inv = A.inv_in[l + 1];
            wide_transform_quant<NT, NKB>(xlo, cd, 0, inv, qlo, qhi);
#pragma unroll
            for (int i = 0; i < NT * 8; ++i) xlo[i] = wide_unpark(xhi[i]);
            wide_transform_quant<NT, NKB>(xlo, cd, 2, inv, qlo, qhi);
        }

        // output layer: one zero-padded M tile, no sine
        {
            wide_enter_chunk(S, cc);
            const unsigned char *buf = lds + (cc & 1) * BLK;
            const dhq_v4i *wA = reinterpret_cast<const dhq_v4i *>(buf);
            const float *wB = reinterpret_cast<const float *>(buf + NKB * 1024);
            dhq_v16i acc;
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[v] = 0;
#pragma unroll
            for (int kb = 0; kb < NKB; ++kb) {
                const dhq_v4i a = wA[kb * 64 + lane];
                acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, cd[kb], acc, 0, 0, 0);
            }
            const float c1 = A.c1[L - 1];
            if (valid) {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int row = 8 * (v >> 2) + 4 * h + (v & 3);
                    if (row < A.m_out)
                        A.out[ci * A.m_out + row] =
                            __builtin_fmaf((float)acc[v], c1, wB[((v >> 2) * 2 + h) * 4 + (v & 3)]);
                }
            }
            cc += 1;
        }
    }
}

// ------------------------------------------------------------------------------- host code
bool dhq_wide_shape_ok(const dhq_model *m)
{
    const int L = m->n_layers;
    if (L < 2) return false;
    if (m->dims[0] > 4 || m->dims[L] > 32) return false;
    if (m->dims[1] != 512) return false;
    for (int l = 1; l < L; ++l)
        if (m->dims[l] != 512) return false;
    return 2 + 4 * (L - 2) <= WIDE_MAX_CHUNKS;
}

int dhq_wide_create(const dhq_model *m, dhq_wide_plan **plan_out)
{
    *plan_out = nullptr;
    if (!dhq_wide_shape_ok(m)) return DHQ_OK;
    const int L = m->n_layers;
    const int nf = 512, NT = nf / 32, NKB = nf / 32;
    dhq_wide_plan *P = new (std::nothrow) dhq_wide_plan();
    if (!P) return DHQ_ENOMEM;
    P->nf = nf;
    memset(&P->args, 0, sizeof(P->args));
    P->bias_off.assign((size_t)L * NT, 0);

    std::vector<unsigned char> blob;
    int n_chunks = 0;
    for (int l = 0; l < L; ++l) {
        const dhq_layer &Ly = m->layer[l];
        const int Mt = (l == L - 1) ? 1 : NT;
        const int Kb = (l == 0) ? 1 : NKB;
        const int ch = (l == 0) ? NT : (l == L - 1 ? 1 : WIDE_CH);  // tiles per chunk
        const int8_t *wq = Ly.wq_host.data();
        for (int T0 = 0; T0 < Mt; T0 += ch) {
            const size_t off = blob.size();
            const size_t frag_bytes = (size_t)ch * Kb * 1024;
            const size_t bias_bytes = (size_t)ch * 128;
            const size_t bytes = (frag_bytes + bias_bytes + 1023) / 1024 * 1024;
            blob.resize(off + bytes, 0);
            int8_t *frag = reinterpret_cast<int8_t *>(blob.data() + off);
            for (int tl = 0; tl < ch; ++tl) {
                const int T = T0 + tl;
                P->bias_off[(size_t)l * NT + T] = (uint32_t)(off + frag_bytes + (size_t)tl * 128);
                for (int kb = 0; kb < Kb; ++kb)
                    for (int ln = 0; ln < 64; ++ln) {
                        const int row = 32 * T + (ln & 31), u = ln >> 5;
                        for (int jj = 0; jj < 16; ++jj) {
                            int8_t val = 0;
                            if (row < Ly.M) {
                                if (l == 0) {
                                    if (u == 0 && jj < Ly.Kp) val = wq[(size_t)row * Ly.Kp + jj];
                                } else {
                                    val = wq[(size_t)row * Ly.Kp + rot_index(16 * kb + jj, u)];
                                }
                            }
                            frag[((size_t)(tl * Kb + kb) * 64 + ln) * 16 + jj] = val;
                        }
                    }
            }
            P->args.chunk_off[n_chunks] = (uint32_t)off;
            P->args.chunk_kib[n_chunks] = (uint32_t)(bytes / 1024);
            ++n_chunks;
        }
    }
    P->args.n_chunks = n_chunks;
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
    P->lds_bytes = (size_t)2 * (WIDE_CH * NKB + 1) * 1024;
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, m->device) != hipSuccess) {
        (void)hipFree(P->blob_dev);
        delete P;
        return DHQ_EHIP;
    }
    P->n_cu = prop.multiProcessorCount;
    *plan_out = P;
    return DHQ_OK;
}

void dhq_wide_destroy(dhq_wide_plan *P)
{
    if (!P) return;
    if (P->blob_dev) (void)hipFree(P->blob_dev);
    delete P;
}

int dhq_wide_update_scales(const dhq_model *m, dhq_wide_plan *P)
{
    if (!P) return DHQ_OK;
    const int L = m->n_layers;
    const int NT = P->nf / 32;
    const double two_pi = 6.283185307179586476925286766559;
    for (int l = 0; l < L; ++l) {
        const dhq_layer &Ly = m->layer[l];
        const bool last = (l == L - 1);
        const double sc = (double)Ly.s_a * (double)Ly.s_w;
        P->args.c1[l] = last ? (float)sc : (float)(sc * (double)m->omega0 / two_pi);
        P->args.inv_in[l] = (float)(1.0 / ((double)Ly.s_a * sqrt((double)Ly.Kp)));
        const std::vector<float> &src = last ? Ly.bias_host : Ly.bias_rev_host;
        const int Mt = last ? 1 : NT;
        for (int T = 0; T < Mt; ++T) {
            float blk[32] = {0};
            for (int i = 0; i < 32; ++i) {
                const int f = 32 * T + i;
                if (f < Ly.M) blk[bias_slot(i)] = src[f];
            }
            if (hipMemcpy(P->blob_dev + P->bias_off[(size_t)l * NT + T], blk, sizeof(blk), hipMemcpyHostToDevice) != hipSuccess)
                return DHQ_EHIP;
        }
    }
    return DHQ_OK;
}

hipError_t dhq_wide_launch(const dhq_wide_plan *P, const float *coords, int64_t n, float *out, hipStream_t st)
{
    if (!P) return hipErrorInvalidValue;
    if (n <= 0) return hipSuccess;
    wide_args a = P->args;
    a.coords = coords;
    a.out = out;
    a.n = n;
    const int64_t tiles = (n + WIDE_TILE - 1) / WIDE_TILE;
    const unsigned grid = (unsigned)(tiles < P->n_cu ? tiles : P->n_cu);
    auto kern = dhq_fused_wide_kernel<512>;
    hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)P->lds_bytes);
    if (e != hipSuccess) return e;
    kern<<<grid, WIDE_THREADS, P->lds_bytes, st>>>(a);
    return hipGetLastError();
}
