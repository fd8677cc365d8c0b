// Helpers shared by the fused whole-network kernels (dhq_fused.hip, dhq_fused_wide.hip).
#ifndef DHQ_FUSED_COMMON_H
#define DHQ_FUSED_COMMON_H

#include "dhq_device.h"

// Feature index held by register s of lane half u after an in-register butterfly network whose
// last stage is the lane swap (the integer un-rotation of the two-sided kernel).
static inline int rot_index(int s, int u)
{
    const int r = (s & ~1) | u;  // register the value came from before the lane swap
    const int H = s & 1;         // the lane-half bit of the output index
    return 32 * (r >> 4) + 8 * ((r >> 2) & 3) + 4 * H + (r & 3);
}

// Rotated feature index held by register s of lane half u when the 32-point factor of the
// transform runs on the matrix unit (its result arrives in the MFMA accumulator layout).
static inline int hm_index(int s, int u) { return 32 * (s >> 4) + 8 * ((s >> 2) & 3) + 4 * u + (s & 3); }

// Position of bias / output feature f inside a layer's bias block: [T][g][h][e].
static inline int bias_slot(int f)
{
    const int T = f >> 5, i = f & 31;
    const int g = i >> 3, h = (i >> 2) & 1, e = i & 3;
    return ((T * 4 + g) * 2 + h) * 4 + e;
}

// Copies `chunks` KiB from device memory straight into LDS: each wave moves 1 KiB per
// instruction (64 lanes x 16 B, LDS address = M0 + lane * 16), the waves of the workgroup take
// the KiB blocks round-robin.
//
// The load is written as inline assembly on purpose.  Through the compiler builtin the
// compiler knows that LDS is being written and, unable to tell which LDS reads could alias,
// makes the next LDS read wait for the whole copy (vmcnt(0)) -- which turns the copy of the
// next layer's weights, meant to run underneath this layer's arithmetic, into a synchronous
// one.  Here the kernels order the copy themselves: the destination buffer is never read
// between this call and the "s_waitcnt vmcnt(0)" + barrier that precedes its first use.
// Loads the compiler does not know about can only make its own vmcnt waits longer (memory
// operations retire in order), never shorter.
__device__ __forceinline__ void fused_issue_copy(const unsigned char *src, unsigned char *lds_dst,
                                                 int chunks, int wave, int lane, int n_waves)
{
    const unsigned lds_base = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char *)lds_dst;
    for (int q = wave; q < chunks; q += n_waves) {
        const unsigned char *g = src + (size_t)q * 1024 + lane * 16;
        const unsigned m0v = __builtin_amdgcn_readfirstlane(lds_base + q * 1024);
        asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
                     :
                     : "v"(g), "s"(m0v)
                     : "memory", "m0");
    }
}

// ---- pieces for running a 32-point Hadamard factor on the matrix unit ------------------------
typedef _Float16 dhq_v8h __attribute__((ext_vector_type(8)));
typedef float dhq_v16f __attribute__((ext_vector_type(16)));

// Two floats to packed binary16, rounded toward zero; element 0 in the low half.  (The
// round-to-nearest form, v_cvt_pk_f16_f32, issues at half the rate and would cost the kernels
// 3 % for a quarter less rounding error in the rotated activations.)
__device__ __forceinline__ unsigned hm_pack_half2(float a, float b)
{
    return __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_pkrtz(a, b));
}

// Splits two activations into binary16 pieces: hi = (a0, a1) rounded toward zero, lo = the
// remainders a - hi (exact in fp32; v_fma_mix_f32 reads the binary16 half in place) rounded
// toward zero.  hi + lo carries a to within 2^-21 |a| (2^-24 absolute below 2^-10).
__device__ __forceinline__ void hm_remainders(float a0, float a1, unsigned hi, float &r0, float &r1)
{
    asm("v_fma_mix_f32 %0, %1, 1.0, -%2 op_sel:[0,0,0] op_sel_hi:[0,0,1]" : "=v"(r0) : "v"(a0), "v"(hi));
    asm("v_fma_mix_f32 %0, %1, 1.0, -%2 op_sel:[0,0,1] op_sel_hi:[0,0,1]" : "=v"(r1) : "v"(a1), "v"(hi));
}
__device__ __forceinline__ void hm_split_pair(float a0, float a1, unsigned &hi, unsigned &lo)
{
    hi = hm_pack_half2(a0, a1);
    float r0, r1;
    hm_remainders(a0, a1, hi, r0, r1);
    lo = hm_pack_half2(r0, r1);
}

// One dword of the A operand of an H_32 product: entries +-1 (binary16) of row `row` of the
// Sylvester matrix at the two tile rows i0 (low half) and i1 (high half).
__device__ __forceinline__ unsigned hm_h32_pair(int row, int i0, int i1)
{
    return ((__builtin_popcount(row & i0) & 1) ? 0xBC00u : 0x3C00u) |
           (((__builtin_popcount(row & i1) & 1) ? 0xBC00u : 0x3C00u) << 16);
}

// The quantizer of the fused kernels for four values at once: round (magic-number add inside the
// scaling fma), clamp (one three-operand median per value) and pack byte 0 of the four results into
// one dword of codes, value i in byte i.  Seven instructions for four codes; clamping with max and
// a sub-dword min that writes its byte in place takes eight.
__device__ __forceinline__ unsigned fused_quant4(float v0, float v1, float v2, float v3, float inv, int lo, int hi)
{
    const float v[4] = {v0, v1, v2, v3};
    unsigned r[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int c;
        asm("v_med3_i32 %0, %1, %2, %3" : "=v"(c) : "v"(__float_as_int(__builtin_fmaf(v[i], inv, DHQ_MAGIC_F))), "v"(lo), "v"(hi));
        r[i] = (unsigned)c;
    }
    const unsigned p01 = __builtin_amdgcn_perm(r[1], r[0], 0x0c0c0400u);  // bytes r0.0, r1.0, 0, 0
    const unsigned p23 = __builtin_amdgcn_perm(r[3], r[2], 0x04000c0cu);  // bytes 0, 0, r2.0, r3.0
    return p01 | p23;
}

// A operand of the H_32 products: a lane supplies row c of H_32 at the eight contraction slots
// 8 h + j of block kk, which stand for tile row 8 (v / 4) + 4 h + v % 4 with v = 8 kk + j (the row
// lane half h holds in accumulator v), as binary16 +-1.
__device__ __forceinline__ void fused_h32_operand(int c, int h, dhq_v4i (&hA)[2])
{
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) {
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            const int v = 8 * kk + 2 * d;  // accumulators v and v + 1: consecutive tile rows
            const int row = 8 * (v >> 2) + 4 * h + (v & 3);
            hA[kk][d] = (int)hm_h32_pair(c, row, row + 1);
        }
    }
}

// The coordinate vector of the input layer (fan-in <= 4): rotated and quantized into code dword 0.
__device__ __forceinline__ int fused_input_codes(const float *__restrict__ coords, int64_t cl, int k0, int k0p, float inv, int qmax)
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
    return (int)dhq_pack4(dhq_quant_bits(v[0], inv, qmax), dhq_quant_bits(v[1], inv, qmax),
                          dhq_quant_bits(v[2], inv, qmax), dhq_quant_bits(v[3], inv, qmax));
}

#endif
