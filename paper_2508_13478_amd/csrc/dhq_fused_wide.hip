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
//     each chunk copied global -> registers -> LDS in small pieces between the GEMM steps of
//     the previous one;
//   - the codes (the MFMA B operand) live in accumulation registers too.
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
    // per layer and tile: byte offsets of the tile's 32 biases in the blob.  A hidden layer's
    // chunk also carries the biases of the tile before its first one (that tile's
    // accumulators are drained while this chunk is resident), hence up to two places.
    std::vector<uint32_t> bias_off, bias_off_dup;
};

// ----------------------------------------------------------------------------- device code
// State of the weight stream: `cc` counts the chunks this workgroup has entered so far;
// chunk j lives in LDS buffer j & 1.  While chunk j is being consumed, chunk j+1 is copied
// into the other buffer: cp_* describe that copy for this wave (it moves the 1 KiB blocks
// wave, wave + 4, wave + 8, ... of the chunk).
struct wide_stream {
    const wide_args *A;
    unsigned char *lds;
    int blk;           // bytes per LDS buffer
    int wave, lane;
    const unsigned char *cp_src;  // first byte of the chunk being copied in (uniform)
    unsigned cp_voff;             // wave * 1024 + lane * 16
    unsigned cp_dst;              // LDS address of this lane's 16 bytes of block `wave` in the destination
    int cp_kib;                   // blocks in that chunk
};

__device__ __forceinline__ unsigned wide_lds_addr(const unsigned char *p)
{
    return (unsigned)(size_t)(__attribute__((address_space(3))) const unsigned char *)p;
}

// Entering chunk `cc`: every wave has written its share of it to LDS (the wait, then the
// barrier) and nobody reads chunk cc-1 any more, so chunk cc+1 may overwrite it.
__device__ __forceinline__ void wide_enter_chunk(wide_stream &S, int cc)
{
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
    __syncthreads();
    // After the workgroup's last chunk this copies the first chunk of a pass that will not
    // happen, into the buffer nobody reads any more: harmless, and it keeps the pipeline
    // below free of branches.
    const int j = cc + 1;
    const int t = j % S.A->n_chunks;
    S.cp_src = S.A->blob + S.A->chunk_off[t];
    S.cp_kib = (int)S.A->chunk_kib[t];
    S.cp_dst = wide_lds_addr(S.lds + (j & 1) * S.blk) + S.cp_voff;
}

// The copy goes global -> registers -> LDS, one 1 KiB block (64 lanes x 16 B) per
// instruction pair, and is spread over the GEMM steps of the chunk being consumed.  (The
// direct global -> LDS load moves only about 32 B per clock and keeps the LDS busy meanwhile,
// which starves the A-fragment reads of all four waves; a ds_write_b128 moves 128 B per
// clock.)  The staging registers are accumulation registers, which are plentiful here, and
// both halves are inline assembly on registers the compiler does not know about: nothing may
// touch a staging register between the load and the write, because the data arrives
// asynchronously.  Each write waits with
// vmcnt(N), N = number of this wave's loads issued after the one it consumes (loads retire in
// order; anything else outstanding only makes the wait longer).
//
// Register map of the accumulation registers (the kernel caps the compiler at 256 + 160
// vector registers, so it never touches a160 and up; these are addressed by number in the
// assembly below and nothing the compiler does can move or copy them):
//   a0   .. a159  the compiler's: the parked half of the activations, spills
//   a160 .. a223  the codes of the current layer input (MFMA B operand), dword d of k block kb
//                 in a[160 + 4 kb + d]
//   a224 .. a255  eight staging tuples of the weight copy
#define WIDE_AGPR_COMPILER 160
#define WIDE_AGPR_CODES 160
#define WIDE_AGPR_STAGE 224
#define WIDE_STAGE 8    // staging tuples = loads in flight per wave
#define WIDE_SLOTS 17   // 1 KiB blocks per wave and chunk (chunks are at most 65 KiB)

// Slot I moves block wave + 4 I.  FULL: the chunk is taken to be 65 blocks long whatever its
// real size (a shorter chunk is followed in the blob by at least that many readable bytes,
// and the surplus lands in a part of the LDS buffer nobody reads); only the last slot, whose
// block exists for wave 0 alone, needs a decision -- the other waves fetch block `wave` again.
// Otherwise (the short copy at the end of a pass) every slot is checked against cp_kib.
template <int I, bool FULL>
__device__ __forceinline__ bool wide_copy_again(const wide_stream &S)
{
    if (FULL) return I == WIDE_SLOTS - 1 && S.wave != 0;
    return S.wave + 4 * I >= S.cp_kib;
}

template <int I, bool FULL>
__device__ __forceinline__ void wide_copy_load(const wide_stream &S)
{
    constexpr int R = WIDE_AGPR_STAGE + 4 * (I % WIDE_STAGE);
    const unsigned char *src = S.cp_src + (wide_copy_again<I, FULL>(S) ? 0 : I * 4096);  // scalar arithmetic
    asm volatile("global_load_dwordx4 a[%2:%3], %0, %1" : : "v"(S.cp_voff), "s"(src), "n"(R), "n"(R + 3) : "memory");
}

template <int I, bool FULL, int N>
__device__ __forceinline__ void wide_copy_store(const wide_stream &S)
{
    constexpr int R = WIDE_AGPR_STAGE + 4 * (I % WIDE_STAGE);
    if constexpr (FULL && I < 16) {
        asm volatile("s_waitcnt vmcnt(%3)\n\tds_write_b128 %0, a[%1:%2] offset:%4"
                     : : "v"(S.cp_dst), "n"(R), "n"(R + 3), "n"(N), "n"(I * 4096) : "memory");
    } else {
        const unsigned dst = S.cp_dst + (wide_copy_again<I, FULL>(S) ? 0 : I * 4096);
        asm volatile("s_waitcnt vmcnt(%3)\n\tds_write_b128 %0, a[%1:%2]" : : "v"(dst), "n"(R), "n"(R + 3), "n"(N) : "memory");
    }
}

// Step (of the layer's GEMM pipeline below) at which slot i of the copy that runs while
// chunk c of the layer is consumed is loaded / written.  Hidden layers (KB > 1): a chunk
// lasts CHM steps and is entered PF steps before its first MFMA; a load every second step,
// the write 16 steps later.  Input layer (KB == 1, one chunk, long steps): two loads per
// step, written two steps later.
template <int KB, int CHM, int PF>
constexpr int wide_load_step(int c, int i) { return KB == 1 ? i / 2 : c * CHM + 2 * i - PF; }
template <int KB, int CHM, int PF>
constexpr int wide_store_step(int c, int i) { return KB == 1 ? i / 2 + 2 : c * CHM + 2 * i + 16 - PF; }
template <int KB, int CHM, int PF>
constexpr int wide_store_vmcnt(int c, int i)
{
    int n = 0;
    for (int k = i + 1; k < WIDE_SLOTS; ++k)
        if (wide_load_step<KB, CHM, PF>(c, k) < wide_store_step<KB, CHM, PF>(c, i)) ++n;
    return n;
}

template <int KB, int CHM, int PF, int G, int IS>
__device__ __forceinline__ void wide_copy_slot_store(const wide_stream &S)
{
    constexpr int c = IS / WIDE_SLOTS, i = IS % WIDE_SLOTS;
    if constexpr (wide_store_step<KB, CHM, PF>(c, i) == G) wide_copy_store<i, true, wide_store_vmcnt<KB, CHM, PF>(c, i)>(S);
}
template <int KB, int CHM, int PF, int G, int IS>
__device__ __forceinline__ void wide_copy_slot_load(const wide_stream &S)
{
    constexpr int c = IS / WIDE_SLOTS, i = IS % WIDE_SLOTS;
    if constexpr (wide_load_step<KB, CHM, PF>(c, i) == G) wide_copy_load<i, true>(S);
}
template <int KB, int CHM, int PF, int NC, int G, int... Is>
__device__ __forceinline__ void wide_copy_step_impl(const wide_stream &S, std::integer_sequence<int, Is...>)
{
    // Is runs over c * WIDE_SLOTS + i; writes first, so that a staging tuple is free again
    // before the load of the same step takes it
    (wide_copy_slot_store<KB, CHM, PF, G, Is>(S), ...);
    (wide_copy_slot_load<KB, CHM, PF, G, Is>(S), ...);
}

template <int KB, int CHM, int PF, int NC, int G>
constexpr bool wide_copy_step_busy()
{
    for (int c = 0; c < NC; ++c)
        for (int i = 0; i < WIDE_SLOTS; ++i)
            if (wide_load_step<KB, CHM, PF>(c, i) == G || wide_store_step<KB, CHM, PF>(c, i) == G) return true;
    return false;
}

template <int KB, int CHM, int PF, int NC, int G>
__device__ __forceinline__ void wide_copy_step(const wide_stream &S)
{
    if constexpr (wide_copy_step_busy<KB, CHM, PF, NC, G>())
        wide_copy_step_impl<KB, CHM, PF, NC, G>(S, std::make_integer_sequence<int, NC * WIDE_SLOTS>{});
}

__device__ __forceinline__ int wide_park(float v)
{
    int a;
    asm volatile("v_accvgpr_write_b32 %0, %1" : "=a"(a) : "v"(v));
    return a;
}
// dword D of the codes (see the register map above)
template <int D>
__device__ __forceinline__ void wide_code_write(int v)
{
    asm volatile("v_accvgpr_write_b32 a[%1], %0" : : "v"(v), "n"(WIDE_AGPR_CODES + D));
}
__device__ __forceinline__ float wide_unpark(int a)
{
    float v;
    asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(v) : "a"(a));
    return v;
}

// The MFMA with its B operand (the codes) read from the fixed accumulation registers, which
// frees 64 vector registers.  The compiler has no builtin form for that, so it is inline assembly,
// and the wait states the matrix unit needs before the vector ALU reads its result are kept
// by construction: a tile's accumulators are first read a whole pipeline step (more than
// eleven instructions) after the tile's last MFMA was issued, plus an explicit s_nop.
template <int KBI>
__device__ __forceinline__ void wide_mfma_first(dhq_v16i &acc, const dhq_v4i &a)
{
    constexpr int R = WIDE_AGPR_CODES + 4 * KBI;
    asm volatile("v_mfma_i32_32x32x32_i8 %0, %1, a[%2:%3], 0" : "=&v"(acc) : "v"(a), "n"(R), "n"(R + 3));
}
template <int KBI>
__device__ __forceinline__ void wide_mfma_next(dhq_v16i &acc, const dhq_v4i &a)
{
    constexpr int R = WIDE_AGPR_CODES + 4 * KBI;
    asm volatile("v_mfma_i32_32x32x32_i8 %0, %1, a[%2:%3], %0" : "+v"(acc) : "v"(a), "n"(R), "n"(R + 3));
}

// N idle issue slots that the accumulators' readers cannot be moved ahead of.
template <int N>
__device__ __forceinline__ void wide_mfma_settle(dhq_v16i &acc)
{
    static_assert(N == 4 || N == 16, "");
    if (N == 4)
        asm volatile("s_nop 3" : "+v"(acc));
    else
        asm volatile("s_nop 7\n\ts_nop 7" : "+v"(acc));
}

__device__ __forceinline__ float wide_comp(const float4 &v, int i) { return i == 0 ? v.x : i == 1 ? v.y : i == 2 ? v.z : v.w; }

// One layer's GEMM + epilogue + in-tile butterflies, tiles one after the other, as a
// software pipeline over steps g (every step is its own template instance, so all register
// indices are compile-time constants):
//   step g                MFMA (tile g / KB, k block g % KB); its A fragment was fetched from
//                         LDS PF steps earlier; when that prefetch crosses into the next
//                         chunk of CH tiles the chunk is entered first
//   hidden layers (KB = 16, one accumulator per step): value e = g - KB is converted, value
//                         e - 1 gets its multiply-add with the bias, value e - 2 its sine --
//                         the three dependent instructions of one value sit in three
//                         different steps; the four butterfly stages of a tile follow, two
//                         butterflies per step
//   input layer (KB = 1): step g runs the 32 butterflies of tile g - 1, then drains all 16
//                         accumulators of tile g
// After its last butterfly, rows 0-7 of a tile go to xlo and rows 8-15 are parked in xhi.
// Biases are read from LDS a few steps before use; those of tile T sit in the bias block
// of the chunk that is resident while T is drained (see the host-side packing).
template <int NT, int KB, int NCD>
struct wide_gemm_ctx {
    static constexpr int PF = (NT * KB >= 4) ? 4 : (NT * KB >= 2 ? 2 : 1);
    wide_stream &S;
    float (&xlo)[NT * 8];
    int (&xhi)[NT * 8];
    const unsigned char *bufs[2];
    int cc;
    float c1;
    int h;
    dhq_v4i fr[PF + 1];
    float4 bq[2];
    float4 bq0[4];  // input layer: the 16 biases of the tile drained next
    dhq_v16i acc[2];
    float tv[2][16];
    float ex, ey;
    __device__ __forceinline__ wide_gemm_ctx(wide_stream &S_, float (&xlo_)[NT * 8], int (&xhi_)[NT * 8])
        : S(S_), xlo(xlo_), xhi(xhi_)
    {
    }
};

// input layer (one chunk, bias block [tile][g][h][e]): the biases of tile T
template <int NT, int KB, int NCD, int CHM>
__device__ __forceinline__ void wide_load_bias0(wide_gemm_ctx<NT, KB, NCD> &C, int T)
{
#pragma unroll
    for (int gg = 0; gg < 4; ++gg)
        C.bq0[gg] = *reinterpret_cast<const float4 *>(C.bufs[0] + CHM * 1024 + T * 128 + gg * 32 + C.h * 16);
}

template <int NT, int KB, int CH, int NCD, int G>
__device__ __forceinline__ void wide_gemm_step(wide_gemm_ctx<NT, KB, NCD> &C)
{
    constexpr int NM = NT * KB;
    constexpr int CHM = CH * KB;  // MFMAs per chunk
    constexpr int NC = NT / CH;
    constexpr int NE = NT * 16;   // accumulators per lane and layer
    constexpr int PF = wide_gemm_ctx<NT, KB, NCD>::PF;
    if constexpr (G < NM) {
        constexpr int pf = G + PF;
        if constexpr (pf < NM) {
            if constexpr (pf % CHM == 0) wide_enter_chunk(C.S, C.cc + pf / CHM);
            C.fr[pf % (PF + 1)] =
                reinterpret_cast<const dhq_v4i *>(C.bufs[(pf / CHM) & 1])[(pf % CHM) * 64 + C.S.lane];
        }
    }
    wide_copy_step<KB, CHM, PF, NC, G>(C.S);
    if constexpr (G < NM) {
        constexpr int T = G / KB, kb = G % KB;
        constexpr int ab = (KB == 1) ? 0 : (T & 1);
        if constexpr (kb == 0)
            wide_mfma_first<kb>(C.acc[ab], C.fr[G % (PF + 1)]);
        else
            wide_mfma_next<kb>(C.acc[ab], C.fr[G % (PF + 1)]);
    }
    // the MFMA stays ahead of the step's vector work (this is what keeps the distance between
    // a tile's last MFMA and the first read of its accumulators)
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (KB == 1) {
        // input layer: one MFMA per tile; the previous tile's butterflies come first, which
        // also gives this tile's MFMA time to finish before its accumulators are read
        if constexpr (G >= 1 && G <= NT) {
            constexpr int Tb = G - 1;
#pragma unroll
            for (int b = 0; b < 32; ++b) {
                const int st = b >> 3, q = b & 7;
                const int r = ((q >> st) << (st + 1)) | (q & ((1 << st) - 1));
                const float u = C.tv[0][r], w = C.tv[0][r | (1 << st)];
                C.tv[0][r] = u + w;
                C.tv[0][r | (1 << st)] = u - w;
            }
#pragma unroll
            for (int r = 0; r < 8; ++r) {
                C.xlo[8 * Tb + r] = C.tv[0][r];
                C.xhi[8 * Tb + r] = wide_park(C.tv[0][8 + r]);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (G < NT) {
            if constexpr (G == 0) wide_mfma_settle<16>(C.acc[0]);
            float x[16];
#pragma unroll
            for (int v = 0; v < 16; ++v) x[v] = (float)C.acc[0][v];
#pragma unroll
            for (int v = 0; v < 16; ++v) x[v] = __builtin_fmaf(x[v], C.c1, wide_comp(C.bq0[v >> 2], v & 3));
#pragma unroll
            for (int v = 0; v < 16; ++v) C.tv[0][v] = dhq_sin_rev(x[v]);
        }
        if constexpr (G + 1 < NT) wide_load_bias0<NT, KB, NCD, CHM>(C, G + 1);  // for the next step
    } else {
        static_assert(KB == 1 || KB == 16, "one accumulator per step");
        constexpr int e0 = G - KB, e1 = e0 - 1, e2 = e0 - 2;
        if constexpr (e2 >= 0 && e2 < NE) C.tv[(e2 / 16) & 1][e2 % 16] = dhq_sin_rev(C.ey);
        if constexpr (e1 >= 0 && e1 < NE) C.ey = __builtin_fmaf(C.ex, C.c1, wide_comp(C.bq[(e1 / 4) & 1], e1 % 4));
        if constexpr (e0 >= 0 && e0 < NE) {
            if constexpr (e0 % 16 == 0) wide_mfma_settle<4>(C.acc[(e0 / 16) & 1]);
            C.ex = (float)C.acc[(e0 / 16) & 1][e0 % 16];
        }
        if constexpr (e0 + 4 >= 0 && (e0 + 4) % 4 == 0 && e0 + 4 < NE) {
            // biases of values e0+4 .. e0+7: tile Tg, rows group gg; chunk cT is resident while Tg is drained
            constexpr int ge = (e0 + 4) / 4, Tg = ge / 4, gg = ge % 4;
            constexpr int cT = ((Tg + 1) / CH < NC - 1) ? (Tg + 1) / CH : NC - 1;
            constexpr int tg = Tg - (cT * CH - 1);
            C.bq[ge & 1] =
                *reinterpret_cast<const float4 *>(C.bufs[cT & 1] + CHM * 1024 + tg * 128 + gg * 32 + C.h * 16);
        }
    }
    if constexpr (KB > 1) {
        constexpr int SK = 2;
        constexpr int BPS = 32 / KB;
        constexpr int gb = G - 2 * KB - SK;
        if constexpr (gb >= 0 && gb < NM) {
            constexpr int Tb = gb / KB, pos = gb % KB;
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
    }
    __builtin_amdgcn_sched_barrier(0);
}

template <int NT, int KB, int CH, int NCD, int... Gs>
__device__ __forceinline__ void wide_gemm_steps(wide_gemm_ctx<NT, KB, NCD> &C, std::integer_sequence<int, Gs...>)
{
    (wide_gemm_step<NT, KB, CH, NCD, Gs>(C), ...);
}
template <int KB, int CHM, int PF, int NC, int... Ps>
__device__ __forceinline__ void wide_copy_prologue(const wide_stream &S, std::integer_sequence<int, Ps...>)
{
    (wide_copy_step<KB, CHM, PF, NC, Ps - PF>(S), ...);  // steps -PF .. -1
}

// cc is the running chunk count on entry and is advanced by the chunks consumed.
template <int NT, int KB, int CH, int NCD>
__device__ __forceinline__ void wide_gemm_sine(wide_stream &S, int &cc, float c1, float (&xlo)[NT * 8], int (&xhi)[NT * 8],
                                               int h)
{
    constexpr int NM = NT * KB;
    constexpr int PF = wide_gemm_ctx<NT, KB, NCD>::PF;
    constexpr int NSTEPS = (KB == 1) ? NT + 1 : NM + 2 * KB + 2;
    static_assert(CH * KB >= PF, "a chunk must be longer than the prefetch distance");
    wide_gemm_ctx<NT, KB, NCD> C(S, xlo, xhi);
    C.cc = cc;
    C.c1 = c1;
    C.h = h;
    C.ex = C.ey = 0.f;
    wide_enter_chunk(S, cc);
    C.bufs[0] = S.lds + (cc & 1) * S.blk;
    C.bufs[1] = S.lds + ((cc + 1) & 1) * S.blk;
#pragma unroll
    for (int m = 0; m < PF; ++m)
        if (m < NM) C.fr[m % (PF + 1)] = reinterpret_cast<const dhq_v4i *>(C.bufs[0])[m * 64 + S.lane];
    if constexpr (KB == 1) wide_load_bias0<NT, KB, NCD, CH * KB>(C, 0);
    wide_copy_prologue<KB, CH * KB, PF, NT / CH>(S, std::make_integer_sequence<int, PF>{});
    wide_gemm_steps<NT, KB, CH, NCD>(C, std::make_integer_sequence<int, NSTEPS>{});
    cc += NT / CH;
}

// Remaining transform stages and the quantizer on one half (128 values, index 8 T + r):
// the stages over the tile index, then per group of four registers the stage over the
// lane-half bit fused with the quantizer.  The codes of rows r..r+3 of tile T become dword
// DW0 + r / 4 of k block T, kept in an accumulation register (the MFMA reads them there).
template <int DW0, int W>
__device__ __forceinline__ void wide_quant_group(const float *xv, float inv, int qlo, int qhi)
{
    unsigned packed = 0;
#pragma unroll
    for (int pr = 0; pr < 2; ++pr) {
        const int s0 = 4 * W + 2 * pr;
        const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(xv[s0]), __float_as_uint(xv[s0 + 1]), false, false);
        const float r0 = __uint_as_float(r[0]), r1 = __uint_as_float(r[1]);
        fused_quant_byte(packed, r0 + r1, inv, qlo, qhi, 2 * pr);
        fused_quant_byte(packed, r0 - r1, inv, qlo, qhi, 2 * pr + 1);
    }
    wide_code_write<(W / 2) * 4 + DW0 + (W & 1)>((int)packed);
}
template <int DW0, int NV, int... Ws>
__device__ __forceinline__ void wide_quant_groups(const float (&xv)[NV], float inv, int qlo, int qhi,
                                                  std::integer_sequence<int, Ws...>)
{
    (wide_quant_group<DW0, Ws>(xv, inv, qlo, qhi), ...);
}
template <int NT, int DW0>
__device__ __forceinline__ void wide_transform_quant(float (&xv)[NT * 8], float inv, int qlo, int qhi)
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
    wide_quant_groups<DW0, NV>(xv, inv, qlo, qhi, std::make_integer_sequence<int, NV / 4>{});
}

template <int NKB, int... Ks>
__device__ __forceinline__ void wide_out_mfmas(dhq_v16i &acc, const dhq_v4i *wA, int lane, std::integer_sequence<int, Ks...>)
{
    ((Ks == 0 ? wide_mfma_first<Ks>(acc, wA[Ks * 64 + lane]) : wide_mfma_next<Ks>(acc, wA[Ks * 64 + lane])), ...);
}

template <int NF>
__global__ __launch_bounds__(WIDE_THREADS) __attribute__((amdgpu_num_vgpr(256 + WIDE_AGPR_COMPILER)))
void dhq_fused_wide_kernel(const wide_args A)
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
    S.wave = __builtin_amdgcn_readfirstlane(wave);
    S.lane = lane;
    S.cp_voff = (unsigned)(wave * 1024 + lane * 16);
    S.cp_kib = 0;
    S.cp_src = A.blob;
    S.cp_dst = 0;
    int cc = 0;
    // the very first chunk has nobody to copy it in the background
    for (int q = wave; q < (int)A.chunk_kib[0]; q += WIDE_WAVES)
        reinterpret_cast<dhq_v4i *>(lds)[q * 64 + lane] =
            reinterpret_cast<const dhq_v4i *>(A.blob + A.chunk_off[0])[q * 64 + lane];

    // the registers addressed by number count towards the kernel's register allocation
    asm volatile("" ::: "a255");
    static_assert(WIDE_AGPR_CODES + 4 * NKB <= WIDE_AGPR_STAGE && WIDE_AGPR_STAGE + 4 * WIDE_STAGE <= 256, "register map");

    for (int it = 0; it < my_tiles; ++it) {
        const int64_t tile = (int64_t)blockIdx.x + (int64_t)it * gridDim.x;
        const int64_t ci = tile * WIDE_TILE + wave * 32 + c;
        const bool valid = ci < A.n;
        const int64_t cl = valid ? ci : A.n - 1;

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
            // only k positions 0..3 of the input layer's fragments are non-zero, so whatever the
            // other code dwords still hold from the previous pass is multiplied by zero
            wide_code_write<0>((int)dhq_pack4(dhq_quant_bits(v[0], inv, A.qmax), dhq_quant_bits(v[1], inv, A.qmax),
                                              dhq_quant_bits(v[2], inv, A.qmax), dhq_quant_bits(v[3], inv, A.qmax)));
        }

        float xlo[NT * 8];
        int xhi[NT * 8];
        wide_gemm_sine<NT, 1, NT, NKB>(S, cc, A.c1[0], xlo, xhi, h);
        for (int l = 1;; ++l) {
            // transform + quantize the output of layer l-1 (first rows 0-7 of every tile, then
            // the parked rows 8-15), which is the input of layer l
            const float inv = A.inv_in[l];
            wide_transform_quant<NT, 0>(xlo, inv, qlo, qhi);
#pragma unroll
            for (int i = 0; i < NT * 8; ++i) xlo[i] = wide_unpark(xhi[i]);
            wide_transform_quant<NT, 2>(xlo, inv, qlo, qhi);
            if (l == L - 1) break;
            wide_gemm_sine<NT, NKB, WIDE_CH, NKB>(S, cc, A.c1[l], xlo, xhi, h);
        }

        // output layer: one zero-padded M tile, no sine; meanwhile the next pass's first chunk
        // (at most 5 blocks per wave) is copied in
        {
            wide_enter_chunk(S, cc);
            const unsigned char *buf = lds + (cc & 1) * BLK;
            const dhq_v4i *wA = reinterpret_cast<const dhq_v4i *>(buf);
            const float *wB = reinterpret_cast<const float *>(buf + NKB * 1024);
            wide_copy_load<0, false>(S); wide_copy_load<1, false>(S); wide_copy_load<2, false>(S); wide_copy_load<3, false>(S);
            wide_copy_load<4, false>(S);
            dhq_v16i acc;
            wide_out_mfmas<NKB>(acc, wA, lane, std::make_integer_sequence<int, NKB>{});
            float bias[16];
#pragma unroll
            for (int v = 0; v < 16; ++v) bias[v] = wB[((v >> 2) * 2 + h) * 4 + (v & 3)];
            wide_copy_store<0, false, 4>(S); wide_copy_store<1, false, 3>(S); wide_copy_store<2, false, 2>(S);
            wide_copy_store<3, false, 1>(S); wide_copy_store<4, false, 0>(S);
            wide_mfma_settle<16>(acc);
            const float c1 = A.c1[L - 1];
            if (valid) {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int row = 8 * (v >> 2) + 4 * h + (v & 3);
                    if (row < A.m_out) A.out[ci * A.m_out + row] = __builtin_fmaf((float)acc[v], c1, bias[v]);
                }
            }
            cc += 1;
        }
    }
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
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
    P->bias_off_dup.assign((size_t)L * NT, 0);

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
            const bool hidden = (l != 0 && l != L - 1);
            const size_t bias_bytes = (size_t)(hidden ? ch + 1 : ch) * 128;  // hidden: [previous tile][ch tiles]
            const size_t bytes = (frag_bytes + bias_bytes + 1023) / 1024 * 1024;
            blob.resize(off + bytes, 0);
            int8_t *frag = reinterpret_cast<int8_t *>(blob.data() + off);
            for (int tl = 0; tl < ch; ++tl) {
                const int T = T0 + tl;
                P->bias_off[(size_t)l * NT + T] = (uint32_t)(off + frag_bytes + (size_t)(hidden ? tl + 1 : tl) * 128);
                if (hidden && tl == 0 && T > 0) P->bias_off_dup[(size_t)l * NT + T - 1] = (uint32_t)(off + frag_bytes);
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
    // the in-kernel copy always fetches 65 KiB from a chunk's start (see wide_copy_load)
    blob.resize(blob.size() + (size_t)(WIDE_CH * NKB + 1) * 1024, 0);
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
    for (int l = 0; l < L; ++l) {
        const dhq_layer &Ly = m->layer[l];
        const bool last = (l == L - 1);
        P->args.c1[l] = dhq_c1(m, l);
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
            const uint32_t dup = P->bias_off_dup[(size_t)l * NT + T];
            if (dup && hipMemcpy(P->blob_dev + dup, blk, sizeof(blk), hipMemcpyHostToDevice) != hipSuccess) return DHQ_EHIP;
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
