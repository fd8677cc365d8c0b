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
//   - the transformed activations of a layer (the outputs of the H_32 products on the matrix
//     unit, see dhq_fused.hip) are written by those MFMAs straight into accumulation
//     registers, which the vector ALU cannot compute on but which cost one move out; the
//     stages over the tile index and the quantizer then fetch them a quarter at a time (rows
//     4q .. 4q+3 of every tile: those stages never mix rows of a tile);
//   - a 512 x 512 layer is 256 KiB of int8, more than LDS holds: it is streamed in four
//     chunks of four M tiles (64 KiB of A fragments + their biases) through two LDS buffers,
//     each chunk copied global -> registers -> LDS in small pieces between the GEMM steps of
//     the previous one.
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
    float c2;                           // wavelet activation: 2 pi s0 sqrt(log2 e) / omega0
    float c1[DHQ_MAX_LAYERS];           // sine layers: s_a s_w omega0 / (2 pi); output layer: s_a s_w
    float inv_in[DHQ_MAX_LAYERS];       // 1 / (s_a sqrt(Kp))
    uint32_t chunk_off[WIDE_MAX_CHUNKS];  // byte offset of each chunk in the blob
    uint32_t chunk_kib[WIDE_MAX_CHUNKS];  // its size in KiB
};

struct dhq_wide_plan {
    int nf = 0;
    int act_kind = DHQ_ACT_KIND_SINE;  // the activation after every layer but the last
    unsigned char *blob_dev = nullptr;
    size_t blob_bytes = 0;
    wide_args args;
    size_t lds_bytes = 0;
    int n_cu = 0;
    int device = 0;
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
// Register map of the accumulation registers (the kernel caps the compiler at 256 vector
// registers, so it never touches an accumulation register; these are addressed by number in
// the assembly below and nothing the compiler does can move or copy them):
//   a0   .. a223  the transformed activations of tiles 0 .. 13, tile T in a[16 T .. 16 T + 15]
//                 (the D operand of its H_32 products); tiles 14 and 15 stay in vector registers
//   a224 .. a255  eight staging tuples of the weight copy
#define WIDE_AGPR_COMPILER 0
#define WIDE_AGPR_TILES 14
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

// Row v of transformed tile T (< WIDE_AGPR_TILES), fetched from its accumulation register.
template <int T, int V>
__device__ __forceinline__ float wide_tile_read()
{
    float x;
    asm volatile("v_accvgpr_read_b32 %0, a[%1]" : "=v"(x) : "n"(16 * T + V));
    return x;
}

// H_32 product number K (0: low pieces of block 0, 1: high pieces of block 0, 2 and 3: the same
// for block 1; small pieces first) of tile T, accumulated in a[16 T .. 16 T + 15].  The
// compiler has no way to pin an MFMA result to given accumulation registers, so it is inline
// assembly.  The compiler may have gathered an operand with a vector move just before it and
// cannot know that an MFMA follows, hence the two wait states in front.  A chain on one
// accumulator needs none between its links; the first read of the result (wide_tile_read)
// comes a whole transform phase later.
template <int T, int K>
__device__ __forceinline__ void wide_h32_mfma(const dhq_v4i &ha, const dhq_v4i &b)
{
    constexpr int R = 16 * T;
    if constexpr (K == 0)
        asm volatile("s_nop 1\n\tv_mfma_f32_32x32x16_f16 a[%2:%3], %0, %1, 0" : : "v"(ha), "v"(b), "n"(R), "n"(R + 15));
    else
        asm volatile("s_nop 1\n\tv_mfma_f32_32x32x16_f16 a[%2:%3], %0, %1, a[%2:%3]" : : "v"(ha), "v"(b), "n"(R), "n"(R + 15));
}

__device__ __forceinline__ float wide_comp(const float4 &v, int i) { return i == 0 ? v.x : i == 1 ? v.y : i == 2 ? v.z : v.w; }

// One layer's GEMM + epilogue + the H_32 factor of the transform, tiles one after the other,
// as a software pipeline over steps g (every step is its own template instance, so all
// register indices are compile-time constants):
//   step g                MFMA (tile g / KB, k block g % KB); its A fragment was fetched from
//                         LDS PF steps earlier; when that prefetch crosses into the next
//                         chunk of CH tiles the chunk is entered first
//   hidden layers (KB = 16, one accumulator per step): value e = g - KB is converted, value
//                         e - 1 gets its multiply-add with the bias, value e - 2 its sine --
//                         the three dependent instructions of one value sit in three
//                         different steps; so do the three steps of splitting a finished
//                         pair of activations into binary16 pieces, and the four H_32
//                         products of a tile issue one per step once their pieces exist: two
//                         after the tile's 8th value, two after its 16th
//   input layer (KB = 1): step g issues the four H_32 products of tile g - 1, then drains all
//                         16 accumulators of tile g and splits them
// Biases are read from LDS a few steps before use; those of tile T sit in the bias block
// of the chunk that is resident while T is drained (see the host-side packing).
// ACTK: the activation after the layer (sine, or the wavelet with envelope constant c2).
template <int NT, int KB, int NCD, int ACTK>
struct wide_gemm_ctx {
    static constexpr int PF = (NT * KB >= 4) ? 4 : (NT * KB >= 2 ? 2 : 1);
    wide_stream &S;
    const dhq_v4i (&cd)[NCD];                    // codes of the layer input: the B operands
    dhq_v16f (&xtop)[NT - WIDE_AGPR_TILES];      // transformed tiles that stay in vector registers
    const dhq_v4i (&hA)[2];                      // H_32 as an MFMA A operand, two k blocks
    const unsigned char *bufs[2];
    int cc;
    float c1, c2;
    int h;
    dhq_v4i fr[PF + 1];
    float4 bq[2];
    float4 bq0[4];  // input layer: the 16 biases of the tile drained next
    dhq_v16i acc[2];
    unsigned hp[2][8], lp[2][8];  // binary16 pieces of the tile being drained and of the one before
    float ex, ey;
    float ar[4];  // the last four activations
    float er[2];  // remainders of the pair being split
    __device__ __forceinline__ wide_gemm_ctx(wide_stream &S_, const dhq_v4i (&cd_)[NCD],
                                             dhq_v16f (&xtop_)[NT - WIDE_AGPR_TILES], const dhq_v4i (&hA_)[2])
        : S(S_), cd(cd_), xtop(xtop_), hA(hA_)
    {
    }
};

// input layer (one chunk, bias block [tile][g][h][e]): the biases of tile T
template <int NT, int KB, int NCD, int CHM, int ACTK>
__device__ __forceinline__ void wide_load_bias0(wide_gemm_ctx<NT, KB, NCD, ACTK> &C, int T)
{
#pragma unroll
    for (int gg = 0; gg < 4; ++gg)
        C.bq0[gg] = *reinterpret_cast<const float4 *>(C.bufs[0] + CHM * 1024 + T * 128 + gg * 32 + C.h * 16);
}

// H_32 product K of tile T from the pieces in hp / lp [T & 1].
template <int NT, int KB, int NCD, int T, int K, int ACTK>
__device__ __forceinline__ void wide_h32_step(wide_gemm_ctx<NT, KB, NCD, ACTK> &C)
{
    constexpr int blk = K >> 1;
    dhq_v4i b;
#pragma unroll
    for (int d = 0; d < 4; ++d) b[d] = (int)((K & 1) ? C.hp[T & 1][4 * blk + d] : C.lp[T & 1][4 * blk + d]);
    if constexpr (T < WIDE_AGPR_TILES) {
        wide_h32_mfma<T, K>(C.hA[blk], b);
    } else {
        dhq_v16f d;
        if constexpr (K == 0) {
#pragma unroll
            for (int v = 0; v < 16; ++v) d[v] = 0.f;
        } else {
            d = C.xtop[T - WIDE_AGPR_TILES];
        }
        C.xtop[T - WIDE_AGPR_TILES] = __builtin_amdgcn_mfma_f32_32x32x16_f16(
            __builtin_bit_cast(dhq_v8h, C.hA[blk]), __builtin_bit_cast(dhq_v8h, b), d, 0, 0, 0);
    }
}

template <int NT, int KB, int CH, int NCD, int G, int ACTK>
__device__ __forceinline__ void wide_gemm_step(wide_gemm_ctx<NT, KB, NCD, ACTK> &C)
{
    constexpr int NM = NT * KB;
    constexpr int CHM = CH * KB;  // MFMAs per chunk
    constexpr int NC = NT / CH;
    constexpr int NE = NT * 16;   // accumulators per lane and layer
    constexpr int PF = wide_gemm_ctx<NT, KB, NCD, ACTK>::PF;
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
        if constexpr (kb == 0) {
#pragma unroll
            for (int v = 0; v < 16; ++v) C.acc[ab][v] = 0;
        }
        C.acc[ab] = __builtin_amdgcn_mfma_i32_32x32x32_i8(C.fr[G % (PF + 1)], C.cd[kb], C.acc[ab], 0, 0, 0);
    }
    if constexpr (KB == 1) {
        // input layer: the previous tile's H_32 products, then this tile's drain
        if constexpr (G >= 1 && G <= NT) {
            wide_h32_step<NT, KB, NCD, G - 1, 0>(C);
            wide_h32_step<NT, KB, NCD, G - 1, 1>(C);
            wide_h32_step<NT, KB, NCD, G - 1, 2>(C);
            wide_h32_step<NT, KB, NCD, G - 1, 3>(C);
        }
        // the matrix unit's work stays ahead of the step's vector work
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (G < NT) {
            float x[16];
#pragma unroll
            for (int v = 0; v < 16; ++v) x[v] = (float)C.acc[0][v];
#pragma unroll
            for (int v = 0; v < 16; ++v) x[v] = __builtin_fmaf(x[v], C.c1, wide_comp(C.bq0[v >> 2], v & 3));
#pragma unroll
            for (int v = 0; v < 16; ++v) x[v] = dhq_activate_rev(x[v], dhq_act{ACTK, C.c2});
#pragma unroll
            for (int d = 0; d < 8; ++d) hm_split_pair(x[2 * d], x[2 * d + 1], C.hp[G & 1][d], C.lp[G & 1][d]);
        }
        if constexpr (G + 1 < NT) wide_load_bias0<NT, KB, NCD, CHM>(C, G + 1);  // for the next step
    } else {
        static_assert(KB == 1 || KB == 16, "one accumulator per step");
        constexpr int e0 = G - KB, e1 = e0 - 1, e2 = e0 - 2;
        // A lone wave pays for every instruction that needs the result of the one before it, so
        // the chain convert -> multiply-add -> sine -> pack high pieces -> two remainders -> pack low
        // pieces of a value is spread over six steps: value e2 gets its sine here, the pair finished
        // one step ago its high pieces, the pair before its remainders or its low pieces.
        // H_32 products: the pieces of block 0 (values 0..7) of tile t are complete after the step
        // with e2 = 16 t + 10, those of block 1 after e2 = 16 t + 18.
        constexpr int hq = e2 - 11;  // 16 t + {0, 1, 8, 9} -> product 0, 1, 2, 3 of tile t
        if constexpr (hq >= 0 && hq / 16 < NT) {
            constexpr int Th = hq / 16, r = hq % 16;
            if constexpr (r == 0) wide_h32_step<NT, KB, NCD, Th, 0>(C);
            if constexpr (r == 1) wide_h32_step<NT, KB, NCD, Th, 1>(C);
            if constexpr (r == 8) wide_h32_step<NT, KB, NCD, Th, 2>(C);
            if constexpr (r == 9) wide_h32_step<NT, KB, NCD, Th, 3>(C);
        }
        // the matrix unit's work stays ahead of the step's vector work
        __builtin_amdgcn_sched_barrier(0);
        if constexpr ((e2 & 1) == 0) {
            constexpr int pl = (e2 - 4) / 2, ph = (e2 - 2) / 2;  // pairs whose low / high pieces are packed now
            if constexpr (e2 >= 4 && pl < NE / 2) C.lp[(pl / 8) & 1][pl % 8] = hm_pack_half2(C.er[0], C.er[1]);
            if constexpr (e2 >= 2 && ph < NE / 2)
                C.hp[(ph / 8) & 1][ph % 8] = hm_pack_half2(C.ar[(e2 - 2) & 3], C.ar[(e2 - 1) & 3]);
        } else {
            constexpr int pm = (e2 - 3) / 2;  // pair whose remainders are taken now
            if constexpr (e2 >= 3 && pm < NE / 2)
                hm_remainders(C.ar[(e2 - 3) & 3], C.ar[(e2 - 2) & 3], C.hp[(pm / 8) & 1][pm % 8], C.er[0], C.er[1]);
        }
        if constexpr (e2 >= 0 && e2 < NE) C.ar[e2 & 3] = dhq_activate_rev(C.ey, dhq_act{ACTK, C.c2});
        if constexpr (e1 >= 0 && e1 < NE) C.ey = __builtin_fmaf(C.ex, C.c1, wide_comp(C.bq[(e1 / 4) & 1], e1 % 4));
        if constexpr (e0 >= 0 && e0 < NE) C.ex = (float)C.acc[(e0 / 16) & 1][e0 % 16];
        if constexpr (e0 + 4 >= 0 && (e0 + 4) % 4 == 0 && e0 + 4 < NE) {
            // biases of values e0+4 .. e0+7: tile Tg, rows group gg; chunk cT is resident while Tg is drained
            constexpr int ge = (e0 + 4) / 4, Tg = ge / 4, gg = ge % 4;
            constexpr int cT = ((Tg + 1) / CH < NC - 1) ? (Tg + 1) / CH : NC - 1;
            constexpr int tg = Tg - (cT * CH - 1);
            C.bq[ge & 1] =
                *reinterpret_cast<const float4 *>(C.bufs[cT & 1] + CHM * 1024 + tg * 128 + gg * 32 + C.h * 16);
        }
    }
    __builtin_amdgcn_sched_barrier(0);
}

template <int NT, int KB, int CH, int NCD, int ACTK, int... Gs>
__device__ __forceinline__ void wide_gemm_steps(wide_gemm_ctx<NT, KB, NCD, ACTK> &C, std::integer_sequence<int, Gs...>)
{
    (wide_gemm_step<NT, KB, CH, NCD, Gs>(C), ...);
}
template <int KB, int CHM, int PF, int NC, int... Ps>
__device__ __forceinline__ void wide_copy_prologue(const wide_stream &S, std::integer_sequence<int, Ps...>)
{
    (wide_copy_step<KB, CHM, PF, NC, Ps - PF>(S), ...);  // steps -PF .. -1
}

// cc is the running chunk count on entry and is advanced by the chunks consumed.
template <int NT, int KB, int CH, int NCD, int ACTK>
__device__ __forceinline__ void wide_gemm_sine(wide_stream &S, int &cc, float c1, float c2, const dhq_v4i (&cd)[NCD],
                                               dhq_v16f (&xtop)[NT - WIDE_AGPR_TILES], const dhq_v4i (&hA)[2], int h)
{
    constexpr int NM = NT * KB;
    constexpr int PF = wide_gemm_ctx<NT, KB, NCD, ACTK>::PF;
    // last step with work: the fourth H_32 product of the last tile (e2 - 11 = 16 (NT - 1) + 9)
    constexpr int NSTEPS = (KB == 1) ? NT + 1 : 16 * (NT - 1) + 9 + 11 + 2 + KB + 1;
    static_assert(CH * KB >= PF, "a chunk must be longer than the prefetch distance");
    wide_gemm_ctx<NT, KB, NCD, ACTK> C(S, cd, xtop, hA);
    C.cc = cc;
    C.c1 = c1;
    C.c2 = c2;
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
    wide_gemm_steps<NT, KB, CH, NCD, ACTK>(C, std::make_integer_sequence<int, NSTEPS>{});
    cc += NT / CH;
}

// The stages of the transform over the tile index and the quantizer, on rows 4 Q .. 4 Q + 3 of
// every tile (64 values, index 4 T + b): fetched from the accumulation registers (tiles 14 and 15
// from their vector registers), NT / 2 x log2(NT) butterflies per row, and per tile the four codes
// of these rows: dword Q of k block T of the next layer's B operand.
template <int NT, int Q, int... Ts>
__device__ __forceinline__ void wide_fetch_rows(float (&xv)[NT * 4], std::integer_sequence<int, Ts...>)
{
    ((xv[4 * Ts + 0] = wide_tile_read<Ts, 4 * Q + 0>(), xv[4 * Ts + 1] = wide_tile_read<Ts, 4 * Q + 1>(),
      xv[4 * Ts + 2] = wide_tile_read<Ts, 4 * Q + 2>(), xv[4 * Ts + 3] = wide_tile_read<Ts, 4 * Q + 3>()),
     ...);
}
// xrow (test hook only): where this lane's coordinate keeps its row of x^; feature 32 T + 8 Q + 4 h + b.
template <int NT, int NCD, int Q, bool DUMP = false>
__device__ __forceinline__ void wide_transform_quant(const dhq_v16f (&xtop)[NT - WIDE_AGPR_TILES], dhq_v4i (&cd)[NCD],
                                                     float inv, int qlo, int qhi, float *xrow = nullptr, int h = 0)
{
    float xv[NT * 4];
    wide_fetch_rows<NT, Q>(xv, std::make_integer_sequence<int, WIDE_AGPR_TILES>{});
#pragma unroll
    for (int T = WIDE_AGPR_TILES; T < NT; ++T)
#pragma unroll
        for (int b = 0; b < 4; ++b) xv[4 * T + b] = xtop[T - WIDE_AGPR_TILES][4 * Q + b];
#pragma unroll
    for (int s = 4; s < NT * 4; s <<= 1) {
#pragma unroll
        for (int i = 0; i < NT * 4; ++i) {
            if ((i & s) == 0) {
                const float a = xv[i], b = xv[i | s];
                xv[i] = a + b;
                xv[i | s] = a - b;
            }
        }
    }
    if constexpr (DUMP) {
#pragma unroll
        for (int T = 0; T < NT; ++T)
            *reinterpret_cast<float4 *>(xrow + 32 * T + 8 * Q + 4 * h) = make_float4(xv[4 * T], xv[4 * T + 1], xv[4 * T + 2], xv[4 * T + 3]);
    }
#pragma unroll
    for (int T = 0; T < NT; ++T) {
        cd[T][Q] = (int)fused_quant4(xv[4 * T], xv[4 * T + 1], xv[4 * T + 2], xv[4 * T + 3], inv, qlo, qhi);
    }
}

template <int NF, int ACTK>
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
    static_assert(16 * WIDE_AGPR_TILES <= WIDE_AGPR_STAGE && WIDE_AGPR_STAGE + 4 * WIDE_STAGE <= 256 && WIDE_AGPR_TILES < NT,
                  "register map");

    // A operand of the H_32 products: this lane supplies row c of H_32 at the eight contraction
    // slots 8 h + j of block kk, which stand for tile row 8 (v / 4) + 4 h + v % 4 with v = 8 kk + j
    // (the row lane half h holds in accumulator v), as binary16 +-1.
    dhq_v4i hA[2];
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) {
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            const int v = 8 * kk + 2 * d;
            const int row = 8 * (v >> 2) + 4 * h + (v & 3);
            hA[kk][d] = (int)hm_h32_pair(c, row, row + 1);
        }
    }
    dhq_v4i cd[NKB];  // activation codes: the B operands of the next GEMM
#pragma unroll
    for (int kb = 0; kb < NKB; ++kb) cd[kb] = dhq_v4i{0, 0, 0, 0};

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
            cd[0][0] = (int)dhq_pack4(dhq_quant_bits(v[0], inv, A.qmax), dhq_quant_bits(v[1], inv, A.qmax),
                                      dhq_quant_bits(v[2], inv, A.qmax), dhq_quant_bits(v[3], inv, A.qmax));
        }

        dhq_v16f xtop[NT - WIDE_AGPR_TILES];
        wide_gemm_sine<NT, 1, NT, NKB, ACTK>(S, cc, A.c1[0], A.c2, cd, xtop, hA, h);
        for (int l = 1;; ++l) {
            // finish the transform of the output of layer l-1 and quantize it: the input of layer l
            const float inv = A.inv_in[l];
            wide_transform_quant<NT, NKB, 0>(xtop, cd, inv, qlo, qhi);
            wide_transform_quant<NT, NKB, 1>(xtop, cd, inv, qlo, qhi);
            wide_transform_quant<NT, NKB, 2>(xtop, cd, inv, qlo, qhi);
            wide_transform_quant<NT, NKB, 3>(xtop, cd, inv, qlo, qhi);
            if (l == L - 1) break;
            wide_gemm_sine<NT, NKB, WIDE_CH, NKB, ACTK>(S, cc, A.c1[l], A.c2, cd, xtop, hA, h);
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
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[v] = 0;
#pragma unroll
            for (int kb = 0; kb < NKB; ++kb)
                acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(wA[kb * 64 + lane], cd[kb], acc, 0, 0, 0);
            float bias[16];
#pragma unroll
            for (int v = 0; v < 16; ++v) bias[v] = wB[((v >> 2) * 2 + h) * 4 + (v & 3)];
            wide_copy_store<0, false, 4>(S); wide_copy_store<1, false, 3>(S); wide_copy_store<2, false, 2>(S);
            wide_copy_store<3, false, 1>(S); wide_copy_store<4, false, 0>(S);
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

// ---- test hook: one layer of the kernel above on caller-supplied codes ------------------------
// Runs wide_gemm_sine and wide_transform_quant, the code of dhq_fused_wide_kernel, on the same
// packed weights and through the same chunk stream (started at the layer's first chunk); the
// codes come in from a row-major n x Kp array (rotated-feature order), and the un-normalised
// transform x^ of the layer's output, the next layer's codes and the integer accumulators (from
// a second, plain MFMA loop that reads the fragments from device memory) go out to row-major
// n x NF arrays.  One coordinate tile per workgroup.
struct wide_dargs {
    wide_args w;
    const int8_t *codes_in;
    float *xhat;        // rows rounded up to whole tiles
    int8_t *codes_out;  // the same
    int32_t *acc;       // n rows (wide_debug_acc_kernel)
    int layer, kp_in;
};

// The integer accumulators of the layer for the test hook: a plain MFMA loop over the layer's packed
// fragments, read from device memory, and the codes gathered as below.  One wave per 32 coordinates.
template <int NF>
__global__ __launch_bounds__(64) void wide_debug_acc_kernel(const wide_dargs D)
{
    constexpr int NT = NF / 32, NKB = NF / 32;
    const wide_args &A = D.w;
    const int lane = threadIdx.x & 63;
    const int c = lane & 31, h = lane >> 5;
    const int l = D.layer;
    const int cc0 = (l == 0) ? 0 : 1 + (NT / WIDE_CH) * (l - 1);
    const int KB = (l == 0) ? 1 : NKB, ch = (l == 0) ? NT : WIDE_CH;
    const int64_t ci = (int64_t)blockIdx.x * 32 + c;
    const bool valid = ci < A.n;
    const int64_t cl = valid ? ci : A.n - 1;
    for (int T = 0; T < NT; ++T) {
        const dhq_v4i *fr = reinterpret_cast<const dhq_v4i *>(A.blob + A.chunk_off[cc0 + T / ch]) + (size_t)(T % ch) * KB * 64;
        dhq_v16i acc;
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[v] = 0;
        for (int kb = 0; kb < KB; ++kb) {
            dhq_v4i b = dhq_v4i{0, 0, 0, 0};
            if (l == 0) {
                unsigned w = 0;
                for (int k = 0; k < D.kp_in; ++k) w |= (unsigned)(uint8_t)D.codes_in[cl * D.kp_in + k] << (8 * k);
                b[0] = (int)w;
            } else {
#pragma unroll
                for (int j = 0; j < 16; ++j) {
                    const int s = 16 * kb + j;
                    const int f = 32 * (s >> 4) + 8 * ((s >> 2) & 3) + 4 * h + (s & 3);  // rotated feature of register s
                    b[j >> 2] |= (int)((unsigned)(uint8_t)D.codes_in[cl * D.kp_in + f] << (8 * (j & 3)));
                }
            }
            acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(fr[kb * 64 + lane], b, acc, 0, 0, 0);
        }
        if (valid) {
#pragma unroll
            for (int v = 0; v < 16; ++v) D.acc[ci * NF + 32 * T + 8 * (v >> 2) + 4 * h + (v & 3)] = acc[v];
        }
    }
}

template <int NF, int ACTK>
__global__ __launch_bounds__(WIDE_THREADS) __attribute__((amdgpu_num_vgpr(256 + WIDE_AGPR_COMPILER)))
void dhq_fused_wide_kernel_debug(const wide_dargs D)
{
    constexpr int NT = NF / 32;
    constexpr int NKB = NF / 32;
    constexpr int BLK = (WIDE_CH * NKB + 1) * 1024;
    const wide_args &A = D.w;
    extern __shared__ __align__(16) unsigned char lds[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = lane & 31, h = lane >> 5;
    const int l = D.layer;
    const int qlo = DHQ_MAGIC_I - A.qmax, qhi = DHQ_MAGIC_I + A.qmax;
    const int cc0 = (l == 0) ? 0 : 1 + (NT / WIDE_CH) * (l - 1);  // the layer's first chunk

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
    int cc = cc0;
    for (int q = wave; q < (int)A.chunk_kib[cc0]; q += WIDE_WAVES)
        reinterpret_cast<dhq_v4i *>(lds + (cc0 & 1) * BLK)[q * 64 + lane] =
            reinterpret_cast<const dhq_v4i *>(A.blob + A.chunk_off[cc0])[q * 64 + lane];
    asm volatile("" ::: "a255");

    dhq_v4i hA[2];
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) {
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            const int v = 8 * kk + 2 * d;
            const int row = 8 * (v >> 2) + 4 * h + (v & 3);
            hA[kk][d] = (int)hm_h32_pair(c, row, row + 1);
        }
    }
    const int64_t ci = (int64_t)blockIdx.x * WIDE_TILE + wave * 32 + c;
    const bool valid = ci < A.n;
    const int64_t cl = valid ? ci : A.n - 1;
    dhq_v4i cd[NKB];
#pragma unroll
    for (int kb = 0; kb < NKB; ++kb) cd[kb] = dhq_v4i{0, 0, 0, 0};
    if (l == 0) {
        unsigned w = 0;
        for (int k = 0; k < D.kp_in; ++k) w |= (unsigned)(uint8_t)D.codes_in[cl * D.kp_in + k] << (8 * k);
        cd[0][0] = (int)w;
    } else {
        // four consecutive rotated features per dword (4-byte aligned: Kp is a multiple of 32); the
        // scheduling barrier keeps the compiler from gathering all 64 loads first, which this
        // kernel has no registers for
#pragma unroll
        for (int w = 0; w < NF / 8; ++w) {
            const int f = 32 * (w >> 2) + 8 * (w & 3) + 4 * h;  // rotated features f .. f + 3 of registers 4 w .. 4 w + 3
            cd[w >> 2][w & 3] = *reinterpret_cast<const int *>(D.codes_in + cl * D.kp_in + f);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    dhq_v16f xtop[NT - WIDE_AGPR_TILES];
    if (l == 0)
        wide_gemm_sine<NT, 1, NT, NKB, ACTK>(S, cc, A.c1[0], A.c2, cd, xtop, hA, h);
    else
        wide_gemm_sine<NT, NKB, WIDE_CH, NKB, ACTK>(S, cc, A.c1[l], A.c2, cd, xtop, hA, h);
    const float inv = A.inv_in[l + 1];
    // The coordinate index is worked out again from the thread index (through an empty asm, so that
    // the compiler cannot tell it is the value from above): kept alive across the layer it would be
    // parked in an accumulation register, which this kernel addresses by number.
    unsigned tid = threadIdx.x;
    asm volatile("" : "+v"(tid));
    const int64_t ci2 = (int64_t)blockIdx.x * WIDE_TILE + (tid >> 6) * 32 + (tid & 31);
    const bool valid2 = ci2 < A.n;
    (void)valid2;
    // both outputs go to workspace buffers with room for whole tiles, so nothing here is conditional
    float *xrow = D.xhat + ci2 * NF;
    wide_transform_quant<NT, NKB, 0, true>(xtop, cd, inv, qlo, qhi, xrow, h);
    wide_transform_quant<NT, NKB, 1, true>(xtop, cd, inv, qlo, qhi, xrow, h);
    wide_transform_quant<NT, NKB, 2, true>(xtop, cd, inv, qlo, qhi, xrow, h);
    wide_transform_quant<NT, NKB, 3, true>(xtop, cd, inv, qlo, qhi, xrow, h);
#pragma unroll
    for (int w = 0; w < NF / 8; ++w) {
        const int f = 32 * (w >> 2) + 8 * (w & 3) + 4 * h;
        *reinterpret_cast<int *>(D.codes_out + ci2 * NF + f) = cd[w >> 2][w & 3];
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
    // per layer and tile: byte offsets of the tile's 32 biases in the blob.  A hidden layer's
    // chunk also carries the biases of the tile before its first one (that tile's
    // accumulators are drained while this chunk is resident), hence up to two places.
    std::vector<uint32_t> bias_off((size_t)L * NT, 0), bias_off_dup((size_t)L * NT, 0);

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
                bias_off[(size_t)l * NT + T] = (uint32_t)(off + frag_bytes + (size_t)(hidden ? tl + 1 : tl) * 128);
                if (hidden && tl == 0 && T > 0) bias_off_dup[(size_t)l * NT + T - 1] = (uint32_t)(off + frag_bytes);
                for (int kb = 0; kb < Kb; ++kb)
                    for (int ln = 0; ln < 64; ++ln) {
                        const int row = 32 * T + (ln & 31), u = ln >> 5;
                        for (int jj = 0; jj < 16; ++jj) {
                            int8_t val = 0;
                            if (row < Ly.M) {
                                if (l == 0) {
                                    if (u == 0 && jj < Ly.Kp) val = wq[(size_t)row * Ly.Kp + jj];
                                } else {
                                    val = wq[(size_t)row * Ly.Kp + hm_index(16 * kb + jj, u)];
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
    // the biases (they do not depend on the activation scales): [g][h][e] within a tile, in
    // revolutions for the layers that end in an activation
    for (int l = 0; l < L; ++l) {
        const dhq_layer &Ly = m->layer[l];
        const bool last = (l == L - 1);
        const std::vector<float> &src = last ? Ly.bias_host : Ly.bias_rev_host;
        const int Mt = last ? 1 : NT;
        for (int T = 0; T < Mt; ++T) {
            float blk[32] = {0};
            for (int i = 0; i < 32; ++i) {
                const int f = 32 * T + i;
                if (f < Ly.M) blk[bias_slot(i)] = src[f];
            }
            memcpy(blob.data() + bias_off[(size_t)l * NT + T], blk, sizeof(blk));
            const uint32_t dup = bias_off_dup[(size_t)l * NT + T];
            if (dup) memcpy(blob.data() + dup, blk, sizeof(blk));
        }
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
    P->args.c2 = dhq_hidden_act(m).c2;
    P->act_kind = m->act_kind;
    P->lds_bytes = (size_t)2 * (WIDE_CH * NKB + 1) * 1024;
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
    for (int l = 0; l < L; ++l) {
        const dhq_layer &Ly = m->layer[l];
        P->args.c1[l] = dhq_c1(m, l);
        P->args.inv_in[l] = (float)(1.0 / ((double)Ly.s_a * sqrt((double)Ly.Kp)));
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
    auto kern = (P->act_kind == DHQ_ACT_KIND_WAVELET) ? dhq_fused_wide_kernel<512, DHQ_ACT_KIND_WAVELET>
                                                      : dhq_fused_wide_kernel<512, DHQ_ACT_KIND_SINE>;
    hipError_t e = dhq_lds_limit_once(kern, P->lds_bytes, P->device);
    if (e != hipSuccess) return e;
    kern<<<grid, WIDE_THREADS, P->lds_bytes, st>>>(a);
    return hipGetLastError();
}

// Test hook behind dhq_forward_debug_fused for hidden width 512.
hipError_t dhq_wide_debug_launch(const dhq_model *m, int layer, const int8_t *codes_in, int64_t n, float *xhat, int8_t *codes_out,
                                 int32_t *acc, hipStream_t st)
{
    const dhq_wide_plan *P = m->wide;
    if (!P || layer < 0 || layer >= m->n_layers - 1) return hipErrorInvalidValue;
    if (n <= 0) return hipSuccess;
    if (n > DHQ_CHUNK) return hipErrorInvalidValue;  // the outputs pass through the model's workspace (whole tiles)
    wide_dargs d;
    memset(&d, 0, sizeof(d));
    d.w = P->args;
    d.w.n = n;
    d.codes_in = codes_in;
    d.xhat = m->act0;
    d.codes_out = m->codes;
    d.acc = acc;
    d.layer = layer;
    d.kp_in = m->layer[layer].Kp;
    const unsigned grid = (unsigned)((n + WIDE_TILE - 1) / WIDE_TILE);
    auto kern = (P->act_kind == DHQ_ACT_KIND_WAVELET) ? dhq_fused_wide_kernel_debug<512, DHQ_ACT_KIND_WAVELET>
                                                      : dhq_fused_wide_kernel_debug<512, DHQ_ACT_KIND_SINE>;
    hipError_t e = dhq_lds_limit_once(kern, P->lds_bytes, P->device);
    if (e != hipSuccess) return e;
    if (acc) {
        wide_debug_acc_kernel<512><<<(unsigned)((n + 31) / 32), 64, 0, st>>>(d);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    if (!xhat && !codes_out) return hipSuccess;
    kern<<<grid, WIDE_THREADS, P->lds_bytes, st>>>(d);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    if (xhat && (e = hipMemcpyAsync(xhat, m->act0, sizeof(float) * (size_t)n * 512, hipMemcpyDeviceToDevice, st)) != hipSuccess) return e;
    if (codes_out && (e = hipMemcpyAsync(codes_out, m->codes, (size_t)n * 512, hipMemcpyDeviceToDevice, st)) != hipSuccess) return e;
    return hipSuccess;
}
