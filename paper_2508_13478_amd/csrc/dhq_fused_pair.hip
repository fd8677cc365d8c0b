// Whole-network fused DHQ forward for hidden width 512, two waves per SIMD (gfx950).
//
// Same arithmetic, same data layout inside a wave and the same packed weight fragments as
// dhq_fused_wide.hip (features are the MFMA M dimension, a lane holds half of one coordinate's
// feature vector, the 32-point factor of the Walsh-Hadamard transform of Eq. 3 runs on the matrix
// unit over binary16 pieces, the factor over the tile index as register butterflies).  What
// differs is who holds what.  A 512-wide layer gives a lane 256 activations, which leaves room
// for one wave per SIMD only; such a lone wave pays the latency of every dependent instruction
// and cannot overlap its own matrix and vector instruction issue.  Here two waves share 32
// coordinates and split the output features of every layer:
//
//   wave role 0 computes M tiles 0..7, role 1 tiles 8..15 (half of the GEMM, of the epilogue, of
//   the split into binary16 pieces and of the H_32 products each); both hold all 512 input codes;
//
//   the transform over the tile index needs tile T and tile T + 8 together.  Its stages never mix
//   the rows of a tile, so the work is re-split by rows: of every pair (T, T + 8) role 0 finishes
//   rows 0..7 and role 1 rows 8..15.  Each wave therefore hands half of its H_32 results (8 of
//   the 16 values per tile and lane) to its partner through LDS and receives as many, then runs
//   all four stages on 16 tiles x 8 rows and quantizes them;
//
//   the two code dwords per k block that a wave produces and the two its partner produces are
//   joined in LDS, from where both read the whole B operand of the next layer.
//
// So that both roles run the same instructions on the same register numbers, role 1 takes the
// rows of H_32 in the order "16..31, 0..15" as the A operand of its H_32 products: the rows it
// keeps then sit in registers 0..7 of a tile like role 0's, and it sends registers 8..15 like
// role 0.  Its difference "own - partner" is minus the true one (it owns T + 8), which a negated
// quantizer multiplier for that half undoes.  Everything that tells the roles apart is a
// wave-uniform run-time value: an LDS or fragment offset, the H_32 operand, one sign.
//
// LDS: two 32 KiB weight buffers (a 512 x 512 layer is streamed in eight chunks, one M tile per
// role each, copied straight from device memory into LDS by all eight waves while the previous
// chunk is consumed), a 64 KiB exchange area and three 2 KiB bias blocks (the input layer's, and
// those of the hidden / output layers by layer parity, each copied in while the layer before runs).
#include <math.h>
#include <string.h>

#include <new>
#include <utility>
#include <vector>

#include "dhq_device.h"
#include "dhq_fused_common.h"
#include "dhq_internal.h"

#define PAIR_WAVES 8
#define PAIR_THREADS (PAIR_WAVES * 64)
#define PAIR_TILE 128          // coordinates per workgroup pass: four groups of 32
#define PAIR_NT 8              // M tiles per wave
#define PAIR_KB 16             // k blocks of a hidden layer
#define PAIR_BUF 32768         // bytes per weight buffer = bytes per chunk
#define PAIR_X 65536           // exchange area
#define PAIR_BIAS (2 * PAIR_BUF + PAIR_X)  // LDS offset of the bias blocks, 2 KiB each: [layer parity 0, 1, input layer]
#define PAIR_PF 2              // LDS prefetch distance of the A fragments, in MFMAs
#define PAIR_EARLY 4           // tiles whose outgoing rows leave during the GEMM phase

struct pair_args {
    const float *coords;
    float *out;
    const unsigned char *blob;
    int64_t n;
    int n_layers;
    int k0, k0p;
    int m_out;
    int qmax;
    int n_chunks;              // weight chunks a coordinate pass goes through, in a cycle: 2 + 8 (n_layers - 2) (the whole network)
    int chunk_base;            // first of them: 0 (the whole network), or a single layer's first chunk
    uint32_t bias_off;         // byte offset of the bias table in the blob: [layer][512] floats, bias_slot order per tile
    float c2;                  // wavelet activation: 2 pi s0 sqrt(log2 e) / omega0
    float c1[DHQ_MAX_LAYERS];
    float inv_in[DHQ_MAX_LAYERS];
};

struct dhq_pair_plan {
    int act_kind = DHQ_ACT_KIND_SINE;
    unsigned char *blob_dev = nullptr;
    size_t blob_bytes = 0;
    pair_args args;
    size_t lds_bytes = 0;
    int n_cu = 0;
    int device = 0;
};

// ----------------------------------------------------------------------------- device code
struct pair_stream {
    const pair_args *A;
    unsigned char *lds;        // buffer 0, buffer 1, exchange area
    int wave, lane, role, grp;
    const unsigned char *cp_src;  // chunk being copied in: this wave's first block (uniform)
    unsigned cp_dst;              // LDS address of that block in the buffer it goes to (uniform)
    unsigned voff;                // lane * 16
};

__device__ __forceinline__ unsigned pair_lds_addr(const unsigned char *p)
{
    return (unsigned)(size_t)(__attribute__((address_space(3))) const unsigned char *)p;
}

// One KiB from device memory straight into LDS: lane i's 16 bytes go to LDS address dst + 16 i
// (dst travels in M0).  Inline assembly for the reason given at fused_issue_copy: the kernel orders
// these copies itself -- a destination is never read between the load and the "s_waitcnt vmcnt(0)" +
// barrier that precedes its first use -- and loads the compiler does not know about can only make its
// own vmcnt waits longer, never shorter.
__device__ __forceinline__ void pair_copy_kib(const pair_stream &S, const unsigned char *src, unsigned dst)
{
    // the source is wave-uniform; its halves go through readfirstlane so that the operand is a scalar register pair
    // whatever the compiler knows about it
    const unsigned long long a = (unsigned long long)src;
    const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)a), hi = __builtin_amdgcn_readfirstlane((unsigned)(a >> 32));
    const unsigned long long sa = ((unsigned long long)hi << 32) | lo;
    const unsigned m0v = __builtin_amdgcn_readfirstlane(dst);
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" : : "v"(S.voff), "s"(sa), "s"(m0v) : "memory", "m0");
}

// LDS block of layer l's biases.
__device__ __forceinline__ int pair_bias_slot(int l) { return l == 0 ? 2 : (l & 1); }
// Layer l's biases (2 KiB) into their block: waves 0 and 1 move one KiB each.
__device__ __forceinline__ void pair_copy_bias(const pair_stream &S, int l)
{
    if (S.wave < 2)
        pair_copy_kib(S, S.A->blob + S.A->bias_off + (size_t)l * 2048 + S.wave * 1024,
                      pair_lds_addr(S.lds) + PAIR_BIAS + pair_bias_slot(l) * 2048 + S.wave * 1024);
}

// Entering chunk `cc` (a running count; chunk cc lives in buffer cc & 1): every wave has written
// its share of it (the wait, then the barrier) and nobody reads chunk cc - 1 any more, so chunk
// cc + 1 may overwrite that one.
__device__ __forceinline__ void pair_enter_chunk(pair_stream &S, int cc)
{
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
    __syncthreads();
    const int j = S.A->chunk_base + (cc + 1) % S.A->n_chunks;
    S.cp_src = S.A->blob + (size_t)j * PAIR_BUF + S.wave * 1024;
    S.cp_dst = pair_lds_addr(S.lds) + ((cc + 1) & 1) * PAIR_BUF + S.wave * 1024;
}

// Slot i of a chunk's copy moves the 1 KiB block wave + 8 i (i = 0..3: 32 blocks, eight waves).
template <int I>
__device__ __forceinline__ void pair_copy_slot(const pair_stream &S)
{
    pair_copy_kib(S, S.cp_src + I * 8192, S.cp_dst + I * 8192);
}

// Where wave w parks the outgoing half of tile t (slot t & 3), as two float4 per lane.
__device__ __forceinline__ float4 *pair_x_slot(const pair_stream &S, int w, int t)
{
    return reinterpret_cast<float4 *>(S.lds + 2 * PAIR_BUF + w * 8192 + (t & 3) * 2048) + S.lane;
}

template <int ACTK>
struct pair_ctx {
    pair_stream &S;
    dhq_v4i (&cd)[PAIR_KB];       // codes of the layer input: the B operands
    dhq_v16f (&y)[PAIR_NT];       // H_32 products of this wave's tiles
    const dhq_v4i (&hA)[2];       // H_32 (rows in this role's order) as an MFMA A operand, two k blocks
    const unsigned char *bufs[2];
    const float4 *bias;           // this layer's biases in LDS, this wave's first tile, lane half folded in
    int cc, layer;
    float c1, c2;
    dhq_v4i fr[PAIR_PF + 1];
    float4 bq[3];
    float4 bq0[4];
    dhq_v16i acc[2];
    unsigned hp[2][8], lp[2][8];  // binary16 pieces of the tile being drained and of the one before
    float ex, ey, et;             // et: the complex wavelet's real-part argument, waiting for the imaginary one
    float ar[4];
    float er[2];
    __device__ __forceinline__ pair_ctx(pair_stream &S_, dhq_v4i (&cd_)[PAIR_KB], dhq_v16f (&y_)[PAIR_NT], const dhq_v4i (&hA_)[2])
        : S(S_), cd(cd_), y(y_), hA(hA_)
    {
    }
};

__device__ __forceinline__ float pair_comp(const float4 &v, int i) { return i == 0 ? v.x : i == 1 ? v.y : i == 2 ? v.z : v.w; }

// H_32 product K (0: low pieces of block 0, 1: high pieces of block 0, 2, 3: block 1) of tile T.
template <int T, int K, int ACTK>
__device__ __forceinline__ void pair_h32(pair_ctx<ACTK> &C)
{
    constexpr int blk = K >> 1;
    dhq_v4i b;
#pragma unroll
    for (int d = 0; d < 4; ++d) b[d] = (int)((K & 1) ? C.hp[T & 1][4 * blk + d] : C.lp[T & 1][4 * blk + d]);
    dhq_v16f d;
    if constexpr (K == 0) {
#pragma unroll
        for (int v = 0; v < 16; ++v) d[v] = 0.f;
    } else {
        d = C.y[T];
    }
    C.y[T] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(dhq_v8h, C.hA[blk]), __builtin_bit_cast(dhq_v8h, b), d, 0, 0, 0);
}

// The outgoing half of tile T (registers 8..15) to this wave's exchange slot.
template <int T, int ACTK>
__device__ __forceinline__ void pair_send(pair_ctx<ACTK> &C)
{
    float4 *dst = pair_x_slot(C.S, C.S.wave, T);
    dst[0] = make_float4(C.y[T][8], C.y[T][9], C.y[T][10], C.y[T][11]);
    dst[64] = make_float4(C.y[T][12], C.y[T][13], C.y[T][14], C.y[T][15]);
}

// The weight copy that runs while a hidden layer's chunk is consumed, by steps since the chunk was
// entered.
template <int REL, int ACTK>
__device__ __forceinline__ void pair_copy_rel(pair_ctx<ACTK> &C)
{
    if constexpr (REL == 1) pair_copy_slot<0>(C.S);
    if constexpr (REL == 3) pair_copy_slot<1>(C.S);
    if constexpr (REL == 5) pair_copy_slot<2>(C.S);
    if constexpr (REL == 7) pair_copy_slot<3>(C.S);
}

// One step of a hidden layer's GEMM + epilogue + H_32 pipeline (every step is its own template
// instance, so all register indices are compile-time constants):
//   step G   MFMA (tile G / 16, k block G % 16); its A fragment was fetched PF steps earlier, and
//            when that prefetch crosses into the next chunk the chunk is entered first;
//            accumulator e = G - 16 is converted, e - 1 gets its multiply-add with the bias,
//            e - 2 its activation; the split of a finished pair of activations into binary16
//            pieces takes three more steps, and the four H_32 products of a tile issue one per
//            step once their pieces exist (two after the tile's 8th value, two after its 16th);
//            the outgoing halves of the first tiles leave for the exchange area once complete.
template <int G, int ACTK>
__device__ __forceinline__ void pair_step(pair_ctx<ACTK> &C)
{
    constexpr int NM = PAIR_NT * PAIR_KB, NE = PAIR_NT * 16, PF = PAIR_PF;
    if constexpr (G >= 0 && G < NM) {
        constexpr int pf = G + PF;
        if constexpr (pf < NM) {
            if constexpr (pf % PAIR_KB == 0) pair_enter_chunk(C.S, C.cc + pf / PAIR_KB);
            C.fr[pf % (PF + 1)] = reinterpret_cast<const dhq_v4i *>(C.bufs[(pf / PAIR_KB) & 1])[(pf % PAIR_KB) * 64 + C.S.lane];
        }
    }
    if constexpr (G + PF >= 0 && G + PF < NM) pair_copy_rel<(G + PF) % PAIR_KB>(C);
    if constexpr (G == 9) pair_copy_bias(C.S, C.layer + 1);  // the next layer's biases; in place long before its first step
    if constexpr (G >= 0 && G < NM) {
        constexpr int t = G / PAIR_KB, kb = G % PAIR_KB;
        if constexpr (kb == 0) {
#pragma unroll
            for (int v = 0; v < 16; ++v) C.acc[t & 1][v] = 0;
        }
        C.acc[t & 1] = __builtin_amdgcn_mfma_i32_32x32x32_i8(C.fr[G % (PF + 1)], C.cd[kb], C.acc[t & 1], 0, 0, 0);
    }
    if constexpr (G >= 0) {
        constexpr int e0 = G - PAIR_KB, e1 = e0 - 1, e2 = e0 - 2;
        constexpr int hq = e2 - 11;  // 16 t + {0, 1, 8, 9} -> product 0, 1, 2, 3 of tile t
        if constexpr (hq >= 0 && hq / 16 < PAIR_NT) {
            constexpr int Th = hq / 16, r = hq % 16;
            if constexpr (r == 0) pair_h32<Th, 0>(C);
            if constexpr (r == 1) pair_h32<Th, 1>(C);
            if constexpr (r == 8) pair_h32<Th, 2>(C);
            if constexpr (r == 9) pair_h32<Th, 3>(C);
            if constexpr (r == 12 && Th < PAIR_EARLY) pair_send<Th>(C);
        }
        __builtin_amdgcn_sched_barrier(0);
        if constexpr ((e2 & 1) == 0) {
            constexpr int pl = (e2 - 4) / 2, ph = (e2 - 2) / 2;  // pairs whose low / high pieces are packed now
            if constexpr (e2 >= 4 && pl < NE / 2) C.lp[(pl / 8) & 1][pl % 8] = hm_pack_half2(C.er[0], C.er[1]);
            if constexpr (e2 >= 2 && ph < NE / 2) C.hp[(ph / 8) & 1][ph % 8] = hm_pack_half2(C.ar[(e2 - 2) & 3], C.ar[(e2 - 1) & 3]);
        } else {
            constexpr int pm = (e2 - 3) / 2;  // pair whose remainders are taken now
            if constexpr (e2 >= 3 && pm < NE / 2)
                hm_remainders(C.ar[(e2 - 3) & 3], C.ar[(e2 - 2) & 3], C.hp[(pm / 8) & 1][pm % 8], C.er[0], C.er[1]);
        }
        if constexpr (e2 >= 0 && e2 < NE) {
            if constexpr (ACTK == DHQ_ACT_KIND_WAVELET_COMPLEX) {
                // accumulators e2 - 1, e2 (e2 odd) are the features 2m, 2m + 1 = (Re, Im) of one complex feature; both
                // results are consumed from the step after this one on (the packing of the high pieces)
                if constexpr ((e2 & 1) == 0) C.et = C.ey;
                else dhq_activate_pair_rev<false>(C.et, C.ey, C.c2, C.ar[(e2 - 1) & 3], C.ar[e2 & 3]);
            } else {
                C.ar[e2 & 3] = dhq_activate_rev(C.ey, dhq_act{ACTK, C.c2});
            }
        }
        if constexpr (e1 >= 0 && e1 < NE) C.ey = __builtin_fmaf(C.ex, C.c1, pair_comp(C.bq[(e1 / 4) % 3], e1 % 4));
        if constexpr (e0 >= 0 && e0 < NE) C.ex = (float)C.acc[(e0 / 16) & 1][e0 % 16];
        if constexpr (e0 + 8 >= 0 && (e0 + 8) % 4 == 0 && e0 + 8 < NE) {
            // biases of values e0 + 8 .. e0 + 11 (tile ge / 4, row group ge % 4), from device memory; the ring
            // slot's previous tenant, group ge - 3, had its last use in the multiply-add just above
            constexpr int ge = (e0 + 8) / 4;
            C.bq[ge % 3] = C.bias[ge * 2];
        }
    }
    __builtin_amdgcn_sched_barrier(0);
}

template <int ACTK, int... Gs>
__device__ __forceinline__ void pair_steps(pair_ctx<ACTK> &C, std::integer_sequence<int, Gs...>)
{
    (pair_step<Gs - PAIR_PF>(C), ...);  // steps -PF (the copy's first steps) .. NSTEPS - 1
}

// A hidden layer: reads the input codes the transform left in the exchange area, then the GEMM
// pipeline over this wave's eight tiles.  cc is the running chunk count and is advanced.
template <int ACTK>
__device__ __forceinline__ void pair_hidden(pair_stream &S, int &cc, int layer, float c1, dhq_v4i (&cd)[PAIR_KB],
                                            dhq_v16f (&y)[PAIR_NT], const dhq_v4i (&hA)[2], int h)
{
    // last step with work: the send after the fourth H_32 product of the last tile would be
    // e2 - 11 = 16 * 7 + 12, the product itself 16 * 7 + 9
    constexpr int NSTEPS = 16 * (PAIR_NT - 1) + 9 + 11 + 2 + PAIR_KB + 1;
    pair_ctx<ACTK> C(S, cd, y, hA);
    C.cc = cc;
    C.c1 = c1;
    C.c2 = S.A->c2;
    C.ex = C.ey = C.et = 0.f;
    C.layer = layer;
    C.bias = reinterpret_cast<const float4 *>(S.lds + PAIR_BIAS + pair_bias_slot(layer) * 2048) + S.role * 64 + h;
    pair_enter_chunk(S, cc);
    {
        const dhq_v4i *src = reinterpret_cast<const dhq_v4i *>(S.lds + 2 * PAIR_BUF + S.grp * 16384) + S.lane;
#pragma unroll
        for (int T = 0; T < PAIR_KB; ++T) cd[T] = src[T * 64];
    }
    C.bufs[0] = S.lds + (cc & 1) * PAIR_BUF + S.role * 16384;
    C.bufs[1] = S.lds + ((cc + 1) & 1) * PAIR_BUF + S.role * 16384;
#pragma unroll
    for (int m = 0; m < PAIR_PF; ++m) C.fr[m % (PAIR_PF + 1)] = reinterpret_cast<const dhq_v4i *>(C.bufs[0])[m * 64 + S.lane];
    pair_steps<ACTK>(C, std::make_integer_sequence<int, NSTEPS + PAIR_PF>{});
    cc += PAIR_NT;
}

// The input layer (fan-in <= 4: one k block, one chunk with all sixteen tiles): step G issues the
// MFMA of tile G and the four H_32 products of tile G - 1, then drains tile G.
template <int G, int ACTK>
__device__ __forceinline__ void pair_step0(pair_ctx<ACTK> &C, int h)
{
    constexpr int PF = PAIR_PF;
    if constexpr (G + PF < PAIR_NT) C.fr[(G + PF) % (PF + 1)] = reinterpret_cast<const dhq_v4i *>(C.bufs[0])[(G + PF) * 64 + C.S.lane];
    if constexpr (G == 0) pair_copy_slot<0>(C.S);
    if constexpr (G == 1) pair_copy_slot<1>(C.S);
    if constexpr (G == 2) pair_copy_slot<2>(C.S);
    if constexpr (G == 3) pair_copy_slot<3>(C.S);
    if constexpr (G == 4) pair_copy_bias(C.S, 1);
    if constexpr (G < PAIR_NT) {
#pragma unroll
        for (int v = 0; v < 16; ++v) C.acc[0][v] = 0;
        C.acc[0] = __builtin_amdgcn_mfma_i32_32x32x32_i8(C.fr[G % (PF + 1)], C.cd[0], C.acc[0], 0, 0, 0);
    }
    if constexpr (G >= 1 && G <= PAIR_NT) {
        pair_h32<G - 1, 0>(C);
        pair_h32<G - 1, 1>(C);
        pair_h32<G - 1, 2>(C);
        pair_h32<G - 1, 3>(C);
    }
    if constexpr (G >= 2 && G - 2 < PAIR_EARLY) pair_send<G - 2>(C);
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (G < PAIR_NT) {
        float x[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) x[v] = (float)C.acc[0][v];
#pragma unroll
        for (int v = 0; v < 16; ++v) x[v] = __builtin_fmaf(x[v], C.c1, pair_comp(C.bq0[v >> 2], v & 3));
        if constexpr (ACTK == DHQ_ACT_KIND_WAVELET_COMPLEX) {
#pragma unroll
            for (int d = 0; d < 8; ++d) dhq_activate_pair_rev<false>(x[2 * d], x[2 * d + 1], C.c2, x[2 * d], x[2 * d + 1]);
        } else {
#pragma unroll
            for (int v = 0; v < 16; ++v) x[v] = dhq_activate_rev(x[v], dhq_act{ACTK, C.c2});
        }
#pragma unroll
        for (int d = 0; d < 8; ++d) hm_split_pair(x[2 * d], x[2 * d + 1], C.hp[G & 1][d], C.lp[G & 1][d]);
    }
    if constexpr (G + 1 < PAIR_NT) {
#pragma unroll
        for (int gg = 0; gg < 4; ++gg) C.bq0[gg] = C.bias[((G + 1) * 4 + gg) * 2];
    }
    __builtin_amdgcn_sched_barrier(0);
}
template <int ACTK, int... Gs>
__device__ __forceinline__ void pair_steps0(pair_ctx<ACTK> &C, int h, std::integer_sequence<int, Gs...>)
{
    (pair_step0<Gs>(C, h), ...);
}

template <int ACTK>
__device__ __forceinline__ void pair_input_layer(pair_stream &S, int &cc, float c1, dhq_v4i (&cd)[PAIR_KB], dhq_v16f (&y)[PAIR_NT],
                                                 const dhq_v4i (&hA)[2], int h)
{
    pair_ctx<ACTK> C(S, cd, y, hA);
    C.cc = cc;
    C.c1 = c1;
    C.c2 = S.A->c2;
    C.layer = 0;
    C.bias = reinterpret_cast<const float4 *>(S.lds + PAIR_BIAS + pair_bias_slot(0) * 2048) + S.role * 64 + h;
    pair_enter_chunk(S, cc);
    C.bufs[0] = S.lds + (cc & 1) * PAIR_BUF + S.role * 8192;  // fragments [tile 0..15], 1 KiB each
    C.bufs[1] = C.bufs[0];
#pragma unroll
    for (int m = 0; m < PAIR_PF; ++m) C.fr[m % (PAIR_PF + 1)] = reinterpret_cast<const dhq_v4i *>(C.bufs[0])[m * 64 + S.lane];
#pragma unroll
    for (int gg = 0; gg < 4; ++gg) C.bq0[gg] = C.bias[gg * 2];
    pair_steps0<ACTK>(C, h, std::make_integer_sequence<int, PAIR_NT + 1>{});
    cc += 1;
}

// What the partner parked for tile T, combined with the kept half of this wave's tile T:
// zl = own + partner (tile T of the stage over tile-index bit 3), zh = own - partner (tile T + 8;
// minus that for role 1, which owns T + 8).
template <int T>
__device__ __forceinline__ void pair_recv(const pair_stream &S, const dhq_v16f (&y)[PAIR_NT], float (&zl)[PAIR_NT][8],
                                          float (&zh)[PAIR_NT][8])
{
    const float4 *src = pair_x_slot(S, S.wave ^ 4, T);
    const float4 p0 = src[0], p1 = src[64];
    const float p[8] = {p0.x, p0.y, p0.z, p0.w, p1.x, p1.y, p1.z, p1.w};
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        zl[T][i] = y[T][i] + p[i];
        zh[T][i] = y[T][i] - p[i];
    }
}

__device__ __forceinline__ void pair_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __syncthreads();
}

// The rest of the transform: on return zl[T][i] / zh[T][i] hold the un-normalised x^ of rotated features
// 32 T + 8 (i / 4 + 2 role) + 4 h + i % 4 and 256 + the same (zh of role 1 with its sign flipped), and
// the exchange area is free.
template <bool AFTER_INPUT_LAYER>
__device__ __forceinline__ void pair_transform(pair_stream &S, dhq_v16f (&y)[PAIR_NT], float (&zl)[PAIR_NT][8], float (&zh)[PAIR_NT][8])
{
    // the halves sent during the GEMM phase are in place: a hidden layer's last sends precede its last chunk
    // barriers, the input layer has none
    if constexpr (AFTER_INPUT_LAYER) pair_barrier();
    pair_recv<0>(S, y, zl, zh);
    pair_recv<1>(S, y, zl, zh);
    pair_recv<2>(S, y, zl, zh);
    pair_recv<3>(S, y, zl, zh);
    pair_barrier();  // everyone has read them: the slots are free again
    {
        float4 *d4 = pair_x_slot(S, S.wave, 4), *d5 = pair_x_slot(S, S.wave, 5), *d6 = pair_x_slot(S, S.wave, 6), *d7 = pair_x_slot(S, S.wave, 7);
        d4[0] = make_float4(y[4][8], y[4][9], y[4][10], y[4][11]); d4[64] = make_float4(y[4][12], y[4][13], y[4][14], y[4][15]);
        d5[0] = make_float4(y[5][8], y[5][9], y[5][10], y[5][11]); d5[64] = make_float4(y[5][12], y[5][13], y[5][14], y[5][15]);
        d6[0] = make_float4(y[6][8], y[6][9], y[6][10], y[6][11]); d6[64] = make_float4(y[6][12], y[6][13], y[6][14], y[6][15]);
        d7[0] = make_float4(y[7][8], y[7][9], y[7][10], y[7][11]); d7[64] = make_float4(y[7][12], y[7][13], y[7][14], y[7][15]);
    }
    pair_barrier();
    pair_recv<4>(S, y, zl, zh);
    pair_recv<5>(S, y, zl, zh);
    pair_recv<6>(S, y, zl, zh);
    pair_recv<7>(S, y, zl, zh);
    pair_barrier();  // the exchange area is free for the codes
    // stages over tile-index bits 0..2, within each half
#pragma unroll
    for (int s = 1; s < PAIR_NT; s <<= 1) {
#pragma unroll
        for (int t = 0; t < PAIR_NT; ++t) {
            if ((t & s) == 0) {
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const float a = zl[t][i], b = zl[t | s][i];
                    zl[t][i] = a + b;
                    zl[t | s][i] = a - b;
                    const float c = zh[t][i], d = zh[t | s][i];
                    zh[t][i] = c + d;
                    zh[t | s][i] = c - d;
                }
            }
        }
    }
}

// The rest of the transform and the next layer's quantizer.  On return the exchange area holds,
// per coordinate group, the next layer's whole B operand ([k block][lane] x 16 B); it may be read
// after the next barrier.  xrow (test hook): where this lane's coordinate keeps its row of x^.
template <bool DUMP, bool AFTER_INPUT_LAYER = true>
__device__ __forceinline__ void pair_transform_quant(pair_stream &S, dhq_v16f (&y)[PAIR_NT], float inv, int qlo, int qhi, int h,
                                                     float *xrow = nullptr, int *crow = nullptr)
{
    float zl[PAIR_NT][8], zh[PAIR_NT][8];
    pair_transform<AFTER_INPUT_LAYER>(S, y, zl, zh);
    const float inv_hi = S.role ? -inv : inv;
    if constexpr (DUMP) {
        // rotated feature of zl[T][i]: 32 T + 8 (i / 4 + 2 role) + 4 h + i % 4; zh: tile T + 8, sign as above
        const float sg = S.role ? -1.f : 1.f;
#pragma unroll
        for (int T = 0; T < PAIR_NT; ++T) {
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                float *p = xrow + 32 * T + 8 * (q + 2 * S.role) + 4 * h;
                *reinterpret_cast<float4 *>(p) = make_float4(zl[T][4 * q], zl[T][4 * q + 1], zl[T][4 * q + 2], zl[T][4 * q + 3]);
                *reinterpret_cast<float4 *>(p + 256) =
                    make_float4(sg * zh[T][4 * q], sg * zh[T][4 * q + 1], sg * zh[T][4 * q + 2], sg * zh[T][4 * q + 3]);
            }
        }
    }
    // this wave's two dwords of every k block: bytes 8 role .. 8 role + 7 of the lane's 16
    unsigned char *dst = S.lds + 2 * PAIR_BUF + S.grp * 16384 + S.lane * 16 + S.role * 8;
#pragma unroll
    for (int T = 0; T < PAIR_NT; ++T) {
        const unsigned a0 = fused_quant4(zl[T][0], zl[T][1], zl[T][2], zl[T][3], inv, qlo, qhi);
        const unsigned a1 = fused_quant4(zl[T][4], zl[T][5], zl[T][6], zl[T][7], inv, qlo, qhi);
        const unsigned b0 = fused_quant4(zh[T][0], zh[T][1], zh[T][2], zh[T][3], inv_hi, qlo, qhi);
        const unsigned b1 = fused_quant4(zh[T][4], zh[T][5], zh[T][6], zh[T][7], inv_hi, qlo, qhi);
        *reinterpret_cast<uint2 *>(dst + T * 1024) = make_uint2(a0, a1);
        *reinterpret_cast<uint2 *>(dst + (T + 8) * 1024) = make_uint2(b0, b1);
        if constexpr (DUMP) {
            int *c = crow + 8 * T + 2 * (2 * S.role) + h;  // dwords of 4 codes: feature / 4
            c[0] = (int)a0; c[2] = (int)a1; c[64] = (int)b0; c[66] = (int)b1;
        }
    }
}

__device__ __forceinline__ void pair_h32_operand(int c, int h, int role, dhq_v4i (&hA)[2])
{
    fused_h32_operand(c ^ (role << 4), h, hA);
}

__device__ __forceinline__ void pair_stream_init(pair_stream &S, const pair_args *A, unsigned char *lds, int wave, int lane)
{
    S.A = A;
    S.lds = lds;
    S.wave = __builtin_amdgcn_readfirstlane(wave);
    S.lane = lane;
    S.role = S.wave >> 2;
    S.grp = S.wave & 3;
    S.cp_src = A->blob;
    S.cp_dst = pair_lds_addr(lds);
    S.voff = (unsigned)lane * 16;
}

// Copies chunk j into buffer `buf` right now (the first chunk of a kernel has nobody to copy it in the background).
__device__ __forceinline__ void pair_copy_now(const pair_stream &S, int j, int buf)
{
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int q = S.wave + 8 * i;
        reinterpret_cast<dhq_v4i *>(S.lds + buf * PAIR_BUF)[q * 64 + S.lane] =
            reinterpret_cast<const dhq_v4i *>(S.A->blob + (size_t)j * PAIR_BUF)[q * 64 + S.lane];
    }
}

template <int ACTK>
__global__ __launch_bounds__(PAIR_THREADS) void dhq_fused_pair_kernel(const pair_args A)
{
    extern __shared__ __align__(16) unsigned char lds[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = lane & 31, h = lane >> 5;
    const int L = A.n_layers;
    const int64_t n_tiles = (A.n + PAIR_TILE - 1) / PAIR_TILE;
    if ((int64_t)blockIdx.x >= n_tiles) return;
    const int my_tiles = (int)((n_tiles - 1 - blockIdx.x) / gridDim.x) + 1;
    const int qlo = DHQ_MAGIC_I - A.qmax, qhi = DHQ_MAGIC_I + A.qmax;

    pair_stream S;
    pair_stream_init(S, &A, lds, wave, lane);
    int cc = 0;
    pair_copy_now(S, 0, 0);
    pair_copy_bias(S, 0);

    dhq_v4i hA[2];
    pair_h32_operand(c, h, S.role, hA);

    for (int it = 0; it < my_tiles; ++it) {
        const int64_t tile = (int64_t)blockIdx.x + (int64_t)it * gridDim.x;
        // the codes of a layer's input: the input layer uses k block 0 only (and of it only k positions 0..3, the
        // rest of its fragments being zero), every hidden layer reads all sixteen from the exchange area first
        dhq_v4i cd[PAIR_KB];
#pragma unroll
        for (int kb = 0; kb < PAIR_KB; ++kb) cd[kb] = dhq_v4i{0, 0, 0, 0};
        {
            // (the lane's coordinate from the thread index afresh in every pass, like the output layer below: a
            // loop-invariant per-lane address would be carried through all layers in registers it spills)
            unsigned tid = threadIdx.x;
            asm volatile("" : "+v"(tid));
            const int64_t ci = tile * PAIR_TILE + S.grp * 32 + (tid & 31);
            const int64_t cl = ci < A.n ? ci : A.n - 1;  // lanes past the end repeat the last coordinate and store nothing
            cd[0][0] = fused_input_codes(A.coords, cl, A.k0, A.k0p, A.inv_in[0], A.qmax);
        }

        dhq_v16f y[PAIR_NT];
        pair_input_layer<ACTK>(S, cc, A.c1[0], cd, y, hA, h);
        pair_transform_quant<false, true>(S, y, A.inv_in[1], qlo, qhi, h);
        for (int l = 1; l < L - 1; ++l) {
            pair_hidden<ACTK>(S, cc, l, A.c1[l], cd, y, hA, h);
            pair_transform_quant<false, false>(S, y, A.inv_in[l + 1], qlo, qhi, h);
        }

        // output layer: one zero-padded M tile, no activation; role 0 computes it while all waves
        // copy in the next pass's first chunk
        {
            pair_enter_chunk(S, cc);
            const unsigned char *buf = lds + (cc & 1) * PAIR_BUF;
            pair_copy_slot<0>(S); pair_copy_slot<1>(S); pair_copy_slot<2>(S); pair_copy_slot<3>(S);
            pair_copy_bias(S, 0);
            if (S.role == 0) {
                // The coordinate index, the lane's place and its lane half are worked out again from the thread
                // index (through an empty asm, so that the compiler cannot tell they are the values from the
                // top of the pass): kept alive across all layers they would be spilled to scratch memory.
                unsigned tid = threadIdx.x;
                asm volatile("" : "+v"(tid));
                const int lane = tid & 63, h = (tid >> 5) & 1;
                const int64_t ci = tile * PAIR_TILE + S.grp * 32 + (tid & 31);
                const bool valid = ci < A.n;
                const dhq_v4i *src = reinterpret_cast<const dhq_v4i *>(lds + 2 * PAIR_BUF + S.grp * 16384) + lane;
                const dhq_v4i *wA = reinterpret_cast<const dhq_v4i *>(buf);
                dhq_v16i acc;
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[v] = 0;
#pragma unroll
                for (int kb = 0; kb < PAIR_KB; ++kb) acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(wA[kb * 64 + lane], src[kb * 64], acc, 0, 0, 0);
                const float *wB = reinterpret_cast<const float *>(lds + PAIR_BIAS + pair_bias_slot(L - 1) * 2048);
                const float c1 = A.c1[L - 1];
                if (valid) {
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int row = 8 * (v >> 2) + 4 * h + (v & 3);
                        if (row < A.m_out) A.out[ci * A.m_out + row] = __builtin_fmaf((float)acc[v], c1, wB[((v >> 2) * 2 + h) * 4 + (v & 3)]);
                    }
                }
            }
            cc += 1;
        }
    }
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
}

// ---- one layer per launch: the dynamic quantization module (Sec. 3.3) at this width -----------
// With scales measured on line a layer's quantizer needs max |x^| over the whole batch before it
// can emit a code, so the whole-network kernel is cut at exactly that point, as
// dhq_fused_layer_kernel cuts the narrower one: a launch folds the per-workgroup maxima its
// predecessor left into this layer's constants (every workgroup for itself), quantizes its input
// with them, runs the layer with the code of the kernel above and writes the un-normalised
// transform x^ of its output (fp32) plus the workgroup's max |x^|.  x^ crosses device memory in the
// waves' register order: [128-coordinate tile][wave][q = 4 T + {zl 0..3, zl 4..7, zh 0..3, zh 4..7}][lane]
// x 16 B, every access of a wave 1 KiB contiguous; a wave reads back exactly what the wave in its
// place wrote (zh of role 1 with its sign flipped, which the negated multiplier undoes).
//   MODE 0  input layer: coordinates in, x^ out        MODE 1  hidden layer: x^ in, x^ out
//   MODE 2  output layer: x^ in, signal values out
struct pair_largs {
    pair_args w;               // n_chunks / chunk_base: this layer's chunks; c1 and inv_in are not used
    const float4 *xin;         // MODE 1, 2
    float4 *xout;              // MODE 0, 1
    const float *partial_in;   // max |x^| of this layer's input, one float per workgroup of the launch before
    int partial_count;
    int kp;                    // length of this layer's rotated input
    int layer;
    double c1_over_sa;         // epilogue multiplier divided by the activation scale
    float *dyn;                // this layer's {1 / (s_a sqrt(Kp)), epilogue multiplier, s_a}: written by workgroup 0
    float *partial;            // MODE 0, 1: max |x^| of the output per workgroup (not the buffer partial_in points to)
};

template <int MODE, int ACTK>
__global__ __launch_bounds__(PAIR_THREADS) void dhq_fused_pair_layer_kernel(const pair_largs D)
{
    const pair_args &A = D.w;
    extern __shared__ __align__(16) unsigned char lds[];
    __shared__ float red_in[PAIR_WAVES], red[PAIR_WAVES];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = lane & 31, h = lane >> 5;
    const int64_t n_tiles = (A.n + PAIR_TILE - 1) / PAIR_TILE;  // the grid has at most that many workgroups
    const int my_tiles = (int)((n_tiles - 1 - blockIdx.x) / gridDim.x) + 1;
    const int qlo = DHQ_MAGIC_I - A.qmax, qhi = DHQ_MAGIC_I + A.qmax;

    pair_stream S;
    pair_stream_init(S, &A, lds, wave, lane);
    int cc = 0;
    pair_copy_now(S, A.chunk_base, 0);
    pair_copy_bias(S, D.layer);
    dhq_v4i hA[2];
    pair_h32_operand(c, h, S.role, hA);

    // this layer's constants from the maxima of its input
    float inv, c1, s_a;
    {
        float mi = 0.f;
        for (int i = threadIdx.x; i < D.partial_count; i += PAIR_THREADS) mi = fmaxf(mi, D.partial_in[i]);
#pragma unroll
        for (int m = 1; m < 64; m *= 2) mi = fmaxf(mi, __shfl_xor(mi, m, 64));
        if (lane == 0) red_in[wave] = mi;
        __syncthreads();
        mi = red_in[0];
#pragma unroll
        for (int w = 1; w < PAIR_WAVES; ++w) mi = fmaxf(mi, red_in[w]);
        dhq_dyn_constants(mi, D.kp, A.qmax, D.c1_over_sa, inv, c1, s_a);
        if (blockIdx.x == 0 && threadIdx.x == 0) {
            D.dyn[0] = inv; D.dyn[1] = c1; D.dyn[2] = s_a;
        }
    }
    float mx = 0.f;
    for (int it = 0; it < my_tiles; ++it) {
        const int64_t tile = (int64_t)blockIdx.x + (int64_t)it * gridDim.x;
        const size_t slot = ((size_t)tile * PAIR_WAVES + S.wave) * (4 * PAIR_NT) * 64 + lane;
        dhq_v4i cd[PAIR_KB];
#pragma unroll
        for (int kb = 0; kb < PAIR_KB; ++kb) cd[kb] = dhq_v4i{0, 0, 0, 0};
        if constexpr (MODE == 0) {
            const int64_t ci = tile * PAIR_TILE + S.grp * 32 + c;
            const int64_t cl = ci < A.n ? ci : A.n - 1;  // lanes past the end repeat the last coordinate: no effect on the maximum
            cd[0][0] = fused_input_codes(A.coords, cl, A.k0, A.k0p, inv, A.qmax);
        } else {
            // the output layer's role-0 waves may still be reading the previous tile's codes
            if constexpr (MODE == 2) pair_barrier();
            // this wave's 128 values of the layer's input: quantized, its two dwords of every k block to the exchange
            // area, where pair_transform_quant puts them in the whole-network kernel
            const float inv_hi = S.role ? -inv : inv;
            unsigned char *dst = lds + 2 * PAIR_BUF + S.grp * 16384 + lane * 16 + S.role * 8;
#pragma unroll
            for (int T = 0; T < PAIR_NT; ++T) {
                const float4 l0 = D.xin[slot + (size_t)(4 * T) * 64], l1 = D.xin[slot + (size_t)(4 * T + 1) * 64];
                const float4 h0 = D.xin[slot + (size_t)(4 * T + 2) * 64], h1 = D.xin[slot + (size_t)(4 * T + 3) * 64];
                const unsigned a0 = fused_quant4(l0.x, l0.y, l0.z, l0.w, inv, qlo, qhi);
                const unsigned a1 = fused_quant4(l1.x, l1.y, l1.z, l1.w, inv, qlo, qhi);
                const unsigned b0 = fused_quant4(h0.x, h0.y, h0.z, h0.w, inv_hi, qlo, qhi);
                const unsigned b1 = fused_quant4(h1.x, h1.y, h1.z, h1.w, inv_hi, qlo, qhi);
                *reinterpret_cast<uint2 *>(dst + T * 1024) = make_uint2(a0, a1);
                *reinterpret_cast<uint2 *>(dst + (T + 8) * 1024) = make_uint2(b0, b1);
            }
        }
        if constexpr (MODE == 2) {
            // one zero-padded M tile, no activation: role 0 computes it while all waves copy the chunk in again
            pair_enter_chunk(S, cc);
            const unsigned char *buf = lds + (cc & 1) * PAIR_BUF;
            pair_copy_slot<0>(S); pair_copy_slot<1>(S); pair_copy_slot<2>(S); pair_copy_slot<3>(S);
            if (S.role == 0) {
                const int64_t ci = tile * PAIR_TILE + S.grp * 32 + c;
                const dhq_v4i *src = reinterpret_cast<const dhq_v4i *>(lds + 2 * PAIR_BUF + S.grp * 16384) + lane;
                const dhq_v4i *wA = reinterpret_cast<const dhq_v4i *>(buf);
                dhq_v16i acc;
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[v] = 0;
#pragma unroll
                for (int kb = 0; kb < PAIR_KB; ++kb) acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(wA[kb * 64 + lane], src[kb * 64], acc, 0, 0, 0);
                const float *wB = reinterpret_cast<const float *>(lds + PAIR_BIAS + pair_bias_slot(D.layer) * 2048);
                if (ci < A.n) {
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int row = 8 * (v >> 2) + 4 * h + (v & 3);
                        if (row < A.m_out) A.out[ci * A.m_out + row] = __builtin_fmaf((float)acc[v], c1, wB[((v >> 2) * 2 + h) * 4 + (v & 3)]);
                    }
                }
            }
            cc += 1;
        } else {
            dhq_v16f y[PAIR_NT];
            float zl[PAIR_NT][8], zh[PAIR_NT][8];
            if constexpr (MODE == 0) {
                pair_input_layer<ACTK>(S, cc, c1, cd, y, hA, h);
                pair_transform<true>(S, y, zl, zh);
            } else {
                pair_hidden<ACTK>(S, cc, D.layer, c1, cd, y, hA, h);
                pair_transform<false>(S, y, zl, zh);
            }
#pragma unroll
            for (int T = 0; T < PAIR_NT; ++T) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const float(&z)[8] = (q < 2) ? zl[T] : zh[T];
                    const float4 x = make_float4(z[4 * (q & 1)], z[4 * (q & 1) + 1], z[4 * (q & 1) + 2], z[4 * (q & 1) + 3]);
                    mx = fmaxf(fmaxf(mx, fmaxf(fabsf(x.x), fabsf(x.y))), fmaxf(fabsf(x.z), fabsf(x.w)));
                    D.xout[slot + (size_t)(4 * T + q) * 64] = x;
                }
            }
        }
    }
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
    if constexpr (MODE != 2) {
#pragma unroll
        for (int m = 1; m < 64; m *= 2) mx = fmaxf(mx, __shfl_xor(mx, m, 64));
        if (lane == 0) red[wave] = mx;
        __syncthreads();
        if (threadIdx.x == 0) {
            float r = red[0];
#pragma unroll
            for (int w = 1; w < PAIR_WAVES; ++w) r = fmaxf(r, red[w]);
            D.partial[blockIdx.x] = r;
        }
    }
}

// ---- test hook: one layer of the kernel above on caller-supplied codes ------------------------
struct pair_dargs {
    pair_args w;
    const int8_t *codes_in;
    float *xhat;        // rows rounded up to whole workgroup tiles
    int8_t *codes_out;  // the same
    int32_t *acc;       // n rows
    int layer, kp_in;
};

// The integer accumulators for the test hook: a plain MFMA loop over the layer's packed fragments,
// read from device memory.  One wave per 32 coordinates.
__global__ __launch_bounds__(64) void pair_debug_acc_kernel(const pair_dargs D)
{
    const pair_args &A = D.w;
    const int lane = threadIdx.x & 63;
    const int c = lane & 31, h = lane >> 5;
    const int l = D.layer;
    const int64_t ci = (int64_t)blockIdx.x * 32 + c;
    const bool valid = ci < A.n;
    const int64_t cl = valid ? ci : A.n - 1;
    const int KB = (l == 0) ? 1 : PAIR_KB;
    for (int T = 0; T < 16; ++T) {
        // input layer: chunk 0, fragments [tile]; hidden layer l: chunk 1 + 8 (l - 1) + T % 8, fragments [role = T / 8][k block]
        const dhq_v4i *fr = (l == 0) ? reinterpret_cast<const dhq_v4i *>(A.blob) + (size_t)T * 64
                                     : reinterpret_cast<const dhq_v4i *>(A.blob + (size_t)(1 + 8 * (l - 1) + (T & 7)) * PAIR_BUF + (T >> 3) * 16384);
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
                for (int j = 0; j < 4; ++j) b[j] = *reinterpret_cast<const int *>(D.codes_in + cl * D.kp_in + 32 * kb + 8 * j + 4 * h);
            }
            acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(fr[kb * 64 + lane], b, acc, 0, 0, 0);
        }
        if (valid) {
#pragma unroll
            for (int v = 0; v < 16; ++v) D.acc[ci * 512 + 32 * T + 8 * (v >> 2) + 4 * h + (v & 3)] = acc[v];
        }
    }
}

template <int ACTK>
__global__ __launch_bounds__(PAIR_THREADS) void dhq_fused_pair_kernel_debug(const pair_dargs D)
{
    const pair_args &A = D.w;
    extern __shared__ __align__(16) unsigned char lds[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = lane & 31, h = lane >> 5;
    const int l = D.layer;
    const int qlo = DHQ_MAGIC_I - A.qmax, qhi = DHQ_MAGIC_I + A.qmax;
    const int cc0 = (l == 0) ? 0 : 1 + 8 * (l - 1);  // the layer's first chunk

    pair_stream S;
    pair_stream_init(S, &A, lds, wave, lane);
    int cc = cc0;
    pair_copy_now(S, cc0, cc0 & 1);
    pair_copy_bias(S, l);
    dhq_v4i hA[2];
    pair_h32_operand(c, h, S.role, hA);
    const int64_t ci = (int64_t)blockIdx.x * PAIR_TILE + S.grp * 32 + c;
    const int64_t cl = ci < A.n ? ci : A.n - 1;
    dhq_v4i cd[PAIR_KB];
#pragma unroll
    for (int kb = 0; kb < PAIR_KB; ++kb) cd[kb] = dhq_v4i{0, 0, 0, 0};
    dhq_v16f y[PAIR_NT];
    if (l == 0) {
        unsigned w = 0;
        for (int k = 0; k < D.kp_in; ++k) w |= (unsigned)(uint8_t)D.codes_in[cl * D.kp_in + k] << (8 * k);
        cd[0][0] = (int)w;
        pair_input_layer<ACTK>(S, cc, A.c1[0], cd, y, hA, h);
    } else {
        // the hidden layer reads its codes from the exchange area: [group][k block][lane] x 16 B,
        // dword q of k block T = rotated features 32 T + 8 q + 4 h .. + 3; role r brings in dwords 2 r, 2 r + 1
        unsigned char *dst = lds + 2 * PAIR_BUF + S.grp * 16384 + lane * 16 + S.role * 8;
#pragma unroll
        for (int T = 0; T < PAIR_KB; ++T) {
            const int f = 32 * T + 16 * S.role + 4 * h;
            const unsigned a0 = *reinterpret_cast<const unsigned *>(D.codes_in + cl * D.kp_in + f);
            const unsigned a1 = *reinterpret_cast<const unsigned *>(D.codes_in + cl * D.kp_in + f + 8);
            *reinterpret_cast<uint2 *>(dst + T * 1024) = make_uint2(a0, a1);
        }
        pair_hidden<ACTK>(S, cc, l, A.c1[l], cd, y, hA, h);
    }
    // both outputs go to workspace buffers with room for whole workgroup tiles, so nothing here is conditional
    pair_transform_quant<true>(S, y, A.inv_in[l + 1], qlo, qhi, h, D.xhat + ci * 512, reinterpret_cast<int *>(D.codes_out + ci * 512));
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
}

// ------------------------------------------------------------------------------- host code
bool dhq_pair_shape_ok(const dhq_model *m)
{
    const int L = m->n_layers;
    if (L < 2) return false;
    if (m->dims[0] > 4 || m->dims[L] > 32) return false;
    for (int l = 1; l < L; ++l)
        if (m->dims[l] != 512) return false;
    return true;
}

// k position jj of lane half u in k block kb of a hidden layer's A fragment holds rotated input
// feature hm_index(16 kb + jj, u): the order in which the transform leaves the codes.
static void pair_pack_tile(const dhq_layer &Ly, int T, int Kb, bool first, int8_t *frag)
{
    const int8_t *wq = Ly.wq_host.data();
    for (int kb = 0; kb < Kb; ++kb)
        for (int ln = 0; ln < 64; ++ln) {
            const int row = 32 * T + (ln & 31), u = ln >> 5;
            for (int jj = 0; jj < 16; ++jj) {
                int8_t val = 0;
                if (row < Ly.M) {
                    if (first) {
                        if (u == 0 && jj < Ly.Kp) val = wq[(size_t)row * Ly.Kp + jj];
                    } else {
                        val = wq[(size_t)row * Ly.Kp + hm_index(16 * kb + jj, u)];
                    }
                }
                frag[((size_t)kb * 64 + ln) * 16 + jj] = val;
            }
        }
}

int dhq_pair_create(const dhq_model *m, dhq_pair_plan **plan_out)
{
    *plan_out = nullptr;
    if (!dhq_pair_shape_ok(m)) return DHQ_OK;
    const int L = m->n_layers;
    dhq_pair_plan *P = new (std::nothrow) dhq_pair_plan();
    if (!P) return DHQ_ENOMEM;
    memset(&P->args, 0, sizeof(P->args));
    const int n_chunks = 2 + 8 * (L - 2);
    // chunks, one more chunk of padding (the in-kernel copy always moves 32 KiB), then the bias table
    const size_t bias_off = (size_t)(n_chunks + 1) * PAIR_BUF;
    std::vector<unsigned char> blob(bias_off + (size_t)L * 512 * sizeof(float), 0);
    for (int l = 0; l < L; ++l) {
        const dhq_layer &Ly = m->layer[l];
        if (l == 0) {
            for (int T = 0; T < 16; ++T) pair_pack_tile(Ly, T, 1, true, reinterpret_cast<int8_t *>(blob.data()) + (size_t)T * 1024);
        } else if (l == L - 1) {
            pair_pack_tile(Ly, 0, PAIR_KB, false, reinterpret_cast<int8_t *>(blob.data()) + (size_t)(n_chunks - 1) * PAIR_BUF);
        } else {
            for (int T = 0; T < 16; ++T)
                pair_pack_tile(Ly, T, PAIR_KB, false,
                               reinterpret_cast<int8_t *>(blob.data()) + (size_t)(1 + 8 * (l - 1) + (T & 7)) * PAIR_BUF + (size_t)(T >> 3) * 16384);
        }
        // biases: bias_slot order within a tile, in revolutions for the layers that end in an activation
        float *bias = reinterpret_cast<float *>(blob.data() + bias_off) + (size_t)l * 512;
        const std::vector<float> &src = (l == L - 1) ? Ly.bias_host : Ly.bias_rev_host;
        for (int f = 0; f < Ly.M; ++f) bias[bias_slot(f)] = src[f];
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
    P->args.n_chunks = n_chunks;
    P->args.bias_off = (uint32_t)bias_off;
    P->args.c2 = dhq_hidden_act(m).c2;
    P->act_kind = m->act_kind;
    P->lds_bytes = (size_t)PAIR_BIAS + 3 * 2048;
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

void dhq_pair_destroy(dhq_pair_plan *P)
{
    if (!P) return;
    if (P->blob_dev) (void)hipFree(P->blob_dev);
    delete P;
}

int dhq_pair_update_scales(const dhq_model *m, dhq_pair_plan *P)
{
    if (!P) return DHQ_OK;
    for (int l = 0; l < m->n_layers; ++l) {
        const dhq_layer &Ly = m->layer[l];
        P->args.c1[l] = dhq_c1(m, l);
        P->args.inv_in[l] = (float)(1.0 / ((double)Ly.s_a * sqrt((double)Ly.Kp)));
    }
    return DHQ_OK;
}

hipError_t dhq_pair_launch(const dhq_pair_plan *P, const float *coords, int64_t n, float *out, hipStream_t st)
{
    if (!P) return hipErrorInvalidValue;
    if (n <= 0) return hipSuccess;
    pair_args a = P->args;
    a.coords = coords;
    a.out = out;
    a.n = n;
    const int64_t tiles = (n + PAIR_TILE - 1) / PAIR_TILE;
    const unsigned grid = (unsigned)(tiles < P->n_cu ? tiles : P->n_cu);
    auto kern = (P->act_kind == DHQ_ACT_KIND_WAVELET) ? dhq_fused_pair_kernel<DHQ_ACT_KIND_WAVELET>
                : (P->act_kind == DHQ_ACT_KIND_WAVELET_COMPLEX) ? dhq_fused_pair_kernel<DHQ_ACT_KIND_WAVELET_COMPLEX> : dhq_fused_pair_kernel<DHQ_ACT_KIND_SINE>;
    hipError_t e = dhq_lds_limit_once(kern, P->lds_bytes, P->device);
    if (e != hipSuccess) return e;
    kern<<<grid, PAIR_THREADS, P->lds_bytes, st>>>(a);
    return hipGetLastError();
}

// The dynamic mode on the per-layer kernels above (same contract as dhq_fused_dynamic_launch): ws0 / ws1 hold
// dhq_pair_dynamic_rows(n) x 512 floats each.
size_t dhq_pair_dynamic_rows(int64_t n) { return (size_t)((n + PAIR_TILE - 1) / PAIR_TILE) * PAIR_TILE; }

template <int MODE, int ACTK>
static hipError_t pairl_launch_t(const dhq_pair_plan *P, const pair_largs &a, unsigned grid, hipStream_t st)
{
    auto kern = dhq_fused_pair_layer_kernel<MODE, ACTK>;
    hipError_t e = dhq_lds_limit_once(kern, P->lds_bytes, P->device);
    if (e != hipSuccess) return e;
    kern<<<grid, PAIR_THREADS, P->lds_bytes, st>>>(a);
    return hipGetLastError();
}

hipError_t dhq_pair_dynamic_launch(const dhq_model *m, const float *coords, int64_t n, float *out, float *ws0, float *ws1,
                                   float *partial, float *dyn, hipStream_t st)
{
    const dhq_pair_plan *P = m->pair;
    if (!P) return hipErrorInvalidValue;
    if (n <= 0) return hipSuccess;
    const int L = m->n_layers;
    const bool wav = (P->act_kind == DHQ_ACT_KIND_WAVELET), cpx = (P->act_kind == DHQ_ACT_KIND_WAVELET_COMPLEX);
    const int64_t tiles = (n + PAIR_TILE - 1) / PAIR_TILE;
    const unsigned grid = (unsigned)(tiles < P->n_cu ? tiles : P->n_cu);
    if (grid > DHQ_ABSMAX_PARTIALS) return hipErrorInvalidValue;
    // the input layer's scale: max over the rotated coordinates, left as per-workgroup maxima
    float *pbuf[2] = {partial, partial + DHQ_ABSMAX_PARTIALS};
    int count = 0;
    hipError_t e = dhq_launch_wht_absmax_partials(coords, n, m->layer[0].K, m->layer[0].Kp, pbuf[0], &count, st);
    if (e != hipSuccess) return e;
    float *bufs[2] = {ws0, ws1};
    for (int l = 0; l < L; ++l) {
        pair_largs a;
        memset(&a, 0, sizeof(a));
        a.w = P->args;
        a.w.coords = coords;
        a.w.out = out;
        a.w.n = n;
        // the chunks of this layer alone, in a cycle
        a.w.chunk_base = (l == 0) ? 0 : (l == L - 1 ? P->args.n_chunks - 1 : 1 + 8 * (l - 1));
        a.w.n_chunks = (l == 0 || l == L - 1) ? 1 : 8;
        a.xin = reinterpret_cast<const float4 *>(bufs[(l + 1) & 1]);
        a.xout = reinterpret_cast<float4 *>(bufs[l & 1]);
        a.partial_in = pbuf[l & 1];
        a.partial_count = count;
        a.kp = m->layer[l].Kp;
        a.layer = l;
        a.c1_over_sa = dhq_c1_over_sa(m, l);
        a.dyn = dyn + 3 * l;
        a.partial = pbuf[(l + 1) & 1];
        if (l == 0) e = wav ? pairl_launch_t<0, DHQ_ACT_KIND_WAVELET>(P, a, grid, st) : cpx ? pairl_launch_t<0, DHQ_ACT_KIND_WAVELET_COMPLEX>(P, a, grid, st)
                                                                                        : pairl_launch_t<0, DHQ_ACT_KIND_SINE>(P, a, grid, st);
        else if (l < L - 1) e = wav ? pairl_launch_t<1, DHQ_ACT_KIND_WAVELET>(P, a, grid, st) : cpx ? pairl_launch_t<1, DHQ_ACT_KIND_WAVELET_COMPLEX>(P, a, grid, st)
                                                                                                : pairl_launch_t<1, DHQ_ACT_KIND_SINE>(P, a, grid, st);
        else e = pairl_launch_t<2, DHQ_ACT_KIND_NONE>(P, a, grid, st);  // the output layer has no activation
        if (e != hipSuccess) return e;
        count = (int)grid;
    }
    return hipSuccess;
}

// Test hook behind dhq_forward_debug_fused for the two-wave kernel.
hipError_t dhq_pair_debug_launch(const dhq_model *m, int layer, const int8_t *codes_in, int64_t n, float *xhat, int8_t *codes_out,
                                 int32_t *acc, hipStream_t st)
{
    const dhq_pair_plan *P = m->pair;
    if (!P || layer < 0 || layer >= m->n_layers - 1) return hipErrorInvalidValue;
    if (n <= 0) return hipSuccess;
    if (n > DHQ_CHUNK) return hipErrorInvalidValue;  // the outputs pass through the model's workspace (whole tiles)
    pair_dargs d;
    memset(&d, 0, sizeof(d));
    d.w = P->args;
    d.w.n = n;
    d.codes_in = codes_in;
    d.xhat = m->act0;
    d.codes_out = m->codes;
    d.acc = acc;
    d.layer = layer;
    d.kp_in = m->layer[layer].Kp;
    const unsigned grid = (unsigned)((n + PAIR_TILE - 1) / PAIR_TILE);
    auto kern = (P->act_kind == DHQ_ACT_KIND_WAVELET) ? dhq_fused_pair_kernel_debug<DHQ_ACT_KIND_WAVELET>
                : (P->act_kind == DHQ_ACT_KIND_WAVELET_COMPLEX) ? dhq_fused_pair_kernel_debug<DHQ_ACT_KIND_WAVELET_COMPLEX>
                                                                : dhq_fused_pair_kernel_debug<DHQ_ACT_KIND_SINE>;
    hipError_t e = dhq_lds_limit_once(kern, P->lds_bytes, P->device);
    if (e != hipSuccess) return e;
    if (acc) {
        pair_debug_acc_kernel<<<(unsigned)((n + 31) / 32), 64, 0, st>>>(d);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    if (!xhat && !codes_out) return hipSuccess;
    kern<<<grid, PAIR_THREADS, P->lds_bytes, st>>>(d);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    if (xhat && (e = hipMemcpyAsync(xhat, m->act0, sizeof(float) * (size_t)n * 512, hipMemcpyDeviceToDevice, st)) != hipSuccess) return e;
    if (codes_out && (e = hipMemcpyAsync(codes_out, m->codes, (size_t)n * 512, hipMemcpyDeviceToDevice, st)) != hipSuccess) return e;
    return hipSuccess;
}
