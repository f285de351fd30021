// Streaming dequant-GEMV kernels for small batches (M <= 16), native layout, grouped launch.
//
// Computes y = x * Deq(W)^T (the W. products of App. A.1) for several matrices in one launch,
// each SQ or VQ as its flag says (Sec. 3.1, Eq. "optimization goal").  The work is bound by
// reading the packed weights once from HBM, so everything else is arranged around keeping
// 16-byte coalesced loads in flight while spending as few issue slots per weight as possible.
//
//   * decode_kernel<MT>: one wavefront owns one 16-row tile of one matrix and streams its
//     256-column tiles in order with DEPTH tiles in flight (tile_pipeline); four wavefronts form a
//     workgroup (64 rows).  Up to 256 matrices per launch, longest rows first; a workgroup finds
//     its matrix with ballots over the table in the kernel arguments.
//   * Batch 1 (MT = 1), all formats, on the vector ALU: lane (r, kg) owns row r's columns of column
//     group kg; the sixteen lanes of a row each load one activation pair, and every
//     v_dot2c_f32_f16 names the lane that holds its pair through the DPP control row_newbcast - no
//     LDS for the activations.  SQ codes are multiplied as they are: masked in place, a 3-bit code
//     at mantissa bits b..b+2 of an fp16 half is the subnormal q 2^(b-24); three accumulators (one
//     per bit position) are combined with exact powers of two per group, and
//     y += s (sum q x - z X) with X from four DPP adds.  VQ weights are gathered pair by pair from
//     the block's codebook in a wavefront-private LDS region.
//   * decode_splitk_kernel<S>: batch 1 for launches too small to fill the device (the stages of a
//     block): one workgroup of S wavefronts per row tile, the column tiles dealt round-robin, the
//     partial sums added in LDS in a fixed order.  With MixedDecodeArgs the token-shift mix of
//     Eq. "time mixing r/k/v" is applied while the activations are loaded; with PostMixArgs the
//     outputs also leave as the mixes of the stage that follows (store_post_mix).  The squared ReLU
//     and the gates of App. A.1 can be applied where an output is stored (store_post).
//   * decode_rkv_wkv_kernel: the three projections of time mixing and the wkv step of Eq. "time
//     mixing wkv" in one launch (a workgroup takes a row tile of r, k and v and steps its 16 channels).
//   * Batch 2..32 (MT = 4, 16, 32) on the matrix cores (v_mfma_f32_16x16x32_f16, activations = A
//     operand, weights = B operand): the activation tile of a column tile is fetched once per
//     workgroup into LDS (two buffers, one barrier per tile); SQ codes enter as 8 + q (one shift
//     and one and-or per pair), the group sums X come from one more MFMA against an all-ones
//     operand, y += s (acc - (8 + z) X); VQ pairs are LDS gathers.  A wavefront takes two row
//     tiles of W, and with MT = 32 two groups of 16 batch rows: every unpacked weight operand
//     feeds one MFMA per group.
//   * bf16 activations are converted to fp16 on load, group by group under an exact power-of-two
//     scale (see "bf16 activations" below), so their whole range is accepted.
#include "common.h"
#include "../../include/rwkvq.h"
#include <algorithm>

namespace rwkvq {

// Batch 1: column tiles in flight beyond the one being consumed, and the wavefronts per SIMD the compiler must leave
// registers for.  One tile ahead keeps the grouped kernel at 64 registers, eight wavefronts per SIMD; two tiles ahead
// (79 registers, six per SIMD) put more bytes in flight per compute unit (72 against 48 KB) and were slower once the
// weight loads carried the non-temporal hint: 7B stack 5.79 -> 5.96 TB/s, 14B-class stack 5.65 -> 5.75 TB/s, the token
// step of the 7B blocks (split-K kernels, 65 registers instead of 79-106) 1.008 -> 0.935 ms, same box, alternating.
#ifndef RWKVQ_DECODE_MINBLOCKS
#define RWKVQ_DECODE_MINBLOCKS 8
#endif
#ifndef RWKVQ_DECODE_DEPTH
#define RWKVQ_DECODE_DEPTH 1
#endif
constexpr int kMaxGroupMats = 256;    // matrices per grouped launch (descriptor table in kernarg: a whole
                                      // 32-layer stack is one launch, one ramp-up and one tail)
constexpr int kXStride = 272;         // fp16 per staged activation row: 34 units of 16 bytes, so that the 16 lanes an LDS
                                      // cycle serves (rows m..m+7 of column groups kg, kg+1) fall into 16 distinct units
#ifndef RWKVQ_SPLIT_TARGET
#define RWKVQ_SPLIT_TARGET 2048
#endif
constexpr int kSplitTarget = RWKVQ_SPLIT_TARGET;   // wavefronts a batch-1 launch should have before it stops splitting K
#ifndef RWKVQ_DECODE_RT
#define RWKVQ_DECODE_RT 1
#endif
constexpr int kRT = RWKVQ_DECODE_RT;  // batch 1: 16-row tiles per wavefront
static_assert(kRT == 1, "the batch-1 tile loops hold one row tile per wavefront");
#ifndef RWKVQ_DECODE_BATCH_RT
#define RWKVQ_DECODE_BATCH_RT 2
#endif
#ifndef RWKVQ_BATCH_UB2
#define RWKVQ_BATCH_UB2 0            // batch 2..16: 1 = read the activation fragments of both column halves of a tile up front
#endif
#ifndef RWKVQ_BATCH_DEPTH
#define RWKVQ_BATCH_DEPTH 1          // batch 2..32: tiles in flight beyond the one being consumed
#endif
#ifndef RWKVQ_BATCH16_MINBLOCKS
#define RWKVQ_BATCH16_MINBLOCKS 4    // wavefronts per SIMD the compiler must leave registers for (batch 5..16)
#endif
#ifndef RWKVQ_BATCH4_MINBLOCKS
#define RWKVQ_BATCH4_MINBLOCKS 4
#endif
// Batch 2..16: row tiles per wavefront.  Every wavefront reads the whole activation tile from LDS as
// its A operands; with two row tiles those reads serve twice the weights (the batched path is bound
// by LDS traffic: M = 16 gained 12-16 % per format over one row tile).
constexpr int kBRT = RWKVQ_DECODE_BATCH_RT;
static_assert(kBRT == 1 || kBRT == 2 || kBRT == 4, "row tiles of a wavefront share a 256-row codebook block");
constexpr int rt_of(int MT) { return MT == 1 ? kRT : kBRT; }
#ifndef RWKVQ_BATCH_WAVES
#define RWKVQ_BATCH_WAVES 4
#endif
// Batch 2..32: wavefronts per workgroup (4 or 8).  They share the staged activation tile, so its reads from
// the L2 (M x 512 bytes per column tile and workgroup) are spread over that many rows of W.  Measured on the
// 14B-class shapes: eight wavefronts gain 1.5-3 % on single-format stacks at batch 16 and lose 2-8 % on the
// mixed stack at batch 4 and 32 (longer tails of the larger workgroups): four is the default.
constexpr int kBW = RWKVQ_BATCH_WAVES;
static_assert(kBW == 4 || kBW == 8, "sixteen or thirty-two threads stage a batch row");
constexpr int waves_of(int MT) { return MT == 1 ? 4 : kBW; }
// Batch 2..32: row passes of a workgroup per column tile (1 or 2, a template parameter of the kernel).  With two,
// the staged activation tile (and, for VQ, the tile's codebook) serves a second stretch of rows before the
// next tile is staged: half the activation reads from the L2, half the staging work and half the barriers
// per weight (configuration 5 at batch 16: 4.44 -> 4.79 TB/s).  The launcher takes two passes when the launch
// still has RWKVQ_OPT_STREAM_TWO_PASS_MIN_WGS workgroups that way (2048 unless set), and one otherwise: a single
// 4096 x 4096 matrix is 32 workgroups of 128 rows, and halving that count costs more than the staging saves
// (25 -> 40 us at 17..32 rows).
constexpr bool kTwoPassFits = 16 * kBW * kBRT * 2 <= 256;   // the rows of a workgroup share a 256-row codebook block
constexpr int wg_rows(int MT, int P = 1) { return 16 * waves_of(MT) * rt_of(MT) * (MT == 1 ? 1 : P); }   // rows of W per workgroup

struct DecodeMat {
    const uint32_t* codes;
    const uint16_t* aux;
    const void* x;
    void* y;
    int N, K, fmt;
    int post;                         // PostOp applied to the output before it is stored (batch 1)
    const void* gate;                 // POST_SIGMOID_GATE: [N] values of the output type
};
// A matrix whose input is mixed on the fly: x (of DecodeMat) is x_t.
struct MixedMat : DecodeMat {
    const uint16_t* xprev;            // x_{t-1}, same type and length as x
    const uint8_t* mix_idx;           // K / 2 indices of the mix weight
    const uint32_t* mix_cb;           // its codebook: mix_E entries of two fp16
    int mix_E, pad2;
};
constexpr int kMaxMixedMats = 64;
constexpr int kGrid2DMaxMats = 8;     // split-K kernels: launches of at most this many matrices are two-dimensional grids (matrix, row tile)
// A matrix whose output also leaves as the token-shift mixes of the stage that follows (up to four
// projections): out_p[n] = mu_p[n] y[n] + (1 - mu_p[n]) xprev[n].
struct PostMix { const uint8_t* idx; const uint32_t* cb; void* out; };
struct PostMixMat : DecodeMat {
    const void* xprev;                // the previous token's y, type of y
    PostMix mix[4];
    int n_mix, pad2;
};
struct PostMixArgs {
    static constexpr bool kMixed = false;
    static constexpr bool kPostMix = true;
    static constexpr int kMats = kMaxMixedMats;
    int wg_end[kMaxMixedMats];
    PostMixMat m[kMaxMixedMats];
    int M, xdt, ydt, pad;
};
struct MixedDecodeArgs {
    static constexpr bool kMixed = true;
    static constexpr bool kPostMix = false;
    static constexpr int kMats = kMaxMixedMats;
    int wg_end[kMaxMixedMats];
    MixedMat m[kMaxMixedMats];
    int M, xdt, ydt, pad;
};
struct DecodeArgs {                   // 15 KB of kernel arguments
    static constexpr bool kMixed = false;
    static constexpr bool kPostMix = false;
    static constexpr int kMats = kMaxGroupMats;
    int wg_end[kMaxGroupMats];        // first workgroup index after matrix i (INT_MAX when unused)
    DecodeMat m[kMaxGroupMats];
    int M, xdt, ydt, pad;
};

// Batch-1 output with the element-wise operator that follows the projection in the block (App. A.1)
// applied on the way out.  The value is first rounded to the output type, as a separate pass would
// have read it from memory, then max(y, 0)^2 (Eq. "channel mixing o", input of W'_v) or
// sigma(gate) * y (the gates of Eq. "time mixing o" / "channel mixing o") in binary32, then rounded
// for the store: the same bits as the projection followed by rwkvq_relu2 / rwkvq_sigmoid_gate.
// A value of the given type as its bits, and back: what the lanes that store a row tile ask memory for at the start of
// a split-K kernel (gate, previous token, mix indices) stays bits until the end, so that nothing in front of the
// multiply waits for it (converted at once, each load is a trip to memory that the wavefront sits out).
__device__ __forceinline__ uint32_t load_bits(const void* p, size_t i, int dt) {
    return dt == DT_F32 ? ((const uint32_t*)p)[i] : (uint32_t)((const uint16_t*)p)[i];
}
__device__ __forceinline__ float bits_to_f32(uint32_t b, int dt) {
    return dt == DT_F16 ? f16_bits_to_f32((uint16_t)b) : dt == DT_BF16 ? bf16_bits_to_f32((uint16_t)b) : __uint_as_float(b);
}
// gate_bits: the gate's bits if the caller fetched them ahead (have_gate), else it is loaded here
__device__ __forceinline__ float store_post(const DecodeMat& mt, size_t i, int ydt, float v, bool have_gate = false,
                                            uint32_t gate_bits = 0) {
    if (mt.post != POST_NONE) {
        if (ydt == DT_F16) v = f16_bits_to_f32(f32_to_f16_bits(v));
        else if (ydt == DT_BF16) v = bf16_bits_to_f32(f32_to_bf16_bits(v));
        if (mt.post == POST_RELU2) {
            const float m = fmaxf(v, 0.0f);
            v = m * m;
        } else {
            v = gate_f32(have_gate ? bits_to_f32(gate_bits, ydt) : load_as_f32(mt.gate, i, ydt), v);
        }
    }
    store_from_f32(mt.y, i, ydt, v);
    return v;
}

// The same, and the stored value again as the token-shift mixes of the stage that follows (Eq. "time
// mixing r/k/v", "channel mixing r/k"): the mix is element-wise, so it can be taken where the vector is
// produced, once, instead of by every workgroup of the stage that consumes it.  Arithmetic as the mix
// pass and the fused mix: the stored (rounded) y, binary32, one rounding per operation, rounded to the type.
// The previous token's value and the indices are fetched by post_mix_prefetch at the start of the kernel
// (their latency hides behind the GEMV); the codebook entries, which depend on the indices, here, in one
// batch of loads.
struct PostMixPre { uint32_t xp, ix[4], gate; };        // as bits (see load_bits)
__device__ __forceinline__ void post_mix_prefetch(PostMixPre& pre, const PostMixMat& mt, size_t i, int ydt) {
    if (mt.post == POST_SIGMOID_GATE) pre.gate = load_bits(mt.gate, i, ydt);
    if (mt.n_mix > 0) {
        pre.xp = load_bits(mt.xprev, i, ydt);
        // every load unconditional (a mix that is not there reads the first one's index): no branch, no wait between them;
        // the aligned word that holds the index byte (a byte load is widened on the spot, which waits for it; the index
        // arrays are 16-byte aligned and N / 2 is a multiple of 8); static indices: mt stays in registers
#pragma unroll
        for (int p = 0; p < 4; ++p) pre.ix[p] = ((const uint32_t*)(p < mt.n_mix ? mt.mix[p].idx : mt.mix[0].idx))[i >> 3];
    }
}
__device__ __forceinline__ void store_post_mix(const PostMixMat& mt, size_t i, int ydt, float v, const PostMixPre& pre) {
    v = store_post(mt, i, ydt, v, true, pre.gate);
    if (mt.n_mix > 0) {
        const float xt = ydt == DT_F16 ? f16_bits_to_f32(f32_to_f16_bits(v)) : bf16_bits_to_f32(f32_to_bf16_bits(v));
        const float xp = bits_to_f32(pre.xp, ydt);
        uint32_t e[4];
#pragma unroll
        for (int p = 0; p < 4; ++p) e[p] = p < mt.n_mix ? mt.mix[p].cb[(pre.ix[p] >> (8 * ((i >> 1) & 3))) & 255u] : 0u;
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            if (p < mt.n_mix) {
                const float m = f16_bits_to_f32((uint16_t)((i & 1) ? e[p] >> 16 : e[p] & 0xFFFFu));
                const float o = __fadd_rn(__fmul_rn(m, xt), __fmul_rn(__fsub_rn(1.0f, m), xp));
                store_from_f32(mt.mix[p].out, i, ydt, o);
            }
        }
    }
}

template <int P>
__device__ __forceinline__ uint32_t sq_pair_f16(uint32_t w0, uint32_t w1, uint32_t w2, uint32_t mask,
                                                uint32_t magic) {
    // two 3-bit codes -> fp16x2 (8 + q_even, 8 + q_odd); mask = 0x03800380, magic = 0x48004800
    if constexpr (P < 15) {
        constexpr int p = P % 5, sh = 6 - 3 * p;
        uint32_t w = (P / 5 == 0) ? w0 : (P / 5 == 1) ? w1 : w2;
        uint32_t v = sh > 0 ? (w << (sh > 0 ? sh : 0)) : sh < 0 ? (w >> (sh < 0 ? -sh : 0)) : w;
        return (v & mask) | magic;
    } else {
        // bit b of the pair's two codes sits at bits 0 and 16 of word b
        uint32_t v = (w0 & 0x00010001u) | ((w1 & 0x00010001u) << 1) | ((w2 & 0x00010001u) << 2);
        return (v << 7) | magic;
    }
}

template <int T>
__device__ __forceinline__ half8_t sq_operand(uint32_t w0, uint32_t w1, uint32_t w2, uint32_t mask,
                                              uint32_t magic) {
    uint4_t v = {sq_pair_f16<4 * T + 0>(w0, w1, w2, mask, magic), sq_pair_f16<4 * T + 1>(w0, w1, w2, mask, magic),
                 sq_pair_f16<4 * T + 2>(w0, w1, w2, mask, magic), sq_pair_f16<4 * T + 3>(w0, w1, w2, mask, magic)};
    return __builtin_bit_cast(half8_t, v);
}

__device__ __forceinline__ half8_t vq8_operand(uint32_t w, const uint32_t* cb) {
    uint4_t v = {cb[w & 255u], cb[(w >> 8) & 255u], cb[(w >> 16) & 255u], cb[w >> 24]};
    return __builtin_bit_cast(half8_t, v);
}

// ---- activation staging (per wavefront) ----------------------------------------------------
// LDS regions are private to one wavefront and the LDS unit serves one wavefront's requests in
// issue order, so no hardware barrier is needed between a lane's store and another lane's load;
// the wavefront-scope fences only stop the compiler from moving accesses across this point.
__device__ __forceinline__ void wave_lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Batch 2..32: the activation tile [MT rows][256 columns] of a column tile is shared by the wavefronts of the
// workgroup.  kRowThreads threads fetch a row of it, kRowCols columns each (rows beyond M repeat row
// M - 1: every load is unconditional, see tile_pipeline) and later store them, converted to fp16,
// into one of two LDS buffers.
struct XShared { uint4_t a, b; };           // b: only with sixteen threads per row
constexpr int kRowThreads = 4 * kBW, kRowCols = 256 / kRowThreads;

__device__ __forceinline__ void x_load_wg(XShared& r, const uint16_t* x, int M, int K, int T, int tid, int g = 0) {
    const int row = 16 * g + tid / kRowThreads < M ? 16 * g + tid / kRowThreads : M - 1;
    const uint16_t* p = x + (size_t)row * K + 256 * T + kRowCols * (tid % kRowThreads);
    r.a = *(const uint4_t*)p;
    if constexpr (kRowCols == 16) r.b = *(const uint4_t*)(p + 8);
}

// ---- bf16 activations -----------------------------------------------------------------------
// These kernels multiply fp16 operands (codebook entries are fp16, SQ codes are fp16 subnormals in
// place), so bf16 activations are converted, and fp16 holds a bf16 value exactly only for
// magnitudes in [2^-17, 65536).  Activations that share an accumulator (batch 1: the 64 columns a
// row of sixteen lanes multiplies in a tile; batch > 1: the 256 columns of one batch row in a tile)
// are therefore first multiplied by the power of two that brings the largest magnitude among them to
// [2^15, 2^16), and their partial sum is multiplied by the inverse power before it joins the running
// output.  Both steps are exact, so every activation within 2^-32 of its group's largest enters the
// sum exactly, whatever the magnitudes are; a smaller one is cut off below 2^-39 of that largest (the
// conversion rounds toward zero, which only matters there), far below the resolution of the
// binary32 sum it joins.
typedef unsigned short ushort2_t __attribute__((ext_vector_type(2)));

// Larger of the two halves of max(|a|, |b|) taken per bf16 half: the magnitude bits of the largest of four values.
__device__ __forceinline__ uint32_t bf16x2_absmax(uint32_t a, uint32_t b) {
    const ushort2_t m = __builtin_elementwise_max(__builtin_bit_cast(ushort2_t, a & 0x7FFF7FFFu),
                                                  __builtin_bit_cast(ushort2_t, b & 0x7FFF7FFFu));
    const uint32_t w = __builtin_bit_cast(uint32_t, m);
    return max(w >> 16, w & 0xFFFFu);
}
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_max(uint32_t v) {   // lanes the control leaves out contribute zero
    const uint32_t o = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xF, 0xF, true);
    return max(v, o);
}
// All sixteen lanes of a row get the row's maximum.
__device__ __forceinline__ uint32_t dpp_row_max(uint32_t v) {
    v = dpp_max<0xB1>(v);       // quad_perm [1, 0, 3, 2]
    v = dpp_max<0x4E>(v);       // quad_perm [2, 3, 0, 1]
    v = dpp_max<0x141>(v);      // row_half_mirror
    return dpp_max<0x140>(v);   // row_mirror
}
// Exponent n of the scale 2^n for a group whose largest bf16 magnitude has the bits `amax`: the
// largest lands in [2^15, 2^16).  An all-zero (or tiny) group takes the largest n whose inverse
// 2^-n is still a normal binary32 number.
__device__ __forceinline__ int bf16_scale_exponent(uint32_t amax) {
    const int e = (int)(amax >> 7);                 // biased exponent, 0..254 for finite values
    return 142 - (e > 16 ? e : 16);
}
// Two bf16 -> two fp16, each multiplied by 2^n first.  Exact where fp16 can hold the product.
__device__ __forceinline__ uint32_t bf16x2_to_f16x2(uint32_t v, int n) {
    const float lo = ldexpf(__builtin_bit_cast(float, v << 16), n);
    const float hi = ldexpf(__builtin_bit_cast(float, v & 0xFFFF0000u), n);
    return __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(lo, hi));
}

// bf16: the threads that hold one batch row's 256 columns are one or two DPP rows of sixteen lanes; they agree
// on the row's scale for this tile, convert, and the first of them leaves the inverse scale in xsc[row].
template <int MT>
__device__ __forceinline__ void x_store_wg(const XShared& r, half_t* xs, float* xsc, int tid, bool bf16, int g = 0) {
    const int row = 16 * g + tid / kRowThreads;
    uint4_t a = r.a, b = r.b;
    if (bf16) {
        const ushort2_t m01 = __builtin_elementwise_max(__builtin_bit_cast(ushort2_t, a.x & 0x7FFF7FFFu), __builtin_bit_cast(ushort2_t, a.y & 0x7FFF7FFFu));
        const ushort2_t m23 = __builtin_elementwise_max(__builtin_bit_cast(ushort2_t, a.z & 0x7FFF7FFFu), __builtin_bit_cast(ushort2_t, a.w & 0x7FFF7FFFu));
        ushort2_t mm = __builtin_elementwise_max(m01, m23);
        if constexpr (kRowCols == 16) {
            const ushort2_t m45 = __builtin_elementwise_max(__builtin_bit_cast(ushort2_t, b.x & 0x7FFF7FFFu), __builtin_bit_cast(ushort2_t, b.y & 0x7FFF7FFFu));
            const ushort2_t m67 = __builtin_elementwise_max(__builtin_bit_cast(ushort2_t, b.z & 0x7FFF7FFFu), __builtin_bit_cast(ushort2_t, b.w & 0x7FFF7FFFu));
            mm = __builtin_elementwise_max(mm, __builtin_elementwise_max(m45, m67));
        }
        const uint32_t w = __builtin_bit_cast(uint32_t, mm);
        uint32_t amax = dpp_row_max(max(w >> 16, w & 0xFFFFu));
        if constexpr (kRowThreads == 32) amax = max(amax, (uint32_t)__shfl_xor((int)amax, 16, 64));   // the row's other sixteen lanes
        const int n = bf16_scale_exponent(amax);
        a.x = bf16x2_to_f16x2(a.x, n); a.y = bf16x2_to_f16x2(a.y, n); a.z = bf16x2_to_f16x2(a.z, n); a.w = bf16x2_to_f16x2(a.w, n);
        if constexpr (kRowCols == 16) {
            b.x = bf16x2_to_f16x2(b.x, n); b.y = bf16x2_to_f16x2(b.y, n); b.z = bf16x2_to_f16x2(b.z, n); b.w = bf16x2_to_f16x2(b.w, n);
        }
        if (tid % kRowThreads == 0) xsc[row] = ldexpf(1.0f, -n);      // rows beyond MT repeat row M - 1: written, never used
    }
    if (row < MT) {
        half_t* d = xs + row * kXStride + kRowCols * (tid % kRowThreads);
        *(uint4_t*)d = a;
        if constexpr (kRowCols == 16) *(uint4_t*)(d + 8) = b;
    }
}

// Packed weights (and their scales) are read exactly once per launch: loaded with the non-temporal hint,
// so that the stream does not displace the activations (read by every workgroup of a matrix) from the L2.
// Measured on the 7B shapes, batch 1, SQ: 5.9 -> 6.3 TB/s.
template <class T>
__device__ __forceinline__ T stream_load(const T* p) { return __builtin_nontemporal_load(p); }

// Batch 2..32, small launches (decode_splitk_batched_kernel): a wavefront takes its A operands straight from global
// memory in the layout the MFMA wants - lane (m, kg) = (lane % 16, lane / 16) holds, for column half u and k-step t of
// a 256-column tile, the eight consecutive activations 128 u + 32 t + 8 kg ... of batch row m (rows beyond M repeat
// row M - 1) - so nothing is staged in LDS and no workgroup barrier is needed: f[4 u + t].
struct XFrags { uint4_t f[8]; };
__device__ __forceinline__ void x_load_frags(XFrags& r, const uint16_t* x, int M, int K, int T, int lane, int g = 0) {
    const int m = 16 * g + (lane & 15) < M ? 16 * g + (lane & 15) : M - 1;     // g: group of 16 batch rows
    const uint16_t* p = x + (size_t)m * K + 256 * T + 8 * (lane >> 4);
#pragma unroll
    for (int i = 0; i < 8; ++i) r.f[i] = *(const uint4_t*)(p + 128 * (i >> 2) + 32 * (i & 3));
}
// bf16 fragments -> fp16, scaled by the power of two of the batch row's largest magnitude in this tile (the four lanes
// that hold a row agree through two exchanges); lane m < 16 leaves the row's inverse scale in scw[m].
__device__ __forceinline__ void x_frags_to_f16(XFrags& r, float* scw, int lane) {
    uint32_t amax = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) amax = max(amax, max(bf16x2_absmax(r.f[i].x, r.f[i].y), bf16x2_absmax(r.f[i].z, r.f[i].w)));
    amax = max(amax, (uint32_t)__shfl_xor((int)amax, 16, 64));
    amax = max(amax, (uint32_t)__shfl_xor((int)amax, 32, 64));
    const int n = bf16_scale_exponent(amax);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        r.f[i].x = bf16x2_to_f16x2(r.f[i].x, n); r.f[i].y = bf16x2_to_f16x2(r.f[i].y, n);
        r.f[i].z = bf16x2_to_f16x2(r.f[i].z, n); r.f[i].w = bf16x2_to_f16x2(r.f[i].w, n);
    }
    if (lane < 16) scw[lane] = ldexpf(1.0f, -n);
}

// v_dot2_f32_f16 on two packed fp16 pairs.
__device__ __forceinline__ float dot2(uint32_t w, uint32_t x, float acc) {   // two fp16 pairs, scalars in
    return __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, w), __builtin_bit_cast(half2_t, x), acc, false);
}

// v + (v of the lane that the DPP control selects); lanes the control leaves out add zero.
template <int CTRL, int ROW_MASK = 0xF>
__device__ __forceinline__ float dpp_add(float v) {
    const int o = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, ROW_MASK, 0xF, ROW_MASK == 0xF);
    return v + __builtin_bit_cast(float, o);
}


// ---- per-format tile loops ------------------------------------------------------------------

#define RWKVQ_MFMA(a, b, c) __builtin_amdgcn_mfma_f32_16x16x32_f16((a), (b), (c), 0, 0, 0)

// Software pipeline over the column tiles T = 0 .. KT-1 with DEPTH tiles in flight from HBM
// *while* a tile is being consumed: there is one register set more than the depth, and the load
// of tile T + DEPTH is issued before tile T is computed (a wavefront that only reloaded a set
// after consuming it would have one tile fewer in flight for the whole of its compute phase,
// which is what bounds a latency-limited stream).  Every load is unconditional, so the compiler
// counts outstanding loads exactly and waits only for the tile about to be consumed: past the
// end of the row the loads fetch the last tile again (cache hits, never used).
template <int DEPTH, class Regs, class Load, class Compute>
__device__ __forceinline__ void tile_pipeline(int KT, Load load, Compute compute) {
    static_assert(DEPTH == 1 || DEPTH == 2 || DEPTH == 3, "pipeline depth");
    const int last = KT - 1;
    auto c = [&](int T) { return T < KT ? T : last; };
    if constexpr (DEPTH == 1) {                  // two register sets: the next tile in flight while one is consumed
        Regs q0, q1;
        auto issue1 = [&](Regs& r, int T) {
            load(r, c(T));
            __builtin_amdgcn_sched_barrier(0);
        };
        __builtin_amdgcn_sched_barrier(0);
        issue1(q0, 0);
        for (int T = 0; T < KT; T += 2) {
            issue1(q1, T + 1);
            compute(q0, T);
            issue1(q0, T + 2);
            if (T + 1 < KT) compute(q1, T + 1);
        }
        return;
    }
    Regs r0, r1, r2, r3;
    // The fences keep each tile's loads together and in program order, in the prologue too: the
    // wait the compiler derives for a tile then lets all younger tiles stay in flight.
    auto issue = [&](Regs& r, int T) {
        load(r, c(T));
        __builtin_amdgcn_sched_barrier(0);
    };
    __builtin_amdgcn_sched_barrier(0);
    issue(r0, 0);
    issue(r1, 1);
    if (DEPTH == 3) issue(r2, 2);
    for (int T = 0; T < KT; T += DEPTH + 1) {
        if (DEPTH == 2) {
            issue(r2, T + 2);
            compute(r0, T);
            issue(r0, T + 3);
            if (T + 1 < KT) compute(r1, T + 1);
            issue(r1, T + 4);
            if (T + 2 < KT) compute(r2, T + 2);
        } else {
            issue(r3, T + 3);
            compute(r0, T);
            issue(r0, T + 4);
            if (T + 1 < KT) compute(r1, T + 1);
            issue(r1, T + 5);
            if (T + 2 < KT) compute(r2, T + 2);
            issue(r2, T + 6);
            if (T + 3 < KT) compute(r3, T + 3);
        }
    }
}

// Batch 2..32 with two row passes per column tile: the units of the pipeline are (tile, pass) pairs, one in
// flight while one is consumed.  Pass 0 of a tile carries the activation tile (and the codebook) and stages
// them; pass 1 streams only weights and reads what pass 0 staged.
template <int J> struct PassTag { static constexpr int value = J; };
template <class Regs, class Load, class Compute>
__device__ __forceinline__ void tile_pipeline_two_pass(int KT, Load load, Compute compute) {
    Regs q0, q1;
    const int last = KT - 1;
    __builtin_amdgcn_sched_barrier(0);
    load(q0, 0, PassTag<0>{});
    __builtin_amdgcn_sched_barrier(0);
    for (int T = 0; T < KT; ++T) {
        load(q1, T, PassTag<1>{});
        __builtin_amdgcn_sched_barrier(0);
        compute(q0, T, PassTag<0>{});
        load(q0, T < last ? T + 1 : last, PassTag<0>{});
        __builtin_amdgcn_sched_barrier(0);
        compute(q1, T, PassTag<1>{});
    }
}
template <int DEPTH, int P, class Regs, class Load, class Compute>
__device__ __forceinline__ void batched_pipeline(int KT, Load load, Compute compute) {
    static_assert(P == 1 || P == 2, "row passes per column tile");
    if constexpr (P == 2) tile_pipeline_two_pass<Regs>(KT, load, compute);
    else tile_pipeline<DEPTH, Regs>(KT, [&](Regs& r, int T) { load(r, T, PassTag<0>{}); },
                                    [&](const Regs& r, int T) { compute(r, T, PassTag<0>{}); });
}

template <int P>
__device__ __forceinline__ uint32_t vq6_lds_addr(uint32_t w0, uint32_t w1, uint32_t w2, uint32_t m, uint32_t base) {
    // LDS byte address of codebook entry P: (index * 4) | base, base aligned to 256 bytes
    if constexpr (P < 15) {
        constexpr int p = P % 5;
        uint32_t w = (P / 5 == 0) ? w0 : (P / 5 == 1) ? w1 : w2;
        return ((w >> (6 * p)) & m) | base;
    } else {
        return ((w0 & 3u) << 2) | ((w1 & 3u) << 4) | ((w2 & 3u) << 6) | base;
    }
}
__device__ __forceinline__ uint32_t lds_gather(uint32_t byte_addr) {
    return *(const __attribute__((address_space(3))) uint32_t*)(uintptr_t)byte_addr;
}
template <int T4>
__device__ __forceinline__ uint4_t vq6_gather4(uint32_t w0, uint32_t w1, uint32_t w2, uint32_t m, uint32_t base) {
    uint4_t v = {lds_gather(vq6_lds_addr<4 * T4 + 0>(w0, w1, w2, m, base)), lds_gather(vq6_lds_addr<4 * T4 + 1>(w0, w1, w2, m, base)),
                 lds_gather(vq6_lds_addr<4 * T4 + 2>(w0, w1, w2, m, base)), lds_gather(vq6_lds_addr<4 * T4 + 3>(w0, w1, w2, m, base))};
    return v;
}

// G = groups of 16 batch rows (1 for batch <= 16, 2 for batch 17..32)
constexpr int groups_of(int MT) { return MT <= 16 ? 1 : MT / 16; }
template <int G> struct SqRegs { uint4_t a[kBRT]; uint2_t b[kBRT]; uint2_t sz[kBRT]; XShared x[G]; XFrags xf[G]; };
template <int G> struct Vq6Regs { uint4_t a[kBRT]; uint2_t b[kBRT]; uint32_t cb; XShared x[G]; XFrags xf[G]; };
template <int G> struct Vq8Regs { uint4_t a[kBRT]; uint4_t b[kBRT]; uint4_t cb; XShared x[G]; XFrags xf[G]; };

// Everything a tile loop needs about its wavefront's position; R[i] are its row tiles (R[i] == R[0]
// for the tiles past the end of the matrix: worked on again, not stored).
struct WavePos {
    int R[4], M, lane, tid;
    int Rn[4];           // batch > 1, second row pass: its row tiles (Rn[i] == R[0] past the end of the matrix)
    bool xbf16;
    int t0, ts, nt;      // split-K (batch 1): this wavefront's column tiles are t0, t0 + ts, ... (nt of them)
    // fused token-shift mix (batch 1): the previous token's activations, the mix weight's indices
    // (one per column pair) and its codebook staged in LDS by this wavefront
    const uint16_t* xprev;
    const uint8_t* mix_idx;
    const uint32_t* mix_cb;
};

// Batch 2..16 on the matrix cores: activations = A operand (row m of the MFMA = batch row m, read
// from the shared LDS tile), weights = B operand.  `xs` points at the two activation buffers; the
// one workgroup barrier per tile both publishes tile T and guards the buffer tile T + 1 will
// overwrite (every wavefront has finished reading it once it has passed the barrier of tile T).
//
// SQ: the codes enter as 8 + q (one shift and one and-or per pair).  The group sums of the
// activations come from the matrix cores too: one more MFMA per k-step with an all-ones B operand
// leaves X_g[m] in the accumulator layout of the products, and y += s (acc - (8 + z) X_g).
template <int MT, int DEPTH, bool XB, int P, bool DIRECT = false>
__device__ __forceinline__ void run_sq(const DecodeMat& mt, const WavePos& wp, half_t* xs, float* xsc,
                                       float4_t (&out)[P][groups_of(MT)][kBRT]) {
    constexpr int G = groups_of(MT), UB = (G == 1 && RWKVQ_BATCH_UB2) ? 2 : 1;   // one group: the fragments of both column halves up front
    using Regs = SqRegs<G>;
    const int KT = mt.K >> 8, lane = wp.lane, M = wp.M;
    const uint32_t* codes[P][kBRT];
    const uint2_t* sz[P][kBRT];
#pragma unroll
    for (int j = 0; j < P; ++j)
#pragma unroll
        for (int rt = 0; rt < kBRT; ++rt) {
            const int R = j == 0 ? wp.R[rt] : wp.Rn[rt];
            codes[j][rt] = mt.codes + (size_t)R * KT * 384;
            sz[j][rt] = (const uint2_t*)mt.aux + (size_t)R * KT * 16;
        }
    int xoff[G];
#pragma unroll
    for (int g = 0; g < G; ++g) xoff[g] = (16 * g + (lane & 15) < M ? 16 * g + (lane & 15) : M - 1) * kXStride + 8 * (lane >> 4);
    // The and-or that builds 8 + q takes its mask from a VGPR and the fp16 pattern of 8.0 from an
    // SGPR: a VOP3 instruction of this ISA takes no literal and at most one scalar operand.
    uint32_t mask, magic;
    asm("v_mov_b32 %0, 0x03800380" : "=v"(mask));
    asm("s_mov_b32 %0, 0x48004800" : "=s"(magic));
    const uint4_t ones4 = {0x3C003C00u, 0x3C003C00u, 0x3C003C00u, 0x3C003C00u};
    const half8_t ones = __builtin_bit_cast(half8_t, ones4);
    static_assert(!DIRECT || P == 1, "fragments from global memory: one row pass");
    auto load = [&](Regs& r, int T, auto pass) {
        constexpr int J = decltype(pass)::value;
        if constexpr (DIRECT) T = wp.t0 + T * wp.ts;     // this wavefront's column tiles
#pragma unroll
        for (int rt = 0; rt < kBRT; ++rt) {
            const uint32_t* t = codes[J][rt] + (size_t)T * 384;
            r.a[rt] = stream_load((const uint4_t*)(t + 4 * lane));
            r.b[rt] = stream_load((const uint2_t*)(t + 256 + 2 * lane));
            r.sz[rt] = stream_load(sz[J][rt] + (size_t)T * 16 + (lane & 15));
        }
        if constexpr (DIRECT) {
#pragma unroll
            for (int g = 0; g < G; ++g) x_load_frags(r.xf[g], (const uint16_t*)mt.x, M, mt.K, T, lane, g);
        } else if constexpr (J == 0) {
#pragma unroll
            for (int g = 0; g < G; ++g) x_load_wg(r.x[g], (const uint16_t*)mt.x, M, mt.K, T, wp.tid, g);
        }
    };
    auto compute = [&](const Regs& r, int T, auto pass) {
        constexpr int J = decltype(pass)::value;
        half_t* buf = xs + (T & 1) * (MT * kXStride);
        float* scb = xsc + (T & 1) * (16 * G);
        XFrags xf[G];
        if constexpr (DIRECT) {
#pragma unroll
            for (int g = 0; g < G; ++g) {
                xf[g] = r.xf[g];
                if (XB) x_frags_to_f16(xf[g], scb + 16 * g, lane);
            }
            if (XB) wave_lds_sync();
        } else if constexpr (J == 0) {
#pragma unroll
            for (int g = 0; g < G; ++g) x_store_wg<MT>(r.x[g], buf, scb, wp.tid, XB, g);
            __syncthreads();
        }
        float4_t sc[G];                              // bf16: inverse scale of this tile for the lane's batch rows
#pragma unroll
        for (int g = 0; g < G; ++g) sc[g] = XB ? *(const float4_t*)(scb + 16 * g + 4 * (lane >> 4)) : float4_t{1, 1, 1, 1};
#pragma unroll
        for (int ub = 0; ub < 2; ub += UB) {
            half8_t xa[UB][G][4];
#pragma unroll
            for (int uu = 0; uu < UB; ++uu)
#pragma unroll
                for (int g = 0; g < G; ++g)
#pragma unroll
                    for (int t = 0; t < 4; ++t)
                        xa[uu][g][t] = DIRECT ? __builtin_bit_cast(half8_t, xf[g].f[4 * (ub + uu) + t]) : *(const half8_t*)(buf + xoff[g] + 128 * (ub + uu) + 32 * t);
#pragma unroll
            for (int uu = 0; uu < UB; ++uu) {
                const int u = ub + uu;
                float4_t X[G];                       // X_g[m] for the lane's batch rows
#pragma unroll
                for (int g = 0; g < G; ++g) {
                    X[g] = float4_t{0, 0, 0, 0};
#pragma unroll
                    for (int t = 0; t < 4; ++t) X[g] = RWKVQ_MFMA(xa[uu][g][t], ones, X[g]);
                }
#pragma unroll
                for (int rt = 0; rt < kBRT; ++rt) {
                    const uint32_t w0 = u == 0 ? r.a[rt].x : r.a[rt].w, w1 = u == 0 ? r.a[rt].y : r.b[rt].x,
                                   w2 = u == 0 ? r.a[rt].z : r.b[rt].y;
                    const half8_t op0 = sq_operand<0>(w0, w1, w2, mask, magic), op1 = sq_operand<1>(w0, w1, w2, mask, magic),
                                  op2 = sq_operand<2>(w0, w1, w2, mask, magic), op3 = sq_operand<3>(w0, w1, w2, mask, magic);
                    const uint32_t szw = u == 0 ? r.sz[rt].x : r.sz[rt].y;
                    const float s = f16_bits_to_f32((uint16_t)(szw & 0xFFFFu));
                    const float z8 = f16_bits_to_f32((uint16_t)(szw >> 16)) + 8.0f;
#pragma unroll
                    for (int g = 0; g < G; ++g) {
                        float4_t acc = {0, 0, 0, 0};
                        acc = RWKVQ_MFMA(xa[uu][g][0], op0, acc);
                        acc = RWKVQ_MFMA(xa[uu][g][1], op1, acc);
                        acc = RWKVQ_MFMA(xa[uu][g][2], op2, acc);
                        acc = RWKVQ_MFMA(xa[uu][g][3], op3, acc);
#pragma unroll
                        for (int i = 0; i < 4; ++i) out[J][g][rt][i] = fmaf(XB ? s * sc[g][i] : s, fmaf(-z8, X[g][i], acc[i]), out[J][g][rt][i]);
                    }
                }
            }
        }
    };
    batched_pipeline<DEPTH, P, Regs>(DIRECT ? wp.nt : KT, load, compute);
}

// 6-bit VQ: the codebook of a tile (64 entries, one per lane) goes through a wavefront-private LDS
// slot and every weight pair is one ds_read_b32 gather (cheaper on this part than ds_bpermute).
template <int MT, int DEPTH, bool XB, int P, bool DIRECT = false>
__device__ __forceinline__ void run_vq6(const DecodeMat& mt, const WavePos& wp, half_t* xs, float* xsc, uint32_t* cb_lds,
                                        float4_t (&out)[P][groups_of(MT)][kBRT]) {
    constexpr int G = groups_of(MT), UB = (G == 1 && RWKVQ_BATCH_UB2) ? 2 : 1;
    using Regs = Vq6Regs<G>;
    const int KT = mt.K >> 8, lane = wp.lane, M = wp.M;
    const uint32_t* codes[P][kBRT];
#pragma unroll
    for (int j = 0; j < P; ++j)
#pragma unroll
        for (int rt = 0; rt < kBRT; ++rt) codes[j][rt] = mt.codes + (size_t)(j == 0 ? wp.R[rt] : wp.Rn[rt]) * KT * 384;
    const uint32_t* cbs = (const uint32_t*)mt.aux + (size_t)(wp.R[0] >> 4) * KT * 64;
    int xoff[G];
#pragma unroll
    for (int g = 0; g < G; ++g) xoff[g] = (16 * g + (lane & 15) < M ? 16 * g + (lane & 15) : M - 1) * kXStride + 8 * (lane >> 4);
    const uint32_t base0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint32_t*)cb_lds;
    uint32_t m;
    asm("v_mov_b32 %0, 0xfc" : "=v"(m));
    static_assert(!DIRECT || P == 1, "fragments from global memory: one row pass");
    auto load = [&](Regs& r, int T, auto pass) {
        constexpr int J = decltype(pass)::value;
        if constexpr (DIRECT) T = wp.t0 + T * wp.ts;     // this wavefront's column tiles
#pragma unroll
        for (int rt = 0; rt < kBRT; ++rt) {
            const uint32_t* t = codes[J][rt] + (size_t)T * 384;
            r.a[rt] = stream_load((const uint4_t*)(t + 4 * lane));
            r.b[rt] = stream_load((const uint2_t*)(t + 256 + 2 * lane));
        }
        if constexpr (DIRECT) {
            r.cb = (cbs + (size_t)T * 64)[lane];
#pragma unroll
            for (int g = 0; g < G; ++g) x_load_frags(r.xf[g], (const uint16_t*)mt.x, M, mt.K, T, lane, g);
        } else if constexpr (J == 0) {
            r.cb = (cbs + (size_t)T * 64)[lane];
#pragma unroll
            for (int g = 0; g < G; ++g) x_load_wg(r.x[g], (const uint16_t*)mt.x, M, mt.K, T, wp.tid, g);
        }
    };
    auto compute = [&](const Regs& r, int T, auto pass) {
        constexpr int J = decltype(pass)::value;
        half_t* buf = xs + (T & 1) * (MT * kXStride);
        float* scb = xsc + (T & 1) * (16 * G);
        XFrags xf[G];
        if constexpr (DIRECT) {
#pragma unroll
            for (int g = 0; g < G; ++g) {
                xf[g] = r.xf[g];
                if (XB) x_frags_to_f16(xf[g], scb + 16 * g, lane);
            }
            cb_lds[(T & 1) * 256 + lane] = r.cb;
            wave_lds_sync();
        } else if constexpr (J == 0) {
#pragma unroll
            for (int g = 0; g < G; ++g) x_store_wg<MT>(r.x[g], buf, scb, wp.tid, XB, g);
            cb_lds[(T & 1) * 256 + lane] = r.cb;     // two slots, 1 KB apart (the gather address ORs the index in)
            __syncthreads();
        }
        const uint32_t base = base0 + (T & 1) * 1024;
        // bf16: the tile's products are summed on their own and join the output through the rows' inverse scales
        float4_t part[G][kBRT];
        float4_t (&acc)[G][kBRT] = *(XB ? &part : &out[J]);
        if (XB) {
#pragma unroll
            for (int g = 0; g < G; ++g)
#pragma unroll
                for (int rt = 0; rt < kBRT; ++rt) part[g][rt] = float4_t{0, 0, 0, 0};
        }
#pragma unroll
        for (int ub = 0; ub < 2; ub += UB) {
            half8_t xa[UB][G][4];
#pragma unroll
            for (int uu = 0; uu < UB; ++uu)
#pragma unroll
                for (int g = 0; g < G; ++g)
#pragma unroll
                    for (int t = 0; t < 4; ++t)
                        xa[uu][g][t] = DIRECT ? __builtin_bit_cast(half8_t, xf[g].f[4 * (ub + uu) + t]) : *(const half8_t*)(buf + xoff[g] + 128 * (ub + uu) + 32 * t);
#pragma unroll
            for (int uu = 0; uu < UB; ++uu) {
                const int u = ub + uu;
#pragma unroll
                for (int rt = 0; rt < kBRT; ++rt) {
                    const uint32_t w0 = u == 0 ? r.a[rt].x : r.a[rt].w, w1 = u == 0 ? r.a[rt].y : r.b[rt].x,
                                   w2 = u == 0 ? r.a[rt].z : r.b[rt].y;
                    const half8_t op0 = __builtin_bit_cast(half8_t, vq6_gather4<0>(w0, w1, w2, m, base)),
                                  op1 = __builtin_bit_cast(half8_t, vq6_gather4<1>(w0, w1, w2, m, base)),
                                  op2 = __builtin_bit_cast(half8_t, vq6_gather4<2>(w0, w1, w2, m, base)),
                                  op3 = __builtin_bit_cast(half8_t, vq6_gather4<3>(w0, w1, w2, m, base));
#pragma unroll
                    for (int g = 0; g < G; ++g) {
                        acc[g][rt] = RWKVQ_MFMA(xa[uu][g][0], op0, acc[g][rt]);
                        acc[g][rt] = RWKVQ_MFMA(xa[uu][g][1], op1, acc[g][rt]);
                        acc[g][rt] = RWKVQ_MFMA(xa[uu][g][2], op2, acc[g][rt]);
                        acc[g][rt] = RWKVQ_MFMA(xa[uu][g][3], op3, acc[g][rt]);
                    }
                }
            }
        }
        if (XB) {
#pragma unroll
            for (int g = 0; g < G; ++g) {
                const float4_t sc = *(const float4_t*)(scb + 16 * g + 4 * (lane >> 4));
#pragma unroll
                for (int rt = 0; rt < kBRT; ++rt)
#pragma unroll
                    for (int i = 0; i < 4; ++i) out[J][g][rt][i] = fmaf(part[g][rt][i], sc[i], out[J][g][rt][i]);
            }
        }
    };
    batched_pipeline<DEPTH, P, Regs>(DIRECT ? wp.nt : KT, load, compute);
}

// 8-bit VQ: the codebook of a tile (256 entries) goes through a wavefront-private LDS region; the
// workgroup barrier that publishes the activations also orders that store before the gathers.
template <int MT, int DEPTH, bool XB, int P, bool DIRECT = false>
__device__ __forceinline__ void run_vq8(const DecodeMat& mt, const WavePos& wp, half_t* xs, float* xsc, uint32_t* cb_lds,
                                        float4_t (&out)[P][groups_of(MT)][kBRT]) {
    constexpr int G = groups_of(MT);
    using Regs = Vq8Regs<G>;
    const int KT = mt.K >> 8, lane = wp.lane, M = wp.M;
    const uint32_t* codes[P][kBRT];
#pragma unroll
    for (int j = 0; j < P; ++j)
#pragma unroll
        for (int rt = 0; rt < kBRT; ++rt) codes[j][rt] = mt.codes + (size_t)(j == 0 ? wp.R[rt] : wp.Rn[rt]) * KT * 512;
    const uint4_t* cbs = (const uint4_t*)mt.aux + (size_t)(wp.R[0] >> 4) * KT * 64;
    int xoff[G];
#pragma unroll
    for (int g = 0; g < G; ++g) xoff[g] = (16 * g + (lane & 15) < M ? 16 * g + (lane & 15) : M - 1) * kXStride + 8 * (lane >> 4);
    static_assert(!DIRECT || P == 1, "fragments from global memory: one row pass");
    auto load = [&](Regs& r, int T, auto pass) {
        constexpr int J = decltype(pass)::value;
        if constexpr (DIRECT) T = wp.t0 + T * wp.ts;     // this wavefront's column tiles
#pragma unroll
        for (int rt = 0; rt < kBRT; ++rt) {
            const uint32_t* t = codes[J][rt] + (size_t)T * 512;
            r.a[rt] = stream_load((const uint4_t*)(t + 4 * lane));
            r.b[rt] = stream_load((const uint4_t*)(t + 256 + 4 * lane));
        }
        if constexpr (DIRECT) {
            r.cb = (cbs + (size_t)T * 64)[lane];
#pragma unroll
            for (int g = 0; g < G; ++g) x_load_frags(r.xf[g], (const uint16_t*)mt.x, M, mt.K, T, lane, g);
        } else if constexpr (J == 0) {
            r.cb = (cbs + (size_t)T * 64)[lane];
#pragma unroll
            for (int g = 0; g < G; ++g) x_load_wg(r.x[g], (const uint16_t*)mt.x, M, mt.K, T, wp.tid, g);
        }
    };
    auto compute = [&](const Regs& r, int T, auto pass) {
        constexpr int J = decltype(pass)::value;
        half_t* buf = xs + (T & 1) * (MT * kXStride);
        float* scb = xsc + (T & 1) * (16 * G);
        uint32_t* cbuf = cb_lds + (T & 1) * 256;     // two codebook slots, like the activations
        XFrags xf[G];
        if constexpr (DIRECT) {
#pragma unroll
            for (int g = 0; g < G; ++g) {
                xf[g] = r.xf[g];
                if (XB) x_frags_to_f16(xf[g], scb + 16 * g, lane);
            }
            *(uint4_t*)(cbuf + 4 * lane) = r.cb;
            wave_lds_sync();
        } else if constexpr (J == 0) {
#pragma unroll
            for (int g = 0; g < G; ++g) x_store_wg<MT>(r.x[g], buf, scb, wp.tid, XB, g);
            *(uint4_t*)(cbuf + 4 * lane) = r.cb;
            __syncthreads();
        }
        float4_t part[G][kBRT];                      // bf16: as in run_vq6
        float4_t (&acc)[G][kBRT] = *(XB ? &part : &out[J]);
        if (XB) {
#pragma unroll
            for (int g = 0; g < G; ++g)
#pragma unroll
                for (int rt = 0; rt < kBRT; ++rt) part[g][rt] = float4_t{0, 0, 0, 0};
        }
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            half8_t xa[G][4];
#pragma unroll
            for (int g = 0; g < G; ++g)
#pragma unroll
                for (int t = 0; t < 4; ++t)
                    xa[g][t] = DIRECT ? __builtin_bit_cast(half8_t, xf[g].f[4 * u + t]) : *(const half8_t*)(buf + xoff[g] + 128 * u + 32 * t);
#pragma unroll
            for (int rt = 0; rt < kBRT; ++rt) {
                const uint4_t w = u == 0 ? r.a[rt] : r.b[rt];
                const half8_t op0 = vq8_operand(w.x, cbuf), op1 = vq8_operand(w.y, cbuf), op2 = vq8_operand(w.z, cbuf),
                              op3 = vq8_operand(w.w, cbuf);
#pragma unroll
                for (int g = 0; g < G; ++g) {
                    acc[g][rt] = RWKVQ_MFMA(xa[g][0], op0, acc[g][rt]);
                    acc[g][rt] = RWKVQ_MFMA(xa[g][1], op1, acc[g][rt]);
                    acc[g][rt] = RWKVQ_MFMA(xa[g][2], op2, acc[g][rt]);
                    acc[g][rt] = RWKVQ_MFMA(xa[g][3], op3, acc[g][rt]);
                }
            }
        }
        if (XB) {
#pragma unroll
            for (int g = 0; g < G; ++g) {
                const float4_t sc = *(const float4_t*)(scb + 16 * g + 4 * (lane >> 4));
#pragma unroll
                for (int rt = 0; rt < kBRT; ++rt)
#pragma unroll
                    for (int i = 0; i < 4; ++i) out[J][g][rt][i] = fmaf(part[g][rt][i], sc[i], out[J][g][rt][i]);
            }
        }
    };
    batched_pipeline<DEPTH, P, Regs>(DIRECT ? wp.nt : KT, load, compute);
}

// ------------------------------------------------------------------------------------------
// Batch 1 (GEMV proper).  Same streaming structure and native layout, but the contraction is
// done by the vector ALU (v_dot2c_f32_f16: two multiply-adds per lane, binary32 accumulate):
// with a single activation row fifteen sixteenths of every MFMA would be spent on padding, and
// the padded MFMA costs the same issue time as the dot products.  Lane (r, kg) accumulates the part
// of row r's dot product that falls on its own columns; the four kg lanes of a row are summed at
// the end.  The activations are not staged in LDS: lane (kg, i) loads pair i of the sixteen
// column pairs that column group kg multiplies in a unit, and each dot product names the lane of
// its row that holds its pair (DPP row broadcast).
//   SQ:  the codes are multiplied in place as fp16 subnormals; per group
//        y += s * (sum q x - z * Xp), Xp = the sum of the lane's own activations of the group.
//   VQ:  the codebook of the current block sits in a wavefront-private LDS region; each pair of
//        weights is one ds_read_b32 gather feeding one dot2.

// acc += w . x, where x is the fp16 pair that lane N of the 16-lane row holds in xp (DPP
// row_newbcast): the sixteen rows' lanes of a column group all multiply by the same activations,
// which therefore need neither LDS nor a copy per lane.
template <int N>
__device__ __forceinline__ float dot2_row_bcast(float acc, uint32_t xp, uint32_t w) {
    asm("v_dot2c_f32_f16_dpp %0, %1, %2 row_newbcast:%3 row_mask:0xf bank_mask:0xf" : "+v"(acc) : "v"(xp), "v"(w), "n"(N));
    return acc;
}
// The dot products above are opaque to the compiler's hazard checks.  On this ISA the result of
// a dot instruction may be read (or overwritten) by a different vector-ALU instruction only
// three wait states later; accumulating dot products of the same kind need none.  Call this
// between the last dot product into an accumulator and any other use of it.
#define RWKVQ_DOT_RESULT_FENCE(...) asm volatile("s_nop 2" : __VA_ARGS__)

template <int T>
__device__ __forceinline__ float dot8_row_bcast(float acc, uint32_t xp, const uint4_t b) {
    const uint32_t b0 = b.x, b1 = b.y, b2 = b.z, b3 = b.w;
    acc = dot2_row_bcast<4 * T + 0>(acc, xp, b0);
    acc = dot2_row_bcast<4 * T + 1>(acc, xp, b1);
    acc = dot2_row_bcast<4 * T + 2>(acc, xp, b2);
    acc = dot2_row_bcast<4 * T + 3>(acc, xp, b3);
    return acc;
}

// Activations of a tile for the row-broadcast dot products: lane (kg, i) holds, for unit u, the
// pair of columns 128 u + 32 (i / 4) + 8 kg + 2 (i % 4) + {0, 1}, i.e. pair i of the sixteen
// that the lanes of column group kg multiply in that unit, in MFMA-step order.
struct XPairs { uint32_t p[2]; };
__device__ __forceinline__ void xpairs_load(XPairs& r, const uint16_t* x, int T, int lane) {
    const int i = lane & 15, kg = lane >> 4;
    const uint16_t* xt = x + 256 * T + 32 * (i >> 2) + 8 * kg + 2 * (i & 3);
    r.p[0] = *(const uint32_t*)xt;
    r.p[1] = *(const uint32_t*)(xt + 128);
}

// Fused token-shift mix (Eq. "time mixing r/k/v"): the wavefront loads, beside its pairs of x_t, the
// same pairs of x_{t-1} and the two index bytes of the mix weight (one 2-vector of the weight covers
// exactly one column pair), and mixes before the dot products: fl(fl(m x_t) + fl(fl(1 - m) x_{t-1}))
// per element in binary32, rounded to the activation type - the values a separate mix pass would
// have stored.
__device__ __forceinline__ void mix_load(XPairs& xq, uint32_t& mi, const WavePos& wp, int T, int lane) {
    xpairs_load(xq, wp.xprev, T, lane);
    const int i = lane & 15, kg = lane >> 4;
    const uint8_t* p = wp.mix_idx + 128 * T + 16 * (i >> 2) + 4 * kg + (i & 3);
    mi = (uint32_t)p[0] | ((uint32_t)p[64] << 8);
}
__device__ __forceinline__ uint32_t mix_pair(uint32_t xt, uint32_t xp, uint32_t entry, bool bf16) {
    const half2_t mh = __builtin_bit_cast(half2_t, entry);
    const half_t ma = mh.x, mb = mh.y;
    const float m0 = (float)ma, m1 = (float)mb;
    float t0, t1, u0, u1;
    if (bf16) {
        t0 = __uint_as_float(xt << 16); t1 = __uint_as_float(xt & 0xFFFF0000u);
        u0 = __uint_as_float(xp << 16); u1 = __uint_as_float(xp & 0xFFFF0000u);
    } else {
        const half2_t th = __builtin_bit_cast(half2_t, xt), uh = __builtin_bit_cast(half2_t, xp);
        const half_t ta = th.x, tb = th.y, ua = uh.x, ub = uh.y;
        t0 = (float)ta; t1 = (float)tb; u0 = (float)ua; u1 = (float)ub;
    }
    const float o0 = __fadd_rn(__fmul_rn(m0, t0), __fmul_rn(__fsub_rn(1.0f, m0), u0));
    const float o1 = __fadd_rn(__fmul_rn(m1, t1), __fmul_rn(__fsub_rn(1.0f, m1), u1));
    if (bf16) return (uint32_t)f32_to_bf16_bits(o0) | ((uint32_t)f32_to_bf16_bits(o1) << 16);
    return (uint32_t)f32_to_f16_bits(o0) | ((uint32_t)f32_to_f16_bits(o1) << 16);
}
template <class Regs>
__device__ __forceinline__ void mix_apply(const Regs& r, const WavePos& wp, uint32_t& x0, uint32_t& x1) {
    x0 = mix_pair(r.x.p[0], r.xq.p[0], wp.mix_cb[r.mi & 255u], wp.xbf16);
    x1 = mix_pair(r.x.p[1], r.xq.p[1], wp.mix_cb[(r.mi >> 8) & 255u], wp.xbf16);
}

struct Vq6M1Regs { uint4_t a[kRT]; uint2_t b[kRT]; uint32_t cb; XPairs x, xq; uint32_t mi; };

template <int DEPTH, bool SPLIT, bool MIXED, bool XB>
__device__ __forceinline__ void run_vq6_m1(const DecodeMat& mt, const WavePos& wp, uint32_t* cb_lds, float (&out)[kRT]) {
    const int KT = mt.K >> 8, lane = wp.lane;
    const uint32_t* codes[2] = {mt.codes + (size_t)wp.R[0] * KT * 384, mt.codes + (size_t)wp.R[1] * KT * 384};
    const uint32_t* cbs = (const uint32_t*)mt.aux + (size_t)(wp.R[0] >> 4) * KT * 64;
    const uint32_t base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint32_t*)cb_lds;
    uint32_t m;
    asm("v_mov_b32 %0, 0xfc" : "=v"(m));
    float acc1 = 0.f;                      // second accumulation chain, folded in at the end
    auto load = [&](Vq6M1Regs& r, int T) {
        if (SPLIT) T = wp.t0 + T * wp.ts;
#pragma unroll
        for (int rt = 0; rt < kRT; ++rt) {
            const uint32_t* t = codes[rt] + (size_t)T * 384;
            r.a[rt] = stream_load((const uint4_t*)(t + 4 * lane));
            r.b[rt] = stream_load((const uint2_t*)(t + 256 + 2 * lane));
        }
        r.cb = (cbs + (size_t)T * 64)[lane];
        xpairs_load(r.x, (const uint16_t*)mt.x, T, lane);
        if (MIXED) mix_load(r.xq, r.mi, wp, T, lane);
    };
    auto compute = [&](const Vq6M1Regs& r, int) {
        wave_lds_sync();
        cb_lds[lane] = r.cb;
        wave_lds_sync();
        uint32_t x0 = r.x.p[0], x1 = r.x.p[1];
        if (MIXED) mix_apply(r, wp, x0, x1);
        int nx = 0;                                       // bf16: x0, x1 enter as 2^nx times the activations
        if (XB) {
            nx = bf16_scale_exponent(dpp_row_max(bf16x2_absmax(x0, x1)));
            x0 = bf16x2_to_f16x2(x0, nx); x1 = bf16x2_to_f16x2(x1, nx);
        }
        // a DPP read needs two wait states after a vector-ALU write of the register
        asm volatile("s_nop 1" : "+v"(x0), "+v"(x1));
        // All sixteen gathers of a unit are issued before its dot products, and the second
        // unit's before the first unit's dot products, so the LDS latency is paid once per tile.
        static_assert(kRT == 1, "one row tile per wavefront");
        uint4_t g[2][4];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const uint32_t w0 = u == 0 ? r.a[0].x : r.a[0].w, w1 = u == 0 ? r.a[0].y : r.b[0].x,
                           w2 = u == 0 ? r.a[0].z : r.b[0].y;
            g[u][0] = vq6_gather4<0>(w0, w1, w2, m, base);
            g[u][1] = vq6_gather4<1>(w0, w1, w2, m, base);
            g[u][2] = vq6_gather4<2>(w0, w1, w2, m, base);
            g[u][3] = vq6_gather4<3>(w0, w1, w2, m, base);
        }
        __builtin_amdgcn_sched_barrier(0);
        // two accumulation chains (one per unit), interleaved, so that a dot product never waits
        // for the one issued just before it
        if (XB) {
            // the tile's products on their own, then into the output through the inverse scale
            float p0 = 0.f, p1 = 0.f;
            p1 = dot8_row_bcast<0>(p1, x1, g[1][0]);
            p0 = dot8_row_bcast<0>(p0, x0, g[0][0]);
            p1 = dot8_row_bcast<1>(p1, x1, g[1][1]);
            p0 = dot8_row_bcast<1>(p0, x0, g[0][1]);
            p1 = dot8_row_bcast<2>(p1, x1, g[1][2]);
            p0 = dot8_row_bcast<2>(p0, x0, g[0][2]);
            p1 = dot8_row_bcast<3>(p1, x1, g[1][3]);
            p0 = dot8_row_bcast<3>(p0, x0, g[0][3]);
            RWKVQ_DOT_RESULT_FENCE("+v"(p0), "+v"(p1));
            out[0] += ldexpf(p0 + p1, -nx);
        } else {
            acc1 = dot8_row_bcast<0>(acc1, x1, g[1][0]);
            out[0] = dot8_row_bcast<0>(out[0], x0, g[0][0]);
            acc1 = dot8_row_bcast<1>(acc1, x1, g[1][1]);
            out[0] = dot8_row_bcast<1>(out[0], x0, g[0][1]);
            acc1 = dot8_row_bcast<2>(acc1, x1, g[1][2]);
            out[0] = dot8_row_bcast<2>(out[0], x0, g[0][2]);
            acc1 = dot8_row_bcast<3>(acc1, x1, g[1][3]);
            out[0] = dot8_row_bcast<3>(out[0], x0, g[0][3]);
        }
    };
    tile_pipeline<DEPTH, Vq6M1Regs>(SPLIT ? wp.nt : KT, load, compute);
    RWKVQ_DOT_RESULT_FENCE("+v"(out[0]), "+v"(acc1));
    out[0] += acc1;
}

// Batch-1 SQ on the vector ALU.  The codes are multiplied as they are, with no 8 + q pattern: a
// 3-bit code left at mantissa bits b..b+2 of an fp16 half is the subnormal q * 2^(b-24), which
// v_dot2c_f32_f16 multiplies exactly.  A pair of codes therefore costs one AND (codes at bits 1, 4
// or 7 of the halves) or a share of one shift by 9 that brings the codes at bits 10 and 13 down
// to bits 1 and 4.  Products of different bit positions go to different accumulators (acc[0..2] for
// bits 1, 4, 7), which are combined with exact powers of two once per group.
struct SqM1Regs { uint4_t a[kRT]; uint2_t b[kRT]; uint2_t sz[kRT]; XPairs x, xq; uint32_t mi; };

template <int P>
__device__ __forceinline__ void sq_dot_pair(float (&acc)[3], uint32_t xp, uint32_t w0, uint32_t w1, uint32_t w2,
                                            uint32_t s0, uint32_t s1, uint32_t s2) {
    // s0..s2 = w0..w2 >> 9
    if constexpr (P < 15) {
        constexpr int p = P % 5;
        const uint32_t w = (P / 5 == 0) ? w0 : (P / 5 == 1) ? w1 : w2;
        const uint32_t sh = (P / 5 == 0) ? s0 : (P / 5 == 1) ? s1 : s2;
        if constexpr (p == 0) acc[0] = dot2_row_bcast<P>(acc[0], xp, w & 0x000E000Eu);
        else if constexpr (p == 1) acc[1] = dot2_row_bcast<P>(acc[1], xp, w & 0x00700070u);
        else if constexpr (p == 2) acc[2] = dot2_row_bcast<P>(acc[2], xp, w & 0x03800380u);
        else if constexpr (p == 3) acc[0] = dot2_row_bcast<P>(acc[0], xp, sh & 0x000E000Eu);
        else acc[1] = dot2_row_bcast<P>(acc[1], xp, sh & 0x00700070u);
    } else {
        // bit b of the pair's two codes sits at bits 0 and 16 of word b; assembled at bits 1..3
        const uint32_t t = (((w2 & 0x00010001u) << 1) | (w1 & 0x00010001u)) << 1 | (w0 & 0x00010001u);
        acc[0] = dot2_row_bcast<15>(acc[0], xp, t << 1);
    }
}

template <int... P>
__device__ __forceinline__ void sq_dot_pairs(float (&acc)[3], uint32_t xp, uint32_t w0, uint32_t w1, uint32_t w2,
                                             uint32_t s0, uint32_t s1, uint32_t s2) {
    (sq_dot_pair<P>(acc, xp, w0, w1, w2, s0, s1, s2), ...);
}

template <int DEPTH, bool SPLIT, bool MIXED, bool XB>
__device__ __forceinline__ void run_sq_m1(const DecodeMat& mt, const WavePos& wp, float (&out)[kRT]) {
    static_assert(kRT == 1, "one row tile per wavefront");
    const int KT = mt.K >> 8, lane = wp.lane;
    const uint32_t* codes = mt.codes + (size_t)wp.R[0] * KT * 384;
    const uint2_t* sz = (const uint2_t*)mt.aux + (size_t)wp.R[0] * KT * 16;
    auto load = [&](SqM1Regs& r, int T) {
        if (SPLIT) T = wp.t0 + T * wp.ts;
        const uint32_t* t = codes + (size_t)T * 384;
        r.a[0] = stream_load((const uint4_t*)(t + 4 * lane));
        r.b[0] = stream_load((const uint2_t*)(t + 256 + 2 * lane));
        r.sz[0] = stream_load(sz + (size_t)T * 16 + (lane & 15));
        xpairs_load(r.x, (const uint16_t*)mt.x, T, lane);
        if (MIXED) mix_load(r.xq, r.mi, wp, T, lane);
    };
    auto compute = [&](const SqM1Regs& r, int) {
        uint32_t x0 = r.x.p[0], x1 = r.x.p[1];
        if (MIXED) mix_apply(r, wp, x0, x1);
        int nx = 0;                                       // bf16: x0, x1 enter as 2^nx times the activations
        if (XB) {
            nx = bf16_scale_exponent(dpp_row_max(bf16x2_absmax(x0, x1)));
            x0 = bf16x2_to_f16x2(x0, nx); x1 = bf16x2_to_f16x2(x1, nx);
        }
        asm volatile("s_nop 1" : "+v"(x0), "+v"(x1));     // vector-ALU write -> DPP read
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const uint32_t xp = u == 0 ? x0 : x1;
            const uint32_t w0 = u == 0 ? r.a[0].x : r.a[0].w, w1 = u == 0 ? r.a[0].y : r.b[0].x,
                           w2 = u == 0 ? r.a[0].z : r.b[0].y;
            // Xp = 2^-17 times the sum of the activations this lane's column group multiplies in the
            // unit: the sixteen lanes of the row hold one pair each
            float Xp = dot2(xp, 0x00800080u, 0.f);         // 2^-17 (x_lo + x_hi): fp16 0x0080 = 2^-17
            Xp = dpp_add<0xB1>(Xp);
            Xp = dpp_add<0x4E>(Xp);
            Xp = dpp_add<0x141>(Xp);
            Xp = dpp_add<0x140>(Xp);
            float acc[3] = {0.f, 0.f, 0.f};
            sq_dot_pairs<0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15>(acc, xp, w0, w1, w2, w0 >> 9, w1 >> 9, w2 >> 9);
            RWKVQ_DOT_RESULT_FENCE("+v"(acc[0]), "+v"(acc[1]), "+v"(acc[2]));
            // sum x q = 2^17 S with S = 64 acc0 + 8 acc1 + acc2; Xp carries the same 2^-17, and so
            // does the running output, which is scaled back once at the end
            const float S = fmaf(acc[0], 64.f, fmaf(acc[1], 8.f, acc[2]));
            const uint32_t szw = u == 0 ? r.sz[0].x : r.sz[0].y;
            const float s = f16_bits_to_f32((uint16_t)(szw & 0xFFFFu));
            const float z = f16_bits_to_f32((uint16_t)(szw >> 16));
            out[0] = fmaf(XB ? ldexpf(s, -nx) : s, fmaf(-z, Xp, S), out[0]);
        }
    };
    tile_pipeline<DEPTH, SqM1Regs>(SPLIT ? wp.nt : KT, load, compute);
    out[0] *= 131072.f;
}

struct Vq8M1Regs { uint4_t a[kRT]; uint4_t b[kRT]; uint4_t cb; XPairs x, xq; uint32_t mi; };

template <int DEPTH, bool SPLIT, bool MIXED, bool XB>
__device__ __forceinline__ void run_vq8_m1(const DecodeMat& mt, const WavePos& wp, uint32_t* cb_lds, float (&out)[kRT]) {
    static_assert(kRT == 1, "one row tile per wavefront");
    const int KT = mt.K >> 8, lane = wp.lane;
    const uint32_t* codes = mt.codes + (size_t)wp.R[0] * KT * 512;
    const uint4_t* cbs = (const uint4_t*)mt.aux + (size_t)(wp.R[0] >> 4) * KT * 64;
    float acc1 = 0.f;
    auto load = [&](Vq8M1Regs& r, int T) {
        if (SPLIT) T = wp.t0 + T * wp.ts;
        const uint32_t* t = codes + (size_t)T * 512;
        r.a[0] = stream_load((const uint4_t*)(t + 4 * lane));
        r.b[0] = stream_load((const uint4_t*)(t + 256 + 4 * lane));
        r.cb = (cbs + (size_t)T * 64)[lane];
        xpairs_load(r.x, (const uint16_t*)mt.x, T, lane);
        if (MIXED) mix_load(r.xq, r.mi, wp, T, lane);
    };
    auto compute = [&](const Vq8M1Regs& r, int) {
        wave_lds_sync();
        *(uint4_t*)(cb_lds + 4 * lane) = r.cb;
        wave_lds_sync();
        uint32_t x0 = r.x.p[0], x1 = r.x.p[1];
        if (MIXED) mix_apply(r, wp, x0, x1);
        int nx = 0;                                       // bf16: x0, x1 enter as 2^nx times the activations
        if (XB) {
            nx = bf16_scale_exponent(dpp_row_max(bf16x2_absmax(x0, x1)));
            x0 = bf16x2_to_f16x2(x0, nx); x1 = bf16x2_to_f16x2(x1, nx);
        }
        asm volatile("s_nop 1" : "+v"(x0), "+v"(x1));     // vector-ALU write -> DPP read
        uint4_t g[2][4];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const uint4_t w = u == 0 ? r.a[0] : r.b[0];
            g[u][0] = __builtin_bit_cast(uint4_t, vq8_operand(w.x, cb_lds));
            g[u][1] = __builtin_bit_cast(uint4_t, vq8_operand(w.y, cb_lds));
            g[u][2] = __builtin_bit_cast(uint4_t, vq8_operand(w.z, cb_lds));
            g[u][3] = __builtin_bit_cast(uint4_t, vq8_operand(w.w, cb_lds));
        }
        __builtin_amdgcn_sched_barrier(0);
        if (XB) {
            // the tile's products on their own, then into the output through the inverse scale
            float p0 = 0.f, p1 = 0.f;
            p1 = dot8_row_bcast<0>(p1, x1, g[1][0]);
            p0 = dot8_row_bcast<0>(p0, x0, g[0][0]);
            p1 = dot8_row_bcast<1>(p1, x1, g[1][1]);
            p0 = dot8_row_bcast<1>(p0, x0, g[0][1]);
            p1 = dot8_row_bcast<2>(p1, x1, g[1][2]);
            p0 = dot8_row_bcast<2>(p0, x0, g[0][2]);
            p1 = dot8_row_bcast<3>(p1, x1, g[1][3]);
            p0 = dot8_row_bcast<3>(p0, x0, g[0][3]);
            RWKVQ_DOT_RESULT_FENCE("+v"(p0), "+v"(p1));
            out[0] += ldexpf(p0 + p1, -nx);
        } else {
            acc1 = dot8_row_bcast<0>(acc1, x1, g[1][0]);
            out[0] = dot8_row_bcast<0>(out[0], x0, g[0][0]);
            acc1 = dot8_row_bcast<1>(acc1, x1, g[1][1]);
            out[0] = dot8_row_bcast<1>(out[0], x0, g[0][1]);
            acc1 = dot8_row_bcast<2>(acc1, x1, g[1][2]);
            out[0] = dot8_row_bcast<2>(out[0], x0, g[0][2]);
            acc1 = dot8_row_bcast<3>(acc1, x1, g[1][3]);
            out[0] = dot8_row_bcast<3>(out[0], x0, g[0][3]);
        }
    };
    tile_pipeline<DEPTH, Vq8M1Regs>(SPLIT ? wp.nt : KT, load, compute);
    RWKVQ_DOT_RESULT_FENCE("+v"(out[0]), "+v"(acc1));
    out[0] += acc1;
}

// The batch-1 tile loop of a matrix's format; XB = the activations are bf16.
template <int DEPTH, bool SPLIT, bool MIXED>
__device__ __forceinline__ void run_m1(const DecodeMat& mt, const WavePos& wp, uint32_t* cb_lds, float (&part)[kRT]) {
    if (wp.xbf16) {
        if (mt.fmt == FMT_SQ3) run_sq_m1<DEPTH, SPLIT, MIXED, true>(mt, wp, part);
        else if (mt.fmt == FMT_VQ6) run_vq6_m1<DEPTH, SPLIT, MIXED, true>(mt, wp, cb_lds, part);
        else run_vq8_m1<DEPTH, SPLIT, MIXED, true>(mt, wp, cb_lds, part);
    } else {
        if (mt.fmt == FMT_SQ3) run_sq_m1<DEPTH, SPLIT, MIXED, false>(mt, wp, part);
        else if (mt.fmt == FMT_VQ6) run_vq6_m1<DEPTH, SPLIT, MIXED, false>(mt, wp, cb_lds, part);
        else run_vq8_m1<DEPTH, SPLIT, MIXED, false>(mt, wp, cb_lds, part);
    }
}
// The same for batch 2..32.  DIRECT: the split-K form (activation fragments from global memory, see XFrags).
template <int MT, int DEPTH, int P, bool DIRECT = false>
__device__ __forceinline__ void run_batched(const DecodeMat& mt, const WavePos& wp, half_t* xs, float* xsc, uint32_t* cb_lds,
                                            float4_t (&out)[P][groups_of(MT)][kBRT]) {
    if (wp.xbf16) {
        if (mt.fmt == FMT_SQ3) run_sq<MT, DEPTH, true, P, DIRECT>(mt, wp, xs, xsc, out);
        else if (mt.fmt == FMT_VQ6) run_vq6<MT, DEPTH, true, P, DIRECT>(mt, wp, xs, xsc, cb_lds, out);
        else run_vq8<MT, DEPTH, true, P, DIRECT>(mt, wp, xs, xsc, cb_lds, out);
    } else {
        if (mt.fmt == FMT_SQ3) run_sq<MT, DEPTH, false, P, DIRECT>(mt, wp, xs, xsc, out);
        else if (mt.fmt == FMT_VQ6) run_vq6<MT, DEPTH, false, P, DIRECT>(mt, wp, xs, xsc, cb_lds, out);
        else run_vq8<MT, DEPTH, false, P, DIRECT>(mt, wp, xs, xsc, cb_lds, out);
    }
}

// Workgroups per compute unit the compiler must leave registers for: the macros give wavefronts per SIMD.
constexpr int min_blocks(int MT) {
    if (MT == 1) return RWKVQ_DECODE_MINBLOCKS;
    const int per_simd = MT == 4 ? RWKVQ_BATCH4_MINBLOCKS : MT == 16 ? RWKVQ_BATCH16_MINBLOCKS : 2;
    return per_simd * 4 / kBW > 0 ? per_simd * 4 / kBW : 1;
}

// MT = number of activation rows carried (1, 4, 16 or 32 >= M).  MT = 1 runs every format on the
// vector ALU (run_*_m1); the others on the matrix cores, whose D layout is: lane holds batch rows
// 4*(lane/16) + i of output column lane%16.
template <int MT, int P = 1>
__global__ void __launch_bounds__(64 * waves_of(MT), min_blocks(MT)) decode_kernel(DecodeArgs a) {
    static_assert(MT > 1 || P == 1, "batch 1 has no staged activation tile to share");
    constexpr int DEPTH = MT == 1 ? RWKVQ_DECODE_DEPTH : RWKVQ_BATCH_DEPTH;
    // batch > 1: two activation tiles shared by the workgroup; codebook slots per wavefront
    __shared__ __attribute__((aligned(16))) half_t xs[MT == 1 ? 8 : 2 * MT * kXStride];
    __shared__ __attribute__((aligned(1024))) uint32_t cb_all[waves_of(MT)][MT == 1 ? 256 : 512];
    __shared__ __attribute__((aligned(16))) float xsc[MT == 1 ? 4 : 2 * 16 * groups_of(MT)];   // bf16: inverse scales per tile and batch row

    // Which matrix does this workgroup belong to?  Lane i compares against the end of matrix i
    // (one load per wavefront from the argument block); the count of matrices that end at or
    // before this workgroup is its matrix index.
    const int wg = blockIdx.x;
    static_assert(kMaxGroupMats % 64 == 0, "one table entry per lane and pass");
    int mi = 0;
#pragma unroll
    for (int j = 0; j < kMaxGroupMats; j += 64)
        mi += __builtin_popcountll(__builtin_amdgcn_ballot_w64(wg >= a.wg_end[j + (threadIdx.x & 63)]));
    const DecodeMat mt = a.m[mi];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int M = a.M;
    const bool xbf16 = a.xdt == DT_BF16;

    const int NR = mt.N >> 4;
    WavePos wp;
    constexpr int RT = rt_of(MT);
    wp.R[0] = RT * (waves_of(MT) * P * (wg - (mi ? a.wg_end[mi - 1] : 0)) + wave);
    const bool live = wp.R[0] < NR;                // rows beyond N (N not a multiple of the workgroup's rows)
    wp.M = M; wp.lane = lane; wp.tid = threadIdx.x; wp.xbf16 = xbf16;

    if constexpr (MT == 1) {
        if (!live) return;
        wp.R[1] = wp.R[2] = wp.R[3] = wp.R[0];
        float part[kRT];
#pragma unroll
        for (int rt = 0; rt < kRT; ++rt) part[rt] = 0.f;
        run_m1<DEPTH, false, false>(mt, wp, cb_all[wave], part);
#pragma unroll
        for (int rt = 0; rt < kRT; ++rt) {
            float v = part[rt];                    // sum the four column groups of each row
            v += __shfl_xor(v, 16, 64);
            v += __shfl_xor(v, 32, 64);
            if (lane < 16) store_post(mt, (size_t)16 * wp.R[rt] + lane, a.ydt, v);
        }
    } else {
        // every wavefront takes part in the shared activation tiles and their barriers; one
        // beyond the last row tile works on the last tile again and stores nothing
        if (!live) wp.R[0] = NR - 1;
#pragma unroll
        for (int rt = 1; rt < 4; ++rt) wp.R[rt] = (rt < RT && wp.R[0] + rt < NR) ? wp.R[0] + rt : wp.R[0];
        // second pass: the same positions one stretch of waves_of(MT) * RT row tiles further on
#pragma unroll
        for (int rt = 0; rt < 4; ++rt) {
            const int r2 = wp.R[0] + RT * waves_of(MT) + rt;
            wp.Rn[rt] = (live && rt < RT && r2 < NR) ? r2 : wp.R[0];
        }
        constexpr int G = groups_of(MT);
        float4_t out[P][G][RT];
#pragma unroll
        for (int j = 0; j < P; ++j)
#pragma unroll
            for (int g = 0; g < G; ++g)
#pragma unroll
                for (int rt = 0; rt < RT; ++rt) out[j][g][rt] = float4_t{0, 0, 0, 0};
        run_batched<MT, DEPTH, P>(mt, wp, xs, xsc, cb_all[wave], out);
        if (!live) return;
        // D layout of the MFMA: lane (n, mg) holds batch rows 4 mg .. 4 mg + 3 (of its group) of output column n
#pragma unroll
        for (int j = 0; j < P; ++j)
#pragma unroll
            for (int rt = 0; rt < RT; ++rt) {
                const int R = j == 0 ? wp.R[rt] : wp.Rn[rt];
                if ((j > 0 || rt > 0) && R == wp.R[0]) continue;
                const int n = 16 * R + (lane & 15);
#pragma unroll
                for (int g = 0; g < G; ++g)
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const int m = 16 * g + 4 * (lane >> 4) + i;
                        if (m < M) store_from_f32(mt.y, (size_t)m * mt.N + n, a.ydt, out[j][g][rt][i]);
                    }
            }
    }
}

// Batch 1 when a launch holds too few row tiles to fill the device (a single projection, the
// matrices of one stage of a block): one workgroup per 16-row tile, its S wavefronts take the
// column tiles s, s + S, s + 2S, ... and their partial sums meet in LDS in a fixed order.  The
// grouped kernel above gives one wavefront a whole row tile, which keeps 4096 x 4096 on a quarter
// of the SIMDs.
template <int S, class Args, bool GRID2D>
__global__ void __launch_bounds__(64 * S) decode_splitk_kernel(Args a) {
    constexpr int DEPTH = RWKVQ_DECODE_DEPTH;
    constexpr bool MIXED = Args::kMixed;
    static_assert(kRT == 1, "one row tile per wavefront");
    __shared__ __attribute__((aligned(1024))) uint32_t cb_all[S][256];
    __shared__ uint32_t cb_mix[MIXED ? S : 1][256];
    __shared__ float red[S][16];
    // Which matrix, which row tile?  A launch of a few matrices (a stage of a block) is a two-dimensional grid,
    // blockIdx.y the matrix and blockIdx.x the row tile (workgroups past a shorter matrix's last tile leave at once):
    // the descriptor is then one load away.  The table of first-workgroup indices of the other form costs a load of
    // its own in front of it, and these launches last three or four trips to memory in all.
    int mi = 0, tile;
    if constexpr (GRID2D) {
        mi = blockIdx.y;
        tile = blockIdx.x;
    } else {
        const int wg = blockIdx.x;
#pragma unroll
        for (int j = 0; j < Args::kMats; j += 64)
            mi += __builtin_popcountll(__builtin_amdgcn_ballot_w64(wg >= a.wg_end[j + (threadIdx.x & 63)]));
        tile = wg - (mi ? a.wg_end[mi - 1] : 0);                                   // here wg_end counts row tiles
    }
    const int xdt = a.xdt, ydt = a.ydt;    // the end of the argument block: asked for together with the descriptor
    const auto mt = a.m[mi];
    asm volatile("" :: "s"(xdt), "s"(ydt), "s"(mt.N));
    if (GRID2D && tile >= ((mt.N + 15) >> 4)) return;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int KT = mt.K >> 8;
    WavePos wp;
    wp.R[0] = wp.R[1] = wp.R[2] = wp.R[3] = tile;
    wp.M = 1; wp.lane = lane; wp.tid = threadIdx.x; wp.xbf16 = xdt == DT_BF16;
    wp.t0 = wave; wp.ts = S; wp.nt = wave < KT ? (KT - wave + S - 1) / S : 0;
    if constexpr (MIXED) {
        for (int e = lane; e < mt.mix_E; e += 64) cb_mix[wave][e] = mt.mix_cb[e];
        wave_lds_sync();
        wp.xprev = mt.xprev; wp.mix_idx = mt.mix_idx; wp.mix_cb = cb_mix[wave];
    }
    PostMixPre pre{};
    if constexpr (Args::kPostMix) {
        if (wave == 0 && lane < 16) post_mix_prefetch(pre, mt, (size_t)16 * wp.R[0] + lane, ydt);
    } else {
        if (wave == 0 && lane < 16 && mt.post == POST_SIGMOID_GATE) pre.gate = load_bits(mt.gate, (size_t)16 * wp.R[0] + lane, ydt);
    }
    float part[kRT] = {0.f};
    if (wp.nt > 0) {
        run_m1<DEPTH, true, MIXED>(mt, wp, cb_all[wave], part);
    }
    float v = part[0];                             // sum the four column groups of each row
    v += __shfl_xor(v, 16, 64);
    v += __shfl_xor(v, 32, 64);
    if (lane < 16) red[wave][lane] = v;
    __syncthreads();
    if (wave == 0 && lane < 16) {
        float t = red[0][lane];
#pragma unroll
        for (int s = 1; s < S; ++s) t += red[s][lane];
        if constexpr (Args::kPostMix) store_post_mix(mt, (size_t)16 * wp.R[0] + lane, ydt, t, pre);
        else store_post(mt, (size_t)16 * wp.R[0] + lane, ydt, t, true, pre.gate);
    }
}

// Batch 2..16 when a launch holds too few rows to fill the device with the kernel above (a single projection, the
// matrices of one stage of a block): one workgroup per 32 rows of W (two 16-row tiles, which share every activation
// fragment), its S wavefronts take the column tiles s, s + S, ...; each fetches its activation fragments itself
// (from the L2: every workgroup reads all of x, which is why this form is for small launches only), nothing is
// staged for the workgroup and no barrier sits in the tile loop; the partial sums meet in LDS in a fixed order.
template <int MT, int S, bool GRID2D>
__global__ void __launch_bounds__(64 * S, 1) decode_splitk_batched_kernel(DecodeArgs a) {
    static_assert(MT == 16 || MT == 32, "one or two groups of sixteen batch rows");
    constexpr int G = groups_of(MT);
    __shared__ __attribute__((aligned(1024))) uint32_t cb_all[S][512];
    __shared__ __attribute__((aligned(16))) float xsc[S][2 * 16 * G];
    __shared__ __attribute__((aligned(16))) float red[S][G][kBRT][256];
    // matrix and stretch of rows: from a two-dimensional grid (launches of at most kGrid2DMaxMats matrices, see
    // decode_splitk_kernel) or from the table of first workgroups
    int mi = 0, stretch;
    if constexpr (GRID2D) {
        mi = blockIdx.y;
        stretch = blockIdx.x;
    } else {
        const int wg = blockIdx.x;
#pragma unroll
        for (int j = 0; j < kMaxGroupMats; j += 64)
            mi += __builtin_popcountll(__builtin_amdgcn_ballot_w64(wg >= a.wg_end[j + (threadIdx.x & 63)]));
        stretch = wg - (mi ? a.wg_end[mi - 1] : 0);                // here wg_end counts stretches of kBRT row tiles
    }
    const int M = a.M, xdt = a.xdt, ydt = a.ydt;                   // the end of the argument block: asked for with the descriptor
    const DecodeMat mt = a.m[mi];
    asm volatile("" :: "s"(M), "s"(xdt), "s"(ydt), "s"(mt.N));
    if (GRID2D && stretch >= (mt.N + 16 * kBRT - 1) / (16 * kBRT)) return;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int KT = mt.K >> 8, NR = mt.N >> 4;
    WavePos wp;
    wp.R[0] = kBRT * stretch;
#pragma unroll
    for (int rt = 1; rt < 4; ++rt) wp.R[rt] = (rt < kBRT && wp.R[0] + rt < NR) ? wp.R[0] + rt : wp.R[0];
#pragma unroll
    for (int rt = 0; rt < 4; ++rt) wp.Rn[rt] = wp.R[0];
    wp.M = M; wp.lane = lane; wp.tid = threadIdx.x; wp.xbf16 = xdt == DT_BF16;
    wp.t0 = wave; wp.ts = S; wp.nt = wave < KT ? (KT - wave + S - 1) / S : 0;
    float4_t out[1][G][kBRT];
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
        for (int rt = 0; rt < kBRT; ++rt) out[0][g][rt] = float4_t{0, 0, 0, 0};
    if (wp.nt > 0) run_batched<MT, 1, 1, true>(mt, wp, nullptr, xsc[wave], cb_all[wave], out);
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
        for (int rt = 0; rt < kBRT; ++rt) *(float4_t*)&red[wave][g][rt][4 * lane] = out[0][g][rt];
    __syncthreads();
    // D layout of the MFMA: lane (n, mg) holds batch rows 4 mg .. 4 mg + 3 (of its group) of output column n;
    // wavefront rt sums row tile rt
    static_assert(kBRT <= 2, "the wavefront that sums row tile rt is picked with a select, not an index");
    const int Rw = wave == 0 ? wp.R[0] : wp.R[1];
    if (wave < kBRT && (wave == 0 || Rw != wp.R[0])) {
        const int n = 16 * Rw + (lane & 15);
#pragma unroll
        for (int g = 0; g < G; ++g) {
            float4_t t = *(const float4_t*)&red[0][g][wave & 1][4 * lane];
#pragma unroll
            for (int s = 1; s < S; ++s) {
                const float4_t v = *(const float4_t*)&red[s][g][wave & 1][4 * lane];
#pragma unroll
                for (int i = 0; i < 4; ++i) t[i] += v[i];
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int m = 16 * g + 4 * (lane >> 4) + i;
                if (m < M) store_from_f32(mt.y, (size_t)m * mt.N + n, ydt, t[i]);
            }
        }
    }
}


// Time mixing's r, k, v and the wkv step in one launch.  The recurrence is per channel, and channel c
// needs r[c], k[c], v[c]: output row c of three matrices.  A workgroup of 12 wavefronts takes row tile R
// of all three (four wavefronts per matrix, the column tiles dealt as in the split-K kernel with S = 4,
// the same order of summation), and the 16 lanes that hold the tile's sums step the recurrence for
// channels 16 R .. 16 R + 15 and store sigma(r) wkv, the vector W_o multiplies: no launch and no pass
// over memory between the projections and the recurrence, and every channel's state is touched by
// exactly one lane.  Arithmetic and bits as rwkvq_linear_dispatch on the three matrices followed by
// rwkvq_wkv (the projections are rounded to the output type before they enter the recurrence, as
// they would be read back).
struct WkvFuseArgs {
    DecodeMat m[3];
    const float* w; const float* u; float* state; void* out;
    int d, xdt, ydt, pad;
};
__global__ void __launch_bounds__(768) decode_rkv_wkv_kernel(WkvFuseArgs a) {
    constexpr int DEPTH = RWKVQ_DECODE_DEPTH, S = 4;
    __shared__ __attribute__((aligned(1024))) uint32_t cb_all[3 * S][256];
    __shared__ float red[3 * S][16];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int mi = wave >> 2, s = wave & 3;
    const DecodeMat mt = mi == 0 ? a.m[0] : mi == 1 ? a.m[1] : a.m[2];
    const int xdt = a.xdt;
    // the descriptor, the types and the recurrence's pointers sit in four cache lines of the argument block: all asked
    // for before the first wait (one after the other each is a trip of its own at the start of a kernel that lasts 8 us)
    asm volatile("" :: "s"(mt.codes), "s"(mt.K), "s"(xdt), "s"(a.state), "s"(a.d));
    const int KT = mt.K >> 8;
    WavePos wp;
    wp.R[0] = wp.R[1] = wp.R[2] = wp.R[3] = blockIdx.x;
    wp.M = 1; wp.lane = lane; wp.tid = threadIdx.x; wp.xbf16 = xdt == DT_BF16;
    wp.t0 = s; wp.ts = S; wp.nt = s < KT ? (KT - s + S - 1) / S : 0;
    wp.xprev = nullptr; wp.mix_idx = nullptr; wp.mix_cb = nullptr;
    // the recurrence's operands for this tile's channels: fetched now, used after the GEMV
    const size_t c = (size_t)16 * blockIdx.x + (lane & 15);
    float sa = 0.f, sb = 0.f, sp = 0.f, wc = 0.f, uc = 0.f;
    if (wave == 0 && lane < 16) {
        sa = a.state[c]; sb = a.state[(size_t)a.d + c]; sp = a.state[2 * (size_t)a.d + c];
        wc = a.w[c]; uc = a.u[c];
    }
    float part[kRT] = {0.f};
    if (wp.nt > 0) {
        run_m1<DEPTH, true, false>(mt, wp, cb_all[wave], part);
    }
    float v = part[0];                             // sum the four column groups of each row
    v += __shfl_xor(v, 16, 64);
    v += __shfl_xor(v, 32, 64);
    if (lane < 16) red[wave][lane] = v;
    __syncthreads();
    if (wave == 0 && lane < 16) {
        float y[3];
#pragma unroll
        for (int m = 0; m < 3; ++m) {
            float t = red[S * m][lane];
#pragma unroll
            for (int j = 1; j < S; ++j) t += red[S * m + j][lane];
            store_from_f32(m == 0 ? a.m[0].y : m == 1 ? a.m[1].y : a.m[2].y, c, a.ydt, t);
            y[m] = a.ydt == DT_F16 ? f16_bits_to_f32(f32_to_f16_bits(t)) : bf16_bits_to_f32(f32_to_bf16_bits(t));
        }
        store_from_f32(a.out, c, a.ydt, gate_f32(y[0], wkv_out(sa, sb, sp, uc, y[1], y[2])));
        wkv_advance(sa, sb, sp, wc, y[1], y[2]);
        a.state[c] = sa; a.state[(size_t)a.d + c] = sb; a.state[2 * (size_t)a.d + c] = sp;
    }
}

hipError_t launch_decode_rkv_wkv(const MatDev* rkv, const WkvDev& wkv, int x_dtype, int y_dtype, hipStream_t s) {
    WkvFuseArgs a;
    for (int i = 0; i < 3; ++i)
        a.m[i] = DecodeMat{rkv[i].codes, rkv[i].aux, rkv[i].x, rkv[i].y, rkv[i].N, rkv[i].K, rkv[i].fmt, POST_NONE, nullptr};
    a.w = wkv.w; a.u = wkv.u; a.state = wkv.state; a.out = wkv.out;
    a.d = rkv[0].N; a.xdt = x_dtype; a.ydt = y_dtype; a.pad = 0;
    hipLaunchKernelGGL(decode_rkv_wkv_kernel, dim3(rkv[0].N / 16), dim3(768), 0, s, a);
    return hipGetLastError();
}

// Smallest S of 4, 8, 16 that brings `tiles` row tiles to kSplitTarget wavefronts.
static int pick_split(int tiles) { return tiles * 4 >= kSplitTarget ? 4 : tiles * 8 >= kSplitTarget ? 8 : 16; }

// n_mats <= kGrid2DMaxMats: grid (longest matrix's row tiles, matrices); else one row of `wgs` workgroups and the table
template <class Args>
static hipError_t launch_splitk(int split, int wgs, Args& a, int n_mats, hipStream_t s) {
    a.pad = 0;
    if (n_mats <= kGrid2DMaxMats && option(RWKVQ_OPT_SPLIT_GRID_2D) == 1) {
        int longest = 0;
        for (int i = 0; i < n_mats; ++i) longest = std::max(longest, a.wg_end[i] - (i ? a.wg_end[i - 1] : 0));
        const dim3 grid(longest, n_mats);
        if (split == 4) hipLaunchKernelGGL((decode_splitk_kernel<4, Args, true>), grid, dim3(256), 0, s, a);
        else if (split == 8) hipLaunchKernelGGL((decode_splitk_kernel<8, Args, true>), grid, dim3(512), 0, s, a);
        else hipLaunchKernelGGL((decode_splitk_kernel<16, Args, true>), grid, dim3(1024), 0, s, a);
        return hipGetLastError();
    }
    const dim3 grid(wgs);
    if (split == 4) hipLaunchKernelGGL((decode_splitk_kernel<4, Args, false>), grid, dim3(256), 0, s, a);
    else if (split == 8) hipLaunchKernelGGL((decode_splitk_kernel<8, Args, false>), grid, dim3(512), 0, s, a);
    else hipLaunchKernelGGL((decode_splitk_kernel<16, Args, false>), grid, dim3(1024), 0, s, a);
    return hipGetLastError();
}

// Batch 1 with the token-shift mix fused into the activation load: always the split-K kernel
// (these are the stages of a block; 64 matrices per launch).
hipError_t launch_decode_mixed(const MatDev* mats, const MixDev* mixes, int n_mats, int x_dtype, int y_dtype,
                               hipStream_t s, const PostDev* posts) {
    for (int base = 0; base < n_mats; base += kMaxMixedMats) {
        MixedDecodeArgs a;
        const int cnt = n_mats - base < kMaxMixedMats ? n_mats - base : kMaxMixedMats;
        int tiles = 0;
        for (int i = 0; i < cnt; ++i) tiles += (mats[base + i].N + 15) / 16;
        int wgs = 0;
        for (int i = 0; i < kMaxMixedMats; ++i) {
            if (i < cnt) {
                const MatDev& m = mats[base + i];
                const MixDev& x = mixes[base + i];
                wgs += (m.N + 15) / 16;
                MixedMat mm;
                mm.codes = m.codes; mm.aux = m.aux; mm.x = m.x; mm.y = m.y; mm.N = m.N; mm.K = m.K; mm.fmt = m.fmt;
                mm.post = posts ? posts[base + i].op : POST_NONE; mm.gate = posts ? posts[base + i].gate : nullptr;
                mm.xprev = (const uint16_t*)x.x_prev; mm.mix_idx = x.idx; mm.mix_cb = (const uint32_t*)x.cb; mm.mix_E = x.E; mm.pad2 = 0;
                a.m[i] = mm;
                a.wg_end[i] = wgs;
            } else {
                a.m[i] = MixedMat{};
                a.wg_end[i] = 0x7FFFFFFF;
            }
        }
        a.M = 1; a.xdt = x_dtype; a.ydt = y_dtype; a.pad = 0;
        hipError_t e = launch_splitk(pick_split(tiles), wgs, a, cnt, s);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

// Batch 1 with the outputs also leaving as the mixes of the next stage: the split-K kernel (these are
// single projections of a block).
hipError_t launch_decode_postmix(const MatDev* mats, const PostDev* posts, const PostMixDev* pm, int n_mats,
                                 int x_dtype, int y_dtype, hipStream_t s) {
    for (int base = 0; base < n_mats; base += kMaxMixedMats) {
        PostMixArgs a;
        const int cnt = n_mats - base < kMaxMixedMats ? n_mats - base : kMaxMixedMats;
        int tiles = 0;
        for (int i = 0; i < cnt; ++i) tiles += (mats[base + i].N + 15) / 16;
        int wgs = 0;
        for (int i = 0; i < kMaxMixedMats; ++i) {
            PostMixMat mm{};
            if (i < cnt) {
                const MatDev& m = mats[base + i];
                const PostMixDev& x = pm[base + i];
                wgs += (m.N + 15) / 16;
                mm.codes = m.codes; mm.aux = m.aux; mm.x = m.x; mm.y = m.y; mm.N = m.N; mm.K = m.K; mm.fmt = m.fmt;
                mm.post = posts[base + i].op; mm.gate = posts[base + i].gate;
                mm.xprev = x.x_prev; mm.n_mix = x.n_mix; mm.pad2 = 0;
                for (int p = 0; p < 4; ++p)
                    mm.mix[p] = p < x.n_mix ? PostMix{x.idx[p], (const uint32_t*)x.cb[p], x.out[p]} : PostMix{nullptr, nullptr, nullptr};
                a.wg_end[i] = wgs;
            } else {
                a.wg_end[i] = 0x7FFFFFFF;
            }
            a.m[i] = mm;
        }
        a.M = 1; a.xdt = x_dtype; a.ydt = y_dtype; a.pad = 0;
        hipError_t e = launch_splitk(pick_split(tiles), wgs, a, cnt, s);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t launch_decode(const MatDev* mats, int n_mats, int M, int x_dtype, int y_dtype, hipStream_t s,
                         const PostDev* posts) {
    for (int base = 0; base < n_mats; base += kMaxGroupMats) {
        DecodeArgs a;
        int cnt = n_mats - base < kMaxGroupMats ? n_mats - base : kMaxGroupMats;
        // Workgroups are handed out in index order and a workgroup's running time grows with K:
        // the matrices of a launch go longest rows first, so that the launch does not end on a
        // few long workgroups (the outputs are independent, the order is free).
        int order[kMaxGroupMats];
        for (int i = 0; i < cnt; ++i) order[i] = base + i;
        std::stable_sort(order, order + cnt, [&](int p, int q) { return mats[p].K > mats[q].K; });
        // Batch 1 with fewer row tiles than two per SIMD: split the columns over S wavefronts of a
        // workgroup (one workgroup per row tile), S the smallest of 4, 8, 16 that reaches that count
        // (measured on the stages of a 7B block: 2048 beats 1024 and 4096 by 3-8 %, 16384 loses 40 %).
        int tiles = 0;
        for (int i = 0; i < cnt; ++i) tiles += (mats[order[i]].N + 15) / 16;
        int split = 0;
        if (M == 1 && tiles < kSplitTarget) split = pick_split(tiles);
        // batch 2..32 with few rows in the launch: one workgroup per 32 rows, S wavefronts over its column tiles
        if (M > 1 && M <= 32) {
            long long stretches = 0;
            for (int i = 0; i < cnt; ++i) stretches += (mats[order[i]].N + 16 * kBRT - 1) / (16 * kBRT);
            // measured on the RWKV-6-7B shapes: the form wins up to about 2000 stretches at batch 16 and 3500 at batch <= 8
            // (what it pays is every workgroup's own read of x, which grows with the batch)
            // (above batch 16 a workgroup carries two groups of fragments and the row-workgroup form catches up at a
            // third of that: one 4096-row matrix still gains 25-35 %, the two 14336-row matrices of channel mixing lose)
            const long long max_work = option(RWKVQ_OPT_STREAM_SPLIT_MAX_WORK);
            if (stretches * (16 + M) <= (M <= 16 || max_work >= 1000000 ? max_work : max_work / 3)) {
                const int S = stretches * 8 >= kSplitTarget ? 4 : 8;      // sixteen wavefronts would leave 128 registers each
                int wgs = 0;
                for (int i = 0; i < cnt; ++i) {
                    const MatDev& m = mats[order[i]];
                    wgs += (m.N + 16 * kBRT - 1) / (16 * kBRT);
                    a.m[i] = DecodeMat{m.codes, m.aux, m.x, m.y, m.N, m.K, m.fmt, POST_NONE, nullptr};
                    a.wg_end[i] = wgs;
                }
                for (int i = cnt; i < kMaxGroupMats; ++i) {
                    a.m[i] = DecodeMat{nullptr, nullptr, nullptr, nullptr, 0, 0, 0, POST_NONE, nullptr};
                    a.wg_end[i] = 0x7FFFFFFF;
                }
                a.M = M; a.xdt = x_dtype; a.ydt = y_dtype; a.pad = 0;
                if (cnt <= kGrid2DMaxMats && option(RWKVQ_OPT_SPLIT_GRID_2D) == 1) {
                    int longest = 0;
                    for (int i = 0; i < cnt; ++i) longest = std::max(longest, a.wg_end[i] - (i ? a.wg_end[i - 1] : 0));
                    const dim3 grid(longest, cnt);
                    if (M <= 16 && S == 4) hipLaunchKernelGGL((decode_splitk_batched_kernel<16, 4, true>), grid, dim3(256), 0, s, a);
                    else if (M <= 16) hipLaunchKernelGGL((decode_splitk_batched_kernel<16, 8, true>), grid, dim3(512), 0, s, a);
                    else if (S == 4) hipLaunchKernelGGL((decode_splitk_batched_kernel<32, 4, true>), grid, dim3(256), 0, s, a);
                    else hipLaunchKernelGGL((decode_splitk_batched_kernel<32, 8, true>), grid, dim3(512), 0, s, a);
                } else if (M <= 16 && S == 4) hipLaunchKernelGGL((decode_splitk_batched_kernel<16, 4, false>), dim3(wgs), dim3(256), 0, s, a);
                else if (M <= 16) hipLaunchKernelGGL((decode_splitk_batched_kernel<16, 8, false>), dim3(wgs), dim3(512), 0, s, a);
                else if (S == 4) hipLaunchKernelGGL((decode_splitk_batched_kernel<32, 4, false>), dim3(wgs), dim3(256), 0, s, a);
                else hipLaunchKernelGGL((decode_splitk_batched_kernel<32, 8, false>), dim3(wgs), dim3(512), 0, s, a);
                hipError_t e = hipGetLastError();
                if (e != hipSuccess) return e;
                continue;
            }
        }
        // batch > 1: two row passes per workgroup if the launch keeps enough workgroups that way
        int passes = 1;
        if (M > 1) {
            long long wgs2 = 0;
            for (int i = 0; i < cnt; ++i) wgs2 += (mats[order[i]].N + wg_rows(M, 2) - 1) / wg_rows(M, 2);
            if (kTwoPassFits && wgs2 >= option(RWKVQ_OPT_STREAM_TWO_PASS_MIN_WGS)) passes = 2;
        }
        const int rows = wg_rows(M, passes);
        int wgs = 0;
        for (int i = 0; i < cnt; ++i) {
            const MatDev& m = mats[order[i]];
            wgs += split ? (m.N + 15) / 16 : (m.N + rows - 1) / rows;
            a.m[i] = DecodeMat{m.codes, m.aux, m.x, m.y, m.N, m.K, m.fmt, posts ? posts[order[i]].op : POST_NONE,
                               posts ? posts[order[i]].gate : nullptr};
            a.wg_end[i] = wgs;
        }
        for (int i = cnt; i < kMaxGroupMats; ++i) {
            a.m[i] = DecodeMat{nullptr, nullptr, nullptr, nullptr, 0, 0, 0, POST_NONE, nullptr};
            a.wg_end[i] = 0x7FFFFFFF;
        }
        a.M = M; a.xdt = x_dtype; a.ydt = y_dtype; a.pad = 0;
        const dim3 grid(wgs), wide(64 * kBW);
        if (split) { hipError_t e = launch_splitk(split, wgs, a, cnt, s); if (e != hipSuccess) return e; }
        else if (M == 1) hipLaunchKernelGGL(decode_kernel<1>, grid, dim3(256), 0, s, a);
        else if (M <= 4 && passes == 1) hipLaunchKernelGGL((decode_kernel<4, 1>), grid, wide, 0, s, a);
        else if (M <= 4) hipLaunchKernelGGL((decode_kernel<4, 2>), grid, wide, 0, s, a);
        else if (M <= 16 && passes == 1) hipLaunchKernelGGL((decode_kernel<16, 1>), grid, wide, 0, s, a);
        else if (M <= 16) hipLaunchKernelGGL((decode_kernel<16, 2>), grid, wide, 0, s, a);
        else if (passes == 1) hipLaunchKernelGGL((decode_kernel<32, 1>), grid, wide, 0, s, a);
        else hipLaunchKernelGGL((decode_kernel<32, 2>), grid, wide, 0, s, a);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace rwkvq
