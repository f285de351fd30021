// Matrix-core path for large batches (prefill): y[M][N] = x[M][K] * Deq(W)^T with tiles of W
// dequantized into LDS and multiplied by v_mfma_f32_16x16x32_{bf16,f16} in the type of x,
// binary32 accumulate.  Grouped launch: the tiles of several matrices (each SQ or VQ as its flag
// says, Sec. 3.1 Eq. "optimization goal") share one grid so that all compute units stay busy.
//
// What is fed to the multipliers: Deq(W) exactly as defined in Sec. 2.2 (SQ: (q - z) * s in
// binary32; VQ: the fp16 codebook entry) rounded once, to nearest even, to the type of x.
//
// Tiling: workgroup = 256 threads = 2 x 2 wavefronts, block tile 256 (m) x 256 (n) x 64 (k),
// wavefront tile 128 x 128 = 8 x 8 MFMA tiles (256 accumulator registers).  A second instance
// with 128 rows of x per workgroup (wavefront tile 64 x 128) serves launches that would otherwise
// leave compute units without a tile; the launcher picks per launch (pick_bm).  Both operand tiles
// live in LDS as 256 rows of 128 bytes (64 k), with the eight 16-byte chunks of a row stored at
// chunk ^ (row & 7), so that the 16-row fragment reads of the 16 x 16 x 32 MFMAs and the tile
// writes are free of bank conflicts without padding (the conflict counter reads zero).
//   * activations: copied global -> LDS by the load unit itself (global_load_lds_dwordx4), no
//     registers and no vector-ALU work; each lane fetches the chunk that belongs at its slot;
//   * weights: packed words are fetched once per 256 columns, unpacked by the vector ALU one
//     k-step ahead of the matrix cores, and written with 16-byte LDS stores.
// Two LDS buffers for W and three for x (two with 8-bit VQ); one workgroup barrier per k-step;
// waits on the load counter are placed by hand (the activations of step i + 2 are in flight during
// the MFMAs of step i).  The unpack and the copies are cut into micro-slices placed right behind
// individual MFMAs (see mma_step).
//
// Workgroup -> tile order: the m-tile index runs fastest, so workgroups that are dispatched
// round-robin over the 8 XCDs keep one slice of x (256 rows) per XCD L2 when there are 8 m-tiles.
#include "common.h"
#include "../../include/rwkvq.h"

#include <algorithm>
#include <atomic>
#include <vector>

namespace rwkvq {

constexpr int kPfMaxMats = 64;
constexpr int BM = 256, BN = 256;              // block tile; the k-step is 64 columns
constexpr int kRowBytes = 128;                 // 64 k * 2 B
constexpr int kTileBytes = 256 * kRowBytes;    // one operand tile (32 KB)
constexpr int kCb8Bytes = 1024;                // converted 8-bit-index codebook
// Activation tiles in LDS: three (the copy of a k-step is issued two k-steps ahead of its use, so
// that its round trip to the cache hides behind a whole k-step of MFMAs) except with 8-bit VQ,
// whose converted codebooks take the room of the third.
constexpr int x_buffers(int fmt) { return fmt == FMT_VQ8 ? 2 : 3; }
constexpr int pf_lds_bytes(int fmt) { return (2 + x_buffers(fmt)) * kTileBytes + (fmt == FMT_VQ8 ? 2 * kCb8Bytes : 0); }

struct PfMat {
    const uint32_t* codes;
    const uint16_t* aux;
    const void* x;
    void* y;
    int N, K, fmt, pad;
};
struct PfArgs {
    int wg_end[kPfMaxMats];
    PfMat m[kPfMaxMats];
    int M, ydt, m_tiles, pad;
};

// s_waitcnt immediates (gfx9 encoding): only the named counter is waited for.
#define RWKVQ_WAIT_VM0_LGKM0() __builtin_amdgcn_s_waitcnt(0x0070)   /* vmcnt(0) lgkmcnt(0) */
#define RWKVQ_WAIT_VM8_LGKM0() __builtin_amdgcn_s_waitcnt(0x0078)   /* vmcnt(8) lgkmcnt(0) */
#define RWKVQ_WAIT_VM4_LGKM0() __builtin_amdgcn_s_waitcnt(0x0074)   /* vmcnt(4) lgkmcnt(0) */
// Publish LDS writes (ds_write and load-unit copies) to the workgroup: the caller has waited for
// its own writes; the barrier orders them against the other wavefronts' reads.
#define RWKVQ_BARRIER() asm volatile("s_barrier" ::: "memory")

template <bool BF16> struct Elem;
template <> struct Elem<true> {
    // accumulate in place; the "a" constraint pins the accumulator to the AGPR half of the
    // register file (left to itself the allocator starts it in VGPRs and shuffles it all loop long)
    static __device__ __forceinline__ void mfma(uint4_t a, uint4_t b, float4_t& c) {
        asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(c) : "v"(a), "v"(b));
    }
    static __device__ __forceinline__ uint32_t pack(float lo, float hi) {   // v_cvt_pk_bf16_f32
        typedef __bf16 bf2 __attribute__((ext_vector_type(2)));
        bf2 v = {(__bf16)lo, (__bf16)hi};
        return __builtin_bit_cast(uint32_t, v);
    }
    static __device__ __forceinline__ uint32_t from_f16x2(uint32_t h) {
        half2_t v = __builtin_bit_cast(half2_t, h);
        return pack((float)v.x, (float)v.y);
    }
};
template <> struct Elem<false> {
    static __device__ __forceinline__ void mfma(uint4_t a, uint4_t b, float4_t& c) {
        asm volatile("v_mfma_f32_16x16x32_f16 %0, %1, %2, %0" : "+a"(c) : "v"(a), "v"(b));
    }
    static __device__ __forceinline__ uint32_t pack(float lo, float hi) {
        half2_t v = {(half_t)lo, (half_t)hi};
        return __builtin_bit_cast(uint32_t, v);
    }
    static __device__ __forceinline__ uint32_t from_f16x2(uint32_t h) { return h; }
};

// Field c (compile-time) of a native SQ unit.
template <int C>
__device__ __forceinline__ uint32_t sq_code(uint32_t w0, uint32_t w1, uint32_t w2) {
    constexpr int P = C >> 1, e = C & 1;
    if constexpr (P < 15) {
        uint32_t w = (P / 5 == 0) ? w0 : (P / 5 == 1) ? w1 : w2;
        return (w >> (1 + 3 * (P % 5) + 16 * e)) & 7u;
    } else {
        constexpr int b = 16 * e;
        return ((w0 >> b) & 1u) | (((w1 >> b) & 1u) << 1) | (((w2 >> b) & 1u) << 2);
    }
}
template <int P>
__device__ __forceinline__ uint32_t vq6_byteaddr(uint32_t w0, uint32_t w1, uint32_t w2) {
    if constexpr (P < 15) {
        uint32_t w = (P / 5 == 0) ? w0 : (P / 5 == 1) ? w1 : w2;
        return (w >> (6 * (P % 5))) & 0xFCu;
    } else {
        return ((w0 & 3u) << 2) | ((w1 & 3u) << 4) | ((w2 & 3u) << 6);
    }
}

// The two weights of pair P of a native SQ unit, dequantised as Sec. 2.2 Eq. "SQ" prescribes
// (q - z rounded, times s rounded).  The codes are not extracted: masked in place, a 3-bit code at
// mantissa bits b..b+2 of an fp16 half is the subnormal q * 2^(b-24); a mixed-precision FMA reads
// the half, multiplies by 2^(24-b) (exact) and subtracts z with the single rounding of q - z.  The
// codes at bits 10 and 13 of the halves come down to bits 1 and 4 with one shift by 9 per word.
template <int P>
__device__ __forceinline__ void sq_pair_deq(uint32_t w0, uint32_t w1, uint32_t w2, float s, float z, float& lo,
                                            float& hi) {
    uint32_t m;
    float c;
    if constexpr (P < 15) {
        constexpr int p = P % 5;
        const uint32_t w = (P / 5 == 0) ? w0 : (P / 5 == 1) ? w1 : w2;
        if constexpr (p == 0) { m = w & 0x000E000Eu; c = 8388608.f; }
        else if constexpr (p == 1) { m = w & 0x00700070u; c = 1048576.f; }
        else if constexpr (p == 2) { m = w & 0x03800380u; c = 131072.f; }
        else if constexpr (p == 3) { m = (w >> 9) & 0x000E000Eu; c = 8388608.f; }
        else { m = (w >> 9) & 0x00700070u; c = 1048576.f; }
    } else {
        // bit b of the pair's two codes sits at bits 0 and 16 of word b
        m = (w0 & 0x00010001u) | ((w1 & 0x00010001u) << 1) | ((w2 & 0x00010001u) << 2);
        c = 16777216.f;
    }
    const half2_t h = __builtin_bit_cast(half2_t, m);
    lo = __fmul_rn(fmaf((float)h.x, c, -z), s);
    hi = __fmul_rn(fmaf((float)h.y, c, -z), s);
}

// Eight consecutive-k weights (step T4 of a unit) of one lane, as four packed pairs.
template <bool BF16, int T4>
__device__ __forceinline__ uint4_t sq_chunk(uint32_t w0, uint32_t w1, uint32_t w2, float s, float z) {
    uint4_t o;
    float a, b;
    sq_pair_deq<4 * T4 + 0>(w0, w1, w2, s, z, a, b); o.x = Elem<BF16>::pack(a, b);
    sq_pair_deq<4 * T4 + 1>(w0, w1, w2, s, z, a, b); o.y = Elem<BF16>::pack(a, b);
    sq_pair_deq<4 * T4 + 2>(w0, w1, w2, s, z, a, b); o.z = Elem<BF16>::pack(a, b);
    sq_pair_deq<4 * T4 + 3>(w0, w1, w2, s, z, a, b); o.w = Elem<BF16>::pack(a, b);
    return o;
}
template <int T4>
__device__ __forceinline__ uint4_t vq6_chunk(uint32_t w0, uint32_t w1, uint32_t w2, uint32_t cb) {
    uint4_t o;
    o.x = __builtin_amdgcn_ds_bpermute(vq6_byteaddr<4 * T4 + 0>(w0, w1, w2), cb);
    o.y = __builtin_amdgcn_ds_bpermute(vq6_byteaddr<4 * T4 + 1>(w0, w1, w2), cb);
    o.z = __builtin_amdgcn_ds_bpermute(vq6_byteaddr<4 * T4 + 2>(w0, w1, w2), cb);
    o.w = __builtin_amdgcn_ds_bpermute(vq6_byteaddr<4 * T4 + 3>(w0, w1, w2), cb);
    return o;
}
__device__ __forceinline__ uint4_t vq8_chunk(uint32_t w, const uint32_t* cb) {
    uint4_t o = {cb[w & 255u], cb[(w >> 8) & 255u], cb[(w >> 16) & 255u], cb[w >> 24]};
    return o;
}

// Packed words of one 256-column tile for the 4 row tiles (of 16 rows) a thread unpacks.
template <int FMT> struct WRegs;
template <> struct WRegs<FMT_SQ3> { uint4_t a[4]; uint2_t b[4]; uint2_t sz[4]; };   // sz: (scale,zero) x 2 units
template <> struct WRegs<FMT_VQ6> { uint4_t a[4]; uint2_t b[4]; uint32_t cb; };     // cb: codebook entry `lane`
template <> struct WRegs<FMT_VQ8> { uint4_t a[4]; uint4_t b[4]; uint4_t cb8; };     // cb8: entries 4*lane..+3

// Where a wavefront finds its packed words: uniform tile pointers for its 4 row tiles.
struct WSrc {
    const uint32_t* rows[4];   // start of row tile R0 + 4*wave + i (advance by tile words per T)
    const uint16_t* aux;       // SQ: scale/zero of row tile R0 + 4*wave (16 uint2 per tile and T); VQ: codebooks of the block row
    int KT;
};

template <int FMT>
__device__ __forceinline__ void w_load(WRegs<FMT>& r, const WSrc& src, int T, int lane) {
    constexpr int tw = FMT == FMT_VQ8 ? 512 : 384;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint32_t* tile = src.rows[i] + (size_t)T * tw;
        r.a[i] = *(const uint4_t*)(tile + 4 * lane);
        if constexpr (FMT == FMT_VQ8) r.b[i] = *(const uint4_t*)(tile + 256 + 4 * lane);
        else r.b[i] = *(const uint2_t*)(tile + 256 + 2 * lane);
    }
    if constexpr (FMT == FMT_SQ3) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
            r.sz[i] = ((const uint2_t*)src.aux + ((size_t)i * src.KT + T) * 16)[lane & 15];
    } else if constexpr (FMT == FMT_VQ6) {
        r.cb = ((const uint32_t*)src.aux + (size_t)T * 64)[lane];
    } else {
        r.cb8 = ((const uint4_t*)src.aux + (size_t)T * 64)[lane];
    }
}

// LDS byte offset, inside a tile, of logical 16-byte chunk c (0..7) of row `row`.
__device__ __forceinline__ int tile_off(int row, int c) { return row * kRowBytes + ((c ^ (row & 7)) << 4); }

// Unpack k-step KQ (0..3: 64 columns) of the tile held in r and write it to the W tile in LDS.
// Row tiles I0 .. I1-1 of the thread's four (so that the work can be spread over a k-step).
template <bool BF16, int FMT, int KQ, int I0 = 0, int I1 = 4>
__device__ __forceinline__ void w_unpack(const WRegs<FMT>& r, char* wt, const uint32_t* cb8, int wave, int lane) {
    constexpr int u = KQ >> 1, t0 = 2 * (KQ & 1);
    const int row0 = 64 * wave + (lane & 15), kg = lane >> 4;
    // rows row0 + 16 i share row & 7, so the two chunk offsets are the same for all four
    char* d0 = wt + tile_off(row0, kg);
    char* d1 = wt + tile_off(row0, 4 + kg);
    if constexpr (FMT == FMT_SQ3) {
#pragma unroll
        for (int i = I0; i < I1; ++i) {
            const uint32_t w0 = u == 0 ? r.a[i].x : r.a[i].w, w1 = u == 0 ? r.a[i].y : r.b[i].x,
                           w2 = u == 0 ? r.a[i].z : r.b[i].y;
            const uint32_t szw = u == 0 ? r.sz[i].x : r.sz[i].y;
            const float s = f16_bits_to_f32((uint16_t)(szw & 0xFFFFu)), z = f16_bits_to_f32((uint16_t)(szw >> 16));
            *(uint4_t*)(d0 + 16 * i * kRowBytes) = sq_chunk<BF16, t0>(w0, w1, w2, s, z);
            *(uint4_t*)(d1 + 16 * i * kRowBytes) = sq_chunk<BF16, t0 + 1>(w0, w1, w2, s, z);
        }
    } else if constexpr (FMT == FMT_VQ6) {
        const uint32_t cb = Elem<BF16>::from_f16x2(r.cb);
#pragma unroll
        for (int i = I0; i < I1; ++i) {
            const uint32_t w0 = u == 0 ? r.a[i].x : r.a[i].w, w1 = u == 0 ? r.a[i].y : r.b[i].x,
                           w2 = u == 0 ? r.a[i].z : r.b[i].y;
            *(uint4_t*)(d0 + 16 * i * kRowBytes) = vq6_chunk<t0>(w0, w1, w2, cb);
            *(uint4_t*)(d1 + 16 * i * kRowBytes) = vq6_chunk<t0 + 1>(w0, w1, w2, cb);
        }
    } else {
#pragma unroll
        for (int i = I0; i < I1; ++i) {
            const uint32_t wa = u == 0 ? (t0 == 0 ? r.a[i].x : r.a[i].z) : (t0 == 0 ? r.b[i].x : r.b[i].z);
            const uint32_t wb = u == 0 ? (t0 == 0 ? r.a[i].y : r.a[i].w) : (t0 == 0 ? r.b[i].y : r.b[i].w);
            *(uint4_t*)(d0 + 16 * i * kRowBytes) = vq8_chunk(wa, cb8);
            *(uint4_t*)(d1 + 16 * i * kRowBytes) = vq8_chunk(wb, cb8);
        }
    }
}

// The same work cut into 128 micro-slices, one per MFMA of the previous k-step (see mma_step): a
// weight pair takes four of them (mask / address; subtract the zero point or start the look-up;
// scale; pack and, every fourth pair, store the finished 16-byte chunk).  Micro-slice S works on
// pair (S / 4) % 4 of chunk (S / 16) % 2 of row tile S / 32.  Each is two or three vector
// instructions: what the matrix core leaves room for behind one MFMA of the same wavefront.
template <int FMT> struct UnpackState {
    char *d0, *d1;            // LDS addresses of the lane's two chunks of row tile 0
    uint4_t stage;            // the chunk being assembled
    float s, z;               // SQ: scale and zero point of the current row tile and unit
    float lo, hi;             // SQ: the pair in flight
    uint32_t m;               // masked codes / look-up address / looked-up pair in flight
    uint32_t cb;              // VQ6: the lane's codebook entry, converted to the operand type
};

template <bool BF16, int FMT>
__device__ __forceinline__ void unpack_begin(UnpackState<FMT>& st, const WRegs<FMT>& r, char* wt, int wave, int lane) {
    const int row0 = 64 * wave + (lane & 15), kg = lane >> 4;
    st.d0 = wt + tile_off(row0, kg);
    st.d1 = wt + tile_off(row0, 4 + kg);
    if constexpr (FMT == FMT_VQ6) st.cb = Elem<BF16>::from_f16x2(r.cb);
}

// The SQ pair P as masked in-place codes (fp16 subnormals q * 2^(b-24)) and the power of two that
// undoes the position (see sq_pair_deq).
template <int P>
__device__ __forceinline__ uint32_t sq_pair_mask(uint32_t w0, uint32_t w1, uint32_t w2) {
    if constexpr (P < 15) {
        constexpr int p = P % 5;
        const uint32_t w = (P / 5 == 0) ? w0 : (P / 5 == 1) ? w1 : w2;
        if constexpr (p == 0) return w & 0x000E000Eu;
        else if constexpr (p == 1) return w & 0x00700070u;
        else if constexpr (p == 2) return w & 0x03800380u;
        else if constexpr (p == 3) return (w >> 9) & 0x000E000Eu;
        else return (w >> 9) & 0x00700070u;
    } else {
        return (w0 & 0x00010001u) | ((w1 & 0x00010001u) << 1) | ((w2 & 0x00010001u) << 2);
    }
}
template <int P> constexpr float sq_pair_unscale() {
    return P == 15 ? 16777216.f : (P % 5 == 0 || P % 5 == 3) ? 8388608.f : (P % 5 == 1 || P % 5 == 4) ? 1048576.f : 131072.f;
}

template <bool BF16, int FMT, int KQ, int S>
__device__ __forceinline__ void unpack_micro(UnpackState<FMT>& st, const WRegs<FMT>& r, const uint32_t* cb8) {
    constexpr int u = KQ >> 1, t0 = 2 * (KQ & 1);
    constexpr int i = S >> 5, c = (S >> 4) & 1, p = (S >> 2) & 3, q = S & 3, P = 4 * (t0 + c) + p;
    if constexpr (FMT == FMT_SQ3) {
        const uint32_t w0 = u == 0 ? r.a[i].x : r.a[i].w, w1 = u == 0 ? r.a[i].y : r.b[i].x,
                       w2 = u == 0 ? r.a[i].z : r.b[i].y;
        if constexpr (q == 0) {
            if constexpr ((S & 31) == 0) {
                const uint32_t szw = u == 0 ? r.sz[i].x : r.sz[i].y;
                st.s = f16_bits_to_f32((uint16_t)(szw & 0xFFFFu));
                st.z = f16_bits_to_f32((uint16_t)(szw >> 16));
            }
            st.m = sq_pair_mask<P>(w0, w1, w2);
        } else if constexpr (q == 1) {
            const half2_t h = __builtin_bit_cast(half2_t, st.m);
            st.lo = fmaf((float)h.x, sq_pair_unscale<P>(), -st.z);
            st.hi = fmaf((float)h.y, sq_pair_unscale<P>(), -st.z);
        } else if constexpr (q == 2) {
            st.lo = __fmul_rn(st.lo, st.s);
            st.hi = __fmul_rn(st.hi, st.s);
        } else {
            st.m = Elem<BF16>::pack(st.lo, st.hi);
        }
    } else if constexpr (FMT == FMT_VQ6) {
        const uint32_t w0 = u == 0 ? r.a[i].x : r.a[i].w, w1 = u == 0 ? r.a[i].y : r.b[i].x,
                       w2 = u == 0 ? r.a[i].z : r.b[i].y;
        if constexpr (q == 0) st.m = vq6_byteaddr<P>(w0, w1, w2);
        else if constexpr (q == 1) st.m = __builtin_amdgcn_ds_bpermute(st.m, st.cb);
    } else {
        const uint32_t wa = u == 0 ? (t0 == 0 ? r.a[i].x : r.a[i].z) : (t0 == 0 ? r.b[i].x : r.b[i].z);
        const uint32_t wb = u == 0 ? (t0 == 0 ? r.a[i].y : r.a[i].w) : (t0 == 0 ? r.b[i].y : r.b[i].w);
        const uint32_t w = c == 0 ? wa : wb;
        if constexpr (q == 0) st.m = (w >> (8 * p)) & 255u;
        else if constexpr (q == 1) st.m = cb8[st.m];
    }
    if constexpr (q == 3) {
        if constexpr (p == 0) st.stage.x = st.m;
        else if constexpr (p == 1) st.stage.y = st.m;
        else if constexpr (p == 2) st.stage.z = st.m;
        else {
            st.stage.w = st.m;
            *(uint4_t*)((c == 0 ? st.d0 : st.d1) + 16 * i * kRowBytes) = st.stage;
        }
    }
}

// Copy the activation tile, columns k0..k0+63 of the block's 256 rows, into an LDS tile, 16 bytes
// per lane and instruction, the load unit writing LDS directly.  LDS slot p (16 bytes) = row
// p/8, position p%8; the lane that owns slot p fetches the logical chunk the swizzle stores there.
// xoff[i] is the lane's byte offset (row * K * 2 + chunk * 16) from the tile's first row, computed
// once; xk = activations of the tile's first row at column k0 (uniform).
template <int I>
__device__ __forceinline__ void x_tile_dma_one(const char* xk, const uint32_t (&xoff)[8], char* xt, int wave) {
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(xk + xoff[I]),
                                     (__attribute__((address_space(3))) void*)(xt + (256 * I + 64 * wave) * 16),
                                     16, 0, 0);
}
template <int MF>
__device__ __forceinline__ void x_tile_dma(const char* xk, const uint32_t (&xoff)[8], char* xt, int wave) {
#pragma unroll
    for (int i = 0; i < MF; ++i)
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(xk + xoff[i]),
                                         (__attribute__((address_space(3))) void*)(xt + (256 * i + 64 * wave) * 16),
                                         16, 0, 0);
}

// One k-step (64 columns) of the wavefront tile = 16 rows of 8 MFMAs: x fragment f (f = 0..15:
// m-subtile f%8 of column half f/8) against the eight W fragments of that half.  x fragments are
// read kAhead rows ahead of their use and the W fragments of the second half during rows 4..7,
// so that an LDS round trip is hidden behind several rows of MFMAs.  `early` runs right after
// the first LDS reads have been issued and `mid` between the halves: vector-ALU work placed
// there (unpacking the next k-step) covers more latency.
constexpr int kAhead = 3;
template <int S> struct SliceTag { static constexpr int value = S; };

template <bool BF16, int MF, int F, int NI, class Slice>
__device__ __forceinline__ void mma_one(const uint4_t (&b)[8], const uint4_t af, float4_t (&acc)[MF][8], Slice& slice) {
    // One MFMA of x fragment F, then one micro-slice of vector-ALU work, fenced so that the
    // instruction scheduler leaves it there: a wavefront issues in order, and only the two or
    // three instructions placed right behind an MFMA run while the matrix core is busy with it
    // (left alone, the scheduler gathers the unpack work into long runs before its stores, and
    // the matrix core idles through them).
    Elem<BF16>::mfma(b[NI], af, acc[F % MF][NI]);
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (MF == 8) {
        slice(SliceTag<8 * F + NI>{});
    } else {                                       // half as many MFMAs per k-step: two micro-slices behind each
        slice(SliceTag<2 * (8 * F + NI)>{});
        slice(SliceTag<2 * (8 * F + NI) + 1>{});
    }
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (NI < 7) mma_one<BF16, MF, F, NI + 1>(b, af, acc, slice);
}
template <bool BF16, int MF, int F, class Slice>
__device__ __forceinline__ void mma_row(const uint4_t (&b)[8], const uint4_t af, float4_t (&acc)[MF][8], Slice& slice) {
    mma_one<BF16, MF, F, 0>(b, af, acc, slice);
}

template <bool BF16, int MF, int F, class Slice>
__device__ __forceinline__ void mma_rows(const char* const (&xa)[2], const char* wb1, uint4_t (&b)[8], uint4_t (&b1)[8],
                                         uint4_t (&a)[kAhead + 1], float4_t (&acc)[MF][8], Slice& slice) {
    if constexpr (F < 2 * MF) {
        if constexpr (F + kAhead < 2 * MF)
            a[(F + kAhead) % (kAhead + 1)] = *(const uint4_t*)(xa[(F + kAhead) / MF] + 16 * ((F + kAhead) % MF) * kRowBytes);
        if constexpr (F >= MF - 4 && F < MF) {                  // the last four rows of the first half
            constexpr int J = F - (MF - 4);
            b1[2 * J] = *(const uint4_t*)(wb1 + 16 * (2 * J) * kRowBytes);
            b1[2 * J + 1] = *(const uint4_t*)(wb1 + 16 * (2 * J + 1) * kRowBytes);
        }
        if constexpr (F < MF) mma_row<BF16, MF, F>(b, a[F % (kAhead + 1)], acc, slice);
        else mma_row<BF16, MF, F>(b1, a[F % (kAhead + 1)], acc, slice);
        mma_rows<BF16, MF, F + 1>(xa, wb1, b, b1, a, acc, slice);
    }
}

// One k-step (64 columns) of the wavefront tile = 16 rows of 8 MFMAs: x fragment f (f = 0..15:
// m-subtile f%8 of column half f/8) against the eight W fragments of that half.  x fragments are
// read kAhead rows ahead of their use and the W fragments of the second half during rows 4..7,
// so that an LDS round trip is hidden behind several rows of MFMAs.  `slice(SliceTag<S>)`, S =
// 0..127, is called after MFMA S: the unpacking of the next k-step goes there.
template <bool BF16, int MF, class Slice>
__device__ __forceinline__ void mma_step(const char* xt, const char* wt, int wm, int wn, int lane,
                                         float4_t (&acc)[MF][8], Slice slice) {
    const int r = lane & 15, kg = lane >> 4;
    const char* const xa[2] = {xt + tile_off(16 * MF * wm + r, kg), xt + tile_off(16 * MF * wm + r, 4 + kg)};
    const char* wb0 = wt + tile_off(128 * wn + r, kg);
    const char* wb1 = wt + tile_off(128 * wn + r, 4 + kg);
    uint4_t b[8], b1[8], a[kAhead + 1];
#pragma unroll
    for (int ni = 0; ni < 8; ++ni) b[ni] = *(const uint4_t*)(wb0 + 16 * ni * kRowBytes);
#pragma unroll
    for (int f = 0; f < kAhead; ++f) a[f] = *(const uint4_t*)(xa[0] + 16 * f * kRowBytes);
    mma_rows<BF16, MF, 0>(xa, wb1, b, b1, a, acc, slice);
}

// Convert and stage the 8-bit-index codebook of a tile (256 entries) into LDS.
template <bool BF16>
__device__ __forceinline__ void cb8_store(const WRegs<FMT_VQ8>& r, uint32_t* cb8, int wave, int lane) {
    if (wave == 0) {
        uint4_t c = {Elem<BF16>::from_f16x2(r.cb8.x), Elem<BF16>::from_f16x2(r.cb8.y),
                     Elem<BF16>::from_f16x2(r.cb8.z), Elem<BF16>::from_f16x2(r.cb8.w)};
        *(uint4_t*)(cb8 + 4 * lane) = c;
    }
}

// All matrices of one launch have the format FMT.  The k loop has no conditionals: past the last
// column tile the prefetches simply fetch the last tile again (never used).
// MF = 16-row m-subtiles per wavefront: 8 (block tile 256 x 256) or 4 (128 x 256, for launches that
// would leave compute units without a tile: the same W work per workgroup on half the MFMAs).
template <bool BF16, int FMT, int MF>
__global__ void __launch_bounds__(256, 1) prefill_kernel(PfArgs a) {
    constexpr int BMk = 32 * MF;                           // rows of x per workgroup
    extern __shared__ __attribute__((aligned(1024))) char lds[];
    constexpr int XB = x_buffers(FMT), LA = XB - 1;       // LA = k-steps between a copy and its use
    char* const wt0 = lds;
    char* const wt1 = lds + kTileBytes;
    char* const xbase = lds + 2 * kTileBytes;
    uint32_t* const cb8base = (uint32_t*)(lds + (2 + XB) * kTileBytes);
#define CB8(i) (cb8base + ((i) & 1) * (kCb8Bytes / 4))

    const int wg = blockIdx.x;
    static_assert(kPfMaxMats == 64, "one table entry per lane");
    const int mi_ = __builtin_popcountll(__builtin_amdgcn_ballot_w64(wg >= a.wg_end[threadIdx.x & 63]));
    const PfMat mt = a.m[mi_];
    const int local = wg - (mi_ ? a.wg_end[mi_ - 1] : 0);
    const int m0 = (local % a.m_tiles) * BMk, n0 = (local / a.m_tiles) * BN;
    const int M = a.M, K = mt.K, KT = K >> 8, R0 = n0 >> 4;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), wm = wave >> 1, wn = wave & 1;

    // per-lane activation offsets (rows past M repeat row M - 1)
    uint32_t xoff[8];
#pragma unroll
    for (int i = 0; i < MF; ++i) {
        const int p = 256 * i + 64 * wave + lane;
        const int row = p >> 3, c = (p & 7) ^ (row & 7);
        const int rr = m0 + row < M ? row : M - 1 - m0;
        xoff[i] = (uint32_t)rr * (uint32_t)K * 2u + 16u * c;
    }
    const char* xrow0 = (const char*)mt.x + (size_t)m0 * K * 2;

    WSrc src;
    constexpr int tw = FMT == FMT_VQ8 ? 512 : 384;
#pragma unroll
    for (int i = 0; i < 4; ++i) src.rows[i] = mt.codes + (size_t)(R0 + 4 * wave + i) * KT * tw;
    src.KT = KT;
    if constexpr (FMT == FMT_SQ3) src.aux = (const uint16_t*)((const uint2_t*)mt.aux + (size_t)(R0 + 4 * wave) * KT * 16);
    else if constexpr (FMT == FMT_VQ6) src.aux = (const uint16_t*)((const uint32_t*)mt.aux + (size_t)(R0 >> 4) * KT * 64);
    else src.aux = (const uint16_t*)((const uint4_t*)mt.aux + (size_t)(R0 >> 4) * KT * 64);

    float4_t acc[MF][8];
#pragma unroll
    for (int i = 0; i < MF; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[i][j] = float4_t{0, 0, 0, 0};

    // The activation buffers form a ring (byte offsets from xbase): x0 holds the k-step being
    // multiplied, x1 the next one, x2 (three buffers) the one after.  A k-step's copy is issued LA
    // k-steps ahead; eight copy instructions per thread and k-step, so "all but the newest eight
    // memory operations done" is the wait that lets the newest copy stay in flight.
    int x0 = 0, x1 = kTileBytes, x2 = 2 * kTileBytes;
    const int hmax = 4 * KT - 1;                           // last k-step
    auto xk = [&](int h) { return xrow0 + (size_t)(h < hmax ? h : hmax) * kRowBytes; };
    auto rotate = [&] { if (XB == 3) { const int t = x0; x0 = x1; x1 = x2; x2 = t; } else { const int t = x0; x0 = x1; x1 = t; } };
    auto wait_step = [&] {                                 // all but the newest copy (MF instructions per thread)
        if (LA == 2) { if (MF == 8) RWKVQ_WAIT_VM8_LGKM0(); else RWKVQ_WAIT_VM4_LGKM0(); }
        else RWKVQ_WAIT_VM0_LGKM0();
    };

    // prologue: packed words of tile 0, k-step 0 (and 1) of the activations, k-step 0 of W
    WRegs<FMT> wr;
    UnpackState<FMT> us;
    w_load<FMT>(wr, src, 0, lane);
    x_tile_dma<MF>(xk(0), xoff, xbase + x0, wave);
    if (LA == 2) x_tile_dma<MF>(xk(1), xoff, xbase + x1, wave);
    if constexpr (FMT == FMT_VQ8) {
        cb8_store<BF16>(wr, CB8(0), wave, lane);
        RWKVQ_WAIT_VM0_LGKM0();
        RWKVQ_BARRIER();
    }
    w_unpack<BF16, FMT, 0>(wr, wt0, CB8(0), wave, lane);
    RWKVQ_WAIT_VM0_LGKM0();
    RWKVQ_BARRIER();

    for (int T = 0; T < KT; ++T) {
        const int Tn = T + 1 < KT ? T + 1 : T;
        const int g = 4 * T;                               // k-step index of the tile's first step
        // k-step 0 of the tile is in W buffer 0; steps 1..3 come from the same packed words and are
        // unpacked, a few instructions at a time, behind the MFMAs of the step before; the eight
        // copy instructions of the activation tile LA steps ahead go behind MFMAs as well.
        {
            const char* xsrc = xk(g + LA);
            char* xdst = xbase + (LA == 2 ? x2 : x1);
            unpack_begin<BF16, FMT>(us, wr, wt1, wave, lane);
            mma_step<BF16, MF>(xbase + x0, wt0, wm, wn, lane, acc, [&](auto tag) {
                constexpr int S = decltype(tag)::value;
                if constexpr (S % 8 == 4 && S / 8 < MF) x_tile_dma_one<S / 8>(xsrc, xoff, xdst, wave);
                unpack_micro<BF16, FMT, 1, S>(us, wr, CB8(T));
            });
        }
        wait_step();
        RWKVQ_BARRIER();
        rotate();

        {
            const char* xsrc = xk(g + 1 + LA);
            char* xdst = xbase + (LA == 2 ? x2 : x1);
            unpack_begin<BF16, FMT>(us, wr, wt0, wave, lane);
            mma_step<BF16, MF>(xbase + x0, wt1, wm, wn, lane, acc, [&](auto tag) {
                constexpr int S = decltype(tag)::value;
                if constexpr (S % 8 == 4 && S / 8 < MF) x_tile_dma_one<S / 8>(xsrc, xoff, xdst, wave);
                unpack_micro<BF16, FMT, 2, S>(us, wr, CB8(T));
            });
        }
        wait_step();
        RWKVQ_BARRIER();
        rotate();

        {
            const char* xsrc = xk(g + 2 + LA);
            char* xdst = xbase + (LA == 2 ? x2 : x1);
            unpack_begin<BF16, FMT>(us, wr, wt1, wave, lane);
            mma_step<BF16, MF>(xbase + x0, wt0, wm, wn, lane, acc, [&](auto tag) {
                constexpr int S = decltype(tag)::value;
                if constexpr (S % 8 == 4 && S / 8 < MF) x_tile_dma_one<S / 8>(xsrc, xoff, xdst, wave);
                unpack_micro<BF16, FMT, 3, S>(us, wr, CB8(T));
            });
        }
        wait_step();
        RWKVQ_BARRIER();
        rotate();

        // the packed words of this tile are spent: fetch the next tile's into the same registers
        // (before the activation copy, so that waiting for them leaves the copy in flight); they
        // have a whole MFMA step to arrive
        w_load<FMT>(wr, src, Tn, lane);
        {
            const char* xsrc = xk(g + 3 + LA);
            char* xdst = xbase + (LA == 2 ? x2 : x1);
            mma_step<BF16, MF>(xbase + x0, wt1, wm, wn, lane, acc, [&](auto tag) {
                constexpr int S = decltype(tag)::value;
                if constexpr (S % 8 == 4 && S / 8 < MF) x_tile_dma_one<S / 8>(xsrc, xoff, xdst, wave);
            });
        }
        if constexpr (FMT == FMT_VQ8) {
            cb8_store<BF16>(wr, CB8(T + 1), wave, lane);
            RWKVQ_WAIT_VM0_LGKM0();
            RWKVQ_BARRIER();
        } else {
            wait_step();                                   // the packed words have landed
        }
        w_unpack<BF16, FMT, 0>(wr, wt0, CB8(T + 1), wave, lane);
        wait_step();
        RWKVQ_BARRIER();
        rotate();
    }

    // The MFMAs are opaque to the compiler's hazard checks: let the last ones drain before the
    // accumulators are read (the longest MFMA-to-read hazard is well under 32 cycles).
    asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");

    // epilogue: the W fragment is the A operand of the MFMA, so a lane holds, for every 16 x 16
    // tile, output row m = lane%16 and the four consecutive columns n = 4*(lane/16) + 0..3:
    // one 8-byte (or 16-byte for fp32) store per tile.
    const int N = mt.N;
#pragma unroll
    for (int mi = 0; mi < MF; ++mi) {
        const int m = m0 + 16 * MF * wm + 16 * mi + (lane & 15);
        if (m < M) {
#pragma unroll
            for (int ni = 0; ni < 8; ++ni) {
                const size_t o = (size_t)m * N + n0 + 128 * wn + 16 * ni + 4 * (lane >> 4);
                const float4_t v = acc[mi][ni];
                if (a.ydt == DT_F32) {
                    *(float4_t*)((float*)mt.y + o) = v;
                } else {
                    uint2_t pk;
                    if (a.ydt == DT_BF16) { pk.x = Elem<true>::pack(v[0], v[1]); pk.y = Elem<true>::pack(v[2], v[3]); }
                    else { pk.x = Elem<false>::pack(v[0], v[1]); pk.y = Elem<false>::pack(v[2], v[3]); }
                    *(uint2_t*)((uint16_t*)mt.y + o) = pk;
                }
            }
        }
    }
#undef CB8
}

// The kernels need more dynamic LDS than the default limit: raised once per kernel and device.  Two
// threads that get here together both raise it, which is harmless.
template <bool BF16, int FMT, int MF>
static hipError_t launch_fmt_mf(const PfArgs& a, int wgs, hipStream_t s) {
    static std::atomic<unsigned long long> raised{0ull};        // bit d: done on device d
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const unsigned long long bit = 1ull << (dev & 63);
    if (!(raised.load(std::memory_order_acquire) & bit)) {
        e = hipFuncSetAttribute((const void*)prefill_kernel<BF16, FMT, MF>,
                                hipFuncAttributeMaxDynamicSharedMemorySize, pf_lds_bytes(FMT));
        if (e != hipSuccess) return e;
        raised.fetch_or(bit, std::memory_order_release);
    }
    hipLaunchKernelGGL((prefill_kernel<BF16, FMT, MF>), dim3(wgs), dim3(256), pf_lds_bytes(FMT), s, a);
    return hipGetLastError();
}
template <bool BF16, int FMT>
static hipError_t launch_fmt(const PfArgs& a, int wgs, int mf, hipStream_t s) {
    return mf == 8 ? launch_fmt_mf<BF16, FMT, 8>(a, wgs, s) : launch_fmt_mf<BF16, FMT, 4>(a, wgs, s);
}

// Rows of x per workgroup for a launch whose matrices have `n_tiles` tiles of 256 rows of W in all.
// One workgroup runs per compute unit, so a launch takes about ceil(workgroups / 256) rounds; a round
// of 128-row workgroups does half the MFMAs of a 256-row round at 0.71 of its rate (measured on the
// 7B stack: the W tile is unpacked once per workgroup either way), i.e. costs 0.705 of it.  The
// cheaper of the two wins: 128 rows for launches that would leave compute units without a tile
// (one 4096 x 4096 matrix at M = 2048 is 128 tiles) and for short M.
// rwkvq_set_option(RWKVQ_OPT_PREFILL_TILE_ROWS, 128 | 256) overrides the choice (tests run both kernels).
static int pick_bm(int M, long long n_tiles) {
    const int forced = option(RWKVQ_OPT_PREFILL_TILE_ROWS);
    if (forced == 128 || forced == 256) return forced;
    const long long wg256 = n_tiles * ((M + 255) / 256), wg128 = n_tiles * ((M + 127) / 128);
    const double t256 = (double)((wg256 + 255) / 256), t128 = 0.705 * (double)((wg128 + 255) / 256);
    return t128 < t256 ? 128 : 256;
}

hipError_t launch_prefill(const MatDev* mats_in, int n_mats, int M, int x_dtype, int y_dtype, hipStream_t s) {
    // Workgroups of a matrix with a long K run long: put those matrices first so that the end of
    // a launch is filled by short workgroups.
    std::vector<MatDev> sorted(mats_in, mats_in + n_mats);
    std::stable_sort(sorted.begin(), sorted.end(), [](const MatDev& a, const MatDev& b) { return a.K > b.K; });
    const MatDev* mats = sorted.data();
    // one grouped launch per format and per 64 matrices
    for (int fmt = 0; fmt < 3; ++fmt) {
        int i = 0;
        while (i < n_mats) {
            PfArgs a;
            int cnt = 0, wgs = 0;
            long long n_tiles = 0;                              // tiles along N of the launch's matrices
            for (int j = i, c = 0; j < n_mats && c < kPfMaxMats; ++j)
                if (mats[j].fmt == fmt) { n_tiles += mats[j].N / BN; ++c; }
            const int bm = pick_bm(M, n_tiles);
            const int m_tiles = (M + bm - 1) / bm;
            for (; i < n_mats && cnt < kPfMaxMats; ++i) {
                const MatDev& m = mats[i];
                if (m.fmt != fmt) continue;
                wgs += m_tiles * (m.N / BN);
                a.m[cnt] = PfMat{m.codes, m.aux, m.x, m.y, m.N, m.K, m.fmt, 0};
                a.wg_end[cnt] = wgs;
                ++cnt;
            }
            if (cnt == 0) break;
            for (int j = cnt; j < kPfMaxMats; ++j) {
                a.m[j] = PfMat{nullptr, nullptr, nullptr, nullptr, 0, 0, 0, 0};
                a.wg_end[j] = 0x7FFFFFFF;
            }
            a.M = M; a.ydt = y_dtype; a.m_tiles = m_tiles; a.pad = 0;
            hipError_t e;
            const bool bf = x_dtype == DT_BF16;
            if (fmt == FMT_SQ3) e = bf ? launch_fmt<true, FMT_SQ3>(a, wgs, bm / 32, s) : launch_fmt<false, FMT_SQ3>(a, wgs, bm / 32, s);
            else if (fmt == FMT_VQ6) e = bf ? launch_fmt<true, FMT_VQ6>(a, wgs, bm / 32, s) : launch_fmt<false, FMT_VQ6>(a, wgs, bm / 32, s);
            else e = bf ? launch_fmt<true, FMT_VQ8>(a, wgs, bm / 32, s) : launch_fmt<false, FMT_VQ8>(a, wgs, bm / 32, s);
            if (e != hipSuccess) return e;
        }
    }
    return hipSuccess;
}

}  // namespace rwkvq
