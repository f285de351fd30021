// Matrix-core path for large batches (prefill): y[M][N] = x[M][K] * Deq(W)^T with tiles of W
// dequantized into LDS and multiplied by v_mfma_f32_16x16x32_{bf16,f16} in the type of x,
// binary32 accumulate.  Grouped launch: the tiles of several matrices (each SQ or VQ as its flag
// says, Sec. 3.1 Eq. "optimization goal") share one grid so that all compute units stay busy.
//
// What is fed to the multipliers: Deq(W) exactly as defined in Sec. 2.2 (SQ: (q - z) * s in
// binary32; VQ: the fp16 codebook entry) rounded once, to nearest even, to the type of x.
//
// Tiling: workgroup = 256 threads = 2 x 2 wavefronts, block tile 256 (m) x 256 (n) x 64 (k),
// wavefront tile 128 x 128 = 8 x 8 MFMA tiles (256 accumulator registers).  Both operands live
// in LDS as [row][64 k] with rows padded to 144 bytes, which makes the 16-byte fragment reads and
// the 16-byte tile writes bank-conflict free.  Two LDS buffers: while the matrix cores work on
// k-step i, the activations of step i+1 are in flight from global memory and the weights of step
// i+1 are being unpacked by the vector ALU from packed words that were fetched once per 256
// columns.  One workgroup barrier per k-step.
//
// Workgroup -> tile order: the m-tile index runs fastest, so workgroups that are dispatched
// round-robin over the 8 XCDs keep one slice of x (256 rows) per XCD L2 when there are 8 m-tiles.
#include "common.h"

namespace rwkvq {

constexpr int kPfMaxMats = 32;
constexpr int BM = 256, BN = 256;        // block tile; the k-step is 64 columns
constexpr int kRowBytes = 144;                 // 64 k * 2 B + 16 B pad
constexpr int kTileBytes = 256 * kRowBytes;    // one operand tile
constexpr int kCb8Bytes = 1024;                // converted 8-bit-index codebook
constexpr int kPfLds = 4 * kTileBytes + 2 * kCb8Bytes;

struct PfMat {
    const uint32_t* codes;
    const uint16_t* aux;
    const void* x;
    void* y;
    int N, K, fmt, wg_end;
};
struct PfArgs {
    PfMat m[kPfMaxMats];
    int n_mats, M, ydt, m_tiles;
};

template <bool BF16> struct Elem;
template <> struct Elem<true> {
    static __device__ __forceinline__ float4_t mfma(uint4_t a, uint4_t b, float4_t c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                       __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
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
    static __device__ __forceinline__ float4_t mfma(uint4_t a, uint4_t b, float4_t c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8_t, a),
                                                      __builtin_bit_cast(half8_t, b), c, 0, 0, 0);
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

// Eight consecutive-k weights (step T4 of a unit) of one lane, as four packed pairs.
template <bool BF16, int T4>
__device__ __forceinline__ uint4_t sq_chunk(uint32_t w0, uint32_t w1, uint32_t w2, float s, float z) {
    uint4_t o;
    o.x = Elem<BF16>::pack(sq_deq(sq_code<8 * T4 + 0>(w0, w1, w2), s, z), sq_deq(sq_code<8 * T4 + 1>(w0, w1, w2), s, z));
    o.y = Elem<BF16>::pack(sq_deq(sq_code<8 * T4 + 2>(w0, w1, w2), s, z), sq_deq(sq_code<8 * T4 + 3>(w0, w1, w2), s, z));
    o.z = Elem<BF16>::pack(sq_deq(sq_code<8 * T4 + 4>(w0, w1, w2), s, z), sq_deq(sq_code<8 * T4 + 5>(w0, w1, w2), s, z));
    o.w = Elem<BF16>::pack(sq_deq(sq_code<8 * T4 + 6>(w0, w1, w2), s, z), sq_deq(sq_code<8 * T4 + 7>(w0, w1, w2), s, z));
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
struct WRegs {
    uint4_t a[4];     // words 0..3 of the lane
    uint4_t b[4];     // SQ / VQ6: words 4,5 in .x,.y ; VQ8: words 4..7
    uint2_t sz[4];    // SQ: (scale,zero) of unit 0 and unit 1 for the lane's row
    uint32_t cb;      // VQ6: converted codebook entry `lane`
    uint4_t cb8;      // VQ8: 4 raw codebook entries (4*lane .. 4*lane+3)
};

__device__ __forceinline__ void w_load(WRegs& r, const PfMat& mt, int R0, int T, int wave, int lane) {
    const int KT = mt.K >> 8;
    if (mt.fmt == FMT_VQ8) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t* tile = mt.codes + ((size_t)(R0 + 4 * wave + i) * KT + T) * 512;
            r.a[i] = *(const uint4_t*)(tile + 4 * lane);
            r.b[i] = *(const uint4_t*)(tile + 256 + 4 * lane);
        }
        r.cb8 = ((const uint4_t*)mt.aux)[((size_t)(R0 >> 4) * KT + T) * 64 + lane];
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t* tile = mt.codes + ((size_t)(R0 + 4 * wave + i) * KT + T) * 384;
            r.a[i] = *(const uint4_t*)(tile + 4 * lane);
            uint2_t b = *(const uint2_t*)(tile + 256 + 2 * lane);
            r.b[i].x = b.x; r.b[i].y = b.y;
        }
        if (mt.fmt == FMT_SQ3) {
#pragma unroll
            for (int i = 0; i < 4; ++i)
                r.sz[i] = ((const uint2_t*)mt.aux)[((size_t)(R0 + 4 * wave + i) * KT + T) * 16 + (lane & 15)];
        } else {
            r.cb = ((const uint32_t*)mt.aux)[((size_t)(R0 >> 4) * KT + T) * 64 + lane];
        }
    }
}

// Unpack k-step KQ (0..3: 64 columns) of the tile held in r and write it to the W tile in LDS.
template <bool BF16, int KQ>
__device__ __forceinline__ void w_unpack(const WRegs& r, int fmt, char* wt, uint32_t* cb8, int wave, int lane) {
    constexpr int u = KQ >> 1, t0 = 2 * (KQ & 1);
    char* dst = wt + (64 * wave + (lane & 15)) * kRowBytes + 16 * (lane >> 4);
    if (fmt == FMT_SQ3) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t w0 = u == 0 ? r.a[i].x : r.a[i].w, w1 = u == 0 ? r.a[i].y : r.b[i].x,
                           w2 = u == 0 ? r.a[i].z : r.b[i].y;
            const uint32_t szw = u == 0 ? r.sz[i].x : r.sz[i].y;
            const float s = f16_bits_to_f32((uint16_t)(szw & 0xFFFFu)), z = f16_bits_to_f32((uint16_t)(szw >> 16));
            *(uint4_t*)(dst + 16 * i * kRowBytes) = sq_chunk<BF16, t0>(w0, w1, w2, s, z);
            *(uint4_t*)(dst + 16 * i * kRowBytes + 64) = sq_chunk<BF16, t0 + 1>(w0, w1, w2, s, z);
        }
    } else if (fmt == FMT_VQ6) {
        const uint32_t cb = Elem<BF16>::from_f16x2(r.cb);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t w0 = u == 0 ? r.a[i].x : r.a[i].w, w1 = u == 0 ? r.a[i].y : r.b[i].x,
                           w2 = u == 0 ? r.a[i].z : r.b[i].y;
            *(uint4_t*)(dst + 16 * i * kRowBytes) = vq6_chunk<t0>(w0, w1, w2, cb);
            *(uint4_t*)(dst + 16 * i * kRowBytes + 64) = vq6_chunk<t0 + 1>(w0, w1, w2, cb);
        }
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t wa = u == 0 ? (t0 == 0 ? r.a[i].x : r.a[i].z) : (t0 == 0 ? r.b[i].x : r.b[i].z);
            const uint32_t wb = u == 0 ? (t0 == 0 ? r.a[i].y : r.a[i].w) : (t0 == 0 ? r.b[i].y : r.b[i].w);
            *(uint4_t*)(dst + 16 * i * kRowBytes) = vq8_chunk(wa, cb8);
            *(uint4_t*)(dst + 16 * i * kRowBytes + 64) = vq8_chunk(wb, cb8);
        }
    }
}

struct XTile { uint4_t v[8]; };

__device__ __forceinline__ void x_tile_load(XTile& r, const uint16_t* x, int M, int K, int m0, int k0, int tid) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        int c = tid + 256 * i, row = c >> 3, col = c & 7;
        int m = m0 + row;
        m = m < M ? m : M - 1;
        r.v[i] = *(const uint4_t*)(x + (size_t)m * K + k0 + 8 * col);
    }
}
__device__ __forceinline__ void x_tile_store(const XTile& r, char* xt, int tid) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        int c = tid + 256 * i, row = c >> 3, col = c & 7;
        *(uint4_t*)(xt + row * kRowBytes + 16 * col) = r.v[i];
    }
}

template <bool BF16>
__device__ __forceinline__ void mma_step(const char* xt, const char* wt, int wm, int wn, int lane,
                                         float4_t (&acc)[8][8]) {
    const char* xa = xt + (128 * wm + (lane & 15)) * kRowBytes + 16 * (lane >> 4);
    const char* wb = wt + (128 * wn + (lane & 15)) * kRowBytes + 16 * (lane >> 4);
#pragma unroll
    for (int k32 = 0; k32 < 2; ++k32) {
        uint4_t b[8];
#pragma unroll
        for (int ni = 0; ni < 8; ++ni) b[ni] = *(const uint4_t*)(wb + 16 * ni * kRowBytes + 64 * k32);
#pragma unroll
        for (int mi = 0; mi < 8; ++mi) {
            uint4_t a = *(const uint4_t*)(xa + 16 * mi * kRowBytes + 64 * k32);
#pragma unroll
            for (int ni = 0; ni < 8; ++ni) acc[mi][ni] = Elem<BF16>::mfma(a, b[ni], acc[mi][ni]);
        }
    }
}

// Convert and stage the 8-bit-index codebook of the current tile (256 entries) into LDS.
template <bool BF16>
__device__ __forceinline__ void cb8_store(const WRegs& r, uint32_t* cb8, int wave, int lane) {
    if (wave == 0) {
        uint4_t c = {Elem<BF16>::from_f16x2(r.cb8.x), Elem<BF16>::from_f16x2(r.cb8.y),
                     Elem<BF16>::from_f16x2(r.cb8.z), Elem<BF16>::from_f16x2(r.cb8.w)};
        *(uint4_t*)(cb8 + 4 * lane) = c;
    }
}

template <bool BF16>
__global__ void __launch_bounds__(256, 1) prefill_kernel(PfArgs a) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    char* const xt0 = lds;
    char* const xt1 = lds + kTileBytes;
    char* const wt0 = lds + 2 * kTileBytes;
    char* const wt1 = lds + 3 * kTileBytes;
    uint32_t* const cb8base = (uint32_t*)(lds + 4 * kTileBytes);
#define CB8(i) (cb8base + ((i) & 1) * (kCb8Bytes / 4))

    const int wg = blockIdx.x;
    int mi_ = 0;
    while (mi_ + 1 < a.n_mats && wg >= a.m[mi_].wg_end) ++mi_;
    const PfMat mt = a.m[mi_];
    const int local = wg - (mi_ ? a.m[mi_ - 1].wg_end : 0);
    const int m0 = (local % a.m_tiles) * BM, n0 = (local / a.m_tiles) * BN;
    const int M = a.M, K = mt.K, KT = K >> 8, R0 = n0 >> 4;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, wm = wave >> 1, wn = wave & 1;
    const uint16_t* x = (const uint16_t*)mt.x;
    const int fmt = mt.fmt;

    float4_t acc[8][8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[i][j] = float4_t{0, 0, 0, 0};

    // prologue: tile 0, k-step 0 into buffer 0
    WRegs wr;
    XTile xr;
    w_load(wr, mt, R0, 0, wave, lane);
    x_tile_load(xr, x, M, K, m0, 0, tid);
    if (fmt == FMT_VQ8) {
        cb8_store<BF16>(wr, CB8(0), wave, lane);
        __syncthreads();
    }
    w_unpack<BF16, 0>(wr, fmt, wt0, CB8(0), wave, lane);
    x_tile_store(xr, xt0, tid);
    __syncthreads();

    for (int T = 0; T < KT; ++T) {
        const bool last = T + 1 == KT;
        // k-steps 0..2 of this tile: next step comes from the same packed words
        x_tile_load(xr, x, M, K, m0, 256 * T + 64, tid);
        mma_step<BF16>(xt0, wt0, wm, wn, lane, acc);
        w_unpack<BF16, 1>(wr, fmt, wt1, CB8(T), wave, lane);
        x_tile_store(xr, xt1, tid);
        __syncthreads();

        x_tile_load(xr, x, M, K, m0, 256 * T + 128, tid);
        mma_step<BF16>(xt1, wt1, wm, wn, lane, acc);
        w_unpack<BF16, 2>(wr, fmt, wt0, CB8(T), wave, lane);
        x_tile_store(xr, xt0, tid);
        __syncthreads();

        x_tile_load(xr, x, M, K, m0, 256 * T + 192, tid);
        WRegs wn_;
        if (!last) w_load(wn_, mt, R0, T + 1, wave, lane);
        mma_step<BF16>(xt0, wt0, wm, wn, lane, acc);
        w_unpack<BF16, 3>(wr, fmt, wt1, CB8(T), wave, lane);
        x_tile_store(xr, xt1, tid);
        if (!last && fmt == FMT_VQ8) cb8_store<BF16>(wn_, CB8(T + 1), wave, lane);
        __syncthreads();

        if (!last) x_tile_load(xr, x, M, K, m0, 256 * T + 256, tid);
        mma_step<BF16>(xt1, wt1, wm, wn, lane, acc);
        if (!last) {
            wr = wn_;
            w_unpack<BF16, 0>(wr, fmt, wt0, CB8(T + 1), wave, lane);
            x_tile_store(xr, xt0, tid);
        }
        __syncthreads();
    }

    // epilogue: lane holds rows 4*(lane/16) + i, column lane%16 of every 16 x 16 tile
    const int N = mt.N;
#pragma unroll
    for (int mi = 0; mi < 8; ++mi)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int m = m0 + 128 * wm + 16 * mi + 4 * (lane >> 4) + i;
            if (m < M) {
#pragma unroll
                for (int ni = 0; ni < 8; ++ni) {
                    const int n = n0 + 128 * wn + 16 * ni + (lane & 15);
                    store_from_f32(mt.y, (size_t)m * N + n, a.ydt, acc[mi][ni][i]);
                }
            }
        }
#undef CB8
}

hipError_t launch_prefill(const MatDev* mats, int n_mats, int M, int x_dtype, int y_dtype, hipStream_t s) {
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void*)prefill_kernel<true>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, kPfLds);
        if (e != hipSuccess) return e;
        e = hipFuncSetAttribute((const void*)prefill_kernel<false>,
                                hipFuncAttributeMaxDynamicSharedMemorySize, kPfLds);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int m_tiles = (M + BM - 1) / BM;
    for (int base = 0; base < n_mats; base += kPfMaxMats) {
        PfArgs a;
        int cnt = n_mats - base < kPfMaxMats ? n_mats - base : kPfMaxMats;
        int wgs = 0;
        for (int i = 0; i < cnt; ++i) {
            const MatDev& m = mats[base + i];
            wgs += m_tiles * (m.N / BN);
            a.m[i] = PfMat{m.codes, m.aux, m.x, m.y, m.N, m.K, m.fmt, wgs};
        }
        for (int i = cnt; i < kPfMaxMats; ++i) a.m[i] = PfMat{nullptr, nullptr, nullptr, nullptr, 0, 0, 0, wgs};
        a.n_mats = cnt; a.M = M; a.ydt = y_dtype; a.m_tiles = m_tiles;
        if (x_dtype == DT_BF16) hipLaunchKernelGGL(prefill_kernel<true>, dim3(wgs), dim3(256), kPfLds, s, a);
        else hipLaunchKernelGGL(prefill_kernel<false>, dim3(wgs), dim3(256), kPfLds, s, a);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace rwkvq
