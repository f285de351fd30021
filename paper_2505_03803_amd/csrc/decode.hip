// Streaming dequant-GEMV kernels for small batches (M <= 16), native layout, grouped launch.
//
// Computes y = x * Deq(W)^T (the W. products of App. A.1) for several matrices in one launch,
// each SQ or VQ as its flag says (Sec. 3.1, Eq. "optimization goal").  The work is bound by
// reading the packed weights once from HBM, so everything else is arranged around keeping
// 16-byte coalesced loads in flight:
//
//   * One workgroup (4 wavefronts) owns one 16-row tile of one matrix; its wavefronts take the
//     256-column tiles of that row tile round-robin and their partial sums meet in LDS.
//   * The contraction itself runs on the matrix cores (v_mfma_f32_16x16x32_f16) with the
//     activations as the A operand (rows = batch index) and the weights as the B operand, so
//     the vector ALU only has to turn packed fields into fp16 pairs.  With M = 1 fifteen of the
//     sixteen A rows are idle, which costs nothing: the matrix cores have ~5x headroom here.
//   * SQ: a 3-bit code q is turned into the fp16 number 8 + q by one shift and one and-or
//     (the code lands in the top mantissa bits of 0x4800).  The products sum_k (8 + q) x are
//     accumulated per group of 128 columns together with sum_k x (a second MFMA against a
//     constant ones operand), and the group's scale and zero point are applied in binary32:
//         y += s * (sum (8 + q) x  -  (z + 8) * sum x)  =  s * sum (q - z) x.
//     q, 8 + q and the products are exact; only the binary32 accumulation rounds.
//   * VQ, 6-bit indices: the 64-entry codebook of the current 256 x 256 block is one 32-bit
//     register across the wavefront (lane i holds entry i = two fp16 weights); ds_bpermute_b32
//     gathers entry[index] straight into the B operand.  8-bit indices: the 256-entry codebook
//     is staged in a wavefront-private LDS region and gathered with ds_read_b32.
//   * Activations are staged per wavefront and per column tile in LDS (fp16; bf16 inputs are
//     converted, exact for |x| in [2^-14, 65504]) and read back in A-operand order.
#include "common.h"

namespace rwkvq {

constexpr int kMaxGroupMats = 32;     // matrices per grouped launch (descriptor table in kernarg)
constexpr int kXStride = 264;         // fp16 per staged activation row (256 + 8: bank spread)

struct DecodeMat {
    const uint32_t* codes;
    const uint16_t* aux;
    const void* x;
    void* y;
    int N, K, fmt, wg_end;            // wg_end: first workgroup index after this matrix
};
struct DecodeArgs {
    DecodeMat m[kMaxGroupMats];
    int n_mats, M, xdt, ydt;
};

template <int P>
__device__ __forceinline__ uint32_t sq_pair_f16(uint32_t w0, uint32_t w1, uint32_t w2) {
    // two 3-bit codes -> fp16x2 (8 + q_even, 8 + q_odd)
    constexpr uint32_t kMask = 0x03800380u, kMagic = 0x48004800u;
    if constexpr (P < 15) {
        constexpr int p = P % 5, sh = 6 - 3 * p;
        uint32_t w = (P / 5 == 0) ? w0 : (P / 5 == 1) ? w1 : w2;
        uint32_t v = sh > 0 ? (w << (sh > 0 ? sh : 0)) : sh < 0 ? (w >> (sh < 0 ? -sh : 0)) : w;
        return (v & kMask) | kMagic;
    } else {
        uint32_t v = ((w0 & 0x00010001u) << 7) | ((w1 & 0x00010001u) << 8) | ((w2 & 0x00010001u) << 9);
        return v | kMagic;
    }
}

template <int T>
__device__ __forceinline__ half8_t sq_operand(uint32_t w0, uint32_t w1, uint32_t w2) {
    uint4_t v = {sq_pair_f16<4 * T + 0>(w0, w1, w2), sq_pair_f16<4 * T + 1>(w0, w1, w2),
                 sq_pair_f16<4 * T + 2>(w0, w1, w2), sq_pair_f16<4 * T + 3>(w0, w1, w2)};
    return __builtin_bit_cast(half8_t, v);
}

template <int P>
__device__ __forceinline__ uint32_t vq6_addr(uint32_t w0, uint32_t w1, uint32_t w2) {
    // byte address (index * 4) of codebook entry P for ds_bpermute
    if constexpr (P < 15) {
        constexpr int p = P % 5;
        uint32_t w = (P / 5 == 0) ? w0 : (P / 5 == 1) ? w1 : w2;
        return (w >> (6 * p)) & 0xFCu;
    } else {
        return ((w0 & 3u) << 2) | ((w1 & 3u) << 4) | ((w2 & 3u) << 6);
    }
}

template <int T>
__device__ __forceinline__ half8_t vq6_operand(uint32_t w0, uint32_t w1, uint32_t w2, uint32_t cb) {
    uint4_t v;
    v.x = __builtin_amdgcn_ds_bpermute(vq6_addr<4 * T + 0>(w0, w1, w2), cb);
    v.y = __builtin_amdgcn_ds_bpermute(vq6_addr<4 * T + 1>(w0, w1, w2), cb);
    v.z = __builtin_amdgcn_ds_bpermute(vq6_addr<4 * T + 2>(w0, w1, w2), cb);
    v.w = __builtin_amdgcn_ds_bpermute(vq6_addr<4 * T + 3>(w0, w1, w2), cb);
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

template <int MT>
struct XRegs { uint2_t v[MT]; };

template <int MT>
__device__ __forceinline__ void x_load(XRegs<MT>& r, const void* x, int M, int K, int T, int lane) {
#pragma unroll
    for (int m = 0; m < MT; ++m)
        if (m < M) r.v[m] = *(const uint2_t*)((const uint16_t*)x + (size_t)m * K + 256 * T + 4 * lane);
}

__device__ __forceinline__ uint2_t bf16x4_to_f16x4(uint2_t v) {
    half_t h0 = (half_t)__builtin_bit_cast(float, v.x << 16);
    half_t h1 = (half_t)__builtin_bit_cast(float, v.x & 0xFFFF0000u);
    half_t h2 = (half_t)__builtin_bit_cast(float, v.y << 16);
    half_t h3 = (half_t)__builtin_bit_cast(float, v.y & 0xFFFF0000u);
    uint2_t o;
    o.x = (uint32_t)__builtin_bit_cast(uint16_t, h0) | ((uint32_t)__builtin_bit_cast(uint16_t, h1) << 16);
    o.y = (uint32_t)__builtin_bit_cast(uint16_t, h2) | ((uint32_t)__builtin_bit_cast(uint16_t, h3) << 16);
    return o;
}

template <int MT>
__device__ __forceinline__ void x_store(const XRegs<MT>& r, half_t* xs, int M, int lane, bool bf16) {
#pragma unroll
    for (int m = 0; m < MT; ++m)
        if (m < M) *(uint2_t*)(xs + m * kXStride + 4 * lane) = bf16 ? bf16x4_to_f16x4(r.v[m]) : r.v[m];
}

// ---- per-format tile loops ------------------------------------------------------------------
template <int MT> struct Acc { static constexpr int n = MT == 1 ? 1 : 4; };

#define RWKVQ_MFMA(a, b, c) __builtin_amdgcn_mfma_f32_16x16x32_f16((a), (b), (c), 0, 0, 0)

template <int MT>
__device__ __forceinline__ void run_sq(const DecodeMat& mt, int R, int M, bool xbf16, int wave, int lane,
                                       half_t* xs, float4_t& out) {
    const int KT = mt.K >> 8;
    const uint32_t* codes = mt.codes + (size_t)R * KT * 384;
    const uint2_t* sz = (const uint2_t*)mt.aux + (size_t)R * KT * 16 + (lane & 15);
    const half_t* xrow = xs + ((lane & 15) < M ? (lane & 15) : M - 1) * kXStride + 8 * (lane >> 4);
    const half8_t ones = {1, 1, 1, 1, 1, 1, 1, 1};
    if (wave >= KT) return;
    uint4_t a = *(const uint4_t*)(codes + (size_t)wave * 384 + 4 * lane);
    uint2_t b = *(const uint2_t*)(codes + (size_t)wave * 384 + 256 + 2 * lane);
    uint2_t szr = sz[(size_t)wave * 16];
    XRegs<MT> xr;
    x_load<MT>(xr, mt.x, M, mt.K, wave, lane);
    for (int T = wave; T < KT; T += 4) {
        wave_lds_sync();
        x_store<MT>(xr, xs, M, lane, xbf16);
        wave_lds_sync();
        uint4_t ca = a;
        uint2_t cb = b, csz = szr;
        const int Tn = T + 4;
        if (Tn < KT) {
            a = *(const uint4_t*)(codes + (size_t)Tn * 384 + 4 * lane);
            b = *(const uint2_t*)(codes + (size_t)Tn * 384 + 256 + 2 * lane);
            szr = sz[(size_t)Tn * 16];
            x_load<MT>(xr, mt.x, M, mt.K, Tn, lane);
        }
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const uint32_t w0 = u == 0 ? ca.x : ca.w, w1 = u == 0 ? ca.y : cb.x, w2 = u == 0 ? ca.z : cb.y;
            float4_t acc = {0, 0, 0, 0}, accx = {0, 0, 0, 0};
            half8_t xa;
            xa = *(const half8_t*)(xrow + 128 * u + 0);
            acc = RWKVQ_MFMA(xa, sq_operand<0>(w0, w1, w2), acc);
            accx = RWKVQ_MFMA(xa, ones, accx);
            xa = *(const half8_t*)(xrow + 128 * u + 32);
            acc = RWKVQ_MFMA(xa, sq_operand<1>(w0, w1, w2), acc);
            accx = RWKVQ_MFMA(xa, ones, accx);
            xa = *(const half8_t*)(xrow + 128 * u + 64);
            acc = RWKVQ_MFMA(xa, sq_operand<2>(w0, w1, w2), acc);
            accx = RWKVQ_MFMA(xa, ones, accx);
            xa = *(const half8_t*)(xrow + 128 * u + 96);
            acc = RWKVQ_MFMA(xa, sq_operand<3>(w0, w1, w2), acc);
            accx = RWKVQ_MFMA(xa, ones, accx);
            const uint32_t szw = u == 0 ? csz.x : csz.y;
            const float s = f16_bits_to_f32((uint16_t)(szw & 0xFFFFu));
            const float zz = f16_bits_to_f32((uint16_t)(szw >> 16)) + 8.0f;
#pragma unroll
            for (int i = 0; i < Acc<MT>::n; ++i) out[i] = fmaf(s, fmaf(-zz, accx[i], acc[i]), out[i]);
        }
    }
}

template <int MT>
__device__ __forceinline__ void run_vq6(const DecodeMat& mt, int R, int M, bool xbf16, int wave, int lane,
                                        half_t* xs, float4_t& out) {
    const int KT = mt.K >> 8;
    const uint32_t* codes = mt.codes + (size_t)R * KT * 384;
    const uint32_t* cbs = (const uint32_t*)mt.aux + (size_t)(R >> 4) * KT * 64 + lane;
    const half_t* xrow = xs + ((lane & 15) < M ? (lane & 15) : M - 1) * kXStride + 8 * (lane >> 4);
    if (wave >= KT) return;
    uint4_t a = *(const uint4_t*)(codes + (size_t)wave * 384 + 4 * lane);
    uint2_t b = *(const uint2_t*)(codes + (size_t)wave * 384 + 256 + 2 * lane);
    uint32_t cbr = cbs[(size_t)wave * 64];
    XRegs<MT> xr;
    x_load<MT>(xr, mt.x, M, mt.K, wave, lane);
    for (int T = wave; T < KT; T += 4) {
        wave_lds_sync();
        x_store<MT>(xr, xs, M, lane, xbf16);
        wave_lds_sync();
        uint4_t ca = a;
        uint2_t cb = b;
        uint32_t ccb = cbr;
        const int Tn = T + 4;
        if (Tn < KT) {
            a = *(const uint4_t*)(codes + (size_t)Tn * 384 + 4 * lane);
            b = *(const uint2_t*)(codes + (size_t)Tn * 384 + 256 + 2 * lane);
            cbr = cbs[(size_t)Tn * 64];
            x_load<MT>(xr, mt.x, M, mt.K, Tn, lane);
        }
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const uint32_t w0 = u == 0 ? ca.x : ca.w, w1 = u == 0 ? ca.y : cb.x, w2 = u == 0 ? ca.z : cb.y;
            out = RWKVQ_MFMA(*(const half8_t*)(xrow + 128 * u + 0), vq6_operand<0>(w0, w1, w2, ccb), out);
            out = RWKVQ_MFMA(*(const half8_t*)(xrow + 128 * u + 32), vq6_operand<1>(w0, w1, w2, ccb), out);
            out = RWKVQ_MFMA(*(const half8_t*)(xrow + 128 * u + 64), vq6_operand<2>(w0, w1, w2, ccb), out);
            out = RWKVQ_MFMA(*(const half8_t*)(xrow + 128 * u + 96), vq6_operand<3>(w0, w1, w2, ccb), out);
        }
    }
}

template <int MT>
__device__ __forceinline__ void run_vq8(const DecodeMat& mt, int R, int M, bool xbf16, int wave, int lane,
                                        half_t* xs, uint32_t* cb_lds, float4_t& out) {
    const int KT = mt.K >> 8;
    const uint32_t* codes = mt.codes + (size_t)R * KT * 512;
    const uint4_t* cbs = (const uint4_t*)mt.aux + (size_t)(R >> 4) * KT * 64 + lane;
    const half_t* xrow = xs + ((lane & 15) < M ? (lane & 15) : M - 1) * kXStride + 8 * (lane >> 4);
    if (wave >= KT) return;
    uint4_t a = *(const uint4_t*)(codes + (size_t)wave * 512 + 4 * lane);
    uint4_t b = *(const uint4_t*)(codes + (size_t)wave * 512 + 256 + 4 * lane);
    uint4_t cbr = cbs[(size_t)wave * 64];
    XRegs<MT> xr;
    x_load<MT>(xr, mt.x, M, mt.K, wave, lane);
    for (int T = wave; T < KT; T += 4) {
        wave_lds_sync();
        x_store<MT>(xr, xs, M, lane, xbf16);
        *(uint4_t*)(cb_lds + 4 * lane) = cbr;
        wave_lds_sync();
        uint4_t ca = a, cb = b;
        const int Tn = T + 4;
        if (Tn < KT) {
            a = *(const uint4_t*)(codes + (size_t)Tn * 512 + 4 * lane);
            b = *(const uint4_t*)(codes + (size_t)Tn * 512 + 256 + 4 * lane);
            cbr = cbs[(size_t)Tn * 64];
            x_load<MT>(xr, mt.x, M, mt.K, Tn, lane);
        }
        out = RWKVQ_MFMA(*(const half8_t*)(xrow + 0), vq8_operand(ca.x, cb_lds), out);
        out = RWKVQ_MFMA(*(const half8_t*)(xrow + 32), vq8_operand(ca.y, cb_lds), out);
        out = RWKVQ_MFMA(*(const half8_t*)(xrow + 64), vq8_operand(ca.z, cb_lds), out);
        out = RWKVQ_MFMA(*(const half8_t*)(xrow + 96), vq8_operand(ca.w, cb_lds), out);
        out = RWKVQ_MFMA(*(const half8_t*)(xrow + 128), vq8_operand(cb.x, cb_lds), out);
        out = RWKVQ_MFMA(*(const half8_t*)(xrow + 160), vq8_operand(cb.y, cb_lds), out);
        out = RWKVQ_MFMA(*(const half8_t*)(xrow + 192), vq8_operand(cb.z, cb_lds), out);
        out = RWKVQ_MFMA(*(const half8_t*)(xrow + 224), vq8_operand(cb.w, cb_lds), out);
    }
}

// One workgroup = one 16-row tile of one matrix.  MT = number of activation rows carried
// (1, 4 or 16 >= M).  D layout of the MFMA: lane holds rows 4*(lane/16) + i, column lane%16.
template <int MT>
__global__ void __launch_bounds__(256) decode_kernel(DecodeArgs a) {
    __shared__ __attribute__((aligned(16))) half_t xs_all[4][MT * kXStride];
    __shared__ __attribute__((aligned(16))) uint32_t cb_all[4][256];
    __shared__ float red[4][MT][16];

    const int wg = blockIdx.x;
    int mi = 0;
    while (mi + 1 < a.n_mats && wg >= a.m[mi].wg_end) ++mi;
    const DecodeMat mt = a.m[mi];
    const int R = wg - (mi ? a.m[mi - 1].wg_end : 0);
    const int M = a.M;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const bool xbf16 = a.xdt == DT_BF16;

    float4_t out = {0, 0, 0, 0};
    if (mt.fmt == FMT_SQ3) run_sq<MT>(mt, R, M, xbf16, wave, lane, xs_all[wave], out);
    else if (mt.fmt == FMT_VQ6) run_vq6<MT>(mt, R, M, xbf16, wave, lane, xs_all[wave], out);
    else run_vq8<MT>(mt, R, M, xbf16, wave, lane, xs_all[wave], cb_all[wave], out);

    if (MT == 16) {
#pragma unroll
        for (int i = 0; i < 4; ++i) red[wave][(4 * (lane >> 4) + i) % MT][lane & 15] = out[i];
    } else if (lane < 16) {
#pragma unroll
        for (int i = 0; i < Acc<MT>::n; ++i) red[wave][i % MT][lane] = out[i];
    }
    __syncthreads();
    const int t = threadIdx.x;
    if (t < MT * 16) {
        const int m = t >> 4, n = t & 15;
        if (m < M) {
            float v = (red[0][m][n] + red[1][m][n]) + (red[2][m][n] + red[3][m][n]);
            store_from_f32(mt.y, (size_t)m * mt.N + 16 * R + n, a.ydt, v);
        }
    }
}

hipError_t launch_decode(const MatDev* mats, int n_mats, int M, int x_dtype, int y_dtype, hipStream_t s) {
    for (int base = 0; base < n_mats; base += kMaxGroupMats) {
        DecodeArgs a;
        int cnt = n_mats - base < kMaxGroupMats ? n_mats - base : kMaxGroupMats;
        int wgs = 0;
        for (int i = 0; i < cnt; ++i) {
            const MatDev& m = mats[base + i];
            wgs += m.N / 16;
            a.m[i] = DecodeMat{m.codes, m.aux, m.x, m.y, m.N, m.K, m.fmt, wgs};
        }
        for (int i = cnt; i < kMaxGroupMats; ++i) a.m[i] = DecodeMat{nullptr, nullptr, nullptr, nullptr, 0, 0, 0, wgs};
        a.n_mats = cnt; a.M = M; a.xdt = x_dtype; a.ydt = y_dtype;
        if (M == 1) hipLaunchKernelGGL(decode_kernel<1>, dim3(wgs), dim3(256), 0, s, a);
        else if (M <= 4) hipLaunchKernelGGL(decode_kernel<4>, dim3(wgs), dim3(256), 0, s, a);
        else hipLaunchKernelGGL(decode_kernel<16>, dim3(wgs), dim3(256), 0, s, a);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace rwkvq
