// Prepack (canonical -> native layout) and dense dequantization kernels.
//
// Dequantization follows Sec. 2.2: SQ  w = (q - z) * s  per group of 128 input channels
// (inverse of Eq. "SQ"), VQ  (w[n,2j], w[n,2j+1]) = codebook[block(n, 2j)][index[n,j]]
// (Eq. "VQ").  These kernels are plain gathers: one thread per output word / element.
#include "common.h"

namespace rwkvq {

// ------------------------------------------------------------------ prepack

// One thread per native word.  Grid covers N/16 * K/256 * 384 words.
__global__ void sq_prepack_codes_kernel(const uint32_t* __restrict__ codes, int N, int K,
                                        uint32_t* __restrict__ out) {
    size_t gid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t total = (size_t)(N / 16) * (K / 256) * 384;
    if (gid >= total) return;
    int wi = (int)(gid % 384);
    size_t tile = gid / 384;
    int T = (int)(tile % (K / 256));
    int R = (int)(tile / (K / 256));
    int lane, i;
    if (wi < 256) { lane = wi >> 2; i = wi & 3; } else { lane = (wi - 256) >> 1; i = 4 + ((wi - 256) & 1); }
    int u = i / 3, w = i % 3;
    const uint32_t* row = codes + (size_t)(16 * R + (lane & 15)) * (K * 3 / 32);
    uint32_t word = 0;
    for (int p = 0; p < 5; ++p)
        for (int e = 0; e < 2; ++e) {
            int c = 2 * (5 * w + p) + e;
            uint32_t q = canon_field(row, 3, 256 * T + tile_col(lane, u, c));
            word |= q << (1 + 3 * p + 16 * e);
        }
    for (int e = 0; e < 2; ++e) {                    // pair 15: bit w of codes 30 and 31
        uint32_t q = canon_field(row, 3, 256 * T + tile_col(lane, u, 30 + e));
        word |= ((q >> w) & 1u) << (16 * e);
    }
    out[gid] = word;
}

// One thread per (row, group): interleave scale and zero into the native buffer.
__global__ void sq_prepack_sz_kernel(const uint16_t* __restrict__ scales,
                                     const uint16_t* __restrict__ zeros, int N, int K,
                                     uint16_t* __restrict__ out) {
    size_t gid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    int G = K / kGroup;
    if (gid >= (size_t)N * G) return;
    int n = (int)(gid / G), g = (int)(gid % G);
    size_t o = native_sz_index(n, g, K);
    out[o] = scales[gid];
    out[o + 1] = zeros[gid];
}

__global__ void vq_prepack_kernel(const uint32_t* __restrict__ indices, int N, int K, int kbits,
                                  uint32_t* __restrict__ out) {
    size_t gid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    int tw = kbits == 8 ? 512 : 384;
    size_t total = (size_t)(N / 16) * (K / 256) * tw;
    if (gid >= total) return;
    int wi = (int)(gid % tw);
    size_t tile = gid / tw;
    int T = (int)(tile % (K / 256));
    int R = (int)(tile / (K / 256));
    uint32_t word = 0;
    if (kbits == 8) {
        int lane, i;
        if (wi < 256) { lane = wi >> 2; i = wi & 3; } else { lane = (wi - 256) >> 2; i = 4 + ((wi - 256) & 3); }
        int u = i >> 2, w = i & 3;
        const uint32_t* row = indices + (size_t)(16 * R + (lane & 15)) * (K / 2 * 8 / 32);
        for (int b = 0; b < 4; ++b) {
            int P = 4 * w + b;
            int col = 256 * T + tile_col(lane, u, 2 * P);
            word |= canon_field(row, 8, col >> 1) << (8 * b);
        }
    } else {
        int lane, i;
        if (wi < 256) { lane = wi >> 2; i = wi & 3; } else { lane = (wi - 256) >> 1; i = 4 + ((wi - 256) & 1); }
        int u = i / 3, w = i % 3;
        const uint32_t* row = indices + (size_t)(16 * R + (lane & 15)) * (K / 2 * 6 / 32);
        for (int p = 0; p < 5; ++p) {
            int P = 5 * w + p;
            int col = 256 * T + tile_col(lane, u, 2 * P);
            word |= canon_field(row, 6, col >> 1) << (2 + 6 * p);
        }
        int col = 256 * T + tile_col(lane, u, 30);   // index 15: bits 2w, 2w+1 into bits 0,1
        uint32_t idx = canon_field(row, 6, col >> 1);
        word |= (idx >> (2 * w)) & 3u;
    }
    out[gid] = word;
}

// ------------------------------------------------------------------ dequant

// Element (n, k) of Deq(W) in binary32, from either layout.  This is the definition the
// streaming and matrix-core kernels are checked against; it is written for clarity, not speed.
__device__ float deq_element(const MatDev& m, int n, int k) {
    const int K = m.K;
    if (m.fmt == FMT_SQ3) {
        uint32_t q;
        float s, z;
        int g = k / kGroup;
        if (m.layout == 0) {
            q = canon_field(m.codes + (size_t)n * (K * 3 / 32), 3, k);
            s = f16_bits_to_f32(m.aux[(size_t)n * (K / kGroup) + g]);
            z = f16_bits_to_f32(m.aux2[(size_t)n * (K / kGroup) + g]);
        } else {
            TilePos p = tile_pos(n & 15, k & 255);
            const uint32_t* tile = m.codes + ((size_t)(n >> 4) * (K / 256) + (k >> 8)) * 384;
            uint32_t w[3];
            for (int i = 0; i < 3; ++i) w[i] = tile[tile6_word(p.lane, 3 * p.u + i)];
            q = native_sq_field(w, p.c);
            size_t o = native_sz_index(n, g, K);
            s = f16_bits_to_f32(m.aux[o]);
            z = f16_bits_to_f32(m.aux[o + 1]);
        }
        return sq_deq(q, s, z);
    }
    const int kbits = m.fmt == FMT_VQ8 ? 8 : 6;
    uint32_t idx;
    if (m.layout == 0) {
        idx = canon_field(m.codes + (size_t)n * (K / 2 * kbits / 32), kbits, k >> 1);
    } else {
        TilePos p = tile_pos(n & 15, k & 255);
        int P = p.c >> 1;
        if (kbits == 8) {
            const uint32_t* tile = m.codes + ((size_t)(n >> 4) * (K / 256) + (k >> 8)) * 512;
            uint32_t w = tile[tile8_word(p.lane, 4 * p.u + (P >> 2))];
            idx = (w >> (8 * (P & 3))) & 255u;
        } else {
            const uint32_t* tile = m.codes + ((size_t)(n >> 4) * (K / 256) + (k >> 8)) * 384;
            uint32_t w[3];
            for (int i = 0; i < 3; ++i) w[i] = tile[tile6_word(p.lane, 3 * p.u + i)];
            idx = native_vq6_index(w, P);
        }
    }
    size_t cb = (size_t)(n / kBlock) * (K / kBlock) + (k / kBlock);
    return f16_bits_to_f32(m.aux[((cb << kbits) + idx) * 2 + (k & 1)]);
}

__global__ void dequant_kernel(MatDev m, void* __restrict__ out, int dt) {
    size_t gid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t total = (size_t)m.N * m.K;
    if (gid >= total) return;
    int n = (int)(gid / m.K), k = (int)(gid % m.K);
    store_from_f32(out, gid, dt, deq_element(m, n, k));
}

static inline unsigned blocks_for(size_t n, int bs) { return (unsigned)((n + bs - 1) / bs); }

hipError_t launch_sq_prepack(const uint32_t* codes, const uint16_t* scales, const uint16_t* zeros,
                             int N, int K, uint32_t* codes_native, uint16_t* sz_native, hipStream_t s) {
    size_t words = (size_t)(N / 16) * (K / 256) * 384;
    hipLaunchKernelGGL(sq_prepack_codes_kernel, dim3(blocks_for(words, 256)), dim3(256), 0, s, codes, N,
                       K, codes_native);
    size_t groups = (size_t)N * (K / kGroup);
    hipLaunchKernelGGL(sq_prepack_sz_kernel, dim3(blocks_for(groups, 256)), dim3(256), 0, s, scales,
                       zeros, N, K, sz_native);
    return hipGetLastError();
}

hipError_t launch_vq_prepack(const uint32_t* indices, int N, int K, int kbits, uint32_t* out,
                             hipStream_t s) {
    size_t words = (size_t)(N / 16) * (K / 256) * (kbits == 8 ? 512 : 384);
    hipLaunchKernelGGL(vq_prepack_kernel, dim3(blocks_for(words, 256)), dim3(256), 0, s, indices, N, K,
                       kbits, out);
    return hipGetLastError();
}

hipError_t launch_dequant(const MatDev& m, void* w_out, int w_dtype, hipStream_t s) {
    size_t total = (size_t)m.N * m.K;
    hipLaunchKernelGGL(dequant_kernel, dim3(blocks_for(total, 256)), dim3(256), 0, s, m, w_out, w_dtype);
    return hipGetLastError();
}

// ------------------------------------------------------------------ reference GEMM

// y[m][n] = sum_k Deq(W)[n][k] * x[m][k], binary32 accumulate.  One block per (n, 8 rows of x);
// each thread strides over k, then the block reduces.  Works for both layouts and any M.
constexpr int kRefRows = 8;
__global__ void __launch_bounds__(256) ref_gemm_kernel(MatDev m, int M, int xdt, int ydt) {
    __shared__ float red[kRefRows][256];
    int n = blockIdx.x, m0 = blockIdx.y * kRefRows;
    float acc[kRefRows];
    for (int i = 0; i < kRefRows; ++i) acc[i] = 0.f;
    for (int k = threadIdx.x; k < m.K; k += 256) {
        float w = deq_element(m, n, k);
        for (int i = 0; i < kRefRows; ++i)
            if (m0 + i < M) acc[i] = fmaf(w, load_as_f32(m.x, (size_t)(m0 + i) * m.K + k, xdt), acc[i]);
    }
    for (int i = 0; i < kRefRows; ++i) red[i][threadIdx.x] = acc[i];
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
        if ((int)threadIdx.x < s)
            for (int i = 0; i < kRefRows; ++i) red[i][threadIdx.x] += red[i][threadIdx.x + s];
        __syncthreads();
    }
    if (threadIdx.x < kRefRows && m0 + (int)threadIdx.x < M)
        store_from_f32(m.y, (size_t)(m0 + threadIdx.x) * m.N + n, ydt, red[threadIdx.x][0]);
}

hipError_t launch_ref_gemm(const MatDev& m, int M, int x_dtype, int y_dtype, hipStream_t s) {
    // grid.y is limited to 65535 blocks: M <= 524280 rows per launch is far beyond any use here.
    hipLaunchKernelGGL(ref_gemm_kernel, dim3(m.N, (M + kRefRows - 1) / kRefRows), dim3(256), 0, s, m, M,
                       x_dtype, y_dtype);
    return hipGetLastError();
}

}  // namespace rwkvq
