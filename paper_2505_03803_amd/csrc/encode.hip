// The two encoders of Sec. 2.2: round-to-nearest scalar quantization (Eq. "SQ") and assignment of
// each weight pair to its nearest codebook entry (Eq. "VQ").  Dense weights in, canonical-layout
// codes / indices out (per-row little-endian bit strings, see include/rwkvq.h).  Every
// floating-point step is one binary32 operation rounded to nearest even, written with the
// intrinsics so that the compiler can neither fuse nor reorder them: the codes are integers and
// must come out the same as from any other implementation of these steps.
#include "common.h"

namespace rwkvq {

__device__ __forceinline__ void wave_fence() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}
__device__ __forceinline__ float wave_min(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fminf(v, __shfl_xor(v, off, 64));
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
    return v;
}

// One wavefront per (row, group of 128 columns), two weights per lane.
//   s = (max - min) / 7 -> fp16;  z = -min / s -> fp16;  q = clamp(rne(w / s + z), 0, 7)
// with the stored (fp16) s and z; a constant group, or one whose fp16 scale would be zero, takes
// s = 1, z = -min.
__global__ void __launch_bounds__(256) sq_encode_kernel(const void* __restrict__ w, int wdt, int N, int K,
                                                        uint32_t* __restrict__ codes, uint16_t* __restrict__ scales,
                                                        uint16_t* __restrict__ zeros) {
    __shared__ uint32_t words[4][12];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int G = K / kGroup;
    const long long unit = (long long)blockIdx.x * 4 + wave;       // (row, group) index
    if (unit >= (long long)N * G) return;                           // whole wavefronts leave together
    const int n = (int)(unit / G), g = (int)(unit % G);
    const size_t e0 = (size_t)n * K + (size_t)g * kGroup + 2 * lane;
    const float w0 = load_as_f32(w, e0, wdt), w1 = load_as_f32(w, e0 + 1, wdt);
    const float lo = wave_min(fminf(w0, w1)), hi = wave_max(fmaxf(w0, w1));
    float s32 = __fdiv_rn(__fsub_rn(hi, lo), 7.0f);
    uint16_t s16 = f32_to_f16_bits(s32);
    if (hi == lo || (s16 & 0x7FFFu) == 0) { s32 = 1.0f; s16 = f32_to_f16_bits(1.0f); }
    const float s = f16_bits_to_f32(s16);
    const uint16_t z16 = f32_to_f16_bits(__fdiv_rn(-lo, s));
    const float z = f16_bits_to_f32(z16);
    const float q0 = fminf(fmaxf(rintf(__fadd_rn(__fdiv_rn(w0, s), z)), 0.0f), 7.0f);
    const float q1 = fminf(fmaxf(rintf(__fadd_rn(__fdiv_rn(w1, s), z)), 0.0f), 7.0f);
    // codes 2 lane, 2 lane + 1 are bits [6 lane, 6 lane + 6) of the group's 384-bit string
    // (the LDS unit serves a wavefront's requests in issue order; the fences only keep the
    // compiler from moving the accesses across these points)
    if (lane < 12) words[wave][lane] = 0u;
    wave_fence();
    const uint32_t field = (uint32_t)q0 | ((uint32_t)q1 << 3);
    const int pos = 6 * lane, wd = pos >> 5, sh = pos & 31;
    atomicOr(&words[wave][wd], field << sh);
    if (sh > 26) atomicOr(&words[wave][wd + 1], field >> (32 - sh));
    wave_fence();
    if (lane < 12) codes[(size_t)n * (3 * K / 32) + 12 * g + lane] = words[wave][lane];
    if (lane == 0) { scales[(size_t)n * G + g] = s16; zeros[(size_t)n * G + g] = z16; }
}

// One workgroup per 256 x 256 block, one thread per row of the block: 128 weight pairs, each
// compared with every entry of the block's codebook (staged in LDS as binary32, read by all
// threads at the same address: a broadcast).  Eight pairs share one pass over the entries.
template <int KBITS>
__global__ void __launch_bounds__(256) vq_assign_kernel(const void* __restrict__ w, int wdt, int N, int K,
                                                        const uint16_t* __restrict__ codebooks,
                                                        uint32_t* __restrict__ indices) {
    constexpr int E = 1 << KBITS;
    __shared__ float cb0[E], cb1[E];
    const int bj = blockIdx.x % (K / kBlock), bi = blockIdx.x / (K / kBlock);
    const uint16_t* cb = codebooks + ((size_t)bi * (K / kBlock) + bj) * E * 2;
    for (int e = threadIdx.x; e < E; e += 256) {
        cb0[e] = f16_bits_to_f32(cb[2 * e]);
        cb1[e] = f16_bits_to_f32(cb[2 * e + 1]);
    }
    __syncthreads();
    const int n = bi * kBlock + threadIdx.x;
    const size_t e0 = (size_t)n * K + (size_t)bj * kBlock;
    constexpr int wpr = KBITS == 6 ? 3 : 4;                        // output words per 16 pairs
    uint32_t* out = indices + (size_t)n * (K / 2 * KBITS / 32) + (size_t)bj * (kBlock / 2 * KBITS / 32);
    for (int c = 0; c < 8; ++c) {                                  // 16 pairs per step
        uint32_t idx[16];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            float v0[8], v1[8], best[8];
            uint32_t arg[8];
#pragma unroll
            for (int p = 0; p < 8; ++p) {
                v0[p] = load_as_f32(w, e0 + 32 * c + 16 * h + 2 * p, wdt);
                v1[p] = load_as_f32(w, e0 + 32 * c + 16 * h + 2 * p + 1, wdt);
                best[p] = __builtin_inff();
                arg[p] = 0u;
            }
            for (int e = 0; e < E; ++e) {
                const float c0 = cb0[e], c1 = cb1[e];
#pragma unroll
                for (int p = 0; p < 8; ++p) {
                    const float t0 = __fsub_rn(v0[p], c0), t1 = __fsub_rn(v1[p], c1);
                    const float d = __fadd_rn(__fmul_rn(t0, t0), __fmul_rn(t1, t1));
                    if (d < best[p]) { best[p] = d; arg[p] = (uint32_t)e; }   // strict: lowest index wins ties
                }
            }
#pragma unroll
            for (int p = 0; p < 8; ++p) idx[8 * h + p] = arg[p];
        }
        if (KBITS == 6) {
            unsigned long long lo = 0;                             // 16 x 6 bits = 96 bits
            uint32_t hi = 0;
#pragma unroll
            for (int p = 0; p < 10; ++p) lo |= (unsigned long long)idx[p] << (6 * p);
            lo |= (unsigned long long)(idx[10] & 0xFu) << 60;      // index 10 straddles bit 64
            hi = idx[10] >> 4;
#pragma unroll
            for (int p = 11; p < 16; ++p) hi |= idx[p] << (6 * p - 64);
            out[wpr * c + 0] = (uint32_t)lo;
            out[wpr * c + 1] = (uint32_t)(lo >> 32);
            out[wpr * c + 2] = hi;
        } else {
#pragma unroll
            for (int q = 0; q < 4; ++q)
                out[wpr * c + q] = idx[4 * q] | (idx[4 * q + 1] << 8) | (idx[4 * q + 2] << 16) | (idx[4 * q + 3] << 24);
        }
    }
}

hipError_t launch_sq_encode(const void* w, int wdt, int N, int K, uint32_t* codes, uint16_t* scales,
                            uint16_t* zeros, hipStream_t s) {
    const long long units = (long long)N * (K / kGroup);
    hipLaunchKernelGGL(sq_encode_kernel, dim3((unsigned)((units + 3) / 4)), dim3(256), 0, s, w, wdt, N, K, codes,
                       scales, zeros);
    return hipGetLastError();
}

hipError_t launch_vq_assign(const void* w, int wdt, int N, int K, int kbits, const uint16_t* codebooks,
                            uint32_t* indices, hipStream_t s) {
    const unsigned blocks = (unsigned)((N / kBlock) * (K / kBlock));
    if (kbits == 6) hipLaunchKernelGGL(vq_assign_kernel<6>, dim3(blocks), dim3(256), 0, s, w, wdt, N, K, codebooks, indices);
    else hipLaunchKernelGGL(vq_assign_kernel<8>, dim3(blocks), dim3(256), 0, s, w, wdt, N, K, codebooks, indices);
    return hipGetLastError();
}

}  // namespace rwkvq
