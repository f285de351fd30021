// The two encoders of Sec. 2.2: round-to-nearest scalar quantization (Eq. "SQ") and assignment of
// each weight pair to its nearest codebook entry (Eq. "VQ").  Dense weights in, canonical-layout
// codes / indices out (per-row little-endian bit strings, see include/rwkvq.h).  Every
// floating-point step is one binary32 operation rounded to nearest even, written with the
// intrinsics so that the compiler can neither fuse nor reorder them: the codes are integers and
// must come out the same as from any other implementation of these steps.
#include "common.h"

namespace rwkvq {

// min / max over the 16 lanes of a DPP row (quad permutes, then the two mirrors)
template <int CTRL>
__device__ __forceinline__ float dpp_get(float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}
__device__ __forceinline__ float row_min(float v) {
    v = fminf(v, dpp_get<0xB1>(v)); v = fminf(v, dpp_get<0x4E>(v));
    v = fminf(v, dpp_get<0x141>(v)); v = fminf(v, dpp_get<0x140>(v));
    return v;
}
__device__ __forceinline__ float row_max(float v) {
    v = fmaxf(v, dpp_get<0xB1>(v)); v = fmaxf(v, dpp_get<0x4E>(v));
    v = fmaxf(v, dpp_get<0x141>(v)); v = fmaxf(v, dpp_get<0x140>(v));
    return v;
}

// Sixteen lanes per (row, group of 128 columns), eight consecutive weights per lane (one 16-byte
// load for 16-bit weights), four groups per wavefront.
//   s = (max - min) / 7 -> fp16;  z = -min / s -> fp16;  q = clamp(rne(w / s + z), 0, 7)
// with the stored (fp16) s and z; a constant group, or one whose fp16 scale would be zero, takes
// s = 1, z = -min.  A lane's eight codes are 24 bits of the group's 384-bit string: the four lanes
// of a quad hold 96 bits = three words, assembled with one quad permute.
__global__ void __launch_bounds__(256) sq_encode_kernel(const void* __restrict__ w, int wdt, int N, int K,
                                                        uint32_t* __restrict__ codes, uint16_t* __restrict__ scales,
                                                        uint16_t* __restrict__ zeros) {
    const int lane = threadIdx.x & 63, sub = lane & 15;
    const long long units = (long long)N * (K / kGroup);
    long long unit = ((long long)blockIdx.x * 4 + (threadIdx.x >> 6)) * 4 + (lane >> 4);   // (row, group) index
    const bool live = unit < units;
    if (!live) unit = units - 1;                      // surplus rows of lanes redo the last group, store nothing
    const size_t e0 = (size_t)unit * kGroup + 8 * sub;   // groups are consecutive in a row-major matrix
    float v[8];
    if (wdt == DT_F32) {
        const float4_t a = __builtin_nontemporal_load((const float4_t*)((const float*)w + e0)), b = __builtin_nontemporal_load((const float4_t*)((const float*)w + e0 + 4));   // the dense weights are read once
        v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
    } else {
        const uint4_t p = __builtin_nontemporal_load((const uint4_t*)((const uint16_t*)w + e0));
        const uint32_t pw[4] = {p.x, p.y, p.z, p.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            v[2 * i] = wdt == DT_F16 ? f16_bits_to_f32((uint16_t)(pw[i] & 0xFFFFu)) : bf16_bits_to_f32((uint16_t)(pw[i] & 0xFFFFu));
            v[2 * i + 1] = wdt == DT_F16 ? f16_bits_to_f32((uint16_t)(pw[i] >> 16)) : bf16_bits_to_f32((uint16_t)(pw[i] >> 16));
        }
    }
    float lo = v[0], hi = v[0];
#pragma unroll
    for (int i = 1; i < 8; ++i) { lo = fminf(lo, v[i]); hi = fmaxf(hi, v[i]); }
    lo = row_min(lo);
    hi = row_max(hi);
    float s32 = __fdiv_rn(__fsub_rn(hi, lo), 7.0f);
    uint16_t s16 = f32_to_f16_bits(s32);
    if (hi == lo || (s16 & 0x7FFFu) == 0) s16 = f32_to_f16_bits(1.0f);
    const float s = f16_bits_to_f32(s16);
    const uint16_t z16 = f32_to_f16_bits(__fdiv_rn(-lo, s));
    const float z = f16_bits_to_f32(z16);
    uint32_t field = 0;                               // eight codes, 24 bits
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const float q = fminf(fmaxf(rintf(__fadd_rn(__fdiv_rn(v[i], s), z)), 0.0f), 7.0f);
        field |= (uint32_t)q << (3 * i);
    }
    // quad lanes 0..3 hold f0..f3: word0 = f0 | f1 << 24, word1 = f1 >> 8 | f2 << 16, word2 = f2 >> 16 | f3 << 8
    const uint32_t next = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)field, 0x39, 0xF, 0xF, true);   // quad_perm [1,2,3,0]
    const int ql = lane & 3;
    const uint32_t word = ql == 0 ? (field | (next << 24)) : ql == 1 ? ((field >> 8) | (next << 16))
                                                                     : ((field >> 16) | (next << 8));
    if (live && ql < 3) codes[(size_t)unit * 12 + 3 * (sub >> 2) + ql] = word;
    if (live && sub == 0) { scales[unit] = s16; zeros[unit] = z16; }
}

// Sixteen consecutive weights (eight pairs) starting at element e, widened to binary32, with
// 16-byte loads.
__device__ __forceinline__ void load_pairs8(const void* w, int wdt, size_t e, float (&v0)[8], float (&v1)[8]) {
    if (wdt == DT_F32) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float4_t a = *(const float4_t*)((const float*)w + e + 4 * i);
            v0[2 * i] = a.x; v1[2 * i] = a.y; v0[2 * i + 1] = a.z; v1[2 * i + 1] = a.w;
        }
    } else {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const uint4_t p = *(const uint4_t*)((const uint16_t*)w + e + 8 * i);
            const uint32_t pw[4] = {p.x, p.y, p.z, p.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint16_t lo = (uint16_t)(pw[j] & 0xFFFFu), hi = (uint16_t)(pw[j] >> 16);
                v0[4 * i + j] = wdt == DT_F16 ? f16_bits_to_f32(lo) : bf16_bits_to_f32(lo);
                v1[4 * i + j] = wdt == DT_F16 ? f16_bits_to_f32(hi) : bf16_bits_to_f32(hi);
            }
        }
    }
}

// Four workgroups per 256 x 256 block, each 64 rows; a thread takes one row and a quarter of its
// columns (the four threads of a row read 512 consecutive bytes of 16-bit weights):
// 32 weight pairs, each compared with every entry of the block's codebook (staged in LDS as
// binary32, read by all threads at the same address: a broadcast).  Eight pairs share one pass
// over the entries.
template <int KBITS>
__global__ void __launch_bounds__(256) vq_assign_kernel(const void* __restrict__ w, int wdt, int N, int K,
                                                        const uint16_t* __restrict__ codebooks,
                                                        uint32_t* __restrict__ indices) {
    constexpr int E = 1 << KBITS;
    __shared__ float cb0[E], cb1[E];
    const int quarter = blockIdx.x & 3, blk = blockIdx.x >> 2;
    const int bj = blk % (K / kBlock), bi = blk / (K / kBlock);
    const uint16_t* cb = codebooks + ((size_t)bi * (K / kBlock) + bj) * E * 2;
    for (int e = threadIdx.x; e < E; e += 256) {
        cb0[e] = f16_bits_to_f32(cb[2 * e]);
        cb1[e] = f16_bits_to_f32(cb[2 * e + 1]);
    }
    __syncthreads();
    const int n = bi * kBlock + 64 * quarter + (threadIdx.x >> 2), cq = threadIdx.x & 3;
    const size_t e0 = (size_t)n * K + (size_t)bj * kBlock + 64 * cq;
    constexpr int wpr = KBITS == 6 ? 3 : 4;                        // output words per 16 pairs
    uint32_t* out = indices + (size_t)n * (K / 2 * KBITS / 32) + (size_t)bj * (kBlock / 2 * KBITS / 32) + 2 * wpr * cq;
    for (int c = 0; c < 2; ++c) {                                  // 16 pairs per step
        uint32_t idx[16];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            float v0[8], v1[8], best[8];
            uint32_t arg[8];
            load_pairs8(w, wdt, e0 + 32 * c + 16 * h, v0, v1);
#pragma unroll
            for (int p = 0; p < 8; ++p) { best[p] = __builtin_inff(); arg[p] = 0u; }
#pragma unroll 4
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
    hipLaunchKernelGGL(sq_encode_kernel, dim3((unsigned)((units + 15) / 16)), dim3(256), 0, s, w, wdt, N, K, codes,
                       scales, zeros);
    return hipGetLastError();
}

hipError_t launch_vq_assign(const void* w, int wdt, int N, int K, int kbits, const uint16_t* codebooks,
                            uint32_t* indices, hipStream_t s) {
    const unsigned blocks = 4u * (unsigned)((N / kBlock) * (K / kBlock));
    if (kbits == 6) hipLaunchKernelGGL(vq_assign_kernel<6>, dim3(blocks), dim3(256), 0, s, w, wdt, N, K, codebooks, indices);
    else hipLaunchKernelGGL(vq_assign_kernel<8>, dim3(blocks), dim3(256), 0, s, w, wdt, N, K, codebooks, indices);
    return hipGetLastError();
}

}  // namespace rwkvq
