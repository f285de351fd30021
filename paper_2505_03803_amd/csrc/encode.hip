// The two encoders of Sec. 2.2: round-to-nearest scalar quantization (Eq. "SQ") and assignment of
// each weight pair to its nearest codebook entry (Eq. "VQ").  Dense weights in, canonical-layout
// codes / indices out (per-row little-endian bit strings, see include/rwkvq.h).  Every
// floating-point step is one binary32 operation rounded to nearest even, written with the
// intrinsics so that the compiler can neither fuse nor reorder them: the codes are integers and
// must come out the same as from any other implementation of these steps.
#include "common.h"

#ifndef RWKVQ_SQ_ENCODE_PASSES
#define RWKVQ_SQ_ENCODE_PASSES 1   // stretches of 32 groups per workgroup of the SQ encoder
#endif

namespace rwkvq {

// Three-operand minimum / maximum and one butterfly step of a minimum / maximum across lanes
// (the data-parallel-primitive form of the instruction reads its first operand from the partner
// lane).  Written as instructions: the C library forms first canonicalise every operand, which
// doubles their cost, and keep the cross-lane move a separate instruction.  The two idle cycles
// in front of a cross-lane read are the ones the architecture asks for after a vector write of
// the register it reads.
__device__ __forceinline__ float min3f(float a, float b, float c) {
    float r;
    asm("v_min3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}
__device__ __forceinline__ float max3f(float a, float b, float c) {
    float r;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}
#define RWKVQ_LANE_STEP(op, v, ctrl) \
    asm volatile("s_nop 1\n\t" op " %0, %1, %1 " ctrl " row_mask:0xf bank_mask:0xf" : "=v"(v) : "v"(v))
// over the eight lanes of half a DPP row: quad permutes [1,0,3,2] and [2,3,0,1], then the mirror of the half row
__device__ __forceinline__ float half_row_min(float v) {
    RWKVQ_LANE_STEP("v_min_f32_dpp", v, "quad_perm:[1,0,3,2]");
    RWKVQ_LANE_STEP("v_min_f32_dpp", v, "quad_perm:[2,3,0,1]");
    RWKVQ_LANE_STEP("v_min_f32_dpp", v, "row_half_mirror");
    return v;
}
__device__ __forceinline__ float half_row_max(float v) {
    RWKVQ_LANE_STEP("v_max_f32_dpp", v, "quad_perm:[1,0,3,2]");
    RWKVQ_LANE_STEP("v_max_f32_dpp", v, "quad_perm:[2,3,0,1]");
    RWKVQ_LANE_STEP("v_max_f32_dpp", v, "row_half_mirror");
    return v;
}

// v / d for a divisor d whose correctly rounded reciprocal r is at hand: q0 = rn(v * r), then
// correction steps q' = rn(q + rn(v - d * q) * r), whose residual one fused multiply-add gives
// exactly.  Two steps yield the correctly rounded quotient whenever nothing over- or underflows
// on the way (one makes q faithful, the second rounds it correctly: Markstein's theorem); for a
// dividend that is a bf16 or fp16 value and a divisor that is an fp16 value one step does
// (checked on the host over every such pair with the dividend zero or in [2^-60, 2^60]:
// tests/host/quotient_check.c).
template <int STEPS>
__device__ __forceinline__ float quotient(float v, float d, float r) {
    float q = __fmul_rn(v, r);
#pragma unroll
    for (int i = 0; i < STEPS; ++i) q = __fmaf_rn(__fmaf_rn(-d, q, v), r, q);
    return q;
}

// Eight lanes per (row, group of 128 columns); a lane holds columns 8 l .. 8 l + 7 and
// 64 + 8 l .. 64 + 8 l + 7 of the group (two fully coalesced 16-byte loads for 16-bit weights),
// eight groups per wavefront and pass; a workgroup makes U passes over consecutive stretches of
// 32 groups, with the loads of all passes issued before the first is used.
//   s = (max - min) / 7 -> fp16;  z = -min / s -> fp16;  q = clamp(rne(w / s + z), 0, 7)
// with the stored (fp16) s and z; a constant group, or one whose fp16 scale would be zero, takes
// s = 1, z = -min.  All divisions are exact (correctly rounded binary32): the 16 + 1 by s share
// one reciprocal, refined from the hardware's approximation by one Newton step, which lands on
// the correctly rounded reciprocal of every fp16 value when the approximation is within four
// units in the last place (checked on the host).  A lane whose values leave the range the short
// sequence is proven for (a non-zero magnitude outside [2^-60, 2^60], a non-finite scale) takes
// the hardware division sequence instead.
// A lane's eight codes of one half are 24 bits of the group's 384-bit string, gathered in a
// binary32 (an integer below 2^24, so every step is exact): the four lanes of a quad hold
// 96 bits = three words, assembled with one quad permute.
template <int STEPS>
__device__ __forceinline__ void sq_encode_group(const float (&v)[16], int lane, bool live, long long unit,
                                                uint32_t* __restrict__ codes, uint16_t* __restrict__ scales,
                                                uint16_t* __restrict__ zeros) {
    const int sub = lane & 7;
    float lo = min3f(v[0], v[1], v[2]), hi = max3f(v[0], v[1], v[2]);
#pragma unroll
    for (int i = 3; i < 15; i += 2) { lo = min3f(lo, v[i], v[i + 1]); hi = max3f(hi, v[i], v[i + 1]); }
    lo = min3f(lo, v[15], v[15]);
    hi = max3f(hi, v[15], v[15]);
    lo = half_row_min(lo);
    hi = half_row_max(hi);
    const float range = __fsub_rn(hi, lo);
    float s32;
    if (range >= 0x1p-40f && range <= 0x1p100f) s32 = quotient<2>(range, 7.0f, 0x1.24924ap-3f);   // rn(1 / 7)
    else s32 = __fdiv_rn(range, 7.0f);
    uint16_t s16 = f32_to_f16_bits(s32);
    if (hi == lo || (s16 & 0x7FFFu) == 0) s16 = f32_to_f16_bits(1.0f);
    const float s = f16_bits_to_f32(s16);
    const bool s_finite = (s16 & 0x7C00u) != 0x7C00u;
    float r = __builtin_amdgcn_rcpf(s);
    r = __fmaf_rn(__fmaf_rn(-s, r, 1.0f), r, r);
    const float alo = fabsf(lo);
    float zf;
    if (lo == 0.0f) zf = -lo;                         // a zero of the right sign (the short sequence loses the sign of a zero)
    else if (s_finite && alo >= 0x1p-60f && alo <= 0x1p60f) zf = quotient<STEPS>(-lo, s, r);
    else zf = __fdiv_rn(-lo, s);
    const uint16_t z16 = f32_to_f16_bits(zf);
    const float z = f16_bits_to_f32(z16);
    int emin = 0;                                     // binary exponents (value = m 2^e, 1/2 <= m < 1; zero counts as 0)
#pragma unroll
    for (int i = 0; i < 16; i += 2)
        emin = min(emin, min(__builtin_amdgcn_frexp_expf(v[i]), __builtin_amdgcn_frexp_expf(v[i + 1])));
    const bool plain = !s_finite || emin < -59 || !(fmaxf(alo, fabsf(hi)) <= 0x1p60f);
    float quo[16];
    if (!plain) {
#pragma unroll
        for (int i = 0; i < 16; ++i) quo[i] = quotient<STEPS>(v[i], s, r);
    } else {
#pragma unroll
        for (int i = 0; i < 16; ++i) quo[i] = __fdiv_rn(v[i], s);
    }
    uint32_t field[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        float acc = 0.0f;
#pragma unroll
        for (int i = 7; i >= 0; --i) {                // Horner in base 8: code i lands at bits 3 i .. 3 i + 2
            const float q = rintf(__builtin_amdgcn_fmed3f(__fadd_rn(quo[8 * h + i], z), 0.0f, 7.0f));
            acc = __fmaf_rn(acc, 8.0f, q);
        }
        field[h] = (uint32_t)acc;
    }
    // quad lanes 0..3 hold f0..f3: word0 = f0 | f1 << 24, word1 = f1 >> 8 | f2 << 16, word2 = f2 >> 16 | f3 << 8
    const int ql = lane & 3;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const uint32_t f = field[h];
        const uint32_t next = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)f, 0x39, 0xF, 0xF, true);   // quad_perm [1,2,3,0]
        const uint32_t word = ql == 0 ? (f | (next << 24)) : ql == 1 ? ((f >> 8) | (next << 16)) : ((f >> 16) | (next << 8));
        if (live && ql < 3) __builtin_nontemporal_store(word, codes + (size_t)unit * 12 + 6 * h + 3 * (sub >> 2) + ql);
    }
    if (live && sub == 0) { scales[unit] = s16; zeros[unit] = z16; }
}

template <int U, int WDT>
__global__ void __launch_bounds__(256) sq_encode_kernel(const void* __restrict__ w, int N, int K,
                                                        uint32_t* __restrict__ codes, uint16_t* __restrict__ scales,
                                                        uint16_t* __restrict__ zeros) {
    const int lane = threadIdx.x & 63, sub = lane & 7;
    const long long units = (long long)N * (K / kGroup);
    long long unit[U];                                // (row, group) indices
    bool live[U];
#pragma unroll
    for (int j = 0; j < U; ++j) {
        unit[j] = ((long long)blockIdx.x * U + j) * 32 + (threadIdx.x >> 6) * 8 + (lane >> 3);
        live[j] = unit[j] < units;
        if (!live[j]) unit[j] = units - 1;            // surplus rows of lanes redo the last group, store nothing
    }
    // groups are consecutive in a row-major matrix; the dense weights are read once
    if (WDT == DT_F32) {
        float4_t a[U][4];
#pragma unroll
        for (int j = 0; j < U; ++j) {
            const float* src = (const float*)w + (size_t)unit[j] * kGroup + 8 * sub;
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                a[j][2 * h] = __builtin_nontemporal_load((const float4_t*)(src + 64 * h));
                a[j][2 * h + 1] = __builtin_nontemporal_load((const float4_t*)(src + 64 * h + 4));
            }
        }
#pragma unroll
        for (int j = 0; j < U; ++j) {
            float v[16];
#pragma unroll
            for (int i = 0; i < 4; ++i) { v[4 * i] = a[j][i].x; v[4 * i + 1] = a[j][i].y; v[4 * i + 2] = a[j][i].z; v[4 * i + 3] = a[j][i].w; }
            sq_encode_group<2>(v, lane, live[j], unit[j], codes, scales, zeros);
        }
    } else {
        uint4_t p[U][2];
#pragma unroll
        for (int j = 0; j < U; ++j) {
            const uint16_t* src = (const uint16_t*)w + (size_t)unit[j] * kGroup + 8 * sub;
            p[j][0] = __builtin_nontemporal_load((const uint4_t*)src);
            p[j][1] = __builtin_nontemporal_load((const uint4_t*)(src + 64));
        }
#pragma unroll
        for (int j = 0; j < U; ++j) {
            const uint32_t pw[8] = {p[j][0].x, p[j][0].y, p[j][0].z, p[j][0].w, p[j][1].x, p[j][1].y, p[j][1].z, p[j][1].w};
            float v[16];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                v[2 * i] = WDT == DT_F16 ? f16_bits_to_f32((uint16_t)(pw[i] & 0xFFFFu)) : bf16_bits_to_f32((uint16_t)(pw[i] & 0xFFFFu));
                v[2 * i + 1] = WDT == DT_F16 ? f16_bits_to_f32((uint16_t)(pw[i] >> 16)) : bf16_bits_to_f32((uint16_t)(pw[i] >> 16));
            }
            sq_encode_group<1>(v, lane, live[j], unit[j], codes, scales, zeros);
        }
    }
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
    constexpr int U = RWKVQ_SQ_ENCODE_PASSES;
    const dim3 grid((unsigned)((units + 32 * U - 1) / (32 * U)));
    if (wdt == DT_F32) hipLaunchKernelGGL((sq_encode_kernel<U, DT_F32>), grid, dim3(256), 0, s, w, N, K, codes, scales, zeros);
    else if (wdt == DT_F16) hipLaunchKernelGGL((sq_encode_kernel<U, DT_F16>), grid, dim3(256), 0, s, w, N, K, codes, scales, zeros);
    else hipLaunchKernelGGL((sq_encode_kernel<U, DT_BF16>), grid, dim3(256), 0, s, w, N, K, codes, scales, zeros);
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
