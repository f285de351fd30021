// Element-wise operators of the RWKV block between the quantized projections (App. A.1):
//   wkv_kernel        Eq. "time mixing wkv" carried as a running state, times the gate sigma(r_t)
//                     of Eq. "time mixing o" (the vector that W_o multiplies);
//   relu2_kernel      max(k'_t, 0)^2, the vector that W'_v multiplies (Eq. "channel mixing o");
//   gate_kernel       sigma(r'_t) (.) y, the output of channel mixing.
// All arithmetic is binary32; inputs and outputs are the 16-bit activation type.
//
// wkv as a state.  For channel c, Eq. "time mixing wkv" is num_t / den_t with
//   num_t = sum_{i<t} exp(-(t-1-i) w + k_i) v_i + exp(u + k_t) v_t,   den_t likewise without v.
// The sums over i < t obey  S_{t+1} = exp(-w) S_t + exp(k_t) v_t,  so three numbers per channel carry
// them: (a, b, p) with  sum_{i<t} ... v_i = a exp(p)  and  sum_{i<t} ... = b exp(p).  p is the largest
// exponent seen so far, which keeps every exp() argument <= 0: no overflow for any key.  A fresh
// sequence starts from a = b = 0 and p = -1e38 (the empty sums), which makes wkv_1 = v_1.
#include "common.h"

namespace rwkvq {

template <bool BF16>
__device__ __forceinline__ float ld16(const uint16_t* p, size_t i) {
    return BF16 ? bf16_bits_to_f32(p[i]) : f16_bits_to_f32(p[i]);
}
template <bool BF16>
__device__ __forceinline__ uint16_t st16(float v) {
    return BF16 ? f32_to_bf16_bits(v) : f32_to_f16_bits(v);
}

// One thread per channel, tokens in order.  The loads of kTok tokens are issued together so that a
// chunk (M > 1) is not one memory round trip per token.
constexpr int kTok = 8;
constexpr int kWkvChunkedMinTokens = 128;   // from here on the time-parallel kernel below
template <bool BF16>
__global__ void __launch_bounds__(64) wkv_kernel(const uint16_t* __restrict__ r, const uint16_t* __restrict__ k,
                                                 const uint16_t* __restrict__ v, int M, int d,
                                                 const float* __restrict__ w, const float* __restrict__ u,
                                                 float* __restrict__ state, uint16_t* __restrict__ out) {
    const int c = blockIdx.x * 64 + threadIdx.x;
    if (c >= d) return;
    float a = state[c], b = state[(size_t)d + c], p = state[2 * (size_t)d + c];
    const float wc = w[c], uc = u[c];
    for (int t0 = 0; t0 < M; t0 += kTok) {
        float rr[kTok], kk[kTok], vv[kTok];
#pragma unroll
        for (int j = 0; j < kTok; ++j) {
            const int t = t0 + j < M ? t0 + j : M - 1;              // tail: re-read the last token, not used
            const size_t at = (size_t)t * d + c;
            rr[j] = ld16<BF16>(r, at); kk[j] = ld16<BF16>(k, at); vv[j] = ld16<BF16>(v, at);
        }
#pragma unroll
        for (int j = 0; j < kTok; ++j) {
            if (t0 + j < M) {
                // output of token t: past sums (a, b) exp(p) plus the current token with the bonus u;
                // then the sums advanced: decayed by exp(-w), the current token added without the bonus
                out[(size_t)(t0 + j) * d + c] = st16<BF16>(gate_f32(rr[j], wkv_out(a, b, p, uc, kk[j], vv[j])));
                wkv_advance(a, b, p, wc, kk[j], vv[j]);
            }
        }
    }
    state[c] = a; state[(size_t)d + c] = b; state[2 * (size_t)d + c] = p;
}

// Chunks of many tokens (prefill): the recurrence is linear in the carried sums, S_out = exp(-n w) S_in
// + (the sums of the n tokens alone), so the tokens are cut into kChunks pieces that run side by side.
// A workgroup owns 16 channels; thread (channel, piece) first runs its piece from the empty state,
// 16 threads then chain the pieces (64 merges per channel) and leave the state in front of every
// piece in LDS, and each thread runs its piece again from there, now with outputs.  Twice the
// arithmetic, 64 times the parallelism.  The merges re-associate the sums: the result agrees with the
// token-by-token kernel to rounding, not bit for bit.
constexpr int kChunks = 64, kWgChannels = 16;

template <bool BF16>
__global__ void __launch_bounds__(kChunks * kWgChannels) wkv_chunked_kernel(
    const uint16_t* __restrict__ r, const uint16_t* __restrict__ k, const uint16_t* __restrict__ v, int M, int d,
    const float* __restrict__ w, const float* __restrict__ u, float* __restrict__ state, uint16_t* __restrict__ out) {
    __shared__ float loc[3][kChunks][kWgChannels];        // sums of piece i alone
    __shared__ float in[3][kChunks][kWgChannels];         // sums in front of piece i
    const int cc = threadIdx.x & (kWgChannels - 1), ch = threadIdx.x / kWgChannels;
    const int c = blockIdx.x * kWgChannels + cc;
    const bool live = c < d;
    const int L = (M + kChunks - 1) / kChunks;
    const int t0 = ch * L < M ? ch * L : M, t1 = t0 + L < M ? t0 + L : M;      // piece [t0, t1), may be empty
    const float wc = live ? w[c] : 0.f, uc = live ? u[c] : 0.f;

    float a = 0.f, b = 0.f, p = -1e38f;
    if (live) {
        for (int tb = t0; tb < t1; tb += kTok) {
            float kk[kTok], vv[kTok];
#pragma unroll
            for (int j = 0; j < kTok; ++j) {
                const int t = tb + j < t1 ? tb + j : t1 - 1;
                kk[j] = ld16<BF16>(k, (size_t)t * d + c); vv[j] = ld16<BF16>(v, (size_t)t * d + c);
            }
#pragma unroll
            for (int j = 0; j < kTok; ++j)
                if (tb + j < t1) wkv_advance(a, b, p, wc, kk[j], vv[j]);
        }
    }
    loc[0][ch][cc] = a; loc[1][ch][cc] = b; loc[2][ch][cc] = p;
    __syncthreads();
    if (ch == 0 && live) {
        float A = state[c], Bs = state[(size_t)d + c], P = state[2 * (size_t)d + c];
        for (int i = 0; i < kChunks; ++i) {
            in[0][i][cc] = A; in[1][i][cc] = Bs; in[2][i][cc] = P;
            const int s0 = i * L < M ? i * L : M, s1 = s0 + L < M ? s0 + L : M;
            if (s1 > s0) {
                const float Pd = P - (float)(s1 - s0) * wc;                     // n tokens of decay
                const float lp = loc[2][i][cc];
                const float q = fmaxf(Pd, lp);
                const float e1 = expf(Pd - q), e2 = expf(lp - q);
                A = e1 * A + e2 * loc[0][i][cc];
                Bs = e1 * Bs + e2 * loc[1][i][cc];
                P = q;
            }
        }
        state[c] = A; state[(size_t)d + c] = Bs; state[2 * (size_t)d + c] = P;
    }
    __syncthreads();
    if (!live) return;
    a = in[0][ch][cc]; b = in[1][ch][cc]; p = in[2][ch][cc];
    for (int tb = t0; tb < t1; tb += kTok) {
        float rr[kTok], kk[kTok], vv[kTok];
#pragma unroll
        for (int j = 0; j < kTok; ++j) {
            const int t = tb + j < t1 ? tb + j : t1 - 1;
            const size_t at = (size_t)t * d + c;
            rr[j] = ld16<BF16>(r, at); kk[j] = ld16<BF16>(k, at); vv[j] = ld16<BF16>(v, at);
        }
#pragma unroll
        for (int j = 0; j < kTok; ++j) {
            if (tb + j < t1) {
                out[(size_t)(tb + j) * d + c] = st16<BF16>(gate_f32(rr[j], wkv_out(a, b, p, uc, kk[j], vv[j])));
                wkv_advance(a, b, p, wc, kk[j], vv[j]);
            }
        }
    }
}

// 8 values per thread (one 16-byte load per operand).  OP 0: max(x, 0)^2;  OP 1: sigmoid(x) * y.
template <bool BF16, int OP>
__global__ void __launch_bounds__(256) pointwise_kernel(const uint16_t* __restrict__ x, const uint16_t* __restrict__ y,
                                                        long long n, uint16_t* __restrict__ out) {
    const long long i0 = ((long long)blockIdx.x * 256 + threadIdx.x) * 8;
    if (i0 >= n) return;
    if (i0 + 8 <= n) {
        const uint4 xv = *(const uint4*)(x + i0);
        uint4 yv = xv;
        if (OP == 1) yv = *(const uint4*)(y + i0);
        const uint32_t xs[4] = {xv.x, xv.y, xv.z, xv.w}, ys[4] = {yv.x, yv.y, yv.z, yv.w};
        uint32_t o[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            float r[2];
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const uint16_t xb = (uint16_t)(xs[j] >> (16 * h)), yb = (uint16_t)(ys[j] >> (16 * h));
                const float xf = BF16 ? bf16_bits_to_f32(xb) : f16_bits_to_f32(xb);
                if (OP == 0) {
                    const float m = fmaxf(xf, 0.0f);
                    r[h] = m * m;
                } else {
                    const float yf = BF16 ? bf16_bits_to_f32(yb) : f16_bits_to_f32(yb);
                    r[h] = gate_f32(xf, yf);
                }
            }
            o[j] = (uint32_t)st16<BF16>(r[0]) | ((uint32_t)st16<BF16>(r[1]) << 16);
        }
        *(uint4*)(out + i0) = make_uint4(o[0], o[1], o[2], o[3]);
    } else {
        for (long long i = i0; i < n; ++i) {
            const float xf = ld16<BF16>(x, (size_t)i);
            float r;
            if (OP == 0) {
                const float m = fmaxf(xf, 0.0f);
                r = m * m;
            } else {
                r = gate_f32(xf, ld16<BF16>(y, (size_t)i));
            }
            out[i] = st16<BF16>(r);
        }
    }
}

hipError_t launch_wkv(const void* r, const void* k, const void* v, int dt, int M, int d, const float* w, const float* u,
                      float* state, void* out, hipStream_t s) {
    if (M >= kWkvChunkedMinTokens) {
        const dim3 grid((d + kWgChannels - 1) / kWgChannels), block(kChunks * kWgChannels);
        if (dt == DT_BF16)
            hipLaunchKernelGGL(wkv_chunked_kernel<true>, grid, block, 0, s, (const uint16_t*)r, (const uint16_t*)k,
                               (const uint16_t*)v, M, d, w, u, state, (uint16_t*)out);
        else
            hipLaunchKernelGGL(wkv_chunked_kernel<false>, grid, block, 0, s, (const uint16_t*)r, (const uint16_t*)k,
                               (const uint16_t*)v, M, d, w, u, state, (uint16_t*)out);
        return hipGetLastError();
    }
    const dim3 grid((d + 63) / 64), block(64);
    if (dt == DT_BF16)
        hipLaunchKernelGGL(wkv_kernel<true>, grid, block, 0, s, (const uint16_t*)r, (const uint16_t*)k, (const uint16_t*)v,
                           M, d, w, u, state, (uint16_t*)out);
    else
        hipLaunchKernelGGL(wkv_kernel<false>, grid, block, 0, s, (const uint16_t*)r, (const uint16_t*)k, (const uint16_t*)v,
                           M, d, w, u, state, (uint16_t*)out);
    return hipGetLastError();
}

hipError_t launch_pointwise(int op, const void* x, const void* y, int dt, long long n, void* out, hipStream_t s) {
    const dim3 grid((unsigned)((n + 2047) / 2048)), block(256);
    const uint16_t* xp = (const uint16_t*)x;
    const uint16_t* yp = (const uint16_t*)y;
    uint16_t* op_ = (uint16_t*)out;
    if (op == 0) {
        if (dt == DT_BF16) hipLaunchKernelGGL((pointwise_kernel<true, 0>), grid, block, 0, s, xp, yp, n, op_);
        else hipLaunchKernelGGL((pointwise_kernel<false, 0>), grid, block, 0, s, xp, yp, n, op_);
    } else {
        if (dt == DT_BF16) hipLaunchKernelGGL((pointwise_kernel<true, 1>), grid, block, 0, s, xp, yp, n, op_);
        else hipLaunchKernelGGL((pointwise_kernel<false, 1>), grid, block, 0, s, xp, yp, n, op_);
    }
    return hipGetLastError();
}

}  // namespace rwkvq
