// Element-wise multiplication weights (Sec. 3.2, "Codebook Optimization for Element-wise
// Multiplication") and the token-shift mix that consumes them (Eq. "time mixing r/k/v", Eq.
// "channel mixing r/k"):
//   clip_mean_kernel      the representative activation of a calibration batch: per position, the
//                         samples limited to their [p, 100 - p] percentile range, then averaged;
//   mu_kmeans_kernel      X^2-weighted Lloyd iterations on the weight's 2-vectors (the loss of Eq.
//                         "quantization loss of mul"), one workgroup per weight tensor;
//   token_shift_mix_kernel  mu_hat * x_t + (1 - mu_hat) * x_{t-1} for all projections of a layer
//                         in one pass over the activations, mu_hat looked up in its codebook.
// Every decision (argmin, percentile rank) is taken on binary32 / binary64 values computed with one
// rounding per operation in a fixed formula, so that any implementation of the same steps takes
// the same decisions.
#include "common.h"

#include <vector>

namespace rwkvq {

// ---------------------------------------------------------------------------------- clip_mean
// The order statistics are found by rank counting (rank of sample i = number of samples that sort
// before it, ties by sample index): B^2 comparisons per position.  B is a calibration batch (128 in
// Sec. 4).
//
// clip_mean_tile_kernel<P>: a workgroup takes P consecutive positions and stages all B samples of them
// in LDS (B x P floats); thread (position p, group g) ranks the samples g, g + G, ... of its position
// against all B (LDS reads of one row of the tile per step: consecutive banks), the four order
// statistics the percentiles need are left in LDS by whichever thread finds them, and one thread per
// position then forms the clipped mean as a binary64 sum in sample order.  The same comparisons and the
// same sum as the plain kernel below, which remains for batches too large for the tile.
template <int P>
__global__ void __launch_bounds__(256) clip_mean_tile_kernel(const void* __restrict__ x, int dt, int B, int n, int k_lo,
                                                             double f_lo, int k_hi, double f_hi, float* __restrict__ out) {
    extern __shared__ float tile[];                  // [B][P]
    __shared__ float stat[4][P];
    constexpr int G = 256 / P;
    const int tid = threadIdx.x, p = tid % P, g = tid / P;
    const int j0 = blockIdx.x * P, j = j0 + p;
    const bool live = j < n;
    for (int b = g; b < B; b += G) tile[b * P + p] = live ? load_as_f32(x, (size_t)b * n + j, dt) : 0.f;
    __syncthreads();
    const int k_lo1 = k_lo + 1 < B ? k_lo + 1 : B - 1, k_hi1 = k_hi + 1 < B ? k_hi + 1 : B - 1;
    for (int i = g; i < B; i += G) {
        const float vi = tile[i * P + p];
        int rank = 0;
        for (int b = 0; b < B; ++b) {
            const float vb = tile[b * P + p];
            rank += (vb < vi || (vb == vi && b < i)) ? 1 : 0;
        }
        if (rank == k_lo) stat[0][p] = vi;
        if (rank == k_lo1) stat[1][p] = vi;
        if (rank == k_hi) stat[2][p] = vi;
        if (rank == k_hi1) stat[3][p] = vi;
    }
    __syncthreads();
    if (g == 0 && live) {
        const float v_lo = stat[0][p], v_lo1 = stat[1][p], v_hi = stat[2][p], v_hi1 = stat[3][p];
        const double lo = __dadd_rn((double)v_lo, __dmul_rn(f_lo, __dsub_rn((double)v_lo1, (double)v_lo)));
        const double hi = __dadd_rn((double)v_hi, __dmul_rn(f_hi, __dsub_rn((double)v_hi1, (double)v_hi)));
        double acc = 0.0;
        for (int b = 0; b < B; ++b) {                   // sample order: the sum is reproducible
            double v = (double)tile[b * P + p];
            v = v < lo ? lo : v;
            v = v > hi ? hi : v;
            acc = __dadd_rn(acc, v);
        }
        out[j] = (float)(acc / (double)B);
    }
}

// One thread per position, samples re-read from memory: any batch size.
__global__ void __launch_bounds__(256) clip_mean_kernel(const void* __restrict__ x, int dt, int B, int n, int k_lo,
                                                        double f_lo, int k_hi, double f_hi, float* __restrict__ out) {
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (j >= n) return;
    const int k_lo1 = k_lo + 1 < B ? k_lo + 1 : B - 1, k_hi1 = k_hi + 1 < B ? k_hi + 1 : B - 1;
    float v_lo = 0.f, v_lo1 = 0.f, v_hi = 0.f, v_hi1 = 0.f;
    for (int i = 0; i < B; ++i) {
        const float vi = load_as_f32(x, (size_t)i * n + j, dt);
        int rank = 0;
        for (int b = 0; b < B; ++b) {
            const float vb = load_as_f32(x, (size_t)b * n + j, dt);
            rank += (vb < vi || (vb == vi && b < i)) ? 1 : 0;
        }
        if (rank == k_lo) v_lo = vi;
        if (rank == k_lo1) v_lo1 = vi;
        if (rank == k_hi) v_hi = vi;
        if (rank == k_hi1) v_hi1 = vi;
    }
    // linear interpolation between neighbouring order statistics, binary64, one rounding per step
    const double lo = __dadd_rn((double)v_lo, __dmul_rn(f_lo, __dsub_rn((double)v_lo1, (double)v_lo)));
    const double hi = __dadd_rn((double)v_hi, __dmul_rn(f_hi, __dsub_rn((double)v_hi1, (double)v_hi)));
    double acc = 0.0;
    for (int b = 0; b < B; ++b) {                       // sample order: the sum is reproducible
        double v = (double)load_as_f32(x, (size_t)b * n + j, dt);
        v = v < lo ? lo : v;
        v = v > hi ? hi : v;
        acc = __dadd_rn(acc, v);
    }
    out[j] = (float)(acc / (double)B);
}

hipError_t launch_clip_mean(const void* x, int dt, int B, int n, int k_lo, double f_lo, int k_hi, double f_hi,
                            float* out, hipStream_t s) {
    // the tile of B x P floats has to fit 64 KB of LDS: 64 positions per workgroup up to B = 256, 16 up to 1024
    if (B <= 256)
        hipLaunchKernelGGL(clip_mean_tile_kernel<64>, dim3((n + 63) / 64), dim3(256), (size_t)B * 64 * 4, s, x, dt, B, n, k_lo, f_lo, k_hi, f_hi, out);
    else if (B <= 1024)
        hipLaunchKernelGGL(clip_mean_tile_kernel<16>, dim3((n + 15) / 16), dim3(256), (size_t)B * 16 * 4, s, x, dt, B, n, k_lo, f_lo, k_hi, f_hi, out);
    else
        hipLaunchKernelGGL(clip_mean_kernel, dim3((n + 255) / 256), dim3(256), 0, s, x, dt, B, n, k_lo, f_lo, k_hi, f_hi, out);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------- weighted KMeans
constexpr int kMuMaxTensors = 64;
struct MuTensor {
    const void* mu;          // n elements, storage type of the launch
    const float* xbar;       // n representative activations
    uint16_t* cb;            // in: initial entries, out: final entries; fp16 [E][2]
    uint8_t* idx;            // out: n / 2 indices
    int n, pad;
};
struct MuArgs {
    MuTensor t[kMuMaxTensors];
    int dt, kbits, iters, pad;
};

// binary64 -> fp16 with a single rounding: truncate to binary32, keep inexactness in the last bit
// (round to odd), then let the binary32 -> fp16 conversion round to nearest even.
__device__ __forceinline__ uint16_t f64_to_f16_bits(double d) {
    float f = __double2float_rz(d);
    if ((double)f != d) f = __uint_as_float(__float_as_uint(f) | 1u);
    return f32_to_f16_bits(f);
}

// One workgroup per weight tensor.  The vectors go through LDS in chunks of 2048: every vector of a chunk is
// assigned to its cheapest entry (index, weight and value staged in LDS), then the sums of an entry's
// coordinate are continued by S = 1024 / (2 E) threads, each over a contiguous share of the chunk in index
// order; after the last chunk the S partial sums are added in share order.  Binary64 sums in a fixed order:
// a call gives the same codebook every time.
template <int E>
__global__ void __launch_bounds__(1024) mu_kmeans_kernel(MuArgs a) {
    constexpr int S = 1024 / (2 * E);                 // threads per (entry, coordinate)
    constexpr int kChunk = 2048, kPer = kChunk / S;   // vectors per chunk and per share
    constexpr int kRow = kPer + 1;                    // padded: the S shares of a chunk start in different LDS banks
    __shared__ float cb[E][2];
    __shared__ uint32_t s_idx[S * kRow];
    __shared__ float s_m[S * kRow][2], s_w[S * kRow][2];
    __shared__ double num[2 * E][S], den[2 * E][S];
    const MuTensor t = a.t[blockIdx.x];
    const int V = t.n >> 1, tid = threadIdx.x;
    for (int e = tid; e < E; e += 1024) {
        cb[e][0] = f16_bits_to_f32(t.cb[2 * e]);
        cb[e][1] = f16_bits_to_f32(t.cb[2 * e + 1]);
    }
    __syncthreads();
    const int pair = tid / S, seg = tid % S;          // update phase: pair = 2 e + coordinate
    for (int it = 0; it <= a.iters; ++it) {
        const bool last = it == a.iters;
        double sn = 0.0, sd = 0.0;
        for (int c0 = 0; c0 < V; c0 += kChunk) {
#pragma unroll
            for (int h = 0; h < kChunk / 1024; ++h) {
                const int vl = h * 1024 + tid, v = c0 + vl;
                const int slot = (vl / kPer) * kRow + vl % kPer;
                if (v < V) {
                    const float m0 = load_as_f32(t.mu, 2 * (size_t)v, a.dt), m1 = load_as_f32(t.mu, 2 * (size_t)v + 1, a.dt);
                    const float x0 = t.xbar[2 * (size_t)v], x1 = t.xbar[2 * (size_t)v + 1];
                    const float w0 = __fmul_rn(x0, x0), w1 = __fmul_rn(x1, x1);
                    int best = 0;
                    float bestc = __builtin_inff();
                    for (int e = 0; e < E; ++e) {
                        const float t0 = __fsub_rn(m0, cb[e][0]), t1 = __fsub_rn(m1, cb[e][1]);
                        const float c = __fadd_rn(__fmul_rn(w0, __fmul_rn(t0, t0)), __fmul_rn(w1, __fmul_rn(t1, t1)));
                        if (c < bestc) { bestc = c; best = e; }
                    }
                    if (last) t.idx[v] = (uint8_t)best;
                    s_idx[slot] = (uint32_t)best;
                    s_m[slot][0] = m0; s_m[slot][1] = m1; s_w[slot][0] = w0; s_w[slot][1] = w1;
                } else {
                    s_idx[slot] = 0xFFFFFFFFu;       // past the end: matches no entry
                }
            }
            if (last) continue;                       // the final pass only assigns
            __syncthreads();
            {
                const uint32_t e = (uint32_t)(pair >> 1);
                const int c = pair & 1;
                for (int i = 0; i < kPer; ++i) {
                    const int slot = seg * kRow + i;
                    const bool mine = s_idx[slot] == e;
                    const double w = (double)s_w[slot][c];
                    // the product of two binary32 values is exact in binary64; vectors of other entries add +0
                    sn += mine ? w * (double)s_m[slot][c] : 0.0;
                    sd += mine ? w : 0.0;
                }
            }
            __syncthreads();
        }
        if (last) break;
        num[pair][seg] = sn;
        den[pair][seg] = sd;
        __syncthreads();
        for (int p = tid; p < 2 * E; p += 1024) {
            double tn = 0.0, td = 0.0;
#pragma unroll
            for (int g = 0; g < S; ++g) { tn += num[p][g]; td += den[p][g]; }
            if (td > 0.0) (&cb[0][0])[p] = f16_bits_to_f32(f64_to_f16_bits(tn / td));
        }
        __syncthreads();
    }
    __syncthreads();
    for (int e = tid; e < 2 * E; e += 1024) t.cb[e] = f32_to_f16_bits((&cb[0][0])[e]);
}

hipError_t launch_mu_codebook(const void* const* mus, const float* const* xbars, const int* n_elems, int n_tensors,
                              int dt, int kbits, int iters, void* const* cbs, uint8_t* const* idx, hipStream_t s) {
    for (int base = 0; base < n_tensors; base += kMuMaxTensors) {
        MuArgs a;
        const int cnt = n_tensors - base < kMuMaxTensors ? n_tensors - base : kMuMaxTensors;
        for (int i = 0; i < kMuMaxTensors; ++i) {
            const int k = base + (i < cnt ? i : 0);
            a.t[i] = MuTensor{mus[k], xbars[k], (uint16_t*)cbs[k], idx[k], n_elems[k], 0};
        }
        a.dt = dt; a.kbits = kbits; a.iters = iters; a.pad = 0;
        if (kbits == 6) hipLaunchKernelGGL(mu_kmeans_kernel<64>, dim3(cnt), dim3(1024), 0, s, a);
        else hipLaunchKernelGGL(mu_kmeans_kernel<256>, dim3(cnt), dim3(1024), 0, s, a);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

// ---------------------------------------------------------------------------------- token-shift mix
constexpr int kMixMaxProj = 8;
struct MixArgs {
    const void* x;           // [M][d]
    const void* x_prev;      // [d]: the token before row 0
    const uint8_t* idx[kMixMaxProj];    // [d / 2] per projection
    const uint16_t* cb[kMixMaxProj];    // fp16 [E][2] per projection
    void* out[kMixMaxProj];             // [M][d] per projection
    int M, d, dt, n_proj, E, pad;
};

// A thread owns 8 consecutive channels of one row: one 16-byte load of x_t, one of x_{t-1}, and per
// projection four index bytes, four codebook look-ups (codebooks staged in LDS) and one 16-byte
// store.  HBM-bound: 2 (n_proj + 1) bytes per element (x_{t-1} is x_t's neighbouring row, a cache hit).
template <bool BF16> struct MixElem;
template <> struct MixElem<true> {
    static __device__ __forceinline__ void widen(uint32_t w, float& lo, float& hi) {
        lo = __uint_as_float(w << 16); hi = __uint_as_float(w & 0xFFFF0000u);
    }
    static __device__ __forceinline__ uint32_t narrow(float lo, float hi) {      // v_cvt_pk_bf16_f32: nearest even
        typedef __bf16 bf2 __attribute__((ext_vector_type(2)));
        bf2 v = {(__bf16)lo, (__bf16)hi};
        return __builtin_bit_cast(uint32_t, v);
    }
};
template <> struct MixElem<false> {
    static __device__ __forceinline__ void widen(uint32_t w, float& lo, float& hi) {
        const half2_t h = __builtin_bit_cast(half2_t, w);
        const half_t a = h.x, b = h.y;
        lo = (float)a; hi = (float)b;
    }
    static __device__ __forceinline__ uint32_t narrow(float lo, float hi) {
        half2_t v = {(half_t)lo, (half_t)hi};
        return __builtin_bit_cast(uint32_t, v);
    }
};

template <bool BF16>
__global__ void __launch_bounds__(256) token_shift_mix_kernel(MixArgs a) {
    __shared__ uint32_t cbs[kMixMaxProj][256];
    for (int i = threadIdx.x; i < a.n_proj * a.E; i += 256) {
        const int p = i / a.E, e = i - p * a.E;
        cbs[p][e] = ((const uint32_t*)a.cb[p])[e];
    }
    __syncthreads();
    const int chunks = a.d >> 3;
    // Workgroups are dealt round-robin to the 8 XCDs, each with its own L2: give every XCD one
    // contiguous range of rows, so that x_{t-1} (the row above) is in the L2 that just read it as x_t
    // (with the plain order the two reads of a row came from different XCDs: twice the fetches).
    const int per_xcd = gridDim.x >> 3;                    // the grid is a multiple of 8 workgroups
    const long long blk = (long long)(blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    const long long g = blk * 256 + threadIdx.x;
    if (g >= (long long)a.M * chunks) return;
    const int row = (int)(g / chunks), c = (int)(g - (long long)row * chunks);
    const uint4_t xt = ((const uint4_t*)a.x)[(size_t)row * chunks + c];
    const uint4_t xp = row == 0 ? ((const uint4_t*)a.x_prev)[c] : ((const uint4_t*)a.x)[(size_t)(row - 1) * chunks + c];
    const uint32_t xtw[4] = {xt.x, xt.y, xt.z, xt.w}, xpw[4] = {xp.x, xp.y, xp.z, xp.w};
    float t[8], u[8];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        MixElem<BF16>::widen(xtw[q], t[2 * q], t[2 * q + 1]);
        MixElem<BF16>::widen(xpw[q], u[2 * q], u[2 * q + 1]);
    }
    for (int p = 0; p < a.n_proj; ++p) {
        const uint32_t four = ((const uint32_t*)a.idx[p])[c];      // channels 8c..8c+7 = vectors 4c..4c+3
        uint32_t ow[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            float m0, m1;
            MixElem<false>::widen(cbs[p][(four >> (8 * q)) & 255u], m0, m1);
            const float o0 = __fadd_rn(__fmul_rn(m0, t[2 * q]), __fmul_rn(__fsub_rn(1.0f, m0), u[2 * q]));
            const float o1 = __fadd_rn(__fmul_rn(m1, t[2 * q + 1]), __fmul_rn(__fsub_rn(1.0f, m1), u[2 * q + 1]));
            ow[q] = MixElem<BF16>::narrow(o0, o1);
        }
        // written once, read by a later launch: stored with the non-temporal hint, so that the outputs do not
        // displace the rows of x (each read twice, as x_t and as x_{t-1}) from the L2
        __builtin_nontemporal_store(uint4_t{ow[0], ow[1], ow[2], ow[3]}, (uint4_t*)a.out[p] + (size_t)row * chunks + c);
    }
}

hipError_t launch_token_shift_mix(const void* x, const void* x_prev, int dt, int M, int d, const uint8_t* const* idx,
                                  const void* const* cbs, int kbits, int n_proj, void* const* outs, hipStream_t s) {
    MixArgs a;
    a.x = x; a.x_prev = x_prev;
    for (int p = 0; p < kMixMaxProj; ++p) {
        const int k = p < n_proj ? p : 0;
        a.idx[p] = idx[k]; a.cb[p] = (const uint16_t*)cbs[k]; a.out[p] = outs[k];
    }
    a.M = M; a.d = d; a.dt = dt; a.n_proj = n_proj; a.E = 1 << kbits; a.pad = 0;
    const long long threads = (long long)M * (d >> 3);
    const dim3 grid((unsigned)((((threads + 255) / 256) + 7) / 8 * 8));
    if (dt == DT_BF16) hipLaunchKernelGGL(token_shift_mix_kernel<true>, grid, dim3(256), 0, s, a);
    else hipLaunchKernelGGL(token_shift_mix_kernel<false>, grid, dim3(256), 0, s, a);
    return hipGetLastError();
}

}  // namespace rwkvq
