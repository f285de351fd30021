// The coarse-to-fine proxy of Sec. 3.1 ("Coarse-grained Proxy", "Fine-grained Proxy") for weight
// matrices stored as fp16 or bf16.
//
// The paper sorts the flattened weights and works on the intervals between neighbours.  Sixteen-bit
// weights take at most 65 536 distinct values, so the sorted sequence is fully described by how
// often each value occurs: one pass over the matrix builds that histogram (HBM-bound, the only
// part that touches the matrix), and everything else is a sum over at most 65 535 non-zero
// intervals plus a closed-form term for the intervals of length zero between equal weights:
//
//   n = oc*ic - 1 intervals, sum(G) = max - min, t_i = G_i / (sum(G) / n) = n G'_i
//   P_c = ln n - H(G')           = (1/n) sum_i t_i ln t_i                 (0 ln 0 := 0)
//   v_k |M_k| = n^k/(k(k-1)) |sum_i delta_i^k| / n = |sum_i (t_i - 1)^k| / (n k (k-1))
//
// Both right-hand sides are the paper's expressions with G' = t/n substituted; they keep every
// quantity of order one where n^k delta^k would leave the range of the arithmetic.  All sums are
// binary64 in a fixed order, so results are reproducible bit for bit.
#include "common.h"

namespace rwkvq {

constexpr int kProxyBins = 65536;
constexpr int kHistThreads = 512;
constexpr int kHistChunk = 61440;       // elements between two flushes: < 65 536, so the 16-bit
                                        // counters packed two per LDS word cannot overflow
static_assert(kHistChunk % (8 * kHistThreads) == 0, "whole 16-byte loads per thread");

// Order-preserving map of a sign-magnitude 16-bit float pattern to an unsigned key.
__device__ __forceinline__ uint32_t sort_key(uint32_t bits) {
    return (bits & 0x8000u) ? (~bits & 0xFFFFu) : (bits | 0x8000u);
}
__device__ __forceinline__ uint32_t key_bits(uint32_t key) {
    return (key & 0x8000u) ? (key & 0x7FFFu) : (~key & 0xFFFFu);
}
__device__ __forceinline__ double key_value(uint32_t key, int dtype) {
    const uint16_t b = (uint16_t)key_bits(key);
    return dtype == DT_F16 ? (double)f16_bits_to_f32(b) : (double)bf16_bits_to_f32(b);
}

__global__ void __launch_bounds__(256) proxy_clear_kernel(uint32_t* hist) {
    hist[blockIdx.x * 256 + threadIdx.x] = 0u;
}

// Histogram of the 16-bit patterns of w[0 .. count).  Each workgroup counts chunks of kHistChunk
// elements in LDS (ds_add_u32 on counters packed two per word) and adds the non-zero counters of
// a chunk to the global histogram before the next chunk.
__global__ void __launch_bounds__(kHistThreads, 1)
proxy_hist_kernel(const uint16_t* __restrict__ w, unsigned long long count, uint32_t* __restrict__ hist) {
    __shared__ uint32_t cnt[kProxyBins / 2];
    const int tid = threadIdx.x;
    for (int i = tid; i < kProxyBins / 2; i += kHistThreads) cnt[i] = 0u;
    __syncthreads();
    const unsigned long long nchunks = (count + kHistChunk - 1) / kHistChunk;
    for (unsigned long long c = blockIdx.x; c < nchunks; c += gridDim.x) {
        const unsigned long long base = c * kHistChunk;
        const unsigned long long end = base + kHistChunk < count ? base + kHistChunk : count;
        auto add = [&](uint32_t bits) {
            const uint32_t k = sort_key(bits);
            atomicAdd(&cnt[k >> 1], (k & 1u) ? 0x10000u : 1u);
        };
        if (end - base == kHistChunk) {
            const uint4_t* src = (const uint4_t*)(w + base);
#pragma unroll 5
            for (int i = 0; i < kHistChunk / (8 * kHistThreads); ++i) {
                const uint4_t v = src[i * kHistThreads + tid];
                const uint32_t a = v.x, b = v.y, cc = v.z, d = v.w;
                add(a & 0xFFFFu); add(a >> 16); add(b & 0xFFFFu); add(b >> 16);
                add(cc & 0xFFFFu); add(cc >> 16); add(d & 0xFFFFu); add(d >> 16);
            }
        } else {                                     // the ragged last chunk, element by element
            for (unsigned long long i = base + tid; i < end; i += kHistThreads) add(w[i]);
        }
        __syncthreads();
        for (int i = tid; i < kProxyBins / 2; i += kHistThreads) {
            const uint32_t v = cnt[i];
            if (v) {
                cnt[i] = 0u;
                if (v & 0xFFFFu) atomicAdd(&hist[2 * i], v & 0xFFFFu);
                if (v >> 16) atomicAdd(&hist[2 * i + 1], v >> 16);
            }
        }
        __syncthreads();
    }
}

constexpr int kFinalThreads = 1024;
constexpr int kKeysPerThread = kProxyBins / kFinalThreads;     // 64 consecutive keys per thread
constexpr int kMaxTerms = 8;

// Fixed-order sum over the workgroup (binary64): lanes of a wavefront first, then the wavefronts.
__device__ __forceinline__ double block_sum(double v, double* scratch) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
    __syncthreads();
    if (lane == 0) scratch[wave] = v;
    __syncthreads();
    double s = 0.0;
    for (int i = 0; i < kFinalThreads / 64; ++i) s += scratch[i];
    return s;
}

// out[0] = P_c, out[1] = P_f, *phi = 1 (SQ) iff P_c < tau_c and P_f < tau_f.
__global__ void __launch_bounds__(kFinalThreads, 1)
proxy_final_kernel(const uint32_t* __restrict__ hist, int dtype, unsigned long long count, int terms,
                   double tau_c, double tau_f, double* __restrict__ out, int32_t* __restrict__ phi) {
    __shared__ int last_present[kFinalThreads];      // largest present key of a thread's range, or -1
    __shared__ int first_present[kFinalThreads];
    __shared__ double scratch[kFinalThreads / 64];
    const int tid = threadIdx.x, k0 = tid * kKeysPerThread;

    int first = -1, last = -1, distinct = 0;
    for (int i = 0; i < kKeysPerThread; ++i)
        if (hist[k0 + i]) {
            if (first < 0) first = k0 + i;
            last = k0 + i;
            ++distinct;
        }
    last_present[tid] = last;
    first_present[tid] = first;
    __syncthreads();
    // inclusive running maximum of last_present over the threads (ten doubling steps)
    for (int off = 1; off < kFinalThreads; off <<= 1) {
        const int other = tid >= off ? last_present[tid - off] : -1;
        __syncthreads();
        if (other > last_present[tid]) last_present[tid] = other;
        __syncthreads();
    }
    const int prev_before = tid ? last_present[tid - 1] : -1;   // last present key below k0
    const int kmax = last_present[kFinalThreads - 1];
    // smallest present key: the first thread whose range holds one
    int kmin = -1;
    for (int i = 0; i < kFinalThreads; ++i)
        if (first_present[i] >= 0) { kmin = first_present[i]; break; }
    const double D = block_sum((double)distinct, scratch);

    const double n = (double)(count - 1ull);
    const double span = key_value((uint32_t)kmax, dtype) - key_value((uint32_t)kmin, dtype);
    if (!(span > 0.0)) {                         // constant matrix: no intervals to normalise
        if (tid == 0) { out[0] = 0.0; out[1] = 0.0; *phi = (0.0 < tau_c && 0.0 < tau_f) ? 1 : 0; }
        return;
    }
    const double inv_mean = n / span;            // 1 / (sum(G) / n)

    double sc = 0.0, sk[kMaxTerms + 1];
    for (int k = 0; k <= kMaxTerms; ++k) sk[k] = 0.0;
    int prev = prev_before;
    for (int i = 0; i < kKeysPerThread; ++i) {
        const int key = k0 + i;
        if (!hist[key]) continue;
        if (prev >= 0) {
            const double g = key_value((uint32_t)key, dtype) - key_value((uint32_t)prev, dtype);   // exact
            const double t = g * inv_mean;
            if (t > 0.0) sc += t * log(t);
            const double u = t - 1.0;
            double p = u;
            for (int k = 2; k <= terms; ++k) { p *= u; sk[k] += p; }
        }
        prev = key;
    }
    const double sum_c = block_sum(sc, scratch);
    double sum_k[kMaxTerms + 1];
    for (int k = 2; k <= terms; ++k) sum_k[k] = block_sum(sk[k], scratch);

    if (tid == 0) {
        // the count - D intervals between equal weights have t = 0: t ln t = 0, (t - 1)^k = (-1)^k
        const double zero_gaps = (double)count - D;
        double Pf = 0.0;
        for (int k = 2; k <= terms; ++k) {
            const double s = sum_k[k] + ((k & 1) ? -zero_gaps : zero_gaps);
            Pf += fabs(s) / (n * (double)(k * (k - 1)));
        }
        const double Pc = sum_c / n;
        out[0] = Pc;
        out[1] = Pf;
        *phi = (Pc < tau_c && Pf < tau_f) ? 1 : 0;
    }
}

hipError_t launch_proxy(const void* w, int dtype, unsigned long long count, int terms, double tau_c,
                        double tau_f, uint32_t* hist, double* out, int32_t* phi, hipStream_t s) {
    hipLaunchKernelGGL(proxy_clear_kernel, dim3(kProxyBins / 256), dim3(256), 0, s, hist);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const unsigned long long nchunks = (count + kHistChunk - 1) / kHistChunk;
    const int grid = (int)(nchunks < 256 ? nchunks : 256);     // one workgroup (128 KB of LDS) per CU
    hipLaunchKernelGGL(proxy_hist_kernel, dim3(grid), dim3(kHistThreads), 0, s, (const uint16_t*)w, count, hist);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(proxy_final_kernel, dim3(1), dim3(kFinalThreads), 0, s, hist, dtype, count, terms, tau_c,
                       tau_f, out, phi);
    return hipGetLastError();
}

}  // namespace rwkvq
