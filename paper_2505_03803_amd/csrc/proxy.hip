// The coarse-to-fine proxy of Sec. 3.1 ("Coarse-grained Proxy", "Fine-grained Proxy") for weight
// matrices stored as fp16 or bf16.
//
// The paper sorts the flattened weights and works on the intervals between neighbours.  Sixteen-bit
// weights take at most 65 536 distinct values, and the sums below depend only on WHICH values occur
// (equal weights contribute intervals of length zero, whose number is oc*ic minus the number of
// distinct values).  One pass over the matrix therefore only records the set of occurring bit
// patterns (HBM-bound, the only part that touches the matrix); the rest is a sum over at most
// 65 535 non-zero intervals plus a closed-form term for the zero ones:
//
//   n = oc*ic - 1 intervals, sum(G) = max - min, t_i = G_i / (sum(G) / n) = n G'_i
//   P_c = ln n - H(G')           = (1/n) sum_i t_i ln t_i                 (0 ln 0 := 0)
//   v_k |M_k| = n^k/(k(k-1)) |sum_i delta_i^k| / n = |sum_i (t_i - 1)^k| / (n k (k-1))
//
// Both right-hand sides are the paper's expressions with G' = t/n substituted; they keep every
// quantity of order one where n^k delta^k would leave the range of the arithmetic.  All sums are
// binary64 in a fixed order, so results are reproducible bit for bit.
#include "common.h"
#include "../../include/rwkvq.h"

#include <mutex>

namespace rwkvq {

constexpr int kProxyKeys = 65536;
constexpr int kBitmapWords = kProxyKeys / 32;     // the workspace: one bit per 16-bit pattern
constexpr int kSetThreads = 1024;                 // two workgroups of 64 KB LDS fit a CU
constexpr int kSetMaxWgs = 128;                   // workgroups per matrix
constexpr int kProxyMaxMats = 64;                 // matrices per launch (one table entry per lane)

struct ProxyArgs {
    int wg_end[kProxyMaxMats];                    // running sum of workgroups per matrix
    const uint16_t* w[kProxyMaxMats];
    unsigned long long count[kProxyMaxMats];
    uint32_t* bitmaps;                            // kBitmapWords words per matrix
    double* out;                                  // two doubles per matrix
    int32_t* phi;                                 // one flag per matrix
    int n_mats, dtype, terms, pad;
    double tau_c, tau_f;
};

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

__global__ void __launch_bounds__(256) proxy_clear_kernel(uint32_t* bitmap) {
    bitmap[blockIdx.x * 256 + threadIdx.x] = 0u;
}

// Set of the 16-bit patterns in w[0 .. count): every workgroup marks the keys of its share in a
// byte-per-key table in LDS (plain byte stores: lanes that store the same flag do not need to be
// ordered), packs the table to bits and ORs its non-zero words into the global bitmap.
__global__ void __launch_bounds__(kSetThreads, 2) proxy_set_kernel(ProxyArgs a) {
    __shared__ uint32_t flags[kProxyKeys / 4];
    const int tid = threadIdx.x;
    const int wg = blockIdx.x;
    const int mi = __builtin_popcountll(__builtin_amdgcn_ballot_w64(wg >= a.wg_end[tid & 63]));
    const int wg0 = mi ? a.wg_end[mi - 1] : 0;
    const int local = wg - wg0, nwg = a.wg_end[mi] - wg0;        // this matrix's workgroups
    const uint16_t* __restrict__ w = a.w[mi];
    const unsigned long long count = a.count[mi];
    uint32_t* __restrict__ bitmap = a.bitmaps + (size_t)mi * kBitmapWords;
    for (int i = tid; i < kProxyKeys / 4; i += kSetThreads) flags[i] = 0u;
    __syncthreads();
    volatile uint8_t* flag = (volatile uint8_t*)flags;
    const unsigned long long nvec = count / 8;                 // whole 16-byte groups of 8 weights
    const uint4_t* src = (const uint4_t*)w;
    for (unsigned long long i = (unsigned long long)local * kSetThreads + tid; i < nvec;
         i += (unsigned long long)nwg * kSetThreads) {
        const uint4_t v = __builtin_nontemporal_load(src + i);      // read once
        const uint32_t a = v.x, b = v.y, c = v.z, d = v.w;
        flag[sort_key(a & 0xFFFFu)] = 1; flag[sort_key(a >> 16)] = 1;
        flag[sort_key(b & 0xFFFFu)] = 1; flag[sort_key(b >> 16)] = 1;
        flag[sort_key(c & 0xFFFFu)] = 1; flag[sort_key(c >> 16)] = 1;
        flag[sort_key(d & 0xFFFFu)] = 1; flag[sort_key(d >> 16)] = 1;
    }
    if (local == 0 && (unsigned long long)tid < count - 8 * nvec)        // the ragged tail
        flag[sort_key(w[8 * nvec + tid])] = 1;
    __syncthreads();
    // 32 flags -> one bitmap word; the walk starts at a different word in every workgroup so that
    // the workgroups do not all hit the same global words at the same time
    for (int j = tid; j < kBitmapWords; j += kSetThreads) {
        const int i = (j + 37 * local) & (kBitmapWords - 1);
        uint32_t m = 0;
#pragma unroll
        for (int q = 0; q < 8; ++q)      // four flag bytes (0 or 1) -> four bits: one multiply
            m |= ((((flags[8 * i + q] & 0x01010101u) * 0x01020408u) >> 24) & 0xFu) << (4 * q);
        if (m) atomicOr(&bitmap[i], m);
    }
}

constexpr int kFinalThreads = 1024;               // one thread per 64 consecutive keys
constexpr int kMaxTerms = 8;
static_assert(kFinalThreads * 64 == kProxyKeys, "one 64-bit presence word per thread");

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

// One workgroup per matrix: out[0] = P_c, out[1] = P_f, *phi = 1 (SQ) iff P_c < tau_c and
// P_f < tau_f.  Thread t first owns presence word t (keys 64 t .. 64 t + 63); running sums over the words give
// the rank of every present key, and each thread then walks an equal share of the ranks (the
// present keys of near-Gaussian weights crowd into a few words: a thread per word would leave
// most threads idle while a few evaluate 64 logarithms each).
__global__ void __launch_bounds__(kFinalThreads, 1) proxy_final_kernel(ProxyArgs a) {
    const int mat = blockIdx.x;                      // one workgroup per matrix
    const uint32_t* __restrict__ bitmap = a.bitmaps + (size_t)mat * kBitmapWords;
    const unsigned long long count = a.count[mat];
    const int dtype = a.dtype, terms = a.terms;
    const double tau_c = a.tau_c, tau_f = a.tau_f;
    double* __restrict__ out = a.out + 2 * mat;
    int32_t* __restrict__ phi = a.phi + mat;
    __shared__ unsigned long long present[kFinalThreads];
    __shared__ int before[kFinalThreads + 1];        // number of present keys below word t
    __shared__ int last_present[kFinalThreads];      // largest present key up to and including word t
    __shared__ double scratch[kFinalThreads / 64];
    const int tid = threadIdx.x;

    const unsigned long long mine = ((const unsigned long long*)bitmap)[tid];
    present[tid] = mine;
    before[tid + 1] = __builtin_popcountll(mine);
    last_present[tid] = mine ? 64 * tid + 63 - __builtin_clzll(mine) : -1;
    if (tid == 0) before[0] = 0;
    __syncthreads();
    for (int off = 1; off < kFinalThreads; off <<= 1) {          // inclusive running sum / maximum
        const int add = tid >= off ? before[tid + 1 - off] : 0;
        const int other = tid >= off ? last_present[tid - off] : -1;
        __syncthreads();
        before[tid + 1] += add;
        if (other > last_present[tid]) last_present[tid] = other;
        __syncthreads();
    }
    const int D = before[kFinalThreads];                         // distinct values (>= 1)
    const int kmax = last_present[kFinalThreads - 1];
    int lo = 0, hi = kFinalThreads - 1;                          // first non-empty word
    while (lo < hi) { const int mid = (lo + hi) >> 1; if (before[mid + 1] > 0) hi = mid; else lo = mid + 1; }
    const int kmin = 64 * lo + __builtin_ctzll(present[lo]);

    const double n = (double)(count - 1ull);
    const double span = key_value((uint32_t)kmax, dtype) - key_value((uint32_t)kmin, dtype);
    if (!(span > 0.0)) {                         // constant matrix: no intervals to normalise
        if (tid == 0) { out[0] = 0.0; out[1] = 0.0; *phi = (0.0 < tau_c && 0.0 < tau_f) ? 1 : 0; }
        return;
    }
    const double inv_mean = n / span;            // 1 / (sum(G) / n)

    // ranks r0 .. r1-1 of the present keys are this thread's
    const int r0 = (int)((long long)tid * D / kFinalThreads), r1 = (int)((long long)(tid + 1) * D / kFinalThreads);
    double sc = 0.0, sk[kMaxTerms + 1];
    for (int k = 0; k <= kMaxTerms; ++k) sk[k] = 0.0;
    if (r1 > r0) {
        lo = 0; hi = kFinalThreads - 1;                          // the word that holds rank r0
        while (lo < hi) { const int mid = (lo + hi) >> 1; if (before[mid + 1] > r0) hi = mid; else lo = mid + 1; }
        int wd = lo;
        unsigned long long m = present[wd];
        for (int skip = r0 - before[wd]; skip > 0; --skip) m &= m - 1;   // drop the keys ranked below r0
        const unsigned long long dropped = present[wd] ^ m;
        int prev = dropped ? 64 * wd + 63 - __builtin_clzll(dropped) : (wd ? last_present[wd - 1] : -1);
        for (int r = r0; r < r1; ++r) {
            while (!m) m = present[++wd];
            const int key = 64 * wd + __builtin_ctzll(m);
            m &= m - 1;
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
    }
    const double sum_c = block_sum(sc, scratch);
    double sum_k[kMaxTerms + 1];
    for (int k = 2; k <= terms; ++k) sum_k[k] = block_sum(sk[k], scratch);

    if (tid == 0) {
        // the count - D intervals between equal weights have t = 0: t ln t = 0, (t - 1)^k = (-1)^k
        const double zero_gaps = (double)count - (double)D;
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

hipError_t launch_proxy(const void* const* ws, const int* Ns, const int* Ks, int n_mats, int dtype, int terms,
                        double tau_c, double tau_f, uint32_t* bitmaps, double* out, int32_t* phi, hipStream_t s) {
    for (int base = 0; base < n_mats; base += kProxyMaxMats) {
        ProxyArgs a;
        const int cnt = n_mats - base < kProxyMaxMats ? n_mats - base : kProxyMaxMats;
        int wgs = 0;
        for (int i = 0; i < cnt; ++i) {
            const unsigned long long count = (unsigned long long)Ns[base + i] * (unsigned long long)Ks[base + i];
            const unsigned long long nvec = count / 8;
            unsigned long long g = (nvec + 16ull * kSetThreads - 1) / (16ull * kSetThreads);   // >= 128 weights per thread
            g = g < 1 ? 1 : g > (unsigned long long)kSetMaxWgs ? kSetMaxWgs : g;
            wgs += (int)g;
            a.wg_end[i] = wgs;
            a.w[i] = (const uint16_t*)ws[base + i];
            a.count[i] = count;
        }
        for (int i = cnt; i < kProxyMaxMats; ++i) { a.wg_end[i] = 0x7FFFFFFF; a.w[i] = nullptr; a.count[i] = 0; }
        a.bitmaps = bitmaps + (size_t)base * kBitmapWords;
        a.out = out + 2 * base;
        a.phi = phi + base;
        a.n_mats = cnt; a.dtype = dtype; a.terms = terms; a.pad = 0;
        a.tau_c = tau_c; a.tau_f = tau_f;
        hipLaunchKernelGGL(proxy_clear_kernel, dim3(cnt * kBitmapWords / 256), dim3(256), 0, s, a.bitmaps);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(proxy_set_kernel, dim3(wgs), dim3(kSetThreads), 0, s, a);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(proxy_final_kernel, dim3(cnt), dim3(kFinalThreads), 0, s, a);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

int check_proxy_args(const void* const* ws, const int* Ns, const int* Ks, int n_mats, int w_dtype, int terms,
                     const double* proxies, const int32_t* phi, bool allow_f32) {
    if (!ws || !Ns || !Ks || !proxies || !phi) return RWKVQ_ERR_NULL;
    if (n_mats < 1) return RWKVQ_ERR_SHAPE;
    if (w_dtype != RWKVQ_F16 && w_dtype != RWKVQ_BF16 && !(allow_f32 && w_dtype == RWKVQ_F32)) return RWKVQ_ERR_UNSUPPORTED;
    if (terms < 2 || terms > kMaxTerms) return RWKVQ_ERR_UNSUPPORTED;
    if (((uintptr_t)proxies & 15u) || ((uintptr_t)phi & 3u)) return RWKVQ_ERR_ALIGN;
    for (int i = 0; i < n_mats; ++i) {
        if (!ws[i]) return RWKVQ_ERR_NULL;
        if ((uintptr_t)ws[i] & 15u) return RWKVQ_ERR_ALIGN;
        if (Ns[i] < 1 || Ks[i] < 1) return RWKVQ_ERR_SHAPE;
        const unsigned long long count = (unsigned long long)Ns[i] * (unsigned long long)Ks[i];
        if (count < 2ull || count > 0xFFFFFFFFull) return RWKVQ_ERR_SHAPE;
    }
    return RWKVQ_OK;
}

// ---- the same call for callers that cannot allocate -------------------------------------------
// The bitmaps live in a file-scope device array instead of a caller's workspace.  The array's name
// is a host-side stand-in in host code: its device address is looked up once per device
// (hipGetSymbolAddress with that device current) and only that address is handed to the kernels.
constexpr int kStaticMaxMats = RWKVQ_PROXY_STATIC_MAX_MATS;
static __device__ __align__(256) uint32_t scratch[(size_t)kStaticMaxMats * kBitmapWords];   // 2 MiB per device

constexpr int kMaxDevices = 64;
static std::mutex scratch_mutex;
static uint32_t* scratch_addr[kMaxDevices];       // device address of `scratch` on device i, once known

static hipError_t scratch_of_current_device(uint32_t** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (!scratch_addr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        scratch_addr[dev] = (uint32_t*)p;
    }
    *out = scratch_addr[dev];
    return hipSuccess;
}

}  // namespace rwkvq

extern "C" int rwkvq_proxy_static(const void* const* ws, const int* Ns, const int* Ks, int n_mats, int w_dtype,
                                  int terms, double tau_c, double tau_f, double* proxies, int32_t* phi, void* stream) {
    using namespace rwkvq;
    const int st = check_proxy_args(ws, Ns, Ks, n_mats, w_dtype, terms, proxies, phi, false);
    if (st != RWKVQ_OK) return st;
    if (n_mats > kStaticMaxMats) return RWKVQ_ERR_SHAPE;
    uint32_t* bitmaps = nullptr;
    if (scratch_of_current_device(&bitmaps) != hipSuccess) return RWKVQ_ERR_DEVICE;
    hipError_t e = launch_proxy(ws, Ns, Ks, n_mats, w_dtype == RWKVQ_F16 ? DT_F16 : DT_BF16, terms, tau_c, tau_f, bitmaps,
                                proxies, phi, (hipStream_t)stream);
    return e == hipSuccess ? RWKVQ_OK : RWKVQ_ERR_DEVICE;
}
