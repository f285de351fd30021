// The coarse-to-fine proxy of Sec. 3.1 for weight matrices stored as binary32: the recipe as the
// paper states it.  The flattened weights are sorted in ascending order ("Coarse-grained Proxy"),
// the intervals between neighbours are normalised (Eqs. "interval", "interval_norm"), and the
// entropy and the central moments of the normalised intervals give P_c and P_f (Eqs. "ie",
// "coarse_proxy", "fine_proxy").  Sixteen-bit matrices take the shortcut of proxy.hip (the set of
// occurring bit patterns); binary32 weights have no such shortcut, so they are really sorted:
//
//   * keys: the order-preserving map of the binary32 patterns to unsigned integers;
//   * least-significant-digit radix sort, four passes of 8 bits, each pass three steps:
//       sort_hist_kernel     per tile of 4096 keys, how many keys have each digit value;
//       sort_scan_kernel     running sums of those counts, digit-major (the position of every
//                            (digit, tile) run in the output);
//       sort_scatter_kernel  every key to its position: its rank among the keys of its digit within
//                            the tile comes from wavefront ballots (no atomics, the order of equal
//                            digits is kept, which a least-significant-digit sort needs), the tile is
//                            reordered in LDS so that runs leave as contiguous stores;
//   * gap_sum_kernel / gap_final_kernel: the sums over the intervals in binary64, in a fixed order
//     (a partial sum per 16384 intervals, then one workgroup adds the partial sums), with
//     t_i = G_i / mean(G) as in proxy.hip:  P_c = (1/n) sum t ln t,  v_k |M_k| = |sum (t-1)^k| / (n k (k-1)).
//
// Matrices of a call are processed one after another on the stream and share the sort buffers.
#include "common.h"
#include "../../include/rwkvq.h"

namespace rwkvq {

constexpr int kSortThreads = 256;
constexpr int kSortRounds = 16;                              // keys per thread
constexpr int kSortTile = kSortThreads * kSortRounds;        // 4096 keys per workgroup
constexpr int kDigits = 256;
constexpr int kGapThreads = 256;
constexpr int kGapPerThread = 64;
constexpr int kGapTile = kGapThreads * kGapPerThread;        // 16384 intervals per workgroup
constexpr int kGapMaxTerms = 8;
constexpr int kGapSums = kGapMaxTerms + 1;                   // [0] = sum t ln t, [k] = sum (t-1)^k

__device__ __forceinline__ uint32_t f32_key(uint32_t bits) {      // a < b as numbers  =>  key(a) < key(b); -0 sorts below +0
    return (bits & 0x80000000u) ? ~bits : (bits | 0x80000000u);
}
__device__ __forceinline__ double key_f64(uint32_t key) {
    const uint32_t bits = (key & 0x80000000u) ? (key & 0x7FFFFFFFu) : ~key;
    return (double)__builtin_bit_cast(float, bits);
}

// Lanes of the wavefront whose 8-bit digit equals this lane's (among the lanes with valid = true).
__device__ __forceinline__ unsigned long long same_digit_lanes(uint32_t digit, bool valid) {
    unsigned long long m = __builtin_amdgcn_ballot_w64(valid);
#pragma unroll
    for (int b = 0; b < 8; ++b) {
        const bool bit = (digit >> b) & 1u;
        const unsigned long long set = __builtin_amdgcn_ballot_w64(bit);
        m &= bit ? set : ~set;
    }
    return m;
}
__device__ __forceinline__ unsigned long long lanes_below(int lane) { return (1ull << lane) - 1ull; }

// LDS traffic of one wavefront is served in issue order; the fences keep the compiler from moving
// a lane's read of a counter past the leader's update of it.
__device__ __forceinline__ void wave_order() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// counts[digit * n_tiles + tile] = number of keys of the tile whose digit (bits shift .. shift+7) has that value.
// FIRST: the input holds binary32 patterns, not keys yet.
template <bool FIRST>
__global__ void __launch_bounds__(kSortThreads) sort_hist_kernel(const uint32_t* __restrict__ in, uint32_t n, int shift,
                                                                 uint32_t* __restrict__ counts, uint32_t n_tiles) {
    __shared__ uint32_t h[kDigits];
    const int tid = threadIdx.x, lane = tid & 63;
    h[tid] = 0u;
    __syncthreads();
    const size_t base = (size_t)blockIdx.x * kSortTile;
#pragma unroll 4
    for (int r = 0; r < kSortRounds; ++r) {
        const size_t i = base + (size_t)r * kSortThreads + tid;
        const bool valid = i < n;
        uint32_t k = valid ? in[i] : 0u;
        if (FIRST) k = f32_key(k);
        const uint32_t d = (k >> shift) & 255u;
        // Counting needs no order: one LDS addition per key, except that a wavefront whose valid lanes all hold
        // the same digit (the low bytes of binary32 patterns that came from 16-bit values, a run of equal
        // weights) adds once - 64 additions to one address would be served one after the other.
        const unsigned long long live = __builtin_amdgcn_ballot_w64(valid);
        const uint32_t d0 = (uint32_t)__builtin_amdgcn_readfirstlane((int)d);      // digit of the first valid lane
        const unsigned long long same = __builtin_amdgcn_ballot_w64(valid && d == d0);
        if (same == live) {
            if (valid && (live & lanes_below(lane)) == 0ull) atomicAdd(&h[d], (uint32_t)__builtin_popcountll(live));
        } else if (valid) {
            atomicAdd(&h[d], 1u);
        }
    }
    __syncthreads();
    counts[(size_t)tid * n_tiles + blockIdx.x] = h[tid];
}

// In place: counts[d][t] <- number of keys with digit d in tiles before t; totals[d] <- keys with digit d.
__global__ void __launch_bounds__(256) sort_scan_rows_kernel(uint32_t* __restrict__ counts, uint32_t n_tiles,
                                                             uint32_t* __restrict__ totals) {
    __shared__ uint32_t part[256];
    uint32_t* row = counts + (size_t)blockIdx.x * n_tiles;
    const int tid = threadIdx.x;
    const uint32_t per = (n_tiles + 255u) / 256u;
    const uint32_t lo = min(n_tiles, tid * per), hi = min(n_tiles, lo + per);
    uint32_t s = 0;
    for (uint32_t i = lo; i < hi; ++i) s += row[i];
    part[tid] = s;
    __syncthreads();
    for (int off = 1; off < 256; off <<= 1) {                  // inclusive running sum of the 256 segment sums
        const uint32_t add = tid >= off ? part[tid - off] : 0u;
        __syncthreads();
        part[tid] += add;
        __syncthreads();
    }
    uint32_t run = tid ? part[tid - 1] : 0u;
    for (uint32_t i = lo; i < hi; ++i) { const uint32_t c = row[i]; row[i] = run; run += c; }
    if (tid == 255) totals[blockIdx.x] = part[255];
}

// totals[d] <- number of keys with a smaller digit.
__global__ void __launch_bounds__(256) sort_scan_totals_kernel(uint32_t* __restrict__ totals) {
    __shared__ uint32_t part[256];
    const int tid = threadIdx.x;
    const uint32_t mine = totals[tid];
    part[tid] = mine;
    __syncthreads();
    for (int off = 1; off < 256; off <<= 1) {
        const uint32_t add = tid >= off ? part[tid - off] : 0u;
        __syncthreads();
        part[tid] += add;
        __syncthreads();
    }
    totals[tid] = part[tid] - mine;
}

// Every key of the tile to out[position of its (digit, tile) run + its rank in the run].  Order inside a tile:
// wavefront w owns keys 1024 w .. 1024 w + 1023, in rounds of 64.
template <bool FIRST>
__global__ void __launch_bounds__(kSortThreads) sort_scatter_kernel(const uint32_t* __restrict__ in, uint32_t* __restrict__ out,
                                                                    uint32_t n, int shift, const uint32_t* __restrict__ before,
                                                                    const uint32_t* __restrict__ smaller, uint32_t n_tiles) {
    __shared__ uint32_t seen[4][kDigits];     // per wavefront: keys of each digit so far; later: keys of the digit in earlier wavefronts
    __shared__ uint32_t start[kDigits];       // first slot of each digit in the tile's sorted order
    __shared__ uint32_t run_pos[kDigits];     // position in `out` of the tile's first key of each digit
    __shared__ uint32_t sorted[kSortTile];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
#pragma unroll
    for (int w = 0; w < 4; ++w) seen[w][tid] = 0u;
    run_pos[tid] = smaller[tid] + before[(size_t)tid * n_tiles + blockIdx.x];
    __syncthreads();
    const size_t base = (size_t)blockIdx.x * kSortTile + (size_t)wave * (kSortTile / 4);
    uint32_t key[kSortRounds], rank[kSortRounds];
#pragma unroll
    for (int r = 0; r < kSortRounds; ++r) {
        const size_t i = base + (size_t)r * 64 + lane;
        const bool valid = i < n;
        uint32_t k = valid ? in[i] : 0xFFFFFFFFu;
        if (FIRST && valid) k = f32_key(k);
        const uint32_t d = (k >> shift) & 255u;
        const unsigned long long m = same_digit_lanes(d, valid);
        const uint32_t below = (uint32_t)__builtin_popcountll(m & lanes_below(lane));
        const uint32_t old = seen[wave][d];
        wave_order();
        if (valid && below == 0u) seen[wave][d] = old + (uint32_t)__builtin_popcountll(m);
        wave_order();
        key[r] = k;
        rank[r] = old + below;                 // rank among the wavefront's keys of this digit
    }
    __syncthreads();
    {   // digit t: keys per wavefront -> keys in earlier wavefronts; tile totals -> first slots
        const uint32_t c0 = seen[0][tid], c1 = seen[1][tid], c2 = seen[2][tid], c3 = seen[3][tid];
        seen[0][tid] = 0u; seen[1][tid] = c0; seen[2][tid] = c0 + c1; seen[3][tid] = c0 + c1 + c2;
        const uint32_t total = c0 + c1 + c2 + c3;
        start[tid] = total;
        __syncthreads();
        for (int off = 1; off < 256; off <<= 1) {
            const uint32_t add = tid >= off ? start[tid - off] : 0u;
            __syncthreads();
            start[tid] += add;
            __syncthreads();
        }
        const uint32_t incl = start[tid];
        __syncthreads();
        start[tid] = incl - total;
        __syncthreads();
    }
    const size_t tile_base = (size_t)blockIdx.x * kSortTile;
    const uint32_t in_tile = (uint32_t)(n - tile_base < (size_t)kSortTile ? n - tile_base : (size_t)kSortTile);
#pragma unroll
    for (int r = 0; r < kSortRounds; ++r) {
        const size_t i = base + (size_t)r * 64 + lane;
        if (i < n) {
            const uint32_t d = (key[r] >> shift) & 255u;
            sorted[start[d] + seen[wave][d] + rank[r]] = key[r];
        }
    }
    __syncthreads();
    for (uint32_t s = tid; s < in_tile; s += kSortThreads) {
        const uint32_t k = sorted[s];
        const uint32_t d = (k >> shift) & 255u;
        out[(size_t)run_pos[d] + (s - start[d])] = k;
    }
}

// Partial sums over the intervals of one tile: partial[tile][0] = sum t ln t, [k] = sum (t - 1)^k, k = 2 .. terms.
__global__ void __launch_bounds__(kGapThreads) gap_sum_kernel(const uint32_t* __restrict__ keys, uint32_t count, int terms,
                                                              double* __restrict__ partial) {
    __shared__ double red[kGapThreads / 64][kGapSums];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t n = count - 1u;                                   // intervals
    const double span = key_f64(keys[count - 1]) - key_f64(keys[0]);
    double s[kGapSums];
#pragma unroll
    for (int k = 0; k < kGapSums; ++k) s[k] = 0.0;
    if (span > 0.0) {
        const double inv_mean = (double)n / span;
        const size_t base = (size_t)blockIdx.x * kGapTile;
        for (int j = 0; j < kGapPerThread; ++j) {
            const size_t i = base + (size_t)j * kGapThreads + tid;
            if (i < n) {
                const double g = key_f64(keys[i + 1]) - key_f64(keys[i]);    // exact: both are binary32 values
                const double t = g * inv_mean;
                if (t > 0.0) s[0] += t * log(t);
                const double u = t - 1.0;
                double p = u;
                for (int k = 2; k <= terms; ++k) { p *= u; s[k] += p; }
            }
        }
    }
#pragma unroll
    for (int k = 0; k < kGapSums; ++k) {
        double v = s[k];
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
        if (lane == 0) red[wave][k] = v;
    }
    __syncthreads();
    if (tid < kGapSums) {
        double v = 0.0;
        for (int w = 0; w < kGapThreads / 64; ++w) v += red[w][tid];
        partial[(size_t)blockIdx.x * kGapSums + tid] = v;
    }
}

// One workgroup: the partial sums in tile order, then P_c, P_f and the decision of Eq. "multi_scale_proxy".
__global__ void __launch_bounds__(256) gap_final_kernel(const uint32_t* __restrict__ keys, uint32_t count, int terms,
                                                        const double* __restrict__ partial, uint32_t n_tiles, double tau_c,
                                                        double tau_f, double* __restrict__ out, int32_t* __restrict__ phi) {
    __shared__ double red[256][kGapSums];
    const int tid = threadIdx.x;
    double s[kGapSums];
#pragma unroll
    for (int k = 0; k < kGapSums; ++k) s[k] = 0.0;
    const uint32_t per = (n_tiles + 255u) / 256u;
    const uint32_t lo = min(n_tiles, tid * per), hi = min(n_tiles, lo + per);
    for (uint32_t t = lo; t < hi; ++t)
#pragma unroll
        for (int k = 0; k < kGapSums; ++k) s[k] += partial[(size_t)t * kGapSums + k];
#pragma unroll
    for (int k = 0; k < kGapSums; ++k) red[tid][k] = s[k];
    __syncthreads();
    if (tid == 0) {
        double tot[kGapSums];
        for (int k = 0; k < kGapSums; ++k) { tot[k] = 0.0; for (int i = 0; i < 256; ++i) tot[k] += red[i][k]; }
        const double n = (double)(count - 1u);
        const double span = key_f64(keys[count - 1]) - key_f64(keys[0]);
        double Pc = 0.0, Pf = 0.0;
        if (span > 0.0) {                        // a constant matrix has no intervals to normalise: both proxies 0
            Pc = tot[0] / n;
            for (int k = 2; k <= terms; ++k) Pf += fabs(tot[k]) / (n * (double)(k * (k - 1)));
        }
        out[0] = Pc;
        out[1] = Pf;
        *phi = (Pc < tau_c && Pf < tau_f) ? 1 : 0;
    }
}

static size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

struct F32Layout { size_t keys_a, keys_b, counts, totals, partial, bytes; };
static F32Layout f32_layout(unsigned long long max_count) {
    const size_t tiles = (size_t)((max_count + kSortTile - 1) / kSortTile);
    const size_t gap_tiles = (size_t)((max_count + kGapTile - 1) / kGapTile);
    F32Layout L;
    size_t o = 0;
    L.keys_a = o; o += align256((size_t)max_count * 4);
    L.keys_b = o; o += align256((size_t)max_count * 4);
    L.counts = o; o += align256(tiles * kDigits * 4);
    L.totals = o; o += align256(kDigits * 4);
    L.partial = o; o += align256(gap_tiles * kGapSums * 8);
    L.bytes = o;
    return L;
}

size_t proxy_f32_workspace_bytes(const int* Ns, const int* Ks, int n_mats) {
    unsigned long long mx = 0;
    for (int i = 0; i < n_mats; ++i) {
        const unsigned long long c = (unsigned long long)Ns[i] * (unsigned long long)Ks[i];
        mx = c > mx ? c : mx;
    }
    return f32_layout(mx).bytes;
}

hipError_t launch_proxy_f32(const void* const* ws, const int* Ns, const int* Ks, int n_mats, int terms, double tau_c,
                            double tau_f, void* workspace, double* out, int32_t* phi, hipStream_t s) {
    unsigned long long mx = 0;
    for (int i = 0; i < n_mats; ++i) {
        const unsigned long long c = (unsigned long long)Ns[i] * (unsigned long long)Ks[i];
        mx = c > mx ? c : mx;
    }
    const F32Layout L = f32_layout(mx);
    char* base = (char*)workspace;
    uint32_t* buf[2] = {(uint32_t*)(base + L.keys_a), (uint32_t*)(base + L.keys_b)};
    uint32_t* counts = (uint32_t*)(base + L.counts);
    uint32_t* totals = (uint32_t*)(base + L.totals);
    double* partial = (double*)(base + L.partial);
    for (int i = 0; i < n_mats; ++i) {
        const uint32_t count = (uint32_t)((unsigned long long)Ns[i] * (unsigned long long)Ks[i]);
        const uint32_t tiles = (uint32_t)(((unsigned long long)count + kSortTile - 1) / kSortTile);   // count may be 2^32 - 1
        const uint32_t* src = (const uint32_t*)ws[i];
        for (int pass = 0; pass < 4; ++pass) {
            uint32_t* dst = buf[pass & 1];
            if (pass == 0) hipLaunchKernelGGL(sort_hist_kernel<true>, dim3(tiles), dim3(kSortThreads), 0, s, src, count, 0, counts, tiles);
            else hipLaunchKernelGGL(sort_hist_kernel<false>, dim3(tiles), dim3(kSortThreads), 0, s, src, count, 8 * pass, counts, tiles);
            hipLaunchKernelGGL(sort_scan_rows_kernel, dim3(kDigits), dim3(256), 0, s, counts, tiles, totals);
            hipLaunchKernelGGL(sort_scan_totals_kernel, dim3(1), dim3(256), 0, s, totals);
            if (pass == 0) hipLaunchKernelGGL(sort_scatter_kernel<true>, dim3(tiles), dim3(kSortThreads), 0, s, src, dst, count, 0, counts, totals, tiles);
            else hipLaunchKernelGGL(sort_scatter_kernel<false>, dim3(tiles), dim3(kSortThreads), 0, s, src, dst, count, 8 * pass, counts, totals, tiles);
            hipError_t e = hipGetLastError();
            if (e != hipSuccess) return e;
            src = dst;
        }
        const uint32_t gap_tiles = (uint32_t)(((unsigned long long)count - 1 + kGapTile - 1) / kGapTile);
        hipLaunchKernelGGL(gap_sum_kernel, dim3(gap_tiles), dim3(kGapThreads), 0, s, src, count, terms, partial);
        hipLaunchKernelGGL(gap_final_kernel, dim3(1), dim3(256), 0, s, src, count, terms, partial, gap_tiles, tau_c, tau_f,
                           out + 2 * i, phi + i);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace rwkvq
