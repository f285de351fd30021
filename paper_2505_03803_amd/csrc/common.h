// Shared device helpers of librwkvq: number formats, the canonical bit-string reader and the
// index arithmetic of the native tile layout (see include/rwkvq.h for both layouts).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace rwkvq {

enum Fmt : int { FMT_SQ3 = 0, FMT_VQ6 = 1, FMT_VQ8 = 2 };
enum DT : int { DT_F16 = 0, DT_BF16 = 1, DT_F32 = 2 };

constexpr int kGroup = 128;       // SQ group length along K
constexpr int kTileRows = 16;     // native tile: 16 rows
constexpr int kTileCols = 256;    //              x 256 columns
constexpr int kBlock = 256;       // VQ codebook block edge

// One matrix as the kernels see it (device pointers, already validated).
struct MatDev {
    const uint32_t* codes;   // SQ codes / VQ indices
    const uint16_t* aux;     // SQ canonical: scales; SQ native: scale/zero buffer; VQ: codebooks
    const uint16_t* aux2;    // SQ canonical: zeros; otherwise unused
    const void* x;
    void* y;
    int N, K;
    int fmt;                 // Fmt
    int layout;              // 0 canonical, 1 native
};

typedef _Float16 half_t;
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef float float16_t __attribute__((ext_vector_type(16)));
typedef uint32_t uint4_t __attribute__((ext_vector_type(4)));
typedef uint32_t uint2_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float f16_bits_to_f32(uint16_t h) {
    return (float)__builtin_bit_cast(half_t, h);            // exact widening
}
__device__ __forceinline__ float bf16_bits_to_f32(uint16_t b) {
    return __builtin_bit_cast(float, (uint32_t)b << 16);
}
__device__ __forceinline__ uint16_t f32_to_f16_bits(float f) {
    return __builtin_bit_cast(uint16_t, (half_t)f);          // v_cvt_f16_f32, nearest even
}
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f) {  // finite inputs, nearest even
    uint32_t u = __builtin_bit_cast(uint32_t, f);
    return (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
}
__device__ __forceinline__ float load_as_f32(const void* p, size_t i, int dt) {
    if (dt == DT_F16) return f16_bits_to_f32(((const uint16_t*)p)[i]);
    if (dt == DT_BF16) return bf16_bits_to_f32(((const uint16_t*)p)[i]);
    return ((const float*)p)[i];
}
__device__ __forceinline__ void store_from_f32(void* p, size_t i, int dt, float v) {
    if (dt == DT_F16) ((uint16_t*)p)[i] = f32_to_f16_bits(v);
    else if (dt == DT_BF16) ((uint16_t*)p)[i] = f32_to_bf16_bits(v);
    else ((float*)p)[i] = v;
}

// The logistic function of the block's gates (App. A.1), binary32.
__device__ __forceinline__ float sigmoid_f32(float r) { return 1.0f / (1.0f + expf(-r)); }
// sigma(r) * y as a binary32 product of its own.  The empty asm keeps the compiler from merging the
// multiplication with the conversion to a 16-bit type that follows it (one mixed-precision
// instruction, one rounding instead of two): every kernel that applies a gate must store the same bits.
__device__ __forceinline__ float gate_f32(float r, float y) {
    float p = sigmoid_f32(r) * y;
    asm volatile("" : "+v"(p));
    return p;
}

// One token of Eq. "time mixing wkv" carried as a state (a, b, p) per channel: the sums over earlier
// tokens equal a exp(p) and b exp(p), p the largest exponent so far, so every exp() argument is <= 0.
// wkv_out: the output for the current (k, v) with the bonus u; wkv_advance: the sums decayed by
// exp(-w) and the current token added without the bonus.  Shared by every kernel that steps the
// recurrence, so that they store the same bits.
__device__ __forceinline__ float wkv_out(float a, float b, float p, float uc, float kk, float vv) {
    const float ww = uc + kk;
    const float q = fmaxf(p, ww);
    const float e1 = expf(p - q), e2 = expf(ww - q);
    return (e1 * a + e2 * vv) / (e1 * b + e2);
}
__device__ __forceinline__ void wkv_advance(float& a, float& b, float& p, float wc, float kk, float vv) {
    const float pw = p - wc;
    const float q2 = fmaxf(pw, kk);
    const float f1 = expf(pw - q2), f2 = expf(kk - q2);
    a = f1 * a + f2 * vv;
    b = f1 * b + f2;
    p = q2;
}

// The SQ inverse of Sec. 2.2 Eq. "SQ": subtract, round, multiply, round.  The intrinsics keep
// the compiler from fusing the two steps.
__device__ __forceinline__ float sq_deq(uint32_t q, float s, float z) {
    return __fmul_rn(__fsub_rn((float)q, z), s);
}

// Field `index` of width `width` of a little-endian bit string (canonical layout).
__device__ __forceinline__ uint32_t canon_field(const uint32_t* row, int width, int index) {
    int p = width * index;
    int w = p >> 5, off = p & 31;
    uint64_t two = row[w];
    if (off + width > 32) two |= (uint64_t)row[w + 1] << 32;
    return (uint32_t)(two >> off) & ((1u << width) - 1u);
}

// ---- native layout index arithmetic ------------------------------------------------------
// Column k of a tile-local position: kk = k & 255 -> unit u, step t, lane group kg, slot j.
struct TilePos { int u, lane, c; };   // c = 8*t + j : field number within the lane's unit
__host__ __device__ __forceinline__ TilePos tile_pos(int r, int kk) {
    TilePos p;
    p.u = kk >> 7;
    int t = (kk >> 5) & 3, kg = (kk >> 3) & 3, j = kk & 7;
    p.lane = kg * 16 + r;
    p.c = 8 * t + j;
    return p;
}
// Inverse: lane, unit, field -> tile-local column.
__host__ __device__ __forceinline__ int tile_col(int lane, int u, int c) {
    return 128 * u + 32 * (c >> 3) + 8 * (lane >> 4) + (c & 7);
}
// Word index (within a 384-word SQ / 6-bit VQ tile) of lane word i = 0..5.
__host__ __device__ __forceinline__ int tile6_word(int lane, int i) {
    return i < 4 ? 4 * lane + i : 256 + 2 * lane + (i - 4);
}
// Word index (within a 512-word 8-bit VQ tile) of lane word i = 0..7.
__host__ __device__ __forceinline__ int tile8_word(int lane, int i) {
    return i < 4 ? 4 * lane + i : 256 + 4 * lane + (i - 4);
}
__host__ __device__ __forceinline__ int tile_words(int fmt) { return fmt == FMT_VQ8 ? 512 : 384; }

// Native SQ field c of a unit whose three words are w[0..2].
__device__ __forceinline__ uint32_t native_sq_field(const uint32_t* w, int c) {
    int P = c >> 1, e = c & 1;
    if (P < 15) return (w[P / 5] >> (1 + 3 * (P % 5) + 16 * e)) & 7u;
    int b = 16 * e;
    return ((w[0] >> b) & 1u) | (((w[1] >> b) & 1u) << 1) | (((w[2] >> b) & 1u) << 2);
}
// Native 6-bit VQ index P of a unit whose three words are w[0..2].
__device__ __forceinline__ uint32_t native_vq6_index(const uint32_t* w, int P) {
    if (P < 15) return (w[P / 5] >> (2 + 6 * (P % 5))) & 63u;
    return (w[0] & 3u) | ((w[1] & 3u) << 2) | ((w[2] & 3u) << 4);
}
// Native SQ scale/zero buffer: index (in fp16 units) of the scale of (row n, group g); zero at +1.
__host__ __device__ __forceinline__ size_t native_sz_index(int n, int g, int K) {
    int R = n >> 4, r = n & 15, T = g >> 1, u = g & 1;
    return ((((size_t)R * (K / kTileCols) + T) * 16 + r) * 2 + u) * 2;
}

// Internal launchers (each returns the launch's hipError_t).
hipError_t launch_sq_prepack(const uint32_t* codes, const uint16_t* scales, const uint16_t* zeros,
                             int N, int K, uint32_t* codes_native, uint16_t* sz_native, hipStream_t s);
hipError_t launch_vq_prepack(const uint32_t* indices, int N, int K, int kbits, uint32_t* out,
                             hipStream_t s);
hipError_t launch_dequant(const MatDev& m, void* w_out, int w_dtype, hipStream_t s);
hipError_t launch_ref_gemm(const MatDev& m, int M, int x_dtype, int y_dtype, hipStream_t s);
// The token-shift mix in front of a batch-1 GEMV: the previous token's activations and the mix
// weight (indices of 2-vectors, one per column pair, and its codebook of E fp16 pairs).
struct MixDev { const void* x_prev; const uint8_t* idx; const uint16_t* cb; int E; };
// Element-wise operator on a batch-1 projection's output (values as in rwkvq.h's RWKVQ_POST_*).
enum PostOp : int { POST_NONE = 0, POST_RELU2 = 1, POST_SIGMOID_GATE = 2 };
struct PostDev { int op; const void* gate; };
// The output of a batch-1 projection also written as up to four token-shift mixes (next stage's inputs).
struct PostMixDev { const void* x_prev; int n_mix; const uint8_t* idx[4]; const uint16_t* cb[4]; void* out[4]; };
hipError_t launch_decode_postmix(const MatDev* mats, const PostDev* posts, const PostMixDev* pm, int n_mats,
                                 int x_dtype, int y_dtype, hipStream_t s);
// Batch 1: the three projections r, k, v of time mixing (equal N) and, in the same launch, the wkv step
// with its gate for the 16 channels of every row tile (state updated in place, `out` = sigma(r) wkv).
struct WkvDev { const float* w; const float* u; float* state; void* out; };
hipError_t launch_decode_rkv_wkv(const MatDev* rkv, const WkvDev& wkv, int x_dtype, int y_dtype, hipStream_t s);
// posts: nullptr, or one PostDev per matrix (M must be 1 then)
hipError_t launch_decode_mixed(const MatDev* mats, const MixDev* mixes, int n_mats, int x_dtype, int y_dtype,
                               hipStream_t s, const PostDev* posts = nullptr);
hipError_t launch_decode(const MatDev* mats, int n_mats, int M, int x_dtype, int y_dtype,
                         hipStream_t s, const PostDev* posts = nullptr);
hipError_t launch_prefill(const MatDev* mats, int n_mats, int M, int x_dtype, int y_dtype,
                          hipStream_t s);

hipError_t launch_proxy(const void* const* ws, const int* Ns, const int* Ks, int n_mats, int dtype,
                        int terms, double tau_c, double tau_f, uint32_t* bitmaps, double* out, int32_t* phi,
                        hipStream_t s);
// Host-side checks of a proxy call (everything but the workspace); RWKVQ_OK or the status to return.
int check_proxy_args(const void* const* ws, const int* Ns, const int* Ks, int n_mats, int w_dtype, int terms,
                     const double* proxies, const int32_t* phi, bool allow_f32);
// binary32 matrices: really sorted (proxy_f32.hip); the matrices of a call share the sort buffers
size_t proxy_f32_workspace_bytes(const int* Ns, const int* Ks, int n_mats);
hipError_t launch_proxy_f32(const void* const* ws, const int* Ns, const int* Ks, int n_mats, int terms, double tau_c,
                            double tau_f, void* workspace, double* out, int32_t* phi, hipStream_t s);

hipError_t launch_sq_encode(const void* w, int wdt, int N, int K, uint32_t* codes, uint16_t* scales,
                            uint16_t* zeros, hipStream_t s);
hipError_t launch_vq_assign(const void* w, int wdt, int N, int K, int kbits, const uint16_t* codebooks,
                            uint32_t* indices, hipStream_t s);
hipError_t launch_clip_mean(const void* x, int dt, int B, int n, int k_lo, double f_lo, int k_hi, double f_hi,
                            float* out, hipStream_t s);
hipError_t launch_mu_codebook(const void* const* mus, const float* const* xbars, const int* n_elems, int n_tensors,
                              int dt, int kbits, int iters, void* const* cbs, uint8_t* const* idx, hipStream_t s);
hipError_t launch_token_shift_mix(const void* x, const void* x_prev, int dt, int M, int d, const uint8_t* const* idx,
                                  const void* const* cbs, int kbits, int n_proj, void* const* outs, hipStream_t s);
hipError_t launch_wkv(const void* r, const void* k, const void* v, int dt, int M, int d, const float* w, const float* u,
                      float* state, void* out, hipStream_t s);
hipError_t launch_pointwise(int op, const void* x, const void* y, int dt, long long n, void* out, hipStream_t s);

// Process-wide settings behind rwkvq_set_option (values of RWKVQ_OPT_* in rwkvq.h); option() is an atomic load.
constexpr int kOptionCount = 10;
int option(int which);

constexpr int kDecodeMaxM = 16;    // native layout: M <= this goes to the streaming kernels
constexpr int kDecodeMaxK = 20480; // ... whose per-group activation sums for K columns fit their LDS

}  // namespace rwkvq
