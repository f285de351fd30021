// The C ABI of librwkvq (declared in include/rwkvq.h): argument validation on the host, then
// the launch.  No entry point allocates device memory or synchronises.
#include "common.h"
#include "../../include/rwkvq.h"

#include <cmath>
#include <algorithm>
#include <atomic>
#include <vector>

using namespace rwkvq;

namespace {

inline bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

int check_dtype_x(int dt) { return (dt == RWKVQ_F16 || dt == RWKVQ_BF16) ? RWKVQ_OK : RWKVQ_ERR_UNSUPPORTED; }
int check_dtype_y(int dt) {
    return (dt == RWKVQ_F16 || dt == RWKVQ_BF16 || dt == RWKVQ_F32) ? RWKVQ_OK : RWKVQ_ERR_UNSUPPORTED;
}

int check_sq_format(int N, int K, int bits, int group) {
    if (bits != 3 || group != kGroup) return RWKVQ_ERR_UNSUPPORTED;
    if (N <= 0 || K <= 0 || N % kTileRows != 0 || K % kTileCols != 0) return RWKVQ_ERR_SHAPE;
    return RWKVQ_OK;
}
int check_vq_format(int N, int K, int vdim, int kbits, int br, int bc) {
    if (vdim != 2 || (kbits != 6 && kbits != 8) || br != kBlock || bc != kBlock) return RWKVQ_ERR_UNSUPPORTED;
    if (N <= 0 || K <= 0 || N % kBlock != 0 || K % kBlock != 0) return RWKVQ_ERR_SHAPE;
    return RWKVQ_OK;
}
int check_layout(int layout) {
    return (layout == RWKVQ_CANONICAL || layout == RWKVQ_NATIVE) ? RWKVQ_OK : RWKVQ_ERR_UNSUPPORTED;
}

// Validate one descriptor and translate it for the kernels.
int to_dev(const rwkvq_matrix& m, const void* x, void* y, MatDev* out) {
    int st;
    if ((st = check_layout(m.layout)) != RWKVQ_OK) return st;
    if (m.kind == RWKVQ_SQ) {
        if ((st = check_sq_format(m.N, m.K, m.bits, m.group)) != RWKVQ_OK) return st;
        if (!m.codes || !m.scales) return RWKVQ_ERR_NULL;
        if (m.layout == RWKVQ_CANONICAL && !m.zeros) return RWKVQ_ERR_NULL;
        if (m.layout == RWKVQ_NATIVE && m.zeros) return RWKVQ_ERR_UNSUPPORTED;
        if (!aligned16(m.codes) || !aligned16(m.scales) || !aligned16(m.zeros)) return RWKVQ_ERR_ALIGN;
        *out = MatDev{(const uint32_t*)m.codes, (const uint16_t*)m.scales, (const uint16_t*)m.zeros, x, y,
                      m.N, m.K, FMT_SQ3, m.layout};
    } else if (m.kind == RWKVQ_VQ) {
        if ((st = check_vq_format(m.N, m.K, m.vdim, m.kbits, m.block_rows, m.block_cols)) != RWKVQ_OK) return st;
        if (!m.codes || !m.codebooks) return RWKVQ_ERR_NULL;
        if (!aligned16(m.codes) || !aligned16(m.codebooks)) return RWKVQ_ERR_ALIGN;
        *out = MatDev{(const uint32_t*)m.codes, (const uint16_t*)m.codebooks, nullptr, x, y, m.N, m.K,
                      m.kbits == 8 ? FMT_VQ8 : FMT_VQ6, m.layout};
    } else {
        return RWKVQ_ERR_UNSUPPORTED;
    }
    return RWKVQ_OK;
}

int finish(hipError_t e) { return e == hipSuccess ? RWKVQ_OK : RWKVQ_ERR_DEVICE; }

rwkvq_matrix sq_desc(const void* codes, const void* scales, const void* zeros, int layout, int N, int K,
                     int bits, int group) {
    rwkvq_matrix m{};
    m.kind = RWKVQ_SQ; m.layout = layout; m.N = N; m.K = K; m.bits = bits; m.group = group;
    m.codes = codes; m.scales = scales; m.zeros = zeros;
    return m;
}
rwkvq_matrix vq_desc(const void* indices, const void* codebooks, int layout, int N, int K, int vdim,
                     int kbits, int br, int bc) {
    rwkvq_matrix m{};
    m.kind = RWKVQ_VQ; m.layout = layout; m.N = N; m.K = K; m.vdim = vdim; m.kbits = kbits;
    m.block_rows = br; m.block_cols = bc; m.codes = indices; m.codebooks = codebooks;
    return m;
}

// Estimated cost, in microseconds, of the two ways to run native-layout matrices at 16 < M <= 128:
// a streaming pass over 17..32 batch rows moves `wide` GB/s of packed weights and costs at least
// `wide_min` us, one over <= 16 rows `narrow` GB/s and at least `narrow_min` us; a k-step of a 128-row
// matrix-core workgroup takes `kstep` ns, one workgroup per compute unit.  The defaults (rwkvq.h) were
// measured on the 7B shapes on one MI355X; rwkvq_set_option replaces them, or forces one path.
constexpr int kStreamPassesMaxM = 128;
constexpr int kStreamPassRows = 32;    // batch rows per pass of the streaming kernels (their largest instance)
bool stream_passes_cheaper(const std::vector<MatDev>& mats, int M) {
    for (const MatDev& d : mats)
        if (d.K > kDecodeMaxK) return false;
    const int forced = option(RWKVQ_OPT_SMALL_BATCH_PATH);
    if (forced == RWKVQ_SMALL_BATCH_STREAM) return true;
    if (forced == RWKVQ_SMALL_BATCH_MATRIX_CORES) return false;
    double bytes = 0.0, work = 0.0, longest = 0.0;
    for (const MatDev& d : mats) {
        const double nk = (double)d.N * d.K;
        bytes += d.fmt == FMT_SQ3 ? nk * 3 / 8 + nk / kGroup * 4 : nk * (d.fmt == FMT_VQ8 ? 8 : 6) / 16;
        work += (double)(d.N / 256) * (d.K / 64);
        longest = std::max(longest, (double)(d.K / 64));
    }
    const double wide = std::max(bytes / (1e3 * option(RWKVQ_OPT_STREAM_WIDE_GBPS)), (double)option(RWKVQ_OPT_STREAM_WIDE_MIN_US));
    const double narrow = std::max(bytes / (1e3 * option(RWKVQ_OPT_STREAM_NARROW_GBPS)), (double)option(RWKVQ_OPT_STREAM_NARROW_MIN_US));
    const int full = M / kStreamPassRows, rest = M % kStreamPassRows;
    const double t_stream = full * wide + (rest == 0 ? 0.0 : rest <= kDecodeMaxM ? narrow : wide);
    const double t_mfma = 1e-3 * option(RWKVQ_OPT_MFMA_KSTEP_NS) * std::max(work / 256.0, longest);
    return t_stream < t_mfma;
}

// Which kernels run each matrix of a call (values of RWKVQ_PATH_*): the one place that decides.
void plan_paths(const std::vector<MatDev>& devs, int M, std::vector<int>* path) {
    path->assign(devs.size(), RWKVQ_PATH_REFERENCE);
    std::vector<MatDev> mfma;
    for (size_t i = 0; i < devs.size(); ++i) {
        const MatDev& d = devs[i];
        if (d.layout == RWKVQ_CANONICAL) continue;
        if (M <= kDecodeMaxM && d.K <= kDecodeMaxK) (*path)[i] = RWKVQ_PATH_STREAM;
        else if (M > kDecodeMaxM && d.N % 256 == 0) { (*path)[i] = RWKVQ_PATH_MATRIX_CORES; mfma.push_back(d); }
        else if (M > kDecodeMaxM && M <= kStreamPassesMaxM && d.K <= kDecodeMaxK)
            (*path)[i] = RWKVQ_PATH_STREAM_PASSES;        // N not a multiple of 256: no matrix-core tiles
    }
    // 16 < M <= 128: the matrix-core kernel pads M to 128 rows, and a call of a few matrices gives
    // it few tiles; ceil(M / 32) passes of the streaming kernels over row blocks of x can be cheaper.
    if (!mfma.empty() && M <= kStreamPassesMaxM && stream_passes_cheaper(mfma, M))
        for (int& p : *path)
            if (p == RWKVQ_PATH_MATRIX_CORES) p = RWKVQ_PATH_STREAM_PASSES;
}

}  // namespace

namespace rwkvq {
static const int kOptionDefault[kOptionCount] = {RWKVQ_SMALL_BATCH_AUTO, 0, 2800, 4100, 24, 12, 1500, 2048, 65536, 1};
static std::atomic<int> g_option[kOptionCount] = {{RWKVQ_SMALL_BATCH_AUTO}, {0}, {2800}, {4100}, {24}, {12}, {1500}, {2048}, {65536}, {1}};
int option(int which) { return g_option[which].load(std::memory_order_relaxed); }
}  // namespace rwkvq

extern "C" {

int rwkvq_version(void) { return 101; }

int rwkvq_set_option(int opt, int value) {
    if (opt < 0 || opt >= kOptionCount) return RWKVQ_ERR_UNSUPPORTED;
    if (opt == RWKVQ_OPT_SMALL_BATCH_PATH) {
        if (value != RWKVQ_SMALL_BATCH_AUTO && value != RWKVQ_SMALL_BATCH_STREAM && value != RWKVQ_SMALL_BATCH_MATRIX_CORES)
            return RWKVQ_ERR_UNSUPPORTED;
    } else if (opt == RWKVQ_OPT_PREFILL_TILE_ROWS) {
        if (value != 0 && value != 128 && value != 256) return RWKVQ_ERR_UNSUPPORTED;
    } else {
        if (value < 0 || value > 1000000) return RWKVQ_ERR_UNSUPPORTED;
        if (value == 0) value = kOptionDefault[opt];
    }
    g_option[opt].store(value, std::memory_order_relaxed);
    return RWKVQ_OK;
}

int rwkvq_get_option(int opt, int* value) {
    if (!value) return RWKVQ_ERR_NULL;
    if (opt < 0 || opt >= kOptionCount) return RWKVQ_ERR_UNSUPPORTED;
    *value = option(opt);
    return RWKVQ_OK;
}

const char* rwkvq_status_string(int status) {
    switch (status) {
        case RWKVQ_OK: return "ok";
        case RWKVQ_ERR_NULL: return "null pointer";
        case RWKVQ_ERR_SHAPE: return "bad shape";
        case RWKVQ_ERR_UNSUPPORTED: return "unsupported format or dtype";
        case RWKVQ_ERR_ALIGN: return "pointer not 16-byte aligned";
        case RWKVQ_ERR_DEVICE: return "HIP launch error";
        default: return "unknown status";
    }
}

int rwkvq_sq_prepack(const void* codes, const void* scales, const void* zeros, int N, int K, int bits,
                     int group, void* codes_native, void* sz_native, void* stream) {
    int st = check_sq_format(N, K, bits, group);
    if (st != RWKVQ_OK) return st;
    if (!codes || !scales || !zeros || !codes_native || !sz_native) return RWKVQ_ERR_NULL;
    if (!aligned16(codes) || !aligned16(scales) || !aligned16(zeros) || !aligned16(codes_native) ||
        !aligned16(sz_native))
        return RWKVQ_ERR_ALIGN;
    return finish(launch_sq_prepack((const uint32_t*)codes, (const uint16_t*)scales, (const uint16_t*)zeros,
                                    N, K, (uint32_t*)codes_native, (uint16_t*)sz_native, (hipStream_t)stream));
}

int rwkvq_vq_prepack(const void* indices, int N, int K, int vdim, int kbits, void* indices_native,
                     void* stream) {
    int st = check_vq_format(N, K, vdim, kbits, kBlock, kBlock);
    if (st != RWKVQ_OK) return st;
    if (!indices || !indices_native) return RWKVQ_ERR_NULL;
    if (!aligned16(indices) || !aligned16(indices_native)) return RWKVQ_ERR_ALIGN;
    return finish(launch_vq_prepack((const uint32_t*)indices, N, K, kbits, (uint32_t*)indices_native,
                                    (hipStream_t)stream));
}

int rwkvq_sq_dequant(const void* codes, const void* scales, const void* zeros, int layout, int N, int K,
                     int bits, int group, void* w_out, int w_dtype, void* stream) {
    MatDev d;
    int st = to_dev(sq_desc(codes, scales, zeros, layout, N, K, bits, group), nullptr, nullptr, &d);
    if (st != RWKVQ_OK) return st;
    if ((st = check_dtype_y(w_dtype)) != RWKVQ_OK) return st;
    if (!w_out) return RWKVQ_ERR_NULL;
    if (!aligned16(w_out)) return RWKVQ_ERR_ALIGN;
    return finish(launch_dequant(d, w_out, w_dtype, (hipStream_t)stream));
}

int rwkvq_vq_dequant(const void* indices, const void* codebooks, int layout, int N, int K, int vdim,
                     int kbits, int block_rows, int block_cols, void* w_out, int w_dtype, void* stream) {
    MatDev d;
    int st = to_dev(vq_desc(indices, codebooks, layout, N, K, vdim, kbits, block_rows, block_cols), nullptr,
                    nullptr, &d);
    if (st != RWKVQ_OK) return st;
    if ((st = check_dtype_y(w_dtype)) != RWKVQ_OK) return st;
    if (!w_out) return RWKVQ_ERR_NULL;
    if (!aligned16(w_out)) return RWKVQ_ERR_ALIGN;
    return finish(launch_dequant(d, w_out, w_dtype, (hipStream_t)stream));
}

int rwkvq_linear_dispatch(const rwkvq_matrix* mats, const void* const* xs, void* const* ys, int n_mats,
                          int M, int x_dtype, int y_dtype, void* stream) {
    if (!mats || !xs || !ys) return RWKVQ_ERR_NULL;
    if (n_mats <= 0 || M <= 0 || M > (1 << 19)) return RWKVQ_ERR_SHAPE;
    int st;
    if ((st = check_dtype_x(x_dtype)) != RWKVQ_OK) return st;
    if ((st = check_dtype_y(y_dtype)) != RWKVQ_OK) return st;
    std::vector<MatDev> devs((size_t)n_mats);
    for (int i = 0; i < n_mats; ++i) {
        if (!xs[i] || !ys[i]) return RWKVQ_ERR_NULL;
        if (!aligned16(xs[i]) || !aligned16(ys[i])) return RWKVQ_ERR_ALIGN;
        if ((st = to_dev(mats[i], xs[i], ys[i], &devs[(size_t)i])) != RWKVQ_OK) return st;
    }
    std::vector<int> path;
    plan_paths(devs, M, &path);
    std::vector<MatDev> decode, prefill, passes, ref;
    for (size_t i = 0; i < devs.size(); ++i)
        (path[i] == RWKVQ_PATH_STREAM ? decode : path[i] == RWKVQ_PATH_MATRIX_CORES ? prefill
         : path[i] == RWKVQ_PATH_STREAM_PASSES ? passes : ref).push_back(devs[i]);
    hipStream_t s = (hipStream_t)stream;
    for (const MatDev& d : ref) {
        hipError_t e = launch_ref_gemm(d, M, x_dtype, y_dtype, s);
        if (e != hipSuccess) return RWKVQ_ERR_DEVICE;
    }
    if (!decode.empty()) {
        hipError_t e = launch_decode(decode.data(), (int)decode.size(), M, x_dtype, y_dtype, s);
        if (e != hipSuccess) return RWKVQ_ERR_DEVICE;
    }
    if (!passes.empty()) {
        const size_t ysz = y_dtype == RWKVQ_F32 ? 4 : 2;
        std::vector<MatDev> blk(passes);
        for (int m0 = 0; m0 < M; m0 += kStreamPassRows) {
            for (size_t i = 0; i < blk.size(); ++i) {
                blk[i].x = (const char*)passes[i].x + (size_t)m0 * passes[i].K * 2;
                blk[i].y = (char*)passes[i].y + (size_t)m0 * passes[i].N * ysz;
            }
            hipError_t e = launch_decode(blk.data(), (int)blk.size(), M - m0 < kStreamPassRows ? M - m0 : kStreamPassRows,
                                         x_dtype, y_dtype, s);
            if (e != hipSuccess) return RWKVQ_ERR_DEVICE;
        }
    }
    if (!prefill.empty()) {
        hipError_t e = launch_prefill(prefill.data(), (int)prefill.size(), M, x_dtype, y_dtype, s);
        if (e != hipSuccess) return RWKVQ_ERR_DEVICE;
    }
    return RWKVQ_OK;
}

int rwkvq_linear_dispatch_plan(const rwkvq_matrix* mats, int n_mats, int M, int32_t* paths) {
    if (!mats || !paths) return RWKVQ_ERR_NULL;
    if (n_mats <= 0 || M <= 0 || M > (1 << 19)) return RWKVQ_ERR_SHAPE;
    std::vector<MatDev> devs((size_t)n_mats);
    for (int i = 0; i < n_mats; ++i) {
        int st = to_dev(mats[i], nullptr, nullptr, &devs[(size_t)i]);
        if (st != RWKVQ_OK) return st;
    }
    std::vector<int> path;
    plan_paths(devs, M, &path);
    for (int i = 0; i < n_mats; ++i) paths[i] = path[(size_t)i];
    return RWKVQ_OK;
}

int rwkvq_sq_gemm(const void* codes, const void* scales, const void* zeros, int layout, const void* x,
                  void* y, int M, int N, int K, int bits, int group, int x_dtype, int y_dtype, void* stream) {
    rwkvq_matrix m = sq_desc(codes, scales, zeros, layout, N, K, bits, group);
    return rwkvq_linear_dispatch(&m, &x, &y, 1, M, x_dtype, y_dtype, stream);
}

int rwkvq_vq_gemm(const void* indices, const void* codebooks, int layout, const void* x, void* y, int M,
                  int N, int K, int vdim, int kbits, int block_rows, int block_cols, int x_dtype,
                  int y_dtype, void* stream) {
    rwkvq_matrix m = vq_desc(indices, codebooks, layout, N, K, vdim, kbits, block_rows, block_cols);
    return rwkvq_linear_dispatch(&m, &x, &y, 1, M, x_dtype, y_dtype, stream);
}

size_t rwkvq_proxy_workspace_bytes(int n_mats) {          /* one bit per 16-bit pattern and matrix */
    return n_mats > 0 ? (size_t)n_mats * (65536 / 8) : 0;
}

size_t rwkvq_proxy_workspace_size(const int* Ns, const int* Ks, int n_mats, int w_dtype) {
    if (!Ns || !Ks || n_mats < 1) return 0;
    if (w_dtype == RWKVQ_F16 || w_dtype == RWKVQ_BF16) return rwkvq_proxy_workspace_bytes(n_mats);
    if (w_dtype != RWKVQ_F32) return 0;
    for (int i = 0; i < n_mats; ++i)
        if (Ns[i] < 1 || Ks[i] < 1 || (unsigned long long)Ns[i] * (unsigned long long)Ks[i] > 0xFFFFFFFFull) return 0;
    return proxy_f32_workspace_bytes(Ns, Ks, n_mats);
}

int rwkvq_proxy(const void* const* ws, const int* Ns, const int* Ks, int n_mats, int w_dtype, int terms,
                double tau_c, double tau_f, void* workspace, double* proxies, int32_t* phi, void* stream) {
    if (!workspace) return RWKVQ_ERR_NULL;
    const int st = check_proxy_args(ws, Ns, Ks, n_mats, w_dtype, terms, proxies, phi, true);
    if (st != RWKVQ_OK) return st;
    if (!aligned16(workspace)) return RWKVQ_ERR_ALIGN;
    hipError_t e;
    if (w_dtype == RWKVQ_F32)
        e = launch_proxy_f32(ws, Ns, Ks, n_mats, terms, tau_c, tau_f, workspace, proxies, phi, (hipStream_t)stream);
    else
        e = launch_proxy(ws, Ns, Ks, n_mats, w_dtype == RWKVQ_F16 ? DT_F16 : DT_BF16, terms, tau_c, tau_f,
                         (uint32_t*)workspace, proxies, phi, (hipStream_t)stream);
    return e == hipSuccess ? RWKVQ_OK : RWKVQ_ERR_DEVICE;
}

static int dense_dtype(int w_dtype) {
    return w_dtype == RWKVQ_F16 ? DT_F16 : w_dtype == RWKVQ_BF16 ? DT_BF16 : w_dtype == RWKVQ_F32 ? DT_F32 : -1;
}

int rwkvq_sq_encode(const void* w, int w_dtype, int N, int K, int bits, int group, void* codes, void* scales,
                    void* zeros, void* stream) {
    if (!w || !codes || !scales || !zeros) return RWKVQ_ERR_NULL;
    if (bits != 3 || group != 128 || dense_dtype(w_dtype) < 0) return RWKVQ_ERR_UNSUPPORTED;
    if (N < 1 || K < 1 || K % 128 != 0) return RWKVQ_ERR_SHAPE;
    if (!aligned16(w) || !aligned16(codes) || !aligned16(scales) || !aligned16(zeros)) return RWKVQ_ERR_ALIGN;
    hipError_t e = launch_sq_encode(w, dense_dtype(w_dtype), N, K, (uint32_t*)codes, (uint16_t*)scales,
                                    (uint16_t*)zeros, (hipStream_t)stream);
    return e == hipSuccess ? RWKVQ_OK : RWKVQ_ERR_DEVICE;
}

int rwkvq_vq_assign(const void* w, int w_dtype, const void* codebooks, int N, int K, int vdim, int kbits,
                    int block_rows, int block_cols, void* indices, void* stream) {
    if (!w || !codebooks || !indices) return RWKVQ_ERR_NULL;
    if (vdim != 2 || (kbits != 6 && kbits != 8) || block_rows != 256 || block_cols != 256 || dense_dtype(w_dtype) < 0)
        return RWKVQ_ERR_UNSUPPORTED;
    if (N < 1 || K < 1 || N % 256 != 0 || K % 256 != 0) return RWKVQ_ERR_SHAPE;
    if (!aligned16(w) || !aligned16(codebooks) || !aligned16(indices)) return RWKVQ_ERR_ALIGN;
    hipError_t e = launch_vq_assign(w, dense_dtype(w_dtype), N, K, kbits, (const uint16_t*)codebooks,
                                    (uint32_t*)indices, (hipStream_t)stream);
    return e == hipSuccess ? RWKVQ_OK : RWKVQ_ERR_DEVICE;
}

int rwkvq_clip_mean(const void* x, int x_dtype, int n_samples, int n, double percentile, float* xbar, void* stream) {
    if (!x || !xbar) return RWKVQ_ERR_NULL;
    if (dense_dtype(x_dtype) < 0) return RWKVQ_ERR_UNSUPPORTED;
    if (n_samples < 1 || n_samples > 65536 || n < 1) return RWKVQ_ERR_SHAPE;
    if (!(percentile >= 0.0 && percentile <= 50.0)) return RWKVQ_ERR_UNSUPPORTED;
    if (!aligned16(x) || ((uintptr_t)xbar & 3u)) return RWKVQ_ERR_ALIGN;
    // rank of the q-th percentile among B ordered samples: r = (B - 1) q / 100, split into its
    // integer part and the interpolation weight (binary64, the formula the definition states)
    const double r_lo = (n_samples - 1) * (percentile / 100.0), r_hi = (n_samples - 1) * ((100.0 - percentile) / 100.0);
    const int k_lo = (int)std::floor(r_lo), k_hi = (int)std::floor(r_hi);
    hipError_t e = launch_clip_mean(x, dense_dtype(x_dtype), n_samples, n, k_lo, r_lo - k_lo, k_hi, r_hi - k_hi, xbar,
                                    (hipStream_t)stream);
    return e == hipSuccess ? RWKVQ_OK : RWKVQ_ERR_DEVICE;
}

int rwkvq_mu_codebook(const void* const* mus, const float* const* xbars, const int* n_elems, int n_tensors,
                      int mu_dtype, int kbits, int iters, void* const* codebooks, uint8_t* const* indices,
                      void* stream) {
    if (!mus || !xbars || !n_elems || !codebooks || !indices) return RWKVQ_ERR_NULL;
    if (n_tensors < 1) return RWKVQ_ERR_SHAPE;
    if ((kbits != 6 && kbits != 8) || dense_dtype(mu_dtype) < 0 || iters < 0 || iters > 1000) return RWKVQ_ERR_UNSUPPORTED;
    for (int i = 0; i < n_tensors; ++i) {
        if (!mus[i] || !xbars[i] || !codebooks[i] || !indices[i]) return RWKVQ_ERR_NULL;
        if (n_elems[i] < 2 || (n_elems[i] & 1)) return RWKVQ_ERR_SHAPE;
        if (!aligned16(mus[i]) || !aligned16(xbars[i]) || !aligned16(codebooks[i])) return RWKVQ_ERR_ALIGN;
    }
    hipError_t e = launch_mu_codebook(mus, xbars, n_elems, n_tensors, dense_dtype(mu_dtype), kbits, iters, codebooks,
                                      indices, (hipStream_t)stream);
    return e == hipSuccess ? RWKVQ_OK : RWKVQ_ERR_DEVICE;
}

int rwkvq_token_shift_mix(const void* x, const void* x_prev, int x_dtype, int M, int d, const uint8_t* const* indices,
                          const void* const* codebooks, int kbits, int n_proj, void* const* outs, void* stream) {
    if (!x || !x_prev || !indices || !codebooks || !outs) return RWKVQ_ERR_NULL;
    if (x_dtype != RWKVQ_F16 && x_dtype != RWKVQ_BF16) return RWKVQ_ERR_UNSUPPORTED;
    if ((kbits != 6 && kbits != 8) || n_proj < 1 || n_proj > 8) return RWKVQ_ERR_UNSUPPORTED;
    if (M < 1 || d < 8 || d % 8 != 0 || (long long)M * d > (1ll << 40)) return RWKVQ_ERR_SHAPE;
    if (!aligned16(x) || !aligned16(x_prev)) return RWKVQ_ERR_ALIGN;
    for (int p = 0; p < n_proj; ++p) {
        if (!indices[p] || !codebooks[p] || !outs[p]) return RWKVQ_ERR_NULL;
        if (!aligned16(indices[p]) || !aligned16(codebooks[p]) || !aligned16(outs[p])) return RWKVQ_ERR_ALIGN;
    }
    hipError_t e = launch_token_shift_mix(x, x_prev, x_dtype == RWKVQ_F16 ? DT_F16 : DT_BF16, M, d, indices, codebooks,
                                          kbits, n_proj, outs, (hipStream_t)stream);
    return e == hipSuccess ? RWKVQ_OK : RWKVQ_ERR_DEVICE;
}

int rwkvq_linear_dispatch_mixed(const rwkvq_matrix* mats, const rwkvq_mix_input* mixes, void* const* ys, int n_mats,
                                int x_dtype, int y_dtype, void* stream) {
    if (!mats || !mixes || !ys) return RWKVQ_ERR_NULL;
    if (n_mats <= 0) return RWKVQ_ERR_SHAPE;
    int st;
    if ((st = check_dtype_x(x_dtype)) != RWKVQ_OK) return st;
    if ((st = check_dtype_y(y_dtype)) != RWKVQ_OK) return st;
    std::vector<MatDev> md((size_t)n_mats);
    std::vector<MixDev> xd((size_t)n_mats);
    for (int i = 0; i < n_mats; ++i) {
        const rwkvq_mix_input& x = mixes[i];
        if (!x.x || !x.x_prev || !x.indices || !x.codebook || !ys[i]) return RWKVQ_ERR_NULL;
        if (x.kbits != 6 && x.kbits != 8) return RWKVQ_ERR_UNSUPPORTED;
        if (!aligned16(x.x) || !aligned16(x.x_prev) || !aligned16(x.indices) || !aligned16(x.codebook) || !aligned16(ys[i]))
            return RWKVQ_ERR_ALIGN;
        if ((st = to_dev(mats[i], x.x, ys[i], &md[(size_t)i])) != RWKVQ_OK) return st;
        if (md[(size_t)i].layout != RWKVQ_NATIVE || md[(size_t)i].K > kDecodeMaxK) return RWKVQ_ERR_UNSUPPORTED;
        xd[(size_t)i] = MixDev{x.x_prev, x.indices, (const uint16_t*)x.codebook, 1 << x.kbits};
    }
    hipError_t e = launch_decode_mixed(md.data(), xd.data(), n_mats, x_dtype, y_dtype, (hipStream_t)stream);
    return e == hipSuccess ? RWKVQ_OK : RWKVQ_ERR_DEVICE;
}

int rwkvq_linear_dispatch_post(const rwkvq_matrix* mats, const void* const* xs, const rwkvq_mix_input* mixes,
                               const rwkvq_post_op* posts, void* const* ys, int n_mats, int x_dtype, int y_dtype,
                               void* stream) {
    if (!mats || !posts || !ys || (!xs && !mixes)) return RWKVQ_ERR_NULL;
    if (n_mats <= 0) return RWKVQ_ERR_SHAPE;
    int st;
    if ((st = check_dtype_x(x_dtype)) != RWKVQ_OK) return st;
    if ((st = check_dtype_y(y_dtype)) != RWKVQ_OK) return st;
    std::vector<MatDev> md((size_t)n_mats);
    std::vector<MixDev> xd((size_t)n_mats);
    std::vector<PostDev> pd((size_t)n_mats);
    std::vector<PostMixDev> pmd((size_t)n_mats);
    bool any_mix = false;
    for (int i = 0; i < n_mats; ++i) {
        const void* x = mixes ? mixes[i].x : xs[i];
        if (!x || !ys[i]) return RWKVQ_ERR_NULL;
        if (!aligned16(x) || !aligned16(ys[i])) return RWKVQ_ERR_ALIGN;
        if (mixes) {
            const rwkvq_mix_input& m = mixes[i];
            if (!m.x_prev || !m.indices || !m.codebook) return RWKVQ_ERR_NULL;
            if (m.kbits != 6 && m.kbits != 8) return RWKVQ_ERR_UNSUPPORTED;
            if (!aligned16(m.x_prev) || !aligned16(m.indices) || !aligned16(m.codebook)) return RWKVQ_ERR_ALIGN;
            xd[(size_t)i] = MixDev{m.x_prev, m.indices, (const uint16_t*)m.codebook, 1 << m.kbits};
        }
        const rwkvq_post_op& p = posts[i];
        if (p.op != RWKVQ_POST_NONE && p.op != RWKVQ_POST_RELU2 && p.op != RWKVQ_POST_SIGMOID_GATE) return RWKVQ_ERR_UNSUPPORTED;
        if (p.op == RWKVQ_POST_SIGMOID_GATE) {
            if (!p.gate) return RWKVQ_ERR_NULL;
            if (!aligned16(p.gate)) return RWKVQ_ERR_ALIGN;
        }
        pd[(size_t)i] = PostDev{p.op, p.op == RWKVQ_POST_SIGMOID_GATE ? p.gate : nullptr};
        if (p.n_mix < 0 || p.n_mix > 4) return RWKVQ_ERR_UNSUPPORTED;
        PostMixDev& pm = pmd[(size_t)i];
        pm = PostMixDev{};
        pm.n_mix = p.n_mix;
        if (p.n_mix > 0) {
            any_mix = true;
            if (mixes || (y_dtype != RWKVQ_F16 && y_dtype != RWKVQ_BF16)) return RWKVQ_ERR_UNSUPPORTED;
            if (!p.x_prev) return RWKVQ_ERR_NULL;
            if (!aligned16(p.x_prev)) return RWKVQ_ERR_ALIGN;
            pm.x_prev = p.x_prev;
            for (int q = 0; q < p.n_mix; ++q) {
                const rwkvq_post_mix& m = p.mix[q];
                if (!m.indices || !m.codebook || !m.out) return RWKVQ_ERR_NULL;
                if (m.kbits != 6 && m.kbits != 8) return RWKVQ_ERR_UNSUPPORTED;
                if (!aligned16(m.indices) || !aligned16(m.codebook) || !aligned16(m.out)) return RWKVQ_ERR_ALIGN;
                pm.idx[q] = m.indices; pm.cb[q] = (const uint16_t*)m.codebook; pm.out[q] = m.out;
            }
        }
        if ((st = to_dev(mats[i], x, ys[i], &md[(size_t)i])) != RWKVQ_OK) return st;
        if (md[(size_t)i].layout != RWKVQ_NATIVE || md[(size_t)i].K > kDecodeMaxK) return RWKVQ_ERR_UNSUPPORTED;
    }
    hipError_t e = mixes     ? launch_decode_mixed(md.data(), xd.data(), n_mats, x_dtype, y_dtype, (hipStream_t)stream, pd.data())
                   : any_mix ? launch_decode_postmix(md.data(), pd.data(), pmd.data(), n_mats, x_dtype, y_dtype, (hipStream_t)stream)
                             : launch_decode(md.data(), n_mats, 1, x_dtype, y_dtype, (hipStream_t)stream, pd.data());
    return e == hipSuccess ? RWKVQ_OK : RWKVQ_ERR_DEVICE;
}

int rwkvq_rkv_wkv(const rwkvq_matrix* rkv, const void* const* xs, void* const* ys, const float* w, const float* u,
                  float* state, void* out, int x_dtype, int y_dtype, void* stream) {
    if (!rkv || !xs || !ys || !w || !u || !state || !out) return RWKVQ_ERR_NULL;
    int st;
    if ((st = check_dtype_x(x_dtype)) != RWKVQ_OK) return st;
    if (y_dtype != RWKVQ_F16 && y_dtype != RWKVQ_BF16) return RWKVQ_ERR_UNSUPPORTED;
    MatDev md[3];
    for (int i = 0; i < 3; ++i) {
        if (!xs[i] || !ys[i]) return RWKVQ_ERR_NULL;
        if (!aligned16(xs[i]) || !aligned16(ys[i])) return RWKVQ_ERR_ALIGN;
        if ((st = to_dev(rkv[i], xs[i], ys[i], &md[i])) != RWKVQ_OK) return st;
        if (md[i].layout != RWKVQ_NATIVE || md[i].K > kDecodeMaxK) return RWKVQ_ERR_UNSUPPORTED;
        if (md[i].N != md[0].N) return RWKVQ_ERR_SHAPE;
    }
    if (!aligned16(out) || ((uintptr_t)w & 3u) || ((uintptr_t)u & 3u) || ((uintptr_t)state & 3u)) return RWKVQ_ERR_ALIGN;
    hipError_t e = launch_decode_rkv_wkv(md, WkvDev{w, u, state, out}, x_dtype, y_dtype, (hipStream_t)stream);
    return e == hipSuccess ? RWKVQ_OK : RWKVQ_ERR_DEVICE;
}

int rwkvq_wkv(const void* r, const void* k, const void* v, int x_dtype, int M, int d, const float* w, const float* u,
              float* state, void* out, void* stream) {
    if (!r || !k || !v || !w || !u || !state || !out) return RWKVQ_ERR_NULL;
    if (x_dtype != RWKVQ_F16 && x_dtype != RWKVQ_BF16) return RWKVQ_ERR_UNSUPPORTED;
    if (M < 1 || d < 1 || (long long)M * d > (1ll << 40)) return RWKVQ_ERR_SHAPE;
    if (!aligned16(r) || !aligned16(k) || !aligned16(v) || !aligned16(out) || ((uintptr_t)w & 3u) || ((uintptr_t)u & 3u) ||
        ((uintptr_t)state & 3u))
        return RWKVQ_ERR_ALIGN;
    hipError_t e = launch_wkv(r, k, v, x_dtype == RWKVQ_F16 ? DT_F16 : DT_BF16, M, d, w, u, state, out, (hipStream_t)stream);
    return e == hipSuccess ? RWKVQ_OK : RWKVQ_ERR_DEVICE;
}

static int pointwise(int op, const void* x, const void* y, int x_dtype, long long n, void* out, void* stream) {
    if (!x || !y || !out) return RWKVQ_ERR_NULL;
    if (x_dtype != RWKVQ_F16 && x_dtype != RWKVQ_BF16) return RWKVQ_ERR_UNSUPPORTED;
    if (n < 1 || n > (1ll << 40)) return RWKVQ_ERR_SHAPE;
    if (!aligned16(x) || !aligned16(y) || !aligned16(out)) return RWKVQ_ERR_ALIGN;
    hipError_t e = launch_pointwise(op, x, y, x_dtype == RWKVQ_F16 ? DT_F16 : DT_BF16, n, out, (hipStream_t)stream);
    return e == hipSuccess ? RWKVQ_OK : RWKVQ_ERR_DEVICE;
}

int rwkvq_relu2(const void* x, int x_dtype, long long n, void* out, void* stream) {
    return pointwise(0, x, x, x_dtype, n, out, stream);
}

int rwkvq_sigmoid_gate(const void* r, const void* y, int x_dtype, long long n, void* out, void* stream) {
    return pointwise(1, r, y, x_dtype, n, out, stream);
}

}  // extern "C"
