// C ABI of the qvggt library: argument validation on the host, then kernel launches on the
// caller's stream.  Declarations and the meaning of every argument are in include/qvggt.h.
#include "qvggt_common.h"
#include "../../include/qvggt.h"

#include <atomic>
#include <cmath>
#include <mutex>

// The library's own workspace (see own_workspace_ptr below): device memory, one copy per device.
static __device__ __align__(256) unsigned char scratch[QVGGT_OWN_WORKSPACE_BYTES];

namespace qvggt {
namespace {
// What the library remembers between calls: which kernels need a raised dynamic-LDS limit (a list written while the library
// is loaded, read-only afterwards) and on which devices that has been done.
constexpr int kMaxLdsKernels = 96, kMaxDevices = 64;
struct LdsRegistry {
    LdsKernel kernels[kMaxLdsKernels];
    int n;
};
LdsRegistry &lds_registry()
{
    static LdsRegistry r{};      // function-local: constructed before the first static LdsKernels object uses it
    return r;
}
std::atomic<int> device_ready[kMaxDevices];
std::mutex prepare_mutex;

// The library's own workspace, for qvggt_linear_e2m3_own_workspace: what qvggt_linear_e2m3 keeps in its workspace argument (the
// activation codes as E2M3 blocks and the per-token steps between the two kernels) lives here instead.  Every device that runs the
// library holds its own copy of the array at its own address until the process ends; in host code the array's name is only a
// handle for hipGetSymbolAddress, the address kernels are given is own_workspace_ptr[device].
void *own_workspace_ptr[kMaxDevices];      // written under prepare_mutex before device_ready is released
}  // namespace

void register_lds_kernels(const LdsKernel *list, int n)
{
    LdsRegistry &r = lds_registry();
    for (int i = 0; i < n && r.n < kMaxLdsKernels; ++i) r.kernels[r.n++] = list[i];
}

hipError_t prepare_device(int *device)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    if (device != nullptr) *device = dev;
    if (device_ready[dev].load(std::memory_order_acquire)) return hipSuccess;
    std::lock_guard<std::mutex> lock(prepare_mutex);
    if (device_ready[dev].load(std::memory_order_relaxed)) return hipSuccess;
    const LdsRegistry &r = lds_registry();
    for (int i = 0; i < r.n; ++i) {
        e = hipFuncSetAttribute(r.kernels[i].fn, hipFuncAttributeMaxDynamicSharedMemorySize, r.kernels[i].lds_bytes);
        if (e != hipSuccess) return e;
    }
    void *p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));      // this device's copy of the array
    if (e != hipSuccess) return e;
    if (p == nullptr) return hipErrorInvalidSymbol;
    own_workspace_ptr[dev] = p;
    device_ready[dev].store(1, std::memory_order_release);
    return hipSuccess;
}

// the current device's copy of the library's own workspace (nullptr and an error if the device cannot be prepared)
static hipError_t own_workspace(void **ptr)
{
    int dev = -1;
    *ptr = nullptr;
    hipError_t e = prepare_device(&dev);
    if (e != hipSuccess) return e;
    *ptr = own_workspace_ptr[dev];
    return hipSuccess;
}

hipError_t run_rotate_smooth_quant(const void *X, bool f32, int rows, int K, const int8_t *signs, const float *mul,
                                   int mul_mode, uint8_t *packed, float *scale, const float *step, int step_stride,
                                   int bits, hipStream_t stream);
hipError_t run_rotated_col_absmax(const void *X, bool f32, int rows, int K, const int8_t *signs, float *absmax,
                                  hipStream_t stream);
hipError_t run_smooth_factor(float *buf, const float *act_absmax, int K, float alpha, hipStream_t stream);
hipError_t run_inv_from_factor(float *buf, const float *c, int K, hipStream_t stream);
hipError_t run_fill_f32(float *p, int n, float v, hipStream_t stream);
hipError_t run_pack_int4(const int8_t *codes, int rows, int K, uint8_t *packed, hipStream_t stream);
hipError_t run_unpack_int4(const uint8_t *packed, int rows, int K, int8_t *codes, hipStream_t stream);
bool general_size_supported(int K);
hipError_t run_ln_rotate_smooth_quant(const void *X, bool f32, int rows, int K, LnParams ln, const int8_t *signs, const float *mul,
                                      uint8_t *packed, float *scale, hipStream_t stream);
hipError_t run_rotate_smooth_quant_asym(const void *X, bool f32, int rows, int K, const int8_t *signs, const float *mul,
                                        uint8_t *packed, float *scale, float *zero, hipStream_t stream);
hipError_t run_code_sums(const uint8_t *packed, int rows, int K, float *sums, hipStream_t stream);
hipError_t run_w4a4_gemm_asym(const uint8_t *Xq, const float *sx, const float *xzero, const uint8_t *Wq, const float *sw,
                              const float *wsum, const void *bias, int M, int N, int K, void *Y, hipStream_t stream);
hipError_t run_rotate_quant_e2m3_mfma(const void *X, int rows, int K, const int8_t *signs, const float *mul, uint8_t *out,
                                      float *scale, hipStream_t stream);
hipError_t run_ln_rotate_quant_e2m3_mfma(const void *X, int rows, const int8_t *signs, const float *mul, uint8_t *out, float *scale,
                                         LnParams ln, hipStream_t stream);
hipError_t run_rotate_quant_e2m3_shifted_mfma(const void *X, int rows, int K, const int8_t *signs, const float *mul, uint8_t *out,
                                              float *scale, float *zero, const float *step, int step_stride, hipStream_t stream);
hipError_t run_e2m3_gemm_shifted(const uint8_t *Xf, const float *sx, const float *xzero, const uint8_t *Wf, const float *sw,
                                 const float *wsum, const void *bias, int M, int N, int K, void *Y, hipStream_t stream);
hipError_t run_gelu_rotate_quant_mfma(const void *X, int rows, int K, const int8_t *signs, const float *mul, const void *gelu_table,
                                      uint8_t *out, float *scale, bool e2m3, hipStream_t stream);
hipError_t run_gelu_table(void *table, hipStream_t stream);
hipError_t run_mfma_ceiling(int kind, int iters, float *sink, hipStream_t stream);
hipError_t run_rotate_only(const void *X, bool f32, int rows, int K, const int8_t *signs, float *out, hipStream_t stream);
size_t calib_workspace_bytes(int T, int N, int K);
hipError_t run_calib_loss_grad(const float *R, const float *V, const float *y_ref, const void *bias, const float *c_hat,
                               const float *w_step, const float *x_step, int T, int N, int K, int bits, float *loss, float *grad_c,
                               float *grad_w_step, float *grad_x_step, void *workspace, hipStream_t stream);
hipError_t run_descent_step(float *theta, const float *grad, int n, float lr, float floor_, hipStream_t stream);
hipError_t run_int8_to_blocks(const int8_t *src, int rows, int K, uint8_t *dst, hipStream_t stream);
hipError_t run_rotate_quant_i8b_mfma(const void *X, int rows, int K, const int8_t *signs, const float *mul, uint8_t *out,
                                     float *scale, int bits, hipStream_t stream);
hipError_t run_i8b_gemm(const int8_t *Xb, const float *sx, const int8_t *Wb, const float *sw, const void *bias, int M, int N,
                        int K, void *Y, int32_t *acc_debug, hipStream_t stream);
hipError_t run_codes_to_e2m3(const uint8_t *packed, int rows, int K, uint8_t *out, unsigned int *n_unrepresentable, hipStream_t stream);
hipError_t run_e2m3_gemm(const uint8_t *Xf, const float *sx, const uint8_t *Wf, const float *sw, const void *bias, int M, int N,
                         int K, void *Y, int32_t *acc_debug, hipStream_t stream);
hipError_t run_layout_int8(const int8_t *src, int rows, int K, int8_t *dst, int to_library, hipStream_t stream);
hipError_t run_w4a4_gemm(const uint8_t *Xq, const float *sx, const uint8_t *Wq, const float *sw, const void *bias,
                         int M, int N, int K, void *Y, int32_t *acc_debug, hipStream_t stream);
hipError_t run_i8_gemm(const int8_t *Xq, const float *sx, const int8_t *Wq, const float *sw, const void *bias, int M, int N,
                       int K, void *Y, int32_t *acc_debug, hipStream_t stream);
size_t nfds_workspace_bytes(int rows, long long count, bool f32);
hipError_t run_nfds_moments(const void *A, bool f32, int rows, long long count, float *mean, float *var, double *ws,
                            hipStream_t stream);
hipError_t run_nfds_frame_correlation(const void *A, bool f32, int samples, int f, long long dhat, float *c, double *ws,
                                      hipStream_t stream);
hipError_t run_nfds_scores(const float *m, const float *s, int D, int L, double eps, float *score, hipStream_t stream);
hipError_t run_nfds_keep_lowest(const float *score, int D, int n_keep, uint8_t *keep, hipStream_t stream);
hipError_t run_nfds_kmeans_step(const float *c, int n, int dim, int K, const float *cin, float *cout, int32_t *labels,
                                hipStream_t stream);
}  // namespace qvggt

namespace {

// a power of two in [128, 8192], or one of the sizes 2^n * m (m = 12, 20, 28) the general rotation kernel is built for
bool valid_k(int K) { return (K >= qvggt::kMinK && K <= qvggt::kMaxK && (K & (K - 1)) == 0) || qvggt::general_size_supported(K); }
bool valid_n(int N) { return N >= 16 && (N % 16) == 0; }
bool valid_dtype(int d) { return d == QVGGT_BF16 || d == QVGGT_F32; }
bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
int hip_status(hipError_t e) { return e == hipSuccess ? QVGGT_OK : QVGGT_ERR_HIP; }
size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
bool valid_wide_bits(int bits) { return bits >= 4 && bits <= 8; }

// offline half for either storage: bits == 4 writes packed nibbles, kInt8Container + b int8 codes of width b
int prep_weights(const void *W, int w_dtype, int N, int K, const float *act_absmax_rot, const int8_t *signs, float alpha,
                 int bits, void *Wq, float *w_scale, float *inv_smooth, void *stream)
{
    if (!valid_dtype(w_dtype)) return QVGGT_ERR_DTYPE;
    if (!valid_n(N) || !valid_k(K)) return QVGGT_ERR_SHAPE;
    if (!W || !Wq || !w_scale || !inv_smooth) return QVGGT_ERR_NULL;
    if (!aligned16(W) || !aligned16(Wq) || !aligned16(w_scale) || !aligned16(inv_smooth) ||
        !aligned16(act_absmax_rot) || !aligned16(signs))
        return QVGGT_ERR_ALIGN;
    if (!std::isfinite(alpha) || alpha < 0.0f || alpha > 1.0f) return QVGGT_ERR_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const bool f32 = w_dtype == QVGGT_F32;
    hipError_t e;
    if (act_absmax_rot != nullptr) {
        // inv_smooth doubles as the scratch for the rotated weight statistic w_j
        e = qvggt::run_rotated_col_absmax(W, f32, N, K, signs, inv_smooth, s);
        if (e != hipSuccess) return QVGGT_ERR_HIP;
        e = qvggt::run_smooth_factor(inv_smooth, act_absmax_rot, K, alpha, s);
    } else {
        e = qvggt::run_fill_f32(inv_smooth, K, 1.0f / std::sqrt((float)K), s);
    }
    if (e != hipSuccess) return QVGGT_ERR_HIP;
    // rows of W go through the same rotate / scale / quantize kernel, with c_j / sqrt(K) as the multiplier
    return hip_status(qvggt::run_rotate_smooth_quant(W, f32, N, K, signs, inv_smooth, 1, static_cast<uint8_t *>(Wq), w_scale,
                                                     nullptr, 0, bits, s));
}

}  // namespace

extern "C" {

int qvggt_init(void) { return hip_status(qvggt::prepare_device()); }

int qvggt_mfma_ceiling(int kind, int iters, float *sink, void *stream)
{
    if ((kind != 0 && kind != 1) || iters < 1 || iters > (1 << 24)) return QVGGT_ERR_ARG;
    if (!sink) return QVGGT_ERR_NULL;
    if (!aligned16(sink)) return QVGGT_ERR_ALIGN;
    return hip_status(qvggt::run_mfma_ceiling(kind, iters, sink, static_cast<hipStream_t>(stream)));
}

const char *qvggt_status_string(int status)
{
    switch (status) {
        case QVGGT_OK: return "QVGGT_OK";
        case QVGGT_ERR_NULL: return "QVGGT_ERR_NULL: a required pointer is NULL";
        case QVGGT_ERR_SHAPE: return "QVGGT_ERR_SHAPE: unsupported M, N or K";
        case QVGGT_ERR_ALIGN: return "QVGGT_ERR_ALIGN: pointer not 16-byte aligned";
        case QVGGT_ERR_DTYPE: return "QVGGT_ERR_DTYPE: dtype must be QVGGT_BF16 or QVGGT_F32";
        case QVGGT_ERR_WORKSPACE: return "QVGGT_ERR_WORKSPACE: workspace too small";
        case QVGGT_ERR_ARG: return "QVGGT_ERR_ARG: a scalar argument is outside its documented range (alpha, p in [0, 1]; flags 0 or 1; bits in 4..8; eps >= 0)";
        case QVGGT_ERR_HIP: return "QVGGT_ERR_HIP: a HIP call failed (kernel launch, or no usable device)";
        default: return "unknown qvggt status";
    }
}

int qvggt_rotated_col_absmax(const void *X_cal, int x_dtype, int M, int K, const int8_t *signs, float *absmax_rot,
                             void *stream)
{
    if (!valid_dtype(x_dtype)) return QVGGT_ERR_DTYPE;
    if (M < 0 || !valid_k(K)) return QVGGT_ERR_SHAPE;
    if (!absmax_rot || (M > 0 && !X_cal)) return QVGGT_ERR_NULL;
    if (!aligned16(X_cal) || !aligned16(absmax_rot) || !aligned16(signs)) return QVGGT_ERR_ALIGN;
    return hip_status(qvggt::run_rotated_col_absmax(X_cal, x_dtype == QVGGT_F32, M, K, signs, absmax_rot,
                                                    static_cast<hipStream_t>(stream)));
}

int qvggt_prep_weights(const void *W, int w_dtype, int N, int K, const float *act_absmax_rot, const int8_t *signs,
                       float alpha, uint8_t *Wq, float *w_scale, float *inv_smooth, void *stream)
{
    return prep_weights(W, w_dtype, N, K, act_absmax_rot, signs, alpha, 4, Wq, w_scale, inv_smooth, stream);
}

int qvggt_prep_weights_given(const void *W, int w_dtype, int N, int K, const float *c_hat, const int8_t *signs, const float *w_step,
                             int bits, void *Wq, float *w_scale, float *inv_smooth, void *stream)
{
    if (!valid_dtype(w_dtype)) return QVGGT_ERR_DTYPE;
    if (!valid_n(N) || !valid_k(K)) return QVGGT_ERR_SHAPE;
    if (!valid_wide_bits(bits)) return QVGGT_ERR_ARG;
    if (!W || !Wq || !w_scale || !inv_smooth) return QVGGT_ERR_NULL;
    if (!aligned16(W) || !aligned16(Wq) || !aligned16(w_scale) || !aligned16(inv_smooth) || !aligned16(c_hat) || !aligned16(signs) ||
        !aligned16(w_step))
        return QVGGT_ERR_ALIGN;
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipError_t e = c_hat ? qvggt::run_inv_from_factor(inv_smooth, c_hat, K, s)
                         : qvggt::run_fill_f32(inv_smooth, K, 1.0f / std::sqrt((float)K), s);
    if (e != hipSuccess) return QVGGT_ERR_HIP;
    // the same kernel as qvggt_prep_weights, with the steps given (clamp live) when w_step is not NULL
    return hip_status(qvggt::run_rotate_smooth_quant(W, w_dtype == QVGGT_F32, N, K, signs, inv_smooth, 1, static_cast<uint8_t *>(Wq),
                                                     w_scale, w_step, 1, bits == 4 ? 4 : qvggt::kInt8Container + bits, s));
}

int qvggt_prep_weights_i8(const void *W, int w_dtype, int N, int K, const float *act_absmax_rot, const int8_t *signs,
                          float alpha, int bits, int8_t *Wq, float *w_scale, float *inv_smooth, void *stream)
{
    if (!valid_wide_bits(bits)) return QVGGT_ERR_ARG;
    return prep_weights(W, w_dtype, N, K, act_absmax_rot, signs, alpha, qvggt::kInt8Container + bits, Wq, w_scale, inv_smooth, stream);
}

int qvggt_rotate_smooth_quant(const void *X, int x_dtype, int M, int K, const int8_t *signs, const float *inv_smooth,
                              uint8_t *Xq, float *x_scale, void *stream)
{
    if (!valid_dtype(x_dtype)) return QVGGT_ERR_DTYPE;
    if (M < 0 || !valid_k(K)) return QVGGT_ERR_SHAPE;
    if (M == 0) return QVGGT_OK;
    if (!X || !Xq || !x_scale) return QVGGT_ERR_NULL;
    if (!aligned16(X) || !aligned16(Xq) || !aligned16(x_scale) || !aligned16(inv_smooth) || !aligned16(signs))
        return QVGGT_ERR_ALIGN;
    return hip_status(qvggt::run_rotate_smooth_quant(X, x_dtype == QVGGT_F32, M, K, signs, inv_smooth, 0, Xq, x_scale,
                                                     nullptr, 0, 4, static_cast<hipStream_t>(stream)));
}

int qvggt_rotate_smooth_quant_i8(const void *X, int x_dtype, int M, int K, const int8_t *signs, const float *inv_smooth,
                                 int bits, int8_t *Xq, float *x_scale, void *stream)
{
    if (!valid_dtype(x_dtype)) return QVGGT_ERR_DTYPE;
    if (M < 0 || !valid_k(K)) return QVGGT_ERR_SHAPE;
    if (!valid_wide_bits(bits)) return QVGGT_ERR_ARG;
    if (M == 0) return QVGGT_OK;
    if (!X || !Xq || !x_scale) return QVGGT_ERR_NULL;
    if (!aligned16(X) || !aligned16(Xq) || !aligned16(x_scale) || !aligned16(inv_smooth) || !aligned16(signs))
        return QVGGT_ERR_ALIGN;
    return hip_status(qvggt::run_rotate_smooth_quant(X, x_dtype == QVGGT_F32, M, K, signs, inv_smooth, 0,
                                                     reinterpret_cast<uint8_t *>(Xq), x_scale, nullptr, 0,
                                                     qvggt::kInt8Container + bits, static_cast<hipStream_t>(stream)));
}

int qvggt_layernorm_rotate_smooth_quant(const void *X, int x_dtype, int M, int K, const float *gamma, const float *beta, float eps,
                                        const int8_t *signs, const float *inv_smooth, uint8_t *Xq, float *x_scale, void *stream)
{
    if (!valid_dtype(x_dtype)) return QVGGT_ERR_DTYPE;
    if (M < 0 || K < qvggt::kMinK || K > 4096 || (K & (K - 1)) != 0) return QVGGT_ERR_SHAPE;   // powers of two up to 4096 only
    if (!(eps >= 0.0f) || !std::isfinite(eps)) return QVGGT_ERR_ARG;
    if (M == 0) return QVGGT_OK;
    if (!X || !Xq || !x_scale) return QVGGT_ERR_NULL;
    if (!aligned16(X) || !aligned16(Xq) || !aligned16(x_scale) || !aligned16(inv_smooth) || !aligned16(signs) ||
        !aligned16(gamma) || !aligned16(beta))
        return QVGGT_ERR_ALIGN;
    const qvggt::LnParams ln{gamma, beta, eps, 1};
    return hip_status(qvggt::run_ln_rotate_smooth_quant(X, x_dtype == QVGGT_F32, M, K, ln, signs, inv_smooth, Xq, x_scale,
                                                        static_cast<hipStream_t>(stream)));
}

int qvggt_rotate_smooth_quant_static(const void *X, int x_dtype, int M, int K, const int8_t *signs, const float *inv_smooth,
                                     const float *x_step, int per_token, uint8_t *Xq, float *x_scale, void *stream)
{
    if (!valid_dtype(x_dtype)) return QVGGT_ERR_DTYPE;
    if (M < 0 || !valid_k(K)) return QVGGT_ERR_SHAPE;
    if (per_token != 0 && per_token != 1) return QVGGT_ERR_ARG;
    if (M == 0) return QVGGT_OK;
    if (!X || !Xq || !x_scale || !x_step) return QVGGT_ERR_NULL;
    if (!aligned16(X) || !aligned16(Xq) || !aligned16(x_scale) || !aligned16(inv_smooth) || !aligned16(signs) ||
        (reinterpret_cast<uintptr_t>(x_step) & 3u) != 0)
        return QVGGT_ERR_ALIGN;
    return hip_status(qvggt::run_rotate_smooth_quant(X, x_dtype == QVGGT_F32, M, K, signs, inv_smooth, 0, Xq, x_scale,
                                                     x_step, per_token, 4, static_cast<hipStream_t>(stream)));
}

int qvggt_w4a4_gemm(const uint8_t *Xq, const float *x_scale, const uint8_t *Wq, const float *w_scale, const void *bias,
                    int M, int N, int K, void *Y, int32_t *acc_debug, void *stream)
{
    if (M < 0 || !valid_n(N) || !valid_k(K)) return QVGGT_ERR_SHAPE;
    if (M == 0) return QVGGT_OK;
    if (!Xq || !x_scale || !Wq || !w_scale || !Y) return QVGGT_ERR_NULL;
    if (!aligned16(Xq) || !aligned16(x_scale) || !aligned16(Wq) || !aligned16(w_scale) || !aligned16(bias) ||
        !aligned16(Y) || !aligned16(acc_debug))
        return QVGGT_ERR_ALIGN;
    return hip_status(qvggt::run_w4a4_gemm(Xq, x_scale, Wq, w_scale, bias, M, N, K, Y, acc_debug,
                                           static_cast<hipStream_t>(stream)));
}

int qvggt_rotate_smooth_quant_asym(const void *X, int x_dtype, int M, int K, const int8_t *signs, const float *inv_smooth,
                                   uint8_t *Xq, float *x_scale, float *x_zero, void *stream)
{
    if (!valid_dtype(x_dtype)) return QVGGT_ERR_DTYPE;
    if (M < 0 || K < qvggt::kMinK || K > qvggt::kMaxK || (K & (K - 1)) != 0) return QVGGT_ERR_SHAPE;   // powers of two only
    if (M == 0) return QVGGT_OK;
    if (!X || !Xq || !x_scale || !x_zero) return QVGGT_ERR_NULL;
    if (!aligned16(X) || !aligned16(Xq) || !aligned16(x_scale) || !aligned16(x_zero) || !aligned16(inv_smooth) || !aligned16(signs))
        return QVGGT_ERR_ALIGN;
    return hip_status(qvggt::run_rotate_smooth_quant_asym(X, x_dtype == QVGGT_F32, M, K, signs, inv_smooth, Xq, x_scale, x_zero,
                                                          static_cast<hipStream_t>(stream)));
}

int qvggt_weight_code_sums(const uint8_t *Wq, int N, int K, float *w_codesum, void *stream)
{
    if (N < 0 || !valid_k(K)) return QVGGT_ERR_SHAPE;
    if (N == 0) return QVGGT_OK;
    if (!Wq || !w_codesum) return QVGGT_ERR_NULL;
    if (!aligned16(Wq) || !aligned16(w_codesum)) return QVGGT_ERR_ALIGN;
    return hip_status(qvggt::run_code_sums(Wq, N, K, w_codesum, static_cast<hipStream_t>(stream)));
}

int qvggt_w4a4_gemm_asym(const uint8_t *Xq, const float *x_scale, const float *x_zero, const uint8_t *Wq, const float *w_scale,
                         const float *w_codesum, const void *bias, int M, int N, int K, void *Y, void *stream)
{
    if (M < 0 || !valid_n(N) || !valid_k(K)) return QVGGT_ERR_SHAPE;
    if (M == 0) return QVGGT_OK;
    if (!Xq || !x_scale || !x_zero || !Wq || !w_scale || !w_codesum || !Y) return QVGGT_ERR_NULL;
    if (!aligned16(Xq) || !aligned16(x_scale) || !aligned16(x_zero) || !aligned16(Wq) || !aligned16(w_scale) ||
        !aligned16(w_codesum) || !aligned16(bias) || !aligned16(Y))
        return QVGGT_ERR_ALIGN;
    return hip_status(qvggt::run_w4a4_gemm_asym(Xq, x_scale, x_zero, Wq, w_scale, w_codesum, bias, M, N, K, Y,
                                                static_cast<hipStream_t>(stream)));
}

size_t qvggt_i8b_bytes(int rows, int K)
{
    if (rows < 0 || !valid_k(K)) return 0;
    return round_up((size_t)rows, 128) * (size_t)K;
}

int qvggt_int8_to_blocks(const int8_t *src, int rows, int K, int8_t *dst, void *stream)
{
    if (rows < 0 || !valid_k(K)) return QVGGT_ERR_SHAPE;
    if (rows == 0) return QVGGT_OK;
    if (!src || !dst) return QVGGT_ERR_NULL;
    if (!aligned16(src) || !aligned16(dst)) return QVGGT_ERR_ALIGN;
    return hip_status(qvggt::run_int8_to_blocks(src, rows, K, reinterpret_cast<uint8_t *>(dst), static_cast<hipStream_t>(stream)));
}

static bool blocks_direct(int x_dtype, int K) { return x_dtype == QVGGT_BF16 && (K == 1024 || K == 2048 || K == 4096); }

int qvggt_rotate_smooth_quant_i8b(const void *X, int x_dtype, int M, int K, const int8_t *signs, const float *inv_smooth, int bits,
                                  int8_t *Xb, float *x_scale, void *stream)
{
    if (!valid_dtype(x_dtype)) return QVGGT_ERR_DTYPE;
    if (M < 0 || !valid_k(K)) return QVGGT_ERR_SHAPE;
    if (!blocks_direct(x_dtype, K)) return x_dtype == QVGGT_BF16 ? QVGGT_ERR_SHAPE : QVGGT_ERR_DTYPE;
    if (!valid_wide_bits(bits)) return QVGGT_ERR_ARG;
    if (M == 0) return QVGGT_OK;
    if (!X || !Xb || !x_scale) return QVGGT_ERR_NULL;
    if (!aligned16(X) || !aligned16(Xb) || !aligned16(x_scale) || !aligned16(inv_smooth) || !aligned16(signs)) return QVGGT_ERR_ALIGN;
    return hip_status(qvggt::run_rotate_quant_i8b_mfma(X, M, K, signs, inv_smooth, reinterpret_cast<uint8_t *>(Xb), x_scale, bits,
                                                       static_cast<hipStream_t>(stream)));
}

int qvggt_i8b_gemm(const int8_t *Xb, const float *x_scale, const int8_t *Wb, const float *w_scale, const void *bias, int M, int N,
                   int K, void *Y, int32_t *acc_debug, void *stream)
{
    if (M < 0 || !valid_n(N) || !valid_k(K)) return QVGGT_ERR_SHAPE;
    if (M == 0) return QVGGT_OK;
    if (!Xb || !x_scale || !Wb || !w_scale || !Y) return QVGGT_ERR_NULL;
    if (!aligned16(Xb) || !aligned16(x_scale) || !aligned16(Wb) || !aligned16(w_scale) || !aligned16(bias) || !aligned16(Y) ||
        !aligned16(acc_debug))
        return QVGGT_ERR_ALIGN;
    return hip_status(qvggt::run_i8b_gemm(Xb, x_scale, Wb, w_scale, bias, M, N, K, Y, acc_debug, static_cast<hipStream_t>(stream)));
}

size_t qvggt_workspace_bytes_i8b(int M, int N, int K)
{
    if (M < 0 || !valid_n(N) || !valid_k(K)) return 0;
    return round_up(qvggt_i8b_bytes(M, K), 256) + round_up((size_t)M * sizeof(float), 256);
}

int qvggt_linear_i8b(const void *X, int x_dtype, int M, int N, int K, const int8_t *signs, const float *inv_smooth, int bits,
                     const int8_t *Wb, const float *w_scale, const void *bias, void *Y, void *workspace, size_t workspace_bytes,
                     void *stream)
{
    if (!valid_dtype(x_dtype)) return QVGGT_ERR_DTYPE;
    if (M < 0 || !valid_n(N) || !valid_k(K)) return QVGGT_ERR_SHAPE;
    if (!blocks_direct(x_dtype, K)) return x_dtype == QVGGT_BF16 ? QVGGT_ERR_SHAPE : QVGGT_ERR_DTYPE;
    if (!valid_wide_bits(bits)) return QVGGT_ERR_ARG;
    if (M == 0) return QVGGT_OK;
    if (!X || !Wb || !w_scale || !Y || !workspace) return QVGGT_ERR_NULL;
    if (!aligned16(X) || !aligned16(Wb) || !aligned16(w_scale) || !aligned16(bias) || !aligned16(Y) || !aligned16(workspace) ||
        !aligned16(inv_smooth) || !aligned16(signs))
        return QVGGT_ERR_ALIGN;
    if (workspace_bytes < qvggt_workspace_bytes_i8b(M, N, K)) return QVGGT_ERR_WORKSPACE;
    uint8_t *Xb = static_cast<uint8_t *>(workspace);
    float *x_scale = reinterpret_cast<float *>(Xb + round_up(qvggt_i8b_bytes(M, K), 256));
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipError_t e = qvggt::run_rotate_quant_i8b_mfma(X, M, K, signs, inv_smooth, Xb, x_scale, bits, s);
    if (e != hipSuccess) return QVGGT_ERR_HIP;
    return hip_status(qvggt::run_i8b_gemm(reinterpret_cast<const int8_t *>(Xb), x_scale, Wb, w_scale, bias, M, N, K, Y, nullptr, s));
}

size_t qvggt_e2m3_bytes(int rows, int K)
{
    if (rows < 0 || !valid_k(K)) return 0;
    return round_up((size_t)rows, 128) * ((size_t)K / 4 * 3);
}

int qvggt_codes_to_e2m3(const uint8_t *packed, int rows, int K, uint8_t *out, uint32_t *n_unrepresentable, void *stream)
{
    if (rows < 0 || !valid_k(K)) return QVGGT_ERR_SHAPE;
    if (!n_unrepresentable) return QVGGT_ERR_NULL;       // also for rows == 0: a caller that cannot see the count must not get QVGGT_OK
    if (reinterpret_cast<uintptr_t>(n_unrepresentable) & 3u) return QVGGT_ERR_ALIGN;
    if (rows == 0) return QVGGT_OK;
    if (!packed || !out) return QVGGT_ERR_NULL;
    if (!aligned16(packed) || !aligned16(out)) return QVGGT_ERR_ALIGN;
    return hip_status(qvggt::run_codes_to_e2m3(packed, rows, K, out, n_unrepresentable, static_cast<hipStream_t>(stream)));
}

static bool e2m3_direct(int x_dtype, int K) { return x_dtype == QVGGT_BF16 && (K == 1024 || K == 2048 || K == 4096); }

int qvggt_rotate_smooth_quant_e2m3(const void *X, int x_dtype, int M, int K, const int8_t *signs, const float *inv_smooth,
                                   uint8_t *Xf, float *x_scale, void *stream)
{
    if (!valid_dtype(x_dtype)) return QVGGT_ERR_DTYPE;
    if (M < 0 || !valid_k(K)) return QVGGT_ERR_SHAPE;
    if (!e2m3_direct(x_dtype, K)) return x_dtype == QVGGT_BF16 ? QVGGT_ERR_SHAPE : QVGGT_ERR_DTYPE;
    if (M == 0) return QVGGT_OK;
    if (!X || !Xf || !x_scale) return QVGGT_ERR_NULL;
    if (!aligned16(X) || !aligned16(Xf) || !aligned16(x_scale) || !aligned16(inv_smooth) || !aligned16(signs))
        return QVGGT_ERR_ALIGN;
    return hip_status(qvggt::run_rotate_quant_e2m3_mfma(X, M, K, signs, inv_smooth, Xf, x_scale, static_cast<hipStream_t>(stream)));
}

size_t qvggt_gelu_table_bytes(void) { return QVGGT_GELU_TABLE_BYTES; }

int qvggt_gelu_table(void *table, void *stream)
{
    if (!table) return QVGGT_ERR_NULL;
    if (!aligned16(table)) return QVGGT_ERR_ALIGN;
    return hip_status(qvggt::run_gelu_table(table, static_cast<hipStream_t>(stream)));
}

static int gelu_rotate_smooth_quant(const void *X, int x_dtype, int M, int K, const int8_t *signs, const float *inv_smooth,
                                   const void *gelu_table, uint8_t *out, float *x_scale, bool e2m3, void *stream)
{
    if (!valid_dtype(x_dtype)) return QVGGT_ERR_DTYPE;
    if (M < 0 || !valid_k(K)) return QVGGT_ERR_SHAPE;
    if (!e2m3_direct(x_dtype, K)) return x_dtype == QVGGT_BF16 ? QVGGT_ERR_SHAPE : QVGGT_ERR_DTYPE;
    if (M == 0) return QVGGT_OK;
    if (!X || !out || !x_scale || !gelu_table) return QVGGT_ERR_NULL;
    if (!aligned16(X) || !aligned16(out) || !aligned16(x_scale) || !aligned16(inv_smooth) || !aligned16(signs) || !aligned16(gelu_table))
        return QVGGT_ERR_ALIGN;
    return hip_status(qvggt::run_gelu_rotate_quant_mfma(X, M, K, signs, inv_smooth, gelu_table, out, x_scale, e2m3,
                                                        static_cast<hipStream_t>(stream)));
}

int qvggt_gelu_rotate_smooth_quant(const void *X, int x_dtype, int M, int K, const int8_t *signs, const float *inv_smooth,
                                   const void *gelu_table, uint8_t *Xq, float *x_scale, void *stream)
{
    return gelu_rotate_smooth_quant(X, x_dtype, M, K, signs, inv_smooth, gelu_table, Xq, x_scale, false, stream);
}

int qvggt_gelu_rotate_smooth_quant_e2m3(const void *X, int x_dtype, int M, int K, const int8_t *signs, const float *inv_smooth,
                                        const void *gelu_table, uint8_t *Xf, float *x_scale, void *stream)
{
    return gelu_rotate_smooth_quant(X, x_dtype, M, K, signs, inv_smooth, gelu_table, Xf, x_scale, true, stream);
}

int qvggt_layernorm_rotate_smooth_quant_e2m3(const void *X, int x_dtype, int M, int K, const float *gamma, const float *beta,
                                             float eps, const int8_t *signs, const float *inv_smooth, uint8_t *Xf, float *x_scale,
                                             void *stream)
{
    if (!valid_dtype(x_dtype)) return QVGGT_ERR_DTYPE;
    if (x_dtype != QVGGT_BF16) return QVGGT_ERR_DTYPE;
    if (M < 0 || K != 1024) return QVGGT_ERR_SHAPE;                  // VGGT-1B's normalised layer inputs
    if (!(eps >= 0.0f) || !std::isfinite(eps)) return QVGGT_ERR_ARG;
    if (M == 0) return QVGGT_OK;
    if (!X || !Xf || !x_scale) return QVGGT_ERR_NULL;
    if (!aligned16(X) || !aligned16(Xf) || !aligned16(x_scale) || !aligned16(inv_smooth) || !aligned16(signs) ||
        !aligned16(gamma) || !aligned16(beta))
        return QVGGT_ERR_ALIGN;
    const qvggt::LnParams ln{gamma, beta, eps, 1};
    return hip_status(qvggt::run_ln_rotate_quant_e2m3_mfma(X, M, signs, inv_smooth, Xf, x_scale, ln, static_cast<hipStream_t>(stream)));
}

// kernel 1 whose codes fill the whole 4-bit range, as E2M3 half-integers: x_step == NULL -> affine codes, else a static step
static int rsq_e2m3_shifted(const void *X, int x_dtype, int M, int K, const int8_t *signs, const float *inv_smooth, const float *x_step,
                            int per_token, bool is_static, uint8_t *Xf, float *x_scale, float *x_zero, void *stream)
{
    if (!valid_dtype(x_dtype)) return QVGGT_ERR_DTYPE;
    if (M < 0 || !valid_k(K)) return QVGGT_ERR_SHAPE;
    if (!e2m3_direct(x_dtype, K)) return x_dtype == QVGGT_BF16 ? QVGGT_ERR_SHAPE : QVGGT_ERR_DTYPE;
    if (is_static && per_token != 0 && per_token != 1) return QVGGT_ERR_ARG;
    if (M == 0) return QVGGT_OK;
    if (!X || !Xf || !x_scale || !x_zero || (is_static && !x_step)) return QVGGT_ERR_NULL;
    if (!aligned16(X) || !aligned16(Xf) || !aligned16(x_scale) || !aligned16(x_zero) || !aligned16(inv_smooth) || !aligned16(signs) ||
        (reinterpret_cast<uintptr_t>(x_step) & 3u) != 0)
        return QVGGT_ERR_ALIGN;
    return hip_status(qvggt::run_rotate_quant_e2m3_shifted_mfma(X, M, K, signs, inv_smooth, Xf, x_scale, x_zero,
                                                                is_static ? x_step : nullptr, per_token,
                                                                static_cast<hipStream_t>(stream)));
}

int qvggt_rotate_smooth_quant_asym_e2m3(const void *X, int x_dtype, int M, int K, const int8_t *signs, const float *inv_smooth,
                                        uint8_t *Xf, float *x_scale, float *x_zero, void *stream)
{
    return rsq_e2m3_shifted(X, x_dtype, M, K, signs, inv_smooth, nullptr, 0, false, Xf, x_scale, x_zero, stream);
}

int qvggt_rotate_smooth_quant_static_e2m3(const void *X, int x_dtype, int M, int K, const int8_t *signs, const float *inv_smooth,
                                          const float *x_step, int per_token, uint8_t *Xf, float *x_scale, float *x_zero,
                                          void *stream)
{
    return rsq_e2m3_shifted(X, x_dtype, M, K, signs, inv_smooth, x_step, per_token, true, Xf, x_scale, x_zero, stream);
}

int qvggt_e2m3_gemm_shifted(const uint8_t *Xf, const float *x_scale, const float *x_zero, const uint8_t *Wf, const float *w_scale,
                            const float *w_codesum, const void *bias, int M, int N, int K, void *Y, void *stream)
{
    if (M < 0 || !valid_n(N) || !valid_k(K)) return QVGGT_ERR_SHAPE;
    if (M == 0) return QVGGT_OK;
    if (!Xf || !x_scale || !x_zero || !Wf || !w_scale || !w_codesum || !Y) return QVGGT_ERR_NULL;
    if (!aligned16(Xf) || !aligned16(x_scale) || !aligned16(x_zero) || !aligned16(Wf) || !aligned16(w_scale) ||
        !aligned16(w_codesum) || !aligned16(bias) || !aligned16(Y))
        return QVGGT_ERR_ALIGN;
    return hip_status(qvggt::run_e2m3_gemm_shifted(Xf, x_scale, x_zero, Wf, w_scale, w_codesum, bias, M, N, K, Y,
                                                   static_cast<hipStream_t>(stream)));
}

size_t qvggt_workspace_bytes_e2m3(int M, int N, int K)
{
    if (M < 0 || !valid_n(N) || !valid_k(K)) return 0;
    return round_up(qvggt_e2m3_bytes(M, K), 256) + round_up((size_t)M * sizeof(float), 256);
}

static int linear_e2m3(const void *gelu_table, const void *X, int x_dtype, int M, int N, int K, const int8_t *signs, const float *inv_smooth,
                      const uint8_t *Wf, const float *w_scale, const void *bias, void *Y, void *workspace,
                      size_t workspace_bytes, void *stream)
{
    if (!valid_dtype(x_dtype)) return QVGGT_ERR_DTYPE;
    if (M < 0 || !valid_n(N) || !valid_k(K)) return QVGGT_ERR_SHAPE;
    if (!e2m3_direct(x_dtype, K)) return x_dtype == QVGGT_BF16 ? QVGGT_ERR_SHAPE : QVGGT_ERR_DTYPE;
    if (M == 0) return QVGGT_OK;
    if (!X || !Wf || !w_scale || !Y || !workspace) return QVGGT_ERR_NULL;
    if (!aligned16(X) || !aligned16(Wf) || !aligned16(w_scale) || !aligned16(bias) || !aligned16(Y) ||
        !aligned16(workspace) || !aligned16(inv_smooth) || !aligned16(signs))
        return QVGGT_ERR_ALIGN;
    if (workspace_bytes < qvggt_workspace_bytes_e2m3(M, N, K)) return QVGGT_ERR_WORKSPACE;
    uint8_t *Xf = static_cast<uint8_t *>(workspace);
    float *x_scale = reinterpret_cast<float *>(Xf + round_up(qvggt_e2m3_bytes(M, K), 256));
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipError_t e = gelu_table ? qvggt::run_gelu_rotate_quant_mfma(X, M, K, signs, inv_smooth, gelu_table, Xf, x_scale, true, s)
                              : qvggt::run_rotate_quant_e2m3_mfma(X, M, K, signs, inv_smooth, Xf, x_scale, s);
    if (e != hipSuccess) return QVGGT_ERR_HIP;
    return hip_status(qvggt::run_e2m3_gemm(Xf, x_scale, Wf, w_scale, bias, M, N, K, Y, nullptr, s));
}

int qvggt_linear_e2m3(const void *X, int x_dtype, int M, int N, int K, const int8_t *signs, const float *inv_smooth,
                      const uint8_t *Wf, const float *w_scale, const void *bias, void *Y, void *workspace,
                      size_t workspace_bytes, void *stream)
{
    return linear_e2m3(nullptr, X, x_dtype, M, N, K, signs, inv_smooth, Wf, w_scale, bias, Y, workspace, workspace_bytes, stream);
}

size_t qvggt_own_workspace_bytes(void) { return QVGGT_OWN_WORKSPACE_BYTES; }

int qvggt_linear_e2m3_own_workspace(const void *X, int x_dtype, int M, int N, int K, const int8_t *signs, const float *inv_smooth,
                                    const uint8_t *Wf, const float *w_scale, const void *bias, void *Y, void *stream)
{
    // shape first: an invalid shape has no workspace size to compare
    if (!valid_dtype(x_dtype)) return QVGGT_ERR_DTYPE;
    if (M < 0 || !valid_n(N) || !valid_k(K)) return QVGGT_ERR_SHAPE;
    if (!e2m3_direct(x_dtype, K)) return x_dtype == QVGGT_BF16 ? QVGGT_ERR_SHAPE : QVGGT_ERR_DTYPE;
    if (qvggt_workspace_bytes_e2m3(M, N, K) > QVGGT_OWN_WORKSPACE_BYTES) return QVGGT_ERR_WORKSPACE;
    if (M == 0) return QVGGT_OK;
    if (!X || !Wf || !w_scale || !Y) return QVGGT_ERR_NULL;     // before the device is touched: argument errors need no GPU
    if (!aligned16(X) || !aligned16(Wf) || !aligned16(w_scale) || !aligned16(bias) || !aligned16(Y) || !aligned16(inv_smooth) ||
        !aligned16(signs))
        return QVGGT_ERR_ALIGN;
    void *ws = nullptr;
    if (qvggt::own_workspace(&ws) != hipSuccess) return QVGGT_ERR_HIP;
    // nothing in the workspace has to start from zero: kernel 1 writes every row below M, and what the GEMM reads of the rows
    // past M (the last 128-row block's padding, left over from an earlier call) only reaches tile rows it never stores
    return linear_e2m3(nullptr, X, x_dtype, M, N, K, signs, inv_smooth, Wf, w_scale, bias, Y, ws, QVGGT_OWN_WORKSPACE_BYTES, stream);
}

int qvggt_gelu_linear_e2m3(const void *X, int x_dtype, int M, int N, int K, const int8_t *signs, const float *inv_smooth,
                           const void *gelu_table, const uint8_t *Wf, const float *w_scale, const void *bias, void *Y, void *workspace,
                           size_t workspace_bytes, void *stream)
{
    if (M > 0 && !gelu_table) return QVGGT_ERR_NULL;
    if (!aligned16(gelu_table)) return QVGGT_ERR_ALIGN;
    return linear_e2m3(gelu_table, X, x_dtype, M, N, K, signs, inv_smooth, Wf, w_scale, bias, Y, workspace, workspace_bytes, stream);
}

int qvggt_e2m3_gemm(const uint8_t *Xf, const float *x_scale, const uint8_t *Wf, const float *w_scale, const void *bias,
                    int M, int N, int K, void *Y, int32_t *acc_debug, void *stream)
{
    if (M < 0 || !valid_n(N) || !valid_k(K)) return QVGGT_ERR_SHAPE;
    if (M == 0) return QVGGT_OK;
    if (!Xf || !x_scale || !Wf || !w_scale || !Y) return QVGGT_ERR_NULL;
    if (!aligned16(Xf) || !aligned16(x_scale) || !aligned16(Wf) || !aligned16(w_scale) || !aligned16(bias) ||
        !aligned16(Y) || !aligned16(acc_debug))
        return QVGGT_ERR_ALIGN;
    return hip_status(qvggt::run_e2m3_gemm(Xf, x_scale, Wf, w_scale, bias, M, N, K, Y, acc_debug,
                                           static_cast<hipStream_t>(stream)));
}

int qvggt_i8_gemm(const int8_t *Xq, const float *x_scale, const int8_t *Wq, const float *w_scale, const void *bias,
                  int M, int N, int K, void *Y, int32_t *acc_debug, void *stream)
{
    if (M < 0 || !valid_n(N) || !valid_k(K)) return QVGGT_ERR_SHAPE;
    if (M == 0) return QVGGT_OK;
    if (!Xq || !x_scale || !Wq || !w_scale || !Y) return QVGGT_ERR_NULL;
    if (!aligned16(Xq) || !aligned16(x_scale) || !aligned16(Wq) || !aligned16(w_scale) || !aligned16(bias) ||
        !aligned16(Y) || !aligned16(acc_debug))
        return QVGGT_ERR_ALIGN;
    return hip_status(qvggt::run_i8_gemm(Xq, x_scale, Wq, w_scale, bias, M, N, K, Y, acc_debug,
                                         static_cast<hipStream_t>(stream)));
}

size_t qvggt_workspace_bytes_i8(int M, int N, int K)
{
    if (M < 0 || !valid_n(N) || !valid_k(K)) return 0;
    return round_up((size_t)M * (size_t)K, 256) + round_up((size_t)M * sizeof(float), 256) + 256;
}

int qvggt_linear_i8(const void *X, int x_dtype, int M, int N, int K, const int8_t *signs, const float *inv_smooth, int bits,
                    const int8_t *Wq, const float *w_scale, const void *bias, void *Y, void *workspace,
                    size_t workspace_bytes, void *stream)
{
    if (!valid_dtype(x_dtype)) return QVGGT_ERR_DTYPE;
    if (M < 0 || !valid_n(N) || !valid_k(K)) return QVGGT_ERR_SHAPE;
    if (!valid_wide_bits(bits)) return QVGGT_ERR_ARG;
    if (M == 0) return QVGGT_OK;
    if (!X || !Wq || !w_scale || !Y || !workspace) return QVGGT_ERR_NULL;
    if (!aligned16(X) || !aligned16(Wq) || !aligned16(w_scale) || !aligned16(bias) || !aligned16(Y) ||
        !aligned16(workspace) || !aligned16(inv_smooth) || !aligned16(signs))
        return QVGGT_ERR_ALIGN;
    if (workspace_bytes < qvggt_workspace_bytes_i8(M, N, K)) return QVGGT_ERR_WORKSPACE;
    uint8_t *Xq = static_cast<uint8_t *>(workspace);
    float *x_scale = reinterpret_cast<float *>(Xq + round_up((size_t)M * (size_t)K, 256));
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipError_t e = qvggt::run_rotate_smooth_quant(X, x_dtype == QVGGT_F32, M, K, signs, inv_smooth, 0, Xq, x_scale, nullptr, 0, qvggt::kInt8Container + bits, s);
    if (e != hipSuccess) return QVGGT_ERR_HIP;
    return hip_status(qvggt::run_i8_gemm(reinterpret_cast<const int8_t *>(Xq), x_scale, Wq, w_scale, bias, M, N, K, Y, nullptr, s));
}

int qvggt_layout_int8(const int8_t *src, int rows, int K, int8_t *dst, int to_library, void *stream)
{
    if (rows < 0 || !valid_k(K)) return QVGGT_ERR_SHAPE;
    if (to_library != 0 && to_library != 1) return QVGGT_ERR_ARG;
    if (rows == 0) return QVGGT_OK;
    if (!src || !dst) return QVGGT_ERR_NULL;
    if (!aligned16(src) || !aligned16(dst)) return QVGGT_ERR_ALIGN;
    return hip_status(qvggt::run_layout_int8(src, rows, K, dst, to_library, static_cast<hipStream_t>(stream)));
}

size_t qvggt_workspace_bytes(int M, int N, int K)
{
    if (M < 0 || !valid_n(N) || !valid_k(K)) return 0;
    return round_up((size_t)M * (size_t)(K / 2), 256) + round_up((size_t)M * sizeof(float), 256) + 256;
}

int qvggt_linear(const void *X, int x_dtype, int M, int N, int K, const int8_t *signs, const float *inv_smooth,
                 const uint8_t *Wq, const float *w_scale, const void *bias, void *Y, void *workspace,
                 size_t workspace_bytes, void *stream)
{
    if (!valid_dtype(x_dtype)) return QVGGT_ERR_DTYPE;
    if (M < 0 || !valid_n(N) || !valid_k(K)) return QVGGT_ERR_SHAPE;
    if (M == 0) return QVGGT_OK;
    if (!X || !Wq || !w_scale || !Y || !workspace) return QVGGT_ERR_NULL;
    if (!aligned16(X) || !aligned16(Wq) || !aligned16(w_scale) || !aligned16(bias) || !aligned16(Y) ||
        !aligned16(workspace) || !aligned16(inv_smooth) || !aligned16(signs))
        return QVGGT_ERR_ALIGN;
    if (workspace_bytes < qvggt_workspace_bytes(M, N, K)) return QVGGT_ERR_WORKSPACE;
    uint8_t *Xq = static_cast<uint8_t *>(workspace);
    float *x_scale = reinterpret_cast<float *>(Xq + round_up((size_t)M * (size_t)(K / 2), 256));
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipError_t e = qvggt::run_rotate_smooth_quant(X, x_dtype == QVGGT_F32, M, K, signs, inv_smooth, 0, Xq, x_scale, nullptr, 0, 4, s);
    if (e != hipSuccess) return QVGGT_ERR_HIP;
    return hip_status(qvggt::run_w4a4_gemm(Xq, x_scale, Wq, w_scale, bias, M, N, K, Y, nullptr, s));
}

int qvggt_pack_int4(const int8_t *codes, int rows, int K, uint8_t *packed, void *stream)
{
    if (rows < 0 || !valid_k(K)) return QVGGT_ERR_SHAPE;
    if (rows == 0) return QVGGT_OK;
    if (!codes || !packed) return QVGGT_ERR_NULL;
    if (!aligned16(codes) || !aligned16(packed)) return QVGGT_ERR_ALIGN;
    return hip_status(qvggt::run_pack_int4(codes, rows, K, packed, static_cast<hipStream_t>(stream)));
}

int qvggt_unpack_int4(const uint8_t *packed, int rows, int K, int8_t *codes, void *stream)
{
    if (rows < 0 || !valid_k(K)) return QVGGT_ERR_SHAPE;
    if (rows == 0) return QVGGT_OK;
    if (!codes || !packed) return QVGGT_ERR_NULL;
    if (!aligned16(codes) || !aligned16(packed)) return QVGGT_ERR_ALIGN;
    return hip_status(qvggt::run_unpack_int4(packed, rows, K, codes, static_cast<hipStream_t>(stream)));
}

// ---- calibration: the learnable smoothing factor and steps (appendix "Experiment Settings")
static bool aligned4(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 3u) == 0; }
static bool valid_calib_shape(int T, int N, int K) { return T >= 1 && T <= (1 << 22) && N >= 1 && N <= (1 << 20) && K >= 4 && K <= qvggt::kMaxK && K % 4 == 0; }

int qvggt_rotate_rows(const void *X, int x_dtype, int M, int K, const int8_t *signs, float *R, void *stream)
{
    if (!valid_dtype(x_dtype)) return QVGGT_ERR_DTYPE;
    if (M < 0 || K < qvggt::kMinK || K > qvggt::kMaxK || (K & (K - 1)) != 0) return QVGGT_ERR_SHAPE;
    if (M == 0) return QVGGT_OK;
    if (!X || !R) return QVGGT_ERR_NULL;
    if (!aligned16(X) || !aligned16(R) || !aligned16(signs)) return QVGGT_ERR_ALIGN;
    return hip_status(qvggt::run_rotate_only(X, x_dtype == QVGGT_F32, M, K, signs, R, static_cast<hipStream_t>(stream)));
}

size_t qvggt_calib_workspace_bytes(int T, int N, int K)
{
    if (!valid_calib_shape(T, N, K)) return 0;
    return qvggt::calib_workspace_bytes(T, N, K) + 256;
}

int qvggt_calib_loss_grad(const float *R, const float *V, const float *y_ref, const void *bias, const float *c_hat, const float *w_step,
                          const float *x_step, int T, int N, int K, int bits, float *loss, float *grad_c, float *grad_w_step,
                          float *grad_x_step, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!valid_calib_shape(T, N, K)) return QVGGT_ERR_SHAPE;
    if (!valid_wide_bits(bits)) return QVGGT_ERR_ARG;
    if (!R || !V || !y_ref || !c_hat || !w_step || !loss || !grad_c || !grad_w_step || !workspace) return QVGGT_ERR_NULL;
    if ((x_step != nullptr) != (grad_x_step != nullptr)) return QVGGT_ERR_NULL;      // a static step and its derivative come together
    if (!aligned16(R) || !aligned16(V) || !aligned16(y_ref) || !aligned16(workspace) || !aligned4(c_hat) || !aligned4(w_step) ||
        !aligned4(x_step) || !aligned4(loss) || !aligned4(grad_c) || !aligned4(grad_w_step) || !aligned4(grad_x_step) ||
        (reinterpret_cast<uintptr_t>(bias) & 1u))
        return QVGGT_ERR_ALIGN;
    if (workspace_bytes < qvggt_calib_workspace_bytes(T, N, K)) return QVGGT_ERR_WORKSPACE;
    return hip_status(qvggt::run_calib_loss_grad(R, V, y_ref, bias, c_hat, w_step, x_step, T, N, K, bits, loss, grad_c, grad_w_step,
                                                 grad_x_step, workspace, static_cast<hipStream_t>(stream)));
}

int qvggt_calib_descent_step(float *theta, const float *grad, int n, float lr, float floor, void *stream)
{
    if (n < 0) return QVGGT_ERR_SHAPE;
    if (!std::isfinite(lr) || !(floor > 0.0f) || !std::isfinite(floor)) return QVGGT_ERR_ARG;
    if (n == 0) return QVGGT_OK;
    if (!theta || !grad) return QVGGT_ERR_NULL;
    if (!aligned4(theta) || !aligned4(grad)) return QVGGT_ERR_ALIGN;
    return hip_status(qvggt::run_descent_step(theta, grad, n, lr, floor, static_cast<hipStream_t>(stream)));
}

// ---- calibration-set arithmetic (Sec. 3.3)
namespace {
// a row of `count` elements must be a whole number of 16-byte vectors, and the totals must stay addressable
bool valid_row(long long count, int dtype) { return count > 0 && count <= (1LL << 40) && (count * (dtype == QVGGT_F32 ? 4 : 2)) % 16 == 0; }
}  // namespace

size_t qvggt_nfds_workspace_bytes(int rows, long long count, int dtype)
{
    if (rows < 0 || rows > (1 << 22) || !valid_dtype(dtype) || !valid_row(count, dtype)) return 0;
    return round_up(qvggt::nfds_workspace_bytes(rows, count, dtype == QVGGT_F32), 256) + 256;
}

int qvggt_nfds_moments(const void *A, int dtype, int rows, long long count, float *mean, float *var, void *workspace,
                       size_t workspace_bytes, void *stream)
{
    if (!valid_dtype(dtype)) return QVGGT_ERR_DTYPE;
    if (rows < 0 || rows > (1 << 22) || !valid_row(count, dtype)) return QVGGT_ERR_SHAPE;
    if (rows == 0) return QVGGT_OK;
    if (!A || !mean || !var || !workspace) return QVGGT_ERR_NULL;
    if (!aligned16(A) || !aligned16(workspace) || (reinterpret_cast<uintptr_t>(mean) & 3u) || (reinterpret_cast<uintptr_t>(var) & 3u))
        return QVGGT_ERR_ALIGN;
    if (workspace_bytes < qvggt_nfds_workspace_bytes(rows, count, dtype)) return QVGGT_ERR_WORKSPACE;
    return hip_status(qvggt::run_nfds_moments(A, dtype == QVGGT_F32, rows, count, mean, var, static_cast<double *>(workspace),
                                              static_cast<hipStream_t>(stream)));
}

int qvggt_nfds_frame_correlation(const void *A, int dtype, int samples, int frames, long long frame_elems, float *corr,
                                 void *workspace, size_t workspace_bytes, void *stream)
{
    if (!valid_dtype(dtype)) return QVGGT_ERR_DTYPE;
    if (samples < 0 || frames < 2 || frames > 4096 || (long long)samples * frames > (1 << 22) || !valid_row(frame_elems, dtype))
        return QVGGT_ERR_SHAPE;
    if (samples == 0) return QVGGT_OK;
    if (!A || !corr || !workspace) return QVGGT_ERR_NULL;
    if (!aligned16(A) || !aligned16(workspace) || (reinterpret_cast<uintptr_t>(corr) & 3u)) return QVGGT_ERR_ALIGN;
    if (workspace_bytes < qvggt_nfds_workspace_bytes(samples * frames, frame_elems, dtype)) return QVGGT_ERR_WORKSPACE;
    return hip_status(qvggt::run_nfds_frame_correlation(A, dtype == QVGGT_F32, samples, frames, frame_elems, corr,
                                                        static_cast<double *>(workspace), static_cast<hipStream_t>(stream)));
}

int qvggt_nfds_scores(const float *m, const float *s, int D, int L, double eps, float *score, void *stream)
{
    if (D < 1 || D > 65536 || L < 1 || L > 2048) return QVGGT_ERR_SHAPE;
    if (!(eps >= 0.0) || !std::isfinite(eps)) return QVGGT_ERR_ARG;
    if (!m || !s || !score) return QVGGT_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(m) & 3u) || (reinterpret_cast<uintptr_t>(s) & 3u) || (reinterpret_cast<uintptr_t>(score) & 3u))
        return QVGGT_ERR_ALIGN;
    return hip_status(qvggt::run_nfds_scores(m, s, D, L, eps, score, static_cast<hipStream_t>(stream)));
}

int qvggt_nfds_keep_lowest(const float *score, int D, double p, uint8_t *keep, void *stream)
{
    if (D < 1 || D > 65536) return QVGGT_ERR_SHAPE;
    if (!(p >= 0.0 && p <= 1.0)) return QVGGT_ERR_ARG;
    if (!score || !keep) return QVGGT_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(score) & 3u) return QVGGT_ERR_ALIGN;
    return hip_status(qvggt::run_nfds_keep_lowest(score, D, (int)std::floor(p * (double)D), keep, static_cast<hipStream_t>(stream)));
}

int qvggt_nfds_kmeans_step(const float *c, int n, int dim, int K, const float *centres_in, float *centres_out,
                           int32_t *labels, void *stream)
{
    if (n < 1 || n > 65536 || dim < 1 || dim > 4096 || K < 1 || K > 256) return QVGGT_ERR_SHAPE;
    if (!c || !centres_in || !centres_out || !labels) return QVGGT_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(c) & 3u) || (reinterpret_cast<uintptr_t>(centres_in) & 3u) ||
        (reinterpret_cast<uintptr_t>(centres_out) & 3u) || (reinterpret_cast<uintptr_t>(labels) & 3u))
        return QVGGT_ERR_ALIGN;
    if (centres_in == centres_out) return QVGGT_ERR_ARG;
    return hip_status(qvggt::run_nfds_kmeans_step(c, n, dim, K, centres_in, centres_out, labels, static_cast<hipStream_t>(stream)));
}

}  // extern "C"
