// Calibration side: the reconstruction loss of one quantized linear layer over a calibration batch and its derivatives with
// respect to the smoothing factor and the quantization steps (paper, appendix "Experiment Settings": c_hat and Delta are
// learnable during calibration, learning rates 5e-3 and 5e-2; Sec. 3.1.2, Eq. "loss_ori_overall": squared distance between the
// full-precision and the quantized function over the calibration set).  The paper gives no update rule; the reading is:
//
//   z = (X H) / c,  x_hat = step_x * clamp(round(z / step_x)),      v = (W H) * c,  w_hat[o] = step_w[o] * clamp(round(v[o] / step_w[o])),
//   y_q = x_hat . w_hat^T + b,      L = (1 / T) sum_t || y_q[t] - y_ref[t] ||^2,
//   rounding passed straight through, a clamped value (one whose ROUNDED code leaves the range) passing nothing,
//   d(quantized) / d(step) = round(u) - u inside the range and the clamp bound outside, c_hat moving through both operands (d v / d c = V, d z / d c = -z / c), a dynamic per-token
//   activation step (max |z| / qmax) recomputed from the row and held constant in the derivative, a static one (one value) learnable.
//
// Offline work on batches of a few thousand tokens: plain fp32 kernels (row-wise fake quantization, a tiled fp32 GEMM used
// three ways, fixed-order reductions so that results do not vary from run to run), none of it on the inference path.
#include "qvggt_common.h"
#include "rotate_rows.h"

namespace qvggt {

namespace {

// ---- X -> X H (orthonormal Hadamard, input-side signs), fp32, natural order: what the loss takes as R and V
template <int K, bool F32>
__global__ __launch_bounds__(256) void rotate_only_kernel(const void *__restrict__ X, int rows, const int8_t *__restrict__ signs,
                                                          float *__restrict__ out)
{
    constexpr int V = RowMap<K>::V, C = RowMap<K>::C, R = RowMap<K>::R;
    const int lane = threadIdx.x & 63;
    const int wave = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6), nwaves = gridDim.x * (blockDim.x >> 6);
    const float rs = 1.0f / sqrtf((float)K);
    for (int row = wave; row < rows; row += nwaves) {
        float x[R];
        load_row<K, F32>(X, (size_t)row, lane, x);
        if (signs != nullptr) {
#pragma unroll
            for (int c = 0; c < C; ++c)
#pragma unroll
                for (int i = 0; i < V; ++i)
                    if (signs[c * 64 * V + lane * V + i] < 0) x[c * V + i] = -x[c * V + i];
        }
        fwht_row<K>(x, lane);
#pragma unroll
        for (int c = 0; c < C; ++c)
#pragma unroll
            for (int i = 0; i < V; ++i) out[(size_t)row * K + c * 64 * V + lane * V + i] = x[c * V + i] * rs;
    }
}

// block-wide sum / max of one float per thread (256 threads), result in every thread; fixed order
__device__ inline float block_sum(float v, float *red)
{
    v = sum_over_64_lanes(v);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    const float s = (red[0] + red[1]) + (red[2] + red[3]);
    __syncthreads();
    return s;
}
__device__ inline float block_max(float v, float *red)
{
    v = max_over_64_lanes(v);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    const float s = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    __syncthreads();
    return s;
}

struct QRange {
    float lo, hi;
};

// the scaled value u = a / step (a = A / c or A * c), its code, whether it was clamped: shared by the forward and the reductions
__device__ inline float operand_value(float a, float c, bool divide) { return divide ? a / c : a * c; }

// ---- row-wise fake quantization: hat[r, j] = step_r * clamp(round(a / step_r)); one block per row.
// step_mode 0: dynamic, step_r = max_j |a| / hi, written to steps_out[r]; 1: steps[r]; 2: steps[0] for every row
__global__ __launch_bounds__(256) void fake_quant_rows_kernel(const float *__restrict__ A, const float *__restrict__ c, bool divide,
                                                              const float *__restrict__ steps, int step_mode, QRange q, int K,
                                                              float *__restrict__ hat, float *__restrict__ steps_out)
{
    __shared__ float red[4];
    const size_t row = blockIdx.x;
    const float *a = A + row * K;
    float step;
    if (step_mode == 0) {
        float m = 0.0f;
        for (int j = threadIdx.x; j < K; j += 256) m = fmaxf(m, fabsf(operand_value(a[j], c[j], divide)));
        m = block_max(m, red);
        step = m >= q.hi * kMinStep ? m / q.hi : 0.0f;
        if (threadIdx.x == 0) steps_out[row] = step;
    } else {
        step = steps[step_mode == 1 ? row : 0];
    }
    const bool live = step >= kMinStep;
    for (int j = threadIdx.x; j < K; j += 256) {
        const float u = operand_value(a[j], c[j], divide) / (live ? step : 1.0f);
        const float code = fminf(fmaxf(rintf(u), q.lo), q.hi);
        hat[row * K + j] = live ? step * code : 0.0f;
    }
}

// ---- C[i, j] = sum_k A(i, k) B(k, j) in fp32, operands addressed through strides (so the same kernel serves X_hat W_hat^T,
// E W_hat and E^T X_hat).  64 x 64 tile per block, 16-deep steps through LDS, 4 x 4 outputs per thread.
// EPI 0: C = sum.  EPI 1: C = sum + bias[j] - ref[i, j] (the residual E), and the block's sum of squares to partial[block].
template <int EPI>
__global__ __launch_bounds__(256) void sgemm_kernel(const float *__restrict__ A, long long sa_i, long long sa_k,
                                                    const float *__restrict__ B, long long sb_k, long long sb_j, int M, int N, int Kd,
                                                    float *__restrict__ Cm, const uint16_t *__restrict__ bias,
                                                    const float *__restrict__ ref, float *__restrict__ partial)
{
    __shared__ float As[16][64 + 4], Bs[16][64 + 4];
    __shared__ float red[4];
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    const int i0 = blockIdx.y * 64, j0 = blockIdx.x * 64;
    float acc[4][4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) acc[a][b] = 0.0f;
    for (int k0 = 0; k0 < Kd; k0 += 16) {
        // 64 x 16 elements of each operand: four per thread
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int idx = e * 256 + threadIdx.x;
            const int ii = idx & 63, kk = idx >> 6;            // consecutive threads walk the 64 rows / columns of the tile
            const int gi = i0 + ii, gj = j0 + ii, gk = k0 + kk;
            As[kk][ii] = (gi < M && gk < Kd) ? A[gi * sa_i + gk * sa_k] : 0.0f;
            Bs[kk][ii] = (gj < N && gk < Kd) ? B[gk * sb_k + gj * sb_j] : 0.0f;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < 16; ++kk) {
            const float4 av = *reinterpret_cast<const float4 *>(&As[kk][ty * 4]);
            const float4 bv = *reinterpret_cast<const float4 *>(&Bs[kk][tx * 4]);
            const float a4[4] = {av.x, av.y, av.z, av.w}, b4[4] = {bv.x, bv.y, bv.z, bv.w};
#pragma unroll
            for (int a = 0; a < 4; ++a)
#pragma unroll
                for (int b = 0; b < 4; ++b) acc[a][b] = fmaf(a4[a], b4[b], acc[a][b]);
        }
        __syncthreads();
    }
    float sq = 0.0f;
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const int i = i0 + ty * 4 + a, j = j0 + tx * 4 + b;
            if (i < M && j < N) {
                float v = acc[a][b];
                if constexpr (EPI == 1) {
                    if (bias != nullptr) v += bf16_bits_to_float(bias[j]);
                    v -= ref[(size_t)i * N + j];
                    sq = fmaf(v, v, sq);
                }
                Cm[(size_t)i * N + j] = v;
            }
        }
    if constexpr (EPI == 1) {
        sq = block_sum(sq, red);
        if (threadIdx.x == 0) partial[blockIdx.y * gridDim.x + blockIdx.x] = sq;
    }
}

// ---- fixed-order sum of n partials, times `scale`, to out[0] (one block)
__global__ __launch_bounds__(256) void sum_partials_kernel(const float *__restrict__ partial, int n, float scale, float *__restrict__ out)
{
    __shared__ float red[4];
    float s = 0.0f;
    for (int i = threadIdx.x; i < n; i += 256) s += partial[i];
    s = block_sum(s, red);
    if (threadIdx.x == 0) out[0] = s * scale;
}

// ---- per row r: scale * sum_j G[r, j] * d(hat) / d(step_r), with u = a / step_r recomputed (one block per row).
// For the weights this is dL / d step_w[o] itself; for a static activation step the rows are summed afterwards.
__global__ __launch_bounds__(256) void grad_step_rows_kernel(const float *__restrict__ G, const float *__restrict__ A,
                                                             const float *__restrict__ c, bool divide, const float *__restrict__ steps,
                                                             int step_mode, QRange q, int K, float scale, float *__restrict__ out)
{
    __shared__ float red[4];
    const size_t row = blockIdx.x;
    const float step = steps[step_mode == 1 ? row : 0];
    const bool live = step >= kMinStep;
    float s = 0.0f;
    if (live) {
        for (int j = threadIdx.x; j < K; j += 256) {
            const float u = operand_value(A[row * K + j], c[j], divide) / step;
            const float r = rintf(u), code = fminf(fmaxf(r, q.lo), q.hi);
            const float d = (r >= q.lo && r <= q.hi) ? code - u : code;          // clamped: the rounded code left the range
            s = fmaf(G[row * K + j], d, s);
        }
    }
    s = block_sum(s, red);
    if (threadIdx.x == 0) out[row] = s * scale;
}

// ---- dL / d c_hat[j] = scale * ( sum_o GW[o, j] [inside] V[o, j]  +  sum_t GX[t, j] [inside] (-z[t, j] / c_j) ).
// A block owns 64 columns; its 4 row groups walk the rows in a fixed order and are folded in a fixed order.
__global__ __launch_bounds__(256) void grad_c_kernel(const float *__restrict__ GW, const float *__restrict__ V, const float *__restrict__ w_step,
                                                     int N, const float *__restrict__ GX, const float *__restrict__ R,
                                                     const float *__restrict__ x_steps, int x_step_mode, int T, const float *__restrict__ c,
                                                     QRange q, int K, float scale, float *__restrict__ grad_c)
{
    __shared__ float red[4][64];
    const int col = blockIdx.x * 64 + (threadIdx.x & 63), grp = threadIdx.x >> 6;
    float s = 0.0f;
    if (col < K) {
        const float cj = c[col];
        for (int o = grp; o < N; o += 4) {
            const float step = w_step[o];
            if (step < kMinStep) continue;
            const float v = V[(size_t)o * K + col], r = rintf(v * cj / step);
            if (r >= q.lo && r <= q.hi) s = fmaf(GW[(size_t)o * K + col], v, s);
        }
        for (int t = grp; t < T; t += 4) {
            const float step = x_steps[x_step_mode == 2 ? 0 : t];
            if (step < kMinStep) continue;
            const float z = R[(size_t)t * K + col] / cj, r = rintf(z / step);
            if (r >= q.lo && r <= q.hi) s = fmaf(GX[(size_t)t * K + col], -z / cj, s);
        }
    }
    red[grp][threadIdx.x & 63] = s;
    __syncthreads();
    if (grp == 0 && col < K) grad_c[col] = ((red[0][threadIdx.x] + red[1][threadIdx.x]) + (red[2][threadIdx.x] + red[3][threadIdx.x])) * scale;
}

__global__ void descent_step_kernel(float *__restrict__ theta, const float *__restrict__ grad, int n, float lr, float floor_)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) theta[i] = fmaxf(theta[i] - lr * grad[i], floor_);
}

size_t align256(size_t v) { return (v + 255) / 256 * 256; }

}  // namespace

hipError_t run_rotate_only(const void *X, bool f32, int rows, int K, const int8_t *signs, float *out, hipStream_t stream)
{
    if (rows <= 0) return hipSuccess;
    const int blocks = std::min((rows + 3) / 4, 2048);
#define QVGGT_ROT(KK)                                                                                          \
    case KK:                                                                                                   \
        if (f32) rotate_only_kernel<KK, true><<<blocks, 256, 0, stream>>>(X, rows, signs, out);               \
        else rotate_only_kernel<KK, false><<<blocks, 256, 0, stream>>>(X, rows, signs, out);                  \
        break;
    switch (K) {
        QVGGT_ROT(128) QVGGT_ROT(256) QVGGT_ROT(512) QVGGT_ROT(1024) QVGGT_ROT(2048) QVGGT_ROT(4096) QVGGT_ROT(8192)
        default: return hipErrorInvalidValue;
    }
#undef QVGGT_ROT
    return hipGetLastError();
}

// workspace: x_hat [T, K], w_hat [N, K], E [T, N], GX [T, K], GW [N, K], dynamic steps [T], partial sums
size_t calib_workspace_bytes(int T, int N, int K)
{
    const size_t tk = align256((size_t)T * K * 4), nk = align256((size_t)N * K * 4), tn = align256((size_t)T * N * 4);
    const size_t tiles = (size_t)((T + 63) / 64) * ((N + 63) / 64);
    return 2 * tk + 2 * nk + tn + align256((size_t)T * 4) + align256(std::max<size_t>(tiles, (size_t)T) * 4);
}

hipError_t run_calib_loss_grad(const float *R, const float *V, const float *y_ref, const void *bias, const float *c_hat,
                               const float *w_step, const float *x_step, int T, int N, int K, int bits, float *loss, float *grad_c,
                               float *grad_w_step, float *grad_x_step, void *workspace, hipStream_t stream)
{
    const size_t tk = align256((size_t)T * K * 4), nk = align256((size_t)N * K * 4), tn = align256((size_t)T * N * 4);
    uint8_t *p = static_cast<uint8_t *>(workspace);
    float *x_hat = reinterpret_cast<float *>(p); p += tk;
    float *w_hat = reinterpret_cast<float *>(p); p += nk;
    float *E = reinterpret_cast<float *>(p); p += tn;
    float *GX = reinterpret_cast<float *>(p); p += tk;
    float *GW = reinterpret_cast<float *>(p); p += nk;
    float *dyn_steps = reinterpret_cast<float *>(p); p += align256((size_t)T * 4);
    float *partial = reinterpret_cast<float *>(p);
    const QRange q{-(float)(1 << (bits - 1)), (float)((1 << (bits - 1)) - 1)};
    const int x_mode = x_step ? 2 : 0;
    const float *x_steps = x_step ? x_step : dyn_steps;
    const float scale = 2.0f / (float)T;                 // dL / dy_q = (2 / T) E: folded into the last reductions

    fake_quant_rows_kernel<<<T, 256, 0, stream>>>(R, c_hat, true, x_step, x_mode, q, K, x_hat, dyn_steps);
    fake_quant_rows_kernel<<<N, 256, 0, stream>>>(V, c_hat, false, w_step, 1, q, K, w_hat, nullptr);
    // E = x_hat . w_hat^T + b - y_ref, and the loss
    const dim3 g_tn((N + 63) / 64, (T + 63) / 64);
    sgemm_kernel<1><<<g_tn, 256, 0, stream>>>(x_hat, K, 1, w_hat, 1, K, T, N, K, E, reinterpret_cast<const uint16_t *>(bias), y_ref, partial);
    sum_partials_kernel<<<1, 256, 0, stream>>>(partial, (int)(g_tn.x * g_tn.y), 1.0f / (float)T, loss);
    // GX = E . w_hat  [T, K];  GW = E^T . x_hat  [N, K]
    const dim3 g_tk((K + 63) / 64, (T + 63) / 64), g_nk((K + 63) / 64, (N + 63) / 64);
    sgemm_kernel<0><<<g_tk, 256, 0, stream>>>(E, N, 1, w_hat, K, 1, T, K, N, GX, nullptr, nullptr, nullptr);
    sgemm_kernel<0><<<g_nk, 256, 0, stream>>>(E, 1, N, x_hat, K, 1, N, K, T, GW, nullptr, nullptr, nullptr);
    grad_step_rows_kernel<<<N, 256, 0, stream>>>(GW, V, c_hat, false, w_step, 1, q, K, scale, grad_w_step);
    if (x_step != nullptr && grad_x_step != nullptr) {
        grad_step_rows_kernel<<<T, 256, 0, stream>>>(GX, R, c_hat, true, x_step, 2, q, K, 1.0f, partial);
        sum_partials_kernel<<<1, 256, 0, stream>>>(partial, T, scale, grad_x_step);
    }
    grad_c_kernel<<<(K + 63) / 64, 256, 0, stream>>>(GW, V, w_step, N, GX, R, x_steps, x_mode, T, c_hat, q, K, scale, grad_c);
    return hipGetLastError();
}

hipError_t run_descent_step(float *theta, const float *grad, int n, float lr, float floor_, hipStream_t stream)
{
    if (n <= 0) return hipSuccess;
    descent_step_kernel<<<(n + 255) / 256, 256, 0, stream>>>(theta, grad, n, lr, floor_);
    return hipGetLastError();
}

}  // namespace qvggt
