// Arithmetic of the calibration-set construction (paper Sec. 3.3, Noise-Filtered Diverse Sampling): the two reductions
// that read whole activation tensors (per-layer mean / variance of a sample, frame-to-first-frame cosine of a feature
// map) and the small per-pool steps built on their results (noise score, percentile filter, one K-Means iteration).
//
// The reductions are bound by HBM: every element is read once with 16-byte loads, converted to double and summed in
// double (sum, sum of squares / dot product), so that the variance formula E[x^2] - E[x]^2 has no cancellation problem
// and the result does not depend on the size of the tensor.  A row is split over several blocks; each block leaves a
// pair of partial sums in the workspace and a second, tiny kernel adds them in a fixed order (deterministic results).
// The per-pool steps handle a few hundred samples: one block each, double arithmetic, written for clarity.
#include "qvggt_common.h"

#include <algorithm>

namespace qvggt {

namespace nfds {
constexpr int THREADS = 256;
constexpr int MAX_BLOCKS_PER_ROW = 1024;
constexpr int TARGET_BLOCKS = 2048;          // blocks in flight on the 256 compute units
constexpr int MIN_VEC_PER_BLOCK = 4 * THREADS;  // 16-byte vectors a block handles at least: keeps the partials few for small rows

__host__ inline int blocks_per_row(int rows, long long count, int elt_bytes)
{
    const long long vecs = count * elt_bytes / 16;
    long long want = std::max(1LL, (long long)TARGET_BLOCKS / std::max(rows, 1));
    const long long cap = std::max(1LL, vecs / MIN_VEC_PER_BLOCK);
    want = std::min(std::min(want, cap), (long long)MAX_BLOCKS_PER_ROW);
    return (int)want;
}

// the 8 bf16 or 4 f32 values of one 16-byte vector, as doubles
template <bool F32>
__device__ inline int unpack(const uint4 &v, double (&x)[8])
{
    if constexpr (F32) {
        x[0] = (double)__uint_as_float(v.x); x[1] = (double)__uint_as_float(v.y);
        x[2] = (double)__uint_as_float(v.z); x[3] = (double)__uint_as_float(v.w);
        return 4;
    } else {
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            x[2 * q] = (double)__uint_as_float(w[q] << 16);
            x[2 * q + 1] = (double)__uint_as_float(w[q] & 0xFFFF0000u);
        }
        return 8;
    }
}

__device__ inline double block_sum(double v, double *lds)
{
#pragma unroll
    for (int m = 1; m < kWave; m <<= 1) v += __shfl_xor(v, m);
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    __syncthreads();
    if (lane == 0) lds[wave] = v;
    __syncthreads();
    double t = 0.0;
    for (int w = 0; w < THREADS / kWave; ++w) t += lds[w];
    return t;
}
}  // namespace nfds

// partial[(row * bpr + b) * 2 + {0, 1}] = sum of a * b, sum of b * b over block b's share of row `row`,
// where b is the row itself and a is either the row again (moments: first sum is replaced by the plain sum)
// or the first row of its group of `group` rows (frame correlation).
template <bool F32, bool CORR>
__global__ __launch_bounds__(nfds::THREADS) void nfds_partial_kernel(const void *__restrict__ A, long long count, int bpr,
                                                                    int group, double *__restrict__ partial)
{
    __shared__ double lds[nfds::THREADS / kWave];
    const int row = blockIdx.x / bpr, b = blockIdx.x % bpr;
    const long long vecs = count * (F32 ? 4 : 2) / 16;
    const long long v0 = vecs * b / bpr, v1 = vecs * (b + 1) / bpr;
    const uint4 *x = reinterpret_cast<const uint4 *>(reinterpret_cast<const uint8_t *>(A) + (size_t)row * count * (F32 ? 4 : 2));
    const uint4 *ref = reinterpret_cast<const uint4 *>(reinterpret_cast<const uint8_t *>(A) +
                                                       (size_t)(row - row % group) * count * (F32 ? 4 : 2));
    double s0 = 0.0, s1 = 0.0;
    for (long long v = v0 + threadIdx.x; v < v1; v += nfds::THREADS) {
        double xv[8], rv[8];
        const int n = nfds::unpack<F32>(x[v], xv);
        if constexpr (CORR) {
            nfds::unpack<F32>(ref[v], rv);
#pragma unroll
            for (int i = 0; i < 8; ++i)
                if (i < n) { s0 += rv[i] * xv[i]; s1 += xv[i] * xv[i]; }
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i)
                if (i < n) { s0 += xv[i]; s1 += xv[i] * xv[i]; }
        }
    }
    s0 = nfds::block_sum(s0, lds);
    s1 = nfds::block_sum(s1, lds);
    if (threadIdx.x == 0) {
        partial[((size_t)row * bpr + b) * 2] = s0;
        partial[((size_t)row * bpr + b) * 2 + 1] = s1;
    }
}

// mean = S1 / n, var = S2 / n - mean^2 (population variance), one thread per row
__global__ void nfds_moments_final_kernel(const double *__restrict__ partial, int rows, int bpr, long long count,
                                          float *__restrict__ mean, float *__restrict__ var)
{
    const int row = blockIdx.x * blockDim.x + threadIdx.x;
    if (row >= rows) return;
    double s1 = 0.0, s2 = 0.0;
    for (int b = 0; b < bpr; ++b) { s1 += partial[((size_t)row * bpr + b) * 2]; s2 += partial[((size_t)row * bpr + b) * 2 + 1]; }
    const double m = s1 / (double)count;
    mean[row] = (float)m;
    var[row] = (float)fmax(s2 / (double)count - m * m, 0.0);
}

// c[sample, t - 1] = <a_0, a_t> / (|a_0| |a_t|), one thread per (sample, t >= 1)
__global__ void nfds_corr_final_kernel(const double *__restrict__ partial, int samples, int f, int bpr, float *__restrict__ c)
{
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= samples * (f - 1)) return;
    const int i = idx / (f - 1), t = idx % (f - 1) + 1;
    double dot = 0.0, nt = 0.0, n0 = 0.0;
    for (int b = 0; b < bpr; ++b) {
        dot += partial[((size_t)(i * f + t) * bpr + b) * 2];
        nt += partial[((size_t)(i * f + t) * bpr + b) * 2 + 1];
        n0 += partial[((size_t)(i * f) * bpr + b) * 2 + 1];
    }
    c[idx] = (float)(dot / (sqrt(n0) * sqrt(nt)));
}

// noise score of every sample of the pool from its per-layer moments: one block, layers then samples dealt to threads
__global__ __launch_bounds__(nfds::THREADS) void nfds_scores_kernel(const float *__restrict__ m, const float *__restrict__ s, int D,
                                                                   int L, double eps, float *__restrict__ score)
{
    extern __shared__ double stat[];     // mu, sigma, nu, tau: 4 * L
    for (int j = threadIdx.x; j < L; j += nfds::THREADS) {
        double mu = 0.0, nu = 0.0;
        for (int i = 0; i < D; ++i) { mu += (double)m[(size_t)i * L + j]; nu += (double)s[(size_t)i * L + j]; }
        mu /= D; nu /= D;
        double vm = 0.0, vs = 0.0;
        for (int i = 0; i < D; ++i) {
            const double dm = (double)m[(size_t)i * L + j] - mu, ds = (double)s[(size_t)i * L + j] - nu;
            vm += dm * dm; vs += ds * ds;
        }
        stat[j] = mu; stat[L + j] = sqrt(vm / D + eps);
        stat[2 * L + j] = nu; stat[3 * L + j] = sqrt(vs / D + eps);
    }
    __syncthreads();
    for (int i = threadIdx.x; i < D; i += nfds::THREADS) {
        double acc_m = 0.0, acc_s = 0.0;
        for (int j = 0; j < L; ++j) {
            const double zm = ((double)m[(size_t)i * L + j] - stat[j]) / stat[L + j];
            const double zs = ((double)s[(size_t)i * L + j] - stat[2 * L + j]) / stat[3 * L + j];
            acc_m += zm * zm; acc_s += zs * zs;
        }
        score[i] = (float)sqrt(acc_m + acc_s);
    }
}

// keep[i] = 1 for the n_keep samples of lowest score, equal scores ordered by index
__global__ void nfds_keep_lowest_kernel(const float *__restrict__ score, int D, int n_keep, uint8_t *__restrict__ keep)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= D) return;
    const float si = score[i];
    int rank = 0;
    for (int k = 0; k < D; ++k) {
        const float sk = score[k];
        rank += (sk < si || (sk == si && k < i)) ? 1 : 0;
    }
    keep[i] = rank < n_keep ? 1 : 0;
}

// one Lloyd iteration: labels, then every centre coordinate as the mean of its points (one block)
__global__ __launch_bounds__(nfds::THREADS) void nfds_kmeans_step_kernel(const float *__restrict__ c, int n, int dim, int K,
                                                                        const float *__restrict__ cin, float *__restrict__ cout,
                                                                        int32_t *__restrict__ labels)
{
    for (int i = threadIdx.x; i < n; i += nfds::THREADS) {
        int best = 0;
        double best_d = 0.0;
        for (int k = 0; k < K; ++k) {
            double d = 0.0;
            for (int j = 0; j < dim; ++j) {
                const double e = (double)c[(size_t)i * dim + j] - (double)cin[(size_t)k * dim + j];
                d += e * e;
            }
            if (k == 0 || d < best_d) { best = k; best_d = d; }
        }
        labels[i] = best;
    }
    __threadfence_block();
    __syncthreads();
    for (int e = threadIdx.x; e < K * dim; e += nfds::THREADS) {
        const int k = e / dim, j = e % dim;
        double sum = 0.0;
        int cnt = 0;
        for (int i = 0; i < n; ++i)
            if (labels[i] == k) { sum += (double)c[(size_t)i * dim + j]; ++cnt; }
        cout[e] = cnt > 0 ? (float)(sum / cnt) : cin[e];
    }
}

// ---------------------------------------------------------------------------------------------------------------
size_t nfds_workspace_bytes(int rows, long long count, bool f32)
{
    return (size_t)rows * nfds::blocks_per_row(rows, count, f32 ? 4 : 2) * 2 * sizeof(double);
}

hipError_t run_nfds_moments(const void *A, bool f32, int rows, long long count, float *mean, float *var, double *ws,
                            hipStream_t stream)
{
    if (rows <= 0) return hipSuccess;
    const int bpr = nfds::blocks_per_row(rows, count, f32 ? 4 : 2);
    if (f32) nfds_partial_kernel<true, false><<<rows * bpr, nfds::THREADS, 0, stream>>>(A, count, bpr, 1, ws);
    else nfds_partial_kernel<false, false><<<rows * bpr, nfds::THREADS, 0, stream>>>(A, count, bpr, 1, ws);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    nfds_moments_final_kernel<<<(rows + 255) / 256, 256, 0, stream>>>(ws, rows, bpr, count, mean, var);
    return hipGetLastError();
}

hipError_t run_nfds_frame_correlation(const void *A, bool f32, int samples, int f, long long dhat, float *c, double *ws,
                                      hipStream_t stream)
{
    if (samples <= 0) return hipSuccess;
    const int rows = samples * f;
    const int bpr = nfds::blocks_per_row(rows, dhat, f32 ? 4 : 2);
    if (f32) nfds_partial_kernel<true, true><<<rows * bpr, nfds::THREADS, 0, stream>>>(A, dhat, bpr, f, ws);
    else nfds_partial_kernel<false, true><<<rows * bpr, nfds::THREADS, 0, stream>>>(A, dhat, bpr, f, ws);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int n = samples * (f - 1);
    nfds_corr_final_kernel<<<(n + 255) / 256, 256, 0, stream>>>(ws, samples, f, bpr, c);
    return hipGetLastError();
}

hipError_t run_nfds_scores(const float *m, const float *s, int D, int L, double eps, float *score, hipStream_t stream)
{
    nfds_scores_kernel<<<1, nfds::THREADS, 4 * L * sizeof(double), stream>>>(m, s, D, L, eps, score);
    return hipGetLastError();
}

hipError_t run_nfds_keep_lowest(const float *score, int D, int n_keep, uint8_t *keep, hipStream_t stream)
{
    nfds_keep_lowest_kernel<<<(D + 255) / 256, 256, 0, stream>>>(score, D, n_keep, keep);
    return hipGetLastError();
}

hipError_t run_nfds_kmeans_step(const float *c, int n, int dim, int K, const float *cin, float *cout, int32_t *labels,
                                hipStream_t stream)
{
    nfds_kmeans_step_kernel<<<1, nfds::THREADS, 0, stream>>>(c, n, dim, K, cin, cout, labels);
    return hipGetLastError();
}

}  // namespace qvggt
