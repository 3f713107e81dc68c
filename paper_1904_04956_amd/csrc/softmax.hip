// Row-wise softmax cross-entropy on a materialised logit matrix, fixed-order sums, and
// column sums for the bias gradients.
#include "common.hpp"
#include "kernels.hpp"

namespace blstm {
namespace {

__device__ __forceinline__ float block_reduce(float v, bool is_max, float* sh) {
    v = is_max ? wave_max(v) : wave_sum(v);
    const int wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sh[wave] = v;
    __syncthreads();
    float r = sh[0];
    for (int w = 1; w < nw; ++w) r = is_max ? fmaxf(r, sh[w]) : r + sh[w];
    return r;
}

// One workgroup per row: max, sum of exponentials, loss term, then u <- s (p - onehot) in place.
template <typename TS>
__global__ __launch_bounds__(256) void softmax_rows_kernel(TS* u, long long ldu, const int32_t* labels,
                                                           float* row_loss, int V, float s) {
    __shared__ float sh[4];
    const int m = blockIdx.x;
    TS* row = u + (long long)m * ldu;
    float mx = -INFINITY;
    for (int v = threadIdx.x; v < V; v += blockDim.x) mx = fmaxf(mx, ld_f(row + v));
    mx = block_reduce(mx, true, sh);
    float sum = 0.0f;
    for (int v = threadIdx.x; v < V; v += blockDim.x) sum += expf(ld_f(row + v) - mx);
    sum = block_reduce(sum, false, sh);
    const int lab = labels[m];
    const float inv = 1.0f / sum;
    if (threadIdx.x == 0) row_loss[m] = s * (logf(sum) + mx - ld_f(row + lab));
    __syncthreads();                                   // the label's logit is read before it is overwritten
    for (int v = threadIdx.x; v < V; v += blockDim.x) {
        float p = expf(ld_f(row + v) - mx) * inv;
        st_f(row + v, s * (p - (v == lab ? 1.0f : 0.0f)));
    }
}

__global__ __launch_bounds__(1024) void sum_to_scalar_kernel(const float* v, int M, float* out) {
    __shared__ float sh[16];
    float acc = 0.0f;
    for (int i = threadIdx.x; i < M; i += blockDim.x) acc += v[i];
    acc = block_reduce(acc, false, sh);
    if (threadIdx.x == 0) out[0] = acc;
}

// 64 columns x 4 row groups per workgroup; every column is summed in a fixed order.
template <typename TS>
__global__ __launch_bounds__(256) void colsum_kernel(const TS* A, long long lda, int M, int N,
                                                     float* out_lo, float* out_hi, int split) {
    __shared__ float sh[4][64];
    const int cx = threadIdx.x & 63, rg = threadIdx.x >> 6;
    const int n = blockIdx.x * 64 + cx;
    float acc = 0.0f;
    if (n < N)
        for (int m = rg; m < M; m += 4) acc += ld_f(A + (long long)m * lda + n);
    sh[rg][cx] = acc;
    __syncthreads();
    if (rg == 0 && n < N) {
        float t = (sh[0][cx] + sh[1][cx]) + (sh[2][cx] + sh[3][cx]);
        if (n < split) out_lo[n] = t; else out_hi[n - split] = t;
    }
}

}  // namespace

hipError_t launch_softmax_rows(void* u, long long ldu, const int32_t* labels, float* row_loss,
                               int M, int V, float s, DType store, hipStream_t st) {
    if (M <= 0) return hipSuccess;
    if (store == DT_BF16)
        hipLaunchKernelGGL(softmax_rows_kernel<bf16_t>, dim3(M), dim3(256), 0, st, static_cast<bf16_t*>(u), ldu, labels, row_loss, V, s);
    else
        hipLaunchKernelGGL(softmax_rows_kernel<float>, dim3(M), dim3(256), 0, st, static_cast<float*>(u), ldu, labels, row_loss, V, s);
    return hipGetLastError();
}

hipError_t launch_sum_to_scalar(const float* v, int M, float* out, hipStream_t st) {
    hipLaunchKernelGGL(sum_to_scalar_kernel, dim3(1), dim3(1024), 0, st, v, M, out);
    return hipGetLastError();
}

hipError_t launch_colsum(const void* A, long long lda, int M, int N, float* out_lo, float* out_hi, int split,
                         DType store, hipStream_t st) {
    if (N <= 0) return hipSuccess;
    dim3 grid((unsigned)((N + 63) / 64)), block(256);
    if (store == DT_BF16)
        hipLaunchKernelGGL(colsum_kernel<bf16_t>, grid, block, 0, st, static_cast<const bf16_t*>(A), lda, M, N, out_lo, out_hi, split);
    else
        hipLaunchKernelGGL(colsum_kernel<float>, grid, block, 0, st, static_cast<const float*>(A), lda, M, N, out_lo, out_hi, split);
    return hipGetLastError();
}

}  // namespace blstm
