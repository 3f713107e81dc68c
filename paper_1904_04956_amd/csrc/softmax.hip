// Row-wise softmax cross-entropy on a materialised logit matrix, with fixed-order sums.
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

}  // namespace blstm
