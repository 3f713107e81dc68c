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
// General form: three passes over the row (the second and third normally hit L2).
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
    // a label outside [0, V) is never used as an index: the frame's loss term becomes NaN and its row p without a one-hot
    const int lab = labels[m];
    const bool lab_ok = (unsigned)lab < (unsigned)V;
    const float inv = 1.0f / sum;
    if (threadIdx.x == 0) row_loss[m] = lab_ok ? s * (logf(sum) + mx - ld_f(row + lab)) : __builtin_nanf("");
    __syncthreads();                                   // the label's logit is read before it is overwritten
    for (int v = threadIdx.x; v < V; v += blockDim.x) {
        float p = expf(ld_f(row + v) - mx) * inv;
        st_f(row + v, s * (p - ((lab_ok && v == lab) ? 1.0f : 0.0f)));
    }
}

// bf16 rows that fit the registers of one workgroup (V <= NT * 8 * NC, V a multiple of 8, rows
// 16-byte aligned): the row is read once with 16-byte loads, kept in registers as packed bf16,
// reduced, and written back as dE/du with 16-byte stores.  HBM traffic: one read and one write.
// A long row is spread over more threads rather than more registers per thread, so that several
// rows per CU are in flight and one row's loads and stores run under another's arithmetic.
template <int NC, int NT>
__global__ __launch_bounds__(NT) void softmax_rows_bf16_regs_kernel(bf16_t* u, long long ldu, const int32_t* labels,
                                                                      float* row_loss, int V, float s) {
    __shared__ float sh[NT / 64];
    const int m = blockIdx.x;
    bf16_t* row = u + (long long)m * ldu;
    const int nchunks = V >> 3;
    uint4 r[NC];
    float mx = -INFINITY;
#pragma unroll
    for (int i = 0; i < NC; ++i) {
        const int c = threadIdx.x + NT * i;
        if (c < nchunks) {
            r[i] = *reinterpret_cast<const uint4*>(row + 8 * c);
            const uint32_t w[4] = {r[i].x, r[i].y, r[i].z, r[i].w};
#pragma unroll
            for (int q = 0; q < 4; ++q) mx = fmaxf(mx, fmaxf(bf2f((bf16_t)(w[q] & 0xFFFFu)), bf2f((bf16_t)(w[q] >> 16))));
        } else {
            r[i] = make_uint4(0, 0, 0, 0);
        }
    }
    mx = block_reduce(mx, true, sh);
    // exp(x - mx) = exp2(x * log2(e) - mx * log2(e)): one multiply-add and the hardware exp2 per element
    // (the argument is <= 0; a result below the normal range flushes to 0, as its probability does in bf16)
    const float L2E = 1.44269504f;
    const float mxl = mx * L2E;
    float sum = 0.0f;
#pragma unroll
    for (int i = 0; i < NC; ++i) {
        const int c = threadIdx.x + NT * i;
        if (c < nchunks) {
            const uint32_t w[4] = {r[i].x, r[i].y, r[i].z, r[i].w};
#pragma unroll
            for (int q = 0; q < 4; ++q)
                sum += __builtin_amdgcn_exp2f(__builtin_fmaf(bf2f((bf16_t)(w[q] & 0xFFFFu)), L2E, -mxl)) +
                       __builtin_amdgcn_exp2f(__builtin_fmaf(bf2f((bf16_t)(w[q] >> 16)), L2E, -mxl));
        }
    }
    sum = block_reduce(sum, false, sh);
    const int lab = labels[m];
    const bool lab_ok = (unsigned)lab < (unsigned)V;   // (as in the general kernel: an out-of-range label gives a NaN loss term)
    const float sinv = s / sum;
    if (threadIdx.x == 0) row_loss[m] = lab_ok ? s * (logf(sum) + mx - bf2f(row[lab])) : __builtin_nanf("");
    __syncthreads();                                   // the label's logit is read before the row is overwritten
    const int labc = lab_ok ? lab >> 3 : -1;           // the one chunk whose output also carries the -s of the one-hot
#pragma unroll
    for (int i = 0; i < NC; ++i) {
        const int c = threadIdx.x + NT * i;
        if (c < nchunks) {
            const uint32_t w[4] = {r[i].x, r[i].y, r[i].z, r[i].w};
            float p[8];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                p[2 * q] = __builtin_amdgcn_exp2f(__builtin_fmaf(bf2f((bf16_t)(w[q] & 0xFFFFu)), L2E, -mxl)) * sinv;
                p[2 * q + 1] = __builtin_amdgcn_exp2f(__builtin_fmaf(bf2f((bf16_t)(w[q] >> 16)), L2E, -mxl)) * sinv;
            }
            if (c == labc) {
#pragma unroll
                for (int e = 0; e < 8; ++e) p[e] -= (e == (lab & 7)) ? s : 0.0f;
            }
            *reinterpret_cast<uint4*>(row + 8 * c) = make_uint4(pack_bf2(p[0], p[1]), pack_bf2(p[2], p[3]), pack_bf2(p[4], p[5]), pack_bf2(p[6], p[7]));
        }
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
    if (store == DT_BF16) {
        bf16_t* ub = static_cast<bf16_t*>(u);
        const bool vec = (V % 8 == 0) && (ldu % 8 == 0) && (reinterpret_cast<uintptr_t>(u) % 16 == 0);
        const int nchunks = V / 8;
#define BLSTM_SOFTMAX_REGS(NC, NT) \
    hipLaunchKernelGGL((softmax_rows_bf16_regs_kernel<NC, NT>), dim3(M), dim3(NT), 0, st, ub, ldu, labels, row_loss, V, s)
        if (vec && nchunks <= 4 * 256) BLSTM_SOFTMAX_REGS(4, 256);
        else if (vec && nchunks <= 4 * 512) BLSTM_SOFTMAX_REGS(4, 512);
        else if (vec && nchunks <= 4 * 1024) BLSTM_SOFTMAX_REGS(4, 1024);
        else if (vec && nchunks <= 8 * 1024) BLSTM_SOFTMAX_REGS(8, 1024);
#undef BLSTM_SOFTMAX_REGS
        else hipLaunchKernelGGL(softmax_rows_kernel<bf16_t>, dim3(M), dim3(256), 0, st, ub, ldu, labels, row_loss, V, s);
    }
    else
        hipLaunchKernelGGL(softmax_rows_kernel<float>, dim3(M), dim3(256), 0, st, static_cast<float*>(u), ldu, labels, row_loss, V, s);
    return hipGetLastError();
}

hipError_t launch_sum_to_scalar(const float* v, int M, float* out, hipStream_t st) {
    hipLaunchKernelGGL(sum_to_scalar_kernel, dim3(1), dim3(1024), 0, st, v, M, out);
    return hipGetLastError();
}

}  // namespace blstm
