// Launchers of the non-GEMM kernels.  All pointers are device pointers unless said otherwise.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>
#include "gemm.hpp"

namespace blstm {

constexpr int BLSTM_MAX_PAIRS = 32;                  // pairs of one matching (64 replicas)

// ---- LSTM cell, one visited frame of both directions ---------------------------------
// Index d = direction.  Row strides are in elements.
struct CellFwdArgs {
    const float* pre[2];      // pre-activations a = W_x x + U_h h_prev + b, [B][4H] rows of stride ld_pre
    long long ld_pre;
    const float* c_prev[2];   // [B][H] rows of stride 2H, or null at the first visited frame
    float* c[2];              // [B][H] rows of stride 2H
    void* gates[2];           // activations i,f,g,o: [B][4H] rows of stride 8H (storage type)
    void* y[2];               // h: [B][H] rows of stride 2H (storage type)
    int B, H;
};
hipError_t launch_cell_fwd(const CellFwdArgs& a, DType store, hipStream_t s);

struct CellBwdArgs {
    const void* dy[2];        // dE/dh from the layer above, rows of stride 2H (storage type)
    const float* dh_rec[2];   // [B][H] contiguous, or null at the last visited frame
    float* dc_rec[2];         // [B][H] contiguous, read (unless first != 0) and overwritten
    const void* gates[2];     // rows of stride 8H
    const float* c[2];        // rows of stride 2H
    const float* c_prev[2];   // rows of stride 2H, or null at the first visited frame
    void* da[2];              // dE/da: [B][4H] rows of stride 8H (storage type)
    int B, H;
    int first;                // != 0: dc_rec is taken as zero (last visited frame)
};
hipError_t launch_cell_bwd(const CellBwdArgs& a, DType store, hipStream_t s);

// ---- softmax cross-entropy over rows of the logit matrix -----------------------------
// u [M][V] (storage type) is overwritten by dE/du = s (p - onehot); row_loss[m] = -s log p[label].
hipError_t launch_softmax_rows(void* u, long long ldu, const int32_t* labels, float* row_loss,
                               int M, int V, float s, DType store, hipStream_t st);
// out[0] = sum_m v[m], one workgroup, fixed summation order.
hipError_t launch_sum_to_scalar(const float* v, int M, float* out, hipStream_t st);

// ---- column sums: out[n] = sum_m A[m][n]; columns >= split go to out_hi[n - split] -------------
hipError_t launch_colsum(const void* A, long long lda, int M, int N, float* out_lo, float* out_hi, int split,
                         DType store, hipStream_t st);

// ---- weight update and replica averaging ---------------------------------------------
hipError_t launch_sgd(float* theta, unsigned short* shadow, const float* grad, size_t n, float lr, float mu,
                      float* vel, hipStream_t st);
struct MixPairs {
    float* a[BLSTM_MAX_PAIRS];
    float* b[BLSTM_MAX_PAIRS];
    unsigned short* sa[BLSTM_MAX_PAIRS];
    unsigned short* sb[BLSTM_MAX_PAIRS];
    int npairs;
};
hipError_t launch_mix(const MixPairs& p, size_t n, hipStream_t st);
hipError_t launch_shadow(const float* theta, unsigned short* shadow, size_t n, hipStream_t st);

}  // namespace blstm
