// Tiled MFMA GEMM used by every dense contraction of the training step.
#pragma once
#include <hip/hip_runtime.h>

namespace blstm {

enum DType { DT_F32 = 0, DT_BF16 = 1 };

// One (A, B) operand pair contributing  sum_k A(m,k) * B(n,k)  to C(m,n).
//   A(m,k) = atrans ? A[k*lda + m] : A[m*lda + k]
//   B(n,k) = btrans ? B[k*ldb + n] : B[n*ldb + k]
// sA/sB are element strides added per batch index (blockIdx.z); they may be negative.
struct GemmSeg {
    const void* A;
    const void* B;
    long long lda, ldb, sA, sB;
    int K;
};

struct GemmDesc {
    GemmSeg seg[2];
    int nseg;                 // 1 or 2; both segments accumulate into the same C tile
    void* C;                  // [M][N] row-major, leading dimension ldc, element type out_type
    long long ldc, sC;
    const void* bias;         // per column n, element type in_type, or null
    long long sBias;
    const float* add;         // float [M][N] added to the product, or null
    long long ldadd, sAdd;
    float* rowsum;            // rowsum[m] = sum_k A(m,k) of segment 0 (bias gradients), or null
    long long sRowsum;
    float* partial;           // scratch for split-K partial tiles (float), or null: never split
    size_t partial_bytes;
    int M, N, batch;
    int Npad;                 // 0, or a multiple of the tile width >= N up to which B(n, .) may be read (it holds zeros or
                              // anything there): the product runs on whole tiles, C keeps its N columns
    bool atrans, btrans;
    DType in_type, out_type;  // in_type is the element type of A and B
};

// How a product is run: the tile shape, and into how many K ranges it is split.
enum GemmTile { GEMM_TILE_128 = 0,        // 128x128, every element type and shape
                GEMM_TILE_256 = 1,        // 256x256, float operands of large products
                GEMM_TILE_256X128 = 2 };  // 256x128, bf16 operands loaded straight into LDS
struct GemmPlan {
    int tile;                 // a GemmTile
    bool deep;                // 128x128 tile with the loads further ahead (launches of at most one workgroup per CU)
    int splits;
    size_t partial_bytes;     // scratch the split needs (0 when splits == 1)
};
GemmPlan plan_gemm(const GemmDesc& d);
// Scratch bytes a product of this shape would use if it were given unlimited scratch.
size_t gemm_partial_bytes(int M, int N, int K, int batch, DType in_type);

// Validates nothing (the caller's shapes are trusted); returns the launch status.
hipError_t launch_gemm(const GemmDesc& d, hipStream_t stream);
// n independent products of the A^T B form (atrans and btrans, bf16 operands, float result, optional row sums, no
// bias, one segment) in one launch where the shapes allow it (gemm_group_ok); otherwise one launch each.  A grouped
// launch never splits along K and uses no scratch.
bool gemm_group_ok(const GemmDesc* d, int n);
hipError_t launch_gemm_group(const GemmDesc* d, int n, hipStream_t stream);

}  // namespace blstm
