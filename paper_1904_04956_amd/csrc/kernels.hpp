// Launchers of the non-GEMM kernels.  All pointers are device pointers unless said otherwise.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>
#include "gemm.hpp"

namespace blstm {

constexpr int BLSTM_MAX_PAIRS = 32;                  // pairs of one matching (64 replicas)
constexpr int BLSTM_MAX_REPLICA_PTRS = 64;           // replicas of one average (equals BLSTM_MAX_REPLICAS of the C header)

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

// ---- persistent recurrent kernels (bf16 storage, H one of 128, 256, 512, 1024) -------------------
struct RecFwdArgs {
    const unsigned short* uh[2];  // U_h per direction, [4H][H]
    const float* ax;              // W_x x + b for every frame, [M][8H]
    unsigned short* y;            // layer output h, [M][2H]
    unsigned short* hx;           // h again in exchange order, [T][2][tiles][H/16][2][32][8]; pre-filled with 0xFFFF in sentinel mode
    unsigned short* gates;        // gate activations for rec_bwd_kernel only, as per-lane records [T][2][tiles][H/32][2][256] 16-byte words (not the per-frame path's [M][8H])
    float* c;                     // cell states, records [T][2][tiles][H/32][256] of four floats; both sized for whole 32-row tiles
    unsigned* cnt;                // [2*nbg][tiles_per_group] counters, zero before the launch
    unsigned* abort_word;         // raised when a wait ran out of time
    unsigned long long limit_ticks;   // wait limit in ticks of the 100 MHz wall clock
    // fill_words 16-byte words at `fill` are set to 0xFF bytes while the kernel runs (the backward kernel's exchange copy
    // of this layer, marked "not written yet" off the frame-to-frame path instead of by a launch of its own); null: none
    void* fill;
    unsigned long long fill_words;
    int T, B, H, nbg, tiles_per_group;
};
struct RecBwdArgs {
    const unsigned short* uht[2]; // U_h^T per direction, [H][4H]
    const unsigned short* dy;     // dE/dh from above, [M][2H]
    const unsigned short* gates;  // as rec_fwd_kernel wrote them (per-lane records)
    const float* c;               // likewise
    unsigned short* da;           // dE/da, [M][8H]
    unsigned short* dax;          // dE/da again in exchange order, [T][2][tiles][4H/16][2][32][8]; pre-filled with 0xFFFF in sentinel mode
    float* dc;                    // carried dE/dc, records [2][tiles][H/32][256] of four floats (whole 32-row tiles)
    unsigned* cnt;
    unsigned* abort_word;
    unsigned long long limit_ticks;
    int T, B, H, nbg, tiles_per_group;
};
// Wavefronts per workgroup of the persistent kernels for this H, 0 if H is not supported.
int rec_waves_for(int H, int B);
// Whether launch_rec_fwd for this width honours RecFwdArgs::fill.
bool rec_fwd_fills(int H);
// *launched is false (and nothing was enqueued) when the grid cannot be co-resident on this device.
hipError_t launch_rec_fwd(const RecFwdArgs& a, bool sentinel, hipStream_t st, bool* launched);
hipError_t launch_rec_bwd(const RecBwdArgs& a, bool sentinel, hipStream_t st, bool* launched);
// Transposes `count` matrices U_h [4H][H] (one per layer and direction) into dst + k * 4H*H.
struct TransposeUhArgs {
    const unsigned short* src[128];
    unsigned short* dst;
    int count;
};
hipError_t launch_transpose_uh(const TransposeUhArgs& a, int H, hipStream_t st);
hipError_t launch_fill_u32(unsigned* p, int n, unsigned v, hipStream_t st);
// Copies up to three row-major 16-bit matrices [rows][cols] (leading dimension ld) into [rows][cols_p] ones
// with zeros in columns cols .. cols_p - 1 (cols_p a multiple of 8, dst 16-byte aligned).
struct PadColsArgs {
    const unsigned short* src[3];
    unsigned short* dst[3];
    long long ld[3];
    int rows[3];
    int count, cols, cols_p;
};
hipError_t launch_pad_cols(const PadColsArgs& a, hipStream_t st);
// Fills bytes/16 16-byte words with the 32-bit pattern v.
hipError_t launch_fill_bytes16(void* p, size_t bytes, unsigned v, hipStream_t st);

// ---- softmax cross-entropy over rows of the logit matrix -----------------------------
// u [M][V] (storage type) is overwritten by dE/du = s (p - onehot); row_loss[m] = -s log p[label].
hipError_t launch_softmax_rows(void* u, long long ldu, const int32_t* labels, float* row_loss,
                               int M, int V, float s, DType store, hipStream_t st);
// out[0] = sum_m v[m], one workgroup, fixed summation order.
hipError_t launch_sum_to_scalar(const float* v, int M, float* out, hipStream_t st);

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
hipError_t launch_sgd_mix_pair(float* ti, float* tj, const float* gi, const float* gj, float* vi, float* vj,
                               unsigned short* si, unsigned short* sj, size_t n, float lr, float mu, hipStream_t st);
struct ReplicaSet {
    float* t[BLSTM_MAX_REPLICA_PTRS];
    unsigned short* s[BLSTM_MAX_REPLICA_PTRS];
    int R;
};
hipError_t launch_sync_average(const ReplicaSet& p, size_t n, hipStream_t st);

}  // namespace blstm
