// Element-wise LSTM cell, forward and backward, for one visited frame of both directions.
// Used by the step-by-step path (one launch per frame); the gate order is i, f, g, o.
#include "common.hpp"
#include "kernels.hpp"

namespace blstm {
namespace {

template <typename TS>
__global__ __launch_bounds__(256) void cell_fwd_kernel(CellFwdArgs a) {
    const int H = a.H;
    const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    const int d = blockIdx.y;
    if (idx >= (long long)a.B * H) return;
    const int b = (int)(idx / H), j = (int)(idx % H);
    const float* pre = a.pre[d] + (long long)b * a.ld_pre + j;
    const float ai = pre[0], af = pre[H], ag = pre[2 * H], ao = pre[3 * H];
    const float gi = sigmoidf_(ai), gf = sigmoidf_(af), gg = tanhf_(ag), go = sigmoidf_(ao);
    const float cp = a.c_prev[d] ? a.c_prev[d][(long long)b * 2 * H + j] : 0.0f;
    const float c = gf * cp + gi * gg;
    const float h = go * tanhf_(c);
    a.c[d][(long long)b * 2 * H + j] = c;
    TS* g = static_cast<TS*>(a.gates[d]) + (long long)b * 8 * H + j;
    st_f(g, gi); st_f(g + H, gf); st_f(g + 2 * H, gg); st_f(g + 3 * H, go);
    st_f(static_cast<TS*>(a.y[d]) + (long long)b * 2 * H + j, h);
}

template <typename TS>
__global__ __launch_bounds__(256) void cell_bwd_kernel(CellBwdArgs a) {
    const int H = a.H;
    const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    const int d = blockIdx.y;
    if (idx >= (long long)a.B * H) return;
    const int b = (int)(idx / H), j = (int)(idx % H);
    const TS* g = static_cast<const TS*>(a.gates[d]) + (long long)b * 8 * H + j;
    const float gi = ld_f(g), gf = ld_f(g + H), gg = ld_f(g + 2 * H), go = ld_f(g + 3 * H);
    const float c = a.c[d][(long long)b * 2 * H + j];
    const float cp = a.c_prev[d] ? a.c_prev[d][(long long)b * 2 * H + j] : 0.0f;
    const float tc = tanhf_(c);
    float dh = ld_f(static_cast<const TS*>(a.dy[d]) + (long long)b * 2 * H + j);
    if (a.dh_rec[d]) dh += a.dh_rec[d][(long long)b * H + j];
    float dc = dh * go * (1.0f - tc * tc);
    if (!a.first) dc += a.dc_rec[d][(long long)b * H + j];
    const float da_o = dh * tc * go * (1.0f - go);
    const float da_i = dc * gg * gi * (1.0f - gi);
    const float da_f = dc * cp * gf * (1.0f - gf);
    const float da_g = dc * gi * (1.0f - gg * gg);
    a.dc_rec[d][(long long)b * H + j] = dc * gf;
    TS* da = static_cast<TS*>(a.da[d]) + (long long)b * 8 * H + j;
    st_f(da, da_i); st_f(da + H, da_f); st_f(da + 2 * H, da_g); st_f(da + 3 * H, da_o);
}

}  // namespace

hipError_t launch_cell_fwd(const CellFwdArgs& a, DType store, hipStream_t s) {
    const long long n = (long long)a.B * a.H;
    dim3 grid((unsigned)((n + 255) / 256), 2), block(256);
    if (store == DT_BF16) hipLaunchKernelGGL(cell_fwd_kernel<bf16_t>, grid, block, 0, s, a);
    else hipLaunchKernelGGL(cell_fwd_kernel<float>, grid, block, 0, s, a);
    return hipGetLastError();
}

hipError_t launch_cell_bwd(const CellBwdArgs& a, DType store, hipStream_t s) {
    const long long n = (long long)a.B * a.H;
    dim3 grid((unsigned)((n + 255) / 256), 2), block(256);
    if (store == DT_BF16) hipLaunchKernelGGL(cell_bwd_kernel<bf16_t>, grid, block, 0, s, a);
    else hipLaunchKernelGGL(cell_bwd_kernel<float>, grid, block, 0, s, a);
    return hipGetLastError();
}

}  // namespace blstm
