// Streaming kernels over the flat parameter vector: SGD update (Eq. 1c), pairwise replica
// averaging (Eq. 4, second line) and the bf16 shadow.  All are bound by HBM bandwidth:
// every element is read once and written once with 16-byte accesses.
#include "common.hpp"
#include "kernels.hpp"

namespace blstm {
namespace {

constexpr int UPD_THREADS = 256;
typedef unsigned int u32x2_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint2 pack4(float4 v) { return make_uint2(pack_bf2(v.x, v.y), pack_bf2(v.z, v.w)); }

constexpr int SGD_U = 2;
template <bool SHADOW, bool MOM>
__global__ __launch_bounds__(UPD_THREADS) void sgd_kernel(float* __restrict__ theta, unsigned short* __restrict__ shadow,
                                                          const float* __restrict__ grad, float* __restrict__ vel,
                                                          size_t n, float lr, float mu) {
    // one contiguous span of SGD_U * UPD_THREADS 16-byte words per workgroup, all loads of a span before its first store
    const size_t n4 = n / 4;
    const size_t base = (size_t)blockIdx.x * SGD_U * UPD_THREADS + threadIdx.x;
    f32x4_t t[SGD_U], g[SGD_U], v[SGD_U];
#pragma unroll
    for (int k = 0; k < SGD_U; ++k) {
        const size_t i = base + (size_t)k * UPD_THREADS;
        if (i < n4) {
            t[k] = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(theta) + i);
            g[k] = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(grad) + i);
            if (MOM) v[k] = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(vel) + i);
        }
    }
#pragma unroll
    for (int k = 0; k < SGD_U; ++k) {
        const size_t i = base + (size_t)k * UPD_THREADS;
        if (i < n4) {
            if (MOM) {
                g[k] = mu * v[k] + g[k];
                __builtin_nontemporal_store(g[k], reinterpret_cast<f32x4_t*>(vel) + i);
            }
            const f32x4_t r = t[k] - lr * g[k];
            __builtin_nontemporal_store(r, reinterpret_cast<f32x4_t*>(theta) + i);
            if (SHADOW) {
                u32x2_t q; q[0] = pack_bf2(r[0], r[1]); q[1] = pack_bf2(r[2], r[3]);
                __builtin_nontemporal_store(q, reinterpret_cast<u32x2_t*>(shadow) + i);
            }
        }
    }
    // tail (n not a multiple of four)
    if (blockIdx.x == 0 && threadIdx.x < (n & 3)) {
        const size_t i = n4 * 4 + threadIdx.x;
        float g = grad[i];
        if (MOM) { g = mu * vel[i] + g; vel[i] = g; }
        const float t = theta[i] - lr * g;
        theta[i] = t;
        if (SHADOW) shadow[i] = f2bf(t);
    }
}

// Both members of pair blockIdx.y become their average.  A workgroup owns one contiguous span of MIX_SPAN 16-byte
// words of the pair (many small workgroups, each streaming one 16 KB piece per operand, measured a few percent above
// a grid-stride walk); its four independent 16-byte loads per operand are issued before the first store so that
// enough bytes are in flight to cover HBM latency.  Non-temporal loads and stores.
constexpr int MIX_U = 4;
constexpr size_t MIX_SPAN = (size_t)MIX_U * UPD_THREADS;
template <bool SHADOW>
__global__ __launch_bounds__(UPD_THREADS) void mix_kernel(MixPairs p, size_t n) {
    const int pr = blockIdx.y;
    f32x4_t* __restrict__ a = reinterpret_cast<f32x4_t*>(p.a[pr]);
    f32x4_t* __restrict__ b = reinterpret_cast<f32x4_t*>(p.b[pr]);
    u32x2_t* __restrict__ sa = reinterpret_cast<u32x2_t*>(p.sa[pr]);
    u32x2_t* __restrict__ sb = reinterpret_cast<u32x2_t*>(p.sb[pr]);
    const size_t n4 = n / 4;
    const size_t i = (size_t)blockIdx.x * MIX_SPAN + threadIdx.x;
    if ((size_t)(blockIdx.x + 1) * MIX_SPAN <= n4) {        // a whole span
        f32x4_t x[MIX_U], y[MIX_U];
#pragma unroll
        for (int k = 0; k < MIX_U; ++k) { x[k] = __builtin_nontemporal_load(a + i + k * UPD_THREADS); y[k] = __builtin_nontemporal_load(b + i + k * UPD_THREADS); }
#pragma unroll
        for (int k = 0; k < MIX_U; ++k) {
            const f32x4_t m = 0.5f * (x[k] + y[k]);
            __builtin_nontemporal_store(m, a + i + k * UPD_THREADS);
            __builtin_nontemporal_store(m, b + i + k * UPD_THREADS);
            if (SHADOW) {
                u32x2_t s; s[0] = pack_bf2(m[0], m[1]); s[1] = pack_bf2(m[2], m[3]);
                __builtin_nontemporal_store(s, sa + i + k * UPD_THREADS);
                __builtin_nontemporal_store(s, sb + i + k * UPD_THREADS);
            }
        }
    } else {                                               // the last, partial span
        for (size_t j = i; j < n4; j += UPD_THREADS) {
            const f32x4_t m = 0.5f * (a[j] + b[j]);
            a[j] = m; b[j] = m;
            if (SHADOW) { u32x2_t s; s[0] = pack_bf2(m[0], m[1]); s[1] = pack_bf2(m[2], m[3]); sa[j] = s; sb[j] = s; }
        }
    }
    if (blockIdx.x == 0 && threadIdx.x < (n & 3)) {
        const size_t j = n4 * 4 + threadIdx.x;
        float* fa = p.a[pr]; float* fb = p.b[pr];
        const float m = 0.5f * (fa[j] + fb[j]);
        fa[j] = m; fb[j] = m;
        if (SHADOW) { p.sa[pr][j] = f2bf(m); p.sb[pr][j] = f2bf(m); }
    }
}

// Eq. 4 in one pass for a pair: theta_i' = theta_i - lr g_i, theta_j' likewise (Eq. 1c, same arithmetic
// as sgd_kernel, momentum included), then both become (theta_i' + theta_j')/2.  One read of each
// operand and one write of each result: 24 B per parameter of the pair against 40 B for sgd_kernel
// twice plus mix_kernel (fp32, no momentum).  GJ = false: replica j has no gradient here (its own learner
// has applied its update already) and enters the average as it stands: a learner's own update and its
// averaging with a neighbour in one pass, 20 B per parameter against 28 B for sgd_kernel plus mix_kernel.
template <bool SHADOW, bool MOM, bool GJ>
__global__ __launch_bounds__(UPD_THREADS) void sgd_mix_pair_kernel(float* __restrict__ ti, float* __restrict__ tj,
                                                                   const float* __restrict__ gi, const float* __restrict__ gj,
                                                                   float* __restrict__ vi, float* __restrict__ vj,
                                                                   unsigned short* __restrict__ si, unsigned short* __restrict__ sj,
                                                                   size_t n, float lr, float mu) {
    // one contiguous span of PAIR_U * UPD_THREADS 16-byte words per workgroup, all loads of a span before its first store
    constexpr int PAIR_U = 2;
    const size_t n4 = n / 4;
    const size_t base = (size_t)blockIdx.x * PAIR_U * UPD_THREADS + threadIdx.x;
    f32x4_t a[PAIR_U], b[PAIR_U], ga[PAIR_U], gb[PAIR_U], va[PAIR_U], vb[PAIR_U];
#pragma unroll
    for (int k = 0; k < PAIR_U; ++k) {
        const size_t i = base + (size_t)k * UPD_THREADS;
        if (i < n4) {
            a[k] = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(ti) + i);
            b[k] = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(tj) + i);
            ga[k] = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(gi) + i);
            if (GJ) gb[k] = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(gj) + i);
            if (MOM) {
                va[k] = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(vi) + i);
                if (GJ) vb[k] = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(vj) + i);
            }
        }
    }
#pragma unroll
    for (int k = 0; k < PAIR_U; ++k) {
        const size_t i = base + (size_t)k * UPD_THREADS;
        if (i < n4) {
            if (MOM) {
                ga[k] = mu * va[k] + ga[k];
                __builtin_nontemporal_store(ga[k], reinterpret_cast<f32x4_t*>(vi) + i);
                if (GJ) {
                    gb[k] = mu * vb[k] + gb[k];
                    __builtin_nontemporal_store(gb[k], reinterpret_cast<f32x4_t*>(vj) + i);
                }
            }
            const f32x4_t x = a[k] - lr * ga[k];
            f32x4_t y = b[k];
            if (GJ) y = b[k] - lr * gb[k];
            const f32x4_t m = 0.5f * (x + y);
            __builtin_nontemporal_store(m, reinterpret_cast<f32x4_t*>(ti) + i);
            __builtin_nontemporal_store(m, reinterpret_cast<f32x4_t*>(tj) + i);
            if (SHADOW) {
                u32x2_t q; q[0] = pack_bf2(m[0], m[1]); q[1] = pack_bf2(m[2], m[3]);
                __builtin_nontemporal_store(q, reinterpret_cast<u32x2_t*>(si) + i);
                __builtin_nontemporal_store(q, reinterpret_cast<u32x2_t*>(sj) + i);
            }
        }
    }
    if (blockIdx.x == 0 && threadIdx.x < (n & 3)) {
        const size_t i = n4 * 4 + threadIdx.x;
        float ga1 = gi[i], gb1 = GJ ? gj[i] : 0.0f;
        if (MOM) { ga1 = mu * vi[i] + ga1; vi[i] = ga1; if (GJ) { gb1 = mu * vj[i] + gb1; vj[i] = gb1; } }
        const float a1 = ti[i] - lr * ga1, b1 = GJ ? tj[i] - lr * gb1 : tj[i];
        const float m = 0.5f * (a1 + b1);
        ti[i] = m; tj[i] = m;
        if (SHADOW) { si[i] = f2bf(m); sj[i] = f2bf(m); }
    }
}

// Every replica becomes the mean of all R replicas, summed in the order r = 0, 1, .., R-1 in float and
// scaled by 1/R once (the in-HBM form of "allreduce(W') / lambda").
template <bool SHADOW>
__global__ __launch_bounds__(UPD_THREADS) void sync_average_kernel(ReplicaSet p, size_t n, float inv_r) {
    const size_t n4 = n / 4;
    // a workgroup owns one contiguous span of SYNC_U * UPD_THREADS 16-byte words of every replica
    constexpr int SYNC_U = 2;
#pragma unroll
    for (int k = 0; k < SYNC_U; ++k) {
        const size_t i = ((size_t)blockIdx.x * SYNC_U + k) * UPD_THREADS + threadIdx.x;
        if (i >= n4) break;
        // four replicas' loads in flight at a time, added in index order
        f32x4_t acc = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(p.t[0]) + i);
        int r = 1;
        for (; r + 3 < p.R; r += 4) {
            const f32x4_t x0 = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(p.t[r]) + i);
            const f32x4_t x1 = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(p.t[r + 1]) + i);
            const f32x4_t x2 = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(p.t[r + 2]) + i);
            const f32x4_t x3 = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(p.t[r + 3]) + i);
            acc += x0; acc += x1; acc += x2; acc += x3;
        }
        for (; r < p.R; ++r) acc += __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(p.t[r]) + i);
        acc *= inv_r;
        u32x2_t q; q[0] = pack_bf2(acc[0], acc[1]); q[1] = pack_bf2(acc[2], acc[3]);
        for (r = 0; r < p.R; ++r) {
            __builtin_nontemporal_store(acc, reinterpret_cast<f32x4_t*>(p.t[r]) + i);
            if (SHADOW) __builtin_nontemporal_store(q, reinterpret_cast<u32x2_t*>(p.s[r]) + i);
        }
    }
    if (blockIdx.x == 0 && threadIdx.x < (n & 3)) {
        const size_t i = n4 * 4 + threadIdx.x;
        float acc = p.t[0][i];
        for (int r = 1; r < p.R; ++r) acc += p.t[r][i];
        acc *= inv_r;
        for (int r = 0; r < p.R; ++r) { p.t[r][i] = acc; if (SHADOW) p.s[r][i] = f2bf(acc); }
    }
}

__global__ __launch_bounds__(UPD_THREADS) void shadow_kernel(const float* __restrict__ theta, unsigned short* __restrict__ shadow, size_t n) {
    const size_t n4 = n / 4;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += stride)
        reinterpret_cast<uint2*>(shadow)[i] = pack4(reinterpret_cast<const float4*>(theta)[i]);
    if (blockIdx.x == 0 && threadIdx.x < (n & 3)) {
        const size_t i = n4 * 4 + threadIdx.x;
        shadow[i] = f2bf(theta[i]);
    }
}

unsigned blocks_for(size_t n4, unsigned cap) {
    size_t b = (n4 + UPD_THREADS - 1) / UPD_THREADS;
    if (b < 1) b = 1;
    return (unsigned)(b < cap ? b : cap);
}

}  // namespace

hipError_t launch_sgd(float* theta, unsigned short* shadow, const float* grad, size_t n, float lr, float mu,
                      float* vel, hipStream_t st) {
    if (n == 0) return hipSuccess;
    const size_t spans = (n / 4 + SGD_U * UPD_THREADS - 1) / (SGD_U * UPD_THREADS);
    dim3 grid((unsigned)(spans < 1 ? 1 : spans)), block(UPD_THREADS);
    const bool mom = (mu != 0.0f);
    if (shadow && mom) hipLaunchKernelGGL((sgd_kernel<true, true>), grid, block, 0, st, theta, shadow, grad, vel, n, lr, mu);
    else if (shadow) hipLaunchKernelGGL((sgd_kernel<true, false>), grid, block, 0, st, theta, shadow, grad, vel, n, lr, mu);
    else if (mom) hipLaunchKernelGGL((sgd_kernel<false, true>), grid, block, 0, st, theta, shadow, grad, vel, n, lr, mu);
    else hipLaunchKernelGGL((sgd_kernel<false, false>), grid, block, 0, st, theta, shadow, grad, vel, n, lr, mu);
    return hipGetLastError();
}

hipError_t launch_mix(const MixPairs& p, size_t n, hipStream_t st) {
    if (n == 0 || p.npairs == 0) return hipSuccess;
    const size_t spans = (n / 4 + MIX_SPAN - 1) / MIX_SPAN;
    dim3 grid((unsigned)(spans < 1 ? 1 : spans), (unsigned)p.npairs), block(UPD_THREADS);
    if (p.sa[0]) hipLaunchKernelGGL(mix_kernel<true>, grid, block, 0, st, p, n);
    else hipLaunchKernelGGL(mix_kernel<false>, grid, block, 0, st, p, n);
    return hipGetLastError();
}

hipError_t launch_sgd_mix_pair(float* ti, float* tj, const float* gi, const float* gj, float* vi, float* vj,
                               unsigned short* si, unsigned short* sj, size_t n, float lr, float mu, hipStream_t st) {
    if (n == 0) return hipSuccess;
    const size_t spans = (n / 4 + 2 * UPD_THREADS - 1) / (2 * UPD_THREADS);      // (PAIR_U words per thread)
    dim3 grid((unsigned)(spans < 1 ? 1 : spans)), block(UPD_THREADS);
    const bool mom = (mu != 0.0f), sh = si != nullptr;
#define BLSTM_PAIR(S, M, G) hipLaunchKernelGGL((sgd_mix_pair_kernel<S, M, G>), grid, block, 0, st, ti, tj, gi, gj, vi, vj, si, sj, n, lr, mu)
    if (gj) {
        if (sh && mom) BLSTM_PAIR(true, true, true); else if (sh) BLSTM_PAIR(true, false, true);
        else if (mom) BLSTM_PAIR(false, true, true); else BLSTM_PAIR(false, false, true);
    } else {
        if (sh && mom) BLSTM_PAIR(true, true, false); else if (sh) BLSTM_PAIR(true, false, false);
        else if (mom) BLSTM_PAIR(false, true, false); else BLSTM_PAIR(false, false, false);
    }
#undef BLSTM_PAIR
    return hipGetLastError();
}

hipError_t launch_sync_average(const ReplicaSet& p, size_t n, hipStream_t st) {
    if (n == 0 || p.R < 1) return hipSuccess;
    const size_t spans = (n / 4 + 2 * UPD_THREADS - 1) / (2 * UPD_THREADS);      // (SYNC_U words per thread)
    dim3 grid((unsigned)(spans < 1 ? 1 : spans)), block(UPD_THREADS);
    const float inv_r = 1.0f / (float)p.R;
    if (p.s[0]) hipLaunchKernelGGL(sync_average_kernel<true>, grid, block, 0, st, p, n, inv_r);
    else hipLaunchKernelGGL(sync_average_kernel<false>, grid, block, 0, st, p, n, inv_r);
    return hipGetLastError();
}

hipError_t launch_shadow(const float* theta, unsigned short* shadow, size_t n, hipStream_t st) {
    if (n == 0) return hipSuccess;
    hipLaunchKernelGGL(shadow_kernel, dim3(blocks_for(n / 4, 256 * 16)), dim3(UPD_THREADS), 0, st, theta, shadow, n);
    return hipGetLastError();
}

}  // namespace blstm
