// Persistent recurrent kernels: all T frames of one layer, both directions, in one launch.
//
// A workgroup owns 32 hidden units of one direction (all four gate rows of each) and a group
// of 32-row batch tiles.  Its slice of U_h stays in vector registers for the whole launch:
// NW wavefronts split the contraction index, each holding 128 VGPRs of MFMA B-fragments.
// Per frame and batch tile a workgroup multiplies the previous h (forward) or the previous
// frame's gate gradients (backward) by its slice, reduces the NW partial accumulators through
// LDS, applies the cell arithmetic with all four gates of a unit in one lane, and writes its
// 32 columns.  The NU = H/32 workgroups that share a batch tile exchange these columns through
// global memory; a per-(group, tile) counter, incremented with release semantics at agent
// scope after a workgroup's stores and polled with acquire semantics before the next frame's
// loads, orders the exchange.  Every wait is bounded by a wall-clock limit: on expiry the
// workgroup raises a global abort word that all other waits observe, so every wave exits.
#include "common.hpp"
#include "kernels.hpp"

namespace blstm {
namespace {

constexpr int KW = 128;                                  // contraction elements per wavefront (forward)

__device__ __forceinline__ f32x16_t mfma_bf16(const uint4& a, const uint4& b, f32x16_t c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
}

// Waits until *cnt >= target.  Thread 0 polls; returns true for the whole workgroup if the wait
// was abandoned (time limit or another workgroup's abort).  Contains two barriers.
__device__ __forceinline__ bool wait_counter(unsigned* cnt, unsigned target, unsigned* abort_word,
                                             unsigned long long limit_ticks, int* s_flag) {
    if (threadIdx.x == 0) {
        int bad = 0;
        const unsigned long long t0 = wall_clock64();
        unsigned it = 0;
        while (__hip_atomic_load(cnt, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target) {
            __builtin_amdgcn_s_sleep(1);
            if ((++it & 63u) == 0) {
                if (__hip_atomic_load(abort_word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) { bad = 1; break; }
                if (wall_clock64() - t0 > limit_ticks) {
                    __hip_atomic_store(abort_word, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    bad = 1;
                    break;
                }
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
        *s_flag = bad;
    }
    __syncthreads();
    const bool bad = *s_flag != 0;
    __syncthreads();
    return bad;
}

// After the workgroup's stores: make them visible at agent scope, then count this workgroup in.
__device__ __forceinline__ void signal_counter(unsigned* cnt) {
    __syncthreads();
    if (threadIdx.x == 0) __hip_atomic_fetch_add(cnt, 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
}

struct GroupMap { int d, u, bg, group; };

// Workgroups that exchange data sit on one XCD when ids are dealt round-robin over eight XCDs
// (a performance assumption only; correctness rests on the agent-scope ordering above).
__device__ __forceinline__ GroupMap map_block(int NU, int nbg) {
    const int ngroups = 2 * nbg;
    const int x = blockIdx.x;
    int group, u;
    if ((ngroups & 7) == 0) {
        const int slot = x >> 3;
        group = (x & 7) + 8 * (slot / NU);
        u = slot % NU;
    } else {
        group = x / NU;
        u = x % NU;
    }
    GroupMap m;
    m.group = group; m.u = u; m.d = group / nbg; m.bg = group % nbg;
    return m;
}

// ------------------------------------------------------------------------------ forward
template <int NW>
__global__ __launch_bounds__(64 * NW) void rec_fwd_kernel(RecFwdArgs a) {
    constexpr int EPT = 16 / NW;                         // accumulator registers (batch rows) per thread
    constexpr int KSTEPS = KW / 16;                      // MFMA steps per gate per wavefront
    extern __shared__ float lds[];                       // [NW][4][4][64][4] partial accumulators
    __shared__ int s_flag;
    const int H = a.H, B = a.B, T = a.T;
    const int NU = H / 32;
    const GroupMap gm = map_block(NU, a.nbg);
    const int d = gm.d, u = gm.u;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l32 = lane & 31, lh = lane >> 5;

    // this wavefront's slice of U_h as B-fragments: unit row l32 of each gate, 8 consecutive k per lane
    uint4 bfrag[4][KSTEPS];
    {
        const bf16_t* uh = a.uh[d];
#pragma unroll
        for (int g = 0; g < 4; ++g)
#pragma unroll
            for (int q = 0; q < KSTEPS; ++q)
                bfrag[g][q] = *reinterpret_cast<const uint4*>(uh + (size_t)(g * H + u * 32 + l32) * H + wave * KW + q * 16 + 8 * lh);
    }
    unsigned* cnt = a.cnt + (size_t)gm.group * a.tiles_per_group;
    const int j = u * 32 + l32;                          // this thread's hidden unit
    bool dead = false;

    for (int n = 0; n < T && !dead; ++n) {
        const int t = d ? T - 1 - n : n;
        const int tp = d ? T - n : n - 1;
        for (int i = 0; i < a.tiles_per_group; ++i) {
            const int b0 = (gm.bg * a.tiles_per_group + i) * 32;
            if (b0 >= B) break;
            // this thread's EPT batch rows: accumulator register r = EPT*wave + e
            float ax[EPT][4], cp[EPT];
#pragma unroll
            for (int e = 0; e < EPT; ++e) {
                const int r = EPT * wave + e;
                const int b = b0 + 8 * (r >> 2) + 4 * lh + (r & 3);
                const bool ok = b < B;
                const float* p = a.ax + ((size_t)t * B + (ok ? b : 0)) * 8 * H + (size_t)d * 4 * H + j;
#pragma unroll
                for (int g = 0; g < 4; ++g) ax[e][g] = ok ? p[(size_t)g * H] : 0.0f;
                cp[e] = (ok && n > 0) ? a.c[((size_t)tp * B + b) * 2 * H + (size_t)d * H + j] : 0.0f;
            }
            float sum[EPT][4];
#pragma unroll
            for (int e = 0; e < EPT; ++e)
#pragma unroll
                for (int g = 0; g < 4; ++g) sum[e][g] = 0.0f;
            if (n > 0) {
                if (wait_counter(cnt + i, (unsigned)(NU * n), a.abort_word, a.limit_ticks, &s_flag)) { dead = true; break; }
                // previous h of this batch tile: row l32, 8 consecutive k per lane
                const int row = b0 + l32;
                const bf16_t* hp = a.y + ((size_t)tp * B + (row < B ? row : 0)) * 2 * H + (size_t)d * H + wave * KW + 8 * lh;
                uint4 afrag[KSTEPS];
#pragma unroll
                for (int q = 0; q < KSTEPS; ++q)
                    afrag[q] = row < B ? *reinterpret_cast<const uint4*>(hp + q * 16) : make_uint4(0, 0, 0, 0);
                f32x16_t acc[4];
#pragma unroll
                for (int g = 0; g < 4; ++g)
#pragma unroll
                    for (int e = 0; e < 16; ++e) acc[g][e] = 0.0f;
#pragma unroll
                for (int q = 0; q < KSTEPS; ++q)
#pragma unroll
                    for (int g = 0; g < 4; ++g) acc[g] = mfma_bf16(afrag[q], bfrag[g][q], acc[g]);
                // partial accumulators -> LDS as [wave][gate][reg/4][lane][reg%4]
                float4* l4 = reinterpret_cast<float4*>(lds);
#pragma unroll
                for (int g = 0; g < 4; ++g)
#pragma unroll
                    for (int rq = 0; rq < 4; ++rq)
                        l4[((wave * 4 + g) * 4 + rq) * 64 + lane] =
                            make_float4(acc[g][4 * rq], acc[g][4 * rq + 1], acc[g][4 * rq + 2], acc[g][4 * rq + 3]);
                __syncthreads();
#pragma unroll
                for (int w2 = 0; w2 < NW; ++w2)
#pragma unroll
                    for (int g = 0; g < 4; ++g)
#pragma unroll
                        for (int e = 0; e < EPT; ++e) {
                            const int r = EPT * wave + e;
                            sum[e][g] += lds[((((w2 * 4 + g) * 4 + (r >> 2)) * 64 + lane) << 2) + (r & 3)];
                        }
            }
#pragma unroll
            for (int e = 0; e < EPT; ++e) {
                const int r = EPT * wave + e;
                const int b = b0 + 8 * (r >> 2) + 4 * lh + (r & 3);
                if (b < B) {
                    const float gi = sigmoidf_(ax[e][0] + sum[e][0]);
                    const float gf = sigmoidf_(ax[e][1] + sum[e][1]);
                    const float gg = tanhf_(ax[e][2] + sum[e][2]);
                    const float go = sigmoidf_(ax[e][3] + sum[e][3]);
                    const float c = gf * cp[e] + gi * gg;
                    const float h = go * tanhf_(c);
                    const size_t m = (size_t)t * B + b;
                    a.c[m * 2 * H + (size_t)d * H + j] = c;
                    bf16_t* gp = a.gates + m * 8 * H + (size_t)d * 4 * H + j;
                    gp[0] = f2bf(gi); gp[(size_t)H] = f2bf(gf); gp[(size_t)2 * H] = f2bf(gg); gp[(size_t)3 * H] = f2bf(go);
                    a.y[m * 2 * H + (size_t)d * H + j] = f2bf(h);
                }
            }
            signal_counter(cnt + i);                     // also the barrier that frees the LDS buffer
        }
    }
}

// ------------------------------------------------------------------------------ backward
template <int NW>
__global__ __launch_bounds__(64 * NW) void rec_bwd_kernel(RecBwdArgs a) {
    constexpr int EPT = 16 / NW;
    constexpr int KSTEPS = 4 * KW / 16;                  // the contraction runs over the 4H gate rows
    extern __shared__ float lds[];                       // [NW][4][64][4]
    __shared__ int s_flag;
    const int H = a.H, B = a.B, T = a.T;
    const int NU = H / 32;
    const GroupMap gm = map_block(NU, a.nbg);
    const int d = gm.d, u = gm.u;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l32 = lane & 31, lh = lane >> 5;
    const int KWB = 4 * H / NW;                          // gate rows per wavefront (= 4 * KW)

    // U_h^T slice: output unit l32, 8 consecutive gate rows per lane
    uint4 bfrag[KSTEPS];
    {
        const bf16_t* uht = a.uht[d];
#pragma unroll
        for (int q = 0; q < KSTEPS; ++q)
            bfrag[q] = *reinterpret_cast<const uint4*>(uht + (size_t)(u * 32 + l32) * 4 * H + wave * KWB + q * 16 + 8 * lh);
    }
    unsigned* cnt = a.cnt + (size_t)gm.group * a.tiles_per_group;
    const int j = u * 32 + l32;
    bool dead = false;

    for (int n = T - 1; n >= 0 && !dead; --n) {
        const int t = d ? T - 1 - n : n;
        const int tp = d ? T - n : n - 1;                // frame visited before t (its c is c_prev)
        const int tn = d ? T - 2 - n : n + 1;            // frame visited after t (its da feeds dh)
        for (int i = 0; i < a.tiles_per_group; ++i) {
            const int b0 = (gm.bg * a.tiles_per_group + i) * 32;
            if (b0 >= B) break;
            float dh[EPT], gi[EPT], gf[EPT], gg[EPT], go[EPT], cc[EPT], cp[EPT], dcr[EPT];
#pragma unroll
            for (int e = 0; e < EPT; ++e) {
                const int r = EPT * wave + e;
                const int b = b0 + 8 * (r >> 2) + 4 * lh + (r & 3);
                const bool ok = b < B;
                const size_t m = (size_t)t * B + (ok ? b : 0);
                const bf16_t* gp = a.gates + m * 8 * H + (size_t)d * 4 * H + j;
                gi[e] = ok ? bf2f(gp[0]) : 0.0f; gf[e] = ok ? bf2f(gp[(size_t)H]) : 0.0f;
                gg[e] = ok ? bf2f(gp[(size_t)2 * H]) : 0.0f; go[e] = ok ? bf2f(gp[(size_t)3 * H]) : 0.0f;
                cc[e] = ok ? a.c[m * 2 * H + (size_t)d * H + j] : 0.0f;
                cp[e] = (ok && n > 0) ? a.c[((size_t)tp * B + b) * 2 * H + (size_t)d * H + j] : 0.0f;
                dh[e] = ok ? bf2f(a.dy[m * 2 * H + (size_t)d * H + j]) : 0.0f;
                dcr[e] = (ok && n < T - 1) ? a.dc[((size_t)d * B + b) * H + j] : 0.0f;
            }
            if (n < T - 1) {
                if (wait_counter(cnt + i, (unsigned)(NU * (T - 1 - n)), a.abort_word, a.limit_ticks, &s_flag)) { dead = true; break; }
                const int row = b0 + l32;
                const bf16_t* ap = a.da + ((size_t)tn * B + (row < B ? row : 0)) * 8 * H + (size_t)d * 4 * H + wave * KWB + 8 * lh;
                f32x16_t acc;
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[e] = 0.0f;
#pragma unroll
                for (int q0 = 0; q0 < KSTEPS; q0 += 8) {
                    uint4 afrag[8];
#pragma unroll
                    for (int q = 0; q < 8; ++q)
                        afrag[q] = row < B ? *reinterpret_cast<const uint4*>(ap + (q0 + q) * 16) : make_uint4(0, 0, 0, 0);
#pragma unroll
                    for (int q = 0; q < 8; ++q) acc = mfma_bf16(afrag[q], bfrag[q0 + q], acc);
                }
                float4* l4 = reinterpret_cast<float4*>(lds);
#pragma unroll
                for (int rq = 0; rq < 4; ++rq)
                    l4[(wave * 4 + rq) * 64 + lane] = make_float4(acc[4 * rq], acc[4 * rq + 1], acc[4 * rq + 2], acc[4 * rq + 3]);
                __syncthreads();
#pragma unroll
                for (int w2 = 0; w2 < NW; ++w2)
#pragma unroll
                    for (int e = 0; e < EPT; ++e) {
                        const int r = EPT * wave + e;
                        dh[e] += lds[(((w2 * 4 + (r >> 2)) * 64 + lane) << 2) + (r & 3)];
                    }
            }
#pragma unroll
            for (int e = 0; e < EPT; ++e) {
                const int r = EPT * wave + e;
                const int b = b0 + 8 * (r >> 2) + 4 * lh + (r & 3);
                if (b < B) {
                    const float tc = tanhf_(cc[e]);
                    const float dc = dh[e] * go[e] * (1.0f - tc * tc) + dcr[e];
                    const float da_o = dh[e] * tc * go[e] * (1.0f - go[e]);
                    const float da_i = dc * gg[e] * gi[e] * (1.0f - gi[e]);
                    const float da_f = dc * cp[e] * gf[e] * (1.0f - gf[e]);
                    const float da_g = dc * gi[e] * (1.0f - gg[e] * gg[e]);
                    a.dc[((size_t)d * B + b) * H + j] = dc * gf[e];
                    bf16_t* dp = a.da + ((size_t)t * B + b) * 8 * H + (size_t)d * 4 * H + j;
                    dp[0] = f2bf(da_i); dp[(size_t)H] = f2bf(da_f); dp[(size_t)2 * H] = f2bf(da_g); dp[(size_t)3 * H] = f2bf(da_o);
                }
            }
            signal_counter(cnt + i);
        }
    }
}

// U_h [4H][H] -> U_h^T [H][4H], 32x32 tiles through LDS; blockIdx.z = direction.
__global__ __launch_bounds__(256) void transpose_uh_kernel(const bf16_t* src0, const bf16_t* src1, bf16_t* dst0, bf16_t* dst1, int H) {
    __shared__ bf16_t tile[32][33];
    const bf16_t* src = blockIdx.z ? src1 : src0;
    bf16_t* dst = blockIdx.z ? dst1 : dst0;
    const int r0 = blockIdx.y * 32, c0 = blockIdx.x * 32;     // rows of U_h (4H), columns (H)
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    for (int rr = ty; rr < 32; rr += 8) tile[rr][tx] = src[(size_t)(r0 + rr) * H + c0 + tx];
    __syncthreads();
    for (int rr = ty; rr < 32; rr += 8) dst[(size_t)(c0 + rr) * 4 * H + r0 + tx] = tile[tx][rr];
}

__global__ void fill_u32_kernel(unsigned* p, int n, unsigned v) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

template <typename K>
hipError_t prepare(K kernel, int threads, size_t dyn_lds, int grid, bool* fits) {
    static thread_local int cus = 0;
    if (cus == 0) {
        int dev = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e != hipSuccess) return e;
        e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
        if (e != hipSuccess) return e;
    }
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)dyn_lds);
    if (e != hipSuccess) return e;
    int per_cu = 0;
    e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, threads, dyn_lds);
    if (e != hipSuccess) return e;
    *fits = (long long)per_cu * cus >= grid;
    return hipSuccess;
}

}  // namespace

int rec_waves_for(int H) {
    if (H % KW != 0) return 0;
    const int nw = H / KW;
    return (nw == 1 || nw == 2 || nw == 4) ? nw : 0;
}

hipError_t launch_fill_u32(unsigned* p, int n, unsigned v, hipStream_t st) {
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(fill_u32_kernel, dim3((n + 255) / 256), dim3(256), 0, st, p, n, v);
    return hipGetLastError();
}

hipError_t launch_transpose_uh(const unsigned short* src0, const unsigned short* src1, unsigned short* dst0,
                               unsigned short* dst1, int H, hipStream_t st) {
    hipLaunchKernelGGL(transpose_uh_kernel, dim3(H / 32, 4 * H / 32, 2), dim3(256), 0, st, src0, src1, dst0, dst1, H);
    return hipGetLastError();
}

hipError_t launch_rec_fwd(const RecFwdArgs& a, hipStream_t st, bool* launched) {
    *launched = false;
    const int nw = rec_waves_for(a.H);
    if (nw == 0) return hipSuccess;
    const int grid = 2 * a.nbg * (a.H / 32);
    const size_t lds = (size_t)nw * 4 * 4 * 64 * 16;
    bool fits = false;
    hipError_t e;
#define BLSTM_REC_CASE(NWV)                                                                         \
    case NWV:                                                                                       \
        e = prepare(rec_fwd_kernel<NWV>, 64 * NWV, lds, grid, &fits);                               \
        if (e != hipSuccess || !fits) return e;                                                     \
        hipLaunchKernelGGL(rec_fwd_kernel<NWV>, dim3(grid), dim3(64 * NWV), lds, st, a);            \
        break;
    switch (nw) {
        BLSTM_REC_CASE(1) BLSTM_REC_CASE(2) BLSTM_REC_CASE(4)
        default: return hipSuccess;
    }
#undef BLSTM_REC_CASE
    *launched = true;
    return hipGetLastError();
}

hipError_t launch_rec_bwd(const RecBwdArgs& a, hipStream_t st, bool* launched) {
    *launched = false;
    const int nw = rec_waves_for(a.H);
    if (nw == 0) return hipSuccess;
    const int grid = 2 * a.nbg * (a.H / 32);
    const size_t lds = (size_t)nw * 4 * 64 * 16;
    bool fits = false;
    hipError_t e;
#define BLSTM_REC_CASE(NWV)                                                                         \
    case NWV:                                                                                       \
        e = prepare(rec_bwd_kernel<NWV>, 64 * NWV, lds, grid, &fits);                               \
        if (e != hipSuccess || !fits) return e;                                                     \
        hipLaunchKernelGGL(rec_bwd_kernel<NWV>, dim3(grid), dim3(64 * NWV), lds, st, a);            \
        break;
    switch (nw) {
        BLSTM_REC_CASE(1) BLSTM_REC_CASE(2) BLSTM_REC_CASE(4)
        default: return hipSuccess;
    }
#undef BLSTM_REC_CASE
    *launched = true;
    return hipGetLastError();
}

}  // namespace blstm
