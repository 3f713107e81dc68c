// C(m,n) = sum_k A(m,k) B(n,k) (+ bias[n]) (+ add[m][n]) on the matrix cores of gfx950.
//
// One workgroup of four wavefronts owns a 128x128 tile of C; each wavefront owns a
// 64x64 quarter as 2x2 MFMA 32x32 accumulators.  A K-slab of eight 16-byte chunks per
// row (64 bf16 or 32 float) is staged through LDS, double buffered, with the next
// slab's global loads in flight while the current one is multiplied.  Operands whose
// contraction index is the slow one in memory ("transposed") are loaded along their
// fast index and transposed in registers on the way to LDS, so all three forms of a
// training step's products (X W^T, dA W, dA^T X) run through the same inner loop.
// LDS rows are XOR-swizzled at chunk granularity so that both the row-wise stores and
// the MFMA fragment reads spread over the banks.
#include "common.hpp"
#include "gemm.hpp"

namespace blstm {
namespace {

constexpr int BM = 128, BN = 128, NTHREADS = 256;
constexpr int CHUNKS = 8;                       // 16-byte chunks per LDS row and K-slab

template <typename T> struct Vec { };
template <> struct Vec<float>  { static constexpr int N = 4; };
template <> struct Vec<bf16_t> { static constexpr int N = 8; };

__device__ __forceinline__ int swz(int row) { return ((row >> 2) ^ row) & 7; }

struct Operand {
    const void* p;
    long long ld;
    int rows;       // extent of the non-contracted index (M for A, N for B)
    int fast;       // bit 0: the widest vector load is legal; bit 1: 8-byte loads are legal (bf16, K fast)
};

struct Params {
    Operand A[2], B[2];
    int K[2];
    int nseg;
    void* C; long long ldc;
    const void* bias;               // element type of the inputs
    const float* add; long long ldadd;
    float* rowsum;                  // rowsum[m] = sum_k A(m,k) over segment 0, or null
    int M, N, ntm, ntn;
    long long sA[2], sB[2], sC, sBias, sAdd, sRowsum;
};

// ---- guarded element-wise fallbacks ------------------------------------------------
// 16-bit elements, NE of them, packed two per word
template <typename T, int NE>
__device__ __forceinline__ void load_elems(uint32_t* out, const T* p, int nvalid) {
    static_assert(sizeof(T) == 2, "generic form is for 16-bit elements");
    T tmp[NE];
#pragma unroll
    for (int e = 0; e < NE; ++e) tmp[e] = (e < nvalid) ? p[e] : (T)0;
    constexpr int W = NE * sizeof(T) / 4;
#pragma unroll
    for (int w = 0; w < W; ++w)
        out[w] = (uint32_t)(unsigned short)tmp[2 * w] | ((uint32_t)(unsigned short)tmp[2 * w + 1] << 16);
}
template <>
__device__ __forceinline__ void load_elems<float, 4>(uint32_t* out, const float* p, int nvalid) {
#pragma unroll
    for (int e = 0; e < 4; ++e) out[e] = (e < nvalid) ? __builtin_bit_cast(uint32_t, p[e]) : 0u;
}

// ---- global -> registers ---------------------------------------------------------
// K is the fast index in memory: thread owns chunks c = tid + 256 i, row = c / 8, chunk = c % 8.
template <typename T>
__device__ __forceinline__ void gload_kfast(uint4 (&r)[4], const Operand& op, int row0, int K, int k0, int tid) {
    constexpr int VEC = Vec<T>::N;
    const T* base = static_cast<const T*>(op.p);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int c = tid + NTHREADS * i;
        int row = row0 + (c >> 3);
        int k = k0 + (c & 7) * VEC;
        uint32_t w[4] = {0u, 0u, 0u, 0u};
        if (row < op.rows && k < K) {
            const T* p = base + (long long)row * op.ld + k;
            if ((op.fast & 1) && k + VEC <= K) {
                uint4 v = *reinterpret_cast<const uint4*>(p);
                w[0] = v.x; w[1] = v.y; w[2] = v.z; w[3] = v.w;
            } else if (sizeof(T) == 2 && (op.fast & 2)) {
                if (k + 4 <= K) { uint2 v = *reinterpret_cast<const uint2*>(p); w[0] = v.x; w[1] = v.y; }
                else load_elems<T, 4>(&w[0], p, K - k);
                if (k + 8 <= K) { uint2 v = *reinterpret_cast<const uint2*>(p + 4); w[2] = v.x; w[3] = v.y; }
                else if (k + 4 < K) load_elems<T, 4>(&w[2], p + 4, K - k - 4);
            } else {
                load_elems<T, VEC>(w, p, K - k);
            }
        }
        r[i] = make_uint4(w[0], w[1], w[2], w[3]);
    }
}

// The non-contracted index is the fast one in memory.  Thread owns rows rq*4..rq*4+3
// (rq = tid % 32) and the K-chunk tid / 32: VEC loads of four consecutive rows each.
template <typename T>
__device__ __forceinline__ void gload_rowfast(uint4 (&r)[4], const Operand& op, int row0, int K, int k0, int tid) {
    constexpr int VEC = Vec<T>::N;
    const T* base = static_cast<const T*>(op.p);
    const int row = row0 + (tid & 31) * 4;
    const int kb = k0 + (tid >> 5) * VEC;
    uint32_t w[16];
#pragma unroll
    for (int i = 0; i < VEC; ++i) {
        constexpr int WPL = 16 / VEC;                    // 32-bit words per load: 4 (float) or 2 (bf16)
        uint32_t* o = &w[i * WPL];
#pragma unroll
        for (int q = 0; q < WPL; ++q) o[q] = 0u;
        int k = kb + i;
        if (k < K && row < op.rows) {
            const T* p = base + (long long)k * op.ld + row;
            if ((op.fast & 1) && row + 4 <= op.rows) {
                if (sizeof(T) == 4) { uint4 v = *reinterpret_cast<const uint4*>(p); o[0] = v.x; o[1] = v.y; o[2] = v.z; o[3] = v.w; }
                else { uint2 v = *reinterpret_cast<const uint2*>(p); o[0] = v.x; o[1] = v.y; }
            } else {
                load_elems<T, 4>(o, p, op.rows - row);
            }
        }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) r[i] = make_uint4(w[4 * i], w[4 * i + 1], w[4 * i + 2], w[4 * i + 3]);
}

// ---- registers -> LDS -------------------------------------------------------------
__device__ __forceinline__ void sstore_kfast(uint4* s, const uint4 (&r)[4], int tid) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int c = tid + NTHREADS * i;
        int row = c >> 3;
        s[row * CHUNKS + ((c & 7) ^ swz(row))] = r[i];
    }
}

template <typename T>
__device__ __forceinline__ void sstore_rowfast(uint4* s, const uint4 (&r)[4], int tid) {
    const int rq = tid & 31, kc = tid >> 5;
    if (sizeof(T) == 4) {
        // r[i] = rows 0..3 at k = i  ->  chunk of row j = (r[0][j], r[1][j], r[2][j], r[3][j])
        const uint32_t a[4][4] = {{r[0].x, r[0].y, r[0].z, r[0].w}, {r[1].x, r[1].y, r[1].z, r[1].w},
                                  {r[2].x, r[2].y, r[2].z, r[2].w}, {r[3].x, r[3].y, r[3].z, r[3].w}};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            int row = rq * 4 + j;
            s[row * CHUNKS + (kc ^ swz(row))] = make_uint4(a[0][j], a[1][j], a[2][j], a[3][j]);
        }
    } else {
        // load i (k = i) holds rows 0..3 as two words: L[i][0] = rows 0,1 ; L[i][1] = rows 2,3
        const uint32_t L[8][2] = {{r[0].x, r[0].y}, {r[0].z, r[0].w}, {r[1].x, r[1].y}, {r[1].z, r[1].w},
                                  {r[2].x, r[2].y}, {r[2].z, r[2].w}, {r[3].x, r[3].y}, {r[3].z, r[3].w}};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            uint32_t w[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                uint32_t lo = L[2 * q][j >> 1], hi = L[2 * q + 1][j >> 1];
                // pick the 16-bit half (j & 1) of both words: result = half(lo) | half(hi) << 16
                w[q] = (j & 1) ? __builtin_amdgcn_perm(hi, lo, 0x07060302u)
                               : __builtin_amdgcn_perm(hi, lo, 0x05040100u);
            }
            int row = rq * 4 + j;
            s[row * CHUNKS + (kc ^ swz(row))] = make_uint4(w[0], w[1], w[2], w[3]);
        }
    }
}

// ---- one pair of chunks through the matrix cores ----------------------------------------
template <typename T>
__device__ __forceinline__ void mma(f32x16_t& acc, const uint4& a, const uint4& b) {
    if (sizeof(T) == 2) {
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b),
                                                      acc, 0, 0, 0);
    } else {
        // lanes 0..31 carry chunk 2q, lanes 32..63 chunk 2q+1; word e of both goes into one 32x32x2 product
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__builtin_bit_cast(float, a.x), __builtin_bit_cast(float, b.x), acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__builtin_bit_cast(float, a.y), __builtin_bit_cast(float, b.y), acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__builtin_bit_cast(float, a.z), __builtin_bit_cast(float, b.z), acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__builtin_bit_cast(float, a.w), __builtin_bit_cast(float, b.w), acc, 0, 0, 0);
    }
}

template <typename TI, typename TO, bool AT, bool BT>
__global__ __launch_bounds__(NTHREADS) void gemm_kernel(Params P) {
    constexpr int VEC = Vec<TI>::N;
    constexpr int BK = CHUNKS * VEC;
    __shared__ uint4 sA[2][BM * CHUNKS];
    __shared__ uint4 sB[2][BN * CHUNKS];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;

    // Workgroup ids are dealt round-robin to the eight XCDs; give each XCD a contiguous
    // range of tiles so that its L2 sees neighbouring tiles, then walk the range in bands
    // of eight tile rows so that concurrently resident tiles share A rows and B columns.
    const int nt = P.ntm * P.ntn;
    int lin = blockIdx.x;
    {
        const int nt8 = nt & ~7;
        if (lin < nt8) lin = (lin & 7) * (nt8 >> 3) + (lin >> 3);
    }
    const int band = 8 * P.ntn;
    const int first_m = (lin / band) * 8;
    const int bh = min(P.ntm - first_m, 8);
    const int tm = first_m + (lin % band) % bh;
    const int tn = (lin % band) / bh;
    const int row0 = tm * BM, col0 = tn * BN;
    const int z = blockIdx.z;

    f32x16_t acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    // Row sums of A ride along as one more product against a fragment of ones; only the
    // workgroups of the first tile column, and in them the waves of the first half, do it.
    const bool do_rs = P.rowsum != nullptr && tn == 0 && wn == 0;
    f32x16_t rs[2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) rs[i][e] = 0.0f;
    const uint32_t one_w = sizeof(TI) == 2 ? 0x3F803F80u : 0x3F800000u;
    const uint4 ones = make_uint4(one_w, one_w, one_w, one_w);

    int ntiles[2];
    ntiles[0] = (P.K[0] + BK - 1) / BK;
    ntiles[1] = P.nseg > 1 ? (P.K[1] + BK - 1) / BK : 0;
    const int total = ntiles[0] + ntiles[1];

    Operand opA[2], opB[2];
#pragma unroll
    for (int s = 0; s < 2; ++s) {
        opA[s] = P.A[s]; opB[s] = P.B[s];
        opA[s].p = static_cast<const TI*>(P.A[s].p) + z * P.sA[s];
        opB[s].p = static_cast<const TI*>(P.B[s].p) + z * P.sB[s];
    }

    uint4 ra[4], rb[4];
    auto gload = [&](int it) {
        const int s = (it >= ntiles[0]) ? 1 : 0;
        const int k0 = (it - (s ? ntiles[0] : 0)) * BK;
        if (AT) gload_rowfast<TI>(ra, opA[s], row0, P.K[s], k0, tid);
        else    gload_kfast<TI>(ra, opA[s], row0, P.K[s], k0, tid);
        if (BT) gload_rowfast<TI>(rb, opB[s], col0, P.K[s], k0, tid);
        else    gload_kfast<TI>(rb, opB[s], col0, P.K[s], k0, tid);
    };
    auto sstore = [&](int buf) {
        if (AT) sstore_rowfast<TI>(sA[buf], ra, tid); else sstore_kfast(sA[buf], ra, tid);
        if (BT) sstore_rowfast<TI>(sB[buf], rb, tid); else sstore_kfast(sB[buf], rb, tid);
    };

    if (total > 0) {
        gload(0);
        sstore(0);
    }
    __syncthreads();
    for (int it = 0; it < total; ++it) {
        const int buf = it & 1;
        if (it + 1 < total) gload(it + 1);
        const uint4* a_s = sA[buf];
        const uint4* b_s = sB[buf];
#pragma unroll
        for (int q = 0; q < CHUNKS / 2; ++q) {
            const int kc = 2 * q + (lane >> 5);
            uint4 af[2], bfr[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                int ar = wm * 64 + i * 32 + (lane & 31);
                af[i] = a_s[ar * CHUNKS + (kc ^ swz(ar))];
                int br = wn * 64 + i * 32 + (lane & 31);
                bfr[i] = b_s[br * CHUNKS + (kc ^ swz(br))];
            }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j) mma<TI>(acc[i][j], af[i], bfr[j]);
            if (do_rs && it < ntiles[0]) {
#pragma unroll
                for (int i = 0; i < 2; ++i) mma<TI>(rs[i], af[i], ones);
            }
        }
        if (it + 1 < total) sstore(buf ^ 1);
        __syncthreads();
    }

    if (do_rs && (lane & 31) == 0) {
        float* out = P.rowsum + z * P.sRowsum;
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int row = row0 + wm * 64 + i * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
                if (row < P.M) out[row] = rs[i][e];
            }
    }

    // Epilogue: accumulator register e of lane l is row 8*(e/4) + 4*(l/32) + e%4, column l%32.
    TO* C = static_cast<TO*>(P.C) + z * P.sC;
    const TI* bias = P.bias ? static_cast<const TI*>(P.bias) + z * P.sBias : nullptr;
    const float* add = P.add ? P.add + z * P.sAdd : nullptr;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int col = col0 + wn * 64 + j * 32 + (lane & 31);
            if (col >= P.N) continue;
            const float bv = bias ? ld_f(bias + col) : 0.0f;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int row = row0 + wm * 64 + i * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
                if (row < P.M) {
                    float v = acc[i][j][e] + bv;
                    if (add) v += add[(long long)row * P.ldadd + col];
                    st_f(&C[(long long)row * P.ldc + col], v);
                }
            }
        }
}

inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

template <typename TI>
int fast_flags(const void* p, long long ld, long long stride, int batch, bool rowfast) {
    const long long es = sizeof(TI);
    if (batch <= 1) stride = 0;
    int f = 0;
    if (!rowfast) {
        if (aligned(p, 16) && (ld * es) % 16 == 0 && (stride * es) % 16 == 0) f |= 1;
        if (es == 2 && aligned(p, 8) && (ld * es) % 8 == 0 && (stride * es) % 8 == 0) f |= 2;
    } else {
        const long long w = 4 * es;                       // four consecutive rows per load
        if (aligned(p, w) && (ld * es) % w == 0 && (stride * es) % w == 0) f |= 1;
    }
    return f;
}

template <typename TI, typename TO>
hipError_t dispatch(const GemmDesc& d, hipStream_t stream) {
    Params P{};
    P.nseg = d.nseg;
    for (int s = 0; s < d.nseg; ++s) {
        const GemmSeg& g = d.seg[s];
        P.A[s] = Operand{g.A, g.lda, d.M, fast_flags<TI>(g.A, g.lda, g.sA, d.batch, d.atrans)};
        P.B[s] = Operand{g.B, g.ldb, d.N, fast_flags<TI>(g.B, g.ldb, g.sB, d.batch, d.btrans)};
        P.K[s] = g.K; P.sA[s] = g.sA; P.sB[s] = g.sB;
    }
    P.C = d.C; P.ldc = d.ldc; P.sC = d.sC;
    P.bias = d.bias; P.sBias = d.sBias;
    P.add = d.add; P.ldadd = d.ldadd; P.sAdd = d.sAdd;
    P.rowsum = d.rowsum; P.sRowsum = d.sRowsum;
    P.M = d.M; P.N = d.N;
    P.ntm = (d.M + BM - 1) / BM; P.ntn = (d.N + BN - 1) / BN;
    dim3 grid((unsigned)(P.ntm * P.ntn), 1, (unsigned)(d.batch > 0 ? d.batch : 1));
    dim3 block(NTHREADS);
    if (!d.atrans && !d.btrans) hipLaunchKernelGGL((gemm_kernel<TI, TO, false, false>), grid, block, 0, stream, P);
    else if (!d.atrans && d.btrans) hipLaunchKernelGGL((gemm_kernel<TI, TO, false, true>), grid, block, 0, stream, P);
    else if (d.atrans && d.btrans) hipLaunchKernelGGL((gemm_kernel<TI, TO, true, true>), grid, block, 0, stream, P);
    else hipLaunchKernelGGL((gemm_kernel<TI, TO, true, false>), grid, block, 0, stream, P);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_gemm(const GemmDesc& d, hipStream_t stream) {
    if (d.M <= 0 || d.N <= 0) return hipSuccess;
    if (d.in_type == DT_F32 && d.out_type == DT_F32) return dispatch<float, float>(d, stream);
    if (d.in_type == DT_BF16 && d.out_type == DT_BF16) return dispatch<bf16_t, bf16_t>(d, stream);
    if (d.in_type == DT_BF16 && d.out_type == DT_F32) return dispatch<bf16_t, float>(d, stream);
    return hipErrorInvalidValue;
}

}  // namespace blstm
