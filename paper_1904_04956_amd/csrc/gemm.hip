// C(m,n) = sum_k A(m,k) B(n,k) (+ bias[n]) (+ add[m][n]) on the matrix cores of gfx950.
//
// A workgroup of 2 x WN wavefronts owns a (64 TM) x (32 TN WN) tile of C; each wavefront owns a
// (32 TM) x (32 TN) part as TM x TN MFMA 32x32 accumulators.  A K-slab of eight 16-byte chunks per
// row (64 bf16 or 32 float) lives in LDS, rows XOR-swizzled at chunk granularity so that loads,
// stores and the MFMA fragment reads all spread over the banks.  Operands whose contraction index
// is the slow one in memory ("transposed") are loaded along their fast index, so all three forms
// of a training step's products (X W^T, dA W, dA^T X) run through the same inner loop: 16-bit ones
// of full tiles lie in LDS as they lie in memory and are transposed by the LDS read itself
// (ds_read_b64_tr_b16); the others are transposed in registers on the way to LDS.
//
// Two ways of bringing a slab into LDS:
//   direct   bf16 operands, whole tiles, aligned: global_load_lds_dwordx4 writes the slab straight
//            into LDS in the swizzled layout (each lane fetches the chunk that belongs at its LDS
//            slot).  Tiles: 256x128 on four wavefronts with ONE LDS buffer, a slab's fragments all
//            read into registers before the next slab's loads overwrite it, two workgroups per CU
//            taking turns on the matrix cores (the workhorse: 3/4 of the operand bytes of 128x128
//            per flop, and the vector-memory path of a CU, about 45 bytes per clock from L2, is what
//            bounds these products); 128x128 with a ring of two or three buffers for products with
//            too few large tiles; 256x256 on eight wavefronts for a handful of tiles with a very
//            long contraction.
//   staged   every other case (float operands, ragged shapes, unaligned rows): global loads into
//            registers two or four slabs ahead, LDS stores, double-buffered LDS.
// Products with a small output and a long contraction are split along K over blockIdx.y into float
// partial tiles that a second kernel sums in a fixed order.  Several independent products of one
// form can share one launch (gemm_group_kernel).
#include "common.hpp"
#include "gemm.hpp"

namespace blstm {
namespace {

typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2_t __attribute__((ext_vector_type(2)));

constexpr int NTHREADS = 256;
constexpr int CHUNKS = 8;                       // 16-byte chunks per LDS row and K-slab

template <typename T> struct Vec { };
template <> struct Vec<float>  { static constexpr int N = 4; };
template <> struct Vec<bf16_t> { static constexpr int N = 8; };

// Chunk column of a row is XORed with swz(row).  Any eight consecutive rows (fragment reads), the rows
// 4l + j and 8l + j of eight consecutive l (the two row-fast store patterns) and one row's eight chunks
// (K-fast stores) all spread over the eight 16-byte columns.  Period 64 rows; swz(row + 32) = swz(row) ^ 4.
__device__ __forceinline__ int swz(int row) { return ((row >> 3) ^ row) & 7; }

struct Operand {
    const void* p;
    long long ld;
    int rows;       // extent of the non-contracted index (M for A, N for B)
    int fast;       // bit 0: the widest vector load is legal; bit 1: 8-byte loads are legal (bf16, K fast); bit 2: 16-byte loads of eight rows (bf16, row fast)
};

struct Params {
    Operand A[2], B[2];
    int K[2];
    int nseg;
    void* C; long long ldc;
    const void* bias;               // element type of the inputs
    const float* add; long long ldadd;
    float* rowsum;                  // rowsum[m] = sum_k A(m,k) over segment 0, or null
    float* partial;                 // split-K: float [batch][splits][M][N], or null
    float* rs_partial;              // split-K: float [batch][splits][M] row sums
    int M, N, ntm, ntn, splits;
    int c_vec;                      // C rows may be written with 16-byte (float) / 8-byte (bf16) stores, whole tiles of them
    int p_vec;                      // the same for the float partial tiles of a split
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
template <typename T, int NCH>
__device__ __forceinline__ void gload_kfast(uint4 (&r)[NCH], const Operand& op, int row0, int K, int k0, int tid) {
    constexpr int VEC = Vec<T>::N;
    const T* base = static_cast<const T*>(op.p);
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
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

// The non-contracted index is the fast one in memory.  Per pass of 128 rows a thread owns rows
// rq*4..rq*4+3 (rq = tid % 32) and the K-chunk tid / 32: VEC loads of four consecutive rows each.
template <typename T, int NCH>
__device__ __forceinline__ void gload_rowfast(uint4 (&r)[NCH], const Operand& op, int row0, int K, int k0, int tid) {
    constexpr int VEC = Vec<T>::N;
    const T* base = static_cast<const T*>(op.p);
    const int kb = k0 + (tid >> 5) * VEC;
#pragma unroll
    for (int pass = 0; pass < NCH / 4; ++pass) {
        const int row = row0 + pass * 128 + (tid & 31) * 4;
        uint32_t w[16];
#pragma unroll
        for (int i = 0; i < VEC; ++i) {
            constexpr int WPL = 16 / VEC;                // 32-bit words per load: 4 (float) or 2 (bf16)
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
        for (int i = 0; i < 4; ++i) r[pass * 4 + i] = make_uint4(w[4 * i], w[4 * i + 1], w[4 * i + 2], w[4 * i + 3]);
    }
}

// ---- unguarded forms: tile fully inside the matrices, K a multiple of the slab, aligned -------
// `base` is uniform (tile origin and slab applied, in bytes); `voff` is this thread's byte offset.
template <typename T, int NCH>
__device__ __forceinline__ void gload_kfast_fast(uint4 (&r)[NCH], const char* base, long long rowstep, uint32_t voff) {  // rowstep: bytes per pass of rows
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
        const u32x4_t v = *reinterpret_cast<const u32x4_t*>(base + i * rowstep + voff);
        r[i] = make_uint4(v[0], v[1], v[2], v[3]);
    }
}
template <typename T, int NCH, int PR>
__device__ __forceinline__ void gload_rowfast_fast(uint4 (&r)[NCH], const char* base, long long kstep, uint32_t voff) {
    constexpr int VEC = Vec<T>::N;
#pragma unroll
    for (int pass = 0; pass < NCH / 4; ++pass) {
        const char* pb = base + pass * PR * (int)sizeof(T) + voff;
        if (sizeof(T) == 4) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const u32x4_t v = *reinterpret_cast<const u32x4_t*>(pb + i * kstep);
                r[pass * 4 + i] = make_uint4(v[0], v[1], v[2], v[3]);
            }
        } else {
            u32x2_t w[VEC];
#pragma unroll
            for (int i = 0; i < VEC; ++i) w[i] = *reinterpret_cast<const u32x2_t*>(pb + i * kstep);
#pragma unroll
            for (int q = 0; q < 4; ++q) r[pass * 4 + q] = make_uint4(w[2 * q][0], w[2 * q][1], w[2 * q + 1][0], w[2 * q + 1][1]);
        }
    }
}

// 16-bit operands whose non-contracted index is the fast one in memory, unguarded: the slab
// stays in LDS as it lies in memory, [k][row] with 16-byte chunks of eight rows, and the LDS read that
// feeds the matrix cores transposes it (ds_read_b64_tr_b16: sixteen lanes read a 4 x 16 block of 16-bit
// elements, lane j of them receives column j).  No transposes in registers, plain 16-byte loads and stores.
// CPR = chunks per k-row.  A thread owns chunk tid % CPR of the k-rows tid / CPR + 16 i.
// Swizzle: the 32-byte pair of chunks p of k-row k sits at pair p ^ ((k & 3) << 1), so that the four k-rows
// a group of sixteen lanes reads, and the neighbouring group's, fall on different banks.
template <int NCH>
__device__ __forceinline__ void gload_tr(uint4 (&r)[NCH], const char* base, long long pass_step, uint32_t voff) {
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
        const u32x4_t v = *reinterpret_cast<const u32x4_t*>(base + voff + i * pass_step);
        r[i] = make_uint4(v[0], v[1], v[2], v[3]);
    }
}
template <int NCH, int CPR>
__device__ __forceinline__ void sstore_tr(uint4* s, const uint4 (&r)[NCH], int soff) {
#pragma unroll
    for (int i = 0; i < NCH; ++i) s[soff + i * 16 * CPR] = r[i];
}
typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) s16x4_t* lds_s16x4_ptr;
// eight consecutive k of one row: two transposing reads, k-rows kb .. kb+3 and kb+4 .. kb+7 (ROWB bytes per k-row)
template <int ROWB>
__device__ __forceinline__ uint4 lfrag_tr(const char* s, int kb) {
    const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(s + kb * ROWB));
    const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(s + (kb + 4) * ROWB));
    const uint2 l2 = __builtin_bit_cast(uint2, lo), h2 = __builtin_bit_cast(uint2, hi);
    return make_uint4(l2.x, l2.y, h2.x, h2.y);
}

// LDS stores through offsets computed once per thread (uint4 units): soff for the K-fast form,
// soffj[j] for row j of the four-row group of the row-fast form.
template <int NCH, int RP>
__device__ __forceinline__ void sstore_kfast_off(uint4* s, const uint4 (&r)[NCH], int soff) {
#pragma unroll
    for (int i = 0; i < NCH; ++i) s[(((i * RP) & 32) ? (soff ^ 4) : soff) + i * RP * CHUNKS] = r[i];   // swz(row + 32) = swz(row) ^ 4
}
template <typename T, int NCH, int PR>
__device__ __forceinline__ void sstore_rowfast_off(uint4* s, const uint4 (&r)[NCH], const int (&soffj)[4]) {
#pragma unroll
    for (int pass = 0; pass < NCH / 4; ++pass) {
        const uint4* rp = &r[pass * 4];
        if (sizeof(T) == 4) {
            const uint32_t a[4][4] = {{rp[0].x, rp[0].y, rp[0].z, rp[0].w}, {rp[1].x, rp[1].y, rp[1].z, rp[1].w},
                                      {rp[2].x, rp[2].y, rp[2].z, rp[2].w}, {rp[3].x, rp[3].y, rp[3].z, rp[3].w}};
#pragma unroll
            for (int j = 0; j < 4; ++j) s[soffj[j] + pass * PR * CHUNKS] = make_uint4(a[0][j], a[1][j], a[2][j], a[3][j]);
        } else {
            const uint32_t L[8][2] = {{rp[0].x, rp[0].y}, {rp[0].z, rp[0].w}, {rp[1].x, rp[1].y}, {rp[1].z, rp[1].w},
                                      {rp[2].x, rp[2].y}, {rp[2].z, rp[2].w}, {rp[3].x, rp[3].y}, {rp[3].z, rp[3].w}};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                uint32_t w[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    uint32_t lo = L[2 * q][j >> 1], hi = L[2 * q + 1][j >> 1];
                    w[q] = (j & 1) ? __builtin_amdgcn_perm(hi, lo, 0x07060302u) : __builtin_amdgcn_perm(hi, lo, 0x05040100u);
                }
                s[soffj[j] + pass * PR * CHUNKS] = make_uint4(w[0], w[1], w[2], w[3]);
            }
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

// D = sets of staging registers = slabs the global loads run ahead.  Two leaves room for two workgroups per
// CU; four is for launches with at most one workgroup per CU, which have nothing else to cover the
// latency of their loads with and the whole register file to themselves.
// NS = 0: slabs are staged through registers as described above (any element type, guarded or not).
// NS >= 1: direct mode, for 16-bit operands in the unguarded form.  The slabs go from global memory straight into LDS
// (global_load_lds_dwordx4: lane l of a wavefront writes its 16 bytes at the wave-uniform LDS address in M0 plus
// 16 l), in the same swizzled layouts the fragment reads expect: no staging registers, no LDS stores, no transposes
// in registers.  These loads are written in assembly and waited for with explicit vmcnt counts; the compiler does
// not see them.  NS >= 2: a ring of NS LDS buffers, the loads of slab it + NS - 1 issued at the top of iteration it,
// one barrier per slab.  NS = 1: one LDS buffer; all fragments of a slab are read into registers, a barrier frees the
// buffer for the next slab's loads, and the products run from registers while those loads are in flight; workgroups
// sharing a CU take turns on the matrix cores (one multiplies while another reads its fragments).
// `lin`, `split`, `z`: tile index within the product, K range and batch index of this workgroup; xcd_remap: lin is
// the workgroup id of a launch of this product alone and is still to be regrouped by XCD (below).
template <typename TI, typename TO, bool AT, bool BT, int TM, int TN, int WN, bool FAST, bool RS, int D, int NS>
__device__ __forceinline__ void gemm_tile(const Params& P, int lin, const int split, const int z, const bool xcd_remap) {
    static_assert(NS == 0 || (FAST && sizeof(TI) == 2 && D == 2), "direct mode is built for the unguarded 16-bit form");
    static_assert(D == 2 || (D == 4 && FAST && WN == 2), "the deep pipeline exists for the unguarded 128x128 tile only");
    static_assert(WN == 2 || (FAST && !RS), "the eight-wave shape exists in the unguarded form only");
    constexpr int NT = 128 * WN;                        // threads: 2 x WN wavefronts
    constexpr int VEC = Vec<TI>::N;
    constexpr int BK = CHUNKS * VEC;
    constexpr int BM = 64 * TM, BN = 32 * TN * WN;
    constexpr int RP = NT / 8;                          // rows one pass of K-fast loads covers
    constexpr int PR = NT / 2;                          // rows one pass of row-fast loads covers
    constexpr int NCA = BM * 8 / NT, NCB = BN * 8 / NT; // 16-byte chunks staged per thread and slab
    extern __shared__ uint4 smem[];                     // [2][(BM + BN) * CHUNKS]
    constexpr int STAGE = (BM + BN) * CHUNKS;           // 16-byte words per buffer: A rows, then B rows

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;

    // Workgroup ids are dealt round-robin to the eight XCDs; give each XCD a contiguous
    // range of tiles so that its L2 sees neighbouring tiles, then walk the range in bands
    // of eight tile rows so that concurrently resident tiles share A rows and B columns.
    const int nt = P.ntm * P.ntn;
    if (xcd_remap) {
        const int nt8 = nt & ~7;
        if (lin < nt8) lin = (lin & 7) * (nt8 >> 3) + (lin >> 3);
    }
    const int band = 8 * P.ntn;
    const int first_m = (lin / band) * 8;
    const int bh = min(P.ntm - first_m, 8);
    const int tm = first_m + (lin % band) % bh;
    const int tn = (lin % band) / bh;
    const int row0 = tm * BM, col0 = tn * BN;

    f32x16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    // Row sums of A ride along on the vector ALU, which the loop leaves mostly idle: the waves of the first
    // half of the workgroups of the first tile column add up the fragments they feed to the matrix cores
    // (a lane holds eight consecutive k of one row; lanes l and l + 32 hold the two halves of a sub-step).
    // (RS is instantiated for the 128x128 shape with both operands transposed only: the
    // weight-gradient products are the ones that need row sums.)
    constexpr int NRS = RS ? TM : 1;
    const bool do_rs = RS && P.rowsum != nullptr && tn == 0 && wn == 0;
    float rs[NRS];
#pragma unroll
    for (int i = 0; i < NRS; ++i) rs[i] = 0.0f;
    auto add_row = [](float acc, const uint4& f) {
        if constexpr (sizeof(TI) == 2) {
            typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
            const bf16x2_t one = __builtin_bit_cast(bf16x2_t, 0x3F803F80u);
            acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, f.x), one, acc, false);
            acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, f.y), one, acc, false);
            acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, f.z), one, acc, false);
            acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, f.w), one, acc, false);
        } else {
            acc += __builtin_bit_cast(float, f.x); acc += __builtin_bit_cast(float, f.y);
            acc += __builtin_bit_cast(float, f.z); acc += __builtin_bit_cast(float, f.w);
        }
        return acc;
    };

    int ntiles[2];
    ntiles[0] = (P.K[0] + BK - 1) / BK;
    ntiles[1] = P.nseg > 1 ? (P.K[1] + BK - 1) / BK : 0;
    int it_begin = 0, it_end = ntiles[0] + ntiles[1];
    if (P.splits > 1) {                                  // slabs [it_begin, it_end) of this split (one segment only)
        const int per = (ntiles[0] + P.splits - 1) / P.splits;
        it_begin = split * per;
        it_end = min(ntiles[0], it_begin + per);
        if (it_end < it_begin) it_end = it_begin;
    }

    // Segment operands as scalars selected per slab (indexing an array of structs at run time
    // would put it in scratch memory).
    Operand a0 = P.A[0], a1 = P.A[1], b0 = P.B[0], b1 = P.B[1];
    a0.p = static_cast<const TI*>(P.A[0].p) + z * P.sA[0];
    a1.p = static_cast<const TI*>(P.A[1].p) + z * P.sA[1];
    b0.p = static_cast<const TI*>(P.B[0].p) + z * P.sB[0];
    b1.p = static_cast<const TI*>(P.B[1].p) + z * P.sB[1];
    const int K0 = P.K[0], K1 = P.K[1];

    // per-thread LDS offsets (uint4 units), computed once
    const int soff_k = (tid >> 3) * CHUNKS + ((tid & 7) ^ swz(tid >> 3));
    int soff_r[4];
    const int rsub = (tid >> 8) * 128 + (tid & 31) * 4;   // row-fast form: first of this thread's four rows in a pass
    const int kch = (tid >> 5) & 7;                        // ... and its K chunk
#pragma unroll
    for (int j = 0; j < 4; ++j) { const int r = rsub + j; soff_r[j] = r * CHUNKS + (kch ^ swz(r)); }
    const int arow = wm * (32 * TM) + (lane & 31);
    const int brow = wn * (32 * TN) + (lane & 31);
    int roff_a[CHUNKS / 2], roff_b[CHUNKS / 2];
#pragma unroll
    for (int q = 0; q < CHUNKS / 2; ++q) {
        roff_a[q] = arow * CHUNKS + ((2 * q + (lane >> 5)) ^ swz(arow));
        roff_b[q] = brow * CHUNKS + ((2 * q + (lane >> 5)) ^ swz(brow));
    }
    // per-thread global byte offsets of the unguarded loads
    constexpr int ES = (int)sizeof(TI);
    const uint32_t voff_a = AT ? (uint32_t)(kch * VEC * a0.ld * ES + rsub * ES)
                               : (uint32_t)((tid >> 3) * a0.ld * ES + (tid & 7) * 16);
    const uint32_t voff_b = BT ? (uint32_t)(kch * VEC * b0.ld * ES + rsub * ES)
                               : (uint32_t)((tid >> 3) * b0.ld * ES + (tid & 7) * 16);

    // transposing-read form (16-bit, unguarded): per-thread store offset, load offset, and the byte offsets of the
    // fragment reads of each 32-row block (lane group g = lane / 16: rows 16 (g & 1) .., k-rows 8 (g / 2) ..)
    constexpr bool TRP = FAST && sizeof(TI) == 2;
    constexpr int CPR_A = BM / 8, CPR_B = BN / 8;
    static_assert(NS > 0 || !TRP || (NT / CPR_A == 16 && NT / CPR_B == 16), "a pass of loads covers sixteen k-rows");
    auto tr_soff = [&](int cpr) { const int kt = tid / cpr, mc = tid % cpr; return kt * cpr + ((((mc >> 1) ^ ((kt & 3) << 1)) << 1) | (mc & 1)); };
    const int soff_ta = tr_soff(CPR_A), soff_tb = tr_soff(CPR_B);
    const uint32_t voff_ta = (uint32_t)((tid / CPR_A) * a0.ld * ES + (tid % CPR_A) * 16);
    const uint32_t voff_tb = (uint32_t)((tid / CPR_B) * b0.ld * ES + (tid % CPR_B) * 16);
    int troff_a[TM], troff_b[TN];
    {
        const int g = lane >> 4, li = lane & 15, sw = (li >> 2) << 1;
#pragma unroll
        for (int i = 0; i < TM; ++i)
            troff_a[i] = (8 * (g >> 1) + (li >> 2)) * (BM * 2) + (((wm * 2 * TM + 2 * i + (g & 1)) ^ sw) << 5) + (li & 3) * 8;
#pragma unroll
        for (int j = 0; j < TN; ++j)
            troff_b[j] = (8 * (g >> 1) + (li >> 2)) * (BN * 2) + (((wn * 2 * TN + 2 * j + (g & 1)) ^ sw) << 5) + (li & 3) * 8;
    }

    // (rows 32 apart: the swizzle flips bit 2 of the chunk column, which is the offset of sub-step q ^ 2)
    auto lfrag = [&](const uint4* a_s, const uint4* b_s, int q, uint4 (&af)[TM], uint4 (&bf)[TN]) {
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            if constexpr (AT && TRP) af[i] = lfrag_tr<BM * 2>(reinterpret_cast<const char*>(a_s) + troff_a[i], 16 * q);
            else af[i] = a_s[roff_a[(i & 1) ? (q ^ 2) : q] + i * 32 * CHUNKS];
        }
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            if constexpr (BT && TRP) bf[j] = lfrag_tr<BN * 2>(reinterpret_cast<const char*>(b_s) + troff_b[j], 16 * q);
            else bf[j] = b_s[roff_b[(j & 1) ? (q ^ 2) : q] + j * 32 * CHUNKS];
        }
    };

    const int nslab = it_end - it_begin;
    if constexpr (NS > 0) {
        // ---- direct mode ----------------------------------------------------------------------------------------
        constexpr int NWV = 2 * WN;                         // wavefronts
        constexpr int NIA = BM * 8 / 64 / NWV, NIB = BN * 8 / 64 / NWV;   // load instructions per wavefront, slab and operand
        const int wv = __builtin_amdgcn_readfirstlane(wave);
        const unsigned lds0 = (unsigned)(uintptr_t)(__attribute__((address_space(3))) void*)smem;
        // Instruction j of wavefront wv fills the 64 LDS words (16 bytes each) starting at word 64 (j NWV + wv) of its
        // operand's buffer; lane l fetches the chunk that belongs at word 64 (j NWV + wv) + l in the swizzled layout.
        unsigned voa[NIA], vob[NIB];
#pragma unroll
        for (int j = 0; j < NIA; ++j) {
            const int jj = j * NWV + wv;
            if constexpr (AT) {
                const int kt = (64 / CPR_A) * jj + lane / CPR_A, pos = lane % CPR_A;
                const int mc = ((((pos >> 1) ^ ((kt & 3) << 1))) << 1) | (pos & 1);
                voa[j] = (unsigned)(kt * a0.ld * ES + mc * 16);
            } else {
                const int r = 8 * jj + (lane >> 3);
                voa[j] = (unsigned)(r * a0.ld * ES + (((lane & 7) ^ swz(r)) << 4));
            }
        }
#pragma unroll
        for (int j = 0; j < NIB; ++j) {
            const int jj = j * NWV + wv;
            if constexpr (BT) {
                const int kt = (64 / CPR_B) * jj + lane / CPR_B, pos = lane % CPR_B;
                const int mc = ((((pos >> 1) ^ ((kt & 3) << 1))) << 1) | (pos & 1);
                vob[j] = (unsigned)(kt * b0.ld * ES + mc * 16);
            } else {
                const int r = 8 * jj + (lane >> 3);
                vob[j] = (unsigned)(r * b0.ld * ES + (((lane & 7) ^ swz(r)) << 4));
            }
        }
        auto dma = [](unsigned lds_addr, const char* gbase, unsigned voff) __attribute__((always_inline)) {
            asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" :: "s"(lds_addr), "v"(voff), "s"(gbase) : "memory");
        };
        auto issue = [&](int it) __attribute__((always_inline)) {
            const bool s2 = it >= ntiles[0];
            const int k0 = (it - (s2 ? ntiles[0] : 0)) * BK;
            const char* pa = static_cast<const char*>(s2 ? a1.p : a0.p);
            const char* pb = static_cast<const char*>(s2 ? b1.p : b0.p);
            const long long lda = a0.ld, ldb = b0.ld;      // (both segments share their leading dimensions in the unguarded form)
            pa += AT ? ((long long)k0 * lda + row0) * ES : ((long long)row0 * lda + k0) * ES;
            pb += BT ? ((long long)k0 * ldb + col0) * ES : ((long long)col0 * ldb + k0) * ES;
            const unsigned sb = lds0 + (unsigned)(((it - it_begin) % NS) * STAGE * 16);
#pragma unroll
            for (int j = 0; j < NIA; ++j) dma(sb + (unsigned)((j * NWV + wv) * 1024), pa, voa[j]);
#pragma unroll
            for (int j = 0; j < NIB; ++j) dma(sb + (unsigned)(BM * 128 + (j * NWV + wv) * 1024), pb, vob[j]);
        };
        if constexpr (NS == 1) {
            // One LDS buffer: a slab's fragments are all read into registers, a barrier frees the buffer for the next
            // slab's loads, and the products run from registers while those loads are in flight.  Two workgroups per
            // CU take turns on the matrix cores: one multiplies while the other reads its fragments.
            uint4 fa[CHUNKS / 2][TM], fb[CHUNKS / 2][TN];
            if (nslab > 0) issue(it_begin);
            for (int it = it_begin; it < it_end; ++it) {
                asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
#pragma unroll
                for (int q = 0; q < CHUNKS / 2; ++q) lfrag(smem, smem + BM * CHUNKS, q, fa[q], fb[q]);
                asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
                if (it + 1 < it_end) issue(it + 1);
#pragma unroll
                for (int q = 0; q < CHUNKS / 2; ++q) {
#pragma unroll
                    for (int i = 0; i < TM; ++i)
#pragma unroll
                        for (int j = 0; j < TN; ++j) mma<TI>(acc[i][j], fa[q][i], fb[q][j]);
                    if (RS && do_rs && it < ntiles[0]) {
#pragma unroll
                        for (int i = 0; i < NRS; ++i) rs[i] = add_row(rs[i], fa[q][i]);
                    }
                }
            }
            __syncthreads();
        } else {
#pragma unroll
        for (int u = 0; u < NS - 1; ++u)
            if (nslab > u) issue(it_begin + u);
        for (int it = it_begin; it < it_end; ++it) {
            // this wavefront's loads of slab `it` have landed when at most the loads of the younger slabs are outstanding
            if constexpr (NS == 2) asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
            else {
                const int younger = min(NS - 2, it_end - 1 - it);
                if (younger == 0) asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
                else if (younger == 1) asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" :: "n"(NIA + NIB) : "memory");
                else asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" :: "n"(2 * (NIA + NIB)) : "memory");
            }
            // (behind the barrier every wavefront has finished the products of slab it - 1, whose buffer the next loads overwrite)
            if (it + NS - 1 < it_end) issue(it + NS - 1);
            const uint4* a_s = smem + ((it - it_begin) % NS) * STAGE;
            const uint4* b_s = a_s + BM * CHUNKS;
            constexpr int NF = (TM * TN <= 4) ? 2 : 1;
            uint4 af[NF][TM], bf[NF][TN];
            if (NF == 2) lfrag(a_s, b_s, 0, af[0], bf[0]);
#pragma unroll
            for (int q = 0; q < CHUNKS / 2; ++q) {
                if (NF == 2) { if (q + 1 < CHUNKS / 2) lfrag(a_s, b_s, q + 1, af[(q + 1) % NF], bf[(q + 1) % NF]); }
                else lfrag(a_s, b_s, q, af[0], bf[0]);
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j) mma<TI>(acc[i][j], af[q % NF][i], bf[q % NF][j]);
                if (RS && do_rs && it < ntiles[0]) {
#pragma unroll
                    for (int i = 0; i < NRS; ++i) rs[i] = add_row(rs[i], af[q % NF][i]);
                }
            }
        }
        __syncthreads();                                    // the epilogue reuses the buffers
        }
    } else {
    // D sets of staging registers: the loads of slab it + D are issued while slab it is multiplied and
    // slabs it + 1 .. it + D - 1 (loaded in earlier iterations) wait in the other sets for their LDS buffer.
    uint4 ra[D][NCA], rb[D][NCB];
    auto gload = [&](int it, uint4 (&ra)[NCA], uint4 (&rb)[NCB]) {
        const bool s = it >= ntiles[0];
        const int k0 = (it - (s ? ntiles[0] : 0)) * BK;
        Operand oa, ob;
        oa.p = s ? a1.p : a0.p; oa.ld = s ? a1.ld : a0.ld; oa.rows = a0.rows; oa.fast = s ? a1.fast : a0.fast;
        ob.p = s ? b1.p : b0.p; ob.ld = s ? b1.ld : b0.ld; ob.rows = b0.rows; ob.fast = s ? b1.fast : b0.fast;
        if constexpr (FAST) {
            // (both segments of a two-segment product share their leading dimensions in this mode)
            const char* pa = static_cast<const char*>(oa.p);
            const char* pb = static_cast<const char*>(ob.p);
            if constexpr (AT && TRP) gload_tr<NCA>(ra, pa + ((long long)k0 * oa.ld + row0) * ES, 16 * oa.ld * ES, voff_ta);
            else if constexpr (AT) gload_rowfast_fast<TI, NCA, PR>(ra, pa + ((long long)k0 * oa.ld + row0) * ES, oa.ld * ES, voff_a);
            else    gload_kfast_fast<TI, NCA>(ra, pa + ((long long)row0 * oa.ld + k0) * ES, RP * oa.ld * ES, voff_a);
            if constexpr (BT && TRP) gload_tr<NCB>(rb, pb + ((long long)k0 * ob.ld + col0) * ES, 16 * ob.ld * ES, voff_tb);
            else if constexpr (BT) gload_rowfast_fast<TI, NCB, PR>(rb, pb + ((long long)k0 * ob.ld + col0) * ES, ob.ld * ES, voff_b);
            else    gload_kfast_fast<TI, NCB>(rb, pb + ((long long)col0 * ob.ld + k0) * ES, RP * ob.ld * ES, voff_b);
        } else {
            const int K = s ? K1 : K0;
            if constexpr (AT) gload_rowfast<TI, NCA>(ra, oa, row0, K, k0, tid);
            else              gload_kfast<TI, NCA>(ra, oa, row0, K, k0, tid);
            if constexpr (BT) gload_rowfast<TI, NCB>(rb, ob, col0, K, k0, tid);
            else              gload_kfast<TI, NCB>(rb, ob, col0, K, k0, tid);
        }
    };
    auto sstore = [&](int buf, const uint4 (&ra)[NCA], const uint4 (&rb)[NCB]) {
        uint4* a_s = smem + buf * STAGE;
        uint4* b_s = a_s + BM * CHUNKS;
        if constexpr (AT && TRP) sstore_tr<NCA, CPR_A>(a_s, ra, soff_ta);
        else if constexpr (AT) sstore_rowfast_off<TI, NCA, PR>(a_s, ra, soff_r);
        else sstore_kfast_off<NCA, RP>(a_s, ra, soff_k);
        if constexpr (BT && TRP) sstore_tr<NCB, CPR_B>(b_s, rb, soff_tb);
        else if constexpr (BT) sstore_rowfast_off<TI, NCB, PR>(b_s, rb, soff_r);
        else sstore_kfast_off<NCB, RP>(b_s, rb, soff_k);
    };
    if (nslab > 0) {
        gload(it_begin, ra[0], rb[0]);
        sstore(0, ra[0], rb[0]);
    }
#pragma unroll
    for (int u = 1; u < D; ++u)
        if (nslab > u) gload(it_begin + u, ra[u], rb[u]);
    __syncthreads();
    // slab j = it - it_begin lives in LDS buffer j & 1 and was staged through register set j % D
    // `steady`: slabs it + 1 and it + D exist for sure, so the loads and the LDS stores are unconditional
    // (every path through the steady loop then has the same loads in flight, which lets the compiler
    // wait for exactly the older set before the stores).
    auto step = [&](int it, const bool steady, uint4 (&ra_cur)[NCA], uint4 (&rb_cur)[NCB], const uint4 (&ra_nxt)[NCA],
                    const uint4 (&rb_nxt)[NCB]) __attribute__((always_inline)) {
        const int buf = (it - it_begin) & 1;
        if (steady || it + D < it_end) gload(it + D, ra_cur, rb_cur);
        const uint4* a_s = smem + buf * STAGE;
        const uint4* b_s = a_s + BM * CHUNKS;
        // the 64x64 wave tile keeps two sets of fragments in flight
        constexpr int NF = (TM * TN <= 4) ? 2 : 1;
        uint4 af[NF][TM], bf[NF][TN];
        if (NF == 2) lfrag(a_s, b_s, 0, af[0], bf[0]);
#pragma unroll
        for (int q = 0; q < CHUNKS / 2; ++q) {
            if (NF == 2) { if (q + 1 < CHUNKS / 2) lfrag(a_s, b_s, q + 1, af[(q + 1) % NF], bf[(q + 1) % NF]); }
            else lfrag(a_s, b_s, q, af[0], bf[0]);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) mma<TI>(acc[i][j], af[q % NF][i], bf[q % NF][j]);
            if (RS && do_rs && it < ntiles[0]) {
#pragma unroll
                for (int i = 0; i < NRS; ++i) rs[i] = add_row(rs[i], af[q % NF][i]);
            }
        }
        if (steady || it + 1 < it_end) sstore(buf ^ 1, ra_nxt, rb_nxt);
        __syncthreads();
    };
    int it = it_begin;
    for (; it + 2 * D - 1 < it_end; it += D) {
#pragma unroll
        for (int u = 0; u < D; ++u) step(it + u, true, ra[u], rb[u], ra[(u + 1) % D], rb[(u + 1) % D]);
    }
    for (; it < it_end; it += D) {                        // the last slabs
#pragma unroll
        for (int u = 0; u < D; ++u)
            if (it + u < it_end) step(it + u, false, ra[u], rb[u], ra[(u + 1) % D], rb[(u + 1) % D]);
    }

    }

    if (RS && do_rs) {
        float* out = P.splits > 1 ? P.rs_partial + ((long long)z * P.splits + split) * P.M : P.rowsum + z * P.sRowsum;
#pragma unroll
        for (int i = 0; i < NRS; ++i) {
            const float total = rs[i] + __shfl_xor(rs[i], 32);          // the other half of every sub-step
            const int row = row0 + wm * (32 * TM) + i * 32 + (lane & 31);
            if (lane < 32 && row < P.M) out[row] = total;
        }
    }

    // Epilogue: accumulator register e of lane l is row 8*(e/4) + 4*(l/32) + e%4, column l%32.
    if constexpr (FAST) {
        // Full tiles go through LDS (free after the loop's last barrier), 64 or 128 tile rows at a time, so that every
        // store instruction writes whole rows, 16 bytes per lane (four floats or eight bf16).  A wavefront's store
        // costs the memory pipeline about the same whatever its width, so the number of store instructions is what
        // an output-heavy product (the logits: K = 256) pays for.
        // The same for the float partial tiles of a split.  16-byte column groups are XOR-swizzled with the row so
        // that both sides spread over the banks.
        const bool to_part = P.splits > 1;
        if (to_part ? P.p_vec != 0 : (P.c_vec != 0 && P.add == nullptr)) {
            float* cs = reinterpret_cast<float*>(smem);
            float* part = to_part ? P.partial + ((long long)z * P.splits + split) * (long long)P.M * P.N : nullptr;
            TO* Cz = static_cast<TO*>(P.C) + z * P.sC;
            const TI* bz = (!to_part && P.bias) ? static_cast<const TI*>(P.bias) + z * P.sBias : nullptr;
            constexpr int LDSB = (NS > 0 ? NS : 2) * STAGE * 16;
            constexpr int RR = 128 * BN * 4 <= LDSB ? 128 : 64;   // tile rows per round: RR x BN floats fit the LDS of the main loop
            static_assert(RR * BN * 4 <= LDSB, "a round of the staged epilogue must fit the LDS of the main loop");
            // A round stages RR tile rows: the row blocks h IBR .. h IBR + IBR - 1 of BOTH wave rows, so that every
            // wavefront takes part in every round.  Staging row s = wm 32 IBR + ib 32 + r is tile row
            // wm 32 TM + (h IBR + ib) 32 + r.
            constexpr int IBR = RR / 64, ROUNDS = TM / IBR;
            static_assert(TM % IBR == 0, "row blocks per round divide the wave tile");
            auto tile_row = [](int s, int h) { return (s / (32 * IBR)) * (32 * TM) + h * IBR * 32 + (s % (32 * IBR)); };
            constexpr int GPR = BN / 4, RPP = NT / GPR;     // 16-byte float groups per row, rows per pass of the stores
            constexpr int GPR8 = BN / 8, RPP8 = NT / GPR8;  // the same for eight bf16 per lane
#pragma unroll
            for (int h = 0; h < ROUNDS; ++h) {
                if (h > 0) __syncthreads();
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    const int col = wn * (32 * TN) + j * 32 + (lane & 31);
                    const float bv = bz ? ld_f(bz + col0 + col) : 0.0f;
#pragma unroll
                    for (int ib = 0; ib < IBR; ++ib) {
                        const int i = h * IBR + ib;
#pragma unroll
                        for (int e = 0; e < 16; ++e) {
                            const int row = wm * (32 * IBR) + ib * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
                            cs[row * BN + ((((col >> 2) ^ (row & 7))) << 2) + (col & 3)] = acc[i][j][e] + bv;
                        }
                    }
                }
                __syncthreads();
                if (to_part) {
                    const int g = tid % GPR;
                    float* dst0 = part + (long long)row0 * P.N + col0 + 4 * g;
#pragma unroll 4
                    for (int pass = 0; pass < RR / RPP; ++pass) {
                        const int r = pass * RPP + tid / GPR;
                        *reinterpret_cast<float4*>(dst0 + (long long)tile_row(r, h) * P.N) = *reinterpret_cast<const float4*>(&cs[r * BN + ((g ^ (r & 7)) << 2)]);
                    }
                } else if (sizeof(TO) == 2 && P.c_vec == 2) {   // eight bf16 per lane: 16-byte stores
                    const int g = tid % GPR8;
                    TO* dst0 = Cz + (long long)row0 * P.ldc + col0 + 8 * g;
#pragma unroll 4
                    for (int pass = 0; pass < RR / RPP8; ++pass) {
                        const int r = pass * RPP8 + tid / GPR8;
                        const float4 v = *reinterpret_cast<const float4*>(&cs[r * BN + (((2 * g) ^ (r & 7)) << 2)]);
                        const float4 w = *reinterpret_cast<const float4*>(&cs[r * BN + (((2 * g + 1) ^ (r & 7)) << 2)]);
                        *reinterpret_cast<uint4*>(dst0 + (long long)tile_row(r, h) * P.ldc) =
                            make_uint4(pack_bf2(v.x, v.y), pack_bf2(v.z, v.w), pack_bf2(w.x, w.y), pack_bf2(w.z, w.w));
                    }
                } else {
                    const int g = tid % GPR;
                    TO* dst0 = Cz + (long long)row0 * P.ldc + col0 + 4 * g;
#pragma unroll 4
                    for (int pass = 0; pass < RR / RPP; ++pass) {
                        const int r = pass * RPP + tid / GPR;
                        const float4 v = *reinterpret_cast<const float4*>(&cs[r * BN + ((g ^ (r & 7)) << 2)]);
                        TO* dst = dst0 + (long long)tile_row(r, h) * P.ldc;
                        if constexpr (sizeof(TO) == 4) *reinterpret_cast<float4*>(dst) = v;
                        else *reinterpret_cast<uint2*>(dst) = make_uint2(pack_bf2(v.x, v.y), pack_bf2(v.z, v.w));
                    }
                }
            }
            return;
        }
    }
    if (P.splits > 1) {
        float* part = P.partial + ((long long)z * P.splits + split) * (long long)P.M * P.N;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int col = col0 + wn * (32 * TN) + j * 32 + (lane & 31);
                if (col >= P.N) continue;
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int row = row0 + wm * (32 * TM) + i * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
                    if (row < P.M) part[(long long)row * P.N + col] = acc[i][j][e];
                }
            }
        return;
    }
    TO* C = static_cast<TO*>(P.C) + z * P.sC;
    const TI* bias = P.bias ? static_cast<const TI*>(P.bias) + z * P.sBias : nullptr;
    const float* add = P.add ? P.add + z * P.sAdd : nullptr;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int col = col0 + wn * (32 * TN) + j * 32 + (lane & 31);
            if (col >= P.N) continue;
            const float bv = bias ? ld_f(bias + col) : 0.0f;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int row = row0 + wm * (32 * TM) + i * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
                if (row < P.M) {
                    float v = acc[i][j][e] + bv;
                    if (add) v += add[(long long)row * P.ldadd + col];
                    st_f(&C[(long long)row * P.ldc + col], v);
                }
            }
        }
}

// Workgroups per CU the launch bounds allow for: by LDS in the ring modes, by registers with one buffer.
template <int TM, int TN, int WN, int D, int NS>
constexpr int occupancy_target() {
    if (NS == 1) return TM * TN <= 4 ? 3 : 2;
    if (NS > 1) return NS * (64 * TM + 32 * TN * WN) * 128 <= 80 * 1024 ? 2 : 1;
    return D == 2 ? 2 : 1;
}

template <typename TI, typename TO, bool AT, bool BT, int TM, int TN, int WN, bool FAST, bool RS, int D, int NS>
__global__ __launch_bounds__(128 * WN, (occupancy_target<TM, TN, WN, D, NS>())) void gemm_kernel(Params P) {
    gemm_tile<TI, TO, AT, BT, TM, TN, WN, FAST, RS, D, NS>(P, (int)blockIdx.x, (int)blockIdx.y, (int)blockIdx.z, true);
}

// Several independent products of one form in one launch (the weight gradients of all layers).  All tiles of all
// products are numbered in one sequence (product by product, batch-major within a product); workgroup ids are dealt
// round-robin to the eight XCDs, so XCD x takes the x-th eighth of that sequence: the tiles that run at the same time
// on one XCD then belong to one or two products and share their operand panels in that XCD's L2 (with every XCD
// walking every product, each L2 fetched its own copy of every panel: 3.4 times the algorithmic bytes, and the launch
// ran at the HBM-side bandwidth).  Tile v belongs to the product g with first[g] <= v < first[g + 1].  No split along K.
constexpr int GROUP_MAX = 14;                          // (a six-layer model: two products per layer, the bottleneck's and the softmax layer's)
struct GroupParams {
    Params p[GROUP_MAX];
    int first[GROUP_MAX + 1];
    int n;
};
static_assert(sizeof(GroupParams) <= 4096, "kernel arguments are limited to 4 KB");
template <typename TI, typename TO, bool AT, bool BT, int TM, int TN, int WN, bool FAST, bool RS, int D, int NS>
__global__ __launch_bounds__(128 * WN, (occupancy_target<TM, TN, WN, D, NS>())) void gemm_group_kernel(GroupParams G) {
    int x = (int)blockIdx.x;
    const int total8 = G.first[G.n] & ~7;
    if (x < total8) x = (x & 7) * (total8 >> 3) + (x >> 3);
    int g = 0;
    for (int k = 1; k < G.n; ++k) if (x >= G.first[k]) g = k;
    const Params& P = G.p[g];
    const int local = x - G.first[g], per = P.ntm * P.ntn;
    gemm_tile<TI, TO, AT, BT, TM, TN, WN, FAST, RS, D, NS>(P, local % per, 0, local / per, false);
}

// C[m][n] = sum over splits of partial[z][s][m][n] (+ bias[n]) in the order s = 0, 1, ...
template <typename TI, typename TO>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float* __restrict__ partial, int splits, int M, int N,
                                                            TO* __restrict__ C, long long ldc, long long sC,
                                                            const TI* __restrict__ bias, long long sBias,
                                                            const float* __restrict__ rs_partial, float* __restrict__ rowsum,
                                                            long long sRowsum, int vec4) {
    const int z = blockIdx.z;
    const long long total = (long long)M * N;
    if (rowsum)
        for (long long m = (long long)blockIdx.x * blockDim.x + threadIdx.x; m < M; m += (long long)gridDim.x * blockDim.x) {
            float v = 0.0f;
            for (int s = 0; s < splits; ++s) v += rs_partial[((long long)z * splits + s) * M + m];
            rowsum[z * sRowsum + m] = v;
        }
    const float* part = partial + (long long)z * splits * total;
    TO* Cz = C + z * sC;
    const TI* bz = bias ? bias + z * sBias : nullptr;
    if (vec4) {                                          // N a multiple of 4, rows of C and of the partial tiles 16-byte aligned
        const long long total4 = total >> 2;
        const int n4 = N >> 2;
        for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < total4; i += (long long)gridDim.x * blockDim.x) {
            float4 v = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
            for (int s = 0; s < splits; ++s) {
                const float4 p4 = *reinterpret_cast<const float4*>(part + s * total + 4 * i);
                v.x += p4.x; v.y += p4.y; v.z += p4.z; v.w += p4.w;
            }
            const int m = (int)(i / n4), n = (int)(i % n4) * 4;
            if (bz) { v.x += ld_f(bz + n); v.y += ld_f(bz + n + 1); v.z += ld_f(bz + n + 2); v.w += ld_f(bz + n + 3); }
            TO* dst = &Cz[(long long)m * ldc + n];
            if constexpr (sizeof(TO) == 4) *reinterpret_cast<float4*>(dst) = v;
            else *reinterpret_cast<uint2*>(dst) = make_uint2(pack_bf2(v.x, v.y), pack_bf2(v.z, v.w));
        }
        return;
    }
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (long long)gridDim.x * blockDim.x) {
        float v = 0.0f;
        for (int s = 0; s < splits; ++s) v += part[s * total + i];
        const int m = (int)(i / N), n = (int)(i % N);
        if (bz) v += ld_f(bz + n);
        st_f(&Cz[(long long)m * ldc + n], v);
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
        if (es == 2 && aligned(p, 16) && (ld * es) % 16 == 0 && (stride * es) % 16 == 0) f |= 4;   // eight rows per load
    }
    return f;
}

template <typename K>
hipError_t allow_lds(K kernel, size_t lds, bool* done) {
    if (*done || lds <= 48 * 1024) return hipSuccess;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e == hipSuccess) *done = true;
    return e;
}

template <typename TI, typename TO, bool AT, bool BT, int TM, int TN, int WN, bool FAST, bool RS, int D = 2, int NS = 0>
hipError_t launch_kernel(const Params& P, dim3 grid, hipStream_t stream) {
    constexpr size_t lds = (NS > 0 ? NS : 2) * (size_t)(64 * TM + 32 * TN * WN) * CHUNKS * 16;
    static thread_local bool attr_set = false;
    hipError_t e = allow_lds(&gemm_kernel<TI, TO, AT, BT, TM, TN, WN, FAST, RS, D, NS>, lds, &attr_set);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((gemm_kernel<TI, TO, AT, BT, TM, TN, WN, FAST, RS, D, NS>), grid, dim3(128 * WN), lds, stream, P);
    return hipGetLastError();
}

// ---- register-staged kernels: float operands, guarded shapes, the A^T B^T... forms the direct mode does not build ----
template <typename TI, typename TO, bool AT, bool BT, int TM, int TN, int WN>
hipError_t launch_shape(const Params& P, bool fast, bool deep, dim3 grid, hipStream_t stream) {
    if constexpr (WN != 2) {
        if (P.rowsum || !fast) return hipErrorInvalidValue;   // the large tile is built unguarded and without row sums
        return launch_kernel<TI, TO, AT, BT, TM, TN, WN, true, false>(P, grid, stream);
    } else {
        if constexpr (AT && BT) {
            if (P.rowsum) {
                if (fast && deep) return launch_kernel<TI, TO, AT, BT, TM, TN, WN, true, true, 4>(P, grid, stream);
                return fast ? launch_kernel<TI, TO, AT, BT, TM, TN, WN, true, true>(P, grid, stream)
                            : launch_kernel<TI, TO, AT, BT, TM, TN, WN, false, true>(P, grid, stream);
            }
        }
        if (P.rowsum) return hipErrorInvalidValue;           // row sums exist for the dA^T X form on 128x128 tiles only
        if constexpr (AT && BT) {                             // (the deep pipeline is built for the dA^T X form, where it pays)
            if (fast && deep) return launch_kernel<TI, TO, AT, BT, TM, TN, WN, true, false, 4>(P, grid, stream);
        }
        return fast ? launch_kernel<TI, TO, AT, BT, TM, TN, WN, true, false>(P, grid, stream)
                    : launch_kernel<TI, TO, AT, BT, TM, TN, WN, false, false>(P, grid, stream);
    }
}

template <typename TI, typename TO, int TM, int TN, int WN>
hipError_t launch_form(const GemmDesc& d, const Params& P, bool fast, bool deep, dim3 grid, hipStream_t stream) {
    if (!d.atrans && !d.btrans) return launch_shape<TI, TO, false, false, TM, TN, WN>(P, fast, deep, grid, stream);
    if (!d.atrans && d.btrans) return launch_shape<TI, TO, false, true, TM, TN, WN>(P, fast, deep, grid, stream);
    if (d.atrans && d.btrans) return launch_shape<TI, TO, true, true, TM, TN, WN>(P, fast, deep, grid, stream);
    return launch_shape<TI, TO, true, false, TM, TN, WN>(P, fast, deep, grid, stream);
}

// ---- direct-mode kernels: bf16 operands, unguarded, forms X W^T, dA W and dA^T X -------------------------------
// variant 0: 128x128 tile, two LDS buffers, two workgroups per CU; 1: 128x128, three buffers (launches of at most one
// workgroup per CU); 2: 256x128 tile, one buffer, fragments in registers, two workgroups per CU; 3: 256x256 tile on
// eight wavefronts, two buffers, one workgroup per CU (the dA W form only: the softmax layer's input gradient).
template <typename TO, bool AT, bool BT, bool RS>
hipError_t launch_direct_rs(const Params& P, int variant, dim3 grid, hipStream_t stream) {
    if (variant == 2) return launch_kernel<bf16_t, TO, AT, BT, 4, 2, 2, true, RS, 2, 1>(P, grid, stream);
    if constexpr (!AT && BT && !RS) {
        if (variant == 3) return launch_kernel<bf16_t, TO, AT, BT, 4, 2, 4, true, false, 2, 2>(P, grid, stream);
    }
    if (variant == 3) return hipErrorInvalidValue;
    if constexpr (AT && BT) {
        if (variant == 1) return launch_kernel<bf16_t, TO, AT, BT, 2, 2, 2, true, RS, 2, 3>(P, grid, stream);
    }
    return launch_kernel<bf16_t, TO, AT, BT, 2, 2, 2, true, RS, 2, 2>(P, grid, stream);
}
template <typename TO>
hipError_t launch_direct(const GemmDesc& d, const Params& P, int variant, dim3 grid, hipStream_t stream) {
    if (d.atrans && d.btrans) {
        if constexpr (sizeof(TO) == 4) {                      // (row sums go with the float weight gradients)
            if (P.rowsum) return launch_direct_rs<TO, true, true, true>(P, variant, grid, stream);
        }
        if (P.rowsum) return hipErrorInvalidValue;
        return launch_direct_rs<TO, true, true, false>(P, variant, grid, stream);
    }
    if (P.rowsum) return hipErrorInvalidValue;
    if (!d.atrans && d.btrans) return launch_direct_rs<TO, false, true, false>(P, variant, grid, stream);
    if (!d.atrans && !d.btrans) return launch_direct_rs<TO, false, false, false>(P, variant, grid, stream);
    return hipErrorInvalidValue;
}

// The unguarded kernel applies when every tile is full, every segment's K is a whole number of
// slabs, all loads may be of the widest kind, the per-thread offsets fit 32 bits, and the two
// segments (if any) share their leading dimensions.
template <typename TI>
bool can_run_fast(const GemmDesc& d, const Params& P, int tile_m, int tile_n) {
    const int bk = CHUNKS * Vec<TI>::N;
    if (d.M % tile_m || (d.Npad > 0 ? d.Npad : d.N) % tile_n) return false;
    for (int s = 0; s < d.nseg; ++s) {
        if (d.seg[s].K % bk) return false;
        if (!(P.A[s].fast & 1) || !(P.B[s].fast & 1)) return false;
        if (sizeof(TI) == 2 && ((d.atrans && !(P.A[s].fast & 4)) || (d.btrans && !(P.B[s].fast & 4)))) return false;
        if (d.seg[s].lda != d.seg[0].lda || d.seg[s].ldb != d.seg[0].ldb) return false;
        if (d.seg[s].lda * (long long)sizeof(TI) * 64 > 0x3FFFFFFF || d.seg[s].ldb * (long long)sizeof(TI) * 64 > 0x3FFFFFFF) return false;
    }
    return true;
}

constexpr int kTileM[3] = {128, 256, 256}, kTileN[3] = {128, 256, 128};

GemmPlan make_plan(const GemmDesc& d, bool allow_r);

template <typename TI>
Params make_params(const GemmDesc& d) {
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
    P.splits = 1;
    return P;
}
// Tile counts and store modes for a tile shape; `fast`: the unguarded kernel runs.
template <typename TO>
void set_tiles(const GemmDesc& d, Params& P, int tm, int tn, bool fast) {
    const size_t w = sizeof(TO) == 4 ? 16 : 8;
    P.c_vec = aligned(d.C, w) && d.ldc % 4 == 0 && ((d.batch > 1 ? d.sC : 0) % 4 == 0);
    if (sizeof(TO) == 2 && P.c_vec && aligned(d.C, 16) && d.ldc % 8 == 0 && ((d.batch > 1 ? d.sC : 0) % 8 == 0)) P.c_vec = 2;   // 16-byte bf16 stores
    if (fast && d.Npad > 0) P.c_vec = 0;                 // whole tiles are computed, the stores stop at column N
    P.p_vec = (d.N % 4 == 0 && !(fast && d.Npad > 0)) ? 1 : 0;   // (the scratch itself is 256-byte aligned)
    P.ntm = (d.M + tm - 1) / tm;
    P.ntn = ((fast && d.Npad > 0 ? d.Npad : d.N) + tn - 1) / tn;
}

template <typename TI, typename TO>
hipError_t dispatch(const GemmDesc& d, hipStream_t stream) {
    Params P = make_params<TI>(d);
    const int batch = d.batch > 0 ? d.batch : 1;
    const bool direct_form = sizeof(TI) == 2 && !d.add && !(d.atrans && !d.btrans);
    GemmPlan plan = make_plan(d, direct_form);
    // the plan looks at the shape only: check what it chose against the operands' alignment and fall back
    if (plan.tile == GEMM_TILE_256X128 && !can_run_fast<TI>(d, P, 256, 128)) plan = make_plan(d, false);
    if (plan.tile == GEMM_TILE_256 && (!can_run_fast<TI>(d, P, 256, 256) || (sizeof(TI) == 2 && !(direct_form && !d.atrans && d.btrans)))) {
        plan = make_plan(d, false);
        if (plan.tile == GEMM_TILE_256) { plan.tile = GEMM_TILE_128; plan.splits = 1; plan.partial_bytes = 0; plan.deep = false; }
    }
    const int tm = kTileM[plan.tile], tn = kTileN[plan.tile];
    const bool fast = can_run_fast<TI>(d, P, tm, tn);
    set_tiles<TO>(d, P, tm, tn, fast);
    P.splits = plan.splits;
    P.partial = plan.splits > 1 ? d.partial : nullptr;
    P.rs_partial = plan.splits > 1 ? d.partial + (size_t)plan.splits * batch * d.M * d.N : nullptr;
    dim3 grid((unsigned)(P.ntm * P.ntn), (unsigned)plan.splits, (unsigned)batch);
    const bool direct = direct_form && fast;
    const int variant = plan.tile == GEMM_TILE_256X128 ? 2 : plan.tile == GEMM_TILE_256 ? 3 : (plan.deep ? 1 : 0);
    hipError_t e;
    if (plan.splits > 1) {
        // partial tiles are float whatever the output type
        if constexpr (sizeof(TI) == 2) {
            if (direct) e = launch_direct<float>(d, P, variant, grid, stream);
            else e = launch_form<TI, float, 2, 2, 2>(d, P, fast, plan.deep, grid, stream);
        } else {
            e = plan.tile == GEMM_TILE_256 ? launch_form<TI, float, 4, 2, 4>(d, P, fast, false, grid, stream)
                                           : launch_form<TI, float, 2, 2, 2>(d, P, fast, plan.deep, grid, stream);
        }
        if (e != hipSuccess) return e;
        const long long total = (long long)d.M * d.N;
        unsigned blocks = (unsigned)((total + 255) / 256 < 2048 ? (total + 255) / 256 : 2048);
        hipLaunchKernelGGL((splitk_reduce_kernel<TI, TO>), dim3(blocks, 1, batch), dim3(256), 0, stream, d.partial, plan.splits,
                           d.M, d.N, static_cast<TO*>(d.C), d.ldc, d.sC, static_cast<const TI*>(d.bias), d.sBias,
                           P.rs_partial, d.rowsum, d.sRowsum, (P.c_vec && d.N % 4 == 0) ? 1 : 0);
        return hipGetLastError();
    }
    if constexpr (sizeof(TI) == 2) {
        if (direct) return launch_direct<TO>(d, P, variant, grid, stream);
        return launch_form<TI, TO, 2, 2, 2>(d, P, fast, plan.deep, grid, stream);
    } else {
        return plan.tile == GEMM_TILE_256 ? launch_form<TI, TO, 4, 2, 4>(d, P, fast, false, grid, stream)
                                          : launch_form<TI, TO, 2, 2, 2>(d, P, fast, plan.deep, grid, stream);
    }
}

// How a product of this shape is run.  allow_r: the 256x128 direct tile may be chosen (bf16 operands in one of its forms).
GemmPlan make_plan(const GemmDesc& d, bool allow_r) {
    GemmPlan p{GEMM_TILE_128, false, 1, 0};
    const int batch = d.batch > 0 ? d.batch : 1;
    const int Ne = d.Npad > 0 ? d.Npad : d.N;             // (the caller sets Npad only where the unguarded kernel applies)
    const long long t256 = (long long)((d.M + 255) / 256) * ((Ne + 255) / 256) * batch;
    const long long t128 = (long long)((d.M + 127) / 128) * ((Ne + 127) / 128) * batch;
    int ktot = 0;
    bool whole_slabs = true;
    for (int s = 0; s < d.nseg; ++s) { ktot += d.seg[s].K; whole_slabs = whole_slabs && d.seg[s].K % 64 == 0; }
    if (d.in_type == DT_BF16) {
        if (allow_r && d.M % 256 == 0 && Ne % 128 == 0 && whole_slabs) {
            const long long tr = (long long)(d.M / 256) * (Ne / 128) * batch;
            // Enough 256x128 tiles to put two on (nearly) every CU: the tile that moves 3/4 of the operand bytes of
            // 128x128 per flop, and the only one whose loop keeps the matrix cores above half of their rate.
            if (tr >= 480) { p.tile = GEMM_TILE_256X128; return p; }
            // Fewer tiles than that but a long contraction next to a narrow output (the softmax layer's input gradient
            // at large batch): the same tile, split along K into the smallest number of parts that fills whole
            // rounds of 512 resident workgroups to 90 %, if every part keeps 64 slabs and the float partial tiles
            // stay below an eighth of the operand bytes.
            if (tr >= 128 && d.nseg == 1 && d.partial && !d.rowsum) {
                const int slabs = d.seg[0].K / 64;
                for (int s = 1; s <= 8; ++s) {
                    const double rounds = (double)tr * s / 512.0;
                    const double eff = rounds / (double)(long long)(rounds + 0.999999);
                    if (eff < 0.9 || slabs / s < 64) continue;
                    const size_t need = s > 1 ? (size_t)s * batch * ((size_t)d.M * d.N + d.M) * sizeof(float) : 0;
                    if (s > 1 && ((long long)16 * s * d.N > d.seg[0].K || need > d.partial_bytes)) break;
                    p.tile = GEMM_TILE_256X128; p.splits = s; p.partial_bytes = need;
                    return p;
                }
            }
        }
        // A handful of large tiles and a very long contraction (the softmax layer's input gradient, dA W form): the
        // 256x256 tile, which moves half the operand bytes of 128x128 per flop, split along K over up to one
        // workgroup per CU, if every part keeps at least 24 slabs and the parts fill three quarters of the CUs.
        if (allow_r && d.nseg == 1 && !d.rowsum && d.partial && !d.atrans && d.btrans && t256 <= 64 &&
            d.M % 256 == 0 && Ne % 256 == 0 && whole_slabs) {
            const int slabs = d.seg[0].K / 64;
            int s = (int)(256 / t256);
            if (s > 16) s = 16;
            while (s > 1 && slabs / s < 24) --s;
            const size_t need = (size_t)s * batch * ((size_t)d.M * d.N + d.M) * sizeof(float);
            if (s > 1 && t256 * s >= 192 && need <= d.partial_bytes) { p.tile = GEMM_TILE_256; p.splits = s; p.partial_bytes = need; return p; }
        }
    } else {
        // float operands: the 256x256 tile has one workgroup per CU, so its prologue and epilogue are exposed: it pays
        // only when the contraction is long enough to amortise them
        if (t256 >= 512 && !d.rowsum && ktot >= 512) { p.tile = GEMM_TILE_256; return p; }
    }
    // Few output tiles and a long contraction: split K.  Up to one workgroup per CU whenever each part
    // keeps at least 8 slabs; up to two per CU (the number that fit) when each part keeps at least 64,
    // so that the float partial tiles and the reduction stay small next to the product itself.
    if (d.nseg == 1 && !d.add && d.partial && t128 <= 256) {
        const int bk = d.in_type == DT_BF16 ? 64 : 32;
        const int slabs = (d.seg[0].K + bk - 1) / bk;
        auto parts = [&](long long target, int min_slabs) {
            int s = (int)(target / t128);
            if (s > 8) s = 8;
            while (s > 1 && slabs / s < min_slabs) --s;
            return s < 1 ? 1 : s;
        };
        const int s1 = parts(256, 8), s2 = parts(512, 64);
        const int s = s1 > s2 ? s1 : s2;
        const size_t need = (size_t)s * batch * ((size_t)d.M * d.N + d.M) * sizeof(float);
        if (s > 1 && need <= d.partial_bytes) {
            p.splits = s;
            p.partial_bytes = need;
        }
    }
    // at most one 128x128 workgroup per CU: run the loads further ahead (three LDS buffers, or four register sets)
    p.deep = t128 * p.splits <= 256;
    return p;
}

}  // namespace

GemmPlan plan_gemm(const GemmDesc& d) {
    return make_plan(d, d.in_type == DT_BF16 && !d.add && !(d.atrans && !d.btrans));
}

size_t gemm_partial_bytes(int M, int N, int K, int batch, DType in_type) {
    GemmDesc d{};
    d.M = M; d.N = N; d.batch = batch; d.nseg = 1; d.seg[0].K = K; d.in_type = in_type;
    d.partial = reinterpret_cast<float*>(16); d.partial_bytes = ~size_t(0);
    // the largest of what the tile families would use in any operand form: alignment decides between them only at launch time
    size_t need = make_plan(d, false).partial_bytes;
    for (int form = 0; form < 3; ++form) {
        d.atrans = form == 2; d.btrans = form >= 1;
        const size_t a = make_plan(d, true).partial_bytes;
        if (a > need) need = a;
    }
    return need;
}

hipError_t launch_gemm(const GemmDesc& d, hipStream_t stream) {
    if (d.M <= 0 || d.N <= 0) return hipSuccess;
    if (d.in_type == DT_F32 && d.out_type == DT_F32) return dispatch<float, float>(d, stream);
    if (d.in_type == DT_BF16 && d.out_type == DT_BF16) return dispatch<bf16_t, bf16_t>(d, stream);
    if (d.in_type == DT_BF16 && d.out_type == DT_F32) return dispatch<bf16_t, float>(d, stream);
    return hipErrorInvalidValue;
}

// Independent products of the dA^T X form with bf16 operands and float results, one launch for up to GROUP_MAX of
// them (the weight gradients of several layers: together they fill the device, one by one most of them leave half of
// it idle).
bool gemm_group_ok(const GemmDesc* descs, int n) {
    for (int i = 0; i < n; ++i) {
        const GemmDesc& d = descs[i];
        if (!(d.in_type == DT_BF16 && d.out_type == DT_F32 && d.atrans && d.btrans && !d.add && !d.bias && d.nseg == 1 && d.M > 0 && d.N > 0)) return false;
        const Params P = make_params<bf16_t>(d);
        if (!can_run_fast<bf16_t>(d, P, 128, 128)) return false;
    }
    return n > 0;
}

// Products the grouped kernel cannot take run one by one.
hipError_t launch_gemm_group(const GemmDesc* descs, int n, hipStream_t stream) {
    if (n <= 0) return hipSuccess;
    if (n == 1) return launch_gemm(descs[0], stream);
    if (!gemm_group_ok(descs, n)) {
        for (int i = 0; i < n; ++i) { hipError_t e = launch_gemm(descs[i], stream); if (e != hipSuccess) return e; }
        return hipSuccess;
    }
    bool all_r = true;
    for (int i = 0; i < n && all_r; ++i) {
        const Params P = make_params<bf16_t>(descs[i]);
        if (!can_run_fast<bf16_t>(descs[i], P, 256, 128)) all_r = false;
    }
    const int tile = all_r ? GEMM_TILE_256X128 : GEMM_TILE_128;
    for (int i0 = 0; i0 < n; i0 += GROUP_MAX) {
        GroupParams G{};
        G.n = n - i0 < GROUP_MAX ? n - i0 : GROUP_MAX;
        int total = 0;
        for (int k = 0; k < G.n; ++k) {
            const GemmDesc& d = descs[i0 + k];
            G.p[k] = make_params<bf16_t>(d);
            set_tiles<float>(d, G.p[k], kTileM[tile], kTileN[tile], true);
            G.first[k] = total;
            total += G.p[k].ntm * G.p[k].ntn * (d.batch > 0 ? d.batch : 1);
        }
        G.first[G.n] = total;
        if (all_r) {
            constexpr size_t lds = (size_t)(256 + 128) * CHUNKS * 16;
            static thread_local bool attr_set = false;
            hipError_t e = allow_lds(&gemm_group_kernel<bf16_t, float, true, true, 4, 2, 2, true, true, 2, 1>, lds, &attr_set);
            if (e != hipSuccess) return e;
            hipLaunchKernelGGL((gemm_group_kernel<bf16_t, float, true, true, 4, 2, 2, true, true, 2, 1>), dim3((unsigned)total), dim3(256), lds, stream, G);
        } else {
            constexpr size_t lds = 2 * (size_t)(128 + 128) * CHUNKS * 16;
            static thread_local bool attr_set = false;
            hipError_t e = allow_lds(&gemm_group_kernel<bf16_t, float, true, true, 2, 2, 2, true, true, 2, 2>, lds, &attr_set);
            if (e != hipSuccess) return e;
            hipLaunchKernelGGL((gemm_group_kernel<bf16_t, float, true, true, 2, 2, 2, true, true, 2, 2>), dim3((unsigned)total), dim3(256), lds, stream, G);
        }
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace blstm
