// Persistent recurrent kernels: all T frames of one layer, both directions, in one launch.
//
// A workgroup owns 32 hidden units of one direction (all four gate rows of each) and a group
// of 32-row batch tiles.  Its slice of U_h stays in vector registers for the whole launch:
// NW wavefronts split the contraction index, each holding its part as MFMA B-fragments (64 to 256
// VGPRs per lane, by width).
// Per frame and batch tile a workgroup multiplies the previous h (forward) or the previous
// frame's gate gradients (backward) by its slice, reduces the NW partial accumulators through
// LDS, applies the cell arithmetic with all four gates of a unit in one lane, and writes its
// 32 columns.  The NU = H/32 workgroups that share a batch tile exchange these columns through
// global memory.  The exchanged tensor is a copy kept in the order the consumers' MFMA A-fragments
// want it, [frame][direction][32-row tile][16-column pair of chunks][chunk][row][8 columns]: a
// wavefront's load of one fragment is then one contiguous KB (row-major storage makes the same
// load touch 32 separate cache lines and runs three times slower), and a producer's 32 columns
// of a tile are one contiguous 2 KB block.  The row-major tensors the products outside these
// kernels read (h for the next layer, dE/da for the weight and input gradients) are written
// as well, off the frame-to-frame path.  Two protocols order the exchange:
//
//   SENTINEL  The exchanged tensor (h, or dE/da) is filled with the bf16 bit pattern 0xFFFF (a
//             NaN no finite value converts to) before the launch.  Producers store write-through
//             at agent scope, consumers load cache-bypassing at agent scope and take a chunk only
//             when none of its elements is the sentinel.  Each element is written once and is
//             its own ready flag: no counters, no fences, no barriers beyond the LDS reduction.
//   FENCED    Plain stores and loads ordered by a per-(group, tile) counter that is incremented
//             with agent-scope release semantics and polled with acquire semantics.
//
// Every wait is bounded by a wall-clock limit.  On expiry the wave raises a global abort word;
// every later wait returns at once when it sees the word, so all waves run to the end of the
// kernel.  A wave that abandoned a wait adds NaN to everything it writes from then on (h in the
// forward kernel, dE/da in the backward one), so the failure travels in-band into the loss, the
// gradient and the updated weights; blstm_device_status reports it as well.
#include "common.hpp"
#include "kernels.hpp"

namespace blstm {
namespace {

constexpr unsigned SENT16 = 0xFFFFu;

__device__ __forceinline__ f32x16_t mfma_bf16(const uint4& a, const uint4& b, f32x16_t c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
}

__device__ __forceinline__ unsigned ld_coh_u32(const unsigned* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }

// ---- FENCED protocol ----------------------------------------------------------------------------
// Waits until *cnt >= target; thread 0 polls.  One barrier inside.  Returns true (to every thread) if the
// wait was abandoned.
__device__ __forceinline__ bool wait_counter(unsigned* cnt, unsigned target, unsigned* abort_word, unsigned long long limit_ticks) {
    int gave_up = 0;
    if (threadIdx.x == 0) {
        const unsigned long long t0 = wall_clock64();
        unsigned it = 0;
        while (ld_coh_u32(cnt) < target) {
            __builtin_amdgcn_s_sleep(1);
            if ((++it & 63u) == 0) {
                if (ld_coh_u32(abort_word) != 0) { gave_up = 1; break; }
                if (wall_clock64() - t0 > limit_ticks) {
                    __hip_atomic_store(abort_word, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    gave_up = 1;
                    break;
                }
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    }
    return __syncthreads_or(gave_up) != 0;
}
// After the workgroup's stores: the barrier orders them before thread 0's agent-scope release.
__device__ __forceinline__ void signal_counter(unsigned* cnt) {
    __syncthreads();
    if (threadIdx.x == 0) __hip_atomic_fetch_add(cnt, 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
}

// ---- SENTINEL protocol --------------------------------------------------------------------------
__device__ __forceinline__ bf16_t coh_bf16(float v) {
    bf16_t b = f2bf(v);
    return b == SENT16 ? (bf16_t)0x7FC0 : b;             // a NaN result must not look like "not written yet"
}
__device__ __forceinline__ void st_coh_bf16(bf16_t* p, float v) {
    __hip_atomic_store(p, coh_bf16(v), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_coh_8B(bf16_t* p, const uint2& v) {
    __hip_atomic_store(reinterpret_cast<unsigned long long*>(p), (unsigned long long)v.x | ((unsigned long long)v.y << 32),
                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// One 16-byte store with the cache policy of an agent-scope atomic store (write-through to L2: sc1), written in assembly
// because atomics stop at 8 bytes and a store instruction costs the memory pipeline the same whatever its width.  The
// protocol needs no atomicity beyond each 16-bit element's, which every aligned store gives.  (The compiler does not
// count this store in its vmcnt bookkeeping; its own waits then only wait for more than they need.)
typedef unsigned int u32x4s_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void st_coh_16B(bf16_t* p, const uint4& v) {
    const u32x4s_t w = {v.x, v.y, v.z, v.w};
    // (s_nop: a store of more than 8 bytes reads its data registers over several cycles, and a vector-ALU write to them
    // must not follow at once; the compiler inserts that wait state for stores it knows, but cannot see into this one)
    asm volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_nop 1" :: "v"(p), "v"(w) : "memory");
}
__device__ __forceinline__ uint4 ld_coh_16B(const bf16_t* p) {
    const unsigned long long* q = reinterpret_cast<const unsigned long long*>(p);
    const unsigned long long lo = __hip_atomic_load(q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const unsigned long long hi = __hip_atomic_load(q + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return make_uint4((unsigned)lo, (unsigned)(lo >> 32), (unsigned)hi, (unsigned)(hi >> 32));
}
// The chunks are checked on every frame, so the test is branch-free and one operation per word:
// 0xFFFF is the largest 16-bit value, so a packed unsigned maximum over all words has a 0xFFFF half
// iff some word has one; the zero-halfword test on the complement of that maximum decides.
typedef unsigned short u16x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ unsigned max_halves(unsigned x, unsigned y) {
    return __builtin_bit_cast(unsigned, __builtin_elementwise_max(__builtin_bit_cast(u16x2_t, x), __builtin_bit_cast(u16x2_t, y)));
}
__device__ __forceinline__ unsigned max_halves(const uint4& v) { return max_halves(max_halves(v.x, v.y), max_halves(v.z, v.w)); }
__device__ __forceinline__ bool has_sentinel_half(unsigned w) { return ((~w - 0x00010001u) & w & 0x80008000u) != 0; }

// Bounded wait of one wave.  `probe` points, for the lanes with probing set, at one element of each
// producer's block: a cheap first look before the full loads.  Returns true if the wait was
// abandoned (time limit, or the abort word raised by anyone).  Wave-uniform control flow.
__device__ __forceinline__ bool wait_probe(const bf16_t* probe, bool probing, unsigned* abort_word,
                                           unsigned long long limit_ticks) {
    const unsigned long long t0 = wall_clock64();
    unsigned it = 0;
    for (;;) {
        bool ready = true;
        if (probing) ready = __hip_atomic_load(probe, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != SENT16;
        if (__all(ready)) return false;
        __builtin_amdgcn_s_sleep(1);
        if ((++it & 31u) == 0) {
            if (ld_coh_u32(abort_word) != 0) return true;
            if (wall_clock64() - t0 > limit_ticks) {
                __hip_atomic_store(abort_word, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                return true;
            }
        }
    }
}

constexpr int XPAIR = 2 * 32 * 8;                      // elements of one pair of 8-column chunks over 32 rows (1 KB)
template <int NQ>
__device__ __forceinline__ void load_chunks(uint4 (&frag)[NQ], const bf16_t* p, bool valid) {
#pragma unroll
    for (int q = 0; q < NQ; ++q) frag[q] = valid ? ld_coh_16B(p + q * XPAIR) : make_uint4(0, 0, 0, 0);
}
template <int NQ>
__device__ __forceinline__ bool all_written(const uint4 (&frag)[NQ]) {
    unsigned m = 0;
#pragma unroll
    for (int q = 0; q < NQ; ++q) m = max_halves(m, max_halves(frag[q]));
    return __all(!has_sentinel_half(m));
}
// The chunks in frag were loaded once; reloads them until no element of any lane is the sentinel
// (or the wait is abandoned).  Normally the first check passes.
template <int NQ>
__device__ __forceinline__ bool ensure_written(uint4 (&frag)[NQ], const bf16_t* p, bool valid, bool give_up,
                                               unsigned* abort_word, unsigned long long limit_ticks) {
    if (give_up || all_written<NQ>(frag)) return give_up;
    const unsigned long long t0 = wall_clock64();
    unsigned it = 0;
    for (;;) {
        __builtin_amdgcn_s_sleep(1);
        load_chunks<NQ>(frag, p, valid);
        if (all_written<NQ>(frag)) return false;
        if ((++it & 31u) == 0) {
            if (ld_coh_u32(abort_word) != 0) return true;
            if (wall_clock64() - t0 > limit_ticks) {
                __hip_atomic_store(abort_word, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                return true;
            }
        }
    }
}

// Barrier for LDS hazards only: waits for this wave's LDS operations, not for its global loads and
// write-through stores (a full __syncthreads would drain the loads issued ahead for the next item
// and the acknowledgements of the exchange stores on every item).
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

struct GroupMap { int d, u, bg, group; };

// Workgroups that exchange data sit on one XCD when ids are dealt round-robin over eight XCDs
// (a performance assumption only; correctness rests on the protocols above).
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

// First attempt at the exchanged chunks: ordinary cached loads.  Every element is either the
// sentinel or its final value (it is written once, after the pre-fill), so whatever cache level
// answers, a chunk without sentinels is correct; anything else is re-read cache-bypassing by
// ensure_written.
template <int NQ>
__device__ __forceinline__ void load_chunks_cached(uint4 (&frag)[NQ], const bf16_t* p, bool valid) {
#pragma unroll
    for (int q = 0; q < NQ; ++q) frag[q] = valid ? *reinterpret_cast<const uint4*>(p + q * XPAIR) : make_uint4(0, 0, 0, 0);
}
// Element offset of column c (within a direction), row r of a tile, in the exchange order.
__device__ __forceinline__ unsigned xoff(int c, int r) { return (unsigned)((c >> 3) * 256 + r * 8 + (c & 7)); }

// Saved activations of the persistent kernels ("records"): the forward kernel's lane (workgroup of unit slice u, thread
// tid) owns four cells of a (frame, direction, batch tile) and the backward kernel's lane of the same ids owns the same
// four, so what one saves for the other is indexed [frame][direction][tile][unit slice][word][thread] in 16-byte
// words: a lane reads back exactly what it wrote, with one wide access per word instead of one per cell.
__device__ __forceinline__ size_t rec_index(int t, int d, int tile, int NT, int NU, int u) {
    return ((size_t)(t * 2 + d) * NT + tile) * NU + u;
}

// Number of 32-row batch tiles of this workgroup's group that lie inside the batch.
__device__ __forceinline__ int tiles_in_batch(int bg, int tiles_per_group, int B) {
    const int first = bg * tiles_per_group * 32;
    if (first >= B) return 0;
    const int n = (B - first + 31) / 32;
    return n < tiles_per_group ? n : tiles_per_group;
}

// ------------------------------------------------------------------------------ forward
// KW = contraction elements per wavefront: H = NW * KW.
// FULL: B is a multiple of 32, so every row of every tile exists and no access is predicated.
// MULTI: a workgroup owns several batch tiles (tiles_per_group > 1); only then is there a next item
// whose exchanged chunks can be loaded ahead, and only then are registers set aside for them.
template <int NW, int KW, bool SENTINEL, bool FULL, bool MULTI>
__global__ __launch_bounds__(64 * NW) void rec_fwd_kernel(RecFwdArgs a) {
    constexpr int EPT = 16 / NW;                         // accumulator registers (batch rows) per thread
    constexpr int KSTEPS = KW / 16;                      // MFMA steps per gate per wavefront
    extern __shared__ float lds[];                       // [NW][4][4][64][4] partial accumulators
    constexpr int H = NW * KW;                           // (the launcher picks NW and KW from a.H)
    const int B = a.B, T = a.T;
    constexpr int NU = H / 32;
    const GroupMap gm = map_block(NU, a.nbg);
    const int d = gm.d, u = gm.u;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l32 = lane & 31, lh = lane >> 5;
    const int ntl = tiles_in_batch(gm.bg, a.tiles_per_group, B);
    // This workgroup's share of the region to fill (the widest slice of U_h leaves no register for it: KW <= 128 only):
    // words [fill_pos, fill_end) of its share, a few words per thread and item.
    constexpr bool FILLS = KW <= 128;
    const unsigned long long fill_per_wg = (FILLS && a.fill) ? (a.fill_words + gridDim.x - 1) / gridDim.x : 0ull;
    const unsigned long long fill_begin = min(a.fill_words, (unsigned long long)blockIdx.x * fill_per_wg);
    uint4* const fill_base = static_cast<uint4*>(a.fill) + fill_begin;                     // uniform
    const unsigned fill_end = (unsigned)(min(a.fill_words, fill_begin + fill_per_wg) - fill_begin);   // (a share is far below 2^32 words)
    unsigned fill_pos = threadIdx.x;
    const int fill_per_item = ntl > 0 ? (int)((fill_per_wg + (unsigned long long)(64 * NW) * (T * ntl) - 1) / ((unsigned long long)(64 * NW) * (T * ntl))) : 0;
    auto fill_some = [&](int words) __attribute__((always_inline)) {
        if constexpr (FILLS)
            for (int k = 0; k < words && fill_pos < fill_end; ++k, fill_pos += 64 * NW) fill_base[fill_pos] = make_uint4(~0u, ~0u, ~0u, ~0u);
    };
    if (ntl == 0) {                                      // no batch tile of its own: only its share of the fill
        if constexpr (FILLS) while (fill_pos < fill_end) fill_some(1 << 20);
        return;
    }

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
    float4* l4 = reinterpret_cast<float4*>(lds);

    // Addresses are a per-item uniform base (frame and tile origin) plus per-thread 32-bit element
    // offsets computed once: brow[e] is the batch row of accumulator register e within a tile.
    // Register e is batch row rb + re(e) of the tile: rb per thread, re(e) a compile-time constant.
    const int rb = 2 * EPT * wave + 4 * lh;
    auto re = [](int e) { return 8 * (e >> 2) + (e & 3); };
    const unsigned o8b = (unsigned)(rb * 8 * H + d * 4 * H + j); // into the row-major [.][8H] tensor (a_x)
    const int NT = (B + 31) / 32;                        // 32-row tiles of the batch
    constexpr int XH = H / 16 * XPAIR;                   // exchange elements per (frame, direction, tile)
    const unsigned ohp = (unsigned)(wave * (KW / 16) * XPAIR + lane * 8);   // this lane's 16 bytes of each chunk pair

    // Per-item inputs that do not depend on the exchange (a_x of the frame, previous cell state) are
    // loaded one item ahead, so that their HBM latency never sits on the frame-to-frame path.
    // Item = (visited frame n, batch tile i); this thread's EPT batch rows are accumulator
    // registers r = EPT*wave + e.
    auto issue_inputs = [&](int item, float (&ax)[EPT][4], float (&cp)[EPT]) {
        const int n = item / ntl, i = item - n * ntl;
        const int t = d ? T - 1 - n : n;
        const int tp = d ? T - n : n - 1;
        const int b0 = (gm.bg * a.tiles_per_group + i) * 32;
        const float* axb = a.ax + ((size_t)t * B + b0) * 8 * H;
        // (a_x fetched as 16-byte pieces and transposed through LDS, a quarter of these loads, was measured: no gain with
        // one tile per workgroup, where the loads hide under the exchange wait, and slower with several)
#pragma unroll
        for (int e = 0; e < EPT; ++e) {
            const bool ok = FULL || b0 + rb + re(e) < B;
#pragma unroll
            for (int g = 0; g < 4; ++g) ax[e][g] = ok ? axb[o8b + (unsigned)((re(e) * 8 + g) * H)] : 0.0f;
        }
        // the previous cell state of this lane's four cells is one 16-byte word of the saved records (one tile: c stays in registers)
        float4 c4 = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        if (n > 0 && ntl > 1) c4 = reinterpret_cast<const float4*>(a.c)[rec_index(tp, d, b0 >> 5, NT, NU, u) * 256 + threadIdx.x];
        cp[0] = c4.x; cp[1] = c4.y; cp[2] = c4.z; cp[3] = c4.w;
    };

    const int nitems = T * ntl;
    // Two sets of input registers used in turn: an item computes from one while the next item's loads land
    // in the other, so nothing is copied (a copy would have to wait for loads issued a moment before).
    float ax0[EPT][4], cp0[EPT], ax1[EPT][4], cp1[EPT];
    issue_inputs(0, ax0, cp0);
    // Waited for here, once: the compiler places its waits for the worst path into the loop, and with these
    // loads still in flight on the way in, that path would make every item wait for its freshly issued loads.
    __builtin_amdgcn_s_waitcnt(0x0F70);                  // vmcnt(0) (expcnt and lgkmcnt left alone)
    float ccarry[EPT];                                   // one tile per workgroup: its cell state of the frame before
#pragma unroll
    for (int e = 0; e < EPT; ++e) ccarry[e] = 0.0f;
    // With several batch tiles per workgroup the next item's h was written a whole frame ago: its
    // chunks are loaded while this item computes (checked for the sentinel like any other load).
    uint4 apre[MULTI ? KSTEPS : 1];
    bool have_pre = false;
    // The row-major outputs of an item (c, the gates, h for the next layer) are not on the frame-to-frame path:
    // they wait in registers until the next item has issued its loads of the exchanged h, and go out behind them.
    struct Tail { int t, b0; bool have, xok; float cn[EPT]; uint2 g[EPT]; uint2 hq; } tail;
    tail.have = false;
    // NaN once this wave has abandoned a wait, or from the start if an earlier launch left the abort word raised:
    // added to every h it writes
    float poison = ld_coh_u32(a.abort_word) != 0 ? __builtin_nanf("") : 0.0f;
    auto flush_tail = [&]() __attribute__((always_inline)) {
        if (!tail.have) return;
        tail.have = false;
        bf16_t* yb = a.y + ((size_t)tail.t * B + tail.b0) * 2 * H;
        // What the backward kernel needs of this lane's four cells goes out as the lane's record: three 16-byte words
        // (gates of cells 0-1, gates of cells 2-3, the four cell states), each word array contiguous over the workgroup.
        {
            const size_t r = rec_index(tail.t, d, tail.b0 >> 5, NT, NU, u);
            uint4* g4 = reinterpret_cast<uint4*>(a.gates) + r * 2 * 256 + threadIdx.x;
            g4[0] = make_uint4(tail.g[0].x, tail.g[0].y, tail.g[1].x, tail.g[1].y);
            g4[256] = make_uint4(tail.g[2].x, tail.g[2].y, tail.g[3].x, tail.g[3].y);
            reinterpret_cast<float4*>(a.c)[r * 256 + threadIdx.x] = make_float4(tail.cn[0], tail.cn[1], tail.cn[2], tail.cn[3]);
        }
        const int lane_ = threadIdx.x & 63;
        const int xrow_ = 2 * EPT * (int)(threadIdx.x >> 6) + 4 * (lane_ >> 5) + ((lane_ >> 3) & 3);
        const unsigned xcol_ = (unsigned)(u * 32 + 8 * ((lane_ >> 1) & 3) + 4 * (lane_ & 1));
        if (tail.xok) *reinterpret_cast<uint2*>(yb + ((unsigned)xrow_ * (unsigned)(2 * H) + (unsigned)(d * H) + xcol_)) = tail.hq;
        fill_some(fill_per_item);
    };
    auto do_item = [&](const int item, const float (&ax)[EPT][4], const float (&cpl)[EPT], float (&axn)[EPT][4],
                       float (&cpn)[EPT]) __attribute__((always_inline)) {
        const int n = item / ntl, i = item - n * ntl;
        const int t = d ? T - 1 - n : n;
        const int tp = d ? T - n : n - 1;
        const int b0 = (gm.bg * a.tiles_per_group + i) * 32;
        float sum[EPT][4];
#pragma unroll
        for (int e = 0; e < EPT; ++e)
#pragma unroll
            for (int g = 0; g < 4; ++g) sum[e][g] = 0.0f;
        if (n > 0) {
            // previous h of this batch tile: row l32, 8 consecutive k per lane
            const int row = b0 + l32;
            const bool valid = FULL || row < B;
            const bf16_t* hb = a.hx + ((size_t)(tp * 2 + d) * NT + (b0 >> 5)) * XH;   // uniform: previous frame, this tile
            const bf16_t* hp = hb + ohp;
            uint4 afrag[KSTEPS];
            if (SENTINEL) {
                // one probe per producing workgroup of this wavefront's k-range: its last unit, last valid row
                const int prow = FULL ? b0 + 31 : min(b0 + 31, B - 1);
                const bf16_t* probe = hb + xoff(wave * KW + (lane & (KW / 32 - 1)) * 32 + 31, prow - b0);
                bool got = false, gu = false;
                if constexpr (MULTI) {
                    if (have_pre) {
#pragma unroll
                        for (int q = 0; q < KSTEPS; ++q) afrag[q] = apre[q];
                        got = all_written<KSTEPS>(afrag);
                    }
                }
                if (!got) {
                    // Straight for the data: this wavefront's loads queue behind its own stores of the item
                    // before, whose acknowledgements take about as long as the other workgroups' h takes to
                    // arrive, so the first look nearly always finds everything.  If not: the cheap probe, then
                    // cache-bypassing loads (the first ones may have left lines with sentinels in the L1).
                    // (The widest slice has no registers for two attempts: probe first, then the data.)
                    if constexpr (KW <= 128) {
                        load_chunks_cached<KSTEPS>(afrag, hp, valid);
                        flush_tail();
                        if (!all_written<KSTEPS>(afrag)) {
                            gu = wait_probe(probe, lane < KW / 32, a.abort_word, a.limit_ticks);
                            asm volatile("" ::: "memory");
                            load_chunks<KSTEPS>(afrag, hp, valid);
                        }
                    } else {
                        gu = wait_probe(probe, lane < KW / 32, a.abort_word, a.limit_ticks);
                        asm volatile("" ::: "memory");
                        load_chunks_cached<KSTEPS>(afrag, hp, valid);
                    }
                }
                if (ensure_written<KSTEPS>(afrag, hp, valid, gu, a.abort_word, a.limit_ticks)) poison = __builtin_nanf("");
            } else {
                if (wait_counter(cnt + i, (unsigned)(NU * n), a.abort_word, a.limit_ticks)) poison = __builtin_nanf("");
#pragma unroll
                for (int q = 0; q < KSTEPS; ++q)
                    afrag[q] = valid ? *reinterpret_cast<const uint4*>(hp + q * XPAIR) : make_uint4(0, 0, 0, 0);
            }
            f32x16_t acc[4];
#pragma unroll
            for (int g = 0; g < 4; ++g)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[g][e] = 0.0f;
#pragma unroll
            for (int q = 0; q < KSTEPS; ++q)
#pragma unroll
                for (int g = 0; g < 4; ++g) acc[g] = mfma_bf16(afrag[q], bfrag[g][q], acc[g]);
            have_pre = false;
            if constexpr (MULTI && SENTINEL && KW == 128) if (ntl >= 2 && item + 1 < nitems) {
                const int n2 = (item + 1) / ntl, i2 = (item + 1) - n2 * ntl;
                const int tp2 = d ? T - n2 : n2 - 1;
                const int b02 = (gm.bg * a.tiles_per_group + i2) * 32;
                const bool valid2 = FULL || b02 + l32 < B;
                const bf16_t* hb2 = a.hx + ((size_t)(tp2 * 2 + d) * NT + (b02 >> 5)) * XH;
                load_chunks_cached<KSTEPS>(apre, hb2 + ohp, valid2);
                have_pre = true;
            }
            // partial accumulators -> LDS as [wave][gate][reg/4][lane][reg%4]
#pragma unroll
            for (int g = 0; g < 4; ++g)
#pragma unroll
                for (int rq = 0; rq < 4; ++rq)
                    l4[((wave * 4 + g) * 4 + rq) * 64 + lane] =
                        make_float4(acc[g][4 * rq], acc[g][4 * rq + 1], acc[g][4 * rq + 2], acc[g][4 * rq + 3]);
            if (SENTINEL) lds_barrier(); else __syncthreads();
            // all partial sums of this thread's rows are read before any is added: the reads then
            // overlap instead of each waiting for its LDS round trip
            static_assert(EPT % 4 == 0, "rows per thread come in groups of four accumulator registers");
            float4 part[NW][4][EPT / 4];
#pragma unroll
            for (int w2 = 0; w2 < NW; ++w2)
#pragma unroll
                for (int g = 0; g < 4; ++g)
#pragma unroll
                    for (int e4 = 0; e4 < EPT / 4; ++e4) part[w2][g][e4] = l4[((w2 * 4 + g) * 4 + (EPT / 4) * wave + e4) * 64 + lane];
#pragma unroll
            for (int w2 = 0; w2 < NW; ++w2)
#pragma unroll
                for (int g = 0; g < 4; ++g)
#pragma unroll
                    for (int e4 = 0; e4 < EPT / 4; ++e4) {
                        const float4 v = part[w2][g][e4];
                        sum[4 * e4][g] += v.x; sum[4 * e4 + 1][g] += v.y; sum[4 * e4 + 2][g] += v.z; sum[4 * e4 + 3][g] += v.w;
                    }
        }
        // (The next item's inputs come from HBM, and a CU's vector memory pipeline returns data in order: issued
        // before the barrier above they would sit in front of another wavefront's loads of the exchanged h and
        // add their latency to the frame-to-frame path.  They are issued below, once h has gone out.)
        flush_tail();                                     // at the latest here: the loads issued below may read what it stores
        float cp[EPT];
#pragma unroll
        for (int e = 0; e < EPT; ++e) cp[e] = (ntl == 1) ? ccarry[e] : cpl[e];
        if (KW > 128 && item + 1 < nitems) issue_inputs(item + 1, axn, cpn);   // (widest slice: registers are short later on)
        // cell arithmetic; h goes out first because it is all the other workgroups wait for
        float gi[EPT], gf[EPT], gg[EPT], go[EPT], cn[EPT], hn[EPT];
        bf16_t* hxb = a.hx + ((size_t)(t * 2 + d) * NT + (b0 >> 5)) * XH;
#pragma unroll
        for (int e = 0; e < EPT; ++e) {
            gi[e] = fast_sigmoid(ax[e][0] + sum[e][0]);
            gf[e] = fast_sigmoid(ax[e][1] + sum[e][1]);
            gg[e] = fast_tanh(ax[e][2] + sum[e][2]);
            go[e] = fast_sigmoid(ax[e][3] + sum[e][3]);
            cn[e] = gf[e] * cp[e] + gi[e] * gg[e];
            hn[e] = go[e] * fast_tanh(cn[e]) + poison;
        }
        // A lane holds four rows of one unit; both copies of h want the units of a row side by side.  Regrouped
        // through LDS inside the wavefront (as dE/da in the backward kernel), every lane stores four units of one
        // row: one 8-byte store per copy instead of four 2-byte ones.
        static_assert(EPT == 4, "the regrouping below is written for four rows per lane");
        unsigned* xs = reinterpret_cast<unsigned*>(lds) + NW * 4 * 4 * 64 * 4 + wave * 128;
        xs[(lh * 2 + 0) * 32 + l32] = (unsigned)coh_bf16(hn[0]) | ((unsigned)coh_bf16(hn[1]) << 16);
        xs[(lh * 2 + 1) * 32 + l32] = (unsigned)coh_bf16(hn[2]) | ((unsigned)coh_bf16(hn[3]) << 16);
        const int xh = lane & 1, xk = (lane >> 1) & 3, xr = (lane >> 3) & 3, xl = lane >> 5;
        uint2 hq;                                         // units 8 xk + 4 xh .. + 3 of row xrow
        {
            const uint4 w = *reinterpret_cast<const uint4*>(xs + (xl * 2 + (xr >> 1)) * 32 + 8 * xk + 4 * xh);
            const unsigned sel = (xr & 1) ? 0x07060302u : 0x05040100u;
            hq = make_uint2(__builtin_amdgcn_perm(w.y, w.x, sel), __builtin_amdgcn_perm(w.w, w.z, sel));
        }
        const int xrow = 2 * EPT * wave + 4 * xl + xr;    // row of the tile
        const bool xok = FULL || b0 + xrow < B;
        const unsigned xcol = (unsigned)(u * 32 + 8 * xk + 4 * xh);
        if (xok) {
            bf16_t* xp = hxb + ((xcol >> 3) * 256u + (unsigned)xrow * 8u + (xcol & 7u));
            if (SENTINEL) st_coh_8B(xp, hq); else *reinterpret_cast<uint2*>(xp) = hq;
        }
        if (KW <= 128 && item + 1 < nitems) issue_inputs(item + 1, axn, cpn);
        if (SENTINEL) lds_barrier();                     // frees the LDS buffer for the next item
        else signal_counter(cnt + i);                    // barrier inside: same role
        // row-major outputs (h for the next layer, c and the gates for the backward pass): kept for flush_tail
        tail.t = t; tail.b0 = b0; tail.have = true; tail.xok = xok; tail.hq = hq;
#pragma unroll
        for (int e = 0; e < EPT; ++e) {
            tail.cn[e] = cn[e];
            tail.g[e] = make_uint2(pack_bf2(gi[e], gf[e]), pack_bf2(gg[e], go[e]));
        }
        // with one tile per workgroup the next item's previous cell state is the one just computed
#pragma unroll
        for (int e = 0; e < EPT; ++e) ccarry[e] = cn[e];
    };
    if constexpr (KW <= 128) {
        for (int item = 0; item < nitems; item += 2) {
            do_item(item, ax0, cp0, ax1, cp1);
            if (item + 1 < nitems) do_item(item + 1, ax1, cp1, ax0, cp0);
        }
    } else {
        // (the widest slice of U_h leaves no room for the loop body twice: one body, and a copy at its end)
        for (int item = 0; item < nitems; ++item) {
            do_item(item, ax0, cp0, ax1, cp1);
#pragma unroll
            for (int e = 0; e < EPT; ++e) {
#pragma unroll
                for (int g = 0; g < 4; ++g) ax0[e][g] = ax1[e][g];
                cp0[e] = cp1[e];
            }
        }
    }
    flush_tail();
    if constexpr (FILLS) while (fill_pos < fill_end) fill_some(1 << 20);   // (whatever rounding left over)
}

// ------------------------------------------------------------------------------ backward
template <int NW, int KW, bool SENTINEL, bool FULL, bool MULTI>
__global__ __launch_bounds__(64 * NW) void rec_bwd_kernel(RecBwdArgs a) {
    constexpr int EPT = 16 / NW;
    constexpr int KSTEPS = 4 * KW / 16;                  // the contraction runs over the 4H gate rows
    extern __shared__ float lds[];                       // [NW][4][64][4]
    constexpr int H = NW * KW;                           // (the launcher picks NW and KW from a.H)
    const int B = a.B, T = a.T;
    constexpr int NU = H / 32;
    const GroupMap gm = map_block(NU, a.nbg);
    const int d = gm.d, u = gm.u;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l32 = lane & 31, lh = lane >> 5;
    constexpr int KWB = 4 * H / NW;                         // gate rows per wavefront (= 4 * KW)
    const int ntl = tiles_in_batch(gm.bg, a.tiles_per_group, B);
    if (ntl == 0) return;

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
    float4* l4 = reinterpret_cast<float4*>(lds);

    // per-thread 32-bit element offsets, added to per-item uniform bases (as in the forward kernel)
    const int rb = 2 * EPT * wave + 4 * lh;              // register e is batch row rb + re(e) of the tile
    auto re = [](int e) { return 8 * (e >> 2) + (e & 3); };
    const unsigned o2b = (unsigned)(rb * 2 * H + d * H + j);     // into [.][2H] (dy)
    const int NT = (B + 31) / 32;
    constexpr int XA = 4 * H / 16 * XPAIR;               // exchange elements per (frame, direction, tile)
    const unsigned oap = (unsigned)(wave * (KWB / 16) * XPAIR + lane * 8);   // this lane's 16 bytes of each chunk pair

    // Saved activations of an item, loaded one item ahead (raw bf16 for the gates and dy).
    // dy of a wavefront's cells is eight rows of 32 units: 512 contiguous-by-row bytes.  With one tile per workgroup
    // 32 lanes fetch it as one 16-byte piece each (dyr) and the wavefront spreads it through LDS at the start of the item
    // (one vector-memory instruction instead of four); with several tiles each lane loads its four values (see the
    // forward kernel's a_x for why).
    constexpr bool WIDE_DY = !MULTI;
    struct Inputs { uint2 g[EPT]; bf16_t dy[EPT]; uint4 dyr; float c[EPT], cp[EPT], dcr[EPT]; };   // g: (i, f), (g, o) as bf16 pairs
    auto issue_inputs = [&](int item, Inputs& in) {
        const int ni = item / ntl, i = item - ni * ntl;
        const int n = T - 1 - ni;
        const int t = d ? T - 1 - n : n;
        const int tp = d ? T - n : n - 1;
        const int b0 = (gm.bg * a.tiles_per_group + i) * 32;
        const size_t m0 = (size_t)t * B + b0;
        const bf16_t* dyb = a.dy + m0 * 2 * H;
        // the lane's records (see rec_index): gates of its four cells, their cell states, those of the frame visited before
        const size_t r = rec_index(t, d, b0 >> 5, NT, NU, u);
        const uint4* g4 = reinterpret_cast<const uint4*>(a.gates) + r * 2 * 256 + threadIdx.x;
        const uint4 g01 = g4[0], g23 = g4[256];
        float4 c4 = make_float4(0.0f, 0.0f, 0.0f, 0.0f), cp4 = c4, dc4 = c4;
        if (ntl > 1 || item == 0) c4 = reinterpret_cast<const float4*>(a.c)[r * 256 + threadIdx.x];   // (one tile: the c of this frame was the item before's c_prev)
        if (n > 0) cp4 = reinterpret_cast<const float4*>(a.c)[rec_index(tp, d, b0 >> 5, NT, NU, u) * 256 + threadIdx.x];
        if (n < T - 1 && ntl > 1) dc4 = reinterpret_cast<const float4*>(a.dc)[((size_t)(d * NT + (b0 >> 5)) * NU + u) * 256 + threadIdx.x];   // (one tile: carried in registers)
        if constexpr (WIDE_DY) {                         // piece lane % 32: row (lane % 32) / 4 of the wavefront's eight, units 8 (lane % 4) .. + 7
            const int row = 2 * EPT * wave + (l32 >> 2);
            in.dyr = make_uint4(0u, 0u, 0u, 0u);
            if (FULL || b0 + row < B) in.dyr = *reinterpret_cast<const uint4*>(dyb + (size_t)row * 2 * H + d * H + u * 32 + (l32 & 3) * 8);
        }
        static_assert(EPT == 4, "a record holds four cells");
        in.g[0] = make_uint2(g01.x, g01.y); in.g[1] = make_uint2(g01.z, g01.w);
        in.g[2] = make_uint2(g23.x, g23.y); in.g[3] = make_uint2(g23.z, g23.w);
        in.c[0] = c4.x; in.c[1] = c4.y; in.c[2] = c4.z; in.c[3] = c4.w;
        in.cp[0] = cp4.x; in.cp[1] = cp4.y; in.cp[2] = cp4.z; in.cp[3] = cp4.w;
        in.dcr[0] = dc4.x; in.dcr[1] = dc4.y; in.dcr[2] = dc4.z; in.dcr[3] = dc4.w;
#pragma unroll
        for (int e = 0; e < EPT; ++e) {
            const bool ok = FULL || b0 + rb + re(e) < B;
            if constexpr (!WIDE_DY) in.dy[e] = ok ? dyb[o2b + (unsigned)(re(e) * 2 * H)] : (bf16_t)0;
            if (!ok) { in.g[e] = make_uint2(0u, 0u); in.c[e] = 0.0f; in.cp[e] = 0.0f; in.dcr[e] = 0.0f; }
        }
    };

    static_assert(EPT <= 8, "two sets of inputs (this item's and the next one's) must fit in registers");
    const int nitems = T * ntl;
    Inputs in0, in1;                                     // two sets used in turn, as in the forward kernel
    issue_inputs(0, in0);
    __builtin_amdgcn_s_waitcnt(0x0F70);                  // vmcnt(0): see the forward kernel
    // One tile per workgroup: dE/dc of the frame visited before and that frame's c_prev (this frame's c) stay in
    // registers; a wavefront can have 63 vector-memory operations in flight, and an item of this kernel issues about 50.
    float dccarry[EPT], ccarry[EPT];
#pragma unroll
    for (int e = 0; e < EPT; ++e) { dccarry[e] = 0.0f; ccarry[e] = 0.0f; }
    uint4 apre[MULTI ? 8 : 1];                           // first slab of the next item, loaded ahead (several tiles only)
    bool have_pre = false;
    // NaN once this wave has abandoned a wait, or from the start if the abort word is already raised: added to
    // every dE/da it writes
    float poison = ld_coh_u32(a.abort_word) != 0 ? __builtin_nanf("") : 0.0f;
    auto do_item = [&](const int item, const Inputs& cur, Inputs& nxt) __attribute__((always_inline)) {
        const int ni = item / ntl, i = item - ni * ntl;
        const int n = T - 1 - ni;
        const int t = d ? T - 1 - n : n;
        const int tn = d ? T - 2 - n : n + 1;            // frame visited after t (its da feeds dh)
        const int b0 = (gm.bg * a.tiles_per_group + i) * 32;
        float dh[EPT];
#pragma unroll
        for (int e = 0; e < EPT; ++e) dh[e] = 0.0f;
        bf16_t dyv[EPT];
        if constexpr (WIDE_DY) {
            bf16_t* dys = reinterpret_cast<bf16_t*>(lds + NW * 4 * 64 * 4 + NW * 512) + wave * 256;   // 512 bytes per wavefront: [row][unit]
            if (lane < 32) reinterpret_cast<uint4*>(dys)[lane] = cur.dyr;
#pragma unroll
            for (int e = 0; e < EPT; ++e) dyv[e] = dys[(4 * lh + e) * 32 + l32];
        } else {
#pragma unroll
            for (int e = 0; e < EPT; ++e) dyv[e] = cur.dy[e];
        }
        if (n < T - 1) {
            const int row = b0 + l32;
            const bool valid = FULL || row < B;
            const bf16_t* ab = a.dax + ((size_t)(tn * 2 + d) * NT + (b0 >> 5)) * XA;   // uniform: the frame visited before, this tile
            const bf16_t* ap = ab + oap;
            f32x16_t acc;
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[e] = 0.0f;
            if (SENTINEL) {
                // the gate rows of this wavefront come from KWB/32 producers: probe each one's last unit,
                // then stream the slabs of 128 gate rows with the next slab's loads in flight
                const int prow = FULL ? b0 + 31 : min(b0 + 31, B - 1);
                const bf16_t* probe = ab + xoff(wave * KWB + (lane & (4 * KW / 32 - 1)) * 32 + 31, prow - b0);
                uint4 afrag[2][8];
                bool got = false, gu = false;
                if constexpr (MULTI) {
                    if (have_pre) {
#pragma unroll
                        for (int q = 0; q < 8; ++q) afrag[0][q] = apre[q];
                        got = all_written<8>(afrag[0]);
                    }
                }
                if (!got) {
                    // (straight for the data, the probe only if the first look fails: see the forward kernel)
                    load_chunks_cached<8>(afrag[0], ap, valid);
                    if (!all_written<8>(afrag[0])) {
                        gu = wait_probe(probe, lane < 4 * KW / 32, a.abort_word, a.limit_ticks);
                        asm volatile("" ::: "memory");
                        load_chunks<8>(afrag[0], ap, valid);
                    }
                }
#pragma unroll
                for (int sl = 0; sl < KSTEPS / 8; ++sl) {
                    if (sl + 1 < KSTEPS / 8) load_chunks_cached<8>(afrag[(sl + 1) & 1], ap + (sl + 1) * 8 * XPAIR, valid);
                    else {
                        have_pre = false;
                        if constexpr (MULTI && KW == 128) if (ntl >= 2 && item + 1 < nitems) {
                            const int ni2 = (item + 1) / ntl, i2 = (item + 1) - ni2 * ntl;
                            const int n2 = T - 1 - ni2;
                            if (n2 < T - 1) {
                                const int tn2 = d ? T - 2 - n2 : n2 + 1;
                                const int b02 = (gm.bg * a.tiles_per_group + i2) * 32;
                                const bool valid2 = FULL || b02 + l32 < B;
                                const bf16_t* ab2 = a.dax + ((size_t)(tn2 * 2 + d) * NT + (b02 >> 5)) * XA;
                                load_chunks_cached<8>(apre, ab2 + oap, valid2);
                                have_pre = true;
                            }
                        }
                    }
                    gu = ensure_written<8>(afrag[sl & 1], ap + sl * 8 * XPAIR, valid, gu, a.abort_word, a.limit_ticks);
#pragma unroll
                    for (int q = 0; q < 8; ++q) acc = mfma_bf16(afrag[sl & 1][q], bfrag[sl * 8 + q], acc);
                }
                if (gu) poison = __builtin_nanf("");
            } else {
                if (wait_counter(cnt + i, (unsigned)(NU * (T - 1 - n)), a.abort_word, a.limit_ticks)) poison = __builtin_nanf("");
#pragma unroll
                for (int q0 = 0; q0 < KSTEPS; q0 += 8) {
                    uint4 afrag[8];
#pragma unroll
                    for (int q = 0; q < 8; ++q)
                        afrag[q] = valid ? *reinterpret_cast<const uint4*>(ap + (q0 + q) * XPAIR) : make_uint4(0, 0, 0, 0);
#pragma unroll
                    for (int q = 0; q < 8; ++q) acc = mfma_bf16(afrag[q], bfrag[q0 + q], acc);
                }
            }
#pragma unroll
            for (int rq = 0; rq < 4; ++rq)
                l4[(wave * 4 + rq) * 64 + lane] = make_float4(acc[4 * rq], acc[4 * rq + 1], acc[4 * rq + 2], acc[4 * rq + 3]);
            if (SENTINEL) lds_barrier(); else __syncthreads();
            // this thread's rows are EPT/4 whole float4 of each wavefront's partial tile; all are read
            // before any is added so that the LDS round trips overlap
            static_assert(EPT % 4 == 0, "rows per thread come in groups of four accumulator registers");
            float4 part[NW][EPT / 4];
#pragma unroll
            for (int w2 = 0; w2 < NW; ++w2)
#pragma unroll
                for (int e4 = 0; e4 < EPT / 4; ++e4) part[w2][e4] = l4[(w2 * 4 + (EPT / 4) * wave + e4) * 64 + lane];
#pragma unroll
            for (int w2 = 0; w2 < NW; ++w2)
#pragma unroll
                for (int e4 = 0; e4 < EPT / 4; ++e4) {
                    const float4 v = part[w2][e4];
                    dh[4 * e4] += v.x; dh[4 * e4 + 1] += v.y; dh[4 * e4 + 2] += v.z; dh[4 * e4 + 3] += v.w;
                }
        }
        float dcr[EPT];
#pragma unroll
        for (int e = 0; e < EPT; ++e) dcr[e] = (ntl == 1) ? dccarry[e] : cur.dcr[e];
        float cthis[EPT];
#pragma unroll
        for (int e = 0; e < EPT; ++e) cthis[e] = (ntl == 1 && item > 0) ? ccarry[e] : cur.c[e];
        if (KW > 128 && item + 1 < nitems) issue_inputs(item + 1, nxt);
        float dcf[EPT];
        unsigned dav[EPT][2];                             // (i, f) and (g, o) as bf16 pairs: kept for the row-major copy below
        bf16_t* dxb = a.dax + ((size_t)(t * 2 + d) * NT + (b0 >> 5)) * XA;
#pragma unroll
        for (int e = 0; e < EPT; ++e) {
            const float gi = bf2f((bf16_t)(cur.g[e].x & 0xFFFFu)), gf = bf2f((bf16_t)(cur.g[e].x >> 16));
            const float gg = bf2f((bf16_t)(cur.g[e].y & 0xFFFFu)), go = bf2f((bf16_t)(cur.g[e].y >> 16));
            const float dht = dh[e] + bf2f(dyv[e]) + poison;
            const float tc = fast_tanh(cthis[e]);
            const float dc = dht * go * (1.0f - tc * tc) + dcr[e];
            const float da_o = dht * tc * go * (1.0f - go);
            const float da_i = dc * gg * gi * (1.0f - gi);
            const float da_f = dc * cur.cp[e] * gf * (1.0f - gf);
            const float da_g = dc * gi * (1.0f - gg * gg);
            dcf[e] = dc * gf;
            dav[e][0] = (unsigned)coh_bf16(da_i) | ((unsigned)coh_bf16(da_f) << 16);
            dav[e][1] = (unsigned)coh_bf16(da_g) | ((unsigned)coh_bf16(da_o) << 16);
        }
        // A lane holds four rows of one unit; a 16-byte word of either copy of dE/da is eight units of one row.
        // Regrouped through LDS inside the wavefront (its LDS operations execute in order), every lane ends up with
        // the eight units of one (row, pair of gates): two 16-byte stores per copy instead of sixteen 2-byte ones
        // (the memory pipeline takes about as long for a 2-byte store of a wavefront as for a 16-byte one).
        static_assert(EPT == 4, "the regrouping below is written for four rows per lane");
        unsigned* xs = reinterpret_cast<unsigned*>(lds) + NW * 4 * 64 * 4 + wave * 512;
#pragma unroll
        for (int e = 0; e < EPT; ++e) {
            xs[((lh * 4 + e) * 2 + 0) * 32 + l32] = dav[e][0];
            xs[((lh * 4 + e) * 2 + 1) * 32 + l32] = dav[e][1];
        }
        const int xk = lane & 3, xq = (lane >> 2) & 1, xr = (lane >> 3) & 3, xl = lane >> 5;
        uint4 cga, cgb;                                   // gate 2 xq and gate 2 xq + 1, units 8 xk .. 8 xk + 7, row xrow
        {
            const uint4* src = reinterpret_cast<const uint4*>(xs + ((xl * 4 + xr) * 2 + xq) * 32 + 8 * xk);
            const uint4 w0 = src[0], w1 = src[1];
            cga = make_uint4(__builtin_amdgcn_perm(w0.y, w0.x, 0x05040100u), __builtin_amdgcn_perm(w0.w, w0.z, 0x05040100u),
                             __builtin_amdgcn_perm(w1.y, w1.x, 0x05040100u), __builtin_amdgcn_perm(w1.w, w1.z, 0x05040100u));
            cgb = make_uint4(__builtin_amdgcn_perm(w0.y, w0.x, 0x07060302u), __builtin_amdgcn_perm(w0.w, w0.z, 0x07060302u),
                             __builtin_amdgcn_perm(w1.y, w1.x, 0x07060302u), __builtin_amdgcn_perm(w1.w, w1.z, 0x07060302u));
        }
        const int xrow = 2 * EPT * wave + 4 * xl + xr;    // row of the tile
        const bool xok = FULL || b0 + xrow < B;
        const unsigned xcol = (unsigned)(2 * xq * H + u * 32 + 8 * xk);   // column of gate 2 xq within the direction; + H: gate 2 xq + 1
        if (xok) {
            bf16_t* pa = dxb + ((xcol >> 3) * 256u + (unsigned)xrow * 8u);
            bf16_t* pb = dxb + (((xcol + (unsigned)H) >> 3) * 256u + (unsigned)xrow * 8u);
            if (SENTINEL) { st_coh_16B(pa, cga); st_coh_16B(pb, cgb); }
            else { *reinterpret_cast<uint4*>(pa) = cga; *reinterpret_cast<uint4*>(pb) = cgb; }
        }
        if (KW <= 128 && item + 1 < nitems) issue_inputs(item + 1, nxt);
        if (SENTINEL) lds_barrier();
        else signal_counter(cnt + i);
        // row-major dE/da for the weight- and input-gradient products, and the carried dE/dc
        bf16_t* dab = a.da + ((size_t)t * B + b0) * 8 * H;
        if (xok) {
            bf16_t* pr = dab + ((unsigned)xrow * (unsigned)(8 * H) + (unsigned)(d * 4 * H) + xcol);
            *reinterpret_cast<uint4*>(pr) = cga;
            *reinterpret_cast<uint4*>(pr + H) = cgb;
        }
        if (ntl > 1)                                      // carried dE/dc of the lane's four cells: one 16-byte word
            reinterpret_cast<float4*>(a.dc)[((size_t)(d * NT + (b0 >> 5)) * NU + u) * 256 + threadIdx.x] = make_float4(dcf[0], dcf[1], dcf[2], dcf[3]);
        // next item's inputs; with one tile per workgroup its carried dE/dc is the one just computed
#pragma unroll
        for (int e = 0; e < EPT; ++e) { dccarry[e] = dcf[e]; ccarry[e] = cur.cp[e]; }
    };
    if constexpr (KW <= 128) {
        for (int item = 0; item < nitems; item += 2) {
            do_item(item, in0, in1);
            if (item + 1 < nitems) do_item(item + 1, in1, in0);
        }
    } else {
        for (int item = 0; item < nitems; ++item) {
            do_item(item, in0, in1);
            in0 = in1;
        }
    }
}

// U_h [4H][H] -> U_h^T [H][4H], 32x32 tiles through LDS; blockIdx.z = 2 * layer + direction.
__global__ __launch_bounds__(256) void transpose_uh_kernel(TransposeUhArgs a, int H) {
    __shared__ bf16_t tile[32][33];
    const bf16_t* src = a.src[blockIdx.z];
    bf16_t* dst = a.dst + (size_t)blockIdx.z * 4 * H * H;
    const int r0 = blockIdx.y * 32, c0 = blockIdx.x * 32;     // rows of U_h (4H), columns (H)
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    for (int rr = ty; rr < 32; rr += 8) tile[rr][tx] = src[(size_t)(r0 + rr) * H + c0 + tx];
    __syncthreads();
    for (int rr = ty; rr < 32; rr += 8) dst[(size_t)(c0 + rr) * 4 * H + r0 + tx] = tile[tx][rr];
}

// dst[r][0..cols_p) = src[r][0..cols) followed by zeros: one thread per 8-column chunk, grid-stride.
__global__ __launch_bounds__(256) void pad_cols_kernel(PadColsArgs a) {
    const int k = blockIdx.y;
    const unsigned short* src = a.src[k];
    unsigned short* dst = a.dst[k];
    const long long ld = a.ld[k];
    const int cpr = a.cols_p >> 3;
    const long long n = (long long)a.rows[k] * cpr;
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (long long)gridDim.x * blockDim.x) {
        const long long r = i / cpr;
        const int c = (int)(i - r * cpr) * 8;
        uint4 out;
        const unsigned short* p = src + r * ld + c;
        if (c + 8 <= a.cols && (reinterpret_cast<uintptr_t>(p) & 7) == 0) {      // whole chunk, 8-byte aligned: two loads
            const uint2 lo = *reinterpret_cast<const uint2*>(p), hi = *reinterpret_cast<const uint2*>(p + 4);
            out = make_uint4(lo.x, lo.y, hi.x, hi.y);
        } else {
            unsigned short v[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = (c + e < a.cols) ? p[e] : (unsigned short)0;
            out = make_uint4(v[0] | ((unsigned)v[1] << 16), v[2] | ((unsigned)v[3] << 16), v[4] | ((unsigned)v[5] << 16), v[6] | ((unsigned)v[7] << 16));
        }
        *reinterpret_cast<uint4*>(dst + r * a.cols_p + c) = out;
    }
}

// p[0..n) = v for 16-byte words, grid-stride.
__global__ __launch_bounds__(256) void fill_u128_kernel(uint4* p, size_t n, unsigned v) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    const uint4 w = make_uint4(v, v, v, v);
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) p[i] = w;
}
__global__ void fill_u32_kernel(unsigned* p, int n, unsigned v) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

// Whether `grid` workgroups of this kernel can be resident at once (the persistent kernels wait on each other).  The
// attribute call and the occupancy query are made once per kernel instantiation and thread; the answer depends on
// the kernel and the device only, so it is kept (cache: per instantiation, one slot).
struct FitCache { bool known; int per_device; };
template <typename K>
hipError_t prepare(K kernel, int threads, size_t dyn_lds, int grid, FitCache* cache, bool* fits) {
    if (!cache->known) {
        int dev = 0, cus = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e != hipSuccess) return e;
        e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
        if (e != hipSuccess) return e;
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)dyn_lds);
        if (e != hipSuccess) return e;
        int per_cu = 0;
        e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, threads, dyn_lds);
        if (e != hipSuccess) return e;
        cache->per_device = per_cu * cus;
        cache->known = true;
    }
    *fits = cache->per_device >= grid;
    return hipSuccess;
}

template <int NW, int KW, bool S, bool FULL, bool MULTI>
hipError_t run_fwd_m(const RecFwdArgs& a, int grid, hipStream_t st, bool* launched) {
    const size_t lds = (size_t)NW * 4 * 4 * 64 * 16 + (size_t)NW * 512;   // partial sums; regrouping of h, 512 bytes per wavefront
    bool fits = false;
    static thread_local FitCache cache{false, 0};
    hipError_t e = prepare(rec_fwd_kernel<NW, KW, S, FULL, MULTI>, 64 * NW, lds, grid, &cache, &fits);
    if (e != hipSuccess || !fits) return e;
    hipLaunchKernelGGL((rec_fwd_kernel<NW, KW, S, FULL, MULTI>), dim3(grid), dim3(64 * NW), lds, st, a);
    *launched = true;
    return hipGetLastError();
}
template <int NW, int KW, bool S, bool FULL>
hipError_t run_fwd_as(const RecFwdArgs& a, int grid, hipStream_t st, bool* launched) {
    return a.tiles_per_group > 1 ? run_fwd_m<NW, KW, S, FULL, true>(a, grid, st, launched) : run_fwd_m<NW, KW, S, FULL, false>(a, grid, st, launched);
}
template <int NW, int KW, bool S>
hipError_t run_fwd(const RecFwdArgs& a, int grid, hipStream_t st, bool* launched) {
    return a.B % 32 == 0 ? run_fwd_as<NW, KW, S, true>(a, grid, st, launched) : run_fwd_as<NW, KW, S, false>(a, grid, st, launched);
}
template <int NW, int KW, bool S, bool FULL, bool MULTI>
hipError_t run_bwd_m(const RecBwdArgs& a, int grid, hipStream_t st, bool* launched) {
    const size_t lds = (size_t)NW * 4 * 64 * 16 + (size_t)NW * 2048 + (size_t)NW * 512;   // partial sums; regrouping of dE/da, 2 KB per wavefront; spreading dy, 512 bytes per wavefront
    bool fits = false;
    static thread_local FitCache cache{false, 0};
    hipError_t e = prepare(rec_bwd_kernel<NW, KW, S, FULL, MULTI>, 64 * NW, lds, grid, &cache, &fits);
    if (e != hipSuccess || !fits) return e;
    hipLaunchKernelGGL((rec_bwd_kernel<NW, KW, S, FULL, MULTI>), dim3(grid), dim3(64 * NW), lds, st, a);
    *launched = true;
    return hipGetLastError();
}
template <int NW, int KW, bool S, bool FULL>
hipError_t run_bwd_as(const RecBwdArgs& a, int grid, hipStream_t st, bool* launched) {
    return a.tiles_per_group > 1 ? run_bwd_m<NW, KW, S, FULL, true>(a, grid, st, launched) : run_bwd_m<NW, KW, S, FULL, false>(a, grid, st, launched);
}
template <int NW, int KW, bool S>
hipError_t run_bwd(const RecBwdArgs& a, int grid, hipStream_t st, bool* launched) {
    return a.B % 32 == 0 ? run_bwd_as<NW, KW, S, true>(a, grid, st, launched) : run_bwd_as<NW, KW, S, false>(a, grid, st, launched);
}

}  // namespace

// Supported widths: H = 128, 256, 512 and 1024, always on four wavefronts that split the contraction
// (32, 64, 128, 256 elements each: four batch rows per thread in every variant).  At H = 1024 the U_h
// slice fills 256 registers per lane, which leaves no room for the predicates of a ragged batch, so
// that width needs B to be a multiple of 32.  Returns the wavefronts per workgroup, 0 if unsupported.
// Whether the forward kernel for this width also fills RecFwdArgs::fill (the widest one has no register to spare).
bool rec_fwd_fills(int H) { return H == 128 || H == 256 || H == 512; }

int rec_waves_for(int H, int B) {
    if (H == 128 || H == 256 || H == 512) return 4;
    if (H == 1024 && B % 32 == 0) return 4;
    return 0;
}

hipError_t launch_fill_u32(unsigned* p, int n, unsigned v, hipStream_t st) {
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(fill_u32_kernel, dim3((n + 255) / 256), dim3(256), 0, st, p, n, v);
    return hipGetLastError();
}

hipError_t launch_fill_bytes16(void* p, size_t bytes, unsigned v, hipStream_t st) {
    const size_t n = bytes / 16;
    if (n == 0) return hipSuccess;
    size_t blocks = (n + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(fill_u128_kernel, dim3((unsigned)blocks), dim3(256), 0, st, static_cast<uint4*>(p), n, v);
    return hipGetLastError();
}

hipError_t launch_pad_cols(const PadColsArgs& a, hipStream_t st) {
    if (a.count <= 0) return hipSuccess;
    long long most = 0;
    for (int k = 0; k < a.count; ++k) { const long long n = (long long)a.rows[k] * (a.cols_p / 8); if (n > most) most = n; }
    if (most == 0) return hipSuccess;
    long long blocks = (most + 255) / 256;
    if (blocks > 2048) blocks = 2048;
    hipLaunchKernelGGL(pad_cols_kernel, dim3((unsigned)blocks, (unsigned)a.count), dim3(256), 0, st, a);
    return hipGetLastError();
}

hipError_t launch_transpose_uh(const TransposeUhArgs& a, int H, hipStream_t st) {
    if (a.count <= 0) return hipSuccess;
    hipLaunchKernelGGL(transpose_uh_kernel, dim3(H / 32, 4 * H / 32, a.count), dim3(256), 0, st, a, H);
    return hipGetLastError();
}

hipError_t launch_rec_fwd(const RecFwdArgs& a, bool sentinel, hipStream_t st, bool* launched) {
    *launched = false;
    const int grid = 2 * a.nbg * (a.H / 32);
    switch (a.H) {
        case 128: return sentinel ? run_fwd<4, 32, true>(a, grid, st, launched) : run_fwd<4, 32, false>(a, grid, st, launched);
        case 256: return sentinel ? run_fwd<4, 64, true>(a, grid, st, launched) : run_fwd<4, 64, false>(a, grid, st, launched);
        case 512: return sentinel ? run_fwd<4, 128, true>(a, grid, st, launched) : run_fwd<4, 128, false>(a, grid, st, launched);
        case 1024:
            if (a.B % 32 != 0) return hipSuccess;
            return sentinel ? run_fwd_as<4, 256, true, true>(a, grid, st, launched) : run_fwd_as<4, 256, false, true>(a, grid, st, launched);
        default: return hipSuccess;
    }
}

hipError_t launch_rec_bwd(const RecBwdArgs& a, bool sentinel, hipStream_t st, bool* launched) {
    *launched = false;
    const int grid = 2 * a.nbg * (a.H / 32);
    switch (a.H) {
        case 128: return sentinel ? run_bwd<4, 32, true>(a, grid, st, launched) : run_bwd<4, 32, false>(a, grid, st, launched);
        case 256: return sentinel ? run_bwd<4, 64, true>(a, grid, st, launched) : run_bwd<4, 64, false>(a, grid, st, launched);
        case 512: return sentinel ? run_bwd<4, 128, true>(a, grid, st, launched) : run_bwd<4, 128, false>(a, grid, st, launched);
        case 1024:
            if (a.B % 32 != 0) return hipSuccess;
            return sentinel ? run_bwd_as<4, 256, true, true>(a, grid, st, launched) : run_bwd_as<4, 256, false, true>(a, grid, st, launched);
        default: return hipSuccess;
    }
}

}  // namespace blstm
