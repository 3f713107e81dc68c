// C-ABI of the library: argument validation, parameter and workspace layout, and the
// launch order of one training step.  Host code only; every step of the path runs in the
// kernels of gemm.hip, cell.hip, softmax.hip and update.hip.
#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "../../include/blstm_mi355.h"
#include "gemm.hpp"
#include "kernels.hpp"

using namespace blstm;

namespace {

thread_local std::string g_err;

int fail(int code, const char* fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_err = buf;
    return code;
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }
inline size_t up256(size_t v) { return (v + 255) & ~size_t(255); }

enum ProfClass {
    PC_GEMM_INPUT = 0, PC_GEMM_REC_FWD, PC_CELL_FWD, PC_GEMM_BOTTLENECK, PC_GEMM_LOGITS, PC_SOFTMAX_ROWS,
    PC_GEMM_SOFTMAX_BWD, PC_GEMM_REC_BWD, PC_CELL_BWD, PC_GEMM_WGRAD, PC_GEMM_DGRAD, PC_MISC,
    PC_REC_FWD, PC_REC_BWD, PC_COUNT
};
const char* const kProfNames[PC_COUNT] = {
    "gemm_input_projection", "gemm_recurrent_fwd", "cell_fwd", "gemm_bottleneck", "gemm_logits", "softmax_rows",
    "gemm_softmax_bwd", "gemm_recurrent_bwd", "cell_bwd", "gemm_wgrad", "gemm_dgrad", "misc",
    "recurrent_fwd_persistent", "recurrent_bwd_persistent"};

struct ProfRec { hipEvent_t a, b; int cls; };

}  // namespace

struct blstm_ctx {
    blstm_config cfg;
    int T, B, D, H, L, P, V, M, zdim;
    DType st;                 // storage type of activations and of theta as seen by forward/backward
    size_t esz;               // bytes per stored element
    float s;
    size_t nparam;
    std::vector<size_t> off_wx[2], off_uh[2], off_b[2];
    size_t off_wp, off_bp, off_ws, off_bs;
    // workspace (byte offsets)
    std::vector<size_t> wY, wG, wC;
    std::vector<size_t> wDA;  // dE/da of every layer: all of them feed the weight-gradient products at the end of the backward pass
    size_t wAX, wPRE, wDY[2], wDH, wDC, wLOGITS, wROWLOSS, wUHT, wCNT, wPART, wHX, wDAX, hx_bytes, dax_bytes, part_bytes, ws_bytes;
    int Dp;                   // 0, or the first layer's input width rounded up to whole tiles (padded copies of x and W_x)
    size_t wXP, wWP;
    int rec_nbg, rec_tiles;   // batch groups per direction and 32-row tiles per group of the persistent kernels
    int rec_path;             // 0 = persistent kernels where supported, 1 = one launch per frame
    int rec_sync;             // exchange of the persistent kernels: 0 = fenced counters, 1 = sentinel-tagged data
    bool dax_filled;          // the forward pass's persistent kernels have marked every exchange copy of dE/da "not written yet"
    bool abort_clean;         // the abort word has been zeroed since the workspace was bound
    bool test_abort;          // failure-handling tests: the next forward pass raises the abort word itself
    bool defer_ws;            // softmax_xent_fwd_bwd leaves dW_s and db_s to the next blstm_backward's grouped launch
    const void* pend_z;       // ... and has done so: the z it was given (null: nothing pending) and the gradient vector
    float* pend_grad;
    bool keep_copies;         // the caller reports weight changes (blstm_weights_changed): derived copies are kept across steps
    const void* wxp_of;       // the weights the padded W_x of layer 0 was made from (null: to be made), likewise the transposed U_h
    const void* uht_of;
    char* ws;
    size_t ws_bound;
    bool have_forward;
    std::vector<char> fwd_persistent;   // per layer: the forward pass ran the persistent kernel (whose saved gates only its backward twin reads)
    // profiling
    bool prof;
    std::vector<ProfRec> recs;
    size_t recs_used;
    double prof_ms[PC_COUNT];
    int64_t prof_n[PC_COUNT];

    int din(int l) const { return l == 0 ? D : 2 * H; }
};

namespace {

struct Scope {                // records a pair of events around one launch when profiling is on
    blstm_ctx* c; hipStream_t s; int cls; ProfRec* r;
    Scope(blstm_ctx* c_, hipStream_t s_, int cls_) : c(c_), s(s_), cls(cls_), r(nullptr) {
        if (!c->prof) return;
        if (c->recs_used == c->recs.size()) {
            ProfRec n{};
            if (hipEventCreate(&n.a) != hipSuccess || hipEventCreate(&n.b) != hipSuccess) return;
            c->recs.push_back(n);
        }
        r = &c->recs[c->recs_used++];
        r->cls = cls;
        (void)hipEventRecord(r->a, s);
    }
    ~Scope() { if (r) (void)hipEventRecord(r->b, s); }
};

int check_hip(hipError_t e, const char* what) {
    if (e == hipSuccess) return BLSTM_OK;
    return fail(BLSTM_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

#define RUN(cls, what, expr)                                         \
    do {                                                             \
        hipError_t e_;                                               \
        { Scope sc_(ctx, st, cls); e_ = (expr); }                    \
        if (e_ != hipSuccess) return check_hip(e_, what);            \
    } while (0)

GemmDesc gemm_desc(const blstm_ctx* c, DType in, DType out) {
    GemmDesc d{};
    d.nseg = 1; d.batch = 1; d.in_type = in; d.out_type = out;
    d.partial = reinterpret_cast<float*>(c->ws + c->wPART);
    d.partial_bytes = c->part_bytes;
    return d;
}

inline const char* at(const void* base, size_t elems, size_t esz) { return static_cast<const char*>(base) + elems * esz; }
inline char* at(void* base, size_t elems, size_t esz) { return static_cast<char*>(base) + elems * esz; }


// Scratch of the softmax cross-entropy: the logit matrix [M][V] (storage type, overwritten in place by dE/du),
// one loss term per frame, and the float partial tiles of products split along K.
struct SoftmaxScratch { char* logits; float* row_loss; float* partial; size_t partial_bytes; };

// dW_s = du^T z with db_s as the row sums of du^T (du [M][V] in the storage type, left by the row kernel).
GemmDesc softmax_wgrad_desc(const blstm_ctx* ctx, const char* U, const void* z, float* grad) {
    GemmDesc d = gemm_desc(ctx, ctx->st, DT_F32);
    d.M = ctx->V; d.N = ctx->zdim; d.atrans = true; d.btrans = true;
    d.seg[0] = GemmSeg{U, z, ctx->V, ctx->zdim, 0, 0, ctx->M};
    d.C = grad + ctx->off_ws; d.ldc = ctx->zdim;
    d.rowsum = grad + ctx->off_bs;                     // db_s = sum over frames of du
    return d;
}

// defer: the W_s and b_s slices of grad are left to the next blstm_backward (the product joins its grouped launch).
int softmax_xent_run(blstm_ctx* ctx, const SoftmaxScratch& sc, const void* theta, const void* z, const int32_t* labels,
                     float* loss_dev, void* dz, float* grad, hipStream_t st, bool defer) {
    const int M = ctx->M, V = ctx->V, Z = ctx->zdim;
    const size_t e = ctx->esz;
    const DType S = ctx->st;
    char* U = sc.logits;
    auto desc = [&](DType in, DType out) {
        GemmDesc d = gemm_desc(ctx, in, out);
        d.partial = sc.partial; d.partial_bytes = sc.partial_bytes;
        return d;
    };
    {   // u = W_s z + b_s
        GemmDesc d = desc(S, S);
        d.M = M; d.N = V;
        d.seg[0] = GemmSeg{z, at(theta, ctx->off_ws, e), Z, Z, 0, 0, Z};
        d.C = U; d.ldc = V;
        d.bias = at(theta, ctx->off_bs, e);
        RUN(PC_GEMM_LOGITS, "logits", launch_gemm(d, st));
    }
    RUN(PC_SOFTMAX_ROWS, "softmax rows", launch_softmax_rows(U, V, labels, sc.row_loss, M, V, ctx->s, S, st));
    RUN(PC_MISC, "loss sum", launch_sum_to_scalar(sc.row_loss, M, loss_dev, st));
    {   // dz = du W_s
        GemmDesc d = desc(S, S);
        d.M = M; d.N = Z; d.btrans = true;
        d.seg[0] = GemmSeg{U, at(theta, ctx->off_ws, e), V, Z, 0, 0, V};
        d.C = dz; d.ldc = Z;
        RUN(PC_GEMM_SOFTMAX_BWD, "dz", launch_gemm(d, st));
    }
    if (defer) { ctx->pend_z = z; ctx->pend_grad = grad; return BLSTM_OK; }
    ctx->pend_z = nullptr;
    {   // dW_s = du^T z
        GemmDesc d = softmax_wgrad_desc(ctx, U, z, grad);
        d.partial = sc.partial; d.partial_bytes = sc.partial_bytes;
        RUN(PC_GEMM_SOFTMAX_BWD, "dW_s", launch_gemm(d, st));
    }
    return BLSTM_OK;
}

// ---- scratch that lives in the library's own code object, for callers that cannot allocate --------------------
// Each GPU the library runs on holds its own copy of this array, at its own address, until the process ends.
// In host code the array's name is only a handle for hipGetSymbolAddress: kernels are given the address that call
// returns for the current device, looked up once per device.
__device__ __align__(256) static unsigned char g_noalloc_scratch[BLSTM_NOALLOC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
char* g_scratch_ptr[kMaxDevices];                  // per device, null until looked up

int resident_scratch(char** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return check_hip(e, "hipGetDevice");
    if (dev < 0 || dev >= kMaxDevices) return fail(BLSTM_ERR_DIM, "device index %d beyond the %d this library keeps scratch for", dev, kMaxDevices);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(g_noalloc_scratch));     // the copy on the current device
        if (e != hipSuccess) return check_hip(e, "hipGetSymbolAddress");
        if (!p) return fail(BLSTM_ERR_HIP, "hipGetSymbolAddress returned a null address");
        g_scratch_ptr[dev] = static_cast<char*>(p);
    }
    *out = g_scratch_ptr[dev];
    return BLSTM_OK;
}

}  // namespace

extern "C" {

const char* blstm_last_error(void) { return g_err.c_str(); }

int blstm_create(const blstm_config* cfg, blstm_ctx** out) {
    if (!cfg || !out) return fail(BLSTM_ERR_NULL, "blstm_create: null argument");
    *out = nullptr;
    if (cfg->T < 1 || cfg->B < 1 || cfg->D < 1 || cfg->H < 1 || cfg->L < 1 || cfg->P < 0 || cfg->V < 1)
        return fail(BLSTM_ERR_DIM, "blstm_create: T,B,D,H,L,V must be >= 1 and P >= 0");
    if (cfg->mode != 0 && cfg->mode != 1) return fail(BLSTM_ERR_DIM, "blstm_create: mode must be 0 (fp32) or 1 (bf16)");
    const long long Mll = (long long)cfg->T * cfg->B;
    if (Mll > (1LL << 24) || cfg->H > (1 << 14) || cfg->D > (1 << 16) || cfg->V > (1 << 22) || cfg->P > (1 << 14) || cfg->L > 64)
        return fail(BLSTM_ERR_DIM, "blstm_create: dimension beyond the supported range");
    blstm_ctx* c = new (std::nothrow) blstm_ctx();
    if (!c) return fail(BLSTM_ERR_DIM, "blstm_create: out of host memory");
    c->cfg = *cfg;
    c->T = cfg->T; c->B = cfg->B; c->D = cfg->D; c->H = cfg->H; c->L = cfg->L; c->P = cfg->P; c->V = cfg->V;
    c->M = (int)Mll;
    c->zdim = cfg->P > 0 ? cfg->P : 2 * cfg->H;
    c->st = cfg->mode == 1 ? DT_BF16 : DT_F32;
    c->esz = cfg->mode == 1 ? 2 : 4;
    c->s = cfg->loss_scale > 0.0f ? cfg->loss_scale : 1.0f / (float)Mll;
    // flat parameter layout
    size_t off = 0;
    const size_t H = c->H;
    for (int l = 0; l < c->L; ++l)
        for (int d = 0; d < 2; ++d) {
            c->off_wx[d].push_back(off); off += 4 * H * (size_t)c->din(l);
            c->off_uh[d].push_back(off); off += 4 * H * H;
            c->off_b[d].push_back(off);  off += 4 * H;
        }
    c->off_wp = off; if (c->P > 0) off += (size_t)c->P * 2 * H;
    c->off_bp = off; if (c->P > 0) off += (size_t)c->P;
    c->off_ws = off; off += (size_t)c->V * c->zdim;
    c->off_bs = off; off += (size_t)c->V;
    c->nparam = off;
    // workspace layout
    const size_t M = (size_t)c->M, B = (size_t)c->B, e = c->esz;
    const size_t Br = (B + 31) / 32 * 32, Mr = (size_t)c->T * Br;      // rows rounded up to whole batch tiles
    size_t w = 0;
    for (int l = 0; l < c->L; ++l) { c->wY.push_back(w); w += up256(M * 2 * H * e); }
    for (int l = 0; l < c->L; ++l) {
        // (whole 32-row batch tiles: the persistent kernels keep these two as per-lane records)
        c->wG.push_back(w); w += up256(Mr * 8 * H * e);
        c->wC.push_back(w); w += up256(Mr * 2 * H * 4);
    }
    c->wAX = w;      w += up256(M * 8 * H * 4);
    c->wPRE = w;     w += up256(2 * B * 4 * H * 4);
    for (int l = 0; l < c->L; ++l) { c->wDA.push_back(w); w += up256(M * 8 * H * e); }
    c->wDY[0] = w;   w += up256(M * 2 * H * e);
    c->wDY[1] = w;   w += up256(M * 2 * H * e);
    c->wDH = w;      w += up256(2 * B * H * 4);
    c->wDC = w;      w += up256(2 * Br * H * 4);
    c->wLOGITS = w;  w += up256(M * (size_t)c->V * e);
    c->wROWLOSS = w; w += up256(M * 4);
    // A feature width that is not a whole number of tiles (the paper's 260) would put the first layer's two
    // products on the guarded kernel, three times slower: zero-padded bf16 copies of x and of W_x of layer 0
    // (a few MB) keep them on the unguarded one.
    c->Dp = 0; c->wXP = w; c->wWP = w;
    if (c->st == DT_BF16 && c->D % 128 != 0 && c->M % 128 == 0 && (4 * c->H) % 128 == 0) {
        c->Dp = (c->D + 127) / 128 * 128;
        c->wXP = w; w += up256(M * (size_t)c->Dp * 2);
        c->wWP = w; w += up256((size_t)2 * 4 * H * c->Dp * 2);
    }
    // persistent recurrent kernels: transposed U_h per layer and direction, counters, abort word
    c->rec_nbg = 0; c->rec_tiles = 0; c->rec_path = 0; c->rec_sync = 1; c->abort_clean = false; c->test_abort = false;
    c->dax_filled = false;
    c->fwd_persistent.assign(c->L, 0);
    c->wUHT = w; c->wCNT = w; c->wHX = w; c->wDAX = w; c->hx_bytes = 0; c->dax_bytes = 0;
    if (c->st == DT_BF16 && rec_waves_for(c->H, c->B) > 0) {
        const int NU = c->H / 32, tiles = (c->B + 31) / 32;
        int nbg = 256 / (2 * NU);
        if (nbg > tiles) nbg = tiles;
        if (nbg < 1) nbg = 1;
        c->rec_nbg = nbg;
        c->rec_tiles = (tiles + nbg - 1) / nbg;
        w += up256((size_t)c->L * 2 * 4 * H * H * 2);
        c->wCNT = w;
        w += up256(((size_t)2 * nbg * c->rec_tiles + 64) * 4);
        // exchange copies of h and dE/da in MFMA-fragment order, one per layer (whole 32-row tiles),
        // contiguous so that one fill marks all of a pass's copies as "not written yet"
        const size_t Mx = (size_t)c->T * tiles * 32;
        c->hx_bytes = up256(Mx * 2 * H * 2);
        c->dax_bytes = up256(Mx * 8 * H * 2);
        c->wHX = w;  w += c->hx_bytes * c->L;
        c->wDAX = w; w += c->dax_bytes * c->L;
    }
    {   // split-K scratch: the largest need among the products with a small output
        const DType S = c->st;
        size_t need = 0;
        auto upd = [&](int m, int n, int k, int batch) { size_t b = gemm_partial_bytes(m, n, k, batch, S); if (b > need) need = b; };
        upd(c->M, c->zdim, c->V, 1);                              // dz
        upd(c->V, c->zdim, c->M, 1);                              // dW_s
        if (c->P > 0) { upd(c->P, 2 * c->H, c->M, 1); upd(c->M, 2 * c->H, c->P, 1); }
        for (int l = 0; l < c->L; ++l) { upd(4 * c->H, c->din(l), c->M, 2); upd(4 * c->H, c->H, (c->T - 1) * c->B, 2); }
        upd(c->B, c->H, 4 * c->H, 2);                             // recurrent gradient of the step-by-step path
        c->wPART = w; c->part_bytes = up256(need);
        w += c->part_bytes;
    }
    c->keep_copies = false; c->wxp_of = nullptr; c->uht_of = nullptr;
    c->defer_ws = false; c->pend_z = nullptr; c->pend_grad = nullptr;
    c->ws_bytes = w;
    c->ws = nullptr; c->ws_bound = 0; c->have_forward = false;
    c->prof = false; c->recs_used = 0;
    memset(c->prof_ms, 0, sizeof c->prof_ms);
    memset(c->prof_n, 0, sizeof c->prof_n);
    *out = c;
    return BLSTM_OK;
}

void blstm_destroy(blstm_ctx* c) {
    if (!c) return;
    for (auto& r : c->recs) { (void)hipEventDestroy(r.a); (void)hipEventDestroy(r.b); }
    delete c;
}

size_t blstm_param_count(const blstm_ctx* c) { return c ? c->nparam : 0; }
size_t blstm_workspace_bytes(const blstm_ctx* c) { return c ? c->ws_bytes : 0; }

int blstm_param_offset(const blstm_ctx* c, int layer, int dir, int which, size_t* off, size_t* len) {
    if (!c || !off || !len) return fail(BLSTM_ERR_NULL, "blstm_param_offset: null argument");
    const size_t H = c->H;
    if (which >= BLSTM_WX && which <= BLSTM_B) {
        if (layer < 0 || layer >= c->L || dir < 0 || dir > 1) return fail(BLSTM_ERR_DIM, "blstm_param_offset: layer/dir out of range");
        if (which == BLSTM_WX) { *off = c->off_wx[dir][layer]; *len = 4 * H * (size_t)c->din(layer); }
        else if (which == BLSTM_UH) { *off = c->off_uh[dir][layer]; *len = 4 * H * H; }
        else { *off = c->off_b[dir][layer]; *len = 4 * H; }
        return BLSTM_OK;
    }
    switch (which) {
        case BLSTM_WP: *off = c->off_wp; *len = c->P > 0 ? (size_t)c->P * 2 * H : 0; return BLSTM_OK;
        case BLSTM_BP: *off = c->off_bp; *len = c->P > 0 ? (size_t)c->P : 0; return BLSTM_OK;
        case BLSTM_WS: *off = c->off_ws; *len = (size_t)c->V * c->zdim; return BLSTM_OK;
        case BLSTM_BS: *off = c->off_bs; *len = (size_t)c->V; return BLSTM_OK;
    }
    return fail(BLSTM_ERR_DIM, "blstm_param_offset: unknown tensor id %d", which);
}

int blstm_bind(blstm_ctx* c, void* workspace, size_t bytes) {
    if (!c || !workspace) return fail(BLSTM_ERR_NULL, "blstm_bind: null argument");
    if (!aligned16(workspace)) return fail(BLSTM_ERR_ALIGN, "blstm_bind: workspace must be 16-byte aligned");
    if (bytes < c->ws_bytes) return fail(BLSTM_ERR_WORKSPACE, "blstm_bind: %zu bytes given, %zu needed", bytes, c->ws_bytes);
    c->ws = static_cast<char*>(workspace);
    c->ws_bound = bytes;
    c->have_forward = false;
    c->abort_clean = false;
    c->wxp_of = nullptr; c->uht_of = nullptr;
    c->pend_z = nullptr;
    return BLSTM_OK;
}

int blstm_forward(blstm_ctx* ctx, const void* theta, const void* x, void* z_out, void* stream) {
    if (!ctx || !theta || !x || !z_out) return fail(BLSTM_ERR_NULL, "blstm_forward: null argument");
    if (!ctx->ws) return fail(BLSTM_ERR_WORKSPACE, "blstm_forward: no workspace bound");
    if (!aligned16(theta) || !aligned16(x) || !aligned16(z_out)) return fail(BLSTM_ERR_ALIGN, "blstm_forward: pointers must be 16-byte aligned");
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int T = ctx->T, B = ctx->B, H = ctx->H, M = ctx->M;
    const size_t e = ctx->esz;
    const DType S = ctx->st;
    float* AX = reinterpret_cast<float*>(ctx->ws + ctx->wAX);
    float* PRE = reinterpret_cast<float*>(ctx->ws + ctx->wPRE);
    ctx->have_forward = false;
    ctx->dax_filled = false;
    ctx->pend_z = nullptr;                              // (a softmax weight gradient left over from an earlier step is dropped)
    const bool persistent = ctx->rec_nbg > 0 && ctx->rec_path == 0;
    if (persistent && ctx->rec_sync == 1)    // h of every layer starts as "not written yet"
        RUN(PC_MISC, "sentinel fill of h", launch_fill_bytes16(ctx->ws + ctx->wHX, ctx->hx_bytes * ctx->L, 0xFFFFFFFFu, st));
    for (int l = 0; l < ctx->L; ++l) {
        const void* Xin = l == 0 ? x : static_cast<const void*>(ctx->ws + ctx->wY[l - 1]);
        const int Din = ctx->din(l);
        char* Y = ctx->ws + ctx->wY[l];
        char* G = ctx->ws + ctx->wG[l];
        float* C = reinterpret_cast<float*>(ctx->ws + ctx->wC[l]);
        {   // a_x = W_x x + b for every frame, both directions
            GemmDesc d = gemm_desc(ctx, S, DT_F32);
            d.batch = 2; d.M = M; d.N = 4 * H;
            d.seg[0] = GemmSeg{Xin, at(theta, ctx->off_wx[0][l], e), Din, Din, 0,
                               (long long)(ctx->off_wx[1][l] - ctx->off_wx[0][l]), Din};
            if (l == 0 && ctx->Dp > 0) {                 // zero-padded copies: K = Dp, whole slabs
                PadColsArgs pa{};
                unsigned short* XP = reinterpret_cast<unsigned short*>(ctx->ws + ctx->wXP);
                unsigned short* WP = reinterpret_cast<unsigned short*>(ctx->ws + ctx->wWP);
                pa.src[0] = static_cast<const unsigned short*>(x); pa.dst[0] = XP; pa.ld[0] = Din; pa.rows[0] = M;
                for (int dd = 0; dd < 2; ++dd) {
                    pa.src[1 + dd] = reinterpret_cast<const unsigned short*>(at(theta, ctx->off_wx[dd][0], e));
                    pa.dst[1 + dd] = WP + (size_t)dd * 4 * H * ctx->Dp; pa.ld[1 + dd] = Din; pa.rows[1 + dd] = 4 * H;
                }
                // (the copy of W_x is kept while the caller vouches for the weights: see blstm_weights_changed)
                const bool have_wp = ctx->keep_copies && ctx->wxp_of == theta;
                pa.count = have_wp ? 1 : 3; pa.cols = Din; pa.cols_p = ctx->Dp;
                ctx->wxp_of = theta;
                RUN(PC_MISC, "padded copies of x and W_x", launch_pad_cols(pa, st));
                // (rows are Dp long for the weight gradient's whole tiles; the contraction needs whole slabs of 64 only)
                d.seg[0] = GemmSeg{XP, WP, ctx->Dp, ctx->Dp, 0, (long long)4 * H * ctx->Dp, (Din + 63) / 64 * 64};
            }
            d.C = AX; d.ldc = 8 * H; d.sC = 4 * H;
            d.bias = at(theta, ctx->off_b[0][l], e); d.sBias = (long long)(ctx->off_b[1][l] - ctx->off_b[0][l]);
            RUN(PC_GEMM_INPUT, "input projection", launch_gemm(d, st));
        }
        ctx->fwd_persistent[l] = 0;
        if (ctx->rec_nbg > 0 && ctx->rec_path == 0) {   // all T frames of both directions in one launch
            unsigned* cnt = reinterpret_cast<unsigned*>(ctx->ws + ctx->wCNT);
            const int ncnt = 2 * ctx->rec_nbg * ctx->rec_tiles;
            if (!ctx->abort_clean || ctx->test_abort) {
                RUN(PC_MISC, "abort word", launch_fill_u32(cnt + ncnt, 1, ctx->test_abort ? 1u : 0u, st));
                ctx->abort_clean = true;
                ctx->test_abort = false;
            }
            if (ctx->rec_sync == 0) RUN(PC_MISC, "counters", launch_fill_u32(cnt, ncnt, 0u, st));
            RecFwdArgs a{};
            a.uh[0] = reinterpret_cast<const unsigned short*>(at(theta, ctx->off_uh[0][l], e));
            a.uh[1] = reinterpret_cast<const unsigned short*>(at(theta, ctx->off_uh[1][l], e));
            a.ax = AX; a.y = reinterpret_cast<unsigned short*>(Y);
            a.hx = reinterpret_cast<unsigned short*>(ctx->ws + ctx->wHX + ctx->hx_bytes * l);
            a.gates = reinterpret_cast<unsigned short*>(G); a.c = C;
            a.cnt = cnt; a.abort_word = cnt + ncnt; a.limit_ticks = 200000000ull;
            a.T = T; a.B = B; a.H = H; a.nbg = ctx->rec_nbg; a.tiles_per_group = ctx->rec_tiles;
            if (ctx->rec_sync == 1 && rec_fwd_fills(H)) {   // the backward twin's exchange copy is pre-filled on the side
                a.fill = ctx->ws + ctx->wDAX + ctx->dax_bytes * l;
                a.fill_words = ctx->dax_bytes / 16;
            }
            bool launched = false;
            RUN(PC_REC_FWD, "persistent recurrent forward", launch_rec_fwd(a, ctx->rec_sync == 1, st, &launched));
            ctx->fwd_persistent[l] = launched ? 1 : 0;
            if (launched) continue;
        }
        for (int n = 0; n < T; ++n) {
            const int t[2] = {n, T - 1 - n};
            const int tp[2] = {n - 1, T - n};
            if (n > 0) {   // a = a_x + U_h h_prev
                GemmDesc d = gemm_desc(ctx, S, DT_F32);
                d.batch = 2; d.M = B; d.N = 4 * H;
                const char* A0 = Y + ((size_t)tp[0] * B * 2 * H) * e;
                const char* A1 = Y + ((size_t)tp[1] * B * 2 * H + H) * e;
                d.seg[0] = GemmSeg{A0, at(theta, ctx->off_uh[0][l], e), 2 * H, H, (long long)((A1 - A0) / (long long)e),
                                   (long long)(ctx->off_uh[1][l] - ctx->off_uh[0][l]), H};
                d.C = PRE; d.ldc = 4 * H; d.sC = (long long)B * 4 * H;
                const float* add0 = AX + (size_t)t[0] * B * 8 * H;
                const float* add1 = AX + (size_t)t[1] * B * 8 * H + 4 * H;
                d.add = add0; d.ldadd = 8 * H; d.sAdd = add1 - add0;
                RUN(PC_GEMM_REC_FWD, "recurrent product", launch_gemm(d, st));
            }
            CellFwdArgs a{};
            a.B = B; a.H = H;
            for (int dd = 0; dd < 2; ++dd) {
                if (n > 0) { a.pre[dd] = PRE + (size_t)dd * B * 4 * H; a.ld_pre = 4 * H; }
                else { a.pre[dd] = AX + (size_t)t[dd] * B * 8 * H + (size_t)dd * 4 * H; a.ld_pre = 8 * H; }
                a.c_prev[dd] = n > 0 ? C + (size_t)tp[dd] * B * 2 * H + (size_t)dd * H : nullptr;
                a.c[dd] = C + (size_t)t[dd] * B * 2 * H + (size_t)dd * H;
                a.gates[dd] = G + ((size_t)t[dd] * B * 8 * H + (size_t)dd * 4 * H) * e;
                a.y[dd] = Y + ((size_t)t[dd] * B * 2 * H + (size_t)dd * H) * e;
            }
            RUN(PC_CELL_FWD, "cell forward", launch_cell_fwd(a, S, st));
        }
    }
    const char* YL = ctx->ws + ctx->wY[ctx->L - 1];
    if (ctx->P > 0) {
        GemmDesc d = gemm_desc(ctx, S, S);
        d.M = M; d.N = ctx->P;
        d.seg[0] = GemmSeg{YL, at(theta, ctx->off_wp, e), 2 * H, 2 * H, 0, 0, 2 * H};
        d.C = z_out; d.ldc = ctx->P;
        d.bias = at(theta, ctx->off_bp, e);
        RUN(PC_GEMM_BOTTLENECK, "bottleneck", launch_gemm(d, st));
    } else {
        RUN(PC_MISC, "copy of the LSTM output", hipMemcpyAsync(z_out, YL, (size_t)M * 2 * H * e, hipMemcpyDeviceToDevice, st));
    }
    ctx->have_forward = true;
    ctx->dax_filled = persistent && ctx->rec_sync == 1 && rec_fwd_fills(H);
    return BLSTM_OK;
}

int softmax_xent_fwd_bwd(blstm_ctx* ctx, const void* theta, const void* z, const int32_t* labels,
                         float* loss_dev, void* dz, float* grad, void* stream) {
    if (!ctx || !theta || !z || !labels || !loss_dev || !dz || !grad) return fail(BLSTM_ERR_NULL, "softmax_xent_fwd_bwd: null argument");
    if (!ctx->ws) return fail(BLSTM_ERR_WORKSPACE, "softmax_xent_fwd_bwd: no workspace bound");
    if (!aligned16(theta) || !aligned16(z) || !aligned16(dz) || !aligned16(grad))
        return fail(BLSTM_ERR_ALIGN, "softmax_xent_fwd_bwd: pointers must be 16-byte aligned");
    SoftmaxScratch sc{ctx->ws + ctx->wLOGITS, reinterpret_cast<float*>(ctx->ws + ctx->wROWLOSS),
                      reinterpret_cast<float*>(ctx->ws + ctx->wPART), ctx->part_bytes};
    return softmax_xent_run(ctx, sc, theta, z, labels, loss_dev, dz, grad, static_cast<hipStream_t>(stream), ctx->defer_ws);
}

int softmax_xent_fwd_bwd_noalloc(blstm_ctx* ctx, const void* theta, const void* z, const int32_t* labels,
                                 float* loss_dev, void* dz, float* grad, void* stream) {
    if (!ctx || !theta || !z || !labels || !loss_dev || !dz || !grad) return fail(BLSTM_ERR_NULL, "softmax_xent_fwd_bwd_noalloc: null argument");
    if (!aligned16(theta) || !aligned16(z) || !aligned16(dz) || !aligned16(grad))
        return fail(BLSTM_ERR_ALIGN, "softmax_xent_fwd_bwd_noalloc: pointers must be 16-byte aligned");
    // layout of the resident array: logits, row losses, split-K partial tiles (whatever is left)
    const size_t logits = up256((size_t)ctx->M * (size_t)ctx->V * ctx->esz), rows = up256((size_t)ctx->M * 4);
    size_t part = gemm_partial_bytes(ctx->M, ctx->zdim, ctx->V, 1, ctx->st);
    const size_t part2 = gemm_partial_bytes(ctx->V, ctx->zdim, ctx->M, 1, ctx->st);
    if (part2 > part) part = part2;
    part = up256(part);
    if (logits + rows + part > BLSTM_NOALLOC_SCRATCH_BYTES)
        return fail(BLSTM_ERR_WORKSPACE, "softmax_xent_fwd_bwd_noalloc: T*B = %d frames of V = %d classes need %zu bytes of scratch, "
                    "the resident array holds %zu", ctx->M, ctx->V, logits + rows + part, (size_t)BLSTM_NOALLOC_SCRATCH_BYTES);
    char* base = nullptr;
    const int rc = resident_scratch(&base);
    if (rc != BLSTM_OK) return rc;
    SoftmaxScratch sc{base, reinterpret_cast<float*>(base + logits), reinterpret_cast<float*>(base + logits + rows),
                      BLSTM_NOALLOC_SCRATCH_BYTES - logits - rows};
    return softmax_xent_run(ctx, sc, theta, z, labels, loss_dev, dz, grad, static_cast<hipStream_t>(stream), false);
}

int blstm_backward(blstm_ctx* ctx, const void* theta, const void* x, const void* dz, float* grad, void* stream) {
    if (!ctx || !theta || !x || !dz || !grad) return fail(BLSTM_ERR_NULL, "blstm_backward: null argument");
    if (!ctx->ws) return fail(BLSTM_ERR_WORKSPACE, "blstm_backward: no workspace bound");
    if (!ctx->have_forward) return fail(BLSTM_ERR_WORKSPACE, "blstm_backward: no forward pass is held in the workspace");
    if (!aligned16(theta) || !aligned16(x) || !aligned16(dz) || !aligned16(grad))
        return fail(BLSTM_ERR_ALIGN, "blstm_backward: pointers must be 16-byte aligned");
    if (ctx->pend_z && ctx->pend_grad != grad)
        return fail(BLSTM_ERR_DIM, "blstm_backward: the softmax layer's weight gradient was left to this call for another gradient vector");
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int T = ctx->T, B = ctx->B, H = ctx->H, M = ctx->M, P = ctx->P;
    const size_t e = ctx->esz;
    const DType S = ctx->st;
    float* DH = reinterpret_cast<float*>(ctx->ws + ctx->wDH);
    float* DC = reinterpret_cast<float*>(ctx->ws + ctx->wDC);
    // The weight-gradient products only feed the gradient vector and depend on nothing but each layer's dE/da, so
    // they are collected here and run as one grouped launch at the end (every layer keeps its own dE/da buffer): one
    // by one most of them have too few tiles for the device, together they fill it.  (Running a layer's products on
    // a second stream beside the next layer's recurrence was measured and dropped: sharing the CUs slows the
    // recurrence, a chain of latencies, by more than the products gain.)
    std::vector<GemmDesc> wgrads;
    wgrads.reserve(2 * ctx->L + 2);
    bool persistent = false;                            // some layer's forward pass ran the persistent kernel
    for (int l = 0; l < ctx->L; ++l) persistent = persistent || ctx->fwd_persistent[l] != 0;
    const bool sentinel = persistent && ctx->rec_sync == 1;
    if (persistent && !(ctx->keep_copies && ctx->uht_of == theta)) {   // U_h^T of every layer and direction in one launch
        TransposeUhArgs ta{};
        for (int l = 0; l < ctx->L; ++l)
            for (int d = 0; d < 2; ++d)
                ta.src[2 * l + d] = reinterpret_cast<const unsigned short*>(at(theta, ctx->off_uh[d][l], e));
        ta.dst = reinterpret_cast<unsigned short*>(ctx->ws + ctx->wUHT);
        ta.count = 2 * ctx->L;
        RUN(PC_MISC, "U_h transposes", launch_transpose_uh(ta, H, st));
        ctx->uht_of = theta;
    }
    // In sentinel mode every layer's exchange copy of dE/da starts as "not written yet": the forward pass's persistent
    // kernels have seen to that, each for its layer; otherwise (protocol switched in between, a second backward pass on
    // one forward pass) one fill.
    if (sentinel && !ctx->dax_filled)
        RUN(PC_MISC, "sentinel fill of da", launch_fill_bytes16(ctx->ws + ctx->wDAX, ctx->dax_bytes * ctx->L, 0xFFFFFFFFu, st));
    ctx->dax_filled = false;
    const char* dY;
    int next_buf = 0;
    if (P > 0) {
        const char* YL = ctx->ws + ctx->wY[ctx->L - 1];
        {   // dW_p = dz^T y
            GemmDesc d = gemm_desc(ctx, S, DT_F32);
            d.M = P; d.N = 2 * H; d.atrans = true; d.btrans = true;
            d.seg[0] = GemmSeg{dz, YL, P, 2 * H, 0, 0, M};
            d.C = grad + ctx->off_wp; d.ldc = 2 * H;
            d.rowsum = grad + ctx->off_bp;             // db_p = sum over frames of dz
            wgrads.push_back(d);
        }
        {   // dy = dz W_p
            GemmDesc d = gemm_desc(ctx, S, S);
            d.M = M; d.N = 2 * H; d.btrans = true;
            d.seg[0] = GemmSeg{dz, at(theta, ctx->off_wp, e), P, 2 * H, 0, 0, P};
            d.C = ctx->ws + ctx->wDY[0]; d.ldc = 2 * H;
            RUN(PC_GEMM_DGRAD, "dy of the bottleneck", launch_gemm(d, st));
        }
        dY = ctx->ws + ctx->wDY[0];
        next_buf = 1;
    } else {
        dY = static_cast<const char*>(dz);
    }
    for (int l = ctx->L - 1; l >= 0; --l) {
        const void* Xin = l == 0 ? x : static_cast<const void*>(ctx->ws + ctx->wY[l - 1]);
        const int Din = ctx->din(l);
        const char* Y = ctx->ws + ctx->wY[l];
        const char* G = ctx->ws + ctx->wG[l];
        const float* C = reinterpret_cast<const float*>(ctx->ws + ctx->wC[l]);
        char* DA = ctx->ws + ctx->wDA[l];
        // The layer's backward recurrence takes the path its forward recurrence took: the two persistent
        // kernels share the order of the saved gates, the per-frame kernels theirs.
        bool rec_done = false;
        if (ctx->fwd_persistent[l]) {
            unsigned* cnt = reinterpret_cast<unsigned*>(ctx->ws + ctx->wCNT);
            const int ncnt = 2 * ctx->rec_nbg * ctx->rec_tiles;
            unsigned short* uht0 = reinterpret_cast<unsigned short*>(ctx->ws + ctx->wUHT) + (size_t)l * 2 * 4 * H * H;
            unsigned short* uht1 = uht0 + (size_t)4 * H * H;
            if (!sentinel) RUN(PC_MISC, "counters", launch_fill_u32(cnt, ncnt, 0u, st));
            RecBwdArgs a{};
            a.uht[0] = uht0; a.uht[1] = uht1;
            a.dy = reinterpret_cast<const unsigned short*>(dY);
            a.gates = reinterpret_cast<const unsigned short*>(G); a.c = C;
            a.da = reinterpret_cast<unsigned short*>(DA); a.dc = DC;
            a.dax = reinterpret_cast<unsigned short*>(ctx->ws + ctx->wDAX + ctx->dax_bytes * l);
            a.cnt = cnt; a.abort_word = cnt + ncnt; a.limit_ticks = 200000000ull;
            a.T = T; a.B = B; a.H = H; a.nbg = ctx->rec_nbg; a.tiles_per_group = ctx->rec_tiles;
            RUN(PC_REC_BWD, "persistent recurrent backward", launch_rec_bwd(a, ctx->rec_sync == 1, st, &rec_done));
            if (!rec_done)
                return fail(BLSTM_ERR_HIP, "blstm_backward: the persistent kernel that must follow its forward twin cannot be launched");
        }
        for (int n = T - 1; n >= 0 && !rec_done; --n) {
            const int t[2] = {n, T - 1 - n};
            const int tp[2] = {n - 1, T - n};
            CellBwdArgs a{};
            a.B = B; a.H = H; a.first = (n == T - 1);
            for (int dd = 0; dd < 2; ++dd) {
                a.dy[dd] = dY + ((size_t)t[dd] * B * 2 * H + (size_t)dd * H) * e;
                a.dh_rec[dd] = (n == T - 1) ? nullptr : DH + (size_t)dd * B * H;
                a.dc_rec[dd] = DC + (size_t)dd * B * H;
                a.gates[dd] = G + ((size_t)t[dd] * B * 8 * H + (size_t)dd * 4 * H) * e;
                a.c[dd] = C + (size_t)t[dd] * B * 2 * H + (size_t)dd * H;
                a.c_prev[dd] = n > 0 ? C + (size_t)tp[dd] * B * 2 * H + (size_t)dd * H : nullptr;
                a.da[dd] = DA + ((size_t)t[dd] * B * 8 * H + (size_t)dd * 4 * H) * e;
            }
            RUN(PC_CELL_BWD, "cell backward", launch_cell_bwd(a, S, st));
            if (n > 0) {   // dh_rec = da U_h
                GemmDesc d = gemm_desc(ctx, S, DT_F32);
                d.batch = 2; d.M = B; d.N = H; d.btrans = true;
                const char* A0 = DA + ((size_t)t[0] * B * 8 * H) * e;
                const char* A1 = DA + ((size_t)t[1] * B * 8 * H + 4 * H) * e;
                d.seg[0] = GemmSeg{A0, at(theta, ctx->off_uh[0][l], e), 8 * H, H, (long long)((A1 - A0) / (long long)e),
                                   (long long)(ctx->off_uh[1][l] - ctx->off_uh[0][l]), 4 * H};
                d.C = DH; d.ldc = H; d.sC = (long long)B * H;
                RUN(PC_GEMM_REC_BWD, "recurrent gradient", launch_gemm(d, st));
            }
        }
        GemmDesc lw[2];
        {   // dW_x = da^T x, both directions
            GemmDesc& d = lw[0];
            d = gemm_desc(ctx, S, DT_F32);
            d.batch = 2; d.M = 4 * H; d.N = Din; d.atrans = true; d.btrans = true;
            d.seg[0] = GemmSeg{DA, Xin, 8 * H, Din, 4 * H, 0, M};
            if (l == 0 && ctx->Dp > 0) {                 // the forward pass's padded x: whole tiles of columns, N of them stored
                d.seg[0] = GemmSeg{DA, ctx->ws + ctx->wXP, 8 * H, ctx->Dp, 4 * H, 0, M};
                d.Npad = ctx->Dp;
            }
            d.C = grad + ctx->off_wx[0][l]; d.ldc = Din; d.sC = (long long)(ctx->off_wx[1][l] - ctx->off_wx[0][l]);
            d.rowsum = grad + ctx->off_b[0][l];        // db = sum over frames of da
            d.sRowsum = (long long)(ctx->off_b[1][l] - ctx->off_b[0][l]);
        }
        {   // dU_h = da^T h_prev: forward direction pairs da[t] with h[t-1], backward direction with h[t+1] (T = 1: an empty sum)
            GemmDesc& d = lw[1];
            d = gemm_desc(ctx, S, DT_F32);
            d.batch = 2; d.M = 4 * H; d.N = H; d.atrans = true; d.btrans = true;
            const char* A0 = DA + ((size_t)B * 8 * H) * e;
            const char* A1 = DA + ((size_t)4 * H) * e;
            const char* B0 = Y;
            const char* B1 = Y + ((size_t)B * 2 * H + H) * e;
            d.seg[0] = GemmSeg{A0, B0, 8 * H, 2 * H, (long long)((A1 - A0) / (long long)e), (long long)((B1 - B0) / (long long)e), (T - 1) * B};
            d.C = grad + ctx->off_uh[0][l]; d.ldc = H; d.sC = (long long)(ctx->off_uh[1][l] - ctx->off_uh[0][l]);
        }
        wgrads.push_back(lw[0]); wgrads.push_back(lw[1]);
        if (l > 0) {   // dx = da_fwd W_x_fwd + da_bwd W_x_bwd, the gradient of the layer below's output
            GemmDesc d = gemm_desc(ctx, S, S);
            d.M = M; d.N = Din; d.btrans = true; d.nseg = 2;
            d.seg[0] = GemmSeg{DA, at(theta, ctx->off_wx[0][l], e), 8 * H, Din, 0, 0, 4 * H};
            d.seg[1] = GemmSeg{DA + (size_t)4 * H * e, at(theta, ctx->off_wx[1][l], e), 8 * H, Din, 0, 0, 4 * H};
            d.C = ctx->ws + ctx->wDY[next_buf]; d.ldc = Din;
            RUN(PC_GEMM_DGRAD, "dx", launch_gemm(d, st));
            dY = ctx->ws + ctx->wDY[next_buf];
            next_buf ^= 1;
        }
    }
    if (ctx->pend_z) {
        // the softmax layer's weight gradient, left to this call: dE/du still lies in the workspace.  It joins the
        // grouped launch when it can run there (else the whole group would run product by product).
        const GemmDesc d = softmax_wgrad_desc(ctx, ctx->ws + ctx->wLOGITS, ctx->pend_z, grad);
        ctx->pend_z = nullptr;
        if (gemm_group_ok(&d, 1)) wgrads.push_back(d);
        else RUN(PC_GEMM_SOFTMAX_BWD, "dW_s", launch_gemm(d, st));
    }
    RUN(PC_GEMM_WGRAD, "weight gradients", launch_gemm_group(wgrads.data(), (int)wgrads.size(), st));
    return BLSTM_OK;
}

int sgd_step(float* theta, void* shadow, const float* grad, size_t n, float lr, float momentum, float* velocity, void* stream) {
    if (!theta || !grad) return fail(BLSTM_ERR_NULL, "sgd_step: null argument");
    if (momentum != 0.0f && !velocity) return fail(BLSTM_ERR_NULL, "sgd_step: momentum needs a velocity buffer");
    if (!aligned16(theta) || !aligned16(grad) || (shadow && !aligned16(shadow)) || (momentum != 0.0f && !aligned16(velocity)))
        return fail(BLSTM_ERR_ALIGN, "sgd_step: pointers must be 16-byte aligned");
    return check_hip(launch_sgd(theta, static_cast<unsigned short*>(shadow), grad, n, lr, momentum, velocity,
                                static_cast<hipStream_t>(stream)), "sgd_step");
}

int adpsgd_mix(float* const* theta, void* const* shadow, size_t n, int R, const int32_t* partner, void* stream) {
    if (!theta || !partner) return fail(BLSTM_ERR_NULL, "adpsgd_mix: null argument");
    if (R < 1 || R > BLSTM_MAX_REPLICAS) return fail(BLSTM_ERR_DIM, "adpsgd_mix: R must be in 1..%d", BLSTM_MAX_REPLICAS);
    for (int i = 0; i < R; ++i) {
        const int j = partner[i];
        if (j < 0 || j >= R || partner[j] != i) return fail(BLSTM_ERR_DIM, "adpsgd_mix: partner is not an involution at %d", i);
        if (!theta[i] || (shadow && !shadow[i])) return fail(BLSTM_ERR_NULL, "adpsgd_mix: null replica pointer %d", i);
        if (!aligned16(theta[i]) || (shadow && !aligned16(shadow[i]))) return fail(BLSTM_ERR_ALIGN, "adpsgd_mix: replica %d is not 16-byte aligned", i);
        for (int k = 0; k < i; ++k)
            if (theta[k] == theta[i]) return fail(BLSTM_ERR_DIM, "adpsgd_mix: replicas %d and %d share a buffer", k, i);
    }
    MixPairs p{};
    for (int i = 0; i < R; ++i) {
        const int j = partner[i];
        if (j <= i) continue;
        p.a[p.npairs] = theta[i]; p.b[p.npairs] = theta[j];
        p.sa[p.npairs] = shadow ? static_cast<unsigned short*>(shadow[i]) : nullptr;
        p.sb[p.npairs] = shadow ? static_cast<unsigned short*>(shadow[j]) : nullptr;
        ++p.npairs;
    }
    return check_hip(launch_mix(p, n, static_cast<hipStream_t>(stream)), "adpsgd_mix");
}

int sgd_mix_pair(float* theta_i, float* theta_j, void* shadow_i, void* shadow_j, const float* grad_i, const float* grad_j,
                 size_t n, float lr, float momentum, float* velocity_i, float* velocity_j, void* stream) {
    // grad_j == NULL: replica j is averaged as it stands (no update, no velocity of its own here)
    if (!theta_i || !theta_j || !grad_i) return fail(BLSTM_ERR_NULL, "sgd_mix_pair: null argument");
    if ((shadow_i == nullptr) != (shadow_j == nullptr)) return fail(BLSTM_ERR_NULL, "sgd_mix_pair: give both bf16 copies or neither");
    if (momentum != 0.0f && (!velocity_i || (grad_j && !velocity_j))) return fail(BLSTM_ERR_NULL, "sgd_mix_pair: momentum needs a velocity buffer for every replica that has a gradient");
    if (theta_i == theta_j) return fail(BLSTM_ERR_DIM, "sgd_mix_pair: the two replicas share a buffer");
    if (!aligned16(theta_i) || !aligned16(theta_j) || !aligned16(grad_i) || (grad_j && !aligned16(grad_j)) ||
        (shadow_i && (!aligned16(shadow_i) || !aligned16(shadow_j))) ||
        (momentum != 0.0f && (!aligned16(velocity_i) || (grad_j && !aligned16(velocity_j)))))
        return fail(BLSTM_ERR_ALIGN, "sgd_mix_pair: pointers must be 16-byte aligned");
    return check_hip(launch_sgd_mix_pair(theta_i, theta_j, grad_i, grad_j, velocity_i, velocity_j,
                                         static_cast<unsigned short*>(shadow_i), static_cast<unsigned short*>(shadow_j),
                                         n, lr, momentum, static_cast<hipStream_t>(stream)), "sgd_mix_pair");
}

int sync_average(float* const* theta, void* const* shadow, size_t n, int R, void* stream) {
    if (!theta) return fail(BLSTM_ERR_NULL, "sync_average: null argument");
    if (R < 1 || R > BLSTM_MAX_REPLICAS) return fail(BLSTM_ERR_DIM, "sync_average: R must be in 1..%d", BLSTM_MAX_REPLICAS);
    static_assert(BLSTM_MAX_REPLICAS == BLSTM_MAX_REPLICA_PTRS, "the kernel's pointer table must hold every replica");
    ReplicaSet p{};
    p.R = R;
    for (int i = 0; i < R; ++i) {
        if (!theta[i] || (shadow && !shadow[i])) return fail(BLSTM_ERR_NULL, "sync_average: null replica pointer %d", i);
        if (!aligned16(theta[i]) || (shadow && !aligned16(shadow[i]))) return fail(BLSTM_ERR_ALIGN, "sync_average: replica %d is not 16-byte aligned", i);
        for (int k = 0; k < i; ++k)
            if (theta[k] == theta[i]) return fail(BLSTM_ERR_DIM, "sync_average: replicas %d and %d share a buffer", k, i);
        p.t[i] = theta[i];
        p.s[i] = shadow ? static_cast<unsigned short*>(shadow[i]) : nullptr;
    }
    return check_hip(launch_sync_average(p, n, static_cast<hipStream_t>(stream)), "sync_average");
}

double blstm_lr_schedule(int epoch, double base_lr, double peak_lr, int warmup_epochs, int anneal_from) {
    if (epoch <= warmup_epochs) {
        if (warmup_epochs <= 1) return peak_lr;
        return base_lr + (peak_lr - base_lr) * (double)(epoch - 1) / (double)(warmup_epochs - 1);
    }
    int k = epoch - anneal_from + 1;
    if (k < 0) k = 0;
    double lr = peak_lr;
    for (int i = 0; i < k; ++i) lr *= 0.70710678118654752440;
    return lr;
}

int adpsgd_ring_partner(int R, int64_t step, int32_t* partner_out) {
    if (!partner_out) return fail(BLSTM_ERR_NULL, "adpsgd_ring_partner: null argument");
    if (R < 2 || (R & 1) || step < 0) return fail(BLSTM_ERR_DIM, "adpsgd_ring_partner: R must be even and >= 2, step >= 0");
    const bool right = (step % 2) == 0;
    for (int i = 0; i < R; i += 2) {
        const int j = right ? (i + 1) % R : (i + R - 1) % R;
        partner_out[i] = j;
        partner_out[j] = i;
    }
    return BLSTM_OK;
}

int blstm_shadow_refresh(const float* theta, void* shadow, size_t n, void* stream) {
    if (!theta || !shadow) return fail(BLSTM_ERR_NULL, "blstm_shadow_refresh: null argument");
    if (!aligned16(theta) || !aligned16(shadow)) return fail(BLSTM_ERR_ALIGN, "blstm_shadow_refresh: pointers must be 16-byte aligned");
    return check_hip(launch_shadow(theta, static_cast<unsigned short*>(shadow), n, static_cast<hipStream_t>(stream)), "blstm_shadow_refresh");
}

int blstm_set_option(blstm_ctx* c, int option, int value) {
    if (!c) return fail(BLSTM_ERR_NULL, "blstm_set_option: null argument");
    if (option == BLSTM_OPT_RECURRENT_PATH && (value == 0 || value == 1)) { c->rec_path = value; return BLSTM_OK; }
    if (option == BLSTM_OPT_RECURRENT_SYNC && (value == 0 || value == 1)) { c->rec_sync = value; return BLSTM_OK; }
    if (option == BLSTM_OPT_KEEP_WEIGHT_COPIES && (value == 0 || value == 1)) {
        c->keep_copies = value != 0; c->wxp_of = nullptr; c->uht_of = nullptr;
        return BLSTM_OK;
    }
    if (option == BLSTM_OPT_TEST_ABORT && (value == 0 || value == 1)) { c->test_abort = value != 0; return BLSTM_OK; }
    if (option == BLSTM_OPT_DEFER_SOFTMAX_WGRAD && (value == 0 || value == 1)) {
        c->defer_ws = value != 0;
        if (!c->defer_ws) c->pend_z = nullptr;
        return BLSTM_OK;
    }
    return fail(BLSTM_ERR_DIM, "blstm_set_option: unknown option %d or value %d", option, value);
}

int blstm_weights_changed(blstm_ctx* c) {
    if (!c) return fail(BLSTM_ERR_NULL, "blstm_weights_changed: null argument");
    c->wxp_of = nullptr; c->uht_of = nullptr;
    return BLSTM_OK;
}

int blstm_device_status(blstm_ctx* c, void* stream) {
    if (!c) return fail(BLSTM_ERR_NULL, "blstm_device_status: null argument");
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipError_t e = hipStreamSynchronize(st);
    if (e != hipSuccess) return check_hip(e, "blstm_device_status");
    if (!c->ws || c->rec_nbg == 0 || !c->abort_clean) return BLSTM_OK;
    unsigned* word = reinterpret_cast<unsigned*>(c->ws + c->wCNT) + 2 * c->rec_nbg * c->rec_tiles;
    unsigned v = 0;
    e = hipMemcpy(&v, word, sizeof v, hipMemcpyDeviceToHost);
    if (e != hipSuccess) return check_hip(e, "blstm_device_status");
    if (v != 0) {
        c->abort_clean = false;          // the next forward pass zeroes the word again
        return fail(BLSTM_ERR_HIP, "a persistent recurrent kernel abandoned a wait: its workgroups were not co-resident");
    }
    return BLSTM_OK;
}

int blstm_profile_classes(void) { return PC_COUNT; }
const char* blstm_profile_name(int k) { return (k >= 0 && k < PC_COUNT) ? kProfNames[k] : ""; }

int blstm_profile_enable(blstm_ctx* c, int enable) {
    if (!c) return fail(BLSTM_ERR_NULL, "blstm_profile_enable: null argument");
    c->prof = enable != 0;
    c->recs_used = 0;
    memset(c->prof_ms, 0, sizeof c->prof_ms);
    memset(c->prof_n, 0, sizeof c->prof_n);
    return BLSTM_OK;
}

int blstm_profile_read(blstm_ctx* c, double* ms_out, int64_t* launches_out, int n_classes) {
    if (!c || !ms_out || !launches_out) return fail(BLSTM_ERR_NULL, "blstm_profile_read: null argument");
    for (size_t i = 0; i < c->recs_used; ++i) {
        ProfRec& r = c->recs[i];
        hipError_t e = hipEventSynchronize(r.b);
        if (e != hipSuccess) return check_hip(e, "blstm_profile_read");
        float ms = 0.0f;
        e = hipEventElapsedTime(&ms, r.a, r.b);
        if (e != hipSuccess) return check_hip(e, "blstm_profile_read");
        c->prof_ms[r.cls] += ms;
        c->prof_n[r.cls] += 1;
    }
    c->recs_used = 0;
    for (int k = 0; k < n_classes && k < PC_COUNT; ++k) { ms_out[k] = c->prof_ms[k]; launches_out[k] = c->prof_n[k]; }
    return BLSTM_OK;
}

}  // extern "C"
