// Host side of the C ABI declared in include/tesseract.h: argument validation,
// mapping of the three Tesseract products onto one batched-panel GEMM launch,
// kernel/tile/split selection.  No HIP call happens before validation has passed.
#include "tess_internal.h"
#include "tesseract_diag.h"

#include <atomic>
#include <mutex>

namespace tess {

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Tuning overrides of the diagnostic interface (0 = the cost model decides).
static std::atomic<int> g_force_tile{0}, g_force_splits{0};

// Shape-only part of the plan (what tess_linear_workspace_bytes can know).  a_kc / b_kc:
// operand orientation of the call (see GemmArgs).
static Plan shape_plan(int64_t M, int64_t N, int64_t Kp, int q, bool in_bf16, bool a_kc, bool b_kc)
{
    Plan p{};
    p.path = Path::Generic;
    p.bm = p.bn = 0;
    p.splits = 1;
    p.direct = 0;
    p.ws_bytes = 0;
    if (!in_bf16) return p;
    // the matrix-core path moves 16-byte granules (8 bf16) along the contiguous index of
    // each operand: extents that are no multiple of 8 take the plain kernel
    if (a_kc ? (Kp % 8 != 0) : (M % 8 != 0)) return p;
    if (b_kc ? (Kp % 8 != 0) : (N % 8 != 0)) return p;
    p.path = Path::Mfma;
    const int64_t kt_total = (int64_t)q * ((Kp + BK_HOST - 1) / BK_HOST);
    p.direct = (Kp % BK_HOST == 0) ? 1 : 0;
    // Tile and K-split are chosen with a small cost model in microseconds, fitted to
    // timings of this kernel on MI355X.  A launch runs in rounds of 256 workgroups (one
    // per compute unit).  A workgroup costs a fixed start/finish time plus its 64-deep
    // stages; a stage is slower the fuller the round is (shared clock and fabric).  A
    // split adds a reduction launch that streams every fp32 partial tile once more.
    struct TileCost { int t; double fixed_us, stage_idle_us, stage_full_us; };
    const TileCost cands[2] = {{256, 10.0, 1.0, 1.6}, {128, 5.0, 0.36, 0.60}};
    const double kLaunchUs = 4.0, kReduceLaunchUs = 2.0, kReduceBytesPerUs = 4.0e6;
    const int kCU = 256;
    double best = 1e30;
    for (int ci = 0; ci < 2; ++ci) {
        const TileCost& tc = cands[ci];
        const int t = tc.t;
        // the register-staged loader (ragged K) only exists for the small tile
        if (t == 256 && !(p.direct && M >= 256 && N >= 256)) continue;
        const int64_t tiles = ((M + t - 1) / t) * ((N + t - 1) / t);
        for (int sp = 1; sp <= 16; ++sp) {
            if (sp > 1 && kt_total / sp < 8) break;       // keep at least 8 stages per split
            const int64_t wgs = tiles * sp;
            const double kt = (double)((kt_total + sp - 1) / sp);
            const int64_t full_rounds = wgs / kCU, rem = wgs % kCU;
            double cost = kLaunchUs + (double)full_rounds * (tc.fixed_us + kt * tc.stage_full_us);
            if (rem) {
                const double fill = (double)rem / kCU;
                cost += tc.fixed_us + kt * (tc.stage_idle_us + fill * (tc.stage_full_us - tc.stage_idle_us));
            }
            if (sp > 1)
                cost += kReduceLaunchUs + (double)wgs * t * t * sizeof(float) / kReduceBytesPerUs;
            if (cost < best) { best = cost; p.bm = p.bn = t; p.splits = sp; }
        }
    }
    // tuning overrides of the diagnostic interface; the workspace query, the plan query and
    // the launch all pass through here, so they agree
    if (const int v = g_force_tile.load(std::memory_order_relaxed)) { if (v == 128 || (v == 256 && p.direct && M >= 256 && N >= 256)) p.bm = p.bn = v; }
    if (const int v = g_force_splits.load(std::memory_order_relaxed)) { if (v >= 1 && kt_total / v >= 1) { p.splits = v; } }
    const int64_t tiles = ((M + p.bm - 1) / p.bm) * ((N + p.bn - 1) / p.bn);
    if (p.splits > 1)
        p.ws_bytes = (size_t)p.splits * tiles * p.bm * p.bn * sizeof(float) +
                     (((size_t)p.splits * N * sizeof(float) + 255) & ~(size_t)255);   // + column sums
    return p;
}

// Plan of a launch with its operands: the shape plan, refused when the matrix-core path
// that the shape selects cannot take these pointers or leading dimensions (a silent drop
// to the plain kernel would be orders of magnitude slower than what tess_linear_plan says).
static tess_status make_plan(const GemmArgs& g, Plan& p)
{
    p = shape_plan(g.M, g.N, g.Kp, g.q, !g.in_f32, g.a_kc != 0, g.b_kc != 0);
    if (p.path != Path::Mfma) return TESS_OK;
    if (g.lda % 8 != 0 || g.ldb % 8 != 0) return TESS_ERR_ALIGN;
    for (int t = 0; t < g.q; ++t)
        if (!aligned16(g.a[t]) || !aligned16(g.b[t])) return TESS_ERR_ALIGN;
    // 32-bit byte offsets inside a panel (the loaders add up to 4 KiB to every offset)
    const int64_t a_rows = g.a_kc ? g.M : g.Kp, b_rows = g.b_kc ? g.N : g.Kp;
    const int64_t lim = ((int64_t)1 << 32) - 4096;
    if (a_rows * g.lda * 2 >= lim || b_rows * g.ldb * 2 >= lim) return TESS_ERR_UNSUPPORTED;
    return TESS_OK;
}

static tess_status check_desc(const tess_desc* d)
{
    if (!d) return TESS_ERR_NULL;
    if (d->q < 1 || d->d < 1 || d->d > d->q || d->q > TESS_MAX_Q) return TESS_ERR_GRID;
    if (d->i < 0 || d->i >= d->q || d->j < 0 || d->j >= d->q || d->k < 0 || d->k >= d->d)
        return TESS_ERR_GRID;
    if (d->a < 1 || d->b < 1 || d->c < 1) return TESS_ERR_SHAPE;
    if (d->a % ((int64_t)d->q * d->d) != 0 || d->b % d->q != 0 || d->c % d->q != 0)
        return TESS_ERR_SHAPE;
    if (d->in_dtype != TESS_F32 && d->in_dtype != TESS_BF16) return TESS_ERR_UNSUPPORTED;
    if (d->out_dtype != TESS_F32 && d->out_dtype != TESS_BF16) return TESS_ERR_UNSUPPORTED;
    const int64_t lim = (int64_t)1 << 30;
    if (d->a / ((int64_t)d->q * d->d) >= lim || d->b / d->q >= lim || d->c / d->q >= lim)
        return TESS_ERR_UNSUPPORTED;
    return TESS_OK;
}

static tess_status check_panels(const void* const* p, int q)
{
    if (!p) return TESS_ERR_NULL;
    for (int t = 0; t < q; ++t)
        if (!p[t]) return TESS_ERR_NULL;
    return TESS_OK;
}

static tess_status run(GemmArgs& g, void* workspace, size_t workspace_bytes, void* stream)
{
    Plan p;
    const tess_status ps = make_plan(g, p);
    if (ps != TESS_OK) return ps;
    if (p.ws_bytes > 0) {
        if (!workspace || workspace_bytes < p.ws_bytes) return TESS_ERR_WORKSPACE;
        if (reinterpret_cast<uintptr_t>(workspace) & 255u) return TESS_ERR_WORKSPACE;
        g.ws = static_cast<float*>(workspace);
    }
#ifdef TESS_STAMPS
    // diagnostic build: the time stamps follow the workspace proper (the caller leaves 1 MiB of room)
    g.stamps = reinterpret_cast<unsigned long long*>(static_cast<char*>(workspace) + ((p.ws_bytes + 255) & ~(size_t)255));
#endif
    g.splits = p.splits;
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipError_t e = (p.path == Path::Mfma) ? launch_mfma(g, p, s) : launch_generic(g, s);
    return e == hipSuccess ? TESS_OK : TESS_ERR_HIP;
}

}  // namespace tess

// Scratch of tess_linear_bwd_dw_noalloc: part of the code object, one copy per device, held
// until the process ends.  In host code the array's name is only a handle: the device
// address comes from hipGetSymbolAddress, once per device with that device current.
#define TESS_NOALLOC_SCRATCH_BYTES (80u << 20)
#ifdef __HIPCC__
static __device__ __align__(256) unsigned char scratch[TESS_NOALLOC_SCRATCH_BYTES];
#else
// host-only build of this file for the sanitizer tests (plain C++, no device code, kernel
// launchers stubbed): a host array stands in, nothing ever dereferences it
alignas(256) static unsigned char scratch[TESS_NOALLOC_SCRATCH_BYTES];
#endif

namespace tess {

static hipError_t scratch_of_current_device(void** out)
{
    constexpr int kMaxDev = 64;
    static void* ptrs[kMaxDev] = {};
    static std::mutex mu;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDev) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(mu);
    if (!ptrs[dev]) {
        void* p = nullptr;
#ifdef __HIPCC__
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
#else
        p = scratch;
#endif
        if (!p) return hipErrorInvalidSymbol;
        ptrs[dev] = p;
    }
    *out = ptrs[dev];
    return hipSuccess;
}

}  // namespace tess

using namespace tess;

extern "C" {

tess_status tess_desc_check(const tess_desc* desc) { return check_desc(desc); }

tess_status tess_block_shape(const tess_desc* desc, int64_t* m, int64_t* kb, int64_t* n)
{
    tess_status st = check_desc(desc);
    if (st != TESS_OK) return st;
    if (!m || !kb || !n) return TESS_ERR_NULL;
    *m = desc->a / ((int64_t)desc->q * desc->d);
    *kb = desc->b / desc->q;
    *n = desc->c / desc->q;
    return TESS_OK;
}

size_t tess_linear_workspace_bytes(const tess_desc* desc, int op)
{
    if (check_desc(desc) != TESS_OK) return 0;
    const int64_t m = desc->a / ((int64_t)desc->q * desc->d), kb = desc->b / desc->q,
                  n = desc->c / desc->q;
    const bool bf = desc->in_dtype == TESS_BF16;
    switch (op) {
        case TESS_OP_FWD: return shape_plan(m, n, kb, desc->q, bf, true, false).ws_bytes;
        case TESS_OP_BWD_DX: return shape_plan(m, kb, n, desc->q, bf, true, true).ws_bytes;
        case TESS_OP_BWD_DW: return shape_plan(kb, n, m, desc->q, bf, false, false).ws_bytes;
        case TESS_OP_BWD_DX_STEP: return shape_plan(m, kb, n, 1, bf, true, true).ws_bytes;
        case TESS_OP_BWD_DW_STEP: return shape_plan(kb, n, m, 1, bf, false, false).ws_bytes;
        default: return 0;
    }
}

tess_status tess_linear_plan(const tess_desc* desc, int op, int32_t* tile_m, int32_t* tile_n,
                             int32_t* k_splits)
{
    tess_status st = check_desc(desc);
    if (st != TESS_OK) return st;
    if (!tile_m || !tile_n || !k_splits) return TESS_ERR_NULL;
    const int64_t m = desc->a / ((int64_t)desc->q * desc->d), kb = desc->b / desc->q,
                  n = desc->c / desc->q;
    const bool bf = desc->in_dtype == TESS_BF16;
    Plan p;
    switch (op) {
        case TESS_OP_FWD: p = shape_plan(m, n, kb, desc->q, bf, true, false); break;
        case TESS_OP_BWD_DX: p = shape_plan(m, kb, n, desc->q, bf, true, true); break;
        case TESS_OP_BWD_DW: p = shape_plan(kb, n, m, desc->q, bf, false, false); break;
        case TESS_OP_BWD_DX_STEP: p = shape_plan(m, kb, n, 1, bf, true, true); break;
        case TESS_OP_BWD_DW_STEP: p = shape_plan(kb, n, m, 1, bf, false, false); break;
        default: return TESS_ERR_UNSUPPORTED;
    }
    *tile_m = p.bm; *tile_n = p.bn; *k_splits = p.splits;
    return TESS_OK;
}

tess_status tess_linear_fwd(const tess_desc* desc, const void* const* a_panels, int64_t lda,
                            const void* const* b_panels, int64_t ldb, const void* bias, int act,
                            void* c_out, int64_t ldc, void* preact_out, void* workspace,
                            size_t workspace_bytes, void* hip_stream)
{
    tess_status st = check_desc(desc);
    if (st != TESS_OK) return st;
    if ((st = check_panels(a_panels, desc->q)) != TESS_OK) return st;
    if ((st = check_panels(b_panels, desc->q)) != TESS_OK) return st;
    if (!c_out) return TESS_ERR_NULL;
    if (act != TESS_ACT_NONE && act != TESS_ACT_GELU_ERF && act != TESS_ACT_GELU_TANH)
        return TESS_ERR_UNSUPPORTED;
    const int64_t m = desc->a / ((int64_t)desc->q * desc->d), kb = desc->b / desc->q,
                  n = desc->c / desc->q;
    if (lda < kb || ldb < n || ldc < n) return TESS_ERR_SHAPE;
    GemmArgs g{};
    for (int t = 0; t < desc->q; ++t) { g.a[t] = a_panels[t]; g.b[t] = b_panels[t]; }
    g.q = desc->q; g.M = (int32_t)m; g.N = (int32_t)n; g.Kp = (int32_t)kb;
    g.lda = lda; g.ldb = ldb; g.out = c_out; g.ldo = ldc; g.preact = preact_out; g.bias = bias;
    g.act = act; g.out_f32 = desc->out_dtype == TESS_F32; g.accumulate = 0;
    g.a_kc = 1; g.b_kc = 0; g.in_f32 = desc->in_dtype == TESS_F32;
    return run(g, workspace, workspace_bytes, hip_stream);
}

static tess_status bwd_dx_impl(const tess_desc* desc, const void* const* dy_panels, int64_t lddy,
                               const void* const* w_panels, int64_t ldw, const void* preact,
                               int64_t ldz, int act, bool with_act, void* dx_out, int64_t lddx,
                               void* workspace, size_t workspace_bytes, void* hip_stream)
{
    tess_status st = check_desc(desc);
    if (st != TESS_OK) return st;
    if ((st = check_panels(dy_panels, desc->q)) != TESS_OK) return st;
    if ((st = check_panels(w_panels, desc->q)) != TESS_OK) return st;
    if (!dx_out) return TESS_ERR_NULL;
    const int64_t m = desc->a / ((int64_t)desc->q * desc->d), kb = desc->b / desc->q,
                  n = desc->c / desc->q;
    if (lddy < n || ldw < n || lddx < kb) return TESS_ERR_SHAPE;
    if (with_act) {
        if (act != TESS_ACT_NONE && act != TESS_ACT_GELU_ERF && act != TESS_ACT_GELU_TANH)
            return TESS_ERR_UNSUPPORTED;
        if (act != TESS_ACT_NONE) {
            if (!preact) return TESS_ERR_NULL;
            if (ldz < kb) return TESS_ERR_SHAPE;
        }
    }
    GemmArgs g{};
    if (with_act && act != TESS_ACT_NONE) { g.zin = preact; g.ldz = ldz; g.dact = act; }
    for (int t = 0; t < desc->q; ++t) { g.a[t] = dy_panels[t]; g.b[t] = w_panels[t]; }
    g.q = desc->q; g.M = (int32_t)m; g.N = (int32_t)kb; g.Kp = (int32_t)n;
    g.lda = lddy; g.ldb = ldw; g.out = dx_out; g.ldo = lddx; g.preact = nullptr; g.bias = nullptr;
    g.act = TESS_ACT_NONE; g.out_f32 = desc->out_dtype == TESS_F32; g.accumulate = 0;
    g.a_kc = 1; g.b_kc = 1; g.in_f32 = desc->in_dtype == TESS_F32;
    return run(g, workspace, workspace_bytes, hip_stream);
}

tess_status tess_linear_bwd_dx(const tess_desc* desc, const void* const* dy_panels, int64_t lddy,
                               const void* const* w_panels, int64_t ldw, void* dx_out,
                               int64_t lddx, void* workspace, size_t workspace_bytes,
                               void* hip_stream)
{
    return bwd_dx_impl(desc, dy_panels, lddy, w_panels, ldw, nullptr, 0, TESS_ACT_NONE, false,
                       dx_out, lddx, workspace, workspace_bytes, hip_stream);
}

tess_status tess_linear_bwd_dx_act(const tess_desc* desc, const void* const* dy_panels,
                                   int64_t lddy, const void* const* w_panels, int64_t ldw,
                                   const void* preact, int64_t ldz, int act, void* dz_out,
                                   int64_t lddz, void* workspace, size_t workspace_bytes,
                                   void* hip_stream)
{
    return bwd_dx_impl(desc, dy_panels, lddy, w_panels, ldw, preact, ldz, act, true, dz_out, lddz,
                       workspace, workspace_bytes, hip_stream);
}

static tess_status bwd_dw_impl(const tess_desc* desc, const void* const* x_panels, int64_t ldx,
                               const void* const* dy_panels, int64_t lddy, void* dw_out,
                               int64_t lddw, void* dbias_out, bool with_bias, int accumulate,
                               void* workspace, size_t workspace_bytes, void* hip_stream,
                               bool static_scratch = false)
{
    tess_status st = check_desc(desc);
    if (st != TESS_OK) return st;
    if ((st = check_panels(x_panels, desc->q)) != TESS_OK) return st;
    if ((st = check_panels(dy_panels, desc->q)) != TESS_OK) return st;
    if (!dw_out || (with_bias && !dbias_out)) return TESS_ERR_NULL;
    if (accumulate != 0 && accumulate != 1) return TESS_ERR_UNSUPPORTED;
    const int64_t m = desc->a / ((int64_t)desc->q * desc->d), kb = desc->b / desc->q,
                  n = desc->c / desc->q;
    if (ldx < kb || lddy < n || lddw < n) return TESS_ERR_SHAPE;
    GemmArgs g{};
    for (int t = 0; t < desc->q; ++t) { g.a[t] = x_panels[t]; g.b[t] = dy_panels[t]; }
    g.q = desc->q; g.M = (int32_t)kb; g.N = (int32_t)n; g.Kp = (int32_t)m;
    g.lda = ldx; g.ldb = lddy; g.out = dw_out; g.ldo = lddw; g.preact = nullptr; g.bias = nullptr;
    g.act = TESS_ACT_NONE; g.out_f32 = accumulate ? 1 : (desc->out_dtype == TESS_F32);
    g.accumulate = accumulate;
    g.a_kc = 0; g.b_kc = 0; g.in_f32 = desc->in_dtype == TESS_F32;
    g.colsum = with_bias ? static_cast<float*>(dbias_out) : nullptr;
    if (static_scratch) {
        // the size check needs no device: it comes before the first HIP call
        Plan p;
        const tess_status ps = make_plan(g, p);
        if (ps != TESS_OK) return ps;
        if (p.ws_bytes > TESS_NOALLOC_SCRATCH_BYTES) return TESS_ERR_WORKSPACE;
        if (p.ws_bytes > 0) {
            if (scratch_of_current_device(&workspace) != hipSuccess) return TESS_ERR_HIP;
            workspace_bytes = TESS_NOALLOC_SCRATCH_BYTES;
        }
    }
    return run(g, workspace, workspace_bytes, hip_stream);
}

tess_status tess_linear_bwd_dw(const tess_desc* desc, const void* const* x_panels, int64_t ldx,
                               const void* const* dy_panels, int64_t lddy, void* dw_out,
                               int64_t lddw, int accumulate, void* workspace,
                               size_t workspace_bytes, void* hip_stream)
{
    return bwd_dw_impl(desc, x_panels, ldx, dy_panels, lddy, dw_out, lddw, nullptr, false,
                       accumulate, workspace, workspace_bytes, hip_stream);
}

tess_status tess_linear_bwd_dw_noalloc(const tess_desc* desc, const void* const* x_panels, int64_t ldx,
                                       const void* const* dy_panels, int64_t lddy, void* dw_out,
                                       int64_t lddw, int accumulate, void* hip_stream)
{
    return bwd_dw_impl(desc, x_panels, ldx, dy_panels, lddy, dw_out, lddw, nullptr, false,
                       accumulate, nullptr, 0, hip_stream, true);
}

size_t tess_noalloc_scratch_bytes(void) { return TESS_NOALLOC_SCRATCH_BYTES; }

tess_status tess_linear_bwd_dw_bias(const tess_desc* desc, const void* const* x_panels,
                                    int64_t ldx, const void* const* dy_panels, int64_t lddy,
                                    void* dw_out, int64_t lddw, void* dbias_out, int accumulate,
                                    void* workspace, size_t workspace_bytes, void* hip_stream)
{
    return bwd_dw_impl(desc, x_panels, ldx, dy_panels, lddy, dw_out, lddw, dbias_out, true,
                       accumulate, workspace, workspace_bytes, hip_stream);
}

tess_status tess_linear_bwd_dx_step(const tess_desc* desc, const void* dy_block, int64_t lddy,
                                    const void* w_block, int64_t ldw, void* partial_out,
                                    int64_t ldp, int accumulate, void* workspace,
                                    size_t workspace_bytes, void* hip_stream)
{
    tess_status st = check_desc(desc);
    if (st != TESS_OK) return st;
    if (!dy_block || !w_block || !partial_out) return TESS_ERR_NULL;
    if (accumulate != 0 && accumulate != 1) return TESS_ERR_UNSUPPORTED;
    const int64_t m = desc->a / ((int64_t)desc->q * desc->d), kb = desc->b / desc->q,
                  n = desc->c / desc->q;
    if (lddy < n || ldw < n || ldp < kb) return TESS_ERR_SHAPE;
    GemmArgs g{};
    g.a[0] = dy_block; g.b[0] = w_block;
    g.q = 1; g.M = (int32_t)m; g.N = (int32_t)kb; g.Kp = (int32_t)n;
    g.lda = lddy; g.ldb = ldw; g.out = partial_out; g.ldo = ldp;
    g.act = TESS_ACT_NONE; g.out_f32 = 1; g.accumulate = accumulate;
    g.a_kc = 1; g.b_kc = 1; g.in_f32 = desc->in_dtype == TESS_F32;
    return run(g, workspace, workspace_bytes, hip_stream);
}

tess_status tess_linear_bwd_dw_step(const tess_desc* desc, const void* x_block, int64_t ldx,
                                    const void* dy_block, int64_t lddy, void* partial_out,
                                    int64_t ldp, int accumulate, void* workspace,
                                    size_t workspace_bytes, void* hip_stream)
{
    tess_status st = check_desc(desc);
    if (st != TESS_OK) return st;
    if (!x_block || !dy_block || !partial_out) return TESS_ERR_NULL;
    if (accumulate != 0 && accumulate != 1) return TESS_ERR_UNSUPPORTED;
    const int64_t m = desc->a / ((int64_t)desc->q * desc->d), kb = desc->b / desc->q,
                  n = desc->c / desc->q;
    if (ldx < kb || lddy < n || ldp < n) return TESS_ERR_SHAPE;
    GemmArgs g{};
    g.a[0] = x_block; g.b[0] = dy_block;
    g.q = 1; g.M = (int32_t)kb; g.N = (int32_t)n; g.Kp = (int32_t)m;
    g.lda = ldx; g.ldb = lddy; g.out = partial_out; g.ldo = ldp;
    g.act = TESS_ACT_NONE; g.out_f32 = 1; g.accumulate = accumulate;
    g.a_kc = 0; g.b_kc = 0; g.in_f32 = desc->in_dtype == TESS_F32;
    return run(g, workspace, workspace_bytes, hip_stream);
}

tess_status tess_layernorm_row_sums(const void* x, int64_t m, int64_t w, int64_t ldx, int dtype,
                                    void* sums_out, int accumulate, void* hip_stream)
{
    if (!x || !sums_out) return TESS_ERR_NULL;
    if (m < 1 || w < 1 || ldx < w || m > ((int64_t)1 << 32)) return TESS_ERR_SHAPE;
    if ((dtype != TESS_F32 && dtype != TESS_BF16) || (accumulate != 0 && accumulate != 1))
        return TESS_ERR_UNSUPPORTED;
    hipError_t e = launch_row_sums(x, m, w, ldx, dtype == TESS_F32, accumulate,
                                   static_cast<float*>(sums_out), static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? TESS_OK : TESS_ERR_HIP;
}

tess_status tess_layernorm_normalize(const void* x, int64_t m, int64_t w, int64_t ldx, int dtype,
                                     const void* sums, int64_t n_total, float eps, void* xhat_out,
                                     int64_t ldo, void* hip_stream)
{
    if (!x || !sums || !xhat_out) return TESS_ERR_NULL;
    if (m < 1 || w < 1 || ldx < w || ldo < w || n_total < w || m > ((int64_t)1 << 32)) return TESS_ERR_SHAPE;
    if ((dtype != TESS_F32 && dtype != TESS_BF16) || !(eps >= 0.0f)) return TESS_ERR_UNSUPPORTED;
    hipError_t e = launch_normalize(x, m, w, ldx, dtype == TESS_F32, static_cast<const float*>(sums),
                                    1.0f / (float)n_total, eps, xhat_out, ldo,
                                    static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? TESS_OK : TESS_ERR_HIP;
}

tess_status tess_layernorm_bwd_row_sums(const void* xhat, int64_t ldx, const void* g, int64_t ldg,
                                        int64_t m, int64_t w, int dtype, void* sums_out,
                                        int accumulate, void* hip_stream)
{
    if (!xhat || !g || !sums_out) return TESS_ERR_NULL;
    if (m < 1 || w < 1 || ldx < w || ldg < w || m > ((int64_t)1 << 32)) return TESS_ERR_SHAPE;
    if ((dtype != TESS_F32 && dtype != TESS_BF16) || (accumulate != 0 && accumulate != 1))
        return TESS_ERR_UNSUPPORTED;
    hipError_t e = launch_row_sums_bwd(xhat, g, m, w, ldx, ldg, dtype == TESS_F32, accumulate,
                                       static_cast<float*>(sums_out), static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? TESS_OK : TESS_ERR_HIP;
}

tess_status tess_layernorm_bwd_apply(const void* xhat, int64_t ldx, const void* g, int64_t ldg,
                                     int64_t m, int64_t w, int dtype, const void* sums_bwd,
                                     const void* sums_fwd, int64_t n_total, float eps,
                                     void* dx_out, int64_t ldo, void* hip_stream)
{
    if (!xhat || !g || !sums_bwd || !sums_fwd || !dx_out) return TESS_ERR_NULL;
    if (m < 1 || w < 1 || ldx < w || ldg < w || ldo < w || n_total < w || m > ((int64_t)1 << 32))
        return TESS_ERR_SHAPE;
    if ((dtype != TESS_F32 && dtype != TESS_BF16) || !(eps >= 0.0f)) return TESS_ERR_UNSUPPORTED;
    hipError_t e = launch_layernorm_bwd(xhat, g, m, w, ldx, ldg, dtype == TESS_F32,
                                        static_cast<const float*>(sums_bwd),
                                        static_cast<const float*>(sums_fwd), 1.0f / (float)n_total, eps,
                                        dx_out, ldo, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? TESS_OK : TESS_ERR_HIP;
}

tess_status tess_probe_mfma_rate(void* sink, int32_t workgroups, int32_t iters, int32_t data,
                                 void* hip_stream)
{
    if (!sink) return TESS_ERR_NULL;
    if (workgroups < 1 || workgroups > 65536 || iters < 1) return TESS_ERR_SHAPE;
    if (data != 0 && data != 1) return TESS_ERR_UNSUPPORTED;
    hipError_t e = launch_mfma_probe(static_cast<float*>(sink), workgroups, iters, data,
                                     static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? TESS_OK : TESS_ERR_HIP;
}

tess_status tess_diag_set_plan_override(int32_t tile, int32_t k_splits)
{
    if ((tile != 0 && tile != 128 && tile != 256) || k_splits < 0 || k_splits > 64) return TESS_ERR_UNSUPPORTED;
    g_force_tile.store(tile, std::memory_order_relaxed);
    g_force_splits.store(k_splits, std::memory_order_relaxed);
    return TESS_OK;
}

tess_status tess_tile_of_block(int32_t block, int32_t tiles_m, int32_t tiles_n, int32_t* tm,
                               int32_t* tn)
{
    if (!tm || !tn) return TESS_ERR_NULL;
    if (tiles_m < 1 || tiles_n < 1 || tiles_m > 32768 || tiles_n > 32768) return TESS_ERR_SHAPE;
    if (block < 0 || (int64_t)block >= (int64_t)tiles_m * tiles_n) return TESS_ERR_SHAPE;
    int r, c;
    tile_of_block(block, tiles_m, tiles_n, r, c);
    *tm = r;
    *tn = c;
    return TESS_OK;
}

const char* tess_status_string(int status)
{
    switch (status) {
        case TESS_OK: return "TESS_OK";
        case TESS_ERR_NULL: return "TESS_ERR_NULL";
        case TESS_ERR_GRID: return "TESS_ERR_GRID";
        case TESS_ERR_SHAPE: return "TESS_ERR_SHAPE";
        case TESS_ERR_ALIGN: return "TESS_ERR_ALIGN";
        case TESS_ERR_UNSUPPORTED: return "TESS_ERR_UNSUPPORTED";
        case TESS_ERR_WORKSPACE: return "TESS_ERR_WORKSPACE";
        case TESS_ERR_HIP: return "TESS_ERR_HIP";
        default: return "TESS_ERR_?";
    }
}

const char* tess_version(void) { return "0.1"; }

}  // extern "C"
