// extern "C" boundary of the sparsified-FFN library: argument checks, workspace carving, and the
// order of kernel launches of Alg. 1 / Alg. 2 (paper Section 3).  No allocation, no synchronisation.
#include <stdio.h>
#include <string.h>

#include "../../include/sparseffn.h"
#include "kernels.hpp"

using namespace sffn;

namespace {

thread_local char g_err[256] = "";

int fail(int code, const char* fmt, const char* a = "") {
    snprintf(g_err, sizeof(g_err), fmt, a);
    return code;
}
int hipfail(hipError_t e, const char* where) {
    snprintf(g_err, sizeof(g_err), "%s: %s", where, hipGetErrorString(e));
    return SFFN_EHIP;
}
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline bool mult64(int64_t v) { return v > 0 && (v % 64) == 0; }
inline size_t up256(size_t v) { return (v + 255) & ~(size_t)255; }
inline bool fits_int(int64_t v) { return v < ((int64_t)1 << 31); }
// V:N:M shapes that are built: V = 64 rows, N = 2, M = 8 (fused step, fastest kernels) or 16 / 32 / 64 columns
inline bool vnm_ok(int V, int M) { return V == 64 && (M == 8 || M == 16 || M == 32 || M == 64); }

#define REQUIRE(cond, code, msg) do { if (!(cond)) return fail(code, "%s", msg); } while (0)
#define LAUNCH(expr, where) do { hipError_t e_ = (expr); if (e_ != hipSuccess) return hipfail(e_, where); } while (0)
// inside ffn_sparse_step: launch, then (when profiling) drop an event behind it
#define STAGE(expr, where) do { LAUNCH(expr, where); if (g_prof_on && g_prof_n < kMaxStages) { g_prof_name[g_prof_n] = where; \
        ++g_prof_n; (void)hipEventRecord(g_prof_ev[g_prof_n], s); } } while (0)

// Optional per-launch timing of ffn_sparse_step (measurement aid): events recorded on the caller's
// stream between consecutive launches.
constexpr int kMaxStages = 32;
bool g_prof_on = false;
hipEvent_t g_prof_ev[kMaxStages + 1];
const char* g_prof_name[kMaxStages];
int g_prof_n = 0;

// The workspace is three regions laid end to end, [scratch | saved | weights] (the split forward / backward calls take them as three buffers):
//   scratch  nothing in it outlives a call (layers and micro-batches may share one)
//   saved    what the backward pass reads of the forward pass (Alg. 2 line 1), per layer and micro-batch in flight
//   weights  what the pruning passes write: per layer, good until the weights change (SFFN_FLAG_WEIGHTS_PACKED reads it)
struct FullLayout {
    sffn_ws_layout pub;
    // internal operands of the GEMMs, all in the blocked layout
    size_t w1_vblk, w1_mblk, w2t_vblk, w2t_mblk, x_blk, xt_blk, dy_blk, dyt_blk, w2_blk, w1t_blk, a24_vblk, a24_mblk, at_blk, kmask, total;
    size_t scratch_end, saved_end;      // region boundaries: scratch = [0, scratch_end), saved = [scratch_end, saved_end), weights = [saved_end, total)
};

// Where the three regions of a step's workspace live: one buffer (the one-call entry points) or three (the split calls)
struct Regions {
    unsigned char *scratch = nullptr, *saved = nullptr, *weights = nullptr;
    size_t scratch_end = 0, saved_end = 0;
    unsigned char* at(size_t off) const { return off < scratch_end ? scratch + off : off < saved_end ? saved + (off - scratch_end) : weights + (off - saved_end); }
};
// buf == nullptr: `workspace` holds [scratch | saved | weights] back to back.  Returns 0 or the error code to hand back.
inline int place_regions(const sffn_buffers* buf, void* workspace, size_t ws_bytes, size_t scratch_end, size_t saved_end, size_t total, Regions* r) {
    r->scratch_end = scratch_end; r->saved_end = saved_end;
    if (!buf) {
        if (!workspace || ws_bytes < total) return SFFN_EWORKSPACE;
        r->scratch = (unsigned char*)workspace; r->saved = r->scratch + scratch_end; r->weights = r->scratch + saved_end;
        return SFFN_OK;
    }
    if (!buf->scratch || !buf->saved || !buf->weights) return SFFN_EWORKSPACE;
    if (buf->scratch_bytes < scratch_end || buf->saved_bytes < saved_end - scratch_end || buf->weights_bytes < total - saved_end) return SFFN_EWORKSPACE;
    if ((reinterpret_cast<uintptr_t>(buf->scratch) | reinterpret_cast<uintptr_t>(buf->saved) | reinterpret_cast<uintptr_t>(buf->weights)) & 255u) return SFFN_EINVAL;
    {   // the three regions must not overlap (one allocation carved into three consecutive pieces is fine)
        const uintptr_t lo[3] = {reinterpret_cast<uintptr_t>(buf->scratch), reinterpret_cast<uintptr_t>(buf->saved), reinterpret_cast<uintptr_t>(buf->weights)};
        const size_t len[3] = {scratch_end, saved_end - scratch_end, total - saved_end};
        for (int i = 0; i < 3; ++i)
            for (int j = i + 1; j < 3; ++j)
                if (lo[i] < lo[j] + len[j] && lo[j] < lo[i] + len[i]) return SFFN_EINVAL;
    }
    r->scratch = (unsigned char*)buf->scratch; r->saved = (unsigned char*)buf->saved; r->weights = (unsigned char*)buf->weights;
    return SFFN_OK;
}

// Blocks of M = 16, 32, 64 columns take the fused path (V:N:M epilogues inside eqs. (1), (4), gathered-row eqs. (3), (7)) when the
// gathered-row kernel covers the shape and the caller does not ask for the unfused reference path.
bool fused_wide(const sffn_cfg* c) {
    return c->M != 8 && !(c->flags & SFFN_FLAG_UNFUSED) && vnm_spmm_gather_ok(c->T, c->D, c->F, c->M) && c->F * c->D * 2 < ((int64_t)1 << 31);
}

// E = number of experts (1 for the plain step): every weight-shaped tensor holds E matrices back to back.
bool make_layout(const sffn_cfg* c, FullLayout* L, int n_experts = 1) {
    if (!c || !mult64(c->T) || !mult64(c->D) || !mult64(c->F) || n_experts < 1) return false;
    if (!vnm_ok(c->V, c->M)) return false;
    const size_t M = (size_t)c->M;                                    // wider blocks: smaller packed tensors, unfused path
    if (c->F % (2 * M) != 0) return false;
    // the dense y1 / dy2 exist only where a kernel stores them: on request in the fused step, always in the unfused one
    const bool fused = M == 8 || fused_wide(c);
    const bool dense = (c->flags & SFFN_FLAG_KEEP_DENSE) || !fused;
    const bool lean = fused && (c->flags & SFFN_FLAG_LEAN);          // canonical copies that are not written take no room
    const size_t T = c->T, D = c->D, F = (size_t)c->F * n_experts;   // F only sizes weight-shaped tensors below ...
    const size_t TF = T * (size_t)c->F;                               // ... token x hidden tensors use TF
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += up256(bytes); return o; };
    // ---- scratch -----------------------------------------------------------------------------------------------------------------------
    L->pub.y1 = take(dense ? TF * 2 : 0);
    L->pub.dy2 = take(dense ? TF * 2 : 0);
    L->pub.y2_vals = take(lean && M == 8 ? 0 : TF * 4 / M);        // (M >= 16: eqs. (3), (7) read the canonical arrays)
    L->pub.dy1_vals = take(lean && M == 8 ? 0 : TF * 4 / M);
    L->x_blk = take(T * D * 2);
    L->dy_blk = take(T * D * 2);           L->dyt_blk = take(D * T * 2);
    L->a24_vblk = take(TF);             // M = 8: the survivors in the V:2:8 kernel's units; unfused path: the plain-2:4 view
    L->w1t_blk = take(fused ? 0 : D * F * 2);      // unfused path only: W2.T or W1.T, row-major
    L->scratch_end = off;
    // ---- saved -------------------------------------------------------------------------------------------------------------------------
    L->pub.y2_meta = take(TF / (2 * M));   L->pub.colidx = take(TF / 64 / M * 4);
    L->pub.y1_kept_bytes = fused ? TF * 4 / M : 0;
    L->pub.y1_kept = take(L->pub.y1_kept_bytes);
    L->xt_blk = take(D * T * 2);
    L->a24_mblk = take(TF / 8);         // M = 8: metadata and regrouped column offsets for the V:2:8 kernel (eq. (7) reads them again)
    L->at_blk = take(M == 8 ? TF : 2 * TF);   // M = 8: transposed activation compacted to the kept hidden units [F / 2, T]; wider: dense [F, T]
    L->kmask = take(TF / 64 / 8);       // kept-column bit mask per (64-token block, group of 8 hidden units)
    L->saved_end = off;
    // ---- weights -----------------------------------------------------------------------------------------------------------------------
    L->pub.w1_vals = take(lean ? 0 : F * D);          L->pub.w1_meta = take(lean ? 0 : F * D / 8);
    L->pub.w2t_vals = take(lean ? 0 : F * D);         L->pub.w2t_meta = take(lean ? 0 : F * D / 8);
    L->w1_vblk = take(F * D);              L->w1_mblk = take(F * D / 8);
    L->w2t_vblk = take(F * D);             L->w2t_mblk = take(F * D / 8);
    L->w2_blk = take(fused ? D * F * 2 : 0);       // fused paths: W2.T [F, D] per expert, written by the pruning pass of W2
    L->total = off;
    L->pub.total = off;
    return true;
}

}  // namespace

extern "C" {

int sffn_version(void) { return 110; }
const char* sffn_last_error(void) { return g_err; }
// internal (not declared in the public header): lets the library's other source files leave a text behind sffn_last_error()
int sffn_noalloc_set_error(int code, const char* text) { return fail(code, "%s", text); }

size_t sffn_workspace_bytes(const sffn_cfg* cfg) {
    FullLayout L;
    return make_layout(cfg, &L) ? L.total : 0;
}

int sffn_workspace_layout(const sffn_cfg* cfg, sffn_ws_layout* out) {
    FullLayout L;
    REQUIRE(out != nullptr, SFFN_EINVAL, "sffn_workspace_layout: out is null");
    REQUIRE(make_layout(cfg, &L), SFFN_EINVAL, "sffn_workspace_layout: T, D, F must be positive multiples of 64, V = 64, M in {8, 16, 32, 64}, F a multiple of 2 M");
    *out = L.pub;
    return SFFN_OK;
}

size_t sffn_vnm_spmm_workspace_bytes(int64_t T, int64_t N, int64_t Kfull, int w_kmajor) {
    if (!mult64(T) || !mult64(N) || !mult64(Kfull)) return 0;
    (void)w_kmajor;         // either orientation may need the other one's copy of Wd (plain-2:4 route: [N, Kfull]; gathered route: [Kfull, N])
    return up256((size_t)T * Kfull) + up256((size_t)T * Kfull / 8) + up256((size_t)N * Kfull * 2);
}

size_t sffn_vnm_wgrad_workspace_bytes(int64_t T, int64_t F, int64_t N) {
    if (!mult64(T) || !mult64(N) || !mult64(F)) return 0;
    return up256((size_t)F * T * 2) + up256((size_t)N * T * 2);
}

int prune24_compress(const uint16_t* src, int64_t R, int64_t K, int64_t ld, int trans, int mode, uint16_t* vals,
                     uint8_t* meta, void* stream) {
    REQUIRE(src && vals && meta, SFFN_EINVAL, "prune24_compress: null pointer");
    REQUIRE(mult64(R) && mult64(K), SFFN_EINVAL, "prune24_compress: R and K must be positive multiples of 64");
    REQUIRE(ld >= (trans ? R : K) && ld % 8 == 0, SFFN_EINVAL, "prune24_compress: ld too small or not a multiple of 8");
    REQUIRE(mode == SFFN_MODE_HARD || mode == SFFN_MODE_SOFT, SFFN_EINVAL, "prune24_compress: unknown mode");
    REQUIRE(trans == 0 || trans == 1, SFFN_EINVAL, "prune24_compress: trans must be 0 or 1");
    REQUIRE(aligned16(src) && aligned16(vals) && aligned16(meta), SFFN_EINVAL, "prune24_compress: pointers must be 16-byte aligned");
    REQUIRE(fits_int(R) && fits_int(K), SFFN_EUNSUPPORTED, "prune24_compress: dimension above 2^31");
    LAUNCH(launch_prune24(src, R, K, ld, trans, mode, vals, meta, (hipStream_t)stream), "prune24_compress");
    return SFFN_OK;
}

int sqrelu_vnm_compress(const uint16_t* y1, int64_t T, int64_t F, int V, int M, uint16_t* vals, uint8_t* meta,
                        uint8_t* colidx, void* stream) {
    REQUIRE(y1 && vals && meta && colidx, SFFN_EINVAL, "sqrelu_vnm_compress: null pointer");
    REQUIRE(mult64(T) && mult64(F), SFFN_EINVAL, "sqrelu_vnm_compress: T and F must be positive multiples of 64");
    REQUIRE(vnm_ok(V, M), SFFN_EUNSUPPORTED, "sqrelu_vnm_compress: only V=64 with M in {8, 16, 32, 64} is built");
    REQUIRE(F % (2 * M) == 0, SFFN_EINVAL, "sqrelu_vnm_compress: F must be a multiple of 2 M");
    REQUIRE(aligned16(y1) && aligned16(vals) && aligned16(meta) && aligned16(colidx), SFFN_EINVAL,
            "sqrelu_vnm_compress: pointers must be 16-byte aligned");
    REQUIRE(fits_int(T) && fits_int(F) && T / 64 < 65536, SFFN_EUNSUPPORTED, "sqrelu_vnm_compress: T too large");
    LAUNCH(launch_sqrelu_vnm_compress_m(y1, T, F, M, vals, meta, colidx, (hipStream_t)stream), "sqrelu_vnm_compress");
    return SFFN_OK;
}

static int spmm24_common(const char* name, const uint16_t* X, const uint16_t* w_vals, const uint8_t* w_meta, const float* bias,
                         int64_t T, int64_t N, int64_t K, uint16_t* out, void* stream) {
    REQUIRE(X && w_vals && w_meta && out, SFFN_EINVAL, "spmm24: null pointer");
    REQUIRE(mult64(T) && mult64(N) && mult64(K), SFFN_EINVAL, "spmm24: T, N, K must be positive multiples of 64");
    REQUIRE(aligned16(X) && aligned16(w_vals) && aligned16(w_meta) && aligned16(out) && aligned16(bias), SFFN_EINVAL,
            "spmm24: pointers must be 16-byte aligned");
    REQUIRE(fits_int(T) && fits_int(N) && fits_int(K), SFFN_EUNSUPPORTED, "spmm24: dimension above 2^31");
    LAUNCH(launch_gemm_nt(1, w_vals, w_meta, X, bias, N, T, K, 1, out, N, (hipStream_t)stream), name);
    return SFFN_OK;
}

int spmm24_fwd(const uint16_t* X, const uint16_t* w_vals, const uint8_t* w_meta, const float* bias, int64_t T, int64_t N,
               int64_t K, uint16_t* out, void* stream) {
    return spmm24_common("spmm24_fwd", X, w_vals, w_meta, bias, T, N, K, out, stream);
}

int spmm24_dgrad(const uint16_t* dY, const uint16_t* wt_vals, const uint8_t* wt_meta, int64_t T, int64_t N, int64_t K,
                 uint16_t* out, void* stream) {
    return spmm24_common("spmm24_dgrad", dY, wt_vals, wt_meta, nullptr, T, N, K, out, stream);
}

// ---- "prepared" 2:4 operand: the packed matrix in the layout the tile kernel streams fastest (1 KB blocks of values, 256-byte
//      metadata units), produced by the pruning pass itself, so that the stand-alone GEMMs run the same main loop as the fused step ----
size_t sffn_prepared24_bytes(int64_t R, int64_t K) {
    if (!mult64(R) || !mult64(K)) return 0;
    return up256((size_t)R * K) + up256((size_t)R * K / 8);
}

int prune24_compress_prepared(const uint16_t* src, int64_t R, int64_t K, int64_t ld, int mode, uint16_t* vals, uint8_t* meta, void* prepared,
                              void* stream) {
    REQUIRE(src && vals && meta && prepared, SFFN_EINVAL, "prune24_compress_prepared: null pointer");
    REQUIRE(mult64(R) && mult64(K), SFFN_EINVAL, "prune24_compress_prepared: R and K must be positive multiples of 64");
    REQUIRE(ld >= K && ld % 8 == 0, SFFN_EINVAL, "prune24_compress_prepared: ld too small or not a multiple of 8");
    REQUIRE(mode == SFFN_MODE_HARD || mode == SFFN_MODE_SOFT, SFFN_EINVAL, "prune24_compress_prepared: unknown mode");
    REQUIRE(aligned16(src) && aligned16(vals) && aligned16(meta) && aligned16(prepared), SFFN_EINVAL, "prune24_compress_prepared: pointers must be 16-byte aligned");
    REQUIRE(fits_int(R) && fits_int(K) && R / 16 < 65536 * 16, SFFN_EUNSUPPORTED, "prune24_compress_prepared: dimension too large");
    uint8_t* pb = (uint8_t*)prepared;
    LAUNCH(launch_prune24_step(src, R, K, ld, 0, mode, vals, meta, (uint16_t*)pb, pb + up256((size_t)R * K), nullptr, (hipStream_t)stream),
           "prune24_compress_prepared");
    return SFFN_OK;
}

size_t sffn_spmm24_prepared_workspace_bytes(int64_t T, int64_t K) {
    if (!mult64(T) || !mult64(K)) return 0;
    return up256((size_t)T * K * 2);
}

int spmm24_prepared(const uint16_t* X, const void* w_prepared, const float* bias, int64_t T, int64_t N, int64_t K, uint16_t* out,
                    void* workspace, size_t ws_bytes, void* stream) {
    REQUIRE(X && w_prepared && out, SFFN_EINVAL, "spmm24_prepared: null pointer");
    REQUIRE(mult64(T) && mult64(N) && mult64(K), SFFN_EINVAL, "spmm24_prepared: T, N, K must be positive multiples of 64");
    REQUIRE(aligned16(X) && aligned16(w_prepared) && aligned16(out) && aligned16(bias) && aligned16(workspace), SFFN_EINVAL,
            "spmm24_prepared: pointers must be 16-byte aligned");
    REQUIRE(fits_int(T) && fits_int(N) && fits_int(K) && T / 64 < 65536, SFFN_EUNSUPPORTED, "spmm24_prepared: dimension too large");
    REQUIRE(workspace && ws_bytes >= sffn_spmm24_prepared_workspace_bytes(T, K), SFFN_EWORKSPACE, "spmm24_prepared: workspace missing or too small");
    hipStream_t s = (hipStream_t)stream;
    uint16_t* xb = (uint16_t*)workspace;
    const uint8_t* pb = (const uint8_t*)w_prepared;
    LAUNCH(launch_transpose(X, T, K, K, nullptr, 1, xb, s), "spmm24_prepared/block(X)");         // X once through HBM into 1 KB blocks
    const VnmEpilogue plain;
    LAUNCH(launch_gemm_vnm_epilogue((const uint16_t*)pb, pb + up256((size_t)N * K), xb, bias, N, T, K, out, plain, s), "spmm24_prepared/gemm");
    return SFFN_OK;
}

int vnm_spmm(const uint16_t* a_vals, const uint8_t* a_meta, const uint8_t* a_colidx, const uint16_t* Wd, int64_t ldw,
             int w_kmajor, int64_t T, int64_t N, int64_t Kfull, int V, int M, uint16_t* out, void* workspace,
             size_t ws_bytes, void* stream) {
    REQUIRE(a_vals && a_meta && a_colidx && Wd && out, SFFN_EINVAL, "vnm_spmm: null pointer");
    REQUIRE(mult64(T) && mult64(N) && mult64(Kfull), SFFN_EINVAL, "vnm_spmm: T, N, Kfull must be positive multiples of 64");
    REQUIRE(vnm_ok(V, M), SFFN_EUNSUPPORTED, "vnm_spmm: only V=64 with M in {8, 16, 32, 64} is built");
    REQUIRE(Kfull % (2 * M) == 0, SFFN_EINVAL, "vnm_spmm: Kfull must be a multiple of 2 M");
    REQUIRE(w_kmajor == 0 || w_kmajor == 1, SFFN_EINVAL, "vnm_spmm: w_kmajor must be 0 or 1");
    REQUIRE(ldw >= (w_kmajor ? N : Kfull) && ldw % 8 == 0, SFFN_EINVAL, "vnm_spmm: ldw too small or not a multiple of 8");
    REQUIRE(w_kmajor == 1 || ldw == Kfull, SFFN_EUNSUPPORTED, "vnm_spmm: a padded row stride needs w_kmajor=1");
    REQUIRE(aligned16(a_vals) && aligned16(a_meta) && aligned16(a_colidx) && aligned16(Wd) && aligned16(out) && aligned16(workspace),
            SFFN_EINVAL, "vnm_spmm: pointers must be 16-byte aligned");
    REQUIRE(fits_int(T) && fits_int(N) && fits_int(Kfull) && T < 65536 * 64, SFFN_EUNSUPPORTED, "vnm_spmm: dimension too large");
    REQUIRE(workspace && ws_bytes >= sffn_vnm_spmm_workspace_bytes(T, N, Kfull, w_kmajor), SFFN_EWORKSPACE,
            "vnm_spmm: workspace missing or too small");
    hipStream_t s = (hipStream_t)stream;
    unsigned char* ws = (unsigned char*)workspace;
    uint16_t* v24 = (uint16_t*)ws;
    uint8_t* m24 = ws + up256((size_t)T * Kfull);
    const uint16_t* W = Wd;
    uint16_t* wcopy = (uint16_t*)(m24 + up256((size_t)T * Kfull / 8));
    if (M == 8 && vnm8_gemm_ok(T, N, Kfull, w_kmajor ? ldw : N)) {
        // the 256-token tile kernel of the fused step: the packed arrays regrouped into its units (one small pass), Wd contraction-major
        uint16_t* vcb = v24;
        uint8_t* mcb = m24;
        uint8_t* cixt = m24 + up256((size_t)T * Kfull / 16);
        int64_t ldk = ldw;
        if (!w_kmajor) {
            LAUNCH(launch_transpose(Wd, N, Kfull, ldw, wcopy, 0, nullptr, s), "vnm_spmm/transpose");
            W = wcopy; ldk = N;
        }
        LAUNCH(launch_vnm8_repack(a_vals, a_meta, a_colidx, T, Kfull, vcb, mcb, cixt, s), "vnm_spmm/repack");
        LAUNCH(launch_vnm8_gemm(vcb, mcb, cixt, W, ldk, T, N, Kfull, out, N, s), "vnm_spmm/gemm");
        return SFFN_OK;
    }
    if ((M >= 16 || w_kmajor) && vnm_spmm_gather_ok(T, N, Kfull, M) && Kfull * (w_kmajor ? ldw : N) * 2 < ((int64_t)1 << 31)) {
        // contract over the 4 Kfull / M kept columns only, gathering their rows of the [Kfull, N] operand (M = 8: the two routes
        // are equally fast, so it is taken only when it saves the transpose of Wd)
        int64_t ldk = ldw;
        if (!w_kmajor) {
            LAUNCH(launch_transpose(Wd, N, Kfull, ldw, wcopy, 0, nullptr, s), "vnm_spmm/transpose");
            W = wcopy; ldk = N;
        }
        LAUNCH(launch_vnm_spmm_gather(a_vals, a_meta, a_colidx, W, ldk, T, N, Kfull, M, out, N, s), "vnm_spmm/gather");
        return SFFN_OK;
    }
    REQUIRE(T < 65536, SFFN_EUNSUPPORTED, "vnm_spmm: T must be below 65536 on the plain-2:4 route (shapes the gathered-row kernel does not cover)");
    if (M == 8) LAUNCH(launch_vnm_to_24(a_vals, a_meta, a_colidx, T, Kfull, v24, m24, s), "vnm_spmm/to24");
    else        LAUNCH(launch_vnm_to_24_m(a_vals, a_meta, a_colidx, T, Kfull, M, v24, m24, s), "vnm_spmm/to24");
    if (w_kmajor) {
        uint16_t* wt = wcopy;
        LAUNCH(launch_transpose(Wd, Kfull, N, ldw, wt, 0, nullptr, s), "vnm_spmm/transpose");
        W = wt;
    }
    LAUNCH(launch_gemm_nt(1, v24, m24, W, nullptr, T, N, Kfull, 0, out, N, s), "vnm_spmm/gemm");
    return SFFN_OK;
}

int dsqrelu_vnm(const uint16_t* dy2, const uint16_t* y1, const uint8_t* meta, const uint8_t* colidx, int64_t T, int64_t F,
                int V, int M, uint16_t* dvals, void* stream) {
    REQUIRE(dy2 && y1 && meta && colidx && dvals, SFFN_EINVAL, "dsqrelu_vnm: null pointer");
    REQUIRE(mult64(T) && mult64(F), SFFN_EINVAL, "dsqrelu_vnm: T and F must be positive multiples of 64");
    REQUIRE(vnm_ok(V, M), SFFN_EUNSUPPORTED, "dsqrelu_vnm: only V=64 with M in {8, 16, 32, 64} is built");
    REQUIRE(F % (2 * M) == 0, SFFN_EINVAL, "dsqrelu_vnm: F must be a multiple of 2 M");
    REQUIRE(aligned16(dy2) && aligned16(y1) && aligned16(meta) && aligned16(colidx) && aligned16(dvals), SFFN_EINVAL,
            "dsqrelu_vnm: pointers must be 16-byte aligned");
    REQUIRE(fits_int(T) && fits_int(F) && T < 65536, SFFN_EUNSUPPORTED, "dsqrelu_vnm: T must be below 65536");
    if (M == 8) LAUNCH(launch_dsqrelu_vnm(dy2, y1, meta, colidx, T, F, dvals, (hipStream_t)stream), "dsqrelu_vnm");
    else        LAUNCH(launch_dsqrelu_vnm_m(dy2, y1, meta, colidx, T, F, M, dvals, (hipStream_t)stream), "dsqrelu_vnm");
    return SFFN_OK;
}

int vnm_wgrad(const uint16_t* a_vals, const uint8_t* a_meta, const uint8_t* a_colidx, const uint16_t* G, int64_t T,
              int64_t F, int64_t N, int V, int M, int out_f_major, uint16_t* out, void* workspace, size_t ws_bytes,
              void* stream) {
    REQUIRE(a_vals && a_meta && a_colidx && G && out, SFFN_EINVAL, "vnm_wgrad: null pointer");
    REQUIRE(mult64(T) && mult64(N) && mult64(F), SFFN_EINVAL, "vnm_wgrad: T, F, N must be positive multiples of 64");
    REQUIRE(vnm_ok(V, M), SFFN_EUNSUPPORTED, "vnm_wgrad: only V=64 with M in {8, 16, 32, 64} is built");
    REQUIRE(F % (2 * M) == 0, SFFN_EINVAL, "vnm_wgrad: F must be a multiple of 2 M");
    REQUIRE(out_f_major == 0 || out_f_major == 1, SFFN_EINVAL, "vnm_wgrad: out_f_major must be 0 or 1");
    REQUIRE(aligned16(a_vals) && aligned16(a_meta) && aligned16(a_colidx) && aligned16(G) && aligned16(out) && aligned16(workspace),
            SFFN_EINVAL, "vnm_wgrad: pointers must be 16-byte aligned");
    REQUIRE(fits_int(T) && fits_int(N) && fits_int(F) && T < 65536 * 64, SFFN_EUNSUPPORTED, "vnm_wgrad: dimension too large");
    REQUIRE(workspace && ws_bytes >= sffn_vnm_wgrad_workspace_bytes(T, F, N), SFFN_EWORKSPACE,
            "vnm_wgrad: workspace missing or too small");
    hipStream_t s = (hipStream_t)stream;
    uint16_t* at = (uint16_t*)workspace;
    uint16_t* gt = (uint16_t*)((unsigned char*)workspace + up256((size_t)F * T * 2));
    if (M == 8) LAUNCH(launch_vnm_expand_t(a_vals, a_meta, a_colidx, T, F, at, 0, s), "vnm_wgrad/expand");
    else        LAUNCH(launch_vnm_expand_t_m(a_vals, a_meta, a_colidx, T, F, M, at, s), "vnm_wgrad/expand");
    LAUNCH(launch_transpose(G, T, N, N, gt, 0, nullptr, s), "vnm_wgrad/transpose");
    // C[i=f][j=n]; out_f_major: out[f*N + n] (j contiguous) else out[n*F + f] (i contiguous)
    if (out_f_major) LAUNCH(launch_gemm_nt(0, at, nullptr, gt, nullptr, F, N, T, 0, out, N, s), "vnm_wgrad/gemm");
    else             LAUNCH(launch_gemm_nt(0, at, nullptr, gt, nullptr, F, N, T, 1, out, F, s), "vnm_wgrad/gemm");
    return SFFN_OK;
}

// ---- Section 3.4, closing paragraph: fp8 (E4M3) operands, quantised inside the sparsification passes --------------------------
static inline bool scale_ok(float s) { return s > 0.0f && s < 3.0e38f && (1.0f / s) < 3.0e38f; }
inline bool mult128(int64_t v) { return v > 0 && (v % 128) == 0; }

int quantize_fp8(const uint16_t* src, int64_t n, float scale, uint8_t* codes, float* amax, void* stream) {
    REQUIRE(src && codes, SFFN_EINVAL, "quantize_fp8: null pointer");
    REQUIRE(n > 0 && n % 8 == 0, SFFN_EINVAL, "quantize_fp8: n must be a positive multiple of 8");
    REQUIRE(scale_ok(scale), SFFN_EINVAL, "quantize_fp8: scale must be a positive finite float");
    REQUIRE(aligned16(src) && aligned16(codes) && ((uintptr_t)amax & 3u) == 0, SFFN_EINVAL, "quantize_fp8: pointers must be 16-byte aligned");
    LAUNCH(launch_quantize_fp8(src, n, 1.0f / scale, codes, amax, (hipStream_t)stream), "quantize_fp8");
    return SFFN_OK;
}

int prune24_compress_fp8(const uint16_t* src, int64_t R, int64_t K, int64_t ld, int trans, int mode, float scale, uint8_t* codes, uint8_t* meta,
                         float* amax, void* stream) {
    REQUIRE(src && codes && meta, SFFN_EINVAL, "prune24_compress_fp8: null pointer");
    REQUIRE(mult64(R) && mult64(K), SFFN_EINVAL, "prune24_compress_fp8: R and K must be positive multiples of 64");
    REQUIRE(ld >= (trans ? R : K) && ld % 8 == 0, SFFN_EINVAL, "prune24_compress_fp8: ld too small or not a multiple of 8");
    REQUIRE(mode == SFFN_MODE_HARD || mode == SFFN_MODE_SOFT, SFFN_EINVAL, "prune24_compress_fp8: unknown mode");
    REQUIRE(trans == 0 || trans == 1, SFFN_EINVAL, "prune24_compress_fp8: trans must be 0 or 1");
    REQUIRE(scale_ok(scale), SFFN_EINVAL, "prune24_compress_fp8: scale must be a positive finite float");
    REQUIRE(aligned16(src) && aligned16(codes) && aligned16(meta) && ((uintptr_t)amax & 3u) == 0, SFFN_EINVAL, "prune24_compress_fp8: pointers must be 16-byte aligned");
    REQUIRE(fits_int(R) && fits_int(K), SFFN_EUNSUPPORTED, "prune24_compress_fp8: dimension above 2^31");
    LAUNCH(launch_prune24_fp8(src, R, K, ld, trans, mode, 1.0f / scale, codes, meta, amax, (hipStream_t)stream), "prune24_compress_fp8");
    return SFFN_OK;
}

int sqrelu_vnm_compress_fp8(const uint16_t* y1, int64_t T, int64_t F, int V, int M, float scale, uint8_t* codes, uint8_t* meta, uint8_t* colidx,
                            float* amax, void* stream) {
    REQUIRE(y1 && codes && meta && colidx, SFFN_EINVAL, "sqrelu_vnm_compress_fp8: null pointer");
    REQUIRE(mult64(T) && mult64(F), SFFN_EINVAL, "sqrelu_vnm_compress_fp8: T and F must be positive multiples of 64");
    REQUIRE(vnm_ok(V, M), SFFN_EUNSUPPORTED, "sqrelu_vnm_compress_fp8: only V=64 with M in {8, 16, 32, 64} is built");
    REQUIRE(F % (2 * M) == 0, SFFN_EINVAL, "sqrelu_vnm_compress_fp8: F must be a multiple of 2 M");
    REQUIRE(scale_ok(scale), SFFN_EINVAL, "sqrelu_vnm_compress_fp8: scale must be a positive finite float");
    REQUIRE(aligned16(y1) && aligned16(codes) && aligned16(meta) && aligned16(colidx) && ((uintptr_t)amax & 3u) == 0, SFFN_EINVAL,
            "sqrelu_vnm_compress_fp8: pointers must be 16-byte aligned");
    REQUIRE(fits_int(T) && fits_int(F) && T / 64 < 65536, SFFN_EUNSUPPORTED, "sqrelu_vnm_compress_fp8: T too large");
    LAUNCH(launch_sqrelu_vnm_compress_fp8(y1, T, F, M, 1.0f / scale, codes, meta, colidx, amax, (hipStream_t)stream), "sqrelu_vnm_compress_fp8");
    return SFFN_OK;
}

int spmm24_fp8(const uint8_t* Xq, float scale_x, const uint8_t* w_codes, const uint8_t* w_meta, float scale_w, const float* bias, int64_t T,
               int64_t N, int64_t K, uint16_t* out, void* stream) {
    REQUIRE(Xq && w_codes && w_meta && out, SFFN_EINVAL, "spmm24_fp8: null pointer");
    REQUIRE(mult64(T) && mult64(N) && mult128(K), SFFN_EINVAL, "spmm24_fp8: T, N must be positive multiples of 64 and K of 128");
    REQUIRE(scale_ok(scale_x) && scale_ok(scale_w), SFFN_EINVAL, "spmm24_fp8: scales must be positive finite floats");
    REQUIRE(aligned16(Xq) && aligned16(w_codes) && aligned16(w_meta) && aligned16(out) && aligned16(bias), SFFN_EINVAL,
            "spmm24_fp8: pointers must be 16-byte aligned");
    REQUIRE(fits_int(T) && fits_int(N) && fits_int(K), SFFN_EUNSUPPORTED, "spmm24_fp8: dimension above 2^31");
    LAUNCH(launch_spmm24_fp8(w_codes, w_meta, Xq, bias, scale_x * scale_w, N, T, K, 1, out, N, (hipStream_t)stream), "spmm24_fp8");
    return SFFN_OK;
}

size_t sffn_vnm_spmm_fp8_workspace_bytes(int64_t T, int64_t N, int64_t Kfull) {
    if (!mult64(T) || !mult64(N) || !mult128(Kfull)) return 0;
    return up256((size_t)T * Kfull / 2) + up256((size_t)T * Kfull / 8) + up256((size_t)N * Kfull);
}

int vnm_spmm_fp8(const uint8_t* a_codes, const uint8_t* a_meta, const uint8_t* a_colidx, float scale_a, const uint8_t* Wq, float scale_w,
                 int w_kmajor, int64_t T, int64_t N, int64_t Kfull, int V, int M, uint16_t* out, void* workspace, size_t ws_bytes, void* stream) {
    REQUIRE(a_codes && a_meta && a_colidx && Wq && out, SFFN_EINVAL, "vnm_spmm_fp8: null pointer");
    REQUIRE(mult64(T) && mult64(N) && mult128(Kfull), SFFN_EINVAL, "vnm_spmm_fp8: T, N must be positive multiples of 64 and Kfull of 128");
    REQUIRE(vnm_ok(V, M), SFFN_EUNSUPPORTED, "vnm_spmm_fp8: only V=64 with M in {8, 16, 32, 64} is built");
    REQUIRE(Kfull % (2 * M) == 0, SFFN_EINVAL, "vnm_spmm_fp8: Kfull must be a multiple of 2 M");
    REQUIRE(w_kmajor == 0 || w_kmajor == 1, SFFN_EINVAL, "vnm_spmm_fp8: w_kmajor must be 0 or 1");
    REQUIRE(scale_ok(scale_a) && scale_ok(scale_w), SFFN_EINVAL, "vnm_spmm_fp8: scales must be positive finite floats");
    REQUIRE(aligned16(a_codes) && aligned16(a_meta) && aligned16(a_colidx) && aligned16(Wq) && aligned16(out) && aligned16(workspace), SFFN_EINVAL,
            "vnm_spmm_fp8: pointers must be 16-byte aligned");
    REQUIRE(fits_int(T) && fits_int(N) && fits_int(Kfull) && T < 65536, SFFN_EUNSUPPORTED, "vnm_spmm_fp8: T must be below 65536");
    REQUIRE(workspace && ws_bytes >= sffn_vnm_spmm_fp8_workspace_bytes(T, N, Kfull), SFFN_EWORKSPACE, "vnm_spmm_fp8: workspace missing or too small");
    hipStream_t s = (hipStream_t)stream;
    uint8_t* ws = (uint8_t*)workspace;
    uint8_t* c24 = ws;
    uint8_t* m24 = ws + up256((size_t)T * Kfull / 2);
    uint8_t* wt = m24 + up256((size_t)T * Kfull / 8);
    const uint8_t* W = Wq;
    if (M == 8 && vnm8_gemm_fp8_ok(T, N, Kfull, N)) {
        // the 256-token tile kernel of the fp8 step: the packed arrays regrouped into its units (one small pass), Wq contraction-major
        uint8_t* vcb = c24;
        uint8_t* mcb = m24;
        uint8_t* cixt = m24 + up256((size_t)T * Kfull / 16);
        if (!w_kmajor) {
            LAUNCH(launch_transpose_u8(Wq, N, Kfull, Kfull, wt, s), "vnm_spmm_fp8/transpose");
            W = wt;
        }
        LAUNCH(launch_vnm8_repack_fp8(a_codes, a_meta, a_colidx, T, Kfull, vcb, mcb, cixt, s), "vnm_spmm_fp8/repack");
        LAUNCH(launch_vnm8_gemm_fp8(vcb, mcb, cixt, W, N, scale_a * scale_w, T, N, Kfull, out, N, s), "vnm_spmm_fp8/gemm");
        return SFFN_OK;
    }
    if (M >= 16 && vnm_spmm_gather_fp8_ok(T, N, Kfull, M) && Kfull * N < ((int64_t)1 << 31)) {
        // contract over the 4 Kfull / M kept columns only, gathering their rows of the [Kfull, N] codes (the fp8 step's kernel for wide blocks)
        if (!w_kmajor) {
            LAUNCH(launch_transpose_u8(Wq, N, Kfull, Kfull, wt, s), "vnm_spmm_fp8/transpose");
            W = wt;
        }
        LAUNCH(launch_vnm_spmm_gather_fp8(a_codes, a_meta, a_colidx, W, N, scale_a * scale_w, T, N, Kfull, M, out, N, s), "vnm_spmm_fp8/gather");
        return SFFN_OK;
    }
    LAUNCH(launch_vnm_to_24_fp8(a_codes, a_meta, a_colidx, T, Kfull, M, c24, m24, s), "vnm_spmm_fp8/to24");
    if (w_kmajor) {
        LAUNCH(launch_transpose_u8(Wq, Kfull, N, N, wt, s), "vnm_spmm_fp8/transpose");
        W = wt;
    }
    LAUNCH(launch_spmm24_fp8(c24, m24, W, nullptr, scale_a * scale_w, T, N, Kfull, 0, out, N, s), "vnm_spmm_fp8/gemm");
    return SFFN_OK;
}

// ---- the training step with fp8 operands in eqs. (1), (3), (4), (7) (Section 3.4, closing paragraph) ---------------------------
namespace {
struct Fp8Layout {
    sffn_fp8_ws_layout pub;
    size_t w1_blk, w1_mblk, w2t_blk, w2t_mblk, xq, xt_blk, dyq, dyt_blk, w2q, w1tq, v24, m24, at_blk, kmask, amax_slots, total;
    size_t scratch_end, saved_end;      // [scratch | saved | weights], as in FullLayout
};
// E = number of experts (1 for the plain step): weight-shaped tensors hold E matrices back to back
bool make_fp8_layout(const sffn_cfg* c, Fp8Layout* L, int n_experts = 1) {
    if (!c || !mult64(c->T) || !mult128(c->D) || !mult128(c->F) || c->V != 64 || n_experts < 1) return false;
    if (c->M != 8 && !(vnm_ok(c->V, c->M) && vnm_spmm_gather_fp8_ok(c->T, c->D, c->F, c->M))) return false;
    if (c->flags & ~(SFFN_FLAG_KEEP_DENSE | SFFN_FLAG_FP8_WGRAD | SFFN_FLAG_LEAN | SFFN_FLAG_WEIGHTS_PACKED | SFFN_FLAG_DW_FP32_ACCUMULATE)) return false;
    const bool dense = (c->flags & SFFN_FLAG_KEEP_DENSE) != 0;
    const bool lean = (c->flags & SFFN_FLAG_LEAN) != 0;              // canonical copies that are not written take no room
    const size_t T = c->T, D = c->D, F = (size_t)c->F * n_experts, TF = T * (size_t)c->F, M = (size_t)c->M;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += up256(bytes); return o; };
    // ---- scratch -----------------------------------------------------------------------------------------------------------------------
    L->pub.y1 = take(dense ? TF * 2 : 0);
    L->pub.dy2 = take(dense ? TF * 2 : 0);
    L->pub.y2_codes = take(lean && M == 8 ? 0 : 2 * TF / M);        // (M >= 16: eq. (3) reads the canonical codes)
    L->pub.dy1_vals = take(M == 8 ? TF / 2 : 2 * TF / M);
    L->xq = take(T * D);                   L->dyq = take(T * D);
    L->dyt_blk = take(T * D * 2);
    L->v24 = take(TF / 2);
    L->amax_slots = take((size_t)6 * 64 * 64 * sizeof(float));      // 6 tensors x 64 slots x 256 bytes
    L->scratch_end = off;
    // ---- saved (what the backward pass reads of the forward pass) -------------------------------------------------------------------------
    L->pub.y2_meta = take(TF / (2 * M));    L->pub.colidx = take(TF / 64 / M * 4);
    L->pub.y1_kept = take(4 * TF / M);
    L->xt_blk = take(T * D * 2);
    L->m24 = take(TF / 8);
    L->at_blk = take(TF);                  L->kmask = take(TF / 64 / 8);
    L->saved_end = off;
    // ---- weights (what the two weight passes write; eq. (7) reads W1's codes from here) ---------------------------------------------------
    L->pub.w1_codes = take(lean ? 0 : F * D / 2);     L->pub.w1_meta = take(lean ? 0 : F * D / 8);
    L->pub.w2t_codes = take(lean ? 0 : F * D / 2);    L->pub.w2t_meta = take(lean ? 0 : F * D / 8);
    L->w1_blk = take(F * D / 2);           L->w2t_blk = take(F * D / 2);
    L->w1_mblk = take(F * D / 8);          L->w2t_mblk = take(F * D / 8);
    L->w2q = take(D * F);                  L->w1tq = take(D * F);
    L->total = off;
    L->pub.total = off;
    return true;
}

int run_fp8_step(const sffn_cfg* cfg, const sffn_fp8_scales* sc, int n_experts, const int64_t* seg, const uint16_t* X, const uint16_t* W1,
                 const uint16_t* W2, const float* b1, const uint16_t* dY, uint16_t* Y3, uint16_t* dX, uint16_t* dW1, uint16_t* dW2, void* workspace,
                 size_t ws_bytes, float* amax, void* stream, int phase = 3, const sffn_buffers* buf = nullptr) {
    // phase: bit 0 = Alg. 1 (forward pass), bit 1 = Alg. 2 (backward pass); a split call's halves meet through the workspace
    const bool fwd = (phase & 1) != 0, bwd = (phase & 2) != 0;
    REQUIRE(cfg != nullptr && sc != nullptr, SFFN_EINVAL, "ffn_sparse_step_fp8: cfg or scales is null");
    REQUIRE(aligned16(amax), SFFN_EINVAL, "ffn_sparse_step_fp8: amax must be 16-byte aligned");
    Fp8Layout L;
    REQUIRE(n_experts >= 1 && n_experts <= GemmGroup::kMaxExperts, SFFN_EINVAL, "ffn_sparse_step_fp8_grouped: n_experts must be in 1..64");
    REQUIRE(vnm_ok(cfg->V, cfg->M), SFFN_EUNSUPPORTED, "ffn_sparse_step_fp8: only V = 64 with M in {8, 16, 32, 64} is built");
    REQUIRE(make_fp8_layout(cfg, &L, n_experts), SFFN_EINVAL,
            "ffn_sparse_step_fp8: T must be a positive multiple of 64, D and F of 128 (M >= 16: 4 F / M a multiple of 128); flags: "
            "SFFN_FLAG_KEEP_DENSE, SFFN_FLAG_FP8_WGRAD, SFFN_FLAG_LEAN, SFFN_FLAG_WEIGHTS_PACKED, SFFN_FLAG_DW_FP32_ACCUMULATE");
    REQUIRE(cfg->mode == SFFN_MODE_HARD || cfg->mode == SFFN_MODE_SOFT, SFFN_EINVAL, "ffn_sparse_step_fp8: unknown mode");
    REQUIRE((!fwd || (X && W1 && W2 && Y3)) && (!bwd || (dY && dX && dW1 && dW2)), SFFN_EINVAL, "ffn_sparse_step_fp8: null pointer");
    REQUIRE(aligned16(X) && aligned16(W1) && aligned16(W2) && aligned16(dY) && aligned16(Y3) && aligned16(dX) && aligned16(dW1) && aligned16(dW2) &&
            aligned16(b1) && aligned16(workspace), SFFN_EINVAL, "ffn_sparse_step_fp8: pointers must be 16-byte aligned");
    REQUIRE(scale_ok(sc->x) && scale_ok(sc->w1) && scale_ok(sc->w2) && scale_ok(sc->y2) && scale_ok(sc->dy) && scale_ok(sc->dy1), SFFN_EINVAL,
            "ffn_sparse_step_fp8: scales must be positive finite floats");
    const int64_t T = cfg->T, D = cfg->D, F = cfg->F, E = n_experts;
    REQUIRE(fits_int(T) && fits_int(D) && fits_int(F * E) && T / 64 < 65536 && F * D < ((int64_t)1 << 31) && T * D < ((int64_t)1 << 31), SFFN_EUNSUPPORTED,
            "ffn_sparse_step_fp8: dimension too large");
    GemmGroup g;                                    // g.n = 0: plain step
    if (seg) {
        REQUIRE(seg[0] == 0 && seg[E] == T, SFFN_EINVAL, "ffn_sparse_step_fp8_grouped: seg_offsets must start at 0 and end at T");
        for (int e = 0; e < E; ++e)
            REQUIRE(seg[e + 1] >= seg[e] && seg[e + 1] % 64 == 0, SFFN_EINVAL, "ffn_sparse_step_fp8_grouped: seg_offsets must be ascending multiples of 64");
        g.n = (int)E;
        for (int e = 0; e <= E; ++e) g.seg[e] = (int32_t)seg[e];
    }
    Regions rg;
    {
        const int rc = place_regions(buf, workspace, ws_bytes, L.scratch_end, L.saved_end, L.total, &rg);
        REQUIRE(rc != SFFN_EINVAL, SFFN_EINVAL, "ffn_sparse_forward_fp8 / ffn_sparse_backward_fp8: the three buffers must be 256-byte aligned and must not overlap");
        REQUIRE(rc == SFFN_OK, SFFN_EWORKSPACE, "ffn_sparse_step_fp8: workspace missing or too small (sffn_fp8_workspace_bytes)");
    }
    hipStream_t s = (hipStream_t)stream;
    uint8_t *w1c = rg.at(L.pub.w1_codes), *w1m = rg.at(L.pub.w1_meta), *w2c = rg.at(L.pub.w2t_codes), *w2m = rg.at(L.pub.w2t_meta);
    uint16_t *y1 = (uint16_t*)(rg.at(L.pub.y1)), *dy2 = (uint16_t*)(rg.at(L.pub.dy2)), *dy1v = (uint16_t*)(rg.at(L.pub.dy1_vals)), *ykept = (uint16_t*)(rg.at(L.pub.y1_kept));
    uint8_t *y2c = rg.at(L.pub.y2_codes), *y2m = rg.at(L.pub.y2_meta), *cix = rg.at(L.pub.colidx);
    uint8_t *w1mb = rg.at(L.w1_mblk), *w2mb = rg.at(L.w2t_mblk);
    uint8_t *w1b = rg.at(L.w1_blk), *w2b = rg.at(L.w2t_blk), *xq = rg.at(L.xq), *dyq = rg.at(L.dyq), *w2q = rg.at(L.w2q), *w1tq = rg.at(L.w1tq);
    uint16_t *xtb = (uint16_t*)(rg.at(L.xt_blk)), *dytb = (uint16_t*)(rg.at(L.dyt_blk)), *atb = (uint16_t*)(rg.at(L.at_blk));
    uint8_t *v24 = rg.at(L.v24), *m24 = rg.at(L.m24), *kmask = rg.at(L.kmask);
    const int keep_dense = (cfg->flags & SFFN_FLAG_KEEP_DENSE) ? 1 : 0;
    const bool acc32 = (cfg->flags & SFFN_FLAG_DW_FP32_ACCUMULATE) != 0;      // dW1 / dW2 are float32 accumulators that eqs. (8) / (5) add to
    const bool w8 = (cfg->flags & SFFN_FLAG_FP8_WGRAD) != 0;      // eqs. (5), (8) on codes too: X.T, dY.T and the compact transposed survivors as codes
    if (cfg->flags & SFFN_FLAG_LEAN) {      // no canonical copies of the packed tensors (dy1 stays: eq. (8) in bf16 does not need it either, but it is small)
        w1c = w1m = w2c = w2m = nullptr;
        if (cfg->M == 8) y2c = nullptr;     // (M >= 16: the gathered-row kernel reads the canonical codes)
    }
    const float ix = 1.0f / sc->x, iw1 = 1.0f / sc->w1, iw2 = 1.0f / sc->w2, idy = 1.0f / sc->dy;
    // the three ways a token segment meets its expert's weights (see GemmGroup); strides in the units the kernels index: pairs of codes
    GemmGroup g_packed = g, g_dense = g, g_wgrad = g;
    g_packed.role = 1; g_packed.a_stride = F * D / 4; g_packed.m_stride = F * D / 8; g_packed.bias_stride = F;
    g_dense.role = 0;  g_dense.b_stride = D * F / 2;
    g_wgrad.role = 2;  g_wgrad.out_stride = D * F;
    const GemmGroup* gp = g.n ? &g_packed : nullptr;
    const GemmGroup* gd = g.n ? &g_dense : nullptr;
    const GemmGroup* gw = g.n ? &g_wgrad : nullptr;
    // amax[0..5] = largest magnitude of x, w1, w2, y2's survivors, dy, dy1's survivors (what next step's scales are made of)
    // (collected in 64 slots per tensor inside the workspace, folded by the last launch)
    float* slots = amax ? (float*)(rg.at(L.amax_slots)) : nullptr;
    auto slot_of = [&](int i) { return slots ? slots + (size_t)i * 64 * 64 : nullptr; };
    float *ax = slot_of(0), *aw1 = slot_of(1), *aw2 = slot_of(2), *ay2 = slot_of(3), *ady = slot_of(4), *ady1 = slot_of(5);
    if (g_prof_on) { g_prof_n = 0; (void)hipEventRecord(g_prof_ev[0], s); }
    // amax: the forward pass owns tensors 0-3 (x, w1, w2, y2), the backward pass 4-5 (dy, dy1); a split call clears and folds only its own
    const int a_first = fwd ? 0 : 4, a_count = (bwd ? 6 : 4) - a_first;
    if (amax) STAGE(launch_amax_clear(slot_of(a_first), a_count, s), "step/clear(amax)");
    // One data flow for every block width.  M = 8: the epilogues of eqs. (1), (4) also write the survivors' codes in the units of the V:2:8
    // activation GEMM (gemm_vnm8.hip), which picks the kept rows of the quantised W2.T / W1 while it reads its fragments.  M = 16, 32, 64
    // (Table 5): the general-M epilogues; eqs. (3), (7) fetch only the kept rows (gemm_gather.hip) and read the canonical codes.
    const int M = cfg->M, logM = M == 8 ? 3 : M == 16 ? 4 : M == 32 ? 5 : 6;
    const bool wide = M != 8;
    uint8_t *w2tq = w2q, *w1q = w1tq;                   // W2.T and W1 as row-major codes [F, D] per expert (contraction index = row)
    uint8_t* dy1c = (uint8_t*)dy1v;                     // wide blocks: dy1's survivors leave as codes only
    uint8_t *vcb = v24, *mcb = m24, *cixt = m24 + up256((size_t)T * F / 16);
    GemmGroup g_rows = g;
    g_rows.role = 0; g_rows.b_stride = F * D;
    const GemmGroup* gr = g.n ? &g_rows : nullptr;
    // ---- Alg. 1 -------------------------------------------------------------------------------
    if (fwd && w8) {       // X.T codes for eq. (8) and X codes for eq. (1) in one pass over X
        STAGE(launch_transpose_quantize_fp8_blocked(X, T, D, D, ix, (uint8_t*)xtb, s, ax, xq), "step/quantize(X, X.T)");
    } else if (fwd) {
        STAGE(launch_transpose(X, T, D, D, xtb, 1, nullptr, s), "step/X.T");                                // bf16, for eq. (8)
        STAGE(launch_quantize_fp8_blocked(X, T, D, D, ix, xq, s, ax), "step/quantize(X)");
    }
    // W1 in one pass per expert: pruned (canonical + blocked codes) for eq. (1), and the un-pruned W1 as codes for eq. (7)
    const bool packed = (cfg->flags & SFFN_FLAG_WEIGHTS_PACKED) != 0;    // both weight passes skipped: the previous call's codes are still in the workspace
    for (int64_t e = 0; e < E && fwd && !packed; ++e)
        STAGE(launch_prune24_fp8_step(W1 + e * F * D, F, D, D, 0, cfg->mode, iw1, w1c ? w1c + e * F * D / 2 : nullptr, w1m ? w1m + e * F * D / 8 : nullptr,
                                      w1b + e * F * D / 2, w1mb + e * F * D / 8, s, aw1, w1q + e * F * D), "step/prune24_fp8(W1)+quantize(W1)");
    if (fwd) {   // eq. (1) on codes, then eq. (2) + V:N:M compression on the bf16 tile; the survivors leave as codes (and in bf16 for eq. (5))
        VnmEpilogue ep;
        ep.mode = wide ? 5 : 1; ep.logM = logM; ep.store_dense = keep_dense; ep.vals = (uint16_t*)y2c; ep.meta = y2m; ep.colidx = cix; ep.kmask = kmask;
        ep.ykept = ykept; ep.at = atb; ep.inv_out = 1.0f / sc->y2; ep.at_fp8 = w8; ep.amax = ay2;
        if (!wide) { ep.vcb = (uint16_t*)vcb; ep.mcb = mcb; ep.cixt = cixt; }
        STAGE(launch_gemm_fp8_blocked(w1b, w1mb, xq, b1, sc->x * sc->w1, F, T, D, y1, F, &ep, s, gp), "step/y1+sqrelu_vnm_compress");
    }
    for (int64_t e = 0; e < E && fwd && !packed; ++e)
        STAGE(launch_prune24_fp8_step(W2 + e * D * F, F, D, F, 1, cfg->mode, iw2, w2c ? w2c + e * F * D / 2 : nullptr, w2m ? w2m + e * F * D / 8 : nullptr,
                                      w2b + e * F * D / 2, w2mb + e * F * D / 8, s, aw2, w2tq + e * F * D), "step/prune24_fp8(W2.T)+quantize(W2.T)");
    if (fwd) {
        if (wide) STAGE(launch_vnm_spmm_gather_fp8(y2c, y2m, cix, w2tq, D, sc->y2 * sc->w2, T, D, F, M, Y3, D, s, gr), "step/y3");      // eq. (3)
        else STAGE(launch_vnm8_gemm_fp8(vcb, mcb, cixt, w2tq, D, sc->y2 * sc->w2, T, D, F, Y3, D, s, gr), "step/y3");
    }
    // ---- Alg. 2 -------------------------------------------------------------------------------
    if (bwd && w8) {
        STAGE(launch_transpose_quantize_fp8_blocked(dY, T, D, D, idy, (uint8_t*)dytb, s, ady, dyq), "step/quantize(dY, dY.T)");
    } else if (bwd) {
        STAGE(launch_transpose(dY, T, D, D, dytb, 1, nullptr, s), "step/dY.T");                             // bf16, for eq. (5)
        STAGE(launch_quantize_fp8_blocked(dY, T, D, D, idy, dyq, s, ady), "step/quantize(dY)");
    }
    if (bwd) {
        if (w8) STAGE(launch_wgrad_vnm_fp8((const uint8_t*)atb, kmask, (const uint8_t*)dytb, sc->y2 * sc->dy, F, D, T, 1, dW2, F, s, gw, acc32), "step/dW2");   // eq. (5) on codes
        else STAGE(launch_wgrad_vnm(atb, kmask, dytb, F, D, T, 1, dW2, F, s, gw, acc32), "step/dW2");               // eq. (5), bf16
    }
    if (bwd) {   // eq. (4) on codes, then eq. (6) in bf16 on y2's kept slots; dy1 leaves as codes (eq. (7)) and, at M = 8, in bf16 (canonical)
        VnmEpilogue ep;
        ep.mode = wide ? 6 : 2; ep.logM = logM; ep.store_dense = keep_dense; ep.vals = wide ? (uint16_t*)dy1c : dy1v; ep.meta = y2m; ep.colidx = cix;
        ep.ykept = ykept; ep.at = atb; ep.inv_out = 1.0f / sc->dy1; ep.at_fp8 = w8; ep.amax = ady1;
        if (!wide) ep.vcb = (uint16_t*)vcb;
        STAGE(launch_gemm_fp8_blocked(w2b, w2mb, dyq, nullptr, sc->dy * sc->w2, F, T, D, dy2, F, &ep, s, gp), "step/dy2+dsqrelu_vnm");
    }
    if (bwd) {
        if (wide) STAGE(launch_vnm_spmm_gather_fp8(dy1c, y2m, cix, w1q, D, sc->dy1 * sc->w1, T, D, F, M, dX, D, s, gr), "step/dX");     // eq. (7)
        else STAGE(launch_vnm8_gemm_fp8(vcb, mcb, cixt, w1q, D, sc->dy1 * sc->w1, T, D, F, dX, D, s, gr), "step/dX");
    }
    if (bwd) {
        if (w8) STAGE(launch_wgrad_vnm_fp8((const uint8_t*)atb, kmask, (const uint8_t*)xtb, sc->dy1 * sc->x, F, D, T, 0, dW1, D, s, gw, acc32), "step/dW1");   // eq. (8) on codes
        else STAGE(launch_wgrad_vnm(atb, kmask, xtb, F, D, T, 0, dW1, D, s, gw, acc32), "step/dW1");                // eq. (8), bf16
    }
    if (amax) STAGE(launch_amax_finish(slot_of(a_first), a_count, amax + a_first, s), "step/finish(amax)");
    return SFFN_OK;
}
}  // namespace

size_t sffn_fp8_workspace_bytes(const sffn_cfg* cfg) {
    Fp8Layout L;
    return make_fp8_layout(cfg, &L) ? L.total : 0;
}

int sffn_fp8_workspace_layout(const sffn_cfg* cfg, sffn_fp8_ws_layout* out) {
    Fp8Layout L;
    REQUIRE(out != nullptr, SFFN_EINVAL, "sffn_fp8_workspace_layout: out is null");
    REQUIRE(make_fp8_layout(cfg, &L), SFFN_EINVAL, "sffn_fp8_workspace_layout: T a multiple of 64, D and F of 128, V = 64, M = 8, flags: SFFN_FLAG_KEEP_DENSE, SFFN_FLAG_FP8_WGRAD");
    *out = L.pub;
    return SFFN_OK;
}

int sffn_fp8_grouped_workspace_layout(const sffn_cfg* cfg, int n_experts, sffn_fp8_ws_layout* out) {
    Fp8Layout L;
    REQUIRE(out != nullptr, SFFN_EINVAL, "sffn_fp8_grouped_workspace_layout: out is null");
    REQUIRE(make_fp8_layout(cfg, &L, n_experts), SFFN_EINVAL,
            "sffn_fp8_grouped_workspace_layout: T a multiple of 64, D and F of 128, V = 64, M = 8, n_experts >= 1, flags: SFFN_FLAG_KEEP_DENSE, SFFN_FLAG_FP8_WGRAD");
    *out = L.pub;
    return SFFN_OK;
}

int ffn_sparse_step_fp8(const sffn_cfg* cfg, const sffn_fp8_scales* sc, const uint16_t* X, const uint16_t* W1, const uint16_t* W2, const float* b1,
                        const uint16_t* dY, uint16_t* Y3, uint16_t* dX, uint16_t* dW1, uint16_t* dW2, void* workspace, size_t ws_bytes, float* amax,
                        void* stream) {
    return run_fp8_step(cfg, sc, 1, nullptr, X, W1, W2, b1, dY, Y3, dX, dW1, dW2, workspace, ws_bytes, amax, stream);
}

int ffn_sparse_step_fp8_grouped(const sffn_cfg* cfg, const sffn_fp8_scales* sc, int n_experts, const int64_t* seg_offsets, const uint16_t* X,
                                const uint16_t* W1, const uint16_t* W2, const float* b1, const uint16_t* dY, uint16_t* Y3, uint16_t* dX, uint16_t* dW1,
                                uint16_t* dW2, void* workspace, size_t ws_bytes, float* amax, void* stream) {
    REQUIRE(seg_offsets != nullptr, SFFN_EINVAL, "ffn_sparse_step_fp8_grouped: seg_offsets is null");
    return run_fp8_step(cfg, sc, n_experts, seg_offsets, X, W1, W2, b1, dY, Y3, dX, dW1, dW2, workspace, ws_bytes, amax, stream);
}

// Alg. 1 / Alg. 2 as separate calls; the halves meet through the `saved` and `weights` buffers
int sffn_fp8_buffer_sizes(const sffn_cfg* cfg, int n_experts, sffn_buffers* out) {
    Fp8Layout L;
    REQUIRE(out != nullptr, SFFN_EINVAL, "sffn_fp8_buffer_sizes: out is null");
    REQUIRE(make_fp8_layout(cfg, &L, n_experts), SFFN_EINVAL, "sffn_fp8_buffer_sizes: shape or flags outside what ffn_sparse_step_fp8 accepts");
    out->scratch = out->saved = out->weights = nullptr;
    out->scratch_bytes = L.scratch_end; out->saved_bytes = L.saved_end - L.scratch_end; out->weights_bytes = L.total - L.saved_end;
    return SFFN_OK;
}
int ffn_sparse_forward_fp8(const sffn_cfg* cfg, const sffn_fp8_scales* sc, const uint16_t* X, const uint16_t* W1, const uint16_t* W2, const float* b1,
                           uint16_t* Y3, const sffn_buffers* buf, float* amax, void* stream) {
    REQUIRE(buf != nullptr, SFFN_EINVAL, "ffn_sparse_forward_fp8: buf is null");
    return run_fp8_step(cfg, sc, 1, nullptr, X, W1, W2, b1, nullptr, Y3, nullptr, nullptr, nullptr, nullptr, 0, amax, stream, 1, buf);
}
int ffn_sparse_backward_fp8(const sffn_cfg* cfg, const sffn_fp8_scales* sc, const uint16_t* dY, uint16_t* dX, uint16_t* dW1, uint16_t* dW2,
                            const sffn_buffers* buf, float* amax, void* stream) {
    REQUIRE(buf != nullptr, SFFN_EINVAL, "ffn_sparse_backward_fp8: buf is null");
    return run_fp8_step(cfg, sc, 1, nullptr, nullptr, nullptr, nullptr, nullptr, dY, nullptr, dX, dW1, dW2, nullptr, 0, amax, stream, 2, buf);
}
int ffn_sparse_forward_fp8_grouped(const sffn_cfg* cfg, const sffn_fp8_scales* sc, int n_experts, const int64_t* seg_offsets, const uint16_t* X,
                                   const uint16_t* W1, const uint16_t* W2, const float* b1, uint16_t* Y3, const sffn_buffers* buf, float* amax,
                                   void* stream) {
    REQUIRE(seg_offsets != nullptr && buf != nullptr, SFFN_EINVAL, "ffn_sparse_forward_fp8_grouped: seg_offsets or buf is null");
    return run_fp8_step(cfg, sc, n_experts, seg_offsets, X, W1, W2, b1, nullptr, Y3, nullptr, nullptr, nullptr, nullptr, 0, amax, stream, 1, buf);
}
int ffn_sparse_backward_fp8_grouped(const sffn_cfg* cfg, const sffn_fp8_scales* sc, int n_experts, const int64_t* seg_offsets, const uint16_t* dY,
                                    uint16_t* dX, uint16_t* dW1, uint16_t* dW2, const sffn_buffers* buf, float* amax, void* stream) {
    REQUIRE(seg_offsets != nullptr && buf != nullptr, SFFN_EINVAL, "ffn_sparse_backward_fp8_grouped: seg_offsets or buf is null");
    return run_fp8_step(cfg, sc, n_experts, seg_offsets, nullptr, nullptr, nullptr, nullptr, dY, nullptr, dX, dW1, dW2, nullptr, 0, amax, stream, 2, buf);
}

// ---- Section 3.3 / Alg. 3: neuron-level experts that emit the V:N:M format ----------------------------------------
int64_t sffn_venom_rows(int64_t T, int M) {
    if (T < 0 || !vnm_ok(64, M)) return 0;
    return (T + 63) / 64 * 64 + 64 * (M / 4);
}

size_t sffn_venom_route_workspace_bytes(int64_t T, int M) {
    const int64_t cap = sffn_venom_rows(T, M);
    if (cap == 0) return 0;
    return up256((size_t)((cap + 1023) / 1024) * (M / 4) * sizeof(int32_t));
}

int venom_route(const uint16_t* X, const uint16_t* means, int64_t T, int64_t D, int M, int32_t* expert, int32_t* perm,
                int32_t* row_of_token, int32_t* seg, float* scores, void* workspace, size_t ws_bytes, void* stream) {
    REQUIRE(X && means && expert && perm && row_of_token && seg, SFFN_EINVAL, "venom_route: null pointer");
    REQUIRE(vnm_ok(64, M), SFFN_EUNSUPPORTED, "venom_route: M must be 8, 16, 32 or 64 (M / 4 experts)");
    REQUIRE(T > 0 && D > 0 && D % 8 == 0, SFFN_EINVAL, "venom_route: T must be positive and D a positive multiple of 8");
    REQUIRE(fits_int(T) && fits_int(D) && T < 65536 * 64, SFFN_EUNSUPPORTED, "venom_route: dimension too large");
    REQUIRE(aligned16(X) && aligned16(means) && aligned16(expert) && aligned16(perm) && aligned16(row_of_token) && aligned16(seg) &&
                aligned16(scores) && aligned16(workspace), SFFN_EINVAL, "venom_route: pointers must be 16-byte aligned");
    REQUIRE(workspace && ws_bytes >= sffn_venom_route_workspace_bytes(T, M), SFFN_EWORKSPACE, "venom_route: workspace missing or too small");
    hipStream_t s = (hipStream_t)stream;
    const int E = M / 4;
    LAUNCH(launch_venom_route(X, means, T, D, E, expert, scores, s), "venom_route/scores");
    LAUNCH(launch_venom_permute(expert, T, E, sffn_venom_rows(T, M), (int32_t*)workspace, seg, perm, row_of_token, s), "venom_route/permute");
    return SFFN_OK;
}

size_t sffn_venom_matmul_workspace_bytes(int64_t T, int64_t D, int64_t F, int M) {
    const int64_t cap = sffn_venom_rows(T, M);
    if (cap == 0 || !mult64(D) || !mult64(F) || (4 * F / M) % 64 != 0) return 0;
    // permuted X (blocked) + the expert-major packed W1: canonical and blocked copies
    return up256((size_t)cap * D * 2) + 2 * (up256((size_t)F * D) + up256((size_t)F * D / 8));
}

int venom_expert_matmul(const sffn_cfg* cfg, const int64_t* seg_offsets, const uint16_t* X, const int32_t* perm, const uint16_t* W1,
                        const float* b1, uint16_t* y1c, uint16_t* vals, uint8_t* meta, uint8_t* colidx, void* workspace, size_t ws_bytes,
                        void* stream) {
    REQUIRE(cfg && seg_offsets && X && perm && W1 && vals && meta && colidx, SFFN_EINVAL, "venom_expert_matmul: null pointer");
    REQUIRE(vnm_ok(cfg->V, cfg->M), SFFN_EUNSUPPORTED, "venom_expert_matmul: only V=64 with M in {8, 16, 32, 64} is built");
    const int64_t T = cfg->T, D = cfg->D, F = cfg->F;
    const int M = cfg->M, E = M / 4;
    REQUIRE(T > 0 && mult64(D) && mult64(F), SFFN_EINVAL, "venom_expert_matmul: T must be positive, D and F positive multiples of 64");
    const int64_t Kc = 4 * F / M, cap = sffn_venom_rows(T, M);
    REQUIRE(Kc % 64 == 0, SFFN_EINVAL, "venom_expert_matmul: 4 F / M (hidden units per expert) must be a multiple of 64");
    REQUIRE(cfg->mode == SFFN_MODE_HARD || cfg->mode == SFFN_MODE_SOFT, SFFN_EINVAL, "venom_expert_matmul: unknown mode");
    REQUIRE(cap < 65536 * 64 && fits_int(F) && fits_int(D) && fits_int(cap * (D / 8)), SFFN_EUNSUPPORTED, "venom_expert_matmul: dimension too large");
    REQUIRE(aligned16(X) && aligned16(perm) && aligned16(W1) && aligned16(b1) && aligned16(y1c) && aligned16(vals) && aligned16(meta) &&
                aligned16(colidx) && aligned16(workspace), SFFN_EINVAL, "venom_expert_matmul: pointers must be 16-byte aligned");
    REQUIRE(workspace && ws_bytes >= sffn_venom_matmul_workspace_bytes(T, D, F, M), SFFN_EWORKSPACE,
            "venom_expert_matmul: workspace missing or too small");
    GemmGroup g;
    g.n = E; g.role = 1;
    REQUIRE(seg_offsets[0] == 0 && seg_offsets[E] <= cap, SFFN_EINVAL, "venom_expert_matmul: seg_offsets must start at 0 and end within the row capacity");
    for (int e = 0; e < E; ++e)
        REQUIRE(seg_offsets[e + 1] >= seg_offsets[e] && seg_offsets[e + 1] % 64 == 0, SFFN_EINVAL,
                "venom_expert_matmul: seg_offsets must be ascending multiples of 64");
    for (int e = 0; e <= E; ++e) g.seg[e] = (int32_t)seg_offsets[e];
    g.a_stride = Kc * D / 2; g.m_stride = Kc * D / 8; g.bias_stride = 4;

    hipStream_t s = (hipStream_t)stream;
    unsigned char* ws = (unsigned char*)workspace;
    uint16_t* xb = (uint16_t*)ws;                      ws += up256((size_t)cap * D * 2);
    uint16_t* wv = (uint16_t*)ws;                      ws += up256((size_t)F * D);
    uint8_t* wm = ws;                                  ws += up256((size_t)F * D / 8);
    uint16_t* wvb = (uint16_t*)ws;                     ws += up256((size_t)F * D);
    uint8_t* wmb = ws;
    LAUNCH(launch_venom_gather_x(X, perm, cap, D, xb, s), "venom_expert_matmul/gather(X)");
    LAUNCH(launch_prune24_step(W1, F, D, D, 0, cfg->mode, wv, wm, wvb, wmb, nullptr, s, 1, M), "venom_expert_matmul/prune24(W1)");
    LAUNCH(launch_venom_colidx(g, cap, F / M, colidx, s), "venom_expert_matmul/colidx");
    // rows past the last run are never touched by the grouped contraction: clear them (they are padding)
    if (seg_offsets[E] < cap) {
        TailFill tf;
        tf.add(vals, Kc, 0); tf.add(meta, Kc / 8, 0x44);
        if (y1c) tf.add(y1c, Kc * 2, 0);
        LAUNCH(launch_fill_tail_rows(tf, nullptr, seg_offsets[E], cap, cap - seg_offsets[E], s), "venom_expert_matmul/clear");
    }
    VnmEpilogue ep;
    ep.mode = 3; ep.store_dense = y1c ? 1 : 0; ep.vals = vals; ep.meta = meta; ep.perm = perm;
    ep.logM = M == 8 ? 3 : M == 16 ? 4 : M == 32 ? 5 : 6;
    LAUNCH(launch_gemm_vnm_epilogue(wvb, wmb, xb, b1, Kc, cap, D, y1c, ep, s, &g), "venom_expert_matmul/gemm");
    return SFFN_OK;
}

namespace {
struct RouterLayout {
    sffn_router_layout pub;
    size_t xpt, xb, dypt, dyb, w1cv, w1cm, w1cvb, w1cmb, w2t, w2cv, w2cm, w2cvb, w2cmb, at, avb, amb, w2e, w1et, total;
};
bool make_router_layout(const sffn_cfg* c, RouterLayout* L) {
    if (!c || c->T <= 0 || !mult64(c->D) || !mult64(c->F) || !vnm_ok(c->V, c->M)) return false;
    const size_t D = c->D, F = c->F, M = c->M, rows = (size_t)sffn_venom_rows(c->T, c->M), Kc = 4 * F / M;
    if (Kc % 64 != 0) return false;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += up256(bytes); return o; };
    L->pub.y1c = take(rows * Kc * 2);      L->pub.vals = take(rows * Kc);          L->pub.meta = take(rows * Kc / 8);
    L->pub.colidx = take(rows / 64 * (F / M) * 4);
    L->pub.dy2c = take(rows * Kc * 2);     L->pub.dvals = take(rows * Kc);
    L->xpt = take(rows * D * 2);  L->xb = take(rows * D * 2);
    L->dypt = take(rows * D * 2); L->dyb = take(rows * D * 2);
    L->w1cv = take(F * D); L->w1cm = take(F * D / 8); L->w1cvb = take(F * D); L->w1cmb = take(F * D / 8);
    L->w2t = take(F * D * 2);
    L->w2cv = take(F * D); L->w2cm = take(F * D / 8); L->w2cvb = take(F * D); L->w2cmb = take(F * D / 8);
    L->at = take(rows * Kc * 2);
    L->avb = take(rows * Kc); L->amb = take(rows * Kc / 8);     // packed activation (y2, then dy1) in the blocked operand layout
    L->w2e = take(F * D * 2);                                    // per expert: its slice of W2 as [D, Kc], blocked (eq. (3))
    L->w1et = take(F * D * 2);                                   // per expert: its slice of W1.T as [D, Kc], blocked (eq. (7))
    L->total = off; L->pub.total = off;
    return true;
}
}  // namespace

size_t sffn_router_workspace_bytes(const sffn_cfg* cfg) {
    RouterLayout L;
    return make_router_layout(cfg, &L) ? L.total : 0;
}

int sffn_router_workspace_layout(const sffn_cfg* cfg, sffn_router_layout* out) {
    RouterLayout L;
    REQUIRE(out, SFFN_EINVAL, "sffn_router_workspace_layout: null pointer");
    REQUIRE(make_router_layout(cfg, &L), SFFN_EINVAL, "sffn_router_workspace_layout: T > 0, D and F multiples of 64, M in {8,16,32,64}, 4F/M a multiple of 64");
    *out = L.pub;
    return SFFN_OK;
}

// The router's training step.  The run offsets come either as a host array (validated here, passed to the kernels by value)
// or as a device array written earlier on the same stream by this library's own grouping kernels (seg_dev).
static int run_router_step(const sffn_cfg* cfg, const int64_t* seg_offsets, const int32_t* seg_dev, const int32_t* perm, const uint16_t* X,
                           const uint16_t* W1, const uint16_t* W2, const float* b1, const uint16_t* dY, uint16_t* Y3, uint16_t* dX,
                           uint16_t* dW1, uint16_t* dW2, void* workspace, size_t ws_bytes, void* stream, bool check_only = false, int phase = 3) {
    // phase: bit 0 = Alg. 1 with Alg. 3 as the sparsifier (forward pass), bit 1 = Alg. 2 (backward pass); the halves of a split call meet in the workspace
    const bool fwd = (phase & 1) != 0, bwd = (phase & 2) != 0;
    REQUIRE(cfg && (seg_offsets || seg_dev) && perm && (!fwd || (X && W1 && W2 && Y3)) && (!bwd || (dY && dX && dW1 && dW2)), SFFN_EINVAL,
            "ffn_router_step: null pointer");
    REQUIRE(vnm_ok(cfg->V, cfg->M), SFFN_EUNSUPPORTED, "ffn_router_step: only V=64 with M in {8, 16, 32, 64} is built");
    RouterLayout L;
    REQUIRE(make_router_layout(cfg, &L), SFFN_EINVAL, "ffn_router_step: T > 0, D and F positive multiples of 64, 4F/M a multiple of 64");
    REQUIRE(cfg->mode == SFFN_MODE_HARD || cfg->mode == SFFN_MODE_SOFT, SFFN_EINVAL, "ffn_router_step: unknown mode");
    REQUIRE(!(cfg->flags & SFFN_FLAG_DW_FP32_ACCUMULATE), SFFN_EUNSUPPORTED, "ffn_router_step: SFFN_FLAG_DW_FP32_ACCUMULATE is not built for the router's step");
    const int64_t T = cfg->T, D = cfg->D, F = cfg->F;
    const int M = cfg->M, E = M / 4;
    const int64_t Kc = 4 * F / M, rows = sffn_venom_rows(T, M);
    REQUIRE(rows < 65536 * 64 && fits_int(F) && fits_int(D) && fits_int(rows * (D / 8)) && fits_int(rows * (Kc / 8)), SFFN_EUNSUPPORTED,
            "ffn_router_step: dimension too large");
    REQUIRE(aligned16(perm) && aligned16(X) && aligned16(W1) && aligned16(W2) && aligned16(b1) && aligned16(dY) &&
                aligned16(Y3) && aligned16(dX) && aligned16(dW1) && aligned16(dW2) && aligned16(workspace), SFFN_EINVAL,
            "ffn_router_step: pointers must be 16-byte aligned");
    REQUIRE(workspace && ws_bytes >= L.total, SFFN_EWORKSPACE, "ffn_router_step: workspace missing or too small");
    GemmGroup g1;                                       // experts = weight operands, token runs = segments along j
    g1.n = E; g1.role = 1;
    if (seg_dev) {
        g1.seg_dev = seg_dev; g1.cap_rows = rows;
    } else {
        REQUIRE(seg_offsets[0] == 0 && seg_offsets[E] <= rows, SFFN_EINVAL, "ffn_router_step: seg_offsets must start at 0 and end within the row capacity");
        for (int e = 0; e < E; ++e)
            REQUIRE(seg_offsets[e + 1] >= seg_offsets[e] && seg_offsets[e + 1] % 64 == 0, SFFN_EINVAL, "ffn_router_step: seg_offsets must be ascending multiples of 64");
        for (int e = 0; e <= E; ++e) g1.seg[e] = (int32_t)seg_offsets[e];
    }
    g1.a_stride = Kc * D / 2; g1.m_stride = Kc * D / 8; g1.bias_stride = 4;
    GemmGroup g0 = g1;                                  // eqs. (3), (7): token runs along i, the expert's [D, Kc] weight slice as B
    g0.role = 0; g0.a_stride = g0.m_stride = g0.bias_stride = 0; g0.b_stride = D * Kc;
    g0.out_row_map = perm;                              // results go straight to token order; padding rows are not stored
    GemmGroup g2 = g1;                                  // weight gradients: every expert contracts over its own run
    g2.role = 2; g2.a_stride = g2.m_stride = g2.bias_stride = 0; g2.out_stride = 0;
    const int logM = M == 8 ? 3 : M == 16 ? 4 : M == 32 ? 5 : 6;
    g2.map_logM = logM;
    const int64_t used = seg_dev ? 0 : seg_offsets[E];   // (device table: the end of the last run is only known on the device)
    if (check_only) return SFFN_OK;                      // every argument check is above this line, every launch below it

    hipStream_t s = (hipStream_t)stream;
    unsigned char* ws = (unsigned char*)workspace;
    uint16_t* y1c = (uint16_t*)(ws + L.pub.y1c);   uint16_t* vals = (uint16_t*)(ws + L.pub.vals);   uint8_t* meta = ws + L.pub.meta;
    uint8_t* colidx = ws + L.pub.colidx;           uint16_t* dy2c = (uint16_t*)(ws + L.pub.dy2c);   uint16_t* dvals = (uint16_t*)(ws + L.pub.dvals);
    uint16_t* xpt = (uint16_t*)(ws + L.xpt);   uint16_t* xb = (uint16_t*)(ws + L.xb);
    uint16_t* dypt = (uint16_t*)(ws + L.dypt); uint16_t* dyb = (uint16_t*)(ws + L.dyb);
    uint16_t* w1cv = (uint16_t*)(ws + L.w1cv); uint8_t* w1cm = ws + L.w1cm; uint16_t* w1cvb = (uint16_t*)(ws + L.w1cvb); uint8_t* w1cmb = ws + L.w1cmb;
    uint16_t* w2t = (uint16_t*)(ws + L.w2t);
    uint16_t* w2cv = (uint16_t*)(ws + L.w2cv); uint8_t* w2cm = ws + L.w2cm; uint16_t* w2cvb = (uint16_t*)(ws + L.w2cvb); uint8_t* w2cmb = ws + L.w2cmb;
    uint16_t* at = (uint16_t*)(ws + L.at);
    uint16_t* avb = (uint16_t*)(ws + L.avb); uint8_t* amb = ws + L.amb;
    uint16_t* w2e = (uint16_t*)(ws + L.w2e); uint16_t* w1et = (uint16_t*)(ws + L.w1et);
    uint16_t* dw2t = w2t;                               // eq. (5)'s transposed result: W2.T is only needed while the weights are prepared
    // SFFN_FLAG_WEIGHTS_PACKED: the five weight-preparation launches (all in the forward half) are skipped; the workspace still holds
    // what they wrote for the previous call (Section 3.4: weights are converted once per optimizer step)
    const bool packed = (cfg->flags & SFFN_FLAG_WEIGHTS_PACKED) != 0;

    if (g_prof_on) { g_prof_n = 0; (void)hipEventRecord(g_prof_ev[0], s); }
    // ---- Alg. 1 with Alg. 3 as the sparsifier ---------------------------------------------------------------------
    if (fwd) STAGE(launch_transpose(X, rows, D, D, xpt, 0, xb, s, 1, 0, perm), "router/X[perm].T");     // permuted rows: transposed (eq. (8)) and blocked (eq. (1))
    if (fwd && !packed) STAGE(launch_prune24_step(W1, F, D, D, 0, cfg->mode, w1cv, w1cm, w1cvb, w1cmb, nullptr, s, 1, M), "router/prune24(W1)");
    if (fwd) STAGE(launch_venom_colidx(g1, rows, F / M, colidx, s), "router/colidx");
    if (fwd) {   // rows past the last run are padding that no contraction writes: one launch clears them in the five row-indexed outputs
        TailFill tf;
        tf.add(vals, Kc, 0); tf.add(meta, Kc / 8, 0x44); tf.add(y1c, Kc * 2, 0); tf.add(dy2c, Kc * 2, 0); tf.add(dvals, Kc, 0);
        if (seg_dev) LAUNCH(launch_fill_tail_rows(tf, seg_dev + E, 0, rows, 64 * (E + 1), s), "router/clear");      // at most 64 (E + 1) such rows
        else if (used < rows) LAUNCH(launch_fill_tail_rows(tf, nullptr, used, rows, rows - used, s), "router/clear");
    }
    // Inside a run every 64-row block keeps the same columns, so eqs. (3), (7) are plain grouped 2:4 contractions of the
    // packed [rows, Kc] activation with the expert's own [D, Kc] slice of W2 / W1.T (256 x 256 tiles; gathering rows per
    // 64-row block would re-read the same lines from every CU at once)
    if (fwd) {
        VnmEpilogue ep;
        ep.mode = 3; ep.store_dense = 1; ep.vals = vals; ep.meta = meta; ep.perm = perm; ep.logM = logM; ep.v24 = avb; ep.m24 = amb;
        STAGE(launch_gemm_vnm_epilogue(w1cvb, w1cmb, xb, b1, Kc, rows, D, y1c, ep, s, &g1), "router/y1c+sqrelu+2:4");    // eqs. (1), (2), Section 2.3
    }
    if (fwd && !packed) {       // the rest of the weight preparation, Alg. 2 line 2 included: the backward half prepares nothing
        STAGE(launch_transpose(W2, D, F, F, w2t, 0, nullptr, s), "router/W2.T");
        STAGE(launch_transpose(w2t, Kc, D, D, w2e, 1, nullptr, s, E, M), "router/W2[:,e]");
        STAGE(launch_prune24_step(w2t, F, D, D, 0, cfg->mode, w2cv, w2cm, w2cvb, w2cmb, nullptr, s, 1, M), "router/prune24(W2.T)");
        STAGE(launch_transpose(W1, Kc, D, D, w1et, 1, nullptr, s, E, M), "router/W1[e].T");
    }
    if (fwd) STAGE(launch_spmm_blocked(avb, amb, w2e, nullptr, rows, D, Kc, 0, Y3, D, s, &g0), "router/y3");                       // eq. (3)
    // ---- Alg. 2 ------------------------------------------------------------------------------------------------------
    if (bwd) STAGE(launch_transpose(dY, rows, D, D, dypt, 0, dyb, s, 1, 0, perm), "router/dY[perm].T");
    if (bwd) STAGE(launch_venom_expand_t_compact(vals, meta, rows, Kc, at, s), "router/expand(y2)");
    // eq. (5) is computed as dW2.T [F, D] (whole 2 D-byte rows per hidden unit) and transposed: writing dW2 [D, F] directly
    // would scatter 8-byte pieces M hidden units apart
    if (bwd) STAGE(launch_gemm_nt(0, at, nullptr, dypt, nullptr, Kc, D, rows, 0, dw2t, D, s, &g2), "router/dW2.T");                 // eq. (5)
    if (bwd) STAGE(launch_transpose(dw2t, F, D, D, dW2, 0, nullptr, s), "router/dW2");
    if (bwd) {   // eq. (4) at the expert's hidden units, then eq. (6) on y2's slots while the tile is in LDS; dy2c itself only on request
        GemmGroup g4 = g1;
        g4.bias_stride = 0;
        VnmEpilogue ep;
        ep.mode = 4; ep.store_dense = (cfg->flags & SFFN_FLAG_KEEP_DENSE) ? 1 : 0; ep.vals = dvals; ep.meta = meta; ep.ykept = y1c; ep.v24 = avb;
        STAGE(launch_gemm_vnm_epilogue(w2cvb, w2cmb, dyb, nullptr, Kc, rows, D, dy2c, ep, s, &g4), "router/dy2c+dsqrelu");
    }
    if (bwd) STAGE(launch_spmm_blocked(avb, amb, w1et, nullptr, rows, D, Kc, 0, dX, D, s, &g0), "router/dX");                       // eq. (7)
    if (bwd) STAGE(launch_venom_expand_t_compact(dvals, meta, rows, Kc, at, s), "router/expand(dy1)");
    if (bwd) STAGE(launch_gemm_nt(0, at, nullptr, xpt, nullptr, Kc, D, rows, 0, dW1, D, s, &g2), "router/dW1");                    // eq. (8)
    return SFFN_OK;
}

int ffn_router_step(const sffn_cfg* cfg, const int64_t* seg_offsets, const int32_t* perm, const uint16_t* X,
                    const uint16_t* W1, const uint16_t* W2, const float* b1, const uint16_t* dY, uint16_t* Y3, uint16_t* dX, uint16_t* dW1,
                    uint16_t* dW2, void* workspace, size_t ws_bytes, void* stream) {
    REQUIRE(seg_offsets, SFFN_EINVAL, "ffn_router_step: null pointer");
    return run_router_step(cfg, seg_offsets, nullptr, perm, X, W1, W2, b1, dY, Y3, dX, dW1, dW2, workspace, ws_bytes, stream);
}

// Alg. 1 (with Alg. 3 as the sparsifier) and Alg. 2 of the router's step as separate calls on one workspace
int ffn_router_forward(const sffn_cfg* cfg, const int64_t* seg_offsets, const int32_t* perm, const uint16_t* X, const uint16_t* W1,
                       const uint16_t* W2, const float* b1, uint16_t* Y3, void* workspace, size_t ws_bytes, void* stream) {
    REQUIRE(seg_offsets, SFFN_EINVAL, "ffn_router_forward: null pointer");
    return run_router_step(cfg, seg_offsets, nullptr, perm, X, W1, W2, b1, nullptr, Y3, nullptr, nullptr, nullptr, workspace, ws_bytes, stream, false, 1);
}
int ffn_router_backward(const sffn_cfg* cfg, const int64_t* seg_offsets, const int32_t* perm, const uint16_t* dY, uint16_t* dX, uint16_t* dW1,
                        uint16_t* dW2, void* workspace, size_t ws_bytes, void* stream) {
    REQUIRE(seg_offsets, SFFN_EINVAL, "ffn_router_backward: null pointer");
    return run_router_step(cfg, seg_offsets, nullptr, perm, nullptr, nullptr, nullptr, nullptr, dY, nullptr, dX, dW1, dW2, workspace, ws_bytes, stream, false, 2);
}

// Routing buffers of ffn_router_full_step, behind the step's own workspace: expert [T], perm [rows], row_of_token [T],
// seg [E + 1], per-block counts.
namespace {
struct RouteArea { size_t expert, perm, row_of_token, seg, counts, total; };
bool make_route_area(const sffn_cfg* c, size_t base, RouteArea* A) {
    if (!c || c->T <= 0 || !vnm_ok(c->V, c->M)) return false;
    const size_t T = c->T, rows = (size_t)sffn_venom_rows(c->T, c->M);
    size_t off = base;
    auto take = [&](size_t bytes) { size_t o = off; off += up256(bytes); return o; };
    A->expert = take(T * 4); A->perm = take(rows * 4); A->row_of_token = take(T * 4); A->seg = take(68 * 4);
    A->counts = take(sffn_venom_route_workspace_bytes(c->T, c->M));
    A->total = off;
    return true;
}
}  // namespace

size_t sffn_router_full_workspace_bytes(const sffn_cfg* cfg) {
    RouterLayout L;
    RouteArea A;
    if (!make_router_layout(cfg, &L) || !make_route_area(cfg, L.total, &A)) return 0;
    return A.total;
}

namespace {
int run_router_full(const sffn_cfg* cfg, const uint16_t* means, const uint16_t* X, const uint16_t* W1, const uint16_t* W2,
                    const float* b1, const uint16_t* dY, uint16_t* Y3, uint16_t* dX, uint16_t* dW1, uint16_t* dW2, void* workspace,
                    size_t ws_bytes, void* stream, int phase) {
    REQUIRE(cfg && (!(phase & 1) || (means && X)) && workspace, SFFN_EINVAL, "ffn_router_full_step: null pointer");
    REQUIRE(vnm_ok(cfg->V, cfg->M), SFFN_EUNSUPPORTED, "ffn_router_full_step: only V=64 with M in {8, 16, 32, 64} is built");
    RouterLayout L;
    RouteArea A;
    REQUIRE(make_router_layout(cfg, &L) && make_route_area(cfg, L.total, &A), SFFN_EINVAL,
            "ffn_router_full_step: T > 0, D and F positive multiples of 64, 4F/M a multiple of 64");
    REQUIRE(aligned16(workspace) && aligned16(means), SFFN_EINVAL, "ffn_router_full_step: pointers must be 16-byte aligned");
    REQUIRE(ws_bytes >= A.total, SFFN_EWORKSPACE, "ffn_router_full_step: workspace too small");
    unsigned char* ws = (unsigned char*)workspace;
    int32_t* expert = (int32_t*)(ws + A.expert);
    int32_t* perm = (int32_t*)(ws + A.perm);
    int32_t* seg = (int32_t*)(ws + A.seg);
    // the step's own argument checks run first, so that a rejected call leaves nothing on the stream
    const int pre = run_router_step(cfg, nullptr, seg, perm, X, W1, W2, b1, dY, Y3, dX, dW1, dW2, workspace, L.total, stream, true, phase);
    if (pre != SFFN_OK) return pre;
    if (phase & 1) {        // the backward half of a split call reads the routing its forward half left in the workspace
        const int rc = venom_route(X, means, cfg->T, cfg->D, cfg->M, expert, perm, (int32_t*)(ws + A.row_of_token), seg, nullptr, ws + A.counts,
                                   A.total - A.counts, stream);
        if (rc != SFFN_OK) return rc;
    }
    // the run offsets stay on the device: no read-back, the grouped launches are sized for the worst case
    return run_router_step(cfg, nullptr, seg, perm, X, W1, W2, b1, dY, Y3, dX, dW1, dW2, workspace, L.total, stream, false, phase);
}
}  // namespace

int ffn_router_full_step(const sffn_cfg* cfg, const uint16_t* means, const uint16_t* X, const uint16_t* W1, const uint16_t* W2,
                         const float* b1, const uint16_t* dY, uint16_t* Y3, uint16_t* dX, uint16_t* dW1, uint16_t* dW2, void* workspace,
                         size_t ws_bytes, void* stream) {
    return run_router_full(cfg, means, X, W1, W2, b1, dY, Y3, dX, dW1, dW2, workspace, ws_bytes, stream, 3);
}
int ffn_router_full_forward(const sffn_cfg* cfg, const uint16_t* means, const uint16_t* X, const uint16_t* W1, const uint16_t* W2,
                            const float* b1, uint16_t* Y3, void* workspace, size_t ws_bytes, void* stream) {
    return run_router_full(cfg, means, X, W1, W2, b1, nullptr, Y3, nullptr, nullptr, nullptr, workspace, ws_bytes, stream, 1);
}
int ffn_router_full_backward(const sffn_cfg* cfg, const uint16_t* dY, uint16_t* dX, uint16_t* dW1, uint16_t* dW2, void* workspace, size_t ws_bytes,
                             void* stream) {
    return run_router_full(cfg, nullptr, nullptr, nullptr, nullptr, nullptr, dY, nullptr, dX, dW1, dW2, workspace, ws_bytes, stream, 2);
}

// Alg. 1 + Alg. 2 for n_experts independent FFNs over consecutive token segments (n_experts = 1, seg = nullptr:
// the plain step).  Every stage is one launch; the GEMMs find their expert from the segment table.
static int run_step(const sffn_cfg* cfg, int n_experts, const int64_t* seg, const uint16_t* X, const uint16_t* W1,
                    const uint16_t* W2, const float* b1, const uint16_t* dY, uint16_t* Y3, uint16_t* dX, uint16_t* dW1,
                    uint16_t* dW2, void* workspace, size_t ws_bytes, void* stream, int phase = 3, const sffn_buffers* buf = nullptr) {
    // phase: bit 0 = Alg. 1 (forward pass), bit 1 = Alg. 2 (backward pass); the two halves of a split call meet through the workspace
    const bool fwd = (phase & 1) != 0, bwd = (phase & 2) != 0;
    REQUIRE(cfg && W1 && (!fwd || (X && W2 && Y3)) && (!bwd || (dY && dX && dW1 && dW2)), SFFN_EINVAL, "ffn_sparse_step: null pointer");
    FullLayout L;
    REQUIRE(n_experts >= 1 && n_experts <= GemmGroup::kMaxExperts, SFFN_EINVAL, "ffn_sparse_step_grouped: n_experts must be in 1..64");
    REQUIRE(vnm_ok(cfg->V, cfg->M), SFFN_EUNSUPPORTED, "ffn_sparse_step: only V=64 with M in {8, 16, 32, 64} is built");
    REQUIRE(make_layout(cfg, &L, n_experts), SFFN_EINVAL, "ffn_sparse_step: T, D, F must be positive multiples of 64 and F a multiple of 2 M");
    REQUIRE(cfg->M == 8 || fused_wide(cfg) || (seg == nullptr && n_experts == 1), SFFN_EUNSUPPORTED,
            "ffn_sparse_step_grouped: blocks of 16 / 32 / 64 columns need 4 F / M to be a multiple of 64 and at most 7168 (and no SFFN_FLAG_UNFUSED)");
    REQUIRE(cfg->mode == SFFN_MODE_HARD || cfg->mode == SFFN_MODE_SOFT, SFFN_EINVAL, "ffn_sparse_step: unknown mode");
    REQUIRE(!(cfg->flags & ~(SFFN_FLAG_KEEP_DENSE | SFFN_FLAG_UNFUSED | SFFN_FLAG_FP8_WGRAD | SFFN_FLAG_LEAN | SFFN_FLAG_WEIGHTS_PACKED | SFFN_FLAG_DW_FP32_ACCUMULATE)), SFFN_EINVAL,
            "ffn_sparse_step: unknown flag");
    REQUIRE(aligned16(X) && aligned16(W1) && aligned16(W2) && aligned16(b1) && aligned16(dY) && aligned16(Y3) && aligned16(dX) &&
                aligned16(dW1) && aligned16(dW2) && aligned16(workspace),
            SFFN_EINVAL, "ffn_sparse_step: pointers must be 16-byte aligned");
    REQUIRE(cfg->T < 65536 && fits_int(cfg->F * n_experts) && fits_int(cfg->D), SFFN_EUNSUPPORTED,
            "ffn_sparse_step: T must be below 65536 and F * n_experts below 2^31");
    const int64_t T = cfg->T, D = cfg->D, F = cfg->F, E = n_experts;
    REQUIRE(cfg->M != 8 || F * D * 2 < ((int64_t)1 << 31), SFFN_EUNSUPPORTED, "ffn_sparse_step: a weight matrix must stay below 2 GiB");
    Regions rg;
    {
        const int rc = place_regions(buf, workspace, ws_bytes, L.scratch_end, L.saved_end, L.total, &rg);
        REQUIRE(rc != SFFN_EINVAL, SFFN_EINVAL, "ffn_sparse_forward / ffn_sparse_backward: the three buffers must be 256-byte aligned and must not overlap");
        REQUIRE(rc == SFFN_OK, SFFN_EWORKSPACE, "ffn_sparse_step: workspace missing or too small");
    }
    GemmGroup g;                                    // g.n = 0: plain step
    if (seg) {
        REQUIRE(seg[0] == 0 && seg[E] == T, SFFN_EINVAL, "ffn_sparse_step_grouped: seg_offsets must start at 0 and end at T");
        for (int e = 0; e < E; ++e)
            REQUIRE(seg[e + 1] >= seg[e] && seg[e + 1] % 64 == 0, SFFN_EINVAL,
                    "ffn_sparse_step_grouped: seg_offsets must be ascending multiples of 64");
        g.n = (int)E;
        for (int e = 0; e <= E; ++e) g.seg[e] = (int32_t)seg[e];
    }

    hipStream_t s = (hipStream_t)stream;
    uint16_t* w1v = (uint16_t*)(rg.at(L.pub.w1_vals));    uint8_t* w1m = rg.at(L.pub.w1_meta);
    uint16_t* w2v = (uint16_t*)(rg.at(L.pub.w2t_vals));   uint8_t* w2m = rg.at(L.pub.w2t_meta);
    uint16_t* y1 = (uint16_t*)(rg.at(L.pub.y1));
    uint16_t* y2v = (uint16_t*)(rg.at(L.pub.y2_vals));    uint8_t* y2m = rg.at(L.pub.y2_meta);   uint8_t* cix = rg.at(L.pub.colidx);
    uint16_t* dy2 = (uint16_t*)(rg.at(L.pub.dy2));
    uint16_t* dy1v = (uint16_t*)(rg.at(L.pub.dy1_vals));
    uint16_t* w1vb = (uint16_t*)(rg.at(L.w1_vblk));       uint8_t* w1mb = rg.at(L.w1_mblk);
    uint16_t* w2vb = (uint16_t*)(rg.at(L.w2t_vblk));      uint8_t* w2mb = rg.at(L.w2t_mblk);
    uint16_t* xb = (uint16_t*)(rg.at(L.x_blk));           uint16_t* xtb = (uint16_t*)(rg.at(L.xt_blk));
    uint16_t* dyb = (uint16_t*)(rg.at(L.dy_blk));         uint16_t* dytb = (uint16_t*)(rg.at(L.dyt_blk));
    uint16_t* w2b = (uint16_t*)(rg.at(L.w2_blk));         uint16_t* w1tb = (uint16_t*)(rg.at(L.w1t_blk));
    uint16_t* a24v = (uint16_t*)(rg.at(L.a24_vblk));      uint8_t* a24m = rg.at(L.a24_mblk);
    uint16_t* atb = (uint16_t*)(rg.at(L.at_blk));
    uint8_t* kmask = rg.at(L.kmask);
    uint16_t* ykept = (uint16_t*)(rg.at(L.pub.y1_kept));
    const int keep_dense = (cfg->flags & SFFN_FLAG_KEEP_DENSE) ? 1 : 0;
    // SFFN_FLAG_WEIGHTS_PACKED: the workspace still holds the packed weights (and W2.T) of the previous call: no pruning passes (Section 3.4:
    // the conversion is paid once per optimizer step, not once per micro-batch)
    const bool packed = (cfg->flags & SFFN_FLAG_WEIGHTS_PACKED) != 0;
    REQUIRE(!packed || cfg->M == 8 || fused_wide(cfg), SFFN_EUNSUPPORTED, "ffn_sparse_step: SFFN_FLAG_WEIGHTS_PACKED is not built for the unfused path");
    // SFFN_FLAG_DW_FP32_ACCUMULATE: dW1 / dW2 are float32 accumulators that eqs. (8) / (5) add to (micro-batches of one optimizer step)
    const bool acc32 = (cfg->flags & SFFN_FLAG_DW_FP32_ACCUMULATE) != 0;
    REQUIRE(!acc32 || cfg->M == 8 || fused_wide(cfg), SFFN_EUNSUPPORTED, "ffn_sparse_step: SFFN_FLAG_DW_FP32_ACCUMULATE is not built for the unfused path");
    REQUIRE(phase == 3 || cfg->M == 8 || fused_wide(cfg), SFFN_EUNSUPPORTED, "ffn_sparse_forward / ffn_sparse_backward: not built for the unfused path");
    if (fused_wide(cfg)) {
        // Blocks of M = 16, 32, 64 columns (Table 5), fused like the M = 8 step: eq. (2) + compression in the epilogue of eq. (1), eq. (6)
        // in the epilogue of eq. (4) (the dense y1 / dy2 stay in LDS), eqs. (3), (7) on the kept rows of W2.T / W1 only (the pruning
        // pass of W2 also writes W2.T), eqs. (5), (8) on the compacted transposed activation that the epilogues write in the M = 8 format
        // (no group of 8 hidden units keeps more than 4 when a block of M >= 16 keeps 4).  10 launches.
        const int M = cfg->M, logM = M == 16 ? 4 : M == 32 ? 5 : 6;
        GemmGroup g_packed = g, g_rows = g, g_wgrad = g;
        g_packed.role = 1; g_packed.a_stride = F * D / 2; g_packed.m_stride = F * D / 8; g_packed.bias_stride = F;
        g_rows.role = 0;   g_rows.b_stride = F * D;
        g_wgrad.role = 2;  g_wgrad.out_stride = D * F;
        const GemmGroup* gp = g.n ? &g_packed : nullptr;
        const GemmGroup* gr = g.n ? &g_rows : nullptr;
        const GemmGroup* gw = g.n ? &g_wgrad : nullptr;
        uint16_t* w2t = w2b;                             // W2.T [F, D] per expert
        if (g_prof_on) { g_prof_n = 0; (void)hipEventRecord(g_prof_ev[0], s); }
        const bool lean_w = (cfg->flags & SFFN_FLAG_LEAN) != 0;        // no canonical copies of the packed weights (the packed activations stay: eqs. (3), (7) read them)
        if (fwd) STAGE(launch_transpose(X, T, D, D, xtb, 1, xb, s), "step/X.T");
        if (fwd && !packed) STAGE(launch_prune24_step(W1, E * F, D, D, 0, cfg->mode, lean_w ? nullptr : w1v, lean_w ? nullptr : w1m, w1vb, w1mb, nullptr, s), "step/prune24(W1)");
        if (fwd) {
            VnmEpilogue ep;
            ep.mode = 5; ep.logM = logM; ep.store_dense = keep_dense; ep.vals = y2v; ep.meta = y2m; ep.colidx = cix; ep.kmask = kmask; ep.ykept = ykept; ep.at = atb;
            STAGE(launch_gemm_vnm_epilogue(w1vb, w1mb, xb, b1, F, T, D, y1, ep, s, gp), "step/y1+sqrelu_vnm_compress");         // eqs. (1), (2), Section 2.3
        }
        if (fwd && !packed) STAGE(launch_prune24_step(W2, F, D, F, 1, cfg->mode, lean_w ? nullptr : w2v, lean_w ? nullptr : w2m, w2vb, w2mb, nullptr, s, (int)E, 0, w2t), "step/prune24(W2.T)");
        if (fwd) STAGE(launch_vnm_spmm_gather(y2v, y2m, cix, w2t, D, T, D, F, M, Y3, D, s, gr), "step/y3");                              // eq. (3)
        if (bwd) STAGE(launch_transpose(dY, T, D, D, dytb, 1, dyb, s), "step/dY.T");
        if (bwd) STAGE(launch_wgrad_vnm(atb, kmask, dytb, F, D, T, 1, dW2, F, s, gw, acc32), "step/dW2");                                       // eq. (5)
        if (bwd) {
            VnmEpilogue ep;
            ep.mode = 6; ep.logM = logM; ep.store_dense = keep_dense; ep.vals = dy1v; ep.meta = y2m; ep.colidx = cix; ep.ykept = ykept; ep.at = atb;
            STAGE(launch_gemm_vnm_epilogue(w2vb, w2mb, dyb, nullptr, F, T, D, dy2, ep, s, gp), "step/dy2+dsqrelu_vnm");         // eqs. (4), (6)
        }
        if (bwd) STAGE(launch_vnm_spmm_gather(dy1v, y2m, cix, W1, D, T, D, F, M, dX, D, s, gr), "step/dX");                              // eq. (7), dense W1 as is
        if (bwd) STAGE(launch_wgrad_vnm(atb, kmask, xtb, F, D, T, 0, dW1, D, s, gw, acc32), "step/dW1");                                        // eq. (8)
        return SFFN_OK;
    }
    if (cfg->M != 8) {
        // Wider blocks (Table 5): the same Alg. 1 / Alg. 2 without the fused epilogues.  Eqs. (1), (4) run on the blocked
        // operands like the M = 8 step but only store the dense y1 / dy2 (they are what the stand-alone eq. (2) / eq. (6)
        // kernels read; y1_kept is not produced); eqs. (3), (7) gather the kept rows of W2.T / W1; eqs. (5), (8) contract
        // the expanded transposed activation.
        const int M = cfg->M;
        if (g_prof_on) { g_prof_n = 0; (void)hipEventRecord(g_prof_ev[0], s); }
        uint16_t* at = atb;                              // dense [F, T]
        uint16_t* xt = xtb;                              // X.T and dY.T [D, T], row-major here
        uint16_t* dyt = dytb;
        uint16_t* w1t = w1tb;                            // W2.T (gathered route) or W1.T (plain-2:4 route), [F, D] / [D, F] row-major
        const VnmEpilogue plain;                         // eqs. (1), (4) on the blocked operands, dense output only
        STAGE(launch_transpose(X, T, D, D, xt, 0, xb, s), "step/X.T");
        STAGE(launch_prune24_step(W1, F, D, D, 0, cfg->mode, w1v, w1m, w1vb, w1mb, nullptr, s), "step/prune24(W1)");
        STAGE(launch_gemm_vnm_epilogue(w1vb, w1mb, xb, b1, F, T, D, y1, plain, s), "step/y1");                        // eq. (1)
        STAGE(launch_sqrelu_vnm_compress_m(y1, T, F, M, y2v, y2m, cix, s), "step/sqrelu_vnm_compress");               // eq. (2), Section 2.3
        // eqs. (3), (7): gather the kept rows of the dense operand (matrix work and traffic shrink with 4 / M); shapes the
        // gathered kernel does not cover re-express the activation as plain 2:4 over all F columns instead
        const bool gather = vnm_spmm_gather_ok(T, D, F, M) && F * D * 2 < ((int64_t)1 << 31);
        if (gather) {
            STAGE(launch_transpose(W2, D, F, F, w1t, 0, nullptr, s), "step/W2.T");
            STAGE(launch_vnm_spmm_gather(y2v, y2m, cix, w1t, D, T, D, F, M, Y3, D, s), "step/y3");                    // eq. (3)
        } else {
            STAGE(launch_vnm_to_24_m(y2v, y2m, cix, T, F, M, a24v, a24m, s), "step/to24(y2)");
            STAGE(launch_gemm_nt(1, a24v, a24m, W2, nullptr, T, D, F, 0, Y3, D, s), "step/y3");                       // eq. (3)
        }
        STAGE(launch_prune24_step(W2, F, D, F, 1, cfg->mode, w2v, w2m, w2vb, w2mb, nullptr, s), "step/prune24(W2.T)");
        // eq. (5) before eq. (4): the weight-gradient kernel is faster while dY.T is still in the last-level cache
        STAGE(launch_transpose(dY, T, D, D, dyt, 0, dyb, s), "step/dY.T");
        STAGE(launch_vnm_expand_t_m(y2v, y2m, cix, T, F, M, at, s), "step/expand(y2)");
        STAGE(launch_gemm_nt(0, at, nullptr, dyt, nullptr, F, D, T, 1, dW2, F, s), "step/dW2");                       // eq. (5)
        STAGE(launch_gemm_vnm_epilogue(w2vb, w2mb, dyb, nullptr, F, T, D, dy2, plain, s), "step/dy2");                // eq. (4)
        STAGE(launch_dsqrelu_vnm_m(dy2, y1, y2m, cix, T, F, M, dy1v, s), "step/dsqrelu_vnm");                         // eq. (6)
        if (gather) {
            STAGE(launch_vnm_spmm_gather(dy1v, y2m, cix, W1, D, T, D, F, M, dX, D, s), "step/dX");                    // eq. (7)
        } else {
            STAGE(launch_vnm_to_24_m(dy1v, y2m, cix, T, F, M, a24v, a24m, s), "step/to24(dy1)");
            STAGE(launch_transpose(W1, F, D, D, w1t, 0, nullptr, s), "step/W1.T");
            STAGE(launch_gemm_nt(1, a24v, a24m, w1t, nullptr, T, D, F, 0, dX, D, s), "step/dX");                      // eq. (7)
        }
        STAGE(launch_vnm_expand_t_m(dy1v, y2m, cix, T, F, M, at, s), "step/expand(dy1)");
        STAGE(launch_gemm_nt(0, at, nullptr, xt, nullptr, F, D, T, 0, dW1, D, s), "step/dW1");                        // eq. (8)
        (void)keep_dense;
        return SFFN_OK;
    }
    // the three ways a token segment meets its expert's weights (see GemmGroup)
    GemmGroup g_packed = g, g_dense = g, g_wgrad = g;
    g_packed.role = 1; g_packed.a_stride = F * D / 2; g_packed.m_stride = F * D / 8; g_packed.bias_stride = F;
    g_dense.role = 0;  g_dense.b_stride = D * F;
    g_wgrad.role = 2;  g_wgrad.out_stride = D * F;
    const GemmGroup* gp = g.n ? &g_packed : nullptr;
    const GemmGroup* gd = g.n ? &g_dense : nullptr;
    const GemmGroup* gw = g.n ? &g_wgrad : nullptr;

    if (g_prof_on) { g_prof_n = 0; (void)hipEventRecord(g_prof_ev[0], s); }
    // Every GEMM operand is first brought into the layout its kernel reads by the pass that reads or produces it anyway: X and dY
    // by the transposes the weight-gradient GEMMs need, the pruned weights by their pruning passes (W2's also writes the unpruned
    // W2.T, contraction-major, for eq. (3)), the activations by the fused epilogues of eqs. (1) and (4).  Eqs. (3), (7) contract the
    // V:2:8 activation as it is (gemm_vnm8.hip): the kept rows of W2.T / W1 are picked while the fragments are read, so W1 is used
    // in place and no 2:4 view of the activation over all F columns is written.
    // ---- Alg. 1 -------------------------------------------------------------------------------
    // SFFN_FLAG_LEAN: the canonical copies of the packed tensors (inspection aids: w1 / w2t vals + meta, y2 vals, dy1 vals) are not
    // written; every consumer inside the step reads the kernels' own copies
    const bool lean = (cfg->flags & SFFN_FLAG_LEAN) != 0;
    uint16_t* vcb = a24v;                                        // the activation's survivors / metadata / regrouped offsets for eqs. (3), (7)
    uint8_t* mcb = a24m;
    uint8_t* cixt = a24m + up256((size_t)T * F / 16);
    uint16_t* w2t = w2b;                                         // W2.T [F, D] per expert
    g_dense.b_stride = F * D;
    if (fwd) STAGE(launch_transpose(X, T, D, D, xtb, 1, xb, s), "step/X.T");
    // row pruning is per row, so the E stacked [F, D] matrices are one [E * F, D] matrix
    if (fwd && !packed) STAGE(launch_prune24_step(W1, E * F, D, D, 0, cfg->mode, lean ? nullptr : w1v, lean ? nullptr : w1m, w1vb, w1mb, nullptr, s), "step/prune24(W1)");
    if (fwd) {   // eq. (1), then eq. (2) + V:N:M compression on the tile while it is still in LDS
        VnmEpilogue ep;
        ep.mode = 1; ep.store_dense = keep_dense; ep.vals = lean ? nullptr : y2v; ep.meta = y2m; ep.colidx = cix; ep.kmask = kmask; ep.ykept = ykept;
        ep.vcb = vcb; ep.mcb = mcb; ep.cixt = cixt; ep.at = atb;
        STAGE(launch_gemm_vnm_epilogue(w1vb, w1mb, xb, b1, F, T, D, y1, ep, s, gp), "step/y1+sqrelu_vnm_compress");
    }
    if (fwd && !packed) STAGE(launch_prune24_step(W2, F, D, F, 1, cfg->mode, lean ? nullptr : w2v, lean ? nullptr : w2m, w2vb, w2mb, nullptr, s, (int)E, 0, w2t), "step/prune24(W2.T)");
    if (fwd) STAGE(launch_vnm8_gemm(vcb, mcb, cixt, w2t, D, T, D, F, Y3, D, s, gd), "step/y3");                         // eq. (3)
    // ---- Alg. 2 -------------------------------------------------------------------------------
    if (bwd) STAGE(launch_transpose(dY, T, D, D, dytb, 1, dyb, s), "step/dY.T");
    if (bwd) STAGE(launch_wgrad_vnm(atb, kmask, dytb, F, D, T, 1, dW2, F, s, gw, acc32), "step/dW2");                          // eq. (5)
    if (bwd) {   // eq. (4), then eq. (6) on y2's kept slots; overwrites the survivors and the transposed tile with dy1's
        VnmEpilogue ep;
        ep.mode = 2; ep.store_dense = keep_dense; ep.vals = lean ? nullptr : dy1v; ep.meta = y2m; ep.colidx = cix; ep.ykept = ykept;
        ep.vcb = vcb; ep.at = atb;
        STAGE(launch_gemm_vnm_epilogue(w2vb, w2mb, dyb, nullptr, F, T, D, dy2, ep, s, gp), "step/dy2+dsqrelu_vnm");
    }
    if (bwd) STAGE(launch_vnm8_gemm(vcb, mcb, cixt, W1, D, T, D, F, dX, D, s, gd), "step/dX");                          // eq. (7), dense W1 as is
    if (bwd) STAGE(launch_wgrad_vnm(atb, kmask, xtb, F, D, T, 0, dW1, D, s, gw, acc32), "step/dW1");                           // eq. (8)
    (void)w1tb;
    return SFFN_OK;
}

int ffn_sparse_step(const sffn_cfg* cfg, const uint16_t* X, const uint16_t* W1, const uint16_t* W2, const float* b1,
                    const uint16_t* dY, uint16_t* Y3, uint16_t* dX, uint16_t* dW1, uint16_t* dW2, void* workspace,
                    size_t ws_bytes, void* stream) {
    return run_step(cfg, 1, nullptr, X, W1, W2, b1, dY, Y3, dX, dW1, dW2, workspace, ws_bytes, stream);
}

// Alg. 1 / Alg. 2 as separate calls (other layers run between a layer's forward and backward pass); the halves meet through the
// `saved` and `weights` buffers
int sffn_buffer_sizes(const sffn_cfg* cfg, int n_experts, sffn_buffers* out) {
    FullLayout L;
    REQUIRE(out != nullptr, SFFN_EINVAL, "sffn_buffer_sizes: out is null");
    REQUIRE(make_layout(cfg, &L, n_experts), SFFN_EINVAL, "sffn_buffer_sizes: T, D, F must be positive multiples of 64, V = 64, M in {8, 16, 32, 64}, n_experts >= 1");
    out->scratch = out->saved = out->weights = nullptr;
    out->scratch_bytes = L.scratch_end; out->saved_bytes = L.saved_end - L.scratch_end; out->weights_bytes = L.total - L.saved_end;
    return SFFN_OK;
}
int ffn_sparse_forward(const sffn_cfg* cfg, const uint16_t* X, const uint16_t* W1, const uint16_t* W2, const float* b1, uint16_t* Y3,
                       const sffn_buffers* buf, void* stream) {
    REQUIRE(buf != nullptr, SFFN_EINVAL, "ffn_sparse_forward: buf is null");
    return run_step(cfg, 1, nullptr, X, W1, W2, b1, nullptr, Y3, nullptr, nullptr, nullptr, nullptr, 0, stream, 1, buf);
}
int ffn_sparse_backward(const sffn_cfg* cfg, const uint16_t* W1, const uint16_t* dY, uint16_t* dX, uint16_t* dW1, uint16_t* dW2,
                        const sffn_buffers* buf, void* stream) {
    REQUIRE(buf != nullptr, SFFN_EINVAL, "ffn_sparse_backward: buf is null");
    return run_step(cfg, 1, nullptr, nullptr, W1, nullptr, nullptr, dY, nullptr, dX, dW1, dW2, nullptr, 0, stream, 2, buf);
}
int ffn_sparse_forward_grouped(const sffn_cfg* cfg, int n_experts, const int64_t* seg_offsets, const uint16_t* X, const uint16_t* W1,
                               const uint16_t* W2, const float* b1, uint16_t* Y3, const sffn_buffers* buf, void* stream) {
    REQUIRE(seg_offsets != nullptr && buf != nullptr, SFFN_EINVAL, "ffn_sparse_forward_grouped: seg_offsets or buf is null");
    return run_step(cfg, n_experts, seg_offsets, X, W1, W2, b1, nullptr, Y3, nullptr, nullptr, nullptr, nullptr, 0, stream, 1, buf);
}
int ffn_sparse_backward_grouped(const sffn_cfg* cfg, int n_experts, const int64_t* seg_offsets, const uint16_t* W1, const uint16_t* dY,
                                uint16_t* dX, uint16_t* dW1, uint16_t* dW2, const sffn_buffers* buf, void* stream) {
    REQUIRE(seg_offsets != nullptr && buf != nullptr, SFFN_EINVAL, "ffn_sparse_backward_grouped: seg_offsets or buf is null");
    return run_step(cfg, n_experts, seg_offsets, nullptr, W1, nullptr, nullptr, dY, nullptr, dX, dW1, dW2, nullptr, 0, stream, 2, buf);
}

size_t sffn_grouped_workspace_bytes(const sffn_cfg* cfg, int n_experts) {
    FullLayout L;
    return make_layout(cfg, &L, n_experts) ? L.total : 0;
}

int sffn_grouped_workspace_layout(const sffn_cfg* cfg, int n_experts, sffn_ws_layout* out) {
    FullLayout L;
    REQUIRE(out != nullptr, SFFN_EINVAL, "sffn_grouped_workspace_layout: out is null");
    REQUIRE(make_layout(cfg, &L, n_experts), SFFN_EINVAL, "sffn_grouped_workspace_layout: T, D, F must be positive multiples of 64, V = 64, M in {8, 16, 32, 64}, n_experts >= 1");
    *out = L.pub;
    return SFFN_OK;
}

int ffn_sparse_step_grouped(const sffn_cfg* cfg, int n_experts, const int64_t* seg_offsets, const uint16_t* X, const uint16_t* W1,
                            const uint16_t* W2, const float* b1, const uint16_t* dY, uint16_t* Y3, uint16_t* dX, uint16_t* dW1,
                            uint16_t* dW2, void* workspace, size_t ws_bytes, void* stream) {
    REQUIRE(seg_offsets != nullptr, SFFN_EINVAL, "ffn_sparse_step_grouped: seg_offsets is null");
    return run_step(cfg, n_experts, seg_offsets, X, W1, W2, b1, dY, Y3, dX, dW1, dW2, workspace, ws_bytes, stream);
}

int sffn_profile_enable(int on) {
    if (on && !g_prof_on) {
        for (int i = 0; i <= kMaxStages; ++i)
            if (hipEventCreate(&g_prof_ev[i]) != hipSuccess) return fail(SFFN_EHIP, "%s", "sffn_profile_enable: hipEventCreate failed");
        g_prof_on = true;
    } else if (!on && g_prof_on) {
        for (int i = 0; i <= kMaxStages; ++i) (void)hipEventDestroy(g_prof_ev[i]);
        g_prof_on = false;
    }
    g_prof_n = 0;
    return SFFN_OK;
}

int sffn_profile_read(float* ms, const char** names, int max_n) {
    if (!g_prof_on || g_prof_n == 0) return 0;
    if (hipEventSynchronize(g_prof_ev[g_prof_n]) != hipSuccess) return fail(SFFN_EHIP, "%s", "sffn_profile_read: hipEventSynchronize failed");
    const int n = g_prof_n < max_n ? g_prof_n : max_n;
    for (int i = 0; i < n; ++i) {
        float t = 0.f;
        (void)hipEventElapsedTime(&t, g_prof_ev[i], g_prof_ev[i + 1]);
        if (ms) ms[i] = t;
        if (names) names[i] = g_prof_name[i];
    }
    return n;
}

}  // extern "C"
