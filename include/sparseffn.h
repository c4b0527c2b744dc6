/*
 * sparseffn.h — C ABI of the MI355X (gfx950) sparsified Transformer-FFN training step.
 *
 * Method: "To 2:4 Sparsity and Beyond" (arXiv 2602.06183), Section 3 "Proposed Design":
 * Alg. 1 (forward) and Alg. 2 (backward) over eqs. (1)-(8) of Section 2.1, with the 2:4
 * weight sparsifier of Section 2.2 and the V:N:M activation format of Section 2.3.
 *
 * Conventions common to every entry point
 *   - bf16 tensors are uint16_t bit patterns, row-major; all tensor pointers are DEVICE
 *     pointers owned by the caller.  The library never allocates, frees or synchronises:
 *     it only enqueues kernels on `stream` (a hipStream_t passed as void*; NULL = the
 *     default stream).  Outputs are fully overwritten.
 *   - Return value: SFFN_OK, or a negative code with nothing enqueued for SFFN_EINVAL /
 *     SFFN_EUNSUPPORTED / SFFN_EWORKSPACE.  sffn_last_error() gives a thread-local text.
 *   - Shape rules: T % 64 == 0, D % 64 == 0, F % 64 == 0 (R, K, N below follow the same
 *     rule); base pointers 16-byte aligned.  V must be 64; M is 8, 16, 32 or 64 (Table 5 of the paper) and the
 *     compressed axis a multiple of 2 M.
 *   - Rounding: products accumulate in fp32 on the matrix cores; every stored bf16 is one
 *     round-to-nearest-even of an fp32 value.
 *
 * Packed formats (bit-exact contract)
 *   2:4   logical S[R,K]; group g of row r is S[r,4g..4g+3]; the two entries of largest
 *         magnitude survive (rank by magnitude descending, index ascending; magnitude is the
 *         bf16 pattern with the sign cleared, compared as an integer), at positions p0 < p1.
 *         vals[r,2g] = S[r,4g+p0], vals[r,2g+1] = S[r,4g+p1]; nibble = p0 | p1<<2;
 *         meta[r,g/2] holds group 2j in bits 3:0 and group 2j+1 in bits 7:4.
 *   V:N:M (V=64, N=2; written out for M=8) block (tb,g) = rows 64tb..64tb+63, columns 8g..8g+7.  Column
 *         score = fp32 sum of |y2| over the 64 rows, added in ascending row order from +0.
 *         The four columns of largest score survive (ties to the lower column);
 *         colidx[tb,g,0..3] are their offsets in ascending order.  Per row those four
 *         entries form one 2:4 group packed as above: vals[t,2g..2g+1], meta[t,g/2].  Wider blocks (M = 16,
 *         32, 64) are the same with M columns per block: vals [T, 2F/M], meta [T, F/(2M)], colidx [T/64, F/M, 4].
 */
#ifndef SPARSEFFN_H
#define SPARSEFFN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SFFN_OK            0
#define SFFN_EINVAL       (-1)  /* null pointer, bad shape or alignment */
#define SFFN_EUNSUPPORTED (-2)  /* valid request outside what is built (V != 64, M not in {8, 16, 32, 64}, a dimension too large) */
#define SFFN_EWORKSPACE   (-3)  /* workspace pointer null or too small */
#define SFFN_EHIP         (-4)  /* a HIP launch failed; see sffn_last_error() */

#define SFFN_MODE_HARD 0        /* Section 2.2, plain magnitude mask */
#define SFFN_MODE_SOFT 1        /* Section 2.2, soft-thresholding: survivors shrink by t = |t2| */

typedef struct sffn_cfg {
    int64_t T;      /* tokens (rows of X, dY) */
    int64_t D;      /* d_model */
    int64_t F;      /* d_ffn */
    int32_t V;      /* V:N:M block height, 64 */
    int32_t M;      /* V:N:M block width: 8, 16, 32 or 64 (Table 5) */
    int32_t mode;   /* SFFN_MODE_HARD or SFFN_MODE_SOFT for both weight sparsifiers */
    int32_t flags;  /* SFFN_FLAG_* */
} sffn_cfg;

/* ffn_sparse_step fuses eq. (2) + V:N:M compression into the epilogue of eq. (1) and eq. (6) into the
 * epilogue of eq. (4), so the dense y1 and dy2 never have to reach HBM: the backward pass only needs y1 at
 * y2's kept slots (y1_kept).  With this flag the step also stores the dense y1 and dy2 (same kernels, same
 * arithmetic, two extra [T,F] writes), which is what lets a checker reproduce every stage bit for bit. */
#define SFFN_FLAG_KEEP_DENSE 1
/* Blocks of 16 / 32 / 64 columns only: run the unfused path (eqs. (2), (6) as separate kernels, the dense y1 and dy2 through
 * HBM, 15 launches).  It is what the fused path is checked against bit for bit; shapes the gathered-row kernel does not cover
 * (4 F / M not a multiple of 64 or above 7168) take it in any case. */
#define SFFN_FLAG_UNFUSED 2
#define SFFN_FLAG_FP8_WGRAD 4     /* ffn_sparse_step_fp8 only: eqs. (5), (8) on codes as well */
/* ffn_sparse_step / ffn_sparse_step_grouped: do not write the canonical copies w1_vals / w1_meta, w2t_vals / w2t_meta and, at M = 8,
 * y2_vals and dy1_vals of sffn_ws_layout (at M >= 16 eqs. (3), (7) read those two).  They are inspection aids: every consumer inside the
 * step reads its own operand layouts, and Y3, dX, dW1, dW2, y2_meta, colidx, y1_kept are the same bits with or without the flag.  Ignored
 * by the unfused path.  With the flag those regions of the workspace are empty (0 bytes): sffn_workspace_bytes() and the layouts
 * depend on it.  The fp8 steps have the same flag (w1 / w2t codes and metadata; at M = 8 y2_codes). */
#define SFFN_FLAG_LEAN 8
/* ffn_sparse_step, ffn_sparse_step_grouped, ffn_sparse_step_fp8, ffn_sparse_step_fp8_grouped, the router's steps (not the unfused
 * path: SFFN_EUNSUPPORTED there): the weights are already packed.  Section 3.4 notes that the conversion of a weight to 2:4 is paid
 * once per optimizer step and amortised over the micro-batches that pass through the layer before the weights change.  The caller
 * promises that the previous call on this workspace ran without this flag on the same cfg (apart from this flag), W1 and W2 (fp8: and
 * the same scales w1, w2), and that nothing else has written the workspace since; the step then skips Alg. 1 line 4 and Alg. 2 line 2
 * (both pruning passes, with them the W2.T copy and, fp8, the weight quantisation) and reads what that call left.  Every output is the
 * same bits as without the flag.  The library cannot check the promise.  fp8: amax[1], amax[2] (w1, w2) come back as 0. */
#define SFFN_FLAG_WEIGHTS_PACKED 16
/* Same entry points (and their backward halves): dW1 and dW2 are float32 matrices of the same shapes ([F, D] and [D, F]; grouped:
 * [n_experts, ...]) that the call ADDS to - dW32 = dW32 + (eq. (8) / eq. (5) in float32) - instead of bf16 matrices that it overwrites:
 * the gradient buffers a training loop keeps across the micro-batches of an optimizer step (the amortisation of Section 3.4 presumes
 * such micro-batches).  The pointers are passed through the uint16_t* parameters; the caller owns and zeroes the buffers.  Every
 * element is updated by exactly one thread, so the sum is deterministic.  16-byte alignment as before. */
#define SFFN_FLAG_DW_FP32_ACCUMULATE 32

/* Byte offsets, inside the workspace of ffn_sparse_step, of the tensors Alg. 2 line 1 saves
 * from the forward pass and of the other intermediates (all filled when the step returns).  The workspace is three regions laid
 * end to end, [scratch | saved | weights] (see sffn_buffers below): y1, dy2, y2_vals, dy1_vals lie in the first, y2_meta, colidx,
 * y1_kept in the second, the packed weights in the third. */
typedef struct sffn_ws_layout {
    size_t w1_vals, w1_meta;        /* sparsify24(W1):   [F, D/2] bf16, [F, D/8] u8 */
    size_t w2t_vals, w2t_meta;      /* sparsify24(W2.T): [F, D/2] bf16, [F, D/8] u8 */
    size_t y1;                      /* [T, F] bf16, eq. (1) plus bias.  Present with SFFN_FLAG_KEEP_DENSE and on the unfused path; otherwise
                                     * the region is empty (0 bytes) and the workspace is smaller by 2 * 2 T F bytes (y1 and dy2) */
    size_t y2_vals, y2_meta, colidx;/* V:N:M y2: [T, F/4] bf16, [T, F/16] u8, [T/64, F/8, 4] u8 */
    size_t dy2;                     /* [T, F] bf16, eq. (4); present under the same condition as y1 */
    size_t dy1_vals;                /* [T, F/4] bf16, eq. (6) in y2's slots */
    size_t y1_kept;                 /* T*2F/M bf16, y1 at y2's kept slots (what Alg. 2 line 1 needs of y1), stored as
                                     * [T/64][F/64][64 tokens][64/M column blocks][2]; absent (0 bytes) on the unfused path */
    size_t y1_kept_bytes;
    size_t total;                   /* bytes needed */
} sffn_ws_layout;

int         sffn_version(void);
const char* sffn_last_error(void);

/* Workspace sizes in bytes (0 on invalid arguments: a dimension that is not a positive multiple of 64, V != 64, M outside
 * {8, 16, 32, 64}, F not a multiple of 2 M).  The size depends on cfg->flags: see sffn_ws_layout.y1. */
size_t sffn_workspace_bytes(const sffn_cfg* cfg);                       /* ffn_sparse_step */
int    sffn_workspace_layout(const sffn_cfg* cfg, sffn_ws_layout* out); /* its layout */
size_t sffn_vnm_spmm_workspace_bytes(int64_t T, int64_t N, int64_t Kfull, int w_kmajor);
size_t sffn_vnm_wgrad_workspace_bytes(int64_t T, int64_t F, int64_t N);

/* Section 2.2 / Alg. 1 line 4 and Alg. 2 line 2 (sparsify24): 2:4 prune-and-pack along K.
 * Logical S[R,K]: trans=0 -> S[r,k] = src[r*ld + k]; trans=1 -> S[r,k] = src[k*ld + r]
 * (so sparsify24(W2.T) reads W2 [D,F] in place with R=F, K=D, ld=F).
 * out: vals [R,K/2] bf16, meta [R,K/8] u8.  mode SOFT: survivor a -> a -/+ t evaluated in fp32
 * then rounded to bf16, t = third-largest magnitude of the group; same metadata as HARD. */
int prune24_compress(const uint16_t* src, int64_t R, int64_t K, int64_t ld, int trans, int mode,
                     uint16_t* vals, uint8_t* meta, void* stream);

/* eq. (2) + Section 2.3 / Alg. 1 lines 5-6: y2 = bf16(max(y1,0)^2) compressed on the fly to V:N:M.
 * y1 [T,F]; out vals [T,F/4], meta [T,F/16], colidx [T/64,F/8,4]. */
int sqrelu_vnm_compress(const uint16_t* y1, int64_t T, int64_t F, int V, int M,
                        uint16_t* vals, uint8_t* meta, uint8_t* colidx, void* stream);

/* eq. (1) / Alg. 1 line 4: out[t,n] = bf16( sum_k X[t,k] * Ws[n,k] + bias[n] ), Ws packed 2:4
 * ([N,K/2], [N,K/8]); bias fp32 [N] or NULL; X [T,K]; out [T,N]. */
int spmm24_fwd(const uint16_t* X, const uint16_t* w_vals, const uint8_t* w_meta, const float* bias,
               int64_t T, int64_t N, int64_t K, uint16_t* out, void* stream);

/* eq. (4) / Alg. 2 line 2: out[t,n] = bf16( sum_k dY[t,k] * WTs[n,k] ), WTs = packed sparsify24(W2.T). */
int spmm24_dgrad(const uint16_t* dY, const uint16_t* wt_vals, const uint8_t* wt_meta,
                 int64_t T, int64_t N, int64_t K, uint16_t* out, void* stream);

/* The same two contractions on a "prepared" weight operand.  prune24_compress_prepared (rows K-contiguous) writes, next to the
 * canonical vals / meta, the packed matrix in the layout the matrix-core kernel streams fastest (opaque to the caller:
 * sffn_prepared24_bytes(R, K) bytes holding 1 KB blocks of 16 rows x 32 values and 256-byte metadata units of 32 rows x 64 k);
 * spmm24_prepared then computes out[t,n] = bf16( sum_k X[t,k] * Ws[n,k] + bias[n] ) (bias may be NULL: eq. (4)) with the main
 * loop of the fused step, after one pass that copies X into the same block layout (workspace:
 * sffn_spmm24_prepared_workspace_bytes(T, K) = 2 T K bytes).  Same sums as spmm24_fwd (fp32 accumulation order may differ). */
size_t sffn_prepared24_bytes(int64_t R, int64_t K);
int prune24_compress_prepared(const uint16_t* src, int64_t R, int64_t K, int64_t ld, int mode, uint16_t* vals, uint8_t* meta,
                              void* prepared, void* stream);
size_t sffn_spmm24_prepared_workspace_bytes(int64_t T, int64_t K);
int spmm24_prepared(const uint16_t* X, const void* w_prepared, const float* bias, int64_t T, int64_t N, int64_t K,
                    uint16_t* out, void* workspace, size_t ws_bytes, void* stream);

/* eq. (3) / Alg. 1 line 7 (w_kmajor=0, Wd = W2 [N,Kfull]) and eq. (7) / Alg. 2 line 5
 * (w_kmajor=1, Wd = W1 [Kfull,N]): out[t,n] = bf16( sum_f Av[t,f] * W(n,f) ) with Av the V:N:M
 * matrix (a_vals [T,Kfull/4], a_meta [T,Kfull/16], a_colidx [T/64,Kfull/8,4]) and W dense.
 * ldw = row stride of Wd in elements.  workspace: sffn_vnm_spmm_workspace_bytes() (the same size
 * for both orientations: scratch for the activation in the layout the kernel of the route reads and for a
 * transposed copy of Wd).  Routes: M = 8 (Wd below 2 GiB): the packed activation as it is on 256-token tiles, the
 * kept rows of the contraction-major W picked while the fragments are read; M >= 16 with 4*Kfull/M a multiple of 64
 * and at most 7168: only the kept rows of W are fetched (gathered per 64-token block); otherwise the activation
 * is contracted as a plain 2:4 matrix over all Kfull columns.  All routes compute the same sums (fp32 accumulation
 * order differs).  T is below 2^22, and below 65536 on the plain-2:4 route (SFFN_EUNSUPPORTED beyond, nothing enqueued). */
int vnm_spmm(const uint16_t* a_vals, const uint8_t* a_meta, const uint8_t* a_colidx,
             const uint16_t* Wd, int64_t ldw, int w_kmajor, int64_t T, int64_t N, int64_t Kfull,
             int V, int M, uint16_t* out, void* workspace, size_t ws_bytes, void* stream);

/* eq. (6) / Alg. 2 line 4 on y2's mask: dvals[t,s] = bf16( 2 * dy2[t,c] * max(y1[t,c],0) ) where
 * slot s of row t sits at column c according to (meta, colidx); dvals [T,F/4]. */
int dsqrelu_vnm(const uint16_t* dy2, const uint16_t* y1, const uint8_t* meta, const uint8_t* colidx,
                int64_t T, int64_t F, int V, int M, uint16_t* dvals, void* stream);

/* eq. (5) / Alg. 2 line 3 (out_f_major=0: out [N,F] = dW2) and eq. (8) / Alg. 2 line 6
 * (out_f_major=1: out [F,N] = dW1): C[f,n] = bf16( sum_t Av[t,f] * G[t,n] ), G [T,N] dense.
 * workspace: sffn_vnm_wgrad_workspace_bytes(). */
int vnm_wgrad(const uint16_t* a_vals, const uint8_t* a_meta, const uint8_t* a_colidx,
              const uint16_t* G, int64_t T, int64_t F, int64_t N, int V, int M, int out_f_major,
              uint16_t* out, void* workspace, size_t ws_bytes, void* stream);

/* fp8 operands (Section 3.4, closing paragraph: quantisation is orthogonal to the two sparsities and can be fused into the
 * sparsification scans; Section 1: the 2:4 hardware covers bf16 and fp8).  Format: OCP E4M3, finite-only (largest finite
 * 448), one uint8 code per value.  One float32 `scale` per tensor, GIVEN by the caller (delayed scaling): a real x becomes
 * code = E4M3_RNE(clamp(float32(x) * (1.0f / scale), -448, 448)); real ~ decode(code) * scale.  `amax` (optional device
 * float, zeroed by the caller) receives, by atomic max, the largest magnitude that was quantised: the next step's scale is
 * amax / 448.  Selection looks at the bf16 magnitudes BEFORE quantisation, so metadata and column indices are bit-identical
 * to the bf16 entry points; only the stored survivors change (in SOFT mode the float32 a -/+ t goes straight to fp8).
 *   quantize_fp8            the dense operand of eqs. (1), (3), (4), (7): n bf16 values -> n codes (n a multiple of 8)
 *   prune24_compress_fp8    Section 2.2 + quantisation: arguments of prune24_compress; codes [R, K/2] u8, meta [R, K/8]
 *   sqrelu_vnm_compress_fp8 eq. (2) + Section 2.3 + quantisation: arguments of sqrelu_vnm_compress; codes [T, 2F/M] u8
 *   spmm24_fp8              eqs. (1), (4): out[t,n] = bf16( (sum_k dec(Xq[t,k]) dec(Ws[n,k])) * (scale_x*scale_w) + bias[n] ) on the
 *                           fp8 structured-sparse matrix cores; Xq [T, K] codes, Ws packed ([N, K/2], [N, K/8]); K a multiple of 128
 *   vnm_spmm_fp8            eqs. (3), (7): the V:N:M code matrix (a_codes [T, 2 Kfull/M]) times dense W codes, [N, Kfull]
 *                           (w_kmajor = 0) or [Kfull, N] (1, contiguous rows); Kfull a multiple of 128, T below 65536;
 *                           workspace: sffn_vnm_spmm_fp8_workspace_bytes().  M = 8 runs on the 256-token tile kernel of the fp8
 *                           step after a small regrouping pass (w_kmajor = 1 then needs no transpose), M >= 16 with 4 Kfull / M a
 *                           multiple of 128 gathers the kept rows of W (the wide-block fp8 step's kernel), anything else goes as
 *                           plain 2:4 over all Kfull columns
 * The weight gradients (eqs. (5), (8), contraction over tokens) have no stand-alone fp8 entry point; ffn_sparse_step_fp8 below is the
 * whole step and can run them on the codes (SFFN_FLAG_FP8_WGRAD). */
int quantize_fp8(const uint16_t* src, int64_t n, float scale, uint8_t* codes, float* amax, void* stream);
int prune24_compress_fp8(const uint16_t* src, int64_t R, int64_t K, int64_t ld, int trans, int mode, float scale,
                         uint8_t* codes, uint8_t* meta, float* amax, void* stream);
int sqrelu_vnm_compress_fp8(const uint16_t* y1, int64_t T, int64_t F, int V, int M, float scale, uint8_t* codes,
                            uint8_t* meta, uint8_t* colidx, float* amax, void* stream);
int spmm24_fp8(const uint8_t* Xq, float scale_x, const uint8_t* w_codes, const uint8_t* w_meta, float scale_w,
               const float* bias, int64_t T, int64_t N, int64_t K, uint16_t* out, void* stream);
size_t sffn_vnm_spmm_fp8_workspace_bytes(int64_t T, int64_t N, int64_t Kfull);
int vnm_spmm_fp8(const uint8_t* a_codes, const uint8_t* a_meta, const uint8_t* a_colidx, float scale_a, const uint8_t* Wq,
                 float scale_w, int w_kmajor, int64_t T, int64_t N, int64_t Kfull, int V, int M, uint16_t* out,
                 void* workspace, size_t ws_bytes, void* stream);

/* Alg. 1 + Alg. 2 with fp8 operands in the four contractions whose sparse operand is 2:4 along the contraction (eqs. (1), (3),
 * (4), (7)); the reading of Section 3.4's closing paragraph applied to the whole step.  Six per-tensor scales, given by the caller
 * (host struct): x, w1, w2, y2, dy, dy1; a weight keeps one scale for both of its uses.  X, dY, the dense W2 (eq. (3)) and the
 * dense W1 (eq. (7)) are quantised by plain scans, the pruned W1 / W2.T inside the pruning pass, y2's and dy1's survivors inside
 * the epilogues of eqs. (1) / (4).  Everything that decides a position stays bf16 (y1, y2, the column scores, the 2:4 choices,
 * eq. (6)), so metadata and column indices are those the bf16 rules give on this step's own y1; the weight gradients (eqs. (5),
 * (8)) are the bf16 contractions on the bf16 survivors.  out = bf16( (sum dec * dec) * (scale_a * scale_b) [+ b1] ).
 * With SFFN_FLAG_FP8_WGRAD the weight gradients also contract codes, the ones the forward / input-gradient contractions already use:
 * dW2 = bf16( (sum_t dec(y2q[t,f]) dec(dYq[t,d])) * (s_y2 s_dy) ), dW1 = bf16( (sum_t dec(dy1q[t,f]) dec(Xq[t,d])) * (s_dy1 s_x) ).
 * amax (device, 6 floats in the order of the scales, or NULL): the step clears it and leaves the largest magnitude of X, W1, W2, y2's
 * survivors, dY and dy1's survivors there (exact maxima; what the caller derives the next step's scales from).
 * Shapes: V = 64, M in {8, 16, 32, 64} (Table 5's blocks), T a multiple of 64, D and F multiples of 128, for M >= 16 also 4 F / M a
 * multiple of 128 (eqs. (3), (7) then contract only the kept rows of the quantised W2.T / W1, gathered per token block);
 * cfg->flags: any of SFFN_FLAG_KEEP_DENSE, SFFN_FLAG_FP8_WGRAD, SFFN_FLAG_LEAN (the canonical w1 / w2t codes + meta and, at M = 8, the
 * y2 codes are not written and take no room), SFFN_FLAG_WEIGHTS_PACKED, SFFN_FLAG_DW_FP32_ACCUMULATE.
 * Workspace: sffn_fp8_workspace_bytes(cfg); after the call it holds, at the offsets of sffn_fp8_workspace_layout: the pruned
 * weights (codes [F, D/2] u8 + meta [F, D/8]), y2 (codes [T, 2F/M] u8, meta [T, F/(2M)], colidx [T/64, F/M, 4]), dy1 at y2's slots
 * (dy1_vals: bf16 [T, F/4] at M = 8, codes [T, 2F/M] u8 at M >= 16), y1 at y2's slots (y1_kept, laid out as in ffn_sparse_step) and,
 * with KEEP_DENSE, y1 / dy2. */
typedef struct { float x, w1, w2, y2, dy, dy1; } sffn_fp8_scales;
typedef struct {
    size_t w1_codes, w1_meta, w2t_codes, w2t_meta, y1, y2_codes, y2_meta, colidx, dy2, dy1_vals, y1_kept, total;
} sffn_fp8_ws_layout;
size_t sffn_fp8_workspace_bytes(const sffn_cfg* cfg);
int sffn_fp8_workspace_layout(const sffn_cfg* cfg, sffn_fp8_ws_layout* out);
int ffn_sparse_step_fp8(const sffn_cfg* cfg, const sffn_fp8_scales* scales, const uint16_t* X, const uint16_t* W1,
                        const uint16_t* W2, const float* b1, const uint16_t* dY, uint16_t* Y3, uint16_t* dX, uint16_t* dW1,
                        uint16_t* dW2, void* workspace, size_t ws_bytes, float* amax, void* stream);
/* The mixture-of-experts form (as ffn_sparse_step_grouped: expert e owns token rows seg_offsets[e] .. seg_offsets[e+1], a host array of
 * n_experts + 1 ascending multiples of 64 from 0 to T; W1 [E, F, D], W2 [E, D, F], b1 [E, F], dW1 / dW2 likewise).  One scale per
 * stacked tensor (all experts' W1 share s_w1, ...); amax likewise over all experts.  The contractions are one grouped launch per stage;
 * the weight passes run once per expert.  Workspace: sffn_fp8_grouped_workspace_layout(cfg, n_experts, &l).total bytes. */
int sffn_fp8_grouped_workspace_layout(const sffn_cfg* cfg, int n_experts, sffn_fp8_ws_layout* out);
int ffn_sparse_step_fp8_grouped(const sffn_cfg* cfg, const sffn_fp8_scales* scales, int n_experts, const int64_t* seg_offsets,
                                const uint16_t* X, const uint16_t* W1, const uint16_t* W2, const float* b1, const uint16_t* dY,
                                uint16_t* Y3, uint16_t* dX, uint16_t* dW1, uint16_t* dW2, void* workspace, size_t ws_bytes,
                                float* amax, void* stream);

/* Section 3.3 / Alg. 3 ("Convert Activation to Venom") and the conversion steps 1-3 of Section 3.4: neuron-level
 * experts that produce the V:N:M activation directly.  Reading built here: E = M/4 experts; expert e owns the hidden
 * units f with (f mod M)/4 == e (the offline clustering is taken as already applied to W1's row order), so a block of
 * 64 token rows routed to e keeps exactly the block columns 4e..4e+3; a token goes to one expert.
 *
 * venom_route = steps 1-2.  means [M/4, D] bf16 (unit-normalised offline, which makes the product below rank experts
 * like the cosine similarity).  s[t,e] = sum_d X[t,d]*means[e,d] in fp32 with a fixed order (products in chunks of 8
 * consecutive d; partial sum l of 64 takes chunks l, l+64, ... in ascending d; the partials are folded by 32, 16, 8,
 * 4, 2, 1); expert[t] = argmax_e, ties to the lower e.  Then a stable grouping: tokens of one expert in ascending
 * order, every run padded to a multiple of 64 rows.  Outputs (device): expert [T]; perm [rows] = token of a row or -1
 * (padding), rows = sffn_venom_rows(T, M) = ceil64(T) + 64 M/4; row_of_token [T]; seg [M/4 + 1] int32 run offsets;
 * scores [T, M/4] fp32 or NULL.  D a positive multiple of 8.  The caller copies seg to the host for the next call. */
int64_t sffn_venom_rows(int64_t T, int M);
size_t  sffn_venom_route_workspace_bytes(int64_t T, int M);
int venom_route(const uint16_t* X, const uint16_t* means, int64_t T, int64_t D, int M, int32_t* expert,
                int32_t* perm, int32_t* row_of_token, int32_t* seg, float* scores, void* workspace,
                size_t ws_bytes, void* stream);

/* venom_expert_matmul = step 3, the batched matmul that emits V:N:M: for row r of expert e's run and compact column j
 * (hidden unit f = (j/4) M + 4e + j%4): y1c[r,j] = bf16( sum_d X[perm[r],d] * W1s[f,d] + b1[f] ), W1s = sparsify24(W1)
 * (Alg. 1 line 4, cfg->mode); then eq. (2) and the 2:4 rule of Section 2.3 on every four consecutive compact columns.
 * cfg: T tokens, D, F, V = 64, M; seg_offsets: HOST array [M/4 + 1] as produced by venom_route (validated here);
 * outputs over rows = sffn_venom_rows(T, M): vals [rows, 2F/M], meta [rows, F/(2M)], colidx [rows/64, F/M, 4] in the
 * packed layout above (padding rows are +0), y1c [rows, 4F/M] or NULL.  4F/M must be a multiple of 64.  One grouped
 * launch on the structured-sparse matrix cores; (vals, meta, colidx) feed vnm_spmm / vnm_wgrad / dsqrelu_vnm as is. */
size_t sffn_venom_matmul_workspace_bytes(int64_t T, int64_t D, int64_t F, int M);
int venom_expert_matmul(const sffn_cfg* cfg, const int64_t* seg_offsets, const uint16_t* X, const int32_t* perm,
                        const uint16_t* W1, const float* b1, uint16_t* y1c, uint16_t* vals, uint8_t* meta,
                        uint8_t* colidx, void* workspace, size_t ws_bytes, void* stream);

/* Alg. 1 + Alg. 2 with Alg. 3 as the activation sparsifier (Alg. 1 line 6, MoEToVenom): the whole training step of the
 * neuron-level router, given the routing of venom_route (seg_offsets: HOST array; perm: device).
 * Forward: y1c / V:N:M y2 as in venom_expert_matmul, Y3 = y2v W2.T (eq. (3), dense W2).  Backward: dy2 = dY sparsify24(W2.T)
 * evaluated at the routed expert's hidden units only (eq. (4)), eq. (6) on y2's slots, dX with the dense W1 (eq. (7)), and
 * both weight gradients (eqs. (5), (8)); every contraction is grouped by expert, so all six shrink with 4/M.  Y3, dX [T,D]
 * come back in token order; dW1 [F,D], dW2 [D,F] are fully overwritten (hidden units of an expert without tokens: zeros).
 * Intermediates land in `workspace` at the offsets of sffn_router_workspace_layout() (row order of perm, rows =
 * sffn_venom_rows(T, M)); dy2c is stored only with SFFN_FLAG_KEEP_DENSE (eq. (6) runs in the epilogue of eq. (4)).
 * Needs 4F/M a multiple of 64. */
typedef struct {
    size_t y1c, vals, meta, colidx, dy2c, dvals, total;   /* y1c, dy2c [rows,4F/M] bf16; vals, dvals [rows,2F/M]; meta [rows,F/(2M)] */
} sffn_router_layout;
size_t sffn_router_workspace_bytes(const sffn_cfg* cfg);
int    sffn_router_workspace_layout(const sffn_cfg* cfg, sffn_router_layout* out);
int ffn_router_step(const sffn_cfg* cfg, const int64_t* seg_offsets, const int32_t* perm, const uint16_t* X,
                    const uint16_t* W1, const uint16_t* W2, const float* b1, const uint16_t* dY, uint16_t* Y3,
                    uint16_t* dX, uint16_t* dW1, uint16_t* dW2, void* workspace, size_t ws_bytes, void* stream);

/* venom_route + ffn_router_step in one call without a read-back: the run offsets stay on the device (they are written and
 * read by this library's own kernels on `stream`), the grouped launches are sized for the worst case.  means as in
 * venom_route; the step's intermediates sit at the offsets of sffn_router_workspace_layout(), the routing buffers behind
 * them.  Same results as the two-call form. */
size_t sffn_router_full_workspace_bytes(const sffn_cfg* cfg);
int ffn_router_full_step(const sffn_cfg* cfg, const uint16_t* means, const uint16_t* X, const uint16_t* W1,
                         const uint16_t* W2, const float* b1, const uint16_t* dY, uint16_t* Y3, uint16_t* dX,
                         uint16_t* dW1, uint16_t* dW2, void* workspace, size_t ws_bytes, void* stream);

/* The router's step as two calls (forward: Alg. 1 with Alg. 3 as the sparsifier, eqs. (1)-(3), and ALL of the weight preparation,
 * Alg. 2 line 2 and the experts' slices of W2 and W1.T included; backward: Alg. 2, eqs. (4)-(8)), for a training loop in which other
 * layers run in between.  Same kernels and bits as the one-call forms.  The two halves meet in `workspace`, which the caller keeps
 * untouched between them (one per layer in flight; the backward call consumes what the forward call left, so each forward call is
 * followed by one backward call); the backward call takes the same seg_offsets and perm as the forward call
 * (ffn_router_full_backward reads the routing that ffn_router_full_forward left in the workspace) and no weights.
 * SFFN_FLAG_WEIGHTS_PACKED (one-call and forward forms): the five weight-preparation launches are skipped and the call reads what
 * the previous call on this workspace prepared from the same W1, W2 (the caller's promise, as for ffn_sparse_step). */
int ffn_router_forward(const sffn_cfg* cfg, const int64_t* seg_offsets, const int32_t* perm, const uint16_t* X,
                       const uint16_t* W1, const uint16_t* W2, const float* b1, uint16_t* Y3, void* workspace, size_t ws_bytes,
                       void* stream);
int ffn_router_backward(const sffn_cfg* cfg, const int64_t* seg_offsets, const int32_t* perm, const uint16_t* dY, uint16_t* dX,
                        uint16_t* dW1, uint16_t* dW2, void* workspace, size_t ws_bytes, void* stream);
int ffn_router_full_forward(const sffn_cfg* cfg, const uint16_t* means, const uint16_t* X, const uint16_t* W1,
                            const uint16_t* W2, const float* b1, uint16_t* Y3, void* workspace, size_t ws_bytes, void* stream);
int ffn_router_full_backward(const sffn_cfg* cfg, const uint16_t* dY, uint16_t* dX, uint16_t* dW1, uint16_t* dW2,
                             void* workspace, size_t ws_bytes, void* stream);

/* Alg. 1 + Alg. 2, one call: X [T,D], W1 [F,D], W2 [D,F], b1 fp32 [F] or NULL, dY [T,D] ->
 * Y3 [T,D], dX [T,D], dW1 [F,D], dW2 [D,F]; intermediates land in `workspace` at the offsets of
 * sffn_workspace_layout().  Both weight matrices are re-pruned inside the call (SFFN_FLAG_WEIGHTS_PACKED: a later micro-batch
 * of the same optimizer step reuses what the previous call packed).
 * Size limits (SFFN_EUNSUPPORTED beyond them, nothing enqueued): T below 65536; one weight matrix below 2 GiB (F * D below 2^30 elements;
 * fp8 step: below 2^31), because the kernels of eqs. (3), (7) address the dense weight with 32-bit offsets (cfg->M = 16, 32, 64 in bf16:
 * a larger weight takes the unfused path, which contracts the activation as plain 2:4 and has no such limit).
 * cfg->M = 16, 32 or 64 (Table 5): the same algorithm and the same fusion; eqs. (3), (7) contract only the kept rows of
 * W2.T / W1 (see vnm_spmm), and the packed activation tensors have the sizes given above.  Shapes whose 4 F / M is not a
 * multiple of 64 or exceeds 7168, and calls with SFFN_FLAG_UNFUSED, run eqs. (2), (6) as separate kernels instead: the dense
 * y1 and dy2 are then always stored and y1_kept is not produced. */
int ffn_sparse_step(const sffn_cfg* cfg, const uint16_t* X, const uint16_t* W1, const uint16_t* W2,
                    const float* b1, const uint16_t* dY, uint16_t* Y3, uint16_t* dX, uint16_t* dW1,
                    uint16_t* dW2, void* workspace, size_t ws_bytes, void* stream);

/* ffn_sparse_step for callers that cannot allocate device memory or hand over a workspace: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments, kernels and results as ffn_sparse_step, but the
 * workspace is a device array built into the library (SFFN_NOALLOC_WORKSPACE_MAX bytes, held by every GPU the library has
 * run on until the process ends); the call allocates and frees nothing.  Shapes whose sffn_workspace_bytes() exceed that
 * size are refused with SFFN_EWORKSPACE before anything is enqueued (e.g. T = 1024, D = 512, F = 2048 fits; the benchmark
 * layers do not: they take ffn_sparse_step).  The intermediates stay inside the library.  All calls on one GPU share the
 * one array: calls that overlap in time on the same GPU (two streams, two threads) race; calls on one stream are ordered
 * and need no clearing in between, whatever their shapes. */
#define SFFN_NOALLOC_WORKSPACE_MAX (32u << 20)
int ffn_sparse_step_noalloc(const sffn_cfg* cfg, const uint16_t* X, const uint16_t* W1, const uint16_t* W2,
                            const float* b1, const uint16_t* dY, uint16_t* Y3, uint16_t* dX, uint16_t* dW1,
                            uint16_t* dW2, void* stream);

/* Mixture-of-experts form of the step (Section 1 states the method carries over to MoE FFNs; every expert is
 * one Alg. 1 + Alg. 2 FFN): n_experts (1..64) experts with their own weights, each applied to one consecutive
 * segment of the T token rows.  seg_offsets is a HOST array of n_experts + 1 ascending multiples of 64 with
 * seg_offsets[0] = 0 and seg_offsets[n_experts] = cfg->T (it is read during the call, not afterwards); a segment
 * may be empty, its expert then gets zero weight gradients.  Rows the caller pads a segment with must be zero in X
 * and dY.  X, dY, Y3, dX: [T, D]; W1, dW1: [n_experts, F, D]; W2, dW2: [n_experts, D, F]; b1: [n_experts, F] or NULL.
 * Every stage is a single launch over all experts (cfg->M = 16, 32, 64: fused path only, SFFN_EUNSUPPORTED for shapes it does
 * not cover).  The workspace has the layout of ffn_sparse_step with every
 * weight-shaped tensor holding n_experts matrices back to back (sffn_grouped_workspace_layout()).  The router,
 * the token permutation and the weighted combine of an MoE layer are outside this library. */
size_t sffn_grouped_workspace_bytes(const sffn_cfg* cfg, int n_experts);
int    sffn_grouped_workspace_layout(const sffn_cfg* cfg, int n_experts, sffn_ws_layout* out);
int ffn_sparse_step_grouped(const sffn_cfg* cfg, int n_experts, const int64_t* seg_offsets, const uint16_t* X,
                            const uint16_t* W1, const uint16_t* W2, const float* b1, const uint16_t* dY, uint16_t* Y3,
                            uint16_t* dX, uint16_t* dW1, uint16_t* dW2, void* workspace, size_t ws_bytes, void* stream);

/* Alg. 1 (forward pass) and Alg. 2 (backward pass) as separate calls, for a training loop in which other layers run between a
 * layer's forward and its backward pass.  Together the two calls enqueue exactly the launches of the one-call step, in its order, and
 * give the same bits in every output and intermediate.
 *   forward  = Alg. 1, eqs. (1)-(3): X, W1, W2, b1 -> Y3.  It also packs W2.T (Alg. 2 line 2), because that pass over W2 is the one that
 *              writes the W2.T copy eq. (3) reads.  SFFN_FLAG_WEIGHTS_PACKED applies to this call.
 *   backward = Alg. 2, eqs. (4)-(8): dY -> dX, dW1, dW2.  The bf16 form reads the dense W1 in place (eq. (7)); the fp8 form reads the
 *              codes of W1 that its forward call wrote and takes no weight argument.
 * The one-call step's workspace is three regions with different lifetimes, and these calls take them as three DEVICE buffers
 * (256-byte aligned, not overlapping: SFFN_EINVAL otherwise; sizes from sffn_buffer_sizes / sffn_fp8_buffer_sizes, which fill the
 * *_bytes fields and clear the pointers):
 *   scratch  nothing in it outlives a call: every layer and micro-batch on a stream can hand over the same buffer;
 *   saved    written by forward, read by backward: what Alg. 2 line 1 saves (y2's metadata and column offsets, y1 at y2's kept slots, X.T,
 *            the compacted y2v.T).  One per layer and micro-batch in flight; the caller keeps it untouched between the two calls.
 *            The backward call consumes it (eq. (6)'s results take the place of y2's in part of it): one backward call per forward call;
 *   weights  written by a forward call without SFFN_FLAG_WEIGHTS_PACKED (both packed weights, W2.T; fp8: W1's codes too), read by that
 *            call, by its backward call and by every later call with the flag.  One per layer, good until the weights change.
 * The library cannot check what the buffers hold.  Arguments, shapes, alignment, error codes otherwise: those of the one-call entry
 * points (a missing or short buffer: SFFN_EWORKSPACE).  Not built for the unfused wide-block path (SFFN_EUNSUPPORTED); the router's
 * step has its own pair, ffn_router_forward / ffn_router_backward.  fp8: the forward call writes amax[0..3] (x, w1, w2, y2) and leaves amax[4], amax[5] alone, the backward call writes
 * amax[4], amax[5] (dy, dy1) only. */
typedef struct sffn_buffers {
    void*  scratch;  size_t scratch_bytes;
    void*  saved;    size_t saved_bytes;
    void*  weights;  size_t weights_bytes;
} sffn_buffers;
int sffn_buffer_sizes(const sffn_cfg* cfg, int n_experts, sffn_buffers* out);        /* n_experts = 1: the plain step */
int sffn_fp8_buffer_sizes(const sffn_cfg* cfg, int n_experts, sffn_buffers* out);
int ffn_sparse_forward(const sffn_cfg* cfg, const uint16_t* X, const uint16_t* W1, const uint16_t* W2, const float* b1,
                       uint16_t* Y3, const sffn_buffers* buf, void* stream);
int ffn_sparse_backward(const sffn_cfg* cfg, const uint16_t* W1, const uint16_t* dY, uint16_t* dX, uint16_t* dW1,
                        uint16_t* dW2, const sffn_buffers* buf, void* stream);
int ffn_sparse_forward_grouped(const sffn_cfg* cfg, int n_experts, const int64_t* seg_offsets, const uint16_t* X,
                               const uint16_t* W1, const uint16_t* W2, const float* b1, uint16_t* Y3, const sffn_buffers* buf,
                               void* stream);
int ffn_sparse_backward_grouped(const sffn_cfg* cfg, int n_experts, const int64_t* seg_offsets, const uint16_t* W1,
                                const uint16_t* dY, uint16_t* dX, uint16_t* dW1, uint16_t* dW2, const sffn_buffers* buf,
                                void* stream);
int ffn_sparse_forward_fp8(const sffn_cfg* cfg, const sffn_fp8_scales* scales, const uint16_t* X, const uint16_t* W1,
                           const uint16_t* W2, const float* b1, uint16_t* Y3, const sffn_buffers* buf, float* amax, void* stream);
int ffn_sparse_backward_fp8(const sffn_cfg* cfg, const sffn_fp8_scales* scales, const uint16_t* dY, uint16_t* dX,
                            uint16_t* dW1, uint16_t* dW2, const sffn_buffers* buf, float* amax, void* stream);
int ffn_sparse_forward_fp8_grouped(const sffn_cfg* cfg, const sffn_fp8_scales* scales, int n_experts,
                                   const int64_t* seg_offsets, const uint16_t* X, const uint16_t* W1, const uint16_t* W2,
                                   const float* b1, uint16_t* Y3, const sffn_buffers* buf, float* amax, void* stream);
int ffn_sparse_backward_fp8_grouped(const sffn_cfg* cfg, const sffn_fp8_scales* scales, int n_experts,
                                    const int64_t* seg_offsets, const uint16_t* dY, uint16_t* dX, uint16_t* dW1,
                                    uint16_t* dW2, const sffn_buffers* buf, float* amax, void* stream);

/* Measurement aid (not part of the method): when enabled, ffn_sparse_step records a HIP event on the
 * caller's stream behind every kernel launch.  sffn_profile_read() waits for the last event of the
 * most recent step and returns the number of launches, filling ms[i] (duration of launch i) and
 * names[i] (static strings naming the stage).  Not thread-safe; enable/disable create/destroy events. */
int sffn_profile_enable(int on);
int sffn_profile_read(float* ms, const char** names, int max_n);

/* Measurement aid (not part of the method): the two element-wise operations of the DENSE FFN step that the benchmark
 * times as its baseline, each as one pass over HBM: eq. (2) y2 = bf16(max(y1, 0)^2) and eq. (6)
 * dy1 = bf16(2 * dy2 * max(y1, 0)) of Section 2.1 on n contiguous bf16 elements (n a positive multiple of 8, pointers
 * 16-byte aligned, device memory; outputs may not alias inputs).  SFFN_EINVAL with nothing enqueued otherwise. */
int sffn_dense_sqrelu(const uint16_t* y1, uint16_t* y2, int64_t n, void* stream);
int sffn_dense_dsqrelu(const uint16_t* dy2, const uint16_t* y1, uint16_t* dy1, int64_t n, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SPARSEFFN_H */
