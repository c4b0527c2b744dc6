// Host-side launchers of the gfx950 kernels (internal to the library).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sffn {

// Fused V:N:M epilogue of the two GEMMs whose output feeds the activation sparsifier (ffn_sparse_step only).
//   mode 1 (eq. (1) -> eq. (2) + Section 2.3): the tile of y1 is squared-ReLU'd and compressed in place: outputs the
//          canonical V:N:M y2 (vals, meta, colidx), y1 at the kept slots (ykept, same indexing as vals), the plain
//          2:4 view (v24, m24; blocked layout) and the transposed y2v compacted to the four kept hidden units of every
//          (64-token block, group of 8) (at; [F / 2, T], blocked layout; see gemm_wgrad.hip).
//   mode 2 (eq. (4) -> eq. (6)): the tile of dy2 meets (meta, colidx, ykept) and becomes dy1 in y2's slots: outputs
//          vals (= dy1 values), v24 / m24 and at as above.
//   store_dense: also write the dense GEMM output (y1 / dy2) to `out`.
struct VnmEpilogue {
    int mode = 0;                   // 0: no V:N:M epilogue, only the dense output
    int store_dense = 1;
    uint16_t* vals = nullptr;
    uint8_t* meta = nullptr;
    uint8_t* colidx = nullptr;
    uint8_t* kmask = nullptr;       // mode 1: one byte per (64-token block, group of 8): bit c = column c of the group is kept
    uint16_t* ykept = nullptr;
    uint16_t* v24 = nullptr;
    uint8_t* m24 = nullptr;
    uint16_t* at = nullptr;
    // mode 3 (Section 3.3, neuron-level experts; grouped launch, A = one expert's hidden units in compact-column order):
    //        the tile of y1c gets the bias of its hidden units, is squared-ReLU'd and 2:4-pruned on every four consecutive
    //        compact columns: outputs vals, meta; padding rows (perm < 0) come out as zeros; `out` = y1c [rows, F] if store_dense.
    // mode 4 (the same experts, backward): the tile of dy2c meets (meta, ykept = the stored y1c [rows, F]) and becomes dy1 in y2's
    //        slots: outputs vals (canonical) and v24 (the same, blocked); `out` = dy2c if store_dense.
    // mode 5 / 6 (blocks of M = 2^logM = 16, 32, 64 columns, Table 5): as modes 1 / 2 with outputs vals, meta, colidx (mode 5), ykept
    //        ([T/64][F/64][64 tokens][64/M blocks] pairs), `at` + kmask (mode 5) exactly as for modes 1 / 2 (a block of M columns keeps 4, so no
    //        group of 8 hidden units keeps more than 4); no v24 / m24 (eqs. (3), (7) gather the kept rows of the dense operand from the
    //        canonical arrays).
    const int32_t* perm = nullptr;
    int logM = 3;
    // fp8 operands (launch_gemm_fp8_blocked, modes 1 / 2): the survivors leave as E4M3 codes quantised with 1 / scale = inv_out: mode 1 writes
    // vals as codes [T, F / 4], mode 2 keeps vals = dy1 in bf16; both write the codes into vcb.  ykept, at, kmask, colidx, meta stay as in the bf16 modes.
    // fp8 modes 5 / 6: vals = the survivors' codes [T, 2 F / M] in both directions (the operand of the gathered-row kernel); the rest as above.
    float inv_out = 1.0f;
    int at_fp8 = 0;                 // fp8 modes 1 / 2: `at` receives codes (pairs in the blocked layout, [F / 2, T]) instead of bf16
    float* amax = nullptr;          // fp8 modes 1 / 2: amax slots for the survivors' magnitudes (y2 / dy1)
    // modes 1 / 2: the operands of the V:2:8 activation GEMM (gemm_vnm8.hip; layouts: vcb_off, mcb_off, cixt_off in common.hpp, fp8: vcb8_off, ...):
    // vcb = the survivors (both modes; fp8: their codes), mcb = their metadata and cixt = the regrouped kept-column offsets (mode 1; mode 2 reuses them)
    uint16_t* vcb = nullptr;
    uint8_t* mcb = nullptr;
    uint8_t* cixt = nullptr;
};

// Grouped (mixture-of-experts) form of a contraction: the token axis is cut into n consecutive segments, one per
// expert (offsets seg[0] = 0 <= ... <= seg[n] = all tokens, multiples of 64), and each segment meets its own
// expert's weight operand.  `role` says which axis of the NT contraction the tokens are:
//   0: the i rows (A is token-indexed, B is the expert's weight matrix, out rows are tokens);
//   1: the j rows (A is the expert's packed weight matrix, B is token-indexed);
//   2: the contraction axis (A and B are [., all tokens] matrices, every expert gets its own output).
// Strides are per expert, in elements of the pointed-to type.  Token-indexed tensors always carry all tokens.
struct GemmGroup {
    static constexpr int kMaxExperts = 64;
    int n = 0;                      // 0: ordinary single contraction
    int role = 0;
    int64_t a_stride = 0, m_stride = 0, b_stride = 0, bias_stride = 0, out_stride = 0;
    // role 2 on row-major operands (weight gradients of the neuron-level experts, Section 3.3): output index i of expert e is
    // compact column i of its hidden units and lands at hidden unit (i / 4) * M + 4 e + i % 4 of the one shared output (0: off)
    int map_logM = 0;
    // roles 0 / none with the i-major output: row i goes to row out_row_map[i] of the output (negative: not stored)
    const int32_t* out_row_map = nullptr;
    // Segment offsets kept on the device (written by an earlier kernel of the same call, e.g. the router's grouping): when set,
    // the kernels read seg_dev[0..n] instead of seg[], and the launch is sized for the worst case of `cap_rows` token rows in n
    // runs (workgroups past the real tile count exit at once).  gemm_v2.hip kernels and the router's helpers only.
    const int32_t* seg_dev = nullptr;
    int64_t cap_rows = 0;
    int32_t seg[kMaxExperts + 1] = {0};
};

hipError_t launch_prune24(const uint16_t* src, int64_t R, int64_t K, int64_t ld, int trans, int mode, uint16_t* vals,
                          uint8_t* meta, hipStream_t stream);
hipError_t launch_dsqrelu_vnm(const uint16_t* dy2, const uint16_t* y1, const uint8_t* meta, const uint8_t* colidx,
                              int64_t T, int64_t F, uint16_t* dvals, hipStream_t s);
// 2:4 prune-and-pack for the fused step: canonical outputs plus the blocked copies the GEMMs read;
// trans = 1 can also emit a blocked copy of the source matrix itself (rows = its rows, K = its columns).
// batch > 1 (trans = 1 only): `batch` matrices of the same shape, consecutive in every argument.
hipError_t launch_prune24_step(const uint16_t* src, int64_t R, int64_t K, int64_t ld, int trans, int mode, uint16_t* vals,
                               uint8_t* meta, uint16_t* vblk, uint8_t* mblk, uint16_t* src_blk, hipStream_t stream, int batch = 1,
                               int cluster_M = 0,    // cluster_M (trans = 0): rows come out expert-major, see prune24.hip
                               uint16_t* src_t = nullptr);   // trans = 1: also the unpruned transposed source [R, K] row-major
// vnm_general.hip: the stand-alone compressor for M in {8, 16, 32, 64}, and eq. (6) / 2:4 re-expression / transposed expansion for M in {16, 32, 64}.
hipError_t launch_sqrelu_vnm_compress_m(const uint16_t* y1, int64_t T, int64_t F, int M, uint16_t* vals, uint8_t* meta, uint8_t* colidx,
                                        hipStream_t s);
hipError_t launch_dsqrelu_vnm_m(const uint16_t* dy2, const uint16_t* y1, const uint8_t* meta, const uint8_t* colidx, int64_t T, int64_t F,
                                int M, uint16_t* dvals, hipStream_t s);
hipError_t launch_vnm_to_24_m(const uint16_t* vals, const uint8_t* meta, const uint8_t* colidx, int64_t T, int64_t F, int M,
                              uint16_t* vals24, uint8_t* meta24, hipStream_t s);
hipError_t launch_vnm_expand_t_m(const uint16_t* vals, const uint8_t* meta, const uint8_t* colidx, int64_t T, int64_t F, int M,
                                 uint16_t* out, hipStream_t s);
// eqs. (3), (7) with the rows of the dense operand gathered per token block (gemm_gather.hip):
// out[t, n] = sum over the kept columns f of A[t, f] * Wk[f, n]; Wk = [F, ldw] (contraction index = row).
// vnm_spmm_gather_ok: shapes the kernel covers (4 F / M a multiple of 64 and at most 7168); others take the plain-2:4 route.
bool vnm_spmm_gather_ok(int64_t T, int64_t N, int64_t F, int M);
// grp (role 0, host segment table): the token blocks of segment e take expert e's matrix Wk + e * b_stride.
hipError_t launch_vnm_spmm_gather(const uint16_t* a_vals, const uint8_t* a_meta, const uint8_t* colidx, const uint16_t* Wk, int64_t ldw,
                                  int64_t T, int64_t N, int64_t F, int M, uint16_t* out, int64_t ldo, hipStream_t s, const GemmGroup* grp = nullptr);
// eqs. (3), (7) for M = 8 on a 256-token tile (gemm_vnm8.hip): the activation as the epilogues' vcb / mcb / cixt arrays, Wk = [F, ldw] with the
// contraction index as row; T, N, F multiples of 64.  grp as above (b_stride in elements).
bool vnm8_gemm_ok(int64_t T, int64_t N, int64_t F, int64_t ldw);
hipError_t launch_vnm8_gemm(const uint16_t* vcb, const uint8_t* mcb, const uint8_t* cixt, const uint16_t* Wk, int64_t ldw, int64_t T, int64_t N,
                            int64_t F, uint16_t* out, int64_t ldo, hipStream_t s, const GemmGroup* grp = nullptr);
// vnm.hip: the canonical V:2:8 arrays (vals [T, F/4], meta [T, F/16], colidx [T/64, F/8, 4]) regrouped into those units
hipError_t launch_vnm8_repack(const uint16_t* vals, const uint8_t* meta, const uint8_t* colidx, int64_t T, int64_t F, uint16_t* vcb, uint8_t* mcb,
                              uint8_t* cixt, hipStream_t s);
// (fp8 step: codes; F a multiple of 128, Wq = [F, ldw bytes], out = bf16(alpha * sum); the arrays in the layouts of vcb8_off, mcb8_off, cixt8_off)
bool vnm8_gemm_fp8_ok(int64_t T, int64_t N, int64_t F, int64_t ldw);
// fp8.hip: the canonical fp8 V:2:8 arrays (codes [T, F/4], meta, colidx) regrouped into those units; F a multiple of 128
hipError_t launch_vnm8_repack_fp8(const uint8_t* codes, const uint8_t* meta, const uint8_t* colidx, int64_t T, int64_t F, uint8_t* vcb, uint8_t* mcb,
                                  uint8_t* cixt, hipStream_t s);
hipError_t launch_vnm8_gemm_fp8(const uint8_t* vcb, const uint8_t* mcb, const uint8_t* cixt, const uint8_t* Wq, int64_t ldw, float alpha, int64_t T,
                                int64_t N, int64_t F, uint16_t* out, int64_t ldo, hipStream_t s, const GemmGroup* grp = nullptr);
// The same on E4M3 codes: a_codes [T, 2 F / M] + the same metadata and column offsets, Wq = codes [F, ldw bytes], out = bf16(alpha * sum);
// 4 F / M a multiple of 128; b_stride of grp in bytes.
bool vnm_spmm_gather_fp8_ok(int64_t T, int64_t N, int64_t F, int M);
hipError_t launch_vnm_spmm_gather_fp8(const uint8_t* a_codes, const uint8_t* a_meta, const uint8_t* colidx, const uint8_t* Wq, int64_t ldw, float alpha,
                                      int64_t T, int64_t N, int64_t F, int M, uint16_t* out, int64_t ldo, hipStream_t s, const GemmGroup* grp = nullptr);
hipError_t launch_vnm_to_24(const uint16_t* vals, const uint8_t* meta, const uint8_t* colidx, int64_t T, int64_t F,
                            uint16_t* vals24, uint8_t* meta24, hipStream_t s);
hipError_t launch_vnm_expand_t(const uint16_t* vals, const uint8_t* meta, const uint8_t* colidx, int64_t T, int64_t F,
                               uint16_t* out, int blocked, hipStream_t s);
// batch > 1: `batch` matrices [R, C] (ld = C) back to back, transposed one by one.
// cluster_M (with batch = M / 4 experts, R = hidden units per expert): matrix e reads the rows of `in` that belong to expert e,
// row r of it = row (r / 4) * M + 4 e + r % 4 of the one [F, C] source (Section 3.3's expert-major order).
// in_perm (batch = 1): row r of the [R, C] matrix is row in_perm[r] of `in` (a negative entry: a zero row).
hipError_t launch_transpose(const uint16_t* in, int64_t R, int64_t C, int64_t ld, uint16_t* out, int blocked, uint16_t* out_same,
                            hipStream_t s, int batch = 1, int cluster_M = 0, const int32_t* in_perm = nullptr);

// C[i, j] = sum_k A[i, k] * B[j, k]  (both operands K-contiguous).
//   sparse_a: A given as 2:4 packed (a_vals [Ra, K/2], a_meta [Ra, K/8]) and multiplied on the
//             structured-sparse matrix cores; else a_vals is a dense [Ra, K] matrix.
//   out_i_contig: 1 -> out[j * ldo + i] (+ bias[i]);  0 -> out[i * ldo + j].
//   launch_spmm_blocked: A packed 2:4; both operands (and the metadata) are in the blocked layout of common.hpp;
//   out_i_contig must be 0 (eqs. (3), (7) of the fused step).
// eq. (1) / eq. (4) with the fused epilogue above: A packed 2:4 [Ra = F rows], B = [Rb = T rows], all blocked; out [T, F].
// grp (optional, blocked launchers only): grouped form, see GemmGroup; Ra / Rb / K then count all tokens on the token axis.
hipError_t launch_gemm_vnm_epilogue(const uint16_t* a_vals, const uint8_t* a_meta, const uint16_t* B, const float* bias, int64_t F,
                                    int64_t T, int64_t K, uint16_t* out, const VnmEpilogue& ep, hipStream_t s,
                                    const GemmGroup* grp = nullptr);
hipError_t launch_spmm_blocked(const uint16_t* a_vals, const uint8_t* a_meta, const uint16_t* B, const float* bias, int64_t Ra, int64_t Rb,
                               int64_t K, int out_i_contig, uint16_t* out, int64_t ldo, hipStream_t s, const GemmGroup* grp = nullptr);
hipError_t launch_gemm_nt(int sparse_a, const uint16_t* a_vals, const uint8_t* a_meta, const uint16_t* B, const float* bias,
                          int64_t Ra, int64_t Rb, int64_t K, int out_i_contig, uint16_t* out, int64_t ldo, hipStream_t s,
                          const GemmGroup* grp = nullptr);   // grp: dense A only, role 2 (every expert contracts over its own k range)

// eqs. (5), (8): C[f, n] = sum_t A[t, f] * G[t, n] with A given as `atc` (compacted transposed activation written by the
// V:N:M epilogue) + kmask (kept-column bit masks, [T / 64, F / 8]), G = [N rows, T] in the blocked layout; out_i_contig: out[n * ldo + f], else out[f * ldo + n].
// grp (role 2): every expert contracts over its own token segment into its own output (out_stride).
// Section 3.3 / Alg. 3 (router.hip): routing scores + top-1, stable grouping by expert, permuted X, colidx of the result.
hipError_t launch_venom_route(const uint16_t* X, const uint16_t* means, int64_t T, int64_t D, int E, int32_t* expert, float* scores,
                              hipStream_t s);
hipError_t launch_venom_permute(const int32_t* expert, int64_t T, int E, int64_t cap, int32_t* blockcnt, int32_t* seg, int32_t* perm,
                                int32_t* row_of_token, hipStream_t s);
hipError_t launch_venom_gather_x(const uint16_t* X, const int32_t* perm, int64_t cap, int64_t D, uint16_t* xb, hipStream_t s);
hipError_t launch_venom_expand_t_compact(const uint16_t* vals, const uint8_t* meta, int64_t rows, int64_t Kc, uint16_t* at, hipStream_t s);
struct TailFill {                   // up to five arrays of `rows` rows whose tail rows get a fill word
    int n = 0;
    uint32_t* p[5] = {nullptr, nullptr, nullptr, nullptr, nullptr};
    int64_t row_words[5] = {0, 0, 0, 0, 0};
    uint32_t v[5] = {0, 0, 0, 0, 0};
    void add(void* ptr, int64_t row_bytes, uint8_t byte) { p[n] = (uint32_t*)ptr; row_words[n] = row_bytes / 4; v[n] = 0x01010101u * byte; ++n; }
};
hipError_t launch_fill_tail_rows(const TailFill& f, const int32_t* first_dev, int64_t first_imm, int64_t rows, int64_t max_tail_rows,
                                 hipStream_t s);
hipError_t launch_venom_colidx(const GemmGroup& g, int64_t cap, int64_t groups, uint8_t* colidx, hipStream_t s);

// fp8 operands (fp8.hip; Section 3.4's closing paragraph): E4M3 codes, inv = 1 / scale; amax (optional, device float) receives the largest
// magnitude quantised through an atomic max.
hipError_t launch_quantize_fp8(const uint16_t* src, int64_t n, float inv, uint8_t* codes, float* amax, hipStream_t s);
hipError_t launch_prune24_fp8(const uint16_t* src, int64_t R, int64_t K, int64_t ld, int trans, int mode, float inv, uint8_t* codes, uint8_t* meta,
                              float* amax, hipStream_t s);
hipError_t launch_sqrelu_vnm_compress_fp8(const uint16_t* y1, int64_t T, int64_t F, int M, float inv, uint8_t* codes, uint8_t* meta, uint8_t* colidx,
                                          float* amax, hipStream_t s);
hipError_t launch_vnm_to_24_fp8(const uint8_t* codes, const uint8_t* meta, const uint8_t* colidx, int64_t T, int64_t F, int M, uint8_t* codes24,
                                uint8_t* meta24, hipStream_t s);
hipError_t launch_transpose_u8(const uint8_t* in, int64_t R, int64_t C, int64_t ld, uint8_t* out, hipStream_t s);
// C[i, j] = alpha * sum_k dec(A[i, k]) * dec(B[j, k]) (+ bias[i] when out_i_contig) on v_smfmac_f32_32x32x64_fp8_fp8: A packed 2:4 codes
// [Ra, K/2] + metadata [Ra, K/8], B codes [Rb, K], both row-major; K a multiple of 128; out bf16 as launch_gemm_nt.
hipError_t launch_spmm24_fp8(const uint8_t* a_codes, const uint8_t* a_meta, const uint8_t* Bq, const float* bias, float alpha, int64_t Ra, int64_t Rb,
                             int64_t K, int out_i_contig, uint16_t* out, int64_t ldo, hipStream_t s);

// The same contraction on operands in the blocked layout with a pair of codes per 2-byte element (the fused fp8 step): a_codes = packed 2:4
// codes [Ra, K/2], a_meta in the fp8 metadata units of common.hpp, Bq = codes [Rb, K]; eq. (1) / eq. (4) with the fused V:N:M epilogue ep
// (mode 1 or 2: M = 8; mode 5 or 6: M = 2^logM = 16, 32, 64), Ra = hidden units, Rb = tokens, out [T, F] if ep->store_dense.
hipError_t launch_gemm_fp8_blocked(const uint8_t* a_codes, const uint8_t* a_meta, const uint8_t* Bq, const float* bias, float alpha, int64_t Ra,
                                   int64_t Rb, int64_t K, uint16_t* out, int64_t ldo, const VnmEpilogue* ep, hipStream_t s, const GemmGroup* grp = nullptr);
// fp8.hip, producers of such operands: quantised copy in the same orientation / transposed; 2:4 pruning that also writes the blocked codes
// (amax, optional: the tensor's amax slots, see below)
hipError_t launch_quantize_fp8_blocked(const uint16_t* src, int64_t R, int64_t C, int64_t ld, float inv, uint8_t* out_blk, hipStream_t s, float* amax = nullptr);
// (out_same_blk: also the codes in the source's orientation)
hipError_t launch_transpose_quantize_fp8_blocked(const uint16_t* src, int64_t R, int64_t C, int64_t ld, float inv, uint8_t* out_t_blk, hipStream_t s,
                                                 float* amax = nullptr, uint8_t* out_same_blk = nullptr);
// amax slots of the fused fp8 step: n tensors x 64 slots x 256 bytes (kAmaxSlots, kAmaxSlotStride in common.hpp); the step's kernels take a tensor's slot base
hipError_t launch_amax_clear(float* slots, int n, hipStream_t s);
hipError_t launch_amax_finish(const float* slots, int n, float* out, hipStream_t s);
// 2:4 pruning + quantisation for the fp8 step, rows (trans = 0) or strided groups (trans = 1): the packed codes blocked (codes_blk) with the metadata in
// the fp8 units of common.hpp (meta_blk), and s_q = the unpruned logical matrix [R, K] itself as row-major codes (the operand of eqs. (3), (7),
// whose kept rows are picked or gathered per token block); amax_src: amax slots of the unpruned tensor; codes / meta (canonical) may be null
hipError_t launch_prune24_fp8_step(const uint16_t* src, int64_t R, int64_t K, int64_t ld, int trans, int mode, float inv, uint8_t* codes, uint8_t* meta,
                                   uint8_t* codes_blk, uint8_t* meta_blk, hipStream_t s, float* amax_src, uint8_t* s_q);

// the same on E4M3 codes (atc: compact transposed codes [F / 2, T], Gq [N, T], both in the blocked pair layout): out = bf16(alpha * sum)
hipError_t launch_wgrad_vnm_fp8(const uint8_t* atc, const uint8_t* kmask, const uint8_t* Gq, float alpha, int64_t F, int64_t N, int64_t T,
                                int out_i_contig, uint16_t* out, int64_t ldo, hipStream_t s, const GemmGroup* grp = nullptr, bool acc32 = false);
// acc32: `out` is a float32 matrix of the same shape (ldo in float32 elements; grouped form: out_stride in float32 elements) that the
// result is added to, out32 += alpha * sum, instead of a bf16 matrix that is overwritten
hipError_t launch_wgrad_vnm(const uint16_t* atc, const uint8_t* kmask, const uint16_t* G, int64_t F, int64_t N, int64_t T,
                            int out_i_contig, uint16_t* out, int64_t ldo, hipStream_t s, const GemmGroup* grp = nullptr, bool acc32 = false);


}  // namespace sffn
