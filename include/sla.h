/* sla.h - C ABI of the MI355X sparse-linear attention (SLA) library.
 *
 * SLA (arxiv 2509.24006) computes, per batch and head, for Q, K, V in R^{N x d}
 * (Section 2.1; tensors here are packed [B, H, N, d] or [B, N, H, d], d contiguous):
 *
 *   1. block scores  s = pool(Q) pool(K)^T / sqrt(d), pool = mean over each block of
 *      b_q (queries) or b_kv = 64 (keys) consecutive tokens (Eq. 2; the last block may be
 *      short); T_q = ceil(N / b_q) query blocks, T = ceil(N / 64) key blocks;
 *   2. a three-way block mask M_c[i, j] in {1, 0, -1}, T_q x T: per query-block row the n_h
 *      highest scores are critical (1), the n_l lowest of the rest negligible (-1),
 *      the others marginal (0) (Eq. 3, Alg. 1 mask line);
 *   3. O^s: online-softmax attention over the critical blocks only (Eq. 4);
 *   4. O^l = phi(Q_i) H_i / (phi(Q_i) Z_i) with H_i, Z_i the sums of the per-key-block
 *      states h_j = phi(K_j)^T V_j, z_j = rowsum(phi(K_j)^T) over the marginal blocks
 *      of row i (Eq. 5, Alg. 1);
 *   5. O = O^s + O^l W with a learned d x d matrix W ("Proj", Eq. 6);
 * and the matching gradients dQ, dK, dV, dW (Alg. 2, Eq. 7-8, plus the chain rule
 * through phi and W).  The mask is a constant of the backward pass.
 *
 * Conventions
 *   - Every pointer except `sla_params*` / `sla_sizes_t*` is DEVICE memory owned by the
 *     caller.  The library never allocates, frees or keeps device memory, and holds no
 *     state between calls.  Pointers must be 16-byte aligned (a misaligned one is SLA_EINVAL);
 *     any allocator's buffers are.
 *   - All work is enqueued on `stream` (a hipStream_t passed as void*, NULL = the null
 *     stream); no call synchronises the host.
 *   - Outputs are overwritten, never accumulated into.
 *   - Return value: SLA_OK, or a negative error code; nothing was enqueued when the code
 *     is SLA_EINVAL, SLA_EUNSUPPORTED or SLA_ENOSPACE.
 *   - Block counts (T = number of key blocks): n_h = floor(k_h*T + 1/2) clamped to [0, T];
 *     n_l = min(floor(k_l*T + 1/2), T - n_h); n_0 = T - n_h - n_l.  Every row of M_c has
 *     exactly n_h ones and n_l minus-ones.  Ties: critical = first n_h under (score
 *     descending, block index ascending); negligible = first n_l of the remaining
 *     entries under (score ascending, index ascending).
 *   - n_h = 0 gives O^s = 0 and L = -inf; n_0 = 0 gives O^l = 0, H_i = Z_i = 0.
 */
#ifndef SLA_H_
#define SLA_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { SLA_OK = 0, SLA_EINVAL = -1, SLA_EUNSUPPORTED = -2, SLA_ENOSPACE = -3, SLA_EHIP = -4 };
enum { SLA_PHI_SOFTMAX = 0, SLA_PHI_ELU1 = 1 };   /* feature map of the linear branch */
enum { SLA_F32 = 0, SLA_BF16 = 1 };               /* storage type of Q,K,V,W,O,dO,dQ,dK,dV */
enum { SLA_BHND = 0, SLA_BNHD = 1, SLA_STRIDED = 2 }; /* memory order of Q,K,V,O,dO,dQ,dK,dV      */

/* Problem statement (Alg. 1 input line: Q, K, V, block sizes, k_h, k_l; Section 6.1: phi). */
typedef struct sla_params {
  int32_t B, H, N, d; /* batch, heads, tokens, head dim; d in {64, 128}; N >= 1            */
  int32_t bq, bkv;    /* query / key block size: bkv = 64; bq = 64, 128, 192 or 256.  The
                         kernels work on 64-token tiles; a larger query block gives its
                         mask row to each of its 64-token tiles, so tables and saved states
                         are per tile (T rows) while M_c has T_q = ceil(N / bq) rows       */
  double k_h, k_l;    /* fractions in [0, 1] of critical / negligible blocks per row       */
  int32_t phi;        /* SLA_PHI_*                                                         */
  int32_t dtype;      /* SLA_F32 or SLA_BF16; statistics and dW are always float           */
  int32_t layout;     /* SLA_BHND: Q,K,V,O,dO,dQ,dK,dV packed [B,H,N,d]; SLA_BNHD: packed
                         [B,N,H,d] (token-major, as a transformer block's projections leave
                         them); SLA_STRIDED: element (b, h, n, c) of each of these tensors
                         sits stride_b b + stride_h h + stride_n n + c elements after its
                         pointer, e.g. Q, K, V as the three slices of one fused projection
                         output [B,N,3,H,d] (stride_b = 3 N H d, stride_h = d, stride_n =
                         3 H d; K = Q + H d, V = Q + 2 H d).  Masks, tables, saved tensors
                         and workspaces are packed per (b, h) in every case.               */
  int64_t stride_b, stride_h, stride_n; /* SLA_STRIDED only: element strides, multiples of 16
                         bytes, stride_n >= d, N stride_n elements below 2^31 bytes; rows of
                         different (b, h, n) must not overlap                               */
} sla_params;

/* Derived sizes and the layout of the opaque buffers (all offsets in bytes).
 * "state row" below means one block's linear-attention state stored as d*d + d floats:
 * first the d x d matrix TRANSPOSED (element [c][e] of the paper's matrix at e*d + c),
 * then the d-vector. */
typedef struct sla_sizes_t {
  int32_t T, n_h, n_l, n_0;   /* T = ceil(N / 64): key blocks = 64-token query tiles        */
  int32_t Tq, reserved;       /* Tq = ceil(N / bq): rows of M_c (= T when bq = 64)          */
  uint64_t mask_bytes;        /* int8  [B,H,Tq,T]                                           */
  uint64_t luts_bytes;        /* the buffer ends with scratch of the table build             */
  uint64_t lut_row_idx;       /* int32 [B,H,T,n_h]   ascending critical key blocks per query tile
                                 (below, row i of M_c stands for query tile i: the row i / (bq/64)) */
  uint64_t lut_col_ptr;       /* int32 [B,H,T+1]     CSC pointers of the critical entries   */
  uint64_t lut_col_rows;      /* int32 [B,H,T*n_h]   ascending query blocks per key block   */
  uint64_t lut_ind;           /* uint64 [B,H,T,Tw]   bit b of word q: M_c[i][64q+b] = 0 (marginal), Tw = ceil(T/64) */
  uint64_t lut_ind_t;         /* uint64 [B,H,T,Tw]   the same, transposed: bit b of [j][q]: M_c[64q+b][j] = 0 */
  uint64_t lut_col_order;     /* int32 [B,H,T]       key blocks by descending column count  */
  uint64_t saved_bytes;
  uint64_t saved_Os;          /* dtype [B,H,N,d]     O^s (this order whatever the layout)   */
  uint64_t saved_Ol;          /* dtype [B,H,N,d]     O^l                                    */
  uint64_t saved_L;           /* float [B,H,N]       L = m + log l                          */
  uint64_t saved_HZ;          /* float tensors: float [B,H,T] state rows (H_i transposed, then Z_i);
                                 bf16 tensors: bf16 [B,H,T,d*d] (H_i transposed) here and ...   */
  uint64_t saved_Z;           /* ... float [B,H,T,d] (Z_i) here; float tensors: = saved_HZ + 4 d d,
                                 rows d*d + d floats apart                                       */
  uint64_t ws_mask_bytes;
  uint64_t ws_mask_qbar;      /* float [B,H,Tq,d]    pool(Q), left in the workspace         */
  uint64_t ws_mask_kbar;      /* float [B,H,T,d]     pool(K)                                */
  uint64_t ws_mask_scores;    /* float [B,H,Tq,T]    pre-softmax block scores s             */
  uint64_t ws_forward_bytes;
  uint64_t ws_backward_bytes;
} sla_sizes_t;

/* Fills *out for the given problem.  Host-only, touches no device. */
int sla_sizes(const sla_params* p, sla_sizes_t* out);

/* Eq. 2 - Eq. 3 and the lookup tables of Appendix A.3.
 * Q, K: dtype [B,H,N,d] (or [B,N,H,d], see sla_params.layout).  Mc: int8 [B,H,Tq,T] (out).  luts: luts_bytes (out).
 * workspace: >= ws_mask_bytes; on return it holds pool(Q), pool(K) and s at the offsets
 * above.  Scores are computed in float in one fixed order (sequential sum over a block's
 * tokens, IEEE division by the token count, fused multiply-add chain over the features,
 * times the float 1/sqrt(d)), so the mask is reproducible bit for bit. */
int sla_build_mask(const sla_params* p, const void* Q, const void* K, int8_t* Mc, void* luts,
                   void* workspace, size_t workspace_bytes, void* stream);

/* sla_build_mask for callers that cannot allocate device memory (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): the same kernels, with the workspace in
 * a device array that is part of the library image instead of a caller's buffer.  The call
 * allocates nothing and frees nothing (keep sla_profile_enable off: its events are created per
 * launch).  Limit: problems whose ws_mask_bytes (see sla_sizes) exceed SLA_STATIC_WS_BYTES are
 * refused with SLA_ENOSPACE before anything is enqueued; the headline shape (12 heads, N = 32760)
 * needs 18.9 MB.  Each GPU holds one copy of the array for the life of the process; all calls on
 * a GPU share it, so two calls that may overlap on one GPU (different streams, or threads) race:
 * serialise them.  The array keeps the last call's pool(Q), pool(K) and scores; no call reads
 * them before writing them.  Q, K, Mc, luts, stream: as for sla_build_mask. */
#define SLA_STATIC_WS_BYTES (32u << 20)
int sla_build_mask_static(const sla_params* p, const void* Q, const void* K, int8_t* Mc, void* luts,
                          void* stream);

/* Eq. 3 alone: classify given float scores s [B,H,Tq,T] (device) and build the tables. */
int sla_classify_scores(const sla_params* p, const float* s, int8_t* Mc, void* luts, void* stream);

/* Algorithm 1 + Eq. 6.  Q, K, V, O: dtype [B,H,N,d] (or [B,N,H,d]); W: dtype [d,d] row-major,
 * O = O^s + O^l W.  Mc, luts: from sla_build_mask for the same params.
 * saved: saved_bytes (out) for sla_backward, or NULL for inference.
 * workspace: >= ws_forward_bytes. */
int sla_forward(const sla_params* p, const void* Q, const void* K, const void* V, const void* W,
                const int8_t* Mc, const void* luts, void* O, void* saved, void* workspace,
                size_t workspace_bytes, void* stream);

/* Algorithm 2, with dQ, dK scaled by 1/sqrt(d), dV accumulated over both branches, and the
 * chain rule through phi and W.  dO, dQ, dK, dV: dtype [B,H,N,d] (or [B,N,H,d]); dW: float [d,d] (out,
 * summed over batch, heads and tokens).  saved: as written by sla_forward with the same
 * inputs.  workspace: >= ws_backward_bytes. */
int sla_backward(const sla_params* p, const void* Q, const void* K, const void* V, const void* W,
                 const int8_t* Mc, const void* luts, const void* saved, const void* dO, void* dQ,
                 void* dK, void* dV, float* dW, void* workspace, size_t workspace_bytes,
                 void* stream);

/* Alg. 1's accumulation line on its own, by a chosen method:
 *   H_i = sum of h_j over the marginal key blocks j of query tile i,  Z_i likewise from z_j.
 * SLA_AGG_GEMM is what sla_forward and sla_backward use (a product with the 0/1 marginal
 * indicator on the matrix cores); the others are the forms the paper describes, kept for
 * comparison: SLA_AGG_ADD one addition per marginal block (Alg. 1 as written), SLA_AGG_PREAGG
 * the sum over all blocks minus the non-marginal ones and SLA_AGG_FOUR_RUSSIANS tabulated
 * subset sums of groups of four blocks (both Appendix A.3).
 * bf16 only (p->dtype == SLA_BF16).  h: bf16 [B,H,T,d*d + d] state rows (the matrix
 * transposed, then the vector, see "state row" above).  luts: from sla_build_mask or
 * sla_classify_scores for the same params.  outH: bf16 [B,H,T,d*d]; outZ: float [B,H,T,d].
 * workspace: >= the bytes sla_aggregate_ws_bytes reports for the method (may be NULL when
 * that is 0). */
enum { SLA_AGG_GEMM = 0, SLA_AGG_ADD = 1, SLA_AGG_PREAGG = 2, SLA_AGG_FOUR_RUSSIANS = 3 };
int sla_aggregate_ws_bytes(const sla_params* p, int method, uint64_t* bytes);
int sla_aggregate_states(const sla_params* p, int method, const void* luts, const void* h, void* outH,
                         float* outZ, void* workspace, size_t workspace_bytes, void* stream);

/* Optional per-kernel timing for benchmarks.  While enabled, each kernel the library
 * launches is bracketed by a pair of HIP events on the caller's stream.
 * sla_profile_read waits for the recorded events, writes one line "name count total_ms"
 * per kernel into buf (NUL-terminated) and forgets them.  Disabled by default. */
int sla_profile_enable(int on);
int sla_profile_read(char* buf, size_t buf_bytes);

/* Query blocks of 128 or 256 tokens (Section 2.1's b_q): with on != 0 the forward and the row-wise
 * backward kernel run one workgroup of eight waves per pair of adjacent 64-query tiles of a block,
 * which fetches each K_j, V_j tile into LDS once for both tiles.  Off by default: measured on the
 * headline shape the eight-wave kernels are 8 % (forward) to 15 % (dQ) slower than two four-wave
 * workgroups that share the tiles through the L2, at every density.  Process-wide; results are the
 * same either way up to rounding order.  Returns SLA_OK. */
int sla_wide_query_tiles(int on);

/* Measured matrix-core peak of the device at hand, for the benchmark's roofline: runs a
 * register-only loop of `iters` x 4 independent v_mfma_f32_32x32x16_bf16 per wave on every
 * compute unit (8 waves per SIMD), times it with HIP events on `stream`, WAITS for it, and writes
 * the sustained rate in TFLOP/s to *tflops (a host pointer).  iters in [1, 2^20]; 4096 runs about
 * 2 ms.  The nominal figure the roofline is priced against is 2500 (dense bf16). */
int sla_profile_mfma_peak(int iters, double* tflops, void* stream);

/* Measurement behind a design decision (dQ by a second, row-wise kernel that recomputes S and dP,
 * not by atomics from the column-wise kernel as Alg. 2's loop is written): issues exactly the
 * float atomic additions the fused form would make -- one workgroup per key block walks its column
 * list (luts from sla_build_mask for p) and adds a 64 x d tile of ones into acc (float [B,H,N,d],
 * device) per critical pair -- times the launch with HIP events on `stream`, WAITS for it and
 * writes the milliseconds to *ms (host).  acc ends up holding, per query row, its number of
 * critical key blocks (n_h) if it was zero before. */
int sla_profile_dq_atomics(const sla_params* p, const void* luts, float* acc, double* ms, void* stream);

/* Static description of an error code. */
const char* sla_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* SLA_H_ */
