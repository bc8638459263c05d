/*
 * sla.h -- C ABI of the MI355X (gfx950) Sparse-Linear Attention forward library.
 *
 * The operation is the attention operator of the paper's inference path
 * (Section 1.3: SLA computed by a low-bit kernel built on SageAttention;
 * Section 1.1: SageAttention2++-style 8-bit QK^T / PV plus Sparse-Linear
 * Attention; Section 2.1: Top-K ratio 0.1 = 90 % block sparsity).  For one
 * (batch, head) slice with N tokens split into consecutive blocks of block_q
 * queries / block_k keys (last block possibly short):
 *
 *   1. block means of Q and K, score s[i][j] = mean(Q_i).mean(K_j)/sqrt(d);
 *   2. per query block i: the n_c highest-scoring key blocks are CRITICAL (+1),
 *      the next n_m MARGINAL (0), the rest NEGLIGIBLE (-1); equal scores rank by
 *      ascending j;  n_c = min(Tk, max(1, floor(topk_ratio*Tk + 1e-9))),
 *      n_m = min(Tk - n_c, floor(marginal_ratio*Tk + 1e-9));
 *   3. sparse branch: softmax attention of the block's queries over the keys of
 *      its critical blocks, in one pass in ascending j.  K is smoothed (channel
 *      mean over all N tokens removed) and quantised to INT8 with one scale per
 *      key block, Q to INT8 with one scale per query block, V to FP8 E4M3 with
 *      one scale per channel: scale = max|.| / 127 (INT8) or / 448 (FP8), code =
 *      value / scale rounded to nearest with ties to even -- the quotient taken
 *      as 127 x / max (448 v / max), so that a 16-bit value lying exactly between
 *      two codes is rounded as the tie it is.  With t = log2(e) * (Q8.K8) dq dk / sqrt(d) the
 *      base-2 logit (the integer product is exact), each query keeps a reference
 *      level r, an INTEGER: after every run of 32 keys r = max(r, ceil(largest t
 *      of the run)).  The weights of the run are P = 448 * 2^(t - r), at most 448,
 *      rounded to E4M3 (nearest even); what was gathered before is scaled by the
 *      power of two 2^(r_old - r), exactly.  The P.V products accumulate in fp32,
 *      and the row sum is the sum of the ROUNDED weights, so numerator and
 *      denominator use the same numbers:  O_s = sum(P8 V8) dv / sum(P8).
 *      (Against the textbook form -- running maximum itself as the reference,
 *      one refresh per block, row sum of the unrounded weights -- only the points
 *      at which P is rounded move; without rounding the results coincide.)
 *   4. linear branch: with phi a per-token feature map (softmax over channels by
 *      default) on the ORIGINAL Q and K, O_l = phi(Q) H_i / (phi(Q).Z_i) where
 *      H_i = sum of phi(K_j)^T V_j and Z_i = sum of column sums of phi(K_j) over
 *      the marginal blocks j of i;
 *   5. out = O_s + O_l W^T (+ b), rounded to bf16 (nearest even); the linear term
 *      and the bias are absent when n_m == 0.
 *
 * General rules for every entry point
 *   - Every tensor pointer is a DEVICE pointer owned by the caller; `Tq`, `Tk`,
 *     `n_crit`, `n_marg` out-parameters of sla_block_counts are HOST pointers.
 *   - Layout: q, k, v, out are [B, H, N, d] contiguous, d fastest, bf16.
 *   - The library allocates nothing, frees nothing and never synchronises; all
 *     work is enqueued on `stream`.  Scratch lives in `workspace` (256-byte
 *     aligned, at least sla_workspace_bytes(...) bytes); its contents are
 *     undefined before and after a call.  Calls sharing a workspace must be
 *     stream-ordered.
 *   - Inputs are never written; outputs must not alias inputs or the workspace.
 *   - Return value: SLA_OK (0) or a negative sla_status.  Argument errors are
 *     found on the host before anything is launched (nothing is enqueued then).
 *     SLA_ERR_HIP reports a failed launch.  Nothing throws or aborts.
 *   - Supported: d == 128; block_k == 64; block_q in {64, 128}; 1 <= N with
 *     ceil(N/64) <= 8192; B*H*ceil(N/block_q) < 2^31; phi in sla_phi;
 *     quant_mode SLA_QUANT_QK_INT8_PV_FP8 (the paper's inference path),
 *     SLA_QUANT_NONE (bf16 products: the training-time operator that
 *     sla_bwd.h differentiates) or SLA_QUANT_QK_INT8 (see sla_quant).
 *   - Results are deterministic: no floating-point atomics anywhere (sla_bwd.h included).
 */
#ifndef SLA_H_
#define SLA_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ihipStream_t* sla_stream_t; /* a hipStream_t; NULL = the default stream */

typedef enum {
  SLA_OK = 0,
  SLA_ERR_NULL = -1,        /* a required pointer is NULL */
  SLA_ERR_SHAPE = -2,       /* B, H, N <= 0; d != 128; sizes beyond the stated limits */
  SLA_ERR_BLOCK = -3,       /* block_q not in {64,128} or block_k != 64 */
  SLA_ERR_RATIO = -4,       /* topk_ratio not in (0,1], marginal_ratio not in [0,1], or sum > 1 */
  SLA_ERR_WORKSPACE = -5,   /* workspace NULL, misaligned or too small */
  SLA_ERR_UNSUPPORTED = -6, /* phi_kind / quant_mode outside what this build implements */
  SLA_ERR_HIP = -7,         /* a kernel launch reported an error */
  SLA_ERR_LAYOUT = -8,      /* strides negative, not multiples of 8 elements, token stride < d, or a
                               base pointer not 16-byte aligned */
  SLA_ERR_STATIC_LIMIT = -9 /* sla_classify_blocks_static: the problem needs more than SLA_STATIC_SCRATCH_BYTES */
} sla_status;

typedef enum { SLA_PHI_SOFTMAX = 0, SLA_PHI_ELU1 = 1, SLA_PHI_RELU = 2 } sla_phi;

typedef enum {
  SLA_QUANT_NONE = 0,            /* bf16 products, fp32 accumulation and softmax: plain SLA (sla_attention_fwd only) */
  SLA_QUANT_QK_INT8 = 1,         /* scores from the INT8 codes of Q and of the smoothed K (integer products, exact), P and
                                    V in bf16: separates the INT8 error from the FP8 error (sla_attention_fwd only).  A
                                    diagnostic mode: the codes travel as bf16 numbers through the 16-bit matrix pipe, whose
                                    products and fp32 sums of such integers are exact, so the scores are bit for bit what
                                    an INT8 product gives */
  SLA_QUANT_QK_INT8_PV_FP8 = 2   /* INT8 QK^T with K-smoothing, FP8 E4M3 PV */
} sla_quant;

/* Library version: major*10000 + minor*100 + patch. */
int sla_version(void);

/* Static string for a status code (never NULL). */
const char* sla_status_string(int status);

/* Host-only.  Block grid and per-row counts (step 2 above).  Any out pointer may
 * be NULL.  Returns SLA_OK, SLA_ERR_SHAPE, SLA_ERR_BLOCK or SLA_ERR_RATIO. */
int sla_block_counts(int N, int block_q, int block_k, double topk_ratio, double marginal_ratio,
                     int* Tq, int* Tk, int* n_crit, int* n_marg);

/* Host-only.  Bytes of workspace that any entry point below needs for this
 * problem (one size serves all of them); 0 if the arguments are invalid. */
size_t sla_workspace_bytes(int B, int H, int N, int d, int block_q, int block_k,
                           double topk_ratio, double marginal_ratio, int quant_mode);

/* The whole forward pass, steps 1-5.
 *   q, k, v   in   bf16 [B,H,N,d]
 *   out       out  bf16 [B,H,N,d]
 *   proj_w    in   bf16 [d,d] row-major (out channel, in channel), shared by all
 *                  heads; NULL = identity
 *   proj_b    in   bf16 [d]; NULL = none */
int sla_attention_fwd(const void* q, const void* k, const void* v, void* out,
                      int B, int H, int N, int d, int block_q, int block_k,
                      double topk_ratio, double marginal_ratio,
                      const void* proj_w, const void* proj_b, int phi_kind, int quant_mode,
                      void* workspace, size_t workspace_bytes, sla_stream_t stream);

/* Where the tokens of a tensor indexed [b][h][n][channel] lie: element (b,h,n,c) is at
 * base + b*batch + h*head + n*token + c, in ELEMENTS; the d channels of a token are always
 * contiguous.  [B,H,N,d] is {H*N*d, N*d, d}; the layout a fused QKV projection leaves,
 * [B,N,H,d], is {N*H*d, d, H*d}; q of a packed [B,N,3,H,d] is {N*3*H*d, d, 3*H*d}. */
typedef struct {
  int64_t batch, head, token;
} sla_strides;

/* sla_attention_fwd for inputs and an output that are not [B,H,N,d]-contiguous (Section 1.3:
 * the kernel replaces the attention of a DiT block, which sits between a QKV projection and
 * an output projection that produce and consume token-major tensors; reading and writing
 * them in place saves three transposes in and one out).  Every argument is as in sla_attention_fwd; in addition
 *   q_strides, k_strides, v_strides, out_strides   in  HOST pointers, read during the call;
 *                  NULL = [B,H,N,d] contiguous.
 * Each stride must be a non-negative multiple of 8 elements with token >= d, and each base
 * pointer 16-byte aligned, else SLA_ERR_LAYOUT.  Rows of `out` must not overlap each other
 * or any input (not checked).  Results are bit-identical to the contiguous call on the
 * same values. */
int sla_attention_fwd_strided(const void* q, const void* k, const void* v, void* out,
                              const sla_strides* q_strides, const sla_strides* k_strides,
                              const sla_strides* v_strides, const sla_strides* out_strides,
                              int B, int H, int N, int d, int block_q, int block_k,
                              double topk_ratio, double marginal_ratio,
                              const void* proj_w, const void* proj_b, int phi_kind, int quant_mode,
                              void* workspace, size_t workspace_bytes, sla_stream_t stream);

/* The low-bit forward pass (SLA_QUANT_QK_INT8_PV_FP8) in two calls, for callers that want the K/V-side
 * work out of the way early -- e.g. enqueued as soon as the QKV projection has written q, k, v, while
 * other work of the block still runs (Section 1.3: the operator sits right behind that projection):
 *   sla_fwd_prepass   steps 1-2, the quantisation of K and V, the per-block linear summaries and their
 *                     sums over the marginal blocks: everything the attention kernel reads, left in
 *                     `workspace` (its contents are then DEFINED until the next call that uses it);
 *   sla_fwd_attend    the attention kernel with the fused linear term: reads q and the workspace a
 *                     sla_fwd_prepass call on the same q, sizes, blocks, ratios and phi_kind left,
 *                     writes out.  proj_w belongs to the first call, proj_b to the second.
 * Together they enqueue exactly the kernels of sla_attention_fwd_strided and give the same bits.
 * Strides as there (HOST pointers; NULL = [B,H,N,d] contiguous). */
int sla_fwd_prepass(const void* q, const void* k, const void* v, const sla_strides* q_strides,
                    const sla_strides* k_strides, const sla_strides* v_strides,
                    int B, int H, int N, int d, int block_q, int block_k,
                    double topk_ratio, double marginal_ratio, const void* proj_w, int phi_kind,
                    void* workspace, size_t workspace_bytes, sla_stream_t stream);
int sla_fwd_attend(const void* q, void* out, const sla_strides* q_strides, const sla_strides* out_strides,
                   int B, int H, int N, int d, int block_q, int block_k,
                   double topk_ratio, double marginal_ratio, const void* proj_b, int phi_kind,
                   void* workspace, size_t workspace_bytes, sla_stream_t stream);

/* Steps 1-2 alone.
 *   mask           out  int8  [B,H,Tq,Tk], values +1 / 0 / -1
 *   crit_idx       out  int32 [B,H,Tq,n_crit], ascending j          (may be NULL)
 *   marg_idx       out  int32 [B,H,Tq,n_marg], ascending j          (may be NULL)
 *   pooled_scores  out  fp32  [B,H,Tq,Tk], s[i][j]                  (may be NULL) */
int sla_classify_blocks(const void* q, const void* k, int B, int H, int N, int d,
                        int block_q, int block_k, double topk_ratio, double marginal_ratio,
                        int8_t* mask, int32_t* crit_idx, int32_t* marg_idx, float* pooled_scores,
                        void* workspace, size_t workspace_bytes, sla_stream_t stream);

/* sla_classify_blocks for callers that cannot allocate or hand over device memory beyond inputs and
 * outputs: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments and results (bit for bit) as sla_classify_blocks, minus the workspace: the block means,
 * the statistics and -- when pooled_scores is NULL -- the scores live in an array built into the
 * library, SLA_STATIC_SCRATCH_BYTES per GPU, held from the library's load until the process ends.
 * The call allocates and frees nothing and does not synchronise.  It needs
 *   256-byte-rounded  4 B H (Tq + Tk) d + 4 B H Tq + 4 B H d  (+ 4 B H Tq Tk if pooled_scores is NULL)
 * bytes (e.g. 37 MiB for H = 40, N = 32760, block_q = 128); a larger problem returns
 * SLA_ERR_STATIC_LIMIT and launches nothing.  Every call on a GPU uses that GPU's one array: calls
 * that may overlap on one GPU (different streams, different threads) race and must be ordered by
 * the caller.  Nothing in the array needs to survive between calls. */
#define SLA_STATIC_SCRATCH_BYTES (64u << 20)
int sla_classify_blocks_static(const void* q, const void* k, int B, int H, int N, int d,
                               int block_q, int block_k, double topk_ratio, double marginal_ratio,
                               int8_t* mask, int32_t* crit_idx, int32_t* marg_idx, float* pooled_scores,
                               sla_stream_t stream);

/* Step 3 alone, for a caller-supplied critical list.
 *   crit_idx  in   int32 [B,H,Tq,n_crit]; each row strictly ascending, entries in
 *                  [0,Tk) (not checked: out-of-range entries are undefined behaviour)
 *   out_s     out  fp32 [B,H,N,d]   O_s
 *   lse       out  fp32 [B,H,N]     log-sum-exp of each row's (smoothed, quantised)
 *                  logits over its critical keys, natural log    (may be NULL) */
int sla_sparse_attn_fwd(const void* q, const void* k, const void* v,
                        const int32_t* crit_idx, int n_crit, float* out_s, float* lse,
                        int B, int H, int N, int d, int block_q, int block_k, int quant_mode,
                        void* workspace, size_t workspace_bytes, sla_stream_t stream);

/* Step 4 and the projection of step 5 alone, for a caller-supplied block mask.
 *   mask   in   int8 [B,H,Tq,Tk]; blocks with value 0 are the marginal ones
 *   out_l  out  fp32 [B,H,N,d]   O_l W^T (+ b); zero rows where a query block
 *               has no marginal block */
int sla_linear_attn_fwd(const void* q, const void* k, const void* v, const int8_t* mask,
                        const void* proj_w, const void* proj_b, int phi_kind, float* out_l,
                        int B, int H, int N, int d, int block_q, int block_k,
                        void* workspace, size_t workspace_bytes, sla_stream_t stream);

/* Optional per-stage timing of sla_attention_fwd (for benchmarks; off by default).
 * The stages are: 0 pooling + statistics, 1 scores + block selection, 2 K/V
 * quantisation + linear summaries, 3 marginal-summary accumulation, 4 the fused
 * sparse attention kernel.
 *   sla_profile_enable(n): creates the HIP events (host objects, no device memory)
 *     for timing up to n calls; n <= 0 disables timing and destroys them.  While
 *     enabled, each sla_attention_fwd call records SLA_N_STAGES + 1 events on its
 *     stream (no synchronisation) until n calls have been recorded.
 *   sla_profile_reset(): forget the recorded calls (the next call is record 0).
 *   sla_profile_read(stage_ms, max_calls, n_calls): HOST pointers; waits for the
 *     recorded calls to finish and writes stage_ms[call][SLA_N_STAGES] in
 *     milliseconds and the number of calls read.
 * Not thread-safe: enable / reset / read must not overlap calls of sla_attention_fwd. */
#define SLA_N_STAGES 5
int sla_profile_enable(int max_calls);
int sla_profile_reset(void);
int sla_profile_read(float* stage_ms, int max_calls, int* n_calls);

/* Measurement aid (Section 1.1 names the INT8 and FP8 matrix units the method runs on; the
 * benchmark sets what a kernel achieves beside what those units sustain on the chip at hand):
 * enqueues a kernel in which every SIMD issues nothing but independent matrix products of one
 * kind -- kind 0: INT8 32x32x32, 1: FP8 32x32x64, 2: bf16 32x32x16 -- `iters` rounds of four
 * per wavefront, two workgroups of four wavefronts per compute unit, no memory traffic.
 * *ops (HOST pointer) receives the number of operations (2 per multiply-add) the launch
 * performs; the caller times the launch.  scratch: device memory of at least 2048 bytes per
 * compute unit (results nobody reads), else SLA_ERR_WORKSPACE; another kind: SLA_ERR_UNSUPPORTED;
 * iters < 1: SLA_ERR_SHAPE. */
int sla_calibrate_mfma(int kind, int iters, void* scratch, size_t scratch_bytes, double* ops, sla_stream_t stream);

/* Format check: converts n fp32 values (device) to FP8 E4M3 codes (device) with
 * the same instruction sequence the kernels use for P and V (round to nearest
 * even, saturating at +-448).  For tests of the number format only. */
int sla_debug_e4m3_encode(const float* in, uint8_t* out, size_t n, sla_stream_t stream);

/* Exposes the quantised operands the sparse branch consumes, in plain layouts,
 * for tests: K codes int8 [B,H,N,d], their per-block scales fp32 [B,H,Tk], the
 * channel mean fp32 [B,H,d], V codes (E4M3) uint8 [B,H,N,d] and per-channel scales
 * fp32 [B,H,d].  Any output may be NULL. */
int sla_debug_quantize_kv(const void* k, const void* v, int B, int H, int N, int d, int block_k,
                          int8_t* k_codes, float* k_scale, float* k_mean,
                          uint8_t* v_codes, float* v_scale,
                          void* workspace, size_t workspace_bytes, sla_stream_t stream);

/* The same for Q: its INT8 codes int8 [B,H,N,d] and the per-query-block scales fp32
 * [B,H,ceil(N/block_q)] (step 3: symmetric, scale = max|block| / 127, round to nearest, ties to the
 * even code).  Either output may be NULL. */
int sla_debug_quantize_q(const void* q, int B, int H, int N, int d, int block_q,
                         int8_t* q_codes, float* q_scale,
                         void* workspace, size_t workspace_bytes, sla_stream_t stream);

#ifdef __cplusplus
}
#endif
#endif /* SLA_H_ */
