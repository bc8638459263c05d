/*
 * sla_bwd.h -- C ABI of the backward pass of Sparse-Linear Attention on MI355X (gfx950),
 * part of libsla.so.
 *
 * The paper's training stage (Section 1.2) replaces full attention by SLA and finetunes the
 * model; inference (Section 1.3) then swaps in the low-bit core.  So the function that is
 * differentiated here is the UNQUANTISED SLA forward pass,
 *
 *     O = O^s + O^l W^T (+ b)
 *     O^s[n] = sum_{t in the critical key blocks of n's query block} softmax_t(Q[n].K[t]/sqrt(d)) V[t]
 *     O^l[n] = phi(Q[n]) H_i / (phi(Q[n]) . Z_i),   H_i = sum_{j marginal for i} phi(K_j)^T V_j,
 *                                                  Z_i = sum_{j marginal for i} sum_t phi(K_j[t]),
 *
 * with the block mask computed exactly as in sla_attention_fwd (pooled scores, Top-K) and held
 * fixed: it is piecewise constant in Q and K and passes no gradient.  The paper gives no
 * backward formula; the result is the gradient of the function above, computed in bf16 on the
 * matrix cores with fp32 accumulation (softmax statistics, delta = dO . O^s and the row
 * normalisers in fp32).
 *
 * Rules as in sla.h: every tensor pointer is a DEVICE pointer owned by the caller; the library
 * allocates nothing and never synchronises; work is enqueued on `stream`; scratch lives in
 * `workspace` (256-byte aligned, at least sla_bwd_workspace_bytes(...) bytes, contents undefined
 * before and after); inputs are never written; outputs must not alias inputs or the workspace.
 * Returns SLA_OK or a negative sla_status; argument errors are found on the host before any launch.
 * Supported: what sla_attention_fwd supports for shapes, blocks and ratios; contiguous [B,H,N,d]
 * tensors (other layouts: the _strided entry points below); any phi_kind of sla_phi (relu's gradient is taken as 0 at x <= 0).
 */
#ifndef SLA_BWD_H_
#define SLA_BWD_H_

#include <stddef.h>
#include <stdint.h>

#include "sla.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Host-only.  Workspace bytes of sla_attention_bwd; 0 if the arguments are not supported. */
size_t sla_bwd_workspace_bytes(int B, int H, int N, int d, int block_q, int block_k, double topk_ratio,
                               double marginal_ratio);

/* Gradients of the SLA forward pass defined above.
 *   q, k, v   in   bf16 [B,H,N,d]
 *   dout      in   bf16 [B,H,N,d]   gradient of the loss with respect to O
 *   proj_w    in   bf16 [d,d] (row = output channel) or NULL = identity, as in sla_attention_fwd
 *   dq,dk,dv  out  bf16 [B,H,N,d]
 *   dproj_w   out  fp32 [d,d]  sum over all (b,h,n) of dout[n]^T O^l[n]; NULL = not wanted.
 *                  Zero when there is no marginal block.
 *   dproj_b   out  fp32 [d]    sum over all (b,h,n) of dout[n] (the bias gradient); NULL = not
 *                  wanted.  Zero when there is no marginal block (the forward pass then adds no
 *                  bias).
 * Every output is deterministic: dproj_w and dproj_b are per-workgroup partial sums added in a
 * fixed order by a second kernel (no floating-point atomics anywhere).
 * With sla_profile_enable (sla.h) a call records the same number of stage events as a forward
 * call; the stages are: 0 block mask, 1 softmax statistics (lse, delta),
 * 2 linear branch and projection (summaries, dQ share, transposed accumulation, dK / dV shares),
 * 3 dQ, 4 dK and dV. */
int sla_attention_bwd(const void* q, const void* k, const void* v, const void* dout, const void* proj_w,
                      void* dq, void* dk, void* dv, float* dproj_w, float* dproj_b, int B, int H, int N, int d,
                      int block_q, int block_k, double topk_ratio, double marginal_ratio, int phi_kind,
                      void* workspace, size_t workspace_bytes, sla_stream_t stream);

/* ---- Handing the forward pass's statistics over (a training step: forward, then backward) ----
 *
 * sla_attention_fwd_train is sla_attention_fwd with SLA_QUANT_NONE (all
 * three feature maps) that also fills `saved` with what the backward pass would otherwise compute
 * again: every row's log-sum-exp over its critical keys and O^s.  sla_attention_bwd_saved is
 * sla_attention_bwd without its statistics pass: it takes them from `saved`, which must come from
 * sla_attention_fwd_train on the same q, k, v, sizes, blocks and ratios (delta = dO . O^s is then
 * formed from the bf16 O^s, a difference far below the tolerance of the result).
 *   saved   device, 256-byte aligned, sla_saved_bytes(...) bytes; opaque; written by the forward
 *           entry point, read by the backward one; NULL in sla_attention_bwd_saved = recompute
 *           (exactly sla_attention_bwd).  The buffer starts with a record of the problem it was
 *           filled for (B, H, N, block_q, critical blocks per row).  The backward pass checks it ON
 *           THE DEVICE (the host cannot read it without synchronising): a buffer that was not filled
 *           for the same problem makes every gradient NaN instead of plausibly wrong; the call
 *           itself still returns SLA_OK. */
size_t sla_saved_bytes(int B, int H, int N, int d, int block_q);

int sla_attention_fwd_train(const void* q, const void* k, const void* v, void* out, int B, int H, int N, int d,
                            int block_q, int block_k, double topk_ratio, double marginal_ratio, const void* proj_w,
                            const void* proj_b, int phi_kind, void* saved, size_t saved_bytes, void* workspace,
                            size_t workspace_bytes, sla_stream_t stream);

int sla_attention_bwd_saved(const void* q, const void* k, const void* v, const void* dout, const void* proj_w,
                            void* dq, void* dk, void* dv, float* dproj_w, float* dproj_b, int B, int H, int N, int d,
                            int block_q, int block_k, double topk_ratio, double marginal_ratio, int phi_kind,
                            const void* saved, size_t saved_bytes, void* workspace, size_t workspace_bytes,
                            sla_stream_t stream);

/* ---- Token-major and packed layouts (Section 1.3: the operator sits between a QKV projection and
 * an output projection that produce and consume token-major tensors; in training their gradients do
 * too) ----
 *
 * The same calls for tensors that are not [B,H,N,d]-contiguous; strides as in sla.h (sla_strides:
 * elements; channels contiguous; non-negative multiples of 8; token stride >= d; 16-byte aligned
 * bases; else SLA_ERR_LAYOUT).  NULL strides = contiguous.  Results are bit-identical to the
 * contiguous calls on the same values.  sla_attention_fwd_strided (sla.h) takes every quant_mode. */
int sla_attention_fwd_train_strided(const void* q, const void* k, const void* v, void* out,
                                    const sla_strides* q_strides, const sla_strides* k_strides,
                                    const sla_strides* v_strides, const sla_strides* out_strides,
                                    int B, int H, int N, int d, int block_q, int block_k,
                                    double topk_ratio, double marginal_ratio, const void* proj_w, const void* proj_b,
                                    int phi_kind, void* saved, size_t saved_bytes, void* workspace,
                                    size_t workspace_bytes, sla_stream_t stream);

/* One layout per tensor of the backward pass (HOST pointers, read during the call; any may be NULL
 * = contiguous). */
typedef struct {
  const sla_strides *q, *k, *v, *dout, *dq, *dk, *dv;
} sla_bwd_strides;

/* sla_attention_bwd_saved (saved == NULL: sla_attention_bwd) with a layout per tensor; strides ==
 * NULL: all contiguous.  Rows of dq, dk, dv must not overlap each other or any input (not checked). */
int sla_attention_bwd_strided(const void* q, const void* k, const void* v, const void* dout, const void* proj_w,
                              void* dq, void* dk, void* dv, float* dproj_w, float* dproj_b,
                              const sla_bwd_strides* strides, int B, int H, int N, int d, int block_q, int block_k,
                              double topk_ratio, double marginal_ratio, int phi_kind, const void* saved,
                              size_t saved_bytes, void* workspace, size_t workspace_bytes, sla_stream_t stream);

#ifdef __cplusplus
}
#endif
#endif /* SLA_BWD_H_ */
