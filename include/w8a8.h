/*
 * w8a8.h -- C ABI of the MI355X (gfx950) W8A8 Linear layer (part of libsla.so).
 *
 * The operation is the paper's Linear-layer quantisation (Section 1.1, fourth technique;
 * Section 1.3, "Linear layer quantization"): weights and activations are INT8, the
 * quantisation granularity of both is a block of 128 x 128, and the product runs on INT8
 * matrix units.  The paper gives no formula; this library takes the plain symmetric
 * block-wise scheme:
 *
 *   - a block of a matrix A[R, C] is rows 128 r .. 128 r + 127 x columns 128 c .. 128 c + 127
 *     (rows ragged at the end); its scale is s[r, c] = max|A_block| / 127 (1 if the block is
 *     all zero); its codes are rint(A_block / s[r, c]), ties to even, in [-127, 127];
 *   - for activations X[M, K] (tokens x input features), weights W[N, K] (output x input
 *     features) and kb running over the K / 128 feature blocks,
 *
 *         Y[m, n] = sum_kb sX[m / 128, kb] * sW[n / 128, kb] * sum_{k in kb} X8[m, k] W8[n, k]
 *                   (+ bias[n]),    rounded once to bf16 (nearest even);
 *
 *     the inner sums are exact (int32); the outer one is accumulated in fp32 by one fma per
 *     block that reads the integer accumulator as a float (offset by a constant of about
 *     2^23.4 integer steps, whose sign alternates from block to block and whose remainder is
 *     taken out at the end), so each block adds an error of at most 2 steps sX*sW of the
 *     largest block -- far below the rounding of the INT8 codes themselves, which is half a
 *     step per product term.
 *
 * General rules (as for sla.h)
 *   - Every tensor pointer is a DEVICE pointer owned by the caller.  x, w, y and bias are
 *     bf16, row-major and contiguous.
 *   - The library allocates nothing, frees nothing and never synchronises; all work is
 *     enqueued on `stream`.  Scratch lives in `workspace` (256-byte aligned, at least
 *     w8a8_workspace_bytes(...) bytes; contents undefined before and after a call).
 *   - Inputs are never written; outputs must not alias inputs, the weight object or the
 *     workspace.
 *   - Return value: SLA_OK (0) or a negative sla_status (sla.h); argument errors are found
 *     on the host before anything is launched.
 *   - Supported: K and N multiples of 128, 128 <= K <= 65536, 128 <= N <= 65536,
 *     1 <= M <= 2^22.
 */
#ifndef W8A8_H_
#define W8A8_H_

#include <stddef.h>
#include <stdint.h>

#include "sla.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Host-only.  Bytes of the quantised weight object of an [N, K] weight (codes in the order
 * the matrix units take them, then the block scales); 0 if N or K is not supported. */
size_t w8a8_weight_bytes(int N, int K);

/* Quantises a weight once (offline in the paper's flow).
 *   w    in   bf16 [N, K]
 *   wq   out  the weight object, w8a8_weight_bytes(N, K) bytes, 256-byte aligned; opaque:
 *             valid only for w8a8_linear_fwd / w8a8_debug_unpack of this library version */
int w8a8_quantize_weight(const void* w, int N, int K, void* wq, sla_stream_t stream);

/* Host-only.  Workspace bytes of w8a8_linear_fwd for M tokens of K features (the quantised
 * activations); 0 if the arguments are not supported. */
size_t w8a8_workspace_bytes(int M, int K);

/* y = W8A8-linear(x) as defined above: quantises x block-wise into the workspace, then runs
 * the INT8 product with the fp32 block-scale accumulation.
 *   x     in   bf16 [M, K]
 *   wq    in   weight object of an [N, K] weight (w8a8_quantize_weight)
 *   bias  in   bf16 [N]; NULL = none
 *   y     out  bf16 [M, N] */
int w8a8_linear_fwd(const void* x, const void* wq, const void* bias, void* y, int M, int N, int K,
                    void* workspace, size_t workspace_bytes, sla_stream_t stream);

/* The two halves of w8a8_linear_fwd, for callers that keep quantised activations (and for
 * timing the product alone): w8a8_quantize_act fills the workspace from x; w8a8_gemm_fwd
 * computes y from a workspace filled for the same M and K. */
int w8a8_quantize_act(const void* x, int M, int K, void* workspace, size_t workspace_bytes,
                      sla_stream_t stream);
int w8a8_gemm_fwd(const void* workspace, size_t workspace_bytes, const void* wq, const void* bias,
                  void* y, int M, int N, int K, sla_stream_t stream);

/* For tests: the codes and scales held by a weight object (R = N) or by a workspace filled
 * for R = M tokens, in plain layouts: codes int8 [R, K] row-major, scales fp32
 * [ceil(R / 128), K / 128] row-major.  Either output may be NULL.
 *   is_weight   non-zero: `q` is a weight object; zero: `q` is a filled workspace */
int w8a8_debug_unpack(const void* q, int is_weight, int R, int K, int8_t* codes, float* scales,
                      sla_stream_t stream);

#ifdef __cplusplus
}
#endif
#endif /* W8A8_H_ */
