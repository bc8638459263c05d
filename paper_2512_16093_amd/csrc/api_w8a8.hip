// C ABI of the W8A8 Linear layer: argument checking, the layout of the weight object and of
// the workspace, and the launch sequence.  See include/w8a8.h for the contract.
#pragma GCC visibility push(default)
#include "../../include/w8a8.h"
#pragma GCC visibility pop

#include "common.h"

namespace sla {
void launch_w8a8_quantize(const void* a, int R, int K, int RP, bool negate_odd, int8_t* codes, float* scales,
                          hipStream_t stream);
void launch_w8a8_unpack(const int8_t* frag, const float* s, int R, int K, int RP, bool negate_odd, int8_t* codes,
                        float* scales, hipStream_t stream);
void launch_w8a8_gemm(const int8_t* x8, const float* sx, int MP, const int8_t* w8, const float* sw,
                      const void* bias, void* y, int M, int N, int K, hipStream_t stream);
}  // namespace sla

using namespace sla;

namespace {

bool dims_ok(int R, int K, bool weight) {
  if (K < 128 || K > 65536 || (K & 127)) return false;
  if (weight) return R >= 128 && R <= 65536 && !(R & 127);
  return R >= 1 && R <= (1 << 22);
}
// activations are padded to whole 256-token tiles of the product, weights need no padding
int padded_rows(int R, bool weight) { return weight ? R : (R + 255) / 256 * 256; }
size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }
// a quantised matrix: codes in operand order, then the block scales
size_t codes_bytes(int RP, int K) { return align256((size_t)RP * K); }
size_t object_bytes(int RP, int K) { return codes_bytes(RP, K) + align256((size_t)(RP / 128) * (K / 128) * 4); }
int launch_status() { return hipGetLastError() == hipSuccess ? SLA_OK : SLA_ERR_HIP; }

}  // namespace

#pragma GCC visibility push(default)
extern "C" {

size_t w8a8_weight_bytes(int N, int K) { return dims_ok(N, K, true) ? object_bytes(N, K) : 0; }

size_t w8a8_workspace_bytes(int M, int K) { return dims_ok(M, K, false) ? object_bytes(padded_rows(M, false), K) : 0; }

int w8a8_quantize_weight(const void* w, int N, int K, void* wq, sla_stream_t stream) {
  if (!w || !wq) return SLA_ERR_NULL;
  if (!dims_ok(N, K, true)) return SLA_ERR_SHAPE;
  if ((uintptr_t)wq & 255) return SLA_ERR_WORKSPACE;
  launch_w8a8_quantize(w, N, K, N, true, (int8_t*)wq, (float*)((unsigned char*)wq + codes_bytes(N, K)), (hipStream_t)stream);
  return launch_status();
}

int w8a8_quantize_act(const void* x, int M, int K, void* workspace, size_t workspace_bytes, sla_stream_t stream) {
  if (!x) return SLA_ERR_NULL;
  if (!dims_ok(M, K, false)) return SLA_ERR_SHAPE;
  const int MP = padded_rows(M, false);
  if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < object_bytes(MP, K)) return SLA_ERR_WORKSPACE;
  launch_w8a8_quantize(x, M, K, MP, false, (int8_t*)workspace, (float*)((unsigned char*)workspace + codes_bytes(MP, K)),
                       (hipStream_t)stream);
  return launch_status();
}

int w8a8_gemm_fwd(const void* workspace, size_t workspace_bytes, const void* wq, const void* bias, void* y, int M,
                  int N, int K, sla_stream_t stream) {
  if (!wq || !y) return SLA_ERR_NULL;
  if (!dims_ok(M, K, false) || !dims_ok(N, K, true)) return SLA_ERR_SHAPE;
  const int MP = padded_rows(M, false);
  if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < object_bytes(MP, K)) return SLA_ERR_WORKSPACE;
  if ((uintptr_t)wq & 255) return SLA_ERR_WORKSPACE;
  if (((uintptr_t)y & 15) || (bias && ((uintptr_t)bias & 7))) return SLA_ERR_LAYOUT;
  launch_w8a8_gemm((const int8_t*)workspace, (const float*)((const unsigned char*)workspace + codes_bytes(MP, K)), MP,
                   (const int8_t*)wq, (const float*)((const unsigned char*)wq + codes_bytes(N, K)), bias, y, M, N, K,
                   (hipStream_t)stream);
  return launch_status();
}

int w8a8_linear_fwd(const void* x, const void* wq, const void* bias, void* y, int M, int N, int K, void* workspace,
                    size_t workspace_bytes, sla_stream_t stream) {
  if (!x || !wq || !y) return SLA_ERR_NULL;
  if (!dims_ok(M, K, false) || !dims_ok(N, K, true)) return SLA_ERR_SHAPE;
  int st = w8a8_quantize_act(x, M, K, workspace, workspace_bytes, stream);
  if (st != SLA_OK) return st;
  return w8a8_gemm_fwd(workspace, workspace_bytes, wq, bias, y, M, N, K, stream);
}

int w8a8_debug_unpack(const void* q, int is_weight, int R, int K, int8_t* codes, float* scales, sla_stream_t stream) {
  if (!q) return SLA_ERR_NULL;
  if (!dims_ok(R, K, is_weight != 0)) return SLA_ERR_SHAPE;
  const int RP = padded_rows(R, is_weight != 0);
  launch_w8a8_unpack((const int8_t*)q, (const float*)((const unsigned char*)q + codes_bytes(RP, K)), R, K, RP,
                     is_weight != 0, codes, scales, (hipStream_t)stream);
  return launch_status();
}

}  // extern "C"
#pragma GCC visibility pop
