// C ABI of the SLA forward library: argument checking, workspace carving and the
// launch sequence.  See include/sla.h for the contract of every entry point.
#pragma GCC visibility push(default)
#include "../../include/sla.h"
#include "../../include/sla_bwd.h"
#pragma GCC visibility pop

#include <math.h>

#include "common.h"

#include <mutex>

using namespace sla;

// Built-in scratch of sla_classify_blocks_static: one copy per GPU, held until the process ends.
// In host code this name is only a handle for hipGetSymbolAddress; the device address is looked
// up once per device (static_scratch_ptr) and that pointer is what the kernels receive.
static __device__ __align__(256) unsigned char scratch[SLA_STATIC_SCRATCH_BYTES];

namespace {

constexpr int MAX_DEVICES = 64;
void* g_scratch_ptr[MAX_DEVICES] = {};
std::mutex g_scratch_mutex;

// Device address of `scratch` on the current device (nullptr on any HIP error).
void* static_scratch_ptr() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return nullptr;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
    g_scratch_ptr[dev] = ptr;
  }
  return g_scratch_ptr[dev];
}

// Scratch of the block classification alone: block means, the statistics pass's by-products, scores.
struct ClassifyScratch {
  size_t qbar, kbar, dq, amax_v, scores, total;
};
ClassifyScratch make_classify_scratch(const Problem& p, bool own_scores) {
  ClassifyScratch c;
  size_t o = 0;
  auto take = [&](size_t bytes) { size_t r = o; o = align256(o + bytes); return r; };
  c.qbar = take((size_t)p.BH * p.Tq * D * 4);
  c.kbar = take((size_t)p.BH * p.Tk * D * 4);
  c.dq = take((size_t)p.BH * p.Tq * 4);
  c.amax_v = take((size_t)p.BH * D * 4);
  c.scores = take(own_scores ? (size_t)p.BH * p.Tq * p.Tk * 4 : 0);
  c.total = o;
  return c;
}

int count_blocks(int N, int block_q, int block_k, double rc, double rm, int* Tq, int* Tk, int* nc,
                 int* nm) {
  if (N <= 0) return SLA_ERR_SHAPE;
  if ((block_q != 64 && block_q != 128) || block_k != BK) return SLA_ERR_BLOCK;
  if (!(rc > 0.0) || rc > 1.0 || !(rm >= 0.0) || rm > 1.0 || rc + rm > 1.0 + 1e-9) return SLA_ERR_RATIO;
  const long long tq = ((long long)N + block_q - 1) / block_q, tk = ((long long)N + block_k - 1) / block_k;
  if (tk > 8192) return SLA_ERR_SHAPE;
  long long c = (long long)floor(rc * (double)tk + 1e-9);
  if (c < 1) c = 1;
  if (c > tk) c = tk;
  long long m = (long long)floor(rm * (double)tk + 1e-9);
  if (m > tk - c) m = tk - c;
  if (Tq) *Tq = (int)tq;
  if (Tk) *Tk = (int)tk;
  if (nc) *nc = (int)c;
  if (nm) *nm = (int)m;
  return SLA_OK;
}

// Shape / block / ratio checks shared by every device entry point.
int make_problem(int B, int H, int N, int d, int block_q, int block_k, double rc, double rm, Problem* p) {
  if (B <= 0 || H <= 0 || N <= 0 || d != D) return SLA_ERR_SHAPE;
  int Tq, Tk, nc, nm;
  const int st = count_blocks(N, block_q, block_k, rc, rm, &Tq, &Tk, &nc, &nm);
  if (st != SLA_OK) return st;
  const long long rows = (long long)B * H * Tq;
  if ((long long)B * H > 65535 || rows >= (1ll << 31) - 8 || (long long)B * H * Tk >= (1ll << 31)) return SLA_ERR_SHAPE;
  p->B = B; p->H = H; p->N = N; p->block_q = block_q;
  p->BH = B * H; p->Tq = Tq; p->Tk = Tk; p->n_c = nc; p->n_m = nm;
  p->lq = p->lk = p->lv = p->lo = p->ld = p->ldq = p->ldk = p->ldv = contiguous_layout(H, N);
  return SLA_OK;
}

// A caller-given layout: rows of d contiguous channels, 16-byte aligned, at non-negative strides.
int make_layout(const void* base, const sla_strides* st, int H, int N, Layout* L) {
  if (!st) {
    *L = contiguous_layout(H, N);
    return SLA_OK;
  }
  if (st->batch < 0 || st->head < 0 || st->token < D) return SLA_ERR_LAYOUT;
  if ((st->batch | st->head | st->token) & 7) return SLA_ERR_LAYOUT;
  if ((uintptr_t)base & 15) return SLA_ERR_LAYOUT;
  L->sb = st->batch; L->sh = st->head; L->sn = st->token;
  return SLA_OK;
}

int check_ws(const void* ws, size_t bytes, size_t need) {
  if (!ws || ((uintptr_t)ws & 255) || bytes < need) return SLA_ERR_WORKSPACE;
  return SLA_OK;
}

int launch_status() { return hipGetLastError() == hipSuccess ? SLA_OK : SLA_ERR_HIP; }

// Optional stage timing of sla_attention_fwd: SLA_N_STAGES + 1 events per recorded call,
// created by sla_profile_enable and recorded on the call's stream between the stages.
struct Profiler {
  hipEvent_t* ev = nullptr;
  int capacity = 0, used = 0;
} g_prof;

inline void mark(hipStream_t s, int rec, int idx) {
  if (rec >= 0) (void)hipEventRecord(g_prof.ev[rec * (SLA_N_STAGES + 1) + idx], s);
}

template <class T>
T* at(void* ws, size_t off) { return (T*)((unsigned char*)ws + off); }

// The forward entry points' workspace (one size serves all of them): with room for the INT8 codes of Q,
// whole groups of 128 rows per (b,h).
size_t q8_rows(const Problem& p) { return (size_t)((p.N + 127) / 128) * 128; }
Workspace fwd_workspace(const Problem& p, size_t n_c, size_t n_m, size_t code_tensor_elems = 0) {
  return make_workspace(p.BH, p.Tq, p.Tk, n_c, n_m, code_tensor_elems, q8_rows(p));
}

void run_stats(const void* q, const void* k, const void* v, const void* proj_w, const Problem& p, void* ws,
               const Workspace& W, hipStream_t s, bool want_q8 = false) {
  launch_pool_stats(q, k, v, p, at<float>(ws, W.qbar), at<float>(ws, W.kbar), at<float>(ws, W.dq),
                    at<uint32_t>(ws, W.amax_v), want_q8 ? at<int8_t>(ws, W.q8) : nullptr, s);
  launch_finalize_stats(p, at<float>(ws, W.kbar), at<uint32_t>(ws, W.amax_v), at<float>(ws, W.mu_k),
                        at<float>(ws, W.dv), (const bf16_t*)proj_w, at<bf16_t>(ws, W.wfrag), s);
}

// The unquantised forward pass (bf16 products): the launch sequence of sla_attention_fwd with
// SLA_QUANT_NONE; save_lse2 / save_os, if given, receive what a backward pass can reuse.
// With codes16 (SLA_QUANT_QK_INT8) the scores are the integer products of the INT8 codes of Q and of the
// smoothed K: the codes travel as bf16 numbers, whose products and fp32 sums are exact, through the same
// kernel; P and V stay 16-bit.
int fwd_bf16(const void* q, const void* k, const void* v, void* out, const Problem& p, const void* proj_w,
             const void* proj_b, int phi_kind, void* ws, const Workspace& W, hipStream_t s, int rec, float* save_lse2,
             void* save_os, bool codes16 = false) {
  const bool lin = p.n_m > 0;
  mark(s, rec, 0);
  run_stats(q, k, v, proj_w, p, ws, W, s, codes16);
  mark(s, rec, 1);
  launch_scores(p, at<float>(ws, W.qbar), at<float>(ws, W.kbar), at<float>(ws, W.scores), s);
  launch_select(p, at<float>(ws, W.scores), nullptr, at<int32_t>(ws, W.crit), nullptr,
                lin ? at<uint32_t>(ws, W.m0) : nullptr, s);
  mark(s, rec, 2);
  if (lin || codes16)
    launch_prep_kv(k, v, p, at<float>(ws, W.mu_k), at<uint32_t>(ws, W.amax_v), at<bf16_t>(ws, W.wfrag), phi_kind, codes16, lin,
                   at<int8_t>(ws, W.k8), at<uint8_t>(ws, W.v8), at<float>(ws, W.dk), at<bf16_t>(ws, W.hz), s);
  if (codes16)
    launch_code_tensors(p, at<int8_t>(ws, W.q8), at<int8_t>(ws, W.k8), at<bf16_t>(ws, W.qc), at<bf16_t>(ws, W.kc), s);
  mark(s, rec, 3);
  if (lin) launch_lin_accumulate(p, at<uint32_t>(ws, W.m0), at<bf16_t>(ws, W.hz), at<bf16_t>(ws, W.HZ), s);
  mark(s, rec, 4);
  const CodeScales cs{at<float>(ws, W.dq), at<float>(ws, W.dk), q};
  if (launch_fwd_bf16(p, codes16 ? at<bf16_t>(ws, W.qc) : q, codes16 ? at<bf16_t>(ws, W.kc) : k, v, at<int32_t>(ws, W.crit),
                      lin ? at<bf16_t>(ws, W.HZ) : nullptr, (const bf16_t*)proj_b, phi_kind, out, save_lse2, save_os,
                      codes16 ? &cs : nullptr, s) != 0)
    return SLA_ERR_HIP;
  mark(s, rec, 5);
  return launch_status();
}

// The low-bit forward pass in two parts.  run_prepass: statistics, block classification, K/V quantisation with
// the linear summaries, marginal accumulation -- everything the attention kernel reads from the workspace.
// run_attend: the attention kernel with the fused linear epilogue.
void run_prepass(const void* q, const void* k, const void* v, const void* proj_w, const Problem& p, int phi_kind,
                 void* ws, const Workspace& W, hipStream_t s, int rec) {
  const bool lin = p.n_m > 0;
  mark(s, rec, 0);
  run_stats(q, k, v, proj_w, p, ws, W, s, true);
  mark(s, rec, 1);
  launch_scores(p, at<float>(ws, W.qbar), at<float>(ws, W.kbar), at<float>(ws, W.scores), s);
  launch_select(p, at<float>(ws, W.scores), nullptr, at<int32_t>(ws, W.crit), nullptr,
                lin ? at<uint32_t>(ws, W.m0) : nullptr, s);
  mark(s, rec, 2);
  launch_prep_kv(k, v, p, at<float>(ws, W.mu_k), at<uint32_t>(ws, W.amax_v), at<bf16_t>(ws, W.wfrag), phi_kind, true, lin,
                 at<int8_t>(ws, W.k8), at<uint8_t>(ws, W.v8), at<float>(ws, W.dk), at<bf16_t>(ws, W.hz), s);
  mark(s, rec, 3);
  if (lin) launch_lin_accumulate(p, at<uint32_t>(ws, W.m0), at<bf16_t>(ws, W.hz), at<bf16_t>(ws, W.HZ), s);
  mark(s, rec, 4);
}

void run_attend(const void* q, void* out, const void* proj_b, const Problem& p, int phi_kind, void* ws,
                const Workspace& W, hipStream_t s) {
  launch_sparse_fwd(q, at<int8_t>(ws, W.q8), p, at<int32_t>(ws, W.crit), p.n_c, at<int8_t>(ws, W.k8), at<uint8_t>(ws, W.v8),
                    at<float>(ws, W.dq), at<float>(ws, W.dk), at<float>(ws, W.dv), at<bf16_t>(ws, W.HZ),
                    (const bf16_t*)proj_b, phi_kind, p.n_m > 0, out, false, nullptr, at<int32_t>(ws, W.pair_list),
                    at<int32_t>(ws, W.pair_len), s);
}

// What sla_attention_fwd_train hands to sla_attention_bwd_saved: a header naming the problem the state
// belongs to (SavedHeader; checked on the device by the backward pass, which cannot read it on the host
// without synchronising), the rows' base-2 log-sum-exp (fp32, padded to whole query blocks), then O^s
// (bf16 [BH, N, D]).
struct SavedState {
  size_t hdr, lse2, os, total;
};
SavedState make_saved(const Problem& p) {
  SavedState v;
  v.hdr = 0;
  v.lse2 = 256;
  v.os = v.lse2 + align256((size_t)p.BH * p.Tq * p.block_q * 4);
  v.total = v.os + align256((size_t)p.BH * p.N * D * 2);
  return v;
}
SavedHeader saved_header(const Problem& p) {
  return SavedHeader{SAVED_MAGIC, p.B, p.H, p.N, p.block_q, p.n_c, 0, 0};
}

// Scratch of the backward pass, laid out after the forward pass's workspace map.
struct BwdWorkspace {
  size_t lse2, delta;        // fp32 [BH, 32 T32q]
  size_t dql;                // fp32 [BH, N, D]: the linear branch's share of dQ
  size_t dHZ;                // bf16 [BH, Tq, HZ_ROWS, D]: per query block dH^T and dZ
  size_t mbits_t;            // transposed marginal bit matrix
  size_t wt;                 // bf16 [D, D]: W^T
  size_t dw_part;            // fp32 per-workgroup partial sums of dW and db (bwd_lin_q_partial_bytes)
  size_t total;
};

BwdWorkspace make_bwd_workspace(const Problem& p, const Workspace& W) {
  BwdWorkspace b;
  size_t o = W.total;
  auto take = [&](size_t bytes) { size_t r = o; o = align256(o + bytes); return r; };
  const size_t BH = p.BH, T32q = (size_t)p.Tq * (p.block_q / 32);
  b.lse2 = take(BH * T32q * 32 * 4); b.delta = take(BH * T32q * 32 * 4);
  const bool lin = p.n_m > 0;
  const size_t grad = lin ? BH * (size_t)p.N * D * 4 : 0;
  b.dql = take(grad);
  b.dHZ = take(lin ? BH * (size_t)p.Tq * HZ_ELEMS * 2 : 0);
  b.mbits_t = take(lin ? marginal_bits_t_bytes(p) : 0);
  b.wt = take(D * D * 2);
  b.dw_part = take(lin ? bwd_lin_q_partial_bytes(p) : 0);
  b.total = o;
  return b;
}

}  // namespace

#pragma GCC visibility push(default)
extern "C" {

int sla_version(void) { return 100; }

const char* sla_status_string(int status) {
  switch (status) {
    case SLA_OK: return "ok";
    case SLA_ERR_NULL: return "a required pointer is NULL";
    case SLA_ERR_SHAPE: return "unsupported shape (need B,H,N > 0, d == 128, sizes within limits)";
    case SLA_ERR_BLOCK: return "unsupported block size (block_q in {64,128}, block_k == 64)";
    case SLA_ERR_RATIO: return "ratios out of range (0 < topk <= 1, 0 <= marginal <= 1, sum <= 1)";
    case SLA_ERR_WORKSPACE: return "workspace NULL, not 256-byte aligned, or too small";
    case SLA_ERR_UNSUPPORTED: return "phi_kind or quant_mode not implemented";
    case SLA_ERR_HIP: return "a kernel launch failed";
    case SLA_ERR_STATIC_LIMIT: return "problem needs more scratch than the built-in SLA_STATIC_SCRATCH_BYTES";
    case SLA_ERR_LAYOUT: return "unsupported strides (non-negative multiples of 8 elements, token stride >= d, 16-byte aligned base)";
    default: return "unknown status";
  }
}

int sla_block_counts(int N, int block_q, int block_k, double topk_ratio, double marginal_ratio, int* Tq,
                     int* Tk, int* n_crit, int* n_marg) {
  return count_blocks(N, block_q, block_k, topk_ratio, marginal_ratio, Tq, Tk, n_crit, n_marg);
}

size_t sla_workspace_bytes(int B, int H, int N, int d, int block_q, int block_k, double topk_ratio,
                           double marginal_ratio, int quant_mode) {
  Problem p;
  if (quant_mode < SLA_QUANT_NONE || quant_mode > SLA_QUANT_QK_INT8_PV_FP8) return 0;
  if (make_problem(B, H, N, d, block_q, block_k, topk_ratio, marginal_ratio, &p) != SLA_OK) return 0;
  // (sized by the given ratios; SLA_QUANT_QK_INT8 adds the two 16-bit code tensors)
  return fwd_workspace(p, p.n_c, p.n_m, quant_mode == SLA_QUANT_QK_INT8 ? (size_t)p.BH * p.N * D : 0).total;
}

int sla_attention_fwd(const void* q, const void* k, const void* v, void* out, int B, int H, int N, int d,
                      int block_q, int block_k, double topk_ratio, double marginal_ratio,
                      const void* proj_w, const void* proj_b, int phi_kind, int quant_mode, void* workspace,
                      size_t workspace_bytes, sla_stream_t stream) {
  return sla_attention_fwd_strided(q, k, v, out, nullptr, nullptr, nullptr, nullptr, B, H, N, d, block_q, block_k,
                                   topk_ratio, marginal_ratio, proj_w, proj_b, phi_kind, quant_mode, workspace,
                                   workspace_bytes, stream);
}

int sla_attention_fwd_strided(const void* q, const void* k, const void* v, void* out,
                              const sla_strides* q_strides, const sla_strides* k_strides,
                              const sla_strides* v_strides, const sla_strides* out_strides, int B, int H, int N,
                              int d, int block_q, int block_k, double topk_ratio, double marginal_ratio,
                              const void* proj_w, const void* proj_b, int phi_kind, int quant_mode,
                              void* workspace, size_t workspace_bytes, sla_stream_t stream) {
  if (!q || !k || !v || !out) return SLA_ERR_NULL;
  Problem p;
  int st = make_problem(B, H, N, d, block_q, block_k, topk_ratio, marginal_ratio, &p);
  if (st != SLA_OK) return st;
  if ((st = make_layout(q, q_strides, H, N, &p.lq)) != SLA_OK) return st;
  if ((st = make_layout(k, k_strides, H, N, &p.lk)) != SLA_OK) return st;
  if ((st = make_layout(v, v_strides, H, N, &p.lv)) != SLA_OK) return st;
  if ((st = make_layout(out, out_strides, H, N, &p.lo)) != SLA_OK) return st;
  if (phi_kind < SLA_PHI_SOFTMAX || phi_kind > SLA_PHI_RELU) return SLA_ERR_UNSUPPORTED;
  if (quant_mode < SLA_QUANT_NONE || quant_mode > SLA_QUANT_QK_INT8_PV_FP8) return SLA_ERR_UNSUPPORTED;
  const Workspace W = fwd_workspace(p, p.n_c, p.n_m, quant_mode == SLA_QUANT_QK_INT8 ? (size_t)p.BH * p.N * D : 0);
  if ((st = check_ws(workspace, workspace_bytes, W.total)) != SLA_OK) return st;
  hipStream_t s = (hipStream_t)stream;
  const int rec = (g_prof.ev && g_prof.used < g_prof.capacity) ? g_prof.used++ : -1;
  if (quant_mode != SLA_QUANT_QK_INT8_PV_FP8)
    return fwd_bf16(q, k, v, out, p, proj_w, proj_b, phi_kind, workspace, W, s, rec, nullptr, nullptr,
                    quant_mode == SLA_QUANT_QK_INT8);
  run_prepass(q, k, v, proj_w, p, phi_kind, workspace, W, s, rec);
  run_attend(q, out, proj_b, p, phi_kind, workspace, W, s);
  mark(s, rec, 5);
  return launch_status();
}

int sla_fwd_prepass(const void* q, const void* k, const void* v, const sla_strides* q_strides,
                    const sla_strides* k_strides, const sla_strides* v_strides, int B, int H, int N, int d,
                    int block_q, int block_k, double topk_ratio, double marginal_ratio, const void* proj_w,
                    int phi_kind, void* workspace, size_t workspace_bytes, sla_stream_t stream) {
  if (!q || !k || !v) return SLA_ERR_NULL;
  Problem p;
  int st = make_problem(B, H, N, d, block_q, block_k, topk_ratio, marginal_ratio, &p);
  if (st != SLA_OK) return st;
  if ((st = make_layout(q, q_strides, H, N, &p.lq)) != SLA_OK) return st;
  if ((st = make_layout(k, k_strides, H, N, &p.lk)) != SLA_OK) return st;
  if ((st = make_layout(v, v_strides, H, N, &p.lv)) != SLA_OK) return st;
  if (phi_kind < SLA_PHI_SOFTMAX || phi_kind > SLA_PHI_RELU) return SLA_ERR_UNSUPPORTED;
  const Workspace W = fwd_workspace(p, p.n_c, p.n_m);
  if ((st = check_ws(workspace, workspace_bytes, W.total)) != SLA_OK) return st;
  run_prepass(q, k, v, proj_w, p, phi_kind, workspace, W, (hipStream_t)stream, -1);
  return launch_status();
}

int sla_fwd_attend(const void* q, void* out, const sla_strides* q_strides, const sla_strides* out_strides, int B,
                   int H, int N, int d, int block_q, int block_k, double topk_ratio, double marginal_ratio,
                   const void* proj_b, int phi_kind, void* workspace, size_t workspace_bytes, sla_stream_t stream) {
  if (!q || !out) return SLA_ERR_NULL;
  Problem p;
  int st = make_problem(B, H, N, d, block_q, block_k, topk_ratio, marginal_ratio, &p);
  if (st != SLA_OK) return st;
  if ((st = make_layout(q, q_strides, H, N, &p.lq)) != SLA_OK) return st;
  if ((st = make_layout(out, out_strides, H, N, &p.lo)) != SLA_OK) return st;
  if (phi_kind < SLA_PHI_SOFTMAX || phi_kind > SLA_PHI_RELU) return SLA_ERR_UNSUPPORTED;
  const Workspace W = fwd_workspace(p, p.n_c, p.n_m);
  if ((st = check_ws(workspace, workspace_bytes, W.total)) != SLA_OK) return st;
  run_attend(q, out, proj_b, p, phi_kind, workspace, W, (hipStream_t)stream);
  return launch_status();
}

int sla_profile_enable(int max_calls) {
  if (g_prof.ev) {
    for (int i = 0; i < g_prof.capacity * (SLA_N_STAGES + 1); ++i) (void)hipEventDestroy(g_prof.ev[i]);
    delete[] g_prof.ev;
    g_prof = Profiler();
  }
  if (max_calls <= 0) return SLA_OK;
  const int n = max_calls * (SLA_N_STAGES + 1);
  g_prof.ev = new hipEvent_t[n];
  for (int i = 0; i < n; ++i) {
    if (hipEventCreate(&g_prof.ev[i]) != hipSuccess) return SLA_ERR_HIP;
  }
  g_prof.capacity = max_calls;
  return SLA_OK;
}

int sla_profile_reset(void) {
  g_prof.used = 0;
  return SLA_OK;
}

int sla_profile_read(float* stage_ms, int max_calls, int* n_calls) {
  if (!stage_ms || !n_calls) return SLA_ERR_NULL;
  const int n = g_prof.used < max_calls ? g_prof.used : max_calls;
  for (int r = 0; r < n; ++r) {
    hipEvent_t* e = g_prof.ev + r * (SLA_N_STAGES + 1);
    if (hipEventSynchronize(e[SLA_N_STAGES]) != hipSuccess) return SLA_ERR_HIP;
    for (int st = 0; st < SLA_N_STAGES; ++st) {
      if (hipEventElapsedTime(&stage_ms[r * SLA_N_STAGES + st], e[st], e[st + 1]) != hipSuccess) return SLA_ERR_HIP;
    }
  }
  *n_calls = n;
  return SLA_OK;
}

int sla_classify_blocks(const void* q, const void* k, int B, int H, int N, int d, int block_q, int block_k,
                        double topk_ratio, double marginal_ratio, int8_t* mask, int32_t* crit_idx,
                        int32_t* marg_idx, float* pooled_scores, void* workspace, size_t workspace_bytes,
                        sla_stream_t stream) {
  if (!q || !k || !mask) return SLA_ERR_NULL;
  Problem p;
  int st = make_problem(B, H, N, d, block_q, block_k, topk_ratio, marginal_ratio, &p);
  if (st != SLA_OK) return st;
  const Workspace W = fwd_workspace(p, p.n_c, p.n_m);
  if ((st = check_ws(workspace, workspace_bytes, W.total)) != SLA_OK) return st;
  hipStream_t s = (hipStream_t)stream;
  void* ws = workspace;
  // V is not an input here: the statistics pass reads K in its place (its V outputs are unused)
  launch_pool_stats(q, k, k, p, at<float>(ws, W.qbar), at<float>(ws, W.kbar), at<float>(ws, W.dq),
                    at<uint32_t>(ws, W.amax_v), nullptr, s);
  float* sc = pooled_scores ? pooled_scores : at<float>(ws, W.scores);
  launch_scores(p, at<float>(ws, W.qbar), at<float>(ws, W.kbar), sc, s);
  launch_select(p, sc, mask, crit_idx, p.n_m > 0 ? marg_idx : nullptr, nullptr, s);
  return launch_status();
}

int sla_classify_blocks_static(const void* q, const void* k, int B, int H, int N, int d, int block_q, int block_k,
                               double topk_ratio, double marginal_ratio, int8_t* mask, int32_t* crit_idx,
                               int32_t* marg_idx, float* pooled_scores, sla_stream_t stream) {
  if (!q || !k || !mask) return SLA_ERR_NULL;
  Problem p;
  const int st = make_problem(B, H, N, d, block_q, block_k, topk_ratio, marginal_ratio, &p);
  if (st != SLA_OK) return st;
  const ClassifyScratch C = make_classify_scratch(p, pooled_scores == nullptr);
  if (C.total > (size_t)SLA_STATIC_SCRATCH_BYTES) return SLA_ERR_STATIC_LIMIT;
  void* ws = static_scratch_ptr();
  if (!ws) return SLA_ERR_HIP;
  hipStream_t s = (hipStream_t)stream;
  // the same kernels as sla_classify_blocks; the statistics pass zeroes what it accumulates into
  launch_pool_stats(q, k, k, p, at<float>(ws, C.qbar), at<float>(ws, C.kbar), at<float>(ws, C.dq),
                    at<uint32_t>(ws, C.amax_v), nullptr, s);
  float* sc = pooled_scores ? pooled_scores : at<float>(ws, C.scores);
  launch_scores(p, at<float>(ws, C.qbar), at<float>(ws, C.kbar), sc, s);
  launch_select(p, sc, mask, crit_idx, p.n_m > 0 ? marg_idx : nullptr, nullptr, s);
  return launch_status();
}

int sla_sparse_attn_fwd(const void* q, const void* k, const void* v, const int32_t* crit_idx, int n_crit,
                        float* out_s, float* lse, int B, int H, int N, int d, int block_q, int block_k,
                        int quant_mode, void* workspace, size_t workspace_bytes, sla_stream_t stream) {
  if (!q || !k || !v || !crit_idx || !out_s) return SLA_ERR_NULL;
  Problem p;
  int st = make_problem(B, H, N, d, block_q, block_k, 1.0, 0.0, &p);
  if (st != SLA_OK) return st;
  if (n_crit < 1 || n_crit > p.Tk) return SLA_ERR_SHAPE;
  if (quant_mode != SLA_QUANT_QK_INT8_PV_FP8) return SLA_ERR_UNSUPPORTED;
  // the internal index lists are not used here, so the smallest workspace that
  // sla_workspace_bytes can return for this shape is enough
  const Workspace Wmin = fwd_workspace(p, 1, 0);
  if ((st = check_ws(workspace, workspace_bytes, Wmin.total)) != SLA_OK) return st;
  hipStream_t s = (hipStream_t)stream;
  void* ws = workspace;
  run_stats(q, k, v, nullptr, p, ws, Wmin, s, true);
  launch_prep_kv(k, v, p, at<float>(ws, Wmin.mu_k), at<uint32_t>(ws, Wmin.amax_v), at<bf16_t>(ws, Wmin.wfrag), 0, true,
                 false, at<int8_t>(ws, Wmin.k8), at<uint8_t>(ws, Wmin.v8), at<float>(ws, Wmin.dk), nullptr, s);
  launch_sparse_fwd(q, at<int8_t>(ws, Wmin.q8), p, crit_idx, n_crit, at<int8_t>(ws, Wmin.k8), at<uint8_t>(ws, Wmin.v8),
                    at<float>(ws, Wmin.dq), at<float>(ws, Wmin.dk), at<float>(ws, Wmin.dv), nullptr, nullptr, 0,
                    false, out_s, true, lse, nullptr, nullptr, s);
  return launch_status();
}

int sla_linear_attn_fwd(const void* q, const void* k, const void* v, const int8_t* mask, const void* proj_w,
                        const void* proj_b, int phi_kind, float* out_l, int B, int H, int N, int d,
                        int block_q, int block_k, void* workspace, size_t workspace_bytes,
                        sla_stream_t stream) {
  if (!q || !k || !v || !mask || !out_l) return SLA_ERR_NULL;
  Problem p;
  int st = make_problem(B, H, N, d, block_q, block_k, 1.0, 0.0, &p);
  if (st != SLA_OK) return st;
  if (phi_kind < SLA_PHI_SOFTMAX || phi_kind > SLA_PHI_RELU) return SLA_ERR_UNSUPPORTED;
  const Workspace W = fwd_workspace(p, 1, 0);
  if ((st = check_ws(workspace, workspace_bytes, W.total)) != SLA_OK) return st;
  hipStream_t s = (hipStream_t)stream;
  void* ws = workspace;
  run_stats(q, k, v, proj_w, p, ws, W, s, true);
  launch_prep_kv(k, v, p, at<float>(ws, W.mu_k), at<uint32_t>(ws, W.amax_v), at<bf16_t>(ws, W.wfrag), phi_kind, false, true, nullptr,
                 nullptr, nullptr, at<bf16_t>(ws, W.hz), s);
  launch_marginal_bits(p, mask, at<uint32_t>(ws, W.m0), s);
  launch_lin_accumulate(p, at<uint32_t>(ws, W.m0), at<bf16_t>(ws, W.hz), at<bf16_t>(ws, W.HZ), s);
  // the attention kernel with an empty critical list leaves only the linear term
  launch_sparse_fwd(q, at<int8_t>(ws, W.q8), p, nullptr, 0, at<int8_t>(ws, W.k8), at<uint8_t>(ws, W.v8), at<float>(ws, W.dq),
                    at<float>(ws, W.dk), at<float>(ws, W.dv), at<bf16_t>(ws, W.HZ), (const bf16_t*)proj_b,
                    phi_kind, true, out_l, true, nullptr, nullptr, nullptr, s);
  return launch_status();
}

int sla_debug_e4m3_encode(const float* in, uint8_t* out, size_t n, sla_stream_t stream) {
  if (!in || !out) return SLA_ERR_NULL;
  launch_e4m3_encode(in, out, n, (hipStream_t)stream);
  return launch_status();
}

int sla_calibrate_mfma(int kind, int iters, void* scratch, size_t scratch_bytes, double* ops, sla_stream_t stream) {
  if (!scratch || !ops) return SLA_ERR_NULL;
  if (kind < 0 || kind > 2) return SLA_ERR_UNSUPPORTED;
  if (iters < 1) return SLA_ERR_SHAPE;
  int dev = 0, n_cu = 0;
  if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n_cu <= 0)
    return SLA_ERR_HIP;
  if (scratch_bytes < (size_t)2 * n_cu * 256 * sizeof(float)) return SLA_ERR_WORKSPACE;
  *ops = launch_mfma_rate(kind, iters, n_cu, (float*)scratch, (hipStream_t)stream);
  return launch_status();
}

int sla_debug_quantize_kv(const void* k, const void* v, int B, int H, int N, int d, int block_k,
                          int8_t* k_codes, float* k_scale, float* k_mean, uint8_t* v_codes, float* v_scale,
                          void* workspace, size_t workspace_bytes, sla_stream_t stream) {
  if (!k || !v) return SLA_ERR_NULL;
  Problem p;
  int st = make_problem(B, H, N, d, 64, block_k, 1.0, 0.0, &p);
  if (st != SLA_OK) return st;
  const Workspace W = fwd_workspace(p, 1, 0);
  if ((st = check_ws(workspace, workspace_bytes, W.total)) != SLA_OK) return st;
  hipStream_t s = (hipStream_t)stream;
  void* ws = workspace;
  run_stats(k, k, v, nullptr, p, ws, W, s);
  launch_prep_kv(k, v, p, at<float>(ws, W.mu_k), at<uint32_t>(ws, W.amax_v), at<bf16_t>(ws, W.wfrag), 0, true, false,
                 at<int8_t>(ws, W.k8), at<uint8_t>(ws, W.v8), at<float>(ws, W.dk), nullptr, s);
  launch_unfragment_kv(p, at<int8_t>(ws, W.k8), at<uint8_t>(ws, W.v8), k_codes, v_codes, s);
  const size_t bhd = (size_t)p.BH * D * 4;
  if (k_scale && hipMemcpyAsync(k_scale, at<float>(ws, W.dk), (size_t)p.BH * p.Tk * 4, hipMemcpyDeviceToDevice, s) != hipSuccess) return SLA_ERR_HIP;
  if (k_mean && hipMemcpyAsync(k_mean, at<float>(ws, W.mu_k), bhd, hipMemcpyDeviceToDevice, s) != hipSuccess) return SLA_ERR_HIP;
  if (v_scale && hipMemcpyAsync(v_scale, at<float>(ws, W.dv), bhd, hipMemcpyDeviceToDevice, s) != hipSuccess) return SLA_ERR_HIP;
  return launch_status();
}

int sla_debug_quantize_q(const void* q, int B, int H, int N, int d, int block_q, int8_t* q_codes, float* q_scale,
                         void* workspace, size_t workspace_bytes, sla_stream_t stream) {
  if (!q) return SLA_ERR_NULL;
  Problem p;
  int st = make_problem(B, H, N, d, block_q, BK, 1.0, 0.0, &p);
  if (st != SLA_OK) return st;
  const Workspace W = fwd_workspace(p, 1, 0);
  if ((st = check_ws(workspace, workspace_bytes, W.total)) != SLA_OK) return st;
  hipStream_t s = (hipStream_t)stream;
  void* ws = workspace;
  launch_pool_stats(q, q, q, p, at<float>(ws, W.qbar), at<float>(ws, W.kbar), at<float>(ws, W.dq),
                    at<uint32_t>(ws, W.amax_v), at<int8_t>(ws, W.q8), s);
  if (q_codes) launch_unpack_q8(p, at<int8_t>(ws, W.q8), q_codes, s);
  if (q_scale && hipMemcpyAsync(q_scale, at<float>(ws, W.dq), (size_t)p.BH * p.Tq * 4, hipMemcpyDeviceToDevice, s) != hipSuccess) return SLA_ERR_HIP;
  return launch_status();
}

size_t sla_bwd_workspace_bytes(int B, int H, int N, int d, int block_q, int block_k, double topk_ratio,
                               double marginal_ratio) {
  Problem p;
  if (make_problem(B, H, N, d, block_q, block_k, topk_ratio, marginal_ratio, &p) != SLA_OK) return 0;
  return make_bwd_workspace(p, make_workspace(p.BH, p.Tq, p.Tk, p.n_c, p.n_m)).total;
}

size_t sla_saved_bytes(int B, int H, int N, int d, int block_q) {
  Problem p;
  if (make_problem(B, H, N, d, block_q, BK, 1.0, 0.0, &p) != SLA_OK) return 0;
  return make_saved(p).total;
}

int sla_attention_fwd_train(const void* q, const void* k, const void* v, void* out, int B, int H, int N, int d,
                            int block_q, int block_k, double topk_ratio, double marginal_ratio, const void* proj_w,
                            const void* proj_b, int phi_kind, void* saved, size_t saved_bytes, void* workspace,
                            size_t workspace_bytes, sla_stream_t stream) {
  return sla_attention_fwd_train_strided(q, k, v, out, nullptr, nullptr, nullptr, nullptr, B, H, N, d, block_q, block_k,
                                         topk_ratio, marginal_ratio, proj_w, proj_b, phi_kind, saved, saved_bytes,
                                         workspace, workspace_bytes, stream);
}

int sla_attention_fwd_train_strided(const void* q, const void* k, const void* v, void* out, const sla_strides* q_strides,
                                    const sla_strides* k_strides, const sla_strides* v_strides,
                                    const sla_strides* out_strides, int B, int H, int N, int d, int block_q, int block_k,
                                    double topk_ratio, double marginal_ratio, const void* proj_w, const void* proj_b,
                                    int phi_kind, void* saved, size_t saved_bytes, void* workspace,
                                    size_t workspace_bytes, sla_stream_t stream) {
  if (!q || !k || !v || !out || !saved) return SLA_ERR_NULL;
  Problem p;
  int st = make_problem(B, H, N, d, block_q, block_k, topk_ratio, marginal_ratio, &p);
  if (st != SLA_OK) return st;
  if ((st = make_layout(q, q_strides, H, N, &p.lq)) != SLA_OK) return st;
  if ((st = make_layout(k, k_strides, H, N, &p.lk)) != SLA_OK) return st;
  if ((st = make_layout(v, v_strides, H, N, &p.lv)) != SLA_OK) return st;
  if ((st = make_layout(out, out_strides, H, N, &p.lo)) != SLA_OK) return st;
  if (phi_kind < SLA_PHI_SOFTMAX || phi_kind > SLA_PHI_RELU) return SLA_ERR_UNSUPPORTED;
  const Workspace W = make_workspace(p.BH, p.Tq, p.Tk, p.n_c, p.n_m);
  if ((st = check_ws(workspace, workspace_bytes, W.total)) != SLA_OK) return st;
  const SavedState V = make_saved(p);
  if ((st = check_ws(saved, saved_bytes, V.total)) != SLA_OK) return st;
  const int rec = (g_prof.ev && g_prof.used < g_prof.capacity) ? g_prof.used++ : -1;
  launch_write_saved_header(saved_header(p), at<SavedHeader>(saved, V.hdr), (hipStream_t)stream);
  return fwd_bf16(q, k, v, out, p, proj_w, proj_b, phi_kind, workspace, W, (hipStream_t)stream, rec,
                  at<float>(saved, V.lse2), at<bf16_t>(saved, V.os));
}

int sla_attention_bwd(const void* q, const void* k, const void* v, const void* dout, const void* proj_w,
                      void* dq, void* dk, void* dv, float* dproj_w, float* dproj_b, int B, int H, int N, int d,
                      int block_q, int block_k, double topk_ratio, double marginal_ratio, int phi_kind,
                      void* workspace, size_t workspace_bytes, sla_stream_t stream) {
  return sla_attention_bwd_strided(q, k, v, dout, proj_w, dq, dk, dv, dproj_w, dproj_b, nullptr, B, H, N, d, block_q,
                                   block_k, topk_ratio, marginal_ratio, phi_kind, nullptr, 0, workspace, workspace_bytes,
                                   stream);
}

int sla_attention_bwd_saved(const void* q, const void* k, const void* v, const void* dout, const void* proj_w,
                            void* dq, void* dk, void* dv, float* dproj_w, float* dproj_b, int B, int H, int N, int d,
                            int block_q, int block_k, double topk_ratio, double marginal_ratio, int phi_kind,
                            const void* saved, size_t saved_bytes, void* workspace, size_t workspace_bytes,
                            sla_stream_t stream) {
  return sla_attention_bwd_strided(q, k, v, dout, proj_w, dq, dk, dv, dproj_w, dproj_b, nullptr, B, H, N, d, block_q,
                                   block_k, topk_ratio, marginal_ratio, phi_kind, saved, saved_bytes, workspace,
                                   workspace_bytes, stream);
}

int sla_attention_bwd_strided(const void* q, const void* k, const void* v, const void* dout, const void* proj_w,
                              void* dq, void* dk, void* dv, float* dproj_w, float* dproj_b,
                              const sla_bwd_strides* strides, int B, int H, int N, int d, int block_q, int block_k,
                              double topk_ratio, double marginal_ratio, int phi_kind, const void* saved,
                              size_t saved_bytes, void* workspace, size_t workspace_bytes, sla_stream_t stream) {
  if (!q || !k || !v || !dout || !dq || !dk || !dv) return SLA_ERR_NULL;
  Problem p;
  int st = make_problem(B, H, N, d, block_q, block_k, topk_ratio, marginal_ratio, &p);
  if (st != SLA_OK) return st;
  if (strides) {
    if ((st = make_layout(q, strides->q, H, N, &p.lq)) != SLA_OK) return st;
    if ((st = make_layout(k, strides->k, H, N, &p.lk)) != SLA_OK) return st;
    if ((st = make_layout(v, strides->v, H, N, &p.lv)) != SLA_OK) return st;
    if ((st = make_layout(dout, strides->dout, H, N, &p.ld)) != SLA_OK) return st;
    if ((st = make_layout(dq, strides->dq, H, N, &p.ldq)) != SLA_OK) return st;
    if ((st = make_layout(dk, strides->dk, H, N, &p.ldk)) != SLA_OK) return st;
    if ((st = make_layout(dv, strides->dv, H, N, &p.ldv)) != SLA_OK) return st;
  }
  if (phi_kind < SLA_PHI_SOFTMAX || phi_kind > SLA_PHI_RELU) return SLA_ERR_UNSUPPORTED;
  const SavedState V = make_saved(p);
  if (saved && (st = check_ws(saved, saved_bytes, V.total)) != SLA_OK) return st;
  const Workspace W = make_workspace(p.BH, p.Tq, p.Tk, p.n_c, p.n_m);
  const BwdWorkspace X = make_bwd_workspace(p, W);
  if ((st = check_ws(workspace, workspace_bytes, X.total)) != SLA_OK) return st;
  hipStream_t s = (hipStream_t)stream;
  void* ws = workspace;
  const bool lin = p.n_m > 0;
  const int rec = (g_prof.ev && g_prof.used < g_prof.capacity) ? g_prof.used++ : -1;
  mark(s, rec, 0);

  // the block mask, exactly as the forward pass finds it
  run_stats(q, k, v, nullptr, p, ws, W, s);   // (no projection folded into the summaries here)
  launch_scores(p, at<float>(ws, W.qbar), at<float>(ws, W.kbar), at<float>(ws, W.scores), s);
  launch_select(p, at<float>(ws, W.scores), at<int8_t>(ws, W.mask), at<int32_t>(ws, W.crit), nullptr,
                lin ? at<uint32_t>(ws, W.m0) : nullptr, s);
  mark(s, rec, 1);
  const float* lse2 = at<float>(ws, X.lse2);
  if (saved) {  // the forward pass's statistics: only delta = dO . O^s is left to do
    launch_bwd_delta(p, dout, (const unsigned char*)saved + V.os, (const SavedHeader*)((const unsigned char*)saved + V.hdr),
                     saved_header(p), (const float*)((const unsigned char*)saved + V.lse2), at<float>(ws, X.lse2),
                     at<float>(ws, X.delta), s);
  } else {
    if (launch_bwd_stats(p, q, k, v, dout, at<int32_t>(ws, W.crit), at<float>(ws, X.lse2), at<float>(ws, X.delta), s) != 0)
      return SLA_ERR_HIP;
  }
  mark(s, rec, 2);
  // (with no marginal block there is no linear term: the projection and the bias receive no gradient)
  if (dproj_w && !lin) launch_zero_u32((uint32_t*)dproj_w, (size_t)D * D, s);
  if (dproj_b && !lin) launch_zero_u32((uint32_t*)dproj_b, (size_t)D, s);
  if (lin) {
    // H_i, Z_i of the forward pass (unprojected), then the linear branch's gradients
    launch_prep_kv(k, v, p, at<float>(ws, W.mu_k), at<uint32_t>(ws, W.amax_v), at<bf16_t>(ws, W.wfrag), phi_kind, false, true,
                   at<int8_t>(ws, W.k8), at<uint8_t>(ws, W.v8), at<float>(ws, W.dk), at<bf16_t>(ws, W.hz), s);
    launch_lin_accumulate(p, at<uint32_t>(ws, W.m0), at<bf16_t>(ws, W.hz), at<bf16_t>(ws, W.HZ), s);
    launch_bwd_wt((const bf16_t*)proj_w, at<bf16_t>(ws, X.wt), s);
    if (launch_bwd_lin_q(p, q, dout, at<bf16_t>(ws, W.HZ), at<bf16_t>(ws, X.wt), phi_kind, at<float>(ws, X.dql),
                         at<bf16_t>(ws, X.dHZ), dproj_w, dproj_b, at<float>(ws, X.dw_part), s) != 0)
      return SLA_ERR_HIP;
    // G_j = sum of dH_i over the query blocks that hold key block j as marginal: the forward's
    // accumulation kernel on the transposed mask (its output reuses the per-key-block summaries' buffer)
    Problem pt = p;
    pt.Tq = p.Tk;
    pt.Tk = p.Tq;
    launch_marginal_bits_t(p, at<int8_t>(ws, W.mask), at<uint32_t>(ws, X.mbits_t), s);
    launch_lin_accumulate(pt, at<uint32_t>(ws, X.mbits_t), at<bf16_t>(ws, X.dHZ), at<bf16_t>(ws, W.hz), s);
  }
  mark(s, rec, 3);
  if (launch_bwd_dq(p, q, dout, k, v, at<int32_t>(ws, W.crit), lse2, at<float>(ws, X.delta),
                    lin ? at<float>(ws, X.dql) : nullptr, dq, s) != 0)
    return SLA_ERR_HIP;
  mark(s, rec, 4);
  if (launch_bwd_dkv(p, q, dout, k, v, at<int8_t>(ws, W.mask), lse2, at<float>(ws, X.delta),
                     lin ? at<bf16_t>(ws, W.hz) : nullptr, phi_kind, dk, dv, s) != 0)
    return SLA_ERR_HIP;
  mark(s, rec, 5);
  return launch_status();
}

}  // extern "C"
#pragma GCC visibility pop
