// Shared device helpers and the workspace map for the SLA forward kernels (gfx950).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sla {

constexpr int D = 128;          // head dimension (fixed)
constexpr int BK = 64;          // key block size (fixed)
constexpr int HZ_ROWS = D + 1;  // per key block: 128 rows of h'^T plus the z row
constexpr int HZ_ELEMS = HZ_ROWS * D;
constexpr int KV_FRAG_BYTES = BK * D;  // 8 KiB of INT8 K codes / FP8 V codes per key block
constexpr float E4M3_MAX = 448.0f;
constexpr float LOG2_448 = 8.807354922057604f;
constexpr float LOG2E = 1.4426950408889634f;

// The linear branch's feature maps in the element-wise form the backward kernels use
// (PHI = SLA_PHI_SOFTMAX 0: softmax over the channels, given the row's maximum mx and 1 / sum;
// 1: elu(x) + 1;  2: relu; for these two mx is unused and scale is 1, or 0 for a row that does not exist).
template <int PHI>
__device__ __forceinline__ float phi_value(float x, float mx, float scale) {
  if constexpr (PHI == 0) return __builtin_amdgcn_exp2f((x - mx) * LOG2E) * scale;
  else if constexpr (PHI == 1) return (x > 0.f ? x + 1.0f : __builtin_amdgcn_exp2f(x * LOG2E)) * scale;
  else return fmaxf(x, 0.f) * scale;
}
// d loss / d x from a = phi(x), d = d loss / d phi(x) and -- softmax only -- sdot = sum over the row of a d.
template <int PHI>
__device__ __forceinline__ float phi_backward(float x, float a, float d, float sdot) {
  if constexpr (PHI == 0) return a * (d - sdot);
  else if constexpr (PHI == 1) return x > 0.f ? d : a * d;   // (x <= 0: phi = exp(x) = its own derivative)
  else return x > 0.f ? d : 0.f;
}
constexpr float LN2 = 0.6931471805599453f;

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef unsigned short bf16_t;  // raw bfloat16 bits

__device__ __forceinline__ float bf16_to_f32(bf16_t b) { return __uint_as_float(((uint32_t)b) << 16); }
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// fp32 -> bf16 bits, round to nearest even (NaN stays NaN): the hardware conversion
// v_cvt_pk_bf16_f32, two values per instruction.
typedef __bf16 v2bf __attribute__((ext_vector_type(2)));
typedef float v2f __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v2f{lo, hi}, v2bf));
}
__device__ __forceinline__ bf16_t f32_to_bf16(float f) { return (bf16_t)(pack_bf16x2(f, 0.f) & 0xffffu); }

// Two fp32 -> two E4M3 codes packed into the low or high half of `old`.  The
// hardware conversion rounds to nearest even and turns anything above 464 into
// NaN, so callers keep |x| <= 448 (clamp_e4m3) first.
__device__ __forceinline__ float clamp_e4m3(float x) { return __builtin_fminf(__builtin_fmaxf(x, -E4M3_MAX), E4M3_MAX); }
__device__ __forceinline__ int cvt_pk_e4m3(float a, float b, int old, bool hi) {
  return hi ? __builtin_amdgcn_cvt_pk_fp8_f32(a, b, old, true) : __builtin_amdgcn_cvt_pk_fp8_f32(a, b, old, false);
}

// INT8 code of x at the scale amax / 127, as the low byte (two's complement) of the returned word: the correctly
// rounded quotient 127 x / amax (the product 127 x is exact for a 16-bit x; the reciprocal's estimate takes one
// correction step whose residual the fma forms exactly), rounded to the nearest integer, ties to even, by adding
// 1.5 * 2^23.  A value that lies exactly half way between two codes so reaches the rounding as the tie it is --
// multiplying by a rounded reciprocal of the scale instead would let that reciprocal's last bit decide such
// values, and 16-bit inputs make them common (x = amax / 2 is one).  |x| <= amax, so no clamp is needed.
// The caller passes the block's maximum through code_scale() once: amax brought into the range where its
// reciprocal is finite (a power-of-two factor `up`, exact, for maxima below 2^-100: 16-bit inputs reach down to
// 2^-133), that reciprocal (0 if amax is 0: all codes 0), and k = 127 * up (448 * up for the FP8 quotient).
struct CodeScale { float amax, ramax, k; };
__device__ __forceinline__ CodeScale code_scale(float amax, float levels) {
  const float up = amax < 0x1p-100f ? 0x1p64f : 1.0f;
  const float a = amax * up;
  return CodeScale{a, a > 0.f ? 1.0f / a : 0.f, levels * up};
}
// levels * x / amax, correctly rounded (exact where the quotient is representable: ties stay ties).
__device__ __forceinline__ float exact_quotient(float x, const CodeScale& cs) {
  const float y = x * cs.k;
  const float t0 = y * cs.ramax;
  const float r = __builtin_fmaf(-t0, cs.amax, y);
  return __builtin_fmaf(r, cs.ramax, t0);
}
__device__ __forceinline__ uint32_t int8_code_word_exact(float x, const CodeScale& cs) {
  return __float_as_uint(exact_quotient(x, cs) + 12582912.0f);
}
// Where channel c's code sits in a row of the Q code tensor: the 64 bytes a lane half of the attention kernel
// takes as its B operands are contiguous (lane half hf holds channels 32 s + 16 hf + 0..15 of step s = 0..3).
__host__ __device__ inline int q8_byte_offset(int c) { return 64 * ((c >> 4) & 1) + 16 * (c >> 5) + (c & 15); }
// The low bytes of four such words, first in the lowest byte.
__device__ __forceinline__ uint32_t pack_low_bytes(uint32_t b0, uint32_t b1, uint32_t b2, uint32_t b3) {
  return __builtin_amdgcn_perm(__builtin_amdgcn_perm(b3, b2, 0x0c0c0400u), __builtin_amdgcn_perm(b1, b0, 0x0c0c0400u),
                               0x05040100u);
}

// Value held by the partner lane (lane ^ 32) of a 64-wide wavefront.
__device__ __forceinline__ float partner_f32(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_int(x), __float_as_int(x), false, false);
  // lanes < 32: r[1] is the upper half's value; lanes >= 32: r[0] is the lower half's value
  return __int_as_float((threadIdx.x & 32) ? r[0] : r[1]);
}
__device__ __forceinline__ int partner_i32(int x) {
  auto r = __builtin_amdgcn_permlane32_swap(x, x, false, false);
  return (threadIdx.x & 32) ? r[0] : r[1];
}

// ---------------------------------------------------------------------------
// Fragment order of the quantised K / V tiles (one 8 KiB record per key block).
//
// K record: 16-byte chunks indexed [t][s][lane], t = key tile (32 keys), s = step
// of 32 channels, lane = (key % 32) + 32*hf; the chunk holds channels
// 32*s + 16*hf + (0..15) of key 32*t + (lane % 32).  A wavefront reading chunk
// [t][s][its lane] gets the A operand of v_mfma_i32_32x32x32_i8.
__device__ __forceinline__ int kfrag_offset(int key, int ch) {
  int t = key >> 5, s = ch >> 5, hf = (ch >> 4) & 1;
  return (((t * 4 + s) * 64) + (key & 31) + 32 * hf) * 16 + (ch & 15);
}
// V record: 16-byte chunks indexed [ct][half][lane], ct = channel tile (32
// channels), lane = (ch % 32) + 32*hf; byte e of the chunk is key slot
// u = 16*half + e of that lane, and slot u of lane-half hf is key
// 32*(u/16) + 8*((u%16)/4) + 4*hf + (u%4) -- the order in which the score
// accumulators of v_mfma_i32_32x32x32_i8 sit in a lane, so the FP8 P codes can be
// used as the B operand of v_mfma_f32_32x32x64_f8f6f4 without any shuffle.
__device__ __forceinline__ int vfrag_offset(int key, int ch) {
  int t = key >> 5, g = (key >> 3) & 3, hf = (key >> 2) & 1, cc = key & 3;
  int u = 16 * t + 4 * g + cc;
  return ((((ch >> 5) * 2 + (u >> 4)) * 64) + (ch & 31) + 32 * hf) * 16 + (u & 15);
}

// ---------------------------------------------------------------------------
// Workspace map (all offsets 256-byte aligned).
struct Workspace {
  size_t qbar, kbar;        // fp32 [BH,Tq,D], [BH,Tk,D] block means
  size_t dq;                // fp32 [BH,Tq]  per-query-block INT8 scale
  size_t q8;                // int8 [BH, ceil(N/128)*128, D]: codes of Q, a row's 128 bytes in q8_byte_offset order
  size_t mu_k, amax_v, dv;  // fp32 [BH,D]   channel mean of K, max|V| (as uint bits), V scale
  size_t dk;                // fp32 [BH,Tk]  per-key-block INT8 scale
  size_t scores;            // fp32 [BH,Tq,Tk]
  size_t mask;              // int8 [BH,Tq,Tk]
  size_t m0;                // uint32 marginal bit matrix [BH, ceil(Tk/32), Tq rounded up to 384, + 128]: bit e of word (kt, i) = block 32 kt + e marginal for query block i
  size_t crit, marg;        // int32 [BH,Tq,n_c], [BH,Tq,n_m]
  size_t pair_list, pair_len;  // query blocks of 64: merged critical lists of adjacent pairs, int32 [BH,ceil(Tq/2),2 n_c], and their lengths
  size_t k8, v8;            // [BH,Tk] records of KV_FRAG_BYTES
  size_t hz;                // bf16 [BH,Tk,HZ_ROWS,D]
  size_t HZ;                // bf16 [BH,Tq,HZ_ROWS,D]
  size_t wfrag;             // bf16 [D,D]: the projection (identity if none) in the operand order of prep_kv
  size_t qc, kc;            // bf16 [BH,N,D]: INT8 codes of Q and K as bf16 numbers (SLA_QUANT_QK_INT8 only)
  size_t total;
};

inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

inline Workspace make_workspace(size_t BH, size_t Tq, size_t Tk, size_t n_c, size_t n_m, size_t code_tensor_elems = 0,
                                size_t q8_rows = 0) {
  Workspace w;
  size_t o = 0;
  auto take = [&](size_t bytes) { size_t r = o; o = align256(o + bytes); return r; };
  w.qbar = take(BH * Tq * D * 4);
  w.kbar = take(BH * Tk * D * 4);
  w.dq = take(BH * Tq * 4);
  w.q8 = take(BH * q8_rows * D);
  w.mu_k = take(BH * D * 4);
  w.amax_v = take(BH * D * 4);
  w.dv = take(BH * D * 4);
  w.dk = take(BH * Tk * 4);
  w.scores = take(BH * Tq * Tk * 4);
  w.mask = take(BH * Tq * Tk);
  w.m0 = take(BH * ((Tk + 31) / 32) * ((Tq + 383) / 384 * 384 + 128) * 4);
  w.crit = take(BH * Tq * n_c * 4);
  w.pair_list = take(BH * ((Tq + 1) / 2) * 2 * n_c * 4);
  w.pair_len = take(BH * ((Tq + 1) / 2) * 4);
  w.marg = take(BH * Tq * (n_m ? n_m : 1) * 4);
  w.k8 = take(BH * Tk * KV_FRAG_BYTES);
  w.v8 = take(BH * Tk * KV_FRAG_BYTES);
  w.hz = take(BH * Tk * HZ_ELEMS * 2);
  w.HZ = take(BH * Tq * HZ_ELEMS * 2);
  w.wfrag = take(D * D * 2);
  w.qc = take(code_tensor_elems * 2);
  w.kc = take(code_tensor_elems * 2);
  w.total = o;
  return w;
}

// Problem description handed to the launchers.
// Where the d contiguous channels of token n of slice (b,h) of a [B,H,N,d]-indexed bf16 tensor
// start, in elements: b * sb + h * sh + n * sn.  Any layout with contiguous channels fits
// ([B,H,N,d]: sn = d; [B,N,H,d]: sh = d, sn = H d; a packed [B,N,3,H,d]: sn = 3 H d).
struct Layout {
  long long sb, sh, sn;
};
inline Layout contiguous_layout(int H, int N) {
  return {(long long)H * N * D, (long long)N * D, (long long)D};
}

// Order of the 128 x 128 part of a block summary (h'^T, entry [o][c]) in hz and HZ: 16-byte chunk
// hz_frag_chunk(ot, ks, lane) holds row o = 32 ot + lane % 32, channels
// 32 (ks / 2) + 16 (lane / 32) + 8 (ks % 2) + 0..7 -- what lane `lane` feeds to
// v_mfma_f32_32x32x16_bf16 as the A operand for output tile ot and contraction step ks.  The z
// row follows at element 128 * 128, plain.
__host__ __device__ inline int hz_frag_chunk(int ot, int ks, int lane) { return (ot * 8 + ks) * 64 + lane; }

struct Problem {
  int B, H, N, block_q;
  int BH, Tq, Tk, n_c, n_m;
  Layout lq, lk, lv, lo;  // of q, k, v and out
  Layout ld, ldq, ldk, ldv;  // backward pass: of dout, dq, dk and dv
};

// Launchers (one per kernel file); every one only enqueues work on `stream`.
void launch_pool_stats(const void* q, const void* k, const void* v, const Problem& p, float* qbar,
                       float* kbar, float* dq, uint32_t* amax_v, int8_t* q8, hipStream_t stream);
void launch_finalize_stats(const Problem& p, const float* kbar, const uint32_t* amax_v, float* mu_k,
                           float* dv, const bf16_t* proj_w, bf16_t* wfrag, hipStream_t stream);
void launch_scores(const Problem& p, const float* qbar, const float* kbar, float* scores, hipStream_t stream);
void launch_select(const Problem& p, const float* scores, int8_t* mask, int32_t* crit, int32_t* marg,
                   uint32_t* mbits, hipStream_t stream);
void launch_prep_kv(const void* k, const void* v, const Problem& p, const float* mu_k, const uint32_t* amax_v,
                    const bf16_t* wfrag, int phi_kind, bool want_quant, bool want_linear, int8_t* k8,
                    uint8_t* v8, float* dk, bf16_t* hz, hipStream_t stream);
void launch_marginal_bits(const Problem& p, const int8_t* mask, uint32_t* mbits, hipStream_t stream);
void launch_lin_accumulate(const Problem& p, const uint32_t* mbits, const bf16_t* hz, bf16_t* HZ,
                           hipStream_t stream);
void launch_sparse_fwd(const void* q, const int8_t* q8, const Problem& p, const int32_t* crit, int n_c, const int8_t* k8,
                       const uint8_t* v8, const float* dq, const float* dk, const float* dv,
                       const bf16_t* HZ, const bf16_t* proj_b, int phi_kind, bool has_linear,
                       void* out, bool out_f32, float* lse, int32_t* pair_list, int32_t* pair_len,
                       hipStream_t stream);
// Backward pass (k_bwd.hip, k_bwd_lin.hip; the transposed bit matrix lives with lin_accumulate).
size_t marginal_bits_t_bytes(const Problem& p);
void launch_marginal_bits_t(const Problem& p, const int8_t* mask, uint32_t* mbits_t, hipStream_t stream);
int launch_bwd_stats(const Problem& p, const void* q, const void* k, const void* v, const void* dout,
                     const int32_t* crit, float* lse2, float* delta, hipStream_t stream);
// qk_scales: nullptr, or {delta_Q [BH,Tq], delta_K [BH,Tk]} when q and k hold INT8 codes (q_lin: the
// original Q for the linear term's feature map)
struct CodeScales { const float* dq; const float* dk; const void* q_lin; };
int launch_fwd_bf16(const Problem& p, const void* q, const void* k, const void* v, const int32_t* crit,
                    const bf16_t* HZ, const bf16_t* proj_b, int phi_kind, void* out, float* save_lse2, void* save_os,
                    const CodeScales* codes, hipStream_t stream);
void launch_unpack_q8(const Problem& p, const int8_t* q8, int8_t* q_codes, hipStream_t stream);
void launch_code_tensors(const Problem& p, const int8_t* q8, const int8_t* k8, bf16_t* qc, bf16_t* kc, hipStream_t stream);
// First bytes of the state a training forward pass saves: which problem it belongs to.
constexpr int SAVED_MAGIC = 0x534C4153;
struct SavedHeader { int magic, B, H, N, block_q, n_c, pad0, pad1; };
void launch_write_saved_header(const SavedHeader& h, SavedHeader* dst, hipStream_t stream);
void launch_bwd_delta(const Problem& p, const void* dout, const void* os, const SavedHeader* hdr, const SavedHeader& want,
                      const float* lse_saved, float* lse2, float* delta, hipStream_t stream);
int launch_bwd_dq(const Problem& p, const void* q, const void* dout, const void* k, const void* v, const int32_t* crit,
                   const float* lse2, const float* delta, const float* dq_lin, void* dq, hipStream_t stream);
int launch_bwd_dkv(const Problem& p, const void* q, const void* dout, const void* k, const void* v, const int8_t* mask,
                    const float* lse2, const float* delta, const bf16_t* G, int phi_kind, void* dk, void* dv, hipStream_t stream);
void launch_bwd_wt(const bf16_t* proj_w, bf16_t* wt, hipStream_t stream);
size_t bwd_lin_q_partial_bytes(const Problem& p);
double launch_mfma_rate(int kind, int iters, int n_cu, float* sink, hipStream_t stream);
int launch_bwd_lin_q(const Problem& p, const void* q, const void* dout, const bf16_t* HZ, const bf16_t* wt,
                     int phi_kind, float* dq_lin, bf16_t* dHZ, float* dW, float* db, float* partials, hipStream_t stream);
void launch_zero_u32(uint32_t* p, size_t n, hipStream_t stream);
void launch_unfragment_kv(const Problem& p, const int8_t* k8, const uint8_t* v8, int8_t* k_codes,
                          uint8_t* v_codes, hipStream_t stream);
void launch_e4m3_encode(const float* in, uint8_t* out, size_t n, hipStream_t stream);

}  // namespace sla
