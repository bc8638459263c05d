// Backward pass of SLA, sparse branch (the operator of the paper's finetuning stage, Section 1.2):
// the gradient of the unquantised block-sparse softmax attention
//     O^s[n] = sum_{t in critical blocks of n's query block} softmax_t(Q[n].K[t] / sqrt(d)) V[t]
// with respect to Q, K and V, in bf16 on the matrix cores with fp32 accumulation.
//
//   bwd_stats_kernel    per query block: online-softmax pass over its critical key blocks ->
//                       lse (base-2 log-sum-exp of the scaled scores) and delta = dO . O^s per token.
//   bwd_dq_kernel       per query block, over its critical key blocks:
//                       P = exp2(S - lse), dS = P o (dO V^T - delta), dQ += dS K / sqrt(d).
//   bwd_dkv_kernel      per key block, over the query blocks that hold it as critical:
//                       dV += P^T dO, dK += dS^T Q / sqrt(d).
//
// All products are formed transposed where that saves a shuffle: a wavefront owns 32 tokens, one per
// lane (two lanes per token, each with half of the rows of an accumulator tile), so row statistics
// stay inside a lane pair, and an accumulator tile converted to bf16 is directly the B operand of
// the next product (its contraction index = the accumulator's rows).
//
// Operand tiles (32 tokens x 128 channels) are staged in LDS row-major as they are in memory.  A
// product that contracts over the channels reads its operand with one 16-byte read per step; a
// product that contracts over the tile's tokens reads the same tile with the transposing LDS read
// of gfx950 (ds_read_b64_tr_b16), so no transposed copy of any tensor is ever made.
#include <initializer_list>

#include "common.h"

namespace sla {

constexpr float QK_LOG2 = LOG2E / 11.313708498984761f;   // log2(e) / sqrt(d)
constexpr float INV_SQRT_D = 1.0f / 11.313708498984761f;

__device__ __forceinline__ v8bf as_v8bf(const uint4& x) { return __builtin_bit_cast(v8bf, x); }
__device__ __forceinline__ v16f mfma_bf16(const uint4& a, const uint4& b, const v16f& c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_v8bf(a), as_v8bf(b), c, 0, 0, 0);
}
// Accumulator registers 8 s .. 8 s + 7 of a tile as a bf16 operand: contraction step s (16 rows) of
// the product that contracts over the tile's rows.  Row of element kk for lane half hf:
// 16 s + 8 (kk / 4) + 4 hf + kk % 4 -- the order t_op (below) reads a staged tile's rows in.
__device__ __forceinline__ uint4 acc_operand(const v16f& a, int s) {
  return uint4{pack_bf16x2(a[8 * s], a[8 * s + 1]), pack_bf16x2(a[8 * s + 2], a[8 * s + 3]),
               pack_bf16x2(a[8 * s + 4], a[8 * s + 5]), pack_bf16x2(a[8 * s + 6], a[8 * s + 7])};
}

constexpr int TP = 304;             // bytes per staged row: 256 of data + 48 of skew (76 dwords: within a group of 16 lanes neither
                                    // the 16-byte operand reads nor the transposing reads collide)
constexpr int TILE_B = 32 * TP;     // one 32-token tile

typedef short v4s __attribute__((ext_vector_type(4)));
__device__ __forceinline__ v4s read_tr(const unsigned char* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4s*)p);
}
// Operand for a contraction over the channels: token (row) l32 of the tile, channels 16 ks + 8 hf + 0..7.
__device__ __forceinline__ uint4 n_op(const unsigned char* tile, int l32, int hf, int ks) {
  return *(const uint4*)(tile + l32 * TP + ks * 32 + hf * 16);
}
// This lane's address inside a 4-row x 16-column patch for the transposing read: in every group of
// 16 lanes, lane i receives element i of rows 0..3 of the patch that the group's lanes address
// (lane s: row s / 4, columns 4 (s % 4) .. + 3).  Lane group g = lane / 16 serves channels
// 16 (g % 2) .. + 15 of a 32-channel tile and the token rows of lane half g / 2.
__device__ __forceinline__ int tr_lane_offset(int lane) {
  return (4 * (lane >> 5) + ((lane & 15) >> 2)) * TP + (16 * ((lane >> 4) & 1) + 4 * (lane & 3)) * 2;
}
// Operand for a contraction over the tile's tokens, step s (16 tokens), channel tile ct: channel
// 32 ct + l32, tokens 16 s + 8 (kk / 4) + 4 hf + kk % 4 for kk = 0..7 -- the order in which
// acc_operand hands over the rows of an accumulator tile.
__device__ __forceinline__ uint4 t_op(const unsigned char* tile, int tr_off, int ct, int s) {
  union { v4s h[2]; uint4 v; } u;
  u.h[0] = read_tr(tile + tr_off + (16 * s) * TP + ct * 64);
  u.h[1] = read_tr(tile + tr_off + (16 * s + 8) * TP + ct * 64);
  return u.v;
}
// The same operand as n_op straight from memory (a workgroup's own rows, read once).
// (x: the (b,h) slice's first token; sn: elements from one token to the next)
__device__ __forceinline__ void own_rows(const bf16_t* x, long long sn, long long row, int N, int hf, uint4 (&f)[8]) {
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) f[ks] = row < N ? *(const uint4*)(x + row * sn + 16 * ks + 8 * hf) : uint4{0u, 0u, 0u, 0u};
}
// A tensor's layout as the kernel uses it: the caller's (ST) or, for the instances that serve contiguous
// [B,H,N,d] tensors only, compile-time strides (the row stride then folds into the address arithmetic).
template <bool ST>
__device__ __forceinline__ Layout lay(const Layout& L, int H, int N) {
  if constexpr (ST) return L;
  else return Layout{(long long)H * N * D, (long long)N * D, (long long)D};
}
#define SLA_BWD_LAYOUTS                                                                                         \
  const Layout L_q = lay<ST>(dm.lq, dm.H, dm.N), L_k = lay<ST>(dm.lk, dm.H, dm.N), L_v = lay<ST>(dm.lv, dm.H, dm.N), \
               L_d = lay<ST>(dm.ld, dm.H, dm.N), L_dq = lay<ST>(dm.ldq, dm.H, dm.N), L_dk = lay<ST>(dm.ldk, dm.H, dm.N), \
               L_dv = lay<ST>(dm.ldv, dm.H, dm.N), L_o = lay<ST>(dm.lo, dm.H, dm.N);                              \
  (void)L_q; (void)L_k; (void)L_v; (void)L_d; (void)L_dq; (void)L_dk; (void)L_dv; (void)L_o;
// First token of slice bh = b H + h of a tensor laid out by L.
__device__ __forceinline__ const bf16_t* slice_of(const bf16_t* x, const Layout& L, int bh, int H) {
  const int b = bh / H;
  return x + b * L.sb + (bh - b * H) * L.sh;
}
__device__ __forceinline__ bf16_t* slice_of(bf16_t* x, const Layout& L, int bh, int H) {
  const int b = bh / H;
  return x + b * L.sb + (bh - b * H) * L.sh;
}

// ROWS consecutive token rows of a [N, 128] tensor -> LDS tile(s), through registers (loaded one
// step ahead); rows beyond N are zero.  NT threads take part.
template <int NT, int ROWS>
struct RowStage {
  static constexpr int PER = ROWS * 16 / NT;
  uint4 pf[PER];
  __device__ __forceinline__ void load(const bf16_t* x, long long sn, long long r0, int N, int t) {
    if (r0 + ROWS <= N) {  // (uniform) every row exists: no per-row test
#pragma unroll
      for (int u = 0; u < PER; ++u) {
        const int c = u * NT + t;
        pf[u] = *(const uint4*)(x + (r0 + (c >> 4)) * sn + (c & 15) * 8);
      }
    } else {
#pragma unroll
      for (int u = 0; u < PER; ++u) {
        const int c = u * NT + t;
        const long long r = r0 + (c >> 4);
        pf[u] = r < N ? *(const uint4*)(x + r * sn + (c & 15) * 8) : uint4{0u, 0u, 0u, 0u};
      }
    }
  }
  // The same with rows beyond N replaced by row N - 1 and no branch: for callers that give such rows
  // a weight of exactly zero and want every call to issue the same loads (N > 0).
  __device__ __forceinline__ void load_clamped(const bf16_t* x, long long sn, int r0, int N, int t) {
#pragma unroll
    for (int u = 0; u < PER; ++u) {
      const int c = u * NT + t;
      const uint4 got = *(const uint4*)(x + (long long)min(r0 + (c >> 4), N - 1) * sn + (c & 15) * 8);
      pf[u] = got;  // (through a named value: assigning the dereferenced pointer straight to the member left the arrays in scratch memory)
    }
  }
  __device__ __forceinline__ void store(unsigned char* lds, int t) const {
#pragma unroll
    for (int u = 0; u < PER; ++u) {
      const int c = u * NT + t;
      *(uint4*)(lds + (c >> 4) * TP + (c & 15) * 16) = pf[u];
    }
  }
};

struct BwdDims {
  int N, Tq, Tk, n_c, T32q, H;
  Layout lq, lk, lv, ld;      // of q, k, v and dout (dq, dk, dv: ldq, ldk, ldv; the forward's out: lo)
  Layout ldq, ldk, ldv, lo;
};

// Workgroup -> (block, head) for a 1-D grid of 8 * ceil(T / 8) * BH workgroups.  Consecutive workgroup
// ids go to the 8 XCDs in turn; this order gives each XCD a contiguous run of a head's blocks, so
// the workgroups resident on one XCD at a time work on neighbouring blocks.  Returns false for the padding.
__device__ __forceinline__ bool xcd_block(int T, int& block, int& bh) {
  const int per_xcd = (T + 7) >> 3, xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  bh = slot / per_xcd;
  block = xcd * per_xcd + (slot - bh * per_xcd);
  return block < T;
}

// Scores of one key tile, transposed: lane = query, registers = keys.
__device__ __forceinline__ v16f score_tile(const unsigned char* ktile, const uint4 (&qf)[8], int l32, int hf) {
  v16f s = v16f{};
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) s = mfma_bf16(n_op(ktile, l32, hf, ks), qf[ks], s);
  return s;
}

// lse2[bh][32 T + r], delta[bh][32 T + r] for every token row of every query tile (rows beyond N:
// lse2 = +inf, delta = 0, so that their P is exactly 0 wherever they are used).
//
// With FWD the same pass is the unquantised SLA forward (Section 1.2's training-time operator):
// instead of the statistics it writes O = O^s + (phi(Q) H'_i) / (phi(Q) . Z_i) (+ b) in bf16, H'_i
// being the projected summaries the forward pass accumulates.
struct FwdEpilogue {
  const bf16_t* HZ;    // [BH, Tq, HZ_ROWS, D] or nullptr (no marginal block: no linear term)
  const bf16_t* bias;  // [D] or nullptr
  bf16_t* out;         // [BH, N, D]
  int phi;
  float* save_lse2;    // [BH, 32 T32q] or nullptr: the rows' log-sum-exp (base 2), as bwd_stats_kernel<.., false> writes it
  bf16_t* save_os;     // [BH, N, D] or nullptr: O^s alone (for delta = dO . O^s of a later backward pass)
  // CODES: q and k hold INT8 codes as bf16 numbers; a score is their (exact) product times
  // delta_Q[i] delta_K[j] / sqrt(d), and the feature map of the linear term reads the original Q
  const float* code_dq;  // [BH, Tq]
  const float* code_dk;  // [BH, Tk]
  const bf16_t* q_lin;   // the original Q, laid out by lq_lin
  Layout lq_lin;
};
template <int NW, bool FWD, bool CODES = false, bool ST = false>
__global__ void __launch_bounds__(NW * 64, NW == 4 ? 2 : 1) bwd_stats_kernel(const bf16_t* __restrict__ q, const bf16_t* __restrict__ k,
                                                            const bf16_t* __restrict__ v, const bf16_t* __restrict__ dout,
                                                            const int32_t* __restrict__ crit, float* __restrict__ lse2,
                                                            float* __restrict__ delta, BwdDims dm, FwdEpilogue fe) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_all[];  // two buffers of: K (2 tiles) then V (2 tiles) of a key block
  int i, bh;
  if (!xcd_block(dm.Tq, i, bh)) return;
  SLA_BWD_LAYOUTS
  const int t = threadIdx.x, lane = t & 63, w = t >> 6, l32 = lane & 31, hf = lane >> 5;
  const int tr_off = tr_lane_offset(lane);
  const int T = i * NW + w;
  const long long qrow = 32ll * T + l32;
  const bool qok = qrow < dm.N;
  const size_t head = (size_t)bh * dm.N * D;   // (of the library's own contiguous tensors)
  const bf16_t* qh = slice_of(q, L_q, bh, dm.H);
  const bf16_t* kh = slice_of(k, L_k, bh, dm.H);
  const bf16_t* vh = slice_of(v, L_v, bh, dm.H);
  uint4 qf[8];
  own_rows(qh, L_q.sn, qrow, dm.N, hf, qf);
  const int32_t* crow = crit + ((size_t)bh * dm.Tq + i) * dm.n_c;
  RowStage<NW * 64, 64> sk, sv;
  v16f o[4];
#pragma unroll
  for (int ct = 0; ct < 4; ++ct) o[ct] = v16f{};
  float m = -INFINITY;
  const float qscale = CODES ? QK_LOG2 * fe.code_dq[(size_t)bh * dm.Tq + i] : QK_LOG2;
  v16f lacc = v16f{};  // register 0: the running sum of P over the keys (see the ones operand below)
  // key blocks travel memory -> registers -> LDS one step ahead, into the buffer the step before
  // last has left: one barrier per step
  if (dm.n_c > 0) {
    sk.load(kh, L_k.sn, 64ll * crow[0], dm.N, t);
    sv.load(vh, L_v.sn, 64ll * crow[0], dm.N, t);
    sk.store(lds_all, t);
    sv.store(lds_all + 2 * TILE_B, t);
  }
  // Everything requested so far has to be in before the loop: a load the compiler cannot prove
  // finished on every path into the loop would be waited for each time round, in the middle of the
  // products and together with the loads of the next block just issued.  For the same reason the
  // loop's own loads and stores are unconditional (rows beyond N come as row N - 1; their P is 0).
  __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
  __syncthreads();
  for (int b = 0; b < dm.n_c; ++b) {
    const int j = crow[b];
    const float c2 = CODES ? qscale * fe.code_dk[(size_t)bh * dm.Tk + j] : QK_LOG2;   // score -> base-2 logit
    const unsigned char* lds = lds_all + (b & 1) * 4 * TILE_B;
    unsigned char* lds_next = lds_all + ((b + 1) & 1) * 4 * TILE_B;
    {  // the next block (after the last one: the last one again), the same loads every time round -- see below
      const int jn = 64 * crow[min(b + 1, dm.n_c - 1)];
      sk.load_clamped(kh, L_k.sn, jn, dm.N, t);
      sv.load_clamped(vh, L_v.sn, jn, dm.N, t);
    }
    v16f s[2];
    float mx = -INFINITY;
#pragma unroll
    for (int kt = 0; kt < 2; ++kt) {
      uint4 ak[8];  // operand reads grouped ahead of the matrix products that use them
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) ak[ks] = n_op(lds + kt * TILE_B, l32, hf, ks);
      s[kt] = v16f{};
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) s[kt] = mfma_bf16(ak[ks], qf[ks], s[kt]);
      __builtin_amdgcn_sched_group_barrier(0x100, 8, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, 8, 0);
      if (64 * j + 64 <= dm.N) {  // (uniform) only the sequence's last key block can hold keys that do not exist
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[kt][r]);
      } else {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = 64 * j + 32 * kt + 8 * (r >> 2) + 4 * hf + (r & 3);
          if (key >= dm.N) s[kt][r] = -INFINITY;
          mx = fmaxf(mx, s[kt][r]);
        }
      }
    }
    // The reference m moves only when the block's maximum exceeds it by more than 2^8: P then stays
    // below 2^8 (harmless in bf16 and fp32) and the accumulators are rescaled a few times per row
    // instead of every step.  (mx is finite: a block holds at least one valid key.)
    mx = fmaxf(mx, partner_f32(mx)) * c2;
    const bool moves = mx > m + 8.0f;
    if (__any(moves)) {
      const float m_new = moves ? mx : m;
      const float alpha = __builtin_amdgcn_exp2f(m - m_new);
      m = m_new;
      lacc[0] *= alpha;
#pragma unroll
      for (int ct = 0; ct < 4; ++ct)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[ct][r] *= alpha;
    }
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
      for (int r = 0; r < 16; ++r) s[kt][r] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[kt][r], c2, -m));
    const uint4 ones = uint4{0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u};  // bf16 1.0: sums P over the keys
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
      for (int sx = 0; sx < 2; ++sx) {
        const uint4 pb = acc_operand(s[kt], sx);
        uint4 tv[4];
#pragma unroll
        for (int ct = 0; ct < 4; ++ct) tv[ct] = t_op(lds + (2 + kt) * TILE_B, tr_off, ct, sx);
#pragma unroll
        for (int ct = 0; ct < 4; ++ct) o[ct] = mfma_bf16(tv[ct], pb, o[ct]);
        lacc = mfma_bf16(ones, pb, lacc);  // every row of this tile = the key sum of P (as rounded for the product above)
        __builtin_amdgcn_sched_group_barrier(0x100, 8, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 5, 0);
      }
    sk.store(lds_next, t);  // (after the last block: into the buffer nobody reads any more)
    sv.store(lds_next + 2 * TILE_B, t);
    __syncthreads();
  }
  const float l = lacc[0];
  if constexpr (FWD) {
    const float inv_l = dm.n_c > 0 ? 1.0f / l : 0.f;
#pragma unroll
    for (int ct = 0; ct < 4; ++ct)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[ct][r] *= inv_l;
    if (fe.save_lse2) {  // what a backward pass needs of this one
      if (hf == 0) fe.save_lse2[(size_t)bh * dm.T32q * 32 + 32 * T + l32] = (qok && dm.n_c > 0) ? m + __builtin_amdgcn_logf(l) : INFINITY;
      if (qok) {
#pragma unroll
        for (int ct = 0; ct < 4; ++ct)
#pragma unroll
          for (int g = 0; g < 4; ++g)
            *(uint2*)(fe.save_os + head + qrow * D + 32 * ct + 8 * g + 4 * hf) =
                uint2{pack_bf16x2(o[ct][4 * g], o[ct][4 * g + 1]), pack_bf16x2(o[ct][4 * g + 2], o[ct][4 * g + 3])};
      }
    }
    if (fe.HZ) {
      // linear term, transposed like everything else: O_l^T[o][n] = sum_c H'[c][o] phi(Q)[n][c]; the
      // stored chunks of H' are this product's A operand, phi(Q) follows their channel order
      const bf16_t* Hi = fe.HZ + ((size_t)bh * dm.Tq + i) * HZ_ELEMS;
      float x[64];
      uint4 bq[8];
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        const int c0 = 32 * (ks >> 1) + 16 * hf + 8 * (ks & 1);
        const bf16_t* ql = CODES ? slice_of(fe.q_lin, fe.lq_lin, bh, dm.H) + qrow * fe.lq_lin.sn : qh + qrow * L_q.sn;
        const uint4 qv = qok ? *(const uint4*)(ql + c0) : uint4{0u, 0u, 0u, 0u};
        x[8 * ks] = bf16_lo(qv.x); x[8 * ks + 1] = bf16_hi(qv.x); x[8 * ks + 2] = bf16_lo(qv.y); x[8 * ks + 3] = bf16_hi(qv.y);
        x[8 * ks + 4] = bf16_lo(qv.z); x[8 * ks + 5] = bf16_hi(qv.z); x[8 * ks + 6] = bf16_lo(qv.w); x[8 * ks + 7] = bf16_hi(qv.w);
      }
      if (fe.phi == 0) {
        float mx = x[0];
#pragma unroll
        for (int e = 1; e < 64; ++e) mx = fmaxf(mx, x[e]);
        mx = fmaxf(mx, partner_f32(mx));
        float sum = 0.f;
#pragma unroll
        for (int e = 0; e < 64; ++e) {
          x[e] = __builtin_amdgcn_exp2f((x[e] - mx) * LOG2E);
          sum += x[e];
        }
        sum += partner_f32(sum);
        const float inv = 1.0f / sum;
#pragma unroll
        for (int e = 0; e < 64; ++e) x[e] *= inv;
      } else if (fe.phi == 1) {
#pragma unroll
        for (int e = 0; e < 64; ++e) x[e] = x[e] > 0.f ? x[e] + 1.0f : __builtin_amdgcn_exp2f(x[e] * LOG2E);
      } else {
#pragma unroll
        for (int e = 0; e < 64; ++e) x[e] = fmaxf(x[e], 0.f);
      }
      float den = 0.f;
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        const int c0 = 32 * (ks >> 1) + 16 * hf + 8 * (ks & 1);
        const uint4 zv = *(const uint4*)(Hi + D * D + c0);
        const float z[8] = {bf16_lo(zv.x), bf16_hi(zv.x), bf16_lo(zv.y), bf16_hi(zv.y),
                            bf16_lo(zv.z), bf16_hi(zv.z), bf16_lo(zv.w), bf16_hi(zv.w)};
        bq[ks] = uint4{pack_bf16x2(x[8 * ks], x[8 * ks + 1]), pack_bf16x2(x[8 * ks + 2], x[8 * ks + 3]),
                       pack_bf16x2(x[8 * ks + 4], x[8 * ks + 5]), pack_bf16x2(x[8 * ks + 6], x[8 * ks + 7])};
        const uint32_t bw[4] = {bq[ks].x, bq[ks].y, bq[ks].z, bq[ks].w};
#pragma unroll
        for (int e = 0; e < 8; ++e) den = __builtin_fmaf(e & 1 ? bf16_hi(bw[e >> 1]) : bf16_lo(bw[e >> 1]), z[e], den);
      }
      den += partner_f32(den);
      const float inv_den = den != 0.f ? 1.0f / den : 0.f;  // no marginal block: no linear term
#pragma unroll
      for (int ot = 0; ot < 4; ++ot) {
        v16f al = v16f{};
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) al = mfma_bf16(*(const uint4*)(Hi + (size_t)hz_frag_chunk(ot, ks, lane) * 8), bq[ks], al);
#pragma unroll
        for (int r = 0; r < 16; ++r) o[ot][r] = __builtin_fmaf(al[r], inv_den, o[ot][r]);
      }
      if (fe.bias) {
#pragma unroll
        for (int ct = 0; ct < 4; ++ct)
#pragma unroll
          for (int r = 0; r < 16; ++r) o[ct][r] += bf16_to_f32(fe.bias[32 * ct + 8 * (r >> 2) + 4 * hf + (r & 3)]);
      }
    }
    if (qok) {
#pragma unroll
      for (int ct = 0; ct < 4; ++ct)
#pragma unroll
        for (int g = 0; g < 4; ++g)
          *(uint2*)(slice_of(fe.out, L_o, bh, dm.H) + qrow * L_o.sn + 32 * ct + 8 * g + 4 * hf) =
              uint2{pack_bf16x2(o[ct][4 * g], o[ct][4 * g + 1]), pack_bf16x2(o[ct][4 * g + 2], o[ct][4 * g + 3])};
    }
    return;
  }
  float dl = 0.f;
  if (qok && dm.n_c > 0) {
    const bf16_t* drow = slice_of(dout, L_d, bh, dm.H) + qrow * L_d.sn;
#pragma unroll
    for (int ct = 0; ct < 4; ++ct)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const uint2 dv = *(const uint2*)(drow + 32 * ct + 8 * g + 4 * hf);
        dl += bf16_lo(dv.x) * o[ct][4 * g] + bf16_hi(dv.x) * o[ct][4 * g + 1] + bf16_lo(dv.y) * o[ct][4 * g + 2] +
              bf16_hi(dv.y) * o[ct][4 * g + 3];
      }
  }
  dl += partner_f32(dl);
  if (hf == 0) {
    const bool live = qok && dm.n_c > 0;
    const size_t idx = (size_t)bh * dm.T32q * 32 + 32 * T + l32;
    lse2[idx] = live ? m + __builtin_amdgcn_logf(l) : INFINITY;
    delta[idx] = live ? dl / l : 0.f;
  }
}

// 4 accumulated values of one 8-channel group -> bf16, plus the linear branch's share if given.
__device__ __forceinline__ void store_grad4(bf16_t* dst, const float* lin, float a0, float a1, float a2, float a3) {
  if (lin) {
    const float4 x = *(const float4*)lin;
    a0 += x.x; a1 += x.y; a2 += x.z; a3 += x.w;
  }
  *(uint2*)dst = uint2{pack_bf16x2(a0, a1), pack_bf16x2(a2, a3)};
}

template <int NW, bool ST = false>
__global__ void __launch_bounds__(NW * 64, NW == 4 ? 2 : 1) bwd_dq_kernel(const bf16_t* __restrict__ q, const bf16_t* __restrict__ dout,
                                                         const bf16_t* __restrict__ k, const bf16_t* __restrict__ v,
                                                         const int32_t* __restrict__ crit, const float* __restrict__ lse2,
                                                         const float* __restrict__ delta, const float* __restrict__ dq_lin,
                                                         bf16_t* __restrict__ dq, BwdDims dm) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_all[];  // two buffers of: K (2 tiles) then V (2 tiles) of a key block
  int i, bh;
  if (!xcd_block(dm.Tq, i, bh)) return;
  const int t = threadIdx.x, lane = t & 63, w = t >> 6, l32 = lane & 31, hf = lane >> 5;
  const int tr_off = tr_lane_offset(lane);
  const int T = i * NW + w;
  const long long qrow = 32ll * T + l32;
  SLA_BWD_LAYOUTS
  const size_t head = (size_t)bh * dm.N * D;   // (of the library's own contiguous tensors)
  const bf16_t* kh = slice_of(k, L_k, bh, dm.H);
  const bf16_t* vh = slice_of(v, L_v, bh, dm.H);
  uint4 qf[8], dof[8];
  own_rows(slice_of(q, L_q, bh, dm.H), L_q.sn, qrow, dm.N, hf, qf);
  own_rows(slice_of(dout, L_d, bh, dm.H), L_d.sn, qrow, dm.N, hf, dof);
  const size_t sidx = (size_t)bh * dm.T32q * 32 + 32 * T + l32;
  const float lse_q = lse2[sidx], delta_q = delta[sidx];
  const int32_t* crow = crit + ((size_t)bh * dm.Tq + i) * dm.n_c;
  RowStage<NW * 64, 64> sk, sv;
  v16f acc[4];
#pragma unroll
  for (int ct = 0; ct < 4; ++ct) acc[ct] = v16f{};
  if (dm.n_c > 0) {
    sk.load(kh, L_k.sn, 64ll * crow[0], dm.N, t);
    sv.load(vh, L_v.sn, 64ll * crow[0], dm.N, t);
    sk.store(lds_all, t);
    sv.store(lds_all + 2 * TILE_B, t);
  }
  // Everything requested so far has to be in before the loop: a load the compiler cannot prove
  // finished on every path into the loop would be waited for each time round, in the middle of the
  // products and together with the loads of the next block just issued.  For the same reason the
  // loop's own loads and stores are unconditional (rows beyond N come as row N - 1; their P is 0).
  __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
  __syncthreads();
  for (int b = 0; b < dm.n_c; ++b) {
    const int j = crow[b];
    const unsigned char* lds = lds_all + (b & 1) * 4 * TILE_B;
    unsigned char* lds_next = lds_all + ((b + 1) & 1) * 4 * TILE_B;
    {  // the next block (after the last one: the last one again), the same loads every time round -- see below
      const int jn = 64 * crow[min(b + 1, dm.n_c - 1)];
      sk.load_clamped(kh, L_k.sn, jn, dm.N, t);
      sv.load_clamped(vh, L_v.sn, jn, dm.N, t);
    }
#pragma unroll
    for (int kt = 0; kt < 2; ++kt) {
      const unsigned char* ktile = lds + kt * TILE_B;
      const unsigned char* vtile = lds + (2 + kt) * TILE_B;
      // operand reads grouped ahead of the matrix products that use them
      uint4 ak[8], av[8];
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        ak[ks] = n_op(ktile, l32, hf, ks);
        av[ks] = n_op(vtile, l32, hf, ks);
      }
      v16f s = v16f{}, dp = v16f{};
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) s = mfma_bf16(ak[ks], qf[ks], s);
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) dp = mfma_bf16(av[ks], dof[ks], dp);
      // K reads; the score products, one V read behind each; the dO V^T products
      __builtin_amdgcn_sched_group_barrier(0x100, 8, 0);
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      }
      __builtin_amdgcn_sched_group_barrier(0x008, 8, 0);
      if (64 * j + 64 <= dm.N) {  // (uniform) only the sequence's last key block can hold keys that do not exist
#pragma unroll
        for (int r = 0; r < 16; ++r) s[r] = __builtin_amdgcn_exp2f(s[r] * QK_LOG2 - lse_q) * (dp[r] - delta_q);
      } else {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = 64 * j + 32 * kt + 8 * (r >> 2) + 4 * hf + (r & 3);
          const float p = key < dm.N ? __builtin_amdgcn_exp2f(s[r] * QK_LOG2 - lse_q) : 0.f;
          s[r] = p * (dp[r] - delta_q);
        }
      }
#pragma unroll
      for (int sx = 0; sx < 2; ++sx) {
        const uint4 dsb = acc_operand(s, sx);
        uint4 tk[4];
#pragma unroll
        for (int ct = 0; ct < 4; ++ct) tk[ct] = t_op(ktile, tr_off, ct, sx);
#pragma unroll
        for (int ct = 0; ct < 4; ++ct) acc[ct] = mfma_bf16(tk[ct], dsb, acc[ct]);
        __builtin_amdgcn_sched_group_barrier(0x100, 8, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
      }
    }
    sk.store(lds_next, t);  // (after the last block: into the buffer nobody reads any more)
    sv.store(lds_next + 2 * TILE_B, t);
    __syncthreads();
  }
  if (qrow < dm.N) {
    const size_t row = head + qrow * D;          // (the linear branch's share: the library's own tensor)
    bf16_t* dqrow = slice_of(dq, L_dq, bh, dm.H) + qrow * L_dq.sn;
#pragma unroll
    for (int ct = 0; ct < 4; ++ct)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int ch = 32 * ct + 8 * g + 4 * hf;
        store_grad4(dqrow + ch, dq_lin ? dq_lin + row + ch : nullptr, acc[ct][4 * g] * INV_SQRT_D,
                    acc[ct][4 * g + 1] * INV_SQRT_D, acc[ct][4 * g + 2] * INV_SQRT_D, acc[ct][4 * g + 3] * INV_SQRT_D);
      }
  }
}

// The linear branch's share of dK and dV for the 32 keys of a wavefront (Section 1.2's operator:
// h_j = phi(K_j)^T V_j, z_j = column sums of phi(K_j), phi = softmax over the channels), given
// G_j = the sum of dH_i over the query blocks that hold key block j as marginal, and the same sum
// of dZ_i, in the summaries' storage order (hz_frag_chunk):
//     d phi(K)^T[c][n] = sum_o G[c][o] V[n][o] + dZ[c]   ->  dK[n] = phi o (d phi - phi . d phi)
//     dV^T[o][n]       = sum_c G[c][o] phi(K)[n][c]
// Called by every thread of the workgroup (NT of them): G_j is staged in LDS transposed (gc,
// 128 rows of GP elements; gz, 128 floats); both barriers are inside.  Results in the accumulator
// layout of the sparse-branch kernels (lane = key, registers = channels).
constexpr int GP = 136;  // row pitch of the staged G (elements)
template <int NT, int PHI>
__device__ __forceinline__ void linear_kv_share(const bf16_t* __restrict__ k, const bf16_t* __restrict__ v,   // (the token's rows)
                                                bool ok, const bf16_t* __restrict__ rec, bf16_t* gc, float* gz, int t,
                                                int lane, v16f (&dk_share)[4], v16f (&dv_share)[4]) {
  const int l32 = lane & 31, hf = lane >> 5;
  for (int x = t; x < 2048; x += NT) {
    const int ln = x & 63, ks = (x >> 6) & 7, ot = x >> 9;
    const int o = 32 * ot + (ln & 31), c0 = 32 * (ks >> 1) + 16 * (ln >> 5) + 8 * (ks & 1);
    const uint4 val = *(const uint4*)(rec + (size_t)x * 8);
    const uint32_t wv[4] = {val.x, val.y, val.z, val.w};
#pragma unroll
    for (int e = 0; e < 8; ++e) gc[(c0 + e) * GP + o] = (bf16_t)(e & 1 ? wv[e >> 1] >> 16 : wv[e >> 1] & 0xffffu);
  }
  if (t < 128) gz[t] = bf16_to_f32(rec[128 * 128 + t]);
  __syncthreads();
  // phi(K[n]) at the channels the storage order feeds per step: 32 (ks / 2) + 16 hf + 8 (ks % 2) + kk
  float cv[64];
  uint4 cf[8], vf[8];
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) {
    uint4 kv = uint4{0u, 0u, 0u, 0u};
    vf[ks] = kv;
    if (ok) {
      kv = *(const uint4*)(k + 32 * (ks >> 1) + 16 * hf + 8 * (ks & 1));
      vf[ks] = *(const uint4*)(v + 16 * ks + 8 * hf);
    }
    cv[8 * ks] = bf16_lo(kv.x); cv[8 * ks + 1] = bf16_hi(kv.x); cv[8 * ks + 2] = bf16_lo(kv.y); cv[8 * ks + 3] = bf16_hi(kv.y);
    cv[8 * ks + 4] = bf16_lo(kv.z); cv[8 * ks + 5] = bf16_hi(kv.z); cv[8 * ks + 6] = bf16_lo(kv.w); cv[8 * ks + 7] = bf16_hi(kv.w);
  }
  float kmax = 0.f, sum = 1.0f;
  if constexpr (PHI == 0) {
    kmax = cv[0];
#pragma unroll
    for (int e = 1; e < 64; ++e) kmax = fmaxf(kmax, cv[e]);
    kmax = fmaxf(kmax, partner_f32(kmax));
    sum = 0.f;
#pragma unroll
    for (int e = 0; e < 64; ++e) {
      cv[e] = __builtin_amdgcn_exp2f((cv[e] - kmax) * LOG2E);
      sum += cv[e];
    }
    sum += partner_f32(sum);
  } else {
#pragma unroll
    for (int e = 0; e < 64; ++e) cv[e] = phi_value<PHI>(cv[e], 0.f, 1.0f);
  }
  const float rsum = ok ? 1.0f / sum : 0.f;  // keys beyond the sequence take no part
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) {
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) cv[8 * ks + kk] *= rsum;
    cf[ks] = uint4{pack_bf16x2(cv[8 * ks], cv[8 * ks + 1]), pack_bf16x2(cv[8 * ks + 2], cv[8 * ks + 3]),
                   pack_bf16x2(cv[8 * ks + 4], cv[8 * ks + 5]), pack_bf16x2(cv[8 * ks + 6], cv[8 * ks + 7])};
  }
#pragma unroll
  for (int ot = 0; ot < 4; ++ot) {
    uint4 ag[8], ac[8];  // operand reads grouped ahead of the matrix products
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      ag[ks] = *(const uint4*)(rec + (size_t)hz_frag_chunk(ot, ks, lane) * 8);  // the stored chunks are this product's A operand as they are
      ac[ks] = *(const uint4*)(gc + (32 * ot + l32) * GP + 16 * ks + 8 * hf);
    }
    dv_share[ot] = v16f{};
    dk_share[ot] = v16f{};
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      dv_share[ot] = mfma_bf16(ag[ks], cf[ks], dv_share[ot]);
      dk_share[ot] = mfma_bf16(ac[ks], vf[ks], dk_share[ot]);  // d phi(K)^T for now
    }
    __builtin_amdgcn_sched_group_barrier(0x020, 8, 0);
    __builtin_amdgcn_sched_group_barrier(0x100, 8, 0);
    __builtin_amdgcn_sched_group_barrier(0x008, 16, 0);
  }
  // through the feature map: phi at the accumulator's channels 32 ct + 8 g + 4 hf + e, from K again
  float sdot = 0.f;
  uint2 kw[4][4];
#pragma unroll
  for (int ct = 0; ct < 4; ++ct)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int c0 = 32 * ct + 8 * g + 4 * hf;
      kw[ct][g] = ok ? *(const uint2*)(k + c0) : uint2{0u, 0u};
      const float xk[4] = {bf16_lo(kw[ct][g].x), bf16_hi(kw[ct][g].x), bf16_lo(kw[ct][g].y), bf16_hi(kw[ct][g].y)};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        dk_share[ct][4 * g + e] += gz[c0 + e];
        if constexpr (PHI == 0) sdot += phi_value<0>(xk[e], kmax, rsum) * dk_share[ct][4 * g + e];
      }
    }
  sdot += partner_f32(sdot);
#pragma unroll
  for (int ct = 0; ct < 4; ++ct)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const float xk[4] = {bf16_lo(kw[ct][g].x), bf16_hi(kw[ct][g].x), bf16_lo(kw[ct][g].y), bf16_hi(kw[ct][g].y)};
#pragma unroll
      for (int e = 0; e < 4; ++e)
        dk_share[ct][4 * g + e] = phi_backward<PHI>(xk[e], phi_value<PHI>(xk[e], kmax, rsum), dk_share[ct][4 * g + e], sdot);
    }
  __syncthreads();  // the staged G is consumed: the caller may reuse the LDS
}

// One workgroup of four wavefronts per PAIR of adjacent key blocks (2 J, 2 J + 1): wavefronts 0, 1
// own the two key tiles of the first block, wavefronts 2, 3 those of the second (one key per lane
// pair).  The workgroup walks over the query blocks that hold either block as critical (found from
// the two mask columns; two flag bits per entry), staging each query tile's Q and dO once for both;
// a wavefront whose block is not critical for the current query block sits the step out.
// (KB = 2, 64 query rows per step.)  With KB = 1 a workgroup of two wavefronts serves one key block
// over its own list, 64 query rows per step as well, and two workgroups share a compute unit: every
// staged tile then serves one key block only, but no wavefront ever sits out.
template <int KB, int TILES, int PHI, bool ST = false>
__global__ void __launch_bounds__(128 * KB) bwd_dkv_kernel(const bf16_t* __restrict__ q, const bf16_t* __restrict__ dout,
                                                      const bf16_t* __restrict__ k, const bf16_t* __restrict__ v,
                                                      const int8_t* __restrict__ mask, const float* __restrict__ lse2,
                                                      const float* __restrict__ delta, const bf16_t* __restrict__ G,
                                                      bf16_t* __restrict__ dk, bf16_t* __restrict__ dv, int pair_shift,
                                                      BwdDims dm) {
  constexpr int NT = 128 * KB, ROWS = 32 * TILES;  // threads; query rows per step
  // two buffers of: Q (TILES tiles) then dO (TILES tiles) of ROWS consecutive query rows; then their lse, delta
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  constexpr int BUF_B = 2 * TILES * TILE_B;
  float (*stat)[2][ROWS] = (float (*)[2][ROWS])(lds + 2 * BUF_B);
  unsigned short* qlist = (unsigned short*)(lds + 2 * BUF_B + 2 * 2 * ROWS * 4);  // [Tq]
  __shared__ int wcnt[4];
  int J, bh;
  if (!xcd_block((dm.Tk + KB - 1) / KB, J, bh)) return;
  const int t = threadIdx.x, lane = t & 63, w = t >> 6, l32 = lane & 31, hf = lane >> 5;
  const int tr_off = tr_lane_offset(lane);
  const int half = KB == 2 ? w >> 1 : 0;
  // ---- the query blocks of the two key blocks, ascending; bit 14 / 15 = first / second block has it
  int nq = 0;
  const bool has2 = KB == 2 && 2 * J + 1 < dm.Tk;
  for (int base = 0; base < dm.Tq; base += NT) {
    const int i = base + t;
    int fl = 0;
    if (i < dm.Tq) {
      const int8_t* mrow = mask + ((size_t)bh * dm.Tq + i) * dm.Tk + KB * J;
      fl = (mrow[0] == 1 ? 1 : 0) | (has2 && mrow[1] == 1 ? 2 : 0);
    }
    const unsigned long long bal = __ballot(fl != 0);
    if (lane == 0) wcnt[w] = __popcll(bal);
    __syncthreads();
    int off = nq + __popcll(bal & ((1ull << lane) - 1ull));
    for (int x = 0; x < w; ++x) off += wcnt[x];
    if (fl) qlist[off] = (unsigned short)(i | (fl << 14));
#pragma unroll
    for (int x = 0; x < NT / 64; ++x) nq += wcnt[x];
    __syncthreads();
  }
  SLA_BWD_LAYOUTS
  const bf16_t* kh = slice_of(k, L_k, bh, dm.H);
  const bf16_t* vh = slice_of(v, L_v, bh, dm.H);
  const bf16_t* qh = slice_of(q, L_q, bh, dm.H);
  const bf16_t* doh = slice_of(dout, L_d, bh, dm.H);
  const long long key = 64ll * (KB * J + half) + 32 * (w & 1) + l32;
  const bool kok = key < dm.N;
  uint4 kf[8], vf[8];
  own_rows(kh, L_k.sn, key, dm.N, hf, kf);
  own_rows(vh, L_v.sn, key, dm.N, hf, vf);
  // the accumulators start from the linear branch's share (G = nullptr: there is none); dK is scaled
  // by 1 / sqrt(d) at the end, so its share goes in multiplied by sqrt(d)
  v16f dkt[4], dvt[4];
  if (G) {
    // each key block's two wavefronts stage its G_j in their own part of the (still unused) staging buffers
    constexpr int LIN_B = 128 * GP * 2 + 128 * 4;
    static_assert(KB * LIN_B <= 2 * BUF_B, "the staged G fits in the staging buffers");
    const int jb = min(KB * J + half, dm.Tk - 1);  // (the missing second block of an odd last pair: its keys do not exist)
    linear_kv_share<128, PHI>(kh + (kok ? key : 0) * L_k.sn, vh + (kok ? key : 0) * L_v.sn, kok, G + ((size_t)bh * dm.Tk + jb) * HZ_ELEMS,
                         (bf16_t*)(lds + half * LIN_B), (float*)(lds + half * LIN_B + 128 * GP * 2), t & 127, lane, dkt, dvt);
#pragma unroll
    for (int ct = 0; ct < 4; ++ct)
#pragma unroll
      for (int r = 0; r < 16; ++r) dkt[ct][r] *= 11.313708498984761f;
  } else {
#pragma unroll
    for (int ct = 0; ct < 4; ++ct) {
      dkt[ct] = v16f{};
      dvt[ct] = v16f{};
    }
  }
  // Steps = (list entry, pair of tiles of its query block): 64 query rows at a time.  They travel
  // memory -> registers -> LDS: while step s is computed from one LDS buffer, step s + 1 is moved from
  // registers to the other buffer and, where the registers allow a second set (KB = 2), step s + 2 is
  // on its way from memory; one barrier per step.  Within a step the two tiles are independent, which
  // lets the matrix products of one run under the exponentials of the other.
  const int steps = nq << pair_shift, pair_mask = (1 << pair_shift) - 1;
  RowStage<NT, ROWS> sq0, sd0, sq1, sd1;
  float ps0 = 0.f, ps1 = 0.f;
  auto rows_of = [&](int step) { return ROWS * (((qlist[step >> pair_shift] & 0x3fff) << pair_shift) + (step & pair_mask)); };
#define DKV_LOAD(SQ, SD, PS, STEP)                                                                   \
  {                                                                                                  \
    const int r_ = rows_of(min((STEP), steps - 1));                                                  \
    SQ.load_clamped(qh, L_q.sn, r_, dm.N, t);                                                      \
    SD.load_clamped(doh, L_d.sn, r_, dm.N, t);                                                     \
    PS = ((t & ROWS) ? delta : lse2)[(size_t)bh * dm.T32q * 32 + r_ + (t & (ROWS - 1))];             \
  }
#define DKV_STORE(SQ, SD, PS, BUF)                                                                   \
  {                                                                                                  \
    SQ.store(lds + (BUF) * BUF_B, t);                                                                \
    SD.store(lds + (BUF) * BUF_B + TILES * TILE_B, t);                                               \
    if (t < 2 * ROWS) stat[BUF][t / ROWS][t & (ROWS - 1)] = PS;                                      \
  }
  auto compute = [&](int step, int buf) __attribute__((always_inline)) {
    if (!((qlist[step >> pair_shift] >> (14 + half)) & 1)) return;  // (wave-uniform; always set when KB == 1)
    const unsigned char* qt0 = lds + buf * BUF_B;
    const unsigned char* dt0 = qt0 + TILES * TILE_B;
    v16f s[TILES], dp[TILES], p[TILES];
    // Operand reads are grouped ahead of the matrix products that use them (the compiler would
    // otherwise issue each read right before its product and wait for it every time).
#pragma unroll
    for (int u = 0; u < TILES; ++u) {
      uint4 aq[8], ad[8];
      float4 ls[4], dl[4];
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        aq[ks] = n_op(qt0 + u * TILE_B, l32, hf, ks);
        ad[ks] = n_op(dt0 + u * TILE_B, l32, hf, ks);
      }
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        ls[g] = *(const float4*)&stat[buf][0][32 * u + 8 * g + 4 * hf];
        dl[g] = *(const float4*)&stat[buf][1][32 * u + 8 * g + 4 * hf];
      }
      s[u] = v16f{};
      dp[u] = v16f{};
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        s[u] = mfma_bf16(aq[ks], kf[ks], s[u]);
        dp[u] = mfma_bf16(ad[ks], vf[ks], dp[u]);
      }
      __builtin_amdgcn_sched_group_barrier(0x100, 24, 0);  // 24 LDS reads (operands, then lse and delta)
      __builtin_amdgcn_sched_group_barrier(0x008, 16, 0);  // then 16 matrix products
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const float lsv[4] = {ls[g].x, ls[g].y, ls[g].z, ls[g].w}, dlv[4] = {dl[g].x, dl[g].y, dl[g].z, dl[g].w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float pe = __builtin_amdgcn_exp2f(s[u][4 * g + e] * QK_LOG2 - lsv[e]);  // (a key beyond N: a finite value in a column that is never stored)
          p[u][4 * g + e] = pe;
          s[u][4 * g + e] = pe * (dp[u][4 * g + e] - dlv[e]);
        }
      }
    }
#pragma unroll
    for (int u = 0; u < TILES; ++u) {
#pragma unroll
      for (int sx = 0; sx < 2; ++sx) {
        const uint4 pb = acc_operand(p[u], sx), dsb = acc_operand(s[u], sx);
        uint4 td[4], tq[4];
#pragma unroll
        for (int ct = 0; ct < 4; ++ct) {
          td[ct] = t_op(dt0 + u * TILE_B, tr_off, ct, sx);
          tq[ct] = t_op(qt0 + u * TILE_B, tr_off, ct, sx);
        }
#pragma unroll
        for (int ct = 0; ct < 4; ++ct) {
          dvt[ct] = mfma_bf16(td[ct], pb, dvt[ct]);
          dkt[ct] = mfma_bf16(tq[ct], dsb, dkt[ct]);
        }
        __builtin_amdgcn_sched_group_barrier(0x100, 16, 0);  // 16 transposing LDS reads
        __builtin_amdgcn_sched_group_barrier(0x008, 8, 0);   // then 8 matrix products
      }
    }
  };
  // The same for two tiles per step (one key block per workgroup), laid out so that the vector work of
  // one tile (exponentials, dS, conversions) is issued between the matrix products of the other: a
  // lone wavefront per SIMD has nobody else to fill the matrix pipe while it computes exponentials.
  auto compute_interleaved = [&](int step, int buf) __attribute__((always_inline)) {
    if (!((qlist[step >> pair_shift] >> (14 + half)) & 1)) return;  // (always set; keeps the compiler from hoisting reads over the step boundary)
    const unsigned char* qt0 = lds + buf * BUF_B;
    const unsigned char* dt0 = qt0 + TILES * TILE_B;
    v16f s[2], dp[2], p[2];
    float4 ls[4], dl[4];
    uint4 aq[8], ad[8];
    auto read_ops = [&](int u) __attribute__((always_inline)) {
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        aq[ks] = n_op(qt0 + u * TILE_B, l32, hf, ks);
        ad[ks] = n_op(dt0 + u * TILE_B, l32, hf, ks);
      }
    };
    auto read_stats = [&](int u) __attribute__((always_inline)) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        ls[g] = *(const float4*)&stat[buf][0][32 * u + 8 * g + 4 * hf];
        dl[g] = *(const float4*)&stat[buf][1][32 * u + 8 * g + 4 * hf];
      }
    };
    auto weight = [&](int u, int r) __attribute__((always_inline)) {  // P and dS of tile u, accumulator register r
      const float4 l4 = ls[r >> 2], d4 = dl[r >> 2];
      const float lv = (r & 3) == 0 ? l4.x : (r & 3) == 1 ? l4.y : (r & 3) == 2 ? l4.z : l4.w;
      const float dv_ = (r & 3) == 0 ? d4.x : (r & 3) == 1 ? d4.y : (r & 3) == 2 ? d4.z : d4.w;
      const float pe = __builtin_amdgcn_exp2f(s[u][r] * QK_LOG2 - lv);  // (a key beyond N: a finite value in a column that is never stored)
      p[u][r] = pe;
      s[u][r] = pe * (dp[u][r] - dv_);
    };
    // The step as an explicit schedule: every piece ends with a full scheduling fence, so the order
    // below is the order of issue.  Tile 0's scores; tile 1's scores with tile 0's exponentials
    // between the products; tile 0's gradient products with tile 1's exponentials between them;
    // tile 1's gradient products.  The LDS reads of each section are issued one section early, a
    // pair behind every product that has just consumed its operands (whose registers they take
    // over), so that no section starts by waiting for its reads.
#define FENCE __builtin_amdgcn_sched_barrier(0);
    uint4 bq[8], bd[8];          // tile 1's score operands
    uint4 td[4], tq[4], te[4], tr[4];  // transposed operands of the gradient products, two sets in turn
    read_ops(0);
    FENCE
    s[0] = v16f{};
    dp[0] = v16f{};
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      s[0] = mfma_bf16(aq[ks], kf[ks], s[0]);
      dp[0] = mfma_bf16(ad[ks], vf[ks], dp[0]);
      bq[ks] = n_op(qt0 + TILE_B, l32, hf, ks);
      bd[ks] = n_op(dt0 + TILE_B, l32, hf, ks);
      FENCE
    }
    read_stats(0);
    FENCE
    s[1] = v16f{};
    dp[1] = v16f{};
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      s[1] = mfma_bf16(bq[ks], kf[ks], s[1]);
      weight(0, 2 * ks);
      FENCE
      dp[1] = mfma_bf16(bd[ks], vf[ks], dp[1]);
      weight(0, 2 * ks + 1);
      if (ks & 1) {
        td[ks >> 1] = t_op(dt0, tr_off, ks >> 1, 0);
        tq[ks >> 1] = t_op(qt0, tr_off, ks >> 1, 0);
      }
      FENCE
    }
    read_stats(1);
    {
      const uint4 pb = acc_operand(p[0], 0), dsb = acc_operand(s[0], 0);
      FENCE
#pragma unroll
      for (int ct = 0; ct < 4; ++ct) {
        dvt[ct] = mfma_bf16(td[ct], pb, dvt[ct]);
        weight(1, 2 * ct);
        FENCE
        dkt[ct] = mfma_bf16(tq[ct], dsb, dkt[ct]);
        weight(1, 2 * ct + 1);
        te[ct] = t_op(dt0, tr_off, ct, 1);
        tr[ct] = t_op(qt0, tr_off, ct, 1);
        FENCE
      }
    }
    {
      const uint4 pb = acc_operand(p[0], 1), dsb = acc_operand(s[0], 1);
      FENCE
#pragma unroll
      for (int ct = 0; ct < 4; ++ct) {
        dvt[ct] = mfma_bf16(te[ct], pb, dvt[ct]);
        weight(1, 8 + 2 * ct);
        FENCE
        dkt[ct] = mfma_bf16(tr[ct], dsb, dkt[ct]);
        weight(1, 8 + 2 * ct + 1);
        td[ct] = t_op(dt0 + TILE_B, tr_off, ct, 0);
        tq[ct] = t_op(qt0 + TILE_B, tr_off, ct, 0);
        FENCE
      }
    }
    {
      const uint4 pb = acc_operand(p[1], 0), dsb = acc_operand(s[1], 0);
      FENCE
#pragma unroll
      for (int ct = 0; ct < 4; ++ct) {
        dvt[ct] = mfma_bf16(td[ct], pb, dvt[ct]);
        dkt[ct] = mfma_bf16(tq[ct], dsb, dkt[ct]);
        te[ct] = t_op(dt0 + TILE_B, tr_off, ct, 1);
        tr[ct] = t_op(qt0 + TILE_B, tr_off, ct, 1);
        FENCE
      }
    }
    {
      const uint4 pb = acc_operand(p[1], 1), dsb = acc_operand(s[1], 1);
      FENCE
#pragma unroll
      for (int ct = 0; ct < 4; ++ct) {
        dvt[ct] = mfma_bf16(te[ct], pb, dvt[ct]);
        dkt[ct] = mfma_bf16(tr[ct], dsb, dkt[ct]);
      }
      FENCE
    }
#undef FENCE
  };
  // One step: load step S + 2 into the set that step S has left, compute S, publish S + 1.  Every
  // step issues the same loads and stores whatever the step number (past the end the last step is
  // loaded again and a stale set is published to the buffer nobody reads any more; rows beyond N
  // come as row N - 1, their lse = +inf makes their P and dS exactly 0): with nothing conditional
  // the compiler can count the loads in flight and waits for those of step S + 1 only -- with the
  // loads under "if (step < steps)" it waited for everything, the loads just issued included,
  // before every publish, and again in the middle of the first group of products.
#define DKV_STEP(S, AHEAD, BUF, SQL, SDL, PSL, SQN, SDN, PSN)  \
  if ((S) >= steps) break;                                     \
  DKV_LOAD(SQL, SDL, PSL, (S) + (AHEAD))                       \
  if constexpr (KB == 1 && TILES == 2) compute_interleaved((S), BUF); else compute((S), BUF); \
  DKV_STORE(SQN, SDN, PSN, 1 - (BUF))                          \
  __syncthreads();
  if (steps > 0) {
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): the workgroup's own K, V rows are in (else the loop would wait for them each time round)
    DKV_LOAD(sq0, sd0, ps0, 0)
    if constexpr (NT * 2 >= ROWS * 8) {  // two register sets in rotation, two steps in flight
      DKV_LOAD(sq1, sd1, ps1, 1)
      DKV_STORE(sq0, sd0, ps0, 0)
      __syncthreads();
      for (int step = 0;; step += 2) {  // (every exit test is uniform over the workgroup)
        DKV_STEP(step, 2, 0, sq0, sd0, ps0, sq1, sd1, ps1)
        DKV_STEP(step + 1, 2, 1, sq1, sd1, ps1, sq0, sd0, ps0)
      }
    } else {                             // (a set is 64 registers here) one set, one step ahead
      DKV_STORE(sq0, sd0, ps0, 0)
      __syncthreads();
      for (int step = 0;; step += 2) {
        DKV_STEP(step, 1, 0, sq0, sd0, ps0, sq0, sd0, ps0)
        DKV_STEP(step + 1, 1, 1, sq0, sd0, ps0, sq0, sd0, ps0)
      }
    }
  }
#undef DKV_STEP
#undef DKV_LOAD
#undef DKV_STORE
  if (kok) {
    bf16_t* dkrow = slice_of(dk, L_dk, bh, dm.H) + key * L_dk.sn;
    bf16_t* dvrow = slice_of(dv, L_dv, bh, dm.H) + key * L_dv.sn;
#pragma unroll
    for (int ct = 0; ct < 4; ++ct)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int ch = 32 * ct + 8 * g + 4 * hf;
        store_grad4(dkrow + ch, nullptr, dkt[ct][4 * g] * INV_SQRT_D, dkt[ct][4 * g + 1] * INV_SQRT_D,
                    dkt[ct][4 * g + 2] * INV_SQRT_D, dkt[ct][4 * g + 3] * INV_SQRT_D);
        store_grad4(dvrow + ch, nullptr, dvt[ct][4 * g], dvt[ct][4 * g + 1], dvt[ct][4 * g + 2], dvt[ct][4 * g + 3]);
      }
  }
}

// ---------------------------------------------------------------------------------------------
constexpr int KV_STAGE_BYTES = 2 * 4 * TILE_B;  // dynamic LDS of the two per-query-block kernels
template <class K>
static bool allow_lds(K kernel) {
  return hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, KV_STAGE_BYTES) == hipSuccess;
}

// Do all of these layouts equal the contiguous [B,H,N,d] one?  (Then the instances with compile-time strides serve.)
static bool contiguous(const Problem& p, std::initializer_list<const Layout*> ls) {
  const Layout c = contiguous_layout(p.H, p.N);
  for (const Layout* L : ls)
    if (L->sb != c.sb || L->sh != c.sh || L->sn != c.sn) return false;
  return true;
}

static BwdDims bwd_dims(const Problem& p) {
  return BwdDims{p.N, p.Tq, p.Tk, p.n_c, p.Tq * (p.block_q / 32), p.H, p.lq, p.lk, p.lv, p.ld, p.ldq, p.ldk, p.ldv, p.lo};
}

// The launchers below return 0, or -1 when the kernel's LDS allowance could not be set (then nothing is
// launched; the result of the attribute call is cached, the failure is reported on every call).
int launch_bwd_stats(const Problem& p, const void* q, const void* k, const void* v, const void* dout,
                     const int32_t* crit, float* lse2, float* delta, hipStream_t stream) {
  const unsigned grid = (unsigned)(8 * ((p.Tq + 7) / 8) * p.BH);
  static const bool ok = allow_lds(bwd_stats_kernel<4, false>) && allow_lds(bwd_stats_kernel<2, false>) &&
                         allow_lds(bwd_stats_kernel<4, false, false, true>) && allow_lds(bwd_stats_kernel<2, false, false, true>);
  if (!ok) return -1;
  const FwdEpilogue none{nullptr, nullptr, nullptr, 0, nullptr, nullptr, nullptr, nullptr, nullptr, p.lq};
  const bool st = !contiguous(p, {&p.lq, &p.lk, &p.lv, &p.ld});
#define SLA_STATS(NW, ST) bwd_stats_kernel<NW, false, false, ST><<<grid, NW * 64, KV_STAGE_BYTES, stream>>>( \
      (const bf16_t*)q, (const bf16_t*)k, (const bf16_t*)v, (const bf16_t*)dout, crit, lse2, delta, bwd_dims(p), none)
  if (p.block_q == 128) {
    if (st) SLA_STATS(4, true); else SLA_STATS(4, false);
  } else {
    if (st) SLA_STATS(2, true); else SLA_STATS(2, false);
  }
#undef SLA_STATS
  return 0;
}

// The unquantised forward pass: the same kernel with the output epilogue; with `codes`, the same on
// INT8 codes of Q and K (SLA_QUANT_QK_INT8: integer products, 16-bit P and V).
int launch_fwd_bf16(const Problem& p, const void* q, const void* k, const void* v, const int32_t* crit,
                    const bf16_t* HZ, const bf16_t* proj_b, int phi_kind, void* out, float* save_lse2, void* save_os,
                    const CodeScales* codes, hipStream_t stream) {
  const unsigned grid = (unsigned)(8 * ((p.Tq + 7) / 8) * p.BH);
  static const bool ok = allow_lds(bwd_stats_kernel<4, true>) && allow_lds(bwd_stats_kernel<2, true>) &&
                         allow_lds(bwd_stats_kernel<4, true, true>) && allow_lds(bwd_stats_kernel<2, true, true>) &&
                         allow_lds(bwd_stats_kernel<4, true, false, true>) && allow_lds(bwd_stats_kernel<2, true, false, true>) &&
                         allow_lds(bwd_stats_kernel<4, true, true, true>) && allow_lds(bwd_stats_kernel<2, true, true, true>);
  if (!ok) return -1;
  const FwdEpilogue fe{HZ, HZ ? proj_b : nullptr, (bf16_t*)out, phi_kind, save_lse2, (bf16_t*)save_os,
                       codes ? codes->dq : nullptr, codes ? codes->dk : nullptr, codes ? (const bf16_t*)codes->q_lin : nullptr, p.lq};
  BwdDims dm = bwd_dims(p);
  if (codes) dm.lq = dm.lk = contiguous_layout(p.H, p.N);   // the code tensors are the library's own
  const bool st = codes ? !contiguous(p, {&p.lv, &p.lo}) : !contiguous(p, {&p.lq, &p.lk, &p.lv, &p.lo});
#define SLA_FWD16(NW, CODES, ST) bwd_stats_kernel<NW, true, CODES, ST><<<grid, NW * 64, KV_STAGE_BYTES, stream>>>( \
      (const bf16_t*)q, (const bf16_t*)k, (const bf16_t*)v, nullptr, crit, nullptr, nullptr, dm, fe)
#define SLA_FWD16_ST(NW, CODES) { if (st) SLA_FWD16(NW, CODES, true); else SLA_FWD16(NW, CODES, false); }
  if (p.block_q == 128) {
    if (codes) SLA_FWD16_ST(4, true) else SLA_FWD16_ST(4, false)
  } else {
    if (codes) SLA_FWD16_ST(2, true) else SLA_FWD16_ST(2, false)
  }
#undef SLA_FWD16_ST
#undef SLA_FWD16
  return 0;
}

// (the header's 256 bytes are written in full, so that two buffers filled for one problem are the same bytes)
__global__ void write_saved_header_kernel(SavedHeader h, int* __restrict__ dst) {
  const int v[8] = {h.magic, h.B, h.H, h.N, h.block_q, h.n_c, h.pad0, h.pad1};
  int x = 0;
#pragma unroll
  for (int e = 0; e < 8; ++e)
    if ((int)threadIdx.x == e) x = v[e];
  dst[threadIdx.x] = x;
}

void launch_write_saved_header(const SavedHeader& h, SavedHeader* dst, hipStream_t stream) {
  write_saved_header_kernel<<<1, 64, 0, stream>>>(h, (int*)dst);
}

// delta[bh][row] = dO[row] . O^s[row] from a saved O^s (rows beyond N: 0); one wavefront per 8 rows.
// The saved state's header must name this problem (shape, query block size, critical blocks per row): a
// buffer that no training forward pass of the same problem filled gives delta = lse = NaN, and with them NaN in
// every gradient, instead of plausible wrong numbers (the host cannot look without synchronising).
__global__ void __launch_bounds__(256) bwd_delta_kernel(const bf16_t* __restrict__ dout, const bf16_t* __restrict__ os,
                                                        const SavedHeader* __restrict__ hdr, SavedHeader want,
                                                        const float* __restrict__ lse_saved, float* __restrict__ lse2,
                                                        float* __restrict__ delta, int N, int rows_padded, int BH, int H,
                                                        Layout ld) {
  const long long gr = (long long)blockIdx.x * 32 + (threadIdx.x >> 3);  // padded row index over all heads
  if (gr >= (long long)BH * rows_padded) return;
  const SavedHeader got = *hdr;
  const bool mine = got.magic == want.magic && got.B == want.B && got.H == want.H && got.N == want.N &&
                    got.block_q == want.block_q && got.n_c == want.n_c;
  const int bh = (int)(gr / rows_padded), row = (int)(gr - (long long)bh * rows_padded), part = threadIdx.x & 7;
  float s = 0.f;
  if (row < N) {
    const size_t off = ((size_t)bh * N + row) * D + 16 * part;   // (O^s: the library's own tensor)
    const bf16_t* drow = slice_of(dout, ld, bh, H) + (long long)row * ld.sn + 16 * part;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const uint4 a = *(const uint4*)(drow + 8 * h), b = *(const uint4*)(os + off + 8 * h);
      s += bf16_lo(a.x) * bf16_lo(b.x) + bf16_hi(a.x) * bf16_hi(b.x) + bf16_lo(a.y) * bf16_lo(b.y) + bf16_hi(a.y) * bf16_hi(b.y) +
           bf16_lo(a.z) * bf16_lo(b.z) + bf16_hi(a.z) * bf16_hi(b.z) + bf16_lo(a.w) * bf16_lo(b.w) + bf16_hi(a.w) * bf16_hi(b.w);
    }
  }
  s += __shfl_xor(s, 1);
  s += __shfl_xor(s, 2);
  s += __shfl_xor(s, 4);
  if (part == 0) {  // (the log-sum-exp goes to the workspace copy the other kernels read: poisoned alike)
    delta[gr] = mine ? s : __builtin_nanf("");
    lse2[gr] = mine ? lse_saved[gr] : __builtin_nanf("");
  }
}

void launch_bwd_delta(const Problem& p, const void* dout, const void* os, const SavedHeader* hdr, const SavedHeader& want,
                      const float* lse_saved, float* lse2, float* delta, hipStream_t stream) {
  const int rows_padded = p.Tq * p.block_q;
  const long long total = (long long)p.BH * rows_padded;
  bwd_delta_kernel<<<(unsigned)((total + 31) / 32), 256, 0, stream>>>((const bf16_t*)dout, (const bf16_t*)os, hdr, want, lse_saved, lse2, delta, p.N,
                                                                     rows_padded, p.BH, p.H, p.ld);
}

int launch_bwd_dq(const Problem& p, const void* q, const void* dout, const void* k, const void* v, const int32_t* crit,
                  const float* lse2, const float* delta, const float* dq_lin, void* dq, hipStream_t stream) {
  const unsigned grid = (unsigned)(8 * ((p.Tq + 7) / 8) * p.BH);
  static const bool ok = allow_lds(bwd_dq_kernel<4>) && allow_lds(bwd_dq_kernel<2>) && allow_lds(bwd_dq_kernel<4, true>) &&
                         allow_lds(bwd_dq_kernel<2, true>);
  if (!ok) return -1;
  const bool st = !contiguous(p, {&p.lq, &p.lk, &p.lv, &p.ld, &p.ldq});
#define SLA_DQ(NW, ST) bwd_dq_kernel<NW, ST><<<grid, NW * 64, KV_STAGE_BYTES, stream>>>( \
      (const bf16_t*)q, (const bf16_t*)dout, (const bf16_t*)k, (const bf16_t*)v, crit, lse2, delta, dq_lin, (bf16_t*)dq, bwd_dims(p))
  if (p.block_q == 128) {
    if (st) SLA_DQ(4, true); else SLA_DQ(4, false);
  } else {
    if (st) SLA_DQ(2, true); else SLA_DQ(2, false);
  }
#undef SLA_DQ
  return 0;
}

constexpr int DKV1_TILES = 2;  // tiles per step of the one-key-block variant: 2 (78 KB of LDS per workgroup) runs compute_interleaved, 1 the plain step
template <int PHI, bool ST>
static int launch_bwd_dkv_phi(const Problem& p, const void* q, const void* dout, const void* k, const void* v, const int8_t* mask,
                               const float* lse2, const float* delta, const bf16_t* G, void* dk, void* dv, hipStream_t stream) {
  // dynamic LDS: two staging buffers, the rows' lse and delta, the list of query blocks
  const int list_bytes = (2 * p.Tq + 15) & ~15;
  const int lds2 = 2 * 4 * TILE_B + 2 * 2 * 64 * 4 + list_bytes;
  const int lds1 = 2 * 2 * DKV1_TILES * TILE_B + 2 * 2 * 32 * DKV1_TILES * 4 + list_bytes;
  static const bool ok =
      hipFuncSetAttribute((const void*)bwd_dkv_kernel<2, 2, PHI, ST>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024 - 256) == hipSuccess &&
      hipFuncSetAttribute((const void*)bwd_dkv_kernel<1, DKV1_TILES, PHI, ST>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024 - 256) == hipSuccess;
  if (!ok) return -1;
  const int tiles = p.block_q / 32;  // of a query block: 2 or 4
  // Two key blocks per workgroup halve the bytes streamed where their lists coincide and idle half
  // a workgroup where they do not: worth it only when most blocks are critical (at the paper's
  // 10-15 % the lists of neighbours share 60 % and one key block per workgroup is 25 % faster).
  const bool paired = 2 * p.n_c > p.Tk;
  if (paired) {
    const int pairs = (p.Tk + 1) / 2;
    bwd_dkv_kernel<2, 2, PHI, ST><<<(unsigned)(8 * ((pairs + 7) / 8) * p.BH), 256, lds2, stream>>>(
        (const bf16_t*)q, (const bf16_t*)dout, (const bf16_t*)k, (const bf16_t*)v, mask, lse2, delta, G,
        (bf16_t*)dk, (bf16_t*)dv, tiles == 4 ? 1 : 0, bwd_dims(p));
  } else {
    bwd_dkv_kernel<1, DKV1_TILES, PHI, ST><<<(unsigned)(8 * ((p.Tk + 7) / 8) * p.BH), 128, lds1, stream>>>(
        (const bf16_t*)q, (const bf16_t*)dout, (const bf16_t*)k, (const bf16_t*)v, mask, lse2, delta, G,
        (bf16_t*)dk, (bf16_t*)dv, (tiles == 4 ? 2 : 1) - (DKV1_TILES == 2 ? 1 : 0), bwd_dims(p));
  }
  return 0;
}

// (the feature map matters to the prologue only -- the linear branch's share -- and only when G is given)
int launch_bwd_dkv(const Problem& p, const void* q, const void* dout, const void* k, const void* v, const int8_t* mask,
                   const float* lse2, const float* delta, const bf16_t* G, int phi_kind, void* dk, void* dv, hipStream_t stream) {
  const int phi = G ? phi_kind : 0;
  if (contiguous(p, {&p.lq, &p.lk, &p.lv, &p.ld, &p.ldk, &p.ldv})) {
    if (phi == 0) return launch_bwd_dkv_phi<0, false>(p, q, dout, k, v, mask, lse2, delta, G, dk, dv, stream);
    if (phi == 1) return launch_bwd_dkv_phi<1, false>(p, q, dout, k, v, mask, lse2, delta, G, dk, dv, stream);
    return launch_bwd_dkv_phi<2, false>(p, q, dout, k, v, mask, lse2, delta, G, dk, dv, stream);
  }
  if (phi == 0) return launch_bwd_dkv_phi<0, true>(p, q, dout, k, v, mask, lse2, delta, G, dk, dv, stream);
  if (phi == 1) return launch_bwd_dkv_phi<1, true>(p, q, dout, k, v, mask, lse2, delta, G, dk, dv, stream);
  return launch_bwd_dkv_phi<2, true>(p, q, dout, k, v, mask, lse2, delta, G, dk, dv, stream);
}

}  // namespace sla
