// Backward pass of SLA, sparse branch (the operator of the paper's finetuning stage, Section 1.2):
// the gradient of the unquantised block-sparse softmax attention
//     O^s[n] = sum_{t in critical blocks of n's query block} softmax_t(Q[n].K[t] / sqrt(d)) V[t]
// with respect to Q, K and V, in bf16 on the matrix cores with fp32 accumulation.
//
//   bwd_pack_kernel     Q, K, V, dO -> per 32-token tile, two 8 KiB records in MFMA operand order:
//                       the n-record (contraction over channels) and the t-record (contraction
//                       over the tile's tokens).
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
#include "common.h"

namespace sla {

constexpr int REC_CHUNKS = 512;                          // 16-byte chunks per 32-token record
constexpr float QK_LOG2 = LOG2E / 11.313708498984761f;   // log2(e) / sqrt(d)
constexpr float INV_SQRT_D = 1.0f / 11.313708498984761f;

__device__ __forceinline__ v8bf as_v8bf(const uint4& x) { return __builtin_bit_cast(v8bf, x); }
__device__ __forceinline__ v16f mfma_bf16(const uint4& a, const uint4& b, const v16f& c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_v8bf(a), as_v8bf(b), c, 0, 0, 0);
}
// Accumulator registers 8 s .. 8 s + 7 of a tile as a bf16 operand: contraction step s (16 rows) of
// the product that contracts over the tile's rows.  Row of element kk for lane half hf:
// 16 s + 8 (kk / 4) + 4 hf + kk % 4 -- the order the t-records are written in.
__device__ __forceinline__ uint4 acc_operand(const v16f& a, int s) {
  return uint4{pack_bf16x2(a[8 * s], a[8 * s + 1]), pack_bf16x2(a[8 * s + 2], a[8 * s + 3]),
               pack_bf16x2(a[8 * s + 4], a[8 * s + 5]), pack_bf16x2(a[8 * s + 6], a[8 * s + 7])};
}

// ---------------------------------------------------------------------------------------------
// Records.  Tile T of a [N, 128] tensor X (rows 32 T .. 32 T + 31, zero beyond N):
//   n-record  chunk ks * 64 + lane           = X[32 T + lane % 32][16 ks + 8 (lane / 32) + 0..7]
//   t-record  chunk (ct * 2 + s) * 64 + lane = X[32 T + 16 s + 8 (kk / 4) + 4 (lane / 32) + kk % 4][32 ct + lane % 32], kk = 0..7
// One wavefront per tile.
__global__ void __launch_bounds__(64) bwd_pack_kernel(const bf16_t* __restrict__ x, Layout L, int H, int N, int T32,
                                                      uint4* __restrict__ nrec, uint4* __restrict__ trec) {
  __shared__ __attribute__((aligned(16))) bf16_t tile[32][136];
  const int T = blockIdx.x, bh = blockIdx.y, lane = threadIdx.x, l32 = lane & 31, hf = lane >> 5;
  const int b = bh / H, h = bh - b * H;
  const bf16_t* src = x + b * L.sb + h * L.sh;
#pragma unroll
  for (int it = 0; it < 8; ++it) {
    const int c = it * 64 + lane, row = c >> 4, cc = c & 15;
    const long long r = 32ll * T + row;
    uint4 v = uint4{0u, 0u, 0u, 0u};
    if (r < N) v = *(const uint4*)(src + r * L.sn + cc * 8);
    *(uint4*)&tile[row][cc * 8] = v;
  }
  __syncthreads();
  const size_t base = ((size_t)bh * T32 + T) * REC_CHUNKS;
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) nrec[base + ks * 64 + lane] = *(const uint4*)&tile[l32][16 * ks + 8 * hf];
#pragma unroll
  for (int ct = 0; ct < 4; ++ct) {
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      uint32_t w[4];
#pragma unroll
      for (int kk = 0; kk < 8; kk += 2) {
        const int r0 = 16 * s + 8 * (kk >> 2) + 4 * hf + (kk & 3);
        w[kk >> 1] = (uint32_t)tile[r0][32 * ct + l32] | ((uint32_t)tile[r0 + 1][32 * ct + l32] << 16);
      }
      trec[base + (ct * 2 + s) * 64 + lane] = uint4{w[0], w[1], w[2], w[3]};
    }
  }
}

// Shared skeleton of the two per-query-block kernels: NW wavefronts, wavefront w owns tile
// T = i NW + w of query block i; per critical key block, NREC records of 1024 chunks (the block's
// two key tiles) are staged in LDS through registers, one block ahead.
template <int NW, int NREC>
struct KeyStage {
  static constexpr int PER = NREC * 2 * REC_CHUNKS / (NW * 64);  // chunks per thread per key block
  uint4 pf[PER];
  __device__ __forceinline__ void load(const uint4* const (&src)[NREC], size_t rec0, int t) {
#pragma unroll
    for (int u = 0; u < PER; ++u) {
      const int c = u * NW * 64 + t;                 // chunk of the staged step
      const int which = c / (2 * REC_CHUNKS);        // (compile-time per u: NW * 64 divides 1024)
      pf[u] = src[which][rec0 + (c - which * 2 * REC_CHUNKS)];
    }
  }
  __device__ __forceinline__ void store(uint4* lds, int t) const {
#pragma unroll
    for (int u = 0; u < PER; ++u) lds[u * NW * 64 + t] = pf[u];
  }
};

struct BwdDims {
  int N, Tq, Tk, n_c, T32q, T32k;
};

// Scaled scores of one key tile, transposed: lane = query, registers = keys.
__device__ __forceinline__ v16f score_tile(const uint4* kn_tile, const uint4 (&qf)[8], int lane) {
  v16f s = v16f{};
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) s = mfma_bf16(kn_tile[ks * 64 + lane], qf[ks], s);
  return s;
}

// lse2[bh][32 T + r], delta[bh][32 T + r] for every token row of every query tile (rows beyond N:
// lse2 = +inf, delta = 0, so that their P is exactly 0 wherever they are used).
template <int NW>
__global__ void __launch_bounds__(NW * 64) bwd_stats_kernel(const uint4* __restrict__ qn, const uint4* __restrict__ kn,
                                                            const uint4* __restrict__ vt, const bf16_t* __restrict__ dout,
                                                            const int32_t* __restrict__ crit, float* __restrict__ lse2,
                                                            float* __restrict__ delta, BwdDims dm) {
  __shared__ uint4 lds[2 * 2 * REC_CHUNKS];  // Kn then Vt of the current key block
  const int i = blockIdx.x, bh = blockIdx.y, t = threadIdx.x, lane = t & 63, w = t >> 6, l32 = lane & 31, hf = lane >> 5;
  const int T = i * NW + w;
  const long long q = 32ll * T + l32;
  const bool qok = q < dm.N;
  uint4 qf[8];
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) qf[ks] = qn[((size_t)bh * dm.T32q + T) * REC_CHUNKS + ks * 64 + lane];
  const int32_t* crow = crit + ((size_t)bh * dm.Tq + i) * dm.n_c;
  const uint4* const srcs[2] = {kn, vt};
  KeyStage<NW, 2> st;
  v16f o[4];
#pragma unroll
  for (int ct = 0; ct < 4; ++ct) o[ct] = v16f{};
  float m = -INFINITY, lsum = 0.f;
  if (dm.n_c > 0) st.load(srcs, ((size_t)bh * dm.T32k + 2 * crow[0]) * REC_CHUNKS, t);
  for (int b = 0; b < dm.n_c; ++b) {
    const int j = crow[b];
    __syncthreads();
    st.store(lds, t);
    __syncthreads();
    if (b + 1 < dm.n_c) st.load(srcs, ((size_t)bh * dm.T32k + 2 * crow[b + 1]) * REC_CHUNKS, t);
    v16f s[2];
    float mx = -INFINITY;
#pragma unroll
    for (int kt = 0; kt < 2; ++kt) {
      s[kt] = score_tile(lds + kt * REC_CHUNKS, qf, lane);
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int key = 64 * j + 32 * kt + 8 * (r >> 2) + 4 * hf + (r & 3);
        s[kt][r] = key < dm.N ? s[kt][r] * QK_LOG2 : -INFINITY;
        mx = fmaxf(mx, s[kt][r]);
      }
    }
    mx = fmaxf(mx, partner_f32(mx));
    const float m_new = fmaxf(m, mx);           // finite: a block holds at least one valid key
    const float alpha = __builtin_amdgcn_exp2f(m - m_new);
    m = m_new;
    float rs = 0.f;
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        s[kt][r] = __builtin_amdgcn_exp2f(s[kt][r] - m_new);
        rs += s[kt][r];
      }
    lsum = lsum * alpha + rs;
#pragma unroll
    for (int ct = 0; ct < 4; ++ct)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[ct][r] *= alpha;
    const uint4* vtl = lds + 2 * REC_CHUNKS;
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
      for (int sidx = 0; sidx < 2; ++sidx) {
        const uint4 pb = acc_operand(s[kt], sidx);
#pragma unroll
        for (int ct = 0; ct < 4; ++ct)
          o[ct] = mfma_bf16(vtl[kt * REC_CHUNKS + (ct * 2 + sidx) * 64 + lane], pb, o[ct]);
      }
  }
  const float l = lsum + partner_f32(lsum);
  float dl = 0.f;
  if (qok && dm.n_c > 0) {
    const bf16_t* drow = dout + ((size_t)bh * dm.N + q) * D;
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

template <int NW>
__global__ void __launch_bounds__(NW * 64) bwd_dq_kernel(const uint4* __restrict__ qn, const uint4* __restrict__ don,
                                                         const uint4* __restrict__ kn, const uint4* __restrict__ ktr,
                                                         const uint4* __restrict__ vn, const int32_t* __restrict__ crit,
                                                         const float* __restrict__ lse2, const float* __restrict__ delta,
                                                         const float* __restrict__ dq_lin, bf16_t* __restrict__ dq,
                                                         BwdDims dm) {
  __shared__ uint4 lds[3 * 2 * REC_CHUNKS];  // Kn, Kt, Vn of the current key block
  const int i = blockIdx.x, bh = blockIdx.y, t = threadIdx.x, lane = t & 63, w = t >> 6, l32 = lane & 31, hf = lane >> 5;
  const int T = i * NW + w;
  const long long q = 32ll * T + l32;
  uint4 qf[8], dof[8];
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) {
    qf[ks] = qn[((size_t)bh * dm.T32q + T) * REC_CHUNKS + ks * 64 + lane];
    dof[ks] = don[((size_t)bh * dm.T32q + T) * REC_CHUNKS + ks * 64 + lane];
  }
  const size_t sidx = (size_t)bh * dm.T32q * 32 + 32 * T + l32;
  const float lse_q = lse2[sidx], delta_q = delta[sidx];
  const int32_t* crow = crit + ((size_t)bh * dm.Tq + i) * dm.n_c;
  const uint4* const srcs[3] = {kn, ktr, vn};
  KeyStage<NW, 3> st;
  v16f acc[4];
#pragma unroll
  for (int ct = 0; ct < 4; ++ct) acc[ct] = v16f{};
  if (dm.n_c > 0) st.load(srcs, ((size_t)bh * dm.T32k + 2 * crow[0]) * REC_CHUNKS, t);
  for (int b = 0; b < dm.n_c; ++b) {
    const int j = crow[b];
    __syncthreads();
    st.store(lds, t);
    __syncthreads();
    if (b + 1 < dm.n_c) st.load(srcs, ((size_t)bh * dm.T32k + 2 * crow[b + 1]) * REC_CHUNKS, t);
    const uint4* knl = lds;
    const uint4* ktl = lds + 2 * REC_CHUNKS;
    const uint4* vnl = lds + 4 * REC_CHUNKS;
#pragma unroll
    for (int kt = 0; kt < 2; ++kt) {
      v16f s = score_tile(knl + kt * REC_CHUNKS, qf, lane);
      v16f dp = v16f{};
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) dp = mfma_bf16(vnl[kt * REC_CHUNKS + ks * 64 + lane], dof[ks], dp);
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int key = 64 * j + 32 * kt + 8 * (r >> 2) + 4 * hf + (r & 3);
        const float p = key < dm.N ? __builtin_amdgcn_exp2f(s[r] * QK_LOG2 - lse_q) : 0.f;
        s[r] = p * (dp[r] - delta_q);
      }
#pragma unroll
      for (int sx = 0; sx < 2; ++sx) {
        const uint4 dsb = acc_operand(s, sx);
#pragma unroll
        for (int ct = 0; ct < 4; ++ct)
          acc[ct] = mfma_bf16(ktl[kt * REC_CHUNKS + (ct * 2 + sx) * 64 + lane], dsb, acc[ct]);
      }
    }
  }
  if (q < dm.N) {
    const size_t row = ((size_t)bh * dm.N + q) * D;
#pragma unroll
    for (int ct = 0; ct < 4; ++ct)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int ch = 32 * ct + 8 * g + 4 * hf;
        store_grad4(dq + row + ch, dq_lin ? dq_lin + row + ch : nullptr, acc[ct][4 * g] * INV_SQRT_D,
                    acc[ct][4 * g + 1] * INV_SQRT_D, acc[ct][4 * g + 2] * INV_SQRT_D, acc[ct][4 * g + 3] * INV_SQRT_D);
      }
  }
}

// One workgroup of two wavefronts per key block; wavefront w owns key tile 2 j + w (one key per
// lane pair).  The query blocks that hold block j as critical are found from the mask column.
constexpr int DKV_MAX_TQ = 8192;
__global__ void __launch_bounds__(128) bwd_dkv_kernel(const uint4* __restrict__ qn, const uint4* __restrict__ qtr,
                                                      const uint4* __restrict__ don, const uint4* __restrict__ dotr,
                                                      const uint4* __restrict__ kn, const uint4* __restrict__ vn,
                                                      const int8_t* __restrict__ mask, const float* __restrict__ lse2,
                                                      const float* __restrict__ delta, const float* __restrict__ dk_lin,
                                                      const float* __restrict__ dv_lin, bf16_t* __restrict__ dk,
                                                      bf16_t* __restrict__ dv, int tiles_per_qblock, BwdDims dm) {
  __shared__ uint4 lds[4 * REC_CHUNKS];  // Qn, Qt, dOn, dOt of the current query tile
  __shared__ __attribute__((aligned(16))) float stat[2][32];
  __shared__ unsigned short qlist[DKV_MAX_TQ];
  __shared__ int wcnt[2];
  const int j = blockIdx.x, bh = blockIdx.y, t = threadIdx.x, lane = t & 63, w = t >> 6, l32 = lane & 31, hf = lane >> 5;
  // ---- the query blocks of this key block, ascending
  int nq = 0;
  for (int base = 0; base < dm.Tq; base += 128) {
    const int i = base + t;
    const bool hit = i < dm.Tq && mask[((size_t)bh * dm.Tq + i) * dm.Tk + j] == 1;
    const unsigned long long bal = __ballot(hit);
    if (lane == 0) wcnt[w] = __popcll(bal);
    __syncthreads();
    const int off = nq + (w ? wcnt[0] : 0) + __popcll(bal & ((1ull << lane) - 1ull));
    if (hit) qlist[off] = (unsigned short)i;
    nq += wcnt[0] + wcnt[1];
    __syncthreads();
  }
  const int Tkey = 2 * j + w;
  const long long key = 32ll * Tkey + l32;
  const bool kok = key < dm.N;
  uint4 kf[8], vf[8];
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) {
    kf[ks] = kn[((size_t)bh * dm.T32k + Tkey) * REC_CHUNKS + ks * 64 + lane];
    vf[ks] = vn[((size_t)bh * dm.T32k + Tkey) * REC_CHUNKS + ks * 64 + lane];
  }
  v16f dkt[4], dvt[4];
#pragma unroll
  for (int ct = 0; ct < 4; ++ct) {
    dkt[ct] = v16f{};
    dvt[ct] = v16f{};
  }
  const int steps = nq * tiles_per_qblock;
  const uint4* const srcs[4] = {qn, qtr, don, dotr};
  uint4 pf[16];
  float pstat = 0.f;
  auto load = [&](int step) {
    const int T = qlist[step / tiles_per_qblock] * tiles_per_qblock + step % tiles_per_qblock;
    const size_t rec0 = ((size_t)bh * dm.T32q + T) * REC_CHUNKS;
#pragma unroll
    for (int u = 0; u < 16; ++u) pf[u] = srcs[u >> 2][rec0 + (u & 3) * 128 + t];
    if (t < 64) pstat = (t < 32 ? lse2 : delta)[(size_t)bh * dm.T32q * 32 + 32 * T + (t & 31)];
  };
  if (steps > 0) load(0);
  for (int step = 0; step < steps; ++step) {
    __syncthreads();
#pragma unroll
    for (int u = 0; u < 16; ++u) lds[(u >> 2) * REC_CHUNKS + (u & 3) * 128 + t] = pf[u];
    if (t < 64) stat[t >> 5][t & 31] = pstat;
    __syncthreads();
    if (step + 1 < steps) load(step + 1);
    const uint4* qnl = lds;
    const uint4* qtl = lds + REC_CHUNKS;
    const uint4* donl = lds + 2 * REC_CHUNKS;
    const uint4* dotl = lds + 3 * REC_CHUNKS;
    v16f s = v16f{}, dp = v16f{};
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      s = mfma_bf16(qnl[ks * 64 + lane], kf[ks], s);
      dp = mfma_bf16(donl[ks * 64 + lane], vf[ks], dp);
    }
    v16f p;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const float4 ls = *(const float4*)&stat[0][8 * g + 4 * hf];
      const float4 dl = *(const float4*)&stat[1][8 * g + 4 * hf];
      const float lsv[4] = {ls.x, ls.y, ls.z, ls.w}, dlv[4] = {dl.x, dl.y, dl.z, dl.w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float pe = kok ? __builtin_amdgcn_exp2f(s[4 * g + e] * QK_LOG2 - lsv[e]) : 0.f;
        p[4 * g + e] = pe;
        s[4 * g + e] = pe * (dp[4 * g + e] - dlv[e]);
      }
    }
#pragma unroll
    for (int sx = 0; sx < 2; ++sx) {
      const uint4 pb = acc_operand(p, sx), dsb = acc_operand(s, sx);
#pragma unroll
      for (int ct = 0; ct < 4; ++ct) {
        dvt[ct] = mfma_bf16(dotl[(ct * 2 + sx) * 64 + lane], pb, dvt[ct]);
        dkt[ct] = mfma_bf16(qtl[(ct * 2 + sx) * 64 + lane], dsb, dkt[ct]);
      }
    }
  }
  if (kok) {
    const size_t row = ((size_t)bh * dm.N + key) * D;
#pragma unroll
    for (int ct = 0; ct < 4; ++ct)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int ch = 32 * ct + 8 * g + 4 * hf;
        store_grad4(dk + row + ch, dk_lin ? dk_lin + row + ch : nullptr, dkt[ct][4 * g] * INV_SQRT_D,
                    dkt[ct][4 * g + 1] * INV_SQRT_D, dkt[ct][4 * g + 2] * INV_SQRT_D, dkt[ct][4 * g + 3] * INV_SQRT_D);
        store_grad4(dv + row + ch, dv_lin ? dv_lin + row + ch : nullptr, dvt[ct][4 * g], dvt[ct][4 * g + 1],
                    dvt[ct][4 * g + 2], dvt[ct][4 * g + 3]);
      }
  }
}

// ---------------------------------------------------------------------------------------------
void launch_bwd_pack(const void* x, const Layout& L, const Problem& p, int T32, uint4* nrec, uint4* trec,
                     hipStream_t stream) {
  bwd_pack_kernel<<<dim3((unsigned)T32, (unsigned)p.BH), 64, 0, stream>>>((const bf16_t*)x, L, p.H, p.N, T32, nrec, trec);
}

static BwdDims bwd_dims(const Problem& p) {
  return BwdDims{p.N, p.Tq, p.Tk, p.n_c, p.Tq * (p.block_q / 32), p.Tk * 2};
}

void launch_bwd_stats(const Problem& p, const uint4* qn, const uint4* kn, const uint4* vt, const void* dout,
                      const int32_t* crit, float* lse2, float* delta, hipStream_t stream) {
  const dim3 grid((unsigned)p.Tq, (unsigned)p.BH);
  if (p.block_q == 128)
    bwd_stats_kernel<4><<<grid, 256, 0, stream>>>(qn, kn, vt, (const bf16_t*)dout, crit, lse2, delta, bwd_dims(p));
  else
    bwd_stats_kernel<2><<<grid, 128, 0, stream>>>(qn, kn, vt, (const bf16_t*)dout, crit, lse2, delta, bwd_dims(p));
}

void launch_bwd_dq(const Problem& p, const uint4* qn, const uint4* don, const uint4* kn, const uint4* ktr,
                   const uint4* vn, const int32_t* crit, const float* lse2, const float* delta, const float* dq_lin,
                   void* dq, hipStream_t stream) {
  const dim3 grid((unsigned)p.Tq, (unsigned)p.BH);
  if (p.block_q == 128)
    bwd_dq_kernel<4><<<grid, 256, 0, stream>>>(qn, don, kn, ktr, vn, crit, lse2, delta, dq_lin, (bf16_t*)dq, bwd_dims(p));
  else
    bwd_dq_kernel<2><<<grid, 128, 0, stream>>>(qn, don, kn, ktr, vn, crit, lse2, delta, dq_lin, (bf16_t*)dq, bwd_dims(p));
}

void launch_bwd_dkv(const Problem& p, const uint4* qn, const uint4* qtr, const uint4* don, const uint4* dotr,
                    const uint4* kn, const uint4* vn, const int8_t* mask, const float* lse2, const float* delta,
                    const float* dk_lin, const float* dv_lin, void* dk, void* dv, hipStream_t stream) {
  bwd_dkv_kernel<<<dim3((unsigned)p.Tk, (unsigned)p.BH), 128, 0, stream>>>(qn, qtr, don, dotr, kn, vn, mask, lse2, delta,
                                                                         dk_lin, dv_lin, (bf16_t*)dk, (bf16_t*)dv,
                                                                         p.block_q / 32, bwd_dims(p));
}

}  // namespace sla
