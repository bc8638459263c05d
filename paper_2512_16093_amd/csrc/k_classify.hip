// Block pooling / statistics, pooled scores and the three-way block selection.
//
// Steps 1-2 of the path: per-block channel means of Q and K, the score
// s[i][j] = mean(Q_i).mean(K_j)/sqrt(d), and per query block the n_c best key
// blocks (critical), the next n_m (marginal), the rest negligible, equal scores
// ranking by ascending j (Section 2.1 fixes only the Top-K ratio; the rest is
// this library's stated reading, see sla.h).  The same pass over Q, K, V also
// produces what the low-bit branch needs later: the per-query-block INT8 scale,
// the channel mean of K (K-smoothing) and the per-channel max |V| (FP8 scale).
#include "common.h"

namespace sla {

// ---------------------------------------------------------------------------
// pool_stats: one workgroup per (b,h, 128-token group); 256 threads; thread
// (rg = t/16, cg = t%16) reads 8 channels of rows rg + 16 r, r = 0..7.
// HBM-bound: reads Q, K, V exactly once (6 N d bytes per slice).
// ---------------------------------------------------------------------------
__global__ void __launch_bounds__(256) pool_stats_kernel(
    const bf16_t* __restrict__ q, const bf16_t* __restrict__ k, const bf16_t* __restrict__ v,
    int N, int block_q, int Tq, int Tk, int groups, int H, Layout lq, Layout lk, Layout lv,
    float* __restrict__ qbar, float* __restrict__ kbar, float* __restrict__ dq,
    uint32_t* __restrict__ amax_v, int8_t* __restrict__ q8) {
  __shared__ float sQ[16][2][D];
  __shared__ float s_qmax[2];
  __shared__ float sK[16][2][D];
  __shared__ float sV[16][D];
  __shared__ float sQa[2][256];
  const int bh = blockIdx.x / groups, g = blockIdx.x % groups;
  const int t = threadIdx.x, cg = t & 15, rg = t >> 4;
  const int b_ = bh / H, h_ = bh - b_ * H;
  const bf16_t* qs_ = q + b_ * lq.sb + h_ * lq.sh;
  const bf16_t* ks_ = k + b_ * lk.sb + h_ * lk.sh;
  const bf16_t* vs_ = v + b_ * lv.sb + h_ * lv.sh;
  const int row0 = g * 128;

  float qs[2][8] = {}, ks[2][8] = {}, va[8] = {}, qa[2] = {0.f, 0.f};
  uint4 qkeep[8];  // this thread's Q values, kept for the codes (formed once the block maxima are known)
#pragma unroll
  for (int r = 0; r < 8; ++r) {
    const int row = row0 + rg + 16 * r, half = r >> 2;
    qkeep[r] = make_uint4(0u, 0u, 0u, 0u);
    if (row < N) {
      const uint4 xq = *(const uint4*)(qs_ + row * lq.sn + cg * 8);
      qkeep[r] = xq;
      const uint4 xk = *(const uint4*)(ks_ + row * lk.sn + cg * 8);
      const uint4 xv = *(const uint4*)(vs_ + row * lv.sn + cg * 8);
      const uint32_t wq[4] = {xq.x, xq.y, xq.z, xq.w}, wk[4] = {xk.x, xk.y, xk.z, xk.w},
                     wv[4] = {xv.x, xv.y, xv.z, xv.w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float q0 = bf16_lo(wq[e]), q1 = bf16_hi(wq[e]);
        qs[half][2 * e] += q0;
        qs[half][2 * e + 1] += q1;
        qa[half] = fmaxf(qa[half], fmaxf(fabsf(q0), fabsf(q1)));
        ks[half][2 * e] += bf16_lo(wk[e]);
        ks[half][2 * e + 1] += bf16_hi(wk[e]);
        va[2 * e] = fmaxf(va[2 * e], fabsf(bf16_lo(wv[e])));
        va[2 * e + 1] = fmaxf(va[2 * e + 1], fabsf(bf16_hi(wv[e])));
      }
    }
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    sQ[rg][0][cg * 8 + e] = qs[0][e];
    sQ[rg][1][cg * 8 + e] = qs[1][e];
    sK[rg][0][cg * 8 + e] = ks[0][e];
    sK[rg][1][cg * 8 + e] = ks[1][e];
    sV[rg][cg * 8 + e] = va[e];
  }
  sQa[0][t] = qa[0];
  sQa[1][t] = qa[1];
  __syncthreads();

  const int half = t >> 7, c = t & 127;
  float sq = 0.f, sk = 0.f;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    sq += sQ[r][half][c];
    sk += sK[r][half][c];
  }
  const int cnt0 = min(64, max(0, N - row0)), cnt1 = min(64, max(0, N - row0 - 64));
  const int cnt = half ? cnt1 : cnt0;
  if (cnt > 0) kbar[((size_t)bh * Tk + 2 * g + half) * D + c] = sk / (float)cnt;
  if (block_q == 64) {
    if (cnt > 0) qbar[((size_t)bh * Tq + 2 * g + half) * D + c] = sq / (float)cnt;
  } else {
    // both halves belong to query block g: combine the two partial sums
    __syncthreads();
    sQ[0][half][c] = sq;
    __syncthreads();
    if (half == 0) qbar[((size_t)bh * Tq + g) * D + c] = (sQ[0][0][c] + sQ[0][1][c]) / (float)(cnt0 + cnt1);
  }
  if (t < 128) {
    float m = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) m = fmaxf(m, sV[r][t]);
    // max of non-negative floats == max of their bit patterns: order-independent, exact
    atomicMax(amax_v + (size_t)bh * D + t, __float_as_uint(m));
  }
  if (t < 64) {  // wave 0 reduces the |Q| maxima of both halves
    float m0 = 0.f, m1 = 0.f;
    for (int r = t; r < 256; r += 64) {
      m0 = fmaxf(m0, sQa[0][r]);
      m1 = fmaxf(m1, sQa[1][r]);
    }
    for (int o = 32; o > 0; o >>= 1) {
      m0 = fmaxf(m0, __shfl_xor(m0, o));
      m1 = fmaxf(m1, __shfl_xor(m1, o));
    }
    if (t == 0) {
      if (block_q == 64) {
        if (cnt0 > 0) dq[(size_t)bh * Tq + 2 * g] = m0 > 0.f ? m0 / 127.0f : 1.0f;
        if (cnt1 > 0) dq[(size_t)bh * Tq + 2 * g + 1] = m1 > 0.f ? m1 / 127.0f : 1.0f;
        s_qmax[0] = m0;
        s_qmax[1] = m1;
      } else {
        const float m = fmaxf(m0, m1);
        dq[(size_t)bh * Tq + g] = m > 0.f ? m / 127.0f : 1.0f;
        s_qmax[0] = s_qmax[1] = m;
      }
    }
  }
  // ---- INT8 codes of Q at the scale just found (max|Q block| / 127), ties exact: every row's 128 bytes in the
  // order the attention kernel's lanes take them (q8_byte_offset); this thread: 8 adjacent bytes of 8 rows.
  if (q8 == nullptr) return;  // (uniform)
  __syncthreads();
  int8_t* dst = q8 + ((size_t)(bh * groups + g) * 128) * D + q8_byte_offset(cg * 8);
#pragma unroll
  for (int r = 0; r < 8; ++r) {
    const int rl = rg + 16 * r;
    if (row0 + rl >= N) continue;
    const CodeScale cs = code_scale(s_qmax[r >> 2], 127.0f);
    const uint32_t wq[4] = {qkeep[r].x, qkeep[r].y, qkeep[r].z, qkeep[r].w};
    uint32_t c[8];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      c[2 * e] = int8_code_word_exact(bf16_lo(wq[e]), cs);
      c[2 * e + 1] = int8_code_word_exact(bf16_hi(wq[e]), cs);
    }
    *(uint2*)(dst + (size_t)rl * D) = make_uint2(pack_low_bytes(c[0], c[1], c[2], c[3]), pack_low_bytes(c[4], c[5], c[6], c[7]));
  }
}

__global__ void zero_u32_kernel(uint32_t* p, size_t n) {
  size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0u;
}

// finalize_stats: eight workgroups of 1024 threads per (b,h), each for 16 channels:
// mu_K[c] = sum_j cnt_j kbar[j][c] / N (summed in a fixed order), delta_V[c] = max|V[:,c]| / 448
// (1 if zero).  Workgroup 0 also lays the output projection (the identity if none is given) out
// in the order in which prep_kv's first product takes it as the B operand of
// v_mfma_f32_32x32x16_bf16: 16-byte chunk [tile of 32 output channels][step of 16 input
// channels][lane] = W[32 tile + lane % 32][16 step + 8 (lane / 32) + 0..7], so that a wavefront
// fetches an operand as one contiguous KiB.
__global__ void __launch_bounds__(1024) finalize_stats_kernel(
    const float* __restrict__ kbar, const uint32_t* __restrict__ amax_v, int N, int Tk,
    float* __restrict__ mu_k, float* __restrict__ dv, const bf16_t* __restrict__ proj_w,
    bf16_t* __restrict__ wfrag) {
  __shared__ float red[64][17];
  const int bh = blockIdx.x >> 3, c0 = (blockIdx.x & 7) * 16, t = threadIdx.x, cl = t & 15, rgrp = t >> 4;
  float s = 0.f;
  for (int j = rgrp; j < Tk; j += 64) {
    const int cnt = min(BK, N - j * BK);
    s += kbar[((size_t)bh * Tk + j) * D + c0 + cl] * (float)cnt;
  }
  red[rgrp][cl] = s;
  __syncthreads();
  if (t < 16) {
    float tot = 0.f;
    for (int r = 0; r < 64; ++r) tot += red[r][t];
    mu_k[(size_t)bh * D + c0 + t] = tot / (float)N;
    const float am = __uint_as_float(amax_v[(size_t)bh * D + c0 + t]);
    dv[(size_t)bh * D + c0 + t] = am > 0.f ? am / E4M3_MAX : 1.0f;
  }
  if (blockIdx.x == 0) {
    for (int idx = t; idx < D * D / 8; idx += 1024) {
      const int lane = idx & 63, row = 32 * (idx >> 9) + (lane & 31), col = 16 * ((idx >> 6) & 7) + 8 * (lane >> 5);
      for (int e = 0; e < 8; ++e)
        wfrag[idx * 8 + e] = proj_w ? proj_w[row * D + col + e] : (row == col + e ? (bf16_t)0x3f80 : (bf16_t)0);
    }
  }
}

// scores: s[bh][i][j] = qbar_i . kbar_j / sqrt(d) in fp32 on the matrix pipe
// (v_mfma_f32_32x32x2_f32: fp32 operands and accumulation, the vector-fp32 rate without its issue
// limits).  A wavefront owns a 32-row tile of query blocks, whose means it keeps in registers, and
// sweeps SC_JT 32-column tiles of key blocks; the four wavefronts of a workgroup take four
// consecutive row tiles over the SAME columns, so three of their four reads of a key tile hit
// the L1.  The instruction contracts two channels per step, one per lane half; which two is
// free as long as both operands agree: lane half h holds channels 64 h .. 64 h + 63 of its row
// (16 contiguous 16-byte loads) and step t contracts channels t and 64 + t.
constexpr int SC_JT = 4;
typedef float v16f_sc __attribute__((ext_vector_type(16)));
__global__ void __launch_bounds__(256, 2) scores_kernel(const float* __restrict__ qbar,
                                                        const float* __restrict__ kbar, int Tq, int Tk,
                                                        float* __restrict__ scores) {
  const int bh = blockIdx.z, lane = threadIdx.x & 63, w = threadIdx.x >> 6, l32 = lane & 31, h = lane >> 5;
  const int i0 = (blockIdx.y * 4 + w) * 32;
  if (i0 >= Tq) return;  // (whole wavefront; no barriers in this kernel)
  const int jt0 = blockIdx.x * SC_JT, jts = (Tk + 31) / 32;
  float a[64], b[64];
  {
    const float4* src = (const float4*)(qbar + ((size_t)bh * Tq + min(i0 + l32, Tq - 1)) * D + 64 * h);
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      const float4 x = src[u];
      a[4 * u] = x.x; a[4 * u + 1] = x.y; a[4 * u + 2] = x.z; a[4 * u + 3] = x.w;
    }
  }
  auto load_b = [&](int jt) {
    const float4* src = (const float4*)(kbar + ((size_t)bh * Tk + min(jt * 32 + l32, Tk - 1)) * D + 64 * h);
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      const float4 x = src[u];
      b[4 * u] = x.x; b[4 * u + 1] = x.y; b[4 * u + 2] = x.z; b[4 * u + 3] = x.w;
    }
  };
  for (int jt = jt0; jt < min(jt0 + SC_JT, jts); ++jt) {
    load_b(jt);
    v16f_sc acc = {};
#pragma unroll
    for (int t = 0; t < 64; ++t) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[t], b[t], acc, 0, 0, 0);
    // accumulator register r of lane (l32, h): row 8 (r / 4) + 4 h + r % 4, column l32
    const int j = jt * 32 + l32;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int i = i0 + 8 * (r >> 2) + 4 * h + (r & 3);
      if (i < Tq && j < Tk) scores[((size_t)bh * Tq + i) * Tk + j] = acc[r] / 11.313708498984761f;
    }
  }
}

// select: one WAVEFRONT per (b,h,i) row; the row's scores live in registers (KPL per lane,
// block j = lane + 64 m in register m) as order-preserving 32-bit keys.  The n_c-th and the
// (n_c+n_m)-th largest keys are found exactly, bit by bit from the top: a bit of the threshold
// is set when at least `rank` keys are >= the candidate with that bit set.  The counts come
// from wave-wide compares (one vector compare per register, the population count and the sum
// on the scalar unit), so there is no shared-memory traffic and no atomic.  Blocks whose key
// equals a threshold key are ranked by ascending j with ballots, so equal scores rank by
// ascending block index and the result is exact and deterministic.  Outputs: the int8 mask
// row, the ascending critical list, and the marginal ballots as words of the bit matrix the
// accumulation kernel reads (see lin_accumulate).
__device__ __forceinline__ uint32_t order_bits(float f) {
  const uint32_t u = __float_as_uint(f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

template <int KPL>
__global__ void __launch_bounds__(256) select_kernel(const float* __restrict__ scores, int rows, int Tq, int Tk,
                                                     int n_c, int n_m, int8_t* __restrict__ mask,
                                                     int32_t* __restrict__ crit, int32_t* __restrict__ marg,
                                                     uint32_t* __restrict__ mbits) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const size_t row = (size_t)blockIdx.x * 4 + w;
  if (row >= (size_t)rows) return;  // whole wavefront; no workgroup barrier is used below
  const float* srow = scores + row * Tk;
  uint32_t key[KPL];
#pragma unroll
  for (int m = 0; m < KPL; ++m) {
    const int j = lane + 64 * m;
    key[m] = j < Tk ? order_bits(srow[j]) : 0u;
  }
  // Subtract the row minimum and shift out the common leading zeros: order and ties are
  // unchanged, padding (key 0) ties with the minimum, and the search below only has to visit
  // the bits in which the keys can differ.
  int low;
  {
    uint32_t kmin = 0xffffffffu, kmax = 0u;
#pragma unroll
    for (int m = 0; m < KPL; ++m)
      if (lane + 64 * m < Tk) {
        kmin = min(kmin, key[m]);
        kmax = max(kmax, key[m]);
      }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      kmin = min(kmin, (uint32_t)__shfl_xor((int)kmin, o));
      kmax = max(kmax, (uint32_t)__shfl_xor((int)kmax, o));
    }
    const uint32_t span = kmax - kmin;
    const int lz = span ? __builtin_clz(span) : 0;
    low = span ? lz : 32;  // all keys equal: nothing to search
#pragma unroll
    for (int m = 0; m < KPL; ++m) key[m] = (lane + 64 * m < Tk) ? ((key[m] - kmin) << lz) : 0u;  // padding ties with the minimum: never above a threshold
  }
  // k1 / k2: the n_c-th / (n_c+n_m)-th largest key; t1 / t2: how many of the keys equal to
  // it belong to the top n_c / n_c+n_m (>= 1).  Bits below `low` are zero in every key.
  // A threshold's search stops early once exactly the wanted number of keys reaches the
  // candidate c: the set is then {key >= c}, which the code below takes as "key > c - 1" with
  // no ties to rank (with ~1000 distinct keys that happens after about log2(Tk) + 2 bits).
  uint32_t k1 = 0, k2 = 0;
  const int rank2 = n_c + n_m;
  bool open1 = true, open2 = n_m > 0;
  for (int bit = 31; bit >= low && (open1 || open2); --bit) {
    const uint32_t c1 = k1 | (1u << bit), c2 = k2 | (1u << bit);
    int n1 = 0, n2 = 0;
#pragma unroll
    for (int m = 0; m < KPL; ++m) {  // (padding keys are 0 and never reach a candidate)
      if (open1) n1 += __popcll(__ballot(key[m] >= c1));
      if (open2) n2 += __popcll(__ballot(key[m] >= c2));
    }
    if (open1) {
      if (n1 == n_c) { k1 = c1 - 1u; open1 = false; }
      else if (n1 > n_c) k1 = c1;
    }
    if (open2) {
      if (n2 == rank2) { k2 = c2 - 1u; open2 = false; }
      else if (n2 > rank2) k2 = c2;
    }
  }
  int t1 = n_c, t2 = rank2;
#pragma unroll
  for (int m = 0; m < KPL; ++m) {
    t1 -= __popcll(__ballot(key[m] > k1));
    if (n_m > 0) t2 -= __popcll(__ballot(key[m] > k2));
  }

  const unsigned long long lt = (1ull << lane) - 1ull;
  const int bh = (int)(row / Tq), i = (int)(row % Tq);
  const int KT = (Tk + 31) / 32, TqP = (Tq + 383) / 384 * 384 + 128;  // layout of the marginal bit matrix (see lin_accumulate)
  int eq1 = 0, eq2 = 0, nc = 0, nm = 0;  // running counts in ascending-j order
#pragma unroll
  for (int m = 0; m < KPL; ++m) {
    const int j = lane + 64 * m;
    if (64 * m >= Tk) break;
    const bool valid = j < Tk;
    const bool e1 = valid && key[m] == k1, e2 = valid && n_m > 0 && key[m] == k2;
    const unsigned long long b1 = __ballot(e1), b2 = __ballot(e2);
    const int r1 = eq1 + __popcll(b1 & lt), r2 = eq2 + __popcll(b2 & lt);
    eq1 += __popcll(b1);
    eq2 += __popcll(b2);
    const bool is_c = valid && (key[m] > k1 || (e1 && r1 < t1));
    const bool is_m = valid && !is_c && n_m > 0 && (key[m] > k2 || (e2 && r2 < t2));
    if (mask && valid) mask[row * Tk + j] = is_c ? 1 : (is_m ? 0 : -1);
    const unsigned long long bc = __ballot(is_c), bm = __ballot(is_m);
    if (crit && is_c) crit[row * n_c + nc + __popcll(bc & lt)] = j;
    if (marg && is_m) marg[row * n_m + nm + __popcll(bm & lt)] = j;
    nc += __popcll(bc);
    nm += __popcll(bm);
    if (mbits && lane < 2) {  // the marginal ballot of these 64 key blocks = two words of the bit matrix
      const int kt = 2 * m + lane;
      if (kt < KT) mbits[((size_t)bh * KT + kt) * TqP + i] = (uint32_t)(bm >> (32 * lane));
    }
  }
}

// ---------------------------------------------------------------------------
void launch_zero_u32(uint32_t* p, size_t n, hipStream_t stream) {
  zero_u32_kernel<<<(unsigned)((n + 255) / 256), 256, 0, stream>>>(p, n);
}

void launch_pool_stats(const void* q, const void* k, const void* v, const Problem& p, float* qbar,
                       float* kbar, float* dq, uint32_t* amax_v, int8_t* q8, hipStream_t stream) {
  const size_t n = (size_t)p.BH * D;
  zero_u32_kernel<<<(unsigned)((n + 255) / 256), 256, 0, stream>>>(amax_v, n);
  const int groups = (p.N + 127) / 128;
  pool_stats_kernel<<<p.BH * groups, 256, 0, stream>>>((const bf16_t*)q, (const bf16_t*)k,
                                                        (const bf16_t*)v, p.N, p.block_q, p.Tq, p.Tk,
                                                        groups, p.H, p.lq, p.lk, p.lv, qbar, kbar, dq,
                                                        amax_v, q8);
}

void launch_finalize_stats(const Problem& p, const float* kbar, const uint32_t* amax_v, float* mu_k,
                           float* dv, const bf16_t* proj_w, bf16_t* wfrag, hipStream_t stream) {
  finalize_stats_kernel<<<p.BH * 8, 1024, 0, stream>>>(kbar, amax_v, p.N, p.Tk, mu_k, dv, proj_w, wfrag);
}

void launch_scores(const Problem& p, const float* qbar, const float* kbar, float* scores,
                   hipStream_t stream) {
  dim3 grid(((p.Tk + 31) / 32 + SC_JT - 1) / SC_JT, (p.Tq + 127) / 128, p.BH);
  scores_kernel<<<grid, 256, 0, stream>>>(qbar, kbar, p.Tq, p.Tk, scores);
}

void launch_select(const Problem& p, const float* scores, int8_t* mask, int32_t* crit, int32_t* marg,
                   uint32_t* mbits, hipStream_t stream) {
  const int rows = p.BH * p.Tq;
  const unsigned grid = (unsigned)((rows + 3) / 4);
  const int need = (p.Tk + 63) / 64;
#define SLA_SELECT(K) select_kernel<K><<<grid, 256, 0, stream>>>(scores, rows, p.Tq, p.Tk, p.n_c, p.n_m, mask, crit, marg, mbits)
  // registers per lane: the smallest instantiation that holds the row
  if (need <= 2) SLA_SELECT(2);
  else if (need <= 4) SLA_SELECT(4);
  else if (need <= 8) SLA_SELECT(8);
  else if (need <= 12) SLA_SELECT(12);
  else if (need <= 16) SLA_SELECT(16);
  else if (need <= 20) SLA_SELECT(20);
  else if (need <= 24) SLA_SELECT(24);
  else if (need <= 32) SLA_SELECT(32);
  else if (need <= 48) SLA_SELECT(48);
  else if (need <= 64) SLA_SELECT(64);
  else if (need <= 96) SLA_SELECT(96);
  else SLA_SELECT(128);
#undef SLA_SELECT
}

}  // namespace sla
