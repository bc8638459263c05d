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
    int N, int block_q, int Tq, int Tk, int groups, float* __restrict__ qbar,
    float* __restrict__ kbar, float* __restrict__ dq, uint32_t* __restrict__ amax_v) {
  __shared__ float sQ[16][2][D];
  __shared__ float sK[16][2][D];
  __shared__ float sV[16][D];
  __shared__ float sQa[2][256];
  const int bh = blockIdx.x / groups, g = blockIdx.x % groups;
  const int t = threadIdx.x, cg = t & 15, rg = t >> 4;
  const size_t base = ((size_t)bh * N) * D;
  const int row0 = g * 128;

  float qs[2][8] = {}, ks[2][8] = {}, va[8] = {}, qa[2] = {0.f, 0.f};
#pragma unroll
  for (int r = 0; r < 8; ++r) {
    const int row = row0 + rg + 16 * r, half = r >> 2;
    if (row < N) {
      const size_t off = base + (size_t)row * D + cg * 8;
      const uint4 xq = *(const uint4*)(q + off);
      const uint4 xk = *(const uint4*)(k + off);
      const uint4 xv = *(const uint4*)(v + off);
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
      } else {
        const float m = fmaxf(m0, m1);
        dq[(size_t)bh * Tq + g] = m > 0.f ? m / 127.0f : 1.0f;
      }
    }
  }
}

__global__ void zero_u32_kernel(uint32_t* p, size_t n) {
  size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0u;
}

// finalize_stats: one workgroup of 1024 threads per (b,h): mu_K[c] = sum_j cnt_j kbar[j][c] / N,
// delta_V[c] = max|V[:,c]| / 448 (1 if zero).  Workgroup 0 also writes the bf16 identity.
__global__ void __launch_bounds__(1024) finalize_stats_kernel(
    const float* __restrict__ kbar, const uint32_t* __restrict__ amax_v, int N, int Tk,
    float* __restrict__ mu_k, float* __restrict__ dv, bf16_t* __restrict__ eye) {
  __shared__ float red[8][D];
  const int bh = blockIdx.x, t = threadIdx.x, c = t & 127, rgrp = t >> 7;
  float s = 0.f;
  for (int j = rgrp; j < Tk; j += 8) {
    const int cnt = min(BK, N - j * BK);
    s += kbar[((size_t)bh * Tk + j) * D + c] * (float)cnt;
  }
  red[rgrp][c] = s;
  __syncthreads();
  if (t < 128) {
    float tot = 0.f;
#pragma unroll
    for (int r = 0; r < 8; ++r) tot += red[r][t];
    mu_k[(size_t)bh * D + t] = tot / (float)N;
    const float am = __uint_as_float(amax_v[(size_t)bh * D + t]);
    dv[(size_t)bh * D + t] = am > 0.f ? am / E4M3_MAX : 1.0f;
  }
  if (bh == 0) {
    for (int i = t; i < D * D; i += 1024) eye[i] = (i / D == i % D) ? (bf16_t)0x3f80 : (bf16_t)0;
  }
}

// scores: s[bh][i][j] = qbar_i . kbar_j / sqrt(d), 64x64 tile per workgroup, fp32 FMA.
__global__ void __launch_bounds__(256) scores_kernel(const float* __restrict__ qbar,
                                                     const float* __restrict__ kbar, int Tq, int Tk,
                                                     float* __restrict__ scores) {
  __shared__ float sq[64][65];
  __shared__ float sk[64][65];
  const int bh = blockIdx.z, i0 = blockIdx.y * 64, j0 = blockIdx.x * 64;
  const int t = threadIdx.x, tx = t & 15, ty = t >> 4;
  float acc[4][4] = {};
  for (int c0 = 0; c0 < D; c0 += 64) {
    __syncthreads();
    for (int e = t; e < 64 * 64; e += 256) {
      const int r = e >> 6, c = e & 63;
      sq[r][c] = (i0 + r < Tq) ? qbar[((size_t)bh * Tq + i0 + r) * D + c0 + c] : 0.f;
      sk[r][c] = (j0 + r < Tk) ? kbar[((size_t)bh * Tk + j0 + r) * D + c0 + c] : 0.f;
    }
    __syncthreads();
#pragma unroll 8
    for (int c = 0; c < 64; ++c) {
      float a[4], b[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        a[u] = sq[ty * 4 + u][c];
        b[u] = sk[tx + 16 * u][c];
      }
#pragma unroll
      for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int w = 0; w < 4; ++w) acc[u][w] = __builtin_fmaf(a[u], b[w], acc[u][w]);
    }
  }
#pragma unroll
  for (int u = 0; u < 4; ++u)
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const int i = i0 + ty * 4 + u, j = j0 + tx + 16 * w;
      if (i < Tq && j < Tk) scores[((size_t)bh * Tq + i) * Tk + j] = acc[u][w] / 11.313708498984761f;
    }
}

// select: one workgroup per (b,h,i) row.  Keys (order-preserving score bits, ~j) are
// sorted descending by a bitonic network in LDS, so equal scores rank by ascending j
// and the result is exact and deterministic.  Then the class of each j is scattered
// back and the ascending index lists come from a prefix count.
__device__ __forceinline__ uint32_t order_bits(float f) {
  const uint32_t u = __float_as_uint(f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__global__ void __launch_bounds__(256) select_kernel(const float* __restrict__ scores, int Tk, int P,
                                                     int n_c, int n_m, int8_t* __restrict__ mask,
                                                     int32_t* __restrict__ crit,
                                                     int32_t* __restrict__ marg) {
  extern __shared__ unsigned long long smem[];
  unsigned long long* keys = smem;                 // [P]
  int8_t* cls = (int8_t*)(keys + P);               // [P]
  __shared__ int wave_c[4], wave_m[4];
  const size_t row = blockIdx.x;
  const int t = threadIdx.x;
  const float* srow = scores + row * Tk;
  for (int j = t; j < P; j += 256) {
    keys[j] = (j < Tk) ? (((unsigned long long)order_bits(srow[j]) << 32) | (uint32_t)(~(uint32_t)j)) : 0ull;
    cls[j] = -1;
  }
  __syncthreads();
  for (int k = 2; k <= P; k <<= 1) {
    for (int j = k >> 1; j > 0; j >>= 1) {
      for (int idx = t; idx < (P >> 1); idx += 256) {
        const int a = 2 * j * (idx / j) + (idx % j), b = a + j;
        const bool desc = (a & k) == 0;
        const unsigned long long x = keys[a], y = keys[b];
        if ((x < y) == desc) {
          keys[a] = y;
          keys[b] = x;
        }
      }
      __syncthreads();
    }
  }
  for (int p = t; p < n_c + n_m; p += 256) {
    const uint32_t j = ~(uint32_t)(keys[p] & 0xffffffffull);
    cls[j] = (p < n_c) ? 1 : 0;
  }
  __syncthreads();
  if (mask) {
    for (int j = t; j < Tk; j += 256) mask[row * Tk + j] = cls[j];
  }
  if (crit || marg) {
    const int ch = (Tk + 255) / 256, lo = min(Tk, t * ch), hi = min(Tk, lo + ch);
    int cc = 0, cm = 0;
    for (int j = lo; j < hi; ++j) {
      cc += cls[j] == 1;
      cm += cls[j] == 0;
    }
    int ic = cc, im = cm;  // inclusive scans within the wave
    const int lane = t & 63, w = t >> 6;
    for (int o = 1; o < 64; o <<= 1) {
      const int uc = __shfl_up(ic, o), um = __shfl_up(im, o);
      if (lane >= o) {
        ic += uc;
        im += um;
      }
    }
    if (lane == 63) {
      wave_c[w] = ic;
      wave_m[w] = im;
    }
    __syncthreads();
    int oc = ic - cc, om = im - cm;
    for (int u = 0; u < w; ++u) {
      oc += wave_c[u];
      om += wave_m[u];
    }
    for (int j = lo; j < hi; ++j) {
      if (cls[j] == 1 && crit) crit[row * n_c + oc] = j;
      if (cls[j] == 1) ++oc;
      if (cls[j] == 0 && marg) marg[row * n_m + om] = j;
      if (cls[j] == 0) ++om;
    }
  }
}

// ---------------------------------------------------------------------------
void launch_pool_stats(const void* q, const void* k, const void* v, const Problem& p, float* qbar,
                       float* kbar, float* dq, uint32_t* amax_v, hipStream_t stream) {
  const size_t n = (size_t)p.BH * D;
  zero_u32_kernel<<<(unsigned)((n + 255) / 256), 256, 0, stream>>>(amax_v, n);
  const int groups = (p.N + 127) / 128;
  pool_stats_kernel<<<p.BH * groups, 256, 0, stream>>>((const bf16_t*)q, (const bf16_t*)k,
                                                        (const bf16_t*)v, p.N, p.block_q, p.Tq, p.Tk,
                                                        groups, qbar, kbar, dq, amax_v);
}

void launch_finalize_stats(const Problem& p, const float* kbar, const uint32_t* amax_v, float* mu_k,
                           float* dv, bf16_t* eye, hipStream_t stream) {
  finalize_stats_kernel<<<p.BH, 1024, 0, stream>>>(kbar, amax_v, p.N, p.Tk, mu_k, dv, eye);
}

void launch_scores(const Problem& p, const float* qbar, const float* kbar, float* scores,
                   hipStream_t stream) {
  dim3 grid((p.Tk + 63) / 64, (p.Tq + 63) / 64, p.BH);
  scores_kernel<<<grid, 256, 0, stream>>>(qbar, kbar, p.Tq, p.Tk, scores);
}

void launch_select(const Problem& p, const float* scores, int8_t* mask, int32_t* crit, int32_t* marg,
                   hipStream_t stream) {
  int P = 2;
  while (P < p.Tk) P <<= 1;
  const size_t lds = (size_t)P * 9;
  select_kernel<<<p.BH * p.Tq, 256, lds, stream>>>(scores, p.Tk, P, p.n_c, p.n_m, mask, crit, marg);
}

}  // namespace sla
