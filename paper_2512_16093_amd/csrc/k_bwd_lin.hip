// Backward pass of SLA, linear branch and projection (Section 1.2; the forward pass it differentiates:
//     a = phi(Q[n]),  num = a H_i,  den = a . Z_i,  O^l[n] = num / den,   O += O^l W^T + b,
//     H_i = sum_{j marginal for i} phi(K_j)^T V_j,   Z_i = sum_{j marginal for i} sum_t phi(K_j[t]),
// phi = softmax over the channels).
//
//   bwd_lin_q_kernel   per query block i (a workgroup walks over several and keeps dW, db in
//                      registers): dO^l = dO W, dnum = dO^l / den, dden = -(dO^l . O^l) / den,
//                      d phi(Q) = dnum H_i^T + dden Z_i -> dQ (softmax backward), and the block's
//                      dH_i = a^T dnum, dZ_i = a^T dden, written in the summaries' storage order so
//                      that the forward's accumulation kernel can sum them over the transposed mask.
//   (the key side -- per key block j, with G_j = sum_{i : j marginal for i} dH_i and the dZ sum:
//   d phi(K) = V G_j^T + dZ -> dK, dV = phi(K) G_j -- is the prologue of the dK/dV kernel, k_bwd.hip)
//
// As in the sparse-branch kernels a wavefront owns 32 tokens, one per lane pair, and every product
// is formed with the tokens as accumulator columns, so per-token reductions stay in a lane pair.
#include "common.h"

namespace sla {

namespace {

constexpr int LP = 136;  // row pitch (elements) of the bf16 LDS matrices: 272 bytes, 16-byte aligned, bank-skewed

__device__ __forceinline__ v16f mfma_bf16(const uint4& a, const uint4& b, const v16f& c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, a), __builtin_bit_cast(v8bf, b), c, 0, 0, 0);
}
__device__ __forceinline__ uint4 lds_frag(const bf16_t* m, int row, int k0) { return *(const uint4*)(m + row * LP + k0); }

// Where entry [o][c .. c+3] (c a multiple of 4) of a 128 x 128 summary sits in the storage order of
// hz / HZ (hz_frag_chunk): element offset of the 4-element run.
__device__ __forceinline__ int hz_run_offset(int o, int c) {
  const int G = c >> 3, ks = 2 * (G >> 2) + (G & 1), lanep = (o & 31) + 32 * ((G >> 1) & 1);
  return hz_frag_chunk(o >> 5, ks, lanep) * 8 + (c & 7);
}

// Softmax over the 128 channels of this lane pair's token; x holds the lane's 64 channels.
// Returns the row maximum and 1 / sum(exp) through the references; x becomes exp(x - max).
__device__ __forceinline__ void softmax_stats(float (&x)[64], float& mx, float& rsum) {
  mx = x[0];
#pragma unroll
  for (int e = 1; e < 64; ++e) mx = fmaxf(mx, x[e]);
  mx = fmaxf(mx, partner_f32(mx));
  float s = 0.f;
#pragma unroll
  for (int e = 0; e < 64; ++e) {
    x[e] = __builtin_amdgcn_exp2f((x[e] - mx) * LOG2E);
    s += x[e];
  }
  s += partner_f32(s);
  rsum = 1.0f / s;
}

__device__ __forceinline__ void unpack8(const uint4& v, float* out) {
  out[0] = bf16_lo(v.x); out[1] = bf16_hi(v.x); out[2] = bf16_lo(v.y); out[3] = bf16_hi(v.y);
  out[4] = bf16_lo(v.z); out[5] = bf16_hi(v.z); out[6] = bf16_lo(v.w); out[7] = bf16_hi(v.w);
}
__device__ __forceinline__ uint4 pack8(const float* x) {
  return uint4{pack_bf16x2(x[0], x[1]), pack_bf16x2(x[2], x[3]), pack_bf16x2(x[4], x[5]), pack_bf16x2(x[6], x[7])};
}

}  // namespace

// wt[c][r] = W[r][c] (identity when there is no projection): the A operand of dO^l = dO W.
__global__ void __launch_bounds__(256) bwd_wt_kernel(const bf16_t* __restrict__ w, bf16_t* __restrict__ wt) {
  for (int x = blockIdx.x * 256 + threadIdx.x; x < D * D; x += gridDim.x * 256) {
    const int c = x >> 7, r = x & 127;
    wt[x] = w ? w[r * D + c] : (bf16_t)(r == c ? 0x3F80 : 0);
  }
}

template <int NW, int PHI>
__global__ void __launch_bounds__(NW * 64, 1)
    bwd_lin_q_kernel(const bf16_t* __restrict__ q, const bf16_t* __restrict__ dout, const bf16_t* __restrict__ HZ,
                     const bf16_t* __restrict__ wt, float* __restrict__ dq_lin, bf16_t* __restrict__ dHZ,
                     float* __restrict__ dW_part, float* __restrict__ db_part, int N, int Tq, int H, Layout lq, Layout ld) {
  constexpr int BQ = 32 * NW;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  bf16_t* Wt = (bf16_t*)smem;              // [c'][r]
  bf16_t* R1 = Wt + 128 * LP;              // Hn[o][c]            -> dnum[n][o]
  bf16_t* R2 = R1 + 128 * LP;              // Ht[c][o]            -> aT[c][n]   -> gT[r][n]
  bf16_t* R3 = R2 + 128 * LP;              // dnumT[o][n]         -> OlT[c][n]
  float* zv = (float*)(R3 + 128 * LP);     // Z[c]
  float* dden_s = zv + 128;                // dden[n]
  const int bh = blockIdx.y, t = threadIdx.x, lane = t & 63, w = t >> 6, l32 = lane & 31, hf = lane >> 5;
  const int nl = 32 * w + l32;             // this lane pair's token within the query block

  for (int x = t; x < 128 * 16; x += NW * 64) *(uint4*)(Wt + (x >> 4) * LP + (x & 15) * 8) = *(const uint4*)(wt + x * 8);

  constexpr int RT = 4 / NW;               // row tiles of dW per wavefront
  v16f dwacc[RT][4];
#pragma unroll
  for (int a = 0; a < RT; ++a)
#pragma unroll
    for (int ct = 0; ct < 4; ++ct) dwacc[a][ct] = v16f{};
  float dbacc = 0.f;

  for (int i = blockIdx.x; i < Tq; i += gridDim.x) {
    // ---- stage H_i twice ([o][c] and [c][o]) and Z_i
    const bf16_t* hz = HZ + ((size_t)bh * Tq + i) * HZ_ELEMS;
    for (int x = t; x < 2048; x += NW * 64) {
      const int ln = x & 63, ks = (x >> 6) & 7, ot = x >> 9;
      const int o = 32 * ot + (ln & 31), c0 = 32 * (ks >> 1) + 16 * (ln >> 5) + 8 * (ks & 1);
      const uint4 v = *(const uint4*)(hz + (size_t)x * 8);
      *(uint4*)(R1 + o * LP + c0) = v;
      const uint32_t wv[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int e = 0; e < 8; ++e) R2[(c0 + e) * LP + o] = (bf16_t)(e & 1 ? wv[e >> 1] >> 16 : wv[e >> 1] & 0xffffu);
    }
    if (t < 128) zv[t] = bf16_to_f32(hz[128 * 128 + t]);
    __syncthreads();

    // ---- this wavefront's 32 tokens
    const long long n = (long long)i * BQ + nl;
    const bool ok = n < N;
    const size_t row = ((size_t)bh * N + (ok ? n : 0)) * D;   // (in the library's own dq_lin)
    const int b_ = bh / H, h_ = bh - b_ * H;
    const bf16_t* qrow = q + b_ * lq.sb + h_ * lq.sh + (long long)(ok ? n : 0) * lq.sn;
    const bf16_t* drow = dout + b_ * ld.sb + h_ * ld.sh + (long long)(ok ? n : 0) * ld.sn;
    float av[64];                // a = phi(Q[n]) at channels 16 ks + 8 hf + kk  (index 8 ks + kk)
    uint4 af[8], gf[8];
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      uint4 qv = uint4{0u, 0u, 0u, 0u};
      gf[ks] = qv;
      if (ok) {
        qv = *(const uint4*)(qrow + 16 * ks + 8 * hf);
        gf[ks] = *(const uint4*)(drow + 16 * ks + 8 * hf);
      }
      unpack8(qv, &av[8 * ks]);
    }
    float qmax = 0.f, rsum = 1.0f;
    if constexpr (PHI == 0) softmax_stats(av, qmax, rsum);
    else {
#pragma unroll
      for (int e = 0; e < 64; ++e) av[e] = phi_value<PHI>(av[e], 0.f, 1.0f);
    }
    if (!ok) rsum = 0.f;         // rows beyond the sequence take no part in dH, dZ, dW
    float den = 0.f;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
#pragma unroll
      for (int kk = 0; kk < 8; ++kk) {
        av[8 * ks + kk] *= rsum;
        den += av[8 * ks + kk] * zv[16 * ks + 8 * hf + kk];
      }
      af[ks] = pack8(&av[8 * ks]);
    }
    den += partner_f32(den);
    const float rden = den > 0.f ? 1.0f / den : 0.f;

    // numT[o][n] = sum_c H[c][o] a[n][c]  ->  O^l;   glT[c'][n] = sum_r W[r][c'] dO[n][r]
    v16f ol[4], gl[4];
    // (here and below: the LDS operand reads of a tile are grouped ahead of its matrix products;
    // left alone the compiler issues each read right before its product and waits for it every time)
#pragma unroll
    for (int ot = 0; ot < 4; ++ot) {
      uint4 ah[8], aw[8];
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        ah[ks] = lds_frag(R1, 32 * ot + l32, 16 * ks + 8 * hf);
        aw[ks] = lds_frag(Wt, 32 * ot + l32, 16 * ks + 8 * hf);
      }
      ol[ot] = v16f{};
      gl[ot] = v16f{};
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        ol[ot] = mfma_bf16(ah[ks], af[ks], ol[ot]);
        gl[ot] = mfma_bf16(aw[ks], gf[ks], gl[ot]);
      }
      __builtin_amdgcn_sched_group_barrier(0x100, 16, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, 16, 0);
    }
    float dden = 0.f;
#pragma unroll
    for (int ot = 0; ot < 4; ++ot)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        ol[ot][r] *= rden;
        dden += gl[ot][r] * ol[ot][r];
        gl[ot][r] *= rden;       // dnum
      }
    dden += partner_f32(dden);
    dden *= -rden;
    uint2 olp[4][4];             // O^l rounded to bf16 (all that is used of it from here on: the dW product)
#pragma unroll
    for (int ot = 0; ot < 4; ++ot)
#pragma unroll
      for (int g = 0; g < 4; ++g)
        olp[ot][g] = uint2{pack_bf16x2(ol[ot][4 * g], ol[ot][4 * g + 1]), pack_bf16x2(ol[ot][4 * g + 2], ol[ot][4 * g + 3])};
    __syncthreads();             // every wavefront is done with Hn

    // ---- d phi(Q) = dnum H^T + dden Z, then through the softmax
#pragma unroll
    for (int ot = 0; ot < 4; ++ot)
#pragma unroll
      for (int g = 0; g < 4; ++g)
        *(uint2*)(R1 + nl * LP + 32 * ot + 8 * g + 4 * hf) =
            uint2{pack_bf16x2(gl[ot][4 * g], gl[ot][4 * g + 1]), pack_bf16x2(gl[ot][4 * g + 2], gl[ot][4 * g + 3])};
    // (own rows only: written and read back by this wavefront, in program order)
    v16f da[4];
    uint4 bn[8];                 // this token's dnum row: the B operand of all four tiles
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) bn[ks] = lds_frag(R1, nl, 16 * ks + 8 * hf);
    __builtin_amdgcn_sched_group_barrier(0x100, 8, 0);
#pragma unroll
    for (int ct = 0; ct < 4; ++ct) {
      uint4 ah[8];
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) ah[ks] = lds_frag(R2, 32 * ct + l32, 16 * ks + 8 * hf);
      da[ct] = v16f{};
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) da[ct] = mfma_bf16(ah[ks], bn[ks], da[ct]);
      __builtin_amdgcn_sched_group_barrier(0x100, 8, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, 8, 0);
    }
    // a at the accumulator's channels 32 ct + 8 g + 4 hf + e: from Q again (its words are kept, a
    // itself is formed twice rather than held in 64 registers)
    uint2 qw[4][4];
    float sdot = 0.f;
#pragma unroll
    for (int ct = 0; ct < 4; ++ct)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int c0 = 32 * ct + 8 * g + 4 * hf;
        qw[ct][g] = ok ? *(const uint2*)(qrow + c0) : uint2{0u, 0u};
        const float xq[4] = {bf16_lo(qw[ct][g].x), bf16_hi(qw[ct][g].x), bf16_lo(qw[ct][g].y), bf16_hi(qw[ct][g].y)};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          da[ct][4 * g + e] += zv[c0 + e] * dden;
          if constexpr (PHI == 0) sdot += phi_value<0>(xq[e], qmax, rsum) * da[ct][4 * g + e];
        }
      }
    sdot += partner_f32(sdot);
    if (ok) {
#pragma unroll
      for (int ct = 0; ct < 4; ++ct)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const float xq[4] = {bf16_lo(qw[ct][g].x), bf16_hi(qw[ct][g].x), bf16_lo(qw[ct][g].y), bf16_hi(qw[ct][g].y)};
          float o[4];
#pragma unroll
          for (int e = 0; e < 4; ++e)
            o[e] = phi_backward<PHI>(xq[e], phi_value<PHI>(xq[e], qmax, rsum), da[ct][4 * g + e], sdot);
          *(float4*)(dq_lin + row + 32 * ct + 8 * g + 4 * hf) = float4{o[0], o[1], o[2], o[3]};
        }
    }
    __syncthreads();             // every wavefront is done with Ht (and with its dnum rows)

    // ---- dH_i^T[o][c] = sum_n dnum[n][o] a[n][c], dZ_i[c] = sum_n a[n][c] dden[n]: transposed copies with the tokens contiguous
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      const uint32_t aw[4] = {af[ks].x, af[ks].y, af[ks].z, af[ks].w};
#pragma unroll
      for (int kk = 0; kk < 8; ++kk)
        R2[(16 * ks + 8 * hf + kk) * LP + nl] = (bf16_t)(kk & 1 ? aw[kk >> 1] >> 16 : aw[kk >> 1] & 0xffffu);
    }
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {  // dnum: this token's row of R1 again (written above), not 64 registers held since
      const uint4 dv = lds_frag(R1, nl, 16 * ks + 8 * hf);
      const uint32_t dw[4] = {dv.x, dv.y, dv.z, dv.w};
#pragma unroll
      for (int kk = 0; kk < 8; ++kk)
        R3[(16 * ks + 8 * hf + kk) * LP + nl] = (bf16_t)(kk & 1 ? dw[kk >> 1] >> 16 : dw[kk >> 1] & 0xffffu);
    }
    if (hf == 0) dden_s[nl] = dden;
    __syncthreads();
    bf16_t* dst = dHZ + ((size_t)bh * Tq + i) * HZ_ELEMS;
    // (the store offsets below are formed from a value the compiler cannot see through: as loop
    // invariants they were kept in scratch memory, and each reload made its store wait for the one before)
    int lane_o = l32;
    asm volatile("" : "+v"(lane_o));
    for (int ct = w; ct < 4; ct += NW) {
      v16f acc[4];
#pragma unroll
      for (int ot = 0; ot < 4; ++ot) {
        acc[ot] = v16f{};
        uint4 aa[BQ / 16], bb[BQ / 16];
#pragma unroll
        for (int ks = 0; ks < BQ / 16; ++ks) {
          aa[ks] = lds_frag(R2, 32 * ct + l32, 16 * ks + 8 * hf);
          bb[ks] = lds_frag(R3, 32 * ot + l32, 16 * ks + 8 * hf);
        }
#pragma unroll
        for (int ks = 0; ks < BQ / 16; ++ks) acc[ot] = mfma_bf16(aa[ks], bb[ks], acc[ot]);
        __builtin_amdgcn_sched_group_barrier(0x100, BQ / 8, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, BQ / 16, 0);
        // lane: o = 32 ot + l32; registers: c = 32 ct + 8 g + 4 hf + e
#pragma unroll
        for (int g = 0; g < 4; ++g)
          *(uint2*)(dst + hz_run_offset(32 * ot + lane_o, 32 * ct + 8 * g + 4 * hf)) =
              uint2{pack_bf16x2(acc[ot][4 * g], acc[ot][4 * g + 1]), pack_bf16x2(acc[ot][4 * g + 2], acc[ot][4 * g + 3])};
      }
    }
    if (t < 128) {  // dZ_i[c = t] = sum_n a[n][c] dden[n], eight tokens per read
      float s = 0.f;
#pragma unroll
      for (int m = 0; m < BQ; m += 8) {
        float a8[8];
        unpack8(*(const uint4*)(R2 + t * LP + m), a8);
        const float4 d0 = *(const float4*)(dden_s + m), d1 = *(const float4*)(dden_s + m + 4);
        s += a8[0] * d0.x + a8[1] * d0.y + a8[2] * d0.z + a8[3] * d0.w + a8[4] * d1.x + a8[5] * d1.y + a8[6] * d1.z + a8[7] * d1.w;
      }
      dst[128 * 128 + t] = f32_to_bf16(s);
    }
    __syncthreads();             // aT and dnumT are consumed

    // ---- dW[r][c] += sum_n dO[n][r] O^l[n][c],  db[r] += sum_n dO[n][r]
    if (dW_part || db_part) {
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        const uint32_t gw[4] = {gf[ks].x, gf[ks].y, gf[ks].z, gf[ks].w};
#pragma unroll
        for (int kk = 0; kk < 8; ++kk)
          R2[(16 * ks + 8 * hf + kk) * LP + nl] = (bf16_t)(kk & 1 ? gw[kk >> 1] >> 16 : gw[kk >> 1] & 0xffffu);
      }
#pragma unroll
      for (int ot = 0; ot < 4; ++ot)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int c0 = 32 * ot + 8 * g + 4 * hf;
          R3[(c0 + 0) * LP + nl] = (bf16_t)(olp[ot][g].x & 0xffffu);
          R3[(c0 + 1) * LP + nl] = (bf16_t)(olp[ot][g].x >> 16);
          R3[(c0 + 2) * LP + nl] = (bf16_t)(olp[ot][g].y & 0xffffu);
          R3[(c0 + 3) * LP + nl] = (bf16_t)(olp[ot][g].y >> 16);
        }
      __syncthreads();
      if (dW_part) {             // (only the bias gradient wanted: no products)
#pragma unroll
      for (int a = 0; a < RT; ++a) {
        const int rt = w + a * NW;
        uint4 ag[BQ / 16];       // this row tile of dO^T: the A operand of all four column tiles
#pragma unroll
        for (int ks = 0; ks < BQ / 16; ++ks) ag[ks] = lds_frag(R2, 32 * rt + l32, 16 * ks + 8 * hf);
        __builtin_amdgcn_sched_group_barrier(0x100, BQ / 16, 0);
#pragma unroll
        for (int ct = 0; ct < 4; ++ct) {
          uint4 bo[BQ / 16];
#pragma unroll
          for (int ks = 0; ks < BQ / 16; ++ks) bo[ks] = lds_frag(R3, 32 * ct + l32, 16 * ks + 8 * hf);
#pragma unroll
          for (int ks = 0; ks < BQ / 16; ++ks) dwacc[a][ct] = mfma_bf16(ag[ks], bo[ks], dwacc[a][ct]);
          __builtin_amdgcn_sched_group_barrier(0x100, BQ / 16, 0);
          __builtin_amdgcn_sched_group_barrier(0x008, BQ / 16, 0);
        }
      }
      }
      if (t < 128) {  // db[r = t] += sum_n dO[n][r]
        float s = 0.f;
#pragma unroll
        for (int m = 0; m < BQ; m += 8) {
          float g8[8];
          unpack8(*(const uint4*)(R2 + t * LP + m), g8);
          s += ((g8[0] + g8[1]) + (g8[2] + g8[3])) + ((g8[4] + g8[5]) + (g8[6] + g8[7]));
        }
        dbacc += s;
      }
      __syncthreads();
    }
  }
  // This workgroup's share of dW and db goes to its own slice; bwd_reduce_partials_kernel adds the
  // slices in a fixed order, so the sums do not depend on which workgroup finishes first.
  const size_t wg = (size_t)blockIdx.y * gridDim.x + blockIdx.x;
  if (dW_part) {
    float* mine = dW_part + wg * (D * D);
#pragma unroll
    for (int a = 0; a < RT; ++a)
#pragma unroll
      for (int ct = 0; ct < 4; ++ct)
#pragma unroll
        for (int r = 0; r < 16; ++r)
          mine[(32 * (w + a * NW) + 8 * (r >> 2) + 4 * hf + (r & 3)) * D + 32 * ct + l32] = dwacc[a][ct][r];
  }
  if (db_part && t < 128) db_part[wg * D + t] = dbacc;
}

// out[x] = sum over p of part[p][x], p ascending: one thread per entry, a fixed order of additions.
__global__ void __launch_bounds__(256) bwd_reduce_partials_kernel(const float* __restrict__ part, int n_part, int n,
                                                                  float* __restrict__ out) {
  const int x = blockIdx.x * 256 + threadIdx.x;
  if (x >= n) return;
  float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;   // four chains for latency; the order is still fixed
  int p = 0;
  for (; p + 4 <= n_part; p += 4) {
    s0 += part[(size_t)p * n + x];
    s1 += part[(size_t)(p + 1) * n + x];
    s2 += part[(size_t)(p + 2) * n + x];
    s3 += part[(size_t)(p + 3) * n + x];
  }
  for (; p < n_part; ++p) s0 += part[(size_t)p * n + x];
  out[x] = (s0 + s1) + (s2 + s3);
}

// ---------------------------------------------------------------------------------------------
void launch_bwd_wt(const bf16_t* proj_w, bf16_t* wt, hipStream_t stream) {
  bwd_wt_kernel<<<64, 256, 0, stream>>>(proj_w, wt);
}

size_t bwd_lin_q_lds_bytes() { return (size_t)4 * 128 * LP * 2 + 128 * 4 + 128 * 4; }

// Workgroups per head of bwd_lin_q_kernel are at most this many (the partial sums' buffer is sized by it).
constexpr int LIN_Q_MAX_CHUNKS = 64;
size_t bwd_lin_q_partial_bytes(const Problem& p) { return (size_t)LIN_Q_MAX_CHUNKS * p.BH * (D * D + D) * 4; }

template <int PHI>
static int launch_bwd_lin_q_phi(const Problem& p, const void* q, const void* dout, const bf16_t* HZ, const bf16_t* wt,
                                float* dq_lin, bf16_t* dHZ, float* dW, float* db, float* partials, hipStream_t stream) {
  // workgroups per head: enough of them to fill the compute units a whole number of times where
  // that is possible (one workgroup per unit), few enough that the per-workgroup partial sums of dW, db stay small
  static int n_cu = 0;
  if (n_cu == 0) {
    int dev = 0, v = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v <= 0) v = 256;
    n_cu = v;
  }
  int chunks = 16;
  for (int c = 16; c <= LIN_Q_MAX_CHUNKS; ++c)
    if ((long long)c * p.BH % n_cu == 0) {
      chunks = c;
      break;
    }
  if (chunks > p.Tq) chunks = p.Tq;
  const dim3 grid((unsigned)chunks, (unsigned)p.BH);
  const size_t lds = bwd_lin_q_lds_bytes();
  static bool attr_set = false;
  if (!attr_set) {
    if (hipFuncSetAttribute((const void*)bwd_lin_q_kernel<4, PHI>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess ||
        hipFuncSetAttribute((const void*)bwd_lin_q_kernel<2, PHI>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
      return -1;
    attr_set = true;
  }
  // per-workgroup partial sums: dW slices first, then db slices
  const int n_part = chunks * p.BH;
  float* dW_part = dW ? partials : nullptr;
  float* db_part = db ? partials + (size_t)LIN_Q_MAX_CHUNKS * p.BH * D * D : nullptr;
  if (p.block_q == 128)
    bwd_lin_q_kernel<4, PHI><<<grid, 256, lds, stream>>>((const bf16_t*)q, (const bf16_t*)dout, HZ, wt, dq_lin, dHZ, dW_part, db_part, p.N, p.Tq, p.H, p.lq, p.ld);
  else
    bwd_lin_q_kernel<2, PHI><<<grid, 128, lds, stream>>>((const bf16_t*)q, (const bf16_t*)dout, HZ, wt, dq_lin, dHZ, dW_part, db_part, p.N, p.Tq, p.H, p.lq, p.ld);
  if (dW) bwd_reduce_partials_kernel<<<(D * D + 255) / 256, 256, 0, stream>>>(dW_part, n_part, D * D, dW);
  if (db) bwd_reduce_partials_kernel<<<1, 256, 0, stream>>>(db_part, n_part, D, db);
  return 0;
}

int launch_bwd_lin_q(const Problem& p, const void* q, const void* dout, const bf16_t* HZ, const bf16_t* wt,
                     int phi_kind, float* dq_lin, bf16_t* dHZ, float* dW, float* db, float* partials, hipStream_t stream) {
  if (phi_kind == 0) return launch_bwd_lin_q_phi<0>(p, q, dout, HZ, wt, dq_lin, dHZ, dW, db, partials, stream);
  if (phi_kind == 1) return launch_bwd_lin_q_phi<1>(p, q, dout, HZ, wt, dq_lin, dHZ, dW, db, partials, stream);
  return launch_bwd_lin_q_phi<2>(p, q, dout, HZ, wt, dq_lin, dHZ, dW, db, partials, stream);
}

}  // namespace sla
