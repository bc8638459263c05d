// prep_kv: per key block, the operands of both branches.
//
//  * Low-bit sparse branch (Section 1.1 names the scheme; the granularity is this
//    library's reading, see sla.h): K~ = K - mean_K, INT8 codes with one scale per key
//    block; V / delta_V[c] as FP8 E4M3 codes.  Both are written in MFMA fragment order
//    (common.h) so the attention kernel stages them with straight 16-byte copies.
//  * Linear branch: with phi the per-token feature map on the ORIGINAL K,
//        hz[o][c] = sum_rows (V W^T)[row][o] * phi(K)[row][c]   (o < 128)
//        hz[128][c] = sum_rows phi(K)[row][c]
//    i.e. the block summary h_j with the output projection already folded in
//    (transposed, c contiguous) and z_j as row 128.  Two bf16 MFMA products with fp32
//    accumulation; the first product's accumulators are fed to the second as its A
//    operand directly from registers (the contraction order of the second product is
//    permuted to match, for both operands).
//
// One workgroup (4 wavefronts) per (b,h,j).  HBM-bound: reads 32 KiB, writes 16 KiB of
// codes and 33 KiB of summaries per block.
#include "common.h"

namespace sla {

constexpr int STAGE_STRIDE = 2 * D + 16;  // bytes per staged hz row (padded against bank conflicts)

template <int PHI>
__global__ void __launch_bounds__(256, 4) prep_kv_kernel(
    const bf16_t* __restrict__ k, const bf16_t* __restrict__ v, int N, int Tk, int H, Layout lk, Layout lv,
    const float* __restrict__ mu_k, const uint32_t* __restrict__ amax_v,
    const bf16_t* __restrict__ wfrag,
    int want_quant, int want_linear, int8_t* __restrict__ k8, uint8_t* __restrict__ v8,
    float* __restrict__ dk, bf16_t* __restrict__ hz) {
  __shared__ __attribute__((aligned(16))) unsigned char smem[128 * STAGE_STRIDE + 4 * D * 4];
  __shared__ float wave_amax[4];
  unsigned char* kq = smem;                       // [8192]  K codes, fragment order
  unsigned char* vq = smem + KV_FRAG_BYTES;       // [8192]  V codes, fragment order
  unsigned char* vbf = smem;                      // [64][STAGE_STRIDE] V rows as bf16 (aliases kq / vq, after their last read)
  unsigned char* phit = smem + BK * STAGE_STRIDE; // [16384] phi(K)^T bf16, B-operand order
  unsigned char* stage = smem;                    // [128][STAGE_STRIDE] aliases everything above
  float* zred = (float*)(smem + 128 * STAGE_STRIDE);  // [4][128] per-wavefront column sums of phi(K)

  const int bh = blockIdx.x / Tk, j = blockIdx.x % Tk;
  const int t = threadIdx.x, cg = t & 15, m = t >> 4, lane = t & 63, w = t >> 6;
  const int valid = min(BK, N - j * BK);
  const int b_ = bh / H, h_ = bh - b_ * H;
  const bf16_t* kblk = k + b_ * lk.sb + h_ * lk.sh + (long long)j * BK * lk.sn;
  const bf16_t* vblk = v + b_ * lv.sb + h_ * lv.sh + (long long)j * BK * lv.sn;

  float kf[4][8];
  uint4 vraw[4];  // V stays packed: it is quantised from these words and staged for product 1 as they are
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int row = 4 * m + r;
    uint4 xk = make_uint4(0, 0, 0, 0);
    vraw[r] = make_uint4(0, 0, 0, 0);
    if (row < valid) {
      xk = *(const uint4*)(kblk + row * lk.sn + cg * 8);
      vraw[r] = *(const uint4*)(vblk + row * lv.sn + cg * 8);
    }
    const uint32_t wk[4] = {xk.x, xk.y, xk.z, xk.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      kf[r][2 * e] = bf16_lo(wk[e]);
      kf[r][2 * e + 1] = bf16_hi(wk[e]);
    }
  }

  if (want_quant) {
    float mu[8];
    CodeScale vcs[8];  // per channel: max|V| (its scale is this / 448), its reciprocal, 448
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      mu[e] = mu_k[(size_t)bh * D + cg * 8 + e];
      vcs[e] = code_scale(__uint_as_float(amax_v[(size_t)bh * D + cg * 8 + e]), E4M3_MAX);
    }
    float kt[4][8], amax = 0.f;
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        kt[r][e] = (4 * m + r < valid) ? kf[r][e] - mu[e] : 0.f;
        amax = fmaxf(amax, fabsf(kt[r][e]));
      }
    for (int o = 32; o > 0; o >>= 1) amax = fmaxf(amax, __shfl_xor(amax, o));
    if (lane == 0) wave_amax[w] = amax;
    __syncthreads();
    amax = fmaxf(fmaxf(wave_amax[0], wave_amax[1]), fmaxf(wave_amax[2], wave_amax[3]));
    const float delta = amax > 0.f ? amax / 127.0f : 1.0f;
    // K codes by multiplication with the reciprocal: differs from a true division only at
    // rounding ties, where one INT8 step moves a score by delta_Q delta_K (the FP8 V codes, whose
    // steps are coarse, keep the true division).  Adding 1.5 * 2^23 inside the fma rounds the
    // product to the nearest integer (ties to even) and leaves its two's-complement low byte in
    // the low byte of the float; |k~ / delta| <= 127 by construction, so no clamp is needed.
    const float inv_delta = 1.0f / delta;
    if (t == 0) dk[(size_t)bh * Tk + j] = delta;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      uint32_t b[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) b[e] = __float_as_uint(__builtin_fmaf(kt[r][e], inv_delta, 12582912.0f));
      const uint32_t lo = __builtin_amdgcn_perm(__builtin_amdgcn_perm(b[3], b[2], 0x0c0c0400u),
                                                __builtin_amdgcn_perm(b[1], b[0], 0x0c0c0400u), 0x05040100u);
      const uint32_t hi = __builtin_amdgcn_perm(__builtin_amdgcn_perm(b[7], b[6], 0x0c0c0400u),
                                                __builtin_amdgcn_perm(b[5], b[4], 0x0c0c0400u), 0x05040100u);
      *(uint2*)(kq + kfrag_offset(4 * m + r, cg * 8)) = make_uint2(lo, hi);
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      float x[4];
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        // v / delta_V = 448 v / max|V|: the product 448 v is exact for a 16-bit v, and reciprocal + one
        // correction step (the fma forms the residual exactly) gives the correctly rounded quotient, so a
        // value exactly half way between two FP8 values reaches the conversion as the tie it is -- at a
        // third of the cost of the general division sequence
        const uint32_t word = (e >> 1) == 0 ? vraw[r].x : (e >> 1) == 1 ? vraw[r].y : (e >> 1) == 2 ? vraw[r].z : vraw[r].w;
        const float qv = exact_quotient((e & 1) ? bf16_hi(word) : bf16_lo(word), vcs[e]);
        x[r] = clamp_e4m3(qv);
      }
      int code = cvt_pk_e4m3(x[0], x[1], 0, false);
      code = cvt_pk_e4m3(x[2], x[3], code, true);
      *(int*)(vq + vfrag_offset(4 * m, cg * 8 + e)) = code;
    }
    __syncthreads();
    const size_t rec = ((size_t)bh * Tk + j) * KV_FRAG_BYTES;
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const int o = (u * 256 + t) * 16;
      *(uint4*)(k8 + rec + o) = *(const uint4*)(kq + o);
      *(uint4*)(v8 + rec + o) = *(const uint4*)(vq + o);
    }
  }
  if (!want_linear) return;

  // ---- phi(K): rows live across the 16 lanes that share m
  float ph[4][8];
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const bool ok = 4 * m + r < valid;
    if (PHI == 0) {
      float mx = kf[r][0];
#pragma unroll
      for (int e = 1; e < 8; ++e) mx = fmaxf(mx, kf[r][e]);
      for (int o = 8; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
      float s = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        ph[r][e] = __builtin_amdgcn_exp2f((kf[r][e] - mx) * LOG2E);
        s += ph[r][e];
      }
      for (int o = 8; o > 0; o >>= 1) s += __shfl_xor(s, o);
      const float inv = ok ? 1.0f / s : 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) ph[r][e] *= inv;
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float x = kf[r][e];
        float y;
        if (PHI == 1) y = x > 0.f ? x + 1.0f : __builtin_amdgcn_exp2f(x * LOG2E);
        else y = fmaxf(x, 0.f);
        ph[r][e] = ok ? y : 0.f;
      }
    }
  }
  __syncthreads();  // kq / vq reads are done; phit may now be written
  {
    const int tt = m >> 3, g = (m & 7) >> 1, hf = m & 1, s2 = tt * 2 + (g >> 1);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int c = cg * 8 + e;
      const uint2 pk = make_uint2(pack_bf16x2(ph[0][e], ph[1][e]), pack_bf16x2(ph[2][e], ph[3][e]));
      *(uint2*)(phit + ((s2 * 128 + c) * 2 + hf) * 16 + (g & 1) * 8) = pk;
      float zs = ph[0][e] + ph[1][e] + ph[2][e] + ph[3][e];  // 4 rows of this thread, then the 4 row groups of the wavefront
      zs += __shfl_xor(zs, 16);
      zs += __shfl_xor(zs, 32);
      if (lane < 16) zred[w * D + c] = zs;
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) *(uint4*)(vbf + (4 * m + r) * STAGE_STRIDE + cg * 16) = vraw[r];
  }
  __syncthreads();  // phit, zred and the V rows are complete

  // ---- product 1: VW[row][o] for o in this wavefront's tile of 32 output channels
  const int hfl = lane >> 5, l32 = lane & 31;
  v16f d1[2];
#pragma unroll
  for (int rt = 0; rt < 2; ++rt) {
    d1[rt] = v16f{};
    const int row = 32 * rt + l32;  // rows past the end of a ragged block were staged as zeros
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      const v8bf a = *(const v8bf*)(vbf + row * STAGE_STRIDE + 32 * ks + 16 * hfl);
      const v8bf b = *(const v8bf*)(wfrag + ((w * 8 + ks) * 64 + lane) * 8);
      d1[rt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, d1[rt], 0, 0, 0);
    }
  }

  // ---- product 2, transposed: hz^T[c][o] = sum over rows of phi[row][c] VW[row][o], so that a lane
  // ends up with four consecutive c of one o in consecutive registers (8-byte staging writes)
  v16f d2[4];
#pragma unroll
  for (int ct = 0; ct < 4; ++ct) d2[ct] = v16f{};
#pragma unroll
  for (int s2 = 0; s2 < 4; ++s2) {
    v8bf a;
#pragma unroll
    for (int e = 0; e < 8; ++e) a[e] = (__bf16)d1[s2 >> 1][8 * (s2 & 1) + e];
#pragma unroll
    for (int ct = 0; ct < 4; ++ct) {
      const v8bf b = *(const v8bf*)(phit + ((s2 * 128 + 32 * ct + l32) * 2 + hfl) * 16);
      d2[ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b, a, d2[ct], 0, 0, 0);
    }
  }
  float zsum = 0.f;
  if (t < D) {
#pragma unroll
    for (int r = 0; r < 4; ++r) zsum += zred[r * D + t];
  }
  __syncthreads();  // every wavefront is done reading phit: the staging area may overwrite it
#pragma unroll
  for (int ct = 0; ct < 4; ++ct)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const v16f& x = d2[ct];
      *(uint2*)(stage + (32 * w + l32) * STAGE_STRIDE + (32 * ct + 8 * g + 4 * hfl) * 2) =
          make_uint2(pack_bf16x2(x[4 * g], x[4 * g + 1]), pack_bf16x2(x[4 * g + 2], x[4 * g + 3]));
    }
  __syncthreads();
  bf16_t* dst = hz + ((size_t)bh * Tk + j) * HZ_ELEMS;
  // h'^T leaves in the order in which the attention kernel's epilogue takes it as the A operand of
  // v_mfma_f32_32x32x16_bf16 (hz_frag_chunk in common.h); the accumulation over marginal blocks in
  // between is element-wise and does not care.  16-byte chunk d of the destination = row o,
  // channels 8 cq .. 8 cq + 7 of the staged tile.
  for (int d = t; d < 128 * 16; d += 256) {
    const int ot = d >> 9, ks = (d >> 6) & 7, ln = d & 63;
    const int o = 32 * ot + (ln & 31), cq = 4 * (ks >> 1) + 2 * (ln >> 5) + (ks & 1);
    *(uint4*)(dst + d * 8) = *(const uint4*)(stage + o * STAGE_STRIDE + cq * 16);
  }
  if (t < D) dst[D * D + t] = f32_to_bf16(zsum);
}

// Plain-layout copies of the codes (tests only).
__global__ void unfragment_kv_kernel(const int8_t* __restrict__ k8, const uint8_t* __restrict__ v8,
                                     int N, int Tk, int8_t* __restrict__ k_codes,
                                     uint8_t* __restrict__ v_codes) {
  const int bh = blockIdx.x / Tk, j = blockIdx.x % Tk;
  const size_t rec = ((size_t)bh * Tk + j) * KV_FRAG_BYTES;
  for (int e = threadIdx.x; e < BK * D; e += blockDim.x) {
    const int key = e / D, ch = e % D;
    const int row = j * BK + key;
    if (row >= N) continue;
    const size_t o = ((size_t)bh * N + row) * D + ch;
    if (k_codes) k_codes[o] = k8[rec + kfrag_offset(key, ch)];
    if (v_codes) v_codes[o] = v8[rec + vfrag_offset(key, ch)];
  }
}

__global__ void unpack_q8_kernel(const int8_t* __restrict__ q8, int N, int q8_rows, size_t total, int8_t* __restrict__ q_codes) {
  const size_t x = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
  if (x >= total) return;
  const int ch = (int)(x % D);
  const size_t row = (x / D) % N, bh = x / ((size_t)D * N);
  q_codes[x] = q8[(bh * q8_rows + row) * D + q8_byte_offset(ch)];
}

// SLA_QUANT_QK_INT8: the INT8 codes of Q and of the smoothed K as bf16 numbers (integers up to 127
// are exact in bf16), [BH, N, D] contiguous, for the 16-bit attention kernel: its products of such
// operands are the integer products, exactly (|sum| < 2^24 in the fp32 accumulator).
// One workgroup per key block; the same for the query rows it covers.
__global__ void __launch_bounds__(256) code_tensors_kernel(const int8_t* __restrict__ q8, const int8_t* __restrict__ k8,
                                                           int N, int Tk, int q8_rows, bf16_t* __restrict__ qc,
                                                           bf16_t* __restrict__ kc) {
  const int bh = blockIdx.x / Tk, j = blockIdx.x % Tk;
  const size_t rec = ((size_t)bh * Tk + j) * KV_FRAG_BYTES;
  for (int e = threadIdx.x; e < BK * D; e += 256) {
    const int key = e / D, ch = e % D, row = j * BK + key;
    if (row >= N) continue;
    const size_t o = ((size_t)bh * N + row) * D + ch;
    kc[o] = f32_to_bf16((float)k8[rec + kfrag_offset(key, ch)]);
    qc[o] = f32_to_bf16((float)q8[((size_t)bh * q8_rows + row) * D + q8_byte_offset(ch)]);  // the low-bit kernel's own codes
  }
}

__global__ void e4m3_encode_kernel(const float* __restrict__ in, uint8_t* __restrict__ out, size_t n) {
  const size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
  if (i < n) out[i] = (uint8_t)(cvt_pk_e4m3(clamp_e4m3(in[i]), 0.f, 0, false) & 0xff);
}

void launch_prep_kv(const void* k, const void* v, const Problem& p, const float* mu_k, const uint32_t* amax_v,
                    const bf16_t* wfrag, int phi_kind, bool want_quant, bool want_linear, int8_t* k8,
                    uint8_t* v8, float* dk, bf16_t* hz, hipStream_t stream) {
  const unsigned grid = (unsigned)(p.BH * p.Tk);
  const bf16_t* kk = (const bf16_t*)k;
  const bf16_t* vv = (const bf16_t*)v;
  if (phi_kind == 0)
    prep_kv_kernel<0><<<grid, 256, 0, stream>>>(kk, vv, p.N, p.Tk, p.H, p.lk, p.lv, mu_k, amax_v, wfrag, want_quant, want_linear, k8, v8, dk, hz);
  else if (phi_kind == 1)
    prep_kv_kernel<1><<<grid, 256, 0, stream>>>(kk, vv, p.N, p.Tk, p.H, p.lk, p.lv, mu_k, amax_v, wfrag, want_quant, want_linear, k8, v8, dk, hz);
  else
    prep_kv_kernel<2><<<grid, 256, 0, stream>>>(kk, vv, p.N, p.Tk, p.H, p.lk, p.lv, mu_k, amax_v, wfrag, want_quant, want_linear, k8, v8, dk, hz);
}

void launch_unfragment_kv(const Problem& p, const int8_t* k8, const uint8_t* v8, int8_t* k_codes,
                          uint8_t* v_codes, hipStream_t stream) {
  unfragment_kv_kernel<<<p.BH * p.Tk, 256, 0, stream>>>(k8, v8, p.N, p.Tk, k_codes, v_codes);
}

void launch_unpack_q8(const Problem& p, const int8_t* q8, int8_t* q_codes, hipStream_t stream) {
  const size_t total = (size_t)p.BH * p.N * D;
  unpack_q8_kernel<<<(unsigned)((total + 255) / 256), 256, 0, stream>>>(q8, p.N, (p.N + 127) / 128 * 128, total, q_codes);
}

void launch_code_tensors(const Problem& p, const int8_t* q8, const int8_t* k8, bf16_t* qc, bf16_t* kc, hipStream_t stream) {
  code_tensors_kernel<<<p.BH * p.Tk, 256, 0, stream>>>(q8, k8, p.N, p.Tk, (p.N + 127) / 128 * 128, qc, kc);
}

void launch_e4m3_encode(const float* in, uint8_t* out, size_t n, hipStream_t stream) {
  if (n == 0) return;
  e4m3_encode_kernel<<<(unsigned)((n + 255) / 256), 256, 0, stream>>>(in, out, n);
}

}  // namespace sla
