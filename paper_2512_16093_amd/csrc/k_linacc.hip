// lin_accumulate: per query block, the sums of the marginal key blocks' summaries,
//     HZ[i][n] = sum_{j : block j marginal for i} hz[j][n],   n over the 129*128 entries
// of a summary (h'^T and the z row), written as one dense contraction per (b,h):
//     HZ[Tq x 16512] = M0[Tq x Tk] . hz[Tk x 16512],   M0 = 1 where the mask is 0.
// This really is a GEMM (every summary is needed by ~n_m/Tk of all query blocks), so it
// runs on bf16 MFMA with fp32 accumulation; gathering n_m summaries per query block
// instead would move ~50x more bytes.
//
// Workgroup = 4 wavefronts (2 x 2), tile 256 query blocks x 128 columns, looping over
// all row tiles of its column stripe so the stripe of hz is fetched from HBM once and
// re-read from L2.  The hz tile (32 key blocks x 128 columns) is staged row-major in LDS
// and read back transposed (2-byte reads) into the B operand.
#include "common.h"

namespace sla {

constexpr int LA_KT = 32;                 // key blocks per staged tile
constexpr int LA_STRIDE = 2 * 128 + 8;    // bytes per staged row (pad: the two lane halves hit different banks)

// m0 rows: uint8 [BH][Tq][Tkp], 1 = marginal, zero padded to Tkp (a multiple of 32).
__global__ void marginal_rows_kernel(const int8_t* __restrict__ mask, int Tk, int Tkp,
                                     uint8_t* __restrict__ m0) {
  const size_t row = blockIdx.x;
  for (int j = threadIdx.x; j < Tkp; j += blockDim.x)
    m0[row * Tkp + j] = (j < Tk && mask[row * Tk + j] == 0) ? 1 : 0;
}

__device__ __forceinline__ v8bf expand_mask8(uint2 b) {
  // each byte is 0 or 1; bf16 1.0 = 0x3f80
  union { uint32_t u[4]; v8bf v; } r;
  r.u[0] = ((b.x & 0x1u) * 0x3f80u) | (((b.x >> 8) & 0x1u) * 0x3f800000u);
  r.u[1] = (((b.x >> 16) & 0x1u) * 0x3f80u) | (((b.x >> 24) & 0x1u) * 0x3f800000u);
  r.u[2] = ((b.y & 0x1u) * 0x3f80u) | (((b.y >> 8) & 0x1u) * 0x3f800000u);
  r.u[3] = (((b.y >> 16) & 0x1u) * 0x3f80u) | (((b.y >> 24) & 0x1u) * 0x3f800000u);
  return r.v;
}

__global__ void __launch_bounds__(256) lin_accumulate_kernel(const uint8_t* __restrict__ m0,
                                                             const bf16_t* __restrict__ hz, int Tq,
                                                             int Tk, int Tkp, bf16_t* __restrict__ HZ) {
  __shared__ __attribute__((aligned(16))) unsigned char sB[2][LA_KT * LA_STRIDE];
  const int bh = blockIdx.y, n0 = blockIdx.x * 128;
  const int t = threadIdx.x, lane = t & 63, w = t >> 6, l32 = lane & 31, hf = lane >> 5;
  const int wm = w >> 1, wn = w & 1;  // wavefront grid 2 x 2: rows 128*wm.., columns 64*wn..
  const bf16_t* hz_bh = hz + (size_t)bh * Tk * HZ_ELEMS + n0;
  const int ktiles = Tkp / LA_KT;
  // staging role: thread -> (row jr = t/8, 32-byte piece pc = t%8) of the [32][128] tile
  const int jr = t >> 3, pc = t & 7;

  for (int i0 = 0; i0 < Tq; i0 += 256) {
    v16f acc[4][2];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
      for (int b = 0; b < 2; ++b) acc[a][b] = v16f{};

    uint4 g0 = make_uint4(0, 0, 0, 0), g1 = g0;
    auto gload = [&](int kt) {
      const int j = kt * LA_KT + jr;
      g0 = g1 = make_uint4(0, 0, 0, 0);
      if (j < Tk) {
        const uint4* src = (const uint4*)(hz_bh + (size_t)j * HZ_ELEMS + pc * 16);
        g0 = src[0];
        g1 = src[1];
      }
    };
    auto lstore = [&](int buf) {
      uint4* dst = (uint4*)(sB[buf] + jr * LA_STRIDE + pc * 32);
      // rows are 8-byte aligned only: store as four 8-byte pieces
      uint2* d2 = (uint2*)dst;
      d2[0] = make_uint2(g0.x, g0.y);
      d2[1] = make_uint2(g0.z, g0.w);
      d2[2] = make_uint2(g1.x, g1.y);
      d2[3] = make_uint2(g1.z, g1.w);
    };
    __syncthreads();  // previous row tile is done with both buffers
    gload(0);
    lstore(0);
    __syncthreads();
    for (int kt = 0; kt < ktiles; ++kt) {
      const int buf = kt & 1;
      if (kt + 1 < ktiles) gload(kt + 1);
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
        v8bf bop[2];
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) {
          const unsigned char* col = sB[buf] + (16 * ks + 8 * hf) * LA_STRIDE + (64 * wn + 32 * nt + l32) * 2;
          union { bf16_t h[8]; v8bf v; } u;
#pragma unroll
          for (int e = 0; e < 8; ++e) u.h[e] = *(const bf16_t*)(col + e * LA_STRIDE);
          bop[nt] = u.v;
        }
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) {
          const int i = i0 + 128 * wm + 32 * mt + l32;
          uint2 mb = make_uint2(0, 0);
          if (i < Tq) mb = *(const uint2*)(m0 + ((size_t)bh * Tq + i) * Tkp + kt * LA_KT + 16 * ks + 8 * hf);
          const v8bf aop = expand_mask8(mb);
#pragma unroll
          for (int nt = 0; nt < 2; ++nt)
            acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aop, bop[nt], acc[mt][nt], 0, 0, 0);
        }
      }
      if (kt + 1 < ktiles) lstore(buf ^ 1);
      __syncthreads();
    }
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
      for (int nt = 0; nt < 2; ++nt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int i = i0 + 128 * wm + 32 * mt + 8 * (r >> 2) + 4 * hf + (r & 3);
          if (i < Tq)
            HZ[((size_t)bh * Tq + i) * HZ_ELEMS + n0 + 64 * wn + 32 * nt + l32] = f32_to_bf16(acc[mt][nt][r]);
        }
  }
}

void launch_marginal_rows(const Problem& p, const int8_t* mask, uint8_t* m0, hipStream_t stream) {
  const int Tkp = (p.Tk + 31) / 32 * 32;
  marginal_rows_kernel<<<p.BH * p.Tq, 256, 0, stream>>>(mask, p.Tk, Tkp, m0);
}

void launch_lin_accumulate(const Problem& p, const uint8_t* m0, const bf16_t* hz, bf16_t* HZ,
                           hipStream_t stream) {
  const int Tkp = (p.Tk + 31) / 32 * 32;
  dim3 grid(HZ_ELEMS / 128, p.BH);
  lin_accumulate_kernel<<<grid, 256, 0, stream>>>(m0, hz, p.Tq, p.Tk, Tkp, HZ);
}

}  // namespace sla
