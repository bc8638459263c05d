// Measurement aid: what this chip sustains for a matrix instruction ALONE.  Every SIMD gets two
// wavefronts that issue nothing but independent products of one kind (four accumulator tiles in
// turn, operands that never change, no memory traffic); timing the launch from the host gives
// the rate to set beside the published peak, which assumes the full clock.  The benchmark prints
// both, so that a kernel's fraction of peak can be read against what the pipe reaches by itself.
#include "common.h"

namespace sla {

// operand bits that differ from lane to lane, register to register and product to product
__device__ __forceinline__ uint32_t calib_bits(uint32_t lane, uint32_t e, uint32_t set) {
  uint32_t x = lane * 0x9E3779B1u + e * 0x85EBCA77u + set * 0xC2B2AE3Du + 0x27D4EB2Fu;
  x ^= x >> 15; x *= 0x2C1B3C6Du; x ^= x >> 12; x *= 0x297A2D39u; x ^= x >> 15;
  return x;
}

// The four products of a round take four different operand pairs of pseudo-random values (the
// pipe's power, and with it the clock the chip holds, depends on how much its inputs change
// from one product to the next: a loop over one constant operand pair runs near the full clock
// and says little about a kernel on real data).
template <int KIND>
__global__ void __launch_bounds__(256, 2) mfma_rate_kernel(int iters, float* __restrict__ sink) {
  const uint32_t lane = threadIdx.x & 63;
  if constexpr (KIND == 0) {  // v_mfma_i32_32x32x32_i8: 2 * 32 * 32 * 32 operations
    v4i a[4], b[4];
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        a[u][e] = (int)calib_bits(lane, e, 2 * u);
        b[u][e] = (int)calib_bits(lane, e, 2 * u + 1);
      }
    v16i c0 = {}, c1 = {}, c2 = {}, c3 = {};
    for (int i = 0; i < iters; ++i) {
      c0 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[0], b[0], c0, 0, 0, 0);
      c1 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[1], b[1], c1, 0, 0, 0);
      c2 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[2], b[2], c2, 0, 0, 0);
      c3 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[3], b[3], c3, 0, 0, 0);
    }
    const v16i s = c0 + c1 + c2 + c3;
    int x = 0;
#pragma unroll
    for (int e = 0; e < 16; ++e) x ^= s[e];
    sink[blockIdx.x * 256 + threadIdx.x] = (float)x;
  } else if constexpr (KIND == 1) {  // v_mfma_scale_f32_32x32x64_f8f6f4 on FP8 operands: 2 * 32 * 32 * 64
    v8i a[4], b[4];  // FP8 E4M3 bytes of magnitude below 2 and either sign (no NaN codes, sums stay finite)
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        a[u][e] = (int)(calib_bits(lane, e, 2 * u) & 0xBFBFBFBFu);
        b[u][e] = (int)(calib_bits(lane, e, 2 * u + 1) & 0xBFBFBFBFu);
      }
    v16f c0 = {}, c1 = {}, c2 = {}, c3 = {};
    for (int i = 0; i < iters; ++i) {
      c0 = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a[0], b[0], c0, 0, 0, 0, 127, 0, 127);
      c1 = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a[1], b[1], c1, 0, 0, 0, 127, 0, 127);
      c2 = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a[2], b[2], c2, 0, 0, 0, 127, 0, 127);
      c3 = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a[3], b[3], c3, 0, 0, 0, 127, 0, 127);
    }
    const v16f s = c0 + c1 + c2 + c3;
    float x = 0.f;
#pragma unroll
    for (int e = 0; e < 16; ++e) x += s[e];
    sink[blockIdx.x * 256 + threadIdx.x] = x;
  } else {  // v_mfma_f32_32x32x16_bf16: 2 * 32 * 32 * 16
    v8bf a[4], b[4];  // values in [-2, 2)
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        a[u][e] = (__bf16)((float)(int)(calib_bits(lane, e, 2 * u) & 0xffu) * (1.0f / 64.0f) - 2.0f);
        b[u][e] = (__bf16)((float)(int)(calib_bits(lane, e, 2 * u + 1) & 0xffu) * (1.0f / 64.0f) - 2.0f);
      }
    v16f c0 = {}, c1 = {}, c2 = {}, c3 = {};
    for (int i = 0; i < iters; ++i) {
      c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[0], b[0], c0, 0, 0, 0);
      c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[1], b[1], c1, 0, 0, 0);
      c2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[2], b[2], c2, 0, 0, 0);
      c3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[3], b[3], c3, 0, 0, 0);
    }
    const v16f s = c0 + c1 + c2 + c3;
    float x = 0.f;
#pragma unroll
    for (int e = 0; e < 16; ++e) x += s[e];
    sink[blockIdx.x * 256 + threadIdx.x] = x;
  }
}

// Launches the loop on every compute unit (two workgroups of four wavefronts each); returns the
// number of operations the launch performs, 0 if the kind is unknown.
double launch_mfma_rate(int kind, int iters, int n_cu, float* sink, hipStream_t stream) {
  const unsigned grid = 2u * (unsigned)n_cu;
  const double per = kind == 0 ? 2.0 * 32 * 32 * 32 : kind == 1 ? 2.0 * 32 * 32 * 64 : 2.0 * 32 * 32 * 16;
  if (kind == 0) mfma_rate_kernel<0><<<grid, 256, 0, stream>>>(iters, sink);
  else if (kind == 1) mfma_rate_kernel<1><<<grid, 256, 0, stream>>>(iters, sink);
  else if (kind == 2) mfma_rate_kernel<2><<<grid, 256, 0, stream>>>(iters, sink);
  else return 0.0;
  return per * 4.0 * (double)iters * 4.0 * (double)grid;  // 4 products per iteration, 4 wavefronts per workgroup
}

}  // namespace sla
