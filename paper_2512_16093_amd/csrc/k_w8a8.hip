// W8A8 Linear layer for gfx950: block-wise (128 x 128) INT8 quantisation of weights and
// activations and their product on the INT8 matrix units (Section 1.1, fourth technique;
// Section 1.3, "Linear layer quantization"; the formula is stated in include/w8a8.h).
//
// Operand order.  A quantised matrix A8[RP][K] (RP = rows padded to whole tiles, K a multiple
// of 128) is stored as 16-byte chunks
//     chunk ((kb * RT + rt) * 4 + ks) * 64 + lane,   RT = RP / 32,
// holding A8[32 rt + lane % 32][128 kb + 32 ks + 16 (lane / 32) + 0..15]: exactly what lane
// `lane` feeds to v_mfma_i32_32x32x32_i8 for row tile rt and contraction step ks of feature
// block kb.  Everything a workgroup needs of one feature block is then contiguous (4 KiB per
// row tile, consecutive row tiles adjacent), so operands move with straight 16-byte-per-lane
// copies.  Scales: s[kb * RB + rb], RB = RP / 128.  Rows past the end hold zero codes.
//
// Kernels
//   w8a8_quantize_kernel   one workgroup per 128 x 128 block: amax, scale, codes through LDS
//                          into operand order.  HBM-bound (reads 2 bytes, writes 1 per element).
//   w8a8_gemm_kernel       workgroup tile 256 tokens x 128 outputs, four wavefronts of 64 x 128.
//                          The weight tile of a feature block (16 KiB) is staged in LDS by
//                          asynchronous copies, three stages deep; a wavefront's activation
//                          operands (8 KiB per feature block) go from global memory straight to
//                          registers, one feature block ahead.  INT8 MFMA bound.
#include "common.h"

namespace sla {

constexpr int QB = 128;                      // quantisation block edge
constexpr int W8_WG_M = 256, W8_WG_N = 128;  // workgroup tile of the product
// The integer accumulators start from the bit pattern of the float 1 / (2 pi), which the MFMA
// takes as its C operand: a finished accumulator, reinterpreted as fp32, is then exactly
// W8_C0 + s * 2^-26 for every block sum |s| <= 127 * 127 * 128 (the pattern stays inside the
// binade [1/8, 1/4)), so scaling and accumulating a block is ONE fma per element, with no
// int -> float conversion.  The constant's share must stay small next to the sums it rides on
// (fp32 rounds at the magnitude of the running total): the weight codes of ODD feature blocks
// are stored negated and their blocks scaled by -s_X s_W, which leaves the products' share
// unchanged and makes the constants alternate in sign; what is left of them, W8_C0 * (signed
// sum of the scales), is uniform over a wavefront's tile and is taken out at the end.
constexpr int W8_BIAS_I = 0x3E22F983;
constexpr float W8_C0 = 0.15915494f;         // the float with that bit pattern
constexpr float W8_STEP_INV = 67108864.0f;   // 2^26

__host__ __device__ inline size_t w8_chunk(int kb, int RT, int rt, int ks) {
  return (((size_t)kb * RT + rt) * 4 + ks) * 64;  // index of the first of the 64 chunks (lanes)
}

// ---------------------------------------------------------------------------
// Quantisation of one 128 x 128 block per workgroup.  Thread t: columns 8 (t % 16) .. +7 of
// rows t / 16 + 16 i, i = 0..7.
// ---------------------------------------------------------------------------
// negate_odd (weights): the codes of odd feature blocks are stored negated (see W8_BIAS_I).
__global__ void __launch_bounds__(256) w8a8_quantize_kernel(const bf16_t* __restrict__ a, int R, int K, int RP,
                                                            int negate_odd, int8_t* __restrict__ codes,
                                                            float* __restrict__ scales) {
  __shared__ uint4 blk[QB * QB / 16];
  __shared__ float wave_amax[4];
  const int KB = K / QB, RB = RP / QB, RT = RP / 32;
  const int rb = blockIdx.x / KB, kb = blockIdx.x % KB;
  const int t = threadIdx.x, cg = t & 15, r0 = t >> 4, lane = t & 63, w = t >> 6;
  uint4 x[8];
  float amax = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int row = rb * QB + r0 + 16 * i;
    x[i] = make_uint4(0, 0, 0, 0);
    if (row < R) x[i] = *(const uint4*)(a + (size_t)row * K + kb * QB + cg * 8);
    const uint32_t wd[4] = {x[i].x, x[i].y, x[i].z, x[i].w};
#pragma unroll
    for (int e = 0; e < 4; ++e) amax = fmaxf(amax, fmaxf(fabsf(bf16_lo(wd[e])), fabsf(bf16_hi(wd[e]))));
  }
  for (int o = 32; o > 0; o >>= 1) amax = fmaxf(amax, __shfl_xor(amax, o));
  if (lane == 0) wave_amax[w] = amax;
  __syncthreads();
  amax = fmaxf(fmaxf(wave_amax[0], wave_amax[1]), fmaxf(wave_amax[2], wave_amax[3]));
  const float s = amax > 0.f ? amax / 127.0f : 1.0f;
  if (t == 0) scales[kb * RB + rb] = s;
  // codes = the correctly rounded quotient 127 x / amax, rounded to the nearest integer with ties to even
  // (int8_code_word_exact: exact ties stay ties -- with 16-bit inputs they are common, x = amax / 2 is one);
  // the two's-complement low byte of the returned word is the code; |x / s| <= 127.
  const CodeScale cs = code_scale(amax, 127.0f);
  const float sgn = (negate_odd && (kb & 1)) ? -1.0f : 1.0f;
  unsigned char* out = (unsigned char*)blk;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const uint32_t wd[4] = {x[i].x, x[i].y, x[i].z, x[i].w};
    uint32_t b[8];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      b[2 * e] = int8_code_word_exact(sgn * bf16_lo(wd[e]), cs);
      b[2 * e + 1] = int8_code_word_exact(sgn * bf16_hi(wd[e]), cs);
    }
    const uint32_t lo = __builtin_amdgcn_perm(__builtin_amdgcn_perm(b[3], b[2], 0x0c0c0400u),
                                              __builtin_amdgcn_perm(b[1], b[0], 0x0c0c0400u), 0x05040100u);
    const uint32_t hi = __builtin_amdgcn_perm(__builtin_amdgcn_perm(b[7], b[6], 0x0c0c0400u),
                                              __builtin_amdgcn_perm(b[5], b[4], 0x0c0c0400u), 0x05040100u);
    const int rl = r0 + 16 * i;  // row within the block
    const int off = (((rl >> 5) * 4 + (cg >> 2)) * 64 + (rl & 31) + 32 * ((cg >> 1) & 1)) * 16 + 8 * (cg & 1);
    *(uint2*)(out + off) = make_uint2(lo, hi);
  }
  __syncthreads();
  // the block's four row tiles x four steps are one contiguous 16 KiB in operand order
  uint4* dst = (uint4*)codes + w8_chunk(kb, RT, 4 * rb, 0);
#pragma unroll
  for (int u = 0; u < 4; ++u) dst[u * 256 + t] = blk[u * 256 + t];
}

// Plain-layout copies of codes and scales (tests only).
__global__ void w8a8_unpack_kernel(const int8_t* __restrict__ frag, const float* __restrict__ s, int R, int K, int RP,
                                   int negate_odd, int8_t* __restrict__ codes, float* __restrict__ scales) {
  const int KB = K / QB, RB = RP / QB, RT = RP / 32;
  const size_t total = (size_t)R * K;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
    const int r = (int)(i / K), k = (int)(i % K);
    const int kb = k / QB, ks = (k % QB) / 32, half = (k % 32) / 16, byte = k % 16;
    const int8_t c = frag[(w8_chunk(kb, RT, r / 32, ks) + (r % 32) + 32 * half) * 16 + byte];
    if (codes) codes[i] = (negate_odd && (kb & 1)) ? (int8_t)-c : c;
  }
  const int rbn = (R + QB - 1) / QB;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; scales && i < (size_t)rbn * KB;
       i += (size_t)gridDim.x * blockDim.x)
    scales[i] = s[(i % KB) * RB + i / KB];
}

// ---------------------------------------------------------------------------
// The product.
// ---------------------------------------------------------------------------
typedef __attribute__((address_space(3))) void* w8_lds_ptr_t;
// Asynchronous 16-bytes-per-lane copy global -> LDS (lane l reads base + voff, the data lands at
// lds + 16 l), issued from inline assembly so that the compiler does not make every LDS read
// wait for all copies in flight; the pipeline waits for them by explicit counts.
__device__ __forceinline__ void w8_copy16(const void* base, unsigned voff, const void* lds) {
  const unsigned lds_addr = (unsigned)(uintptr_t)(w8_lds_ptr_t)lds;
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %0"
               :
               : "s"(base), "v"(voff), "s"(lds_addr)
               : "memory", "m0");
}
__device__ __forceinline__ void w8_barrier() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

constexpr int W8_EPI_STRIDE = W8_WG_N * 2 + 16;  // bytes per staged output row

__global__ void __launch_bounds__(256, 2) w8a8_gemm_kernel(
    const int8_t* __restrict__ x8, const float* __restrict__ sx, const int8_t* __restrict__ w8,
    const float* __restrict__ sw, const bf16_t* __restrict__ bias, bf16_t* __restrict__ y, int M, int N, int K,
    int RTx, int RBx, int RTw, int RBw, int MT, int NT) {
  __shared__ uint4 bst[3][QB * W8_WG_N / 16];  // three stages of a 128-feature x 128-output weight tile
  static_assert(4 * 32 * W8_EPI_STRIDE <= (int)sizeof(uint4) * 3 * QB * W8_WG_N / 16, "output staging fits the stages");
  // Workgroup ids are dealt round-robin over the 8 XCDs: XCD x takes the token tiles mt = x, x + 8,
  // ...  Inside an XCD 64 consecutive workgroups -- what its 32 compute units hold at a time --
  // form a patch of 8 token tiles x 8 output tiles and walk the feature blocks at the same pace,
  // so each activation and weight tile of a feature block is fetched into that L2 once for
  // eight users (the patches cover the XCD's tiles row of patches by row of patches).
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int pcols = (NT + 7) >> 3, patch = slot >> 6, q = slot & 63;
  const int mt = __builtin_amdgcn_readfirstlane((((patch / pcols) << 3) + (q >> 3)) * 8 + xcd);
  const int nt = __builtin_amdgcn_readfirstlane(((patch % pcols) << 3) + (q & 7));
  if (mt >= MT || nt >= NT) return;
  const int t = threadIdx.x, lane = t & 63, w = __builtin_amdgcn_readfirstlane(t >> 6), l32 = lane & 31, hf = lane >> 5;
  const int KB = K / QB;
  const int rt0 = mt * (W8_WG_M / 32) + 2 * w;  // this wavefront's two row tiles (64 tokens)
  const int rb = mt * 2 + (w >> 1);             // and their quantisation block row
  const unsigned char* xa = (const unsigned char*)x8 + (size_t)rt0 * 4096 + (size_t)lane * 16;
  const size_t xkb = (size_t)RTx * 4096;        // bytes from one feature block to the next
  const unsigned char* wb = (const unsigned char*)w8 + (size_t)(4 * nt) * 4096;
  const size_t wkb = (size_t)RTw * 4096;

  auto fetch_b = [&](int kb) {  // 16 KiB weight tile of feature block kb -> its stage; four 1 KiB pieces per wavefront
    const unsigned char* src = wb + (size_t)kb * wkb;
    unsigned char* dst = (unsigned char*)bst[kb % 3];
#pragma unroll
    for (int u = 0; u < 4; ++u) w8_copy16(src, (unsigned)((w * 4 + u) * 1024 + lane * 16), dst + (w * 4 + u) * 1024);
  };
  auto load_a = [&](int kb, v4i (&a)[2][4]) {
    const unsigned char* src = xa + (size_t)kb * xkb;
#pragma unroll
    for (int rtl = 0; rtl < 2; ++rtl)
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) a[rtl][ks] = *(const v4i*)(src + (rtl * 4 + ks) * 1024);
  };

  v16f facc[2][4];
#pragma unroll
  for (int r = 0; r < 2; ++r)
#pragma unroll
    for (int c = 0; c < 4; ++c) facc[r][c] = v16f{};
  v16i bias16;  // (only the idle value of `pend` below; the chains take the pattern as an inline constant)
#pragma unroll
  for (int e = 0; e < 16; ++e) bias16[e] = W8_BIAS_I;
  float csum = 0.f;                 // scales whose constant share is still inside facc

  v4i a0[2][4], a1[2][4];  // this wavefront's activation operands of the current and the next feature block

  // One feature block: products against the staged weight tile, then one fma per element.  The
  // product is taken transposed (weights as the A operand) so that a lane owns ONE token and runs
  // of four consecutive outputs.
  // The first product of a chain takes the pattern W8_BIAS_I as an inline constant (0.15915494 is
  // the assembler's spelling of 1 / (2 pi)); the compiler would keep the constant in sixteen
  // registers instead.  Every product of a chain is an assembly statement whose accumulator is ONE
  // in/out operand, so the chain accumulates in place by construction (destination = C operand,
  // the case the hardware interlocks) whatever registers are allocated, and each product still
  // takes its operands as they arrive.  The compiler does not know the statements hold
  // matrix products and adds no wait states before a vector instruction that reads the result, so
  // the data flow itself keeps every reader a whole chain (four dependent products, > 100 cycles)
  // behind: a chain's result may only be read after it has been handed through the SECOND product
  // of the next chain as `carry` (an in/out operand the statement does not touch; that product
  // cannot issue before the next chain's first one has finished, 64 cycles after the carried
  // chain's last one was issued), or, after the loop, through a statement of explicit wait states.
  auto chain = [&](const v4i (&b)[4], const v4i (&ar)[4], v16i& carry) {
    v16i acc;
    asm volatile("v_mfma_i32_32x32x32_i8 %0, %1, %2, 0.15915494" : "=&v"(acc) : "v"(b[0]), "v"(ar[0]));
    asm volatile("v_mfma_i32_32x32x32_i8 %0, %2, %3, %0" : "+v"(acc), "+v"(carry) : "v"(b[1]), "v"(ar[1]));
    asm volatile("v_mfma_i32_32x32x32_i8 %0, %1, %2, %0" : "+v"(acc) : "v"(b[2]), "v"(ar[2]));
    asm volatile("v_mfma_i32_32x32x32_i8 %0, %1, %2, %0" : "+v"(acc) : "v"(b[3]), "v"(ar[3]));
    return acc;
  };
  auto scale_in = [&](const v16i& acc, float sc, v16f& f) {
#pragma unroll
    for (int e = 0; e < 16; ++e) f[e] = __builtin_fmaf(__int_as_float(acc[e]), sc, f[e]);
  };
  // The chains (4 output tiles x 2 token tiles per feature block) run back to back on the matrix
  // pipe, each with the fmas of the chain before it interleaved for the vector ALU -- across
  // feature blocks too: the last chain of a block is scaled in next to the first chain of the
  // next one.  Scheduling barriers and register anchors keep the compiler from stretching that
  // window (and the registers it needs).
  v16i pend = bias16;   // finished chain still to be scaled in (token tile 1, output tile 3); none yet: s = 0
  float pend_sc = 0.f;
  auto compute = [&](int kb, const v4i (&a)[2][4]) {
    const float mag = sx[(size_t)kb * RBx + rb] * sw[(size_t)kb * RBw + nt] * W8_STEP_INV;
    const float sc = (kb & 1) ? -mag : mag;
    const uint4* st = bst[kb % 3];
    v16i acc0;
#pragma unroll
    for (int ct = 0; ct < 4; ++ct) {
      v4i b[4];
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        union { uint4 u; v4i v; } x;
        x.u = st[(ct * 4 + ks) * 64 + lane];
        b[ks] = x.v;
      }
      acc0 = chain(b, a[0], pend);       // (from here on the previous chain's result may be read)
      v16f& ftile = facc[1][(ct + 3) & 3];
      scale_in(pend, pend_sc, ftile);
      asm volatile("" : "+v"(ftile) : : "memory");  // (the fmas stay in this window)
      asm volatile("" : "+v"(acc0) : : "memory");
      __builtin_amdgcn_sched_barrier(0);
      {
        v16i fresh = chain(b, a[1], acc0);
        pend = fresh;
      }
      pend_sc = sc;
      scale_in(acc0, sc, facc[0][ct]);
      asm volatile("" : "+v"(facc[0][ct]) : : "memory");
      asm volatile("" : "+v"(pend) : : "memory");
      __builtin_amdgcn_sched_barrier(0);
    }
    csum += sc;
  };

  // Pipeline.  The weight tiles run two feature blocks ahead of the products (three LDS stages),
  // the activation operands one block ahead (two register sets).  At the top of step kb
  // everything this wavefront has requested is waited for -- all of it was requested at least a
  // whole block earlier; the barrier then publishes everybody's share of stage kb and retires
  // stage kb - 1, which the copy of block kb + 2 overwrites.
  fetch_b(0);
  if (KB > 1) fetch_b(1);
  load_a(0, a0);
#define W8_STEP(KBI, ACUR, ANEXT)                       \
  {                                                     \
    const int kb_ = (KBI);                              \
    __builtin_amdgcn_s_waitcnt(0x0F70); /* vmcnt(0) */  \
    w8_barrier();                                       \
    if (kb_ + 2 < KB) fetch_b(kb_ + 2);                 \
    if (kb_ + 1 < KB) load_a(kb_ + 1, ANEXT);           \
    compute(kb_, ACUR);                                 \
  }
  {
    int kb = 0;
    for (; kb + 2 <= KB; kb += 2) {
      W8_STEP(kb, a0, a1)
      W8_STEP(kb + 1, a1, a0)
    }
    if (kb < KB) W8_STEP(kb, a0, a1)
  }
#undef W8_STEP
  // (the last chain's result: the wait states a vector read of a matrix product's result needs)
  asm volatile("s_nop 7\n\ts_nop 7\n\ts_nop 3" : "+v"(pend));
  scale_in(pend, pend_sc, facc[1][3]);

  // Epilogue: constant share out, bias in, bf16, through LDS so that rows leave as 256 contiguous
  // bytes.  Lane = token 32 rt + l32 of this wavefront; registers 4 g .. 4 g + 3 of tile ct =
  // outputs 32 ct + 8 g + 4 hf + 0..3.
  const float corr = W8_C0 * csum;
  w8_barrier();  // every wavefront is done with the stages
  unsigned char* my = (unsigned char*)bst + w * (32 * W8_EPI_STRIDE);
  const int n0 = nt * W8_WG_N;
#pragma unroll
  for (int r = 0; r < 2; ++r) {
#pragma unroll
    for (int ct = 0; ct < 4; ++ct)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        float bv[4] = {0.f, 0.f, 0.f, 0.f};
        if (bias) {
          const uint2 bw = *(const uint2*)(bias + n0 + 32 * ct + 8 * g + 4 * hf);
          bv[0] = bf16_lo(bw.x); bv[1] = bf16_hi(bw.x); bv[2] = bf16_lo(bw.y); bv[3] = bf16_hi(bw.y);
        }
        const v16f& f = facc[r][ct];
        *(uint2*)(my + l32 * W8_EPI_STRIDE + (32 * ct + 8 * g + 4 * hf) * 2) =
            make_uint2(pack_bf16x2(f[4 * g] - corr + bv[0], f[4 * g + 1] - corr + bv[1]),
                       pack_bf16x2(f[4 * g + 2] - corr + bv[2], f[4 * g + 3] - corr + bv[3]));
      }
    __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0): this wavefront's staging writes are done
    asm volatile("" ::: "memory");
#pragma unroll
    for (int it = 0; it < 8; ++it) {
      const int row = it * 4 + (lane >> 4), part = lane & 15;
      const int m = mt * W8_WG_M + 64 * w + 32 * r + row;
      const uint4 v = *(const uint4*)(my + row * W8_EPI_STRIDE + part * 16);
      if (m < M) *(uint4*)(y + (size_t)m * N + n0 + part * 8) = v;
    }
    asm volatile("" ::: "memory");
  }
}

// ---------------------------------------------------------------------------
void launch_w8a8_quantize(const void* a, int R, int K, int RP, bool negate_odd, int8_t* codes, float* scales,
                          hipStream_t stream) {
  const unsigned grid = (unsigned)((RP / QB) * (K / QB));
  w8a8_quantize_kernel<<<grid, 256, 0, stream>>>((const bf16_t*)a, R, K, RP, negate_odd ? 1 : 0, codes, scales);
}

void launch_w8a8_unpack(const int8_t* frag, const float* s, int R, int K, int RP, bool negate_odd, int8_t* codes,
                        float* scales, hipStream_t stream) {
  w8a8_unpack_kernel<<<2048, 256, 0, stream>>>(frag, s, R, K, RP, negate_odd ? 1 : 0, codes, scales);
}

void launch_w8a8_gemm(const int8_t* x8, const float* sx, int MP, const int8_t* w8, const float* sw,
                      const void* bias, void* y, int M, int N, int K, hipStream_t stream) {
  const int MT = MP / W8_WG_M, NT = N / W8_WG_N;
  const int mtx = (MT + 7) / 8;  // token tiles per XCD
  const unsigned grid = (unsigned)(8 * ((mtx + 7) / 8) * ((NT + 7) / 8) * 64);
  w8a8_gemm_kernel<<<grid, 256, 0, stream>>>(x8, sx, w8, sw, (const bf16_t*)bias, (bf16_t*)y, M, N, K, MP / 32,
                                             MP / QB, N / 32, N / QB, MT, NT);
}

}  // namespace sla
