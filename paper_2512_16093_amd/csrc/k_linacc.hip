// lin_accumulate: per query block, the sums of the marginal key blocks' summaries,
//     HZ[i][n] = sum_{j : block j marginal for i} hz[j][n],   n over the 129*128 entries
// of a summary (h'^T and the z row), written as one dense contraction per (b,h):
//     HZ[Tq x 16512] = M0[Tq x Tk] . hz[Tk x 16512],   M0 = 1 where the mask is 0.
// This really is a GEMM (every summary is needed by ~n_m/Tk of all query blocks), so it
// runs on bf16 MFMA with fp32 accumulation; gathering n_m summaries per query block
// instead would move ~50x more bytes.
//
// Workgroup = 4 wavefronts (2 x 2), tile 256 query blocks x 256 columns (128 x 128 per
// wavefront, 256 accumulator registers), looping over the row tiles of its column stripe so
// the stripe of hz comes from HBM once and is re-read from L2.  Operand tiles for 32 key
// blocks at a time are copied global -> LDS asynchronously, three stages deep:
//   A (mask as bf16 0/1) is pre-arranged in global memory in MFMA fragment order by
//     marginal_frag_kernel, so its copy is linear and its LDS reads are 16-byte, conflict free;
//   B (hz rows, n contiguous) is copied as is and read back transposed with 2-byte LDS reads
//     (the contraction index j is the slow index of hz; there is no way around one transposition).
#include "common.h"

namespace sla {

constexpr int LA_KT = 32;                      // key blocks per staged tile
constexpr int LA_TM = 256, LA_TN = 256;        // workgroup tile
constexpr int LA_A_BYTES = LA_TM * LA_KT * 2;  // 16 KiB
constexpr int LA_B_ROW = LA_TN * 2;            // 512 bytes per staged hz row
constexpr int LA_B_BYTES = LA_KT * LA_B_ROW + 3 * 64;  // each group of 8 rows starts 64 bytes after the previous
                                                     // one ends, so the two lane halves hit different banks
constexpr int LA_STAGE = LA_A_BYTES + LA_B_BYTES + 832;  // keep stages 1 KiB aligned
static_assert(LA_STAGE % 1024 == 0, "stage alignment");

__host__ __device__ inline int la_row_tiles(int Tq) { return (Tq + LA_TM - 1) / LA_TM; }
__host__ __device__ inline int la_k_tiles(int Tk) { return (Tk + LA_KT - 1) / LA_KT; }

// mA[bh][rt][kt][p][row][e] (bf16): 1.0 where block kt*32 + p*8 + e is marginal for query
// block rt*256 + row, else 0 (also outside the mask).  One 16-byte chunk per (p, row).
__global__ void marginal_frag_kernel(const int8_t* __restrict__ mask, int Tq, int Tk, bf16_t* __restrict__ mA) {
  const int RT = la_row_tiles(Tq), KT = la_k_tiles(Tk);
  const int kt = blockIdx.x % KT, rt = (blockIdx.x / KT) % RT, bh = blockIdx.x / (KT * RT);
  uint4* dst = (uint4*)(mA + ((size_t)(bh * RT + rt) * KT + kt) * (LA_A_BYTES / 2));
  for (int c = threadIdx.x; c < 4 * LA_TM; c += blockDim.x) {
    const int p = c / LA_TM, row = c % LA_TM, i = rt * LA_TM + row;
    uint32_t w[4] = {0, 0, 0, 0};
    if (i < Tq) {
      const int8_t* src = mask + ((size_t)bh * Tq + i) * Tk;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int j = kt * LA_KT + p * 8 + e;
        if (j < Tk && src[j] == 0) w[e >> 1] |= (e & 1) ? 0x3f800000u : 0x3f80u;
      }
    }
    dst[c] = make_uint4(w[0], w[1], w[2], w[3]);
  }
}

typedef __attribute__((address_space(3))) void* la_lds_ptr_t;

__device__ __forceinline__ void la_barrier() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

__global__ void __launch_bounds__(256, 1) lin_accumulate_kernel(const bf16_t* __restrict__ mA,
                                                                const bf16_t* __restrict__ hz, int Tq, int Tk,
                                                                bf16_t* __restrict__ HZ) {
  __shared__ __attribute__((aligned(1024))) unsigned char st0[LA_STAGE];
  __shared__ __attribute__((aligned(1024))) unsigned char st1[LA_STAGE];
  __shared__ __attribute__((aligned(1024))) unsigned char st2[LA_STAGE];
  const int bh = blockIdx.y;
  const int n0 = min((int)blockIdx.x * LA_TN, HZ_ELEMS - LA_TN);  // the last stripe overlaps its neighbour
  const int t = threadIdx.x, lane = t & 63, l32 = lane & 31, hf = lane >> 5;
  const int w = __builtin_amdgcn_readfirstlane(t >> 6), wm = w >> 1, wn = w & 1;
  const int RT = la_row_tiles(Tq), KT = la_k_tiles(Tk);
  const char* hz_bh = (const char*)(hz + (size_t)bh * Tk * HZ_ELEMS + n0);
  const unsigned lane16 = (unsigned)lane * 16u;

  for (int rt = 0; rt < RT; ++rt) {
    const char* a_rt = (const char*)(mA + ((size_t)(bh * RT + rt) * KT) * (LA_A_BYTES / 2));
    // asynchronous copy of k-tile kt into a stage: 4 + 4 one-KiB pieces per wavefront
    auto fetch = [&](int kt, unsigned char* st) {
      const char* a = a_rt + (size_t)kt * LA_A_BYTES;
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int piece = u * 4 + w;  // 16 pieces of 1 KiB
        __builtin_amdgcn_global_load_lds((const void*)(a + piece * 1024 + lane16),
                                         (la_lds_ptr_t)(st + piece * 1024), 16, 0, 0);
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int pr = u * 4 + w;  // pair of hz rows 2*pr, 2*pr+1; lanes 0..31 -> first row
        const int j = min(kt * LA_KT + 2 * pr + hf, Tk - 1);  // rows past Tk repeat the last one (their mask is 0)
        __builtin_amdgcn_global_load_lds((const void*)(hz_bh + (size_t)j * (HZ_ELEMS * 2) + (unsigned)l32 * 16u),
                                         (la_lds_ptr_t)(st + LA_A_BYTES + pr * 1024 + (pr >> 2) * 64), 16, 0, 0);
      }
    };
    v16f acc[4][4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
      for (int b = 0; b < 4; ++b) acc[a][b] = v16f{};

    auto compute = [&](const unsigned char* st) {
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
        v8bf aop[4], bop[4];
#pragma unroll
        for (int mt = 0; mt < 4; ++mt)
          aop[mt] = *(const v8bf*)(st + (((2 * ks + hf) * LA_TM) + 128 * wm + 32 * mt + l32) * 16);
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) {
          union { bf16_t h[8]; v8bf v; } u;
          const int r0 = 16 * ks + 8 * hf;  // 8 consecutive staged rows, all in one shifted/unshifted group
          const unsigned char* col = st + LA_A_BYTES + r0 * LA_B_ROW + (r0 >> 3) * 64 + (128 * wn + 32 * nt + l32) * 2;
#pragma unroll
          for (int e = 0; e < 8; ++e) u.h[e] = *(const bf16_t*)(col + e * LA_B_ROW);
          bop[nt] = u.v;
        }
#pragma unroll
        for (int mt = 0; mt < 4; ++mt)
#pragma unroll
          for (int nt = 0; nt < 4; ++nt)
            acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aop[mt], bop[nt], acc[mt][nt], 0, 0, 0);
      }
    };

#define LA_STEP(KTI, CUR, FILL)                                                            \
  {                                                                                        \
    const int kt_ = (KTI);                                                                 \
    if (kt_ + 2 < KT) fetch(kt_ + 2, FILL);                                                \
    compute(CUR);                                                                          \
    if (kt_ + 2 < KT) __builtin_amdgcn_s_waitcnt(0x0F78); else __builtin_amdgcn_s_waitcnt(0x0F70); \
    la_barrier();                                                                          \
  }
    __syncthreads();  // the previous row tile no longer reads any stage
    fetch(0, st0);
    if (KT > 1) fetch(1, st1);
    if (KT > 1) __builtin_amdgcn_s_waitcnt(0x0F78); else __builtin_amdgcn_s_waitcnt(0x0F70);
    la_barrier();
    int kt = 0;
    for (; kt + 3 <= KT; kt += 3) {
      LA_STEP(kt, st0, st2)
      LA_STEP(kt + 1, st1, st0)
      LA_STEP(kt + 2, st2, st1)
    }
    if (kt < KT) LA_STEP(kt, st0, st2)
    if (kt + 1 < KT) LA_STEP(kt + 1, st1, st0)
#undef LA_STEP

#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
      for (int nt = 0; nt < 4; ++nt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int i = rt * LA_TM + 128 * wm + 32 * mt + 8 * (r >> 2) + 4 * hf + (r & 3);
          if (i < Tq)
            HZ[((size_t)bh * Tq + i) * HZ_ELEMS + n0 + 128 * wn + 32 * nt + l32] = f32_to_bf16(acc[mt][nt][r]);
        }
  }
}

size_t marginal_frag_bytes(const Problem& p) {
  return (size_t)p.BH * la_row_tiles(p.Tq) * la_k_tiles(p.Tk) * LA_A_BYTES;
}

void launch_marginal_frag(const Problem& p, const int8_t* mask, bf16_t* mA, hipStream_t stream) {
  const unsigned grid = (unsigned)(p.BH * la_row_tiles(p.Tq) * la_k_tiles(p.Tk));
  marginal_frag_kernel<<<grid, 256, 0, stream>>>(mask, p.Tq, p.Tk, mA);
}

void launch_lin_accumulate(const Problem& p, const bf16_t* mA, const bf16_t* hz, bf16_t* HZ, hipStream_t stream) {
  dim3 grid((HZ_ELEMS + LA_TN - 1) / LA_TN, p.BH);
  lin_accumulate_kernel<<<grid, 256, 0, stream>>>(mA, hz, p.Tq, p.Tk, HZ);
}

}  // namespace sla
