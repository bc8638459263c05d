// lin_accumulate: per query block, the sums of the marginal key blocks' summaries,
//     HZ[i][n] = sum_{j : block j marginal for i} hz[j][n],   n over the 129*128 entries
// of a summary (h'^T and the z row), written as one dense contraction per (b,h):
//     HZ[Tq x 16512] = M0[Tq x Tk] . hz[Tk x 16512],   M0 = 1 where the mask is 0.
// This really is a GEMM (every summary is needed by ~n_m/Tk of all query blocks), so it
// runs on bf16 MFMA with fp32 accumulation; gathering n_m summaries per query block
// instead would move ~50x more bytes.
//
// The two operands could not be more different: hz is the big one (tens of MB per head) and
// M0 is a bit matrix.  So a workgroup owns a 128-column stripe of hz for 384 query blocks at
// once, the (few) row chunks of a stripe run at the same time on one XCD so that hz comes
// from HBM once, and M0 travels as bits: one 32-bit word per (query block,
// tile of 32 key blocks), 3 KiB per staged tile against 8 KiB of hz.  The bf16 A operand of a
// wavefront is made from its mask byte through a 256-entry table in LDS (entry b = the eight
// bf16 values 0.0 / 1.0 of the bits of b), one 16-byte LDS read per fragment.
//
// Workgroup = 4 wavefronts, two workgroups per CU (independent, so the two wavefronts of a
// SIMD are not in step); in a full chunk wavefront w owns query blocks [96 w, 96 w + 96) x 128
// columns (3 x 4 MFMA tiles of 32 x 32, 192 accumulator registers); a head's shorter last chunk
// is dealt to the wavefronts in even runs of row tiles and runs a copy of the loop with fewer
// tiles per wavefront.  Tiles are accumulated transposed (the hz fragment is the MFMA's A
// operand) so that a lane ends up with runs of consecutive entries of one query block's
// summary and can store 8 bytes at a time.  Operand tiles for 64 key blocks at a time are
// copied global -> LDS asynchronously, three stages deep (one barrier per tile).  hz rows are copied
// as they are (n contiguous) and read back with the LDS transposing read of gfx950
// (ds_read_b64_tr_b16): the contraction index j is the slow index of hz, so one transposition
// is unavoidable, and this one costs 8 LDS reads per 12 MFMAs and no vector-ALU work.
#include <type_traits>

#include "common.h"

namespace sla {

constexpr int LA_KSUB = 2;                       // 32-block groups per staged tile
constexpr int LA_KT = 32 * LA_KSUB;              // key blocks per staged tile (one barrier per tile)
constexpr int LA_ROWS = 384, LA_COLS = 128;      // workgroup tile
constexpr int LA_WAVES = 4;
constexpr int LA_M_ROWS = 512;                   // mask words staged per 32-block group (two 1 KiB pieces; 384 used)
constexpr int LA_B_ROW = LA_COLS * 2;            // 256 bytes per staged hz row
// each group of 8 staged rows starts 64 bytes after the previous one ends, so the two lane
// halves (which read rows 8 apart) hit different banks
constexpr int LA_B_BYTES = LA_KT * LA_B_ROW + (LA_KT / 8 - 1) * 64;
constexpr int LA_B_STAGE = (LA_B_BYTES + 255) / 256 * 256;
constexpr int LA_M_PIECES = 2 * LA_KSUB;         // 1 KiB pieces of mask words per tile
static_assert(HZ_ELEMS % LA_COLS == 0, "the stripes tile a summary exactly");
static_assert(LA_M_PIECES == LA_WAVES && 8 * LA_KSUB % LA_WAVES == 0, "every wavefront copies the same number of pieces");

__host__ __device__ inline int la_k_tiles(int Tk) { return (Tk + 31) / 32; }  // word columns of the bit matrix
__host__ __device__ inline int la_row_chunks(int Tq) { return (Tq + LA_ROWS - 1) / LA_ROWS; }
// row stride of the bit matrix: the chunks, plus the slack the last chunk's 512-word copies run into
__host__ __device__ inline int la_rows_padded(int Tq) { return la_row_chunks(Tq) * LA_ROWS + (LA_M_ROWS - LA_ROWS); }

// mbits[bh][kt][i] (kt < ceil(Tk/32), i < la_rows_padded(Tq)): bit e = 1 where key block 32 kt + e is marginal
// for query block i.  Words of rows >= Tq are never written and never matter (their results
// are not stored); bits of key blocks >= Tk are 0.
__global__ void marginal_bits_kernel(const int8_t* __restrict__ mask, int Tq, int Tk, int BH,
                                     uint32_t* __restrict__ mbits) {
  const int KT = la_k_tiles(Tk), TqP = la_rows_padded(Tq);
  const size_t total = (size_t)BH * KT * Tq;
  for (size_t x = (size_t)blockIdx.x * blockDim.x + threadIdx.x; x < total; x += (size_t)gridDim.x * blockDim.x) {
    const int i = (int)(x % Tq), kt = (int)((x / Tq) % KT), bh = (int)(x / ((size_t)Tq * KT));
    const int8_t* src = mask + ((size_t)bh * Tq + i) * Tk;
    uint32_t w = 0;
    for (int e = 0; e < 32; ++e) {
      const int j = kt * 32 + e;
      if (j < Tk && src[j] == 0) w |= 1u << e;
    }
    mbits[((size_t)bh * KT + kt) * TqP + i] = w;
  }
}

typedef __attribute__((address_space(3))) void* la_lds_ptr_t;

// Asynchronous 16-bytes-per-lane copy global -> LDS: lane l reads base + voff and the data lands
// at LDS address lds + 16 l.  Written as inline assembly on purpose: the compiler then neither
// knows nor cares that copies are in flight (it would otherwise make every LDS read it cannot
// prove disjoint wait for ALL of them); the pipeline below waits for them by explicit counts.
// Loads the compiler does not know about only make its own waits more conservative.
__device__ __forceinline__ void la_copy16(const void* base, unsigned voff, const void* lds) {
  const unsigned lds_addr = (unsigned)(uintptr_t)(la_lds_ptr_t)lds;
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %0"
               :
               : "s"(base), "v"(voff), "s"(lds_addr)
               : "memory", "m0");
}

// LDS read with transposition (16-bit elements): in every group of 16 lanes, lane i receives, for
// e = 0..3, element i % 4 of the 8 bytes addressed by lane 4 e + i / 4 of the group.  With lane
// s of a group addressing row s / 4, columns 4 (s % 4) .. +3 of a 4-row x 16-column patch, lane
// i ends up with the four rows of column i: a k-contiguous MFMA operand out of a row-major tile.
typedef short v4s __attribute__((ext_vector_type(4)));
__device__ __forceinline__ v4s la_read_tr(const unsigned char* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4s*)p);
}

__device__ __forceinline__ void la_barrier() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

__global__ void __launch_bounds__(LA_WAVES * 64, 2) lin_accumulate_kernel(const uint32_t* __restrict__ mbits,
                                                                          const bf16_t* __restrict__ hz, int Tq, int Tk,
                                                                          int n_items, bf16_t* __restrict__ HZ) {
  // three stages, each a tile of hz rows and the mask words that go with it; separate objects,
  // so the compiler can tell the asynchronous fill of one stage from the reads of another
  __shared__ __attribute__((aligned(1024))) unsigned char hz0[LA_B_STAGE], hz1[LA_B_STAGE], hz2[LA_B_STAGE];
  __shared__ __attribute__((aligned(1024))) uint32_t mw0[LA_KSUB * LA_M_ROWS], mw1[LA_KSUB * LA_M_ROWS], mw2[LA_KSUB * LA_M_ROWS];
  __shared__ uint4 lut[256];
  const int t = threadIdx.x, lane = t & 63, l32 = lane & 31, hf = lane >> 5;
  const int w = __builtin_amdgcn_readfirstlane(t >> 6);
  const int KT32 = la_k_tiles(Tk), KT = (KT32 + LA_KSUB - 1) / LA_KSUB, TqP = la_rows_padded(Tq);
  constexpr int STRIPES = HZ_ELEMS / LA_COLS;
  const int chunks = la_row_chunks(Tq);

  {  // table: mask byte -> eight bf16 0.0 / 1.0 (256 threads = 256 entries)
    uint32_t x[4];
#pragma unroll
    for (int e = 0; e < 4; ++e)
      x[e] = ((t >> (2 * e)) & 1 ? 0x3f80u : 0u) | ((t >> (2 * e + 1)) & 1 ? 0x3f800000u : 0u);
    lut[t] = make_uint4(x[0], x[1], x[2], x[3]);
  }

  const unsigned lane16 = (unsigned)lane * 16u;
  // this lane's address inside a B patch for the transposing reads: lane group g = lane / 16
  // serves columns 16 (g % 2) .. +15 and staged rows 8 (g / 2) + (0..3) [+ 4 for the second read]
  const int tr_off = (8 * (lane >> 5) + ((lane & 15) >> 2)) * LA_B_ROW + (lane >> 5) * 64 +
                     (16 * ((lane >> 4) & 1) + 4 * (lane & 3)) * 2;
  __syncthreads();  // publishes the table

  // Persistent workgroups, two per compute unit: each takes work items (b,h, stripe, row chunk)
  // in turn.  The row chunks of one stripe are consecutive items, and consecutive items go to
  // workgroups of the same XCD (workgroup ids are dealt round-robin over the 8 XCDs), so the
  // chunks of a stripe run at the same time on one L2 and the stripe comes from HBM once.  The
  // stripes of one head run next to each other in time (they share the head's mask words).
  // The stores of a finished item drain while the next item's copies and MFMAs already run.
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3, slots = gridDim.x >> 3;  // gridDim.x is a multiple of 8
  const int groups = n_items / chunks;  // (b,h, stripe) pairs; group g runs on XCD g % 8
  for (int it = slot; it < (groups + 7) / 8 * chunks; it += slots) {
  // item = 8 * (it / chunks) ... : groups of `chunks` consecutive items stay on one XCD
  // (the chunk a slot takes rotates from one round of the slots to the next: a head's last chunk
  // is usually shorter, and every workgroup should get its share of short ones)
  const int grp = it / chunks, rot = grp / max(1, slots / chunks);
  const int item = (grp * 8 + xcd) * chunks + (it % chunks + rot) % chunks;
  if (item >= n_items) continue;  // (uniform)
  const int chunk = item % chunks, stripe = (item / chunks) % STRIPES, bh = item / (chunks * STRIPES);
  const int n0 = stripe * LA_COLS, row0 = chunk * LA_ROWS;

  // asynchronous copy of tile kt into a stage, in 1 KiB pieces (4 hz rows, or 256 mask words)
  // dealt round-robin to the wavefronts
  const char* hz_bh = (const char*)(hz + (size_t)bh * Tk * HZ_ELEMS + n0);  // uniform
  const char* mb_bh = (const char*)(mbits + (size_t)bh * KT32 * TqP + row0);
  auto fetch = [&](int kt, unsigned char* hzs, uint32_t* mws) {
#pragma unroll
    for (int u = 0; u < 8 * LA_KSUB / LA_WAVES; ++u) {
      const int p = w + LA_WAVES * u;
      const int j = min(kt * LA_KT + 4 * p + (lane >> 4), Tk - 1);  // rows past Tk repeat the last one (their mask bits are 0)
      const unsigned off = (unsigned)j * (unsigned)(HZ_ELEMS * 2) + (unsigned)(lane & 15) * 16u;
      la_copy16(hz_bh, off, hzs + p * 1024 + (p >> 1) * 64);
    }
    {
      const int sub = w >> 1, part = w & 1;  // one mask piece per wavefront
      const int kt32 = min(kt * LA_KSUB + sub, KT32 - 1);  // (a word column past the end is ignored by the consumer)
      la_copy16(mb_bh + ((size_t)kt32 * TqP + 256 * part) * 4, lane16, mws + sub * LA_M_ROWS + part * 256);
    }
  };
  // copies of a wavefront per tile, and the wait that leaves at most one tile's worth in flight
  constexpr int PER_TILE = 8 * LA_KSUB / LA_WAVES + 1;
  static_assert(PER_TILE <= 15, "wait count immediate");
  auto wait_keep = [&](bool keep_one) {
    if (keep_one) __builtin_amdgcn_s_waitcnt(0x0F70 | PER_TILE);
    else __builtin_amdgcn_s_waitcnt(0x0F70);
  };

  // The chunk's row tiles (of 32 query blocks; 12 in a full chunk, fewer in a head's last one)
  // are dealt to the four wavefronts as evenly as consecutive runs allow, and the loop below is
  // instantiated for the largest share, so a short last chunk costs its share of MFMAs only.
  const int tiles_c = min(LA_ROWS / 32, (Tq - row0 + 31) / 32);
  const int t_base = tiles_c >> 2, t_rem = tiles_c & 3;
  const int my_tiles = t_base + (w < t_rem ? 1 : 0), wrow = 32 * (w * t_base + min(w, t_rem));
  auto run_item = [&](auto nmt_tag) {
  constexpr int NMT = decltype(nmt_tag)::value;
  v16f acc[NMT][4];
#pragma unroll
  for (int a = 0; a < NMT; ++a)
#pragma unroll
    for (int b = 0; b < 4; ++b) acc[a][b] = v16f{};

#define LA_COMPUTE(KTI, HZS, MWS)                                                                         \
  _Pragma("unroll") for (int sub = 0; sub < LA_KSUB; ++sub) {                                             \
    uint32_t mw[NMT];                                                                                     \
    const bool live = (KTI) * LA_KSUB + sub < KT32; /* uniform: the last tile may be partly past the end */ \
    _Pragma("unroll") for (int mt = 0; mt < NMT; ++mt)                                                    \
      mw[mt] = live ? MWS[sub * LA_M_ROWS + wrow + 32 * mt + l32] : 0u;                                   \
    _Pragma("unroll") for (int ks = 0; ks < 2; ++ks) {                                                    \
      v8bf aop[NMT], bop[4];                                                                              \
      _Pragma("unroll") for (int mt = 0; mt < NMT; ++mt) {                                                \
        union { uint4 u; v8bf v; } c;                                                                     \
        c.u = lut[(mw[mt] >> (16 * ks + 8 * hf)) & 0xffu];                                                \
        aop[mt] = c.v;                                                                                    \
      }                                                                                                   \
      _Pragma("unroll") for (int nt = 0; nt < 4; ++nt) {                                                  \
        /* staged rows r0 + 8 hf + (0..7) of column 32 nt + l32, by two transposing reads */              \
        union { v4s h[2]; v8bf v; } u;                                                                    \
        const int r0 = 32 * sub + 16 * ks, c0 = 64 * nt;                                                  \
        u.h[0] = la_read_tr(&HZS[tr_off + r0 * LA_B_ROW + (r0 >> 3) * 64 + c0]);                          \
        u.h[1] = la_read_tr(&HZS[tr_off + (r0 + 4) * LA_B_ROW + (r0 >> 3) * 64 + c0]);                    \
        bop[nt] = u.v;                                                                                    \
      }                                                                                                   \
      _Pragma("unroll") for (int mt = 0; mt < NMT; ++mt)                                                  \
        _Pragma("unroll") for (int nt = 0; nt < 4; ++nt)                                                  \
          acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bop[nt], aop[mt], acc[mt][nt], 0, 0, 0);  \
    }                                                                                                     \
  }

#define LA_STEP(KTI, HC, MC, HF, MF)           \
  {                                            \
    const int kt_ = (KTI);                     \
    if (kt_ + 2 < KT) fetch(kt_ + 2, HF, MF);  \
    LA_COMPUTE(kt_, HC, MC)                    \
    wait_keep(kt_ + 2 < KT);                   \
    la_barrier();                              \
  }
  fetch(0, hz0, mw0);
  if (KT > 1) fetch(1, hz1, mw1);
  wait_keep(KT > 1);
  la_barrier();
  int kt = 0;
  for (; kt + 3 <= KT; kt += 3) {
    LA_STEP(kt, hz0, mw0, hz2, mw2)
    LA_STEP(kt + 1, hz1, mw1, hz0, mw0)
    LA_STEP(kt + 2, hz2, mw2, hz1, mw1)
  }
  if (kt < KT) LA_STEP(kt, hz0, mw0, hz2, mw2)
  if (kt + 1 < KT) LA_STEP(kt + 1, hz1, mw1, hz0, mw0)
#undef LA_STEP
#undef LA_COMPUTE

  // The tiles were accumulated transposed (summary entries along the MFMA rows, query blocks
  // along its columns), so a lane owns ONE query block and runs of 4 consecutive entries of
  // its summary: 8-byte stores, the two lane halves completing 16 contiguous bytes.
  // (a wavefront with fewer row tiles than NMT has accumulated a neighbour's rows in the spare
  // tiles; it does not store them)
#pragma unroll
  for (int mt = 0; mt < NMT; ++mt) {
    const int i = row0 + wrow + 32 * mt + l32;
    if (mt < my_tiles && i < Tq) {
      bf16_t* dst = HZ + ((size_t)bh * Tq + i) * HZ_ELEMS + n0 + 4 * hf;
#pragma unroll
      for (int nt = 0; nt < 4; ++nt)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const v16f& a = acc[mt][nt];
          *(uint2*)(dst + 32 * nt + 8 * g) = make_uint2(pack_bf16x2(a[4 * g], a[4 * g + 1]), pack_bf16x2(a[4 * g + 2], a[4 * g + 3]));
        }
    }
  }
  };  // run_item
  const int nmt_item = t_base + (t_rem ? 1 : 0);
  if (nmt_item == 3) run_item(std::integral_constant<int, 3>{});
  else if (nmt_item == 2) run_item(std::integral_constant<int, 2>{});
  else run_item(std::integral_constant<int, 1>{});
  }  // work items
}

// The same bit matrix for the transposed mask (backward pass: sums over the query blocks that hold a
// key block as marginal): mbits_t[bh][qt][j] (qt < ceil(Tq/32), j < la_rows_padded(Tk)): bit e = 1 where
// key block j is marginal for query block 32 qt + e.
__global__ void marginal_bits_t_kernel(const int8_t* __restrict__ mask, int Tq, int Tk, int BH,
                                       uint32_t* __restrict__ mbits_t) {
  const int QT = la_k_tiles(Tq), TkP = la_rows_padded(Tk);
  const size_t total = (size_t)BH * QT * Tk;
  for (size_t x = (size_t)blockIdx.x * blockDim.x + threadIdx.x; x < total; x += (size_t)gridDim.x * blockDim.x) {
    const int j = (int)(x % Tk), qt = (int)((x / Tk) % QT), bh = (int)(x / ((size_t)Tk * QT));
    uint32_t w = 0;
    for (int e = 0; e < 32; ++e) {
      const int i = qt * 32 + e;
      if (i < Tq && mask[((size_t)bh * Tq + i) * Tk + j] == 0) w |= 1u << e;
    }
    mbits_t[((size_t)bh * QT + qt) * TkP + j] = w;
  }
}

size_t marginal_bits_t_bytes(const Problem& p) {
  return (size_t)p.BH * la_k_tiles(p.Tq) * la_rows_padded(p.Tk) * 4;
}

void launch_marginal_bits_t(const Problem& p, const int8_t* mask, uint32_t* mbits_t, hipStream_t stream) {
  const size_t total = (size_t)p.BH * la_k_tiles(p.Tq) * p.Tk;
  const size_t want = (total + 255) / 256;
  const unsigned grid = (unsigned)(want < 1048560 ? want : 1048560);
  marginal_bits_t_kernel<<<grid, 256, 0, stream>>>(mask, p.Tq, p.Tk, p.BH, mbits_t);
}

size_t marginal_bits_bytes(const Problem& p) {
  return (size_t)p.BH * la_k_tiles(p.Tk) * la_rows_padded(p.Tq) * 4;
}

void launch_marginal_bits(const Problem& p, const int8_t* mask, uint32_t* mbits, hipStream_t stream) {
  const size_t total = (size_t)p.BH * la_k_tiles(p.Tk) * p.Tq;
  const size_t want = (total + 255) / 256;
  const unsigned grid = (unsigned)(want < 1048560 ? want : 1048560);
  marginal_bits_kernel<<<grid, 256, 0, stream>>>(mask, p.Tq, p.Tk, p.BH, mbits);
}

void launch_lin_accumulate(const Problem& p, const uint32_t* mbits, const bf16_t* hz, bf16_t* HZ, hipStream_t stream) {
  const int n_items = (HZ_ELEMS / LA_COLS) * la_row_chunks(p.Tq) * p.BH;
  static int n_cu = 0;  // two workgroups per compute unit (192 accumulator registers per lane)
  if (n_cu == 0) {
    int dev = 0, v = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v <= 0) v = 256;
    n_cu = v;
  }
  int grid = 2 * n_cu / 8 * 8;  // a multiple of 8 (see the item order in the kernel)
  if (grid < 8) grid = 8;
  lin_accumulate_kernel<<<grid, LA_WAVES * 64, 0, stream>>>(mbits, hz, p.Tq, p.Tk, n_items, HZ);
}

}  // namespace sla
