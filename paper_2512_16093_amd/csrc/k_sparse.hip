// sparse_fwd: the block-sparse low-bit softmax branch with the linear branch fused
// into its epilogue (Section 1.3: SLA computed by one low-bit attention kernel;
// Section 1.1: INT8 QK^T / FP8 PV in the SageAttention2++ manner).
//
// One workgroup per (b,h,query block); one wavefront per 32 queries.  Everything is
// computed transposed so that a lane owns ONE query (column) throughout:
//   S^T[key][query]  = K8 . Q8^T      v_mfma_i32_32x32x32_i8, A = K fragment (LDS), B = Q8 (registers)
//   P8 = e4m3(448 2^(t - r))          in registers; r = integer running reference of the query, shared
//                                     by its two lanes (lane, lane^32): one permlane swap per 32 keys
//   O^T[ch][query] += V8^T . P8^T     v_mfma_f32_32x32x64_f8f6f4, A = V fragment (LDS), B = P8 as it
//                                     sits in the accumulators' order (V was stored in that key order)
// so the rescale factor, the row sum and the final normalisation are per-lane scalars and P
// never touches LDS.  K/V fragments of the next critical blocks are copied global -> LDS
// asynchronously (no registers) into a ring of staging buffers while the current ones are
// consumed (one barrier per block).
//
// The kernel is bound by the vector ALU (exp2, FP8 packing, the row maximum), not by the matrix
// pipe, and a wavefront issues at most one vector instruction every ~5 cycles; so the main loop
// is arranged for every MFMA to have independent vector work of the same wavefront behind it:
// the two 32-key halves of a block are pipelined against each other (while the matrix pipe
// computes the scores of one half, the vector ALU turns the other half's scores into P codes),
// and the P.V product runs one block behind.  A query's reference level only ever rises and is
// usually final after a few blocks, so the step tests each half's maximum in its own lane first
// and joins the lane pairs, rounds up and rescales only when some lane of the wavefront passes.
//
// Epilogue: O_s = acc * delta_V / l;  optional linear term phi(Q) H_i / (phi(Q).Z_i) as bf16 MFMA
// (H_i already contains the output projection), bias, then a transposing pass through LDS so
// the global stores are row-contiguous.
#include "common.h"

namespace sla {

struct SparseDims {
  int N, Tq, Tk, n_c, total, per_xcd, phi, has_lin, out_f32, H;
  int q8_rows;       // rows per (b,h) of the Q code tensor (N rounded up to whole groups of 128)
  int TqW, ustride;  // workgroup tiles per (b,h); entries per row of the paired lists (see PAIRED)
  Layout lq, lo;  // of q and out
};
// The pointers are separate __restrict__ kernel parameters (not struct members) so the
// compiler knows the index list and the scales are never written by this kernel and can
// fetch them through the scalar unit.
struct SparseArgs {
  const bf16_t* __restrict__ q;
  const int8_t* __restrict__ q8;
  const int32_t* __restrict__ crit;
  const int8_t* __restrict__ k8;
  const uint8_t* __restrict__ v8;
  const float* __restrict__ dq;
  const float* __restrict__ dk;
  const float* __restrict__ dv;
  const bf16_t* __restrict__ HZ;
  const bf16_t* __restrict__ bias;
  void* __restrict__ out;
  float* __restrict__ lse;
  int N, Tq, Tk, n_c, total, per_xcd, phi, has_lin, out_f32, H;
  Layout lq, lo;
  int TqW, ustride, q8_rows;
  const int32_t* __restrict__ ulen;
};

constexpr int EPI_STRIDE = 32 * 4 + 16;         // bytes per staged output row (32 fp32 + pad)
// Score bias: the integer accumulators of the score MFMAs start from the bit pattern of the
// float 1/(2 pi), which the instruction takes as an inline constant (no registers).  A finished
// accumulator, reinterpreted as fp32, is then the float BIAS_F + s * 2^-26 exactly, for every
// score |s| <= 127 * 127 * 128 < 0x22F983 (the pattern stays inside the binade [1/8, 1/4)):
// no int -> float conversion is needed, and patterns order like the scores.
constexpr int BIAS_I = 0x3E22F983;
constexpr int BIAS_FLOOR = 0x3E000000;          // pattern below every reachable score (masked keys)
constexpr float SCORE_STEP = 1.0f / 67108864.f;  // 2^-26: what one score unit adds to the float

__device__ __forceinline__ void load_q16(const bf16_t* p, bool ok, float* x) {
  uint4 a = make_uint4(0, 0, 0, 0), b = a;
  if (ok) {
    a = ((const uint4*)p)[0];
    b = ((const uint4*)p)[1];
  }
  const uint32_t w[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    x[2 * e] = bf16_lo(w[e]);
    x[2 * e + 1] = bf16_hi(w[e]);
  }
}

// Row state (per lane = per query): `r` is the running reference level, an INTEGER number of
// binary orders of magnitude (r = max over the 32-key tiles seen so far of ceil(log2(e) * row
// max)), so that P = 448 * 2^(t - r) <= 448 fits E4M3; `R` is the level the accumulators are
// expressed in.  Because r - R is an integer, a tile's contribution is brought to level R by
// the E8M0 block scale of the FP8 MFMA (2^(r-R) on the P operand): the accumulators are never
// rescaled on the vector ALU, except for a rare renormalisation when r - R exceeds 64.  The
// hardware takes the scale of a lane pair's registers 0..3 (keys 0..31 of the block) from the
// lower lane and that of registers 4..7 (keys 32..63) from the upper lane, so the two halves of
// a block may sit at different levels.  The row sum of the rounded P comes out of the same
// MFMA through a tile of ones.

__device__ __forceinline__ v4i as_v4i(const uint4& x) { return v4i{(int)x.x, (int)x.y, (int)x.z, (int)x.w}; }
__device__ __forceinline__ v8i as_v8i(const uint4& a, const uint4& b) {
  return v8i{(int)a.x, (int)a.y, (int)a.z, (int)a.w, (int)b.x, (int)b.y, (int)b.z, (int)b.w};
}

// Four consecutive 16-byte chunks (first, first + 1, ...) of a K or V record from LDS.
__device__ __forceinline__ void read4(const uint4* __restrict__ rec, int lane, int first, uint4 (&f)[4]) {
#pragma unroll
  for (int u = 0; u < 4; ++u) f[u] = rec[(first + u) * 64 + lane];
}

// One step (32 channels) of S^T = K8 . Q8^T for one 32-key half.
__device__ __forceinline__ v16i qk_step(const uint4& kf, const v4i& q8, const v16i& c) {
  return __builtin_amdgcn_mfma_i32_32x32x32_i8(as_v4i(kf), q8, c, 0, 0, 0);
}

// One 32-channel tile of O^T += V8^T . P8^T, P scaled by 2^(scale_p - 127).
__device__ __forceinline__ void pv_tile(const uint4& v0, const uint4& v1, const v8i& pb, int scale_p, v16f& acc) {
  acc = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(as_v8i(v0, v1), pb, acc, 0, 0, 0, 127, 0, scale_p);
}
// The row sum of P through the ones tile, same scale.
__device__ __forceinline__ void pv_rowsum(const v8i& ones, const v8i& pb, int scale_p, v16f& accl) {
  accl = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(ones, pb, accl, 0, 0, 0, 127, 0, scale_p);
}

// Maximum of this lane's 16 biased scores of one half (keys key0 .. key0 + 31), as a pattern.
template <bool tail>
__device__ __forceinline__ int half_max(v16i& s, int key0, int hf, int kvalid) {
  if (tail) {  // keys past the end of the sequence (last key block only) never win the max
#pragma unroll
    for (int q = 0; q < 16; ++q)
      if (key0 + 8 * (q >> 2) + 4 * hf + (q & 3) >= kvalid) s[q] = BIAS_FLOOR;
  }
  // two chains of three-operand maxima (7 + 9 values), joined at the end: 8 instructions
  int m0 = max(max(s[0], s[1]), s[2]), m1 = max(max(s[7], s[8]), s[9]);
  m0 = max(max(m0, s[3]), s[4]);
  m1 = max(max(m1, s[10]), s[11]);
  m0 = max(max(m0, s[5]), s[6]);
  m1 = max(max(m1, s[12]), s[13]);
  m1 = max(max(m1, s[14]), s[15]);
  return max(m0, m1);
}

// Per key block: the constants that turn a biased score pattern into exponents.  With
// c2s = c2 * 2^26 (c2 = log2(e) / sqrt(d) * delta_Q * delta_K) and x the pattern as a float,
//   t = c2 * s = fma(x, c2s, nb),   nb = -BIAS * c2s.
struct BlockConsts {
  float c2s;   // slope
  float nbg;   // nb + one score step: the guard keeps t - r <= 0 whatever the rounding of the products
  float lnb;   // log2(448) + nb: offs = lnb - r makes exp2(fma(x, c2s, offs)) = 448 * 2^(t - r)
};
__device__ __forceinline__ BlockConsts block_consts(float c2s) {
  // (explicit fused operations: the values must not depend on what the compiler chooses to contract)
  const float nb = -__int_as_float(BIAS_I) * c2s;
  return BlockConsts{c2s, __builtin_fmaf(c2s, SCORE_STEP, nb), __builtin_fmaf(c2s, -__int_as_float(BIAS_I), LOG2_448)};
}

// Row maximum over both lanes of the query -> new reference level r; returns offs (see above).
__device__ __forceinline__ float new_reference(int imax, const BlockConsts& bc, float pos_inf, float& r) {
  // after the swap one register holds the lower lane's value and the other the upper lane's, in both lanes
  const auto sw = __builtin_amdgcn_permlane32_swap(imax, imax, false, false);
  imax = max((int)sw[0], (int)sw[1]);
  const float cand = __builtin_ceilf(__builtin_fmaf(__int_as_float(imax), bc.c2s, bc.nbg));
  r = __builtin_amdgcn_fmed3f(r, cand, pos_inf);  // max(r, cand) in one instruction (both are finite)
  return bc.lnb - r;
}

// In-lane test value of a half's maximum: exceeds the (integer) reference level r exactly when the
// rounded-up level of this lane's scores would.
__device__ __forceinline__ float level_probe(int imax, const BlockConsts& bc) {
  return __builtin_fmaf(__int_as_float(imax), bc.c2s, bc.nbg);
}

// Four biased scores (accumulator registers 4g .. 4g+3 of one half) -> four FP8 codes of P in
// the returned word; `dst` supplies the register to overwrite half by half.
template <bool tail>
__device__ __forceinline__ int codes_quad(const v16i& s, int g, int key0, int hf, float c2s, float offs, int kvalid,
                                          int dst) {
  float p[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) p[e] = __builtin_amdgcn_exp2f(__builtin_fmaf(__int_as_float(s[4 * g + e]), c2s, offs));
  if (tail) {
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if (key0 + 8 * g + 4 * hf + e >= kvalid) p[e] = 0.f;
  }
  return cvt_pk_e4m3(p[2], p[3], cvt_pk_e4m3(p[0], p[1], dst, false), true);
}

// E8M0 code of 2^(r_prev - R): brings the P codes made at level r_prev to the accumulators'
// level R (r_prev - R <= 64 by the renormalisation rule; far below R the contribution vanishes).
// Rm127 = R - 127 is kept alongside R.
__device__ __forceinline__ int level_scale(float r_prev, float Rm127) {
  return (int)__builtin_amdgcn_fmed3f(r_prev - Rm127, 0.f, 254.f);
}

// Rare: the reference level has run more than 64 binades ahead of the accumulators' level
// (always so after the first block, whose R starts at "minus infinity"): bring them to level r.
__device__ __forceinline__ void renormalise(float r, float& R, float& Rm127, v16f (&acc)[4], v16f& accl) {
  const bool up = r - R > 64.f;
  const float down = up ? __builtin_amdgcn_exp2f(R - r) : 1.0f;
  if (up) {
    R = r;
    Rm127 = r - 127.f;
  }
#pragma unroll
  for (int ct = 0; ct < 4; ++ct)
#pragma unroll
    for (int q = 0; q < 16; ++q) acc[ct][q] *= down;
#pragma unroll
  for (int q = 0; q < 16; ++q) accl[q] *= down;
}

typedef __attribute__((address_space(3))) void* lds_ptr_t;

// Workgroup barrier for the staging pipeline.  __syncthreads() would also wait for EVERY
// outstanding memory operation, including the asynchronous copies of the blocks still in
// flight, which is exactly what the pipeline must not do.  Each wavefront has already waited
// (s_waitcnt vmcnt) for its own pieces of the block being published and has consumed (through
// its MFMAs) every LDS read of the stage being retired, so a bare s_barrier is sufficient; the
// empty asm statements only stop the compiler from moving memory accesses across it.
__device__ __forceinline__ void stage_barrier() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

// PAIRED (query blocks of 64, NW = 4): a workgroup serves TWO adjacent query blocks, wavefronts 0-1
// the first and 2-3 the second, over the merged list of their critical key blocks (crit_ then
// holds, per pair, the ascending union; bit 30 / 31 of an entry says that the first / second
// block of the pair has this key block in its own list; ulen_ holds the lengths).  Every K/V
// record is fetched once for both blocks and there are two wavefronts per SIMD (a workgroup of
// two wavefronts per 64 KB of staging rings would leave one).  A wavefront whose block does not
// have the current key block in its list goes through the step like the others and then drops
// what it computed: zero codes contribute nothing, the reference level is put back.
template <int NW, bool PAIRED>
__global__ void __launch_bounds__(NW * 64, 2) sparse_fwd_kernel(
    const bf16_t* __restrict__ q_, const int8_t* __restrict__ q8_, const int32_t* __restrict__ crit_, const int8_t* __restrict__ k8_,
    const uint8_t* __restrict__ v8_, const float* __restrict__ dq_, const float* __restrict__ dk_,
    const float* __restrict__ dv_, const bf16_t* __restrict__ HZ_, const bf16_t* __restrict__ bias_,
    void* __restrict__ out_, float* __restrict__ lse_, const int32_t* __restrict__ ulen_, const SparseDims dims) {
  static_assert(!PAIRED || NW == 4, "paired mode: four wavefronts, two per query block of 64");
  const SparseArgs A = {q_, q8_, crit_, k8_, v8_, dq_, dk_, dv_, HZ_, bias_, out_, lse_, dims.N, dims.Tq, dims.Tk,
                        dims.n_c, dims.total, dims.per_xcd, dims.phi, dims.has_lin, dims.out_f32, dims.H,
                        dims.lq, dims.lo, dims.TqW, dims.ustride, dims.q8_rows, ulen_};
  constexpr int NT = NW * 64;
  constexpr int CH = 2 * (KV_FRAG_BYTES / 16) / NT;  // 16-byte chunks per thread per block
  constexpr int BQ = NW * 32;
  // Rings of four K and four V staging buffers, declared as separate objects so the compiler
  // can tell the asynchronous fill of one from the reads of another; after the main loop
  // wavefront w reuses K buffer w for the output transposition.
  __shared__ uint4 kst0[KV_FRAG_BYTES / 16], kst1[KV_FRAG_BYTES / 16], kst2[KV_FRAG_BYTES / 16], kst3[KV_FRAG_BYTES / 16];
  __shared__ uint4 vst0[KV_FRAG_BYTES / 16], vst1[KV_FRAG_BYTES / 16], vst2[KV_FRAG_BYTES / 16], vst3[KV_FRAG_BYTES / 16];
  static_assert(32 * EPI_STRIDE <= KV_FRAG_BYTES, "output staging must fit one stage buffer");

  // Workgroup ids are dealt round-robin over the 8 XCDs.  All XCDs work on the SAME head at
  // the same time, each on its own contiguous eighth of that head's query blocks: the set of
  // K/V records in use chip-wide is then one head's (a few tens of MB, resident in the
  // Infinity Cache instead of being re-fetched from HBM), and the workgroups that share an
  // XCD's L2 are neighbouring query blocks, whose critical sets overlap.
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  // (the division runs on the vector ALU; its uniform result goes back to scalar registers)
  const int bh = __builtin_amdgcn_readfirstlane(slot / A.per_xcd);  // per_xcd = ceil(TqW / 8)
  const int i = xcd * A.per_xcd + (slot - bh * A.per_xcd);       // workgroup tile (of BQ queries)
  if (i >= A.TqW) return;

  const int t = threadIdx.x, lane = t & 63, w = t >> 6, l32 = lane & 31, hf = lane >> 5;
  const int pair_half = PAIRED ? __builtin_amdgcn_readfirstlane(w >> 1) : 0;
  // the query block whose scale, summaries and list membership this wavefront uses (an odd block
  // count leaves the last pair's second half without queries: clamped, nothing of it is stored)
  const int iq = PAIRED ? min(2 * i + pair_half, A.Tq - 1) : i;
  const int rowid = bh * A.Tq + iq;
  const int qrow = i * BQ + 32 * w + l32;
  const bool qok = qrow < A.N;
  const int b_ = __builtin_amdgcn_readfirstlane(bh / A.H), h_ = bh - b_ * A.H;
  const bf16_t* qptr = A.q + b_ * A.lq.sb + h_ * A.lq.sh + (qok ? qrow : 0) * A.lq.sn;

  // ---- Q block -> INT8 B operands (4 steps of 32 channels; this lane: 16 of each): the codes were made
  // with the block statistics (exact ties, see int8_code_word_exact); a lane half's 64 bytes are contiguous.
  const float dqi = A.dq[(size_t)rowid];
  v4i q8[4];
  {
    const v4i* src = (const v4i*)(A.q8 + ((size_t)bh * A.q8_rows + (qok ? qrow : 0)) * D + 64 * hf);
#pragma unroll
    for (int s = 0; s < 4; ++s) q8[s] = qok ? src[s] : v4i{0, 0, 0, 0};
  }
  const float cq = dqi * (LOG2E / 11.313708498984761f) * 67108864.f;  // log2(e) / sqrt(d) * delta_Q * 2^26 (see BIAS_I)

  v16f acc[4], accl = v16f{};
#pragma unroll
  for (int ct = 0; ct < 4; ++ct) acc[ct] = v16f{};
  // R starts far below any reachable level, so the first block renormalises (0 * 0) and sets R
  float r = -1e30f, R = -1e30f, Rm127 = -1e30f;
  float pos_inf = INFINITY;
  asm volatile("" : "+s"(pos_inf));  // in a scalar register: the third operand of the med3 that serves as max
  // A operand that sums P over the keys: FP8 1.0 in rows 0 and 4 of a 32-row tile, so the
  // row sum of a query lands in accumulator register 0 of both of its lanes.
  const int one4 = (l32 == 0 || l32 == 4) ? 0x38383838 : 0;
  v8i ones = {one4, one4, one4, one4, one4, one4, one4, one4};
  v16i bias16;
#pragma unroll
  for (int e = 0; e < 16; ++e) bias16[e] = BIAS_I;
  asm volatile("" : "+v"(bias16));  // kept in registers: the C operand of the first score MFMA of every half

  const int listrow = bh * A.TqW + i;
  const int n_c = PAIRED ? A.ulen[listrow] : A.n_c;
  // the critical list and the K scales are read through the scalar unit (uniform addresses)
  const int32_t* __restrict__ crow = PAIRED ? A.crit + (size_t)listrow * A.ustride : A.crit + (size_t)rowid * n_c;
  constexpr int JMASK = PAIRED ? 0x3FFFFFFF : -1;  // an entry's key block index
  // does this wavefront's query block have entry e in its own list?
  auto mine = [&](int e) { return !PAIRED || ((e >> (30 + pair_half)) & 1); };
  const float* __restrict__ dkrow = A.dk + (size_t)bh * A.Tk;
  const size_t rec0 = (size_t)bh * A.Tk * KV_FRAG_BYTES;
  // Asynchronous global -> LDS copy of one block's K or V record (no registers in between).
  // Wavefront w copies the PW adjacent 1 KiB pieces [PW w, PW w + PW) of the record, lane l
  // supplying bytes [16 l, 16 l + 16) of a piece; the instruction's immediate offset is added
  // to the global and to the LDS address alike.
  constexpr int PW = CH / 2;
  static_assert(PW == 2 || PW == 4, "pieces per wavefront per record");
  const int w_s = __builtin_amdgcn_readfirstlane(w);  // wavefront index as a scalar
  const unsigned lane_off = (unsigned)(w * PW * 1024 + lane * 16);
  const char* const k8_bh = (const char*)A.k8 + rec0;  // this (b,h)'s records: uniform, loop invariant
  const char* const v8_bh = (const char*)A.v8 + rec0;
  // Written as inline assembly so that (a) the record's address stays in scalar registers (base +
  // j * 8 KiB by scalar arithmetic, one loop-invariant vector offset per lane) and (b) the compiler
  // does not know copies are in flight: it would otherwise make every LDS read it cannot prove
  // disjoint wait for ALL of them.  The pipeline waits for them by explicit counts (loads the
  // compiler does not know about only make its own waits more conservative).
  auto fetch_rec = [&](const char* base_bh, int j, uint4* dst) {
    static_assert(KV_FRAG_BYTES == 1 << 13, "record size");
    const char* rec = base_bh + (unsigned)__builtin_amdgcn_readfirstlane(j << 13);
    const unsigned lds_addr = (unsigned)(uintptr_t)(lds_ptr_t)(dst + w_s * PW * 64);
    if constexpr (PW == 2) {
      asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\t"
                   "global_load_lds_dwordx4 %1, %0\n\t"
                   "global_load_lds_dwordx4 %1, %0 offset:1024"
                   :
                   : "s"(rec), "v"(lane_off), "s"(lds_addr)
                   : "memory", "m0");
    } else {
      asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\t"
                   "global_load_lds_dwordx4 %1, %0\n\t"
                   "global_load_lds_dwordx4 %1, %0 offset:1024\n\t"
                   "global_load_lds_dwordx4 %1, %0 offset:2048\n\t"
                   "global_load_lds_dwordx4 %1, %0 offset:3072"
                   :
                   : "s"(rec), "v"(lane_off), "s"(lds_addr)
                   : "memory", "m0");
    }
  };
  auto dk_of = [&](int j) { return *(const float*)((const char*)dkrow + (unsigned)__builtin_amdgcn_readfirstlane(j << 2)); };
  const int kvalid_last = A.N - (A.Tk - 1) * BK;  // valid keys of the last key block
  const bool ragged = kvalid_last < BK;

  // Software pipeline over the critical list.  Entering step b, the scores of keys 0..31 of
  // block b (s0) are finished and the K fragments of its keys 32..63 (kfB) are in registers.
  // Step b has two phases of the same shape, each a chain of MFMAs with one piece of vector-ALU
  // work behind every MFMA (scheduling barriers pin the pieces there: a wavefront issues in
  // order, and the pieces execute while the MFMA in front of them runs):
  //   phase 1  MFMAs: scores of keys 32..63 of block b (s1), P.V tiles 0, 1 of block b-1
  //            vector: s0 -> maximum -> reference level -> FP8 codes of keys 0..31 of block b
  //   phase 2  MFMAs: scores of keys 0..31 of block b+1 (new s0), P.V tiles 2, 3 and the row sum
  //            of block b-1;  vector: s1 -> ... -> codes of keys 32..63 of block b
  // Each phase starts by reading from LDS the fragments the NEXT phase's MFMAs need (V of block
  // b-1, K of block b+1) and by starting the copy of K(b+4) resp. V(b+2) into the ring slot
  // retired in step b-1 (past the end of the list the last block is copied again, into slots
  // nothing reads any more: the step stays free of branches).  At its end the wavefront waits
  // for its own pieces of K(b+2) / V(b) and meets the others at one barrier, which publishes
  // those and retires K slot (b+1)%4 and V slot (b-1)%4.  The L2 / HBM latency of a block is thus
  // covered by the arithmetic of two to three steps.  A ragged last key block can only be the
  // last entry of the (ascending) list; it is peeled off the loop so that masking its missing
  // keys costs the other blocks nothing.
  const int last = n_c - 1;
  const bool has_tail = ragged && n_c > 0 && (crow[last] & JMASK) == A.Tk - 1;
  // (SLA_FULL_WAITS: a checking build that waits for EVERY copy at each step instead of counting the
  // copies still allowed in flight; results must be bit-identical to the counting build.)
#ifdef SLA_FULL_WAITS
  constexpr int WAIT_KEEP2 = 0x0070;
#else
  constexpr int WAIT_KEEP2 = (2 * CH >= 16) ? 0x4070 : (0x0070 | (2 * CH));  // s_waitcnt vmcnt(2*CH) lgkmcnt(0)
#endif
  constexpr int WAIT_ALL = 0x0070;                                            // s_waitcnt vmcnt(0) lgkmcnt(0)
  constexpr int WAIT_KEEP_ALL_VM = 0xC07F;                                    // s_waitcnt lgkmcnt(0) only (vmcnt 63)
  v16i s0, s1;
  v8i pb_a = {}, pb_b = {};   // P codes of blocks b-1 / b (alternating); all-zero codes contribute nothing
  uint4 kfA[4], kfB[4], vfa[4], vfb[4];
  int sc_prev = 127;          // E8M0 scale of the P codes of block b-1 (this lane's half of it)

#define SB __builtin_amdgcn_sched_barrier(0);
#define SLA_STEP_P(B, KNEXT, VPREV, KFILL, VFILL, PBP, PBN)                                           \
  {                                                                                                   \
    const int b_ = (B);                                                                               \
    /* ---- phase 1 */                                                                                \
    read4(VPREV, lane, 0, vfa);                                                                       \
    read4(KNEXT, lane, 0, kfA);                                                                       \
    fetch_rec(k8_bh, j4, KFILL);                                                                       \
    const int jn_ = crow[min(b_ + 5, last)] & JMASK;                                                  \
    const int eb_ = PAIRED ? crow[b_] : 0;                                                            \
    const float rk_ = r;                                                                              \
    const float dn_ = dk_of(j4);                                                                      \
    const BlockConsts bc_ = block_consts(cq * d0);                                                    \
    SB s1 = qk_step(kfB[0], q8[0], bias16);                                                           \
    SB const int mA_ = half_max<false>(s0, 0, hf, 0);                                                 \
    SB s1 = qk_step(kfB[1], q8[1], s1);                                                               \
    SB const float offsA_ = new_reference(mA_, bc_, pos_inf, r);                                      \
    const float rA_ = r;                                                                              \
    SB s1 = qk_step(kfB[2], q8[2], s1);                                                               \
    SB PBN[0] = codes_quad<false>(s0, 0, 0, hf, bc_.c2s, offsA_, 0, PBN[0]);                                      \
    SB s1 = qk_step(kfB[3], q8[3], s1);                                                               \
    SB PBN[1] = codes_quad<false>(s0, 1, 0, hf, bc_.c2s, offsA_, 0, PBN[1]);                                      \
    SB pv_tile(vfa[0], vfa[1], PBP, sc_prev, acc[0]);                                                 \
    SB PBN[2] = codes_quad<false>(s0, 2, 0, hf, bc_.c2s, offsA_, 0, PBN[2]);                                      \
    SB pv_tile(vfa[2], vfa[3], PBP, sc_prev, acc[1]);                                                 \
    SB PBN[3] = codes_quad<false>(s0, 3, 0, hf, bc_.c2s, offsA_, 0, PBN[3]);                                      \
    /* ---- phase 2 */                                                                                \
    read4(VPREV, lane, 4, vfb);                                                                       \
    read4(KNEXT, lane, 4, kfB);                                                                       \
    fetch_rec(v8_bh, j2, VFILL);                                                                       \
    SB s0 = qk_step(kfA[0], q8[0], bias16);                                                           \
    SB const int mB_ = half_max<false>(s1, 32, hf, 0);                                                \
    SB s0 = qk_step(kfA[1], q8[1], s0);                                                               \
    SB const float offsB_ = new_reference(mB_, bc_, pos_inf, r);                                      \
    SB s0 = qk_step(kfA[2], q8[2], s0);                                                               \
    SB PBN[4] = codes_quad<false>(s1, 0, 32, hf, bc_.c2s, offsB_, 0, PBN[4]);                                     \
    SB s0 = qk_step(kfA[3], q8[3], s0);                                                               \
    SB PBN[5] = codes_quad<false>(s1, 1, 32, hf, bc_.c2s, offsB_, 0, PBN[5]);                                     \
    SB pv_tile(vfb[0], vfb[1], PBP, sc_prev, acc[2]);                                                 \
    SB PBN[6] = codes_quad<false>(s1, 2, 32, hf, bc_.c2s, offsB_, 0, PBN[6]);                                     \
    SB pv_tile(vfb[2], vfb[3], PBP, sc_prev, acc[3]);                                                 \
    SB PBN[7] = codes_quad<false>(s1, 3, 32, hf, bc_.c2s, offsB_, 0, PBN[7]);                                     \
    SB pv_rowsum(ones, PBP, sc_prev, accl);                                                           \
    if constexpr (PAIRED) {                                                                           \
      if (!mine(eb_)) { PBN = v8i{}; r = rk_; }                                                       \
    }                                                                                                 \
    SB const float rsel_ = (PAIRED && !mine(eb_)) ? rk_ : (hf ? r : rA_);   /* level of this lane's half of the new codes */ \
    j2 = j3; j3 = j4; j4 = jn_;                                                                       \
    d0 = d1; d1 = d2; d2 = d3; d3 = dn_;                                                              \
    /* anchor: keeps every piece inside this step */                                                  \
    asm volatile("" : "+v"(PBN), "+v"(acc[0]), "+v"(acc[1]), "+v"(acc[2]), "+v"(acc[3]), "+v"(accl),  \
                 "+v"(s0), "+s"(j4), "+s"(d3));                                                       \
    SB if (__any(r - R > 64.f)) renormalise(r, R, Rm127, acc, accl);                                  \
    sc_prev = level_scale(rsel_, Rm127);                                                                  \
    __builtin_amdgcn_s_waitcnt(WAIT_KEEP2);                                                           \
    stage_barrier();                                                                                  \
  }

  // The same step for unpaired workgroups, with the reference bookkeeping off the common path.  A
  // query's level r only ever rises, and after the first few blocks it has usually reached its
  // final value: a half's maximum is first tested in each lane alone (one fma and one compare: r
  // is an integer, so the rounded-up level of a lane pair exceeds r exactly when one of its two
  // lanes' own value does), and only if some lane of the wavefront passes does the wavefront join
  // the lane pairs, round up and raise r (a wave-uniform branch).  The exponent offset is formed
  // once per step, the scale of the codes just made is recomputed only in a step in which r moved
  // (and in the one after it, when the two halves of a block may still sit at different levels),
  // and the accumulators' level is looked at only then.
#define SLA_RAISE(IMAX)                                                                                \
  {                                                                                                   \
    const auto sw_ = __builtin_amdgcn_permlane32_swap(IMAX, IMAX, false, false);                      \
    const int im_ = max((int)sw_[0], (int)sw_[1]);                                                    \
    const float cand_ = __builtin_ceilf(__builtin_fmaf(__int_as_float(im_), bc_.c2s, bc_.nbg));       \
    r = __builtin_amdgcn_fmed3f(r, cand_, pos_inf);                                                   \
    offs_ = bc_.lnb - r;                                                                              \
    moved = 1;                                                                                        \
  }
#define SLA_STEP_F(B, KNEXT, VPREV, KFILL, VFILL, PBP, PBN)                                           \
  {                                                                                                   \
    const int b_ = (B);                                                                               \
    /* ---- phase 1 */                                                                                \
    read4(VPREV, lane, 0, vfa);                                                                       \
    read4(KNEXT, lane, 0, kfA);                                                                       \
    fetch_rec(k8_bh, j4, KFILL);                                                                       \
    const int jn_ = crow[min(b_ + 5, last)];                                                          \
    const float dn_ = dk_of(j4);                                                                      \
    const BlockConsts bc_ = block_consts(cq * d0);                                                    \
    float offs_ = bc_.lnb - r;                                                                        \
    const int moved_before = moved;                                                                   \
    moved = 0;                                                                                        \
    SB s1 = qk_step(kfB[0], q8[0], bias16);                                                           \
    SB const int mA_ = half_max<false>(s0, 0, hf, 0);                                                 \
    SB s1 = qk_step(kfB[1], q8[1], s1);                                                               \
    SB if (__any(level_probe(mA_, bc_) > r)) SLA_RAISE(mA_)                                           \
    const float rA_ = r;                                                                              \
    SB s1 = qk_step(kfB[2], q8[2], s1);                                                               \
    SB PBN[0] = codes_quad<false>(s0, 0, 0, hf, bc_.c2s, offs_, 0, PBN[0]);                           \
    SB s1 = qk_step(kfB[3], q8[3], s1);                                                               \
    SB PBN[1] = codes_quad<false>(s0, 1, 0, hf, bc_.c2s, offs_, 0, PBN[1]);                           \
    SB pv_tile(vfa[0], vfa[1], PBP, sc_prev, acc[0]);                                                 \
    SB PBN[2] = codes_quad<false>(s0, 2, 0, hf, bc_.c2s, offs_, 0, PBN[2]);                           \
    SB pv_tile(vfa[2], vfa[3], PBP, sc_prev, acc[1]);                                                 \
    SB PBN[3] = codes_quad<false>(s0, 3, 0, hf, bc_.c2s, offs_, 0, PBN[3]);                           \
    /* anchor: the branch below must not draw this phase's pieces past it */                          \
    asm volatile("" : "+v"(PBN), "+v"(s1), "+v"(acc[0]), "+v"(acc[1]));                               \
    /* ---- phase 2 */                                                                                \
    read4(VPREV, lane, 4, vfb);                                                                       \
    read4(KNEXT, lane, 4, kfB);                                                                       \
    fetch_rec(v8_bh, j2, VFILL);                                                                       \
    SB s0 = qk_step(kfA[0], q8[0], bias16);                                                           \
    SB const int mB_ = half_max<false>(s1, 32, hf, 0);                                                \
    SB s0 = qk_step(kfA[1], q8[1], s0);                                                               \
    SB if (__any(level_probe(mB_, bc_) > r)) SLA_RAISE(mB_)                                           \
    SB s0 = qk_step(kfA[2], q8[2], s0);                                                               \
    SB PBN[4] = codes_quad<false>(s1, 0, 32, hf, bc_.c2s, offs_, 0, PBN[4]);                          \
    SB s0 = qk_step(kfA[3], q8[3], s0);                                                               \
    SB PBN[5] = codes_quad<false>(s1, 1, 32, hf, bc_.c2s, offs_, 0, PBN[5]);                          \
    SB pv_tile(vfb[0], vfb[1], PBP, sc_prev, acc[2]);                                                 \
    SB PBN[6] = codes_quad<false>(s1, 2, 32, hf, bc_.c2s, offs_, 0, PBN[6]);                          \
    SB pv_tile(vfb[2], vfb[3], PBP, sc_prev, acc[3]);                                                 \
    SB PBN[7] = codes_quad<false>(s1, 3, 32, hf, bc_.c2s, offs_, 0, PBN[7]);                          \
    SB pv_rowsum(ones, PBP, sc_prev, accl);                                                           \
    j2 = j3; j3 = j4; j4 = jn_;                                                                       \
    d0 = d1; d1 = d2; d2 = d3; d3 = dn_;                                                              \
    /* anchor: keeps every piece inside this step */                                                  \
    asm volatile("" : "+v"(PBN), "+v"(acc[0]), "+v"(acc[1]), "+v"(acc[2]), "+v"(acc[3]), "+v"(accl),  \
                 "+v"(s0), "+s"(j4), "+s"(d3));                                                       \
    SB if (moved | moved_before) {                                                                    \
      if (__any(r - R > 64.f)) renormalise(r, R, Rm127, acc, accl);                                   \
      sc_prev = level_scale(hf ? r : rA_, Rm127);   /* level of this lane's half of the new codes */  \
    }                                                                                                 \
    __builtin_amdgcn_s_waitcnt(WAIT_KEEP2);                                                           \
    stage_barrier();                                                                                  \
  }
#define SLA_STEP(B, KNEXT, VPREV, KFILL, VFILL, PBP, PBN)                                             \
  if constexpr (PAIRED) SLA_STEP_P(B, KNEXT, VPREV, KFILL, VFILL, PBP, PBN)                           \
  else SLA_STEP_F(B, KNEXT, VPREV, KFILL, VFILL, PBP, PBN)
  int moved = 1;              // did the reference level of any query of this wavefront rise in the last step?

  if (n_c > 0) {  // (an empty list leaves only the linear term of the epilogue)
    // step 0 has no previous block: it multiplies all-zero P codes with this all-zero V slot
    for (int e = t; e < KV_FRAG_BYTES / 16; e += NT) vst3[e] = make_uint4(0, 0, 0, 0);
    // indices of blocks 0..4 and K scales of blocks 0..3 (clamped to the list)
    const int j0 = crow[0] & JMASK, j1 = crow[min(1, last)] & JMASK;
    int j2 = crow[min(2, last)] & JMASK, j3 = crow[min(3, last)] & JMASK, j4 = crow[min(4, last)] & JMASK;
    float d0 = dk_of(j0), d1 = dk_of(j1), d2 = dk_of(j2), d3 = dk_of(j3);
    // three groups of copies, in the order the steps will wait for them
    fetch_rec(k8_bh, j0, kst0);
    fetch_rec(k8_bh, j1, kst1);
    fetch_rec(k8_bh, j2, kst2);
    fetch_rec(v8_bh, j0, vst0);
    fetch_rec(k8_bh, j3, kst3);
    fetch_rec(v8_bh, j1, vst1);
    __builtin_amdgcn_s_waitcnt(WAIT_KEEP2);  // K(0), K(1) have landed
    stage_barrier();
    read4(kst0, lane, 0, kfA);
    read4(kst0, lane, 4, kfB);
    // Step 0 refills K slot 0 right away: every wavefront must have its fragments of block 0 in
    // registers before any wavefront starts that copy (inside the loop the barrier that ends a step
    // plays this part for the slot the next step refills).
    __builtin_amdgcn_s_waitcnt(WAIT_KEEP_ALL_VM);
    stage_barrier();
    s0 = qk_step(kfA[0], q8[0], bias16);
#pragma unroll
    for (int u = 1; u < 4; ++u) s0 = qk_step(kfA[u], q8[u], s0);
    const int nb_main = has_tail ? n_c - 1 : n_c;
    int b = 0;
    for (; b + 4 <= nb_main; b += 4) {
      SLA_STEP(b, kst1, vst3, kst0, vst2, pb_b, pb_a)
      SLA_STEP(b + 1, kst2, vst0, kst1, vst3, pb_a, pb_b)
      SLA_STEP(b + 2, kst3, vst1, kst2, vst0, pb_b, pb_a)
      SLA_STEP(b + 3, kst0, vst2, kst3, vst1, pb_a, pb_b)
    }
    // the (up to three) remaining steps keep the a/b alternation by copying the codes back
    if (b < nb_main) {
      SLA_STEP(b, kst1, vst3, kst0, vst2, pb_b, pb_a)
      pb_b = pb_a;
    }
    if (b + 1 < nb_main) {
      SLA_STEP(b + 1, kst2, vst0, kst1, vst3, pb_b, pb_a)
      pb_b = pb_a;
    }
    if (b + 2 < nb_main) {
      SLA_STEP(b + 2, kst3, vst1, kst2, vst0, pb_b, pb_a)
      pb_b = pb_a;
    }
    // drain: wait for every copy (the repeated ones too) and publish; from here on plain reads
    __builtin_amdgcn_s_waitcnt(WAIT_ALL);
    stage_barrier();
    if (has_tail) {  // the ragged last key block: s0 and kfB are ready, P.V of the block before it is due
      const int sp = (nb_main + 3) & 3;
      const uint4* vp = sp == 0 ? vst0 : sp == 1 ? vst1 : sp == 2 ? vst2 : vst3;
      read4(vp, lane, 0, vfa);
      read4(vp, lane, 4, vfb);
      const BlockConsts bct = block_consts(cq * d0);
      s1 = qk_step(kfB[0], q8[0], bias16);
#pragma unroll
      for (int u = 1; u < 4; ++u) s1 = qk_step(kfB[u], q8[u], s1);
      pv_tile(vfa[0], vfa[1], pb_b, sc_prev, acc[0]);
      pv_tile(vfa[2], vfa[3], pb_b, sc_prev, acc[1]);
      pv_tile(vfb[0], vfb[1], pb_b, sc_prev, acc[2]);
      pv_tile(vfb[2], vfb[3], pb_b, sc_prev, acc[3]);
      pv_rowsum(ones, pb_b, sc_prev, accl);
      const float rkt = r;
      const int mAt = half_max<true>(s0, 0, hf, kvalid_last);
      const float offsAt = new_reference(mAt, bct, pos_inf, r);
      const float rAt = r;
      v8i pb_t = {};
#pragma unroll
      for (int g = 0; g < 4; ++g) pb_t[g] = codes_quad<true>(s0, g, 0, hf, bct.c2s, offsAt, kvalid_last, pb_t[g]);
      const int mBt = half_max<true>(s1, 32, hf, kvalid_last);
      const float offsBt = new_reference(mBt, bct, pos_inf, r);
#pragma unroll
      for (int g = 0; g < 4; ++g) pb_t[4 + g] = codes_quad<true>(s1, g, 32, hf, bct.c2s, offsBt, kvalid_last, pb_t[4 + g]);
      pb_b = pb_t;
      if constexpr (PAIRED) {
        if (!mine(crow[last])) { pb_b = v8i{}; r = rkt; }
      }
      if (__any(r - R > 64.f)) renormalise(r, R, Rm127, acc, accl);
      sc_prev = level_scale((PAIRED && !mine(crow[last])) ? rkt : (hf ? r : rAt), Rm127);
    }
    {  // P.V of the last block
      const int sl = last & 3;
      const uint4* vc = sl == 0 ? vst0 : sl == 1 ? vst1 : sl == 2 ? vst2 : vst3;
      read4(vc, lane, 0, vfa);
      read4(vc, lane, 4, vfb);
      pv_tile(vfa[0], vfa[1], pb_b, sc_prev, acc[0]);
      pv_tile(vfa[2], vfa[3], pb_b, sc_prev, acc[1]);
      pv_tile(vfb[0], vfb[1], pb_b, sc_prev, acc[2]);
      pv_tile(vfb[2], vfb[3], pb_b, sc_prev, acc[3]);
      pv_rowsum(ones, pb_b, sc_prev, accl);
    }
  }
#undef SLA_STEP
#undef SLA_STEP_P
#undef SLA_STEP_F
#undef SLA_RAISE
#undef SB

  // ---- normalise: O_s[q][ch] = acc * delta_V[ch] / l
  const float ltot = accl[0];  // sum of the rounded P (scaled by 448), at level R
  const float inv_l = ltot > 0.f ? 1.0f / ltot : 0.f;
  if (A.lse && hf == 0 && qok)
    A.lse[(size_t)bh * A.N + qrow] = (R + __builtin_amdgcn_logf(ltot) - LOG2_448) * LN2;
#pragma unroll
  for (int ct = 0; ct < 4; ++ct)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const float4 d4 = *(const float4*)(A.dv + (size_t)bh * D + 32 * ct + 8 * g + 4 * hf);
      acc[ct][4 * g + 0] *= d4.x * inv_l;
      acc[ct][4 * g + 1] *= d4.y * inv_l;
      acc[ct][4 * g + 2] *= d4.z * inv_l;
      acc[ct][4 * g + 3] *= d4.w * inv_l;
    }

  // ---- linear branch: O_l^T[o][q] = sum_c H[o][c] phi(Q)[q][c], divided by phi(Q).Z
  if (A.has_lin) {
    const bf16_t* Hi = A.HZ + (size_t)rowid * HZ_ELEMS;
    v8bf bq[8];
    float den = 0.f;
    {
      float x[64];
#pragma unroll
      for (int s = 0; s < 4; ++s) load_q16(qptr + 32 * s + 16 * hf, qok, x + 16 * s);
      if (A.phi == 0) {
        float mx = x[0];
#pragma unroll
        for (int e = 1; e < 64; ++e) mx = fmaxf(mx, x[e]);
        mx = fmaxf(mx, partner_f32(mx));
        float sum = 0.f;
#pragma unroll
        for (int e = 0; e < 64; ++e) {
          x[e] = __builtin_amdgcn_exp2f((x[e] - mx) * LOG2E);
          sum += x[e];
        }
        sum += partner_f32(sum);
        const float inv = 1.0f / sum;
#pragma unroll
        for (int e = 0; e < 64; ++e) x[e] *= inv;
      } else if (A.phi == 1) {
#pragma unroll
        for (int e = 0; e < 64; ++e) x[e] = x[e] > 0.f ? x[e] + 1.0f : __builtin_amdgcn_exp2f(x[e] * LOG2E);
      } else {
#pragma unroll
        for (int e = 0; e < 64; ++e) x[e] = fmaxf(x[e], 0.f);
      }
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        float z[16];
        load_q16(Hi + D * D + 32 * s + 16 * hf, true, z);
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const __bf16 pb16 = (__bf16)x[16 * s + e];
          bq[2 * s + (e >> 3)][e & 7] = pb16;
          den = __builtin_fmaf((float)pb16, z[e], den);
        }
      }
    }
    den += partner_f32(den);
    const float inv_den = den != 0.f ? 1.0f / den : 0.f;  // no marginal block: no linear term
#pragma unroll
    for (int ot = 0; ot < 4; ++ot) {
      v16f al = v16f{};
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        const v8bf a = *(const v8bf*)(Hi + (size_t)hz_frag_chunk(ot, ks, lane) * 8);  // 1 KiB contiguous per wavefront
        al = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bq[ks], al, 0, 0, 0);
      }
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[ot][r] = __builtin_fmaf(al[r], inv_den, acc[ot][r]);
    }
    if (A.bias) {
#pragma unroll
      for (int ct = 0; ct < 4; ++ct)
#pragma unroll
        for (int r = 0; r < 16; ++r)
          acc[ct][r] += bf16_to_f32(A.bias[32 * ct + 8 * (r >> 2) + 4 * hf + (r & 3)]);
    }
  }

  // ---- transpose through LDS (per wavefront: 32 rows x 32 channels fp32 at a time) and store.
  // Wavefront w stages in K slot w, which nobody reads or fills any more (the drain barrier above came
  // after the last read of a K slot and after every copy had landed), so no workgroup barrier is
  // needed: a wavefront's LDS operations execute in the order it issues them.
  unsigned char* my = (unsigned char*)(w == 0 ? kst0 : w == 1 ? kst1 : w == 2 ? kst2 : kst3);
#pragma unroll
  for (int ct = 0; ct < 4; ++ct) {
    __builtin_amdgcn_wave_barrier();   // (compiler fence: the stores below stay behind the reads of the pass before)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const v16f& a = acc[ct];
      *(float4*)(my + l32 * EPI_STRIDE + (8 * g + 4 * hf) * 4) = make_float4(a[4 * g], a[4 * g + 1], a[4 * g + 2], a[4 * g + 3]);
    }
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int it = 0; it < 4; ++it) {
      const int rr = it * 8 + (lane >> 3), c4 = lane & 7;
      const int grow = i * BQ + 32 * w + rr;
      const float4 val = *(const float4*)(my + rr * EPI_STRIDE + c4 * 16);
      if (grow < A.N) {
        const size_t o = (size_t)(b_ * A.lo.sb + h_ * A.lo.sh + grow * A.lo.sn) + 32 * ct + 4 * c4;
        if (A.out_f32) {
          *(float4*)((float*)A.out + o) = val;
        } else {
          *(uint2*)((bf16_t*)A.out + o) = make_uint2(pack_bf16x2(val.x, val.y), pack_bf16x2(val.z, val.w));
        }
      }
    }
  }
}

// Paired mode (query blocks of 64): per pair of adjacent query blocks, the ascending union of
// their critical lists; bit 30 / 31 of an entry = the first / second block of the pair has it.
// One workgroup of 256 threads per pair; thread t owns key blocks 32 t .. 32 t + 31 (Tk <= 8192).
__global__ void __launch_bounds__(256) pair_union_kernel(const int32_t* __restrict__ crit, int Tq, int n_c, int TqW,
                                                         int ustride, int32_t* __restrict__ ulist,
                                                         int32_t* __restrict__ ulen) {
  __shared__ uint32_t bm[2][256];
  __shared__ int wave_cnt[4];
  const int row = blockIdx.x, bh = row / TqW, i = row - bh * TqW, t = threadIdx.x;
  bm[0][t] = 0u;
  bm[1][t] = 0u;
  __syncthreads();
  const int32_t* ra = crit + ((size_t)bh * Tq + 2 * i) * n_c;
  const bool has_b = 2 * i + 1 < Tq;
  for (int idx = t; idx < n_c; idx += 256) {
    const int a = ra[idx];
    atomicOr(&bm[0][a >> 5], 1u << (a & 31));
    if (has_b) {
      const int b = ra[n_c + idx];
      atomicOr(&bm[1][b >> 5], 1u << (b & 31));
    }
  }
  __syncthreads();
  const uint32_t wa = bm[0][t], wb = bm[1][t];
  uint32_t u = wa | wb;
  const int cnt = __popc(u);
  // exclusive prefix sum of cnt over the 256 threads
  int incl = cnt;
  for (int o = 1; o < 64; o <<= 1) {
    const int v = __shfl_up(incl, o);
    if ((t & 63) >= o) incl += v;
  }
  if ((t & 63) == 63) wave_cnt[t >> 6] = incl;
  __syncthreads();
  int base = 0;
  for (int k = 0; k < (t >> 6); ++k) base += wave_cnt[k];
  int pos = base + incl - cnt;
  int32_t* dst = ulist + (size_t)row * ustride;
  while (u) {
    const int bit = __ffs(u) - 1;
    u &= u - 1;
    dst[pos++] = (32 * t + bit) | (int)(((wa >> bit) & 1u) << 30) | (int)(((wb >> bit) & 1u) << 31);
  }
  if (t == 255) ulen[row] = base + incl;
}

void launch_sparse_fwd(const void* q, const int8_t* q8, const Problem& p, const int32_t* crit, int n_c, const int8_t* k8,
                       const uint8_t* v8, const float* dq, const float* dk, const float* dv,
                       const bf16_t* HZ, const bf16_t* proj_b, int phi_kind, bool has_linear,
                       void* out, bool out_f32, float* lse, int32_t* pair_list, int32_t* pair_len,
                       hipStream_t stream) {
  SparseDims dm;
  dm.N = p.N;
  dm.Tq = p.Tq;
  dm.Tk = p.Tk;
  dm.n_c = n_c;
  dm.total = p.BH * p.Tq;
  dm.phi = phi_kind;
  dm.has_lin = has_linear ? 1 : 0;
  dm.out_f32 = out_f32 ? 1 : 0;
  dm.H = p.H;
  dm.q8_rows = (p.N + 127) / 128 * 128;
  dm.lq = p.lq;
  dm.lo = p.lo;
  const bool paired = p.block_q == 64 && n_c > 0 && pair_list && pair_len;
  dm.TqW = paired ? (p.Tq + 1) / 2 : p.Tq;
  dm.ustride = 2 * n_c;
  dm.per_xcd = (dm.TqW + 7) / 8;  // workgroup tiles of one head per XCD
  const bf16_t* bias = has_linear ? proj_b : nullptr;
  const unsigned grid = (unsigned)(8 * dm.per_xcd * p.BH);
  if (paired) {
    pair_union_kernel<<<(unsigned)(p.BH * dm.TqW), 256, 0, stream>>>(crit, p.Tq, n_c, dm.TqW, dm.ustride, pair_list,
                                                                     pair_len);
    sparse_fwd_kernel<4, true><<<grid, 256, 0, stream>>>((const bf16_t*)q, q8, pair_list, k8, v8, dq, dk, dv, HZ, bias, out,
                                                         lse, pair_len, dm);
  } else if (p.block_q == 128) {
    sparse_fwd_kernel<4, false><<<grid, 256, 0, stream>>>((const bf16_t*)q, q8, crit, k8, v8, dq, dk, dv, HZ, bias, out, lse,
                                                          nullptr, dm);
  } else {
    sparse_fwd_kernel<2, false><<<grid, 128, 0, stream>>>((const bf16_t*)q, q8, crit, k8, v8, dq, dk, dv, HZ, bias, out, lse,
                                                          nullptr, dm);
  }
}

}  // namespace sla
