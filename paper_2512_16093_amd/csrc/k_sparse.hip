// sparse_fwd: the block-sparse low-bit softmax branch with the linear branch fused
// into its epilogue (Section 1.3: SLA computed by one low-bit attention kernel;
// Section 1.1: INT8 QK^T / FP8 PV in the SageAttention2++ manner).
//
// One workgroup per (b,h,query block); one wavefront per 32 queries.  Everything is
// computed transposed so that a lane owns ONE query (column) throughout:
//   S^T[key][query]  = K8 . Q8^T      v_mfma_i32_32x32x32_i8, A = K fragment (LDS), B = Q8 (registers)
//   P8 = e4m3(448 2^(t - r))          in registers; r = integer running reference of the query, shared
//                                     by its two lanes (lane, lane^32): one permlane swap per block
//   O^T[ch][query] += V8^T . P8^T     v_mfma_f32_32x32x64_f8f6f4, A = V fragment (LDS), B = P8 as it
//                                     sits in the accumulators' order (V was stored in that key order)
// so the rescale factor, the row sum and the final normalisation are per-lane scalars and P
// never touches LDS.  K/V fragments of the next three critical blocks are copied global -> LDS
// asynchronously (no registers) into the other staging buffers while the current one is
// consumed (one barrier per block).
//
// Epilogue: O_s = acc * delta_V / l;  optional linear term phi(Q) H_i / (phi(Q).Z_i) as bf16 MFMA
// (H_i already contains the output projection), bias, then a transposing pass through LDS so
// the global stores are row-contiguous.
#include "common.h"

namespace sla {

struct SparseDims {
  int N, Tq, Tk, n_c, total, per_xcd, phi, has_lin, out_f32;
};
// The pointers are separate __restrict__ kernel parameters (not struct members) so the
// compiler knows the index list and the scales are never written by this kernel and can
// fetch them through the scalar unit.
struct SparseArgs {
  const bf16_t* __restrict__ q;
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
  int N, Tq, Tk, n_c, total, per_xcd, phi, has_lin, out_f32;
};

constexpr int STAGE_BYTES = 2 * KV_FRAG_BYTES;  // K + V record of one key block
constexpr int EPI_STRIDE = 32 * 4 + 16;         // bytes per staged output row (32 fp32 + pad)
constexpr int IDX_CAP = 1024;                   // critical-list entries held in LDS at a time
constexpr int BIAS_I = 0x4B400000;              // bit pattern of 1.5 * 2^23
constexpr float BIAS_F = 12582912.0f;           // 1.5 * 2^23

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
// binary orders of magnitude (r = max over blocks of ceil(log2(e) * row max)), so that
// P = 448 * 2^(t - r) <= 448 fits E4M3; `R` is the level the accumulators are expressed in.
// Because r - R is an integer, a block's contribution is brought to level R by the E8M0
// block scale of the FP8 MFMA (2^(r-R) on the P operand): the accumulators are never
// rescaled on the vector ALU, except for a rare renormalisation when r - R exceeds 64.
// The row sum of the rounded P comes out of the same MFMA through a tile of ones.
//
// The three parts of a block are separate so the main loop can run the P.V product one block
// behind the scores: in step b a wavefront issues the score MFMAs of block b, then the P.V
// MFMAs of block b-1, then does the softmax arithmetic of block b on the vector ALU while
// those MFMAs execute.

// S^T = K8 . Q8^T for one key block (64 keys x this wavefront's 32 queries).  The integer
// accumulators start from BIAS_I = bits of 1.5 * 2^23, so each finished score, reinterpreted
// as fp32, IS the float 1.5 * 2^23 + s (exact for |s| < 2^22; here |s| <= 127 * 127 * 128):
// no int -> float conversion is needed afterwards.
__device__ __forceinline__ void qk_scores(const uint4* __restrict__ kl, int lane, const v4i (&q8)[4],
                                          const v16i& bias16, v16i& s0, v16i& s1) {
  uint4 kf[8];
#pragma unroll
  for (int u = 0; u < 8; ++u) kf[u] = kl[u * 64 + lane];
  s0 = bias16;
  s1 = bias16;
#pragma unroll
  for (int s = 0; s < 4; ++s) {
    s0 = __builtin_amdgcn_mfma_i32_32x32x32_i8(v4i{(int)kf[s].x, (int)kf[s].y, (int)kf[s].z, (int)kf[s].w}, q8[s], s0, 0, 0, 0);
    s1 = __builtin_amdgcn_mfma_i32_32x32x32_i8(v4i{(int)kf[4 + s].x, (int)kf[4 + s].y, (int)kf[4 + s].z, (int)kf[4 + s].w}, q8[s], s1, 0, 0, 0);
  }
}

// O^T += V8^T . P8^T (and the row sum through the ones tile), P scaled by 2^(scale_p - 127).
__device__ __forceinline__ void pv_accumulate(const uint4* __restrict__ vl, int lane, const v8i& pb, int scale_p,
                                              const v8i& ones, v16f (&acc)[4], v16f& accl) {
  uint4 vf[8];
#pragma unroll
  for (int u = 0; u < 8; ++u) vf[u] = vl[u * 64 + lane];
#pragma unroll
  for (int ct = 0; ct < 4; ++ct) {
    const uint4 a0 = vf[2 * ct], a1 = vf[2 * ct + 1];
    const v8i av = {(int)a0.x, (int)a0.y, (int)a0.z, (int)a0.w, (int)a1.x, (int)a1.y, (int)a1.z, (int)a1.w};
    acc[ct] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(av, pb, acc[ct], 0, 0, 0, 127, 0, scale_p);
  }
  accl = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(ones, pb, accl, 0, 0, 0, 127, 0, scale_p);
}

// First half of a block's softmax: row maximum of the biased scores -> reference level r
// (and the rare renormalisation of the accumulators).  Returns the exponent offset `offs`
// such that P = 448 * 2^(t - r) = exp2(fma(biased score, c2, offs)).
template <bool tail>
__device__ __forceinline__ float softmax_reference(v16i& s0, v16i& s1, int hf, float c2, int kvalid, float& r,
                                                   float& R, v16f (&acc)[4], v16f& accl) {
  if (tail) {  // keys past the end of the sequence (last key block only) never win the max
#pragma unroll
    for (int q = 0; q < 16; ++q) {
      const int key = 8 * (q >> 2) + 4 * hf + (q & 3);
      if (key >= kvalid) s0[q] = BIAS_I - 4000000;
      if (32 + key >= kvalid) s1[q] = BIAS_I - 4000000;
    }
  }
  int imax = s0[0];  // biased scores order like the scores themselves
#pragma unroll
  for (int q = 1; q < 16; ++q) imax = max(imax, s0[q]);
#pragma unroll
  for (int q = 0; q < 16; ++q) imax = max(imax, s1[q]);
  imax = max(imax, partner_i32(imax));
  // t = s * c2 = fma(bias + s, c2, -bias * c2); the guard of one score step keeps t - r <= 0
  // whatever the rounding of the two products
  const float nbc2 = -BIAS_F * c2;
  r = fmaxf(r, __builtin_ceilf(__builtin_fmaf(__int_as_float(imax), c2, nbc2) + c2));
  if (__any(r - R > 64.f)) {  // first block (R = -inf) or a jump of more than 64 binades
    const float down = (r - R > 64.f) ? __builtin_amdgcn_exp2f(R - r) : 1.0f;
    if (r - R > 64.f) R = r;
#pragma unroll
    for (int ct = 0; ct < 4; ++ct)
#pragma unroll
      for (int q = 0; q < 16; ++q) acc[ct][q] *= down;
#pragma unroll
    for (int q = 0; q < 16; ++q) accl[q] *= down;
  }
  return (LOG2_448 - r) + nbc2;
}

// Second half: biased scores -> FP8 codes of P.
template <bool tail>
__device__ __forceinline__ void softmax_codes(const v16i& s0, const v16i& s1, int hf, float c2, float offs,
                                              int kvalid, v8i& pb) {
  int code = 0;
#pragma unroll
  for (int g = 0; g < 4; ++g) {
    float p[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) p[e] = __builtin_amdgcn_exp2f(__builtin_fmaf(__int_as_float(s0[4 * g + e]), c2, offs));
    if (tail) {
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (8 * g + 4 * hf + e >= kvalid) p[e] = 0.f;
    }
    code = cvt_pk_e4m3(p[2], p[3], cvt_pk_e4m3(p[0], p[1], code, false), true);  // both halves overwritten
    pb[g] = code;
#pragma unroll
    for (int e = 0; e < 4; ++e) p[e] = __builtin_amdgcn_exp2f(__builtin_fmaf(__int_as_float(s1[4 * g + e]), c2, offs));
    if (tail) {
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (32 + 8 * g + 4 * hf + e >= kvalid) p[e] = 0.f;
    }
    code = cvt_pk_e4m3(p[2], p[3], cvt_pk_e4m3(p[0], p[1], code, false), true);
    pb[4 + g] = code;
  }
}

// E8M0 code of 2^(r_prev - R): brings the P codes made at level r_prev to the accumulators'
// level R (which may have moved up since; far below R the contribution vanishes).
__device__ __forceinline__ int level_scale(float r_prev, float R) {
  return 127 + (int)fmaxf(r_prev - R, -127.f);
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

template <int NW>
__global__ void __launch_bounds__(NW * 64, 2) sparse_fwd_kernel(
    const bf16_t* __restrict__ q_, const int32_t* __restrict__ crit_, const int8_t* __restrict__ k8_,
    const uint8_t* __restrict__ v8_, const float* __restrict__ dq_, const float* __restrict__ dk_,
    const float* __restrict__ dv_, const bf16_t* __restrict__ HZ_, const bf16_t* __restrict__ bias_,
    void* __restrict__ out_, float* __restrict__ lse_, const SparseDims dims) {
  const SparseArgs A = {q_, crit_, k8_, v8_, dq_, dk_, dv_, HZ_, bias_, out_, lse_, dims.N, dims.Tq, dims.Tk,
                        dims.n_c, dims.total, dims.per_xcd, dims.phi, dims.has_lin, dims.out_f32};
  constexpr int NT = NW * 64;
  constexpr int CH = 2 * (KV_FRAG_BYTES / 16) / NT;  // 16-byte chunks per thread per block
  constexpr int BQ = NW * 32;
  // Rings of four K and four V staging buffers, declared as separate objects so the compiler
  // can tell the asynchronous fill of one from the reads of another; after the main loop
  // wavefront w reuses K buffer w for the output transposition.  sidx / sdk hold the critical
  // list of this query block and the matching K scales (IDX_CAP entries at a time).
  __shared__ uint4 kst0[KV_FRAG_BYTES / 16], kst1[KV_FRAG_BYTES / 16], kst2[KV_FRAG_BYTES / 16], kst3[KV_FRAG_BYTES / 16];
  __shared__ uint4 vst0[KV_FRAG_BYTES / 16], vst1[KV_FRAG_BYTES / 16], vst2[KV_FRAG_BYTES / 16], vst3[KV_FRAG_BYTES / 16];
  __shared__ int sidx[IDX_CAP];
  __shared__ float sdk[IDX_CAP];
  static_assert(32 * EPI_STRIDE <= KV_FRAG_BYTES, "output staging must fit one stage buffer");

  // Workgroup ids are dealt round-robin over the 8 XCDs.  All XCDs work on the SAME head at
  // the same time, each on its own contiguous eighth of that head's query blocks: the set of
  // K/V records in use chip-wide is then one head's (a few tens of MB, resident in the
  // Infinity Cache instead of being re-fetched from HBM), and the workgroups that share an
  // XCD's L2 are neighbouring query blocks, whose critical sets overlap.
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int bh = slot / A.per_xcd, i = xcd * A.per_xcd + slot % A.per_xcd;  // per_xcd = ceil(Tq / 8)
  if (i >= A.Tq) return;
  const int rowid = bh * A.Tq + i;

  const int t = threadIdx.x, lane = t & 63, w = t >> 6, l32 = lane & 31, hf = lane >> 5;
  const int qrow = i * BQ + 32 * w + l32;
  const bool qok = qrow < A.N;
  const bf16_t* qptr = A.q + ((size_t)bh * A.N + (qok ? qrow : 0)) * D;

  // ---- Q block -> INT8 B operands (4 steps of 32 channels; this lane: 16 of each)
  const float dqi = A.dq[(size_t)bh * A.Tq + i];
  v4i q8[4];
#pragma unroll
  for (int s = 0; s < 4; ++s) {
    float x[16];
    load_q16(qptr + 32 * s + 16 * hf, qok, x);
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      uint32_t wv = 0;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        float c = __builtin_rintf(x[4 * g + e] / dqi);
        c = fminf(fmaxf(c, -127.f), 127.f);
        wv |= ((uint32_t)((int)c) & 0xffu) << (8 * e);
      }
      q8[s][g] = (int)wv;
    }
  }
  const float cq = dqi * (LOG2E / 11.313708498984761f);

  v16f acc[4], accl = v16f{};
#pragma unroll
  for (int ct = 0; ct < 4; ++ct) acc[ct] = v16f{};
  float r = -INFINITY, R = -INFINITY;
  // A operand that sums P over the keys: FP8 1.0 in rows 0 and 4 of a 32-row tile, so the
  // row sum of a query lands in accumulator register 0 of both of its lanes.
  const int one4 = (l32 == 0 || l32 == 4) ? 0x38383838 : 0;
  v8i ones = {one4, one4, one4, one4, one4, one4, one4, one4};
  v16i bias16;
#pragma unroll
  for (int e = 0; e < 16; ++e) bias16[e] = BIAS_I;
  asm volatile("" : "+v"(bias16));  // keep it in registers: it is the C operand of every first score MFMA

  const int n_c = A.n_c;
  const int32_t* crow = A.crit + (size_t)rowid * n_c;
  const float* dkrow = A.dk + (size_t)bh * A.Tk;
  const size_t rec0 = (size_t)bh * A.Tk * KV_FRAG_BYTES;
  // Asynchronous global -> LDS copy of one block's K and V records (no registers in between):
  // each wavefront fills 1 KiB pieces, lane l supplying bytes [16 l, 16 l + 16) of a piece.
  const int w_s = __builtin_amdgcn_readfirstlane(w);  // wavefront index as a scalar
  const unsigned lane_off = (unsigned)t * 16u;
  auto fetch_k = [&](int j, uint4* dst) {
    // uniform base (scalar registers) + 32-bit per-lane offset: no vector address arithmetic
    const char* ks = (const char*)A.k8 + rec0 + (size_t)j * KV_FRAG_BYTES;
#pragma unroll
    for (int u = 0; u < CH / 2; ++u)
      __builtin_amdgcn_global_load_lds((const void*)(ks + u * NT * 16 + lane_off),
                                       (lds_ptr_t)(dst + u * NT + w_s * 64), 16, 0, 0);
  };
  auto fetch_v = [&](int j, uint4* dst) {
    const char* vs = (const char*)A.v8 + rec0 + (size_t)j * KV_FRAG_BYTES;
#pragma unroll
    for (int u = 0; u < CH / 2; ++u)
      __builtin_amdgcn_global_load_lds((const void*)(vs + u * NT * 16 + lane_off),
                                       (lds_ptr_t)(dst + u * NT + w_s * 64), 16, 0, 0);
  };
  const int kvalid_last = A.N - (A.Tk - 1) * BK;  // valid keys of the last key block
  const bool ragged = kvalid_last < BK;

  // Software pipeline over the critical list.  In step b a wavefront
  //   - starts the copies of K(b+3) and V(b+2) into the ring slots retired in step b-1,
  //   - issues the score MFMAs of block b (K ring slot b%4) and reduces them to the new
  //     reference level r,
  //   - then, in ONE scheduling region, issues the P.V MFMAs of block b-1 (V ring slot
  //     (b-1)%4, P codes kept from step b-1) interleaved with the exp / FP8-pack arithmetic
  //     that turns the scores of block b into P codes: a wavefront that issues MFMAs back to
  //     back stalls once the matrix pipe's queue is full, so the vector-ALU work has to sit
  //     between them in program order to run while they execute,
  //   - waits for its own pieces of K(b+1) / V(b) and meets the other wavefronts at one barrier,
  //     which publishes those and retires K slot b%4 and V slot (b-1)%4.
  // The L2 / HBM latency of a block is thus covered by the arithmetic of three steps.  A ragged
  // last key block can only be the last entry of the (ascending) list; it is peeled off the
  // loop so that masking its missing keys costs the other blocks nothing.
  const bool has_tail = ragged && n_c > 0 && crow[n_c - 1] == A.Tk - 1;
  constexpr int WAIT_KEEP2 = (2 * CH >= 16) ? 0x4F70 : (0x0F70 | (2 * CH));  // s_waitcnt vmcnt(2*CH)
  v16i s0, s1;
  v8i pb_prev = {}, pb_new;   // P codes of block b-1 / b; all-zero codes contribute nothing
  float r_prev = 0.f;

#define SLA_STEP(B, KCUR, VPREV, KFILL, VFILL)                                                        \
  {                                                                                                   \
    const int b_ = (B);                                                                               \
    if (b_ + 3 < nb) fetch_k(__builtin_amdgcn_readfirstlane(jk3), KFILL);                             \
    if (b_ + 2 < nb) fetch_v(__builtin_amdgcn_readfirstlane(jv2), VFILL);                             \
    jv2 = jk3;                                                                                        \
    jk3 = sidx[min(b_ + 4, nb - 1)];                                                                  \
    const float c2_ = cq * dkv;                                                                       \
    dkv = sdk[min(b_ + 1, nb - 1)];                                                                   \
    qk_scores(KCUR, lane, q8, bias16, s0, s1);                                                        \
    __builtin_amdgcn_sched_barrier(0);                                                                \
    const float offs_ = softmax_reference<false>(s0, s1, hf, c2_, 0, r, R, acc, accl);                \
    const int sc_ = level_scale(r_prev, R);                                                           \
    __builtin_amdgcn_sched_barrier(0);                                                                \
    pv_accumulate(VPREV, lane, pb_prev, sc_, ones, acc, accl);                                        \
    softmax_codes<false>(s0, s1, hf, c2_, offs_, 0, pb_new);                                          \
    /* 8 LDS reads, then 5 x (1 MFMA, 17 vector-ALU instructions) */                                  \
    __builtin_amdgcn_sched_group_barrier(0x100, 8, 0);                                                \
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                                \
    __builtin_amdgcn_sched_group_barrier(0x002, 17, 0);                                               \
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                                \
    __builtin_amdgcn_sched_group_barrier(0x002, 17, 0);                                               \
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                                \
    __builtin_amdgcn_sched_group_barrier(0x002, 17, 0);                                               \
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                                \
    __builtin_amdgcn_sched_group_barrier(0x002, 17, 0);                                               \
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                                \
    __builtin_amdgcn_sched_group_barrier(0x002, 17, 0);                                               \
    /* anchor: P codes and accumulators are final here (keeps both computations inside this step) */  \
    asm volatile("" : "+v"(jk3), "+v"(jv2), "+v"(dkv), "+v"(pb_new), "+v"(acc[0]), "+v"(acc[1]),      \
                 "+v"(acc[2]), "+v"(acc[3]), "+v"(accl));                                             \
    __builtin_amdgcn_sched_barrier(0);                                                                \
    pb_prev = pb_new;                                                                                 \
    r_prev = r;                                                                                       \
    if (b_ + 3 < nb) __builtin_amdgcn_s_waitcnt(WAIT_KEEP2); else __builtin_amdgcn_s_waitcnt(0x0F70); \
    stage_barrier();                                                                                  \
  }

  for (int c0 = 0; c0 < n_c; c0 += IDX_CAP) {
    const int nb = min(IDX_CAP, n_c - c0);
    __syncthreads();  // the previous chunk's list and stages are no longer in use
    for (int e = t; e < nb; e += NT) {
      const int j = crow[c0 + e];
      sidx[e] = j;
      sdk[e] = dkrow[j];
    }
    // step 0 has no previous block: it multiplies all-zero P codes with this all-zero V slot
    for (int e = t; e < KV_FRAG_BYTES / 16; e += NT) vst3[e] = make_uint4(0, 0, 0, 0);
    __syncthreads();
    fetch_k(__builtin_amdgcn_readfirstlane(sidx[0]), kst0);
    fetch_v(__builtin_amdgcn_readfirstlane(sidx[0]), vst0);
    if (nb > 1) fetch_k(__builtin_amdgcn_readfirstlane(sidx[1]), kst1);
    if (nb > 1) fetch_v(__builtin_amdgcn_readfirstlane(sidx[1]), vst1);
    if (nb > 2) fetch_k(__builtin_amdgcn_readfirstlane(sidx[2]), kst2);
    int jk3 = sidx[min(3, nb - 1)];   // index of block b+3 (for K), read one step ahead of its use
    int jv2 = sidx[min(2, nb - 1)];   // index of block b+2 (for V)
    float dkv = sdk[0];               // K scale of block b, likewise
    if (nb > 2) __builtin_amdgcn_s_waitcnt(WAIT_KEEP2); else __builtin_amdgcn_s_waitcnt(0x0F70);
    stage_barrier();
    const int nb_main = (has_tail && c0 + nb == n_c) ? nb - 1 : nb;
    int b = 0;
    for (; b + 4 <= nb_main; b += 4) {
      SLA_STEP(b, kst0, vst3, kst3, vst2)
      SLA_STEP(b + 1, kst1, vst0, kst0, vst3)
      SLA_STEP(b + 2, kst2, vst1, kst1, vst0)
      SLA_STEP(b + 3, kst3, vst2, kst2, vst1)
    }
    if (b < nb_main) SLA_STEP(b, kst0, vst3, kst3, vst2)
    if (b + 1 < nb_main) SLA_STEP(b + 1, kst1, vst0, kst0, vst3)
    if (b + 2 < nb_main) SLA_STEP(b + 2, kst2, vst1, kst1, vst0)
    // drain: everything of this chunk has landed and been published (the last step waited for
    // all copies), so plain reads of any slot are safe from here on
    if (nb_main < nb) {  // the ragged last key block
      const int st = nb_main & 3, sp = (nb_main + 3) & 3;
      const uint4* kc = st == 0 ? kst0 : st == 1 ? kst1 : st == 2 ? kst2 : kst3;
      const uint4* vp = sp == 0 ? vst0 : sp == 1 ? vst1 : sp == 2 ? vst2 : vst3;
      qk_scores(kc, lane, q8, bias16, s0, s1);
      const float c2t = cq * sdk[nb_main];
      const float offs_t = softmax_reference<true>(s0, s1, hf, c2t, kvalid_last, r, R, acc, accl);
      pv_accumulate(vp, lane, pb_prev, level_scale(r_prev, R), ones, acc, accl);
      softmax_codes<true>(s0, s1, hf, c2t, offs_t, kvalid_last, pb_new);
      pb_prev = pb_new;
      r_prev = r;
    }
    {  // P.V of the chunk's last block
      const int sl = (nb - 1) & 3;
      const uint4* vc = sl == 0 ? vst0 : sl == 1 ? vst1 : sl == 2 ? vst2 : vst3;
      pv_accumulate(vc, lane, pb_prev, level_scale(r_prev, R), ones, acc, accl);
      pb_prev = v8i{};
    }
  }
#undef SLA_STEP

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
        const v8bf a = *(const v8bf*)(Hi + (size_t)(32 * ot + l32) * D + 32 * (ks >> 1) + 16 * hf + 8 * (ks & 1));
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

  // ---- transpose through LDS (per wavefront: 32 rows x 32 channels fp32 at a time) and store
  unsigned char* my = (unsigned char*)(w == 0 ? kst0 : w == 1 ? kst1 : w == 2 ? kst2 : kst3);
#pragma unroll
  for (int ct = 0; ct < 4; ++ct) {
    __syncthreads();
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const v16f& a = acc[ct];
      *(float4*)(my + l32 * EPI_STRIDE + (8 * g + 4 * hf) * 4) = make_float4(a[4 * g], a[4 * g + 1], a[4 * g + 2], a[4 * g + 3]);
    }
    __syncthreads();
#pragma unroll
    for (int it = 0; it < 4; ++it) {
      const int rr = it * 8 + (lane >> 3), c4 = lane & 7;
      const int grow = i * BQ + 32 * w + rr;
      const float4 val = *(const float4*)(my + rr * EPI_STRIDE + c4 * 16);
      if (grow < A.N) {
        const size_t o = ((size_t)bh * A.N + grow) * D + 32 * ct + 4 * c4;
        if (A.out_f32) {
          *(float4*)((float*)A.out + o) = val;
        } else {
          *(uint2*)((bf16_t*)A.out + o) = make_uint2(pack_bf16x2(val.x, val.y), pack_bf16x2(val.z, val.w));
        }
      }
    }
  }
}

void launch_sparse_fwd(const void* q, const Problem& p, const int32_t* crit, int n_c, const int8_t* k8,
                       const uint8_t* v8, const float* dq, const float* dk, const float* dv,
                       const bf16_t* HZ, const bf16_t* proj_b, int phi_kind, bool has_linear,
                       void* out, bool out_f32, float* lse, hipStream_t stream) {
  SparseDims dm;
  dm.N = p.N;
  dm.Tq = p.Tq;
  dm.Tk = p.Tk;
  dm.n_c = n_c;
  dm.total = p.BH * p.Tq;
  dm.per_xcd = (p.Tq + 7) / 8;  // query blocks of one head per XCD
  dm.phi = phi_kind;
  dm.has_lin = has_linear ? 1 : 0;
  dm.out_f32 = out_f32 ? 1 : 0;
  const bf16_t* bias = has_linear ? proj_b : nullptr;
  const unsigned grid = (unsigned)(8 * dm.per_xcd * p.BH);
  if (p.block_q == 128) {
    sparse_fwd_kernel<4><<<grid, 256, 0, stream>>>((const bf16_t*)q, crit, k8, v8, dq, dk, dv, HZ, bias, out, lse, dm);
  } else {
    sparse_fwd_kernel<2><<<grid, 128, 0, stream>>>((const bf16_t*)q, crit, k8, v8, dq, dk, dv, HZ, bias, out, lse, dm);
  }
}

}  // namespace sla
