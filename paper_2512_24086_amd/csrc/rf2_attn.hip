// Block-sparse flash attention (Sec. 3.1, eqs. 1-4 with the block skip rule) for gfx950.
//
// One workgroup owns one Q block (BLK rows) of one (batch, head) and walks that row's
// list of kept K/V blocks.  Work split inside the workgroup: wavefront (a, c) owns the
// 64 query rows of half `a` of the Q block and the keys of half `c` of every K/V block,
// with its own running (max, sum, output); the two key halves are merged once, after
// the last block, by the usual log-sum-exp combination.  Each A operand read from LDS
// then feeds two MFMAs (two 32-query tiles), which keeps LDS traffic at half the rate
// the matrix cores could consume.
//
// Both products are computed transposed so that no register shuffling is needed between
// them (v_mfma_f32_32x32x16_bf16, D = A(32xk) * B(kx32) + C):
//   S^T[key][query]  = K (A, from LDS)  * Q^T (B, registers, loaded once)
//   O^T[chan][query] = V^T (A, from LDS) * P^T (B, registers = exp of the S^T accumulators)
// In the accumulator layout lane l holds query column l%32 and, per 32-key tile, keys
// 8*(i/4) + 4*(l/32) + i%4 for i = 0..15.  Eight consecutive accumulator values are
// exactly one B operand of the second product provided the A operand (V^T) lists the keys
// of each 16-key group in the order 0-3, 8-11, 4-7, 12-15 -- the order rf2_permute writes.
// Row statistics are per lane (one query column) plus one exchange with lane l^32.
//
// The loop is software-pipelined over "units" (one 32-key tile per wavefront, i.e. a
// K/V block is KT = BLK/64 units): step s issues the matrix products S_{s+1} and
// O += V P_{s-1} around the softmax arithmetic of unit s, so the matrix cores and the
// vector ALU of a SIMD work at the same time although only one wavefront lives on it.
// K and V unit parts stream from global memory straight into two 4-deep LDS rings, three
// steps ahead of their use, with one barrier per step.
#include "rf2_internal.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;

template <int D, int BLK>
struct AttnCfg {
  static constexpr int NW = BLK / 32;           // wavefronts: (BLK/64 query halves) x (2 key halves)
  static constexpr int NT = NW * 64;
  static constexpr int KH = BLK / 2;            // keys per wavefront per block
  static constexpr int KT = KH / 32;            // units (32-key tiles per wavefront) per block
  static constexpr int QT = 2;                  // 32-query tiles per wavefront
  static constexpr int DS = D / 16;             // k-steps of the first product
  static constexpr int DT = D / 32;             // 32-channel tiles of the output
  static constexpr int TILE_BYTES = BLK * D * 2;
  static constexpr int UNIT_BYTES = TILE_BYTES / KT;   // K (or V^T) part of one unit: 64 keys x D
  static constexpr int LPW = UNIT_BYTES / 1024 / NW;   // 1 KiB direct-to-LDS loads per wavefront per unit part
  static constexpr int PENDING = 2 * 2 * LPW;          // loads a wavefront issues in two steps
  static_assert(LPW >= 1 && PENDING < 63, "vmcnt range");
};

// rf2_permute stores every K and V^T block as KT contiguous unit parts in exactly the
// order the operand reads below walk them ([chunk][64 rows][8 bf16], see rf2.h), so a
// part is copied verbatim: each wavefront-wide load deposits 64 x 16 B at consecutive
// LDS addresses (M0 = LDS base of that KiB), wavefront w taking KiB u*NW + w for
// u = 0..LPW-1.  In LDS the 16 lanes of a quarter-wave read 16 consecutive 16-byte slots
// (no bank conflicts) and all reads of a product share one per-lane base address plus
// compile-time offsets.
// The load is written in assembly on purpose: the compiler then does not track it, and
// the only waits for it are the explicit vmcnt waits of ring_barrier below (its own
// bookkeeping of direct-to-LDS loads runs out of slots with eight ring buffers and falls
// back to waiting for every outstanding load before unrelated LDS reads).
template <int NW, int LPW>
__device__ __forceinline__ void dma_unit(unsigned char* lds, const unsigned char* g, int wave, uint32_t tid16) {
  const uint32_t lds_base = (uint32_t)(size_t)(__attribute__((address_space(3))) unsigned char*)lds;
#pragma unroll
  for (int u = 0; u < LPW; ++u) {
    const uint32_t m0 = lds_base + (uint32_t)((u * NW + wave) * 1024);
    const unsigned char* src = g + u * (NW * 1024) + tid16;
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(m0), "v"(src) : "memory");
  }
}

// Workgroup barrier of the steady-state loop: waits until at most N of this wavefront's
// direct-to-LDS loads are still in flight, then s_barrier.  __syncthreads() cannot be used
// there: its release fence would wait for ALL outstanding loads, i.e. also for the parts
// prefetched for later steps.  LDS operand reads have completed before the barrier because
// the MFMAs consuming them were issued; the asm memory clobbers keep the compiler from
// moving LDS accesses across.
template <int N>
__device__ __forceinline__ void ring_barrier() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

template <int D, int BLK>
__global__ void __launch_bounds__(BLK * 2) block_sparse_attn_kernel(
    const __bf16* __restrict__ qp, const __bf16* __restrict__ kp, const __bf16* __restrict__ vp,
    const int32_t* __restrict__ blk_idx, const int32_t* __restrict__ blk_cnt, __bf16* __restrict__ op,
    float* __restrict__ lse, const int32_t* __restrict__ row_order, int rows_per_xcd, int Tb, int k_row,
    int last_valid, float scale_log2) {
  using C = AttnCfg<D, BLK>;
  // Rings of 4 K parts and 4 V^T parts.
  __shared__ __attribute__((aligned(1024))) unsigned char ring[8 * C::UNIT_BYTES];
  unsigned char* const K0 = ring;
  unsigned char* const K1 = ring + 1 * C::UNIT_BYTES;
  unsigned char* const K2 = ring + 2 * C::UNIT_BYTES;
  unsigned char* const K3 = ring + 3 * C::UNIT_BYTES;
  unsigned char* const V0 = ring + 4 * C::UNIT_BYTES;
  unsigned char* const V1 = ring + 5 * C::UNIT_BYTES;
  unsigned char* const V2 = ring + 6 * C::UNIT_BYTES;
  unsigned char* const V3 = ring + 7 * C::UNIT_BYTES;

  // ---- which Q block ---------------------------------------------------------------
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int bh = slot / rows_per_xcd;
  const int qi = row_order[xcd * rows_per_xcd + slot % rows_per_xcd];
  if (qi < 0) return;
  const size_t row_id = (size_t)bh * Tb + qi;
  int cnt = blk_cnt[row_id];
  const bool dense = (cnt == Tb);
  cnt = dense ? Tb : min(max(cnt, 0), k_row);
  const int32_t* __restrict__ list = blk_idx + row_id * k_row;
  const int U = cnt * C::KT;                            // units to process

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wavefront-uniform, kept in a scalar register
  const uint32_t tid16 = (uint32_t)tid * 16u;
  const int wa = wave >> 1, wc = wave & 1;
  const int l32 = lane & 31, lh = lane >> 5;
  const size_t head_off = (size_t)bh * Tb * BLK * D;    // elements; same for qp, kp, vp, op
  const unsigned char* __restrict__ kbase = reinterpret_cast<const unsigned char*>(kp + head_off);
  const unsigned char* __restrict__ vbase = reinterpret_cast<const unsigned char*>(vp + head_off);
  // LDS byte offsets of this lane's first operand chunk inside a K part / a V^T part
  const uint32_t k_lane = (uint32_t)((lh * 64 + wc * 32 + l32) * 16);
  const uint32_t v_lane = (uint32_t)(((wc * 4 + lh) * D + l32) * 16);
  auto block_at = [&](int it) {
    const int j = dense ? it : list[it];
    return min(max(j, 0), Tb - 1);                      // a corrupt list can give wrong results, never a fault
  };
  // global byte offset of unit x's part inside kp / vp of this head (x clamped: loads past the
  // end re-fetch the last unit into a free slot, which keeps the outstanding-load count uniform)
  auto unit_off = [&](int x) {
    x = min(x, U - 1);
    return (size_t)block_at(x / C::KT) * C::TILE_BYTES + (size_t)(x % C::KT) * C::UNIT_BYTES;
  };
  // Only the last listed block can be the ragged last block of the sequence (lists ascend).
  int partial_begin = U;
  if (U > 0 && last_valid < BLK && block_at(cnt - 1) == Tb - 1) partial_begin = (cnt - 1) * C::KT;

  bf16x8 qf[C::QT][C::DS];
  f32x16 o[C::DT][C::QT];
#pragma unroll
  for (int dt = 0; dt < C::DT; ++dt)
#pragma unroll
    for (int qt = 0; qt < C::QT; ++qt)
#pragma unroll
      for (int i = 0; i < 16; ++i) o[dt][qt][i] = 0.f;
  float m_run[C::QT], l_run[C::QT];
#pragma unroll
  for (int qt = 0; qt < C::QT; ++qt) { m_run[qt] = -INFINITY; l_run[qt] = 0.f; }

  // ---- building blocks ------------------------------------------------------------------
  // S^T of one unit (eq. 1, unscaled): 32 keys x 64 queries.
  auto qk = [&](const unsigned char* Kb, f32x16 (&S)[C::QT]) {
#pragma unroll
    for (int qt = 0; qt < C::QT; ++qt)
#pragma unroll
      for (int i = 0; i < 16; ++i) S[qt][i] = 0.f;
#pragma unroll
    for (int ds = 0; ds < C::DS; ++ds) {
      const bf16x8 a = *reinterpret_cast<const bf16x8*>(Kb + k_lane + ds * 2048);   // chunk 2*ds + lh, row wc*32 + l32
#pragma unroll
      for (int qt = 0; qt < C::QT; ++qt)
        S[qt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[qt][ds], S[qt], 0, 0, 0);
    }
  };
  // O^T += V^T P^T for one unit (eq. 4).
  auto pv = [&](const unsigned char* Vb, const bf16x8 (&P)[C::QT][2]) {
#pragma unroll
    for (int dt = 0; dt < C::DT; ++dt)
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
        const bf16x8 a = *reinterpret_cast<const bf16x8*>(Vb + v_lane + (2 * ks * D + 32 * dt) * 16);
#pragma unroll
        for (int qt = 0; qt < C::QT; ++qt)
          o[dt][qt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, P[qt][ks], o[dt][qt], 0, 0, 0);
      }
  };
  // The same two products with the A operands fetched from LDS ahead of time, so that the
  // LDS latency is paid once per step (under the row-maximum arithmetic), not per MFMA.
  auto load_k = [&](const unsigned char* Kb, bf16x8 (&A)[C::DS]) {
#pragma unroll
    for (int ds = 0; ds < C::DS; ++ds) A[ds] = *reinterpret_cast<const bf16x8*>(Kb + k_lane + ds * 2048);
  };
  auto load_v = [&](const unsigned char* Vb, bf16x8 (&A)[C::DT][2]) {
#pragma unroll
    for (int dt = 0; dt < C::DT; ++dt)
#pragma unroll
      for (int ks = 0; ks < 2; ++ks)
        A[dt][ks] = *reinterpret_cast<const bf16x8*>(Vb + v_lane + (2 * ks * D + 32 * dt) * 16);
  };
  auto qk_r = [&](const bf16x8 (&A)[C::DS], f32x16 (&S)[C::QT]) {
#pragma unroll
    for (int qt = 0; qt < C::QT; ++qt)
#pragma unroll
      for (int i = 0; i < 16; ++i) S[qt][i] = 0.f;
#pragma unroll
    for (int ds = 0; ds < C::DS; ++ds)
#pragma unroll
      for (int qt = 0; qt < C::QT; ++qt)
        S[qt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A[ds], qf[qt][ds], S[qt], 0, 0, 0);
  };
  auto pv_r = [&](const bf16x8 (&A)[C::DT][2], const bf16x8 (&P)[C::QT][2]) {
#pragma unroll
    for (int dt = 0; dt < C::DT; ++dt)
#pragma unroll
      for (int ks = 0; ks < 2; ++ks)
#pragma unroll
        for (int qt = 0; qt < C::QT; ++qt)
          o[dt][qt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A[dt][ks], P[qt][ks], o[dt][qt], 0, 0, 0);
  };
  // scaled row maxima of one unit, per query column (both lane halves end up with the same value)
  auto rowmax = [&](const f32x16 (&S)[C::QT], float (&mx)[C::QT]) {
#pragma unroll
    for (int qt = 0; qt < C::QT; ++qt) {
      float v = S[qt][0];
#pragma unroll
      for (int i = 1; i < 16; ++i) v = fmaxf(v, S[qt][i]);
      // exchange with lane l^32 on the vector ALU (an LDS shuffle would have to wait for the operand reads in flight)
      const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
      mx[qt] = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1])) * scale_log2;
    }
  };
  // Rarely taken: raise the running maximum (eq. 2) and rescale sum and output (eqs. 3, 4);
  // also where keys past the end of the sequence are masked out.
  // The maximum is only raised when a unit exceeds it by more than 2^8: until then
  // probabilities are at most 256 (the exact final normalisation makes the reference point
  // irrelevant) and the 128-register output rescale is skipped for most units.
  auto slow_path = [&](f32x16 (&S)[C::QT], float (&mx)[C::QT], int s) {
    if (s >= partial_begin) {
      const int kt = s % C::KT;
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int key = wc * C::KH + 32 * kt + 8 * (i / 4) + 4 * lh + (i % 4);
        if (key >= last_valid) {
#pragma unroll
          for (int qt = 0; qt < C::QT; ++qt) S[qt][i] = -INFINITY;
        }
      }
      rowmax(S, mx);
    }
#pragma unroll
    for (int qt = 0; qt < C::QT; ++qt) {
      const bool raise = mx[qt] > m_run[qt] + 8.0f;       // -inf + 8 = -inf: the first finite unit always raises
      if (__builtin_amdgcn_ballot_w64(raise) != 0ull) {
        const float alpha = raise ? __builtin_amdgcn_exp2f(m_run[qt] - mx[qt]) : 1.0f;   // exp2(-inf) = 0
        m_run[qt] = raise ? mx[qt] : m_run[qt];
        l_run[qt] *= alpha;
#pragma unroll
        for (int dt = 0; dt < C::DT; ++dt)
#pragma unroll
          for (int i = 0; i < 16; ++i) o[dt][qt][i] *= alpha;
      }
    }
  };
  auto need_slow = [&](const float (&mx)[C::QT], int s) {
    bool raise = false;
#pragma unroll
    for (int qt = 0; qt < C::QT; ++qt) raise |= mx[qt] > m_run[qt] + 8.0f;
    return (__builtin_amdgcn_ballot_w64(raise) != 0ull) || (s >= partial_begin);
  };
  // probabilities of one unit relative to the running maximum, packed as B operands (eqs. 2, 3)
  auto expsum = [&](const f32x16 (&S)[C::QT], bf16x8 (&P)[C::QT][2]) {
#pragma unroll
    for (int qt = 0; qt < C::QT; ++qt) {
      const float m_use = (m_run[qt] == -INFINITY) ? 0.f : m_run[qt];
      float rs = 0.f;
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(S[qt][i], scale_log2, -m_use));
        rs += p;
        P[qt][i / 8][i % 8] = (__bf16)p;
      }
      l_run[qt] += rs;
    }
  };

  if (U > 0) {
    // ---- prologue: fill the rings, load Q, first unit ------------------------------------
    dma_unit<C::NW, C::LPW>(K0, kbase + unit_off(0), wave, tid16);
    dma_unit<C::NW, C::LPW>(V0, vbase + unit_off(0), wave, tid16);
    dma_unit<C::NW, C::LPW>(K1, kbase + unit_off(1), wave, tid16);
    dma_unit<C::NW, C::LPW>(K2, kbase + unit_off(2), wave, tid16);
    dma_unit<C::NW, C::LPW>(K3, kbase + unit_off(3), wave, tid16);
    dma_unit<C::NW, C::LPW>(V1, vbase + unit_off(1), wave, tid16);
#pragma unroll
    for (int qt = 0; qt < C::QT; ++qt) {
      const __bf16* qrow = qp + head_off + ((size_t)qi * BLK + 64 * wa + 32 * qt + l32) * D + 8 * lh;
#pragma unroll
      for (int ds = 0; ds < C::DS; ++ds) qf[qt][ds] = *reinterpret_cast<const bf16x8*>(qrow + 16 * ds);
    }
    f32x16 Sa[C::QT], Sb[C::QT];
    bf16x8 Pa[C::QT][2], Pb[C::QT][2];
    float mx[C::QT];
    bf16x8 ak[C::DS], av[C::DT][2];
    ring_barrier<0>();
    qk(K0, Sa);                                           // S_0
    __syncthreads();                                      // everyone is done with slot K0
    // step 0 (no P yet): softmax of unit 0 around S_1
    dma_unit<C::NW, C::LPW>(K0, kbase + unit_off(4), wave, tid16);
    dma_unit<C::NW, C::LPW>(V2, vbase + unit_off(2), wave, tid16);
    rowmax(Sa, mx);
    slow_path(Sa, mx, 0);
    expsum(Sa, Pa);
    qk(K1, Sb);

    // ---- steady state: step s = products S_{s+1} and V P_{s-1} around the softmax of unit s --
    // Ring slots: K part of unit x and V^T part of unit x live in slot x % 4.  Step s loads the
    // K part of unit s+4 and the V^T part of unit s+2 into the slots freed by step s-1.
#define RF2_STEP(s_, Kissue, Vissue, Vprev, Knext, Scur, Snext, Pprev, Pcur)                 \
  {                                                                                          \
    ring_barrier<C::PENDING>();                                                              \
    dma_unit<C::NW, C::LPW>(Kissue, kbase + off_k, wave, tid16);                             \
    dma_unit<C::NW, C::LPW>(Vissue, vbase + off_v, wave, tid16);                             \
    off_k = unit_off((s_) + 5); /* for the next step: the list entry is fetched a step ahead */ \
    off_v = unit_off((s_) + 3);                                                              \
    load_v(Vprev, av);                                                                       \
    load_k(Knext, ak);                                                                       \
    rowmax(Scur, mx);                                                                        \
    if (need_slow(mx, (s_))) {                                                               \
      /* the pending product must reach O before O is rescaled; it is then neutralised */    \
      pv_r(av, Pprev);                                                                       \
      _Pragma("unroll") for (int qt = 0; qt < C::QT; ++qt)                                   \
        _Pragma("unroll") for (int ks = 0; ks < 2; ++ks)                                     \
          _Pragma("unroll") for (int e = 0; e < 8; ++e) Pprev[qt][ks][e] = (__bf16)0.f;      \
      slow_path(Scur, mx, (s_));                                                             \
    }                                                                                        \
    pv_r(av, Pprev);                                                                         \
    expsum(Scur, Pcur);                                                                      \
    qk_r(ak, Snext);                                                                         \
  }
    size_t off_k = unit_off(5), off_v = unit_off(3);
    for (int s = 1; s < U; s += 4) {
      RF2_STEP(s, K1, V3, V0, K2, Sb, Sa, Pa, Pb)
      if (s + 1 < U) RF2_STEP(s + 1, K2, V0, V1, K3, Sa, Sb, Pb, Pa)
      if (s + 2 < U) RF2_STEP(s + 2, K3, V1, V2, K0, Sb, Sa, Pa, Pb)
      if (s + 3 < U) RF2_STEP(s + 3, K0, V2, V3, K1, Sa, Sb, Pb, Pa)
    }
#undef RF2_STEP
    // ---- last product: O += V P_{U-1} ------------------------------------------------------
    ring_barrier<0>();
    switch ((U - 1) & 3) {
      case 0: pv(V0, Pa); break;
      case 1: pv(V1, Pb); break;
      case 2: pv(V2, Pa); break;
      default: pv(V3, Pb); break;
    }
  }

  // ---- merge the two key halves and write the Q block -------------------------------------
  __syncthreads();                                        // every wavefront is done with the rings
  float* ml = reinterpret_cast<float*>(V0);               // [wa][wc][qt][m|l][lane]: 4 KiB at most
  static_assert((BLK / 64) * 2 * C::QT * 2 * 64 * 4 <= C::UNIT_BYTES, "");
  float l_tot[C::QT];
#pragma unroll
  for (int qt = 0; qt < C::QT; ++qt) {
    l_tot[qt] = l_run[qt] + __shfl_xor(l_run[qt], 32);
    ml[(((wa * 2 + wc) * C::QT + qt) * 2 + 0) * 64 + lane] = m_run[qt];
    ml[(((wa * 2 + wc) * C::QT + qt) * 2 + 1) * 64 + lane] = l_tot[qt];
  }
  __syncthreads();
  float f_mine[C::QT], m_all[C::QT], l_all[C::QT];
#pragma unroll
  for (int qt = 0; qt < C::QT; ++qt) {
    const float m_o = ml[(((wa * 2 + (wc ^ 1)) * C::QT + qt) * 2 + 0) * 64 + lane];
    const float l_o = ml[(((wa * 2 + (wc ^ 1)) * C::QT + qt) * 2 + 1) * 64 + lane];
    const float m = fmaxf(m_run[qt], m_o);
    const float m_ref = (m == -INFINITY) ? 0.f : m;
    const float w_mine = __builtin_amdgcn_exp2f(m_run[qt] - m_ref), w_o = __builtin_amdgcn_exp2f(m_o - m_ref);
    m_all[qt] = m;
    l_all[qt] = l_tot[qt] * w_mine + l_o * w_o;
    f_mine[qt] = l_all[qt] > 0.f ? w_mine / l_all[qt] : 0.f;   // a row with no kept key yields zeros
  }
  // The c=1 wavefront of each query half hands its scaled partial output to the c=0 one through
  // the (now idle) K ring, in 8 KiB units of one (wa, dt) each.
  constexpr int XU_FLOATS = C::QT * 16 * 64;
  constexpr int UPB = C::UNIT_BYTES / (XU_FLOATS * 4);    // exchange units per ring slot
  static_assert(UPB >= 1 && (BLK / 64) * C::DT <= 4 * UPB, "exchange area must fit the K ring");
  auto xunit = [&](int dt) -> float* {
    const int u = wa * C::DT + dt, b = u / UPB;
    unsigned char* base = b == 0 ? K0 : b == 1 ? K1 : b == 2 ? K2 : K3;
    return reinterpret_cast<float*>(base) + (u % UPB) * XU_FLOATS;
  };
  if (wc == 1) {
#pragma unroll
    for (int dt = 0; dt < C::DT; ++dt)
#pragma unroll
      for (int qt = 0; qt < C::QT; ++qt)
#pragma unroll
        for (int i = 0; i < 16; ++i) xunit(dt)[(qt * 16 + i) * 64 + lane] = o[dt][qt][i] * f_mine[qt];
  }
  __syncthreads();
  if (wc == 0) {
#pragma unroll
    for (int qt = 0; qt < C::QT; ++qt) {
      const size_t row = (size_t)qi * BLK + 64 * wa + 32 * qt + l32;
      __bf16* orow = op + head_off + row * D;
#pragma unroll
      for (int dt = 0; dt < C::DT; ++dt)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          bf16x4 pk;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int i = 4 * g + e;
            const float other = xunit(dt)[(qt * 16 + i) * 64 + lane];
            pk[e] = (__bf16)(o[dt][qt][i] * f_mine[qt] + other);
          }
          *reinterpret_cast<bf16x4*>(orow + 32 * dt + 8 * g + 4 * lh) = pk;
        }
      if (lse != nullptr && lh == 0)
        lse[(size_t)bh * Tb * BLK + row] = m_all[qt] * 0.6931471805599453f + __logf(l_all[qt]);
    }
  }
}

template <int D, int BLK>
int launch_attn(const rf2_plan* plan, const void* qp, const void* kp, const void* vp, const int32_t* blk_idx,
                const int32_t* blk_cnt, void* op, float* lse, hipStream_t st) {
  using C = AttnCfg<D, BLK>;
  const rf2_config& c = plan->cfg;
  const rf2_info& in = plan->info;
  auto kern = block_sparse_attn_kernel<D, BLK>;
  const float scale_log2 = (float)(1.4426950408889634 / sqrt((double)D));
  const unsigned grid = 8u * (unsigned)plan->rows_per_xcd * (unsigned)(c.batch * c.heads);
  kern<<<dim3(grid), dim3(C::NT), 0, st>>>((const __bf16*)qp, (const __bf16*)kp, (const __bf16*)vp, blk_idx,
                                                     blk_cnt, (__bf16*)op, lse, plan->d_row_order, plan->rows_per_xcd,
                                                     in.n_blocks, in.k_row, in.last_block_valid, scale_log2);
  RF2_LAUNCH_CHECK();
  return RF2_OK;
}

}  // namespace

extern "C" int rf2_block_sparse_attn(const rf2_plan* plan, const void* qp, const void* kp, const void* vp,
                                     const int32_t* blk_idx, const int32_t* blk_cnt, void* op, float* lse,
                                     void* stream) {
  if (!plan || !qp || !kp || !vp || !blk_idx || !blk_cnt || !op) return RF2_ERR_INVALID_ARG;
  if (plan->device < 0) { rf2_note_hip_error(hipErrorNoDevice); return RF2_ERR_HIP; }
  const rf2_config& c = plan->cfg;
  hipStream_t st = (hipStream_t)stream;
  if (c.head_dim == 128 && c.block == 128) return launch_attn<128, 128>(plan, qp, kp, vp, blk_idx, blk_cnt, op, lse, st);
  if (c.head_dim == 64 && c.block == 64) return launch_attn<64, 64>(plan, qp, kp, vp, blk_idx, blk_cnt, op, lse, st);
  if (c.head_dim == 128 && c.block == 64) return launch_attn<128, 64>(plan, qp, kp, vp, blk_idx, blk_cnt, op, lse, st);
  if (c.head_dim == 64 && c.block == 128) return launch_attn<64, 128>(plan, qp, kp, vp, blk_idx, blk_cnt, op, lse, st);
  return RF2_ERR_UNSUPPORTED;
}
