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

#include <type_traits>

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
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
// The S^T product is issued through assembly so that its accumulators are ordinary vector
// registers: the compiler's own MFMA selection keeps every accumulator of this kernel in
// the accumulation register file, from which the softmax arithmetic would need one copy
// instruction per element.  The compiler does not know these statements are MFMAs, so the
// wait states it would insert between the last MFMA of a chain and the first vector-ALU
// read of its result are part of qk_last (18 >= the 12 that an 8-pass MFMA needs here).
// Operands come from LDS reads and from the resident Q fragments, never from a preceding
// vector-ALU write, and the accumulator is not touched by anything else in between.
__device__ __forceinline__ void qk_first(f32x16& S, const bf16x8& a, const bf16x8& b) {
  asm("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(S) : "v"(a), "v"(b));
}
__device__ __forceinline__ void qk_next(f32x16& S, const bf16x8& a, const bf16x8& b) {
  asm("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(S) : "v"(a), "v"(b));
}
__device__ __forceinline__ void qk_last(f32x16& S0, f32x16& S1, const bf16x8& a, const bf16x8& b0, const bf16x8& b1) {
  asm("v_mfma_f32_32x32x16_bf16 %0, %2, %3, %0\n\tv_mfma_f32_32x32x16_bf16 %1, %2, %4, %1\n\t"
      "s_nop 7\n\ts_nop 7\n\ts_nop 1"
      : "+v"(S0), "+v"(S1)
      : "v"(a), "v"(b0), "v"(b1));
}

// Tells the compiler that a pointer is the same in every lane (it then lives in scalar registers).
__device__ __forceinline__ const unsigned char* uniform_ptr(const void* p) {
  const uint64_t v = (uint64_t)p;
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
  return (const unsigned char*)(((uint64_t)hi << 32) | lo);
}

// One wavefront-wide direct-to-LDS load: 64 x 16 B from g + voff (scalar base, per-lane 32-bit
// byte offset) to the KiB of LDS at `lds_kib`.
__device__ __forceinline__ void dma_one(uint32_t lds_kib, const unsigned char* g, uint32_t voff) {
  asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_kib), "v"(voff), "s"(g) : "memory");
}

// A whole unit part (LPW KiB per wavefront): wavefront w takes KiB u*NW + w for u = 0..LPW-1.
template <int NW, int LPW>
__device__ __forceinline__ void dma_unit(unsigned char* lds, const unsigned char* g, int wave, uint32_t tid16) {
  const uint32_t lds_base = (uint32_t)(size_t)(__attribute__((address_space(3))) unsigned char*)lds;
  g = uniform_ptr(g);
#pragma unroll
  for (int u = 0; u < LPW; ++u) dma_one(lds_base + (uint32_t)((u * NW + wave) * 1024), g + u * (NW * 1024), tid16);
}

__device__ __forceinline__ void wait_all_loads() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

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
    float* __restrict__ lse, const int32_t* __restrict__ row_order, int sink_per_xcd, int plain_per_xcd, int n_bh, int Tb, int k_row,
    int last_valid, float scale_log2, const int32_t* __restrict__ scatter, int n_tokens, int heads, rf2_strides st) {
  using C = AttnCfg<D, BLK>;
  // Rings of 4 K parts (slots 0-3) and 4 V^T parts (slots 4-7); unit x uses slot x % 4 of each.
  __shared__ __attribute__((aligned(1024))) unsigned char ring[8 * C::UNIT_BYTES];
  unsigned char* const kring = ring;
  unsigned char* const vring = ring + 4 * C::UNIT_BYTES;

  // ---- which Q block ---------------------------------------------------------------
  // Slots of an XCD, in issue order: the all-column sink rows are several times longer than
  // ordinary rows, so the sink rows of head h are issued LEAD heads ahead of its ordinary rows
  // (sink(0..LEAD-1), then sink(h+LEAD), plain(h) for each h, then the last plain rows): no long
  // row is left running alone at the end, while only a few heads' K/V are live at a time.
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int lead = min(2, n_bh), both = sink_per_xcd + plain_per_xcd;
  int bh, entry;
  if (slot < lead * sink_per_xcd) {
    bh = slot / sink_per_xcd;
    entry = slot % sink_per_xcd;
  } else {
    const int t = slot - lead * sink_per_xcd;
    if (t < (n_bh - lead) * both) {
      const int ph = t / both, r = t % both;
      bh = r < sink_per_xcd ? ph + lead : ph;
      entry = r;
    } else {
      const int u = t - (n_bh - lead) * both;
      bh = n_bh - lead + u / plain_per_xcd;
      entry = sink_per_xcd + u % plain_per_xcd;
    }
  }
  const int qi = row_order[xcd * (sink_per_xcd + plain_per_xcd) + entry];
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
  const unsigned char* const kbase = uniform_ptr(kp + head_off);
  const unsigned char* const vbase = uniform_ptr(vp + head_off);
  // LDS byte offsets of this lane's first operand chunk inside a K part / a V^T part
  const uint32_t k_lane = (uint32_t)((lh * 64 + wc * 32 + l32) * 16);
  const uint32_t v_lane = (uint32_t)(((wc * 4 + lh) * D + l32) * 16);
  auto block_at = [&](int it) {
    const int j = dense ? it : list[it];
    return min(max(j, 0), Tb - 1);                      // a corrupt list can give wrong results, never a fault
  };
  // Byte offset of unit x's part inside kp / vp of this head (x clamped: loads past the end
  // re-fetch the last unit into a free slot, which keeps the outstanding-load count uniform).
  // The list entry is read one step before it is needed (list_entry), and turned into an offset
  // only when it is used (part_off), so that no step waits for a scalar memory load.
  auto list_entry = [&](int x) {
    const int it = min(x, U - 1) / C::KT;
    return dense ? it : list[it];
  };
  auto part_off = [&](int entry, int x) {
    const int j = min(max(entry, 0), Tb - 1);            // a corrupt list can give wrong results, never a fault
    return (uint32_t)j * (uint32_t)C::TILE_BYTES + (uint32_t)(min(x, U - 1) % C::KT) * (uint32_t)C::UNIT_BYTES;
  };
  auto unit_off = [&](int x) { return (size_t)part_off(list_entry(x), x); };
  const uint32_t ring_lds = (uint32_t)(size_t)(__attribute__((address_space(3))) unsigned char*)ring;
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
  // One step has NQ + NP "slots" of two MFMAs each (one A operand from LDS, two query tiles):
  // slots 0..NQ-1 are the k-steps of S^T_{s+1} = K Q^T (eq. 1, unscaled), slots NQ.. are the
  // (channel tile, k-step) pairs of O^T += V^T P^T_{s-1} (eq. 4).
  constexpr int NQ = C::DS, NP = C::DT * 2, NSLOT = NQ + NP;
  constexpr int PD = 4;                                  // operand reads run this many slots ahead
  constexpr int EPS = 32 / NSLOT;                        // softmax elements handled per slot
  static_assert(32 % NSLOT == 0 && EPS % 2 == 0 && NQ >= 2 && 2 * C::LPW <= NSLOT, "slot plan");
  auto operand = [&](uint32_t k_addr, uint32_t v_addr, int g) -> bf16x8 {
    if (g < NQ) return *reinterpret_cast<const bf16x8*>(ring + k_addr + g * 2048);   // chunk 2g+lh, row wc*32+l32
    const int dt = (g - NQ) / 2, ks = (g - NQ) % 2;      // key chunk wc*4 + 2ks + lh, channel 32dt + l32
    return *reinterpret_cast<const bf16x8*>(ring + v_addr + (2 * ks * D + 32 * dt) * 16);
  };
  // scaled row maxima of one unit, per query column (both lane halves end up with the same value)
  auto rowmax = [&](const f32x16 (&S)[C::QT], float (&mx)[C::QT]) {
#pragma unroll
    for (int qt = 0; qt < C::QT; ++qt) {
      float v = S[qt][0];
#pragma unroll
      for (int i = 1; i < 16; ++i) v = fmaxf(v, S[qt][i]);
      // exchange with lane l^32 on the vector ALU (an LDS shuffle would wait for operand reads in flight)
      const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
      mx[qt] = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1])) * scale_log2;
    }
  };
  // The running maximum (eq. 2) is only raised when a unit exceeds it by more than 2^8: until
  // then probabilities are at most 256 (the exact final normalisation makes the reference point
  // irrelevant) and the 128-register output rescale of eqs. 3, 4 is skipped for most units.
  auto need_slow = [&](const float (&mx)[C::QT], int s) {
    bool raise = false;
#pragma unroll
    for (int qt = 0; qt < C::QT; ++qt) raise |= mx[qt] > m_run[qt] + 8.0f;   // -inf + 8 = -inf: first unit raises
    return (__builtin_amdgcn_ballot_w64(raise) != 0ull) || (s >= partial_begin);
  };
  // Rarely taken, before the step proper: the pending product V P_{s-1} must reach O before O
  // is rescaled (it is then neutralised); keys past the end of the sequence are masked here.
  auto slow_path = [&](f32x16 (&S)[C::QT], float (&mx)[C::QT], bf16x8 (&Pprev)[C::QT][2], uint32_t v_addr, int s) {
#pragma unroll
    for (int g = NQ; g < NSLOT; ++g) {
      const bf16x8 a = operand(0, v_addr, g);
      const int dt = (g - NQ) / 2, ks = (g - NQ) % 2;
#pragma unroll
      for (int qt = 0; qt < C::QT; ++qt)
        o[dt][qt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, Pprev[qt][ks], o[dt][qt], 0, 0, 0);
    }
#pragma unroll
    for (int qt = 0; qt < C::QT; ++qt)
#pragma unroll
      for (int ks = 0; ks < 2; ++ks)
#pragma unroll
        for (int e = 0; e < 8; ++e) Pprev[qt][ks][e] = (__bf16)0.f;
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
      const bool raise = mx[qt] > m_run[qt] + 8.0f;
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

  int entry_k = 0, entry_v = 0;                          // list entries of the units loaded by the next step
  bool slow = true;
  // Step s: products S_{s+1} and V P_{s-1} around the softmax arithmetic of unit s (eqs. 2, 3),
  // the loads of the K part of unit s+4 and the V^T part of unit s+2 spread between them, and
  // the row maxima of unit s+1 at the end.  Unit x lives in slot x % 4 of its ring.
  auto step = [&](int s, f32x16 (&Scur)[C::QT], f32x16 (&Snext)[C::QT], bf16x8 (&Pprev)[C::QT][2],
                  bf16x8 (&Pcur)[C::QT][2], float (&mxcur)[C::QT], float (&mxnext)[C::QT]) {
    ring_barrier<C::PENDING>();
    const uint32_t k_addr = (uint32_t)(((s + 1) & 3) * C::UNIT_BYTES) + k_lane;                        // K part of unit s+1
    const uint32_t v_addr = (uint32_t)((4 + ((s + 3) & 3)) * C::UNIT_BYTES) + v_lane;                  // V^T part of unit s-1
    if (slow) slow_path(Scur, mxcur, Pprev, v_addr, s);
    // direct-to-LDS loads of this step: K part of unit s+4 -> slot s % 4, V^T part of unit s+2 -> slot (s+2) % 4
    const uint32_t k_dst = ring_lds + (uint32_t)((s & 3) * C::UNIT_BYTES + wave * 1024);
    const uint32_t v_dst = ring_lds + (uint32_t)((4 + ((s + 2) & 3)) * C::UNIT_BYTES + wave * 1024);
    const uint32_t k_voff = tid16 + part_off(entry_k, s + 4);
    const uint32_t v_voff = tid16 + part_off(entry_v, s + 2);
    // the entries fetched by the previous step are consumed before the next fetches are issued:
    // scalar loads return out of order, so a wait for the old ones would also wait for new ones
    __builtin_amdgcn_sched_barrier(0);
    float m_use[C::QT], rs[C::QT];
#pragma unroll
    for (int qt = 0; qt < C::QT; ++qt) {
      m_use[qt] = (m_run[qt] == -INFINITY) ? 0.f : m_run[qt];
      rs[qt] = 0.f;
    }
    bf16x8 opnd[NSLOT];
#pragma unroll
    for (int g = 0; g < PD; ++g) opnd[g] = operand(k_addr, v_addr, g);
    entry_k = list_entry(s + 5);  // for the next step
    entry_v = list_entry(s + 3);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int g = 0; g < NSLOT; ++g) {
      if (g + PD < NSLOT) opnd[g + PD] = operand(k_addr, v_addr, g + PD);
      if (g == 0) {
        qk_first(Snext[0], opnd[g], qf[0][g]);
        qk_first(Snext[1], opnd[g], qf[1][g]);
      } else if (g < NQ - 1) {
        qk_next(Snext[0], opnd[g], qf[0][g]);
        qk_next(Snext[1], opnd[g], qf[1][g]);
      } else if (g == NQ - 1) {
        qk_last(Snext[0], Snext[1], opnd[g], qf[0][g], qf[1][g]);
      } else {
        const int dt = (g - NQ) / 2, ks = (g - NQ) % 2;
#pragma unroll
        for (int qt = 0; qt < C::QT; ++qt)
          o[dt][qt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(opnd[g], Pprev[qt][ks], o[dt][qt], 0, 0, 0);
      }
      // softmax arithmetic of unit s: EPS of the 32 values of this lane per slot
#pragma unroll
      for (int e = g * EPS; e < (g + 1) * EPS; e += 2) {
        const int qt = e / 16, i = e % 16;
        const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(Scur[qt][i], scale_log2, -m_use[qt]));
        const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(Scur[qt][i + 1], scale_log2, -m_use[qt]));
        const bf16x2 pk = {(__bf16)p0, (__bf16)p1};
        rs[qt] += p0 + p1;   // (a bf16 dot-product instruction would halve the adds, but it stalls the MFMA pipe)
        Pcur[qt][i / 8][i % 8] = pk[0];
        Pcur[qt][i / 8][i % 8 + 1] = pk[1];
      }
      // one direct-to-LDS load per slot until both parts are on their way
      if (g < C::LPW) dma_one(k_dst + g * (C::NW * 1024), kbase + g * (C::NW * 1024), k_voff);
      else if (g < 2 * C::LPW) dma_one(v_dst + (g - C::LPW) * (C::NW * 1024), vbase + (g - C::LPW) * (C::NW * 1024), v_voff);
      if (g == NQ + 1) rowmax(Snext, mxnext);            // S_{s+1} is complete since slot NQ-1
      // Slots stay in this order: the operand reads keep their PD-slot lead over the MFMAs that
      // consume them (left alone, the scheduler packs each read right in front of its consumer).
      __builtin_amdgcn_sched_barrier(0);
    }
    // Keep the softmax arithmetic inside this block (its results are only consumed by the next
    // step, and the compiler would otherwise sink it there, out from under the MFMAs).
#pragma unroll
    for (int qt = 0; qt < C::QT; ++qt) {
      asm volatile("" : "+v"(Pcur[qt][0]), "+v"(Pcur[qt][1]), "+v"(rs[qt]));
      l_run[qt] += rs[qt];
    }
    slow = need_slow(mxnext, s + 1);
  };

  if (U > 0) {
    // ---- prologue: fill the rings, load Q, S of unit 0 -------------------------------------
    dma_unit<C::NW, C::LPW>(kring + 0 * C::UNIT_BYTES, kbase + unit_off(0), wave, tid16);
    dma_unit<C::NW, C::LPW>(vring + 0 * C::UNIT_BYTES, vbase + unit_off(0), wave, tid16);
    dma_unit<C::NW, C::LPW>(kring + 1 * C::UNIT_BYTES, kbase + unit_off(1), wave, tid16);
    dma_unit<C::NW, C::LPW>(kring + 2 * C::UNIT_BYTES, kbase + unit_off(2), wave, tid16);
    dma_unit<C::NW, C::LPW>(kring + 3 * C::UNIT_BYTES, kbase + unit_off(3), wave, tid16);
    dma_unit<C::NW, C::LPW>(vring + 1 * C::UNIT_BYTES, vbase + unit_off(1), wave, tid16);
#pragma unroll
    for (int qt = 0; qt < C::QT; ++qt) {
      const __bf16* qrow = qp + head_off + ((size_t)qi * BLK + 64 * wa + 32 * qt + l32) * D + 8 * lh;
#pragma unroll
      for (int ds = 0; ds < C::DS; ++ds) qf[qt][ds] = *reinterpret_cast<const bf16x8*>(qrow + 16 * ds);
    }
    f32x16 Sa[C::QT], Sb[C::QT];
    bf16x8 Pa[C::QT][2], Pb[C::QT][2];
    float mxa[C::QT], mxb[C::QT];
    ring_barrier<0>();
#pragma unroll
    for (int ds = 0; ds < C::DS; ++ds) {
      const bf16x8 a = operand(k_lane, 0, ds);
      if (ds == 0) {
        qk_first(Sa[0], a, qf[0][ds]);
        qk_first(Sa[1], a, qf[1][ds]);
      } else if (ds < C::DS - 1) {
        qk_next(Sa[0], a, qf[0][ds]);
        qk_next(Sa[1], a, qf[1][ds]);
      } else {
        qk_last(Sa[0], Sa[1], a, qf[0][ds], qf[1][ds]);
      }
    }
#pragma unroll
    for (int qt = 0; qt < C::QT; ++qt)
#pragma unroll
      for (int ks = 0; ks < 2; ++ks)
#pragma unroll
        for (int e = 0; e < 8; ++e) Pb[qt][ks][e] = (__bf16)0.f;   // "P_{-1}": step 0 adds V_0 * 0
    rowmax(Sa, mxa);
    slow = true;                                         // the first unit always sets the maximum
    entry_k = list_entry(4);
    entry_v = list_entry(2);
    // step 0 reads "V part of unit -1" from slot 3 of the V ring, which nothing has filled yet:
    // point it at finite data (the product is multiplied by zero probabilities)
    dma_unit<C::NW, C::LPW>(vring + 3 * C::UNIT_BYTES, vbase + unit_off(0), wave, tid16);
    wait_all_loads();

    // ---- steady state ------------------------------------------------------------------------
    for (int s = 0; s < U; s += 2) {
      step(s, Sa, Sb, Pb, Pa, mxa, mxb);
      if (s + 1 < U) step(s + 1, Sb, Sa, Pa, Pb, mxb, mxa);
    }
    // ---- last product: O += V P_{U-1} ----------------------------------------------------------
    ring_barrier<0>();
    {
      const uint32_t v_addr = (uint32_t)((4 + ((U - 1) & 3)) * C::UNIT_BYTES) + v_lane;
      if ((U - 1) & 1) {
        float dummy[C::QT] = {};
        (void)dummy;
#pragma unroll
        for (int g = NQ; g < NSLOT; ++g) {
          const bf16x8 a = operand(0, v_addr, g);
          const int dt = (g - NQ) / 2, ks = (g - NQ) % 2;
#pragma unroll
          for (int qt = 0; qt < C::QT; ++qt)
            o[dt][qt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, Pb[qt][ks], o[dt][qt], 0, 0, 0);
        }
      } else {
#pragma unroll
        for (int g = NQ; g < NSLOT; ++g) {
          const bf16x8 a = operand(0, v_addr, g);
          const int dt = (g - NQ) / 2, ks = (g - NQ) % 2;
#pragma unroll
          for (int qt = 0; qt < C::QT; ++qt)
            o[dt][qt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, Pa[qt][ks], o[dt][qt], 0, 0, 0);
        }
      }
    }
  }

  // ---- merge the two key halves and write the Q block -------------------------------------
  __syncthreads();                                        // every wavefront is done with the rings
  float* ml = reinterpret_cast<float*>(vring);            // [wa][wc][qt][m|l][lane]: 4 KiB at most
  static_assert((BLK / 64) * 2 * C::QT * 2 * 64 * 4 <= C::UNIT_BYTES, "");
  float l_tot[C::QT];
#pragma unroll
  for (int qt = 0; qt < C::QT; ++qt) {
    const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(l_run[qt]), __float_as_uint(l_run[qt]), false, false);
    l_tot[qt] = __uint_as_float(sw[0]) + __uint_as_float(sw[1]);
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
  // the (now idle) K ring, 8 KiB per (wa, dt).
  constexpr int XU_FLOATS = C::QT * 16 * 64;
  static_assert((BLK / 64) * C::DT * XU_FLOATS * 4 <= 4 * C::UNIT_BYTES, "exchange area must fit the K ring");
  auto xunit = [&](int dt) -> float* { return reinterpret_cast<float*>(kring) + (wa * C::DT + dt) * XU_FLOATS; };
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
      // plain output: row `row` of the permuted layout; fused inverse permutation: the token's raster row
      const int target = scatter ? scatter[row] : (int)row;
      if (target < 0) continue;                              // padding row of the last block
      __bf16* orow = scatter ? op + ((bh / heads) * st.batch + (bh % heads) * st.head + (long long)target * st.token) * D
                             : op + head_off + row * D;
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
        lse[scatter ? (size_t)bh * n_tokens + target : (size_t)bh * Tb * BLK + row] =
            m_all[qt] * 0.6931471805599453f + __logf(l_all[qt]);
    }
  }
}


// ======================================================================================
// Variant X: 32 query rows per wavefront, every wavefront walks all keys, two workgroups
// per compute unit (two wavefronts per SIMD).
// ======================================================================================
#ifndef X_OCC
#define X_OCC 2
#endif
#ifndef X_PD
#define X_PD 4
#endif
#ifndef X_FREEZE
#define X_FREEZE 1
#endif
#ifndef X_NOSOFTMAX
#define X_NOSOFTMAX 0
#endif
#ifndef X_ORDER
#define X_ORDER 0
#endif
#ifndef X_NOLDS
#define X_NOLDS 0
#endif
#ifndef X_DMASAME
#define X_DMASAME 0
#endif
#ifndef X_PVASM
#define X_PVASM 0
#endif
#ifndef X_NODMA
#define X_NODMA 0
#endif
template <int D, int BLK>
struct XCfg {
  static constexpr int NW = BLK / 32;           // wavefronts, 32 query rows each
  static constexpr int NT = NW * 64;
  static constexpr int KH = BLK / 2;
  static constexpr int PB = BLK / 64;           // 64-key parts per block
  static constexpr int UB = BLK / 32;           // 32-key units per block
  static constexpr int DS = D / 16;
  static constexpr int DT = D / 32;
  static constexpr int TILE_BYTES = BLK * D * 2;
  static constexpr int PART_BYTES = 64 * D * 2;
  static constexpr int LPW = PART_BYTES / 1024 / NW;   // 1 KiB loads per wavefront per part
  static constexpr int NK = 3, NV = 2;                 // ring depths in parts
  static_assert(LPW >= 1 && 2 * LPW < 63, "vmcnt range");
};

// O^T += A * B with the accumulator tile held in the accumulation register file.
__device__ __forceinline__ void pv_acc(f32x16& O, const bf16x8& a, const bf16x8& b) {
#if X_PVASM
  asm("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(O) : "v"(a), "v"(b));
#else
  O = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, O, 0, 0, 0);
#endif
}
__device__ __forceinline__ void qk_last1(f32x16& S0, const bf16x8& a, const bf16x8& b0) {
  asm("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0\n\t"
      "s_nop 7\n\ts_nop 7\n\ts_nop 1"
      : "+v"(S0)
      : "v"(a), "v"(b0));
}

template <int D, int BLK>
__global__ void __launch_bounds__(BLK * 2, X_OCC) block_sparse_attn_kernel_x(
    const __bf16* __restrict__ qp, const __bf16* __restrict__ kp, const __bf16* __restrict__ vp,
    const int32_t* __restrict__ blk_idx, const int32_t* __restrict__ blk_cnt, __bf16* __restrict__ op,
    float* __restrict__ lse, const int32_t* __restrict__ row_order, int sink_per_xcd, int plain_per_xcd, int n_bh, int Tb, int k_row,
    int last_valid, float scale_log2, const int32_t* __restrict__ scatter, int n_tokens, int heads, rf2_strides st) {
  using C = XCfg<D, BLK>;
  __shared__ __attribute__((aligned(1024))) unsigned char ring[(C::NK + C::NV) * C::PART_BYTES];
  constexpr uint32_t VRING = C::NK * C::PART_BYTES;

  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int lead = min(2, n_bh), both = sink_per_xcd + plain_per_xcd;
  int bh, entry;
  if (slot < lead * sink_per_xcd) {
    bh = slot / sink_per_xcd;
    entry = slot % sink_per_xcd;
  } else {
    const int t = slot - lead * sink_per_xcd;
    if (t < (n_bh - lead) * both) {
      const int ph = t / both, r = t % both;
      bh = r < sink_per_xcd ? ph + lead : ph;
      entry = r;
    } else {
      const int u = t - (n_bh - lead) * both;
      bh = n_bh - lead + u / plain_per_xcd;
      entry = sink_per_xcd + u % plain_per_xcd;
    }
  }
  const int qi = row_order[xcd * (sink_per_xcd + plain_per_xcd) + entry];
  if (qi < 0) return;
  const size_t row_id = (size_t)bh * Tb + qi;
  int cnt = blk_cnt[row_id];
  const bool dense = (cnt == Tb);
  cnt = dense ? Tb : min(max(cnt, 0), k_row);
  const int32_t* __restrict__ list = blk_idx + row_id * k_row;
  const int U = cnt * C::UB;                            // 32-key units to process (even)
  const int NPARTS = cnt * C::PB;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const uint32_t tid16 = (uint32_t)tid * 16u;
  const int l32 = lane & 31, lh = lane >> 5;
  const size_t head_off = (size_t)bh * Tb * BLK * D;
  const unsigned char* const kbase = uniform_ptr(kp + head_off);
  const unsigned char* const vbase = uniform_ptr(vp + head_off);
  // LDS byte offsets of this lane's first operand chunk inside a K part / a V^T part (tile 0)
  const uint32_t k_lane = (uint32_t)((lh * 64 + l32) * 16);
  const uint32_t v_lane = (uint32_t)((lh * D + l32) * 16);
  constexpr uint32_t K_TILE = 32 * 16, V_TILE = 4 * D * 16;   // offset of tile 1 inside a part
  auto list_entry = [&](int P) {
    const int it = min(P, NPARTS - 1) / C::PB;
    return dense ? it : list[it];
  };
  auto part_off = [&](int entry, int P) {
    const int j = min(max(entry, 0), Tb - 1);            // a corrupt list can give wrong results, never a fault
    return (uint32_t)j * (uint32_t)C::TILE_BYTES + (uint32_t)(min(P, NPARTS - 1) % C::PB) * (uint32_t)C::PART_BYTES;
  };
  auto part_at = [&](int P) { return (size_t)part_off(list_entry(P), P); };
  const uint32_t ring_lds = (uint32_t)(size_t)(__attribute__((address_space(3))) unsigned char*)ring;
  int partial_begin = U;
  if (U > 0 && last_valid < BLK) {
    const int jl = dense ? cnt - 1 : list[cnt - 1];
    if (min(max(jl, 0), Tb - 1) == Tb - 1) partial_begin = (cnt - 1) * C::UB;
  }

  bf16x8 qf[C::DS];
  f32x16 o[C::DT];
#pragma unroll
  for (int dt = 0; dt < C::DT; ++dt)
#pragma unroll
    for (int i = 0; i < 16; ++i) o[dt][i] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;

  constexpr int NQ = C::DS, NP = C::DT * 2, NSLOT = NQ + NP;
  constexpr int PD = X_PD;
  constexpr int SPP = NSLOT / 8;                         // slots per softmax pair (8 pairs per unit)
  static_assert(NSLOT % 8 == 0 && NQ >= 2 && 2 * C::LPW <= NSLOT, "slot plan");
  // Slot g of a step is the QK k-step qk_of(g) (if >= 0) or the PV product (dt, ks) = pv_of(g).
  // X_ORDER 0: all QK slots, then PV slots pairwise per channel tile; 1: QK and PV alternate and
  // consecutive PV products go to different accumulators (no MFMA depends on its predecessor).
  auto qk_of = [](int g) { return X_ORDER ? ((g & 1) ? -1 : g / 2) : (g < NQ ? g : -1); };
  auto pv_dt = [](int g) { return X_ORDER ? (g / 2) % C::DT : (g - NQ) / 2; };
  auto pv_ks = [](int g) { return X_ORDER ? (g / 2) / C::DT : (g - NQ) % 2; };
  auto k_operand = [&](uint32_t k_addr, int c) -> bf16x8 {
    return *reinterpret_cast<const bf16x8*>(ring + k_addr + c * 2048);
  };
  auto v_operand = [&](uint32_t v_addr, int dt, int ks) -> bf16x8 {
    return *reinterpret_cast<const bf16x8*>(ring + v_addr + (2 * ks * D + 32 * dt) * 16);
  };
  auto operand = [&](uint32_t k_addr, uint32_t v_addr, int g) -> bf16x8 {
    return qk_of(g) >= 0 ? k_operand(k_addr, qk_of(g)) : v_operand(v_addr, pv_dt(g), pv_ks(g));
  };
  auto rowmax = [&](const f32x16& S) -> float {
    float v = S[0];
#pragma unroll
    for (int i = 1; i < 16; ++i) v = fmaxf(v, S[i]);
    const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1])) * scale_log2;
  };
  auto need_slow = [&](float mx, int s) {
    const bool raise = mx > m_run + 8.0f;
    return (__builtin_amdgcn_ballot_w64(raise) != 0ull) || (s >= partial_begin);
  };
  auto slow_path = [&](f32x16& S, float& mx, bf16x8 (&Pprev)[2], uint32_t v_addr, int s) {
#pragma unroll
    for (int j = 0; j < NP; ++j) {
      const int dt = j % C::DT, ks = j / C::DT;
      pv_acc(o[dt], v_operand(v_addr, dt, ks), Pprev[ks]);
    }
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
#pragma unroll
      for (int e = 0; e < 8; ++e) Pprev[ks][e] = (__bf16)0.f;
    if (s >= partial_begin) {
      const int t = s & 1, p = (s >> 1) % C::PB;
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int key = t * C::KH + 32 * p + 8 * (i / 4) + 4 * lh + (i % 4);
        if (key >= last_valid) S[i] = -INFINITY;
      }
      mx = rowmax(S);
    }
    const bool raise = mx > m_run + 8.0f;
    if (__builtin_amdgcn_ballot_w64(raise) != 0ull) {
      const float alpha = raise ? __builtin_amdgcn_exp2f(m_run - mx) : 1.0f;
      m_run = raise ? mx : m_run;
      l_run *= alpha;
#pragma unroll
      for (int dt = 0; dt < C::DT; ++dt)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[dt][i] *= alpha;
    }
  };

  int entry_k = 0, entry_v = 0;       // list entries of the parts loaded by the next odd step
  bool slow = true;
  // Step s (unit s = tile s%2 of part s/2): products S_{s+1} and V P_{s-1} around the softmax
  // arithmetic of unit s.  Part P lives in slot P % NK of the K ring and P % NV of the V ring.
  // Odd steps s = 2P+1 start with the barrier and issue the loads of V part P+1 and K part P+3.
  auto step = [&](auto odd_tag, int s, int kslot, int vslot, int kfree, int vfree, f32x16& Scur, f32x16& Snext,
                  bf16x8 (&Pprev)[2], bf16x8 (&Pcur)[2], float& mxcur, float& mxnext) {
    constexpr bool ODD = decltype(odd_tag)::value;
    if constexpr (ODD) ring_barrier<C::LPW>();
    // unit s+1 and unit s-1 are both tile (s+1)%2 = ODD ? 0 : 1
    const uint32_t k_addr = (uint32_t)(kslot * C::PART_BYTES) + (ODD ? 0u : K_TILE) + k_lane;
    const uint32_t v_addr = VRING + (uint32_t)(vslot * C::PART_BYTES) + (ODD ? 0u : V_TILE) + v_lane;
    if (slow) slow_path(Scur, mxcur, Pprev, v_addr, s);
    uint32_t k_dst = 0, v_dst = 0, k_voff = 0, v_voff = 0;
    if constexpr (ODD) {
      const int P = s >> 1;
      k_dst = ring_lds + (uint32_t)(kfree * C::PART_BYTES + wave * 1024);
      v_dst = ring_lds + VRING + (uint32_t)(vfree * C::PART_BYTES + wave * 1024);
      k_voff = tid16 + (X_DMASAME ? 0u : part_off(entry_k, P + 3));
      v_voff = tid16 + (X_DMASAME ? 0u : part_off(entry_v, P + 1));
    }
    __builtin_amdgcn_sched_barrier(0);
    const float m_use = (m_run == -INFINITY) ? 0.f : m_run;
    float rs = 0.f;
    bf16x8 opnd[NSLOT];
#pragma unroll
    for (int g = 0; g < PD; ++g) opnd[g] = operand(k_addr, v_addr, g);
    if constexpr (ODD) {
      const int P = s >> 1;
      entry_k = list_entry(P + 4);   // for the next odd step
      entry_v = list_entry(P + 2);
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int g = 0; g < NSLOT; ++g) {
      if (g + PD < NSLOT && !X_NOLDS) opnd[g + PD] = operand(k_addr, v_addr, g + PD);
      {
        const int c = qk_of(g);
        if (c == 0) qk_first(Snext, opnd[g], qf[0]);
        else if (c > 0 && c < NQ - 1) qk_next(Snext, opnd[g], qf[c]);
        else if (c == NQ - 1) qk_last1(Snext, opnd[g], qf[c]);
        else pv_acc(o[pv_dt(g)], opnd[g], Pprev[pv_ks(g)]);
      }
      if (g % SPP == 0 && !X_NOSOFTMAX) {
        const int i = 2 * (g / SPP);
        const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(Scur[i], scale_log2, -m_use));
        const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(Scur[i + 1], scale_log2, -m_use));
        const bf16x2 pk = {(__bf16)p0, (__bf16)p1};
        rs += p0 + p1;
        Pcur[i / 8][i % 8] = pk[0];
        Pcur[i / 8][i % 8 + 1] = pk[1];
      }
      if constexpr (ODD && !X_NODMA) {
        // V^T part first, K part second: the barrier of the next odd step then waits for all but the K loads
        if (g < C::LPW) dma_one(v_dst + g * (C::NW * 1024), vbase + g * (C::NW * 1024), v_voff);
        else if (g < 2 * C::LPW) dma_one(k_dst + (g - C::LPW) * (C::NW * 1024), kbase + (g - C::LPW) * (C::NW * 1024), k_voff);
      }
      if (!X_ORDER && g == NQ + 1) mxnext = rowmax(Snext);
      if (X_FREEZE) __builtin_amdgcn_sched_barrier(0);
    }
    if (X_ORDER) mxnext = rowmax(Snext);
    asm volatile("" : "+v"(Pcur[0]), "+v"(Pcur[1]), "+v"(rs));
    l_run += rs;
    slow = need_slow(mxnext, s + 1);
  };

  if (U > 0) {
    // ---- prologue: K parts 0..2, V^T part 0 (and a finite stand-in for "part -1"), Q, S of unit 0 ----
    dma_unit<C::NW, C::LPW>(ring + 0 * C::PART_BYTES, kbase + part_at(0), wave, tid16);
    dma_unit<C::NW, C::LPW>(ring + VRING + 0 * C::PART_BYTES, vbase + part_at(0), wave, tid16);
    dma_unit<C::NW, C::LPW>(ring + 1 * C::PART_BYTES, kbase + part_at(1), wave, tid16);
    dma_unit<C::NW, C::LPW>(ring + 2 * C::PART_BYTES, kbase + part_at(2), wave, tid16);
    dma_unit<C::NW, C::LPW>(ring + VRING + 1 * C::PART_BYTES, vbase + part_at(0), wave, tid16);
    {
      const __bf16* qrow = qp + head_off + ((size_t)qi * BLK + 32 * wave + l32) * D + 8 * lh;
#pragma unroll
      for (int ds = 0; ds < C::DS; ++ds) qf[ds] = *reinterpret_cast<const bf16x8*>(qrow + 16 * ds);
    }
    f32x16 Sa, Sb;
    bf16x8 Pa[2], Pb[2];
    float mxa, mxb = 0.f;
    ring_barrier<0>();
#pragma unroll
    for (int ds = 0; ds < C::DS; ++ds) {
      const bf16x8 a = k_operand(k_lane, ds);
      if (ds == 0) qk_first(Sa, a, qf[ds]);
      else if (ds < C::DS - 1) qk_next(Sa, a, qf[ds]);
      else qk_last1(Sa, a, qf[ds]);
    }
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
#pragma unroll
      for (int e = 0; e < 8; ++e) Pb[ks][e] = (__bf16)0.f;
    mxa = rowmax(Sa);
    slow = true;
    entry_k = list_entry(3);
    entry_v = list_entry(1);

    // ---- steady state: two steps per part ---------------------------------------------------
    int k0 = 0, k1 = 1;                                   // K ring slots of parts P and P+1
    for (int s = 0; s < U; s += 2) {
      const int P = s >> 1;
      // even step: S of unit s+1 (part P, tile 1), V P of unit s-1 (part P-1, tile 1)
      step(std::false_type{}, s, k0, (P + 1) & 1, 0, 0, Sa, Sb, Pb, Pa, mxa, mxb);
      // odd step: S of unit s+2 (part P+1, tile 0), V P of unit s (part P, tile 0);
      // loads K part P+3 into the slot of part P and V^T part P+1 into the slot of part P-1
      step(std::true_type{}, s + 1, k1, P & 1, k0, (P + 1) & 1, Sb, Sa, Pa, Pb, mxb, mxa);
      k0 = k1;
      k1 = (k1 == C::NK - 1) ? 0 : k1 + 1;
    }
    // ---- last product: O += V P_{U-1} (part U/2-1, tile 1; P_{U-1} is in Pb) ----------------------
    ring_barrier<0>();
    {
      const int P = (U >> 1) - 1;
      const uint32_t v_addr = VRING + (uint32_t)((P & 1) * C::PART_BYTES) + V_TILE + v_lane;
#pragma unroll
      for (int j = 0; j < NP; ++j) {
        const int dt = j % C::DT, ks = j / C::DT;
        pv_acc(o[dt], v_operand(v_addr, dt, ks), Pb[ks]);
      }
    }
  }

  // ---- normalise (eq. 4's final division) and write the 32 rows of this wavefront --------------
  const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(l_run), __float_as_uint(l_run), false, false);
  const float l_tot = __uint_as_float(sw[0]) + __uint_as_float(sw[1]);
  const float f = l_tot > 0.f ? 1.0f / l_tot : 0.f;      // a row with no kept key yields zeros
  const size_t row = (size_t)qi * BLK + 32 * wave + l32;
  const int target = scatter ? scatter[row] : (int)row;
  if (target < 0) return;                                 // padding row of the last block
  __bf16* orow = scatter ? op + ((bh / heads) * st.batch + (bh % heads) * st.head + (long long)target * st.token) * D
                         : op + head_off + row * D;
#pragma unroll
  for (int dt = 0; dt < C::DT; ++dt)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      bf16x4 pk;
#pragma unroll
      for (int e = 0; e < 4; ++e) pk[e] = (__bf16)(o[dt][4 * g + e] * f);
      *reinterpret_cast<bf16x4*>(orow + 32 * dt + 8 * g + 4 * lh) = pk;
    }
  if (lse != nullptr && lh == 0)
    lse[scatter ? (size_t)bh * n_tokens + target : (size_t)bh * Tb * BLK + row] =
        m_run * 0.6931471805599453f + __logf(l_tot);
}

template <int D, int BLK>
int launch_attn(const rf2_plan* plan, const void* qp, const void* kp, const void* vp, const int32_t* blk_idx,
                const int32_t* blk_cnt, void* op, float* lse, bool scatter, hipStream_t st) {
  using C = AttnCfg<D, BLK>;
  const rf2_config& c = plan->cfg;
  const rf2_info& in = plan->info;
#ifdef RF2_ATTN_X
  auto kern = block_sparse_attn_kernel_x<D, BLK>;
#else
  auto kern = block_sparse_attn_kernel<D, BLK>;
#endif
  const float scale_log2 = (float)(1.4426950408889634 / sqrt((double)D));
  const int n_bh = c.batch * c.heads;
  const unsigned grid = 8u * (unsigned)(plan->sink_per_xcd + plan->plain_per_xcd) * (unsigned)n_bh;
  kern<<<dim3(grid), dim3(C::NT), 0, st>>>((const __bf16*)qp, (const __bf16*)kp, (const __bf16*)vp, blk_idx,
                                                     blk_cnt, (__bf16*)op, lse, plan->d_row_order, plan->sink_per_xcd,
                                       plan->plain_per_xcd, n_bh,
                                                     in.n_blocks, in.k_row, in.last_block_valid, scale_log2,
                                                     scatter ? plan->d_perm : nullptr, (int)in.N, c.heads,
                                                     rf2_qkv_strides(plan));
  RF2_LAUNCH_CHECK();
  return RF2_OK;
}

int dispatch_attn(const rf2_plan* plan, const void* qp, const void* kp, const void* vp, const int32_t* blk_idx,
                  const int32_t* blk_cnt, void* out, float* lse, bool scatter, void* stream) {
  if (!plan || !qp || !kp || !vp || !blk_idx || !blk_cnt || !out) return RF2_ERR_INVALID_ARG;
  if (plan->device < 0) { rf2_note_hip_error(hipErrorNoDevice); return RF2_ERR_HIP; }
  const rf2_config& c = plan->cfg;
  hipStream_t st = (hipStream_t)stream;
  if (c.head_dim == 128 && c.block == 128) return launch_attn<128, 128>(plan, qp, kp, vp, blk_idx, blk_cnt, out, lse, scatter, st);
  if (c.head_dim == 64 && c.block == 64) return launch_attn<64, 64>(plan, qp, kp, vp, blk_idx, blk_cnt, out, lse, scatter, st);
  if (c.head_dim == 128 && c.block == 64) return launch_attn<128, 64>(plan, qp, kp, vp, blk_idx, blk_cnt, out, lse, scatter, st);
  if (c.head_dim == 64 && c.block == 128) return launch_attn<64, 128>(plan, qp, kp, vp, blk_idx, blk_cnt, out, lse, scatter, st);
  return RF2_ERR_UNSUPPORTED;
}

}  // namespace

extern "C" int rf2_block_sparse_attn(const rf2_plan* plan, const void* qp, const void* kp, const void* vp,
                                     const int32_t* blk_idx, const int32_t* blk_cnt, void* op, float* lse,
                                     void* stream) {
  return dispatch_attn(plan, qp, kp, vp, blk_idx, blk_cnt, op, lse, false, stream);
}

extern "C" int rf2_block_sparse_attn_unpermuted(const rf2_plan* plan, const void* qp, const void* kp, const void* vp,
                                                const int32_t* blk_idx, const int32_t* blk_cnt, void* o, float* lse,
                                                void* stream) {
  return dispatch_attn(plan, qp, kp, vp, blk_idx, blk_cnt, o, lse, true, stream);
}
