// Block-sparse flash attention (Sec. 3.1, eqs. 1-4 with the block skip rule) for gfx950.
//
// One workgroup owns one Q block (b_q rows) of one (batch, head) and walks that row's list of
// kept K/V blocks (b_k rows each; b_q and b_k may differ).  Every wavefront owns 32 query rows
// and sees all keys, so there is nothing to merge at the end; a workgroup needs at most 80 KiB of
// LDS and 256 registers per lane, so two workgroups share a compute unit (two wavefronts per
// SIMD) and each hides the barriers, LDS latencies and vector-ALU phases of the other.
//
// Both products are computed transposed so that no register shuffling is needed between them
// (v_mfma_f32_32x32x16_bf16, D = A(32xk) * B(kx32) + C):
//   S^T[key][query]  = K (A, from LDS)  * Q^T (B, registers, loaded once)
//   O^T[chan][query] = V^T (A, from LDS) * P^T (B, registers = exp of the S^T accumulators)
// In the accumulator layout lane l holds query column l%32 and, per 32-key tile, keys
// 8*(i/4) + 4*(l/32) + i%4 for i = 0..15.  Eight consecutive accumulator values are exactly one
// B operand of the second product provided the A operand (V^T) lists the keys of each 16-key
// group in the order 0-3, 8-11, 4-7, 12-15 -- the order rf2_permute writes.  Row statistics are
// per lane (one query column) plus one exchange with lane l^32.
//
// Softmax (eqs. 2, 3) without a per-unit row maximum: a probability is exp2(fma(q.k, c, -m_ref c))
// with c = log2(e)/sqrt(d), the subtraction of eq. (2) riding on the multiply-add that applies the
// scale.  m_ref is set exactly from the first unit of the row and afterwards only moved when the row
// sum of a unit leaves the range fp32/bf16 carry without loss (> 2^40, or not finite); the final
// division by the row sum makes the reference point irrelevant.  The common path is one fused
// multiply-add, one exp2, one add and half a bf16 pack per probability.
//
// The loop is software-pipelined over "units" (one 32-key tile; a 64-key part of a K/V block is
// two units): step s issues the matrix products S_{s+1} and O += V P_{s-1} around the softmax
// arithmetic of unit s.  K and V^T parts stream from global memory straight into LDS rings (3 K
// parts, 2 V^T parts); the workgroup meets at one barrier per part (every second step).
#include "rf2_internal.h"

#include <type_traits>

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;

// BQ rows per Q block (one workgroup), BK rows per K/V block (Sec. 3.1: b_q and b_k).
template <int D, int BQ, int BK>
struct AttnCfg {
  static constexpr int NW = BQ / 32;            // wavefronts, 32 query rows each
  static constexpr int NT = NW * 64;
  static constexpr int KH = BK / 2;             // K block rows r and r + KH share a part (see rf2.h)
  static constexpr int PB = BK / 64;            // 64-key parts per K/V block
  static constexpr int UB = BK / 32;            // 32-key units per K/V block
  static constexpr int DS = D / 16;             // k-steps of the first product
  static constexpr int DT = D / 32;             // 32-channel tiles of the output
  static constexpr int TILE_BYTES = BK * D * 2;
  static constexpr int PART_BYTES = 64 * D * 2;
  static constexpr int LPW = PART_BYTES / 1024 / NW;   // 1 KiB direct-to-LDS loads per wavefront per part
  static constexpr int NK = 3, NV = 2;                 // ring depths in parts
  static_assert(LPW >= 1 && 2 * LPW < 63, "vmcnt range");
};

// rf2_permute stores every K and V^T block as PB contiguous parts in exactly the order the
// operand reads below walk them ([chunk][64 rows][8 bf16], see rf2.h), so a part is copied
// verbatim: each wavefront-wide load deposits 64 x 16 B at consecutive LDS addresses (M0 = LDS
// base of that KiB), wavefront w taking KiB u*NW + w for u = 0..LPW-1.  In LDS the 16 lanes of a
// quarter-wave read 16 consecutive 16-byte slots (no bank conflicts) and all reads of a product
// share one per-lane base address plus compile-time offsets.
// The load is written in assembly on purpose: the compiler then does not track it, and the only
// waits for it are the explicit vmcnt waits of ring_barrier below (its own bookkeeping of
// direct-to-LDS loads falls back to waiting for every outstanding load before unrelated LDS reads).
//
// The S^T product is issued through assembly so that its accumulators are ordinary vector
// registers that the softmax arithmetic reads in place.  The compiler does not know these
// statements are MFMAs, so what it would do for an MFMA is done by hand:
//  * between the last MFMA of a chain and the first vector-ALU read of its result lie the wait states
//    an 8-pass MFMA needs.  In the loop the chain ends in slot NQ-1 of a step and its accumulators are
//    first read in the following step, behind the NP matrix products of the remaining slots (their
//    order is frozen by the scheduling barriers), so nothing is added there; the chain of the
//    prologue is followed by code the compiler orders freely and ends in qk_last_wait, which carries
//    the wait states itself (18 >= the 12 needed);
//  * the first MFMA of a chain takes the constant 0 as its addend, so no register is read by the
//    matrix core after issue except the A and B operands;
//  * A and B operands are read at issue; they come from LDS reads and the resident Q fragments.
__device__ __forceinline__ void qk_first(f32x16& S, const bf16x8& a, const bf16x8& b) {
  asm("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(S) : "v"(a), "v"(b));
}
__device__ __forceinline__ void qk_next(f32x16& S, const bf16x8& a, const bf16x8& b) {
  asm("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(S) : "v"(a), "v"(b));
}
__device__ __forceinline__ void qk_last_wait(f32x16& S, const bf16x8& a, const bf16x8& b) {
  asm("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0\n\t"
      "s_nop 7\n\ts_nop 7\n\ts_nop 1"
      : "+v"(S)
      : "v"(a), "v"(b));
}

// Tells the compiler that a pointer is the same in every lane (it then lives in scalar registers).
__device__ __forceinline__ const unsigned char* uniform_ptr(const void* p) {
  const uint64_t v = (uint64_t)p;
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
  return (const unsigned char*)(((uint64_t)hi << 32) | lo);
}

// One wavefront-wide direct-to-LDS load: 64 x 16 B from g + voff (scalar base, per-lane 32-bit
// byte offset) to the KiB of LDS at `lds_kib`.
// M0 is written here and named as clobbered.  The compiler reserves M0 for itself (and says so with a
// warning, silenced below): it sets M0 immediately in front of each of its own uses (LDS-direct builtins,
// relative moves, message and GWS instructions), none of which this translation unit contains.
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void dma_one(uint32_t lds_kib, const unsigned char* g, uint32_t voff) {
  asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_kib), "v"(voff), "s"(g) : "memory", "m0");
}
#pragma clang diagnostic pop

// A whole part (LPW KiB per wavefront): wavefront w takes KiB u*NW + w for u = 0..LPW-1.
template <int NW, int LPW>
__device__ __forceinline__ void dma_part(unsigned char* lds, const unsigned char* g, int wave, uint32_t tid16) {
  const uint32_t lds_base = (uint32_t)(size_t)(__attribute__((address_space(3))) unsigned char*)lds;
  g = uniform_ptr(g);
#pragma unroll
  for (int u = 0; u < LPW; ++u) dma_one(lds_base + (uint32_t)((u * NW + wave) * 1024), g + u * (NW * 1024), tid16);
}

// Workgroup barrier of the loop: waits until at most N of this wavefront's direct-to-LDS loads
// are still in flight, then s_barrier.  __syncthreads() cannot be used there: its release fence
// would wait for ALL outstanding loads, i.e. also for the parts prefetched for later steps.  LDS
// operand reads have completed before the barrier because the MFMAs consuming them were issued;
// the asm memory clobbers keep the compiler from moving LDS accesses across.
template <int N>
__device__ __forceinline__ void ring_barrier() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

// (second launch bound: wavefronts per SIMD the register budget is sized for; a 64-row Q block has only
// two wavefronts per workgroup, which LDS limits to one per SIMD anyway; a 256-row Q block is one
// workgroup of eight wavefronts per compute unit)
template <int D, int BQ, int BK>
__global__ void __launch_bounds__(BQ * 2, BQ >= 128 ? 2 : 1) block_sparse_attn_kernel(
    const __bf16* __restrict__ qp, const __bf16* __restrict__ kp, const __bf16* __restrict__ vp,
    const int32_t* __restrict__ blk_idx, const int32_t* __restrict__ blk_cnt, __bf16* __restrict__ op,
    float* __restrict__ lse, const int32_t* __restrict__ row_order, int plain_per_xcd, int n_bh, int sink_row_begin,
    int n_sink_rows, int sink_slots,
    int Tq, int Tb, int k_row, int last_valid, float scale_log2, const int32_t* __restrict__ scatter, int n_tokens,
    int heads, rf2_strides st) {
  // Tq: Q blocks per head (rows of the block mask); Tb: K/V blocks per head (its columns); last_valid:
  // tokens in the last K/V block.
  using C = AttnCfg<D, BQ, BK>;
  // Part P lives in slot P % NK of the K ring (first) and slot P % NV of the V^T ring (behind it).
  __shared__ __attribute__((aligned(1024))) unsigned char ring[(C::NK + C::NV) * C::PART_BYTES];
  constexpr uint32_t VRING = C::NK * C::PART_BYTES;

  // ---- which Q block ---------------------------------------------------------------
  // Slots of an XCD, in issue order: the all-column sink rows of every head first, then the ordinary
  // rows head by head.  A sink row is several times longer than an ordinary one; issued first (longest
  // jobs first) none of them is left running alone at the end, and the short rows fill the tail evenly.
  // (workgroups with equal blockIdx % 8 share an XCD; which of the eight it is varies from launch to launch)
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  int bh, qi;
  if (slot < sink_slots) {
    // The sink rows of all heads, numbered head by head, are cut into 8 contiguous runs of sink_slots
    // rows, one per XCD: an XCD gets whole heads where it can (with 40 heads of 29 sink rows: five heads
    // each).  Rows of one head have the same list (every column) and the same length: side by side on
    // one XCD they run in step and find each other's tiles in its L2.
    const int g = xcd * sink_slots + slot;
    if (g >= n_bh * n_sink_rows) return;
    bh = g / n_sink_rows;
    qi = sink_row_begin + g % n_sink_rows;
  } else {
    // The work table deals a head's ordinary rows to 8 shares of slightly different size (contiguous
    // ranges); the share an XCD takes rotates with the head so that no XCD collects the large shares of
    // every head.
    const int t = slot - sink_slots;
    bh = t / plain_per_xcd;
    qi = row_order[((xcd + bh) & 7) * plain_per_xcd + t % plain_per_xcd];
    if (qi < 0) return;
  }
  const size_t row_id = (size_t)bh * Tq + qi;
  int cnt = blk_cnt[row_id];
  const bool dense = (cnt == Tb);
  cnt = dense ? Tb : min(max(cnt, 0), k_row);
  const int32_t* __restrict__ list = blk_idx + row_id * k_row;
  const int U = cnt * C::UB;                            // 32-key units to process (even)
  const int NPARTS = cnt * C::PB;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wavefront-uniform, kept in a scalar register
  const uint32_t tid16 = (uint32_t)tid * 16u;
  const int l32 = lane & 31, lh = lane >> 5;
  const size_t q_head_off = (size_t)bh * Tq * BQ * D;   // elements; qp and op
  const size_t k_head_off = (size_t)bh * Tb * BK * D;   // kp and vp
  const unsigned char* const kbase = uniform_ptr(kp + k_head_off);
  const unsigned char* const vbase = uniform_ptr(vp + k_head_off);
  // LDS byte offsets of this lane's first operand chunk inside a K part / a V^T part, for the
  // first 32-key tile of the part; the second tile lies K_TILE / V_TILE bytes further.
  const uint32_t k_lane = (uint32_t)((lh * 64 + l32) * 16);
  const uint32_t v_lane = (uint32_t)((lh * D + l32) * 16);
  constexpr uint32_t K_TILE = 32 * 16, V_TILE = 4 * D * 16;
  // Part P of the walk is part P % PB of listed block P / PB (P clamped: loads past the end
  // re-fetch the last part into a free slot, which keeps the outstanding-load count uniform).
  // A list entry is read one odd step before it is needed (list_entry) and turned into an offset
  // only when it is used (part_off), so that no step waits for a scalar memory load.
  // (part numbers are never negative: unsigned division and remainder are a shift and a mask)
  auto list_entry = [&](int P) {
    const int it = (int)((unsigned)min(P, NPARTS - 1) / (unsigned)C::PB);
    return dense ? it : list[it];
  };
  auto part_off = [&](int entry, int P) {
    const int j = min(max(entry, 0), Tb - 1);            // a corrupt list can give wrong results, never a fault
    return (uint32_t)j * (uint32_t)C::TILE_BYTES + ((unsigned)min(P, NPARTS - 1) % (unsigned)C::PB) * (uint32_t)C::PART_BYTES;
  };
  auto part_at = [&](int P) { return (size_t)part_off(list_entry(P), P); };
  const uint32_t ring_lds = (uint32_t)(size_t)(__attribute__((address_space(3))) unsigned char*)ring;
  // Only the last listed block can be the ragged last block of the sequence (lists ascend).
  int partial_begin = U;
  if (U > 0 && last_valid < BK) {
    const int jl = dense ? cnt - 1 : list[cnt - 1];
    if (min(max(jl, 0), Tb - 1) == Tb - 1) partial_begin = (cnt - 1) * C::UB;
  }

  bf16x8 qf[C::DS];
  f32x16 o[C::DT];
#pragma unroll
  for (int dt = 0; dt < C::DT; ++dt)
#pragma unroll
    for (int i = 0; i < 16; ++i) o[dt][i] = 0.f;
  // Softmax reference m_ref (per query column, in units of the raw products q.k) and nmc = -m_ref * c,
  // the addend of the multiply-add in front of every exp2.  l_run lags one unit behind: rs_last, the
  // row sum of the latest unit, is still to be added.
  float m_ref = 0.f, nmc = 0.f, l_run = 0.f, rs_last = 0.f;

  // ---- building blocks ------------------------------------------------------------------
  // One step has NQ + NP "slots" of one MFMA each: slots 0..NQ-1 are the k-steps of
  // S^T_{s+1} = K Q^T (eq. 1, unscaled), slots NQ.. are the (channel tile, k-step) pairs of
  // O^T += V^T P^T_{s-1} (eq. 4).
  constexpr int NQ = C::DS, NP = C::DT * 2, NSLOT = NQ + NP;
  constexpr int PD = 4;                                  // operand reads run this many slots ahead
  constexpr int SPP = NSLOT / 8;                         // slots per pair of probabilities (8 pairs per unit)
  static_assert(NSLOT % 8 == 0 && NQ >= 2 && 2 * C::LPW <= NSLOT, "slot plan");
  auto k_operand = [&](uint32_t k_addr, int c) -> bf16x8 {        // chunk 2c+lh of the tile
    return *reinterpret_cast<const bf16x8*>(ring + k_addr + c * 2048);
  };
  auto v_operand = [&](uint32_t v_addr, int dt, int ks) -> bf16x8 {   // key chunk 2ks+lh, channel 32dt+l32
    return *reinterpret_cast<const bf16x8*>(ring + v_addr + (2 * ks * D + 32 * dt) * 16);
  };
  auto operand = [&](uint32_t k_addr, uint32_t v_addr, int g) -> bf16x8 {
    return g < NQ ? k_operand(k_addr, g) : v_operand(v_addr, (g - NQ) / 2, (g - NQ) % 2);
  };
  // largest accumulator of one unit per query column (both lane halves end up with the same value)
  auto rowmax = [&](const f32x16& S) -> float {
    float v = S[0];
#pragma unroll
    for (int i = 1; i < 16; ++i) v = fmaxf(v, S[i]);
    // exchange with lane l^32 on the vector ALU (an LDS shuffle would wait for operand reads in flight)
    const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
  };
  // Moves the reference by delta (per query column): everything accumulated so far is rescaled
  // (eqs. 3, 4).  The accumulators hold raw products, so nothing else changes.
  auto move_reference = [&](float delta) {
    // (the very first move may go down; nothing has been accumulated then, any finite factor will do)
    const float alpha = __builtin_amdgcn_exp2f(-fmaxf(delta, 0.f) * scale_log2);
    m_ref += delta;
    nmc = -m_ref * scale_log2;
    l_run *= alpha;
#pragma unroll
    for (int dt = 0; dt < C::DT; ++dt)
#pragma unroll
      for (int i = 0; i < 16; ++i) o[dt][i] *= alpha;
  };
  // The probabilities P of the unit whose accumulators are in S were out of range; O holds all
  // earlier units, so the reference moves up and P (and rs_last) are recomputed.
  auto redo_unit = [&](f32x16& S, bf16x8 (&P)[2]) {
    const float mx = rowmax(S);
    move_reference(mx > m_ref ? mx - m_ref : 0.f);
    rs_last = 0.f;
#pragma unroll
    for (int i = 0; i < 16; i += 2) {
      const float p0 = __builtin_amdgcn_exp2f(fmaf(S[i], scale_log2, nmc));
      const float p1 = __builtin_amdgcn_exp2f(fmaf(S[i + 1], scale_log2, nmc));
      const bf16x2 pk = {(__bf16)p0, (__bf16)p1};
      rs_last += p0 + p1;
      P[i / 8][i % 8] = pk[0];
      P[i / 8][i % 8 + 1] = pk[1];
    }
  };
  // Rare work before the step of unit s: redo of unit s-1 (its accumulators are still in Sprev, the
  // buffer this step overwrites), the first unit (sets the reference exactly), and the units of the
  // ragged last block (keys past the end of the sequence are masked here).
  auto pre_step = [&](f32x16& S, f32x16& Sprev, bf16x8 (&Pprev)[2], uint32_t v_addr, int s, bool redo) {
    if (redo) redo_unit(Sprev, Pprev);
    if (s == 0 || s >= partial_begin) {
      // the pending product V P_{s-1} must reach O before O is rescaled; it is then neutralised
#pragma unroll
      for (int j = 0; j < NP; ++j) {
        const int dt = j % C::DT, ks = j / C::DT;
        o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(v_operand(v_addr, dt, ks), Pprev[ks], o[dt], 0, 0, 0);
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
      }
      const float mx = rowmax(S);
      // first unit: exact reference (it has at least one valid key); later: only upwards
      const bool move = (s == 0) ? true : (mx > m_ref);
      if (__builtin_amdgcn_ballot_w64(move) != 0ull) {
        l_run += rs_last;                                  // unit s-1 is in O now: rescale it with the rest
        rs_last = 0.f;
        move_reference(move ? mx - m_ref : 0.f);
      }
    }
  };

  int entry_k = 0, entry_v = 0;       // list entries of the parts loaded by the next odd step
  bool slow = true, redo = false;     // pre_step is needed for the coming unit / the latest unit must be redone
  // Step s (unit s = tile s%2 of part s/2): products S_{s+1} and V P_{s-1} around the softmax
  // arithmetic of unit s, in NSLOT slots of {operand read PD slots ahead, one MFMA, part of the
  // softmax arithmetic, one direct-to-LDS load}.  Odd steps s = 2P+1 start with the barrier and
  // issue the loads of V^T part P+NV-1 (into the slot of part P-1) and K part P+NK (into the slot of
  // part P); the V^T part is needed at the next barrier and goes first, the K loads may stay in
  // flight across it.
  auto step = [&](auto odd_tag, int s, int kslot, int vslot, int kfree, int vfree, f32x16& Scur, f32x16& Snext,
                  bf16x8 (&Pprev)[2], bf16x8 (&Pcur)[2]) {
    constexpr bool ODD = decltype(odd_tag)::value;
    if constexpr (ODD) ring_barrier<C::LPW>();
    // Through the step that issues a part's loads a wavefront takes precedence over the other wavefront
    // of its SIMD (which belongs to the other workgroup of the compute unit and is, as a rule, in an even
    // step): its loads leave earlier.  Measured +0.6 ... +1.1 % on 128- and 256-row Q blocks; a 64-row Q
    // block has its SIMD to itself (-0.2 %).
    constexpr bool PRIO = ODD && BQ >= 128;
    if constexpr (PRIO) __builtin_amdgcn_s_setprio(2);
    // unit s+1 and unit s-1 are both tile (s+1)%2 of their parts
    const uint32_t k_addr = (uint32_t)(kslot * C::PART_BYTES) + (ODD ? 0u : K_TILE) + k_lane;
    const uint32_t v_addr = VRING + (uint32_t)(vslot * C::PART_BYTES) + (ODD ? 0u : V_TILE) + v_lane;
    if (slow) pre_step(Scur, Snext, Pprev, v_addr, s, redo);
    l_run += rs_last;
    uint32_t k_dst = 0, v_dst = 0, k_voff = 0, v_voff = 0;
    if constexpr (ODD) {
      const int P = s >> 1;
      k_dst = ring_lds + (uint32_t)(kfree * C::PART_BYTES + wave * 1024);
      v_dst = ring_lds + VRING + (uint32_t)(vfree * C::PART_BYTES + wave * 1024);
      k_voff = tid16 + part_off(entry_k, P + C::NK);
      v_voff = tid16 + part_off(entry_v, P + C::NV - 1);
    }
    // the entries fetched by the previous odd step are consumed before the next fetches are issued:
    // scalar loads return out of order, so a wait for the old ones would also wait for new ones
    __builtin_amdgcn_sched_barrier(0);
    float rs = 0.f, e0 = 0.f, e1 = 0.f;
    bf16x8 opnd[NSLOT];
#pragma unroll
    for (int g = 0; g < PD; ++g) opnd[g] = operand(k_addr, v_addr, g);
    if constexpr (ODD) {
      const int P = s >> 1;
      entry_k = list_entry(P + 1 + C::NK);   // for the next odd step
      entry_v = list_entry(P + C::NV);
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int g = 0; g < NSLOT; ++g) {
      if (g + PD < NSLOT) opnd[g + PD] = operand(k_addr, v_addr, g + PD);
      if (g == 0) qk_first(Snext, opnd[g], qf[g]);
      else if (g < NQ) qk_next(Snext, opnd[g], qf[g]);
      else {
        const int dt = (g - NQ) / 2, ks = (g - NQ) % 2;
        o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(opnd[g], Pprev[ks], o[dt], 0, 0, 0);
      }
      if (g % SPP == 0) {
        // exponentials of pair g/SPP now, sum and bf16 packing of the previous pair (its exponentials
        // have long left the pipeline: no instruction here waits for the one before it)
        const int i = 2 * (g / SPP);
        if (i > 0) {
          const bf16x2 pk = {(__bf16)e0, (__bf16)e1};
          rs = (i == 2) ? e0 + e1 : rs + (e0 + e1);
          Pcur[(i - 2) / 8][(i - 2) % 8] = pk[0];
          Pcur[(i - 2) / 8][(i - 2) % 8 + 1] = pk[1];
        }
        e0 = __builtin_amdgcn_exp2f(fmaf(Scur[i], scale_log2, nmc));
        e1 = __builtin_amdgcn_exp2f(fmaf(Scur[i + 1], scale_log2, nmc));
        if (i == 14) {
          const bf16x2 pk = {(__bf16)e0, (__bf16)e1};
          rs += e0 + e1;
          Pcur[1][6] = pk[0];
          Pcur[1][7] = pk[1];
        }
      }
      if constexpr (ODD) {
        // at d = 128 the loads go into the slots of the second product (measured: +0.5 % over issuing them
        // from slot 0 on; at d = 64, where a step has half as many slots, -1.4 %), V^T first
        constexpr int G0 = (D == 128 && NQ + 2 * C::LPW <= NSLOT) ? NQ : 0;
        const int gl = g - G0;
        if (gl >= 0 && gl < C::LPW) dma_one(v_dst + gl * (C::NW * 1024), vbase + gl * (C::NW * 1024), v_voff);
        else if (gl >= C::LPW && gl < 2 * C::LPW)
          dma_one(k_dst + (gl - C::LPW) * (C::NW * 1024), kbase + (gl - C::LPW) * (C::NW * 1024), k_voff);
      }
      // Slots stay in this order: the operand reads keep their PD-slot lead over the MFMAs that
      // consume them (left alone, the scheduler packs each read right in front of its consumer).
      __builtin_amdgcn_sched_barrier(0);
    }
    // Keep the softmax arithmetic inside this block (its results are only consumed by the next
    // step, and the compiler would otherwise sink it there, out from under the MFMAs).
    asm volatile("" : "+v"(Pcur[0]), "+v"(Pcur[1]), "+v"(rs));
    if constexpr (PRIO) __builtin_amdgcn_s_setprio(0);
    rs_last = rs;
    redo = __builtin_amdgcn_ballot_w64(!(rs <= 1.0995e12f)) != 0ull;   // rare: above 2^40 or not finite
    slow = redo || (s + 1 >= partial_begin);
  };

  if (U > 0) {
    // ---- prologue: fill the rings, load Q, S of unit 0 -------------------------------------
    // (at raised priority: a row that starts has nothing to compute on until its first parts arrive; +0.3 %)
    __builtin_amdgcn_s_setprio(3);
#pragma unroll
    for (int P = 0; P < C::NK; ++P) dma_part<C::NW, C::LPW>(ring + P * C::PART_BYTES, kbase + part_at(P), wave, tid16);
#pragma unroll
    for (int P = 0; P < C::NV - 1; ++P)
      dma_part<C::NW, C::LPW>(ring + VRING + P * C::PART_BYTES, vbase + part_at(P), wave, tid16);
    // the slot of "part -1" (read by step 0 with zero probabilities) gets finite data
    dma_part<C::NW, C::LPW>(ring + VRING + (C::NV - 1) * C::PART_BYTES, vbase + part_at(0), wave, tid16);
    {
      const __bf16* qrow = qp + q_head_off + ((size_t)qi * BQ + 32 * wave + l32) * D + 8 * lh;
#pragma unroll
      for (int ds = 0; ds < C::DS; ++ds) qf[ds] = *reinterpret_cast<const bf16x8*>(qrow + 16 * ds);
    }
    f32x16 Sa, Sb;
    bf16x8 Pa[2], Pb[2];
    ring_barrier<0>();
#pragma unroll
    for (int ds = 0; ds < C::DS; ++ds) {
      const bf16x8 a = k_operand(k_lane, ds);
      if (ds == 0) qk_first(Sa, a, qf[ds]);
      else if (ds < C::DS - 1) qk_next(Sa, a, qf[ds]);
      else qk_last_wait(Sa, a, qf[ds]);
    }
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
#pragma unroll
      for (int e = 0; e < 8; ++e) Pb[ks][e] = (__bf16)0.f;   // "P_{-1}": step 0 adds V * 0
#pragma unroll
    for (int i = 0; i < 16; ++i) Sb[i] = 0.f;
    entry_k = list_entry(C::NK);
    entry_v = list_entry(C::NV - 1);

    __builtin_amdgcn_s_setprio(0);
    // ---- steady state: two steps per part ---------------------------------------------------
    int k0 = 0, k1 = 1;                                   // K ring slots of parts P and P+1
    int vm = C::NV - 1, vc = 0;                           // V^T ring slots of parts P-1 and P
    for (int s = 0; s < U; s += 2) {
      // even step: S of unit s+1 (part P, tile 1), V P of unit s-1 (part P-1, tile 1)
      step(std::false_type{}, s, k0, vm, 0, 0, Sa, Sb, Pb, Pa);
      // odd step: S of unit s+2 (part P+1, tile 0), V P of unit s (part P, tile 0)
      step(std::true_type{}, s + 1, k1, vc, k0, vm, Sb, Sa, Pa, Pb);
      k0 = k1;
      k1 = (k1 == C::NK - 1) ? 0 : k1 + 1;
      vm = vc;
      vc = (vc == C::NV - 1) ? 0 : vc + 1;
    }
    // ---- last product: O += V P_{U-1} (tile 1 of the last part; P_{U-1} is in Pb) ---------------
    ring_barrier<0>();
    if (redo) redo_unit(Sb, Pb);
    l_run += rs_last;
    {
      const uint32_t v_addr = VRING + (uint32_t)(vm * C::PART_BYTES) + V_TILE + v_lane;
#pragma unroll
      for (int j = 0; j < NP; ++j) {
        const int dt = j % C::DT, ks = j / C::DT;
        o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(v_operand(v_addr, dt, ks), Pb[ks], o[dt], 0, 0, 0);
      }
    }
  }

  // ---- normalise (the final division of eq. 4) and write the 32 rows of this wavefront ----------
  const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(l_run), __float_as_uint(l_run), false, false);
  const float l_tot = __uint_as_float(sw[0]) + __uint_as_float(sw[1]);
  const float f = l_tot > 0.f ? 1.0f / l_tot : 0.f;      // a row with no kept key yields zeros
  const size_t row = (size_t)qi * BQ + 32 * wave + l32;
  // plain output: row `row` of the permuted layout; fused inverse permutation: the token's raster row
  const int target = scatter ? scatter[row] : (int)row;
  if (target < 0) return;                                 // padding row of the last block
  __bf16* orow = scatter ? op + ((bh / heads) * st.batch + (bh % heads) * st.head + (long long)target * st.token) * D
                         : op + q_head_off + row * D;
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
    lse[scatter ? (size_t)bh * n_tokens + target : (size_t)bh * Tq * BQ + row] =
        m_ref * scale_log2 * 0.6931471805599453f + __logf(l_tot);
}

template <int D, int BQ, int BK>
int launch_attn(const rf2_plan* plan, const void* qp, const void* kp, const void* vp, const int32_t* blk_idx,
                const int32_t* blk_cnt, void* op, float* lse, bool scatter, hipStream_t st) {
  using C = AttnCfg<D, BQ, BK>;
  const rf2_config& c = plan->cfg;
  const rf2_info& in = plan->info;
  const float scale_log2 = (float)(1.4426950408889634 / sqrt((double)D));
  const int n_bh = c.batch * c.heads;
  // slots of an XCD: its run of the sink rows of all heads, then plain_per_xcd ordinary rows of every head
  const int n_sink_rows = in.sink_block_end - in.sink_block_begin;
  const int sink_slots = (int)(((int64_t)n_bh * n_sink_rows + 7) / 8);
  const unsigned grid = 8u * ((unsigned)sink_slots + (unsigned)n_bh * (unsigned)plan->plain_per_xcd);
  if (grid == 0) return RF2_OK;
  block_sparse_attn_kernel<D, BQ, BK><<<dim3(grid), dim3(C::NT), 0, st>>>(
      (const __bf16*)qp, (const __bf16*)kp, (const __bf16*)vp, blk_idx, blk_cnt, (__bf16*)op, lse, plan->d_row_order,
      plan->plain_per_xcd, n_bh, in.sink_block_begin, n_sink_rows, sink_slots, in.n_blocks, in.n_blocks_k, in.k_row, in.last_block_valid_k,
      scale_log2, scatter ? plan->d_perm : nullptr, (int)in.N, c.heads, rf2_qkv_strides(plan));
  RF2_LAUNCH_CHECK();
  return RF2_OK;
}

template <int D>
int dispatch_blocks(const rf2_plan* plan, const void* qp, const void* kp, const void* vp, const int32_t* blk_idx,
                    const int32_t* blk_cnt, void* out, float* lse, bool scatter, hipStream_t st) {
  const int bq = plan->cfg.block, bk = plan->info.block_k;
#define RF2_ATTN_CASE(Q, K) \
  if (bq == Q && bk == K) return launch_attn<D, Q, K>(plan, qp, kp, vp, blk_idx, blk_cnt, out, lse, scatter, st);
  RF2_ATTN_CASE(128, 128)
  RF2_ATTN_CASE(64, 64)
  RF2_ATTN_CASE(128, 64)
  RF2_ATTN_CASE(64, 128)
  RF2_ATTN_CASE(256, 128)
  RF2_ATTN_CASE(256, 64)
#undef RF2_ATTN_CASE
  return RF2_ERR_UNSUPPORTED;
}

int dispatch_attn(const rf2_plan* plan, const void* qp, const void* kp, const void* vp, const int32_t* blk_idx,
                  const int32_t* blk_cnt, void* out, float* lse, bool scatter, void* stream) {
  if (!plan || !qp || !kp || !vp || !blk_idx || !blk_cnt || !out) return RF2_ERR_INVALID_ARG;
  if (const int rc = rf2_check_device(plan)) return rc;
  hipStream_t st = (hipStream_t)stream;
  if (plan->cfg.head_dim == 128) return dispatch_blocks<128>(plan, qp, kp, vp, blk_idx, blk_cnt, out, lse, scatter, st);
  if (plan->cfg.head_dim == 64) return dispatch_blocks<64>(plan, qp, kp, vp, blk_idx, blk_cnt, out, lse, scatter, st);
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
