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
  static constexpr int KT = KH / 32;            // 32-key tiles per wavefront
  static constexpr int QT = 2;                  // 32-query tiles per wavefront
  static constexpr int DS = D / 16;             // k-steps of the first product
  static constexpr int DT = D / 32;             // 32-channel tiles of the output
  static constexpr int KS = KH / 16;            // k-steps of the second product
  static constexpr int TILE_BYTES = BLK * D * 2;
  static constexpr int DMA = TILE_BYTES / 1024 / NW;   // 1 KiB direct-to-LDS loads per wavefront per tile
};

// K and V^T blocks are stored in global memory as operand tiles (see rf2.h): chunk-major
// [chunk][row][8 bf16], TILE_BYTES contiguous.  A tile goes straight from global memory
// into LDS, unchanged: each wavefront-wide load deposits 64 x 16 B at consecutive LDS
// addresses, wavefront w taking KiB u*NW + w of the tile for u = 0..NDMA-1.  In LDS the
// 16 lanes of a quarter-wave then read the same chunk of 16 consecutive rows = 256
// contiguous bytes (no bank conflicts), and all reads of a product share one per-lane
// base address plus compile-time offsets.
template <int NW, int NDMA>
__device__ __forceinline__ void dma_tile(unsigned char* lds_tile, const unsigned char* gtile, int wave, uint32_t tid16) {
#pragma unroll
  for (int u = 0; u < NDMA; ++u) {
    __builtin_amdgcn_global_load_lds(
        (const __attribute__((address_space(1))) void*)(gtile + u * (NW * 1024) + tid16),
        (__attribute__((address_space(3))) void*)(lds_tile + (u * NW + wave) * 1024), 16, 0, 0);
  }
}

template <int D, int BLK>
__global__ void __launch_bounds__(BLK * 2) block_sparse_attn_kernel(
    const __bf16* __restrict__ qp, const __bf16* __restrict__ kp, const __bf16* __restrict__ vp,
    const int32_t* __restrict__ blk_idx, const int32_t* __restrict__ blk_cnt, __bf16* __restrict__ op,
    float* __restrict__ lse, const int32_t* __restrict__ row_order, int rows_per_xcd, int Tb, int k_row,
    int last_valid, float scale_log2) {
  using C = AttnCfg<D, BLK>;
  // Two K and two V^T buffers.  They are separate objects on purpose: the compiler then
  // knows that a direct-to-LDS load into one buffer does not alias reads of another and
  // does not wait for it.
  __shared__ __attribute__((aligned(1024))) unsigned char KsA[C::TILE_BYTES];
  __shared__ __attribute__((aligned(1024))) unsigned char KsB[C::TILE_BYTES];
  __shared__ __attribute__((aligned(1024))) unsigned char VsA[C::TILE_BYTES];
  __shared__ __attribute__((aligned(1024))) unsigned char VsB[C::TILE_BYTES];
  __shared__ float ml[(BLK / 64) * 2 * C::QT * 2 * 64];   // [wa][wc][qt][m|l][lane]

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

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wavefront-uniform, kept in a scalar register
  const uint32_t tid16 = (uint32_t)tid * 16u;
  const int wa = wave >> 1, wc = wave & 1;
  const int l32 = lane & 31, lh = lane >> 5;
  const size_t head_off = (size_t)bh * Tb * BLK * D;    // elements; same for qp, kp, vp, op
  const unsigned char* __restrict__ kbase = reinterpret_cast<const unsigned char*>(kp + head_off);
  const unsigned char* __restrict__ vbase = reinterpret_cast<const unsigned char*>(vp + head_off);
  const uint32_t k_lane = (uint32_t)((lh * BLK + wc * C::KH + l32) * 16);          // LDS byte offsets of this lane's
  const uint32_t v_lane = (uint32_t)(((2 * wc * C::KS + lh) * D + l32) * 16);      // first K / V^T operand chunk
  auto block_at = [&](int it) {
    const int j = dense ? it : list[it];
    return min(max(j, 0), Tb - 1);                      // a corrupt list can give wrong results, never a fault
  };

  if (cnt > 0) {
    const size_t off = (size_t)block_at(0) * C::TILE_BYTES;
    dma_tile<C::NW, C::DMA>(KsA, kbase + off, wave, tid16);
    dma_tile<C::NW, C::DMA>(VsA, vbase + off, wave, tid16);
  }

  // ---- Q fragments (B operand of S^T), resident for the whole kernel -----------------
  bf16x8 qf[C::QT][C::DS];
#pragma unroll
  for (int qt = 0; qt < C::QT; ++qt) {
    const __bf16* qrow = qp + head_off + ((size_t)qi * BLK + 64 * wa + 32 * qt + l32) * D + 8 * lh;
#pragma unroll
    for (int s = 0; s < C::DS; ++s) qf[qt][s] = *reinterpret_cast<const bf16x8*>(qrow + 16 * s);
  }

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

  // One K/V block: wait for its tiles, start the loads of the next block into the other
  // buffers, then S^T, softmax, O^T.
  auto step = [&](const unsigned char* Kc, const unsigned char* Vc, unsigned char* Kn, unsigned char* Vn, int it) {
    const int j = block_at(it);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();     // tiles of block `it` are complete; nobody still reads the other buffers
    if (it + 1 < cnt) {
      const size_t off = (size_t)block_at(it + 1) * C::TILE_BYTES;
      dma_tile<C::NW, C::DMA>(Kn, kbase + off, wave, tid16);
      dma_tile<C::NW, C::DMA>(Vn, vbase + off, wave, tid16);
    }

    // ---- S^T = K Q^T (eq. 1, unscaled) ----------------------------------------------------
    f32x16 s[C::KT][C::QT];
#pragma unroll
    for (int kt = 0; kt < C::KT; ++kt) {
#pragma unroll
      for (int qt = 0; qt < C::QT; ++qt)
#pragma unroll
        for (int i = 0; i < 16; ++i) s[kt][qt][i] = 0.f;
#pragma unroll
      for (int ds = 0; ds < C::DS; ++ds) {
        // chunk 2*ds + lh of key row wc*KH + 32*kt + l32
        const bf16x8 a = *reinterpret_cast<const bf16x8*>(Kc + k_lane + (2 * ds * BLK + 32 * kt) * 16);
#pragma unroll
        for (int qt = 0; qt < C::QT; ++qt)
          s[kt][qt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[qt][ds], s[kt][qt], 0, 0, 0);
      }
    }
    // keys past the end of the sequence exist only in the last block
    if (j == Tb - 1 && last_valid < BLK) {
#pragma unroll
      for (int kt = 0; kt < C::KT; ++kt)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int key = wc * C::KH + 32 * kt + 8 * (i / 4) + 4 * lh + (i % 4);
          if (key >= last_valid) {
#pragma unroll
            for (int qt = 0; qt < C::QT; ++qt) s[kt][qt][i] = -INFINITY;
          }
        }
    }

    // ---- online softmax (eqs. 2, 3), one query column per lane ---------------------------
    // The running maximum is only raised when a block exceeds it by more than 2^8: until
    // then probabilities are at most 256 (exact final normalisation makes the reference
    // point irrelevant), and the 128-register output rescale is skipped for most blocks.
    bf16x8 pf[C::QT][C::KS];
#pragma unroll
    for (int qt = 0; qt < C::QT; ++qt) {
      float mx = -INFINITY;
#pragma unroll
      for (int kt = 0; kt < C::KT; ++kt)
#pragma unroll
        for (int i = 0; i < 16; ++i) mx = fmaxf(mx, s[kt][qt][i]);
      mx = fmaxf(mx, __shfl_xor(mx, 32)) * scale_log2;
      const bool raise = mx > m_run[qt] + 8.0f;           // -inf + 8 = -inf: the first finite block always raises
      if (__builtin_amdgcn_ballot_w64(raise) != 0ull) {
        const float m_new = raise ? mx : m_run[qt];
        const float alpha = raise ? __builtin_amdgcn_exp2f(m_run[qt] - m_new) : 1.0f;   // exp2(-inf) = 0
        m_run[qt] = m_new;
        l_run[qt] *= alpha;
#pragma unroll
        for (int dt = 0; dt < C::DT; ++dt)
#pragma unroll
          for (int i = 0; i < 16; ++i) o[dt][qt][i] *= alpha;
      }
      const float m_use = (m_run[qt] == -INFINITY) ? 0.f : m_run[qt];
      float rs = 0.f;
#pragma unroll
      for (int kt = 0; kt < C::KT; ++kt)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s[kt][qt][i], scale_log2, -m_use));
          s[kt][qt][i] = p;
          rs += p;
        }
      l_run[qt] += rs;
#pragma unroll
      for (int ks = 0; ks < C::KS; ++ks)
#pragma unroll
        for (int e = 0; e < 8; ++e) pf[qt][ks][e] = (__bf16)s[ks / 2][qt][8 * (ks % 2) + e];
    }

    // ---- O^T += V^T P^T (eq. 4) ---------------------------------------------------------
#pragma unroll
    for (int dt = 0; dt < C::DT; ++dt) {
#pragma unroll
      for (int ks = 0; ks < C::KS; ++ks) {
        // key chunk 2*(wc*KS + ks) + lh of channel row 32*dt + l32
        const bf16x8 a = *reinterpret_cast<const bf16x8*>(Vc + v_lane + (2 * ks * D + 32 * dt) * 16);
#pragma unroll
        for (int qt = 0; qt < C::QT; ++qt)
          o[dt][qt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf[qt][ks], o[dt][qt], 0, 0, 0);
      }
    }
  };

  for (int it = 0; it < cnt; it += 2) {
    step(KsA, VsA, KsB, VsB, it);
    if (it + 1 < cnt) step(KsB, VsB, KsA, VsA, it + 1);
  }

  // ---- merge the two key halves and write the Q block -------------------------------------
  __syncthreads();                                        // every wavefront is done with the tiles
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
    f_mine[qt] = w_mine / l_all[qt];
  }
  // The c=1 wavefront of each query half hands its scaled partial output to the c=0 one.
  // The exchange area is the (now idle) pair of K buffers, in 8 KiB units of one (wa, dt) each.
  constexpr int UNIT_FLOATS = C::QT * 16 * 64;
  constexpr int UPB = C::TILE_BYTES / (UNIT_FLOATS * 4);     // units per buffer
  static_assert(UPB >= 1 && (BLK / 64) * C::DT <= 2 * UPB, "exchange area must fit the two K buffers");
  auto unit = [&](int dt) -> float* {
    const int u = wa * C::DT + dt;
    return reinterpret_cast<float*>(u < UPB ? KsA : KsB) + (u % UPB) * UNIT_FLOATS;
  };
  if (wc == 1) {
#pragma unroll
    for (int dt = 0; dt < C::DT; ++dt)
#pragma unroll
      for (int qt = 0; qt < C::QT; ++qt)
#pragma unroll
        for (int i = 0; i < 16; ++i)
          unit(dt)[(qt * 16 + i) * 64 + lane] = o[dt][qt][i] * f_mine[qt];
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
            const float other = unit(dt)[(qt * 16 + i) * 64 + lane];
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
