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

// LDS tiles hold rows of C 16-byte chunks; chunk c of row r is stored at chunk slot
// swz(r, c) so that the 16 lanes of a quarter-wave, which read the same logical chunk of
// 16 consecutive rows, hit 16 distinct slots of one 256-byte bank line.
template <int C>
__device__ __forceinline__ int swz(int row, int c) {
  if constexpr (C == 16) return c ^ (row & 15);
  else return c ^ ((row >> 1) & 7);
}

template <int D, int BLK>
struct AttnCfg {
  static constexpr int NT = BLK * 2;            // threads: (BLK/64 query halves) x (2 key halves) wavefronts
  static constexpr int KH = BLK / 2;            // keys per wavefront per block
  static constexpr int KT = KH / 32;            // 32-key tiles per wavefront
  static constexpr int QT = 2;                  // 32-query tiles per wavefront
  static constexpr int DS = D / 16;             // k-steps of the first product
  static constexpr int DT = D / 32;             // 32-channel tiles of the output
  static constexpr int KS = KH / 16;            // k-steps of the second product
  static constexpr int CHK = D / 8;             // 16-byte chunks per K row
  static constexpr int CHV = BLK / 8;           // 16-byte chunks per V^T row
  static constexpr int STAGE = (BLK * CHK) / NT;  // chunks per thread per tile (same for K and V^T)
  static constexpr int TILE_BYTES = BLK * D * 2;
  static constexpr int MERGE_BYTES = (BLK / 64) * DT * QT * 16 * 64 * 4;   // output partials of the c=1 wavefronts
  static constexpr int ML_FLOATS = (BLK / 64) * 2 * QT * 2 * 64;
  static constexpr int LDS_BYTES =
      (2 * TILE_BYTES > MERGE_BYTES ? 2 * TILE_BYTES : MERGE_BYTES) + ML_FLOATS * 4;
};

template <int D, int BLK>
__global__ void __launch_bounds__(BLK * 2) block_sparse_attn_kernel(
    const __bf16* __restrict__ qp, const __bf16* __restrict__ kp, const __bf16* __restrict__ vp,
    const int32_t* __restrict__ blk_idx, const int32_t* __restrict__ blk_cnt, __bf16* __restrict__ op,
    float* __restrict__ lse, const int32_t* __restrict__ row_order, int rows_per_xcd, int Tb, int k_row,
    int last_valid, float scale_log2) {
  using C = AttnCfg<D, BLK>;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  unsigned char* Ks = smem;
  unsigned char* Vs = smem + C::TILE_BYTES;

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

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wa = wave >> 1, wc = wave & 1;
  const int l32 = lane & 31, lh = lane >> 5;
  const size_t head_off = (size_t)bh * Tb * BLK * D;    // elements; same for qp, kp, vp, op
  const __bf16* __restrict__ kbase = kp + head_off;
  const __bf16* __restrict__ vbase = vp + head_off;

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

  // ---- tile staging through registers -------------------------------------------------
  uint4 stage[C::STAGE];
  auto load_tile = [&](const __bf16* tile) {           // a tile is TILE_BYTES contiguous bytes
    const uint4* src = reinterpret_cast<const uint4*>(tile);
#pragma unroll
    for (int u = 0; u < C::STAGE; ++u) stage[u] = src[tid + C::NT * u];
  };
  auto store_k = [&]() {
#pragma unroll
    for (int u = 0; u < C::STAGE; ++u) {
      const int id = tid + C::NT * u, row = id / C::CHK, c = id % C::CHK;
      *reinterpret_cast<uint4*>(Ks + row * (D * 2) + swz<C::CHK>(row, c) * 16) = stage[u];
    }
  };
  auto store_v = [&]() {
#pragma unroll
    for (int u = 0; u < C::STAGE; ++u) {
      const int id = tid + C::NT * u, row = id / C::CHV, c = id % C::CHV;
      *reinterpret_cast<uint4*>(Vs + row * (BLK * 2) + swz<C::CHV>(row, c) * 16) = stage[u];
    }
  };
  auto block_at = [&](int it) {
    const int j = dense ? it : list[it];
    return min(max(j, 0), Tb - 1);
  };

  if (cnt > 0) load_tile(kbase + (size_t)block_at(0) * BLK * D);
  for (int it = 0; it < cnt; ++it) {
    const int j = block_at(it);
    store_k();
    __syncthreads();
    load_tile(vbase + (size_t)j * BLK * D);

    // ---- S^T = K Q^T ------------------------------------------------------------------
    f32x16 s[C::KT][C::QT];
#pragma unroll
    for (int kt = 0; kt < C::KT; ++kt) {
#pragma unroll
      for (int qt = 0; qt < C::QT; ++qt)
#pragma unroll
        for (int i = 0; i < 16; ++i) s[kt][qt][i] = 0.f;
      const int row = wc * C::KH + 32 * kt + l32;
#pragma unroll
      for (int ds = 0; ds < C::DS; ++ds) {
        const bf16x8 a = *reinterpret_cast<const bf16x8*>(Ks + row * (D * 2) + swz<C::CHK>(row, 2 * ds + lh) * 16);
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

    // ---- online softmax (eqs. 2, 3), one query column per lane -------------------------
    bf16x8 pf[C::QT][C::KS];
#pragma unroll
    for (int qt = 0; qt < C::QT; ++qt) {
      float mx = -INFINITY;
#pragma unroll
      for (int kt = 0; kt < C::KT; ++kt)
#pragma unroll
        for (int i = 0; i < 16; ++i) mx = fmaxf(mx, s[kt][qt][i]);
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      const float m_new = fmaxf(m_run[qt], mx * scale_log2);
      const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
      const float alpha = __builtin_amdgcn_exp2f(m_run[qt] - m_use);
      m_run[qt] = m_new;
      float rs = 0.f;
#pragma unroll
      for (int kt = 0; kt < C::KT; ++kt)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s[kt][qt][i], scale_log2, -m_use));
          s[kt][qt][i] = p;
          rs += p;
        }
      l_run[qt] = l_run[qt] * alpha + rs;
#pragma unroll
      for (int dt = 0; dt < C::DT; ++dt)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[dt][qt][i] *= alpha;
#pragma unroll
      for (int ks = 0; ks < C::KS; ++ks)
#pragma unroll
        for (int e = 0; e < 8; ++e) pf[qt][ks][e] = (__bf16)s[ks / 2][qt][8 * (ks % 2) + e];
    }

    store_v();
    __syncthreads();
    if (it + 1 < cnt) load_tile(kbase + (size_t)block_at(it + 1) * BLK * D);

    // ---- O^T += V^T P^T (eq. 4) ---------------------------------------------------------
#pragma unroll
    for (int dt = 0; dt < C::DT; ++dt) {
      const int row = 32 * dt + l32;
#pragma unroll
      for (int ks = 0; ks < C::KS; ++ks) {
        const bf16x8 a =
            *reinterpret_cast<const bf16x8*>(Vs + row * (BLK * 2) + swz<C::CHV>(row, 2 * (wc * C::KS + ks) + lh) * 16);
#pragma unroll
        for (int qt = 0; qt < C::QT; ++qt)
          o[dt][qt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf[qt][ks], o[dt][qt], 0, 0, 0);
      }
    }
  }

  // ---- merge the two key halves and write the Q block -------------------------------------
  __syncthreads();                                        // every wavefront is done with the tiles
  float* obuf = reinterpret_cast<float*>(smem);           // [wa][DT*QT*16][64 lanes]
  float* ml = reinterpret_cast<float*>(smem + C::LDS_BYTES - C::ML_FLOATS * 4);   // [wa][wc][qt][m|l][64]
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
    const float w_mine = __builtin_amdgcn_exp2f(m_run[qt] - m), w_o = __builtin_amdgcn_exp2f(m_o - m);
    m_all[qt] = m;
    l_all[qt] = l_tot[qt] * w_mine + l_o * w_o;
    f_mine[qt] = w_mine / l_all[qt];
  }
  if (wc == 1) {
#pragma unroll
    for (int dt = 0; dt < C::DT; ++dt)
#pragma unroll
      for (int qt = 0; qt < C::QT; ++qt)
#pragma unroll
        for (int i = 0; i < 16; ++i)
          obuf[((wa * C::DT * C::QT + dt * C::QT + qt) * 16 + i) * 64 + lane] = o[dt][qt][i] * f_mine[qt];
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
            const float other = obuf[((wa * C::DT * C::QT + dt * C::QT + qt) * 16 + i) * 64 + lane];
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
  RF2_HIP(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_BYTES));
  const float scale_log2 = (float)(1.4426950408889634 / sqrt((double)D));
  const unsigned grid = 8u * (unsigned)plan->rows_per_xcd * (unsigned)(c.batch * c.heads);
  kern<<<dim3(grid), dim3(C::NT), C::LDS_BYTES, st>>>((const __bf16*)qp, (const __bf16*)kp, (const __bf16*)vp, blk_idx,
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
