// Block-mask prediction: S_hat = qbar kbar^T (Sec. 3.2, eq. 7) in fp32 on the matrix cores,
// then per-row top-n selection (eq. 8) with the first-frame sink (Sec. 3.4), fused in one
// kernel.  A workgroup owns 16 rows (Q blocks) of one head: its 4 wavefronts first fill a 16 x Tk
// score strip in LDS (Tk = number of K blocks; the mask is Tq x Tk, square unless b_q != b_k),
// then each wavefront selects 4 of the rows with a bitwise threshold search over
// order-preserving integer keys and emits the ascending block list.
// The cumulative-mass variant (RF2_SELECT_CDF) runs the same search on probability mass
// instead of counts: the threshold is the largest key whose upper set carries >= tau of the
// row's softmax mass.
#include "rf2_internal.h"

namespace {

typedef __attribute__((ext_vector_type(4))) float f32x4;

// Order-preserving map float -> uint32 (larger float <=> larger key); -0 is folded into +0.
__device__ __forceinline__ uint32_t order_key(float x) {
  x = (x == 0.f) ? 0.f : x;
  const uint32_t u = __float_as_uint(x);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ int popc64(unsigned long long m) { return __builtin_popcountll(m); }

// Butterfly reductions: every lane ends with the same bits (a + b and b + a are the same float).
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
  return v;
}

template <int D, int EMAX, bool CDF>
__global__ void __launch_bounds__(256) predict_mask_kernel(
    const float* __restrict__ qbar, const float* __restrict__ kbar, int32_t* __restrict__ blk_idx,
    int32_t* __restrict__ blk_cnt, uint8_t* __restrict__ mask_dense, float* __restrict__ scores,
    int Tq, int Tb, int LD, int row_sink_begin, int row_sink_end, int sink_begin, int sink_end, int k_row, int k_sel,
    float tau, float scale_log2) {
  // Tb, sink_begin, sink_end describe the COLUMNS (K blocks) from here on; rows use Tq and row_sink_*.
  extern __shared__ __attribute__((aligned(16))) float sc[];   // [16][LD]
  const int bh = blockIdx.y;
  const int i0 = blockIdx.x * 16;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int lr = lane & 15, lk = lane >> 4;
  const float* __restrict__ qb = qbar + (size_t)bh * Tq * D;
  const float* __restrict__ kb = kbar + (size_t)bh * Tb * D;

  // ---- scores: 16 x 16 tiles with v_mfma_f32_16x16x4_f32 -------------------------------
  // Lane (lr, lk) feeds row lr of each operand.  Per 16 channels it loads 4 consecutive
  // floats at 16*kk + 4*lk; MFMA step e uses element e, so "k slot lk" stands for channel
  // 16*kk + 4*lk + e in both operands (a dot product does not care about summation order).
  f32x4 a[D / 16];
  {
    const int row = min(i0 + lr, Tq - 1);
#pragma unroll
    for (int kk = 0; kk < D / 16; ++kk) a[kk] = *reinterpret_cast<const f32x4*>(qb + (size_t)row * D + 16 * kk + 4 * lk);
  }
  const int n_ct = (Tb + 15) / 16;
  // the operand rows of the next column tile are requested before the products of the current one are
  // issued (a wavefront has ~10 tiles; unpipelined, each tile waits out a full trip to L2)
  auto load_tile = [&](f32x4 (&b)[D / 16], int ct) {
    const int col = min(ct * 16 + lr, Tb - 1);
#pragma unroll
    for (int kk = 0; kk < D / 16; ++kk) b[kk] = *reinterpret_cast<const f32x4*>(kb + (size_t)col * D + 16 * kk + 4 * lk);
  };
  f32x4 bcur[D / 16], bnext[D / 16];
  if (wave < n_ct) load_tile(bcur, wave);
  for (int ct = wave; ct < n_ct; ct += 4) {
    if (ct + 4 < n_ct) load_tile(bnext, ct + 4);
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kk = 0; kk < D / 16; ++kk) {
#pragma unroll
      for (int e = 0; e < 4; ++e) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a[kk][e], bcur[kk][e], acc, 0, 0, 0);
    }
    // acc[i] = S_hat[i0 + 4*lk + i][ct*16 + lr]
#pragma unroll
    for (int i = 0; i < 4; ++i) sc[(4 * lk + i) * LD + ct * 16 + lr] = acc[i];
#pragma unroll
    for (int kk = 0; kk < D / 16; ++kk) bcur[kk] = bnext[kk];
  }
  __syncthreads();

  if (scores != nullptr) {
    for (int r = 0; r < 16 && i0 + r < Tq; ++r)
      for (int j = threadIdx.x; j < Tb; j += 256)
        scores[((size_t)bh * Tq + i0 + r) * Tb + j] = sc[r * LD + j];
  }

  // ---- selection: wavefront `wave` handles rows wave, wave+4, wave+8, wave+12 ------------
  const int E = (Tb + 63) / 64;
  const unsigned long long lt_mask = (1ull << lane) - 1ull;
  for (int r = wave; r < 16; r += 4) {
    const int i = i0 + r;
    if (i >= Tq) break;
    int32_t* __restrict__ out = blk_idx + ((size_t)bh * Tq + i) * k_row;
    uint8_t* __restrict__ mrow = mask_dense ? mask_dense + ((size_t)bh * Tq + i) * Tb : nullptr;
    if (i >= row_sink_begin && i < row_sink_end) {  // sink row: keeps every column
      if (lane == 0) blk_cnt[(size_t)bh * Tq + i] = Tb;
      for (int j = lane; j < k_row; j += 64) out[j] = j;
      if (mrow) for (int j = lane; j < Tb; j += 64) mrow[j] = 1;
      continue;
    }
    uint32_t key[EMAX];
#pragma unroll
    for (int e = 0; e < EMAX; ++e) {
      const int j = 64 * e + lane;
      const bool cand = (e < E) && (j < Tb) && !(j >= sink_begin && j < sink_end);
      key[e] = cand ? order_key(sc[r * LD + j]) : 0u;   // 0 is below the key of every finite float
    }
    uint32_t T = 0xffffffffu;
    int need_eq;                                      // equal keys to take, lowest column first
    if constexpr (!CDF) {
      // Largest T with |{key >= T}| >= k_sel, built bit by bit: T is the k_sel-th largest key.
      if (k_sel > 0) {
        T = 0u;
        for (int bit = 31; bit >= 0; --bit) {
          const uint32_t cand = T | (1u << bit);
          int cnt = 0;
#pragma unroll
          for (int e = 0; e < EMAX; ++e)
            cnt += popc64(__builtin_amdgcn_ballot_w64(key[e] >= cand));   // (keys past the row are 0 < cand)
          if (cnt >= k_sel) T = cand;
          // exactly k_sel keys at or above T: lower bits can only raise T towards the smallest of them
          // without changing that set, and the tie rule below sees the same set either way
          if (cnt == k_sel) break;
        }
      }
      int greater = 0;
#pragma unroll
      for (int e = 0; e < EMAX; ++e)
        greater += popc64(__builtin_amdgcn_ballot_w64(key[e] > T));
      need_eq = k_sel - greater;
    } else {
      // Softmax mass of every candidate (relative to the row maximum, unnormalised), then the
      // largest T whose upper set {key >= T} carries at least tau of the total: the columns above
      // T are the shortest prefix of the descending order that reaches tau, up to ties at T.
      float mx = -INFINITY;
#pragma unroll
      for (int e = 0; e < EMAX; ++e)
        if (key[e] != 0u) mx = fmaxf(mx, sc[r * LD + 64 * e + lane]);
      mx = wave_max(mx);
      float ev[EMAX], part = 0.f;
#pragma unroll
      for (int e = 0; e < EMAX; ++e) {
        ev[e] = (key[e] != 0u) ? __builtin_amdgcn_exp2f((sc[r * LD + 64 * e + lane] - mx) * scale_log2) : 0.f;
        part += ev[e];
      }
      const float target = tau * wave_sum(part);
      T = 0u;
      for (int bit = 31; bit >= 0; --bit) {
        const uint32_t cand = T | (1u << bit);
        float mass = 0.f;
#pragma unroll
        for (int e = 0; e < EMAX; ++e) mass += (key[e] >= cand) ? ev[e] : 0.f;
        if (wave_sum(mass) >= target) T = cand;
      }
      float above = 0.f, tie = 0.f;
#pragma unroll
      for (int e = 0; e < EMAX; ++e) {
        above += (key[e] > T) ? ev[e] : 0.f;
        tie = fmaxf(tie, (key[e] == T) ? ev[e] : 0.f);
      }
      above = wave_sum(above);
      tie = wave_max(tie);                            // equal keys have equal mass
      need_eq = max(1, (int)ceilf((target - above) / tie));
    }
    int eq_run = 0, out_run = 0;
#pragma unroll
    for (int e = 0; e < EMAX; ++e) {
      if (e < E) {
        const int j = 64 * e + lane;
        const bool is_sink = (j < Tb) && (j >= sink_begin) && (j < sink_end);
        const bool eq = (key[e] == T) && (CDF ? key[e] != 0u : k_sel > 0);
        const unsigned long long eq_m = __builtin_amdgcn_ballot_w64(eq);
        const bool sel = is_sink || (key[e] > T) || (eq && (eq_run + popc64(eq_m & lt_mask) < need_eq));
        const unsigned long long sel_m = __builtin_amdgcn_ballot_w64(sel);
        if (sel) out[out_run + popc64(sel_m & lt_mask)] = j;
        if (mrow && j < Tb) mrow[j] = sel ? 1 : 0;
        eq_run += popc64(eq_m);
        out_run += popc64(sel_m);
      }
    }
    if (lane == 0) blk_cnt[(size_t)bh * Tq + i] = out_run;   // top-n: == k_row by construction
  }
}

// Shape of the launch for a plan, and the kernel instance that serves it.
struct MaskLaunch {
  const void* kernel;
  int E, LD;
  size_t lds;
};

// The kernel is instantiated for a few row widths (EMAX keys per lane): the search loops run over
// EMAX keys without bounds checks (keys past the row are 0), so a snug width saves compares.
template <int D>
const void* mask_kernel_for(int E, bool cdf) {
  if (E <= 8) return cdf ? (const void*)predict_mask_kernel<D, 8, true> : (const void*)predict_mask_kernel<D, 8, false>;
  if (E <= 12) return cdf ? (const void*)predict_mask_kernel<D, 12, true> : (const void*)predict_mask_kernel<D, 12, false>;
  if (E <= 16) return cdf ? (const void*)predict_mask_kernel<D, 16, true> : (const void*)predict_mask_kernel<D, 16, false>;
  if (E <= 20) return cdf ? (const void*)predict_mask_kernel<D, 20, true> : (const void*)predict_mask_kernel<D, 20, false>;
  if (E <= 24) return cdf ? (const void*)predict_mask_kernel<D, 24, true> : (const void*)predict_mask_kernel<D, 24, false>;
  return cdf ? (const void*)predict_mask_kernel<D, 32, true> : (const void*)predict_mask_kernel<D, 32, false>;
}

MaskLaunch mask_launch(const rf2_plan* plan) {
  MaskLaunch m;
  m.E = (plan->info.n_blocks_k + 63) / 64;
  m.LD = m.E * 64 + 4;                              // +4: the 4 row groups of a tile store hit distinct banks
  m.lds = (size_t)16 * m.LD * sizeof(float);
  const bool cdf = (plan->cfg.select_mode == RF2_SELECT_CDF);
  m.kernel = plan->cfg.head_dim == 128 ? mask_kernel_for<128>(m.E, cdf) : mask_kernel_for<64>(m.E, cdf);
  return m;
}

}  // namespace

// Called once by rf2_plan_create: a score strip wider than the default dynamic-LDS limit needs the limit of
// its kernel raised.  Doing it here keeps rf2_predict_mask free of anything but the launch (so it can be
// recorded into a HIP graph).
int rf2_mask_prepare(const rf2_plan* plan) {
  const MaskLaunch m = mask_launch(plan);
  if (m.lds > 48 * 1024)
    RF2_HIP(hipFuncSetAttribute(m.kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)m.lds));
  return RF2_OK;
}

extern "C" int rf2_predict_mask(const rf2_plan* plan, const float* qbar, const float* kbar, int32_t* blk_idx,
                                int32_t* blk_cnt, uint8_t* mask_dense, float* scores, void* workspace,
                                void* stream) {
  (void)workspace;
  if (!plan || !qbar || !kbar || !blk_idx || !blk_cnt) return RF2_ERR_INVALID_ARG;
  if (const int rc = rf2_check_device(plan)) return rc;
  const rf2_config& c = plan->cfg;
  const rf2_info& in = plan->info;
  const MaskLaunch m = mask_launch(plan);
  int Tq = in.n_blocks, Tk = in.n_blocks_k, LD = m.LD;   // rows and columns of the block mask
  int rb = in.sink_block_begin, re = in.sink_block_end, cb = in.sink_block_begin_k, ce = in.sink_block_end_k;
  int k_row = in.k_row, k_sel = in.k_sel;
  float tau = c.cdf_threshold, scale_log2 = (float)(1.4426950408889634 / sqrt((double)c.head_dim));
  void* args[] = {&qbar, &kbar, &blk_idx, &blk_cnt, &mask_dense, &scores, &Tq, &Tk, &LD, &rb, &re, &cb, &ce,
                  &k_row, &k_sel, &tau, &scale_log2};
  const dim3 grid((Tq + 15) / 16, c.batch * c.heads, 1);
  RF2_HIP(hipLaunchKernel(m.kernel, grid, dim3(256), args, m.lds, (hipStream_t)stream));
  return RF2_OK;
}
