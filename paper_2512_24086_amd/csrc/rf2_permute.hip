// Token permutation (Sec. 3.3 / 3.4) fused with block-mean pooling (Sec. 3.2, eqs. 5-6),
// the key-major re-tiling of V for the attention kernel, and the inverse permutation.
// All three kernels are pure HBM traffic: every row moves as 16-byte vectors, a group of
// d/8 neighbouring lanes moving one whole row.
#include "rf2_internal.h"

namespace {

typedef unsigned short u16;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

// Every row is read once and written once: non-temporal accesses keep the stream from displacing
// other data in the caches on its way (measured on the 720p layer: loads alone -4 %, stores alone
// +0.5 %, both -9 % of the time of the three kernels).
__device__ __forceinline__ uint4 ld_stream(const uint4* p) {
  const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void st_stream(uint4* p, uint4 v) {
  const u32x4 w = {v.x, v.y, v.z, v.w};
  __builtin_nontemporal_store(w, reinterpret_cast<u32x4*>(p));
}

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// One workgroup gathers one block of BLK permuted rows of Q (IS_K = false) or K (true),
// writes them in permuted order and reduces their column sums to the block mean.
// Q rows stay row-major; a K block is written as BLK/64 operand parts [D/8][64][8]: with
// KH = BLK/2, the 16-byte chunk c of block row r lands in part (r % KH) / 32 at chunk slot
// c*64 + (r / KH)*32 + r % 32 -- the order in which the attention kernel's matrix-core
// operand reads walk it (a part holds one 32-key tile of each key half).
template <int D, int BLK, bool IS_K>
__global__ void __launch_bounds__(256) permute_pool_kernel(
    const uint4* __restrict__ x, uint4* __restrict__ xp, float* __restrict__ mean, const int32_t* __restrict__ perm,
    int N, int n_blocks, int last_valid, int heads, rf2_strides st) {
  constexpr int CH = D / 8;          // 16-byte chunks per row
  constexpr int RG = 256 / CH;       // rows moved per pass
  const int blk = blockIdx.x;
  const int bh = blockIdx.y;
  const uint4* __restrict__ src = x + ((bh / heads) * st.batch + (bh % heads) * st.head) * CH;
  uint4* __restrict__ dst = xp + ((size_t)bh * n_blocks + blk) * BLK * CH;
  // Q: CH neighbouring lanes move one row (row-major stores).  K: 8 neighbouring lanes move half a row
  // (one 128-byte line) and a wavefront covers 8 rows x 8 chunks, so that its stores of a chunk
  // column (8 consecutive rows x 16 bytes in the operand layout) are whole 128-byte lines too.
  int c = threadIdx.x % CH, rg = threadIdx.x / CH;
  if constexpr (IS_K && CH == 16) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    c = (lane & 7) + 8 * (wave & 1);
    rg = (lane >> 3) + 8 * (wave >> 1);
  }

  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll 4
  for (int r = rg; r < BLK; r += RG) {
    const int n = perm[blk * BLK + r];
    uint4 v = make_uint4(0u, 0u, 0u, 0u);
    if (n >= 0) v = ld_stream(&src[(size_t)n * st.token * CH + c]);
    constexpr int KH = BLK / 2;
    const int kslot = ((r % KH) / 32 * CH + c) * 64 + (r / KH) * 32 + r % 32;
    st_stream(&dst[IS_K ? kslot : r * CH + c], v);
    acc[0] += bf16_lo(v.x); acc[1] += bf16_hi(v.x);
    acc[2] += bf16_lo(v.y); acc[3] += bf16_hi(v.y);
    acc[4] += bf16_lo(v.z); acc[5] += bf16_hi(v.z);
    acc[6] += bf16_lo(v.w); acc[7] += bf16_hi(v.w);
  }
  if (mean == nullptr) return;
  __shared__ float part[RG][D + 1];
#pragma unroll
  for (int e = 0; e < 8; ++e) part[rg][c * 8 + e] = acc[e];
  __syncthreads();
  if (threadIdx.x < D) {
    float s = 0.f;
#pragma unroll
    for (int g = 0; g < RG; ++g) s += part[g][threadIdx.x];   // fixed order: bit-reproducible
    const int cnt = (blk == n_blocks - 1) ? last_valid : BLK;
    mean[((size_t)bh * n_blocks + blk) * D + threadIdx.x] = s / (float)cnt;
  }
}

// Position inside a 16-key group of the key-major V tile -> key offset (see rf2.h).
__device__ __forceinline__ int rho(int r) { return (r & 3) | ((r & 4) << 1) | ((r & 8) >> 1); }

// One workgroup gathers the 64 permuted rows of V that make up one operand part into LDS and writes
// the part [8][D][8] of the attention kernel's second product (16 KiB or 8 KiB, contiguous).
// Storage position s of a key inside its block: each 16-key group is listed in the order
// 0-3, 8-11, 4-7, 12-15.  With KH = BLK/2, position s goes to part (s % KH) / 32, chunk
// g = (s / KH)*4 + (s % 32) / 8, element s % 8; the 16-byte chunk (part, g, ch) holds
// channel ch of those 8 keys.  A part thus holds the block rows 32*part .. 32*part+31 and
// KH + 32*part .. KH + 32*part + 31 (the reordering stays inside a 16-key group).
template <int D, int BLK>
__global__ void __launch_bounds__(256) permute_vtile_kernel(
    const uint4* __restrict__ v, uint4* __restrict__ vp, const int32_t* __restrict__ perm, int N, int n_blocks,
    int heads, rf2_strides st) {
  constexpr int CH = D / 8;
  constexpr int RG = 256 / CH;
  constexpr int PITCH = D + 2;       // u16 elements per LDS row: odd number of dwords
  constexpr int PB = BLK / 64, KH = BLK / 2;
  __shared__ __attribute__((aligned(16))) u16 tile[64 * PITCH];
  const int blk = blockIdx.x / PB, part = blockIdx.x % PB, bh = blockIdx.y;
  const uint4* __restrict__ src = v + ((bh / heads) * st.batch + (bh % heads) * st.head) * CH;
  const int c = threadIdx.x % CH, rg = threadIdx.x / CH;
#pragma unroll
  for (int lr = rg; lr < 64; lr += RG) {                      // local row -> block row
    const int r = (lr / 32) * KH + part * 32 + lr % 32;
    const int n = perm[blk * BLK + r];
    uint4 x = make_uint4(0u, 0u, 0u, 0u);
    if (n >= 0) x = ld_stream(&src[(size_t)n * st.token * CH + c]);
    uint32_t* row = reinterpret_cast<uint32_t*>(tile + lr * PITCH + c * 8);  // 4-byte aligned: PITCH, c*8 even
    row[0] = x.x; row[1] = x.y; row[2] = x.z; row[3] = x.w;
  }
  __syncthreads();
  uint4* __restrict__ dst = vp + (((size_t)bh * n_blocks + blk) * PB + part) * D * 8;
  for (int o = threadIdx.x; o < D * 8; o += 256) {
    const int g = o / D, ch = o % D;   // consecutive lanes -> consecutive channels: contiguous 16-byte stores
    const int sbase = (g / 4) * 32 + (g % 4) * 8;             // first local storage position of this chunk
    uint32_t w[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int s0 = sbase + 2 * e, s1 = s0 + 1;
      const int k0 = (s0 & ~15) + rho(s0 & 15), k1 = (s1 & ~15) + rho(s1 & 15);
      w[e] = (uint32_t)tile[k0 * PITCH + ch] | ((uint32_t)tile[k1 * PITCH + ch] << 16);
    }
    st_stream(&dst[o], make_uint4(w[0], w[1], w[2], w[3]));
  }
}

// o[n] = op[inv[n]]: gathered reads, fully sequential writes.
template <int D>
__global__ void __launch_bounds__(256) unpermute_kernel(
    const uint4* __restrict__ op, uint4* __restrict__ o, const int32_t* __restrict__ inv, int N, size_t N_pad,
    int heads, rf2_strides st) {
  constexpr int CH = D / 8;
  constexpr int RG = 256 / CH;
  const int bh = blockIdx.y;
  const uint4* __restrict__ src = op + (size_t)bh * N_pad * CH;
  uint4* __restrict__ dst = o + ((bh / heads) * st.batch + (bh % heads) * st.head) * CH;
  const int c = threadIdx.x % CH, rg = threadIdx.x / CH;
  const int n0 = blockIdx.x * 128;
#pragma unroll 4
  for (int r = rg; r < 128; r += RG) {
    const int n = n0 + r;
    if (n < N) st_stream(&dst[(size_t)n * st.token * CH + c], ld_stream(&src[(size_t)inv[n] * CH + c]));
  }
}

}  // namespace

namespace {

template <int D, int BQ>
void launch_permute_q(const rf2_plan* plan, const void* q, void* qp, float* qbar, hipStream_t st) {
  const rf2_info& in = plan->info;
  const dim3 grid(in.n_blocks, plan->cfg.batch * plan->cfg.heads, 1);
  permute_pool_kernel<D, BQ, false><<<grid, 256, 0, st>>>((const uint4*)q, (uint4*)qp, qbar, plan->d_perm, (int)in.N,
                                                           in.n_blocks, in.last_block_valid, plan->cfg.heads,
                                                           rf2_qkv_strides(plan));
}

template <int D, int BK>
void launch_permute_kv(const rf2_plan* plan, const void* k, const void* v, void* kp, void* vp, float* kbar,
                       hipStream_t st) {
  const rf2_info& in = plan->info;
  const dim3 grid(in.n_blocks_k, plan->cfg.batch * plan->cfg.heads, 1);
  permute_pool_kernel<D, BK, true><<<grid, 256, 0, st>>>((const uint4*)k, (uint4*)kp, kbar, plan->d_perm, (int)in.N,
                                                          in.n_blocks_k, in.last_block_valid_k, plan->cfg.heads,
                                                          rf2_qkv_strides(plan));
  const dim3 grid_v(in.n_blocks_k * (BK / 64), plan->cfg.batch * plan->cfg.heads, 1);   // one workgroup per 64-key part
  permute_vtile_kernel<D, BK><<<grid_v, 256, 0, st>>>((const uint4*)v, (uint4*)vp, plan->d_perm, (int)in.N,
                                                       in.n_blocks_k, plan->cfg.heads, rf2_qkv_strides(plan));
}

template <int D>
int permute_for_dim(const rf2_plan* plan, const void* q, const void* k, const void* v, void* qp, void* kp, void* vp,
                    float* qbar, float* kbar, hipStream_t st) {
  switch (plan->cfg.block) {
    case 64: launch_permute_q<D, 64>(plan, q, qp, qbar, st); break;
    case 128: launch_permute_q<D, 128>(plan, q, qp, qbar, st); break;
    case 256: launch_permute_q<D, 256>(plan, q, qp, qbar, st); break;
    default: return RF2_ERR_UNSUPPORTED;
  }
  RF2_LAUNCH_CHECK();
  switch (plan->info.block_k) {
    case 64: launch_permute_kv<D, 64>(plan, k, v, kp, vp, kbar, st); break;
    case 128: launch_permute_kv<D, 128>(plan, k, v, kp, vp, kbar, st); break;
    default: return RF2_ERR_UNSUPPORTED;
  }
  RF2_LAUNCH_CHECK();
  return RF2_OK;
}

}  // namespace

extern "C" int rf2_permute(const rf2_plan* plan, const void* q, const void* k, const void* v, void* qp, void* kp,
                           void* vp, float* qbar, float* kbar, void* stream) {
  if (!plan || !q || !k || !v || !qp || !kp || !vp) return RF2_ERR_INVALID_ARG;
  if ((qbar == nullptr) != (kbar == nullptr)) return RF2_ERR_INVALID_ARG;
  if (const int rc = rf2_check_device(plan)) return rc;
  hipStream_t st = (hipStream_t)stream;
  if (plan->cfg.head_dim == 128) return permute_for_dim<128>(plan, q, k, v, qp, kp, vp, qbar, kbar, st);
  if (plan->cfg.head_dim == 64) return permute_for_dim<64>(plan, q, k, v, qp, kp, vp, qbar, kbar, st);
  return RF2_ERR_UNSUPPORTED;
}

extern "C" int rf2_unpermute(const rf2_plan* plan, const void* op, void* o, void* stream) {
  if (!plan || !op || !o) return RF2_ERR_INVALID_ARG;
  if (const int rc = rf2_check_device(plan)) return rc;
  const rf2_config& c = plan->cfg;
  const rf2_info& in = plan->info;
  hipStream_t st = (hipStream_t)stream;
  const dim3 grid((unsigned)((in.N + 127) / 128), c.batch * c.heads, 1);
  if (c.head_dim == 128)
    unpermute_kernel<128><<<grid, 256, 0, st>>>((const uint4*)op, (uint4*)o, plan->d_inv, (int)in.N, (size_t)in.N_pad,
                                         c.heads, rf2_qkv_strides(plan));
  else
    unpermute_kernel<64><<<grid, 256, 0, st>>>((const uint4*)op, (uint4*)o, plan->d_inv, (int)in.N, (size_t)in.N_pad,
                                         c.heads, rf2_qkv_strides(plan));
  RF2_LAUNCH_CHECK();
  return RF2_OK;
}
