// Host side of librf2: configuration checks, permutation tables, block budget, error text.
#include <cmath>
#include <cstdio>
#include <cstring>
#include <new>
#include <string>

#include "rf2_internal.h"

namespace {

thread_local std::string g_hip_error_text;
thread_local std::string g_strerror_buf;

struct Window {
  int wt, wh, ww;
};

// Default window: volume equals the block so that an interior window is exactly one block.
Window default_window(int block, bool video) {
  if (block == 256) return video ? Window{4, 8, 8} : Window{1, 16, 16};
  if (block == 128) return video ? Window{2, 8, 8} : Window{1, 8, 16};
  return video ? Window{4, 4, 4} : Window{1, 8, 8};
}

// [begin, end) of the blocks of b tokens that hold at least one always-dense token (Sec. 3.4).
void dense_block_range(int64_t N, int64_t n_sink, int64_t n_text, bool tail, int b, int32_t* begin, int32_t* end) {
  const int32_t Tb = (int32_t)((N + b - 1) / b);
  if (n_sink + n_text == 0) { *begin = *end = 0; }
  else if (tail) { *begin = (int32_t)((N - n_sink - n_text) / b); *end = Tb; }
  else { *begin = 0; *end = (int32_t)((n_sink + b - 1) / b); }
}

// Position of token (tp, h, w) inside a group of Tn frames ordered window by window
// (Sec. 3.3): windows in raster order over the window grid, raster order inside a
// window, edge windows truncated.  Closed form of that enumeration.
int64_t window_position(int Tn, int H, int W, int wt, int wh, int ww, int tp, int h, int w) {
  const int a = tp / wt, b = h / wh, c = w / ww;
  const int u = tp % wt, v = h % wh, x = w % ww;
  const int64_t et = std::min(wt, Tn - a * wt);
  const int64_t eh = std::min(wh, H - b * wh);
  const int64_t ew = std::min(ww, W - c * ww);
  return (int64_t)a * wt * H * W      // all earlier window slabs along t are full slabs
         + et * ((int64_t)b * wh * W) // earlier window rows inside this slab
         + et * eh * ((int64_t)c * ww) // earlier windows inside this window row
         + (int64_t)u * eh * ew + (int64_t)v * ew + x;
}

}  // namespace

int rf2_note_hip_error(hipError_t e) {
  g_hip_error_text = hipGetErrorString(e);
  (void)hipGetLastError();  // clear the sticky-less error state
  return RF2_ERR_HIP;
}

extern "C" {

int rf2_version(void) { return 100; }

const char* rf2_strerror(int code) {
  switch (code) {
    case RF2_OK: return "ok";
    case RF2_ERR_INVALID_ARG: return "invalid argument";
    case RF2_ERR_UNSUPPORTED: return "unsupported head_dim / block size / problem size";
    case RF2_ERR_ALLOC: return "allocation failed";
    case RF2_ERR_TOO_LARGE: return "size exceeds the capacity of the library's static device array";
    case RF2_ERR_HIP:
      g_strerror_buf = "HIP error: " + g_hip_error_text;
      return g_strerror_buf.c_str();
    default: return "unknown error code";
  }
}

int rf2_plan_create(const rf2_config* cfg, rf2_plan** out) {
  if (!cfg || !out) return RF2_ERR_INVALID_ARG;
  *out = nullptr;
  const rf2_config& c = *cfg;
  if (c.batch < 1 || c.heads < 1 || c.T < 1 || c.H < 1 || c.W < 1) return RF2_ERR_INVALID_ARG;
  if (c.sink_frames < 0 || c.sink_frames >= c.T) return RF2_ERR_INVALID_ARG;
  if (c.sink_at_end != 0 && c.sink_at_end != 1) return RF2_ERR_INVALID_ARG;
  if (!(c.sparsity >= 0.0f && c.sparsity < 1.0f)) return RF2_ERR_INVALID_ARG;  // also rejects NaN
  if (c.budget_mode < RF2_BUDGET_GLOBAL || c.budget_mode > RF2_BUDGET_ROW_PLUS_SINK) return RF2_ERR_INVALID_ARG;
  if (c.qkv_layout != RF2_LAYOUT_BHND && c.qkv_layout != RF2_LAYOUT_BNHD) return RF2_ERR_INVALID_ARG;
  if (c.text_tokens < 0) return RF2_ERR_INVALID_ARG;
  if (c.select_mode != RF2_SELECT_TOPN && c.select_mode != RF2_SELECT_CDF) return RF2_ERR_INVALID_ARG;
  if (c.select_mode == RF2_SELECT_CDF && !(c.cdf_threshold > 0.0f && c.cdf_threshold < 1.0f)) return RF2_ERR_INVALID_ARG;
  // the always-dense tokens must form one run of the permuted sequence
  if (c.text_tokens > 0 && c.sink_frames > 0 && !c.sink_at_end) return RF2_ERR_UNSUPPORTED;
  if (c.wt < 0 || c.wh < 0 || c.ww < 0) return RF2_ERR_INVALID_ARG;
  const bool win_default = (c.wt == 0 && c.wh == 0 && c.ww == 0);
  if (!win_default && (c.wt < 1 || c.wh < 1 || c.ww < 1)) return RF2_ERR_INVALID_ARG;
  if (c.head_dim != 64 && c.head_dim != 128) return RF2_ERR_UNSUPPORTED;
  if (c.block != 64 && c.block != 128 && c.block != 256) return RF2_ERR_UNSUPPORTED;
  if (c.block_k != 0 && c.block_k != 64 && c.block_k != 128) return RF2_ERR_UNSUPPORTED;
  if (c.block_k == 0 && c.block == 256) return RF2_ERR_UNSUPPORTED;   // K/V blocks have 64 or 128 rows
  const int64_t n_video = (int64_t)c.T * c.H * c.W;
  const int64_t N = n_video + c.text_tokens;
  if (N > (int64_t)1 << 24) return RF2_ERR_UNSUPPORTED;  // 16 Mi tokens: keeps every index in int32
  if ((int64_t)c.batch * c.heads > 65535) return RF2_ERR_UNSUPPORTED;  // grid y dimension

  rf2_plan* p = new (std::nothrow) rf2_plan();
  if (!p) return RF2_ERR_ALLOC;
  p->cfg = c;
  p->d_perm = p->d_inv = p->d_row_order = nullptr;
  const Window win = win_default ? default_window(c.block, c.T > 1) : Window{c.wt, c.wh, c.ww};

  rf2_info& in = p->info;
  const int b = c.block, bk = c.block_k ? c.block_k : c.block;
  in.N = N;
  in.n_blocks = (int32_t)((N + b - 1) / b);
  in.N_pad = (int64_t)in.n_blocks * b;
  in.last_block_valid = (int32_t)(N - (int64_t)(in.n_blocks - 1) * b);
  in.block_k = bk;
  in.n_blocks_k = (int32_t)((N + bk - 1) / bk);
  in.N_pad_k = (int64_t)in.n_blocks_k * bk;
  in.last_block_valid_k = (int32_t)(N - (int64_t)(in.n_blocks_k - 1) * bk);
  in.wt = win.wt; in.wh = win.wh; in.ww = win.ww;
  const int Tb = in.n_blocks, Tk = in.n_blocks_k;       // rows and columns of the block mask
  // one row of block scores must fit the selection kernel's LDS
  if (Tb > 2048 || Tk > 2048) { delete p; return RF2_ERR_UNSUPPORTED; }

  // Always-dense blocks: every block that holds at least one sink-frame or text token (Sec. 3.4).
  const int64_t frame = (int64_t)c.H * c.W;
  const int64_t n_sink = (int64_t)c.sink_frames * frame;
  const bool tail = c.sink_at_end || n_sink == 0;
  dense_block_range(N, n_sink, c.text_tokens, tail, b, &in.sink_block_begin, &in.sink_block_end);
  dense_block_range(N, n_sink, c.text_tokens, tail, bk, &in.sink_block_begin_k, &in.sink_block_end_k);
  const int nS = in.sink_block_end - in.sink_block_begin;          // sink rows
  const int nSk = in.sink_block_end_k - in.sink_block_begin_k;     // sink columns

  // K blocks kept per non-sink row.  The sparsity is a float; the arithmetic is double.
  const double keep = 1.0 - (double)c.sparsity;
  int k_row;
  if (nS >= Tb) {
    k_row = Tk;
  } else {
    if (c.budget_mode == RF2_BUDGET_GLOBAL)
      k_row = (int)std::floor((keep * Tb * Tk - (double)nS * Tk) / (double)(Tb - nS));
    else if (c.budget_mode == RF2_BUDGET_ROW_INCL_SINK)
      k_row = (int)std::ceil(keep * Tk);
    else
      k_row = (int)std::ceil(keep * Tk) + nSk;
    k_row = std::min(std::max(std::max(k_row, nSk), 1), Tk);
  }
  in.k_row = k_row;
  in.k_sel = nS >= Tb ? 0 : k_row - nSk;
  in.kept_pairs_per_head = (int64_t)(Tb - nS) * k_row + (int64_t)nS * Tk;
  in.achieved_sparsity = 1.0 - (double)in.kept_pairs_per_head / ((double)Tb * Tk);
  if (c.select_mode == RF2_SELECT_CDF) {   // row lengths depend on the data: k_row is the list capacity
    in.k_row = Tk;
    in.k_sel = 0;
    in.kept_pairs_per_head = -1;
    in.achieved_sparsity = -1.0;
  }
  in.workspace_bytes = 0;

  // Permutation tables from the closed form.
  try {
    p->perm.assign((size_t)N, -1);
    p->inv.assign((size_t)N, -1);
  } catch (...) { delete p; return RF2_ERR_ALLOC; }
  const int Tbody = c.T - c.sink_frames;
  const int64_t body_tokens = (int64_t)Tbody * frame;
  for (int t = 0; t < c.T; ++t)
    for (int h = 0; h < c.H; ++h)
      for (int w = 0; w < c.W; ++w) {
        int64_t pos;
        if (t >= c.sink_frames) {
          pos = window_position(Tbody, c.H, c.W, win.wt, win.wh, win.ww, t - c.sink_frames, h, w);
          if (!c.sink_at_end) pos += n_sink;
        } else {
          pos = window_position(c.sink_frames, c.H, c.W, 1, win.wh, win.ww, t, h, w);
          if (c.sink_at_end) pos += body_tokens;
        }
        const int64_t n = ((int64_t)t * c.H + h) * c.W + w;
        p->inv[(size_t)n] = (int32_t)pos;
        p->perm[(size_t)pos] = (int32_t)n;
      }
  for (int64_t n = n_video; n < N; ++n) p->inv[(size_t)n] = p->perm[(size_t)n] = (int32_t)n;   // text: in place, last

  // Work table of the attention kernel.  Workgroups g with equal g % 8 run on one XCD.  Each XCD gets a
  // contiguous range of a head's ordinary Q blocks (neighbouring blocks tend to pick the same K blocks, so
  // they share its L2).  The all-column sink rows need no table: the kernel deals them out itself, in
  // contiguous runs over all heads, and issues them ahead of the ordinary rows.
  const int sb = in.sink_block_begin;
  std::vector<std::vector<int32_t>> plain_xcd(8);
  const int n_plain = Tb - nS;
  for (int r = 0; r < n_plain; ++r) {
    const int i = r < sb ? r : r + nS;
    plain_xcd[(int)(((int64_t)r * 8) / std::max(n_plain, 1))].push_back(i);
  }
  size_t ppx = 0;
  for (int x = 0; x < 8; ++x) ppx = std::max(ppx, plain_xcd[x].size());
  p->plain_per_xcd = (int32_t)ppx;
  std::vector<int32_t> order(std::max<size_t>(8 * ppx, 1), -1);      // [share][slot], -1 = no work
  for (int x = 0; x < 8; ++x)
    for (size_t r = 0; r < plain_xcd[x].size(); ++r) order[x * ppx + r] = plain_xcd[x][r];

  std::vector<int32_t> perm_pad((size_t)std::max(in.N_pad, in.N_pad_k), -1);
  std::memcpy(perm_pad.data(), p->perm.data(), (size_t)N * sizeof(int32_t));

  // Without a HIP device the plan stays host-only: info and tables work, compute calls fail.
  int n_dev = 0;
  if (hipGetDeviceCount(&n_dev) != hipSuccess || n_dev == 0) {
    (void)hipGetLastError();
    p->device = -1;
    *out = p;
    return RF2_OK;
  }
  if (hipGetDevice(&p->device) != hipSuccess) { delete p; return rf2_note_hip_error(hipGetLastError()); }
  hipError_t e = hipMalloc((void**)&p->d_perm, perm_pad.size() * sizeof(int32_t));
  if (e == hipSuccess) e = hipMalloc((void**)&p->d_inv, (size_t)N * sizeof(int32_t));
  if (e == hipSuccess) e = hipMalloc((void**)&p->d_row_order, order.size() * sizeof(int32_t));
  if (e == hipSuccess) e = hipMemcpy(p->d_perm, perm_pad.data(), perm_pad.size() * sizeof(int32_t), hipMemcpyHostToDevice);
  if (e == hipSuccess) e = hipMemcpy(p->d_inv, p->inv.data(), (size_t)N * sizeof(int32_t), hipMemcpyHostToDevice);
  if (e == hipSuccess) e = hipMemcpy(p->d_row_order, order.data(), order.size() * sizeof(int32_t), hipMemcpyHostToDevice);
  if (e != hipSuccess) {
    const int rc = (e == hipErrorOutOfMemory) ? RF2_ERR_ALLOC : rf2_note_hip_error(e);
    rf2_plan_destroy(p);
    return rc;
  }
  const int prep = rf2_mask_prepare(p);
  if (prep != RF2_OK) { rf2_plan_destroy(p); return prep; }
  *out = p;
  return RF2_OK;
}

int rf2_plan_destroy(rf2_plan* p) {
  if (!p) return RF2_OK;
  if (p->d_perm) (void)hipFree(p->d_perm);
  if (p->d_inv) (void)hipFree(p->d_inv);
  if (p->d_row_order) (void)hipFree(p->d_row_order);
  delete p;
  return RF2_OK;
}

int rf2_plan_info(const rf2_plan* p, rf2_info* out) {
  if (!p || !out) return RF2_ERR_INVALID_ARG;
  *out = p->info;
  return RF2_OK;
}

int rf2_plan_perm(const rf2_plan* p, int32_t* perm_host, int32_t* inv_host) {
  if (!p) return RF2_ERR_INVALID_ARG;
  if (perm_host) std::memcpy(perm_host, p->perm.data(), p->perm.size() * sizeof(int32_t));
  if (inv_host) std::memcpy(inv_host, p->inv.data(), p->inv.size() * sizeof(int32_t));
  return RF2_OK;
}

}  // extern "C"
