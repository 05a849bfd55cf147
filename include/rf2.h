/*
 * rf2.h -- C ABI of librf2: one block-sparse attention layer of a Diffusion
 * Transformer as described by RainFusion2.0 (arXiv 2512.24086), for one AMD
 * MI355X (gfx950).
 *
 * The layer, in the order the paper gives it (Fig. 1):
 *   rf2_permute           Sec. 3.3 window permutation (+ Sec. 3.4 first frame moved
 *                         to the sequence end) fused with the block means of
 *                         Sec. 3.2, eqs. (5) and (6)
 *   rf2_predict_mask      Sec. 3.2, eq. (7) block scores and eq. (8) top-n
 *                         selection, plus the first-frame sink of Sec. 3.4
 *   rf2_block_sparse_attn Sec. 3.1, eqs. (1)-(4) with the block skip rule
 *   rf2_unpermute         inverse of the Sec. 3.3 permutation
 *   (rf2_block_sparse_attn_unpermuted does the last two in one kernel.)
 *
 * Conventions
 *   - Every function returns an int: RF2_OK (0) or a negative RF2_ERR_* code.
 *     Nothing throws, aborts or synchronises the device behind the caller's back.
 *   - Pointers named *_host are host memory; every other tensor pointer is DEVICE
 *     memory on the device that was current when the plan was created.  The
 *     caller owns all tensors; the plan owns only its index tables.  A compute
 *     call made while another device is current returns RF2_ERR_INVALID_ARG
 *     (it would launch against the wrong device's tables); a plan created
 *     without any device returns RF2_ERR_HIP from every compute call.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All
 *     work is enqueued asynchronously on it.
 *   - Tensors are dense, contiguous, row-major in the stated shape.  "bf16" is the
 *     16-bit brain float (upper half of an IEEE binary32).
 *   - Arguments are validated on the host before any launch; a failed call has
 *     launched nothing.
 *   - A plan is immutable after creation; calls sharing a plan may run
 *     concurrently on different streams.
 *
 * Notation: B batch, Hh heads, d head_dim, N = T*H*W (+ text_tokens) tokens, b block
 * size, Tb = ceil(N/b) blocks, N_pad = Tb*b.  Q blocks have b = `block` rows; K and V
 * blocks have `block_k` rows when that is set (b_q != b_k): then every K-side quantity
 * -- kp, vp, kbar, the entries of the block lists, the columns of the block mask, the
 * count that flags a dense row -- uses b = block_k and Tb = rf2_info.n_blocks_k, and
 * the block mask is n_blocks x n_blocks_k.
 */
#ifndef RF2_H
#define RF2_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  RF2_OK = 0,
  RF2_ERR_INVALID_ARG = -1, /* NULL where not allowed, size out of range, inconsistent config */
  RF2_ERR_UNSUPPORTED = -2, /* head_dim or block size this build has no kernel for */
  RF2_ERR_ALLOC = -3,       /* host or device allocation of the plan's tables failed */
  RF2_ERR_HIP = -4,         /* a HIP runtime call or kernel launch reported an error */
  RF2_ERR_TOO_LARGE = -5    /* a size beyond the fixed capacity of the library's static device array */
};

/* How `sparsity` becomes a per-row block count (the paper only names a sparsity level). */
enum {
  RF2_BUDGET_GLOBAL = 0,        /* s = skipped fraction of the whole Tb x Tb block mask, sink included */
  RF2_BUDGET_ROW_INCL_SINK = 1, /* each row keeps ceil((1-s) Tb) blocks, sink blocks among them */
  RF2_BUDGET_ROW_PLUS_SINK = 2  /* each row selects ceil((1-s) Tb) blocks in addition to the sink */
};

/* How a row chooses its non-sink columns. */
enum {
  RF2_SELECT_TOPN = 0, /* eq. (8): the k_sel largest scores, k_sel from `sparsity` and `budget_mode` */
  RF2_SELECT_CDF = 1   /* cumulative-mass rule (the paper's Sec. 2 describes it for online adaptive patterns):
                          softmax over the non-sink columns of S_hat / sqrt(d); columns are taken in the
                          order of eq. (8) until their cumulative probability reaches `cdf_threshold`; at
                          least one.  Row lengths then depend on the data: rf2_info.k_row = Tb is only the
                          capacity of a list row, k_sel = 0, kept_pairs_per_head = -1 and
                          achieved_sparsity = -1 (unknown before the mask exists); `sparsity` is ignored. */
};

/* Memory order of the caller's q, k, v and o tensors (the paper only says Q, K, V are N x d per head). */
enum {
  RF2_LAYOUT_BHND = 0, /* [B, Hh, N, d]: one contiguous N x d matrix per head */
  RF2_LAYOUT_BNHD = 1  /* [B, N, Hh, d]: token-major, heads interleaved, as many DiT code bases hold them */
};

typedef struct {
  int32_t batch, heads, head_dim; /* head_dim in {64, 128} */
  int32_t T, H, W;                /* latent grid (frames, height, width); T = 1 for an image */
  int32_t wt, wh, ww;             /* window of the Sec. 3.3 permutation; all three 0 = default:
                                     b=256: video (4,8,8), image (1,16,16); b=128: video (2,8,8), image (1,8,16);
                                     b=64: video (4,4,4), image (1,8,8) */
  int32_t block;                  /* b_q, rows of a Q block, in {64, 128, 256}; also b_k unless block_k is set */
  int32_t sink_frames;            /* leading frames treated as the Sec. 3.4 sink: 0 or more, < T */
  int32_t sink_at_end;            /* 1: sink tokens placed after the body (Sec. 3.4, last paragraph); 0: before */
  float sparsity;                 /* target s in [0, 1) */
  int32_t budget_mode;            /* RF2_BUDGET_* */
  int32_t qkv_layout;             /* RF2_LAYOUT_*: order of q, k, v (rf2_permute) and o (rf2_unpermute,
                                     rf2_block_sparse_attn_unpermuted); the gathers absorb it for free.
                                     Permuted tensors, means, lists and lse are always head-major. */
  int32_t text_tokens;            /* tokens of the other modality appended after the T*H*W video tokens
                                     (Sec. 3.4, last paragraph); they keep their order, sit at the very end of
                                     the permuted sequence and are always dense, like the sink frames.
                                     >= 0; with text_tokens > 0 the sink frames must be at the end. */
  int32_t select_mode;            /* RF2_SELECT_* */
  float cdf_threshold;            /* tau of RF2_SELECT_CDF, strictly between 0 and 1; ignored otherwise */
  int32_t block_k;                /* b_k, rows of a K/V block, in {64, 128}; 0 = same as `block` (Sec. 3.1 lets
                                     b_q and b_k differ).  The block mask then has ceil(N/b_q) rows and
                                     ceil(N/b_k) columns; a larger b_q means fewer, longer Q rows that share
                                     one K list (less K/V traffic per query), a coarser prediction. */
} rf2_config;

typedef struct {
  int64_t N, N_pad;         /* N = T*H*W + text_tokens; N_pad = n_blocks * block (rows of qp and op) */
  int32_t n_blocks;         /* Tb = Tq: Q blocks = rows of the block mask */
  int32_t last_block_valid; /* tokens in the last Q block, 1..b_q */
  int32_t sink_block_begin, sink_block_end; /* [begin, end) of blocks holding >= 1 sink-frame or text token;
                                               equal if none */
  int32_t k_row;            /* K blocks kept by every non-sink row, sink blocks included */
  int32_t k_sel;            /* of those, chosen by score among non-sink columns = k_row - (end - begin) */
  int32_t wt, wh, ww;       /* window actually used */
  int64_t kept_pairs_per_head;
  double achieved_sparsity; /* 1 - kept_pairs_per_head / (Tq * Tk) */
  int64_t workspace_bytes;  /* size rf2_predict_mask needs at `workspace` (currently 0) */
  /* K side of the block mask; equal to the Q side unless block_k differs from block.  Wherever the
     entry points below say Tb for a COLUMN count (list entries, blk_cnt == Tb, kp/vp/kbar, the columns of
     mask_dense and scores) it is n_blocks_k, and b there is block_k. */
  int32_t block_k;            /* b_k actually used */
  int32_t n_blocks_k;         /* Tk = ceil(N / b_k) */
  int32_t last_block_valid_k; /* tokens in the last K block, 1..b_k */
  int32_t sink_block_begin_k, sink_block_end_k; /* K blocks holding >= 1 sink-frame or text token */
  int64_t N_pad_k;            /* n_blocks_k * block_k (rows of kp and vp) */
} rf2_info;

typedef struct rf2_plan rf2_plan; /* opaque */

/*
 * Host-only set-up (Sec. 3.3, 3.4): validates `cfg`, builds the permutation table
 *   perm[p] = input index of the token at permuted position p (video token (t, h, w) has
 *             input index (t*H + h)*W + w; text token i has T*H*W + i)
 * and uploads it to the current device.  Window order: body frames (t >= sink_frames)
 * are cut into windows of (wt, wh, ww) tokens, edge windows truncated; windows are
 * listed in raster order of the window grid, tokens in raster order inside a window;
 * sink frames use (1, wh, ww) windows frame by frame and follow (sink_at_end) or
 * precede the body; text tokens come last, in their own order.  *out receives a plan to be released with rf2_plan_destroy.
 * If the process sees no HIP device the plan is host-only: rf2_plan_info and
 * rf2_plan_perm work, every compute call returns RF2_ERR_HIP.
 * Limits: N <= 2^24, Tq and Tk <= 2048, B*Hh <= 65535 (RF2_ERR_UNSUPPORTED beyond).
 */
int rf2_plan_create(const rf2_config* cfg, rf2_plan** out);
int rf2_plan_destroy(rf2_plan* plan);
int rf2_plan_info(const rf2_plan* plan, rf2_info* out);
/* Copies the tables to host arrays of N int32 each (either may be NULL): inv[perm[p]] = p. */
int rf2_plan_perm(const rf2_plan* plan, int32_t* perm_host, int32_t* inv_host);

/*
 * Sec. 3.3 permutation of Q, K, V fused with the block means of eqs. (5), (6).
 *   q, k, v : [B, Hh, N, d] (or [B, N, Hh, d], see qkv_layout) bf16, tokens in
 *             [T, H, W] raster order                                       (in)
 *   qp      : [B, Hh, N_pad, d] bf16, qp[p] = q[perm[p]]; rows >= N zero  (out)
 *   (below, b = block_k and Tb = n_blocks_k: K and V are cut into K/V blocks)
 *   kp      : [B, Hh, Tb, b/64, d/8, 64, 8] bf16 operand tiles.  With KH = b/2, channel
 *             8c+e of the permuted key row blk*b + r is element
 *                 (blk, part = (r % KH) / 32, c, (r / KH)*32 + r % 32, e);
 *             rows >= N zero                                               (out)
 *   vp      : [B, Hh, Tb, b/64, 8, d, 8] bf16 operand tiles.  Inside a block the keys
 *             take storage positions s = 0..b-1, position s holding block row
 *                 16*(s/16) + rho(s%16),
 *             rho(r) = r for r in 0..3 and 12..15, r+4 for 4..7, r-4 for 8..11
 *             (each 16-key group is stored in the order 0-3, 8-11, 4-7, 12-15);
 *             channel ch of position s is element
 *                 (blk, part = (s % KH) / 32, g = (s / KH)*4 + (s % 32) / 8, ch, s % 8);
 *             rows >= N zero                                               (out)
 *             kp and vp are the layouts the attention kernel's matrix-core operand
 *             reads consume: every part (64 keys x d, contiguous) is copied to
 *             on-chip memory verbatim.  For b = 64 there is one part per block.
 *   qbar, kbar : [B, Hh, Tb, d] fp32 means over the valid rows of each block of
 *             qp / kp (the last block divides by last_block_valid).  Pass both
 *             NULL to skip pooling.                                        (out)
 * v/vp or q/qp/k/kp groups may not be NULL individually: all six are required.
 */
int rf2_permute(const rf2_plan* plan, const void* q, const void* k, const void* v,
                void* qp, void* kp, void* vp, float* qbar, float* kbar, void* stream);

/*
 * Eq. (7): S_hat[i][j] = <qbar_i, kbar_j> in fp32; eq. (8): every non-sink row i keeps
 * the k_sel non-sink columns with the largest S_hat[i][.] (equal scores: lower column
 * first) and all sink columns; sink rows keep every column (Sec. 3.4).  With
 * RF2_SELECT_CDF the non-sink columns are chosen by cumulative softmax mass instead and the
 * count of a row is whatever the rule yields (sums are fp32: a row whose cumulative mass
 * passes the threshold by less than ~1e-5 may be cut one column earlier or later than in
 * exact arithmetic).
 *   blk_idx : [B, Hh, Tb, k_row] int32, kept columns of each row in ascending order;
 *             for sink rows the first k_row entries of the row are 0..k_row-1 and the
 *             row is flagged dense by its count                            (out)
 *   blk_cnt : [B, Hh, Tb] int32: k_row (CDF: the row's own count), or Tb for a row that
 *             keeps everything                                             (out)
 *   mask_dense : optional [B, Hh, Tb, Tb] uint8 0/1, may be NULL            (out)
 *   scores  : optional [B, Hh, Tb, Tb] fp32 S_hat, may be NULL              (out)
 *   workspace : rf2_info.workspace_bytes of device memory (may be NULL when 0)
 */
int rf2_predict_mask(const rf2_plan* plan, const float* qbar, const float* kbar,
                     int32_t* blk_idx, int32_t* blk_cnt, uint8_t* mask_dense, float* scores,
                     void* workspace, void* stream);

/*
 * Sec. 3.1: for every Q block i, softmax(Q_i K_j^T / sqrt(d)) V_j accumulated over
 * the kept blocks j by the online recurrences (1)-(4); blocks not listed are skipped.
 * Keys at permuted positions >= N are excluded.  bf16 operands, fp32 accumulation.
 *   qp, kp, vp : as written by rf2_permute                                 (in)
 *   blk_idx, blk_cnt : any valid list in the rf2_predict_mask format: row stride
 *             k_row, entries ascending, distinct, in [0, Tb), count in [1, k_row]
 *             or == Tb (then the list is ignored and all blocks are used).  A count
 *             of 0 yields zero output rows and lse = -inf; counts above k_row are
 *             clamped to k_row, entries outside [0, Tb) to the nearest valid block
 *             (wrong values, never a fault).  Keys past N are masked only when the
 *             ragged last block is the LAST entry of its list, as it is in ascending
 *             lists.                                                       (in)
 *   op      : [B, Hh, N_pad, d] bf16 in permuted order; rows >= N unspecified (out)
 *   lse     : optional [B, Hh, N_pad] fp32 natural-log sum-exp of the scaled
 *             logits over the kept keys, may be NULL                       (out)
 */
int rf2_block_sparse_attn(const rf2_plan* plan, const void* qp, const void* kp, const void* vp,
                          const int32_t* blk_idx, const int32_t* blk_cnt, void* op, float* lse,
                          void* stream);

/*
 * The same attention with the inverse permutation fused into its epilogue (the layer then
 * needs no rf2_unpermute and no op buffer): row p of the result goes to token perm[p].
 *   o   : [B, Hh, N, d] (or [B, N, Hh, d], see qkv_layout) bf16, raster order (out)
 *   lse : optional [B, Hh, N] fp32, raster order, may be NULL              (out)
 * All other arguments as for rf2_block_sparse_attn; the values written are identical.
 */
int rf2_block_sparse_attn_unpermuted(const rf2_plan* plan, const void* qp, const void* kp, const void* vp,
                                     const int32_t* blk_idx, const int32_t* blk_cnt, void* o, float* lse,
                                     void* stream);

/* o[perm[p]] = op[p] for p < N.  op: [B, Hh, N_pad, d] bf16; o: [B, Hh, N, d] (or [B, N, Hh, d]) bf16. */
int rf2_unpermute(const rf2_plan* plan, const void* op, void* o, void* stream);

/*
 * Measurement aid, not part of the layer: the ceilings of the device the calling thread is on, so
 * that a benchmark can quote roofline fractions against measured as well as published peaks.
 *   mfma_bf16_tflops : rate of a loop of nothing but v_mfma_f32_32x32x16_bf16 (4 independent chains
 *                      per wavefront, 8 wavefronts per compute unit), TFLOP/s; may be NULL  (host, out)
 *   copy_gbps        : read + write bandwidth of a plain copy kernel over 1 GiB, GB/s; may be NULL
 *                                                                                         (host, out)
 * Allocates (and frees) 2 GiB of device memory and synchronises with `stream`; takes ~0.1 s.
 */
int rf2_measure_peaks(double* mfma_bf16_tflops, double* copy_gbps, void* stream);

/*
 * Measurement aid: the bf16 MFMA rate the device SUSTAINS for `seconds` (0 < seconds <= 30) of a loop of
 * nothing but v_mfma_f32_32x32x16_bf16 on pseudo-random operands.  The matrix cores draw much more power
 * on varying data than on the constant operands of rf2_measure_peaks, and a loop of this length runs at
 * the clock the power limit allows; this is the ceiling a kernel made of real products can approach.
 * The first third of the time is warm-up, the rate is taken over the rest.
 *   mfma_bf16_tflops : TFLOP/s (host, out)
 * Allocates and frees a few bytes of device memory; synchronises with `stream`.
 */
int rf2_measure_sustained_mfma(double seconds, double* mfma_bf16_tflops, void* stream);

/*
 * Measurement aid: do the workgroups g of a one-dimensional grid with equal g % 8 share an XCD, and do
 * the eight residue classes sit on eight different XCDs?  The attention kernel's work order relies on
 * exactly that (each XCD has its own L2; the Q blocks handed to the workgroups of one class are a
 * contiguous range of a head).  Which XCD a class lands on is NOT fixed: the hardware continues its
 * round-robin where the previous launch stopped, so workgroup 0 may start on any XCD.  Launches 8192
 * workgroups that read the hardware's XCC_ID register.
 *   n_agree      : workgroups that run on the XCD of their class, the classes being on 8 different XCDs
 *                  (0 if they are not)                                               (host, out)
 *   n_workgroups : workgroups launched                                              (host, out)
 *   first_xcd    : XCD of workgroup 0, may be NULL                                  (host, out)
 * Allocates and frees 32 KiB of device memory; synchronises with `stream`.
 */
int rf2_probe_xcd_mapping(int32_t* n_agree, int32_t* n_workgroups, int32_t* first_xcd, void* stream);

/*
 * rf2_probe_xcd_mapping for callers that cannot allocate: code between other work of a serving loop,
 * harnesses that forbid hipMalloc, callers that must not block.  Same probe kernel, same count; the
 * per-workgroup table lives in a static device array of the library (32 KiB on every GPU the library
 * runs on, held until the process ends), the count is taken by a second kernel, and the answer is left
 * in device memory.  Calls no hipMalloc / hipFree and no other allocating routine, copies nothing to
 * the host and does not synchronise: three kernel launches on `stream`.
 *   n_launch : workgroups to launch, 8 <= n_launch <= RF2_XCD_PROBE_MAX_WORKGROUPS; fewer than 8:
 *              RF2_ERR_INVALID_ARG; more: RF2_ERR_TOO_LARGE (nothing is launched)
 *   result   : [2] int32 (device, out): result[0] = workgroups g < n_launch that ran on the XCD of
 *              workgroup g % 8, the first eight being on eight different XCDs (0 if they are not),
 *              i.e. rf2_probe_xcd_mapping's n_agree for n_launch workgroups; result[1] = XCD of
 *              workgroup 0.  Valid once the work on `stream` has completed.
 * The first call on a device looks the array's address up (hipGetSymbolAddress); every call on a GPU
 * shares that GPU's array, which keeps the previous call's contents (the entries a call reads are
 * reset by the call itself): calls that overlap on one GPU, on different streams, race.
 */
#define RF2_XCD_PROBE_MAX_WORKGROUPS 8192
int rf2_probe_xcd_mapping_static(int32_t n_launch, int32_t* result, void* stream);

/* Static description of an error code; for RF2_ERR_HIP the text of the last HIP error seen
 * by the calling thread is appended. */
const char* rf2_strerror(int code);
/* major*10000 + minor*100 + patch */
int rf2_version(void);

#ifdef __cplusplus
}
#endif
#endif /* RF2_H */
