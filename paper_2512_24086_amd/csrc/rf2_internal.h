// Internal declarations shared by the translation units of librf2 (not installed).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <vector>

#include "rf2.h"

struct rf2_plan {
  rf2_config cfg;
  rf2_info info;
  int device;
  std::vector<int32_t> perm, inv;  // host copies, N entries each
  int32_t* d_perm;                 // device, N_pad entries; -1 marks a padding row
  int32_t* d_inv;                  // device, N entries
  int32_t* d_row_order;            // device, [8][plain_per_xcd]: ordinary Q block of each workgroup slot of a head, -1 = none
  int32_t plain_per_xcd;
};

// Strides (in rows of d elements) of the caller's q, k, v, o tensors: row of token n of head h of
// batch b = b*batch + h*head + n*token.
struct rf2_strides {
  long long batch, head, token;
};
inline rf2_strides rf2_qkv_strides(const rf2_plan* p) {
  const long long N = p->info.N, Hh = p->cfg.heads;
  if (p->cfg.qkv_layout == RF2_LAYOUT_BNHD) return {N * Hh, 1, Hh};
  return {Hh * N, N, 1};
}

// Per-plan preparation of the mask kernel (dynamic LDS limit); defined in rf2_mask.hip.
int rf2_mask_prepare(const rf2_plan* plan);

// Remembers the text of a failed HIP call for rf2_strerror (per calling thread).
int rf2_note_hip_error(hipError_t e);

#define RF2_HIP(call)                                   \
  do {                                                  \
    hipError_t e__ = (call);                            \
    if (e__ != hipSuccess) return rf2_note_hip_error(e__); \
  } while (0)

// Compute entry points run on the device the plan's tables live on: a plan without a device
// cannot compute (RF2_ERR_HIP), and a call made while another device is current is rejected
// (RF2_ERR_INVALID_ARG) instead of launching against the wrong GPU's tables.
inline int rf2_check_device(const rf2_plan* plan) {
  if (plan->device < 0) return rf2_note_hip_error(hipErrorNoDevice);
  int current = -1;
  const hipError_t e = hipGetDevice(&current);
  if (e != hipSuccess) return rf2_note_hip_error(e);
  return current == plan->device ? RF2_OK : RF2_ERR_INVALID_ARG;
}

// Launch check used after every kernel launch.
#define RF2_LAUNCH_CHECK() RF2_HIP(hipGetLastError())
