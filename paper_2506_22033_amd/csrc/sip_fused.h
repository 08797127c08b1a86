// finish_kernel and rescue_kernel in one, for batches of at most one row per compute unit: a
// workgroup finishes its row from the list (finish_row) and, if the list does not settle it,
// goes on with the heavier logic (rescue_row) itself, at once.  No queue, no second launch
// behind it -- whose four microseconds, the latency of starting any kernel, are a fifteenth of
// such a call.  The price is the LDS of the heavier logic for every workgroup (one workgroup per
// compute unit), which a batch this small does not feel.
#pragma once
#include "sip_final.h"
#include "sip_finish.h"

namespace sip {

constexpr size_t kFusedRawBytes = 122880;   // final_lds_fixed() of the largest vocabulary of the single-pass kernels
static_assert(sizeof(FinShared) <= kFusedRawBytes, "the finishing tables lie inside the same LDS");

template <int DT, bool SH>
__global__ __launch_bounds__(kFinalThreads) void finish_rescue_kernel(Args a_by_value) {
  (void)a_by_value;
  const Args& a = *(const Args*)__builtin_amdgcn_kernarg_segment_ptr();
  warm_kernel_arguments();
  __shared__ union __align__(16) { FinShared fs; unsigned char raw[kFusedRawBytes]; } u;
  __shared__ ExactShared ex;
  __shared__ FastShared fsr;
  static_assert(kFinThreads == kFinalThreads, "one workgroup shape for both parts");
  const int b = blockIdx.x;
  FinHint hint;
  const int code = finish_row(a, b, u.fs, &hint);
  if (threadIdx.x == 0) {
    a.row_path[b] = code;
    a.row_why[b] = code;
  }
  if (code == 1) return;                     // uniform
  __syncthreads();
  RescueSeen seen;
  if (hint.valid) { seen.why = code; seen.retry_ok = hint.retry_ok; seen.m = hint.m; seen.zmax = hint.zmax; seen.T = hint.T; }
  rescue_row<DT, SH>(a, b, u.raw, ex, fsr, seen);
}

}  // namespace sip
