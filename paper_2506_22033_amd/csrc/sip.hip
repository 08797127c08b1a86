// Host side of the C boundary declared in include/sip.h: argument checks, workspace
// carving and kernel launches.  No allocation, no synchronisation.
#include <hip/hip_runtime.h>

#include "../../include/sip.h"
#include "sip_device.h"
#include "sip_exact.h"

namespace {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

struct Layout {
  size_t side_z, side_c, total;
};

bool shape_ok(int32_t B, int32_t V, int dtype, int64_t nnz, int32_t k_lp) {
  return B > 0 && V > 0 && (dtype == SIP_F32 || dtype == SIP_BF16) && nnz >= 0 && k_lp >= -1;
}

Layout make_layout(int32_t, int32_t, int64_t nnz) {
  Layout l;
  size_t off = 0;
  l.side_z = off; off += align_up((size_t)nnz * sizeof(float));
  l.side_c = off; off += align_up((size_t)nnz * sizeof(unsigned int));
  l.total = off ? off : kAlign;
  return l;
}

}  // namespace

extern "C" {

size_t sip_workspace_bytes(int32_t B, int32_t V, sip_dtype dtype, int64_t hist_nnz, int32_t k_logprobs) {
  if (!shape_ok(B, V, (int)dtype, hist_nnz, k_logprobs)) return 0;
  if (V > SIP_MAX_V || k_logprobs > SIP_MAX_K_LOGPROBS) return 0;
  return make_layout(B, V, hist_nnz).total;
}

sip_status sip_sample(const void* logits, int32_t B, int32_t V, int64_t row_stride, sip_dtype dtype,
                      const sip_params* params, const int64_t* hist_indptr, const int32_t* hist_tokens,
                      int64_t hist_nnz, uint64_t seed, uint64_t step, int32_t* out_ids, int32_t* out_lp_ids,
                      float* out_lp, int32_t k_logprobs, void* workspace, size_t workspace_bytes,
                      void* hip_stream) {
  if (!shape_ok(B, V, (int)dtype, hist_nnz, k_logprobs)) return SIP_ERR_INVALID_ARG;
  if (!logits || !out_ids || row_stride < V) return SIP_ERR_INVALID_ARG;
  if ((k_logprobs >= 0) != (out_lp_ids != nullptr) || (k_logprobs >= 0) != (out_lp != nullptr))
    return SIP_ERR_INVALID_ARG;
  if (hist_nnz > 0 && (!hist_indptr || !hist_tokens)) return SIP_ERR_INVALID_ARG;
  const size_t esz = dtype == SIP_F32 ? 4 : 2;
  if ((reinterpret_cast<uintptr_t>(logits) & 15u) != 0 || ((size_t)row_stride * esz) % 16 != 0)
    return SIP_ERR_INVALID_ARG;
  if (V > SIP_MAX_V || k_logprobs > SIP_MAX_K_LOGPROBS) return SIP_ERR_UNSUPPORTED;
  const Layout lay = make_layout(B, V, hist_nnz);
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & (kAlign - 1)) != 0 || workspace_bytes < lay.total)
    return SIP_ERR_WORKSPACE;

  sip::Args a;
  a.logits = logits;
  a.B = B; a.V = V; a.row_stride = row_stride;
  if (params) a.p = *params; else a.p = sip_params{};
  a.indptr = reinterpret_cast<const long long*>(hist_indptr);
  a.tokens = hist_tokens;
  a.nnz = (hist_indptr && hist_tokens) ? hist_nnz : 0;
  a.seed = seed; a.step = step;
  a.out_ids = out_ids; a.out_lp_ids = out_lp_ids; a.out_lp = out_lp; a.k_lp = k_logprobs;
  char* ws = static_cast<char*>(workspace);
  a.side_z = reinterpret_cast<float*>(ws + lay.side_z);
  a.side_c = reinterpret_cast<unsigned int*>(ws + lay.side_c);

  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const size_t words = ((size_t)V + 31) / 32;
  const size_t dyn = 2 * words * sizeof(uint32_t);
  auto kern = dtype == SIP_F32 ? sip::exact_kernel<SIP_F32> : sip::exact_kernel<SIP_BF16>;
  if (dyn > 32 * 1024) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)dyn) != hipSuccess) {
      (void)hipGetLastError();
      return SIP_ERR_HIP;
    }
  }
  hipLaunchKernelGGL(kern, dim3(B), dim3(sip::kExactThreads), dyn, stream, a);
  if (hipGetLastError() != hipSuccess) return SIP_ERR_HIP;
  return SIP_OK;
}

const char* sip_status_string(sip_status status) {
  switch (status) {
    case SIP_OK: return "ok";
    case SIP_ERR_INVALID_ARG: return "invalid argument";
    case SIP_ERR_UNSUPPORTED: return "unsupported shape";
    case SIP_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case SIP_ERR_HIP: return "HIP runtime error";
  }
  return "unknown status";
}

int sip_version(void) { return 100; }

}  // extern "C"
