// Host side of the C boundary declared in include/sip.h: argument checks, workspace
// carving and kernel launches.  No allocation, no synchronisation.
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <algorithm>
#include <atomic>

#include "../../include/sip.h"
#include "sip_device.h"
#include "sip_exact.h"
#include "sip_final.h"
#include "sip_stream.h"

namespace {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

// Launch shape of the single-pass path; a function of (B, V, dtype) only.
struct Plan {
  bool fast;       // false: vocabulary outside what the single-pass kernels are built for
  int S, cap_w, nc_cap;
  size_t final_lds;
};

constexpr int kFastMinV = 16384;
constexpr int kFastMaxV = 262144;

Plan make_plan(int32_t B, int32_t V, int dtype) {
  Plan p{};
  p.fast = V >= kFastMinV && V <= kFastMaxV;
  if (!p.fast) return p;
  const int tile = sip::kStreamThreads * sip::kStreamLoads * (dtype == SIP_F32 ? 4 : 8);
  const int n_tiles = (V + tile - 1) / tile;
  // Chunks per row.  Small batches: as many workgroups as fit on the chip at once (4 per compute
  // unit), so that there is a single, full round.  Large batches: 4, which makes many rounds
  // and lets the per-wave candidate queues (kQueueCap each) add up to 16K entries per row.
  constexpr int kResident = 256 * 4;
  int want = B * 4 <= kResident ? kResident / B : (B * 2 <= kResident ? kResident / B : 4);
  want = std::max(1, std::min({want, sip::kMaxChunks, std::max(1, n_tiles / 2)}));
  p.S = want;                                          // <= n_tiles / 2: every chunk holds at least two tiles
  p.cap_w = sip::kQueueCap;
  p.nc_cap = sip::kFinalThreads * sip::kCandLong;     // the finishing kernel holds the list in registers
  p.final_lds = sip::final_lds_fixed(V);
  return p;
}

struct Layout {
  size_t row_path, side_z, side_c, chunks, cand, total;
};

thread_local hipEvent_t g_prof[4] = {nullptr, nullptr, nullptr, nullptr};   // one-shot, see sip_profile_kernel_events()

// Kernels that use more than the default 64 KB of dynamic LDS have to be told so once.
constexpr int kMaxDynLds = 144 * 1024;
bool allow_big_lds(const void* kernel, int slot) {
  static std::atomic<bool> done[4];
  if (done[slot].load(std::memory_order_acquire)) return true;
  if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, kMaxDynLds) != hipSuccess) {
    (void)hipGetLastError();
    return false;
  }
  done[slot].store(true, std::memory_order_release);
  return true;
}

bool shape_ok(int32_t B, int32_t V, int dtype, int64_t nnz, int32_t k_lp) {
  return B > 0 && V > 0 && (dtype == SIP_F32 || dtype == SIP_BF16) && nnz >= 0 && k_lp >= -1;
}

Layout make_layout(int32_t B, const Plan& p, int64_t nnz) {
  Layout l;
  size_t off = 0;
  l.row_path = off; off += align_up((size_t)B * sizeof(int) + 8 + 64 * 8);   // first, so that callers can find it
  l.side_z = off; off += align_up((size_t)nnz * sizeof(float));
  l.side_c = off; off += align_up((size_t)nnz * sizeof(unsigned int));
  l.chunks = off;
  if (p.fast) off += align_up((size_t)B * p.S * sizeof(sip::ChunkOut));
  l.cand = off;
  if (p.fast) off += align_up((size_t)B * p.S * sip::kStreamWaves * (size_t)p.cap_w * sizeof(uint2));
  l.total = off ? off : kAlign;
  return l;
}

}  // namespace

extern "C" {

size_t sip_workspace_bytes(int32_t B, int32_t V, sip_dtype dtype, int64_t hist_nnz, int32_t k_logprobs) {
  if (!shape_ok(B, V, (int)dtype, hist_nnz, k_logprobs)) return 0;
  if (V > SIP_MAX_V || k_logprobs > SIP_MAX_K_LOGPROBS) return 0;
  return make_layout(B, make_plan(B, V, (int)dtype), hist_nnz).total;
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
  const Plan plan = make_plan(B, V, (int)dtype);
  const Layout lay = make_layout(B, plan, hist_nnz);
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
  a.row_path = reinterpret_cast<int*>(ws + lay.row_path);
  a.side_z = reinterpret_cast<float*>(ws + lay.side_z);
  a.side_c = reinterpret_cast<unsigned int*>(ws + lay.side_c);
  a.chunks = reinterpret_cast<sip::ChunkOut*>(ws + lay.chunks);
  a.cand = reinterpret_cast<uint2*>(ws + lay.cand);
  a.S = plan.S; a.cap_w = plan.cap_w; a.nc_cap = plan.nc_cap;

  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const size_t words = ((size_t)V + 31) / 32;
  if (!plan.fast) {
    // every row takes the exact multi-pass path
    const size_t dyn = 2 * words * sizeof(uint32_t);
    auto kern = dtype == SIP_F32 ? sip::exact_kernel<SIP_F32> : sip::exact_kernel<SIP_BF16>;
    if (!allow_big_lds(reinterpret_cast<const void*>(kern), dtype == SIP_F32 ? 0 : 1)) return SIP_ERR_HIP;
    hipLaunchKernelGGL(kern, dim3(B), dim3(sip::kExactThreads), dyn, stream, a);
    if (hipGetLastError() != hipSuccess) return SIP_ERR_HIP;
    return SIP_OK;
  }
  auto k_stream = dtype == SIP_F32 ? sip::stream_kernel<SIP_F32> : sip::stream_kernel<SIP_BF16>;
  auto k_final = dtype == SIP_F32 ? sip::final_kernel<SIP_F32> : sip::final_kernel<SIP_BF16>;
  const size_t dyn = std::max(plan.final_lds, 2 * words * sizeof(uint32_t));
  if (!allow_big_lds(reinterpret_cast<const void*>(k_final), dtype == SIP_F32 ? 2 : 3)) return SIP_ERR_HIP;
  hipEvent_t ev[4];
  for (int i = 0; i < 4; ++i) { ev[i] = g_prof[i]; g_prof[i] = nullptr; }
  if (ev[0] || ev[1])       // the events take the dispatch's own begin / end time stamps
    hipExtLaunchKernelGGL(k_stream, dim3(B * plan.S), dim3(sip::kStreamThreads), 0, stream, ev[0], ev[1], 0, a);
  else
    hipLaunchKernelGGL(k_stream, dim3(B * plan.S), dim3(sip::kStreamThreads), 0, stream, a);
  if (hipGetLastError() != hipSuccess) return SIP_ERR_HIP;
  if (ev[2] || ev[3])
    hipExtLaunchKernelGGL(k_final, dim3(B), dim3(sip::kFinalThreads), dyn, stream, ev[2], ev[3], 0, a);
  else
    hipLaunchKernelGGL(k_final, dim3(B), dim3(sip::kFinalThreads), dyn, stream, a);
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

void sip_profile_kernel_events(void* stream_start, void* stream_stop, void* final_start, void* final_stop) {
  g_prof[0] = static_cast<hipEvent_t>(stream_start);
  g_prof[1] = static_cast<hipEvent_t>(stream_stop);
  g_prof[2] = static_cast<hipEvent_t>(final_start);
  g_prof[3] = static_cast<hipEvent_t>(final_stop);
}

int sip_version(void) { return 100; }

}  // extern "C"
