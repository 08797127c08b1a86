// Host side of the C boundary declared in include/sip.h: argument checks, workspace
// carving and kernel launches.  No allocation, no synchronisation.
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <algorithm>
#include <cmath>
#include <atomic>
#include <chrono>
#include <mutex>

#include "../../include/sip.h"
#include "../../include/sip_diag.h"
#include "sip_device.h"
#include "sip_exact.h"
#include "sip_final.h"
#include "sip_finish.h"
#include "sip_fused.h"
#include "sip_handoff.h"
#include "sip_state.h"
#include "sip_stream.h"

namespace {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

// Launch shape of the single-pass path; a function of (B, V, dtype) only.
struct Plan {
  bool fast;       // false: vocabulary outside what the single-pass kernels are built for
  int S, cap_c, nc_cap;
  size_t final_lds;
};

constexpr int kFastMinV = 16384;
constexpr int kFastMaxV = 262144;
constexpr int kFastMinPiece = 8192;      // smallest vocabulary shard: its sample blocks (at most 32 of 256 elements) must fit

// `t` > 0: the logits come in t vocabulary shards of V / t elements (0: one piece).
Plan make_plan(int32_t B, int32_t V, int dtype, int t = 0) {
  Plan p{};
  const int pieces = t > 0 ? t : 1;
  const int Vp = V / pieces;                           // elements per piece
  p.fast = V >= kFastMinV && V <= kFastMaxV && Vp >= kFastMinPiece && pieces <= sip::kMaxChunks;
  if (!p.fast) return p;
  const int tile = sip::kStreamThreads * sip::kStreamLoads * (dtype == SIP_F32 ? 4 : 8);
  const int n_tiles = (Vp + tile - 1) / tile * pieces;
  // Chunks per row.  Up to 256 rows: as many workgroups as fit on the chip at once (4 per compute
  // unit), so that there is a single, full round.  Larger batches run in rounds of that many
  // workgroups, and every workgroup pays a fixed set-up (sample, threshold, history bitmap: about
  // what streaming 38 elements per lane costs) before it streams its V / (S * 512) elements per
  // lane: take the S with the cheapest rounds x (set-up + stream).
  constexpr int kResident = 256 * 4;
  int want;
  if (B * 4 <= kResident) {
    want = kResident / B;
  } else {
    // (from 2 on: one chunk's queues alone are short for a long list plus a long history)
    double best_cost = 0.0;
    want = 2;
    for (int S = 2; S <= sip::kMaxChunks; ++S) {
      const double rounds = std::ceil((double)B * S / kResident);
      const double cost = rounds * (38.0 + (double)V / (S * (double)sip::kStreamThreads));
      if (S == 2 || cost < best_cost) { best_cost = cost; want = S; }
    }
  }
  want = std::max(1, std::min({want, sip::kMaxChunks, std::max(1, n_tiles / 2)}));
  if (want >= pieces) {
    want = want / pieces * pieces;                     // a chunk is part of one piece: a multiple of their number
  } else {
    // a chunk is several whole pieces: the divisor of their number nearest to `want` (by ratio)
    int best = pieces;
    for (int dv = 1; dv <= pieces; ++dv)
      if (pieces % dv == 0) {
        const double r0 = std::fabs(std::log((double)best / want)), r1 = std::fabs(std::log((double)dv / want));
        if (r1 < r0 || (r1 == r0 && dv > best)) best = dv;
      }
    want = best;
  }
  // the streaming kernel marks a chunk's history tokens in an LDS bitmap of kChunkBitsMax bits:
  // cut finer (first at the piece boundaries, then inside the pieces) until a chunk fits
  {
    const int unit = sip::kWave * (dtype == SIP_F32 ? 4 : 8);
    const int n_units = (Vp + unit - 1) / unit;
    auto max_chunk = [&](int S) {
      return S >= pieces ? (n_units + S / pieces - 1) / (S / pieces) * unit : pieces / S * Vp;
    };
    while (max_chunk(want) > sip::kChunkBitsMax) {
      const int next = want >= pieces ? want + pieces : pieces;
      if (next > sip::kMaxChunks) { p.fast = false; return p; }
      want = next;
    }
  }
  p.S = want;                                          // <= n_tiles / 2: every chunk holds at least two tiles
  p.cap_c = sip::kChunkCap;
  // the longest list a row may have: what the heavier per-row logic holds in registers, and what
  // the row's chunks can hand over
  p.nc_cap = std::min(sip::kFinalThreads * sip::kCandLong, p.S * sip::kChunkCap);
  p.final_lds = sip::final_lds_fixed(V);
  return p;
}

struct Layout {
  size_t row_path, rescue, side_z, side_c, rowinfo, chunks, cand, gather, total;
};

thread_local hipEvent_t g_prof[6] = {nullptr, nullptr, nullptr, nullptr, nullptr, nullptr};   // one-shot, see sip_profile_kernel_events()

// Kernels that use more than the default 64 KB of dynamic LDS have to be told so once per device.
constexpr int kMaxDynLds = 144 * 1024;
constexpr int kMaxDevices = 64;
constexpr int kRescueGrid = 256;         // workgroups of the rescue kernel (one per compute unit)

// Built-in scratch of sip_sample_noalloc(): one copy per device, at that device's own address.
// In host code the name below is only a handle for hipGetSymbolAddress; the address the kernels
// get is the one looked up in device_setup().
constexpr size_t kNoallocBytes = (size_t)40 << 20;     // holds a call of 256 rows at V = 152064 (33.6 MB)
static __device__ __align__(256) unsigned char scratch[kNoallocBytes];

struct DeviceSetup {
  std::atomic<int> state{0};                // 0: not done, 1: done
  void* scratch_ptr = nullptr;
  int compute_units = 0;
};
DeviceSetup g_dev[kMaxDevices];
std::mutex g_dev_mutex;

// Per-device set-up (see sip_init in the header).  Returns the device's entry, or nullptr.
DeviceSetup* device_setup() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) { (void)hipGetLastError(); return nullptr; }
  DeviceSetup& d = g_dev[dev];
  if (d.state.load(std::memory_order_acquire) == 1) return &d;
  std::lock_guard<std::mutex> lock(g_dev_mutex);
  if (d.state.load(std::memory_order_acquire) == 1) return &d;
  const void* big[] = {
      reinterpret_cast<const void*>(sip::exact_kernel<SIP_F32, false>), reinterpret_cast<const void*>(sip::exact_kernel<SIP_BF16, false>),
      reinterpret_cast<const void*>(sip::exact_kernel<SIP_F32, true>),  reinterpret_cast<const void*>(sip::exact_kernel<SIP_BF16, true>),
      reinterpret_cast<const void*>(sip::rescue_kernel<SIP_F32, false>), reinterpret_cast<const void*>(sip::rescue_kernel<SIP_BF16, false>),
      reinterpret_cast<const void*>(sip::rescue_kernel<SIP_F32, true>),  reinterpret_cast<const void*>(sip::rescue_kernel<SIP_BF16, true>)};
  for (const void* k : big)
    if (hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, kMaxDynLds) != hipSuccess) {
      (void)hipGetLastError();
      return nullptr;
    }
  void* p = nullptr;
  if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) { (void)hipGetLastError(); return nullptr; }
  d.scratch_ptr = p;
  if (hipDeviceGetAttribute(&d.compute_units, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) {
    (void)hipGetLastError();
    d.compute_units = 0;
  }
  d.state.store(1, std::memory_order_release);
  return &d;
}

bool shape_ok(int32_t B, int32_t V, int dtype, int64_t nnz, int32_t k_lp) {
  return B > 0 && V > 0 && (dtype == SIP_F32 || dtype == SIP_BF16) && nnz >= 0 && k_lp >= -1;
}

// `gather_row_bytes` > 0 (sharded logits): room for B whole rows.
Layout make_layout(int32_t B, const Plan& p, int64_t nnz, size_t gather_row_bytes = 0) {
  Layout l;
  size_t off = 0;
  l.row_path = off; off += align_up((size_t)2 * B * sizeof(int));            // first, so that callers can find it: path
                                                                             // codes, then the finishing kernel's own codes
  l.rescue = off; off += align_up(((size_t)B + 1) * sizeof(int) + 16);       // count, row numbers, the state's call counter
  l.side_z = off; off += align_up((size_t)nnz * sizeof(float));
  l.side_c = off; off += align_up((size_t)nnz * sizeof(unsigned int));
  l.rowinfo = off;
  if (p.fast) off += align_up((size_t)B * sizeof(sip::RowInfo));
  l.chunks = off;
  if (p.fast) off += align_up((size_t)B * p.S * sizeof(sip::ChunkOut));
  l.cand = off;
  if (p.fast) off += align_up((size_t)B * p.S * (size_t)p.cap_c * sizeof(uint2));
  l.gather = off; off += align_up((size_t)B * gather_row_bytes);
  l.total = off ? off : kAlign;
  return l;
}

// Where a call's token histories come from: a CSR handed in by the caller, or the slots of a
// device-resident state.
struct HistSource {
  const int64_t* indptr = nullptr;
  const int32_t* tokens = nullptr;
  int64_t nnz = 0;                                   // entries the side tables of the workspace are sized for
  const int64_t* p_indptr = nullptr;                 // separate prompt tokens (CSR), or none
  const int32_t* p_tokens = nullptr;
  int64_t p_nnz = 0;
  const int32_t* slot = nullptr;
  sip::StateView state{};                            // valid when slot != nullptr
  int L_max = 0, slots = 0;
};

// Vocabulary shards of a call (sip_sample_sharded); t == 0: the logits are one matrix.
struct ShardSource {
  const void* const* base = nullptr;                 // host array of t device pointers
  int t = 0, V_shard = 0;
  int64_t stride = 0;
};

template <bool SH>
sip_status launch(const sip::Args& a, int32_t B, int dtype, const Plan& plan, bool state, sip::StateHeader* head,
                  hipStream_t stream);

// Argument checks common to the entry points, workspace carving and the kernel launches.
sip_status sample_impl(const void* logits, int32_t B, int32_t V, int64_t row_stride, sip_dtype dtype,
                       const sip_params* params, const HistSource& h, uint64_t seed, uint64_t step,
                       int32_t* out_ids, int32_t* out_lp_ids, float* out_lp, int32_t k_logprobs, void* workspace,
                       size_t workspace_bytes, hipStream_t stream, const ShardSource& sh = ShardSource{}) {
  if (!shape_ok(B, V, (int)dtype, h.nnz, k_logprobs) || h.p_nnz < 0) return SIP_ERR_INVALID_ARG;
  if (!out_ids) return SIP_ERR_INVALID_ARG;
  if ((k_logprobs >= 0) != (out_lp_ids != nullptr) || (k_logprobs >= 0) != (out_lp != nullptr))
    return SIP_ERR_INVALID_ARG;
  const size_t esz = dtype == SIP_F32 ? 4 : 2;
  if (sh.t == 0) {
    if (!logits || row_stride < V) return SIP_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(logits) & 15u) != 0 || ((size_t)row_stride * esz) % 16 != 0)
      return SIP_ERR_INVALID_ARG;
  } else {
    if (!sh.base || sh.stride < sh.V_shard) return SIP_ERR_INVALID_ARG;
    if (((size_t)sh.V_shard * esz) % 16 != 0 || ((size_t)sh.stride * esz) % 16 != 0) return SIP_ERR_INVALID_ARG;
    for (int i = 0; i < sh.t; ++i)
      if (!sh.base[i] || (reinterpret_cast<uintptr_t>(sh.base[i]) & 15u) != 0) return SIP_ERR_INVALID_ARG;
  }
  if (B > SIP_MAX_B || V > SIP_MAX_V || k_logprobs > SIP_MAX_K_LOGPROBS) return SIP_ERR_UNSUPPORTED;
  const Plan plan = make_plan(B, V, (int)dtype, sh.t);
  const Layout lay = make_layout(B, plan, h.nnz + h.p_nnz, sh.t ? (size_t)V * esz : 0);
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & (kAlign - 1)) != 0 || workspace_bytes < lay.total)
    return SIP_ERR_WORKSPACE;

  sip::Args a;
  a.logits = logits;
  a.B = B; a.V = V; a.row_stride = row_stride;
  for (int i = 0; i < 8; ++i) a.shard[i] = nullptr;
  a.t_shards = 1; a.V_shard = V; a.shard_stride = row_stride;
  if (sh.t) {
    // whole-row code paths read the row from the workspace, where its workgroup puts it together first
    a.logits = static_cast<char*>(workspace) + lay.gather;
    a.row_stride = V;
    for (int i = 0; i < sh.t; ++i) a.shard[i] = sh.base[i];
    a.t_shards = sh.t; a.V_shard = sh.V_shard; a.shard_stride = sh.stride;
  }
  a.inv_V_shard = 1.0f / (float)a.V_shard;
  {
    const int epl = dtype == SIP_F32 ? 4 : 8, unit = sip::kWave * epl;
    const int nsb = sip::kSampleSize / (sip::kStreamThreads * epl) * sip::kStreamWaves;   // sample blocks per row
    a.smp_bps = (nsb + a.t_shards - 1) / a.t_shards;
    a.smp_inv = (65536 + a.smp_bps - 1) / a.smp_bps;
    a.smp_step = a.V_shard / a.smp_bps / unit * unit;
  }
  if (params) a.p = *params; else a.p = sip_params{};
  a.indptr = reinterpret_cast<const long long*>(h.indptr);
  a.tokens = h.tokens;
  a.nnz = h.slot ? (long long)h.slots * h.L_max : ((h.indptr && h.tokens) ? h.nnz : 0);
  a.p_indptr = reinterpret_cast<const long long*>(h.p_indptr);
  a.p_tokens = h.p_tokens;
  a.p_nnz = (h.p_indptr && h.p_tokens) ? h.p_nnz : 0;
  a.slot = h.slot; a.L_max = h.L_max; a.slots = h.slots;
  a.st_len = h.state.len; a.st_ndist = h.state.ndist; a.st_tokens = h.state.tokens; a.st_table = h.state.table;
  a.st_tick = h.slot ? &h.state.head->tick : nullptr;
  a.st_overflow = h.slot ? &h.state.head->overflow : nullptr;
  a.call_tick = nullptr;
  a.seed = seed; a.step = step;
  a.out_ids = out_ids; a.out_lp_ids = out_lp_ids; a.out_lp = out_lp; a.k_lp = k_logprobs;
  char* ws = static_cast<char*>(workspace);
  a.row_path = reinterpret_cast<int*>(ws + lay.row_path);
  a.side_z = reinterpret_cast<float*>(ws + lay.side_z);
  a.side_c = reinterpret_cast<unsigned int*>(ws + lay.side_c);
  a.rowinfo = reinterpret_cast<sip::RowInfo*>(ws + lay.rowinfo);
  a.fin_tps = plan.fast ? sip::kFinThreads / plan.S : sip::kFinThreads;
  a.fin_inv = (65536 + a.fin_tps - 1) / a.fin_tps;
  a.chunks = reinterpret_cast<sip::ChunkOut*>(ws + lay.chunks);
  a.cand = reinterpret_cast<uint2*>(ws + lay.cand);
  a.S = plan.S; a.cap_c = plan.cap_c; a.nc_cap = plan.nc_cap;
  a.row_why = a.row_path + B;
  a.rescue_n = reinterpret_cast<int*>(ws + lay.rescue);
  a.rescue_rows = a.rescue_n + 1;
  a.rescue_tick = reinterpret_cast<unsigned long long*>(ws + lay.rescue + (((size_t)B + 1) * sizeof(int) + 7) / 8 * 8);

  sip::StateHeader* head = h.slot ? h.state.head : nullptr;
  return sh.t ? launch<true>(a, B, (int)dtype, plan, h.slot != nullptr, head, stream)
              : launch<false>(a, B, (int)dtype, plan, h.slot != nullptr, head, stream);
}

template <bool SH>
sip_status launch(const sip::Args& a_in, int32_t B, int dtype, const Plan& plan, bool state, sip::StateHeader* head,
                  hipStream_t stream) {
  const DeviceSetup* dev = device_setup();
  if (!dev) return SIP_ERR_HIP;
  sip::Args a = a_in;
  const size_t words = ((size_t)a.V + 31) / 32;
  if (!plan.fast) {
    // every row takes the exact multi-pass path
    const size_t dyn = 2 * words * sizeof(uint32_t);
    auto kern = dtype == SIP_F32 ? sip::exact_kernel<SIP_F32, SH> : sip::exact_kernel<SIP_BF16, SH>;
    hipLaunchKernelGGL(kern, dim3(B), dim3(sip::kExactThreads), dyn, stream, a);
    if (hipGetLastError() != hipSuccess) return SIP_ERR_HIP;
    if (state) {
      hipLaunchKernelGGL(sip::state_tick_kernel, dim3(1), dim3(64), 0, stream, head);
      if (hipGetLastError() != hipSuccess) return SIP_ERR_HIP;
    }
    return SIP_OK;
  }
  a.call_tick = state ? a.rescue_tick : nullptr;   // the streaming kernel takes the state's counter and leaves it here
  auto k_stream = dtype == SIP_F32 ? sip::stream_kernel<SIP_F32, SH> : sip::stream_kernel<SIP_BF16, SH>;
  auto k_rescue = dtype == SIP_F32 ? sip::rescue_kernel<SIP_F32, SH> : sip::rescue_kernel<SIP_BF16, SH>;
  const size_t dyn = std::max(plan.final_lds, 2 * words * sizeof(uint32_t));
  hipEvent_t ev[6];
  for (int i = 0; i < 6; ++i) { ev[i] = g_prof[i]; g_prof[i] = nullptr; }
  const bool timed = ev[0] || ev[1] || ev[2] || ev[3] || ev[4] || ev[5];
  // The pass over the logits, then one workgroup per row on what it left.  A batch of no more rows
  // than the device has compute units: the workgroup also takes its row through the heavier logic
  // if the list does not settle it (sip_fused.h).  Larger batches: the lean finishing kernel, two
  // workgroups per compute unit, and a small fixed grid behind it for the rows (normally none) that
  // need more.
  const bool fused = B <= dev->compute_units && (size_t)plan.final_lds <= sip::kFusedRawBytes &&
                     2 * words * sizeof(uint32_t) <= sip::kFusedRawBytes;
  if (timed) hipExtLaunchKernelGGL(k_stream, dim3(B * plan.S), dim3(sip::kStreamThreads), 0, stream, ev[0], ev[1], 0, a);
  else hipLaunchKernelGGL(k_stream, dim3(B * plan.S), dim3(sip::kStreamThreads), 0, stream, a);
  if (fused) {
    auto k_fused = dtype == SIP_F32 ? sip::finish_rescue_kernel<SIP_F32, SH> : sip::finish_rescue_kernel<SIP_BF16, SH>;
    if (timed) {             // the events take the dispatches' own begin / end time stamps
      hipExtLaunchKernelGGL(k_fused, dim3(B), dim3(sip::kFinalThreads), 0, stream, ev[2], ev[3], 0, a);
      if (ev[4]) (void)hipEventRecord(ev[4], stream);       // no third kernel: an empty interval
      if (ev[5]) (void)hipEventRecord(ev[5], stream);
    } else {
      hipLaunchKernelGGL(k_fused, dim3(B), dim3(sip::kFinalThreads), 0, stream, a);
    }
  } else {
    const int n_rescue_wg = std::min<int>(B, kRescueGrid);
    if (timed) {
      hipExtLaunchKernelGGL(sip::finish_kernel, dim3(B), dim3(sip::kFinThreads), 0, stream, ev[2], ev[3], 0, a);
      hipExtLaunchKernelGGL(k_rescue, dim3(n_rescue_wg), dim3(sip::kFinalThreads), dyn, stream, ev[4], ev[5], 0, a);
    } else {
      hipLaunchKernelGGL(sip::finish_kernel, dim3(B), dim3(sip::kFinThreads), 0, stream, a);
      hipLaunchKernelGGL(k_rescue, dim3(n_rescue_wg), dim3(sip::kFinalThreads), dyn, stream, a);
    }
  }
  if (hipGetLastError() != hipSuccess) return SIP_ERR_HIP;
  return SIP_OK;
}

bool state_shape_ok(int32_t slots, int32_t L_max) {
  return slots > 0 && L_max > 0 && slots <= SIP_MAX_SLOTS && L_max <= SIP_MAX_L;
}
bool state_ok(const void* state, size_t state_bytes, int32_t slots, int32_t L_max) {
  return state && (reinterpret_cast<uintptr_t>(state) & (kAlign - 1)) == 0 &&
         state_bytes >= sip::state_total(slots, L_max);
}

}  // namespace

extern "C" {

size_t sip_workspace_bytes(int32_t B, int32_t V, sip_dtype dtype, int64_t hist_nnz, int32_t k_logprobs) {
  if (!shape_ok(B, V, (int)dtype, hist_nnz, k_logprobs)) return 0;
  if (B > SIP_MAX_B || V > SIP_MAX_V || k_logprobs > SIP_MAX_K_LOGPROBS) return 0;
  return make_layout(B, make_plan(B, V, (int)dtype), hist_nnz).total;
}

sip_status sip_sample(const void* logits, int32_t B, int32_t V, int64_t row_stride, sip_dtype dtype,
                      const sip_params* params, const int64_t* hist_indptr, const int32_t* hist_tokens,
                      int64_t hist_nnz, uint64_t seed, uint64_t step, int32_t* out_ids, int32_t* out_lp_ids,
                      float* out_lp, int32_t k_logprobs, void* workspace, size_t workspace_bytes,
                      void* hip_stream) {
  if (hist_nnz > 0 && (!hist_indptr || !hist_tokens)) return SIP_ERR_INVALID_ARG;
  HistSource h;
  h.indptr = hist_indptr; h.tokens = hist_tokens; h.nnz = hist_nnz;
  return sample_impl(logits, B, V, row_stride, dtype, params, h, seed, step, out_ids, out_lp_ids, out_lp,
                     k_logprobs, workspace, workspace_bytes, static_cast<hipStream_t>(hip_stream));
}

sip_status sip_init(void) { return device_setup() ? SIP_OK : SIP_ERR_HIP; }

size_t sip_noalloc_scratch_bytes(void) { return kNoallocBytes; }

sip_status sip_sample_noalloc(const void* logits, int32_t B, int32_t V, int64_t row_stride, sip_dtype dtype,
                              const sip_params* params, const int64_t* hist_indptr, const int32_t* hist_tokens,
                              int64_t hist_nnz, uint64_t seed, uint64_t step, int32_t* out_ids,
                              int32_t* out_lp_ids, float* out_lp, int32_t k_logprobs, void* hip_stream) {
  if (!logits || !out_ids) return SIP_ERR_INVALID_ARG;     // (the rest is checked by sample_impl, before anything is enqueued)
  if (hist_nnz > 0 && (!hist_indptr || !hist_tokens)) return SIP_ERR_INVALID_ARG;
  if (!shape_ok(B, V, (int)dtype, hist_nnz, k_logprobs)) return SIP_ERR_INVALID_ARG;
  if (B > SIP_MAX_B || V > SIP_MAX_V || k_logprobs > SIP_MAX_K_LOGPROBS) return SIP_ERR_UNSUPPORTED;
  const size_t need = make_layout(B, make_plan(B, V, (int)dtype), hist_nnz).total;
  if (need > kNoallocBytes) return SIP_ERR_SCRATCH;
  DeviceSetup* d = device_setup();                 // the current device's copy of the array
  if (!d) return SIP_ERR_HIP;
  // Nothing in the workspace has to start at zero: every kernel writes what it later reads.
  HistSource h;
  h.indptr = hist_indptr; h.tokens = hist_tokens; h.nnz = hist_nnz;
  return sample_impl(logits, B, V, row_stride, dtype, params, h, seed, step, out_ids, out_lp_ids, out_lp,
                     k_logprobs, d->scratch_ptr, kNoallocBytes, static_cast<hipStream_t>(hip_stream));
}

size_t sip_workspace_bytes_sharded(int32_t B, int32_t V_shard, int32_t t, sip_dtype dtype, int64_t hist_nnz,
                                   int32_t k_logprobs) {
  if (t < 1 || t > SIP_MAX_SHARDS || V_shard <= 0 || (int64_t)V_shard * t > SIP_MAX_V || B > SIP_MAX_B) return 0;
  const int32_t V = V_shard * t;
  if (!shape_ok(B, V, (int)dtype, hist_nnz, k_logprobs) || k_logprobs > SIP_MAX_K_LOGPROBS) return 0;
  return make_layout(B, make_plan(B, V, (int)dtype, t), hist_nnz, (size_t)V * (dtype == SIP_F32 ? 4 : 2)).total;
}

sip_status sip_sample_sharded(const void* const* shard_logits, int32_t t, int32_t B, int32_t V_shard,
                              int64_t shard_stride, sip_dtype dtype, const sip_params* params,
                              const int64_t* hist_indptr, const int32_t* hist_tokens, int64_t hist_nnz,
                              uint64_t seed, uint64_t step, int32_t* out_ids, int32_t* out_lp_ids, float* out_lp,
                              int32_t k_logprobs, void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (t < 1 || t > SIP_MAX_SHARDS || V_shard <= 0 || !shard_logits) return SIP_ERR_INVALID_ARG;
  if ((int64_t)V_shard * t > SIP_MAX_V || B > SIP_MAX_B) return SIP_ERR_UNSUPPORTED;
  if (hist_nnz > 0 && (!hist_indptr || !hist_tokens)) return SIP_ERR_INVALID_ARG;
  HistSource h;
  h.indptr = hist_indptr; h.tokens = hist_tokens; h.nnz = hist_nnz;
  ShardSource sh;
  sh.base = shard_logits; sh.t = t; sh.V_shard = V_shard; sh.stride = shard_stride;
  return sample_impl(nullptr, B, V_shard * t, 0, dtype, params, h, seed, step, out_ids, out_lp_ids, out_lp,
                     k_logprobs, workspace, workspace_bytes, static_cast<hipStream_t>(hip_stream), sh);
}

size_t sip_state_bytes(int32_t slots, int32_t L_max) {
  if (!state_shape_ok(slots, L_max)) return 0;
  return sip::state_total(slots, L_max);
}

sip_status sip_state_init(void* state, size_t state_bytes, int32_t slots, int32_t L_max, void* hip_stream) {
  if (!state_shape_ok(slots, L_max)) return SIP_ERR_INVALID_ARG;
  if (!state_ok(state, state_bytes, slots, L_max)) return SIP_ERR_WORKSPACE;
  const sip::StateView v = sip::state_view(state, slots, L_max);
  hipLaunchKernelGGL(sip::state_init_kernel, dim3(slots), dim3(sip::kStateThreads), 0,
                     static_cast<hipStream_t>(hip_stream), v.head, v.len, v.ndist, v.table, slots);
  return hipGetLastError() == hipSuccess ? SIP_OK : SIP_ERR_HIP;
}

sip_status sip_state_assign(void* state, size_t state_bytes, int32_t slots, int32_t L_max, int32_t n,
                            const int32_t* slot_ids, const int64_t* indptr, const int32_t* tokens, int64_t nnz,
                            void* hip_stream) {
  if (!state_shape_ok(slots, L_max) || n < 0 || nnz < 0) return SIP_ERR_INVALID_ARG;
  if (n > 0 && !slot_ids) return SIP_ERR_INVALID_ARG;
  if (nnz > 0 && (!indptr || !tokens)) return SIP_ERR_INVALID_ARG;
  if (!state_ok(state, state_bytes, slots, L_max)) return SIP_ERR_WORKSPACE;
  if (n == 0) return SIP_OK;
  const sip::StateView v = sip::state_view(state, slots, L_max);
  hipLaunchKernelGGL(sip::state_assign_kernel, dim3(n), dim3(sip::kStateThreads), 0,
                     static_cast<hipStream_t>(hip_stream), v.head, v.len, v.ndist, v.tokens, v.table, slots, L_max, slot_ids,
                     reinterpret_cast<const long long*>(indptr), tokens, (long long)nnz);
  return hipGetLastError() == hipSuccess ? SIP_OK : SIP_ERR_HIP;
}

sip_status sip_sample_state(const void* logits, int32_t B, int32_t V, int64_t row_stride, sip_dtype dtype,
                            const sip_params* params, void* state, size_t state_bytes, int32_t slots,
                            int32_t L_max, const int32_t* slot_of_row, uint64_t seed, uint64_t step,
                            int32_t* out_ids, int32_t* out_lp_ids, float* out_lp, int32_t k_logprobs,
                            void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!state_shape_ok(slots, L_max) || !slot_of_row || B <= 0) return SIP_ERR_INVALID_ARG;
  if (!state_ok(state, state_bytes, slots, L_max)) return SIP_ERR_WORKSPACE;
  HistSource h;
  h.state = sip::state_view(state, slots, L_max);
  h.tokens = h.state.tokens; h.nnz = (int64_t)B * L_max;
  h.slot = slot_of_row; h.L_max = L_max; h.slots = slots;
  // the kernels append the ids to the slots and count the call themselves
  return sample_impl(logits, B, V, row_stride, dtype, params, h, seed, step, out_ids, out_lp_ids, out_lp,
                     k_logprobs, workspace, workspace_bytes, static_cast<hipStream_t>(hip_stream));
}

namespace {
// Checks of a sip_call that sample_impl does not make, and its two sources.
sip_status call_sources(const sip_call* c, HistSource& h, ShardSource& sh, int32_t& V) {
  if (!c || c->B <= 0) return SIP_ERR_INVALID_ARG;
  if (c->t_shards < 0 || c->t_shards > SIP_MAX_SHARDS) return SIP_ERR_INVALID_ARG;
  if (c->t_shards > 0) {
    if (c->V_shard <= 0 || !c->shard_logits) return SIP_ERR_INVALID_ARG;
    if ((int64_t)c->V_shard * c->t_shards > SIP_MAX_V || c->B > SIP_MAX_B) return SIP_ERR_UNSUPPORTED;
    sh.base = c->shard_logits; sh.t = c->t_shards; sh.V_shard = c->V_shard; sh.stride = c->shard_stride;
    V = c->V_shard * c->t_shards;
  } else {
    V = c->V;
  }
  if (c->state) {
    if (c->hist_indptr || c->hist_tokens || c->hist_nnz != 0) return SIP_ERR_INVALID_ARG;   // one source of history
    if (!state_shape_ok(c->slots, c->L_max) || !c->slot_of_row) return SIP_ERR_INVALID_ARG;
    if (!state_ok(c->state, c->state_bytes, c->slots, c->L_max)) return SIP_ERR_WORKSPACE;
    h.state = sip::state_view(c->state, c->slots, c->L_max);
    h.tokens = h.state.tokens; h.nnz = (int64_t)c->B * c->L_max;
    h.slot = c->slot_of_row; h.L_max = c->L_max; h.slots = c->slots;
  } else {
    if (c->hist_nnz < 0 || (c->hist_nnz > 0 && (!c->hist_indptr || !c->hist_tokens))) return SIP_ERR_INVALID_ARG;
    h.indptr = c->hist_indptr; h.tokens = c->hist_tokens; h.nnz = c->hist_nnz;
  }
  if (c->prompt_nnz < 0 || (c->prompt_nnz > 0 && (!c->prompt_indptr || !c->prompt_tokens))) return SIP_ERR_INVALID_ARG;
  if (c->prompt_nnz > 0 && c->state) return SIP_ERR_INVALID_ARG;      // a state's slots hold prompt and output as one history
  h.p_indptr = c->prompt_indptr; h.p_tokens = c->prompt_tokens; h.p_nnz = c->prompt_nnz;
  if ((c->host_ids != nullptr) != (c->host_flag != nullptr)) return SIP_ERR_INVALID_ARG;
  if (c->host_flag && ((reinterpret_cast<uintptr_t>(c->host_flag) & 7u) != 0 ||
                       (reinterpret_cast<uintptr_t>(c->host_ids) & 3u) != 0))
    return SIP_ERR_INVALID_ARG;
  return SIP_OK;
}
}  // namespace

size_t sip_call_workspace_bytes(const sip_call* c) {
  HistSource h; ShardSource sh; int32_t V = 0;
  if (call_sources(c, h, sh, V) != SIP_OK) return 0;
  if (!shape_ok(c->B, V, (int)c->dtype, h.nnz, c->k_logprobs)) return 0;
  if (c->B > SIP_MAX_B || V > SIP_MAX_V || c->k_logprobs > SIP_MAX_K_LOGPROBS) return 0;
  const size_t esz = c->dtype == SIP_F32 ? 4 : 2;
  return make_layout(c->B, make_plan(c->B, V, (int)c->dtype, sh.t), h.nnz + h.p_nnz, sh.t ? (size_t)V * esz : 0).total;
}

sip_status sip_sample_call(const sip_call* c) {
  HistSource h; ShardSource sh; int32_t V = 0;
  const sip_status ok = call_sources(c, h, sh, V);
  if (ok != SIP_OK) return ok;
  hipStream_t stream = static_cast<hipStream_t>(c->hip_stream);
  const sip_status st = sample_impl(c->logits, c->B, V, c->row_stride, c->dtype, c->params, h, c->seed, c->step,
                                    c->out_ids, c->out_lp_ids, c->out_lp, c->k_logprobs, c->workspace,
                                    c->workspace_bytes, stream, sh);
  if (st != SIP_OK || !c->host_flag) return st;
  return sip_publish_ids(c->out_ids, c->B, c->host_ids, c->host_flag, c->ticket, c->hip_stream);
}

sip_status sip_publish_ids(const int32_t* ids, int32_t B, int32_t* host_ids, uint64_t* host_flag, uint64_t ticket,
                           void* hip_stream) {
  if (!ids || !host_ids || !host_flag || B <= 0) return SIP_ERR_INVALID_ARG;
  if ((reinterpret_cast<uintptr_t>(host_flag) & 7u) != 0 || (reinterpret_cast<uintptr_t>(host_ids) & 3u) != 0)
    return SIP_ERR_INVALID_ARG;
  hipLaunchKernelGGL(sip::publish_kernel, dim3(1), dim3(sip::kPublishThreads), 0,
                     static_cast<hipStream_t>(hip_stream), ids, B, host_ids,
                     reinterpret_cast<unsigned long long*>(host_flag), (unsigned long long)ticket);
  return hipGetLastError() == hipSuccess ? SIP_OK : SIP_ERR_HIP;
}

sip_status sip_wait_ids(const uint64_t* host_flag, uint64_t ticket, uint64_t timeout_ns) {
  if (!host_flag || (reinterpret_cast<uintptr_t>(host_flag) & 7u) != 0) return SIP_ERR_INVALID_ARG;
  const auto t0 = std::chrono::steady_clock::now();
  unsigned spins = 0;
  for (;;) {
    if (__atomic_load_n(host_flag, __ATOMIC_ACQUIRE) >= ticket) return SIP_OK;
    __builtin_ia32_pause();
    if ((++spins & 1023u) == 0 && timeout_ns != UINT64_MAX) {
      const auto dt = std::chrono::duration_cast<std::chrono::nanoseconds>(std::chrono::steady_clock::now() - t0);
      if ((uint64_t)dt.count() >= timeout_ns) return SIP_ERR_TIMEOUT;
    }
  }
}

sip_status sip_probe_read(const void* src, size_t bytes, int32_t workgroups, void* workspace,
                          size_t workspace_bytes, void* start_event, void* stop_event, void* hip_stream) {
  if (!src || bytes < 16 || workgroups <= 0 || workgroups > 65536) return SIP_ERR_INVALID_ARG;
  if ((reinterpret_cast<uintptr_t>(src) & 15u) != 0) return SIP_ERR_INVALID_ARG;
  if (!workspace || workspace_bytes < (size_t)workgroups * sizeof(float)) return SIP_ERR_WORKSPACE;
  hipExtLaunchKernelGGL(sip::probe_read_kernel, dim3(workgroups), dim3(sip::kProbeThreads), 0,
                        static_cast<hipStream_t>(hip_stream), static_cast<hipEvent_t>(start_event),
                        static_cast<hipEvent_t>(stop_event), 0, static_cast<const uint4*>(src), bytes / 16,
                        (int)workgroups, static_cast<float*>(workspace));
  return hipGetLastError() == hipSuccess ? SIP_OK : SIP_ERR_HIP;
}

int32_t sip_plan_chunks(int32_t B, int32_t V, sip_dtype dtype, int32_t t_shards) {
  if (B <= 0 || B > SIP_MAX_B || V <= 0 || (dtype != SIP_F32 && dtype != SIP_BF16) || t_shards < 0 || t_shards > SIP_MAX_SHARDS) return -1;
  if (t_shards > 0 && V % t_shards != 0) return -1;
  const Plan p = make_plan(B, V, (int)dtype, t_shards);
  return p.fast ? p.S : 0;
}

const char* sip_status_string(sip_status status) {
  switch (status) {
    case SIP_OK: return "ok";
    case SIP_ERR_INVALID_ARG: return "invalid argument";
    case SIP_ERR_UNSUPPORTED: return "unsupported shape";
    case SIP_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case SIP_ERR_HIP: return "HIP runtime error";
    case SIP_ERR_TIMEOUT: return "timed out";
    case SIP_ERR_SCRATCH: return "call needs more scratch than the library's built-in array holds";
  }
  return "unknown status";
}

void sip_profile_kernel_events(void* stream_start, void* stream_stop, void* finish_start, void* finish_stop,
                               void* rescue_start, void* rescue_stop) {
  g_prof[0] = static_cast<hipEvent_t>(stream_start);
  g_prof[1] = static_cast<hipEvent_t>(stream_stop);
  g_prof[2] = static_cast<hipEvent_t>(finish_start);
  g_prof[3] = static_cast<hipEvent_t>(finish_stop);
  g_prof[4] = static_cast<hipEvent_t>(rescue_start);
  g_prof[5] = static_cast<hipEvent_t>(rescue_stop);
}

int sip_version(void) { return 100; }

}  // extern "C"
