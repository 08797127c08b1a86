// Hand-off of the sampled ids to the host without a stream synchronisation: a kernel, ordered on
// the stream after the sampling call, copies the ids into pinned host memory and then publishes a
// ticket in a host flag that a scheduler thread polls.  (The paper's sampler hands its ids back
// through a ring of slots that the consumer polls, Sec. 6 "BIC-O"; this is the same idea at the
// device / host boundary.)
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sip {

constexpr int kPublishThreads = 256;

// One workgroup: every id is stored and made visible system-wide before the ticket is.
__global__ __launch_bounds__(kPublishThreads) void publish_kernel(const int* ids, int B, int* host_ids,
                                                                   unsigned long long* host_flag,
                                                                   unsigned long long ticket) {
  for (int i = threadIdx.x; i < B; i += kPublishThreads)
    __hip_atomic_store(&host_ids[i], ids[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
  __threadfence_system();
  __syncthreads();
  if (threadIdx.x == 0) __hip_atomic_store(host_flag, ticket, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
}

// Measurement aid: the bare streaming read that stream_kernel is compared with.  Same launch
// shape (workgroups of 512 threads, each on one contiguous piece, 16-byte loads, two tiles of two
// loads per lane in rotation); all it does with the data is add it up.
constexpr int kProbeThreads = 512;
__global__ __launch_bounds__(kProbeThreads) void probe_read_kernel(const uint4* src, size_t n16, int pieces,
                                                                    float* out) {
  const size_t per = (n16 + pieces - 1) / pieces;
  const size_t lo = (size_t)blockIdx.x * per, hi = lo + per < n16 ? lo + per : n16;
  float acc = 0.0f;
  auto add = [&](const uint4& q) {
    acc += __uint_as_float(q.x) + __uint_as_float(q.y) + __uint_as_float(q.z) + __uint_as_float(q.w);
  };
  constexpr size_t kTile = 2 * kProbeThreads;
  const size_t last = hi > 0 ? hi - 1 : 0;
  uint4 a0, a1, b0, b1;
  size_t t = lo;
  auto load = [&](size_t at, uint4& x, uint4& y) {
    const size_t i0 = at + threadIdx.x, i1 = at + kProbeThreads + threadIdx.x;
    x = src[i0 < hi ? i0 : last]; y = src[i1 < hi ? i1 : last];
  };
  auto use = [&](size_t at, const uint4& x, const uint4& y) {
    if (at + threadIdx.x < hi) add(x);
    if (at + kProbeThreads + threadIdx.x < hi) add(y);
  };
  if (lo < hi) {
    load(t, a0, a1);
    if (t + kTile < hi) load(t + kTile, b0, b1);
    while (t < hi) {
      use(t, a0, a1);
      if (t + 2 * kTile < hi) load(t + 2 * kTile, a0, a1);
      t += kTile;
      if (t < hi) {
        use(t, b0, b1);
        if (t + 2 * kTile < hi) load(t + 2 * kTile, b0, b1);
        t += kTile;
      }
    }
  }
  __shared__ float red[kProbeThreads / 64];
  for (int o = 32; o > 0; o >>= 1) acc += __shfl_down(acc, o, 64);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = acc;
  __syncthreads();
  if (threadIdx.x == 0) {
    float s = 0.0f;
    for (int w = 0; w < kProbeThreads / 64; ++w) s += red[w];
    out[blockIdx.x] = s;
  }
}

}  // namespace sip
