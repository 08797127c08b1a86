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

}  // namespace sip
