// Device-resident sampler state: the token history of every live sequence stays in HBM from one
// decode iteration to the next, and the sampler appends its own output to it (Sec. 5.1, "memory
// reuse": a preallocated output table that each iteration adds a row to, instead of rebuilding
// the history for every call).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sip {

constexpr size_t kStateHeaderBytes = 256;

struct StateHeader {
  unsigned long long tick;      // sampling calls made on this state
  unsigned int overflow;        // ids (or prompts) that did not fit into their slot
};

// Host-side view of the pieces of one state buffer.
struct StateView {
  StateHeader* head;
  int* len;        // [slots]
  int* ndist;      // [slots] upper bound on the distinct tokens of the slot's history, -1 = unknown
  int* tokens;     // [slots, L_max]
  size_t total;
};

inline size_t state_len_bytes(int slots) { return ((size_t)slots * sizeof(int) + 255) / 256 * 256; }
inline size_t state_total(int slots, int L_max) {
  return kStateHeaderBytes + 2 * state_len_bytes(slots) + (size_t)slots * (size_t)L_max * sizeof(int);
}
inline StateView state_view(void* base, int slots, int L_max) {
  StateView v;
  char* p = static_cast<char*>(base);
  const size_t len_bytes = state_len_bytes(slots);
  v.head = reinterpret_cast<StateHeader*>(p);
  v.len = reinterpret_cast<int*>(p + kStateHeaderBytes);
  v.ndist = reinterpret_cast<int*>(p + kStateHeaderBytes + len_bytes);
  v.tokens = reinterpret_cast<int*>(p + kStateHeaderBytes + 2 * len_bytes);
  v.total = state_total(slots, L_max);
  return v;
}

constexpr int kStateThreads = 256;

// Header and every slot's length to zero.  A kernel rather than a memset so that the call can be
// recorded into a graph like the others.
__global__ __launch_bounds__(kStateThreads) void state_init_kernel(StateHeader* head, int* len, int* ndist, int slots) {
  const int i = blockIdx.x * kStateThreads + threadIdx.x;
  if (i == 0) { head->tick = 0; head->overflow = 0; }
  if (i < slots) { len[i] = 0; ndist[i] = 0; }
}

// One workgroup per (slot, prompt) pair: the slot's history becomes the prompt (its first L_max
// tokens).  Pairs whose slot is outside [0, slots) are skipped.
__global__ __launch_bounds__(kStateThreads) void state_assign_kernel(StateHeader* head, int* len, int* ndist,
                                                                      int* tokens, int slots, int L_max, const int* slot_ids,
                                                                      const long long* indptr, const int* src,
                                                                      long long src_nnz) {
  const int s = slot_ids[blockIdx.x];
  if (s < 0 || s >= slots) return;
  long long lo = 0, hi = 0;
  if (indptr && src && src_nnz > 0) {
    lo = indptr[blockIdx.x]; hi = indptr[blockIdx.x + 1];
    lo = lo < 0 ? 0 : (lo > src_nnz ? src_nnz : lo);
    hi = hi < lo ? lo : (hi > src_nnz ? src_nnz : hi);
  }
  const long long n = hi - lo;
  const int keep = (int)(n < (long long)L_max ? n : (long long)L_max);
  int* dst = tokens + (size_t)s * (size_t)L_max;
  for (int i = threadIdx.x; i < keep; i += kStateThreads) dst[i] = src[lo + i];
  if (threadIdx.x == 0) {
    len[s] = keep;
    ndist[s] = keep == 0 ? 0 : -1;                 // a prompt's distinct tokens are not counted here
    if (n > (long long)L_max) atomicAdd(&head->overflow, 1u);
  }
}

// A call on a shape that the single-pass kernels do not serve is counted after its one kernel.
__global__ void state_tick_kernel(StateHeader* head) {
  if (blockIdx.x == 0 && threadIdx.x == 0) head->tick += 1;
}

}  // namespace sip
