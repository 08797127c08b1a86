// Device-resident sampler state: the token history of every live sequence stays in HBM from one
// decode iteration to the next, and the sampler appends its own output to it (Sec. 5.1, "memory
// reuse": a preallocated output table that each iteration adds a row to, instead of rebuilding
// the history for every call).
//
// Beside the raw history every slot keeps a table of multiplicities (token -> occurrences, the
// hash table of sip_device.h) that is updated at the one new token per call instead of being
// rebuilt from the history (Sec. 5.1, "incremental penalty construction"): the finishing kernel
// copies it where the stateless entry point has to count the history's tokens.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sip_device.h"

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
  int* ndist;      // [slots] distinct tokens in the slot's table of multiplicities, -1 = table not valid
  int* tokens;     // [slots, L_max]
  uint32_t* table; // [slots, 2 * kTableSlots]: keys, then multiplicities
  size_t total;
};

inline size_t state_len_bytes(int slots) { return ((size_t)slots * sizeof(int) + 255) / 256 * 256; }
inline size_t state_tokens_bytes(int slots, int L_max) {
  return ((size_t)slots * (size_t)L_max * sizeof(int) + 255) / 256 * 256;
}
inline size_t state_total(int slots, int L_max) {
  return kStateHeaderBytes + 2 * state_len_bytes(slots) + state_tokens_bytes(slots, L_max) +
         (size_t)slots * (size_t)(2 * kTableSlots) * sizeof(uint32_t);
}
inline StateView state_view(void* base, int slots, int L_max) {
  StateView v;
  char* p = static_cast<char*>(base);
  const size_t len_bytes = state_len_bytes(slots);
  v.head = reinterpret_cast<StateHeader*>(p);
  v.len = reinterpret_cast<int*>(p + kStateHeaderBytes);
  v.ndist = reinterpret_cast<int*>(p + kStateHeaderBytes + len_bytes);
  v.tokens = reinterpret_cast<int*>(p + kStateHeaderBytes + 2 * len_bytes);
  v.table = reinterpret_cast<uint32_t*>(p + kStateHeaderBytes + 2 * len_bytes + state_tokens_bytes(slots, L_max));
  v.total = state_total(slots, L_max);
  return v;
}

constexpr int kStateThreads = 256;

// One workgroup per slot: length zero, table empty; workgroup 0 also clears the header.  A kernel
// rather than a memset so that the call can be recorded into a graph like the others.
__global__ __launch_bounds__(kStateThreads) void state_init_kernel(StateHeader* head, int* len, int* ndist,
                                                                    uint32_t* table, int slots) {
  const int s = blockIdx.x;
  if (s == 0 && threadIdx.x == 0) { head->tick = 0; head->overflow = 0; }
  if (s >= slots) return;
  uint32_t* key = table + (size_t)s * (size_t)(2 * kTableSlots);
  for (int i = threadIdx.x; i < kTableSlots; i += kStateThreads) { key[i] = kTableEmpty; key[kTableSlots + i] = 0u; }
  if (threadIdx.x == 0) { len[s] = 0; ndist[s] = 0; }
}

// One workgroup per (slot, prompt) pair: the slot's history becomes the prompt (its first L_max
// tokens) and its table of multiplicities is built from those tokens (in LDS, then written out).
// Pairs whose slot is outside [0, slots) are skipped.
__global__ __launch_bounds__(kStateThreads) void state_assign_kernel(StateHeader* head, int* len, int* ndist,
                                                                      int* tokens, uint32_t* table, int slots, int L_max,
                                                                      const int* slot_ids, const long long* indptr,
                                                                      const int* src, long long src_nnz) {
  __shared__ __align__(16) uint32_t tkey[kTableSlots];
  __shared__ uint32_t tval[kTableSlots];
  __shared__ int n_new, failed;
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
  for (int i = threadIdx.x; i < kTableSlots; i += kStateThreads) { tkey[i] = kTableEmpty; tval[i] = 0u; }
  if (threadIdx.x == 0) { n_new = 0; failed = 0; }
  __syncthreads();
  int mine = 0;
  for (int i = threadIdx.x; i < keep; i += kStateThreads) {
    const int t = src[lo + i];
    dst[i] = t;
    if (t >= 0) {                                  // negative ids are padding: stored, never counted
      const int r = table_insert_shared(tkey, tval, (uint32_t)t);
      if (r < 0) failed = 1; else mine += r;
    }
  }
  if (mine) atomicAdd(&n_new, mine);
  __syncthreads();
  uint32_t* key = table + (size_t)s * (size_t)(2 * kTableSlots);
  for (int i = threadIdx.x; i < kTableSlots; i += kStateThreads) { key[i] = tkey[i]; key[kTableSlots + i] = tval[i]; }
  if (threadIdx.x == 0) {
    len[s] = keep;
    ndist[s] = (failed || n_new > kTableMaxDistinct) ? -1 : n_new;
    if (n > (long long)L_max) atomicAdd(&head->overflow, 1u);
  }
}

// A call on a shape that the single-pass kernels do not serve is counted after its one kernel.
__global__ void state_tick_kernel(StateHeader* head) {
  if (blockIdx.x == 0 && threadIdx.x == 0) head->tick += 1;
}

}  // namespace sip
