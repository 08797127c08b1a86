// Device-side building blocks shared by the sampler kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/sip.h"

namespace sip {

constexpr int kWave = 64;
constexpr int kFixShift = 40;          // masses are carried as integers in units of 2^-40 of the row maximum's mass
constexpr float kFixScale = 1099511627776.0f;   // 2^40

// Bit 31 of a list entry's index: the token occurs in the row's history and the row has a penalty
// switched on, so the entry's value is the raw logit that the penalty still has to be applied to.
constexpr uint32_t kTagBit = 0x80000000u;
constexpr int kPromptFlag = 1 << 30;             // RowInfo::target: tokens of a separate prompt are tagged too
constexpr uint32_t kCntOverflow = 0xFFFFFFFFu;   // ChunkOut::cnt of a chunk whose queue overflowed

// What the streaming workgroup of one chunk leaves behind.  Its list (the chunk's segment in
// Args::cand) holds every element with z >= Tc and every element whose token is in the row's
// history (tagged, see kTagBit); `bulk` is the softmax mass of all other elements.
struct ChunkOut {
  unsigned long long bulk;  // sum over the elements not in the list of 2^(z*c - R), in units of 2^-30
  float Tc;                 // every element of the chunk with z >= Tc is in the segment
  int R;                    // integer reference exponent of `bulk`
  unsigned int cnt;         // entries in the chunk's segment, or kCntOverflow
  unsigned int pad[3];
};

// What the streaming kernel (the workgroup of a row's first chunk) leaves for the finishing
// kernel about row b: its sampling parameters, the extent of its history in Args::tokens and
// the length the list was asked to have (0: the row cannot be finished from a list).
struct RowInfo {
  float tau, top_p, min_p, theta, phi, psi;
  int top_k, target;
  unsigned long long row_id;
  long long lo, hi;
  int slot;                 // device-resident state: the row's slot, -1 = none (or a CSR call)
  int ndist;                // ... and the distinct tokens in the slot's table of multiplicities, -1 = table not valid
};
static_assert(sizeof(RowInfo) == 64, "one 64-byte record per row");

// Everything one call needs, passed by value to the kernels.
struct Args {
  const void* logits;
  int B, V;
  long long row_stride;
  sip_params p;
  const long long* indptr;
  const int* tokens;
  long long nnz;
  // separate prompt tokens (CSR; nullptr = none): the repetition penalty looks at them too
  const long long* p_indptr;
  const int* p_tokens;
  long long p_nnz;
  unsigned long long seed, step;
  int* out_ids;
  int* out_lp_ids;
  float* out_lp;
  int k_lp;
  // workspace of the exact path
  float* side_z;          // [nnz]  penalised value of the r-th distinct history token of a row
  unsigned int* side_c;   // [nnz]  its multiplicity
  // workspace and launch shape of the single-pass path
  RowInfo* rowinfo;         // [B]
  int fin_tps, fin_inv;     // finishing kernel: threads per list segment (512 / S), and ceil(2^16 / that)
  ChunkOut* chunks;         // [B * S]
  uint2* cand;              // [B * S * cap_c]  (value bits, index | tag): one segment per chunk
  int S;                    // chunks per row
  int cap_c;                // list entries per chunk segment
  int nc_cap;               // longest list any finishing path can hold
  int* row_path;            // [B] diagnostic: 1 = finished by the single-pass path, >1 = exact path (reason)
  int* row_why;             // [B] diagnostic: 1, or why the finishing kernel handed the row to the rescue kernel
  int* rescue_n;            // rows the finishing kernel could not settle from the list ...
  int* rescue_rows;         // [B] ... and which; the rescue kernel takes them from here
  unsigned long long* rescue_tick;   // room in the workspace for `call_tick`
  // Device-resident history (sip_sample_state): `slot` != nullptr replaces the CSR above.  Row b's
  // history is tokens[slot[b] * L_max .. + st_len[slot[b]]); `tokens` then points at the state's
  // token table and nnz = slots * L_max.
  const int* slot;                     // [B]; outside [0, slots): the row has no history
  int* st_len;                         // [slots]
  int* st_ndist;                       // [slots] distinct tokens in the slot's table of multiplicities, -1 = table not valid
  uint32_t* st_table;                  // [slots, 2 * kTableSlots]: per slot, keys then multiplicities
  unsigned long long* call_tick;       // workspace: the state's call counter as this call found it
  int* st_tokens;                      // [slots, L_max]: same memory as `tokens`, for the append
  unsigned long long* st_tick;         // sampling calls made on the state so far; added to `step`
  unsigned int* st_overflow;           // ids that found their slot full
  // Vocabulary-sharded logits (sip_sample_sharded): row b is the concatenation of t_shards pieces of
  // V_shard elements, piece i at shard[i] + b * shard_stride elements.  `logits` / `row_stride` then
  // describe the workspace rows that a workgroup gathers its row into before any whole-row access.
  const void* shard[8];
  int t_shards, V_shard;
  long long shard_stride;
  float inv_V_shard;                   // 1 / V_shard
  // where the row's sample blocks lie (the streaming kernel's threshold estimate): block sb is the
  // (sb % smp_bps)-th of shard sb / smp_bps, smp_step elements after the one before it;
  // smp_inv = ceil(2^16 / smp_bps) turns the division into a multiplication (sb < 64)
  int smp_bps, smp_inv, smp_step;
  int L_max, slots;
};

// Extent of row b's history in a.tokens, clamped so that no read leaves the array, and where the
// row's part of the exact path's side tables starts.
struct HistRange { long long lo, hi, side; };
__device__ __forceinline__ HistRange hist_range(const Args& a, int b) {
  HistRange h{0, 0, 0};
  if (a.slot) {
    const int s = a.slot[b];
    h.side = (long long)b * a.L_max;
    if (s >= 0 && s < a.slots) {
      const int n = a.st_len[s];
      h.lo = (long long)s * a.L_max;
      h.hi = h.lo + (n < 0 ? 0 : (n > a.L_max ? a.L_max : n));
    }
  } else if (a.indptr && a.tokens && a.nnz > 0) {
    h.lo = a.indptr[b]; h.hi = a.indptr[b + 1];
    h.lo = h.lo < 0 ? 0 : (h.lo > a.nnz ? a.nnz : h.lo);
    h.hi = h.hi < h.lo ? h.lo : (h.hi > a.nnz ? a.nnz : h.hi);
    h.side = h.lo;
  }
  return h;
}
// The same for a call without a state, from the row's two CSR offsets as they were read.
__device__ __forceinline__ HistRange hist_range_csr(const Args& a, long long lo, long long hi) {
  HistRange h{0, 0, 0};
  if (a.indptr && a.tokens && a.nnz > 0) {
    h.lo = lo < 0 ? 0 : (lo > a.nnz ? a.nnz : lo);
    h.hi = hi < h.lo ? h.lo : (hi > a.nnz ? a.nnz : hi);
    h.side = h.lo;
  }
  return h;
}
// Which tokens of row b carry a penalty and what has to be known about them (Sec. 2.1 step 3 (1);
// Sec. 5.1 CalcPenalty): the row's history (the generated tokens: all three penalties) and,
// if the caller hands them in separately, its prompt tokens (repetition penalty only).
struct PenaltyPlan {
  HistRange h;
  long long p_lo, p_hi;   // extent of the prompt in a.p_tokens; empty unless the repetition penalty is on
  long long side;         // where the row's part of the exact path's side tables starts
  bool any;               // some token of the row carries a penalty
  bool prompt_on;
  bool counts;            // the tokens' multiplicities in the history are needed ...
  unsigned int dflt;      // ... otherwise every penalised token is taken to occur this often in it
};
// (`h`: the row's history extent; `p0`, `p1`: the row's raw offsets into the prompt tokens, looked
// at only if the call has prompt tokens)
__device__ __forceinline__ PenaltyPlan penalty_plan_of(const Args& a, const HistRange h, long long p0, long long p1,
                                                       float theta, float phi, float psi) {
  PenaltyPlan q;
  q.h = h;
  q.p_lo = q.p_hi = 0;
  long long p_before = 0;   // prompt tokens of the rows before this one: they shift the row's part of the side tables
  if (a.p_indptr && a.p_tokens && a.p_nnz > 0) {
    p0 = p0 < 0 ? 0 : (p0 > a.p_nnz ? a.p_nnz : p0);
    p1 = p1 < p0 ? p0 : (p1 > a.p_nnz ? a.p_nnz : p1);
    p_before = p0;
    if (theta != 1.0f) { q.p_lo = p0; q.p_hi = p1; }
  }
  const bool hist = q.h.hi > q.h.lo;
  q.prompt_on = q.p_hi > q.p_lo;
  q.any = (hist && (theta != 1.0f || phi != 0.0f || psi != 0.0f)) || q.prompt_on;
  q.counts = hist && (phi != 0.0f || (q.prompt_on && psi != 0.0f));
  q.dflt = hist ? 1u : 0u;
  q.side = q.h.side + p_before;
  return q;
}
__device__ __forceinline__ PenaltyPlan penalty_plan(const Args& a, int b, float theta, float phi, float psi) {
  long long p0 = 0, p1 = 0;
  if (a.p_indptr && a.p_tokens && a.p_nnz > 0) { p0 = a.p_indptr[b]; p1 = a.p_indptr[b + 1]; }
  return penalty_plan_of(a, hist_range(a, b), p0, p1, theta, phi, psi);
}
// Base of shard `sh` (uniform or per lane): a chain of selects, because the table lives in the
// kernel-argument segment and must be indexed with constants.
__device__ __forceinline__ const char* shard_base(const Args& a, int sh) {
  const void* p = a.shard[0];
#pragma unroll
  for (int i = 1; i < 8; ++i)
    if (sh == i) p = a.shard[i];
  return reinterpret_cast<const char*>(p);
}
// Gather row b of a sharded call into its workspace row (a.logits / a.row_stride describe those
// rows), for the code paths that walk a whole row.  Called by all threads of the row's workgroup.
template <int DT>
__device__ __attribute__((noinline)) void gather_row(const Args& a, int b) {
  constexpr int ESZ = (DT == SIP_F32) ? 4 : 2;
  char* dst = const_cast<char*>(reinterpret_cast<const char*>(a.logits)) + (size_t)b * (size_t)a.row_stride * ESZ;
  const size_t piece = (size_t)a.V_shard * ESZ / 16;                  // 16-byte groups per piece
  for (int sh = 0; sh < a.t_shards; ++sh) {
    const uint4* src = reinterpret_cast<const uint4*>(shard_base(a, sh) + (size_t)b * (size_t)a.shard_stride * ESZ);
    uint4* d = reinterpret_cast<uint4*>(dst) + (size_t)sh * piece;
    for (size_t i = threadIdx.x; i < piece; i += blockDim.x) d[i] = src[i];
  }
  __syncthreads();
}
// The kernels read their arguments where they use them, straight from the kernel-argument
// segment, and a first read of each of its 64-byte lines misses the scalar cache: spread over a
// kernel those are as many round trips one after the other.  This touches every line at once,
// at the start (scalar loads only, results thrown away).
__device__ __forceinline__ void warm_kernel_arguments() {
  static_assert(sizeof(Args) >= 0x1c4 && sizeof(Args) <= 0x200, "eight lines of 64 bytes");
  const void* p = (const void*)__builtin_amdgcn_kernarg_segment_ptr();
  uint32_t t0, t1, t2, t3, t4, t5, t6, t7;
  asm volatile(
      "s_load_dword %0, %8, 0x0\n\t"
      "s_load_dword %1, %8, 0x40\n\t"
      "s_load_dword %2, %8, 0x80\n\t"
      "s_load_dword %3, %8, 0xc0\n\t"
      "s_load_dword %4, %8, 0x100\n\t"
      "s_load_dword %5, %8, 0x140\n\t"
      "s_load_dword %6, %8, 0x180\n\t"
      "s_load_dword %7, %8, 0x1c0\n\t"
      "s_waitcnt lgkmcnt(0)"
      : "=&s"(t0), "=&s"(t1), "=&s"(t2), "=&s"(t3), "=&s"(t4), "=&s"(t5), "=&s"(t6), "=&s"(t7)
      : "s"(p));
}

// Philox step of this call: on a state, `step` plus the number of calls made on the state before
// this one.  The streaming kernel takes that number (one atomic add, so that calls in flight at
// once on one state each get their own) and leaves it in the call's workspace; a call that has no
// streaming kernel reads the counter itself and counts afterwards.
__device__ __forceinline__ unsigned long long step_of(const Args& a) {
  if (!a.st_tick) return a.step;
  return a.step + (a.call_tick ? *a.call_tick : *a.st_tick);
}

// ---------------------------------------------------------------- table of multiplicities
// token -> number of occurrences in a history, as an open-addressing hash table of
// kTableSlots / 4 buckets of four slots: `key[kTableSlots]` (kTableEmpty = free) and
// `val[kTableSlots]`.  A token lives in the first bucket, from its home bucket on, that had a
// free slot when it came; the slots of a bucket fill in order, and a key, once there, stays.
// The finishing kernel builds one per row in LDS, or copies the one a device-resident state
// keeps per slot and updates at the one new token per call (Sec. 5.1, incremental penalty
// construction).
constexpr int kTableSlots = 4096;
constexpr int kTableMaxDistinct = 3072;            // beyond this load the table is given up
constexpr uint32_t kTableEmpty = 0xFFFFFFFFu;
static_assert(kTableSlots == 4096, "table_home() yields 10 bits: 1024 buckets of 4 slots");
__device__ __forceinline__ uint32_t table_home(uint32_t t) { return (t * 0x9E3779B1u) >> 22; }

// Insert by many threads at once (LDS).  Returns 1 if this call claimed a new slot, 0 if the
// token was there already, -1 if the table is full.
__device__ __forceinline__ int table_insert_shared(uint32_t* key, uint32_t* val, uint32_t t) {
  const uint4* key4 = reinterpret_cast<const uint4*>(key);
  uint32_t bk = table_home(t);
  for (int probe = 0; probe < kTableSlots / 4; ++probe) {
    const uint4 k4 = key4[bk];
    const uint32_t ks[4] = {k4.x, k4.y, k4.z, k4.w};
    int j = -1, fresh = 0;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      if (j < 0 && ks[e] == t) j = e;
      if (j < 0 && ks[e] == kTableEmpty) {                 // free when read: try to take it
        const uint32_t old = atomicCAS(&key[4 * bk + e], kTableEmpty, t);
        if (old == kTableEmpty) { fresh = 1; j = e; } else if (old == t) j = e;
      }
    }
    if (j >= 0) { atomicAdd(&val[4 * bk + j], 1u); return fresh; }
    bk = (bk + 1) & (kTableSlots / 4 - 1);
  }
  return -1;
}
// Insert by the one thread that owns the table (global memory): one 16-byte read per bucket
// looked at.  Same return values.
__device__ __forceinline__ int table_insert_single(uint32_t* key, uint32_t* val, uint32_t t) {
  const uint4* key4 = reinterpret_cast<const uint4*>(key);
  uint32_t bk = table_home(t);
  for (int probe = 0; probe < kTableSlots / 4; ++probe) {
    const uint4 k4 = key4[bk];
    const uint32_t hit = (uint32_t)(k4.x == t) | ((uint32_t)(k4.y == t) << 1) | ((uint32_t)(k4.z == t) << 2) |
                         ((uint32_t)(k4.w == t) << 3);
    const uint32_t free = (uint32_t)(k4.x == kTableEmpty) | ((uint32_t)(k4.y == kTableEmpty) << 1) |
                          ((uint32_t)(k4.z == kTableEmpty) << 2) | ((uint32_t)(k4.w == kTableEmpty) << 3);
    if (hit) { val[4 * bk + (uint32_t)(__ffs((int)hit) - 1)] += 1u; return 0; }
    if (free) {
      const uint32_t e = 4 * bk + (uint32_t)(__ffs((int)free) - 1);
      key[e] = t; val[e] = 1u;
      return 1;
    }
    bk = (bk + 1) & (kTableSlots / 4 - 1);
  }
  return -1;
}

// Row b's sampled id joins the history of its slot, and the slot's table of multiplicities.  For
// one thread of the row's workgroup, once out_ids[b] is written and visible to it.  Nobody else
// reads or writes this slot during the call (the slots of a call are distinct).
__device__ __forceinline__ void state_append_row(const Args& a, int b) {
  const int s = a.slot[b];
  if (s < 0 || s >= a.slots) return;
  const int n = a.st_len[s];
  if (n >= 0 && n < a.L_max) {
    const int tok = a.out_ids[b];
    a.st_tokens[(size_t)s * (size_t)a.L_max + n] = tok;
    a.st_len[s] = n + 1;
    int nd = a.st_ndist[s];
    if (nd >= 0 && tok >= 0) {
      uint32_t* key = a.st_table + (size_t)s * (size_t)(2 * kTableSlots);
      const int r = table_insert_single(key, key + kTableSlots, (uint32_t)tok);
      nd = r < 0 ? -1 : nd + r;
      if (nd > kTableMaxDistinct) nd = -1;
      a.st_ndist[s] = nd;
    }
  } else {
    atomicAdd(a.st_overflow, 1u);
  }
}

// A row is cut into S chunks of whole units of `unit` elements (what one wave reads with one
// 16-byte load per lane), the chunk sizes differing by at most one unit.  First element of
// chunk ch; chunk_begin(S) is V.
// (32-bit arithmetic on purpose: V <= 2^19 and ch <= 17, and a 64-bit division by S is a long
// routine on the device.)
__host__ __device__ inline int chunk_begin(int ch, int V, int S, int unit) {
  const unsigned int n = ((unsigned int)V + (unsigned int)unit - 1u) / (unsigned int)unit;
  const unsigned int e = (unsigned int)ch * n / (unsigned int)S * (unsigned int)unit;
  return (int)(e < (unsigned int)V ? e : (unsigned int)V);
}

// ApplyPenalty for one seen token: repetition, then frequency, then presence, one fp32
// rounding per operation (Sec. 2.1 step 3 (1); Sec. 5.1).  `count`: occurrences among the
// generated tokens; 0 = the token is in the separately given prompt only, which the frequency
// and presence penalties do not look at.
__device__ __forceinline__ float penalise(float z, unsigned int count, float theta, float phi, float psi) {
  if (theta != 1.0f) z = (z > 0.0f) ? __fdiv_rn(z, theta) : __fmul_rn(z, theta);
  if (count != 0u) {
    if (phi != 0.0f) z = __fsub_rn(z, __fmul_rn(phi, (float)count));
    if (psi != 0.0f) z = __fsub_rn(z, psi);
  }
  return z;
}

// ---------------------------------------------------------------- keys
// Order-preserving map fp32 -> u32 (larger float <=> larger key); -0 and +0 share a key.
__device__ __forceinline__ uint32_t key_of(float s) {
  s = s + 0.0f;
  uint32_t b = __float_as_uint(s);
  return b ^ ((b & 0x80000000u) ? 0xFFFFFFFFu : 0x80000000u);
}
__device__ __forceinline__ float value_of(uint32_t key) {
  return __uint_as_float((key & 0x80000000u) ? (key ^ 0x80000000u) : ~key);
}

// ---------------------------------------------------------------- Philox4x32-10
// Salmon et al., SC'11.  counter = (row lo, row hi, step lo, step hi), key = (seed lo, seed hi).
__device__ __forceinline__ uint32_t philox_word0(unsigned long long seed, unsigned long long row,
                                                 unsigned long long step) {
  uint32_t c0 = (uint32_t)row, c1 = (uint32_t)(row >> 32), c2 = (uint32_t)step, c3 = (uint32_t)(step >> 32);
  uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
    const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
    const uint32_t n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
    c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
    k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
  }
  return c0;
}

// ---------------------------------------------------------------- wave / block collectives
__device__ __forceinline__ int lane_id() { return threadIdx.x & (kWave - 1); }
__device__ __forceinline__ int wave_id() { return threadIdx.x >> 6; }

template <typename T>
__device__ __forceinline__ T wave_sum(T v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}

__device__ __forceinline__ unsigned long long shfl_u64(unsigned long long v, int src) {
  int lo = __shfl((int)(uint32_t)v, src, kWave), hi = __shfl((int)(uint32_t)(v >> 32), src, kWave);
  return ((unsigned long long)(uint32_t)hi << 32) | (uint32_t)lo;
}
__device__ __forceinline__ unsigned long long shfl_up_u64(unsigned long long v, int d) {
  int lo = __shfl_up((int)(uint32_t)v, d, kWave), hi = __shfl_up((int)(uint32_t)(v >> 32), d, kWave);
  return ((unsigned long long)(uint32_t)hi << 32) | (uint32_t)lo;
}
__device__ __forceinline__ unsigned long long shfl_xor_u64(unsigned long long v, int m) {
  int lo = __shfl_xor((int)(uint32_t)v, m, kWave), hi = __shfl_xor((int)(uint32_t)(v >> 32), m, kWave);
  return ((unsigned long long)(uint32_t)hi << 32) | (uint32_t)lo;
}
__device__ __forceinline__ unsigned long long wave_sum_u64(unsigned long long v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += shfl_xor_u64(v, o);
  return v;
}
// inclusive prefix sum across the 64 lanes
__device__ __forceinline__ unsigned long long wave_incl_scan_u64(unsigned long long v) {
  const int l = lane_id();
#pragma unroll
  for (int d = 1; d < kWave; d <<= 1) {
    unsigned long long t = shfl_up_u64(v, d);
    if (l >= d) v += t;
  }
  return v;
}
__device__ __forceinline__ uint32_t wave_incl_scan_u32(uint32_t v) {
  const int l = lane_id();
#pragma unroll
  for (int d = 1; d < kWave; d <<= 1) {
    uint32_t t = (uint32_t)__shfl_up((int)v, d, kWave);
    if (l >= d) v += t;
  }
  return v;
}

// ---------------------------------------------------------------- DPP wave collectives
// Cross-lane sums and maxima that stay in the VALU (data-parallel-primitive row shifts and
// row broadcasts) instead of going through the LDS crossbar.  Pattern: Hillis-Steele inside
// each row of 16 lanes (row_shr 1,2,4,8), then lane 15 of rows 0/2 into rows 1/3
// (row_bcast:15), then lane 31 into rows 2,3 (row_bcast:31).  Lane i ends up with the
// inclusive result over lanes 0..i; lane 63 holds the wave total.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ uint32_t dpp_mov(uint32_t old, uint32_t v) {
  return (uint32_t)__builtin_amdgcn_update_dpp((int)old, (int)v, CTRL, ROW_MASK, 0xf, false);
}
#define SIP_DPP_STEPS(OP, ID)                    \
  v = OP(v, dpp_mov<0x111, 0xf>(ID, v));         \
  v = OP(v, dpp_mov<0x112, 0xf>(ID, v));         \
  v = OP(v, dpp_mov<0x114, 0xf>(ID, v));         \
  v = OP(v, dpp_mov<0x118, 0xf>(ID, v));         \
  v = OP(v, dpp_mov<0x142, 0xa>(ID, v));         \
  v = OP(v, dpp_mov<0x143, 0xc>(ID, v));
__device__ __forceinline__ uint32_t op_add(uint32_t a, uint32_t b) { return a + b; }
__device__ __forceinline__ uint32_t op_max(uint32_t a, uint32_t b) { return a > b ? a : b; }
__device__ __forceinline__ uint32_t op_min(uint32_t a, uint32_t b) { return a < b ? a : b; }
__device__ __forceinline__ uint32_t dpp_scan_add_u32(uint32_t v) { SIP_DPP_STEPS(op_add, 0u) return v; }
__device__ __forceinline__ uint32_t dpp_scan_max_u32(uint32_t v) { SIP_DPP_STEPS(op_max, 0u) return v; }
__device__ __forceinline__ uint32_t dpp_scan_min_u32(uint32_t v) { SIP_DPP_STEPS(op_min, 0xFFFFFFFFu) return v; }
#undef SIP_DPP_STEPS
__device__ __forceinline__ unsigned long long dpp_scan_add_u64(unsigned long long v) {
#define SIP_DPP64(CTRL, RM)                                                                   \
  v += ((unsigned long long)dpp_mov<CTRL, RM>(0u, (uint32_t)(v >> 32)) << 32) | dpp_mov<CTRL, RM>(0u, (uint32_t)v);
  SIP_DPP64(0x111, 0xf) SIP_DPP64(0x112, 0xf) SIP_DPP64(0x114, 0xf) SIP_DPP64(0x118, 0xf)
  SIP_DPP64(0x142, 0xa) SIP_DPP64(0x143, 0xc)
#undef SIP_DPP64
  return v;
}
__device__ __forceinline__ uint32_t last_lane_u32(uint32_t v) { return (uint32_t)__builtin_amdgcn_readlane((int)v, kWave - 1); }
__device__ __forceinline__ unsigned long long last_lane_u64(unsigned long long v) {
  return ((unsigned long long)last_lane_u32((uint32_t)(v >> 32)) << 32) | last_lane_u32((uint32_t)v);
}

__device__ __forceinline__ unsigned long long readlane_u64(unsigned long long v, int l) {
  return ((unsigned long long)(uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(v >> 32), l) << 32) |
         (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)v, l);
}

// fp32 mass in (0, 1] -> integer units of 2^-40 (truncating); exact above 2^-16
__device__ __forceinline__ unsigned long long fix_of(float e) {
  return (unsigned long long)(e * kFixScale);
}

}  // namespace sip
