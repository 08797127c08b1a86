// The general, always-exact path: one 1024-thread workgroup owns one row and answers every
// question about it (maximum, masses, k-th largest value, nucleus cut, draw, best-n) by
// re-reading the row, one radix digit or one prefix per pass.  It makes no assumption about
// the size of the kept set, so it is also where any row goes that the single-pass path
// cannot finish.
//
// Definitions implemented (paper Sec. 2.1 step 3 and Sec. 5.1; the readings the paper leaves
// open are spelled out at each step):
//   z'  = ApplyPenalty(z, y_<s)             fp32, seen tokens only
//   s   = z' / tau                          fp32 IEEE division; greedy rows use s = z'
//   e_v = exp(s_v - max s)                  carried as integers in units of 2^-40
//   K1  = { v : #{w : s_w > s_v} < k }      top-k, ties kept together
//   K2  = { v in K1 : mass{w in K1 : s_w > s_v} < p * mass(K1) }     top-p
//   K3  = { v in K2 : fp32(s_v - max s) >= fp32(ln min_p) }          min-p
//   id  = min { v in K3 : mass{w in K3 : w <= v} > u * mass(K3) }    draw, vocabulary order
//   logprob(v) = s_v - max s - ln sum_w e_w                          full vocabulary
#pragma once
#include "sip_device.h"

namespace sip {

constexpr int kExactThreads = 1024;                   // the stand-alone kernel's workgroup; exact_row itself
constexpr int kExactWaves = kExactThreads / kWave;    // adapts to any multiple of 64 up to this

struct ExactShared {
  uint32_t hcnt[256];
  unsigned long long hmass[256];
  unsigned long long red64[kExactWaves];
  uint32_t red32[kExactWaves];
  float redf[kExactWaves];
  int redi[kExactWaves];
  uint32_t bc_u32[4];
  unsigned long long bc_u64[2];
  int bc_i32[2];
  uint32_t tn_key[SIP_MAX_K_LOGPROBS];
  int tn_idx[SIP_MAX_K_LOGPROBS];
  float tn_s[SIP_MAX_K_LOGPROBS];
  uint32_t tn_cnt;
};

struct RowView {
  const char* row;      // first element of the row
  int V;
  int wave_range;       // elements owned by one wave (multiple of 256), contiguous, in wave order
  bool has_pen;
  const uint32_t* bm;   // LDS: bit v set <=> token v occurs in the history
  const uint32_t* pre;  // LDS: number of set bits in words before this one
  const float* side_z;  // global: penalised value of the r-th distinct history token
  float tau;
  bool greedy;
  float m;              // max_v s_v
};

// Four consecutive elements starting at e0 (multiple of 4, < V), penalties applied.
// Lanes past the end of the row get -inf in the unused slots.
template <int DT>
__device__ __forceinline__ void load_group(const RowView& r, int e0, float z[4]) {
  if (DT == SIP_F32) {
    const float4 q = *reinterpret_cast<const float4*>(r.row + (size_t)e0 * 4);
    z[0] = q.x; z[1] = q.y; z[2] = q.z; z[3] = q.w;
  } else {
    const uint2 q = *reinterpret_cast<const uint2*>(r.row + (size_t)e0 * 2);
    z[0] = __uint_as_float(q.x << 16); z[1] = __uint_as_float(q.x & 0xFFFF0000u);
    z[2] = __uint_as_float(q.y << 16); z[3] = __uint_as_float(q.y & 0xFFFF0000u);
  }
#pragma unroll
  for (int j = 0; j < 4; ++j)
    if (e0 + j >= r.V) z[j] = -INFINITY;
  if (r.has_pen) {
    const uint32_t word = r.bm[e0 >> 5];
    const int sh = e0 & 31;
    uint32_t nib = (word >> sh) & 0xFu;
    if (nib) {
      uint32_t rank = r.pre[e0 >> 5] + __popc(word & ((1u << sh) - 1u));
#pragma unroll
      for (int j = 0; j < 4; ++j)
        if ((nib >> j) & 1u) z[j] = r.side_z[rank++];
    }
  }
}

template <int DT>
__device__ __forceinline__ float load_one(const RowView& r, int v) {
  float z[4];
  load_group<DT>(r, v & ~3, z);
  return z[v & 3];
}

__device__ __forceinline__ float scaled(const RowView& r, float z) {
  return r.greedy ? z : __fdiv_rn(z, r.tau);
}
__device__ __forceinline__ unsigned long long mass_of(const RowView& r, float s) {
  return fix_of(expf(__fsub_rn(s, r.m)));
}

// f(index, z') for every element of the row; each wave walks its own contiguous range.
template <int DT, class F>
__device__ __forceinline__ void for_each_elem(const RowView& r, F&& f) {
  const int wbase = wave_id() * r.wave_range;
  for (int off = lane_id() * 4; off < r.wave_range; off += 256) {
    const int e0 = wbase + off;
    if (e0 >= r.V) break;
    float z[4];
    load_group<DT>(r, e0, z);
#pragma unroll
    for (int j = 0; j < 4; ++j)
      if (e0 + j < r.V) f(e0 + j, z[j]);
  }
}

__device__ __forceinline__ unsigned long long block_sum_u64(unsigned long long v, ExactShared& sh) {
  v = wave_sum_u64(v);
  __syncthreads();
  if (lane_id() == 0) sh.red64[wave_id()] = v;
  __syncthreads();
  unsigned long long t = 0;
  for (int w = 0; w < ((int)blockDim.x >> 6); ++w) t += sh.red64[w];
  return t;
}

// exclusive prefix over the 1024 threads, and the grand total
__device__ __forceinline__ uint32_t block_excl_scan_u32(uint32_t v, ExactShared& sh, uint32_t& total) {
  const uint32_t incl = wave_incl_scan_u32(v);
  __syncthreads();
  if (lane_id() == kWave - 1) sh.red32[wave_id()] = incl;
  __syncthreads();
  uint32_t off = 0, tot = 0;
  for (int w = 0; w < ((int)blockDim.x >> 6); ++w) {
    const uint32_t t = sh.red32[w];
    if (w < wave_id()) off += t;
    tot += t;
  }
  total = tot;
  return off + incl - v;
}

// Histogram adders that merge runs of equal digits before touching LDS: the leading digits
// of a row's keys are nearly constant, and same-address LDS atomics serialise.
struct CountRuns {
  uint32_t* h; int cur; uint32_t n;
  __device__ CountRuns(uint32_t* h_) : h(h_), cur(-1), n(0) {}
  __device__ __forceinline__ void add(int d) {
    if (d != cur) { flush(); cur = d; }
    ++n;
  }
  __device__ __forceinline__ void flush() { if (n) atomicAdd(&h[cur], n); n = 0; }
};
struct MassRuns {
  uint32_t* hc; unsigned long long* hm; int cur; uint32_t n; unsigned long long w;
  __device__ MassRuns(uint32_t* c, unsigned long long* m) : hc(c), hm(m), cur(-1), n(0), w(0) {}
  __device__ __forceinline__ void add(int d, unsigned long long x) {
    if (d != cur) { flush(); cur = d; }
    ++n; w += x;
  }
  __device__ __forceinline__ void flush() {
    if (n) { atomicAdd(&hc[cur], n); if (w) atomicAdd(&hm[cur], w); }
    n = 0; w = 0;
  }
};

// Wave 0: the digit d with  sum_{d'>d} cnt < k <= sum_{d'>=d} cnt  (1 <= k <= total).
__device__ __forceinline__ void pick_count_digit(const uint32_t* cnt, uint32_t k, ExactShared& sh) {
  const int l = lane_id();
  uint32_t c[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) c[j] = cnt[4 * l + j];
  const uint32_t lane_tot = c[0] + c[1] + c[2] + c[3];
  const uint32_t incl = wave_incl_scan_u32(lane_tot);
  const uint32_t total = (uint32_t)__shfl((int)incl, kWave - 1, kWave);
  if (k > total) k = total;
  if (k < 1) k = 1;
  uint32_t ex = total - incl;            // everything in lanes above
#pragma unroll
  for (int j = 3; j >= 0; --j) {
    if (ex < k && k <= ex + c[j]) {
      sh.bc_u32[0] = 4 * l + j;          // digit
      sh.bc_u32[1] = ex;                 // keys strictly above this digit
      sh.bc_u32[2] = c[j];               // keys with this digit
    }
    ex += c[j];
  }
}

// Wave 0: the smallest non-empty digit d with  above + sum_{d'>d} mass < limit.
__device__ __forceinline__ void pick_mass_digit(const uint32_t* cnt, const unsigned long long* mass,
                                                unsigned long long above, unsigned long long limit,
                                                ExactShared& sh) {
  const int l = lane_id();
  uint32_t c[4];
  unsigned long long w[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) { c[j] = cnt[4 * l + j]; w[j] = mass[4 * l + j]; }
  const unsigned long long lane_tot = w[0] + w[1] + w[2] + w[3];
  const unsigned long long incl = wave_incl_scan_u64(lane_tot);
  const unsigned long long total = shfl_u64(incl, kWave - 1);
  unsigned long long ex = above + (total - incl);
  int best = 1 << 20, top = -1;
  unsigned long long best_ex = 0, top_ex = 0;
#pragma unroll
  for (int j = 3; j >= 0; --j) {
    if (c[j] > 0) {
      if (top < 0) { top = 4 * l + j; top_ex = ex; }
      if (ex < limit) { best = 4 * l + j; best_ex = ex; }
    }
    ex += w[j];
  }
  // lowest qualifying digit over the wave; if none qualifies (p <= 0), the highest non-empty one
  int b = best;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) b = min(b, __shfl_xor(b, o, kWave));
  int t = top;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) t = max(t, __shfl_xor(t, o, kWave));
  if (b < (1 << 20)) {
    if (best == b) { sh.bc_u32[0] = (uint32_t)b; sh.bc_u64[0] = best_ex; }
  } else if (top == t && t >= 0) {
    sh.bc_u32[0] = (uint32_t)t; sh.bc_u64[0] = top_ex;
  }
}

// k-th largest key (1-based) over elements accepted by `in(index, s, key)`; also how many
// accepted keys are strictly larger and how many are equal.
template <int DT, class In>
__device__ __forceinline__ uint32_t select_kth(const RowView& r, uint32_t k, ExactShared& sh, In&& in,
                                               uint32_t& n_greater, uint32_t& n_equal) {
  uint32_t prefix = 0, himask = 0, greater = 0, equal = 0;
  for (int shift = 24; shift >= 0; shift -= 8) {
    __syncthreads();
    if (threadIdx.x < 256) sh.hcnt[threadIdx.x] = 0;
    __syncthreads();
    CountRuns agg(sh.hcnt);
    for_each_elem<DT>(r, [&](int v, float z) {
      const float s = scaled(r, z);
      const uint32_t key = key_of(s);
      if ((key & himask) == prefix && in(v, s, key)) agg.add((int)((key >> shift) & 255u));
    });
    agg.flush();
    __syncthreads();
    if (wave_id() == 0) pick_count_digit(sh.hcnt, k, sh);
    __syncthreads();
    const uint32_t d = sh.bc_u32[0], ex = sh.bc_u32[1];
    equal = sh.bc_u32[2];
    k = (k > ex) ? k - ex : 1;
    greater += ex;
    prefix |= d << shift;
    himask |= 255u << shift;
  }
  n_greater = greater;
  n_equal = equal;
  return prefix;
}

// Nucleus threshold: the smallest key x present in K1 (keys >= key_k1) whose strictly-larger
// K1 mass is below `limit`.
template <int DT>
__device__ __forceinline__ uint32_t select_nucleus(const RowView& r, uint32_t key_k1, unsigned long long limit,
                                                   ExactShared& sh) {
  uint32_t prefix = 0, himask = 0;
  unsigned long long above = 0;
  for (int shift = 24; shift >= 0; shift -= 8) {
    __syncthreads();
    if (threadIdx.x < 256) { sh.hcnt[threadIdx.x] = 0; sh.hmass[threadIdx.x] = 0; }
    __syncthreads();
    MassRuns agg(sh.hcnt, sh.hmass);
    for_each_elem<DT>(r, [&](int, float z) {
      const float s = scaled(r, z);
      const uint32_t key = key_of(s);
      if ((key & himask) == prefix && key >= key_k1) agg.add((int)((key >> shift) & 255u), mass_of(r, s));
    });
    agg.flush();
    __syncthreads();
    if (wave_id() == 0) pick_mass_digit(sh.hcnt, sh.hmass, above, limit, sh);
    __syncthreads();
    prefix |= sh.bc_u32[0] << shift;
    above = sh.bc_u64[0];
    himask |= 255u << shift;
  }
  return prefix;
}

// First index v (vocabulary order) at which the running sum of weight(index, z') exceeds
// `target`.  Two passes: per-wave totals of contiguous ranges, then the one wave that holds
// the crossing walks its range again with lane-level prefixes.
template <int DT, class W>
__device__ __forceinline__ int first_crossing(const RowView& r, unsigned long long target, ExactShared& sh,
                                              W&& weight) {
  unsigned long long mine = 0;
  for_each_elem<DT>(r, [&](int v, float z) { mine += weight(v, z); });
  mine = wave_sum_u64(mine);
  __syncthreads();
  if (lane_id() == 0) sh.red64[wave_id()] = mine;
  if (threadIdx.x == 0) sh.bc_i32[0] = -1;
  __syncthreads();
  unsigned long long before = 0;
  for (int w = 0; w < wave_id(); ++w) before += sh.red64[w];
  if (before <= target && target < before + mine) {          // at most one wave
    const int wbase = wave_id() * r.wave_range;
    unsigned long long running = before;
    int found = -1;
    for (int off0 = 0; off0 < r.wave_range && wbase + off0 < r.V && found < 0; off0 += 256) {
      const int e0 = wbase + off0 + lane_id() * 4;
      unsigned long long w4[4] = {0, 0, 0, 0};
      if (e0 < r.V) {
        float z[4];
        load_group<DT>(r, e0, z);
#pragma unroll
        for (int j = 0; j < 4; ++j)
          if (e0 + j < r.V) w4[j] = weight(e0 + j, z[j]);
      }
      const unsigned long long lane_tot = w4[0] + w4[1] + w4[2] + w4[3];
      const unsigned long long incl = wave_incl_scan_u64(lane_tot);
      unsigned long long c = running + incl - lane_tot;
      int hit = -1;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        c += w4[j];
        if (hit < 0 && c > target) hit = e0 + j;
      }
      const unsigned long long ball = __ballot(hit >= 0);
      if (ball) found = __shfl(hit, __ffsll((long long)ball) - 1, kWave);
      running += shfl_u64(incl, kWave - 1);
    }
    if (lane_id() == 0) sh.bc_i32[0] = found;
  }
  __syncthreads();
  return sh.bc_i32[0];
}

template <typename T>
__device__ __forceinline__ T param_or(const T* p, int b, T dflt) { return p ? p[b] : dflt; }

// One row, start to finish, by the calling workgroup (any multiple of 64 threads up to 1024).
// `dyn` is 2 * ceil(V/32) words of LDS.  Not inlined: it is the rarely taken path of the
// finishing kernel and must not cost that kernel registers or instruction cache.
template <int DT>
__device__ __attribute__((noinline)) void exact_row(const Args& a, const int b, uint32_t* dyn, ExactShared& sh) {
  const int tid = threadIdx.x;
  const int V = a.V;
  const int W = (V + 31) >> 5;
  uint32_t* bm = dyn;
  uint32_t* pre = dyn + W;

  RowView r;
  r.row = reinterpret_cast<const char*>(a.logits) + (size_t)b * (size_t)a.row_stride * (DT == SIP_F32 ? 4 : 2);
  r.V = V;
  r.wave_range = (((V + ((int)blockDim.x >> 6) - 1) / ((int)blockDim.x >> 6)) + 255) & ~255;
  r.bm = bm; r.pre = pre;
  r.tau = param_or(a.p.temperature, b, 1.0f);
  const int top_k = param_or(a.p.top_k, b, 0);
  const float top_p = param_or(a.p.top_p, b, 1.0f);
  const float min_p = param_or(a.p.min_p, b, 0.0f);
  const float theta = param_or(a.p.repetition_penalty, b, 1.0f);
  const float phi = param_or(a.p.frequency_penalty, b, 0.0f);
  const float psi = param_or(a.p.presence_penalty, b, 0.0f);
  const unsigned long long row_id = a.p.row_id ? (unsigned long long)a.p.row_id[b] : (unsigned long long)b;
  r.greedy = (r.tau == 0.0f) || (top_k == 1);

  // ---- (1) history -> bitmap, ranks, multiplicities, penalised values  (Sec. 5.1 CalcPenalty)
  const PenaltyPlan pen = penalty_plan(a, b, theta, phi, psi);
  const long long lo = pen.h.lo, hi = pen.h.hi;
  r.has_pen = pen.any;
  r.side_z = a.side_z + pen.side;
  if (r.has_pen) {
    float* side_z = a.side_z + pen.side;
    unsigned int* side_c = a.side_c + pen.side;
    for (int w = tid; w < W; w += (int)blockDim.x) bm[w] = 0;
    __syncthreads();
    for (long long i = lo + tid; i < hi; i += (int)blockDim.x) {
      const int t = a.tokens[i];
      if (t >= 0 && t < V) atomicOr(&bm[t >> 5], 1u << (t & 31));
    }
    for (long long i = pen.p_lo + tid; i < pen.p_hi; i += (int)blockDim.x) {     // a separate prompt: presence only
      const int t = a.p_tokens[i];
      if (t >= 0 && t < V) atomicOr(&bm[t >> 5], 1u << (t & 31));
    }
    __syncthreads();
    const int per = (W + (int)blockDim.x - 1) / (int)blockDim.x;
    const int w0 = tid * per, w1 = min(W, w0 + per);
    uint32_t local = 0;
    for (int w = w0; w < w1; ++w) local += __popc(bm[w]);
    uint32_t ndist;
    uint32_t run = block_excl_scan_u32(local, sh, ndist);
    for (int w = w0; w < w1; ++w) { pre[w] = run; run += __popc(bm[w]); }
    __syncthreads();
    const bool need_counts = pen.counts;
    if (need_counts) {
      for (uint32_t i = tid; i < ndist; i += (int)blockDim.x) side_c[i] = 0;
      __threadfence();
      __syncthreads();
      for (long long i = lo + tid; i < hi; i += (int)blockDim.x) {
        const int t = a.tokens[i];
        if (t >= 0 && t < V) {
          const uint32_t word = bm[t >> 5];
          const uint32_t rank = pre[t >> 5] + __popc(word & ((1u << (t & 31)) - 1u));
          atomicAdd(&side_c[rank], 1u);
        }
      }
      __threadfence();
      __syncthreads();
    }
    // penalised value of every distinct token: repetition, then frequency, then presence,
    // one fp32 rounding per operation
    RowView raw = r;
    raw.has_pen = false;
    for (int w = tid; w < W; w += (int)blockDim.x) {
      uint32_t bits = bm[w];
      uint32_t rank = pre[w];
      while (bits) {
        const int v = (w << 5) + __ffs((int)bits) - 1;
        bits &= bits - 1;
        const float z = load_one<DT>(raw, v);
        unsigned int c = pen.dflt;
        if (need_counts) c = __hip_atomic_load(&side_c[rank], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        side_z[rank] = penalise(z, c, theta, phi, psi);
        ++rank;
      }
    }
    __threadfence();
    __syncthreads();
  }

  // ---- (2) maximum of z' and its lowest index
  float best = -INFINITY;
  int best_i = 0x7FFFFFFF;
  for_each_elem<DT>(r, [&](int v, float z) {
    if (z > best || (z == best && v < best_i)) { best = z; best_i = v; }
  });
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const float ob = __shfl_xor(best, o, kWave);
    const int oi = __shfl_xor(best_i, o, kWave);
    if (ob > best || (ob == best && oi < best_i)) { best = ob; best_i = oi; }
  }
  if (lane_id() == 0) { sh.redf[wave_id()] = best; sh.redi[wave_id()] = best_i; }
  __syncthreads();
  best = sh.redf[0]; best_i = sh.redi[0];
  for (int w = 1; w < ((int)blockDim.x >> 6); ++w) {
    const float ob = sh.redf[w]; const int oi = sh.redi[w];
    if (ob > best || (ob == best && oi < best_i)) { best = ob; best_i = oi; }
  }
  if (best_i == 0x7FFFFFFF) best_i = 0;
  r.m = scaled(r, best);

  // ---- (3) total mass -> ln sum exp
  unsigned long long part = 0;
  for_each_elem<DT>(r, [&](int, float z) { part += mass_of(r, scaled(r, z)); });
  const unsigned long long S0 = block_sum_u64(part, sh);
  const double lnZ = log((double)S0) - (double)kFixShift * 0.6931471805599453094;

  int token = best_i;
  if (!r.greedy) {
    // ---- (4) top-k
    uint32_t key_k = 0;
    unsigned long long S1 = S0;
    if (top_k >= 2 && top_k < V) {
      uint32_t g, e;
      key_k = select_kth<DT>(r, (uint32_t)top_k, sh, [](int, float, uint32_t) { return true; }, g, e);
      unsigned long long p1 = 0;
      for_each_elem<DT>(r, [&](int, float z) {
        const float s = scaled(r, z);
        if (key_of(s) >= key_k) p1 += mass_of(r, s);
      });
      S1 = block_sum_u64(p1, sh);
    }
    // ---- (5) top-p on the mass that survived top-k
    uint32_t key_cut = key_k;
    if (top_p < 1.0f) {
      const double lim = ceil((double)top_p * (double)S1);
      const unsigned long long limit = lim > 0.0 ? (unsigned long long)lim : 0ull;
      const uint32_t key_p = select_nucleus<DT>(r, key_k, limit, sh);
      key_cut = max(key_k, key_p);
    }
    // ---- (6) min-p
    const bool minp_on = min_p > 0.0f;
    const float t_minp = minp_on ? (float)log((double)min_p) : 0.0f;
    auto kept_mass = [&](int, float z) -> unsigned long long {
      const float s = scaled(r, z);
      if (key_of(s) < key_cut) return 0ull;
      if (minp_on && !(__fsub_rn(s, r.m) >= t_minp)) return 0ull;
      return mass_of(r, s);
    };
    // ---- (7) draw: first index whose running kept mass exceeds u * S3, u = (x0 >> 8) / 2^24
    unsigned long long p3 = 0;
    for_each_elem<DT>(r, [&](int v, float z) { p3 += kept_mass(v, z); });
    const unsigned long long S3 = block_sum_u64(p3, sh);
    const unsigned long long j = philox_word0(a.seed, row_id, step_of(a)) >> 8;
    // floor(j * S3 / 2^24), exact in 128-bit integer arithmetic
    const unsigned long long target = (__umul64hi(j, S3) << 40) | ((j * S3) >> 24);
    const int hit = first_crossing<DT>(r, target, sh, kept_mass);
    token = hit >= 0 ? hit : best_i;
  }
  if (tid == 0) a.out_ids[b] = token;

  // ---- (8) log-probabilities: sampled token, then the n best of the whole vocabulary
  if (a.k_lp >= 0) {
    const int cols = 1 + a.k_lp;
    if (tid == 0) {
      const float s = scaled(r, load_one<DT>(r, token));
      a.out_lp_ids[(size_t)b * cols] = token;
      a.out_lp[(size_t)b * cols] = (float)((double)s - (double)r.m - lnZ);
    }
    const int n = min(a.k_lp, V);
    for (int c = n + tid; c < a.k_lp; c += (int)blockDim.x) {      // vocabulary smaller than k_logprobs
      a.out_lp_ids[(size_t)b * cols + 1 + c] = -1;
      a.out_lp[(size_t)b * cols + 1 + c] = -INFINITY;
    }
    if (n > 0) {
      uint32_t g, e;
      const uint32_t key_n = select_kth<DT>(r, (uint32_t)n, sh, [](int, float, uint32_t) { return true; }, g, e);
      const uint32_t need_eq = (uint32_t)n - g;                  // >= 1
      int idx_limit = 0x7FFFFFFF;
      if (e > need_eq) {
        idx_limit = first_crossing<DT>(r, (unsigned long long)need_eq - 1ull, sh,
                                       [&](int, float z) -> unsigned long long {
                                         return key_of(scaled(r, z)) == key_n ? 1ull : 0ull;
                                       });
      }
      if (tid == 0) sh.tn_cnt = 0;
      __syncthreads();
      for_each_elem<DT>(r, [&](int v, float z) {
        const float s = scaled(r, z);
        const uint32_t key = key_of(s);
        if (key > key_n || (key == key_n && v <= idx_limit)) {
          const uint32_t slot = atomicAdd(&sh.tn_cnt, 1u);
          if (slot < (uint32_t)SIP_MAX_K_LOGPROBS) { sh.tn_key[slot] = key; sh.tn_idx[slot] = v; sh.tn_s[slot] = s; }
        }
      });
      __syncthreads();
      const int got = min((int)sh.tn_cnt, n);
      if (tid < got) {
        const uint32_t key = sh.tn_key[tid];
        const int v = sh.tn_idx[tid];
        int rank = 0;
        for (int q = 0; q < got; ++q) {
          const uint32_t kq = sh.tn_key[q];
          rank += (kq > key || (kq == key && sh.tn_idx[q] < v)) ? 1 : 0;
        }
        a.out_lp_ids[(size_t)b * cols + 1 + rank] = v;
        a.out_lp[(size_t)b * cols + 1 + rank] = (float)((double)sh.tn_s[tid] - (double)r.m - lnZ);
      }
    }
  }
}

template <int DT, bool SH>
__global__ __launch_bounds__(kExactThreads) void exact_kernel(Args a) {
  extern __shared__ uint32_t dyn[];
  __shared__ ExactShared sh;
  if (SH) gather_row<DT>(a, blockIdx.x);                  // sharded logits: the row is put together first
  exact_row<DT>(a, blockIdx.x, dyn, sh);
  if (threadIdx.x == 0) { a.row_path[blockIdx.x] = 14; a.row_why[blockIdx.x] = 14; }   // 14: shape outside the single-pass kernels
  if (a.slot) {                                          // device-resident history: the row's id joins it
    __syncthreads();
    if (threadIdx.x == 0) state_append_row(a, blockIdx.x);
  }
}

}  // namespace sip
