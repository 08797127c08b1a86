// Single pass over the logits: the only kernel that touches all B*V elements.
//
// A row is cut into S chunks, one 512-thread workgroup each.  The workgroup never learns the
// row's maximum; instead it picks, from a 8192-element sample spread over the row, a value
// threshold Tc such that only the top ~1-3 % of the row lies at or above it, and then streams
// its chunk once:
//   * elements >= Tc ("candidates") are collected, value and index, in per-wave LDS queues
//     (a wave that finds more than its queue holds reports an overflow and the row falls back
//     to the exact path) and written out to per-wave segments in the workspace at the end --
//     every question that needs exact
//     values (top-k, top-p, min-p, draw, best-n, maximum) is answered later from these few
//     thousand entries per row;
//   * all other elements only contribute their softmax mass 2^(z*c - R), c = log2(e)/tau,
//     R = ceil(Tc*c).  Because z < Tc, every term is <= 1: no running maximum, no rescaling
//     (Sec. 5.1 row-wise softmax, here fused with temperature scaling).  Each thread adds its
//     terms in fp32 in a fixed order; the per-thread sums are combined as integers in units
//     of 2^-30.
// History penalties (Sec. 5.1 ApplyPenalty) touch at most |history| elements of a row.  The
// workgroup marks the row's history tokens that fall into its chunk in an LDS bitmap (one bit
// per element of the chunk); an element whose bit is set goes into the list whatever its
// value, tagged, and stays out of the bulk mass, so that the finishing kernel finds the raw
// logit of every token it has to penalise in the list and never reads the logits itself.
#pragma once
#include "sip_device.h"

namespace sip {

constexpr int kStreamThreads = 512;
constexpr int kStreamWaves = kStreamThreads / kWave;
static_assert(kStreamWaves == 8, "a chunk's segment is made of eight wave queues");
constexpr int kStreamLoads = 2;             // 16-byte loads per thread per tile
constexpr int kStreamBufs = 2;              // tiles held in registers: one being processed, the others in flight
constexpr int kSampleBins = 8192;           // 13-bit keys: sign, exponent, 4 mantissa bits
constexpr int kSampleSize = 8192;           // elements of a row the threshold is estimated from
constexpr int kQueueCap = 480;              // entries of one wave's LDS candidate queue
constexpr int kChunkCap = kStreamWaves * kQueueCap;   // entries of one chunk's segment in the workspace
constexpr int kChunkBitsMax = 73728;        // most elements a chunk may have (history bitmap: 9 KB of LDS)
constexpr int kStreamHistRegs = 8;          // history tokens a thread requests at once
constexpr float kBulkScale = 1073741824.0f; // 2^30

// Per-row decisions shared by the streaming and the finishing kernel.
struct RowParams {
  float tau, top_p, min_p, theta, phi, psi;
  int top_k;
  unsigned long long row_id;
  bool greedy;
};

__device__ __forceinline__ RowParams load_row_params(const Args& a, int b) {
  RowParams r;
  r.tau = a.p.temperature ? a.p.temperature[b] : 1.0f;
  r.top_k = a.p.top_k ? a.p.top_k[b] : 0;
  r.top_p = a.p.top_p ? a.p.top_p[b] : 1.0f;
  r.min_p = a.p.min_p ? a.p.min_p[b] : 0.0f;
  r.theta = a.p.repetition_penalty ? a.p.repetition_penalty[b] : 1.0f;
  r.phi = a.p.frequency_penalty ? a.p.frequency_penalty[b] : 0.0f;
  r.psi = a.p.presence_penalty ? a.p.presence_penalty[b] : 0.0f;
  r.row_id = a.p.row_id ? (unsigned long long)a.p.row_id[b] : (unsigned long long)b;
  r.greedy = (r.tau == 0.0f) || (r.top_k == 1);
  return r;
}

// The threshold of a row whose list is to hold `target` entries is the j-th largest value of a
// sample, j = target * (sample size) / V, so the list comes out at target * (1 +- 1/sqrt(j)).
// Lists of kWholeFrom entries and more are the ones that may outgrow the 4096 entries of the
// finishing kernel's faster variants (twice the time for that row), so they are estimated from
// the whole sample of kSampleSize elements as long as that keeps j small (<= kTailRank: a thread
// then only tracks its three largest values); every other list from every other sample block.
constexpr int kTailRank = 256;
constexpr int kWholeFrom = 2048;
__device__ __forceinline__ bool whole_sample(int target, int V) {
  // ceil(target * kSampleSize / V) <= kTailRank, without the division (target <= 2^14, V <= 2^19)
  return target >= kWholeFrom && (uint32_t)target * (uint32_t)kSampleSize <= (uint32_t)kTailRank * (uint32_t)V;
}

// How many of the row's largest elements the candidate list should hold; 0 = this row
// cannot be finished from a candidate list (k is too large) and takes the exact multi-pass
// path instead.
__device__ __forceinline__ int candidate_target(const RowParams& r, const Args& a) {
  if (!(r.tau >= 0.0f)) return 0;
  if (r.greedy) return 512;
  const int k = (r.top_k >= 2 && r.top_k < a.V) ? r.top_k : 0;
  const bool p_on = r.top_p < 1.0f, minp_on = r.min_p > 0.0f;
  if (k == 0 && !p_on && !minp_on) return 1024;       // plain temperature sampling: the list serves the maximum
                                                      // and best-n, the draw re-reads the row
  int t;
  if (k > 0) {
    // top-k needs its k largest in the list.  The threshold is the j-th largest of kSampleSize
    // sampled values, j = t * kSampleSize / V, so the list comes out t * (1 +- 1/sqrt(j)): ask
    // for 3.5 such deviations more than k (whatever top-p and min-p do afterwards happens
    // inside those k)
    t = k + 256 + (int)(3.5f * sqrtf((float)k * (float)a.V * (1.0f / (float)kSampleSize)));
    if (!whole_sample(t, a.V)) t = k + 256 + (int)(3.5f * sqrtf((float)k * (float)a.V * (2.0f / (float)kSampleSize)));
  } else {
    // a nucleus with nothing else to bound it tends to be longer than one cut by min-p, so it
    // starts from a longer list -- as long as still fits the 8 entries per thread of the
    // finishing kernel's faster variants
    t = minp_on ? 1920 : 2816;
    // min-p keeps what lies within tau * ln(1/min_p) of the maximum: the list must reach that
    // far down, and how many elements that is grows quickly with the temperature
    if (minp_on && r.min_p < 1.0f) t = max(t, 1280 + (int)(400.0f * r.tau * -__logf(r.min_p)));
  }
  // the threshold comes from a sample: allow for a list a quarter longer than asked for
  if (t + (t >> 2) > a.nc_cap) return 0;
  return t;
}

// log2(e)/tau as an unevaluated fp32 sum hi + lo (greedy rows: tau = 1)
__device__ __forceinline__ void scale_pair(const RowParams& r, float& hi, float& lo) {
  const double c = 1.4426950408889634074 / (r.greedy ? 1.0 : (double)r.tau);
  hi = (float)c;
  lo = (float)(c - (double)hi);
}

// Softmax mass of a non-candidate element relative to the threshold: 2^((z - Tc) * c + r0)
// with c = log2(e)/tau and r0 = Tc*c - ceil(Tc*c) in (-1, 0], i.e. 2^(z*c - R).  Taking the
// difference to Tc first keeps the product small where the term is not negligible, so one
// fp32 multiplier is accurate enough; z = -inf gives exactly 0.
struct BulkRef {
  float Tc, c, r0;
  int R;
};
__device__ __forceinline__ BulkRef make_bulk_ref(float Tc, const RowParams& rp) {
  float chi, clo;
  scale_pair(rp, chi, clo);
  const double tc = (double)Tc * ((double)chi + (double)clo);
  BulkRef r;
  r.Tc = Tc; r.c = chi; r.R = 0; r.r0 = 0.0f;
  const double tr = ceil(tc);
  if (tr > -1048576.0 && tr < 1048576.0) { r.R = (int)tr; r.r0 = (float)(tc - tr); }
  return r;
}
__device__ __forceinline__ float bulk_term(float z, const BulkRef& r) {
  return __builtin_amdgcn_exp2f(__fmaf_rn(__fsub_rn(z, r.Tc), r.c, r.r0));
}
// per-thread fp32 partial sum -> integer units of 2^-30
__device__ __forceinline__ unsigned long long bulk_units(float acc) {
  return acc > 0.0f ? (unsigned long long)(acc * kBulkScale) : 0ull;
}


template <int DT, bool SH>
__global__ __launch_bounds__(kStreamThreads) __attribute__((amdgpu_waves_per_eu(8, 8))) void stream_kernel(Args a) {
  constexpr int EPL = (DT == SIP_F32) ? 4 : 8;      // elements per 16-byte load
  constexpr int ESZ = (DT == SIP_F32) ? 4 : 2;
  constexpr int SUB = kStreamThreads * EPL;         // elements per workgroup-wide load
  constexpr int TILE = SUB * kStreamLoads;
  constexpr int SLOADS = kSampleSize / SUB;         // sample loads per thread (4 fp32, 2 bf16)
  constexpr int NSB = SLOADS * kStreamWaves;        // 1 KB sample blocks spread over the row
  // 30 KB of LDS: first the sample histogram (two 16-bit counters per word, 16 KB), then the
  // per-wave candidate queues; 9 KB for the history bitmap of the chunk (39.6 KB in all: four
  // workgroups per compute unit)
  __shared__ __align__(16) unsigned char smem[(kSampleBins * 2 > kStreamWaves * kQueueCap * 8) ? kSampleBins * 2 : kStreamWaves * kQueueCap * 8];
  __shared__ uint32_t bmw[kChunkBitsMax / 32];
  uint32_t* hist = reinterpret_cast<uint32_t*>(smem);
  __shared__ uint32_t red32[kStreamWaves];
  __shared__ unsigned long long red64[kStreamWaves];
  __shared__ uint32_t wave_cnt[kStreamWaves];
  __shared__ uint32_t key_thr, need_thr;            // 13-bit key of the threshold bin; entries still wanted from inside it
  __shared__ uint32_t sub_hist[32];                 // that bin, split by the next 5 key bits

  const int tid = threadIdx.x, lane = lane_id(), wave = wave_id();
  // Workgroups are handed to the 8 XCDs round-robin by their id.  The chunks of one row read
  // the same sample, so they are renumbered to land on the same XCD (and its L2): id i works
  // on logical chunk (i % 8) * (n / 8) + i / 8 when n, the grid size, is a multiple of 8.
  int wg = blockIdx.x;
  if ((gridDim.x & 7) == 0) wg = (blockIdx.x & 7) * (gridDim.x >> 3) + (blockIdx.x >> 3);
  const int b = wg / a.S, ch = wg - b * a.S;
  const int V = a.V;
  // SH (vocabulary-sharded logits): the row's chunks are dealt out to the shards, S / t_shards
  // each, and a chunk lies inside its shard; c0, c1 and every element index below are then
  // relative to the shard, `ibase` being the shard's first vocabulary id.
  // With more chunks than shards a chunk is a part of one shard (np = 1 piece); with fewer, it is
  // np whole shards in a row, streamed one after the other.
  const bool split = !SH || a.S >= a.t_shards;       // uniform
  const int S_sh = !SH ? a.S : (split ? a.S / a.t_shards : 1);
  const int np = (SH && !split) ? a.t_shards / a.S : 1;
  const int sh = !SH ? 0 : (split ? ch / S_sh : ch * np);
  const int lc = !SH ? ch : (split ? ch - sh * S_sh : 0);
  const int Vl = SH ? a.V_shard : V;
  const uint32_t ibase = SH ? (uint32_t)(sh * Vl) : 0u;
  const int c0 = chunk_begin(lc, Vl, S_sh, kWave * EPL);
  const int c1 = chunk_begin(lc + 1, Vl, S_sh, kWave * EPL);
  if (c0 >= c1) return;                              // host guarantees every chunk is non-empty
  const char* row = SH ? shard_base(a, sh) + (size_t)b * (size_t)a.shard_stride * ESZ      // (moves on with the pieces)
                       : reinterpret_cast<const char*>(a.logits) + (size_t)b * (size_t)a.row_stride * ESZ;

  // Loads are unconditional (a select on the loaded value would make the wave wait for it at
  // once): lanes past the end of the chunk re-read its last 16 bytes and `process` discards
  // what they hold by index.
  const int e_last = ((c1 - 1) / EPL) * EPL;
  auto load_tile = [&](int t0, uint4 (&buf)[kStreamLoads]) {
#pragma unroll
    for (int j = 0; j < kStreamLoads; ++j) {
      const int e0 = min(t0 + j * SUB + tid * EPL, e_last);
      buf[j] = *reinterpret_cast<const uint4*>(row + (size_t)e0 * ESZ);
    }
  };
  auto unpack = [&](const uint4& q, float (&z)[EPL]) {
    if (DT == SIP_F32) {
      z[0] = __uint_as_float(q.x); z[1] = __uint_as_float(q.y);
      z[2] = __uint_as_float(q.z); z[3] = __uint_as_float(q.w);
    } else {
      const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        z[2 * i] = __uint_as_float(w[i] << 16);
        z[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
      }
    }
  };

  // ---- The row's small records -- parameters, history and prompt extents -- are read first, all
  // at once and without a branch in between (where branches meet, the compiler waits for every
  // load in flight).  Their addresses are the same for the whole workgroup and nothing has been
  // stored by this kernel so far, so the compiler reads them through the scalar cache into scalar
  // registers: one round trip, and no vector registers held while they travel.  What a call does
  // not have (a NULL parameter array, no history) is read from memory that is there anyway and
  // replaced by its default afterwards.
  const char* const dummy = reinterpret_cast<const char*>(a.chunks);
  auto rec = [&](const void* arr, size_t off) { return arr ? reinterpret_cast<const char*>(arr) + off : dummy; };
  const bool csr_on = !a.slot && a.indptr && a.tokens && a.nnz > 0;
  const bool prompt_csr = a.p_indptr && a.p_tokens && a.p_nnz > 0;
  const float r_tau = *reinterpret_cast<const float*>(rec(a.p.temperature, 4 * (size_t)b));
  const int r_k = *reinterpret_cast<const int*>(rec(a.p.top_k, 4 * (size_t)b));
  const float r_p = *reinterpret_cast<const float*>(rec(a.p.top_p, 4 * (size_t)b));
  const float r_minp = *reinterpret_cast<const float*>(rec(a.p.min_p, 4 * (size_t)b));
  const float r_theta = *reinterpret_cast<const float*>(rec(a.p.repetition_penalty, 4 * (size_t)b));
  const float r_phi = *reinterpret_cast<const float*>(rec(a.p.frequency_penalty, 4 * (size_t)b));
  const float r_psi = *reinterpret_cast<const float*>(rec(a.p.presence_penalty, 4 * (size_t)b));
  const long long r_id = *reinterpret_cast<const long long*>(rec(a.p.row_id, 8 * (size_t)b));
  const long long r_h0 = *reinterpret_cast<const long long*>(rec(csr_on ? a.indptr : nullptr, 8 * (size_t)b));
  const long long r_h1 = *reinterpret_cast<const long long*>(rec(csr_on ? a.indptr : nullptr, 8 * (size_t)b + 8));
  const long long r_p0 = *reinterpret_cast<const long long*>(rec(prompt_csr ? a.p_indptr : nullptr, 8 * (size_t)b));
  const long long r_p1 = *reinterpret_cast<const long long*>(rec(prompt_csr ? a.p_indptr : nullptr, 8 * (size_t)b + 8));
  // (all of them are named here, once: otherwise the compiler moves each read to the branch that
  // first looks at its value, and the round trips follow one another)
  asm volatile("" ::"s"(r_tau), "s"(r_k), "s"(r_p), "s"(r_minp), "s"(r_theta), "s"(r_phi), "s"(r_psi), "s"(r_id),
               "s"(r_h0), "s"(r_h1), "s"(r_p0), "s"(r_p1));
  // ---- the records: defaults for what the call does not have
  RowParams rp;
  rp.tau = a.p.temperature ? r_tau : 1.0f;
  rp.top_k = a.p.top_k ? r_k : 0;
  rp.top_p = a.p.top_p ? r_p : 1.0f;
  rp.min_p = a.p.min_p ? r_minp : 0.0f;
  rp.theta = a.p.repetition_penalty ? r_theta : 1.0f;
  rp.phi = a.p.frequency_penalty ? r_phi : 0.0f;
  rp.psi = a.p.presence_penalty ? r_psi : 0.0f;
  rp.row_id = a.p.row_id ? (unsigned long long)r_id : (unsigned long long)b;
  rp.greedy = (rp.tau == 0.0f) || (rp.top_k == 1);
  const int target = candidate_target(rp, a);
  // ---- What one thread of the grid does for the whole call.  Device-resident history: the call
  // takes its number from the state's call counter (one atomic add, so that calls in flight at once
  // on one state each get their own) and leaves it in the workspace, where the kernels behind this
  // one read it (step_of()).  The finishing kernel counts the rows it passes on from zero.
  // (Here, on the one path that every workgroup takes, and not before the records above have been
  // read: with no store ahead of them in the kernel the compiler reads them through the scalar
  // cache.)
  if (a.call_tick && blockIdx.x == 0 && tid == 0) *a.call_tick = atomicAdd(a.st_tick, 1ull);
  if (blockIdx.x == 0 && tid == 0) *a.rescue_n = 0;
  if (target == 0) {
    if (ch == 0 && tid == 0) a.rowinfo[b].target = 0;                        // the finishing kernel looks at nothing else
    return;
  }
  // ---- the first tiles of the chunk are requested before anything else is worked out, so that
  // they travel meanwhile
  uint4 buf[kStreamBufs][kStreamLoads];
  int tnext = c0;                                    // first element of the next tile to request
#pragma unroll
  for (int k = 0; k < kStreamBufs; ++k) {
    load_tile(tnext, buf[k]);                        // (past the chunk's end: its last 16 bytes again, never looked at)
    tnext += TILE;
  }

  // ---- threshold: the same 8192-element sample (1 KB blocks spread evenly over the row) is
  // read by every chunk of the row, so all chunks agree on Tc = the j-th largest sample value
  // rounded down to an 18-bit key (found in two levels: 13 bits, then 5 more), j / 8192 = target / V
  // (for long lists: half of the blocks, j / 4096 = target / V; see whole_sample())
  // All blocks are requested, whether or not the row's rank calls for the whole sample: a branch
  // around a load makes the compiler wait for that load where the branches meet, one exposed
  // memory latency per block.
  uint4 smp[SLOADS];
#pragma unroll
  for (int j = 0; j < SLOADS; ++j) {
    const int sb = wave * SLOADS + j;                  // even j: every other block of the row
    if (!SH) {
      const int e0 = (int)(((long long)sb * V / NSB) / (kWave * EPL)) * (kWave * EPL) + lane * EPL;
      smp[j] = *reinterpret_cast<const uint4*>(row + (size_t)e0 * ESZ);    // e0 + EPL <= V since V >= 16384
    } else {
      // the same NSB blocks for every chunk of the row, smp_bps to a shard (the last shard may get
      // fewer), evenly spread inside it; V_shard >= 8192, so a block fits
      // (wave-uniform, and said so: with a per-lane index the table of piece pointers would be read
      // through a vector load from the kernel-argument segment, and waiting for that one also waits
      // for the tiles requested above)
      const int ssh = __builtin_amdgcn_readfirstlane((sb * a.smp_inv) >> 16);   // sb / smp_bps
      const int e0 = (sb - ssh * a.smp_bps) * a.smp_step + lane * EPL;
      const char* srow = shard_base(a, ssh) + (size_t)b * (size_t)a.shard_stride * ESZ;
      smp[j] = *reinterpret_cast<const uint4*>(srow + (size_t)e0 * ESZ);
    }
  }
  const bool whole = whole_sample(target, V);        // workgroup-uniform, like everything about the threshold
  // ---- history bitmap of the chunk: bit (v - g0) for every history token v in [g0, g1), the
  // vocabulary ids this workgroup streams.  Requested here, entered after the first barrier.
  // (A device-resident state's extent takes two dependent reads of its own.)
  const HistRange hr = a.slot ? hist_range(a, b) : hist_range_csr(a, r_h0, r_h1);
  const PenaltyPlan pen = penalty_plan_of(a, hr, r_p0, r_p1, rp.theta, rp.phi, rp.psi);
  const bool has_pen = pen.any;                                                                       // uniform
  const bool hist_pen = has_pen && hr.hi > hr.lo;
  const int g0 = (int)ibase + c0;
  const int g1 = (!SH || split) ? (int)ibase + c1 : (int)ibase + np * Vl;
  if (ch == 0 && tid == 0) {               // the row's record for the finishing kernel
    RowInfo ri;
    ri.tau = rp.tau; ri.top_p = rp.top_p; ri.min_p = rp.min_p; ri.theta = rp.theta; ri.phi = rp.phi; ri.psi = rp.psi;
    ri.top_k = rp.top_k; ri.target = target | (pen.prompt_on ? kPromptFlag : 0);
    ri.row_id = rp.row_id; ri.lo = hr.lo; ri.hi = hr.hi;
    ri.slot = -1; ri.ndist = -1;
    if (a.slot) {
      const int sl = a.slot[b];
      if (sl >= 0 && sl < a.slots) { ri.slot = sl; ri.ndist = a.st_ndist[sl]; }
    }
    a.rowinfo[b] = ri;
  }
  int htok[kStreamHistRegs];
#pragma unroll
  for (int j = 0; j < kStreamHistRegs; ++j) {
    const long long i = hr.lo + tid + (long long)j * kStreamThreads;
    htok[j] = (hist_pen && i < hr.hi) ? a.tokens[i] : -1;
  }
  for (int i = tid; i < kSampleBins / 2; i += kStreamThreads) hist[i] = 0;
  for (int i = tid; i < kChunkBitsMax / 32; i += kStreamThreads) bmw[i] = 0;
  if (tid < 32) sub_hist[tid] = 0;
  __syncthreads();
  if (has_pen) {
    auto mark = [&](int t) {
      const uint32_t r = (uint32_t)(t - g0);
      if (t >= g0 && t < g1) atomicOr(&bmw[r >> 5], 1u << (r & 31));
    };
#pragma unroll
    for (int j = 0; j < kStreamHistRegs; ++j) mark(htok[j]);
    for (long long i0 = hr.lo + (long long)kStreamHistRegs * kStreamThreads; i0 < hr.hi;
         i0 += (long long)kStreamHistRegs * kStreamThreads) {
#pragma unroll
      for (int j = 0; j < kStreamHistRegs; ++j) {
        const long long i = i0 + tid + (long long)j * kStreamThreads;
        htok[j] = i < hr.hi ? a.tokens[i] : -1;
      }
#pragma unroll
      for (int j = 0; j < kStreamHistRegs; ++j) mark(htok[j]);
    }
    for (long long i = pen.p_lo + tid; i < pen.p_hi; i += kStreamThreads) mark(a.p_tokens[i]);   // separate prompt
  }
  // Only the upper tail of the sample matters.  When j is small, a thread enters just the
  // three largest of its values: far fewer LDS atomics, and hardly any on the same word.
  // (Should one thread hold more than three of the j largest, the threshold comes out a
  // little low, which only lengthens the candidate list.)
  const int n_smp = whole ? kSampleSize : kSampleSize / 2;
  uint32_t want = ((uint32_t)target * (uint32_t)n_smp + (uint32_t)V - 1u) / (uint32_t)V;     // < 2^32: target <= 2^14
  if (want < 2u) want = 2u;
  if (want > (uint32_t)n_smp) want = (uint32_t)n_smp;
  const uint32_t j = want;
  const bool tail_only = whole || j <= (uint32_t)(kTailRank / 2);
  uint32_t t0 = 0, t1 = 0, t2 = 0;                   // full keys of this thread's three largest sample values
  {
    if (tail_only) {
      // the three largest as floats, one maximum and two medians per value
      float f0 = -INFINITY, f1 = -INFINITY, f2 = -INFINITY;
#pragma unroll
      for (int l = 0; l < SLOADS; ++l) {
        if (!whole && (l & 1)) continue;
        float z[EPL];
        unpack(smp[l], z);
#pragma unroll
        for (int i = 0; i < EPL; ++i) {
          const float x = z[i];
          f2 = __builtin_amdgcn_fmed3f(f1, f2, x);
          f1 = __builtin_amdgcn_fmed3f(f0, f1, x);
          f0 = fmaxf(f0, x);
        }
      }
      t0 = key_of(f0); t1 = key_of(f1); t2 = key_of(f2);
    } else {
#pragma unroll
      for (int l = 0; l < SLOADS; l += 2) {
        float z[EPL];
        unpack(smp[l], z);
#pragma unroll
        for (int i = 0; i < EPL; ++i) {
          const uint32_t k13 = key_of(z[i]) >> 19;
          atomicAdd(&hist[k13 >> 1], (k13 & 1u) ? 0x10000u : 1u);
        }
      }
    }
    if (tail_only) {
      atomicAdd(&hist[t0 >> 20], ((t0 >> 19) & 1u) ? 0x10000u : 1u);
      atomicAdd(&hist[t1 >> 20], ((t1 >> 19) & 1u) ? 0x10000u : 1u);
      atomicAdd(&hist[t2 >> 20], ((t2 >> 19) & 1u) ? 0x10000u : 1u);
    }
  }
  __syncthreads();
  {
    constexpr int WPT = kSampleBins / 2 / kStreamThreads;      // words per thread (16)
    const int wtop = kSampleBins / 2 - tid * WPT;              // thread 0 owns the highest bins
    uint32_t local = 0;
#pragma unroll
    for (int i = 1; i <= WPT; ++i) { const uint32_t w = hist[wtop - i]; local += (w & 0xFFFFu) + (w >> 16); }
    const uint32_t incl_w = dpp_scan_add_u32(local);
    if (lane == kWave - 1) red32[wave] = incl_w;
    __syncthreads();
    uint32_t off = 0;
    for (int w = 0; w < wave; ++w) off += red32[w];
    const uint32_t incl = off + incl_w, excl = incl - local;
    if (excl < j && j <= incl) {
      uint32_t run = excl, found = 0, need = 1;      // run: sample values above the bin looked at
      for (int i = 1; i <= WPT; ++i) {
        const uint32_t w = hist[wtop - i];
        if (run + (w >> 16) >= j) { found = 2u * (uint32_t)(wtop - i) + 1u; need = j - run; break; }
        run += (w >> 16);
        if (run + (w & 0xFFFFu) >= j) { found = 2u * (uint32_t)(wtop - i); need = j - run; break; }
        run += (w & 0xFFFFu);
      }
      key_thr = found; need_thr = need;
    }
    __syncthreads();                                 // also: the histogram is dead from here on
  }
  // ---- second level: the threshold bin is as wide as 1/16 of its values (and bf16 logits
  // or a spike-and-bulk row put hundreds of sample values into it), so it is split by the
  // next 5 key bits and only as many of its sub-bins are taken as the target asks for
  {
    const uint32_t K = key_thr;
    auto enter = [&](uint32_t kf) {
      if ((kf >> 19) == K) atomicAdd(&sub_hist[(kf >> 14) & 31u], 1u);
    };
    if (tail_only) {
      enter(t0); enter(t1); enter(t2);
    } else {
#pragma unroll
      for (int l = 0; l < SLOADS; l += 2) {
        float z[EPL];
        unpack(smp[l], z);
#pragma unroll
        for (int i = 0; i < EPL; ++i) enter(key_of(z[i]));
      }
    }
    __syncthreads();
    if (wave == 0) {
      const uint32_t c = lane < 32 ? sub_hist[31 - min(lane, 31)] : 0u;       // lane l: sub-bin 31 - l, descending
      const uint32_t incl = dpp_scan_add_u32(c);
      const unsigned long long reach = __ballot(lane < 32 && incl >= need_thr);
      const uint32_t first = reach ? (uint32_t)__ffsll((long long)reach) - 1u : 31u;
      if (lane == 0) key_thr = (K << 5) | (31u - first);                       // 18-bit key from here on
    }
    __syncthreads();
  }
  // A row that is masked almost everywhere (-inf for all but a few hundred tokens, as a grammar
  // constraint leaves it) has fewer finite values in its sample than the list asks for, and the
  // threshold has landed among the -inf (keys up to 511 in 18 bits: -inf and the negative NaNs).
  // Then the lowest finite sample value is the threshold: the list takes every finite element
  // from there up, and what lies below it is bulk as usual.  (No finite sample value at all: the
  // lowest finite float, which makes the finishing kernel pass the row on.)
  if (key_thr <= 511u) {                                                       // workgroup-uniform
    float lo = INFINITY;
#pragma unroll
    for (int l = 0; l < SLOADS; ++l) {
      float z[EPL];
      unpack(smp[l], z);
#pragma unroll
      for (int i = 0; i < EPL; ++i)
        if (z[i] > -INFINITY && z[i] < lo) lo = z[i];
    }
    uint32_t klo = last_lane_u32(dpp_scan_min_u32(lo == INFINITY ? 0xFFFFFFFFu : key_of(lo)));
    __syncthreads();                                                           // red32 is free again
    if (lane == 0) red32[wave] = klo;
    __syncthreads();
    klo = red32[0];
#pragma unroll
    for (int w = 1; w < kStreamWaves; ++w) klo = min(klo, red32[w]);
    const uint32_t k18 = klo == 0xFFFFFFFFu ? 512u : max(klo >> 14, 512u);
    __syncthreads();
    if (tid == 0) key_thr = k18;
    __syncthreads();
  }
  const uint32_t kb = key_thr << 14;
  const float Tc = value_of(kb);
  const BulkRef ref = make_bulk_ref(Tc, rp);
  const int R = ref.R;

  // ---- stream
  uint2* queue = reinterpret_cast<uint2*>(smem) + wave * kQueueCap;          // this wave's LDS queue
  const unsigned char* bm8 = reinterpret_cast<const unsigned char*>(bmw);
  uint32_t qn = 0;                          // wave-uniform: list entries seen (entries beyond the queue are dropped)
  float acc = 0.0f;                         // this thread's bulk mass, fixed order of additions

  uint32_t ib = ibase;                      // SH: first vocabulary id of the piece being processed
  // `hb`: the history bits of the EPL elements (bit i: element e0 + i carries a penalty)
  auto process = [&](const uint4& q, int e0, bool guard, uint32_t hb) {
    float z[EPL];
    unpack(q, z);
    if (guard) {
#pragma unroll
      for (int i = 0; i < EPL; ++i)
        if (e0 + i >= c1) { z[i] = -INFINITY; hb &= ~(1u << i); }
    }
    float g = 0.0f;
#pragma unroll
    for (int i = 0; i < EPL; ++i) {
      // One comparison decides "at or above the threshold, or a history token": the history bit,
      // spread over the word, is or-ed into the value's bits, which turns a tagged value into a
      // NaN, and "not below" holds for every NaN.
      const uint32_t tagm = (uint32_t)((int)(hb << (31 - i)) >> 31);          // 0 or all ones
      const bool hit = !(__uint_as_float(__float_as_uint(z[i]) | tagm) < Tc);
      const unsigned long long mask = __ballot(hit);
      if (mask) {
        const uint32_t pos = qn + __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32),
                                      __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
        if (hit && pos < (uint32_t)kQueueCap)
          queue[pos] = make_uint2(__float_as_uint(z[i]), ((uint32_t)(e0 + i) + (SH ? ib : 0u)) | (tagm & kTagBit));
        qn += (uint32_t)__popcll(mask);
      }
      float e = bulk_term(z[i], ref);
      e = hit ? 0.0f : e;
      g += e;
    }
    acc += g;
  };
  // Element e0 of the piece being processed is bit (ib - ibase) + e0 - c0 of the bitmap, a
  // multiple of EPL: the bits of one 16-byte load are half a byte (fp32) or one byte (bf16).
  // Lanes past the end of the chunk read the last byte; `process` masks what they get.
  auto hist_bits = [&](int e0) -> uint32_t {
    const uint32_t bit0 = (uint32_t)(e0 - c0) + (SH ? ib - ibase : 0u);
    const uint32_t byte = bm8[min(bit0 >> 3, (uint32_t)(kChunkBitsMax / 8 - 1))];
    return DT == SIP_F32 ? (byte >> (bit0 & 4u)) & 0xFu : byte;
  };
  auto process_tile = [&](const uint4 (&buf)[kStreamLoads], int t0) {
    const bool partial = t0 + TILE > c1;
    uint32_t hb[kStreamLoads];
#pragma unroll
    for (int j = 0; j < kStreamLoads; ++j) hb[j] = hist_bits(t0 + j * SUB + tid * EPL);
#pragma unroll
    for (int j = 0; j < kStreamLoads; ++j) {
      const int e0 = t0 + j * SUB + tid * EPL;
      if (!partial) process(buf[j], e0, false, hb[j]);
      else if (t0 + j * SUB < c1) process(buf[j], e0, true, hb[j]);     // workgroup-uniform condition
    }
  };

  // kStreamBufs register buffers in rotation: while one tile is processed the loads of the
  // others are in flight
  if (!SH) {
    int tcur = c0;
    bool more = true;
    while (more) {
#pragma unroll
      for (int k = 0; k < kStreamBufs; ++k) {
        if (tcur < c1) {
          process_tile(buf[k], tcur);
          if (tnext < c1) load_tile(tnext, buf[k]);
          tnext += TILE;
          tcur += TILE;
        } else {
          more = false;
        }
      }
    }
  } else {
    // the same rotation over np pieces: every piece is [c0, c1) of its shard; the requests run
    // ahead of the processing across the piece boundaries (`row` is what load_tile reads from)
    int c_pj = 0, tcur = c0;                         // tile being processed
    int n_pj = 0;                                    // piece of the next tile to request, `tnext` its first element
    auto roll = [&]() {
      if (tnext >= c1) {
        ++n_pj; tnext = c0;
        if (n_pj < np) row = shard_base(a, sh + n_pj) + (size_t)b * (size_t)a.shard_stride * ESZ;
      }
    };
    roll();
    bool more = true;
    while (more) {
#pragma unroll
      for (int k = 0; k < kStreamBufs; ++k) {
        if (c_pj < np) {
          process_tile(buf[k], tcur);
          if (n_pj < np) { load_tile(tnext, buf[k]); tnext += TILE; roll(); }
          tcur += TILE;
          if (tcur >= c1) { ++c_pj; tcur = c0; ib += (uint32_t)Vl; }
        } else {
          more = false;
        }
      }
    }
  }
  // ---- chunk summary; the eight queues go out, one behind the other, to the chunk's segment
  // (no global stores inside the loop: they would force every wait on a tile load to drain the
  // whole memory queue)
  const unsigned long long wsum = dpp_scan_add_u64(bulk_units(acc));      // integer from here on
  if (lane == kWave - 1) { red64[wave] = wsum; wave_cnt[wave] = qn; }
  __syncthreads();
  uint32_t off = 0, tot = 0;
  bool overflow = false;
#pragma unroll
  for (int w = 0; w < kStreamWaves; ++w) {
    const uint32_t c = wave_cnt[w];
    overflow |= c > (uint32_t)kQueueCap;
    const uint32_t cc = min(c, (uint32_t)kQueueCap);
    if (w < wave) off += cc;
    tot += cc;
  }
  uint2* seg = a.cand + (size_t)wg * (size_t)kChunkCap + off;
  for (uint32_t i = lane; i < min(qn, (uint32_t)kQueueCap); i += kWave) seg[i] = queue[i];
  if (tid == 0) {
    ChunkOut o;
    o.bulk = 0;
#pragma unroll
    for (int w = 0; w < kStreamWaves; ++w) o.bulk += red64[w];
    o.Tc = Tc;
    o.R = R;
    o.cnt = overflow ? kCntOverflow : tot;
    o.pad[0] = o.pad[1] = o.pad[2] = 0;
    a.chunks[wg] = o;
  }
}

}  // namespace sip
