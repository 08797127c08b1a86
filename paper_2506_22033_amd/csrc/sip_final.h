// The heavier per-row logic of the single-pass path, for the rows that the finishing kernel
// (sip_finish.h) cannot settle from the list the streaming kernel left behind: rescue_row(),
// run by rescue_kernel on the rows queued for it or, in small batches, by the workgroup that
// just tried (sip_fused.h).  It tries, in this order,
//   - the row's list again in register variants that hold up to 24 entries per thread
//     (fast_row: lists of up to 12288 entries, as top_k in the thousands makes them), with the
//     history tokens' multiplicities from a bitmap over the vocabulary, popcount ranks and side
//     tables in LDS;
//   - a second, longer list, made by reading the row once more with a lower threshold
//     (restream_row), and the same logic on that one;
//   - the continuations over the whole row (whole_row_finish): a nucleus that reaches below any
//     list is cut by a radix descent on the exact fp32 s, and a row without any filter is drawn
//     over all its elements;
//   - the exact multi-pass path (sip_exact.h).
//
// fast_row keeps the list in registers: every thread holds its share of the entries (key,
// index, mass, value bin) from the moment they are read until the end.  Every sum is an
// integer sum (masses in units of 2^-40 of the maximum's mass), so no result depends on the
// order in which threads add.  Selection works on 2048 linear value bins between the
// completeness threshold and the maximum: one histogram locates the bin that holds the k-th
// largest value, the nucleus cut or the n-th best, and the handful of entries in that bin are
// then resolved by all-pairs comparison.  The draw does the same over 2048 bins of the
// vocabulary index.
//
// Whenever a list cannot prove the answer (a cut falls below the completeness threshold,
// a bin or a segment overflows, too many distinct history tokens, ...) fast_row returns a
// reason code > 1 and rescue_row goes on to the next of the above; 1 means the row is finished.
#pragma once
#include <type_traits>

#include "sip_device.h"
#include "sip_exact.h"
#include "sip_stream.h"

namespace sip {

constexpr int kFinalThreads = 512;
constexpr int kFinalWaves = kFinalThreads / kWave;
constexpr int kBins = 2048;
constexpr int kBinsPerThread = kBins / kFinalThreads;
constexpr int kMembers = 256;        // entries of one bin that can be resolved by all-pairs comparison
constexpr int kSideMax = 4096;       // distinct history tokens per row the fast path handles
constexpr int kMaxChunks = 16;       // chunks (= list segments) per row
constexpr int kTopList = kFinalThreads / 2 < 256 ? kFinalThreads / 2 : 256;        // entries at or above the bin of the n-th best (half a workgroup ranks them)
constexpr int kTokRegs = 8;          // history tokens a thread keeps in registers between phases
constexpr int kWordRegs = 16;        // bitmap words a thread owns (2^18 / 32 / kFinalThreads)
constexpr uint32_t kNoIdx = 0xFFFFFFFFu;
constexpr int kNeedLong = 30;        // internal: more history tokens than this variant holds per thread
constexpr int kNeedLongList = 31;    // internal: more candidates than this variant holds per thread
constexpr int kWholeRowCut = 32;     // internal: the nucleus cut lies below the list -- settle it, and draw, over the whole row
constexpr int kWholeRow = 33;        // internal: no filter at all -- draw over the whole row
constexpr int kCandLong = 24;        // candidate entries per thread of the largest variant

struct FastShared {
  float Tc[kMaxChunks];
  int R[kMaxChunks];
  unsigned long long bulk[kMaxChunks];
  uint32_t segoff[kMaxChunks + 1];
  unsigned long long r64[kFinalWaves];
  uint32_t r32[kFinalWaves];
  uint32_t rkey[kFinalWaves];
  uint32_t ridx[kFinalWaves];
  uint32_t fail_seg, anyc, dropped;
  float m_out, zmax_out, trow_out;      // for a second attempt: max of s, max of z', threshold used
  unsigned long long limit_out;         // for the whole-row continuation: top-p limit, ln Z, whether penalties apply
  double lnz_out;
  int has_pen_out;
  int retry_ok_out;                     // a second, longer list can hold the nucleus (lower bound on its length)
  uint32_t rq_n;                         // candidates found by the second pass
  const char* shard_row[8];             // sharded logits: this row's piece in every shard
  int ndist_out;                        // distinct history tokens of the row, -1 while not counted (thread 0 only)
  int bin_k, bin_n, bin_p, bin_low, bin_d;
  uint32_t above_k, above_n;
  uint32_t key_k, key_p, token_key;
  int token;
  unsigned long long s1_part, before_d;
  uint32_t n_memb, n_memb2, n_memb3;
  uint32_t m_key[kMembers];
  uint32_t m_idx[kMembers];
  unsigned long long m_E[kMembers];
  uint32_t n_top;
  uint32_t t_key[kTopList];
  uint32_t t_idx[kTopList];
};

// Bytes of dynamic LDS the finishing kernel needs for vocabulary V, before the candidates.
__host__ __device__ inline size_t final_lds_fixed(int V) {
  const size_t W = ((size_t)V + 31) / 32;
  return ((W * 4 + W * 2 + 15) / 16) * 16 + (size_t)kBins * 20 + (size_t)kSideMax * 8;
}

template <int DT>
__device__ __forceinline__ float load_elem(const char* row, int v) {
  if (DT == SIP_F32) return reinterpret_cast<const float*>(row)[v];
  return __uint_as_float((uint32_t)reinterpret_cast<const unsigned short*>(row)[v] << 16);
}


// One attempt at finishing row b from its candidate list.  CR / SR = candidate entries /
// distinct history tokens a thread can hold in registers: the list, once read, never goes to
// memory again -- each thread keeps its share with key, index, mass and value bin in
// registers, and the phases below talk to each other only through the LDS histograms and a few
// small gathered lists.  Every register round is unrolled code that costs time even when it
// holds nothing (0.5-0.7 us each), hence several instantiations and a caller that picks the
// smallest one that fits.  Returns 1 (finished), kNeedLong / kNeedLongList (the row does not fit
// SR / CR entries per thread) or a reason code > 1; outputs written before a failure are overwritten
// by the path that takes the row over.
template <int DT, int CR, int SR, bool SH>
__device__ __forceinline__ int fast_row(const Args& a, const int b, const RowParams& rp, unsigned char* dyn,
                                        FastShared& fs, const int S, const int cap_c) {
  constexpr int NT = kFinalThreads;
  constexpr int NE = CR + SR;                               // register entries per thread
  constexpr bool STORE = CR <= 8;
  typedef typename std::conditional<(NE <= 32), uint32_t, unsigned long long>::type mask_t;                           // keep mass and bin in registers too
  constexpr int NS = STORE ? NE : 1;
  const int tid = threadIdx.x, lane = lane_id(), wave = wave_id();
  const int V = a.V;
  const int W = (V + 31) >> 5;
  // ---- LDS carving
  uint32_t* bm = reinterpret_cast<uint32_t*>(dyn);
  unsigned short* pre = reinterpret_cast<unsigned short*>(dyn + (size_t)W * 4);
  unsigned char* p2 = dyn + (((size_t)W * 6 + 15) / 16) * 16;
  unsigned long long* hm = reinterpret_cast<unsigned long long*>(p2);      // value bins: mass
  unsigned long long* hd = hm + kBins;                                      // index bins: kept mass
  uint32_t* hc = reinterpret_cast<uint32_t*>(hd + kBins);                   // value bins: count
  uint32_t* cnt = hc + kBins;                                               // multiplicity per history slot
  uint32_t* stok = cnt + kSideMax;                                          // token per history slot
  const char* row = reinterpret_cast<const char*>(a.logits) + (size_t)b * (size_t)a.row_stride * (DT == SIP_F32 ? 4 : 2);
  auto scaled_s = [&](float z) { return rp.greedy ? z : __fdiv_rn(z, rp.tau); };

  // ---- (0) chunk summaries, history extent; clear the LDS tables meanwhile
  const PenaltyPlan pen = penalty_plan(a, b, rp.theta, rp.phi, rp.psi);
  const long long lo = pen.h.lo, hi = pen.h.hi;
  const bool has_pen = pen.any;
  const int nseg = S;                                       // one list segment per chunk
  if (tid == 0) {
    fs.fail_seg = 0; fs.anyc = 0; fs.dropped = 0;
    fs.bin_k = -1; fs.bin_n = -1; fs.bin_p = 1 << 30; fs.bin_low = 1 << 30; fs.bin_d = -1;
    fs.key_p = 0xFFFFFFFFu; fs.n_memb = 0; fs.n_memb2 = 0; fs.n_memb3 = 0; fs.n_top = 0;
    fs.token = 0x7FFFFFFF; fs.key_k = 0; fs.s1_part = 0;
  }
  if (SH && tid == 0) {                   // constant indices: the piece pointers come through scalar loads
#pragma unroll
    for (int i = 0; i < 8; ++i)
      if (i < a.t_shards)
        fs.shard_row[i] = reinterpret_cast<const char*>(a.shard[i]) + (size_t)b * (size_t)a.shard_stride * (DT == SIP_F32 ? 4 : 2);
  }
  if (tid < S) {
    const ChunkOut co = a.chunks[(size_t)b * a.S + tid];
    fs.Tc[tid] = co.Tc; fs.R[tid] = co.R; fs.bulk[tid] = co.bulk;
    fs.segoff[tid] = co.cnt;
  }
  // history tokens of this thread (the first kTokRegs rounds stay in registers)
  int tok[kTokRegs];
#pragma unroll
  for (int j = 0; j < kTokRegs; ++j) {
    const long long i = lo + tid + (long long)j * NT;
    tok[j] = (has_pen && i < hi) ? a.tokens[i] : -1;
  }
  {
    uint4* z4 = reinterpret_cast<uint4*>(p2);               // hm, hd, hc: kBins * 20 bytes
    for (int i = tid; i < kBins * 20 / 16; i += NT) z4[i] = make_uint4(0, 0, 0, 0);
  }
  if (has_pen) {
    for (int w = tid; w < W; w += NT) bm[w] = 0;
    for (int i = tid; i < kSideMax; i += NT) cnt[i] = 0;
  }
  // row constants that take long arithmetic, worked out while the loads above travel
  const bool minp_on = !rp.greedy && rp.min_p > 0.0f;
  const float t_minp = minp_on ? (float)log((double)rp.min_p) : 0.0f;
  const unsigned long long j24 = rp.greedy ? 0ull : (unsigned long long)(philox_word0(a.seed, rp.row_id, step_of(a)) >> 8);
  __syncthreads();

  // ---- (1) prefix of the segment sizes (wave 0); presence bitmap of the history (everyone)
  if (wave == 0) {
    const uint32_t c0 = 2 * lane < nseg ? fs.segoff[2 * lane] : 0u;
    const uint32_t c1 = 2 * lane + 1 < nseg ? fs.segoff[2 * lane + 1] : 0u;
    const uint32_t incl = dpp_scan_add_u32(c0 + c1);
    const uint32_t total = last_lane_u32(incl);
    if (c0 > (uint32_t)cap_c || c1 > (uint32_t)cap_c) fs.fail_seg = 1;       // a queue overflowed
    if (c0 + c1 < c0 || incl < c0 + c1) fs.fail_seg = 1;                       // (the overflow mark wraps the sums)
    if (2 * lane < nseg) fs.segoff[2 * lane] = incl - c0 - c1;
    if (2 * lane + 1 < nseg) fs.segoff[2 * lane + 1] = incl - c1;
    if (lane == 0) fs.segoff[nseg] = total;
  }
  if (has_pen) {
#pragma unroll
    for (int j = 0; j < kTokRegs; ++j) {
      const int t = tok[j];
      if (t >= 0 && t < V) atomicOr(&bm[t >> 5], 1u << (t & 31));
    }
    for (long long i = lo + tid + (long long)kTokRegs * NT; i < hi; i += NT) {
      const int t = a.tokens[i];
      if (t >= 0 && t < V) atomicOr(&bm[t >> 5], 1u << (t & 31));
    }
    for (long long i = pen.p_lo + tid; i < pen.p_hi; i += NT) {             // a separate prompt: presence only
      const int t = a.p_tokens[i];
      if (t >= 0 && t < V) atomicOr(&bm[t >> 5], 1u << (t & 31));
    }
  }
  __syncthreads();
  // largest chunk threshold and reference exponent: lane c reads chunk c (S <= 32), then a wave maximum
  float T_row;
  int R_max;
  {
    const int c = min(lane, S - 1);
    const uint32_t kt = key_of(fs.Tc[c]);
    const uint32_t kr = (uint32_t)fs.R[c] ^ 0x80000000u;
    T_row = value_of(last_lane_u32(dpp_scan_max_u32(kt)));
    R_max = (int)(last_lane_u32(dpp_scan_max_u32(kr)) ^ 0x80000000u);
  }
  if (fs.fail_seg || !(T_row == T_row)) return 3;                             // uniform
  const uint32_t total_seg = fs.segoff[nseg];
  if (total_seg > (uint32_t)a.nc_cap) return 5;                               // uniform
  if (total_seg > (uint32_t)(NT * CR)) return kNeedLongList;                  // uniform

  // ---- (2) The two dependent global reads of this kernel -- the candidate segments and the raw
  // logits of the history tokens -- are issued as early as their addresses are known and
  // consumed as late as possible, with the LDS work in between.
  // (2a) thread t takes list positions per*t .. per*t + per-1: one segment search, then it walks along
  const uint2* segs = a.cand + (size_t)b * (size_t)a.S * (size_t)a.cap_c;
  const int per = (int)((total_seg + NT - 1) / NT);                           // uniform, <= CR
  uint2 creg[CR];
  {
    const uint32_t i0 = (uint32_t)(tid * per);
    int sg = 0;
    if (i0 < total_seg) {
      int s1 = nseg;
      while (s1 - sg > 1) {
        const int mid = (sg + s1) >> 1;
        if (fs.segoff[mid] <= i0) sg = mid; else s1 = mid;
      }
    }
    uint32_t lo_off = fs.segoff[sg], hi_off = fs.segoff[sg + 1];
#pragma unroll
    for (int r = 0; r < CR; ++r) {
      creg[r] = make_uint2(0u, kNoIdx);
      if (r < per) {
        const uint32_t i = i0 + (uint32_t)r;
        if (i < total_seg) {
          while (i >= hi_off) { ++sg; lo_off = hi_off; hi_off = fs.segoff[sg + 1]; }   // skips empty segments too
          creg[r] = segs[(size_t)sg * cap_c + (i - lo_off)];
        }
      }
    }
  }
  // (2b) slots of the distinct history tokens, in token order: each thread owns a contiguous
  // run of bitmap words
  uint32_t ndist = 0;
  if (has_pen) {
    const int perw = (W + NT - 1) / NT;                   // <= kWordRegs because V <= 262144
    const int w0 = tid * perw;
    uint32_t wd[kWordRegs];                                // all reads go out together
#pragma unroll
    for (int j = 0; j < kWordRegs; ++j) wd[j] = bm[min(w0 + j, W - 1)];
    uint32_t local = 0;
#pragma unroll
    for (int j = 0; j < kWordRegs; ++j) {
      if (!(j < perw && w0 + j < W)) wd[j] = 0;
      local += (uint32_t)__popc(wd[j]);
    }
    const uint32_t incl = dpp_scan_add_u32(local);
    if (lane == kWave - 1) fs.r32[wave] = incl;
    __syncthreads();
    uint32_t slot = incl - local;
#pragma unroll
    for (int ww = 0; ww < kFinalWaves; ++ww) {
      const uint32_t t = fs.r32[ww];
      if (ww < wave) slot += t;
      ndist += t;
    }
    if (tid == 0) fs.ndist_out = (int)ndist;
    if (ndist > (uint32_t)kSideMax) return 4;                                 // uniform
    if (ndist > (uint32_t)(NT * SR)) return kNeedLong;                        // uniform
#pragma unroll
    for (int j = 0; j < kWordRegs; ++j) {
      uint32_t bits = wd[j];
      if (bits) pre[w0 + j] = (unsigned short)slot;
      while (bits) {                                                          // token of each slot
        stok[slot] = (uint32_t)(((w0 + j) << 5) + __ffs((int)bits) - 1);
        bits &= bits - 1;
        ++slot;
      }
    }
    __syncthreads();
  }
  // Register entries: 0..CR-1 candidates, CR..NE-1 history tokens.  idx == kNoIdx: no entry.
  uint32_t idx[NE], key[NE];                 // key[] holds the bits of z' until (5) turns them into keys
  // (2c) request the raw logits of this thread's history tokens
  float raw[SR];
#pragma unroll
  for (int r = 0; r < SR; ++r) {
    idx[CR + r] = kNoIdx; raw[r] = 0.0f;
    if ((uint32_t)(r * NT) < ndist) {                                        // uniform
      const uint32_t i = (uint32_t)(r * NT + tid);
      const uint32_t t = stok[min(i, (uint32_t)kSideMax - 1)];
      if (i < ndist) idx[CR + r] = t;
    }
  }
#pragma unroll
  for (int r = 0; r < SR; ++r)
    if (idx[CR + r] != kNoIdx) {
      if (!SH) {
        raw[r] = load_elem<DT>(row, (int)idx[CR + r]);
      } else {                                  // the token's shard, then its place inside it
        const int v = (int)idx[CR + r];
        int sh = min((int)((float)v * a.inv_V_shard), a.t_shards - 1);
        sh += (v >= (sh + 1) * a.V_shard) - (v < sh * a.V_shard);
        raw[r] = load_elem<DT>(fs.shard_row[sh], v - sh * a.V_shard);
      }
    }
  // ---- (3) multiplicities of the history tokens
  if (has_pen && pen.counts) {
    auto count = [&](int t) {
      if (t >= 0 && t < V) {
        const uint32_t word = bm[t >> 5];
        atomicAdd(&cnt[pre[t >> 5] + __popc(word & ((1u << (t & 31)) - 1u))], 1u);
      }
    };
    const int rounds = (int)min((long long)kTokRegs, (hi - lo + NT - 1) / NT);   // uniform
    uint32_t cw[kTokRegs], cp[kTokRegs];
#pragma unroll
    for (int j = 0; j < kTokRegs; ++j) {
      if (j < rounds) {
        const int t = min(max(tok[j], 0), V - 1);
        cw[j] = bm[t >> 5]; cp[j] = pre[t >> 5];
      }
    }
#pragma unroll
    for (int j = 0; j < kTokRegs; ++j) {
      const int t = tok[j];
      if (j < rounds && t >= 0 && t < V) atomicAdd(&cnt[cp[j] + __popc(cw[j] & ((1u << (t & 31)) - 1u))], 1u);
    }
    for (long long i = lo + tid + (long long)kTokRegs * NT; i < hi; i += NT) count(a.tokens[i]);
  }
  // (2d) candidates that carry a penalty are dropped: they come back with their penalised value
  // as history entries
  bool anyc = false;
  uint32_t fw[CR];
#pragma unroll
  for (int r = 0; r < CR; ++r) {
    fw[r] = 0;
    if (r < per && creg[r].y != kNoIdx) creg[r].y &= ~kTagBit;                  // the tag repeats what the bitmap says
    if (r < per && has_pen) fw[r] = bm[min(creg[r].y, (uint32_t)V - 1) >> 5];   // uniform condition
  }
#pragma unroll
  for (int r = 0; r < CR; ++r) {
    const uint2 e = creg[r];
    const bool keep = (r < per) & (e.y < (uint32_t)V) & (((fw[r] >> (e.y & 31)) & 1u) == 0);
    idx[r] = keep ? e.y : kNoIdx;
    key[r] = e.x;
    anyc |= keep & (__uint_as_float(e.x) >= T_row);
  }
  __syncthreads();

  // ---- (4) penalised values of the history entries; maximum of the list (lowest index on ties)
  // (the streaming pass, and restream_row, keep history tokens out of the bulk mass, so nothing
  // has to be taken back out of it)
  uint32_t bkey = 0, bidx = kNoIdx;
  {
    // everything these rounds read from LDS is requested first, then used
    uint32_t mult[SR];
#pragma unroll
    for (int r = 0; r < SR; ++r)
      if ((uint32_t)(r * NT) < ndist) mult[r] = pen.counts ? cnt[r * NT + tid] : pen.dflt;   // uniform
#pragma unroll
    for (int r = 0; r < SR; ++r) {
      if ((uint32_t)(r * NT) < ndist && idx[CR + r] != kNoIdx)
        key[CR + r] = __float_as_uint(penalise(raw[r], mult[r], rp.theta, rp.phi, rp.psi));
    }
  }
#pragma unroll
  for (int r = 0; r < NE; ++r) {
    if (idx[r] != kNoIdx) {
      const uint32_t kz = key_of(__uint_as_float(key[r]));
      if (kz > bkey || (kz == bkey && idx[r] < bidx)) { bkey = kz; bidx = idx[r]; }
    }
  }
  {
    const uint32_t wk = last_lane_u32(dpp_scan_max_u32(bkey));
    const uint32_t wi = last_lane_u32(dpp_scan_min_u32(bkey == wk ? bidx : kNoIdx));
    if (lane == kWave - 1) { fs.rkey[wave] = wk; fs.ridx[wave] = wi; }
    if (__any(anyc) && lane == 0) fs.anyc = 1;
  }
  __syncthreads();
  bkey = 0; bidx = kNoIdx;
#pragma unroll
  for (int w = 0; w < kFinalWaves; ++w) {
    const uint32_t ok = fs.rkey[w], oi = fs.ridx[w];
    if (ok > bkey || (ok == bkey && oi < bidx)) { bkey = ok; bidx = oi; }
  }
  // an unpenalised candidate at or above T_row proves that nothing outside the list is larger
  if (!fs.anyc || bidx == kNoIdx) return 6;                                   // uniform
  const int best_i = (int)bidx;
  const float m = scaled_s(value_of(bkey));
  const float s_c = scaled_s(T_row);            // entries with s > s_c: every such element of the row is in the list
  const uint32_t key_c = key_of(s_c);
  if (tid == 0) { fs.m_out = m; fs.zmax_out = value_of(bkey); fs.trow_out = T_row; }
  const float span = __fsub_rn(m, s_c);
  if (!(span >= 0.0f) || !(span < 3.0e38f)) return 7;                         // uniform
  const float binscale = span > 0.0f ? (float)(kBins - 2) / span : 0.0f;
  auto bin_of = [&](float s, uint32_t k) -> int {
    if (k <= key_c) return 0;
    const int q = (int)(__fsub_rn(s, s_c) * binscale);
    return 1 + min(kBins - 2, max(q, 0));
  };
  auto mass = [&](float s) { return fix_of(expf(__fsub_rn(s, m))); };
  // which register rounds hold anything at all (workgroup-uniform)
  auto live = [&](int r) { return r < CR ? r < per : (uint32_t)((r - CR) * NT) < ndist; };

  // ---- (5) keys, masses, value histogram (count and mass per bin)
  unsigned long long Ereg[NS];
  short breg[NS];
#pragma unroll
  for (int r = 0; r < NE; ++r) {
    if (live(r)) {
      unsigned long long E = 0;
      int bin = -1;
      uint32_t k = 0;
      if (idx[r] != kNoIdx) {
        const float s = scaled_s(__uint_as_float(key[r]));
        k = key_of(s);
        bin = bin_of(s, k);
        E = mass(s);
        atomicAdd(&hc[bin], 1u);
        if (E) atomicAdd(&hm[bin], E);
      }
      key[r] = k;
      if (r >= CR) cnt[(r - CR) * NT + tid] = k;      // slot -> key, for the whole-row draw (this thread's own slot)
      if constexpr (STORE) { Ereg[r] = E; breg[r] = (short)bin; }
    } else {
      key[r] = 0;
      if constexpr (STORE) { Ereg[r] = 0; breg[r] = -1; }
    }
  }
  auto E_of = [&](int r) -> unsigned long long {
    if constexpr (STORE) return Ereg[r]; else return mass(value_of(key[r]));
  };
  auto b_of = [&](int r) -> int {
    if constexpr (STORE) return (int)breg[r]; else return bin_of(value_of(key[r]), key[r]);
  };
  __syncthreads();
  const bool k_act = !rp.greedy && rp.top_k >= 2 && rp.top_k < V;
  const uint32_t n_top = (uint32_t)max(0, min(a.k_lp, V));
  unsigned long long S_cand;
  {
    // thread t owns bins kBins-1-4t .. kBins-4-4t; scan in descending bin order
    const int b0 = kBins - 1 - kBinsPerThread * tid;
    uint32_t c[kBinsPerThread];
    unsigned long long w[kBinsPerThread];
    uint32_t csum = 0;
    unsigned long long msum = 0;
#pragma unroll
    for (int j = 0; j < kBinsPerThread; ++j) { c[j] = hc[b0 - j]; w[j] = hm[b0 - j]; csum += c[j]; msum += w[j]; }
    const uint32_t cinc = dpp_scan_add_u32(csum);
    const unsigned long long minc = dpp_scan_add_u64(msum);
    if (lane == kWave - 1) { fs.r32[wave] = cinc; fs.r64[wave] = minc; }
    __syncthreads();
    uint32_t cex = cinc - csum;
    unsigned long long mex = minc - msum, mtot = 0;
#pragma unroll
    for (int ww = 0; ww < kFinalWaves; ++ww) {
      if (ww < wave) { cex += fs.r32[ww]; mex += fs.r64[ww]; }
      mtot += fs.r64[ww];
    }
    S_cand = mtot;
    const uint32_t k = (uint32_t)rp.top_k;
    int mylow = 1 << 30;
#pragma unroll
    for (int j = 0; j < kBinsPerThread; ++j) {
      const int bin = b0 - j;
      hm[bin] = mex;                                                         // exclusive suffix mass
      if (bin >= 1) {                                                        // bin 0 is the incomplete region
        if (k_act && cex < k && k <= cex + c[j]) { fs.bin_k = bin; fs.above_k = cex; }
        if (n_top > 0 && cex < n_top && n_top <= cex + c[j]) { fs.bin_n = bin; fs.above_n = cex; }
        if (c[j]) mylow = bin;                                               // bins descend: the last one wins
      }
      cex += c[j]; mex += w[j];
    }
    const uint32_t wlow = last_lane_u32(dpp_scan_min_u32((uint32_t)mylow));
    if (lane == kWave - 1 && wlow < (1u << 30)) atomicMin(&fs.bin_low, (int)wlow);
  }
  __syncthreads();
  if ((k_act && fs.bin_k < 0) || (n_top > 0 && fs.bin_n < 0)) return 8;      // uniform: k-th / n-th not provably in the list
  const int bin_k = k_act ? fs.bin_k : 0, bin_n = fs.bin_n;

  // bulk mass -> units of 2^-40 relative to the maximum
  unsigned long long bulk;
  {
    const int c = min(lane, S - 1);
    const int sh = R_max - fs.R[c];
    const unsigned long long bc = fs.bulk[c];
    bulk = last_lane_u64(dpp_scan_add_u64((lane < S && sh < 64) ? (bc >> sh) : 0ull));
  }
  // 2^x with x split into integer and fraction: the fraction goes through the hardware exp2 (1 ulp,
  // far inside the accuracy of the fp32 bulk sums), the integer part is an exponent shift
  const double ln2 = 0.6931471805599453094, log2e = 1.4426950408889634074;
  const double x = fmin(fmax((double)R_max + 10.0 - (double)m * log2e, -2000.0), 2000.0);
  const double xi = floor(x);
  const double bulk_rel = ldexp((double)bulk * (double)__builtin_amdgcn_exp2f((float)(x - xi)), (int)xi);
  const unsigned long long S0 = S_cand + (bulk_rel < 9.0e18 ? (unsigned long long)bulk_rel : 0ull);
  // ln S0 from exponent and mantissa: S0 = f * 2^e, f in [0.5, 1)
  int e2;
  const float f2 = (float)frexp((double)S0, &e2);
  const double lnZ = ((double)__builtin_amdgcn_logf(f2) + (double)(e2 - kFixShift)) * ln2;

  // ---- (6) gather the bin of the k-th largest and everything at or above the bin of the n-th best
  if (k_act || n_top > 0) {
    mask_t mk = 0, mt = 0;            // bit r: register entry r lies in the bin of the k-th / belongs to the top list
#pragma unroll
    for (int r = 0; r < NE; ++r) {
      if (live(r) && idx[r] != kNoIdx) {
        const int bin = b_of(r);
        mk |= (mask_t)(k_act & (bin == bin_k)) << r;
        mt |= (mask_t)((n_top > 0) & (bin >= bin_n)) << r;
      }
    }
    uint32_t qk = 0, qt = 0;            // one reservation per thread and list
    if (mk) qk = atomicAdd(&fs.n_memb, (uint32_t)__popcll((unsigned long long)mk));
    if (mt) qt = atomicAdd(&fs.n_top, (uint32_t)__popcll((unsigned long long)mt));
    if (mk | mt) {
#pragma unroll
      for (int r = 0; r < NE; ++r) {
        if ((mk >> r) & 1u) {
          if (qk < (uint32_t)kMembers) { fs.m_key[qk] = key[r]; fs.m_E[qk] = E_of(r); }
          ++qk;
        }
        if ((mt >> r) & 1u) {
          if (qt < (uint32_t)kTopList) { fs.t_key[qt] = key[r]; fs.t_idx[qt] = idx[r]; }
          ++qt;
        }
      }
    }
    __syncthreads();
    if (fs.n_memb > (uint32_t)kMembers || fs.n_top > (uint32_t)kTopList) return 9;   // uniform
  }
  // best-n (upper half of the workgroup) and the k-th largest (lower half) side by side
  // The gathered list holds every element at or above the bin of the n-th best, so an entry's
  // rank in this list is its rank in the row.  Up to 64 entries are ranked by one wave out of
  // its own registers; longer lists by half the workgroup out of LDS.
  const uint32_t nt_all = (a.k_lp >= 0 && n_top > 0) ? (uint32_t)__builtin_amdgcn_readfirstlane((int)fs.n_top) : 0u;
  if (nt_all > 0 && nt_all <= (uint32_t)kWave) {
    if (wave == 1) {
      const int cols = 1 + a.k_lp;
      const uint32_t kt = fs.t_key[lane], v = fs.t_idx[lane];
      uint32_t rank = 0;
      for (uint32_t q = 0; q < nt_all; ++q) {
        const uint32_t kq = (uint32_t)__builtin_amdgcn_readlane((int)kt, (int)q);
        const uint32_t iq = (uint32_t)__builtin_amdgcn_readlane((int)v, (int)q);
        rank += (uint32_t)((kq > kt) | ((kq == kt) & (iq < v)));
      }
      if ((uint32_t)lane < nt_all && rank < n_top) {
        a.out_lp_ids[(size_t)b * cols + 1 + rank] = (int)v;
        a.out_lp[(size_t)b * cols + 1 + rank] = (float)((double)value_of(kt) - (double)m - lnZ);
      }
    }
  } else if (nt_all > 0 && tid >= NT / 2) {
    const int cols = 1 + a.k_lp;
    const uint32_t nt = nt_all;
    const uint32_t t = (uint32_t)(tid - NT / 2);
    if (t < nt) {
      const uint32_t kt = fs.t_key[t], v = fs.t_idx[t];
      uint32_t rank = 0;
#pragma unroll 8
      for (uint32_t q = 0; q < nt; ++q) {
        const uint32_t kq = fs.t_key[q];
        rank += (kq > kt || (kq == kt && fs.t_idx[q] < v)) ? 1u : 0u;
      }
      if (rank < n_top) {
        a.out_lp_ids[(size_t)b * cols + 1 + rank] = (int)v;
        a.out_lp[(size_t)b * cols + 1 + rank] = (float)((double)value_of(kt) - (double)m - lnZ);
      }
    }
  }
  uint32_t key_k = 0;
  unsigned long long S1 = S0;
  if (k_act) {
    const uint32_t nm = (uint32_t)__builtin_amdgcn_readfirstlane((int)fs.n_memb), k_rem = (uint32_t)rp.top_k - fs.above_k;
    if (nm <= (uint32_t)kWave) {
      if (wave == 0) {                    // members in the lanes of one wave, compared through readlane
        const uint32_t kt = fs.m_key[lane];
        const unsigned long long Et = fs.m_E[lane];
        uint32_t gt = 0, ge = 0;
        unsigned long long sum_ge = 0;
        for (uint32_t q = 0; q < nm; ++q) {
          const uint32_t kq = (uint32_t)__builtin_amdgcn_readlane((int)kt, (int)q);
          const unsigned long long Eq = readlane_u64(Et, (int)q);
          gt += kq > kt; ge += kq >= kt;
          sum_ge += kq >= kt ? Eq : 0ull;
        }
        if ((uint32_t)lane < nm && gt < k_rem && k_rem <= ge) { fs.key_k = kt; fs.s1_part = sum_ge; }
      }
    } else if ((uint32_t)tid < nm) {
      const uint32_t kt = fs.m_key[tid];
      uint32_t gt = 0, ge = 0;
      unsigned long long sum_ge = 0;
#pragma unroll 8
      for (uint32_t q = 0; q < nm; ++q) {
        const uint32_t kq = fs.m_key[q];
        gt += kq > kt; ge += kq >= kt;
        sum_ge += kq >= kt ? fs.m_E[q] : 0ull;
      }
      // the k-th largest of the row: ties write the same two values
      if (gt < k_rem && k_rem <= ge) { fs.key_k = kt; fs.s1_part = sum_ge; }
    }
    __syncthreads();
    key_k = fs.key_k;
    S1 = hm[bin_k] + fs.s1_part;
  }

  int token = best_i;
  uint32_t token_key = key_of(m);
  if (!rp.greedy) {
    // ---- (7) top-p
    // every element missing from the list fails min-p  <=>  the completeness threshold itself fails it
    const bool minp_bounds = minp_on && !(__fsub_rn(s_c, m) >= t_minp);
    uint32_t key_cut = key_k;
    bool whole_row = false;
    if (rp.top_p < 1.0f) {
      const double lim = ceil((double)rp.top_p * (double)S1);
      const unsigned long long limit = lim > 0.0 ? (unsigned long long)lim : 0ull;
      const int lowbin = k_act ? bin_k : 1;
      {
        const int b0 = kBins - 1 - kBinsPerThread * tid;
        int mine = 1 << 30;
#pragma unroll
        for (int j = 0; j < kBinsPerThread; ++j) {
          const int bin = b0 - j;
          if (bin >= lowbin && hc[bin] && hm[bin] < limit) mine = bin;       // bins descend: the last one wins
        }
        const uint32_t wmin = last_lane_u32(dpp_scan_min_u32((uint32_t)mine));
        if (lane == kWave - 1 && wmin < (1u << 30)) atomicMin(&fs.bin_p, (int)wmin);
      }
      __syncthreads();
      const int bin_p = fs.bin_p;
      if (bin_p >= kBins) return 10;                                          // uniform (p <= 0)
      {
        mask_t mp = 0;
#pragma unroll
        for (int r = 0; r < NE; ++r)
          if (live(r) && idx[r] != kNoIdx) mp |= (mask_t)((key[r] >= key_k) & (b_of(r) == bin_p)) << r;
        if (mp) {
          uint32_t q = atomicAdd(&fs.n_memb2, (uint32_t)__popcll((unsigned long long)mp));
#pragma unroll
          for (int r = 0; r < NE; ++r) {
            if ((mp >> r) & 1u) {
              if (q < (uint32_t)kMembers) { fs.m_key[q] = key[r]; fs.m_E[q] = E_of(r); }
              ++q;
            }
          }
        }
      }
      __syncthreads();
      const uint32_t nm = (uint32_t)__builtin_amdgcn_readfirstlane((int)fs.n_memb2);
      if (nm > (uint32_t)kMembers) return 9;                                  // uniform
      if (nm <= (uint32_t)kWave) {
        if (wave == 0) {
          const uint32_t kt = fs.m_key[lane];
          const unsigned long long Et = fs.m_E[lane];
          unsigned long long G = hm[bin_p];
          for (uint32_t q = 0; q < nm; ++q) {
            const uint32_t kq = (uint32_t)__builtin_amdgcn_readlane((int)kt, (int)q);
            const unsigned long long Eq = readlane_u64(Et, (int)q);
            G += kq > kt ? Eq : 0ull;
          }
          const bool member = (uint32_t)lane < nm;
          const uint32_t kp = last_lane_u32(dpp_scan_min_u32((member && G < limit) ? kt : 0xFFFFFFFFu));
          const bool drop = __any(member && !(G < limit));
          if (lane == 0) { fs.key_p = kp; if (drop) fs.dropped = 1; }
        }
      } else if ((uint32_t)tid < nm) {
        const uint32_t kt = fs.m_key[tid];
        unsigned long long G = hm[bin_p];
#pragma unroll 8
        for (uint32_t q = 0; q < nm; ++q)
          if (fs.m_key[q] > kt) G += fs.m_E[q];
        if (G < limit) atomicMin(&fs.key_p, kt); else fs.dropped = 1;
      }
      __syncthreads();
      const bool inside = k_act || bin_p > fs.bin_low || fs.dropped != 0;
      if (!inside && !minp_bounds) {
        // uniform: the cut may lie below the list; it is settled, and the token drawn, over the
        // whole row by the caller (out of this function: code that is rarely needed slows it down)
        if (tid == 0) {
          fs.limit_out = limit; fs.lnz_out = lnZ; fs.has_pen_out = has_pen;
          // Every token below the list weighs at most what the completeness threshold weighs, so
          // the nucleus needs at least (limit - mass of the complete part of the list) / that many
          // more: if even this bound does not fit a second list, do not try one.
          const unsigned long long have = hm[0], e_c = mass(s_c);
          const unsigned long long lack = limit > have ? limit - have : 0ull;
          // (and a list that holds less than three quarters of the nucleus' mass is taken as a sign
          // that the rest is far longer than this bound)
          // With min-p on, the kept set ends at the min-p threshold at the latest, which is known
          // exactly by now: a second list cut there settles the row if it fits (the caller checks).
          fs.retry_ok_out = minp_on ||
                            (e_c > 0 && lack / e_c + total_seg < 10000ull && have >= limit - (limit >> 2));
        }
        return kWholeRowCut;
      }
      key_cut = max(key_k, fs.key_p);
    } else if (!k_act && !minp_bounds) {
      if (minp_on) return 12;                                                 // uniform: min-p reaches below the list
      whole_row = true;                                                       // no filter at all: every token is kept
    }

    if (whole_row) {
      if (tid == 0) { fs.limit_out = 0; fs.lnz_out = lnZ; fs.has_pen_out = has_pen; }
      return kWholeRow;                                                       // uniform: finished by the caller
    } else {
      // ---- (8) draw: kept mass per index bin, prefix, then resolve inside the crossing bin
      auto kept = [&](uint32_t k) {
        return k >= key_cut && k > key_c && (!minp_on || __fsub_rn(value_of(k), m) >= t_minp);
      };
      int ishift = 0;
      while (((V - 1) >> ishift) >= kBins) ++ishift;
      mask_t keptmask = 0;                                // bit r: register entry r is in the kept set
#pragma unroll
      for (int r = 0; r < NE; ++r) {
        if (live(r) && idx[r] != kNoIdx && kept(key[r])) {
          const unsigned long long E = E_of(r);
          if (E) { atomicAdd(&hd[idx[r] >> ishift], E); keptmask |= (mask_t)1 << r; }
        }
      }
      __syncthreads();
      unsigned long long target;
      {
        const int b0 = kBinsPerThread * tid;                 // ascending index order
        unsigned long long w[kBinsPerThread], msum = 0;
#pragma unroll
        for (int j = 0; j < kBinsPerThread; ++j) { w[j] = hd[b0 + j]; msum += w[j]; }
        const unsigned long long minc = dpp_scan_add_u64(msum);
        if (lane == kWave - 1) fs.r64[wave] = minc;
        __syncthreads();
        unsigned long long ex = minc - msum, S3 = 0;
#pragma unroll
        for (int ww = 0; ww < kFinalWaves; ++ww) {
          if (ww < wave) ex += fs.r64[ww];
          S3 += fs.r64[ww];
        }
        target = (__umul64hi(j24, S3) << 40) | ((j24 * S3) >> 24);             // floor(j * S3 / 2^24)
#pragma unroll
        for (int j = 0; j < kBinsPerThread; ++j) {
          if (ex <= target && target < ex + w[j]) { fs.bin_d = b0 + j; fs.before_d = ex; }
          ex += w[j];
        }
      }
      __syncthreads();
      const int bin_d = fs.bin_d;
      if (bin_d < 0) return 13;                                               // uniform (no kept mass)
      {
        mask_t md = 0;
#pragma unroll
        for (int r = 0; r < NE; ++r) md |= (mask_t)(((keptmask >> r) & 1u) & (mask_t)((int)(idx[r] >> ishift) == bin_d)) << r;
        if (md) {
          uint32_t q = atomicAdd(&fs.n_memb3, (uint32_t)__popcll((unsigned long long)md));
#pragma unroll
          for (int r = 0; r < NE; ++r) {
            if ((md >> r) & 1u) {
              if (q < (uint32_t)kMembers) { fs.m_key[q] = key[r]; fs.m_idx[q] = idx[r]; fs.m_E[q] = E_of(r); }
              ++q;
            }
          }
        }
      }
      __syncthreads();
      const uint32_t nm = (uint32_t)__builtin_amdgcn_readfirstlane((int)fs.n_memb3);
      if (nm > (uint32_t)kMembers) return 9;                                  // uniform
      if (nm <= (uint32_t)kWave) {
        if (wave == 0) {
          const uint32_t v = fs.m_idx[lane], kt = fs.m_key[lane];
          const unsigned long long Et = fs.m_E[lane];
          unsigned long long C = fs.before_d;
          for (uint32_t q = 0; q < nm; ++q) {
            const uint32_t iq = (uint32_t)__builtin_amdgcn_readlane((int)v, (int)q);
            const unsigned long long Eq = readlane_u64(Et, (int)q);
            C += iq <= v ? Eq : 0ull;
          }
          // members have mass > 0 and distinct indices: exactly one of them is the first crossing
          if ((uint32_t)lane < nm && C > target && C - Et <= target) { fs.token = (int)v; fs.token_key = kt; }
        }
      } else if ((uint32_t)tid < nm) {
        const uint32_t v = fs.m_idx[tid];
        unsigned long long C = fs.before_d;
#pragma unroll 8
        for (uint32_t q = 0; q < nm; ++q)
          if (fs.m_idx[q] <= v) C += fs.m_E[q];
        // members have mass > 0 and distinct indices: exactly one of them is the first crossing
        if (C > target && C - fs.m_E[tid] <= target) { fs.token = (int)v; fs.token_key = fs.m_key[tid]; }
      }
      __syncthreads();
      token = fs.token;
      if (token == 0x7FFFFFFF) return 13;                                     // uniform
      token_key = fs.token_key;
    }
  }

  // ---- (9) the token and its logprob.  Past this point nothing can fail.
  if (tid == 0) {
    a.out_ids[b] = token;
    if (a.k_lp >= 0) {
      const int cols = 1 + a.k_lp;
      a.out_lp_ids[(size_t)b * cols] = token;
      a.out_lp[(size_t)b * cols] = (float)((double)value_of(token_key) - (double)m - lnZ);
    }
  }
  return 1;
}

// Second attempt for a row whose candidate list turned out too short: this workgroup reads
// the row again (it is still in the last-level cache) with a lower threshold `Tc` and leaves
// the result where the first attempt's data was: one segment of S * cap_c entries and one
// chunk summary.  Same arithmetic as stream_kernel; `bm` (if not null) is the row's history
// bitmap that the first attempt left in LDS: tokens in it stay out of the bulk mass.
template <int DT>
__device__ __attribute__((noinline)) void restream_row(const Args& a, const int b, const RowParams rp, const float Tc,
                                                       FastShared& fs, const uint32_t* bm) {
  constexpr int NT = kFinalThreads;
  constexpr int EPL = (DT == SIP_F32) ? 4 : 8;
  constexpr int ESZ = (DT == SIP_F32) ? 4 : 2;
  const int tid = threadIdx.x, lane = lane_id(), wave = wave_id();
  const int V = a.V;
  const char* row = reinterpret_cast<const char*>(a.logits) + (size_t)b * (size_t)a.row_stride * ESZ;
  uint2* region = a.cand + (size_t)b * (size_t)a.S * (size_t)a.cap_c;
  const uint32_t cap = (uint32_t)(a.S * a.cap_c);
  const BulkRef ref = make_bulk_ref(Tc, rp);
  const int R = ref.R;
  __syncthreads();
  if (tid == 0) fs.rq_n = 0;
  __syncthreads();
  float acc = 0.0f;
  constexpr int UNR = 4;                                    // loads in flight per thread
  for (int t0 = 0; t0 < V; t0 += UNR * NT * EPL) {
    uint4 q[UNR];
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      const int e0 = t0 + (u * NT + tid) * EPL;
      q[u] = e0 < V ? *reinterpret_cast<const uint4*>(row + (size_t)e0 * ESZ) : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      const int e0 = t0 + (u * NT + tid) * EPL;
      float z[EPL];
      if (DT == SIP_F32) {
        z[0] = __uint_as_float(q[u].x); z[1] = __uint_as_float(q[u].y);
        z[2] = __uint_as_float(q[u].z); z[3] = __uint_as_float(q[u].w);
      } else {
        const uint32_t w[4] = {q[u].x, q[u].y, q[u].z, q[u].w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          z[2 * i] = __uint_as_float(w[i] << 16);
          z[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
        }
      }
      float g = 0.0f;
      // the elements of one load share a bitmap word (e0 is a multiple of EPL <= 8)
      const uint32_t hw = bm ? bm[min(e0, V - 1) >> 5] >> (e0 & 31) : 0u;
#pragma unroll
      for (int i = 0; i < EPL; ++i) {
        if (e0 + i >= V) z[i] = -INFINITY;
        const bool hit = z[i] >= Tc;
        if (hit) {
          const uint32_t pos = atomicAdd(&fs.rq_n, 1u);
          if (pos < cap) region[pos] = make_uint2(__float_as_uint(z[i]), (uint32_t)(e0 + i));
        }
        float e = bulk_term(z[i], ref);
        e = (hit || ((hw >> i) & 1u)) ? 0.0f : e;
        g += e;
      }
      acc += g;
    }
  }
  const unsigned long long wsum = dpp_scan_add_u64(bulk_units(acc));
  if (lane == kWave - 1) fs.r64[wave] = wsum;
  __syncthreads();
  if (tid == 0) {
    ChunkOut o;
    o.bulk = 0;
    for (int w = 0; w < kFinalWaves; ++w) o.bulk += fs.r64[w];
    o.Tc = Tc; o.R = R;
    o.cnt = fs.rq_n;
    o.pad[0] = o.pad[1] = o.pad[2] = 0;
    a.chunks[(size_t)b * a.S] = o;
  }
  // what this workgroup wrote to global memory is read back by other waves of it
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
  __syncthreads();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
}

// Rarely needed continuations, defined after the kernel (see there).
template <int DT>
__device__ int whole_row_finish(const Args& a, const int b, const RowParams rp, unsigned char* dyn, FastShared& fs,
                                const bool cut);

// Runs the smallest instantiation of fast_row that can hold the row: the history length bounds
// the number of distinct tokens; a variant that turns out too small says so early and the next
// one starts over.  Three variants, one after the other: every further instantiation in this
// kernel was measured to slow all of them down (0.6-1 us each).
template <int DT, bool SH>
__device__ __forceinline__ int fast_any(const Args& a, const int b, const RowParams& rp, unsigned char* dyn,
                                        FastShared& fs, const int S, const int cap_c, const long long ndist_ub) {
  constexpr int NT = kFinalThreads;
  int r = kNeedLong;
  if (ndist_ub <= 2 * NT) r = fast_row<DT, 8, 2, SH>(a, b, rp, dyn, fs, S, cap_c);
  if (r == kNeedLong) r = fast_row<DT, 8, 8, SH>(a, b, rp, dyn, fs, S, cap_c);
  if (r == kNeedLong || r == kNeedLongList) r = fast_row<DT, kCandLong, 8, SH>(a, b, rp, dyn, fs, S, cap_c);
  return (r == kNeedLong || r == kNeedLongList) ? 5 : r;
}

// One row that the finishing logic could not settle from its list is taken through the heavier
// logic below -- the same list in larger register variants, a second and longer list, the
// continuations over the whole row, the exact multi-pass path -- by the calling workgroup.
// `dynraw`: final_lds_fixed(V) (and at least 2 * ceil(V / 32) words) of LDS.
// Bitmap over the vocabulary of the row's history (and prompt) tokens, as restream_row() wants it.
__device__ __forceinline__ void history_bitmap(const Args& a, const int b, const PenaltyPlan& pen, uint32_t* bm) {
  const int W = (a.V + 31) / 32, V = a.V;
  for (int w = threadIdx.x; w < W; w += kFinalThreads) bm[w] = 0;
  __syncthreads();
  for (long long i = pen.h.lo + threadIdx.x; i < pen.h.hi; i += kFinalThreads) {
    const int t = a.tokens[i];
    if (t >= 0 && t < V) atomicOr(&bm[t >> 5], 1u << (t & 31));
  }
  for (long long i = pen.p_lo + threadIdx.x; i < pen.p_hi; i += kFinalThreads) {
    const int t = a.p_tokens[i];
    if (t >= 0 && t < V) atomicOr(&bm[t >> 5], 1u << (t & 31));
  }
  __syncthreads();
}

// `seen`: what a finishing attempt on the row's first list has already found out (finish_row()
// in the same workgroup), or nothing.
struct RescueSeen {
  int why = 0;               // finish_row()'s code; 0 = nothing is known
  bool retry_ok = false;
  float m = 0.0f, zmax = 0.0f, T = 0.0f;
};
template <int DT, bool SH>
__device__ __forceinline__ void rescue_row(const Args& a, const int b, unsigned char* dynraw, ExactShared& ex,
                                           FastShared& fs, const RescueSeen seen = RescueSeen()) {
  const RowParams rp = load_row_params(a, b);
  int how = 2;                                   // 2: not eligible for the single-pass path
  int code = 0;
  bool gathered = false;                         // sharded logits: the row has been put together in the workspace
  const int target = candidate_target(rp, a);
  if (target != 0) {
    // Upper bound on the row's distinct history tokens, which decides the instantiation that is
    // tried first: the history's length, or what a device-resident state remembers from the
    // slot's previous call.
    const PenaltyPlan pen0 = penalty_plan(a, b, rp.theta, rp.phi, rp.psi);
    const HistRange hr = pen0.h;
    long long ndist_ub = (hr.hi - hr.lo) + (pen0.p_hi - pen0.p_lo);
    if (a.slot && hr.hi > hr.lo) {
      const int hint = a.st_ndist[a.slot[b]];
      if (hint >= 0 && hint < ndist_ub) ndist_ub = hint;
    }
    if (threadIdx.x == 0) fs.ndist_out = -1;
    // At most two attempts, written as a loop so that the kernel holds one copy of the code.
    int S = a.S, cap_c = a.cap_c;
#pragma nounroll
    for (int attempt = 0; attempt < 2; ++attempt) {
      int r;
      bool cut_below = false;
      const bool skipped = attempt == 0 && (seen.why == 12 || (seen.why == 11 && seen.retry_ok));
      if (skipped) {
        // The first list has been looked at already and is known to be too short for a cut whose
        // place a second list can reach: go straight on to that one.
        r = seen.why;
        cut_below = seen.why == 11;
        if (threadIdx.x == 0) { fs.m_out = seen.m; fs.zmax_out = seen.zmax; fs.trow_out = seen.T; }
      } else {
        r = fast_any<DT, SH>(a, b, rp, dynraw, fs, S, cap_c, ndist_ub);
      }
      if (attempt == 0 && r == kWholeRowCut) {
        // a nucleus somewhat longer than the list is cheaper to settle from a second list than
        // over the whole row
        __syncthreads();
        if (fs.retry_ok_out) { r = 11; cut_below = true; }
      }
      if (attempt == 1) {
        const bool fine = r == 1 || r == kWholeRowCut || r == kWholeRow;
        how = fine ? r : 16 + r;                 // 17..29: failed again after the retry
        if (fine) code = 15;                     // 15: finished by the retry (still one HBM pass)
        break;
      }
      how = r;
      if (r != 8 && r != 11 && r != 12) break;
      // The list was complete but too short.  Where min-p is on, the threshold that bounds the
      // kept set is known exactly now that the maximum is; otherwise lower the threshold by
      // three tenths of its distance to the maximum.  One retry, then the exact path.
      __syncthreads();
      const float m = fs.m_out, zmax = fs.zmax_out, t_old = fs.trow_out;
      float t_new = t_old - 0.3f * (zmax - t_old);
      if (rp.min_p > 0.0f && !rp.greedy) {
        const float zt = (m + (float)log((double)rp.min_p)) * rp.tau;
        t_new = fminf(t_new, zt - 1.0e-5f * fabsf(zt) - 1.0e-30f);
        if (r != 8) t_new = zt - 1.0e-5f * fabsf(zt) - 1.0e-30f;
      }
      if (!(t_new < t_old)) break;
      if (SH && !gathered) { gather_row<DT>(a, b); gathered = true; }
      const PenaltyPlan pen1 = penalty_plan(a, b, rp.theta, rp.phi, rp.psi);
      const uint32_t* bm1 = pen1.any ? reinterpret_cast<const uint32_t*>(dynraw) : nullptr;
      if (skipped && pen1.any) history_bitmap(a, b, pen1, reinterpret_cast<uint32_t*>(dynraw));   // (else the first attempt left it there)
      restream_row<DT>(a, b, rp, t_new, fs, bm1);
      S = 1; cap_c = a.S * a.cap_c;
      if (cut_below && fs.rq_n > (uint32_t)(kFinalThreads * kCandLong)) {
        // The second list does not fit either: the cut is settled over the whole row, from the
        // tables of an attempt on the first list -- which are there, untouched, unless that
        // attempt was skipped: then the first list is made again (the second one lies where it
        // was) and looked at now.
        how = kWholeRowCut;
        if (skipped) {
          restream_row<DT>(a, b, rp, t_old, fs, bm1);
          how = fast_any<DT, SH>(a, b, rp, dynraw, fs, S, cap_c, ndist_ub);
        }
        break;
      }
    }
  }
  if (how == kWholeRowCut || how == kWholeRow) {
    // rows that are finished over the whole row: nucleus cut below the list, or no filter at all
    if (SH && !gathered) { gather_row<DT>(a, b); gathered = true; }
    how = whole_row_finish<DT>(a, b, rp, dynraw, fs, how == kWholeRowCut);
    code = how == 1 ? 16 : 0;                    // 16: finished over the whole row by this workgroup
  }
  if (how != 1) {
    __syncthreads();
    if (SH && !gathered) { gather_row<DT>(a, b); gathered = true; }
    exact_row<DT>(a, b, reinterpret_cast<uint32_t*>(dynraw), ex);
  }
  if (threadIdx.x == 0) a.row_path[b] = code ? code : how;
  if (a.slot) {                                  // device-resident history: the row's id joins it
    __syncthreads();
    if (threadIdx.x == 0) state_append_row(a, b);
  }
}

// The rows that finish_kernel could not settle (it leaves their numbers in Args::rescue_rows),
// one workgroup per row at a time.  Launched with a fixed, small grid after every finish_kernel;
// with nothing to rescue a workgroup reads the count and returns.
template <int DT, bool SH>
__global__ __launch_bounds__(kFinalThreads) void rescue_kernel(Args a_by_value) {
  // The arguments are read where they are used, straight from the kernel-argument segment
  // (the struct is the only parameter, so it starts at offset 0), instead of being held in
  // scalar registers from the first instruction on: there are more of them than registers.
  (void)a_by_value;
  const Args& a = *(const Args*)__builtin_amdgcn_kernarg_segment_ptr();
  extern __shared__ __align__(16) unsigned char dynraw[];
  __shared__ ExactShared ex;
  __shared__ FastShared fs;
  const int n_rescue = min(max(*a.rescue_n, 0), a.B);
#pragma nounroll
  for (int qi = blockIdx.x; qi < n_rescue; qi += gridDim.x) {
    if (qi != (int)blockIdx.x) __syncthreads();    // the row before this one is done with the tables in LDS
    rescue_row<DT, SH>(a, min(max(a.rescue_rows[qi], 0), a.B - 1), dynraw, ex, fs);
  }
}

// Draw over the whole row: for a row without any filter (plain temperature sampling), or, with
// `key_cut` / min-p, for a row whose kept set reaches below the candidate list.  Maximum,
// total mass and best-n came from the list; the draw itself needs every element's mass in
// vocabulary order, so the row is read once more here (it is still in the last-level cache),
// plus the one block in which the running mass crosses the target.  Out of line: rarely needed,
// and the finishing kernel gets slower with every piece of code inlined into it.  Leaves the
// token and its key in fs; returns 1, or 13 if there is no mass to draw from.
template <int DT>
__device__ __attribute__((noinline)) int whole_row_draw(const char* row, const int V, const bool has_pen,
                                                        const uint32_t* bm, const unsigned short* pre,
                                                        const uint32_t* cnt, unsigned long long* hd, FastShared& fs,
                                                        const float tau, const bool greedy, const float m,
                                                        const float zmax, const float c_row,
                                                        const unsigned long long j24, const uint32_t key_cut,
                                                        const bool minp_on, const float t_minp) {
  const int tid = threadIdx.x, lane = lane_id(), wave = wave_id();
  const bool filtered = key_cut != 0 || minp_on;        // uniform: only part of the row is kept
  auto scaled_s = [&](float z) { return greedy ? z : __fdiv_rn(z, tau); };
  constexpr int EPL = (DT == SIP_F32) ? 4 : 8;
  constexpr int ESZ = (DT == SIP_F32) ? 4 : 2;
  const int e_last = ((V - 1) / EPL) * EPL;
  auto ldrow = [&](int e0) {                            // clamped: always a valid address
    return *reinterpret_cast<const uint4*>(row + (size_t)min(e0, e_last) * ESZ);
  };
  // Masses as fp32, relative to the maximum; a lane adds those of one 16-byte load in a fixed
  // order and only the sum becomes an integer (units of 2^-40), so that both reads of the row
  // agree bit for bit on every partial sum while converting once per load, not per element.
  auto masses = [&](const uint4& q, int e0, float (&E)[EPL], uint32_t (&keys)[EPL]) {
    float z[EPL];
    if (DT == SIP_F32) {
      z[0] = __uint_as_float(q.x); z[1] = __uint_as_float(q.y);
      z[2] = __uint_as_float(q.z); z[3] = __uint_as_float(q.w);
    } else {
      const uint32_t w4[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        z[2 * i] = __uint_as_float(w4[i] << 16);
        z[2 * i + 1] = __uint_as_float(w4[i] & 0xFFFF0000u);
      }
    }
    // the elements of one load share a bitmap word (e0 is a multiple of EPL <= 8)
    const uint32_t word = has_pen ? bm[min(e0, V - 1) >> 5] : 0u;
#pragma unroll
    for (int i = 0; i < EPL; ++i) {
      const int v = e0 + i;
      E[i] = 0.0f; keys[i] = 0;
      if (v < V) {
        if ((word >> (v & 31)) & 1u) {                                     // carries a penalty: value from the list
          const float sv = value_of(cnt[pre[v >> 5] + __popc(word & ((1u << (v & 31)) - 1u))]);
          keys[i] = key_of(sv);
          E[i] = expf(__fsub_rn(sv, m));
          if (filtered && !(keys[i] >= key_cut && (!minp_on || __fsub_rn(sv, m) >= t_minp))) E[i] = 0.0f;
        } else if (filtered) {
          // a cut by value: the exact s decides who is kept; the mass is exp(s - max) with the
          // hardware exp2, the same expression in both passes below
          const float sv = scaled_s(z[i]);
          keys[i] = key_of(sv);
          const bool keep = keys[i] >= key_cut && (!minp_on || __fsub_rn(sv, m) >= t_minp);
          E[i] = keep ? __builtin_amdgcn_exp2f(__fmul_rn(__fsub_rn(sv, m), 1.44269504f)) : 0.0f;
        } else {
          // exp(z/tau - max) as 2^((z - zmax) * c): no division, hardware exp2; the two passes
          // below use the same expression, which is all the draw needs
          keys[i] = __float_as_uint(z[i]);                                 // raw bits, turned into a key on a hit
          E[i] = __builtin_amdgcn_exp2f(__fmul_rn(__fsub_rn(z[i], zmax), c_row));
        }
      }
    }
  };
  // first read: mass of every block of BLK consecutive elements (one block = UNR loads per
  // lane of one wave) into hd[] (still all zero); waves take contiguous runs of blocks
  constexpr int UNR = 4;
  constexpr int BLK = UNR * kWave * EPL;
  const int nblk = (V + BLK - 1) / BLK;                 // <= kBins because V <= 262144
  const int per_wave = (nblk + kFinalWaves - 1) / kFinalWaves;
  for (int blk = wave * per_wave; blk < min(nblk, (wave + 1) * per_wave); ++blk) {
    const int base = blk * BLK;
    uint4 q[UNR];
#pragma unroll
    for (int u = 0; u < UNR; ++u) q[u] = ldrow(base + (u * kWave + lane) * EPL);
    unsigned long long mine = 0;
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      float E[EPL];
      uint32_t keys[EPL];
      masses(q[u], base + (u * kWave + lane) * EPL, E, keys);        // zero past the end of the row
      float part = 0.0f;
#pragma unroll
      for (int i = 0; i < EPL; ++i) part += E[i];
      mine += fix_of(part);
    }
    mine = dpp_scan_add_u64(mine);
    if (lane == kWave - 1) hd[blk] = mine;
  }
  __syncthreads();
  // prefix over the blocks, find the block that holds the crossing
  unsigned long long target;
  {
    const int b0 = kBinsPerThread * tid;
    unsigned long long w[kBinsPerThread], msum = 0;
#pragma unroll
    for (int j = 0; j < kBinsPerThread; ++j) { w[j] = hd[b0 + j]; msum += w[j]; }
    const unsigned long long minc = dpp_scan_add_u64(msum);
    if (lane == kWave - 1) fs.r64[wave] = minc;
    __syncthreads();
    unsigned long long ex = minc - msum, S3 = 0;
#pragma unroll
    for (int ww = 0; ww < kFinalWaves; ++ww) {
      if (ww < wave) ex += fs.r64[ww];
      S3 += fs.r64[ww];
    }
    target = (__umul64hi(j24, S3) << 40) | ((j24 * S3) >> 24);           // floor(j * S3 / 2^24)
#pragma unroll
    for (int j = 0; j < kBinsPerThread; ++j) {
      if (ex <= target && target < ex + w[j]) { fs.bin_d = b0 + j; fs.before_d = ex; }
      ex += w[j];
    }
  }
  __syncthreads();
  const int blk_d = fs.bin_d;
  if (blk_d < 0) return 13;                                               // uniform (no mass at all)
  // second read, one block, one wave: lane prefixes in vocabulary order
  if (wave == 0) {
    const int base = blk_d * BLK;
    unsigned long long running = fs.before_d;
    int found = -1;
    uint32_t found_key = 0;
    uint4 q[UNR];
#pragma unroll
    for (int u = 0; u < UNR; ++u) q[u] = ldrow(base + (u * kWave + lane) * EPL);
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      const int e0 = base + (u * kWave + lane) * EPL;
      float E[EPL];
      uint32_t keys[EPL];
      masses(q[u], e0, E, keys);
      float part = 0.0f;
#pragma unroll
      for (int i = 0; i < EPL; ++i) part += E[i];
      const unsigned long long lane_tot = fix_of(part);
      const unsigned long long incl = dpp_scan_add_u64(lane_tot);
      const unsigned long long c = running + incl - lane_tot;
      int hit = -1;
      uint32_t hit_key = 0;
      float upto = 0.0f;                             // same additions in the same order as `part`
#pragma unroll
      for (int i = 0; i < EPL; ++i) {
        upto += E[i];
        if (hit < 0 && E[i] > 0.0f && c + fix_of(upto) > target) { hit = e0 + i; hit_key = keys[i]; }   // key, or raw bits if unpenalised
      }
      const unsigned long long ball = __ballot(hit >= 0);
      if (ball && found < 0) {
        const int src = __ffsll((long long)ball) - 1;
        found = __builtin_amdgcn_readlane(hit, src);
        found_key = (uint32_t)__builtin_amdgcn_readlane((int)hit_key, src);
      }
      running += last_lane_u64(incl);
    }
    if (lane == 0) {
      if (!filtered && found >= 0 && !(has_pen && ((bm[found >> 5] >> (found & 31)) & 1u)))
        found_key = key_of(scaled_s(__uint_as_float(found_key)));
      fs.token = found; fs.token_key = found_key;
    }
  }
  __syncthreads();
  const int token = fs.token;
  return (token == 0x7FFFFFFF || token < 0) ? 13 : 1;
}

// Nucleus cut of a row whose cut lies below the candidate list (top-p alone on a flat
// distribution keeps tens of thousands of tokens): a radix descent over the whole row on the
// exact fp32 s.  Each level is one read of the row (it is in the last-level cache): count
// and integer mass per bin, 2048 bins over the current interval of s, monotone in s so that
// equal values never part; the bin in which the mass of everything larger first stays short
// of the limit becomes the next interval.  Once that bin holds at most kMembers elements
// they are gathered and resolved by all-pairs comparison as in the list path.  Leaves the key
// of the smallest kept value in fs.key_p and returns 1, or returns 11 (more than kMembers equal
// values at the cut, no mass): the caller then takes the row to the exact path.
template <int DT>
__device__ __attribute__((noinline)) int whole_row_cut(const char* row, const int V, const bool has_pen,
                                                       const uint32_t* bm, const unsigned short* pre,
                                                       const uint32_t* cnt, unsigned long long* hm, uint32_t* hc,
                                                       FastShared& fs, const float tau, const float m,
                                                       const unsigned long long limit) {
  const int tid = threadIdx.x, lane = lane_id(), wave = wave_id();
  constexpr int NT = kFinalThreads;
  constexpr int EPL = (DT == SIP_F32) ? 4 : 8;
  constexpr int ESZ = (DT == SIP_F32) ? 4 : 2;
  constexpr int kLevels = 3;
  constexpr float kSpan = 28.0f;                          // exp(-28) * 2^40 < 1: nothing below has mass
  // s of every element of one 16-byte load (penalised elements take theirs from the slot table)
  auto svals = [&](int e0, float (&sv)[EPL]) {
    const int e_last = ((V - 1) / EPL) * EPL;
    const uint4 q = *reinterpret_cast<const uint4*>(row + (size_t)min(e0, e_last) * ESZ);
    float z[EPL];
    if (DT == SIP_F32) {
      z[0] = __uint_as_float(q.x); z[1] = __uint_as_float(q.y);
      z[2] = __uint_as_float(q.z); z[3] = __uint_as_float(q.w);
    } else {
      const uint32_t w4[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        z[2 * i] = __uint_as_float(w4[i] << 16);
        z[2 * i + 1] = __uint_as_float(w4[i] & 0xFFFF0000u);
      }
    }
#pragma unroll
    for (int i = 0; i < EPL; ++i) {
      const int v = min(e0 + i, V - 1);
      const uint32_t word = has_pen ? bm[v >> 5] : 0u;
      sv[i] = ((word >> (v & 31)) & 1u) ? value_of(cnt[pre[v >> 5] + __popc(word & ((1u << (v & 31)) - 1u))])
                                        : __fdiv_rn(z[i], tau);
    }
  };
  auto mass = [&](float sv) { return fix_of(__builtin_amdgcn_exp2f(__fmul_rn(__fsub_rn(sv, m), 1.44269504f))); };
  float lo[kLevels], sc[kLevels];
  int pick[kLevels];
  auto bin_at = [&](int l, float sv) { return min(kBins - 1, max(0, (int)(__fsub_rn(sv, lo[l]) * sc[l]))); };
  float cur_lo = m - kSpan, cur_w = kSpan;
  unsigned long long above = 0;                           // mass of everything larger than the current interval
  uint32_t n_in = 0;
  int levels = 0;
#pragma unroll
  for (int level = 0; level < kLevels; ++level) {
    const float cur_sc = (float)kBins / cur_w;
    lo[level] = cur_lo; sc[level] = cur_sc; pick[level] = 0;
    __syncthreads();
    for (int i = tid; i < kBins; i += NT) { hm[i] = 0; hc[i] = 0; }
    if (tid == 0) fs.bin_p = 1 << 30;
    __syncthreads();
    for (int e0 = tid * EPL; e0 < V; e0 += NT * EPL) {
      float sv[EPL];
      svals(e0, sv);
#pragma unroll
      for (int i = 0; i < EPL; ++i) {
        bool in = e0 + i < V && sv[i] == sv[i];
#pragma unroll
        for (int l = 0; l < kLevels; ++l)
          if (l < level) in = in && bin_at(l, sv[i]) == pick[l];
        if (in) {
          const int bin = min(kBins - 1, max(0, (int)(__fsub_rn(sv[i], cur_lo) * cur_sc)));
          atomicAdd(&hc[bin], 1u);
          const unsigned long long E = mass(sv[i]);
          if (E) atomicAdd(&hm[bin], E);
        }
      }
    }
    __syncthreads();
    {
      // thread t owns bins kBins-1-4t .. kBins-4-4t; exclusive suffix mass in descending bin order
      const int b0 = kBins - 1 - kBinsPerThread * tid;
      uint32_t c[kBinsPerThread];
      unsigned long long w[kBinsPerThread], msum = 0;
#pragma unroll
      for (int j = 0; j < kBinsPerThread; ++j) { c[j] = hc[b0 - j]; w[j] = hm[b0 - j]; msum += w[j]; }
      const unsigned long long minc = dpp_scan_add_u64(msum);
      if (lane == kWave - 1) fs.r64[wave] = minc;
      __syncthreads();
      unsigned long long mex = above + minc - msum;
#pragma unroll
      for (int ww = 0; ww < kFinalWaves; ++ww)
        if (ww < wave) mex += fs.r64[ww];
      int mine = 1 << 30;
      unsigned long long mex_j[kBinsPerThread];
#pragma unroll
      for (int j = 0; j < kBinsPerThread; ++j) {
        mex_j[j] = mex;
        if (c[j] && mex < limit) mine = b0 - j;           // bins descend: the last one wins
        mex += w[j];
      }
      const uint32_t wmin = last_lane_u32(dpp_scan_min_u32((uint32_t)mine));
      if (lane == kWave - 1 && wmin < (1u << 30)) atomicMin(&fs.bin_p, (int)wmin);
      __syncthreads();
      const int bp = fs.bin_p;
#pragma unroll
      for (int j = 0; j < kBinsPerThread; ++j)
        if (b0 - j == bp) { fs.before_d = mex_j[j]; fs.n_memb3 = c[j]; }
    }
    __syncthreads();
    const int bp = fs.bin_p;
    if (bp >= kBins) return 11;                           // uniform: nothing qualifies (limit of 0)
    pick[level] = bp; above = fs.before_d; n_in = fs.n_memb3;
    levels = level + 1;
    if (n_in <= (uint32_t)kMembers) break;                // uniform
    cur_w = cur_w * (1.0f / (float)kBins);
    cur_lo = lo[level] + (float)bp * cur_w;
  }
  if (n_in > (uint32_t)kMembers) return 11;               // uniform
  // gather the elements of the last bin and resolve them
  __syncthreads();
  if (tid == 0) { fs.n_memb2 = 0; fs.key_p = 0xFFFFFFFFu; }
  __syncthreads();
  for (int e0 = tid * EPL; e0 < V; e0 += NT * EPL) {
    float sv[EPL];
    svals(e0, sv);
#pragma unroll
    for (int i = 0; i < EPL; ++i) {
      bool in = e0 + i < V && sv[i] == sv[i];
#pragma unroll
      for (int l = 0; l < kLevels; ++l)
        if (l < levels) in = in && bin_at(l, sv[i]) == pick[l];
      if (in) {
        const uint32_t q = atomicAdd(&fs.n_memb2, 1u);
        if (q < (uint32_t)kMembers) { fs.m_key[q] = key_of(sv[i]); fs.m_E[q] = mass(sv[i]); }
      }
    }
  }
  __syncthreads();
  const uint32_t nm = min(fs.n_memb2, (uint32_t)kMembers);
  if ((uint32_t)tid < nm) {
    const uint32_t kt = fs.m_key[tid];
    unsigned long long G = above;
    for (uint32_t q = 0; q < nm; ++q) {
      const uint32_t kq = fs.m_key[q];
      const unsigned long long Eq = fs.m_E[q];
      G += kq > kt ? Eq : 0ull;
    }
    if (G < limit) atomicMin(&fs.key_p, kt);
  }
  __syncthreads();
  return fs.key_p == 0xFFFFFFFFu ? 11 : 1;
}

// Continuation of fast_row for the two kinds of row that are finished over the whole row
// (codes kWholeRowCut and kWholeRow): nucleus cut if asked for, draw, token and its logprob.
// The best-n list is already written.  Returns 1, or a code that sends the row to the exact path.
template <int DT>
__device__ __attribute__((noinline)) int whole_row_finish(const Args& a, const int b, const RowParams rp,
                                                          unsigned char* dyn, FastShared& fs, const bool cut) {
  const int V = a.V;
  const int W = (V + 31) >> 5;
  const uint32_t* bm = reinterpret_cast<const uint32_t*>(dyn);
  const unsigned short* pre = reinterpret_cast<const unsigned short*>(dyn + (size_t)W * 4);
  unsigned char* p2 = dyn + (((size_t)W * 6 + 15) / 16) * 16;
  unsigned long long* hm = reinterpret_cast<unsigned long long*>(p2);
  unsigned long long* hd = hm + kBins;
  uint32_t* hc = reinterpret_cast<uint32_t*>(hd + kBins);
  const uint32_t* cnt = hc + kBins;
  const char* row = reinterpret_cast<const char*>(a.logits) + (size_t)b * (size_t)a.row_stride * (DT == SIP_F32 ? 4 : 2);
  __syncthreads();
  const float m = fs.m_out, zmax = fs.zmax_out;
  const unsigned long long limit = fs.limit_out;
  const double lnZ = fs.lnz_out;
  const bool has_pen = fs.has_pen_out != 0;
  const bool minp_on = cut && rp.min_p > 0.0f;
  const float t_minp = minp_on ? (float)log((double)rp.min_p) : 0.0f;
  const unsigned long long j24 = (unsigned long long)(philox_word0(a.seed, rp.row_id, step_of(a)) >> 8);
  float c_row, c_lo;
  scale_pair(rp, c_row, c_lo);
  uint32_t key_cut = 0;
  if (cut) {
    if (whole_row_cut<DT>(row, V, has_pen, bm, pre, cnt, hm, hc, fs, rp.tau, m, limit) != 1) return 10;   // uniform
    key_cut = fs.key_p;
  }
  if (whole_row_draw<DT>(row, V, has_pen, bm, pre, cnt, hd, fs, rp.tau, rp.greedy, m, zmax, c_row, j24, key_cut,
                         minp_on, t_minp) != 1)
    return 13;                                                                // uniform
  if (threadIdx.x == 0) {
    const int token = fs.token;
    a.out_ids[b] = token;
    if (a.k_lp >= 0) {
      const int cols = 1 + a.k_lp;
      a.out_lp_ids[(size_t)b * cols] = token;
      a.out_lp[(size_t)b * cols] = (float)((double)value_of(fs.token_key) - (double)m - lnZ);
    }
  }
  return 1;
}

}  // namespace sip
