// Finishing kernel of the single-pass path: one 1024-thread workgroup per row turns what the
// streaming kernel left behind -- a few thousand (value, index) candidates that are complete
// above a value threshold, plus the integer mass of everything else -- into the row's token,
// its logprob and the best-n list, without reading the logits again (except for the at most
// |history| elements that carry a penalty).
//
// The candidate list L is held in LDS.  Every sum is an integer sum (masses in units of 2^-40
// of the maximum's mass), so no result depends on the order in which threads add.
// Selection works on 2048 linear value bins between the completeness threshold and the
// maximum: one histogram pass locates the bin that holds the k-th largest value, the nucleus
// cut or the n-th best, and the handful of entries in that bin are then resolved by
// all-pairs comparison.  The draw does the same over 2048 bins of the vocabulary index.
//
// Whenever the list cannot prove the answer (a cut falls below the completeness threshold,
// a bin or a segment overflows, too many distinct history tokens, ...) the function returns a
// reason code > 1 before writing any output and the caller runs the exact multi-pass path on
// the row; 1 means the row is finished.
#pragma once
#include "sip_device.h"
#include "sip_exact.h"
#include "sip_stream.h"

namespace sip {

constexpr int kFinalThreads = kExactThreads;
constexpr int kFinalWaves = kFinalThreads / kWave;
constexpr int kBins = 2048;
constexpr int kMembers = 256;        // entries of one bin that can be resolved by all-pairs comparison
constexpr int kSideMax = 4096;       // distinct history tokens per row the fast path handles
constexpr int kMaxChunks = 32;
constexpr int kTopList = 320;        // entries at or above the bin of the n-th best

struct FastShared {
  float Tc[kMaxChunks];
  int R[kMaxChunks];
  unsigned long long bulk[kMaxChunks];
  uint32_t segoff[kMaxChunks * kStreamWaves + 1];
  unsigned long long r64[kFinalWaves];
  long long rcorr[kFinalWaves];
  uint32_t r32[kFinalWaves];
  float rf[kFinalWaves];
  int ri[kFinalWaves];
  uint32_t fail, ndist, nlist, anyc, dropped;
  int bin_k, bin_n, bin_p, bin_low, bin_d;
  uint32_t above_k, above_n, cnt_complete;
  uint32_t key_k, key_p, token_key;
  int token;
  unsigned long long s1_part, before_d;
  uint32_t n_memb;
  uint32_t m_key[kMembers];
  uint32_t m_idx[kMembers];
  unsigned long long m_E[kMembers];
  uint32_t n_top;
  uint32_t t_key[kTopList];
  uint32_t t_idx[kTopList];
  uint32_t t_bin[kTopList];
};

// Bytes of dynamic LDS the finishing kernel needs for vocabulary V and nc_cap candidates.
__host__ __device__ inline size_t final_lds_fixed(int V) {
  const size_t W = ((size_t)V + 31) / 32;
  return ((W * 4 + W * 2 + 15) / 16) * 16 + (size_t)kBins * 12;
}

template <int DT>
__device__ __forceinline__ float load_elem(const char* row, int v) {
  if (DT == SIP_F32) return reinterpret_cast<const float*>(row)[v];
  return __uint_as_float((uint32_t)reinterpret_cast<const unsigned short*>(row)[v] << 16);
}

// Development aid: with -DSIP_TIMING workgroup 0 records a 100 MHz timestamp at each mark
// behind the per-row path codes in the workspace.
#ifdef SIP_TIMING
#define SIP_MARK(i) do { if (blockIdx.x == 0 && threadIdx.x == 0) \
    reinterpret_cast<long long*>(a.row_path + ((a.B + 1) & ~1))[i] = wall_clock64(); } while (0)
#else
#define SIP_MARK(i) do { } while (0)
#endif

template <int DT>
__device__ int fast_row(const Args& a, const int b, const RowParams& rp, unsigned char* dyn, FastShared& fs) {
  const int tid = threadIdx.x, lane = lane_id(), wave = wave_id();
  const int V = a.V, S = a.S;
  const int W = (V + 31) >> 5;
  // ---- LDS carving
  uint32_t* bm = reinterpret_cast<uint32_t*>(dyn);
  unsigned short* pre = reinterpret_cast<unsigned short*>(dyn + (size_t)W * 4);
  unsigned char* p2 = dyn + (((size_t)W * 6 + 15) / 16) * 16;
  unsigned long long* hm = reinterpret_cast<unsigned long long*>(p2);
  uint32_t* hc = reinterpret_cast<uint32_t*>(p2 + (size_t)kBins * 8);
  uint32_t* ck = reinterpret_cast<uint32_t*>(p2 + (size_t)kBins * 12);
  uint32_t* ci = ck + a.nc_cap;
  const uint32_t nc_cap = (uint32_t)a.nc_cap;
  const char* row = reinterpret_cast<const char*>(a.logits) + (size_t)b * (size_t)a.row_stride * (DT == SIP_F32 ? 4 : 2);

  auto scaled_s = [&](float z) { return rp.greedy ? z : __fdiv_rn(z, rp.tau); };
  // checkpoint: returns true (uniformly) if any thread has reported a failure so far
  auto failed = [&]() {
    __syncthreads();
    const uint32_t f = fs.fail;
    __syncthreads();
    return f != 0;
  };

  SIP_MARK(0);
  // ---- (0) chunk summaries
  if (tid == 0) {
    fs.fail = 0; fs.ndist = 0; fs.nlist = 0; fs.anyc = 0; fs.dropped = 0;
    fs.bin_k = -1; fs.bin_n = -1; fs.bin_p = 1 << 30; fs.bin_low = 1 << 30; fs.bin_d = -1;
    fs.key_p = 0xFFFFFFFFu; fs.s1_part = 0; fs.n_memb = 0; fs.n_top = 0; fs.token = 0x7FFFFFFF;
  }
  if (tid < S) {
    const ChunkOut co = a.chunks[(size_t)b * S + tid];
    fs.Tc[tid] = co.Tc; fs.R[tid] = co.R; fs.bulk[tid] = co.bulk;
#pragma unroll
    for (int w = 0; w < kStreamWaves; ++w) fs.segoff[tid * kStreamWaves + w + 1] = co.cnt[w];
  }
  __syncthreads();
  const int nseg = S * kStreamWaves;
  if (tid < nseg && fs.segoff[tid + 1] > (uint32_t)a.cap_w) fs.fail = 1;      // a segment overflowed
  float T_row = -INFINITY;
  int R_max = -(1 << 30);
  for (int c = 0; c < S; ++c) { T_row = fmaxf(T_row, fs.Tc[c]); R_max = max(R_max, fs.R[c]); }
  if (!(T_row == T_row)) fs.fail = 1;
  if (failed()) return 3;
  // prefix of segment sizes (thread 0 .. nseg-1 each sum their predecessors; nseg <= 128)
  uint32_t my_off = 0;
  if (tid <= nseg)
    for (int i = 1; i <= tid; ++i) my_off += fs.segoff[i];
  __syncthreads();
  if (tid <= nseg) fs.segoff[tid] = my_off;
  __syncthreads();
  const uint32_t total_seg = fs.segoff[nseg];

  float chi, clo;
  scale_pair(rp, chi, clo);

  SIP_MARK(1);
  // ---- (1) history: which tokens carry a penalty, how often they occur, their penalised value
  long long lo = 0, hi = 0;
  if (a.indptr && a.tokens && a.nnz > 0) {
    lo = a.indptr[b]; hi = a.indptr[b + 1];
    lo = lo < 0 ? 0 : (lo > a.nnz ? a.nnz : lo);
    hi = hi < lo ? lo : (hi > a.nnz ? a.nnz : hi);
  }
  const bool has_pen = (hi > lo) && (rp.theta != 1.0f || rp.phi != 0.0f || rp.psi != 0.0f);
  uint32_t ndist = 0;
  long long corr = 0;               // mass the streaming pass counted for elements that carry a penalty
  if (has_pen) {
    uint32_t* cnt = reinterpret_cast<uint32_t*>(hm);       // kSideMax counters, before the bins are needed
    for (int w = tid; w < W; w += kFinalThreads) bm[w] = 0;
    for (int i = tid; i < kSideMax; i += kFinalThreads) cnt[i] = 0;
    __syncthreads();
    for (long long i = lo + tid; i < hi; i += kFinalThreads) {
      const int t = a.tokens[i];
      if (t >= 0 && t < V) atomicOr(&bm[t >> 5], 1u << (t & 31));
    }
    __syncthreads();
    for (int w = tid; w < W; w += kFinalThreads) {
      const uint32_t bits = bm[w];
      if (bits) {
        const uint32_t base = atomicAdd(&fs.ndist, (uint32_t)__popc(bits));
        pre[w] = (unsigned short)min(base, 65535u);
      }
    }
    __syncthreads();
    ndist = fs.ndist;
    if (ndist > (uint32_t)kSideMax || ndist > nc_cap) return 4;       // uniform: nothing written yet
    if (rp.phi != 0.0f) {
      for (long long i = lo + tid; i < hi; i += kFinalThreads) {
        const int t = a.tokens[i];
        if (t >= 0 && t < V) {
          const uint32_t word = bm[t >> 5];
          atomicAdd(&cnt[pre[t >> 5] + __popc(word & ((1u << (t & 31)) - 1u))], 1u);
        }
      }
      __syncthreads();
    }
    for (int w = tid; w < W; w += kFinalThreads) {
      uint32_t bits = bm[w];
      uint32_t slot = pre[w];
      while (bits) {
        const int v = (w << 5) + __ffs((int)bits) - 1;
        bits &= bits - 1;
        const float raw = load_elem<DT>(row, v);
        ck[slot] = __float_as_uint(penalise(raw, cnt[slot], rp.theta, rp.phi, rp.psi));
        ci[slot] = (uint32_t)v;
        // the streaming pass saw the raw value: if it was below its chunk's threshold it went
        // into the bulk sum and has to come out again
        const int c = v / a.chunk_len;
        if (!(raw >= fs.Tc[c])) {
          const float zb = fmaxf(raw, -3.0e38f);
          float y = __fmaf_rn(zb, chi, -(float)fs.R[c]);
          y = __fmaf_rn(zb, clo, y);
          const unsigned long long u = (unsigned long long)(uint32_t)(__builtin_amdgcn_exp2f(y) * kBulkScale);
          const int sh = R_max - fs.R[c];
          corr += (long long)(sh < 64 ? (u >> sh) : 0ull);
        }
        ++slot;
      }
    }
  }

  SIP_MARK(2);
  // ---- (2) candidates of all segments -> LDS, minus the ones that carry a penalty
  {
    const uint2* segs = a.cand + (size_t)b * (size_t)nseg * (size_t)a.cap_w;
    for (uint32_t base = 0; base < total_seg; base += kFinalThreads) {
      const uint32_t i = base + tid;
      bool keep = false;
      uint2 e = make_uint2(0, 0);
      if (i < total_seg) {
        int s0 = 0, s1 = nseg;                     // segoff[s0] <= i < segoff[s1]
        while (s1 - s0 > 1) {
          const int mid = (s0 + s1) >> 1;
          if (fs.segoff[mid] <= i) s0 = mid; else s1 = mid;
        }
        e = segs[(size_t)s0 * a.cap_w + (i - fs.segoff[s0])];
        keep = e.y < (uint32_t)V;
        if (keep && has_pen) keep = ((bm[e.y >> 5] >> (e.y & 31)) & 1u) == 0;
      }
      const unsigned long long mask = __ballot(keep);
      uint32_t wbase = 0;
      if (lane == 0 && mask) wbase = atomicAdd(&fs.nlist, (uint32_t)__popcll(mask));
      wbase = (uint32_t)__shfl((int)wbase, 0, kWave);
      if (keep) {
        const uint32_t pos = ndist + wbase + __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32),
                                                 __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
        if (pos < nc_cap) { ck[pos] = e.x; ci[pos] = e.y; }
      }
    }
  }
  __syncthreads();
  const uint32_t nlist = ndist + fs.nlist;
  if (nlist > nc_cap || nlist == 0) return 5;                           // uniform

  SIP_MARK(3);
  // ---- (3) maximum (lowest index on ties) and whether the list is complete where it matters
  float best = -INFINITY;
  int best_i = 0x7FFFFFFF;
  bool anyc = false;
  for (uint32_t i = tid; i < nlist; i += kFinalThreads) {
    const float z = __uint_as_float(ck[i]);
    const int v = (int)ci[i];
    if (z > best || (z == best && v < best_i)) { best = z; best_i = v; }
    anyc |= (i >= ndist) && (z >= T_row);
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const float ob = __shfl_xor(best, o, kWave);
    const int oi = __shfl_xor(best_i, o, kWave);
    if (ob > best || (ob == best && oi < best_i)) { best = ob; best_i = oi; }
  }
  corr = wave_sum((long long)corr);
  if (lane == 0) { fs.rf[wave] = best; fs.ri[wave] = best_i; fs.rcorr[wave] = corr; }
  if (__any(anyc) && lane == 0) fs.anyc = 1;
  __syncthreads();
  best = fs.rf[0]; best_i = fs.ri[0];
  long long corr_total = fs.rcorr[0];
  for (int w = 1; w < kFinalWaves; ++w) {
    const float ob = fs.rf[w]; const int oi = fs.ri[w];
    if (ob > best || (ob == best && oi < best_i)) { best = ob; best_i = oi; }
    corr_total += fs.rcorr[w];
  }
  // an unpenalised candidate at or above T_row proves that nothing outside the list is larger
  if (!fs.anyc || best_i == 0x7FFFFFFF) return 6;                       // uniform
  const float m = scaled_s(best);
  const float s_c = scaled_s(T_row);            // entries with s > s_c: every such element of the row is in L
  const uint32_t key_c = key_of(s_c);
  const float span = __fsub_rn(m, s_c);
  if (!(span >= 0.0f) || !(span < 3.0e38f)) return 7;                   // uniform
  const float binscale = span > 0.0f ? (float)(kBins - 2) / span : 0.0f;
  auto bin_of = [&](float s, uint32_t key) -> int {
    if (key <= key_c) return 0;
    const int q = (int)(__fsub_rn(s, s_c) * binscale);
    return 1 + min(kBins - 2, max(q, 0));
  };
  auto mass = [&](float s) { return fix_of(expf(__fsub_rn(s, m))); };

  SIP_MARK(4);
  // ---- (4) keys, value histogram (count and mass per bin), suffix sums
  for (int i = tid; i < kBins; i += kFinalThreads) { hc[i] = 0; hm[i] = 0; }
  __syncthreads();
  for (uint32_t i = tid; i < nlist; i += kFinalThreads) {
    const float s = scaled_s(__uint_as_float(ck[i]));
    const uint32_t key = key_of(s);
    ck[i] = key;
    const int bin = bin_of(s, key);
    atomicAdd(&hc[bin], 1u);
    const unsigned long long E = mass(s);
    if (E) atomicAdd(&hm[bin], E);
  }
  __syncthreads();
  const bool k_act = !rp.greedy && rp.top_k >= 2 && rp.top_k < V;
  const uint32_t n_top = (uint32_t)max(0, min(a.k_lp, V));
  unsigned long long S_cand;
  {
    // thread t owns bins kBins-1-2t (upper) and kBins-2-2t (lower); scan in descending bin order
    const int bu = kBins - 1 - 2 * tid, bl = bu - 1;
    const uint32_t cu = hc[bu], cl = hc[bl];
    const unsigned long long mu = hm[bu], ml = hm[bl];
    const uint32_t c2 = cu + cl;
    const unsigned long long m2 = mu + ml;
    const uint32_t cinc = wave_incl_scan_u32(c2);
    const unsigned long long minc = wave_incl_scan_u64(m2);
    if (lane == kWave - 1) { fs.r32[wave] = cinc; fs.r64[wave] = minc; }
    __syncthreads();
    uint32_t coff = 0, ctot = 0;
    unsigned long long moff = 0, mtot = 0;
    for (int w = 0; w < kFinalWaves; ++w) {
      if (w < wave) { coff += fs.r32[w]; moff += fs.r64[w]; }
      ctot += fs.r32[w]; mtot += fs.r64[w];
    }
    S_cand = mtot;
    const uint32_t cex_u = coff + cinc - c2, cex_l = cex_u + cu;          // entries in bins above
    const unsigned long long mex_u = moff + minc - m2, mex_l = mex_u + mu;
    hm[bu] = mex_u; hm[bl] = mex_l;                                        // exclusive suffix mass
    if (tid == 0) fs.cnt_complete = ctot - hc[0];
    // bins >= 1 only: bin 0 is the incomplete region
    if (k_act) {
      const uint32_t k = (uint32_t)rp.top_k;
      if (bu >= 1 && cex_u < k && k <= cex_u + cu) { fs.bin_k = bu; fs.above_k = cex_u; }
      if (bl >= 1 && cex_l < k && k <= cex_l + cl) { fs.bin_k = bl; fs.above_k = cex_l; }
    }
    if (n_top > 0) {
      if (bu >= 1 && cex_u < n_top && n_top <= cex_u + cu) { fs.bin_n = bu; fs.above_n = cex_u; }
      if (bl >= 1 && cex_l < n_top && n_top <= cex_l + cl) { fs.bin_n = bl; fs.above_n = cex_l; }
    }
    if (bu >= 1 && cu) atomicMin(&fs.bin_low, bu);
    if (bl >= 1 && cl) atomicMin(&fs.bin_low, bl);
  }
  __syncthreads();
  if ((k_act && fs.bin_k < 0) || (n_top > 0 && fs.bin_n < 0)) return 8;  // uniform: k-th / n-th not provably in L
  const int bin_k = k_act ? fs.bin_k : 0, bin_n = fs.bin_n;

  SIP_MARK(5);
  // bulk mass -> units of 2^-40 relative to the maximum
  unsigned long long bulk = 0;
  for (int c = 0; c < S; ++c) {
    const int sh = R_max - fs.R[c];
    bulk += sh < 64 ? (fs.bulk[c] >> sh) : 0ull;
  }
  bulk = (long long)bulk > corr_total ? bulk - (unsigned long long)corr_total : 0ull;
  const double ln2 = 0.6931471805599453094, log2e = 1.4426950408889634074;
  const double bulk_rel = (double)bulk * exp2((double)R_max + 10.0 - (double)m * (rp.greedy ? log2e : log2e));
  const unsigned long long S0 = S_cand + (bulk_rel < 9.0e18 ? (unsigned long long)bulk_rel : 0ull);
  const double lnZ = log((double)S0) - (double)kFixShift * ln2;

  SIP_MARK(6);
  // ---- (5) gather the bin of the k-th largest and everything at or above the bin of the n-th best
  for (uint32_t i = tid; i < nlist; i += kFinalThreads) {
    const uint32_t key = ck[i];
    const float s = value_of(key);
    const int bin = bin_of(s, key);
    if (k_act && bin == bin_k) {
      const uint32_t q = atomicAdd(&fs.n_memb, 1u);
      if (q < (uint32_t)kMembers) { fs.m_key[q] = key; fs.m_E[q] = mass(s); }
    }
    if (n_top > 0 && bin >= bin_n) {
      const uint32_t q = atomicAdd(&fs.n_top, 1u);
      if (q < (uint32_t)kTopList) { fs.t_key[q] = key; fs.t_idx[q] = ci[i]; fs.t_bin[q] = (uint32_t)bin; }
    }
  }
  __syncthreads();
  if (fs.n_memb > (uint32_t)kMembers || fs.n_top > (uint32_t)kTopList) return 9;   // uniform
  uint32_t key_k = 0;
  unsigned long long S1 = S0;
  if (k_act) {
    const uint32_t nm = fs.n_memb, k_rem = (uint32_t)rp.top_k - fs.above_k;
    if ((uint32_t)tid < nm) {
      const uint32_t key = fs.m_key[tid];
      uint32_t gt = 0, ge = 0;
      for (uint32_t q = 0; q < nm; ++q) { const uint32_t kq = fs.m_key[q]; gt += kq > key; ge += kq >= key; }
      if (gt < k_rem && k_rem <= ge) fs.key_k = key;
    }
    __syncthreads();
    key_k = fs.key_k;
    if ((uint32_t)tid < nm && fs.m_key[tid] >= key_k) atomicAdd(&fs.s1_part, fs.m_E[tid]);
    __syncthreads();
    S1 = hm[bin_k] + fs.s1_part;
    __syncthreads();
    if (tid == 0) fs.n_memb = 0;
  }

  int token = best_i;
  uint32_t token_key = key_of(m);
  if (!rp.greedy) {
    SIP_MARK(7);
    // ---- (6) top-p
    const bool minp_on = rp.min_p > 0.0f;
    const float t_minp = minp_on ? (float)log((double)rp.min_p) : 0.0f;
    // every element missing from L fails min-p  <=>  the completeness threshold itself fails it
    const bool minp_bounds = minp_on && !(__fsub_rn(s_c, m) >= t_minp);
    uint32_t key_cut = key_k;
    if (rp.top_p < 1.0f) {
      const double lim = ceil((double)rp.top_p * (double)S1);
      const unsigned long long limit = lim > 0.0 ? (unsigned long long)lim : 0ull;
      const int lowbin = k_act ? bin_k : 1;
      {
        const int bu = kBins - 1 - 2 * tid, bl = bu - 1;
        if (bu >= lowbin && hc[bu] && hm[bu] < limit) atomicMin(&fs.bin_p, bu);
        if (bl >= lowbin && hc[bl] && hm[bl] < limit) atomicMin(&fs.bin_p, bl);
      }
      __syncthreads();
      const int bin_p = fs.bin_p;
      if (bin_p >= kBins) return 10;                                      // uniform (p <= 0)
      for (uint32_t i = tid; i < nlist; i += kFinalThreads) {
        const uint32_t key = ck[i];
        const float s = value_of(key);
        if (key >= key_k && bin_of(s, key) == bin_p) {
          const uint32_t q = atomicAdd(&fs.n_memb, 1u);
          if (q < (uint32_t)kMembers) { fs.m_key[q] = key; fs.m_E[q] = mass(s); }
        }
      }
      __syncthreads();
      const uint32_t nm = fs.n_memb;
      if (nm > (uint32_t)kMembers) return 9;                                 // uniform
      if ((uint32_t)tid < nm) {
        const uint32_t key = fs.m_key[tid];
        unsigned long long G = hm[bin_p];
        for (uint32_t q = 0; q < nm; ++q)
          if (fs.m_key[q] > key) G += fs.m_E[q];
        if (G < limit) atomicMin(&fs.key_p, key); else fs.dropped = 1;
      }
      __syncthreads();
      const bool inside = k_act || bin_p > fs.bin_low || fs.dropped != 0;
      if (!inside && !minp_bounds) return 11;                             // uniform: the cut may lie below L
      key_cut = max(key_k, fs.key_p);
      __syncthreads();
      if (tid == 0) fs.n_memb = 0;
    } else if (!k_act && !minp_bounds) {
      return 12;                                                             // uniform: nothing bounds the kept set inside L
    }

    SIP_MARK(8);
    // ---- (7) draw: kept mass per index bin, prefix, then resolve inside the crossing bin
    auto kept = [&](float s, uint32_t key) {
      return key >= key_cut && key > key_c && (!minp_on || __fsub_rn(s, m) >= t_minp);
    };
    int ishift = 0;
    while (((V - 1) >> ishift) >= kBins) ++ishift;
    __syncthreads();
    for (int i = tid; i < kBins; i += kFinalThreads) hm[i] = 0;
    __syncthreads();
    for (uint32_t i = tid; i < nlist; i += kFinalThreads) {
      const uint32_t key = ck[i];
      const float s = value_of(key);
      if (kept(s, key)) {
        const unsigned long long E = mass(s);
        if (E) atomicAdd(&hm[ci[i] >> ishift], E);
      }
    }
    __syncthreads();
    unsigned long long target;
    {
      const unsigned long long m0 = hm[2 * tid], m1 = hm[2 * tid + 1];
      const unsigned long long m2 = m0 + m1;
      const unsigned long long minc = wave_incl_scan_u64(m2);
      if (lane == kWave - 1) fs.r64[wave] = minc;
      __syncthreads();
      unsigned long long moff = 0, S3 = 0;
      for (int w = 0; w < kFinalWaves; ++w) {
        if (w < wave) moff += fs.r64[w];
        S3 += fs.r64[w];
      }
      const unsigned long long j = philox_word0(a.seed, rp.row_id, a.step) >> 8;
      target = (__umul64hi(j, S3) << 40) | ((j * S3) >> 24);               // floor(j * S3 / 2^24)
      const unsigned long long ex0 = moff + minc - m2, ex1 = ex0 + m0;
      if (ex0 <= target && target < ex0 + m0) { fs.bin_d = 2 * tid; fs.before_d = ex0; }
      if (ex1 <= target && target < ex1 + m1) { fs.bin_d = 2 * tid + 1; fs.before_d = ex1; }
    }
    __syncthreads();
    const int bin_d = fs.bin_d;
    if (bin_d < 0) return 13;                                             // uniform (no kept mass)
    for (uint32_t i = tid; i < nlist; i += kFinalThreads) {
      const uint32_t key = ck[i];
      const float s = value_of(key);
      if ((int)(ci[i] >> ishift) == bin_d && kept(s, key)) {
        const uint32_t q = atomicAdd(&fs.n_memb, 1u);
        if (q < (uint32_t)kMembers) { fs.m_key[q] = key; fs.m_idx[q] = ci[i]; fs.m_E[q] = mass(s); }
      }
    }
    __syncthreads();
    const uint32_t nm = fs.n_memb;
    if (nm > (uint32_t)kMembers) return 9;                                   // uniform
    if ((uint32_t)tid < nm) {
      const uint32_t v = fs.m_idx[tid];
      unsigned long long C = fs.before_d;
      for (uint32_t q = 0; q < nm; ++q)
        if (fs.m_idx[q] <= v) C += fs.m_E[q];
      if (C > target) atomicMin(&fs.token, (int)v);
    }
    __syncthreads();
    token = fs.token;
    if (token == 0x7FFFFFFF) return 13;                                   // uniform
    if ((uint32_t)tid < nm && fs.m_idx[tid] == (uint32_t)token) fs.token_key = fs.m_key[tid];
    __syncthreads();
    token_key = fs.token_key;
  }

  SIP_MARK(9);
  // ---- (8) outputs.  Past this point nothing can fail.
  if (tid == 0) a.out_ids[b] = token;
  if (a.k_lp >= 0) {
    const int cols = 1 + a.k_lp;
    if (tid == 0) {
      a.out_lp_ids[(size_t)b * cols] = token;
      a.out_lp[(size_t)b * cols] = (float)((double)value_of(token_key) - (double)m - lnZ);
    }
    if (n_top > 0) {
      const uint32_t nt = fs.n_top, need = n_top - fs.above_n;     // entries wanted from the n-th best's own bin
      bool sel = false;
      uint32_t key = 0, v = 0;
      if ((uint32_t)tid < nt) {
        key = fs.t_key[tid]; v = fs.t_idx[tid];
        if ((int)fs.t_bin[tid] > bin_n) sel = true;
        else {
          uint32_t rank = 0;
          for (uint32_t q = 0; q < nt; ++q)
            if ((int)fs.t_bin[q] == bin_n) {
              const uint32_t kq = fs.t_key[q];
              rank += (kq > key || (kq == key && fs.t_idx[q] < v)) ? 1u : 0u;
            }
          sel = rank < need;
        }
      }
      __syncthreads();
      if ((uint32_t)tid < nt) fs.t_bin[tid] = sel ? 1u : 0u;
      __syncthreads();
      if (sel) {
        uint32_t pos = 0;
        for (uint32_t q = 0; q < nt; ++q)
          if (fs.t_bin[q]) {
            const uint32_t kq = fs.t_key[q];
            pos += (kq > key || (kq == key && fs.t_idx[q] < v)) ? 1u : 0u;
          }
        a.out_lp_ids[(size_t)b * cols + 1 + pos] = (int)v;
        a.out_lp[(size_t)b * cols + 1 + pos] = (float)((double)value_of(key) - (double)m - lnZ);
      }
    }
  }
  SIP_MARK(10);
  return 1;
}

template <int DT>
__global__ __launch_bounds__(kFinalThreads) void final_kernel(Args a) {
  extern __shared__ __align__(16) unsigned char dynraw[];
  __shared__ ExactShared ex;
  __shared__ FastShared fs;
  const int b = blockIdx.x;
  const RowParams rp = load_row_params(a, b);
  int how = 2;                                   // 2: not eligible for the single-pass path
  if (candidate_target(rp, a) != 0) how = fast_row<DT>(a, b, rp, dynraw, fs);
  if (how != 1) {
    __syncthreads();
    exact_row<DT>(a, b, reinterpret_cast<uint32_t*>(dynraw), ex);
  }
  if (threadIdx.x == 0) a.row_path[b] = how;
}

}  // namespace sip
