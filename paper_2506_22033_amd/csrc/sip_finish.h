// Finishing kernel of the single-pass path: one workgroup per row turns what the streaming
// kernel left behind -- a list of a few thousand (value, index) entries that holds every
// element at or above a value threshold and every element that carries a penalty, plus the
// integer mass of everything else -- into the row's token, its logprob and the best-n list.
// It never reads the logits.
//
// Steps (Sec. 2.1 step 3 (1)-(3); Sec. 5.1 ApplyPenalty / temperature / softmax / filters /
// draw), every sum an integer sum (masses in units of 2^-40 of the maximum's mass) so that no
// result depends on the order in which threads add:
//   (1) multiplicities of the history tokens in an LDS hash table (frequency penalty only);
//   (2) penalised value of every tagged entry, maximum of the list (lowest index on ties);
//   (3) s = z'/tau (IEEE), key, mass and value bin of every entry; count and mass per bin
//       (1024 linear bins between the completeness threshold and the maximum);
//   (4) one descending scan over the bins gives, per bin, the number and the mass of all
//       entries above it: that locates the bin of the k-th largest, of the n-th best and of
//       the nucleus cut, and is the position at which the bin's entries are then laid down in
//       LDS (a counting sort by bin), so that the members of any bin, and everything above
//       it, are a contiguous range;
//   (5) one wave settles top-k, then top-p, inside their bins (all pairs through readlane,
//       or by descending over the distinct keys of a bin with many ties) while another wave
//       ranks the best-n;
//   (6) draw: kept sets of up to 64 entries by that same wave from its registers; larger
//       ones through a histogram of kept mass over 1024 vocabulary-index bins.
//
// Whatever the list cannot prove (a cut that may lie below the completeness threshold, an
// overflow, a bin with too many members, ...) makes the row's number go to the rescue queue
// with a reason code; rescue_kernel (sip_final.h) then takes the row over.
#pragma once
#include "sip_device.h"
#include "sip_stream.h"

namespace sip {
constexpr int kFinThreads = 512;
constexpr int kFinWaves = kFinThreads / kWave;
constexpr int kFinCR = 10;                             // list entries a thread holds in registers
constexpr int kFinBins = 1024;
constexpr int kFinBPT = kFinBins / kFinThreads;        // bins per thread in the scans
constexpr int kFinList = 4352;                         // entries of the bin-sorted list in LDS
constexpr int kFinHash = 4096;                         // slots of the multiplicity table
constexpr int kFinHashMax = 3072;                      // distinct history tokens it takes
constexpr int kFinMembers = 512;                       // members of one index bin the draw resolves
constexpr int kFinTopMax = 256;                        // entries at or above the bin of the n-th best
constexpr int kFinKeySteps = 64;                       // distinct keys of one bin that are stepped through
constexpr uint32_t kFinNone = 0xFFFFFFFFu;
constexpr int kFinDrawBig = -1;                        // internal: the draw goes through the index histogram
static_assert(kFinBPT == 2, "scan code below is written for two bins per thread");

struct __align__(16) FinShared {
  uint32_t hcnt[kFinBins];                  // entries per value bin
  uint32_t off[kFinBins];                   // entries in all higher bins = where the bin starts in the sorted list
  uint32_t fill[kFinBins];                  // entries of the bin laid down so far
  unsigned long long hmass[kFinBins];       // mass per value bin; after the scan: mass of all higher bins
  unsigned long long hidx[kFinBins];        // kept mass per vocabulary-index bin
  union {
    struct { uint32_t skey[kFinList]; uint32_t sidx[kFinList]; } list;      // entries sorted by bin, descending
    struct { uint32_t key[kFinHash]; uint32_t val[kFinHash]; } hash;        // token -> multiplicity (before the list exists)
  } u;
  uint32_t m_key[kFinMembers];
  uint32_t m_idx[kFinMembers];
  unsigned long long m_E[kFinMembers];
  unsigned long long r64[kFinWaves];
  uint32_t r32[kFinWaves], rkey[kFinWaves], ridx[kFinWaves];
  int bin_k, bin_n, bin_d;
  int code, code_top;
  int retry_ok;                             // code 11 only: a second, longer list can be expected to hold the nucleus
  uint32_t hash_fail, n_memb, key_cut, n_hi;
  uint32_t token, token_key;
  unsigned long long before_d;
};

// Sum / maximum over the 64 lanes, result in every lane (through scalar registers).
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v) { return last_lane_u32(dpp_scan_max_u32(v)); }
__device__ __forceinline__ uint32_t wave_min_u32(uint32_t v) { return last_lane_u32(dpp_scan_min_u32(v)); }
__device__ __forceinline__ uint32_t wave_add_u32(uint32_t v) { return last_lane_u32(dpp_scan_add_u32(v)); }
__device__ __forceinline__ unsigned long long wave_add_u64(unsigned long long v) { return last_lane_u64(dpp_scan_add_u64(v)); }

// Barrier for code that only exchanges data through LDS: unlike __syncthreads() it does not wait
// for global loads that are still in flight.
__device__ __forceinline__ void lds_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// What a caller that goes on with a row this function could not settle may reuse (uniform).
struct FinHint {
  bool valid = false;        // m, zmax and T are the row's
  bool retry_ok = false;     // code 11: a second, longer list can be expected to hold the nucleus
  float m = 0.0f;            // maximum of s
  float zmax = 0.0f;         // maximum of z'
  float T = 0.0f;            // every element of the row above T is in the list
};

// Row b, start to finish.  Returns 1 (finished: outputs written) or the reason why the list
// does not settle the row.  Every return value is workgroup-uniform.
__device__ __forceinline__ int finish_row(const Args& a, const int b, FinShared& fs, FinHint* hint = nullptr) {
  constexpr int NT = kFinThreads;
  constexpr int CR = kFinCR;
  const int tid = threadIdx.x, lane = lane_id(), wave = wave_id();
  const int V = a.V;
  const int S = a.S;

  // ---- (0) Everything this kernel reads from memory has an address that does not depend on
  // anything else it reads, except the history tokens: the row's parameters and history extent
  // (one record, left by the streaming kernel), the chunk summaries (lane c reads chunk c) and
  // the list itself are requested at once.  The list is read before the segment sizes are
  // known: thread t belongs to segment t / tps and takes, in round r, slot r * tps + t % tps of
  // it; slots beyond the segment's size are dropped afterwards.
  const int tps = a.fin_tps;                                   // kFinThreads / S
  int c_seg = (tid * a.fin_inv) >> 16;                         // tid / tps, put right below
  c_seg -= c_seg * tps > tid;
  const int j_seg = tid - c_seg * tps;
  const bool seg_thread = c_seg < S;
  uint2* seg = a.cand + ((size_t)b * (size_t)S + (size_t)min(c_seg, S - 1)) * (size_t)a.cap_c;
  uint2 creg[CR];                          // (bits of z, later of z' and then the key of s; index | tag, later index)
  auto slot_of = [&](int bt, int r) { return (bt * CR + r) * tps + j_seg; };
  // Unchecked against the sizes, and unconditional (a branch around a load makes the compiler wait
  // for every load in flight where the branches meet): slots past the segment's capacity read its
  // last slot, threads without a segment the last segment's; drop_beyond() discards what they get.
  auto load_batch = [&](int bt) {
#pragma unroll
    for (int r = 0; r < CR; ++r) creg[r] = seg[min(slot_of(bt, r), a.cap_c - 1)];
  };
  // (the two small records first: loads come back in the order of their requests, and what
  // depends on the records -- the history loads, the plan of the phases -- need not wait for the list)
  // The early exits below name the list's registers as well: with no use of the list on those
  // paths the compiler would move the list's loads behind the exits' branches, that is, behind the
  // wait for the records.
  // (The same goes for the part of the chunk summary that the exits do not look at.)
  unsigned long long my_bulk = 0;
  auto list_is_used = [&]() {
#pragma unroll
    for (int r = 0; r < CR; ++r) asm volatile("" ::"v"(creg[r].x), "v"(creg[r].y));
    asm volatile("" ::"v"((uint32_t)my_bulk), "v"((uint32_t)(my_bulk >> 32)));
  };
  const RowInfo ri = a.rowinfo[b];
  const ChunkOut co = a.chunks[(size_t)b * S + min(lane, S - 1)];
  load_batch(0);
  uint32_t my_cnt = 0;
  float Tc;
  int R;
  {
    if (lane < S) { my_cnt = co.cnt; my_bulk = co.bulk; }
    Tc = __uint_as_float((uint32_t)__builtin_amdgcn_readfirstlane((int)__float_as_uint(co.Tc)));   // the chunks of a row share
    R = __builtin_amdgcn_readfirstlane(co.R);                                                      // threshold and exponent
  }
  if ((ri.target & ~kPromptFlag) == 0) { list_is_used(); return 2; }          // uniform: k beyond any list
  const bool prompt_on = (ri.target & kPromptFlag) != 0;                     // tokens of a separate prompt are tagged too
  RowParams rp;
  rp.tau = ri.tau; rp.top_p = ri.top_p; rp.min_p = ri.min_p; rp.theta = ri.theta; rp.phi = ri.phi; rp.psi = ri.psi;
  rp.top_k = ri.top_k; rp.row_id = ri.row_id;
  rp.greedy = (rp.tau == 0.0f) || (rp.top_k == 1);
  auto scaled_s = [&](float z) { return rp.greedy ? z : __fdiv_rn(z, rp.tau); };
  const long long h_lo = ri.lo, h_hi = ri.hi;
  // multiplicities in the history are needed for the frequency penalty, and, next to a separate
  // prompt, to tell the tokens that frequency and presence apply to (see penalty_plan())
  const bool need_hash = (h_hi > h_lo) && (rp.phi != 0.0f || (prompt_on && rp.psi != 0.0f));
  const uint32_t mult_dflt = (h_hi > h_lo) ? 1u : 0u;
  // a device-resident state keeps the row's table of multiplicities: copy it instead of counting
  // (32 KB to copy against 4 bytes and two LDS atomics per history token: it pays from about two
  // thousand tokens on)
  const bool use_table = need_hash && ri.slot >= 0 && ri.ndist >= 0 && ri.hi - ri.lo > 2048;
  static_assert(kFinHash == kTableSlots && kFinHashMax == kTableMaxDistinct, "one table geometry");
  constexpr int HR = 8;                    // history tokens a thread requests at once
  int htok[HR];
#pragma unroll
  for (int j = 0; j < HR; ++j) {
    const long long i = h_lo + tid + (long long)j * NT;
    htok[j] = (need_hash && !use_table && i < h_hi) ? a.tokens[i] : -1;
  }
  {
    // hcnt, off, fill, hmass, hidx are contiguous: 28 KB, of which `off` need not be cleared
    uint4* z4 = reinterpret_cast<uint4*>(fs.hcnt);
    for (int i = tid; i < kFinBins * 4 / 16; i += NT) z4[i] = make_uint4(0, 0, 0, 0);
    z4 = reinterpret_cast<uint4*>(fs.fill);
    for (int i = tid; i < kFinBins * 20 / 16; i += NT) z4[i] = make_uint4(0, 0, 0, 0);
    if (use_table) {                       // keys and multiplicities lie one behind the other, here as there
      const uint4* t4 = reinterpret_cast<const uint4*>(a.st_table + (size_t)ri.slot * (size_t)(2 * kTableSlots));
      uint4* k4 = reinterpret_cast<uint4*>(fs.u.hash.key);
      uint4 tq[2 * kFinHash * 4 / 16 / NT];
#pragma unroll
      for (int j = 0; j < 2 * kFinHash * 4 / 16 / NT; ++j) tq[j] = t4[j * NT + tid];
#pragma unroll
      for (int j = 0; j < 2 * kFinHash * 4 / 16 / NT; ++j) k4[j * NT + tid] = tq[j];
    } else if (need_hash) {
      uint4* k4 = reinterpret_cast<uint4*>(fs.u.hash.key);
      for (int i = tid; i < kFinHash * 4 / 16; i += NT) k4[i] = make_uint4(kFinNone, kFinNone, kFinNone, kFinNone);
      uint4* v4 = reinterpret_cast<uint4*>(fs.u.hash.val);
      for (int i = tid; i < kFinHash * 4 / 16; i += NT) v4[i] = make_uint4(0, 0, 0, 0);
    }
    if (tid == 0) {
      fs.bin_k = -1; fs.bin_n = -1; fs.bin_d = -1; fs.code = 0; fs.code_top = 0; fs.hash_fail = 0; fs.n_memb = 0;
      fs.token = kFinNone; fs.token_key = 0;
    }
  }
  // row constants that take long arithmetic, worked out while the loads above travel
  const bool minp_on = !rp.greedy && rp.min_p > 0.0f;
  const float t_minp = minp_on ? (float)log((double)rp.min_p) : 0.0f;
  const unsigned long long j24 = rp.greedy ? 0ull : (unsigned long long)(philox_word0(a.seed, rp.row_id, step_of(a)) >> 8);
  const bool k_act = !rp.greedy && rp.top_k >= 2 && rp.top_k < V;
  const uint32_t n_top = (uint32_t)max(0, min(a.k_lp, V));

  const bool any_over = __any(my_cnt > (uint32_t)a.cap_c);                   // includes the overflow mark
  const uint32_t total = wave_add_u32(my_cnt);
  const uint32_t longest = wave_max_u32(my_cnt);
  const unsigned long long bulk = wave_add_u64(my_bulk);
  if (any_over || !(Tc == Tc)) { list_is_used(); return 3; }                 // uniform
  if (total > (uint32_t)a.nc_cap) { list_is_used(); return 5; }              // uniform
  const int nb = (int)((longest + (uint32_t)(CR * tps) - 1) / (uint32_t)(CR * tps));   // uniform: batches of CR rounds
  const int cnt_seg = seg_thread ? __shfl((int)my_cnt, c_seg, kWave) : 0;    // size of this thread's segment
  // whether round r of batch bt holds anything at all (uniform): every round is unrolled code that
  // costs time even when no lane has an entry, unless the whole wave branches around it
  auto live = [&](int bt, int r) { return (uint32_t)((bt * CR + r) * tps) < longest; };
  auto drop_beyond = [&](int bt) {
#pragma unroll
    for (int r = 0; r < CR; ++r)
      if (!(slot_of(bt, r) < cnt_seg)) creg[r] = make_uint2(0u, kFinNone);
  };
  lds_barrier();                                                             // LDS is clear

  // ---- (1) multiplicities: a hash table of kFinHash / 4 buckets of four slots, keyed by token.
  // A bucket's four keys are one 16-byte LDS read; a token lives in the first bucket, from its
  // home bucket on, that had a free slot when it came.  Slots of a bucket fill in order (a thread
  // claims the first slot it finds free, by compare-and-swap), so a key, once there, stays.
  uint4* const hkey4 = reinterpret_cast<uint4*>(fs.u.hash.key);
  auto home = [](uint32_t t) { return (t * 0x9E3779B1u) >> 22; };
  static_assert(kFinHash == 4096, "home() yields 10 bits: 1024 buckets of 4 slots");
  if (need_hash && !use_table) {
    uint32_t mine = 0;                     // slots this thread claimed = distinct tokens it saw first
    auto insert = [&](int ti) {
      if (ti < 0 || ti >= V) return;
      const uint32_t t = (uint32_t)ti;
      uint32_t bk = home(t);
      for (int probe = 0; probe < kFinHash / 4; ++probe) {
        const uint4 k4 = hkey4[bk];
        const uint32_t ks[4] = {k4.x, k4.y, k4.z, k4.w};
        int j = -1;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          if (j < 0 && ks[e] == t) j = e;
          if (j < 0 && ks[e] == kFinNone) {                 // free when read: try to take it
            const uint32_t old = atomicCAS(&fs.u.hash.key[4 * bk + e], kFinNone, t);
            if (old == kFinNone) { ++mine; j = e; } else if (old == t) j = e;
          }
        }
        if (j >= 0) { atomicAdd(&fs.u.hash.val[4 * bk + j], 1u); return; }
        bk = (bk + 1) & (kFinHash / 4 - 1);
      }
      fs.hash_fail = 1;                    // table full
    };
#pragma unroll
    for (int j = 0; j < HR; ++j)
      if ((long long)j * NT < h_hi - h_lo) insert(htok[j]);                  // uniform condition
    for (long long i0 = h_lo + (long long)HR * NT; i0 < h_hi; i0 += (long long)HR * NT) {
#pragma unroll
      for (int j = 0; j < HR; ++j) {
        const long long i = i0 + tid + (long long)j * NT;
        htok[j] = i < h_hi ? a.tokens[i] : -1;
      }
#pragma unroll
      for (int j = 0; j < HR; ++j) insert(htok[j]);
    }
    const uint32_t wtot = wave_add_u32(mine);
    if (lane == 0) fs.r32[wave] = wtot;
    lds_barrier();
    uint32_t ndist = 0;
#pragma unroll
    for (int w = 0; w < kFinWaves; ++w) ndist += fs.r32[w];
    if (fs.hash_fail || ndist > (uint32_t)kFinHashMax) return 4;            // uniform
  }
  // multiplicity of token t, searched from bucket bk on (the rare continuation of the lookup
  // below: t's home bucket is full of other tokens); 0 = not in the history (a prompt token)
  auto count_slow = [&](uint32_t t, uint32_t bk) -> uint32_t {
    for (int probe = 0; probe < kFinHash / 4; ++probe) {
      const uint4 k4 = hkey4[bk];
      if (k4.x == t) return fs.u.hash.val[4 * bk];
      if (k4.y == t) return fs.u.hash.val[4 * bk + 1];
      if (k4.z == t) return fs.u.hash.val[4 * bk + 2];
      if (k4.w == t) return fs.u.hash.val[4 * bk + 3];
      if (k4.w == kFinNone) return 0u;     // slots fill in order: a free last slot ends the search
      bk = (bk + 1) & (kFinHash / 4 - 1);
    }
    return 0u;
  };

  // ---- (2) penalised values (Sec. 5.1 ApplyPenalty); maximum of the list, lowest index on ties
  uint32_t bkey = 0, bidx = kFinNone;
  for (int bt = 0; bt < nb; ++bt) {
    if (bt > 0) load_batch(bt);
    drop_beyond(bt);
    // the home buckets of all entries are read from the table together, then the counts
    uint32_t hv[CR];
    if (need_hash) {
      uint4 hk[CR];
#pragma unroll
      for (int r = 0; r < CR; ++r)
        if (live(bt, r)) hk[r] = hkey4[home(creg[r].y & ~kTagBit)];
#pragma unroll
      for (int r = 0; r < CR; ++r) {
        hv[r] = 0u;
        if (!live(bt, r)) continue;
        const uint32_t v = creg[r].y & ~kTagBit, bk = home(v);
        const uint32_t hs = hk[r].x == v ? 4 * bk : hk[r].y == v ? 4 * bk + 1 : hk[r].z == v ? 4 * bk + 2 : hk[r].w == v ? 4 * bk + 3 : kFinNone;
        if (hs != kFinNone) hv[r] = fs.u.hash.val[hs];
        else if (hk[r].w != kFinNone && (creg[r].y & kTagBit) && creg[r].y != kFinNone) hv[r] = count_slow(v, (bk + 1) & (kFinHash / 4 - 1));
      }
    }
#pragma unroll
    for (int r = 0; r < CR; ++r) {
      if (live(bt, r) && creg[r].y != kFinNone) {
        const uint32_t v = creg[r].y & ~kTagBit;
        float z = __uint_as_float(creg[r].x);
        if (creg[r].y & kTagBit) {
          z = penalise(z, need_hash ? hv[r] : mult_dflt, rp.theta, rp.phi, rp.psi);
          // lists of several batches are read again from memory: leave the penalised value there
          if (nb > 1) seg[slot_of(bt, r)] = make_uint2(__float_as_uint(z), v);
        }
        creg[r] = make_uint2(__float_as_uint(z), v < (uint32_t)V ? v : kFinNone);
        const uint32_t kz = key_of(z);
        if (creg[r].y != kFinNone && (kz > bkey || (kz == bkey && v < bidx))) { bkey = kz; bidx = v; }
      }
    }
  }
  {
    const uint32_t wk = wave_max_u32(bkey);
    const uint32_t wi = wave_min_u32(bkey == wk ? bidx : kFinNone);
    if (lane == 0) { fs.rkey[wave] = wk; fs.ridx[wave] = wi; }
  }
  lds_barrier();
  bkey = 0; bidx = kFinNone;
#pragma unroll
  for (int w = 0; w < kFinWaves; ++w) {
    const uint32_t ok = fs.rkey[w], oi = fs.ridx[w];
    if (ok > bkey || (ok == bkey && oi < bidx)) { bkey = ok; bidx = oi; }
  }
  // Every element outside the list is unpenalised and below Tc: a list maximum at or above Tc
  // is the row's maximum, and its lowest index the row's.
  const float zmax = value_of(bkey);
  if (bidx == kFinNone || !(zmax >= Tc)) return 6;                            // uniform
  const float m = scaled_s(zmax);
  if (hint) { hint->valid = true; hint->m = m; hint->zmax = zmax; hint->T = Tc; }
  const float s_c = scaled_s(Tc);          // entries with s > s_c: every such element of the row is in the list
  const uint32_t key_c = key_of(s_c);
  const float span = __fsub_rn(m, s_c);
  if (!(span >= 0.0f) || !(span < 3.0e38f)) return 7;                         // uniform
  const float binscale = span > 0.0f ? (float)(kFinBins - 2) / span : 0.0f;
  auto bin_of = [&](float s, uint32_t k) -> int {
    if (k <= key_c) return 0;
    const int q = (int)(__fsub_rn(s, s_c) * binscale);
    return 1 + min(kFinBins - 2, max(q, 0));
  };
  auto mass = [&](float s) { return fix_of(expf(__fsub_rn(s, m))); };
  auto emit = [&](uint32_t token, uint32_t token_key, double lnZ) {          // one thread
    a.out_ids[b] = (int)token;
    if (a.k_lp >= 0) {
      const int cols = 1 + a.k_lp;
      a.out_lp_ids[(size_t)b * cols] = (int)token;
      a.out_lp[(size_t)b * cols] = (float)((double)value_of(token_key) - (double)m - lnZ);
    }
    if (a.slot) state_append_row(a, b);
  };
  if (rp.greedy && a.k_lp < 0) {           // the arg max is all that is asked for
    if (tid == 0) emit(bidx, key_of(m), 0.0);
    return 1;
  }

  // ---- (3) keys, masses, value histogram
  for (int bt = 0; bt < nb; ++bt) {
    if (nb > 1) { load_batch(bt); drop_beyond(bt); }
#pragma unroll
    for (int r = 0; r < CR; ++r) {
      if (live(bt, r) && creg[r].y != kFinNone) {
        const float s = scaled_s(__uint_as_float(creg[r].x));
        const uint32_t k = key_of(s);
        const int bin = bin_of(s, k);
        const unsigned long long E = mass(s);
        atomicAdd(&fs.hcnt[bin], 1u);
        if (E) atomicAdd(&fs.hmass[bin], E);
        creg[r].x = k;                     // from here on: the key of s
      }
    }
  }
  lds_barrier();

  // ---- (4) descending scan over the bins: thread t owns bins kFinBins-1-2t and kFinBins-2-2t
  unsigned long long S_cand;
  {
    const int b0 = kFinBins - 1 - kFinBPT * tid;
    uint32_t c[kFinBPT];
    unsigned long long w[kFinBPT];
#pragma unroll
    for (int j = 0; j < kFinBPT; ++j) { c[j] = fs.hcnt[b0 - j]; w[j] = fs.hmass[b0 - j]; }
    const uint32_t csum = c[0] + c[1];
    const unsigned long long msum = w[0] + w[1];
    const uint32_t cinc = dpp_scan_add_u32(csum);
    const unsigned long long minc = dpp_scan_add_u64(msum);
    if (lane == kWave - 1) { fs.r32[wave] = cinc; fs.r64[wave] = minc; }
    lds_barrier();
    uint32_t cex = cinc - csum;
    unsigned long long mex = minc - msum, mtot = 0;
#pragma unroll
    for (int ww = 0; ww < kFinWaves; ++ww) {
      const uint32_t c32 = fs.r32[ww];
      const unsigned long long m64 = fs.r64[ww];
      if (ww < wave) { cex += c32; mex += m64; }
      mtot += m64;
    }
    S_cand = mtot;
    const uint32_t k = (uint32_t)rp.top_k;
#pragma unroll
    for (int j = 0; j < kFinBPT; ++j) {
      const int bin = b0 - j;
      fs.off[bin] = cex;
      fs.hmass[bin] = mex;
      if (bin >= 1) {                                                          // bin 0 is the incomplete region
        if (k_act && cex < k && k <= cex + c[j]) fs.bin_k = bin;
        if (n_top > 0 && cex < n_top && n_top <= cex + c[j]) fs.bin_n = bin;
      }
      cex += c[j]; mex += w[j];
    }
  }
  lds_barrier();
  const int bin_k = fs.bin_k, bin_n = fs.bin_n;
  if ((k_act && bin_k < 0) || (n_top > 0 && bin_n < 0)) return 8;              // uniform: k-th / n-th not provably in the list

  // total mass: the list's plus the bulk's, brought to units of 2^-40 of the maximum's mass.
  // 2^x with x split into integer and fraction: the fraction goes through the hardware exp2,
  // the integer part is an exponent shift.  (Only the waves that use it work it out.)
  auto total_mass = [&](double& lnZ) -> unsigned long long {
    const double ln2 = 0.6931471805599453094, log2e = 1.4426950408889634074;
    const double x = fmin(fmax((double)R + 10.0 - (double)m * log2e, -2000.0), 2000.0);
    const double xi = floor(x);
    const double bulk_rel = ldexp((double)bulk * (double)__builtin_amdgcn_exp2f((float)(x - xi)), (int)xi);
    const unsigned long long S0 = S_cand + (bulk_rel < 9.0e18 ? (unsigned long long)bulk_rel : 0ull);
    int e2;
    const float f2 = (float)frexp((double)S0, &e2);
    lnZ = ((double)__builtin_amdgcn_logf(f2) + (double)(e2 - kFixShift)) * ln2;
    return S0;
  };

  // lowest bin any later step looks into: everything from there up is laid down, sorted by bin
  int bin_minp = 1;                        // entries below this bin fail min-p (the reverse need not hold)
  if (minp_on) {
    const float sm = __fadd_rn(m, t_minp);
    const float sm_lo = sm - fabsf(sm) * 1.0e-6f - 1.0e-30f;
    bin_minp = max(1, bin_of(sm_lo, key_of(sm_lo)));
  }
  // every element missing from the list fails min-p  <=>  the completeness threshold itself fails it
  const bool minp_bounds = minp_on && !(__fsub_rn(s_c, m) >= t_minp);
  int lowbin = kFinBins;
  if (!rp.greedy) lowbin = k_act ? bin_k : bin_minp;
  if (n_top > 0) lowbin = min(lowbin, bin_n);
  uint32_t n_list = 0;
  if (lowbin < kFinBins) {
    n_list = fs.off[lowbin] + fs.hcnt[lowbin];
    if (n_list > (uint32_t)kFinList) return 9;                                 // uniform
    for (int bt = 0; bt < nb; ++bt) {
      if (nb > 1) {                         // keys again (the registers hold the last batch only)
        load_batch(bt);
        drop_beyond(bt);
#pragma unroll
        for (int r = 0; r < CR; ++r)
          if (creg[r].y != kFinNone) creg[r].x = key_of(scaled_s(__uint_as_float(creg[r].x)));
      }
#pragma unroll
      for (int r = 0; r < CR; ++r) {
        if (live(bt, r) && creg[r].y != kFinNone) {
          const uint32_t k = creg[r].x;
          const int bin = bin_of(value_of(k), k);
          if (bin >= lowbin) {
            const uint32_t pos = fs.off[bin] + atomicAdd(&fs.fill[bin], 1u);
            if (pos < (uint32_t)kFinList) { fs.u.list.skey[pos] = k; fs.u.list.sidx[pos] = creg[r].y; }
          }
        }
      }
    }
  }
  lds_barrier();

  // ---- (5) wave 1: best-n.  The range [0, nt) of the sorted list holds every element of the
  // row at or above the bin of the n-th best, so an entry's rank in it is its rank in the row.
  if (wave == 1 && n_top > 0) {
    double lnZ;
    total_mass(lnZ);
    const uint32_t nt = fs.off[bin_n] + fs.hcnt[bin_n];
    const int cols = 1 + a.k_lp;
    if (nt <= (uint32_t)kWave) {
      const uint32_t kt = (uint32_t)lane < nt ? fs.u.list.skey[lane] : 0u;
      const uint32_t v = (uint32_t)lane < nt ? fs.u.list.sidx[lane] : kFinNone;
      uint32_t rank = 0;
      for (uint32_t q0 = 0; q0 < nt; q0 += 8) {       // lanes past the members hold neutral values
#pragma unroll
        for (uint32_t q = q0; q < q0 + 8; ++q) {
          const uint32_t kq = (uint32_t)__builtin_amdgcn_readlane((int)kt, (int)q);
          const uint32_t iq = (uint32_t)__builtin_amdgcn_readlane((int)v, (int)q);
          rank += (uint32_t)((kq > kt) | ((kq == kt) & (iq < v)));
        }
      }
      if ((uint32_t)lane < nt && rank < n_top) {
        a.out_lp_ids[(size_t)b * cols + 1 + rank] = (int)v;
        a.out_lp[(size_t)b * cols + 1 + rank] = (float)((double)value_of(kt) - (double)m - lnZ);
      }
    } else if (nt <= (uint32_t)kFinTopMax) {
      for (uint32_t e = lane; e < nt; e += kWave) {
        const uint32_t kt = fs.u.list.skey[e], v = fs.u.list.sidx[e];
        uint32_t rank = 0;
        for (uint32_t q = 0; q < nt; ++q) {
          const uint32_t kq = fs.u.list.skey[q];
          rank += (kq > kt || (kq == kt && fs.u.list.sidx[q] < v)) ? 1u : 0u;
        }
        if (rank < n_top) {
          a.out_lp_ids[(size_t)b * cols + 1 + rank] = (int)v;
          a.out_lp[(size_t)b * cols + 1 + rank] = (float)((double)value_of(kt) - (double)m - lnZ);
        }
      }
    } else if (lane == 0) {
      fs.code_top = 9;                      // too many ties around the n-th best for this kernel
    }
  }

  // ---- (5) wave 0: top-k, top-p, and the draw if the kept set is small
  auto kept_key = [&](uint32_t k, uint32_t key_cut) {
    return k >= key_cut && k > key_c && (!minp_on || __fsub_rn(value_of(k), m) >= t_minp);
  };
  if (wave == 0 && rp.greedy) {
    if (lane == 0) { fs.token = bidx; fs.token_key = key_of(m); fs.code = 1; }
  } else if (wave == 0) {
    int code = 0;
    uint32_t key_k = 0;
    double lnZ0;
    const unsigned long long S0 = total_mass(lnZ0);
    unsigned long long S1 = S0;
    // Members of a bin: the range [p0, p0 + nm) of the sorted list.  Up to 64 of them sit one per
    // lane and are compared through readlane; more (many equal values: bf16 logits) are stepped
    // through by distinct key, largest first, each step one pass of the wave over the members.
    // next_key(): the largest member key below `below`, how many members have it and their mass.
    auto next_key = [&](uint32_t p0, uint32_t nm, uint32_t below, uint32_t& cnt_eq, unsigned long long& mass_eq) -> uint32_t {
      uint32_t best = 0, n = 0;
      bool any = false;
      for (uint32_t e = lane; e < nm; e += kWave) {
        const uint32_t k = fs.u.list.skey[p0 + e];
        if (k < below && (!any || k > best)) { best = k; n = 0; any = true; }
        n += (any && k == best) ? 1u : 0u;
      }
      const uint32_t top = wave_max_u32(any ? best : 0u);
      const bool mine = any && best == top;
      cnt_eq = wave_add_u32(mine ? n : 0u);
      mass_eq = (unsigned long long)cnt_eq * mass(value_of(top));             // equal keys, equal masses
      return __any(any) ? top : kFinNone;
    };
    if (k_act) {
      const uint32_t p0 = fs.off[bin_k], nm = fs.hcnt[bin_k];
      const uint32_t k_rem = (uint32_t)rp.top_k - p0;                          // 1 <= k_rem <= nm
      unsigned long long part = 0;
      if (nm <= (uint32_t)kWave) {
        const uint32_t kt = (uint32_t)lane < nm ? fs.u.list.skey[p0 + lane] : 0u;
        const unsigned long long Et = (uint32_t)lane < nm ? mass(value_of(kt)) : 0ull;
        uint32_t gt = 0, ge = 0;
        unsigned long long sum_ge = 0;
        for (uint32_t q0 = 0; q0 < nm; q0 += 8) {       // lanes past the members hold neutral values
#pragma unroll
          for (uint32_t q = q0; q < q0 + 8; ++q) {
            const uint32_t kq = (uint32_t)__builtin_amdgcn_readlane((int)kt, (int)q);
            const unsigned long long Eq = readlane_u64(Et, (int)q);
            gt += kq > kt; ge += kq >= kt;
            sum_ge += kq >= kt ? Eq : 0ull;
          }
        }
        const unsigned long long ball = __ballot((uint32_t)lane < nm && gt < k_rem && k_rem <= ge);
        if (ball) {
          const int src = __ffsll((long long)ball) - 1;
          key_k = (uint32_t)__builtin_amdgcn_readlane((int)kt, src);
          part = readlane_u64(sum_ge, src);
        } else {
          code = 8;
        }
      } else {
        uint32_t below = kFinNone, seen = 0;
        int step = 0;
        for (; step < kFinKeySteps; ++step) {
          uint32_t ce;
          unsigned long long me;
          const uint32_t k = next_key(p0, nm, below, ce, me);
          if (k == kFinNone) { code = 8; break; }
          seen += ce; part += me; below = k;
          if (seen >= k_rem) { key_k = k; break; }
        }
        if (step == kFinKeySteps) code = 9;
      }
      S1 = fs.hmass[bin_k] + part;
    }
    uint32_t key_cut = key_k;
    if (code == 0 && rp.top_p < 1.0f) {
      // ---- top-p: the lowest bin whose entries may still be kept (mass of everything above it
      // short of the limit), then the cut inside it
      const double lim = ceil((double)rp.top_p * (double)S1);
      const unsigned long long limit = lim > 0.0 ? (unsigned long long)lim : 0ull;
      // (without top-k, bins below the one that min-p reaches are not in the sorted list, and
      // need not be: their entries fail min-p wherever the nucleus ends)
      const int lowb = k_act ? bin_k : bin_minp;
      int bin_p = 1 << 30, bin_low = 1 << 30;
      {
        constexpr int PER = kFinBins / kWave;                                  // 16 bins per lane, 64 apart: consecutive
#pragma unroll                                                                 // lanes read consecutive words
        for (int j = PER - 1; j >= 0; --j) {                                   // descending: the last hit is the lowest
          const int bin = j * kWave + lane;
          const uint32_t c = fs.hcnt[bin];
          const unsigned long long above = fs.hmass[bin];
          if (bin >= 1 && c) bin_low = bin;
          if (bin >= lowb && c && above < limit) bin_p = bin;
        }
        bin_p = (int)wave_min_u32((uint32_t)bin_p);
        bin_low = (int)wave_min_u32((uint32_t)bin_low);
      }
      if (bin_p >= kFinBins) {
        code = 10;                                                             // p <= 0
      } else {
        const uint32_t p0 = fs.off[bin_p], nm = fs.hcnt[bin_p];
        const unsigned long long base_mass = fs.hmass[bin_p];
        uint32_t key_p = kFinNone;
        bool dropped = false;
        if (nm <= (uint32_t)kWave) {
          const bool member = (uint32_t)lane < nm;
          const uint32_t kt = member ? fs.u.list.skey[p0 + lane] : 0u;
          const unsigned long long Et = member ? mass(value_of(kt)) : 0ull;
          unsigned long long G = base_mass;
          for (uint32_t q0 = 0; q0 < nm; q0 += 8) {       // lanes past the members hold neutral values
#pragma unroll
            for (uint32_t q = q0; q < q0 + 8; ++q) {
              const uint32_t kq = (uint32_t)__builtin_amdgcn_readlane((int)kt, (int)q);
              const unsigned long long Eq = readlane_u64(Et, (int)q);
              G += kq > kt ? Eq : 0ull;
            }
          }
          const bool in_k1 = member && kt >= key_k;
          key_p = wave_min_u32((in_k1 && G < limit) ? kt : kFinNone);
          dropped = __any(in_k1 && !(G < limit));
        } else {
          unsigned long long G = base_mass;
          uint32_t below = kFinNone;
          int step = 0;
          for (; step < kFinKeySteps; ++step) {
            uint32_t ce;
            unsigned long long me;
            const uint32_t k = next_key(p0, nm, below, ce, me);
            if (k == kFinNone || k < key_k) break;                             // no more members of K1
            if (!(G < limit)) { dropped = true; break; }
            key_p = k; G += me; below = k;
          }
          if (step == kFinKeySteps) code = 9;
        }
        // the cut is proven to lie inside the list if some complete entry fell on its far side
        const bool inside = k_act || bin_p > bin_low || dropped;
        if (code == 0 && key_p == kFinNone) code = 10;
        if (code == 0 && !inside && !minp_bounds) {
          code = 11;                                                           // the nucleus may reach below the list
          // Every token below the list weighs at most what the completeness threshold weighs, so
          // the nucleus needs at least (limit - mass of the complete part of the list) / that many
          // more entries: a second list is worth trying if that bound fits one and the list
          // already holds three quarters of the nucleus' mass.  With min-p on the kept set ends
          // at the min-p threshold at the latest, so a list cut there settles the row if it fits.
          const unsigned long long have = fs.hmass[0], e_c = mass(s_c);
          const unsigned long long lack = limit > have ? limit - have : 0ull;
          const bool ok = minp_on || (e_c > 0 && lack / e_c + total < 10000ull && have >= limit - (limit >> 2));
          if (lane == 0) fs.retry_ok = ok ? 1 : 0;
        }
        key_cut = max(key_k, key_p);
      }
    } else if (code == 0 && !k_act && !minp_bounds) {
      code = minp_on ? 12 : 13;                                                // min-p reaches below the list / no filter at all
    }
    if (code == 0) {
      // ---- (6) draw.  The kept set is a range [0, n_hi) of the sorted list minus the entries of
      // its last bins that fail the exact tests.
      int bin_c = key_cut ? bin_of(value_of(key_cut), key_cut) : 1;
      bin_c = max(max(bin_c, 1), minp_on ? bin_minp : 1);
      const uint32_t n_hi = fs.off[bin_c] + fs.hcnt[bin_c];
      if (n_hi <= (uint32_t)kWave) {
        const bool have = (uint32_t)lane < n_hi;
        const uint32_t kt = have ? fs.u.list.skey[lane] : 0u;
        const uint32_t v = have ? fs.u.list.sidx[lane] : kFinNone;
        const unsigned long long Et = (have && kept_key(kt, key_cut)) ? mass(value_of(kt)) : 0ull;
        const unsigned long long S3 = wave_add_u64(Et);
        const unsigned long long target = (__umul64hi(j24, S3) << 40) | ((j24 * S3) >> 24);   // floor(j * S3 / 2^24)
        // The entries are brought into vocabulary order across the lanes: an entry's rank is the
        // number of smaller indices (the indices are distinct), lane `rank` receives its mass and
        // the lane it came from, and a prefix sum over the lanes is the running mass.
        uint32_t rank = 0;
        for (uint32_t q0 = 0; q0 < n_hi; q0 += 8) {                            // lanes past the entries hold an index above all
#pragma unroll
          for (uint32_t q = q0; q < q0 + 8; ++q) rank += (uint32_t)__builtin_amdgcn_readlane((int)v, (int)q) < v;
        }
        if (!have) rank = (uint32_t)lane;                                      // lanes without an entry keep their place
        const int dst = (int)(rank << 2);
        const unsigned long long Es =
            ((unsigned long long)(uint32_t)__builtin_amdgcn_ds_permute(dst, (int)(uint32_t)(Et >> 32)) << 32) |
            (uint32_t)__builtin_amdgcn_ds_permute(dst, (int)(uint32_t)Et);
        const int from = __builtin_amdgcn_ds_permute(dst, lane);
        const unsigned long long C = dpp_scan_add_u64(Es);
        // kept entries have mass > 0: exactly one of them is the first crossing
        const unsigned long long ball = __ballot(Es > 0 && C > target && C - Es <= target);
        if (ball) {
          const int src = __builtin_amdgcn_readlane(from, __ffsll((long long)ball) - 1);
          if (lane == 0) {
            fs.token = (uint32_t)__builtin_amdgcn_readlane((int)v, src);
            fs.token_key = (uint32_t)__builtin_amdgcn_readlane((int)kt, src);
          }
          code = 1;
        } else {
          code = 14;                                                           // no kept mass
        }
      } else {
        if (lane == 0) { fs.key_cut = key_cut; fs.n_hi = n_hi; }
        code = kFinDrawBig;
      }
    }
    if (lane == 0) fs.code = code;
  }
  lds_barrier();
  int code = fs.code_top ? fs.code_top : fs.code;                              // a failure of the best-n ranking stands
  if (hint && code == 11) hint->retry_ok = fs.retry_ok != 0;
  if (code == kFinDrawBig) {
    // ---- (6') kept mass per vocabulary-index bin, prefix, then the crossing inside one bin
    const uint32_t key_cut = fs.key_cut, n_hi = fs.n_hi;
    int ishift = 0;
    while (((V - 1) >> ishift) >= kFinBins) ++ishift;
    for (uint32_t p = tid; p < n_hi; p += NT) {
      const uint32_t k = fs.u.list.skey[p];
      if (kept_key(k, key_cut)) {
        const unsigned long long E = mass(value_of(k));
        if (E) atomicAdd(&fs.hidx[fs.u.list.sidx[p] >> ishift], E);
      }
    }
    lds_barrier();
    unsigned long long target;
    {
      const int b0 = kFinBPT * tid;                      // ascending index order
      const unsigned long long w0 = fs.hidx[b0], w1 = fs.hidx[b0 + 1];
      const unsigned long long msum = w0 + w1;
      const unsigned long long minc = dpp_scan_add_u64(msum);
      if (lane == kWave - 1) fs.r64[wave] = minc;
      lds_barrier();
      unsigned long long ex = minc - msum, S3 = 0;
#pragma unroll
      for (int ww = 0; ww < kFinWaves; ++ww) {
        const unsigned long long m64 = fs.r64[ww];
        if (ww < wave) ex += m64;
        S3 += m64;
      }
      target = (__umul64hi(j24, S3) << 40) | ((j24 * S3) >> 24);               // floor(j * S3 / 2^24)
      if (ex <= target && target < ex + w0) { fs.bin_d = b0; fs.before_d = ex; }
      ex += w0;
      if (ex <= target && target < ex + w1) { fs.bin_d = b0 + 1; fs.before_d = ex; }
    }
    lds_barrier();
    const int bin_d = fs.bin_d;
    if (bin_d < 0) return 14;                                                  // uniform (no kept mass)
    for (uint32_t p = tid; p < n_hi; p += NT) {
      const uint32_t k = fs.u.list.skey[p], v = fs.u.list.sidx[p];
      if ((int)(v >> ishift) == bin_d && kept_key(k, key_cut)) {
        const unsigned long long E = mass(value_of(k));
        if (E) {
          const uint32_t q = atomicAdd(&fs.n_memb, 1u);
          if (q < (uint32_t)kFinMembers) { fs.m_key[q] = k; fs.m_idx[q] = v; fs.m_E[q] = E; }
        }
      }
    }
    lds_barrier();
    const uint32_t nm = fs.n_memb;
    if (nm > (uint32_t)kFinMembers) return 9;                                  // uniform
    if (wave == 0) {
      const unsigned long long before = fs.before_d;
      if (nm <= (uint32_t)kWave) {
        const bool have = (uint32_t)lane < nm;
        const uint32_t v = have ? fs.m_idx[lane] : kFinNone, kt = have ? fs.m_key[lane] : 0u;
        const unsigned long long Et = have ? fs.m_E[lane] : 0ull;
        unsigned long long C = before;
        for (uint32_t q0 = 0; q0 < nm; q0 += 8) {       // lanes past the members hold neutral values
#pragma unroll
          for (uint32_t q = q0; q < q0 + 8; ++q) {
            const uint32_t iq = (uint32_t)__builtin_amdgcn_readlane((int)v, (int)q);
            const unsigned long long Eq = readlane_u64(Et, (int)q);
            C += iq <= v ? Eq : 0ull;
          }
        }
        if (have && C > target && C - Et <= target) { fs.token = v; fs.token_key = kt; }
      } else {
        for (uint32_t e = lane; e < nm; e += kWave) {
          const uint32_t v = fs.m_idx[e];
          unsigned long long C = before;
          for (uint32_t q = 0; q < nm; ++q)
            if (fs.m_idx[q] <= v) C += fs.m_E[q];
          if (C > target && C - fs.m_E[e] <= target) { fs.token = v; fs.token_key = fs.m_key[e]; }
        }
      }
    }
    lds_barrier();
    code = fs.token == kFinNone ? 14 : 1;
  }
  if (code != 1) return code;                                                  // uniform
  if (tid == 0) {
    double lnZ;
    total_mass(lnZ);
    emit(fs.token, fs.token_key, lnZ);
  }
  return 1;
}

__global__ __launch_bounds__(kFinThreads) __attribute__((amdgpu_waves_per_eu(4, 4))) void finish_kernel(Args a_by_value) {
  // The arguments are read where they are used, straight from the kernel-argument segment
  // (the struct is the only parameter, so it starts at offset 0), instead of being held in
  // scalar registers from the first instruction on: there are more of them than registers.
  (void)a_by_value;
  const Args& a = *(const Args*)__builtin_amdgcn_kernarg_segment_ptr();
  warm_kernel_arguments();
  __shared__ FinShared fs;
  const int b = blockIdx.x;
  const int code = finish_row(a, b, fs);
  if (threadIdx.x == 0) {
    a.row_path[b] = code;
    a.row_why[b] = code;
    if (code != 1) {
      const int q = atomicAdd(a.rescue_n, 1);
      if (q >= 0 && q < a.B) a.rescue_rows[q] = b;
    }
  }
}

}  // namespace sip
