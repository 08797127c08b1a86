/*
 * cw_sampler.c -- CPU sampler laid out the way the paper's host sampler is (Sec. 5.1).
 * BASELINE / TEST INFRASTRUCTURE ONLY: built and called by tests/ and by bench.py's CPU leg,
 * never by the HIP library, with which it shares no code.  It is checked against the slow
 * oracle (oracle/sip_oracle.py), which remains the definition of a correct result.
 *
 * What is taken from Sec. 5.1:
 *   - column-wise layout: logits are held as Z^T (V x B, one token's B values contiguous), so
 *     every per-token operation is one contiguous vector over the batch;
 *   - incremental penalty construction: a persistent table f (V x B) of token frequencies that
 *     each iteration updates at the B newly generated tokens only; penalties are then one dense
 *     pass "Z^T -= alpha * f" over the table (here fused with the temperature division);
 *   - the vocabulary pieces of t workers go side by side into Z^T (cw_load_* takes a row
 *     stride and a column offset);
 *   - many workers in parallel, each on its own part of the batch (here: OpenMP threads on
 *     blocks of 16 batch columns, one cache line of Z^T per token).
 * What the paper leaves open (how top-k / top-p / min-p are found, the random numbers, ties,
 * what a logprob is) follows the oracle's readings.  Selection: one pass builds, per column, a
 * 4096-bin histogram (count, mass) over an order-preserving key of the scaled logit; the bins
 * that can hold a cut are known from it; a second pass gathers the tokens of those bins and
 * above; the short list is sorted and the oracle's definitions are applied to it literally.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <omp.h>
#include <sys/mman.h>

#define CW 16            /* batch columns per block = floats per 64-byte line */
#define NBIN 4096
#define HUGE ((size_t)2 << 20)
#define PF 24           /* table rows a worker prefetches ahead (past the end: a hint, never a fault) */

struct hbin { uint32_t cnt; float mass; };   /* tokens of a key bin and (roughly) their mass */

typedef struct {
  int B, Bp, V, threads;
  float* Z;              /* [V][Bp]  Z^T, overwritten by the scaled logits during a step */
  uint16_t* f;           /* [V][Bp]  occurrences of token v in column b's history */
  struct hbin* hist;     /* per thread [CW][NBIN] */
} cw_state;

typedef struct {
  const float* temperature; const int32_t* top_k; const float* top_p; const float* min_p;
  const float* repetition_penalty; const float* frequency_penalty; const float* presence_penalty;
  const int64_t* row_id;
} cw_params;

typedef struct { float s; int32_t v; } cand_t;

/* ---- Philox4x32-10 (Salmon et al., SC'11): counter (row lo, row hi, step lo, step hi), key (seed lo, hi) */
static uint32_t philox_x0(uint64_t seed, uint64_t row, uint64_t step) {
  uint32_t c0 = (uint32_t)row, c1 = (uint32_t)(row >> 32), c2 = (uint32_t)step, c3 = (uint32_t)(step >> 32);
  uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
  for (int r = 0; r < 10; ++r) {
    const uint64_t p0 = (uint64_t)0xD2511F53u * c0, p1 = (uint64_t)0xCD9E8D57u * c2;
    const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0, n1 = (uint32_t)p1;
    const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1, n3 = (uint32_t)p0;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
  }
  return c0;
}

static inline uint32_t key_of(float s) {
  union { float f; uint32_t u; } x;
  x.f = s + 0.0f;
  return x.u ^ ((x.u & 0x80000000u) ? 0xFFFFFFFFu : 0x80000000u);
}
static inline int bin_of(float s) { return (int)(key_of(s) >> 20); }

cw_state* cw_create(int B, int V, int threads) {
  if (B <= 0 || V <= 0) return NULL;
  cw_state* st = (cw_state*)calloc(1, sizeof(cw_state));
  if (!st) return NULL;
  st->B = B; st->V = V; st->Bp = (B + CW - 1) / CW * CW;
  st->threads = threads > 0 ? threads : omp_get_max_threads();
  /* a worker walks its block of columns with a stride of one table row: ask for large pages */
  const size_t zb = ((size_t)V * st->Bp * sizeof(float) + HUGE - 1) / HUGE * HUGE;
  const size_t fb = ((size_t)V * st->Bp * sizeof(uint16_t) + HUGE - 1) / HUGE * HUGE;
  st->Z = (float*)aligned_alloc(HUGE, zb);
  st->f = (uint16_t*)aligned_alloc(HUGE, fb);
  if (st->Z) madvise(st->Z, zb, MADV_HUGEPAGE);
  if (st->f) madvise(st->f, fb, MADV_HUGEPAGE);
  st->hist = (struct hbin*)malloc((size_t)st->threads * CW * NBIN * sizeof(struct hbin));
  if (!st->Z || !st->f || !st->hist) return NULL;
  memset(st->Z, 0, (size_t)V * st->Bp * sizeof(float));
  memset(st->f, 0, (size_t)V * st->Bp * sizeof(uint16_t));
  return st;
}

void cw_destroy(cw_state* st) {
  if (!st) return;
  free(st->Z); free(st->f); free(st->hist); free(st);
}

int cw_threads(const cw_state* st) { return st->threads; }

/* Incremental penalty construction: one new token per column (ids outside [0, V) are skipped). */
void cw_push_tokens(cw_state* st, const int32_t* tokens) {
  for (int b = 0; b < st->B; ++b) {
    const int32_t t = tokens[b];
    if (t >= 0 && t < st->V) {
      uint16_t* p = &st->f[(size_t)t * st->Bp + b];
      if (*p != 0xFFFFu) ++*p;
    }
  }
}

/* Sequence turnover: column b starts over with the given history. */
void cw_set_history(cw_state* st, int b, const int32_t* toks, int64_t n) {
  for (int v = 0; v < st->V; ++v) st->f[(size_t)v * st->Bp + b] = 0;
  for (int64_t i = 0; i < n; ++i) {
    const int32_t t = toks[i];
    if (t >= 0 && t < st->V) {
      uint16_t* p = &st->f[(size_t)t * st->Bp + b];
      if (*p != 0xFFFFu) ++*p;
    }
  }
}

/* A piece of the logits, row-major [B][row_stride] as a worker emits it, goes into Z^T at
   vocabulary offset v0 (transposed in 16 x 16 tiles). */
void cw_load_f32(cw_state* st, const float* src, int64_t row_stride, int v0, int nv) {
  const int Bp = st->Bp, B = st->B;
#pragma omp parallel for num_threads(st->threads) schedule(static)
  for (int vt = 0; vt < nv; vt += 16) {
    const int vn = nv - vt < 16 ? nv - vt : 16;
    for (int bt = 0; bt < B; bt += 16) {
      const int bn = B - bt < 16 ? B - bt : 16;
      for (int i = 0; i < vn; ++i) {
        float* d = st->Z + (size_t)(v0 + vt + i) * Bp + bt;
        for (int j = 0; j < bn; ++j) d[j] = src[(size_t)(bt + j) * row_stride + vt + i];
      }
    }
  }
}
void cw_load_bf16(cw_state* st, const uint16_t* src, int64_t row_stride, int v0, int nv) {
  const int Bp = st->Bp, B = st->B;
#pragma omp parallel for num_threads(st->threads) schedule(static)
  for (int vt = 0; vt < nv; vt += 16) {
    const int vn = nv - vt < 16 ? nv - vt : 16;
    for (int bt = 0; bt < B; bt += 16) {
      const int bn = B - bt < 16 ? B - bt : 16;
      for (int i = 0; i < vn; ++i) {
        float* d = st->Z + (size_t)(v0 + vt + i) * Bp + bt;
        for (int j = 0; j < bn; ++j) {
          union { uint32_t u; float f; } x;
          x.u = (uint32_t)src[(size_t)(bt + j) * row_stride + vt + i] << 16;
          d[j] = x.f;
        }
      }
    }
  }
}

/* e = exp(z - m) and the key bin of z for one block row.  Relaxed floating-point rules in this
   function only, so that it becomes vector code: 2^t with t = (z - m) * log2(e) split into its
   nearest integer and a remainder in [-1/2, 1/2], a degree-6 polynomial for the latter (relative
   error 2e-7).  These values feed the total mass and the histogram, never a decision. */
__attribute__((optimize("fast-math"))) static void exp_block(const float* z, const float* m, float* e, uint32_t* bin) {
#pragma omp simd
  for (int c = 0; c < CW; ++c) {
    float t = (z[c] - m[c]) * 1.44269504f;
    t = t < -126.0f ? -126.0f : t;
    const float n = __builtin_roundf(t), f = t - n;
    const float p = 1.0f + f * (0.693147181f + f * (0.240226507f + f * (0.0555041087f + f * (0.00961812911f +
                    f * (0.00133335581f + f * 0.000154035304f)))));
    union { int32_t i; float f; } sc;
    sc.i = ((int32_t)n + 127) << 23;
    e[c] = (z[c] - m[c]) < -87.0f ? 0.0f : p * sc.f;
    union { float f; uint32_t u; } x;
    x.f = z[c] + 0.0f;
    bin[c] = (x.u ^ ((x.u & 0x80000000u) ? 0xFFFFFFFFu : 0x80000000u)) >> 20;
  }
}

static int cmp_desc(const void* a, const void* b) {
  const cand_t* x = (const cand_t*)a; const cand_t* y = (const cand_t*)b;
  if (x->s > y->s) return -1;
  if (x->s < y->s) return 1;
  return x->v < y->v ? -1 : (x->v > y->v ? 1 : 0);
}

/* One column, from the tokens of its upper bins (`g`, in ascending vocabulary order; every token
   of the column with a larger scaled logit than any token outside g is in g). */
static void finish_column(const cand_t* g, int ng, float m, double Zsum, float tau, int k, float p, float minp,
                          int greedy, int V, double u, int n_lp, int arg_max,
                          int32_t* out_id, int32_t* lp_ids, float* lp) {
  const double logZ = log(Zsum);
  cand_t* srt = (cand_t*)malloc((size_t)(ng > 0 ? ng : 1) * sizeof(cand_t));
  memcpy(srt, g, (size_t)ng * sizeof(cand_t));
  qsort(srt, (size_t)ng, sizeof(cand_t), cmp_desc);
  int token = arg_max;
  if (!greedy) {
    double* e = (double*)malloc((size_t)(ng > 0 ? ng : 1) * sizeof(double));
    for (int i = 0; i < ng; ++i) e[i] = exp((double)srt[i].s - (double)m);
    /* top-k: everything not smaller than the k-th largest value */
    int n1 = ng;
    double S1 = Zsum;
    if (k >= 2 && k < V) {
      const float tk = srt[k - 1 < ng ? k - 1 : ng - 1].s;
      n1 = 0;
      while (n1 < ng && srt[n1].s >= tk) ++n1;
      S1 = 0.0;
      for (int i = 0; i < n1; ++i) S1 += e[i];
    }
    /* top-p: keep v iff the mass of strictly larger kept tokens is below p * S1 */
    int n2 = n1;
    if (p > 0.0f && p < 1.0f) {
      const double target = (double)p * S1;
      double cum = 0.0, mass_gt = 0.0;
      n2 = 0;
      for (int i = 0; i < n1; ++i) {
        if (i == 0 || srt[i].s != srt[i - 1].s) mass_gt = cum;    /* first of its value group */
        if (!(mass_gt < target)) break;
        cum += e[i];
        n2 = i + 1;
      }
    }
    /* min-p: fp32 (s - m) >= fp32(ln min_p); the kept tokens are a prefix of the order as well */
    int n3 = n2;
    if (minp > 0.0f) {
      const float t = (float)log((double)minp);
      n3 = 0;
      while (n3 < n2 && (float)(srt[n3].s - m) >= t) ++n3;
    }
    /* draw over the kept set in ascending vocabulary order: g is in that order already */
    const float s_last = n3 > 0 ? srt[n3 - 1].s : m;
    double S3 = 0.0;                                                  /* summed in index order, like the CDF below */
    for (int i = 0; i < ng; ++i)
      if (g[i].s >= s_last) S3 += exp((double)g[i].s - (double)m);
    const double target = u * S3;
    double cdf = 0.0;
    int last = arg_max;
    token = -1;
    for (int i = 0; i < ng; ++i) {
      if (!(g[i].s >= s_last)) continue;
      cdf += exp((double)g[i].s - (double)m);
      last = g[i].v;
      if (cdf > target) { token = g[i].v; break; }
    }
    if (token < 0) token = last;
    free(e);
  }
  *out_id = token;
  if (lp_ids) {
    float s_tok = m;
    for (int i = 0; i < ng; ++i) if (g[i].v == token) { s_tok = g[i].s; break; }
    lp_ids[0] = token;
    lp[0] = (float)(((double)s_tok - (double)m) - logZ);
    for (int j = 0; j < n_lp; ++j) {
      if (j < ng) { lp_ids[1 + j] = srt[j].v; lp[1 + j] = (float)(((double)srt[j].s - (double)m) - logZ); }
      else { lp_ids[1 + j] = -1; lp[1 + j] = -INFINITY; }
    }
  }
  free(srt);
}

/*
 * One sampling step over the logits loaded into Z^T and the frequency table as it stands.
 * out_lp_ids / out_lp: [B][1 + n_lp] or NULL.  Returns 0.
 */
int cw_sample(cw_state* st, const cw_params* P, uint64_t seed, uint64_t step, int n_lp,
              int32_t* out_ids, int32_t* out_lp_ids, float* out_lp) {
  const int V = st->V, B = st->B, Bp = st->Bp;
  const int nblk = Bp / CW;
#pragma omp parallel for num_threads(st->threads) schedule(dynamic, 1)
  for (int blk = 0; blk < nblk; ++blk) {
    const int tid = omp_get_thread_num();
    struct hbin* hb = st->hist + (size_t)tid * CW * NBIN;
    const int b0 = blk * CW;
    float tau[CW], theta[CW], phi[CW], psi[CW], pp[CW], mp[CW], m[CW];
    int kk[CW], greedy[CW], arg[CW], live[CW];
    for (int c = 0; c < CW; ++c) {
      const int b = b0 + c;
      live[c] = b < B;
      const int bb = live[c] ? b : 0;
      tau[c] = P->temperature ? P->temperature[bb] : 1.0f;
      kk[c] = P->top_k ? P->top_k[bb] : 0;
      pp[c] = P->top_p ? P->top_p[bb] : 1.0f;
      mp[c] = P->min_p ? P->min_p[bb] : 0.0f;
      theta[c] = P->repetition_penalty ? P->repetition_penalty[bb] : 1.0f;
      phi[c] = P->frequency_penalty ? P->frequency_penalty[bb] : 0.0f;
      psi[c] = P->presence_penalty ? P->presence_penalty[bb] : 0.0f;
      greedy[c] = (tau[c] == 0.0f) || (kk[c] == 1);
      m[c] = -INFINITY; arg[c] = 0;
    }
    /* pass A: penalties from f (dense), temperature, running maximum -- all vectors over the block.
       Written without branches: a feature that is off has the neutral parameter (theta = 1,
       phi = psi = 0, and 1 for the temperature of a greedy row), which leaves the value bit for bit. */
    float tdiv[CW];
    for (int c = 0; c < CW; ++c) tdiv[c] = greedy[c] ? 1.0f : tau[c];
    for (int v = 0; v < V; ++v) {
      float* z = st->Z + (size_t)v * Bp + b0;
      const uint16_t* f = st->f + (size_t)v * Bp + b0;
      /* the block's lines are a table row apart: too far for the hardware prefetcher */
      __builtin_prefetch(z + (size_t)PF * Bp, 1);
      __builtin_prefetch(f + (size_t)PF * Bp, 0);
#pragma omp simd
      for (int c = 0; c < CW; ++c) {
        const float x = z[c];
        const float cnt = (float)f[c];
        float y = x > 0.0f ? x / theta[c] : x * theta[c];
        y = y - phi[c] * cnt;
        y = y - psi[c];
        const float s = (f[c] ? y : x) / tdiv[c];
        z[c] = s;
        m[c] = s > m[c] ? s : m[c];
      }
    }
    /* pass B: total mass, the (count, mass) histogram over 12-bit keys, lowest index of the maximum */
    memset(hb, 0, (size_t)CW * NBIN * sizeof(struct hbin));
    double Zs[CW];
    for (int c = 0; c < CW; ++c) { Zs[c] = 0.0; arg[c] = -1; }
    for (int v = 0; v < V; ++v) {
      const float* z = st->Z + (size_t)v * Bp + b0;
      float e[CW];
      uint32_t bin[CW];
      __builtin_prefetch(z + (size_t)PF * Bp, 0);
      exp_block(z, m, e, bin);
      for (int c = 0; c < CW; ++c) {
        struct hbin* h = &hb[c * NBIN + bin[c]];
        Zs[c] += (double)e[c];
        h->cnt += 1u;
        h->mass += e[c];
        if (z[c] == m[c] && arg[c] < 0) arg[c] = v;
      }
    }
    for (int c = 0; c < CW; ++c) if (arg[c] < 0) arg[c] = 0;
    /* lowest bin each column has to gather */
    int low[CW], plain[CW];
    size_t off[CW + 1];
    off[0] = 0;
    for (int c = 0; c < CW; ++c) {
      const int k = kk[c];
      const int k_on = !greedy[c] && k >= 2 && k < V, p_on = !greedy[c] && pp[c] > 0.0f && pp[c] < 1.0f;
      const int m_on = !greedy[c] && mp[c] > 0.0f;
      plain[c] = !greedy[c] && !k_on && !p_on && !m_on;
      int lo = NBIN - 1;
      uint32_t want = (uint32_t)(n_lp > 0 ? n_lp : 1);
      if (k_on && (uint32_t)k > want) want = (uint32_t)k;
      if (plain[c]) {
        lo = 0;                                         /* no filter: the draw runs over the whole column */
      } else {
        uint32_t cnt = 0;
        int bq = NBIN - 1;
        for (; bq > 0; --bq) { cnt += hb[c * NBIN + bq].cnt; if (cnt >= want) break; }
        lo = bq;
        if (!k_on && p_on) {
          /* the bin masses are fp32 sums: good to a part in a thousand, and one bin more is taken anyway */
          const double limit = (double)pp[c] * Zs[c] * (1.0 + 2e-3);
          double cum = 0.0;
          int bp = NBIN - 1;
          for (; bp > 0; --bp) { cum += (double)hb[c * NBIN + bp].mass; if (cum >= limit) break; }
          bp = bp > 0 ? bp - 1 : 0;
          int bound = bp;
          if (m_on) {                                  /* the kept set also ends at the min-p threshold */
            int bm = bin_of(m[c] + (float)log((double)mp[c])) - 1;
            if (bm < 0) bm = 0;
            if (bm > bound) bound = bm;
          }
          if (bound < lo) lo = bound;
        } else if (!k_on && m_on) {
          int bm = bin_of(m[c] + (float)log((double)mp[c])) - 1;
          if (bm < 0) bm = 0;
          if (bm < lo) lo = bm;
        }
      }
      if (!live[c]) lo = NBIN;                          /* padding column: gather nothing */
      low[c] = lo;
      size_t n = 0;
      for (int bq = lo; bq < NBIN; ++bq) n += hb[c * NBIN + bq].cnt;
      off[c + 1] = off[c] + n;
    }
    /* pass C: gather the tokens of those bins, ascending vocabulary order per column */
    cand_t* pool = (cand_t*)malloc((off[CW] > 0 ? off[CW] : 1) * sizeof(cand_t));
    size_t fill[CW];
    for (int c = 0; c < CW; ++c) fill[c] = off[c];
    float thr[CW];                                       /* smallest value of bin low[c] */
    for (int c = 0; c < CW; ++c) {
      union { uint32_t u; float f; } x;
      const uint32_t key = (uint32_t)low[c] << 20;
      x.u = (key & 0x80000000u) ? (key ^ 0x80000000u) : ~key;
      thr[c] = low[c] <= 0 ? -INFINITY : (low[c] >= NBIN ? INFINITY : x.f);
    }
    for (int v = 0; v < V; ++v) {
      const float* z = st->Z + (size_t)v * Bp + b0;
      int any = 0;
      __builtin_prefetch(z + (size_t)PF * Bp, 0);
#pragma omp simd reduction(| : any)
      for (int c = 0; c < CW; ++c) any |= z[c] >= thr[c];
      if (!any) continue;
      for (int c = 0; c < CW; ++c)
        if (z[c] >= thr[c] && fill[c] < off[c + 1]) { pool[fill[c]].s = z[c]; pool[fill[c]].v = v; ++fill[c]; }
    }
    for (int c = 0; c < CW; ++c) {
      if (!live[c]) continue;
      const int b = b0 + c;
      const uint64_t row = P->row_id ? (uint64_t)P->row_id[b] : (uint64_t)b;
      const double u = (double)(philox_x0(seed, row, step) >> 8) * (1.0 / 16777216.0);
      finish_column(pool + off[c], (int)(off[c + 1] - off[c]), m[c], Zs[c], tau[c], kk[c], pp[c], mp[c], greedy[c], V, u,
                    n_lp, arg[c], &out_ids[b], out_lp_ids ? out_lp_ids + (size_t)b * (1 + n_lp) : NULL,
                    out_lp ? out_lp + (size_t)b * (1 + n_lp) : NULL);
    }
    free(pool);
  }
  return 0;
}
