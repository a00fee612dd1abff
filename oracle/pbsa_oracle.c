/*
 * CPU oracle for the PBSA decode path of "Sparse Forcing" -- TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, obviously-correct loops written from the paper.  Nothing in the product path may
 * call this file; it shares no code with the HIP kernels.  Only tests, the smoke check and the
 * cpu_baseline leg of the benchmark use it.
 *
 * Precision.  Everything that decides an integer (pooled representatives, coarse logits, the
 * persistence scores) is computed in IEEE fp32 in a fixed operation order, because the block
 * sets and slot assignments it produces are compared bit-for-bit with the GPU:
 *   pool      acc = acc + x[t] over valid tokens t ascending from 0.0f, then acc / (float)len
 *   dot       acc = fmaf(q[x], k[x], acc) over x ascending from 0.0f, then acc * scale
 *   softmax   m = exact max; e = pexp(z - m); sum = sum + e over j ascending; a = e / sum
 *   col mean  acc = acc + a[i][j] over i ascending, then acc / (float)nqb
 *   fold      S_sum = S_sum + x over losing blocks in candidate order
 * (compile with -ffp-contract=off, no fast-math).  The fine attention itself, whose output is
 * only compared within a tolerance, is computed in fp64.
 *
 * Layouts (all host pointers, all dense):
 *   Q            [H][Nq][d]              bf16 bits, token-major; query block i = tokens iB..iB+len_i-1
 *   Kl, Vl       [H][n_loc_cap][B][d]    bf16 bits, physical local slots (ring)
 *   l_map        [n_loc]                 logical local block (oldest first, chunk last) -> physical slot
 *   l_len, l_id  [n_loc]                 valid tokens / global id of each logical local block
 *   Kc_l         [H][n_loc_cap][d]       fp32 pooled keys by physical slot
 *   Kp, Vp       [H][C+1][B][d]          bf16 bits, persistent slots; slot C is the summary block
 *   p_len        [H][C+1]                valid tokens per slot, 0 = empty
 *   Kc_p, p_id   [H][C][d] fp32, [H][C] int64
 *   S_sum, S_cnt [H][2][B][d] fp32 (K then V), [H][B] int32
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct orc_cfg {
  int32_t H, d, B;        /* heads, head dim, tokens per block                                  */
  int32_t Nq, nqb;        /* chunk tokens, ceil(Nq/B)                                           */
  int32_t n_loc;          /* logical local blocks incl. the chunk's nqb (chunk = last nqb)      */
  int32_t n_loc_cap;      /* physical local slots per head                                      */
  int32_t C, n_sink;      /* persistent slots (summary = slot C), pinned leading slots          */
  int32_t k;              /* local blocks selected per query block                              */
  int32_t causal;         /* 1: query block i sees local blocks 0..n_loc-nqb+i ; 0: all         */
  int32_t n_evict;        /* leading local blocks leaving the window at this update             */
  int32_t pool_from;      /* pooled keys of logical blocks >= pool_from are recomputed          */
  float scale;            /* 1/sqrt(d)                                                          */
} orc_cfg;

#ifdef _OPENMP
#include <omp.h>
int orc_num_threads(void) { return omp_get_max_threads(); }
#else
int orc_num_threads(void) { return 1; }
#endif

static inline float bf2f(uint16_t b) {
  uint32_t u = (uint32_t)b << 16;
  float f;
  memcpy(&f, &u, 4);
  return f;
}

static inline uint16_t f2bf(float f) { /* round to nearest even; inputs are finite */
  uint32_t u;
  memcpy(&u, &f, 4);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

/* exp(x) for x <= 0 as the interface's arithmetic contract words it (fp32 multiply, fused multiply-add and
 * round-to-nearest-integer only, so that any implementation of the same steps gives the same bits):
 * 0 below -64; otherwise n = the integer nearest to x * log2(e); the remainder r = x - n ln 2 with ln 2 split into
 * 0.693359375 (so that n times it is exact) and the correction -2.12194440e-4; e^r by the Taylor polynomial of
 * degree 6, coefficients rounded to fp32, evaluated by Horner's rule from the highest term; scaled by 2^n. */
float orc_pexp(float x) {
  static const float taylor[7] = {(float)(1.0 / 720.0), (float)(1.0 / 120.0), (float)(1.0 / 24.0), (float)(1.0 / 6.0),
                                  0.5f, 1.0f, 1.0f};
  const float log2e = (float)1.4426950408889634, ln2_head = 0.693359375f, ln2_tail = -2.12194440e-4f;
  if (x < -64.0f) return 0.0f;
  const float n = nearbyintf(x * log2e);
  const float r = fmaf(n, -ln2_tail, fmaf(n, -ln2_head, x));
  float poly = taylor[0];
  for (int i = 1; i < 7; ++i) poly = fmaf(poly, r, taylor[i]);
  return ldexpf(poly, (int)n);          /* poly is in [0.5, 1.5] and n >= -93: the scaling is exact */
}

/* Block representative by average pooling (Eq. 6 with the pooling operator of Sec. 4.1):
 * mean over the block's valid tokens, per dimension.  rows: [len][d] bf16 with row pitch d. */
void orc_pool_block(const uint16_t* rows, int len, int d, float* out) {
  for (int x = 0; x < d; ++x) {
    float acc = 0.0f;
    for (int t = 0; t < len; ++t) acc = acc + bf2f(rows[(size_t)t * d + x]);
    out[x] = len > 0 ? acc / (float)len : 0.0f;
  }
}

static inline int q_block_len(const orc_cfg* c, int i) {
  int rem = c->Nq - i * c->B;
  return rem < c->B ? rem : c->B;
}

static inline int n_visible(const orc_cfg* c, int i) {
  return c->causal ? c->n_loc - c->nqb + i + 1 : c->n_loc;
}

static inline float dot_scaled(const float* q, const float* k, int d, float scale) {
  float acc = 0.0f;
  for (int x = 0; x < d; ++x) acc = fmaf(q[x], k[x], acc);
  return acc * scale;
}

/* Coarse routing inside the local region (Eq. 10-11): pooled representatives, scaled block
 * logits, row-wise top-k with ties going to the lowest block index.  Softmax is monotone per
 * row, so the top-k of the logits is the top-k of Eq. 10's probabilities.
 * Z (optional, [H][nqb][n_loc]) receives the logits; entries not visible are set to -INFINITY.
 * sel [H][nqb][k]: selected logical local blocks in ascending order, padded with -1. */
int orc_select(const orc_cfg* c, const uint16_t* Q, const uint16_t* Kl, const int32_t* l_len,
               const int32_t* l_map, float* Kc_l, float* Qc, int32_t* sel, float* Z) {
  const int d = c->d, B = c->B;
  float* z = (float*)malloc(sizeof(float) * (size_t)(c->n_loc > 0 ? c->n_loc : 1));
  char* taken = (char*)malloc((size_t)(c->n_loc > 0 ? c->n_loc : 1));
  if (!z || !taken) return -1;
  for (int h = 0; h < c->H; ++h) {
    for (int l = c->pool_from; l < c->n_loc; ++l) {
      size_t slot = (size_t)h * c->n_loc_cap + l_map[l];
      orc_pool_block(Kl + slot * B * d, l_len[l], d, Kc_l + slot * d);
    }
    for (int i = 0; i < c->nqb; ++i) {
      float* qc = Qc + ((size_t)h * c->nqb + i) * d;
      orc_pool_block(Q + ((size_t)h * c->Nq + (size_t)i * B) * d, q_block_len(c, i), d, qc);
      const int nvis = n_visible(c, i);
      for (int l = 0; l < c->n_loc; ++l) {
        const float* kc = Kc_l + ((size_t)h * c->n_loc_cap + l_map[l]) * d;
        z[l] = l < nvis ? dot_scaled(qc, kc, d, c->scale) : -INFINITY;
        if (Z) Z[((size_t)h * c->nqb + i) * c->n_loc + l] = z[l];
      }
      memset(taken, 0, (size_t)c->n_loc);
      const int kk = c->k < nvis ? c->k : nvis;
      for (int r = 0; r < kk; ++r) {
        int best = -1;
        for (int l = 0; l < nvis; ++l)
          if (!taken[l] && (best < 0 || z[l] > z[best])) best = l; /* strict >: lowest index wins ties */
        taken[best] = 1;
      }
      int32_t* out = sel + ((size_t)h * c->nqb + i) * c->k;
      int n = 0;
      for (int l = 0; l < nvis; ++l)
        if (taken[l]) out[n++] = l;
      for (; n < c->k; ++n) out[n] = -1;
    }
  }
  free(z);
  free(taken);
  return 0;
}

/* PBSA fine stage (Eq. 3-5) for a list of query rows: one softmax over every valid token of the
 * occupied persistent slots (0..C, the summary slot included) and every valid token of the local
 * blocks in the row's block set; everything else is masked out.  fp64 throughout.
 * rows_h/rows_t [n_rows]: head and chunk-token index of each requested row.
 * O [n_rows][d] fp64; lse [n_rows] fp64 (natural log of the softmax normaliser), may be NULL.
 * A row that sees no key at all gets O = 0 and lse = -INFINITY. */
int orc_attention_rows(const orc_cfg* c, const uint16_t* Q, const uint16_t* Kp, const uint16_t* Vp,
                       const int32_t* p_len, const uint16_t* Kl, const uint16_t* Vl,
                       const int32_t* l_len, const int32_t* l_map, const int32_t* sel, int64_t n_rows,
                       const int32_t* rows_h, const int32_t* rows_t, double* O, double* lse) {
  const int d = c->d, B = c->B;
  const size_t max_keys = (size_t)(c->C + 1 + c->k) * B + 1;
  int fail = 0;
#pragma omp parallel
  {
    double* z = (double*)malloc(sizeof(double) * max_keys);
    const uint16_t** vrow = (const uint16_t**)malloc(sizeof(void*) * max_keys);
    double* q = (double*)malloc(sizeof(double) * (size_t)d);
    if (!z || !vrow || !q) {
#pragma omp atomic write
      fail = 1;
    } else {
#pragma omp for schedule(dynamic, 16)
      for (int64_t r = 0; r < n_rows; ++r) {
        const int h = rows_h[r], t = rows_t[r], i = t / B;
        const uint16_t* qrow = Q + ((size_t)h * c->Nq + t) * d;
        for (int x = 0; x < d; ++x) q[x] = (double)bf2f(qrow[x]);
        size_t n = 0;
        for (int s = 0; s <= c->C; ++s) {
          const int len = p_len[(size_t)h * (c->C + 1) + s];
          const size_t base = ((size_t)h * (c->C + 1) + s) * B * d;
          for (int u = 0; u < len; ++u) {
            const uint16_t* krow = Kp + base + (size_t)u * d;
            double acc = 0.0;
            for (int x = 0; x < d; ++x) acc += q[x] * (double)bf2f(krow[x]);
            z[n] = acc * (double)c->scale;
            vrow[n++] = Vp + base + (size_t)u * d;
          }
        }
        const int32_t* row_sel = sel + ((size_t)h * c->nqb + i) * c->k;
        for (int j = 0; j < c->k; ++j) {
          const int l = row_sel[j];
          if (l < 0) continue;
          const size_t base = ((size_t)h * c->n_loc_cap + l_map[l]) * B * d;
          for (int u = 0; u < l_len[l]; ++u) {
            const uint16_t* krow = Kl + base + (size_t)u * d;
            double acc = 0.0;
            for (int x = 0; x < d; ++x) acc += q[x] * (double)bf2f(krow[x]);
            z[n] = acc * (double)c->scale;
            vrow[n++] = Vl + base + (size_t)u * d;
          }
        }
        double* o = O + (size_t)r * d;
        for (int x = 0; x < d; ++x) o[x] = 0.0;
        if (n == 0) {
          if (lse) lse[r] = -INFINITY;
          continue;
        }
        double m = z[0];
        for (size_t j = 1; j < n; ++j) m = z[j] > m ? z[j] : m;
        double sum = 0.0;
        for (size_t j = 0; j < n; ++j) {
          z[j] = exp(z[j] - m);
          sum += z[j];
        }
        for (size_t j = 0; j < n; ++j) {
          const double p = z[j] / sum;
          const uint16_t* v = vrow[j];
          for (int x = 0; x < d; ++x) o[x] += p * (double)bf2f(v[x]);
        }
        if (lse) lse[r] = m + log(sum);
      }
    }
    free(z);
    free(vrow);
    free(q);
  }
  return fail ? -1 : 0;
}

/* Coarse scoring for persistence (Eq. 7-8): block-level softmax of every query block over
 * U = occupied persistent slots 0..C-1 (slot order) followed by all n_loc local blocks (no
 * causal or top-k mask), then the mean over query blocks.
 * s_p [H][C] (0 for empty slots), s_l [H][n_loc]. */
int orc_scores(const orc_cfg* c, const float* Qc, const float* Kc_l, const int32_t* l_map,
               const float* Kc_p, const int32_t* p_len, float* s_p, float* s_l) {
  const int d = c->d, nU_max = c->C + c->n_loc;
  const float** kc = (const float**)malloc(sizeof(void*) * (size_t)(nU_max > 0 ? nU_max : 1));
  float* e = (float*)malloc(sizeof(float) * (size_t)(nU_max > 0 ? nU_max : 1));
  float* col = (float*)malloc(sizeof(float) * (size_t)(nU_max > 0 ? nU_max : 1));
  if (!kc || !e || !col) return -1;
  for (int h = 0; h < c->H; ++h) {
    int nU = 0;
    for (int s = 0; s < c->C; ++s)
      if (p_len[(size_t)h * (c->C + 1) + s] > 0) kc[nU++] = Kc_p + ((size_t)h * c->C + s) * d;
    for (int l = 0; l < c->n_loc; ++l) kc[nU++] = Kc_l + ((size_t)h * c->n_loc_cap + l_map[l]) * d;
    for (int j = 0; j < nU; ++j) col[j] = 0.0f;
    for (int i = 0; i < c->nqb; ++i) {
      const float* qc = Qc + ((size_t)h * c->nqb + i) * d;
      float m = -INFINITY;
      for (int j = 0; j < nU; ++j) {
        e[j] = dot_scaled(qc, kc[j], d, c->scale);
        m = e[j] > m ? e[j] : m;
      }
      float sum = 0.0f;
      for (int j = 0; j < nU; ++j) {
        e[j] = orc_pexp(e[j] - m);
        sum = sum + e[j];
      }
      for (int j = 0; j < nU; ++j) col[j] = col[j] + e[j] / sum;
    }
    int j = 0;
    for (int s = 0; s < c->C; ++s)
      s_p[(size_t)h * c->C + s] = p_len[(size_t)h * (c->C + 1) + s] > 0 ? col[j++] / (float)c->nqb : 0.0f;
    for (int l = 0; l < c->n_loc; ++l) s_l[(size_t)h * c->n_loc + l] = col[j++] / (float)c->nqb;
  }
  free(kc);
  free(e);
  free(col);
  return 0;
}

/* Retention, slot assignment and fold, given the scores (Eq. 9 and its footnote, plus the
 * compressed-history block):
 *  - candidates = occupants of slots n_sink..C-1 (slot order) then the n_evict leading local
 *    blocks (block order); the top C-n_sink by (score desc, candidate index asc) are kept;
 *  - a kept occupant stays in its slot; kept newcomers, in ascending block order, fill the vacated
 *    and empty slots in ascending slot order (K, V, pooled key, len and id move with the block);
 *  - every dropped candidate is folded, position by position, into the running mean kept as
 *    S_sum / S_cnt, whose bf16 view becomes slot C (skipped when S_sum is NULL).
 * s_p [H][C]: score of each slot (ignored for empty ones); s_l [H][n_loc]: of each local block
 * (only the first n_evict are read).
 * scores [H][C+n_evict] (optional): score of slot 0..C-1 (0 if empty) then of each evicted block.
 * slot_src [H][C]: -1 = slot unchanged, e >= 0 = filled from local block e. */
static int retain_and_fold(const orc_cfg* c, const float* s_p, const float* s_l, const float* Kc_l, uint16_t* Kp,
                           uint16_t* Vp, float* Kc_p, int32_t* p_len, int64_t* p_id, float* S_sum, int32_t* S_cnt,
                           const uint16_t* Kl, const uint16_t* Vl, const int32_t* l_len, const int32_t* l_map,
                           const int64_t* l_id, float* scores, int32_t* slot_src) {
  const int d = c->d, B = c->B, C = c->C, C1 = c->C + 1;
  const size_t blk = (size_t)B * d;
  const int ncand_max = C + c->n_evict;
  int* cand = (int*)malloc(sizeof(int) * (size_t)(ncand_max + 1));   /* <C: slot, else C+e */
  float* cs = (float*)malloc(sizeof(float) * (size_t)(ncand_max + 1));
  char* win = (char*)malloc((size_t)(ncand_max + 1));
  if (!cand || !cs || !win) return -1;
  for (int h = 0; h < c->H; ++h) {
    int32_t* plen = p_len + (size_t)h * C1;
    if (scores) {
      for (int s = 0; s < C; ++s) scores[(size_t)h * ncand_max + s] = s_p[(size_t)h * C + s];
      for (int e = 0; e < c->n_evict; ++e) scores[(size_t)h * ncand_max + C + e] = s_l[(size_t)h * c->n_loc + e];
    }
    int nc = 0;
    for (int s = c->n_sink; s < C; ++s)
      if (plen[s] > 0) { cand[nc] = s; cs[nc++] = s_p[(size_t)h * C + s]; }
    for (int e = 0; e < c->n_evict; ++e) { cand[nc] = C + e; cs[nc++] = s_l[(size_t)h * c->n_loc + e]; }
    const int places = C - c->n_sink;
    for (int a = 0; a < nc; ++a) {
      int rank = 0;
      for (int b = 0; b < nc; ++b)
        if (cs[b] > cs[a] || (cs[b] == cs[a] && b < a)) ++rank;
      win[a] = rank < places;
    }
    /* fold the losers first: their data is read before any slot is overwritten */
    if (S_sum) {
      float* ssum = S_sum + (size_t)h * 2 * blk;
      int32_t* scnt = S_cnt + (size_t)h * B;
      int any = 0;
      for (int a = 0; a < nc; ++a) {
        if (win[a]) continue;
        any = 1;
        const uint16_t *kb, *vb;
        int len;
        if (cand[a] < C) {
          kb = Kp + ((size_t)h * C1 + cand[a]) * blk;
          vb = Vp + ((size_t)h * C1 + cand[a]) * blk;
          len = plen[cand[a]];
        } else {
          const int e = cand[a] - C;
          kb = Kl + ((size_t)h * c->n_loc_cap + l_map[e]) * blk;
          vb = Vl + ((size_t)h * c->n_loc_cap + l_map[e]) * blk;
          len = l_len[e];
        }
        for (int t = 0; t < len; ++t) {
          for (int x = 0; x < d; ++x) {
            ssum[(size_t)t * d + x] = ssum[(size_t)t * d + x] + bf2f(kb[(size_t)t * d + x]);
            ssum[blk + (size_t)t * d + x] = ssum[blk + (size_t)t * d + x] + bf2f(vb[(size_t)t * d + x]);
          }
          scnt[t] += 1;
        }
      }
      if (any) {
        int n = 0;
        for (int t = 0; t < B; ++t) {
          if (scnt[t] <= 0) continue;
          ++n;
          for (int x = 0; x < d; ++x) {
            Kp[((size_t)h * C1 + C) * blk + (size_t)t * d + x] = f2bf(ssum[(size_t)t * d + x] / (float)scnt[t]);
            Vp[((size_t)h * C1 + C) * blk + (size_t)t * d + x] = f2bf(ssum[blk + (size_t)t * d + x] / (float)scnt[t]);
          }
        }
        plen[C] = n;
      }
    }
    /* slot assignment */
    int32_t* src = slot_src + (size_t)h * C;
    for (int s = 0; s < C; ++s) src[s] = -1;
    for (int a = 0; a < nc; ++a)
      if (!win[a] && cand[a] < C) plen[cand[a]] = 0;   /* vacate */
    int s = c->n_sink;
    for (int a = 0; a < nc; ++a) {
      if (!win[a] || cand[a] < C) continue;
      const int e = cand[a] - C;
      while (s < C && plen[s] > 0) ++s;
      if (s >= C) return -2;                           /* cannot happen: winners <= places */
      const size_t from = ((size_t)h * c->n_loc_cap + l_map[e]) * blk;
      const size_t to = ((size_t)h * C1 + s) * blk;
      memcpy(Kp + to, Kl + from, blk * sizeof(uint16_t));
      memcpy(Vp + to, Vl + from, blk * sizeof(uint16_t));
      memcpy(Kc_p + ((size_t)h * C + s) * d, Kc_l + ((size_t)h * c->n_loc_cap + l_map[e]) * d, sizeof(float) * (size_t)d);
      plen[s] = l_len[e];
      p_id[(size_t)h * C + s] = l_id[e];
      src[s] = e;
    }
    for (int q = c->n_sink; q < C; ++q)
      if (plen[q] == 0) p_id[(size_t)h * C + q] = -1;
  }
  free(cand); free(cs); free(win);
  return 0;
}

/* Persistent-memory update with the coarse persistence scores of Eq. 7-8 (orc_scores), then the
 * retention and fold above. */
int orc_memory_update(const orc_cfg* c, const float* Qc, const float* Kc_l, uint16_t* Kp, uint16_t* Vp,
                      float* Kc_p, int32_t* p_len, int64_t* p_id, float* S_sum, int32_t* S_cnt,
                      const uint16_t* Kl, const uint16_t* Vl, const int32_t* l_len, const int32_t* l_map,
                      const int64_t* l_id, float* scores, int32_t* slot_src) {
  float* s_p = (float*)malloc(sizeof(float) * (size_t)(c->H * c->C + 1));
  float* s_l = (float*)malloc(sizeof(float) * (size_t)(c->H * c->n_loc + 1));
  if (!s_p || !s_l) return -1;
  if (orc_scores(c, Qc, Kc_l, l_map, Kc_p, p_len, s_p, s_l)) return -1;
  const int rc = retain_and_fold(c, s_p, s_l, Kc_l, Kp, Vp, Kc_p, p_len, p_id, S_sum, S_cnt, Kl, Vl, l_len, l_map,
                                 l_id, scores, slot_src);
  free(s_p); free(s_l);
  return rc;
}

/* Attention mass that the fine stage (Eq. 3-5) puts on each key block: the variant of the
 * persistence score that accumulates the token-level attention actually paid, mask included,
 * in place of the block-level softmax of Eq. 7.  For each requested query block (head qb_h[n],
 * block qb_i[n]) and each key block u -- persistent slot u for u <= C (the summary is u = C),
 * local block u - C - 1 beyond --
 *     mass[n][u] = sum over the rows q of the query block and the valid tokens j of block u of
 *                  P[q][j],  P = the row softmax of Eq. 3-5 over what row q attends,
 * and 0 for a block the query block does not attend (an empty slot, a local block outside its
 * row of sel).  fp64; every row adds exactly 1 in total.  mass [n_qb][C+1+n_loc]. */
int orc_attention_mass(const orc_cfg* c, const uint16_t* Q, const uint16_t* Kp, const int32_t* p_len,
                       const uint16_t* Kl, const int32_t* l_len, const int32_t* l_map, const int32_t* sel,
                       int64_t n_qb, const int32_t* qb_h, const int32_t* qb_i, double* mass) {
  const int d = c->d, B = c->B, nu = c->C + 1 + c->n_loc;
  const size_t max_keys = (size_t)(c->C + 1 + c->k) * B + 1;
  int fail = 0;
#pragma omp parallel
  {
    double* z = (double*)malloc(sizeof(double) * max_keys);
    int* unit = (int*)malloc(sizeof(int) * max_keys);
    double* q = (double*)malloc(sizeof(double) * (size_t)d);
    if (!z || !unit || !q) {
#pragma omp atomic write
      fail = 1;
    } else {
#pragma omp for schedule(dynamic, 1)
      for (int64_t n = 0; n < n_qb; ++n) {
        const int h = qb_h[n], i = qb_i[n];
        double* out = mass + (size_t)n * nu;
        for (int u = 0; u < nu; ++u) out[u] = 0.0;
        const int32_t* row_sel = sel + ((size_t)h * c->nqb + i) * c->k;
        for (int t = i * B; t < i * B + q_block_len(c, i); ++t) {
          const uint16_t* qrow = Q + ((size_t)h * c->Nq + t) * d;
          for (int x = 0; x < d; ++x) q[x] = (double)bf2f(qrow[x]);
          size_t nk = 0;
          for (int s = 0; s <= c->C; ++s) {
            const int len = p_len[(size_t)h * (c->C + 1) + s];
            const size_t base = ((size_t)h * (c->C + 1) + s) * B * d;
            for (int j = 0; j < len; ++j) {
              double acc = 0.0;
              for (int x = 0; x < d; ++x) acc += q[x] * (double)bf2f(Kp[base + (size_t)j * d + x]);
              z[nk] = acc * (double)c->scale;
              unit[nk++] = s;
            }
          }
          for (int jj = 0; jj < c->k; ++jj) {
            const int l = row_sel[jj];
            if (l < 0) continue;
            const size_t base = ((size_t)h * c->n_loc_cap + l_map[l]) * B * d;
            for (int j = 0; j < l_len[l]; ++j) {
              double acc = 0.0;
              for (int x = 0; x < d; ++x) acc += q[x] * (double)bf2f(Kl[base + (size_t)j * d + x]);
              z[nk] = acc * (double)c->scale;
              unit[nk++] = c->C + 1 + l;
            }
          }
          if (nk == 0) continue;
          double m = z[0];
          for (size_t j = 1; j < nk; ++j) m = z[j] > m ? z[j] : m;
          double sum = 0.0;
          for (size_t j = 0; j < nk; ++j) {
            z[j] = exp(z[j] - m);
            sum += z[j];
          }
          for (size_t j = 0; j < nk; ++j) out[unit[j]] += z[j] / sum;
        }
      }
    }
    free(z);
    free(unit);
    free(q);
  }
  return fail ? -1 : 0;
}

/* Persistent-memory update ranked by accumulated fine attention mass.  Mt [H][C+1+n_loc][nqb]
 * fp32: mass of key block u (numbered as in orc_attention_mass) from query block i.  The score
 * of a block is its mass per query token, in fp32 in a fixed order because it decides the slots:
 *   acc = acc + Mt[h][u][i] over i ascending from 0.0f, then acc / (float)Nq   (0 for an empty slot);
 * retention, slot assignment and fold are those of the coarse update (Eq. 9). */
int orc_memory_update_fine(const orc_cfg* c, const float* Mt, const float* Kc_l, uint16_t* Kp, uint16_t* Vp,
                           float* Kc_p, int32_t* p_len, int64_t* p_id, float* S_sum, int32_t* S_cnt,
                           const uint16_t* Kl, const uint16_t* Vl, const int32_t* l_len, const int32_t* l_map,
                           const int64_t* l_id, float* scores, int32_t* slot_src) {
  const int nu = c->C + 1 + c->n_loc;
  float* s_p = (float*)malloc(sizeof(float) * (size_t)(c->H * c->C + 1));
  float* s_l = (float*)malloc(sizeof(float) * (size_t)(c->H * c->n_loc + 1));
  if (!s_p || !s_l) return -1;
  for (int h = 0; h < c->H; ++h) {
    for (int u = 0; u < nu; ++u) {
      if (u == c->C) continue;                        /* the summary is never a candidate */
      float acc = 0.0f;
      for (int i = 0; i < c->nqb; ++i) acc = acc + Mt[((size_t)h * nu + u) * c->nqb + i];
      const float s = acc / (float)c->Nq;
      if (u < c->C) s_p[(size_t)h * c->C + u] = p_len[(size_t)h * (c->C + 1) + u] > 0 ? s : 0.0f;
      else s_l[(size_t)h * c->n_loc + (u - c->C - 1)] = s;
    }
  }
  const int rc = retain_and_fold(c, s_p, s_l, Kc_l, Kp, Vp, Kc_p, p_len, p_id, S_sum, S_cnt, Kl, Vl, l_len, l_map,
                                 l_id, scores, slot_src);
  free(s_p); free(s_l);
  return rc;
}

/* Backward of the PBSA fine stage (the gradient of Eq. 3-5; the paper's training kernel): given dO, the
 * gradient of a scalar loss with respect to the output O = P V, with P the masked row softmax of
 * Z = scale * Q K^T over what each row attends,
 *     dV_j  = sum_q P[q][j] dO[q]                      dP[q][j] = dO[q] . V_j
 *     dZ    = P o (dP - D),  D[q] = sum_j P[q][j] dP[q][j]  ( = dO[q] . O[q] )
 *     dQ_q  = scale * sum_j dZ[q][j] K_j               dK_j  = scale * sum_q dZ[q][j] Q_q
 * (the chain rule through a row softmax, written out).  Everything in fp64 from the bf16 inputs; O is
 * recomputed here, not taken from anybody.  Q, dO [H][Nq][d] bf16 bits.  Outputs fp64, each either NULL
 * or zero-filled by the caller: dQ [H][Nq][d], dKp/dVp [H][C+1][B][d], dKl/dVl [H][n_loc_cap][B][d]
 * (physical slots, like Kl).  A key that no row attends, and rows past a block's length, get nothing.
 * row_mask (optional, [H][Nq] bytes): only rows with a non-zero byte take part, so that the cost of a
 * check at full size can be bounded; their dQ is exact, dK/dV are then the sums over those rows only. */
int orc_attention_bwd(const orc_cfg* c, const uint16_t* Q, const uint16_t* Kp, const uint16_t* Vp,
                      const int32_t* p_len, const uint16_t* Kl, const uint16_t* Vl, const int32_t* l_len,
                      const int32_t* l_map, const int32_t* sel, const uint16_t* dO, const uint8_t* row_mask,
                      double* dQ, double* dKp, double* dVp, double* dKl, double* dVl) {
  const int d = c->d, B = c->B;
  const size_t max_keys = (size_t)(c->C + 1 + c->k) * B + 1;
  int fail = 0;
#pragma omp parallel for schedule(dynamic, 1)
  for (int h = 0; h < c->H; ++h) {          /* a head's keys belong to that head alone: no two threads share an output */
    double* z = (double*)malloc(sizeof(double) * max_keys);
    const uint16_t** krow = (const uint16_t**)malloc(sizeof(void*) * max_keys);
    const uint16_t** vrow = (const uint16_t**)malloc(sizeof(void*) * max_keys);
    double** dk = (double**)malloc(sizeof(void*) * max_keys);
    double** dv = (double**)malloc(sizeof(void*) * max_keys);
    double* q = (double*)malloc(sizeof(double) * (size_t)d);
    double* g = (double*)malloc(sizeof(double) * (size_t)d);
    double* o = (double*)malloc(sizeof(double) * (size_t)d);
    if (!z || !krow || !vrow || !dk || !dv || !q || !g || !o) {
#pragma omp atomic write
      fail = 1;
    } else {
      for (int t = 0; t < c->Nq; ++t) {
        if (row_mask && !row_mask[(size_t)h * c->Nq + t]) continue;
        const int i = t / B;
        for (int x = 0; x < d; ++x) {
          q[x] = (double)bf2f(Q[((size_t)h * c->Nq + t) * d + x]);
          g[x] = (double)bf2f(dO[((size_t)h * c->Nq + t) * d + x]);
        }
        size_t n = 0;
        for (int s = 0; s <= c->C; ++s) {
          const size_t base = ((size_t)h * (c->C + 1) + s) * B * d;
          for (int u = 0; u < p_len[(size_t)h * (c->C + 1) + s]; ++u, ++n) {
            krow[n] = Kp + base + (size_t)u * d;
            vrow[n] = Vp + base + (size_t)u * d;
            dk[n] = dKp ? dKp + base + (size_t)u * d : NULL;
            dv[n] = dVp ? dVp + base + (size_t)u * d : NULL;
          }
        }
        const int32_t* row_sel = sel + ((size_t)h * c->nqb + i) * c->k;
        for (int j = 0; j < c->k; ++j) {
          const int l = row_sel[j];
          if (l < 0) continue;
          const size_t base = ((size_t)h * c->n_loc_cap + l_map[l]) * B * d;
          for (int u = 0; u < l_len[l]; ++u, ++n) {
            krow[n] = Kl + base + (size_t)u * d;
            vrow[n] = Vl + base + (size_t)u * d;
            dk[n] = dKl ? dKl + base + (size_t)u * d : NULL;
            dv[n] = dVl ? dVl + base + (size_t)u * d : NULL;
          }
        }
        if (n == 0) continue;
        double m = -INFINITY;
        for (size_t j = 0; j < n; ++j) {
          double acc = 0.0;
          for (int x = 0; x < d; ++x) acc += q[x] * (double)bf2f(krow[j][x]);
          z[j] = acc * (double)c->scale;
          m = z[j] > m ? z[j] : m;
        }
        double sum = 0.0;
        for (size_t j = 0; j < n; ++j) {
          z[j] = exp(z[j] - m);
          sum += z[j];
        }
        for (int x = 0; x < d; ++x) o[x] = 0.0;
        for (size_t j = 0; j < n; ++j) {
          z[j] /= sum;                                      /* P[q][j] */
          for (int x = 0; x < d; ++x) o[x] += z[j] * (double)bf2f(vrow[j][x]);
        }
        double D = 0.0;
        for (int x = 0; x < d; ++x) D += g[x] * o[x];
        for (size_t j = 0; j < n; ++j) {
          double dp = 0.0;
          for (int x = 0; x < d; ++x) dp += g[x] * (double)bf2f(vrow[j][x]);
          const double dz = z[j] * (dp - D) * (double)c->scale;
          if (dQ)
            for (int x = 0; x < d; ++x) dQ[((size_t)h * c->Nq + t) * d + x] += dz * (double)bf2f(krow[j][x]);
          if (dk[j])
            for (int x = 0; x < d; ++x) dk[j][x] += dz * q[x];
          if (dv[j])
            for (int x = 0; x < d; ++x) dv[j][x] += z[j] * g[x];
        }
      }
    }
    free(z); free(krow); free(vrow); free(dk); free(dv); free(q); free(g); free(o);
  }
  return fail ? -1 : 0;
}
