/*
 * NOSA decode-step oracle: a plain, slow, fp64 CPU statement of what the path computes.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the product path may include, link or call
 * this file; it shares no code, header, table or constant with the HIP library.
 * It is written from the paper's definitions, one unit (batch element x KV head)
 * at a time, with no blocking, no online softmax and no reordering:
 *
 *   oracle_pool          block compression f_c (Sec. 2.1) realised as the mean of Eq. (mean
 *                        pooling, Sec. 3.1 "Adapting to Block-wise Selection") on keys and on
 *                        the importance score
 *   oracle_block_score   S_c^q = Q K_c^T (Sec. 2.1; Alg. 1 "Stage 1"), sum over the query
 *                        heads of the GQA group, then the block-level max of Eq. (max pooling)
 *                        applied identically to the query-aware and query-agnostic scores
 *   oracle_select        Eq. (selection): sink and window blocks of the InfLLMv2 mask
 *                        (Sec. 2.1) are forced, Top_{kq/nb} by the query-aware score, then the
 *                        rest of the budget by the importance score
 *   oracle_load          the set difference / replacement mapping of Sec. 4 "Memory Layout and
 *                        Block Selection" (Alg. 1 generate_load_positions)
 *   oracle_fetch         Sec. 4 "Offloading Communication": copy missed blocks host -> slot
 *   oracle_attention     the biased attention output of Sec. 3.1 "Attention Calculation"
 *                        (exp(b_j) exp(q k_j + m_j) normalised), restricted to Gamma(t)
 *   oracle_append        the cache update that precedes Stage 1 in Alg. 1, for a growing context
 *   oracle_split_qkv_evict  QKV split + eviction head (importance-score Eq.; Sec. 4 "Kernel Fusion")
 *
 * Readings taken where the paper is silent (each is a parameter or a stated rule):
 *   - pooling windows are half open, [j*ls, j*ls+lk): exactly lk terms;
 *   - a sub-block belongs to a block only if it lies wholly inside it;
 *   - the G query heads of a KV head are combined by summing their raw scores;
 *   - softmax_scale multiplies q.k only (never the bias); selection scores are unscaled;
 *   - only complete blocks are candidates; the partial tail is attended through the window;
 *   - ties go to the lower block index; Gamma is returned in ascending order, -1 padded;
 *   - victims are the slots (ascending) that are empty or hold a block outside Gamma; the
 *     i-th miss (ascending block index) takes the i-th victim.
 *
 * Element types: dtype 0 = IEEE fp32, dtype 1 = bfloat16 (upper 16 bits of an fp32),
 * both widened exactly to fp64 before any arithmetic.
 *
 * Parity pins (tests/test_oracle_*.py): brute-force dense attention restricted to Gamma,
 * textbook softmax attention when everything is selected and b = 0, exhaustive subset
 * search for the selection on tiny inputs, the single-pass +inf formulation of
 * Eq. (selection), linearity of pooled-key scoring, the locality bound of Theorem 1;
 * oracle_fetch_tokens against a fancy-index row gather and against oracle_fetch on whole blocks.
 * Unpinned (readings, no printed values exist in the paper): the choices listed above.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
  int32_t batch, n_q_heads, n_kv_heads, head_dim;
  int32_t block_size;
  int32_t pool_kernel, pool_stride;
  int32_t k_blocks, kq_blocks;
  int32_t sink_blocks, window_blocks;
  int32_t gpu_slots;
  int32_t max_blocks;   /* Nmax: blocks per unit in the host pool and in the maps */
  int32_t n_sub_max;    /* sub-blocks per unit in k_pooled / se_pooled            */
  int32_t dtype;        /* 0 fp32, 1 bf16                                         */
  int32_t victim_policy; /* 0: free slots in ascending order; 1: least important block first */
  double softmax_scale;
} oracle_params;

static double load_elem(const void *base, int64_t i, int dtype) {
  if (dtype == 0) return (double)((const float *)base)[i];
  uint32_t bits = ((uint32_t)((const uint16_t *)base)[i]) << 16;
  float f;
  memcpy(&f, &bits, 4);
  return (double)f;
}

/* fp64 -> bf16, round to nearest, ties to even, decided in fp64 (no double rounding):
 * the two bf16 neighbours of |x| are found from the fp32 rounding of x (bf16 values are
 * fp32 values, and rounding is monotone), then the nearer one is taken.  Finite inputs. */
static uint16_t to_bf16(double x) {
  float f = (float)x;
  uint32_t u;
  memcpy(&u, &f, 4);
  const uint32_t sign = u & 0x80000000u;
  const uint32_t lo_bits = u & 0x7fff0000u, hi_bits = lo_bits + 0x10000u;
  float lo, hi;
  memcpy(&lo, &lo_bits, 4);
  memcpy(&hi, &hi_bits, 4);
  const double ax = fabs(x), dl = ax - (double)lo, dh = (double)hi - ax;
  uint32_t r;
  if (dl < dh) r = lo_bits;
  else if (dh < dl) r = hi_bits;
  else r = ((lo_bits >> 16) & 1u) ? hi_bits : lo_bits;
  return (uint16_t)((r | sign) >> 16);
}

int oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

void oracle_set_threads(int n) {
#ifdef _OPENMP
  if (n > 0) omp_set_num_threads(n);
#else
  (void)n;
#endif
}

static int n_sub_of(int T, int lk, int ls) { return T < lk ? 0 : (T - lk) / ls + 1; }

/* ---- pooling: K_c[j] = mean_{t in <j>} k_t, S_c^e[j] = mean_{t in <j>} s_t^e -------------
 * keys  [B,Hkv,Nmax,nb,d] (token t of a unit = block t/nb, row t%nb), bias [B,Hkv,Nmax,nb]
 * -> k_pooled [B,Hkv,n_sub_max,d] (dtype, RNE), se_pooled [B,Hkv,n_sub_max] fp32.
 * Sub-blocks that are not complete at n_tokens[b] are written as zero.                     */
void oracle_pool(const oracle_params *p, const void *keys, const float *bias, const int32_t *n_tokens,
                 void *k_pooled, float *se_pooled) {
  const int d = p->head_dim, nb = p->block_size, lk = p->pool_kernel, ls = p->pool_stride;
  const int units = p->batch * p->n_kv_heads;
#pragma omp parallel for schedule(dynamic)
  for (int u = 0; u < units; ++u) {
    const int b = u / p->n_kv_heads;
    const int T = n_tokens[b];
    const int nsub = n_sub_of(T, lk, ls);
    const int64_t kbase = (int64_t)u * p->max_blocks * nb * d;
    const int64_t bbase = (int64_t)u * p->max_blocks * nb;
    for (int j = 0; j < p->n_sub_max; ++j) {
      const int64_t obase = ((int64_t)u * p->n_sub_max + j) * d;
      if (j >= nsub) {
        for (int e = 0; e < d; ++e) {
          if (p->dtype == 0) ((float *)k_pooled)[obase + e] = 0.f;
          else ((uint16_t *)k_pooled)[obase + e] = 0;
        }
        se_pooled[(int64_t)u * p->n_sub_max + j] = 0.f;
        continue;
      }
      for (int e = 0; e < d; ++e) {
        double s = 0.0;
        for (int t = j * ls; t < j * ls + lk; ++t) s += load_elem(keys, kbase + (int64_t)t * d + e, p->dtype);
        s /= (double)lk;
        if (p->dtype == 0) ((float *)k_pooled)[obase + e] = (float)s;
        else ((uint16_t *)k_pooled)[obase + e] = to_bf16(s);
      }
      double sb = 0.0;
      for (int t = j * ls; t < j * ls + lk; ++t) sb += (double)bias[bbase + t];
      se_pooled[(int64_t)u * p->n_sub_max + j] = (float)(sb / (double)lk);
    }
  }
}

/* ---- block scores --------------------------------------------------------------------------
 * q [B,Hq,d], k_pooled [B,Hkv,n_sub_max,d], se_pooled [B,Hkv,n_sub_max]
 * -> sq_blk, se_blk [B,Hkv,Nmax] fp64; -inf where a block holds no complete sub-block.
 * Optionally (sq_head != NULL) the per-head sub-block scores [B,Hq,n_sub_max] before the
 * group sum are returned for inspection.                                                     */
void oracle_block_score(const oracle_params *p, const void *q, const void *k_pooled, const float *se_pooled,
                        const int32_t *n_tokens, double *sq_blk, double *se_blk, double *sq_head) {
  const int d = p->head_dim, nb = p->block_size, lk = p->pool_kernel, ls = p->pool_stride;
  const int G = p->n_q_heads / p->n_kv_heads;
  const int units = p->batch * p->n_kv_heads;
#pragma omp parallel for schedule(dynamic)
  for (int u = 0; u < units; ++u) {
    const int b = u / p->n_kv_heads, h = u % p->n_kv_heads;
    const int T = n_tokens[b];
    const int nsub = n_sub_of(T, lk, ls);
    double *sq = sq_blk + (int64_t)u * p->max_blocks;
    double *se = se_blk + (int64_t)u * p->max_blocks;
    for (int J = 0; J < p->max_blocks; ++J) sq[J] = se[J] = -INFINITY;
    for (int j = 0; j < nsub; ++j) {
      /* query-aware score of sub-block j: one dot product per query head, summed over the group */
      double sgroup = 0.0;
      for (int g = 0; g < G; ++g) {
        const int64_t qb = ((int64_t)b * p->n_q_heads + h * G + g) * d;
        const int64_t kb = ((int64_t)u * p->n_sub_max + j) * d;
        double dot = 0.0;
        for (int e = 0; e < d; ++e) dot += load_elem(q, qb + e, p->dtype) * load_elem(k_pooled, kb + e, p->dtype);
        if (sq_head) sq_head[((int64_t)b * p->n_q_heads + h * G + g) * p->n_sub_max + j] = dot;
        sgroup += dot;
      }
      /* block J contains sub-block j iff [j*ls, j*ls+lk) lies inside [J*nb, (J+1)*nb) */
      const int lo = j * ls, hi = j * ls + lk;
      const int J = lo / nb;
      if (hi > (J + 1) * nb || J >= p->max_blocks) continue;
      if (sgroup > sq[J]) sq[J] = sgroup;
      const double sej = (double)se_pooled[(int64_t)u * p->n_sub_max + j];
      if (sej > se[J]) se[J] = sej;
    }
  }
}

/* ---- constrained selection -----------------------------------------------------------------
 * sq_blk, se_blk [B,Hkv,Nmax] fp64 -> sel_idx [B,Hkv,K] ascending, -1 padded; n_sel [B,Hkv].
 * kind (optional, [B,Hkv,K]): 0 forced (sink/window), 1 query-aware, 2 query-agnostic, -1 pad.  */
static int arg_best(const double *s, const uint8_t *eligible, int n) {
  int best = -1;
  for (int J = 0; J < n; ++J) {
    if (!eligible[J]) continue;
    if (best < 0 || s[J] > s[best]) best = J; /* strict '>' keeps the lower index on ties */
  }
  return best;
}

void oracle_select(const oracle_params *p, const double *sq_blk, const double *se_blk, const int32_t *n_tokens,
                   int32_t *sel_idx, int32_t *n_sel, int32_t *kind) {
  const int nb = p->block_size, K = p->k_blocks;
  const int units = p->batch * p->n_kv_heads;
#pragma omp parallel for schedule(dynamic)
  for (int u = 0; u < units; ++u) {
    const int b = u / p->n_kv_heads;
    const int T = n_tokens[b];
    const int N = (T + nb - 1) / nb, Nc = T / nb;
    const double *sq = sq_blk + (int64_t)u * p->max_blocks;
    const double *se = se_blk + (int64_t)u * p->max_blocks;
    uint8_t *mark = (uint8_t *)calloc((size_t)(N > 0 ? N : 1), 1);     /* 0 none, 1 forced, 2 q, 3 e */
    uint8_t *elig = (uint8_t *)calloc((size_t)(N > 0 ? N : 1), 1);
    int nF = 0;
    for (int J = 0; J < N; ++J) {
      const int sink = J < p->sink_blocks;
      const int window = J >= N - p->window_blocks;
      if (sink || window) { mark[J] = 1; ++nF; }
    }
    int nD = 0;
    for (int J = 0; J < Nc; ++J) if (!mark[J]) { elig[J] = 1; ++nD; }
    int kq = p->kq_blocks < nD ? p->kq_blocks : nD;
    for (int i = 0; i < kq; ++i) {
      const int J = arg_best(sq, elig, Nc);
      mark[J] = 2; elig[J] = 0;
    }
    int ke = K - nF - p->kq_blocks;
    if (ke < 0) ke = 0;
    if (ke > nD - kq) ke = nD - kq;
    for (int i = 0; i < ke; ++i) {
      const int J = arg_best(se, elig, Nc);
      mark[J] = 3; elig[J] = 0;
    }
    int n = 0;
    int32_t *out = sel_idx + (int64_t)u * K;
    int32_t *kd = kind ? kind + (int64_t)u * K : NULL;
    for (int J = 0; J < N && n < K; ++J) {
      if (!mark[J]) continue;
      out[n] = J;
      if (kd) kd[n] = mark[J] - 1;
      ++n;
    }
    n_sel[u] = n;
    for (int i = n; i < K; ++i) { out[i] = -1; if (kd) kd[i] = -1; }
    free(mark); free(elig);
  }
}

/* ---- load positions: Gamma(t) against the resident map -----------------------------------
 * in/out slot_of_block [B,Hkv,Nmax], block_of_slot [B,Hkv,C]; out load_list [B,Hkv,K,2]
 * (block, slot) pairs, -1 padded; n_load [B,Hkv].                                           */
/* victim_policy 1 (a GPU pool larger than the selection, C > K): among the free slots the ones
 * used are the empty ones (or ones holding a block beyond the current context) first, then those
 * whose block has the smallest block-level importance
 * se_blk (ties: lower slot); the chosen slots are then handed out in ascending slot order.        */
typedef struct { int cls; double se; int slot; } victim_key;
static int victim_cmp(const void *a, const void *b) {
  const victim_key *x = (const victim_key *)a, *y = (const victim_key *)b;
  if (x->cls != y->cls) return x->cls - y->cls;
  if (x->se != y->se) return x->se < y->se ? -1 : 1;
  return x->slot - y->slot;
}
static int int_cmp(const void *a, const void *b) { return *(const int *)a - *(const int *)b; }

void oracle_load_policy(const oracle_params *p, const int32_t *sel_idx, const int32_t *n_sel, const double *se_blk,
                        const int32_t *n_tokens, int32_t *slot_of_block, int32_t *block_of_slot, int32_t *load_list,
                        int32_t *n_load) {
  const int K = p->k_blocks, C = p->gpu_slots;
  const int units = p->batch * p->n_kv_heads;
  for (int u = 0; u < units; ++u) {
    const int N = (n_tokens[u / p->n_kv_heads] + p->block_size - 1) / p->block_size;   /* blocks in use */
    const int32_t *sel = sel_idx + (int64_t)u * K;
    int32_t *sob = slot_of_block + (int64_t)u * p->max_blocks;
    int32_t *bos = block_of_slot + (int64_t)u * C;
    int32_t *ll = load_list + (int64_t)u * K * 2;
    uint8_t *in_gamma = (uint8_t *)calloc((size_t)p->max_blocks, 1);
    for (int i = 0; i < n_sel[u]; ++i) in_gamma[sel[i]] = 1;
    int n_miss = 0;
    for (int i = 0; i < n_sel[u]; ++i) if (sob[sel[i]] < 0) ++n_miss;
    victim_key *fr = (victim_key *)malloc(sizeof(victim_key) * (size_t)C);
    int nf = 0;
    for (int s = 0; s < C; ++s) {
      if (bos[s] >= 0 && in_gamma[bos[s]]) continue;
      const int stale = bos[s] < 0 || bos[s] >= N;     /* empty, or a block beyond the current context */
      fr[nf].cls = stale ? 0 : 1;
      fr[nf].se = stale ? 0.0 : se_blk[(int64_t)u * p->max_blocks + bos[s]];
      fr[nf].slot = s;
      ++nf;
    }
    if (p->victim_policy == 1) qsort(fr, (size_t)nf, sizeof(victim_key), victim_cmp);
    const int take = n_miss < nf ? n_miss : nf;
    int *chosen = (int *)malloc(sizeof(int) * (size_t)(take > 0 ? take : 1));
    for (int i = 0; i < take; ++i) chosen[i] = fr[i].slot;
    qsort(chosen, (size_t)take, sizeof(int), int_cmp);
    int nl = 0;
    for (int i = 0; i < n_sel[u] && nl < take; ++i) {
      const int J = sel[i];
      if (sob[J] >= 0) continue;
      const int s = chosen[nl];
      if (bos[s] >= 0) sob[bos[s]] = -1;
      bos[s] = J; sob[J] = s;
      ll[2 * nl] = J; ll[2 * nl + 1] = s;
      ++nl;
    }
    n_load[u] = nl;
    for (int i = nl; i < K; ++i) { ll[2 * i] = -1; ll[2 * i + 1] = -1; }
    free(in_gamma); free(fr); free(chosen);
  }
}

void oracle_load(const oracle_params *p, const int32_t *sel_idx, const int32_t *n_sel,
                 int32_t *slot_of_block, int32_t *block_of_slot, int32_t *load_list, int32_t *n_load) {
  const int K = p->k_blocks, C = p->gpu_slots;
  const int units = p->batch * p->n_kv_heads;
  for (int u = 0; u < units; ++u) {
    const int32_t *sel = sel_idx + (int64_t)u * K;
    int32_t *sob = slot_of_block + (int64_t)u * p->max_blocks;
    int32_t *bos = block_of_slot + (int64_t)u * C;
    int32_t *ll = load_list + (int64_t)u * K * 2;
    uint8_t *in_gamma = (uint8_t *)calloc((size_t)p->max_blocks, 1);
    for (int i = 0; i < n_sel[u]; ++i) in_gamma[sel[i]] = 1;
    int nl = 0, s = 0;
    for (int i = 0; i < n_sel[u]; ++i) {
      const int J = sel[i];
      if (sob[J] >= 0) continue;                       /* hit */
      while (s < C && bos[s] >= 0 && in_gamma[bos[s]]) ++s;   /* next victim */
      if (s >= C) break;                               /* cannot happen when C >= K */
      if (bos[s] >= 0) sob[bos[s]] = -1;
      bos[s] = J; sob[J] = s;
      ll[2 * nl] = J; ll[2 * nl + 1] = s;
      ++nl; ++s;
    }
    n_load[u] = nl;
    for (int i = nl; i < K; ++i) { ll[2 * i] = -1; ll[2 * i + 1] = -1; }
    free(in_gamma);
  }
}

/* ---- fetch: host pool -> GPU pool slots (bytes) ------------------------------------------ */
void oracle_fetch(const oracle_params *p, const void *host_k, const void *host_v, const float *host_bias,
                  void *pool_k, void *pool_v, float *pool_bias, const int32_t *load_list, const int32_t *n_load) {
  const int K = p->k_blocks, C = p->gpu_slots, nb = p->block_size, d = p->head_dim;
  const size_t es = p->dtype == 0 ? 4 : 2;
  const size_t blk = (size_t)nb * d * es;
  const int units = p->batch * p->n_kv_heads;
  for (int u = 0; u < units; ++u) {
    for (int i = 0; i < n_load[u]; ++i) {
      const int J = load_list[((int64_t)u * K + i) * 2], s = load_list[((int64_t)u * K + i) * 2 + 1];
      const size_t src = ((size_t)u * p->max_blocks + J), dst = ((size_t)u * C + s);
      memcpy((char *)pool_k + dst * blk, (const char *)host_k + src * blk, blk);
      memcpy((char *)pool_v + dst * blk, (const char *)host_v + src * blk, blk);
      if (host_bias && pool_bias) memcpy(pool_bias + dst * nb, host_bias + src * nb, (size_t)nb * 4);
    }
  }
}

/* ---- attention over the selected blocks ---------------------------------------------------
 * q [B,Hq,d]; pool_k/pool_v [B,Hkv,C,nb,d]; pool_bias [B,Hkv,C,nb] or NULL;
 * out [B,Hq,d] fp64; lse [B,Hq] fp64 (may be NULL); probs (may be NULL) [B,Hq,K*nb]: the
 * softmax weights in selection order, zero for masked / padded positions.
 * Returns the number of selected blocks found without a slot (must be 0).                   */
int oracle_attention(const oracle_params *p, const void *q, const void *pool_k, const void *pool_v,
                     const float *pool_bias, const int32_t *sel_idx, const int32_t *n_sel,
                     const int32_t *slot_of_block, const int32_t *n_tokens, double *out, double *lse,
                     double *probs) {
  const int d = p->head_dim, nb = p->block_size, K = p->k_blocks, C = p->gpu_slots;
  const int G = p->n_q_heads / p->n_kv_heads;
  const int units = p->batch * p->n_kv_heads;
  int bad = 0;
#pragma omp parallel for schedule(dynamic) reduction(+ : bad)
  for (int u = 0; u < units; ++u) {
    const int b = u / p->n_kv_heads, h = u % p->n_kv_heads;
    const int T = n_tokens[b];
    const int32_t *sel = sel_idx + (int64_t)u * K;
    const int32_t *sob = slot_of_block + (int64_t)u * p->max_blocks;
    double *z = (double *)malloc(sizeof(double) * (size_t)K * nb);
    for (int g = 0; g < G; ++g) {
      const int hq = h * G + g;
      const int64_t qb = ((int64_t)b * p->n_q_heads + hq) * d;
      double zmax = -INFINITY;
      for (int i = 0; i < K; ++i) {
        for (int r = 0; r < nb; ++r) z[i * nb + r] = -INFINITY;
        if (i >= n_sel[u]) continue;
        const int J = sel[i], s = sob[J];
        if (s < 0) { ++bad; continue; }
        for (int r = 0; r < nb; ++r) {
          const int t = J * nb + r;
          if (t >= T) break;
          const int64_t kb = (((int64_t)u * C + s) * nb + r) * d;
          double dot = 0.0;
          for (int e = 0; e < d; ++e) dot += load_elem(q, qb + e, p->dtype) * load_elem(pool_k, kb + e, p->dtype);
          double zz = p->softmax_scale * dot;
          if (pool_bias) zz += (double)pool_bias[((int64_t)u * C + s) * nb + r];
          z[i * nb + r] = zz;
          if (zz > zmax) zmax = zz;
        }
      }
      double denom = 0.0;
      for (int i = 0; i < K * nb; ++i) denom += (z[i] == -INFINITY) ? 0.0 : exp(z[i] - zmax);
      double *o = out + qb;
      for (int e = 0; e < d; ++e) o[e] = 0.0;
      for (int i = 0; i < K; ++i) {
        if (i >= n_sel[u]) break;
        const int J = sel[i], s = sob[J];
        if (s < 0) continue;
        for (int r = 0; r < nb; ++r) {
          if (z[i * nb + r] == -INFINITY) continue;
          const double w = exp(z[i * nb + r] - zmax) / denom;
          const int64_t vb = (((int64_t)u * C + s) * nb + r) * d;
          for (int e = 0; e < d; ++e) o[e] += w * load_elem(pool_v, vb + e, p->dtype);
        }
      }
      if (probs) {
        double *pr = probs + ((int64_t)b * p->n_q_heads + hq) * K * nb;
        for (int i = 0; i < K * nb; ++i) pr[i] = (z[i] == -INFINITY) ? 0.0 : exp(z[i] - zmax) / denom;
      }
      if (lse) lse[(int64_t)b * p->n_q_heads + hq] = zmax + log(denom);
    }
    free(z);
  }
  return bad;
}

/* ---- growing context: append one token per unit (Alg. 1 cache update before Stage 1) ---------
 * k_new, v_new [B,Hkv,d] (dtype), b_new [B,Hkv] fp32.  Token t = n_tokens[b] of every unit of batch
 * element b is written to the host pool (block J = t / nb, row t % nb) and, if block J has a slot,
 * to that slot.  When the token opens a new block (row 0) the block is given a slot first: the lowest
 * empty slot, else the slot whose block has the smallest block-level importance se_blk among the
 * resident blocks that are neither sink blocks nor among the Nw - 1 blocks before J that stay in the
 * window (the block that leaves the window, J - Nw, is a candidate like any other) (ties:
 * lower slot); if there is none the block simply stays non-resident and is fetched like any miss.
 * Evicting the least important resident candidate keeps the Ke best-by-importance candidates
 * resident, which is what the proof of Theorem 1 needs for the per-step fetch bound.
 * n_tokens is incremented once per batch element at the end.  Tokens beyond the table capacity
 * (t >= max_blocks * nb) are ignored.  Pooled arrays are not touched here (see oracle_pool).      */
void oracle_append(const oracle_params *p, const void *k_new, const void *v_new, const float *b_new,
                   void *pool_k, void *pool_v, float *pool_bias, void *host_k, void *host_v, float *host_bias,
                   const double *se_blk, int32_t *n_tokens, int32_t *slot_of_block, int32_t *block_of_slot) {
  const int nb = p->block_size, d = p->head_dim, C = p->gpu_slots;
  const size_t es = p->dtype == 0 ? 4 : 2;
  const size_t rowb = (size_t)d * es;
  const int units = p->batch * p->n_kv_heads;
  for (int u = 0; u < units; ++u) {
    const int b = u / p->n_kv_heads;
    const int t = n_tokens[b];
    if (t >= p->max_blocks * nb) continue;
    const int J = t / nb, row = t % nb;
    int32_t *sob = slot_of_block + (int64_t)u * p->max_blocks;
    int32_t *bos = block_of_slot + (int64_t)u * C;
    const size_t hrow = ((size_t)u * p->max_blocks + J) * nb + row;
    memcpy((char *)host_k + hrow * rowb, (const char *)k_new + (size_t)u * rowb, rowb);
    memcpy((char *)host_v + hrow * rowb, (const char *)v_new + (size_t)u * rowb, rowb);
    host_bias[hrow] = b_new[u];
    if (row == 0 && sob[J] < 0) {
      int best = -1;
      for (int s = 0; s < C && best < 0; ++s) if (bos[s] < 0) best = s;
      if (best < 0) {
        const int protect = p->window_blocks;   /* blocks J-Nw+1 .. J-1 stay in the window */
        for (int s = 0; s < C; ++s) {
          const int Jp = bos[s];
          if (Jp < p->sink_blocks || Jp > J - protect) continue;
          if (best < 0 || se_blk[(int64_t)u * p->max_blocks + Jp] < se_blk[(int64_t)u * p->max_blocks + bos[best]]) best = s;
        }
      }
      if (best >= 0) {
        if (bos[best] >= 0) sob[bos[best]] = -1;
        bos[best] = J;
        sob[J] = best;
      }
    }
    if (sob[J] >= 0) {
      const size_t prow = ((size_t)u * C + sob[J]) * nb + row;
      memcpy((char *)pool_k + prow * rowb, (const char *)k_new + (size_t)u * rowb, rowb);
      memcpy((char *)pool_v + prow * rowb, (const char *)v_new + (size_t)u * rowb, rowb);
      pool_bias[prow] = b_new[u];
    }
  }
  for (int b = 0; b < p->batch; ++b)
    if (n_tokens[b] < p->max_blocks * nb) n_tokens[b] += 1;
}

/* ---- eviction head on the value of the current token (importance-score Eq., Sec. 3.1; ED-DMA row
 * of the table in App. D: b_j = tau(v_j W_1) (.) W_2, tau = softplus, no final exp) together with
 * the split of the fused QKV activation (Alg. 1 fused_linear_projection; Sec. 4 "Kernel Fusion").
 * qkv [B, (Hq + 2 Hkv) d]: all query heads, then all key heads, then all value heads of a token.
 * w1 [d, Hkv] (row e, column m), w2 [Hkv], both fp32.
 *   mode 0 (table, one gate per KV head):  b[b,h] = softplus(v_h . w1[:,h]) * w2[h]
 *   mode 1 (Eq. as printed, W_1 in R^{d x Hkv}, W_2 in R^{Hkv x 1}, shared by the heads):
 *                                          b[b,h] = sum_m softplus(v_h . w1[:,m]) * w2[m]
 * q_out [B,Hq,d], k_new, v_new [B,Hkv,d] are bit copies; b_new [B,Hkv] fp64.                      */
static double softplus64(double x) { return (x > 0 ? x : 0) + log1p(exp(-fabs(x))); }

void oracle_split_qkv_evict(const oracle_params *p, const void *qkv, const float *w1, const float *w2, int mode,
                            void *q_out, void *k_new, void *v_new, double *b_new) {
  const int d = p->head_dim, Hq = p->n_q_heads, Hkv = p->n_kv_heads;
  const size_t es = p->dtype == 0 ? 4 : 2;
  const size_t row = (size_t)(Hq + 2 * Hkv) * d;
  for (int b = 0; b < p->batch; ++b) {
    const char *src = (const char *)qkv + (size_t)b * row * es;
    memcpy((char *)q_out + (size_t)b * Hq * d * es, src, (size_t)Hq * d * es);
    memcpy((char *)k_new + (size_t)b * Hkv * d * es, src + (size_t)Hq * d * es, (size_t)Hkv * d * es);
    memcpy((char *)v_new + (size_t)b * Hkv * d * es, src + (size_t)(Hq + Hkv) * d * es, (size_t)Hkv * d * es);
    for (int h = 0; h < Hkv; ++h) {
      const int64_t vb = (int64_t)b * row + (int64_t)(Hq + Hkv + h) * d;
      double acc = 0.0;
      for (int m = 0; m < Hkv; ++m) {
        if (mode == 0 && m != h) continue;
        double dot = 0.0;
        for (int e = 0; e < d; ++e) dot += load_elem(qkv, vb + e, p->dtype) * (double)w1[(int64_t)e * Hkv + m];
        acc += softplus64(dot) * (double)w2[m];
      }
      b_new[(int64_t)b * Hkv + h] = acc;
    }
  }
}

/* ---- element-wise transfer (Sec. 3.2 "Comparison with DMA": token-granular host-to-device copies,
 * the pattern that block-wise selection avoids).  token_list [B,Hkv,M,2] = (token index in the host
 * cache, row index in the GPU pool viewed as [C*nb] rows), n_list [B,Hkv].  Copies K row, V row, bias. */
void oracle_fetch_tokens(const oracle_params *p, const void *host_k, const void *host_v, const float *host_bias,
                         void *pool_k, void *pool_v, float *pool_bias, const int32_t *token_list, const int32_t *n_list,
                         int max_list) {
  const int nb = p->block_size, d = p->head_dim, C = p->gpu_slots;
  const size_t rowb = (size_t)d * (p->dtype == 0 ? 4 : 2);
  const int units = p->batch * p->n_kv_heads;
  for (int u = 0; u < units; ++u)
    for (int i = 0; i < n_list[u]; ++i) {
      const int t = token_list[((int64_t)u * max_list + i) * 2], r = token_list[((int64_t)u * max_list + i) * 2 + 1];
      const size_t src = (size_t)u * p->max_blocks * nb + t, dst = (size_t)u * C * nb + r;
      memcpy((char *)pool_k + dst * rowb, (const char *)host_k + src * rowb, rowb);
      memcpy((char *)pool_v + dst * rowb, (const char *)host_v + src * rowb, rowb);
      if (host_bias && pool_bias) pool_bias[dst] = host_bias[src];
    }
}
