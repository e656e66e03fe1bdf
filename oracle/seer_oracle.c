/*
 * CPU oracle for the SeerAttention-R decode hot path.  TEST INFRASTRUCTURE ONLY:
 * it defines what the GPU library must compute and is called from tests/, the
 * smoke check and the bench's cpu_baseline leg - never from the product path.
 * It shares no code, header, table or helper with the HIP library.
 *
 * Everything is the plain definition, in fp64, reading the bf16 inputs exactly
 * (a bf16 value is the upper 16 bits of an IEEE fp32 value):
 *
 *   gate score      s_j = sum_c q_gate[c] * k_gate[j][c]      (Eq. 1c, before the
 *                   softmax; Sec. 3.1 notes that top-k needs no softmax)
 *   token budget    block budget = token budget / block size, keep the top-k
 *                   scored blocks (Sec. 3.1), lowest index first among equals
 *   threshold       S = softmax_j(s_j / sqrt(d_gate)) (Eq. 1c); keep S_j > tau
 *                   (Sec. 3.1)
 *   last block      while seqlen is not a multiple of the block size the newest
 *                   cache entry is stale, so the last block is always kept
 *                   (Sec. 3.2, Fig. 3)
 *   sparse decode   softmax(scale * q.K^T) V restricted to the tokens of the
 *                   selected blocks, one block list shared by the query heads of
 *                   a kv head; invalid list entries are skipped (Sec. 3.3)
 *
 * No blocking, no online rescaling, no split-K: two passes over the selected
 * tokens (max, then sums), sums taken in index order.
 *
 *   ground truth    (training side, Sec. 2.3) causal softmax attention of every query
 *                   position; per query row the probabilities are max-pooled over the
 *                   keys of each block (column-wise 1-D pooling), then over the query
 *                   heads that share a kv head, then divided by their sum over blocks
 *
 * Pins (tests/test_oracle_pins.py): dense attention computed independently when all
 * blocks are selected; closed forms for identical keys; needle keys; -inf masking
 * equivalence; lse partition algebra; brute-force subset enumeration for the top-k;
 * exact rational arithmetic for the score; softmax invariants for the threshold.
 * Ground truth (tests/test_oracle_gt_pins.py): zero queries (uniform rows: prefix means and
 * 1 / #visible-blocks in closed form); needle keys (one-hot rows); agreement of out / lse with
 * the decode oracle run per position; a grouped call equals the normalised head-wise maximum of
 * single-head calls; sum-to-one, causality and permutation properties.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static double bf16_value(uint16_t bits) {
  uint32_t u = (uint32_t)bits << 16;
  float f;
  memcpy(&f, &u, sizeof f);
  return (double)f;
}

int oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* ------------------------------------------------------------------ gate */

/* Scores of the full blocks of one (sequence, kv head).  kc rows are kc_stride_block
 * elements apart.  scores[j] for j < nfull. */
static void gate_scores_group(const uint16_t* qg, const uint16_t* kc, int64_t kc_stride_block,
                              int dg, int nfull, double* scores) {
  for (int j = 0; j < nfull; ++j) {
    const uint16_t* row = kc + (int64_t)j * kc_stride_block;
    double s = 0.0;
    for (int c = 0; c < dg; ++c) s += bf16_value(qg[c]) * bf16_value(row[c]);
    scores[j] = s;
  }
}

typedef struct { double s; int j; } scored_t;

/* higher score first; among equal scores the lower block index first */
static int by_score_then_index(const void* a, const void* b) {
  const scored_t* x = (const scored_t*)a;
  const scored_t* y = (const scored_t*)b;
  if (x->s > y->s) return -1;
  if (x->s < y->s) return 1;
  return (x->j > y->j) - (x->j < y->j);
}

static int by_int(const void* a, const void* b) {
  int x = *(const int*)a, y = *(const int*)b;
  return (x > y) - (x < y);
}

/*
 * mode 0: token budget.  k = budget_blocks[i] if given, else ceil(budget_tokens / b);
 *         clamped to [0, min(nb, max_sel)].  With a partial last block, that block takes
 *         one of the k slots and the other k-1 go to the best full blocks.
 * mode 1: threshold on the softmax over full blocks; the partial last block is added.
 * mode 2: top-p on the same softmax (threshold carries p); the partial last block is added.
 * Output per group: ascending block indices, padded with -1 to max_sel; count in nblk.
 * scores_out (optional, [B,Hkv,nb_max]) receives the raw scores (NaN where not computed).
 * Returns 0, or -1 when a threshold selection does not fit max_sel.
 */
int oracle_gate_select(const uint16_t* q_gate, const uint16_t* kc_cache, int64_t kc_stride_batch,
                       int64_t kc_stride_head, int64_t kc_stride_block, const int32_t* seqlens, int B,
                       int Hkv, int Dg, int nb_max, int block_size, int mode, int32_t budget_tokens,
                       const int32_t* budget_blocks, double threshold, int32_t* block_idx,
                       int32_t* nblk, int max_sel, double* scores_out) {
  int failed = 0;
#pragma omp parallel for collapse(2) schedule(dynamic)
  for (int i = 0; i < B; ++i) {
    for (int h = 0; h < Hkv; ++h) {
      const int64_t grp = (int64_t)i * Hkv + h;
      int32_t* out = block_idx + grp * max_sel;
      for (int p = 0; p < max_sel; ++p) out[p] = -1;
      nblk[grp] = 0;
      int S = seqlens[i];
      if (S < 0) S = 0;
      int nfull = S / block_size;
      int nb = (S + block_size - 1) / block_size;
      if (nb > nb_max) { nb = nb_max; if (nfull > nb) nfull = nb; }
      const int partial = nb > nfull;

      double* scores = (double*)malloc(sizeof(double) * (size_t)(nfull > 0 ? nfull : 1));
      gate_scores_group(q_gate + grp * Dg, kc_cache + i * kc_stride_batch + h * kc_stride_head,
                        kc_stride_block, Dg, nfull, scores);
      if (scores_out) {
        double* so = scores_out + grp * nb_max;
        for (int j = 0; j < nb_max; ++j) so[j] = j < nfull ? scores[j] : NAN;
      }

      int* sel = (int*)malloc(sizeof(int) * (size_t)(nb > 0 ? nb : 1));
      int n = 0;
      if (mode == 0) {
        int64_t k = budget_blocks ? (int64_t)budget_blocks[i]
                                  : ((int64_t)budget_tokens + block_size - 1) / block_size;
        if (k < 0) k = 0;
        if (k > nb) k = nb;
        if (k > max_sel) k = max_sel;
        int from_full = (int)k;
        if (partial && k > 0) from_full = (int)k - 1;
        if (from_full > nfull) from_full = nfull;
        scored_t* order = (scored_t*)malloc(sizeof(scored_t) * (size_t)(nfull > 0 ? nfull : 1));
        for (int j = 0; j < nfull; ++j) { order[j].s = scores[j]; order[j].j = j; }
        qsort(order, (size_t)nfull, sizeof(scored_t), by_score_then_index);
        for (int r = 0; r < from_full; ++r) sel[n++] = order[r].j;
        if (partial && k > 0) sel[n++] = nb - 1;
        free(order);
      } else if (mode == 1) {
        if (nfull > 0) {
          const double inv = 1.0 / sqrt((double)Dg);
          double m = -INFINITY;
          for (int j = 0; j < nfull; ++j) { double x = scores[j] * inv; if (x > m) m = x; }
          double Z = 0.0;
          for (int j = 0; j < nfull; ++j) Z += exp(scores[j] * inv - m);
          for (int j = 0; j < nfull; ++j) {
            double Sj = exp(scores[j] * inv - m) / Z;
            if (Sj > threshold) sel[n++] = j;
          }
        }
        if (partial) sel[n++] = nb - 1;
      } else {
        /* top-p (nucleus) selection, named as the way to adaptive sparsity in Sec. 6.2: walk the
         * blocks from the highest score down (equal scores: lower index first) and keep them until
         * their accumulated gate probability reaches p; at least one block is kept.  p >= 1 asks
         * for the whole mass: every softmax probability is positive, so in exact arithmetic only
         * the set of all full blocks has it - that case is decided here and not left to whether a
         * rounded running sum happens to touch 1.0 before the last block. */
        if (nfull > 0) {
          const double inv = 1.0 / sqrt((double)Dg);
          double m = -INFINITY;
          for (int j = 0; j < nfull; ++j) { double x = scores[j] * inv; if (x > m) m = x; }
          double Z = 0.0;
          for (int j = 0; j < nfull; ++j) Z += exp(scores[j] * inv - m);
          scored_t* order = (scored_t*)malloc(sizeof(scored_t) * (size_t)nfull);
          for (int j = 0; j < nfull; ++j) { order[j].s = scores[j]; order[j].j = j; }
          qsort(order, (size_t)nfull, sizeof(scored_t), by_score_then_index);
          double cum = 0.0;
          for (int r = 0; r < nfull; ++r) {
            sel[n++] = order[r].j;
            cum += exp(order[r].s * inv - m) / Z;
            if (threshold < 1.0 && cum >= threshold) break;
          }
          free(order);
        }
        if (partial) sel[n++] = nb - 1;
      }
      qsort(sel, (size_t)n, sizeof(int), by_int);
      if (n > max_sel) {
#pragma omp atomic write
        failed = 1;
        n = max_sel;
      }
      for (int p = 0; p < n; ++p) out[p] = sel[p];
      nblk[grp] = n;
      free(sel);
      free(scores);
    }
  }
  return failed ? -1 : 0;
}

/* ---------------------------------------------------------------- decode */

typedef struct {
  const uint16_t* k;
  const uint16_t* v;
  int64_t stride_seq;   /* elements between sequences (contiguous) or pages (paged) */
  int64_t stride_head;
  int64_t stride_token;
  const int32_t* page_table; /* [B, max_pages] or NULL */
  int32_t max_pages;
  int32_t page_size;
} oracle_kv_t;

static int64_t token_offset(const oracle_kv_t* kv, int i, int hk, int64_t t) {
  if (kv->page_table) {
    int64_t page = kv->page_table[(int64_t)i * kv->max_pages + t / kv->page_size];
    return page * kv->stride_seq + (int64_t)hk * kv->stride_head + (t % kv->page_size) * kv->stride_token;
  }
  return (int64_t)i * kv->stride_seq + (int64_t)hk * kv->stride_head + t * kv->stride_token;
}

/*
 * Attention of every query head over the tokens of the listed blocks.
 * block_idx == NULL: all blocks (dense).  Otherwise the first min(nblk, max_sel) entries of
 * the group's list are used; entries < 0 or >= ceil(S/b) are skipped.
 * out [B,Hq,d] fp64, lse [B,Hq] fp64 (natural log of sum exp(scale*q.k)); an empty token
 * set gives out = 0 and lse = -inf.
 * group_filter (optional, [B*Hkv] bytes): groups with 0 are left untouched.
 */
int oracle_sparse_decode_multi(const uint16_t* q, const oracle_kv_t* kv, const int32_t* seqlens,
                               const int32_t* block_idx, const int32_t* nblk, int max_sel, int B, int T,
                               int Hq, int Hkv, int d, int block_size, float scale, double* out, double* lse,
                               const uint8_t* group_filter);

int oracle_sparse_decode(const uint16_t* q, const oracle_kv_t* kv, const int32_t* seqlens,
                         const int32_t* block_idx, const int32_t* nblk, int max_sel, int B, int Hq,
                         int Hkv, int d, int block_size, float scale, double* out, double* lse,
                         const uint8_t* group_filter) {
  if (Hkv <= 0 || Hq % Hkv) return -1;
  const int g = Hq / Hkv;
#pragma omp parallel for collapse(2) schedule(dynamic)
  for (int i = 0; i < B; ++i) {
    for (int hk = 0; hk < Hkv; ++hk) {
      const int64_t grp = (int64_t)i * Hkv + hk;
      if (group_filter && !group_filter[grp]) continue;
      int S = seqlens[i];
      if (S < 0) S = 0;
      const int nb = (S + block_size - 1) / block_size;

      /* token list of the group */
      int nlist = block_idx ? nblk[grp] : nb;
      if (nlist < 0) nlist = 0;
      if (block_idx && nlist > max_sel) nlist = max_sel;
      int64_t cap = (int64_t)nlist * block_size;
      int64_t* toks = (int64_t*)malloc(sizeof(int64_t) * (size_t)(cap > 0 ? cap : 1));
      int64_t nt = 0;
      for (int p = 0; p < nlist; ++p) {
        int j = block_idx ? block_idx[grp * max_sel + p] : p;
        if (j < 0 || j >= nb) continue;
        int64_t t0 = (int64_t)j * block_size;
        int64_t t1 = t0 + block_size;
        if (t1 > S) t1 = S;
        for (int64_t t = t0; t < t1; ++t) toks[nt++] = t;
      }

      double* x = (double*)malloc(sizeof(double) * (size_t)(nt > 0 ? nt : 1));
      for (int hh = 0; hh < g; ++hh) {
        const int h = hk * g + hh;
        const uint16_t* qrow = q + ((int64_t)i * Hq + h) * d;
        double* orow = out + ((int64_t)i * Hq + h) * d;
        for (int c = 0; c < d; ++c) orow[c] = 0.0;
        if (nt == 0) { lse[(int64_t)i * Hq + h] = -INFINITY; continue; }
        double m = -INFINITY;
        for (int64_t r = 0; r < nt; ++r) {
          const uint16_t* krow = kv->k + token_offset(kv, i, hk, toks[r]);
          double dot = 0.0;
          for (int c = 0; c < d; ++c) dot += bf16_value(qrow[c]) * bf16_value(krow[c]);
          x[r] = (double)scale * dot;
          if (x[r] > m) m = x[r];
        }
        double Z = 0.0;
        for (int64_t r = 0; r < nt; ++r) Z += exp(x[r] - m);
        const double l = m + log(Z);
        for (int64_t r = 0; r < nt; ++r) {
          const double p = exp(x[r] - l);
          const uint16_t* vrow = kv->v + token_offset(kv, i, hk, toks[r]);
          for (int c = 0; c < d; ++c) orow[c] += p * bf16_value(vrow[c]);
        }
        lse[(int64_t)i * Hq + h] = l;
      }
      free(x);
      free(toks);
    }
  }
  return 0;
}

/* ------------------------------------------------------- AttnGate front-end (Eq. 1a, 1b) */

/* fp64 -> bf16 bits, round to nearest even (through an exactly representable fp32 when possible;
 * the double is first rounded to fp32 with the FPU's round-to-nearest-even, then to bf16; to avoid
 * double rounding the bf16 rounding is done directly on the double's value). */
static uint16_t f64_to_bf16_bits(double x) {
  if (x != x) return 0x7fc0;
  float f = (float)x;                 /* candidate; may suffer double rounding, fixed below */
  uint32_t u;
  memcpy(&u, &f, 4);
  uint32_t lo = u & 0xffff0000u;      /* bf16 neighbours of the fp32 candidate */
  uint32_t hi = lo + 0x10000u;
  float flo, fhi;
  memcpy(&flo, &lo, 4);
  memcpy(&fhi, &hi, 4);
  /* flo and fhi bracket x in magnitude (same sign); pick the nearer in exact double arithmetic */
  double dlo = fabs(x - (double)flo), dhi = fabs((double)fhi - x);
  if (isinf(fhi) && !isinf(x)) { /* overflow boundary: keep IEEE behaviour of the candidate */ }
  uint32_t pick;
  if (dlo < dhi) pick = lo;
  else if (dhi < dlo) pick = hi;
  else pick = ((lo >> 16) & 1u) ? hi : lo;   /* tie: even mantissa */
  return (uint16_t)(pick >> 16);
}

/* Rotary embedding in the rotate-half convention of the LLaMA/Qwen family: feature c < D/2 is
 * paired with feature c + D/2; cos_t/sin_t are the caller's tables for this position [D/2]. */
static void rope_rotate_half(double* y, int D, const float* cos_t, const float* sin_t) {
  const int half = D / 2;
  for (int c = 0; c < half; ++c) {
    const double a = y[c], b = y[c + half];
    const double co = (double)cos_t[c], si = (double)sin_t[c];
    y[c] = a * co - b * si;
    y[c + half] = b * co + a * si;
  }
}

/*
 * Q branch of the AttnGate (Eq. 1a): the g pre-RoPE query heads of a kv head are concatenated
 * (head-major) into one vector of g*d features, multiplied by that kv head's weight matrix
 * Wq[h] (Dg x g*d, row-major) and rotated at the position of the current token (seqlens[i] - 1).
 * q_nope bf16 [B,Hq,d]; wq bf16 [Hkv,Dg,g*d]; rope tables fp32 [n_pos, Dg/2].
 * out_f64 [B,Hkv,Dg] unrounded, out_bf16 [B,Hkv,Dg] rounded bits (either may be NULL).
 */
int oracle_gate_q(const uint16_t* q_nope, const uint16_t* wq, const float* rope_cos, const float* rope_sin,
                  int n_pos, const int32_t* seqlens, int B, int Hq, int Hkv, int d, int Dg, double* out_f64,
                  uint16_t* out_bf16) {
  if (Hkv <= 0 || Hq % Hkv || Dg % 2) return -1;
  const int g = Hq / Hkv, gd = g * d;
  int bad = 0;
#pragma omp parallel for collapse(2)
  for (int i = 0; i < B; ++i)
    for (int h = 0; h < Hkv; ++h) {
      int pos = seqlens[i] - 1;
      if (pos < 0) pos = 0;
      if (pos >= n_pos) { bad = 1; pos = n_pos - 1; }
      const uint16_t* x = q_nope + ((int64_t)i * Hq + (int64_t)h * g) * d;   /* g*d contiguous */
      double* y = (double*)malloc(sizeof(double) * (size_t)Dg);
      for (int o = 0; o < Dg; ++o) {
        const uint16_t* wrow = wq + ((int64_t)h * Dg + o) * gd;
        double s = 0.0;
        for (int c = 0; c < gd; ++c) s += bf16_value(wrow[c]) * bf16_value(x[c]);
        y[o] = s;
      }
      rope_rotate_half(y, Dg, rope_cos + (int64_t)pos * (Dg / 2), rope_sin + (int64_t)pos * (Dg / 2));
      for (int o = 0; o < Dg; ++o) {
        const int64_t at = ((int64_t)i * Hkv + h) * Dg + o;
        if (out_f64) out_f64[at] = y[o];
        if (out_bf16) out_bf16[at] = f64_to_bf16_bits(y[o]);
      }
      free(y);
    }
  return bad ? -2 : 0;
}

/*
 * K branch of the AttnGate (Eq. 1b) = one entry of the K Compression Cache (Sec. 3.2): the b
 * pre-RoPE keys of block j are max-, min- and average-pooled over the tokens, the three results
 * concatenated ([max | min | avg], 3d features), multiplied by Wk[h] (Dg x 3d, row-major) and
 * rotated at the position of the block's first token (j*b).
 * k_nope uses the KV-cache addressing (kv->k is read; kv->v ignored).  Blocks
 * [block_begin[i], block_end[i]) of every sequence are computed (clamped to the full blocks of the
 * sequence, seqlens[i] / b, and to nb_max).  out_f64 / out_bf16: [B,Hkv,nb_max,Dg], entries of
 * blocks outside the range are left untouched.
 */
int oracle_kc_update(const oracle_kv_t* kv, const uint16_t* wk, const float* rope_cos, const float* rope_sin,
                     int n_pos, const int32_t* seqlens, const int32_t* block_begin, const int32_t* block_end,
                     int B, int Hkv, int d, int Dg, int nb_max, int block_size, double* out_f64,
                     uint16_t* out_bf16) {
  if (Dg % 2) return -1;
  int bad = 0;
#pragma omp parallel for collapse(2) schedule(dynamic)
  for (int i = 0; i < B; ++i)
    for (int h = 0; h < Hkv; ++h) {
      int S = seqlens[i];
      if (S < 0) S = 0;
      int nfull = S / block_size;
      if (nfull > nb_max) nfull = nb_max;
      int j0 = block_begin ? block_begin[i] : 0, j1 = block_end ? block_end[i] : nfull;
      if (j0 < 0) j0 = 0;
      if (j1 > nfull) j1 = nfull;
      double* u = (double*)malloc(sizeof(double) * (size_t)(3 * d));
      double* y = (double*)malloc(sizeof(double) * (size_t)Dg);
      for (int j = j0; j < j1; ++j) {
        for (int c = 0; c < d; ++c) { u[c] = -INFINITY; u[d + c] = INFINITY; u[2 * d + c] = 0.0; }
        for (int t = 0; t < block_size; ++t) {
          const uint16_t* row = kv->k + token_offset(kv, i, h, (int64_t)j * block_size + t);
          for (int c = 0; c < d; ++c) {
            const double x = bf16_value(row[c]);
            if (x > u[c]) u[c] = x;
            if (x < u[d + c]) u[d + c] = x;
            u[2 * d + c] += x;
          }
        }
        for (int c = 0; c < d; ++c) u[2 * d + c] /= (double)block_size;
        for (int o = 0; o < Dg; ++o) {
          const uint16_t* wrow = wk + ((int64_t)h * Dg + o) * (3 * d);
          double s = 0.0;
          for (int c = 0; c < 3 * d; ++c) s += bf16_value(wrow[c]) * u[c];
          y[o] = s;
        }
        int64_t pos = (int64_t)j * block_size;
        if (pos >= n_pos) { bad = 1; pos = n_pos - 1; }
        rope_rotate_half(y, Dg, rope_cos + pos * (Dg / 2), rope_sin + pos * (Dg / 2));
        for (int o = 0; o < Dg; ++o) {
          const int64_t at = (((int64_t)i * Hkv + h) * nb_max + j) * Dg + o;
          if (out_f64) out_f64[at] = y[o];
          if (out_bf16) out_bf16[at] = f64_to_bf16_bits(y[o]);
        }
      }
      free(u);
      free(y);
    }
  return bad ? -2 : 0;
}


/*
 * Several new tokens per sequence in one step (the multi-token / speculative decoding direction of
 * Sec. 6.3): the T queries of sequence i are its last T tokens, at positions S-T .. S-1 (S =
 * seqlens[i] counts them); query t attends the cached tokens up to and including its own position,
 * restricted to the listed blocks - one list per (sequence, kv head), shared by the T queries.
 * q [B,T,Hq,d]; out [B,T,Hq,d]; lse [B,T,Hq].  Query t is exactly a single-token decode of a
 * sequence of length S-T+1+t with the same list.
 */
int oracle_sparse_decode_multi(const uint16_t* q, const oracle_kv_t* kv, const int32_t* seqlens,
                               const int32_t* block_idx, const int32_t* nblk, int max_sel, int B, int T,
                               int Hq, int Hkv, int d, int block_size, float scale, double* out, double* lse,
                               const uint8_t* group_filter) {
  if (Hkv <= 0 || Hq % Hkv || T <= 0) return -1;
  const int g = Hq / Hkv;
#pragma omp parallel for collapse(2) schedule(dynamic)
  for (int i = 0; i < B; ++i) {
    for (int hk = 0; hk < Hkv; ++hk) {
      const int64_t grp = (int64_t)i * Hkv + hk;
      if (group_filter && !group_filter[grp]) continue;
      int S = seqlens[i];
      if (S < 0) S = 0;
      const int nb = (S + block_size - 1) / block_size;
      int nlist = block_idx ? nblk[grp] : nb;
      if (nlist < 0) nlist = 0;
      if (block_idx && nlist > max_sel) nlist = max_sel;
      for (int t = 0; t < T; ++t) {
        const int64_t limit = (int64_t)S - (T - 1 - t);        /* tokens [0, limit) are visible to query t */
        for (int hh = 0; hh < g; ++hh) {
          const int h = hk * g + hh;
          const int64_t row = ((int64_t)i * T + t) * Hq + h;
          const uint16_t* qrow = q + row * d;
          double* orow = out + row * d;
          for (int c = 0; c < d; ++c) orow[c] = 0.0;
          /* pass 1: max; pass 2: sums (token lists are short enough to recompute the logits) */
          double m = -INFINITY, Z = 0.0;
          for (int pass = 0; pass < 2; ++pass) {
            for (int p = 0; p < nlist; ++p) {
              const int j = block_idx ? block_idx[grp * max_sel + p] : p;
              if (j < 0 || j >= nb) continue;
              int64_t t1 = (int64_t)(j + 1) * block_size;
              if (t1 > limit) t1 = limit;
              for (int64_t tok = (int64_t)j * block_size; tok < t1; ++tok) {
                const int64_t off = token_offset(kv, i, hk, tok);
                double dot = 0.0;
                for (int c = 0; c < d; ++c) dot += bf16_value(qrow[c]) * bf16_value(kv->k[off + c]);
                const double x = (double)scale * dot;
                if (pass == 0) { if (x > m) m = x; }
                else {
                  const double e = exp(x - m);
                  Z += e;
                  for (int c = 0; c < d; ++c) orow[c] += e * bf16_value(kv->v[off + c]);
                }
              }
            }
            if (pass == 0 && m == -INFINITY) break;
          }
          if (m == -INFINITY) { lse[row] = -INFINITY; continue; }
          for (int c = 0; c < d; ++c) orow[c] /= Z;
          lse[row] = m + log(Z);
        }
      }
    }
  }
  return 0;
}

/* ------------------------------------------------ distillation ground truth (Sec. 2.3) */

/*
 * Dense causal attention over whole sequences plus the AttnGate's training target.
 * q [B,T,Hq,d] bf16; keys / values addressed through kv (token s of sequence i, kv head hk);
 * seqlens [B] or NULL (all T): query rows t >= S_i are padding (out = 0, lse = -inf, gt = 0).
 * For query t < S_i and head h (kv head hk = h / g):
 *     x_s = scale * q.k_s, s = 0..t;   P_s = exp(x_s - lse),  lse = log sum_s exp(x_s)
 *     out = sum_s P_s v_s
 *     c[h][j] = max of P_s over the keys s <= t of block j          (1-D column pooling)
 *     r[hk][j] = max of c[h][j] over the g heads of kv head hk      (pooling inside the GQA group)
 *     gt[hk][j] = r[hk][j] / sum_j' r[hk][j']                       (normalised to sum 1)
 * Blocks that start after t hold no visible key: gt = 0 there.
 * out [B,T,Hq,d], lse [B,T,Hq], gt [B,Hkv,T,nb] with nb = ceil(T / block_size); all fp64.
 */
int oracle_attn_ground_truth(const uint16_t* q, const oracle_kv_t* kv, const int32_t* seqlens, int B, int T,
                             int Hq, int Hkv, int d, int block_size, float scale, double* out, double* lse,
                             double* gt) {
  if (Hkv <= 0 || Hq % Hkv || T <= 0 || block_size <= 0) return -1;
  const int g = Hq / Hkv;
  const int nb = (T + block_size - 1) / block_size;
#pragma omp parallel for collapse(3) schedule(dynamic)
  for (int i = 0; i < B; ++i) {
    for (int hk = 0; hk < Hkv; ++hk) {
      for (int t = 0; t < T; ++t) {
        int S = seqlens ? seqlens[i] : T;
        if (S > T) S = T;
        double* grow = gt + (((int64_t)i * Hkv + hk) * T + t) * nb;
        for (int j = 0; j < nb; ++j) grow[j] = 0.0;
        if (t >= S) {
          for (int hh = 0; hh < g; ++hh) {
            const int64_t row = ((int64_t)i * T + t) * Hq + hk * g + hh;
            for (int c = 0; c < d; ++c) out[row * d + c] = 0.0;
            lse[row] = -INFINITY;
          }
          continue;
        }
        double* x = (double*)malloc(sizeof(double) * (size_t)(t + 1));
        for (int hh = 0; hh < g; ++hh) {
          const int64_t row = ((int64_t)i * T + t) * Hq + hk * g + hh;
          const uint16_t* qrow = q + row * d;
          double m = -INFINITY;
          for (int s = 0; s <= t; ++s) {
            const uint16_t* krow = kv->k + token_offset(kv, i, hk, s);
            double dot = 0.0;
            for (int c = 0; c < d; ++c) dot += bf16_value(qrow[c]) * bf16_value(krow[c]);
            x[s] = (double)scale * dot;
            if (x[s] > m) m = x[s];
          }
          double Z = 0.0;
          for (int s = 0; s <= t; ++s) Z += exp(x[s] - m);
          const double l = m + log(Z);
          double* orow = out + row * d;
          for (int c = 0; c < d; ++c) orow[c] = 0.0;
          for (int s = 0; s <= t; ++s) {
            const double p = exp(x[s] - l);
            const uint16_t* vrow = kv->v + token_offset(kv, i, hk, s);
            for (int c = 0; c < d; ++c) orow[c] += p * bf16_value(vrow[c]);
            const int j = s / block_size;
            if (p > grow[j]) grow[j] = p;          /* max over the block's keys and over the heads */
          }
          lse[row] = l;
        }
        double total = 0.0;
        for (int j = 0; j < nb; ++j) total += grow[j];
        for (int j = 0; j < nb; ++j) grow[j] /= total;
        free(x);
      }
    }
  }
  return 0;
}
