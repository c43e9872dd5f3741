/*
 * Reference checker for the rollout decode step (TEST INFRASTRUCTURE ONLY).
 *
 * Plain float64 loops over the logical token order of every sequence.  Nothing here is
 * blocked, fused, split or reordered, and nothing is shared with the GPU library: this file
 * is what the GPU results are compared against.  Only tests, the smoke check and the
 * CPU-baseline leg of the benchmark may load it; the product never calls it.
 *
 * What it follows.  The paper treats the inference backend as a black box (System
 * Implementation, Section 7) and only states that rollout is memory-bound on large KV caches
 * (Rollout-Training Disaggregation, Section 4.1), that every prompt is expanded into several
 * samples sharing its prefix (Parallel Sampling, Section 5.1) and that training uses GRPO
 * (Section 8.1), which consumes per-token log-probabilities.  It prints no formula for
 * either, so the definitions below are the textbook ones:
 *
 *   attention:  x_j = scale * <q, k_j>,  p_j = exp(x_j - max x) / sum_i exp(x_i - max x),
 *               out = sum_j p_j v_j                    over the L = P_g + S_s logical tokens
 *   log-prob:   y_v = logit_v / T,  out = y_tok - (max y + log sum_v exp(y_v - max y))
 *
 * Logical token j of sequence s (group g): j < P_g lives in the group's shared prefix, at
 * page prefix_table[g][j / 16], slot j % 16; otherwise with j' = j - P_g it lives at page
 * suffix_table[s][j' / 16], slot j' % 16 (a suffix always starts at slot 0 of its own page).
 * Query head h reads KV head h / (Hq / Hkv).
 *
 * Physical layout (the library's ABI, indexed here from its written definition):
 *   K[page][kv_head][slot][c]   at ((page*Hkv + kv_head)*16 + slot)*128 + c
 *   V[page][kv_head][c][slot]   at ((page*Hkv + kv_head)*128 + c)*16 + slot
 * bf16 values arrive as raw 16-bit patterns; widening to double is exact.
 *
 * Parity pins for every function here are in tests/test_oracle_*.py.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define PAGE 16
#define HD 128

static double bf16_to_double(uint16_t bits) {
  uint32_t u = ((uint32_t)bits) << 16;
  float f;
  memcpy(&f, &u, sizeof f);
  return (double)f;
}

/* address of the key / value element of one logical token */
static const uint16_t* key_row(const uint16_t* k_pages, int Hkv, int32_t page, int kvh, int slot) {
  return k_pages + (((size_t)page * Hkv + kvh) * PAGE + slot) * HD;
}
static double value_at(const uint16_t* v_pages, int Hkv, int32_t page, int kvh, int slot, int c) {
  return bf16_to_double(v_pages[(((size_t)page * Hkv + kvh) * HD + c) * PAGE + slot]);
}

/* page and slot of logical token j of sequence s */
static void locate(int j, int P, const int32_t* prow, const int32_t* srow, int32_t* page, int* slot) {
  if (j < P) {
    *page = prow[j / PAGE];
    *slot = j % PAGE;
  } else {
    int jj = j - P;
    *page = srow[jj / PAGE];
    *slot = jj % PAGE;
  }
}

/* One (sequence, query head): fills out[128]; if weights != NULL also the L softmax weights.
 * scratch must hold L doubles.  Returns L. */
static int attend_one(int s, int h, int Hq, int Hkv, const uint16_t* q, const uint16_t* k_pages,
                      const uint16_t* v_pages, const int32_t* ptab, int max_pp, const int32_t* stab,
                      int max_sp, const int32_t* plens, const int32_t* slens,
                      const int32_t* group_of_seq, double scale, double* out, double* scratch) {
  const int g = group_of_seq[s];
  const int kvh = h / (Hq / Hkv);
  const int P = plens[g], S = slens[s], L = P + S;
  const int32_t* prow = ptab + (size_t)g * max_pp;
  const int32_t* srow = stab + (size_t)s * max_sp;
  const uint16_t* qrow = q + ((size_t)s * Hq + h) * HD;
  for (int c = 0; c < HD; ++c) out[c] = 0.0;
  if (L == 0) return 0;
  double m = -INFINITY;
  for (int j = 0; j < L; ++j) {
    int32_t page; int slot;
    locate(j, P, prow, srow, &page, &slot);
    const uint16_t* kr = key_row(k_pages, Hkv, page, kvh, slot);
    double dot = 0.0;
    for (int c = 0; c < HD; ++c) dot += bf16_to_double(qrow[c]) * bf16_to_double(kr[c]);
    scratch[j] = scale * dot;
    if (scratch[j] > m) m = scratch[j];
  }
  double Z = 0.0;
  for (int j = 0; j < L; ++j) {
    scratch[j] = exp(scratch[j] - m);
    Z += scratch[j];
  }
  for (int j = 0; j < L; ++j) {
    int32_t page; int slot;
    locate(j, P, prow, srow, &page, &slot);
    const double p = scratch[j] / Z;
    scratch[j] = p;
    for (int c = 0; c < HD; ++c) out[c] += p * value_at(v_pages, Hkv, page, kvh, slot, c);
  }
  return L;
}

/* All sequences and heads.  out: double [NS][Hq][128].  threads <= 0 keeps the OpenMP
 * default; the loop over sequences is the only parallel one (timing convenience).
 * seq_begin/seq_end restrict the work to a slice of the sequences.  Returns the number of
 * threads used, or -1 on allocation failure. */
int oracle_decode_attn(int NS, int NG, int Hq, int Hkv, const uint16_t* q, const uint16_t* k_pages,
                       const uint16_t* v_pages, const int32_t* ptab, int max_pp,
                       const int32_t* stab, int max_sp, const int32_t* plens,
                       const int32_t* slens, const int32_t* group_of_seq, double scale,
                       double* out, int seq_begin, int seq_end, int threads) {
  (void)NG;
  int used = 1, fail = 0;
  if (seq_begin < 0) seq_begin = 0;
  if (seq_end > NS) seq_end = NS;
#ifdef _OPENMP
  if (threads > 0) omp_set_num_threads(threads);
#pragma omp parallel
  {
#pragma omp single
    used = omp_get_num_threads();
  }
#endif
#pragma omp parallel for schedule(dynamic, 1)
  for (int s = seq_begin; s < seq_end; ++s) {
    const int L = plens[group_of_seq[s]] + slens[s];
    double* scratch = (double*)malloc(sizeof(double) * (size_t)(L > 0 ? L : 1));
    if (!scratch) { fail = 1; continue; }
    for (int h = 0; h < Hq; ++h)
      attend_one(s, h, Hq, Hkv, q, k_pages, v_pages, ptab, max_pp, stab, max_sp, plens, slens,
                 group_of_seq, scale, out + ((size_t)s * Hq + h) * HD, scratch);
    free(scratch);
  }
  return fail ? -1 : used;
}

/* Softmax weights of one (sequence, head): weights must hold P_g + S_s doubles; out[128]. */
int oracle_attn_weights(int s, int h, int Hq, int Hkv, const uint16_t* q, const uint16_t* k_pages,
                        const uint16_t* v_pages, const int32_t* ptab, int max_pp,
                        const int32_t* stab, int max_sp, const int32_t* plens,
                        const int32_t* slens, const int32_t* group_of_seq, double scale,
                        double* out, double* weights) {
  return attend_one(s, h, Hq, Hkv, q, k_pages, v_pages, ptab, max_pp, stab, max_sp, plens, slens,
                    group_of_seq, scale, out, weights);
}

/* Per-row log-probability of the chosen token.  logits: bf16 bits [rows][vocab]. */
int oracle_token_logprobs(int rows, int vocab, const uint16_t* logits, const int32_t* tokens,
                          double temperature, double* out, int threads) {
  int used = 1;
#ifdef _OPENMP
  if (threads > 0) omp_set_num_threads(threads);
#pragma omp parallel
  {
#pragma omp single
    used = omp_get_num_threads();
  }
#endif
#pragma omp parallel for schedule(static)
  for (int r = 0; r < rows; ++r) {
    const uint16_t* x = logits + (size_t)r * vocab;
    double m = -INFINITY;
    for (int v = 0; v < vocab; ++v) {
      double y = bf16_to_double(x[v]) / temperature;
      if (y > m) m = y;
    }
    double Z = 0.0;
    for (int v = 0; v < vocab; ++v) Z += exp(bf16_to_double(x[v]) / temperature - m);
    const double lse = m + log(Z);
    out[r] = bf16_to_double(x[tokens[r]]) / temperature - lse;
  }
  return used;
}
