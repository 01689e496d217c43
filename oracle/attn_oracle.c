/*
 * CPU oracle for exact softmax attention (causal, or causal with full-attention spans) and its gradients.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the product path may call, link or load
 * this file; it exists to check the HIP kernels and to serve as the timed CPU
 * baseline of the benchmark.  It shares no code with the HIP path.
 *
 * What it computes is the plain definition, per unsharded sequence, with no
 * chunking, no partial results and no merge:
 *
 *   paper Eq. 1 (Sec. 3.1):  Attn(Q,K,V) = softmax(Q K^T / sqrt(d_k)) V
 *   paper Sec. 4.3:          language models use the causal mask, i.e. query i of a
 *                            sequence sees keys j <= i of the same sequence only;
 *   paper Sec. 4.3 (time estimation, before Eq. 8): multimodal models give SOME tokens full
 *                            attention.  Reading: tokens are marked with a span id (span_id[t] >= 0,
 *                            -1 = unmarked); two tokens of one sequence with the same span id see each
 *                            other in both directions, every other pair is causal.  span_id == NULL
 *                            is the plain causal mask.
 *
 * Inputs are bf16 bit patterns (uint16), widened exactly to double; every sum is
 * carried in double.  Layouts: Q, dO [T, Hq, D]; K, V [T, Hkv, D]; T = all packed
 * tokens; cu_seqlens[n_seqs+1] gives each sequence's first token.  Query head h
 * reads KV head h / (Hq/Hkv).  LSE is the natural log of the sum of exp of the
 * scaled scores.
 *
 * All three entry points take an explicit list of query rows (global token ids),
 * so a caller can ask for one rank's rows only:
 *   fwd:  O, LSE for the listed rows
 *   dq:   dQ for the listed rows
 *   dkv:  dK, dV summed over the listed query rows only (that rank's partial)
 * Backward of loss = sum(O * dO):
 *   p_ij = exp(s_ij - LSE_i),  Delta_i = sum_c dO_ic O_ic,  dP_ij = dO_i . V_j,
 *   dS_ij = p_ij (dP_ij - Delta_i),
 *   dQ_i = scale sum_j dS_ij K_j,  dK_j = scale sum_i dS_ij Q_i,  dV_j = sum_i p_ij dO_i.
 *
 * Pins (tests, CPU only): explicit LxL softmax in numpy, closed forms for constant
 * keys, finite differences, torch float64 autograd on one sequence, row-sum
 * invariants.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static inline double bf(uint16_t b) {
  uint32_t u = ((uint32_t)b) << 16;
  float f;
  memcpy(&f, &u, 4);
  return (double)f;
}

/* index of the sequence that holds global token t */
static int seq_of(const int32_t* cu, int n_seqs, int64_t t) {
  int lo = 0, hi = n_seqs - 1;
  while (lo < hi) {
    int mid = (lo + hi + 1) / 2;
    if (cu[mid] <= t) lo = mid; else hi = mid - 1;
  }
  return lo;
}

/* the mask, by definition: i, j are positions inside the sequence that starts at global token t0 */
static int visible(const int32_t* span_id, int64_t t0, int64_t i, int64_t j) {
  if (j <= i) return 1;
  return span_id && span_id[t0 + i] >= 0 && span_id[t0 + i] == span_id[t0 + j];
}

static double dot_bf(const uint16_t* a, const uint16_t* b, int D) {
  double s = 0.0;
  for (int c = 0; c < D; ++c) s += bf(a[c]) * bf(b[c]);
  return s;
}

/* O [n_rows, Hq, D] and LSE [n_rows, Hq] (row-major in the order of `rows`). */
void oracle_attn_fwd(const uint16_t* q, const uint16_t* k, const uint16_t* v,
                     const int32_t* cu_seqlens, int n_seqs, int hq, int hkv, int D,
                     double scale, const int32_t* span_id, const int64_t* rows, int64_t n_rows,
                     double* O, double* LSE) {
  const int G = hq / hkv;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
  for (int64_t r = 0; r < n_rows; ++r) {
    for (int h = 0; h < hq; ++h) {
      const int64_t t = rows[r];
      const int n = seq_of(cu_seqlens, n_seqs, t);
      const int64_t t0 = cu_seqlens[n];
      const int64_t L = cu_seqlens[n + 1] - t0;
      const int64_t i = t - t0;
      const int g = h / G;
      const uint16_t* qi = q + (t * hq + h) * (int64_t)D;
      double* s = (double*)malloc(sizeof(double) * (size_t)L);
      double m = -INFINITY;
      for (int64_t j = 0; j < L; ++j) {
        if (!visible(span_id, t0, i, j)) continue;
        s[j] = scale * dot_bf(qi, k + ((t0 + j) * hkv + g) * (int64_t)D, D);
        if (s[j] > m) m = s[j];
      }
      double l = 0.0;
      for (int64_t j = 0; j < L; ++j)
        if (visible(span_id, t0, i, j)) l += exp(s[j] - m);
      double* o = O + (r * hq + h) * (int64_t)D;
      for (int c = 0; c < D; ++c) o[c] = 0.0;
      for (int64_t j = 0; j < L; ++j) {
        if (!visible(span_id, t0, i, j)) continue;
        const double p = exp(s[j] - m) / l;
        const uint16_t* vj = v + ((t0 + j) * hkv + g) * (int64_t)D;
        for (int c = 0; c < D; ++c) o[c] += p * bf(vj[c]);
      }
      LSE[r * hq + h] = m + log(l);
      free(s);
    }
  }
}

/* dQ [n_rows, Hq, D].  O, LSE are the oracle's own forward results for the same rows. */
void oracle_attn_dq(const uint16_t* q, const uint16_t* k, const uint16_t* v, const uint16_t* d_o,
                    const int32_t* cu_seqlens, int n_seqs, int hq, int hkv, int D,
                    double scale, const int32_t* span_id, const int64_t* rows, int64_t n_rows,
                    const double* O, const double* LSE, double* dQ) {
  const int G = hq / hkv;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
  for (int64_t r = 0; r < n_rows; ++r) {
    for (int h = 0; h < hq; ++h) {
      const int64_t t = rows[r];
      const int n = seq_of(cu_seqlens, n_seqs, t);
      const int64_t t0 = cu_seqlens[n];
      const int64_t L = cu_seqlens[n + 1] - t0;
      const int64_t i = t - t0;
      const int g = h / G;
      const uint16_t* qi = q + (t * hq + h) * (int64_t)D;
      const uint16_t* doi = d_o + (t * hq + h) * (int64_t)D;
      const double* oi = O + (r * hq + h) * (int64_t)D;
      double delta = 0.0;
      for (int c = 0; c < D; ++c) delta += bf(doi[c]) * oi[c];
      double* dq = dQ + (r * hq + h) * (int64_t)D;
      for (int c = 0; c < D; ++c) dq[c] = 0.0;
      for (int64_t j = 0; j < L; ++j) {
        if (!visible(span_id, t0, i, j)) continue;
        const uint16_t* kj = k + ((t0 + j) * hkv + g) * (int64_t)D;
        const uint16_t* vj = v + ((t0 + j) * hkv + g) * (int64_t)D;
        const double p = exp(scale * dot_bf(qi, kj, D) - LSE[r * hq + h]);
        const double dp = dot_bf(doi, vj, D);
        const double ds = p * (dp - delta);
        for (int c = 0; c < D; ++c) dq[c] += scale * ds * bf(kj[c]);
      }
    }
  }
}

/* dK, dV [n_keys, Hkv, D] for the listed keys (global token ids; keys == NULL means all T
 * tokens in order): sums over the listed query rows only.  Parallel over keys, so every
 * output element has a single writer. */
void oracle_attn_dkv(const uint16_t* q, const uint16_t* k, const uint16_t* v, const uint16_t* d_o,
                     const int32_t* cu_seqlens, int n_seqs, int64_t T, int hq, int hkv, int D,
                     double scale, const int32_t* span_id, const int64_t* rows, int64_t n_rows,
                     const double* O, const double* LSE, const int64_t* keys, int64_t n_keys,
                     double* dK, double* dV) {
  const int G = hq / hkv;
  /* Delta per (row, head) once */
  double* delta = (double*)malloc(sizeof(double) * (size_t)n_rows * hq);
  for (int64_t r = 0; r < n_rows; ++r)
    for (int h = 0; h < hq; ++h) {
      const uint16_t* doi = d_o + (rows[r] * hq + h) * (int64_t)D;
      const double* oi = O + (r * hq + h) * (int64_t)D;
      double d = 0.0;
      for (int c = 0; c < D; ++c) d += bf(doi[c]) * oi[c];
      delta[r * hq + h] = d;
    }
  if (keys == NULL) n_keys = T;
#pragma omp parallel for schedule(dynamic, 16)
  for (int64_t kidx = 0; kidx < n_keys; ++kidx) {
    const int64_t tj = keys ? keys[kidx] : kidx;
    const int n = seq_of(cu_seqlens, n_seqs, tj);
    const int64_t t0 = cu_seqlens[n], t1 = cu_seqlens[n + 1];
    for (int g = 0; g < hkv; ++g) {
      double* dk = dK + (kidx * hkv + g) * (int64_t)D;
      double* dv = dV + (kidx * hkv + g) * (int64_t)D;
      for (int c = 0; c < D; ++c) { dk[c] = 0.0; dv[c] = 0.0; }
    }
    for (int64_t r = 0; r < n_rows; ++r) {
      const int64_t ti = rows[r];
      if (ti < t0 || ti >= t1 || !visible(span_id, t0, ti - t0, tj - t0)) continue;   /* same sequence, key seen */
      for (int h = 0; h < hq; ++h) {
        const int g = h / G;
        const uint16_t* kj = k + (tj * hkv + g) * (int64_t)D;
        const uint16_t* vj = v + (tj * hkv + g) * (int64_t)D;
        double* dk = dK + (kidx * hkv + g) * (int64_t)D;
        double* dv = dV + (kidx * hkv + g) * (int64_t)D;
        const uint16_t* qi = q + (ti * hq + h) * (int64_t)D;
        const uint16_t* doi = d_o + (ti * hq + h) * (int64_t)D;
        const double p = exp(scale * dot_bf(qi, kj, D) - LSE[r * hq + h]);
        const double dp = dot_bf(doi, vj, D);
        const double ds = p * (dp - delta[r * hq + h]);
        for (int c = 0; c < D; ++c) {
          dv[c] += p * bf(doi[c]);
          dk[c] += scale * ds * bf(qi[c]);
        }
      }
    }
  }
  free(delta);
}

int oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}
