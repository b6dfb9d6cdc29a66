/*
 * PerCache hot-path ORACLE -- test infrastructure, not product code.
 *
 * A plain, slow, obviously-correct CPU statement of what the cache-reusing
 * prefill and the query-level match compute.  Tensors are fp32 in memory (the
 * values the GPU side stores in bf16/fp16 are widened exactly); every sum is
 * accumulated in double so results do not depend on summation order.  There is
 * no blocking, no online softmax, no fusion: each function is the definition
 * written out, in the order the paper gives the steps.
 *
 * Nothing here is shared with the HIP library: no headers, no tables, no
 * helpers.  Only tests, the smoke check and the benchmark's CPU-baseline leg
 * may call it.
 *
 * Paper passages followed (PerCache, arXiv 2601.11553):
 *   - Similar Query Reuse (Sec. 4.2.1): cosine similarity against all stored
 *     query embeddings; the best one is a hit if it exceeds tau_query.
 *   - QKV Cache Reuse (Sec. 4.2.2) and App. B.1 (how inference runs over cached tensors):
 *     drop the first L_pre rows of the attention input, project only the
 *     suffix, apply RoPE with the position counter advanced by L_pre, put the
 *     loaded tensors in front of the fresh ones along the sequence axis, then
 *     attention as usual.
 *   - App. B.2 (tokenisation inconsistency): the last few tokens of the final
 *     matched node may be discarded, hence a per-chunk used length.
 *   - Sec. 4.1.1 cache slicer: per-chunk K/V are row ranges of the full
 *     prompt's K/V (the full-prefill routine returns those rows).
 *
 * Pins: tests/test_oracle_*.py (brute-force reuse == full recompute with
 * negative controls, softmax/convex-hull invariants, RoPE closed forms,
 * textbook special cases, scipy/numpy cross-checks).  The paper prints no
 * worked numeric example of these computations.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* ------------------------------------------------------------------ */
/* Sec. 4.2.1: query-level match.                                      */
/* For every probe: s_j = <p, e_j> / (|p| |e_j|) over ALL j; the best   */
/* index (lowest index among equals), its similarity, the runner-up     */
/* similarity, and hit = best > tau (compared in fp32, the precision    */
/* the similarity is reported in).  Zero-norm probe or entry: s_j = 0.  */
/* Empty bank: idx -1, sim -inf, no hit.                                */
/* ------------------------------------------------------------------ */
void oracle_lookup(const float *E, int N, int d, const float *probes, int P,
                   float tau, int32_t *idx, float *sim, uint8_t *hit,
                   float *sim2) {
#pragma omp parallel for schedule(dynamic, 1)
  for (int p = 0; p < P; ++p) {
    const float *q = probes + (size_t)p * d;
    double nq = 0.0;
    for (int k = 0; k < d; ++k) nq += (double)q[k] * (double)q[k];
    nq = sqrt(nq);
    double best = -INFINITY, second = -INFINITY;
    int best_j = -1;
    for (int j = 0; j < N; ++j) {
      const float *e = E + (size_t)j * d;
      double dot = 0.0, ne = 0.0;
      for (int k = 0; k < d; ++k) {
        dot += (double)q[k] * (double)e[k];
        ne += (double)e[k] * (double)e[k];
      }
      ne = sqrt(ne);
      double s = (nq > 0.0 && ne > 0.0) ? dot / (nq * ne) : 0.0;
      if (s > best) {
        second = best;
        best = s;
        best_j = j;
      } else if (s > second) {
        second = s;
      }
    }
    idx[p] = best_j;
    sim[p] = (float)best;
    if (sim2) sim2[p] = (float)second;
    hit[p] = (best_j >= 0 && (float)best > tau) ? 1 : 0;
  }
}

/* All N similarities of one probe (used by tests to judge near-ties). */
void oracle_similarities(const float *E, int N, int d, const float *probe,
                         float *out) {
  double nq = 0.0;
  for (int k = 0; k < d; ++k) nq += (double)probe[k] * (double)probe[k];
  nq = sqrt(nq);
#pragma omp parallel for
  for (int j = 0; j < N; ++j) {
    const float *e = E + (size_t)j * d;
    double dot = 0.0, ne = 0.0;
    for (int k = 0; k < d; ++k) {
      dot += (double)probe[k] * (double)e[k];
      ne += (double)e[k] * (double)e[k];
    }
    ne = sqrt(ne);
    out[j] = (float)((nq > 0.0 && ne > 0.0) ? dot / (nq * ne) : 0.0);
  }
}

/* ------------------------------------------------------------------ */
/* RoPE (App. B.1, last paragraph; RoFormer): rotate the pair           */
/* (u[m], u[m + D/2]) by angle pos * theta^(-2m/D).                     */
/* ------------------------------------------------------------------ */
void oracle_rope(float *u, int D, long pos, double theta) {
  int half = D / 2;
  for (int m = 0; m < half; ++m) {
    double phi = (double)pos * pow(theta, -2.0 * (double)m / (double)D);
    double c = cos(phi), s = sin(phi);
    double a = u[m], b = u[m + half];
    u[m] = (float)(a * c - b * s);
    u[m + half] = (float)(b * c + a * s);
  }
}

/* ------------------------------------------------------------------ */
/* App. B.1: Q/K/V projection of the T retained rows of ONE query,      */
/* y = x W^T with W rows ordered [Q heads | K heads | V heads], then    */
/* RoPE on every q and k head vector at position pos0 + i.              */
/* Outputs head-major: Q[Hq,T,D], K[Hkv,T,D], V[Hkv,T,D].               */
/* ------------------------------------------------------------------ */
/* Model-family variants of the projection (the paper runs Llama and Qwen  */
/* models, Sec. 5.1): bias [(Hq+2Hkv)*D] added to the projection (Qwen2    */
/* style), and RMSNorm over the head dimension of every q and k head with */
/* gains q_gain / k_gain [D] before RoPE (Qwen3 style).  NULL = absent.   */
static void head_rmsnorm(float *u, int D, const float *gain, double eps) {
  double ss = 0.0;
  for (int c = 0; c < D; ++c) ss += (double)u[c] * (double)u[c];
  double r = 1.0 / sqrt(ss / (double)D + eps);
  for (int c = 0; c < D; ++c) u[c] = (float)((double)u[c] * r * (double)gain[c]);
}

void oracle_qkv_rope_ex(const float *X, const float *W, const float *bias,
                        const float *q_gain, const float *k_gain, double eps,
                        int T, int H, int Hq, int Hkv, int D, long pos0,
                        double theta, float *Q, float *K, float *V);

void oracle_qkv_rope(const float *X, const float *W, int T, int H, int Hq,
                     int Hkv, int D, long pos0, double theta, float *Q,
                     float *K, float *V) {
  oracle_qkv_rope_ex(X, W, NULL, NULL, NULL, 0.0, T, H, Hq, Hkv, D, pos0, theta,
                     Q, K, V);
}

void oracle_qkv_rope_ex(const float *X, const float *W, const float *bias,
                        const float *q_gain, const float *k_gain, double eps,
                        int T, int H, int Hq, int Hkv, int D, long pos0,
                        double theta, float *Q, float *K, float *V) {
  int n_out = (Hq + 2 * Hkv) * D;
#pragma omp parallel for collapse(2) schedule(static)
  for (int i = 0; i < T; ++i) {
    for (int o = 0; o < n_out; ++o) {
      const float *x = X + (size_t)i * H;
      const float *w = W + (size_t)o * H;
      double acc = 0.0;
      for (int k = 0; k < H; ++k) acc += (double)x[k] * (double)w[k];
      if (bias) acc += (double)bias[o];
      int head = o / D, c = o % D;
      if (head < Hq)
        Q[((size_t)head * T + i) * D + c] = (float)acc;
      else if (head < Hq + Hkv)
        K[((size_t)(head - Hq) * T + i) * D + c] = (float)acc;
      else
        V[((size_t)(head - Hq - Hkv) * T + i) * D + c] = (float)acc;
    }
  }
#pragma omp parallel for schedule(static)
  for (int i = 0; i < T; ++i) {
    for (int h = 0; h < Hq; ++h) {
      if (q_gain) head_rmsnorm(Q + ((size_t)h * T + i) * D, D, q_gain, eps);
      oracle_rope(Q + ((size_t)h * T + i) * D, D, pos0 + i, theta);
    }
    for (int g = 0; g < Hkv; ++g) {
      if (k_gain) head_rmsnorm(K + ((size_t)g * T + i) * D, D, k_gain, eps);
      oracle_rope(K + ((size_t)g * T + i) * D, D, pos0 + i, theta);
    }
  }
}

/* ------------------------------------------------------------------ */
/* Sec. 4.2.2 / App. B.1: attention of the fresh rows of ONE query over */
/* [loaded chunk K/V in list order ; fresh K/V].                        */
/*   store_k/v : [S, Hkv, C, D]; chunk c contributes tokens             */
/*               0..used_len[c]-1 of slot slot_ids[c].                  */
/*   Row i of head h (kv head h / (Hq/Hkv)) sees every loaded key and   */
/*   fresh keys t <= i.  Two-pass softmax with scale 1/sqrt(D).         */
/* If n_samples > 0 only rows (sample_i[s], sample_h[s]) are computed   */
/* and O is [n_samples, D]; else O is [T, Hq*D].                        */
/* row_sum (optional, same indexing as rows, one float per row/head)    */
/* receives the sum of the normalised probabilities.                    */
/* ------------------------------------------------------------------ */
static void attend_row(const float *q, int g, int i, int T, int Hkv, int D,
                       const float *Kf, const float *Vf, const float *store_k,
                       const float *store_v, int C, const int32_t *slot_ids,
                       const int32_t *used_len, int n_chunks, float *o,
                       float *row_sum) {
  long L_pre = 0;
  for (int c = 0; c < n_chunks; ++c) L_pre += used_len[c];
  long L = L_pre + i + 1;
  double *s = (double *)malloc(sizeof(double) * (size_t)L);
  const float **vrow = (const float **)malloc(sizeof(float *) * (size_t)L);
  double scale = 1.0 / sqrt((double)D);
  long j = 0;
  for (int c = 0; c < n_chunks; ++c) {
    size_t base = (((size_t)slot_ids[c] * Hkv + g) * C) * (size_t)D;
    for (int t = 0; t < used_len[c]; ++t, ++j) {
      const float *k = store_k + base + (size_t)t * D;
      double dot = 0.0;
      for (int x = 0; x < D; ++x) dot += (double)q[x] * (double)k[x];
      s[j] = dot * scale;
      vrow[j] = store_v + base + (size_t)t * D;
    }
  }
  for (int t = 0; t <= i; ++t, ++j) {
    const float *k = Kf + ((size_t)g * T + t) * D;
    double dot = 0.0;
    for (int x = 0; x < D; ++x) dot += (double)q[x] * (double)k[x];
    s[j] = dot * scale;
    vrow[j] = Vf + ((size_t)g * T + t) * D;
  }
  double m = -INFINITY;
  for (long a = 0; a < L; ++a)
    if (s[a] > m) m = s[a];
  double denom = 0.0;
  for (long a = 0; a < L; ++a) {
    s[a] = exp(s[a] - m);
    denom += s[a];
  }
  double psum = 0.0;
  for (long a = 0; a < L; ++a) {
    s[a] /= denom;
    psum += s[a];
  }
  for (int x = 0; x < D; ++x) {
    double acc = 0.0;
    for (long a = 0; a < L; ++a) acc += s[a] * (double)vrow[a][x];
    o[x] = (float)acc;
  }
  if (row_sum) *row_sum = (float)psum;
  free(s);
  free((void *)vrow);
}

void oracle_attention_reuse(const float *Q, const float *Kf, const float *Vf,
                            int T, int Hq, int Hkv, int D,
                            const float *store_k, const float *store_v, int C,
                            const int32_t *slot_ids, const int32_t *used_len,
                            int n_chunks, int n_samples,
                            const int32_t *sample_i, const int32_t *sample_h,
                            float *O, float *row_sum) {
  int G = Hq / Hkv;
  if (n_samples > 0) {
#pragma omp parallel for schedule(dynamic, 1)
    for (int sidx = 0; sidx < n_samples; ++sidx) {
      int i = sample_i[sidx], h = sample_h[sidx];
      attend_row(Q + ((size_t)h * T + i) * D, h / G, i, T, Hkv, D, Kf, Vf,
                 store_k, store_v, C, slot_ids, used_len, n_chunks,
                 O + (size_t)sidx * D, row_sum ? row_sum + sidx : NULL);
    }
    return;
  }
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
  for (int i = 0; i < T; ++i) {
    for (int h = 0; h < Hq; ++h) {
      attend_row(Q + ((size_t)h * T + i) * D, h / G, i, T, Hkv, D, Kf, Vf,
                 store_k, store_v, C, slot_ids, used_len, n_chunks,
                 O + ((size_t)i * Hq + h) * D,
                 row_sum ? row_sum + (size_t)i * Hq + h : NULL);
    }
  }
}

/* ------------------------------------------------------------------ */
/* One query's cache-reusing prefill for one layer's attention module:  */
/* L_pre = sum used_len; project + RoPE the T fresh rows at positions   */
/* L_pre..L_pre+T-1; attend.  n_chunks = 0 is ordinary causal prefill   */
/* of a contiguous prompt (the full recomputation), and the returned    */
/* Kf/Vf rows are what the cache slicer cuts into per-chunk pieces.     */
/* ------------------------------------------------------------------ */
void oracle_prefill_reuse(const float *X, const float *W, int T, int H, int Hq,
                          int Hkv, int D, double theta, const float *store_k,
                          const float *store_v, int C, const int32_t *slot_ids,
                          const int32_t *used_len, int n_chunks, int n_samples,
                          const int32_t *sample_i, const int32_t *sample_h,
                          float *O, float *Kf, float *Vf, float *Qout) {
  long L_pre = 0;
  for (int c = 0; c < n_chunks; ++c) L_pre += used_len[c];
  float *Q = (float *)malloc(sizeof(float) * (size_t)Hq * T * D);
  oracle_qkv_rope(X, W, T, H, Hq, Hkv, D, L_pre, theta, Q, Kf, Vf);
  oracle_attention_reuse(Q, Kf, Vf, T, Hq, Hkv, D, store_k, store_v, C,
                         slot_ids, used_len, n_chunks, n_samples, sample_i,
                         sample_h, O, NULL);
  if (Qout) memcpy(Qout, Q, sizeof(float) * (size_t)Hq * T * D);
  free(Q);
}

/* ------------------------------------------------------------------ */
/* Merge of partial softmax-attention results over a split of the key   */
/* axis: m = max m_s, l = sum l_s e^{m_s-m}, o = sum o_s l_s e^{m_s-m}/l */
/* where o_s is the normalised output of split s.  Used by the tests to */
/* show that splitting the key axis changes nothing.                    */
/* ------------------------------------------------------------------ */
void oracle_lse_merge(const double *m_s, const double *l_s, const double *o_s,
                      int n_splits, int D, double *o) {
  double m = -INFINITY;
  for (int s = 0; s < n_splits; ++s)
    if (m_s[s] > m) m = m_s[s];
  double l = 0.0;
  for (int s = 0; s < n_splits; ++s) l += l_s[s] * exp(m_s[s] - m);
  for (int x = 0; x < D; ++x) {
    double acc = 0.0;
    for (int s = 0; s < n_splits; ++s)
      acc += o_s[(size_t)s * D + x] * l_s[s] * exp(m_s[s] - m);
    o[x] = acc / l;
  }
}

/* Softmax attention of one query vector over an explicit key/value list */
/* returning the un-merged statistics (max, sum of exp, normalised out). */
void oracle_attend_stats(const float *q, const float *K, const float *V, int L,
                         int D, double *m_out, double *l_out, double *o_out) {
  double scale = 1.0 / sqrt((double)D);
  double *s = (double *)malloc(sizeof(double) * (size_t)L);
  double m = -INFINITY;
  for (int j = 0; j < L; ++j) {
    double dot = 0.0;
    for (int x = 0; x < D; ++x)
      dot += (double)q[x] * (double)K[(size_t)j * D + x];
    s[j] = dot * scale;
    if (s[j] > m) m = s[j];
  }
  double l = 0.0;
  for (int j = 0; j < L; ++j) {
    s[j] = exp(s[j] - m);
    l += s[j];
  }
  for (int x = 0; x < D; ++x) {
    double acc = 0.0;
    for (int j = 0; j < L; ++j) acc += s[j] * (double)V[(size_t)j * D + x];
    o_out[x] = acc / l;
  }
  *m_out = m;
  *l_out = l;
  free(s);
}

/* ------------------------------------------------------------------ */
/* The rest of a pre-norm transformer block on the fresh rows, needed   */
/* only to chain layers (App. B.1: after the concatenation the block    */
/* runs as it always does).  RMSNorm with gain and eps; y = x W^T linear; SwiGLU MLP. */
/* ------------------------------------------------------------------ */
void oracle_rmsnorm(const float *X, const float *gain, int T, int H, double eps,
                    float *Y) {
#pragma omp parallel for
  for (int i = 0; i < T; ++i) {
    double ss = 0.0;
    for (int k = 0; k < H; ++k)
      ss += (double)X[(size_t)i * H + k] * (double)X[(size_t)i * H + k];
    double r = 1.0 / sqrt(ss / (double)H + eps);
    for (int k = 0; k < H; ++k)
      Y[(size_t)i * H + k] =
          (float)((double)X[(size_t)i * H + k] * r * (gain ? (double)gain[k] : 1.0));
  }
}

void oracle_linear(const float *X, const float *W, int T, int n_in, int n_out,
                   float *Y) {
#pragma omp parallel for collapse(2)
  for (int i = 0; i < T; ++i) {
    for (int o = 0; o < n_out; ++o) {
      double acc = 0.0;
      for (int k = 0; k < n_in; ++k)
        acc += (double)X[(size_t)i * n_in + k] * (double)W[(size_t)o * n_in + k];
      Y[(size_t)i * n_out + o] = (float)acc;
    }
  }
}

/* h_out = h_mid + W_down( silu(W_gate n) * (W_up n) ), n = rmsnorm(h_mid),  */
/* h_mid = h_in + W_o attn.                                                   */
void oracle_block_tail(const float *h_in, const float *attn, const float *Wo,
                       const float *gain2, const float *Wgate, const float *Wup,
                       const float *Wdown, int T, int H, int n_attn, int F,
                       double eps, float *h_out) {
  float *proj = (float *)malloc(sizeof(float) * (size_t)T * H);
  float *mid = (float *)malloc(sizeof(float) * (size_t)T * H);
  float *nrm = (float *)malloc(sizeof(float) * (size_t)T * H);
  float *gate = (float *)malloc(sizeof(float) * (size_t)T * F);
  float *up = (float *)malloc(sizeof(float) * (size_t)T * F);
  oracle_linear(attn, Wo, T, n_attn, H, proj);
  for (size_t a = 0; a < (size_t)T * H; ++a)
    mid[a] = (float)((double)h_in[a] + (double)proj[a]);
  oracle_rmsnorm(mid, gain2, T, H, eps, nrm);
  oracle_linear(nrm, Wgate, T, H, F, gate);
  oracle_linear(nrm, Wup, T, H, F, up);
  for (size_t a = 0; a < (size_t)T * F; ++a) {
    double gte = gate[a];
    double silu = gte / (1.0 + exp(-gte));
    gate[a] = (float)(silu * (double)up[a]);
  }
  oracle_linear(gate, Wdown, T, F, H, proj);
  for (size_t a = 0; a < (size_t)T * H; ++a)
    h_out[a] = (float)((double)mid[a] + (double)proj[a]);
  free(proj);
  free(mid);
  free(nrm);
  free(gate);
  free(up);
}
