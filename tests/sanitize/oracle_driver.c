/* Sanitizer driver for the CPU oracle (built with -fsanitize=address,undefined, see tests/test_sanitizers.py).
 * Every routine of oracle/percache_oracle.c runs once on small seeded inputs whose buffers are allocated at exactly the
 * documented sizes, so any access outside them, or any undefined arithmetic, ends the program with a report.
 * Values are only checked for being finite (and softmax rows for summing to one): correctness is the pins' job. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include "../../oracle/percache_oracle.c"

static uint32_t rng_state = 12345u;
static float rnd(void) {
  rng_state = rng_state * 1664525u + 1013904223u;
  return (float)((rng_state >> 8) & 0xffff) / 32768.0f - 1.0f;
}
static float *buf(size_t n, int fill) {
  float *p = (float *)malloc(sizeof(float) * (n ? n : 1));
  for (size_t i = 0; i < n; ++i) p[i] = fill ? rnd() : NAN;
  return p;
}
static int finite_all(const float *p, size_t n, const char *what) {
  for (size_t i = 0; i < n; ++i)
    if (!isfinite(p[i])) { printf("non-finite value in %s at %zu\n", what, i); return 0; }
  return 1;
}

int main(void) {
  int ok = 1;
  { /* lookup: ties, a zero row, a zero probe, the empty bank */
    const int N = 37, d = 24, P = 5;
    float *E = buf((size_t)N * d, 1), *pr = buf((size_t)P * d, 1), *sim = buf(P, 0), *sim2 = buf(P, 0), *all = buf(N, 0);
    int32_t *idx = (int32_t *)malloc(sizeof(int32_t) * P);
    uint8_t *hit = (uint8_t *)malloc(P);
    for (int k = 0; k < d; ++k) { E[5 * d + k] = 0.f; E[9 * d + k] = E[3 * d + k]; pr[2 * d + k] = 0.f; pr[1 * d + k] = E[3 * d + k]; }
    oracle_lookup(E, N, d, pr, P, 0.9f, idx, sim, hit, sim2);
    ok &= idx[1] == 3 && hit[1] == 1 && finite_all(sim, P, "lookup sim");
    oracle_similarities(E, N, d, pr + d, all);
    ok &= finite_all(all, N, "similarities");
    oracle_lookup(E, 0, d, pr, P, 0.9f, idx, sim, hit, NULL);
    ok &= idx[0] == -1 && hit[0] == 0;
    free(E); free(pr); free(sim); free(sim2); free(all); free(idx); free(hit);
  }
  { /* one layer: projection variants, RoPE, reuse attention (full and sampled), prefill, statistics, merge */
    const int T = 7, H = 16, Hq = 4, Hkv = 2, D = 8, C = 5, S = 3, n_out = (Hq + 2 * Hkv) * D;
    float *X = buf((size_t)T * H, 1), *W = buf((size_t)n_out * H, 1), *bias = buf(n_out, 1), *qg = buf(D, 1), *kg = buf(D, 1);
    float *Q = buf((size_t)Hq * T * D, 0), *K = buf((size_t)Hkv * T * D, 0), *V = buf((size_t)Hkv * T * D, 0);
    float *sk = buf((size_t)S * Hkv * C * D, 1), *sv = buf((size_t)S * Hkv * C * D, 1);
    const int32_t ids[2] = {2, 0}, used[2] = {5, 3}, si[3] = {0, 6, 3}, sh[3] = {3, 0, 2};
    float *O = buf((size_t)T * Hq * D, 0), *rs = buf((size_t)T * Hq, 0), *Os = buf(3 * D, 0), *rss = buf(3, 0);
    float u[8];
    for (int i = 0; i < D; ++i) u[i] = rnd();
    oracle_rope(u, D, 123456789L, 10000.0);
    ok &= finite_all(u, D, "rope");
    oracle_qkv_rope(X, W, T, H, Hq, Hkv, D, 8, 10000.0, Q, K, V);
    oracle_qkv_rope_ex(X, W, bias, qg, kg, 1e-6, T, H, Hq, Hkv, D, 8, 10000.0, Q, K, V);
    ok &= finite_all(Q, (size_t)Hq * T * D, "Q") && finite_all(K, (size_t)Hkv * T * D, "K") && finite_all(V, (size_t)Hkv * T * D, "V");
    oracle_attention_reuse(Q, K, V, T, Hq, Hkv, D, sk, sv, C, ids, used, 2, 0, NULL, NULL, O, rs);
    ok &= finite_all(O, (size_t)T * Hq * D, "O");
    for (int i = 0; i < T * Hq; ++i) ok &= fabsf(rs[i] - 1.0f) < 1e-5f;
    oracle_attention_reuse(Q, K, V, T, Hq, Hkv, D, sk, sv, C, ids, used, 2, 3, si, sh, Os, rss);
    oracle_attention_reuse(Q, K, V, T, Hq, Hkv, D, NULL, NULL, 1, NULL, NULL, 0, 0, NULL, NULL, O, NULL);
    ok &= finite_all(Os, 3 * D, "sampled O") && finite_all(O, (size_t)T * Hq * D, "causal O");
    oracle_prefill_reuse(X, W, T, H, Hq, Hkv, D, 10000.0, sk, sv, C, ids, used, 2, 0, NULL, NULL, O, K, V, Q);
    oracle_prefill_reuse(X, W, T, H, Hq, Hkv, D, 10000.0, sk, sv, C, ids, used, 2, 3, si, sh, Os, K, V, Q);
    ok &= finite_all(O, (size_t)T * Hq * D, "prefill O") && finite_all(Os, 3 * D, "prefill sampled O");
    double m[3], l[3], o3[3 * 8], om[8];
    for (int s = 0; s < 3; ++s) oracle_attend_stats(Q, sk + (size_t)s * Hkv * C * D, sv + (size_t)s * Hkv * C * D, C, D, &m[s], &l[s], o3 + s * D);
    oracle_lse_merge(m, l, o3, 3, D, om);
    for (int i = 0; i < D; ++i) ok &= isfinite(om[i]) != 0;
    free(X); free(W); free(bias); free(qg); free(kg); free(Q); free(K); free(V); free(sk); free(sv); free(O); free(rs); free(Os); free(rss);
  }
  { /* block tail */
    const int T = 5, H = 12, A = 16, F = 20;
    float *h = buf((size_t)T * H, 1), *attn = buf((size_t)T * A, 1), *Wo = buf((size_t)H * A, 1), *g2 = buf(H, 1), *Wg = buf((size_t)F * H, 1),
          *Wu = buf((size_t)F * H, 1), *Wd = buf((size_t)H * F, 1), *out = buf((size_t)T * H, 0), *nrm = buf((size_t)T * H, 0), *lin = buf((size_t)T * F, 0);
    oracle_rmsnorm(h, g2, T, H, 1e-6, nrm);
    oracle_rmsnorm(h, NULL, T, H, 1e-6, nrm);
    oracle_linear(nrm, Wg, T, H, F, lin);
    oracle_block_tail(h, attn, Wo, g2, Wg, Wu, Wd, T, H, A, F, 1e-6, out);
    ok &= finite_all(nrm, (size_t)T * H, "rmsnorm") && finite_all(lin, (size_t)T * F, "linear") && finite_all(out, (size_t)T * H, "block tail");
    free(h); free(attn); free(Wo); free(g2); free(Wg); free(Wu); free(Wd); free(out); free(nrm); free(lin);
  }
  printf(ok ? "oracle driver: ok (%d threads)\n" : "oracle driver: FAILED (%d threads)\n", oracle_num_threads());
  return ok ? 0 : 1;
}
