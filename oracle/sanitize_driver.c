/*
 * sanitize_driver.c -- calls every function of rc_oracle.c on small random problems and prints a
 * checksum of everything they return.  TEST INFRASTRUCTURE: tests/test_oracle_sanitizers.py builds
 * it twice, plainly and with -fsanitize=address,undefined (no Python in the process), requires
 * both runs to end cleanly and the two checksums to agree.  Exact-size heap buffers, so that a
 * read or write one element past an array is caught.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int rc_oracle_decode(int, const uint16_t*, int64_t, double*);
int rc_oracle_block_norms(int, int, int, int, int, int, int64_t, const uint16_t*, const uint16_t*, int64_t, double*, double*);
int rc_oracle_sqdist(int, const uint16_t*, const uint16_t*, int64_t, double*);
int rc_oracle_score_pairs(int, int, int, int, int, const uint16_t*, const uint16_t*, int64_t, const uint16_t*, const uint16_t*,
                          int64_t, int64_t, const int32_t*, const int32_t*, const int32_t*, double*);
int rc_oracle_match(int, int, int, int, int, int, const uint16_t*, const uint16_t*, int64_t, int64_t, const uint16_t*,
                    const uint16_t*, int64_t, int64_t, const uint8_t*, double, int32_t*, double*, int32_t*, double*, double*);
int rc_oracle_candidates(int, int, int, int, int, int, const uint16_t*, const uint16_t*, int64_t, int64_t, const uint16_t*,
                         const uint16_t*, int64_t, int64_t, const int32_t*, int64_t, const uint8_t*, double, double*, int32_t*,
                         double*, int32_t*);
int rc_oracle_layer_mean(int, int, int, int, int, const uint16_t*, const uint16_t*, int64_t, int64_t, const uint16_t*,
                         const uint16_t*, int64_t, int64_t, const uint8_t*, double, int32_t*, double*, int32_t*, double*, double*);
int rc_oracle_candidate_distances(int, int, int, int, int, const uint16_t*, const uint16_t*, int64_t, int64_t, const uint16_t*,
                                  const uint16_t*, int64_t, int64_t, const int32_t*, int64_t, const uint8_t*, double, double*,
                                  int32_t*, double*, int32_t*);
int rc_oracle_pat_threshold(const float*, int64_t, double, float*, int64_t*);
int rc_oracle_apply_threshold(const int32_t*, const float*, int64_t, float, int32_t*);
int rc_oracle_pool_admit(int, int64_t, int, const uint16_t*, const uint16_t*, int64_t, int64_t, const double*, const double*,
                         uint16_t*, uint16_t*, int64_t, int64_t, double*, double*, uint8_t*, const int32_t*, int32_t*, int32_t*);
int rc_oracle_pool_touch(const int32_t*, int64_t, int32_t, int32_t*, int64_t);
int rc_oracle_refcount_release(const int32_t*, int64_t, int32_t*, int64_t);
int rc_oracle_pool_evict(int64_t, uint8_t*, const int32_t*, const int32_t*, const int32_t*, int64_t, int64_t, int32_t*, int32_t*);
int rc_oracle_remap(int, const int32_t*, int32_t*, int64_t, int64_t, const int32_t*, const int32_t*, const int32_t*, int64_t,
                    int64_t, int64_t, const int32_t*, int32_t*, uint8_t*, int32_t*);

static uint64_t g_state = 88172645463325252ULL, g_sum = 1469598103934665603ULL;
static uint32_t rnd(void) {
  g_state ^= g_state << 13;
  g_state ^= g_state >> 7;
  g_state ^= g_state << 17;
  return (uint32_t)(g_state >> 16);
}
static void mix(const void* p, size_t bytes) {
  const unsigned char* b = (const unsigned char*)p;
  for (size_t i = 0; i < bytes; ++i) g_sum = (g_sum ^ b[i]) * 1099511628211ULL;
}
static void* xmalloc(size_t bytes) {
  void* p = malloc(bytes ? bytes : 1);
  if (!p) exit(3);
  memset(p, 0, bytes);
  return p;
}
/* finite 16-bit patterns of either format: exponent field never all ones */
static uint16_t* rand_kv(int dtype, int64_t n) {
  uint16_t* a = (uint16_t*)xmalloc(sizeof(uint16_t) * (size_t)n);
  for (int64_t i = 0; i < n; ++i) {
    uint16_t b = (uint16_t)rnd();
    if (dtype == 0 && (b & 0x7c00) == 0x7c00) b &= (uint16_t)~0x0400;
    if (dtype == 1 && (b & 0x7f80) == 0x7f80) b &= (uint16_t)~0x0080;
    if (dtype == 1) b = (uint16_t)((b & 0x80ff) | 0x3f00); /* bf16 values of magnitude about 1 */
    if (dtype == 0) b = (uint16_t)((b & 0x83ff) | 0x3c00); /* fp16 values of magnitude about 1 */
    a[i] = b;
  }
  return a;
}
#define CHECK(call)                                   \
  do {                                                \
    int rc_ = (call);                                 \
    if (rc_ != 0) {                                   \
      printf("%s failed with %d\n", #call, rc_);      \
      exit(2);                                        \
    }                                                 \
  } while (0)

static void one_problem(int dtype, int mode, int L, int T, int H, int64_t Q, int64_t P, int64_t C) {
  const int Dh = 128;
  const int64_t D = (int64_t)T * H * Dh, NH = mode ? H : 1;
  uint16_t *kq = rand_kv(dtype, L * Q * D), *vq = rand_kv(dtype, L * Q * D), *kp = rand_kv(dtype, L * P * D),
           *vp = rand_kv(dtype, L * P * D);
  if (P > 0 && Q > 0) { /* a planted duplicate */
    memcpy(kq, kp + (P - 1) * D, sizeof(uint16_t) * (size_t)D);
    memcpy(vq, vp + (P - 1) * D, sizeof(uint16_t) * (size_t)D);
  }
  uint8_t* live = (uint8_t*)xmalloc((size_t)(L * P));
  for (int64_t i = 0; i < L * P; ++i) live[i] = rnd() % 5 != 0;
  double *qk = (double*)xmalloc(sizeof(double) * (size_t)(L * Q * NH)), *qv = (double*)xmalloc(sizeof(double) * (size_t)(L * Q * NH)),
         *pk = (double*)xmalloc(sizeof(double) * (size_t)(L * P * NH)), *pv = (double*)xmalloc(sizeof(double) * (size_t)(L * P * NH));
  CHECK(rc_oracle_block_norms(dtype, mode, L, T, H, Dh, Q * D, kq, vq, Q, qk, qv));
  CHECK(rc_oracle_block_norms(dtype, mode, L, T, H, Dh, P * D, kp, vp, P, pk, pv));
  mix(qk, sizeof(double) * (size_t)(L * Q * NH));
  mix(pv, sizeof(double) * (size_t)(L * P * NH));
  /* exhaustive search with the score matrix */
  int32_t *bi = (int32_t*)xmalloc(sizeof(int32_t) * (size_t)(L * Q)), *mi = (int32_t*)xmalloc(sizeof(int32_t) * (size_t)(L * Q));
  double *bs = (double*)xmalloc(sizeof(double) * (size_t)(L * Q)), *ss = (double*)xmalloc(sizeof(double) * (size_t)(L * Q)),
         *sc = (double*)xmalloc(sizeof(double) * (size_t)(L * Q * P));
  CHECK(rc_oracle_match(dtype, mode, L, T, H, Dh, kq, vq, Q * D, Q, kp, vp, P * D, P, live, 0.9, bi, bs, mi, ss, sc));
  mix(bi, sizeof(int32_t) * (size_t)(L * Q));
  mix(mi, sizeof(int32_t) * (size_t)(L * Q));
  mix(bs, sizeof(double) * (size_t)(L * Q));
  mix(ss, sizeof(double) * (size_t)(L * Q));
  mix(sc, sizeof(double) * (size_t)(L * Q * P));
  CHECK(rc_oracle_match(dtype, mode, L, T, H, Dh, kq, vq, Q * D, Q, kp, vp, P * D, P, NULL, 0.9, bi, bs, mi, ss, NULL));
  mix(bi, sizeof(int32_t) * (size_t)(L * Q));
  /* listed pairs */
  const int64_t np = (P > 0 && Q > 0) ? 7 : 0;
  int32_t *li = (int32_t*)xmalloc(sizeof(int32_t) * (size_t)np), *qi = (int32_t*)xmalloc(sizeof(int32_t) * (size_t)np),
          *pi = (int32_t*)xmalloc(sizeof(int32_t) * (size_t)np);
  for (int64_t i = 0; i < np; ++i) {
    li[i] = (int32_t)(rnd() % (uint32_t)L);
    qi[i] = (int32_t)(rnd() % (uint32_t)Q);
    pi[i] = (int32_t)(rnd() % (uint32_t)P);
  }
  double* ps = (double*)xmalloc(sizeof(double) * (size_t)np);
  CHECK(rc_oracle_score_pairs(dtype, mode, T, H, Dh, kq, vq, Q * D, kp, vp, P * D, np, li, qi, pi, ps));
  mix(ps, sizeof(double) * (size_t)np);
  /* candidate lists, per layer and layer-shared */
  int32_t* cand = (int32_t*)xmalloc(sizeof(int32_t) * (size_t)(L * Q * C));
  for (int64_t i = 0; i < L * Q * C; ++i) cand[i] = (int32_t)(rnd() % (uint32_t)(P + 3)) - 1; /* -1 .. P+1: empty and out of range too */
  double* cs = (double*)xmalloc(sizeof(double) * (size_t)(L * Q * C));
  CHECK(rc_oracle_candidates(dtype, mode, L, T, H, Dh, kq, vq, Q * D, Q, kp, vp, P * D, P, cand, C, live, 0.9, cs, bi, bs, mi));
  mix(cs, sizeof(double) * (size_t)(L * Q * C));
  mix(bi, sizeof(int32_t) * (size_t)(L * Q));
  if (L > 0 && mode == 0) {
    int32_t *b1 = (int32_t*)xmalloc(sizeof(int32_t) * (size_t)Q), *m1 = (int32_t*)xmalloc(sizeof(int32_t) * (size_t)Q);
    double *d1 = (double*)xmalloc(sizeof(double) * (size_t)Q), *s1 = (double*)xmalloc(sizeof(double) * (size_t)Q),
           *dm = (double*)xmalloc(sizeof(double) * (size_t)(Q * P)), *cd = (double*)xmalloc(sizeof(double) * (size_t)(Q * C));
    CHECK(rc_oracle_layer_mean(dtype, L, T, H, Dh, kq, vq, Q * D, Q, kp, vp, P * D, P, live, 0.4, b1, d1, m1, s1, dm));
    mix(b1, sizeof(int32_t) * (size_t)Q);
    mix(d1, sizeof(double) * (size_t)Q);
    mix(s1, sizeof(double) * (size_t)Q);
    mix(dm, sizeof(double) * (size_t)(Q * P));
    CHECK(rc_oracle_candidate_distances(dtype, L, T, H, Dh, kq, vq, Q * D, Q, kp, vp, P * D, P, cand, C, live, 0.4, cd, b1, d1, m1));
    mix(cd, sizeof(double) * (size_t)(Q * C));
    mix(m1, sizeof(int32_t) * (size_t)Q);
    /* admission with the layer-shared decisions */
    int32_t *slot = (int32_t*)xmalloc(sizeof(int32_t) * (size_t)Q), nadm = 0;
    CHECK(rc_oracle_pool_admit(L, D, 1, kq, vq, Q * D, Q, qk, qv, kp, vp, P * D, P, pk, pv, live, m1, slot, &nadm));
    mix(slot, sizeof(int32_t) * (size_t)Q);
    mix(&nadm, sizeof nadm);
    mix(kp, sizeof(uint16_t) * (size_t)(L * P * D));
    free(b1); free(m1); free(d1); free(s1); free(dm); free(cd); free(slot);
  }
  free(kq); free(vq); free(kp); free(vp); free(live); free(qk); free(qv); free(pk); free(pv);
  free(bi); free(mi); free(bs); free(ss); free(sc); free(li); free(qi); free(pi); free(ps); free(cand); free(cs);
}

static void small_functions(void) {
  /* decode and squared distance */
  for (int dtype = 0; dtype < 2; ++dtype) {
    const int64_t n = 1000;
    uint16_t *x = rand_kv(dtype, n), *y = rand_kv(dtype, n);
    double *out = (double*)xmalloc(sizeof(double) * (size_t)n), d2 = 0;
    CHECK(rc_oracle_decode(dtype, x, n, out));
    CHECK(rc_oracle_sqdist(dtype, x, y, n, &d2));
    mix(out, sizeof(double) * (size_t)n);
    mix(&d2, sizeof d2);
    free(x); free(y); free(out);
  }
  /* percentile and decision */
  for (int64_t n = 0; n < 40; n += 13) {
    float *s = (float*)xmalloc(sizeof(float) * (size_t)n), thr = 0;
    int64_t nf = 0;
    for (int64_t i = 0; i < n; ++i) s[i] = (i % 7 == 3) ? INFINITY : (float)(rnd() % 1000) / 100.0f;
    CHECK(rc_oracle_pat_threshold(s, n, 80.0, &thr, &nf));
    mix(&thr, sizeof thr);
    mix(&nf, sizeof nf);
    int32_t *idx = (int32_t*)xmalloc(sizeof(int32_t) * (size_t)n), *m = (int32_t*)xmalloc(sizeof(int32_t) * (size_t)n);
    for (int64_t i = 0; i < n; ++i) idx[i] = (int32_t)(rnd() % 9) - 1;
    CHECK(rc_oracle_apply_threshold(idx, s, n, thr, m));
    mix(m, sizeof(int32_t) * (size_t)n);
    free(s); free(idx); free(m);
  }
  /* block metadata, eviction, remap */
  for (int rep = 0; rep < 6; ++rep) {
    const int64_t P = 1 + rnd() % 90, Q = rnd() % 40, NB = P + Q + 3, R = 1 + rnd() % 3, E = rnd() % 50;
    const int L = 1 + (int)(rnd() % 3);
    uint8_t* live = (uint8_t*)xmalloc((size_t)P);
    int32_t *refc = (int32_t*)xmalloc(sizeof(int32_t) * (size_t)P), *used = (int32_t*)xmalloc(sizeof(int32_t) * (size_t)P),
            *m = (int32_t*)xmalloc(sizeof(int32_t) * (size_t)Q), nf = 0, ne = 0;
    for (int64_t p = 0; p < P; ++p) {
      live[p] = rnd() % 4 != 0;
      refc[p] = (int32_t)(rnd() % 3);
      used[p] = (int32_t)(rnd() % 5);
    }
    for (int64_t q = 0; q < Q; ++q) m[q] = (rnd() % 2) ? -1 : (int32_t)(rnd() % (uint32_t)P);
    CHECK(rc_oracle_pool_touch(m, Q, 99, used, P));
    CHECK(rc_oracle_refcount_release(m, Q, refc, P));
    CHECK(rc_oracle_pool_evict(P, live, rep % 2 ? refc : NULL, used, m, Q, rep, &nf, &ne));
    mix(live, (size_t)P);
    mix(refc, sizeof(int32_t) * (size_t)P);
    mix(used, sizeof(int32_t) * (size_t)P);
    mix(&nf, sizeof nf);
    mix(&ne, sizeof ne);
    int32_t *tin = (int32_t*)xmalloc(sizeof(int32_t) * (size_t)(L * R * E)), *tout = (int32_t*)xmalloc(sizeof(int32_t) * (size_t)(L * R * E)),
            *qid = (int32_t*)xmalloc(sizeof(int32_t) * (size_t)Q), *ml = (int32_t*)xmalloc(sizeof(int32_t) * (size_t)(L * Q)),
            *rin = (int32_t*)xmalloc(sizeof(int32_t) * (size_t)(L * NB)), *rout = (int32_t*)xmalloc(sizeof(int32_t) * (size_t)(L * NB)),
            *nrem = (int32_t*)xmalloc(sizeof(int32_t) * (size_t)L);
    uint8_t* freed = (uint8_t*)xmalloc((size_t)(L * Q));
    for (int64_t i = 0; i < L * R * E; ++i) tin[i] = (int32_t)(rnd() % (uint32_t)(NB + 2)) - 1;
    for (int64_t q = 0; q < Q; ++q) qid[q] = (int32_t)(P + q);
    for (int64_t i = 0; i < L * Q; ++i) ml[i] = (int32_t)(rnd() % (uint32_t)(P + 2)) - 1;
    for (int64_t i = 0; i < L * NB; ++i) rin[i] = (int32_t)(rnd() % 4);
    CHECK(rc_oracle_remap(L, tin, tout, R, E, qid, NULL, ml, Q, P, NB, rin, rout, freed, nrem));
    mix(tout, sizeof(int32_t) * (size_t)(L * R * E));
    mix(rout, sizeof(int32_t) * (size_t)(L * NB));
    mix(freed, (size_t)(L * Q));
    mix(nrem, sizeof(int32_t) * (size_t)L);
    free(live); free(refc); free(used); free(m); free(tin); free(tout); free(qid); free(ml); free(rin); free(rout); free(nrem); free(freed);
  }
}

int main(void) {
  small_functions();
  /* dtype, mode, L, T, H, Q, P, C */
  one_problem(0, 0, 2, 16, 2, 5, 9, 3);
  one_problem(1, 0, 1, 16, 1, 3, 4, 2);
  one_problem(0, 1, 2, 32, 3, 4, 6, 4);
  one_problem(1, 1, 1, 16, 2, 2, 3, 1);
  one_problem(0, 0, 1, 16, 1, 0, 5, 2);  /* no queries */
  one_problem(0, 0, 1, 16, 1, 4, 0, 2);  /* empty pool */
  one_problem(1, 0, 3, 16, 2, 6, 7, 0);  /* empty candidate lists */
  printf("checksum %016llx\n", (unsigned long long)g_sum);
  return 0;
}
