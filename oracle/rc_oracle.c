/*
 * rc_oracle.c -- plain CPU statement of the reusable-KV-block search.
 *
 * TEST INFRASTRUCTURE, not product code: only the tests, the smoke check and the
 * CPU-baseline leg of the benchmark may call this.  It shares nothing with the
 * HIP path.  Everything is the definition written out in double precision on the
 * exact fp16/bf16 bit patterns the GPU sees; the only parallelism is an OpenMP
 * loop over independent pool blocks.
 *
 * What is computed (ReasonCache Sec. IV-A Stage 2 and Sec. IV-B):
 *   - squared L2 norm of a flattened K or V block (the cached terms of the
 *     squared-distance expansion of Stage 2);
 *   - pair score s = (cos(Kq,Kp) + cos(Vq,Vp))/2, cos = <x,y>/sqrt(|x|^2|y|^2),
 *     cos := 0 when a norm is 0.  K and V are normalised separately and averaged,
 *     mirroring the paper's sum of the K distance and the V distance.  For unit
 *     vectors |x-y|^2 = 2 - 2cos, which ties the score to the paper's distance;
 *   - per-head-all mode: the same on each head's [T][Dh] slice, then min over heads;
 *   - best live pool block per query (lowest index on exact ties), runner-up
 *     value, match iff best >= tau (the Stage 2 sharing decision);
 *   - the paper's own measure: layer-mean of (|Kq-Kp| + |Vq-Vp|)/(2dh), one decision per
 *     block shared by all layers, match iff distance <= threshold;
 *   - the percentile threshold of the warm-up distances (nearest rank);
 *   - admission of unmatched query blocks into free pool slots, with their cached norms;
 *   - room for the admissions of a step: unreferenced blocks leave the pool, least recently used first,
 *     with the block metadata (last use, reference counts) the paper keeps per block;
 *   - block-table remap with reference counts (Sec. IV-B).
 *
 * Pins (tests/test_oracle_pins.py): bit decode against two library decoders,
 * integer closed forms for norms, the direct subtract-and-square distance against
 * the expansion, planted duplicates (score exactly 1), disjoint supports (score
 * exactly 0), K/V-averaging and per-head constructions with hand-known values,
 * the 1/sqrt(1+sigma^2) law for noisy copies, tie/dead/threshold cases, and for the
 * remap a hand-worked table plus conservation/idempotence invariants; for the layer-mean
 * distance a hand-worked 3-4-5 example, a library norm routine, metric properties and the
 * expansion identity through the separately pinned norms and scores; for the percentile a
 * library quantile routine, hand cases and the defining inequalities of a quantile.
 * Every function here is pinned; none is "parity unpinned".  tests/test_oracle_mutants.py
 * compiles copies of this file with one planted mistake each and requires the pins to reject
 * every copy.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORC_F16 = 0, ORC_BF16 = 1 };
enum { ORC_BLOCK = 0, ORC_PER_HEAD_ALL = 1 };

/* IEEE binary16: 1 sign, 5 exponent (bias 15), 10 fraction bits. */
static double decode_f16(uint16_t b) {
  int sign = b >> 15, e = (b >> 10) & 31, m = b & 1023;
  double v;
  if (e == 0)
    v = ldexp((double)m, -24); /* subnormal: m * 2^-10 * 2^-14 */
  else if (e == 31)
    v = m ? NAN : INFINITY;
  else
    v = ldexp((double)(1024 + m), e - 25); /* (1 + m/1024) * 2^(e-15) */
  return sign ? -v : v;
}

/* bfloat16 is the upper half of an IEEE binary32. */
static double decode_bf16(uint16_t b) {
  uint32_t u = (uint32_t)b << 16;
  float f;
  memcpy(&f, &u, sizeof f);
  return (double)f;
}

static double decode(int dtype, uint16_t b) { return dtype == ORC_BF16 ? decode_bf16(b) : decode_f16(b); }

static void decode_block(int dtype, const uint16_t* bits, int64_t n, double* out) {
  for (int64_t i = 0; i < n; ++i) out[i] = decode(dtype, bits[i]);
}

int rc_oracle_decode(int dtype, const uint16_t* bits, int64_t n, double* out) {
  if (!bits || !out || n < 0) return 1;
  decode_block(dtype, bits, n, out);
  return 0;
}

/* Index of (token t, head h, dim d) inside one block laid out [T][H][Dh]. */
static int64_t at(int H, int Dh, int t, int h, int d) { return ((int64_t)t * H + h) * Dh + d; }

/* Sum of squares over the whole block (head < 0) or over one head's [T][Dh] slice. */
static double sqnorm(const double* x, int T, int H, int Dh, int head) {
  double acc = 0.0;
  for (int t = 0; t < T; ++t)
    for (int h = 0; h < H; ++h) {
      if (head >= 0 && h != head) continue;
      for (int d = 0; d < Dh; ++d) {
        double a = x[at(H, Dh, t, h, d)];
        acc += a * a;
      }
    }
  return acc;
}

static double dot(const double* x, const double* y, int T, int H, int Dh, int head) {
  double acc = 0.0;
  for (int t = 0; t < T; ++t)
    for (int h = 0; h < H; ++h) {
      if (head >= 0 && h != head) continue;
      for (int d = 0; d < Dh; ++d) acc += x[at(H, Dh, t, h, d)] * y[at(H, Dh, t, h, d)];
    }
  return acc;
}

static double cosine(double xy, double xx, double yy) {
  if (xx == 0.0 || yy == 0.0) return 0.0;
  return xy / sqrt(xx * yy);
}

/* Score of one pair from decoded blocks; norms are recomputed here, by definition. */
static double pair_score(const double* kq, const double* vq, const double* kp, const double* vp,
                         int T, int H, int Dh, int mode) {
  if (mode == ORC_BLOCK) {
    double ck = cosine(dot(kq, kp, T, H, Dh, -1), sqnorm(kq, T, H, Dh, -1), sqnorm(kp, T, H, Dh, -1));
    double cv = cosine(dot(vq, vp, T, H, Dh, -1), sqnorm(vq, T, H, Dh, -1), sqnorm(vp, T, H, Dh, -1));
    return 0.5 * (ck + cv);
  }
  double s = INFINITY;
  for (int h = 0; h < H; ++h) {
    double ck = cosine(dot(kq, kp, T, H, Dh, h), sqnorm(kq, T, H, Dh, h), sqnorm(kp, T, H, Dh, h));
    double cv = cosine(dot(vq, vp, T, H, Dh, h), sqnorm(vq, T, H, Dh, h), sqnorm(vp, T, H, Dh, h));
    double sh = 0.5 * (ck + cv);
    if (sh < s) s = sh;
  }
  return s;
}

static int bad_shape(int L, int T, int H, int Dh, int64_t layer_stride, int64_t n) {
  return L < 0 || T <= 0 || H <= 0 || Dh <= 0 || n < 0 || layer_stride < n * (int64_t)T * H * Dh;
}

/* ksq, vsq: [L][n] (block mode) or [L][n][H] (per-head-all mode), double. */
int rc_oracle_block_norms(int dtype, int mode, int L, int T, int H, int Dh, int64_t layer_stride,
                          const uint16_t* k, const uint16_t* v, int64_t n, double* ksq, double* vsq) {
  if (bad_shape(L, T, H, Dh, layer_stride, n) || !ksq || !vsq || (n > 0 && L > 0 && (!k || !v))) return 1;
  const int64_t D = (int64_t)T * H * Dh;
  double* x = (double*)malloc(sizeof(double) * (size_t)(D > 0 ? D : 1));
  if (!x) return 2;
  for (int l = 0; l < L; ++l)
    for (int64_t b = 0; b < n; ++b)
      for (int which = 0; which < 2; ++which) {
        const uint16_t* src = (which ? v : k) + (int64_t)l * layer_stride + b * D;
        double* dst = which ? vsq : ksq;
        decode_block(dtype, src, D, x);
        if (mode == ORC_BLOCK)
          dst[(int64_t)l * n + b] = sqnorm(x, T, H, Dh, -1);
        else
          for (int h = 0; h < H; ++h) dst[((int64_t)l * n + b) * H + h] = sqnorm(x, T, H, Dh, h);
      }
  free(x);
  return 0;
}

/* Squared Euclidean distance by subtracting and squaring (the left side of the
 * Stage 2 expansion); used by the pins and by nothing else. */
int rc_oracle_sqdist(int dtype, const uint16_t* x, const uint16_t* y, int64_t n, double* out) {
  if (!x || !y || !out || n < 0) return 1;
  double acc = 0.0;
  for (int64_t i = 0; i < n; ++i) {
    double d = decode(dtype, x[i]) - decode(dtype, y[i]);
    acc += d * d;
  }
  *out = acc;
  return 0;
}

/* Scores of listed pairs, each from scratch: out[i] = s(layer li[i], query qi[i], pool pi[i]). */
int rc_oracle_score_pairs(int dtype, int mode, int T, int H, int Dh,
                          const uint16_t* kq, const uint16_t* vq, int64_t q_layer_stride,
                          const uint16_t* kp, const uint16_t* vp, int64_t p_layer_stride,
                          int64_t n_pairs, const int32_t* li, const int32_t* qi, const int32_t* pi,
                          double* out) {
  if (T <= 0 || H <= 0 || Dh <= 0 || n_pairs < 0 || !out) return 1;
  if (n_pairs > 0 && (!kq || !vq || !kp || !vp || !li || !qi || !pi)) return 1;
  const int64_t D = (int64_t)T * H * Dh;
  int err = 0;
#pragma omp parallel for schedule(dynamic, 1)
  for (int64_t i = 0; i < n_pairs; ++i) {
    double* buf = (double*)malloc(sizeof(double) * 4 * (size_t)D);
    if (!buf) { err = 2; continue; }
    decode_block(dtype, kq + (int64_t)li[i] * q_layer_stride + (int64_t)qi[i] * D, D, buf);
    decode_block(dtype, vq + (int64_t)li[i] * q_layer_stride + (int64_t)qi[i] * D, D, buf + D);
    decode_block(dtype, kp + (int64_t)li[i] * p_layer_stride + (int64_t)pi[i] * D, D, buf + 2 * D);
    decode_block(dtype, vp + (int64_t)li[i] * p_layer_stride + (int64_t)pi[i] * D, D, buf + 3 * D);
    out[i] = pair_score(buf, buf + D, buf + 2 * D, buf + 3 * D, T, H, Dh, mode);
    free(buf);
  }
  return err;
}

/*
 * Exhaustive search, one layer after the other.
 *   scores_out   optional [L][Q][P] double, the full score matrix (dead blocks included)
 *   best_idx     [L][Q] argmax over live pool blocks, lowest index on exact ties, -1 if none
 *   best_score   [L][Q] its score (-inf if none)
 *   match_idx    [L][Q] best_idx if best_score >= tau else -1
 *   second_score [L][Q] second-largest live score counted with multiplicity (-inf if < 2 live)
 * The squared norms of a block are computed once and reused for every pair it
 * takes part in (the paper's norm caching); sums run in index order.
 */
int rc_oracle_match(int dtype, int mode, int L, int T, int H, int Dh,
                    const uint16_t* kq, const uint16_t* vq, int64_t q_layer_stride, int64_t Q,
                    const uint16_t* kp, const uint16_t* vp, int64_t p_layer_stride, int64_t P,
                    const uint8_t* live, double tau,
                    int32_t* best_idx, double* best_score, int32_t* match_idx, double* second_score,
                    double* scores_out) {
  if (bad_shape(L, T, H, Dh, q_layer_stride, Q) || bad_shape(L, T, H, Dh, p_layer_stride, P)) return 1;
  if (!best_idx || !best_score || !match_idx || !second_score) return 1;
  if (L > 0 && Q > 0 && (!kq || !vq)) return 1;
  if (L > 0 && P > 0 && (!kp || !vp)) return 1;
  const int64_t D = (int64_t)T * H * Dh;
  const int NH = (mode == ORC_BLOCK) ? 1 : H; /* norm slots per block */
  int err = 0;

  double* qk = (double*)malloc(sizeof(double) * (size_t)(Q * D + 1));
  double* qv = (double*)malloc(sizeof(double) * (size_t)(Q * D + 1));
  double* qkn = (double*)malloc(sizeof(double) * (size_t)(Q * NH + 1));
  double* qvn = (double*)malloc(sizeof(double) * (size_t)(Q * NH + 1));
  double* S = (double*)malloc(sizeof(double) * (size_t)(Q * P + 1));
  if (!qk || !qv || !qkn || !qvn || !S) { err = 2; goto done; }

  for (int l = 0; l < L; ++l) {
    for (int64_t q = 0; q < Q; ++q) {
      decode_block(dtype, kq + (int64_t)l * q_layer_stride + q * D, D, qk + q * D);
      decode_block(dtype, vq + (int64_t)l * q_layer_stride + q * D, D, qv + q * D);
      for (int h = 0; h < NH; ++h) {
        int head = (mode == ORC_BLOCK) ? -1 : h;
        qkn[q * NH + h] = sqnorm(qk + q * D, T, H, Dh, head);
        qvn[q * NH + h] = sqnorm(qv + q * D, T, H, Dh, head);
      }
    }
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t p = 0; p < P; ++p) {
      double* pk = (double*)malloc(sizeof(double) * 2 * (size_t)D);
      if (!pk) { err = 2; continue; }
      double* pv = pk + D;
      double pkn[64], pvn[64];
      decode_block(dtype, kp + (int64_t)l * p_layer_stride + p * D, D, pk);
      decode_block(dtype, vp + (int64_t)l * p_layer_stride + p * D, D, pv);
      for (int h = 0; h < NH; ++h) {
        int head = (mode == ORC_BLOCK) ? -1 : h;
        pkn[h] = sqnorm(pk, T, H, Dh, head);
        pvn[h] = sqnorm(pv, T, H, Dh, head);
      }
      for (int64_t q = 0; q < Q; ++q) {
        double s;
        if (mode == ORC_BLOCK) {
          double ck = cosine(dot(qk + q * D, pk, T, H, Dh, -1), qkn[q], pkn[0]);
          double cv = cosine(dot(qv + q * D, pv, T, H, Dh, -1), qvn[q], pvn[0]);
          s = 0.5 * (ck + cv);
        } else {
          s = INFINITY;
          for (int h = 0; h < H; ++h) {
            double ck = cosine(dot(qk + q * D, pk, T, H, Dh, h), qkn[q * NH + h], pkn[h]);
            double cv = cosine(dot(qv + q * D, pv, T, H, Dh, h), qvn[q * NH + h], pvn[h]);
            double sh = 0.5 * (ck + cv);
            if (sh < s) s = sh;
          }
        }
        S[q * P + p] = s;
      }
      free(pk);
    }
    if (err) goto done;
    for (int64_t q = 0; q < Q; ++q) {
      int32_t bi = -1;
      double bs = -INFINITY, ss = -INFINITY;
      for (int64_t p = 0; p < P; ++p) {
        if (live && !live[(int64_t)l * P + p]) continue;
        double s = S[q * P + p];
        if (s > bs) { ss = bs; bs = s; bi = (int32_t)p; }
        else if (s > ss) ss = s;
      }
      best_idx[(int64_t)l * Q + q] = bi;
      best_score[(int64_t)l * Q + q] = bs;
      second_score[(int64_t)l * Q + q] = ss;
      match_idx[(int64_t)l * Q + q] = (bi >= 0 && bs >= tau) ? bi : -1;
    }
    if (scores_out) memcpy(scores_out + (int64_t)l * Q * P, S, sizeof(double) * (size_t)(Q * P));
  }
done:
  free(qk); free(qv); free(qkn); free(qvn); free(S);
  return err;
}

/*
 * Candidate-restricted scoring: Stage 2 as the paper runs it, only on the blocks of the steps
 * that Stage 1 let through (Sec. IV-A, opening of Stage 2; k candidates with k << m in the
 * complexity analysis).  cand[l][q][c] is a pool index or -1.  Each listed pair is scored from scratch
 * with the same score as the exhaustive search; entries that are -1, out of range or dead
 * score -inf.  best = highest score, ties to the lowest pool index; match iff best >= tau.
 */
int rc_oracle_candidates(int dtype, int mode, int L, int T, int H, int Dh,
                         const uint16_t* kq, const uint16_t* vq, int64_t q_layer_stride, int64_t Q,
                         const uint16_t* kp, const uint16_t* vp, int64_t p_layer_stride, int64_t P,
                         const int32_t* cand, int64_t C, const uint8_t* live, double tau,
                         double* scores, int32_t* best_idx, double* best_score, int32_t* match_idx) {
  if (bad_shape(L, T, H, Dh, q_layer_stride, Q) || bad_shape(L, T, H, Dh, p_layer_stride, P) || C < 0) return 1;
  if (!scores || !best_idx || !best_score || !match_idx || (C > 0 && !cand)) return 1;
  const int64_t D = (int64_t)T * H * Dh;
  int err = 0;
#pragma omp parallel for schedule(dynamic, 1)
  for (int64_t lq = 0; lq < (int64_t)L * Q; ++lq) {
    const int64_t l = lq / Q, q = lq % Q;
    double* buf = (double*)malloc(sizeof(double) * 4 * (size_t)D);
    if (!buf) { err = 2; continue; }
    decode_block(dtype, kq + l * q_layer_stride + q * D, D, buf);
    decode_block(dtype, vq + l * q_layer_stride + q * D, D, buf + D);
    int32_t bi = -1;
    double bs = -INFINITY;
    for (int64_t c = 0; c < C; ++c) {
      const int32_t pidx = cand[(l * Q + q) * C + c];
      double s = -INFINITY;
      if (pidx >= 0 && pidx < P && (!live || live[l * P + pidx])) {
        decode_block(dtype, kp + l * p_layer_stride + (int64_t)pidx * D, D, buf + 2 * D);
        decode_block(dtype, vp + l * p_layer_stride + (int64_t)pidx * D, D, buf + 3 * D);
        s = pair_score(buf, buf + D, buf + 2 * D, buf + 3 * D, T, H, Dh, mode);
        if (s > bs || (s == bs && pidx < bi)) { bs = s; bi = pidx; }
      }
      scores[(l * Q + q) * C + c] = s;
    }
    best_idx[lq] = bi;
    best_score[lq] = bs;
    match_idx[lq] = (bi >= 0 && bs >= tau) ? bi : -1;
    free(buf);
  }
  return err;
}

/*
 * Layer-mean block distance, the paper's own Stage 2 measure (Sec. IV-A, the two per-layer
 * distance equations and the block-distance equation): for every layer the Euclidean distance
 * of the flattened K tensors and of the flattened V tensors of the two blocks, each by
 * subtracting and squaring; their sum divided by 2*d*h (d = T tokens per block, h = H KV
 * heads); the mean of that over the N = L layers.  One decision per query block, shared by all
 * layers: the nearest live pool block (lowest index on exact ties), the runner-up distance,
 * match iff the distance is <= thr (so the largest collected distance used as the threshold
 * accepts everything, the p = 100 row of the percentile table).  live is [P], shared by the layers.
 * dist_out, if given, receives the whole [Q][P] matrix.
 */
int rc_oracle_layer_mean(int dtype, int L, int T, int H, int Dh,
                         const uint16_t* kq, const uint16_t* vq, int64_t q_layer_stride, int64_t Q,
                         const uint16_t* kp, const uint16_t* vp, int64_t p_layer_stride, int64_t P,
                         const uint8_t* live, double thr,
                         int32_t* best_idx, double* best_dist, int32_t* match_idx, double* second_dist,
                         double* dist_out) {
  if (L <= 0) return 1; /* a mean over no layers is undefined */
  if (bad_shape(L, T, H, Dh, q_layer_stride, Q) || bad_shape(L, T, H, Dh, p_layer_stride, P)) return 1;
  if (!best_idx || !best_dist || !match_idx || !second_dist) return 1;
  if (Q > 0 && (!kq || !vq)) return 1;
  if (P > 0 && (!kp || !vp)) return 1;
  const int64_t D = (int64_t)T * H * Dh;
  int err = 0;
  double* qk = (double*)malloc(sizeof(double) * (size_t)(Q * D + 1));
  double* qv = (double*)malloc(sizeof(double) * (size_t)(Q * D + 1));
  double* S = (double*)calloc((size_t)(Q * P + 1), sizeof(double)); /* sum over layers */
  if (!qk || !qv || !S) { err = 2; goto done; }
  for (int l = 0; l < L; ++l) {
    for (int64_t q = 0; q < Q; ++q) {
      decode_block(dtype, kq + (int64_t)l * q_layer_stride + q * D, D, qk + q * D);
      decode_block(dtype, vq + (int64_t)l * q_layer_stride + q * D, D, qv + q * D);
    }
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t p = 0; p < P; ++p) {
      double* pk = (double*)malloc(sizeof(double) * 2 * (size_t)D);
      if (!pk) { err = 2; continue; }
      double* pv = pk + D;
      decode_block(dtype, kp + (int64_t)l * p_layer_stride + p * D, D, pk);
      decode_block(dtype, vp + (int64_t)l * p_layer_stride + p * D, D, pv);
      for (int64_t q = 0; q < Q; ++q) {
        double sk = 0.0, sv = 0.0;
        for (int64_t i = 0; i < D; ++i) {
          const double a = qk[q * D + i] - pk[i], b = qv[q * D + i] - pv[i];
          sk += a * a;
          sv += b * b;
        }
        S[q * P + p] += (sqrt(sk) + sqrt(sv)) / (2.0 * T * H);
      }
      free(pk);
    }
    if (err) goto done;
  }
  for (int64_t q = 0; q < Q; ++q) {
    int32_t bi = -1;
    double bd = INFINITY, sd = INFINITY;
    for (int64_t p = 0; p < P; ++p) {
      const double d = S[q * P + p] / L;
      if (dist_out) dist_out[q * P + p] = d;
      if (live && !live[p]) continue;
      if (d < bd) { sd = bd; bd = d; bi = (int32_t)p; }
      else if (d < sd) sd = d;
    }
    best_idx[q] = bi;
    best_dist[q] = bd;
    second_dist[q] = sd;
    match_idx[q] = (bi >= 0 && bd <= thr) ? bi : -1;
  }
done:
  free(qk); free(qv); free(S);
  return err;
}

/*
 * Stage 2 exactly as the paper runs it: the layer-mean block distance (block-distance equation of
 * Sec. IV-A) of the listed candidate pairs only (the blocks of the steps Stage 1 flagged).
 * cand[q][c] is a pool index or -1, the same list for every layer; live is [P].  Each listed pair
 * is computed from scratch by subtracting and squaring; entries that are -1, out of range or dead
 * get +inf.  best = smallest distance, ties to the lowest pool index; match iff best <= thr.
 */
int rc_oracle_candidate_distances(int dtype, int L, int T, int H, int Dh,
                                  const uint16_t* kq, const uint16_t* vq, int64_t q_layer_stride, int64_t Q,
                                  const uint16_t* kp, const uint16_t* vp, int64_t p_layer_stride, int64_t P,
                                  const int32_t* cand, int64_t C, const uint8_t* live, double thr,
                                  double* dist, int32_t* best_idx, double* best_dist, int32_t* match_idx) {
  if (L <= 0) return 1;
  if (bad_shape(L, T, H, Dh, q_layer_stride, Q) || bad_shape(L, T, H, Dh, p_layer_stride, P) || C < 0) return 1;
  if (!best_idx || !best_dist || !match_idx || (C > 0 && (!cand || !dist))) return 1;
  const int64_t D = (int64_t)T * H * Dh;
  int err = 0;
#pragma omp parallel for schedule(dynamic, 1)
  for (int64_t q = 0; q < Q; ++q) {
    double* buf = (double*)malloc(sizeof(double) * 4 * (size_t)D);
    if (!buf) { err = 2; continue; }
    int32_t bi = -1;
    double bd = INFINITY;
    for (int64_t c = 0; c < C; ++c) {
      const int32_t pidx = cand[q * C + c];
      double d = INFINITY;
      if (pidx >= 0 && pidx < P && (!live || live[pidx])) {
        double sum = 0.0;
        for (int l = 0; l < L; ++l) {
          decode_block(dtype, kq + (int64_t)l * q_layer_stride + q * D, D, buf);
          decode_block(dtype, vq + (int64_t)l * q_layer_stride + q * D, D, buf + D);
          decode_block(dtype, kp + (int64_t)l * p_layer_stride + (int64_t)pidx * D, D, buf + 2 * D);
          decode_block(dtype, vp + (int64_t)l * p_layer_stride + (int64_t)pidx * D, D, buf + 3 * D);
          double sk = 0.0, sv = 0.0;
          for (int64_t i = 0; i < D; ++i) {
            const double a = buf[i] - buf[2 * D + i], b = buf[D + i] - buf[3 * D + i];
            sk += a * a;
            sv += b * b;
          }
          sum += (sqrt(sk) + sqrt(sv)) / (2.0 * T * H);
        }
        d = sum / L;
        if (d < bd || (d == bd && pidx < bi)) { bd = d; bi = pidx; }
      }
      dist[q * C + c] = d;
    }
    best_idx[q] = bi;
    best_dist[q] = bd;
    match_idx[q] = (bi >= 0 && bd <= thr) ? bi : -1;
    free(buf);
  }
  return err;
}

/*
 * Percentile-based adaptive threshold (Sec. IV-A, "Percentile-based Adaptive Thresholding"; the
 * parameter paragraph of the evaluation: the p % of the candidates with the lowest distances are
 * kept).  From the distances collected during warm-up the threshold is the p-th percentile by
 * the nearest-rank rule: with n finite samples sorted ascending, the k-th smallest,
 * k = ceil(p/100 * n) clamped to [1, n] (in double).  It is a member of the sample, so the
 * fraction of samples <= threshold is at least p %, and p = 100 gives the maximum (everything
 * collected would have been accepted).  Non-finite samples (a query that had no candidate) are
 * left out.  No finite sample: threshold = -inf (nothing is shared).
 */
static int cmp_float(const void* a, const void* b) {
  const float x = *(const float*)a, y = *(const float*)b;
  return (x > y) - (x < y);
}

int rc_oracle_pat_threshold(const float* samples, int64_t n, double p, float* threshold, int64_t* n_finite) {
  if (n < 0 || (n > 0 && !samples) || !threshold || !n_finite || !(p >= 0.0 && p <= 100.0)) return 1;
  float* s = (float*)malloc(sizeof(float) * (size_t)(n + 1));
  if (!s) return 2;
  int64_t m = 0;
  for (int64_t i = 0; i < n; ++i)
    if (isfinite(samples[i])) s[m++] = samples[i];
  *n_finite = m;
  if (m == 0) {
    *threshold = -INFINITY;
  } else {
    qsort(s, (size_t)m, sizeof(float), cmp_float);
    int64_t k = (int64_t)ceil(p * (double)m / 100.0);
    if (k < 1) k = 1;
    if (k > m) k = m;
    *threshold = s[k - 1];
  }
  free(s);
  return 0;
}

/* The sharing decision against a threshold that was computed, not given: match iff dist <= thr. */
int rc_oracle_apply_threshold(const int32_t* best_idx, const float* best_dist, int64_t n, float thr, int32_t* match_idx) {
  if (n < 0 || (n > 0 && (!best_idx || !best_dist || !match_idx))) return 1;
  for (int64_t i = 0; i < n; ++i) match_idx[i] = (best_idx[i] >= 0 && best_dist[i] <= thr) ? best_idx[i] : -1;
  return 0;
}

/*
 * Streaming pool maintenance (Sec. IV-B: the search runs inside every decoding step, so a block
 * that found no partner stays resident and is itself a candidate from the next step on; Sec. IV-A:
 * its squared norms are computed once and kept with the block).  Every unmatched query block
 * (match_idx[q] < 0), in ascending q, takes the lowest-numbered slot of the pool that is not
 * live: its K and V tensors of every layer and its cached squared norms are stored there and the
 * slot becomes live.  When the free slots run out the remaining queries are left out
 * (slot_of_query = -1).  Matched queries need no slot: their table entries already point at the
 * partner.  nh = norm values per block (1, or H in per-head mode).  Everything is updated in place.
 */
int rc_oracle_pool_admit(int L, int64_t block_elems, int nh,
                         const uint16_t* kq, const uint16_t* vq, int64_t q_layer_stride, int64_t Q,
                         const double* q_ksq, const double* q_vsq,
                         uint16_t* kp, uint16_t* vp, int64_t p_layer_stride, int64_t P,
                         double* p_ksq, double* p_vsq, uint8_t* live, const int32_t* match_idx,
                         int32_t* slot_of_query, int32_t* n_admitted) {
  if (L < 0 || block_elems <= 0 || nh <= 0 || Q < 0 || P < 0 || !slot_of_query || !n_admitted) return 1;
  if (Q > 0 && (!match_idx || (L > 0 && (!kq || !vq || !q_ksq || !q_vsq)))) return 1;
  if (P > 0 && (!live || (L > 0 && (!kp || !vp || !p_ksq || !p_vsq)))) return 1;
  int64_t next = 0; /* next pool slot to look at */
  int32_t count = 0;
  for (int64_t q = 0; q < Q; ++q) {
    slot_of_query[q] = -1;
    if (match_idx[q] >= 0) continue;
    while (next < P && live[next]) ++next;
    if (next >= P) continue; /* pool full */
    const int64_t s = next;
    for (int l = 0; l < L; ++l) {
      memcpy(kp + (int64_t)l * p_layer_stride + s * block_elems, kq + (int64_t)l * q_layer_stride + q * block_elems,
             sizeof(uint16_t) * (size_t)block_elems);
      memcpy(vp + (int64_t)l * p_layer_stride + s * block_elems, vq + (int64_t)l * q_layer_stride + q * block_elems,
             sizeof(uint16_t) * (size_t)block_elems);
      for (int h = 0; h < nh; ++h) {
        p_ksq[((int64_t)l * P + s) * nh + h] = q_ksq[((int64_t)l * Q + q) * nh + h];
        p_vsq[((int64_t)l * P + s) * nh + h] = q_vsq[((int64_t)l * Q + q) * nh + h];
      }
    }
    live[s] = 1;
    slot_of_query[q] = (int32_t)s;
    ++count;
  }
  *n_admitted = count;
  return 0;
}

/*
 * Block metadata update (Sec. IV-A keeps per-block metadata with an LRU order, i.e. a record of when a
 * block was last used): value goes to array[slots[i]] for every listed slot inside [0, P).  Entries
 * outside that range (-1 = "no slot") are skipped.
 */
int rc_oracle_pool_touch(const int32_t* slots, int64_t n, int32_t value, int32_t* array, int64_t P) {
  if (n < 0 || P < 0 || (n > 0 && !slots) || (P > 0 && !array)) return 1;
  for (int64_t i = 0; i < n; ++i)
    if (slots[i] >= 0 && slots[i] < P) array[slots[i]] = value;
  return 0;
}

/*
 * References that the engine drops (a request has ended; Sec. IV-B: a block goes back to the free pool
 * only when its reference count reaches 0): every listed id inside [0, NB) loses one reference, once per
 * time it is listed.
 */
int rc_oracle_refcount_release(const int32_t* ids, int64_t n, int32_t* refcount, int64_t NB) {
  if (n < 0 || NB < 0 || (n > 0 && !ids) || (NB > 0 && !refcount)) return 1;
  for (int64_t i = 0; i < n; ++i)
    if (ids[i] >= 0 && ids[i] < NB) refcount[ids[i]] -= 1;
  return 0;
}

/*
 * Room for the admissions of a step (Sec. IV-B: the evictor returns a block to the free pool only at
 * reference count 0; Sec. IV-A: block metadata is kept in LRU order).
 *   wanted = number of unmatched queries (match_idx[q] < 0) + extra_wanted;
 *   free   = number of slots that are not live.
 * While free < wanted, the live slot that nobody references (refcount[p] == 0; any live slot when refcount
 * is NULL) and that was used least recently (smallest last_used, equal values by lowest slot number) leaves
 * the pool (live = 0).  Referenced slots never leave; when the unreferenced ones run out the loop stops.
 */
int rc_oracle_pool_evict(int64_t P, uint8_t* live, const int32_t* refcount, const int32_t* last_used,
                         const int32_t* match_idx, int64_t Q, int64_t extra_wanted, int32_t* n_free,
                         int32_t* n_evicted) {
  if (P < 0 || Q < 0 || extra_wanted < 0 || !n_free || !n_evicted) return 1;
  if ((P > 0 && (!live || !last_used)) || (Q > 0 && !match_idx)) return 1;
  int64_t wanted = extra_wanted, free_slots = 0, evicted = 0;
  for (int64_t q = 0; q < Q; ++q) wanted += match_idx[q] < 0;
  for (int64_t p = 0; p < P; ++p) free_slots += !live[p];
  while (free_slots < wanted) {
    int64_t victim = -1;
    for (int64_t p = 0; p < P; ++p) {
      if (!live[p] || (refcount && refcount[p] != 0)) continue;
      if (victim < 0 || last_used[p] < last_used[victim]) victim = p; /* strict: the lowest slot wins a tie */
    }
    if (victim < 0) break;
    live[victim] = 0;
    ++free_slots;
    ++evicted;
  }
  *n_free = (int32_t)free_slots;
  *n_evicted = (int32_t)evicted;
  return 0;
}

/*
 * Block-table remap with reference counts (Sec. IV-B), per layer:
 *   redirect = identity on [0, NB); redirect[query_ids[q]] = target(match_idx[q]) for matched q,
 *   target(m) = pool_ids ? pool_ids[m] : m;
 *   tables_out[e] = redirect[tables_in[e]] for entries in [0, NB), other entries pass through;
 *   cnt[b] = number of entries of tables_in equal to b;
 *   for matched q (b = query_ids[q], m its target): rc[m] += cnt[b]; rc[b] -= cnt[b];
 *   freed[q] = (rc[b] == 0);   n_remapped = number of entries whose value changed.
 * tables_out / refcount_out may alias their inputs.
 */
int rc_oracle_remap(int L, const int32_t* tables_in, int32_t* tables_out, int64_t R, int64_t E,
                    const int32_t* query_ids, const int32_t* pool_ids, const int32_t* match_idx,
                    int64_t Q, int64_t P, int64_t NB,
                    const int32_t* refcount_in, int32_t* refcount_out,
                    uint8_t* freed, int32_t* n_remapped) {
  if (L < 0 || R < 0 || E < 0 || Q < 0 || P < 0 || NB < 0) return 1;
  if (L > 0 && (!n_remapped || (R * E > 0 && (!tables_in || !tables_out)) ||
                (NB > 0 && (!refcount_in || !refcount_out)) || (Q > 0 && (!query_ids || !match_idx || !freed))))
    return 1;
  for (int64_t q = 0; q < Q; ++q)
    if (query_ids[q] < 0 || query_ids[q] >= NB) return 1;
  for (int64_t p = 0; pool_ids && p < P; ++p)
    if (pool_ids[p] < 0 || pool_ids[p] >= NB) return 1;
  if (!pool_ids && P > NB) return 1;
  int32_t* redirect = (int32_t*)malloc(sizeof(int32_t) * (size_t)(NB + 1));
  int64_t* cnt = (int64_t*)malloc(sizeof(int64_t) * (size_t)(NB + 1));
  if (!redirect || !cnt) { free(redirect); free(cnt); return 2; }
  for (int l = 0; l < L; ++l) {
    const int32_t* tin = tables_in + (int64_t)l * R * E;
    int32_t* tout = tables_out + (int64_t)l * R * E;
    const int32_t* m = match_idx + (int64_t)l * Q;
    for (int64_t b = 0; b < NB; ++b) { redirect[b] = (int32_t)b; cnt[b] = 0; }
    for (int64_t q = 0; q < Q; ++q)
      if (m[q] >= 0 && m[q] < P) redirect[query_ids[q]] = pool_ids ? pool_ids[m[q]] : m[q];
    int32_t changed = 0;
    for (int64_t e = 0; e < R * E; ++e) {
      int32_t b = tin[e];
      if (b >= 0 && b < NB) {
        cnt[b] += 1;
        if (redirect[b] != b) changed += 1;
        tout[e] = redirect[b];
      } else {
        tout[e] = b;
      }
    }
    for (int64_t b = 0; b < NB; ++b) refcount_out[(int64_t)l * NB + b] = refcount_in[(int64_t)l * NB + b];
    for (int64_t q = 0; q < Q; ++q) {
      freed[(int64_t)l * Q + q] = 0;
      if (m[q] < 0 || m[q] >= P) continue;
      int32_t b = query_ids[q], tgt = redirect[b];
      refcount_out[(int64_t)l * NB + tgt] += (int32_t)cnt[b];
      refcount_out[(int64_t)l * NB + b] -= (int32_t)cnt[b];
    }
    for (int64_t q = 0; q < Q; ++q)
      if (m[q] >= 0 && m[q] < P) freed[(int64_t)l * Q + q] = (refcount_out[(int64_t)l * NB + query_ids[q]] == 0);
    n_remapped[l] = changed;
  }
  free(redirect);
  free(cnt);
  return 0;
}
