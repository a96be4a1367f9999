// rc_score_candidates: Stage 2 restricted to listed candidates (ReasonCache Sec. IV-A: only the
// blocks of the steps flagged by Stage 1 are compared).  HBM-bound gather: one workgroup per listed
// pair streams the pool block's K and V tensors (the query block comes from the L2, which the other
// candidates of the same query keep warm), accumulates the dot products in fp32 and normalises with
// the cached squared norms.  A second small kernel picks the best candidate of every list.
#include <hip/hip_runtime.h>

#include "rc_common.hpp"

namespace rc {
namespace {

constexpr int kCandThreads = 256;

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// <x, y> of the 8 fp16 / bf16 values packed in two 16-byte words, accumulated in fp32.
template <bool BF16>
__device__ __forceinline__ float dot8(u32x4 x, u32x4 y, float acc) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const unsigned int xi = x[i], yi = y[i];  // copies: a bit_cast applied to the vector element itself reads lane 0
    if (BF16) {
      acc = fmaf(__uint_as_float(xi << 16), __uint_as_float(yi << 16), acc);
      acc = fmaf(__uint_as_float(xi & 0xffff0000u), __uint_as_float(yi & 0xffff0000u), acc);
    } else {
      acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, xi), __builtin_bit_cast(half2_t, yi), acc, false);
    }
  }
  return acc;
}

struct CandParams {
  const char *kq, *vq, *kp, *vp;
  const float *q_ksq, *q_vsq, *p_ksq, *p_vsq;
  const uint8_t* live;
  const int32_t* cand;
  float* scores;
  long long q_lstride_b, p_lstride_b;
  int Q, P, C;
  int block_bytes;  // one K (or V) tensor of a block
  int heads;        // 1 in block mode, H in per-head-all mode
};

// grid = (ceil(C / kCandPerWg), Q, L).  A workgroup scores kCandPerWg candidates of one query: the query
// chunk a thread holds is used against all of them, which divides the query traffic from the L2.
// Thread t takes the 16-byte chunks t, t+256, ...; 16 consecutive chunks are one head of one
// token, so with 16*heads dividing 256 a thread stays in one head: head = (t/16) % heads.
// ANYH (per-head mode with a head count that does not divide 16, e.g. 10 KV heads): the head of a
// thread's chunk changes from one trip to the next, so every trip ends with the sum over the 16
// lanes of a (token, head) group, added by the group's first lane to its own slot
// hpart[candidate][K or V][head][group]: no two groups share a slot, so plain LDS updates do.
constexpr int kCandPerWg = 16;

template <bool BF16, bool ANYH>
__global__ __launch_bounds__(kCandThreads) void candidates_kernel(const CandParams p) {
  __shared__ float part[kCandPerWg][2][kCandThreads / 16];
  __shared__ float head_score[kCandPerWg][16];
  __shared__ float hpart[ANYH ? kCandPerWg : 1][2][ANYH ? 16 : 1][ANYH ? kCandThreads / 16 : 1];
  const int c0 = blockIdx.x * kCandPerWg, q = blockIdx.y, tid = threadIdx.x;
  const long long l = blockIdx.z;
  const long long slot0 = (l * p.Q + q) * p.C + c0;
  int pidx[kCandPerWg];
  bool valid[kCandPerWg];
  const u32x4* xp_k[kCandPerWg];
  const u32x4* xp_v[kCandPerWg];
  bool any = false;
#pragma unroll
  for (int c = 0; c < kCandPerWg; ++c) {  // the same for the whole workgroup
    pidx[c] = (c0 + c < p.C) ? p.cand[slot0 + c] : -1;
    valid[c] = pidx[c] >= 0 && pidx[c] < p.P && (!p.live || p.live[l * p.P + pidx[c]]);
    const long long off = l * p.p_lstride_b + (long long)(valid[c] ? pidx[c] : 0) * p.block_bytes;
    xp_k[c] = reinterpret_cast<const u32x4*>(p.kp + off);
    xp_v[c] = reinterpret_cast<const u32x4*>(p.vp + off);
    any = any || valid[c];
    if (!valid[c] && tid == 0 && c0 + c < p.C) p.scores[slot0 + c] = -INFINITY;
  }
  if (!any) return;
  if (ANYH) {
    float* z = &hpart[0][0][0][0];
    for (int i = tid; i < kCandPerWg * 2 * 16 * (kCandThreads / 16); i += kCandThreads) z[i] = 0.f;
    __syncthreads();
  }
  const u32x4* xq_k = reinterpret_cast<const u32x4*>(p.kq + l * p.q_lstride_b + (long long)q * p.block_bytes);
  const u32x4* xq_v = reinterpret_cast<const u32x4*>(p.vq + l * p.q_lstride_b + (long long)q * p.block_bytes);
  const int chunks = p.block_bytes / 16;
  float dk[kCandPerWg], dv[kCandPerWg];
#pragma unroll
  for (int c = 0; c < kCandPerWg; ++c) dk[c] = dv[c] = 0.f;
  auto trip = [&](int i) {
    const u32x4 qk = xq_k[i], qv = xq_v[i];
    u32x4 pk[kCandPerWg], pv[kCandPerWg];
#pragma unroll
    for (int c = 0; c < kCandPerWg; ++c)
      if (valid[c]) {
        pk[c] = __builtin_nontemporal_load(xp_k[c] + i);
        pv[c] = __builtin_nontemporal_load(xp_v[c] + i);
      }
#pragma unroll
    for (int c = 0; c < kCandPerWg; ++c)
      if (valid[c]) {
        dk[c] = dot8<BF16>(qk, pk[c], dk[c]);
        dv[c] = dot8<BF16>(qv, pv[c], dv[c]);
      }
    if (ANYH) {
      const int head = (i >> 4) % p.heads;
#pragma unroll
      for (int c = 0; c < kCandPerWg; ++c)
        if (valid[c]) {  // the same for the whole workgroup
#pragma unroll
          for (int off = 8; off > 0; off >>= 1) {
            dk[c] += __shfl_xor(dk[c], off);
            dv[c] += __shfl_xor(dv[c], off);
          }
          if ((tid & 15) == 0) {
            hpart[c][0][head][tid >> 4] += dk[c];
            hpart[c][1][head][tid >> 4] += dv[c];
          }
          dk[c] = dv[c] = 0.f;
        }
    }
  
  };
  // chunks = 16*T*H is a multiple of 256
  if (ANYH) {
    for (int i = tid; i < chunks; i += kCandThreads) trip(i);
  } else {
#pragma unroll 2
    for (int i = tid; i < chunks; i += kCandThreads) trip(i);
  }
  // sum over the 16 lanes that share a (token, head) group, then over the groups of a head
#pragma unroll
  for (int c = 0; c < kCandPerWg; ++c) {
#pragma unroll
    for (int off = 8; off > 0; off >>= 1) {
      dk[c] += __shfl_xor(dk[c], off);
      dv[c] += __shfl_xor(dv[c], off);
    }
    if ((tid & 15) == 0) {
      part[c][0][tid >> 4] = dk[c];
      part[c][1][tid >> 4] = dv[c];
    }
  }
  __syncthreads();
  const int c = tid >> 4, h = tid & 15;  // one thread per (candidate, head)
  if (c < kCandPerWg && h < p.heads && valid[c]) {
    float sk = 0.f, sv = 0.f;
    if (ANYH) {
      for (int g = 0; g < kCandThreads / 16; ++g) {
        sk += hpart[c][0][h][g];
        sv += hpart[c][1][h][g];
      }
    } else {
      for (int g = h; g < kCandThreads / 16; g += p.heads) {
        sk += part[c][0][g];
        sv += part[c][1][g];
      }
    }
    const long long oq = (l * p.Q + q) * p.heads + h, op = (l * p.P + pidx[c]) * p.heads + h;
    const float nkq = p.q_ksq[oq], nvq = p.q_vsq[oq], nkp = p.p_ksq[op], nvp = p.p_vsq[op];
    const float ck = (nkq > 0.f && nkp > 0.f) ? sk * __builtin_amdgcn_rsqf(nkq) * __builtin_amdgcn_rsqf(nkp) : 0.f;
    const float cv = (nvq > 0.f && nvp > 0.f) ? sv * __builtin_amdgcn_rsqf(nvq) * __builtin_amdgcn_rsqf(nvp) : 0.f;
    head_score[c][h] = 0.5f * (ck + cv);
  }
  __syncthreads();
  if (tid < kCandPerWg && valid[tid]) {
    float s = head_score[tid][0];
    for (int hh = 1; hh < p.heads; ++hh) s = fminf(s, head_score[tid][hh]);
    p.scores[slot0 + tid] = s;
  }
}

// One thread per (layer, query): best of its list, equal scores to the lowest pool index.
__global__ __launch_bounds__(256) void candidates_select_kernel(const float* __restrict__ scores,
                                                                const int32_t* __restrict__ cand, long long LQ, int C,
                                                                float tau, int32_t* __restrict__ best_idx,
                                                                float* __restrict__ best_score,
                                                                int32_t* __restrict__ match_idx) {
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= LQ) return;
  float best = -INFINITY;
  int bidx = -1;
  for (int c = 0; c < C; ++c) {
    const float s = scores[i * C + c];
    const int pi = cand[i * C + c];
    if (s == -INFINITY) continue;  // empty, out of range or dead
    if (s > best || (s == best && pi < bidx) || bidx < 0) {
      best = s;
      bidx = pi;
    }
  }
  best_idx[i] = bidx;
  best_score[i] = best;
  match_idx[i] = (bidx >= 0 && best >= tau) ? bidx : -1;
}

// ---- layer-mean Euclidean distance of listed pairs (Stage 2 exactly as Sec. IV-A runs it)

typedef float float2_t __attribute__((ext_vector_type(2)));

// sum of (x - y)^2 over the 8 fp16 / bf16 values of two 16-byte words, in fp32 (differences of
// 16-bit values are exact in fp32, so only the squares and the sum round).
template <bool BF16>
__device__ __forceinline__ float sqdiff8(u32x4 x, u32x4 y, float acc) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const unsigned int xi = x[i], yi = y[i];
    float a0, a1, b0, b1;
    if (BF16) {
      a0 = __uint_as_float(xi << 16);
      a1 = __uint_as_float(xi & 0xffff0000u);
      b0 = __uint_as_float(yi << 16);
      b1 = __uint_as_float(yi & 0xffff0000u);
    } else {
      const float2_t a = __builtin_convertvector(__builtin_bit_cast(half2_t, xi), float2_t);
      const float2_t b = __builtin_convertvector(__builtin_bit_cast(half2_t, yi), float2_t);
      a0 = a[0];
      a1 = a[1];
      b0 = b[0];
      b1 = b[1];
    }
    const float d0 = a0 - b0, d1 = a1 - b1;
    acc = fmaf(d0, d0, acc);
    acc = fmaf(d1, d1, acc);
  }
  return acc;
}

struct CandDistParams {
  const char *kq, *vq, *kp, *vp;
  const uint8_t* live;   // [P] or null
  const int32_t* cand;   // [Q][C]
  float* part;           // [groups][Q][C]: sum over the group's layers of |Kq-Kp| + |Vq-Vp|
  long long q_lstride_b, p_lstride_b;
  int Q, P, C, L, G;     // G = layers per group
  int block_bytes;
};

// grid = (ceil(C / kCandPerWg), Q, layer groups).  The workgroup walks the layers of its group; per
// layer it streams the listed pool blocks against the query chunk held in registers, reduces the
// squared differences over the workgroup and adds the two square roots to the running sum that
// thread c keeps for candidate c.
template <bool BF16>
__global__ __launch_bounds__(kCandThreads) void candidate_distances_kernel(const CandDistParams p) {
  __shared__ float s_red[kCandThreads / 64][kCandPerWg][2];
  const int c0 = blockIdx.x * kCandPerWg, q = blockIdx.y, tid = threadIdx.x;
  const int l0 = blockIdx.z * p.G, nl = min(p.G, p.L - l0);
  int pidx[kCandPerWg];
  bool valid[kCandPerWg];
  bool any = false;
#pragma unroll
  for (int c = 0; c < kCandPerWg; ++c) {  // the same for the whole workgroup
    pidx[c] = (c0 + c < p.C) ? p.cand[(long long)q * p.C + c0 + c] : -1;
    valid[c] = pidx[c] >= 0 && pidx[c] < p.P && (!p.live || p.live[pidx[c]]);
    any = any || valid[c];
  }
  if (!any) return;  // the selection kernel derives validity itself and never reads these sums
  const int chunks = p.block_bytes / 16;
  float total = 0.f;
  for (int li = 0; li < nl; ++li) {
    const long long l = l0 + li;
    const u32x4* xq_k = reinterpret_cast<const u32x4*>(p.kq + l * p.q_lstride_b + (long long)q * p.block_bytes);
    const u32x4* xq_v = reinterpret_cast<const u32x4*>(p.vq + l * p.q_lstride_b + (long long)q * p.block_bytes);
    float dk[kCandPerWg], dv[kCandPerWg];
#pragma unroll
    for (int c = 0; c < kCandPerWg; ++c) dk[c] = dv[c] = 0.f;
    for (int i = tid; i < chunks; i += kCandThreads) {
      const u32x4 qk = xq_k[i], qv = xq_v[i];
      u32x4 pk[kCandPerWg], pv[kCandPerWg];
#pragma unroll
      for (int c = 0; c < kCandPerWg; ++c)
        if (valid[c]) {
          const long long off = l * p.p_lstride_b + (long long)pidx[c] * p.block_bytes;
          pk[c] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p.kp + off) + i);
          pv[c] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p.vp + off) + i);
        }
#pragma unroll
      for (int c = 0; c < kCandPerWg; ++c)
        if (valid[c]) {
          dk[c] = sqdiff8<BF16>(qk, pk[c], dk[c]);
          dv[c] = sqdiff8<BF16>(qv, pv[c], dv[c]);
        }
    }
#pragma unroll
    for (int c = 0; c < kCandPerWg; ++c) {
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) {
        dk[c] += __shfl_xor(dk[c], off);
        dv[c] += __shfl_xor(dv[c], off);
      }
      if ((tid & 63) == 0) {
        s_red[tid >> 6][c][0] = dk[c];
        s_red[tid >> 6][c][1] = dv[c];
      }
    }
    __syncthreads();
    if (tid < kCandPerWg) {
      float sk = 0.f, sv = 0.f;
#pragma unroll
      for (int w = 0; w < kCandThreads / 64; ++w) {
        sk += s_red[w][tid][0];
        sv += s_red[w][tid][1];
      }
      total += __builtin_amdgcn_sqrtf(sk) + __builtin_amdgcn_sqrtf(sv);
    }
    __syncthreads();  // s_red is rewritten by the next layer
  }
  if (tid < kCandPerWg && c0 + tid < p.C)
    p.part[((long long)blockIdx.z * p.Q + q) * p.C + c0 + tid] = total;
}

// One thread per query: layer groups added in order, scaled, validity re-derived, nearest candidate.
__global__ __launch_bounds__(256) void candidate_distances_select_kernel(const float* __restrict__ part, int groups,
                                                                        const int32_t* __restrict__ cand,
                                                                        const uint8_t* __restrict__ live, int Q, int P,
                                                                        int C, float scale, float thr,
                                                                        float* __restrict__ dist,
                                                                        int32_t* __restrict__ best_idx,
                                                                        float* __restrict__ best_dist,
                                                                        int32_t* __restrict__ match_idx) {
  const int q = blockIdx.x * blockDim.x + threadIdx.x;
  if (q >= Q) return;
  float best = INFINITY;
  int bidx = -1;
  for (int c = 0; c < C; ++c) {
    const int pi = cand[(long long)q * C + c];
    float d = INFINITY;
    if (pi >= 0 && pi < P && (!live || live[pi])) {
      float sum = 0.f;
      for (int g = 0; g < groups; ++g) sum += part[((long long)g * Q + q) * C + c];
      d = sum * scale;
      if (d < best || (d == best && pi < bidx)) {
        best = d;
        bidx = pi;
      }
    }
    dist[(long long)q * C + c] = d;
  }
  best_idx[q] = bidx;
  best_dist[q] = best;
  match_idx[q] = (bidx >= 0 && best <= thr) ? bidx : -1;
}

// layers per group: enough workgroups to fill the chip, as few groups as that allows
inline int cand_layers_per_group(int L, int64_t Q, int64_t C) {
  const int64_t wgs = Q * ((C + kCandPerWg - 1) / kCandPerWg);
  int64_t groups = (4096 + wgs - 1) / (wgs > 0 ? wgs : 1);
  if (groups < 1) groups = 1;
  if (groups > L) groups = L;
  return (int)((L + groups - 1) / groups);
}

}  // namespace
}  // namespace rc

extern "C" rc_status rc_score_candidates(const rc_kv_desc* qdesc, const rc_kv_desc* pdesc, int32_t mode,
                                         const void* kq, const void* vq, int64_t Q, const float* q_ksq,
                                         const float* q_vsq, const void* kp, const void* vp, int64_t P,
                                         const float* p_ksq, const float* p_vsq, const uint8_t* pool_live,
                                         const int32_t* cand, int64_t C, float tau, float* scores, int32_t* best_idx,
                                         float* best_score, int32_t* match_idx, void* hip_stream) {
  using namespace rc;
  clear_error();
  if (rc_status s = check_desc(qdesc, Q, "rc_score_candidates(query)")) return s;
  if (rc_status s = check_desc(pdesc, P, "rc_score_candidates(pool)")) return s;
  if (mode != RC_SCORE_BLOCK && mode != RC_SCORE_PER_HEAD_ALL)
    return fail(RC_ERR_UNSUPPORTED, "rc_score_candidates: mode %d", mode);
  if (qdesc->n_layers != pdesc->n_layers || qdesc->block_tokens != pdesc->block_tokens ||
      qdesc->n_kv_heads != pdesc->n_kv_heads || qdesc->head_dim != pdesc->head_dim || qdesc->dtype != pdesc->dtype)
    return fail(RC_ERR_INVALID_ARG, "rc_score_candidates: query and pool descriptors differ in more than layer_stride");
  if (C < 0) return fail(RC_ERR_INVALID_ARG, "rc_score_candidates: negative C");
  if (!(tau == tau)) return fail(RC_ERR_INVALID_ARG, "rc_score_candidates: tau is NaN");
  const int H = qdesc->n_kv_heads;
  const int L = qdesc->n_layers;
  if (L == 0 || Q == 0) return RC_OK;
  if (!kq || !vq || !q_ksq || !q_vsq || !best_idx || !best_score || !match_idx)
    return fail(RC_ERR_INVALID_ARG, "rc_score_candidates: NULL query or output pointer");
  if (C > 0 && (!cand || !scores)) return fail(RC_ERR_INVALID_ARG, "rc_score_candidates: NULL cand or scores");
  if (C > 0 && P > 0 && (!kp || !vp || !p_ksq || !p_vsq))
    return fail(RC_ERR_INVALID_ARG, "rc_score_candidates: NULL pool pointer");
  if (!aligned16(kq) || !aligned16(vq) || !aligned16(kp) || !aligned16(vp))
    return fail(RC_ERR_INVALID_ARG, "rc_score_candidates: KV pointer not 16-byte aligned");
  if (C > 0x7fffffffLL || Q > 65535 || L > 65535 || P > 0x7fffffffLL)
    return fail(RC_ERR_UNSUPPORTED, "rc_score_candidates: C, Q or L beyond the grid limits");
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  if (C > 0) {
    CandParams cp;
    cp.kq = static_cast<const char*>(kq);
    cp.vq = static_cast<const char*>(vq);
    cp.kp = static_cast<const char*>(kp);
    cp.vp = static_cast<const char*>(vp);
    cp.q_ksq = q_ksq;
    cp.q_vsq = q_vsq;
    cp.p_ksq = p_ksq;
    cp.p_vsq = p_vsq;
    cp.live = pool_live;
    cp.cand = cand;
    cp.scores = scores;
    cp.q_lstride_b = qdesc->layer_stride * 2;
    cp.p_lstride_b = pdesc->layer_stride * 2;
    cp.Q = (int)Q;
    cp.P = (int)P;
    cp.C = (int)C;
    cp.block_bytes = qdesc->block_tokens * H * qdesc->head_dim * 2;  // T >= 16, Dh = 128: a multiple of 16 KB / 4
    cp.heads = (mode == RC_SCORE_BLOCK) ? 1 : H;
    const dim3 grid((unsigned)((C + kCandPerWg - 1) / kCandPerWg), (unsigned)Q, (unsigned)L);
    const bool any_h = mode == RC_SCORE_PER_HEAD_ALL && (16 % H) != 0;  // a thread's chunks wander over the heads
    if (qdesc->dtype == RC_BF16) {
      if (any_h)
        candidates_kernel<true, true><<<grid, kCandThreads, 0, st>>>(cp);
      else
        candidates_kernel<true, false><<<grid, kCandThreads, 0, st>>>(cp);
    } else {
      if (any_h)
        candidates_kernel<false, true><<<grid, kCandThreads, 0, st>>>(cp);
      else
        candidates_kernel<false, false><<<grid, kCandThreads, 0, st>>>(cp);
    }
    if (rc_status s = check_launch("rc_score_candidates(score)")) return s;
  }
  const long long LQ = (long long)L * Q;
  candidates_select_kernel<<<(unsigned)((LQ + 255) / 256), 256, 0, st>>>(scores, cand, LQ, (int)C, tau, best_idx,
                                                                         best_score, match_idx);
  return check_launch("rc_score_candidates(select)");
}

extern "C" size_t rc_candidate_distances_workspace_size(const rc_kv_desc* qdesc, int64_t Q, int64_t C) {
  using namespace rc;
  if (!qdesc || Q < 0 || C < 0 || qdesc->n_layers <= 0) return 0;
  const int G = cand_layers_per_group(qdesc->n_layers, Q, C);
  const int64_t groups = (qdesc->n_layers + G - 1) / G;
  const int64_t n = groups * Q * C;
  return (size_t)(n > 0 ? n : 1) * sizeof(float);
}

extern "C" rc_status rc_candidate_distances(const rc_kv_desc* qdesc, const rc_kv_desc* pdesc, const void* kq,
                                            const void* vq, int64_t Q, const void* kp, const void* vp, int64_t P,
                                            const uint8_t* pool_live, const int32_t* cand, int64_t C, float threshold,
                                            float* dist, int32_t* best_idx, float* best_dist, int32_t* match_idx,
                                            void* workspace, size_t workspace_bytes, void* hip_stream) {
  using namespace rc;
  clear_error();
  if (rc_status s = check_desc(qdesc, Q, "rc_candidate_distances(query)")) return s;
  if (rc_status s = check_desc(pdesc, P, "rc_candidate_distances(pool)")) return s;
  if (qdesc->n_layers != pdesc->n_layers || qdesc->block_tokens != pdesc->block_tokens ||
      qdesc->n_kv_heads != pdesc->n_kv_heads || qdesc->head_dim != pdesc->head_dim || qdesc->dtype != pdesc->dtype)
    return fail(RC_ERR_INVALID_ARG, "rc_candidate_distances: query and pool descriptors differ in more than layer_stride");
  if (C < 0) return fail(RC_ERR_INVALID_ARG, "rc_candidate_distances: negative C");
  if (!(threshold == threshold)) return fail(RC_ERR_INVALID_ARG, "rc_candidate_distances: threshold is NaN");
  const int L = qdesc->n_layers;
  if (L <= 0) return fail(RC_ERR_INVALID_ARG, "rc_candidate_distances: a mean over %d layers is undefined", L);
  if (Q == 0) return RC_OK;
  if (!kq || !vq || !best_idx || !best_dist || !match_idx)
    return fail(RC_ERR_INVALID_ARG, "rc_candidate_distances: NULL query or output pointer");
  if (C > 0 && (!cand || !dist)) return fail(RC_ERR_INVALID_ARG, "rc_candidate_distances: NULL cand or dist");
  if (C > 0 && P > 0 && (!kp || !vp)) return fail(RC_ERR_INVALID_ARG, "rc_candidate_distances: NULL pool pointer");
  if (!aligned16(kq) || !aligned16(vq) || !aligned16(kp) || !aligned16(vp))
    return fail(RC_ERR_INVALID_ARG, "rc_candidate_distances: KV pointer not 16-byte aligned");
  if (C > 0x7fffffffLL || Q > 65535 || P > 0x7fffffffLL || L > 65535)
    return fail(RC_ERR_UNSUPPORTED, "rc_candidate_distances: C, Q, P or L beyond the grid limits");
  const size_t need = rc_candidate_distances_workspace_size(qdesc, Q, C);
  if (!workspace || workspace_bytes < need || !aligned16(workspace))
    return fail(RC_ERR_WORKSPACE, "rc_candidate_distances: workspace of %zu bytes needed (16-byte aligned), got %zu", need,
                workspace_bytes);
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const int G = cand_layers_per_group(L, Q, C);
  const int groups = (L + G - 1) / G;
  float* part = static_cast<float*>(workspace);
  if (C > 0 && P > 0) {
    CandDistParams cp;
    cp.kq = static_cast<const char*>(kq);
    cp.vq = static_cast<const char*>(vq);
    cp.kp = static_cast<const char*>(kp);
    cp.vp = static_cast<const char*>(vp);
    cp.live = pool_live;
    cp.cand = cand;
    cp.part = part;
    cp.q_lstride_b = qdesc->layer_stride * 2;
    cp.p_lstride_b = pdesc->layer_stride * 2;
    cp.Q = (int)Q;
    cp.P = (int)P;
    cp.C = (int)C;
    cp.L = L;
    cp.G = G;
    cp.block_bytes = qdesc->block_tokens * qdesc->n_kv_heads * qdesc->head_dim * 2;
    const dim3 grid((unsigned)((C + kCandPerWg - 1) / kCandPerWg), (unsigned)Q, (unsigned)groups);
    if (qdesc->dtype == RC_BF16)
      candidate_distances_kernel<true><<<grid, kCandThreads, 0, st>>>(cp);
    else
      candidate_distances_kernel<false><<<grid, kCandThreads, 0, st>>>(cp);
    if (rc_status s = check_launch("rc_candidate_distances(distances)")) return s;
  }
  const float scale = 1.0f / ((float)L * 2.0f * (float)qdesc->block_tokens * (float)qdesc->n_kv_heads);
  candidate_distances_select_kernel<<<(unsigned)((Q + 255) / 256), 256, 0, st>>>(part, groups, cand, pool_live, (int)Q,
                                                                               (int)P, (int)C, scale, threshold, dist,
                                                                               best_idx, best_dist, match_idx);
  return check_launch("rc_candidate_distances(select)");
}
