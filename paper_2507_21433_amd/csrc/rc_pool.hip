// rc_pool_admit: streaming pool maintenance (ReasonCache Sec. IV-B: the search runs inside every
// decoding step, so a new block that found no partner stays resident and is a candidate from the
// next step on; Sec. IV-A: its squared norms are computed once and kept with the block).
// Unmatched query blocks, in ascending order, take the lowest free pool slots.  Four launches,
// no atomics: (1) dead slots per chunk of the pool, (2) one workgroup scans the chunk counts and
// ranks the unmatched queries, (3) every chunk ranks its dead slots and pairs slot rank r with
// unmatched query r, (4) one workgroup per (pair, layer) copies the K and V tensors and the norms.
#include <hip/hip_runtime.h>

#include "rc_common.hpp"

namespace rc {
namespace {

constexpr int kChunk = 4096;  // pool slots per workgroup: 256 threads x 16 consecutive slots

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// Exclusive prefix sum over the workgroup's values (NT threads, NT a multiple of 64); total = sum.
template <int NT>
__device__ __forceinline__ int block_exclusive_scan(int v, int* s_wave /* [NT / 64 + 1] */, int& total) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int incl = v;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int n = __shfl_up(incl, off);
    if (lane >= off) incl += n;
  }
  __syncthreads();  // s_wave may still be read from a previous call
  if (lane == 63) s_wave[wave] = incl;
  __syncthreads();
  int before = 0, sum = 0;
#pragma unroll
  for (int w = 0; w < NT / 64; ++w) {
    const int c = s_wave[w];
    before += (w < wave) ? c : 0;
    sum += c;
  }
  total = sum;
  return before + incl - v;
}

__global__ __launch_bounds__(256) void admit_count_kernel(const uint8_t* __restrict__ live, int P,
                                                          int* __restrict__ chunk_dead) {
  __shared__ int s_wave[5];
  const int base = blockIdx.x * kChunk + threadIdx.x * 16;
  int dead = 0;
#pragma unroll
  for (int i = 0; i < 16; ++i) dead += (base + i < P) && !live[base + i];
  int total;
  block_exclusive_scan<256>(dead, s_wave, total);
  if (threadIdx.x == 0) chunk_dead[blockIdx.x] = total;
}

// One workgroup: chunk_off = exclusive scan of chunk_dead; unmatched queries ranked in ascending
// order; n_admitted = min(free slots, unmatched queries); slot_of_query starts at -1.
__global__ __launch_bounds__(1024) void admit_scan_kernel(const int* __restrict__ chunk_dead, int nchunks,
                                                          int* __restrict__ chunk_off,
                                                          const int32_t* __restrict__ match_idx, int Q,
                                                          int* __restrict__ unmatched, int32_t* __restrict__ slot_of_query,
                                                          int32_t* __restrict__ n_admitted) {
  __shared__ int s_wave[17];
  const int tid = threadIdx.x;
  int carry = 0;
  for (int b = 0; b < nchunks; b += 1024) {
    const int v = (b + tid < nchunks) ? chunk_dead[b + tid] : 0;
    int total;
    const int ex = block_exclusive_scan<1024>(v, s_wave, total);
    if (b + tid < nchunks) chunk_off[b + tid] = carry + ex;
    carry += total;
  }
  const int n_free = carry;
  int rank0 = 0;
  for (int b = 0; b < Q; b += 1024) {
    const int q = b + tid;
    const int v = (q < Q) && (match_idx[q] < 0);
    int total;
    const int ex = block_exclusive_scan<1024>(v, s_wave, total);
    if (q < Q) {
      slot_of_query[q] = -1;
      if (v) unmatched[rank0 + ex] = q;
    }
    rank0 += total;
  }
  if (tid == 0) *n_admitted = min(n_free, rank0);
}

__global__ __launch_bounds__(256) void admit_assign_kernel(uint8_t* __restrict__ live, int P,
                                                           const int* __restrict__ chunk_off,
                                                           const int* __restrict__ unmatched,
                                                           const int32_t* __restrict__ n_admitted,
                                                           int32_t* __restrict__ slot_of_query,
                                                           int* __restrict__ pair_q, int* __restrict__ pair_slot) {
  __shared__ int s_wave[5];
  const int base = blockIdx.x * kChunk + threadIdx.x * 16;
  bool dead[16];
  int cnt = 0;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    dead[i] = (base + i < P) && !live[base + i];
    cnt += dead[i];
  }
  int total;
  int rank = chunk_off[blockIdx.x] + block_exclusive_scan<256>(cnt, s_wave, total);
  const int n = *n_admitted;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    if (dead[i]) {
      if (rank < n) {
        const int q = unmatched[rank];
        slot_of_query[q] = base + i;
        pair_q[rank] = q;
        pair_slot[rank] = base + i;
        live[base + i] = 1;
      }
      ++rank;
    }
  }
}

struct CopyParams {
  const char *kq, *vq;
  char *kp, *vp;
  const float *q_ksq, *q_vsq;
  float *p_ksq, *p_vsq;
  const int *pair_q, *pair_slot;
  const int32_t* n_admitted;
  long long q_lstride_b, p_lstride_b;
  int Q, P, nh;
  int block_bytes;
};

// grid = (Q, L): workgroup (r, l) moves layer l of pair r; pairs past n_admitted do not exist.
__global__ __launch_bounds__(256) void admit_copy_kernel(const CopyParams p) {
  const int r = blockIdx.x;
  if (r >= *p.n_admitted) return;
  const long long l = blockIdx.y;
  const int q = p.pair_q[r], s = p.pair_slot[r];
  const long long so = l * p.q_lstride_b + (long long)q * p.block_bytes, dof = l * p.p_lstride_b + (long long)s * p.block_bytes;
  const u32x4* sk = reinterpret_cast<const u32x4*>(p.kq + so);
  const u32x4* sv = reinterpret_cast<const u32x4*>(p.vq + so);
  u32x4* dk = reinterpret_cast<u32x4*>(p.kp + dof);
  u32x4* dv = reinterpret_cast<u32x4*>(p.vp + dof);
  const int chunks = p.block_bytes / 16;
#pragma unroll 4
  for (int i = threadIdx.x; i < chunks; i += 256) {
    const u32x4 a = __builtin_nontemporal_load(sk + i), b = __builtin_nontemporal_load(sv + i);
    __builtin_nontemporal_store(a, dk + i);
    __builtin_nontemporal_store(b, dv + i);
  }
  if ((int)threadIdx.x < p.nh) {
    p.p_ksq[(l * p.P + s) * p.nh + threadIdx.x] = p.q_ksq[(l * p.Q + q) * p.nh + threadIdx.x];
    p.p_vsq[(l * p.P + s) * p.nh + threadIdx.x] = p.q_vsq[(l * p.Q + q) * p.nh + threadIdx.x];
  }
}

inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

struct AdmitLayout {
  size_t chunk_dead, chunk_off, unmatched, pair_q, pair_slot, total;
};
inline AdmitLayout admit_layout(int64_t Q, int64_t P) {
  const size_t nchunks = (size_t)((P + kChunk - 1) / kChunk);
  AdmitLayout a;
  size_t o = 0;
  a.chunk_dead = o; o += align256((nchunks + 1) * 4);
  a.chunk_off = o; o += align256((nchunks + 1) * 4);
  a.unmatched = o; o += align256((size_t)(Q + 1) * 4);
  a.pair_q = o; o += align256((size_t)(Q + 1) * 4);
  a.pair_slot = o; o += align256((size_t)(Q + 1) * 4);
  a.total = o;
  return a;
}

}  // namespace
}  // namespace rc

extern "C" size_t rc_pool_admit_workspace_size(int64_t Q, int64_t P) {
  if (Q < 0 || P < 0) return 0;
  return rc::admit_layout(Q, P).total;
}

extern "C" rc_status rc_pool_admit(const rc_kv_desc* qdesc, const rc_kv_desc* pdesc, int32_t mode, const void* kq,
                                   const void* vq, int64_t Q, const float* q_ksq, const float* q_vsq, void* kp, void* vp,
                                   int64_t P, float* p_ksq, float* p_vsq, uint8_t* pool_live, const int32_t* match_idx,
                                   int32_t* slot_of_query, int32_t* n_admitted, void* workspace, size_t workspace_bytes,
                                   void* hip_stream) {
  using namespace rc;
  clear_error();
  if (rc_status s = check_desc(qdesc, Q, "rc_pool_admit(query)")) return s;
  if (rc_status s = check_desc(pdesc, P, "rc_pool_admit(pool)")) return s;
  if (mode != RC_SCORE_BLOCK && mode != RC_SCORE_PER_HEAD_ALL) return fail(RC_ERR_UNSUPPORTED, "rc_pool_admit: mode %d", mode);
  if (qdesc->n_layers != pdesc->n_layers || qdesc->block_tokens != pdesc->block_tokens ||
      qdesc->n_kv_heads != pdesc->n_kv_heads || qdesc->head_dim != pdesc->head_dim || qdesc->dtype != pdesc->dtype)
    return fail(RC_ERR_INVALID_ARG, "rc_pool_admit: query and pool descriptors differ in more than layer_stride");
  if (!n_admitted) return fail(RC_ERR_INVALID_ARG, "rc_pool_admit: n_admitted is NULL");
  if (Q > 0 && (!match_idx || !slot_of_query)) return fail(RC_ERR_INVALID_ARG, "rc_pool_admit: NULL match_idx or slot_of_query");
  if (P > 0 && !pool_live) return fail(RC_ERR_INVALID_ARG, "rc_pool_admit: pool_live is NULL");
  const int L = qdesc->n_layers;
  if (L > 0 && Q > 0 && P > 0 && (!kq || !vq || !q_ksq || !q_vsq || !kp || !vp || !p_ksq || !p_vsq))
    return fail(RC_ERR_INVALID_ARG, "rc_pool_admit: NULL KV or norm pointer");
  if (!aligned16(kq) || !aligned16(vq) || !aligned16(kp) || !aligned16(vp))
    return fail(RC_ERR_INVALID_ARG, "rc_pool_admit: KV pointer not 16-byte aligned");
  if (Q > 0x7fffffffLL || P > 0x7fffffffLL - kChunk || L > 65535)
    return fail(RC_ERR_UNSUPPORTED, "rc_pool_admit: Q, P or L beyond the grid limits");
  const AdmitLayout lay = admit_layout(Q, P);
  if (!workspace || workspace_bytes < lay.total || !aligned16(workspace))
    return fail(RC_ERR_WORKSPACE, "rc_pool_admit: workspace of %zu bytes needed (16-byte aligned), got %zu", lay.total,
                workspace_bytes);
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  char* ws = static_cast<char*>(workspace);
  int* chunk_dead = reinterpret_cast<int*>(ws + lay.chunk_dead);
  int* chunk_off = reinterpret_cast<int*>(ws + lay.chunk_off);
  int* unmatched = reinterpret_cast<int*>(ws + lay.unmatched);
  int* pair_q = reinterpret_cast<int*>(ws + lay.pair_q);
  int* pair_slot = reinterpret_cast<int*>(ws + lay.pair_slot);
  const int nchunks = (int)((P + kChunk - 1) / kChunk);
  if (nchunks > 0) {
    admit_count_kernel<<<nchunks, 256, 0, st>>>(pool_live, (int)P, chunk_dead);
    if (rc_status s = check_launch("rc_pool_admit(count)")) return s;
  }
  admit_scan_kernel<<<1, 1024, 0, st>>>(chunk_dead, nchunks, chunk_off, match_idx, (int)Q, unmatched, slot_of_query,
                                        n_admitted);
  if (rc_status s = check_launch("rc_pool_admit(scan)")) return s;
  if (nchunks > 0 && Q > 0) {
    admit_assign_kernel<<<nchunks, 256, 0, st>>>(pool_live, (int)P, chunk_off, unmatched, n_admitted, slot_of_query,
                                                 pair_q, pair_slot);
    if (rc_status s = check_launch("rc_pool_admit(assign)")) return s;
    if (L > 0) {
      CopyParams cp;
      cp.kq = static_cast<const char*>(kq);
      cp.vq = static_cast<const char*>(vq);
      cp.kp = static_cast<char*>(kp);
      cp.vp = static_cast<char*>(vp);
      cp.q_ksq = q_ksq;
      cp.q_vsq = q_vsq;
      cp.p_ksq = p_ksq;
      cp.p_vsq = p_vsq;
      cp.pair_q = pair_q;
      cp.pair_slot = pair_slot;
      cp.n_admitted = n_admitted;
      cp.q_lstride_b = qdesc->layer_stride * 2;
      cp.p_lstride_b = pdesc->layer_stride * 2;
      cp.Q = (int)Q;
      cp.P = (int)P;
      cp.nh = (mode == RC_SCORE_BLOCK) ? 1 : qdesc->n_kv_heads;
      cp.block_bytes = qdesc->block_tokens * qdesc->n_kv_heads * qdesc->head_dim * 2;
      const long long qgrid = Q < 0x7fffffffLL ? Q : 0x7fffffffLL;
      admit_copy_kernel<<<dim3((unsigned)qgrid, (unsigned)L), 256, 0, st>>>(cp);
      if (rc_status s = check_launch("rc_pool_admit(copy)")) return s;
    }
  }
  return RC_OK;
}
