// rc_remap_block_table: zero-copy sharing applied to the PagedAttention block tables
// (ReasonCache Sec. IV-B: the kept block's reference count goes up, the table entry is
// rewritten, nothing is copied; a block is freed only at reference count 0).
//
// Three stream-ordered launches, no atomics anywhere:
//   1. scatter : slot_of[query_ids[q]] = q.  slot_of is never cleared: an entry s read for block b
//                counts only if s < Q and query_ids[s] == b, so stale or uninitialised words are harmless
//   2. gather  : table_out[e] = target of table_in[e] (16-byte loads and stores when the layout
//                allows); references to matched query blocks are counted per workgroup in an LDS
//                histogram that one wave at a time updates (equal keys inside a wave are merged
//                with ballots), then stored as partials; the same workgroups copy their share of
//                refcount_in to refcount_out
//   3. finalize: per layer, cnt[q] = sum of partials; the query block loses cnt references,
//                its target gains them.  Queries that share a target take turns through a
//                small claim table in LDS, one winner per slot and round.
#include <hip/hip_runtime.h>

#include <mutex>

#include "rc_common.hpp"

namespace rc {
namespace {

constexpr int kGatherThreads = 256;
constexpr int kGatherPerThread = 16;                                  // entries a thread keeps in flight
constexpr int kGatherBatch = kGatherThreads * kGatherPerThread;       // entries per batch of a workgroup
constexpr int kMaxQ = 8192;                                           // LDS histogram bins
constexpr int kFinalThreads = 1024;
constexpr int kFinalPerThread = kMaxQ / kFinalThreads;
constexpr int kClaimSlots = 4096;

// How the R*E entries of a layer are cut into workgroups: about 1024 workgroups over all layers
// when the tables are small (to fill 256 compute units), one per layer when there are many layers
// (so the per-workgroup partial histogram of Q ints stays a small fraction of the table traffic).
inline int64_t chunks_per_layer(int64_t RE, int64_t L) {
  int64_t g = (1024 + L - 1) / (L > 0 ? L : 1);
  const int64_t most = RE / kGatherBatch;
  if (g > most) g = most;
  if (g < 1) g = 1;
  if (g > 65535) g = 65535;
  return g;
}

__global__ __launch_bounds__(256) void remap_scatter_kernel(int32_t* __restrict__ slot_of,
                                                            const int32_t* __restrict__ query_ids, int Q, long long NB) {
  const int q = blockIdx.x * blockDim.x + threadIdx.x;
  if (q < Q) {
    const int b = query_ids[q];
    if (b >= 0 && b < NB) slot_of[b] = q;
  }
}

typedef int i32x4 __attribute__((ext_vector_type(4)));

// Query slot of physical block t, or -1.  slot_of may hold anything; a slot counts only if it
// points back at t.  A matched slot is then replaced by its target (out) and kept for counting.
__device__ __forceinline__ int remap_entry(int t, const int32_t* __restrict__ slot_of,
                                           const int32_t* __restrict__ query_ids, const int32_t* __restrict__ pool_ids,
                                           const int32_t* __restrict__ m, int Q, int P, long long NB, int& slot) {
  slot = -1;
  if (t < 0 || t >= NB) return t;
  const int s = slot_of[t];
  if ((unsigned)s >= (unsigned)Q || query_ids[s] != t) return t;
  const int mi = m[s];
  if (mi < 0 || mi >= P) return t;  // unmatched query block: entry stays, nothing to count
  slot = s;
  return pool_ids ? pool_ids[mi] : mi;
}

// grid = (G, L).  Workgroup g rewrites entries [g*chunk, min((g+1)*chunk, RE)) of layer l and copies
// refcounts [g*rc_chunk, ...) of the layer.  VEC: every layer starts 16-byte aligned and chunk % 4 == 0.
template <bool VEC>
__global__ __launch_bounds__(kGatherThreads) void remap_gather_kernel(
    const int32_t* tables_in, int32_t* tables_out, long long RE, long long chunk,
    const int32_t* __restrict__ slot_of, const int32_t* __restrict__ query_ids,
    const int32_t* __restrict__ pool_ids, const int32_t* __restrict__ match_idx, int Q, int P, long long NB,
    int32_t* __restrict__ partial, const int32_t* refcount_in, int32_t* refcount_out, long long rc_chunk,
    int rc_vec) {
  extern __shared__ int hist[];  // Q bins
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const long long l = blockIdx.y, g = blockIdx.x, G = gridDim.x;
  for (int q = tid; q < Q; q += kGatherThreads) hist[q] = 0;
  __syncthreads();
  const int32_t* tin = tables_in + l * RE;
  int32_t* tout = tables_out + l * RE;
  const int32_t* m = match_idx + l * Q;
  const long long lo = g * chunk, hi = (lo + chunk < RE) ? lo + chunk : RE;

  for (long long base = lo; base < hi; base += kGatherBatch) {
    int entry[kGatherPerThread], slot[kGatherPerThread];
    // thread -> 4 consecutive entries per load (VEC) or entries strided by the workgroup size
    auto index_of = [&](int k) {
      return VEC ? base + ((k >> 2) * kGatherThreads + tid) * 4 + (k & 3) : base + (long long)k * kGatherThreads + tid;
    };
    if (VEC) {
#pragma unroll
      for (int k = 0; k < kGatherPerThread; k += 4) {
        const long long e = index_of(k);
        i32x4 v = {-1, -1, -1, -1};
        if (e + 3 < hi) {
          v = __builtin_nontemporal_load(reinterpret_cast<const i32x4*>(tin + e));
        } else {
#pragma unroll
          for (int c = 0; c < 4; ++c)
            if (e + c < hi) v[c] = tin[e + c];
        }
#pragma unroll
        for (int c = 0; c < 4; ++c) entry[k + c] = v[c];
      }
    } else {
#pragma unroll
      for (int k = 0; k < kGatherPerThread; ++k) {
        const long long e = index_of(k);
        entry[k] = (e < hi) ? tin[e] : -1;
      }
    }
    int outv[kGatherPerThread];
#pragma unroll
    for (int k = 0; k < kGatherPerThread; ++k)
      outv[k] = remap_entry(entry[k], slot_of, query_ids, pool_ids, m, Q, P, NB, slot[k]);
    if (VEC) {
#pragma unroll
      for (int k = 0; k < kGatherPerThread; k += 4) {
        const long long e = index_of(k);
        if (e + 3 < hi) {
          i32x4 v = {outv[k], outv[k + 1], outv[k + 2], outv[k + 3]};
          __builtin_nontemporal_store(v, reinterpret_cast<i32x4*>(tout + e));
        } else {
#pragma unroll
          for (int c = 0; c < 4; ++c)
            if (e + c < hi) tout[e + c] = outv[k + c];
        }
      }
    } else {
#pragma unroll
      for (int k = 0; k < kGatherPerThread; ++k) {
        const long long e = index_of(k);
        if (e < hi) tout[e] = outv[k];
      }
    }
    // count the rewritten references, one wave at a time
    bool any = false;
#pragma unroll
    for (int k = 0; k < kGatherPerThread; ++k) any |= slot[k] >= 0;
    if (__syncthreads_or(any)) {
      for (int w = 0; w < kGatherThreads / 64; ++w) {
        if (wave == w) {
#pragma unroll
          for (int k = 0; k < kGatherPerThread; ++k) {
            const int s = slot[k];
            unsigned long long active = __ballot(s >= 0);
            while (active) {
              const int leader = __ffsll((long long)active) - 1;
              const int key = __shfl(s, leader);
              const unsigned long long same = __ballot(s == key);
              if (lane == leader) hist[key] += __popcll(same);
              active &= ~same;
            }
          }
        }
        __syncthreads();
      }
    }
  }
  // this workgroup's share of the refcount copy (the finalize kernel then edits refcount_out)
  if (refcount_in != refcount_out) {
    const long long rlo = g * rc_chunk, rhi = (rlo + rc_chunk < NB) ? rlo + rc_chunk : NB;
    const int32_t* src = refcount_in + l * NB;
    int32_t* dst = refcount_out + l * NB;
    if (rc_vec) {
      for (long long i = rlo + tid * 4LL; i < rhi; i += kGatherThreads * 4LL) {
        if (i + 3 < rhi) {
          __builtin_nontemporal_store(__builtin_nontemporal_load(reinterpret_cast<const i32x4*>(src + i)),
                                      reinterpret_cast<i32x4*>(dst + i));
        } else {
          for (long long c = i; c < rhi; ++c) dst[c] = src[c];
        }
      }
    } else {
      for (long long i = rlo + tid; i < rhi; i += kGatherThreads) dst[i] = src[i];
    }
  }
  __syncthreads();
  int32_t* out = partial + (l * G + g) * Q;
  for (int q = tid; q < Q; q += kGatherThreads) out[q] = hist[q];
}

// grid = L, one workgroup per layer.
__global__ __launch_bounds__(kFinalThreads) void remap_finalize_kernel(
    const int32_t* __restrict__ partial, int G, const int32_t* __restrict__ query_ids,
    const int32_t* __restrict__ pool_ids, const int32_t* __restrict__ match_idx, int Q, int P, long long NB,
    int32_t* refcount_out, uint8_t* __restrict__ freed, int32_t* __restrict__ n_remapped) {
  __shared__ int claim[kClaimSlots];
  __shared__ int wsum[kFinalThreads / 64];
  const int tid = threadIdx.x;
  const long long l = blockIdx.x;
  const int32_t* m = match_idx + l * Q;
  int32_t* rc_l = refcount_out + l * NB;

  int cnt[kFinalPerThread], tgt[kFinalPerThread];
  int moved = 0;
#pragma unroll
  for (int k = 0; k < kFinalPerThread; ++k) {
    const int q = k * kFinalThreads + tid;
    cnt[k] = 0;
    tgt[k] = -1;
    if (q < Q) {
      const int mi = m[q];
      const int b = query_ids[q];
      unsigned char fr = 0;
      if (mi >= 0 && mi < P && b >= 0 && b < NB) {
        int c = 0;
        for (int g = 0; g < G; ++g) c += partial[(l * G + g) * Q + q];
        const int t = pool_ids ? pool_ids[mi] : mi;
        const int left = rc_l[b] - c;
        rc_l[b] = left;  // query ids are distinct: no other thread touches this entry
        fr = (left == 0);
        moved += c;
        if (c > 0 && t >= 0 && t < NB) {
          cnt[k] = c;
          tgt[k] = t;
        }
      }
      freed[l * Q + q] = fr;
    }
  }
  // queries that share a target add their references in turns
  bool pending = false;
#pragma unroll
  for (int k = 0; k < kFinalPerThread; ++k) pending |= tgt[k] >= 0;
  while (__syncthreads_or(pending)) {
#pragma unroll
    for (int k = 0; k < kFinalPerThread; ++k)
      if (tgt[k] >= 0) claim[tgt[k] & (kClaimSlots - 1)] = k * kFinalThreads + tid;
    __syncthreads();
    pending = false;
#pragma unroll
    for (int k = 0; k < kFinalPerThread; ++k)
      if (tgt[k] >= 0) {
        if (claim[tgt[k] & (kClaimSlots - 1)] == k * kFinalThreads + tid) {
          rc_l[tgt[k]] += cnt[k];
          tgt[k] = -1;
        } else {
          pending = true;
        }
      }
    __threadfence_block();
  }
  // n_remapped = total references moved in this layer
  for (int off = 32; off > 0; off >>= 1) moved += __shfl_xor(moved, off);
  if ((tid & 63) == 0) wsum[tid >> 6] = moved;
  __syncthreads();
  if (tid == 0) {
    int s = 0;
    for (int w = 0; w < kFinalThreads / 64; ++w) s += wsum[w];
    n_remapped[l] = s;
  }
}

}  // namespace
}  // namespace rc

extern "C" size_t rc_remap_workspace_size(int32_t n_layers, int64_t R, int64_t E, int64_t Q, int64_t NB) {
  using namespace rc;
  if (n_layers < 0 || R < 0 || E < 0 || Q < 0 || NB < 0) return 0;
  const int64_t G = chunks_per_layer(R * E, n_layers);
  const int64_t ints = ((NB + 3) / 4) * 4 + (int64_t)n_layers * G * Q;
  return (size_t)(ints > 0 ? ints : 4) * sizeof(int32_t);
}

// Scratch of rc_remap_block_table_static: one array per GPU, part of the loaded code object, so it
// exists from the moment the library is loaded on a device until the process ends.  In host code
// the name is only a handle for hipGetSymbolAddress; kernels get the address it returns.
static __device__ __align__(256) unsigned char scratch[RC_REMAP_STATIC_SCRATCH_BYTES];

namespace rc {
namespace {

// Validation and the three launches, shared by the two entry points; `who` names the caller in
// error texts.  Nothing is allocated here.
rc_status remap_run(const char* who, int32_t n_layers, const int32_t* tables_in, int32_t* tables_out, int64_t R,
                    int64_t E, const int32_t* query_ids, const int32_t* pool_ids, const int32_t* match_idx, int64_t Q,
                    int64_t P, int64_t NB, const int32_t* refcount_in, int32_t* refcount_out, uint8_t* freed,
                    int32_t* n_remapped, void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (n_layers < 0 || R < 0 || E < 0 || Q < 0 || P < 0 || NB < 0)
    return fail(RC_ERR_INVALID_ARG, "%s: negative size", who);
  if (Q > kMaxQ) return fail(RC_ERR_UNSUPPORTED, "%s: Q %lld above %d", who, (long long)Q, kMaxQ);
  if (!pool_ids && P > NB) return fail(RC_ERR_INVALID_ARG, "%s: identity pool ids need P <= NB", who);
  if (n_layers == 0) return RC_OK;
  const int64_t RE = R * E;
  if (n_layers > 65535 || NB > 0x7fffffffLL || P > 0x7fffffffLL || RE > (1LL << 40))
    return fail(RC_ERR_UNSUPPORTED, "%s: problem beyond the grid limits", who);
  if (!n_remapped || (RE > 0 && (!tables_in || !tables_out)) || (NB > 0 && (!refcount_in || !refcount_out)) ||
      (Q > 0 && (!query_ids || !match_idx || !freed)))
    return fail(RC_ERR_INVALID_ARG, "%s: NULL pointer", who);
  const size_t need = rc_remap_workspace_size(n_layers, R, E, Q, NB);
  if (!workspace || workspace_bytes < need || !aligned16(workspace))
    return fail(RC_ERR_WORKSPACE, "%s: workspace of %zu bytes needed (16-byte aligned), got %zu", who,
                need, workspace_bytes);
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  int32_t* slot_of = static_cast<int32_t*>(workspace);
  int32_t* partial = slot_of + ((NB + 3) / 4) * 4;
  const int64_t G = chunks_per_layer(RE, n_layers);
  int64_t chunk = (RE + G - 1) / G;
  chunk = (chunk + 3) / 4 * 4;
  int64_t rc_chunk = (NB + G - 1) / G;
  rc_chunk = (rc_chunk + 3) / 4 * 4;
  const bool vec = RE % 4 == 0 && aligned16(tables_in) && aligned16(tables_out);
  const int rc_vec = NB % 4 == 0 && aligned16(refcount_in) && aligned16(refcount_out);

  if (Q > 0 && NB > 0) {
    remap_scatter_kernel<<<(unsigned)((Q + 255) / 256), 256, 0, st>>>(slot_of, query_ids, (int)Q, NB);
    if (rc_status s = check_launch("rc_remap_block_table(scatter)")) return s;
  }
  const dim3 grid((unsigned)G, (unsigned)n_layers);
  const size_t hist_bytes = (size_t)(Q > 0 ? Q : 1) * sizeof(int);
  if (vec)
    remap_gather_kernel<true><<<grid, kGatherThreads, hist_bytes, st>>>(tables_in, tables_out, RE, chunk, slot_of, query_ids,
                                                               pool_ids, match_idx, (int)Q, (int)P, NB, partial,
                                                               refcount_in, refcount_out, rc_chunk, rc_vec);
  else
    remap_gather_kernel<false><<<grid, kGatherThreads, hist_bytes, st>>>(tables_in, tables_out, RE, chunk, slot_of, query_ids,
                                                                pool_ids, match_idx, (int)Q, (int)P, NB, partial,
                                                                refcount_in, refcount_out, rc_chunk, rc_vec);
  if (rc_status s = check_launch("rc_remap_block_table(gather)")) return s;
  remap_finalize_kernel<<<(unsigned)n_layers, kFinalThreads, 0, st>>>(partial, (int)G, query_ids, pool_ids, match_idx,
                                                                      (int)Q, (int)P, NB, refcount_out, freed,
                                                                      n_remapped);
  return check_launch("rc_remap_block_table(finalize)");
}

constexpr size_t kStaticScratchBytes = RC_REMAP_STATIC_SCRATCH_BYTES;

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices];  // device address of `scratch` on each device, nullptr = not asked yet

// Address of the current device's copy of `scratch` (looked up once per device).
rc_status static_scratch(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail(RC_ERR_DEVICE, "rc_remap_block_table_static: hipGetDevice: %s", hipGetErrorString(e));
  if (dev < 0 || dev >= kMaxDevices)
    return fail(RC_ERR_UNSUPPORTED, "rc_remap_block_table_static: device %d beyond the %d devices kept track of", dev,
                kMaxDevices);
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !ptr)
      return fail(RC_ERR_DEVICE, "rc_remap_block_table_static: hipGetSymbolAddress: %s", hipGetErrorString(e));
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return RC_OK;
}

}  // namespace
}  // namespace rc

extern "C" rc_status rc_remap_block_table(int32_t n_layers, const int32_t* tables_in, int32_t* tables_out, int64_t R,
                                          int64_t E, const int32_t* query_ids, const int32_t* pool_ids,
                                          const int32_t* match_idx, int64_t Q, int64_t P, int64_t NB,
                                          const int32_t* refcount_in, int32_t* refcount_out, uint8_t* freed,
                                          int32_t* n_remapped, void* workspace, size_t workspace_bytes,
                                          void* hip_stream) {
  rc::clear_error();
  return rc::remap_run("rc_remap_block_table", n_layers, tables_in, tables_out, R, E, query_ids, pool_ids, match_idx, Q, P,
                       NB, refcount_in, refcount_out, freed, n_remapped, workspace, workspace_bytes, hip_stream);
}

extern "C" size_t rc_remap_static_scratch_size(void) { return rc::kStaticScratchBytes; }

extern "C" rc_status rc_remap_block_table_static(int32_t n_layers, const int32_t* tables_in, int32_t* tables_out,
                                                 int64_t R, int64_t E, const int32_t* query_ids,
                                                 const int32_t* pool_ids, const int32_t* match_idx, int64_t Q,
                                                 int64_t P, int64_t NB, const int32_t* refcount_in,
                                                 int32_t* refcount_out, uint8_t* freed, int32_t* n_remapped,
                                                 void* hip_stream) {
  using namespace rc;
  clear_error();
  if (n_layers < 0 || R < 0 || E < 0 || Q < 0 || P < 0 || NB < 0)
    return fail(RC_ERR_INVALID_ARG, "rc_remap_block_table_static: negative size");
  const size_t need = rc_remap_workspace_size(n_layers, R, E, Q, NB);
  if (need > kStaticScratchBytes)
    return fail(RC_ERR_WORKSPACE,
                "rc_remap_block_table_static: this problem needs %zu bytes of scratch, the built-in buffer has %zu; "
                "use rc_remap_block_table with a workspace of the caller's",
                need, kStaticScratchBytes);
  if (n_layers == 0) return RC_OK;
  void* ptr = nullptr;
  if (rc_status s = static_scratch(&ptr)) return s;
  return remap_run("rc_remap_block_table_static", n_layers, tables_in, tables_out, R, E, query_ids, pool_ids, match_idx, Q,
                   P, NB, refcount_in, refcount_out, freed, n_remapped, ptr, kStaticScratchBytes, hip_stream);
}
