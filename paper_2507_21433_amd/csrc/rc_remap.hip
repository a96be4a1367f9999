// rc_remap_block_table: zero-copy sharing applied to the PagedAttention block tables
// (ReasonCache Sec. IV-B: the kept block's reference count goes up, the table entry is
// rewritten, nothing is copied; a block is freed only at reference count 0).
//
// One launch, or two; no atomics anywhere:
//   gather  : table_out[e] = target of table_in[e], 16-byte loads and stores when the layout allows,
//             the next batch of entries in flight while the current one is worked on.  A workgroup
//             first builds what it needs to decide an entry without touching global memory again:
//             a 16-bit table "block id - lo -> slot + 1 of the matched query block" over the id
//             range of the query blocks and the target of every matched slot, both in LDS (when the
//             ids span at most 32768 blocks and Q <= 4096).  Otherwise every entry follows the chain
//             entry -> slot_of -> query_ids -> match_idx -> pool_ids through global memory;
//             slot_of[query_ids[q]] = q is written by every workgroup for itself and never cleared:
//             an entry s read for block b counts only if s < Q and query_ids[s] == b.
//             References to matched query blocks are counted per workgroup in an LDS histogram: the
//             hits of a batch are compacted into a list (prefix sums), then every wave adds up the
//             keys of its own residue class (equal keys merged with ballots).  The same workgroups
//             copy their share of refcount_in to refcount_out.  With one workgroup per layer (small
//             tables, or many layers) the workgroup goes on to finalize its layer from its histogram.
//   finalize: per layer, cnt[q] = sum of the workgroups' histograms; the query block loses cnt
//             references, its target gains them.  Queries that share a target take turns through
//             a small claim table in LDS, one winner per slot and round.  A launch of its own only
//             when a layer was gathered by several workgroups.
#include <hip/hip_runtime.h>

#include <mutex>

#include "rc_common.hpp"

namespace rc {
namespace {

constexpr int kGatherThreads = 1024;
constexpr int kGatherPerThread = 16;                                  // entries a thread keeps in flight
constexpr int kGatherBatch = kGatherThreads * kGatherPerThread;       // entries per batch of a workgroup
constexpr int kMaxQ = 8192;                                           // LDS histogram bins
constexpr int kLdsIds = 32768;                                        // id range the 16-bit slot table covers
constexpr int kLdsTargets = 4096;                                     // most query slots with their target in LDS
constexpr int kFinalThreads = 1024;
constexpr int kFinalPerThread = kMaxQ / kFinalThreads;
constexpr int kClaimSlots = 4096;

// Workgroups per layer.  One (which then also finalizes its layer) when the layers alone fill the chip or the
// layer's table is small; otherwise as many as keep the launch at one workgroup per compute unit, of at least
// a quarter batch each: the second launch that adds their histograms costs less than what a single compute
// unit takes to stream a large layer (measured at 64 layers of 49 664 entries and 50 176 reference counts:
// 40 us with one workgroup per layer, 30 with 3, 26 with 4, 33 with 8).
inline int64_t chunks_per_layer(int64_t RE, int64_t L) {
  if (L >= 128) return 1;
  int64_t g = 256 / (L > 0 ? L : 1);
  const int64_t most = RE / (kGatherBatch / 4);
  if (g > most) g = most;
  if (g < 1) g = 1;
  if (g > 65535) g = 65535;
  return g;
}

typedef int i32x4 __attribute__((ext_vector_type(4)));

// Workgroup barrier that orders LDS traffic only: table loads and stores stay in flight across it
// (__syncthreads also waits for every outstanding global access of the wave, a memory round trip
// per batch in a kernel whose time at the benchmark's table shape is a chain of round trips).
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// Query slot of physical block t, or -1, through global memory.  slot_of may hold anything; a slot
// counts only if it points back at t.  A matched slot is then replaced by its target (out) and kept
// for counting.
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

// The reference counts of one layer move from the matched query blocks to their targets.
// cnt_of(q) = references to query slot q that the gather rewrote.  All kFinalThreads threads of the
// workgroup call this; `claim` is kClaimSlots ints of LDS, `wsum` kFinalThreads / 64 ints.
template <typename CountOf>
__device__ __forceinline__ void finalize_layer(CountOf cnt_of, const int32_t* __restrict__ query_ids,
                                               const int32_t* __restrict__ pool_ids, const int32_t* __restrict__ m, int Q,
                                               int P, long long NB, int32_t* rc_l, uint8_t* __restrict__ freed_l,
                                               int32_t* __restrict__ n_remapped_l, int* claim, int* wsum) {
  const int tid = threadIdx.x;
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
        const int c = cnt_of(q);
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
      freed_l[q] = fr;
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
    *n_remapped_l = s;
  }
}

struct GatherLds {
  unsigned short slot[kLdsIds];           // block id - lo -> slot + 1 of the matched query block with that id (0 = none)
  int target[kLdsTargets];                // target block of a matched slot
  int hist[kMaxQ];                        // references rewritten per slot
  unsigned short list[kGatherBatch];      // the hits of a batch, compacted; later the claim table of the finalize step
  int wsum[kGatherThreads / 64];
};
static_assert(sizeof(GatherLds) <= 160 * 1024, "fits the LDS of a compute unit");
static_assert(sizeof(unsigned short) * kGatherBatch >= sizeof(int) * kClaimSlots, "the claim table reuses the hit list");
static_assert(kGatherThreads == kFinalThreads, "the fused finalize step runs in the gather workgroup");

// grid = (G, L).  Workgroup g rewrites entries [g*chunk, min((g+1)*chunk, RE)) of layer l and copies
// refcounts [g*rc_chunk, ...) of the layer.  VEC: every layer starts 16-byte aligned and chunk % 4 == 0.
// FUSED (G == 1): the workgroup also moves the layer's reference counts.
template <bool VEC, bool FUSED>
__global__ __launch_bounds__(kGatherThreads) void remap_gather_kernel(
    const int32_t* tables_in, int32_t* tables_out, long long RE, long long chunk, int32_t* slot_of, const int32_t* __restrict__ query_ids, const int32_t* __restrict__ pool_ids,
    const int32_t* __restrict__ match_idx, int Q, int P, long long NB, int32_t* __restrict__ partial,
    const int32_t* refcount_in, int32_t* refcount_out, long long rc_chunk, int rc_vec, uint8_t* __restrict__ freed,
    int32_t* __restrict__ n_remapped) {
  __shared__ GatherLds s;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const long long l = blockIdx.y, g = blockIdx.x, G = gridDim.x;
  const int32_t* tin = tables_in + l * RE;
  int32_t* tout = tables_out + l * RE;
  const int32_t* m = match_idx + l * Q;
  const long long lo_e = g * chunk, hi_e = (lo_e + chunk < RE) ? lo_e + chunk : RE;

  // ---- what decides an entry.  Every workgroup finds the range [id_lo, id_hi] of the query block ids itself.
  int id_lo = 0x7fffffff, id_hi = -1;
  for (int q = tid; q < Q; q += kGatherThreads) {
    const int b = query_ids[q];
    if (b >= 0 && b < NB) {
      id_lo = min(id_lo, b);
      id_hi = max(id_hi, b);
    }
    s.hist[q] = 0;
  }
  for (int off = 32; off > 0; off >>= 1) {
    id_lo = min(id_lo, __shfl_xor(id_lo, off));
    id_hi = max(id_hi, __shfl_xor(id_hi, off));
  }
  if (lane == 0) {
    s.wsum[wave] = id_lo;
    s.list[wave] = 0;  // (keeps the two arrays apart for the reader below)
    reinterpret_cast<int*>(s.list)[64 + wave] = id_hi;
  }
  lds_barrier();
#pragma unroll
  for (int w = 0; w < kGatherThreads / 64; ++w) {
    id_lo = min(id_lo, s.wsum[w]);
    id_hi = max(id_hi, reinterpret_cast<int*>(s.list)[64 + w]);
  }
  lds_barrier();
  const long long span = (long long)id_hi - id_lo + 1;  // <= 0: no query block with a valid id
  const bool in_lds = span <= kLdsIds && Q <= kLdsTargets;
  if (in_lds) {
    // a 16-bit table over the id range and the targets of the matched slots, in LDS
    if (span > 0) {
      unsigned int* z = reinterpret_cast<unsigned int*>(s.slot);
      for (int i = tid; i < (int)((span + 1) / 2); i += kGatherThreads) z[i] = 0u;
      lds_barrier();
      for (int q = tid; q < Q; q += kGatherThreads) {
        const int b = query_ids[q];
        const int mi = m[q];
        if (b >= 0 && b < NB && mi >= 0 && mi < P) {      // a matched query block
          s.slot[b - id_lo] = (unsigned short)(q + 1);    // query ids are distinct: one writer per entry
          s.target[q] = pool_ids ? pool_ids[mi] : mi;
        }
      }
    }
  } else {
    // the reverse index in global memory.  Every workgroup writes all of it (the same values), so each reads
    // what it wrote itself; words that no query block owns are stale or uninitialised and fail the check
    // query_ids[slot_of[t]] == t of the reader.
    for (int q = tid; q < Q; q += kGatherThreads) {
      const int b = query_ids[q];
      if (b >= 0 && b < NB) slot_of[b] = q;
    }
    __threadfence_block();
  }
  __syncthreads();

  // thread -> 4 consecutive entries per load (VEC) or entries strided by the workgroup size
  auto index_of = [&](long long base, int k) {
    return VEC ? base + ((k >> 2) * kGatherThreads + tid) * 4 + (k & 3) : base + (long long)k * kGatherThreads + tid;
  };
  auto load_batch = [&](long long base, int (&entry)[kGatherPerThread]) {
    if (VEC) {
#pragma unroll
      for (int k = 0; k < kGatherPerThread; k += 4) {
        const long long e = index_of(base, k);
        i32x4 v = {-1, -1, -1, -1};
        if (e + 3 < hi_e) {
          v = __builtin_nontemporal_load(reinterpret_cast<const i32x4*>(tin + e));
        } else {
#pragma unroll
          for (int c = 0; c < 4; ++c)
            if (e + c < hi_e) v[c] = tin[e + c];
        }
#pragma unroll
        for (int c = 0; c < 4; ++c) entry[k + c] = v[c];
      }
    } else {
#pragma unroll
      for (int k = 0; k < kGatherPerThread; ++k) {
        const long long e = index_of(base, k);
        entry[k] = (e < hi_e) ? tin[e] : -1;
      }
    }
  };
  // the entries of the next batch are asked for before the current batch is worked on
  int ahead[kGatherPerThread];
  if (lo_e < hi_e) load_batch(lo_e, ahead);
  for (long long base = lo_e; base < hi_e; base += kGatherBatch) {
    int entry[kGatherPerThread], slot[kGatherPerThread];
#pragma unroll
    for (int k = 0; k < kGatherPerThread; ++k) entry[k] = ahead[k];
    if (base + kGatherBatch < hi_e) load_batch(base + kGatherBatch, ahead);
    int outv[kGatherPerThread];
    int hits = 0;
    if (in_lds) {
#pragma unroll
      for (int k = 0; k < kGatherPerThread; ++k) {
        const int t = entry[k];
        const long long d = (long long)t - id_lo;
        int o = t, sl = -1;
        if (span > 0 && t >= 0 && t < NB && d >= 0 && d < span) {
          const int s1 = s.slot[d];
          if (s1) {
            sl = s1 - 1;
            o = s.target[sl];
          }
        }
        outv[k] = o;
        slot[k] = sl;
        hits += sl >= 0;
      }
    } else {
#pragma unroll
      for (int k = 0; k < kGatherPerThread; ++k) {
        outv[k] = remap_entry(entry[k], slot_of, query_ids, pool_ids, m, Q, P, NB, slot[k]);
        hits += slot[k] >= 0;
      }
    }
    if (VEC) {
#pragma unroll
      for (int k = 0; k < kGatherPerThread; k += 4) {
        const long long e = index_of(base, k);
        if (e + 3 < hi_e) {
          i32x4 v = {outv[k], outv[k + 1], outv[k + 2], outv[k + 3]};
          __builtin_nontemporal_store(v, reinterpret_cast<i32x4*>(tout + e));
        } else {
#pragma unroll
          for (int c = 0; c < 4; ++c)
            if (e + c < hi_e) tout[e + c] = outv[k + c];
        }
      }
    } else {
#pragma unroll
      for (int k = 0; k < kGatherPerThread; ++k) {
        const long long e = index_of(base, k);
        if (e < hi_e) tout[e] = outv[k];
      }
    }
    // ---- count the rewritten references of this batch
    // position of this thread's hits in the list: prefix sum over the workgroup
    int incl = hits;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const int n = __shfl_up(incl, off);
      if (lane >= off) incl += n;
    }
    if (lane == 63) s.wsum[wave] = incl;
    lds_barrier();
    int before = 0, total = 0;
#pragma unroll
    for (int w = 0; w < kGatherThreads / 64; ++w) {
      const int c = s.wsum[w];
      before += (w < wave) ? c : 0;
      total += c;
    }
    if (total != 0) {   // the same for every thread
      int pos = before + incl - hits;
#pragma unroll
      for (int k = 0; k < kGatherPerThread; ++k)
        if (slot[k] >= 0) s.list[pos++] = (unsigned short)slot[k];
      lds_barrier();
      // wave w adds up the keys congruent to w: no two waves touch the same bin
      for (int i0 = 0; i0 < total; i0 += 64) {
        const int i = i0 + lane;
        const int key = (i < total) ? (int)s.list[i] : -1;
        const bool mine = key >= 0 && (key & (kGatherThreads / 64 - 1)) == wave;
        unsigned long long active = __ballot(mine);
        while (active) {
          const int leader = __ffsll((long long)active) - 1;
          const int lkey = __shfl(key, leader);
          const unsigned long long same = __ballot(mine && key == lkey);
          if (lane == leader) s.hist[lkey] += __popcll(same);
          active &= ~same;
        }
      }
    }
    lds_barrier();  // the list and the wave sums are free again
  }
  // this workgroup's share of the refcount copy (the finalize step then edits refcount_out)
  if (refcount_in != refcount_out) {
    const long long rlo = g * rc_chunk, rhi = (rlo + rc_chunk < NB) ? rlo + rc_chunk : NB;
    const int32_t* src = refcount_in + l * NB;
    int32_t* dst = refcount_out + l * NB;
    if (rc_vec) {
      constexpr long long kStride = kGatherThreads * 4LL;
      long long i = rlo + tid * 4LL;
      for (; i + 3 * kStride + 3 < rhi; i += 4 * kStride) {  // four loads in flight
        i32x4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = __builtin_nontemporal_load(reinterpret_cast<const i32x4*>(src + i + u * kStride));
#pragma unroll
        for (int u = 0; u < 4; ++u) __builtin_nontemporal_store(v[u], reinterpret_cast<i32x4*>(dst + i + u * kStride));
      }
      for (; i < rhi; i += kStride) {
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
  if (FUSED) {
    // the copy of this layer's reference counts is this workgroup's own (same compute unit, same L1): a fence
    // at workgroup scope orders it before the edits.  (A device-scope fence writes the L2 back: tens of microseconds.)
    __threadfence_block();
    __syncthreads();
    finalize_layer([&](int q) { return s.hist[q]; }, query_ids, pool_ids, m, Q, P, NB, refcount_out + l * NB,
                   freed + l * Q, n_remapped + l, reinterpret_cast<int*>(s.list), s.wsum);
  } else {
    __syncthreads();
    int32_t* out = partial + (l * G + g) * Q;
    for (int q = tid; q < Q; q += kGatherThreads) out[q] = s.hist[q];
  }
}

// grid = L, one workgroup per layer (only when a layer was gathered by several workgroups).
__global__ __launch_bounds__(kFinalThreads) void remap_finalize_kernel(
    const int32_t* __restrict__ partial, int G, const int32_t* __restrict__ query_ids,
    const int32_t* __restrict__ pool_ids, const int32_t* __restrict__ match_idx, int Q, int P, long long NB,
    int32_t* refcount_out, uint8_t* __restrict__ freed, int32_t* __restrict__ n_remapped) {
  __shared__ int claim[kClaimSlots];
  __shared__ int wsum[kFinalThreads / 64];
  const long long l = blockIdx.x;
  finalize_layer(
      [&](int q) {
        int c = 0;
        for (int g = 0; g < G; ++g) c += partial[(l * G + g) * Q + q];
        return c;
      },
      query_ids, pool_ids, match_idx + l * Q, Q, P, NB, refcount_out + l * NB, freed + l * Q, n_remapped + l, claim, wsum);
}

}  // namespace
}  // namespace rc

extern "C" size_t rc_remap_workspace_size(int32_t n_layers, int64_t R, int64_t E, int64_t Q, int64_t NB) {
  using namespace rc;
  if (n_layers < 0 || R < 0 || E < 0 || Q < 0 || NB < 0) return 0;
  const int64_t G = chunks_per_layer(R * E, n_layers);
  const int64_t ints = ((NB + 3) / 4) * 4 + (G > 1 ? (int64_t)n_layers * G * Q : 0);
  return (size_t)(ints > 0 ? ints : 4) * sizeof(int32_t);
}

// Scratch of rc_remap_block_table_static: one array per GPU, part of the loaded code object, so it
// exists from the moment the library is loaded on a device until the process ends.  In host code
// the name is only a handle for hipGetSymbolAddress; kernels get the address it returns.
static __device__ __align__(256) unsigned char scratch[RC_REMAP_STATIC_SCRATCH_BYTES];

namespace rc {
namespace {

// Validation and the launches, shared by the two entry points; `who` names the caller in
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

  const dim3 grid((unsigned)G, (unsigned)n_layers);
#define RC_GATHER(V, F)                                                                                                    \
  remap_gather_kernel<V, F><<<grid, kGatherThreads, 0, st>>>(tables_in, tables_out, RE, chunk, slot_of, query_ids,         \
                                                             pool_ids, match_idx, (int)Q, (int)P, NB, partial,             \
                                                             refcount_in, refcount_out, rc_chunk, rc_vec, freed, n_remapped)
  if (G == 1) {
    if (vec)
      RC_GATHER(true, true);
    else
      RC_GATHER(false, true);
    return check_launch("rc_remap_block_table(gather + finalize)");
  }
  if (vec)
    RC_GATHER(true, false);
  else
    RC_GATHER(false, false);
#undef RC_GATHER
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
