// rc_pool_touch, rc_refcount_release, rc_pool_evict: the block metadata of the streaming pool and
// the step that makes room for a step's admissions (ReasonCache Sec. IV-B: the evictor returns a
// block to the free pool only when its reference count has dropped to 0; Sec. IV-A: per-block
// metadata is kept in LRU order).
//
// rc_pool_evict is one workgroup that walks the per-slot metadata (9 bytes per slot; 0.4 MB for
// the 49 152 slots of the largest benchmark pool) a handful of times: counts, a radix select of
// the need-th smallest last-use stamp among the unreferenced live slots (four passes of 8 bits
// over order-preserving keys), then one pass in slot order that lets every candidate below that
// stamp go and, of those at it, the lowest-numbered ones.  Integer counts only (LDS and global
// integer atomics add up the same whatever the order): the same slots on every run.
#include <hip/hip_runtime.h>

#include "rc_common.hpp"

namespace rc {
namespace {

constexpr int kEvictThreads = 1024;

__global__ __launch_bounds__(256) void touch_kernel(const int32_t* __restrict__ slots, long long n, int32_t value,
                                                    int32_t* __restrict__ array, long long P) {
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const int s = slots[i];
  if (s >= 0 && s < P) array[s] = value;  // a slot listed twice gets the same value twice
}

__global__ __launch_bounds__(256) void release_kernel(const int32_t* __restrict__ ids, long long n,
                                                      int32_t* __restrict__ refcount, long long NB) {
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const int b = ids[i];
  if (b >= 0 && b < NB) atomicSub(&refcount[b], 1);  // an id listed k times loses k references
}

// Sum of one value per thread over the workgroup, to every thread.  s_w: kEvictThreads / 64 words.
__device__ __forceinline__ long long block_sum(long long v, long long* s_w) {
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
  __syncthreads();  // s_w may still be read from the previous call
  if ((threadIdx.x & 63) == 0) s_w[threadIdx.x >> 6] = v;
  __syncthreads();
  long long t = 0;
#pragma unroll
  for (int w = 0; w < kEvictThreads / 64; ++w) t += s_w[w];
  return t;
}

__device__ __forceinline__ unsigned int stamp_key(int32_t s) { return (unsigned int)s ^ 0x80000000u; }  // order-preserving

__global__ __launch_bounds__(kEvictThreads) void evict_kernel(long long P, uint8_t* __restrict__ live,
                                                              const int32_t* __restrict__ refcount,
                                                              const int32_t* __restrict__ last_used,
                                                              const int32_t* __restrict__ match_idx, long long Q,
                                                              long long extra_wanted, int32_t* __restrict__ n_free,
                                                              int32_t* __restrict__ n_evicted) {
  __shared__ long long s_w[kEvictThreads / 64];
  __shared__ unsigned int s_hist[256];
  __shared__ int s_scan[kEvictThreads / 64];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  auto candidate = [&](long long p) { return live[p] && (!refcount || refcount[p] == 0); };

  long long unmatched = 0, dead = 0, cands = 0;
  for (long long q = tid; q < Q; q += kEvictThreads) unmatched += match_idx[q] < 0;
  for (long long p = tid; p < P; p += kEvictThreads) {
    dead += !live[p];
    cands += candidate(p);
  }
  const long long wanted = block_sum(unmatched, s_w) + extra_wanted;
  const long long free0 = block_sum(dead, s_w);
  const long long ncand = block_sum(cands, s_w);
  long long need = wanted - free0;
  if (need > ncand) need = ncand;
  if (need <= 0) {
    if (tid == 0) {
      *n_free = (int32_t)free0;
      *n_evicted = 0;
    }
    return;
  }
  // ---- the need-th smallest stamp among the candidates (ties counted): radix select, 8 bits per pass
  unsigned int prefix = 0;
  long long k = need;  // rank still looked for inside the current prefix
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = 24 - 8 * pass;
    const unsigned int mask = pass == 0 ? 0u : 0xffffffffu << (32 - 8 * pass);
    if (tid < 256) s_hist[tid] = 0u;
    __syncthreads();
    for (long long p = tid; p < P; p += kEvictThreads)
      if (candidate(p)) {
        const unsigned int key = stamp_key(last_used[p]);
        if ((key & mask) == prefix) atomicAdd(&s_hist[(key >> shift) & 255u], 1u);
      }
    __syncthreads();
    // the digit whose bin holds rank k: thread d owns bin d (an exclusive scan over 256 bins)
    long long c = tid < 256 ? (long long)s_hist[tid] : 0, incl = c;
    for (int off = 1; off < 64; off <<= 1) {
      const long long n = __shfl_up(incl, off);
      if (lane >= off) incl += n;
    }
    __syncthreads();
    if (lane == 63) s_w[wave] = incl;
    __syncthreads();
    long long before = 0;
    for (int w = 0; w < 4; ++w) before += (w < wave) ? s_w[w] : 0;   // bins live in waves 0..3
    before += incl - c;
    __syncthreads();
    if (tid < 256 && c > 0 && before < k && k <= before + c) {
      s_w[8] = tid;
      s_w[9] = before;
    }
    __syncthreads();
    prefix |= (unsigned int)s_w[8] << shift;
    k -= s_w[9];
    __syncthreads();
  }
  // prefix = key of the need-th smallest stamp; k = how many of the candidates AT that stamp go (the lowest slots)
  // ---- one pass in slot order
  long long taken_at = 0;  // candidates at the threshold stamp seen so far, the same for every thread
  for (long long base = 0; base < P; base += kEvictThreads) {
    const long long p = base + tid;
    bool below = false, at = false;
    if (p < P && candidate(p)) {
      const unsigned int key = stamp_key(last_used[p]);
      below = key < prefix;
      at = key == prefix;
    }
    // rank of this thread's slot among the at-threshold candidates of this chunk
    const unsigned long long bal = __ballot(at);
    const int in_wave = __popcll(bal & ((1ull << lane) - 1ull));
    if (lane == 0) s_scan[wave] = __popcll(bal);
    __syncthreads();
    int before = 0, total = 0;
#pragma unroll
    for (int w = 0; w < kEvictThreads / 64; ++w) {
      const int cw = s_scan[w];
      before += (w < wave) ? cw : 0;
      total += cw;
    }
    if (below || (at && taken_at + before + in_wave < k)) live[p] = 0;
    taken_at += total;
    __syncthreads();
  }
  if (tid == 0) {
    *n_free = (int32_t)(free0 + need);
    *n_evicted = (int32_t)need;
  }
}

}  // namespace
}  // namespace rc

extern "C" rc_status rc_pool_touch(const int32_t* slots, int64_t n, int32_t value, int32_t* array, int64_t P,
                                   void* hip_stream) {
  using namespace rc;
  clear_error();
  if (n < 0 || P < 0) return fail(RC_ERR_INVALID_ARG, "rc_pool_touch: negative size");
  if (n == 0 || P == 0) return RC_OK;
  if (!slots || !array) return fail(RC_ERR_INVALID_ARG, "rc_pool_touch: NULL pointer");
  if (n > 0x7fffffffLL * 256) return fail(RC_ERR_UNSUPPORTED, "rc_pool_touch: n beyond the grid limits");
  touch_kernel<<<(unsigned)((n + 255) / 256), 256, 0, static_cast<hipStream_t>(hip_stream)>>>(slots, (long long)n, value,
                                                                                             array, (long long)P);
  return check_launch("rc_pool_touch");
}

extern "C" rc_status rc_refcount_release(const int32_t* ids, int64_t n, int32_t* refcount, int64_t NB, void* hip_stream) {
  using namespace rc;
  clear_error();
  if (n < 0 || NB < 0) return fail(RC_ERR_INVALID_ARG, "rc_refcount_release: negative size");
  if (n == 0 || NB == 0) return RC_OK;
  if (!ids || !refcount) return fail(RC_ERR_INVALID_ARG, "rc_refcount_release: NULL pointer");
  if (n > 0x7fffffffLL * 256) return fail(RC_ERR_UNSUPPORTED, "rc_refcount_release: n beyond the grid limits");
  release_kernel<<<(unsigned)((n + 255) / 256), 256, 0, static_cast<hipStream_t>(hip_stream)>>>(ids, (long long)n, refcount,
                                                                                               (long long)NB);
  return check_launch("rc_refcount_release");
}

extern "C" rc_status rc_pool_evict(int64_t P, uint8_t* pool_live, const int32_t* refcount, const int32_t* last_used,
                                   const int32_t* match_idx, int64_t Q, int64_t extra_wanted, int32_t* n_free,
                                   int32_t* n_evicted, void* hip_stream) {
  using namespace rc;
  clear_error();
  if (P < 0 || Q < 0 || extra_wanted < 0) return fail(RC_ERR_INVALID_ARG, "rc_pool_evict: negative size");
  if (!n_free || !n_evicted) return fail(RC_ERR_INVALID_ARG, "rc_pool_evict: NULL output pointer");
  if ((P > 0 && (!pool_live || !last_used)) || (Q > 0 && !match_idx))
    return fail(RC_ERR_INVALID_ARG, "rc_pool_evict: NULL pointer");
  if (P > 0x7fffffffLL || Q > 0x7fffffffLL) return fail(RC_ERR_UNSUPPORTED, "rc_pool_evict: more than 2^31 - 1 slots or queries");
  evict_kernel<<<1, kEvictThreads, 0, static_cast<hipStream_t>(hip_stream)>>>(
      (long long)P, pool_live, refcount, last_used, match_idx, (long long)Q, (long long)extra_wanted, n_free, n_evicted);
  return check_launch("rc_pool_evict");
}
