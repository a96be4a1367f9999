// rc_pat_threshold, rc_apply_threshold: percentile-based adaptive thresholding (ReasonCache
// Sec. IV-A, PAT).  The threshold is the nearest-rank p-th percentile of the distances collected
// during warm-up: an exact order statistic, found by a radix select over the bit patterns (four
// passes of 8 bits, most significant first).  Each pass histograms one byte of the keys that
// still match the prefix chosen so far; the next pass derives that prefix again from the
// histograms (256 bins per pass, every workgroup repeats the short scan), so no pass needs a
// launch of its own for the scan.  Integer counts only: the result is the same on every run.
#include <hip/hip_runtime.h>

#include "rc_common.hpp"

namespace rc {
namespace {

constexpr int kPatThreads = 256;

struct PatState {
  unsigned int hist[4][256];
  unsigned int nonfinite;
  unsigned int pad[3];
};

// Order-preserving map float -> unsigned; every non-finite value becomes the largest key.
__device__ __forceinline__ unsigned int key_of(float x) {
  const unsigned int b = __float_as_uint(x);
  const bool finite = (b & 0x7f800000u) != 0x7f800000u;
  const unsigned int k = (b & 0x80000000u) ? ~b : (b | 0x80000000u);
  return finite ? k : 0xffffffffu;
}

__device__ __forceinline__ float value_of(unsigned int k) {
  return __uint_as_float((k & 0x80000000u) ? (k & 0x7fffffffu) : ~k);
}

__global__ __launch_bounds__(kPatThreads) void pat_clear_kernel(PatState* st) {
  unsigned int* w = reinterpret_cast<unsigned int*>(st);
  for (int i = threadIdx.x; i < (int)(sizeof(PatState) / 4); i += kPatThreads) w[i] = 0u;
}

// Rank of the percentile among the n_f finite samples: ceil(p/100 * n_f) in double, within [1, n_f].
__device__ __forceinline__ long long pat_rank(double p, long long n_f) {
  long long k = (long long)ceil(p * (double)n_f / 100.0);
  if (k < 1) k = 1;
  if (k > n_f) k = n_f;
  return k;
}

// Exclusive prefix sum of one value per thread over the 256 threads of the workgroup.
__device__ __forceinline__ long long scan256(long long v, long long* s_wave /* [4] */) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  long long incl = v;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const long long n = __shfl_up(incl, off);
    if (lane >= off) incl += n;
  }
  __syncthreads();  // s_wave may still be read from the previous call
  if (lane == 63) s_wave[wave] = incl;
  __syncthreads();
  long long before = 0;
#pragma unroll
  for (int w = 0; w < 4; ++w) before += (w < wave) ? s_wave[w] : 0;
  return before + incl - v;
}

// The bytes fixed by passes 0 .. npass-1 (s_h holds their histograms): in every pass the digit
// whose bin contains rank k, found by all 256 threads together (thread d owns bin d).
// Returns the prefix to every thread.  s_sel: two words of scratch.
__device__ __forceinline__ unsigned int pat_prefix(const unsigned int (*s_h)[256], int npass, long long k,
                                                   long long* s_wave, long long* s_sel) {
  unsigned int prefix = 0;
  for (int j = 0; j < npass; ++j) {
    const long long c = s_h[j][threadIdx.x];
    const long long before = scan256(c, s_wave);
    if (threadIdx.x == 0) s_sel[0] = -1;
    __syncthreads();
    if (c > 0 && before < k && k <= before + c) {  // exactly one bin, if k is within the total
      s_sel[0] = threadIdx.x;
      s_sel[1] = before;
    }
    __syncthreads();
    const long long digit = s_sel[0] < 0 ? 255 : s_sel[0];
    k -= s_sel[0] < 0 ? 0 : s_sel[1];
    prefix |= (unsigned int)digit << (24 - 8 * j);
    __syncthreads();
  }
  return prefix;
}

__global__ __launch_bounds__(kPatThreads) void pat_hist_kernel(const float* __restrict__ s, long long n, double p,
                                                               PatState* st, int pass) {
  __shared__ unsigned int s_h[3][256];
  __shared__ unsigned int s_local[256];
  __shared__ long long s_wave[4], s_sel[2];
  __shared__ unsigned int s_bad;
  const int tid = threadIdx.x;
  s_local[tid] = 0u;
  if (tid == 0) s_bad = 0u;
  for (int j = 0; j < pass; ++j) s_h[j][tid] = st->hist[j][tid];
  __syncthreads();
  const long long n_f = n - (long long)st->nonfinite;  // final once pass 0 is complete
  const unsigned int prefix = (pass > 0 && n_f > 0) ? pat_prefix(s_h, pass, pat_rank(p, n_f), s_wave, s_sel) : 0u;
  const unsigned int mask = pass == 0 ? 0u : 0xffffffffu << (32 - 8 * pass);
  const int shift = 24 - 8 * pass;
  unsigned int bad = 0;
  for (long long i = (long long)blockIdx.x * kPatThreads + tid; i < n; i += (long long)gridDim.x * kPatThreads) {
    const unsigned int k = key_of(s[i]);
    if ((k & mask) == prefix) atomicAdd(&s_local[(k >> shift) & 255u], 1u);
    bad += (k == 0xffffffffu);
  }
  if (pass == 0 && bad) atomicAdd(&s_bad, bad);
  __syncthreads();
  if (s_local[tid]) atomicAdd(&st->hist[pass][tid], s_local[tid]);
  if (pass == 0 && tid == 0 && s_bad) atomicAdd(&st->nonfinite, s_bad);
}

__global__ __launch_bounds__(kPatThreads) void pat_final_kernel(long long n, double p, const PatState* st,
                                                                float* __restrict__ threshold,
                                                                long long* __restrict__ n_finite) {
  __shared__ unsigned int s_h[4][256];
  __shared__ long long s_wave[4], s_sel[2];
  const int tid = threadIdx.x;
  for (int j = 0; j < 4; ++j) s_h[j][tid] = st->hist[j][tid];
  __syncthreads();
  const long long n_f = n - (long long)st->nonfinite;
  const unsigned int key = n_f > 0 ? pat_prefix(s_h, 4, pat_rank(p, n_f), s_wave, s_sel) : 0u;
  if (tid == 0) {
    *threshold = n_f > 0 ? value_of(key) : -INFINITY;
    if (n_finite) *n_finite = n_f;
  }
}

__global__ __launch_bounds__(256) void apply_threshold_kernel(const int32_t* __restrict__ best_idx,
                                                              const float* __restrict__ best_dist, long long n,
                                                              const float* __restrict__ threshold,
                                                              int32_t* __restrict__ match_idx) {
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const float thr = *threshold;
  const int idx = best_idx[i];
  match_idx[i] = (idx >= 0 && best_dist[i] <= thr) ? idx : -1;
}

}  // namespace
}  // namespace rc

extern "C" size_t rc_pat_workspace_size(void) { return sizeof(rc::PatState); }

extern "C" rc_status rc_pat_threshold(const float* samples, int64_t n, double p, float* threshold, int64_t* n_finite,
                                      void* workspace, size_t workspace_bytes, void* hip_stream) {
  using namespace rc;
  clear_error();
  if (n < 0 || n > 0x7fffffffLL) return fail(RC_ERR_INVALID_ARG, "rc_pat_threshold: n = %lld outside [0, 2^31)", (long long)n);
  if (!(p >= 0.0 && p <= 100.0)) return fail(RC_ERR_INVALID_ARG, "rc_pat_threshold: p = %g outside [0, 100]", p);
  if (!threshold || (n > 0 && !samples)) return fail(RC_ERR_INVALID_ARG, "rc_pat_threshold: NULL samples or threshold");
  if (!workspace || workspace_bytes < sizeof(PatState) || !aligned16(workspace))
    return fail(RC_ERR_WORKSPACE, "rc_pat_threshold: workspace of %zu bytes needed (16-byte aligned), got %zu",
                sizeof(PatState), workspace_bytes);
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  PatState* state = static_cast<PatState*>(workspace);
  pat_clear_kernel<<<1, kPatThreads, 0, st>>>(state);
  if (rc_status s = check_launch("rc_pat_threshold(clear)")) return s;
  if (n > 0) {
    long long wgs = (n + kPatThreads * 16 - 1) / (kPatThreads * 16);  // about 16 samples per thread
    if (wgs > 2048) wgs = 2048;
    for (int pass = 0; pass < 4; ++pass) {
      pat_hist_kernel<<<(unsigned)wgs, kPatThreads, 0, st>>>(samples, (long long)n, p, state, pass);
      if (rc_status s = check_launch("rc_pat_threshold(histogram)")) return s;
    }
  }
  pat_final_kernel<<<1, kPatThreads, 0, st>>>((long long)n, p, state, threshold,
                                              reinterpret_cast<long long*>(n_finite));
  return check_launch("rc_pat_threshold(final)");
}

extern "C" rc_status rc_apply_threshold(const int32_t* best_idx, const float* best_dist, int64_t n,
                                        const float* threshold, int32_t* match_idx, void* hip_stream) {
  using namespace rc;
  clear_error();
  if (n < 0) return fail(RC_ERR_INVALID_ARG, "rc_apply_threshold: negative n");
  if (n == 0) return RC_OK;
  if (!best_idx || !best_dist || !threshold || !match_idx)
    return fail(RC_ERR_INVALID_ARG, "rc_apply_threshold: NULL pointer");
  if (n > 0x7fffffffLL * 256) return fail(RC_ERR_UNSUPPORTED, "rc_apply_threshold: n beyond the grid limits");
  apply_threshold_kernel<<<(unsigned)((n + 255) / 256), 256, 0, static_cast<hipStream_t>(hip_stream)>>>(
      best_idx, best_dist, (long long)n, threshold, match_idx);
  return check_launch("rc_apply_threshold");
}
