// rc_block_norms: squared L2 norm of every K and V block (ReasonCache Sec. IV-A Stage 2,
// the cached norm terms of the squared-distance expansion).  HBM-bound streaming reduction:
// one workgroup reads one block's K tensor and V tensor with 16-byte coalesced loads.
#include <hip/hip_runtime.h>

#include "rc_common.hpp"

namespace rc {

char* error_buffer() {
  static thread_local char buf[kErrorBufferBytes] = {0};
  return buf;
}

namespace {

constexpr int kNormThreads = 256;

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// Sum of squares of the 8 fp16 / bf16 values packed in a 16-byte word, in fp32.
// A product of two 16-bit floats is exact in fp32.
template <bool BF16>
__device__ __forceinline__ float sumsq8(u32x4 w, float acc) {
  const uint32_t u[4] = {w[0], w[1], w[2], w[3]};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    if (BF16) {
      float lo = __uint_as_float(u[i] << 16);
      float hi = __uint_as_float(u[i] & 0xffff0000u);
      acc = fmaf(lo, lo, acc);
      acc = fmaf(hi, hi, acc);
    } else {
      half2_t h = __builtin_bit_cast(half2_t, u[i]);
      acc = __builtin_amdgcn_fdot2(h, h, acc, false);
    }
  }
  return acc;
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
  return v;
}

// Block mode.  grid = (n_blocks, L); thread t takes 16-byte chunks t, t+256, ... of the tensor.
template <bool BF16>
__global__ __launch_bounds__(kNormThreads) void norms_block_kernel(const char* __restrict__ k,
                                                                   const char* __restrict__ v,
                                                                   float* __restrict__ ksq, float* __restrict__ vsq,
                                                                   long long layer_stride_b, int block_bytes,
                                                                   long long n_blocks) {
  __shared__ float red[2][kNormThreads / 64];
  const long long b = blockIdx.x, l = blockIdx.y;
  const long long off = l * layer_stride_b + b * (long long)block_bytes;
  const u32x4* kp = reinterpret_cast<const u32x4*>(k + off);
  const u32x4* vp = reinterpret_cast<const u32x4*>(v + off);
  const int chunks = block_bytes / 16;
  float ak0 = 0.f, ak1 = 0.f, av0 = 0.f, av1 = 0.f;
  int c = threadIdx.x;
  for (; c + kNormThreads < chunks; c += 2 * kNormThreads) {
    u32x4 a0 = __builtin_nontemporal_load(kp + c), a1 = __builtin_nontemporal_load(kp + c + kNormThreads);
    u32x4 b0 = __builtin_nontemporal_load(vp + c), b1 = __builtin_nontemporal_load(vp + c + kNormThreads);
    ak0 = sumsq8<BF16>(a0, ak0);
    ak1 = sumsq8<BF16>(a1, ak1);
    av0 = sumsq8<BF16>(b0, av0);
    av1 = sumsq8<BF16>(b1, av1);
  }
  for (; c < chunks; c += kNormThreads) {
    ak0 = sumsq8<BF16>(__builtin_nontemporal_load(kp + c), ak0);
    av0 = sumsq8<BF16>(__builtin_nontemporal_load(vp + c), av0);
  }
  float sk = wave_sum(ak0 + ak1), sv = wave_sum(av0 + av1);
  const int wave = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) {
    red[0][wave] = sk;
    red[1][wave] = sv;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    float tk = 0.f, tv = 0.f;
#pragma unroll
    for (int w = 0; w < kNormThreads / 64; ++w) {
      tk += red[0][w];
      tv += red[1][w];
    }
    ksq[l * n_blocks + b] = tk;
    vsq[l * n_blocks + b] = tv;
  }
}

// Per-head mode.  A token holds H*16 chunks of 16 bytes; 16 consecutive chunks are one head.
// tpg = 16*H threads cover one token, 256/tpg tokens are read side by side, so a thread always
// stays in the same head.  Partials are summed per head in a fixed order.
template <bool BF16>
__global__ __launch_bounds__(kNormThreads) void norms_head_kernel(const char* __restrict__ k,
                                                                  const char* __restrict__ v,
                                                                  float* __restrict__ ksq, float* __restrict__ vsq,
                                                                  long long layer_stride_b, int T, int H,
                                                                  long long n_blocks) {
  __shared__ float red[2][kNormThreads];
  const long long b = blockIdx.x, l = blockIdx.y;
  const int tpg = 16 * H, groups = kNormThreads / tpg;
  const long long off = l * layer_stride_b + b * (long long)T * tpg * 16;
  const u32x4* kp = reinterpret_cast<const u32x4*>(k + off);
  const u32x4* vp = reinterpret_cast<const u32x4*>(v + off);
  const int g = threadIdx.x / tpg, j = threadIdx.x % tpg;
  float ak = 0.f, av = 0.f;
  if (g < groups) {
    for (int t = g; t < T; t += groups) {
      ak = sumsq8<BF16>(__builtin_nontemporal_load(kp + t * tpg + j), ak);
      av = sumsq8<BF16>(__builtin_nontemporal_load(vp + t * tpg + j), av);
    }
  }
  red[0][threadIdx.x] = ak;
  red[1][threadIdx.x] = av;
  __syncthreads();
  if (threadIdx.x < 2 * H) {
    const int which = threadIdx.x / H, h = threadIdx.x % H;
    float s = 0.f;
    for (int gg = 0; gg < groups; ++gg)
      for (int i = 0; i < 16; ++i) s += red[which][gg * tpg + h * 16 + i];
    (which ? vsq : ksq)[(l * n_blocks + b) * H + h] = s;
  }
}

}  // namespace
}  // namespace rc

extern "C" rc_status rc_block_norms(const rc_kv_desc* desc, int32_t mode, const void* k, const void* v,
                                    int64_t n_blocks, float* k_sqnorm, float* v_sqnorm, void* hip_stream) {
  using namespace rc;
  clear_error();
  if (rc_status s = check_desc(desc, n_blocks, "rc_block_norms")) return s;
  if (mode != RC_SCORE_BLOCK && mode != RC_SCORE_PER_HEAD_ALL)
    return fail(RC_ERR_UNSUPPORTED, "rc_block_norms: mode %d", mode);
  if (n_blocks == 0 || desc->n_layers == 0) return RC_OK;
  if (!k || !v || !k_sqnorm || !v_sqnorm) return fail(RC_ERR_INVALID_ARG, "rc_block_norms: NULL pointer");
  if (!aligned16(k) || !aligned16(v)) return fail(RC_ERR_INVALID_ARG, "rc_block_norms: KV pointer not 16-byte aligned");
  if (n_blocks > 0x7fffffffLL || desc->n_layers > 65535)
    return fail(RC_ERR_UNSUPPORTED, "rc_block_norms: n_blocks or n_layers beyond the grid limits");
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const dim3 grid((unsigned)n_blocks, (unsigned)desc->n_layers);
  const long long lsb = desc->layer_stride * 2;
  const int T = desc->block_tokens, H = desc->n_kv_heads;
  const int block_bytes = T * H * desc->head_dim * 2;
  const char* kc = static_cast<const char*>(k);
  const char* vc = static_cast<const char*>(v);
  const bool bf = desc->dtype == RC_BF16;
  if (mode == RC_SCORE_BLOCK) {
    if (bf)
      norms_block_kernel<true><<<grid, kNormThreads, 0, st>>>(kc, vc, k_sqnorm, v_sqnorm, lsb, block_bytes, n_blocks);
    else
      norms_block_kernel<false><<<grid, kNormThreads, 0, st>>>(kc, vc, k_sqnorm, v_sqnorm, lsb, block_bytes, n_blocks);
  } else {
    if (bf)
      norms_head_kernel<true><<<grid, kNormThreads, 0, st>>>(kc, vc, k_sqnorm, v_sqnorm, lsb, T, H, n_blocks);
    else
      norms_head_kernel<false><<<grid, kNormThreads, 0, st>>>(kc, vc, k_sqnorm, v_sqnorm, lsb, T, H, n_blocks);
  }
  return check_launch("rc_block_norms");
}

extern "C" const char* rc_last_error(void) { return rc::error_buffer(); }

extern "C" int32_t rc_version(void) { return 200; }  // 0.2.0: layer-mean distance, candidate lists, percentile threshold, admission
