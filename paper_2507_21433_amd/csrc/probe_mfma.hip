// Measurement aid, not part of the search path: the rate at which this chip sustains back-to-back
// v_mfma_f32_32x32x16_f16 on operands like the workload's (random fp16), with nothing else going on.
// The chip lowers its clock under matrix load, so this rate -- not the 2.5 PFLOP/s of the data sheet,
// which is 256 CUs x 4 SIMDs x 1024 FLOP/clock at 2.4 GHz -- is what a kernel made of nothing but MFMA
// would reach on the box the benchmark runs on.  The benchmark reports it next to the score kernel's rate.
// Built into a library of its own (librc_probe.so); the search library does not contain it.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kWaves = 4;   // one per SIMD
constexpr int kTile = 4;    // 4 x 4 accumulators of 32 x 32: all 256 accumulator registers, as in the score kernel

__global__ __launch_bounds__(64 * kWaves, 1) void mfma_rate_kernel(const uint4* operands, int iters, float* sink) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  f16x8 a[kTile], b[kTile];
#pragma unroll
  for (int i = 0; i < kTile; ++i) {
    a[i] = __builtin_bit_cast(f16x8, operands[(wave * 2 * kTile + i) * 64 + lane]);
    b[i] = __builtin_bit_cast(f16x8, operands[(wave * 2 * kTile + kTile + i) * 64 + lane]);
  }
  f32x16 acc[kTile][kTile];
#pragma unroll
  for (int i = 0; i < kTile; ++i)
#pragma unroll
    for (int j = 0; j < kTile; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
#pragma unroll 4
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < kTile; ++i)
#pragma unroll
      for (int j = 0; j < kTile; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[i], b[j], acc[i][j], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < kTile; ++i)
#pragma unroll
    for (int j = 0; j < kTile; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) s += acc[i][j][e];
  sink[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

}  // namespace

// operands: device, 4 waves x 8 fragments x 64 lanes x 16 bytes = 32 KiB of fp16 values (read once);
// sink: device, grid x 256 floats (written once, keeps the accumulators alive); grid: workgroups, one per
// compute unit; stream: hipStream_t.  Every workgroup issues iters x 16 MFMAs per wave, i.e. the launch
// performs grid x 4 x iters x 16 x 32768 FLOP.  Returns 0, or the hipError_t of the launch.
extern "C" int rc_probe_mfma_f16(const void* operands, int32_t iters, float* sink, int32_t grid, void* stream) {
  if (!operands || !sink || iters < 0 || grid <= 0) return (int)hipErrorInvalidValue;
  mfma_rate_kernel<<<grid, 64 * kWaves, 0, static_cast<hipStream_t>(stream)>>>(static_cast<const uint4*>(operands), iters, sink);
  return (int)hipGetLastError();
}
