// Shared host-side helpers of the C-ABI library: error text, argument checks, launch checks.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdint>
#include <cstdio>

#include "rc.h"

namespace rc {

// Thread-local text behind rc_last_error().
char* error_buffer();
constexpr int kErrorBufferBytes = 512;

inline rc_status fail(rc_status code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(error_buffer(), kErrorBufferBytes, fmt, ap);
  va_end(ap);
  return code;
}

inline void clear_error() { error_buffer()[0] = '\0'; }

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Shape rules shared by every entry point that takes a KV descriptor.
inline rc_status check_desc(const rc_kv_desc* d, int64_t n_blocks, const char* who) {
  if (!d) return fail(RC_ERR_INVALID_ARG, "%s: descriptor is NULL", who);
  if (d->n_layers < 0 || n_blocks < 0) return fail(RC_ERR_INVALID_ARG, "%s: negative size", who);
  if (d->dtype != RC_F16 && d->dtype != RC_BF16) return fail(RC_ERR_UNSUPPORTED, "%s: dtype %d", who, d->dtype);
  if (d->head_dim != 128) return fail(RC_ERR_UNSUPPORTED, "%s: head_dim %d (only 128)", who, d->head_dim);
  if (d->block_tokens != 16 && d->block_tokens != 32)
    return fail(RC_ERR_UNSUPPORTED, "%s: block_tokens %d (only 16 or 32)", who, d->block_tokens);
  if (d->n_kv_heads < 1 || d->n_kv_heads > 16)
    return fail(RC_ERR_UNSUPPORTED, "%s: n_kv_heads %d (1..16)", who, d->n_kv_heads);
  const int64_t block_elems = (int64_t)d->block_tokens * d->n_kv_heads * d->head_dim;
  if (d->layer_stride < n_blocks * block_elems)
    return fail(RC_ERR_INVALID_ARG, "%s: layer_stride %lld smaller than n_blocks*T*H*Dh", who,
                (long long)d->layer_stride);
  if ((d->layer_stride * 2) % 16 != 0) return fail(RC_ERR_INVALID_ARG, "%s: layer_stride breaks 16-byte alignment", who);
  return RC_OK;
}

inline rc_status check_launch(const char* who) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(RC_ERR_DEVICE, "%s: %s", who, hipGetErrorString(e));
  return RC_OK;
}

}  // namespace rc
