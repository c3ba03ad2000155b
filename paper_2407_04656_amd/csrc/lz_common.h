// Internal helpers shared by the HIP translation units (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "lazarus_moe.h"

namespace lz {

constexpr int kMaxK = 8;
constexpr int kMaxE = 256;
constexpr int kMaxN = 64;
constexpr int kMaxC = 64;
constexpr int kWave = 64;

inline bool shape_ok(const lz_shape* s) {
  if (!s) return false;
  if (s->T < 0 || s->d < 1 || s->ffn < 1) return false;
  if (s->E < 1 || s->E > kMaxE) return false;
  if (s->k < 1 || s->k > kMaxK || s->k > s->E) return false;
  if (s->N < 1 || s->N > kMaxN || s->c < 1 || s->c > kMaxC) return false;
  if (s->dtype != LZ_F32 && s->dtype != LZ_BF16) return false;
  if (s->act != LZ_GELU && s->act != LZ_SWIGLU) return false;
  if (int64_t(s->T) * s->k > (int64_t(1) << 30)) return false;  // pair and row indices are int32
  return true;
}

inline size_t elem_bytes(int dtype) { return dtype == LZ_F32 ? 4 : 2; }

inline size_t align256(size_t v) { return (v + 255) & ~size_t(255); }

inline int32_t launch_status() { return hipGetLastError() == hipSuccess ? LZ_OK : LZ_EHIP; }

// bf16 <-> fp32 on the device (round to nearest even; inputs are finite)
__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float(uint32_t(b) << 16); }
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return uint16_t(u >> 16);
}

}  // namespace lz
