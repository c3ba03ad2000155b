// Data movement of the dispatcher: the reshuffle into per-slot contiguous buffers
// (Algorithm 1's h -> h') and its inverse fused with the gate-weighted combine (Sec. 2.1).
// Both are pure HBM streaming: one wave per row, 16-byte accesses per lane, several rows'
// worth of loads in flight before the first store.
#include "lz_common.h"

namespace {

constexpr int kRowsPerBlock = 4;  // one wave per row

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));  // one 16-byte access

// xp[row, :] = x[row_to_pair[row] / k, :]   (16-byte vectors; row_bytes % 16 == 0)
__global__ __launch_bounds__(256) void permute_vec_kernel(const u32x4* __restrict__ x,
                                                          const int32_t* __restrict__ row_to_pair,
                                                          long long P, int k, int vec_per_row,
                                                          u32x4* __restrict__ xp) {
  const int lane = threadIdx.x % lz::kWave;
  const long long row = (long long)blockIdx.x * kRowsPerBlock + threadIdx.x / lz::kWave;
  if (row >= P) return;
  const int pair = row_to_pair[row];
  const bool ok = pair >= 0 && pair < P;
  const u32x4* src = x + (size_t)(ok ? pair / k : 0) * vec_per_row;
  u32x4* dst = xp + (size_t)row * vec_per_row;
  const u32x4 zero = {0u, 0u, 0u, 0u};
  int v = lane;
  for (; v + 3 * lz::kWave < vec_per_row; v += 4 * lz::kWave) {
    u32x4 a = src[v], b = src[v + lz::kWave], c = src[v + 2 * lz::kWave], d = src[v + 3 * lz::kWave];
    if (!ok) a = b = c = d = zero;
    __builtin_nontemporal_store(a, dst + v);
    __builtin_nontemporal_store(b, dst + v + lz::kWave);
    __builtin_nontemporal_store(c, dst + v + 2 * lz::kWave);
    __builtin_nontemporal_store(d, dst + v + 3 * lz::kWave);
  }
  for (; v < vec_per_row; v += lz::kWave) {
    u32x4 a = src[v];
    if (!ok) a = zero;
    __builtin_nontemporal_store(a, dst + v);
  }
}

// element-wise fallback for rows that are not a multiple of 16 bytes
template <typename Elem>
__global__ __launch_bounds__(256) void permute_elem_kernel(const Elem* __restrict__ x,
                                                           const int32_t* __restrict__ row_to_pair,
                                                           long long P, int k, int d,
                                                           Elem* __restrict__ xp) {
  const int lane = threadIdx.x % lz::kWave;
  const long long row = (long long)blockIdx.x * kRowsPerBlock + threadIdx.x / lz::kWave;
  if (row >= P) return;
  const int pair = row_to_pair[row];
  const bool ok = pair >= 0 && pair < P;
  const Elem* src = x + (size_t)(ok ? pair / k : 0) * d;
  for (int v = lane; v < d; v += lz::kWave) xp[(size_t)row * d + v] = ok ? src[v] : Elem(0);
}

// Token-major form of the same reshuffle: xp[pair_to_row[t*k+kk], :] = x[t, :] for every pair.
// Each row of x is read once and written k times, which is exactly the compulsory traffic
// (the row-major gather above re-reads x once per copy when the copies land on different XCDs).
// U lane-vectors of the row are loaded before the first is stored.
template <int U>
__global__ __launch_bounds__(256) void permute_scatter_kernel(const u32x4* __restrict__ x,
                                                              const int32_t* __restrict__ pair_to_row,
                                                              int T, int k, long long P, int vec_per_row,
                                                              u32x4* __restrict__ xp) {
  const int lane = threadIdx.x % lz::kWave;
  const long long t = (long long)blockIdx.x * kRowsPerBlock + threadIdx.x / lz::kWave;
  if (t >= T) return;
  long long rows[lz::kMaxK];
#pragma unroll
  for (int kk = 0; kk < lz::kMaxK; ++kk) {
    rows[kk] = -1;
    if (kk < k) {
      const int r = pair_to_row[t * k + kk];
      rows[kk] = (r >= 0 && r < P) ? r : -1;
    }
  }
  const u32x4* src = x + (size_t)t * vec_per_row;
  int v = lane;
  for (; v + (U - 1) * lz::kWave < vec_per_row; v += U * lz::kWave) {
    u32x4 in[U];
#pragma unroll
    for (int u = 0; u < U; ++u) in[u] = __builtin_nontemporal_load(src + v + u * lz::kWave);
#pragma unroll
    for (int kk = 0; kk < lz::kMaxK; ++kk)
      if (kk < k && rows[kk] >= 0) {
        u32x4* dst = xp + (size_t)rows[kk] * vec_per_row + v;
#pragma unroll
        for (int u = 0; u < U; ++u) __builtin_nontemporal_store(in[u], dst + u * lz::kWave);
      }
  }
  for (; v < vec_per_row; v += lz::kWave) {
    const u32x4 a = __builtin_nontemporal_load(src + v);
#pragma unroll
    for (int kk = 0; kk < lz::kMaxK; ++kk)
      if (kk < k && rows[kk] >= 0) __builtin_nontemporal_store(a, xp + (size_t)rows[kk] * vec_per_row + v);
  }
}

template <typename Elem>
__global__ __launch_bounds__(256) void permute_scatter_elem_kernel(const Elem* __restrict__ x,
                                                                   const int32_t* __restrict__ pair_to_row,
                                                                   int T, int k, long long P, int d,
                                                                   Elem* __restrict__ xp) {
  const int lane = threadIdx.x % lz::kWave;
  const long long t = (long long)blockIdx.x * kRowsPerBlock + threadIdx.x / lz::kWave;
  if (t >= T) return;
  for (int kk = 0; kk < k; ++kk) {
    const int r = pair_to_row[t * k + kk];
    if (r < 0 || r >= P) continue;
    for (int v = lane; v < d; v += lz::kWave) xp[(size_t)r * d + v] = x[(size_t)t * d + v];
  }
}

__device__ __forceinline__ void fma8(float* acc, const u32x4& v, float g) {
  const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    acc[2 * q] = fmaf(g, __uint_as_float(w[q] << 16), acc[2 * q]);
    acc[2 * q + 1] = fmaf(g, __uint_as_float(w[q] & 0xFFFF0000u), acc[2 * q + 1]);
  }
}

// y[t, :] = sum_kk gate[t, kk] * yp[pair_to_row[t*k+kk], :]   bf16, 8 elements per lane-vector
// (gates == nullptr: all gates 1, the backward of the reshuffle).  K = top-k (compile time, so the
// row indices and loaded vectors stay in registers); U lane-vectors of every row are loaded before
// the first is used, K * U 16-byte loads in flight per lane.
template <int K, int U>
__global__ __launch_bounds__(256) void combine_bf16_kernel(const u32x4* __restrict__ yp,
                                                           const int32_t* __restrict__ pair_to_row,
                                                           const float* __restrict__ gates, int T,
                                                           long long P, int vec_per_row,
                                                           u32x4* __restrict__ y) {
  const int lane = threadIdx.x % lz::kWave;
  const long long t = (long long)blockIdx.x * kRowsPerBlock + threadIdx.x / lz::kWave;
  if (t >= T) return;
  const u32x4* src[K];
  float g[K];
  bool ok[K];  // a pair without a row adds nothing (the same for the whole wave: no divergence)
#pragma unroll
  for (int kk = 0; kk < K; ++kk) {
    const int r = pair_to_row[t * K + kk];
    ok[kk] = r >= 0 && r < P;
    src[kk] = yp + (size_t)(ok[kk] ? r : 0) * vec_per_row;
    g[kk] = gates ? gates[t * K + kk] : 1.f;
  }
  auto pack = [](const float* acc) {
    u32x4 out;
    out.x = uint32_t(lz::f32_to_bf16(acc[0])) | (uint32_t(lz::f32_to_bf16(acc[1])) << 16);
    out.y = uint32_t(lz::f32_to_bf16(acc[2])) | (uint32_t(lz::f32_to_bf16(acc[3])) << 16);
    out.z = uint32_t(lz::f32_to_bf16(acc[4])) | (uint32_t(lz::f32_to_bf16(acc[5])) << 16);
    out.w = uint32_t(lz::f32_to_bf16(acc[6])) | (uint32_t(lz::f32_to_bf16(acc[7])) << 16);
    return out;
  };
  u32x4* const dst = y + (size_t)t * vec_per_row;
  int v = lane;
  for (; v + (U - 1) * lz::kWave < vec_per_row; v += U * lz::kWave) {
    u32x4 in[U][K];
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int kk = 0; kk < K; ++kk)
        if (ok[kk]) in[u][kk] = __builtin_nontemporal_load(src[kk] + v + u * lz::kWave);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int kk = 0; kk < K; ++kk)
        if (ok[kk]) fma8(acc, in[u][kk], g[kk]);
      dst[v + u * lz::kWave] = pack(acc);
    }
  }
  for (; v < vec_per_row; v += lz::kWave) {
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kk = 0; kk < K; ++kk)
      if (ok[kk]) fma8(acc, __builtin_nontemporal_load(src[kk] + v), g[kk]);
    dst[v] = pack(acc);
  }
}

// generic element-wise combine (fp32 tensors, or bf16 rows not a multiple of 16 bytes)
template <bool BF16>
__global__ __launch_bounds__(256) void combine_elem_kernel(const void* __restrict__ yp_,
                                                           const int32_t* __restrict__ pair_to_row,
                                                           const float* __restrict__ gates, int T,
                                                           int k, long long P, int d,
                                                           void* __restrict__ y_) {
  const int lane = threadIdx.x % lz::kWave;
  const long long t = (long long)blockIdx.x * kRowsPerBlock + threadIdx.x / lz::kWave;
  if (t >= T) return;
  for (int v = lane; v < d; v += lz::kWave) {
    float acc = 0.f;
    for (int kk = 0; kk < k; ++kk) {
      const int r = pair_to_row[t * k + kk];
      if (r < 0 || r >= P) continue;
      float val;
      if (BF16) val = lz::bf16_to_f32(((const uint16_t*)yp_)[(size_t)r * d + v]);
      else val = ((const float*)yp_)[(size_t)r * d + v];
      acc = fmaf(gates ? gates[t * k + kk] : 1.f, val, acc);
    }
    if (BF16) ((uint16_t*)y_)[(size_t)t * d + v] = lz::f32_to_bf16(acc);
    else ((float*)y_)[(size_t)t * d + v] = acc;
  }
}

inline bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }

}  // namespace

extern "C" int32_t lz_permute(const void* x, const int32_t* row_to_pair, const lz_shape* shape,
                              void* xp, void* stream) {
  if (!lz::shape_ok(shape)) return LZ_ESHAPE;
  const long long P = (long long)shape->T * shape->k;
  if (P == 0) return LZ_OK;
  if (!x || !row_to_pair || !xp) return LZ_EINVAL;
  hipStream_t st = (hipStream_t)stream;
  const size_t row_bytes = (size_t)shape->d * lz::elem_bytes(shape->dtype);
  const unsigned blocks = unsigned((P + kRowsPerBlock - 1) / kRowsPerBlock);
  if (row_bytes % 16 == 0 && aligned16(x) && aligned16(xp)) {
    hipLaunchKernelGGL(permute_vec_kernel, dim3(blocks), dim3(256), 0, st, (const u32x4*)x, row_to_pair,
                       P, shape->k, int(row_bytes / 16), (u32x4*)xp);
  } else if (shape->dtype == LZ_F32) {
    hipLaunchKernelGGL(permute_elem_kernel<float>, dim3(blocks), dim3(256), 0, st, (const float*)x,
                       row_to_pair, P, shape->k, shape->d, (float*)xp);
  } else {
    hipLaunchKernelGGL(permute_elem_kernel<uint16_t>, dim3(blocks), dim3(256), 0, st,
                       (const uint16_t*)x, row_to_pair, P, shape->k, shape->d, (uint16_t*)xp);
  }
  return lz::launch_status();
}

extern "C" int32_t lz_permute_scatter(const void* x, const int32_t* pair_to_row, const lz_shape* shape,
                                      void* xp, void* stream) {
  if (!lz::shape_ok(shape)) return LZ_ESHAPE;
  const long long P = (long long)shape->T * shape->k;
  if (P == 0) return LZ_OK;
  if (!x || !pair_to_row || !xp) return LZ_EINVAL;
  hipStream_t st = (hipStream_t)stream;
  const size_t row_bytes = (size_t)shape->d * lz::elem_bytes(shape->dtype);
  const unsigned blocks = unsigned((shape->T + kRowsPerBlock - 1) / kRowsPerBlock);
  if (row_bytes % 16 == 0 && aligned16(x) && aligned16(xp)) {
    hipLaunchKernelGGL(permute_scatter_kernel<4>, dim3(blocks), dim3(256), 0, st, (const u32x4*)x, pair_to_row,
                       shape->T, shape->k, P, int(row_bytes / 16), (u32x4*)xp);
  } else if (shape->dtype == LZ_F32) {
    hipLaunchKernelGGL(permute_scatter_elem_kernel<float>, dim3(blocks), dim3(256), 0, st, (const float*)x,
                       pair_to_row, shape->T, shape->k, P, shape->d, (float*)xp);
  } else {
    hipLaunchKernelGGL(permute_scatter_elem_kernel<uint16_t>, dim3(blocks), dim3(256), 0, st,
                       (const uint16_t*)x, pair_to_row, shape->T, shape->k, P, shape->d, (uint16_t*)xp);
  }
  return lz::launch_status();
}

namespace {

int32_t combine(const void* yp, const int32_t* pair_to_row, const float* topk_gates, const lz_shape* shape,
                void* y, void* stream) {
  hipStream_t st = (hipStream_t)stream;
  const long long P = (long long)shape->T * shape->k;
  const unsigned blocks = unsigned((shape->T + kRowsPerBlock - 1) / kRowsPerBlock);
  if (shape->dtype == LZ_BF16 && shape->d % 8 == 0 && aligned16(yp) && aligned16(y)) {
    const u32x4* src = (const u32x4*)yp;
    u32x4* dst = (u32x4*)y;
    const int T = shape->T, vec = shape->d / 8;
    // lane-vectors of a row loaded ahead: 4 (measured: 5.7 TB/s against 5.2 with one; 8 is no
    // faster), fewer only for rows shorter than that
    const int ahead = vec >= 4 * lz::kWave ? 4 : (vec >= 2 * lz::kWave ? 2 : 1);
#define LZ_COMBINE_U(K, U)                                                                                    \
  hipLaunchKernelGGL((combine_bf16_kernel<K, U>), dim3(blocks), dim3(256), 0, st, src, pair_to_row, topk_gates, \
                     T, P, vec, dst)
#define LZ_COMBINE(K)                       \
  case K:                                   \
    if (ahead == 4) LZ_COMBINE_U(K, 4);     \
    else if (ahead == 2) LZ_COMBINE_U(K, 2); \
    else LZ_COMBINE_U(K, 1);                \
    break
    switch (shape->k) {  // 1 <= k <= kMaxK = 8, checked by shape_ok
      LZ_COMBINE(1);
      LZ_COMBINE(2);
      LZ_COMBINE(3);
      LZ_COMBINE(4);
      LZ_COMBINE(5);
      LZ_COMBINE(6);
      LZ_COMBINE(7);
      LZ_COMBINE(8);
      default: return LZ_ESHAPE;
    }
#undef LZ_COMBINE
#undef LZ_COMBINE_U
  } else if (shape->dtype == LZ_BF16) {
    hipLaunchKernelGGL(combine_elem_kernel<true>, dim3(blocks), dim3(256), 0, st, yp, pair_to_row,
                       topk_gates, shape->T, shape->k, P, shape->d, y);
  } else {
    hipLaunchKernelGGL(combine_elem_kernel<false>, dim3(blocks), dim3(256), 0, st, yp, pair_to_row,
                       topk_gates, shape->T, shape->k, P, shape->d, y);
  }
  return lz::launch_status();
}

}  // namespace

extern "C" int32_t lz_unpermute_combine(const void* yp, const int32_t* pair_to_row,
                                        const float* topk_gates, const lz_shape* shape, void* y,
                                        void* stream) {
  if (!lz::shape_ok(shape)) return LZ_ESHAPE;
  if (shape->T == 0) return LZ_OK;
  if (!yp || !pair_to_row || !topk_gates || !y) return LZ_EINVAL;
  return combine(yp, pair_to_row, topk_gates, shape, y, stream);
}

extern "C" int32_t lz_permute_backward(const void* dxp, const int32_t* pair_to_row, const lz_shape* shape,
                                       void* dx, void* stream) {
  if (!lz::shape_ok(shape)) return LZ_ESHAPE;
  if (shape->T == 0) return LZ_OK;
  if (!dxp || !pair_to_row || !dx) return LZ_EINVAL;
  return combine(dxp, pair_to_row, nullptr, shape, dx, stream);
}
