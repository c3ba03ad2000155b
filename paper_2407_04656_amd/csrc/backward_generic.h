// Training entry points for the shapes the MFMA kernels do not serve (fp32 tensors, bf16 shapes the
// MFMA tiling does not divide): the same chain-rule steps as backward.hip on plain LDS-tiled
// fp32-FMA kernels with full bounds checks.  fp32 accumulation, every stored tensor rounded once
// to the tensor type; the fp32 path uses erff / expf so that it meets the fp32 error bar.
// Device code, not part of the C ABI; included by backward.hip.
#pragma once
#include "gemm_mfma.h"

namespace {

template <typename Elem>
__device__ __forceinline__ float gload(const Elem* p);
template <>
__device__ __forceinline__ float gload<float>(const float* p) { return *p; }
template <>
__device__ __forceinline__ float gload<uint16_t>(const uint16_t* p) { return lz::bf16_to_f32(*p); }
template <typename Elem>
__device__ __forceinline__ void gstore(Elem* p, float v);
template <>
__device__ __forceinline__ void gstore<float>(float* p, float v) { *p = v; }
template <>
__device__ __forceinline__ void gstore<uint16_t>(uint16_t* p, float v) { *p = lz::f32_to_bf16(v); }
template <typename Elem>
__device__ __forceinline__ float ground(float v);  // the value that is stored
template <>
__device__ __forceinline__ float ground<float>(float v) { return v; }
template <>
__device__ __forceinline__ float ground<uint16_t>(float v) { return lz::bf16_to_f32(lz::f32_to_bf16(v)); }

// C[row, n] = sum_k A[row, k] * W[slot](n, k) over the 64-row tiles of the slot table, where element
// (n, k) of a slot's weights lies at W + slot * w_slot + n * ldn + k * ldk (either orientation).
template <typename Elem>
__global__ __launch_bounds__(256) void gemm_rows_generic_kernel(const Elem* __restrict__ A, int K,
                                                                const Elem* __restrict__ W, long long w_slot,
                                                                long long ldn, long long ldk, int n_out,
                                                                Elem* __restrict__ C, TileTable t) {
  constexpr int TM = 64, TN = 64, TK = 16;
  __shared__ float sA[TK][TM + 1];
  __shared__ float sB[TK][TN + 1];
  const int tile = blockIdx.y;
  if (tile >= t.header[0]) return;
  const int slot = t.slot[tile], row0 = t.row0[tile], row_end = t.row_end[tile];
  if (slot < 0) return;
  const int n0 = blockIdx.x * TN;
  const Elem* Ws = W + (size_t)slot * w_slot;
  const int tx = threadIdx.x % 16, ty = threadIdx.x / 16;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += TK) {
    for (int i = threadIdx.x; i < TM * TK; i += 256) {
      const int r = i / TK, kk = i % TK;
      const int row = row0 + r;
      sA[kk][r] = (row < row_end && k0 + kk < K) ? gload<Elem>(A + (size_t)row * K + k0 + kk) : 0.f;
    }
    for (int i = threadIdx.x; i < TN * TK; i += 256) {
      // consecutive threads along whichever of n, k is contiguous in memory
      const int c = ldn == 1 ? i % TN : i / TK, kk = ldn == 1 ? i / TN : i % TK;
      const int n = n0 + c;
      sB[kk][c] = (n < n_out && k0 + kk < K) ? gload<Elem>(Ws + (size_t)n * ldn + (size_t)(k0 + kk) * ldk) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < TK; ++kk) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        a[i] = sA[kk][ty * 4 + i];
        b[i] = sB[kk][tx * 4 + i];
      }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int row = row0 + ty * 4 + i;
    if (row >= row_end) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int n = n0 + tx * 4 + j;
      if (n < n_out) gstore<Elem>(C + (size_t)row * n_out + n, acc[i][j]);
    }
  }
}

// Weight gradient of one slot per blockIdx.z: C[s][m, n] = sum over the slot's rows r of
// A[r, m] * B[r, n]  (A [P, M], B [P, N], C [S, M, N]); an empty slot stores zeros.  With Cacc the
// sum is added to that fp32 matrix instead (an empty slot adds nothing).
template <typename Elem>
__global__ __launch_bounds__(256) void gemm_wgrad_generic_kernel(const Elem* __restrict__ A, int M,
                                                                 const Elem* __restrict__ B, int N,
                                                                 const int32_t* __restrict__ slot_offsets,
                                                                 long long P, Elem* __restrict__ C,
                                                                 float* __restrict__ Cacc) {
  constexpr int TM = 64, TN = 64, TK = 16;
  __shared__ float sA[TK][TM + 1];
  __shared__ float sB[TK][TN + 1];
  const int s = blockIdx.z;
  long long r_lo, r_hi;
  clip_slot(slot_offsets, s, P, &r_lo, &r_hi);
  const int m0 = blockIdx.y * TM, n0 = blockIdx.x * TN;
  const int tx = threadIdx.x % 16, ty = threadIdx.x / 16;
  float acc[4][4] = {};
  for (long long k0 = r_lo; k0 < r_hi; k0 += TK) {
    for (int i = threadIdx.x; i < TM * TK; i += 256) {
      const int m = i % TM, kk = i / TM;  // consecutive threads read consecutive columns of a row
      sA[kk][m] = (m0 + m < M && k0 + kk < r_hi) ? gload<Elem>(A + (size_t)(k0 + kk) * M + m0 + m) : 0.f;
    }
    for (int i = threadIdx.x; i < TN * TK; i += 256) {
      const int n = i % TN, kk = i / TN;
      sB[kk][n] = (n0 + n < N && k0 + kk < r_hi) ? gload<Elem>(B + (size_t)(k0 + kk) * N + n0 + n) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < TK; ++kk) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        a[i] = sA[kk][ty * 4 + i];
        b[i] = sB[kk][tx * 4 + i];
      }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int m = m0 + ty * 4 + i;
    if (m >= M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int n = n0 + tx * 4 + j;
      if (n >= N) continue;
      if (Cacc) Cacc[((size_t)s * M + m) * N + n] += acc[i][j];
      else gstore<Elem>(C + ((size_t)s * M + m) * N + n, acc[i][j]);
    }
  }
}

__device__ __forceinline__ float gelu_exact_f(float v) { return 0.5f * v * (1.0f + erff(v * 0.70710678118654752440f)); }
__device__ __forceinline__ float gelu_grad_exact_f(float v) {
  const float cdf = 0.5f * (1.0f + erff(v * 0.70710678118654752440f));
  return fmaf(v * 0.3989422804014327f, expf(-0.5f * v * v), cdf);
}
__device__ __forceinline__ float sigmoid_f(float v) { return 1.0f / (1.0f + expf(-v)); }

// h = act(z) on the stored (rounded) pre-activations; rows outside every slot are not touched
template <typename Elem, bool SWIGLU>
__global__ __launch_bounds__(256) void act_forward_generic_kernel(const Elem* __restrict__ Z, int ffn,
                                                                  Elem* __restrict__ H, TileTable t) {
  const int tile = blockIdx.y;
  if (tile >= t.header[0]) return;
  const int slot = t.slot[tile], row0 = t.row0[tile], row_end = t.row_end[tile];
  if (slot < 0) return;
  const int n1 = SWIGLU ? 2 * ffn : ffn;
  const int rows = row_end - row0 < 64 ? row_end - row0 : 64;
  for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < (long long)rows * ffn;
       i += (long long)gridDim.x * 256) {
    const long long row = row0 + i / ffn;
    const int f = int(i % ffn);
    const float g = gload<Elem>(Z + row * n1 + f);
    float out;
    if (SWIGLU) out = g * sigmoid_f(g) * gload<Elem>(Z + row * n1 + ffn + f);
    else out = gelu_exact_f(g);
    gstore<Elem>(H + row * ffn + f, out);
  }
}

// dZ = dH * act'(Z), all P rows
template <typename Elem, bool SWIGLU>
__global__ __launch_bounds__(256) void act_backward_generic_kernel(const Elem* __restrict__ dH,
                                                                   const Elem* __restrict__ Z, long long P, int ffn,
                                                                   Elem* __restrict__ dZ) {
  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  if (i >= P * ffn) return;
  const long long row = i / ffn;
  const int f = int(i % ffn);
  const int n1 = SWIGLU ? 2 * ffn : ffn;
  const float g = gload<Elem>(dH + i);
  const float a = gload<Elem>(Z + row * n1 + f);
  if (SWIGLU) {
    const float u = gload<Elem>(Z + row * n1 + ffn + f);
    const float sg = sigmoid_f(a);
    gstore<Elem>(dZ + row * n1 + f, g * u * (sg * fmaf(a, 1.0f - sg, 1.0f)));
    gstore<Elem>(dZ + row * n1 + ffn + f, g * (a * sg));
  } else {
    gstore<Elem>(dZ + row * n1 + f, g * gelu_grad_exact_f(a));
  }
}

// combine backward, one wave per token: dgates[t,kk] = <dy[t], yp[row]>, dyp[row] = gates[t,kk] dy[t]
template <typename Elem>
__global__ __launch_bounds__(256) void combine_backward_generic_kernel(const Elem* __restrict__ dy,
                                                                       const Elem* __restrict__ yp,
                                                                       const int32_t* __restrict__ pair_to_row,
                                                                       const float* __restrict__ gates, int T, int k,
                                                                       long long P, int d, Elem* __restrict__ dyp,
                                                                       float* __restrict__ dgates) {
  const int lane = threadIdx.x % lz::kWave;
  const long long t = (long long)blockIdx.x * 4 + threadIdx.x / lz::kWave;
  if (t >= T) return;
  for (int kk = 0; kk < k; ++kk) {
    const int r = pair_to_row[t * k + kk];
    float dot = 0.f;
    if (r >= 0 && r < P) {
      const float g = gates[t * k + kk];
      for (int v = lane; v < d; v += lz::kWave) {
        const float gy = gload<Elem>(dy + (size_t)t * d + v);
        dot = fmaf(gy, gload<Elem>(yp + (size_t)r * d + v), dot);
        gstore<Elem>(dyp + (size_t)r * d + v, g * gy);
      }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) dot += __shfl_xor(dot, off, 64);
    if (lane == 0) dgates[t * k + kk] = dot;
  }
}

// dW[e] = sum over the slots holding e, ascending slot, fp32 sum, one rounding
template <typename Elem>
__global__ __launch_bounds__(256) void reduce_replicas_generic_kernel(const Elem* __restrict__ dw_slot,
                                                                      const int32_t* __restrict__ slot_expert, int S,
                                                                      long long elems, Elem* __restrict__ dw) {
  const long long v = (long long)blockIdx.x * 256 + threadIdx.x;
  if (v >= elems) return;
  const int e = blockIdx.y;
  float acc = 0.f;
  for (int s = 0; s < S; ++s)
    if (slot_expert[s] == e) acc += gload<Elem>(dw_slot + (size_t)s * elems + v);
  gstore<Elem>(dw + (size_t)e * elems + v, acc);
}

// ---- workspace and drivers of the generic path
struct GenericTrainWorkspace {
  void* dh;     // [P, ffn]
  void* dz;     // [P, n1]
  void* tiles;  // 64-row tiles of the batch
  size_t total_bytes;
  int n1;
};

inline GenericTrainWorkspace carve_train_generic(void* ws, const lz_shape* s) {
  GenericTrainWorkspace w;
  const long long P = (long long)s->T * s->k;
  const size_t eb = lz::elem_bytes(s->dtype);
  w.n1 = s->ffn * (s->act == LZ_SWIGLU ? 2 : 1);
  char* p = (char*)ws;
  auto take = [&](size_t bytes) {
    char* r = p;
    p += lz::align256(bytes);
    return r;
  };
  w.dh = take((size_t)P * s->ffn * eb);
  w.dz = take((size_t)P * w.n1 * eb);
  w.tiles = take(tile_table_bytes(P, s->N * s->c, 64, 1, 0, 0));
  w.total_bytes = size_t(p - (char*)ws);
  return w;
}

template <typename Elem>
int32_t generic_forward_train(const void* xp, const int32_t* slot_offsets, const void* w1, const void* w2,
                              const lz_shape* s, void* z, void* h, void* yp, const GenericTrainWorkspace& w,
                              hipStream_t st) {
  const long long P = (long long)s->T * s->k;
  const int S = s->N * s->c, d = s->d, ffn = s->ffn, n1 = w.n1;
  TileTable t = carve_tiles(w.tiles, P, S, 64, 1, 0, 0);
  hipLaunchKernelGGL(build_tiles_kernel, dim3(1), dim3(256), 0, st, slot_offsets, S, P, 64, 1, 0, 0, t);
  // z = xp W1   (W1[s] = [d, n1]: element (n, k) at k * n1 + n)
  hipLaunchKernelGGL((gemm_rows_generic_kernel<Elem>), dim3((n1 + 63) / 64, t.capacity), dim3(256), 0, st,
                     (const Elem*)xp, d, (const Elem*)w1, (long long)d * n1, 1ll, (long long)n1, n1, (Elem*)z, t);
  const dim3 agrid(16, t.capacity);
  if (s->act == LZ_SWIGLU)
    hipLaunchKernelGGL((act_forward_generic_kernel<Elem, true>), agrid, dim3(256), 0, st, (const Elem*)z, ffn, (Elem*)h, t);
  else
    hipLaunchKernelGGL((act_forward_generic_kernel<Elem, false>), agrid, dim3(256), 0, st, (const Elem*)z, ffn, (Elem*)h, t);
  // yp = h W2   (W2[s] = [ffn, d]: element (n, k) at k * d + n)
  hipLaunchKernelGGL((gemm_rows_generic_kernel<Elem>), dim3((d + 63) / 64, t.capacity), dim3(256), 0, st,
                     (const Elem*)h, ffn, (const Elem*)w2, (long long)ffn * d, 1ll, (long long)d, d, (Elem*)yp, t);
  return lz::launch_status();
}

template <typename Elem>
int32_t generic_ffn_backward(const void* dyp, const void* xp, const void* z, const void* h,
                             const int32_t* slot_offsets, const void* w1, const void* w2, const lz_shape* s,
                             void* dxp, void* dw1, void* dw2, bool accumulate, const GenericTrainWorkspace& w,
                             hipStream_t st) {
  const long long P = (long long)s->T * s->k;
  const int S = s->N * s->c, d = s->d, ffn = s->ffn, n1 = w.n1;
  if (P > 0) {
    TileTable t = carve_tiles(w.tiles, P, S, 64, 1, 0, 0);
    hipLaunchKernelGGL(build_tiles_kernel, dim3(1), dim3(256), 0, st, slot_offsets, S, P, 64, 1, 0, 0, t);
    // dH = dyp W2^T   (element (n = f, k = j) of W2[s] at f * d + j)
    hipLaunchKernelGGL((gemm_rows_generic_kernel<Elem>), dim3((ffn + 63) / 64, t.capacity), dim3(256), 0, st,
                       (const Elem*)dyp, d, (const Elem*)w2, (long long)ffn * d, (long long)d, 1ll, ffn, (Elem*)w.dh, t);
    const unsigned blocks = (unsigned)((P * ffn + 255) / 256);
    if (s->act == LZ_SWIGLU)
      hipLaunchKernelGGL((act_backward_generic_kernel<Elem, true>), dim3(blocks), dim3(256), 0, st,
                         (const Elem*)w.dh, (const Elem*)z, P, ffn, (Elem*)w.dz);
    else
      hipLaunchKernelGGL((act_backward_generic_kernel<Elem, false>), dim3(blocks), dim3(256), 0, st,
                         (const Elem*)w.dh, (const Elem*)z, P, ffn, (Elem*)w.dz);
    // dxp = dZ W1^T   (element (n = i, k = c) of W1[s] at i * n1 + c)
    hipLaunchKernelGGL((gemm_rows_generic_kernel<Elem>), dim3((d + 63) / 64, t.capacity), dim3(256), 0, st,
                       (const Elem*)w.dz, n1, (const Elem*)w1, (long long)d * n1, (long long)n1, 1ll, d, (Elem*)dxp, t);
  }
  // dW2[s] = H_s^T dyp_s  [ffn, d],   dW1[s] = xp_s^T dZ_s  [d, n1]
  hipLaunchKernelGGL((gemm_wgrad_generic_kernel<Elem>), dim3((d + 63) / 64, (ffn + 63) / 64, S), dim3(256), 0, st,
                     (const Elem*)h, ffn, (const Elem*)dyp, d, slot_offsets, P, accumulate ? nullptr : (Elem*)dw2,
                     accumulate ? (float*)dw2 : nullptr);
  hipLaunchKernelGGL((gemm_wgrad_generic_kernel<Elem>), dim3((n1 + 63) / 64, (d + 63) / 64, S), dim3(256), 0, st,
                     (const Elem*)xp, d, (const Elem*)w.dz, n1, slot_offsets, P, accumulate ? nullptr : (Elem*)dw1,
                     accumulate ? (float*)dw1 : nullptr);
  return lz::launch_status();
}

}  // namespace
