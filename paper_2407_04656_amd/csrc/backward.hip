// Backward pass of the MoE layer: the chain rule applied to the forward of Sec. 2.1, step by
// step in reverse (the paper trains the layer and all-reduces each expert's gradient over its
// replicas, Sec. 5, but prints no backward formulas).
//
//   combine      dgates[t,kk] = <dy[t], yp[row]>,  dyp[row] = gates[t,kk] dy[t]      HBM streaming
//   GEMM-2       dH = dyp W2^T          (dgrad)    dW2[s] = H_s^T dyp_s   (wgrad)     MFMA   W2[s] = [ffn, d]
//   activation   dZ = dH * act'(Z)                                                  HBM streaming
//   GEMM-1       dxp = dZ W1^T          (dgrad)    dW1[s] = xp_s^T dZ_s   (wgrad)     MFMA   W1[s] = [d, n1]
//   permute      dx[t] = sum_kk dxp[row(t,kk)]                                      HBM streaming
//   gate         dlogits = softmax backward on the k selected logits
//   replicas     dW[e] = sum over the slots that hold e                             HBM streaming
//
// Every contraction runs on the forward's grouped MFMA kernel in one of its three operand
// modes.  The weights are stored input-major ([d, n1] and [ffn, d]: the forward contracts over
// their rows), so the data gradients contract along their rows' direction (both operands
// k-contiguous) and the weight gradients over a slot's rows of two activation matrices (both
// operands k-major, a different length for every slot).  k-major tiles stream into LDS as they
// lie in memory and are transposed on the way to the registers (gfx950's transposing LDS
// reads): no transposed copy of weights or activations is ever written.  The weight gradients
// run over S x (rows of the weight matrix) virtual rows; each tile takes its contraction range
// from slot_offsets.
#include "backward_generic.h"
#include "gemm_mfma.h"

namespace {

constexpr int kRowsPerBlock = 4;  // streaming kernels: one wave per row
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

__device__ __forceinline__ void unpack8(const u32x4& v, float* f) {
  const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    f[2 * q] = __uint_as_float(w[q] << 16);
    f[2 * q + 1] = __uint_as_float(w[q] & 0xFFFF0000u);
  }
}

__device__ __forceinline__ u32x4 pack8(const float* f) {
  u32x4 o;
  o.x = pack_bf16x2(f[0], f[1]);
  o.y = pack_bf16x2(f[2], f[3]);
  o.z = pack_bf16x2(f[4], f[5]);
  o.w = pack_bf16x2(f[6], f[7]);
  return o;
}

// ---- combine backward: one wave per token.  dy[t] is read once, every yp row once, every
// dyp row written once; the k dot products are reduced over the wave at the end.
__global__ __launch_bounds__(256) void combine_backward_kernel(const u32x4* __restrict__ dy,
                                                               const u32x4* __restrict__ yp,
                                                               const int32_t* __restrict__ pair_to_row,
                                                               const float* __restrict__ gates, int T, int k,
                                                               long long P, int vec_per_row,
                                                               u32x4* __restrict__ dyp,
                                                               float* __restrict__ dgates) {
  const int lane = threadIdx.x % lz::kWave;
  const long long t = (long long)blockIdx.x * kRowsPerBlock + threadIdx.x / lz::kWave;
  if (t >= T) return;
  long long rows[lz::kMaxK];
  float g[lz::kMaxK], dot[lz::kMaxK];
#pragma unroll
  for (int kk = 0; kk < lz::kMaxK; ++kk) {
    rows[kk] = -1;
    g[kk] = 0.f;
    dot[kk] = 0.f;
    if (kk < k) {
      const int r = pair_to_row[t * k + kk];
      rows[kk] = (r >= 0 && r < P) ? r : -1;
      g[kk] = gates[t * k + kk];
    }
  }
  for (int v = lane; v < vec_per_row; v += lz::kWave) {
    float gy[8];
    unpack8(__builtin_nontemporal_load(dy + (size_t)t * vec_per_row + v), gy);
    u32x4 in[lz::kMaxK];
#pragma unroll
    for (int kk = 0; kk < lz::kMaxK; ++kk)
      if (kk < k && rows[kk] >= 0) in[kk] = __builtin_nontemporal_load(yp + (size_t)rows[kk] * vec_per_row + v);
#pragma unroll
    for (int kk = 0; kk < lz::kMaxK; ++kk)
      if (kk < k && rows[kk] >= 0) {
        float y8[8], o[8];
        unpack8(in[kk], y8);
#pragma unroll
        for (int q = 0; q < 8; ++q) {
          dot[kk] = fmaf(gy[q], y8[q], dot[kk]);
          o[q] = g[kk] * gy[q];
        }
        __builtin_nontemporal_store(pack8(o), dyp + (size_t)rows[kk] * vec_per_row + v);
      }
  }
#pragma unroll
  for (int kk = 0; kk < lz::kMaxK; ++kk)
    if (kk < k) {
      const float s = wave_sum(dot[kk]);
      if (lane == 0) dgates[t * k + kk] = s;
    }
}

// ---- gate backward: thread per (token, expert)
__global__ __launch_bounds__(256) void route_backward_kernel(const float* __restrict__ dgates,
                                                             const float* __restrict__ gates,
                                                             const int32_t* __restrict__ ids, int T, int E, int k,
                                                             float* __restrict__ dlogits) {
  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  if (i >= (long long)T * E) return;
  const long long t = i / E;
  const int e = int(i % E);
  float inner = 0.f, mine_g = 0.f, mine_dg = 0.f;
  for (int kk = 0; kk < k; ++kk) {
    const float g = gates[t * k + kk], dg = dgates[t * k + kk];
    inner = fmaf(g, dg, inner);
    if (ids[t * k + kk] == e) {
      mine_g = g;
      mine_dg = dg;
    }
  }
  dlogits[i] = mine_g * (mine_dg - inner);  // an expert the token did not select has mine_g = 0
}

// ---- activations on stored pre-activations (bf16, 8 elements per lane)
__device__ __forceinline__ float sigmoid_fast(float v) {
  return __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.44269504088896341f * v));
}
// gelu'(v) = Phi(v) + v phi(v), Phi through the same rational erf as the forward
__device__ __forceinline__ float gelu_grad_fast(float v) {
  const float x = fabsf(v) * 0.70710678118654752440f;
  const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, x, 1.0f));
  float p = fmaf(1.061405429f, t, -1.453152027f);
  p = fmaf(p, t, 1.421413741f);
  p = fmaf(p, t, -0.284496736f);
  p = fmaf(p, t, 0.254829592f);
  const float e = __builtin_amdgcn_exp2f(-1.44269504088896341f * x * x);  // exp(-v^2/2)
  const float erf_abs = 1.0f - p * t * e;
  const float cdf = 0.5f + 0.5f * (v < 0.f ? -erf_abs : erf_abs);
  return fmaf(v * 0.3989422804014327f, e, cdf);
}

// dZ = dH * act'(Z)
template <bool SWIGLU>
__global__ __launch_bounds__(256) void act_backward_kernel(const u32x4* __restrict__ dH, const u32x4* __restrict__ Z,
                                                           long long P, int ffn_vec, u32x4* __restrict__ dZ) {
  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  if (i >= P * ffn_vec) return;
  const long long row = i / ffn_vec;
  const int v = int(i % ffn_vec);
  const int z_vec = SWIGLU ? 2 * ffn_vec : ffn_vec;
  float g[8], a[8];
  unpack8(__builtin_nontemporal_load(dH + i), g);
  unpack8(__builtin_nontemporal_load(Z + row * z_vec + v), a);
  if (SWIGLU) {
    float u[8], dg[8], du[8];
    unpack8(__builtin_nontemporal_load(Z + row * z_vec + ffn_vec + v), u);
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      const float s = sigmoid_fast(a[q]);
      dg[q] = g[q] * u[q] * (s * fmaf(a[q], 1.0f - s, 1.0f));
      du[q] = g[q] * (a[q] * s);
    }
    __builtin_nontemporal_store(pack8(dg), dZ + row * z_vec + v);
    __builtin_nontemporal_store(pack8(du), dZ + row * z_vec + ffn_vec + v);
  } else {
    float o[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) o[q] = g[q] * gelu_grad_fast(a[q]);
    __builtin_nontemporal_store(pack8(o), dZ + row * z_vec + v);
  }
}

// slot offsets of the S x rows_per_slot virtual rows of the two weight-gradient outputs
__global__ void virtual_rows_kernel(int S, int rows_w2, int rows_w1, int32_t* __restrict__ virt_w2,
                                    int32_t* __restrict__ virt_w1) {
  for (int s = threadIdx.x; s <= S; s += blockDim.x) {
    virt_w2[s] = s * rows_w2;
    virt_w1[s] = s * rows_w1;
  }
}

// dW[e] = sum over slots s with slot_expert[s] == e of dW_slot[s], ascending s, fp32 sum, one rounding
__global__ __launch_bounds__(256) void reduce_replicas_kernel(const u32x4* __restrict__ dw_slot,
                                                              const int32_t* __restrict__ slot_expert, int S,
                                                              long long vec_per_slot, u32x4* __restrict__ dw) {
  const long long v = (long long)blockIdx.x * 256 + threadIdx.x;
  if (v >= vec_per_slot) return;
  const int e = blockIdx.y;
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  for (int s = 0; s < S; ++s) {
    if (slot_expert[s] != e) continue;
    float f[8];
    unpack8(__builtin_nontemporal_load(dw_slot + (size_t)s * vec_per_slot + v), f);
#pragma unroll
    for (int q = 0; q < 8; ++q) acc[q] += f[q];
  }
  __builtin_nontemporal_store(pack8(acc), dw + (size_t)e * vec_per_slot + v);
}

inline bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }

// ---- workspace of the training entry points
struct TrainWorkspace {
  uint16_t* dh;        // [P, ffn]
  uint16_t* dz;        // [P, n1]
  int32_t* virt_w2;    // [S+1]
  int32_t* virt_w1;    // [S+1]
  void* tiles_fwd;     // rows of the batch: lists for the forward's two GEMMs (ffn / 128 or 256, d / 256 column tiles)
  void* tiles_bwd;     // rows of the batch: lists for ffn / 256 and d / 256 column tiles
  void* tiles_w2;      // S * ffn virtual rows, d / 256 column tiles
  void* tiles_w1;      // S * d virtual rows, n1 / 256 column tiles
  size_t total_bytes;
  int n1;
};

inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

TrainWorkspace carve_train(void* ws, const lz_shape* s) {
  TrainWorkspace w;
  const long long P = (long long)s->T * s->k;
  const int S = s->N * s->c;
  w.n1 = s->ffn * (s->act == LZ_SWIGLU ? 2 : 1);
  char* p = (char*)ws;
  auto take = [&](size_t bytes) {
    char* r = p;
    p += lz::align256(bytes);
    return r;
  };
  w.dh = (uint16_t*)take((size_t)P * s->ffn * 2);
  w.dz = (uint16_t*)take((size_t)P * w.n1 * 2);
  w.virt_w2 = (int32_t*)take(sizeof(int32_t) * (S + 1));
  w.virt_w1 = (int32_t*)take(sizeof(int32_t) * (S + 1));
  w.tiles_fwd = take(tile_table_bytes(P, S, BM, kGroupM, ceil_div(s->ffn, s->act == LZ_SWIGLU ? BN / 2 : BN), s->d / BN));
  w.tiles_bwd = take(tile_table_bytes(P, S, BM, kGroupM, ceil_div(s->ffn, BN), s->d / BN));
  w.tiles_w2 = take(tile_table_bytes((long long)S * s->ffn, S, BM, kGroupM, s->d / BN, 0));
  w.tiles_w1 = take(tile_table_bytes((long long)S * s->d, S, BM, kGroupM, ceil_div(w.n1, BN), 0));
  w.total_bytes = size_t(p - (char*)ws);
  return w;
}

// the shapes the MFMA kernel serves: bf16, d a multiple of 256, ffn of 64, a slot's weights within 32-bit offsets
inline bool train_shape(const lz_shape* s) {
  if (!lz::shape_ok(s) || s->dtype != LZ_BF16) return false;
  if (s->d % BN != 0 || s->ffn % 64 != 0) return false;
  if ((long long)s->d * s->ffn * 4 >= (1ll << 31)) return false;
  const long long S = (long long)s->N * s->c;
  return S * s->d * 2 < (1ll << 31) && S * s->ffn * 2 < (1ll << 31);  // virtual row indices are int32
}

int32_t check_train(const lz_shape* shape, void* ws, size_t ws_bytes, TrainWorkspace* w) {
  if (!train_shape(shape)) return LZ_ESHAPE;
  *w = carve_train(ws, shape);
  if (!ws || (uintptr_t)ws % 256 != 0 || ws_bytes < w->total_bytes) return LZ_EWORKSPACE;
  return LZ_OK;
}

int32_t build_table(const int32_t* offsets, int S, long long rows, int n_a, int n_b, void* mem, hipStream_t st,
                    TileTable* out) {
  *out = carve_tiles(mem, rows, S, BM, kGroupM, n_a, n_b);
  hipLaunchKernelGGL(build_tiles_kernel, dim3(1), dim3(256), 0, st, offsets, S, rows, BM, kGroupM, n_a, n_b, *out);
  return lz::launch_status();
}

// C[rows, n_out] = A[rows, K] W[slot][n_out, K]^T over the batch's ragged row ranges
int32_t gemm_nt(const uint16_t* A, const uint16_t* W, uint16_t* C, long long P, int K, int n_out, int which,
                  const TileTable& t, hipStream_t st) {
  MfmaArgs g{};
  g.A = A;
  g.W = W;
  g.C = C;
  g.P = P;
  g.K = K;
  g.w_rows = n_out;
  g.n_out = n_out;
  g.n_tiles = ceil_div(n_out, BN);
  g.which = which;
  g.t = t;
  return launch_mfma<EPI_NONE>(g, st);
}

// C[rows, n_out] = A[rows, K] W[slot][K, n_out] over the batch's ragged row ranges
int32_t gemm_nn(const uint16_t* A, const uint16_t* W, uint16_t* C, long long P, int K, int n_out, int which,
                   const TileTable& t, hipStream_t st) {
  MfmaArgs g{};
  g.A = A;
  g.W = W;
  g.C = C;
  g.P = P;
  g.K = K;
  g.w_rows = n_out;
  g.n_out = n_out;
  g.n_tiles = ceil_div(n_out, BN);
  g.which = which;
  g.t = t;
  g.ldw = n_out;
  return launch_mfma<EPI_NONE, MODE_NN>(g, st);
}

// dW[s] [rows_per_slot, n_out] = A[rows of s, :rows_per_slot]^T W[rows of s, :n_out], stored as bf16 in C,
// or, if Cacc is given, added to that fp32 matrix instead
int32_t gemm_wgrad(const uint16_t* A, const uint16_t* W, uint16_t* C, float* Cacc, int S, long long P,
                   int rows_per_slot, int n_out, const int32_t* slot_offsets, const TileTable& t, hipStream_t st) {
  MfmaArgs g{};
  g.A = A;
  g.W = W;
  g.C = C;
  g.Cacc = Cacc;
  g.P = (long long)S * rows_per_slot;
  g.w_rows = n_out;
  g.n_out = n_out;
  g.n_tiles = ceil_div(n_out, BN);
  g.which = 0;
  g.t = t;
  g.lda = rows_per_slot;
  g.ldw = n_out;
  g.slot_offsets = slot_offsets;
  g.k_rows = P;
  g.rows_per_slot = rows_per_slot;
  // 32-bit byte offsets do if no operand reaches 4 GiB, the K steps past a slot's end included
  const int ld_max = rows_per_slot > n_out ? rows_per_slot : n_out;
  const bool wide = ((unsigned long long)P + 4 * BK) * (unsigned)ld_max * 2ull > 0xFFFFFFFFull;
  if (wide) return Cacc ? launch_mfma<EPI_ACCUM, MODE_TN_WIDE>(g, st) : launch_mfma<EPI_NONE, MODE_TN_WIDE>(g, st);
  return Cacc ? launch_mfma<EPI_ACCUM, MODE_TN>(g, st) : launch_mfma<EPI_NONE, MODE_TN>(g, st);
}

// the generic path takes every valid shape whose 64-row tile count fits a grid dimension
inline bool generic_train_shape(const lz_shape* s) {
  if (!lz::shape_ok(s)) return false;
  return tile_capacity((long long)s->T * s->k, s->N * s->c, 64, 1) <= 65535;
}

int32_t check_train_generic(const lz_shape* shape, void* ws, size_t ws_bytes, GenericTrainWorkspace* w) {
  if (!generic_train_shape(shape)) return LZ_ESHAPE;
  *w = carve_train_generic(ws, shape);
  if (!ws || (uintptr_t)ws % 256 != 0 || ws_bytes < w->total_bytes) return LZ_EWORKSPACE;
  return LZ_OK;
}

}  // namespace

extern "C" size_t lz_train_workspace_bytes(const lz_shape* shape) {
  if (train_shape(shape)) return carve_train(nullptr, shape).total_bytes;
  if (generic_train_shape(shape)) return carve_train_generic(nullptr, shape).total_bytes;
  return 0;
}

extern "C" int32_t lz_ffn_forward_train(const void* xp, const int32_t* slot_offsets, const void* w1, const void* w2,
                                        const lz_shape* shape, void* z, void* h, void* yp, void* ws,
                                        size_t ws_bytes, void* stream) {
  if (!train_shape(shape)) {
    GenericTrainWorkspace gw;
    const int32_t grc = check_train_generic(shape, ws, ws_bytes, &gw);
    if (grc != LZ_OK) return grc;
    if ((long long)shape->T * shape->k == 0) return LZ_OK;
    if (!xp || !slot_offsets || !w1 || !w2 || !z || !h || !yp) return LZ_EINVAL;
    return shape->dtype == LZ_F32
               ? generic_forward_train<float>(xp, slot_offsets, w1, w2, shape, z, h, yp, gw, (hipStream_t)stream)
               : generic_forward_train<uint16_t>(xp, slot_offsets, w1, w2, shape, z, h, yp, gw, (hipStream_t)stream);
  }
  TrainWorkspace w;
  const int32_t rc = check_train(shape, ws, ws_bytes, &w);
  if (rc != LZ_OK) return rc;
  const long long P = (long long)shape->T * shape->k;
  if (P == 0) return LZ_OK;
  if (!xp || !slot_offsets || !w1 || !w2 || !z || !h || !yp) return LZ_EINVAL;
  if (!aligned16(z) || !aligned16(h) || !aligned16(yp) || !aligned16(xp) || !aligned16(w1) || !aligned16(w2))
    return LZ_EINVAL;
  hipStream_t st = (hipStream_t)stream;
  const int S = shape->N * shape->c;
  const bool swiglu = shape->act == LZ_SWIGLU;
  const int n_up = ceil_div(shape->ffn, swiglu ? BN / 2 : BN);
  TileTable t;
  int32_t r = build_table(slot_offsets, S, P, n_up, shape->d / BN, w.tiles_fwd, st, &t);
  if (r != LZ_OK) return r;
  // z = xp W1 and h = act(z) from one epilogue
  MfmaArgs g{};
  g.A = (const uint16_t*)xp;
  g.W = (const uint16_t*)w1;
  g.C = (uint16_t*)h;
  g.Z = (uint16_t*)z;
  g.z_cols = w.n1;
  g.P = P;
  g.K = shape->d;
  g.w_rows = w.n1;
  g.n_out = shape->ffn;
  g.up_row0 = swiglu ? shape->ffn : 0;
  g.n_tiles = n_up;
  g.which = 0;
  g.t = t;
  g.ldw = w.n1;
  r = swiglu ? launch_mfma<EPI_SWIGLU_KEEP, MODE_NN>(g, st) : launch_mfma<EPI_GELU_KEEP, MODE_NN>(g, st);
  if (r != LZ_OK) return r;
  return gemm_nn((const uint16_t*)h, (const uint16_t*)w2, (uint16_t*)yp, P, shape->ffn, shape->d, 1, t, st);
}

extern "C" int32_t lz_combine_backward(const void* dy, const void* yp, const int32_t* pair_to_row,
                                       const float* topk_gates, const lz_shape* shape, void* dyp, float* dgates,
                                       void* stream) {
  if (!lz::shape_ok(shape)) return LZ_ESHAPE;
  if (shape->T == 0) return LZ_OK;
  if (!dy || !yp || !pair_to_row || !topk_gates || !dyp || !dgates) return LZ_EINVAL;
  const long long P = (long long)shape->T * shape->k;
  const unsigned blocks = unsigned((shape->T + kRowsPerBlock - 1) / kRowsPerBlock);
  if (shape->dtype != LZ_BF16 || shape->d % 8 != 0 || !aligned16(dy) || !aligned16(yp) || !aligned16(dyp)) {
    // element-wise kernel: fp32 tensors, rows that are not a multiple of 16 bytes, unaligned buffers
    if (shape->dtype == LZ_F32)
      hipLaunchKernelGGL(combine_backward_generic_kernel<float>, dim3(blocks), dim3(256), 0, (hipStream_t)stream,
                         (const float*)dy, (const float*)yp, pair_to_row, topk_gates, shape->T, shape->k, P,
                         shape->d, (float*)dyp, dgates);
    else
      hipLaunchKernelGGL(combine_backward_generic_kernel<uint16_t>, dim3(blocks), dim3(256), 0, (hipStream_t)stream,
                         (const uint16_t*)dy, (const uint16_t*)yp, pair_to_row, topk_gates, shape->T, shape->k, P,
                         shape->d, (uint16_t*)dyp, dgates);
    return lz::launch_status();
  }
  hipLaunchKernelGGL(combine_backward_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream, (const u32x4*)dy,
                     (const u32x4*)yp, pair_to_row, topk_gates, shape->T, shape->k, P, shape->d / 8, (u32x4*)dyp,
                     dgates);
  return lz::launch_status();
}

extern "C" int32_t lz_route_backward(const float* dgates, const float* topk_gates, const int32_t* topk_ids,
                                     const lz_shape* shape, float* dlogits, void* stream) {
  if (!lz::shape_ok(shape)) return LZ_ESHAPE;
  if (shape->T == 0) return LZ_OK;
  if (!dgates || !topk_gates || !topk_ids || !dlogits) return LZ_EINVAL;
  const long long n = (long long)shape->T * shape->E;
  hipLaunchKernelGGL(route_backward_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, (hipStream_t)stream,
                     dgates, topk_gates, topk_ids, shape->T, shape->E, shape->k, dlogits);
  return lz::launch_status();
}

namespace {

// dw1 / dw2 are bf16 gradients (accumulate == false: overwritten) or fp32 sums (accumulate == true: added to)
int32_t ffn_backward(const void* dyp, const void* xp, const void* z, const void* h, const int32_t* slot_offsets,
                     const void* w1, const void* w2, const lz_shape* shape, void* dxp, void* dw1, void* dw2,
                     bool accumulate, void* ws, size_t ws_bytes, void* stream) {
  if (!train_shape(shape)) {
    GenericTrainWorkspace gw;
    const int32_t grc = check_train_generic(shape, ws, ws_bytes, &gw);
    if (grc != LZ_OK) return grc;
    if (!dw1 || !dw2 || !slot_offsets) return LZ_EINVAL;
    if ((long long)shape->T * shape->k > 0 && (!dyp || !xp || !z || !h || !w1 || !w2 || !dxp)) return LZ_EINVAL;
    return shape->dtype == LZ_F32
               ? generic_ffn_backward<float>(dyp, xp, z, h, slot_offsets, w1, w2, shape, dxp, dw1, dw2, accumulate,
                                             gw, (hipStream_t)stream)
               : generic_ffn_backward<uint16_t>(dyp, xp, z, h, slot_offsets, w1, w2, shape, dxp, dw1, dw2,
                                                accumulate, gw, (hipStream_t)stream);
  }
  TrainWorkspace w;
  const int32_t rc = check_train(shape, ws, ws_bytes, &w);
  if (rc != LZ_OK) return rc;
  const long long P = (long long)shape->T * shape->k;
  const int S = shape->N * shape->c;
  if (!dw1 || !dw2 || !slot_offsets) return LZ_EINVAL;
  if (!aligned16(dw1) || !aligned16(dw2)) return LZ_EINVAL;
  if (P > 0 && (!dyp || !xp || !z || !h || !w1 || !w2 || !dxp)) return LZ_EINVAL;
  if (P > 0 && (!aligned16(dyp) || !aligned16(xp) || !aligned16(z) || !aligned16(h) || !aligned16(dxp) ||
                !aligned16(w1) || !aligned16(w2)))
    return LZ_EINVAL;
  hipStream_t st = (hipStream_t)stream;
  const int d = shape->d, ffn = shape->ffn, n1 = w.n1;
  const bool swiglu = shape->act == LZ_SWIGLU;

  hipLaunchKernelGGL(virtual_rows_kernel, dim3(1), dim3(256), 0, st, S, ffn, d, w.virt_w2, w.virt_w1);
  int32_t r = lz::launch_status();
  if (r != LZ_OK) return r;
  TileTable t_rows, t_w2, t_w1;
  if ((r = build_table(slot_offsets, S, P, ceil_div(ffn, BN), d / BN, w.tiles_bwd, st, &t_rows)) != LZ_OK) return r;
  if ((r = build_table(w.virt_w2, S, (long long)S * ffn, d / BN, 0, w.tiles_w2, st, &t_w2)) != LZ_OK) return r;
  if ((r = build_table(w.virt_w1, S, (long long)S * d, ceil_div(n1, BN), 0, w.tiles_w1, st, &t_w1)) != LZ_OK) return r;

  if (P > 0) {
    // dH = dyp W2^T    (W2 [ffn, d]: contraction along its rows)
    if ((r = gemm_nt((const uint16_t*)dyp, (const uint16_t*)w2, w.dh, P, d, ffn, 0, t_rows, st)) != LZ_OK) return r;
    // dZ = dH * act'(Z)
    const int ffn_vec = ffn / 8;
    const unsigned blocks = (unsigned)((P * ffn_vec + 255) / 256);
    if (swiglu)
      hipLaunchKernelGGL(act_backward_kernel<true>, dim3(blocks), dim3(256), 0, st, (const u32x4*)w.dh,
                         (const u32x4*)z, P, ffn_vec, (u32x4*)w.dz);
    else
      hipLaunchKernelGGL(act_backward_kernel<false>, dim3(blocks), dim3(256), 0, st, (const u32x4*)w.dh,
                         (const u32x4*)z, P, ffn_vec, (u32x4*)w.dz);
    if ((r = lz::launch_status()) != LZ_OK) return r;
    // dxp = dZ W1^T    (W1 [d, n1])
    if ((r = gemm_nt(w.dz, (const uint16_t*)w1, (uint16_t*)dxp, P, n1, d, 1, t_rows, st)) != LZ_OK) return r;
  }
  // dW2[s] = H_s^T dyp_s  [ffn, d],   dW1[s] = xp_s^T dZ_s  [d, n1]
  if ((r = gemm_wgrad((const uint16_t*)h, (const uint16_t*)dyp, accumulate ? nullptr : (uint16_t*)dw2,
                      accumulate ? (float*)dw2 : nullptr, S, P, ffn, d, slot_offsets, t_w2, st)) != LZ_OK)
    return r;
  return gemm_wgrad((const uint16_t*)xp, w.dz, accumulate ? nullptr : (uint16_t*)dw1,
                    accumulate ? (float*)dw1 : nullptr, S, P, d, n1, slot_offsets, t_w1, st);
}

}  // namespace

extern "C" int32_t lz_ffn_backward(const void* dyp, const void* xp, const void* z, const void* h,
                                   const int32_t* slot_offsets, const void* w1, const void* w2,
                                   const lz_shape* shape, void* dxp, void* dw1, void* dw2, void* ws,
                                   size_t ws_bytes, void* stream) {
  return ffn_backward(dyp, xp, z, h, slot_offsets, w1, w2, shape, dxp, dw1, dw2, false, ws, ws_bytes, stream);
}

extern "C" int32_t lz_ffn_backward_accumulate(const void* dyp, const void* xp, const void* z, const void* h,
                                              const int32_t* slot_offsets, const void* w1, const void* w2,
                                              const lz_shape* shape, void* dxp, float* dw1_acc, float* dw2_acc,
                                              void* ws, size_t ws_bytes, void* stream) {
  return ffn_backward(dyp, xp, z, h, slot_offsets, w1, w2, shape, dxp, dw1_acc, dw2_acc, true, ws, ws_bytes,
                      stream);
}

extern "C" int32_t lz_reduce_replica_grads(const void* dw_slot, const int32_t* slot_expert, int32_t S, int32_t E,
                                           int64_t elems_per_slot, void* dw, void* stream) {
  if (S < 1 || E < 1 || E > 65535 || elems_per_slot < 0 || elems_per_slot % 8 != 0) return LZ_ESHAPE;
  if (elems_per_slot == 0) return LZ_OK;
  if (!dw_slot || !slot_expert || !dw || !aligned16(dw_slot) || !aligned16(dw)) return LZ_EINVAL;
  const long long vec = elems_per_slot / 8;
  if ((vec + 255) / 256 > 0x7FFFFFFFll) return LZ_ESHAPE;
  hipLaunchKernelGGL(reduce_replicas_kernel, dim3((unsigned)((vec + 255) / 256), (unsigned)E), dim3(256), 0,
                     (hipStream_t)stream, (const u32x4*)dw_slot, slot_expert, S, vec, (u32x4*)dw);
  return lz::launch_status();
}

extern "C" int32_t lz_reduce_replica_grads_dtype(const void* dw_slot, const int32_t* slot_expert, int32_t S,
                                                 int32_t E, int64_t elems_per_slot, int32_t dtype, void* dw,
                                                 void* stream) {
  if (dtype != LZ_F32 && dtype != LZ_BF16) return LZ_ESHAPE;
  if (dtype == LZ_BF16 && elems_per_slot % 8 == 0 && aligned16(dw_slot) && aligned16(dw))
    return lz_reduce_replica_grads(dw_slot, slot_expert, S, E, elems_per_slot, dw, stream);
  if (S < 1 || E < 1 || E > 65535 || elems_per_slot < 0) return LZ_ESHAPE;
  if (elems_per_slot == 0) return LZ_OK;
  if (!dw_slot || !slot_expert || !dw) return LZ_EINVAL;
  if ((elems_per_slot + 255) / 256 > 0x7FFFFFFFll) return LZ_ESHAPE;
  const dim3 grid((unsigned)((elems_per_slot + 255) / 256), (unsigned)E);
  if (dtype == LZ_F32)
    hipLaunchKernelGGL(reduce_replicas_generic_kernel<float>, grid, dim3(256), 0, (hipStream_t)stream,
                       (const float*)dw_slot, slot_expert, S, (long long)elems_per_slot, (float*)dw);
  else
    hipLaunchKernelGGL(reduce_replicas_generic_kernel<uint16_t>, grid, dim3(256), 0, (hipStream_t)stream,
                       (const uint16_t*)dw_slot, slot_expert, S, (long long)elems_per_slot, (uint16_t*)dw);
  return lz::launch_status();
}
