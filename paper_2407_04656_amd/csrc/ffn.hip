// Expert FFN as a grouped GEMM over the per-slot row ranges (Sec. 2.1: experts are
// parallel FFNs; every replica processes the rows dispatched to its slot).
//
//   GEMM-1   hidden[P, ffn] = act(xp[P, d] * W1[slot])        act = GELU | SwiGLU, fused;  W1[slot] = [d, n1]
//   GEMM-2   yp[P, d]       = hidden[P, ffn] * W2[slot]                                        W2[slot] = [ffn, d]
//
// Group sizes are data dependent and only known on the device, so a one-workgroup kernel
// first turns slot_offsets into a table of row tiles (slot, first row, end row) and, for the
// MFMA path, into one queue of work units per XCD.
//
// bf16 path: the MFMA kernel of gemm_mfma.h.
//
// Generic path (fp32 tensors, or bf16 shapes the MFMA tiling does not divide): a plain
// 64x64x16 LDS-tiled kernel with fp32 FMA accumulation and full bounds checks.
#include "gemm_mfma.h"

namespace {

__device__ __forceinline__ float gelu_exact(float v) {
  return 0.5f * v * (1.0f + erff(v * 0.70710678118654752440f));
}
__device__ __forceinline__ float silu(float v) { return v / (1.0f + expf(-v)); }

// ------------------------------------------------------------------------------------------
// generic tiled kernel
// ------------------------------------------------------------------------------------------
template <typename Elem>
__device__ __forceinline__ float load_elem(const Elem* p);
template <>
__device__ __forceinline__ float load_elem<float>(const float* p) { return *p; }
template <>
__device__ __forceinline__ float load_elem<uint16_t>(const uint16_t* p) { return lz::bf16_to_f32(*p); }
template <typename Elem>
__device__ __forceinline__ void store_elem(Elem* p, float v);
template <>
__device__ __forceinline__ void store_elem<float>(float* p, float v) { *p = v; }
template <>
__device__ __forceinline__ void store_elem<uint16_t>(uint16_t* p, float v) { *p = lz::f32_to_bf16(v); }

// C[rows of the tile, n] = epi( sum_k A[row, k] * W[slot][k, n (+ up_col0)] ),  W[slot] = [K, ldw].
// With a row map (gather != nullptr) row r of the left operand is row gather[r] / gather_k of A,
// zero if the map holds no pair for it.
template <typename Elem, int EPI>
__global__ __launch_bounds__(256) void gemm_generic_kernel(const Elem* __restrict__ A, int K,
                                                           const Elem* __restrict__ W, int ldw, int n_out,
                                                           int up_col0, Elem* __restrict__ C, TileTable t,
                                                           const int32_t* __restrict__ gather, int gather_k,
                                                           long long gather_T) {
  constexpr int BM = 64, BN = 64, BK = 16;
  constexpr bool DUAL = EPI == EPI_SWIGLU;
  __shared__ float sA[BK][BM + 1];
  __shared__ float sB[DUAL ? 2 : 1][BK][BN + 1];
  const int tile = blockIdx.y;
  if (tile >= t.header[0]) return;
  const int slot = t.slot[tile], row0 = t.row0[tile], row_end = t.row_end[tile];
  if (slot < 0) return;
  const int n0 = blockIdx.x * BN;
  const Elem* Ws = W + (size_t)slot * K * ldw;
  const int tx = threadIdx.x % 16, ty = threadIdx.x / 16;
  float acc[4][4] = {}, acc_up[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += BK) {
    for (int i = threadIdx.x; i < BM * BK; i += 256) {
      const int r = i / BK, kk = i % BK;
      const int row = row0 + r;
      long long src = row;
      bool ok = row < row_end && k0 + kk < K;
      if (gather && ok) {
        const long long pair = gather[row];
        ok = pair >= 0 && pair < gather_T * gather_k;
        src = ok ? pair / gather_k : 0;
      }
      sA[kk][r] = ok ? load_elem<Elem>(A + (size_t)src * K + k0 + kk) : 0.f;
    }
    for (int i = threadIdx.x; i < BN * BK; i += 256) {
      const int c = i % BN, kk = i / BN;  // consecutive threads read consecutive columns of a weight row
      const int n = n0 + c;
      const bool ok = n < n_out && k0 + kk < K;
      sB[0][kk][c] = ok ? load_elem<Elem>(Ws + (size_t)(k0 + kk) * ldw + n) : 0.f;
      if (DUAL) sB[DUAL ? 1 : 0][kk][c] = ok ? load_elem<Elem>(Ws + (size_t)(k0 + kk) * ldw + up_col0 + n) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < BK; ++kk) {
      float a[4], b[4], bu[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        a[i] = sA[kk][ty * 4 + i];
        b[i] = sB[0][kk][tx * 4 + i];
        bu[i] = DUAL ? sB[DUAL ? 1 : 0][kk][tx * 4 + i] : 0.f;
      }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
          if (DUAL) acc_up[i][j] = fmaf(a[i], bu[j], acc_up[i][j]);
        }
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
      if (n >= n_out) continue;
      float v = acc[i][j];
      if (EPI == EPI_GELU) v = gelu_exact(v);
      if (EPI == EPI_SWIGLU) v = silu(v) * acc_up[i][j];
      store_elem<Elem>(C + (size_t)row * n_out + n, v);
    }
  }
}

inline bool mfma_shape(const lz_shape* s) {
  if (s->dtype != LZ_BF16) return false;
  if (s->d % BN != 0 || s->ffn % 64 != 0) return false;
  // one slot's weights and one 256-row activation tile are addressed with 32-bit byte offsets
  if ((long long)s->d * s->ffn * 4 >= (1ll << 31)) return false;
  return s->ffn % (s->act == LZ_SWIGLU ? BN / 2 : BN) == 0;
}

struct FfnWorkspace {
  void* hidden;
  void* tiles;
  size_t total_bytes;
  int BMrows;
  int group;
  int n_up, n_down;  // column tiles of the two MFMA GEMMs (0 on the generic path)
};

TileTable tiles_of(const FfnWorkspace& w, const lz_shape* s) {
  return carve_tiles(w.tiles, (long long)s->T * s->k, s->N * s->c, w.BMrows, w.group, w.n_up, w.n_down);
}

FfnWorkspace carve_ffn(void* ws, const lz_shape* s) {
  FfnWorkspace w;
  const long long P = (long long)s->T * s->k;
  w.BMrows = mfma_shape(s) ? BM : 64;
  const size_t hidden_bytes = lz::align256((size_t)P * s->ffn * lz::elem_bytes(s->dtype));
  w.hidden = ws;
  w.tiles = (char*)ws + hidden_bytes;
  w.group = mfma_shape(s) ? kGroupM : 1;
  w.n_up = mfma_shape(s) ? s->ffn / (s->act == LZ_SWIGLU ? BN / 2 : BN) : 0;
  w.n_down = mfma_shape(s) ? s->d / BN : 0;
  w.total_bytes = hidden_bytes + tile_table_bytes(P, s->N * s->c, w.BMrows, w.group, w.n_up, w.n_down);
  return w;
}

}  // namespace

extern "C" size_t lz_ffn_workspace_bytes(const lz_shape* shape) {
  if (!lz::shape_ok(shape)) return 0;
  return carve_ffn(nullptr, shape).total_bytes;
}

namespace {

int32_t check_ffn(const lz_shape* shape, void* ws, size_t ws_bytes, FfnWorkspace* w) {
  if (!lz::shape_ok(shape)) return LZ_ESHAPE;
  *w = carve_ffn(ws, shape);
  if (!ws || (uintptr_t)ws % 256 != 0 || ws_bytes < w->total_bytes) return LZ_EWORKSPACE;
  return LZ_OK;
}

}  // namespace

extern "C" int32_t lz_ffn_tiles(const int32_t* slot_offsets, const lz_shape* shape, void* ws,
                                size_t ws_bytes, void* stream) {
  FfnWorkspace w;
  const int32_t rc = check_ffn(shape, ws, ws_bytes, &w);
  if (rc != LZ_OK) return rc;
  const long long P = (long long)shape->T * shape->k;
  if (P == 0) return LZ_OK;
  if (!slot_offsets) return LZ_EINVAL;
  const int S = shape->N * shape->c;
  TileTable t = tiles_of(w, shape);
  hipLaunchKernelGGL(build_tiles_kernel, dim3(1), dim3(256), 0, (hipStream_t)stream, slot_offsets, S, P,
                     w.BMrows, w.group, w.n_up, w.n_down, t);
  return lz::launch_status();
}

namespace {

// hidden = act(A W1) per slot; A = xp, or x read through the row map when `gather` is given
int32_t ffn_up(const void* xp, const int32_t* gather, const void* w1, const lz_shape* shape, void* ws,
               size_t ws_bytes, void* stream) {
  FfnWorkspace w;
  const int32_t rc = check_ffn(shape, ws, ws_bytes, &w);
  if (rc != LZ_OK) return rc;
  const long long P = (long long)shape->T * shape->k;
  if (P == 0) return LZ_OK;
  if (!xp || !w1) return LZ_EINVAL;
  hipStream_t st = (hipStream_t)stream;
  TileTable t = tiles_of(w, shape);
  const bool swiglu = shape->act == LZ_SWIGLU;
  const int n1 = shape->ffn * (swiglu ? 2 : 1);
  const int gk = shape->k;
  const long long gT = shape->T;
  if (!mfma_shape(shape)) {
    const dim3 grid((shape->ffn + 63) / 64, t.capacity);
    if (shape->dtype == LZ_F32) {
      if (swiglu)
        hipLaunchKernelGGL((gemm_generic_kernel<float, EPI_SWIGLU>), grid, dim3(256), 0, st, (const float*)xp,
                           shape->d, (const float*)w1, n1, shape->ffn, shape->ffn, (float*)w.hidden, t, gather,
                           gk, gT);
      else
        hipLaunchKernelGGL((gemm_generic_kernel<float, EPI_GELU>), grid, dim3(256), 0, st, (const float*)xp,
                           shape->d, (const float*)w1, n1, shape->ffn, 0, (float*)w.hidden, t, gather, gk, gT);
    } else {
      if (swiglu)
        hipLaunchKernelGGL((gemm_generic_kernel<uint16_t, EPI_SWIGLU>), grid, dim3(256), 0, st,
                           (const uint16_t*)xp, shape->d, (const uint16_t*)w1, n1, shape->ffn, shape->ffn,
                           (uint16_t*)w.hidden, t, gather, gk, gT);
      else
        hipLaunchKernelGGL((gemm_generic_kernel<uint16_t, EPI_GELU>), grid, dim3(256), 0, st,
                           (const uint16_t*)xp, shape->d, (const uint16_t*)w1, n1, shape->ffn, 0,
                           (uint16_t*)w.hidden, t, gather, gk, gT);
    }
    return lz::launch_status();
  }
  if ((uintptr_t)xp % 16 != 0 || (uintptr_t)w1 % 16 != 0) return LZ_EINVAL;  // 16-byte loads per lane
  // the MFMA gather addresses all of x with 32-bit byte offsets
  if (gather && (unsigned long long)shape->T * shape->d * 2ull >= (1ull << 32)) return LZ_ESHAPE;
  MfmaArgs g1{};
  g1.A = (const uint16_t*)xp;
  g1.W = (const uint16_t*)w1;
  g1.C = (uint16_t*)w.hidden;
  g1.P = P;
  g1.K = shape->d;
  g1.w_rows = n1;
  g1.n_out = shape->ffn;
  g1.up_row0 = swiglu ? shape->ffn : 0;
  g1.n_tiles = w.n_up;
  g1.which = 0;
  g1.t = t;
  g1.ldw = n1;
  g1.gather = gather;
  g1.gather_k = gk;
  g1.gather_T = gT;
  if (gather)
    return swiglu ? launch_mfma<EPI_SWIGLU, MODE_NN, true>(g1, st) : launch_mfma<EPI_GELU, MODE_NN, true>(g1, st);
  return swiglu ? launch_mfma<EPI_SWIGLU, MODE_NN>(g1, st) : launch_mfma<EPI_GELU, MODE_NN>(g1, st);
}

}  // namespace

extern "C" int32_t lz_ffn_up(const void* xp, const void* w1, const lz_shape* shape, void* ws,
                             size_t ws_bytes, void* stream) {
  return ffn_up(xp, nullptr, w1, shape, ws, ws_bytes, stream);
}

extern "C" int32_t lz_ffn_up_gather(const void* x, const int32_t* row_to_pair, const void* w1,
                                    const lz_shape* shape, void* ws, size_t ws_bytes, void* stream) {
  if (!row_to_pair && shape && (long long)shape->T * shape->k > 0) return LZ_EINVAL;
  return ffn_up(x, row_to_pair, w1, shape, ws, ws_bytes, stream);
}

extern "C" int32_t lz_ffn_down(const void* w2, const lz_shape* shape, void* yp, void* ws,
                               size_t ws_bytes, void* stream) {
  FfnWorkspace w;
  const int32_t rc = check_ffn(shape, ws, ws_bytes, &w);
  if (rc != LZ_OK) return rc;
  const long long P = (long long)shape->T * shape->k;
  if (P == 0) return LZ_OK;
  if (!w2 || !yp) return LZ_EINVAL;
  hipStream_t st = (hipStream_t)stream;
  TileTable t = tiles_of(w, shape);
  if (!mfma_shape(shape)) {
    const dim3 grid((shape->d + 63) / 64, t.capacity);
    if (shape->dtype == LZ_F32)
      hipLaunchKernelGGL((gemm_generic_kernel<float, EPI_NONE>), grid, dim3(256), 0, st,
                         (const float*)w.hidden, shape->ffn, (const float*)w2, shape->d, shape->d, 0,
                         (float*)yp, t, (const int32_t*)nullptr, 1, 0ll);
    else
      hipLaunchKernelGGL((gemm_generic_kernel<uint16_t, EPI_NONE>), grid, dim3(256), 0, st,
                         (const uint16_t*)w.hidden, shape->ffn, (const uint16_t*)w2, shape->d, shape->d, 0,
                         (uint16_t*)yp, t, (const int32_t*)nullptr, 1, 0ll);
    return lz::launch_status();
  }
  if ((uintptr_t)yp % 16 != 0 || (uintptr_t)w2 % 16 != 0) return LZ_EINVAL;  // 16-byte accesses per lane
  MfmaArgs g2{};
  g2.A = (const uint16_t*)w.hidden;
  g2.W = (const uint16_t*)w2;
  g2.C = (uint16_t*)yp;
  g2.P = P;
  g2.K = shape->ffn;
  g2.w_rows = shape->d;
  g2.n_out = shape->d;
  g2.up_row0 = 0;
  g2.n_tiles = w.n_down;
  g2.which = 1;
  g2.t = t;
  g2.ldw = shape->d;
  return launch_mfma<EPI_NONE, MODE_NN>(g2, st);
}

extern "C" int32_t lz_expert_ffn(const void* xp, const int32_t* slot_offsets, const void* w1,
                                 const void* w2, const lz_shape* shape, void* yp, void* ws,
                                 size_t ws_bytes, void* stream) {
  int32_t rc = lz_ffn_tiles(slot_offsets, shape, ws, ws_bytes, stream);
  if (rc != LZ_OK) return rc;
  const long long P = (long long)shape->T * shape->k;
  if (P == 0) return LZ_OK;
  if (!xp || !w1 || !w2 || !yp) return LZ_EINVAL;
  rc = lz_ffn_up(xp, w1, shape, ws, ws_bytes, stream);
  if (rc != LZ_OK) return rc;
  return lz_ffn_down(w2, shape, yp, ws, ws_bytes, stream);
}

extern "C" int32_t lz_expert_ffn_gather(const void* x, const int32_t* row_to_pair, const int32_t* slot_offsets,
                                        const void* w1, const void* w2, const lz_shape* shape, void* yp,
                                        void* ws, size_t ws_bytes, void* stream) {
  int32_t rc = lz_ffn_tiles(slot_offsets, shape, ws, ws_bytes, stream);
  if (rc != LZ_OK) return rc;
  const long long P = (long long)shape->T * shape->k;
  if (P == 0) return LZ_OK;
  if (!x || !row_to_pair || !w1 || !w2 || !yp) return LZ_EINVAL;
  rc = lz_ffn_up_gather(x, row_to_pair, w1, shape, ws, ws_bytes, stream);
  if (rc != LZ_OK) return rc;
  return lz_ffn_down(w2, shape, yp, ws, ws_bytes, stream);
}

// ------------------------------------------------------------------------------------------
// Diagnostic: which XCD does the hardware give the workgroups of a launch shaped like the
// persistent GEMM's (256 threads, the same dynamic LDS, hence one workgroup per CU)?
// ------------------------------------------------------------------------------------------
namespace {
__global__ __launch_bounds__(256, 1) void xcc_ids_kernel(int32_t* __restrict__ out) {
  extern __shared__ __attribute__((aligned(1024))) char smem_probe[];
  uint32_t id;
  asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(id));
  if (threadIdx.x == 0) out[blockIdx.x] = (int32_t)(id & 0xFu);
}
}  // namespace

extern "C" int32_t lz_debug_xcc_ids(int32_t* xcc_of_workgroup, int32_t n_workgroups, void* stream) {
  if (n_workgroups < 0 || n_workgroups > 65535) return LZ_EINVAL;
  if (n_workgroups == 0) return LZ_OK;
  if (!xcc_of_workgroup) return LZ_EINVAL;
  if (hipFuncSetAttribute((const void*)xcc_ids_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes) !=
      hipSuccess)
    return LZ_EHIP;
  hipLaunchKernelGGL(xcc_ids_kernel, dim3(n_workgroups), dim3(256), kLdsBytes, (hipStream_t)stream,
                     xcc_of_workgroup);
  return lz::launch_status();
}
