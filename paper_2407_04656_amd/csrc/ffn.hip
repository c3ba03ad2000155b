// Expert FFN as a grouped GEMM over the per-slot row ranges (Sec. 2.1: experts are
// parallel FFNs; every replica processes the rows dispatched to its slot).
//
//   GEMM-1   hidden[P, ffn] = act(xp[P, d] * W1[slot]^T)      act = GELU | SwiGLU, fused
//   GEMM-2   yp[P, d]       = hidden[P, ffn] * W2[slot]^T
//
// Group sizes are data dependent and only known on the device, so a one-workgroup kernel
// first turns slot_offsets into a table of row tiles (slot, first row, end row) and, for the
// MFMA path, into one queue of work units per XCD.
//
// bf16 path (gfx950 MFMA): persistent kernel, one workgroup per CU, drawing 256x256 tiles from
// its XCD's queue.  4 waves in 2x2, each wave a 128x128 patch = 4x4
// v_mfma_f32_32x32x16_bf16 accumulators (fp32, 256 AGPRs).  Both operands are K-contiguous
// and are streamed HBM -> LDS with 16-byte buffer loads that write LDS directly, through two
// LDS stages of 64 K-columns; fragment reads are software pipelined over two register sets.
// The XOR swizzle that keeps the ds_read_b128 fragment reads conflict-free is applied on the
// global-address side because a direct-to-LDS load fixes the LDS side to lane order.  Buffer
// descriptors bound every load, so ragged tiles cannot fault.  The MFMA takes the weight
// fragment as its row operand, which leaves each lane with 4 consecutive output columns per
// accumulator group: 8-byte bf16 stores, no LDS transpose.  For SwiGLU the weight tile
// interleaves 32-row fragments of Wg and Wu, so the gate and up values of one output element
// sit in the same lane and register index.
//
// Generic path (fp32 tensors, or bf16 shapes the MFMA tiling does not divide): a plain
// 64x64x16 LDS-tiled kernel with fp32 FMA accumulation and full bounds checks.
#include "lz_common.h"

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

constexpr int kTileHeader = 64;  // ints before the tile arrays; [0] = number of row tiles
constexpr int kGroupM = 4;       // row tiles of a work unit (same slot)
constexpr int kGroupN = 8;       // column tiles of a work unit

enum { EPI_NONE = 0, EPI_GELU = 1, EPI_SWIGLU = 2 };

struct TileTable {
  int32_t* header;
  int32_t* slot;
  int32_t* row0;
  int32_t* row_end;
  int32_t* units[2];  // per GEMM (0 = up, 1 = down): 8 lists of unit_cap[g] work units, one list per XCD
  int unit_cap[2];
  int capacity;
};

constexpr int kUnitCount = 16;  // header[kUnitCount + 16*g + x] = length of XCD x's unit list for GEMM g

// Row tiles are listed slot after slot; with group > 1 every slot's list is padded (slot = -1)
// to a multiple of `group`, so that a group of consecutive row tiles never spans two slots.
inline int tile_capacity(long long P, int S, int BM, int group) {
  const long long n = (P + BM - 1) / BM + (long long)S * group;
  return int((n + group - 1) / group * group);
}

// Room in one XCD's list of work units (a unit = one row group x kGroupN column tiles): twice
// an eighth of the worst-case number of units, so that lists of equal cost but unequal length
// normally fit as they are.
inline int unit_capacity(int capacity, int group, int n_tiles) {
  if (n_tiles <= 0) return 0;
  const long long units = (long long)(capacity / group) * ((n_tiles + kGroupN - 1) / kGroupN);
  return int((units + 7) / 8 * 2);
}

inline size_t tile_table_bytes(long long P, int S, int BM, int group, int n_up, int n_down) {
  const int cap = tile_capacity(P, S, BM, group);
  const size_t ints = kTileHeader + 3 * (size_t)cap +
                      8 * ((size_t)unit_capacity(cap, group, n_up) + unit_capacity(cap, group, n_down));
  return lz::align256(sizeof(int32_t) * ints);
}

inline TileTable carve_tiles(void* base, long long P, int S, int BM, int group, int n_up, int n_down) {
  TileTable t;
  t.capacity = tile_capacity(P, S, BM, group);
  t.header = (int32_t*)base;
  t.slot = t.header + kTileHeader;
  t.row0 = t.slot + t.capacity;
  t.row_end = t.row0 + t.capacity;
  t.unit_cap[0] = unit_capacity(t.capacity, group, n_up);
  t.unit_cap[1] = unit_capacity(t.capacity, group, n_down);
  t.units[0] = t.row_end + t.capacity;
  t.units[1] = t.units[0] + 8 * (size_t)t.unit_cap[0];
  return t;
}

__device__ __forceinline__ void clip_slot(const int32_t* slot_offsets, int s, long long P, long long* a,
                                          long long* b) {
  long long lo = slot_offsets[s], hi = slot_offsets[s + 1];
  lo = lo < 0 ? 0 : (lo > P ? P : lo);
  hi = hi < lo ? lo : (hi > P ? P : hi);
  *a = lo;
  *b = hi;
}

// slot_offsets -> row tiles.  Offsets are clipped to [0, P] and made non-decreasing.
//
// For the MFMA GEMMs (n_tiles_up/down > 0) the kernel also deals each GEMM's work units (one
// row group x kGroupN column tiles) to the 8 XCDs' queues: in (row group, column group) order,
// eight at a time, alternate eights in opposite directions.  The XCDs thus work on neighbouring
// column groups of the same row group at the same time and share its activation panel in the
// memory-side cache, and a regular pattern of large and small units (a narrow last column
// group, say) does not pile the large ones on the same XCDs; what imbalance is left the GEMM
// kernel evens out by itself.  (Dealing by estimated cost, least-loaded queue first, was
// within 2 % of this and costs a serial pass over the units; dealing the full row groups
// first and the ragged ones last measured 1-5 % slower.)
__global__ __launch_bounds__(256) void build_tiles_kernel(const int32_t* __restrict__ slot_offsets,
                                                          int S, long long P, int BM, int group,
                                                          int n_tiles_up, int n_tiles_down, TileTable t) {
  __shared__ int s_first[lz::kMaxN * lz::kMaxC + 1];
  // padded tile count of every slot (parallel: the offsets come from global memory), then one
  // thread's running sum over LDS
  for (int s = threadIdx.x; s < S; s += blockDim.x) {
    long long a, b;
    clip_slot(slot_offsets, s, P, &a, &b);
    const int tiles = int((b - a + BM - 1) / BM);
    s_first[s + 1] = (tiles + group - 1) / group * group;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    int running = 0;
    for (int s = 0; s < S; ++s) {
      int padded = s_first[s + 1];
      if (running + padded > t.capacity) padded = t.capacity - running;  // cannot happen for clipped offsets
      s_first[s] = running;
      running += padded;
    }
    s_first[S] = running;
    t.header[0] = running;
    for (int i = 40; i < 64; ++i) t.header[i] = 0;  // tile-queue tickets of the GEMM kernels
  }
  __syncthreads();
  for (int s = threadIdx.x; s < S; s += blockDim.x) {
    long long a, b;
    clip_slot(slot_offsets, s, P, &a, &b);
    for (int i = s_first[s]; i < s_first[s + 1]; ++i) {
      const long long r0 = a + (long long)(i - s_first[s]) * BM;
      t.slot[i] = r0 < b ? s : -1;  // -1: padding entry, no rows
      t.row0[i] = int(r0 < b ? r0 : b);
      t.row_end[i] = int(b);
    }
  }
  // deal the units, in (row group, column group) order, to the XCD queues in rows of eight,
  // alternate rows in opposite directions
  const int n_groups = s_first[S] / group;
  for (int which = 0; which < 2; ++which) {
    const int nt = which == 0 ? n_tiles_up : n_tiles_down;
    const int ncg = (nt + kGroupN - 1) / kGroupN;
    const int n_units = n_groups * ncg;  // 0 on the generic path
    const int cap = t.unit_cap[which];
    for (int u = threadIdx.x; u < n_units; u += blockDim.x) {
      const int row = u / 8, i = u % 8;
      const int x = (row & 1) ? 7 - i : i;
      if (row < cap) t.units[which][(size_t)x * cap + row] = u;  // n_units <= 4 * cap: always true
    }
    if (threadIdx.x < 8) {
      const int rows = n_units / 8, rest = n_units % 8;
      const int i = (rows & 1) ? 7 - (int)threadIdx.x : (int)threadIdx.x;  // position of this XCD in the last row
      t.header[kUnitCount + 16 * which + threadIdx.x] = rows + (i < rest ? 1 : 0);
    }
  }
}

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

// C[rows of the tile, n] = epi( sum_k A[row, k] * W[slot][n (+ n_up), k] )
template <typename Elem, int EPI>
__global__ __launch_bounds__(256) void gemm_generic_kernel(const Elem* __restrict__ A, int K,
                                                           const Elem* __restrict__ W,
                                                           size_t w_slot_stride, int n_out, int up_row0,
                                                           Elem* __restrict__ C, TileTable t) {
  constexpr int BM = 64, BN = 64, BK = 16;
  constexpr bool DUAL = EPI == EPI_SWIGLU;
  __shared__ float sA[BK][BM + 1];
  __shared__ float sB[DUAL ? 2 : 1][BK][BN + 1];
  const int tile = blockIdx.y;
  if (tile >= t.header[0]) return;
  const int slot = t.slot[tile], row0 = t.row0[tile], row_end = t.row_end[tile];
  if (slot < 0) return;
  const int n0 = blockIdx.x * BN;
  const Elem* Ws = W + (size_t)slot * w_slot_stride;
  const int tx = threadIdx.x % 16, ty = threadIdx.x / 16;
  float acc[4][4] = {}, acc_up[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += BK) {
    for (int i = threadIdx.x; i < BM * BK; i += 256) {
      const int r = i / BK, kk = i % BK;
      const int row = row0 + r;
      sA[kk][r] = (row < row_end && k0 + kk < K) ? load_elem<Elem>(A + (size_t)row * K + k0 + kk) : 0.f;
      const int n = n0 + r;
      const bool ok = n < n_out && k0 + kk < K;
      sB[0][kk][r] = ok ? load_elem<Elem>(Ws + (size_t)n * K + k0 + kk) : 0.f;
      if (DUAL) sB[DUAL ? 1 : 0][kk][r] = ok ? load_elem<Elem>(Ws + (size_t)(up_row0 + n) * K + k0 + kk) : 0.f;
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

// ------------------------------------------------------------------------------------------
// gfx950 MFMA kernel, bf16 in / fp32 accumulate / bf16 out
// ------------------------------------------------------------------------------------------
constexpr int BM = 256, BN = 256, BK = 64;
constexpr int kRowBytes = BK * 2;                  // one tile row of a stage in LDS: 128 B = 8 chunks of 16 B
constexpr int kStageBytes = (BM + BN) * kRowBytes; // activation tile (up to 256 rows), then weight tile
constexpr int kLdsBytes = 2 * kStageBytes;         // two stages: 128 KiB of the CU's 160 KiB

struct MfmaArgs {
  const uint16_t* A;    // [P, K]
  const uint16_t* W;    // [S, w_rows, K]
  uint16_t* C;          // [P, n_out]
  long long P;
  int K;
  int w_rows;           // weight rows per slot
  int n_out;            // output columns
  int up_row0;          // SwiGLU: first row of the up projection inside a slot's W
  int n_tiles;          // column tiles per row tile
  int which;            // 0 = GEMM-1, 1 = GEMM-2: which unit lists and tickets of the tile table
  TileTable t;
};

// Activations on the fp32 accumulators of the bf16 path.  The result is rounded to bf16
// (relative step 2^-9), so hardware exp2 / rcp (1 ulp) are used; erf is the
// Abramowitz-Stegun 7.1.26 rational form, absolute error below 2e-7 before those.
__device__ __forceinline__ float silu_fast(float v) {
  return v * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.44269504088896341f * v));
}
__device__ __forceinline__ float gelu_fast(float v) {
  const float x = fabsf(v) * 0.70710678118654752440f;
  const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, x, 1.0f));
  float p = fmaf(1.061405429f, t, -1.453152027f);
  p = fmaf(p, t, 1.421413741f);
  p = fmaf(p, t, -0.284496736f);
  p = fmaf(p, t, 0.254829592f);
  const float e = __builtin_amdgcn_exp2f(-1.44269504088896341f * x * x);
  const float erf_abs = 1.0f - p * t * e;         // erf(|v| / sqrt 2)
  return 0.5f * v + 0.5f * fabsf(v) * erf_abs;    // 0.5 v (1 + sign(v) erf_abs)
}

// Two fp32 -> one dword of two bf16, round to nearest even (v_cvt_pk_bf16_f32 on gfx950).
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  const f32x2 v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// 16-byte chunk c of tile row r lives at chunk position c ^ swz(r) of its 128-byte LDS row.
// LDS has 64 banks of 4 B, so a ds_read_b128 is served 16 lanes at a time: 16 consecutive
// rows at one logical chunk must cover 16 distinct 16-byte bank groups (256 B = 2 rows), hence
// the key row/2.
__device__ __forceinline__ int swz(int row) { return (row >> 1) & 7; }

// Scheduling hint for one 16-wide K slice of NM MFMAs: the ND ds_reads go out one per MFMA from
// the start of the slice (the next slice waits on them), the NV direct-to-LDS loads are spread
// evenly over the slice.
template <int Q, int ND, int NM, int NV>
__device__ __forceinline__ void sched_slice() {
  if constexpr (Q < NM) {
    constexpr int v = (NV * (Q + 1)) / NM - (NV * Q) / NM;
    if constexpr (v > 0) __builtin_amdgcn_sched_group_barrier(0x020, v, 0);       // VMEM read
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                             // MFMA
    if constexpr (Q < ND) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);      // DS read
    sched_slice<Q + 1, ND, NM, NV>();
  }
}

// One output tile of 64*XF rows x 256 weight rows.  XF = 32-row activation fragments per
// wave: the 2x2 waves each own (32*XF) x 128 of the tile, so a slot's ragged last tile costs
// MFMAs and activation loads only for its rows rounded up to 64.
template <int EPI, int XF>
__device__ __forceinline__ void gemm_tile(const MfmaArgs& a, char* smem, int slot, int row0, int row_end, int n0) {
  constexpr int KS = BK / 16;             // 16-wide MFMA slices per stage
  constexpr int kLoadsX = 2 * XF;         // 1-KiB wave loads per wave for the activation tile (8 rows each)
  constexpr int kLoadsW = 8;              // ... for the 256-row weight tile
  // The empty asm keeps the per-lane address arithmetic below inside the tile: hoisted out of
  // the caller's tile loop it would be carried in registers through the whole kernel and spill.
  int tid = threadIdx.x;
  asm volatile("" : "+v"(tid));
  const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;

  // ---- buffer descriptors: out-of-range loads return zero instead of faulting.  The activation
  // descriptor covers just this tile's rows, so 32-bit offsets do however large P is.
  const int n_rows = row_end - row0 < BM ? row_end - row0 : BM;
  const __amdgpu_buffer_rsrc_t rsrcA = __builtin_amdgcn_make_buffer_rsrc(
      (void*)(a.A + (size_t)row0 * a.K), 0, (int)((uint32_t)n_rows * (uint32_t)a.K * 2u), 0x00020000);
  const __amdgpu_buffer_rsrc_t rsrcB = __builtin_amdgcn_make_buffer_rsrc(
      (void*)(a.W + (size_t)slot * a.w_rows * a.K), 0, (int)(uint32_t)((unsigned long long)a.w_rows * a.K * 2),
      0x00020000);
  const __amdgpu_buffer_rsrc_t rsrcNull = __builtin_amdgcn_make_buffer_rsrc((void*)a.A, 0, 0, 0x00020000);

  // ---- per-lane global offsets of the direct-to-LDS loads of one stage.
  // Load u of an operand tile fills LDS bytes [u*1024, u*1024+1024): 8 whole rows, lane l
  // landing at row 8u + l/8, 16-byte chunk l%8.  That LDS chunk must hold logical chunk
  // (l%8) ^ swz(row), so the lane fetches that one (the swizzle is applied on the global side
  // because a direct-to-LDS load fixes the LDS side to lane order).
  int voffX[kLoadsX], voffW[kLoadsW];
#pragma unroll
  for (int i = 0; i < kLoadsX; ++i) {
    const int r = (wave * kLoadsX + i) * 8 + (lane >> 3);
    const int chunk = (lane & 7) ^ swz(r);
    const int ga = r < n_rows ? r : n_rows - 1;  // rows past the tile's end repeat its last row (never stored)
    voffX[i] = (int)(((uint32_t)ga * (uint32_t)a.K + (uint32_t)chunk * 8u) * 2u);
  }
#pragma unroll
  for (int i = 0; i < kLoadsW; ++i) {
    const int r = (wave * kLoadsW + i) * 8 + (lane >> 3);
    const int chunk = (lane & 7) ^ swz(r);
    int gb;
    if (EPI == EPI_SWIGLU) {
      const int f = r >> 5;  // fragment index: even = gate rows, odd = up rows
      gb = n0 + (f >> 1) * 32 + (r & 31) + ((f & 1) ? a.up_row0 : 0);
    } else {
      gb = n0 + r;
    }
    voffW[i] = (int)(((uint32_t)gb * (uint32_t)a.K + (uint32_t)chunk * 8u) * 2u);
  }

  // ---- fragment read addresses: lane l reads row (l%32) of a 32-row fragment, logical chunk
  // 2*ks + l/32 of the stage's K slice
  int fragoff[KS];
  {
    const int r = lane & 31;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) fragoff[ks] = r * kRowBytes + (((ks * 2 + (lane >> 5)) ^ swz(r)) << 4);
  }
  const int xbase = wm * 32 * XF * kRowBytes;               // this wave's activation rows
  const int wbase = BM * kRowBytes + wn * 128 * kRowBytes;  // this wave's 128 weight rows

  f32x16 acc[4][XF];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < XF; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  // ---- main loop: two LDS stages of 64 K-columns, and two register sets of fragments
  // alternating over the four 16-wide slices so that the ds_reads of the next slice are in
  // flight while the MFMAs of the current one run.  One barrier per step, placed after the
  // reads of the step's last slice have been issued: past it nobody reads the current stage any
  // more, so the loads of step kt+2 can start into it, and the next stage (whose loads every
  // wave has waited for before the barrier) can be read.
  //
  // The loads of step kt+2 are not issued in one burst: a wave that issues a burst stands still
  // until the texture unit has accepted it, and the MFMA pipe with it.  Six go out during the
  // slice after barrier kt, the rest during slice 0 of step kt+1, none in slices 1 and 2, which
  // leaves every load two slices to land before the wait at the end of step kt+1; the
  // activation loads go first.  (Measured on three workloads: 6 + rest + 0 beats 8 + half + half
  // by 2-11 %, and 4, 5, 7, 8, 10, 12 or all 16 after the barrier; activations first is 0.7 %
  // ahead of weights first on the first GEMM and level on the second.)
  const int k_steps = a.K / BK;
  constexpr int kLoads = kLoadsW + kLoadsX;
  auto issue = [&](int stage, int step, int q0, int q1) {
    // a step past the end of K is "loaded" through a zero-length descriptor: no memory traffic
    const bool real = step < k_steps;
    const __amdgpu_buffer_rsrc_t ra = real ? rsrcA : rsrcNull;
    const __amdgpu_buffer_rsrc_t rb = real ? rsrcB : rsrcNull;
    char* sX = smem + stage * kStageBytes;
    char* sW = sX + BM * kRowBytes;
#pragma unroll
    for (int q = q0; q < q1; ++q) {
      if (q < kLoadsX) {
        const int u = wave * kLoadsX + q;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(ra, (__attribute__((address_space(3))) void*)(sX + u * 1024), 16,
                                                 voffX[q], step * BK * 2, 0, 0);
      } else {
        const int u = wave * kLoadsW + (q - kLoadsX);
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rb, (__attribute__((address_space(3))) void*)(sW + u * 1024), 16,
                                                 voffW[q - kLoadsX], step * BK * 2, 0, 0);
      }
    }
  };
  constexpr int kAfterBarrier = 6;                 // loads issued in the slice after the barrier,
  constexpr int kSlice0 = kLoads - kAfterBarrier;  // and in slice 0 of the next step
  bf16x8 xf[2][XF], wf[2][4];
  // read order = order of first use by the MFMAs (weight fragment 0, all activation fragments,
  // weight fragments 1..3)
  auto read_frags = [&](const char* stage, int ks, int set) {
    wf[set][0] = *(const bf16x8*)(stage + wbase + fragoff[ks]);
#pragma unroll
    for (int j = 0; j < XF; ++j) xf[set][j] = *(const bf16x8*)(stage + xbase + j * 32 * kRowBytes + fragoff[ks]);
#pragma unroll
    for (int i = 1; i < 4; ++i) wf[set][i] = *(const bf16x8*)(stage + wbase + i * 32 * kRowBytes + fragoff[ks]);
  };
  auto read_one = [&](const char* stage, int ks, int set, int r) {  // r-th fragment in that order
    if (r == 0) wf[set][0] = *(const bf16x8*)(stage + wbase + fragoff[ks]);
    else if (r <= XF) xf[set][r - 1] = *(const bf16x8*)(stage + xbase + (r - 1) * 32 * kRowBytes + fragoff[ks]);
    else wf[set][r - XF] = *(const bf16x8*)(stage + wbase + (r - XF) * 32 * kRowBytes + fragoff[ks]);
  };
  // Fragment reads and direct-to-LDS loads of one slice, alternating in program order.  The
  // compiler cannot tell that a load's LDS destination and a fragment read never overlap, so it
  // keeps the two kinds in the order written: written as "all loads, then all reads", the reads
  // would reach the LDS queue only after the last load and the next slice's first MFMAs would
  // each wait out an LDS round trip.
  auto reads_and_loads = [&](const char* rd_stage, int ks, int set, int ld_stage, int step, int q0, int q1) {
    constexpr int NR = 4 + XF;
    const int NL = q1 - q0;
#pragma unroll
    for (int r = 0; r < NR; ++r) {
      read_one(rd_stage, ks, set, r);
      issue(ld_stage, step, q0 + (NL * r) / NR, q0 + (NL * (r + 1)) / NR);
    }
  };
  auto mma = [&](int set) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < XF; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[set][i], xf[set][j], acc[i][j], 0, 0, 0);
  };

  issue(0, 0, 0, kLoads);
  issue(1, 1, 0, kAfterBarrier);
  // s_waitcnt with only vmcnt set (bits [3:0] and [15:14]): stage 1's first loads may still be in flight
  __builtin_amdgcn_s_waitcnt(0x0F70 | kAfterBarrier);
  __syncthreads();
  read_frags(smem, 0, 0);

  for (int kt = 0; kt < k_steps; ++kt) {
    const int cur = kt & 1;
    const char* st = smem + cur * kStageBytes;
    const char* nx = smem + (cur ^ 1) * kStageBytes;
    reads_and_loads(st, 1, 1, cur ^ 1, kt + 1, kAfterBarrier, kLoads);
    mma(0);
    sched_slice<0, 4 + XF, 4 * XF, kSlice0>();
    read_frags(st, 2, 0);
    mma(1);
    sched_slice<0, 4 + XF, 4 * XF, 0>();
    read_frags(st, 3, 1);
    mma(0);
    sched_slice<0, 4 + XF, 4 * XF, 0>();
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this wave's loads of the next stage are in LDS
    __syncthreads();                     // everyone's are; nobody reads stage `cur` any more
    reads_and_loads(nx, 0, 0, cur, kt + 2, 0, kAfterBarrier);
    mma(1);
    sched_slice<0, 4 + XF, 4 * XF, kAfterBarrier>();
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);  // drain the (empty) trailing loads before LDS is reused

  // ---- epilogue.  acc[i][j] is the 32x32 block (weight fragment i) x (activation fragment j);
  // lane l holds activation row j*32 + l%32 and, for g = 0..3, the 4 consecutive weight rows
  // i*32 + 8g + 4*(l/32) + 0..3  -> 4 consecutive output columns.  Stored straight from there,
  // a wave store would touch 32 rows with 16 bytes each; such partial-line writes cost the
  // second GEMM 10 % (timed with the stores removed).  So each 32-row fragment goes through a
  // per-wave LDS patch (the stages are dead by now; LDS serves a wave's accesses in order) and
  // leaves as 16 bytes per lane, whole 128-byte lines at a time.
  constexpr int kWaveCols = EPI == EPI_SWIGLU ? 64 : 128;  // output columns of this wave
  constexpr int kPitch = kWaveCols * 2 + 16;               // patch row in bytes: 16-byte aligned, rows 4 banks apart
  constexpr int kLanesPerRow = kWaveCols / 8;              // 16-byte pieces of a patch row
  constexpr int kRowsPerStore = 64 / kLanesPerRow;
  char* const patch = smem + wave * (32 * kPitch);
  const int half = lane >> 5;
#pragma unroll
  for (int j = 0; j < XF; ++j) {
    char* const prow = patch + (lane & 31) * kPitch;
    if (EPI == EPI_SWIGLU) {
#pragma unroll
      for (int q = 0; q < 2; ++q)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          float o[4];
#pragma unroll
          for (int r = 0; r < 4; ++r) o[r] = silu_fast(acc[2 * q][j][4 * g + r]) * acc[2 * q + 1][j][4 * g + r];
          uint2 pk;
          pk.x = pack_bf16x2(o[0], o[1]);
          pk.y = pack_bf16x2(o[2], o[3]);
          *(uint2*)(prow + (q * 32 + 8 * g + 4 * half) * 2) = pk;
        }
    } else {
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          float o[4];
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            o[r] = acc[i][j][4 * g + r];
            if (EPI == EPI_GELU) o[r] = gelu_fast(o[r]);
          }
          uint2 pk;
          pk.x = pack_bf16x2(o[0], o[1]);
          pk.y = pack_bf16x2(o[2], o[3]);
          *(uint2*)(prow + (i * 32 + 8 * g + 4 * half) * 2) = pk;
        }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");  // keep the patch writes before the reads below
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
    for (int t = 0; t < 32 / kRowsPerStore; ++t) {
      const int r = t * kRowsPerStore + lane / kLanesPerRow, piece = lane % kLanesPerRow;
      const uint4 v = *(const uint4*)(patch + r * kPitch + piece * 16);
      const int row = row0 + wm * 32 * XF + j * 32 + r;
      if (row < row_end) *(uint4*)(a.C + (size_t)row * a.n_out + n0 + wn * kWaveCols + piece * 8) = v;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");  // ... and the reads before the next fragment's writes
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  }
}

[[maybe_unused]] constexpr int kTicket = 40;  // header[kTicket + 8*g + x]: next entry of XCD x's tile queue for GEMM g
[[maybe_unused]] constexpr int kDone = 56;    // header[kDone + g]: workgroups of GEMM g's launch that have finished

// Persistent kernel: one workgroup per CU.  Every XCD has a queue of tiles (its unit list, 32
// tile slots per unit: kGroupM row tiles of one slot x kGroupN column tiles); a workgroup takes
// the next slot of its own XCD's queue with an atomic ticket, and once that queue is empty
// helps with the other XCDs' queues.  The 32 tiles an XCD works on at a time therefore share
// their activation and weight panels through that XCD's L2, and each XCD drains its queue at
// its own pace.  (The hardware hands the workgroups of an ordinary launch to the XCDs strictly
// in order of their index: there an XCD whose tiles take longer holds back the workgroups
// queued behind it for every other XCD, which costs 10-40 % on ragged plans.)
template <int EPI>
__global__ __launch_bounds__(256, 1) void gemm_mfma_kernel(MfmaArgs a) {
#if defined(__HIP_DEVICE_COMPILE__)  // the host pass only needs the launch stub, not the gfx950 builtins
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  constexpr int BN_OUT = EPI == EPI_SWIGLU ? BN / 2 : BN;
  constexpr int kUnitTiles = kGroupM * kGroupN;
  const int xcd = blockIdx.x % 8;  // workgroups are dealt round-robin to the 8 XCDs
  const int n_col_groups = (a.n_tiles + kGroupN - 1) / kGroupN;
  int* const ticket = a.t.header + kTicket + 8 * a.which;
  const int32_t* const count = a.t.header + kUnitCount + 16 * a.which;
  for (int hop = 0; hop < 8; ++hop) {
    const int q = (xcd + hop) % 8;
    const int n_slots = count[q] * kUnitTiles;
    const int32_t* const list = a.t.units[a.which] + (size_t)q * a.t.unit_cap[a.which];
    for (;;) {
      __syncthreads();  // the previous tile's fragment reads are done: LDS may be reused
      if (threadIdx.x == 0) *(volatile int*)smem = atomicAdd(ticket + q, 1);
      __syncthreads();
      const int t = __builtin_amdgcn_readfirstlane(*(volatile int*)smem);
      __syncthreads();
      if (t >= n_slots) break;  // every workgroup draws one ticket past the end of every queue, no more
      const int unit = list[t / kUnitTiles];
      const int within = t % kUnitTiles;
      const int nt = (unit % n_col_groups) * kGroupN + within / kGroupM;
      if (nt >= a.n_tiles) continue;
      const int row_tile = (unit / n_col_groups) * kGroupM + within % kGroupM;
      const int slot = a.t.slot[row_tile];
      if (slot < 0) continue;
      const int row0 = a.t.row0[row_tile];
      const int row_end = a.t.row_end[row_tile];
      const int n0 = nt * BN_OUT;
      const int rows = row_end - row0;  // > 0; more than 256 means a full tile
      if (rows > 192) gemm_tile<EPI, 4>(a, smem, slot, row0, row_end, n0);
      else if (rows > 128) gemm_tile<EPI, 3>(a, smem, slot, row0, row_end, n0);
      else if (rows > 64) gemm_tile<EPI, 2>(a, smem, slot, row0, row_end, n0);
      else gemm_tile<EPI, 1>(a, smem, slot, row0, row_end, n0);
    }
  }
  // the last workgroup to finish leaves the tickets at zero for the next launch on this table
  if (threadIdx.x == 0) {
    int* const done = a.t.header + kDone + a.which;
    if (atomicAdd(done, 1) == (int)gridDim.x - 1) {
      for (int q = 0; q < 8; ++q) ticket[q] = 0;
      *done = 0;
    }
  }
#endif
}

template <int EPI>
int32_t launch_mfma(const MfmaArgs& a, hipStream_t st) {
  void (*kern)(MfmaArgs) = gemm_mfma_kernel<EPI>;
  static bool configured = false;  // per-process attribute; idempotent, so a benign race at worst
  static int n_workgroups = 0;
  if (!configured) {
    if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes) !=
        hipSuccess)
      return LZ_EHIP;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
      return LZ_EHIP;
    n_workgroups = cus >= 8 ? cus / 8 * 8 : 8;  // one per CU (the LDS a workgroup takes allows no more)
    configured = true;
  }
  hipLaunchKernelGGL(kern, dim3(n_workgroups), dim3(256), kLdsBytes, st, a);
  return lz::launch_status();
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

extern "C" int32_t lz_ffn_up(const void* xp, const void* w1, const lz_shape* shape, void* ws,
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
  if (!mfma_shape(shape)) {
    const dim3 grid((shape->ffn + 63) / 64, t.capacity);
    if (shape->dtype == LZ_F32) {
      if (swiglu)
        hipLaunchKernelGGL((gemm_generic_kernel<float, EPI_SWIGLU>), grid, dim3(256), 0, st, (const float*)xp,
                           shape->d, (const float*)w1, (size_t)n1 * shape->d, shape->ffn, shape->ffn,
                           (float*)w.hidden, t);
      else
        hipLaunchKernelGGL((gemm_generic_kernel<float, EPI_GELU>), grid, dim3(256), 0, st, (const float*)xp,
                           shape->d, (const float*)w1, (size_t)n1 * shape->d, shape->ffn, 0,
                           (float*)w.hidden, t);
    } else {
      if (swiglu)
        hipLaunchKernelGGL((gemm_generic_kernel<uint16_t, EPI_SWIGLU>), grid, dim3(256), 0, st,
                           (const uint16_t*)xp, shape->d, (const uint16_t*)w1, (size_t)n1 * shape->d,
                           shape->ffn, shape->ffn, (uint16_t*)w.hidden, t);
      else
        hipLaunchKernelGGL((gemm_generic_kernel<uint16_t, EPI_GELU>), grid, dim3(256), 0, st,
                           (const uint16_t*)xp, shape->d, (const uint16_t*)w1, (size_t)n1 * shape->d,
                           shape->ffn, 0, (uint16_t*)w.hidden, t);
    }
    return lz::launch_status();
  }
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
  return swiglu ? launch_mfma<EPI_SWIGLU>(g1, st) : launch_mfma<EPI_GELU>(g1, st);
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
                         (const float*)w.hidden, shape->ffn, (const float*)w2,
                         (size_t)shape->d * shape->ffn, shape->d, 0, (float*)yp, t);
    else
      hipLaunchKernelGGL((gemm_generic_kernel<uint16_t, EPI_NONE>), grid, dim3(256), 0, st,
                         (const uint16_t*)w.hidden, shape->ffn, (const uint16_t*)w2,
                         (size_t)shape->d * shape->ffn, shape->d, 0, (uint16_t*)yp, t);
    return lz::launch_status();
  }
  if ((uintptr_t)yp % 16 != 0) return LZ_EINVAL;  // the MFMA epilogue stores 16 bytes per lane
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
  return launch_mfma<EPI_NONE>(g2, st);
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
