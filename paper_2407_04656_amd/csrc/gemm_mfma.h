// Grouped bf16 GEMM on the gfx950 matrix cores and the row-tile table it draws its work from;
// shared by the forward and the backward translation units (device code, not part of the C ABI).
//
//   C[rows of a slot, n] = epi( sum_k A(row, k) * W[slot](n, k) )
//
// Persistent kernel, one workgroup per CU, drawing 256x256 tiles from its XCD's queue.  4 waves
// in 2x2, each wave a 128x128 patch = 4x4 v_mfma_f32_32x32x16_bf16 accumulators (fp32, 256
// AGPRs).  Operand tiles are streamed HBM -> LDS with 16-byte buffer loads that write LDS
// directly, through two LDS stages of 64 k; fragment reads are software pipelined over two
// register sets.  An operand may be k-contiguous ([row, k]: 256 tile rows of 128 B, read with
// ds_read_b128) or k-major ([k, column]: 64 k-rows of 512 B, read with the transposing
// ds_read_b64_tr_b16); see the MODE_* list below.  The XOR swizzles that keep the fragment
// reads free of bank conflicts are applied on the global-address side, because a direct-to-LDS
// load fixes the LDS side to lane order.  Buffer descriptors bound every load, so ragged tiles
// cannot fault.  The MFMA takes the weight fragment as its row operand, which leaves each lane
// with 4 consecutive output columns per accumulator group; the epilogue regroups them through
// a per-wave LDS patch into whole 128-byte lines.  For SwiGLU the weight tile interleaves
// 32-wide fragments of the gate and the up projection, so the gate and up values of one output
// element sit in the same lane and register index.
#pragma once
#include "lz_common.h"
#include <atomic>

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

constexpr int kTileHeader = 64;  // ints before the tile arrays; [0] = number of row tiles
constexpr int kGroupM = 4;       // row tiles of a work unit (same slot)
constexpr int kGroupN = 8;       // column tiles of a work unit

// *_KEEP: the training forward; besides act(z) the pre-activation z goes to MfmaArgs::Z.
// EPI_ACCUM: the result is added to the fp32 matrix MfmaArgs::Cacc (weight gradients summed over
// micro-batches) instead of being stored as bf16.
enum { EPI_NONE = 0, EPI_GELU = 1, EPI_SWIGLU = 2, EPI_GELU_KEEP = 3, EPI_SWIGLU_KEEP = 4, EPI_ACCUM = 5 };

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

// ------------------------------------------------------------------------------------------
// gfx950 MFMA kernel, bf16 in / fp32 accumulate / bf16 out
// ------------------------------------------------------------------------------------------
constexpr int BM = 256, BN = 256, BK = 64;
constexpr int kRowBytes = BK * 2;                  // one tile row of a stage in LDS: 128 B = 8 chunks of 16 B
constexpr int kStageBytes = (BM + BN) * kRowBytes; // activation tile (up to 256 rows), then weight tile
constexpr int kLdsBytes = 2 * kStageBytes;         // two stages: 128 KiB of the CU's 160 KiB

struct MfmaArgs {
  const uint16_t* A;    // MODE_NT, MODE_NN: [P, K];  MODE_TN: [k_rows, lda]
  const uint16_t* W;    // MODE_NT: [S, w_rows, K];  MODE_NN: [S, K, ldw];  MODE_TN: [k_rows, ldw]
  uint16_t* C;          // [P, n_out]
  float* Cacc;          // EPI_ACCUM: [P, n_out] fp32, read, added to and written back
  long long P;          // rows of C (MODE_TN: S * rows_per_slot virtual rows)
  int K;                // contraction length (MODE_TN: per slot, from slot_offsets)
  int w_rows;           // MODE_NT: weight rows per slot
  int n_out;            // output columns
  int up_row0;          // SwiGLU: offset of the up projection inside a slot's W (rows, or columns if k-major)
  int n_tiles;          // column tiles per row tile
  int which;            // which of the tile table's two unit lists and ticket sets this launch draws from
  TileTable t;
  // MODE_TN (weight gradients): slot s contracts over the rows [slot_offsets[s], slot_offsets[s+1])
  // of both operands and owns rows_per_slot rows of C (row index = s * rows_per_slot + m, m =
  // column of A).
  uint16_t* Z;          // *_KEEP epilogues: pre-activations [P, z_cols] (SwiGLU: gate columns, then up columns)
  int z_cols;
  int lda, ldw;         // row strides (elements) of the k-major operands
  const int32_t* slot_offsets;
  long long k_rows;
  int rows_per_slot;
  // GATHER (forward only): A is x [gather_T, K] and row r of the permuted buffer is row
  // gather[r] / gather_k of it (gather = row_to_pair of the dispatcher)
  const int32_t* gather;
  int gather_k;
  long long gather_T;
};

// Operand layouts of the contraction C[m, n] = sum_k A(m, k) W(n, k):
//   MODE_NT  A [m, k], W [n, k]: both contiguous along k (the data gradients)
//   MODE_NN  A [m, k], W [k, n] (the forward: weights are stored input-major)
//   MODE_TN  A [k, m], W [k, n], a different k range for every slot
// A k-major operand tile lies in LDS as 64 k-rows of 256 columns (512 B each) and is read with
// ds_read_b64_tr_b16, which hands every lane four k-values of one column: the 16 lanes of a
// group supply the addresses of 4 k-rows x 4 column quads, and lane i receives column i of the
// group's 16 at those four k.  Two such reads give the lane the same 8 consecutive k of its
// column that a ds_read_b128 gives it from a k-contiguous tile, so the MFMAs and the epilogue
// do not change.
enum { MODE_NT = 0, MODE_NN = 1, MODE_TN = 2 };
typedef short i16x4 __attribute__((ext_vector_type(4)));
typedef int i32x4 __attribute__((ext_vector_type(4)));

// The four words of a raw buffer descriptor (base, stride 0, bytes, data format word).
__device__ __forceinline__ i32x4 rsrc_words(const void* base, uint32_t bytes) {
  const uint64_t b = (uint64_t)base;
  return i32x4{(int)(uint32_t)b, (int)(uint32_t)((b >> 32) & 0xFFFFu), (int)bytes, 0x00020000};
}

// 16 bytes per lane from a buffer straight into LDS at lds_base + 16 * lane, written as assembly:
// in the k-major modes the compiler must not know that loads into LDS are in flight, or it
// makes every transposing LDS read wait for all of them (it cannot tell that the two never
// touch the same bytes).  The kernel orders loads and reads itself (s_waitcnt vmcnt + barrier).
__device__ __forceinline__ void load16_to_lds(i32x4 rsrc, uint32_t lds_base, int voffset, int soffset) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
               :
               : "s"(lds_base), "v"(voffset), "s"(rsrc), "s"(soffset)
               : "memory");  // m0 is scratch to the compiler as well: it loads it right before each use
}

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

// One output tile of 64*XF rows x 256 columns n of the weight operand W(n, k) ("weight rows"
// below, whichever way W lies in memory).  XF = 32-row activation fragments per wave: the 2x2 waves each own (32*XF) x 128 of the tile, so a slot's ragged last tile costs
// MFMAs and activation loads only for its rows rounded up to 64.
template <int EPI, int XF, int MODE, bool GATHER>
__device__ __forceinline__ void gemm_tile(const MfmaArgs& a, char* smem, int slot, int row0, int row_end, int n0) {
  constexpr bool TA = MODE == MODE_TN, TB = MODE != MODE_NT;  // k-major left / right operand
  constexpr bool kGated = EPI == EPI_SWIGLU || EPI == EPI_SWIGLU_KEEP;
  constexpr int KS = BK / 16;             // 16-wide MFMA slices per stage
  constexpr int kLoadsX = TA ? 8 : 2 * XF;  // 1-KiB wave loads per wave for the left tile (8 rows, or 2 k-rows, each)
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
  int K = a.K;
  const uint16_t* tileA;
  const uint16_t* tileW;
  uint32_t a_extent, w_extent;          // bytes the two descriptors cover
  int stepA = BK * 2, stepW = BK * 2;   // bytes one K step advances in each operand
  // MODE_TN: a slot's rows of the k-major operands may cover more than 4 GiB, so the descriptors
  // are rebuilt for every K step (base advanced by whole steps, extent = what is left of the slot)
  [[maybe_unused]] unsigned long long a_bytes = 0, w_bytes = 0, stepA64 = 0, stepW64 = 0;
  if constexpr (MODE == MODE_TN) {
    // The descriptors start at the slot's first row and this tile's first column and end with
    // the slot's last row: the rows of the last, partial K step that belong to the next slot
    // read as zero.
    long long s0, s1;
    clip_slot(a.slot_offsets, slot, a.k_rows, &s0, &s1);
    K = int(s1 - s0);
    const int m0 = row0 - slot * a.rows_per_slot;
    tileA = a.A + (size_t)s0 * a.lda + m0;
    tileW = a.W + (size_t)s0 * a.ldw + n0;
    a_bytes = K > 0 ? ((unsigned long long)K * (unsigned)a.lda - (unsigned)m0) * 2ull : 0ull;
    w_bytes = K > 0 ? ((unsigned long long)K * (unsigned)a.ldw - (unsigned)n0) * 2ull : 0ull;
    stepA64 = 64ull * (unsigned)a.lda * 2ull;
    stepW64 = 64ull * (unsigned)a.ldw * 2ull;
    a_extent = a_bytes > 0xFFFFFFFFull ? 0xFFFFFFFFu : (uint32_t)a_bytes;  // (unused: see issue())
    w_extent = w_bytes > 0xFFFFFFFFull ? 0xFFFFFFFFu : (uint32_t)w_bytes;
    stepA = 0;
    stepW = 0;
  } else if constexpr (MODE == MODE_NN) {
    if constexpr (GATHER) {
      tileA = a.A;  // the whole of x: a tile's rows lie anywhere in it (the host checked that it fits 32-bit offsets)
      a_extent = (uint32_t)((unsigned long long)a.gather_T * (unsigned)K * 2ull);
    } else {
      tileA = a.A + (size_t)row0 * K;
      a_extent = (uint32_t)n_rows * (uint32_t)K * 2u;
    }
    tileW = a.W + (size_t)slot * K * a.ldw;
    w_extent = (uint32_t)K * (uint32_t)a.ldw * 2u;
    stepW = 64 * a.ldw * 2;
  } else {
    tileA = a.A + (size_t)row0 * K;
    a_extent = (uint32_t)n_rows * (uint32_t)K * 2u;
    tileW = a.W + (size_t)slot * a.w_rows * K;
    w_extent = (uint32_t)((unsigned long long)a.w_rows * K * 2);
  }
  const __amdgpu_buffer_rsrc_t rsrcA = __builtin_amdgcn_make_buffer_rsrc((void*)tileA, 0, (int)a_extent, 0x00020000);
  const __amdgpu_buffer_rsrc_t rsrcB = __builtin_amdgcn_make_buffer_rsrc((void*)tileW, 0, (int)w_extent, 0x00020000);
  const __amdgpu_buffer_rsrc_t rsrcNull = __builtin_amdgcn_make_buffer_rsrc((void*)a.A, 0, 0, 0x00020000);
  const i32x4 wordsA = rsrc_words(tileA, a_extent), wordsB = rsrc_words(tileW, w_extent);
  const i32x4 wordsNull = rsrc_words(a.A, 0);
  const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)smem;

  // ---- per-lane global offsets of the direct-to-LDS loads of one stage.
  // Load u of an operand tile fills LDS bytes [u*1024, u*1024+1024): 8 whole rows, lane l
  // landing at row 8u + l/8, 16-byte chunk l%8.  That LDS chunk must hold logical chunk
  // (l%8) ^ swz(row), so the lane fetches that one (the swizzle is applied on the global side
  // because a direct-to-LDS load fixes the LDS side to lane order).
  //
  // k-major operand: load u fills two k-rows of 512 B, lane l landing at k-row 2u + l/32, 16-byte
  // piece l%32, which must hold logical piece (l%32) ^ 4*(k-row % 4): the four k-rows that one
  // transposing read touches at the same columns then lie in four different quarters of the banks.
  auto voff_kmajor = [&](int i, int ld, int col0) {
    const int kr = (wave * 8 + i) * 2 + (lane >> 5);
    const int piece = (lane & 31) ^ ((kr & 3) << 2);
    return (int)(((uint32_t)kr * (uint32_t)ld + (uint32_t)col0 + (uint32_t)piece * 8u) * 2u);
  };
  int voffX[kLoadsX], voffW[kLoadsW];
  // GATHER: the activation rows are looked up through the row map.  The index loads go out first
  // and are waited for only after the first weight loads have been issued (further down), so
  // their latency hides behind the weights' way from HBM.
  [[maybe_unused]] int gidx[kLoadsX];
  if constexpr (GATHER) {
    const i32x4 wordsG = rsrc_words(a.gather + row0, (uint32_t)n_rows * 4u);
#pragma unroll
    for (int i = 0; i < kLoadsX; ++i) {
      const int r = (wave * kLoadsX + i) * 8 + (lane >> 3);
      const int ga = r < n_rows ? r : n_rows - 1;
      asm volatile("buffer_load_dword %0, %1, %2, 0 offen" : "=v"(gidx[i]) : "v"(ga * 4), "s"(wordsG) : "memory");
    }
  }
#pragma unroll
  for (int i = 0; i < kLoadsX; ++i) {
    if constexpr (GATHER) {
      voffX[i] = 0;  // set once the indices have arrived
    } else if constexpr (TA) {
      voffX[i] = voff_kmajor(i, a.lda, 0);  // columns past the operand's edge fetch its neighbours: never stored
    } else {
      const int r = (wave * kLoadsX + i) * 8 + (lane >> 3);
      const int chunk = (lane & 7) ^ swz(r);
      const int ga = r < n_rows ? r : n_rows - 1;  // rows past the tile's end repeat its last row (never stored)
      voffX[i] = (int)(((uint32_t)ga * (uint32_t)K + (uint32_t)chunk * 8u) * 2u);
    }
  }
#pragma unroll
  for (int i = 0; i < kLoadsW; ++i) {
    if constexpr (TB && kGated) {
      // k-major SwiGLU weights [K, 2 ffn]: 32-column fragments alternate gate and up columns
      const int kr = (wave * 8 + i) * 2 + (lane >> 5);
      const int piece = (lane & 31) ^ ((kr & 3) << 2);
      const int f = piece >> 2;
      const int col = n0 + (f >> 1) * 32 + (piece & 3) * 8 + ((f & 1) ? a.up_row0 : 0);
      voffW[i] = (int)(((uint32_t)kr * (uint32_t)a.ldw + (uint32_t)col) * 2u);
    } else if constexpr (TB) {
      voffW[i] = voff_kmajor(i, a.ldw, MODE == MODE_NN ? n0 : 0);
    } else {
      const int r = (wave * kLoadsW + i) * 8 + (lane >> 3);
      const int chunk = (lane & 7) ^ swz(r);
      int gb;
      if (kGated) {
        const int f = r >> 5;  // fragment index: even = gate rows, odd = up rows
        gb = n0 + (f >> 1) * 32 + (r & 31) + ((f & 1) ? a.up_row0 : 0);
      } else {
        gb = n0 + r;
      }
      voffW[i] = (int)(((uint32_t)gb * (uint32_t)K + (uint32_t)chunk * 8u) * 2u);
    }
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
  // k-major tiles: lane 16g + s supplies the address of k-row 8*(g/2) + s/4 (of the 16-wide
  // slice), column quad s%4 of the group's 16 columns (16*(g%2) into the 32-column fragment)
  int tfoX[XF], tfoW[4];
  {
    const int g = lane >> 4, s = lane & 15;
    const int part = (8 * (g >> 1) + (s >> 2)) * 512 + ((2 * (g & 1) + ((s >> 1) & 1)) << 4) + ((s & 1) << 3);
#pragma unroll
    for (int j = 0; j < XF; ++j) tfoX[j] = part + 64 * ((XF * wm + j) ^ (s >> 2));
#pragma unroll
    for (int i = 0; i < 4; ++i) tfoW[i] = BM * kRowBytes + part + 64 * ((4 * wn + i) ^ (s >> 2));
  }
  auto read_kmajor = [&](const char* p) {
    const i16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) i16x4*)p);
    const i16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) i16x4*)(p + 4 * 512));
    return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
  };
  auto frag_x = [&](const char* stage, int ks, int j) {
    if constexpr (TA) return read_kmajor(stage + ks * 16 * 512 + tfoX[j]);
    else return *(const bf16x8*)(stage + xbase + j * 32 * kRowBytes + fragoff[ks]);
  };
  auto frag_w = [&](const char* stage, int ks, int i) {
    if constexpr (TB) return read_kmajor(stage + ks * 16 * 512 + tfoW[i]);
    else return *(const bf16x8*)(stage + wbase + i * 32 * kRowBytes + fragoff[ks]);
  };

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
  // until the texture unit has accepted it, and the MFMA pipe with it.  Six (eight when an
  // operand is k-major) go out during the slice after barrier kt, the rest during slice 0 of
  // step kt+1, none in slices 1 and 2, which leaves every load two slices to land before the
  // wait at the end of step kt+1; the activation loads go first.  (Measured on three workloads with k-contiguous operands: 6 + rest
  // + 0 beats 8 + half + half by 2-11 %, and 4, 5, 7, 8, 10, 12 or all 16 after the barrier;
  // activations first is 0.7 % ahead of weights first on the first GEMM and level on the second.
  // With k-major weights 8 after the barrier is 0.5-2 % ahead of 6, 10 level, 4, 12 and 16 behind.)
  const int k_steps = (K + BK - 1) / BK;
  constexpr int kLoads = kLoadsW + kLoadsX;
  auto issue = [&](int stage, int step, int q0, int q1) {
    // a step past the end of K is "loaded" through a zero-length descriptor: no memory traffic
    const bool real = step < k_steps;
    const __amdgpu_buffer_rsrc_t ra = real ? rsrcA : rsrcNull;
    const __amdgpu_buffer_rsrc_t rb = real ? rsrcB : rsrcNull;
    char* sX = smem + stage * kStageBytes;
    char* sW = sX + BM * kRowBytes;
    if constexpr (MODE != MODE_NT) {
      i32x4 wa = real ? wordsA : wordsNull, wb = real ? wordsB : wordsNull;
      if constexpr (MODE == MODE_TN) {
        const unsigned long long offA = (unsigned long long)(unsigned)step * stepA64;
        const unsigned long long offW = (unsigned long long)(unsigned)step * stepW64;
        const unsigned long long leftA = a_bytes > offA ? a_bytes - offA : 0ull;
        const unsigned long long leftW = w_bytes > offW ? w_bytes - offW : 0ull;
        wa = rsrc_words((const char*)tileA + offA, leftA > 0xFFFFFFFFull ? 0xFFFFFFFFu : (uint32_t)leftA);
        wb = rsrc_words((const char*)tileW + offW, leftW > 0xFFFFFFFFull ? 0xFFFFFFFFu : (uint32_t)leftW);
      }
      const uint32_t ldsX = lds0 + stage * kStageBytes, ldsW = ldsX + BM * kRowBytes;
#pragma unroll
      for (int q = q0; q < q1; ++q) {
        if (q < kLoadsX) load16_to_lds(wa, ldsX + (wave * kLoadsX + q) * 1024, voffX[q], step * stepA);
        else load16_to_lds(wb, ldsW + (wave * kLoadsW + q - kLoadsX) * 1024, voffW[q - kLoadsX], step * stepW);
      }
      return;
    }
#pragma unroll
    for (int q = q0; q < q1; ++q) {
      if (q < kLoadsX) {
        const int u = wave * kLoadsX + q;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(ra, (__attribute__((address_space(3))) void*)(sX + u * 1024), 16,
                                                 voffX[q], step * stepA, 0, 0);
      } else {
        const int u = wave * kLoadsW + (q - kLoadsX);
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rb, (__attribute__((address_space(3))) void*)(sW + u * 1024), 16,
                                                 voffW[q - kLoadsX], step * stepW, 0, 0);
      }
    }
  };
  constexpr int kDsReads = (TB ? 8 : 4) + (TA ? 2 * XF : XF);  // LDS read instructions per slice
  constexpr int kWanted = MODE == MODE_NT ? 6 : 8;
  constexpr int kAfterBarrier = kWanted < kLoads ? kWanted : kLoads;  // loads issued in the slice after the barrier,
  constexpr int kSlice0 = kLoads - kAfterBarrier;  // and in slice 0 of the next step
  bf16x8 xf[2][XF], wf[2][4];
  // read order = order of first use by the MFMAs (weight fragment 0, all activation fragments,
  // weight fragments 1..3)
  auto read_frags = [&](const char* stage, int ks, int set) {
    wf[set][0] = frag_w(stage, ks, 0);
#pragma unroll
    for (int j = 0; j < XF; ++j) xf[set][j] = frag_x(stage, ks, j);
#pragma unroll
    for (int i = 1; i < 4; ++i) wf[set][i] = frag_w(stage, ks, i);
  };
  auto read_one = [&](const char* stage, int ks, int set, int r) {  // r-th fragment in that order
    if (r == 0) wf[set][0] = frag_w(stage, ks, 0);
    else if (r <= XF) xf[set][r - 1] = frag_x(stage, ks, r - 1);
    else wf[set][r - XF] = frag_w(stage, ks, r - XF);
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

  if constexpr (GATHER) {
    issue(0, 0, kLoadsX, kLoads);                        // the weight tile of step 0 does not need the row map
    __builtin_amdgcn_s_waitcnt(0x0F70 | kLoadsW);        // vmcnt: the index loads (issued before those) are back
    const uint32_t gk = (uint32_t)a.gather_k, n_pairs = (uint32_t)(a.gather_T * a.gather_k);
#pragma unroll
    for (int i = 0; i < kLoadsX; ++i) {
      asm volatile("" : "+v"(gidx[i]));                  // nothing below may move above the wait
      const int r = (wave * kLoadsX + i) * 8 + (lane >> 3);
      const int chunk = (lane & 7) ^ swz(r);
      const uint32_t pair = (uint32_t)gidx[i];
      // a row without a pair (never inside a slot) reads past the descriptor's end: zeros
      voffX[i] = pair < n_pairs ? (int)((pair / gk * (uint32_t)K + (uint32_t)chunk * 8u) * 2u) : (int)a_extent;
    }
    issue(0, 0, 0, kLoadsX);
  } else {
    issue(0, 0, 0, kLoads);
  }
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
    sched_slice<0, kDsReads, 4 * XF, kSlice0>();
    read_frags(st, 2, 0);
    mma(1);
    sched_slice<0, kDsReads, 4 * XF, 0>();
    read_frags(st, 3, 1);
    mma(0);
    sched_slice<0, kDsReads, 4 * XF, 0>();
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this wave's loads of the next stage are in LDS
    __syncthreads();                     // everyone's are; nobody reads stage `cur` any more
    reads_and_loads(nx, 0, 0, cur, kt + 2, 0, kAfterBarrier);
    mma(1);
    sched_slice<0, kDsReads, 4 * XF, kAfterBarrier>();
  }
  // The trailing loads (steps past the end of K, zero-length descriptor) still write zeros into
  // stage `cur`, and each wave only waits for its own: with an odd number of K steps that is
  // stage 0, where the epilogue patches of the other waves lie.  Drain this wave's, then wait
  // until every wave has drained its own, before anybody writes a patch.
  __builtin_amdgcn_s_waitcnt(0x0F70);
  __syncthreads();

  // ---- epilogue.  acc[i][j] is the 32x32 block (weight fragment i) x (activation fragment j);
  // lane l holds activation row j*32 + l%32 and, for g = 0..3, the 4 consecutive weight rows
  // i*32 + 8g + 4*(l/32) + 0..3  -> 4 consecutive output columns.  Stored straight from there,
  // a wave store would touch 32 rows with 16 bytes each; such partial-line writes cost the
  // second GEMM 10 % (timed with the stores removed).  So each 32-row fragment goes through a
  // per-wave LDS patch (the stages are dead by now; LDS serves a wave's accesses in order) and
  // leaves as 16 bytes per lane, whole 128-byte lines at a time.
  constexpr int kWaveCols = kGated ? 64 : 128;             // output columns of this wave
  constexpr int kPitch = kWaveCols * 2 + 16;               // patch row in bytes: 16-byte aligned, rows 4 banks apart
  constexpr int kLanesPerRow = kWaveCols / 8;              // 16-byte pieces of a patch row
  constexpr int kRowsPerStore = 64 / kLanesPerRow;
  char* const patch = smem + wave * (32 * kPitch);
  const int half = lane >> 5;
  // One pass of fragment j through the patch: value(blk, v) is the number for patch column
  // blk*32 + 8*(v/4) + 4*half + v%4; the patch then leaves for dst[row, col0 + ...], columns
  // from col_end on are not stored.
  auto pass = [&](int j, auto value, uint16_t* dst, int ld, int col0, int col_end) {
    char* const prow = patch + (lane & 31) * kPitch;
#pragma unroll
    for (int blk = 0; blk < kWaveCols / 32; ++blk)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        uint2 pk;
        pk.x = pack_bf16x2(value(blk, 4 * g), value(blk, 4 * g + 1));
        pk.y = pack_bf16x2(value(blk, 4 * g + 2), value(blk, 4 * g + 3));
        *(uint2*)(prow + (blk * 32 + 8 * g + 4 * half) * 2) = pk;
      }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");  // keep the patch writes before the reads below
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
    for (int t = 0; t < 32 / kRowsPerStore; ++t) {
      const int r = t * kRowsPerStore + lane / kLanesPerRow, piece = lane % kLanesPerRow;
      const uint4 v = *(const uint4*)(patch + r * kPitch + piece * 16);
      const int row = row0 + wm * 32 * XF + j * 32 + r;
      const int col = col0 + piece * 8;  // row lengths are multiples of 8
      if (row < row_end && col < col_end) *(uint4*)(dst + (size_t)row * ld + col) = v;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");  // ... and the reads before the next pass's writes
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  };
  auto rounded = [](float v) { return __uint_as_float(pack_bf16x2(v, 0.f) << 16); };  // the bf16 value that is stored
  const int out0 = n0 + wn * kWaveCols;
  if constexpr (EPI == EPI_ACCUM) {
    // fp32 read-modify-write: one 32 x 32 block at a time through the patch (128-byte rows), so that
    // every row of the block is one whole line of the fp32 matrix
    constexpr int kPitchF = 32 * 4 + 16;
    char* const patchf = smem + wave * (32 * kPitchF);
#pragma unroll
    for (int j = 0; j < XF; ++j)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        char* const prow = patchf + (lane & 31) * kPitchF;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const float4 v = {acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]};
          *(float4*)(prow + (8 * g + 4 * half) * 4) = v;
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          const int r = t * 8 + (lane >> 3), piece = lane & 7;
          const float4 v = *(const float4*)(patchf + r * kPitchF + piece * 16);
          const int row = row0 + wm * 32 * XF + j * 32 + r;
          const int col = n0 + wn * 128 + i * 32 + piece * 4;  // row lengths are multiples of 8
          if (row < row_end && col < a.n_out) {
            float4* const dst = (float4*)(a.Cacc + (size_t)row * a.n_out + col);
            float4 c = *dst;
            c.x += v.x;
            c.y += v.y;
            c.z += v.z;
            c.w += v.w;
            *dst = c;
          }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      }
    return;
  }
#pragma unroll
  for (int j = 0; j < XF; ++j) {
    if constexpr (EPI == EPI_SWIGLU) {
      pass(j, [&](int q, int v) { return silu_fast(acc[2 * q][j][v]) * acc[2 * q + 1][j][v]; }, a.C, a.n_out, out0,
           a.n_out);
    } else if constexpr (EPI == EPI_SWIGLU_KEEP) {
      pass(j, [&](int q, int v) { return acc[2 * q][j][v]; }, a.Z, a.z_cols, out0, a.n_out);
      pass(j, [&](int q, int v) { return acc[2 * q + 1][j][v]; }, a.Z, a.z_cols, a.up_row0 + out0,
           a.up_row0 + a.n_out);
      pass(j, [&](int q, int v) { return silu_fast(rounded(acc[2 * q][j][v])) * rounded(acc[2 * q + 1][j][v]); },
           a.C, a.n_out, out0, a.n_out);
    } else if constexpr (EPI == EPI_GELU_KEEP) {
      pass(j, [&](int i, int v) { return acc[i][j][v]; }, a.Z, a.z_cols, out0, a.n_out);
      pass(j, [&](int i, int v) { return gelu_fast(rounded(acc[i][j][v])); }, a.C, a.n_out, out0, a.n_out);
    } else if constexpr (EPI == EPI_GELU) {
      pass(j, [&](int i, int v) { return gelu_fast(acc[i][j][v]); }, a.C, a.n_out, out0, a.n_out);
    } else {
      pass(j, [&](int i, int v) { return acc[i][j][v]; }, a.C, a.n_out, out0, a.n_out);
    }
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
template <int EPI, int MODE, bool GATHER>
__global__ __launch_bounds__(256, 1) void gemm_mfma_kernel(MfmaArgs a) {
#if defined(__HIP_DEVICE_COMPILE__)  // the host pass only needs the launch stub, not the gfx950 builtins
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  constexpr int BN_OUT = (EPI == EPI_SWIGLU || EPI == EPI_SWIGLU_KEEP) ? BN / 2 : BN;
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
      if (rows > 192) gemm_tile<EPI, 4, MODE, GATHER>(a, smem, slot, row0, row_end, n0);
      else if (rows > 128) gemm_tile<EPI, 3, MODE, GATHER>(a, smem, slot, row0, row_end, n0);
      else if (rows > 64) gemm_tile<EPI, 2, MODE, GATHER>(a, smem, slot, row0, row_end, n0);
      else gemm_tile<EPI, 1, MODE, GATHER>(a, smem, slot, row0, row_end, n0);
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

constexpr int kMaxDevices = 64;

template <int EPI, int MODE = MODE_NT, bool GATHER = false>
int32_t launch_mfma(const MfmaArgs& a, hipStream_t st) {
  static_assert(!GATHER || MODE == MODE_NN, "the gather is part of the forward's first GEMM only");
  void (*kern)(MfmaArgs) = gemm_mfma_kernel<EPI, MODE, GATHER>;
  // per device: the LDS attribute is set and the CU count read on the first launch there (both
  // idempotent, so two threads racing through the set-up do the same thing twice)
  static std::atomic<int> workgroups_of_device[kMaxDevices];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return LZ_EHIP;
  int n_workgroups = workgroups_of_device[dev].load(std::memory_order_acquire);
  if (n_workgroups == 0) {
    if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes) !=
        hipSuccess)
      return LZ_EHIP;
    int cus = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return LZ_EHIP;
    n_workgroups = cus >= 8 ? cus / 8 * 8 : 8;  // one per CU (the LDS a workgroup takes allows no more)
    workgroups_of_device[dev].store(n_workgroups, std::memory_order_release);
  }
  hipLaunchKernelGGL(kern, dim3(n_workgroups), dim3(256), kLdsBytes, st, a);
  return lz::launch_status();
}

}  // namespace
