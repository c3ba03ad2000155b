// Grouped bf16 GEMM on the gfx950 matrix cores and the row-tile table it draws its work from;
// shared by the forward and the backward translation units (device code, not part of the C ABI).
//
//   C[rows of a slot, n] = epi( sum_k A(row, k) * W[slot](n, k) )
//
// Persistent kernel, one workgroup per CU, drawing 256x256 tiles from its XCD's queue.  4 waves
// in 2x2, each wave a 128x128 patch = 8x8 v_mfma_f32_16x16x32_bf16 accumulators (fp32, 256
// AGPRs).  With every CU busy the chip is power-limited, and an MFMA-only loop of this shape
// sustains 15 % more flops than one of v_mfma_f32_32x32x16_bf16 (2.03 against 1.76 PFLOP/s on
// random operands; at a quarter of the CUs both reach the nominal rate).  Operand tiles are
// streamed HBM -> LDS with 16-byte buffer loads that write LDS
// directly, through LDS stages of 64 k (two for the activation tile, three for the weight tile:
// all 160 KiB); fragment reads are software pipelined over two register sets.  An operand may be k-contiguous ([row, k]: 256 tile rows of 128 B, read with
// ds_read_b128) or k-major ([k, column]: 64 k-rows of 512 B, read with the transposing
// ds_read_b64_tr_b16); see the MODE_* list below.  The XOR swizzles that keep the fragment
// reads free of bank conflicts are applied on the global-address side, because a direct-to-LDS
// load fixes the LDS side to lane order.  Buffer descriptors bound every load, so ragged tiles
// cannot fault.  The MFMA takes the weight fragment as its row operand, which leaves each lane
// with 4 consecutive output columns per accumulator group; the epilogue regroups them through
// a per-wave LDS patch into whole 128-byte lines.  For SwiGLU the weight tile interleaves
// 32-wide fragments of the gate and the up projection, so the gate and up values of one output
// element sit in the same lane and register index of two accumulators.
#pragma once
#include "lz_common.h"
#include <atomic>
#include <type_traits>

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;

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
constexpr int kATile = BM * kRowBytes, kWTile = BN * kRowBytes;  // 32 KiB each
// LDS map: two activation stages, then a ring of three weight stages (its loads get two K steps
// to land); together all of the CU's 160 KiB
constexpr int kWStages = 3;
constexpr int kLdsBytes = 2 * kATile + kWStages * kWTile;
__device__ __forceinline__ constexpr int a_stage_off(int s) { return s * kATile; }
__device__ __forceinline__ constexpr int w_stage_off(int w) { return 2 * kATile + w * kWTile; }

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
//   MODE_TN  A [k, m], W [k, n], a different k range for every slot (the weight gradients)
//   MODE_TN_WIDE  the same when an operand may span more than 4 GiB inside one slot (64-bit
//            arithmetic where MODE_TN rebuilds its buffer descriptors for a K step)
// A k-major operand tile lies in LDS as 64 k-rows of 256 columns (512 B each) and is read with
// ds_read_b64_tr_b16, which hands every lane four k-values of one column: the 16 lanes of a
// group supply the addresses of 4 k-rows x 4 column quads, and lane i receives column i of the
// group's 16 at those four k.  Two such reads give the lane the same 8 consecutive k of its
// column that a ds_read_b128 gives it from a k-contiguous tile, so the MFMAs and the epilogue
// do not change.
enum { MODE_NT = 0, MODE_NN = 1, MODE_TN = 2, MODE_TN_WIDE = 3 };
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

// The same load with an MFMA between the write of M0 and the load: the MFMA stands in for the wait
// state the hardware wants there, and the three instructions fit the gap between two MFMAs.
__device__ __forceinline__ void mfma_then_load16_to_lds(f32x4& acc, const bf16x8& w, const bf16x8& x, i32x4 rsrc,
                                                        uint32_t lds_base, int voffset, int soffset) {
  asm volatile("s_mov_b32 m0, %3\n\tv_mfma_f32_16x16x32_bf16 %0, %1, %2, %0\n\tbuffer_load_dwordx4 %4, %5, %6 offen lds"
               : "+a"(acc)
               : "v"(w), "v"(x), "s"(lds_base), "v"(voffset), "s"(rsrc), "s"(soffset)
               : "memory");
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

// 16-byte piece p (8 columns) of k-row kr of a k-major tile lives at piece position p ^ swz_kmajor(kr)
// of its 512-byte LDS row.  A transposing read is served 32 lanes at a time: two lane groups, each
// touching 4 consecutive k-rows (kr % 4 = 0..3) at the same 32 bytes (one 16-column fragment), the
// two groups 8 k-rows apart.  Bits 2-3 of the key move the four k-rows of a group into four
// different quarters of the banks, bit 1 moves the second group's fragments 32 bytes on, so the
// eight 32-byte runs fall into eight different bank groups.
__device__ __forceinline__ int swz_kmajor(int kr) { return ((kr & 3) << 2) | (((kr >> 3) & 1) << 1); }

// One output tile of 64*XF rows x 256 columns n of the weight operand W(n, k) ("weight rows"
// below, whichever way W lies in memory).  XF = 32-row activation fragments per wave: the 2x2 waves each own (32*XF) x 128 of the tile, so a slot's ragged last tile costs
// MFMAs and activation loads only for its rows rounded up to 64.
template <int EPI, int XF, int MODE, bool GATHER>
__device__ __forceinline__ void gemm_tile(const MfmaArgs& a, char* smem, int slot, int row0, int row_end, int n0) {
  constexpr bool TA = MODE == MODE_TN || MODE == MODE_TN_WIDE, TB = MODE != MODE_NT;  // k-major left / right operand
  constexpr bool kGated = EPI == EPI_SWIGLU || EPI == EPI_SWIGLU_KEEP;
  constexpr int KS = BK / 32;             // 32-wide MFMA slices per stage
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
  // MODE_TN, MODE_TN_WIDE: the contraction ends with the slot's last row, wherever in a K step that
  // is, so the descriptors are rebuilt for every K step (base advanced by whole steps, extent =
  // what is left of the slot); in 64-bit arithmetic where a slot's rows may cover more than 4 GiB
  [[maybe_unused]] unsigned long long a_bytes = 0, w_bytes = 0, stepA64 = 0, stepW64 = 0;
  if constexpr (TA) {
    // The descriptors start at the slot's first row and this tile's first column and end with
    // the slot's last row: the rows of the last, partial K step that belong to the next slot
    // read as zero.
    long long s0, s1;
    clip_slot(a.slot_offsets, slot, a.k_rows, &s0, &s1);
    // (the offsets are int32 values read through the vector memory path: tell the compiler that they are
    // the same in every lane, the descriptors built from them are scalar operands)
    s0 = __builtin_amdgcn_readfirstlane((int)s0);
    K = __builtin_amdgcn_readfirstlane(int(s1 - s0));
    const int m0 = row0 - slot * a.rows_per_slot;
    tileA = a.A + (size_t)s0 * a.lda + m0;
    tileW = a.W + (size_t)s0 * a.ldw + n0;
    a_bytes = K > 0 ? ((unsigned long long)K * (unsigned)a.lda - (unsigned)m0) * 2ull : 0ull;
    w_bytes = K > 0 ? ((unsigned long long)K * (unsigned)a.ldw - (unsigned)n0) * 2ull : 0ull;
    stepA64 = 64ull * (unsigned)a.lda * 2ull;
    stepW64 = 64ull * (unsigned)a.ldw * 2ull;
    a_extent = (uint32_t)a_bytes;  // MODE_TN: the host checked that they fit; MODE_TN_WIDE: unused, see issue()
    w_extent = (uint32_t)w_bytes;
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
  // piece l%32, which must hold logical piece (l%32) ^ swz_kmajor(k-row).
  auto voff_kmajor = [&](int i, int ld, int col0) {
    const int kr = (wave * 8 + i) * 2 + (lane >> 5);
    const int piece = (lane & 31) ^ swz_kmajor(kr);
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
      const int piece = (lane & 31) ^ swz_kmajor(kr);
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

  // ---- fragment read addresses.  A fragment is 16 rows (of the activation tile, or weight rows) x
  // the 32 k of a slice; lane l holds row l%16, the 8 consecutive k of chunk l/16 (the operand
  // layout of v_mfma_f32_16x16x32_bf16).  k-contiguous tile: one ds_read_b128 at row l%16, logical
  // chunk 4*slice + l/16 of the stage's 8.
  constexpr int NA = 2 * XF;  // activation fragments per wave (16 rows each)
  constexpr int NW = 8;       // weight fragments per wave (16 weight rows each)
  int fragoff[KS];
  {
    const int r = lane & 15;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) fragoff[ks] = r * kRowBytes + (((ks * 4 + (lane >> 4)) ^ swz(r)) << 4);
  }
  const int xbase = wm * 32 * XF * kRowBytes;               // this wave's activation rows
  const int wbase = wn * 128 * kRowBytes;                   // this wave's 128 weight rows
  // k-major tiles: lane 16g + q supplies the address of k-row 8g + q/4 of the 32-wide slice, column
  // quad q%4 of the fragment's 16 columns; the transposing read hands lane 16g + i column i at those
  // four k-rows, a second read 4 k-rows on completes the lane's 8 consecutive k.
  int tfo[2];  // byte offset inside a stage's k-major tile for fragment 0 (and its second piece position), slice 0
  {
    const int g = lane >> 4, q = lane & 15;
    const int kr = 8 * g + (q >> 2);
    // fragment f = pieces 2f, 2f+1 of the k-row; the swizzle key (even) is added by XOR per fragment below
    tfo[0] = kr * 512 + ((q & 1) << 3) + (((q >> 1) & 1) << 4);
    tfo[1] = swz_kmajor(kr);
  }
  auto kmajor_addr = [&](int frag16) {  // fragment frag16 (0..15) of the 256-column tile, slice 0
    return tfo[0] + ((((frag16 << 1) ^ tfo[1]) & 31) << 4);
  };
  auto read_kmajor = [&](const char* p) {
    const i16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) i16x4*)p);
    const i16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) i16x4*)(p + 4 * 512));
    return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
  };
  auto frag_x = [&](int stage, int ks, int j) {
    const char* base = smem + a_stage_off(stage);
    if constexpr (TA) return read_kmajor(base + ks * 32 * 512 + kmajor_addr(NA * wm + j));
    else return *(const bf16x8*)(base + xbase + j * 16 * kRowBytes + fragoff[ks]);
  };
  auto frag_w = [&](int stage, int ks, int i) {
    const char* base = smem + w_stage_off(stage);
    if constexpr (TB) return read_kmajor(base + ks * 32 * 512 + kmajor_addr(NW * wn + i));
    else return *(const bf16x8*)(base + wbase + i * 16 * kRowBytes + fragoff[ks]);
  };

  f32x4 acc[NW][NA];
#pragma unroll
  for (int i = 0; i < NW; ++i)
#pragma unroll
    for (int j = 0; j < NA; ++j)
#pragma unroll
      for (int v = 0; v < 4; ++v) acc[i][j][v] = 0.f;

  // ---- main loop: K steps of 64 columns; step kt reads activation stage kt%2 and weight stage kt%3.
  // One barrier per step, placed after the last reads of the step's stages have been issued: past it
  // nobody reads them any more, so the activation loads of step kt+2 and the weight loads of step
  // kt+3 can start into them, and the next step's stages (whose loads every wave has waited for
  // before the barrier) can be read.
  //
  // A step's loads are not issued in one burst: a wave that issues a burst stands still until the
  // texture unit has accepted it, and the MFMA pipe with it.  The activation loads go out during
  // the unit after barrier kt (they must have landed by the next barrier); the weight loads, which
  // have a whole step longer, are spread over the three units that follow.
  const int k_steps = (K + BK - 1) / BK;
  constexpr int kLoads = kLoadsW + kLoadsX;
  // Loads [q0, q1) of a wave's 16 per step: the activation loads (q < kLoadsX) of K step a_step into
  // activation stage a_stage, the weight loads of K step w_step into weight stage w_stage.
  // with_mfma: an MFMA (accumulator, weight and activation fragment) to issue together with load q0
  auto issue = [&](int a_stage, int a_step, int w_stage, int w_step, int q0, int q1, f32x4* with_mfma = nullptr,
                   const bf16x8* mw = nullptr, const bf16x8* mx = nullptr) {
    // a step past the end of K is "loaded" through a zero-length descriptor: no memory traffic
    const bool real_a = a_step < k_steps, real_w = w_step < k_steps;
    i32x4 wa = real_a ? wordsA : wordsNull, wb = real_w ? wordsB : wordsNull;
    if constexpr (MODE == MODE_TN) {
      const uint32_t offA = (uint32_t)a_step * (uint32_t)stepA64, offW = (uint32_t)w_step * (uint32_t)stepW64;
      // bytes left of the slot: a step that begins inside the slot begins inside both extents (the
      // tile's first column lies inside the operand's row)
      const uint32_t leftA = real_a ? a_extent - offA : 0u, leftW = real_w ? w_extent - offW : 0u;
      wa = rsrc_words((const char*)tileA + offA, leftA);
      wb = rsrc_words((const char*)tileW + offW, leftW);
    } else if constexpr (MODE == MODE_TN_WIDE) {
      const unsigned long long offA = (unsigned long long)(unsigned)a_step * stepA64;
      const unsigned long long offW = (unsigned long long)(unsigned)w_step * stepW64;
      const unsigned long long leftA = a_bytes > offA ? a_bytes - offA : 0ull;
      const unsigned long long leftW = w_bytes > offW ? w_bytes - offW : 0ull;
      wa = rsrc_words((const char*)tileA + offA, leftA > 0xFFFFFFFFull ? 0xFFFFFFFFu : (uint32_t)leftA);
      wb = rsrc_words((const char*)tileW + offW, leftW > 0xFFFFFFFFull ? 0xFFFFFFFFu : (uint32_t)leftW);
    }
    const uint32_t ldsX = lds0 + a_stage_off(a_stage), ldsW = lds0 + w_stage_off(w_stage);
#pragma unroll
    for (int q = q0; q < q1; ++q) {
      const bool isx = q < kLoadsX;
      const i32x4 words = isx ? wa : wb;
      const uint32_t lds = isx ? ldsX + (wave * kLoadsX + q) * 1024 : ldsW + (wave * kLoadsW + q - kLoadsX) * 1024;
      const int voff = isx ? voffX[q < kLoadsX ? q : 0] : voffW[q >= kLoadsX ? q - kLoadsX : 0];
      const int soff = isx ? a_step * stepA : w_step * stepW;
      if (with_mfma != nullptr && q == q0) mfma_then_load16_to_lds(*with_mfma, *mw, *mx, words, lds, voff, soff);
      else load16_to_lds(words, lds, voff, soff);
    }
  };
  // A stage is consumed as four units: 32-wide slice s (0, 1) x half hw (0, 1) of the wave's weight
  // fragments.  Unit (s, hw) needs the NA activation fragments of slice s and the weight fragments
  // 4 hw .. 4 hw + 3 of slice s: 4 NA MFMAs.  Two register sets of each kind alternate (activation
  // fragments by slice, weight fragments by unit), so that the ds_reads of the next unit are in
  // flight while the MFMAs of the current one run.
  //
  // The MFMAs are written as assembly with the accumulator tied to the destination (left to the
  // register allocator, this MFMA shape gets a destination different from its accumulator input,
  // and with all 256 accumulator registers live the copies that needs go through VGPRs: 3.5 moves
  // per MFMA).  A volatile asm also pins the order: memory operations do not cross it, so the
  // fragment reads and direct-to-LDS loads below issue exactly where they are written, one read per
  // MFMA from the start of a unit (the next unit waits on them), the loads spread over the unit.
  constexpr int kMfmas = 4 * NA;                             // MFMAs per unit
  // Loads [0, kAfterBarrier) go out in the unit after the barrier, [kAfterBarrier, kL1), [kL1, kL2) and
  // [kL2, kLoads) in the three units of the next step: the 8 weight loads as 2 + 3 + 3.
  // (Measured on configs 2-4: with the weight loads bunched behind the activation loads, 4 in the unit after
  // the barrier and 4 in the next, the second GEMM is 3-5 % slower and the first level; all 16 after the barrier
  // costs both 5-7 %; other even spreads, also with half of the activation loads a unit later, are within 1 %.
  // Spreading a unit's loads over the whole unit beats its first half or quarter by 1-3 %; a barrier moved up
  // to just behind the stage's last reads, with all loads after it, is level.)
  constexpr int kAfterBarrier = kLoadsX, kL1 = kLoadsX + 2, kL2 = kLoadsX + 5;
  bf16x8 xf[2][NA], wf[2][4];
  // r-th fragment read of a unit's look-ahead: the weight fragments of unit (s, hw) go into set ws,
  // the activation fragments [j0, j1) of slice xs into set xset; with x_first in the order of first
  // use by the MFMAs (weight fragment 0, the activation fragments, weight fragments 1..3).
  auto read_r = [&](int r, int w_stage, int s, int hw, int ws, int x_stage, int xs, int xset, int j0,
                    int j1, bool x_first) {
    const int NX = j1 - j0;
    int wi = -1, xj = -1;
    if (x_first) {
      if (r == 0) wi = 0;
      else if (r <= NX) xj = j0 + r - 1;
      else wi = r - NX;
    } else {
      if (r < 4) wi = r;
      else xj = j0 + r - 4;
    }
    if (wi >= 0) wf[ws][wi] = frag_w(w_stage, s, 4 * hw + wi);
    else xf[xset][xj] = frag_x(x_stage, xs, xj);
  };
  // One unit: the MFMAs of weight half hw on the sets (xset, ws), interleaved with the reads for the
  // next unit and the loads [q0, q1) of the activation and weight steps named by the ld_ arguments.
  auto unit = [&](int hw, int xset, int ws, int w_stage, int ns, int nhw, int nws, int x_stage, int xs, int nxset, int j0,
                  int j1, bool x_first, int ld_a_stage, int ld_a_step, int ld_w_stage, int ld_w_step, int q0, int q1) {
    const int NR = 4 + (j1 - j0), NL = q1 - q0;
#pragma unroll
    for (int m = 0; m < kMfmas; ++m) {
      if (m < NR) read_r(m, w_stage, ns, nhw, nws, x_stage, xs, nxset, j0, j1, x_first);
      const int l0 = q0 + (NL * m) / kMfmas, l1 = q0 + (NL * (m + 1)) / kMfmas;
      if (l1 > l0) {
        issue(ld_a_stage, ld_a_step, ld_w_stage, ld_w_step, l0, l1, &acc[4 * hw + m / NA][m % NA], &wf[ws][m / NA],
              &xf[xset][m % NA]);
      } else {
        issue(ld_a_stage, ld_a_step, ld_w_stage, ld_w_step, l0, l1);
        asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0"
                     : "+a"(acc[4 * hw + m / NA][m % NA])
                     : "v"(wf[ws][m / NA]), "v"(xf[xset][m % NA]));
      }
    }
  };
  constexpr int kHalf = NA / 2;

  constexpr int D = kWStages;
  if constexpr (GATHER) {
    issue(0, 0, 0, 0, kLoadsX, kLoads);                  // the weight tile of step 0 does not need the row map
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
    issue(0, 0, 0, 0, 0, kLoadsX);
  } else {
    issue(0, 0, 0, 0, 0, kLoads);
  }
  // in flight when the loop starts: the weights of step 1 and what the unit after a barrier issues
  // (the activations of step 1); the units of step 0 issue the weight loads of step 2
  constexpr int kAhead = kLoadsW + kAfterBarrier;
  issue(1, 1, 1, 1, kLoadsX, kLoads);
  issue(1, 1, 2, 2, 0, kAfterBarrier);
  // s_waitcnt with only vmcnt set (bits [3:0] and [15:14]): the later steps' loads may still be in flight
  __builtin_amdgcn_s_waitcnt(0x0F70 | (kAhead & 15) | ((kAhead >> 4) << 14));
  __syncthreads();
#pragma unroll
  for (int r = 0; r < 4 + NA; ++r) read_r(r, 0, 0, 0, 0, 0, 0, 0, 0, NA, true);  // unit (0, 0) of stage 0

  // One K step on activation stage `as` and weight stage `wst`.  The loop below is unrolled so that
  // both are compile-time constants and every LDS address of the step folds into an instruction's
  // offset field or a literal (otherwise a dozen address additions per step queue up at the head of
  // the loop and in front of the loads, and the MFMA pipe waits for them).
  // Loads: after barrier kt the activations of step kt+2 go into the stage just read; the weights
  // of step kt+3 follow in the units of step kt+1, into the weight stage freed by barrier kt.  A
  // step's weight loads are thus still in flight at the next barrier, and its wait leaves the
  // newest kLoadsW loads out.
  auto k_step = [&](int kt, auto as_c, auto wst_c) {
    constexpr int as = decltype(as_c)::value, wst = decltype(wst_c)::value;
    constexpr int as_next = as ^ 1, wst_next = (wst + 1) % D, wst_prev = (wst + D - 1) % D;
    // unit (0, 0) runs; weight fragments of (0, 1), first half of slice 1's activation fragments
    unit(0, 0, 0, wst, 0, 1, 1, as, 1, 1, 0, kHalf, false, as_next, kt + 1, wst_prev, kt - 1 + D, kAfterBarrier, kL1);
    // unit (0, 1) runs; weight fragments of (1, 0), the rest of slice 1's activation fragments
    unit(1, 0, 1, wst, 1, 0, 0, as, 1, 1, kHalf, NA, false, as_next, kt + 1, wst_prev, kt - 1 + D, kL1, kL2);
    // unit (1, 0) runs; weight fragments of (1, 1): the last reads of this stage
    unit(0, 1, 0, wst, 1, 1, 1, as, 1, 1, 0, 0, false, as_next, kt + 1, wst_prev, kt - 1 + D, kL2, kLoads);
    // this wave's loads of the next step are in LDS ...
    __builtin_amdgcn_s_waitcnt(0x0F70 | kLoadsW);
    __syncthreads();  // ... everyone's are; nobody reads these stages any more
    // unit (1, 1) runs; all of unit (0, 0) of the next step
    unit(1, 1, 1, wst_next, 0, 0, 0, as_next, 0, 0, 0, NA, true, as, kt + 2, wst, kt + D, 0, kAfterBarrier);
  };
  {
    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;
    using I2 = std::integral_constant<int, 2>;
    int kt = 0;
    for (; kt + 5 < k_steps; kt += 6) {
      k_step(kt, I0{}, I0{});
      k_step(kt + 1, I1{}, I1{});
      k_step(kt + 2, I0{}, I2{});
      k_step(kt + 3, I1{}, I0{});
      k_step(kt + 4, I0{}, I1{});
      k_step(kt + 5, I1{}, I2{});
    }
    if (kt < k_steps) k_step(kt, I0{}, I0{});
    if (kt + 1 < k_steps) k_step(kt + 1, I1{}, I1{});
    if (kt + 2 < k_steps) k_step(kt + 2, I0{}, I2{});
    if (kt + 3 < k_steps) k_step(kt + 3, I1{}, I0{});
    if (kt + 4 < k_steps) k_step(kt + 4, I0{}, I1{});
  }
  // the compiler does not know that the assembly above is MFMAs: keep their results away from the
  // VALU reads of the epilogue for the wait states such reads need (at most 18)
  asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
  // The trailing loads (steps past the end of K, zero-length descriptor) still write zeros into
  // their stages, and each wave only waits for its own: one of those stages is activation stage 0,
  // where the epilogue patches of the other waves lie.  Drain this wave's, then wait
  // until every wave has drained its own, before anybody writes a patch.
  __builtin_amdgcn_s_waitcnt(0x0F70);
  __syncthreads();

  // ---- epilogue.  acc[i][j] is the 16x16 block (weight fragment i) x (activation fragment j);
  // lane l holds activation row j*16 + l%16 and the 4 consecutive weight rows i*16 + 4*(l/16) + 0..3
  // -> 4 consecutive output columns.  Stored straight from there, a wave store would touch 16
  // rows with 8 bytes each; such partial-line writes cost the second GEMM 10 % (timed with the
  // stores removed).  So 32 rows at a time go through a per-wave LDS patch (the stages are dead by
  // now; LDS serves a wave's accesses in order) and leave as 16 bytes per lane, whole 128-byte
  // lines at a time.
  constexpr int kWaveCols = kGated ? 64 : 128;             // output columns of this wave
  constexpr int kPitch = kWaveCols * 2 + 16;               // patch row in bytes: 16-byte aligned, rows 4 banks apart
  constexpr int kLanesPerRow = kWaveCols / 8;              // 16-byte pieces of a patch row
  constexpr int kRowsPerStore = 64 / kLanesPerRow;
  char* const patch = smem + wave * (32 * kPitch);
  const int quad = lane >> 4;
  // One pass of the 32 activation rows [32 jj, 32 jj + 32) through the patch: value(c, h, v) is the
  // number for patch row 16 h + l%16, patch column 16 c + 4 quad + v; the patch then leaves for
  // dst[row, col0 + ...], columns from col_end on are not stored.
  auto pass = [&](int jj, auto value, uint16_t* dst, int ld, int col0, int col_end) {
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      char* const prow = patch + (16 * h + (lane & 15)) * kPitch;
#pragma unroll
      for (int c = 0; c < kWaveCols / 16; ++c) {
        uint2 pk;
        pk.x = pack_bf16x2(value(c, h, 0), value(c, h, 1));
        pk.y = pack_bf16x2(value(c, h, 2), value(c, h, 3));
        *(uint2*)(prow + (c * 16 + 4 * quad) * 2) = pk;
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");  // keep the patch writes before the reads below
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
    for (int t = 0; t < 32 / kRowsPerStore; ++t) {
      const int r = t * kRowsPerStore + lane / kLanesPerRow, piece = lane % kLanesPerRow;
      const uint4 v = *(const uint4*)(patch + r * kPitch + piece * 16);
      const int row = row0 + wm * 32 * XF + jj * 32 + r;
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
    for (int jj = 0; jj < XF; ++jj)
#pragma unroll
      for (int ii = 0; ii < 4; ++ii) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          char* const prow = patchf + (16 * h + (lane & 15)) * kPitchF;
#pragma unroll
          for (int c = 0; c < 2; ++c) {
            const f32x4& blk = acc[2 * ii + c][2 * jj + h];
            const float4 v = {blk[0], blk[1], blk[2], blk[3]};
            *(float4*)(prow + (16 * c + 4 * quad) * 4) = v;
          }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          const int r = t * 8 + (lane >> 3), piece = lane & 7;
          const float4 v = *(const float4*)(patchf + r * kPitchF + piece * 16);
          const int row = row0 + wm * 32 * XF + jj * 32 + r;
          const int col = n0 + wn * 128 + ii * 32 + piece * 4;  // row lengths are multiples of 8
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
  // Gated weights: the tile's 32-column groups alternate gate and up columns, so of a wave's eight
  // 16-wide weight fragments 0, 1, 4, 5 are gate columns and i + 2 holds the up columns of the same
  // outputs; output column block c (16 wide) of the wave comes from fragment 4 (c/2) + c%2.
  auto gate_frag = [](int c) { return 4 * (c >> 1) + (c & 1); };
#pragma unroll
  for (int jj = 0; jj < XF; ++jj) {
    if constexpr (EPI == EPI_SWIGLU) {
      pass(jj, [&](int c, int h, int v) { return silu_fast(acc[gate_frag(c)][2 * jj + h][v]) * acc[gate_frag(c) + 2][2 * jj + h][v]; },
           a.C, a.n_out, out0, a.n_out);
    } else if constexpr (EPI == EPI_SWIGLU_KEEP) {
      pass(jj, [&](int c, int h, int v) { return acc[gate_frag(c)][2 * jj + h][v]; }, a.Z, a.z_cols, out0, a.n_out);
      pass(jj, [&](int c, int h, int v) { return acc[gate_frag(c) + 2][2 * jj + h][v]; }, a.Z, a.z_cols, a.up_row0 + out0,
           a.up_row0 + a.n_out);
      pass(jj, [&](int c, int h, int v) {
             return silu_fast(rounded(acc[gate_frag(c)][2 * jj + h][v])) * rounded(acc[gate_frag(c) + 2][2 * jj + h][v]);
           },
           a.C, a.n_out, out0, a.n_out);
    } else if constexpr (EPI == EPI_GELU_KEEP) {
      pass(jj, [&](int c, int h, int v) { return acc[c][2 * jj + h][v]; }, a.Z, a.z_cols, out0, a.n_out);
      pass(jj, [&](int c, int h, int v) { return gelu_fast(rounded(acc[c][2 * jj + h][v])); }, a.C, a.n_out, out0, a.n_out);
    } else if constexpr (EPI == EPI_GELU) {
      pass(jj, [&](int c, int h, int v) { return gelu_fast(acc[c][2 * jj + h][v]); }, a.C, a.n_out, out0, a.n_out);
    } else {
      pass(jj, [&](int c, int h, int v) { return acc[c][2 * jj + h][v]; }, a.C, a.n_out, out0, a.n_out);
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
