// The flexible token dispatcher (Algorithm 1, Sec. 4.2) for all source ranks at once.
//
// Four kernels on one stream, no host synchronisation, no order-dependent atomics:
//   count    each wave owns a chunk of <= 128 consecutive pairs of ONE source rank and
//            histograms their expert ids with LDS atomics (counts commute)
//   schedule one workgroup per expert scans the chunk histograms into per-(expert, rank) list
//            positions and evaluates the algorithm's counts in exact integers, in LDS; one
//            more workgroup then cuts every (expert, rank) receive list over that rank's
//            replicas and scans the slot sizes
//   place    each wave revisits its chunk; a pair's position in its (expert, source rank)
//            list is chunk base + ordered rank inside the chunk (wave ballots, one per
//            distinct expert), which fixes destination rank, slot and row
#include <mutex>

#include "lz_common.h"

namespace {

constexpr int kChunk = 128;          // pairs per wave-chunk
constexpr int kWavesPerBlock = 4;
constexpr int kSchedThreads = 1024;
constexpr int kExpertThreads = 256;

struct PlanTables {
  // per chunk
  int32_t* chunkcnt;   // [nch, E]
  int32_t* chunkbase;  // [nch, E]  position of the chunk's first pair of e in its (e, rank) list
  int32_t* chunkflag;  // [nch]
  // per (expert, rank)
  int32_t* Tej;        // [E, N]
  int32_t* R;          // [E, N]
  int32_t* L;          // [E, N]  pairs kept locally
  int32_t* Pres;       // [E, N]  residual capacity
  int32_t* O;          // [E, N]  overflow
  int32_t* recv;       // [E, N]
  int32_t* ejstart;    // [E, N]  index of the first slot of e in rank j's sorted slot list
  int32_t* estatus;    // [E]     status bits raised while scheduling expert e
  // per (expert, src, dst)
  int32_t* D;          // [E, N, N]
  int32_t* cumDst;     // [E, N, N+1] prefix of D over dst
  int32_t* preSrc;     // [E, N, N]   prefix of D over src
  // per slot
  int32_t* slot_sorted;  // [S] rank j's slots ordered by (expert, slot id)
  int32_t* slot_pos;     // [S] position of slot s in that order
  size_t total_bytes;
};

__host__ __device__ inline int max_chunks(long long P, int N) { return int((P + kChunk - 1) / kChunk) + N; }

PlanTables carve(void* ws, const lz_shape* s) {
  PlanTables t{};
  const size_t E = s->E, N = s->N, S = size_t(s->N) * s->c;
  const size_t nch = max_chunks((long long)s->T * s->k, s->N);
  char* base = (char*)ws;
  size_t off = 0;
  auto take = [&](size_t n_ints) {
    int32_t* p = (int32_t*)(base + off);
    off += lz::align256(n_ints * sizeof(int32_t));
    return p;
  };
  t.chunkcnt = take(nch * E);
  t.chunkbase = take(nch * E);
  t.chunkflag = take(nch);
  t.Tej = take(E * N);
  t.R = take(E * N);
  t.L = take(E * N);
  t.Pres = take(E * N);
  t.O = take(E * N);
  t.recv = take(E * N);
  t.ejstart = take(E * N);
  t.estatus = take(E);
  t.D = take(E * N * N);
  t.cumDst = take(E * N * (N + 1));
  t.preSrc = take(E * N * N);
  t.slot_sorted = take(S);
  t.slot_pos = take(S);
  t.total_bytes = off;
  return t;
}

// Sanitised batch split and the chunk table derived from it, rebuilt by every workgroup
// (N <= 64 entries).  Returns true if rank_tok_off had to be repaired.
__device__ bool build_split(const int32_t* __restrict__ rank_tok_off, int T, int N, int k,
                            int* s_off, int* s_cf) {
  bool bad = rank_tok_off[0] != 0 || rank_tok_off[N] != T;
  int prev = 0;
  s_off[0] = 0;
  s_cf[0] = 0;
  for (int i = 1; i <= N; ++i) {
    int v = i == N ? T : rank_tok_off[i];
    if (v < prev || v > T) bad = true;
    v = v < prev ? prev : (v > T ? T : v);
    s_off[i] = v;
    const long long pairs = (long long)(v - prev) * k;
    s_cf[i] = s_cf[i - 1] + int((pairs + kChunk - 1) / kChunk);
    prev = v;
  }
  return bad;
}

// chunk b -> its source rank (or -1) and pair range
__device__ __forceinline__ int chunk_range(int b, int N, int k, const int* s_off, const int* s_cf,
                                           long long* p0, long long* p1) {
  if (b >= s_cf[N]) return -1;
  int i = 0;
  while (s_cf[i + 1] <= b) ++i;
  const long long begin = (long long)s_off[i] * k + (long long)(b - s_cf[i]) * kChunk;
  const long long end = (long long)s_off[i + 1] * k;
  *p0 = begin;
  *p1 = begin + kChunk < end ? begin + kChunk : end;
  return i;
}

__global__ __launch_bounds__(256) void count_kernel(const int32_t* __restrict__ ids,
                                                    const int32_t* __restrict__ rank_tok_off, int T,
                                                    int E, int N, int k, PlanTables t,
                                                    int32_t* __restrict__ row_to_pair) {
  __shared__ int s_off[lz::kMaxN + 1], s_cf[lz::kMaxN + 1];
  __shared__ int s_cnt[kWavesPerBlock][lz::kMaxE];
  const int lane = threadIdx.x % lz::kWave, w = threadIdx.x / lz::kWave;
  if (threadIdx.x == 0) build_split(rank_tok_off, T, N, k, s_off, s_cf);
  for (int e = lane; e < E; e += lz::kWave) s_cnt[w][e] = 0;
  __syncthreads();
  const int b = blockIdx.x * kWavesPerBlock + w;
  long long p0 = 0, p1 = 0;
  const int rank = chunk_range(b, N, k, s_off, s_cf, &p0, &p1);
  if (rank < 0) return;
  int flag = 0;
  for (long long p = p0 + lane; p < p1; p += lz::kWave) {
    const int e = ids[p];
    if (e >= 0 && e < E) atomicAdd(&s_cnt[w][e], 1);
    else flag = LZ_PLAN_BAD_EXPERT_ID;
    row_to_pair[p] = -1;  // rows and pairs share the index range [0, P)
  }
  flag = __any(flag) ? LZ_PLAN_BAD_EXPERT_ID : 0;
  // LDS atomics of this wave have completed before its own later LDS reads
  __builtin_amdgcn_wave_barrier();
  for (int e = lane; e < E; e += lz::kWave) t.chunkcnt[(size_t)b * E + e] = s_cnt[w][e];
  if (lane == 0) t.chunkflag[b] = flag;
}

// Algorithm 1 for one expert per workgroup.  Everything an expert needs (N counts, N x N
// assignments) lives in LDS between the phases, so the chain of dependent steps costs barriers,
// not global-memory round trips; the tables the other kernels read are written out once.
__global__ __launch_bounds__(kExpertThreads) void schedule_expert_kernel(
    const int32_t* __restrict__ rank_tok_off, const int32_t* __restrict__ slot_expert, int T, int E,
    int N, int c, int k, PlanTables t, int32_t* __restrict__ Tej_opt, int32_t* __restrict__ D_opt) {
  __shared__ int s_off[lz::kMaxN + 1], s_cf[lz::kMaxN + 1];
  __shared__ int s_R[lz::kMaxN], s_T[lz::kMaxN], s_L[lz::kMaxN], s_P[lz::kMaxN], s_O[lz::kMaxN];
  __shared__ int s_D[lz::kMaxN * lz::kMaxN];
  const int e = blockIdx.x;
  const int tid = threadIdx.x, lane = tid % lz::kWave, w = tid / lz::kWave;
  if (tid == 0) build_split(rank_tok_off, T, N, k, s_off, s_cf);
  __syncthreads();

  // ---- per source rank j (one wave each): positions of the chunks in the (e, j) list, T[e,j],
  // the replicas of e on rank j and the index of their first slot in j's sorted slot list
  for (int j = w; j < N; j += kExpertThreads / lz::kWave) {
    const int b_end = s_cf[j + 1];
    int running = 0;
    for (int b0 = s_cf[j]; b0 < b_end; b0 += lz::kWave) {
      const int b = b0 + lane;
      const int v = b < b_end ? t.chunkcnt[(size_t)b * E + e] : 0;
      int incl = v;
#pragma unroll
      for (int off = 1; off < lz::kWave; off <<= 1) {
        const int n = __shfl_up(incl, off);
        if (lane >= off) incl += n;
      }
      if (b < b_end) t.chunkbase[(size_t)b * E + e] = running + incl - v;
      running += __shfl(incl, lz::kWave - 1);
    }
    int reps = 0, before = 0;
    for (int l0 = 0; l0 < c; l0 += lz::kWave) {
      const int l = l0 + lane;
      const int se = l < c ? slot_expert[j * c + l] : -1;
      reps += __popcll(__ballot(l < c && se == e));
      before += __popcll(__ballot(l < c && se >= 0 && se < e));
    }
    if (lane == 0) {
      const int idx = e * N + j;
      s_T[j] = running;
      s_R[j] = reps;
      t.Tej[idx] = running;
      if (Tej_opt) Tej_opt[idx] = running;
      t.R[idx] = reps;
      t.ejstart[idx] = before;
    }
  }
  __syncthreads();

  // ---- r_e, t_e (Algorithm 1, first two lines); capacity, local share, residual, overflow
  long long re = 0, te = 0;
  for (int j = 0; j < N; ++j) {
    re += s_R[j];
    te += s_T[j];
  }
  if (tid == 0) t.estatus[e] = (te > 0 && re == 0) ? LZ_PLAN_UNCOVERED_EXPERT : 0;
  if (tid < N) {
    const int j = tid;
    long long lo = 0;
    for (int j2 = 0; j2 < j; ++j2) lo += s_R[j2];
    const long long hi = lo + s_R[j];
    const int cap = re > 0 ? int((hi * te) / re - (lo * te) / re) : 0;
    const int mine = s_T[j];
    const int keep = cap < mine ? cap : mine;
    s_L[j] = keep;
    s_P[j] = cap - keep;
    s_O[j] = mine - keep;
    t.L[e * N + j] = keep;
    t.Pres[e * N + j] = cap - keep;
    t.O[e * N + j] = mine - keep;
  }
  __syncthreads();

  // ---- D[e, i, :]: local share on the diagonal, overflow spread by residual capacity
  if (tid < N) {
    const int i = tid, idx = e * N + i;
    long long tot = 0;
    for (int j = 0; j < N; ++j) tot += s_P[j];
    const long long o = s_O[i];
    long long cumP = 0;
    int cumD = 0;
    int32_t* Drow = t.D + (size_t)idx * N;
    int32_t* Crow = t.cumDst + (size_t)idx * (N + 1);
    for (int j = 0; j < N; ++j) {
      int dval;
      if (j == i) {
        dval = s_L[i];
      } else {
        const long long pj = s_P[j];
        dval = (o > 0 && tot > 0) ? int((o * (cumP + pj)) / tot - (o * cumP) / tot) : 0;
        cumP += pj;
      }
      s_D[i * N + j] = dval;
      Drow[j] = dval;
      if (D_opt) D_opt[(size_t)idx * N + j] = dval;
      Crow[j] = cumD;
      cumD += dval;
    }
    Crow[N] = cumD;
  }
  __syncthreads();

  // ---- receive side: prefix over source ranks, recv[e, j]
  if (tid < N) {
    const int j = tid;
    int running = 0;
    for (int i = 0; i < N; ++i) {
      t.preSrc[((size_t)(e * N + i)) * N + j] = running;
      running += s_D[i * N + j];
    }
    t.recv[e * N + j] = running;
  }
}

// Slot order inside every rank, slot sizes (balanced cut of the (e, j) receive list over its
// R[e, j] slots), their exclusive scan, and the status word.  One workgroup.
__global__ __launch_bounds__(kSchedThreads) void schedule_slots_kernel(
    const int32_t* __restrict__ rank_tok_off, const int32_t* __restrict__ slot_expert, int T, int E,
    int N, int c, int k, PlanTables t, int32_t* __restrict__ slot_counts,
    int32_t* __restrict__ slot_offsets, int32_t* __restrict__ status_opt) {
  __shared__ int s_off[lz::kMaxN + 1], s_cf[lz::kMaxN + 1];
  __shared__ int s_status;
  __shared__ int s_scan[kSchedThreads];
  const int tid = threadIdx.x;
  const int S = N * c;
  if (tid == 0) {
    const bool bad = build_split(rank_tok_off, T, N, k, s_off, s_cf);
    s_status = bad ? LZ_PLAN_BAD_RANK_SPLIT : 0;
  }
  __syncthreads();
  {
    int flag = 0;
    for (int b = tid; b < s_cf[N]; b += kSchedThreads) flag |= t.chunkflag[b];
    for (int e = tid; e < E; e += kSchedThreads) flag |= t.estatus[e];
    if (flag) atomicOr(&s_status, flag);
  }
  for (int s = tid; s < S; s += kSchedThreads) {
    const int j = s / c;
    int se = slot_expert[s];
    const bool valid = se >= 0 && se < E;
    if (!valid) {
      se = E;
      atomicOr(&s_status, LZ_PLAN_BAD_EXPERT_ID);
    }
    int pos = 0;
    for (int l = 0; l < c; ++l) {
      const int s2 = j * c + l;
      int se2 = slot_expert[s2];
      if (se2 < 0 || se2 >= E) se2 = E;
      pos += se2 < se || (se2 == se && s2 < s);
    }
    t.slot_pos[s] = pos;
    t.slot_sorted[j * c + pos] = s;
    int cnt = 0;
    if (valid) {
      const int ej = se * N + j;
      const long long m = pos - t.ejstart[ej];
      const long long n = t.recv[ej], reps = t.R[ej];
      cnt = int(((m + 1) * n) / reps - (m * n) / reps);
    }
    slot_counts[s] = cnt;
  }
  __syncthreads();

  // ---- exclusive scan over slot id (each thread owns a run of consecutive slots)
  const int per = (S + kSchedThreads - 1) / kSchedThreads;
  const int first = tid * per;
  int local = 0;
  for (int s = first; s < first + per && s < S; ++s) local += slot_counts[s];
  s_scan[tid] = local;
  __syncthreads();
  for (int off = 1; off < kSchedThreads; off <<= 1) {
    const int add = tid >= off ? s_scan[tid - off] : 0;
    __syncthreads();
    s_scan[tid] += add;
    __syncthreads();
  }
  int running = s_scan[tid] - local;
  for (int s = first; s < first + per && s < S; ++s) {
    slot_offsets[s] = running;
    running += slot_counts[s];
  }
  if (tid == kSchedThreads - 1) slot_offsets[S] = s_scan[tid];
  if (tid == 0 && status_opt) *status_opt = s_status;
}

__global__ __launch_bounds__(256) void place_kernel(const int32_t* __restrict__ ids,
                                                    const int32_t* __restrict__ rank_tok_off, int T,
                                                    int E, int N, int c, int k, PlanTables t,
                                                    const int32_t* __restrict__ slot_offsets,
                                                    int32_t* __restrict__ pair_to_row,
                                                    int32_t* __restrict__ row_to_pair) {
  __shared__ int s_off[lz::kMaxN + 1], s_cf[lz::kMaxN + 1];
  __shared__ int s_run[kWavesPerBlock][lz::kMaxE];
  const int lane = threadIdx.x % lz::kWave, w = threadIdx.x / lz::kWave;
  if (threadIdx.x == 0) build_split(rank_tok_off, T, N, k, s_off, s_cf);
  __syncthreads();
  const int b = blockIdx.x * kWavesPerBlock + w;
  long long p0 = 0, p1 = 0;
  const int i = chunk_range(b, N, k, s_off, s_cf, &p0, &p1);
  if (i < 0) return;
  for (int e = lane; e < E; e += lz::kWave) s_run[w][e] = t.chunkbase[(size_t)b * E + e];
  __builtin_amdgcn_wave_barrier();
  const unsigned long long lower = (1ull << lane) - 1ull;
  const long long P = (long long)T * k;

  for (long long base = p0; base < p1; base += lz::kWave) {
    const long long p = base + lane;
    const bool in = p < p1;
    const int e = in ? ids[p] : -1;
    const bool valid = in && e >= 0 && e < E;
    // ordered rank of this pair among the chunk's pairs of the same expert
    int q = -1;
    unsigned long long todo = __ballot(valid);
    while (todo) {
      const int leader = __ffsll((long long)todo) - 1;
      const int e0 = __shfl(e, leader);
      const unsigned long long same = __ballot(valid && e == e0);
      if (valid && e == e0) q = s_run[w][e0] + __popcll(same & lower);
      __builtin_amdgcn_wave_barrier();
      if (lane == leader) s_run[w][e0] += __popcll(same);
      __builtin_amdgcn_wave_barrier();
      todo &= ~same;
    }
    int row = -1;
    if (valid) {
      const int ei = e * N + i;
      const int32_t* cum = t.cumDst + (size_t)ei * (N + 1);
      if (q < cum[N]) {
        // destination rank: the last j with cum[j] <= q
        int lo = 0, hi = N - 1;
        while (lo < hi) {
          const int mid = (lo + hi + 1) >> 1;
          if (cum[mid] <= q) lo = mid; else hi = mid - 1;
        }
        const int j = lo;
        const int ej = e * N + j;
        const long long pos = t.preSrc[(size_t)ei * N + j] + (q - cum[j]);
        const long long n = t.recv[ej], reps = t.R[ej];
        if (n > 0 && reps > 0) {
          // slot m of the (e, j) list holds positions [floor(m*n/reps), floor((m+1)*n/reps))
          long long m = ((pos + 1) * reps - 1) / n;
          m = m < reps ? m : reps - 1;
          const int s = t.slot_sorted[j * c + t.ejstart[ej] + (int)m];
          const long long r = slot_offsets[s] + pos - (m * n) / reps;
          if (r >= 0 && r < P) row = (int)r;
        }
      }
    }
    if (in) pair_to_row[p] = row;
    if (row >= 0) row_to_pair[row] = (int)p;
  }
}

}  // namespace

extern "C" size_t lz_plan_workspace_bytes(const lz_shape* shape) {
  if (!lz::shape_ok(shape)) return 0;
  return carve(nullptr, shape).total_bytes;
}

namespace {

// The four launches of the dispatcher on tables carved from `ws` (already checked by the caller).
int32_t enqueue_plan(const int32_t* topk_ids, const lz_shape* shape, const int32_t* rank_tok_off,
                     const int32_t* slot_expert, int32_t* slot_counts, int32_t* slot_offsets,
                     int32_t* pair_to_row, int32_t* row_to_pair, int32_t* Tej_opt, int32_t* D_opt,
                     int32_t* status_opt, const PlanTables& t, hipStream_t st) {
  const long long P = (long long)shape->T * shape->k;
  const int nch = max_chunks(P, shape->N);
  const unsigned blocks = unsigned((nch + kWavesPerBlock - 1) / kWavesPerBlock);
  if (P > 0)
    hipLaunchKernelGGL(count_kernel, dim3(blocks), dim3(256), 0, st, topk_ids, rank_tok_off, shape->T,
                       shape->E, shape->N, shape->k, t, row_to_pair);
  hipLaunchKernelGGL(schedule_expert_kernel, dim3(shape->E), dim3(kExpertThreads), 0, st, rank_tok_off,
                     slot_expert, shape->T, shape->E, shape->N, shape->c, shape->k, t, Tej_opt, D_opt);
  hipLaunchKernelGGL(schedule_slots_kernel, dim3(1), dim3(kSchedThreads), 0, st, rank_tok_off, slot_expert,
                     shape->T, shape->E, shape->N, shape->c, shape->k, t, slot_counts, slot_offsets,
                     status_opt);
  if (P > 0)
    hipLaunchKernelGGL(place_kernel, dim3(blocks), dim3(256), 0, st, topk_ids, rank_tok_off, shape->T,
                       shape->E, shape->N, shape->c, shape->k, t, slot_offsets, pair_to_row,
                       row_to_pair);
  return lz::launch_status();
}

int32_t check_plan_args(const int32_t* topk_ids, const lz_shape* shape, const int32_t* rank_tok_off,
                        const int32_t* slot_expert, const int32_t* slot_counts, const int32_t* slot_offsets,
                        const int32_t* pair_to_row, const int32_t* row_to_pair) {
  if (!lz::shape_ok(shape)) return LZ_ESHAPE;
  if (!rank_tok_off || !slot_expert || !slot_counts || !slot_offsets) return LZ_EINVAL;
  const long long P = (long long)shape->T * shape->k;
  if (P > 0 && (!topk_ids || !pair_to_row || !row_to_pair)) return LZ_EINVAL;
  return LZ_OK;
}

}  // namespace

extern "C" int32_t lz_plan_dispatch(const int32_t* topk_ids, const lz_shape* shape,
                                    const int32_t* rank_tok_off, const int32_t* slot_expert,
                                    int32_t* slot_counts, int32_t* slot_offsets, int32_t* pair_to_row,
                                    int32_t* row_to_pair, int32_t* Tej_opt, int32_t* D_opt,
                                    int32_t* status_opt, void* ws, size_t ws_bytes, void* stream) {
  const int32_t rc = check_plan_args(topk_ids, shape, rank_tok_off, slot_expert, slot_counts, slot_offsets,
                                     pair_to_row, row_to_pair);
  if (rc != LZ_OK) return rc;
  PlanTables t = carve(ws, shape);
  if (!ws || (uintptr_t)ws % 256 != 0 || ws_bytes < t.total_bytes) return LZ_EWORKSPACE;
  return enqueue_plan(topk_ids, shape, rank_tok_off, slot_expert, slot_counts, slot_offsets, pair_to_row,
                      row_to_pair, Tej_opt, D_opt, status_opt, t, (hipStream_t)stream);
}

// ------------------------------------------------------------------------------------------
// The same dispatcher for callers that cannot allocate: its tables live in a fixed array in
// device memory that belongs to the library (one copy per GPU, held until the process ends).
// ------------------------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[LZ_PLAN_NOALLOC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};  // device address of `scratch` on each GPU, looked up once

// Address of this GPU's copy of `scratch`.  In host code the array's name is only a handle for
// the runtime's symbol lookup, never a device address; every GPU has its own copy at its own address.
int32_t scratch_of_current_device(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return LZ_EHIP;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return LZ_EHIP;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return LZ_OK;
}

}  // namespace

extern "C" int32_t lz_plan_dispatch_noalloc(const int32_t* topk_ids, const lz_shape* shape,
                                            const int32_t* rank_tok_off, const int32_t* slot_expert,
                                            int32_t* slot_counts, int32_t* slot_offsets,
                                            int32_t* pair_to_row, int32_t* row_to_pair, int32_t* Tej_opt,
                                            int32_t* D_opt, int32_t* status_opt, void* stream) {
  const int32_t rc = check_plan_args(topk_ids, shape, rank_tok_off, slot_expert, slot_counts, slot_offsets,
                                     pair_to_row, row_to_pair);
  if (rc != LZ_OK) return rc;
  if (carve(nullptr, shape).total_bytes > (size_t)LZ_PLAN_NOALLOC_SCRATCH_BYTES) return LZ_EWORKSPACE;
  void* base = nullptr;
  const int32_t rs = scratch_of_current_device(&base);
  if (rs != LZ_OK) return rs;
  // Every table entry a kernel reads was written earlier in the same call, so what the previous
  // call left in the array does not matter and nothing has to be cleared.
  const PlanTables t = carve(base, shape);
  return enqueue_plan(topk_ids, shape, rank_tok_off, slot_expert, slot_counts, slot_offsets, pair_to_row,
                      row_to_pair, Tej_opt, D_opt, status_opt, t, (hipStream_t)stream);
}
