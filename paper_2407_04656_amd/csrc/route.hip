// Top-k gate routing (Sec. 2.1): for each token the k largest of E logits, descending,
// ties towards the lower expert index, and the softmax over those k logits.
//
// A group of G = next_pow2(ceil(E/4)) <= 64 lanes owns one token; each lane keeps up to four
// logits in registers (the per-lane maximum is plain ALU work, so few lanes per token mean few
// shuffle steps and many tokens per wave).  One selection round is a max-reduction over the group of
// a 64-bit key (order-preserving image of the logit in the high word, ~expert in the low
// word), so the comparison and the tie rule are a single unsigned max.
#include "lz_common.h"

namespace {

constexpr int kMaxPerLane = lz::kMaxE / lz::kWave;  // 4

__device__ __forceinline__ uint32_t ordered_bits(float v) {
  v = v + 0.0f;  // -0.0 -> +0.0 so the two zeros compare equal
  uint32_t u = __float_as_uint(v);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ float from_ordered_bits(uint32_t o) {
  uint32_t u = (o & 0x80000000u) ? (o & 0x7FFFFFFFu) : ~o;
  return __uint_as_float(u);
}

template <int G>
__global__ __launch_bounds__(256) void route_kernel(const float* __restrict__ logits, int T, int E,
                                                    int k, int32_t* __restrict__ ids,
                                                    float* __restrict__ gates) {
  const int lane_in_group = threadIdx.x % G;
  const long long token = (long long)blockIdx.x * (256 / G) + threadIdx.x / G;
  const bool live = token < T;
  const long long tok = live ? token : 0;  // idle groups shadow token 0 and write nothing

  uint64_t key[kMaxPerLane];
#pragma unroll
  for (int v = 0; v < kMaxPerLane; ++v) {
    const int e = lane_in_group + v * G;
    key[v] = 0;  // 0 = absent / already taken; any real key is larger
    if (e < E) {
      const float val = logits[tok * E + e];
      key[v] = (uint64_t(ordered_bits(val)) << 32) | uint32_t(0xFFFFFFFFu - uint32_t(e));
    }
  }

  float sel[lz::kMaxK];
  int sel_id[lz::kMaxK];
#pragma unroll
  for (int kk = 0; kk < lz::kMaxK; ++kk) {
    sel[kk] = 0.f;
    sel_id[kk] = 0;
    if (kk < k) {
      uint64_t best = key[0];
#pragma unroll
      for (int v = 1; v < kMaxPerLane; ++v) best = key[v] > best ? key[v] : best;
#pragma unroll
      for (int off = G / 2; off > 0; off >>= 1) {
        const uint64_t other = __shfl_xor(best, off, G);
        best = other > best ? other : best;
      }
      const int e = int(0xFFFFFFFFu - uint32_t(best));
      sel[kk] = from_ordered_bits(uint32_t(best >> 32));
      sel_id[kk] = e;
#pragma unroll
      for (int v = 0; v < kMaxPerLane; ++v)
        if (lane_in_group + v * G == e) key[v] = 0;
    }
  }

  if (live && lane_in_group == 0) {
    float ex[lz::kMaxK];
    float denom = 0.f;
#pragma unroll
    for (int kk = 0; kk < lz::kMaxK; ++kk) {
      ex[kk] = 0.f;
      if (kk < k) {
        ex[kk] = expf(sel[kk] - sel[0]);
        denom += ex[kk];
      }
    }
#pragma unroll
    for (int kk = 0; kk < lz::kMaxK; ++kk)
      if (kk < k) {
        ids[tok * k + kk] = sel_id[kk];
        gates[tok * k + kk] = ex[kk] / denom;
      }
  }
}

template <int G>
void launch(const float* logits, int T, int E, int k, int32_t* ids, float* gates, hipStream_t st) {
  const int per_block = 256 / G;
  const unsigned blocks = unsigned((T + per_block - 1) / per_block);
  hipLaunchKernelGGL(route_kernel<G>, dim3(blocks), dim3(256), 0, st, logits, T, E, k, ids, gates);
}

}  // namespace

extern "C" int32_t lz_route(const float* logits, int32_t T, int32_t E, int32_t k, int32_t* topk_ids,
                            float* topk_gates, void* stream) {
  if (T < 0 || E < 1 || E > lz::kMaxE || k < 1 || k > lz::kMaxK || k > E) return LZ_ESHAPE;
  if (T == 0) return LZ_OK;
  if (!logits || !topk_ids || !topk_gates) return LZ_EINVAL;
  hipStream_t st = (hipStream_t)stream;
  if (E <= 4) launch<1>(logits, T, E, k, topk_ids, topk_gates, st);
  else if (E <= 8) launch<2>(logits, T, E, k, topk_ids, topk_gates, st);
  else if (E <= 16) launch<4>(logits, T, E, k, topk_ids, topk_gates, st);
  else if (E <= 32) launch<8>(logits, T, E, k, topk_ids, topk_gates, st);
  else if (E <= 64) launch<16>(logits, T, E, k, topk_ids, topk_gates, st);
  else if (E <= 128) launch<32>(logits, T, E, k, topk_ids, topk_gates, st);
  else launch<64>(logits, T, E, k, topk_ids, topk_gates, st);
  return lz::launch_status();
}
