// Host-side planning: replica allocation (Eq. 1), maximum-rank-overlap and spread
// placement (Sec. 4.1, Theorem 1), recovery probability by enumeration (Sec. 6.3) and
// re-planning after rank loss (Sec. 4.3).  Pure integer functions on host arrays.
#include <algorithm>
#include <cstdint>
#include <numeric>
#include <vector>

#include "lazarus_moe.h"

namespace {

// experts by ascending (key1, key2, id)
std::vector<int> sorted_experts(int E, const int64_t* key1, const int64_t* key2) {
  std::vector<int> order(E);
  std::iota(order.begin(), order.end(), 0);
  std::stable_sort(order.begin(), order.end(), [&](int a, int b) {
    if (key1[a] != key1[b]) return key1[a] < key1[b];
    if (key2 && key2[a] != key2[b]) return key2[a] < key2[b];
    return a < b;
  });
  return order;
}

int allocate(const int64_t* t_e, int E, int N, int c, int f, int32_t* r_e) {
  if (!t_e || !r_e || E < 1 || N < 1 || c < 1 || f < 1) return LZ_EINVAL;
  for (int e = 0; e < E; ++e)
    if (t_e[e] < 0) return LZ_EINVAL;
  const int64_t slots = int64_t(N) * c;
  const int64_t f_eff = std::min<int64_t>(f, slots / E);
  if (f_eff < 1) return LZ_EINFEASIBLE;
  std::vector<int> order = sorted_experts(E, t_e, nullptr);
  // tail[pos] = sum of the loads from position pos on, in load order
  std::vector<__int128> tail(E + 1, 0);
  for (int pos = E - 1; pos >= 0; --pos) tail[pos] = tail[pos + 1] + t_e[order[pos]];
  int64_t rem = slots;
  for (int pos = 0; pos < E; ++pos) {
    const int e = order[pos];
    int64_t share;
    if (tail[pos] == 0) {
      share = rem / (E - pos);
    } else {
      share = int64_t((__int128(t_e[e]) * rem) / tail[pos]);
    }
    const int64_t r = std::max(share, f_eff);
    r_e[e] = int32_t(r);
    rem -= r;
  }
  return rem == 0 ? LZ_OK : LZ_EINVAL;
}

int check_counts(const int32_t* r_e, int E, int N, int c) {
  if (!r_e || E < 1 || N < 1 || c < 1) return LZ_EINVAL;
  int64_t sum = 0;
  for (int e = 0; e < E; ++e) {
    if (r_e[e] < 0) return LZ_EINVAL;
    sum += r_e[e];
  }
  return sum == int64_t(N) * c ? LZ_OK : LZ_EINVAL;
}

int place_mro(const int32_t* r_e, const int64_t* t_e, int E, int N, int c, int32_t* slot_expert) {
  int rc = check_counts(r_e, E, N, c);
  if (rc != LZ_OK) return rc;
  if (!t_e || !slot_expert) return LZ_EINVAL;
  for (int e = 0; e < E; ++e)
    if (r_e[e] < 1) return LZ_EINVAL;
  std::vector<int64_t> r64(r_e, r_e + E);
  std::vector<int> order = sorted_experts(E, r64.data(), t_e);
  std::vector<int> left(E);
  for (int q = 0; q < E; ++q) left[q] = r_e[order[q]];
  std::vector<int> fill(N, 0);  // slots already used on each rank
  auto put = [&](int rank, int q) {
    slot_expert[rank * c + fill[rank]++] = order[q];
    --left[q];
  };
  const int G = (E + c - 1) / c;
  if (G == 1) {
    for (int q = 0; q < E; ++q) {
      const int span = std::min(left[q], N);
      for (int j = 0; j < span; ++j) put(j, q);
    }
  } else {
    int node0 = 0;
    for (int g = 0; g < G; ++g) {
      const int first = g * c;
      const int last = std::min(first + c, E);
      const int want = r_e[order[first]];
      const int size = g < G - 1 ? want : std::min(N - node0, want);
      if (size < 1 || node0 + size > N) return LZ_EINVAL;
      for (int j = node0; j < node0 + size; ++j)
        for (int q = first; q < last; ++q) put(j, q);
      node0 += size;
    }
  }
  int cursor = 0;
  for (int j = 0; j < N; ++j) {
    while (fill[j] < c) {
      while (left[cursor % E] == 0) ++cursor;
      put(j, cursor % E);
      ++cursor;
    }
  }
  return LZ_OK;
}

bool covers_all(const int32_t* slot_expert, int E, int c, const std::vector<int>& ranks,
                std::vector<uint8_t>& seen) {
  std::fill(seen.begin(), seen.end(), 0);
  int n = 0;
  for (int j : ranks)
    for (int l = 0; l < c; ++l) {
      const int e = slot_expert[j * c + l];
      if (e >= 0 && e < E && !seen[e]) {
        seen[e] = 1;
        ++n;
      }
    }
  return n == E;
}

}  // namespace

extern "C" {

int32_t lz_allocate_replicas(const int64_t* t_e, int32_t E, int32_t N, int32_t c, int32_t f,
                             int32_t* r_e) {
  return allocate(t_e, E, N, c, f, r_e);
}

int32_t lz_place_mro(const int32_t* r_e, const int64_t* t_e, int32_t E, int32_t N, int32_t c,
                     int32_t* slot_expert) {
  return place_mro(r_e, t_e, E, N, c, slot_expert);
}

int32_t lz_place_spread(const int32_t* r_e, int32_t E, int32_t N, int32_t c, int32_t* slot_expert) {
  int rc = check_counts(r_e, E, N, c);
  if (rc != LZ_OK) return rc;
  if (!slot_expert) return LZ_EINVAL;
  int64_t q = 0;
  for (int e = 0; e < E; ++e)
    for (int n = 0; n < r_e[e]; ++n, ++q) slot_expert[(q % N) * c + q / N] = e;
  return LZ_OK;
}

int32_t lz_place_compact(const int32_t* r_e, int32_t E, int32_t N, int32_t c, int32_t* slot_expert) {
  int rc = check_counts(r_e, E, N, c);
  if (rc != LZ_OK) return rc;
  if (!slot_expert) return LZ_EINVAL;
  int64_t q = 0;
  for (int e = 0; e < E; ++e)
    for (int n = 0; n < r_e[e]; ++n, ++q) slot_expert[q] = e;  // rank q / c, local slot q % c
  return LZ_OK;
}

int32_t lz_recovery_probability(const int32_t* slot_expert, int32_t E, int32_t N, int32_t c,
                                int32_t n_alive, uint64_t* n_recoverable, uint64_t* n_total) {
  if (!slot_expert || !n_recoverable || !n_total || E < 1 || N < 1 || N > 62 || c < 1 ||
      n_alive < 0 || n_alive > N)
    return LZ_EINVAL;
  // per-rank expert sets as bit rows; E can exceed 64, so use a small bitset per rank
  const int words = (E + 63) / 64;
  std::vector<uint64_t> sets(size_t(N) * words, 0);
  for (int j = 0; j < N; ++j)
    for (int l = 0; l < c; ++l) {
      const int e = slot_expert[j * c + l];
      if (e >= 0 && e < E) sets[size_t(j) * words + e / 64] |= uint64_t(1) << (e % 64);
    }
  std::vector<uint64_t> full(words, ~uint64_t(0));
  if (E % 64) full[words - 1] = (uint64_t(1) << (E % 64)) - 1;
  uint64_t good = 0, total = 0;
  std::vector<int> pick(n_alive);
  std::iota(pick.begin(), pick.end(), 0);
  std::vector<uint64_t> acc(words);
  while (true) {
    std::fill(acc.begin(), acc.end(), 0);
    for (int j : pick)
      for (int w = 0; w < words; ++w) acc[w] |= sets[size_t(j) * words + w];
    ++total;
    good += (acc == full);
    // next combination in lexicographic order
    int i = n_alive - 1;
    while (i >= 0 && pick[i] == N - n_alive + i) --i;
    if (i < 0) break;
    ++pick[i];
    for (int x = i + 1; x < n_alive; ++x) pick[x] = pick[x - 1] + 1;
  }
  *n_recoverable = good;
  *n_total = total;
  return LZ_OK;
}

int32_t lz_replan(const int32_t* old_slot_expert, int32_t N_old, int32_t c_old,
                  const uint8_t* alive, const int64_t* t_e, int32_t E, int32_t c_new, int32_t f,
                  int32_t* new_slot_expert, int32_t* plan2phys, lz_transfer* xfers,
                  int32_t* n_xfers, int32_t* N_new_out) {
  if (!old_slot_expert || !alive || !t_e || !new_slot_expert || !plan2phys || !xfers || !n_xfers ||
      !N_new_out || N_old < 1 || c_old < 1 || c_new < 1 || E < 1 || f < 1)
    return LZ_EINVAL;
  std::vector<int> survivors;
  for (int j = 0; j < N_old; ++j)
    if (alive[j]) survivors.push_back(j);
  const int N_new = int(survivors.size());
  *N_new_out = N_new;
  std::vector<uint8_t> seen(E);
  if (N_new == 0 || !covers_all(old_slot_expert, E, c_old, survivors, seen)) return LZ_EUNRECOVERABLE;
  if (*n_xfers < N_new * c_new) return LZ_EINVAL;

  std::vector<int32_t> r(E), plan(size_t(N_new) * c_new);
  int rc = allocate(t_e, E, N_new, c_new, f, r.data());
  if (rc != LZ_OK) return rc;
  rc = place_mro(r.data(), t_e, E, N_new, c_new, plan.data());
  if (rc != LZ_OK) return rc;

  // held[m][e]: survivor m holds expert e in the old plan; first_slot: its lowest such slot
  std::vector<int> first_slot(size_t(N_new) * E, -1);
  for (int m = 0; m < N_new; ++m)
    for (int l = c_old - 1; l >= 0; --l) {
      const int s = survivors[m] * c_old + l;
      const int e = old_slot_expert[s];
      if (e >= 0 && e < E) first_slot[size_t(m) * E + e] = s;
    }
  // greedy node mapping
  std::vector<int> plan_of(N_new, -1);
  std::vector<uint8_t> used(N_new, 0), in_plan(E);
  for (int m = 0; m < N_new; ++m) {
    int best = -1, best_cost = 0;
    for (int q = 0; q < N_new; ++q) {
      if (used[q]) continue;
      std::fill(in_plan.begin(), in_plan.end(), 0);
      int cost = 0;
      for (int l = 0; l < c_new; ++l) {
        const int e = plan[size_t(q) * c_new + l];
        if (!in_plan[e]) {
          in_plan[e] = 1;
          cost += first_slot[size_t(m) * E + e] < 0;
        }
      }
      if (best < 0 || cost < best_cost) {
        best = q;
        best_cost = cost;
      }
    }
    used[best] = 1;
    plan_of[m] = best;
    plan2phys[best] = survivors[m];
  }
  for (int m = 0; m < N_new; ++m)
    for (int l = 0; l < c_new; ++l)
      new_slot_expert[m * c_new + l] = plan[size_t(plan_of[m]) * c_new + l];

  // transfers: owners of each expert among the survivors, requests dealt round-robin
  std::vector<std::vector<int>> owners(E);
  for (int e = 0; e < E; ++e)
    for (int m = 0; m < N_new; ++m)
      if (first_slot[size_t(m) * E + e] >= 0) owners[e].push_back(m);
  std::vector<int> next_owner(E, 0);
  std::vector<int> fetched(size_t(N_new) * E, -1);  // owner index chosen for (m, e)
  int n = 0;
  for (int m = 0; m < N_new; ++m)
    for (int l = 0; l < c_new; ++l) {
      const int e = new_slot_expert[m * c_new + l];
      lz_transfer t;
      t.dst_slot = m * c_new + l;
      t.expert = e;
      if (first_slot[size_t(m) * E + e] >= 0) {
        t.src_slot = first_slot[size_t(m) * E + e];
        t.remote = 0;
      } else {
        int& who = fetched[size_t(m) * E + e];
        if (who < 0) {
          who = owners[e][next_owner[e] % owners[e].size()];
          ++next_owner[e];
        }
        t.src_slot = first_slot[size_t(who) * E + e];
        t.remote = 1;
      }
      xfers[n++] = t;
    }
  *n_xfers = n;
  return LZ_OK;
}

}  // extern "C"
