// Scheduler-side placement pipeline (paper Sec. III-C): entropy, Alg. 1 (expert
// count allocation), Alg. 2 (expert-to-server assignment), Eq. 2-4.  Host code
// only; it turns the activation counts the layer accumulates into the masks the
// layer consumes.  O(N L E log E) per plan.
#include <algorithm>
#include <cmath>
#include <numeric>
#include <vector>

#include "prism_internal.h"
#include "prism_placement.h"

namespace prism {
namespace {

bool bad_dims(int32_t n, int32_t l, int32_t e) { return n < 1 || l < 1 || e < 1; }

bool any_negative(const int64_t* f, size_t n) {
  for (size_t i = 0; i < n; ++i)
    if (f[i] < 0) return true;
  return false;
}

// One layer of Alg. 2 after the top-N initialisation: place the experts nobody holds.
// held[n * E + e] is the layer's slice of the placement, freq[n * E + e] of f.
bool repair_coverage(std::vector<uint8_t>& held, const std::vector<int64_t>& freq, int N, int E) {
  std::vector<int> holders(E, 0);
  for (int n = 0; n < N; ++n)
    for (int e = 0; e < E; ++e) holders[e] += held[(size_t)n * E + e];
  int missing = 0;
  for (int e = 0; e < E; ++e) missing += holders[e] == 0;

  auto n_duplicates = [&](int n) {
    int c = 0;
    for (int e = 0; e < E; ++e) c += held[(size_t)n * E + e] && holders[e] >= 2;
    return c;
  };
  std::vector<int> order(N);
  while (missing > 0) {
    std::vector<int> dups(N);
    for (int n = 0; n < N; ++n) dups[n] = n_duplicates(n);
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return dups[a] < dups[b]; });
    bool replaced = false;
    for (int n : order) {
      if (missing == 0) break;
      const int64_t* fn = &freq[(size_t)n * E];
      uint8_t* hn = &held[(size_t)n * E];
      // this server's least used duplicate (higher index among equals) ...
      int out = -1;
      for (int e = 0; e < E; ++e)
        if (hn[e] && holders[e] >= 2 && (out < 0 || fn[e] <= fn[out])) out = e;
      if (out < 0) continue;
      // ... makes room for the unassigned expert it uses most (lower index among equals)
      int in = -1;
      for (int e = 0; e < E; ++e)
        if (holders[e] == 0 && (in < 0 || fn[e] > fn[in])) in = e;
      hn[out] = 0; --holders[out];
      hn[in] = 1; ++holders[in];
      --missing;
      replaced = true;
    }
    if (!replaced) return false;
  }
  return true;
}

}  // namespace
}  // namespace prism

using namespace prism;

extern "C" {
#pragma GCC visibility push(default)

prism_status prism_activation_entropy(const int64_t* f, int32_t N, int32_t L, int32_t E, double* v) {
  PRISM_RETURN_IF(f == nullptr || v == nullptr || bad_dims(N, L, E), PRISM_ERR_INVALID_ARG);
  PRISM_RETURN_IF(any_negative(f, (size_t)N * L * E), PRISM_ERR_INVALID_ARG);
  for (size_t nl = 0; nl < (size_t)N * L; ++nl) {
    const int64_t* row = f + nl * E;
    double total = 0.0;
    for (int e = 0; e < E; ++e) total += (double)row[e];
    double h = 0.0;
    if (total > 0.0)
      for (int e = 0; e < E; ++e)
        if (row[e] > 0) {
          const double p = (double)row[e] / total;
          h -= p * std::log2(p);
        }
    v[nl] = h;
  }
  return PRISM_OK;
}

prism_status prism_expert_count_allocation(const double* v, const double* server_mem,
                                           double expert_mem, int32_t N, int32_t L, int32_t E,
                                           int32_t* counts, int32_t* feasible) {
  PRISM_RETURN_IF(v == nullptr || server_mem == nullptr || counts == nullptr || feasible == nullptr ||
                      bad_dims(N, L, E),
                  PRISM_ERR_INVALID_ARG);
  PRISM_RETURN_IF(!(expert_mem > 0.0), PRISM_ERR_INVALID_ARG);
  for (int n = 0; n < N; ++n) PRISM_RETURN_IF(!(server_mem[n] > 0.0), PRISM_ERR_INVALID_ARG);
  for (size_t i = 0; i < (size_t)N * L; ++i) PRISM_RETURN_IF(!(v[i] >= 0.0), PRISM_ERR_INVALID_ARG);

  // Step 1: memory split over the layers in proportion to the activation diversity.
  for (int n = 0; n < N; ++n) {
    double vsum = 0.0;
    for (int l = 0; l < L; ++l) vsum += v[(size_t)n * L + l];
    for (int l = 0; l < L; ++l) {
      const double share = vsum > 0.0 ? v[(size_t)n * L + l] / vsum : 1.0 / L;
      const double c = std::floor(server_mem[n] / expert_mem * share);
      counts[(size_t)n * L + l] = c >= (double)E ? E : (int32_t)c;
    }
  }
  // Step 2: layers short of E borrow from the most over-provisioned other layer.
  std::vector<long long> total(L, 0);
  for (int n = 0; n < N; ++n)
    for (int l = 0; l < L; ++l) total[l] += counts[(size_t)n * L + l];
  std::vector<int> order(N);
  std::iota(order.begin(), order.end(), 0);
  std::stable_sort(order.begin(), order.end(),
                   [&](int a, int b) { return server_mem[a] > server_mem[b]; });
  *feasible = 1;
  for (int l = 0; l < L; ++l) {
    while (total[l] < E) {
      bool moved = false;
      for (int n : order) {
        int donor = -1;
        for (int j = 0; j < L; ++j)
          if (j != l && total[j] > E && (donor < 0 || total[j] > total[donor])) donor = j;
        if (donor < 0) break;
        int32_t* row = counts + (size_t)n * L;
        if (row[donor] > 0 && row[l] < E) {
          --row[donor]; ++row[l];
          --total[donor]; ++total[l];
          moved = true;
          if (total[l] == E) break;
        }
      }
      if (!moved) { *feasible = 0; break; }
    }
  }
  return PRISM_OK;
}

prism_status prism_expert_assignment(const int64_t* f, const int32_t* counts, int32_t N, int32_t L,
                                     int32_t E, uint8_t* placement, int32_t* covered) {
  PRISM_RETURN_IF(f == nullptr || counts == nullptr || placement == nullptr || covered == nullptr ||
                      bad_dims(N, L, E),
                  PRISM_ERR_INVALID_ARG);
  PRISM_RETURN_IF(any_negative(f, (size_t)N * L * E), PRISM_ERR_INVALID_ARG);
  for (size_t i = 0; i < (size_t)N * L; ++i)
    PRISM_RETURN_IF(counts[i] < 0 || counts[i] > E, PRISM_ERR_INVALID_ARG);

  // Top-N_{n,l} of every preference list.
  std::vector<int> pref(E);
  for (int n = 0; n < N; ++n)
    for (int l = 0; l < L; ++l) {
      const int64_t* fn = f + ((size_t)n * L + l) * E;
      uint8_t* out = placement + ((size_t)n * L + l) * E;
      std::iota(pref.begin(), pref.end(), 0);
      std::stable_sort(pref.begin(), pref.end(), [&](int a, int b) { return fn[a] > fn[b]; });
      std::fill(out, out + E, (uint8_t)0);
      for (int i = 0; i < counts[(size_t)n * L + l]; ++i) out[pref[i]] = 1;
    }
  // Coverage repair, layer by layer.
  *covered = 1;
  std::vector<uint8_t> held((size_t)N * E);
  std::vector<int64_t> freq((size_t)N * E);
  for (int l = 0; l < L; ++l) {
    for (int n = 0; n < N; ++n)
      for (int e = 0; e < E; ++e) {
        held[(size_t)n * E + e] = placement[((size_t)n * L + l) * E + e];
        freq[(size_t)n * E + e] = f[((size_t)n * L + l) * E + e];
      }
    if (!repair_coverage(held, freq, N, E)) *covered = 0;
    for (int n = 0; n < N; ++n)
      for (int e = 0; e < E; ++e) placement[((size_t)n * L + l) * E + e] = held[(size_t)n * E + e];
  }
  return PRISM_OK;
}

prism_status prism_proxy_cost(const int64_t* f, const uint8_t* placement, int32_t N, int32_t L,
                              int32_t E, int64_t* cost) {
  PRISM_RETURN_IF(f == nullptr || placement == nullptr || cost == nullptr || bad_dims(N, L, E),
                  PRISM_ERR_INVALID_ARG);
  PRISM_RETURN_IF(any_negative(f, (size_t)N * L * E), PRISM_ERR_INVALID_ARG);
  int64_t c = 0;
  for (size_t i = 0; i < (size_t)N * L * E; ++i)
    if (placement[i] == 0) c += f[i];
  *cost = c;
  return PRISM_OK;
}

prism_status prism_migration_cost(const uint8_t* old_placement, const uint8_t* new_placement,
                                  int32_t N, int32_t L, int32_t E, double expert_mem,
                                  const double* speed, double* seconds, int64_t* flips) {
  PRISM_RETURN_IF(old_placement == nullptr || new_placement == nullptr || speed == nullptr ||
                      seconds == nullptr || flips == nullptr || bad_dims(N, L, E),
                  PRISM_ERR_INVALID_ARG);
  PRISM_RETURN_IF(!(expert_mem > 0.0), PRISM_ERR_INVALID_ARG);
  for (int n = 0; n < N; ++n) PRISM_RETURN_IF(!(speed[n] > 0.0), PRISM_ERR_INVALID_ARG);
  double s = 0.0;
  int64_t c = 0;
  for (int n = 0; n < N; ++n) {
    int64_t changed = 0;
    for (size_t i = 0; i < (size_t)L * E; ++i) {
      const size_t k = (size_t)n * L * E + i;
      changed += (old_placement[k] != 0) != (new_placement[k] != 0);
    }
    c += changed;
    s += (double)changed * (expert_mem / speed[n]);
  }
  *seconds = s;
  *flips = c;
  return PRISM_OK;
}

prism_status prism_migration_decision(int64_t cost_old, int64_t cost_new, double t_mig,
                                      double seconds_per_remote_call, int32_t* adopt) {
  PRISM_RETURN_IF(adopt == nullptr || cost_old < 0 || cost_new < 0 || !(t_mig >= 0.0) ||
                      !(seconds_per_remote_call >= 0.0),
                  PRISM_ERR_INVALID_ARG);
  *adopt = (double)cost_new * seconds_per_remote_call + t_mig < (double)cost_old * seconds_per_remote_call;
  return PRISM_OK;
}

prism_status prism_placement_plan(const int64_t* f, const double* server_mem, double expert_mem,
                                  int32_t N, int32_t L, int32_t E, double* v, int32_t* counts,
                                  uint8_t* placement, int32_t* ok) {
  PRISM_RETURN_IF(ok == nullptr || placement == nullptr || f == nullptr || server_mem == nullptr ||
                      bad_dims(N, L, E) || !(expert_mem > 0.0),
                  PRISM_ERR_INVALID_ARG);
  PRISM_RETURN_IF(any_negative(f, (size_t)N * L * E), PRISM_ERR_INVALID_ARG);
  for (int n = 0; n < N; ++n) PRISM_RETURN_IF(!(server_mem[n] > 0.0), PRISM_ERR_INVALID_ARG);
  std::vector<double> v_own;
  std::vector<int32_t> counts_own;
  if (v == nullptr) { v_own.resize((size_t)N * L); v = v_own.data(); }
  if (counts == nullptr) { counts_own.resize((size_t)N * L); counts = counts_own.data(); }
  int32_t feasible = 0, covered = 0;
  PRISM_TRY(prism_activation_entropy(f, N, L, E, v));
  PRISM_TRY(prism_expert_count_allocation(v, server_mem, expert_mem, N, L, E, counts, &feasible));
  PRISM_TRY(prism_expert_assignment(f, counts, N, L, E, placement, &covered));
  *ok = feasible && covered;
  return PRISM_OK;
}

#pragma GCC visibility pop
}  // extern "C"
