// Hierarchical EBV vertex-cut partitioner (Sec. 6) and the partition statistics the paper
// reports (Sec. 6 definitions, Sec. 7 ablation table). Host code only: the assignment is a
// sequential greedy pass over the edges, O(|E| p), with replica sets kept as 64-bit masks.
#include <algorithm>
#include <numeric>
#include <vector>

#include "cdf_common.h"

namespace cdf {

static inline int popcount64(uint64_t x) { return __builtin_popcountll(x); }

}  // namespace cdf

using namespace cdf;

extern "C" int cdf_ebv_partition(int64_t n_vertices, int64_t n_edges, const int64_t* eu, const int64_t* ev,
                                 const cdf_ebv_params* prm, int32_t* part) {
  CDF_REQUIRE(prm != nullptr, "cdf_ebv_partition: null parameters");
  const int p = prm->p, dph = prm->devices_per_host;
  CDF_REQUIRE(n_vertices > 0 && n_edges >= 0, "cdf_ebv_partition: bad sizes");
  CDF_REQUIRE(p >= 1 && p <= 64, "cdf_ebv_partition: p = %d outside [1, 64]", p);
  CDF_REQUIRE(dph >= 1 && p % dph == 0, "cdf_ebv_partition: devices_per_host = %d does not divide p = %d", dph, p);
  CDF_REQUIRE(prm->gamma >= 0.0 && prm->gamma <= 1.0 && prm->alpha >= 0.0 && prm->beta >= 0.0,
              "cdf_ebv_partition: weights out of range");
  if (n_edges == 0) return CDF_OK;
  CDF_REQUIRE(eu && ev && part, "cdf_ebv_partition: null pointer");
  for (int64_t e = 0; e < n_edges; ++e)
    CDF_REQUIRE(eu[e] >= 0 && eu[e] < n_vertices && ev[e] >= 0 && ev[e] < n_vertices && eu[e] != ev[e],
                "cdf_ebv_partition: edge %lld has an endpoint out of range or is a self pair",
                static_cast<long long>(e));
  // processing order: as given, or by ascending sum of the end vertices' degrees (stable)
  std::vector<int64_t> order(n_edges);
  if (prm->sort_edges) {
    // counting sort on the degree sum: stable, O(|E| + largest key)
    std::vector<int64_t> deg(n_vertices, 0);
    for (int64_t e = 0; e < n_edges; ++e) { ++deg[eu[e]]; ++deg[ev[e]]; }
    std::vector<int64_t> key(n_edges);
    int64_t top = 0;
    for (int64_t e = 0; e < n_edges; ++e) {
      key[e] = deg[eu[e]] + deg[ev[e]];
      top = std::max(top, key[e]);
    }
    std::vector<int64_t> start(top + 2, 0);
    for (int64_t e = 0; e < n_edges; ++e) ++start[key[e] + 1];
    for (int64_t k = 0; k <= top; ++k) start[k + 1] += start[k];
    for (int64_t e = 0; e < n_edges; ++e) order[start[key[e]]++] = e;
  } else {
    std::iota(order.begin(), order.end(), int64_t{0});
  }
  std::vector<uint64_t> d_rep(n_vertices, 0), h_rep(n_vertices, 0);
  std::vector<int64_t> e_count(p, 0), v_count(p, 0);
  const double e_norm = static_cast<double>(n_edges) / p, v_norm = static_cast<double>(n_vertices) / p;
  const double g = prm->gamma, a = prm->alpha, b = prm->beta;
  for (int64_t k = 0; k < n_edges; ++k) {
    const int64_t e = order[k], u = eu[e], v = ev[e];
    int best = 0;
    double best_eva = 0.0;
    for (int i = 0; i < p; ++i) {
      const int h = i / dph;
      const double miss_d = static_cast<double>(!((d_rep[u] >> i) & 1)) + static_cast<double>(!((d_rep[v] >> i) & 1));
      const double miss_h = static_cast<double>(!((h_rep[u] >> h) & 1)) + static_cast<double>(!((h_rep[v] >> h) & 1));
      const double eva = (1.0 - g) * miss_d + g * miss_h + a * (static_cast<double>(e_count[i]) / e_norm) +
                         b * (static_cast<double>(v_count[i]) / v_norm);
      if (i == 0 || eva < best_eva) { best = i; best_eva = eva; }
    }
    part[e] = best;
    ++e_count[best];
    const uint64_t bit = uint64_t{1} << best, hbit = uint64_t{1} << (best / dph);
    if (!(d_rep[u] & bit)) { d_rep[u] |= bit; ++v_count[best]; }
    if (!(d_rep[v] & bit)) { d_rep[v] |= bit; ++v_count[best]; }
    h_rep[u] |= hbit;
    h_rep[v] |= hbit;
  }
  return CDF_OK;
}

extern "C" int cdf_cut_statistics(int64_t n_vertices, int64_t n_edges, const int64_t* eu, const int64_t* ev,
                                  const int32_t* part, int32_t p, int32_t devices_per_host, int32_t* master,
                                  cdf_cut_stats* out) {
  CDF_REQUIRE(out != nullptr, "cdf_cut_statistics: null result");
  CDF_REQUIRE(n_vertices > 0 && n_edges >= 0, "cdf_cut_statistics: bad sizes");
  CDF_REQUIRE(p >= 1 && p <= 64, "cdf_cut_statistics: p = %d outside [1, 64]", p);
  CDF_REQUIRE(devices_per_host >= 1 && p % devices_per_host == 0,
              "cdf_cut_statistics: devices_per_host = %d does not divide p = %d", devices_per_host, p);
  CDF_REQUIRE(n_edges == 0 || (eu && ev && part), "cdf_cut_statistics: null pointer");
  std::vector<uint64_t> rep(n_vertices, 0);
  std::vector<int64_t> e_count(p, 0), v_count(p, 0), inner(p, 0), outer(p, 0);
  // per vertex and partition: incident edges held there (decides the master)
  std::vector<int32_t> inc(static_cast<size_t>(n_vertices) * p, 0);
  for (int64_t e = 0; e < n_edges; ++e) {
    const int i = part[e];
    CDF_REQUIRE(i >= 0 && i < p, "cdf_cut_statistics: edge %lld assigned to partition %d", static_cast<long long>(e), i);
    CDF_REQUIRE(eu[e] >= 0 && eu[e] < n_vertices && ev[e] >= 0 && ev[e] < n_vertices,
                "cdf_cut_statistics: edge %lld endpoint out of range", static_cast<long long>(e));
    ++e_count[i];
    rep[eu[e]] |= uint64_t{1} << i;
    rep[ev[e]] |= uint64_t{1} << i;
    ++inc[eu[e] * p + i];
    ++inc[ev[e] * p + i];
  }
  int64_t replicas = 0;
  for (int64_t v = 0; v < n_vertices; ++v) {
    int m = static_cast<int>(v % p);           // a vertex without edges lives on one partition only
    if (rep[v]) {
      m = 0;
      for (int i = 1; i < p; ++i)
        if (inc[v * p + i] > inc[v * p + m]) m = i;
    } else {
      rep[v] = uint64_t{1} << m;
    }
    if (master) master[v] = m;
    replicas += popcount64(rep[v]);
    const int hm = m / devices_per_host;
    for (int i = 0; i < p; ++i) {
      if (!((rep[v] >> i) & 1)) continue;
      ++v_count[i];
      if (i == m) continue;
      // gather: mirror i -> master m ; scatter: master m -> mirror i
      if (i / devices_per_host == hm) { ++inner[i]; ++inner[m]; } else { ++outer[i]; ++outer[m]; }
    }
  }
  out->replicas_total = replicas;
  out->replication_factor = static_cast<double>(replicas) / static_cast<double>(n_vertices);
  out->edge_imbalance = n_edges ? static_cast<double>(*std::max_element(e_count.begin(), e_count.end())) /
                                      (static_cast<double>(n_edges) / p)
                                : 1.0;
  out->vertex_imbalance = static_cast<double>(*std::max_element(v_count.begin(), v_count.end())) /
                          (static_cast<double>(replicas) / p);
  out->max_inner = *std::max_element(inner.begin(), inner.end());
  out->max_outer = *std::max_element(outer.begin(), outer.end());
  return CDF_OK;
}
