// Graph-aware rescheduling (paper, Appendix A.2, Algorithm 1 "pack-and-shuffle"): host routine
// that repacks the graphs of a global batch into micro-batches of balanced atom count, shuffles
// each micro-batch, and tags it comm_free or dist for graph parallelism.  Pure integer host
// code; O(M log M + M log N_mb) with a min-heap of micro-batch loads.
#include <algorithm>
#include <cstdint>
#include <numeric>
#include <queue>
#include <vector>

#include "../../include/mlip.h"

namespace {

// Counter-based generator for the shuffle: splitmix64 finaliser of key(seed, stream) + (counter+1)*golden.
inline uint64_t mix64(uint64_t z) {
  z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ull;
  z ^= z >> 27; z *= 0x94D049BB133111EBull;
  z ^= z >> 31;
  return z;
}
inline uint64_t draw(uint64_t seed, uint64_t stream, uint64_t counter) {
  const uint64_t golden = 0x9E3779B97F4A7C15ull;
  uint64_t key = mix64(seed ^ (stream * golden));
  return mix64(key + (counter + 1) * golden);
}

}  // namespace

extern "C" int mlip_gars_pack(const int32_t* sizes_host, int64_t n_graphs, int32_t n_mb, int32_t d_gp, uint64_t seed,
                              int32_t* mb_ptr_host, int32_t* order_host, int32_t* type_host) {
  if (!sizes_host || !mb_ptr_host || !order_host || !type_host) return MLIP_E_INVALID;
  if (n_graphs < 0 || n_mb < 1 || d_gp < 1) return MLIP_E_INVALID;
  for (int64_t g = 0; g < n_graphs; ++g)
    if (sizes_host[g] < 0) return MLIP_E_INVALID;
  // (1) sort by size, descending (ties: lower graph index first), then longest-first placement
  std::vector<int32_t> idx((size_t)n_graphs);
  std::iota(idx.begin(), idx.end(), 0);
  std::stable_sort(idx.begin(), idx.end(), [&](int32_t a, int32_t b) { return sizes_host[a] > sizes_host[b]; });
  typedef std::pair<int64_t, int32_t> Load;  // (total size, micro-batch): smallest load, then lowest index
  std::priority_queue<Load, std::vector<Load>, std::greater<Load>> heap;
  for (int32_t j = 0; j < n_mb; ++j) heap.push(Load(0, j));
  std::vector<std::vector<int32_t>> mb((size_t)n_mb);
  std::vector<int64_t> load((size_t)n_mb, 0);
  for (int32_t g : idx) {
    Load top = heap.top();
    heap.pop();
    mb[top.second].push_back(g);
    load[top.second] = top.first + sizes_host[g];
    heap.push(Load(load[top.second], top.second));
  }
  // (2) shuffle inside each micro-batch (Fisher-Yates, stream = micro-batch index), (3) tag
  int32_t pos = 0;
  for (int32_t j = 0; j < n_mb; ++j) {
    std::vector<int32_t>& v = mb[j];
    for (int64_t t = (int64_t)v.size() - 1; t >= 1; --t) {
      uint64_t r = draw(seed, (uint64_t)j, (uint64_t)t) % (uint64_t)(t + 1);
      std::swap(v[(size_t)t], v[(size_t)r]);
    }
    mb_ptr_host[j] = pos;
    int64_t biggest = 0;
    for (int32_t g : v) {
      order_host[pos++] = g;
      biggest = std::max<int64_t>(biggest, sizes_host[g]);
    }
    // comm_free iff max size <= sum / d_gp  (compared without division)
    type_host[j] = (biggest * d_gp <= load[j]) ? MLIP_GARS_COMM_FREE : MLIP_GARS_DIST;
  }
  mb_ptr_host[n_mb] = pos;
  return MLIP_OK;
}
