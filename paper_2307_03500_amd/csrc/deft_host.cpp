// Host side of the DEFT selection path: Alg. 2 (partition), Alg. 3 (local k), Alg. 4
// (bin-packing) and the cost model of Eq. 3-8.  Integer and IEEE fp64 arithmetic only; this
// file must be compiled without floating-point contraction so that every product and sum
// rounds once, in the order written.
#include "deft.h"

#include <algorithm>
#include <cmath>
#include <cstring>
#include <numeric>
#include <vector>

namespace {
constexpr int64_t kMaxN = (int64_t(1) << 31) - 1;
}

extern "C" const char* deft_strerror(int status) {
  switch (status) {
    case DEFT_OK: return "ok";
    case DEFT_EINVAL: return "invalid argument";
    case DEFT_ERANGE: return "vector too long: indices are 32-bit, N must be below 2^31";
    case DEFT_EWS: return "workspace too small";
    case DEFT_ECAP: return "output capacity too small";
    case DEFT_EHIP: return "HIP runtime error";
    case DEFT_ELIMIT: return "vector longer than the built-in scratch of the no-allocation entry point allows";
    default: return "unknown status";
  }
}

// Alg. 2 (Sec. 4.1).  A tensor is cut when it holds more than n_g / n_workers elements; for
// integer sizes that is the predicate size * n_workers > n_g whether the quotient is taken as
// real or integer.  Fraction i of a cut tensor of s = q * n + r elements (0 <= r < n) is the
// half-open range [i*q + min(i, r), (i+1)*q + min(i+1, r)) of the tensor: the first r fractions
// hold q + 1 elements, the others q, and together they tile the tensor.  Ranges that come out
// empty (s < n) produce no layer.
namespace {
inline int64_t fraction_begin(int64_t q, int64_t r, int64_t i) { return i * q + std::min(i, r); }
}  // namespace

extern "C" int deft_partition(const int64_t* tensor_sizes, int32_t T, int32_t n_workers,
                              int64_t* offsets, int32_t* layer_tensor, int32_t cap,
                              int32_t* L_out) {
  if (!tensor_sizes || !offsets || !L_out || T < 0 || n_workers < 1 || cap < 0) return DEFT_EINVAL;
  int64_t n_g = 0;
  for (int32_t t = 0; t < T; ++t) {
    if (tensor_sizes[t] < 0) return DEFT_EINVAL;
    n_g += tensor_sizes[t];
    if (n_g > kMaxN) return DEFT_ERANGE;
  }
  const int64_t n = n_workers;
  // layers each tensor contributes: 0 (empty), 1 (kept whole) or min(s, n) (cut)
  int64_t need = 0;
  for (int32_t t = 0; t < T; ++t) {
    const int64_t s = tensor_sizes[t];
    need += s == 0 ? 0 : (s * n > n_g ? std::min(s, n) : 1);
  }
  if (need > cap) return DEFT_ECAP;  // nothing written
  int32_t L = 0;
  int64_t base = 0;  // first element of tensor t in the flat vector
  offsets[0] = 0;
  for (int32_t t = 0; t < T; ++t) {
    const int64_t s = tensor_sizes[t];
    const bool cut = s * n > n_g;
    const int64_t parts = s == 0 ? 0 : (cut ? std::min(s, n) : 1);
    const int64_t q = cut ? s / n : s, r = cut ? s % n : 0;
    for (int64_t i = 0; i < parts; ++i) {
      if (layer_tensor) layer_tensor[L] = t;
      offsets[++L] = base + fraction_begin(q, r, i + 1);
    }
    base += s;
  }
  *L_out = L;
  return DEFT_OK;
}

extern "C" int deft_check_layout(const int64_t* offsets, int32_t L, int64_t N) {
  if (!offsets || L < 1 || N < 0) return DEFT_EINVAL;
  if (N > kMaxN) return DEFT_ERANGE;
  if (offsets[0] != 0 || offsets[L] != N) return DEFT_EINVAL;
  for (int32_t l = 0; l < L; ++l)
    if (offsets[l + 1] < offsets[l]) return DEFT_EINVAL;
  return DEFT_OK;
}

namespace {
// Sorting by (value descending, position ascending) for non-negative finite doubles: their bit
// patterns order like the values, so one integer compare of (~bits, position) does both.
// Adding +0.0 turns a -0.0 into +0.0, which compares equal and must sort as equal.
typedef unsigned __int128 SortKey;
void sort_descending(const double* v, int32_t L, std::vector<SortKey>& out) {
  out.resize(L);
  for (int32_t l = 0; l < L; ++l) {
    const double x = v[l] + 0.0;
    uint64_t bits;
    std::memcpy(&bits, &x, sizeof bits);
    out[l] = ((SortKey)(~bits) << 32) | (uint32_t)l;
  }
  std::sort(out.begin(), out.end());
}
}  // namespace

// First statement of Alg. 3 (k = n_g * d; density as defined in the footnote of Sec. 1), made an
// integer by rounding half up in fp64.
extern "C" int deft_total_k(int64_t N, double d, int64_t* K_out) {
  if (!K_out || N < 1 || N > kMaxN) return N > kMaxN ? DEFT_ERANGE : DEFT_EINVAL;
  if (!(d > 0.0) || !(d <= 1.0)) return DEFT_EINVAL;
  *K_out = (int64_t)std::floor((double)N * d + 0.5);
  return DEFT_OK;
}

// Cyclic local Top-k (Sec. 1; Sec. 3.1): workers take turns, one per iteration.
extern "C" int deft_cltk_leader(int64_t iteration, int32_t n_workers, int32_t* leader_out) {
  if (!leader_out || n_workers < 1 || iteration < 0) return DEFT_EINVAL;
  *leader_out = (int32_t)(iteration % n_workers);
  return DEFT_OK;
}

extern "C" int deft_norms_from_sumsq(const double* sumsq, int32_t L, double* norms) {
  if (!sumsq || !norms || L < 1) return DEFT_EINVAL;
  for (int32_t l = 0; l < L; ++l)
    if (!(sumsq[l] >= 0.0)) return DEFT_EINVAL;
  for (int32_t l = 0; l < L; ++l) norms[l] = std::sqrt(sumsq[l]);
  return DEFT_OK;
}

// Alg. 3.  norm_remain for the layer served at step j is the sum of the norms from step j to
// the end, accumulated from the end: the same quantity the listing obtains by subtracting the
// served norms from the grand total, but free of cancellation, so the last layer's ratio is
// exactly 1 and no ratio exceeds 1.
extern "C" int deft_alloc_k(const double* norms, const int64_t* sizes, int32_t L, int64_t N,
                            double d, int64_t* k_out) {
  if (!norms || !sizes || !k_out || L < 1 || N < 1) return DEFT_EINVAL;
  if (!(d > 0.0) || !(d <= 1.0)) return DEFT_EINVAL;
  for (int32_t l = 0; l < L; ++l) {
    if (sizes[l] < 1) return DEFT_EINVAL;
    if (!(norms[l] >= 0.0) || !std::isfinite(norms[l])) return DEFT_EINVAL;
  }
  // priority order: norm descending, position ascending among equal norms
  thread_local std::vector<SortKey> keyed;
  thread_local std::vector<int32_t> order;
  thread_local std::vector<double> norm_remain;
  sort_descending(norms, L, keyed);
  order.resize(L);
  for (int32_t j = 0; j < L; ++j) order[j] = (int32_t)(uint32_t)keyed[j];
  norm_remain.resize(L);
  double acc = 0.0;
  for (int32_t j = L - 1; j >= 0; --j) {
    acc = norms[order[j]] + acc;
    norm_remain[j] = acc;
  }
  int64_t k_remain = 0;
  const int rc = deft_total_k(N, d, &k_remain);
  if (rc != DEFT_OK) return rc;
  for (int32_t j = 0; j < L; ++j) {
    const int32_t l = order[j];
    double k_temp = 0.0;
    if (norm_remain[j] > 0.0) {
      const double ratio = norms[l] / norm_remain[j];
      k_temp = (double)k_remain * ratio;
    }
    int64_t k;
    if ((double)sizes[l] < k_temp) k = sizes[l];
    else if (k_temp < 2.0) k = 1;     // max(1, floor(k_temp)), also for a k_remain gone negative
    else k = (int64_t)k_temp;         // floor of a positive value below 2^31: truncation
    k_out[l] = k;
    k_remain -= k;
  }
  return DEFT_OK;
}

namespace {
bool check_sizes_k(const int64_t* sizes, const int64_t* k, int32_t L) {
  for (int32_t l = 0; l < L; ++l)
    if (sizes[l] < 1 || k[l] < 1 || k[l] > sizes[l]) return false;
  return true;
}
}  // namespace

// Alg. 4.  The listing rescans the cost list for its maximum and the bin loads for their
// minimum at every step, taking the first occurrence of each; the same choices are made here
// by visiting the layers once in (cost descending, position ascending) order and keeping the
// bins in a heap ordered by (load, id).  ln(1) is exactly 0, so k = 1 layers skip the call.
extern "C" int deft_assign_layers(const int64_t* sizes, const int64_t* k, int32_t L,
                                  int32_t n_workers, int64_t iteration, int32_t rank,
                                  int32_t* owner_bin, int32_t* my_layers, int32_t* my_count) {
  if (!sizes || !k || !owner_bin || !my_layers || !my_count) return DEFT_EINVAL;
  if (L < 1 || n_workers < 1 || rank < 0 || rank >= n_workers || iteration < 0) return DEFT_EINVAL;
  if (!check_sizes_k(sizes, k, L)) return DEFT_EINVAL;
  // the bin -> worker map turns by one place per iteration
  const int32_t my_bin = (int32_t)((iteration % n_workers + rank) % n_workers);
  // layers in (cost descending, position ascending) order
  thread_local std::vector<double> cost;
  thread_local std::vector<SortKey> item;
  thread_local std::vector<std::pair<double, int32_t>> heap;
  cost.resize(L);
  for (int32_t l = 0; l < L; ++l)
    cost[l] = k[l] == 1 ? 0.0 : (double)sizes[l] * std::log((double)k[l]);
  sort_descending(cost.data(), L, item);
  // bins as a binary min-heap on (load, id): its top is the first bin of minimal load
  heap.resize(n_workers);
  for (int32_t b = 0; b < n_workers; ++b) heap[b] = {0.0, b};  // already a valid heap
  const auto lighter = [](const std::pair<double, int32_t>& a, const std::pair<double, int32_t>& b) {
    return a.first < b.first || (a.first == b.first && a.second < b.second);
  };
  int32_t cnt = 0;
  for (int32_t j = 0; j < L; ++j) {
    const int32_t layer = (int32_t)(uint32_t)item[j];  // costliest layer not yet placed
    const int32_t lightest = heap[0].second;
    owner_bin[layer] = lightest;
    if (lightest == my_bin) my_layers[cnt++] = layer;
    heap[0].first = heap[0].first + cost[layer];
    // sift the grown bin down
    int32_t i = 0;
    for (;;) {
      const int32_t a = 2 * i + 1, b = a + 1;
      int32_t best = i;
      if (a < n_workers && lighter(heap[a], heap[best])) best = a;
      if (b < n_workers && lighter(heap[b], heap[best])) best = b;
      if (best == i) break;
      std::swap(heap[i], heap[best]);
      i = best;
    }
  }
  *my_count = cnt;
  return DEFT_OK;
}

// Eq. 4-8.
extern "C" int deft_cost_model(const int64_t* sizes, const int64_t* k, const int32_t* owner_bin,
                               int32_t L, int32_t n_workers, int64_t N, int64_t K, double* C_i,
                               double* out5) {
  if (!sizes || !k || !owner_bin || !out5 || L < 1 || n_workers < 1 || N < 1 || K < 1)
    return DEFT_EINVAL;
  if (!check_sizes_k(sizes, k, L)) return DEFT_EINVAL;
  std::vector<double> load(n_workers, 0.0);
  for (int32_t l = 0; l < L; ++l) {
    if (owner_bin[l] < 0 || owner_bin[l] >= n_workers) return DEFT_EINVAL;
    load[owner_bin[l]] += (double)sizes[l] * std::log((double)k[l]);
  }
  const double C_n = *std::max_element(load.begin(), load.end());
  const double topk = (double)N * std::log((double)K);
  const double C_triv = K > n_workers ? ((double)N / n_workers) * std::log((double)K / n_workers) : 0.0;
  if (C_i) std::copy(load.begin(), load.end(), C_i);
  out5[0] = C_n;
  out5[1] = C_n > 0.0 ? topk / C_n : INFINITY;
  out5[2] = C_triv;
  out5[3] = C_triv > 0.0 ? topk / C_triv : INFINITY;
  out5[4] = topk;
  return DEFT_OK;
}
