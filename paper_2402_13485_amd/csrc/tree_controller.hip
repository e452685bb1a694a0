// Dynamic token-tree generation (Section 4.2): the controller that picks the tree size.
// Host code only: it runs between decoding steps, rarely (Section 4.2.3), on a few hundred
// numbers, and never touches the device.  State lives in caller-owned host memory.
//   Section 4.2.1  running mean of the iteration time per candidate size, weights that decay
//                  with the age of each mean, closed-form weighted line fit
//   Section 4.2.2  running top-k hit frequency per head, accuracy of the k-th ranked token as
//                  the difference of neighbouring frequencies, value of a node as the product
//                  of the accuracies along its path, the root worth 1
//   Section 4.2.3  expected accepted length over estimated time, one scan over the sizes
// The best tree of a size is grown best-first: node values never grow along a path (every
// accuracy is at most 1), so taking the most valuable frontier node each time yields the most
// valuable tree of every size, and the tree of a smaller size is a prefix of a larger one.
#include <math.h>
#include <stdint.h>
#include <string.h>

#include <algorithm>
#include <queue>
#include <vector>

#include "../../include/propd.h"

namespace {

constexpr uint32_t kMagic = 0x50435452u;  // marks an initialised state

struct Header {
  uint32_t magic;
  int32_t n_sizes, n_heads, k_max;
  double alpha, lambda;
  // followed by: int32 sizes[n_sizes] (padded to 8 bytes), double t_perf[n_sizes],
  // double last[n_sizes], uint8 seen[n_sizes] (padded), double P[n_heads*k_max]
};

struct View {
  Header *h;
  int32_t *sizes;
  double *t_perf, *last, *P;
  uint8_t *seen;
};

size_t pad8(size_t n) { return (n + 7) / 8 * 8; }

size_t state_bytes(int n_sizes, int n_heads, int k_max) {
  return pad8(sizeof(Header)) + pad8((size_t)n_sizes * 4) + (size_t)n_sizes * 8 * 2 +
         pad8((size_t)n_sizes) + (size_t)n_heads * k_max * 8;
}

View view_of(void *state) {
  View v;
  char *p = static_cast<char *>(state);
  v.h = reinterpret_cast<Header *>(p);
  p += pad8(sizeof(Header));
  const int n = v.h->n_sizes;
  v.sizes = reinterpret_cast<int32_t *>(p);
  p += pad8((size_t)n * 4);
  v.t_perf = reinterpret_cast<double *>(p);
  p += (size_t)n * 8;
  v.last = reinterpret_cast<double *>(p);
  p += (size_t)n * 8;
  v.seen = reinterpret_cast<uint8_t *>(p);
  p += pad8((size_t)n);
  v.P = reinterpret_cast<double *>(p);
  return v;
}

bool usable(const void *state) {
  return state && reinterpret_cast<uintptr_t>(state) % 8 == 0 &&
         static_cast<const Header *>(state)->magic == kMagic;
}

// accuracy of the rank-k token of a head: P^k - P^(k-1), P^0 = 0 (k is 0-based here)
double rank_accuracy(const View &v, int head, int k) {
  const double *row = v.P + (size_t)head * v.h->k_max;
  return k == 0 ? row[0] : row[k] - row[k - 1];
}

bool fit_line(const View &v, double now, double *beta0, double *beta1) {
  double sw = 0, sx = 0, sy = 0, sxx = 0, sxy = 0;
  for (int j = 0; j < v.h->n_sizes; ++j) {
    if (!v.seen[j]) continue;
    const double w = exp(-v.h->lambda * (now - v.last[j])), x = v.sizes[j], y = v.t_perf[j];
    sw += w;
    sx += w * x;
    sy += w * y;
    sxx += w * x * x;
    sxy += w * x * y;
  }
  if (!(sw > 0)) return false;
  const double den = sw * sxx - sx * sx;
  if (!(den > 1e-12 * sw * sxx)) {  // one size seen (or all weight on one): slope undetermined
    *beta0 = sy / sw;
    *beta1 = 0;
    return true;
  }
  *beta1 = (sw * sxy - sx * sy) / den;
  *beta0 = (sy - *beta1 * sx) / sw;
  return true;
}

struct Cand {
  double value;
  int depth, parent, choice;  // parent: index of the parent in the output order
};
struct Worse {
  // the queue's top is the most valuable candidate; ties go to the shallower node, then to
  // the parent placed earlier, then to the lower rank
  bool operator()(const Cand &a, const Cand &b) const {
    if (a.value != b.value) return a.value < b.value;
    if (a.depth != b.depth) return a.depth > b.depth;
    if (a.parent != b.parent) return a.parent > b.parent;
    return a.choice > b.choice;
  }
};

// Grows the best tree up to `size` nodes (root included).  Returns the number of nodes placed:
// fewer than `size` only when the heads cannot supply that many candidates.
int grow_tree(const View &v, int size, int32_t *parent, int32_t *depth, int32_t *choice,
              double *node_value) {
  std::priority_queue<Cand, std::vector<Cand>, Worse> frontier;
  auto push_children = [&](int idx, int d, double val) {
    if (d >= v.h->n_heads) return;
    for (int k = 0; k < v.h->k_max; ++k)
      frontier.push(Cand{val * rank_accuracy(v, d, k), d + 1, idx, k});
  };
  int n = 0;
  auto place = [&](const Cand &c) {
    if (parent) parent[n] = c.parent;
    if (depth) depth[n] = c.depth;
    if (choice) choice[n] = c.choice;
    if (node_value) node_value[n] = c.value;
    ++n;
  };
  place(Cand{1.0, 0, -1, -1});
  push_children(0, 0, 1.0);
  while (n < size && !frontier.empty()) {
    const Cand c = frontier.top();
    frontier.pop();
    const int idx = n;
    place(c);
    push_children(idx, c.depth, c.value);
  }
  return n;
}

}  // namespace

extern "C" size_t propd_controller_bytes(int32_t n_sizes, int32_t n_heads, int32_t k_max) {
  if (n_sizes < 1 || n_heads < 1 || k_max < 1 || n_sizes > (1 << 20) ||
      (long long)n_heads * k_max > (1 << 24))
    return 0;
  return state_bytes(n_sizes, n_heads, k_max);
}

extern "C" propd_status propd_controller_init(void *state, size_t bytes, const int32_t *sizes,
                                              int32_t n_sizes, int32_t n_heads, int32_t k_max,
                                              double alpha, double lambda,
                                              const double *hit_rate_init) {
  const size_t need = propd_controller_bytes(n_sizes, n_heads, k_max);
  if (!state || !sizes || need == 0 || reinterpret_cast<uintptr_t>(state) % 8 != 0)
    return PROPD_ERR_INVALID_ARG;
  if (bytes < need) return PROPD_ERR_WORKSPACE;
  if (!(alpha > 0.0 && alpha <= 1.0) || !(lambda >= 0.0)) return PROPD_ERR_INVALID_ARG;
  for (int j = 0; j < n_sizes; ++j) {
    if (sizes[j] < 1 || sizes[j] > PROPD_MAX_TREE) return PROPD_ERR_INVALID_ARG;
    if (j > 0 && sizes[j] <= sizes[j - 1]) return PROPD_ERR_INVALID_ARG;  // strictly rising
  }
  if (hit_rate_init)
    for (int i = 0; i < n_heads; ++i)
      for (int k = 0; k < k_max; ++k) {
        const double x = hit_rate_init[(size_t)i * k_max + k];
        if (!(x >= 0.0 && x <= 1.0)) return PROPD_ERR_INVALID_ARG;
        if (k > 0 && x < hit_rate_init[(size_t)i * k_max + k - 1]) return PROPD_ERR_INVALID_ARG;
      }
  memset(state, 0, need);
  Header *h = static_cast<Header *>(state);
  h->n_sizes = n_sizes;
  h->n_heads = n_heads;
  h->k_max = k_max;
  h->alpha = alpha;
  h->lambda = lambda;
  View v = view_of(state);
  memcpy(v.sizes, sizes, (size_t)n_sizes * 4);
  if (hit_rate_init) memcpy(v.P, hit_rate_init, (size_t)n_heads * k_max * 8);
  h->magic = kMagic;
  return PROPD_OK;
}

extern "C" propd_status propd_controller_observe_time(void *state, int32_t size, double t, double now) {
  if (!usable(state) || !(t >= 0.0) || !isfinite(t) || !isfinite(now)) return PROPD_ERR_INVALID_ARG;
  View v = view_of(state);
  const int32_t *begin = v.sizes, *end = v.sizes + v.h->n_sizes;
  const int32_t *it = std::lower_bound(begin, end, size);
  if (it == end || *it != size) return PROPD_ERR_INVALID_ARG;
  const int j = (int)(it - v.sizes);
  if (!v.seen[j]) {
    v.t_perf[j] = t;  // the first sample starts the mean
    v.seen[j] = 1;
  } else {
    v.t_perf[j] = (1.0 - v.h->alpha) * v.t_perf[j] + v.h->alpha * t;
  }
  v.last[j] = now;
  return PROPD_OK;
}

extern "C" propd_status propd_controller_observe_hit(void *state, int32_t head, int32_t rank) {
  if (!usable(state)) return PROPD_ERR_INVALID_ARG;
  View v = view_of(state);
  if (head < 0 || head >= v.h->n_heads) return PROPD_ERR_INVALID_ARG;
  double *row = v.P + (size_t)head * v.h->k_max;
  for (int k = 0; k < v.h->k_max; ++k) {
    const double hit = (rank >= 0 && rank <= k) ? 1.0 : 0.0;  // within the top-(k+1)
    row[k] = (1.0 - v.h->alpha) * row[k] + v.h->alpha * hit;
  }
  return PROPD_OK;
}

extern "C" propd_status propd_controller_fit(const void *state, double now, double *beta0, double *beta1) {
  if (!usable(state) || !beta0 || !beta1 || !isfinite(now)) return PROPD_ERR_INVALID_ARG;
  const View v = view_of(const_cast<void *>(state));
  return fit_line(v, now, beta0, beta1) ? PROPD_OK : PROPD_ERR_UNSUPPORTED;
}

extern "C" propd_status propd_controller_build_tree(const void *state, int32_t size, int32_t *n_built,
                                                    int32_t *parent, int32_t *depth, int32_t *choice,
                                                    double *node_value, double *expected_len) {
  if (!usable(state) || size < 1 || size > PROPD_MAX_TREE || !n_built) return PROPD_ERR_INVALID_ARG;
  const View v = view_of(const_cast<void *>(state));
  double values[PROPD_MAX_TREE];
  const int n = grow_tree(v, size, parent, depth, choice, values);
  double total = 0;
  for (int i = 0; i < n; ++i) total += values[i];
  if (node_value) memcpy(node_value, values, (size_t)n * 8);
  if (expected_len) *expected_len = total;
  *n_built = n;
  return PROPD_OK;
}

extern "C" propd_status propd_controller_best_size(const void *state, double now, int32_t *best_size,
                                                   double *speed, double *beta0, double *beta1) {
  if (!usable(state) || !best_size || !isfinite(now)) return PROPD_ERR_INVALID_ARG;
  const View v = view_of(const_cast<void *>(state));
  double b0, b1;
  if (!fit_line(v, now, &b0, &b1)) return PROPD_ERR_UNSUPPORTED;
  if (beta0) *beta0 = b0;
  if (beta1) *beta1 = b1;
  // one growth to the largest size; the value of size i is the sum over its first i nodes
  double values[PROPD_MAX_TREE];
  const int largest = v.sizes[v.h->n_sizes - 1];
  const int n = grow_tree(v, largest, nullptr, nullptr, nullptr, values);
  double best_v = -1.0, len = 0;
  int placed = 0;
  for (int j = 0; j < v.h->n_sizes; ++j) {
    const int want = v.sizes[j] < n ? v.sizes[j] : n;
    while (placed < want) len += values[placed++];
    const double t_est = b0 + b1 * v.sizes[j];
    const double s = t_est > 0.0 ? len / t_est : 0.0;
    if (speed) speed[j] = s;
    if (s > best_v) {  // ties keep the smaller size
      best_v = s;
      *best_size = v.sizes[j];
    }
  }
  return PROPD_OK;
}
