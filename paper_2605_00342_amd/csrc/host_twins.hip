// Host twins of the three small entry points (acceptance, prefix selection, expert union): the same
// contracts evaluated by plain sequential C++ on host arrays, no GPU involved. They exist for callers
// that hold these small arrays on the host anyway (a scheduler deciding a verification length, tests of
// the error conventions); nothing in the device path calls them and they are no fallback for it.
// Selection arithmetic: single IEEE fp32 operations in the order the header states (no contraction), so
// every output equals the device entry point's bit for bit.
#include <math.h>
#include <string.h>

#include <vector>

#include "common.h"

#pragma clang fp contract(off)

using namespace evict;

namespace {
constexpr int kMaxSelectNodes = EVICT_MAX_SELECT_NODES;

// one tree of the selection; returns the status bits it met
int select_one(const int32_t* parent, const float* prob, const float* cost, float rho, int kmax, int n, int32_t* k_star,
               float* est_len, int32_t* order, float* psum, int32_t* keep, int32_t* new_parent) {
  int st = 0;
  std::vector<int> par(n), rank(n), newi(n);
  std::vector<float> q(n), c(n), score(n), sorted(n);
  for (int i = 0; i < n; ++i) {
    int p = parent[i];
    if (i == 0) p = -1;
    else if (p < 0 || p >= i) { p = 0; st |= ST_BAD_PARENT; }
    par[i] = p;
    float qi = prob[i];
    if (i > 0 && !(qi >= 0.0f && qi <= 1.0f)) { qi = qi > 1.0f ? 1.0f : 0.0f; st |= ST_BAD_PROB; }
    q[i] = qi;
    float ci = (cost && i < kmax) ? cost[i + 1] : 1.0f;
    if (!(ci > 0.0f)) { ci = 0.0f; st |= ST_BAD_COST; }
    c[i] = ci;
  }
  // Eq. 7: one rounded multiply per node, parents first (parent ids are smaller than their children's)
  score[0] = 1.0f;
  for (int i = 1; i < n; ++i) {
    volatile float s = score[par[i]] * q[i];
    score[i] = s;
  }
  // ranking by (score descending, index ascending)
  for (int i = 0; i < n; ++i) {
    int r = 0;
    for (int j = 0; j < n; ++j) r += (score[j] > score[i] || (score[j] == score[i] && j < i)) ? 1 : 0;
    rank[i] = r;
    sorted[r] = score[i];
    if (order) order[r] = i;
  }
  // Eq. 8: sequential running sum over the ranking
  volatile float acc = 0.0f;
  for (int r = 0; r < n; ++r) {
    acc = acc + sorted[r];
    sorted[r] = acc;
    if (psum) psum[r] = acc;
  }
  // Eq. 10 (or the coverage rule): first maximum over 1..min(n, kmax)
  const int kk = n < kmax ? n : kmax;
  float bv = -1.0f;
  int bi = 0x7fffffff;
  for (int i = 0; i < kk; ++i) {
    float u;
    if (rho >= 0.0f) {
      volatile float ratio = sorted[i] / sorted[n - 1];
      u = ratio >= rho ? 1.0f : 0.0f;
    } else if (c[i] > 0.0f) {
      volatile float ratio = sorted[i] / c[i];
      u = ratio;
    } else {
      u = -1.0f;
    }
    if (u > bv || (u == bv && i < bi)) { bv = u; bi = i; }
  }
  if (rho >= 0.0f && bv == 0.0f) bi = kk - 1;
  const int ks = bi + 1;
  *k_star = ks;
  *est_len = sorted[bi];
  // compaction: kept nodes ascending, parents re-indexed
  int out = 0;
  for (int i = 0; i < n; ++i) newi[i] = rank[i] < ks ? out++ : -1;
  for (int i = 0; i < n; ++i)
    if (newi[i] >= 0) {
      keep[newi[i]] = i;
      new_parent[newi[i]] = par[i] < 0 ? -1 : newi[par[i]];
    }
  return st;
}

int select_host_impl(const char* who, const int32_t* tree_off, const int32_t* parent, const float* node_prob, int B, int T,
                     const float* cost, float rho, int Kmax, int32_t* k_star, int32_t* keep, int32_t* new_parent,
                     int32_t* new_tree_off, float* est_len, int32_t* order, float* prefix_sum, int32_t* status_out) {
  EVICT_REQUIRE(tree_off && parent && node_prob && k_star && keep && new_parent && new_tree_off && est_len, EVICT_E_INVALID,
                "%s: null pointer argument", who);
  EVICT_REQUIRE(B >= 1 && T >= B, EVICT_E_INVALID, "%s: need B >= 1 and T >= B (B=%d, T=%d)", who, B, T);
  EVICT_REQUIRE(Kmax >= 1, EVICT_E_INVALID, "%s: Kmax must be >= 1 (got %d)", who, Kmax);
  EVICT_REQUIRE(T <= B * (int64_t)kMaxSelectNodes, EVICT_E_UNSUPPORTED, "%s: more than %d nodes per tree", who, kMaxSelectNodes);
  int st = 0, out = 0;
  // (outputs must not alias inputs, as for the device entry point)
  for (int b = 0; b < B; ++b) {
    const int lo = B == 1 ? 0 : tree_off[b];
    int n = B == 1 ? T : tree_off[b + 1] - lo;
    n = n < 1 ? 1 : (n > kMaxSelectNodes ? kMaxSelectNodes : n);
    new_tree_off[b] = out;
    st |= select_one(parent + lo, node_prob + lo, cost, rho, Kmax, n, k_star + b, est_len + b, order ? order + lo : nullptr,
                     prefix_sum ? prefix_sum + lo : nullptr, keep + out, new_parent + out);
    out += k_star[b];
  }
  new_tree_off[B] = out;
  if (status_out) *status_out |= st;
  return EVICT_OK;
}
}  // namespace

extern "C" {

int evict_accept_path_host(const int32_t* tree_off, const int32_t* parent, const int32_t* draft_tok, const int32_t* target_next,
                           int B, int32_t* path, int path_stride, int32_t* path_len, int32_t* bonus_tok) {
  EVICT_REQUIRE(tree_off && parent && draft_tok && target_next && path && path_len && bonus_tok, EVICT_E_INVALID,
                "evict_accept_path_host: null pointer argument");
  EVICT_REQUIRE(B >= 1, EVICT_E_INVALID, "evict_accept_path_host: B must be >= 1 (got %d)", B);
  EVICT_REQUIRE(path_stride >= 1, EVICT_E_INVALID, "evict_accept_path_host: path_stride must be >= 1");
  for (int b = 0; b < B; ++b) {
    const int lo = tree_off[b];
    int n = tree_off[b + 1] - lo;
    n = n < 1 ? 1 : (n > kMaxSelectNodes ? kMaxSelectNodes : n);
    int32_t* my = path + (size_t)b * path_stride;
    for (int i = 0; i < path_stride; ++i) my[i] = i == 0 ? 0 : -1;
    int cur = 0, len = 1;
    while (true) {
      const int want = target_next[lo + cur];
      int found = -1;
      for (int c = cur + 1; c < n && found < 0; ++c)  // children have larger ids than their parent
        if (parent[lo + c] == cur && draft_tok[lo + c] == want) found = c;
      if (found < 0) break;
      cur = found;
      if (len < path_stride) my[len] = cur;
      ++len;
    }
    path_len[b] = len;
    bonus_tok[b] = target_next[lo + cur];
  }
  return EVICT_OK;
}

int evict_select_prefix_host(const int32_t* tree_off, const int32_t* parent, const float* node_prob, int B, int T,
                             const float* cost, int Kmax, int32_t* k_star, int32_t* keep, int32_t* new_parent,
                             int32_t* new_tree_off, float* est_len, int32_t* order, float* prefix_sum, int32_t* status_out) {
  EVICT_REQUIRE(cost, EVICT_E_INVALID, "evict_select_prefix_host: null cost table");
  return select_host_impl("evict_select_prefix_host", tree_off, parent, node_prob, B, T, cost, -1.0f, Kmax, k_star, keep, new_parent,
                          new_tree_off, est_len, order, prefix_sum, status_out);
}

int evict_select_prefix_coverage_host(const int32_t* tree_off, const int32_t* parent, const float* node_prob, int B, int T,
                                      float rho, int Kmax, int32_t* k_star, int32_t* keep, int32_t* new_parent,
                                      int32_t* new_tree_off, float* est_len, int32_t* order, float* prefix_sum,
                                      int32_t* status_out) {
  EVICT_REQUIRE(rho >= 0.0f && rho <= 1.0f, EVICT_E_INVALID, "evict_select_prefix_coverage_host: rho=%g outside [0, 1]", (double)rho);
  return select_host_impl("evict_select_prefix_coverage_host", tree_off, parent, node_prob, B, T, nullptr, rho, Kmax, k_star, keep,
                          new_parent, new_tree_off, est_len, order, prefix_sum, status_out);
}

int evict_expert_union_host(const int32_t* topk_idx, int T, int k, int E, int32_t* union_ids, int32_t* union_count, int32_t* hist,
                            int32_t* offsets, int32_t* perm, int32_t* inv, int32_t* status_out) {
  EVICT_REQUIRE(topk_idx && union_ids && union_count && hist && offsets && perm && inv, EVICT_E_INVALID,
                "evict_expert_union_host: null pointer argument");
  EVICT_REQUIRE(T >= 1 && k >= 1 && E >= 1, EVICT_E_INVALID, "evict_expert_union_host: T, k, E must be >= 1");
  EVICT_REQUIRE(k <= E, EVICT_E_INVALID, "evict_expert_union_host: k=%d exceeds E=%d", k, E);
  EVICT_REQUIRE((int64_t)T * k <= 8192 && E <= 1024, EVICT_E_UNSUPPORTED, "evict_expert_union_host: T*k=%lld (limit 8192), E=%d (limit 1024)",
                (long long)T * k, E);
  const int P = T * k;
  int st = 0;
  std::vector<int> idx(P), next(E + 1);
  memset(hist, 0, sizeof(int32_t) * (size_t)E);
  for (int p = 0; p < P; ++p) {
    int e = topk_idx[p];
    if (e < 0 || e >= E) { e = 0; st |= ST_BAD_EXPERT; }  // clamped and flagged, as on the device
    idx[p] = e;
    ++hist[e];
  }
  int nu = 0, run = 0;
  for (int e = 0; e < E; ++e) {
    offsets[e] = run;
    next[e] = run;
    run += hist[e];
    if (hist[e] > 0) union_ids[nu++] = e;
  }
  offsets[E] = run;
  for (int e = nu; e < E; ++e) union_ids[e] = -1;
  union_count[0] = nu;
  for (int p = 0; p < P; ++p) {  // ascending pair id inside every expert: the stable grouping of Eq. 5
    const int pos = next[idx[p]]++;
    perm[pos] = p;
    inv[p] = pos;
  }
  if (status_out) *status_out |= st;
  return EVICT_OK;
}

}  // extern "C"
