// Integer / latency-bound parts of the verification step: EVICT prefix selection
// (Sec. 3.1-3.2), greedy acceptance (Sec. 2.1, temperature 0), the expert union and the
// token grouping it induces (Eq. 5), row gather for tree compaction.
#include <stdarg.h>
#include <string.h>

#include <mutex>

#include "ctx.h"
#include "union_device.h"

namespace evict {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}

namespace {

constexpr int kSelThreads = 256;
constexpr int kMaxSel = EVICT_MAX_SELECT_NODES;

// Kept-set compaction of one tree: nodes with rank < kstar, ascending node id; parents
// re-indexed into the kept set. s_flag/s_new are LDS arrays of n ints.
__device__ void compact_tree(int n, int kstar, const int* s_par, const int* s_rank, int* s_new, int* s_wave,
                             int32_t* keep_out, int32_t* newpar_out) {
  const int tid = threadIdx.x;
  // 4 consecutive nodes per thread so that the scan keeps node order
  int f[4], cnt = 0;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    int i = tid * 4 + j;
    f[j] = (i < n && s_rank[i] < kstar) ? 1 : 0;
    cnt += f[j];
  }
  int total;
  int base = block_excl_scan(cnt, s_wave, &total);
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    int i = tid * 4 + j;
    if (i < n) s_new[i] = f[j] ? base : -1;
    base += f[j];
  }
  __syncthreads();
  for (int i = tid; i < n; i += blockDim.x) {
    int ni = s_new[i];
    if (ni >= 0) {
      keep_out[ni] = i;
      int p = s_par[i];
      newpar_out[ni] = p < 0 ? -1 : s_new[p];
    }
  }
}

// One workgroup per tree. Writes k*, S_{k*}, the ranking and the running sums; when
// `single` it also writes the compacted tree (B == 1), otherwise ranks go to rank_ws for
// the second kernel.
__global__ __launch_bounds__(kSelThreads) void select_prefix_kernel(
    const int32_t* __restrict__ tree_off, const int32_t* __restrict__ parent, const float* __restrict__ prob,
    const float* __restrict__ cost, int kmax, int32_t* __restrict__ k_star, float* __restrict__ est_len,
    int32_t* __restrict__ order_out, float* __restrict__ psum_out, int32_t* rank_ws, int single, int32_t* keep,
    int32_t* new_parent, int32_t* __restrict__ new_tree_off, int n_single, float rho, int32_t* __restrict__ status) {
  __shared__ int s_par[kMaxSel];
  __shared__ __attribute__((aligned(16))) float s_score[kMaxSel];
  __shared__ float s_sorted[kMaxSel];
  __shared__ float s_prob[kMaxSel];
  __shared__ float s_cost[kMaxSel];
  __shared__ int s_rank[kMaxSel];
  __shared__ int s_aux[kMaxSel];  // depth, later new index
  __shared__ int s_wave[16];
  __shared__ float s_bestv[4];
  __shared__ int s_besti[4];
  __shared__ int s_maxdep;

  const int b = blockIdx.x, tid = threadIdx.x, lane = lane_id(), w = tid >> 6;
  const int nthreads = blockDim.x, nwaves = nthreads >> 6;  // 64 threads for small trees: barriers cost nothing
  // a single tree spans [0, T): its offsets need not be fetched
  const int lo = n_single > 0 ? 0 : tree_off[b];
  int n = n_single > 0 ? n_single : tree_off[b + 1] - lo;
  n = n < 1 ? 1 : (n > kMaxSel ? kMaxSel : n);

  if (tid == 0) s_maxdep = 0;
  int bad_in = 0;
  for (int i = tid; i < n; i += nthreads) {
    int p = parent[lo + i];
    if (i == 0) p = -1;
    else if (p < 0 || p >= i) { p = 0; bad_in |= ST_BAD_PARENT; }  // invalid ids are clamped and flagged
    s_par[i] = p;
    // all global reads issued together, up front. A probability outside [0, 1] (or NaN) could rank a child
    // above its parent and break the ancestor-closure of the prefixes (Sec. 3.2.1): it is clamped and flagged.
    float q = prob[lo + i];
    if (i > 0 && !(q >= 0.0f && q <= 1.0f)) { q = q > 1.0f ? 1.0f : 0.0f; bad_in |= ST_BAD_PROB; }
    s_prob[i] = q;
    float c = (cost && i < kmax) ? cost[i + 1] : 1.0f;  // s_cost[i] = C(i + 1)
    if (!(c > 0.0f)) { c = 0.0f; bad_in |= ST_BAD_COST; }  // (never selected below)
    s_cost[i] = c;
  }
  if (bad_in && status) atomicOr(status, bad_in);
  __syncthreads();
  // depth of every node (walk to the root; parent ids strictly decrease)
  int mydep_max = 0;
  for (int i = tid; i < n; i += nthreads) {
    int dep = 0;
    for (int p = s_par[i]; p >= 0; p = s_par[p]) ++dep;
    s_aux[i] = dep;
    mydep_max = dep > mydep_max ? dep : mydep_max;
  }
  atomicMax(&s_maxdep, mydep_max);
  if (tid == 0) s_score[0] = 1.0f;  // the root counts as probability 1 (Eq. 7)
  __syncthreads();
  const int maxdep = s_maxdep;
  // Score(v) = Score(parent(v)) * q(v): one rounded fp32 multiply per node, level by level
  for (int lvl = 1; lvl <= maxdep; ++lvl) {
    for (int i = tid; i < n; i += nthreads)
      if (s_aux[i] == lvl) s_score[i] = __fmul_rn(s_score[s_par[i]], s_prob[i]);
    __syncthreads();
  }
  // rank by (score descending, index ascending)
  for (int i = tid; i < n; i += nthreads) {
    const float si = s_score[i];
    int r = 0;
    int j = 0;
#pragma unroll 2
    for (; j + 4 <= n; j += 4) {  // LDS broadcast reads, four scores at a time
      const float4 s4 = *reinterpret_cast<const float4*>(&s_score[j]);
      r += (s4.x > si || (s4.x == si && j < i)) ? 1 : 0;
      r += (s4.y > si || (s4.y == si && j + 1 < i)) ? 1 : 0;
      r += (s4.z > si || (s4.z == si && j + 2 < i)) ? 1 : 0;
      r += (s4.w > si || (s4.w == si && j + 3 < i)) ? 1 : 0;
    }
    for (; j < n; ++j) {
      const float sj = s_score[j];
      r += (sj > si || (sj == si && j < i)) ? 1 : 0;
    }
    s_rank[i] = r;
    s_sorted[r] = si;
    if (order_out) order_out[lo + r] = i;
  }
  __syncthreads();
  // S_k: sequential fp32 running sum over the ranking (one wavefront, lane broadcast)
  if (w == 0) {
    float acc = 0.0f;
    for (int c = 0; c < n; c += 64) {
      const int idx = c + lane;
      const int vbits = __float_as_int(idx < n ? s_sorted[idx] : 0.0f);
      float mine = 0.0f;
      const int lim = (n - c) < 64 ? (n - c) : 64;
      for (int j = 0; j < lim; ++j) {
        acc = __fadd_rn(acc, __int_as_float(__builtin_amdgcn_readlane(vbits, j)));
        if (lane == j) mine = acc;
      }
      if (idx < n) s_sorted[idx] = mine;  // now holds S_{idx+1}
    }
  }
  __syncthreads();
  // u_k = S_k / cost[k]; k* = smallest k attaining the maximum over 1..min(n, kmax)
  const int kk = n < kmax ? n : kmax;
  float bv = -1.0f;
  int bi = 0x7fffffff;
  for (int i = tid; i < n; i += nthreads) {
    const float S = s_sorted[i];
    if (psum_out) psum_out[lo + i] = S;
    if (i < kk) {
      // cost-aware rule: u_k = S_k / C(k). Coverage rule (rho >= 0, the cost-agnostic ablation of
      // Sec. 4.3.2): u_k = 1 where S_k / S_n >= rho, else 0, so that the first maximum is the
      // smallest prefix reaching the coverage.
      float u;
      if (rho >= 0.0f) u = __fdiv_rn(S, s_sorted[n - 1]) >= rho ? 1.0f : 0.0f;
      else u = s_cost[i] > 0.0f ? __fdiv_rn(S, s_cost[i]) : -1.0f;  // (a flagged, unusable cost entry is never the maximum)
      if (u > bv || (u == bv && i < bi)) { bv = u; bi = i; }
    }
  }
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) {
    const float ov = __shfl_xor(bv, o);
    const int oi = __shfl_xor(bi, o);
    if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
  }
  if (lane == 0) { s_bestv[w] = bv; s_besti[w] = bi; }
  __syncthreads();
  bv = s_bestv[0]; bi = s_besti[0];
  for (int i = 1; i < nwaves; ++i) {
    const float ov = s_bestv[i];
    const int oi = s_besti[i];
    if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
  }
  if (rho >= 0.0f && bv == 0.0f) bi = kk - 1;  // coverage not reached within kmax: the whole budget
  const int kstar = bi + 1;
  if (tid == 0) {
    k_star[b] = kstar;
    est_len[b] = s_sorted[bi];
  }
  if (single) {
    if (tid == 0) { new_tree_off[0] = 0; new_tree_off[1] = kstar; }
    compact_tree(n, kstar, s_par, s_rank, s_aux, s_wave, keep, new_parent);
  } else {
    for (int i = tid; i < n; i += nthreads) rank_ws[lo + i] = s_rank[i];
  }
}

// One tree of at most 64 nodes in one wavefront, node i in lane i, everything in registers and
// cross-lane operations: the same arithmetic in the same order as select_prefix_kernel (one
// rounded multiply per node top-down, ranking by (score descending, index ascending), sequential
// fp32 running sum, IEEE division, first maximum), without LDS round trips and barriers.
__global__ __launch_bounds__(64) void select_prefix_wave_kernel(
    const int32_t* __restrict__ parent, const float* __restrict__ prob, const float* __restrict__ cost, int kmax, int n,
    float rho, int32_t* __restrict__ k_star, float* __restrict__ est_len, int32_t* __restrict__ order_out,
    float* __restrict__ psum_out, int32_t* __restrict__ keep, int32_t* __restrict__ new_parent,
    int32_t* __restrict__ new_tree_off, int32_t* __restrict__ status) {
  const int lane = threadIdx.x;
  const bool live = lane < n;
  int p = -1;
  float q = 0.0f, c = 1.0f;
  if (live) {
    int bad_in = 0;
    p = parent[lane];
    q = prob[lane];
    if (cost && lane < kmax) c = cost[lane + 1];  // C(lane + 1)
    if (lane == 0) p = -1;
    else if (p < 0 || p >= lane) { p = 0; bad_in |= ST_BAD_PARENT; }  // invalid ids are clamped and flagged
    // a probability outside [0, 1] (or NaN) could rank a child above its parent and break the ancestor-closure
    // of the prefixes (Sec. 3.2.1): clamped and flagged; an unusable cost entry is never selected
    if (lane > 0 && !(q >= 0.0f && q <= 1.0f)) { q = q > 1.0f ? 1.0f : 0.0f; bad_in |= ST_BAD_PROB; }
    if (!(c > 0.0f)) { c = 0.0f; bad_in |= ST_BAD_COST; }
    if (bad_in && status) atomicOr(status, bad_in);
  }
  // depth by walking up in lock step
  int dep = 0, a = p;
  while (__ballot(a >= 0)) {
    const int up = __shfl(p, a < 0 ? 0 : a);
    if (a >= 0) { ++dep; a = up; }
  }
  int maxdep = dep;
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) {
    const int other = __shfl_xor(maxdep, o);
    maxdep = other > maxdep ? other : maxdep;
  }
  // Score(v) = Score(parent(v)) * q(v), level by level (Eq. 7); the root counts as probability 1
  float sc = lane == 0 ? 1.0f : 0.0f;
  for (int lvl = 1; lvl <= maxdep; ++lvl) {
    const float sp = __shfl(sc, p < 0 ? 0 : p);
    if (live && dep == lvl) sc = __fmul_rn(sp, q);
  }
  // rank by (score descending, index ascending); lanes past the tree keep their own position
  int r = lane;
  if (live) r = 0;
  const int sbits = __float_as_int(sc);
  for (int j = 0; j < n; ++j) {
    const float sj = __int_as_float(__builtin_amdgcn_readlane(sbits, j));
    if (live) r += (sj > sc || (sj == sc && j < lane)) ? 1 : 0;
  }
  if (live && order_out) order_out[r] = lane;
  // scores in rank order: lane i sends its score to lane r
  const int sorted_bits = __builtin_amdgcn_ds_permute(r << 2, live ? sbits : 0);
  // S_k: sequential fp32 running sum over the ranking
  float acc = 0.0f, S = 0.0f;
  for (int j = 0; j < n; ++j) {
    acc = __fadd_rn(acc, __int_as_float(__builtin_amdgcn_readlane(sorted_bits, j)));
    if (lane == j) S = acc;
  }
  if (live && psum_out) psum_out[lane] = S;
  const int kk = n < kmax ? n : kmax;
  const float total = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(S), n - 1));
  float bv = -1.0f;
  int bi = 0x7fffffff;
  if (lane < kk) {
    bv = rho >= 0.0f ? (__fdiv_rn(S, total) >= rho ? 1.0f : 0.0f) : (c > 0.0f ? __fdiv_rn(S, c) : -1.0f);
    bi = lane;
  }
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) {
    const float ov = __shfl_xor(bv, o);
    const int oi = __shfl_xor(bi, o);
    if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
  }
  if (rho >= 0.0f && bv == 0.0f) bi = kk - 1;  // coverage not reached within kmax: the whole budget
  const int kstar = bi + 1;
  const float est = __shfl(S, bi);
  // kept nodes ascending, parents re-indexed by counting kept nodes below
  const unsigned long long kept = __ballot(live && r < kstar);
  if (live && r < kstar) {
    const int ni = __popcll(kept & ((1ull << lane) - 1ull));
    keep[ni] = lane;
    new_parent[ni] = p < 0 ? -1 : __popcll(kept & ((1ull << p) - 1ull));
  }
  if (lane == 0) {
    k_star[0] = kstar;
    est_len[0] = est;
    new_tree_off[0] = 0;
    new_tree_off[1] = kstar;
  }
}

// Second step for batches: one workgroup walks the trees in order, so that tree b's
// compacted output (which starts at or before tree b's own input offset) never overwrites
// ranks of a tree not yet read. rank_ws aliases new_parent.
__global__ __launch_bounds__(kSelThreads) void compact_batch_kernel(
    const int32_t* __restrict__ tree_off, const int32_t* __restrict__ parent, const int32_t* __restrict__ k_star,
    int B, int32_t* rank_ws, int32_t* keep, int32_t* new_parent, int32_t* __restrict__ new_tree_off) {
  __shared__ int s_par[kMaxSel];
  __shared__ int s_rank[kMaxSel];
  __shared__ int s_new[kMaxSel];
  __shared__ int s_wave[16];
  const int tid = threadIdx.x;
  int out = 0;
  for (int b = 0; b < B; ++b) {
    const int lo = tree_off[b];
    int n = tree_off[b + 1] - lo;
    n = n < 1 ? 1 : (n > kMaxSel ? kMaxSel : n);
    const int ks = k_star[b];
    __syncthreads();
    for (int i = tid; i < n; i += kSelThreads) {
      int p = parent[lo + i];
      if (i == 0) p = -1;
      else if (p < 0 || p >= i) p = 0;
      s_par[i] = p;
      s_rank[i] = rank_ws[lo + i];
    }
    __syncthreads();
    if (tid == 0) new_tree_off[b] = out;
    compact_tree(n, ks, s_par, s_rank, s_new, s_wave, keep + out, new_parent + out);
    out += ks;
  }
  if (tid == 0) new_tree_off[B] = out;
}

// One wavefront per tree; the tree is staged in LDS so the walk has no global-memory latency.
__global__ __launch_bounds__(64) void accept_path_kernel(
    const int32_t* __restrict__ tree_off, const int32_t* __restrict__ parent, const int32_t* __restrict__ tok,
    const int32_t* __restrict__ next, int32_t* __restrict__ path, int path_stride, int32_t* __restrict__ path_len,
    int32_t* __restrict__ bonus) {
  __shared__ int s_par[kMaxSel];
  __shared__ int s_tok[kMaxSel];
  __shared__ int s_next[kMaxSel];
  const int b = blockIdx.x, lane = threadIdx.x;
  const int lo = tree_off[b];
  int n = tree_off[b + 1] - lo;
  n = n < 1 ? 1 : (n > kMaxSel ? kMaxSel : n);
  for (int i = lane; i < n; i += 64) {
    s_par[i] = parent[lo + i];
    s_tok[i] = tok[lo + i];
    s_next[i] = next[lo + i];
  }
  int32_t* my = path + (size_t)b * path_stride;
  for (int i = lane; i < path_stride; i += 64) my[i] = i == 0 ? 0 : -1;
  __syncthreads();
  int cur = 0, len = 1;
  while (true) {
    const int want = s_next[cur];
    int found = -1;
    for (int base = cur + 1; base < n; base += 64) {
      const int c = base + lane;
      const bool m = c < n && s_par[c] == cur && s_tok[c] == want;
      const unsigned long long mask = __ballot(m);
      if (mask) { found = base + __ffsll((long long)mask) - 1; break; }
    }
    if (found < 0) break;
    cur = found;  // strictly increasing: the walk ends
    if (lane == 0 && len < path_stride) my[len] = cur;
    ++len;
  }
  if (lane == 0) { path_len[b] = len; bonus[b] = s_next[cur]; }
}

// ------------------------------------------------------------------------------------
// Acceptance under sampling: the sequential sibling rule (Sec. 2.1, Eq. 3).
// ------------------------------------------------------------------------------------
constexpr int kSampThreads = 1024;
constexpr int kSampWaves = kSampThreads / 64;

// Per node: maximum of the logits and the sum of exp((logit - max) / temperature) over the
// vocabulary -- the two numbers that turn any logit of the row into a probability.
__global__ __launch_bounds__(kSampThreads) void softmax_stats_kernel(const float* __restrict__ logits, int V, float inv_temp,
                                                                     float* __restrict__ stats, const int* __restrict__ t_dev) {
  __shared__ float s_red[kSampWaves];
  if ((int)blockIdx.x >= dyn_tokens(t_dev, (int)gridDim.x)) return;  // (rows past the call's actual token count)
  const float* row = logits + (size_t)blockIdx.x * V;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  float m = -INFINITY;
  for (int i = tid; i < V; i += kSampThreads) m = fmaxf(m, row[i]);
  m = wave_max(m);
  if (lane == 0) s_red[w] = m;
  __syncthreads();
  m = s_red[0];
  for (int i = 1; i < kSampWaves; ++i) m = fmaxf(m, s_red[i]);
  __syncthreads();
  float z = 0.0f;
  for (int i = tid; i < V; i += kSampThreads) z += __expf((row[i] - m) * inv_temp);
  z = wave_sum(z);
  if (lane == 0) s_red[w] = z;
  __syncthreads();
  if (tid == 0) {
    float t = 0.0f;
    for (int i = 0; i < kSampWaves; ++i) t += s_red[i];
    stats[2 * blockIdx.x] = m;
    stats[2 * blockIdx.x + 1] = t;
  }
}

__device__ __forceinline__ float wave_incl_scan_f32(float v, int lane) {
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const float t = __shfl_up(v, o);
    if (lane >= o) v += t;
  }
  return v;
}

// One workgroup per tree. Step 1, all threads: the target probability of every node's token
// under its parent's distribution. Step 2, one thread: the walk of Eq. 3 on values in LDS --
// child c of the surviving node is accepted when u_node[c] < p(c) / (1 - mass rejected so
// far at this node), which is what the repeated renormalisation amounts to; a token already
// rejected at this node has no mass left. Step 3, all threads: the final draw from the
// distribution at the last node with the rejected tokens removed, by inverting the cumulative
// sum at u_bonus: 16 contiguous vocabulary segments are summed (one per wavefront), the
// segment holding the target mass is cut into 64 contiguous pieces, the piece is walked.
__global__ __launch_bounds__(kSampThreads) void accept_sampled_kernel(
    const int32_t* __restrict__ tree_off, const int32_t* __restrict__ parent, const int32_t* __restrict__ tok,
    const float* __restrict__ logits, int V, float inv_temp, const float* __restrict__ stats,
    const float* __restrict__ u_node, const float* __restrict__ u_bonus, int32_t* __restrict__ path, int path_stride,
    int32_t* __restrict__ path_len, int32_t* __restrict__ bonus, int32_t* __restrict__ status) {
  __shared__ int s_par[kMaxSel];
  __shared__ int s_tok[kMaxSel];
  __shared__ float s_p[kMaxSel];
  __shared__ float s_u[kMaxSel];
  __shared__ int s_rej[kMaxSel];
  __shared__ int s_cur, s_nrej, s_seg, s_found;
  __shared__ float s_segsum[kSampWaves];
  __shared__ float s_rem;
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int lo = tree_off[b];
  int n = tree_off[b + 1] - lo;
  n = n < 1 ? 1 : (n > kMaxSel ? kMaxSel : n);
  bool bad = false;
  for (int i = tid; i < n; i += kSampThreads) {
    int pa = parent[lo + i];
    int tk = tok[lo + i];
    if (i > 0 && (pa < 0 || pa >= i)) { bad = true; pa = 0; }
    float pr = 0.0f;
    if (i > 0) {
      if (tk < 0 || tk >= V) { bad = true; tk = -1; }  // an invalid token id is never accepted and removes no mass
      else {
        const size_t prow = (size_t)(lo + pa);
        pr = __expf((logits[prow * V + tk] - stats[2 * prow]) * inv_temp) / stats[2 * prow + 1];
      }
    }
    s_par[i] = i == 0 ? -1 : pa;
    s_tok[i] = tk;
    s_p[i] = pr;
    s_u[i] = u_node[lo + i];
  }
  if (bad && status) atomicOr(status, ST_BAD_PARENT);
  int32_t* my = path + (size_t)b * path_stride;
  for (int i = tid; i < path_stride; i += kSampThreads) my[i] = i == 0 ? 0 : -1;
  __syncthreads();
  if (tid == 0) {
    int cur = 0, len = 1, nrej = 0;
    while (true) {
      float removed = 0.0f;
      nrej = 0;
      int nxt = -1;
      for (int c = cur + 1; c < n; ++c) {
        if (s_par[c] != cur) continue;
        const int tk = s_tok[c];
        float pc = s_p[c];
        for (int r = 0; r < nrej; ++r)
          if (s_rej[r] == tk) pc = 0.0f;
        if (s_u[c] < pc / (1.0f - removed)) { nxt = c; break; }
        removed += pc;
        s_rej[nrej++] = tk;
      }
      if (nxt < 0) break;
      cur = nxt;  // strictly increasing: the walk ends
      if (len < path_stride) my[len] = cur;
      ++len;
    }
    path_len[b] = len;
    s_cur = cur;
    s_nrej = nrej;
    s_found = -1;
  }
  __syncthreads();
  const int cur = s_cur, nrej = s_nrej;
  const float* row = logits + (size_t)(lo + cur) * V;
  const float m = stats[2 * (size_t)(lo + cur)];
  auto mass = [&](int i) {
    float e = __expf((row[i] - m) * inv_temp);
    for (int r = 0; r < nrej; ++r)
      if (s_rej[r] == i) e = 0.0f;
    return e;
  };
  // segment sums: segment w = [w * seg, (w + 1) * seg) with seg a multiple of 64
  const int seg = (((V + kSampWaves - 1) / kSampWaves) + 63) & ~63;
  const int sb = w * seg;
  const int se = sb + seg < V ? sb + seg : V;
  float acc = 0.0f;
  for (int i = sb + lane; i < se; i += 64) acc += mass(i);
  acc = wave_sum(acc);
  if (lane == 0) s_segsum[w] = acc;
  __syncthreads();
  if (tid == 0) {
    float total = 0.0f;
    for (int i = 0; i < kSampWaves; ++i) total += s_segsum[i];
    const float target = u_bonus[b] * total;
    float before = 0.0f;
    int pick = -1;
    bool inside = false;
    for (int i = 0; i < kSampWaves && !inside; ++i) {
      if (s_segsum[i] > 0.0f) {
        pick = i;
        inside = target < before + s_segsum[i];
        if (!inside) before += s_segsum[i];
      }
    }
    // (rounding may leave the target past the last sum: the last non-empty segment takes it)
    if (pick >= 0 && !inside) before -= s_segsum[pick];
    s_seg = pick < 0 ? 0 : pick;
    s_rem = target - before;
  }
  __syncthreads();
  if (w == 0) {
    const int cl = seg >> 6;  // contiguous piece per lane
    const int pb = s_seg * seg + lane * cl;
    int pe = pb + cl;
    pe = pe < V ? pe : V;
    float psum = 0.0f;
    for (int i = pb; i < pe; ++i) psum += mass(i);
    const float incl = wave_incl_scan_f32(psum, lane);
    const float rem = s_rem;
    const unsigned long long hit = __ballot(psum > 0.0f && rem < incl);
    const unsigned long long any = __ballot(psum > 0.0f);
    int owner = -1;
    if (hit) owner = __ffsll((long long)hit) - 1;
    else if (any) owner = 63 - __clzll((long long)any);  // rounding: the last piece with mass takes it
    if (lane == owner) {
      const float r2 = rem - (incl - psum);
      float run = 0.0f;
      int pick = -1;
      for (int i = pb; i < pe; ++i) {
        const float e = mass(i);
        if (e > 0.0f) {
          pick = i;
          run += e;
          if (r2 < run) break;
        }
      }
      s_found = pick;
    }
  }
  __syncthreads();
  if (tid == 0) bonus[b] = s_found < 0 ? 0 : s_found;
}

constexpr int kUnionThreads = 1024;  // >= the largest supported E: one expert per thread in the scan

__global__ __launch_bounds__(kUnionThreads) void expert_union_kernel(
    const int32_t* __restrict__ topk_idx, int T, int k, int E, int use_masks, int32_t* __restrict__ union_ids,
    int32_t* __restrict__ union_count, int32_t* __restrict__ hist, int32_t* __restrict__ offsets,
    int32_t* __restrict__ perm, int32_t* __restrict__ inv, int32_t* __restrict__ status) {
  extern __shared__ __attribute__((aligned(8))) int s_mem[];
  expert_union_body(s_mem, topk_idx, T, k, E, use_masks, union_ids, union_count, hist, offsets, perm, inv, status, nullptr,
                    nullptr);
}

typedef __attribute__((ext_vector_type(4))) unsigned int probe_u32x4;

// Streaming read: 512 workgroups x 256 threads, each thread keeps 8 independent 16-byte loads in flight.
__global__ __launch_bounds__(256) void probe_read_kernel(const probe_u32x4* __restrict__ src, size_t n16, unsigned* __restrict__ sink) {
  const size_t per_wg = (n16 + gridDim.x - 1) / gridDim.x;
  const size_t lo = per_wg * blockIdx.x;
  size_t hi = lo + per_wg;
  hi = hi > n16 ? n16 : hi;
  probe_u32x4 acc = {0, 0, 0, 0};
  for (size_t i = lo + threadIdx.x; i < hi; i += 256 * 8) {
    probe_u32x4 v[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const size_t idx = i + (size_t)j * 256;
      v[j] = idx < hi ? __builtin_nontemporal_load(src + idx) : probe_u32x4{0, 0, 0, 0};
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) acc ^= v[j];
  }
  if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x9E3779B9u) sink[threadIdx.x & 3] = acc[0];  // keeps the loads alive
}

__global__ __launch_bounds__(256) void probe_copy_kernel(const probe_u32x4* __restrict__ src, probe_u32x4* __restrict__ dst, size_t n16) {
  const size_t per_wg = (n16 + gridDim.x - 1) / gridDim.x;
  const size_t lo = per_wg * blockIdx.x;
  size_t hi = lo + per_wg;
  hi = hi > n16 ? n16 : hi;
  for (size_t i = lo + threadIdx.x; i < hi; i += 256 * 4) {
    probe_u32x4 v[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const size_t idx = i + (size_t)j * 256;
      if (idx < hi) v[j] = src[idx];
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const size_t idx = i + (size_t)j * 256;
      if (idx < hi) dst[idx] = v[j];
    }
  }
}

__global__ void gather_rows_kernel(const uint32_t* __restrict__ src, uint32_t* __restrict__ dst, int row_words,
                                   const int32_t* __restrict__ tree_off, const int32_t* __restrict__ new_tree_off,
                                   const int32_t* __restrict__ keep, int B) {
  const int r = blockIdx.x;  // destination row
  if (r >= new_tree_off[B]) return;
  int b = 0;
  while (b + 1 < B && new_tree_off[b + 1] <= r) ++b;
  const int s = tree_off[b] + keep[r];
  for (int i = threadIdx.x; i < row_words; i += blockDim.x) dst[(size_t)r * row_words + i] = src[(size_t)s * row_words + i];
}

// Commit of the accepted path to the KV cache: the j-th accepted node of sequence b (depth j, so
// its key was rotated at position ctx_len[b] + j) becomes cache row ctx_len[b] + j of every KV
// head. Grid (path position, sequence); rows are copied as 4-byte words. Rows that would fall
// past the cache capacity are dropped and the new length is clamped.
constexpr int kCommitLayers = 64;  // layers per launch (their pointers travel as a kernel argument)
struct KvLayerPtrs {
  const uint32_t* k_new[kCommitLayers];
  const uint32_t* v_new[kCommitLayers];
  uint32_t* k_cache[kCommitLayers];
  uint32_t* v_cache[kCommitLayers];
};

__global__ __launch_bounds__(256) void kv_commit_kernel(
    const KvLayerPtrs lp, int Hkv, int head_words,
    const int32_t* __restrict__ tree_off, const int32_t* __restrict__ path, int path_stride,
    const int32_t* __restrict__ path_len, long long seq_words, long long head_stride_words,
    const int32_t* __restrict__ ctx_len, int capacity, int32_t* __restrict__ ctx_len_out, int32_t* __restrict__ status,
    const KvPaging pg) {
  const int j = blockIdx.x, b = blockIdx.y, layer = blockIdx.z;
  const uint32_t* __restrict__ k_new = lp.k_new[layer];
  const uint32_t* __restrict__ v_new = lp.v_new[layer];
  uint32_t* __restrict__ k_cache = lp.k_cache[layer];
  uint32_t* __restrict__ v_cache = lp.v_cache[layer];
  int len = path_len[b];
  // an accepted path longer than the rows `path` holds (evict_accept_path truncates it) cannot be committed in
  // full: the rows that are there are committed, the length advances by that many, and the call is flagged
  const bool trunc = len > path_stride;
  len = len < 0 ? 0 : (trunc ? path_stride : len);
  int L = ctx_len[b];
  const bool badL = L < 0 || L > capacity;
  L = L < 0 ? 0 : (L > capacity ? capacity : L);
  const int room = capacity - L;
  if (j == 0 && layer == 0 && threadIdx.x == 0) {
    ctx_len_out[b] = L + (len < room ? len : room);
    if (status && (badL || len > room)) atomicOr(status, ST_BAD_CTXLEN);
    if (status && trunc) atomicOr(status, ST_PATH_TRUNCATED);
  }
  if (j >= len || j >= room) return;
  const int n = tree_off[b + 1] - tree_off[b];
  const int node = path[(size_t)b * path_stride + j];
  if (node < 0 || node >= n) {
    if (status && threadIdx.x == 0) atomicOr(status, ST_BAD_PARENT);
    return;
  }
  const size_t src = (size_t)(tree_off[b] + node) * Hkv * head_words;
  const int row_words = Hkv * head_words;
  // start of the destination row of head 0: contiguous cache, or (paged: seq_words is the distance
  // between pages) the page the table names for position L + j
  size_t row0 = (size_t)b * seq_words + (size_t)(L + j) * head_words;
  if (pg.table) {
    const int pos = L + j;
    const int pid = pg.table[(size_t)b * pg.table_stride + (pos >> pg.page_shift)];
    if ((unsigned)pid >= (unsigned)pg.n_pages) {  // never write through a bad page id
      if (status && threadIdx.x == 0) atomicOr(status, ST_BAD_PAGE);
      return;
    }
    row0 = (size_t)pid * seq_words + (size_t)(pos & ((1 << pg.page_shift) - 1)) * head_words;
  }
  for (int i = threadIdx.x; i < row_words; i += 256) {
    const int h = i / head_words, c = i - h * head_words;
    const size_t dst = row0 + (size_t)h * head_stride_words + c;
    k_cache[dst] = k_new[src + i];
    v_cache[dst] = v_new[src + i];
  }
}

}  // namespace

int union_mask_plan(int T, int k, int E, size_t* lds_bytes) {
  const int P = T * k;
  const size_t words = (size_t)(T + 63) / 64;
  size_t lds = sizeof(int) * union_lds_ints(P, E);
  const size_t mask_bytes = 8 * (size_t)E * words;
  const int use_masks = lds + mask_bytes <= 60 * 1024 ? 1 : 0;
  if (use_masks) lds += mask_bytes;
  *lds_bytes = lds;
  return use_masks;
}

}  // namespace evict

using namespace evict;

// ---- scratch of the allocation-free entry point (evict_accept_path_sampled_noalloc) ----
// Per-node softmax statistics [EVICT_NOALLOC_MAX_NODES][2] floats. Every GPU the library runs on holds its
// own copy of this array until the process ends. In host code the array's name is only a stand-in: the
// device address is looked up once per device and kept; kernels and copies use that pointer.
static __device__ __align__(256) float scratch[EVICT_NOALLOC_MAX_NODES * 2];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
float* g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device (looked up on the first call on that device).
int scratch_address(float** out) {
  int dev = -1;
  EVICT_HIP_CHECK(hipGetDevice(&dev));
  EVICT_REQUIRE(dev >= 0 && dev < kMaxDevices, EVICT_E_UNSUPPORTED, "device ordinal %d outside [0, %d)", dev, kMaxDevices);
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    EVICT_HIP_CHECK(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    EVICT_REQUIRE(p != nullptr, EVICT_E_HIP, "hipGetSymbolAddress returned a null address for the static scratch");
    g_scratch_ptr[dev] = static_cast<float*>(p);
  }
  *out = g_scratch_ptr[dev];
  return EVICT_OK;
}
}  // namespace

extern "C" {

int evict_version(void) { return 1; }

const char* evict_last_error(void) { return g_err; }

int evict_validate_trees_host(const int32_t* tree_off, const int32_t* parent, int B, int max_nodes) {
  EVICT_REQUIRE(tree_off && parent, EVICT_E_INVALID, "null tree arrays");
  EVICT_REQUIRE(B >= 1, EVICT_E_INVALID, "B must be >= 1 (got %d)", B);
  EVICT_REQUIRE(tree_off[0] == 0, EVICT_E_INVALID, "tree_off[0] must be 0");
  for (int b = 0; b < B; ++b) {
    const int lo = tree_off[b], n = tree_off[b + 1] - lo;
    EVICT_REQUIRE(n >= 1, EVICT_E_INVALID, "tree %d has %d nodes", b, n);
    EVICT_REQUIRE(n <= max_nodes, EVICT_E_INVALID, "tree %d has %d nodes, limit %d", b, n, max_nodes);
    EVICT_REQUIRE(parent[lo] == -1, EVICT_E_INVALID, "tree %d: root parent must be -1", b);
    for (int i = 1; i < n; ++i)
      EVICT_REQUIRE(parent[lo + i] >= 0 && parent[lo + i] < i, EVICT_E_INVALID,
                    "tree %d: parent[%d]=%d is not in [0,%d)", b, i, parent[lo + i], i);
  }
  return EVICT_OK;
}

static int select_prefix_impl(const char* who, evict_ctx* ctx, const int32_t* tree_off, const int32_t* parent, const float* node_prob, int B,
                              int T, const float* cost, float rho, int Kmax, int32_t* k_star, int32_t* keep,
                              int32_t* new_parent, int32_t* new_tree_off, float* est_len, int32_t* order,
                              float* prefix_sum, void* stream) {
  EVICT_REQUIRE(tree_off && parent && node_prob && k_star && keep && new_parent && new_tree_off && est_len,
                EVICT_E_INVALID, "%s: null pointer argument", who);
  EVICT_REQUIRE(B >= 1 && T >= B, EVICT_E_INVALID, "%s: need B >= 1 and T >= B (B=%d, T=%d)", who, B, T);
  EVICT_REQUIRE(Kmax >= 1, EVICT_E_INVALID, "%s: Kmax must be >= 1 (got %d)", who, Kmax);
  EVICT_REQUIRE(T <= B * (int64_t)EVICT_MAX_SELECT_NODES, EVICT_E_UNSUPPORTED, "%s: more than %d nodes per tree", who,
                EVICT_MAX_SELECT_NODES);
  hipStream_t s = (hipStream_t)stream;
  int32_t* status = ctx ? ctx->status : nullptr;
  const int single = B == 1;
  if (B == 1 && T <= 64) {  // one small tree: the single-wavefront register kernel
    hipLaunchKernelGGL(select_prefix_wave_kernel, dim3(1), dim3(64), 0, s, parent, node_prob, cost, Kmax, T, rho, k_star,
                       est_len, order, prefix_sum, keep, new_parent, new_tree_off, status);
    return launch_status("select_prefix_wave_kernel");
  }
  const int sel_threads = kSelThreads;
  hipLaunchKernelGGL(select_prefix_kernel, dim3(B), dim3(sel_threads), 0, s, tree_off, parent, node_prob, cost, Kmax,
                     k_star, est_len, order, prefix_sum, new_parent /* rank workspace */, single, keep, new_parent,
                     new_tree_off, single ? T : 0, rho, status);
  int rc = launch_status("select_prefix_kernel");
  if (rc) return rc;
  if (!single) {
    hipLaunchKernelGGL(compact_batch_kernel, dim3(1), dim3(kSelThreads), 0, s, tree_off, parent, k_star, B,
                       new_parent, keep, new_parent, new_tree_off);
    rc = launch_status("compact_batch_kernel");
  }
  return rc;
}

int evict_select_prefix(evict_ctx* ctx, const int32_t* tree_off, const int32_t* parent, const float* node_prob, int B,
                        int T, const float* cost, int Kmax, int32_t* k_star, int32_t* keep, int32_t* new_parent,
                        int32_t* new_tree_off, float* est_len, int32_t* order, float* prefix_sum, void* stream) {
  EVICT_REQUIRE(cost, EVICT_E_INVALID, "evict_select_prefix: null cost table");
  return select_prefix_impl("evict_select_prefix", ctx, tree_off, parent, node_prob, B, T, cost, -1.0f, Kmax, k_star, keep,
                            new_parent, new_tree_off, est_len, order, prefix_sum, stream);
}

int evict_select_prefix_coverage(evict_ctx* ctx, const int32_t* tree_off, const int32_t* parent, const float* node_prob, int B,
                                 int T, float rho, int Kmax, int32_t* k_star, int32_t* keep, int32_t* new_parent,
                                 int32_t* new_tree_off, float* est_len, int32_t* order, float* prefix_sum, void* stream) {
  EVICT_REQUIRE(rho >= 0.0f && rho <= 1.0f, EVICT_E_INVALID, "evict_select_prefix_coverage: rho=%g outside [0, 1]", (double)rho);
  return select_prefix_impl("evict_select_prefix_coverage", ctx, tree_off, parent, node_prob, B, T, nullptr, rho, Kmax, k_star,
                            keep, new_parent, new_tree_off, est_len, order, prefix_sum, stream);
}

int evict_accept_path(evict_ctx*, const int32_t* tree_off, const int32_t* parent, const int32_t* draft_tok,
                      const int32_t* target_next, int B, int32_t* path, int path_stride, int32_t* path_len,
                      int32_t* bonus_tok, void* stream) {
  EVICT_REQUIRE(tree_off && parent && draft_tok && target_next && path && path_len && bonus_tok, EVICT_E_INVALID,
                "evict_accept_path: null pointer argument");
  EVICT_REQUIRE(B >= 1, EVICT_E_INVALID, "evict_accept_path: B must be >= 1 (got %d)", B);
  EVICT_REQUIRE(path_stride >= 1, EVICT_E_INVALID, "evict_accept_path: path_stride must be >= 1");
  hipLaunchKernelGGL(accept_path_kernel, dim3(B), dim3(64), 0, (hipStream_t)stream, tree_off, parent, draft_tok,
                     target_next, path, path_stride, path_len, bonus_tok);
  return launch_status("accept_path_kernel");
}

int evict_expert_union(evict_ctx* ctx, const int32_t* topk_idx, int T, int k, int E, int32_t* union_ids,
                       int32_t* union_count, int32_t* hist, int32_t* offsets, int32_t* perm, int32_t* inv,
                       void* stream) {
  EVICT_REQUIRE(topk_idx && union_ids && union_count && hist && offsets && perm && inv, EVICT_E_INVALID,
                "evict_expert_union: null pointer argument");
  EVICT_REQUIRE(T >= 1 && k >= 1 && E >= 1, EVICT_E_INVALID, "evict_expert_union: T, k, E must be >= 1");
  EVICT_REQUIRE(k <= E, EVICT_E_INVALID, "evict_expert_union: k=%d exceeds E=%d", k, E);
  EVICT_REQUIRE((int64_t)T * k <= 8192 && E <= 1024, EVICT_E_UNSUPPORTED,
                "evict_expert_union: T*k=%lld (limit 8192), E=%d (limit 1024)", (long long)T * k, E);
  size_t lds;
  const int use_masks = union_mask_plan(T, k, E, &lds);
  hipLaunchKernelGGL(expert_union_kernel, dim3(1), dim3(kUnionThreads), lds, (hipStream_t)stream, topk_idx, T, k, E,
                     use_masks, union_ids, union_count, hist, offsets, perm, inv, ctx ? ctx->status : nullptr);
  return launch_status("expert_union_kernel");
}

int evict_probe_read(const void* src, size_t bytes, void* sink, void* stream) {
  EVICT_REQUIRE(src && sink && bytes > 0 && bytes % 16 == 0 && aligned16(src), EVICT_E_INVALID,
                "evict_probe_read: need non-null 16-byte aligned src, sink, and bytes a positive multiple of 16");
  hipLaunchKernelGGL(probe_read_kernel, dim3(2048), dim3(256), 0, (hipStream_t)stream, (const probe_u32x4*)src, bytes / 16,
                     (unsigned*)sink);
  return launch_status("probe_read_kernel");
}

int evict_probe_copy(const void* src, void* dst, size_t bytes, void* stream) {
  EVICT_REQUIRE(src && dst && bytes > 0 && bytes % 16 == 0 && aligned16(src) && aligned16(dst), EVICT_E_INVALID,
                "evict_probe_copy: need non-null 16-byte aligned pointers and bytes a positive multiple of 16");
  hipLaunchKernelGGL(probe_copy_kernel, dim3(2048), dim3(256), 0, (hipStream_t)stream, (const probe_u32x4*)src,
                     (probe_u32x4*)dst, bytes / 16);
  return launch_status("probe_copy_kernel");
}

int evict_gather_rows(const void* src, void* dst, int row_bytes, const int32_t* tree_off, const int32_t* new_tree_off,
                      const int32_t* keep, int B, int T, void* stream) {
  EVICT_REQUIRE(src && dst && tree_off && new_tree_off && keep, EVICT_E_INVALID, "evict_gather_rows: null pointer");
  EVICT_REQUIRE(row_bytes > 0 && row_bytes % 4 == 0, EVICT_E_INVALID, "evict_gather_rows: row_bytes must be a positive multiple of 4");
  EVICT_REQUIRE(B >= 1 && T >= 1, EVICT_E_INVALID, "evict_gather_rows: B, T must be >= 1");
  EVICT_REQUIRE(src != dst, EVICT_E_INVALID, "evict_gather_rows: in-place gather is not supported");
  hipLaunchKernelGGL(gather_rows_kernel, dim3(T), dim3(128), 0, (hipStream_t)stream, (const uint32_t*)src,
                     (uint32_t*)dst, row_bytes / 4, tree_off, new_tree_off, keep, B);
  return launch_status("gather_rows_kernel");
}

int evict_accept_path_sampled(evict_ctx* ctx, const int32_t* tree_off, const int32_t* parent, const int32_t* draft_tok,
                              const float* logits, int vocab, float temperature, const float* u_node, const float* u_bonus,
                              int B, int T, int32_t* path, int path_stride, int32_t* path_len, int32_t* bonus_tok,
                              void* stream) {
  EVICT_REQUIRE(ctx && tree_off && parent && draft_tok && logits && u_node && u_bonus && path && path_len && bonus_tok,
                EVICT_E_INVALID, "evict_accept_path_sampled: null pointer argument");
  EVICT_REQUIRE(B >= 1 && B <= ctx->max_batch, EVICT_E_INVALID, "evict_accept_path_sampled: B=%d outside [1,%d]", B, ctx->max_batch);
  EVICT_REQUIRE(T >= 1 && T <= ctx->max_tokens, EVICT_E_INVALID, "evict_accept_path_sampled: T=%d outside [1,%d]", T, ctx->max_tokens);
  EVICT_REQUIRE(vocab >= 1, EVICT_E_INVALID, "evict_accept_path_sampled: vocab must be >= 1");
  EVICT_REQUIRE(temperature > 0.0f && temperature == temperature, EVICT_E_INVALID,
                "evict_accept_path_sampled: temperature must be > 0 (use evict_accept_path for the greedy rule)");
  EVICT_REQUIRE(path_stride >= 1, EVICT_E_INVALID, "evict_accept_path_sampled: path_stride must be >= 1");
  const float inv_temp = 1.0f / temperature;
  hipStream_t s = (hipStream_t)stream;
  hipLaunchKernelGGL(softmax_stats_kernel, dim3(T), dim3(kSampThreads), 0, s, logits, vocab, inv_temp, ctx->samp_stats, ctx->t_dev);
  int rc = launch_status("softmax_stats_kernel");
  if (rc) return rc;
  hipLaunchKernelGGL(accept_sampled_kernel, dim3(B), dim3(kSampThreads), 0, s, tree_off, parent, draft_tok, logits, vocab,
                     inv_temp, ctx->samp_stats, u_node, u_bonus, path, path_stride, path_len, bonus_tok, ctx->status);
  return launch_status("accept_sampled_kernel");
}

int evict_accept_path_sampled_noalloc(evict_ctx* ctx, const int32_t* tree_off, const int32_t* parent, const int32_t* draft_tok,
                                      const float* logits, int vocab, float temperature, const float* u_node,
                                      const float* u_bonus, int B, int T, int32_t* path, int path_stride, int32_t* path_len,
                                      int32_t* bonus_tok, void* stream) {
  EVICT_REQUIRE(tree_off && parent && draft_tok && logits && u_node && u_bonus && path && path_len && bonus_tok,
                EVICT_E_INVALID, "evict_accept_path_sampled_noalloc: null pointer argument");
  EVICT_REQUIRE(B >= 1 && B <= 65535, EVICT_E_INVALID, "evict_accept_path_sampled_noalloc: B=%d outside [1, 65535]", B);
  EVICT_REQUIRE(T >= B, EVICT_E_INVALID, "evict_accept_path_sampled_noalloc: T=%d is smaller than B=%d", T, B);
  EVICT_REQUIRE(T <= EVICT_NOALLOC_MAX_NODES, EVICT_E_UNSUPPORTED,
                "evict_accept_path_sampled_noalloc: T=%d exceeds the static scratch of %d nodes (use evict_accept_path_sampled)", T,
                EVICT_NOALLOC_MAX_NODES);
  EVICT_REQUIRE(vocab >= 1, EVICT_E_INVALID, "evict_accept_path_sampled_noalloc: vocab must be >= 1");
  EVICT_REQUIRE(temperature > 0.0f && temperature == temperature, EVICT_E_INVALID,
                "evict_accept_path_sampled_noalloc: temperature must be > 0 (use evict_accept_path for the greedy rule)");
  EVICT_REQUIRE(path_stride >= 1, EVICT_E_INVALID, "evict_accept_path_sampled_noalloc: path_stride must be >= 1");
  float* stats = nullptr;
  int rc = scratch_address(&stats);
  if (rc) return rc;
  const float inv_temp = 1.0f / temperature;
  hipStream_t s = (hipStream_t)stream;
  // (rows [0, T) of the statistics are written in full before they are read: nothing has to start at zero)
  hipLaunchKernelGGL(softmax_stats_kernel, dim3(T), dim3(kSampThreads), 0, s, logits, vocab, inv_temp, stats, ctx ? ctx->t_dev : nullptr);
  rc = launch_status("softmax_stats_kernel");
  if (rc) return rc;
  hipLaunchKernelGGL(accept_sampled_kernel, dim3(B), dim3(kSampThreads), 0, s, tree_off, parent, draft_tok, logits, vocab,
                     inv_temp, stats, u_node, u_bonus, path, path_stride, path_len, bonus_tok, ctx ? ctx->status : nullptr);
  return launch_status("accept_sampled_kernel");
}

static int kv_commit_impl(const char* who, evict_ctx* ctx, int dtype, int Hkv, int D, const void* const* k_new,
                          const void* const* v_new, int n_layers, const int32_t* tree_off, const int32_t* path, int path_stride,
                          const int32_t* path_len, void* const* k_caches, void* const* v_caches, int64_t kv_seq_stride,
                          int64_t kv_head_stride, const int32_t* ctx_len, int capacity, int32_t* ctx_len_out, int B,
                          void* stream, const KvPaging pg = KvPaging{nullptr, 0, 0, 0}) {
  EVICT_REQUIRE(k_new && v_new && tree_off && path && path_len && k_caches && v_caches && ctx_len && ctx_len_out,
                EVICT_E_INVALID, "%s: null pointer argument", who);
  EVICT_REQUIRE(dtype == EVICT_F32 || dtype == EVICT_BF16, EVICT_E_INVALID, "%s: unknown dtype %d", who, dtype);
  EVICT_REQUIRE(n_layers >= 1, EVICT_E_INVALID, "%s: n_layers=%d", who, n_layers);
  EVICT_REQUIRE(B >= 1 && B <= 65535 && Hkv >= 1 && D >= 1 && path_stride >= 1 && path_stride <= EVICT_MAX_SELECT_NODES,
                EVICT_E_INVALID, "%s: B, Hkv, D, path_stride out of range", who);
  const int eb = dtype == EVICT_BF16 ? 2 : 4;
  EVICT_REQUIRE((D * eb) % 4 == 0, EVICT_E_INVALID, "%s: a head row must be a multiple of 4 bytes", who);
  if (pg.table) {
    const int64_t page = (int64_t)1 << pg.page_shift;
    EVICT_REQUIRE(capacity >= 1 && (int64_t)pg.table_stride * page >= capacity, EVICT_E_INVALID,
                  "%s: a table row covers %lld positions, capacity is %d", who, (long long)pg.table_stride * page, capacity);
    EVICT_REQUIRE(kv_head_stride >= page * D && kv_seq_stride >= kv_head_stride * Hkv && (kv_head_stride * eb) % 4 == 0 &&
                      (kv_seq_stride * eb) % 4 == 0,
                  EVICT_E_INVALID, "%s: page strides do not hold page_size=%lld rows per head", who, (long long)page);
  } else {
    EVICT_REQUIRE(capacity >= 1 && kv_head_stride >= (int64_t)capacity * D && (kv_head_stride * eb) % 4 == 0 &&
                      (kv_seq_stride * eb) % 4 == 0 && (B == 1 || kv_seq_stride >= kv_head_stride * Hkv),
                  EVICT_E_INVALID, "%s: cache strides do not hold capacity=%d rows per head", who, capacity);
  }
  EVICT_REQUIRE(ctx_len_out != ctx_len, EVICT_E_INVALID, "%s: ctx_len_out must not alias ctx_len", who);
  for (int l = 0; l < n_layers; ++l)
    EVICT_REQUIRE(k_new[l] && v_new[l] && k_caches[l] && v_caches[l], EVICT_E_INVALID, "%s: null pointer for layer %d", who, l);
  const int head_words = D * eb / 4;
  for (int l0 = 0; l0 < n_layers; l0 += kCommitLayers) {
    const int nl = n_layers - l0 < kCommitLayers ? n_layers - l0 : kCommitLayers;
    KvLayerPtrs lp = {};
    for (int l = 0; l < nl; ++l) {
      lp.k_new[l] = (const uint32_t*)k_new[l0 + l];
      lp.v_new[l] = (const uint32_t*)v_new[l0 + l];
      lp.k_cache[l] = (uint32_t*)k_caches[l0 + l];
      lp.v_cache[l] = (uint32_t*)v_caches[l0 + l];
    }
    hipLaunchKernelGGL(kv_commit_kernel, dim3(path_stride, B, nl), dim3(256), 0, (hipStream_t)stream, lp, Hkv, head_words,
                       tree_off, path, path_stride, path_len, (long long)(kv_seq_stride * eb / 4),
                       (long long)(kv_head_stride * eb / 4), ctx_len, capacity, ctx_len_out, ctx ? ctx->status : nullptr, pg);
    int rc = launch_status("kv_commit_kernel");
    if (rc) return rc;
  }
  return EVICT_OK;
}

int evict_kv_commit(evict_ctx* ctx, int dtype, int Hkv, int D, const void* k_new, const void* v_new, const int32_t* tree_off,
                    const int32_t* path, int path_stride, const int32_t* path_len, void* k_cache, void* v_cache,
                    int64_t kv_seq_stride, int64_t kv_head_stride, const int32_t* ctx_len, int capacity, int32_t* ctx_len_out,
                    int B, void* stream) {
  return kv_commit_impl("evict_kv_commit", ctx, dtype, Hkv, D, &k_new, &v_new, 1, tree_off, path, path_stride, path_len,
                        &k_cache, &v_cache, kv_seq_stride, kv_head_stride, ctx_len, capacity, ctx_len_out, B, stream);
}

int evict_kv_commit_stack(evict_ctx* ctx, int dtype, int Hkv, int D, const void* const* k_new, const void* const* v_new,
                          int n_layers, const int32_t* tree_off, const int32_t* path, int path_stride, const int32_t* path_len,
                          void* const* k_caches, void* const* v_caches, int64_t kv_seq_stride, int64_t kv_head_stride,
                          const int32_t* ctx_len, int capacity, int32_t* ctx_len_out, int B, void* stream) {
  return kv_commit_impl("evict_kv_commit_stack", ctx, dtype, Hkv, D, k_new, v_new, n_layers, tree_off, path, path_stride,
                        path_len, k_caches, v_caches, kv_seq_stride, kv_head_stride, ctx_len, capacity, ctx_len_out, B, stream);
}

int evict_kv_commit_stack_paged(evict_ctx* ctx, int dtype, int Hkv, int D, const void* const* k_new, const void* const* v_new,
                                int n_layers, const int32_t* tree_off, const int32_t* path, int path_stride,
                                const int32_t* path_len, void* const* k_pools, void* const* v_pools, int64_t page_stride,
                                int64_t kv_head_stride, const int32_t* block_table, int table_stride, int page_size, int n_pages,
                                const int32_t* ctx_len, int capacity, int32_t* ctx_len_out, int B, void* stream) {
  EVICT_REQUIRE(block_table, EVICT_E_INVALID, "evict_kv_commit_stack_paged: null block table");
  EVICT_REQUIRE(page_size >= 1 && page_size <= 65536 && (page_size & (page_size - 1)) == 0, EVICT_E_INVALID,
                "evict_kv_commit_stack_paged: page_size=%d must be a power of two in [1, 65536]", page_size);
  EVICT_REQUIRE(n_pages >= 1 && table_stride >= 1, EVICT_E_INVALID, "evict_kv_commit_stack_paged: n_pages=%d table_stride=%d",
                n_pages, table_stride);
  int shift = 0;
  while ((1 << shift) < page_size) ++shift;
  return kv_commit_impl("evict_kv_commit_stack_paged", ctx, dtype, Hkv, D, k_new, v_new, n_layers, tree_off, path, path_stride,
                        path_len, k_pools, v_pools, page_stride, kv_head_stride, ctx_len, capacity, ctx_len_out, B, stream,
                        KvPaging{block_table, table_stride, shift, n_pages});
}

}  // extern "C"
