// Kernels of one verification pass through an MoE decoder layer (Sec. 2.1-2.2) other than
// the streaming GEMM: weight packing, tree preparation + RMSNorm, tree-masked attention
// (split over the context) and its merge, router top-k, un-permute/combine.
#include "ctx.h"
#include "gemm_stream.h"
#include "layer_launch.h"

namespace evict {
namespace {

// ------------------------------------------------------------------------------------
// weight packing (one-off)
// ------------------------------------------------------------------------------------
// dst block (strip, kb), lane l <- 16 bytes of source row map(strip*16 + l%16) at byte
// kb*64 + (l/16)*16. head_dim > 0 selects the rotary-friendly row order inside each head:
// strip j of a head holds rows 8j..8j+7 and D/2+8j..D/2+8j+7, so a rotation pair sits in
// one strip.
__global__ void pack_kernel(const char* __restrict__ src, long long src_group_bytes, int rows, long long row_bytes,
                            uint4* __restrict__ dst, int nkb, int dst_strip0, int dst_strip_step,
                            long long dst_group_strips, int head_dim) {
  const int strips = rows >> 4;
  const long long total = (long long)strips * nkb * 64;
  const int g = blockIdx.y;
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (long long)gridDim.x * blockDim.x) {
    const int lane = (int)(i & 63);
    const long long blk = i >> 6;
    const int kb = (int)(blk % nkb);
    const int strip = (int)(blk / nkb);
    int r = strip * 16 + (lane & 15);
    if (head_dim > 0) {
      const int head = r / head_dim, within = r - head * head_dim;
      const int j = within >> 4, m = within & 15;
      r = head * head_dim + (m < 8 ? 8 * j + m : (head_dim >> 1) + 8 * j + (m - 8));
    }
    const uint4 v = *reinterpret_cast<const uint4*>(src + g * src_group_bytes + r * row_bytes + (long long)kb * 64 + (lane >> 4) * 16);
    const long long dstrip = g * dst_group_strips + dst_strip0 + (long long)strip * dst_strip_step;
    dst[(dstrip * nkb + kb) * 64 + lane] = v;
  }
}

// ------------------------------------------------------------------------------------
// tree preparation + pre-attention RMSNorm: one workgroup per token
// ------------------------------------------------------------------------------------
template <typename ST>
__global__ __launch_bounds__(256) void prep_kernel(const int32_t* __restrict__ tree_off, const int32_t* __restrict__ parent,
                                                   int B, const int32_t* __restrict__ ctx_len, int max_ctx,
                                                   const void* __restrict__ x, const void* __restrict__ gain, int d,
                                                   float eps, float theta, int D, uint64_t* __restrict__ anc,
                                                   int32_t* __restrict__ depth, int32_t* __restrict__ seq_of,
                                                   float* __restrict__ rope_cs, void* __restrict__ x_norm,
                                                   int32_t* __restrict__ status) {
  __shared__ int s_par[EVICT_MAX_TREE_NODES];
  __shared__ int s_b, s_depth;
  __shared__ float s_red[4];
  const int t = blockIdx.x, tid = threadIdx.x;
  if (tid == 0) s_b = 0;
  __syncthreads();
  for (int b = tid; b < B; b += 256)
    if (tree_off[b] <= t && t < tree_off[b + 1]) s_b = b;
  __syncthreads();
  const int b = s_b;
  const int lo = tree_off[b];
  int n = tree_off[b + 1] - lo;
  if (n > EVICT_MAX_TREE_NODES) { n = EVICT_MAX_TREE_NODES; if (tid == 0) atomicOr(status, ST_BAD_TREE_SIZE); }
  const int i = t - lo < n ? t - lo : n - 1;
  for (int j = tid; j < n; j += 256) {
    int p = parent[lo + j];
    if (j == 0) p = -1;
    else if (p < 0 || p >= j) { p = 0; atomicOr(status, ST_BAD_PARENT); }
    s_par[j] = p;
  }
  __syncthreads();
  if (tid == 0) {
    uint64_t m0 = 0, m1 = 0;
    int dep = -1;
    for (int v = i; v >= 0; v = s_par[v]) {  // parent ids strictly decrease: the walk ends
      if (v < 64) m0 |= 1ull << v; else m1 |= 1ull << (v - 64);
      ++dep;
    }
    anc[2 * (size_t)t] = m0;
    anc[2 * (size_t)t + 1] = m1;
    depth[t] = dep;
    seq_of[t] = b;
    s_depth = dep;
  }
  __syncthreads();
  int L = ctx_len[b];
  if (L < 0 || L > max_ctx) { L = L < 0 ? 0 : max_ctx; if (tid == 0) atomicOr(status, ST_BAD_CTXLEN); }
  const int half = D >> 1;
  if (tid < half) {
    float cv = 1.0f, sv = 0.0f;
    if (theta > 0.0f) {
      // angle = position * theta^(-2i/D), formed in double so that large positions stay exact
      const double pos = (double)(L + s_depth);
      const double ang = pos * exp2(-(2.0 * tid / D) * log2((double)theta));
      cv = (float)cos(ang);
      sv = (float)sin(ang);
    }
    rope_cs[(size_t)t * D + tid] = cv;
    rope_cs[(size_t)t * D + half + tid] = sv;
  }
  // RMSNorm(x[t]) * gain, rounded to the storage type
  float ss = 0.0f;
  for (int c = tid; c < d; c += 256) {
    const float v = load_elem<ST>(x, (size_t)t * d + c);
    ss += v * v;
  }
  ss = wave_sum(ss);
  if ((tid & 63) == 0) s_red[tid >> 6] = ss;
  __syncthreads();
  const float ms = (s_red[0] + s_red[1] + s_red[2] + s_red[3]) / (float)d;
  const float rinv = 1.0f / sqrtf(ms + eps);
  for (int c = tid; c < d; c += 256) {
    const float v = load_elem<ST>(x, (size_t)t * d + c);
    store_elem<ST>(x_norm, (size_t)t * d + c, v * rinv * load_elem<ST>(gain, c));
  }
}

// ------------------------------------------------------------------------------------
// tree-masked attention, split over keys: grid (splits, Hkv, B), 64 keys per split.
// Splits [0, ctx_splits) cover the KV cache; the last two cover the draft nodes (keys
// 0..63 and 64..127 of the sequence's tree) under the ancestor mask of Fig. 4(c).
// ------------------------------------------------------------------------------------
constexpr int kAttnKeys = 64;

template <typename ST>
__global__ __launch_bounds__(256) void attn_partial_kernel(
    const void* __restrict__ q, const void* __restrict__ kc, const void* __restrict__ vc, long long seq_stride,
    long long head_stride, const int32_t* __restrict__ ctx_len, int max_ctx, const int32_t* __restrict__ tree_off,
    const void* __restrict__ k_new, const void* __restrict__ v_new, const uint64_t* __restrict__ anc, int Hq, int Hkv,
    int D, int ctx_splits, int T, float* __restrict__ part_o, float* __restrict__ part_ml) {
  extern __shared__ float s_dyn[];
  const int ldk = D + 1;
  float* s_k = s_dyn;                    // [64][D+1]
  float* s_v = s_k + kAttnKeys * ldk;    // [64][D+1]
  float* s_q = s_v + kAttnKeys * ldk;    // [4][D]
  float* s_p = s_q + 4 * D;              // [4][64]
  const int split = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int G = Hq / Hkv;
  const int lo = tree_off[b], n = tree_off[b + 1] - lo;
  int L = ctx_len[b];
  L = L < 0 ? 0 : (L > max_ctx ? max_ctx : L);
  const bool tree_part = split >= ctx_splits;
  int key0, nkeys;
  if (!tree_part) {
    key0 = split * kAttnKeys;
    nkeys = L - key0;
  } else {
    key0 = (split - ctx_splits) * kAttnKeys;
    nkeys = n - key0;
  }
  nkeys = nkeys < 0 ? 0 : (nkeys > kAttnKeys ? kAttnKeys : nkeys);
  // stage keys and values (fp32 in LDS)
  for (int idx = tid; idx < nkeys * D; idx += 256) {
    const int j = idx / D, c = idx - j * D;
    size_t src;
    float kv, vv;
    if (!tree_part) {
      src = (size_t)b * seq_stride + (size_t)g * head_stride + (size_t)(key0 + j) * D + c;
      kv = load_elem<ST>(kc, src);
      vv = load_elem<ST>(vc, src);
    } else {
      src = ((size_t)(lo + key0 + j) * Hkv + g) * D + c;
      kv = load_elem<ST>(k_new, src);
      vv = load_elem<ST>(v_new, src);
    }
    s_k[j * ldk + c] = kv;
    s_v[j * ldk + c] = vv;
  }
  __syncthreads();
  const float scale = 1.0f / sqrtf((float)D);
  const int R = n * G;
  for (int r = w; r < R; r += 4) {
    const int i = r / G, h = g * G + (r - i * G);
    const int t = lo + i;
    for (int c = lane; c < D; c += 64) s_q[w * D + c] = load_elem<ST>(q, ((size_t)t * Hq + h) * D + c);
    // (wavefront-private LDS rows: no workgroup barrier needed, LDS ops of a wave are ordered)
    float s = -INFINITY;
    bool vis = lane < nkeys;
    if (vis && tree_part) {
      const int key = key0 + lane;
      const uint64_t mword = anc[2 * (size_t)t + (key >> 6)];
      vis = (mword >> (key & 63)) & 1ull;
    }
    if (vis) {
      float acc = 0.0f;
      for (int c = 0; c < D; ++c) acc += s_q[w * D + c] * s_k[lane * ldk + c];
      s = acc * scale;
    }
    const float m = wave_max(s);
    const float p = vis ? __expf(s - m) : 0.0f;
    const float l = wave_sum(p);
    s_p[w * 64 + lane] = p;
    const size_t prow = ((size_t)split * T + t) * Hq + h;
    for (int c = lane; c < D; c += 64) {
      float o = 0.0f;
      for (int j = 0; j < nkeys; ++j) o += s_p[w * 64 + j] * s_v[j * ldk + c];
      part_o[prow * D + c] = o;
    }
    if (lane == 0) {
      part_ml[prow * 2] = m;
      part_ml[prow * 2 + 1] = l;
    }
  }
}

// merge of the per-split partial softmaxes: grid (T*Hq), block D threads
template <typename ST>
__global__ void attn_merge_kernel(const float* __restrict__ part_o, const float* __restrict__ part_ml, int nsplits,
                                  int T, int Hq, int D, const int32_t* __restrict__ seq_of,
                                  const int32_t* __restrict__ ctx_len, int max_ctx, int keys_per_split, int ctx_splits,
                                  void* __restrict__ out, void* __restrict__ aux_out) {
  const int row = blockIdx.x;  // t * Hq + h
  const int c = threadIdx.x;
  const int t = row / Hq;
  int L = ctx_len[seq_of[t]];
  L = L < 0 ? 0 : (L > max_ctx ? max_ctx : L);
  const int used_ctx = (L + keys_per_split - 1) / keys_per_split;  // splits past the context are skipped
  float M = -INFINITY;
  for (int s = 0; s < nsplits; ++s) {
    if (s >= used_ctx && s < ctx_splits) continue;
    M = fmaxf(M, part_ml[((size_t)s * T * Hq + row) * 2]);
  }
  float l = 0.0f, o = 0.0f;
  for (int s = 0; s < nsplits; ++s) {
    if (s >= used_ctx && s < ctx_splits) continue;
    const size_t pr = (size_t)s * T * Hq + row;
    const float ms = part_ml[pr * 2];
    if (ms == -INFINITY) continue;
    const float sc = __expf(ms - M);
    l += part_ml[pr * 2 + 1] * sc;
    o += part_o[pr * D + c] * sc;
  }
  const float r = o / l;
  store_elem<ST>(out, (size_t)row * D + c, r);
  if (aux_out) store_elem<ST>(aux_out, (size_t)row * D + c, r);
}

// ------------------------------------------------------------------------------------
// router: RMSNorm(h), scores W_g h (Eq. 4), top-k by wavefront shuffles, softmax over the
// selected scores. One workgroup per token.
// ------------------------------------------------------------------------------------
template <typename ST>
__global__ __launch_bounds__(256) void router_kernel(const void* __restrict__ h, const void* __restrict__ gain,
                                                     const void* __restrict__ wg, int d, int E, int k, float eps,
                                                     void* __restrict__ h_norm, float* __restrict__ logits,
                                                     int32_t* __restrict__ topk_idx, float* __restrict__ topk_w,
                                                     void* __restrict__ aux_hn, float* __restrict__ aux_logits,
                                                     int32_t* __restrict__ aux_idx, float* __restrict__ aux_w) {
  extern __shared__ float s_dyn[];
  float* s_h = s_dyn;       // [d]
  float* s_l = s_dyn + d;   // [E]
  __shared__ float s_red[4];
  const int t = blockIdx.x, tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  float ss = 0.0f;
  for (int c = tid; c < d; c += 256) {
    const float v = load_elem<ST>(h, (size_t)t * d + c);
    s_h[c] = v;
    ss += v * v;
  }
  ss = wave_sum(ss);
  if (lane == 0) s_red[w] = ss;
  __syncthreads();
  const float ms = (s_red[0] + s_red[1] + s_red[2] + s_red[3]) / (float)d;
  const float rinv = 1.0f / sqrtf(ms + eps);
  for (int c = tid; c < d; c += 256) {
    const float v = round_store<ST>(s_h[c] * rinv * load_elem<ST>(gain, c));
    s_h[c] = v;
    store_elem<ST>(h_norm, (size_t)t * d + c, v);
    if (aux_hn) store_elem<ST>(aux_hn, (size_t)t * d + c, v);
  }
  __syncthreads();
  // scores: one wavefront per expert, lanes stride over d in 4-element groups
  for (int e = w; e < E; e += 4) {
    float acc = 0.0f;
    for (int c = lane * 4; c < d; c += 256) {
      const f32x4 wv = load4<ST>(wg, (size_t)e * d + c);
      acc += wv[0] * s_h[c] + wv[1] * s_h[c + 1] + wv[2] * s_h[c + 2] + wv[3] * s_h[c + 3];
    }
    acc = wave_sum(acc);
    if (lane == 0) {
      s_l[e] = acc;
      logits[(size_t)t * E + e] = acc;
      if (aux_logits) aux_logits[(size_t)t * E + e] = acc;
    }
  }
  __syncthreads();
  if (w == 0) {
    float sel_v = 0.0f, first = 0.0f, denom = 0.0f;
    int sel_i = 0;
    for (int j = 0; j < k; ++j) {
      float bv = -INFINITY;
      int bi = 0x7fffffff;
      for (int e = lane; e < E; e += 64) {
        const float v = s_l[e];
        if (v > bv) { bv = v; bi = e; }  // ascending e inside a lane keeps the lowest index on ties
      }
#pragma unroll
      for (int o = 32; o >= 1; o >>= 1) {
        const float ov = __shfl_xor(bv, o);
        const int oi = __shfl_xor(bi, o);
        if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
      }
      if (j == 0) first = bv;
      const float ex = __expf(bv - first);
      denom += ex;
      if (lane == j) { sel_v = ex; sel_i = bi; }
      if (lane == 0) s_l[bi] = -INFINITY;  // remove from the candidates
    }
    if (lane < k) {
      const float wv = sel_v / denom;
      topk_idx[(size_t)t * k + lane] = sel_i;
      topk_w[(size_t)t * k + lane] = wv;
      if (aux_idx) aux_idx[(size_t)t * k + lane] = sel_i;
      if (aux_w) aux_w[(size_t)t * k + lane] = wv;
    }
  }
}

// ------------------------------------------------------------------------------------
// un-permute + weighted combine + residual (+ shared experts), fixed slot order
// ------------------------------------------------------------------------------------
template <typename ST>
__global__ __launch_bounds__(256) void combine_kernel(const void* __restrict__ h, const float* __restrict__ y,
                                                      const float* __restrict__ w, const int32_t* __restrict__ inv,
                                                      int k, int d, const float* __restrict__ y_sh, int n_shared, int T,
                                                      void* __restrict__ out) {
  const int t = blockIdx.x;
  for (int c = threadIdx.x * 4; c < d; c += 256 * 4) {
    f32x4 acc = load4<ST>(h, (size_t)t * d + c);
    for (int j = 0; j < k; ++j) {
      const float wj = w[(size_t)t * k + j];
      const f32x4 yv = *reinterpret_cast<const f32x4*>(y + (size_t)inv[(size_t)t * k + j] * d + c);
      acc += wj * yv;
    }
    for (int s = 0; s < n_shared; ++s) acc += *reinterpret_cast<const f32x4*>(y_sh + ((size_t)s * T + t) * d + c);
    store4<ST>(out, (size_t)t * d + c, acc);
  }
}

template <typename ST, int NT, int EPI>
int launch_gemm_nt(const GemmArgs& a, int grid, hipStream_t s) {
  const int need = ((a.nkb > 64 ? 64 : a.nkb) + kGemmWaves - 1) / kGemmWaves;
  if (need <= 4)
    hipLaunchKernelGGL((gemm_stream_kernel<ST, NT, 4, 4, EPI>), dim3(grid), dim3(kGemmThreads), 0, s, a);
  else
    hipLaunchKernelGGL((gemm_stream_kernel<ST, NT, 8, 2, EPI>), dim3(grid), dim3(kGemmThreads), 0, s, a);
  return launch_status("gemm_stream_kernel");
}

template <typename ST, int EPI>
int launch_gemm_st(const GemmArgs& a, int nt, int grid, hipStream_t s) {
  return nt == 1 ? launch_gemm_nt<ST, 1, EPI>(a, grid, s) : launch_gemm_nt<ST, 2, EPI>(a, grid, s);
}

}  // namespace

int launch_gemm(int dtype, int epi, const GemmArgs& a, int nt, int grid, hipStream_t s) {
#define EVICT_GEMM_CASE(E_)                                                   \
  case E_:                                                                    \
    return dtype == EVICT_BF16 ? launch_gemm_st<BF16, E_>(a, nt, grid, s)     \
                               : launch_gemm_st<F32, E_>(a, nt, grid, s);
  switch (epi) {
    EVICT_GEMM_CASE(EPI_QKV)
    EVICT_GEMM_CASE(EPI_RESID)
    EVICT_GEMM_CASE(EPI_SWIGLU)
    EVICT_GEMM_CASE(EPI_F32)
  }
#undef EVICT_GEMM_CASE
  set_error("unknown epilogue %d", epi);
  return EVICT_E_INVALID;
}

int launch_pack(const void* src, long long src_group_bytes, int rows, int cols, int dtype, void* dst, int dst_strip0,
                int dst_strip_step, long long dst_group_strips, int groups, int head_dim, hipStream_t s) {
  const int eb = dtype == EVICT_BF16 ? 2 : 4;
  const long long row_bytes = (long long)cols * eb;
  const int nkb = (int)(row_bytes / 64);
  const long long total = (long long)(rows / 16) * nkb * 64;
  int gx = (int)((total + 255) / 256);
  gx = gx > 4096 ? 4096 : gx;
  hipLaunchKernelGGL(pack_kernel, dim3(gx, groups), dim3(256), 0, s, (const char*)src, src_group_bytes, rows, row_bytes,
                     (uint4*)dst, nkb, dst_strip0, dst_strip_step, dst_group_strips, head_dim);
  return launch_status("pack_kernel");
}

int launch_prep(const evict_ctx* c, const int32_t* tree_off, const int32_t* parent, int B, int T, const int32_t* ctx_len,
                int max_ctx, const void* x, const void* gain, hipStream_t s) {
  const evict_model_desc& m = c->m;
  if (m.dtype == EVICT_BF16)
    hipLaunchKernelGGL(prep_kernel<BF16>, dim3(T), dim3(256), 0, s, tree_off, parent, B, ctx_len, max_ctx, x, gain, m.d,
                       m.rms_eps, m.rope_theta, m.D, c->anc, c->depth, c->seq_of, c->rope_cs, c->x_norm, c->status);
  else
    hipLaunchKernelGGL(prep_kernel<F32>, dim3(T), dim3(256), 0, s, tree_off, parent, B, ctx_len, max_ctx, x, gain, m.d,
                       m.rms_eps, m.rope_theta, m.D, c->anc, c->depth, c->seq_of, c->rope_cs, c->x_norm, c->status);
  return launch_status("prep_kernel");
}

size_t attn_partial_lds_bytes(int D) { return sizeof(float) * (size_t)(2 * kAttnKeys * (D + 1) + 4 * D + 4 * 64); }

int attn_setup() {
  // the partial kernel needs more than the default 64 KiB of dynamic LDS at D = 128
  const size_t need = attn_partial_lds_bytes(128);
  EVICT_HIP_CHECK(hipFuncSetAttribute((const void*)attn_partial_kernel<BF16>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)need));
  EVICT_HIP_CHECK(hipFuncSetAttribute((const void*)attn_partial_kernel<F32>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)need));
  return EVICT_OK;
}

int launch_attention(const evict_ctx* c, const void* kc, const void* vc, long long seq_stride, long long head_stride,
                     const int32_t* ctx_len, int max_ctx_host, const int32_t* tree_off, int B, int T, const void* k_new,
                     const void* v_new, void* aux_out, hipStream_t s) {
  const evict_model_desc& m = c->m;
  const int ctx_splits = (max_ctx_host + kAttnKeys - 1) / kAttnKeys;
  const int nsplits = ctx_splits + EVICT_MAX_TREE_NODES / kAttnKeys;
  const size_t lds = attn_partial_lds_bytes(m.D);
  if (m.dtype == EVICT_BF16) {
    hipLaunchKernelGGL(attn_partial_kernel<BF16>, dim3(nsplits, m.Hkv, B), dim3(256), lds, s, c->q, kc, vc, seq_stride,
                       head_stride, ctx_len, max_ctx_host, tree_off, k_new, v_new, c->anc, m.Hq, m.Hkv, m.D, ctx_splits, T,
                       c->part_o, c->part_ml);
  } else {
    hipLaunchKernelGGL(attn_partial_kernel<F32>, dim3(nsplits, m.Hkv, B), dim3(256), lds, s, c->q, kc, vc, seq_stride,
                       head_stride, ctx_len, max_ctx_host, tree_off, k_new, v_new, c->anc, m.Hq, m.Hkv, m.D, ctx_splits, T,
                       c->part_o, c->part_ml);
  }
  int rc = launch_status("attn_partial_kernel");
  if (rc) return rc;
  if (m.dtype == EVICT_BF16)
    hipLaunchKernelGGL(attn_merge_kernel<BF16>, dim3(T * m.Hq), dim3(m.D), 0, s, c->part_o, c->part_ml, nsplits, T, m.Hq,
                       m.D, c->seq_of, ctx_len, max_ctx_host, kAttnKeys, ctx_splits, c->attn_o, aux_out);
  else
    hipLaunchKernelGGL(attn_merge_kernel<F32>, dim3(T * m.Hq), dim3(m.D), 0, s, c->part_o, c->part_ml, nsplits, T, m.Hq,
                       m.D, c->seq_of, ctx_len, max_ctx_host, kAttnKeys, ctx_splits, c->attn_o, aux_out);
  return launch_status("attn_merge_kernel");
}

int attn_splits_for(int max_ctx) { return (max_ctx + kAttnKeys - 1) / kAttnKeys + EVICT_MAX_TREE_NODES / kAttnKeys; }

int launch_router(const evict_ctx* c, const void* gain, const void* wg, int T, const evict_layer_aux* aux, hipStream_t s) {
  const evict_model_desc& m = c->m;
  const size_t lds = sizeof(float) * (size_t)(m.d + m.E);
  void* a_hn = aux ? aux->h_norm : nullptr;
  float* a_lg = aux ? aux->router_logits : nullptr;
  int32_t* a_ix = aux ? aux->topk_idx : nullptr;
  float* a_w = aux ? aux->topk_w : nullptr;
  if (m.dtype == EVICT_BF16)
    hipLaunchKernelGGL(router_kernel<BF16>, dim3(T), dim3(256), lds, s, c->h, gain, wg, m.d, m.E, m.k, m.rms_eps, c->h_norm,
                       c->logits, c->topk_idx, c->topk_w, a_hn, a_lg, a_ix, a_w);
  else
    hipLaunchKernelGGL(router_kernel<F32>, dim3(T), dim3(256), lds, s, c->h, gain, wg, m.d, m.E, m.k, m.rms_eps, c->h_norm,
                       c->logits, c->topk_idx, c->topk_w, a_hn, a_lg, a_ix, a_w);
  return launch_status("router_kernel");
}

int launch_combine(const evict_ctx* c, int T, void* out, hipStream_t s) {
  const evict_model_desc& m = c->m;
  if (m.dtype == EVICT_BF16)
    hipLaunchKernelGGL(combine_kernel<BF16>, dim3(T), dim3(256), 0, s, c->h, c->y, c->topk_w, c->inv, m.k, m.d, c->y_sh,
                       m.n_shared, T, out);
  else
    hipLaunchKernelGGL(combine_kernel<F32>, dim3(T), dim3(256), 0, s, c->h, c->y, c->topk_w, c->inv, m.k, m.d, c->y_sh,
                       m.n_shared, T, out);
  return launch_status("combine_kernel");
}

}  // namespace evict
