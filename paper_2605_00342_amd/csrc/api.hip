// C-ABI entry points that own state or chain kernels: context, weight packing, the
// per-layer verification pass (Sec. 2.1-2.2).
#include <math.h>
#include <string.h>

#include <new>
#include <vector>

#include "ctx.h"
#include "gemm_stream.h"
#include "layer_launch.h"

using namespace evict;

namespace {

int elem_bytes(int dtype) { return dtype == EVICT_BF16 ? 2 : 4; }

int check_model(const evict_model_desc* m) {
  EVICT_REQUIRE(m, EVICT_E_INVALID, "model description is null");
  EVICT_REQUIRE(m->dtype == EVICT_F32 || m->dtype == EVICT_BF16, EVICT_E_INVALID, "unknown dtype %d", m->dtype);
  EVICT_REQUIRE(m->d > 0 && m->Hq > 0 && m->Hkv > 0 && m->D > 0 && m->E > 0 && m->k > 0 && m->F > 0 && m->n_shared >= 0,
                EVICT_E_INVALID, "model dimensions must be positive");
  EVICT_REQUIRE(m->Hq % m->Hkv == 0, EVICT_E_INVALID, "Hq=%d is not a multiple of Hkv=%d", m->Hq, m->Hkv);
  EVICT_REQUIRE(m->k <= m->E, EVICT_E_INVALID, "k=%d exceeds E=%d", m->k, m->E);
  EVICT_REQUIRE(m->rms_eps >= 0.0f && m->rope_theta >= 0.0f, EVICT_E_INVALID, "rms_eps and rope_theta must be >= 0");
  EVICT_REQUIRE(m->router_norm == 0 || m->router_norm == 1, EVICT_E_INVALID, "router_norm=%d (0 softmax, 1 sigmoid)", m->router_norm);
  const int eb = elem_bytes(m->dtype);
  EVICT_REQUIRE(m->D == 64 || m->D == 128, EVICT_E_UNSUPPORTED, "head dimension %d (supported: 64, 128)", m->D);
  EVICT_REQUIRE(m->d % 16 == 0 && m->F % 16 == 0 && (m->d * eb) % 64 == 0 && (m->F * eb) % 64 == 0,
                EVICT_E_UNSUPPORTED, "d=%d and F=%d must be multiples of 16 rows and of 64 bytes", m->d, m->F);
  EVICT_REQUIRE(m->vocab >= 0 && m->vocab % 16 == 0, EVICT_E_UNSUPPORTED, "vocab=%d must be a non-negative multiple of 16", m->vocab);
  EVICT_REQUIRE(m->k <= 64 && m->E <= 1024 && m->E % 16 == 0, EVICT_E_UNSUPPORTED,
                "k=%d (limit 64), E=%d (limit 1024, multiple of 16)", m->k, m->E);
  return EVICT_OK;
}

template <typename P>
int dev_alloc(P** p, size_t bytes, std::vector<void*>& owned) {
  void* q = nullptr;
  EVICT_HIP_CHECK(hipMalloc(&q, bytes ? bytes : 16));
  owned.push_back(q);
  *p = reinterpret_cast<P*>(q);
  return EVICT_OK;
}

}  // namespace

struct evict_ctx_owner {
  evict_ctx c;
  std::vector<void*> owned;
};

extern "C" {

int evict_create(evict_ctx** out, const evict_model_desc* m, int max_tokens, int max_batch, int max_ctx) {
  EVICT_REQUIRE(out, EVICT_E_INVALID, "evict_create: out is null");
  *out = nullptr;
  int rc = check_model(m);
  if (rc) return rc;
  EVICT_REQUIRE(max_tokens >= 1 && max_batch >= 1 && max_ctx >= 0, EVICT_E_INVALID,
                "evict_create: max_tokens=%d, max_batch=%d, max_ctx=%d", max_tokens, max_batch, max_ctx);
  EVICT_REQUIRE((long long)max_tokens * m->k <= 8192, EVICT_E_UNSUPPORTED, "max_tokens*k=%lld exceeds 8192",
                (long long)max_tokens * m->k);
  // attention scratch: the bf16 kernel cuts any context into at most 32 splits (+ the draft-node split); the
  // fp32 kernel takes 64 keys per split and is kept to 192 splits
  EVICT_REQUIRE(m->dtype == EVICT_BF16 || attn_splits_for(max_ctx) <= 192, EVICT_E_UNSUPPORTED,
                "max_ctx=%d needs more than 192 attention splits (fp32 storage: at most 12160 positions)", max_ctx);
  EVICT_REQUIRE(max_ctx <= (1 << 20), EVICT_E_UNSUPPORTED, "max_ctx=%d exceeds 1048576", max_ctx);
  EVICT_REQUIRE(m->d * (m->dtype == EVICT_BF16 ? 2 : 4) <= 16384, EVICT_E_UNSUPPORTED, "d=%d: rows above 16 KiB are not supported", m->d);
  evict_ctx_owner* o = new (std::nothrow) evict_ctx_owner();
  EVICT_REQUIRE(o, EVICT_E_INVALID, "out of host memory");
  evict_ctx& c = o->c;
  c.m = *m;
  c.max_tokens = max_tokens;
  c.max_batch = max_batch;
  c.max_ctx = max_ctx;
  c.max_splits = m->dtype == EVICT_BF16 ? kAttnMfmaMaxSplits : attn_splits_for(max_ctx);
  const size_t T = max_tokens, eb = elem_bytes(m->dtype);
  const size_t d = m->d, HqD = (size_t)m->Hq * m->D, E = m->E, k = m->k, F = m->F;
  rc = EVICT_OK;
  auto A = [&](auto** p, size_t bytes) { if (!rc) rc = dev_alloc(p, bytes, o->owned); };
  hipError_t he = hipGetDevice(&c.device);
  if (he != hipSuccess) { set_error("hipGetDevice failed: %s", hipGetErrorString(he)); delete o; return EVICT_E_HIP; }
  A(&c.status, 16);
  A(&c.anc, T * 16);
  A(&c.depth, T * 4);
  A(&c.seq_of, T * 4);
  A(&c.rope_cs, T * m->D * 4);
  A(&c.rope_rev, (size_t)(m->D / 2) * 8);
  A(&c.x_norm, T * d * eb);
  A(&c.q, T * HqD * eb);
  A(&c.part_o, (size_t)c.max_splits * T * HqD * 4);
  A(&c.part_ml, (size_t)c.max_splits * T * m->Hq * 2 * 4);
  A(&c.attn_o, T * HqD * eb);
  A(&c.h, T * d * eb);
  A(&c.h_norm, T * d * eb);
  A(&c.logits, T * E * 4);
  A(&c.topk_idx, T * k * 4);
  A(&c.topk_w, T * k * 4);
  A(&c.hist, E * 4);
  A(&c.offsets, (E + 1) * 4);
  A(&c.union_ids, E * 4);
  A(&c.union_count, 16);
  A(&c.perm, T * k * 4);
  A(&c.inv, T * k * 4);
  A(&c.work, (E + T * k / 16 + 1 + (size_t)m->n_shared * (T / 16 + 1)) * sizeof(WorkRec));  // one slot per (expert, 16-token tile)
  A(&c.sched, 16);
  A(&c.tok_of_pos, (T * k + (size_t)m->n_shared * T) * 4);
  A(&c.act, (T * k + (size_t)m->n_shared * T) * F * eb);
  A(&c.y, (T * k + (size_t)m->n_shared * T) * d * 4);
  c.lm_val = nullptr;
  c.lm_idx = nullptr;
  if (m->vocab) {
    A(&c.lm_val, (size_t)(m->vocab / 16) * T * 4);
    A(&c.lm_idx, (size_t)(m->vocab / 16) * T * 4);
  }
  A(&c.samp_stats, T * 2 * 4);
  A(&c.stack_buf[0], T * d * eb);
  A(&c.stack_buf[1], T * d * eb);
  if (!rc) {
    he = hipMemset(c.status, 0, 16);
    if (he == hipSuccess) he = hipMemset(c.sched, 0, 16);
    // rotary frequencies theta^(-2i/D) in revolutions per position, in double: the angle of a large
    // position is reduced to one turn exactly before it meets the fp32 sine and cosine
    std::vector<double> rev((size_t)(m->D / 2), 0.0);
    if (m->rope_theta > 0.0f)
      for (int i = 0; i < m->D / 2; ++i) rev[i] = pow((double)m->rope_theta, -2.0 * i / m->D) / (2.0 * M_PI);
    if (he == hipSuccess) he = hipMemcpy(c.rope_rev, rev.data(), rev.size() * 8, hipMemcpyHostToDevice);
    if (he != hipSuccess) { set_error("hipMemset failed: %s", hipGetErrorString(he)); rc = EVICT_E_HIP; }
  }
  if (!rc) rc = kernels_setup(*m);
  c.timing = 0;
  c.moe_grid = 2048;
  c.moe_pair_down = 2;
  c.moe_down_ws = 0;
  c.moe_prefetch = 1;
  c.moe_down_kernel = 1;
  c.moe_gateup_kernel = 2;
  c.moe_nt_loads = 2;
  c.dense_nt_loads = 2;
  c.dense_nt = 0;
  c.attn_target_wgs = 512;
  c.attn_waves = 0;
  c.moe_nt = 0;
  c.dense_units = 0;
  c.dense_kernel = 2;
  c.moe_lds_dma = 1;
  c.lm_units = 0;
  c.lm_nt = 0;
  c.dense_ntw = 0;
  c.moe_chunk_gateup = 1;
  c.moe_chunk_down = 1;
  for (int cu : {4, 2}) if ((m->d / 16) % cu == 0) { c.moe_chunk_down = cu; break; }
  c.attn_row_blocks = 0;
  c.timed_once = 0;
  c.capturing = 0;
  c.paging = KvPaging{nullptr, 0, 0, 0};
  c.t_dev = nullptr;
  c.prof_ev[0] = c.prof_ev[1] = nullptr;
  for (int i = 0; !rc && i < 2; ++i) {
    he = hipEventCreate(&c.prof_ev[i]);
    if (he != hipSuccess) { set_error("hipEventCreate failed: %s", hipGetErrorString(he)); rc = EVICT_E_HIP; }
  }
  int n_ev = 0;
  for (; !rc && n_ev <= EVICT_N_STAGES; ++n_ev) {
    he = hipEventCreate(&c.ev[n_ev]);
    if (he != hipSuccess) { set_error("hipEventCreate failed: %s", hipGetErrorString(he)); rc = EVICT_E_HIP; break; }
  }
  if (rc) {
    for (int i = 0; i < n_ev; ++i) (void)hipEventDestroy(c.ev[i]);
    for (int i = 0; i < 2; ++i) if (c.prof_ev[i]) (void)hipEventDestroy(c.prof_ev[i]);
    for (void* p : o->owned) (void)hipFree(p);
    delete o;
    return rc;
  }
  *out = &o->c;
  return EVICT_OK;
}

int evict_destroy(evict_ctx* ctx) {
  if (!ctx) return EVICT_OK;
  evict_ctx_owner* o = reinterpret_cast<evict_ctx_owner*>(ctx);  // c is the first member
  int rc = EVICT_OK;
  for (int i = 0; i <= EVICT_N_STAGES; ++i) (void)hipEventDestroy(ctx->ev[i]);
  for (int i = 0; i < 2; ++i) (void)hipEventDestroy(ctx->prof_ev[i]);
  for (void* p : o->owned) {
    hipError_t e = hipFree(p);
    if (e != hipSuccess) { set_error("hipFree failed: %s", hipGetErrorString(e)); rc = EVICT_E_HIP; }
  }
  delete o;
  return rc;
}

size_t evict_packed_bytes(int dtype, int rows, int cols) {
  if (rows <= 0 || cols <= 0 || (dtype != EVICT_F32 && dtype != EVICT_BF16)) return 0;
  return (size_t)rows * cols * elem_bytes(dtype);
}

int evict_pack_dense(int dtype, const void* w, int rows, int cols, void* dst, void* stream) {
  EVICT_REQUIRE(w && dst, EVICT_E_INVALID, "evict_pack_dense: null pointer");
  EVICT_REQUIRE(dtype == EVICT_F32 || dtype == EVICT_BF16, EVICT_E_INVALID, "evict_pack_dense: unknown dtype %d", dtype);
  EVICT_REQUIRE(rows > 0 && cols > 0, EVICT_E_INVALID, "evict_pack_dense: rows=%d cols=%d", rows, cols);
  EVICT_REQUIRE(rows % 16 == 0 && (cols * elem_bytes(dtype)) % 64 == 0, EVICT_E_UNSUPPORTED,
                "evict_pack_dense: rows=%d must be a multiple of 16 and a row (%d bytes) a multiple of 64 bytes", rows,
                cols * elem_bytes(dtype));
  EVICT_REQUIRE(aligned16(w) && aligned16(dst) && w != dst, EVICT_E_INVALID, "evict_pack_dense: pointers must be distinct and 16-byte aligned");
  return launch_pack(w, 0, rows, cols, dtype, dst, 0, 1, 0, 1, 0, (hipStream_t)stream);
}

int evict_pack_qkv(const evict_model_desc* m, const void* wq, const void* wk, const void* wv, void* dst, void* stream) {
  int rc = check_model(m);
  if (rc) return rc;
  EVICT_REQUIRE(wq && wk && wv && dst, EVICT_E_INVALID, "evict_pack_qkv: null pointer");
  EVICT_REQUIRE(aligned16(wq) && aligned16(wk) && aligned16(wv) && aligned16(dst), EVICT_E_INVALID,
                "evict_pack_qkv: pointers must be 16-byte aligned");
  hipStream_t s = (hipStream_t)stream;
  const int q_rows = m->Hq * m->D, kv_rows = m->Hkv * m->D;
  rc = launch_pack(wq, 0, q_rows, m->d, m->dtype, dst, 0, 1, 0, 1, m->D, s);
  if (!rc) rc = launch_pack(wk, 0, kv_rows, m->d, m->dtype, dst, q_rows / 16, 1, 0, 1, m->D, s);
  if (!rc) rc = launch_pack(wv, 0, kv_rows, m->d, m->dtype, dst, (q_rows + kv_rows) / 16, 1, 0, 1, m->D, s);
  return rc;
}

int evict_pack_experts(const evict_model_desc* m, int n_experts, const void* w_gate, const void* w_up, const void* w_down,
                       void* dst_gateup, void* dst_down, void* stream) {
  int rc = check_model(m);
  if (rc) return rc;
  EVICT_REQUIRE(w_gate && w_up && w_down && dst_gateup && dst_down, EVICT_E_INVALID, "evict_pack_experts: null pointer");
  EVICT_REQUIRE(n_experts >= 1 && n_experts <= 65535, EVICT_E_INVALID, "evict_pack_experts: n_experts=%d", n_experts);
  EVICT_REQUIRE(aligned16(w_gate) && aligned16(w_up) && aligned16(w_down) && aligned16(dst_gateup) && aligned16(dst_down),
                EVICT_E_INVALID, "evict_pack_experts: pointers must be 16-byte aligned");
  hipStream_t s = (hipStream_t)stream;
  const int eb = elem_bytes(m->dtype);
  const long long fd = (long long)m->F * m->d * eb;
  const int fs = m->F / 16;
  // gate strip s -> strip 2s, up strip s -> strip 2s+1 of the expert's gate/up matrix
  rc = launch_pack(w_gate, fd, m->F, m->d, m->dtype, dst_gateup, 0, 2, 2 * fs, n_experts, 0, s);
  if (!rc) rc = launch_pack(w_up, fd, m->F, m->d, m->dtype, dst_gateup, 1, 2, 2 * fs, n_experts, 0, s);
  if (!rc) rc = launch_pack(w_down, fd, m->d, m->F, m->dtype, dst_down, 0, 1, m->d / 16, n_experts, 0, s);
  return rc;
}

int evict_device_status(evict_ctx* ctx, int32_t* status_host, void* stream) {
  EVICT_REQUIRE(ctx && status_host, EVICT_E_INVALID, "evict_device_status: null pointer");
  EVICT_HIP_CHECK(hipMemcpyAsync(status_host, ctx->status, 4, hipMemcpyDeviceToHost, (hipStream_t)stream));
  EVICT_HIP_CHECK(hipStreamSynchronize((hipStream_t)stream));
  return EVICT_OK;
}

static int check_layer_args(evict_ctx* ctx, const evict_layer_weights* w, const int32_t* tree_off, const int32_t* parent, int B,
                            int T, const void* k_cache, const void* v_cache, int64_t kv_seq_stride, int64_t kv_head_stride,
                            const int32_t* ctx_len, int max_ctx_host, const void* x_in, void* x_out, void* k_new, void* v_new) {
  EVICT_REQUIRE(ctx && w && tree_off && parent && ctx_len && x_in && x_out && k_new && v_new, EVICT_E_INVALID,
                "evict_verify_layer: null pointer argument");
  const evict_model_desc& m = ctx->m;
  EVICT_REQUIRE(w->g_attn && w->g_moe && w->wqkv_packed && w->wo_packed && w->wg_packed && w->w_gateup_packed && w->w_down_packed,
                EVICT_E_INVALID, "evict_verify_layer: null weight pointer");
  EVICT_REQUIRE(m.n_shared == 0 || (w->ws_gateup_packed && w->ws_down_packed), EVICT_E_INVALID,
                "evict_verify_layer: shared-expert weights missing");
  EVICT_REQUIRE(B >= 1 && B <= ctx->max_batch, EVICT_E_INVALID, "evict_verify_layer: B=%d outside [1,%d]", B, ctx->max_batch);
  EVICT_REQUIRE(T >= B && T <= ctx->max_tokens, EVICT_E_INVALID, "evict_verify_layer: T=%d outside [%d,%d]", T, B, ctx->max_tokens);
  EVICT_REQUIRE(T <= (long long)B * EVICT_MAX_TREE_NODES, EVICT_E_UNSUPPORTED, "evict_verify_layer: more than %d nodes per tree",
                EVICT_MAX_TREE_NODES);
  EVICT_REQUIRE(max_ctx_host >= 0 && max_ctx_host <= ctx->max_ctx, EVICT_E_INVALID,
                "evict_verify_layer: max_ctx_host=%d outside [0,%d]", max_ctx_host, ctx->max_ctx);
  EVICT_REQUIRE(max_ctx_host == 0 || (k_cache && v_cache), EVICT_E_INVALID, "evict_verify_layer: null KV cache");
  if (ctx->paging.table) {
    // paged caches: kv_seq_stride is the distance between pages
    const int64_t page = (int64_t)1 << ctx->paging.page_shift;
    EVICT_REQUIRE(kv_head_stride >= page * m.D, EVICT_E_INVALID, "paged KV: kv_head_stride=%lld is smaller than page_size*D",
                  (long long)kv_head_stride);
    EVICT_REQUIRE(kv_seq_stride >= kv_head_stride * m.Hkv, EVICT_E_INVALID, "paged KV: page_stride=%lld is smaller than Hkv*kv_head_stride",
                  (long long)kv_seq_stride);
    EVICT_REQUIRE(kv_head_stride % 8 == 0 && kv_seq_stride % 8 == 0, EVICT_E_INVALID, "paged KV: strides must be multiples of 8 elements");
  } else {
    EVICT_REQUIRE(kv_head_stride >= (int64_t)max_ctx_host * m.D && kv_seq_stride >= 0, EVICT_E_INVALID,
                  "evict_verify_layer: kv_head_stride=%lld is smaller than max_ctx_host*D", (long long)kv_head_stride);
    EVICT_REQUIRE(B == 1 || kv_seq_stride >= kv_head_stride * m.Hkv, EVICT_E_INVALID, "evict_verify_layer: kv_seq_stride too small");
  }
  EVICT_REQUIRE(aligned16(x_in) && aligned16(x_out) && aligned16(k_new) && aligned16(v_new) && aligned16(k_cache) && aligned16(v_cache),
                EVICT_E_INVALID, "evict_verify_layer: pointers must be 16-byte aligned");
  EVICT_REQUIRE(x_in != x_out, EVICT_E_INVALID, "evict_verify_layer: x_out must not alias x_in");

  return EVICT_OK;
}

static int verify_layer_impl(evict_ctx* ctx, const evict_layer_weights* w, const int32_t* tree_off, const int32_t* parent, int B,
                             int T, const void* k_cache, const void* v_cache, int64_t kv_seq_stride, int64_t kv_head_stride,
                             const int32_t* ctx_len, int max_ctx_host, const void* x_in, void* x_out, void* k_new, void* v_new,
                             const evict_layer_aux* aux, int tree_ready, void* stream, int x_norm_ready = 0,
                             const void* next_gain = nullptr) {
  const evict_model_desc& m = ctx->m;
  hipStream_t s = (hipStream_t)stream;
  const int eb = elem_bytes(m.dtype);
  const int HqD = m.Hq * m.D;
  const bool timing = ctx->timing != 0;
#define EVICT_MARK(i_) do { if (timing) EVICT_HIP_CHECK(hipEventRecord(ctx->ev[i_], s)); } while (0)
  EVICT_MARK(0);
  // (in a stack the previous layer's combine has already normalised this layer's input)
  int rc = (tree_ready && x_norm_ready) ? EVICT_OK
                                        : launch_prep(ctx, tree_off, parent, B, T, ctx_len, max_ctx_host, x_in, w->g_attn, tree_ready, s);
  if (rc) return rc;
  EVICT_MARK(1);

  // token tiles per workgroup in the dense projections: two from 64 tokens on (measured)
  const int nt_dense = ctx->dense_nt ? ctx->dense_nt : (T >= 64 ? 2 : 1);
  const int dense_tiles = (T + 16 * nt_dense - 1) / (16 * nt_dense);
  // QKV takes two token tiles per workgroup already from 17 tokens on: as fast as two workgroups per strip when
  // both tiles are full (9.6 vs 9.8 us at 32 tokens), and when the count in device memory turns out to fill one
  // tile only, there is no second grid half whose workgroups leave at once (7.3 vs 9.4 us at 7 of 32 tokens)
  const int nt_qkv = ctx->dense_nt ? ctx->dense_nt : (T > 16 ? 2 : 1);
  const int qkv_tiles = (T + 16 * nt_qkv - 1) / (16 * nt_qkv);
  // QKV: a workgroup takes several consecutive strips, so its token operand is fetched once and its weight loads
  // run ahead across the strips (measured: 2 strips with one token tile, 4 with more; the output projection, with a
  // third of the strips and twice the contraction length, is better left at one)
  const int qkv_units = ctx->dense_units ? ctx->dense_units : (qkv_tiles >= 2 ? 4 : 2);
  auto dense_grid = [&](int units, int du, int tiles) { return (((units + du - 1) / du + 7) / 8) * 8 * tiles; };
  // Projection weights are fetched with non-temporal loads. (Measured on a 48-layer stack, where no weight is
  // read twice within an iteration: never slower than ordinary loads at 1, 2 and 4 token tiles per strip, 5 % faster
  // per iteration at one tile. A benchmark that rotates few enough weight copies to keep the projections of all
  // of them in the 256 MB memory-side cache shows the opposite and is measuring that cache.)
  const int dense_ntl = ctx->dense_nt_loads == 2 ? 1 : ctx->dense_nt_loads;
  // With many token tiles the projections are ordinary dense GEMMs: one strip per wavefront with the token
  // operand of the workgroup in LDS (gemm_dense_strip_kernel) instead of the contraction split. Measured:
  // pays from 128 tokens on with two token tiles per workgroup (the operand of two tiles must fit in LDS), from
  // 256 tokens on with one.
  auto dense_strip_shape = [&](const GemmArgs& a, int* ntw) {
    if (ctx->dense_kernel == 0) return false;
    int nt = ctx->dense_ntw ? ctx->dense_ntw : (dense_strip_applies(a, 2) ? 2 : 1);
    if (!dense_strip_applies(a, nt)) return false;
    if (ctx->dense_kernel == 2 && T < (nt == 2 ? 128 : 256)) return false;
    *ntw = nt;
    return true;
  };
  {  // q, k, v projections + rotation (positions ctx_len + depth)
    GemmArgs a = {};
    a.W = (const u32x4*)w->wqkv_packed;
    a.n_strips = (m.Hq + 2 * m.Hkv) * m.D / 16;
    a.nkb = m.d * eb / 64;
    a.X = ctx->x_norm;
    a.ldx_bytes = (long long)m.d * eb;
    a.T = T;
    a.T_dev = ctx->t_dev;
    a.out0 = ctx->q; a.out1 = k_new; a.out2 = v_new;
    a.rope_cs = ctx->rope_cs;
    a.Hq = m.Hq; a.Hkv = m.Hkv; a.D = m.D;
    a.dense_tiles = qkv_tiles;
    a.dense_units = qkv_units;
    a.nt_loads = dense_ntl;
    int ntw;
    rc = dense_strip_shape(a, &ntw) ? launch_gemm_dense_strip(m.dtype, EPI_QKV, a, ntw, s)
                                         : launch_gemm(m.dtype, EPI_QKV, a, nt_qkv, dense_grid(a.n_strips, qkv_units, qkv_tiles), s);
    if (rc) return rc;
    if (aux && aux->q) EVICT_HIP_CHECK(hipMemcpyAsync(aux->q, ctx->q, (size_t)T * HqD * eb, hipMemcpyDeviceToDevice, s));
  }
  EVICT_MARK(2);
  rc = launch_attention(ctx, k_cache, v_cache, kv_seq_stride, kv_head_stride, ctx_len, max_ctx_host, tree_off, B, T, k_new,
                        v_new, aux ? aux->attn_out : nullptr, s);
  if (rc) return rc;
  EVICT_MARK(3);
  {  // output projection + residual
    GemmArgs a = {};
    a.W = (const u32x4*)w->wo_packed;
    a.n_strips = m.d / 16;
    a.nkb = HqD * eb / 64;
    a.X = ctx->attn_o;
    a.ldx_bytes = (long long)HqD * eb;
    a.T = T;
    a.T_dev = ctx->t_dev;
    a.out0 = ctx->h;
    a.ldo = m.d;
    a.resid = x_in;
    a.dense_tiles = dense_tiles;
    a.dense_units = 1;
    a.nt_loads = dense_ntl;
    int ntw;
    rc = dense_strip_shape(a, &ntw) ? launch_gemm_dense_strip(m.dtype, EPI_RESID, a, ntw, s)
                                         : launch_gemm(m.dtype, EPI_RESID, a, nt_dense, dense_grid(a.n_strips, 1, dense_tiles), s);
    if (rc) return rc;
    if (aux && aux->h) EVICT_HIP_CHECK(hipMemcpyAsync(aux->h, ctx->h, (size_t)T * m.d * eb, hipMemcpyDeviceToDevice, s));
  }
  EVICT_MARK(4);
  rc = launch_router(ctx, w->g_moe, w->wg_packed, T, aux, s);
  if (rc) return rc;
  EVICT_MARK(5);
  // token tiles per work-list slot of the grouped GEMMs: 2 once experts mostly have more than 16 tokens
  const int nt_exp = ctx->moe_nt ? ctx->moe_nt : 1;
  // expert weights fetched with non-temporal loads: they are read once per call (up to the further token tiles
  // of an expert, which run next to the first on the same XCD), and kept out of the caches they leave the
  // activations and projection weights of the next kernels there
  const int moe_nt = ctx->moe_nt_loads == 2 ? 1 : ctx->moe_nt_loads;
  rc = launch_topk_union(ctx, T, aux, 16 * nt_exp, s);
  if (rc) return rc;
  if (aux) {
    if (aux->union_ids) EVICT_HIP_CHECK(hipMemcpyAsync(aux->union_ids, ctx->union_ids, (size_t)m.E * 4, hipMemcpyDeviceToDevice, s));
    if (aux->union_count) EVICT_HIP_CHECK(hipMemcpyAsync(aux->union_count, ctx->union_count, 4, hipMemcpyDeviceToDevice, s));
    if (aux->hist) EVICT_HIP_CHECK(hipMemcpyAsync(aux->hist, ctx->hist, (size_t)m.E * 4, hipMemcpyDeviceToDevice, s));
  }
  EVICT_MARK(6);
  {  // gate/up projections of the union experts + SiLU gating
    GemmArgs a = {};
    a.W = (const u32x4*)w->w_gateup_packed;
    a.W_shared = (const u32x4*)w->ws_gateup_packed;
    a.n_routed = m.E;
    a.n_strips = 2 * m.F / 16;
    a.nkb = m.d * eb / 64;
    a.group_stride = (long long)a.n_strips * a.nkb * 64;
    a.X = ctx->h_norm;
    a.ldx_bytes = (long long)m.d * eb;
    a.grouped = 1;
    a.union_count = ctx->sched; a.work = ctx->work; a.tok_of_pos = ctx->tok_of_pos;
    a.x_by_token = 1;
    a.out0 = ctx->act;
    a.ldo = m.F;
    a.prefetch = ctx->moe_prefetch;
    a.nt_loads = moe_nt;
    a.lds_dma = ctx->moe_lds_dma;
    // (one strip pair per wavefront pays once experts often have several token tiles: measured from 64 tokens on
    // where its chunks line up with the XCDs, see gateup_waves, else from 128)
    a.wave_strip = ctx->moe_gateup_kernel == 2 ? (T >= (gateup_waves(a) != 4 ? 64 : 128) ? 1 : 0) : ctx->moe_gateup_kernel;
    a.chunk_units = ctx->moe_chunk_gateup;
    rc = launch_gemm(m.dtype, EPI_SWIGLU, a, nt_exp, ctx->moe_grid, s);
    if (rc) return rc;
  }
  EVICT_MARK(7);
  {  // down projections
    GemmArgs a = {};
    a.W = (const u32x4*)w->w_down_packed;
    a.W_shared = (const u32x4*)w->ws_down_packed;
    a.n_routed = m.E;
    a.n_strips = m.d / 16;
    a.nkb = m.F * eb / 64;
    a.group_stride = (long long)a.n_strips * a.nkb * 64;
    a.X = ctx->act;
    a.ldx_bytes = (long long)m.F * eb;
    a.grouped = 1;
    a.union_count = ctx->sched; a.work = ctx->work; a.tok_of_pos = ctx->tok_of_pos;
    a.x_by_token = 0;
    a.out0 = ctx->y;
    a.ldo = m.d;
    a.chunk_units = ctx->moe_chunk_down;
    a.prefetch = ctx->moe_prefetch;
    a.wave_strip = ctx->moe_down_kernel;
    a.nt_loads = moe_nt;
    // An expert with more than 16 tokens has several 16-token slots. The strip-per-wavefront kernel can take two
    // consecutive ones of an expert through one weight stream (its operand of 32 tokens must fit the LDS budget of
    // that kernel); measured to pay once there are enough tokens for such experts to be common.
    // 16 strips per workgroup stage a slot's operand half as often: pays with many slots, costs with few (measured)
    // (from 128 tokens on at expert width 768, from 64 on at width 1408, where an operand is twice as long)
    a.down_ws = ctx->moe_down_ws ? ctx->moe_down_ws : (T >= (a.nkb == 44 ? 64 : 128) ? 16 : 8);
    const bool wide16 = a.nkb == 44 && a.down_ws == 16 && a.n_strips % 16 == 0 && m.dtype == EVICT_BF16;  // (expert width 1408)
    const bool can_pair = nt_exp == 1 && a.wave_strip && a.n_strips % 8 == 0 && (a.nkb * 2 <= 64 || wide16);
    const bool pair = can_pair && (ctx->moe_pair_down == 2 ? T >= 128 : ctx->moe_pair_down == 1);
    a.pair_tiles = pair ? 1 : 0;
    rc = launch_gemm(m.dtype, EPI_F32, a, pair ? 2 : nt_exp, ctx->moe_grid, s);
    if (rc) return rc;
  }
  EVICT_MARK(8);
  // (the always-on shared experts are extra slots of the work list: same two launches)
  EVICT_MARK(9);
  rc = launch_combine(ctx, T, x_out, next_gain, s);
  if (rc) return rc;
  EVICT_MARK(10);
  if (timing) ctx->timed_once = 1;
#undef EVICT_MARK
  return EVICT_OK;
}

int evict_verify_layer(evict_ctx* ctx, const evict_layer_weights* w, const int32_t* tree_off, const int32_t* parent, int B,
                       int T, const void* k_cache, const void* v_cache, int64_t kv_seq_stride, int64_t kv_head_stride,
                       const int32_t* ctx_len, int max_ctx_host, const void* x_in, void* x_out, void* k_new, void* v_new,
                       const evict_layer_aux* aux, void* stream) {
  int rc = check_layer_args(ctx, w, tree_off, parent, B, T, k_cache, v_cache, kv_seq_stride, kv_head_stride, ctx_len,
                            max_ctx_host, x_in, x_out, k_new, v_new);
  if (rc) return rc;
  return verify_layer_impl(ctx, w, tree_off, parent, B, T, k_cache, v_cache, kv_seq_stride, kv_head_stride, ctx_len,
                           max_ctx_host, x_in, x_out, k_new, v_new, aux, 0, stream);
}

int evict_verify_stack(evict_ctx* ctx, const evict_layer_weights* layers, int n_layers, const int32_t* tree_off,
                       const int32_t* parent, int B, int T, const void* const* k_caches, const void* const* v_caches,
                       int64_t kv_seq_stride, int64_t kv_head_stride, const int32_t* ctx_len, int max_ctx_host,
                       const void* x_in, void* x_out, void* const* k_new, void* const* v_new, void* stream) {
  EVICT_REQUIRE(ctx && layers && k_new && v_new, EVICT_E_INVALID, "evict_verify_stack: null pointer argument");
  EVICT_REQUIRE(n_layers >= 1, EVICT_E_INVALID, "evict_verify_stack: n_layers=%d", n_layers);
  EVICT_REQUIRE(max_ctx_host == 0 || (k_caches && v_caches), EVICT_E_INVALID, "evict_verify_stack: null KV cache arrays");
  for (int l = 0; l < n_layers; ++l) {
    const void* in = l == 0 ? x_in : ctx->stack_buf[(l - 1) & 1];
    void* out = l == n_layers - 1 ? x_out : ctx->stack_buf[l & 1];
    const void* kc = k_caches ? k_caches[l] : nullptr;
    const void* vc = v_caches ? v_caches[l] : nullptr;
    int rc = check_layer_args(ctx, layers + l, tree_off, parent, B, T, kc, vc, kv_seq_stride, kv_head_stride, ctx_len,
                              max_ctx_host, in, out, k_new[l], v_new[l]);
    if (rc) return rc;
    rc = verify_layer_impl(ctx, layers + l, tree_off, parent, B, T, kc, vc, kv_seq_stride, kv_head_stride, ctx_len,
                           max_ctx_host, in, out, k_new[l], v_new[l], nullptr, l > 0, stream, l > 0,
                           l + 1 < n_layers ? layers[l + 1].g_attn : nullptr);
    if (rc) return rc;
  }
  return EVICT_OK;
}

int evict_verify_stack_paged(evict_ctx* ctx, const evict_layer_weights* layers, int n_layers, const int32_t* tree_off,
                             const int32_t* parent, int B, int T, const void* const* k_pools, const void* const* v_pools,
                             int64_t page_stride, int64_t kv_head_stride, const int32_t* block_table, int table_stride,
                             int page_size, int n_pages, const int32_t* ctx_len, int max_ctx_host, const void* x_in,
                             void* x_out, void* const* k_new, void* const* v_new, void* stream) {
  EVICT_REQUIRE(ctx && block_table && k_pools && v_pools, EVICT_E_INVALID, "evict_verify_stack_paged: null pointer argument");
  EVICT_REQUIRE(page_size >= 1 && page_size <= 65536 && (page_size & (page_size - 1)) == 0, EVICT_E_INVALID,
                "evict_verify_stack_paged: page_size=%d must be a power of two in [1, 65536]", page_size);
  EVICT_REQUIRE(n_pages >= 1 && table_stride >= 1, EVICT_E_INVALID, "evict_verify_stack_paged: n_pages=%d table_stride=%d", n_pages,
                table_stride);
  EVICT_REQUIRE((int64_t)table_stride * page_size >= max_ctx_host, EVICT_E_INVALID,
                "evict_verify_stack_paged: a table row covers %lld positions, max_ctx_host is %d", (long long)table_stride * page_size,
                max_ctx_host);
  int shift = 0;
  while ((1 << shift) < page_size) ++shift;
  ctx->paging = KvPaging{block_table, table_stride, shift, n_pages};
  const int rc = evict_verify_stack(ctx, layers, n_layers, tree_off, parent, B, T, k_pools, v_pools, page_stride, kv_head_stride,
                                    ctx_len, max_ctx_host, x_in, x_out, k_new, v_new, stream);
  ctx->paging = KvPaging{nullptr, 0, 0, 0};
  return rc;
}

// LM head GEMM (vocabulary rows x T tokens): launch shape. A workgroup takes several consecutive strips, so the
// token operand is fetched once for all of them and the weight loads run ahead across strips, and two token
// tiles once there are more than 16 tokens, so the weights are streamed once instead of once per tile.
// Measured at 151936 x 2048, bf16: 233 -> 134 us at 32 tokens, 120 -> 116 us at 8.
static int launch_lm_gemm(evict_ctx* ctx, int epi, GemmArgs& a, int T, hipStream_t s) {
  const int nt = ctx->lm_nt ? ctx->lm_nt : (T > 16 ? 2 : 1);
  a.dense_tiles = (T + 16 * nt - 1) / (16 * nt);
  a.dense_units = ctx->lm_units ? ctx->lm_units : (T > 16 ? 8 : 2);
  a.nt_loads = ctx->dense_nt_loads == 2 ? (a.dense_tiles == 1 ? 1 : 0) : ctx->dense_nt_loads;  // every strip is read by one workgroup
  const int grid = (((a.n_strips + a.dense_units - 1) / a.dense_units + 7) / 8) * 8 * a.dense_tiles;
  return launch_gemm(ctx->m.dtype, epi, a, nt, grid, s);
}

int evict_lm_head_argmax(evict_ctx* ctx, const void* x, const void* g_final, const void* wlm_packed, int T, int32_t* next,
                         float* best_logit, void* x_norm_out, void* stream) {
  EVICT_REQUIRE(ctx && x && g_final && wlm_packed && next, EVICT_E_INVALID, "evict_lm_head_argmax: null pointer argument");
  const evict_model_desc& m = ctx->m;
  EVICT_REQUIRE(m.vocab > 0, EVICT_E_INVALID, "evict_lm_head_argmax: the context was created without a vocabulary size");
  EVICT_REQUIRE(T >= 1 && T <= ctx->max_tokens, EVICT_E_INVALID, "evict_lm_head_argmax: T=%d outside [1,%d]", T, ctx->max_tokens);
  EVICT_REQUIRE(aligned16(x) && aligned16(wlm_packed), EVICT_E_INVALID, "evict_lm_head_argmax: pointers must be 16-byte aligned");
  hipStream_t s = (hipStream_t)stream;
  const int eb = elem_bytes(m.dtype);
  int rc = launch_prep(ctx, nullptr, nullptr, 1, T, nullptr, 0, x, g_final, 1, s);  // final RMSNorm only
  if (rc) return rc;
  if (x_norm_out) EVICT_HIP_CHECK(hipMemcpyAsync(x_norm_out, ctx->x_norm, (size_t)T * m.d * eb, hipMemcpyDeviceToDevice, s));
  GemmArgs a = {};
  a.W = (const u32x4*)wlm_packed;
  a.n_strips = m.vocab / 16;
  a.nkb = m.d * eb / 64;
  a.X = ctx->x_norm;
  a.ldx_bytes = (long long)m.d * eb;
  a.T = T;
  a.T_dev = ctx->t_dev;
  a.out0 = ctx->lm_val;
  a.out1 = ctx->lm_idx;
  a.ldo = a.n_strips;
  rc = launch_lm_gemm(ctx, EPI_ARGMAX, a, T, s);
  if (rc) return rc;
  return launch_argmax_reduce(ctx->lm_val, ctx->lm_idx, a.n_strips, a.n_strips, T, next, best_logit, ctx->t_dev, s);
}

int evict_lm_head_logits(evict_ctx* ctx, const void* x, const void* g_final, const void* wlm_packed, int T, float* logits,
                         void* x_norm_out, void* stream) {
  EVICT_REQUIRE(ctx && x && g_final && wlm_packed && logits, EVICT_E_INVALID, "evict_lm_head_logits: null pointer argument");
  const evict_model_desc& m = ctx->m;
  EVICT_REQUIRE(m.vocab > 0, EVICT_E_INVALID, "evict_lm_head_logits: the context was created without a vocabulary size");
  EVICT_REQUIRE(T >= 1 && T <= ctx->max_tokens, EVICT_E_INVALID, "evict_lm_head_logits: T=%d outside [1,%d]", T, ctx->max_tokens);
  EVICT_REQUIRE(aligned16(x) && aligned16(wlm_packed) && aligned16(logits), EVICT_E_INVALID,
                "evict_lm_head_logits: pointers must be 16-byte aligned");
  hipStream_t s = (hipStream_t)stream;
  const int eb = elem_bytes(m.dtype);
  int rc = launch_prep(ctx, nullptr, nullptr, 1, T, nullptr, 0, x, g_final, 1, s);  // final RMSNorm only
  if (rc) return rc;
  if (x_norm_out) EVICT_HIP_CHECK(hipMemcpyAsync(x_norm_out, ctx->x_norm, (size_t)T * m.d * eb, hipMemcpyDeviceToDevice, s));
  GemmArgs a = {};
  a.W = (const u32x4*)wlm_packed;
  a.n_strips = m.vocab / 16;
  a.nkb = m.d * eb / 64;
  a.X = ctx->x_norm;
  a.ldx_bytes = (long long)m.d * eb;
  a.T = T;
  a.T_dev = ctx->t_dev;
  a.out0 = logits;
  a.ldo = m.vocab;
  return launch_lm_gemm(ctx, EPI_F32, a, T, s);
}

int evict_profile_cost_union(evict_ctx* ctx, const evict_layer_weights* layers, int n_layers, const int32_t* tree_off,
                             const int32_t* parent, int Kmax, const void* const* k_caches, const void* const* v_caches,
                             int64_t kv_head_stride, const int32_t* ctx_len, int max_ctx_host, const void* x_in, void* x_out,
                             void* const* k_new, void* const* v_new, int reps, float* cost_host, float* union_mean_host,
                             void* stream) {
  EVICT_REQUIRE(ctx && cost_host, EVICT_E_INVALID, "evict_profile_cost: null pointer argument");
  EVICT_REQUIRE(Kmax >= 1 && Kmax <= ctx->max_tokens && Kmax <= EVICT_MAX_TREE_NODES, EVICT_E_INVALID,
                "evict_profile_cost: Kmax=%d outside [1, min(max_tokens, %d)]", Kmax, EVICT_MAX_TREE_NODES);
  EVICT_REQUIRE(reps >= 1 && reps <= 4096, EVICT_E_INVALID, "evict_profile_cost: reps=%d outside [1, 4096]", reps);
  EVICT_REQUIRE(!ctx->capturing, EVICT_E_INVALID, "evict_profile_cost synchronises: not inside a graph capture");
  EVICT_REQUIRE(!ctx->t_dev, EVICT_E_INVALID, "evict_profile_cost: switch evict_dynamic_tokens off first (the profile sets the length per call)");
  hipStream_t s = (hipStream_t)stream;
  cost_host[0] = 0.0f;
  if (union_mean_host) union_mean_host[0] = 0.0f;
  for (int k = 1; k <= Kmax; ++k) {
    EVICT_HIP_CHECK(hipMemsetAsync(ctx->sched + 1, 0, 4, s));  // running total of union sizes
    // B = 1: the kernels take the tree size from T, so the first k nodes are verified as a tree of their own
    for (int r = -1; r < reps; ++r) {
      if (r == 0) EVICT_HIP_CHECK(hipEventRecord(ctx->prof_ev[0], s));
      int rc = evict_verify_stack(ctx, layers, n_layers, tree_off, parent, 1, k, k_caches, v_caches, 0, kv_head_stride,
                                  ctx_len, max_ctx_host, x_in, x_out, k_new, v_new, stream);
      if (rc) return rc;
    }
    EVICT_HIP_CHECK(hipEventRecord(ctx->prof_ev[1], s));
    EVICT_HIP_CHECK(hipEventSynchronize(ctx->prof_ev[1]));
    float ms = 0.0f;
    EVICT_HIP_CHECK(hipEventElapsedTime(&ms, ctx->prof_ev[0], ctx->prof_ev[1]));
    cost_host[k] = ms / (float)reps;
    if (union_mean_host) {
      int32_t total = 0;
      EVICT_HIP_CHECK(hipMemcpyAsync(&total, ctx->sched + 1, 4, hipMemcpyDeviceToHost, s));
      EVICT_HIP_CHECK(hipStreamSynchronize(s));
      union_mean_host[k] = (float)total / ((float)(reps + 1) * (float)n_layers);
    }
  }
  return EVICT_OK;
}

int evict_profile_cost(evict_ctx* ctx, const evict_layer_weights* layers, int n_layers, const int32_t* tree_off,
                       const int32_t* parent, int Kmax, const void* const* k_caches, const void* const* v_caches,
                       int64_t kv_head_stride, const int32_t* ctx_len, int max_ctx_host, const void* x_in, void* x_out,
                       void* const* k_new, void* const* v_new, int reps, float* cost_host, void* stream) {
  return evict_profile_cost_union(ctx, layers, n_layers, tree_off, parent, Kmax, k_caches, v_caches, kv_head_stride, ctx_len,
                                  max_ctx_host, x_in, x_out, k_new, v_new, reps, cost_host, nullptr, stream);
}

int evict_union_total(evict_ctx* ctx, int64_t* total_host, int reset, void* stream) {
  EVICT_REQUIRE(ctx && total_host, EVICT_E_INVALID, "evict_union_total: null argument");
  EVICT_REQUIRE(!ctx->capturing, EVICT_E_INVALID, "evict_union_total synchronises: not inside a graph capture");
  hipStream_t s = (hipStream_t)stream;
  int32_t total = 0;
  EVICT_HIP_CHECK(hipMemcpyAsync(&total, ctx->sched + 1, 4, hipMemcpyDeviceToHost, s));
  if (reset) EVICT_HIP_CHECK(hipMemsetAsync(ctx->sched + 1, 0, 4, s));
  EVICT_HIP_CHECK(hipStreamSynchronize(s));
  *total_host = (int64_t)(uint32_t)total;
  return EVICT_OK;
}

int evict_dynamic_tokens(evict_ctx* ctx, const int32_t* count_dev) {
  EVICT_REQUIRE(ctx, EVICT_E_INVALID, "evict_dynamic_tokens: null context");
  ctx->t_dev = count_dev;
  return EVICT_OK;
}

int evict_tune(evict_ctx* ctx, const char* key, int value) {
  EVICT_REQUIRE(ctx && key, EVICT_E_INVALID, "evict_tune: null argument");
  if (!strcmp(key, "moe_grid")) {
    EVICT_REQUIRE(value >= 1 && value <= 65535, EVICT_E_INVALID, "evict_tune: moe_grid=%d out of range", value);
    ctx->moe_grid = value;
  } else if (!strcmp(key, "moe_prefetch")) {
    EVICT_REQUIRE(value == 1 || value == 3, EVICT_E_INVALID, "evict_tune: moe_prefetch must be 1 or 3");
    ctx->moe_prefetch = value;
  } else if (!strcmp(key, "moe_chunk_gateup")) {
    EVICT_REQUIRE(value >= 1 && (ctx->m.F / 16) % value == 0, EVICT_E_INVALID, "evict_tune: moe_chunk_gateup=%d must divide F/16", value);
    ctx->moe_chunk_gateup = value;
  } else if (!strcmp(key, "moe_chunk_down")) {
    EVICT_REQUIRE(value >= 1 && (ctx->m.d / 16) % value == 0, EVICT_E_INVALID, "evict_tune: moe_chunk_down=%d must divide d/16", value);
    ctx->moe_chunk_down = value;
  } else if (!strcmp(key, "moe_nt")) {
    EVICT_REQUIRE(value >= 0 && value <= 2, EVICT_E_INVALID, "evict_tune: moe_nt must be 0 (auto), 1 or 2");
    ctx->moe_nt = value;
  } else if (!strcmp(key, "attn_waves")) {
    EVICT_REQUIRE(value == 0 || value == 4 || value == 8, EVICT_E_INVALID, "evict_tune: attn_waves must be 0 (auto), 4 or 8");
    ctx->attn_waves = value;
  } else if (!strcmp(key, "attn_target_wgs")) {
    EVICT_REQUIRE(value >= 1 && value <= 65536, EVICT_E_INVALID, "evict_tune: attn_target_wgs out of range");
    ctx->attn_target_wgs = value;
  } else if (!strcmp(key, "dense_units")) {
    EVICT_REQUIRE(value >= 0 && value <= 16, EVICT_E_INVALID, "evict_tune: dense_units must be in [0, 16] (0 = auto)");
    ctx->dense_units = value;
  } else if (!strcmp(key, "lm_nt")) {
    EVICT_REQUIRE(value >= 0 && value <= 2, EVICT_E_INVALID, "evict_tune: lm_nt must be 0, 1 or 2");
    ctx->lm_nt = value;
  } else if (!strcmp(key, "lm_units")) {
    EVICT_REQUIRE(value >= 0 && value <= 64, EVICT_E_INVALID, "evict_tune: lm_units must be in [0, 64] (0 = auto)");
    ctx->lm_units = value;
  } else if (!strcmp(key, "moe_lds_dma")) {
    EVICT_REQUIRE(value == 0 || value == 1, EVICT_E_INVALID, "evict_tune: moe_lds_dma must be 0 or 1");
    ctx->moe_lds_dma = value;
  } else if (!strcmp(key, "dense_kernel")) {
    EVICT_REQUIRE(value >= 0 && value <= 2, EVICT_E_INVALID, "evict_tune: dense_kernel must be 0, 1 or 2 (auto)");
    ctx->dense_kernel = value;
  } else if (!strcmp(key, "dense_ntw")) {
    EVICT_REQUIRE(value >= 0 && value <= 2, EVICT_E_INVALID, "evict_tune: dense_ntw must be 0 (auto), 1 or 2");
    ctx->dense_ntw = value;
  } else if (!strcmp(key, "dense_nt")) {
    EVICT_REQUIRE(value >= 0 && value <= 2, EVICT_E_INVALID, "evict_tune: dense_nt must be 0 (auto), 1 or 2");
    ctx->dense_nt = value;
  } else if (!strcmp(key, "moe_nt_loads")) {
    EVICT_REQUIRE(value >= 0 && value <= 2, EVICT_E_INVALID, "evict_tune: moe_nt_loads must be 0, 1 or 2 (auto)");
    ctx->moe_nt_loads = value;
  } else if (!strcmp(key, "dense_nt_loads")) {
    EVICT_REQUIRE(value >= 0 && value <= 2, EVICT_E_INVALID, "evict_tune: dense_nt_loads must be 0, 1 or 2 (auto)");
    ctx->dense_nt_loads = value;
  } else if (!strcmp(key, "moe_gateup_kernel")) {
    EVICT_REQUIRE(value >= 0 && value <= 2, EVICT_E_INVALID, "evict_tune: moe_gateup_kernel must be 0, 1 or 2 (auto)");
    ctx->moe_gateup_kernel = value;
  } else if (!strcmp(key, "moe_down_kernel")) {
    EVICT_REQUIRE(value == 0 || value == 1, EVICT_E_INVALID, "evict_tune: moe_down_kernel must be 0 or 1");
    ctx->moe_down_kernel = value;
  } else if (!strcmp(key, "moe_down_ws")) {
    EVICT_REQUIRE(value == 0 || value == 8 || value == 16, EVICT_E_INVALID, "evict_tune: moe_down_ws must be 0 (auto), 8 or 16");
    ctx->moe_down_ws = value;
  } else if (!strcmp(key, "moe_pair_down")) {
    EVICT_REQUIRE(value >= 0 && value <= 2, EVICT_E_INVALID, "evict_tune: moe_pair_down must be 0, 1 or 2 (auto)");
    ctx->moe_pair_down = value;
  } else if (!strcmp(key, "attn_row_blocks")) {
    EVICT_REQUIRE(value >= 0 && value <= 64, EVICT_E_INVALID, "evict_tune: attn_row_blocks=%d out of range", value);
    ctx->attn_row_blocks = value;
  } else {
    set_error("evict_tune: unknown key '%s'", key);
    return EVICT_E_INVALID;
  }
  return EVICT_OK;
}

int evict_stage_timing(evict_ctx* ctx, int enable) {
  EVICT_REQUIRE(ctx, EVICT_E_INVALID, "evict_stage_timing: null context");
  ctx->timing = enable ? 1 : 0;
  if (!enable) ctx->timed_once = 0;
  return EVICT_OK;
}

int evict_stage_times(evict_ctx* ctx, float* ms_host) {
  EVICT_REQUIRE(ctx && ms_host, EVICT_E_INVALID, "evict_stage_times: null pointer");
  EVICT_REQUIRE(ctx->timed_once, EVICT_E_INVALID, "evict_stage_times: no call has been timed (enable evict_stage_timing first)");
  EVICT_HIP_CHECK(hipEventSynchronize(ctx->ev[EVICT_N_STAGES]));
  for (int i = 0; i < EVICT_N_STAGES; ++i) EVICT_HIP_CHECK(hipEventElapsedTime(&ms_host[i], ctx->ev[i], ctx->ev[i + 1]));
  return EVICT_OK;
}

// ---- HIP-graph capture of a sequence of calls (one graph per verification length) ----
struct evict_graph {
  hipGraph_t graph;
  hipGraphExec_t exec;
  int device;
};

int evict_graph_begin(evict_ctx* ctx, void* stream) {
  EVICT_REQUIRE(ctx, EVICT_E_INVALID, "evict_graph_begin: null context");
  EVICT_REQUIRE(stream != nullptr, EVICT_E_INVALID, "evict_graph_begin: the default (null) stream cannot be captured");
  EVICT_REQUIRE(!ctx->timing, EVICT_E_INVALID, "evict_graph_begin: switch evict_stage_timing off before capturing");
  EVICT_REQUIRE(!ctx->capturing, EVICT_E_INVALID, "evict_graph_begin: a capture is already open on this context");
  EVICT_HIP_CHECK(hipStreamBeginCapture((hipStream_t)stream, hipStreamCaptureModeThreadLocal));
  ctx->capturing = 1;
  return EVICT_OK;
}

int evict_graph_end(evict_ctx* ctx, void* stream, evict_graph** out) {
  EVICT_REQUIRE(ctx && out, EVICT_E_INVALID, "evict_graph_end: null argument");
  EVICT_REQUIRE(ctx->capturing, EVICT_E_INVALID, "evict_graph_end: no capture is open on this context");
  *out = nullptr;
  ctx->capturing = 0;
  hipGraph_t g = nullptr;
  EVICT_HIP_CHECK(hipStreamEndCapture((hipStream_t)stream, &g));
  EVICT_REQUIRE(g != nullptr, EVICT_E_HIP, "evict_graph_end: the capture was invalidated (a call inside it failed or synchronised)");
  hipGraphExec_t ex = nullptr;
  hipError_t e = hipGraphInstantiate(&ex, g, nullptr, nullptr, 0);
  if (e != hipSuccess) {
    (void)hipGraphDestroy(g);
    set_error("hipGraphInstantiate: %s", hipGetErrorString(e));
    return EVICT_E_HIP;
  }
  evict_graph* h = new (std::nothrow) evict_graph{g, ex, ctx->device};
  if (!h) {
    (void)hipGraphExecDestroy(ex);
    (void)hipGraphDestroy(g);
    set_error("evict_graph_end: out of host memory");
    return EVICT_E_HIP;
  }
  *out = h;
  return EVICT_OK;
}

int evict_graph_launch(evict_graph* g, void* stream) {
  EVICT_REQUIRE(g, EVICT_E_INVALID, "evict_graph_launch: null graph");
  EVICT_HIP_CHECK(hipGraphLaunch(g->exec, (hipStream_t)stream));
  return EVICT_OK;
}

int evict_graph_destroy(evict_graph* g) {
  if (!g) return EVICT_OK;
  (void)hipGraphExecDestroy(g->exec);
  (void)hipGraphDestroy(g->graph);
  delete g;
  return EVICT_OK;
}

}  // extern "C"
