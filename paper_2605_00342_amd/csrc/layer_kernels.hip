// Kernels of one verification pass through an MoE decoder layer (Sec. 2.1-2.2) other than
// the streaming GEMM: weight packing, tree preparation + RMSNorm, tree-masked attention
// (split over the context) and its merge, router top-k, un-permute/combine.
#include "ctx.h"
#include "gemm_stream.h"
#include "layer_launch.h"
#include "union_device.h"

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
                                                   float eps, const double* __restrict__ rope_rev, int D, uint64_t* __restrict__ anc,
                                                   int32_t* __restrict__ depth, int32_t* __restrict__ seq_of,
                                                   float* __restrict__ rope_cs, void* __restrict__ x_norm,
                                                   int32_t* __restrict__ status, int n_single, int norm_only,
                                                   const int* __restrict__ t_dev) {
  constexpr int EB = ST::kBytes;
  constexpr int CE = 16 / EB;
  constexpr int MAXC = 4;  // 16-byte chunks of the row per thread (d <= 256*CE*MAXC)
  __shared__ int s_par[EVICT_MAX_TREE_NODES];
  __shared__ int s_b, s_depth;
  __shared__ float s_red[4];
  const int t = blockIdx.x, tid = threadIdx.x;
  if (t >= dyn_tokens(t_dev, (int)gridDim.x)) return;  // (rows past the call's actual token count)
  // the row and the gain do not depend on the tree: fetch them first
  u32x4 raw[MAXC], graw[MAXC];
#pragma unroll
  for (int i = 0; i < MAXC; ++i) {
    const int c = (tid + 256 * i) * CE;
    raw[i] = u32x4{0, 0, 0, 0};
    graw[i] = u32x4{0, 0, 0, 0};
    if (c < d) {
      raw[i] = *reinterpret_cast<const u32x4*>((const char*)x + ((size_t)t * d + c) * EB);
      graw[i] = *reinterpret_cast<const u32x4*>((const char*)gain + (size_t)c * EB);
    }
  }
  if (norm_only) {
    // the tree is already prepared (later layers of a stack, final norm): RMSNorm only
    float ss = 0.0f;
#pragma unroll
    for (int k = 0; k < MAXC; ++k)
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        if (EB == 2) {
          const float a = __uint_as_float(raw[k][u] << 16), bb = __uint_as_float(raw[k][u] & 0xFFFF0000u);
          ss += a * a + bb * bb;
        } else {
          const float a = __uint_as_float(raw[k][u]);
          ss += a * a;
        }
      }
    ss = wave_sum(ss);
    if ((tid & 63) == 0) s_red[tid >> 6] = ss;
    __syncthreads();
    const float rinv = 1.0f / sqrtf((s_red[0] + s_red[1] + s_red[2] + s_red[3]) / (float)d + eps);
#pragma unroll
    for (int k = 0; k < MAXC; ++k) {
      const int c = (tid + 256 * k) * CE;
      if (c < d) {
        u32x4 packed;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          if (EB == 2) {
            const float a = __uint_as_float(raw[k][u] << 16) * rinv * __uint_as_float(graw[k][u] << 16);
            const float bb = __uint_as_float(raw[k][u] & 0xFFFF0000u) * rinv * __uint_as_float(graw[k][u] & 0xFFFF0000u);
            packed[u] = pack_bf16x2(a, bb);
          } else {
            packed[u] = __float_as_uint(__uint_as_float(raw[k][u]) * rinv * __uint_as_float(graw[k][u]));
          }
        }
        *reinterpret_cast<u32x4*>((char*)x_norm + ((size_t)t * d + c) * EB) = packed;
      }
    }
    return;
  }
  const int half = D >> 1;
  const double rev_per_pos = tid < half ? rope_rev[tid] : 0.0;  // (requested early; used last)
  if (tid == 0) s_b = 0;
  __syncthreads();
  if (n_single == 0)
    for (int b = tid; b < B; b += 256)
      if (tree_off[b] <= t && t < tree_off[b + 1]) s_b = b;
  __syncthreads();
  const int b = s_b;
  // a single tree spans [0, T): its offsets need not be fetched
  const int lo = n_single > 0 ? 0 : tree_off[b];
  int n = n_single > 0 ? n_single : tree_off[b + 1] - lo;
  int L = ctx_len[b];
  if (n > EVICT_MAX_TREE_NODES) { n = EVICT_MAX_TREE_NODES; if (tid == 0) atomicOr(status, ST_BAD_TREE_SIZE); }
  const int i = t - lo < n ? t - lo : n - 1;
  for (int j = tid; j < n; j += 256) {
    int p = parent[lo + j];
    if (j == 0) p = -1;
    else if (p < 0 || p >= j) { p = 0; atomicOr(status, ST_BAD_PARENT); }
    s_par[j] = p;
  }
  // sum of squares while the tree loads are in flight
  float ss = 0.0f;
#pragma unroll
  for (int k = 0; k < MAXC; ++k)
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      if (EB == 2) {
        const float a = __uint_as_float(raw[k][u] << 16), bb = __uint_as_float(raw[k][u] & 0xFFFF0000u);
        ss += a * a + bb * bb;
      } else {
        const float a = __uint_as_float(raw[k][u]);
        ss += a * a;
      }
    }
  ss = wave_sum(ss);
  if ((tid & 63) == 0) s_red[tid >> 6] = ss;
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
  // RMSNorm(x[t]) * gain, rounded to the storage type
  const float ms = (s_red[0] + s_red[1] + s_red[2] + s_red[3]) / (float)d;
  const float rinv = 1.0f / sqrtf(ms + eps);
#pragma unroll
  for (int k = 0; k < MAXC; ++k) {
    const int c = (tid + 256 * k) * CE;
    if (c < d) {
      u32x4 packed;
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        if (EB == 2) {
          const float a = __uint_as_float(raw[k][u] << 16) * rinv * __uint_as_float(graw[k][u] << 16);
          const float bb = __uint_as_float(raw[k][u] & 0xFFFF0000u) * rinv * __uint_as_float(graw[k][u] & 0xFFFF0000u);
          packed[u] = pack_bf16x2(a, bb);
        } else {
          packed[u] = __float_as_uint(__uint_as_float(raw[k][u]) * rinv * __uint_as_float(graw[k][u]));
        }
      }
      *reinterpret_cast<u32x4*>((char*)x_norm + ((size_t)t * d + c) * EB) = packed;
    }
  }
  __syncthreads();
  if (L < 0 || L > max_ctx) { L = L < 0 ? 0 : max_ctx; if (tid == 0) atomicOr(status, ST_BAD_CTXLEN); }
  if (tid < half) {
    // angle = position * theta^(-2i/D): the product in turns is formed in double and reduced to
    // [-1/2, 1/2] there, so large positions stay exact; the hardware sine and cosine take turns.
    // (A zero frequency table, theta = 0, gives the identity rotation.)
    double rev = (double)(L + s_depth) * rev_per_pos;
    rev -= rint(rev);
    rope_cs[(size_t)t * D + tid] = __builtin_amdgcn_cosf((float)rev);
    rope_cs[(size_t)t * D + half + tid] = __builtin_amdgcn_sinf((float)rev);
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
    int D, int ctx_splits, int T, float* __restrict__ part_o, float* __restrict__ part_ml, const KvPaging pg,
    int32_t* __restrict__ status, int n_single) {
  extern __shared__ float s_dyn[];
  const int ldk = D + 1;
  float* s_k = s_dyn;                    // [64][D+1]
  float* s_v = s_k + kAttnKeys * ldk;    // [64][D+1]
  float* s_q = s_v + kAttnKeys * ldk;    // [4][D]
  float* s_p = s_q + 4 * D;              // [4][64]
  const int split = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int G = Hq / Hkv;
  // a single tree spans [0, T) whatever tree_off says (the cost profiler verifies prefixes of a tree that way)
  const int lo = n_single > 0 ? 0 : tree_off[b];
  int n = n_single > 0 ? n_single : tree_off[b + 1] - lo;
  n = n > EVICT_MAX_TREE_NODES ? EVICT_MAX_TREE_NODES : n;
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
      if (pg.table) {
        // paged cache: seq_stride is the distance between pages
        const int pos = key0 + j;
        int pid = pg.table[(size_t)b * pg.table_stride + (pos >> pg.page_shift)];
        if ((unsigned)pid >= (unsigned)pg.n_pages) { atomicOr(status, ST_BAD_PAGE); pid = 0; }
        src = (size_t)pid * seq_stride + (size_t)g * head_stride + (size_t)(pos & ((1 << pg.page_shift) - 1)) * D + c;
      } else {
        src = (size_t)b * seq_stride + (size_t)g * head_stride + (size_t)(key0 + j) * D + c;
      }
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

// ------------------------------------------------------------------------------------
// bf16 tree-masked attention on the matrix cores. Grid (splits * row_blocks, Hkv, B); one
// split = 128 keys of the KV cache, the last split = the draft nodes of the sequence under
// the ancestor mask. K and V of the split are staged once in LDS (K row-major, V
// transposed so that the contraction over keys reads contiguous bytes); each wavefront
// takes 16 query rows (node x query head of this KV group) at a time:
//   S^T = K Q^T  (MFMA, 16 keys x 16 rows per tile),  masked softmax numerators in
//   registers, O = P V (MFMA) with P taken straight from the S^T accumulators.
// Writes un-normalised partial outputs with their (max, sum) for the merge kernel.
// ------------------------------------------------------------------------------------
constexpr int kMfmaKeys = 128;

// NW wavefronts per workgroup, one 16-row query tile each. NW = 4: one LDS buffer, two workgroups
// per CU overlap each other's staging. NW = 8 (many row tiles, several chunks per split): two LDS
// buffers, the next chunk travels global -> registers while the current one is computed and is
// written to the other buffer afterwards; one barrier per chunk.
template <int D, int NW, bool PAGED = false>
__global__ __launch_bounds__(NW * 64) __attribute__((amdgpu_waves_per_eu(2))) void attn_partial_mfma_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ kc, const uint16_t* __restrict__ vc,
    long long seq_stride, long long head_stride, const int32_t* __restrict__ ctx_len, int max_ctx,
    const int32_t* __restrict__ tree_off, const uint16_t* __restrict__ k_new, const uint16_t* __restrict__ v_new,
    const uint64_t* __restrict__ anc, int Hq, int Hkv, int ctx_splits, int keys_per_split, int row_blocks, int T,
    float* __restrict__ part_o, float* __restrict__ part_ml, int n_single, int n_seq, const KvPaging pg,
    int32_t* __restrict__ status, int rb_major) {
  constexpr int LDK = D + 16;           // bf16 per K row in LDS: a row starts 8 banks (of 32) after the one above. A 16-byte
                                        // fragment read is served 8 lanes per clock, and those are not 8 consecutive lanes but
                                        // lanes 4a..4a+3 with lanes 4a+20..4a+23 (or 4a+12..4a+15): rows r..r+3 at one contraction
                                        // quarter with rows r+4..r+7 at the next. (Found with a probe kernel under the bank
                                        // conflict counter: a 4-bank row offset conflicts two-way, 8 banks do not.)
  constexpr int LDV = kMfmaKeys + 4;    // bf16 per V^T row in LDS: 66 dwords. The LDS serves 32 banks of 4 bytes per clock (bank
                                        // conflict counters settle this, not the data sheet): a half wavefront's 8-byte fragment
                                        // reads (16 consecutive rows, one key-pair offset) then hit 32 different banks, and with the
                                        // dword column of output tile dt XORed with 2*dt so do the transposing 4-byte writes (lanes
                                        // 8 rows apart over the 16 d-chunks, two adjacent key pairs per 32 lanes)
  constexpr int CH = D / 8;             // 16-byte chunks per row
  constexpr int KT = kMfmaKeys / 16;    // key tiles
  constexpr int KB = D / 32;            // contraction blocks of Q K^T
  constexpr int DT = D / 16;            // output column tiles
  constexpr int NT = NW * 64;           // threads
  constexpr int NBUF = NW == 8 ? 2 : 1;
  constexpr int BUF = kMfmaKeys * LDK + D * LDV;  // bf16 elements of one K + V^T buffer
  extern __shared__ __attribute__((aligned(16))) uint16_t s_kv[];  // NBUF x { K [128][LDK], V^T [D][LDV/2] key pairs }
  // 1-D grid. Workgroup ids go round-robin over the 8 XCDs, so the row blocks of one (split, KV
  // head, sequence) unit are given ids 8 apart: they share an L2 and the unit's keys and values
  // leave HBM once, not once per row block.
  const unsigned xcd = blockIdx.x & 7u, wi = blockIdx.x >> 3;
  // rb_major (a single tree whose size is only known on the device: most row blocks are likely to be empty):
  // all first row blocks get the lowest ids, so the workgroups that have work are dispatched together instead
  // of one in row_blocks (12.9 vs 14.6 us at 7 of 32 nodes); the row blocks of a unit still share an XCD. With
  // large caches the row blocks of a unit must also run at about the same time to share the unit's keys in L2,
  // hence the default order (4 x 64 nodes, contexts of 3191-5555: 71 vs 79 us).
  const unsigned nu8 = (gridDim.x >> 3) / (unsigned)row_blocks;
  const int rb = rb_major ? (int)(wi / nu8) : (int)(wi % (unsigned)row_blocks);
  const unsigned unit = rb_major ? (wi % nu8) * 8u + xcd : (wi / (unsigned)row_blocks) * 8u + xcd;
  const int nsplits_all = ctx_splits + 1;
  if (unit >= (unsigned)(nsplits_all * Hkv * n_seq)) return;
  const int split = (int)(unit % (unsigned)nsplits_all);
  const int g = (int)((unit / (unsigned)nsplits_all) % (unsigned)Hkv);
  const int b = (int)(unit / (unsigned)(nsplits_all * Hkv));
  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lo = n_single > 0 ? 0 : tree_off[b];
  int n = n_single > 0 ? n_single : tree_off[b + 1] - lo;
  n = n > EVICT_MAX_TREE_NODES ? EVICT_MAX_TREE_NODES : n;
  int L = ctx_len[b];
  L = L < 0 ? 0 : (L > max_ctx ? max_ctx : L);
  const bool tree_part = split >= ctx_splits;
  // keys of this split: a range of the cache, or the sequence's draft nodes
  const int key_begin = tree_part ? 0 : split * keys_per_split;
  int key_end = tree_part ? n : key_begin + keys_per_split;
  if (!tree_part && key_end > L) key_end = L;
  const int G = Hq / Hkv;
  const int R = n * G;
  const int ntiles = (R + 15) >> 4;
  // one 16-row query tile per wavefront (the host sizes row_blocks for that)
  const int rt = rb * NW + w;
  const bool active = rt < ntiles;
  const int kq = lane >> 4, ln = lane & 15;
  if (key_begin >= key_end) {
    // split lies beyond this sequence's context: mark its rows empty for the merge
    if (active && kq == 0 && rt * 16 + ln < R) {
      const int r = rt * 16 + ln, i = r / G, hh = r - i * G;
      const size_t prow = ((size_t)split * T + lo + i) * Hq + g * G + hh;
      part_ml[prow * 2] = -INFINITY;
      part_ml[prow * 2 + 1] = 0.0f;
    }
    return;
  }
  if (rb * NW >= ntiles) return;

  // ---- this wavefront's query rows are fetched before the K/V staging: the round trips overlap
  const float scale = 1.0f / sqrtf((float)D);
  int r = rt * 16 + ln;
  r = r < R ? r : R - 1;
  const int qi = r / G, qh = r - qi * G;
  const int t = lo + qi;
  u32x4 Qf[KB];
  uint64_t a0 = ~0ull, a1 = ~0ull;
  if (active) {
    const uint16_t* qrow = q + ((size_t)t * Hq + g * G + qh) * D + kq * 8;
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) Qf[kb] = *reinterpret_cast<const u32x4*>(qrow + kb * 32);
    if (tree_part) { a0 = anc[2 * (size_t)t]; a1 = anc[2 * (size_t)t + 1]; }
  }
  // (paged cache: seq_stride is the distance between pages and the page comes from the table per key)
  const size_t seq_off = PAGED ? 0 : (size_t)b * seq_stride;
  const uint16_t* kbase = tree_part ? k_new + ((size_t)lo * Hkv + g) * D : kc + seq_off + (size_t)g * head_stride;
  const uint16_t* vbase = tree_part ? v_new + ((size_t)lo * Hkv + g) * D : vc + seq_off + (size_t)g * head_stride;
  const size_t kstep = tree_part ? (size_t)Hkv * D : (size_t)D;  // elements between consecutive keys
  const int32_t* ptab = PAGED ? pg.table + (size_t)b * pg.table_stride : nullptr;
  const int pmask = (1 << pg.page_shift) - 1;

  // running softmax state of this wavefront's 16 rows over the chunks of the split
  f32x4 O[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) O[dt] = f32x4{0, 0, 0, 0};
  // The row sums of the rounded weights come from the matrix cores as well: P times a column of ones, as one
  // more output tile whose column 0 (lanes with ln == 0) holds the sums of rows kq*4 + j. (The vector unit is
  // the busiest unit of this kernel; the matrix cores are not.)
  f32x4 Lsum = {0, 0, 0, 0};
  const uint32_t one2 = ln == 0 ? 0x3F803F80u : 0u;  // two bf16 ones in column 0
  const u32x4 ones = {one2, one2, one2, one2};
  float m_run = -INFINITY;  // running maximum of the scaled scores of row ln
  const float c2 = scale * 1.44269504088896341f;  // raw score -> exponent of 2

  // K/V of a chunk travel global -> registers -> LDS, all loads issued before the first LDS
  // write so one memory round trip covers the chunk. Paged cache: the page ids of all of this
  // thread's keys are requested first (one more round trip per chunk, not one per key), ids
  // outside the pool are replaced by page 0 and reported once.
  constexpr int KI = kMfmaKeys * CH / NT, VI = (kMfmaKeys / 2) * CH / NT;
  u32x4 kreg[KI], vreg0[VI], vreg1[VI];
  // contiguous caches: where this thread's pieces sit relative to the first key of a chunk (elements), worked
  // out once; per chunk only the chunk's base moves, and that is the same for every lane
  unsigned koff[KI], voff[VI];
#pragma unroll
  for (int it = 0; it < KI; ++it) {
    const int idx = tid + NT * it, j = idx / CH, c = idx - j * CH;
    koff[it] = (unsigned)j * (unsigned)kstep + c * 8;
  }
#pragma unroll
  for (int it = 0; it < VI; ++it) {
    const int idx = tid + NT * it, jp = idx / CH, c = idx - jp * CH;
    voff[it] = (unsigned)(2 * jp) * (unsigned)kstep + c * 8;
  }
  auto fetch_chunk = [&](int kc0) __attribute__((always_inline)) {
    int nk = key_end - kc0;
    nk = nk > kMfmaKeys ? kMfmaKeys : nk;
    const bool paged = PAGED && !tree_part;
    if (!paged) {
      const uint16_t* kchunk = kbase + (size_t)kc0 * kstep;
      const uint16_t* vchunk = vbase + (size_t)kc0 * kstep;
#pragma unroll
      for (int it = 0; it < KI; ++it) {
        const int j = (tid + NT * it) / CH;
        kreg[it] = u32x4{0, 0, 0, 0};  // keys past the end are zeros
        if (j < nk) kreg[it] = *reinterpret_cast<const u32x4*>(kchunk + koff[it]);
      }
#pragma unroll
      for (int it = 0; it < VI; ++it) {
        const int jp = (tid + NT * it) / CH;
        vreg0[it] = u32x4{0, 0, 0, 0};
        vreg1[it] = u32x4{0, 0, 0, 0};
        if (2 * jp < nk) vreg0[it] = *reinterpret_cast<const u32x4*>(vchunk + voff[it]);
        if (2 * jp + 1 < nk) vreg1[it] = *reinterpret_cast<const u32x4*>(vchunk + voff[it] + kstep);
      }
      return;
    }
    int pk[KI], pv0[VI], pv1[VI];
    if (paged) {
#pragma unroll
      for (int it = 0; it < KI; ++it) {
        const int j = (tid + NT * it) / CH;
        pk[it] = j < nk ? ptab[(kc0 + j) >> pg.page_shift] : 0;
      }
#pragma unroll
      for (int it = 0; it < VI; ++it) {
        const int jp = (tid + NT * it) / CH;
        pv0[it] = 2 * jp < nk ? ptab[(kc0 + 2 * jp) >> pg.page_shift] : 0;
        pv1[it] = 2 * jp + 1 < nk ? ptab[(kc0 + 2 * jp + 1) >> pg.page_shift] : 0;
      }
      bool bad = false;
#pragma unroll
      for (int it = 0; it < KI; ++it) {
        const bool ok = (unsigned)pk[it] < (unsigned)pg.n_pages;
        bad |= !ok;
        pk[it] = ok ? pk[it] : 0;
      }
#pragma unroll
      for (int it = 0; it < VI; ++it) {
        const bool ok0 = (unsigned)pv0[it] < (unsigned)pg.n_pages, ok1 = (unsigned)pv1[it] < (unsigned)pg.n_pages;
        bad |= !ok0 || !ok1;
        pv0[it] = ok0 ? pv0[it] : 0;
        pv1[it] = ok1 ? pv1[it] : 0;
      }
      if (bad) atomicOr(status, ST_BAD_PAGE);
    }
    // element offset of key position `pos` (page id `pid` when paged) from kbase / vbase
    auto key_off = [&](int pos, int pid) -> size_t {
      return paged ? (size_t)pid * seq_stride + (size_t)(pos & pmask) * D : (size_t)pos * kstep;
    };
#pragma unroll
    for (int it = 0; it < KI; ++it) {
      const int idx = tid + NT * it, j = idx / CH, c = idx - j * CH;
      kreg[it] = u32x4{0, 0, 0, 0};  // keys past the end are zeros
      if (j < nk) kreg[it] = *reinterpret_cast<const u32x4*>(kbase + key_off(kc0 + j, paged ? pk[it] : 0) + c * 8);
    }
#pragma unroll
    for (int it = 0; it < VI; ++it) {
      const int idx = tid + NT * it, jp = idx / CH, c = idx - jp * CH;
      vreg0[it] = u32x4{0, 0, 0, 0};
      vreg1[it] = u32x4{0, 0, 0, 0};
      if (2 * jp < nk) vreg0[it] = *reinterpret_cast<const u32x4*>(vbase + key_off(kc0 + 2 * jp, paged ? pv0[it] : 0) + c * 8);
      if (2 * jp + 1 < nk) vreg1[it] = *reinterpret_cast<const u32x4*>(vbase + key_off(kc0 + 2 * jp + 1, paged ? pv1[it] : 0) + c * 8);
    }
  };
  // K row-major, V transposed (two keys per dword)
  auto write_chunk = [&](int buf) __attribute__((always_inline)) {
    uint16_t* wk = s_kv + (size_t)buf * BUF;
    uint32_t* wv = reinterpret_cast<uint32_t*>(wk + kMfmaKeys * LDK);
#pragma unroll
    for (int it = 0; it < KI; ++it) {
      const int idx = tid + NT * it, j = idx / CH, c = idx - j * CH;
      *reinterpret_cast<u32x4*>(wk + j * LDK + c * 8) = kreg[it];
    }
#pragma unroll
    for (int it = 0; it < VI; ++it) {
      const int idx = tid + NT * it, jp = idx / CH, c = idx - jp * CH;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const uint32_t a = vreg0[it][i], bb = vreg1[it][i];
        const int col = jp ^ ((c >> 1) << 1);  // rows c*8 .. c*8+7 belong to output tile c/2
        wv[(c * 8 + 2 * i) * (LDV / 2) + col] = (a & 0xFFFFu) | (bb << 16);
        wv[(c * 8 + 2 * i + 1) * (LDV / 2) + col] = (a >> 16) | (bb & 0xFFFF0000u);
      }
    }
  };
  fetch_chunk(key_begin);
  write_chunk(0);
  __syncthreads();
  int cur = 0;
  // One chunk, compiled twice: for a whole chunk of cache keys (every key visible to every row: no mask, no test
  // for masked scores) and for the ragged last chunk / the draft nodes under the ancestor mask. (With the choice
  // left to run time the compiler keeps one body and pays the mask arithmetic on every chunk.)
  auto run_chunk = [&](auto full_tag, int kc0) __attribute__((always_inline)) {
    constexpr bool full = decltype(full_tag)::value;
    int nkeys = key_end - kc0;
    nkeys = nkeys > kMfmaKeys ? kMfmaKeys : nkeys;
    const bool more = kc0 + kMfmaKeys < key_end;
    if (NBUF == 2 && more) fetch_chunk(kc0 + kMfmaKeys);  // in flight during the MFMA work below
    const uint16_t* s_k = s_kv + (size_t)cur * BUF;
    const uint32_t* s_vt = reinterpret_cast<const uint32_t*>(s_k + kMfmaKeys * LDK);
    if (active) {
    // S^T tiles: lane holds keys kt*16 + kq*4 + j of query row ln. The K fragments of the next
    // tile are requested from LDS before the MFMAs of the current one (two register buffers), so
    // the LDS latency hides behind the matrix work instead of preceding every MFMA.
    f32x4 S[KT];
    float mx = -INFINITY;
    u32x4 kf[2][KB];
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) kf[0][kb] = *reinterpret_cast<const u32x4*>(s_k + ln * LDK + kb * 32 + kq * 8);
#pragma unroll
    for (int kt = 0; kt < KT; ++kt) {
      if (kt + 1 < KT) {
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
          kf[(kt + 1) & 1][kb] = *reinterpret_cast<const u32x4*>(s_k + ((kt + 1) * 16 + ln) * LDK + kb * 32 + kq * 8);
      }
      __builtin_amdgcn_sched_barrier(0);
      f32x4 acc = {0, 0, 0, 0};
#pragma unroll
      for (int kb = 0; kb < KB; ++kb) acc = mfma_block<BF16>(kf[kt & 1][kb], Qf[kb], acc);
      // (scores stay unscaled here: the scale is positive, so the maximum commutes with it, and it is applied
      // inside the one multiply-add that feeds the exponential below)
      if (full) {  // a whole chunk of cache keys: every key is visible to every row
        // (maximum as the median with +inf: one instruction each, where fmaxf first spends one per operand on
        // quieting signalling NaNs, which matrix-core outputs of finite inputs cannot be)
        const float m01 = __builtin_amdgcn_fmed3f(acc[0], acc[1], INFINITY), m23 = __builtin_amdgcn_fmed3f(acc[2], acc[3], INFINITY);
        mx = __builtin_amdgcn_fmed3f(mx, __builtin_amdgcn_fmed3f(m01, m23, INFINITY), INFINITY);
      } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int key = kt * 16 + kq * 4 + j;  // (the draft-node split has a single chunk: key = node index)
          const uint64_t word = key < 64 ? a0 : a1;
          const bool vis = key < nkeys && ((word >> (key & 63)) & 1ull);
          acc[j] = vis ? acc[j] : -INFINITY;
          mx = fmaxf(mx, acc[j]);
        }
      }
      S[kt] = acc;
      __builtin_amdgcn_sched_barrier(0);
    }
    mx = fmaxf(mx, __shfl_xor(mx, 16));
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    // online softmax: new running maximum, rescale of what has been accumulated so far
    const float m_new = fmaxf(m_run, mx * scale);
    const float alpha = m_run == -INFINITY ? 0.0f : __expf(m_run - m_new);
    const float moff = -m_new * 1.44269504088896341f;  // exp(s*scale - m) = 2^(s*c2 + moff)
    u32x4 Pf[KT / 2];
#pragma unroll
    for (int kt = 0; kt < KT; ++kt) {
      uint32_t pk[2];
#pragma unroll
      for (int jj = 0; jj < 2; ++jj) {
        // (2^(-inf) is 0 for a masked key as long as m is finite, which a visible key guarantees;
        // rows without any visible key in this chunk have m_new = -inf and need the explicit zero)
        const float p0 = (full || S[kt][2 * jj] != -INFINITY) ? __builtin_amdgcn_exp2f(fmaf(S[kt][2 * jj], c2, moff)) : 0.0f;
        const float p1 = (full || S[kt][2 * jj + 1] != -INFINITY) ? __builtin_amdgcn_exp2f(fmaf(S[kt][2 * jj + 1], c2, moff)) : 0.0f;
        pk[jj] = pack_bf16x2(p0, p1);
      }
      // contraction block kt/2 takes keys 32b + 4kq + {0..3} (even tile) and 32b + 16 + 4kq + {0..3} (odd tile)
      if (kt & 1) { Pf[kt >> 1][2] = pk[0]; Pf[kt >> 1][3] = pk[1]; }
      else        { Pf[kt >> 1][0] = pk[0]; Pf[kt >> 1][1] = pk[1]; }
    }
    // O = O * alpha + P V: lane holds rows kq*4 + j (their alpha lives in lane kq*4 + j), column dt*16 + ln.
    // Once the running maxima have settled no row is rescaled any more: the multiplications are skipped then.
    if (__builtin_amdgcn_ballot_w64(m_new != m_run)) {
      f32x4 ar;
#pragma unroll
      for (int j = 0; j < 4; ++j) ar[j] = __shfl(alpha, kq * 4 + j);
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) O[dt] *= ar;
      Lsum *= ar;
    }
    m_run = m_new;
#pragma unroll
    for (int bk = 0; bk < KT / 2; ++bk) Lsum = mfma_block<BF16>(Pf[bk], ones, Lsum);  // the sums use the rounded weights
    // V^T fragments of the next output tile are requested before the MFMAs of the current one
    auto load_v = [&](u32x4(&dst)[KT / 2], int dt) {
#pragma unroll
      for (int bk = 0; bk < KT / 2; ++bk) {
        const uint32_t* vrow = s_vt + (dt * 16 + ln) * (LDV / 2);
        const uint2 lo2 = *reinterpret_cast<const uint2*>(vrow + ((bk * 16 + kq * 2) ^ (dt << 1)));
        const uint2 hi2 = *reinterpret_cast<const uint2*>(vrow + ((bk * 16 + kq * 2 + 8) ^ (dt << 1)));
        dst[bk] = u32x4{lo2.x, lo2.y, hi2.x, hi2.y};
      }
    };
    u32x4 vf[2][KT / 2];
    load_v(vf[0], 0);
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
      if (dt + 1 < DT) load_v(vf[(dt + 1) & 1], dt + 1);
      __builtin_amdgcn_sched_barrier(0);
      f32x4 acc = O[dt];
#pragma unroll
      for (int bk = 0; bk < KT / 2; ++bk) acc = mfma_block<BF16>(Pf[bk], vf[dt & 1][bk], acc);
      O[dt] = acc;
      __builtin_amdgcn_sched_barrier(0);
    }
    }  // active
    if (NBUF == 2) {
      if (more) write_chunk(cur ^ 1);  // nobody reads that buffer during this iteration
      __syncthreads();
      cur ^= 1;
    } else if (more) {
      __syncthreads();  // the chunk has been consumed by every wavefront
      fetch_chunk(kc0 + kMfmaKeys);
      write_chunk(0);
      __syncthreads();
    }
  };
  int kc0 = key_begin;
  if (!tree_part)
    for (; kc0 + kMfmaKeys <= key_end; kc0 += kMfmaKeys) run_chunk(std::true_type{}, kc0);
  if (kc0 < key_end) run_chunk(std::false_type{}, kc0);  // (a cache range ends with at most one ragged chunk; the draft nodes are one chunk)
  if (!active) return;
  if (kq == 0 && rt * 16 + ln < R) {
    const size_t prow = ((size_t)split * T + t) * Hq + g * G + qh;
    part_ml[prow * 2] = m_run;
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int r2 = rt * 16 + kq * 4 + j;
    if (r2 < R) {
      const int i2 = r2 / G, h2 = r2 - i2 * G;
      const size_t prow = ((size_t)split * T + lo + i2) * Hq + g * G + h2;
      if (ln == 0) part_ml[prow * 2 + 1] = Lsum[j];
      float* dst = part_o + prow * D + ln;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) dst[dt * 16] = O[dt][j];
    }
  }
}

// merge of the per-split partial softmaxes. D/4 lanes per (token, head) row, each with four
// consecutive output columns; blockDim / (D/4) rows per workgroup (D is 64 or 128, so the lanes of a
// row sit in one wavefront; one-wavefront workgroups when there are few rows, so that the serial walk
// over the splits is spread over more CUs). Empty splits carry max = -inf and their partial rows are never read
// into the sum. The partial rows of the first splits are requested before the (max, sum) pairs
// are reduced, so the two round trips overlap.
constexpr int kMergeBatch = 17;  // 16 context splits + the draft-node split: the default shape of a 2048-key context

template <typename ST>
__global__ __launch_bounds__(256) void attn_merge_kernel(const float* __restrict__ part_o, const float* __restrict__ part_ml,
                                                         int nsplits, int rows, int D, void* __restrict__ out,
                                                         void* __restrict__ aux_out, int Hq, const int* __restrict__ t_dev) {
  const int lpr = D >> 2;  // lanes per row: 16 or 32
  const int tid = threadIdx.x;
  const int row = blockIdx.x * ((int)blockDim.x / lpr) + tid / lpr;
  const int c4 = tid & (lpr - 1);
  // (`rows` = tokens x heads the partials were laid out for; rows past the call's actual token count hold nothing)
  if (row >= rows || row >= dyn_tokens(t_dev, rows / Hq) * Hq) return;  // (no barrier follows)
  const size_t sstride = (size_t)rows * D;
  const float* po = part_o + (size_t)row * D + c4 * 4;
  const float* pml = part_ml + (size_t)row * 2;
  f32x4 v[kMergeBatch];
#pragma unroll
  for (int i = 0; i < kMergeBatch; ++i)
    v[i] = i < nsplits ? *reinterpret_cast<const f32x4*>(po + (size_t)i * sstride) : f32x4{0, 0, 0, 0};
  // global maximum and normaliser: the lanes of a row share the splits between them
  float M = -INFINITY;
  for (int sp = c4; sp < nsplits; sp += lpr) M = fmaxf(M, pml[(size_t)sp * rows * 2]);
  M = row16_max(M);  // lpr is 16 or 32: DPP inside the rows of 16, one shuffle across the pair
  if (lpr == 32) M = fmaxf(M, __shfl_xor(M, 16));
  float l = 0.0f;
  for (int sp = c4; sp < nsplits; sp += lpr) {
    const float2 ml = *reinterpret_cast<const float2*>(pml + (size_t)sp * rows * 2);
    l += ml.x == -INFINITY ? 0.0f : ml.y * __expf(ml.x - M);
  }
  l = row16_sum(l);
  if (lpr == 32) l += __shfl_xor(l, 16);
  f32x4 acc = {0, 0, 0, 0};
  for (int s0 = 0; s0 < nsplits; s0 += kMergeBatch) {
    if (s0 > 0) {
#pragma unroll
      for (int i = 0; i < kMergeBatch; ++i)
        v[i] = s0 + i < nsplits ? *reinterpret_cast<const f32x4*>(po + (size_t)(s0 + i) * sstride) : f32x4{0, 0, 0, 0};
    }
#pragma unroll
    for (int i = 0; i < kMergeBatch; ++i) {
      if (s0 + i < nsplits) {
        const float ms = pml[(size_t)(s0 + i) * rows * 2];
        const float sc = ms == -INFINITY ? 0.0f : __expf(ms - M);
        if (sc != 0.0f) acc += v[i] * sc;  // rows of empty splits hold no data
      }
    }
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const float r = acc[j] / l;
    store_elem<ST>(out, (size_t)row * D + c4 * 4 + j, r);
    if (aux_out) store_elem<ST>(aux_out, (size_t)row * D + c4 * 4 + j, r);
  }
}

// ------------------------------------------------------------------------------------
// router, part 1: RMSNorm(h) and scores W_g h (Eq. 4) on the matrix cores. Grid (token tiles of
// 16, expert-strip groups); 16 wavefronts split the strips of the group and the contraction
// range between them. W_g is in the packed streaming layout (16-expert strips). Every
// workgroup normalises its 16 tokens (cheap); the first strip group also stores them.
// LDS: token operand blocks [nkb][64] x 16 B, then partial scores [ksplit][strips][16][16].
// ------------------------------------------------------------------------------------
constexpr int kRouterWaves = 16;
constexpr int kRouterThreads = kRouterWaves * 64;
constexpr int kFusedTopkTokens = 32;  // up to here TopK and the union share one workgroup (measured: no loss up to 32;
                                      // two tokens per wavefront at most, which topk_union_kernel relies on)

template <typename ST>
__global__ __launch_bounds__(kRouterThreads) void router_logits_kernel(
    const void* __restrict__ h, const void* __restrict__ gain, const u32x4* __restrict__ wg_packed, int T_max, int d, int E,
    int strips_per_wg, int ksplit, float eps, void* __restrict__ h_norm, float* __restrict__ logits,
    void* __restrict__ aux_hn, float* __restrict__ aux_logits, const int* __restrict__ t_dev) {
  const int T = dyn_tokens(t_dev, T_max);
  constexpr int EB = ST::kBytes;
  constexpr int CE = 16 / EB;   // elements per 16-byte chunk
  constexpr int MAXC = 8;       // 16-byte chunks a lane keeps of its token row (d <= 64*CE*MAXC)
  extern __shared__ __attribute__((aligned(16))) unsigned char s_raw[];
  const int nkb = d * EB / 64;
  u32x4* s_b = reinterpret_cast<u32x4*>(s_raw);                       // [nkb][64] token operand blocks
  f32x4* s_p = reinterpret_cast<f32x4*>(s_raw + (size_t)nkb * 1024);  // [ksplit][strips_per_wg][64]
  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int tok0 = blockIdx.x * 16;
  const int strip_base = blockIdx.y * strips_per_wg;
  const bool writer = blockIdx.y == 0;
  // ---- one token per wavefront: the row stays in registers between the two passes
  {
    const int n = w, t = tok0 + n;
    const bool live = t < T;
    u32x4 raw[MAXC], graw[MAXC];
    float ss = 0.0f;
#pragma unroll
    for (int i = 0; i < MAXC; ++i) {
      const int c = (lane + 64 * i) * CE;
      raw[i] = u32x4{0, 0, 0, 0};
      graw[i] = u32x4{0, 0, 0, 0};
      if (c < d) {
        if (live) raw[i] = *reinterpret_cast<const u32x4*>((const char*)h + ((size_t)t * d + c) * EB);
        graw[i] = *reinterpret_cast<const u32x4*>((const char*)gain + (size_t)c * EB);
      }
    }
#pragma unroll
    for (int i = 0; i < MAXC; ++i) {
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        if (EB == 2) {
          const float a = __uint_as_float(raw[i][u] << 16), b = __uint_as_float(raw[i][u] & 0xFFFF0000u);
          ss += a * a + b * b;
        } else {
          const float a = __uint_as_float(raw[i][u]);
          ss += a * a;
        }
      }
    }
    ss = wave_sum(ss);
    const float rinv = 1.0f / sqrtf(ss / (float)d + eps);
#pragma unroll
    for (int i = 0; i < MAXC; ++i) {
      const int c = (lane + 64 * i) * CE;
      if (c < d) {
        u32x4 packed = {0, 0, 0, 0};
        if (live) {
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            if (EB == 2) {
              const float a = __uint_as_float(raw[i][u] << 16) * rinv * __uint_as_float(graw[i][u] << 16);
              const float b = __uint_as_float(raw[i][u] & 0xFFFF0000u) * rinv * __uint_as_float(graw[i][u] & 0xFFFF0000u);
              packed[u] = pack_bf16x2(a, b);
            } else {
              packed[u] = __float_as_uint(__uint_as_float(raw[i][u]) * rinv * __uint_as_float(graw[i][u]));
            }
          }
          if (writer) {
            *reinterpret_cast<u32x4*>((char*)h_norm + ((size_t)t * d + c) * EB) = packed;
            if (aux_hn) *reinterpret_cast<u32x4*>((char*)aux_hn + ((size_t)t * d + c) * EB) = packed;
          }
        }
        // position in the row -> operand block, quarter, column n. All lanes of this wavefront write column n of
        // different (block, quarter) groups, 256 bytes apart: into one bank group, unless the column is XORed with
        // (quarter | odd block << 2), which sends the 8 lanes the LDS serves per clock to 8 different bank groups
        // (the readers undo it: a permutation inside the 16 columns they read anyway)
        const int byte = c * EB;
        const int kbw = byte >> 6, qw = (byte >> 4) & 3;
        s_b[kbw * 64 + qw * 16 + (n ^ (qw | ((kbw & 1) << 2)))] = packed;
      }
    }
  }
  __syncthreads();
  // ---- scores: (expert strip, contraction slice) items round-robin over the wavefronts
  const int nstrips = E >> 4;
  int my_strips = nstrips - strip_base;
  my_strips = my_strips > strips_per_wg ? strips_per_wg : my_strips;
  const int per = (nkb + ksplit - 1) / ksplit;  // blocks per slice
  for (int item = w; item < my_strips * ksplit; item += kRouterWaves) {
    const int sl = item / ksplit, ks = item - sl * ksplit;
    const int kb_lo = ks * per;
    int kb_hi = kb_lo + per;
    kb_hi = kb_hi > nkb ? nkb : kb_hi;
    const u32x4* wp = wg_packed + (size_t)(strip_base + sl) * nkb * 64 + lane;
    f32x4 acc = {0, 0, 0, 0};
    for (int kb0 = kb_lo; kb0 < kb_hi; kb0 += 8) {
      u32x4 a[8];
#pragma unroll
      for (int j = 0; j < 8; ++j)
        if (kb0 + j < kb_hi) a[j] = wp[(size_t)(kb0 + j) * 64];
#pragma unroll
      for (int j = 0; j < 8; ++j)
        if (kb0 + j < kb_hi)
          acc = mfma_block<ST>(a[j], s_b[(kb0 + j) * 64 + (lane ^ ((lane >> 4) | (((kb0 + j) & 1) << 2)))], acc);
    }
    s_p[((size_t)ks * strips_per_wg + sl) * 64 + lane] = acc;
  }
  __syncthreads();
  // ---- sum the slices in a fixed order, publish the scores: lane holds 4 experts of one token
  for (int idx = tid; idx < my_strips * 64; idx += kRouterThreads) {
    const int sl = idx >> 6, ln = idx & 63;
    f32x4 v = s_p[(size_t)sl * 64 + ln];
    for (int ks = 1; ks < ksplit; ++ks) v += s_p[((size_t)ks * strips_per_wg + sl) * 64 + ln];
    const int t = tok0 + (ln & 15);
    if (t < T) {
      const size_t o = (size_t)t * E + (strip_base + sl) * 16 + (ln >> 4) * 4;
      *reinterpret_cast<f32x4*>(logits + o) = v;
      if (aux_logits) *reinterpret_cast<f32x4*>(aux_logits + o) = v;
    }
  }
}

// ------------------------------------------------------------------------------------
// router, part 2: TopK of every token's scores with the selected scores normalised by softmax
// or by sigmoid (Eq. 4 and the sentence after it); 16 tokens per workgroup, one per wavefront.
// Selection: one wavefront per token; scores become unsigned keys monotone in the float value,
// each of the k picks is a wavefront maximum (DPP row operations) followed by ballots that find
// the lowest expert index holding it, so equal scores go to the lower index.
// ------------------------------------------------------------------------------------
__global__ __launch_bounds__(kRouterThreads) void topk_kernel(
    const float* __restrict__ logits, int T_max, int E, int k, int norm, int32_t* __restrict__ topk_idx,
    float* __restrict__ topk_w, int32_t* __restrict__ aux_idx, float* __restrict__ aux_w, const int* __restrict__ t_dev) {
  extern __shared__ __attribute__((aligned(16))) int s_all[];
  const int T = dyn_tokens(t_dev, T_max);
  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  float* s_sel = reinterpret_cast<float*>(s_all) + w * 64;                                   // [k] per wavefront
  unsigned* s_ord = reinterpret_cast<unsigned*>(s_all) + kRouterWaves * 64 + (size_t)w * E;  // [E] per wavefront
  // The loops below are deliberately not unrolled: with a cold instruction cache the cost of
  // this small kernel follows the size of the code it walks through.
  const int t = blockIdx.x * kRouterWaves + w;  // one token per wavefront
  if (t >= T) return;
  const float* row = logits + (size_t)t * E;
  // scores as unsigned keys, monotone in the float value; 0 marks "taken" (below every key)
#pragma unroll 1
  for (int e = lane; e < E; e += 64) {
    unsigned bits = __float_as_uint(row[e]);
    bits = bits == 0x80000000u ? 0u : bits;  // -0 and +0 compare equal
    const unsigned o = bits ^ ((bits >> 31) ? 0xFFFFFFFFu : 0x80000000u);
    s_ord[e] = o == 0u ? 1u : o;             // (only the most negative NaN pattern maps to 0)
  }
  // k extractions: wavefront maximum by DPP, then the lowest index holding it by ballots
  // (LDS operations of one wavefront complete in order: s_ord / s_sel are visible to its lanes)
#pragma unroll 1
  for (int j = 0; j < k; ++j) {
    unsigned local = 0u;
#pragma unroll 1
    for (int e = lane; e < E; e += 64) {
      const unsigned o = s_ord[e];
      local = o > local ? o : local;
    }
    const unsigned best = wave_max_u32(local);
    int sel = -1;
#pragma unroll 1
    for (int base = 0; base < E && sel < 0; base += 64) {
      const int e = base + lane;
      const unsigned long long m = __ballot(e < E && s_ord[e] == best);
      if (m) sel = base + (int)__ffsll((long long)m) - 1;
    }
    if (lane == 0) {
      s_ord[sel] = 0u;
      s_sel[j] = __uint_as_float(best ^ ((best >> 31) ? 0x80000000u : 0xFFFFFFFFu));
      topk_idx[(size_t)t * k + j] = sel;
      if (aux_idx) aux_idx[(size_t)t * k + j] = sel;
    }
  }
  const float first = s_sel[0];
  const float mine = s_sel[lane < k ? lane : 0];
  // selected scores -> weights: softmax, or sigmoid divided by the sum of the selected sigmoids
  const float ex = lane < k ? (norm ? 1.0f / (1.0f + __expf(-mine)) : __expf(mine - first)) : 0.0f;
  const float denom = wave_sum(ex);
  if (lane < k) {
    const float wv = ex / denom;
    topk_w[(size_t)t * k + lane] = wv;
    if (aux_w) aux_w[(size_t)t * k + lane] = wv;
  }
}

// TopK of one token by one wavefront with the scores held in registers (E <= 64 * NR): the same
// selection rule as topk_kernel, without the LDS round trips. Lane j ends up with the j-th pick.
// Returns the expert index picked at position `lane` (for lane < k) and its softmax weight.
// Lane l holds the NR consecutive experts l*NR .. l*NR + NR - 1 (E <= 64 * NR).
template <int NR>
__device__ __forceinline__ void topk_load_row(const float* __restrict__ row, int E, int lane, float (&raw)[NR]) {
#pragma unroll
  for (int i = 0; i < NR; ++i) {
    const int e = lane * NR + i;
    raw[i] = e < E ? row[e] : 0.0f;
  }
}

// The work of this routine is all instruction issue (16 wavefronts of a workgroup share 4 SIMDs),
// so a pick is kept short: lane maximum, wavefront maximum (DPP), one ballot for the lowest lane
// holding it, and that lane alone finds and retires its lowest such expert. With experts laid out
// consecutively per lane, lowest lane then lowest register is the lowest expert index.
template <int NR>
__device__ __forceinline__ void topk_wave_regs(const float (&raw)[NR], int E, int k, int norm, int lane, int* my_idx,
                                               float* my_w) {
  unsigned key[NR];
#pragma unroll
  for (int i = 0; i < NR; ++i) {
    const int e = lane * NR + i;
    unsigned o = 0u;
    if (e < E) {
      unsigned bits = __float_as_uint(raw[i]);
      bits = bits == 0x80000000u ? 0u : bits;  // -0 and +0 compare equal
      o = bits ^ ((bits >> 31) ? 0xFFFFFFFFu : 0x80000000u);
      o = o == 0u ? 1u : o;  // 0 marks "taken" (below every key)
    }
    key[i] = o;
  }
  unsigned mine = 0u;
  int mine_idx = 0;
#pragma unroll 1
  for (int j = 0; j < k; ++j) {
    unsigned local = key[0];
#pragma unroll
    for (int i = 1; i < NR; ++i) local = key[i] > local ? key[i] : local;
    const unsigned best = wave_max_u32(local);
    const unsigned long long m = __ballot(local == best);
    const int wl = (int)__ffsll((long long)m) - 1;  // lowest lane holding the maximum
    int hit = 0;
    if (lane == wl) {
      bool done = false;
#pragma unroll
      for (int i = 0; i < NR; ++i)
        if (!done && key[i] == best) { key[i] = 0u; hit = i; done = true; }
    }
    const int sel = wl * NR + __builtin_amdgcn_readlane(hit, wl);
    if (lane == j) { mine = best; mine_idx = sel; }
  }
  const float val = __uint_as_float(mine ^ ((mine >> 31) ? 0x80000000u : 0xFFFFFFFFu));
  const float first = __shfl(val, 0);
  const float ex = lane < k ? (norm ? 1.0f / (1.0f + __expf(-val)) : __expf(val - first)) : 0.0f;
  const float denom = wave_sum(ex);
  *my_idx = mine_idx;
  *my_w = ex / denom;
}

// Register variant of topk_kernel for E <= 256: grid over groups of 16 tokens, one per wavefront.
__global__ __launch_bounds__(kRouterThreads) void topk_regs_kernel(
    const float* __restrict__ logits, int T_max, int E, int k, int norm, int32_t* __restrict__ topk_idx, float* __restrict__ topk_w,
    int32_t* __restrict__ aux_idx, float* __restrict__ aux_w, const int* __restrict__ t_dev) {
  const int T = dyn_tokens(t_dev, T_max);
  const int lane = threadIdx.x & 63;
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int t = blockIdx.x * kRouterWaves + w;
  if (t >= T) return;
  int idx;
  float wv;
  if (E <= 128) {
    float raw[2];
    topk_load_row<2>(logits + (size_t)t * E, E, lane, raw);
    topk_wave_regs<2>(raw, E, k, norm, lane, &idx, &wv);
  } else {
    float raw[4];
    topk_load_row<4>(logits + (size_t)t * E, E, lane, raw);
    topk_wave_regs<4>(raw, E, k, norm, lane, &idx, &wv);
  }
  if (lane < k) {
    topk_idx[(size_t)t * k + lane] = idx;
    topk_w[(size_t)t * k + lane] = wv;
    if (aux_idx) aux_idx[(size_t)t * k + lane] = idx;
    if (aux_w) aux_w[(size_t)t * k + lane] = wv;
  }
}

// Small token counts: TopK (register variant) and the expert union in one workgroup, the
// wavefronts taking the tokens in turn; saves a launch when there are few tokens to share out.
__global__ __launch_bounds__(kRouterThreads) void topk_union_kernel(
    const float* __restrict__ logits, int T_max, int E, int k, int norm, int32_t* __restrict__ topk_idx, float* __restrict__ topk_w,
    int32_t* __restrict__ aux_idx, float* __restrict__ aux_w, int use_masks, int32_t* __restrict__ union_ids,
    int32_t* __restrict__ union_count, int32_t* __restrict__ hist, int32_t* __restrict__ offsets,
    int32_t* __restrict__ perm, int32_t* __restrict__ inv, int32_t* __restrict__ status, WorkRec* __restrict__ work,
    int32_t* __restrict__ tok_of_pos, int32_t* __restrict__ slot_count, int n_shared, int tt, const int* __restrict__ t_dev) {
  extern __shared__ __attribute__((aligned(16))) int s_all[];
  const int T = dyn_tokens(t_dev, T_max);
  const int lane = threadIdx.x & 63;
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  // the scores of both tokens a wavefront may have (T <= 32) are requested before either is ranked
  float raw[2][4];
#pragma unroll
  for (int r = 0; r < 2; ++r)
    if (w + r * kRouterWaves < T) {
      if (E <= 128) {
        float r2[2];
        topk_load_row<2>(logits + (size_t)(w + r * kRouterWaves) * E, E, lane, r2);
        raw[r][0] = r2[0]; raw[r][1] = r2[1];
      } else {
        topk_load_row<4>(logits + (size_t)(w + r * kRouterWaves) * E, E, lane, raw[r]);
      }
    }
#pragma unroll
  for (int r = 0; r < 2; ++r) {
    const int t = w + r * kRouterWaves;
    if (t >= T) break;
    int idx;
    float wv;
    if (E <= 128) {
      const float r2[2] = {raw[r][0], raw[r][1]};
      topk_wave_regs<2>(r2, E, k, norm, lane, &idx, &wv);
    } else {
      topk_wave_regs<4>(raw[r], E, k, norm, lane, &idx, &wv);
    }
    if (lane < k) {
      s_all[t * k + lane] = idx;  // where expert_union_body expects the pairs
      topk_idx[(size_t)t * k + lane] = idx;
      topk_w[(size_t)t * k + lane] = wv;
      if (aux_idx) aux_idx[(size_t)t * k + lane] = idx;
      if (aux_w) aux_w[(size_t)t * k + lane] = wv;
    }
  }
  __syncthreads();
  expert_union_body(s_all, nullptr, T, k, E, use_masks, union_ids, union_count, hist, offsets, perm, inv, status, work,
                    tok_of_pos, slot_count, n_shared, tt);
}

// expert union and grouping (Eq. 5) with the device-side work list, one workgroup
__global__ __launch_bounds__(kRouterThreads) void union_worklist_kernel(
    const int32_t* __restrict__ topk_idx, int T_max, int k, int E, int use_masks, int32_t* __restrict__ union_ids,
    int32_t* __restrict__ union_count, int32_t* __restrict__ hist, int32_t* __restrict__ offsets,
    int32_t* __restrict__ perm, int32_t* __restrict__ inv, int32_t* __restrict__ status, WorkRec* __restrict__ work,
    int32_t* __restrict__ tok_of_pos, int32_t* __restrict__ slot_count, int n_shared, int tt, const int* __restrict__ t_dev) {
  extern __shared__ __attribute__((aligned(16))) int s_all[];
  const int T = dyn_tokens(t_dev, T_max);
  expert_union_body(s_all, topk_idx, T, k, E, use_masks, union_ids, union_count, hist, offsets, perm, inv, status, work,
                    tok_of_pos, slot_count, n_shared, tt);
}

// ------------------------------------------------------------------------------------
// LM head, second step: per token, the best (value, row) over the per-strip candidates;
// equal values go to the lower row (vocabulary) index. One workgroup per token.
// ------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void argmax_reduce_kernel(const float* __restrict__ val, const int32_t* __restrict__ idx,
                                                            int nstrips, int ld, int32_t* __restrict__ next,
                                                            float* __restrict__ best_out, const int* __restrict__ t_dev) {
  __shared__ float s_v[4];
  __shared__ int s_i[4];
  const int t = blockIdx.x, tid = threadIdx.x;
  if (t >= dyn_tokens(t_dev, (int)gridDim.x)) return;  // (rows past the call's actual token count)
  float bv = -INFINITY;
  int bi = 0x7fffffff;
  // candidates of a token are contiguous ([T][ld] with ld >= nstrips): eight loads in flight per thread
  const float* vrow = val + (size_t)t * ld;
  const int32_t* irow = idx + (size_t)t * ld;
  for (int s0 = tid; s0 < nstrips; s0 += 256 * 8) {
    float v[8];
    int i[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int s = s0 + 256 * u;
      v[u] = s < nstrips ? vrow[s] : -INFINITY;
      i[u] = s < nstrips ? irow[s] : 0x7fffffff;
    }
#pragma unroll
    for (int u = 0; u < 8; ++u)
      if (v[u] > bv || (v[u] == bv && i[u] < bi)) { bv = v[u]; bi = i[u]; }
  }
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) {
    const float ov = __shfl_xor(bv, o);
    const int oi = __shfl_xor(bi, o);
    if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
  }
  if ((tid & 63) == 0) { s_v[tid >> 6] = bv; s_i[tid >> 6] = bi; }
  __syncthreads();
  if (tid == 0) {
    for (int w = 1; w < 4; ++w)
      if (s_v[w] > bv || (s_v[w] == bv && s_i[w] < bi)) { bv = s_v[w]; bi = s_i[w]; }
    next[t] = bi;
    if (best_out) best_out[t] = bv;
  }
}

// ------------------------------------------------------------------------------------
// un-permute + weighted combine + residual (+ shared experts), fixed slot order; one workgroup
// per token. Optionally also the next layer's pre-attention RMSNorm of the row just produced
// (layer stacks: saves that layer's norm launch). The row is cut into 16-byte chunks exactly as
// prep_kernel cuts it, and the norm is the same arithmetic in the same order, so a stack gives
// bit-identical results to the layers called one by one.
// ------------------------------------------------------------------------------------
template <typename ST>
__global__ __launch_bounds__(256) void combine_kernel(const void* __restrict__ h, const float* __restrict__ y,
                                                      const float* __restrict__ w, const int32_t* __restrict__ inv,
                                                      int k, int d, int n_shared, int T_max,
                                                      void* __restrict__ out, const void* __restrict__ next_gain, float eps,
                                                      void* __restrict__ x_norm, const int* __restrict__ t_dev) {
  constexpr int EB = ST::kBytes;
  constexpr int CE = 16 / EB;
  constexpr int MAXC = 4;  // 16-byte chunks of the row per thread (d <= 256*CE*MAXC, as in prep_kernel)
  __shared__ float s_w[64];
  __shared__ int s_inv[64];
  __shared__ float s_red[4];
  const int t = blockIdx.x, tid = threadIdx.x;
  const int T = dyn_tokens(t_dev, T_max);
  if (t >= T) return;  // (rows past the call's actual token count: whole workgroup, before any barrier)
  const float* y_sh = y + (size_t)T * k * d;  // shared experts' rows follow the T * k routed pairs
  if (tid < k) {
    s_w[tid] = w[(size_t)t * k + tid];
    s_inv[tid] = inv[(size_t)t * k + tid];
  }
  __syncthreads();
  u32x4 raw[MAXC];
#pragma unroll
  for (int i = 0; i < MAXC; ++i) {
    const int c = (tid + 256 * i) * CE;
    raw[i] = u32x4{0, 0, 0, 0};
    if (c < d) {
      f32x4 acc[CE / 4];
#pragma unroll
      for (int q = 0; q < CE / 4; ++q) acc[q] = load4<ST>(h, (size_t)t * d + c + 4 * q);
      for (int j0 = 0; j0 < k; j0 += 8) {  // eight experts' rows requested together, summed in slot order
        f32x4 yv[8][CE / 4];
#pragma unroll
        for (int j = 0; j < 8; ++j)
          if (j0 + j < k) {
            const float* yr = y + (size_t)s_inv[j0 + j] * d + c;
#pragma unroll
            for (int q = 0; q < CE / 4; ++q) yv[j][q] = *reinterpret_cast<const f32x4*>(yr + 4 * q);
          }
#pragma unroll
        for (int j = 0; j < 8; ++j)
          if (j0 + j < k) {
#pragma unroll
            for (int q = 0; q < CE / 4; ++q) acc[q] += s_w[j0 + j] * yv[j][q];
          }
      }
      for (int sh = 0; sh < n_shared; ++sh) {
        const float* yr = y_sh + ((size_t)sh * T + t) * d + c;
#pragma unroll
        for (int q = 0; q < CE / 4; ++q) acc[q] += *reinterpret_cast<const f32x4*>(yr + 4 * q);
      }
      if (EB == 2) {
#pragma unroll
        for (int u = 0; u < 4; ++u)
          raw[i][u] = pack_bf16x2(acc[u >> 1][(2 * u) & 3], acc[u >> 1][(2 * u + 1) & 3]);
      } else {
#pragma unroll
        for (int u = 0; u < 4; ++u) raw[i][u] = __float_as_uint(acc[0][u]);
      }
      *reinterpret_cast<u32x4*>((char*)out + ((size_t)t * d + c) * EB) = raw[i];
    }
  }
  if (!next_gain) return;
  float ss = 0.0f;
#pragma unroll
  for (int kk = 0; kk < MAXC; ++kk)
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      if (EB == 2) {
        const float a = __uint_as_float(raw[kk][u] << 16), bb = __uint_as_float(raw[kk][u] & 0xFFFF0000u);
        ss += a * a + bb * bb;
      } else {
        const float a = __uint_as_float(raw[kk][u]);
        ss += a * a;
      }
    }
  ss = wave_sum(ss);
  if ((tid & 63) == 0) s_red[tid >> 6] = ss;
  __syncthreads();
  const float rinv = 1.0f / sqrtf((s_red[0] + s_red[1] + s_red[2] + s_red[3]) / (float)d + eps);
#pragma unroll
  for (int kk = 0; kk < MAXC; ++kk) {
    const int c = (tid + 256 * kk) * CE;
    if (c < d) {
      const u32x4 graw = *reinterpret_cast<const u32x4*>((const char*)next_gain + (size_t)c * EB);
      u32x4 packed;
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        if (EB == 2) {
          const float a = __uint_as_float(raw[kk][u] << 16) * rinv * __uint_as_float(graw[u] << 16);
          const float bb = __uint_as_float(raw[kk][u] & 0xFFFF0000u) * rinv * __uint_as_float(graw[u] & 0xFFFF0000u);
          packed[u] = pack_bf16x2(a, bb);
        } else {
          packed[u] = __float_as_uint(__uint_as_float(raw[kk][u]) * rinv * __uint_as_float(graw[u]));
        }
      }
      *reinterpret_cast<u32x4*>((char*)x_norm + ((size_t)t * d + c) * EB) = packed;
    }
  }
}

template <typename ST, int NT, int EPI>
int launch_gemm_nt(const GemmArgs& a, int grid, hipStream_t s) {
  // (non-temporal weight loads are a template parameter; they are built for the bf16 production shapes only)
#define EVICT_GEMM_LAUNCH(KBW_, PF_, EXACT_) \
  hipLaunchKernelGGL((gemm_stream_kernel<ST, NT, KBW_, PF_, EPI, EXACT_>), dim3(grid), dim3(kGemmThreads), 0, s, a)
#define EVICT_GEMM_LAUNCH_NT(KBW_, PF_, EXACT_, IS_, NS_)                                                                  \
  do {                                                                                                                    \
    if (a.nt_loads)                                                                                                       \
      hipLaunchKernelGGL((gemm_stream_kernel<ST, NT, KBW_, PF_, EPI, EXACT_, IS_, NS_, true>), dim3(grid), dim3(kGemmThreads), 0, s, a);  \
    else                                                                                                                  \
      hipLaunchKernelGGL((gemm_stream_kernel<ST, NT, KBW_, PF_, EPI, EXACT_, IS_, NS_, false>), dim3(grid), dim3(kGemmThreads), 0, s, a); \
  } while (0)
  const int nkb = a.nkb;
  const int need = ((nkb > 64 ? 64 : nkb) + kGemmWaves - 1) / kGemmWaves;
  constexpr bool bf16 = ST::kBytes == 2;
  if constexpr (bf16) {
  if (nkb % 64 == 0) {
    // the next step's 8 loads are issued right after the MFMAs, so they fly during the
    // partial-tile exchange; one buffer keeps the kernel under 128 VGPRs (2 workgroups per CU)
    if (EPI == EPI_SWIGLU && NT == 1 && a.grouped && a.chunk_units == 1 && nkb == 64 && a.prefetch != 3)
      // one gate/up strip pair per chunk: two steps, known at compile time
      EVICT_GEMM_LAUNCH_NT(8, 1, true, 1, ((EPI == EPI_SWIGLU && NT == 1) ? 2 : 0));
    else if (EPI == EPI_RESID && !a.grouped && a.prefetch != 3 &&
             (a.dense_units > 0 ? a.dense_units : 1) * ((nkb + 63) / 64) == 2)
      // two steps per workgroup (one strip of two 64-block chunks), known at compile time (the QKV
      // variant of this would spill)
      EVICT_GEMM_LAUNCH_NT(8, 1, true, 1, (EPI == EPI_RESID ? 2 : 0));
    else EVICT_GEMM_LAUNCH_NT(8, 1, true, 1, 0);
    return launch_status("gemm_stream_kernel");
  } else if (nkb == 24) {
    // 3 blocks per wavefront per strip: take 4 strips per exchange step when the chunking allows
    if (EPI == EPI_F32 && NT == 1 && a.grouped && a.chunk_units % 4 == 0)
      EVICT_GEMM_LAUNCH_NT(3, 1, true, ((EPI == EPI_F32 && NT == 1) ? 4 : 1), 0);
    else
      EVICT_GEMM_LAUNCH_NT(3, 4, true, 1, 0);
    return launch_status("gemm_stream_kernel");
  }
  }
  if (need <= 4) {
    // four stages of weight loads; three where the epilogue prefetch also needs registers (four would spill)
    constexpr int kStages = (EPI == EPI_QKV || EPI == EPI_RESID) ? 3 : 4;
    EVICT_GEMM_LAUNCH(4, kStages, false);
  } else {
    EVICT_GEMM_LAUNCH(8, 1, false);
  }
#undef EVICT_GEMM_LAUNCH
#undef EVICT_GEMM_LAUNCH_NT
  return launch_status("gemm_stream_kernel");
}

// one strip per wavefront (see gemm_wave_strip_kernel): grouped, fp32 output rows
template <typename ST, int NTW>
int launch_gemm_wave_strip(const GemmArgs& a, int grid, hipStream_t s) {
  const int nkb = a.nkb;
  const size_t lds = (size_t)nkb * 1024 * NTW;
#define EVICT_WS_LAUNCH(WIN_, NB_, EXACT_) \
  hipLaunchKernelGGL((gemm_wave_strip_kernel<ST, WIN_, NB_, EXACT_, NTW>), dim3(grid), dim3(8 * 64), lds, s, a)
#define EVICT_WS_LAUNCH_NT(WIN_, NB_, NKB_)                                                                                       \
  do {                                                                                                                           \
    if (a.nt_loads) hipLaunchKernelGGL((gemm_wave_strip_kernel<ST, WIN_, NB_, true, NTW, 8, NKB_, true>), dim3(grid), dim3(8 * 64), lds, s, a); \
    else hipLaunchKernelGGL((gemm_wave_strip_kernel<ST, WIN_, NB_, true, NTW, 8, NKB_, false>), dim3(grid), dim3(8 * 64), lds, s, a);           \
  } while (0)
  // (windows sized to stay under 128 VGPRs together with the staged operand blocks)
  if (nkb == 24 && a.down_ws == 16 && a.n_strips % 16 == 0 && ST::kBytes == 2) {
    // 16 strips per workgroup: the slot's token operand is staged half as often
    if (a.nt_loads) hipLaunchKernelGGL((gemm_wave_strip_kernel<ST, 12, 2, true, NTW, 16, 24, true>), dim3(grid), dim3(16 * 64), lds, s, a);
    else hipLaunchKernelGGL((gemm_wave_strip_kernel<ST, 12, 2, true, NTW, 16, 24, false>), dim3(grid), dim3(16 * 64), lds, s, a);
  } else if (nkb == 44 && a.down_ws == 16 && a.n_strips % 16 == 0 && ST::kBytes == 2) {
    // expert width 1408, 16 strips per workgroup: with two token tiles the operand takes 88 KiB of LDS, one
    // workgroup of 16 wavefronts per CU
    if (a.nt_loads) hipLaunchKernelGGL((gemm_wave_strip_kernel<ST, 11, 3, true, NTW, 16, 44, true>), dim3(grid), dim3(16 * 64), lds, s, a);
    else hipLaunchKernelGGL((gemm_wave_strip_kernel<ST, 11, 3, true, NTW, 16, 44, false>), dim3(grid), dim3(16 * 64), lds, s, a);
  } else if (nkb == 24) EVICT_WS_LAUNCH_NT(12, 3, 24);
  else if (nkb == 44 && NTW == 1) EVICT_WS_LAUNCH_NT(11, 6, 44);
  else if (nkb == 44) EVICT_WS_LAUNCH(11, 6 / NTW, true);
  else if (nkb % 16 == 0) EVICT_WS_LAUNCH_NT(16, 4 / NTW, 0);
  else if (nkb % 8 == 0) EVICT_WS_LAUNCH(8, 2 / NTW, true);
  else EVICT_WS_LAUNCH(16, 4 / NTW, false);
#undef EVICT_WS_LAUNCH
#undef EVICT_WS_LAUNCH_NT
  return launch_status("gemm_wave_strip_kernel");
}

// one gate/up strip pair per wavefront (see gemm_wave_gateup_kernel)
}  // namespace
int gateup_waves(const GemmArgs& a);
namespace {
bool wave_gateup_applies(const GemmArgs& a, int nt) {
  if (!(a.grouped && a.nkb % 8 == 0 && a.nkb <= 64 && (a.n_strips / 2) % gateup_waves(a) == 0)) return false;
  // two token tiles per slot: only the variant with 6 wavefronts and 64 contraction blocks is built
  return nt == 1 || (nt == 2 && a.nkb == 64 && gateup_waves(a) == 6);  // (gateup_waves: 4, 6 or 11)
}
template <typename ST>
int launch_gemm_wave_gateup(const GemmArgs& a, int nt, int grid, hipStream_t s) {
  const size_t lds = (size_t)a.nkb * 1024 * nt;
  const int ws = gateup_waves(a);
  const int nb = (a.nkb + ws - 1) / ws;
  if (ST::kBytes == 4 && (nb > 8 || nt == 2)) return -1;  // (those variants would spill: the caller falls back)
  if (nt == 2) {
    hipLaunchKernelGGL((gemm_wave_gateup_kernel<ST, 16, 16, 6, 64, 2>), dim3(grid), dim3(6 * 64), lds, s, a);
    return launch_status("gemm_wave_gateup_kernel");
  }
  if (a.lds_dma && a.nkb == 64 && ST::kBytes == 2) {
#define EVICT_GU_DMA(WS_)                                                                                                              \
    do {                                                                                                                               \
      if (a.nt_loads) hipLaunchKernelGGL((gemm_wave_gateup_kernel<ST, 16, 16, WS_, 64, 1, true, true>), dim3(grid), dim3(WS_ * 64), lds, s, a); \
      else hipLaunchKernelGGL((gemm_wave_gateup_kernel<ST, 16, 16, WS_, 64, 1, true, false>), dim3(grid), dim3(WS_ * 64), lds, s, a);           \
    } while (0)
    if (ws == 11) EVICT_GU_DMA(11);
    else if (ws == 6) EVICT_GU_DMA(6);
    else EVICT_GU_DMA(4);
#undef EVICT_GU_DMA
    return launch_status("gemm_wave_gateup_kernel");
  }
#define EVICT_GU_LAUNCH(WS_)                                                                                              \
  if (nb <= 4) hipLaunchKernelGGL((gemm_wave_gateup_kernel<ST, 8, 4, WS_>), dim3(grid), dim3(WS_ * 64), lds, s, a);        \
  else if (nb <= 8) hipLaunchKernelGGL((gemm_wave_gateup_kernel<ST, 8, 8, WS_>), dim3(grid), dim3(WS_ * 64), lds, s, a);   \
  else if (a.nkb == 64) hipLaunchKernelGGL((gemm_wave_gateup_kernel<ST, 16, 16, WS_, 64>), dim3(grid), dim3(WS_ * 64), lds, s, a); \
  else hipLaunchKernelGGL((gemm_wave_gateup_kernel<ST, 8, 16, WS_>), dim3(grid), dim3(WS_ * 64), lds, s, a)
  if (ws == 11) { EVICT_GU_LAUNCH(11); } else if (ws == 6) { EVICT_GU_LAUNCH(6); } else { EVICT_GU_LAUNCH(4); }
#undef EVICT_GU_LAUNCH
  return launch_status("gemm_wave_gateup_kernel");
}

bool wave_strip_applies(const GemmArgs& a, int nt) {
  if (!(a.grouped && a.n_strips % 8 == 0)) return false;
  // (the 16-strip variant for 44 contraction blocks is given 88 KiB of dynamic LDS in kernels_setup)
  return a.nkb * nt <= 64 || (a.nkb == 44 && nt == 2 && a.down_ws == 16 && a.n_strips % 16 == 0);
}

template <typename ST, int EPI>
int launch_gemm_st(const GemmArgs& a, int nt, int grid, hipStream_t s) {
  if (EPI == EPI_SWIGLU && a.wave_strip && wave_gateup_applies(a, nt)) {
    const int rc = launch_gemm_wave_gateup<ST>(a, nt, grid, s);
    if (rc >= 0) return rc;
  }
  if (EPI == EPI_F32 && a.wave_strip && wave_strip_applies(a, nt))
    return nt == 1 ? launch_gemm_wave_strip<ST, 1>(a, grid, s) : launch_gemm_wave_strip<ST, 2>(a, grid, s);
  return nt == 1 ? launch_gemm_nt<ST, 1, EPI>(a, grid, s) : launch_gemm_nt<ST, 2, EPI>(a, grid, s);
}

// dense projections, one strip per wavefront (see gemm_dense_strip_kernel). Every instantiation, once, for
// the launcher and for the LDS attribute.
#define EVICT_DENSE_STRIP_SHAPES(X, ST_, EPI_, NKB_) X(ST_, EPI_, 2, 8, NKB_) X(ST_, EPI_, 1, 8, NKB_)
#define EVICT_DENSE_STRIP_ALL(X)                                                                                   \
  EVICT_DENSE_STRIP_SHAPES(X, BF16, EPI_QKV, 0) EVICT_DENSE_STRIP_SHAPES(X, BF16, EPI_QKV, 64)                     \
  EVICT_DENSE_STRIP_SHAPES(X, BF16, EPI_QKV, 128) EVICT_DENSE_STRIP_SHAPES(X, BF16, EPI_RESID, 0)                  \
  EVICT_DENSE_STRIP_SHAPES(X, BF16, EPI_RESID, 64) EVICT_DENSE_STRIP_SHAPES(X, BF16, EPI_RESID, 128)               \
  EVICT_DENSE_STRIP_SHAPES(X, F32, EPI_QKV, 0) EVICT_DENSE_STRIP_SHAPES(X, F32, EPI_RESID, 0)
constexpr size_t kDenseStripLdsMax = 128 * 1024;

}  // namespace

// Strip pairs (wavefronts) per workgroup: 6 when that makes the chunks per slot a multiple of 8. Chunk ids go
// round-robin over the 8 XCDs, so the same unit of every slot then lands on the same XCD, and the second token
// tile of an expert finds the weights its first tile streamed in that XCD's L2 instead of fetching them again.
int gateup_waves(const GemmArgs& a) {
  const int pairs = a.n_strips / 2;
  if (pairs % 6 == 0 && (pairs / 6) % 8 == 0) return 6;
  // (88 strip pairs: expert width 1408; 11 wavefronts leave 170 VGPRs each, which only the variant without
  // staging registers fits)
  if (pairs % 11 == 0 && (pairs / 11) % 8 == 0 && a.lds_dma && a.nkb == 64) return 11;
  return 4;
}
bool dense_strip_applies(const GemmArgs& a, int ntw) {
  return !a.grouped && a.nkb % 16 == 0 && (size_t)ntw * a.nkb * 1024 <= kDenseStripLdsMax;
}

// ntw in {1, 2} token tiles per workgroup, 8 strips (wavefronts) per workgroup; the caller has checked
// dense_strip_applies(a, ntw). Sets a.dense_tiles itself.
int launch_gemm_dense_strip(int dtype, int epi, GemmArgs a, int ntw, hipStream_t s) {
  const int ws = 8;
  a.dense_tiles = (a.T + 16 * ntw - 1) / (16 * ntw);
  const int n_sg = (a.n_strips + ws - 1) / ws;
  const int grid = ((n_sg + 7) / 8) * 8 * a.dense_tiles;
  const size_t lds = (size_t)ntw * a.nkb * 1024;
  const int nkb_static = (dtype == EVICT_BF16 && (a.nkb == 64 || a.nkb == 128)) ? a.nkb : 0;
  bool launched = false;
#define EVICT_DS_TRY(ST_, EPI_, NTW_, WS_, NKB_)                                                                        \
  if (!launched && dtype == (sizeof(ST_::elem) == 2 ? EVICT_BF16 : EVICT_F32) && epi == EPI_ && ntw == NTW_ && ws == WS_ && \
      nkb_static == NKB_) {                                                                                             \
    hipLaunchKernelGGL((gemm_dense_strip_kernel<ST_, EPI_, NTW_, WS_, NKB_>), dim3(grid), dim3(WS_ * 64), lds, s, a);    \
    launched = true;                                                                                                    \
  }
  EVICT_DENSE_STRIP_ALL(EVICT_DS_TRY)
#undef EVICT_DS_TRY
  if (!launched) {
    set_error("gemm_dense_strip_kernel: no variant for dtype %d epilogue %d ntw %d ws %d", dtype, epi, ntw, ws);
    return EVICT_E_INVALID;
  }
  return launch_status("gemm_dense_strip_kernel");
}

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
    EVICT_GEMM_CASE(EPI_ARGMAX)
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
                int max_ctx, const void* x, const void* gain, int norm_only, hipStream_t s) {
  const evict_model_desc& m = c->m;
  if (m.dtype == EVICT_BF16)
    hipLaunchKernelGGL(prep_kernel<BF16>, dim3(T), dim3(256), 0, s, tree_off, parent, B, ctx_len, max_ctx, x, gain, m.d,
                       m.rms_eps, c->rope_rev, m.D, c->anc, c->depth, c->seq_of, c->rope_cs, c->x_norm, c->status, (B == 1 && !c->t_dev) ? T : 0, norm_only, c->t_dev);
  else
    hipLaunchKernelGGL(prep_kernel<F32>, dim3(T), dim3(256), 0, s, tree_off, parent, B, ctx_len, max_ctx, x, gain, m.d,
                       m.rms_eps, c->rope_rev, m.D, c->anc, c->depth, c->seq_of, c->rope_cs, c->x_norm, c->status, (B == 1 && !c->t_dev) ? T : 0, norm_only, c->t_dev);
  return launch_status("prep_kernel");
}

size_t attn_partial_lds_bytes(int D) { return sizeof(float) * (size_t)(2 * kAttnKeys * (D + 1) + 4 * D + 4 * 64); }
size_t attn_mfma_lds_bytes(int D) { return 2 * (size_t)(kMfmaKeys * (D + 16) + D * (kMfmaKeys + 4)); }
// strips of 16 experts per workgroup and contraction split of the score kernel: enough
// workgroups to spread W_g over the chip, 16 (strip, slice) items per workgroup
int router_strips_per_wg(const evict_model_desc& m) {
  const int nstrips = m.E / 16;
  return nstrips <= 16 ? 1 : (nstrips + 15) / 16;
}
int router_ksplit(const evict_model_desc& m) {
  int ks = kRouterWaves / router_strips_per_wg(m);
  const int nkb = m.d * (m.dtype == EVICT_BF16 ? 2 : 4) / 64;
  ks = ks > nkb ? nkb : ks;
  return ks < 1 ? 1 : ks;
}
size_t router_lds_bytes(const evict_model_desc& m) {
  const size_t eb = m.dtype == EVICT_BF16 ? 2 : 4;
  return (size_t)m.d * eb * 16 + (size_t)router_ksplit(m) * router_strips_per_wg(m) * 64 * sizeof(f32x4);
}
int union_mask_plan(int T, int k, int E, size_t* lds_bytes);  // small_kernels.hip

int kernels_setup(const evict_model_desc& m) {
  // kernels whose dynamic LDS exceeds the default 64 KiB limit
#define EVICT_DS_ATTR(ST_, EPI_, NTW_, WS_, NKB_)                                                            \
  EVICT_HIP_CHECK(hipFuncSetAttribute((const void*)gemm_dense_strip_kernel<ST_, EPI_, NTW_, WS_, NKB_>,      \
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)kDenseStripLdsMax));
  EVICT_DENSE_STRIP_ALL(EVICT_DS_ATTR)
#undef EVICT_DS_ATTR
  EVICT_HIP_CHECK(hipFuncSetAttribute((const void*)gemm_wave_gateup_kernel<BF16, 16, 16, 6, 64, 2>,
                                      hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 1024));
  EVICT_HIP_CHECK(hipFuncSetAttribute((const void*)attn_partial_kernel<BF16>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)attn_partial_lds_bytes(128)));
  EVICT_HIP_CHECK(hipFuncSetAttribute((const void*)attn_partial_kernel<F32>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)attn_partial_lds_bytes(128)));
  EVICT_HIP_CHECK(hipFuncSetAttribute((const void*)attn_partial_mfma_kernel<128, 4>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)attn_mfma_lds_bytes(128)));
  EVICT_HIP_CHECK(hipFuncSetAttribute((const void*)attn_partial_mfma_kernel<64, 4>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)attn_mfma_lds_bytes(64)));
  EVICT_HIP_CHECK(hipFuncSetAttribute((const void*)attn_partial_mfma_kernel<128, 8>, hipFuncAttributeMaxDynamicSharedMemorySize, 2 * (int)attn_mfma_lds_bytes(128)));
  EVICT_HIP_CHECK(hipFuncSetAttribute((const void*)attn_partial_mfma_kernel<64, 8>, hipFuncAttributeMaxDynamicSharedMemorySize, 2 * (int)attn_mfma_lds_bytes(64)));
  EVICT_HIP_CHECK(hipFuncSetAttribute((const void*)attn_partial_mfma_kernel<128, 4, true>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)attn_mfma_lds_bytes(128)));
  EVICT_HIP_CHECK(hipFuncSetAttribute((const void*)attn_partial_mfma_kernel<64, 4, true>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)attn_mfma_lds_bytes(64)));
  EVICT_HIP_CHECK(hipFuncSetAttribute((const void*)attn_partial_mfma_kernel<128, 8, true>, hipFuncAttributeMaxDynamicSharedMemorySize, 2 * (int)attn_mfma_lds_bytes(128)));
  EVICT_HIP_CHECK(hipFuncSetAttribute((const void*)attn_partial_mfma_kernel<64, 8, true>, hipFuncAttributeMaxDynamicSharedMemorySize, 2 * (int)attn_mfma_lds_bytes(64)));
  EVICT_HIP_CHECK(hipFuncSetAttribute((const void*)gemm_wave_strip_kernel<BF16, 11, 3, true, 2, 16, 44, true>, hipFuncAttributeMaxDynamicSharedMemorySize, 88 * 1024));
  EVICT_HIP_CHECK(hipFuncSetAttribute((const void*)gemm_wave_strip_kernel<BF16, 11, 3, true, 2, 16, 44, false>, hipFuncAttributeMaxDynamicSharedMemorySize, 88 * 1024));
  if (m.E > 256)  // LDS variant of TopK: one row of keys per wavefront
    EVICT_HIP_CHECK(hipFuncSetAttribute((const void*)topk_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                        (int)((size_t)kRouterWaves * (64 + m.E) * sizeof(float))));
  const size_t rl = router_lds_bytes(m);
  EVICT_REQUIRE(rl <= 152 * 1024, EVICT_E_UNSUPPORTED, "router needs %zu bytes of LDS (limit 152 KiB): d too large", rl);
  EVICT_REQUIRE(m.d <= 64 * 8 * (m.dtype == EVICT_BF16 ? 8 : 4), EVICT_E_UNSUPPORTED, "router keeps a token row in registers: d=%d too large", m.d);
  if (m.dtype == EVICT_BF16)
    EVICT_HIP_CHECK(hipFuncSetAttribute((const void*)router_logits_kernel<BF16>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)rl));
  else
    EVICT_HIP_CHECK(hipFuncSetAttribute((const void*)router_logits_kernel<F32>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)rl));
  return EVICT_OK;
}

int launch_attention(const evict_ctx* c, const void* kc, const void* vc, long long seq_stride, long long head_stride,
                     const int32_t* ctx_len, int max_ctx_host, const int32_t* tree_off, int B, int T, const void* k_new,
                     const void* v_new, void* aux_out, hipStream_t s) {
  const evict_model_desc& m = c->m;
  int ctx_splits, nsplits, keys;
  if (m.dtype == EVICT_BF16) {
    // one 16-row query tile per wavefront; enough context splits to cover the chip, each a whole
    // number of 128-key chunks (more chunks per split = fewer partial results to merge)
    const int G = m.Hq / m.Hkv;
    const int max_nodes = T < EVICT_MAX_TREE_NODES ? T : EVICT_MAX_TREE_NODES;
    const int ntiles = (max_nodes * G + 15) / 16;
    // (the host knows only T and B: row blocks are provisioned for the largest tree allowed, and
    // those past a sequence's own tiles leave at once; the split count goes by the average tree)
    const int avg_nodes = (T + B - 1) / B < max_nodes ? (T + B - 1) / B : max_nodes;
    const int avg_tiles = (avg_nodes * G + 15) / 16;
    const int chunks = (max_ctx_host + kMfmaKeys - 1) / kMfmaKeys;
    // 8-wavefront workgroups with two LDS buffers (the next chunk is fetched during the matrix work) once
    // there is more than one round of 4-wavefront workgroups to run. With fewer than 8 row tiles some of the
    // 8 wavefronts only stage; measured to pay down to 4 tiles (many KV heads, few rows per head).
    const long long chunk_wgs4 = (long long)chunks * m.Hkv * B * ((avg_tiles + 3) / 4);
    int nw = (avg_tiles >= 4 && chunk_wgs4 > c->attn_target_wgs) ? 8 : 4;
    if (c->attn_waves == 4 || c->attn_waves == 8) nw = c->attn_waves;
    const int rb = c->attn_row_blocks > 0 ? c->attn_row_blocks : (ntiles + nw - 1) / nw;
    const int rb_avg = (avg_tiles + nw - 1) / nw;
    // context splits: two workgroups of 4 wavefronts per CU overlap each other; one of 8 fills it. The
    // draft-node split of every unit comes on top, so one split of the budget is kept for it: a grid a
    // few workgroups above what the chip holds at once would run a nearly empty second round. (Not in a
    // batch: splits past a shorter sequence's context leave at once, so the grid is not what runs.)
    int want = (nw == 8 ? c->attn_target_wgs / 2 : c->attn_target_wgs) / (m.Hkv * B * rb_avg) - (B == 1 ? 1 : 0);
    want = want < 1 ? 1 : want;
    // (the merge walks the splits of a row in batches of 17, one round trip each: beyond about 32 splits a
    // second chunk per workgroup costs less than the extra batches; measured at 8 nodes, ctx 8192)
    want = want > 32 ? 32 : want;
    int cps = (chunks + want - 1) / want;  // chunks per split
    cps = cps < 1 ? 1 : cps;
    keys = cps * kMfmaKeys;
    ctx_splits = (max_ctx_host + keys - 1) / keys;
    nsplits = ctx_splits + 1;
    EVICT_REQUIRE(rb * nw >= ntiles, EVICT_E_INVALID, "attn_row_blocks=%d is too small for %d query tiles", rb, ntiles);
    EVICT_REQUIRE(nsplits <= c->max_splits, EVICT_E_INVALID, "attention: %d splits exceed the scratch of %d", nsplits, c->max_splits);
    const int units = nsplits * m.Hkv * B;
    const dim3 grid(((units + 7) / 8) * 8 * rb);
    const size_t lds = attn_mfma_lds_bytes(m.D) * (nw == 8 ? 2 : 1);
#define EVICT_ATTN_ARGS (const uint16_t*)c->q, (const uint16_t*)kc, (const uint16_t*)vc, seq_stride, head_stride, ctx_len, \
                        max_ctx_host, tree_off, (const uint16_t*)k_new, (const uint16_t*)v_new, c->anc, m.Hq, m.Hkv,       \
                        ctx_splits, keys, rb, T, c->part_o, c->part_ml, (B == 1 && !c->t_dev) ? T : 0, B, c->paging, c->status,   \
                        (B == 1 && c->t_dev) ? 1 : 0
#define EVICT_ATTN_LAUNCH(PAGED_)                                                                                              \
    if (m.D == 128 && nw == 4) hipLaunchKernelGGL((attn_partial_mfma_kernel<128, 4, PAGED_>), grid, dim3(256), lds, s, EVICT_ATTN_ARGS); \
    else if (m.D == 128) hipLaunchKernelGGL((attn_partial_mfma_kernel<128, 8, PAGED_>), grid, dim3(512), lds, s, EVICT_ATTN_ARGS);       \
    else if (nw == 4) hipLaunchKernelGGL((attn_partial_mfma_kernel<64, 4, PAGED_>), grid, dim3(256), lds, s, EVICT_ATTN_ARGS);           \
    else hipLaunchKernelGGL((attn_partial_mfma_kernel<64, 8, PAGED_>), grid, dim3(512), lds, s, EVICT_ATTN_ARGS)
    if (c->paging.table) { EVICT_ATTN_LAUNCH(true); } else { EVICT_ATTN_LAUNCH(false); }
#undef EVICT_ATTN_LAUNCH
#undef EVICT_ATTN_ARGS
  } else {
    keys = kAttnKeys;
    ctx_splits = (max_ctx_host + keys - 1) / keys;
    nsplits = ctx_splits + EVICT_MAX_TREE_NODES / keys;
    hipLaunchKernelGGL(attn_partial_kernel<F32>, dim3(nsplits, m.Hkv, B), dim3(256), attn_partial_lds_bytes(m.D), s, c->q,
                       kc, vc, seq_stride, head_stride, ctx_len, max_ctx_host, tree_off, k_new, v_new, c->anc, m.Hq,
                       m.Hkv, m.D, ctx_splits, T, c->part_o, c->part_ml, c->paging, c->status, (B == 1 && !c->t_dev) ? T : 0);
  }
  int rc = launch_status("attention partial kernel");
  if (rc) return rc;
  const int mrows = T * m.Hq;
  const int mthreads = (long long)mrows * (m.D / 4) >= 256 * 256 ? 256 : 64;  // at least ~256 workgroups, or one wavefront each
  const int rows_per_wg = mthreads / (m.D / 4);
  const dim3 mgrid((mrows + rows_per_wg - 1) / rows_per_wg);
  if (m.dtype == EVICT_BF16)
    hipLaunchKernelGGL(attn_merge_kernel<BF16>, mgrid, dim3(mthreads), 0, s, c->part_o, c->part_ml, nsplits, mrows, m.D,
                       c->attn_o, aux_out, m.Hq, c->t_dev);
  else
    hipLaunchKernelGGL(attn_merge_kernel<F32>, mgrid, dim3(mthreads), 0, s, c->part_o, c->part_ml, nsplits, mrows, m.D,
                       c->attn_o, aux_out, m.Hq, c->t_dev);
  return launch_status("attn_merge_kernel");
}

int attn_splits_for(int max_ctx) { return (max_ctx + kAttnKeys - 1) / kAttnKeys + EVICT_MAX_TREE_NODES / kAttnKeys; }

int launch_router(const evict_ctx* c, const void* gain, const void* wg, int T, const evict_layer_aux* aux, hipStream_t s) {
  const evict_model_desc& m = c->m;
  const size_t lds = router_lds_bytes(m);
  void* a_hn = aux ? aux->h_norm : nullptr;
  float* a_lg = aux ? aux->router_logits : nullptr;
  const int spw = router_strips_per_wg(m);
  const dim3 grid((T + 15) / 16, (m.E / 16 + spw - 1) / spw);
  if (m.dtype == EVICT_BF16)
    hipLaunchKernelGGL(router_logits_kernel<BF16>, grid, dim3(kRouterThreads), lds, s, c->h, gain, (const u32x4*)wg, T, m.d,
                       m.E, spw, router_ksplit(m), m.rms_eps, c->h_norm, c->logits, a_hn, a_lg, c->t_dev);
  else
    hipLaunchKernelGGL(router_logits_kernel<F32>, grid, dim3(kRouterThreads), lds, s, c->h, gain, (const u32x4*)wg, T, m.d,
                       m.E, spw, router_ksplit(m), m.rms_eps, c->h_norm, c->logits, a_hn, a_lg, c->t_dev);
  return launch_status("router_logits_kernel");
}

int launch_topk_union(const evict_ctx* c, int T, const evict_layer_aux* aux, int tile_tokens, hipStream_t s) {
  const evict_model_desc& m = c->m;
  int32_t* a_idx = aux ? aux->topk_idx : nullptr;
  float* a_w = aux ? aux->topk_w : nullptr;
  size_t lds;
  const int use_masks = union_mask_plan(T, m.k, m.E, &lds);
  const bool regs = m.E <= 256;
  if (regs && T <= kFusedTopkTokens) {
    hipLaunchKernelGGL(topk_union_kernel, dim3(1), dim3(kRouterThreads), lds, s, c->logits, T, m.E, m.k, m.router_norm, c->topk_idx,
                       c->topk_w, a_idx, a_w, use_masks, c->union_ids, c->union_count, c->hist, c->offsets, c->perm, c->inv,
                       c->status, c->work, c->tok_of_pos, c->sched, m.n_shared, tile_tokens, c->t_dev);
    return launch_status("topk_union_kernel");
  }
  const dim3 tgrid((T + kRouterWaves - 1) / kRouterWaves);
  if (regs) {
    hipLaunchKernelGGL(topk_regs_kernel, tgrid, dim3(kRouterThreads), 0, s, c->logits, T, m.E, m.k, m.router_norm, c->topk_idx, c->topk_w,
                       a_idx, a_w, c->t_dev);
  } else {
    const size_t lds_topk = (size_t)kRouterWaves * (64 + m.E) * sizeof(float);
    hipLaunchKernelGGL(topk_kernel, tgrid, dim3(kRouterThreads), lds_topk, s, c->logits, T, m.E, m.k, m.router_norm, c->topk_idx, c->topk_w,
                       a_idx, a_w, c->t_dev);
  }
  int rc = launch_status("topk_kernel");
  if (rc) return rc;
  hipLaunchKernelGGL(union_worklist_kernel, dim3(1), dim3(kRouterThreads), lds, s, c->topk_idx, T, m.k, m.E, use_masks,
                     c->union_ids, c->union_count, c->hist, c->offsets, c->perm, c->inv, c->status, c->work, c->tok_of_pos,
                     c->sched, m.n_shared, tile_tokens, c->t_dev);
  return launch_status("union_worklist_kernel");
}

int launch_argmax_reduce(const float* val, const int32_t* idx, int nstrips, int ld, int T, int32_t* next, float* best_out,
                         const int32_t* t_dev, hipStream_t s) {
  hipLaunchKernelGGL(argmax_reduce_kernel, dim3(T), dim3(256), 0, s, val, idx, nstrips, ld, next, best_out, t_dev);
  return launch_status("argmax_reduce_kernel");
}

int launch_combine(const evict_ctx* c, int T, void* out, const void* next_gain, hipStream_t s) {
  const evict_model_desc& m = c->m;
  if (m.dtype == EVICT_BF16)
    hipLaunchKernelGGL(combine_kernel<BF16>, dim3(T), dim3(256), 0, s, c->h, c->y, c->topk_w, c->inv, m.k, m.d,
                       m.n_shared, T, out, next_gain, m.rms_eps, c->x_norm, c->t_dev);
  else
    hipLaunchKernelGGL(combine_kernel<F32>, dim3(T), dim3(256), 0, s, c->h, c->y, c->topk_w, c->inv, m.k, m.d,
                       m.n_shared, T, out, next_gain, m.rms_eps, c->x_norm, c->t_dev);
  return launch_status("combine_kernel");
}

}  // namespace evict
