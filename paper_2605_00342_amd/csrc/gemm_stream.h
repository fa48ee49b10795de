// Weight-streaming skinny GEMM for gfx950: out[token][row] = sum_k W[row][k] * X[token][k]
// with at most a few dozen tokens per weight matrix, so the kernel is bound by reading W
// from HBM exactly once. Used for the QKV / output projections and for the grouped expert
// GEMMs over the union of activated experts (Sec. 2.2, Eq. 5).
//
// Layout: W is pre-packed into 16-row strips; a strip is nkb consecutive 1 KiB blocks, one
// block = one wavefront-wide 16-byte load = one MFMA operand (64 bytes of each of 16 rows).
// A workgroup of 8 wavefronts owns a contiguous range of strips (contiguous in memory, so
// the stream is sequential); the contraction range of a strip is split across the 8
// wavefronts, each keeping its slice of the token operand in registers for as long as the
// expert does not change. Partial tiles meet in LDS, one wavefront (rotating) sums them and
// runs the epilogue. The whole work list (union experts x strips) is cut into equal
// contiguous ranges on the device, so no host knowledge of the union size is needed.
#pragma once
#include <type_traits>

#include "device_utils.h"

namespace evict {

enum { EPI_QKV = 0, EPI_RESID = 1, EPI_SWIGLU = 2, EPI_F32 = 3, EPI_ARGMAX = 4 };

// One slot of the device-side work list = one activated expert and one tile of up to 16 of its
// tokens: the expert, where the tile sits in the grouped order, how many tokens it has, how many
// tiles the expert has, and the token ids of the tile's first positions (so that a workgroup
// learns everything it needs to start loading from one 64-byte record).
constexpr int kWorkToks = 12;
struct WorkRec {
  int expert, p0, ntok, pad;
  int tok[kWorkToks];
};

struct GemmArgs {
  const u32x4* W;        // packed weights
  const u32x4* W_shared; // grouped: packed weights of the always-on shared experts (expert ids >= n_routed)
  int n_routed;          // grouped: number of routed experts E
  long long group_stride;  // u32x4 elements between experts
  int n_strips;          // 16-row strips per matrix (gate/up interleaved: 2 per 16 rows of F)
  int nkb;               // 1 KiB blocks per strip
  const void* X;         // token operand rows, storage dtype
  long long ldx_bytes;   // bytes between rows of X
  int grouped;           // 0: one matrix, tokens 0..T-1; 1: one matrix per union expert
  const int* union_count;  // grouped: number of work slots (expert x token tile)
  const WorkRec* work;   // per union slot (see WorkRec)
  int chunk_units;       // grouped: units per chunk (divides the units per expert)
  const int* tok_of_pos; // token of each grouped position (perm[p] / k)
  int x_by_token;        // grouped: 1 -> X row = tok_of_pos[p], 0 -> X row = p
  int T;                 // dense: token rows (upper bound when T_dev is set)
  const int* T_dev;      // dense: nullptr, or device word holding the actual number of token rows (<= T)
  int dense_tiles;       // dense: workgroups per strip, each taking 16*NT tokens
  int dense_units;       // dense: consecutive strips a workgroup takes (its weight loads run ahead across them)
  int prefetch;          // host-side choice of the kernel variant: 3 = no compile-time step counts (measurement knob)
  int wave_strip;        // host-side: grouped fp32-output GEMM may use gemm_wave_strip_kernel
  int nt_loads;          // host-side choice of the kernel variant: 1 = weights fetched with non-temporal loads
  int lds_dma;           // 1: strip-pair gate/up kernel stages its token operand with direct global-to-LDS loads
  int down_ws;           // gemm_wave_strip_kernel: strips (wavefronts) per workgroup, 8 or 16
  int pair_tiles;        // 1: gemm_wave_strip_kernel with two token tiles takes them from two consecutive 16-token records
  void* out0;            // QKV: q; RESID: h; SWIGLU: act; F32: y; ARGMAX: best value per (token, strip), [T][ldo]
  void* out1;            // QKV: k_new; ARGMAX: row index of the best value per (strip, token)
  void* out2;            // QKV: v_new
  long long ldo;         // elements between output rows (RESID / SWIGLU / F32)
  const void* resid;     // RESID: residual rows, same layout as out0
  const float* rope_cs;  // QKV: [T][D] cos | sin
  int Hq, Hkv, D;
};

constexpr int kGemmWaves = 8;
constexpr int kGemmThreads = kGemmWaves * 64;

// KBW: 1 KiB blocks a wavefront takes per step (EXACT: every step has exactly KBW, no masking);
// PF: steps of weight loads kept in flight; NT: 16-token tiles held in registers; IS: strips
// taken per step (one partial-tile exchange per IS strips).
// NS > 0: steps per segment known at compile time (the step loop is unrolled, so the rolling refill of
// the weight registers is unconditional and every wait is by exact queue position).
// NTL: weights are fetched with non-temporal loads (read once, or by the neighbouring token tile at about the
// same time: kept out of the caches' way). Ordinary loads stream about 15 % slower here and leave L2 and the
// memory-side cache full of weights nobody reads again, which slows the kernels that follow (measured). This is
// a compile-time choice on purpose: a run-time choice per load between a non-temporal and an ordinary load of
// the same address is folded by the compiler into one ordinary load. (Measured too: ordinary loads for all but
// the last token tile of an expert, so that later tiles find the weights in L2, lose more in the following
// kernels than they save in this one.)
template <typename ST, int NT, int KBW, int PF, int EPI, bool EXACT, int IS = 1, int NS = 0, bool NTL = false>
__global__ __launch_bounds__(kGemmThreads) __attribute__((amdgpu_waves_per_eu(NT == 1 ? 4 : 2))) void gemm_stream_kernel(const GemmArgs a) {
  constexpr int SPU = (EPI == EPI_SWIGLU) ? 2 : 1;  // strips per unit of work
  static_assert(EPI != EPI_SWIGLU || IS == 1, "gate/up strips are exchanged one at a time");
  __shared__ f32x4 s_part[2][kGemmWaves][IS * NT][64];

  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);  // wavefront index, known uniform
  const int upg = a.n_strips / SPU;
  const int nkb = a.nkb;
  const int nchunks = (nkb + 63) >> 6;
  int parity = 0;

  // One segment = `nunits` consecutive units (strips, or gate/up strip pairs) of one weight
  // matrix, applied to the tokens [tok_begin, min(ntok, tok_limit)) of its group.
  auto run_segment = [&](auto nt_tag, int grp, int unit_in_grp, int nunits, int tok_begin, int tok_limit) {
    constexpr bool once = decltype(nt_tag)::value;
    const int strip0 = unit_in_grp * SPU;
    const int nitems = nunits * SPU;
    int p0 = 0, ntok = a.grouped ? 0 : dyn_tokens(a.T_dev, a.T);
    int tok_early = 0;  // token id from the work record (grouped, first kWorkToks positions)
    const u32x4* wbase = a.W;
    if (a.grouped) {
      // one hop: the record (scalar) and this lane's token id (vector) are fetched together
      const WorkRec* rec = a.work + grp;
      const int lc = lane & 15;
      tok_early = rec->tok[lc < kWorkToks ? lc : kWorkToks - 1];  // entries past ntok repeat the last token
      p0 = rec->p0;
      ntok = rec->ntok;
      const int ex = rec->expert;
      wbase = ex < a.n_routed ? a.W + (long long)ex * a.group_stride : a.W_shared + (long long)(ex - a.n_routed) * a.group_stride;
    }
    const int nsteps = NS > 0 ? NS : (nitems / IS) * nchunks;  // nitems is a multiple of IS (host-checked)

    const int tok_end = ntok < tok_limit ? ntok : tok_limit;
    for (int tok0 = tok_begin; tok0 < tok_end; tok0 += 16 * NT) {
      u32x4 A[PF][IS * KBW];
      u32x4 Bf[NT][KBW];
      f32x4 acc[IS][NT];
      f32x4 gate[NT];
      f32x4 pre0[IS * NT], pre1[IS * NT];  // epilogue operands requested ahead (QKV / RESID)
#pragma unroll
      for (int q = 0; q < IS * NT; ++q) pre0[q] = pre1[q] = f32x4{0, 0, 0, 0};
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        gate[t] = f32x4{0, 0, 0, 0};
#pragma unroll
        for (int i = 0; i < IS; ++i) acc[i][t] = f32x4{0, 0, 0, 0};
      }

      // block range of this wavefront inside chunk c: [b0, b0 + nb)
      auto range = [&](int c, int& b0, int& nb) {
        if (EXACT) {
          b0 = c * 64 + w * KBW;
          nb = KBW;
        } else {
          int cb = nkb - c * 64;
          cb = cb > 64 ? 64 : cb;
          b0 = c * 64 + (w * cb) / kGemmWaves;
          nb = c * 64 + ((w + 1) * cb) / kGemmWaves - b0;
        }
      };
      auto issue = [&](u32x4(&dst)[IS * KBW], int step) {
        const int it = step / nchunks, c = step - it * nchunks;
        int b0, nb;
        range(c, b0, nb);
#pragma unroll
        for (int i = 0; i < IS; ++i) {
          const u32x4* p = wbase + ((long long)(strip0 + it * IS + i) * nkb + b0) * 64 + lane;
#pragma unroll
          for (int j = 0; j < KBW; ++j)
            if (EXACT || j < nb) dst[i * KBW + j] = once ? __builtin_nontemporal_load(p + j * 64) : p[j * 64];
        }
      };
      // weights first: their addresses need nothing but the expert id
#pragma unroll
      for (int r = 0; r < PF; ++r)
        if (r < nsteps) issue(A[r], r);

      // token operand rows of this lane's column in each tile
      const char* xrow[NT];
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        int col = tok0 + t * 16 + (lane & 15);
        if (col > ntok - 1) col = ntok - 1;  // padded columns repeat the last token; never stored
        long long row = col;
        if (a.grouped) {
          if (!a.x_by_token) row = p0 + col;
          else row = (t == 0 && tok0 == 0 && (lane & 15) < kWorkToks) ? tok_early : a.tok_of_pos[p0 + col];
        }
        xrow[t] = (const char*)a.X + row * a.ldx_bytes + (lane >> 4) * 16;
      }
      auto load_b = [&](int c) {
        int b0, nb;
        range(c, b0, nb);
#pragma unroll
        for (int t = 0; t < NT; ++t) {
          const char* bp = xrow[t] + (long long)b0 * 64;  // one base per tile, constant offsets below
#pragma unroll
          for (int j = 0; j < KBW; ++j)
            if (EXACT || j < nb) Bf[t][j] = *reinterpret_cast<const u32x4*>(bp + j * 64);
        }
      };
      if (nchunks == 1) load_b(0);

#pragma unroll
      for (int s0 = 0; s0 < (NS > 0 ? NS : nsteps); s0 += PF) {
#pragma unroll
        for (int r = 0; r < PF; ++r) {
          const int step = s0 + r;
          if (step < nsteps) {
            const int it = step / nchunks, c = step - it * nchunks;
            if (nchunks > 1) load_b(c);
            if ((EPI == EPI_QKV || EPI == EPI_RESID) && c == 0) {
              // the wavefront that will reduce this strip requests what its epilogue needs (rotation
              // table entries, residual values) now, so that round trip hides behind the weight stream
              const int rb0 = unit_in_grp + it / SPU;
#pragma unroll
              for (int q = 0; q < IS * NT; ++q) {
                if (w == ((rb0 + q) & (kGemmWaves - 1))) {
                  const int t = q % NT;
                  const int strip = strip0 + it * IS + q / NT;
                  const int col = tok0 + t * 16 + (lane & 15);
                  const int tokc = col < ntok ? col : 0;
                  if (EPI == EPI_RESID) {
                    pre0[q] = load4<ST>(a.resid, (long long)tokc * a.ldo + strip * 16 + (lane >> 4) * 4);
                  } else {
                    const int spd = a.D >> 4;
                    const int head = strip / spd, js = strip - head * spd;
                    const int idx = js * 8 + ((lane >> 4) & 1) * 4;
                    const float* cs = a.rope_cs + (long long)tokc * a.D;
                    pre0[q] = *reinterpret_cast<const f32x4*>(cs + idx);
                    pre1[q] = *reinterpret_cast<const f32x4*>(cs + (a.D >> 1) + idx);
                  }
                }
              }
            }
            int b0, nb;
            range(c, b0, nb);
            if (EXACT && PF == 1 && NS > 0) {
              // rolling refill: the block of the next step goes into a register as soon as the MFMA has
              // consumed it, so about KBW loads stay in flight instead of falling to none at the end of
              // a step (same registers; the queue position of every load stays known at compile time)
              const bool more = step + 1 < nsteps;
              const int itn = (step + 1) / nchunks, cn = (step + 1) - itn * nchunks;
              const long long boff = (long long)(cn * 64 + w * KBW);
#pragma unroll
              for (int i = 0; i < IS; ++i) {
                const u32x4* pn = wbase + ((long long)(strip0 + itn * IS + i) * nkb + boff) * 64 + lane;
#pragma unroll
                for (int j = 0; j < KBW; ++j) {
#pragma unroll
                  for (int t = 0; t < NT; ++t) acc[i][t] = mfma_block<ST>(A[r][i * KBW + j], Bf[t][j], acc[i][t]);
                  if (more) A[r][i * KBW + j] = once ? __builtin_nontemporal_load(pn + j * 64) : pn[j * 64];
                  __builtin_amdgcn_sched_barrier(0);  // the refill stays right behind its MFMA
                }
              }
            } else {
#pragma unroll
              for (int i = 0; i < IS; ++i)
#pragma unroll
                for (int j = 0; j < KBW; ++j)
                  if (EXACT || j < nb) {
#pragma unroll
                    for (int t = 0; t < NT; ++t) acc[i][t] = mfma_block<ST>(A[r][i * KBW + j], Bf[t][j], acc[i][t]);
                  }
              if (step + PF < nsteps) issue(A[r], step + PF);
            }
            if (c == nchunks - 1) {
              // strip finished: exchange partial tiles, one wavefront reduces and stores
#pragma unroll
              for (int i = 0; i < IS; ++i)
#pragma unroll
                for (int t = 0; t < NT; ++t) {
                  s_part[parity][w][i * NT + t][lane] = acc[i][t];
                  acc[i][t] = f32x4{0, 0, 0, 0};
                }
              lds_barrier();
              // tile q = (strip i of the step, token tile t) is summed by wavefront (rbase + q) % 8
              const int rbase = unit_in_grp + it / SPU;
#pragma unroll
              for (int q = 0; q < IS * NT; ++q) {
                if (w == ((rbase + q) & (kGemmWaves - 1))) {
                  const int t = q % NT;
                  const int strip = strip0 + it * IS + q / NT;
                  f32x4 sum = s_part[parity][0][q][lane];
#pragma unroll
                  for (int ww = 1; ww < kGemmWaves; ++ww) sum += s_part[parity][ww][q][lane];
                  const int col = tok0 + t * 16 + (lane & 15);
                  const bool valid = col < ntok;
                  const int m0 = (lane >> 4) * 4;  // first of this lane's 4 rows in the strip
                  if (EPI == EPI_ARGMAX) {
                    // best of this lane's 4 rows (lowest row on equal values), then across the 4
                    // lanes that hold the other rows of the same token
                    float bv = sum[0];
                    int bi = strip * 16 + m0;
#pragma unroll
                    for (int i = 1; i < 4; ++i)
                      if (sum[i] > bv) { bv = sum[i]; bi = strip * 16 + m0 + i; }
#pragma unroll
                    for (int o = 16; o <= 32; o <<= 1) {
                      const float ov = __shfl_xor(bv, o);
                      const int oi = __shfl_xor(bi, o);
                      if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
                    }
                    if (valid && lane < 16) {
                      ((float*)a.out0)[(long long)col * a.ldo + strip] = bv;
                      ((int*)a.out1)[(long long)col * a.ldo + strip] = bi;
                    }
                  } else if (EPI == EPI_F32) {
                    if (valid) {
                      const long long orow = a.grouped ? (p0 + col) : col;
                      *reinterpret_cast<f32x4*>((float*)a.out0 + orow * a.ldo + strip * 16 + m0) = sum;
                    }
                  } else if (EPI == EPI_RESID) {
                    if (valid) {
                      const long long o = (long long)col * a.ldo + strip * 16 + m0;
                      store4<ST>(a.out0, o, pre0[q] + sum);
                    }
                  } else if (EPI == EPI_SWIGLU) {
                    if ((it & 1) == 0) {
                      gate[t] = sum;  // gate strip; its up strip is the next item
                    } else if (valid) {
                      f32x4 g = gate[t], r4;
#pragma unroll
                      for (int i = 0; i < 4; ++i) r4[i] = (g[i] / (1.0f + __expf(-g[i]))) * sum[i];
                      const long long orow = a.grouped ? (p0 + col) : col;
                      store4<ST>(a.out0, orow * a.ldo + (strip >> 1) * 16 + m0, r4);
                    }
                  } else {  // EPI_QKV: rotate pairs (i, i + D/2), which sit 32 lanes apart
                    const int spd = a.D >> 4;  // strips per head
                    const int head = strip / spd, js = strip - head * spd;
                    const int half = a.D >> 1;
                    const int g4 = lane >> 4;
                    const int idx = js * 8 + (g4 & 1) * 4;  // index inside the half
                    f32x4 other, r4;
#pragma unroll
                    for (int i = 0; i < 4; ++i) other[i] = __shfl_xor(sum[i], 32);
                    const bool rot = head < a.Hq + a.Hkv;
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                      const float cv = rot ? pre0[q][i] : 1.0f;
                      const float sv = rot ? pre1[q][i] : 0.0f;
                      r4[i] = (g4 < 2) ? (sum[i] * cv - other[i] * sv) : (sum[i] * cv + other[i] * sv);
                    }
                    if (valid) {
                      const int hrow = (g4 < 2 ? 0 : half) + idx;
                      if (head < a.Hq) {
                        store4<ST>(a.out0, ((long long)col * a.Hq + head) * a.D + hrow, r4);
                      } else if (head < a.Hq + a.Hkv) {
                        store4<ST>(a.out1, ((long long)col * a.Hkv + (head - a.Hq)) * a.D + hrow, r4);
                      } else {
                        store4<ST>(a.out2, ((long long)col * a.Hkv + (head - a.Hq - a.Hkv)) * a.D + hrow, r4);
                      }
                    }
                  }
                }
              }
              parity ^= 1;
            }
          }
        }
      }
    }
  };

  if (a.grouped) {
    // Device-side work list: union experts x units, cut into chunks of `chunk_units` units that
    // never straddle an expert. Chunks are dealt round-robin to the workgroups; all chunks cost
    // the same, so this stays balanced for any union size without the host knowing it.
    const int cpg = upg / a.chunk_units;
    const int total = *a.union_count * cpg;
    for (int chunk = blockIdx.x; chunk < total; chunk += gridDim.x) {
      // (the token tiles of one expert are consecutive slots: with cpg a multiple of 8 their
      // chunks land on the same XCD, whose L2 serves the second reader of the weights)
      const int slot = chunk / cpg, uc = chunk - slot * cpg;
      run_segment(std::integral_constant<bool, NTL>{}, slot, uc * a.chunk_units, a.chunk_units, 0, 0x7fffffff);
    }
  } else {
    // one workgroup per (strip, token tile). Workgroup ids go round-robin over the 8 XCDs, so
    // the tiles of one strip are given ids 8 apart: they share an L2 and read the strip from
    // HBM once.
    const unsigned xcd = blockIdx.x & 7u, i = blockIdx.x >> 3;
    const unsigned tile = i % (unsigned)a.dense_tiles;
    const unsigned du = a.dense_units > 0 ? (unsigned)a.dense_units : 1u;
    const unsigned unit = ((i / (unsigned)a.dense_tiles) * 8u + xcd) * du;
    if (unit >= (unsigned)upg) return;
    const unsigned nu = unit + du <= (unsigned)upg ? du : (unsigned)upg - unit;
    run_segment(std::integral_constant<bool, NTL>{}, 0, (int)unit, (int)nu, (int)tile * 16 * NT, (int)(tile + 1) * 16 * NT);
  }
}

// ------------------------------------------------------------------------------------
// Second decomposition for grouped GEMMs with many strips and a short contraction (the down
// projections: d/16 strips of F columns per expert): one strip per wavefront over the whole
// contraction range, so no partial tiles are exchanged and nothing synchronises the wavefronts
// after the token operand has been staged. The 16 x K token operand of the slot sits in LDS as
// ready-made MFMA operand blocks; weight blocks travel through a rolling window of WIN
// registers per lane (WIN KiB in flight per wavefront); NB operand blocks are staged per wavefront and
// pass. A workgroup takes WS consecutive strips
// of one slot (chunk); chunks are dealt round-robin like in gemm_stream_kernel.
// Output: fp32 rows y[p0 + column][strip * 16 + ...] (the EPI_F32 contract). NTW token tiles of 16
// per slot (the work list is built with tiles of 16 * NTW tokens).
// LDS: NTW * nkb KiB (dynamic).
// ------------------------------------------------------------------------------------
// NKB > 0 fixes the number of contraction blocks at compile time: every loop between the issue of
// a weight load and its use is then fully unrolled, which is what lets the compiler wait for a
// load by its exact position in the in-order queue (with run-time trip counts it has to drain the
// queue before the first MFMA, and the window stops rolling).
template <typename ST, int WIN, int NB, bool EXACT, int NTW = 1, int WS = 8, int NKB = 0, bool NTL = false>
__global__ __launch_bounds__(WS * 64) __attribute__((amdgpu_waves_per_eu(4))) void gemm_wave_strip_kernel(const GemmArgs a) {
  extern __shared__ __attribute__((aligned(16))) u32x4 s_b[];  // [NTW token tiles][nkb][64]
  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int nkb = NKB > 0 ? NKB : a.nkb;
  const int cpg = a.n_strips / WS;  // chunks per slot (host-checked: divides)
  const int total = *a.union_count * cpg;
  bool first = true;
  // one chunk; nt_tag: non-temporal weight loads (see gemm_stream_kernel)
  auto run_chunk = [&](auto nt_tag, int chunk) {
    constexpr bool once = decltype(nt_tag)::value;
    const int slot = chunk / cpg, strip = (chunk - slot * cpg) * WS + w;
    const WorkRec* rec = a.work + slot;
    const int p0 = rec->p0, ex = rec->expert;
    int ntok = rec->ntok;
    if (NTW == 2 && a.pair_tiles) {
      // The work list holds 16-token tiles; the tiles of an expert are consecutive records over consecutive
      // positions. An even tile takes its successor along (one weight stream for both), an odd one is done.
      const int ntile = rec->pad & 0xFFFF, ti = rec->pad >> 16;
      if (ti & 1) return;
      if (ti + 1 < ntile) ntok += rec[1].ntok;
    }
    const u32x4* wbase = ex < a.n_routed ? a.W + (long long)ex * a.group_stride
                                         : a.W_shared + (long long)(ex - a.n_routed) * a.group_stride;
    // token operand first, weights behind it: the in-order load counter then lets the operand
    // be consumed while the weight window is still in flight
    const char* xrow[NTW];
    bool valid[NTW];
#pragma unroll
    for (int t = 0; t < NTW; ++t) {
      int col = t * 16 + (lane & 15);
      valid[t] = col < ntok;
      col = valid[t] ? col : ntok - 1;  // padded columns repeat the last token; never stored
      const long long xr = a.x_by_token ? a.tok_of_pos[p0 + col] : p0 + col;
      xrow[t] = (const char*)a.X + xr * a.ldx_bytes + (lane >> 4) * 16;
    }
    constexpr int BMAX = NB;  // operand blocks a wavefront stages per pass and token tile
    const u32x4* wp = wbase + (long long)strip * nkb * 64 + lane;
    u32x4 A[WIN];
#pragma unroll
    for (int kb0 = 0; kb0 < (NKB > 0 ? NKB : nkb); kb0 += BMAX * WS) {
      u32x4 bst[NTW][BMAX];
#pragma unroll
      for (int t = 0; t < NTW; ++t)
#pragma unroll
        for (int i = 0; i < BMAX; ++i) {
          const int kb = kb0 + i * WS + w;
          if (kb < nkb && t * 16 < ntok) bst[t][i] = *reinterpret_cast<const u32x4*>(xrow[t] + (long long)kb * 64);
        }
      if (kb0 == 0) {
#pragma unroll
        for (int j = 0; j < WIN; ++j)
          if (EXACT || j < nkb) A[j] = once ? __builtin_nontemporal_load(wp + j * 64) : wp[j * 64];
        if (!first) lds_barrier();  // every wavefront is done with the previous chunk's operand
      }
#pragma unroll
      for (int t = 0; t < NTW; ++t)
#pragma unroll
        for (int i = 0; i < BMAX; ++i) {
          const int kb = kb0 + i * WS + w;
          if (kb < nkb && t * 16 < ntok) s_b[((size_t)t * nkb + kb) * 64 + lane] = bst[t][i];
        }
    }
    lds_barrier();
    first = false;
    f32x4 acc[NTW];
#pragma unroll
    for (int t = 0; t < NTW; ++t) acc[t] = f32x4{0, 0, 0, 0};
#pragma unroll
    for (int j0 = 0; j0 < (NKB > 0 ? NKB : nkb); j0 += WIN) {
#pragma unroll
      for (int jj = 0; jj < WIN; ++jj) {
        const int j = j0 + jj;
        if (EXACT || j < nkb) {
#pragma unroll
          for (int t = 0; t < NTW; ++t)
            if (t == 0 || ntok > 16) acc[t] = mfma_block<ST>(A[jj], s_b[((size_t)t * nkb + j) * 64 + lane], acc[t]);
          if (j + WIN < nkb) A[jj] = once ? __builtin_nontemporal_load(wp + (j + WIN) * 64) : wp[(j + WIN) * 64];
          if (NKB > 0) __builtin_amdgcn_sched_barrier(0);  // keep the refill right behind its MFMA: the window stays full
        }
      }
    }
#pragma unroll
    for (int t = 0; t < NTW; ++t)
      if (valid[t])
        *reinterpret_cast<f32x4*>((float*)a.out0 + (p0 + t * 16 + (lane & 15)) * a.ldo + strip * 16 + (lane >> 4) * 4) = acc[t];
  };
  for (int chunk = blockIdx.x; chunk < total; chunk += gridDim.x) run_chunk(std::integral_constant<bool, NTL>{}, chunk);
}

// ------------------------------------------------------------------------------------
// The same decomposition for the gate/up projections: one (gate strip, up strip) pair per
// wavefront over the whole contraction range (2 x nkb KiB of weights per wavefront and unit),
// the 16 x d token operand of the slot in LDS, two rolling windows of WIN weight blocks (one per
// strip; a token operand block read from LDS feeds both MFMAs), SiLU(g) * u applied in the
// wavefront that owns the pair. WS wavefronts per workgroup share the staged operand; a
// workgroup lives for WS * 2 * nkb KiB of weights, so the stream has no exchange points.
// Requires nkb % WIN == 0, (n_strips / 2) % WS == 0, NTW * nkb KiB of LDS (NTW tiles of 16 tokens per
// work-list slot). Refills go out in runs of 8
// consecutive blocks per strip once the window is 16 deep.
// ------------------------------------------------------------------------------------
template <typename ST, int WIN, int NB, int WS, int NKB = 0, int NTW = 1, bool DMA = false, bool NTL = false>
__global__ __launch_bounds__(WS * 64) __attribute__((amdgpu_waves_per_eu(2))) void gemm_wave_gateup_kernel(const GemmArgs a) {
  static_assert(!DMA || (NTW == 1 && 2 * WIN <= 48), "direct-to-LDS staging: one token tile, window loads countable in vmcnt");
  extern __shared__ __attribute__((aligned(16))) u32x4 s_b[];  // [NTW token tiles][nkb][64]
  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int nkb = NKB > 0 ? NKB : a.nkb;
  const int cpg = (a.n_strips >> 1) / WS;  // chunks per slot
  const int total = *a.union_count * cpg;
  bool first = true;
  // one chunk; nt_tag: non-temporal weight loads (see gemm_stream_kernel)
  auto run_chunk = [&](auto nt_tag, int chunk) {
    constexpr bool once = decltype(nt_tag)::value;
    const int slot = chunk / cpg, unit = (chunk - slot * cpg) * WS + w;
    const WorkRec* rec = a.work + slot;
    const int lc = lane & 15;
    const int tok_early = rec->tok[lc < kWorkToks ? lc : kWorkToks - 1];
    const int p0 = rec->p0, ntok = rec->ntok, ex = rec->expert;
    const u32x4* wbase = ex < a.n_routed ? a.W + (long long)ex * a.group_stride
                                         : a.W_shared + (long long)(ex - a.n_routed) * a.group_stride;
    // (NTW token tiles of 16 per slot: the work list was built with tiles of 16 * NTW tokens)
    bool valid[NTW];
    const char* xrow[NTW];
#pragma unroll
    for (int t = 0; t < NTW; ++t) {
      int col = t * 16 + lc;
      valid[t] = col < ntok;
      col = valid[t] ? col : ntok - 1;  // padded columns repeat the last token; never stored
      long long xr = p0 + col;
      if (a.x_by_token) xr = (t == 0 && col < kWorkToks) ? tok_early : a.tok_of_pos[p0 + col];
      xrow[t] = (const char*)a.X + xr * a.ldx_bytes + (lane >> 4) * 16;
    }
    // token operand blocks of the first tile first, weights behind them (the in-order load counter lets
    // the operand be consumed while the weight windows are still in flight); a second tile reuses the
    // staging registers once the first is in LDS. DMA: the operand blocks go from global memory straight
    // into LDS (16 bytes per lane, a block = 1 KiB contiguous = exactly the LDS layout), no staging registers.
    u32x4 bst[DMA ? 1 : NB];
    if (DMA) {
      if (!first) lds_barrier();  // every wavefront is done with the previous chunk's operand
#pragma unroll
      for (int i = 0; i < NB; ++i) {
        const int kb = i * WS + w;
        if (kb < nkb)
          __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1)))*)(xrow[0] + (long long)kb * 64),
                                           (void __attribute__((address_space(3)))*)(s_b + (size_t)kb * 64), 16, 0, 0);
      }
    }
    if constexpr (!DMA) {
#pragma unroll
      for (int i = 0; i < NB; ++i) {
        const int kb = i * WS + w;
        if (kb < nkb) bst[i] = *reinterpret_cast<const u32x4*>(xrow[0] + (long long)kb * 64);
      }
    }
    const u32x4* wg = wbase + (long long)(2 * unit) * nkb * 64 + lane;
    const u32x4* wu = wg + (long long)nkb * 64;
    u32x4 Ag[WIN], Au[WIN];
#pragma unroll
    for (int j = 0; j < WIN; ++j) {
      Ag[j] = once ? __builtin_nontemporal_load(wg + j * 64) : wg[j * 64];
      Au[j] = once ? __builtin_nontemporal_load(wu + j * 64) : wu[j * 64];
    }
    if (DMA) {
      // the operand blocks were requested before the 2 * WIN window loads: wait until only those are outstanding
      constexpr int kVm = 2 * WIN;
      __builtin_amdgcn_s_waitcnt((kVm & 0xF) | ((kVm >> 4) << 14) | (0x7 << 4) | (0xF << 8));
    } else if (!first) {
      lds_barrier();  // every wavefront is done with the previous chunk's operand
    }
    if constexpr (!DMA) {
#pragma unroll
      for (int t = 0; t < NTW; ++t) {
        if (t > 0) {
#pragma unroll
          for (int i = 0; i < NB; ++i) {
            const int kb = i * WS + w;
            if (kb < nkb) bst[i] = *reinterpret_cast<const u32x4*>(xrow[t] + (long long)kb * 64);
          }
        }
#pragma unroll
        for (int i = 0; i < NB; ++i) {
          const int kb = i * WS + w;
          if (kb < nkb) s_b[((size_t)t * nkb + kb) * 64 + lane] = bst[i];
        }
      }
    }
    lds_barrier();
    first = false;
    f32x4 accg[NTW], accu[NTW];
#pragma unroll
    for (int t = 0; t < NTW; ++t) accg[t] = accu[t] = f32x4{0, 0, 0, 0};
    constexpr int BURST = WIN >= 16 ? 8 : WIN;  // consecutive blocks requested together (DRAM likes runs)
#pragma unroll
    for (int j0 = 0; j0 < (NKB > 0 ? NKB : nkb); j0 += WIN) {
#pragma unroll
      for (int jj = 0; jj < WIN; ++jj) {
        const int j = j0 + jj;
#pragma unroll
        for (int t = 0; t < NTW; ++t) {
          const u32x4 bf = s_b[((size_t)t * nkb + j) * 64 + lane];
          accg[t] = mfma_block<ST>(Ag[jj], bf, accg[t]);
          accu[t] = mfma_block<ST>(Au[jj], bf, accu[t]);
        }
        if ((jj % BURST) == BURST - 1) {
          // the BURST window entries just consumed are refilled with the blocks WIN further on
          const int r0 = jj - (BURST - 1);
          if (j0 + r0 + WIN < nkb) {
#pragma unroll
            for (int r = 0; r < BURST; ++r)
              Ag[r0 + r] = once ? __builtin_nontemporal_load(wg + (j0 + r0 + r + WIN) * 64) : wg[(j0 + r0 + r + WIN) * 64];
#pragma unroll
            for (int r = 0; r < BURST; ++r)
              Au[r0 + r] = once ? __builtin_nontemporal_load(wu + (j0 + r0 + r + WIN) * 64) : wu[(j0 + r0 + r + WIN) * 64];
          }
          if (NKB > 0) __builtin_amdgcn_sched_barrier(0);  // keep the refills where they are: the windows stay full
        }
      }
    }
#pragma unroll
    for (int t = 0; t < NTW; ++t)
      if (valid[t]) {
        f32x4 r4;
#pragma unroll
        for (int i = 0; i < 4; ++i) r4[i] = (accg[t][i] / (1.0f + __expf(-accg[t][i]))) * accu[t][i];
        store4<ST>(a.out0, (long long)(p0 + t * 16 + lc) * a.ldo + unit * 16 + (lane >> 4) * 4, r4);
      }
  };
  for (int chunk = blockIdx.x; chunk < total; chunk += gridDim.x) run_chunk(std::integral_constant<bool, NTL>{}, chunk);
}

// ------------------------------------------------------------------------------------
// Dense projections with many tokens (QKV, output projection once the call has more than a few
// token tiles): the strip-per-wavefront decomposition of gemm_wave_strip_kernel applied to one
// weight matrix and all T tokens. A workgroup takes WS = 8 consecutive strips (one per wavefront,
// whole contraction range, rolling window of WIN weight blocks per lane) and NTW tiles of 16
// tokens, whose operand blocks it stages in LDS once ([NTW][nkb][64], NTW * nkb KiB); nothing
// is exchanged between wavefronts after that, and every wavefront finishes its 16 x 16 tiles
// itself (QKV: rotation of the pairs (i, i + D/2), which sit 32 lanes apart; output projection:
// residual add). 1-D grid: workgroup ids go round-robin over the 8 XCDs, so the token groups of
// one strip group are given ids 8 apart: they share an L2 and read the strips from HBM once.
// Requires nkb % WIN == 0.
// ------------------------------------------------------------------------------------
template <typename ST, int EPI, int NTW, int WS, int NKB = 0>
__global__ __launch_bounds__(WS * 64) void gemm_dense_strip_kernel(const GemmArgs a) {
  static_assert(EPI == EPI_QKV || EPI == EPI_RESID, "dense projections only");
  constexpr int WIN = 16;
  extern __shared__ __attribute__((aligned(16))) u32x4 s_b[];  // [NTW token tiles][nkb][64]
  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int nkb = NKB > 0 ? NKB : a.nkb;
  const int T = dyn_tokens(a.T_dev, a.T);
  const unsigned ntg = (unsigned)a.dense_tiles;  // token groups of NTW * 16 tokens
  const unsigned xcd = blockIdx.x & 7u, i = blockIdx.x >> 3;
  const unsigned tg = i % ntg;
  const unsigned sg = (i / ntg) * 8u + xcd;  // strip group
  if (sg * WS >= (unsigned)a.n_strips) return;  // (whole workgroup: no barrier is left waiting)
  const int strip_raw = (int)sg * WS + w;
  const bool active = strip_raw < a.n_strips;  // the last group may be short: its idle wavefronts still stage and wait
  const int strip = active ? strip_raw : a.n_strips - 1;
  const int tok0 = (int)tg * NTW * 16;
  if (tok0 >= T) return;  // (a token group past the call's actual token count: whole workgroup, before any barrier)
  const int lc = lane & 15;

  // token operand first, weights behind it
  const char* xrow[NTW];
  bool valid[NTW];
#pragma unroll
  for (int t = 0; t < NTW; ++t) {
    int col = tok0 + t * 16 + lc;
    valid[t] = active && col < T;
    col = col < T ? col : T - 1;  // padded columns repeat the last token; never stored
    xrow[t] = (const char*)a.X + (long long)col * a.ldx_bytes + (lane >> 4) * 16;
  }
  constexpr int BMAX = 4;  // operand blocks a wavefront stages per pass and token tile
  const u32x4* wp = a.W + (long long)strip * nkb * 64 + lane;
  u32x4 A[WIN];
#pragma unroll
  for (int kb0 = 0; kb0 < (NKB > 0 ? NKB : nkb); kb0 += BMAX * WS) {
    u32x4 bst[NTW][BMAX];
#pragma unroll
    for (int t = 0; t < NTW; ++t)
#pragma unroll
      for (int q = 0; q < BMAX; ++q) {
        const int kb = kb0 + q * WS + w;
        if (kb < nkb) bst[t][q] = *reinterpret_cast<const u32x4*>(xrow[t] + (long long)kb * 64);
      }
    if (kb0 == 0) {
#pragma unroll
      for (int j = 0; j < WIN; ++j) A[j] = wp[j * 64];
    }
#pragma unroll
    for (int t = 0; t < NTW; ++t)
#pragma unroll
      for (int q = 0; q < BMAX; ++q) {
        const int kb = kb0 + q * WS + w;
        if (kb < nkb) s_b[((size_t)t * nkb + kb) * 64 + lane] = bst[t][q];
      }
  }
  // what the epilogue needs is requested now, so that its round trip hides behind the weight stream
  f32x4 pre0[NTW], pre1[NTW];
#pragma unroll
  for (int t = 0; t < NTW; ++t) {
    const int col = tok0 + t * 16 + lc;
    const int tokc = col < T ? col : 0;
    if (EPI == EPI_RESID) {
      pre0[t] = load4<ST>(a.resid, (long long)tokc * a.ldo + strip * 16 + (lane >> 4) * 4);
      pre1[t] = f32x4{0, 0, 0, 0};
    } else {
      const int spd = a.D >> 4;
      const int head = strip / spd, js = strip - head * spd;
      const int idx = js * 8 + ((lane >> 4) & 1) * 4;
      const float* cs = a.rope_cs + (long long)tokc * a.D;
      pre0[t] = *reinterpret_cast<const f32x4*>(cs + idx);
      pre1[t] = *reinterpret_cast<const f32x4*>(cs + (a.D >> 1) + idx);
    }
  }
  lds_barrier();
  f32x4 acc[NTW];
#pragma unroll
  for (int t = 0; t < NTW; ++t) acc[t] = f32x4{0, 0, 0, 0};
  // operand blocks are requested from LDS PD steps ahead of their MFMAs (ring of registers), so the LDS
  // latency hides behind the matrix work of the steps in between
  constexpr int PD = 4;
  static_assert(WIN % PD == 0, "ring positions must repeat with the window");
  u32x4 bq[PD][NTW];
#pragma unroll
  for (int p = 0; p < PD; ++p)
#pragma unroll
    for (int t = 0; t < NTW; ++t) bq[p][t] = s_b[((size_t)t * nkb + p) * 64 + lane];
#pragma unroll
  for (int j0 = 0; j0 < (NKB > 0 ? NKB : nkb); j0 += WIN) {
#pragma unroll
    for (int jj = 0; jj < WIN; ++jj) {
      const int j = j0 + jj;
#pragma unroll
      for (int t = 0; t < NTW; ++t) acc[t] = mfma_block<ST>(A[jj], bq[jj % PD][t], acc[t]);
      if (j + PD < nkb) {
#pragma unroll
        for (int t = 0; t < NTW; ++t) bq[jj % PD][t] = s_b[((size_t)t * nkb + j + PD) * 64 + lane];
      }
      if (j + WIN < nkb) A[jj] = wp[(j + WIN) * 64];
      if (NKB > 0) __builtin_amdgcn_sched_barrier(0);  // keep the refills right behind their MFMA: window and ring stay full
    }
  }
  const int m0 = (lane >> 4) * 4;  // first of this lane's 4 rows in the strip
#pragma unroll
  for (int t = 0; t < NTW; ++t) {
    const int col = tok0 + t * 16 + lc;
    const f32x4 sum = acc[t];
    if (EPI == EPI_RESID) {
      if (valid[t]) store4<ST>(a.out0, (long long)col * a.ldo + strip * 16 + m0, pre0[t] + sum);
    } else {  // rotate pairs (i, i + D/2), which sit 32 lanes apart
      const int spd = a.D >> 4;  // strips per head
      const int head = strip / spd, js = strip - head * spd;
      const int half = a.D >> 1;
      const int g4 = lane >> 4;
      const int idx = js * 8 + (g4 & 1) * 4;  // index inside the half
      f32x4 other, r4;
#pragma unroll
      for (int q = 0; q < 4; ++q) other[q] = __shfl_xor(sum[q], 32);
      const bool rot = head < a.Hq + a.Hkv;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const float cv = rot ? pre0[t][q] : 1.0f;
        const float sv = rot ? pre1[t][q] : 0.0f;
        r4[q] = (g4 < 2) ? (sum[q] * cv - other[q] * sv) : (sum[q] * cv + other[q] * sv);
      }
      if (valid[t]) {
        const int hrow = (g4 < 2 ? 0 : half) + idx;
        if (head < a.Hq) {
          store4<ST>(a.out0, ((long long)col * a.Hq + head) * a.D + hrow, r4);
        } else if (head < a.Hq + a.Hkv) {
          store4<ST>(a.out1, ((long long)col * a.Hkv + (head - a.Hq)) * a.D + hrow, r4);
        } else {
          store4<ST>(a.out2, ((long long)col * a.Hkv + (head - a.Hq - a.Hkv)) * a.D + hrow, r4);
        }
      }
    }
  }
}

}  // namespace evict
