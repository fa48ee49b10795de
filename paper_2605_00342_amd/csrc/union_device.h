// Expert union (Eq. 5) and the token grouping it induces, as a device routine run by one
// workgroup; shared by the stand-alone union kernel and the fused top-k + union kernel.
#pragma once
#include "ctx.h"
#include "gemm_stream.h"

namespace evict {

__device__ __forceinline__ int lane_id() { return threadIdx.x & 63; }

// Inclusive prefix sum over the wavefront through DPP row operations (no LDS traffic): shifts by
// 1, 2, 4, 8 inside each row of 16 lanes (lanes without a source add 0), then the total of the
// previous row into rows 1 and 3, then the total of rows 0-1 into rows 2 and 3.
__device__ __forceinline__ int wave_incl_scan(int v) {
  v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xF, 0xF, false);  // row_shr:1
  v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xF, 0xF, false);  // row_shr:2
  v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xF, 0xF, false);  // row_shr:4
  v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xF, 0xF, false);  // row_shr:8
  v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xA, 0xF, false);  // row_bcast:15 into rows 1, 3
  v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xC, 0xF, false);  // row_bcast:31 into rows 2, 3
  return v;
}

// Exclusive prefix sum over the block (blockDim.x multiple of 64, <= 1024 threads).
__device__ int block_excl_scan(int v, int* s_wave, int* total) {
  const int lane = lane_id(), w = threadIdx.x >> 6, nw = blockDim.x >> 6;
  int incl = wave_incl_scan(v);
  __syncthreads();
  if (lane == 63) s_wave[w] = incl;
  __syncthreads();
  int base = 0, tot = 0;
  for (int i = 0; i < nw; ++i) {
    int x = s_wave[i];
    if (i < w) base += x;
    tot += x;
  }
  *total = tot;
  return base + incl - v;
}

// Token t sits at rank r (of n) inside its expert: enter it into the record of its tile of tt
// (16 or 32) tokens; the last token of a tile also fills the record's unused entries (padded
// columns repeat it).
__device__ inline void work_put_token(WorkRec* first, int r, int n, int t, int tt) {
  WorkRec* rec = first + r / tt;
  const int i = r % tt;
  if (i < kWorkToks) rec->tok[i] = t;
  if (i == tt - 1 || r == n - 1)
    for (int j = i + 1; j < kWorkToks; ++j) rec->tok[j] = t;
}

// LDS needed by expert_union_body, in ints (before the optional bitmasks).
__host__ __device__ inline size_t union_lds_ints(int P, int E) { return (size_t)((P + 3 * E + 2) & ~1); }

// Requires blockDim.x >= E (one expert per thread in the scan).
// Fast path (no expert repeated inside a token, which is what TopK produces): per expert a
// bitmask over tokens, built with LDS atomics; counts, ranks inside an expert and the stable
// order all follow from popcounts. General path (repeats present, or masks too large for
// LDS): one thread per expert walks the pairs in ascending pair id.
// topk_idx: global [T*k], or nullptr when s_mem[0..P) already holds the indices.
__device__ inline void expert_union_body(
    int* s_mem, const int32_t* __restrict__ topk_idx, int T, int k, int E, int use_masks, int32_t* __restrict__ union_ids,
    int32_t* __restrict__ union_count, int32_t* __restrict__ hist, int32_t* __restrict__ offsets,
    int32_t* __restrict__ perm, int32_t* __restrict__ inv, int32_t* __restrict__ status, WorkRec* __restrict__ work,
    int32_t* __restrict__ tok_of_pos, int32_t* __restrict__ slot_count = nullptr, int n_shared = 0, int tt = 16) {
  const int P = T * k;
  const int words = (T + 63) >> 6;
  int* s_idx = s_mem;            // [P]
  int* s_hist = s_mem + P;       // [E]
  int* s_off = s_hist + E;       // [E + 1]
  int* s_slot = s_off + E + 1;   // [E] union slot of each activated expert
  unsigned long long* s_mask = reinterpret_cast<unsigned long long*>(s_mem + ((P + 3 * E + 2) & ~1));  // [E][words]
  __shared__ int s_wave[16];
  __shared__ int s_dup;
  const int tid = threadIdx.x, nthreads = blockDim.x;
  // slot_count[1] keeps a running total of the union sizes (read by the cost profiler); the old
  // value is requested now so that its round trip is over long before the total is written back
  const int union_total = (tid == 0 && slot_count) ? slot_count[1] : 0;
  for (int e = tid; e < E; e += nthreads) s_hist[e] = 0;
  if (use_masks)
    for (int i = tid; i < E * words; i += nthreads) s_mask[i] = 0ull;
  if (tid == 0) s_dup = 0;
  __syncthreads();
  bool bad = false;
  for (int p = tid; p < P; p += nthreads) {
    int e = topk_idx ? topk_idx[p] : s_idx[p];  // null: the caller has already filled s_idx
    if (e < 0 || e >= E) { bad = true; e = 0; }
    s_idx[p] = e;
    atomicAdd(&s_hist[e], 1);
    if (use_masks) {
      const int t = p / k;
      const unsigned long long bit = 1ull << (t & 63);
      const unsigned long long old = atomicOr(&s_mask[e * words + (t >> 6)], bit);
      if (old & bit) s_dup = 1;  // the same expert twice in one token
    }
  }
  if (bad && status) atomicOr(status, ST_BAD_EXPERT);
  __syncthreads();
  // one exclusive scan for both the pair counts and the activated flags (packed: count in the
  // low 16 bits, flag above; T*k <= 8192 and E <= 1024 fit), one expert per thread
  const int hcount = tid < E ? s_hist[tid] : 0;
  int tot;
  const int base = block_excl_scan(hcount | ((hcount > 0 ? 1 : 0) << 16), s_wave, &tot);
  const int base_h = base & 0xFFFF, base_f = base >> 16;
  const int tot_h = tot & 0xFFFF, tot_f = tot >> 16;
  // work list: one slot per (activated expert, tile of tt of its tokens); second scan for the slots
  int wslot = 0;
  if (work) {
    int tot_s;
    wslot = block_excl_scan((hcount + tt - 1) / tt, s_wave, &tot_s);
    // always-on shared experts: every token, in token order, appended behind the routed pairs
    // (expert id E + s; positions T*k + s*T + t), one slot per tile of tt tokens
    const int ttiles = (T + tt - 1) / tt;
    if (tid == 0 && slot_count) slot_count[0] = tot_s + n_shared * ttiles;
    for (int q = tid; q < n_shared * ttiles; q += nthreads) {
      const int sh = q / ttiles, i = q - sh * ttiles;
      WorkRec* rec = work + tot_s + q;
      rec->expert = E + sh;
      rec->p0 = P + sh * T + tt * i;
      rec->ntok = T - tt * i < tt ? T - tt * i : tt;
      rec->pad = ttiles | (i << 16);
      for (int j = 0; j < kWorkToks; ++j) rec->tok[j] = tt * i + (j < rec->ntok ? j : rec->ntok - 1);
    }
    if (tok_of_pos)
      for (int q = tid; q < n_shared * T; q += nthreads) tok_of_pos[P + q] = q % T;
  }
  if (tid < E) {
    s_off[tid] = base_h;
    offsets[tid] = base_h;
    hist[tid] = hcount;
    if (hcount > 0) {
      union_ids[base_f] = tid;
      s_slot[tid] = wslot;
      if (work) {
        const int ntile = (hcount + tt - 1) / tt;
        for (int i = 0; i < ntile; ++i) {
          WorkRec* rec = work + wslot + i;
          rec->expert = tid;
          rec->p0 = base_h + tt * i;
          rec->ntok = hcount - tt * i < tt ? hcount - tt * i : tt;
          rec->pad = ntile | (i << 16);  // tiles of this expert (low half), index of this tile (high half)
        }
      }
    }
  }
  for (int e = tot_f + tid; e < E; e += nthreads) union_ids[e] = -1;
  if (tid == 0) {
    offsets[E] = tot_h;
    union_count[0] = tot_f;
    if (slot_count) slot_count[1] = (int)((unsigned)union_total + (unsigned)tot_f);  // (wraps; the profiler resets it)
  }
  __syncthreads();
  if (use_masks && !s_dup) {
    // position of pair (t, slot) inside its expert = number of earlier tokens routed there
    for (int p = tid; p < P; p += nthreads) {
      const int e = s_idx[p], t = p / k;
      const unsigned long long* m = s_mask + e * words;
      int pos = s_off[e];
      for (int wd = 0; wd < (t >> 6); ++wd) pos += __popcll(m[wd]);
      pos += __popcll(m[t >> 6] & ((1ull << (t & 63)) - 1ull));
      perm[pos] = p;
      inv[p] = pos;
      if (tok_of_pos) tok_of_pos[pos] = t;
      if (work) work_put_token(work + s_slot[e], pos - s_off[e], s_hist[e], t, tt);
    }
  } else {
    for (int e = tid; e < E; e += nthreads) {
      if (s_hist[e] == 0) continue;
      int pos = s_off[e];
      for (int p = 0; p < P; ++p) {
        if (s_idx[p] == e) {
          perm[pos] = p;
          inv[p] = pos;
          if (tok_of_pos) tok_of_pos[pos] = p / k;
          if (work) work_put_token(work + s_slot[e], pos - s_off[e], s_hist[e], p / k, tt);
          ++pos;
        }
      }
    }
  }
}

}  // namespace evict
