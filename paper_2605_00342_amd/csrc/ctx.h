// Private definition of the opaque context: model shape plus scratch buffers allocated once.
#pragma once
#include "common.h"

namespace evict { struct WorkRec; }

// Addressing of a paged KV cache: position p of sequence b lives in page table[b][p >> page_shift]
// at row p & (page size - 1). table == nullptr: contiguous caches.
struct KvPaging {
  const int32_t* table;  // [B][table_stride] page ids
  int table_stride;
  int page_shift;        // log2 of the page size in positions
  int n_pages;           // pages in every pool: ids outside [0, n_pages) are flagged and read as page 0
};

struct evict_ctx {
  evict_model_desc m;
  int max_tokens, max_batch, max_ctx;
  int device;
  int max_splits;        // KV splits the attention scratch is sized for (context part)
  int moe_grid, moe_prefetch, moe_chunk_gateup, moe_chunk_down, moe_down_kernel, moe_gateup_kernel, moe_nt_loads, dense_nt_loads, dense_nt, dense_units, attn_target_wgs, attn_waves, moe_nt, attn_row_blocks, dense_kernel, dense_ntw, moe_lds_dma, lm_units, lm_nt, moe_pair_down, moe_down_ws;  // launch-shape knobs (evict_tune)
  int timing;            // record stage events in evict_verify_layer
  int timed_once;        // a timed call has been recorded
  int capturing;         // a stream capture opened by evict_graph_begin is in progress
  KvPaging paging;       // set by the paged entry points for the duration of their call, else table == nullptr
  const int32_t* t_dev;  // evict_dynamic_tokens: device word with the actual token count of the calls that take T, or nullptr
  hipEvent_t ev[EVICT_N_STAGES + 1];
  // ---- device scratch (all sized for max_tokens) ----
  int32_t* status;       // [1] sticky status bits
  uint64_t* anc;         // [T][2] ancestor-or-self bitmask of each node (tree-local bit index)
  int32_t* depth;        // [T]
  int32_t* seq_of;       // [T] sequence index of each token
  float* rope_cs;        // [T][D] cos (first half) and sin (second half) per token
  double* rope_rev;      // [D/2] rotary frequencies in revolutions per position
  void* x_norm;          // [T][d] storage dtype
  void* q;               // [T][Hq*D]
  float* part_o;         // [splits+1][T][Hq][D]
  float* part_ml;        // [splits+1][T][Hq][2]
  void* attn_o;          // [T][Hq*D]
  void* h;               // [T][d]
  void* h_norm;          // [T][d]
  float* logits;         // [T][E]
  int32_t* topk_idx;     // [T][k]
  float* topk_w;         // [T][k]
  int32_t* hist;         // [E]
  int32_t* offsets;      // [E+1]
  int32_t* union_ids;    // [E]
  int32_t* union_count;  // [1]
  int32_t* perm;         // [T*k]
  int32_t* inv;          // [T*k]
  evict::WorkRec* work;  // [E] device-side work list, one record per union slot
  int32_t* sched;        // [4]: [0] work-list slots of the grouped GEMMs, [1] running total of union sizes over layer calls
  int32_t* tok_of_pos;   // [T*k] token of each grouped position
  void* act;             // [T*k + n_shared*T][F] storage dtype (routed pairs, then shared experts x tokens)
  float* y;              // [T*k + n_shared*T][d]
  float* lm_val;         // [T][vocab/16] best logit per token and strip
  int32_t* lm_idx;       // [T][vocab/16]
  float* samp_stats;     // [T][2] per node: max logit, sum of exp((logit - max) / temperature)
  void* stack_buf[2];    // [T][d] ping-pong hidden states of evict_verify_stack
  hipEvent_t prof_ev[2]; // evict_profile_cost
};
