// Host-side launchers of the layer kernels (defined in layer_kernels.hip).
#pragma once
#include "ctx.h"

namespace evict {

struct GemmArgs;
struct WorkRec;

int launch_gemm(int dtype, int epi, const GemmArgs& a, int nt, int grid, hipStream_t s);
bool dense_strip_applies(const GemmArgs& a, int ntw);
int gateup_waves(const GemmArgs& a);
int launch_gemm_dense_strip(int dtype, int epi, GemmArgs a, int ntw, hipStream_t s);
int launch_pack(const void* src, long long src_group_bytes, int rows, int cols, int dtype, void* dst, int dst_strip0,
                int dst_strip_step, long long dst_group_strips, int groups, int head_dim, hipStream_t s);
int launch_prep(const evict_ctx* c, const int32_t* tree_off, const int32_t* parent, int B, int T, const int32_t* ctx_len,
                int max_ctx, const void* x, const void* gain, int norm_only, hipStream_t s);
int kernels_setup(const evict_model_desc& m);
int attn_splits_for(int max_ctx);
constexpr int kAttnMfmaMaxSplits = 34;  // bf16 attention: at most 32 context splits + the draft-node split (+ 1 spare)
int launch_attention(const evict_ctx* c, const void* kc, const void* vc, long long seq_stride, long long head_stride,
                     const int32_t* ctx_len, int max_ctx_host, const int32_t* tree_off, int B, int T, const void* k_new,
                     const void* v_new, void* aux_out, hipStream_t s);
int launch_router(const evict_ctx* c, const void* gain, const void* wg, int T, const evict_layer_aux* aux, hipStream_t s);
int launch_topk_union(const evict_ctx* c, int T, const evict_layer_aux* aux, int tile_tokens, hipStream_t s);
int launch_argmax_reduce(const float* val, const int32_t* idx, int nstrips, int ld, int T, int32_t* next, float* best_out,
                         const int32_t* t_dev, hipStream_t s);
int launch_combine(const evict_ctx* c, int T, void* out, const void* next_gain, hipStream_t s);

}  // namespace evict
