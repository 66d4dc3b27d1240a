// Internal declarations shared by the HIP translation units of libspecvlm (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "specvlm.h"

namespace specvlm {

// Records a failed HIP call for specvlm_last_hip_error().
void note_hip_error(hipError_t e);

inline int32_t check_launch() {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        note_hip_error(e);
        return SPECVLM_HIP_ERROR;
    }
    return SPECVLM_OK;
}

__device__ __forceinline__ float bf16_bits_to_float(uint16_t b) {
    return __uint_as_float(static_cast<uint32_t>(b) << 16);
}

// Kernel-side view of the K/V cache geometry of one request's rows.
struct KvGeom {
    int64_t stride_b, stride_h, stride_t;   // elements
    const int32_t* block_table;             // nullptr => contiguous
    int32_t max_blocks;                     // per request (paged)
    int32_t num_blocks;                     // pool size (paged)
    int32_t capacity;                       // slots per request
};

// Element offset of logical slot `slot` of request b, KV head hk.  `slot` must be < capacity.
// A block id outside [0, num_blocks) sets `bad_block` (the caller reports SPECVLM_ERR_BAD_BLOCK and
// must not write there); the offset returned then lies inside the pool all the same.
__device__ __forceinline__ int64_t kv_row_offset(const KvGeom& g, int b, int hk, int slot, bool& bad_block) {
    if (g.block_table) {
        int blk = g.block_table[static_cast<int64_t>(b) * g.max_blocks + (slot >> 4)];
        if (blk < 0 || blk >= g.num_blocks) bad_block = true;
        blk = min(max(blk, 0), g.num_blocks - 1);
        return blk * g.stride_b + hk * g.stride_h + (slot & 15) * g.stride_t;
    }
    return b * g.stride_b + hk * g.stride_h + slot * g.stride_t;
}

// Launchers (defined next to their kernels).  All return a specvlm_status.
int32_t launch_node_argmax(int32_t dtype, int32_t B, int32_t N_max, int32_t V, const void* logits,
                           int64_t stride_b, int64_t stride_n, const int32_t* num_nodes,
                           int32_t* amax, hipStream_t stream);

int32_t launch_node_argmax_accept(int32_t dtype, int32_t B, int32_t N_max, int32_t V, int32_t path_cap,
                                  const void* logits, int64_t stride_b, int64_t stride_n, const int32_t* num_nodes,
                                  const int32_t* parent, const int32_t* draft_tok, int32_t* amax, int32_t* accept_len,
                                  int32_t* path, int32_t* bonus_tok, int32_t* committed_tok, int32_t* counters,
                                  int32_t* err_flag, hipStream_t stream);

int32_t launch_tree_accept(int32_t B, int32_t N_max, int32_t path_cap, const int32_t* parent,
                           const int32_t* draft_tok, const int32_t* amax, const int32_t* num_nodes,
                           int32_t* accept_len, int32_t* path, int32_t* bonus_tok,
                           int32_t* committed_tok, int32_t* err_flag, hipStream_t stream);

int32_t launch_tree_accept_sample(int32_t dtype, int32_t B, int32_t N_max, int32_t V, int32_t path_cap,
                                  const int32_t* parent, const int32_t* draft_tok, const void* logits,
                                  int64_t stride_b, int64_t stride_n, const int32_t* num_nodes,
                                  float temperature, const float* u_accept, const float* u_bonus,
                                  int32_t* accept_len, int32_t* path, int32_t* bonus_tok,
                                  int32_t* committed_tok, int32_t* err_flag, hipStream_t stream);

int32_t launch_kv_compact(const specvlm_attn_desc& d, int32_t L, void* k_base, void* v_base,
                          int64_t layer_stride, void* const* k_ptrs, void* const* v_ptrs,
                          const int32_t* block_table, const int32_t* prefix_len, const int32_t* path,
                          int32_t path_cap, const int32_t* accept_len, int32_t* new_prefix_len,
                          int32_t* moved_idx, int32_t* err_flag, hipStream_t stream);

int32_t launch_visual_pool(int32_t dtype, int32_t B, int32_t T, int32_t E, int32_t ratio, const void* x,
                           int64_t x_sb, int64_t x_st, const int32_t* num_tokens, void* y, int64_t y_sb,
                           int64_t y_st, int32_t* out_tokens, int32_t* err_flag, hipStream_t stream);
int32_t launch_visual_prune(int32_t elem_bytes, int32_t B, int32_t T, int32_t T_keep, int32_t E, const void* x,
                            int64_t x_sb, int64_t x_st, const int32_t* keep, void* y, int64_t y_sb, int64_t y_st,
                            int32_t* err_flag, hipStream_t stream);

size_t head_argmax_workspace_bytes(int32_t B, int32_t N_max, int32_t V);
int32_t launch_head_argmax(int32_t B, int32_t N_max, int32_t E, int32_t V, const void* hidden,
                           int64_t h_stride_row, const void* W, int64_t w_stride_v, const int32_t* num_nodes,
                           int32_t* amax, float* max_logit, void* workspace, hipStream_t stream);

int32_t launch_draft_topk(int32_t dtype, int32_t B, int32_t W, int32_t V, int32_t K, const void* logits,
                          int64_t stride_b, int64_t stride_w, const float* cum, int64_t cum_stride_b,
                          const int32_t* parent_idx, int64_t parent_stride_b, float* score_out,
                          int32_t* token_out, int32_t* parent_out, int64_t out_stride_b, float* lse_out,
                          int32_t M, int32_t index_base, int32_t* sel_out, float* sel_score_out,
                          int32_t* count_out, int32_t* counters, hipStream_t stream);

int32_t launch_draft_select(int32_t B, int32_t C, int32_t M, const float* score, int64_t score_stride_b,
                            const int32_t* num_cand, int32_t index_base, int32_t* sel_out,
                            float* sel_score_out, int32_t* count_out, hipStream_t stream);

int32_t launch_draft_finalize(int32_t B, int32_t C, int32_t N_max, const float* cand_score,
                              const int32_t* cand_parent, const int32_t* cand_token, int64_t cand_stride_b,
                              const int32_t* num_cand, const int32_t* root_token, int32_t* parent_out,
                              int32_t* draft_tok_out, int32_t* node_cand_out, int32_t* num_nodes_out,
                              int32_t* err_flag, hipStream_t stream);

struct AttnArgs {
    specvlm_attn_desc d;
    float scale;                // resolved softmax scale
    const void* q;
    const void* k;
    const void* v;
    const int32_t* block_table;
    const int32_t* prefix_len;
    const int32_t* num_nodes;
    const int32_t* parent;
    void* o;
    float* lse;
    void* workspace;
    size_t workspace_bytes;
    int32_t* err_flag;
    hipStream_t stream;
};

// fp32 VALU kernel: exact-ish path for SPECVLM_F32 (and a bf16 VALU variant kept for
// comparison measurements).
int32_t launch_attn_valu(const AttnArgs& a);

// bf16 MFMA split-key kernel + merge.
int32_t launch_attn_mfma(const AttnArgs& a);
size_t attn_mfma_workspace_bytes(const specvlm_attn_desc& d);
int32_t attn_mfma_pick_splits(const specvlm_attn_desc& d);
// Device address of the current device's library-owned scratch array (SPECVLM_STATIC_WORKSPACE_BYTES).
int32_t attn_static_workspace(void** ptr_out);

}  // namespace specvlm
