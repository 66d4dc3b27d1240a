// C ABI of libspecvlm: host-side argument checks and kernel dispatch.  See include/specvlm.h
// for the contract of every entry point.
#include <math.h>

#include "common.hpp"

namespace specvlm {

static thread_local int32_t g_last_hip_error = 0;
void note_hip_error(hipError_t e) { g_last_hip_error = static_cast<int32_t>(e); }

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Geometry checks common to attention and compaction.
static int32_t check_kv_geometry(const specvlm_attn_desc& d) {
    if (d.dtype != SPECVLM_BF16 && d.dtype != SPECVLM_F32) return SPECVLM_INVALID_ARG;
    if (d.B < 1 || d.H_kv < 1 || (d.D != 64 && d.D != 128)) return SPECVLM_INVALID_ARG;
    const int vec = d.dtype == SPECVLM_BF16 ? 8 : 4;                 // elements per 16 bytes
    if (d.kv_stride_t < d.D || d.kv_stride_t % vec || d.kv_stride_h % vec || d.kv_stride_b % vec)
        return SPECVLM_INVALID_ARG;
    if (d.kv_stride_h < 0 || d.kv_stride_b < 0) return SPECVLM_INVALID_ARG;
    if (d.kv_stride_t > (1 << 24)) return SPECVLM_INVALID_ARG;       // lane offsets inside a tile are 32-bit
    if (d.paged) {
        if (d.block_size != SPECVLM_PAGE_SIZE || d.max_blocks_per_req < 1 || d.num_blocks < 1)
            return SPECVLM_INVALID_ARG;
    } else if (d.kv_capacity < 1) {
        return SPECVLM_INVALID_ARG;
    }
    return SPECVLM_OK;
}

static int32_t check_attn_desc(const specvlm_attn_desc& d) {
    int32_t rc = check_kv_geometry(d);
    if (rc) return rc;
    if (d.H_q < 1 || d.H_q % d.H_kv) return SPECVLM_INVALID_ARG;
    if (d.N_max < 1 || d.N_max > SPECVLM_MAX_NODES) return SPECVLM_INVALID_ARG;
    if (!(d.softmax_scale >= 0.f) || isinf(d.softmax_scale)) return SPECVLM_INVALID_ARG;
    if (d.num_splits < 0 || d.num_splits > SPECVLM_MAX_SPLITS) return SPECVLM_INVALID_ARG;
    const int vec = d.dtype == SPECVLM_BF16 ? 8 : 4;
    const int64_t st[6] = {d.q_stride_b, d.q_stride_n, d.q_stride_h, d.o_stride_b, d.o_stride_n, d.o_stride_h};
    for (int64_t s : st)
        if (s < 0 || s % vec) return SPECVLM_INVALID_ARG;
    if (d.q_stride_h < d.D || d.o_stride_h < d.D) return SPECVLM_INVALID_ARG;
    return SPECVLM_OK;
}

}  // namespace specvlm

using namespace specvlm;

extern "C" {

int32_t specvlm_version(void) { return 300; }

int32_t specvlm_last_hip_error(void) { return g_last_hip_error; }

size_t specvlm_tree_verify_attn_workspace_bytes(const specvlm_attn_desc* desc) {
    if (!desc || check_attn_desc(*desc)) return 0;
    if (desc->dtype == SPECVLM_F32) return 256;
    return attn_mfma_workspace_bytes(*desc);
}

int32_t specvlm_tree_verify_attn_num_splits(const specvlm_attn_desc* desc) {
    if (!desc || check_attn_desc(*desc)) return 0;
    if (desc->dtype == SPECVLM_F32) return 1;
    return attn_mfma_pick_splits(*desc);
}

enum { kCallerWorkspace = 0, kStaticWorkspace = 1, kVectorAluKernel = 2 };

static int32_t tree_verify_attn(const specvlm_attn_desc* desc, const void* q_dev, const void* k_cache_dev,
                                const void* v_cache_dev, const int32_t* block_table_dev,
                                const int32_t* prefix_len_dev, const int32_t* num_nodes_dev,
                                const int32_t* parent_dev, void* o_dev, float* lse_dev, int mode,
                                void* workspace_dev, size_t workspace_bytes, int32_t* err_flag_dev,
                                void* stream) {
    const bool static_workspace = mode == kStaticWorkspace;
    if (!desc) return SPECVLM_INVALID_ARG;
    int32_t rc = check_attn_desc(*desc);
    if (rc) return rc;
    if (!q_dev || !k_cache_dev || !v_cache_dev || !prefix_len_dev || !parent_dev || !o_dev)
        return SPECVLM_INVALID_ARG;
    if ((desc->paged != 0) != (block_table_dev != nullptr)) return SPECVLM_INVALID_ARG;
    if (!aligned16(q_dev) || !aligned16(k_cache_dev) || !aligned16(v_cache_dev) || !aligned16(o_dev))
        return SPECVLM_INVALID_ARG;
    AttnArgs a;
    a.d = *desc;
    a.scale = desc->softmax_scale > 0.f ? desc->softmax_scale : 1.0f / sqrtf(static_cast<float>(desc->D));
    a.q = q_dev; a.k = k_cache_dev; a.v = v_cache_dev;
    a.block_table = block_table_dev; a.prefix_len = prefix_len_dev; a.num_nodes = num_nodes_dev;
    a.parent = parent_dev; a.o = o_dev; a.lse = lse_dev;
    a.workspace = workspace_dev; a.workspace_bytes = workspace_bytes;
    a.err_flag = err_flag_dev; a.stream = static_cast<hipStream_t>(stream);
    if (desc->dtype == SPECVLM_F32 || mode == kVectorAluKernel) return launch_attn_valu(a);
    const size_t need = attn_mfma_workspace_bytes(*desc);
    if (attn_mfma_pick_splits(*desc) > 1) {
        if (static_workspace) {
            if (need > SPECVLM_STATIC_WORKSPACE_BYTES) return SPECVLM_WORKSPACE_TOO_SMALL;
            rc = attn_static_workspace(&a.workspace);
            if (rc) return rc;
            a.workspace_bytes = SPECVLM_STATIC_WORKSPACE_BYTES;
        }
        if (!a.workspace || (reinterpret_cast<uintptr_t>(a.workspace) & 255u)) return SPECVLM_INVALID_ARG;
        if (a.workspace_bytes < need) return SPECVLM_WORKSPACE_TOO_SMALL;
    }
    return launch_attn_mfma(a);
}

int32_t specvlm_tree_verify_attn(const specvlm_attn_desc* desc, const void* q_dev, const void* k_cache_dev,
                                 const void* v_cache_dev, const int32_t* block_table_dev,
                                 const int32_t* prefix_len_dev, const int32_t* num_nodes_dev,
                                 const int32_t* parent_dev, void* o_dev, float* lse_dev,
                                 void* workspace_dev, size_t workspace_bytes, int32_t* err_flag_dev,
                                 void* stream) {
    return tree_verify_attn(desc, q_dev, k_cache_dev, v_cache_dev, block_table_dev, prefix_len_dev, num_nodes_dev,
                            parent_dev, o_dev, lse_dev, kCallerWorkspace, workspace_dev, workspace_bytes, err_flag_dev, stream);
}

int32_t specvlm_tree_verify_attn_static(const specvlm_attn_desc* desc, const void* q_dev, const void* k_cache_dev,
                                        const void* v_cache_dev, const int32_t* block_table_dev,
                                        const int32_t* prefix_len_dev, const int32_t* num_nodes_dev,
                                        const int32_t* parent_dev, void* o_dev, float* lse_dev,
                                        int32_t* err_flag_dev, void* stream) {
    return tree_verify_attn(desc, q_dev, k_cache_dev, v_cache_dev, block_table_dev, prefix_len_dev, num_nodes_dev,
                            parent_dev, o_dev, lse_dev, kStaticWorkspace, nullptr, 0, err_flag_dev, stream);
}

int32_t specvlm_tree_verify_attn_vector_alu(const specvlm_attn_desc* desc, const void* q_dev, const void* k_cache_dev,
                                            const void* v_cache_dev, const int32_t* block_table_dev,
                                            const int32_t* prefix_len_dev, const int32_t* num_nodes_dev,
                                            const int32_t* parent_dev, void* o_dev, float* lse_dev,
                                            int32_t* err_flag_dev, void* stream) {
    return tree_verify_attn(desc, q_dev, k_cache_dev, v_cache_dev, block_table_dev, prefix_len_dev, num_nodes_dev,
                            parent_dev, o_dev, lse_dev, kVectorAluKernel, nullptr, 0, err_flag_dev, stream);
}

int32_t specvlm_node_argmax(int32_t dtype, int32_t B, int32_t N_max, int32_t V, const void* logits_dev,
                            int64_t stride_b, int64_t stride_n, const int32_t* num_nodes_dev,
                            int32_t* amax_dev, void* stream) {
    if (dtype != SPECVLM_BF16 && dtype != SPECVLM_F32) return SPECVLM_INVALID_ARG;
    if (B < 1 || N_max < 1 || N_max > SPECVLM_MAX_NODES || V < 1) return SPECVLM_INVALID_ARG;
    if (!logits_dev || !amax_dev || stride_b < 0 || stride_n < V) return SPECVLM_INVALID_ARG;
    const uintptr_t es = dtype == SPECVLM_BF16 ? 2 : 4;
    if (reinterpret_cast<uintptr_t>(logits_dev) % es) return SPECVLM_INVALID_ARG;
    return launch_node_argmax(dtype, B, N_max, V, logits_dev, stride_b, stride_n, num_nodes_dev, amax_dev,
                              static_cast<hipStream_t>(stream));
}

int32_t specvlm_tree_accept(int32_t B, int32_t N_max, int32_t path_cap, const int32_t* parent_dev,
                            const int32_t* draft_tok_dev, const int32_t* amax_dev,
                            const int32_t* num_nodes_dev, int32_t* accept_len_dev, int32_t* path_dev,
                            int32_t* bonus_tok_dev, int32_t* committed_tok_dev, int32_t* err_flag_dev,
                            void* stream) {
    if (B < 1 || N_max < 1 || N_max > SPECVLM_MAX_NODES || path_cap < 1 || path_cap > SPECVLM_MAX_NODES)
        return SPECVLM_INVALID_ARG;
    if (!parent_dev || !draft_tok_dev || !amax_dev || !accept_len_dev || !path_dev || !bonus_tok_dev ||
        !committed_tok_dev)
        return SPECVLM_INVALID_ARG;
    return launch_tree_accept(B, N_max, path_cap, parent_dev, draft_tok_dev, amax_dev, num_nodes_dev,
                              accept_len_dev, path_dev, bonus_tok_dev, committed_tok_dev, err_flag_dev,
                              static_cast<hipStream_t>(stream));
}

int32_t specvlm_node_argmax_accept(int32_t dtype, int32_t B, int32_t N_max, int32_t V, int32_t path_cap,
                                   const void* logits_dev, int64_t stride_b, int64_t stride_n,
                                   const int32_t* num_nodes_dev, const int32_t* parent_dev,
                                   const int32_t* draft_tok_dev, int32_t* amax_dev, int32_t* accept_len_dev,
                                   int32_t* path_dev, int32_t* bonus_tok_dev, int32_t* committed_tok_dev,
                                   int32_t* counters_dev, int32_t* err_flag_dev, void* stream) {
    if (dtype != SPECVLM_BF16 && dtype != SPECVLM_F32) return SPECVLM_INVALID_ARG;
    if (B < 1 || N_max < 1 || N_max > SPECVLM_MAX_NODES || V < 1 || path_cap < 1 || path_cap > SPECVLM_MAX_NODES)
        return SPECVLM_INVALID_ARG;
    if (!logits_dev || !amax_dev || stride_b < 0 || stride_n < V) return SPECVLM_INVALID_ARG;
    const uintptr_t es = dtype == SPECVLM_BF16 ? 2 : 4;
    if (reinterpret_cast<uintptr_t>(logits_dev) % es) return SPECVLM_INVALID_ARG;
    if (!parent_dev || !draft_tok_dev || !accept_len_dev || !path_dev || !bonus_tok_dev || !committed_tok_dev ||
        !counters_dev)
        return SPECVLM_INVALID_ARG;
    return launch_node_argmax_accept(dtype, B, N_max, V, path_cap, logits_dev, stride_b, stride_n, num_nodes_dev,
                                     parent_dev, draft_tok_dev, amax_dev, accept_len_dev, path_dev, bonus_tok_dev,
                                     committed_tok_dev, counters_dev, err_flag_dev, static_cast<hipStream_t>(stream));
}

int32_t specvlm_tree_accept_sample(int32_t dtype, int32_t B, int32_t N_max, int32_t V, int32_t path_cap,
                                   const int32_t* parent_dev, const int32_t* draft_tok_dev,
                                   const void* logits_dev, int64_t stride_b, int64_t stride_n,
                                   const int32_t* num_nodes_dev, float temperature,
                                   const float* u_accept_dev, const float* u_bonus_dev,
                                   int32_t* accept_len_dev, int32_t* path_dev, int32_t* bonus_tok_dev,
                                   int32_t* committed_tok_dev, int32_t* err_flag_dev, void* stream) {
    if (dtype != SPECVLM_BF16 && dtype != SPECVLM_F32) return SPECVLM_INVALID_ARG;
    if (B < 1 || N_max < 1 || N_max > SPECVLM_MAX_NODES || V < 1 || path_cap < 1 || path_cap > SPECVLM_MAX_NODES)
        return SPECVLM_INVALID_ARG;
    if (!(temperature > 0.f) || stride_n < V || stride_b < 0) return SPECVLM_INVALID_ARG;
    if (!parent_dev || !draft_tok_dev || !logits_dev || !u_accept_dev || !u_bonus_dev || !accept_len_dev ||
        !path_dev || !bonus_tok_dev || !committed_tok_dev)
        return SPECVLM_INVALID_ARG;
    return launch_tree_accept_sample(dtype, B, N_max, V, path_cap, parent_dev, draft_tok_dev, logits_dev,
                                     stride_b, stride_n, num_nodes_dev, temperature, u_accept_dev, u_bonus_dev,
                                     accept_len_dev, path_dev, bonus_tok_dev, committed_tok_dev, err_flag_dev,
                                     static_cast<hipStream_t>(stream));
}

int32_t specvlm_kv_compact(const specvlm_attn_desc* desc, int32_t L, void* k_base_dev, void* v_base_dev,
                           int64_t layer_stride, void* const* k_layer_ptrs_dev, void* const* v_layer_ptrs_dev,
                           const int32_t* block_table_dev, const int32_t* prefix_len_dev,
                           const int32_t* path_dev, int32_t path_cap, const int32_t* accept_len_dev,
                           int32_t* new_prefix_len_dev, int32_t* moved_idx_dev, int32_t* err_flag_dev,
                           void* stream) {
    if (!desc) return SPECVLM_INVALID_ARG;
    int32_t rc = check_kv_geometry(*desc);
    if (rc) return rc;
    if (L < 1 || L > 32767 || desc->H_kv > 65535 || desc->B > 65535) return SPECVLM_INVALID_ARG;
    if (path_cap < 1 || path_cap > SPECVLM_MAX_NODES) return SPECVLM_INVALID_ARG;
    if (!prefix_len_dev || !path_dev || !accept_len_dev || !new_prefix_len_dev) return SPECVLM_INVALID_ARG;
    if ((desc->paged != 0) != (block_table_dev != nullptr)) return SPECVLM_INVALID_ARG;
    const bool by_ptr = k_layer_ptrs_dev != nullptr || v_layer_ptrs_dev != nullptr;
    if (by_ptr) {
        if (!k_layer_ptrs_dev || !v_layer_ptrs_dev) return SPECVLM_INVALID_ARG;
    } else {
        if (!k_base_dev || !v_base_dev || !aligned16(k_base_dev) || !aligned16(v_base_dev)) return SPECVLM_INVALID_ARG;
        const int vec = desc->dtype == SPECVLM_BF16 ? 8 : 4;
        if (layer_stride < 0 || layer_stride % vec) return SPECVLM_INVALID_ARG;
    }
    return launch_kv_compact(*desc, L, k_base_dev, v_base_dev, layer_stride, k_layer_ptrs_dev,
                             v_layer_ptrs_dev, block_table_dev, prefix_len_dev, path_dev, path_cap,
                             accept_len_dev, new_prefix_len_dev, moved_idx_dev, err_flag_dev,
                             static_cast<hipStream_t>(stream));
}

static bool rows_ok(int32_t dtype, int32_t E, const void* p, int64_t sb, int64_t st) {
    const int vec = dtype == SPECVLM_BF16 ? 8 : 4;
    return p && aligned16(p) && E >= vec && E % vec == 0 && st >= E && st % vec == 0 && sb >= 0 && sb % vec == 0;
}

int32_t specvlm_visual_pool(int32_t dtype, int32_t B, int32_t T, int32_t E, int32_t ratio, const void* x_dev,
                            int64_t x_stride_b, int64_t x_stride_t, const int32_t* num_tokens_dev, void* y_dev,
                            int64_t y_stride_b, int64_t y_stride_t, int32_t* out_tokens_dev, int32_t* err_flag_dev,
                            void* stream) {
    if (dtype != SPECVLM_BF16 && dtype != SPECVLM_F32) return SPECVLM_INVALID_ARG;
    if (B < 1 || B > 65535 || T < 1 || ratio < 1) return SPECVLM_INVALID_ARG;
    if (!rows_ok(dtype, E, x_dev, x_stride_b, x_stride_t) || !rows_ok(dtype, E, y_dev, y_stride_b, y_stride_t))
        return SPECVLM_INVALID_ARG;
    return launch_visual_pool(dtype, B, T, E, ratio, x_dev, x_stride_b, x_stride_t, num_tokens_dev, y_dev,
                              y_stride_b, y_stride_t, out_tokens_dev, err_flag_dev, static_cast<hipStream_t>(stream));
}

int32_t specvlm_visual_prune(int32_t dtype, int32_t B, int32_t T, int32_t T_keep, int32_t E, const void* x_dev,
                             int64_t x_stride_b, int64_t x_stride_t, const int32_t* keep_dev, void* y_dev,
                             int64_t y_stride_b, int64_t y_stride_t, int32_t* err_flag_dev, void* stream) {
    if (dtype != SPECVLM_BF16 && dtype != SPECVLM_F32) return SPECVLM_INVALID_ARG;
    if (B < 1 || B > 65535 || T < 1 || T_keep < 1 || !keep_dev) return SPECVLM_INVALID_ARG;
    if (!rows_ok(dtype, E, x_dev, x_stride_b, x_stride_t) || !rows_ok(dtype, E, y_dev, y_stride_b, y_stride_t))
        return SPECVLM_INVALID_ARG;
    return launch_visual_prune(dtype == SPECVLM_BF16 ? 2 : 4, B, T, T_keep, E, x_dev, x_stride_b, x_stride_t,
                               keep_dev, y_dev, y_stride_b, y_stride_t, err_flag_dev,
                               static_cast<hipStream_t>(stream));
}

size_t specvlm_head_argmax_workspace_bytes(int32_t B, int32_t N_max, int32_t V) {
    if (B < 1 || N_max < 1 || N_max > SPECVLM_MAX_NODES || V < 1 || B > (1 << 20)) return 0;
    return head_argmax_workspace_bytes(B, N_max, V);
}

int32_t specvlm_head_argmax(int32_t dtype, int32_t B, int32_t N_max, int32_t E, int32_t V, const void* hidden_dev,
                            int64_t h_stride_b, int64_t h_stride_n, const void* w_dev, int64_t w_stride_v,
                            const int32_t* num_nodes_dev, int32_t* amax_dev, float* max_logit_dev,
                            void* workspace_dev, size_t workspace_bytes, void* stream) {
    if (dtype != SPECVLM_BF16 && dtype != SPECVLM_F32) return SPECVLM_INVALID_ARG;
    if (B < 1 || B > (1 << 20) || N_max < 1 || N_max > SPECVLM_MAX_NODES || V < 1 || E < 128 || E % 128)
        return SPECVLM_INVALID_ARG;
    if (!hidden_dev || !w_dev || !amax_dev || !workspace_dev) return SPECVLM_INVALID_ARG;
    if (h_stride_n < E || h_stride_n % 8 || w_stride_v < E || w_stride_v % 8 || w_stride_v > (1 << 24) ||
        h_stride_n > (1 << 24))
        return SPECVLM_INVALID_ARG;
    if (B > 1 && h_stride_b != static_cast<int64_t>(N_max) * h_stride_n) return SPECVLM_INVALID_ARG;
    if (!aligned16(hidden_dev) || !aligned16(w_dev) || (reinterpret_cast<uintptr_t>(workspace_dev) & 255u))
        return SPECVLM_INVALID_ARG;
    if (dtype == SPECVLM_F32) return SPECVLM_UNSUPPORTED;
    if (workspace_bytes < head_argmax_workspace_bytes(B, N_max, V)) return SPECVLM_WORKSPACE_TOO_SMALL;
    return launch_head_argmax(B, N_max, E, V, hidden_dev, h_stride_n, w_dev, w_stride_v, num_nodes_dev, amax_dev,
                              max_logit_dev, workspace_dev, static_cast<hipStream_t>(stream));
}

int32_t specvlm_draft_topk(int32_t dtype, int32_t B, int32_t W, int32_t V, int32_t K, const void* logits_dev,
                           int64_t stride_b, int64_t stride_w, const float* cum_dev, int64_t cum_stride_b,
                           const int32_t* parent_idx_dev, int64_t parent_stride_b, float* score_out_dev,
                           int32_t* token_out_dev, int32_t* parent_out_dev, int64_t out_stride_b,
                           float* lse_out_dev, void* stream) {
    if (dtype != SPECVLM_BF16 && dtype != SPECVLM_F32) return SPECVLM_INVALID_ARG;
    if (B < 1 || B > 65535 || W < 1 || V < 1 || K < 1 || K > V || K > SPECVLM_MAX_NODES) return SPECVLM_INVALID_ARG;
    if (!logits_dev || !score_out_dev || !token_out_dev) return SPECVLM_INVALID_ARG;
    if (stride_b < 0 || stride_w < V || cum_stride_b < 0 || parent_stride_b < 0) return SPECVLM_INVALID_ARG;
    if (out_stride_b < static_cast<int64_t>(W) * K) return SPECVLM_INVALID_ARG;
    const uintptr_t es = dtype == SPECVLM_BF16 ? 2 : 4;
    if (reinterpret_cast<uintptr_t>(logits_dev) % es) return SPECVLM_INVALID_ARG;
    return launch_draft_topk(dtype, B, W, V, K, logits_dev, stride_b, stride_w, cum_dev, cum_stride_b,
                             parent_idx_dev, parent_stride_b, score_out_dev, token_out_dev, parent_out_dev,
                             out_stride_b, lse_out_dev, 0, 0, nullptr, nullptr, nullptr, nullptr,
                             static_cast<hipStream_t>(stream));
}

int32_t specvlm_draft_topk_select(int32_t dtype, int32_t B, int32_t W, int32_t V, int32_t K, const void* logits_dev,
                                  int64_t stride_b, int64_t stride_w, const float* cum_dev, int64_t cum_stride_b,
                                  const int32_t* parent_idx_dev, int64_t parent_stride_b, float* score_out_dev,
                                  int32_t* token_out_dev, int32_t* parent_out_dev, int64_t out_stride_b,
                                  float* lse_out_dev, int32_t M, int32_t index_base, int32_t* sel_out_dev,
                                  float* sel_score_out_dev, int32_t* count_out_dev, int32_t* counters_dev,
                                  void* stream) {
    if (dtype != SPECVLM_BF16 && dtype != SPECVLM_F32) return SPECVLM_INVALID_ARG;
    if (B < 1 || B > 65535 || W < 1 || V < 1 || K < 1 || K > V || K > SPECVLM_MAX_NODES) return SPECVLM_INVALID_ARG;
    if (!logits_dev || !score_out_dev || !token_out_dev || !sel_out_dev || !counters_dev) return SPECVLM_INVALID_ARG;
    if (stride_b < 0 || stride_w < V || cum_stride_b < 0 || parent_stride_b < 0) return SPECVLM_INVALID_ARG;
    if (out_stride_b < static_cast<int64_t>(W) * K) return SPECVLM_INVALID_ARG;
    if (static_cast<int64_t>(W) * K > 1024 || M < 1 || M > SPECVLM_MAX_CANDIDATES) return SPECVLM_INVALID_ARG;
    const uintptr_t es = dtype == SPECVLM_BF16 ? 2 : 4;
    if (reinterpret_cast<uintptr_t>(logits_dev) % es) return SPECVLM_INVALID_ARG;
    return launch_draft_topk(dtype, B, W, V, K, logits_dev, stride_b, stride_w, cum_dev, cum_stride_b,
                             parent_idx_dev, parent_stride_b, score_out_dev, token_out_dev, parent_out_dev,
                             out_stride_b, lse_out_dev, M, index_base, sel_out_dev, sel_score_out_dev,
                             count_out_dev, counters_dev, static_cast<hipStream_t>(stream));
}

int32_t specvlm_draft_select(int32_t B, int32_t C, int32_t M, const float* score_dev, int64_t score_stride_b,
                             const int32_t* num_cand_dev, int32_t index_base, int32_t* sel_out_dev,
                             float* sel_score_out_dev, int32_t* count_out_dev, void* stream) {
    if (B < 1 || C < 1 || C > SPECVLM_MAX_CANDIDATES || M < 1 || M > SPECVLM_MAX_CANDIDATES) return SPECVLM_INVALID_ARG;
    if (!score_dev || !sel_out_dev || score_stride_b < C) return SPECVLM_INVALID_ARG;
    return launch_draft_select(B, C, M, score_dev, score_stride_b, num_cand_dev, index_base, sel_out_dev,
                               sel_score_out_dev, count_out_dev, static_cast<hipStream_t>(stream));
}

int32_t specvlm_draft_finalize(int32_t B, int32_t C, int32_t N_max, const float* cand_score_dev,
                               const int32_t* cand_parent_dev, const int32_t* cand_token_dev,
                               int64_t cand_stride_b, const int32_t* num_cand_dev, const int32_t* root_token_dev,
                               int32_t* parent_out_dev, int32_t* draft_tok_out_dev, int32_t* node_cand_out_dev,
                               int32_t* num_nodes_out_dev, int32_t* err_flag_dev, void* stream) {
    if (B < 1 || C < 1 || C > SPECVLM_MAX_CANDIDATES || N_max < 1 || N_max > SPECVLM_MAX_NODES)
        return SPECVLM_INVALID_ARG;
    if (!cand_score_dev || !cand_parent_dev || !cand_token_dev || !root_token_dev || !parent_out_dev ||
        !draft_tok_out_dev || !num_nodes_out_dev || cand_stride_b < C)
        return SPECVLM_INVALID_ARG;
    return launch_draft_finalize(B, C, N_max, cand_score_dev, cand_parent_dev, cand_token_dev, cand_stride_b,
                                 num_cand_dev, root_token_dev, parent_out_dev, draft_tok_out_dev,
                                 node_cand_out_dev, num_nodes_out_dev, err_flag_dev,
                                 static_cast<hipStream_t>(stream));
}

}  // extern "C"
