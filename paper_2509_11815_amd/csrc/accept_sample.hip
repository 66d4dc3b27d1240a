// Sampling-based acceptance walk over a draft tree (temperature > 0).
//
// SpecVLM Sec. 3.1 names speculative sampling as the rule that discards drafted tokens and
// Sec. 4.1 evaluates temperature 1 with the same Top-K tree.  The children of a tree node are
// fixed candidates (top-K expansion), i.e. point-mass proposals, so a child c with token x is
// accepted when its uniform number is below the residual target probability of x at the
// parent, p(x) / (1 - mass already rejected there); a rejected token leaves the distribution;
// the bonus token is drawn from the residual distribution of the last node by inverse CDF in
// vocabulary order.  Every emitted token then follows the target's own distribution.
//
// One 1024-thread workgroup per request.  The walk is sequential (at most path_cap levels);
// per level the workgroup reduces the node's logits row twice (maximum, then the sum of
// exp((l - max) / T), evaluated as exp2 of a scaled difference) in a fixed order, and one thread takes the few accept decisions.  The
// bonus draw is a two-level scan: every thread sums a contiguous chunk of the vocabulary,
// the chunk sums are scanned through LDS, and the thread whose chunk contains the drawn
// position walks its chunk.  A row of 32000 bf16 logits is 64 KB and stays in L2 between the
// passes; the whole call is launch- and latency-bound (T_sample of Sec. 3.1, Eq. 1).
#include "common.hpp"

namespace specvlm {

namespace {

constexpr int kThreadsAS = 1024;

template <typename T>
__device__ __forceinline__ float logit_at(const T* p, int v);
template <>
__device__ __forceinline__ float logit_at<uint16_t>(const uint16_t* p, int v) { return bf16_bits_to_float(p[v]); }
template <>
__device__ __forceinline__ float logit_at<float>(const float* p, int v) { return p[v]; }

// Workgroup reductions with a fixed shape (so that a result never depends on timing):
// xor-butterfly inside a wavefront, then the 16 wavefront results through LDS.
__device__ __forceinline__ float block_max(float x, float* s_red) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) x = fmaxf(x, __shfl_xor(x, off));
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    __syncthreads();                                   // s_red may still be read from a previous call
    if (lane == 0) s_red[wave] = x;
    __syncthreads();
    float r = s_red[0];
#pragma unroll
    for (int w = 1; w < kThreadsAS / 64; ++w) r = fmaxf(r, s_red[w]);
    return r;
}

__device__ __forceinline__ float block_sum(float x, float* s_red) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) x += __shfl_xor(x, off);
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    __syncthreads();
    if (lane == 0) s_red[wave] = x;
    __syncthreads();
    float r = s_red[0];
#pragma unroll
    for (int w = 1; w < kThreadsAS / 64; ++w) r += s_red[w];
    return r;
}

// CH > 0: every thread keeps its chunk of the current row (at most CH consecutive tokens) in
// registers, loaded once per level with 16-byte loads when the row allows; CH == 0: any
// vocabulary size, every pass re-reads the row.
template <typename T, int CH>
__global__ __launch_bounds__(kThreadsAS) void tree_accept_sample_kernel(
    int N_max, int V, int path_cap, const int32_t* __restrict__ parent, const int32_t* __restrict__ draft_tok,
    const T* __restrict__ logits, int64_t stride_b, int64_t stride_n, const int32_t* __restrict__ num_nodes,
    float temperature, const float* __restrict__ u_accept, const float* __restrict__ u_bonus,
    int32_t* __restrict__ accept_len, int32_t* __restrict__ path, int32_t* __restrict__ bonus_tok,
    int32_t* __restrict__ committed_tok, int32_t* __restrict__ err_flag) {
    __shared__ int s_par[SPECVLM_MAX_NODES], s_tok[SPECVLM_MAX_NODES], s_path[SPECVLM_MAX_NODES];
    __shared__ int s_rej[SPECVLM_MAX_NODES];           // tokens rejected at the current node
    __shared__ float s_cex[SPECVLM_MAX_NODES], s_cu[SPECVLM_MAX_NODES];
    __shared__ float s_red[kThreadsAS / 64];
    __shared__ float s_scan[kThreadsAS];
    __shared__ int s_next, s_nrej, s_err, s_pick, s_chunk;
    __shared__ unsigned long long s_kids;

    const int b = blockIdx.x, tid = threadIdx.x;
    int err = 0;
    int n = num_nodes ? num_nodes[b] : N_max;
    if (n < 1 || n > N_max) {
        err |= SPECVLM_ERR_BAD_NUM_NODES;
        n = min(max(n, 1), N_max);
    }
    bool bad = false;
    if (tid < SPECVLM_MAX_NODES) {
        int par = -1, tok = -1;
        if (tid < n) {
            par = parent[b * N_max + tid];
            tok = draft_tok[b * N_max + tid];
            bad = tid == 0 ? par != -1 : (par < 0 || par >= tid);
        }
        s_par[tid] = par;
        s_tok[tid] = tok;
    }
    if (tid == 0) s_err = 0;
    if (__syncthreads_or(bad)) {                       // malformed tree: the root has no usable children
        err |= SPECVLM_ERR_BAD_PARENT;
        n = 1;
    }

    const T* base = logits + b * stride_b;
    int cur = 0, m = 0;
    float mx = 0.f, Z = 0.f;
    // unnormalised probability exp((l - max) / T) as one multiply and one v_exp_f32 (the whole
    // vocabulary goes through it three times on a single compute unit); -inf gives 0
    const float c2 = 1.4426950408889634f / temperature;
    auto prob_of = [&](float l) -> float { return __builtin_amdgcn_exp2f((l - mx) * c2); };
    const int chunk = (V + kThreadsAS - 1) / kThreadsAS;          // consecutive tokens per thread
    const int v0 = min(tid * chunk, V), v1 = min(v0 + chunk, V);
    constexpr int VEC = 16 / sizeof(T);
    float lv[CH > 0 ? CH : 1];                          // this thread's logits of the current row
    for (;;) {
        const T* row = base + cur * stride_n;
        // Wavefront 0, lane c: child c's logit and uniform number, requested now so that they
        // arrive while the row is reduced (a dependent load after the reductions would add a
        // memory round trip to every level of the walk).
        bool is_child = false;
        float child_logit = 0.f, child_u = 1.f;
        int child_tok = -1;
        if (tid < SPECVLM_MAX_NODES) {
            is_child = tid > cur && tid < n && s_par[tid] == cur;
            if (is_child) {
                child_tok = s_tok[tid];
                if (child_tok >= 0 && child_tok < V) child_logit = logit_at<T>(row, child_tok);
                child_u = u_accept[b * N_max + tid];
            }
        }
        // target distribution at cur, unnormalised: e(v) = exp((l_v - max) / T)
        float part = -INFINITY;
        if constexpr (CH > 0) {
            const bool vec_ok = (reinterpret_cast<uintptr_t>(row) & 15u) == 0 && chunk % VEC == 0 && V % VEC == 0;
            if (vec_ok) {                               // uniform
#pragma unroll
                for (int j = 0; j < CH / VEC; ++j) {
                    if (v0 + j * VEC < v1) {
                        const uint4 w = *reinterpret_cast<const uint4*>(row + v0 + j * VEC);
#pragma unroll
                        for (int e = 0; e < VEC; ++e) {
                            if constexpr (sizeof(T) == 2) {
                                const uint32_t x = (&w.x)[e >> 1];
                                lv[j * VEC + e] = __uint_as_float((e & 1) ? (x & 0xFFFF0000u) : (x << 16));
                            } else {
                                lv[j * VEC + e] = __uint_as_float((&w.x)[e]);
                            }
                        }
                    }
                }
            } else {
#pragma unroll
                for (int i = 0; i < CH; ++i)
                    if (v0 + i < v1) lv[i] = logit_at<T>(row, v0 + i);
            }
#pragma unroll
            for (int i = 0; i < CH; ++i)
                if (v0 + i < v1) part = fmaxf(part, lv[i]);
        } else {
            // (loops unrolled so that a batch of independent loads is in flight: the row sits in
            // L2 and the passes are latency-bound otherwise)
#pragma unroll 8
            for (int v = tid; v < V; v += kThreadsAS) part = fmaxf(part, logit_at<T>(row, v));
        }
        mx = block_max(part, s_red);
        part = 0.f;
        if constexpr (CH > 0) {
#pragma unroll
            for (int i = 0; i < CH; ++i)
                if (v0 + i < v1) part += prob_of(lv[i]);
        } else {
#pragma unroll 8
            for (int v = tid; v < V; v += kThreadsAS) part += prob_of(logit_at<T>(row, v));
        }
        Z = block_sum(part, s_red);
        // the candidates of cur, prepared in parallel: lane c holds child c's unnormalised
        // probability and uniform number, so that the sequential decisions below wait for no load
        if (tid < SPECVLM_MAX_NODES) {                  // wavefront 0
            float ex = -1.f;                            // ex < 0 marks "token out of range"
            if (is_child && child_tok >= 0 && child_tok < V) ex = prob_of(child_logit);
            s_cex[tid] = ex;
            s_cu[tid] = child_u;
            const unsigned long long kids = __ballot(is_child);
            if (tid == 0) s_kids = kids;
        }
        __syncthreads();
        if (tid == 0) {
            int next = -1, nrej = 0, e = 0;
            float rejmass = 0.f;
            unsigned long long kids = s_kids;          // children of cur, tried in increasing node index
            const bool has_child = kids != 0;
            if (m + 1 >= path_cap) kids = 0;           // no room for a deeper node: nothing is tested
            while (kids && next < 0) {
                const int c = __builtin_ctzll(kids);
                kids &= kids - 1;
                const int x = s_tok[c];
                const float ex = s_cex[c];
                bool live = ex >= 0.f;
                if (!live) e |= SPECVLM_ERR_BAD_TOKEN;
                for (int r = 0; r < nrej; ++r) live = live && s_rej[r] != x;
                if (!live) continue;                   // residual probability 0: rejected
                const float a = ex / fmaxf(Z - rejmass, ex);   // the residual mass holds x itself
                if (s_cu[c] < a) {
                    next = c;
                } else {
                    s_rej[nrej++] = x;
                    rejmass += ex;
                }
            }
            if (has_child && m + 1 >= path_cap) e |= SPECVLM_ERR_PATH_TOO_LONG;
            s_next = next;
            s_nrej = nrej;
            s_err |= e;
            s_path[m] = cur;
        }
        __syncthreads();
        const int next = s_next;
        if (next < 0) break;                           // uniform
        cur = next;
        ++m;
        __syncthreads();                               // s_next is rewritten in the next round
    }

    // ---- bonus token: inverse CDF over the residual distribution at cur, in vocabulary order ----
    const T* row = base + cur * stride_n;
    const int nrej = s_nrej;
    // Which tokens of this thread's chunk were rejected at cur: a bit mask when the chunk has at
    // most 64 tokens (vocabularies up to 65536), so that the per-token test touches no memory.
    unsigned long long rejmask = 0;
    const bool small_chunk = chunk <= 64;
    if (small_chunk)
        for (int r = 0; r < nrej; ++r) {
            const int x = s_rej[r];
            if (x >= v0 && x < v1) rejmask |= 1ull << (x - v0);
        }
    auto residual = [&](int v) -> float {             // v in [v0, v1); CH == 0 only
        bool live = true;
        if (small_chunk) {
            live = !((rejmask >> (v - v0)) & 1ull);
        } else {
            for (int r = 0; r < nrej; ++r) live = live && s_rej[r] != v;
        }
        return live ? prob_of(logit_at<T>(row, v)) : 0.f;
    };
    float csum = 0.f;
    if constexpr (CH > 0) {                            // lv[] still holds cur's row
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            lv[i] = (v0 + i < v1 && !((rejmask >> i) & 1ull)) ? prob_of(lv[i]) : 0.f;   // now the residual mass
            csum += lv[i];
        }
    } else {
#pragma unroll 8
        for (int v = v0; v < v1; ++v) csum += residual(v);
    }
    // inclusive scan of the chunk sums: inside each wavefront by shuffles, then the 16 wavefront
    // totals (summed in order by every thread) as offsets
    float incl = csum;
    const int lane = tid & 63, wave = tid >> 6;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const float up = __shfl_up(incl, off);
        if (lane >= off) incl += up;
    }
    if (tid == 0) { s_pick = -1; s_chunk = -1; }
    __syncthreads();                                   // s_red is free (last use: the row sum)
    if (lane == 63) s_red[wave] = incl;
    __syncthreads();
    float offset = 0.f;
    for (int w = 0; w < wave; ++w) offset += s_red[w];
    s_scan[tid] = incl + offset;
    __syncthreads();
    const float total = s_scan[kThreadsAS - 1];
    const float t = u_bonus[b] * total;
    const float before = tid ? s_scan[tid - 1] : 0.f;
    if (s_scan[tid] > t && before <= t) s_chunk = tid; // the scan is non-decreasing: exactly one such chunk
    __syncthreads();
    if (s_chunk == tid) {
        float cum = before;
        int pick = -1, last_live = -1;
        if constexpr (CH > 0) {
#pragma unroll
            for (int i = 0; i < CH; ++i) {
                if (lv[i] > 0.f) last_live = v0 + i;
                cum += lv[i];
                if (pick < 0 && cum > t) pick = v0 + i;
            }
        } else {
            for (int v = v0; v < v1 && pick < 0; ++v) {
                const float ev = residual(v);
                if (ev > 0.f) last_live = v;
                cum += ev;
                if (cum > t) pick = v;
            }
        }
        s_pick = pick >= 0 ? pick : last_live;        // rounding inside the chunk: its last live token
    }
    __syncthreads();
    if (tid == 0) {
        int pick = s_pick;
        if (pick < 0) {                                // t landed on the total by rounding: last live token
            for (int v = V - 1; v >= 0 && pick < 0; --v) {
                bool live = true;
                for (int r = 0; r < nrej; ++r) live = live && s_rej[r] != v;
                if (live && prob_of(logit_at<T>(row, v)) > 0.f) pick = v;
            }
            if (pick < 0) pick = 0;
        }
        accept_len[b] = m;
        bonus_tok[b] = pick;
        int32_t* prow = path + b * path_cap;
        int32_t* crow = committed_tok + b * path_cap;
        for (int j = 0; j < path_cap; ++j) {
            prow[j] = j <= m ? s_path[j] : -1;
            crow[j] = j < m ? s_tok[s_path[j + 1]] : (j == m ? pick : -1);
        }
        err |= s_err;
        if (err && err_flag) atomicOr(err_flag, err);
    }
}

}  // namespace

int32_t launch_tree_accept_sample(int32_t dtype, int32_t B, int32_t N_max, int32_t V, int32_t path_cap,
                                  const int32_t* parent, const int32_t* draft_tok, const void* logits,
                                  int64_t stride_b, int64_t stride_n, const int32_t* num_nodes,
                                  float temperature, const float* u_accept, const float* u_bonus,
                                  int32_t* accept_len, int32_t* path, int32_t* bonus_tok,
                                  int32_t* committed_tok, int32_t* err_flag, hipStream_t stream) {
    dim3 grid(B), block(kThreadsAS);
#define SPECVLM_LAUNCH_AS(T, CH)                                                                              \
    hipLaunchKernelGGL((tree_accept_sample_kernel<T, CH>), grid, block, 0, stream, N_max, V, path_cap, parent, \
                       draft_tok, static_cast<const T*>(logits), stride_b, stride_n, num_nodes, temperature,  \
                       u_accept, u_bonus, accept_len, path, bonus_tok, committed_tok, err_flag)
    const int chunk = (V + kThreadsAS - 1) / kThreadsAS;
    if (dtype == SPECVLM_BF16) {
        if (chunk <= 32) SPECVLM_LAUNCH_AS(uint16_t, 32);
        else if (chunk <= 64) SPECVLM_LAUNCH_AS(uint16_t, 64);
        else SPECVLM_LAUNCH_AS(uint16_t, 0);
    } else {
        if (chunk <= 32) SPECVLM_LAUNCH_AS(float, 32);
        else if (chunk <= 64) SPECVLM_LAUNCH_AS(float, 64);
        else SPECVLM_LAUNCH_AS(float, 0);
    }
#undef SPECVLM_LAUNCH_AS
    return check_launch();
}

}  // namespace specvlm
