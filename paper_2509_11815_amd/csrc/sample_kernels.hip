// Per-node vocab argmax, greedy acceptance walk and KV compaction (the T_sample part of a
// speculative round, SpecVLM Sec. 3.1 Eq. 1, plus the cache bookkeeping that follows it).
#include <limits.h>

#include "common.hpp"

namespace specvlm {

// ---------------------------------------------------------------------------------------
// node_argmax: one 1024-thread workgroup per (request, node) row.  A row of 32000 bf16
// logits is 64 KB: 16-byte loads, (value, index) kept per thread, reduced with the
// "greater value, then lower index" order, which is associative and commutative, so the
// result does not depend on the reduction shape.
// ---------------------------------------------------------------------------------------
struct ValIdx {
    float v;
    int i;
};

__device__ __forceinline__ void take_better(ValIdx& a, float v, int i) {
    // -0 == +0 under the float compare, as the definition asks.
    if (v > a.v || (v == a.v && i < a.i)) {
        a.v = v;
        a.i = i;
    }
}

// The same when i is known to be greater than every index taken so far (a thread scans its entries
// in increasing order): equal values keep the earlier index, so only "greater" replaces.
__device__ __forceinline__ void take_later(ValIdx& a, float v, int i) {
    if (v > a.v) {
        a.v = v;
        a.i = i;
    }
}

template <typename T>
struct Elem;
template <>
struct Elem<uint16_t> {
    static constexpr int kPerVec = 8;
    __device__ static float at(const uint4& w, int e) {
        uint32_t x = (&w.x)[e >> 1];
        return __uint_as_float((e & 1) ? (x & 0xFFFF0000u) : (x << 16));
    }
    __device__ static float one(const uint16_t* p) { return bf16_bits_to_float(*p); }
};
template <>
struct Elem<float> {
    static constexpr int kPerVec = 4;
    __device__ static float at(const uint4& w, int e) { return __uint_as_float((&w.x)[e]); }
    __device__ static float one(const float* p) { return *p; }
};

// (defined with the acceptance kernel below)
template <bool COHERENT>
__device__ __forceinline__ void accept_walk(int b, int N_max, int path_cap, const int32_t* __restrict__ parent,
                                            const int32_t* __restrict__ draft_tok, const int32_t* amax,
                                            const int32_t* __restrict__ num_nodes, int32_t* __restrict__ accept_len,
                                            int32_t* __restrict__ path, int32_t* __restrict__ bonus_tok,
                                            int32_t* __restrict__ committed_tok, int32_t* __restrict__ err_flag,
                                            int (&s_par)[64], int (&s_tok)[64], int (&s_am)[64]);

// What the fused form needs on top of the arg-max: the acceptance walk's arguments and one
// arrival counter per request (zero between calls).
struct AcceptArgs {
    int path_cap;
    const int32_t *parent, *draft_tok;
    int32_t *accept_len, *path, *bonus_tok, *committed_tok, *err_flag;
    int32_t* counters;
};

// FUSED: the workgroup that finishes the last row of a request (ticket counter) also runs the
// greedy acceptance walk of that request, so arg-max + acceptance is one launch.
template <typename T, bool FUSED>
__global__ __launch_bounds__(1024) void node_argmax_kernel(int N_max, int V, const T* __restrict__ logits,
                                                           int64_t stride_b, int64_t stride_n,
                                                           const int32_t* __restrict__ num_nodes,
                                                           int32_t* amax, AcceptArgs acc) {
    __shared__ int s_last;
    __shared__ int s_par[64], s_tok[64], s_am[64];
    const int row = blockIdx.x;
    const int b = row / N_max, i = row % N_max;
    const int tid = threadIdx.x;
    int n = num_nodes ? num_nodes[b] : N_max;
    // publishes this row's result; FUSED: then draws the request's ticket, and the workgroup that
    // draws the last one walks the tree (called by all threads of the workgroup)
    auto finish = [&](int result) {
        if constexpr (!FUSED) {
            if (tid == 0) amax[row] = result;
        } else {
            if (tid == 0) {
                __hip_atomic_store(amax + row, result, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory");        // the store has been acknowledged
                int32_t* cnt = acc.counters + b * SPECVLM_COUNTER_STRIDE;     // a cache line per request
                const int ticket = __hip_atomic_fetch_add(cnt, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                const int last = ticket == N_max - 1;
                if (last) __hip_atomic_store(cnt, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                s_last = last;
            }
            __syncthreads();
            if (s_last)                                                   // uniform
                accept_walk<true>(b, N_max, acc.path_cap, acc.parent, acc.draft_tok, amax, num_nodes, acc.accept_len,
                                  acc.path, acc.bonus_tok, acc.committed_tok, acc.err_flag, s_par, s_tok, s_am);
        }
    };
    if (i >= n) {
        finish(-1);
        return;
    }
    const T* p = logits + b * stride_b + i * stride_n;
    constexpr int VEC = Elem<T>::kPerVec;
    ValIdx best{-INFINITY, INT_MAX};

    // scalar head up to the first 16-byte boundary, vector body, scalar tail
    int head = static_cast<int>(((16u - (reinterpret_cast<uintptr_t>(p) & 15u)) & 15u) / sizeof(T));
    head = min(head, V);
    // (every thread meets its entries in increasing index order: head, vector body, tail)
    for (int v = tid; v < head; v += blockDim.x) take_later(best, Elem<T>::one(p + v), v);
    const int nvec = (V - head) / VEC;
    const uint4* pv = reinterpret_cast<const uint4*>(p + head);
    // four 16-byte loads per thread are requested before the first is looked at (a row of 32000 bf16
    // logits is four per thread: one memory round trip instead of four in a row)
    for (int c0 = tid; c0 < nvec; c0 += 4 * blockDim.x) {
        uint4 w[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int c = c0 + u * blockDim.x;
            if (c < nvec) w[u] = pv[c];
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int c = c0 + u * blockDim.x;
            if (c < nvec) {
                const int base = head + c * VEC;
#pragma unroll
                for (int e = 0; e < VEC; ++e) take_later(best, Elem<T>::at(w[u], e), base + e);
            }
        }
    }
    for (int v = head + nvec * VEC + tid; v < V; v += blockDim.x) take_later(best, Elem<T>::one(p + v), v);

    // wavefront (64 lanes) reduction, then across the 16 wavefronts through LDS
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        float ov = __shfl_xor(best.v, off);
        int oi = __shfl_xor(best.i, off);
        take_better(best, ov, oi);
    }
    __shared__ float s_v[16];
    __shared__ int s_i[16];
    const int wave = tid >> 6, lane = tid & 63;
    if (lane == 0) {
        s_v[wave] = best.v;
        s_i[wave] = best.i;
    }
    __syncthreads();
    if (wave == 0) {
        const int nw = blockDim.x >> 6;
        ValIdx r{lane < nw ? s_v[lane] : -INFINITY, lane < nw ? s_i[lane] : INT_MAX};
#pragma unroll
        for (int off = 8; off >= 1; off >>= 1) {
            float ov = __shfl_xor(r.v, off);
            int oi = __shfl_xor(r.i, off);
            take_better(r, ov, oi);
        }
        if (lane == 0) s_i[0] = r.i == INT_MAX ? 0 : r.i;
    }
    __syncthreads();
    finish(s_i[0]);
}

int32_t launch_node_argmax(int32_t dtype, int32_t B, int32_t N_max, int32_t V, const void* logits,
                           int64_t stride_b, int64_t stride_n, const int32_t* num_nodes,
                           int32_t* amax, hipStream_t stream) {
    dim3 grid(B * N_max), block(1024);
    const AcceptArgs none{};
    if (dtype == SPECVLM_BF16)
        hipLaunchKernelGGL((node_argmax_kernel<uint16_t, false>), grid, block, 0, stream, N_max, V,
                           static_cast<const uint16_t*>(logits), stride_b, stride_n, num_nodes, amax, none);
    else
        hipLaunchKernelGGL((node_argmax_kernel<float, false>), grid, block, 0, stream, N_max, V,
                           static_cast<const float*>(logits), stride_b, stride_n, num_nodes, amax, none);
    return check_launch();
}

int32_t launch_node_argmax_accept(int32_t dtype, int32_t B, int32_t N_max, int32_t V, int32_t path_cap,
                                  const void* logits, int64_t stride_b, int64_t stride_n, const int32_t* num_nodes,
                                  const int32_t* parent, const int32_t* draft_tok, int32_t* amax, int32_t* accept_len,
                                  int32_t* path, int32_t* bonus_tok, int32_t* committed_tok, int32_t* counters,
                                  int32_t* err_flag, hipStream_t stream) {
    dim3 grid(B * N_max), block(1024);
    const AcceptArgs acc{path_cap, parent, draft_tok, accept_len, path, bonus_tok, committed_tok, err_flag, counters};
    if (dtype == SPECVLM_BF16)
        hipLaunchKernelGGL((node_argmax_kernel<uint16_t, true>), grid, block, 0, stream, N_max, V,
                           static_cast<const uint16_t*>(logits), stride_b, stride_n, num_nodes, amax, acc);
    else
        hipLaunchKernelGGL((node_argmax_kernel<float, true>), grid, block, 0, stream, N_max, V,
                           static_cast<const float*>(logits), stride_b, stride_n, num_nodes, amax, acc);
    return check_launch();
}

// ---------------------------------------------------------------------------------------
// tree_accept: one wavefront per request, lane i owns node i.  Every lane walks its own
// root path (parent[i] < i bounds the walk by i steps), so a lane knows whether its node
// is accepted and how deep it is; a wavefront max over (depth, -index) picks the node.
// accept_walk is called by ALL threads of a workgroup (it contains a workgroup barrier);
// only the first 64 act.  COHERENT: amax was written by other workgroups of the same
// kernel (device-coherent loads); otherwise by an earlier kernel.
// ---------------------------------------------------------------------------------------
template <bool COHERENT>
__device__ __forceinline__ void accept_walk(int b, int N_max, int path_cap, const int32_t* __restrict__ parent,
                                            const int32_t* __restrict__ draft_tok, const int32_t* amax,
                                            const int32_t* __restrict__ num_nodes, int32_t* __restrict__ accept_len,
                                            int32_t* __restrict__ path, int32_t* __restrict__ bonus_tok,
                                            int32_t* __restrict__ committed_tok, int32_t* __restrict__ err_flag,
                                            int (&s_par)[64], int (&s_tok)[64], int (&s_am)[64]) {
    const int lane = threadIdx.x;
    const bool active = lane < 64;                          // uniform per wavefront
    int err = 0;
    int n = num_nodes ? num_nodes[b] : N_max;
    if (n < 1 || n > N_max) {
        err |= SPECVLM_ERR_BAD_NUM_NODES;
        n = min(max(n, 1), N_max);
    }
    bool bad = false;
    if (active) {
        int par = -1, tok = -1, am = -1;
        if (lane < n) {
            par = parent[b * N_max + lane];
            tok = draft_tok[b * N_max + lane];
            if constexpr (COHERENT)
                am = __hip_atomic_load(amax + b * N_max + lane, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            else
                am = amax[b * N_max + lane];
            bad = lane == 0 ? par != -1 : (par < 0 || par >= lane);
        }
        s_par[lane] = par;
        s_tok[lane] = tok;
        s_am[lane] = am;
    }
    __syncthreads();
    if (!active) return;
    int32_t* prow = path + b * path_cap;
    int32_t* crow = committed_tok + b * path_cap;
    if (__any(bad)) {                       // malformed tree: commit the root only
        err |= SPECVLM_ERR_BAD_PARENT;
        if (lane == 0) {
            accept_len[b] = 0;
            bonus_tok[b] = s_am[0];
            if (err_flag) atomicOr(err_flag, err);
        }
        for (int j = lane; j < path_cap; j += 64) {
            prow[j] = j == 0 ? 0 : -1;
            crow[j] = j == 0 ? s_am[0] : -1;
        }
        return;
    }
    bool ok = lane < n;
    int depth = 0;
    if (lane < n) {
        int t = lane;
        while (s_par[t] != -1) {
            int p = s_par[t];
            ok = ok && (s_tok[t] == s_am[p]);
            t = p;
            ++depth;
        }
    }
    if (ok && depth > path_cap - 1) {
        err |= SPECVLM_ERR_PATH_TOO_LONG;
        ok = false;
    }
    int key = ok ? depth * 64 + (63 - lane) : -1;   // deeper first, then lower index
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) key = max(key, __shfl_xor(key, off));
    const int best = 63 - (key & 63), m = key >> 6;
    if (lane == best) {
        int t = lane;
        for (int j = m; j >= 0; --j) {
            prow[j] = t;
            if (j >= 1) crow[j - 1] = s_tok[t];
            t = s_par[t];
        }
        crow[m] = s_am[best];
        accept_len[b] = m;
        bonus_tok[b] = s_am[best];
    }
    for (int j = m + 1 + lane; j < path_cap; j += 64) {
        prow[j] = -1;
        crow[j] = -1;
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) err |= __shfl_xor(err, off);
    if (lane == 0 && err && err_flag) atomicOr(err_flag, err);
}

__global__ __launch_bounds__(64) void tree_accept_kernel(int N_max, int path_cap,
                                                         const int32_t* __restrict__ parent,
                                                         const int32_t* __restrict__ draft_tok,
                                                         const int32_t* __restrict__ amax,
                                                         const int32_t* __restrict__ num_nodes,
                                                         int32_t* __restrict__ accept_len,
                                                         int32_t* __restrict__ path,
                                                         int32_t* __restrict__ bonus_tok,
                                                         int32_t* __restrict__ committed_tok,
                                                         int32_t* __restrict__ err_flag) {
    __shared__ int s_par[64], s_tok[64], s_am[64];
    accept_walk<false>(blockIdx.x, N_max, path_cap, parent, draft_tok, amax, num_nodes, accept_len, path, bonus_tok,
                       committed_tok, err_flag, s_par, s_tok, s_am);
}

int32_t launch_tree_accept(int32_t B, int32_t N_max, int32_t path_cap, const int32_t* parent,
                           const int32_t* draft_tok, const int32_t* amax, const int32_t* num_nodes,
                           int32_t* accept_len, int32_t* path, int32_t* bonus_tok,
                           int32_t* committed_tok, int32_t* err_flag, hipStream_t stream) {
    hipLaunchKernelGGL(tree_accept_kernel, dim3(B), dim3(64), 0, stream, N_max, path_cap, parent,
                       draft_tok, amax, num_nodes, accept_len, path, bonus_tok, committed_tok, err_flag);
    return check_launch();
}

// ---------------------------------------------------------------------------------------
// kv_compact: one 256-thread workgroup per (layer, K|V, KV head, request).  The rows of
// the accepted path (<= 64 rows of <= 512 bytes) are read into registers as 16-byte
// chunks, the workgroup synchronises, then the chunks are written to their destination
// rows: gather semantics even though source and destination ranges overlap.  Rows that
// do not move (path[j] == j, always true for the root) are skipped.
// ---------------------------------------------------------------------------------------
constexpr int kCompactThreads = 256;
constexpr int kCompactChunksPerThread = 8;   // 64 rows * 32 chunks / 256 threads

__global__ __launch_bounds__(kCompactThreads) void kv_compact_kernel(
    KvGeom g, unsigned char* k_base, unsigned char* v_base, int64_t layer_stride_bytes,
    void* const* k_ptrs, void* const* v_ptrs, int elem_bytes, int row_chunks,
    const int32_t* __restrict__ prefix_len, const int32_t* __restrict__ path, int path_cap,
    const int32_t* __restrict__ accept_len, int32_t* __restrict__ new_prefix_len, int32_t* __restrict__ moved_idx,
    int32_t* __restrict__ err_flag) {
    const int l = blockIdx.x >> 1, which = blockIdx.x & 1;
    const int hk = blockIdx.y, b = blockIdx.z, tid = threadIdx.x;
    // new_prefix_len is given here only when it does not alias prefix_len (which every workgroup
    // of the request reads): then the request's first workgroup writes the bookkeeping outputs
    if (new_prefix_len && blockIdx.x == 0 && hk == 0 && tid < path_cap) {
        const int P0 = prefix_len[b];
        const int m0 = min(max(accept_len[b], 0), path_cap - 1);
        if (moved_idx) {
            moved_idx[(b * path_cap + tid) * 2 + 0] = tid <= m0 ? P0 + path[b * path_cap + tid] : -1;
            moved_idx[(b * path_cap + tid) * 2 + 1] = tid <= m0 ? P0 + tid : -1;
        }
        if (tid == 0) new_prefix_len[b] = P0 + m0 + 1;
    }
    unsigned char* base;
    if (k_ptrs)
        base = static_cast<unsigned char*>(which ? v_ptrs[l] : k_ptrs[l]);
    else
        base = (which ? v_base : k_base) + l * layer_stride_bytes;
    const int P = prefix_len[b];
    const int m = min(max(accept_len[b], 0), path_cap - 1);
    const int total = (m + 1) * row_chunks;
    uint4 regs[kCompactChunksPerThread];
    int64_t dst_off[kCompactChunksPerThread];
#pragma unroll
    for (int c = 0; c < kCompactChunksPerThread; ++c) {
        const int idx = tid + c * kCompactThreads;
        dst_off[c] = -1;
        regs[c] = uint4{0u, 0u, 0u, 0u};
        if (idx < total) {
            const int j = idx / row_chunks, ch = idx - j * row_chunks;
            const int a = path[b * path_cap + j];
            // a row moves only if it is a valid, different slot inside the cache
            if (a != j && a >= 0 && a < SPECVLM_MAX_NODES && P >= 0 && P + a < g.capacity && P + j < g.capacity) {
                bool bad_block = false;
                const int64_t src = kv_row_offset(g, b, hk, P + a, bad_block) * elem_bytes + ch * 16;
                const int64_t dst = kv_row_offset(g, b, hk, P + j, bad_block) * elem_bytes + ch * 16;
                if (!bad_block) {                      // a row whose block id is out of range stays where it is
                    regs[c] = *reinterpret_cast<const uint4*>(base + src);
                    dst_off[c] = dst;
                } else if (err_flag && ch == 0 && blockIdx.x == 0 && hk == 0) {
                    atomicOr(err_flag, SPECVLM_ERR_BAD_BLOCK);
                }
            }
        }
    }
    __syncthreads();
#pragma unroll
    for (int c = 0; c < kCompactChunksPerThread; ++c)
        if (dst_off[c] >= 0) *reinterpret_cast<uint4*>(base + dst_off[c]) = regs[c];
}

__global__ void kv_compact_finish_kernel(int B, const int32_t* __restrict__ prefix_len,
                                         const int32_t* __restrict__ path, int path_cap,
                                         const int32_t* __restrict__ accept_len,
                                         int32_t* new_prefix_len, int32_t* __restrict__ moved_idx) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    const int P = prefix_len[b];
    const int m = min(max(accept_len[b], 0), path_cap - 1);
    if (moved_idx)
        for (int j = 0; j < path_cap; ++j) {
            moved_idx[(b * path_cap + j) * 2 + 0] = j <= m ? P + path[b * path_cap + j] : -1;
            moved_idx[(b * path_cap + j) * 2 + 1] = j <= m ? P + j : -1;
        }
    new_prefix_len[b] = P + m + 1;
}

int32_t launch_kv_compact(const specvlm_attn_desc& d, int32_t L, void* k_base, void* v_base,
                          int64_t layer_stride, void* const* k_ptrs, void* const* v_ptrs,
                          const int32_t* block_table, const int32_t* prefix_len, const int32_t* path,
                          int32_t path_cap, const int32_t* accept_len, int32_t* new_prefix_len,
                          int32_t* moved_idx, int32_t* err_flag, hipStream_t stream) {
    const int eb = d.dtype == SPECVLM_BF16 ? 2 : 4;
    KvGeom g{d.kv_stride_b, d.kv_stride_h, d.kv_stride_t, d.paged ? block_table : nullptr,
             d.max_blocks_per_req, d.num_blocks,
             d.paged ? d.max_blocks_per_req * SPECVLM_PAGE_SIZE : d.kv_capacity};
    dim3 grid(L * 2, d.H_kv, d.B);
    // One launch when new_prefix_len is a buffer of its own; when it aliases prefix_len it may only
    // be written after every workgroup has read the old lengths: a second, tiny launch.
    const bool alias = new_prefix_len == prefix_len;
    hipLaunchKernelGGL(kv_compact_kernel, grid, dim3(kCompactThreads), 0, stream, g,
                       static_cast<unsigned char*>(k_base), static_cast<unsigned char*>(v_base),
                       layer_stride * eb, k_ptrs, v_ptrs, eb, d.D * eb / 16, prefix_len, path,
                       path_cap, accept_len, alias ? nullptr : new_prefix_len, alias ? nullptr : moved_idx, err_flag);
    int32_t rc = check_launch();
    if (rc || !alias) return rc;
    hipLaunchKernelGGL(kv_compact_finish_kernel, dim3((d.B + 63) / 64), dim3(64), 0, stream, d.B,
                       prefix_len, path, path_cap, accept_len, new_prefix_len, moved_idx);
    return check_launch();
}

}  // namespace specvlm
