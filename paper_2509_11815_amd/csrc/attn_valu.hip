// Tree-masked verification attention on the vector ALUs, fp32 arithmetic throughout.
// This is the path for SPECVLM_F32 tensors (tolerance 1e-5, so no reduced-precision matrix
// cores), and a bf16-input variant kept to measure what a VALU-only kernel reaches.
//
// One 256-thread workgroup per (request, query head, tree node).  Thread t visits the
// visible keys t, t+256, ... with a private online softmax (running max, sum and a D-wide
// accumulator in registers); the 256 partial states are merged at the end.
#include "common.hpp"

namespace specvlm {

template <typename T>
__device__ __forceinline__ void load16(const T* p, float* out);   // 16 bytes -> floats

template <>
__device__ __forceinline__ void load16<float>(const float* p, float* out) {
    float4 w = *reinterpret_cast<const float4*>(p);
    out[0] = w.x; out[1] = w.y; out[2] = w.z; out[3] = w.w;
}
template <>
__device__ __forceinline__ void load16<uint16_t>(const uint16_t* p, float* out) {
    uint4 w = *reinterpret_cast<const uint4*>(p);
    const uint32_t x[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        out[2 * e] = __uint_as_float(x[e] << 16);
        out[2 * e + 1] = __uint_as_float(x[e] & 0xFFFF0000u);
    }
}

__device__ __forceinline__ void store_elem(float* p, float x) { *p = x; }
__device__ __forceinline__ void store_elem(uint16_t* p, float x) {
    uint32_t u = __float_as_uint(x);                     // round to nearest even
    u += 0x7FFFu + ((u >> 16) & 1u);
    *p = static_cast<uint16_t>(u >> 16);
}

struct ValuParams {
    KvGeom g;
    int N_max, H_q, group;
    float scale;
    const void *q, *k, *v;
    void* o;
    float* lse;
    int64_t q_sb, q_sn, q_sh, o_sb, o_sn, o_sh;
    const int32_t *prefix_len, *num_nodes, *parent;
    int32_t* err_flag;
};

template <typename T, int D>
__global__ __launch_bounds__(256) void attn_valu_kernel(ValuParams p) {
    constexpr int VEC = 16 / sizeof(T);
    const int i = blockIdx.x, h = blockIdx.y, b = blockIdx.z, tid = threadIdx.x;
    const int hk = h / p.group;
    __shared__ float s_q[D];
    __shared__ unsigned long long s_mask;
    __shared__ int s_err;
    __shared__ float s_red[4][D];
    __shared__ float s_m[4], s_l[4];

    int n = p.num_nodes ? p.num_nodes[b] : p.N_max;
    const int P = p.prefix_len[b];
    int err = 0;
    if (n < 1 || n > p.N_max) err |= SPECVLM_ERR_BAD_NUM_NODES;
    n = min(max(n, 1), p.N_max);
    if (P < 0 || P + n > p.g.capacity) err |= SPECVLM_ERR_BAD_LENGTH;
    if (tid == 0) {
        // ancestor-or-self bit mask of node i; the walk is bounded by 64 steps
        unsigned long long mask = 0;
        if (i < n) {
            int t = i;
            for (int step = 0; step < SPECVLM_MAX_NODES && t != -1; ++step) {
                mask |= 1ull << t;
                const int par = p.parent[b * p.N_max + t];
                if (t == 0 ? par != -1 : (par < 0 || par >= t)) {
                    err |= SPECVLM_ERR_BAD_PARENT;
                    break;
                }
                t = par;
            }
        }
        s_mask = mask;
        s_err = err;
    }
    const T* q = static_cast<const T*>(p.q) + b * p.q_sb + i * p.q_sn + h * p.q_sh;
    if (i < n && !err && tid < D / VEC) {
        float tmp[VEC];
        load16<T>(q + tid * VEC, tmp);
#pragma unroll
        for (int e = 0; e < VEC; ++e) s_q[tid * VEC + e] = tmp[e];
    }
    __syncthreads();
    err = s_err;
    if (err) {
        if (tid == 0 && p.err_flag) atomicOr(p.err_flag, err);
        return;
    }
    if (i >= n) return;
    const unsigned long long mask = s_mask;
    const int S = P + n;
    const T* kbase = static_cast<const T*>(p.k);
    const T* vbase = static_cast<const T*>(p.v);

    float m = -INFINITY, l = 0.f;
    float acc[D];
#pragma unroll
    for (int d = 0; d < D; ++d) acc[d] = 0.f;
    bool bad_block = false;
    for (int j = tid; j < S; j += 256) {
        const bool visible = j < P || ((mask >> (j - P)) & 1ull);
        if (!visible) continue;
        const int64_t off = kv_row_offset(p.g, b, hk, j, bad_block);
        float dot = 0.f;
#pragma unroll
        for (int c = 0; c < D / VEC; ++c) {
            float kk[VEC];
            load16<T>(kbase + off + c * VEC, kk);
#pragma unroll
            for (int e = 0; e < VEC; ++e) dot = fmaf(s_q[c * VEC + e], kk[e], dot);
        }
        const float s = dot * p.scale;
        const float m_new = fmaxf(m, s);
        const float alpha = expf(m - m_new);          // exp(-inf) = 0 on the first key
        const float w = expf(s - m_new);
        l = l * alpha + w;
#pragma unroll
        for (int c = 0; c < D / VEC; ++c) {
            float vv[VEC];
            load16<T>(vbase + off + c * VEC, vv);
#pragma unroll
            for (int e = 0; e < VEC; ++e) acc[c * VEC + e] = fmaf(w, vv[e], acc[c * VEC + e] * alpha);
        }
        m = m_new;
    }
    if (bad_block && p.err_flag) atomicOr(p.err_flag, SPECVLM_ERR_BAD_BLOCK);
    // merge the 256 private states: common max, rescale, sum
    float M = m;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) M = fmaxf(M, __shfl_xor(M, off));
    const int wave = tid >> 6, lane = tid & 63;
    if (lane == 0) s_m[wave] = M;
    __syncthreads();
    M = fmaxf(fmaxf(s_m[0], s_m[1]), fmaxf(s_m[2], s_m[3]));   // finite: node i always sees itself
    const float w = m == -INFINITY ? 0.f : expf(m - M);
    float lw = l * w;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) lw += __shfl_xor(lw, off);
    if (lane == 0) s_l[wave] = lw;
#pragma unroll
    for (int d = 0; d < D; ++d) {
        float x = acc[d] * w;
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) x += __shfl_xor(x, off);
        if (lane == 0) s_red[wave][d] = x;
    }
    __syncthreads();
    const float Z = (s_l[0] + s_l[1]) + (s_l[2] + s_l[3]);
    T* o = static_cast<T*>(p.o) + b * p.o_sb + i * p.o_sn + h * p.o_sh;
    if (tid < D) {
        const float x = (s_red[0][tid] + s_red[1][tid]) + (s_red[2][tid] + s_red[3][tid]);
        store_elem(o + tid, x / Z);
    }
    if (tid == 0 && p.lse) p.lse[(static_cast<int64_t>(b) * p.H_q + h) * p.N_max + i] = M + logf(Z);
}

int32_t launch_attn_valu(const AttnArgs& a) {
    const specvlm_attn_desc& d = a.d;
    ValuParams p;
    p.g = KvGeom{d.kv_stride_b, d.kv_stride_h, d.kv_stride_t, d.paged ? a.block_table : nullptr,
                 d.max_blocks_per_req, d.num_blocks,
                 d.paged ? d.max_blocks_per_req * SPECVLM_PAGE_SIZE : d.kv_capacity};
    p.N_max = d.N_max; p.H_q = d.H_q; p.group = d.H_q / d.H_kv; p.scale = a.scale;
    p.q = a.q; p.k = a.k; p.v = a.v; p.o = a.o; p.lse = a.lse;
    p.q_sb = d.q_stride_b; p.q_sn = d.q_stride_n; p.q_sh = d.q_stride_h;
    p.o_sb = d.o_stride_b; p.o_sn = d.o_stride_n; p.o_sh = d.o_stride_h;
    p.prefix_len = a.prefix_len; p.num_nodes = a.num_nodes; p.parent = a.parent;
    p.err_flag = a.err_flag;
    dim3 grid(d.N_max, d.H_q, d.B), block(256);
    if (d.dtype == SPECVLM_F32) {
        if (d.D == 64) hipLaunchKernelGGL((attn_valu_kernel<float, 64>), grid, block, 0, a.stream, p);
        else hipLaunchKernelGGL((attn_valu_kernel<float, 128>), grid, block, 0, a.stream, p);
    } else {
        if (d.D == 64) hipLaunchKernelGGL((attn_valu_kernel<uint16_t, 64>), grid, block, 0, a.stream, p);
        else hipLaunchKernelGGL((attn_valu_kernel<uint16_t, 128>), grid, block, 0, a.stream, p);
    }
    return check_launch();
}

}  // namespace specvlm
