// Tree-masked verification attention for bf16 caches on the gfx950 matrix cores.
//
// The step is bound by streaming K and V once from HBM (SpecVLM Sec. 3.2); all (up to 64)
// tree queries of a head share that single pass.  Work decomposition:
//
//   grid      one workgroup (4 wavefronts) per (request, query head, key-range split)
//   tiles     the workgroup walks its key range in 64-key tiles.  All 256 threads fetch a
//             tile with fully coalesced 16-byte loads (one 256-byte K or V row per 16
//             lanes), two tiles ahead, into registers, and park it in a double-buffered
//             LDS stage from which the four wavefronts read it: every K/V byte leaves HBM
//             and L2 exactly once
//   queries   wavefront w owns query rows 16w..16w+15 for the whole key range, so its
//             accumulator is only 16 x D and needs no merge inside the workgroup
//   QK^T      S^T[64 keys x 16 q] = K . Q^T with v_mfma_f32_16x16x32_bf16; the K stage is
//             XOR-swizzled so the operand reads (16 different rows per 16 lanes) are free
//             of bank conflicts
//   softmax   online (running max / sum per query) in fp32 on the S^T fragments: a lane
//             holds one query and 16 keys, so row statistics need two cross-lane steps,
//             and exp2(S^T) packed to bf16 is already the B operand of the next MFMA
//   PV        O^T[D x 16 q] += V^T . P^T; V rows are read from LDS as rows and transposed
//             two bytes at a time with v_perm_b32 (the contraction index may be permuted
//             freely, so an operand's "8 consecutive k" are 8 rows of one column)
//   masks     prefix keys need none; only tiles touching the tree region or the end of the
//             range test the per-query ancestor bit mask (select, never multiply: masked
//             slots may hold anything)
//   splits    fp32 partials go to a lane-major workspace; the last workgroup of a
//             (request, head) to finish -- found with a ticket counter -- merges them
#include <stdlib.h>

#include "common.hpp"

namespace specvlm {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kWaves = 4;
constexpr int kThreads = kWaves * 64;
constexpr int kQRows = 64;          // padded query rows: 16 per wavefront
constexpr int kTile = 64;           // keys per tile
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr size_t kCounterAlign = 256;

struct MfmaParams {
    KvGeom g;
    int N_max, H_q, group, num_splits;
    float scale;                // softmax scale
    const uint16_t *q, *k, *v;
    uint16_t* o;
    float* lse;
    int64_t q_sb, q_sn, q_sh, o_sb, o_sn, o_sh;
    const int32_t *prefix_len, *num_nodes, *parent;
    int32_t* err_flag;
    int32_t* ws_cnt;            // [B*H_q] arrival tickets, zero between calls
    float* ws_acc;              // [B*H_q*num_splits][4 qb][NT][64 lanes] f32x4
    float* ws_ml;               // [B*H_q*num_splits][64 q][2] (max, sum)
    int dbg;
};

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    f32x2 f = {lo, hi};
    bf16x2 h = __builtin_convertvector(f, bf16x2);      // v_cvt_pk_bf16_f32, round to nearest even
    return __builtin_bit_cast(uint32_t, h);
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Writes one wavefront's 16 query rows: out[t][i] = O^T[d = NT*(4g+i) + t][q], unnormalised.
template <int NT>
__device__ __forceinline__ void store_rows(const MfmaParams& p, const f32x4 (&out)[NT], float M, float L,
                                           int b, int h, int qi, int g, int n) {
    if (qi >= n) return;
    const float inv = 1.f / L;
    uint16_t* orow = p.o + b * p.o_sb + qi * p.o_sn + h * p.o_sh + 4 * NT * g;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        uint32_t w[NT / 2];
#pragma unroll
        for (int t = 0; t < NT; t += 2) w[t / 2] = pack_bf16x2(out[t][i] * inv, out[t + 1][i] * inv);
        if constexpr (NT == 8)
            *reinterpret_cast<u32x4*>(orow + i * NT) = u32x4{w[0], w[1], w[2], w[3]};
        else
            *reinterpret_cast<u32x2*>(orow + i * NT) = u32x2{w[0], w[1]};
    }
    if (p.lse && g == 0)
        p.lse[(static_cast<int64_t>(b) * p.H_q + h) * p.N_max + qi] = M * p.scale + __log2f(L) * kLn2;
}

template <int D>
__global__ __launch_bounds__(kThreads) void attn_mfma_kernel(MfmaParams p) {
    constexpr int NC = D / 32;                 // QK^T contraction steps of 32
    constexpr int NT = D / 16;                 // PV output row blocks (O^T rows = head dim)
    constexpr int ROWG = D / 8;                // 16-byte granules per K/V row
    constexpr int RPL = kThreads / ROWG;       // rows covered by one load of the workgroup (16 or 32)
    constexpr int LD = kTile / RPL;            // loads per thread per tile, for K and again for V
    constexpr int kStageBytes = kTile * D * 2; // one K (or V) tile

    __shared__ __attribute__((aligned(16))) unsigned char s_k[2][kStageBytes];
    __shared__ __attribute__((aligned(16))) unsigned char s_v[2][kStageBytes];
    __shared__ int s_par[SPECVLM_MAX_NODES];
    __shared__ int s_flag;

    // Workgroups are dealt round-robin to the 8 XCDs; give each XCD a contiguous range of work
    // items so that all splits of a (request, head) share one L2 (their partials meet there).
    int work = blockIdx.x;
    if ((gridDim.x & 7) == 0) work = (blockIdx.x & 7) * (gridDim.x >> 3) + (blockIdx.x >> 3);
    const int split = work % p.num_splits;
    const int bh = work / p.num_splits;
    const int h = bh % p.H_q, b = bh / p.H_q;
    const int hk = h / p.group;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l16 = lane & 15, g = lane >> 4;

    int err = 0;
    int n = p.num_nodes ? p.num_nodes[b] : p.N_max;
    const int P = p.prefix_len[b];
    if (n < 1 || n > p.N_max) err |= SPECVLM_ERR_BAD_NUM_NODES;
    n = min(max(n, 1), p.N_max);
    if (P < 0 || P + n > p.g.capacity) err |= SPECVLM_ERR_BAD_LENGTH;
    if (tid == 0) s_flag = 0;
    __syncthreads();
    if (tid < SPECVLM_MAX_NODES) {
        int par = -1;
        if (tid < n) {
            par = p.parent[b * p.N_max + tid];
            if (tid == 0 ? par != -1 : (par < 0 || par >= tid)) s_flag = SPECVLM_ERR_BAD_PARENT;
        }
        s_par[tid] = par;
    }
    __syncthreads();
    err |= s_flag;
    if (err) {                                  // uniform over the workgroup (and over its splits)
        if (tid == 0 && p.err_flag) atomicOr(p.err_flag, err);
        return;
    }
    const int S = P + n;
    const int nblk = (S + 15) >> 4;                                  // 16-key blocks of this request
    const int per = (nblk + p.num_splits - 1) / p.num_splits;
    const int blk0 = split * per;
    const int blk1 = min(nblk, blk0 + per);                          // this workgroup: blocks [blk0, blk1)
    const int ntile = blk1 > blk0 ? (blk1 - blk0 + 3) >> 2 : 0;      // 64-key tiles (the last may be partial)

    const uint16_t* kbase = p.k + hk * p.g.stride_h;
    const uint16_t* vbase = p.v + hk * p.g.stride_h;
    const float c2 = p.scale * kLog2e;

    // ---- tile fetch: thread -> (row, 16-byte granule); a 16-key block is one load (D=128)
    //      or half a load (D=64) of the workgroup ------------------------------------------
    const int lrow = tid / ROWG, lgran = tid % ROWG;
    auto issue = [&](int tile, u32x4 (&kb)[LD], u32x4 (&vb)[LD]) {
#pragma unroll
        for (int i = 0; i < LD; ++i) {
            const int r = i * RPL + lrow;                             // row within the tile
            const int blk = min(blk0 + 4 * tile + (r >> 4), blk1 - 1);  // past the range: re-read, masked later
            const int rr = min(r & 15, S - 1 - blk * 16);             // rows past the request's end: clamp
            int64_t off;
            if (p.g.block_table) {
                int phys = p.g.block_table[static_cast<int64_t>(b) * p.g.max_blocks + blk];
                phys = min(max(phys, 0), p.g.num_blocks - 1);
                off = phys * p.g.stride_b + rr * p.g.stride_t;
            } else {
                off = b * p.g.stride_b + (static_cast<int64_t>(blk) * 16 + rr) * p.g.stride_t;
            }
            off += lgran * 8;
            kb[i] = *reinterpret_cast<const u32x4*>(kbase + off);
            vb[i] = *reinterpret_cast<const u32x4*>(vbase + off);
        }
    };
    auto park = [&](int stage, const u32x4 (&kb)[LD], const u32x4 (&vb)[LD]) {
#pragma unroll
        for (int i = 0; i < LD; ++i) {
            const int r = i * RPL + lrow;
            *reinterpret_cast<u32x4*>(s_k[stage] + (r * ROWG + (lgran ^ (r & (ROWG - 1)))) * 16) = kb[i];
            *reinterpret_cast<u32x4*>(s_v[stage] + (r * ROWG + lgran) * 16) = vb[i];
        }
    };

    u32x4 kbuf0[LD], vbuf0[LD], kbuf1[LD], vbuf1[LD];
    if (ntile > 0) issue(0, kbuf0, vbuf0);
    if (ntile > 1) issue(1, kbuf1, vbuf1);

    // ---- this wavefront's 16 query rows: Q fragments (B operand of S^T = K Q^T): lane
    //      (q = 16w + l16, g) holds d = 32c + 8g .. +7; rows past the node count are zero ----
    const int qi = wave * 16 + l16;
    const bool wave_active = wave * 16 < n;          // wavefronts without real rows only move data
    bf16x8 qf[NC];
#pragma unroll
    for (int c = 0; c < NC; ++c) {
        u32x4 w = {0u, 0u, 0u, 0u};
        if (qi < n) w = *reinterpret_cast<const u32x4*>(p.q + b * p.q_sb + qi * p.q_sn + h * p.q_sh + (4 * c + g) * 8);
        qf[c] = __builtin_bit_cast(bf16x8, w);
    }
    // ancestor-or-self mask of this lane's query row
    unsigned long long anc = 0;
    {
        int t = qi < n ? qi : -1;
        while (t != -1) {                       // parent[t] < t was checked: at most 64 steps
            anc |= 1ull << t;
            t = s_par[t];
        }
    }

    float m_run = -INFINITY, l_run = 0.f;
    f32x4 acc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};

    auto compute = [&](int tile, int stage) {
        const unsigned char* kt = s_k[stage];
        const unsigned char* vt = s_v[stage];
        // S^T = K Q^T: s[kb][i] = score of key 16kb + 4g + i (of this tile) against query qi
        f32x4 s[4];
#pragma unroll
        for (int kb = 0; kb < 4; ++kb) {
            f32x4 a = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int c = 0; c < NC; ++c) {
                const int r = kb * 16 + l16;
                const int u = 4 * c + g;
                const bf16x8 ka = *reinterpret_cast<const bf16x8*>(kt + (r * ROWG + (u ^ (r & (ROWG - 1)))) * 16);
                a = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka, qf[c], a, 0, 0, 0);
            }
            s[kb] = a;
        }
        // masks: only tiles that reach past the prefix or past this workgroup's range
        const int tb0 = blk0 + 4 * tile;
        const int slot0 = tb0 * 16;
        if (slot0 + kTile > P || tb0 + 4 > blk1) {
#pragma unroll
            for (int kb = 0; kb < 4; ++kb) {
                const bool blk_ok = tb0 + kb < blk1;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int slot = slot0 + kb * 16 + 4 * g + i;
                    const int rel = slot - P;
                    const bool vis = blk_ok && slot < S && (rel < 0 || ((anc >> (rel & 63)) & 1ull));
                    s[kb][i] = vis ? s[kb][i] : -INFINITY;
                }
            }
        }
        // online softmax
        float mx = fmaxf(fmaxf(fmaxf(s[0][0], s[0][1]), fmaxf(s[0][2], s[0][3])),
                         fmaxf(fmaxf(s[1][0], s[1][1]), fmaxf(s[1][2], s[1][3])));
        mx = fmaxf(mx, fmaxf(fmaxf(fmaxf(s[2][0], s[2][1]), fmaxf(s[2][2], s[2][3])),
                             fmaxf(fmaxf(s[3][0], s[3][1]), fmaxf(s[3][2], s[3][3]))));
        mx = fmaxf(mx, __shfl_xor(mx, 16));
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float m_new = fmaxf(m_run, mx);
        const float m_safe = m_new == -INFINITY ? 0.f : m_new;
        const float alpha = fast_exp2((m_run - m_safe) * c2);         // exp2(-inf) = 0
        m_run = m_new;
        const float mc = m_safe * c2;
        float pr[16];
        float sum = 0.f;
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            pr[j] = fast_exp2(fmaf(s[j >> 2][j & 3], c2, -mc));
            sum += pr[j];
        }
        l_run = l_run * alpha + sum;
        if (__any(alpha != 1.f)) {
#pragma unroll
            for (int t = 0; t < NT; ++t) acc[t] *= alpha;
        }
        // O^T += V^T P^T, 32 keys per MFMA: contraction slot 8g + j <-> key 32*half + 16*(j/4) + 4g + j%4
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            u32x4 pw;
#pragma unroll
            for (int x = 0; x < 4; ++x) pw[x] = pack_bf16x2(pr[half * 8 + 2 * x], pr[half * 8 + 2 * x + 1]);
            const bf16x8 pf = __builtin_bit_cast(bf16x8, pw);
            uint32_t vr[8][NT / 2];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int r = half * 32 + (j >> 2) * 16 + 4 * g + (j & 3);
                if constexpr (NT == 8) {
                    const u32x4 w = *reinterpret_cast<const u32x4*>(vt + (r * ROWG + l16) * 16);
                    vr[j][0] = w[0]; vr[j][1] = w[1]; vr[j][2] = w[2]; vr[j][3] = w[3];
                } else {
                    const u32x2 w = *reinterpret_cast<const u32x2*>(vt + r * ROWG * 16 + l16 * 8);
                    vr[j][0] = w[0]; vr[j][1] = w[1];
                }
            }
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                const uint32_t sel = (t & 1) ? 0x07060302u : 0x05040100u;
                u32x4 w;
                w[0] = __builtin_amdgcn_perm(vr[1][t >> 1], vr[0][t >> 1], sel);
                w[1] = __builtin_amdgcn_perm(vr[3][t >> 1], vr[2][t >> 1], sel);
                w[2] = __builtin_amdgcn_perm(vr[5][t >> 1], vr[4][t >> 1], sel);
                w[3] = __builtin_amdgcn_perm(vr[7][t >> 1], vr[6][t >> 1], sel);
                acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, w), pf, acc[t], 0, 0, 0);
            }
        }
    };

    // ---- main loop: stage t%2 is consumed while tile t+1 is parked and t+2, t+3 are in flight
    if (ntile > 0) {
        park(0, kbuf0, vbuf0);
        if (ntile > 2) issue(2, kbuf0, vbuf0);
    }
    __syncthreads();
    for (int t = 0; t < ntile; t += 2) {
        if (t + 1 < ntile) {
            park(1, kbuf1, vbuf1);
            if (t + 3 < ntile) issue(t + 3, kbuf1, vbuf1);
        }
        if (wave_active && !(p.dbg & 4)) compute(t, 0);
        __syncthreads();
        if (t + 1 < ntile) {
            if (t + 2 < ntile) {
                park(0, kbuf0, vbuf0);
                if (t + 4 < ntile) issue(t + 4, kbuf0, vbuf0);
            }
            if (wave_active && !(p.dbg & 4)) compute(t + 1, 1);
            __syncthreads();
        }
    }

    // ---- epilogue ---------------------------------------------------------------------------
    l_run += __shfl_xor(l_run, 16);
    l_run += __shfl_xor(l_run, 32);
    if (p.num_splits == 1) {
        if (wave_active) store_rows<NT>(p, acc, m_run, l_run, b, h, qi, g, n);
        return;
    }
    const int64_t part0 = static_cast<int64_t>(bh) * p.num_splits;
    if (p.dbg & 8) return;
    if (wave_active) {
        f32x4* dst = reinterpret_cast<f32x4*>(p.ws_acc) + ((part0 + split) * 4 + wave) * NT * 64;
#pragma unroll
        for (int t = 0; t < NT; ++t) dst[t * 64 + lane] = acc[t];
        if (g == 0) reinterpret_cast<float2*>(p.ws_ml)[(part0 + split) * kQRows + qi] = make_float2(m_run, l_run);
    }
    // the last workgroup of this (request, head) to arrive merges all partials
    if (p.dbg & 2) return;
    if (!(p.dbg & 1)) __threadfence();
    __syncthreads();
    if (tid == 0) {
        const int ticket = atomicAdd(p.ws_cnt + bh, 1);
        const int last = ticket == p.num_splits - 1;
        if (last) p.ws_cnt[bh] = 0;                 // every other split has already drawn its ticket
        s_flag = last;
    }
    __syncthreads();
    if (!s_flag || !wave_active) return;
    if (!(p.dbg & 1)) __threadfence();
    float M = -INFINITY;
    for (int s = 0; s < p.num_splits; ++s)
        M = fmaxf(M, __builtin_nontemporal_load(p.ws_ml + ((part0 + s) * kQRows + qi) * 2));
    const float m_safe = M == -INFINITY ? 0.f : M;
    float L = 0.f;
    f32x4 out[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) out[t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll 2
    for (int s = 0; s < p.num_splits; ++s) {
        const float* mlp = p.ws_ml + ((part0 + s) * kQRows + qi) * 2;
        const float ms = __builtin_nontemporal_load(mlp), ls = __builtin_nontemporal_load(mlp + 1);
        const float w = fast_exp2((ms - m_safe) * c2);
        L += ls * w;
        const f32x4* src = reinterpret_cast<const f32x4*>(p.ws_acc) + ((part0 + s) * 4 + wave) * NT * 64;
#pragma unroll
        for (int t = 0; t < NT; ++t) out[t] += __builtin_nontemporal_load(src + t * 64 + lane) * w;
    }
    store_rows<NT>(p, out, M, L, b, h, qi, g, n);
}

int32_t attn_mfma_pick_splits(const specvlm_attn_desc& d) {
    if (d.num_splits > 0) return min(d.num_splits, 64);
    const int cus = 256;
    const int bh = d.B * d.H_q;
    const int cap = d.paged ? d.max_blocks_per_req * SPECVLM_PAGE_SIZE : d.kv_capacity;
    // one workgroup per compute unit when a single request must fill the chip; a ragged
    // batch gets a finer grain so that the dispatcher can balance; never less than two
    // 64-key tiles per workgroup
    const int by_work = max(1, cap / (2 * kTile));
    int want = (cus + bh - 1) / bh;
    if (d.B > 1) want *= 4;
    return max(1, min(min(want, by_work), 64));
}

static size_t counter_bytes(const specvlm_attn_desc& d) {
    const size_t raw = static_cast<size_t>(d.B) * d.H_q * sizeof(int32_t);
    return (raw + kCounterAlign - 1) / kCounterAlign * kCounterAlign;
}

size_t attn_mfma_workspace_bytes(const specvlm_attn_desc& d) {
    const int splits = attn_mfma_pick_splits(d);
    if (splits == 1) return 0;
    const size_t parts = static_cast<size_t>(d.B) * d.H_q * splits;
    return counter_bytes(d) + parts * (static_cast<size_t>(kQRows) * d.D * 4 + kQRows * 8);
}

int32_t launch_attn_mfma(const AttnArgs& a) {
    const specvlm_attn_desc& d = a.d;
    MfmaParams p;
    p.g = KvGeom{d.kv_stride_b, d.kv_stride_h, d.kv_stride_t, d.paged ? a.block_table : nullptr,
                 d.max_blocks_per_req, d.num_blocks,
                 d.paged ? d.max_blocks_per_req * SPECVLM_PAGE_SIZE : d.kv_capacity};
    p.N_max = d.N_max; p.H_q = d.H_q; p.group = d.H_q / d.H_kv;
    p.num_splits = attn_mfma_pick_splits(d);
    p.scale = a.scale;
    p.q = static_cast<const uint16_t*>(a.q);
    p.k = static_cast<const uint16_t*>(a.k);
    p.v = static_cast<const uint16_t*>(a.v);
    p.o = static_cast<uint16_t*>(a.o);
    p.lse = a.lse;
    p.q_sb = d.q_stride_b; p.q_sn = d.q_stride_n; p.q_sh = d.q_stride_h;
    p.o_sb = d.o_stride_b; p.o_sn = d.o_stride_n; p.o_sh = d.o_stride_h;
    p.prefix_len = a.prefix_len; p.num_nodes = a.num_nodes; p.parent = a.parent;
    p.err_flag = a.err_flag;
    p.dbg = getenv("SPECVLM_DBG") ? atoi(getenv("SPECVLM_DBG")) : 0;
    const size_t parts = static_cast<size_t>(d.B) * d.H_q * p.num_splits;
    unsigned char* ws = static_cast<unsigned char*>(a.workspace);
    p.ws_cnt = reinterpret_cast<int32_t*>(ws);
    p.ws_acc = reinterpret_cast<float*>(ws + counter_bytes(d));
    p.ws_ml = p.ws_acc + parts * kQRows * d.D;
    const dim3 grid(static_cast<unsigned>(parts)), block(kThreads);
    if (d.D == 128) hipLaunchKernelGGL(attn_mfma_kernel<128>, grid, block, 0, a.stream, p);
    else hipLaunchKernelGGL(attn_mfma_kernel<64>, grid, block, 0, a.stream, p);
    return check_launch();
}

}  // namespace specvlm
