// Tree-masked verification attention for bf16 caches on the gfx950 matrix cores.
//
// The step is bound by streaming K and V once from HBM (SpecVLM Sec. 3.2); all (up to 64)
// tree queries of a head share that single pass.  Work decomposition:
//
//   grid      one workgroup (4 wavefronts) per (request, query head, key-range split)
//   wavefront owns whole 32-key tiles of the split (tile w, w+4, ...) and ALL 64 query
//             rows, so a K/V byte is loaded by exactly one wavefront and never re-read
//   QK^T      S^T[32 keys x 64 q] = K . Q^T with v_mfma_f32_16x16x32_bf16; K rows are
//             fetched with fully coalesced 16-byte loads and re-ordered into the MFMA
//             operand layout through a wavefront-private, XOR-swizzled LDS tile
//   softmax   online (running max / sum per query) in fp32 on the S^T fragments: in that
//             layout a lane holds one query and 8 keys, so row statistics need only two
//             cross-lane steps, and exp2(S^T) is already the B operand of the next MFMA
//   PV        O^T[D x 64 q] += V^T . P^T; V rows are loaded coalesced straight into
//             registers and transposed 2 bytes at a time with v_perm_b32 (the contraction
//             index may be permuted freely, so "8 consecutive k" = 8 rows of one column)
//   masks     prefix keys need none; only tiles touching the tree region / the tail test
//             the per-query ancestor bit mask (select, never multiply: masked slots may
//             hold anything)
//   merge     the 4 wavefronts are merged through LDS; splits are merged by a second
//             small kernel from fp32 partials kept in a lane-major workspace layout
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
constexpr int kQRows = 64;          // padded query rows (4 MFMA column blocks of 16)
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

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
    float* ws_acc;              // [B*H_q*num_splits][4 qb][NT][64 lanes] f32x4
    float* ws_ml;               // [B*H_q*num_splits][64 q][2] (max, sum)
};

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    f32x2 f = {lo, hi};
    bf16x2 h = __builtin_convertvector(f, bf16x2);      // v_cvt_pk_bf16_f32, round to nearest even
    return __builtin_bit_cast(uint32_t, h);
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Request-level checks shared by the split and the merge kernel.  Returns error bits.
__device__ __forceinline__ int request_shape(const MfmaParams& p, int b, int& n, int& P) {
    int err = 0;
    n = p.num_nodes ? p.num_nodes[b] : p.N_max;
    P = p.prefix_len[b];
    if (n < 1 || n > p.N_max) err |= SPECVLM_ERR_BAD_NUM_NODES;
    n = min(max(n, 1), p.N_max);
    if (P < 0 || P + n > p.g.capacity) err |= SPECVLM_ERR_BAD_LENGTH;
    return err;
}

template <int D>
__global__ __launch_bounds__(kThreads) void attn_mfma_split_kernel(MfmaParams p) {
    constexpr int NC = D / 32;            // QK^T contraction steps of 32
    constexpr int NT = D / 16;            // PV output row blocks (O^T rows = head dim)
    constexpr int ROWG = D / 8;           // 16-byte granules per K row
    constexpr int RPI = 64 / ROWG;        // K rows fetched by one wavefront load instruction
    constexpr int KLD = 32 / RPI;         // K load instructions per 32-key tile
    constexpr int VW = NT / 2;            // dwords per lane per V row (NT bf16)
    constexpr int kTileBytes = 32 * D * 2;

    __shared__ __attribute__((aligned(16))) unsigned char s_buf[kWaves * kTileBytes > kWaves * NT * 64 * 16
                                                                   ? kWaves * kTileBytes
                                                                   : kWaves * NT * 64 * 16];
    __shared__ __attribute__((aligned(16))) unsigned char s_q[kQRows * D * 2];
    __shared__ float s_m[kWaves][kQRows];
    __shared__ float s_l[kWaves][kQRows];
    __shared__ int s_par[SPECVLM_MAX_NODES];
    __shared__ int s_bad;

    const int split = blockIdx.x % p.num_splits;
    const int bh = blockIdx.x / p.num_splits;
    const int h = bh % p.H_q, b = bh / p.H_q;
    const int hk = h / p.group;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l16 = lane & 15, g = lane >> 4;

    int n, P;
    int err = request_shape(p, b, n, P);
    if (tid == 0) s_bad = 0;
    __syncthreads();
    if (tid < SPECVLM_MAX_NODES) {
        int par = -1;
        if (tid < n) {
            par = p.parent[b * p.N_max + tid];
            if (tid == 0 ? par != -1 : (par < 0 || par >= tid)) s_bad = SPECVLM_ERR_BAD_PARENT;
        }
        s_par[tid] = par;
    }
    __syncthreads();
    err |= s_bad;
    if (err) {                                  // uniform over the workgroup
        if (tid == 0 && p.err_flag) atomicOr(p.err_flag, err);
        return;
    }
    const int S = P + n;
    const int nblk = (S + 15) >> 4;                                  // 16-key blocks of this request
    const int per = (nblk + p.num_splits - 1) / p.num_splits;
    const int blk0 = split * per;
    const int blk1 = min(nblk, blk0 + per);                          // this workgroup: [blk0, blk1)
    const int ntile = blk1 > blk0 ? (blk1 - blk0 + 1) >> 1 : 0;      // 32-key tiles (last may be half)

    const uint16_t* kbase = p.k + hk * p.g.stride_h;
    const uint16_t* vbase = p.v + hk * p.g.stride_h;
    const float c2 = p.scale * kLog2e;

    // ---- per-wavefront tile fetch -------------------------------------------------------
    u32x4 kreg[KLD];
    uint32_t vnext[8][VW];
    auto block_offset = [&](int kb) -> int64_t {            // element offset of a 16-key block's row 0
        if (p.g.block_table) {
            int blk = p.g.block_table[static_cast<int64_t>(b) * p.g.max_blocks + kb];
            blk = min(max(blk, 0), p.g.num_blocks - 1);
            return blk * p.g.stride_b;
        }
        return b * p.g.stride_b + static_cast<int64_t>(kb) * 16 * p.g.stride_t;
    };
    auto issue_loads = [&](int tile) {
        const int kb0 = blk0 + 2 * tile;
        int64_t boff[2];
        int last_row[2];
#pragma unroll
        for (int x = 0; x < 2; ++x) {
            const int kb = min(kb0 + x, blk1 - 1);           // a block past the range is re-read, then masked
            boff[x] = block_offset(kb);
            last_row[x] = min(15, S - 1 - kb * 16);          // rows past the end of the request are clamped
        }
#pragma unroll
        for (int i = 0; i < KLD; ++i) {
            const int r = i * RPI + lane / ROWG;             // row within the tile, 0..31
            const int x = (i * RPI) >> 4;                    // which 16-key block (compile time)
            const int rr = min(r & 15, last_row[x]);
            const uint16_t* src = kbase + boff[x] + rr * p.g.stride_t + (lane % ROWG) * 8;
            kreg[i] = *reinterpret_cast<const u32x4*>(src);
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int x = j >> 2;
            const int rr = min(4 * g + (j & 3), last_row[x]);
            const uint16_t* src = vbase + boff[x] + rr * p.g.stride_t + l16 * NT;
            if constexpr (VW == 4) {
                u32x4 w = *reinterpret_cast<const u32x4*>(src);
                vnext[j][0] = w[0]; vnext[j][1] = w[1]; vnext[j][2] = w[2]; vnext[j][3] = w[3];
            } else {
                u32x2 w = *reinterpret_cast<const u32x2*>(src);
                vnext[j][0] = w[0]; vnext[j][1] = w[1];
            }
        }
    };

    if (wave < ntile) issue_loads(wave);

    // ---- Q tile -> LDS (B operand of S^T = K Q^T), same XOR swizzle as the K tile; rows
    //      past the node count are zero ---------------------------------------------------
#pragma unroll
    for (int i = 0; i < kQRows * ROWG / kThreads; ++i) {
        const int id = tid + i * kThreads;
        const int r = id / ROWG, u = id % ROWG;
        u32x4 w = {0u, 0u, 0u, 0u};
        if (r < n) w = *reinterpret_cast<const u32x4*>(p.q + b * p.q_sb + r * p.q_sn + h * p.q_sh + u * 8);
        *reinterpret_cast<u32x4*>(s_q + (r * ROWG + (u ^ (r & (ROWG - 1)))) * 16) = w;
    }
    // ---- ancestor-or-self masks of this lane's 4 query rows ------------------------------
    unsigned long long anc[4];
#pragma unroll
    for (int qb = 0; qb < 4; ++qb) {
        unsigned long long mask = 0;
        int t = qb * 16 + l16;
        if (t >= n) t = -1;
        while (t != -1) {                       // parent[t] < t was checked: at most 64 steps
            mask |= 1ull << t;
            t = s_par[t];
        }
        anc[qb] = mask;
    }

    __syncthreads();                                   // Q tile visible to all wavefronts
    float m_run[4], l_run[4];
    f32x4 acc[4][NT];
#pragma unroll
    for (int qb = 0; qb < 4; ++qb) {
        m_run[qb] = -INFINITY;
        l_run[qb] = 0.f;
#pragma unroll
        for (int t = 0; t < NT; ++t) acc[qb][t] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    unsigned char* kt = s_buf + wave * kTileBytes;           // this wavefront's K staging tile
    for (int tile = wave; tile < ntile; tile += kWaves) {
        // K: registers -> swizzled LDS tile; V: keep in registers
#pragma unroll
        for (int i = 0; i < KLD; ++i) {
            const int r = i * RPI + lane / ROWG;
            const int u = lane % ROWG;
            *reinterpret_cast<u32x4*>(kt + (r * ROWG + (u ^ (r & (ROWG - 1)))) * 16) = kreg[i];
        }
        uint32_t vcur[8][VW];
#pragma unroll
        for (int j = 0; j < 8; ++j)
#pragma unroll
            for (int w = 0; w < VW; ++w) vcur[j][w] = vnext[j][w];
        if (tile + kWaves < ntile) issue_loads(tile + kWaves);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

        // S^T = K Q^T
        f32x4 s[2][4];
        bf16x8 ka[2][NC];
#pragma unroll
        for (int x = 0; x < 2; ++x)
#pragma unroll
            for (int c = 0; c < NC; ++c) {
                const int r = x * 16 + l16;
                const int u = 4 * c + g;
                ka[x][c] = *reinterpret_cast<const bf16x8*>(kt + (r * ROWG + (u ^ (r & (ROWG - 1)))) * 16);
            }
#pragma unroll
        for (int qb = 0; qb < 4; ++qb) {
            bf16x8 qf[NC];
#pragma unroll
            for (int c = 0; c < NC; ++c) {
                const int r = qb * 16 + l16;
                const int u = 4 * c + g;
                qf[c] = *reinterpret_cast<const bf16x8*>(s_q + (r * ROWG + (u ^ (r & (ROWG - 1)))) * 16);
            }
#pragma unroll
            for (int x = 0; x < 2; ++x) {
                f32x4 a = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int c = 0; c < NC; ++c) a = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[x][c], qf[c], a, 0, 0, 0);
                s[x][qb] = a;
            }
        }
        __builtin_amdgcn_wave_barrier();

        // masks: only for tiles that reach past the prefix or past this workgroup's range
        const int kb0 = blk0 + 2 * tile;
        const int slot0 = kb0 * 16;
        if (slot0 + 32 > P || kb0 + 2 > blk1) {
#pragma unroll
            for (int x = 0; x < 2; ++x) {
                const bool blk_ok = kb0 + x < blk1;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int slot = slot0 + x * 16 + 4 * g + i;
                    const int rel = slot - P;
#pragma unroll
                    for (int qb = 0; qb < 4; ++qb) {
                        const bool vis = blk_ok && slot < S &&
                                         (rel < 0 || ((anc[qb] >> (rel & 63)) & 1ull));
                        s[x][qb][i] = vis ? s[x][qb][i] : -INFINITY;
                    }
                }
            }
        }

        // online softmax on the fragments; P^T fragments in bf16
        bf16x8 pf[4];
#pragma unroll
        for (int qb = 0; qb < 4; ++qb) {
            float mx = fmaxf(fmaxf(fmaxf(s[0][qb][0], s[0][qb][1]), fmaxf(s[0][qb][2], s[0][qb][3])),
                             fmaxf(fmaxf(s[1][qb][0], s[1][qb][1]), fmaxf(s[1][qb][2], s[1][qb][3])));
            mx = fmaxf(mx, __shfl_xor(mx, 16));
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            const float m_new = fmaxf(m_run[qb], mx);
            const float m_safe = m_new == -INFINITY ? 0.f : m_new;
            const float alpha = fast_exp2((m_run[qb] - m_safe) * c2);     // exp2(-inf) = 0
            m_run[qb] = m_new;
            const float mc = m_safe * c2;
            float pr[8];
            float sum = 0.f;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                pr[j] = fast_exp2(fmaf(s[j >> 2][qb][j & 3], c2, -mc));
                sum += pr[j];
            }
            l_run[qb] = l_run[qb] * alpha + sum;
            if (__any(alpha != 1.f)) {
#pragma unroll
                for (int t = 0; t < NT; ++t) acc[qb][t] *= alpha;
            }
            u32x4 w;
            w[0] = pack_bf16x2(pr[0], pr[1]);
            w[1] = pack_bf16x2(pr[2], pr[3]);
            w[2] = pack_bf16x2(pr[4], pr[5]);
            w[3] = pack_bf16x2(pr[6], pr[7]);
            pf[qb] = __builtin_bit_cast(bf16x8, w);
        }

        // O^T += V^T P^T
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const uint32_t sel = (t & 1) ? 0x07060302u : 0x05040100u;
            u32x4 w;
            w[0] = __builtin_amdgcn_perm(vcur[1][t >> 1], vcur[0][t >> 1], sel);
            w[1] = __builtin_amdgcn_perm(vcur[3][t >> 1], vcur[2][t >> 1], sel);
            w[2] = __builtin_amdgcn_perm(vcur[5][t >> 1], vcur[4][t >> 1], sel);
            w[3] = __builtin_amdgcn_perm(vcur[7][t >> 1], vcur[6][t >> 1], sel);
            const bf16x8 va = __builtin_bit_cast(bf16x8, w);
#pragma unroll
            for (int qb = 0; qb < 4; ++qb) acc[qb][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va, pf[qb], acc[qb][t], 0, 0, 0);
        }
    }

    // ---- merge the 4 wavefronts -----------------------------------------------------------
#pragma unroll
    for (int qb = 0; qb < 4; ++qb) {
        l_run[qb] += __shfl_xor(l_run[qb], 16);
        l_run[qb] += __shfl_xor(l_run[qb], 32);
        if (g == 0) s_m[wave][qb * 16 + l16] = m_run[qb];
    }
    __syncthreads();                                   // also: every wavefront is done with its K tile
    float M[4], L[4];
#pragma unroll
    for (int qb = 0; qb < 4; ++qb) {
        const int qi = qb * 16 + l16;
        M[qb] = fmaxf(fmaxf(s_m[0][qi], s_m[1][qi]), fmaxf(s_m[2][qi], s_m[3][qi]));
        const float m_safe = M[qb] == -INFINITY ? 0.f : M[qb];
        const float w = fast_exp2((m_run[qb] - m_safe) * c2);
        l_run[qb] *= w;
#pragma unroll
        for (int t = 0; t < NT; ++t) acc[qb][t] *= w;
        if (g == 0) s_l[wave][qi] = l_run[qb];
    }
    f32x4* red = reinterpret_cast<f32x4*>(s_buf);      // [wave][t][lane]
    f32x4 out[NT];
#pragma unroll
    for (int qb = 0; qb < 4; ++qb) {
#pragma unroll
        for (int t = 0; t < NT; ++t) red[(wave * NT + t) * 64 + lane] = acc[qb][t];
        __syncthreads();
        if (wave == qb) {
#pragma unroll
            for (int t = 0; t < NT; ++t)
                out[t] = (red[(0 * NT + t) * 64 + lane] + red[(1 * NT + t) * 64 + lane]) +
                         (red[(2 * NT + t) * 64 + lane] + red[(3 * NT + t) * 64 + lane]);
        }
        __syncthreads();
    }
    // wavefront w now holds query block w: out[t][i] = O^T[d = NT*(4g+i) + t][q = 16w + l16]
    const int qi = wave * 16 + l16;
    const float Mq = wave == 0 ? M[0] : wave == 1 ? M[1] : wave == 2 ? M[2] : M[3];
    const float Lq = (s_l[0][qi] + s_l[1][qi]) + (s_l[2][qi] + s_l[3][qi]);
    if (p.num_splits == 1) {
        if (qi < n) {
            const float inv = 1.f / Lq;
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
                p.lse[(static_cast<int64_t>(b) * p.H_q + h) * p.N_max + qi] = Mq * p.scale + __log2f(Lq) * kLn2;
        }
    } else {
        const int64_t part = static_cast<int64_t>(bh) * p.num_splits + split;
        f32x4* dst = reinterpret_cast<f32x4*>(p.ws_acc) + (part * 4 + wave) * NT * 64;
#pragma unroll
        for (int t = 0; t < NT; ++t) dst[t * 64 + lane] = out[t];
        if (g == 0) {
            float2* ml = reinterpret_cast<float2*>(p.ws_ml) + part * kQRows + qi;
            *ml = make_float2(Mq, Lq);
        }
    }
}

// Merge of the key-range splits: one wavefront per (request, head, 16-query block), using
// the same lane layout the split kernel wrote (lane (q = l16, g) holds d = NT*(4g+i)+t).
template <int D>
__global__ __launch_bounds__(64) void attn_mfma_merge_kernel(MfmaParams p) {
    constexpr int NT = D / 16;
    const int qb = blockIdx.x & 3;
    const int bh = blockIdx.x >> 2;
    const int h = bh % p.H_q, b = bh / p.H_q;
    const int lane = threadIdx.x, l16 = lane & 15, g = lane >> 4;
    int n, P;
    if (request_shape(p, b, n, P)) return;
    // a malformed parent array made the split kernel skip this request: skip it here too
    bool bad = false;
    if (lane < n) {
        const int par = p.parent[b * p.N_max + lane];
        bad = lane == 0 ? par != -1 : (par < 0 || par >= lane);
    }
    if (__any(bad)) return;
    if (qb * 16 >= n) return;
    const int qi = qb * 16 + l16;
    const float c2 = p.scale * kLog2e;
    const int64_t part0 = static_cast<int64_t>(bh) * p.num_splits;
    float M = -INFINITY;
    for (int s = 0; s < p.num_splits; ++s)
        M = fmaxf(M, reinterpret_cast<const float2*>(p.ws_ml)[(part0 + s) * kQRows + qi].x);
    const float m_safe = M == -INFINITY ? 0.f : M;
    float L = 0.f;
    f32x4 out[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) out[t] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int s = 0; s < p.num_splits; ++s) {
        const float2 ml = reinterpret_cast<const float2*>(p.ws_ml)[(part0 + s) * kQRows + qi];
        const float w = fast_exp2((ml.x - m_safe) * c2);
        L += ml.y * w;
        const f32x4* src = reinterpret_cast<const f32x4*>(p.ws_acc) + ((part0 + s) * 4 + qb) * NT * 64;
#pragma unroll
        for (int t = 0; t < NT; ++t) out[t] += src[t * 64 + lane] * w;
    }
    if (qi < n) {
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
}

int32_t attn_mfma_pick_splits(const specvlm_attn_desc& d) {
    if (d.num_splits > 0) return min(d.num_splits, 64);
    const int cus = 256;
    const int bh = d.B * d.H_q;
    const int cap = d.paged ? d.max_blocks_per_req * SPECVLM_PAGE_SIZE : d.kv_capacity;
    // enough workgroups to cover every compute unit a few times over, but at least one
    // 32-key tile per wavefront of a workgroup
    int by_work = max(1, cap / (32 * kWaves));
    int want = (cus + bh - 1) / bh;
    if (d.B > 1) want *= 4;                 // ragged batches: finer grain so the dispatcher can balance
    return max(1, min(min(want, by_work), 64));
}

size_t attn_mfma_workspace_bytes(const specvlm_attn_desc& d) {
    const int splits = attn_mfma_pick_splits(d);
    if (splits == 1) return 256;
    const size_t parts = static_cast<size_t>(d.B) * d.H_q * splits;
    return parts * (static_cast<size_t>(kQRows) * d.D * 4 + kQRows * 8) + 256;
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
    const size_t parts = static_cast<size_t>(d.B) * d.H_q * p.num_splits;
    p.ws_acc = static_cast<float*>(a.workspace);
    p.ws_ml = p.ws_acc + parts * kQRows * d.D;
    const dim3 grid(static_cast<unsigned>(parts)), block(kThreads);
    if (d.D == 128) hipLaunchKernelGGL(attn_mfma_split_kernel<128>, grid, block, 0, a.stream, p);
    else hipLaunchKernelGGL(attn_mfma_split_kernel<64>, grid, block, 0, a.stream, p);
    int32_t rc = check_launch();
    if (rc || p.num_splits == 1) return rc;
    const dim3 mgrid(static_cast<unsigned>(d.B) * d.H_q * 4);
    if (d.D == 128) hipLaunchKernelGGL(attn_mfma_merge_kernel<128>, mgrid, dim3(64), 0, a.stream, p);
    else hipLaunchKernelGGL(attn_mfma_merge_kernel<64>, mgrid, dim3(64), 0, a.stream, p);
    return check_launch();
}

}  // namespace specvlm
