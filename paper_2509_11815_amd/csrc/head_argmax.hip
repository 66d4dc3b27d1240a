// Output head fused with the greedy choice (SpecVLM Fig. 3: one output head, shared by target
// and draft; Sec. 4.1: temperature 0): amax[b,i] = argmax_v sum_e hidden[b,i,e] * W[v,e], lowest
// token on ties, without ever storing the [nodes, vocabulary] logits.
//
// The head matrix is read exactly once per up to 512 node rows (262 MB for 32000 x 4096 bf16):
// the kernel is bound by streaming it from HBM, the products run on the matrix cores.
//
//   grid      (vocabulary tiles of 128 rows) x (groups of up to 8 blocks of 64 node rows).  A
//             workgroup is 8 wavefronts: wavefront (vs, nh) owns the 32 x 32 block (vocabulary
//             rows 32vs.., nodes 32nh..) of the tile's 128 x 64 logits of every node block,
//             16 accumulator registers per block
//   fetch     the contraction runs in chunks of 128 hidden units, every workgroup starting at a
//             different chunk (so that the loads in flight spread over all memory channels).  A
//             chunk is 128 rows of W and, per node block, 64 rows of hidden states, 256 bytes
//             each, brought into two three-slot LDS rings (a W chunk serves all node blocks
//             before the next one is consumed) by
//             direct-to-LDS loads (non-temporal for W, which is used once; the hidden states are
//             re-read by every workgroup and stay in L2); one load instruction moves four whole
//             rows, and lands them XOR-swizzled so that the operand reads are conflict-free.
//             Completion is tracked by hand with s_waitcnt vmcnt; one barrier per chunk
//             publishes the landed shares and frees the consumed slot
//   product   logits^T[vocab x node] += W . hidden^T with v_mfma_f32_16x16x32_bf16
//   epilogue  every lane orders its logits by (greater value, lower token) as one 64-bit key;
//             keys are maximised across lanes, wavefronts, and -- through a workspace and a
//             ticket counter -- across the vocabulary tiles by the last workgroup to arrive
#include <limits.h>

#include "common.hpp"

namespace specvlm {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kHeadThreads = 512;
constexpr int kVT = 128;                 // vocabulary rows per workgroup
constexpr int kMB = 64;                  // node rows per block
constexpr int kKC = 128;                 // hidden units per chunk (256-byte rows in LDS)
// Ring depths (slots).  One node block: W and its hidden-state chunk are consumed together, three
// slots each (two chunks ahead).  Several node blocks: a W chunk lives for NB steps, so two W slots
// (one chunk = NB >= 2 steps ahead) leave room for five hidden-state slots (four steps ahead).
template <int NB> struct HeadRing { static constexpr int kW = NB == 1 ? 3 : 2, kH = NB == 1 ? 3 : 5; };
constexpr int kWBytes = kVT * kKC * 2;   // 32 KB: a chunk of W
constexpr int kHBytes = kMB * kKC * 2;   // 16 KB: the same chunk of one block of 64 hidden-state rows
constexpr int kNIW = kVT / 4 / 4;        // load instructions per wavefront for a W chunk (4 rows each, wavefronts 0-3)
constexpr int kNIHid = kMB / 4 / 4;      // ... and for a hidden-state chunk (wavefronts 4-7)

struct HeadParams {
    const uint16_t* hidden;
    const uint16_t* W;
    int64_t h_stride_row;        // elements between consecutive (request, node) rows; rows are b*N_max + i
    int64_t w_stride_v;
    int M, E, V, N_max;
    const int32_t* num_nodes;
    int32_t* amax;
    float* max_logit;
    int32_t* ws_cnt;             // [node blocks] arrival tickets, zero between calls
    unsigned long long* ws_key;  // [node blocks][vocabulary tiles][64] best keys
};

__device__ __forceinline__ void head_dma(const void* sbase, uint32_t voff, uint32_t lds_dst, bool stream_once) {
    if (stream_once)
        asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1 nt"
                     : : "v"(voff), "s"(sbase), "s"(lds_dst) : "memory");
    else
        asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                     : : "v"(voff), "s"(sbase), "s"(lds_dst) : "memory");
}

template <int N>
__device__ __forceinline__ void head_wait_vmcnt() {
    asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N) : "memory");
}

// (logit, token) as one unsigned key ordered by "greater logit, then lower token"; -0 == +0.
__device__ __forceinline__ unsigned long long head_key(float v, int idx) {
    uint32_t u = __float_as_uint(v + 0.0f);
    u = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
    return (static_cast<unsigned long long>(u) << 32) | (0xFFFFFFFFu - static_cast<uint32_t>(idx));
}

__device__ __forceinline__ float head_key_value(unsigned long long k) {
    uint32_t u = static_cast<uint32_t>(k >> 32);
    u = (u & 0x80000000u) ? (u & 0x7FFFFFFFu) : ~u;
    return __uint_as_float(u);
}

// NB blocks of 64 node rows share one pass over W: a step is (chunk j of the hidden dimension,
// node block nb); the W chunk stays in its slot for NB steps while the blocks' hidden-state chunks
// go through their own ring.  W is requested two chunks, hidden states two steps ahead.
template <int NB>
__global__ __launch_bounds__(kHeadThreads) void head_argmax_kernel(HeadParams p) {
    constexpr int kWSlots = HeadRing<NB>::kW, kHSlots = HeadRing<NB>::kH;
    constexpr int LW = kWSlots - 1, LH = kHSlots - 1;      // chunks / steps requested ahead of the one consumed
    __shared__ __attribute__((aligned(1024))) unsigned char s_wring[kWSlots * kWBytes];
    __shared__ __attribute__((aligned(1024))) unsigned char s_hring[kHSlots * kHBytes];
    __shared__ unsigned long long s_key[8][kMB];
    __shared__ int s_flag;

    const int vt = blockIdx.x, nvt = gridDim.x;
    const int mb0 = blockIdx.y * NB;                       // first node block of this workgroup
    const int mblocks = (p.M + kMB - 1) / kMB;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int vs = wave & 3, nh = wave >> 2;
    const int l16 = lane & 15, g = lane >> 4;
    const int v0 = vt * kVT;
    const int nch = p.E / kKC;
    const int nsteps = nch * NB;

    typedef __attribute__((address_space(3))) unsigned char lds_byte;
    const uint32_t wring_lds = (uint32_t)(uintptr_t)(lds_byte*)s_wring;
    const uint32_t hring_lds = (uint32_t)(uintptr_t)(lds_byte*)s_hring;

    // ---- chunk fetch: load instruction i moves rows 4i .. 4i+3 (lane -> row lane/16, granule lane%16,
    // fetched from granule position ^ (row % 16)).  Wavefronts 0-3 fetch W (instructions 8*wave + ii),
    // wavefronts 4-7 the hidden states (instructions 4*(wave-4) + ii): loads complete in order within a
    // wavefront, so with the two kinds in different wavefronts a W chunk can be requested two chunks
    // ahead (HBM latency) while hidden-state chunks are requested two steps ahead (they come from L2).
    // Rows past the vocabulary / past the last node row re-read the last real row.
    const int lrow = lane >> 4, lpos = lane & 15;
    const bool w_issuer = wave < 4;                        // uniform
    const int iw = w_issuer ? wave : wave - 4;
    uint32_t voff_w[kNIW];
    const uint16_t* base_w[kNIW];
#pragma unroll
    for (int ii = 0; ii < kNIW; ++ii) {
        const int r = (kNIW * iw + ii) * 4 + lrow;                          // row of the tile
        const int r0 = min(v0 + (kNIW * iw + ii) * 4, p.V - 1);             // uniform: first row of the group, clamped
        const int rl = min(v0 + r, p.V - 1) - r0;                           // this lane's row relative to it (>= 0)
        base_w[ii] = p.W + static_cast<int64_t>(r0) * p.w_stride_v;
        voff_w[ii] = static_cast<uint32_t>(rl * p.w_stride_v * 2) + (lpos ^ (r & 15)) * 16;
    }
    // The j-th chunk a workgroup takes is chunk (j + rot) mod nch of the hidden dimension: if all
    // workgroups walked the columns of W in step, every load in flight on the chip would sit at the
    // same offset inside an 8 KB row, i.e. on a few of the memory channels (measured at 32000 x 4096:
    // 63 us without the rotation, 55 us with it -- the same as with W repacked into contiguous
    // 32 KB blocks; multipliers 1, 3, 11, 13 gave 56 us, 7 and 9 gave 58 - 62 us).
    const int rot = (5 * vt + vt / 8) % nch;
    auto chunk_of = [&](int j) { const int c = j + rot; return c >= nch ? c - nch : c; };
    auto issue_w = [&](int j) {                            // wavefronts 0-3: chunk j of W
        const uint32_t dst = wring_lds + (j % kWSlots) * kWBytes;
        const int c = chunk_of(j);
#pragma unroll
        for (int ii = 0; ii < kNIW; ++ii)
            head_dma(base_w[ii] + c * kKC, voff_w[ii], dst + (kNIW * iw + ii) * 1024, true);
    };
    auto issue_h = [&](int t) {                            // wavefronts 4-7: hidden states of step t = (chunk t / NB, block t % NB)
        const uint32_t dst = hring_lds + (t % kHSlots) * kHBytes;
        const int c = chunk_of(t / NB);
        const int m0 = (mb0 + t % NB) * kMB;
#pragma unroll
        for (int ii = 0; ii < kNIHid; ++ii) {
            const int r = (kNIHid * iw + ii) * 4 + lrow;
            const int r0 = min(m0 + (kNIHid * iw + ii) * 4, p.M - 1);        // uniform
            const int rl = min(m0 + r, p.M - 1) - r0;
            const uint32_t voff = static_cast<uint32_t>(rl * p.h_stride_row * 2) + (lpos ^ (r & 15)) * 16;
            head_dma(p.hidden + static_cast<int64_t>(r0) * p.h_stride_row + c * kKC, voff,
                     dst + (kNIHid * iw + ii) * 1024, false);
        }
    };
    // waits until at most `ahead` requests of this wavefront's kind (NI loads each) are outstanding
    auto wait_ahead = [&](int ahead) {
        if (w_issuer) {
            if (ahead >= 1 && LW >= 2) head_wait_vmcnt<kNIW>(); else head_wait_vmcnt<0>();
        } else {
            if (ahead >= 3 && LH >= 4) head_wait_vmcnt<3 * kNIHid>();
            else if (ahead == 2 && LH >= 3) head_wait_vmcnt<2 * kNIHid>();
            else if (ahead >= 1) head_wait_vmcnt<kNIHid>();
            else head_wait_vmcnt<0>();
        }
    };
    if (w_issuer) {
#pragma unroll
        for (int t = 0; t < LW; ++t)
            if (t < nch) issue_w(t);
        wait_ahead(min(LW, nch) - 1);                      // chunk 0 has landed
    } else {
#pragma unroll
        for (int t = 0; t < LH; ++t)
            if (t < nsteps) issue_h(t);
        wait_ahead(min(LH, nsteps) - 1);                   // step 0 has landed
    }
    __syncthreads();

    f32x4 acc[NB][2][2];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int x = 0; x < 2; ++x)
#pragma unroll
            for (int y = 0; y < 2; ++y) acc[nb][x][y] = f32x4{0.f, 0.f, 0.f, 0.f};

    for (int j = 0; j < nch; ++j) {
        const unsigned char* wt = s_wring + (j % kWSlots) * kWBytes;
        // A: lane (vocab row 32vs + 16x + l16, g) holds hidden units 32c + 8g .. +7 of the chunk
        bf16x8 wa[2][4];
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            const int s = j * NB + nb;
            // the slot a request goes to was last read before the barrier that ended the previous step:
            // hidden states of step s+LH replace those of step s-1, W chunk j+LW replaces chunk j-1
            if (w_issuer) {
                if (nb == 0 && j + LW < nch) issue_w(j + LW);
            } else if (s + LH < nsteps) {
                issue_h(s + LH);
            }
            if (nb == 0) {
#pragma unroll
                for (int x = 0; x < 2; ++x)
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        const int r = 32 * vs + 16 * x + l16;
                        wa[x][c] = *reinterpret_cast<const bf16x8*>(wt + (r * 16 + ((4 * c + g) ^ (r & 15))) * 16);
                    }
            }
            // B: lane (node 32nh + 16y + l16 of the block, g) holds the same units of that node's hidden state
            const unsigned char* ht = s_hring + (s % kHSlots) * kHBytes;
            bf16x8 hb[2][4];
#pragma unroll
            for (int y = 0; y < 2; ++y)
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const int r = 32 * nh + 16 * y + l16;
                    hb[y][c] = *reinterpret_cast<const bf16x8*>(ht + (r * 16 + ((4 * c + g) ^ (r & 15))) * 16);
                }
#pragma unroll
            for (int c = 0; c < 4; ++c)
#pragma unroll
                for (int x = 0; x < 2; ++x)
#pragma unroll
                    for (int y = 0; y < 2; ++y)
                        acc[nb][x][y] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wa[x][c], hb[y][c], acc[nb][x][y], 0, 0, 0);
            // this wavefront's reads of the slots have returned and its share of the next step's
            // loads has landed; the barrier extends both to the workgroup
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            // what the next step reads must have landed: its hidden states, and its W chunk when it starts one
            if (w_issuer) {
                if (nb == NB - 1) wait_ahead(min(j + LW, nch - 1) - (j + 1));
            } else {
                wait_ahead(min(s + LH, nsteps - 1) - (s + 1));
            }
            __syncthreads();
        }
    }

    // ---- epilogue: acc[nb][x][y][i] = logit of token v0 + 32vs + 16x + 4g + i at node row
    // (mb0 + nb)*64 + 32nh + 16y + l16.  Per node block: best key of the tile into the workspace.
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        if (mb0 + nb >= mblocks) break;                    // uniform
#pragma unroll
        for (int y = 0; y < 2; ++y) {
            unsigned long long best = 0;                   // 0 = no token (a real key is never 0)
#pragma unroll
            for (int x = 0; x < 2; ++x)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int v = v0 + 32 * vs + 16 * x + 4 * g + i;
                    const unsigned long long k = v < p.V ? head_key(acc[nb][x][y][i], v) : 0ull;
                    best = k > best ? k : best;
                }
            unsigned long long o = __shfl_xor(best, 16);
            best = o > best ? o : best;
            o = __shfl_xor(best, 32);
            best = o > best ? o : best;
            if (g == 0) s_key[vs + 4 * nh][16 * y + l16] = best;    // [vs][nh] x 32 nodes: index node within the half
        }
        __syncthreads();
        if (tid < kMB) {
            const int half = tid >> 5, within = tid & 31;
            unsigned long long best = s_key[4 * half][within];
#pragma unroll
            for (int w = 1; w < 4; ++w) {
                const unsigned long long o = s_key[w + 4 * half][within];
                best = o > best ? o : best;
            }
            // write-through: read by another workgroup in this kernel
            __hip_atomic_store(p.ws_key + (static_cast<int64_t>(mb0 + nb) * nvt + vt) * kMB + tid, best,
                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        __syncthreads();                                   // s_key is rewritten for the next block
    }
    head_wait_vmcnt<0>();                                  // the stores have been acknowledged
    __syncthreads();
    if (tid == 0) {                                        // one ticket per node block; bit nb: this workgroup is its last
        int flags = 0;
        for (int nb = 0; nb < NB && mb0 + nb < mblocks; ++nb) {
            int32_t* cnt = p.ws_cnt + mb0 + nb;
            const int ticket = __hip_atomic_fetch_add(cnt, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (ticket == nvt - 1) {
                __hip_atomic_store(cnt, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                flags |= 1 << nb;
            }
        }
        s_flag = flags;
    }
    __syncthreads();
    const int flags = s_flag;
    for (int nb = 0; nb < NB; ++nb) {
        if (!((flags >> nb) & 1)) continue;                // uniform
        const int mb = mb0 + nb;
        // The last workgroup of this node block reads the block's [tiles][64] keys: a thread takes two
        // neighbouring nodes (16 bytes) of every 16th tile, 16 device-coherent loads requested
        // back to back and waited for once (requested one by one, each costs a memory round
        // trip: 8.7 us for 250 tiles, against 1 us this way).  The compiler does not track these
        // loads; every register passes through an empty asm after the wait so that no use can
        // be scheduled before it.  Tile indices past the last tile are clamped: taking a key
        // twice does not change a maximum.
        {
            const int pair = tid & 31, slice = tid >> 5;
            const unsigned char* src = reinterpret_cast<const unsigned char*>(p.ws_key + static_cast<int64_t>(mb) * nvt * kMB);
            unsigned long long best0 = 0, best1 = 0;
            for (int t0 = 0; t0 < nvt; t0 += 256) {        // uniform
                u32x4 r[16];
#pragma unroll
                for (int u = 0; u < 16; ++u) {
                    const uint32_t voff = static_cast<uint32_t>(min(t0 + slice + 16 * u, nvt - 1)) * (kMB * 8) + pair * 16;
                    asm volatile("global_load_dwordx4 %0, %1, %2 sc1" : "=v"(r[u]) : "v"(voff), "s"(src) : "memory");
                }
                head_wait_vmcnt<0>();
#pragma unroll
                for (int u = 0; u < 16; ++u) {
                    asm volatile("" : "+v"(r[u]));
                    const unsigned long long k0 = (static_cast<unsigned long long>(r[u][1]) << 32) | r[u][0];
                    const unsigned long long k1 = (static_cast<unsigned long long>(r[u][3]) << 32) | r[u][2];
                    best0 = k0 > best0 ? k0 : best0;
                    best1 = k1 > best1 ? k1 : best1;
                }
            }
            // a wavefront holds two slices (lanes 0-31 and 32-63) of the same 32 node pairs
            unsigned long long o = __shfl_xor(best0, 32);
            best0 = o > best0 ? o : best0;
            o = __shfl_xor(best1, 32);
            best1 = o > best1 ? o : best1;
            if (lane < 32) {
                s_key[wave][2 * pair] = best0;
                s_key[wave][2 * pair + 1] = best1;
            }
        }
        __syncthreads();
        if (tid < kMB) {
            unsigned long long best = s_key[0][tid];
#pragma unroll
            for (int w = 1; w < 8; ++w) {
                const unsigned long long o = s_key[w][tid];
                best = o > best ? o : best;
            }
            const int row = mb * kMB + tid;
            if (row < p.M) {
                const int b = row / p.N_max, i = row % p.N_max;
                const int n = p.num_nodes ? p.num_nodes[b] : p.N_max;
                const bool real = i < n;
                p.amax[row] = real ? static_cast<int32_t>(0xFFFFFFFFu - static_cast<uint32_t>(best)) : -1;
                if (p.max_logit) p.max_logit[row] = real ? head_key_value(best) : 0.f;
            }
        }
        __syncthreads();                                   // s_key is rewritten for the next block
    }
}

static size_t head_counter_bytes(int mblocks) {
    return (static_cast<size_t>(mblocks) * sizeof(int32_t) + 255) / 256 * 256;
}

}  // namespace

size_t head_argmax_workspace_bytes(int32_t B, int32_t N_max, int32_t V) {
    const int M = B * N_max;
    const int mblocks = (M + kMB - 1) / kMB, nvt = (V + kVT - 1) / kVT;
    return head_counter_bytes(mblocks) + static_cast<size_t>(mblocks) * nvt * kMB * sizeof(unsigned long long);
}

int32_t launch_head_argmax(int32_t B, int32_t N_max, int32_t E, int32_t V, const void* hidden,
                           int64_t h_stride_row, const void* W, int64_t w_stride_v, const int32_t* num_nodes,
                           int32_t* amax, float* max_logit, void* workspace, hipStream_t stream) {
    HeadParams p;
    p.hidden = static_cast<const uint16_t*>(hidden);
    p.W = static_cast<const uint16_t*>(W);
    p.h_stride_row = h_stride_row;
    p.w_stride_v = w_stride_v;
    p.M = B * N_max; p.E = E; p.V = V; p.N_max = N_max;
    p.num_nodes = num_nodes;
    p.amax = amax;
    p.max_logit = max_logit;
    const int mblocks = (p.M + kMB - 1) / kMB, nvt = (V + kVT - 1) / kVT;
    unsigned char* ws = static_cast<unsigned char*>(workspace);
    p.ws_cnt = reinterpret_cast<int32_t*>(ws);
    p.ws_key = reinterpret_cast<unsigned long long*>(ws + head_counter_bytes(mblocks));
    // node blocks that share one pass over W: all of them up to 8
    const dim3 block(kHeadThreads);
    if (mblocks == 1) hipLaunchKernelGGL(head_argmax_kernel<1>, dim3(nvt, 1), block, 0, stream, p);
    else if (mblocks == 2) hipLaunchKernelGGL(head_argmax_kernel<2>, dim3(nvt, 1), block, 0, stream, p);
    else if (mblocks <= 4) hipLaunchKernelGGL(head_argmax_kernel<4>, dim3(nvt, 1), block, 0, stream, p);
    else hipLaunchKernelGGL(head_argmax_kernel<8>, dim3(nvt, (mblocks + 7) / 8), block, 0, stream, p);
    return check_launch();
}

}  // namespace specvlm
