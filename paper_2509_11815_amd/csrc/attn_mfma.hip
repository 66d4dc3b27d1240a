// Tree-masked verification attention for bf16 caches on the gfx950 matrix cores.
//
// The step is bound by streaming K and V once from HBM (SpecVLM Sec. 3.2); all (up to 64)
// tree queries of a head share that single pass.  Work decomposition:
//
//   grid      one workgroup (8 wavefronts, two per SIMD) per (request, query head, split).
//             A workgroup runs 2 independent key "streams"; stream s of the 2*splits streams
//             of a (request, head) owns the 32-key tiles s, s + 2*splits, ... (neighbouring
//             streams read neighbouring memory: measured 5 % faster than one contiguous chunk
//             per stream; a step costs the same whatever part of its tile is real, so cutting
//             the last round into equal shorter spans gained nothing).  Four wavefronts
//             share a stream: each takes 16 of the 64 query rows, so a K/V byte is fetched
//             from HBM exactly once and read from LDS four times.  Two wavefronts per SIMD
//             let one's matrix work overlap the other's softmax arithmetic and LDS latency
//   fetch     every stream keeps a private four-slot LDS ring filled by direct-to-LDS loads
//             (global_load_lds_dwordx4, non-temporal since the bytes are used once: no registers
//             are tied up by bytes in flight); one load
//             instruction moves four whole 256-byte rows, fully coalesced.  Each wavefront of
//             a stream requests 8 of a tile's 32 rows.  Two tiles per stream are in flight
//             ahead of the one consumed (64 KB per compute unit): with every compute unit
//             streaming the chip is saturated at that depth, more in flight measured
//             slower.  Completion is tracked by hand with
//             s_waitcnt vmcnt, and one workgroup barrier per tile publishes the landed
//             shares and frees the consumed slot.  With a contiguous cache a stream's first
//             tile is requested before the request's lengths have arrived
//   QK^T      S^T[32 keys x 64 q] = K . Q^T with v_mfma_f32_16x16x32_bf16; the lanes fetch
//             K granules in XOR-swizzled order so that the operand reads (16 different rows
//             per 16 lanes) are free of LDS bank conflicts; a wavefront's Q fragments stay in
//             registers for the whole kernel (staged once through the idle ring slot)
//   softmax   online (running max / sum per query) in fp32 on the S^T fragments: a lane
//             holds one query and 8 keys, so row statistics need two cross-lane steps, and
//             exp2(S^T) packed to bf16 is already the B operand of the next MFMA
//   PV        O^T[D x 64 q] += V^T . P^T; the V^T operand comes out of LDS transposed
//             (ds_read_b64_tr_b16 on V tiles swizzled in 32-byte chunks; the contraction
//             index may be permuted freely, so an operand's "8 consecutive k" are the 8
//             keys whose probabilities the lane already holds)
//   masks     prefix keys need none; only tiles touching the tree region or the request's
//             end test the per-query ancestor bit mask (select, never multiply)
//   merge     the streams of a workgroup are merged through LDS (one round, the rings are
//             free by then; 4 wavefronts each end up owning 16 query rows); the
//             workgroup's partial goes, as bf16, to a lane-major
//             workspace with write-through stores, and for every query block the last
//             split to arrive -- found with a ticket counter per (request, head, query
//             block) -- merges the splits, adding a split up while the next ones still load
#include <atomic>

#include "common.hpp"

namespace specvlm {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

// ds_read_b64_tr_b16: inside a block of 16 lanes, lane i receives element i % 4 of the four
// 8-byte rows whose addresses lanes i/4, i/4 + 4, i/4 + 8 and i/4 + 12 pass.
__device__ __forceinline__ s16x4 lds_read_tr16(const unsigned char* generic_lds_addr) {
    typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)generic_lds_addr);
}

constexpr int kWaves = 8;           // wavefronts per workgroup: two per SIMD
constexpr int kShare = 4;           // wavefronts sharing one key stream, 64/kShare query rows each
constexpr int kAhead = 2;           // tiles per stream kept in flight ahead of the one being consumed
constexpr int kStreamsPerWg = kWaves / kShare;
constexpr int kThreads = kWaves * 64;
constexpr int kQRows = 64;          // padded query rows: 4 MFMA column blocks of 16
constexpr int kTile = 32;           // keys per tile
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kTau = 8.0f;        // log2 of how far a probability may exceed 1 before the reference max moves
constexpr int kMaxSplitHeads = 1024;  // (request, head) pairs a split call can have: one set of ticket counters each
constexpr int kCounterStride = 32;    // int32 words from one ticket counter to the next: every counter has a 128-byte line of
                                      // its own (with the counters of eight heads in one line, 256 atomics queued up on it:
                                      // 17.1 -> 16.6 us per call at the 2880-visual-token prefix, 12.4 -> 11.3 us at 576)

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
    int32_t* ws_cnt;            // [B*H_q][4 query blocks] arrival tickets, kCounterStride words apart, zero between calls
    float* ws_acc;              // [B*H_q*num_splits][4 qb][NT/2][64 lanes] 16-byte vectors of packed bf16
    float* ws_ml;               // [B*H_q*num_splits][64 q][2] (max, sum)
};

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    f32x2 f = {lo, hi};
    bf16x2 h = __builtin_convertvector(f, bf16x2);      // v_cvt_pk_bf16_f32, round to nearest even
    return __builtin_bit_cast(uint32_t, h);
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// 16 bytes per lane from global memory straight into LDS at lds_dst + 16*lane (the LDS base
// travels in M0).  The compiler does not see the LDS write: every consumer sits behind
// wait_vmcnt<>() below, which is also a compiler memory barrier.
__device__ __forceinline__ void dma16(const void* gsrc, uint32_t lds_dst) {
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off nt"
                 :
                 : "v"(gsrc), "s"(lds_dst)
                 : "memory");
}

// Same with a wavefront-uniform base address and a 32-bit lane offset in bytes.
__device__ __forceinline__ void dma16s(const void* sbase, uint32_t voff, uint32_t lds_dst) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1 nt"
                 :
                 : "v"(voff), "s"(sbase), "s"(lds_dst)
                 : "memory");
}

// Same, 4 bytes per lane: lds_dst + 4*lane.
__device__ __forceinline__ void dma4(const void* gsrc, uint32_t lds_dst) {
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dword %0, off"
                 :
                 : "v"(gsrc), "s"(lds_dst)
                 : "memory");
}

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N) : "memory");
}

// The same for a count that is a constant only after loop unrolling (an even number up to 30).
__device__ __forceinline__ void wait_vmcnt_unrolled(int n) {
    switch (n) {
#define SPECVLM_WAIT_CASE(N) case N: wait_vmcnt<N>(); break;
        SPECVLM_WAIT_CASE(0) SPECVLM_WAIT_CASE(2) SPECVLM_WAIT_CASE(4) SPECVLM_WAIT_CASE(6) SPECVLM_WAIT_CASE(8)
        SPECVLM_WAIT_CASE(10) SPECVLM_WAIT_CASE(12) SPECVLM_WAIT_CASE(14) SPECVLM_WAIT_CASE(16) SPECVLM_WAIT_CASE(18)
        SPECVLM_WAIT_CASE(20) SPECVLM_WAIT_CASE(22) SPECVLM_WAIT_CASE(24) SPECVLM_WAIT_CASE(26) SPECVLM_WAIT_CASE(28)
        SPECVLM_WAIT_CASE(30)
#undef SPECVLM_WAIT_CASE
        default: wait_vmcnt<0>(); break;
    }
}

// Write-through (device-coherent) 16-byte store for data that another workgroup, possibly
// behind another L2, reads in the same kernel.
// (A store of more than 8 bytes reads its data registers for a cycle after it has issued: a
// vector instruction that overwrites them right behind it would corrupt the data of the last
// lanes.  The compiler pads its own stores; it cannot know that this asm is one, hence the s_nop.)
__device__ __forceinline__ void store16_coherent(void* dst, u32x4 v) {
    asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1\n\ts_nop 1" : : "v"(dst), "v"(v) : "memory");
}

__device__ __forceinline__ void store8_coherent(void* dst, u32x2 v) {
    asm volatile("global_store_dwordx2 %0, %1, off sc0 sc1" : : "v"(dst), "v"(v) : "memory");
}

// Writes one wavefront's 16 query rows: out[t][i] = O^T[d = 16t + 4g + i][q], unnormalised.
template <int NT>
__device__ __forceinline__ void store_rows(const MfmaParams& p, const f32x4 (&out)[NT], float M, float L,
                                           int b, int h, int qi, int g, int n) {
    if (qi >= n) return;
    const float inv = 1.f / L;
    // A lane holds 4 consecutive head dims per block t.  Lanes g = 2v and 2v+1 of a query row
    // trade halves so that each stores 8 consecutive dims (16 bytes): the even lane keeps the
    // even blocks, the odd lane the odd ones.
    const bool odd = g & 1;
    uint16_t* orow = p.o + b * p.o_sb + qi * p.o_sn + h * p.o_sh + 4 * (g & ~1);
#pragma unroll
    for (int u = 0; u < NT / 2; ++u) {
        const uint32_t e0 = pack_bf16x2(out[2 * u][0] * inv, out[2 * u][1] * inv);
        const uint32_t e1 = pack_bf16x2(out[2 * u][2] * inv, out[2 * u][3] * inv);
        const uint32_t o0 = pack_bf16x2(out[2 * u + 1][0] * inv, out[2 * u + 1][1] * inv);
        const uint32_t o1 = pack_bf16x2(out[2 * u + 1][2] * inv, out[2 * u + 1][3] * inv);
        const uint32_t r0 = __shfl_xor(odd ? e0 : o0, 16);     // the partner's share of the block this lane keeps
        const uint32_t r1 = __shfl_xor(odd ? e1 : o1, 16);
        const u32x4 w = odd ? u32x4{r0, r1, o0, o1} : u32x4{e0, e1, r0, r1};
        *reinterpret_cast<u32x4*>(orow + 16 * (2 * u + (odd ? 1 : 0))) = w;
    }
    if (p.lse && g == 0)
        p.lse[(static_cast<int64_t>(b) * p.H_q + h) * p.N_max + qi] = M * p.scale + __log2f(L) * kLn2;
}

// WQ wavefronts share a stream (2: 32 query rows each, 4 streams, 2 ring slots; 4: 16 query rows
// each, 2 streams, 4 ring slots); PD tiles per stream are kept in flight ahead of the one consumed.
// Measured on the 2880-visual-token workload: (WQ, PD) = (4, 2) 19.5 us per layer, (4, 3) 20.0,
// (4, 1) 20.8, (2, 1) 21.8; only (kShare, kAhead) is instantiated.
// Two launch shapes of the same body (attn_mfma_body.inc).
//   attn_mfma_kernel      128 KB of rings (four slots per stream, two tiles in flight ahead), one
//                         workgroup per compute unit: few (request, head) pairs, long streams
//   attn_mfma_kernel_2wg  64 KB of rings (two slots, one tile ahead) and at most 128 registers, so
//                         that two workgroups share a compute unit: twice as many (request, head,
//                         split) items are resident at once
template <int D, int WQ, int PD>
__global__ __launch_bounds__(kThreads) void attn_mfma_kernel(MfmaParams p) {
    constexpr int SL = WQ, MB = 8;
#include "attn_mfma_body.inc"
}

template <int D>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(4, 4))) void attn_mfma_kernel_2wg(MfmaParams p) {
    constexpr int WQ = kShare, PD = 1, SL = 2, MB = 3;
#include "attn_mfma_body.inc"
}

// Key-range splits per (request, head) when the caller leaves the choice to the library: the
// count that minimises a small cost model of the kernel on 256 compute units, one workgroup
// each.  A workgroup costs a fixed prologue + merge time plus one step per 32-key tile of its
// longest stream; a step takes the measured time of the loop body with two tiles in flight
// (the same with 160 or 256 units active), or the workgroup's share of HBM bandwidth if that
// is slower; workgroups beyond 256 run as further rounds.  The cache capacity stands in for
// the request lengths, which the host does not know.
int32_t attn_mfma_pick_splits(const specvlm_attn_desc& d) {
    const int64_t heads = static_cast<int64_t>(d.B) * d.H_q;
    if (heads > kMaxSplitHeads) return 1;      // more (request, head) pairs than ticket counters: that many fill the chip unsplit
    if (d.num_splits > 0) return min(d.num_splits, 64);
    const int cus = 256;
    const int bh = d.B * d.H_q;
    const int cap = d.paged ? d.max_blocks_per_req * SPECVLM_PAGE_SIZE : d.kv_capacity;
    const int ntile = (cap + kTile - 1) / kTile;
    const double step_bytes = static_cast<double>(kStreamsPerWg) * kTile * d.D * 2 * 2;   // K and V, bf16
    const double bw = 6.0e6;                                     // bytes per microsecond the loop sustains
    const double step_alone = d.D == 128 ? 1.35 : 0.9;           // microseconds per step of one compute unit by itself
    auto wg_time = [&](int splits, int active) {
        const int steps = (ntile + kStreamsPerWg * splits - 1) / (kStreamsPerWg * splits);
        const double step = fmax(step_alone, step_bytes * active / bw);
        return (splits > 1 ? 8.0 : 5.0) + steps * step;
    };
    const int most = max(1, min(64, ntile / kStreamsPerWg));     // never a stream without a whole tile
    int best = 1;
    double best_t = 1e30;
    for (int s = 1; s <= most; ++s) {
        const long wgs = static_cast<long>(bh) * s;
        const long full = wgs / cus;
        const int rest = static_cast<int>(wgs % cus);
        const double t = full * wg_time(s, cus) + (rest ? wg_time(s, rest) : 0.0);
        if (t < best_t * 0.999) { best_t = t; best = s; }
    }
    return best;
}

// The ticket counters occupy a region of fixed size at the start of the workspace, whatever the
// shape: a later call of another shape then finds its counters where every earlier call left
// zeros, never where one stored partial results.
static size_t counter_bytes(const specvlm_attn_desc&) { return static_cast<size_t>(kMaxSplitHeads) * 4 * kCounterStride * sizeof(int32_t); }

size_t attn_mfma_workspace_bytes(const specvlm_attn_desc& d) {
    const int splits = attn_mfma_pick_splits(d);
    if (splits == 1) return 0;
    const size_t parts = static_cast<size_t>(d.B) * d.H_q * splits;
    return counter_bytes(d) + parts * (static_cast<size_t>(kQRows) * d.D * 2 + kQRows * 8);
}

// ---- library-owned scratch for callers that cannot allocate device memory -----------------------
// One array per GPU (each device holds its own copy of the code object's globals, zero when the
// object is loaded).  Host code must not use the array's name as an address: the device address
// is asked for once per device and kept.
static __device__ __align__(256) unsigned char scratch[SPECVLM_STATIC_WORKSPACE_BYTES];

int32_t attn_static_workspace(void** ptr_out) {
    constexpr int kMaxDevices = 64;
    static std::atomic<void*> ptr_of_device[kMaxDevices];
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        note_hip_error(e != hipSuccess ? e : hipErrorInvalidDevice);
        return SPECVLM_HIP_ERROR;
    }
    void* ptr = ptr_of_device[dev].load(std::memory_order_acquire);
    if (!ptr) {
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));         // this device's copy (the current device)
        if (e != hipSuccess || !ptr) {
            note_hip_error(e != hipSuccess ? e : hipErrorInvalidSymbol);
            return SPECVLM_HIP_ERROR;
        }
        ptr_of_device[dev].store(ptr, std::memory_order_release);   // two threads racing here store the same address
    }
    *ptr_out = ptr;
    return SPECVLM_OK;
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
    unsigned char* ws = static_cast<unsigned char*>(a.workspace);
    p.ws_cnt = reinterpret_cast<int32_t*>(ws);
    p.ws_acc = reinterpret_cast<float*>(ws + counter_bytes(d));
    p.ws_ml = p.ws_acc + parts * kQRows * d.D / 2;
    const dim3 grid(static_cast<unsigned>(parts)), block(kThreads);
    // More work items than compute units, but no more than fit two to a unit: the second shape keeps
    // all of them resident at once instead of running a second, partly filled round (13B-shaped
    // batch of 4 with 3 splits, 480 items: 70.7 against 75.8 us; with 256 items or fewer the first
    // shape's deeper rings win: 16.5 against 23.3 us at the 2880-visual-token prefix).
    if (parts > 256 && parts <= 512) {
        if (d.D == 128) hipLaunchKernelGGL((attn_mfma_kernel_2wg<128>), grid, block, 0, a.stream, p);
        else hipLaunchKernelGGL((attn_mfma_kernel_2wg<64>), grid, block, 0, a.stream, p);
    } else {
        if (d.D == 128) hipLaunchKernelGGL((attn_mfma_kernel<128, kShare, kAhead>), grid, block, 0, a.stream, p);
        else hipLaunchKernelGGL((attn_mfma_kernel<64, kShare, kAhead>), grid, block, 0, a.stream, p);
    }
    return check_launch();
}

}  // namespace specvlm
