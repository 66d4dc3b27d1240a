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
__device__ __forceinline__ void store16_coherent(void* dst, u32x4 v) {
    asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1" : : "v"(dst), "v"(v) : "memory");
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
template <int D, int WQ, int PD>
__global__ __launch_bounds__(kThreads) void attn_mfma_kernel(MfmaParams p) {
    constexpr int kStreams = kWaves / WQ;      // key streams per workgroup, each with a private LDS ring
    constexpr int QBW = 4 / WQ;                // 16-row query blocks per wavefront
    constexpr int kSlots = WQ;                 // ring depth per stream (128 KB of rings in all for D = 128)
    constexpr int NC = D / 32;                 // QK^T contraction steps of 32
    constexpr int NT = D / 16;                 // PV output row blocks (O^T rows = head dim)
    constexpr int ROWG = D / 8;                // 16-byte granules per K/V row
    constexpr int RPI = 64 / ROWG;             // rows moved by one wavefront load (4 or 8)
    constexpr int KLD = kTile / RPI;           // load instructions per tile, for K and again for V
    constexpr int KPW = KLD / WQ;              // of which this wavefront issues KPW (its 32/WQ rows)
    constexpr int NI = 2 * KPW;                // load instructions per wavefront and tile
    constexpr int kTileBytes = kTile * D * 2;  // one K (or V) tile
    constexpr int kSlotBytes = 2 * kTileBytes; // K tile then V tile
    constexpr int kRingBytes = kSlots * kSlotBytes;
    constexpr int QW = 16 * QBW;               // query rows per wavefront
    static_assert(PD >= 1 && PD < kSlots, "a slot must be free for the tile being consumed");
    static_assert(kStreams * kRingBytes >= 4 * (kStreams - 1) * NT * 64 * 16, "merge scratch must fit in the rings");
    static_assert(QW * D * 2 == 2 * KPW * 1024, "a wavefront's Q rows fill exactly its two refill areas of one slot");

    __shared__ __attribute__((aligned(1024))) unsigned char s_ring[kStreams * kRingBytes];
    __shared__ float s_m[kStreams][kQRows];
    __shared__ float s_l[kStreams][kQRows];
    __shared__ int s_par[SPECVLM_MAX_NODES];

    // Workgroups are dealt round-robin to the 8 XCDs; give each XCD a contiguous range of work
    // items so that all splits of a (request, head) share one L2 (their partials meet there).
    int work = blockIdx.x;
    if ((gridDim.x & 7) == 0) work = (blockIdx.x & 7) * (gridDim.x >> 3) + (blockIdx.x >> 3);
    const int split = work % p.num_splits;
    const int bh = work / p.num_splits;
    const int h = bh % p.H_q, b = bh / p.H_q;
    const int hk = h / p.group;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int st = wave % kStreams;            // stream of the workgroup
    const int qw = wave / kStreams;            // query share: rows QW*qw .. QW*qw + QW-1
    const int l16 = lane & 15, g = lane >> 4;

    // Everything this kernel fetches between here and the epilogue goes through the hand-counted
    // direct-to-LDS loads: vmcnt is one in-order counter, so a compiler-managed vector load in
    // between would make the compiler's own wait drain every tile still in flight.  The two
    // request scalars come through the scalar cache (constant address space, uniform index).
    typedef const __attribute__((address_space(4))) int32_t* const_i32;
    const int n_raw = p.num_nodes ? ((const_i32)p.num_nodes)[b] : p.N_max;
    const int P_raw = ((const_i32)p.prefix_len)[b];
    const int nstream = kStreams * p.num_splits;
    const int stream = split * kStreams + st;

    unsigned char* ring = s_ring + st * kRingBytes;
    typedef __attribute__((address_space(3))) unsigned char lds_byte;
    const uint32_t ring_lds = (uint32_t)(uintptr_t)(lds_byte*)ring;      // LDS byte address of the ring

    // ---- tile fetch ------------------------------------------------------------------------
    // Load instruction i of a tile moves rows RPI*i .. RPI*i+RPI-1: lane -> (row, LDS granule
    // position); for K the lane fetches global granule position^(row % ROWG), so the tile
    // lands XOR-swizzled.  The address of a load is a wavefront-uniform 64-bit base (the first
    // row of the group, on the scalar ALU) plus a 32-bit lane offset that never changes (row
    // within the group, granule), so a refill costs a handful of scalar instructions; only a
    // group that reaches past the request's last key takes the slow path, where rows past that
    // key re-read its row (finite data that gets weight zero).
    const int lrow = lane / ROWG, lpos = lane % ROWG;
    const uint32_t row_bytes = static_cast<uint32_t>(p.g.stride_t) * 2u;      // (checked on the host: fits easily)
    uint32_t voff_k[KPW];                                  // lane offset of K load ii of this wavefront
#pragma unroll
    for (int ii = 0; ii < KPW; ++ii)
        voff_k[ii] = lrow * row_bytes + (lpos ^ (((qw * KPW + ii) * RPI + lrow) & (ROWG - 1))) * 16;
    // V tiles land swizzled in 32-byte chunks (16 head dims): chunk c of key row r sits at chunk
    // position c ^ vswz(r), so that the transposing reads of the PV product, which take 32 bytes
    // from each of 8 different rows per half wavefront, hit every LDS bank once.
    auto vswz = [](int r) { return D == 128 ? (r & 7) : ((r >> 1) & 3); };
    auto vgran = [&](int r) { return (((lpos >> 1) ^ vswz(r)) << 1) | (lpos & 1); };   // granule this lane fetches for row r
    uint32_t voff_v[KPW];
#pragma unroll
    for (int ii = 0; ii < KPW; ++ii)
        voff_v[ii] = lrow * row_bytes + vgran((qw * KPW + ii) * RPI + lrow) * 16;
    const int64_t head_off = hk * p.g.stride_h + (p.g.block_table ? 0 : b * p.g.stride_b);   // elements
    // A wavefront requests its 32/WQ rows of the stream's tile, K and V: KPW loads each, into the
    // two areas of the slot that only this wavefront ever fills.
    const uint32_t area = qw * KPW * 1024;                // this wavefront's area inside a K (or V) tile
    auto issue_rows = [&](int j, int lim, const int (&phys)[2]) __attribute__((always_inline)) {   // lim: first row that must not be fetched
        const uint32_t dst = ring_lds + (j % kSlots) * kSlotBytes;
        const int lo = (stream + j * nstream) * kTile;                   // first key
#pragma unroll
        for (int ii = 0; ii < KPW; ++ii) {
            const int i = qw * KPW + ii;
            int r0 = lo + i * RPI;                         // uniform: first row of the group
            uint32_t vk = voff_k[ii], vv = voff_v[ii];
            if (r0 + RPI > lim) {                          // uniform, rare: some row of the group is not real
                r0 = min(r0, ((lim - 1) / RPI) * RPI);     // the last group with a real row
                const uint32_t rl = min(lrow, lim - 1 - r0) * row_bytes;
                vk = rl + (lpos ^ ((i * RPI + lrow) & (ROWG - 1))) * 16;
                vv = rl + vgran(i * RPI + lrow) * 16;
            }
            int64_t base = head_off;                       // elements, uniform
            if (p.g.block_table) {
                // the group's block is block (i*RPI)/16 of the tile, or the request's last block when clamped
                const int id = min(max(phys[(i * RPI) >> 4], 0), p.g.num_blocks - 1);
                base += id * p.g.stride_b + (r0 & 15) * p.g.stride_t;
            } else {
                base += static_cast<int64_t>(r0) * p.g.stride_t;
            }
            dma16s(p.k + base, vk, dst + i * 1024);
            dma16s(p.v + base, vv, dst + kTileBytes + i * 1024);
        }
    };
    // The stream's first tile is requested before the request's lengths are known (they arrive
    // through the scalar cache half a microsecond into the kernel): with a contiguous cache its
    // address needs nothing else, and a tile inside the cache's capacity is memory that may be
    // read.  If the lengths then show that the tile is not entirely real, it is requested again
    // the ordinary way (rows past the last key re-read that key's row).
    // (Sending the query rows out early as well made the call slower: 17.2 against 17.0 us.)
    int phys[2] = {0, 0};
    const bool early = !p.g.block_table && (stream + 1) * kTile <= p.g.capacity;     // uniform
    if (early) issue_rows(0, p.g.capacity, phys);
    int err = 0;
    int n = n_raw;
    const int P = P_raw;
    if (n < 1 || n > p.N_max) err |= SPECVLM_ERR_BAD_NUM_NODES;
    n = min(max(n, 1), p.N_max);
    if (P < 0 || P + n > p.g.capacity) err |= SPECVLM_ERR_BAD_LENGTH;
    const int S = P + n;
    const int ntile = (S + kTile - 1) / kTile;                       // 32-key tiles of this request
    // tiles stream, stream + nstream, ... ; none when the lengths are bad (nothing more may be fetched then)
    const int my_tiles = (!err && stream < ntile) ? (ntile - stream + nstream - 1) / nstream : 0;
    // the workgroup's first stream has the most tiles: the (uniform) trip count of the main loop
    const int wg_tiles = (!err && split * kStreams < ntile) ? (ntile - split * kStreams + nstream - 1) / nstream : 0;
    // the early request is the stream's first tile if that tile exists and every row of it is real
    const bool first_done = early && my_tiles > 0 && (stream + 1) * kTile <= S;
    if (early && !first_done) wait_vmcnt<0>();          // rare: let it land (unused rows of the slot), then go on as without it
    auto issue_part = [&](int j, const int (&ph)[2]) __attribute__((always_inline)) { issue_rows(j, S, ph); };
    // Paged cache: physical ids of the two 16-key blocks of a tile, through the scalar cache.
    // They are looked up one tile ahead of the loads that need them, so the look-up latency
    // never sits between a free ring slot and its refill.
    bool bad_block = false;                     // uniform per wavefront: an id outside the pool was looked up (and clamped)
    auto fetch_blocks = [&](int j, int (&phys)[2]) {
        if (!p.g.block_table) return;
        const int blk0 = (stream + j * nstream) * (kTile >> 4), last_blk = (S - 1) >> 4;
#pragma unroll
        for (int x = 0; x < 2; ++x) {
            phys[x] = ((const_i32)p.g.block_table)[static_cast<int64_t>(b) * p.g.max_blocks + min(blk0 + x, last_blk)];
            bad_block = bad_block || phys[x] < 0 || phys[x] >= p.g.num_blocks;
        }
    };
    typedef __attribute__((address_space(3))) int lds_int;
    // Next in the queue: the parent array (wavefront 0; lanes past N_max re-read its last entry),
    // which is waited for on its own, so that the tree is checked and the ancestor masks are built
    // while the tiles are still in flight.  Then, unless it went out early, this wavefront's share
    // of the first tile, and its query rows -- staged in the ring's last slot, first half of the
    // rows in this wavefront's K area, second half in its V area, the two areas only this
    // wavefront refills later, so no other wavefront can overwrite them before they are read.
    // Those are what the first step needs; the tiles further ahead come after.
    if (wave == 0)
        dma4(p.parent + static_cast<int64_t>(b) * p.N_max + min(lane, p.N_max - 1),
             (uint32_t)(uintptr_t)(lds_int*)s_par);
    if (my_tiles > 0 && !first_done) { fetch_blocks(0, phys); issue_part(0, phys); }
    // this wavefront's QW query rows (B operand of S^T = K Q^T), XOR-swizzled like the K tiles; rows
    // past the node count re-read the last real row (their columns of S^T are never stored)
    constexpr uint32_t kStage = (kSlots - 1) * kSlotBytes;
#pragma unroll
    for (int i = 0; i < 2 * KPW; ++i) {
        const int r = qw * QW + i * RPI + lrow;                          // query row
        const uint16_t* src = p.q + b * p.q_sb + static_cast<int64_t>(min(r, n - 1)) * p.q_sn + h * p.q_sh +
                              (lpos ^ (r & (ROWG - 1))) * 8;
        dma16(src, ring_lds + kStage + (i / KPW) * kTileBytes + area + (i % KPW) * 1024);
    }
#pragma unroll
    for (int t = 1; t < PD; ++t)
        if (t < my_tiles) { fetch_blocks(t, phys); issue_part(t, phys); }
    if (PD < my_tiles) fetch_blocks(PD, phys);

    // waits until at most c tiles' worth (NI instructions each; the query rows are NI too) of this
    // wavefront's loads are outstanding (c uniform, <= PD)
    auto wait_tiles = [&](int c) {
        if constexpr (PD >= 3) { if (c == 3) { wait_vmcnt<3 * NI>(); return; } }
        if constexpr (PD >= 2) { if (c == 2) { wait_vmcnt<2 * NI>(); return; } }
        if (c == 1) { wait_vmcnt<NI>(); return; }
        wait_vmcnt<0>();
    };
    const float c2 = p.scale * kLog2e;
    // ---- the tree: checked once; ancestor-or-self masks of this lane's query rows -----------------
    if (wave == 0) {
        // requested after the parent array: the query rows and the tiles in flight, except a
        // first tile that went out early
        const int after_parent = min(PD, my_tiles) + 1 - (first_done ? 1 : 0);
        if (after_parent == PD + 1) wait_vmcnt<(PD + 1) * NI>(); else wait_tiles(after_parent);
    }
    __syncthreads();
    {
        bool bad = false;
        if (tid < n) {
            const int par = s_par[tid];
            bad = tid == 0 ? par != -1 : (par < 0 || par >= tid);
        }
        if (__syncthreads_or(bad)) err |= SPECVLM_ERR_BAD_PARENT;
    }
    if (err) {                                  // uniform over the workgroup (and over its splits)
        if (tid == 0 && p.err_flag) atomicOr(p.err_flag, err);
        wait_vmcnt<0>();                        // no load may still be writing this workgroup's LDS
        return;
    }
    unsigned long long anc[QBW];
#pragma unroll
    for (int qb = 0; qb < QBW; ++qb) {
        unsigned long long mask = 0;
        int t = qw * QW + qb * 16 + l16;
        if (t >= n) t = -1;
        while (t > 0) {                         // parent[t] < t was checked: at most 64 steps
            mask |= 1ull << t;
            t = s_par[t];
        }
        if (t == 0) mask |= 1ull;
        anc[qb] = mask;
    }
    wait_tiles(max(0, min(PD, my_tiles) - 1));  // the query rows and the first tile share have landed
    __syncthreads();                            // ... those of every wavefront
    // Q fragments (B operand): lane (query 16qb + l16, g) holds d = 32c + 8g .. +7, for the whole kernel
    bf16x8 qf[QBW][NC];
#pragma unroll
    for (int qb = 0; qb < QBW; ++qb)
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            const int rr = qb * 16 + l16;                 // row within this wavefront's QW rows
            const int u = 4 * c + g;
            qf[qb][c] = *reinterpret_cast<const bf16x8*>(ring + kStage + (rr / (QW / 2)) * kTileBytes + area +
                                                         ((rr % (QW / 2)) * ROWG + (u ^ (rr & (ROWG - 1)))) * 16);
        }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");      // staged rows are in registers: the areas may be refilled

    float m_run[QBW], mrc[QBW], l_run[QBW];    // reference max, the same times c2 (0 while -inf), running sum
    f32x4 acc[QBW][NT];
#pragma unroll
    for (int qb = 0; qb < QBW; ++qb) {
        m_run[qb] = -INFINITY;
        mrc[qb] = 0.f;
        l_run[qb] = 0.f;
#pragma unroll
        for (int t = 0; t < NT; ++t) acc[qb][t] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    for (int j = 0; j < wg_tiles; ++j) {
        const unsigned char* kt = ring + (j % kSlots) * kSlotBytes;
        const unsigned char* vt = kt + kTileBytes;
        const int slot0 = (stream + j * nstream) * kTile;
        // The slot of tile j+PD held tile j+PD-kSlots <= j-1, consumed by every wavefront of the
        // stream before the barrier that ended the previous iteration: request the tile into it.
        if (j + PD < my_tiles) issue_part(j + PD, phys);
        if (j + PD + 1 < my_tiles) fetch_blocks(j + PD + 1, phys);     // for the next iteration

        if (j < my_tiles) {
        // K fragments of the tile (A operand): lane (key = 16x + l16, g) holds d = 32c + 8g .. +7
        bf16x8 ka[2][NC];
#pragma unroll
        for (int x = 0; x < 2; ++x)
#pragma unroll
            for (int c = 0; c < NC; ++c) {
                const int r = x * 16 + l16;
                const int u = 4 * c + g;
                ka[x][c] = *reinterpret_cast<const bf16x8*>(kt + (r * ROWG + (u ^ (r & (ROWG - 1)))) * 16);
            }
        const bool tile_masked = slot0 + kTile > P;       // reaches past the prefix: tree region or tail
        bf16x8 pf[QBW];
#pragma unroll
        for (int qb = 0; qb < QBW; ++qb) {
            // S^T = K Q^T: s[x][i] = score of key slot0 + 16x + 4g + i against query QW*qw + 16qb + l16
            f32x4 s[2];
#pragma unroll
            for (int x = 0; x < 2; ++x) {
                f32x4 a = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int c = 0; c < NC; ++c) a = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[x][c], qf[qb][c], a, 0, 0, 0);
                s[x] = a;
            }
            if (tile_masked) {
#pragma unroll
                for (int x = 0; x < 2; ++x)
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        // branch-free on purpose: plain integer logic and one select per score
                        const int slot_key = slot0 + x * 16 + 4 * g + i;
                        const int rel = slot_key - P;
                        const uint32_t in_prefix = static_cast<uint32_t>(rel) >> 31;
                        const uint32_t is_anc = static_cast<uint32_t>(anc[qb] >> (rel & 63)) & 1u;
                        const uint32_t in_range = static_cast<uint32_t>(slot_key - S) >> 31;
                        const uint32_t vis = in_range & (in_prefix | is_anc);
                        s[x][i] = vis ? s[x][i] : -INFINITY;
                    }
            }
            // Online softmax with a lazily updated reference: p = exp2((s - m_ref) * c2) may exceed
            // 1; the reference only moves when some score would exceed it by more than 2^kTau (or
            // on the first visible key), so the common tile does no cross-lane work and never
            // touches the accumulators.  m_ref is identical in the 4 lanes that share a query row.
            const float lmax = fmaxf(fmaxf(fmaxf(s[0][0], s[0][1]), fmaxf(s[0][2], s[0][3])),
                                     fmaxf(fmaxf(s[1][0], s[1][1]), fmaxf(s[1][2], s[1][3])));
            const bool trig = m_run[qb] == -INFINITY ? lmax > -INFINITY : fmaf(lmax, c2, -mrc[qb]) > kTau;
            if (__builtin_expect(__any(trig), 0)) {
                float mx = lmax;
                mx = fmaxf(mx, __shfl_xor(mx, 16));
                mx = fmaxf(mx, __shfl_xor(mx, 32));
                const float m_new = fmaxf(m_run[qb], mx);
                const float m_safe = m_new == -INFINITY ? 0.f : m_new;
                const float alpha = m_run[qb] == -INFINITY ? 1.f : fast_exp2((m_run[qb] - m_safe) * c2);
                m_run[qb] = m_new;
                mrc[qb] = m_safe * c2;
                l_run[qb] *= alpha;                  // both are still zero while m_run was -inf
#pragma unroll
                for (int t = 0; t < NT; ++t) acc[qb][t] *= alpha;
            }
            float pr[8];
            float sum = 0.f;
#pragma unroll
            for (int jj = 0; jj < 8; ++jj) {
                pr[jj] = fast_exp2(fmaf(s[jj >> 2][jj & 3], c2, -mrc[qb]));
                sum += pr[jj];
            }
            l_run[qb] += sum;
            u32x4 w;
#pragma unroll
            for (int x = 0; x < 4; ++x) w[x] = pack_bf16x2(pr[2 * x], pr[2 * x + 1]);
            pf[qb] = __builtin_bit_cast(bf16x8, w);
        }
        // O^T += V^T P^T: contraction slot 8g + jj <-> key 16*(jj/4) + 4g + jj%4 of the tile.
        // A operand of head-dim block t: lane (l16, g) needs V[those 8 keys][d = 16t + l16].  A
        // transposing LDS read hands lane i of a 16-lane block element i%4 of the 8-byte rows
        // whose addresses lanes i/4, i/4+4, i/4+8, i/4+12 supply: with lane j supplying key
        // kb + j/4, dims 16t + 4(j%4) .. +3, lane i receives keys kb .. kb+3 at dim 16t + i --
        // one read for kb = 4g (slots 0-3), one for kb = 16 + 4g (slots 4-7).
        {
            const int jk = l16 >> 2, jd = l16 & 3;
            const int k0 = 4 * g + jk, k1 = 16 + 4 * g + jk;
            const unsigned char* r0 = vt + k0 * (ROWG * 16) + jd * 8;
            const unsigned char* r1 = vt + k1 * (ROWG * 16) + jd * 8;
            const int s0 = vswz(k0), s1 = vswz(k1);
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                const s16x4 lo = lds_read_tr16(r0 + ((t ^ s0) << 5));
                const s16x4 hi = lds_read_tr16(r1 + ((t ^ s1) << 5));
                const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                const bf16x8 va = __builtin_bit_cast(bf16x8, both);
#pragma unroll
                for (int qb = 0; qb < QBW; ++qb) acc[qb][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va, pf[qb], acc[qb][t], 0, 0, 0);
            }
        }
        }
        // This wavefront's reads of the slot have returned (their values fed the MFMAs above) and
        // its share of the next tile has landed (later tiles may still be in flight); the barrier
        // extends both to the whole stream.
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        wait_tiles(max(0, min(j + PD, my_tiles - 1) - (j + 1)));
        __syncthreads();
    }

    if (bad_block && lane == 0 && p.err_flag) atomicOr(p.err_flag, SPECVLM_ERR_BAD_BLOCK);
    // ---- merge the streams of the workgroup ------------------------------------------------------
    // Query block q4 = QBW*qw + qb (16 rows) is owned by one wavefront of query share qw, chosen
    // so that the four owners (wavefront index kStreams*qw + stream) sit on four different SIMDs.  Every wavefront publishes its reference maxima and sums; the other streams
    // of the share also hand the owner their accumulators through LDS, as they are: the owner
    // rescales every part (its own too) to the common maximum.  One barrier.
    int own_qb = -1;                                   // uniform: the query block this wavefront owns, if any
#pragma unroll
    for (int qb = 0; qb < QBW; ++qb) {
        const int qi = qw * QW + qb * 16 + l16;
        const int owner_st = kStreams == 2 ? ((qw * QBW + qb) >> 1) & 1 : (qw * QBW + qb) % kStreams;
        l_run[qb] += __shfl_xor(l_run[qb], 16);
        l_run[qb] += __shfl_xor(l_run[qb], 32);
        if (g == 0) {
            s_m[st][qi] = m_run[qb];
            s_l[st][qi] = l_run[qb];
        }
        if (st == owner_st) {
            own_qb = qb;
        } else {
            const int idx = st < owner_st ? st : st - 1;                 // kStreams-1 contributors per owner
            f32x4* dst = reinterpret_cast<f32x4*>(s_ring) + (((qw * QBW + qb) * (kStreams - 1) + idx) * NT) * 64;
#pragma unroll
            for (int t = 0; t < NT; ++t) dst[t * 64 + lane] = acc[qb][t];
        }
    }
    __syncthreads();                                   // (every stream was done with its ring already)
    const int q4 = qw * QBW + max(own_qb, 0);
    const int qi = q4 * 16 + l16;
    f32x4 out[NT];
    float Mq = s_m[0][qi];
#pragma unroll
    for (int x = 1; x < kStreams; ++x) Mq = fmaxf(Mq, s_m[x][qi]);
    float Lq = 0.f;
    {
        const float m_safe = Mq == -INFINITY ? 0.f : Mq;
#pragma unroll
        for (int qb = 0; qb < QBW; ++qb) {
            if (qb == own_qb) {                        // uniform
                const float w = fast_exp2((m_run[qb] - m_safe) * c2);    // 0 for a stream that saw no visible key
                Lq = l_run[qb] * w;
#pragma unroll
                for (int t = 0; t < NT; ++t) out[t] = acc[qb][t] * w;
            }
        }
        const f32x4* src = reinterpret_cast<const f32x4*>(s_ring) + (q4 * (kStreams - 1) * NT) * 64;
#pragma unroll
        for (int idx = 0; idx < kStreams - 1; ++idx) {
            const int x = idx < st ? idx : idx + 1;    // the idx-th contributor's stream
            const float w = fast_exp2((s_m[x][qi] - m_safe) * c2);
            Lq += s_l[x][qi] * w;
            if (own_qb >= 0) {
#pragma unroll
                for (int t = 0; t < NT; ++t) out[t] += src[(idx * NT + t) * 64 + lane] * w;
            }
        }
    }
    const bool wave_active = own_qb >= 0 && q4 * 16 < n;     // wavefronts that own a real query row
    if (p.num_splits == 1) {
        if (wave_active) store_rows<NT>(p, out, Mq, Lq, b, h, qi, g, n);
        return;
    }
    // ---- split partials: write-through stores, ticket, the last arrival merges ------------------
    // From here on every owner wavefront goes its own way (no workgroup barrier): it stores its
    // query block's partial, draws a ticket of its (request, head, query block), and the wavefront
    // that finds all other splits' tickets drawn merges that block.
    if (!wave_active) return;
    const int64_t part0 = static_cast<int64_t>(bh) * p.num_splits;
    // Partials are kept in bf16 (halves the bytes one compute unit must pull for the merge);
    // the same rounding is applied to the final output anyway.  Dword i*NT/2 + t/2 of a lane
    // packs out[t][i], out[t+1][i].
    constexpr int PV4 = NT / 2;                        // 16-byte vectors per lane per partial
    {
        u32x4* dst = reinterpret_cast<u32x4*>(p.ws_acc) + ((part0 + split) * 4 + q4) * PV4 * 64;
        uint32_t w[4][NT / 2];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int t = 0; t < NT; t += 2) w[i][t / 2] = pack_bf16x2(out[t][i], out[t + 1][i]);
#pragma unroll
        for (int v = 0; v < PV4; ++v) {
            // vector v holds dwords 4v .. 4v+3 of the lane's NT*2 dwords, in (i, t/2) order
            u32x4 x;
#pragma unroll
            for (int e = 0; e < 4; ++e) x[e] = w[(4 * v + e) / (NT / 2)][(4 * v + e) % (NT / 2)];
            store16_coherent(dst + v * 64 + lane, x);
        }
        if (g == 0) {
            float* ml = p.ws_ml + ((part0 + split) * kQRows + qi) * 2;
            store8_coherent(ml, u32x2{__float_as_uint(Mq), __float_as_uint(Lq)});
        }
    }
    wait_vmcnt<0>();                                   // this wavefront's write-through stores have been acknowledged
    int is_last = 0;
    if (lane == 0) {
        int32_t* cnt = p.ws_cnt + (static_cast<int64_t>(bh) * 4 + q4) * kCounterStride;
        const int ticket = __hip_atomic_fetch_add(cnt, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        is_last = ticket == p.num_splits - 1;
        // every other split has already drawn its ticket: leave the counter zero for the next call
        if (is_last) __hip_atomic_store(cnt, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    if (!__builtin_amdgcn_readfirstlane(is_last)) return;
    // The partials are read with device-coherent loads (the encoding of an agent-scope atomic load:
    // they never return what this compute unit or its L2 still holds of the workspace from
    // earlier calls), issued after the ticket was seen; this is cheaper than an acquire fence,
    // which would also invalidate the L2.  The compiler does not track these loads: they are
    // waited for by hand -- loads complete in order, so the reference maxima (requested first) can
    // be reduced and split u can be added up while the partials of the splits after it are still
    // on their way -- and every register passes through an empty asm after its wait, so that no
    // use can be scheduled before it.
    // Addresses are a uniform base (the split) plus a lane offset that never changes, so the 40
    // loads of a batch tie up no address registers.
    const uint32_t voff_part = lane * 16, voff_ml = qi * 8;
    const unsigned char* acc_base = reinterpret_cast<const unsigned char*>(p.ws_acc) + (part0 * 4 + q4) * PV4 * 1024;
    const unsigned char* ml_base = reinterpret_cast<const unsigned char*>(p.ws_ml) + part0 * kQRows * 8;
    auto ld_part = [&](int se, int v) {                 // 16-byte vector v of split se's partial of this query block
        u32x4 r;
        const unsigned char* sb = acc_base + static_cast<int64_t>(se) * (4 * PV4 * 1024) + v * 1024;
        asm volatile("global_load_dwordx4 %0, %1, %2 sc1" : "=v"(r) : "v"(voff_part), "s"(sb) : "memory");
        return r;
    };
    auto ld_ml = [&](int se) {                          // (reference maximum, sum) of split se for this lane's query row
        f32x2 r;
        const unsigned char* sb = ml_base + static_cast<int64_t>(se) * (kQRows * 8);
        asm volatile("global_load_dwordx2 %0, %1, %2 sc1" : "=v"(r) : "v"(voff_ml), "s"(sb) : "memory");
        return r;
    };
    const int last = p.num_splits - 1;
    float Mall = -INFINITY, Lall = 0.f;
    auto add_split = [&](const u32x4 (&pv)[PV4], float w) {     // out += w * partial
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int t = 0; t < NT; t += 2) {
                const int dw = i * (NT / 2) + t / 2;
                const uint32_t x = pv[dw >> 2][dw & 3];
                out[t][i] = fmaf(__uint_as_float(x << 16), w, out[t][i]);
                out[t + 1][i] = fmaf(__uint_as_float(x & 0xFFFF0000u), w, out[t + 1][i]);
            }
    };
    if (p.num_splits <= 8) {                           // uniform; what the library chooses by itself
        // One batch of 8 + 8*PV4 loads: maxima and sums first, then the partials in split order;
        // indices past the last split are clamped and given weight zero, so there is no branch.
        u32x4 part[8][PV4];
        f32x2 ml[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) ml[u] = ld_ml(min(u, last));
#pragma unroll
        for (int u = 0; u < 8; ++u)
#pragma unroll
            for (int v = 0; v < PV4; ++v) part[u][v] = ld_part(min(u, last), v);
        wait_vmcnt<8 * PV4>();                         // the maxima and sums have landed
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            asm volatile("" : "+v"(ml[u]));
            Mall = fmaxf(Mall, ml[u][0]);
        }
        const float m_safe = Mall == -INFINITY ? 0.f : Mall;
#pragma unroll
        for (int t = 0; t < NT; ++t) out[t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            wait_vmcnt_unrolled((7 - u) * PV4);        // the partial of split u has landed
#pragma unroll
            for (int v = 0; v < PV4; ++v) asm volatile("" : "+v"(part[u][v]));
            const float w = u <= last ? fast_exp2((ml[u][0] - m_safe) * c2) : 0.f;
            Lall += ml[u][1] * w;
            add_split(part[u], w);
        }
    } else {                                           // a caller's larger split count: one split at a time
        for (int se = 0; se <= last; ++se) {
            f32x2 t2 = ld_ml(se);
            asm volatile("s_waitcnt vmcnt(0)" : "+v"(t2) : : "memory");
            Mall = fmaxf(Mall, t2[0]);
        }
        const float m_safe = Mall == -INFINITY ? 0.f : Mall;
#pragma unroll
        for (int t = 0; t < NT; ++t) out[t] = f32x4{0.f, 0.f, 0.f, 0.f};
        for (int se = 0; se <= last; ++se) {
            f32x2 t2 = ld_ml(se);
            u32x4 pv[PV4];
#pragma unroll
            for (int v = 0; v < PV4; ++v) pv[v] = ld_part(se, v);
            asm volatile("s_waitcnt vmcnt(0)" : "+v"(t2) : : "memory");
#pragma unroll
            for (int v = 0; v < PV4; ++v) asm volatile("" : "+v"(pv[v]));
            const float w = fast_exp2((t2[0] - m_safe) * c2);
            Lall += t2[1] * w;
            add_split(pv, w);
        }
    }
    store_rows<NT>(p, out, Mall, Lall, b, h, qi, g, n);
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
    if (d.D == 128) hipLaunchKernelGGL((attn_mfma_kernel<128, kShare, kAhead>), grid, block, 0, a.stream, p);
    else hipLaunchKernelGGL((attn_mfma_kernel<64, kShare, kAhead>), grid, block, 0, a.stream, p);
    return check_launch();
}

}  // namespace specvlm
