// Draft-side growth of the token tree (SpecVLM Sec. 4.1: the draft grows an EAGLE-2 style tree
// with Top-K 10, 60 tokens in total, depth 7, which the target then verifies in one pass).
//
// The paper gives the three numbers; the rule is the one of the method it follows.  A node's
// value is the sum of the draft's log-probabilities along its root path.  Every level expands
// the most valuable nodes of the previous level by their Top-K tokens (draft_topk_kernel),
// the most valuable new candidates are expanded next (draft_select_kernel), and in the end the
// most valuable candidates of all levels become the tree (draft_finalize_kernel), numbered in
// increasing candidate index, which is a topological order because a parent is created before
// its children.  "More valuable" is: greater stored fp32 score, the lower candidate index among
// equal scores; Top-K inside a row: greater logit, the lower token among equal logits.
//
// All three are latency-bound single-workgroup-per-row kernels: a row of 32000 bf16 logits is
// 64 KB, a level has at most `width` rows per request, and the candidate lists hold a few
// hundred entries.
#include <limits.h>

#include "common.hpp"

namespace specvlm {

namespace {

constexpr int kThreadsDT = 1024;
constexpr int kWavesDT = kThreadsDT / 64;
constexpr int kCandCap = 1024;           // Top-K fast path: entries at or above the threshold kept in LDS

template <typename T>
struct Lane16;
template <>
struct Lane16<uint16_t> {
    static constexpr int kPerVec = 8;
    __device__ static float at(const uint4& w, int e) {
        const uint32_t x = (&w.x)[e >> 1];
        return __uint_as_float((e & 1) ? (x & 0xFFFF0000u) : (x << 16));
    }
    __device__ static float one(const uint16_t* p) { return bf16_bits_to_float(*p); }
};
template <>
struct Lane16<float> {
    static constexpr int kPerVec = 4;
    __device__ static float at(const uint4& w, int e) { return __uint_as_float((&w.x)[e]); }
    __device__ static float one(const float* p) { return *p; }
};

// NS entries of a row in a thread's registers, as loaded: bf16 entries stay packed two to a
// register and are widened where they are used (one shift or mask).
template <typename T, int NS>
struct RowRegs;
template <int NS>
struct RowRegs<uint16_t, NS> {
    uint32_t w[NS / 2];
    __device__ __forceinline__ float get(int s) const {
        const uint32_t x = w[s >> 1];
        return __uint_as_float((s & 1) ? (x & 0xFFFF0000u) : (x << 16));
    }
    __device__ __forceinline__ void put_vec(int j, const uint4& x) {          // entries 8j .. 8j+7
        w[4 * j] = x.x; w[4 * j + 1] = x.y; w[4 * j + 2] = x.z; w[4 * j + 3] = x.w;
    }
    __device__ __forceinline__ void fill_vec(int j) {                         // -inf
        w[4 * j] = w[4 * j + 1] = w[4 * j + 2] = w[4 * j + 3] = 0xFF80FF80u;
    }
    // Called between two passes over the entries: the compiler then widens the entries again in
    // the next pass instead of keeping NS widened copies alive beside the packed ones.
    __device__ __forceinline__ void repack() {
#pragma unroll
        for (int i = 0; i < NS / 2; ++i) asm volatile("" : "+v"(w[i]));
    }
    __device__ __forceinline__ void put_one(int s, const uint16_t* p) {       // p == nullptr: -inf; even s first
        const uint32_t b = p ? *p : 0xFF80u;
        w[s >> 1] = (s & 1) ? (w[s >> 1] | (b << 16)) : b;
    }
};
template <int NS>
struct RowRegs<float, NS> {
    float f[NS];
    __device__ __forceinline__ float get(int s) const { return f[s]; }
    __device__ __forceinline__ void put_vec(int j, const uint4& x) {          // entries 4j .. 4j+3
        f[4 * j] = __uint_as_float(x.x); f[4 * j + 1] = __uint_as_float(x.y);
        f[4 * j + 2] = __uint_as_float(x.z); f[4 * j + 3] = __uint_as_float(x.w);
    }
    __device__ __forceinline__ void fill_vec(int j) { f[4 * j] = f[4 * j + 1] = f[4 * j + 2] = f[4 * j + 3] = -INFINITY; }
    __device__ __forceinline__ void repack() {}
    __device__ __forceinline__ void put_one(int s, const float* p) { f[s] = p ? *p : -INFINITY; }
};

// (logit, token) as one unsigned key whose order is "greater logit, then lower token".
// -0 and +0 are the same real number and must tie: adding +0 turns -0 into +0.
__device__ __forceinline__ unsigned long long order_key(float v, int idx) {
    uint32_t u = __float_as_uint(v + 0.0f);
    u = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
    return (static_cast<unsigned long long>(u) << 32) | (0xFFFFFFFFu - static_cast<uint32_t>(idx));
}

__device__ __forceinline__ float key_value(unsigned long long k) {     // the logit inside an order_key
    uint32_t u = static_cast<uint32_t>(k >> 32);
    u = (u & 0x80000000u) ? (u & 0x7FFFFFFFu) : ~u;
    return __uint_as_float(u);
}

__device__ __forceinline__ unsigned long long wave_max_u64(unsigned long long x) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const unsigned long long y = __shfl_xor(x, off);
        x = y > x ? y : x;
    }
    return x;
}

// Fixed-shape workgroup reductions (results never depend on timing).
__device__ __forceinline__ float wg_max(float x, float* s_red) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) x = fmaxf(x, __shfl_xor(x, off));
    __syncthreads();
    if ((threadIdx.x & 63) == 0) s_red[threadIdx.x >> 6] = x;
    __syncthreads();
    float r = s_red[0];
#pragma unroll
    for (int w = 1; w < kWavesDT; ++w) r = fmaxf(r, s_red[w]);
    return r;
}

__device__ __forceinline__ float wg_sum(float x, float* s_red) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) x += __shfl_xor(x, off);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) s_red[threadIdx.x >> 6] = x;
    __syncthreads();
    float r = s_red[0];
#pragma unroll
    for (int w = 1; w < kWavesDT; ++w) r += s_red[w];
    return r;
}

// ---------------------------------------------------------------------------------------
// Ranking of scored candidates: candidate i beats j when score[i] > score[j], or the scores
// are equal and i < j -- i.e. when its order_key(score, index) is the greater one.  rank(i) =
// number of candidates that beat i; the M winners are the candidates of rank < M; a winner's
// position is the number of winners of lower index.
// s_key holds the c keys (16-byte aligned).  On return the low word of s_key[i] holds candidate
// i's position among the winners, or -1 (pos_of below); the keys are gone.
// All c*c comparisons run on one compute unit, so what counts is instructions per comparison
// (two, see below) and that every wavefront has work: with few candidates several groups of
// wavefronts share the candidates, each taking a slice of the others.  s_key needs room for an
// even number of keys.
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ int pos_of(const unsigned long long* s_key, int i) {
    return reinterpret_cast<const int*>(s_key)[2 * i];
}

// Many candidates, few winners (the whole tree's 500 candidates, 59 nodes): ranking everybody
// against everybody is mostly wasted on candidates that cannot win.  The candidates are dealt
// into kGroupsDT groups (candidate i -> group i mod kGroupsDT); the M-th largest of the group
// maxima is a key that at least M candidates reach, so nobody below it wins, and at most
// M * ceil(c / kGroupsDT) candidates reach it (the members of M groups).  Only those are ranked,
// among themselves.  Same result as rank_winners' full ranking: keys are distinct, so "the M
// greatest keys" is one set whatever way it is found.  Needs kGroupsDT <= c <= kThreadsDT (every
// group has a member, one candidate per thread) and M <= kGroupsDT.
constexpr int kGroupsDT = 128;

__device__ __forceinline__ void rank_winners_prefiltered(unsigned long long* s_key, int c, int M) {
    __shared__ unsigned long long s_gmax[kGroupsDT];
    __shared__ unsigned long long s_surv[kThreadsDT];
    __shared__ unsigned long long s_thr;
    __shared__ int s_cnt2[kThreadsDT];
    __shared__ int s_wcount2[kWavesDT];
    __shared__ uint32_t s_winmask[kThreadsDT / 32];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const unsigned long long ki = tid < c ? s_key[tid] : 0ull;          // 0: below every real key
    if (tid < kGroupsDT) {
        unsigned long long m = ki;
        for (int i = tid + kGroupsDT; i < c; i += kGroupsDT) {
            const unsigned long long k = s_key[i];
            m = k > m ? k : m;
        }
        s_gmax[tid] = m;
    }
    s_cnt2[tid] = 0;
    if (tid < kThreadsDT / 32) s_winmask[tid] = 0u;
    __syncthreads();
    // rank of every group maximum among the group maxima: four threads per maximum, a quarter each
    {
        const int j = tid & (kGroupsDT - 1), part = tid / kGroupsDT;
        constexpr int kPer = kGroupsDT / (kThreadsDT / kGroupsDT);
        const unsigned long long kj = s_gmax[j];
        int beaten = 0;
#pragma unroll 8
        for (int x = part * kPer; x < (part + 1) * kPer; ++x) beaten += s_gmax[x] > kj ? 1 : 0;
        atomicAdd(&s_cnt2[j], beaten);
    }
    __syncthreads();
    if (tid < kGroupsDT && s_cnt2[tid] == M - 1) s_thr = s_gmax[tid];    // exactly one thread: the ranks are a permutation
    __syncthreads();
    const unsigned long long thr = s_thr;
    // the candidates that reach the threshold, gathered in index order
    const bool surv = ki >= thr;                                         // thr is a real key: never true for tid >= c
    const unsigned long long bal = __ballot(surv);
    if (lane == 0) s_wcount2[wave] = __popcll(bal);
    s_cnt2[tid] = 0;
    __syncthreads();
    int before = 0, ns = 0;
#pragma unroll
    for (int x = 0; x < kWavesDT; ++x) {
        const int n = s_wcount2[x];
        before += x < wave ? n : 0;
        ns += n;
    }
    if (surv) s_surv[before + __popcll(bal & ((1ull << lane) - 1ull))] = ki;
    if (tid < c) reinterpret_cast<int*>(s_key)[2 * tid] = -1;           // every key is in a register or in s_surv by now
    __syncthreads();
    // rank among the ns survivors: `parts` threads per survivor, a slice each
    int nsp = 64;                                                        // uniform: survivors rounded up to a power of two
    while (nsp < ns) nsp *= 2;
    const int parts = kThreadsDT / nsp, per = (ns + parts - 1) / parts;
    const int a = tid & (nsp - 1), part = tid / nsp;
    const unsigned long long ka = a < ns ? s_surv[a] : ~0ull;
    {
        int beaten = 0;
        const int x1 = min(ns, (part + 1) * per);
        for (int x = part * per; x < x1; ++x) beaten += s_surv[x] > ka ? 1 : 0;
        if (a < ns) atomicAdd(&s_cnt2[a], beaten);
    }
    __syncthreads();
    const bool win = part == 0 && a < ns && s_cnt2[a] < M;
    const uint32_t idx = 0xFFFFFFFFu - static_cast<uint32_t>(ka);       // the candidate's index sits in the key's low word
    if (win) atomicOr(&s_winmask[idx >> 5], 1u << (idx & 31));
    __syncthreads();
    if (win) {                                                           // position = winners of lower index
        int pos = __popc(s_winmask[idx >> 5] & ((1u << (idx & 31)) - 1u));
        for (uint32_t w = 0; w < (idx >> 5); ++w) pos += __popc(s_winmask[w]);
        reinterpret_cast<int*>(s_key)[2 * idx] = pos;
    }
    __syncthreads();
}

__device__ __forceinline__ void rank_winners(unsigned long long* s_key, int c, int M) {
    __shared__ int s_wcount[kWavesDT];
    __shared__ int s_cnt[kThreadsDT];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (c >= 2 * kGroupsDT && c <= kThreadsDT && M >= 1 && M <= kGroupsDT / 2) {    // uniform
        rank_winners_prefiltered(s_key, c, M);
        return;
    }
    // `parts` groups of wavefronts share the candidates of a pass: group `part` counts, for every
    // candidate of the pass, the keys of its slice [j0, j1) of the others that beat it.
    int parts = 1, shift = 0;                              // uniform; a group is at least one wavefront
    while (parts < kWavesDT && c * (parts * 2) <= kThreadsDT) { parts *= 2; ++shift; }
    const int per_pass = kThreadsDT >> shift;              // candidates per pass (>= 64)
    const int part = tid / per_pass, slot = tid & (per_pass - 1);
    const int c_even = (c + 1) & ~1;                       // keys are read in pairs: an odd count is padded with a key nothing loses to
    if (tid == 0 && (c & 1)) s_key[c] = 0ull;
    __syncthreads();
    const int per = ((c_even / 2 + parts - 1) / parts) * 2;
    const int j0 = min(part * per, c_even), j1 = min(j0 + per, c_even);
    unsigned winbits = 0;                                  // bit p: this thread's candidate of pass p won (at most 8 passes)
    int pass = 0;
    for (int i0 = 0; i0 < c; i0 += per_pass, ++pass) {     // uniform trip count
        const int i = i0 + slot;
        const unsigned long long ki = i < c ? s_key[i] : ~0ull;
        const uint32_t hi = static_cast<uint32_t>(ki >> 32);
        // The candidates of this wavefront are iw0 .. iw0 + 63.  A key j below all of them beats
        // candidate i when its upper word is >= i's (equal scores: the lower index wins), a key
        // above all of them when it is > : one 32-bit compare and an add-with-carry per key (a
        // 64-bit compare runs at a quarter of that rate).  Only the keys among the wavefront's own
        // candidates need the whole key.  (No score is NaN, so an upper word is never 0.)
        const int iw0 = i0 + ((wave * 64) & (per_pass - 1));
        const int a_end = max(j0, min(j1, iw0 & ~1));             // pairs entirely below iw0
        const int b_end = max(a_end, min(j1, (iw0 + 65) & ~1));   // pairs that may hold one of the wavefront's candidates
        int beaten = 0;
        const uint32_t thr_below = hi - 1u;
#pragma unroll 4
        for (int j = j0; j < a_end; j += 2) {
            const ulonglong2 q = *reinterpret_cast<const ulonglong2*>(s_key + j);
            beaten += static_cast<uint32_t>(q.x >> 32) > thr_below ? 1 : 0;
            beaten += static_cast<uint32_t>(q.y >> 32) > thr_below ? 1 : 0;
        }
        for (int j = a_end; j < b_end; j += 2) {
            const ulonglong2 q = *reinterpret_cast<const ulonglong2*>(s_key + j);
            beaten += q.x > ki ? 1 : 0;
            beaten += q.y > ki ? 1 : 0;
        }
#pragma unroll 4
        for (int j = b_end; j < j1; j += 2) {
            const ulonglong2 q = *reinterpret_cast<const ulonglong2*>(s_key + j);
            beaten += static_cast<uint32_t>(q.x >> 32) > hi ? 1 : 0;
            beaten += static_cast<uint32_t>(q.y >> 32) > hi ? 1 : 0;
        }
        if (parts > 1) {                                   // uniform: add the groups' counts up
            if (part == 0) s_cnt[slot] = 0;
            __syncthreads();
            atomicAdd(&s_cnt[slot], beaten);
            __syncthreads();
            beaten = s_cnt[slot];
            __syncthreads();                               // s_cnt is cleared again by the next pass
        }
        if (i < c && part == 0 && beaten < M) winbits |= 1u << pass;
    }
    __syncthreads();                                       // the keys have been read for the last time
    // position of a winner = winners of lower index: earlier passes, earlier wavefronts, lower lanes
    int base = 0;
    pass = 0;
    for (int i0 = 0; i0 < c; i0 += per_pass, ++pass) {
        const int i = i0 + slot;
        const bool win = (winbits >> pass) & 1u;
        const unsigned long long bal = __ballot(win);
        if (lane == 0) s_wcount[wave] = __popcll(bal);
        __syncthreads();
        int before = base, total = 0;
#pragma unroll
        for (int x = 0; x < kWavesDT; ++x) {
            const int n = s_wcount[x];
            before += x < wave ? n : 0;
            total += n;
        }
        if (i < c && part == 0)
            reinterpret_cast<int*>(s_key)[2 * i] = win ? before + __popcll(bal & ((1ull << lane) - 1ull)) : -1;
        base += total;
        __syncthreads();                                   // s_wcount is rewritten by the next pass
    }
}

// ---------------------------------------------------------------------------------------
// draft_topk_kernel: one workgroup per (request, expanded node) row.
//   NS > 0: every thread keeps NS vocabulary entries of the row in registers (16-byte loads
//           when the row is aligned and V a multiple of the vector width, scalar otherwise);
//   NS == 0: any vocabulary size, every pass re-reads the row (it stays in L2).
// Passes: maximum, sum of exp(l - max) (log-sum-exp), then the K best (logit, token) keys: a
// threshold from the maxima of 16-lane groups and a rank among the few entries that reach it,
// or, when too many do, K rounds of a workgroup-wide arg-max (every thread caches the best key
// among its entries not yet taken; only the owner of a round's winner rescans its entries).
// ---------------------------------------------------------------------------------------
// SEL: the workgroup that finishes a request's last row also chooses the M most valuable of the
// request's W*K new candidates (what draft_select_kernel does in a launch of its own): scores
// are stored write-through, acknowledged, then a ticket per request is drawn.
struct SelArgs {
    int M, index_base;
    int32_t* sel_out;
    float* sel_score_out;
    int32_t* count_out;
    int32_t* counters;            // [B * SPECVLM_COUNTER_STRIDE] tickets, zero between calls
};

template <typename T, int NS, bool SEL>
__global__ __launch_bounds__(kThreadsDT) void draft_topk_kernel(
    int V, int K, const T* __restrict__ logits, int64_t stride_b, int64_t stride_w,
    const float* __restrict__ cum, int64_t cum_stride_b, const int32_t* __restrict__ parent_idx,
    int64_t parent_stride_b, float* score_out, int32_t* __restrict__ token_out,
    int32_t* __restrict__ parent_out, int64_t out_stride_b, float* __restrict__ lse_out, SelArgs sel) {
    __shared__ float s_red[kWavesDT];
    __shared__ unsigned long long s_key[2][kWavesDT];
    __shared__ int s_taken[SPECVLM_MAX_NODES];         // NS == 0: tokens already taken
    __shared__ unsigned long long s_grp[64];
    __shared__ __attribute__((aligned(16))) unsigned long long s_cand[kCandCap];
    __shared__ int s_last;
    __shared__ unsigned long long s_thr;
    __shared__ int s_ncand;

    const int w = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
    const int nrows = gridDim.x;
    const T* row = logits + b * stride_b + w * stride_w;
    constexpr int VEC = Lane16<T>::kPerVec;
    const bool vec = NS > 0 && (reinterpret_cast<uintptr_t>(row) & 15u) == 0 && V % VEC == 0;   // uniform
    // entry s of this thread is vocabulary index idx_of(s)
    auto idx_of = [&](int s) -> int {
        return vec ? (tid + kThreadsDT * (s / VEC)) * VEC + s % VEC : tid + kThreadsDT * s;
    };
    // Entries are compared as floats inside a thread (no logit is NaN, and -0 == +0 as the order
    // demands); a 64-bit key is built only for the few entries that leave the thread.  16
    // wavefronts leave a thread 128 registers: the keys of all entries would not fit beside
    // the entries.  Entries past V hold -inf.
    RowRegs<T, (NS > 0 ? NS : 8)> lv;
    if constexpr (NS > 0) {
        if (vec) {
#pragma unroll
            for (int j = 0; j < NS / VEC; ++j) {
                const int v0 = (tid + kThreadsDT * j) * VEC;
                if (v0 < V) lv.put_vec(j, *reinterpret_cast<const uint4*>(row + v0));
                else lv.fill_vec(j);
            }
        } else {
#pragma unroll
            for (int s = 0; s < NS; ++s) {
                const int v = tid + kThreadsDT * s;
                lv.put_one(s, v < V ? row + v : nullptr);
            }
        }
    }
    // Best entry of this thread among those not in `skip` (bit s = entry s): its key, or 0 when
    // none is left.  A thread's entries are in ascending token order, so "greater" alone keeps
    // the lowest token among equal logits.
    auto thread_best = [&](unsigned long long skip) __attribute__((always_inline)) -> unsigned long long {
        float bf = 0.f;
        int bv = -1;
        if constexpr (NS > 0) {
#pragma unroll
            for (int s = 0; s < NS; ++s) {
                const int v = idx_of(s);
                if (v < V && !((skip >> s) & 1ull) && (bv < 0 || lv.get(s) > bf)) { bf = lv.get(s); bv = v; }
            }
        }
        return bv >= 0 ? order_key(bf, bv) : 0ull;
    };
    const int ns_mem = (V + kThreadsDT - 1) / kThreadsDT;          // NS == 0: entries per thread

    // ---- log-sum-exp of the row -----------------------------------------------------------
    float part = -INFINITY;
    if constexpr (NS > 0) {
#pragma unroll
        for (int s = 0; s < NS; ++s) part = fmaxf(part, lv.get(s));    // entries past V hold -inf
    } else {
#pragma unroll 8
        for (int s = 0; s < ns_mem; ++s) {
            const int v = tid + kThreadsDT * s;
            if (v < V) part = fmaxf(part, Lane16<T>::one(row + v));
        }
    }
    const float tmax = part;                            // NS > 0: this thread's greatest logit
    const float mx = wg_max(part, s_red);
    lv.repack();
    part = 0.f;
    if constexpr (NS > 0) {
#pragma unroll
        for (int s = 0; s < NS; ++s) part += __expf(lv.get(s) - mx);   // exp(-inf) = 0
    } else {
#pragma unroll 8
        for (int s = 0; s < ns_mem; ++s) {
            const int v = tid + kThreadsDT * s;
            if (v < V) part += __expf(Lane16<T>::one(row + v) - mx);
        }
    }
    const float Z = wg_sum(part, s_red);
    lv.repack();
    const float lse = mx + logf(Z);
    const float c = cum ? cum[b * cum_stride_b + w] : 0.f;
    const int par = parent_idx ? parent_idx[b * parent_stride_b + w] : -1;
    if (tid == 0 && lse_out) lse_out[b * nrows + w] = lse;

    const int64_t out0 = b * out_stride_b + static_cast<int64_t>(w) * K;
    auto emit = [&](int k, unsigned long long key) {     // k-th best of the row
        token_out[out0 + k] = static_cast<int>(0xFFFFFFFFu - static_cast<uint32_t>(key));
        const float sc = c + (key_value(key) - lse);
        if constexpr (SEL)                               // read by another workgroup in this kernel
            __hip_atomic_store(reinterpret_cast<uint32_t*>(score_out + out0 + k), __float_as_uint(sc),
                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        else
            score_out[out0 + k] = sc;
        if (parent_out) parent_out[out0 + k] = par;
    };

    // ---- fast path: a threshold that at least K entries reach, then a rank among the few that do ----
    // Every group of 16 lanes reduces the best key of its entries; the K-th best of the 64 group
    // maxima is a key that K entries of the row reach (the maxima of K different groups), so the
    // K best entries are among the entries at or above it -- for logits that do not follow the
    // token order, about 2K of them.  These are collected in LDS and ranked against each other:
    // an entry beaten by r others is the r-th best.  Keys are distinct, so the result does not
    // depend on the order in which the entries were collected.  If more than kCandCap entries
    // reach the threshold (logits sorted along the vocabulary, say) the K rounds below take over.
    bool done = false;                                  // uniform
    {
        unsigned long long mine = 0;
        if constexpr (NS > 0) {
            // the first entry that equals the thread's maximum (found for the log-sum-exp above)
            int bs = NS;
#pragma unroll
            for (int s = NS - 1; s >= 0; --s) bs = lv.get(s) == tmax ? s : bs;
            const int bv = idx_of(bs);
            mine = bv < V ? order_key(tmax, bv) : 0ull;   // a thread whose entries all lie past V has none
        } else {
#pragma unroll 8
            for (int s = 0; s < ns_mem; ++s) {
                const int v = tid + kThreadsDT * s;
                const unsigned long long k = v < V ? order_key(Lane16<T>::one(row + v), v) : 0ull;
                mine = k > mine ? k : mine;
            }
        }
        unsigned long long grp = mine;
#pragma unroll
        for (int off = 8; off >= 1; off >>= 1) {
            const unsigned long long y = __shfl_xor(grp, off);
            grp = y > grp ? y : grp;
        }
        if (tid == 0) { s_ncand = 0; s_thr = 0; }        // threshold 0: every entry qualifies
        if ((tid & 15) == 0) s_grp[tid >> 4] = grp;
        __syncthreads();
        if (tid < 64) {
            const unsigned long long g = s_grp[tid];
            int beaten = 0;
#pragma unroll 8
            for (int x = 0; x < 64; ++x) beaten += s_grp[x] > g ? 1 : 0;
            if (beaten == K - 1 && g != 0) s_thr = g;   // at most one lane (keys are distinct); none when fewer
        }                                               // than K groups hold an entry: the threshold stays 0
        __syncthreads();
        const unsigned long long thr = s_thr;
        lv.repack();
        if constexpr (NS > 0) {
            // Entries whose logit reaches the threshold's logit: a superset of the entries whose
            // key reaches the threshold (it adds higher tokens with the same logit), which the
            // ranking below does not mind.  Only a thread whose maximum reaches it has any.
            const float thr_val = thr ? key_value(thr) : -INFINITY;
            if (tmax >= thr_val) {
#pragma unroll
                for (int s = 0; s < NS; ++s) {
                    const int v = idx_of(s);
                    if (lv.get(s) >= thr_val && v < V) {
                        const int pos = atomicAdd(&s_ncand, 1);
                        if (pos < kCandCap) s_cand[pos] = order_key(lv.get(s), v);
                    }
                }
            }
        } else {
            for (int s = 0; s < ns_mem; ++s) {
                const int v = tid + kThreadsDT * s;
                if (v >= V) break;
                const unsigned long long k = order_key(Lane16<T>::one(row + v), v);
                if (k >= thr) {
                    const int pos = atomicAdd(&s_ncand, 1);
                    if (pos < kCandCap) s_cand[pos] = k;
                }
            }
        }
        __syncthreads();
        const int nc = s_ncand;
        if (nc <= kCandCap) {                           // uniform
            for (int i = tid; i < nc; i += kThreadsDT) {
                const unsigned long long k = s_cand[i];
                int beaten = 0;
                for (int x = 0; x < nc; ++x) beaten += s_cand[x] > k ? 1 : 0;
                if (beaten < K) emit(beaten, k);
            }
            done = true;
        }
    }

    if (!done) {
        // ---- K rounds of arg-max (any input) --------------------------------------------------------
        unsigned long long taken = 0;                       // NS > 0: bit s = entry s was taken
        int ntaken = 0;                                     // NS == 0: length of s_taken
        auto local_best = [&]() __attribute__((always_inline)) -> unsigned long long {
            unsigned long long best = 0;                    // 0 = nothing left
            if constexpr (NS > 0) {
                best = thread_best(taken);
            } else {
                for (int s = 0; s < ns_mem; ++s) {
                    const int v = tid + kThreadsDT * s;
                    if (v >= V) break;
                    bool live = true;
                    for (int r = 0; r < ntaken; ++r) live = live && s_taken[r] != v;
                    if (live) {
                        const unsigned long long k = order_key(Lane16<T>::one(row + v), v);
                        best = k > best ? k : best;
                    }
                }
            }
            return best;
        };
        unsigned long long mine = local_best();
        for (int k = 0; k < K; ++k) {
            const unsigned long long wbest = wave_max_u64(mine);
            if ((tid & 63) == 0) s_key[k & 1][tid >> 6] = wbest;
            __syncthreads();                                // (the other buffer was last read two rounds ago)
            unsigned long long win = s_key[k & 1][0];
    #pragma unroll
            for (int x = 1; x < kWavesDT; ++x) {
                const unsigned long long y = s_key[k & 1][x];
                win = y > win ? y : win;
            }
            const int v = static_cast<int>(0xFFFFFFFFu - static_cast<uint32_t>(win));       // K <= V: never empty
            if constexpr (NS == 0) {
                if (tid == 0) s_taken[k] = v;
                ++ntaken;
                __syncthreads();
            }
            if (mine == win) {                              // exactly one thread: tokens are distinct
                if constexpr (NS > 0) {
    #pragma unroll
                    for (int s = 0; s < NS; ++s)
                        if (idx_of(s) == v) taken |= 1ull << s;
                }
                emit(k, win);
                mine = local_best();
            }
        }
    }
    if constexpr (SEL) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this thread's score stores have been acknowledged
        __syncthreads();
        if (tid == 0) {
            int32_t* cnt = sel.counters + b * SPECVLM_COUNTER_STRIDE;
            const int ticket = __hip_atomic_fetch_add(cnt, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const int last = ticket == nrows - 1;
            if (last) __hip_atomic_store(cnt, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            s_last = last;
        }
        __syncthreads();
        if (!s_last) return;
        // the request's W*K new candidates (at most kCandCap, checked on the host), one per thread
        const int nc = nrows * K;
        float sc = 0.f;
        if (tid < nc) {
            sc = __uint_as_float(__hip_atomic_load(reinterpret_cast<uint32_t*>(score_out + b * out_stride_b + tid),
                                                   __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
            s_cand[tid] = order_key(sc, tid);
        }
        __syncthreads();
        rank_winners(s_cand, nc, sel.M);
        const int count = min(sel.M, nc);
        if (tid < nc) {
            const int pw = pos_of(s_cand, tid);
            if (pw >= 0) {
                sel.sel_out[b * sel.M + pw] = tid + sel.index_base;
                if (sel.sel_score_out) sel.sel_score_out[b * sel.M + pw] = sc;
            }
        }
        for (int pw = count + tid; pw < sel.M; pw += kThreadsDT) {
            sel.sel_out[b * sel.M + pw] = -1;
            if (sel.sel_score_out) sel.sel_score_out[b * sel.M + pw] = -INFINITY;
        }
        if (tid == 0 && sel.count_out) sel.count_out[b] = count;
    }
}

__global__ __launch_bounds__(kThreadsDT) void draft_select_kernel(
    int C, int M, const float* __restrict__ score, int64_t score_stride_b, const int32_t* __restrict__ num_cand,
    int index_base, int32_t* __restrict__ sel_out, float* __restrict__ sel_score_out,
    int32_t* __restrict__ count_out) {
    extern __shared__ __attribute__((aligned(16))) unsigned char s_dyn[];
    unsigned long long* s_key = reinterpret_cast<unsigned long long*>(s_dyn);
    const int b = blockIdx.x, tid = threadIdx.x;
    const int c = num_cand ? min(max(num_cand[b], 0), C) : C;
    for (int i = tid; i < c; i += kThreadsDT) s_key[i] = order_key(score[b * score_stride_b + i], i);
    __syncthreads();
    rank_winners(s_key, c, M);
    const int count = min(M, c);
    for (int i = tid; i < c; i += kThreadsDT) {
        const int p = pos_of(s_key, i);
        if (p >= 0) {
            sel_out[b * M + p] = i + index_base;
            if (sel_score_out) sel_score_out[b * M + p] = score[b * score_stride_b + i];
        }
    }
    for (int p = count + tid; p < M; p += kThreadsDT) {
        sel_out[b * M + p] = -1;
        if (sel_score_out) sel_score_out[b * M + p] = -INFINITY;
    }
    if (tid == 0 && count_out) count_out[b] = count;
}

__global__ __launch_bounds__(kThreadsDT) void draft_finalize_kernel(
    int C, int N_max, const float* __restrict__ cand_score, const int32_t* __restrict__ cand_parent,
    const int32_t* __restrict__ cand_token, int64_t cand_stride_b, const int32_t* __restrict__ num_cand,
    const int32_t* __restrict__ root_token, int32_t* __restrict__ parent_out, int32_t* __restrict__ draft_tok_out,
    int32_t* __restrict__ node_cand_out, int32_t* __restrict__ num_nodes_out, int32_t* __restrict__ err_flag) {
    extern __shared__ __attribute__((aligned(16))) unsigned char s_dyn[];
    unsigned long long* s_key = reinterpret_cast<unsigned long long*>(s_dyn);
    const int b = blockIdx.x, tid = threadIdx.x;
    int err = 0;
    int c = num_cand ? num_cand[b] : C;
    if (c < 0 || c > C) {
        err |= SPECVLM_ERR_BAD_NUM_NODES;
        c = min(max(c, 0), C);
    }
    const int M = N_max - 1;
    const int64_t base = b * cand_stride_b;
    for (int i = tid; i < c; i += kThreadsDT) s_key[i] = order_key(cand_score[base + i], i);
    __syncthreads();
    rank_winners(s_key, c, M);
    const int count = min(M, c);
    for (int i = tid; i < c; i += kThreadsDT) {
        const int p = pos_of(s_key, i);
        if (p < 0) continue;
        const int cp = cand_parent[base + i];
        int pn = -1;
        if (cp < -1 || cp >= i) {
            err |= SPECVLM_ERR_BAD_PARENT;
        } else if (cp < 0) {
            pn = 0;
        } else if (pos_of(s_key, cp) < 0) {
            err |= SPECVLM_ERR_TREE_NOT_CLOSED;         // a chosen candidate whose parent was not chosen
        } else {
            pn = pos_of(s_key, cp) + 1;
        }
        const int node = p + 1;
        parent_out[b * N_max + node] = pn;
        draft_tok_out[b * N_max + node] = cand_token[base + i];
        if (node_cand_out) node_cand_out[b * N_max + node] = i;
    }
    for (int node = count + 1 + tid; node < N_max; node += kThreadsDT) {
        parent_out[b * N_max + node] = -1;
        draft_tok_out[b * N_max + node] = -1;
        if (node_cand_out) node_cand_out[b * N_max + node] = -1;
    }
    if (tid == 0) {
        parent_out[b * N_max] = -1;
        draft_tok_out[b * N_max] = root_token[b];
        if (node_cand_out) node_cand_out[b * N_max] = -1;
        num_nodes_out[b] = count + 1;
    }
    if (err && err_flag) atomicOr(err_flag, err);
}

}  // namespace

int32_t launch_draft_topk(int32_t dtype, int32_t B, int32_t W, int32_t V, int32_t K, const void* logits,
                          int64_t stride_b, int64_t stride_w, const float* cum, int64_t cum_stride_b,
                          const int32_t* parent_idx, int64_t parent_stride_b, float* score_out,
                          int32_t* token_out, int32_t* parent_out, int64_t out_stride_b, float* lse_out,
                          int32_t M, int32_t index_base, int32_t* sel_out, float* sel_score_out,
                          int32_t* count_out, int32_t* counters, hipStream_t stream) {
    const dim3 grid(W, B), block(kThreadsDT);
    const SelArgs sel{M, index_base, sel_out, sel_score_out, count_out, counters};
    const bool fused = counters != nullptr;             // with the selection of the level's candidates
#define SPECVLM_LAUNCH_TK2(T, NS, SEL)                                                                              \
    hipLaunchKernelGGL((draft_topk_kernel<T, NS, SEL>), grid, block, 0, stream, V, K, static_cast<const T*>(logits), \
                       stride_b, stride_w, cum, cum_stride_b, parent_idx, parent_stride_b, score_out,               \
                       token_out, parent_out, out_stride_b, lse_out, sel)
#define SPECVLM_LAUNCH_TK(T, NS)                                      \
    do {                                                              \
        if (fused) SPECVLM_LAUNCH_TK2(T, NS, true);                   \
        else SPECVLM_LAUNCH_TK2(T, NS, false);                        \
    } while (0)
    const int per_thread = (V + kThreadsDT - 1) / kThreadsDT;
    if (dtype == SPECVLM_BF16) {
        if (per_thread <= 32) SPECVLM_LAUNCH_TK(uint16_t, 32);
        else if (per_thread <= 64) SPECVLM_LAUNCH_TK(uint16_t, 64);
        else SPECVLM_LAUNCH_TK(uint16_t, 0);
    } else {
        if (per_thread <= 32) SPECVLM_LAUNCH_TK(float, 32);
        else if (per_thread <= 64) SPECVLM_LAUNCH_TK(float, 64);
        else SPECVLM_LAUNCH_TK(float, 0);
    }
#undef SPECVLM_LAUNCH_TK
#undef SPECVLM_LAUNCH_TK2
    return check_launch();
}

int32_t launch_draft_select(int32_t B, int32_t C, int32_t M, const float* score, int64_t score_stride_b,
                            const int32_t* num_cand, int32_t index_base, int32_t* sel_out,
                            float* sel_score_out, int32_t* count_out, hipStream_t stream) {
    const size_t lds = static_cast<size_t>((C + 1) & ~1) * 8;         // keys are ranked in pairs
    hipLaunchKernelGGL(draft_select_kernel, dim3(B), dim3(kThreadsDT), lds, stream, C, M, score, score_stride_b,
                       num_cand, index_base, sel_out, sel_score_out, count_out);
    return check_launch();
}

int32_t launch_draft_finalize(int32_t B, int32_t C, int32_t N_max, const float* cand_score,
                              const int32_t* cand_parent, const int32_t* cand_token, int64_t cand_stride_b,
                              const int32_t* num_cand, const int32_t* root_token, int32_t* parent_out,
                              int32_t* draft_tok_out, int32_t* node_cand_out, int32_t* num_nodes_out,
                              int32_t* err_flag, hipStream_t stream) {
    const size_t lds = static_cast<size_t>((C + 1) & ~1) * 8;         // keys are ranked in pairs
    hipLaunchKernelGGL(draft_finalize_kernel, dim3(B), dim3(kThreadsDT), lds, stream, C, N_max, cand_score,
                       cand_parent, cand_token, cand_stride_b, num_cand, root_token, parent_out, draft_tok_out,
                       node_cand_out, num_nodes_out, err_flag);
    return check_launch();
}

}  // namespace specvlm
