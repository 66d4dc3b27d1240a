// Parameter-free visual token compressors of the draft side (SpecVLM Sec. 3.4, the elastic
// vision compressor's parameter-free experts: pruning discards a random subset of the visual tokens,
// pooling is a plain pooling operator; Table 4 evaluates ratios 2x .. 30x).  They
// shorten the visual prefix the draft reads; the target keeps the full sequence.
//
//   pool   y[b,j,:] = mean of x[b, j*ratio .. min((j+1)*ratio, T_b) - 1, :]   (fp32 sum, one rounding)
//   prune  y[b,j,:] = x[b, keep[b,j], :]                                       (bit copy)
//
// Both stream [tokens, E] feature rows once: HBM-bound, 16 bytes per lane per access, one
// workgroup per output row -- or per segment of it when there are few rows -- (a row of 4096 bf16
// features is 8 KB), source rows of a window read back to back so that a window is one contiguous span.
#include "common.hpp"

namespace specvlm {

namespace {

constexpr int kCompThreads = 256;

// 16 bytes that are read once: a non-temporal load (no point in keeping the line in a cache).
__device__ __forceinline__ uint4 load_once(const void* p) {
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    const u32x4 v = __builtin_nontemporal_load(static_cast<const u32x4*>(p));
    return uint4{v[0], v[1], v[2], v[3]};
}

template <typename T>
struct Vec16;
template <>
struct Vec16<uint16_t> {
    static constexpr int kPer = 8;
    __device__ static void add(float (&acc)[8], const uint4& w) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const uint32_t x = (&w.x)[e];
            acc[2 * e] += __uint_as_float(x << 16);
            acc[2 * e + 1] += __uint_as_float(x & 0xFFFF0000u);
        }
    }
    __device__ static uint4 pack(const float (&acc)[8], float scale) {
        uint4 w;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            typedef float f32x2 __attribute__((ext_vector_type(2)));
            typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
            const f32x2 f = {acc[2 * e] * scale, acc[2 * e + 1] * scale};
            const bf16x2 h = __builtin_convertvector(f, bf16x2);          // round to nearest even
            (&w.x)[e] = __builtin_bit_cast(uint32_t, h);
        }
        return w;
    }
};
template <>
struct Vec16<float> {
    static constexpr int kPer = 4;
    __device__ static void add(float (&acc)[8], const uint4& w) {
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[e] += __uint_as_float((&w.x)[e]);
    }
    __device__ static uint4 pack(const float (&acc)[8], float scale) {
        uint4 w;
#pragma unroll
        for (int e = 0; e < 4; ++e) (&w.x)[e] = __float_as_uint(acc[e] * scale);
        return w;
    }
};

template <typename T>
__global__ __launch_bounds__(kCompThreads) void visual_pool_kernel(
    int T_max, int E, int ratio, const T* __restrict__ x, int64_t x_sb, int64_t x_st,
    const int32_t* __restrict__ num_tokens, T* __restrict__ y, int64_t y_sb, int64_t y_st,
    int32_t* __restrict__ out_tokens, int32_t* __restrict__ err_flag) {
    const int j = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
    int tb = num_tokens ? num_tokens[b] : T_max;
    if (tb < 0 || tb > T_max) {
        if (tid == 0 && j == 0 && err_flag) atomicOr(err_flag, SPECVLM_ERR_BAD_LENGTH);
        tb = min(max(tb, 0), T_max);
    }
    const int nb = (tb + ratio - 1) / ratio;
    if (j == 0 && tid == 0 && out_tokens) out_tokens[b] = nb;
    if (j >= nb) return;                                      // rows past the request's pooled length: untouched
    const int t0 = j * ratio, t1 = min(t0 + ratio, tb);
    const float scale = 1.0f / static_cast<float>(t1 - t0);
    constexpr int PER = Vec16<T>::kPer;
    const T* src = x + b * x_sb;
    T* dst = y + b * y_sb + j * y_st;
    // blockIdx.z picks one of gridDim.z equal segments of the feature row (few output rows would
    // otherwise leave compute units without a workgroup)
    const int seg = E / gridDim.z, e_lo = blockIdx.z * seg, e_hi = e_lo + seg;
    for (int e0 = e_lo + tid * PER; e0 < e_hi; e0 += kCompThreads * PER) {
        float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        int t = t0;
        for (; t + 10 <= t1; t += 10) {                       // ten, then four independent loads in flight
            uint4 w[10];
#pragma unroll
            for (int u = 0; u < 10; ++u) w[u] = load_once(src + (t + u) * x_st + e0);
#pragma unroll
            for (int u = 0; u < 10; ++u) Vec16<T>::add(acc, w[u]);
        }
        for (; t + 4 <= t1; t += 4) {
            uint4 w[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) w[u] = load_once(src + (t + u) * x_st + e0);
#pragma unroll
            for (int u = 0; u < 4; ++u) Vec16<T>::add(acc, w[u]);
        }
        for (; t < t1; ++t) Vec16<T>::add(acc, load_once(src + t * x_st + e0));
        *reinterpret_cast<uint4*>(dst + e0) = Vec16<T>::pack(acc, scale);
    }
}

__global__ __launch_bounds__(kCompThreads) void visual_prune_kernel(
    int T, int T_keep, int row_bytes, const unsigned char* __restrict__ x, int64_t x_sb_bytes, int64_t x_st_bytes,
    const int32_t* __restrict__ keep, unsigned char* __restrict__ y, int64_t y_sb_bytes, int64_t y_st_bytes,
    int32_t* __restrict__ err_flag) {
    const int j = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
    const int t = keep[b * T_keep + j];
    if (t == -1) return;                                      // padding: the row is left untouched
    if (t < 0 || t >= T) {
        if (tid == 0 && err_flag) atomicOr(err_flag, SPECVLM_ERR_BAD_LENGTH);
        return;
    }
    const unsigned char* src = x + b * x_sb_bytes + t * x_st_bytes;
    unsigned char* dst = y + b * y_sb_bytes + j * y_st_bytes;
    for (int o = tid * 16; o < row_bytes; o += kCompThreads * 16)
        *reinterpret_cast<uint4*>(dst + o) = *reinterpret_cast<const uint4*>(src + o);
}

}  // namespace

int32_t launch_visual_pool(int32_t dtype, int32_t B, int32_t T, int32_t E, int32_t ratio, const void* x,
                           int64_t x_sb, int64_t x_st, const int32_t* num_tokens, void* y, int64_t y_sb,
                           int64_t y_st, int32_t* out_tokens, int32_t* err_flag, hipStream_t stream) {
    const int rows = (T + ratio - 1) / ratio, per = dtype == SPECVLM_BF16 ? 8 : 4;
    int segs = 1;
    while (segs < 8 && static_cast<long>(rows) * B * segs < 1024 && E % (2 * segs * per) == 0) segs *= 2;
    const dim3 grid(rows, B, segs), block(kCompThreads);
    if (dtype == SPECVLM_BF16)
        hipLaunchKernelGGL(visual_pool_kernel<uint16_t>, grid, block, 0, stream, T, E, ratio,
                           static_cast<const uint16_t*>(x), x_sb, x_st, num_tokens, static_cast<uint16_t*>(y), y_sb,
                           y_st, out_tokens, err_flag);
    else
        hipLaunchKernelGGL(visual_pool_kernel<float>, grid, block, 0, stream, T, E, ratio,
                           static_cast<const float*>(x), x_sb, x_st, num_tokens, static_cast<float*>(y), y_sb, y_st,
                           out_tokens, err_flag);
    return check_launch();
}

int32_t launch_visual_prune(int32_t elem_bytes, int32_t B, int32_t T, int32_t T_keep, int32_t E, const void* x,
                            int64_t x_sb, int64_t x_st, const int32_t* keep, void* y, int64_t y_sb, int64_t y_st,
                            int32_t* err_flag, hipStream_t stream) {
    hipLaunchKernelGGL(visual_prune_kernel, dim3(T_keep, B), dim3(kCompThreads), 0, stream, T, T_keep,
                       E * elem_bytes, static_cast<const unsigned char*>(x), x_sb * elem_bytes, x_st * elem_bytes, keep,
                       static_cast<unsigned char*>(y), y_sb * elem_bytes, y_st * elem_bytes, err_flag);
    return check_launch();
}

}  // namespace specvlm
