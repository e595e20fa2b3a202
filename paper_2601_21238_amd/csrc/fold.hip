// Equivalent scaling folded into the weights (Eq. 2) and symmetric per-output-channel weight
// quantization with the row sums the zero-point correction needs.
//
// HBM-bound: 4 B read + 1 B written per weight.  One WAVE owns one output row (four rows per
// block), so the two reductions of a row (absmax, then the sum of its codes) are wave shuffles with
// no block barrier.  Rows up to 4096 columns stay in registers between the two passes; longer rows
// are read a second time (from cache).
#include "common.h"

namespace stwq {

constexpr int kFoldThreads = 256;
constexpr int kFoldRows = kFoldThreads / 64;
constexpr int kFoldCached = 16;            // float4 per lane kept in registers: 64 lanes x 16 x 4 = 4096 columns

__device__ __forceinline__ float4 fold_scaled(const float4* wrow, const float4* s4, int k4) {
    float4 v = wrow[k4];
    if (s4) {
        const float4 sv = s4[k4];
        v.x *= sv.x; v.y *= sv.y; v.z *= sv.z; v.w *= sv.w;
    }
    return v;
}
__device__ __forceinline__ float absmax4(const float4& v) {
    return fmaxf(fmaxf(fabsf(v.x), fabsf(v.y)), fmaxf(fabsf(v.z), fabsf(v.w)));
}
__device__ __forceinline__ int fold_codes(const float4& v, float inv, float lo, float qw, uint32_t* out) {
    const int a = static_cast<int>(fminf(fmaxf(rintf(v.x * inv), lo), qw));
    const int b = static_cast<int>(fminf(fmaxf(rintf(v.y * inv), lo), qw));
    const int c = static_cast<int>(fminf(fmaxf(rintf(v.z * inv), lo), qw));
    const int d = static_cast<int>(fminf(fmaxf(rintf(v.w * inv), lo), qw));
    *out = (static_cast<uint32_t>(a) & 0xFFu) | ((static_cast<uint32_t>(b) & 0xFFu) << 8) |
           ((static_cast<uint32_t>(c) & 0xFFu) << 16) | (static_cast<uint32_t>(d) << 24);
    return a + b + c + d;
}

template <bool CACHED>
__global__ __launch_bounds__(kFoldThreads) void fold_kernel(
    const float* __restrict__ w, const float* __restrict__ s, int N, int K, float qw,
    int8_t* __restrict__ wq, float* __restrict__ dw, int32_t* __restrict__ wsum,
    float* __restrict__ inv_s) {
    const int tid = threadIdx.x, lane = tid & 63;
    const int o = blockIdx.x * kFoldRows + (tid >> 6);
    const int k4n = K >> 2;
    if (blockIdx.x == 0 && inv_s) {
        for (int k = tid; k < K; k += kFoldThreads) inv_s[k] = s ? 1.0f / s[k] : 1.0f;
    }
    if (o >= N) return;                              // whole waves leave; no barrier follows
    const float4* wrow = reinterpret_cast<const float4*>(w + static_cast<size_t>(o) * K);
    const float4* s4 = reinterpret_cast<const float4*>(s);

    float4 keep[CACHED ? kFoldCached : 1];
    float amax = 0.0f;
    if (CACHED) {
#pragma unroll
        for (int i = 0; i < kFoldCached; ++i) {
            const int k4 = lane + 64 * i;
            keep[i] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (k4 < k4n) keep[i] = fold_scaled(wrow, s4, k4);
            amax = fmaxf(amax, absmax4(keep[i]));
        }
    } else {
        for (int k4 = lane; k4 < k4n; k4 += 64) amax = fmaxf(amax, absmax4(fold_scaled(wrow, s4, k4)));
    }
    amax = wave_max(amax);                           // every lane holds the row's maximum
    const float d = amax > 0.0f ? amax / qw : 1.0f;  // IEEE fp32 divide
    const float inv = 1.0f / d;
    const float lo = -(qw + 1.0f);

    int sum = 0;
    uint32_t* qrow = reinterpret_cast<uint32_t*>(wq + static_cast<size_t>(o) * K);
    if (CACHED) {
#pragma unroll
        for (int i = 0; i < kFoldCached; ++i) {
            const int k4 = lane + 64 * i;
            if (k4 < k4n) sum += fold_codes(keep[i], inv, lo, qw, qrow + k4);
        }
    } else {
        for (int k4 = lane; k4 < k4n; k4 += 64) sum += fold_codes(fold_scaled(wrow, s4, k4), inv, lo, qw, qrow + k4);
    }
    sum = wave_sum(sum);
    if (lane == 0) {
        dw[o] = d;
        wsum[o] = sum;
    }
}

}  // namespace stwq

extern "C" int gps_fold_weights(const float* w_dev, const float* s_dev, int N, int K, int w_bits,
                                int8_t* wq_dev, float* dw_dev, int32_t* wsum_dev, float* inv_s_dev,
                                void* stream) {
    using namespace stwq;
    clear_error();
    STWQ_REQUIRE(w_dev && wq_dev && dw_dev && wsum_dev, "gps_fold_weights: null pointer");
    STWQ_REQUIRE(N > 0 && K > 0, "gps_fold_weights: N = %d, K = %d must be positive", N, K);
    STWQ_REQUIRE(K % 16 == 0, "gps_fold_weights: K = %d must be a multiple of 16", K);
    STWQ_REQUIRE(w_bits == 8 || w_bits == 6, "gps_fold_weights: w_bits = %d, expected 6 or 8", w_bits);
    STWQ_REQUIRE(aligned16(w_dev) && aligned16(wq_dev) && (!s_dev || aligned16(s_dev)),
                 "gps_fold_weights: w_dev, s_dev and wq_dev must be 16-byte aligned");
    const float qw = static_cast<float>((1 << (w_bits - 1)) - 1);
    const dim3 grid((N + kFoldRows - 1) / kFoldRows), block(kFoldThreads);
    if (K <= kFoldCached * 256)
        fold_kernel<true><<<grid, block, 0, static_cast<hipStream_t>(stream)>>>(w_dev, s_dev, N, K, qw, wq_dev, dw_dev, wsum_dev, inv_s_dev);
    else
        fold_kernel<false><<<grid, block, 0, static_cast<hipStream_t>(stream)>>>(w_dev, s_dev, N, K, qw, wq_dev, dw_dev, wsum_dev, inv_s_dev);
    return launch_status("fold_kernel");
}
