// Equivalent scaling folded into the weights (Eq. 2) and symmetric per-output-channel weight
// quantization with the row sums the zero-point correction needs.
//
// HBM-bound: 4 B read + 1 B written per weight.  One 256-thread block owns one output row; the
// row is read twice (absmax, then codes), the second time from cache.
#include "common.h"

namespace stwq {

constexpr int kFoldThreads = 256;

__global__ __launch_bounds__(kFoldThreads) void fold_kernel(
    const float* __restrict__ w, const float* __restrict__ s, int K, float qw,
    int8_t* __restrict__ wq, float* __restrict__ dw, int32_t* __restrict__ wsum,
    float* __restrict__ inv_s) {
    __shared__ float red_f[kFoldThreads / 64];
    __shared__ int red_i[kFoldThreads / 64];
    __shared__ float inv_shared;

    const int tid = threadIdx.x;
    const int o = blockIdx.x;
    const int k4n = K >> 2;
    const float4* wrow = reinterpret_cast<const float4*>(w + static_cast<size_t>(o) * K);
    const float4* s4 = reinterpret_cast<const float4*>(s);

    if (o == 0 && inv_s) {
        for (int k = tid; k < K; k += kFoldThreads) inv_s[k] = s ? 1.0f / s[k] : 1.0f;
    }

    float amax = 0.0f;
    for (int k4 = tid; k4 < k4n; k4 += kFoldThreads) {
        float4 v = wrow[k4];
        if (s) {
            const float4 sv = s4[k4];
            v.x *= sv.x; v.y *= sv.y; v.z *= sv.z; v.w *= sv.w;
        }
        amax = fmaxf(amax, fmaxf(fmaxf(fabsf(v.x), fabsf(v.y)), fmaxf(fabsf(v.z), fabsf(v.w))));
    }
    amax = wave_max(amax);
    if ((tid & 63) == 0) red_f[tid >> 6] = amax;
    __syncthreads();
    if (tid == 0) {
        float a = red_f[0];
#pragma unroll
        for (int i = 1; i < kFoldThreads / 64; ++i) a = fmaxf(a, red_f[i]);
        const float d = a > 0.0f ? a / qw : 1.0f;     // IEEE fp32 divide
        dw[o] = d;
        inv_shared = 1.0f / d;
    }
    __syncthreads();
    const float inv = inv_shared;
    const float lo = -(qw + 1.0f);

    int sum = 0;
    uint32_t* qrow = reinterpret_cast<uint32_t*>(wq + static_cast<size_t>(o) * K);
    for (int k4 = tid; k4 < k4n; k4 += kFoldThreads) {
        float4 v = wrow[k4];
        if (s) {
            const float4 sv = s4[k4];
            v.x *= sv.x; v.y *= sv.y; v.z *= sv.z; v.w *= sv.w;
        }
        const int a = static_cast<int>(fminf(fmaxf(rintf(v.x * inv), lo), qw));
        const int b = static_cast<int>(fminf(fmaxf(rintf(v.y * inv), lo), qw));
        const int c = static_cast<int>(fminf(fmaxf(rintf(v.z * inv), lo), qw));
        const int d = static_cast<int>(fminf(fmaxf(rintf(v.w * inv), lo), qw));
        sum += a + b + c + d;
        qrow[k4] = (static_cast<uint32_t>(a) & 0xFFu) | ((static_cast<uint32_t>(b) & 0xFFu) << 8) |
                   ((static_cast<uint32_t>(c) & 0xFFu) << 16) | (static_cast<uint32_t>(d) << 24);
    }
    sum = wave_sum(sum);
    if ((tid & 63) == 0) red_i[tid >> 6] = sum;
    __syncthreads();
    if (tid == 0) {
        int t = 0;
#pragma unroll
        for (int i = 0; i < kFoldThreads / 64; ++i) t += red_i[i];
        wsum[o] = t;
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
    fold_kernel<<<dim3(N), dim3(kFoldThreads), 0, static_cast<hipStream_t>(stream)>>>(
        w_dev, s_dev, K, qw, wq_dev, dw_dev, wsum_dev, inv_s_dev);
    return launch_status("fold_kernel");
}
