// Calibration statistics: per-position min / max of x * inv_s and per-channel min / max / absmax
// of x (ranges of Eq. 1; range step of the GPS algorithm; Section 4.2 offline calibration).
//
// HBM-bound: every element is read once (4 B).  A block owns a 1024-channel slab (one float4 per
// thread) and a strided set of token positions; for one position it walks all samples, so the
// per-position reduction happens once per (position, block) and channel statistics stay in
// registers until the block ends.  Merging into the caller's buffers uses integer atomics on the
// float bit patterns, which is exact and order-independent.
#include "common.h"

namespace stwq {

constexpr int kStatsThreads = 256;
constexpr int kStatsSlab = kStatsThreads * 4;   // channels per block

template <bool POS, bool CH>
__global__ __launch_bounds__(kStatsThreads) void stats_kernel(
    const float* __restrict__ x, int n_samples, int samples_per_z, int L, int C, const float* __restrict__ inv_s,
    float* __restrict__ pos_min, float* __restrict__ pos_max,
    float* __restrict__ ch_min, float* __restrict__ ch_max, float* __restrict__ ch_absmax) {
    __shared__ float red_min[kStatsThreads / 64];
    __shared__ float red_max[kStatsThreads / 64];

    const int tid = threadIdx.x;
    const int c0 = blockIdx.y * kStatsSlab + tid * 4;
    const bool active = c0 < C;
    const float inf = __builtin_inff();

    float4 is = make_float4(1.f, 1.f, 1.f, 1.f);
    if (POS && active && inv_s) is = *reinterpret_cast<const float4*>(inv_s + c0);

    float4 cmin = make_float4(inf, inf, inf, inf);
    float4 cmax = make_float4(-inf, -inf, -inf, -inf);

    const int n_begin = blockIdx.z * samples_per_z;
    const int n_end = min(n_begin + samples_per_z, n_samples);
    const size_t row_stride = static_cast<size_t>(C);
    const size_t sample_stride = static_cast<size_t>(L) * row_stride;

    for (int t = blockIdx.x; t < L; t += gridDim.x) {
        float pmin = inf, pmax = -inf;
        if (active) {
            const float* p = x + static_cast<size_t>(t) * row_stride + c0;
            int n = n_begin;
            for (; n + 4 <= n_end; n += 4) {
                float4 v[4];
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    v[u] = *reinterpret_cast<const float4*>(p + static_cast<size_t>(n + u) * sample_stride);
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    if (CH) {
                        cmin.x = fminf(cmin.x, v[u].x); cmax.x = fmaxf(cmax.x, v[u].x);
                        cmin.y = fminf(cmin.y, v[u].y); cmax.y = fmaxf(cmax.y, v[u].y);
                        cmin.z = fminf(cmin.z, v[u].z); cmax.z = fmaxf(cmax.z, v[u].z);
                        cmin.w = fminf(cmin.w, v[u].w); cmax.w = fmaxf(cmax.w, v[u].w);
                    }
                    if (POS) {
                        const float a = v[u].x * is.x, b = v[u].y * is.y, c = v[u].z * is.z, d = v[u].w * is.w;
                        pmin = fminf(pmin, fminf(fminf(a, b), fminf(c, d)));
                        pmax = fmaxf(pmax, fmaxf(fmaxf(a, b), fmaxf(c, d)));
                    }
                }
            }
            for (; n < n_end; ++n) {
                const float4 v = *reinterpret_cast<const float4*>(p + static_cast<size_t>(n) * sample_stride);
                if (CH) {
                    cmin.x = fminf(cmin.x, v.x); cmax.x = fmaxf(cmax.x, v.x);
                    cmin.y = fminf(cmin.y, v.y); cmax.y = fmaxf(cmax.y, v.y);
                    cmin.z = fminf(cmin.z, v.z); cmax.z = fmaxf(cmax.z, v.z);
                    cmin.w = fminf(cmin.w, v.w); cmax.w = fmaxf(cmax.w, v.w);
                }
                if (POS) {
                    const float a = v.x * is.x, b = v.y * is.y, c = v.z * is.z, d = v.w * is.w;
                    pmin = fminf(pmin, fminf(fminf(a, b), fminf(c, d)));
                    pmax = fmaxf(pmax, fmaxf(fmaxf(a, b), fmaxf(c, d)));
                }
            }
        }
        if (POS) {
            pmin = wave_min(pmin);
            pmax = wave_max(pmax);
            if ((tid & 63) == 0) { red_min[tid >> 6] = pmin; red_max[tid >> 6] = pmax; }
            __syncthreads();
            if (tid == 0) {
                float a = red_min[0], b = red_max[0];
#pragma unroll
                for (int w = 1; w < kStatsThreads / 64; ++w) { a = fminf(a, red_min[w]); b = fmaxf(b, red_max[w]); }
                if (a <= b) {   // false only if this slab held no channel
                    atomic_min_f32(pos_min + t, a);
                    atomic_max_f32(pos_max + t, b);
                }
            }
            __syncthreads();
        }
    }

    if (CH && active) {
        const float mn[4] = {cmin.x, cmin.y, cmin.z, cmin.w};
        const float mx[4] = {cmax.x, cmax.y, cmax.z, cmax.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (mn[j] > mx[j]) continue;   // this block saw no row
            if (ch_min) atomic_min_f32(ch_min + c0 + j, mn[j]);
            if (ch_max) atomic_max_f32(ch_max + c0 + j, mx[j]);
            if (ch_absmax) atomic_max_f32(ch_absmax + c0 + j, fmaxf(fabsf(mn[j]), fabsf(mx[j])));
        }
    }
}

// Channel statistics alone (no position structure needed): a block covers 256 channels (one float4
// per lane) and a contiguous chunk of rows; its four waves take rows 0,1,2,3 mod 4 of the chunk and
// merge through LDS, so only one wave per block touches the global buffers (256 x 3 atomics).
constexpr int kChanThreads = 256;
constexpr int kChanUnroll = 4;

__global__ __launch_bounds__(kChanThreads) void channel_stats_kernel(
    const float* __restrict__ x, long long rows, int C, long long rows_per_block,
    float* __restrict__ ch_min, float* __restrict__ ch_max, float* __restrict__ ch_absmax) {
    __shared__ float4 s_min[kChanThreads];
    __shared__ float4 s_max[kChanThreads];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c0 = blockIdx.y * 256 + lane * 4;
    const bool active = c0 < C;
    const float inf = __builtin_inff();
    float4 cmin = make_float4(inf, inf, inf, inf);
    float4 cmax = make_float4(-inf, -inf, -inf, -inf);
    const long long r0 = blockIdx.x * rows_per_block;
    const long long r1 = min(r0 + rows_per_block, rows);
    if (active) {
        const float* p = x + c0;
        long long r = r0 + wave;
        for (; r + 4 * (kChanUnroll - 1) < r1; r += 4 * kChanUnroll) {
            float4 v[kChanUnroll];
#pragma unroll
            for (int u = 0; u < kChanUnroll; ++u) v[u] = *reinterpret_cast<const float4*>(p + (r + 4 * u) * C);
#pragma unroll
            for (int u = 0; u < kChanUnroll; ++u) {
                cmin.x = fminf(cmin.x, v[u].x); cmax.x = fmaxf(cmax.x, v[u].x);
                cmin.y = fminf(cmin.y, v[u].y); cmax.y = fmaxf(cmax.y, v[u].y);
                cmin.z = fminf(cmin.z, v[u].z); cmax.z = fmaxf(cmax.z, v[u].z);
                cmin.w = fminf(cmin.w, v[u].w); cmax.w = fmaxf(cmax.w, v[u].w);
            }
        }
        for (; r < r1; r += 4) {
            const float4 v = *reinterpret_cast<const float4*>(p + r * C);
            cmin.x = fminf(cmin.x, v.x); cmax.x = fmaxf(cmax.x, v.x);
            cmin.y = fminf(cmin.y, v.y); cmax.y = fmaxf(cmax.y, v.y);
            cmin.z = fminf(cmin.z, v.z); cmax.z = fmaxf(cmax.z, v.z);
            cmin.w = fminf(cmin.w, v.w); cmax.w = fmaxf(cmax.w, v.w);
        }
    }
    s_min[tid] = cmin;
    s_max[tid] = cmax;
    __syncthreads();
    if (wave != 0 || !active) return;
#pragma unroll
    for (int w = 1; w < kChanThreads / 64; ++w) {
        const float4 a = s_min[w * 64 + lane], b = s_max[w * 64 + lane];
        cmin.x = fminf(cmin.x, a.x); cmin.y = fminf(cmin.y, a.y); cmin.z = fminf(cmin.z, a.z); cmin.w = fminf(cmin.w, a.w);
        cmax.x = fmaxf(cmax.x, b.x); cmax.y = fmaxf(cmax.y, b.y); cmax.z = fmaxf(cmax.z, b.z); cmax.w = fmaxf(cmax.w, b.w);
    }
    const float mn[4] = {cmin.x, cmin.y, cmin.z, cmin.w};
    const float mx[4] = {cmax.x, cmax.y, cmax.z, cmax.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        if (mn[j] > mx[j]) continue;   // this block saw no row
        if (ch_min) atomic_min_f32(ch_min + c0 + j, mn[j]);
        if (ch_max) atomic_max_f32(ch_max + c0 + j, mx[j]);
        if (ch_absmax) atomic_max_f32(ch_absmax + c0 + j, fmaxf(fabsf(mn[j]), fabsf(mx[j])));
    }
}

}  // namespace stwq

extern "C" int stwq_calibrate_stats(const float* x_dev, int64_t rows, int L, int C,
                                    const float* inv_s_dev,
                                    float* pos_min_dev, float* pos_max_dev,
                                    float* ch_min_dev, float* ch_max_dev, float* ch_absmax_dev,
                                    void* stream) {
    using namespace stwq;
    clear_error();
    STWQ_REQUIRE(x_dev, "stwq_calibrate_stats: x_dev is null");
    STWQ_REQUIRE(L > 0 && C > 0 && rows > 0, "stwq_calibrate_stats: rows = %lld, L = %d, C = %d must be positive",
                 static_cast<long long>(rows), L, C);
    STWQ_REQUIRE(rows % L == 0, "stwq_calibrate_stats: rows = %lld is not a multiple of L = %d",
                 static_cast<long long>(rows), L);
    STWQ_REQUIRE(rows / L <= INT32_MAX, "stwq_calibrate_stats: too many samples");
    STWQ_REQUIRE(C % 4 == 0, "stwq_calibrate_stats: C = %d must be a multiple of 4", C);
    STWQ_REQUIRE(aligned16(x_dev) && (!inv_s_dev || aligned16(inv_s_dev)),
                 "stwq_calibrate_stats: x_dev and inv_s_dev must be 16-byte aligned");
    STWQ_REQUIRE((pos_min_dev == nullptr) == (pos_max_dev == nullptr),
                 "stwq_calibrate_stats: give both pos_min_dev and pos_max_dev or neither");
    const bool pos = pos_min_dev != nullptr;
    const bool ch = ch_min_dev || ch_max_dev || ch_absmax_dev;
    STWQ_REQUIRE(pos || ch, "stwq_calibrate_stats: no output buffer given");

    const int n_samples = static_cast<int>(rows / L);
    const int slabs = (C + kStatsSlab - 1) / kStatsSlab;
    int gx = 2048 / slabs;                 // about eight 256-thread blocks per CU over 256 CUs
    if (gx < 1) gx = 1;
    if (gx > L) gx = L;
    // few positions (a decode table slice, L = 1): split the samples over blockIdx.z instead
    int gz = 1;
    if (gx * slabs < 1024) {
        gz = 2048 / (gx * slabs);
        const int max_gz = (n_samples + 7) / 8;      // at least eight samples per block
        if (gz > max_gz) gz = max_gz;
        if (gz < 1) gz = 1;
    }
    const int spz = (n_samples + gz - 1) / gz;
    gz = (n_samples + spz - 1) / spz;
    dim3 grid(gx, slabs, gz), block(kStatsThreads);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (pos && ch)
        stats_kernel<true, true><<<grid, block, 0, s>>>(x_dev, n_samples, spz, L, C, inv_s_dev, pos_min_dev, pos_max_dev,
                                                        ch_min_dev, ch_max_dev, ch_absmax_dev);
    else if (pos)
        stats_kernel<true, false><<<grid, block, 0, s>>>(x_dev, n_samples, spz, L, C, inv_s_dev, pos_min_dev, pos_max_dev,
                                                         nullptr, nullptr, nullptr);
    else {
        // channel statistics only: about one block per CU (256 channels x a chunk of rows each).  More blocks
        // means more atomic merges into the same 3 C words, and those, not the reads, then set the time
        // (measured on 21760 x 1024: 256 blocks 18 us, 1024 blocks 37 us, 2048 blocks 65 us).
        const int cslabs = (C + 255) / 256;
        long long chunks = 256 / cslabs;
        if (chunks < 1) chunks = 1;
        long long rpb = (rows + chunks - 1) / chunks;
        if (rpb < 4 * kChanUnroll) rpb = 4 * kChanUnroll;
        chunks = (rows + rpb - 1) / rpb;
        STWQ_REQUIRE(cslabs <= 65535, "stwq_calibrate_stats: C = %d is too large", C);
        channel_stats_kernel<<<dim3(static_cast<unsigned>(chunks), cslabs), dim3(kChanThreads), 0, s>>>(
            x_dev, rows, C, rpb, ch_min_dev, ch_max_dev, ch_absmax_dev);
        return launch_status("channel_stats_kernel");
    }
    return launch_status("stats_kernel");
}
