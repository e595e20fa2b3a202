// The quantized linear layer: int8 x int8 -> int32 product on the MFMA units and the dequantizing
// epilogue (Appendix A.1: xhat = delta (xbar - z)) that writes bf16.
//
//   acc[m,o] = sum_k q[m,k] * wq[o,k]
//   y[m,o]   = bf16( float(acc - (z_t - off) * wsum[o]) * (delta_t * dw[o]) + bias[o] ),  t = m mod L
//
// Operand roles are swapped with respect to the usual "activations are A": the WEIGHT tile is the
// MFMA A operand (its rows become rows of D) and the TOKEN tile is the B operand (its rows become
// columns of D).  With v_mfma_i32_32x32x32_i8 a lane then owns one token (one delta_t, z_t) and
// runs of four consecutive output channels, which are contiguous in the row-major [M, N] output.
// Inside one MFMA both operands take the same 16-byte K chunk per lane, and integer sums commute,
// so any consistent assignment of K chunks to lanes gives the exact result.
#include "common.h"

namespace stwq {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float f2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

struct LinearArgs {
    const int8_t* q;
    const int8_t* wq;
    const float* dw;
    const int32_t* wsum;
    const float* delta;
    const int32_t* zp;
    const float* bias;
    uint16_t* y;
    int32_t* acc_dbg;
    int M, K, N, L, off;
};

__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
    f2 v = {a, b};
    bf16x2 r = __builtin_convertvector(v, bf16x2);      // v_cvt_pk_bf16_f32: round to nearest even
    return *reinterpret_cast<uint32_t*>(&r);
}

// Dequantizes four accumulators of one token (consecutive output channels o4 .. o4+3) and stores
// them.  The integer correction is exact: |z_t - off| <= 128 and |wsum| <= 127 K < 2^23 (K <= 65536)
// fit the 24-bit multiplier, and the difference fits int32.  The rest is fp32.
__device__ __forceinline__ void epilogue_store4(const LinearArgs& p, long long m, int o4, int a0, int a1, int a2,
                                                int a3, float dt, int zs, const float4& dwv, const int4& wsv,
                                                const float4& bv) {
    if (p.acc_dbg) *reinterpret_cast<int4*>(p.acc_dbg + m * p.N + o4) = make_int4(a0, a1, a2, a3);
    const float y0 = fmaf(static_cast<float>(a0 - __mul24(zs, wsv.x)), dt * dwv.x, bv.x);
    const float y1 = fmaf(static_cast<float>(a1 - __mul24(zs, wsv.y)), dt * dwv.y, bv.y);
    const float y2 = fmaf(static_cast<float>(a2 - __mul24(zs, wsv.z)), dt * dwv.z, bv.z);
    const float y3 = fmaf(static_cast<float>(a3 - __mul24(zs, wsv.w)), dt * dwv.w, bv.w);
    uint2 out;
    out.x = pack_bf16(y0, y1);
    out.y = pack_bf16(y2, y3);
    *reinterpret_cast<uint2*>(p.y + m * p.N + o4) = out;
}

// ------------------------------------------------------------------------------------------------
// Generic kernel: one wave per 32 x 32 output tile, operands straight from global memory.
// Serves shapes the tiled kernels do not take (K not a multiple of their K step) and is the
// simplest statement of the lane layout the others share.
// ------------------------------------------------------------------------------------------------
constexpr int kSimpleThreads = 256;

__global__ __launch_bounds__(kSimpleThreads) void linear_simple_kernel(LinearArgs p) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l32 = lane & 31, hi = lane >> 5;
    const long long m_base = static_cast<long long>(blockIdx.x) * 64 + (wave >> 1) * 32;
    const int o_base = blockIdx.y * 64 + (wave & 1) * 32;
    const long long row_m = m_base + l32;
    const int row_o = o_base + l32;
    const bool m_ok = row_m < p.M, o_ok = row_o < p.N;
    const int8_t* pa = p.wq + static_cast<size_t>(o_ok ? row_o : 0) * p.K + hi * 16;
    const int8_t* pb = p.q + static_cast<size_t>(m_ok ? row_m : 0) * p.K + hi * 16;

    v16i acc = {0};
    for (int k0 = 0; k0 < p.K; k0 += 32) {
        const bool k_ok = k0 + hi * 16 < p.K;          // K is a multiple of 16, not necessarily of 32
        v4i a = {0, 0, 0, 0}, b = {0, 0, 0, 0};
        if (o_ok && k_ok) a = *reinterpret_cast<const v4i*>(pa + k0);
        if (m_ok && k_ok) b = *reinterpret_cast<const v4i*>(pb + k0);
        acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, acc, 0, 0, 0);
    }

    // D layout of the 32 x 32 MFMA: lane holds column (lane % 32); register r holds row
    // 8 * (r / 4) + 4 * (lane / 32) + r % 4.
    if (!m_ok) return;
    const int t = static_cast<int>(row_m % p.L);
    const float dt = p.delta[t];
    const int zs = p.zp[t] - p.off;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        const int o4 = o_base + 8 * g + 4 * hi;
        if (o4 >= p.N) continue;                        // N is a multiple of 8: a group is all in or all out
        const float4 dwv = *reinterpret_cast<const float4*>(p.dw + o4);
        const int4 wsv = *reinterpret_cast<const int4*>(p.wsum + o4);
        float4 bv = make_float4(0.f, 0.f, 0.f, 0.f);
        if (p.bias) bv = *reinterpret_cast<const float4*>(p.bias + o4);
        epilogue_store4(p, row_m, o4, acc[4 * g], acc[4 * g + 1], acc[4 * g + 2], acc[4 * g + 3], dt, zs, dwv, wsv, bv);
    }
}

// ------------------------------------------------------------------------------------------------
// Prefill kernel: 256 (output channels) x 256 (tokens) block tile, K step 128, 8 waves in a
// 2 x 4 grid (wave tile 128 x 64 = 4 x 2 MFMA tiles, 128 int32 accumulators per lane).  Both
// operand tiles are staged in LDS by direct global -> LDS loads (no register staging), double
// buffered; MFMA operands are read back with ds_read_b128.
//
// LDS layout of one operand tile: 256 rows x 128 bytes; the eight 16-byte chunks of row r are
// permuted by chunk ^ ((r >> 1) & 7), which spreads the sixteen rows a ds_read_b128 touches per
// pass over all banks.  A direct-to-LDS load writes lane i's 16 bytes at base + 16 * i, so the
// permutation is applied on the global side: the lane that fills physical chunk pc of row r
// fetches logical chunk pc ^ ((r >> 1) & 7).
//
// Rows past the end of either matrix are clamped to the last valid row: their products land in
// accumulators that are never stored.
// ------------------------------------------------------------------------------------------------
constexpr int kTile = 256;
constexpr int kBK = 128;
constexpr int kPrefillThreads = 512;
constexpr int kStageBytes = kTile * kBK;   // one operand, one stage: 32 KB

typedef __attribute__((address_space(3))) void lds_void;
typedef const __attribute__((address_space(1))) void global_void;

__device__ __forceinline__ void load_tile_to_lds(const int8_t* const (&src)[4], int k0, int8_t* stage, int wave) {
#pragma unroll
    for (int pss = 0; pss < 4; ++pss) {
        int8_t* dst = stage + (pss * 64 + wave * 8) * kBK;     // wave-uniform; lane i lands at dst + 16 i
        __builtin_amdgcn_global_load_lds((global_void*)(src[pss] + k0), (lds_void*)dst, 16, 0, 0);
    }
    // keep the prefetch where it is written: ahead of the MFMA work that hides its latency
    __builtin_amdgcn_sched_barrier(0);
}

__device__ __forceinline__ void compute_stage(const int8_t* sW, const int8_t* sX, const int (&offA)[4],
                                              const int (&offB)[4], v16i (&acc)[4][2]) {
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
        v4i a[4], b[2];
#pragma unroll
        for (int i = 0; i < 4; ++i) a[i] = *reinterpret_cast<const v4i*>(sW + offA[ks] + i * 32 * kBK);
#pragma unroll
        for (int j = 0; j < 2; ++j) b[j] = *reinterpret_cast<const v4i*>(sX + offB[ks] + j * 32 * kBK);
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i], b[j], acc[i][j], 0, 0, 0);
    }
}

__global__ __launch_bounds__(kPrefillThreads) void linear_prefill_kernel(LinearArgs p, int tiles_o, int n_blocks) {
    __shared__ __attribute__((aligned(1024))) int8_t sW0[kStageBytes];
    __shared__ __attribute__((aligned(1024))) int8_t sW1[kStageBytes];
    __shared__ __attribute__((aligned(1024))) int8_t sX0[kStageBytes];
    __shared__ __attribute__((aligned(1024))) int8_t sX1[kStageBytes];

    // Workgroups are dealt round-robin to the 8 XCDs, each with its own L2.  Renumber them so
    // that one XCD works on consecutive tiles (same token rows, neighbouring weight columns).
    const int bid = blockIdx.x;
    const int xcd = bid & 7, per = n_blocks >> 3, rem = n_blocks & 7;
    const int logical = xcd * per + min(xcd, rem) + (bid >> 3);
    const int tile_m = logical / tiles_o, tile_o = logical - tile_m * tiles_o;
    const long long m0 = static_cast<long long>(tile_m) * kTile;
    const int o0 = tile_o * kTile;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, hi = lane >> 5;
    const int wo = wave & 1, wm = wave >> 1;

    // global sources of this lane's four 16-byte pieces per operand
    const int8_t* srcW[4];
    const int8_t* srcX[4];
#pragma unroll
    for (int pss = 0; pss < 4; ++pss) {
        const int r = pss * 64 + wave * 8 + (lane >> 3);
        const int lc = (lane & 7) ^ ((r >> 1) & 7);
        const int ro = min(o0 + r, p.N - 1);
        const long long rm = min(m0 + r, static_cast<long long>(p.M) - 1);
        srcW[pss] = p.wq + static_cast<size_t>(ro) * p.K + lc * 16;
        srcX[pss] = p.q + static_cast<size_t>(rm) * p.K + lc * 16;
    }

    // LDS byte offsets of this lane's MFMA operands for the four K steps of a stage
    int offA[4], offB[4];
    const int swz = (l32 >> 1) & 7;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
        const int pc = ((ks * 2 + hi) ^ swz) * 16;
        offA[ks] = (wo * 128 + l32) * kBK + pc;
        offB[ks] = (wm * 64 + l32) * kBK + pc;
    }

    v16i acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = (v16i){0};

    const int nk = p.K / kBK;
    load_tile_to_lds(srcW, 0, sW0, wave);
    load_tile_to_lds(srcX, 0, sX0, wave);
    int it = 0;
    for (; it + 2 <= nk; it += 2) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        load_tile_to_lds(srcW, (it + 1) * kBK, sW1, wave);
        load_tile_to_lds(srcX, (it + 1) * kBK, sX1, wave);
        compute_stage(sW0, sX0, offA, offB, acc);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (it + 2 < nk) {
            load_tile_to_lds(srcW, (it + 2) * kBK, sW0, wave);
            load_tile_to_lds(srcX, (it + 2) * kBK, sX0, wave);
        }
        compute_stage(sW1, sX1, offA, offB, acc);
    }
    if (it < nk) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        compute_stage(sW0, sX0, offA, offB, acc);
    }

    // epilogue
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const long long m = m0 + wm * 64 + j * 32 + l32;
        if (m >= p.M) continue;
        const int t = static_cast<int>(m % p.L);
        const float dt = p.delta[t];
        const int zs = p.zp[t] - p.off;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int o4 = o0 + wo * 128 + i * 32 + 8 * g + 4 * hi;
                if (o4 >= p.N) continue;
                const float4 dwv = *reinterpret_cast<const float4*>(p.dw + o4);
                const int4 wsv = *reinterpret_cast<const int4*>(p.wsum + o4);
                float4 bv = make_float4(0.f, 0.f, 0.f, 0.f);
                if (p.bias) bv = *reinterpret_cast<const float4*>(p.bias + o4);
                epilogue_store4(p, m, o4, acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2],
                                acc[i][j][4 * g + 3], dt, zs, dwv, wsv, bv);
            }
        }
    }
}

static int check_linear_args(const char* who, const int8_t* q, int64_t M, int K, int N, int L, const int8_t* wq,
                             const float* dw, const int32_t* wsum, const float* delta, const int32_t* zp, int a_bits,
                             const float* bias, const uint16_t* y, const int32_t* acc_dbg) {
    STWQ_REQUIRE(q && wq && dw && wsum && delta && zp && y, "%s: null pointer", who);
    STWQ_REQUIRE(M > 0 && K > 0 && N > 0 && L > 0, "%s: M = %lld, K = %d, N = %d, L = %d must be positive", who,
                 static_cast<long long>(M), K, N, L);
    STWQ_REQUIRE(M <= 0x7FFFFFFFLL, "%s: M = %lld is too large", who, static_cast<long long>(M));
    STWQ_REQUIRE(K % 16 == 0, "%s: K = %d must be a multiple of 16", who, K);
    STWQ_REQUIRE(N % 8 == 0, "%s: N = %d must be a multiple of 8", who, N);
    STWQ_REQUIRE(K <= 65536, "%s: K = %d exceeds 65536 (row sums must stay below 2^23)", who, K);
    STWQ_REQUIRE(a_bits == 8 || a_bits == 6, "%s: a_bits = %d, expected 6 or 8", who, a_bits);
    STWQ_REQUIRE(aligned16(q) && aligned16(wq) && aligned16(dw) && aligned16(wsum) && aligned16(y) &&
                     (!bias || aligned16(bias)) && (!acc_dbg || aligned16(acc_dbg)),
                 "%s: q, wq, dw, wsum, bias, y and acc_dbg must be 16-byte aligned", who);
    return STWQ_OK;
}

}  // namespace stwq

static int launch_linear(const stwq::LinearArgs& p, int schedule, hipStream_t s) {
    using namespace stwq;
    const long long M = p.M;
    const bool tiled_ok = p.K % kBK == 0;
    if (schedule == STWQ_SCHEDULE_AUTO) schedule = (tiled_ok && M >= 256) ? STWQ_SCHEDULE_PREFILL : STWQ_SCHEDULE_GENERIC;
    if (schedule == STWQ_SCHEDULE_PREFILL) {
        if (!tiled_ok) return fail(STWQ_EUNSUPPORTED, "stwq_linear: the prefill schedule needs K %% %d == 0 (K = %d)", kBK, p.K);
        const int tiles_o = (p.N + kTile - 1) / kTile;
        const long long n_blocks = ((M + kTile - 1) / kTile) * tiles_o;
        STWQ_REQUIRE(n_blocks <= 0x7FFFFFFFLL, "stwq_linear: too many tiles");
        linear_prefill_kernel<<<dim3(static_cast<unsigned>(n_blocks)), dim3(kPrefillThreads), 0, s>>>(
            p, tiles_o, static_cast<int>(n_blocks));
        return launch_status("linear_prefill_kernel");
    }
    if (schedule == STWQ_SCHEDULE_GENERIC) {
        const long long gx = (M + 63) / 64;
        const int gy = (p.N + 63) / 64;
        STWQ_REQUIRE(gy <= 65535, "stwq_linear: N = %d is too large for the generic schedule", p.N);
        linear_simple_kernel<<<dim3(static_cast<unsigned>(gx), gy), dim3(kSimpleThreads), 0, s>>>(p);
        return launch_status("linear_simple_kernel");
    }
    return fail(STWQ_EINVAL, "stwq_linear: unknown schedule %d", schedule);
}

extern "C" int stwq_linear_ex(const int8_t* q_dev, int64_t M, int K, int N, int L,
                              const int8_t* wq_dev, const float* dw_dev, const int32_t* wsum_dev,
                              const float* delta_dev, const int32_t* zp_dev, int a_bits,
                              const float* bias_dev,
                              uint16_t* y_bf16_dev, int32_t* acc_dbg_dev, int schedule, void* stream) {
    using namespace stwq;
    clear_error();
    const int rc = check_linear_args("stwq_linear", q_dev, M, K, N, L, wq_dev, dw_dev, wsum_dev, delta_dev, zp_dev,
                                     a_bits, bias_dev, y_bf16_dev, acc_dbg_dev);
    if (rc != STWQ_OK) return rc;
    LinearArgs p{q_dev, wq_dev, dw_dev, wsum_dev, delta_dev, zp_dev, bias_dev, y_bf16_dev, acc_dbg_dev,
                 static_cast<int>(M), K, N, L, a_bits == 8 ? 128 : 0};
    return launch_linear(p, schedule, static_cast<hipStream_t>(stream));
}

extern "C" int stwq_linear(const int8_t* q_dev, int64_t M, int K, int N, int L,
                           const int8_t* wq_dev, const float* dw_dev, const int32_t* wsum_dev,
                           const float* delta_dev, const int32_t* zp_dev, int a_bits,
                           const float* bias_dev,
                           uint16_t* y_bf16_dev, int32_t* acc_dbg_dev, void* stream) {
    return stwq_linear_ex(q_dev, M, K, N, L, wq_dev, dw_dev, wsum_dev, delta_dev, zp_dev, a_bits, bias_dev,
                          y_bf16_dev, acc_dbg_dev, STWQ_SCHEDULE_AUTO, stream);
}
