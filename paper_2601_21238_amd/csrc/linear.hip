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
// Prefill kernel: 256 (output channels) x 256 (tokens) block tile, 8 waves in a 2 x 4 grid (wave
// tile 128 x 64 = 4 x 2 MFMA tiles, 128 int32 accumulators per lane), K consumed in stages of 64.
//
// Staging.  Both operand tiles go global -> LDS with direct-to-LDS loads (no register staging)
// into a ring of four 32 KB stages, so three stages (96 KB per CU) are in flight while one is
// consumed; the loaded memory latency here is one to two microseconds and a stage lasts about
// half a microsecond.  A stage's four loads per wave are issued one at a time between MFMA pairs.
//
// LDS layout of one operand stage: 256 rows x 64 bytes; the four 16-byte chunks of row r are
// permuted by chunk ^ ((r >> 2) & 3), which spreads the sixteen rows one ds_read_b128 pass touches
// over all 64 banks.  A direct-to-LDS load writes lane i's 16 bytes at base + 16 i, so the
// permutation is applied on the global side: the lane that fills physical chunk pc of row r
// fetches logical chunk pc ^ ((r >> 2) & 3).
//
// Synchronisation.  One barrier per stage, placed between the two k-steps: by then every wave
// holds the stage's last operands in registers, so the stage can be refilled, and the operands of
// the next stage's first k-step are fetched under the second k-step's MFMAs.  Operand reads and
// their waits are inline asm; the wait counts below are exact (LDS reads and vector-memory loads
// return in order).
//
// Epilogue.  Accumulators are dequantized in registers, staged as bf16 through the wave's own
// 16 KB of the (now idle) ring with a 16-byte XOR swizzle, and written as full 256-byte row
// segments with 16-byte stores.  Per-channel constants come from a 3 KB LDS table filled at kernel
// start.
//
// Rows past the end of either matrix are clamped to the last valid row: their products land in
// accumulators that are never stored.  Workgroups are dealt round-robin to the 8 XCDs (each with
// its own L2); the 32 workgroups one XCD runs together are mapped to a compact patch of tiles.
// ------------------------------------------------------------------------------------------------
constexpr int kTile = 256;
constexpr int kBK = 64;
constexpr int kStages = 4;
constexpr int kPrefillThreads = 512;
constexpr int kOpBytes = kTile * kBK;        // one operand, one stage: 16 KB
constexpr int kStageBytes = 2 * kOpBytes;    // W then X: 32 KB
constexpr int kRingBytes = kStages * kStageBytes;

typedef __attribute__((address_space(3))) void lds_void;
typedef const __attribute__((address_space(1))) void global_void;

// ---- LDS operand reads and waits as inline asm: the compiler's wait-count pass then sees no LDS
// read that could alias the in-flight direct-to-LDS loads, and the waits below are the only ones.
template <int OFF>
__device__ __forceinline__ v4i lds_read16(unsigned addr) {
    v4i v;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
    return v;
}
__device__ __forceinline__ void read_ops(unsigned addrA, unsigned addrB, v4i (&a)[4], v4i (&b)[2]) {
    a[0] = lds_read16<0 * 32 * kBK>(addrA);
    a[1] = lds_read16<1 * 32 * kBK>(addrA);
    a[2] = lds_read16<2 * 32 * kBK>(addrA);
    a[3] = lds_read16<3 * 32 * kBK>(addrA);
    b[0] = lds_read16<0 * 32 * kBK>(addrB);
    b[1] = lds_read16<1 * 32 * kBK>(addrB);
}
// waits until at most N LDS reads are outstanding; the operands are tied to the wait so that no
// MFMA that consumes them can be scheduled above it
template <int N>
__device__ __forceinline__ void wait_ops(v4i (&a)[4], v4i (&b)[2]) {
    asm volatile("s_waitcnt lgkmcnt(%6)"
                 : "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3]), "+v"(b[0]), "+v"(b[1])
                 : "n"(N));
}
__device__ __forceinline__ void mfma_block(const v4i (&a)[4], const v4i (&b)[2], v16i (&acc)[4][2]) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i], b[j], acc[i][j], 0, 0, 0);
}


__device__ __forceinline__ void load_stage(const int8_t* const (&srcW)[2], const int8_t* const (&srcX)[2], int k0,
                                            int8_t* stage, int wave) {
#pragma unroll
    for (int pss = 0; pss < 2; ++pss)
        __builtin_amdgcn_global_load_lds((global_void*)(srcW[pss] + k0), (lds_void*)(stage + (pss * 128 + wave * 16) * kBK), 16, 0, 0);
#pragma unroll
    for (int pss = 0; pss < 2; ++pss)
        __builtin_amdgcn_global_load_lds((global_void*)(srcX[pss] + k0), (lds_void*)(stage + kOpBytes + (pss * 128 + wave * 16) * kBK), 16, 0, 0);
}

// One K stage (two MFMA k-steps).  The four direct-to-LDS loads of stage s+4 are issued one at a
// time between pairs of MFMAs, so that no wave sits in a full address queue with its MFMAs unissued.
template <bool TAIL>
__device__ __forceinline__ void stage_step(int s, int nk, int8_t* smem, unsigned lds_base, const int8_t* const (&srcW)[2],
                                           const int8_t* const (&srcX)[2], const unsigned (&offA)[2], const unsigned (&offB)[2],
                                           int wave, v4i (&a0)[4], v4i (&b0)[2], v4i (&a1)[4], v4i (&b1)[2], v16i (&acc)[4][2]) {
    const unsigned cur = lds_base + (s & 3) * kStageBytes;
    const unsigned nxt = lds_base + ((s + 1) & 3) * kStageBytes;
    read_ops(cur + offA[1], cur + kOpBytes + offB[1], a1, b1);
    wait_ops<6>(a0, b0);
    mfma_block(a0, b0, acc);
    __builtin_amdgcn_sched_barrier(0);   // the MFMAs above cover the latency of the reads waited for below
    if (TAIL) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    else asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
    wait_ops<0>(a1, b1);
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    read_ops(nxt + offA[0], nxt + kOpBytes + offB[0], a0, b0);
    const bool do_load = s + kStages < nk;
    int8_t* dst = smem + (s & 3) * kStageBytes;
    const int k0 = (s + kStages) * kBK;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        if (do_load) {
            const int8_t* src = (i < 2 ? srcW[i] : srcX[i - 2]) + k0;
            int8_t* d = dst + (i < 2 ? 0 : kOpBytes) + ((i & 1) * 128 + wave * 16) * kBK;
            __builtin_amdgcn_global_load_lds((global_void*)src, (lds_void*)d, 16, 0, 0);
        }
        acc[i][0] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a1[i], b1[0], acc[i][0], 0, 0, 0);
        acc[i][1] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a1[i], b1[1], acc[i][1], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
    }
}

__global__ __launch_bounds__(kPrefillThreads) void linear_prefill_kernel(LinearArgs p, int tiles_m, int tiles_o, int patch_o, int patch_m) {
    extern __shared__ __attribute__((aligned(1024))) int8_t smem[];
    __shared__ __attribute__((aligned(16))) float c_dw[kTile];
    __shared__ __attribute__((aligned(16))) int c_ws[kTile];
    __shared__ __attribute__((aligned(16))) float c_bias[kTile];
    const unsigned lds_base = static_cast<unsigned>(reinterpret_cast<uintptr_t>(smem));

    // XCD-aware 2-D patches: the 32 workgroups an XCD runs together form a patch_m x patch_o patch
    const int bid = blockIdx.x;
    const int xcd = bid & 7, j = bid >> 3;
    const int patch = (j >> 5) * 8 + xcd, idx = j & 31;
    const int npo = (tiles_o + patch_o - 1) / patch_o;
    const int po = patch % npo, pm = patch / npo;
    const int tile_o = po * patch_o + idx % patch_o;
    const int tile_m = pm * patch_m + idx / patch_o;
    if (tile_o >= tiles_o || tile_m >= tiles_m) return;
    const long long m0 = static_cast<long long>(tile_m) * kTile;
    const int o0 = tile_o * kTile;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, hi = lane >> 5;
    const int wo = wave & 1, wm = wave >> 1;

    const int8_t* srcW[2];
    const int8_t* srcX[2];
#pragma unroll
    for (int pss = 0; pss < 2; ++pss) {
        const int r = pss * 128 + wave * 16 + (lane >> 2);
        const int lc = (lane & 3) ^ ((r >> 2) & 3);
        const int ro = min(o0 + r, p.N - 1);
        const long long rm = min(m0 + r, static_cast<long long>(p.M) - 1);
        srcW[pss] = p.wq + static_cast<size_t>(ro) * p.K + lc * 16;
        srcX[pss] = p.q + static_cast<size_t>(rm) * p.K + lc * 16;
    }
    unsigned offA[2], offB[2];
    const int swz = (l32 >> 2) & 3;
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
        const int pc = ((ks * 2 + hi) ^ swz) * 16;
        offA[ks] = (wo * 128 + l32) * kBK + pc;
        offB[ks] = (wm * 64 + l32) * kBK + pc;
    }

    v16i acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int jj = 0; jj < 2; ++jj) acc[i][jj] = (v16i){0};

    {   // per-output-channel constants of this tile, read back in the epilogue
        const int o = min(o0 + (tid & 255), p.N - 1);
        if (tid < 256) { c_dw[tid] = p.dw[o]; c_ws[tid] = p.wsum[o]; }
        else c_bias[tid - 256] = p.bias ? p.bias[o] : 0.0f;
    }
    const int nk = p.K / kBK;
    // prologue: up to four stages in flight
#pragma unroll
    for (int s = 0; s < kStages; ++s)
        if (s < nk) load_stage(srcW, srcX, s * kBK, smem + s * kStageBytes, wave);
    if (nk >= 4) asm volatile("s_waitcnt vmcnt(12)" ::: "memory");
    else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    v4i a0[4], b0[2], a1[4], b1[2];
    read_ops(lds_base + offA[0], lds_base + kOpBytes + offB[0], a0, b0);

    int s = 0;
    const int n_steady = nk - 3;
    for (; s < n_steady; ++s) stage_step<false>(s, nk, smem, lds_base, srcW, srcX, offA, offB, wave, a0, b0, a1, b1, acc);
    for (; s < nk; ++s) stage_step<true>(s, nk, smem, lds_base, srcW, srcX, offA, offB, wave, a0, b0, a1, b1, acc);
    wait_ops<0>(a0, b0);   // the last prefetch read stale data; drain it

    if (p.acc_dbg) {   // raw accumulators for the bit-exact check (debug path, not tuned)
#pragma unroll
        for (int jj = 0; jj < 2; ++jj) {
            const long long m = m0 + wm * 64 + jj * 32 + l32;
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int o4 = o0 + wo * 128 + i * 32 + 8 * g + 4 * hi;
                    if (m < p.M && o4 < p.N)
                        *reinterpret_cast<int4*>(p.acc_dbg + m * p.N + o4) =
                            make_int4(acc[i][jj][4 * g], acc[i][jj][4 * g + 1], acc[i][jj][4 * g + 2], acc[i][jj][4 * g + 3]);
                }
        }
    }

    // ---- epilogue: dequantize, stage bf16 through this wave's 16 KB of LDS, store full rows ----
    __syncthreads();   // every wave is done reading operands; also orders the constants written at the start
    int8_t* stage = smem + wave * 16384;
    float dt[2];
    int zs[2];
#pragma unroll
    for (int jj = 0; jj < 2; ++jj) {
        int m = static_cast<int>(m0) + wm * 64 + jj * 32 + l32;
        if (m >= p.M) m = p.M - 1;
        const int t = m % p.L;
        dt[jj] = p.delta[t];
        zs[jj] = p.zp[t] - p.off;
    }
    float4 dwv = *reinterpret_cast<const float4*>(c_dw + wo * 128 + 4 * hi);
    int4 wsv = *reinterpret_cast<const int4*>(c_ws + wo * 128 + 4 * hi);
    float4 bv = *reinterpret_cast<const float4*>(c_bias + wo * 128 + 4 * hi);
#pragma unroll
    for (int c = 0; c < 16; ++c) {           // c = i * 4 + g: output channels wo*128 + 8c + 4hi .. +3
        float4 dwn = dwv, bn = bv;
        int4 wsn = wsv;
        if (c < 15) {
            const int ol = wo * 128 + 8 * (c + 1) + 4 * hi;
            dwn = *reinterpret_cast<const float4*>(c_dw + ol);
            wsn = *reinterpret_cast<const int4*>(c_ws + ol);
            bn = *reinterpret_cast<const float4*>(c_bias + ol);
        }
        const int i = c >> 2, g = c & 3;
#pragma unroll
        for (int jj = 0; jj < 2; ++jj) {
            const int row = jj * 32 + l32;
            const float y0 = fmaf(static_cast<float>(acc[i][jj][4 * g] - __mul24(zs[jj], wsv.x)), dt[jj] * dwv.x, bv.x);
            const float y1 = fmaf(static_cast<float>(acc[i][jj][4 * g + 1] - __mul24(zs[jj], wsv.y)), dt[jj] * dwv.y, bv.y);
            const float y2 = fmaf(static_cast<float>(acc[i][jj][4 * g + 2] - __mul24(zs[jj], wsv.z)), dt[jj] * dwv.z, bv.z);
            const float y3 = fmaf(static_cast<float>(acc[i][jj][4 * g + 3] - __mul24(zs[jj], wsv.w)), dt[jj] * dwv.w, bv.w);
            uint2 out;
            out.x = pack_bf16(y0, y1);
            out.y = pack_bf16(y2, y3);
            *reinterpret_cast<uint2*>(stage + row * 256 + ((c ^ (row & 15)) * 16) + hi * 8) = out;
        }
        dwv = dwn; wsv = wsn; bv = bn;
        __builtin_amdgcn_sched_barrier(0);
    }
    // same wave wrote and reads: LDS operations of one wave complete in order
    const int cc = lane & 15;
    const int o = o0 + wo * 128 + cc * 8;
#pragma unroll
    for (int r0 = 0; r0 < 16; r0 += 4) {
        uint4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int row = (r0 + u) * 4 + (lane >> 4);
            v[u] = *reinterpret_cast<const uint4*>(stage + row * 256 + ((cc ^ (row & 15)) * 16));
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int row = (r0 + u) * 4 + (lane >> 4);
            const long long m = m0 + wm * 64 + row;
            if (m < p.M && o < p.N) *reinterpret_cast<uint4*>(p.y + m * p.N + o) = v[u];
        }
        __builtin_amdgcn_sched_barrier(0);
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
        static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(linear_prefill_kernel),
                                                           hipFuncAttributeMaxDynamicSharedMemorySize, kRingBytes);
        if (attr != hipSuccess) return fail(STWQ_EHIP, "hipFuncSetAttribute failed: %s", hipGetErrorString(attr));
        const int tiles_o = (p.N + kTile - 1) / kTile;
        const long long tiles_m = (M + kTile - 1) / kTile;
        // patch of tiles one XCD works on at a time: patch_o x patch_m = 32
        int patch_o = tiles_o < 4 ? tiles_o : 4;
        while (32 % patch_o) --patch_o;
        const int patch_m = 32 / patch_o;
        const long long n_patches = ((tiles_o + patch_o - 1) / patch_o) * ((tiles_m + patch_m - 1) / patch_m);
        const long long n_blocks = ((n_patches + 7) / 8) * 8 * 32;
        STWQ_REQUIRE(n_blocks <= 0x7FFFFFFFLL, "stwq_linear: too many tiles");
        linear_prefill_kernel<<<dim3(static_cast<unsigned>(n_blocks)), dim3(kPrefillThreads), kRingBytes, s>>>(
            p, static_cast<int>(tiles_m), tiles_o, patch_o, patch_m);
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
