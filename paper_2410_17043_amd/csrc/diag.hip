// Reference measurements of the device itself (not on the layer's path): what the matrix cores sustain with
// operands that never leave the registers, and what a plain streaming copy with the send buffer's traffic
// shape (every byte read once and written twice) sustains.  bench.py prints both beside the layer's numbers,
// so that a figure quoted against the published peaks can also be read against what this machine delivers.
#include "common.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

// A value in [-1, 1) on the bf16 grid from a counter (Weyl sequence on the golden ratio; the arithmetic has no
// meaning beyond giving every lane and register different, well-scaled bits).
__device__ __forceinline__ __bf16 weyl_bf16(uint32_t n) {
    const uint32_t h = n * 2654435769u;
    return (__bf16)((float)(int32_t)h * (1.0f / 2147483648.0f));
}

// One wave per SIMD (256 accumulator registers per lane leave room for no second one), 4 x 4 independent
// 32x32x16 bf16 MFMA tiles per trip, exactly the register blocking of the FFN kernel, but no LDS and no
// memory traffic inside the loop.  Operand registers rotate from trip to trip so that consecutive MFMAs
// never read the same pair.
__global__ __launch_bounds__(256, 1) void mfma_only_kernel(int iters, float* __restrict__ sink) {
    const uint32_t id = (blockIdx.x * 256u + threadIdx.x) * 64u;
    bf16x8 a[4], b[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            a[i][e] = weyl_bf16(id + i * 8 + e);
            b[i][e] = weyl_bf16(id + 32 + i * 8 + e);
        }
    f32x16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
    for (int it = 0; it < iters; it += 4) {
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[(i + u) & 3], b[(j + u) & 3], acc[i][j], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) s += acc[i][j][e];
    sink[blockIdx.x * 256 + threadIdx.x] = s;
}

// dst0[i] = dst1[i] = src[i]: a wave per 8 KB piece, 16 bytes per lane and access, the whole piece requested
// before the first store, cacheable loads and streaming stores (the fastest of the plain variants tried:
// streaming loads, fewer loads in flight and several pieces per wave were all slower).  Every load is issued
// unconditionally (past the end a lane reads the last unit again): a load under a condition makes the compiler
// copy all 32 data registers and wait for each load before it issues the next.
__global__ __launch_bounds__(256) void copy_1r2w_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst0,
                                                        u32x4* __restrict__ dst1, size_t n16) {
    const size_t base = ((size_t)blockIdx.x * 4 + (threadIdx.x >> 6)) * 512 + (threadIdx.x & 63);
    u32x4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = src[min(base + u * 64, n16 - 1)];
#pragma unroll
    for (int u = 0; u < 8; ++u)
        if (base + u * 64 < n16) __builtin_nontemporal_store(v[u], dst0 + base + u * 64);
#pragma unroll
    for (int u = 0; u < 8; ++u)
        if (base + u * 64 < n16) __builtin_nontemporal_store(v[u], dst1 + base + u * 64);
}

// A chain of `run` v_mfma_f32_16x16x32_bf16 per 16 x 16 tile, the first with a zero accumulator:
// d[t][i][j] = fp32 sum over k < 32 run of a[t][i][k] b[t][j][k] as the matrix core forms it, operands and result
// in the lane layout the gate kernel uses (lane l: row l % 16, k = 8 (l / 16) .. + 7 of each 32; result rows
// 4 (l / 16) + i, column l % 16).  One wave per tile.
__global__ __launch_bounds__(64) void mfma_run_sum_kernel(const uint16_t* __restrict__ a, const uint16_t* __restrict__ b,
                                                          int run, float* __restrict__ d) {
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    const int lane = threadIdx.x, r = lane & 15, g = lane >> 4;
    const size_t t = blockIdx.x;
    f32x4 out = {0.f, 0.f, 0.f, 0.f};
    for (int q = 0; q < run; ++q) {
        const bf16x8 av = *reinterpret_cast<const bf16x8*>(a + ((t * 16 + r) * run + q) * 32 + 8 * g);
        const bf16x8 bv = *reinterpret_cast<const bf16x8*>(b + ((t * 16 + r) * run + q) * 32 + 8 * g);
        out = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, bv, out, 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) d[(t * 16 + 4 * g + i) * 16 + r] = out[i];
}

int timed(hipStream_t st, hipEvent_t* ev, float* ms_out) {
    MOE_HIP(hipEventSynchronize(ev[1]));
    MOE_HIP(hipEventElapsedTime(ms_out, ev[0], ev[1]));
    (void)st;
    return MOE_OK;
}

}  // namespace

extern "C" int moe_diag_mfma_only(int32_t n_blocks, int32_t iters, float* sink, void* stream, float* ms_out,
                                  double* flop_out) {
    if (!sink || !ms_out || !flop_out) return moe_set_error(MOE_EINVAL, "moe_diag_mfma_only: NULL argument");
    if (n_blocks < 1 || n_blocks > 65536 || iters < 4 || iters % 4 != 0 || iters > (1 << 24))
        return moe_set_error(MOE_ESHAPE, "moe_diag_mfma_only: need 1 <= n_blocks <= 65536 and iters a multiple of 4 in [4, 2^24]");
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    hipEvent_t ev[2] = {nullptr, nullptr};
    MOE_HIP(hipEventCreate(&ev[0]));
    if (hipEventCreate(&ev[1]) != hipSuccess) { (void)hipEventDestroy(ev[0]); return moe_set_error(MOE_EHIP, "hipEventCreate failed"); }
    int rc = MOE_OK;
    if (hipEventRecord(ev[0], st) != hipSuccess) rc = moe_set_error(MOE_EHIP, "hipEventRecord failed");
    if (rc == MOE_OK) {
        hipLaunchKernelGGL(mfma_only_kernel, dim3(n_blocks), dim3(256), 0, st, iters, sink);
        if (hipGetLastError() != hipSuccess) rc = moe_set_error(MOE_EHIP, "launch mfma_only_kernel failed");
    }
    if (rc == MOE_OK && hipEventRecord(ev[1], st) != hipSuccess) rc = moe_set_error(MOE_EHIP, "hipEventRecord failed");
    if (rc == MOE_OK) rc = timed(st, ev, ms_out);
    (void)hipEventDestroy(ev[0]);
    (void)hipEventDestroy(ev[1]);
    // 4 waves per block, 16 MFMAs per trip, 2 * 32 * 32 * 16 flop each
    *flop_out = (double)n_blocks * 4.0 * (double)iters * 16.0 * 2.0 * 32.0 * 32.0 * 16.0;
    return rc;
}

extern "C" int moe_diag_copy_1r2w(const void* src, void* dst0, void* dst1, size_t bytes, int32_t reps, void* stream,
                                  float* ms_out) {
    if (!src || !dst0 || !dst1 || !ms_out) return moe_set_error(MOE_EINVAL, "moe_diag_copy_1r2w: NULL argument");
    if (bytes == 0 || bytes % 16 != 0) return moe_set_error(MOE_ESHAPE, "moe_diag_copy_1r2w: bytes must be a positive multiple of 16");
    if (reps < 1 || reps > 1000) return moe_set_error(MOE_ESHAPE, "moe_diag_copy_1r2w: reps must be in [1, 1000]");
    if (!aligned16(src) || !aligned16(dst0) || !aligned16(dst1)) return moe_set_error(MOE_EALIGN, "moe_diag_copy_1r2w: 16-byte alignment needed");
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    const size_t n16 = bytes / 16;
    const size_t want = (n16 + 2047) / 2048;                // four 8 KB pieces per block
    if (want > 0x7fffffffull) return moe_set_error(MOE_ESHAPE, "moe_diag_copy_1r2w: too large");
    const int grid = (int)want;
    hipEvent_t ev[2] = {nullptr, nullptr};
    MOE_HIP(hipEventCreate(&ev[0]));
    if (hipEventCreate(&ev[1]) != hipSuccess) { (void)hipEventDestroy(ev[0]); return moe_set_error(MOE_EHIP, "hipEventCreate failed"); }
    int rc = MOE_OK;
    if (hipEventRecord(ev[0], st) != hipSuccess) rc = moe_set_error(MOE_EHIP, "hipEventRecord failed");
    for (int r = 0; r < reps && rc == MOE_OK; ++r) {
        hipLaunchKernelGGL(copy_1r2w_kernel, dim3(grid), dim3(256), 0, st, reinterpret_cast<const u32x4*>(src),
                           reinterpret_cast<u32x4*>(dst0), reinterpret_cast<u32x4*>(dst1), n16);
        if (hipGetLastError() != hipSuccess) rc = moe_set_error(MOE_EHIP, "launch copy_1r2w_kernel failed");
    }
    if (rc == MOE_OK && hipEventRecord(ev[1], st) != hipSuccess) rc = moe_set_error(MOE_EHIP, "hipEventRecord failed");
    if (rc == MOE_OK) rc = timed(st, ev, ms_out);
    if (rc == MOE_OK) *ms_out /= (float)reps;
    (void)hipEventDestroy(ev[0]);
    (void)hipEventDestroy(ev[1]);
    return rc;
}

extern "C" int moe_diag_mfma_run_sum(const void* a, const void* b, float* d, int32_t n_tiles, int32_t run, void* stream) {
    if (!a || !b || !d) return moe_set_error(MOE_EINVAL, "moe_diag_mfma_run_sum: NULL argument");
    if (n_tiles < 1 || n_tiles > (1 << 20) || run < 1 || run > 64)
        return moe_set_error(MOE_ESHAPE, "moe_diag_mfma_run_sum: n_tiles must be in [1, 2^20] and run in [1, 64]");
    if (!aligned16(a) || !aligned16(b)) return moe_set_error(MOE_EALIGN, "moe_diag_mfma_run_sum: 16-byte alignment needed");
    hipLaunchKernelGGL(mfma_run_sum_kernel, dim3(n_tiles), dim3(64), 0, reinterpret_cast<hipStream_t>(stream),
                       reinterpret_cast<const uint16_t*>(a), reinterpret_cast<const uint16_t*>(b), run, d);
    MOE_LAUNCH_CHECK("mfma_run_sum_kernel");
    return MOE_OK;
}
