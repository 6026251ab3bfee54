// Aggregation of Sec. 2.1: y[t] = sum_j w[t,j] * ret[slot_to_row[t*k+j]] (+ shared_out[t]).
//
// `ret` is in send-buffer row order (the second all-to-all is the reverse of the
// first with the same sizes, Sec. 2.2).  One wave per token: the k source rows are
// gathered with 16-byte lanes (1 KB per wave access), accumulated in fp32 in slot
// order j = 0..k-1 and rounded once on the way out.  Every input row is read exactly
// once (plain loads while the rows fit the memory-side cache, streaming loads beyond,
// see kCombineCacheableBytes); the output goes out with streaming stores.
#include "common.h"

namespace {

template <int DT> struct Pack;
template <> struct Pack<MOE_BF16> {
    static constexpr int V = 8;
    __device__ static void unpack(const u32x4& q, float (&f)[8]) {
        const uint32_t u[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            f[2 * i] = __uint_as_float(u[i] << 16);
            f[2 * i + 1] = __uint_as_float(u[i] & 0xffff0000u);
        }
    }
    __device__ static u32x4 pack(const float (&f)[8]) {
        uint32_t u[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) u[i] = f32_to_bf16_bits(f[2 * i]) | (f32_to_bf16_bits(f[2 * i + 1]) << 16);
        return u32x4{u[0], u[1], u[2], u[3]};
    }
};
template <> struct Pack<MOE_F32> {
    static constexpr int V = 4;
    __device__ static void unpack(const u32x4& q, float (&f)[4]) {
        f[0] = __uint_as_float(q.x); f[1] = __uint_as_float(q.y); f[2] = __uint_as_float(q.z); f[3] = __uint_as_float(q.w);
    }
    __device__ static u32x4 pack(const float (&f)[4]) {
        return u32x4{__float_as_uint(f[0]), __float_as_uint(f[1]), __float_as_uint(f[2]), __float_as_uint(f[3])};
    }
};

template <int DT, int K, bool STREAM>
__global__ __launch_bounds__(256) void combine_kernel(const u32x4* __restrict__ ret, const int32_t* __restrict__ slot_to_row,
                                                      const float* __restrict__ topk_w, const u32x4* __restrict__ shared_out,
                                                      int T, int row16, u32x4* __restrict__ y) {
    constexpr int V = Pack<DT>::V;
    constexpr int KM = K;
    const int lane = threadIdx.x & 63;
    const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= T) return;
    int rows[KM];
    float w[KM];
#pragma unroll
    for (int j = 0; j < KM; ++j) {
        rows[j] = slot_to_row[(size_t)t * K + j];
        w[j] = topk_w[(size_t)t * K + j];
    }
    // CPT 16-byte chunks per lane per trip, about eight independent row loads in flight before the first use
    constexpr int CPT = (K < 4) ? 8 / K : 2;
    for (int c0 = lane; c0 < row16; c0 += 64 * CPT) {
        u32x4 q[CPT][KM];
#pragma unroll
        for (int u = 0; u < CPT; ++u) {
            const int c = c0 + 64 * u;
#pragma unroll
            for (int j = 0; j < KM; ++j)
                if (c < row16 && rows[j] >= 0) {
                    const u32x4* p = ret + (size_t)rows[j] * row16 + c;
                    q[u][j] = STREAM ? __builtin_nontemporal_load(p) : *p;
                }
        }
#pragma unroll
        for (int u = 0; u < CPT; ++u) {
            const int c = c0 + 64 * u;
            if (c >= row16) continue;
            float acc[V];
#pragma unroll
            for (int v = 0; v < V; ++v) acc[v] = 0.f;
#pragma unroll
            for (int j = 0; j < KM; ++j) {
                if (rows[j] >= 0) {
                    float f[V];
                    Pack<DT>::unpack(q[u][j], f);
#pragma unroll
                    for (int v = 0; v < V; ++v) acc[v] = fmaf(w[j], f[v], acc[v]);
                }
            }
            if (shared_out) {
                float f[V];
                Pack<DT>::unpack(shared_out[(size_t)t * row16 + c], f);
#pragma unroll
                for (int v = 0; v < V; ++v) acc[v] += f[v];
            }
            __builtin_nontemporal_store(Pack<DT>::pack(acc), y + (size_t)t * row16 + c);
        }
    }
}

// Any k: one token and 1 KB of its rows per wave, four source rows in flight at a time.  The loads are issued
// unconditionally (a slot past k or a dropped one reads a valid row whose value is not used): with the loads of
// a 16-slot array under conditions the compiler kept the whole array in registers (217 of them) and waited
// for each load in turn.
template <int DT, bool STREAM>
__global__ __launch_bounds__(256) void combine_any_k_kernel(const u32x4* __restrict__ ret, const int32_t* __restrict__ slot_to_row,
                                                            const float* __restrict__ topk_w, const u32x4* __restrict__ shared_out,
                                                            int T, int k, int row16, u32x4* __restrict__ y) {
    constexpr int V = Pack<DT>::V;
    const int lane = threadIdx.x & 63;
    const int t = __builtin_amdgcn_readfirstlane(blockIdx.x * 4 + (threadIdx.x >> 6));
    if (t >= T) return;
    const int c0 = blockIdx.y * 64;
    const int c = min(c0 + lane, row16 - 1);
    float acc[V];
#pragma unroll
    for (int v = 0; v < V; ++v) acc[v] = 0.f;
    for (int j0 = 0; j0 < k; j0 += 4) {
        int rows[4];
        float w[4];
        u32x4 d[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int j = min(j0 + i, k - 1);
            rows[i] = (j0 + i < k) ? slot_to_row[(size_t)t * k + j] : -1;
            w[i] = topk_w[(size_t)t * k + j];
            const u32x4* p = ret + (size_t)max(rows[i], 0) * row16 + c;
            d[i] = STREAM ? __builtin_nontemporal_load(p) : *p;
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (rows[i] >= 0) {
                float f[V];
                Pack<DT>::unpack(d[i], f);
#pragma unroll
                for (int v = 0; v < V; ++v) acc[v] = fmaf(w[i], f[v], acc[v]);
            }
        }
    }
    if (shared_out) {
        float f[V];
        Pack<DT>::unpack(shared_out[(size_t)t * row16 + c], f);
#pragma unroll
        for (int v = 0; v < V; ++v) acc[v] += f[v];
    }
    if (c0 + lane < row16) __builtin_nontemporal_store(Pack<DT>::pack(acc), y + (size_t)t * row16 + c0 + lane);
}

// Rows that were just written by the return transfer are still in the memory-side cache (256 MB) when they
// are not too many: plain loads then (17 against 19 us at the Mixtral-shape share, 67 MB); beyond half of that
// cache plain loads only evict each other (103 against 86 us at 403 MB) and streaming loads are used.
constexpr size_t kCombineCacheableBytes = (size_t)128 << 20;

template <int DT, bool STREAM>
int launch_combine(const moe_ctx* c, const void* ret, const int32_t* s2r, const float* w, const void* shared, void* y,
                   hipStream_t st) {
    const moe_shape& s = c->s;
    const int row16 = (int)((int64_t)s.H * elem_size(s.dtype) / 16);
    const dim3 grid((s.T + 3) / 4);
    const u32x4* r = reinterpret_cast<const u32x4*>(ret);
    const u32x4* sh = reinterpret_cast<const u32x4*>(shared);
    u32x4* yo = reinterpret_cast<u32x4*>(y);
    if (s.k == 1) hipLaunchKernelGGL((combine_kernel<DT, 1, STREAM>), grid, dim3(256), 0, st, r, s2r, w, sh, s.T, row16, yo);
    else if (s.k == 2) hipLaunchKernelGGL((combine_kernel<DT, 2, STREAM>), grid, dim3(256), 0, st, r, s2r, w, sh, s.T, row16, yo);
    else if (s.k == 6) hipLaunchKernelGGL((combine_kernel<DT, 6, STREAM>), grid, dim3(256), 0, st, r, s2r, w, sh, s.T, row16, yo);
    else {
        const dim3 grid_any((s.T + 3) / 4, (row16 + 63) / 64);
        hipLaunchKernelGGL((combine_any_k_kernel<DT, STREAM>), grid_any, dim3(256), 0, st, r, s2r, w, sh, s.T, s.k, row16, yo);
    }
    MOE_LAUNCH_CHECK("combine_kernel");
    return MOE_OK;
}

template <int DT>
int launch_combine_dt(const moe_ctx* c, const void* ret, const int32_t* s2r, const float* w, const void* shared, void* y,
                      hipStream_t st) {
    const moe_shape& s = c->s;
    const size_t bytes = (size_t)s.T * s.k * s.H * elem_size(s.dtype);
    if (bytes > kCombineCacheableBytes) return launch_combine<DT, true>(c, ret, s2r, w, shared, y, st);
    return launch_combine<DT, false>(c, ret, s2r, w, shared, y, st);
}

}  // namespace

extern "C" int moe_combine(moe_ctx* ctx, const void* ret, const int32_t* slot_to_row, const float* topk_w,
                           const void* shared_out, void* y, void* stream) {
    if (!ctx || !ret || !slot_to_row || !topk_w || !y) return moe_set_error(MOE_EINVAL, "moe_combine: NULL argument");
    if (!aligned16(ret) || !aligned16(y) || !aligned16(shared_out))
        return moe_set_error(MOE_EALIGN, "moe_combine: ret, y and shared_out must be 16-byte aligned");
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    if (ctx->s.dtype == MOE_BF16) return launch_combine_dt<MOE_BF16>(ctx, ret, slot_to_row, topk_w, shared_out, y, st);
    return launch_combine_dt<MOE_F32>(ctx, ret, slot_to_row, topk_w, shared_out, y, st);
}
