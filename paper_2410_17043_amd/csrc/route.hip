// Gate of Sec. 2.1: logits = x . Wg^T (+ bias), top-k on the logits, softmax weights.
//
// The indices must not depend on summation order, so logits are accumulated in
// fp64 (bf16 x bf16 and fp32 x fp32 products are exact in fp64).
#include "common.h"

namespace {

template <int DT> struct Chunk;
template <> struct Chunk<MOE_BF16> {
    static constexpr int V = 8;
    __device__ static void unpack(const u32x4& q, double (&out)[8]) {
        const uint32_t u[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            out[2 * i] = (double)__uint_as_float(u[i] << 16);
            out[2 * i + 1] = (double)__uint_as_float(u[i] & 0xffff0000u);
        }
    }
    __device__ static void load(const void* base, size_t chunk, double (&out)[8]) {
        unpack(reinterpret_cast<const u32x4*>(base)[chunk], out);
    }
};
template <> struct Chunk<MOE_F32> {
    static constexpr int V = 4;
    __device__ static void unpack(const u32x4& q, double (&out)[4]) {
        out[0] = __uint_as_float(q.x); out[1] = __uint_as_float(q.y); out[2] = __uint_as_float(q.z); out[3] = __uint_as_float(q.w);
    }
    __device__ static void load(const void* base, size_t chunk, double (&out)[4]) {
        unpack(reinterpret_cast<const u32x4*>(base)[chunk], out);
    }
};

// ---------------------------------------------------------------------------------------------
// Logits on the fp64 matrix cores.  x . Wg^T is a dense contraction, and v_mfma_f64_16x16x4_f64
// does 1024 exact-product FMAs per instruction and per pair of operand registers where the
// vector unit does 64: the matrix pipe is no faster than the vector one in fp64 on this chip
// (about 48 against 70 TFLOP/s measured), but it needs a sixteenth of the operand traffic, and
// operand delivery is what bounds a vector kernel here.  A block owns 16
// tokens (one MFMA row tile); its S waves split the hidden dimension.  Lane (r = lane % 16,
// g = lane / 16) supplies row r, k-index g of the A operand and k-index g, column r of the B
// operand; since the order of the sum over the hidden dimension is free, a group of 4 * V hidden
// indices is laid out so that lane group g owns V consecutive ones: every lane fetches whole
// 16-byte chunks of its token row and of its expert row and feeds element s of both to k-step s.
// The result tile D has row (lane / 16) + 4 * reg and column lane % 16.  Chunks are fetched PF
// groups ahead into a register ring.  Partial tiles of the S waves are added in wave order
// through LDS; top-k and softmax then run one token per wave, one candidate expert per lane.
typedef double f64x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ void select_topk(const double* __restrict__ z, int E, int k, int renorm, int t, int lane,
                                            int32_t* __restrict__ topk_idx, float* __restrict__ topk_w) {
    // up to 4 candidate experts per lane: lane, lane + 64, ...
    double cand[MOE_MAX_E / 64];
    bool taken[MOE_MAX_E / 64];
#pragma unroll
    for (int i = 0; i < MOE_MAX_E / 64; ++i) {
        const int e = lane + 64 * i;
        taken[i] = !(e < E);
        cand[i] = (e < E) ? z[e] : 0.0;
    }
    double zmax = 0.0, my_z = 0.0;
    int my_e = 0;
    for (int j = 0; j < k; ++j) {
        double best = 0.0;
        int best_e = 0x7fffffff;                         // "nothing": loses against every real candidate
#pragma unroll
        for (int i = 0; i < MOE_MAX_E / 64; ++i) {
            const int e = lane + 64 * i;
            if (!taken[i] && (best_e == 0x7fffffff || cand[i] > best)) { best = cand[i]; best_e = e; }
        }
#pragma unroll
        for (int o = 32; o >= 1; o >>= 1) {
            const double ob = __shfl_xor(best, o, 64);
            const int oe = __shfl_xor(best_e, o, 64);
            const bool take = (oe != 0x7fffffff) &&
                              (best_e == 0x7fffffff || ob > best || (ob == best && oe < best_e));
            if (take) { best = ob; best_e = oe; }
        }
#pragma unroll
        for (int i = 0; i < MOE_MAX_E / 64; ++i)
            if (lane + 64 * i == best_e) taken[i] = true;
        if (j == 0) zmax = best;
        if (lane == j) { my_z = best; my_e = best_e; }
    }
    // weights: the selection above is exact in fp64; the probabilities only need 1e-5, so the
    // exponentials are taken in fp32 of the fp64 differences (all <= 0)
    float part = 0.f;
#pragma unroll
    for (int i = 0; i < MOE_MAX_E / 64; ++i)
        if (lane + 64 * i < E) part += __expf((float)(cand[i] - zmax));
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) part += __shfl_xor(part, o, 64);
    float wj = (lane < k) ? __expf((float)(my_z - zmax)) / part : 0.f;
    if (renorm) {
        float s = wj;
#pragma unroll
        for (int o = 32; o >= 1; o >>= 1) s += __shfl_xor(s, o, 64);
        wj /= s;
    }
    if (lane < k) {
        topk_idx[(size_t)t * k + lane] = my_e;
        topk_w[(size_t)t * k + lane] = wj;
    }
}

template <int DT, int NT, int PF>
__global__ __launch_bounds__(NT == 1 ? 1024 : 512) void route_mfma_kernel(const void* __restrict__ x, const void* __restrict__ wg,
                                                          const float* __restrict__ bias, int T, int H, int E, int k,
                                                          int renorm, int32_t* __restrict__ topk_idx,
                                                          float* __restrict__ topk_w) {
    constexpr int V = Chunk<DT>::V;
    constexpr int EP = NT * 16;                          // experts per pass
    extern __shared__ double zl[];                       // [16][E] logits, then [S][16][EP] partial tiles
    double* zpart = zl + (size_t)16 * E;
    const int lane = threadIdx.x & 63, r = lane & 15, g = lane >> 4;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), S = blockDim.x >> 6;
    const int tok0 = blockIdx.x * 16;
    const int nchunk = H / V;                            // 16-byte chunks per row
    const int ngrp = (nchunk + 3) / 4;                   // groups of 4 chunks = one chunk per lane group
    const int per = (ngrp + S - 1) / S;
    const int b_lo = wave * per, b_hi = min(b_lo + per, ngrp);
    const u32x4* xrow = reinterpret_cast<const u32x4*>(x) + (size_t)min(tok0 + r, T - 1) * nchunk;

    for (int e0 = 0; e0 < E; e0 += EP) {
        // experts past E are clamped to the last row: computed, never used
        const u32x4* wrow[NT];
#pragma unroll
        for (int n = 0; n < NT; ++n) wrow[n] = reinterpret_cast<const u32x4*>(wg) + (size_t)min(e0 + n * 16 + r, E - 1) * nchunk;
        // CH independent accumulator chains per expert tile (k-steps alternate between them), so that an
        // MFMA never waits for the one issued just before it
        constexpr int CH = (NT >= 4) ? 1 : 4 / NT;
        f64x4 acc[CH][NT];
#pragma unroll
        for (int c = 0; c < CH; ++c)
#pragma unroll
            for (int n = 0; n < NT; ++n) acc[c][n] = f64x4{0.0, 0.0, 0.0, 0.0};
        u32x4 xq[PF], wq[PF][NT];
        auto fetch = [&](int b, u32x4& xo, u32x4 (&wo)[NT]) {   // group b, clamped into this wave's range
            const int c = min(4 * min(b, b_hi - 1) + g, nchunk - 1);
            xo = xrow[c];
#pragma unroll
            for (int n = 0; n < NT; ++n) wo[n] = wrow[n][c];
        };
        if (b_lo < b_hi) {
#pragma unroll
            for (int p = 0; p < PF; ++p) fetch(b_lo + p, xq[p], wq[p]);
        }
        for (int b = b_lo; b < b_hi; b += PF) {
#pragma unroll
            for (int p = 0; p < PF; ++p) {
                if (b + p < b_hi) {
                    double xv[V], wv[NT][V];
                    Chunk<DT>::unpack(xq[p], xv);
#pragma unroll
                    for (int n = 0; n < NT; ++n) Chunk<DT>::unpack(wq[p][n], wv[n]);
                    if (4 * (b + p) + g >= nchunk) {     // ragged last group: this lane group has no chunk
#pragma unroll
                        for (int v = 0; v < V; ++v) xv[v] = 0.0;
                    }
                    fetch(b + p + PF, xq[p], wq[p]);
#pragma unroll
                    for (int v = 0; v < V; ++v)
#pragma unroll
                        for (int n = 0; n < NT; ++n)
                            acc[v % CH][n] = __builtin_amdgcn_mfma_f64_16x16x4f64(xv[v], wv[n][v], acc[v % CH][n], 0, 0, 0);
                }
            }
        }
#pragma unroll
        for (int n = 0; n < NT; ++n)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                double sum = acc[0][n][v];
#pragma unroll
                for (int c = 1; c < CH; ++c) sum += acc[c][n][v];
                zpart[((size_t)wave * 16 + g + 4 * v) * EP + n * 16 + r] = sum;
            }
        __syncthreads();
        for (int i = threadIdx.x; i < 16 * EP; i += blockDim.x) {
            const int tt = i / EP, ee = i % EP;
            if (e0 + ee < E) {
                double sum = zpart[i];
                for (int w = 1; w < S; ++w) sum += zpart[(size_t)w * 16 * EP + i];
                zl[tt * E + e0 + ee] = sum + (bias ? (double)bias[e0 + ee] : 0.0);
            }
        }
        __syncthreads();
    }
    for (int tt = wave; tt < 16; tt += S) {
        const int t = tok0 + tt;
        if (t < T) select_topk(zl + (size_t)tt * E, E, k, renorm, t, lane, topk_idx, topk_w);
    }
}

template <int DT, int NT, int PF>
int launch_route_mfma(const moe_ctx* c, const void* x, const void* wg, const float* bias, int32_t* idx, float* w,
                      hipStream_t st) {
    const moe_shape& s = c->s;
    const int V = Chunk<DT>::V;
    const int blocks = (s.T + 15) / 16, ngrp = (s.H / V + 3) / 4;
    int S = 1;                                            // waves per block: about 2048 waves in all (4096 with one expert tile), at most 8 (16)
    const int s_max = (NT == 1) ? 16 : 8, waves = (NT == 1) ? 4096 : 2048;
    while (S < s_max && blocks * S < waves && 2 * S <= ngrp) S *= 2;
    const size_t lds = ((size_t)16 * s.E + (size_t)S * 16 * NT * 16) * sizeof(double);   // at most 96 KB
    static bool attr_done = false;
    if (!attr_done) {
        MOE_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&route_mfma_kernel<DT, NT, PF>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, 96 * 1024));
        attr_done = true;
    }
    hipLaunchKernelGGL((route_mfma_kernel<DT, NT, PF>), dim3(blocks), dim3(64 * S), lds, st, x, wg, bias, s.T, s.H, s.E,
                       s.k, s.renorm, idx, w);
    MOE_LAUNCH_CHECK("route_mfma_kernel");
    return MOE_OK;
}

template <int DT>
int route_dispatch(const moe_ctx* c, const void* x, const void* wg, const float* bias, int32_t* idx, float* w,
                   hipStream_t st) {
    const int E = c->s.E;
    if (E <= 16) return launch_route_mfma<DT, 1, 4>(c, x, wg, bias, idx, w, st);
    if (E <= 32) return launch_route_mfma<DT, 2, 4>(c, x, wg, bias, idx, w, st);
    return launch_route_mfma<DT, 4, 3>(c, x, wg, bias, idx, w, st);   // E > 64: several passes of 64 experts
}

}  // namespace

extern "C" int moe_route(moe_ctx* ctx, const void* x, const void* Wg, const float* gate_bias, int32_t* topk_idx,
                         float* topk_w, void* stream) {
    if (!ctx || !x || !Wg || !topk_idx || !topk_w) return moe_set_error(MOE_EINVAL, "moe_route: NULL argument");
    if (!aligned16(x) || !aligned16(Wg)) return moe_set_error(MOE_EALIGN, "moe_route: x and Wg must be 16-byte aligned");
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    ctx->rank_src = nullptr;                             // the indices are about to change: cached slot ranks are stale
    if (ctx->s.dtype == MOE_BF16) return route_dispatch<MOE_BF16>(ctx, x, Wg, gate_bias, topk_idx, topk_w, st);
    return route_dispatch<MOE_F32>(ctx, x, Wg, gate_bias, topk_idx, topk_w, st);
}
