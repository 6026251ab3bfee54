// Gate of Sec. 2.1: logits = x . Wg^T (+ bias), top-k on the logits, softmax weights.
//
// The indices must not depend on summation order, so logits are accumulated in
// fp64 (bf16 x bf16 and fp32 x fp32 products are exact in fp64).  fp64 FMA runs at
// the plain fp32 FMA rate on this chip, so there is no faster exact alternative on
// the vector units.
//
// Mapping: a block of 4 waves owns TT tokens; each wave takes a quarter of the hidden
// dimension and its 64 lanes split that quarter in 16-byte chunks (coalesced 1 KB per
// wave per token row), so every token row is read once and enough waves are in flight
// to cover HBM latency.  Each lane keeps TT x ET fp64 partial logits; Wg chunks are read
// through L1/L2 (all blocks read the same few KB).  The cross-lane sum is a halving
// butterfly (each exchange step hands half of the values to the partner lane), after
// which lane l holds one partial logit; the four waves' partials are added through LDS.
// Top-k and softmax then run wave-parallel, one token per wave, one candidate expert
// per lane.
#include "common.h"

namespace {

template <int DT> struct Chunk;
template <> struct Chunk<MOE_BF16> {
    static constexpr int V = 8;
    __device__ static void load(const void* base, size_t chunk, double (&out)[8]) {
        const uint4 q = reinterpret_cast<const uint4*>(base)[chunk];
        const uint32_t u[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            out[2 * i] = (double)__uint_as_float(u[i] << 16);
            out[2 * i + 1] = (double)__uint_as_float(u[i] & 0xffff0000u);
        }
    }
};
template <> struct Chunk<MOE_F32> {
    static constexpr int V = 4;
    __device__ static void load(const void* base, size_t chunk, double (&out)[4]) {
        const float4 q = reinterpret_cast<const float4*>(base)[chunk];
        out[0] = q.x; out[1] = q.y; out[2] = q.z; out[3] = q.w;
    }
};

// Sum v[0..N) over the 64 lanes.  On return lane l holds in v[0] the total of value
// index (N == 64 ? l : l >> (6 - log2 N)).  Written as a compile-time recursion so that
// every array index is a constant and the values stay in registers.
template <int N, int CUR, int O>
struct Halving {
    __device__ static __forceinline__ void run(double (&v)[N], int lane) {
        if constexpr (O >= 1) {
            if constexpr (CUR > 1) {
                constexpr int HALF = CUR / 2;
                const bool upper = (lane & O) != 0;
#pragma unroll
                for (int i = 0; i < HALF; ++i) {
                    const double send = upper ? v[i] : v[i + HALF];
                    const double keep = upper ? v[i + HALF] : v[i];
                    v[i] = keep + __shfl_xor(send, O, 64);
                }
                Halving<N, HALF, O / 2>::run(v, lane);
            } else {
                v[0] += __shfl_xor(v[0], O, 64);
                Halving<N, 1, O / 2>::run(v, lane);
            }
        }
    }
};
template <int N>
__device__ __forceinline__ void halving_reduce(double (&v)[N], int lane) { Halving<N, N, 32>::run(v, lane); }

template <int DT, int TT, int ET>
__global__ __launch_bounds__(256) void route_kernel(const void* __restrict__ x, const void* __restrict__ wg,
                                                    const float* __restrict__ bias, int T, int H, int E, int k,
                                                    int renorm, int32_t* __restrict__ topk_idx,
                                                    float* __restrict__ topk_w) {
    constexpr int V = Chunk<DT>::V;
    constexpr int N = TT * ET;
    extern __shared__ double zl[];                       // [TT][E] logits, then [4 waves][N] partials
    double* zpart = zl + (size_t)TT * E;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int tok0 = blockIdx.x * TT;
    const int nchunk = H / V;
    const int cpw = (nchunk + 3) / 4;                    // chunks per wave
    const int c_lo = wave * cpw, c_hi = min(c_lo + cpw, nchunk);

    for (int e0 = 0; e0 < E; e0 += ET) {
        double acc[N];
#pragma unroll
        for (int i = 0; i < N; ++i) acc[i] = 0.0;
        for (int c = c_lo + lane; c < c_hi; c += 64) {
            double xv[TT][V];
#pragma unroll
            for (int tt = 0; tt < TT; ++tt) {
                const int t = min(tok0 + tt, T - 1);
                Chunk<DT>::load(x, (size_t)t * nchunk + c, xv[tt]);
            }
            // experts past E are clamped to the last row: computed, never written out (keeps every
            // index below a compile-time constant, so the partial logits stay in registers)
#pragma unroll
            for (int e = 0; e < ET; ++e) {
                double wv[V];
                Chunk<DT>::load(wg, (size_t)min(e0 + e, E - 1) * nchunk + c, wv);
#pragma unroll
                for (int tt = 0; tt < TT; ++tt)
#pragma unroll
                    for (int v = 0; v < V; ++v) acc[tt * ET + e] = fma(xv[tt][v], wv[v], acc[tt * ET + e]);
            }
        }
        halving_reduce<N>(acc, lane);
        const int index = (N == 64) ? lane : (lane >> 1);   // N is 32 or 64
        if (N == 64 || (lane & 1) == 0) zpart[wave * N + index] = acc[0];
        __syncthreads();
        if (threadIdx.x < N) {
            const int tt = threadIdx.x / ET, e = e0 + threadIdx.x % ET;
            if (e < E)
                zl[tt * E + e] = ((zpart[threadIdx.x] + zpart[N + threadIdx.x]) +
                                  (zpart[2 * N + threadIdx.x] + zpart[3 * N + threadIdx.x])) +
                                 (bias ? (double)bias[e] : 0.0);
        }
        __syncthreads();
    }

    // one token per wave
    const int tt = wave, t = tok0 + wave;
    if (tt >= TT || t >= T) return;
    const double* z = zl;
    {
        // up to 4 candidate experts per lane: lane, lane + 64, ...
        double cand[MOE_MAX_E / 64];
        bool taken[MOE_MAX_E / 64];
#pragma unroll
        for (int i = 0; i < MOE_MAX_E / 64; ++i) {
            const int e = lane + 64 * i;
            taken[i] = !(e < E);
            cand[i] = (e < E) ? z[tt * E + e] : 0.0;
        }
        double zmax = 0.0, my_z = 0.0;
        int my_e = 0;
        for (int j = 0; j < k; ++j) {
            double best = 0.0;
            int best_e = 0x7fffffff;                     // "nothing": loses against every real candidate
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
        double part = 0.0;
#pragma unroll
        for (int i = 0; i < MOE_MAX_E / 64; ++i)
            if (lane + 64 * i < E) part += exp(cand[i] - zmax);
#pragma unroll
        for (int o = 32; o >= 1; o >>= 1) part += __shfl_xor(part, o, 64);
        double wj = (lane < k) ? exp(my_z - zmax) / part : 0.0;
        if (renorm) {
            double s = wj;
#pragma unroll
            for (int o = 32; o >= 1; o >>= 1) s += __shfl_xor(s, o, 64);
            wj /= s;
        }
        if (lane < k) {
            topk_idx[(size_t)t * k + lane] = my_e;
            topk_w[(size_t)t * k + lane] = (float)wj;
        }
    }
}

template <int DT, int TT, int ET>
int launch_route(const moe_ctx* c, const void* x, const void* wg, const float* bias, int32_t* idx, float* w,
                 hipStream_t st) {
    const moe_shape& s = c->s;
    const int grid = (s.T + TT - 1) / TT;
    const size_t lds = ((size_t)TT * s.E + 4 * TT * ET) * sizeof(double);
    hipLaunchKernelGGL((route_kernel<DT, TT, ET>), dim3(grid), dim3(256), lds, st, x, wg, bias, s.T, s.H, s.E, s.k,
                       s.renorm, idx, w);
    MOE_LAUNCH_CHECK("route_kernel");
    return MOE_OK;
}

template <int DT>
int route_dispatch(const moe_ctx* c, const void* x, const void* wg, const float* bias, int32_t* idx, float* w,
                   hipStream_t st) {
    const int E = c->s.E;
    if (E <= 8) return launch_route<DT, 4, 8>(c, x, wg, bias, idx, w, st);
    if (E <= 16) return launch_route<DT, 4, 16>(c, x, wg, bias, idx, w, st);
    if (E <= 32) return launch_route<DT, 2, 32>(c, x, wg, bias, idx, w, st);
    return launch_route<DT, 1, 64>(c, x, wg, bias, idx, w, st);   // E > 64: several passes of 64 experts
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
