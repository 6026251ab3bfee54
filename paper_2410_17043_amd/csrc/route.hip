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
        // two chunks per trip: all 2*TT token loads are in flight before the first weight is touched
        for (int c = c_lo + lane; c < c_hi; c += 128) {
            u32x4 raw[2][TT];
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int tt = 0; tt < TT; ++tt) {
                    const int t = min(tok0 + tt, T - 1);
                    const int cc = min(c + 64 * u, c_hi - 1);
                    raw[u][tt] = reinterpret_cast<const u32x4*>(x)[(size_t)t * nchunk + cc];
                }
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const int cc = c + 64 * u;
                if (cc >= c_hi) continue;
                double xv[TT][V];
#pragma unroll
                for (int tt = 0; tt < TT; ++tt) Chunk<DT>::unpack(raw[u][tt], xv[tt]);
                // experts past E are clamped to the last row: computed, never written out (keeps every
                // index below a compile-time constant, so the partial logits stay in registers)
#pragma unroll
                for (int e = 0; e < ET; ++e) {
                    double wv[V];
                    Chunk<DT>::load(wg, (size_t)min(e0 + e, E - 1) * nchunk + cc, wv);
#pragma unroll
                    for (int tt = 0; tt < TT; ++tt)
#pragma unroll
                        for (int v = 0; v < V; ++v) acc[tt * ET + e] = fma(xv[tt][v], wv[v], acc[tt * ET + e]);
                }
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
}

// ---------------------------------------------------------------------------------------------
// Many experts (16 < E <= 64): one LANE per token.  The gate weight is first converted to fp64
// and transposed to [H][64] (zero padded), so that the 64 weights of one hidden index are 512
// contiguous bytes that every lane of a wave needs at the same time: they are fetched with scalar
// loads and feed the FMAs as scalar operands (one v_fma_f64 per token, expert and hidden index;
// nothing is converted or shuffled in the inner loop).  A block of S waves owns 64 tokens, wave s
// the s-th part of the hidden dimension; token rows are staged through LDS in 128-byte pieces so
// that memory sees whole lines while each lane reads its own row.  Partial logits meet in LDS;
// wave 0 then picks the top-k of every token with one lane per token.
template <int DT>
__global__ __launch_bounds__(256) void wg_to_f64_kernel(const void* __restrict__ wg, int E, int H, double* __restrict__ out) {
    const int i = blockIdx.x * 256 + threadIdx.x;          // one output element [h][e]
    if (i >= H * 64) return;
    const int h = i >> 6, e = i & 63;
    double v = 0.0;
    if (e < E) {
        if (DT == MOE_BF16) v = (double)__uint_as_float((uint32_t)reinterpret_cast<const uint16_t*>(wg)[(size_t)e * H + h] << 16);
        else v = (double)reinterpret_cast<const float*>(wg)[(size_t)e * H + h];
    }
    out[i] = v;
}

constexpr int kTokPitch = 144;                             // bytes per staged token row piece (128 + 16: spreads banks)

template <int DT, int ET>
__global__ __launch_bounds__(512) void route_tok_kernel(const void* __restrict__ x, const double* __restrict__ wg64t,
                                                         const float* __restrict__ bias, int T, int H, int E, int k,
                                                         int renorm, int S, int32_t* __restrict__ topk_idx,
                                                         float* __restrict__ topk_w) {
    constexpr int V = Chunk<DT>::V;                        // elements per 16 bytes
    constexpr int PIECE = 8 * V;                           // hidden indices per 128-byte piece
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    double* zsum = reinterpret_cast<double*>(smem);        // [ET][64]: logits, expert-major so lanes (tokens) are contiguous
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    unsigned char* stage = smem + (size_t)ET * 64 * sizeof(double) + (size_t)wave * 64 * kTokPitch;
    const int tok0 = blockIdx.x * 64;
    const int n_piece = H / PIECE;                         // H * elem is a multiple of 128 for this kernel
    const int per = (n_piece + S - 1) / S;
    const int p_lo = wave * per, p_hi = min(p_lo + per, n_piece);
    const int row_bytes = H * (DT == MOE_BF16 ? 2 : 4);
    const unsigned char* xb = reinterpret_cast<const unsigned char*>(x);

    double acc[ET];
#pragma unroll
    for (int e = 0; e < ET; ++e) acc[e] = 0.0;
    for (int p = p_lo; p < p_hi; ++p) {
        // 64 rows x 128 bytes: 8 lanes per row, 8 rows per load, whole lines
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const int r = q * 8 + (lane >> 3);
            const int t = min(tok0 + r, T - 1);
            const u32x4 v = *reinterpret_cast<const u32x4*>(xb + (size_t)t * row_bytes + (size_t)p * 128 + (lane & 7) * 16);
            *reinterpret_cast<u32x4*>(stage + r * kTokPitch + (lane & 7) * 16) = v;
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            double xv[V];
            Chunk<DT>::load(stage + lane * kTokPitch, c, xv);        // this lane's token, 16 bytes
            const double* wrow = wg64t + ((size_t)p * PIECE + c * V) * 64;
#pragma unroll
            for (int v = 0; v < V; ++v)
#pragma unroll
                for (int e = 0; e < ET; ++e) acc[e] = fma(xv[v], wrow[v * 64 + e], acc[e]);
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();                   // the stage is rewritten by the next piece
    }
    // partial logits of the S waves, added in wave order
    for (int s = 0; s < S; ++s) {
        if (wave == s) {
#pragma unroll
            for (int e = 0; e < ET; ++e) zsum[e * 64 + lane] = (s == 0 ? 0.0 : zsum[e * 64 + lane]) + acc[e];
        }
        __syncthreads();
    }
    if (wave != 0) return;
    const int t = tok0 + lane;
    double z[ET];
#pragma unroll
    for (int e = 0; e < ET; ++e) z[e] = (e < E) ? zsum[e * 64 + lane] + (bias ? (double)bias[e] : 0.0) : 0.0;
    double zmax = 0.0, mass = 0.0, sel_sum = 0.0;
    unsigned long long taken = 0;                           // bit e: expert e already chosen by this token
    double wsel[MOE_MAX_K];
    int esel[MOE_MAX_K];
#pragma unroll
    for (int j = 0; j < MOE_MAX_K; ++j) {
        if (j < k) {
            double best = 0.0;
            int best_e = -1;
#pragma unroll
            for (int e = 0; e < ET; ++e) {
                const bool free_e = e < E && !((taken >> e) & 1ull);
                if (free_e && (best_e < 0 || z[e] > best)) { best = z[e]; best_e = e; }
            }
            taken |= 1ull << best_e;
            if (j == 0) {
                zmax = best;
#pragma unroll
                for (int e = 0; e < ET; ++e)
                    if (e < E) mass += exp(z[e] - zmax);
            }
            esel[j] = best_e;
            wsel[j] = exp(best - zmax) / mass;
            sel_sum += wsel[j];
        }
    }
    if (t < T) {
#pragma unroll
        for (int j = 0; j < MOE_MAX_K; ++j) {
            if (j < k) {
                topk_idx[(size_t)t * k + j] = esel[j];
                topk_w[(size_t)t * k + j] = (float)(renorm ? wsel[j] / sel_sum : wsel[j]);
            }
        }
    }
}

template <int DT, int ET>
int launch_route_tok(const moe_ctx* c, const void* x, const void* wg, const float* bias, int32_t* idx, float* w,
                     hipStream_t st) {
    const moe_shape& s = c->s;
    hipLaunchKernelGGL((wg_to_f64_kernel<DT>), dim3((s.H * 64 + 255) / 256), dim3(256), 0, st, wg, s.E, s.H, c->wg64t);
    MOE_LAUNCH_CHECK("wg_to_f64_kernel");
    const int groups = (s.T + 63) / 64;
    int S = 1;                                              // waves per block: fill about 2048 wave slots, at most 8
    while (S < 8 && groups * S < 2048) S *= 2;
    const size_t lds = (size_t)ET * 64 * sizeof(double) + (size_t)S * 64 * kTokPitch;
    hipLaunchKernelGGL((route_tok_kernel<DT, ET>), dim3(groups), dim3(64 * S), lds, st, x, c->wg64t, bias, s.T, s.H, s.E,
                       s.k, s.renorm, S, idx, w);
    MOE_LAUNCH_CHECK("route_tok_kernel");
    return MOE_OK;
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
    // one lane per token needs whole 128-byte pieces of every row
    const bool tok_ok = c->wg64t != nullptr && ((size_t)c->s.H * elem_size(c->s.dtype)) % 128 == 0;
    if (E <= 32) return tok_ok ? launch_route_tok<DT, 32>(c, x, wg, bias, idx, w, st) : launch_route<DT, 2, 32>(c, x, wg, bias, idx, w, st);
    if (E <= 64 && tok_ok) return launch_route_tok<DT, 64>(c, x, wg, bias, idx, w, st);
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
