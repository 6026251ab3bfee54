// Gate of Sec. 2.1: logits = x . Wg^T (+ bias), top-k on the logits, softmax weights.
//
// The indices must be those of an exact evaluation of the logits (products of bf16 or fp32 inputs are
// exact in fp64, so fp64 accumulation is exact up to a few ulps of fp64).  Two kernels:
//
//   route_bf16_kernel   bf16 inputs, H a multiple of 32.  Rows of x and Wg are staged through LDS with
//       coalesced direct-to-LDS loads (a wave-load is 16 rows x 64 bytes) and read back in the operand
//       layout of v_mfma_f32_16x16x32_bf16.  One such MFMA with a zero accumulator gives, per (token,
//       expert), the sum of 32 EXACT products rounded to fp32; these run sums are added in fp64.  The
//       same instruction applied to (x, x) and (Wg, Wg) gives the squared norms, hence by Cauchy-Schwarz
//       a bound B on the error of every logit of a token.  A token whose k+1 largest logits are all
//       further apart than 2B has its indices certified.  For any other token (a few per thousand) the
//       block evaluates again, with fp64 FMAs on the vector unit, the logits of every expert within 2B of
//       the k-th largest - no other expert can be among the true k largest - and selects once more.
//   route_mfma_kernel   every token in fp64 on the fp64 matrix cores: fp32 inputs and any H.
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

// Selection for one token by one wave: the k largest of z[0..E) (ties to the lower index), softmax
// weights.  With CHECK the (k+1)-th largest is extracted as well and the function returns whether every gap
// between consecutive ones exceeds `min_gap` (wave-uniform).
template <bool CHECK>
__device__ __forceinline__ bool select_topk(const double* __restrict__ z, int E, int k, int renorm, int t, int lane,
                                            double min_gap, int32_t* __restrict__ topk_idx, float* __restrict__ topk_w) {
    // up to 4 candidate experts per lane: lane, lane + 64, ...
    double cand[MOE_MAX_E / 64];
    bool taken[MOE_MAX_E / 64];
#pragma unroll
    for (int i = 0; i < MOE_MAX_E / 64; ++i) {
        const int e = lane + 64 * i;
        taken[i] = !(e < E);
        cand[i] = (e < E) ? z[e] : 0.0;
    }
    double zmax = 0.0, my_z = 0.0, prev = 0.0;
    int my_e = 0;
    bool safe = true;
    const int n_take = CHECK ? min(k + 1, E) : k;
    for (int j = 0; j < n_take; ++j) {
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
        if (CHECK && j > 0 && !(prev - best > min_gap)) safe = false;
        prev = best;
        if (j < k && lane == j) { my_z = best; my_e = best_e; }
    }
    // weights: the probabilities only need 1e-5, so the exponentials are taken in fp32 of the fp64
    // differences (all <= 0)
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
    return safe;
}

// ---------------------------------------------------------------------------------------------
// Fast path for bf16.
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// A staged piece is 16 rows x 64 bytes = 1 KB, filled by ONE wave-wide direct-to-LDS load (lane l fills the
// 16 bytes at l * 16).  The 16-byte chunk index is XOR-ed with row / 4, which spreads the 16 lanes of an MFMA
// operand read (16 consecutive rows, same chunk) over all LDS banks:
//     slot(r, c) = 4 r + (c ^ (r >> 2)),   r = 0..15, c = 0..3.
__device__ __forceinline__ int piece_slot(int r, int c) { return (r << 2) + (c ^ (r >> 2)); }

// s_waitcnt vmcnt(n) alone (expcnt and lgkmcnt left at "no wait"): n in [0, 63]
#define MOE_WAIT_VM(n) __builtin_amdgcn_s_waitcnt((((n) & 0xF) | (((n) >> 4) << 14) | 0x0F70))

// Error of a run sum.  An MFMA adds 32 exact products (and the previous MFMA's result when runs are chained).
// The matrix core does not add them exactly: it aligns the terms to the largest one and drops what falls below
// about 25 bits (probing shows 2^25 + 31 * 1.0 coming out as 2^25 + 24).  Whatever the order and the internal
// width, a term dropped or cut on alignment loses less than one unit in the last place of fp32 relative to the
// largest partial sum, so one MFMA is off by at most 32 * 2^-23 * sum |x_i w_i| = 2^-18 * sum |x_i w_i|, a chain
// of RUN by RUN times that plus the 33rd term of the later links (3 %), and by Cauchy-Schwarz the whole row by
// RUN * 2^-18 * |x| |w| (the fp64 additions are negligible).  5 % is added for the chain and for the fp32
// rounding of the norms.  A GPU test feeds adversarial operands to the same instruction and holds it to this bound.
constexpr float kLogitErr = 1.05f * 3.814697265625e-6f;     // 1.05 * 2^-18, per MFMA of a chain

// Exchanges inside a group of L = 4 or 16 neighbouring lanes by data-parallel-primitive moves (no trip through
// the LDS crossbar, unlike a general shuffle): for a quad the lane whose index differs in bit 0 or 1, for a
// row of 16 the lane N places further round the row.  Combining a value with its partners at distances
// L/2, ..., 2, 1 leaves every lane of the group with the combination over the whole group.
template <int CTRL> __device__ __forceinline__ int dpp_move(int v) { return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xF, 0xF, true); }
template <int CTRL> __device__ __forceinline__ float dpp_move(float v) { return __int_as_float(dpp_move<CTRL>(__float_as_int(v))); }
template <int CTRL> __device__ __forceinline__ double dpp_move(double v) {
    return __hiloint2double(dpp_move<CTRL>(__double2hiint(v)), dpp_move<CTRL>(__double2loint(v)));
}
constexpr int kQuadXor1 = 0xB1, kQuadXor2 = 0x4E;       // quad_perm [1,0,3,2] and [2,3,0,1]
constexpr int kRowRor1 = 0x121, kRowRor2 = 0x122, kRowRor4 = 0x124, kRowRor8 = 0x128;
template <int L> __device__ __forceinline__ float group_sum(float v) {
    if (L == 16) { v += dpp_move<kRowRor8>(v); v += dpp_move<kRowRor4>(v); v += dpp_move<kRowRor2>(v); v += dpp_move<kRowRor1>(v); }
    else { v += dpp_move<kQuadXor2>(v); v += dpp_move<kQuadXor1>(v); }
    return v;
}
template <int L> __device__ __forceinline__ float group_max(float v) {
    if (L == 16) { v = fmaxf(v, dpp_move<kRowRor8>(v)); v = fmaxf(v, dpp_move<kRowRor4>(v)); v = fmaxf(v, dpp_move<kRowRor2>(v)); v = fmaxf(v, dpp_move<kRowRor1>(v)); }
    else { v = fmaxf(v, dpp_move<kQuadXor2>(v)); v = fmaxf(v, dpp_move<kQuadXor1>(v)); }
    return v;
}

// Selection for one token by a group of L neighbouring lanes (sub = 0..L-1; lane `sub` looks after experts sub,
// sub + L, ..., at most NC of them, read once from zr[0..E) in LDS): the k + 1 largest, ties to the lower index;
// softmax weights; returns whether every gap between consecutive ones exceeds min_gap (a negative min_gap: only
// the k largest are extracted and the answer means nothing), and the k-th largest in *kth.  selw: LDS scratch
// [k] of this token.
template <int NC, int L>
__device__ __forceinline__ bool select_group(const double* __restrict__ zr, int E, int k, int renorm, int t, int sub,
                                             double min_gap, float* __restrict__ selw, int32_t* __restrict__ topk_idx,
                                             float* __restrict__ topk_w, double* kth) {
    double cv[NC];
    bool live[NC];
#pragma unroll
    for (int i = 0; i < NC; ++i) {
        live[i] = sub + L * i < E;
        cv[i] = live[i] ? zr[sub + L * i] : 0.0;
    }
    const int n_take = min(min_gap >= 0.0 ? k + 1 : k, E);   // a negative min_gap: no gaps wanted, the k largest only
    double zmax = 0.0, prev = 0.0;
    float den = 1.f, wsum = 0.f;
    bool safe = true;
    for (int j = 0; j < n_take; ++j) {
        double best = 0.0;
        int best_e = 0x7fffffff;                         // "nothing": loses against every real candidate
#pragma unroll
        for (int i = 0; i < NC; ++i)
            if (live[i] && (best_e == 0x7fffffff || cv[i] > best)) { best = cv[i]; best_e = sub + L * i; }
#define MOE_GROUP_STEP(CTRL)                                                                                    \
        {                                                                                                       \
            const double ob = dpp_move<CTRL>(best);                                                             \
            const int oe = dpp_move<CTRL>(best_e);                                                              \
            if ((oe != 0x7fffffff) && (best_e == 0x7fffffff || ob > best || (ob == best && oe < best_e))) { best = ob; best_e = oe; } \
        }
        if (L == 16) {
            MOE_GROUP_STEP(kRowRor8)
            MOE_GROUP_STEP(kRowRor4)
            MOE_GROUP_STEP(kRowRor2)
            MOE_GROUP_STEP(kRowRor1)
        } else {
            MOE_GROUP_STEP(kQuadXor2)
            MOE_GROUP_STEP(kQuadXor1)
        }
#undef MOE_GROUP_STEP
#pragma unroll
        for (int i = 0; i < NC; ++i)
            if (sub + L * i == best_e) live[i] = false;
        if (j == 0) {
            zmax = best;
            float part = 0.f;
#pragma unroll
            for (int i = 0; i < NC; ++i)
                if (sub + L * i < E) part += __expf((float)(cv[i] - zmax));
            den = group_sum<L>(part);
        } else if (!(prev - best > min_gap)) {
            safe = false;
        }
        prev = best;
        if (j == k - 1) *kth = best;
        if (j < k) {
            const float wj = __expf((float)(best - zmax)) / den;
            wsum += wj;
            if (sub == 0) {
                topk_idx[(size_t)t * k + j] = best_e;
                selw[j] = wj;
            }
        }
    }
    if (sub == 0) {
        const float scale = renorm ? 1.f / wsum : 1.f;
        for (int j = 0; j < k; ++j) topk_w[(size_t)t * k + j] = selw[j] * scale;
    }
    return safe;
}

// NT expert tiles (16 experts each) per pass, MT token tiles (16 tokens each) per block, R ring slots per wave,
// RUN MFMAs chained in fp32 before their sum goes to fp64; a token is selected by L lanes with NC candidate
// experts each (L * NC >= E per pass of the selection, L chosen so that the block's threads cover its tokens once).
// The S waves of a block split the hidden dimension; a wave stages its own pieces (no block barrier in
// the loop) and keeps MT x NT partial tiles in fp64; partial tiles are added in wave order through LDS.
//
// TIMED (diagnostics, moe_diag_route_phases): the same kernel with the 100 MHz wall clock read by lane 0 of every wave
// at the phase boundaries into marks[block][wave (16)][8]: 0 start, 1 own part of the loop done, 2 all waves
// done, 3 partial tiles added, 4 selected, 5 end (left untouched by a block with nothing to evaluate again);
// [block][0][6] = tokens evaluated again.  The ordinary instantiation contains none of it.
template <int NT, int MT, int R, int RUN, int NC, int L, int MAXT, bool TIMED>
__global__ __launch_bounds__(MAXT) void route_bf16_kernel(const uint16_t* __restrict__ x, const uint16_t* __restrict__ wg,
                                                          const float* __restrict__ bias, int T, int H, int E, int k, int renorm,
                                                          int32_t* __restrict__ topk_idx, float* __restrict__ topk_w,
                                                          long long* __restrict__ marks) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];
#define MOE_MARK(i)                                                                                                      \
    do {                                                                                                                 \
        if (TIMED && (threadIdx.x & 63) == 0)                                                                            \
            marks[((size_t)blockIdx.x * 16 + (threadIdx.x >> 6)) * 8 + (i)] = (long long)wall_clock64();                  \
    } while (0)
    MOE_MARK(0);
    constexpr int EP = NT * 16, TP = MT * 16, PIECES = MT + NT, kRouteMaxWaves = MAXT / 64;
    const int lane = threadIdx.x & 63, r = lane & 15, g = lane >> 4;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), S = blockDim.x >> 6;
    const int tok0 = blockIdx.x * TP;
    const int ngrp = H / 32;                             // groups of 32 hidden values = 64 bytes per row
    const int per = (ngrp + S - 1) / S;
    const int b_lo = wave * per, b_hi = min(b_lo + per, ngrp);
    // LDS: [ring: S x R x PIECES KB | aliased after the loop by the partial tiles and norm parts]
    //      [zl] [bias] [thresholds] [xn2] [wn2] [selw] [tokens to evaluate again] [(token, expert) pairs] [2 counters]
    const size_t ring_bytes = (size_t)S * R * PIECES * 1024;
    unsigned char* my_ring = lds + (size_t)wave * R * PIECES * 1024;
    double* zpart = reinterpret_cast<double*>(lds);                               // [S][TP][16]
    float* xn_part = reinterpret_cast<float*>(lds + (size_t)S * TP * 16 * 8);     // [S][TP]
    float* wn_part = xn_part + (size_t)S * TP;                                    // [S][EP]
    const int ZP = E + 4;                                                         // row pitch of zl: spreads the rows over the banks
    double* zl = reinterpret_cast<double*>(lds + ring_bytes);                     // [TP][ZP]
    double* bias_l = zl + (size_t)TP * ZP;                                        // [E]
    double* redo_thr = bias_l + E;                                                // [TP] (k-th largest logit) - 2B of a token
    float* xn2 = reinterpret_cast<float*>(redo_thr + TP);                         // [TP]
    float* wn2 = xn2 + TP;                                                        // [E]
    float* selw = wn2 + E;                                                        // [TP][MOE_MAX_K]
    int* redo_tok = reinterpret_cast<int*>(selw + TP * MOE_MAX_K);                // [TP] tokens to evaluate again
    int* pairs = redo_tok + TP;                                                   // [TP * E] (token << 16) | expert to evaluate exactly
    int* counters = pairs + TP * E;                                               // [2] how many of each
    if (threadIdx.x < 2) counters[threadIdx.x] = 0;
    for (int e = threadIdx.x; e < E; e += blockDim.x) bias_l[e] = bias ? (double)bias[e] : 0.0;   // read long before it is needed
    // the lane's part in filling a piece: row lr of the piece, 16-byte chunk lc of the group
    const int lr = lane >> 2, lc = (lane & 3) ^ (lane >> 4);
    const char* xsrc[MT];
#pragma unroll
    for (int m = 0; m < MT; ++m)
        xsrc[m] = reinterpret_cast<const char*>(x) + (size_t)min(tok0 + m * 16 + lr, T - 1) * H * 2 + lc * 16;
    const int frag_off = piece_slot(r, g) * 16;          // where lane (r, g) finds chunk g of row r inside a piece

    f32x4 xacc[MT];
#pragma unroll
    for (int m = 0; m < MT; ++m) xacc[m] = f32x4{0.f, 0.f, 0.f, 0.f};
    const f32x4 zero4 = {0.f, 0.f, 0.f, 0.f};

    for (int e0 = 0; e0 < E; e0 += EP) {
        const char* wsrc[NT];                            // experts past E are clamped to the last row: computed, never used
#pragma unroll
        for (int n = 0; n < NT; ++n)
            wsrc[n] = reinterpret_cast<const char*>(wg) + (size_t)min(e0 + n * 16 + lr, E - 1) * H * 2 + lc * 16;
        double acc[MT][NT][4];
        f32x4 run[MT][NT];
#pragma unroll
        for (int m = 0; m < MT; ++m)
#pragma unroll
            for (int n = 0; n < NT; ++n) {
                run[m][n] = zero4;
#pragma unroll
                for (int i = 0; i < 4; ++i) acc[m][n][i] = 0.0;
            }
        f32x4 wacc[NT];
#pragma unroll
        for (int n = 0; n < NT; ++n) wacc[n] = zero4;
        auto issue = [&](int b, int slot) {              // group b (clamped into the wave's range) into ring slot `slot`
            const size_t goff = (size_t)min(b, b_hi - 1) * 64;
            unsigned char* dst = my_ring + (size_t)slot * PIECES * 1024;
            // (the source addresses go through locals: handing the builtin an element of a captured array makes
            // the host pass drop the kernel's stub without a diagnostic)
#pragma unroll
            for (int m = 0; m < MT; ++m) {
                const char* gp = xsrc[m] + goff;
                __builtin_amdgcn_global_load_lds(gp, (__attribute__((address_space(3))) void*)(dst + m * 1024), 16, 0, 0);
            }
#pragma unroll
            for (int n = 0; n < NT; ++n) {
                const char* gp = wsrc[n] + goff;
                __builtin_amdgcn_global_load_lds(gp, (__attribute__((address_space(3))) void*)(dst + (MT + n) * 1024), 16, 0, 0);
            }
        };
        if (b_lo < b_hi) {
#pragma unroll
            for (int p = 0; p < R; ++p) issue(b_lo + p, p);
            int slot = 0;
            for (int b = b_lo; b < b_hi; ++b) {
                __builtin_amdgcn_sched_barrier(0);
                MOE_WAIT_VM((R - 1) * PIECES);           // R slots are always in flight: the oldest one has landed
                asm volatile("" ::: "memory");
                const unsigned char* src = my_ring + (size_t)slot * PIECES * 1024 + frag_off;
                bf16x8 xf[MT], wf[NT];
#pragma unroll
                for (int m = 0; m < MT; ++m) xf[m] = *reinterpret_cast<const bf16x8*>(src + m * 1024);
#pragma unroll
                for (int n = 0; n < NT; ++n) wf[n] = *reinterpret_cast<const bf16x8*>(src + (MT + n) * 1024);
                asm volatile("" ::: "memory");
                __builtin_amdgcn_s_waitcnt(0xC07F);      // lgkmcnt(0): the fragments are in registers, the slot is free
                __builtin_amdgcn_sched_barrier(0);
                issue(b + R, slot);
                __builtin_amdgcn_sched_barrier(0);
                const bool flush = RUN == 1 || ((b - b_lo) % RUN) == RUN - 1 || b == b_hi - 1;   // wave-uniform
#pragma unroll
                for (int m = 0; m < MT; ++m) {
                    if (e0 == 0) xacc[m] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xf[m], xf[m], xacc[m], 0, 0, 0);
#pragma unroll
                    for (int n = 0; n < NT; ++n)
                        run[m][n] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xf[m], wf[n], run[m][n], 0, 0, 0);
                }
#pragma unroll
                for (int n = 0; n < NT; ++n) wacc[n] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[n], wf[n], wacc[n], 0, 0, 0);
                if (flush) {
#pragma unroll
                    for (int m = 0; m < MT; ++m)
#pragma unroll
                        for (int n = 0; n < NT; ++n) {
#pragma unroll
                            for (int i = 0; i < 4; ++i) acc[m][n][i] += (double)run[m][n][i];
                            run[m][n] = zero4;
                        }
                }
                slot = (slot + 1 == R) ? 0 : slot + 1;
            }
            MOE_WAIT_VM(0);                              // no load may still target the ring when it is reused below
        }
        MOE_MARK(1);
        __syncthreads();
        MOE_MARK(2);
        // D of the MFMA: lane (r, g) holds rows 4 g + i (tokens), column r (expert), i = 0..3; the diagonal of
        // a (v, v) product (row == column) is therefore in the lanes with r / 4 == g, element r % 4
#pragma unroll
        for (int n = 0; n < NT; ++n)
            if ((r >> 2) == g) wn_part[(size_t)wave * EP + n * 16 + r] = wacc[n][r & 3];
        if (e0 == 0) {
#pragma unroll
            for (int m = 0; m < MT; ++m)
                if ((r >> 2) == g) xn_part[(size_t)wave * TP + m * 16 + r] = xacc[m][r & 3];
        }
#pragma unroll
        for (int n = 0; n < NT; ++n) {
#pragma unroll
            for (int m = 0; m < MT; ++m)
#pragma unroll
                for (int i = 0; i < 4; ++i) zpart[((size_t)wave * TP + m * 16 + 4 * g + i) * 16 + r] = acc[m][n][i];
            __syncthreads();
            // the S parts of an element: all reads first (a loop over S would wait for each in turn), sum in wave order
            for (int q = threadIdx.x; q < TP * 16; q += blockDim.x) {
                const int tt = q >> 4, e = e0 + n * 16 + (q & 15);
                double part[kRouteMaxWaves];
#pragma unroll
                for (int w = 0; w < kRouteMaxWaves; ++w) part[w] = (w < S) ? zpart[(size_t)w * TP * 16 + q] : 0.0;
                double sum = part[0];
#pragma unroll
                for (int w = 1; w < kRouteMaxWaves; ++w)
                    if (w < S) sum += part[w];
                if (e < E) zl[(size_t)tt * ZP + e] = sum + bias_l[e];
            }
            if (n == 0) {
                for (int q = threadIdx.x; q < EP + (e0 == 0 ? TP : 0); q += blockDim.x) {
                    const bool is_w = q < EP;
                    const float* src = is_w ? wn_part + q : xn_part + (q - EP);
                    const int pitch = is_w ? EP : TP;
                    float part[kRouteMaxWaves];
#pragma unroll
                    for (int w = 0; w < kRouteMaxWaves; ++w) part[w] = (w < S) ? src[(size_t)w * pitch] : 0.f;
                    float sum = 0.f;
#pragma unroll
                    for (int w = 0; w < kRouteMaxWaves; ++w) sum += part[w];
                    if (!is_w) xn2[q - EP] = sum;
                    else if (e0 + q < E) wn2[e0 + q] = sum;
                }
            }
            __syncthreads();
        }
    }
    MOE_MARK(3);
    // selection: L lanes per token
    const int sub = threadIdx.x & (L - 1);
    for (int tsel = threadIdx.x / L; tsel < TP && tok0 + tsel < T; tsel += blockDim.x / L) {
        float wmax = 0.f;                                // the largest expert norm
        for (int e = sub; e < E; e += L) wmax = fmaxf(wmax, wn2[e]);
        wmax = group_max<L>(wmax);
        const double min_gap = 2.0 * (double)((float)RUN * kLogitErr * sqrtf(xn2[tsel] * wmax));
        double kth = 0.0;
        const bool safe = select_group<NC, L>(zl + (size_t)tsel * ZP, E, k, renorm, tok0 + tsel, sub, min_gap,
                                              selw + tsel * MOE_MAX_K, topk_idx, topk_w, &kth);
        if (!safe && sub == 0) {                         // the order of this list does not reach any result
            redo_thr[tsel] = kth - min_gap;
            redo_tok[atomicAdd(&counters[0], 1)] = tsel;
        }
    }
    __syncthreads();
    // Tokens that could not be certified.  Every logit is within B of its true value, so an expert whose
    // logit is more than 2B below the k-th largest is truly below k experts and cannot be selected: the true
    // logits of the others (usually k + 1 of them) are evaluated with fp64 FMAs - a wave per (token, expert)
    // pair, the lanes sharing the hidden dimension, lane sums added in a fixed butterfly order - and put in
    // place of the approximate ones; the selection on the patched row is exact.
    const int n_redo = counters[0];
    MOE_MARK(4);
    if (TIMED && threadIdx.x == 0) marks[(size_t)blockIdx.x * 16 * 8 + 6] = n_redo;
    if (n_redo == 0) return;                             // block-uniform
    for (int q = threadIdx.x; q < n_redo * E; q += blockDim.x) {
        const int tsel = redo_tok[q / E], e = q % E;
        if (zl[(size_t)tsel * ZP + e] >= redo_thr[tsel]) pairs[atomicAdd(&counters[1], 1)] = (tsel << 16) | e;
    }
    __syncthreads();
    const int n_pairs = counters[1];
    const int nchunk = H / 8;
    // PU pairs per wave at a time, CU chunks of each per lane: every load of a step is issued before the first
    // is used (one round trip to memory per step)
    constexpr int PU = (MT == 1) ? 1 : 4, CU = (MT == 1) ? 8 : 4;
    for (int p0 = wave * PU; p0 < n_pairs; p0 += S * PU) {
        const u32x4* xr[PU];
        const u32x4* wr[PU];
        double sum[PU];
#pragma unroll
        for (int u = 0; u < PU; ++u) {
            const int pr = pairs[min(p0 + u, n_pairs - 1)];
            xr[u] = reinterpret_cast<const u32x4*>(x) + (size_t)(tok0 + (pr >> 16)) * nchunk;
            wr[u] = reinterpret_cast<const u32x4*>(wg) + (size_t)(pr & 0xffff) * nchunk;
            sum[u] = 0.0;
        }
        for (int c0 = lane; c0 < nchunk; c0 += 64 * CU) {
            u32x4 xq[PU][CU], wq[PU][CU];
#pragma unroll
            for (int u = 0; u < PU; ++u)
#pragma unroll
                for (int v = 0; v < CU; ++v) {
                    const int c = min(c0 + 64 * v, nchunk - 1);          // past the end: fetched again, not added
                    xq[u][v] = xr[u][c];
                    wq[u][v] = wr[u][c];
                }
#pragma unroll
            for (int u = 0; u < PU; ++u)
#pragma unroll
                for (int v = 0; v < CU; ++v) {
                    if (c0 + 64 * v < nchunk) {
                        double xv[8], wv[8];
                        Chunk<MOE_BF16>::unpack(xq[u][v], xv);
                        Chunk<MOE_BF16>::unpack(wq[u][v], wv);
#pragma unroll
                        for (int i = 0; i < 8; ++i) sum[u] = fma(xv[i], wv[i], sum[u]);
                    }
                }
        }
#pragma unroll
        for (int o = 32; o >= 1; o >>= 1)
#pragma unroll
            for (int u = 0; u < PU; ++u) sum[u] += __shfl_xor(sum[u], o, 64);
        if (lane == 0) {
#pragma unroll
            for (int u = 0; u < PU; ++u)
                if (p0 + u < n_pairs) {
                    const int pr = pairs[p0 + u];
                    zl[(size_t)(pr >> 16) * ZP + (pr & 0xffff)] = sum[u] + bias_l[pr & 0xffff];
                }
        }
    }
    __syncthreads();
    for (int f = threadIdx.x / L; f < n_redo; f += blockDim.x / L) {
        const int tsel = redo_tok[f];
        double kth = 0.0;
        select_group<NC, L>(zl + (size_t)tsel * ZP, E, k, renorm, tok0 + tsel, sub, -1.0, selw + tsel * MOE_MAX_K, topk_idx, topk_w, &kth);
    }
    MOE_MARK(5);
#undef MOE_MARK
}

// ---------------------------------------------------------------------------------------------
// Every token in fp64 on the fp64 matrix cores.
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
        if (t < T) select_topk<false>(zl + (size_t)tt * E, E, k, renorm, t, lane, 0.0, topk_idx, topk_w);
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

template <int NT, int MT, int R, int RUN, int NC, int L, int MAXT, bool TIMED>
int launch_route_bf16(const moe_ctx* c, const void* x, const void* wg, const float* bias, int32_t* idx, float* w,
                      hipStream_t st, long long* marks, int32_t* tokens_per_block) {
    const moe_shape& s = c->s;
    const int ngrp = s.H / 32, TP = MT * 16;
    int S = MAXT / 64;                                    // waves per block: no more than there are groups to share out
    while (S > 1 && S > ngrp) S >>= 1;
    const size_t lds = (size_t)S * R * (MT + NT) * 1024 + ((size_t)TP * (s.E + 4) + s.E + TP) * sizeof(double) +
                       (size_t)(TP + s.E + TP * MOE_MAX_K) * sizeof(float) + ((size_t)TP + (size_t)TP * s.E + 2) * sizeof(int);
    static bool attr_done = false;
    if (!attr_done) {
        MOE_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&route_bf16_kernel<NT, MT, R, RUN, NC, L, MAXT, TIMED>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
        attr_done = true;
    }
    if (lds > 160 * 1024) return moe_set_error(MOE_EINTERNAL, "moe_route: %zu bytes of LDS", lds);
    if (tokens_per_block) *tokens_per_block = TP;
    hipLaunchKernelGGL((route_bf16_kernel<NT, MT, R, RUN, NC, L, MAXT, TIMED>), dim3((s.T + TP - 1) / TP), dim3(64 * S), lds, st,
                       reinterpret_cast<const uint16_t*>(x), reinterpret_cast<const uint16_t*>(wg), bias, s.T, s.H, s.E, s.k,
                       s.renorm, idx, w, marks);
    MOE_LAUNCH_CHECK("route_bf16_kernel");
    return MOE_OK;
}

template <int DT>
int route_exact(const moe_ctx* c, const void* x, const void* wg, const float* bias, int32_t* idx, float* w,
                hipStream_t st) {
    const int E = c->s.E;
    if (E <= 16) return launch_route_mfma<DT, 1, 4>(c, x, wg, bias, idx, w, st);
    if (E <= 32) return launch_route_mfma<DT, 2, 4>(c, x, wg, bias, idx, w, st);
    return launch_route_mfma<DT, 4, 3>(c, x, wg, bias, idx, w, st);   // E > 64: several passes of 64 experts
}

// tokens_per_block: where the bf16 kernel says how many tokens a block takes (0: the fp64 kernel ran, no marks)
template <bool TIMED>
int route_dispatch(const moe_ctx* c, const void* x, const void* wg, const float* bias, int32_t* idx, float* w,
                   hipStream_t st, long long* marks, int32_t* tokens_per_block) {
    const moe_shape& s = c->s;
    if (tokens_per_block) *tokens_per_block = 0;
    if (s.dtype == MOE_F32) return route_exact<MOE_F32>(c, x, wg, bias, idx, w, st);
    if (s.H % 32 != 0) return route_exact<MOE_BF16>(c, x, wg, bias, idx, w, st);
#define MOE_ROUTE(...) launch_route_bf16<__VA_ARGS__, TIMED>(c, x, wg, bias, idx, w, st, marks, tokens_per_block)
    // few experts: one token tile per block, 16 waves share the hidden dimension; beyond 64: passes of 64 experts
    if (s.E <= 16) return MOE_ROUTE(1, 1, 4, 1, 1, 16, 1024);
    // up to 64 experts: two token tiles per block and eight waves, two per SIMD, so that one computes while the
    // other waits for its fragments; with many tokens four tiles per block (the gate rows are fetched from L2 once
    // per 64 tokens instead of once per 32) and one wave per SIMD
    const bool few = (s.T + 63) / 64 < 200;
    if (s.E <= 32) return few ? MOE_ROUTE(2, 2, 2, 2, 2, 16, 512) : MOE_ROUTE(2, 4, 3, 2, 8, 4, 256);
    if (s.E <= 64) return few ? MOE_ROUTE(4, 2, 2, 2, 4, 16, 512) : MOE_ROUTE(4, 4, 3, 2, 16, 4, 256);
    return MOE_ROUTE(4, 1, 2, 2, 16, 16, 512);
#undef MOE_ROUTE
}

}  // namespace

extern "C" int moe_route(moe_ctx* ctx, const void* x, const void* Wg, const float* gate_bias, int32_t* topk_idx,
                         float* topk_w, void* stream) {
    if (!ctx || !x || !Wg || !topk_idx || !topk_w) return moe_set_error(MOE_EINVAL, "moe_route: NULL argument");
    if (!aligned16(x) || !aligned16(Wg)) return moe_set_error(MOE_EALIGN, "moe_route: x and Wg must be 16-byte aligned");
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    ctx->rank_src = nullptr;                             // the indices are about to change: cached slot ranks are stale
    return route_dispatch<false>(ctx, x, Wg, gate_bias, topk_idx, topk_w, st, nullptr, nullptr);
}

extern "C" int moe_diag_route_phases(moe_ctx* ctx, const void* x, const void* Wg, const float* gate_bias, int32_t* topk_idx,
                                     float* topk_w, int64_t* marks, size_t marks_len, int32_t* tokens_per_block,
                                     void* stream) {
    if (!ctx || !x || !Wg || !topk_idx || !topk_w || !marks || !tokens_per_block)
        return moe_set_error(MOE_EINVAL, "moe_diag_route_phases: NULL argument");
    if (!aligned16(x) || !aligned16(Wg)) return moe_set_error(MOE_EALIGN, "moe_diag_route_phases: x and Wg must be 16-byte aligned");
    if (marks_len < ((size_t)ctx->s.T / 16 + 1) * 128)
        return moe_set_error(MOE_ESHAPE, "moe_diag_route_phases: marks needs (T / 16 + 1) * 128 elements");
    ctx->rank_src = nullptr;
    static_assert(sizeof(long long) == sizeof(int64_t), "marks are 64-bit");
    return route_dispatch<true>(ctx, x, Wg, gate_bias, topk_idx, topk_w, reinterpret_cast<hipStream_t>(stream),
                                reinterpret_cast<long long*>(marks), tokens_per_block);
}
