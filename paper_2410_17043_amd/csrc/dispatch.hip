// Traffic row (Sec. 4: d_gj) and the buffer layer that fills the send buffer in
// the planned transmission order (Sec. 3, "Communication scheduling").
//
// Both are one stable counting sort of the T*k slots by expert, done without
// atomics so the permutation is the same on every run:
//   1. count_kernel   per block of 1024 consecutive slots: slots per expert
//                     (wave ballots, summed through LDS)          -> block_hist
//   2. scan_kernel    one block: exclusive prefix over blocks per expert, the
//                     capacity rule, the traffic row, segment offsets in send order
//   3. rank_kernel    same ballots again: rank of every slot among the slots of
//                     its expert -> slot_to_row / row_to_slot
//   4. copy_kernel    one wave per token: the row is read once and written to the
//                     send rows of its kept slots (16-byte lanes, 1 KB per wave access)
#include "common.h"

namespace {

struct SegMap {                       // built on the host from expert_to_gpu and dest_order
    int16_t seg_expert[MOE_MAX_E];    // expert at each position of the send order
    uint8_t expert_gpu[MOE_MAX_E];    // destination GPU of each expert
};

constexpr int kChunks = MOE_SLOTS_PER_BLOCK / 64;   // 16 chunks of 64 slots per block, in slot order

// cnt[chunk][e] for this block's 16 chunks; returns this lane's rank inside its chunk
// among the lanes with the same expert (per round, in lane_rank[r]).
template <bool WANT_RANK>
__device__ __forceinline__ void block_chunk_counts(const int32_t* __restrict__ idx, int n_slots, int E, int* cnt,
                                                   int (&my_e)[4], int (&lane_rank)[4]) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int base = blockIdx.x * MOE_SLOTS_PER_BLOCK + wave * 256;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int s = base + r * 64 + lane;
        my_e[r] = (s < n_slots) ? idx[s] : -1;
        lane_rank[r] = 0;
    }
    const unsigned long long lt = (1ull << lane) - 1ull;
    for (int e = 0; e < E; ++e) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const unsigned long long m = __ballot(my_e[r] == e);
            if (WANT_RANK && my_e[r] == e) lane_rank[r] = __popcll(m & lt);
            if (lane == 0) cnt[(wave * 4 + r) * E + e] = __popcll(m);
        }
    }
}

__global__ __launch_bounds__(256) void count_kernel(const int32_t* __restrict__ idx, int n_slots, int E,
                                                    int32_t* __restrict__ block_hist) {
    extern __shared__ int cnt[];      // [16][E]
    int my_e[4], lane_rank[4];
    block_chunk_counts<false>(idx, n_slots, E, cnt, my_e, lane_rank);
    __syncthreads();
    for (int e = threadIdx.x; e < E; e += 256) {
        int s = 0;
#pragma unroll
        for (int c = 0; c < kChunks; ++c) s += cnt[c * E + e];
        block_hist[(size_t)blockIdx.x * E + e] = s;
    }
}

// One block of 256 threads.  Thread e walks the blocks of expert e.
__global__ __launch_bounds__(256) void scan_kernel(int32_t* __restrict__ block_hist, int n_blocks, int E, int G,
                                                   int capacity, SegMap map, int32_t* __restrict__ seg_start,
                                                   int32_t* __restrict__ expert_count, int32_t* __restrict__ dest_count,
                                                   int32_t* __restrict__ n_dropped, int32_t* __restrict__ seg_offset,
                                                   int32_t* __restrict__ seg_expert) {
    __shared__ int kept[MOE_MAX_E];
    __shared__ int raw[MOE_MAX_E];
    const int e = threadIdx.x;
    if (e < E) {
        int run = 0;
        for (int b = 0; b < n_blocks; ++b) {
            const int c = block_hist[(size_t)b * E + e];
            block_hist[(size_t)b * E + e] = run;
            run += c;
        }
        raw[e] = run;
        kept[e] = (capacity > 0 && run > capacity) ? capacity : run;
        if (expert_count) expert_count[e] = kept[e];
    }
    __syncthreads();
    if (dest_count && e < G) {
        int s = 0;
        for (int i = 0; i < E; ++i)
            if (map.expert_gpu[i] == e) s += kept[i];
        dest_count[e] = s;
    }
    if (e == 0) {
        int run = 0, drop = 0;
        for (int p = 0; p < E; ++p) {
            const int ex = map.seg_expert[p];
            if (seg_offset) seg_offset[p] = run;
            if (seg_expert) seg_expert[p] = ex;
            if (seg_start) seg_start[ex] = run;
            run += kept[ex];
            drop += raw[ex] - kept[ex];
        }
        if (seg_offset) seg_offset[E] = run;
        if (n_dropped) *n_dropped = drop;
    }
}

__global__ __launch_bounds__(256) void rank_kernel(const int32_t* __restrict__ idx, int n_slots, int E, int capacity,
                                                   const int32_t* __restrict__ block_base,
                                                   const int32_t* __restrict__ seg_start,
                                                   int32_t* __restrict__ slot_to_row, int32_t* __restrict__ row_to_slot) {
    extern __shared__ int cnt[];      // [16][E], turned into an exclusive prefix over chunks
    int my_e[4], lane_rank[4];
    block_chunk_counts<true>(idx, n_slots, E, cnt, my_e, lane_rank);
    __syncthreads();
    for (int e = threadIdx.x; e < E; e += 256) {
        int run = block_base[(size_t)blockIdx.x * E + e];
#pragma unroll
        for (int c = 0; c < kChunks; ++c) {
            const int v = cnt[c * E + e];
            cnt[c * E + e] = run;
            run += v;
        }
    }
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int base = blockIdx.x * MOE_SLOTS_PER_BLOCK + wave * 256;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int s = base + r * 64 + lane;
        if (s < n_slots) {
            const int e = my_e[r];
            int row = -1;
            if (e >= 0 && e < E) {                      // an index outside [0, E) is treated as a dropped slot
                const int rank = cnt[(wave * 4 + r) * E + e] + lane_rank[r];
                if (capacity <= 0 || rank < capacity) {
                    row = seg_start[e] + rank;
                    row_to_slot[row] = s;
                }
            }
            slot_to_row[s] = row;
        }
    }
}

// One wave per token.  row16 = 16-byte units per row.
template <int K>
__global__ __launch_bounds__(256) void copy_kernel(const u32x4* __restrict__ x, const int32_t* __restrict__ slot_to_row,
                                                   int T, int k_rt, int row16, u32x4* __restrict__ send_buf) {
    const int lane = threadIdx.x & 63;
    const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= T) return;
    const int k = (K > 0) ? K : k_rt;
    int rows[(K > 0) ? K : MOE_MAX_K];
#pragma unroll
    for (int j = 0; j < ((K > 0) ? K : MOE_MAX_K); ++j) rows[j] = (j < k) ? slot_to_row[(size_t)t * k + j] : -1;
    const u32x4* src = x + (size_t)t * row16;
    for (int c0 = 0; c0 < row16; c0 += 256) {
        u32x4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int c = c0 + u * 64 + lane;
            if (c < row16) v[u] = __builtin_nontemporal_load(src + c);
        }
#pragma unroll
        for (int j = 0; j < ((K > 0) ? K : MOE_MAX_K); ++j) {
            if (rows[j] >= 0) {
                u32x4* dst = send_buf + (size_t)rows[j] * row16;
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int c = c0 + u * 64 + lane;
                    if (c < row16) __builtin_nontemporal_store(v[u], dst + c);
                }
            }
        }
    }
}

int build_segmap(const moe_shape& s, const int32_t* expert_to_gpu, const int32_t* dest_order, SegMap* m) {
    for (int e = 0; e < s.E; ++e) {
        if (expert_to_gpu[e] < 0 || expert_to_gpu[e] >= s.G)
            return moe_set_error(MOE_ESHAPE, "expert_to_gpu[%d] = %d outside [0, %d)", e, expert_to_gpu[e], s.G);
        m->expert_gpu[e] = (uint8_t)expert_to_gpu[e];
    }
    bool seen[MOE_MAX_G] = {false};
    int p = 0;
    for (int i = 0; i < s.G; ++i) {
        const int d = dest_order ? dest_order[i] : i;
        if (d < 0 || d >= s.G || seen[d]) return moe_set_error(MOE_ESHAPE, "dest_order is not a permutation of 0..%d", s.G - 1);
        seen[d] = true;
        for (int e = 0; e < s.E; ++e)
            if (expert_to_gpu[e] == d) m->seg_expert[p++] = (int16_t)e;
    }
    return MOE_OK;
}

int launch_count_scan(moe_ctx* c, const int32_t* idx, const SegMap& map, int32_t* expert_count, int32_t* dest_count,
                      int32_t* n_dropped, int32_t* seg_offset, int32_t* seg_expert, hipStream_t st) {
    const moe_shape& s = c->s;
    const size_t lds = (size_t)kChunks * s.E * sizeof(int);
    hipLaunchKernelGGL(count_kernel, dim3(c->n_blocks), dim3(256), lds, st, idx, c->n_slots, s.E, c->block_hist);
    MOE_LAUNCH_CHECK("count_kernel");
    hipLaunchKernelGGL(scan_kernel, dim3(1), dim3(256), 0, st, c->block_hist, c->n_blocks, s.E, s.G, s.capacity, map,
                       c->seg_start, expert_count, dest_count, n_dropped, seg_offset, seg_expert);
    MOE_LAUNCH_CHECK("scan_kernel");
    return MOE_OK;
}

}  // namespace

extern "C" int moe_traffic(moe_ctx* ctx, const int32_t* topk_idx, const int32_t* expert_to_gpu, int32_t* expert_count,
                           int32_t* dest_count, int32_t* n_dropped, void* stream) {
    if (!ctx || !topk_idx || !expert_to_gpu || !expert_count || !dest_count || !n_dropped)
        return moe_set_error(MOE_EINVAL, "moe_traffic: NULL argument");
    SegMap map;
    int rc = build_segmap(ctx->s, expert_to_gpu, nullptr, &map);
    if (rc != MOE_OK) return rc;
    return launch_count_scan(ctx, topk_idx, map, expert_count, dest_count, n_dropped, nullptr, nullptr,
                             reinterpret_cast<hipStream_t>(stream));
}

extern "C" int moe_dispatch(moe_ctx* ctx, const void* x, const int32_t* topk_idx, const int32_t* expert_to_gpu,
                            const int32_t* dest_order, void* send_buf, int32_t* slot_to_row, int32_t* row_to_slot,
                            int32_t* seg_offset, int32_t* seg_expert, void* stream) {
    if (!ctx || !x || !topk_idx || !expert_to_gpu || !dest_order || !send_buf || !slot_to_row || !row_to_slot ||
        !seg_offset || !seg_expert)
        return moe_set_error(MOE_EINVAL, "moe_dispatch: NULL argument");
    if (!aligned16(x) || !aligned16(send_buf)) return moe_set_error(MOE_EALIGN, "moe_dispatch: x and send_buf must be 16-byte aligned");
    const moe_shape& s = ctx->s;
    SegMap map;
    int rc = build_segmap(s, expert_to_gpu, dest_order, &map);
    if (rc != MOE_OK) return rc;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    rc = launch_count_scan(ctx, topk_idx, map, nullptr, nullptr, nullptr, seg_offset, seg_expert, st);
    if (rc != MOE_OK) return rc;
    const size_t lds = (size_t)kChunks * s.E * sizeof(int);
    hipLaunchKernelGGL(rank_kernel, dim3(ctx->n_blocks), dim3(256), lds, st, topk_idx, ctx->n_slots, s.E, s.capacity,
                       ctx->block_hist, ctx->seg_start, slot_to_row, row_to_slot);
    MOE_LAUNCH_CHECK("rank_kernel");
    const int row16 = (int)((int64_t)s.H * elem_size(s.dtype) / 16);
    const dim3 grid((s.T + 3) / 4);
    const u32x4* xs = reinterpret_cast<const u32x4*>(x);
    u32x4* sb = reinterpret_cast<u32x4*>(send_buf);
    if (s.k == 1) hipLaunchKernelGGL(copy_kernel<1>, grid, dim3(256), 0, st, xs, slot_to_row, s.T, s.k, row16, sb);
    else if (s.k == 2) hipLaunchKernelGGL(copy_kernel<2>, grid, dim3(256), 0, st, xs, slot_to_row, s.T, s.k, row16, sb);
    else hipLaunchKernelGGL(copy_kernel<0>, grid, dim3(256), 0, st, xs, slot_to_row, s.T, s.k, row16, sb);
    MOE_LAUNCH_CHECK("copy_kernel");
    return MOE_OK;
}
