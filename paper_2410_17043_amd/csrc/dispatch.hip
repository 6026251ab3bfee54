// Traffic row (Sec. 4: d_gj) and the buffer layer that fills the send buffer in
// the planned transmission order (Sec. 3, "Communication scheduling").
//
// Both rest on one stable counting sort of the T*k slots by expert, done without
// atomics so the permutation is the same on every run.
//
// Rank pass (moe_traffic; moe_dispatch runs it too unless the caller has switched rank reuse on and the
// traffic call on the same indices came directly before):
//   every slot gets its rank among the slots of its expert, in slot order, plus the
//   per-expert totals.  Up to 16384 slots this is ONE block of 16 waves (a launch costs
//   more than the whole count at that size); beyond, three kernels:
//     count_kernel   per block of 1024 consecutive slots: slots per expert (wave ballots)
//     scan_kernel    one block: exclusive prefix over blocks per expert
//     rank_kernel    the same ballots again: block prefix + rank inside the block
//   The capacity rule, the traffic row and the drop count follow from the totals.
//
// Scatter (moe_dispatch): one kernel.  Every wave first turns the per-expert totals into segment
// starts for the requested destination order (a prefix sum over the send-order positions), computes the
// send rows of its tokens' slots from the ranks, writes slot_to_row / row_to_slot, reads its 8 KB of
// token rows once (one long row or a piece of it, or several short rows) and writes them to the rows of
// the kept slots (16-byte lanes, 1 KB per wave access, all 8 loads in flight before the first store,
// cacheable loads - the gate has just read x - and streaming stores).
#include "common.h"
#include <algorithm>
#include <mutex>
#include <new>
#include <vector>

namespace {

struct SegMap {                       // built on the host from expert_to_gpu and dest_order
    int16_t seg_expert[MOE_MAX_E];    // expert at each position of the send order
    uint8_t expert_gpu[MOE_MAX_E];    // destination GPU of each expert
};

constexpr int kChunks = MOE_SLOTS_PER_BLOCK / 64;   // 16 chunks of 64 slots per block, in slot order

// Lanes of the wave whose expert equals this lane's (0 <= e < 256; garbage for e < 0): the lanes that agree
// on every bit of e.
__device__ __forceinline__ unsigned long long same_expert_lanes(int e) {
    unsigned long long peers = __ballot(e >= 0);
#pragma unroll
    for (int b = 0; b < 8; ++b) {                     // MOE_MAX_E = 256 experts: eight bits
        const unsigned long long mb = __ballot((e >> b) & 1);
        peers &= ((e >> b) & 1) ? mb : ~mb;
    }
    return peers;
}

// cnt[chunk][e] for this block's 16 chunks; lane_rank[r] = rank of this lane's slot inside its
// chunk among the lanes with the same expert.
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
    if (E <= 16) {
        for (int e = 0; e < E; ++e) {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const unsigned long long m = __ballot(my_e[r] == e);
                if (WANT_RANK && my_e[r] == e) lane_rank[r] = __popcll(m & lt);
                if (lane == 0) cnt[(wave * 4 + r) * E + e] = __popcll(m);
            }
        }
        return;
    }
    // many experts: nine ballots per round instead of one per expert; the first lane of every group of equal
    // experts writes the group's size, so the table starts from zero
    for (int i = threadIdx.x; i < kChunks * E; i += 256) cnt[i] = 0;
    __syncthreads();
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int e = (my_e[r] >= 0 && my_e[r] < E) ? my_e[r] : -1;
        const unsigned long long peers = same_expert_lanes(e);
        const int rk = __popcll(peers & lt);
        if (WANT_RANK) lane_rank[r] = rk;
        if (e >= 0 && rk == 0) cnt[(wave * 4 + r) * E + e] = __popcll(peers);
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

// Traffic row, drop count and per-expert kept counts from the raw totals.  Thread e < E adds its expert's kept
// count to its destination and its dropped slots to the drop count with LDS atomics (integer sums: the result
// does not depend on their order); a loop over the experts in one thread per destination cost 6 us at 64 experts.
// Called by all threads of a block of at least max(E, G + 1) threads.
__device__ __forceinline__ void traffic_outputs(const int* raw, int* kept, int E, int G, int capacity, const SegMap& map,
                                                int32_t* __restrict__ expert_count, int32_t* __restrict__ dest_count,
                                                int32_t* __restrict__ n_dropped) {
    __shared__ int dest_acc[MOE_MAX_G + 1];                 // [G]: dropped slots
    const int e = threadIdx.x;
    if (e <= G) dest_acc[e] = 0;
    if (e < E) {
        kept[e] = (capacity > 0 && raw[e] > capacity) ? capacity : raw[e];
        if (expert_count) expert_count[e] = kept[e];
    }
    __syncthreads();
    if (e < E) {
        atomicAdd(&dest_acc[map.expert_gpu[e]], kept[e]);
        if (raw[e] > kept[e]) atomicAdd(&dest_acc[G], raw[e] - kept[e]);
    }
    __syncthreads();
    if (dest_count && e < G) dest_count[e] = dest_acc[e];
    if (n_dropped && e == 0) *n_dropped = dest_acc[G];
}

// One block of 256 threads.  Thread e walks the blocks of expert e.
__global__ __launch_bounds__(256) void scan_kernel(int32_t* __restrict__ block_hist, int n_blocks, int E, int G,
                                                   int capacity, SegMap map, int32_t* __restrict__ raw_count,
                                                   int32_t* __restrict__ expert_count, int32_t* __restrict__ dest_count,
                                                   int32_t* __restrict__ n_dropped) {
    __shared__ int kept[MOE_MAX_E];
    __shared__ int raw[MOE_MAX_E];
    const int e = threadIdx.x;
    if (e < E) {
        int run = 0;
        for (int b0 = 0; b0 < n_blocks; b0 += 32) {           // 32 loads in flight per round trip to memory
            int c[32];
#pragma unroll
            for (int u = 0; u < 32; ++u) c[u] = (b0 + u < n_blocks) ? block_hist[(size_t)(b0 + u) * E + e] : 0;
#pragma unroll
            for (int u = 0; u < 32; ++u) {
                if (b0 + u < n_blocks) block_hist[(size_t)(b0 + u) * E + e] = run;
                run += c[u];
            }
        }
        raw[e] = run;
        raw_count[e] = run;
    }
    __syncthreads();
    traffic_outputs(raw, kept, E, G, capacity, map, expert_count, dest_count, n_dropped);
}

__global__ __launch_bounds__(256) void rank_kernel(const int32_t* __restrict__ idx, int n_slots, int E,
                                                   const int32_t* __restrict__ block_base,
                                                   int32_t* __restrict__ slot_rank) {
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
            slot_rank[s] = (e >= 0 && e < E) ? cnt[(wave * 4 + r) * E + e] + lane_rank[r] : -1;
        }
    }
}

constexpr int kSmallMaxSlots = 16384;
constexpr int kSmallRounds = kSmallMaxSlots / (16 * 64);     // rounds of 64 slots per wave

// The whole rank pass in one block of 1024 threads.  Wave w owns the slots [w*spw, (w+1)*spw),
// round by round.  Few experts: one ballot per (expert, round), the running count is wave-uniform.
// Many experts: ballots over the bits of the expert id give every lane the lanes of its round with
// the same expert; the wave's running per-expert counts sit in LDS.
__global__ __launch_bounds__(1024) void small_rank_kernel(const int32_t* __restrict__ idx, int n_slots, int E, int G,
                                                          int capacity, SegMap map, int32_t* __restrict__ raw_count,
                                                          int32_t* __restrict__ slot_rank,
                                                          int32_t* __restrict__ expert_count,
                                                          int32_t* __restrict__ dest_count,
                                                          int32_t* __restrict__ n_dropped) {
    __shared__ int wave_cnt[16][MOE_MAX_E];  // per wave: slots per expert, later the wave's base rank
    __shared__ int kept[MOE_MAX_E], raw[MOE_MAX_E];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int rounds = (n_slots + 1023) / 1024;            // per wave
    const int base = wave * rounds * 64;
    const unsigned long long lt = (1ull << lane) - 1ull;
    int my_e[kSmallRounds], my_rank[kSmallRounds];
#pragma unroll
    for (int r = 0; r < kSmallRounds; ++r) {               // all index loads first
        const int s = base + r * 64 + lane;
        int e = (r < rounds && s < n_slots) ? idx[s] : -1;
        my_e[r] = (e < E) ? e : -1;                         // out of range: no rank
        my_rank[r] = -1;
    }
    int few_cnt = 0;                                       // few experts: lane e ends up with the wave's count of expert e
    if (E <= 16) {
        // few experts: one ballot per (expert, round); the running count is wave-uniform
        for (int e = 0; e < E; ++e) {
            int cnt = 0;
#pragma unroll
            for (int r = 0; r < kSmallRounds; ++r) {
                if (r < rounds) {
                    const unsigned long long m = __ballot(my_e[r] == e);
                    if (my_e[r] == e) my_rank[r] = cnt + __popcll(m & lt);
                    cnt += __popcll(m);
                }
            }
            if (lane == e) few_cnt = cnt;
        }
    } else {
        // many experts: nine ballots per round give every lane the lanes with the same expert; the wave's
        // running counts sit in its row of wave_cnt (only this wave touches it until the barrier below)
        for (int i = lane; i < E; i += 64) wave_cnt[wave][i] = 0;
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
        for (int r = 0; r < kSmallRounds; ++r) {
            if (r < rounds) {
                const int e = my_e[r];
                const unsigned long long peers = same_expert_lanes(e);
                const int rk = __popcll(peers & lt);
                if (e >= 0) {
                    const int before = wave_cnt[wave][e];
                    my_rank[r] = before + rk;
                    if (rk == 0) wave_cnt[wave][e] = before + __popcll(peers);
                }
                // the next round's lanes read counts that other lanes of this wave wrote in this one
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            }
        }
    }
    if (E <= 16) {
        if (lane < E) wave_cnt[wave][lane] = few_cnt;
    }
    __syncthreads();
    if (threadIdx.x < E) {                                 // exclusive scan over the 16 waves
        const int e = threadIdx.x;
        int acc = 0;
#pragma unroll
        for (int w = 0; w < 16; ++w) {
            const int c = wave_cnt[w][e];
            wave_cnt[w][e] = acc;
            acc += c;
        }
        raw[e] = acc;
        raw_count[e] = acc;
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < kSmallRounds; ++r) {
        const int s = base + r * 64 + lane;
        if (r < rounds && s < n_slots) slot_rank[s] = (my_e[r] >= 0) ? wave_cnt[wave][my_e[r]] + my_rank[r] : -1;
    }
    traffic_outputs(raw, kept, E, G, capacity, map, expert_count, dest_count, n_dropped);
}

// Row copying shared by the two scatter kernels.  A wave owns kRowLoads 16-byte loads per lane (8 KB) of input:
// one piece of one long row (rows beyond 8 KB are cut into pieces, grid.y), one whole row, or `tpw` short rows
// (a row of 64 << lsh units with tpw << lsh <= kRowLoads), so that the work that does not depend on the row
// length (segment starts, index loads) is spread over more copying.  The loads and the stores are straight-line
// code (no loop, no divergent branch around a load): every load of the wave is in flight before the first store,
// and the stores follow each other without waiting.  row16 = 16-byte units per row.
constexpr int kRowLoads = 8;
struct RowGeom {
    int row16;     // 16-byte units per row
    int tpw;       // tokens per wave
    int lsh;       // tpw > 1: a row is 64 << lsh units
    int pieces;    // tpw == 1: 8 KB pieces per row (grid.y)
};
RowGeom row_geometry(int row16, int k) {
    RowGeom g{row16, 1, 0, (row16 + 64 * kRowLoads - 1) / (64 * kRowLoads)};
    // Rows of 1, 2 or 4 KB: up to 8, 4 or 2 tokens per wave, as long as a wave writes at most 16 KB (with more
    // stores behind one wave's loads the fine-grained workload, 4 KB rows to 6 slots, lost a sixth of its rate).
    for (int l = 0; l < 3; ++l)
        if (row16 == (64 << l)) {
            g.lsh = l;
            for (g.tpw = kRowLoads >> l; g.tpw > 1 && g.tpw * k * (1 << l) > 16; g.tpw >>= 1) {}
        }
    return g;
}
// token (relative to the wave's first) and first unit inside the row of the wave's load u: wave-uniform values
__device__ __forceinline__ void load_place(const RowGeom& g, int u, int* q, int* c0) {
    if (g.tpw > 1) {
        *q = u >> g.lsh;
        *c0 = (u & ((1 << g.lsh) - 1)) << 6;
    } else {
        *q = 0;
        *c0 = ((int)blockIdx.y * kRowLoads + u) * 64;
    }
}
// Every load is issued whatever the shape: one that has no token or no part of the row left (the tail of T, a row
// that is not a whole number of 1 KB wave-loads, fewer rows than the wave could take) reads the nearest valid
// unit again, which costs a cache hit and keeps the code free of branches (and of the copies of all 32 row
// registers that the compiler makes at every conditional load).
__device__ __forceinline__ void load_rows(const u32x4* __restrict__ x, const RowGeom& g, int t0, int T, int lane,
                                          u32x4 (&v)[kRowLoads]) {
#pragma unroll
    for (int u = 0; u < kRowLoads; ++u) {
        int q, c0;
        load_place(g, u, &q, &c0);
        const int t = min(t0 + min(q, g.tpw - 1), T - 1);
        v[u] = x[(size_t)t * g.row16 + min(c0 + lane, g.row16 - 1)];
    }
}
// lane q * k + j holds the send row of slot j of the wave's token q in my_row (-1: dropped, or no such token)
template <int K>
__device__ __forceinline__ void store_rows(const u32x4 (&v)[kRowLoads], const RowGeom& g, int my_row, int k, int lane,
                                           u32x4* __restrict__ send_buf) {
    constexpr int KM = (K > 0) ? K : MOE_MAX_K;
#pragma unroll
    for (int u = 0; u < kRowLoads; ++u) {
        int q, c0;
        load_place(g, u, &q, &c0);
        if (q >= g.tpw || c0 >= g.row16) continue;                // wave-uniform
#pragma unroll
        for (int j = 0; j < KM; ++j) {
            if (j >= k) continue;
            const int row = __builtin_amdgcn_readlane(my_row, q * k + j);
            if (row >= 0 && c0 + lane < g.row16) __builtin_nontemporal_store(v[u], send_buf + (size_t)row * g.row16 + c0 + lane);
        }
    }
}

template <int K>
__global__ __launch_bounds__(256) void scatter_kernel(const u32x4* __restrict__ x, const int32_t* __restrict__ idx,
                                                      const int32_t* __restrict__ slot_rank,
                                                      const int32_t* __restrict__ raw_count, int T, int k_rt, int E,
                                                      int capacity, SegMap map, RowGeom g,
                                                      u32x4* __restrict__ send_buf, int32_t* __restrict__ slot_to_row,
                                                      int32_t* __restrict__ row_to_slot, int32_t* __restrict__ seg_offset,
                                                      int32_t* __restrict__ seg_expert) {
    __shared__ int seg_first[MOE_MAX_E];   // E > 64: first send row of each expert
    __shared__ int cnt_of[MOE_MAX_E];      // E > 64: total of each expert
    __shared__ int wave_first[4][64];      // E <= 64: first send row of each expert, one copy per wave
    __shared__ int wave_sum[4];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int t0 = __builtin_amdgcn_readfirstlane((blockIdx.x * 4 + wave) * g.tpw);   // first token of this wave
    const int k = (K > 0) ? K : k_rt;
    const int n_slots = T * k;
    const int s_mine = t0 * k + lane;                         // lane q * k + j looks after slot j of token t0 + q
    const bool has_slot = lane < g.tpw * k && s_mine < n_slots;
    const bool first_piece = blockIdx.y == 0;                 // the pieces of a long row work out the same send rows
    // Memory returns a wave's loads in the order they were issued, so the small loads that the send rows
    // depend on go out first (all independent of each other: one round trip), then the 8 KB of token rows;
    // the send rows are worked out while the row data is still in flight.
    int slot_e = -1, slot_rank_v = -1;
    if (has_slot) {
        slot_e = idx[s_mine];
        slot_rank_v = slot_rank[s_mine];
    }
    const int p_blk = (E <= 64) ? lane : threadIdx.x;       // send-order position this thread looks after
    const int ex = (p_blk < E) ? map.seg_expert[p_blk] : 0;
    int cnt_by_id = (p_blk < E) ? raw_count[p_blk] : 0;     // total of expert p_blk; the one of `ex` comes by shuffle / LDS
    __builtin_amdgcn_sched_barrier(0);
    // plain (cacheable) loads: the gate has just read x, so the rows come from the memory-side cache; the
    // send rows are written with streaming stores
    u32x4 v[kRowLoads];
    load_rows(x, g, t0, T, lane, v);
    __builtin_amdgcn_sched_barrier(0);
    // Segment starts in send order.  Up to 64 experts every wave does the prefix sum for itself (lane p =
    // position p, no block barrier); beyond, the block shares one through LDS.
    if (E <= 64) {
        int cnt = __shfl(cnt_by_id, ex, 64);
        if (lane >= E) cnt = 0;
        if (capacity > 0 && cnt > capacity) cnt = capacity;
        int incl = cnt;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int up = __shfl_up(incl, o, 64);
            if (lane >= o) incl += up;
        }
        const int excl = incl - cnt;
        if (lane < E) wave_first[wave][ex] = excl;
        if (blockIdx.x == 0 && first_piece && wave == 0 && lane < E) {
            seg_offset[lane] = excl;
            seg_expert[lane] = ex;
            if (lane == E - 1) seg_offset[E] = incl;
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");     // a wave reads back only what it wrote itself
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    } else {
        if (p_blk < E) cnt_of[p_blk] = cnt_by_id;
        __syncthreads();
        int cnt = (p_blk < E) ? cnt_of[ex] : 0;
        if (capacity > 0 && cnt > capacity) cnt = capacity;
        int incl = cnt;                                     // inclusive scan inside the wave
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int up = __shfl_up(incl, o, 64);
            if (lane >= o) incl += up;
        }
        if (lane == 63) wave_sum[wave] = incl;
        __syncthreads();
        int before = 0;
#pragma unroll
        for (int w = 0; w < 4; ++w)
            if (w < wave) before += wave_sum[w];
        const int excl = before + incl - cnt;
        if (p_blk < E) {
            seg_first[ex] = excl;
            if (blockIdx.x == 0 && first_piece) {
                seg_offset[p_blk] = excl;
                seg_expert[p_blk] = ex;
                if (p_blk == E - 1) seg_offset[E] = excl + cnt;
            }
        }
        __syncthreads();
    }
    if (t0 >= T) return;
    // send rows of this wave's slots, one per lane
    int my_row = -1;
    if (has_slot) {
        const int e = slot_e, rank = slot_rank_v;
        if (e >= 0 && e < E && rank >= 0 && (capacity <= 0 || rank < capacity)) {
            my_row = ((E <= 64) ? wave_first[wave][e] : seg_first[e]) + rank;
            if (first_piece) row_to_slot[my_row] = s_mine;
        }
        if (first_piece) slot_to_row[s_mine] = my_row;
    }
    store_rows<K>(v, g, my_row, k, lane, send_buf);
}

// ------------------------------------------------------------------------------ chunked layout
// Send buffer for a preemptive schedule (Appendix A): the slots of a destination form one sequence
// (expert by expert, then slot order) that is cut into the plan's chunks; the buffer is the chunks
// in plan order, then one left-over chunk per destination.  Everything that depends only on the
// plan is tabulated on the host when the plan is created; a dispatch computes, from the actual
// per-expert counts, where each chunk starts (one block), and the scatter kernel finds the chunk
// of a slot by binary search among its destination's chunks.
constexpr int kMaxPlanChunks = 4096;
constexpr int kMaxChunks = kMaxPlanChunks + MOE_MAX_G;      // plus one left-over chunk per destination
constexpr int kLayoutThreads = 1024;
constexpr int kChunksPerThread = (kMaxChunks + kLayoutThreads - 1) / kLayoutThreads;

struct ChunkTables {                  // device pointers
    int nc;                           // chunks in all (plan + G left-over)
    const int32_t* c_dest;            // [nc] destination, -1: no GPU (always empty)
    const int32_t* c_cumlo;           // [nc] planned slots of the destination before this chunk
    const int32_t* c_cumhi;           // [nc] ... after it; INT_MAX for a left-over chunk
    const int32_t* p_chunk;           // [np] chunk ids grouped by destination, in plan order inside a group
    const int32_t* p_cumhi;           // [np] c_cumhi of p_chunk
    const int32_t* p_begin;           // [G+1] group of destination d is [p_begin[d], p_begin[d+1])
    const int32_t* d_exp;             // [E] the experts of every destination, ascending: d_exp[d_beg[d] .. d_beg[d+1])
    const int32_t* d_beg;             // [G+1]
    int32_t* c_row0;                  // [nc+1] written per dispatch: first send row of each chunk
    int32_t* expert_first;            // [E] written per dispatch: position of the expert's first slot in its destination's sequence
};

// Exclusive prefix sum over one value per thread, 1024 threads; returns the total to every thread.
__device__ __forceinline__ int block_exclusive_scan(int v, int* excl_out, int* wave_tot /* LDS [16] */) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int incl = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int up = __shfl_up(incl, o, 64);
        if (lane >= o) incl += up;
    }
    __syncthreads();                                          // wave_tot may still be read from an earlier scan
    if (lane == 63) wave_tot[wave] = incl;
    __syncthreads();
    int before = 0, total = 0;
#pragma unroll
    for (int w = 0; w < kLayoutThreads / 64; ++w) {
        const int t = wave_tot[w];
        if (w < wave) before += t;
        total += t;
    }
    *excl_out = before + incl - v;
    return total;
}

__global__ __launch_bounds__(kLayoutThreads) void chunk_layout_kernel(ChunkTables tb, const int32_t* __restrict__ raw_count,
                                                                      int E, int G, int capacity, SegMap map,
                                                                      int32_t* __restrict__ chunk_offset,
                                                                      int32_t* __restrict__ piece_offset,
                                                                      int32_t* __restrict__ piece_expert,
                                                                      int32_t* __restrict__ n_pieces) {
    __shared__ int kept[MOE_MAX_E], first[MOE_MAX_E], dest_cnt[MOE_MAX_G], wave_tot[kLayoutThreads / 64];
    __shared__ int d_exp[MOE_MAX_E], d_beg[MOE_MAX_G + 1];    // the plan's tables (which expert lives where), in LDS
    const int tid = threadIdx.x;
    if (tid < E) {
        const int c = raw_count[tid];
        kept[tid] = (capacity > 0 && c > capacity) ? capacity : c;
        d_exp[tid] = tb.d_exp[tid];
    }
    if (tid <= G) d_beg[tid] = tb.d_beg[tid];
    __syncthreads();
    if (tid < G) {                                            // thread d walks the experts of destination d in id order
        int run = 0;
        for (int i = d_beg[tid]; i < d_beg[tid + 1]; ++i) {
            const int e = d_exp[i];
            first[e] = run;
            run += kept[e];
        }
        dest_cnt[tid] = run;                                  // kept slots of the destination
    }
    __syncthreads();
    if (tid < E) tb.expert_first[tid] = first[tid];
    // thread t owns chunks [t * CPT, (t + 1) * CPT): sizes, then the block-wide prefix
    const int c0 = tid * kChunksPerThread;
    int size[kChunksPerThread], pieces[kChunksPerThread], sum = 0, psum = 0;
#pragma unroll
    for (int u = 0; u < kChunksPerThread; ++u) {
        const int c = c0 + u;
        size[u] = 0; pieces[u] = 0;
        if (c < tb.nc) {
            const int d = tb.c_dest[c];
            if (d >= 0) {
                const int lo = min(tb.c_cumlo[c], dest_cnt[d]), hi = min(tb.c_cumhi[c], dest_cnt[d]);
                size[u] = hi - lo;
                if (hi > lo)
                    for (int i = d_beg[d]; i < d_beg[d + 1]; ++i) {   // experts of d whose slots meet [lo, hi)
                        const int e = d_exp[i];
                        if (kept[e] > 0 && first[e] < hi && first[e] + kept[e] > lo) ++pieces[u];
                    }
            }
        }
        sum += size[u];
        psum += pieces[u];
    }
    int row0, piece0;
    const int total = block_exclusive_scan(sum, &row0, wave_tot);
    const int total_pieces = block_exclusive_scan(psum, &piece0, wave_tot);
#pragma unroll
    for (int u = 0; u < kChunksPerThread; ++u) {
        const int c = c0 + u;
        if (c < tb.nc) {
            tb.c_row0[c] = row0;
            chunk_offset[c] = row0;
            if (size[u] > 0) {
                const int d = tb.c_dest[c];
                const int lo = min(tb.c_cumlo[c], dest_cnt[d]), hi = lo + size[u];
                for (int i = d_beg[d]; i < d_beg[d + 1]; ++i) {
                    const int e = d_exp[i];
                    if (kept[e] > 0 && first[e] < hi && first[e] + kept[e] > lo) {
                        piece_offset[piece0] = row0 + max(first[e], lo) - lo;
                        piece_expert[piece0] = e;
                        ++piece0;
                    }
                }
            }
            row0 += size[u];
        }
    }
    if (tid == 0) {
        tb.c_row0[tb.nc] = total;
        chunk_offset[tb.nc] = total;
        piece_offset[total_pieces] = total;
        *n_pieces = total_pieces;
    }
}

// Waves take tokens as in scatter_kernel; the send row of a kept slot comes from the chunk tables.
template <int K>
__global__ __launch_bounds__(256) void scatter_chunks_kernel(const u32x4* __restrict__ x, const int32_t* __restrict__ idx,
                                                             const int32_t* __restrict__ slot_rank, int T, int k_rt, int E,
                                                             int capacity, SegMap map, ChunkTables tb, RowGeom g,
                                                             u32x4* __restrict__ send_buf, int32_t* __restrict__ slot_to_row,
                                                             int32_t* __restrict__ row_to_slot) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int t0 = __builtin_amdgcn_readfirstlane((blockIdx.x * 4 + wave) * g.tpw);
    const int k = (K > 0) ? K : k_rt;
    if (t0 >= T) return;
    const int s_mine = t0 * k + lane;
    const bool has_slot = lane < g.tpw * k && s_mine < T * k;
    const bool first_piece = blockIdx.y == 0;
    int e = -1, rank = -1;
    if (has_slot) {
        e = idx[s_mine];
        rank = slot_rank[s_mine];
    }
    __builtin_amdgcn_sched_barrier(0);
    u32x4 v[kRowLoads];
    load_rows(x, g, t0, T, lane, v);
    __builtin_amdgcn_sched_barrier(0);
    int my_row = -1;
    if (has_slot) {
        if (e >= 0 && e < E && rank >= 0 && (capacity <= 0 || rank < capacity)) {
            const int d = map.expert_gpu[e];
            const int q = tb.expert_first[e] + rank;          // position in the destination's sequence
            int lo = tb.p_begin[d], hi = tb.p_begin[d + 1] - 1;   // the last one is the left-over chunk: q < INT_MAX
            while (lo < hi) {                                 // first chunk of d with q < cumhi
                const int mid = (lo + hi) >> 1;
                if (q < tb.p_cumhi[mid]) hi = mid; else lo = mid + 1;
            }
            const int c = tb.p_chunk[lo];
            my_row = tb.c_row0[c] + q - tb.c_cumlo[c];
            if (first_piece) row_to_slot[my_row] = s_mine;
        }
        if (first_piece) slot_to_row[s_mine] = my_row;
    }
    store_rows<K>(v, g, my_row, k, lane, send_buf);
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

// Scratch of the counting sort: owned by a context, or the static array of moe_dispatch_noalloc.
struct RankScratch {
    int32_t* block_hist;   // [n_blocks][E]
    int32_t* raw_count;    // [E]
    int32_t* slot_rank;    // [n_slots]
};

// Rank pass; the three count outputs may be NULL.
int launch_rank_pass(const moe_shape& s, const RankScratch& sc, const int32_t* idx, const SegMap& map, int32_t* expert_count,
                     int32_t* dest_count, int32_t* n_dropped, hipStream_t st) {
    const int n_slots = s.T * s.k;
    const int n_blocks = (n_slots + MOE_SLOTS_PER_BLOCK - 1) / MOE_SLOTS_PER_BLOCK;
    if (n_slots <= kSmallMaxSlots) {
        hipLaunchKernelGGL(small_rank_kernel, dim3(1), dim3(1024), 0, st, idx, n_slots, s.E, s.G, s.capacity, map,
                           sc.raw_count, sc.slot_rank, expert_count, dest_count, n_dropped);
        MOE_LAUNCH_CHECK("small_rank_kernel");
    } else {
        const size_t lds = (size_t)kChunks * s.E * sizeof(int);
        hipLaunchKernelGGL(count_kernel, dim3(n_blocks), dim3(256), lds, st, idx, n_slots, s.E, sc.block_hist);
        MOE_LAUNCH_CHECK("count_kernel");
        hipLaunchKernelGGL(scan_kernel, dim3(1), dim3(256), 0, st, sc.block_hist, n_blocks, s.E, s.G, s.capacity, map,
                           sc.raw_count, expert_count, dest_count, n_dropped);
        MOE_LAUNCH_CHECK("scan_kernel");
        hipLaunchKernelGGL(rank_kernel, dim3(n_blocks), dim3(256), lds, st, idx, n_slots, s.E, sc.block_hist,
                           sc.slot_rank);
        MOE_LAUNCH_CHECK("rank_kernel");
    }
    return MOE_OK;
}

RankScratch scratch_of(const moe_ctx* c) { return RankScratch{c->block_hist, c->raw_count, c->slot_rank}; }

// Are the ranks that moe_traffic left in the context the ones this dispatch needs?  Only when the caller
// has switched reuse on, the traffic call was the last call on the context, and it was given the same index
// array.  The answer is consumed: a second dispatch computes its own ranks.
bool take_cached_ranks(moe_ctx* c, const int32_t* idx) {
    const bool ok = c->reuse_ranks && c->rank_src != nullptr && c->rank_src == idx;
    c->rank_src = nullptr;
    return ok;
}

int launch_scatter(const moe_shape& s, const RankScratch& sc, const SegMap& map, const void* x, const int32_t* topk_idx,
                   void* send_buf, int32_t* slot_to_row, int32_t* row_to_slot, int32_t* seg_offset, int32_t* seg_expert,
                   hipStream_t st) {
    const int row16 = (int)((int64_t)s.H * elem_size(s.dtype) / 16);
    const RowGeom g = row_geometry(row16, s.k);
    const dim3 grid((s.T + 4 * g.tpw - 1) / (4 * g.tpw), g.pieces);
    const u32x4* xs = reinterpret_cast<const u32x4*>(x);
    u32x4* sb = reinterpret_cast<u32x4*>(send_buf);
#define MOE_SCATTER(KK)                                                                                          \
    hipLaunchKernelGGL(scatter_kernel<KK>, grid, dim3(256), 0, st, xs, topk_idx, sc.slot_rank, sc.raw_count, s.T, \
                       s.k, s.E, s.capacity, map, g, sb, slot_to_row, row_to_slot, seg_offset, seg_expert)
    if (s.k == 1) MOE_SCATTER(1);
    else if (s.k == 2) MOE_SCATTER(2);
    else MOE_SCATTER(0);
#undef MOE_SCATTER
    MOE_LAUNCH_CHECK("scatter_kernel");
    return MOE_OK;
}

}  // namespace

extern "C" int moe_selfcheck_row_geometry(int32_t row16, int32_t k, int32_t* out3) {
    if (row16 < 1 || k < 1 || k > MOE_MAX_K || !out3) return moe_set_error(MOE_EINVAL, "moe_selfcheck_row_geometry: bad argument");
    const RowGeom g = row_geometry(row16, k);
    out3[0] = g.tpw; out3[1] = g.lsh; out3[2] = g.pieces;
    // a wave's kRowLoads loads must hold its rows; lane q * k + j must exist; the pieces must cover the row
    if (g.tpw < 1 || g.pieces < 1 || g.tpw * k > 64) return moe_set_error(MOE_EINTERNAL, "row geometry: %d tokens x %d slots per wave", g.tpw, k);
    if (g.tpw > 1 && (row16 != (64 << g.lsh) || (g.tpw << g.lsh) > kRowLoads || g.pieces != 1))
        return moe_set_error(MOE_EINTERNAL, "row geometry: %d rows of %d units do not fit a wave", g.tpw, row16);
    if ((int64_t)g.pieces * 64 * kRowLoads < row16 || (int64_t)(g.pieces - 1) * 64 * kRowLoads >= row16)
        return moe_set_error(MOE_EINTERNAL, "row geometry: %d pieces for %d units", g.pieces, row16);
    return MOE_OK;
}

extern "C" int moe_traffic(moe_ctx* ctx, const int32_t* topk_idx, const int32_t* expert_to_gpu, int32_t* expert_count,
                           int32_t* dest_count, int32_t* n_dropped, void* stream) {
    if (!ctx || !topk_idx || !expert_to_gpu || !expert_count || !dest_count || !n_dropped)
        return moe_set_error(MOE_EINVAL, "moe_traffic: NULL argument");
    ctx->rank_src = nullptr;
    SegMap map;
    int rc = build_segmap(ctx->s, expert_to_gpu, nullptr, &map);
    if (rc != MOE_OK) return rc;
    rc = launch_rank_pass(ctx->s, scratch_of(ctx), topk_idx, map, expert_count, dest_count, n_dropped,
                          reinterpret_cast<hipStream_t>(stream));
    if (rc == MOE_OK) ctx->rank_src = topk_idx;
    return rc;
}

extern "C" int moe_dispatch(moe_ctx* ctx, const void* x, const int32_t* topk_idx, const int32_t* expert_to_gpu,
                            const int32_t* dest_order, void* send_buf, int32_t* slot_to_row, int32_t* row_to_slot,
                            int32_t* seg_offset, int32_t* seg_expert, void* stream) {
    if (!ctx || !x || !topk_idx || !expert_to_gpu || !dest_order || !send_buf || !slot_to_row || !row_to_slot ||
        !seg_offset || !seg_expert)
        return moe_set_error(MOE_EINVAL, "moe_dispatch: NULL argument");
    const bool cached = take_cached_ranks(ctx, topk_idx);
    if (!aligned16(x) || !aligned16(send_buf)) return moe_set_error(MOE_EALIGN, "moe_dispatch: x and send_buf must be 16-byte aligned");
    const moe_shape& s = ctx->s;
    SegMap map;
    int rc = build_segmap(s, expert_to_gpu, dest_order, &map);
    if (rc != MOE_OK) return rc;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    if (!cached) {
        rc = launch_rank_pass(s, scratch_of(ctx), topk_idx, map, nullptr, nullptr, nullptr, st);
        if (rc != MOE_OK) return rc;
    }
    return launch_scatter(s, scratch_of(ctx), map, x, topk_idx, send_buf, slot_to_row, row_to_slot, seg_offset, seg_expert, st);
}

// ---------------------------------------------------------------------------- no allocation
// moe_dispatch for callers that cannot allocate: the counting-sort scratch that a context would own
// lives in a static device array.  Every GPU holds its own copy at its own address; the host looks the
// address up once per device and passes that pointer to the kernels (the array's name means nothing
// on the host side).
constexpr int kNoAllocMaxSlots = 1 << 20;
constexpr int kNoAllocMaxBlocks = kNoAllocMaxSlots / MOE_SLOTS_PER_BLOCK;
constexpr size_t kNoAllocWords = (size_t)kNoAllocMaxBlocks * MOE_MAX_E + MOE_MAX_E + kNoAllocMaxSlots;   // 5 MiB + 1 KiB
static __device__ __align__(256) int32_t scratch[kNoAllocWords];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
int32_t* g_scratch_ptr[kMaxDevices];        // per device: address of `scratch` there, nullptr until looked up

int scratch_for_current_device(int32_t** out) {
    int dev = -1;
    MOE_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return moe_set_error(MOE_ESHAPE, "moe_dispatch_noalloc: device %d outside [0, %d)", dev, kMaxDevices);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        MOE_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return moe_set_error(MOE_EHIP, "moe_dispatch_noalloc: hipGetSymbolAddress returned no address");
        g_scratch_ptr[dev] = reinterpret_cast<int32_t*>(p);
    }
    *out = g_scratch_ptr[dev];
    return MOE_OK;
}
}  // namespace

extern "C" int moe_dispatch_noalloc(const moe_shape* shape, const void* x, const int32_t* topk_idx,
                                    const int32_t* expert_to_gpu, const int32_t* dest_order, void* send_buf,
                                    int32_t* slot_to_row, int32_t* row_to_slot, int32_t* seg_offset, int32_t* seg_expert,
                                    void* stream) {
    if (!shape || !x || !topk_idx || !expert_to_gpu || !dest_order || !send_buf || !slot_to_row || !row_to_slot ||
        !seg_offset || !seg_expert)
        return moe_set_error(MOE_EINVAL, "moe_dispatch_noalloc: NULL argument");
    int rc = moe_check_shape(shape);
    if (rc != MOE_OK) return rc;
    const moe_shape& s = *shape;
    if ((int64_t)s.T * s.k > kNoAllocMaxSlots)
        return moe_set_error(MOE_ESHAPE, "moe_dispatch_noalloc: T*k = %lld exceeds the static scratch (%d slots); use moe_dispatch",
                             (long long)s.T * s.k, kNoAllocMaxSlots);
    if (!aligned16(x) || !aligned16(send_buf))
        return moe_set_error(MOE_EALIGN, "moe_dispatch_noalloc: x and send_buf must be 16-byte aligned");
    SegMap map;
    rc = build_segmap(s, expert_to_gpu, dest_order, &map);
    if (rc != MOE_OK) return rc;
    int32_t* base = nullptr;
    rc = scratch_for_current_device(&base);
    if (rc != MOE_OK) return rc;
    // same layout as a context's scratch; every word a kernel reads is written earlier in the same call
    // (block histograms for every block, totals for every expert, a rank for every slot), so nothing has
    // to be cleared and what an earlier call left behind is never seen
    const int n_slots = s.T * s.k;
    const int n_blocks = (n_slots + MOE_SLOTS_PER_BLOCK - 1) / MOE_SLOTS_PER_BLOCK;
    RankScratch sc;
    sc.block_hist = base;
    sc.raw_count = base + (size_t)n_blocks * s.E;
    sc.slot_rank = sc.raw_count + s.E;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    rc = launch_rank_pass(s, sc, topk_idx, map, nullptr, nullptr, nullptr, st);
    if (rc != MOE_OK) return rc;
    return launch_scatter(s, sc, map, x, topk_idx, send_buf, slot_to_row, row_to_slot, seg_offset, seg_expert, st);
}

struct moe_chunk_plan {
    SegMap map;
    ChunkTables tb;
    int32_t E, G, n_chunks;
    int32_t* dev;                      // one allocation behind all the tables
};

extern "C" int moe_chunk_plan_create(moe_ctx* ctx, const int32_t* expert_to_gpu, int32_t n_chunks, const int32_t* chunk_dest,
                                     const int32_t* chunk_rows, moe_chunk_plan** out) {
    if (!ctx || !expert_to_gpu || !out || (n_chunks > 0 && (!chunk_dest || !chunk_rows)))
        return moe_set_error(MOE_EINVAL, "moe_chunk_plan_create: NULL argument");
    if (n_chunks < 0 || n_chunks > kMaxPlanChunks)
        return moe_set_error(MOE_ESHAPE, "moe_chunk_plan_create: n_chunks = %d outside [0, %d]", n_chunks, kMaxPlanChunks);
    const moe_shape& s = ctx->s;
    moe_chunk_plan* p = new (std::nothrow) moe_chunk_plan;
    if (!p) return moe_set_error(MOE_ENOMEM, "moe_chunk_plan_create: out of host memory");
    int rc = build_segmap(s, expert_to_gpu, nullptr, &p->map);
    if (rc != MOE_OK) { delete p; return rc; }
    const int G = s.G, nc = n_chunks + G;
    std::vector<int32_t> c_dest(nc), c_cumlo(nc), c_cumhi(nc), p_chunk, p_cumhi, p_begin(G + 1);
    std::vector<int64_t> planned(G, 0);
    for (int c = 0; c < nc; ++c) {
        const bool left_over = c >= n_chunks;
        const int d = left_over ? c - n_chunks : chunk_dest[c];
        if (d < 0 || d >= G) { c_dest[c] = -1; c_cumlo[c] = c_cumhi[c] = 0; continue; }
        const int64_t rows = left_over ? (int64_t)INT32_MAX : (chunk_rows[c] > 0 ? chunk_rows[c] : 0);
        c_dest[c] = d;
        c_cumlo[c] = (int32_t)std::min<int64_t>(planned[d], INT32_MAX);
        planned[d] = std::min<int64_t>(planned[d] + rows, INT32_MAX);
        c_cumhi[c] = (int32_t)planned[d];
    }
    for (int d = 0; d < G; ++d) {
        p_begin[d] = (int32_t)p_chunk.size();
        for (int c = 0; c < nc; ++c)
            if (c_dest[c] == d) { p_chunk.push_back(c); p_cumhi.push_back(c_cumhi[c]); }
    }
    p_begin[G] = (int32_t)p_chunk.size();
    const int np = (int)p_chunk.size();
    std::vector<int32_t> d_exp, d_beg(G + 1);                // which experts live on each destination
    for (int d = 0; d < G; ++d) {
        d_beg[d] = (int32_t)d_exp.size();
        for (int e = 0; e < s.E; ++e)
            if (expert_to_gpu[e] == d) d_exp.push_back(e);
    }
    d_beg[G] = (int32_t)d_exp.size();                         // = E: build_segmap has checked every expert's GPU
    // device layout: c_dest | c_cumlo | c_cumhi | p_chunk | p_cumhi | p_begin | d_exp | d_beg | c_row0 | expert_first
    const size_t n_static = (size_t)3 * nc + 2 * np + (G + 1) + s.E + (G + 1);
    const size_t n_all = n_static + (nc + 1) + s.E;
    std::vector<int32_t> host(n_static);
    size_t o = 0;
    auto put = [&](const std::vector<int32_t>& v, size_t n) { std::copy(v.begin(), v.begin() + n, host.begin() + o); o += n; };
    put(c_dest, nc); put(c_cumlo, nc); put(c_cumhi, nc); put(p_chunk, np); put(p_cumhi, np); put(p_begin, G + 1);
    put(d_exp, s.E); put(d_beg, G + 1);
    hipError_t e = hipMalloc((void**)&p->dev, n_all * sizeof(int32_t));
    if (e != hipSuccess) {
        delete p;
        return moe_set_error(e == hipErrorOutOfMemory ? MOE_ENOMEM : MOE_EHIP, "hipMalloc(%zu): %s", n_all * sizeof(int32_t), hipGetErrorString(e));
    }
    e = hipMemcpy(p->dev, host.data(), n_static * sizeof(int32_t), hipMemcpyHostToDevice);
    if (e != hipSuccess) {
        (void)hipFree(p->dev);
        delete p;
        return moe_set_error(MOE_EHIP, "hipMemcpy: %s", hipGetErrorString(e));
    }
    int32_t* d = p->dev;
    p->tb.nc = nc;
    p->tb.c_dest = d; d += nc;
    p->tb.c_cumlo = d; d += nc;
    p->tb.c_cumhi = d; d += nc;
    p->tb.p_chunk = d; d += np;
    p->tb.p_cumhi = d; d += np;
    p->tb.p_begin = d; d += G + 1;
    p->tb.d_exp = d; d += s.E;
    p->tb.d_beg = d; d += G + 1;
    p->tb.c_row0 = d; d += nc + 1;
    p->tb.expert_first = d;
    p->E = s.E; p->G = G; p->n_chunks = n_chunks;
    *out = p;
    return MOE_OK;
}

extern "C" int moe_chunk_plan_destroy(moe_chunk_plan* plan) {
    if (!plan) return MOE_OK;
    hipError_t e = hipFree(plan->dev);
    delete plan;
    if (e != hipSuccess) return moe_set_error(MOE_EHIP, "hipFree: %s", hipGetErrorString(e));
    return MOE_OK;
}

extern "C" int moe_dispatch_chunks(moe_ctx* ctx, const moe_chunk_plan* plan, const void* x, const int32_t* topk_idx,
                                   void* send_buf, int32_t* slot_to_row, int32_t* row_to_slot, int32_t* chunk_offset,
                                   int32_t* piece_offset, int32_t* piece_expert, int32_t* n_pieces, void* stream) {
    if (!ctx || !plan || !x || !topk_idx || !send_buf || !slot_to_row || !row_to_slot || !chunk_offset || !piece_offset ||
        !piece_expert || !n_pieces)
        return moe_set_error(MOE_EINVAL, "moe_dispatch_chunks: NULL argument");
    const bool cached = take_cached_ranks(ctx, topk_idx);
    if (!aligned16(x) || !aligned16(send_buf))
        return moe_set_error(MOE_EALIGN, "moe_dispatch_chunks: x and send_buf must be 16-byte aligned");
    const moe_shape& s = ctx->s;
    if (plan->E != s.E || plan->G != s.G) return moe_set_error(MOE_ESHAPE, "moe_dispatch_chunks: plan made for another shape");
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    if (!cached) {
        int rc = launch_rank_pass(s, scratch_of(ctx), topk_idx, plan->map, nullptr, nullptr, nullptr, st);
        if (rc != MOE_OK) return rc;
    }
    hipLaunchKernelGGL(chunk_layout_kernel, dim3(1), dim3(kLayoutThreads), 0, st, plan->tb, ctx->raw_count, s.E, s.G,
                       s.capacity, plan->map, chunk_offset, piece_offset, piece_expert, n_pieces);
    MOE_LAUNCH_CHECK("chunk_layout_kernel");
    const int row16 = (int)((int64_t)s.H * elem_size(s.dtype) / 16);
    const RowGeom g = row_geometry(row16, s.k);
    const dim3 grid((s.T + 4 * g.tpw - 1) / (4 * g.tpw), g.pieces);
    const u32x4* xs = reinterpret_cast<const u32x4*>(x);
    u32x4* sb = reinterpret_cast<u32x4*>(send_buf);
#define MOE_SCATTER(KK)                                                                                              \
    hipLaunchKernelGGL(scatter_chunks_kernel<KK>, grid, dim3(256), 0, st, xs, topk_idx, ctx->slot_rank, s.T, s.k, s.E, \
                       s.capacity, plan->map, plan->tb, g, sb, slot_to_row, row_to_slot)
    if (s.k == 1) MOE_SCATTER(1);
    else if (s.k == 2) MOE_SCATTER(2);
    else MOE_SCATTER(0);
#undef MOE_SCATTER
    MOE_LAUNCH_CHECK("scatter_chunks_kernel");
    return MOE_OK;
}
