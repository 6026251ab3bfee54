// Expert FFN of Sec. 2.1 over the rows a GPU received: a ragged grouped GEMM pair.
//
//   GEMM1  Hmid[R,F] = act(recv . W1^T)            (SwiGLU: silu(recv . W1^T) * (recv . Wu^T))
//   GEMM2  out[R,H]  = Hmid . Wd^T
//
// Both operands of both GEMMs are K-contiguous ([rows,K] activations, [out,in]
// weights), which is exactly the operand layout of the CDNA MFMA instructions.
// Rows are grouped in segments, one local expert per segment; a small device kernel
// turns the segment list into a list of M-tiles (adjacent segments of the same
// expert are merged, tiles never straddle experts), so nothing waits for the host.
//
// bf16 path: 256x256 block tile, 32-wide k-tiles, 4 waves in 2x2, each wave 128x128 = 4x4
// tiles of v_mfma_f32_32x32x16_bf16 with fp32 accumulators (256 accumulator registers per
// lane); operands go global -> LDS directly (no register staging) through a 5-stage ring that
// fills the whole 160 KB LDS, in an XOR-swizzled layout that makes every ds_read_b128 of an
// MFMA operand conflict-free on the 64 LDS banks.  Loads, LDS reads and MFMAs are software
// pipelined by hand (see the kernel).  For SwiGLU the B tile holds 128 gate rows and 128 up
// rows arranged so that a wave owns the gate and the up product of the same 64 columns: the
// activation is applied on registers and the intermediate is written once, in bf16, as whole
// 128-byte lines after a transpose through LDS.  Tiles are numbered so that the blocks that
// share an XCD's L2 form a compact patch and all XCDs sweep the N-tiles in step (see
// tile_of_block); the tiles of a mostly empty last round are cut along K (see plan_tail).
//
// Shares of at most 64 rows (bf16) take a pair of weight-streaming kernels instead (gemm_bf16_skinny_kernel):
// 32- or 64-row tiles, 256-byte bursts per weight row, the LDS ring given to loads in flight.
//
// fp32 path (correctness configuration): plain 64x64x16 LDS-tiled vector-ALU GEMM.
#include "common.h"
#include <algorithm>
#include <cstddef>
#include <vector>

namespace {

constexpr int kMaxSeg = 1024;

struct TileMap {
    int32_t* n_tiles;   // [1]
    int32_t* row0;      // [max_tiles] first row of the tile
    int32_t* nrows;     // [max_tiles] valid rows (1..BM)
    int32_t* expert;    // [max_tiles] local expert
    int32_t* gather;    // [max_tiles] 0: the tile is rows row0 .. row0 + nrows - 1; 1: row r is row0 + rel[tile][r]
    int32_t* rel;       // [max_tiles][kRelPitch] row offsets of the gathered tiles (written for those only)
};
constexpr int kRelPitch = 256;

struct ExpertTable {
    const void* w1[MOE_MAX_LOCAL];
    const void* w_up[MOE_MAX_LOCAL];
    const void* w_down[MOE_MAX_LOCAL];
};

__host__ __device__ inline size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }
inline int max_tiles_for(int R) { return R / 64 + 1 + kMaxSeg; }
inline size_t tilemap_bytes(int R) {
    return align256(256 + 4 * sizeof(int32_t) * (size_t)max_tiles_for(R)) + (size_t)max_tiles_for(R) * kRelPitch * sizeof(int32_t);
}

TileMap tilemap_at(void* ws, int R) {
    TileMap m;
    char* p = reinterpret_cast<char*>(ws);
    const size_t n = (size_t)max_tiles_for(R);
    m.n_tiles = reinterpret_cast<int32_t*>(p);
    m.row0 = reinterpret_cast<int32_t*>(p + 256);
    m.nrows = m.row0 + n;
    m.expert = m.nrows + n;
    m.gather = m.expert + n;
    m.rel = reinterpret_cast<int32_t*>(p + align256(256 + 4 * sizeof(int32_t) * n));
    return m;
}

// Tile map.  The received rows come as segments (rows seg_offset[i] .. seg_offset[i+1] - 1 belong to local
// expert seg_expert[i]); with several sources and several local experts the segments of one expert are not
// adjacent, and a segment can be much shorter than a tile (160 rows per source and expert under the
// capacity rule of the Switch-shape workload), so cutting every segment into tiles of its own would leave
// most tiles half empty.  With `gather` the segments of an expert are chained in index order into one
// list of rows that is cut into full tiles: a tile whose rows are not consecutive in memory carries a
// table of row offsets (rel), which the GEMM uses for its A-operand addresses and its output rows.
// Without `gather` only adjacent segments of the same expert are merged (every tile is consecutive rows).
//
// Items are the clamped, non-empty segments in processing order; a group is a maximal chain of items of
// one expert whose rows increase (so offsets from the tile's first row are never negative); tiles never
// straddle groups.  The construction is written once for the device kernel and for the host self check.
struct SegWork {
    int lo[kMaxSeg], hi[kMaxSeg], exp[kMaxSeg];                            // items (rows lo .. hi - 1 of one expert)
    int v0[kMaxSeg];                                                       // position of the item's first row in its group
    int grp[kMaxSeg];                                                      // group of the item
    int gaps[kMaxSeg];                                                     // items up to and including this one that do not follow their predecessor in memory
    int g_first[kMaxSeg + 1], g_tile0[kMaxSeg + 1], g_rows[kMaxSeg];       // groups: first item, first tile, rows
    int raw_off[kMaxSeg + 1], raw_exp[kMaxSeg];                            // the caller's segment list (raw_off: scratch once the items exist)
    int cnt[MOE_MAX_LOCAL], pos[MOE_MAX_LOCAL];
    int n_items, n_groups, n_tiles;
};
constexpr int kMapThreads = 1024;       // one block: a thread per segment / item, 16 waves to hide the LDS latency of the searches

// The steps take (tid, nth) = this thread and the thread count where they run in parallel; a barrier
// separates them.  The host self check runs the same per-element functions with plain loops in place
// of the block-wide ballots and prefix sums of the device kernel.
// 1: an expert outside [0, n_local) (-1) or an empty row range (-2) marks a segment to be skipped
__host__ __device__ inline void tilemap_clean(SegWork& w, int nseg, int R, int n_local, int tid, int nth) {
    for (int i = tid; i < nseg; i += nth) {
        const int lo = w.raw_off[i] > 0 ? w.raw_off[i] : 0;
        const int hi = w.raw_off[i + 1] < R ? w.raw_off[i + 1] : R;
        const int e = w.raw_exp[i];
        if (!(e >= 0 && e < n_local)) w.raw_exp[i] = -1;
        else if (!(hi > lo)) w.raw_exp[i] = -2;             // no rows: neither an item nor the end of a run
    }
    for (int e = tid; e < n_local; e += nth) w.cnt[e] = 0;
}
// 2 (gather), host form: rank of every segment among the segments of its expert, and the count per expert
inline void tilemap_rank_host(SegWork& w, int nseg) {
    for (int i = 0; i < nseg; ++i) {
        const int e = w.raw_exp[i];
        if (e < 0) continue;
        w.v0[i] = w.cnt[e]++;                        // the rank is parked in v0 until step 4
    }
}
// 3 (gather), host form: where the items of every expert start
inline void tilemap_starts_host(SegWork& w, int n_local) {
    int p = 0;
    for (int e = 0; e < n_local; ++e) { w.pos[e] = p; p += w.cnt[e]; }
    w.n_items = p;
}
// 4 (gather): segment i becomes item pos[e] + rank
__host__ __device__ inline void tilemap_place(SegWork& w, int nseg, int R, int tid, int nth) {
    for (int i = tid; i < nseg; i += nth) {
        const int e = w.raw_exp[i];
        if (e < 0) continue;
        const int k = w.pos[e] + w.v0[i];
        w.lo[k] = w.raw_off[i] > 0 ? w.raw_off[i] : 0;
        w.hi[k] = w.raw_off[i + 1] < R ? w.raw_off[i + 1] : R;
        w.exp[k] = e;
    }
}
// 2-4 without gathering (one thread): adjacent segments of the same expert merged
__host__ __device__ inline void tilemap_merge(SegWork& w, int nseg, int R) {
    int ni = 0, i = 0;
    while (i < nseg) {
        const int e = w.raw_exp[i];
        if (e < 0) { ++i; continue; }
        int j = i + 1;
        while (j < nseg && (w.raw_exp[j] == e || w.raw_exp[j] == -2)) ++j;
        const int lo = w.raw_off[i] > 0 ? w.raw_off[i] : 0;
        const int hi = w.raw_off[j] < R ? w.raw_off[j] : R;
        if (hi > lo) { w.lo[ni] = lo; w.hi[ni] = hi; w.exp[ni] = e; ++ni; }
        i = j;
    }
    w.n_items = ni;
}
// 5: does item k open a group / does it leave a gap behind its predecessor
__host__ __device__ inline bool tilemap_opens(const SegWork& w, int k, bool gather) {
    return !(gather && k > 0 && w.exp[k] == w.exp[k - 1] && w.lo[k] >= w.hi[k - 1]);
}
__host__ __device__ inline bool tilemap_gap(const SegWork& w, int k, bool gather) {
    return !tilemap_opens(w, k, gather) && w.lo[k] != w.hi[k - 1];
}
// 5, host form: groups and their tiles
inline void tilemap_groups_host(SegWork& w, int BM, bool gather) {
    const int ni = w.n_items;
    int ng = 0, nt = 0, rows = 0, gaps = 0;
    for (int k = 0; k < ni; ++k) {
        if (tilemap_opens(w, k, gather)) {
            if (ng > 0) { w.g_rows[ng - 1] = rows; nt += (rows + BM - 1) / BM; }
            w.g_first[ng] = k; w.g_tile0[ng] = nt; rows = 0;
            ++ng;
        }
        gaps += tilemap_gap(w, k, gather) ? 1 : 0;
        w.gaps[k] = gaps;
        w.v0[k] = rows;
        w.grp[k] = ng - 1;
        rows += w.hi[k] - w.lo[k];
    }
    if (ng > 0) { w.g_rows[ng - 1] = rows; nt += (rows + BM - 1) / BM; }
    w.g_first[ng] = ni; w.g_tile0[ng] = nt;
    w.n_groups = ng;
    w.n_tiles = nt;
}

// item of group g that holds group row v: the largest item with v0 <= v
__host__ __device__ inline int tilemap_item_of(const SegWork& w, int g, int v) {
    int c = w.g_first[g], d = w.g_first[g + 1];
    while (d - c > 1) { const int mid = (c + d) >> 1; if (w.v0[mid] <= v) c = mid; else d = mid; }
    return c;
}
struct TileSpan { int v_lo, v_hi, first_item, row0, gather; };
// tile q of group g: its range of group rows, its first row in memory, whether its rows have gaps
__host__ __device__ inline TileSpan tilemap_span(const SegWork& w, int g, int q, int BM) {
    TileSpan s;
    s.v_lo = q * BM;
    s.v_hi = w.g_rows[g] < s.v_lo + BM ? w.g_rows[g] : s.v_lo + BM;
    s.first_item = tilemap_item_of(w, g, s.v_lo);
    const int last_item = tilemap_item_of(w, g, s.v_hi - 1);
    s.row0 = w.lo[s.first_item] + (s.v_lo - w.v0[s.first_item]);
    s.gather = (w.gaps[last_item] - w.gaps[s.first_item] > 0) ? 1 : 0;   // a gap in front of an item that starts inside the tile
    return s;
}
// 6: the record of tile t
__host__ __device__ inline void tilemap_tile(const SegWork& w, int t, int BM, const TileMap& m) {
    int a = 0, b = w.n_groups;                       // largest group with g_tile0 <= t
    while (b - a > 1) { const int mid = (a + b) >> 1; if (w.g_tile0[mid] <= t) a = mid; else b = mid; }
    const TileSpan s = tilemap_span(w, a, t - w.g_tile0[a], BM);
    m.row0[t] = s.row0;
    m.nrows[t] = s.v_hi - s.v_lo;
    m.expert[t] = w.exp[s.first_item];
    m.gather[t] = s.gather;
}
// 7: the offset tables, item by item.  Only the first and the last tile of an item can have gaps (the
// tiles in between lie inside the item); for each of the two, if it has gaps, the item's rows in it are a
// run of consecutive table entries with consecutive values: rel[dst + r] = val + r for r < cnt.
struct RelJob { int dst, cnt, val; };
__host__ __device__ inline void tilemap_rel_jobs(const SegWork& w, int k, int BM, int n_tiles, RelJob (&job)[2]) {
    job[0] = job[1] = RelJob{0, 0, 0};
    const int g = w.grp[k], len = w.hi[k] - w.lo[k];
    const int q_a = w.v0[k] / BM, q_b = (w.v0[k] + len - 1) / BM;
    for (int pass = 0; pass < 2; ++pass) {
        const int q = pass == 0 ? q_a : q_b;
        if (pass == 1 && q_b == q_a) break;
        const int tile = w.g_tile0[g] + q;
        if (tile >= n_tiles) continue;
        const TileSpan s = tilemap_span(w, g, q, BM);
        if (!s.gather) continue;
        const int v_a = w.v0[k] > s.v_lo ? w.v0[k] : s.v_lo;                 // the item's rows inside the tile
        const int v_b = w.v0[k] + len < s.v_hi ? w.v0[k] + len : s.v_hi;
        job[pass].dst = tile * kRelPitch + (v_a - s.v_lo);
        job[pass].cnt = v_b - v_a;
        job[pass].val = w.lo[k] + (v_a - w.v0[k]) - s.row0;
    }
}

// Barrier that orders LDS traffic only (lgkmcnt(0), then s_barrier): the steps of the map exchange data
// through LDS alone, and __syncthreads() would also wait for every global store to land.
__device__ __forceinline__ void lds_barrier() {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt(0xC07F);              // lgkmcnt(0); vmcnt and expcnt untouched
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}
// exclusive prefix sums of three values per thread over the block; totals to every thread
struct Int3 { int a, b, c; };
__device__ __forceinline__ Int3 block_scan3(Int3 v, Int3* excl, int* wave_tot /* LDS [3][16] */) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
    Int3 incl = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int ua = __shfl_up(incl.a, o, 64), ub = __shfl_up(incl.b, o, 64), uc = __shfl_up(incl.c, o, 64);
        if (lane >= o) { incl.a += ua; incl.b += ub; incl.c += uc; }
    }
    lds_barrier();                                 // wave_tot may still be read from an earlier scan
    if (lane == 63) { wave_tot[wave] = incl.a; wave_tot[16 + wave] = incl.b; wave_tot[32 + wave] = incl.c; }
    lds_barrier();
    Int3 before = {0, 0, 0}, total = {0, 0, 0};
#pragma unroll
    for (int wv = 0; wv < nw; ++wv) {
        const int ta = wave_tot[wv], tb = wave_tot[16 + wv], tc = wave_tot[32 + wv];
        if (wv < wave) { before.a += ta; before.b += tb; before.c += tc; }
        total.a += ta; total.b += tb; total.c += tc;
    }
    excl->a = before.a + incl.a - v.a; excl->b = before.b + incl.b - v.b; excl->c = before.c + incl.c - v.c;
    return total;
}

// One block, a thread per segment.  The segment list is read into LDS in one round trip; the stable order
// by expert comes from wave ballots (segments of the same expert inside a wave) plus a scan over the 16
// waves; groups, positions inside the groups and the tiles of the groups come from two block-wide prefix
// sums; then one thread per tile writes the tile records and the items fill the offset tables.
__global__ __launch_bounds__(kMapThreads) void tilemap_kernel(const int32_t* __restrict__ seg_offset,
                                                              const int32_t* __restrict__ seg_expert, int nseg, int R,
                                                              int BM, int n_local, int gather, int max_tiles, TileMap m) {
    __shared__ SegWork w;
    __shared__ int wave_cnt[kMapThreads / 64][MOE_MAX_LOCAL];
    __shared__ int wave_tot[3 * 16];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nth = blockDim.x, nw = nth >> 6;       // at least as many threads as segments (the launch sees to that)
    for (int i = tid; i <= nseg; i += nth) {
        w.raw_off[i] = seg_offset[i];
        if (i < nseg) w.raw_exp[i] = seg_expert[i];
    }
    for (int i = tid; i < (kMapThreads / 64) * MOE_MAX_LOCAL; i += nth) (&wave_cnt[0][0])[i] = 0;
    lds_barrier();
    tilemap_clean(w, nseg, R, n_local, tid, nth);
    lds_barrier();
    if (gather) {
        // rank among the segments of the same expert: inside the wave from ballots over the bits of the expert id
        const int e = tid < nseg ? w.raw_exp[tid] : -1;
        unsigned long long peers = __ballot(e >= 0);
#pragma unroll
        for (int b = 0; b < 6; ++b) {                // MOE_MAX_LOCAL = 64 experts: six bits
            const unsigned long long mb = __ballot((e >> b) & 1);
            peers &= ((e >> b) & 1) ? mb : ~mb;
        }
        const int rank_in_wave = __popcll(peers & ((1ull << lane) - 1ull));
        if (e >= 0 && rank_in_wave == 0) wave_cnt[wave][e] = __popcll(peers);
        lds_barrier();
        if (tid < n_local) {                         // exclusive scan over the waves, total per expert
            int run = 0;
#pragma unroll
            for (int wv = 0; wv < nw; ++wv) {
                const int c = wave_cnt[wv][tid];
                wave_cnt[wv][tid] = run;
                run += c;
            }
            w.cnt[tid] = run;
        }
        lds_barrier();
        if (e >= 0) w.v0[tid] = wave_cnt[wave][e] + rank_in_wave;
        if (wave == 0) {                             // where the items of every expert start
            const int c = lane < n_local ? w.cnt[lane] : 0;
            int incl = c;
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const int up = __shfl_up(incl, o, 64);
                if (lane >= o) incl += up;
            }
            if (lane < n_local) w.pos[lane] = incl - c;
            if (lane == 63) w.n_items = incl;
        }
        lds_barrier();
        tilemap_place(w, nseg, R, tid, nth);
    } else if (tid == 0) {
        tilemap_merge(w, nseg, R);
    }
    lds_barrier();
    // groups: item tid opens one or not; prefix sums give the group of every item, the rows in front of it
    // and the gaps up to it
    const int ni = w.n_items;
    const bool live = tid < ni;
    const bool opens = live && tilemap_opens(w, tid, gather != 0);
    const bool gap = live && tilemap_gap(w, tid, gather != 0);
    const int len = live ? w.hi[tid] - w.lo[tid] : 0;
    Int3 ex;
    const Int3 tot = block_scan3(Int3{opens ? 1 : 0, len, gap ? 1 : 0}, &ex, wave_tot);
    const int ng = tot.a;
    int* rows_before = w.raw_off;                    // rows in front of each group (the raw list is no longer needed)
    if (live) {
        w.grp[tid] = ex.a + (opens ? 1 : 0) - 1;
        w.gaps[tid] = ex.c + (gap ? 1 : 0);
        if (opens) { w.g_first[ex.a] = tid; rows_before[ex.a] = ex.b; }
    }
    if (tid == 0) { w.g_first[ng] = ni; rows_before[ng] = tot.b; w.n_groups = ng; }
    lds_barrier();
    if (live) w.v0[tid] = ex.b - rows_before[w.grp[tid]];
    const int g_rows = tid < ng ? rows_before[tid + 1] - rows_before[tid] : 0;
    Int3 ex2;
    const Int3 tot2 = block_scan3(Int3{tid < ng ? (g_rows + BM - 1) / BM : 0, 0, 0}, &ex2, wave_tot);
    if (tid < ng) { w.g_rows[tid] = g_rows; w.g_tile0[tid] = ex2.a; }
    // a well-formed list (non-decreasing offsets) stays below the bound; overlapping segments are cut off here
    const int nt = tot2.a < max_tiles ? tot2.a : max_tiles;
    if (tid == 0) { w.g_tile0[ng] = tot2.a; w.n_tiles = nt; *m.n_tiles = nt; }
    lds_barrier();
    for (int t = tid; t < nt; t += nth) tilemap_tile(w, t, BM, m);
    if (!gather) return;
    // offset tables: every item works out its (at most two) runs of table entries; the runs are then parked
    // in LDS, over the item arrays that nobody needs any more, and written by whole waves, 64 entries a time
    RelJob job[2] = {{0, 0, 0}, {0, 0, 0}};
    if (live) tilemap_rel_jobs(w, tid, BM, nt, job);
    lds_barrier();
    static_assert(offsetof(SegWork, gaps) == 5 * kMaxSeg * sizeof(int), "the six item arrays must be contiguous");
    int* jd = &w.lo[0];                              // [2 * kMaxSeg] each
    int* jc = jd + 2 * kMaxSeg;
    int* jv = jc + 2 * kMaxSeg;
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
        jd[2 * tid + pass] = job[pass].dst;
        jc[2 * tid + pass] = job[pass].cnt;
        jv[2 * tid + pass] = job[pass].val;
    }
    lds_barrier();
    // the runs go round the waves (run j to wave j % nw) so that a short list still uses all of them; lane l of
    // wave w holds runs w + nw * l and w + nw * (64 + l), and the wave walks through them one at a time
    int d_reg[2], c_reg[2], v_reg[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int j = wave + nw * (64 * h + lane);
        d_reg[h] = jd[j];
        c_reg[h] = jc[j];
        v_reg[h] = jv[j];
    }
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        unsigned long long todo = __ballot(c_reg[h] > 0);
        while (todo) {
            const int src = __builtin_ctzll(todo);
            todo &= todo - 1;
            const int dst = __builtin_amdgcn_readlane(d_reg[h], src), cnt = __builtin_amdgcn_readlane(c_reg[h], src);
            const int val = __builtin_amdgcn_readlane(v_reg[h], src);
            for (int r = lane; r < cnt; r += 64) m.rel[(size_t)dst + r] = val + r;
        }
    }
}

enum { EPI_PLAIN = 0, EPI_SILU = 1, EPI_GELU = 2, EPI_SWIGLU = 3 };

__device__ __forceinline__ float silu_f(float a) { return a / (1.f + __expf(-a)); }
__device__ __forceinline__ float gelu_tanh_f(float a) {
    const float u = 0.7978845608028654f * (a + 0.044715f * a * a * a);
    return 0.5f * a * (1.f + tanhf(u));
}
template <int EPI> __device__ __forceinline__ float epilogue(float a, float b) {
    if (EPI == EPI_SILU) return silu_f(a);
    if (EPI == EPI_GELU) return gelu_tanh_f(a);
    if (EPI == EPI_SWIGLU) return silu_f(a) * b;
    return a;
}

// Tile number `id` of `total` = tiles_m * tiles_n -> (tile_m, tile_n); a bijection for every shape.
// Blocks are handed to the 8 XCDs round-robin (XCD = id % 8), each XCD has its own L2, and all of them
// share the memory-side cache.  The map gives XCD x a band of tiles_m / 8 consecutive M-tiles and lets it
// walk ALL N-tiles for that band, in groups of 8 (then 4, 2, 1) M-tiles, M fastest: the blocks resident on an
// XCD form a patch of a few M-tiles by a few N-tiles (few distinct operand tiles in its L2), and the 8 XCDs
// sweep the N-tiles in step with each other, so a B tile fetched for one XCD is in the memory-side cache
// when the other seven ask for it and the A bands stay there for the whole sweep.  The tiles_m % 8
// M-tiles that do not fill a band come last, cut evenly over the XCDs.
__host__ __device__ __forceinline__ void tile_of_block_bands(int id, int tiles_m, int tiles_n, int* tm, int* tn) {
    const int x = id % 8, j = id / 8;                        // XCD and position in that XCD's sequence
    const int q = tiles_m / 8;                               // M-tiles per band
    const int band = q * tiles_n;                            // tiles of a band
    if (j < band) {
        // group heights: 8 as often as it fits, then the binary digits of the rest, so that a height always
        // divides the 32 blocks resident on an XCD (a 8 x 4, 4 x 8, ... patch with no straddling rows)
        int in_g = j, h = 8, first = 0, rest = q;
        while (true) {
            while (h > rest) h >>= 1;
            const int sz = h * tiles_n;
            if (in_g < sz) break;
            in_g -= sz; first += h; rest -= h;
        }
        *tm = q * x + first + in_g % h;
        *tn = in_g / h;
        return;
    }
    const int lm = tiles_m - 8 * q;                          // left-over M-tiles (lm >= 1 here)
    const int left = lm * tiles_n;
    const int v = x * (left / 8) + min(x, left % 8) + (j - band);
    *tm = 8 * q + v % lm;
    *tn = v / lm;
}
// With fewer than 32 M-tiles a band is at most three rows of tiles (patches of 1 x 32 or 2 x 16 tiles: 33 or
// 18 operand tiles for the 32 resident blocks instead of 12); when the N side has thicker bands the same
// numbering is used with the roles of M and N exchanged: XCD x owns a band of N-tiles and all XCDs sweep
// the M-tiles in step.  Measured at the 4096 -> 14336 -> 4096 shape: +7 % on both GEMMs at 2000 rows (bands
// of one row), +2.5 % at 6745 and 7900 rows (three rows), +1 % at 4147 and 5000 (two rows); with bands of
// four to seven rows the exchange gains or loses less than 1 %, so those keep the M bands.
__host__ __device__ __forceinline__ void tile_of_block(int id, int total, int tiles_m, int tiles_n, int* tm, int* tn) {
    (void)total;
    if (tiles_m / 8 < 4 && tiles_n / 8 > tiles_m / 8) tile_of_block_bands(id, tiles_n, tiles_m, tn, tm);
    else tile_of_block_bands(id, tiles_m, tiles_n, tm, tn);
}

// Tail splitting.  The grid runs in rounds of `ncu` tiles (one block per CU); the tiles of a last,
// mostly empty round would leave most CUs idle for a whole tile time.  When that round has at most
// ncu / 2 tiles, each of them is cut along K into `parts` pieces that run as separate blocks
// (1/parts of a tile time) and write fp32 partial tiles; a second small kernel adds the pieces
// of a tile in piece order and applies the epilogue.  Everything here depends
// only on the shapes, so results do not vary from run to run.
struct TailPlan {
    int n_full;        // tiles handled whole: ids [0, n_full)
    int n_tail;        // tiles cut in pieces: ids [n_full, n_full + n_tail)
    int parts;         // pieces per tail tile (1: no tail)
    int pairs_per;     // k-tile pairs per piece
};
__host__ __device__ __forceinline__ TailPlan plan_tail(int total, int ncu, int nk) {
    TailPlan p;
    p.n_full = total; p.n_tail = 0; p.parts = 1; p.pairs_per = nk / 2;
    const int rem = total % ncu;
    const int npairs = nk / 2;
    if (rem == 0) return p;
    // up to 8 pieces of at least 16 k-tiles (more only add partial tiles); 2 or 3 pieces pay for the extra
    // pass only when a piece is still long (64 k-tiles)
    const int parts = min(min(ncu / rem, npairs / 8), 8);
    if (parts < 2 || (parts < 4 && npairs / parts < 32)) return p;
    p.pairs_per = (npairs + parts - 1) / parts;
    p.parts = (npairs + p.pairs_per - 1) / p.pairs_per;
    p.n_tail = rem;
    p.n_full = total - rem;
    return p;
}
constexpr size_t kPartialBytes = (size_t)256 * 256 * sizeof(float);   // one fp32 partial tile

// ------------------------------------------------------------------------------------ fp32
// C[r, n] = epi( sum_k A[r,k] * B0[n,k], sum_k A[r,k] * B1[n,k] ), 64x64 tile, 4x4 per thread.
template <int EPI>
__global__ __launch_bounds__(256) void gemm_f32_kernel(const float* __restrict__ A, int lda, TileMap m,
                                                       ExpertTable tab, int which0, int which1, int N, int K,
                                                       float* __restrict__ C, int ldc, int tiles_n) {
    __shared__ float As[16][65], B0s[16][65], B1s[(EPI == EPI_SWIGLU) ? 16 : 1][65];
    const int tile_m = blockIdx.x / tiles_n, tile_n = blockIdx.x % tiles_n;
    if (tile_m >= *m.n_tiles) return;
    const int row0 = m.row0[tile_m], nrows = m.nrows[tile_m], ex = m.expert[tile_m];
    auto pick = [&](int which) -> const float* {
        return reinterpret_cast<const float*>(which == 0 ? tab.w1[ex] : which == 1 ? tab.w_up[ex] : tab.w_down[ex]);
    };
    const float* B0 = pick(which0);
    const float* B1 = (EPI == EPI_SWIGLU) ? pick(which1) : nullptr;
    const int n0 = tile_n * 64;
    const int tx = threadIdx.x % 16, ty = threadIdx.x / 16;
    float acc0[4][4] = {}, acc1[4][4] = {};
    for (int k0 = 0; k0 < K; k0 += 16) {
        for (int q = threadIdx.x; q < 64 * 16; q += 256) {
            const int r = q / 16, kk = q % 16;
            const int gr = row0 + min(r, nrows - 1);
            As[kk][r] = (k0 + kk < K) ? A[(size_t)gr * lda + k0 + kk] : 0.f;
            const int gn = n0 + r;
            const bool ok = gn < N && k0 + kk < K;
            B0s[kk][r] = ok ? B0[(size_t)gn * K + k0 + kk] : 0.f;
            if (EPI == EPI_SWIGLU) B1s[kk][r] = ok ? B1[(size_t)gn * K + k0 + kk] : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < 16; ++kk) {
            float a[4], b0[4], b1[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) { a[i] = As[kk][ty * 4 + i]; b0[i] = B0s[kk][tx * 4 + i]; }
            if (EPI == EPI_SWIGLU)
#pragma unroll
                for (int i = 0; i < 4; ++i) b1[i] = B1s[kk][tx * 4 + i];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    acc0[i][j] = fmaf(a[i], b0[j], acc0[i][j]);
                    if (EPI == EPI_SWIGLU) acc1[i][j] = fmaf(a[i], b1[j], acc1[i][j]);
                }
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int r = ty * 4 + i;
        if (r >= nrows) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int n = n0 + tx * 4 + j;
            if (n < N) C[(size_t)(row0 + r) * ldc + n] = epilogue<EPI>(acc0[i][j], acc1[i][j]);
        }
    }
}

// ------------------------------------------------------------------------------------ bf16 MFMA
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int BM = 256, BN = 256, BK = 32, STAGES = 5;
constexpr int kTileBytes = BM * BK * 2;        // one 256 x 32 bf16 operand tile: 16 KB
constexpr int kStageBytes = 2 * kTileBytes;    // A tile then B tile
constexpr int kLdsBytes = STAGES * kStageBytes;   // 160 KB: the whole LDS of a CU

// An operand tile is stored as 16 blocks of 16 rows; a block is 1 KB = 64 slots of
// 16 bytes and is filled by ONE wave-wide direct-to-LDS load (lane l fills slot l).
// Inside a block the rows are kept row-major (4 slots per row, so 4 neighbouring
// lanes fetch 64 contiguous bytes of one row from memory), with the 16-byte chunk
// index XOR-ed by row/4:
//     slot(r, c) = 4*r + (c ^ (r >> 2)),   r = 0..15, c = 0..3.
// The LDS has 64 banks and serves a ds_read_b128 sixteen lanes at a time; the 16
// lanes of one MFMA operand read (16 consecutive rows, same chunk) then fall on
// slots with 16 different values of slot % 16, i.e. on all 64 banks once.
__device__ __forceinline__ int slot_of(int r, int c) { return (r << 2) + (c ^ (r >> 2)); }
// inverse for the loading lane: which (row, chunk) of the block lane l must fetch
__device__ __forceinline__ void rc_of_slot(int l, int* r, int* c) {
    *r = l >> 2;
    *c = (l & 3) ^ (l >> 4);
}
// byte offset of (row, chunk) inside a 256-row tile
__device__ __forceinline__ int tile_off(int row, int c) { return ((row >> 4) << 10) + (slot_of(row & 15, c) << 4); }

__device__ __forceinline__ float fast_silu(float a) {
    return a * __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(-1.44269504088896f * a));
}
// tanh-form GELU: 0.5 a (1 + tanh(u)) = a * sigmoid(2u), u = sqrt(2/pi) (a + 0.044715 a^3); one exp2 and one rcp
// (the exponent -log2(e) * 2u = a * (k1 + k2 a^2) is formed with the constants folded: five plain operations around the two slow ones)
__device__ __forceinline__ float fast_gelu(float a) {
    const float k1 = -1.44269504088896f * 1.5957691216057308f, k2 = k1 * 0.044715f;
    const float arg = a * __builtin_fmaf(k2, a * a, k1);
    return a * __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(arg));
}
template <int EPI> __device__ __forceinline__ float epilogue_bf16(float a, float b) {
    if (EPI == EPI_SILU) return fast_silu(a);
    if (EPI == EPI_GELU) return fast_gelu(a);
    if (EPI == EPI_SWIGLU) return fast_silu(a) * b;
    return a;
}
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
    const f32x2 v = {lo, hi};
    const bf16x2 b = __builtin_convertvector(v, bf16x2);      // round to nearest even in hardware
    return *reinterpret_cast<const uint32_t*>(&b);
}

// Epilogue of a tile in two steps: activation on registers, pack to bf16 and write to LDS (which
// must be idle) for one 32-row tile i of every wave; then whole-line stores of row tiles
// [i_lo, i_hi).  acc_i[j][e] is output row  i*32 + lane%32  and output column
// j*32 + (e/4)*8 + (lane/32)*4 + e%4  of the wave's 128 x (NJ*32) block.
template <int EPI> struct EpiGeom {
    static constexpr int NOUT = (EPI == EPI_SWIGLU) ? 128 : 256;   // output columns per block
    static constexpr int NW = NOUT / 2;                            // output columns per wave
    static constexpr int NJ = NW / 32;                             // 32-wide output column tiles per wave
    static constexpr int PITCH = NW * 2 + 8;                       // bytes; the +8 spreads the 32 rows of a write over all banks
};
template <int EPI>
__device__ __forceinline__ void stage_rows(const f32x16 (&acc_i)[4], int i, unsigned char* lds) {
    using G = EpiGeom<EPI>;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int fr = lane & 31, fk = lane >> 5;
    unsigned char* region = lds + wave * (128 * G::PITCH);
#pragma unroll
    for (int j = 0; j < G::NJ; ++j)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            float v[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const float up = (EPI == EPI_SWIGLU) ? acc_i[j + 2][4 * g + t] : 0.f;
                v[t] = epilogue_bf16<EPI>(acc_i[j][4 * g + t], up);
            }
            const u32x2 p = {pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3])};
            *reinterpret_cast<u32x2*>(region + (i * 32 + fr) * G::PITCH + (j * 32 + g * 8 + fk * 4) * 2) = p;
        }
}
template <int EPI, bool GATHER>
__device__ __forceinline__ void flush_rows_impl(int i_lo, int i_hi, const unsigned char* lds, int row0, int nrows,
                                                const int32_t* __restrict__ rel, int n0, int N, uint16_t* __restrict__ C, int ldc) {
    using G = EpiGeom<EPI>;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const unsigned char* region = lds + wave * (128 * G::PITCH);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");     // a wave reads back only what it wrote itself
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    constexpr int LPR = G::NW * 2 / 16;            // lanes per output row (16 bytes each)
    constexpr int RPI = 64 / LPR;                  // rows per store instruction
    const int sub_r = lane / LPR, sub_c = lane % LPR;
    const int col = n0 + wn * G::NW + sub_c * 8;
#pragma unroll 4
    for (int it = i_lo * 32 / RPI; it < i_hi * 32 / RPI; ++it) {
        const int r = it * RPI + sub_r;            // row inside this wave's 128
        const unsigned char* src = region + r * G::PITCH + sub_c * 16;
        const u32x2 lo = *reinterpret_cast<const u32x2*>(src);
        const u32x2 hi = *reinterpret_cast<const u32x2*>(src + 8);
        const int gr = wm * 128 + r;
        if (gr < nrows && col < N) {
            const u32x4 q = {lo.x, lo.y, hi.x, hi.y};
            const int orow = row0 + (GATHER ? rel[gr] : gr);   // gathered tile: its rows are not consecutive
            *reinterpret_cast<u32x4*>(C + (size_t)orow * ldc + col) = q;
        }
    }
}
// two copies of the store loop: the common one keeps its plain row arithmetic
template <int EPI>
__device__ __forceinline__ void flush_rows(int i_lo, int i_hi, const unsigned char* lds, int row0, int nrows,
                                           const int32_t* __restrict__ rel, int n0, int N, uint16_t* __restrict__ C, int ldc) {
    if (rel) flush_rows_impl<EPI, true>(i_lo, i_hi, lds, row0, nrows, rel, n0, N, C, ldc);
    else flush_rows_impl<EPI, false>(i_lo, i_hi, lds, row0, nrows, rel, n0, N, C, ldc);
}

// C[r, n] = epi(sum_k A[r,k] B0[n,k] , sum_k A[r,k] B1[n,k]) for one 256-row M-tile and one
// N-tile.  SwiGLU: the B tile's 256 rows are, per wave-column wn (64 output columns), 64 rows
// of W1 followed by the 64 rows of Wu for the same columns, so the gate and the up product of
// a column live in the same lane and the activation needs no exchange.
//
// Pipeline: 5 LDS stages of one 32-wide k-tile each (160 KB).  Loads are direct-to-LDS and
// issued in PAIRS of k-tiles (2q, 2q+1) every second iteration, interleaved so that the two
// halves of every 128-byte memory line are requested back to back: half-line requests that
// come a whole k-tile apart cost about twice the L2 bandwidth.  The pair (kt+4, kt+5) is issued
// in iteration kt (kt even) and first needed 2.5 iterations later.
// The MFMAs are issued as D = B . A^T (operands swapped), so a lane ends up with 4 consecutive
// output COLUMNS of one row: the epilogue packs them to 8 bytes, transposes through LDS and
// writes whole 128-byte lines.
//
// TIMED (diagnostics, moe_diag_ffn_phases): the same kernel with the 100 MHz wall clock read by lane 0 of every wave
// into marks[block][wave][4]: 0 start, 1 first operands in LDS (loop about to start), 2 loop done, 3 end.  The
// ordinary instantiation contains none of it.
template <int EPI, bool TIMED>
__global__ __launch_bounds__(256, 1) void gemm_bf16_kernel(const uint16_t* __restrict__ A, int lda, TileMap m,
                                                           ExpertTable tab, int which0, int which1, int N, int K,
                                                           uint16_t* __restrict__ C, int ldc, int tiles_n, int ncu,
                                                           float* __restrict__ partial, long long* __restrict__ marks) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];
#define MOE_MARK(i)                                                                                                 \
    do {                                                                                                            \
        if (TIMED && (threadIdx.x & 63) == 0)                                                                       \
            marks[((size_t)blockIdx.x * 4 + (threadIdx.x >> 6)) * 4 + (i)] = (long long)wall_clock64();              \
    } while (0)
    MOE_MARK(0);
    constexpr int NOUT = (EPI == EPI_SWIGLU) ? 128 : 256;                  // output columns per block
    const int n_tiles_m = *m.n_tiles;
    const int total = n_tiles_m * tiles_n;
    const TailPlan plan = plan_tail(total, ncu, K / BK);
    int tile_id = blockIdx.x, piece = -1;                                   // piece < 0: the whole K range
    if ((int)blockIdx.x >= plan.n_full) {
        const int j = blockIdx.x - plan.n_full;
        if (j >= plan.n_tail * plan.parts) return;
        tile_id = plan.n_full + j % plan.n_tail;
        piece = j / plan.n_tail;
    }
    int tile_m, tile_n;
    tile_of_block(tile_id, total, n_tiles_m, tiles_n, &tile_m, &tile_n);
    // everything read from the tile map is the same for the whole block: keep it in scalar registers
    const int row0 = __builtin_amdgcn_readfirstlane(m.row0[tile_m]);
    const int nrows = __builtin_amdgcn_readfirstlane(m.nrows[tile_m]);
    const int ex = __builtin_amdgcn_readfirstlane(m.expert[tile_m]);
    const int32_t* rel = __builtin_amdgcn_readfirstlane(m.gather[tile_m]) ? m.rel + (size_t)tile_m * kRelPitch : nullptr;
    auto pick = [&](int which) -> const uint16_t* {
        return reinterpret_cast<const uint16_t*>(which == 0 ? tab.w1[ex] : which == 1 ? tab.w_up[ex] : tab.w_down[ex]);
    };
    const uint16_t* B0 = pick(which0);
    const uint16_t* B1 = (EPI == EPI_SWIGLU) ? pick(which1) : B0;
    const int n0 = tile_n * NOUT;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform by construction; tell the compiler
    const int wm = wave >> 1, wn = wave & 1;

    // Direct-to-LDS staging.  A stage is 32 blocks of 1 KB (16 of A, 16 of B); wave w
    // fills blocks w, w+4, ...: 4 of A and 4 of B per stage.  Addresses are kept as a wave-uniform
    // 64-bit base (advanced with k by scalar adds) plus a fixed 32-bit byte offset per lane, so a
    // load costs no vector address arithmetic.
    int lr, lc;
    rc_of_slot(lane, &lr, &lc);
    // k-tiles [kt_lo, kt_lo + nk) of the row: everything for a whole tile, one piece for a tail tile
    const int kt_lo = (piece < 0) ? 0 : piece * plan.pairs_per * 2;
    const int nk = (piece < 0) ? K / BK : min(plan.pairs_per * 2, K / BK - kt_lo);   // even: K is a multiple of 64
    const char* a_base = reinterpret_cast<const char*>(A + (size_t)row0 * lda) + (size_t)kt_lo * BK * 2;
    const char* b_base[4];
    uint32_t a_voff[4], b_voff[4];
    int a_row[4];                                            // row (relative to row0) of the tile rows this lane fetches
#pragma unroll
    for (int i = 0; i < 4; ++i) a_row[i] = min((wave + 4 * i) * 16 + lr, nrows - 1);
    if (rel) {                                               // gathered tile: offsets from row0, below 2^32 bytes (checked
        int t[4];                                            // on the host); the four loads go out together
#pragma unroll
        for (int i = 0; i < 4; ++i) t[i] = rel[a_row[i]];
#pragma unroll
        for (int i = 0; i < 4; ++i) a_row[i] = t[i];
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int blk = wave + 4 * i;                        // 16-row block of the tile (wave-uniform)
        const int r = blk * 16 + lr;                         // tile row this lane fetches
        const int ar = a_row[i];
        a_voff[i] = (uint32_t)ar * (uint32_t)lda * 2u + (uint32_t)lc * 16u;
        int col;
        if (EPI == EPI_SWIGLU) {
            const int w = r >> 7, sub = r & 127;
            b_base[i] = reinterpret_cast<const char*>(((blk * 16) & 64) ? B1 : B0) + (size_t)kt_lo * BK * 2;   // sub >= 64 for the whole block or not at all
            col = n0 + w * 64 + (sub & 63);
        } else {
            b_base[i] = reinterpret_cast<const char*>(B0) + (size_t)kt_lo * BK * 2;
            col = n0 + r;
        }
        b_voff[i] = (uint32_t)min(col, N - 1) * (uint32_t)K * 2u + (uint32_t)lc * 16u;
        // opaque to the optimiser from here on: it must stay a 32-bit lane offset next to a scalar base
        asm volatile("" : "+v"(a_voff[i]), "+v"(b_voff[i]));
    }
    // k-tiles t and t+1 (t even) into the stages at LDS byte offsets so0 and so1; past the end the last pair is fetched again (into stages nobody reads any more) so that
    // the count of outstanding loads stays uniform
    auto issue_part = [&](int t, int so0, int so1, int i_lo, int i_hi) {
        t = min(t, nk - 2);
        unsigned char* s0 = lds + so0;
        unsigned char* s1 = lds + so1;
        const size_t kb = (size_t)t * BK * 2;                // byte offset of k-tile t inside a row
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (i < i_lo || i >= i_hi) continue;
            const int blk = (wave + 4 * i) * 1024;
            const char* ak = a_base + kb;
            const char* bk = b_base[i] + kb;
            uint32_t &av = a_voff[i], &bv = b_voff[i];
            // opaque here, so that scalar base + zero-extended 32-bit lane offset is still visible when the
            // load is selected (saddr form: half the address registers, no 64-bit vector add per load)
            const char* ak1 = ak + BK * 2;
            const char* bk1 = bk + BK * 2;
            asm volatile("" : "+s"(ak), "+s"(bk), "+s"(ak1), "+s"(bk1), "+v"(av), "+v"(bv));
            __builtin_amdgcn_global_load_lds(ak + av, (__attribute__((address_space(3))) void*)(s0 + blk), 16, 0, 0);
            __builtin_amdgcn_global_load_lds(ak1 + av, (__attribute__((address_space(3))) void*)(s1 + blk), 16, 0, 0);
            __builtin_amdgcn_global_load_lds(bk + bv, (__attribute__((address_space(3))) void*)(s0 + kTileBytes + blk), 16, 0, 0);
            __builtin_amdgcn_global_load_lds(bk1 + bv, (__attribute__((address_space(3))) void*)(s1 + kTileBytes + blk), 16, 0, 0);
        }
    };

    f32x16 acc[4][4];                                        // [m-tile i][n-tile j], holds D^T: rows n, columns m
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    issue_part(0, 0, kStageBytes, 0, 4);
    issue_part(2, 2 * kStageBytes, 3 * kStageBytes, 0, 3);   // its last group goes out in the first trip below

    const int fr = lane & 31, fk = lane >> 5;      // fragment row within a 32-row tile, which k-half
    int a_off[2], b_off[2];                        // byte offsets inside a stage of 32-row tile 0, per k-step;
#pragma unroll                                     // tile i lies 2 KB further (two 16-row blocks)
    for (int s = 0; s < 2; ++s) {
        a_off[s] = tile_off(wm * 128 + fr, 2 * s + fk);
        b_off[s] = kTileBytes + tile_off(wn * 128 + fr, 2 * s + fk);
    }

    auto load_frags = [&](bf16x8 (&af)[4], bf16x8 (&bfr)[4], const unsigned char* st, int s) {
        const unsigned char* pa = st + a_off[s];
        const unsigned char* pb = st + b_off[s];
#pragma unroll
        for (int i = 0; i < 4; ++i) af[i] = *reinterpret_cast<const bf16x8*>(pa + i * 2048);
#pragma unroll
        for (int j = 0; j < 4; ++j) bfr[j] = *reinterpret_cast<const bf16x8*>(pb + j * 2048);
    };
    auto mma = [&](const bf16x8 (&af)[4], const bf16x8 (&bfr)[4]) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[j], af[i], acc[i][j], 0, 0, 0);
    };

    // Software pipeline, two k-tiles per trip, four phases of 16 MFMAs each:
    //   A(kt)   read fragments (kt, k-step 1)     | MFMAs (kt, step 0)   | load group 3 of pair (kt+2, kt+3)
    //   barrier: every wave is done with the stages of tiles kt-1 and kt
    //   B(kt)   read fragments (kt+1, step 0)     | MFMAs (kt, step 1)   | load group 0 of pair (kt+4, kt+5)
    //   A(kt+1) read fragments (kt+1, step 1)     | MFMAs (kt+1, step 0) | load group 1
    //   wait until only groups 0 and 1 (8 loads per wave) are outstanding: pair (kt+2, kt+3) is in LDS; barrier
    //   B(kt+1) read fragments (kt+2, step 0)     | MFMAs (kt+1, step 1) | load group 2
    // A group is 4 loads per wave (one 16-row block of A and of B, both k-tiles of the pair).  The
    // loads are spread evenly, one per four MFMAs: a CU sustains roughly one wave-load per 40 clocks
    // when the lines come from HBM, and a load that cannot be accepted stalls the wave's MFMA issue too.
    // A bare s_barrier is used: __syncthreads() would add a fence that waits for ALL outstanding loads.
    bf16x8 a0[4], b0[4], a1[4], b1[4];
    __builtin_amdgcn_s_waitcnt(0x0F7C);            // vmcnt(12): pair (0, 1) is in LDS
    __builtin_amdgcn_s_barrier();
    MOE_MARK(1);
    load_frags(a0, b0, lds, 0);
#define MOE_PHASE_SCHED()                                                                      \
    _Pragma("unroll") for (int q = 0; q < 8; ++q) {   /* (MFMA, LDS read) x 8 */                \
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                     \
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);                                     \
    }                                                                                          \
    _Pragma("unroll") for (int q = 0; q < 4; ++q) {   /* (MFMA, MFMA, global->LDS load) x 4 */  \
        __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);                                     \
        __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);                                     \
    }
    // so[j] is the LDS byte offset of the stage that holds k-tile kt + j; the five values rotate by two per
    // trip, which keeps modulo arithmetic out of the instruction stream
    int so[STAGES];
#pragma unroll
    for (int j = 0; j < STAGES; ++j) so[j] = j * kStageBytes;
    for (int kt = 0; kt < nk; kt += 2) {
        __builtin_amdgcn_sched_barrier(0);
        load_frags(a1, b1, lds + so[0], 1);
        issue_part(kt + 2, so[2], so[3], 3, 4);
        mma(a0, b0);
        MOE_PHASE_SCHED()
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
        load_frags(a0, b0, lds + so[1], 0);
        issue_part(kt + 4, so[4], so[0], 0, 1);
        mma(a1, b1);
        MOE_PHASE_SCHED()
        __builtin_amdgcn_sched_barrier(0);
        load_frags(a1, b1, lds + so[1], 1);
        issue_part(kt + 4, so[4], so[0], 1, 2);
        mma(a0, b0);
        MOE_PHASE_SCHED()
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_waitcnt(0x0F78);        // vmcnt(8): only groups 0 and 1 of the next pair may be outstanding
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
        load_frags(a0, b0, lds + so[2], 0);
        issue_part(kt + 4, so[4], so[0], 2, 3);
        mma(a1, b1);
        MOE_PHASE_SCHED()
        __builtin_amdgcn_sched_barrier(0);
        const int t0 = so[0], t1 = so[1];
        so[0] = so[2]; so[1] = so[3]; so[2] = so[4]; so[3] = t0; so[4] = t1;
    }
#undef MOE_PHASE_SCHED
    // no load may still target LDS, and no wave may still read operands, when LDS is reused below
    __builtin_amdgcn_s_waitcnt(0x0070);            // vmcnt(0) lgkmcnt(0)
    __builtin_amdgcn_s_barrier();
    MOE_MARK(2);

    if (piece >= 0) {
        // a piece of a tail tile: the raw accumulators, 16 bytes per lane and store (whole 4 KB per store)
        f32x4* dst = reinterpret_cast<f32x4*>(reinterpret_cast<char*>(partial) +
                                              ((size_t)(tile_id - plan.n_full) * plan.parts + piece) * kPartialBytes);
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const f32x4 v = {acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
                    dst[((i * 4 + j) * 4 + q) * 256 + tid] = v;
                }
        MOE_MARK(3);
        return;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) stage_rows<EPI>(acc[i], i, lds);
    flush_rows<EPI>(0, 4, lds, row0, nrows, rel, n0, N, C, ldc);
    MOE_MARK(3);
#undef MOE_MARK
}

// Adds the pieces of one 32-row tile per wave (blockIdx.x % 4) of tail tile blockIdx.x / 4 in piece
// order and finishes those rows like a whole tile's.
template <int EPI>
__global__ __launch_bounds__(256) void gemm_bf16_tail_kernel(TileMap m, int N, int K, uint16_t* __restrict__ C, int ldc,
                                                             int tiles_n, int ncu, const float* __restrict__ partial) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];
    const int n_tiles_m = *m.n_tiles;
    const int total = n_tiles_m * tiles_n;
    const TailPlan plan = plan_tail(total, ncu, K / BK);
    const int tt = blockIdx.x >> 2, i = blockIdx.x & 3;
    if (tt >= plan.n_tail) return;
    int tile_m, tile_n;
    tile_of_block(plan.n_full + tt, total, n_tiles_m, tiles_n, &tile_m, &tile_n);
    const int row0 = m.row0[tile_m], nrows = m.nrows[tile_m];
    const int32_t* rel = m.gather[tile_m] ? m.rel + (size_t)tile_m * kRelPitch : nullptr;
    const int tid = threadIdx.x;
    const f32x4* src = reinterpret_cast<const f32x4*>(reinterpret_cast<const char*>(partial) +
                                                      (size_t)tt * plan.parts * kPartialBytes) + (size_t)i * 16 * 256 + tid;
    // all pieces of four accumulator quads are requested before the first is added (plan_tail makes at most
    // 8 pieces): the pass is a latency-bound stream otherwise
    f32x4 sum[16];
#pragma unroll
    for (int q0 = 0; q0 < 16; q0 += 4) {
        f32x4 v[8][4];
#pragma unroll
        for (int p = 0; p < 8; ++p)
#pragma unroll
            for (int u = 0; u < 4; ++u)
                v[p][u] = (p < plan.parts) ? src[(size_t)p * (kPartialBytes / 16) + (q0 + u) * 256] : f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            sum[q0 + u] = v[0][u];
#pragma unroll
            for (int p = 1; p < 8; ++p)
                if (p < plan.parts) sum[q0 + u] += v[p][u];
        }
    }
    f32x16 acc_i[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int t = 0; t < 4; ++t) acc_i[j][4 * q + t] = sum[j * 4 + q][t];
    stage_rows<EPI>(acc_i, i, lds);
    flush_rows<EPI>(i, i + 1, lds, row0, nrows, rel, tile_n * EpiGeom<EPI>::NOUT, N, C, ldc);
}

// ------------------------------------------------------------------------------------------------
// Shares of at most 64 rows (decode-sized).  The FLOPs are negligible and every weight is used once: the job
// is to stream the weights at HBM speed, which takes bytes in flight.  The big kernel keeps only 32 KB of
// weight loads outstanding per CU (the other half of its ring is the mostly empty 256-row A tile) and streams
// at a third of HBM speed.  Here a tile is 32 or 64 rows x 128 weight rows and a stage of the LDS ring is 128
// elements of K: a wave-load fetches 4 rows x 256 contiguous bytes, a stage is 8 or 16 KB of A and 32 KB of
// weights, four or three stages fit and all but one of them (96 or 64 KB of weights) are always in flight.
// Wave w owns weight rows 32 w .. 32 w + 31 of the tile (SwiGLU: 16 gate rows, then the 16 up rows of the
// same output columns) and all rows of A: MT x 1 tiles of v_mfma_f32_32x32x16_bf16, eight k-steps per stage.
// A wave loads the weight rows it reads itself; the A tile is shared (one barrier per stage).  With fewer
// tiles than CUs every tile is cut along K into `parts` pieces (fp32 partial tiles, added in piece order by a
// second kernel: results do not depend on the run).
//
// LDS layout of a stage: blocks of 1 KB = 4 rows x 16 chunks of 16 bytes, filled by ONE wave-wide
// direct-to-LDS load (lane l fills slot l).  Inside a block slot(r, c) = 16 r + (c ^ (4 r + blk % 4)):
// the 16 lanes that an MFMA operand read serves at a time (16 consecutive rows = 4 blocks, same chunk) then
// fall on 16 different values of slot % 16, i.e. on all 64 banks once.
// MT = 1 or 2 MFMA row tiles: shares of at most 32 rows take 32-row tiles, whose smaller A part leaves room for a
// fourth stage (96 KB of weights in flight).
constexpr int SBN = 128;                                 // weight rows per tile
constexpr int SKW = 128;                                 // elements of K per stage (256 bytes of a row)
template <int MT> struct SkinnyGeom {
    static constexpr int BM_ = 32 * MT;                  // rows per tile
    static constexpr int A_BYTES = BM_ * SKW * 2;        // 8 or 16 KB
    static constexpr int STAGE = A_BYTES + SBN * SKW * 2;   // 40 or 48 KB
    static constexpr int STAGES = (MT == 1) ? 4 : 3;
    static constexpr int LDS = STAGES * STAGE;           // 160 or 144 KB
    static constexpr int LOADS = 2 * MT + 8;             // wave-loads per stage and wave
    static constexpr size_t PARTIAL = (size_t)BM_ * SBN * sizeof(float);   // one fp32 partial tile
};
constexpr int kSkinnyRows = 64;                          // shares up to this many rows take this path

struct SkinnyPlan {
    int parts;     // pieces per tile
    int per;       // stages per piece (the last piece may be shorter)
};
__host__ __device__ __forceinline__ SkinnyPlan plan_skinny(int total, int ncu, int ns) {
    SkinnyPlan p{1, ns};
    if (total <= 0 || total >= ncu) return p;
    int parts = min(min(ncu / total, ns / 2), 32);       // at least 2 stages per piece
    if (parts < 2) return p;
    p.per = (ns + parts - 1) / parts;
    p.parts = (ns + p.per - 1) / p.per;
    return p;
}

// byte offset of (row, 16-byte chunk c of the stage's 256 bytes) inside a tile region
__device__ __forceinline__ int skinny_off(int row, int c) {
    const int blk = row >> 2, r = row & 3;
    return (blk << 10) + (((r << 4) + (c ^ ((r << 2) | (blk & 3)))) << 4);
}

// Activation and store of a wave's (32 MT) x 32 block of products held in the MFMA result layout: acc[i][e] is
// row i * 32 + lane % 32 of the tile and weight row 32 w + (e / 4) * 8 + (lane / 32) * 4 + e % 4.
template <int EPI, int MT>
__device__ __forceinline__ void skinny_store(const f32x16 (&acc)[MT], int wave, int lane, int row0, int nrows,
                                             const int32_t* __restrict__ rel, int n0, int N, uint16_t* __restrict__ C, int ldc) {
    const int fr = lane & 31, fk = lane >> 5;
#pragma unroll
    for (int i = 0; i < MT; ++i) {
        const int gr = i * 32 + fr;
        if (gr >= nrows) continue;
        uint16_t* crow = C + (size_t)(row0 + (rel ? rel[gr] : gr)) * ldc;
#pragma unroll
        for (int g = 0; g < ((EPI == EPI_SWIGLU) ? 2 : 4); ++g) {
            float v[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const float up = (EPI == EPI_SWIGLU) ? acc[i][4 * (g + 2) + t] : 0.f;
                v[t] = epilogue_bf16<EPI>(acc[i][4 * g + t], up);
            }
            const int col = n0 + ((EPI == EPI_SWIGLU) ? wave * 16 : wave * 32) + g * 8 + fk * 4;
            if (col < N) *reinterpret_cast<u32x2*>(crow + col) = u32x2{pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3])};
        }
    }
}

template <int EPI, int MT>
__global__ __launch_bounds__(256, 1) void gemm_bf16_skinny_kernel(const uint16_t* __restrict__ A, int lda, TileMap m,
                                                                  ExpertTable tab, int which0, int which1, int N, int K,
                                                                  uint16_t* __restrict__ C, int ldc, int tiles_n, int ncu,
                                                                  float* __restrict__ partial) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];
    using G = SkinnyGeom<MT>;
    constexpr int NOUT = (EPI == EPI_SWIGLU) ? SBN / 2 : SBN;
    const int n_tiles_m = *m.n_tiles;
    const int total = n_tiles_m * tiles_n;
    const int ns_all = K / SKW;
    const SkinnyPlan plan = plan_skinny(total, ncu, ns_all);
    if ((int)blockIdx.x >= total * plan.parts) return;
    const int tile_id = blockIdx.x % total, piece = blockIdx.x / total;
    const int tile_m = tile_id % n_tiles_m, tile_n = tile_id / n_tiles_m;
    const int row0 = __builtin_amdgcn_readfirstlane(m.row0[tile_m]);
    const int nrows = __builtin_amdgcn_readfirstlane(m.nrows[tile_m]);
    const int ex = __builtin_amdgcn_readfirstlane(m.expert[tile_m]);
    const int32_t* rel = __builtin_amdgcn_readfirstlane(m.gather[tile_m]) ? m.rel + (size_t)tile_m * kRelPitch : nullptr;
    auto pick = [&](int which) -> const uint16_t* {
        return reinterpret_cast<const uint16_t*>(which == 0 ? tab.w1[ex] : which == 1 ? tab.w_up[ex] : tab.w_down[ex]);
    };
    const uint16_t* B0 = pick(which0);
    const uint16_t* B1 = (EPI == EPI_SWIGLU) ? pick(which1) : B0;
    const int n0 = tile_n * NOUT;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int s_lo = piece * plan.per;
    const int ns = min(plan.per, ns_all - s_lo);

    // What this lane fetches.  A: blocks NA wave .. NA wave + NA - 1 of the 4 NA (NA = 2 MT); weights: blocks
    // 8 wave .. 8 wave + 7 of the 32 (the rows this wave reads).  In block blk the lane has row lane / 16 and
    // chunk (lane % 16) ^ (4 row + blk % 4).
    constexpr int NA = 2 * MT;
    const int lrow = lane >> 4;
    const char* a_ptr[NA];
    const char* b_ptr[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        if (i < NA) {
            const int blk = NA * wave + i;
            const int lc = (lane & 15) ^ ((lrow << 2) | (blk & 3));
            int ar = min(blk * 4 + lrow, nrows - 1);
            if (rel) ar = rel[ar];
            a_ptr[i] = reinterpret_cast<const char*>(A + (size_t)row0 * lda) + (size_t)ar * lda * 2 + lc * 16 + (size_t)s_lo * SKW * 2;
        }
        const int lc = (lane & 15) ^ ((lrow << 2) | (i & 3));
        const int rr = (8 * wave + i) * 4 + lrow;           // row of the 128-row weight tile
        int col;
        const uint16_t* base;
        if (EPI == EPI_SWIGLU) {
            base = (i >= 4) ? B1 : B0;                      // rows 16 .. 31 of a wave's 32 are the up rows
            col = n0 + wave * 16 + (rr & 15);
        } else {
            base = B0;
            col = n0 + rr;
        }
        b_ptr[i] = reinterpret_cast<const char*>(base) + (size_t)min(col, N - 1) * K * 2 + lc * 16 + (size_t)s_lo * SKW * 2;
    }
    auto issue = [&](int t) {                               // stage t of this piece into ring slot t % STAGES
        const int tc = min(t, ns - 1);                      // past the end: the last stage again, into a slot nobody reads
        unsigned char* st = lds + (t % G::STAGES) * G::STAGE;
        const size_t kb = (size_t)tc * SKW * 2;
#pragma unroll
        for (int i = 0; i < NA; ++i) {
            const char* ap = a_ptr[i] + kb;
            __builtin_amdgcn_global_load_lds(ap, (__attribute__((address_space(3))) void*)(st + (NA * wave + i) * 1024), 16, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const char* bp = b_ptr[i] + kb;
            __builtin_amdgcn_global_load_lds(bp, (__attribute__((address_space(3))) void*)(st + G::A_BYTES + (8 * wave + i) * 1024), 16, 0, 0);
        }
    };

    f32x16 acc[MT];
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;

#pragma unroll
    for (int t = 0; t < G::STAGES - 1; ++t) issue(t);
    const int fr = lane & 31, fk = lane >> 5;
    for (int t = 0; t < ns; ++t) {
        // LOADS loads per stage and wave; stages t .. t + STAGES - 2 are outstanding: stage t has landed when at
        // most (STAGES - 2) * LOADS remain: 12 (MT = 2: three stages of 12) or 20 (MT = 1: four stages of 10)
        if (MT == 2) __builtin_amdgcn_s_waitcnt(0x0F7C);    // vmcnt(12)
        else __builtin_amdgcn_s_waitcnt(0x4F74);            // vmcnt(20): low four bits 4, high two bits 1
        __builtin_amdgcn_s_barrier();                       // everybody's part of stage t is in LDS; the slot of stage t - 1 is free
        issue(t + G::STAGES - 1);
        const unsigned char* st = lds + (t % G::STAGES) * G::STAGE;
#pragma unroll
        for (int s2 = 0; s2 < SKW / 16; ++s2) {
            const bf16x8 bfr = *reinterpret_cast<const bf16x8*>(st + G::A_BYTES + skinny_off(wave * 32 + fr, 2 * s2 + fk));
#pragma unroll
            for (int i = 0; i < MT; ++i) {
                const bf16x8 af = *reinterpret_cast<const bf16x8*>(st + skinny_off(i * 32 + fr, 2 * s2 + fk));
                acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr, af, acc[i], 0, 0, 0);
            }
        }
    }
    __builtin_amdgcn_s_waitcnt(0x0070);                      // no load may still be on its way to LDS when the block ends
    if (plan.parts > 1) {
        f32x4* dst = reinterpret_cast<f32x4*>(reinterpret_cast<char*>(partial) + ((size_t)tile_id * plan.parts + piece) * G::PARTIAL);
#pragma unroll
        for (int i = 0; i < MT; ++i)
#pragma unroll
            for (int q = 0; q < 4; ++q)
                dst[(i * 4 + q) * 256 + tid] = f32x4{acc[i][4 * q], acc[i][4 * q + 1], acc[i][4 * q + 2], acc[i][4 * q + 3]};
        return;
    }
    skinny_store<EPI, MT>(acc, wave, lane, row0, nrows, rel, n0, N, C, ldc);
}

// Adds the pieces of a tile in piece order (a block per tile, a thread per lane of the GEMM block) and finishes it.
template <int EPI, int MT>
__global__ __launch_bounds__(256) void gemm_bf16_skinny_sum_kernel(TileMap m, int N, int K, uint16_t* __restrict__ C, int ldc,
                                                                   int tiles_n, int ncu, const float* __restrict__ partial) {
    constexpr int NOUT = (EPI == EPI_SWIGLU) ? SBN / 2 : SBN;
    const int n_tiles_m = *m.n_tiles;
    const int total = n_tiles_m * tiles_n;
    const SkinnyPlan plan = plan_skinny(total, ncu, K / SKW);
    const int tile_id = blockIdx.x;
    if (plan.parts < 2 || tile_id >= total) return;
    const int tile_m = tile_id % n_tiles_m, tile_n = tile_id / n_tiles_m;
    const int row0 = m.row0[tile_m], nrows = m.nrows[tile_m];
    const int32_t* rel = m.gather[tile_m] ? m.rel + (size_t)tile_m * kRelPitch : nullptr;
    const int tid = threadIdx.x;
    using G = SkinnyGeom<MT>;
    const f32x4* src = reinterpret_cast<const f32x4*>(reinterpret_cast<const char*>(partial) + (size_t)tile_id * plan.parts * G::PARTIAL) + tid;
    f32x4 sum[4 * MT];
#pragma unroll
    for (int q = 0; q < 4 * MT; ++q) sum[q] = src[q * 256];
    for (int p = 1; p < plan.parts; ++p) {
        f32x4 v[4 * MT];
#pragma unroll
        for (int q = 0; q < 4 * MT; ++q) v[q] = src[(size_t)p * (G::PARTIAL / 16) + q * 256];
#pragma unroll
        for (int q = 0; q < 4 * MT; ++q) sum[q] += v[q];
    }
    f32x16 acc[MT];
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int t = 0; t < 4; ++t) acc[i][4 * q + t] = sum[i * 4 + q][t];
    skinny_store<EPI, MT>(acc, tid >> 6, tid & 63, row0, nrows, rel, tile_n * NOUT, N, C, ldc);
}

constexpr int kMaxCU = 256;                    // tail pieces per launch, at most: sizes the partial-tile workspace

// number of CUs of the current device (a round of the grid), at most kMaxCU
int round_size() {
    static int ncu = 0;
    if (ncu == 0) {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
            n = kMaxCU;
        ncu = n < kMaxCU ? n : kMaxCU;
    }
    return ncu;
}

template <int EPI, bool TIMED = false>
int launch_bf16(const void* A, int lda, const TileMap& m, const ExpertTable& tab, int which0, int which1, int N, int K,
                void* C, int ldc, int R, int nseg, float* partial, hipStream_t st, long long* marks = nullptr,
                size_t marks_len = 0) {
    const int nout = (EPI == EPI_SWIGLU) ? 128 : 256;
    const int tiles_n = (N + nout - 1) / nout;
    const int max_tiles_m = (R + BM - 1) / BM + nseg;
    const int ncu = round_size();
    const size_t lds = (size_t)kLdsBytes;
    static bool attr_done = false;
    if (!attr_done) {
        MOE_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_bf16_kernel<EPI, TIMED>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        MOE_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_bf16_tail_kernel<EPI>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        attr_done = true;
    }
    // whole tiles first, then at most ncu pieces of tail tiles; blocks past the real tile count exit at once
    if (TIMED && marks_len < (size_t)(max_tiles_m * tiles_n + ncu) * 16)
        return moe_set_error(MOE_ESHAPE, "moe_diag_ffn_phases: marks needs %zu elements", (size_t)(max_tiles_m * tiles_n + ncu) * 16);
    hipLaunchKernelGGL((gemm_bf16_kernel<EPI, TIMED>), dim3(max_tiles_m * tiles_n + ncu), dim3(256), lds, st,
                       reinterpret_cast<const uint16_t*>(A), lda, m, tab, which0, which1, N, K,
                       reinterpret_cast<uint16_t*>(C), ldc, tiles_n, ncu, partial, marks);
    MOE_LAUNCH_CHECK("gemm_bf16_kernel");
    // the tile count is only known on the device, but with a short K no count at all gives a tail (plan_tail
    // wants pieces of a minimum length): then there is nothing to add up and the launch is left out
    bool tail_possible = false;
    for (int rem = 1; rem < ncu && !tail_possible; ++rem) tail_possible = plan_tail(rem, ncu, K / BK).n_tail > 0;
    if (tail_possible) {
        hipLaunchKernelGGL((gemm_bf16_tail_kernel<EPI>), dim3(2 * ncu), dim3(256), lds, st, m, N, K,   // ncu / 2 tiles at most, 4 blocks each
                           reinterpret_cast<uint16_t*>(C), ldc, tiles_n, ncu, partial);
        MOE_LAUNCH_CHECK("gemm_bf16_tail_kernel");
    }
    return MOE_OK;
}

// Shares of at most kSkinnyRows rows (the tile map is then made of 32 MT-row tiles).
inline int skinny_tile_rows(int R) { return R <= 32 ? 32 : 64; }
template <int EPI, int MT>
int launch_bf16_skinny_mt(const void* A, int lda, const TileMap& m, const ExpertTable& tab, int which0, int which1, int N, int K,
                          void* C, int ldc, int R, int nseg, float* partial, hipStream_t st) {
    using G = SkinnyGeom<MT>;
    const int nout = (EPI == EPI_SWIGLU) ? SBN / 2 : SBN;
    const int tiles_n = (N + nout - 1) / nout;
    const int max_total = ((R + G::BM_ - 1) / G::BM_ + nseg) * tiles_n;
    const int ncu = round_size();
    static bool attr_done = false;
    if (!attr_done) {
        MOE_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_bf16_skinny_kernel<EPI, MT>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, G::LDS));
        attr_done = true;
    }
    // a tile count below the CU count is multiplied by its pieces up to at most ncu blocks
    hipLaunchKernelGGL((gemm_bf16_skinny_kernel<EPI, MT>), dim3(std::max(max_total, ncu)), dim3(256), G::LDS, st,
                       reinterpret_cast<const uint16_t*>(A), lda, m, tab, which0, which1, N, K,
                       reinterpret_cast<uint16_t*>(C), ldc, tiles_n, ncu, partial);
    MOE_LAUNCH_CHECK("gemm_bf16_skinny_kernel");
    // with more than ncu / 2 tiles along N alone no tile is ever cut (plan_skinny): nothing to add up
    if (2 * tiles_n <= ncu) {
        hipLaunchKernelGGL((gemm_bf16_skinny_sum_kernel<EPI, MT>), dim3(std::min(max_total, ncu)), dim3(256), 0, st, m, N, K,
                           reinterpret_cast<uint16_t*>(C), ldc, tiles_n, ncu, partial);
        MOE_LAUNCH_CHECK("gemm_bf16_skinny_sum_kernel");
    }
    return MOE_OK;
}
template <int EPI>
int launch_bf16_skinny(const void* A, int lda, const TileMap& m, const ExpertTable& tab, int which0, int which1, int N, int K,
                       void* C, int ldc, int R, int nseg, float* partial, hipStream_t st) {
    if (skinny_tile_rows(R) == 32) return launch_bf16_skinny_mt<EPI, 1>(A, lda, m, tab, which0, which1, N, K, C, ldc, R, nseg, partial, st);
    return launch_bf16_skinny_mt<EPI, 2>(A, lda, m, tab, which0, which1, N, K, C, ldc, R, nseg, partial, st);
}

template <int EPI>
int launch_f32(const void* A, int lda, const TileMap& m, const ExpertTable& tab, int which0, int which1, int N, int K,
               void* C, int ldc, int R, int nseg, hipStream_t st) {
    const int tiles_n = (N + 63) / 64;
    const int max_tiles_m = (R + 63) / 64 + nseg;
    hipLaunchKernelGGL((gemm_f32_kernel<EPI>), dim3(max_tiles_m * tiles_n), dim3(256), 0, st,
                       reinterpret_cast<const float*>(A), lda, m, tab, which0, which1, N, K,
                       reinterpret_cast<float*>(C), ldc, tiles_n);
    MOE_LAUNCH_CHECK("gemm_f32_kernel");
    return MOE_OK;
}

}  // namespace

// Host-side self check of the tile numbering and of the tail plan for a tiles_m x tiles_n grid with nk k-tiles
// (not part of the published interface; used by the CPU tests): every tile is produced exactly once, whole
// or as `parts` pieces that cover its k-tiles exactly once.
extern "C" int moe_selfcheck_tile_order(int32_t tiles_m, int32_t tiles_n, int32_t ncu, int32_t nk) {
    if (tiles_m < 1 || tiles_n < 1 || ncu < 1 || nk < 2 || (nk & 1)) return moe_set_error(MOE_EINVAL, "moe_selfcheck_tile_order: bad argument");
    const int total = tiles_m * tiles_n;
    std::vector<int> seen((size_t)total, 0);
    for (int id = 0; id < total; ++id) {
        int tm = -1, tn = -1;
        tile_of_block(id, total, tiles_m, tiles_n, &tm, &tn);
        if (tm < 0 || tm >= tiles_m || tn < 0 || tn >= tiles_n) return moe_set_error(MOE_EINTERNAL, "tile %d maps outside the grid", id);
        if (seen[(size_t)tm * tiles_n + tn]++) return moe_set_error(MOE_EINTERNAL, "tile (%d, %d) is produced twice", tm, tn);
    }
    const TailPlan p = plan_tail(total, ncu, nk);
    if (p.n_full + p.n_tail != total || p.n_full % ncu != 0 && p.n_tail != 0) return moe_set_error(MOE_EINTERNAL, "tail plan does not partition the tiles");
    if (p.n_tail * p.parts > ncu && p.parts > 1) return moe_set_error(MOE_EINTERNAL, "more pieces than CUs");
    if (p.parts > 1) {
        int covered = 0;
        for (int piece = 0; piece < p.parts; ++piece) {
            const int lo = piece * p.pairs_per * 2, n = std::min(p.pairs_per * 2, nk - lo);
            if (lo != covered || n < 2) return moe_set_error(MOE_EINTERNAL, "pieces do not tile the k range");
            covered += n;
        }
        if (covered != nk) return moe_set_error(MOE_EINTERNAL, "pieces do not cover the k range");
    }
    return p.parts;
}

// Host-side self check of the tile map (not part of the published interface; used by the CPU tests): runs
// the steps that the device kernel runs, on the host, and verifies that every row of every non-empty
// segment of a known expert lies in exactly one tile of that expert, that tile rows increase, that exactly
// the tiles with gaps are marked as gathered and that their offset tables are complete.  Returns the
// number of tiles, or a negative status.
extern "C" int moe_selfcheck_skinny_plan(int32_t total, int32_t ncu, int32_t ns) {
    if (total < 1 || ncu < 1 || ns < 1) return moe_set_error(MOE_EINVAL, "moe_selfcheck_skinny_plan: total, ncu and ns must be positive");
    const SkinnyPlan p = plan_skinny(total, ncu, ns);
    // every stage in exactly one piece, no empty piece, no more blocks than max(total, ncu), pieces of at least 2 stages
    if (p.parts < 1 || p.per < 1 || (int64_t)p.parts * p.per < ns || (int64_t)(p.parts - 1) * p.per >= ns)
        return moe_set_error(MOE_EINTERNAL, "skinny plan: %d pieces of %d stages do not cover %d stages once", p.parts, p.per, ns);
    if ((int64_t)total * p.parts > std::max(total, ncu))
        return moe_set_error(MOE_EINTERNAL, "skinny plan: %d tiles x %d pieces exceed the launch", total, p.parts);
    if (p.parts > 1 && (p.per < 2 || total >= ncu)) return moe_set_error(MOE_EINTERNAL, "skinny plan: pieces too short or not needed");
    return p.parts;
}

extern "C" int moe_selfcheck_tile_map(const int32_t* seg_offset, const int32_t* seg_expert, int32_t nseg, int32_t R,
                                      int32_t bm, int32_t n_local, int32_t gather) {
    if (!seg_offset || !seg_expert || nseg < 0 || nseg > kMaxSeg || R < 0 || bm < 1 || bm > kRelPitch || n_local < 1 || n_local > MOE_MAX_LOCAL)
        return moe_set_error(MOE_EINVAL, "moe_selfcheck_tile_map: bad argument");
    std::vector<SegWork> store(1);
    SegWork& w = store[0];
    for (int i = 0; i <= nseg; ++i) w.raw_off[i] = seg_offset[i];
    for (int i = 0; i < nseg; ++i) w.raw_exp[i] = seg_expert[i];
    const int nth = 7;                                    // any thread count and order must give the same map
    for (int t = 0; t < nth; ++t) tilemap_clean(w, nseg, R, n_local, t, nth);
    if (gather) {
        tilemap_rank_host(w, nseg);
        tilemap_starts_host(w, n_local);
        for (int t = nth - 1; t >= 0; --t) tilemap_place(w, nseg, R, t, nth);
    } else {
        tilemap_merge(w, nseg, R);
    }
    tilemap_groups_host(w, bm, gather != 0);
    const int max_tiles = (R + bm - 1) / bm + nseg;
    const int nt = w.n_tiles;
    if (nt > max_tiles) return moe_set_error(MOE_EINTERNAL, "%d tiles exceed the bound %d", nt, max_tiles);
    std::vector<int32_t> row0(nt), nrows(nt), expert(nt), gat(nt), rel((size_t)nt * kRelPitch, -1);
    int32_t n_tiles = nt;
    TileMap m{&n_tiles, row0.data(), nrows.data(), expert.data(), gat.data(), rel.data()};
    for (int t = nt - 1; t >= 0; --t) tilemap_tile(w, t, bm, m);
    if (gather)
        for (int k = 0; k < w.n_items; ++k) {
            RelJob job[2];
            tilemap_rel_jobs(w, k, bm, nt, job);
            for (int pass = 0; pass < 2; ++pass)
                for (int r = 0; r < job[pass].cnt; ++r) {
                    int32_t& slot = rel[(size_t)job[pass].dst + r];
                    if (slot != -1) return moe_set_error(MOE_EINTERNAL, "offset table entry %d written twice", job[pass].dst + r);
                    slot = job[pass].val + r;
                }
        }
    std::vector<int> owner((size_t)R, -1);
    for (int i = 0; i < nseg; ++i) {
        const int lo = std::max(seg_offset[i], 0), hi = std::min(seg_offset[i + 1], R);
        if (hi > lo && seg_expert[i] >= 0 && seg_expert[i] < n_local)
            for (int r = lo; r < hi; ++r) owner[r] = seg_expert[i];
    }
    std::vector<int> hits((size_t)R, 0);
    for (int t = 0; t < nt; ++t) {
        if (nrows[t] < 1 || nrows[t] > bm) return moe_set_error(MOE_EINTERNAL, "tile %d has %d rows", t, nrows[t]);
        if (gat[t] && !gather) return moe_set_error(MOE_EINTERNAL, "tile %d is gathered but gathering is off", t);
        int prev = -1;
        bool gaps = false;
        for (int r = 0; r < nrows[t]; ++r) {
            const int off = gat[t] ? rel[(size_t)t * kRelPitch + r] : r;
            if (!gat[t] && rel[(size_t)t * kRelPitch + r] != -1) return moe_set_error(MOE_EINTERNAL, "tile %d has no gaps but an offset table", t);
            const int row = row0[t] + off;
            if (off < 0 || row < 0 || row >= R) return moe_set_error(MOE_EINTERNAL, "tile %d row %d maps to %d", t, r, row);
            if (r == 0 && off != 0) return moe_set_error(MOE_EINTERNAL, "tile %d does not start at its first row", t);
            if (row <= prev) return moe_set_error(MOE_EINTERNAL, "tile %d: rows do not increase", t);
            if (prev >= 0 && row != prev + 1) gaps = true;
            if (owner[row] != expert[t]) return moe_set_error(MOE_EINTERNAL, "tile %d of expert %d holds row %d of expert %d", t, expert[t], row, owner[row]);
            ++hits[row];
            prev = row;
        }
        if (gaps != (gat[t] != 0)) return moe_set_error(MOE_EINTERNAL, "tile %d: gather flag %d but gaps %d", t, gat[t], (int)gaps);
    }
    for (int r = 0; r < R; ++r)
        if (hits[r] != (owner[r] >= 0 ? 1 : 0)) return moe_set_error(MOE_EINTERNAL, "row %d is in %d tiles", r, hits[r]);
    return nt;
}

extern "C" size_t moe_ffn_workspace_bytes(int32_t R_max, int32_t H, int32_t F, int32_t act, int32_t dtype) {
    if (R_max < 0 || H <= 0 || F <= 0 || act < 0 || act > 2 || (dtype != MOE_F32 && dtype != MOE_BF16)) return 0;
    const size_t partial = (dtype == MOE_BF16) ? (size_t)kMaxCU * kPartialBytes : 0;   // pieces of tail tiles
    return tilemap_bytes(R_max) + align256((size_t)R_max * F * elem_size(dtype)) + partial + 256;
}

// timed_gemm: 0 none, 1 / 2: that GEMM runs as its TIMED instantiation and writes marks (bf16, more than 64 rows)
static int ffn_impl(const void* recv, int32_t R, const int32_t* seg_offset, const int32_t* seg_expert, int32_t nseg,
                    const moe_expert_w* experts, int32_t n_local, int32_t H, int32_t F, int32_t act, int32_t dtype,
                    void* out, void* workspace, size_t workspace_bytes, hipStream_t st, hipEvent_t* ev,
                    int timed_gemm = 0, long long* marks = nullptr, size_t marks_len = 0) {
    if (!recv || !seg_offset || !seg_expert || !experts || !out || !workspace)
        return moe_set_error(MOE_EINVAL, "moe_expert_ffn: NULL argument");
    if (R < 0 || nseg < 0 || H <= 0 || F <= 0) return moe_set_error(MOE_EINVAL, "moe_expert_ffn: negative size");
    if (dtype != MOE_F32 && dtype != MOE_BF16) return moe_set_error(MOE_EDTYPE, "moe_expert_ffn: unknown dtype %d", dtype);
    if (act < 0 || act > 2) return moe_set_error(MOE_EDTYPE, "moe_expert_ffn: unknown act %d", act);
    if (n_local < 1 || n_local > MOE_MAX_LOCAL || nseg > kMaxSeg)
        return moe_set_error(MOE_ESHAPE, "moe_expert_ffn: need 1 <= n_local <= %d and nseg <= %d", MOE_MAX_LOCAL, kMaxSeg);
    if (dtype == MOE_BF16 && (H % 128 != 0 || F % 128 != 0))
        return moe_set_error(MOE_ESHAPE, "moe_expert_ffn: bf16 needs H and F to be multiples of 128");
    if (dtype == MOE_BF16 && (size_t)H * (size_t)F * 2 > 0xFFFFFFFFull)
        return moe_set_error(MOE_ESHAPE, "moe_expert_ffn: bf16 weight matrices are limited to 4 GiB each (32-bit lane offsets)");
    if (dtype == MOE_F32 && (H % 4 != 0 || F % 4 != 0))
        return moe_set_error(MOE_EALIGN, "moe_expert_ffn: fp32 needs H and F to be multiples of 4");
    if (!aligned16(recv) || !aligned16(out) || (reinterpret_cast<uintptr_t>(workspace) & 255u))
        return moe_set_error(MOE_EALIGN, "moe_expert_ffn: recv/out need 16-byte, workspace 256-byte alignment");
    if (workspace_bytes < moe_ffn_workspace_bytes(R, H, F, act, dtype))
        return moe_set_error(MOE_ESHAPE, "moe_expert_ffn: workspace too small (%zu < %zu)", workspace_bytes,
                             moe_ffn_workspace_bytes(R, H, F, act, dtype));
    ExpertTable tab;
    for (int e = 0; e < n_local; ++e) {
        if (!experts[e].w1 || !experts[e].w_down || (act == MOE_ACT_SWIGLU && !experts[e].w_up))
            return moe_set_error(MOE_EINVAL, "moe_expert_ffn: expert %d has a NULL weight", e);
        if (!aligned16(experts[e].w1) || !aligned16(experts[e].w_down) || !aligned16(experts[e].w_up))
            return moe_set_error(MOE_EALIGN, "moe_expert_ffn: expert %d weights must be 16-byte aligned", e);
        tab.w1[e] = experts[e].w1;
        tab.w_up[e] = experts[e].w_up;
        tab.w_down[e] = experts[e].w_down;
    }
    if (R == 0 || nseg == 0) {
        if (ev) for (int i = 0; i < 4; ++i) MOE_HIP(hipEventRecord(ev[i], st));
        return MOE_OK;
    }
    TileMap m = tilemap_at(workspace, R);
    void* hmid = reinterpret_cast<char*>(workspace) + tilemap_bytes(R);
    float* partial = reinterpret_cast<float*>(reinterpret_cast<char*>(hmid) + align256((size_t)R * F * elem_size(dtype)));
    const bool skinny = dtype == MOE_BF16 && R <= kSkinnyRows;
    if (timed_gemm != 0 && (dtype != MOE_BF16 || skinny))
        return moe_set_error(MOE_ESHAPE, "moe_diag_ffn_phases: bf16 and more than %d rows needed", kSkinnyRows);
    const int bm = skinny ? skinny_tile_rows(R) : (dtype == MOE_BF16) ? BM : 64;
    if (ev) MOE_HIP(hipEventRecord(ev[0], st));
    // gathered tiles address their rows by 32-bit byte offsets from the tile's first row
    const int gather = (dtype == MOE_BF16 && (size_t)R * (size_t)std::max(H, F) * 2 <= 0xFFFFFFFFull) ? 1 : 0;
    // A thread per segment, and whole waves write the row-offset tables of the gathered tiles.  With a handful of
    // segments a quarter of the block does it as fast and its barriers are cheaper (10 against 12.7 us with 8
    // segments); one wave alone was too few for the tables (18 against 12 us with 64 segments, 10 k table rows).
    const int map_threads = (nseg <= 16) ? 256 : kMapThreads;
    hipLaunchKernelGGL(tilemap_kernel, dim3(1), dim3(map_threads), 0, st, seg_offset, seg_expert, nseg, R, bm, n_local, gather,
                       (R + bm - 1) / bm + nseg, m);
    MOE_LAUNCH_CHECK("tilemap_kernel");
    if (ev) MOE_HIP(hipEventRecord(ev[1], st));
    int rc;
    if (skinny) {
        if (act == MOE_ACT_SWIGLU) rc = launch_bf16_skinny<EPI_SWIGLU>(recv, H, m, tab, 0, 1, F, H, hmid, F, R, nseg, partial, st);
        else if (act == MOE_ACT_GELU_MLP) rc = launch_bf16_skinny<EPI_GELU>(recv, H, m, tab, 0, 0, F, H, hmid, F, R, nseg, partial, st);
        else rc = launch_bf16_skinny<EPI_SILU>(recv, H, m, tab, 0, 0, F, H, hmid, F, R, nseg, partial, st);
        if (rc != MOE_OK) return rc;
        if (ev) MOE_HIP(hipEventRecord(ev[2], st));
        rc = launch_bf16_skinny<EPI_PLAIN>(hmid, F, m, tab, 2, 2, H, F, out, H, R, nseg, partial, st);
    } else if (dtype == MOE_BF16) {
        if (timed_gemm == 1) {
            if (act == MOE_ACT_SWIGLU) rc = launch_bf16<EPI_SWIGLU, true>(recv, H, m, tab, 0, 1, F, H, hmid, F, R, nseg, partial, st, marks, marks_len);
            else if (act == MOE_ACT_GELU_MLP) rc = launch_bf16<EPI_GELU, true>(recv, H, m, tab, 0, 0, F, H, hmid, F, R, nseg, partial, st, marks, marks_len);
            else rc = launch_bf16<EPI_SILU, true>(recv, H, m, tab, 0, 0, F, H, hmid, F, R, nseg, partial, st, marks, marks_len);
        } else if (act == MOE_ACT_SWIGLU) rc = launch_bf16<EPI_SWIGLU>(recv, H, m, tab, 0, 1, F, H, hmid, F, R, nseg, partial, st);
        else if (act == MOE_ACT_GELU_MLP) rc = launch_bf16<EPI_GELU>(recv, H, m, tab, 0, 0, F, H, hmid, F, R, nseg, partial, st);
        else rc = launch_bf16<EPI_SILU>(recv, H, m, tab, 0, 0, F, H, hmid, F, R, nseg, partial, st);
        if (rc != MOE_OK) return rc;
        if (ev) MOE_HIP(hipEventRecord(ev[2], st));
        if (timed_gemm == 2) rc = launch_bf16<EPI_PLAIN, true>(hmid, F, m, tab, 2, 2, H, F, out, H, R, nseg, partial, st, marks, marks_len);
        else rc = launch_bf16<EPI_PLAIN>(hmid, F, m, tab, 2, 2, H, F, out, H, R, nseg, partial, st);
    } else {
        if (act == MOE_ACT_SWIGLU) rc = launch_f32<EPI_SWIGLU>(recv, H, m, tab, 0, 1, F, H, hmid, F, R, nseg, st);
        else if (act == MOE_ACT_GELU_MLP) rc = launch_f32<EPI_GELU>(recv, H, m, tab, 0, 0, F, H, hmid, F, R, nseg, st);
        else rc = launch_f32<EPI_SILU>(recv, H, m, tab, 0, 0, F, H, hmid, F, R, nseg, st);
        if (rc != MOE_OK) return rc;
        if (ev) MOE_HIP(hipEventRecord(ev[2], st));
        rc = launch_f32<EPI_PLAIN>(hmid, F, m, tab, 2, 2, H, F, out, H, R, nseg, st);
    }
    if (rc != MOE_OK) return rc;
    if (ev) MOE_HIP(hipEventRecord(ev[3], st));
    return MOE_OK;
}

extern "C" int moe_expert_ffn(const void* recv, int32_t R, const int32_t* seg_offset, const int32_t* seg_expert,
                              int32_t nseg, const moe_expert_w* experts, int32_t n_local, int32_t H, int32_t F,
                              int32_t act, int32_t dtype, void* out, void* workspace, size_t workspace_bytes,
                              void* stream) {
    return ffn_impl(recv, R, seg_offset, seg_expert, nseg, experts, n_local, H, F, act, dtype, out, workspace,
                    workspace_bytes, reinterpret_cast<hipStream_t>(stream), nullptr);
}

extern "C" int moe_expert_ffn_timed(const void* recv, int32_t R, const int32_t* seg_offset, const int32_t* seg_expert,
                                    int32_t nseg, const moe_expert_w* experts, int32_t n_local, int32_t H, int32_t F,
                                    int32_t act, int32_t dtype, void* out, void* workspace, size_t workspace_bytes,
                                    void* stream, float* ms_out) {
    if (!ms_out) return moe_set_error(MOE_EINVAL, "moe_expert_ffn_timed: ms_out is NULL");
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    hipEvent_t ev[4] = {nullptr, nullptr, nullptr, nullptr};
    int rc = MOE_OK;
    for (int i = 0; i < 4 && rc == MOE_OK; ++i)
        if (hipEventCreate(&ev[i]) != hipSuccess) rc = moe_set_error(MOE_EHIP, "hipEventCreate failed");
    if (rc == MOE_OK)
        rc = ffn_impl(recv, R, seg_offset, seg_expert, nseg, experts, n_local, H, F, act, dtype, out, workspace,
                      workspace_bytes, st, ev);
    if (rc == MOE_OK && hipEventSynchronize(ev[3]) != hipSuccess) rc = moe_set_error(MOE_EHIP, "hipEventSynchronize failed");
    for (int i = 0; i < 3 && rc == MOE_OK; ++i)
        if (hipEventElapsedTime(&ms_out[i], ev[i], ev[i + 1]) != hipSuccess) rc = moe_set_error(MOE_EHIP, "hipEventElapsedTime failed");
    for (int i = 0; i < 4; ++i)
        if (ev[i]) (void)hipEventDestroy(ev[i]);
    return rc;
}

extern "C" int moe_diag_ffn_phases(const void* recv, int32_t R, const int32_t* seg_offset, const int32_t* seg_expert,
                                   int32_t nseg, const moe_expert_w* experts, int32_t n_local, int32_t H, int32_t F,
                                   int32_t act, int32_t dtype, void* out, void* workspace, size_t workspace_bytes,
                                   int32_t which_gemm, int64_t* marks, size_t marks_len, void* stream) {
    if (!marks || (which_gemm != 1 && which_gemm != 2))
        return moe_set_error(MOE_EINVAL, "moe_diag_ffn_phases: marks is NULL or which_gemm is not 1 or 2");
    static_assert(sizeof(long long) == sizeof(int64_t), "marks are 64-bit");
    return ffn_impl(recv, R, seg_offset, seg_expert, nseg, experts, n_local, H, F, act, dtype, out, workspace,
                    workspace_bytes, reinterpret_cast<hipStream_t>(stream), nullptr, which_gemm,
                    reinterpret_cast<long long*>(marks), marks_len);
}
