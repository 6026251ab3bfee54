/*
 * aurora_moe.h - C ABI of the MI355X (gfx950) MoE-layer share library.
 *
 * One GPU's share of an expert-parallel MoE layer, in the order the paper's
 * Sec. 2.1 lists the phases: Gate -> first all-to-all (only its buffer side is
 * built: the send buffer, laid out in the transmission order planned by
 * Sec. 4.2) -> expert FFN -> second all-to-all (only its layout contract) ->
 * Aggregation; plus the host-side planners of Sec. 4.2 / 5.2 (transmission
 * order; Appendix A rounds as a chunk plan for the send buffer), Sec. 5.1 (GPU
 * assignment), Sec. 6.2 and 7.2 (expert colocation by bottleneck matching) and
 * the inference-time expressions of Sec. 4.1 and 6.1.
 *
 * Conventions
 *   - Every function returns MOE_OK (0) or a negative moe_status; nothing
 *     throws, aborts or exits.  moe_last_error() gives a thread-local detail
 *     string for the last failing call on the calling thread.
 *   - "device" pointers are HIP device memory owned by the caller; "host"
 *     pointers are ordinary host memory.  The library never frees or keeps a
 *     caller's pointer beyond the call (device work is asynchronous on
 *     `stream`, so device buffers must stay alive until that work is done).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Device entry points only enqueue work: no synchronisation, no
 *     device-to-host copy.  The transmission order is planned offline from
 *     historical statistics (Sec. 2.4), so it is an input, never waited for.
 *   - Matrices are row-major.  A "slot" is a (token, choice) pair, id t*k + j.
 *   - dtype: MOE_F32 (0) = IEEE fp32 storage; MOE_BF16 (1) = bfloat16 storage.
 *     Accumulation is fp64 in the gate (indices must not depend on summation
 *     order) and fp32 elsewhere.
 *   - Arguments are validated before anything is launched: NULL where not
 *     allowed / non-positive sizes -> MOE_EINVAL; inconsistent sizes (k > E,
 *     limits exceeded, maps out of range, dest_order not a permutation)
 *     -> MOE_ESHAPE; unknown dtype/act -> MOE_EDTYPE; row size not a multiple of
 *     16 bytes or a pointer not 16-byte aligned -> MOE_EALIGN; a failing HIP call
 *     -> MOE_EHIP (hipGetErrorString in moe_last_error()).
 *   - Limits: E <= 256, G <= 64, k <= 16, T*k < 2^31.
 */
#ifndef AURORA_MOE_H
#define AURORA_MOE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    MOE_OK = 0,
    MOE_EINVAL = -1,
    MOE_ESHAPE = -2,
    MOE_EDTYPE = -3,
    MOE_EALIGN = -4,
    MOE_ENOMEM = -5,
    MOE_EHIP = -6,
    MOE_EINTERNAL = -7
} moe_status;

enum { MOE_F32 = 0, MOE_BF16 = 1 };
enum { MOE_ACT_SILU_MLP = 0, MOE_ACT_GELU_MLP = 1, MOE_ACT_SWIGLU = 2 };

/* Name of a status code; static storage. */
const char* moe_status_str(int status);
/* Detail of the last error on this thread; static thread-local storage, "" if none. */
const char* moe_last_error(void);

/* Shape of one GPU's share (notation of Sec. 4, Table 1, with n = G GPUs). */
typedef struct {
    int32_t T;        /* local tokens */
    int32_t H;        /* hidden size */
    int32_t E;        /* routed experts in the layer */
    int32_t k;        /* experts per token ("one or two" in Sec. 2.1; any 1..16 here) */
    int32_t G;        /* GPUs the experts are spread over */
    int32_t dtype;    /* storage type of x, Wg, send/return buffers, y */
    int32_t renorm;   /* 0: combine weight = softmax probability; 1: divided by the sum of the k chosen */
    int32_t capacity; /* rows kept per expert on this source GPU; 0 = unlimited */
} moe_shape;

/* Opaque per-shape context.  Owns small device scratch for the counting sort
 * (4 bytes per slot plus a few KB), allocated once in moe_ctx_create on the
 * current device.  A context must not be used by two streams at once.
 *
 * moe_traffic and moe_dispatch both need the rank of every slot inside its
 * expert.  By default each computes it for itself, so a dispatch never depends
 * on what an earlier call saw.  moe_ctx_set_rank_reuse(ctx, 1) lets a
 * moe_dispatch / moe_dispatch_chunks reuse the ranks of a moe_traffic when that
 * moe_traffic was given the SAME topk_idx pointer and no moe_route, dispatch,
 * moe_ctx_invalidate or moe_ctx_set_rank_reuse came in between; the dispatch is
 * then a single kernel.  The ranks are used once: the next dispatch computes its
 * own unless another moe_traffic precedes it.  With reuse on, the caller
 * promises that the indices at that address are not rewritten between the two
 * calls by anything but this library (the check is on the pointer value, which
 * an allocator may hand out again), and that the two calls are captured into a
 * HIP graph together or not at all.  moe_ctx_invalidate drops the ranks. */
typedef struct moe_ctx moe_ctx;
int moe_ctx_create(moe_ctx** out, const moe_shape* shape);
int moe_ctx_set_rank_reuse(moe_ctx* ctx, int32_t enable);
int moe_ctx_invalidate(moe_ctx* ctx);
int moe_ctx_destroy(moe_ctx* ctx); /* NULL is accepted */

/* Gate (Sec. 2.1): logit[t,e] = sum_h x[t,h]*Wg[e,h] (+ gate_bias[e]); the k
 * largest logits are chosen, listed by descending logit, equal logits resolved
 * to the lower expert index; weight = softmax over all E logits at the chosen
 * expert (divided by the sum of the k weights when renorm = 1).
 *   x          device [T,H] dtype      Wg        device [E,H] dtype
 *   gate_bias  device [E] fp32, may be NULL
 *   topk_idx   device [T,k] int32 out  topk_w    device [T,k] fp32 out
 * Logits are accumulated in fp64, so the indices equal those of an exact
 * evaluation whenever the k-th and (k+1)-th logits differ by more than a few
 * ulps of fp64. */
int moe_route(moe_ctx* ctx, const void* x, const void* Wg, const float* gate_bias,
              int32_t* topk_idx, float* topk_w, void* stream);

/* Row g of the first all-to-all's traffic matrix D_N (Sec. 4: d_gj = tokens GPU
 * g sends to GPU j), in slots, after the capacity rule: a slot is kept iff fewer
 * than `capacity` slots with a smaller id chose the same expert.
 *   topk_idx       device [T,k]      expert_to_gpu  HOST [E], values in [0,G)
 *   expert_count   device [E] out: kept slots per expert
 *   dest_count     device [G] out: kept slots per destination GPU (self included)
 *   n_dropped      device [1] out */
int moe_traffic(moe_ctx* ctx, const int32_t* topk_idx, const int32_t* expert_to_gpu,
                int32_t* expert_count, int32_t* dest_count, int32_t* n_dropped, void* stream);

/* Buffer layer in the planned transmission order (Sec. 3, "Communication
 * scheduling"): kept slots are copied into the send buffer destination by
 * destination in `dest_order`; inside a destination expert by expert (ascending
 * id); inside an expert by ascending slot id.
 *   x            device [T,H] dtype     topk_idx  device [T,k]
 *   expert_to_gpu HOST [E]              dest_order HOST [G], a permutation of 0..G-1
 *   send_buf     device [T*k,H] dtype out (rows beyond the kept count untouched)
 *   slot_to_row  device [T*k] out, -1 for a dropped slot
 *   row_to_slot  device [T*k] out (entries beyond the kept count untouched)
 *   seg_offset   device [E+1] out: first row of each (destination, expert) segment in send order
 *   seg_expert   device [E] out: expert id of each segment */
int moe_dispatch(moe_ctx* ctx, const void* x, const int32_t* topk_idx, const int32_t* expert_to_gpu,
                 const int32_t* dest_order, void* send_buf, int32_t* slot_to_row,
                 int32_t* row_to_slot, int32_t* seg_offset, int32_t* seg_expert, void* stream);

/* moe_dispatch for callers that cannot allocate device memory: code that runs
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * It needs no context: the scratch of the counting sort (block histograms,
 * per-expert totals, 4 bytes per slot) lives in a static device array of
 * 5 MiB + 1 KiB that every GPU the library runs on holds until the process ends.
 * The call allocates and frees nothing, on the device or through any library.
 *   shape        HOST, the checks of moe_ctx_create apply; additionally
 *                T*k <= 1048576 slots, else MOE_ESHAPE (use moe_dispatch)
 *   other arguments, layouts and results exactly as moe_dispatch
 * The ranks are always computed by the call itself (nothing is reused from
 * moe_traffic).  All calls on one GPU share that GPU's array: two calls that
 * overlap in time on one GPU (two streams, two threads) race; calls on one stream
 * are ordered by the stream.  Nothing in the array needs clearing between calls:
 * each call writes every word it later reads.  The array's device address is
 * looked up on the first call on each device (current device = the stream's). */
int moe_dispatch_noalloc(const moe_shape* shape, const void* x, const int32_t* topk_idx,
                         const int32_t* expert_to_gpu, const int32_t* dest_order, void* send_buf,
                         int32_t* slot_to_row, int32_t* row_to_slot, int32_t* seg_offset, int32_t* seg_expert,
                         void* stream);

/* A preemptive send plan (Appendix A; see aurora_chunks): chunk c carries the
 * next chunk_rows[c] slots of destination chunk_dest[c].  The slots of a
 * destination form one sequence - expert by expert (ascending id), inside an
 * expert by ascending slot id, the order moe_dispatch uses - and a chunk gets
 * fewer slots (possibly none) when the sequence runs out; a chunk whose dest is
 * no GPU stays empty; negative row counts count as 0.  Whatever the plan does not
 * cover follows after the last chunk, one left-over chunk per destination in
 * ascending GPU id (so the plan may come from historical statistics, Sec. 2.4).
 *   expert_to_gpu HOST [E]; chunk_dest, chunk_rows HOST [n_chunks], n_chunks <= 4096
 * The plan owns device tables that a dispatch rewrites: dispatches that share a
 * plan must not overlap.  Creation and destruction synchronise with the device. */
typedef struct moe_chunk_plan moe_chunk_plan;
int moe_chunk_plan_create(moe_ctx* ctx, const int32_t* expert_to_gpu, int32_t n_chunks, const int32_t* chunk_dest,
                          const int32_t* chunk_rows, moe_chunk_plan** out);
int moe_chunk_plan_destroy(moe_chunk_plan* plan);

/* moe_dispatch for a preemptive plan: the send buffer is the chunks in plan
 * order, then the left-over chunks.  With nc = n_chunks + G:
 *   chunk_offset  device [nc+1] out: first send row of each chunk, then the row count
 *   piece_offset  device [nc+E+1] out, piece_expert device [nc+E] out, n_pieces device [1] out:
 *                 a piece is a maximal run of rows of one chunk and one expert, listed in
 *                 buffer order; piece_offset[n_pieces] is the row count
 * Other arguments, rank reuse and error behaviour as for moe_dispatch. */
int moe_dispatch_chunks(moe_ctx* ctx, const moe_chunk_plan* plan, const void* x, const int32_t* topk_idx,
                        void* send_buf, int32_t* slot_to_row, int32_t* row_to_slot, int32_t* chunk_offset,
                        int32_t* piece_offset, int32_t* piece_expert, int32_t* n_pieces, void* stream);

/* One expert's weights, stored [out,in] row-major in `dtype`, device memory. */
typedef struct {
    const void* w1;     /* [F,H]: the only up-projection (MLP) or the gate projection (SwiGLU) */
    const void* w_up;   /* [F,H] for SwiGLU, NULL otherwise */
    const void* w_down; /* [H,F] */
} moe_expert_w;

/* Bytes of device workspace moe_expert_ffn needs for up to R_max rows (the
 * [R,F] intermediate, a tile map of about 1 KiB per 64 rows plus 1 MiB and, for
 * bf16, 64 MiB of fp32 partial tiles); 0 if an argument is invalid. */
size_t moe_ffn_workspace_bytes(int32_t R_max, int32_t H, int32_t F, int32_t act, int32_t dtype);

/* Expert FFN (Sec. 2.1) over the rows this GPU received: rows
 * [seg_offset[i], seg_offset[i+1]) go through local expert seg_expert[i].
 * Input and output rows have the same size (Sec. 2.2), so `out` mirrors `recv`.
 *   act 0: Wd.silu(W1.x)   1: Wd.gelu_tanh(W1.x)   2: Wd.(silu(W1.x) * (Wu.x))
 *   recv        device [R,H] dtype       R  rows in recv/out (>= seg_offset[nseg])
 *   seg_offset  device [nseg+1] int32, non-decreasing, seg_offset[0] >= 0
 *   seg_expert  device [nseg] int32 in [0,n_local)
 *   experts     HOST [n_local], n_local <= 64
 *   out         device [R,H] dtype; rows outside every segment are left untouched
 *   workspace   device, >= moe_ffn_workspace_bytes(R,H,F,act,dtype), 256-byte aligned
 * The segments of one expert need not be adjacent and may be short: bf16 tiles
 * are filled from all of an expert's segments in index order (as long as
 * R * max(H,F) * 2 bytes is at most 4 GiB; beyond that only adjacent segments of
 * an expert share tiles).
 * bf16: H and F must be multiples of 128 and H*F*2 bytes (one weight matrix) at
 * most 4 GiB, else MOE_ESHAPE; the [R,F] intermediate is rounded to bf16 once.
 * fp32: any sizes with H, F multiples of 4. */
int moe_expert_ffn(const void* recv, int32_t R, const int32_t* seg_offset, const int32_t* seg_expert,
                   int32_t nseg, const moe_expert_w* experts, int32_t n_local, int32_t H, int32_t F,
                   int32_t act, int32_t dtype, void* out, void* workspace, size_t workspace_bytes,
                   void* stream);

/* Diagnostic twin of moe_expert_ffn (same arguments, same result): records HIP
 * events on `stream` around each of its kernels, WAITS for the last one, and
 * returns the durations in milliseconds in ms_out (HOST [3]): tile map, first GEMM
 * with the activation (Sec. 2.1's FFN up-projection), second GEMM.  For measurement
 * only: unlike every other device entry point it synchronises with the host. */
int moe_expert_ffn_timed(const void* recv, int32_t R, const int32_t* seg_offset, const int32_t* seg_expert,
                         int32_t nseg, const moe_expert_w* experts, int32_t n_local, int32_t H, int32_t F,
                         int32_t act, int32_t dtype, void* out, void* workspace, size_t workspace_bytes,
                         void* stream, float* ms_out);

/* Aggregation (Sec. 2.1): y[t] = sum_j topk_w[t,j] * ret[slot_to_row[t*k+j]] over
 * kept slots (+ shared_out[t]).  `ret` is in send-buffer row order: the second
 * all-to-all reverses the first with equal sizes (Sec. 2.2).
 *   ret         device [T*k,H] dtype     slot_to_row device [T*k]
 *   topk_w      device [T,k] fp32        shared_out  device [T,H] dtype or NULL
 *   y           device [T,H] dtype out (fp32 accumulation, rounded once) */
int moe_combine(moe_ctx* ctx, const void* ret, const int32_t* slot_to_row, const float* topk_w,
                const void* shared_out, void* y, void* stream);

/* ------------------------------------------------------------------ diagnostics
 * Host-side self checks used by the CPU tests; they launch nothing and are not needed to run the layer.
 * Not thread-safe beyond what the rest of the library is: the FFN launch path keeps the number of compute
 * units of the device it first ran on and the "LDS size raised" marks in process-wide statics, i.e. it
 * assumes one kind of device per process. */

/* Tile numbering and tail plan of the bf16 FFN GEMM for a tiles_m x tiles_n grid with nk k-tiles (nk even)
 * on ncu compute units: checks that every tile is produced exactly once, whole or as pieces that cover its
 * k-tiles exactly once.  Returns the number of pieces a tail tile is cut into (1 = no tail), or a negative
 * moe_status. */
int moe_selfcheck_tile_order(int32_t tiles_m, int32_t tiles_n, int32_t ncu, int32_t nk);

/* Plan of the weight-streaming FFN kernels (shares of at most 64 rows) for `total` tiles of `ns` stages of K on
 * ncu compute units: checks that the pieces cover the stages exactly once, are at least two stages long and fit
 * the launch.  Returns the number of pieces per tile (1 = whole tiles), or a negative moe_status. */
int moe_selfcheck_skinny_plan(int32_t total, int32_t ncu, int32_t ns);

/* How the scatter kernels share rows of row16 16-byte units among waves for k slots per token: out3 (HOST) =
 * {tokens per wave, log2 of the 1 KB wave-loads per row when several tokens share a wave, 8 KB pieces per row};
 * checks that the rows fit a wave's loads, that every slot has a lane and that the pieces cover the row. */
int moe_selfcheck_row_geometry(int32_t row16, int32_t k, int32_t* out3);

/* Tile map of the FFN for a segment list (HOST seg_offset [nseg+1], seg_expert [nseg]; R rows, tiles of bm
 * rows, n_local experts; gather = chain the segments of an expert into full tiles): runs the steps of the
 * device kernel on the host and checks that every row of every non-empty segment of a known expert lies in
 * exactly one tile of that expert.  Returns the number of tiles or a negative moe_status. */
int moe_selfcheck_tile_map(const int32_t* seg_offset, const int32_t* seg_expert, int32_t nseg, int32_t R, int32_t bm,
                           int32_t n_local, int32_t gather);

/* Reference measurements of the device (used by bench.py's box_reference; both record HIP events on `stream`
 * around their one kernel, WAIT for it and return its duration in milliseconds in ms_out, HOST [1]).
 *
 * moe_diag_mfma_only: n_blocks blocks of 4 waves, every wave issues iters x 16 independent
 * v_mfma_f32_32x32x16_bf16 (the FFN kernel's 4 x 4 register blocking) on operands that stay in registers: what
 * the matrix cores sustain with no operand traffic at all.  sink: device [n_blocks*256] fp32 out (sums, so
 * that the work cannot be dropped).  flop_out HOST [1]: the floating-point operations issued.
 * iters a multiple of 4 in [4, 2^24], 1 <= n_blocks <= 65536.
 *
 * moe_diag_copy_1r2w: dst0 = dst1 = src, `bytes` (a multiple of 16) read once and written twice with 16-byte
 * accesses, a wave per 8 KB: the traffic shape of a top-2 send buffer without any indexing.  The kernel is
 * launched `reps` times (1..1000) back to back between the two events; ms_out is the average per launch. */
/* moe_expert_ffn with one of its two GEMMs (which_gemm = 1 or 2) run as a second instantiation of the same kernel
 * template that reads the 100 MHz wall clock: marks[(b * 4 + w) * 4 + i] (DEVICE, zeroed by the caller) is the
 * clock of wave w of block b at 0 start, 1 first operands in LDS (loop about to start), 2 loop done, 3 end; a block
 * that found no tile writes mark 0 only.  marks_len >= (((R + 255) / 256 + nseg) * tiles_n + 256) * 16 elements with
 * tiles_n = ceil(N / 128) for the first GEMM of a SwiGLU expert (N = F), ceil(F / 256) for the other activations,
 * ceil(H / 256) for the second GEMM; MOE_ESHAPE otherwise, and for fp32 or shares of at most 64 rows (other
 * kernels).  Everything else as moe_expert_ffn. */
int moe_diag_ffn_phases(const void* recv, int32_t R, const int32_t* seg_offset, const int32_t* seg_expert, int32_t nseg,
                        const moe_expert_w* experts, int32_t n_local, int32_t H, int32_t F, int32_t act, int32_t dtype,
                        void* out, void* workspace, size_t workspace_bytes, int32_t which_gemm, int64_t* marks,
                        size_t marks_len, void* stream);

/* moe_route with the 100 MHz wall clock read at the phase boundaries of the bf16 kernel (the ordinary kernel
 * contains none of this).  marks: DEVICE, marks_len >= (T / 16 + 1) * 128 elements, zeroed by the caller; on return
 * (after the stream has been synchronised) marks[(b * 16 + w) * 8 + i] is the clock of wave w of block b at
 * boundary i: 0 start, 1 its part of the streaming loop done, 2 all waves done, 3 partial tiles added,
 * 4 selected, 5 end (0 for a block that had no token to evaluate again: it ends at 4); marks[b * 128 + 6] = tokens
 * that block evaluated again.  *tokens_per_block (HOST) = tokens per block, i.e. ceil(T / that) blocks; 0 when the
 * shape takes the fp64 kernel, which writes no marks.  Outputs as moe_route.  MOE_ESHAPE when marks is too short. */
int moe_diag_route_phases(moe_ctx* ctx, const void* x, const void* Wg, const float* gate_bias, int32_t* topk_idx,
                          float* topk_w, int64_t* marks, size_t marks_len, int32_t* tokens_per_block, void* stream);

/* moe_diag_mfma_run_sum: what the gate's fast pass builds on, exposed so that a test can hold the hardware to
 * the error model the gate assumes: d[t][i][j] = a chain of `run` v_mfma_f32_16x16x32_bf16, the first with a
 * zero accumulator, i.e. the sum over k < 32 run of the exact products a[t][i][k] * b[t][j][k] as the matrix core
 * forms and rounds it.
 *   a, b  device [n_tiles][16][32 run] bf16 (16-byte aligned)    d  device [n_tiles][16][16] fp32 out
 *   1 <= run <= 64.  Asynchronous on `stream` like the layer's entry points. */
int moe_diag_mfma_run_sum(const void* a, const void* b, float* d, int32_t n_tiles, int32_t run, void* stream);

int moe_diag_mfma_only(int32_t n_blocks, int32_t iters, float* sink, void* stream, float* ms_out, double* flop_out);
int moe_diag_copy_1r2w(const void* src, void* dst0, void* dst1, size_t bytes, int32_t reps, void* stream, float* ms_out);

/* ------------------------------------------------------------------ host planners */

/* Result of aurora_order; arrays are owned by the library until
 * aurora_schedule_free (which also zeroes the struct). */
typedef struct {
    int32_t n;
    int32_t n_rounds;
    double* duration;        /* [n_rounds] length of each round */
    int32_t* dst;            /* [n_rounds*n] receiver of GPU i in round r, -1 = idle */
    int32_t* dest_order;     /* [n*n] row i: the order in which GPU i sends to all n destinations when whole
                                flows go out back to back; the row to hand to moe_dispatch (non-empty flows,
                                then empty ones, then i itself) */
    int32_t* alg1_order;     /* [n*n] the same for Algorithm 1's plan: real flows by planned start */
    double* start;           /* [n*n] Algorithm 1: planned start of flow i->j, -1 if empty */
    double bmax;             /* Theorem 2 / Theorem 4 lower bound */
    double port_bound;       /* looser bound max(sum_j d_ij/B_i, sum_i d_ij/B_j) */
    double makespan_rounds;  /* sum of round durations (== bmax up to rounding) */
    double makespan_order;   /* Algorithm 1: end of the last flow in its plan (flows wait for their slot) */
    double order_time;       /* aurora_simulate of dest_order */
    double candidate_time[4];/* aurora_simulate of the four candidate orders (see below) */
    int32_t order_source;    /* which candidate dest_order grew from: 0..3 */
} aurora_schedule;

/* Transmission order of one all-to-all (Sec. 4.2 Theorem 2 and Algorithm 1;
 * Sec. 5.2 Theorem 4 / Appendix B for per-GPU rates).
 *   n   GPUs (1..64)      D  HOST [n*n] tokens i->j, diagonal ignored, entries >= 0
 *   B   HOST [n] link rates > 0, or NULL for all 1
 * Traffic is scaled to p_ij = d_ij / min(B_i,B_j).  `rounds` is the schedule of
 * Appendix A: the padded matrix is decomposed into permutations, in each round
 * every GPU sends to a distinct GPU; it attains bmax (aurora_chunks turns it
 * into a send plan).  `alg1_order`, `start`, `makespan_order` are a greedy
 * reading of Algorithm 1 on whole flows: the bottleneck GPU's binding side back
 * to back from time 0, then GPUs by remaining traffic, each flow placed in the
 * earliest gap free at both ends.  A send buffer that holds whole flows is sent
 * back to back, without the waits of that plan, so `dest_order` is chosen by
 * what aurora_simulate gives: the best of (0) Algorithm 1's order, (1)
 * destinations by their first round in the Appendix A schedule, (2) an order
 * built while playing the transfer forward (an idle GPU starts the flow whose
 * receiver has the fewest incoming flows, then the largest flow), (3) the shifted
 * order i -> i+1, i+2, ... (mod n), contention-free when all flows are equal;
 * then neighbouring
 * flows of a GPU are exchanged while that shortens the simulated time (at most
 * 64 n trials).  order_time >= port_bound always, >= bmax for equal rates. */
int aurora_order(int32_t n, const int64_t* D, const double* B, aurora_schedule* out);
void aurora_schedule_free(aurora_schedule* s);

/* The send plan of GPU g under the rounds of `s` (Appendix A: in every time slot a
 * GPU sends to one GPU; a flow may be served in several slots): one chunk per
 * round in which g sends real traffic, in round order.  A chunk carries whole
 * tokens: the cumulative amount sent to that destination by the end of the
 * round, rounded down, minus what earlier chunks carried; the counts of a
 * destination add up to d_g,dest.  D and B must be the ones `s` was made from.
 *   chunk_dest, chunk_rows  HOST [s->n_rounds] out     n_chunks  HOST [1] out */
int aurora_chunks(const aurora_schedule* s, const int64_t* D, const double* B, int32_t g, int32_t* chunk_dest,
                  int32_t* chunk_rows, int32_t* n_chunks);

/* Completion time of the all-to-all on the big-switch model (Sec. 2.4) when GPU
 * i sends to order[i*n .. i*n+n) one destination after another; a receiver with
 * m incoming flows gives each B_recv/m, a flow runs at min(B_send, share). */
int aurora_simulate(int32_t n, const int64_t* D, const double* B, const int32_t* order, double* time_out);

/* Expert colocation of two models (Sec. 6.2, Case II): edge weight
 * max(a_i + b_j, a_{n+i} + b_{n+j}) from the off-diagonal row (send) and column
 * (receive) sums of Da and Db; minimise the largest weight over matchings that
 * give every expert of a (na <= nb) a distinct expert of b.  Binary search over
 * the sorted weights with Hopcroft-Karp as the feasibility test.
 *   Da HOST [na*na], Db HOST [nb*nb], entries >= 0;  pair HOST [na] out;  bottleneck HOST [1] out */
int colocate_match(int32_t na, int32_t nb, const int64_t* Da, const int64_t* Db, int32_t* pair,
                   double* bottleneck);

/* GPU assignment on a heterogeneous cluster (Sec. 5.1, Theorem 3): experts sorted
 * by the tokens they process, descending, meet GPUs sorted by performance,
 * descending; ties keep the lower index first.  One expert per GPU.
 *   load HOST [n] >= 0, perf HOST [n] > 0, expert_to_gpu HOST [n] out; n <= 256 */
int aurora_assign(int32_t n, const int64_t* load, const double* perf, int32_t* expert_to_gpu);

/* Bottleneck assignment (the matching of Sec. 6.2 Case II on an arbitrary table):
 * one item per GPU, minimising the largest W[g*n + item]; binary search over the
 * sorted weights with Hopcroft-Karp as the feasibility test.
 *   W HOST [n*n] finite, item_of_gpu HOST [n] out, bottleneck HOST [1] out; n <= 256 */
int aurora_bottleneck_assign(int32_t n, const double* W, int32_t* item_of_gpu, double* bottleneck);

/* Colocation on a heterogeneous cluster by the decoupled method of Sec. 7.2: first
 * colocate_match on the traffic alone, then GPUs against the pairs found, the edge
 * weight being the inference time of the pair on that GPU.  The paper prints no
 * formula for that time, so it is an input:
 *   time3 HOST [n*n*n] finite: time3[(g*n + i)*n + j] = GPU g hosting expert i of a and j of b
 *   pair HOST [n] out (expert of b with expert i of a), gpu_of_pair HOST [n] out,
 *   value HOST [1] out = the largest time3 used; n <= 64 */
int colocate_hetero_match(int32_t n, const int64_t* Da, const int64_t* Db, const double* time3, int32_t* pair,
                          int32_t* gpu_of_pair, double* value);

/* Eqn. 1 (Sec. 4.1): max_i(G_i + N_i) + max_j(F_j + C_j) + max_k A_k over the n GPUs.
 *   G, N, F, C, A HOST [n] durations; t_out HOST [1] */
int aurora_layer_time(int32_t n, const double* G, const double* N, const double* F, const double* C,
                      const double* A, double* t_out);

/* End times of the components of two colocated models (Sec. 6.1, Table 2) and the
 * inference time t = E_{A^b} + |G^a| (Eqn. 4).  Na, Nb: stand-alone durations of the
 * first all-to-alls, NaNb: their aggregated duration; the second all-to-alls are the
 * first ones reversed and take the same durations.  A communication component ends at
 * the later of the table's aggregated duration and its earliest start plus its own
 * duration (read as absolute times the table's entries could end before the component
 * may start).  All inputs finite and >= 0. */
typedef struct {
    double Gb, Na, Fa, Nb, Fb, Ca, Aa, Cb, Ab, Ga, t;
} aurora_coloc_times;
int aurora_colocated_time(double Ga, double Gb, double Fa, double Fb, double Aa, double Ab, double Na, double Nb,
                          double NaNb, aurora_coloc_times* out);

#ifdef __cplusplus
}
#endif
#endif /* AURORA_MOE_H */
