/*
 * flmoe - MoE expert-parallel dispatch/combine token shuffle for MI355X (gfx950).
 *
 * C ABI of the shared library.  One GPU hosts the whole expert-parallel group as
 * simulated ranks; the "fabric" between ranks is a device-side copy whose
 * completion is signalled only through per-source arrival counters (the
 * paper's ImmCounter idea, section TransferEngine / Completion Notification:
 * a counter advances when payload has been delivered, a receiver compares it
 * with what the exchanged counts tell it to expect, and nothing else orders
 * transfers).
 *
 * Problem statement (section MoE Dispatch/Combine, Architecture): N ranks host E
 * experts (expert e lives on rank e / (E/N)); every rank holds up to T tokens of
 * H hidden values and routes each to K distinct experts (the paper's R).
 *
 * Conventions for every entry point
 *   - All tensor arguments are DEVICE pointers unless marked "host".  The library
 *     never allocates or frees device memory: inputs, outputs and the workspace
 *     belong to the caller and must stay valid until fl_moe_destroy.
 *   - Device pointers must be 16-byte aligned, hidden*2 must be a multiple of 16,
 *     the e4m3 dispatch needs hidden % 128 == 0.
 *   - Tensors are rank-major: element [r] of the leading dimension belongs to
 *     simulated rank r.  Each call acts for ranks [rank_begin, rank_begin +
 *     rank_count); code acting for rank r reads only rank r's tensors and
 *     receive buffers, and writes other ranks' memory only through the fabric
 *     copy and its counters.  Ranks on separate GPUs would each pass rank_count = 1
 *     (their calls then run at the same time, each on its own device).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  The
 *     five shuffle calls only enqueue kernels: they never synchronise, never
 *     allocate, and can be captured in a HIP graph.  A call that moves several GB
 *     enqueues its kernels once per group of ranks (very large launches run
 *     measurably slower than the same work in launches of about a GB), except
 *     with FL_FLAG_PROGRESSIVE_RECV.
 *   - One step = the five calls once each, in the order layout, dispatch_send,
 *     dispatch_recv, combine_send, combine_reduce, with every rank of the group
 *     taking part in each.  The payload calls may be split over several launches
 *     by rank range.  fl_moe_layout is different: it waits INSIDE the call for every
 *     peer's counts, as ranks on separate GPUs wait for each other.  On one GPU the
 *     peers' layout calls must therefore be able to run at the same time: all ranks
 *     in one call (rank_count = N), or in calls on different streams; calls for
 *     part of the ranks one after another on ONE stream cannot complete (the first
 *     waits for counts that only the later ones would send).  A call whose peers
 *     never ran ends with FL_STATUS_TIMEOUT after the bounded wait, not with a hang.
 *   - A context is not thread-safe: its calls come from one host thread at a
 *     time.  Several contexts (each with its own workspace) are independent.
 *   - Return value: FL_OK or a negative FL_ERR_* for errors the host can see
 *     (nothing is enqueued then).  Errors found on the device (bad expert id,
 *     capacity overflow, arrival time-out) make the affected step a no-op on every
 *     rank and latch a bit that fl_moe_status reports; they never cause an
 *     out-of-bounds access or an unbounded wait.
 */
#ifndef FLMOE_H
#define FLMOE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define FL_OK 0
#define FL_ERR_INVALID_ARG (-1)
#define FL_ERR_ALIGNMENT (-2)
#define FL_ERR_WORKSPACE (-3)
#define FL_ERR_HIP (-4)
#define FL_ERR_STATIC_LIMIT (-5) /* fl_moe_layout_static: the configuration needs more scratch
                                    than FL_STATIC_SCRATCH_BYTES                             */

/* bits of the device status word */
#define FL_STATUS_BAD_INDEX 1 /* expert id outside [0,E) or repeated inside a token */
#define FL_STATUS_CAPACITY 2  /* a rank would receive more rows than its capacity    */
#define FL_STATUS_TIMEOUT 4   /* an arrival counter did not reach its expectation     */

#define FL_DTYPE_BF16 0
/* OCP E4M3 (finite-only) bytes plus one fp32 scale per 128 elements, quantised
 * by dispatch_send (workload of section Kernel Microbenchmarks: 7168 fp8 values
 * and 56 fp32 scaling factors per token).  Per block of 128: scale = max|x| / 448
 * (1 when the maximum is 0), code = e4m3(x / scale), round to nearest even,
 * saturating; both divisions IEEE fp32.  Non-finite inputs (the paper is silent; the
 * rule is applied as written): a NaN is skipped by the maximum and becomes the NaN
 * code 0x7f with its own sign, its neighbours are quantised as if it were absent; an
 * Inf makes the block's scale +Inf, every finite value of that block a signed zero and
 * every Inf the NaN code with its sign; a block of NaNs only has scale 1. */
#define FL_DTYPE_E4M3_BLOCK128 1

#define FL_FLAG_ZERO_PAD 1 /* dispatch_recv writes zeros into the padding rows between experts */
/* How senders and receivers are ordered.
 *
 * Default (neither flag below): the arrival counters are the only thing that orders a
 * sender and a receiver, the ImmCounter contract with no ordering assumed (section
 * TransferEngine, Completion Notification).  Send and receive calls of different ranks
 * may be issued on any streams, in any order, and may overlap in time.
 *   - A send call enqueues its payload kernels and, behind them in the same stream, a
 *     small kernel that adds each whole (sender, receiver) transfer to the receiver's
 *     counter with release semantics: it starts once the payload kernels have ended
 *     (the sender's own stream order, as a NIC posts the immediate after its WRITE),
 *     so the counter never runs ahead of the payload.
 *   - A receive call first enqueues a gate kernel of one wave per rank that polls the
 *     rank's counters with acquire semantics until every source has delivered what
 *     the exchanged counts promised (bounded: FL_STATUS_TIMEOUT), and behind it the
 *     receive kernel proper, on a full grid.  Waiting occupies one wave per rank.
 * What a rank still orders itself is its OWN five calls of a step, and one step after
 * the other (one stream per rank does that, or events).  That also covers the re-use of
 * the two staging buffers of a context (combine replies land in the senders' dispatch
 * send buffers, the dispatch receive buffers become the combine send buffers; the paper
 * puts a barrier before buffers are re-used, section Combine): rank d issues
 * combine_send after its dispatch_recv, whose gate passed only after EVERY peer's
 * announce kernel had run, and a peer's announce kernel runs only after all of that
 * peer's dispatch payload kernels have ended, so nobody reads a send buffer any more
 * when the first reply is written into it; and rank s issues the next step's
 * dispatch_send after its combine_reduce, whose gate passed only after every peer's
 * combine payload kernels had ended, so nobody reads a combine send buffer any more
 * when the next step's rows are written into it.  (On one GPU a waiting gate kernel
 * occupies its hardware queue: enqueue the sends of a phase before the receives that
 * wait for them whenever streams may share a queue.)
 *
 * FL_FLAG_STREAM_ORDERED: the caller promises that each send call precedes the matching
 * receive call in stream order (one stream, or events between streams).  The library
 * then launches no announce and no gate kernels (four launches fewer per step): one
 * wave of the last payload kernel of a send call advances the counters while other
 * waves may still be storing, so here the counters are bookkeeping that only the
 * kernel boundary makes trustworthy - they are still checked (bounded) by the
 * receivers, but they do not signal completion by themselves. */
#define FL_FLAG_STREAM_ORDERED 2
/* Every peer's receive buffer can be stored to directly, as between ranks of one
 * node (section Dispatch: within a node the send kernel pushes payloads over the
 * load/store interconnect instead of handing them to the NIC; here: always, all
 * simulated ranks live on one GPU).  The send calls then write each row and its
 * sidecar straight into the destination's receive buffer: no send buffer is
 * filled and no scatter kernel runs; the arrival counters advance as in the
 * staged path (by the announce kernel, inside the kernel that stores the payload
 * with FL_FLAG_STREAM_ORDERED, per workgroup with FL_FLAG_PROGRESSIVE_RECV).
 * Receivers, counters, capacities and every result
 * are unchanged; only the bytes moved per step shrink (one write per sent row
 * instead of write + read + write).  Combines with the other flags and
 * max_private_rows. */
#define FL_FLAG_PEER_PUSH 4
/* Combine with sender-side partial sums (section Comparison with DeepEP and the
 * prefill results of section Performance: pre-accumulating on the sending side
 * moves fewer bytes, at the price of bf16 precision between the two stages and of
 * a result that is no longer one fp32 sum in a fixed order).  NOT bit-identical
 * to the default combine; its own definition, which the oracle states the same way:
 *   partial(d) = bf16( fp32 fused multiply-add chain from +0, ascending k, of
 *                weights[k] * y over the token's experts hosted by rank d )
 *   out        = bf16( fp32 sum from +0 of float(partial(d)), ranks in the order
 *                of their first k )
 * The weights are applied on the expert ranks, so they travel with the tokens:
 * dispatch must be issued with fl_moe_dispatch_send_weighted, and every rank
 * answers each row it received with one row (D rows per step instead of P). */
#define FL_FLAG_PARTIAL_SUMS 8
/* Receivers that start on each source's rows as soon as that source has landed,
 * whatever the other sources do (not with FL_FLAG_STREAM_ORDERED).  Senders write their
 * payload through to memory with device-scope stores, wait for the acknowledgement and
 * every wave adds what it delivered, so a receiver sees a source complete as early as
 * possible; the receive kernels poll the counters themselves, invalidate their caches
 * whenever they come to rely on arrivals they had not seen before, and run on grids
 * capped to a fraction of the machine so that pollers can never keep senders from
 * being scheduled.  The form for receivers whose sources land far apart in time; on
 * one GPU, where all simulated senders finish together, it only costs.  A counter then
 * says "this transfer has landed", not "this sender has finished", so here the caller
 * must itself keep every dispatch call of a step before any combine_send, and every
 * combine call before the next step's dispatch_send (events between streams).  Its
 * visibility argument is about the hardware (a device-scope store that was
 * acknowledged is in memory; a cache invalidated after the counter was observed
 * cannot hold older bytes), not about the HIP memory model alone. */
#define FL_FLAG_PROGRESSIVE_RECV 16

#define FL_MAX_RANKS 64
#define FL_MAX_EXPERTS 1024
#define FL_MAX_TOPK 16
#define FL_MAX_EXPERTS_PER_RANK 256

typedef struct fl_moe_ctx fl_moe_ctx;

typedef struct fl_moe_config {
    int32_t n_ranks;        /* N, 1..FL_MAX_RANKS                                        */
    int32_t n_experts;      /* E, multiple of N, <= FL_MAX_EXPERTS                       */
    int32_t max_tokens;     /* T, upper bound of tokens per rank                         */
    int32_t top_k;          /* K, 1..min(E, FL_MAX_TOPK)                                 */
    int32_t hidden;         /* H, 8..2^20, 2*H a multiple of 16                           */
    int32_t dispatch_dtype; /* FL_DTYPE_*: payload type of dispatch; combine is bf16      */
    int32_t expert_align;   /* every local expert but the first starts on a multiple of
                               this many rows (the padding between experts that section
                               Dispatch leaves optional); >= 1                            */
    int32_t flags;          /* FL_FLAG_*                                                  */
    int64_t recv_capacity_rows;   /* per rank: deduplicated rows it can receive; 0 = N*T  */
    int64_t expert_capacity_rows; /* per rank: rows of its expert-major layout, padding
                                     included; 0 = N*T*min(K, E/N) + padding              */
    int64_t spin_limit;     /* polls of an arrival counter before FL_STATUS_TIMEOUT (a waiting wave
                               polls about every 2 us); 0 = default, about 2 s                    */
    int32_t max_private_rows; /* P: the first P rows a source sends to a destination go to fixed
                               private slots at the head of the destination's receive buffer, in a
                               scatter of their own that needs no exchanged counts; only the rows
                               beyond P are packed into the shared contiguous range (section
                               Dispatch, figure "Dispatch into private and contiguous buffers";
                               section Ablation: Private Buffer Size).  0 = one scatter into the
                               shared range; values above T act as T.  The receive buffer grows by
                               N*P rows per rank; recv_capacity_rows bounds the shared range only. */
    int32_t reserved;       /* must be 0 */
} fl_moe_config;

typedef struct fl_moe_sizes {
    size_t workspace_bytes;       /* device bytes fl_moe_create needs (256-byte aligned)  */
    int64_t recv_capacity_rows;   /* resolved capacities                                  */
    int64_t expert_capacity_rows; /* also the rank stride, in rows, of expert_x/expert_y  */
    int64_t send_capacity_rows;   /* T * min(K, N)                                        */
    int64_t x_row_bytes;          /* 2*H                                                  */
    int64_t wire_row_bytes;       /* bytes of one dispatched row in the send/receive
                                     buffers: 2*H, or H + 4*H/128 rounded up to 128 for e4m3 */
    int64_t expert_x_row_bytes;   /* 2*H or H                                             */
    int64_t scales_per_row;       /* 0 or H/128                                           */
    int64_t combine_row_bytes;    /* 2*H                                                  */
    int64_t private_rows;         /* resolved P = min(max_private_rows, T)                */
    int64_t recv_buffer_rows;     /* rows of one rank's dispatch receive buffer: N*P private
                                     slots, then recv_capacity_rows of shared range       */
} fl_moe_sizes;

/* Device pointers into the workspace, valid until fl_moe_destroy; contents are
 * those of the last fl_moe_layout on the stream.  All int32. */
typedef struct fl_moe_layout_view {
    const int32_t *counts;            /* C [N][E]    pairs per (source rank, expert)                 */
    const int32_t *dedup_counts;      /* M [N][N]    distinct tokens per (source, destination rank)   */
    const int32_t *tokens_per_expert; /* G [N][E/N]                                                   */
    const int32_t *send_off;          /* [N][N+1]  exclusive scan of M[s][.]                          */
    const int32_t *recv_off;          /* [N][N+1]  exclusive scan of M[.][d]: source s owns received
                                         rows [recv_off[d][s], recv_off[d][s+1]) of rank d; with
                                         max_private_rows = 0 these are also the rows of d's receive
                                         buffer, otherwise the first P of each source sit in its
                                         private slots and the rest in the shared range               */
    const int32_t *expert_off;        /* [N][E/N+1] first row of each local expert; last = end of rows */
    const int32_t *comb_off;          /* [N][N+1]  start of each peer's reply in the combine receive
                                         buffer of rank s                                              */
    const int32_t *comb_pos;          /* [N][T][K] row of pair (s,t,k) in that buffer                  */
    const int32_t *plan_ok;           /* [N] 1 when the step is valid for the rank                     */
} fl_moe_layout_view;

/* Test/diagnostic view of internal buffers (layouts are the library's own). */
typedef struct fl_moe_debug_view {
    void *buf_a;              /* per rank: dispatch send buffer / combine receive buffer  */
    void *buf_b;              /* per rank: dispatch receive buffer / combine send buffer  */
    int64_t buf_a_rank_bytes;
    int64_t buf_b_rank_bytes;
    uint32_t *arrive_route;   /* [N][N] route records received, [destination][source]      */
    uint32_t *epoch_route;    /* [N] number of layout calls of each rank                   */
    uint32_t *arrive_disp;    /* [N][N] monotone payload counters, [destination][source]:  */
    uint32_t *arrive_comb;    /*        16-byte units delivered, plus one per transfer     */
    uint32_t *expect_disp;    /* [N][N] what the receiver expects, from the counts it got  */
    uint32_t *expect_comb;
    int32_t *status;          /* the device status word                                    */
} fl_moe_debug_view;

/* Sizes and strides implied by a configuration.  Host only; no GPU needed. */
int fl_moe_query_sizes(const fl_moe_config *cfg /*host*/, fl_moe_sizes *out /*host*/);

/* Binds a context to a caller-owned device workspace of at least
 * sizes.workspace_bytes bytes and clears its counters (this call synchronises;
 * it is set-up, not part of the hot path).  The workspace must be 256-byte
 * aligned; when it is 2 MB aligned (large device allocations are) the big payload
 * buffers inside it start on 2 MB pages too, which the copy kernels measurably
 * like. */
int fl_moe_create(const fl_moe_config *cfg /*host*/, void *workspace, size_t workspace_bytes,
                  fl_moe_ctx **out /*host*/);
int fl_moe_destroy(fl_moe_ctx *ctx);

/* Step 1 (section Dispatch: count tokens per expert; section Architecture: peers
 * exchange per-expert counts to find a unique range in each contiguous receive
 * buffer).  indices [N][T][K] int32 expert ids, distinct within a token;
 * num_tokens [N] int32 (<= T).  For every rank in the range it counts pairs per
 * expert and distinct tokens per destination rank with LDS bit matrices and
 * popcount prefix scans (deterministic, no ticket atomics), pushes the counts to
 * every peer, and derives all offsets of the step from the counts it received.
 * Both arrays must stay unchanged until the step's combine_reduce has run.
 * `view` (host, may be NULL) receives pointers to the resulting tables. */
int fl_moe_layout(fl_moe_ctx *ctx, int rank_begin, int rank_count, const int32_t *indices,
                  const int32_t *num_tokens, fl_moe_layout_view *view /*host*/, void *stream);

/* fl_moe_layout for callers that cannot allocate device memory or hold a context:
 * code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  It needs no fl_moe_ctx and no workspace: the route records, message
 * counters and per-pair tables that fl_moe_layout keeps in the caller's workspace
 * live in an array of FL_STATIC_SCRATCH_BYTES bytes inside the library's device
 * image (every GPU the library runs on holds one copy until the process ends),
 * and the call itself allocates nothing (no hipMalloc / hipFree, no events, no host
 * allocation).  It acts for all cfg->n_ranks ranks in one launch and writes the
 * same tables, with the same contents, that fl_moe_layout's view points to, into
 * the caller's buffers:
 *   counts [N][E], dedup_counts [N][N], tokens_per_expert [N][E/N],
 *   send_off [N][N+1], recv_off [N][N+1], expert_off [N][E/N+1], comb_off [N][N+1],
 *   comb_pos [N][T][K], plan_ok [N], status [1] (the FL_STATUS_* bits of THIS call;
 *   0 when the step is valid) - all int32 device pointers, 4-byte aligned, non-NULL.
 * Capacities, expert_align, max_private_rows and the flags of cfg are honoured
 * as in fl_moe_layout (capacity overflow and bad expert ids clear plan_ok on every
 * rank and set the status bits).  Returns FL_ERR_STATIC_LIMIT, and enqueues
 * nothing, when the configuration's tables do not fit the array (it holds the
 * 32-rank, 256-expert, top-8 shape up to about 3000 tokens per rank).  The call
 * only enqueues kernels on `stream`; the scratch is cleared by a kernel of the
 * call, not by a memset.  The first call on each device looks up the array's
 * address (hipGetSymbolAddress); make that call outside graph capture.
 * Every call on one GPU uses that GPU's one array: calls that overlap in time on
 * the same GPU (different streams, or a graph replay racing an eager call) race
 * and give undefined tables; calls on one stream, or ordered by events, are fine. */
#define FL_STATIC_SCRATCH_BYTES (8u << 20)
typedef struct fl_moe_layout_out {
    int32_t *counts, *dedup_counts, *tokens_per_expert, *send_off, *recv_off, *expert_off,
        *comb_off, *comb_pos, *plan_ok, *status;
} fl_moe_layout_out;
int fl_moe_layout_static(const fl_moe_config *cfg /*host*/, const int32_t *indices,
                         const int32_t *num_tokens, const fl_moe_layout_out *out /*host*/,
                         void *stream);

/* Step 2 (section Dispatch: tokens are copied into send buffers, a contiguous
 * source per peer, then scattered).  x [N][T][H] bf16; all T rows of a rank
 * must be addressable (rows of absent tokens may be read, they are never used).
 * Packs one copy of each token per distinct destination rank (quantising to
 * e4m3 when configured), copies every (source, destination) segment into the
 * destination's receive buffer and announces every transfer, empty ones included,
 * on arrive_disp[destination][source]: its payload in 16-byte units plus one. */
int fl_moe_dispatch_send(fl_moe_ctx *ctx, int rank_begin, int rank_count, const void *x,
                         void *stream);

/* Step 2 for a context created with FL_FLAG_PARTIAL_SUMS (fl_moe_dispatch_send
 * returns FL_ERR_INVALID_ARG there, and this call does without the flag): the
 * same dispatch, and each copy's sidecar also carries weights [N][T][K] fp32 of
 * the token's experts on the destination rank, which forms the partial sum in
 * fl_moe_combine_send.  fl_moe_combine_reduce then only adds; it still takes the
 * weights pointer (unused, non-NULL). */
int fl_moe_dispatch_send_weighted(fl_moe_ctx *ctx, int rank_begin, int rank_count, const void *x,
                                  const float *weights, void *stream);

/* Step 2 for tokens the caller has already quantised (section Kernel
 * Microbenchmarks: each dispatched token is 7168 fp8 values and 56 fp32 scaling
 * factors).  Needs dispatch_dtype FL_DTYPE_E4M3_BLOCK128.  codes [N][T][H] e4m3
 * bytes, scales [N][T][H/128] fp32 (one per 128 values, as fl_moe_dispatch_send
 * would have produced them); both are copied unchanged into the wire rows, so
 * expert_x / expert_scales receive exactly these bytes.  weights: NULL, or
 * [N][T][K] when the context has FL_FLAG_PARTIAL_SUMS. */
int fl_moe_dispatch_send_e4m3(fl_moe_ctx *ctx, int rank_begin, int rank_count, const void *codes,
                              const float *scales, const float *weights, void *stream);

/* Step 3 (section Dispatch: wait for all transfers, then reorder tokens with
 * optional padding into a layout suitable for grouped GEMM).  expert_x
 * [N][expert_capacity_rows][H] (bf16 or e4m3 bytes): rows of rank d ordered by
 * (local expert, source rank, token index).  expert_scales
 * [N][expert_capacity_rows][H/128] fp32, e4m3 only (else NULL).
 * tokens_per_expert [N][E/N] int32 out. */
int fl_moe_dispatch_recv(fl_moe_ctx *ctx, int rank_begin, int rank_count, void *expert_x,
                         float *expert_scales, int32_t *tokens_per_expert, void *stream);

/* Step 4 (section Combine: a single scatter per peer re-using the routing
 * information).  expert_y [N][expert_capacity_rows][H] bf16, same row layout as
 * expert_x.  Packs each peer's rows contiguously, copies them into the peer's
 * combine receive buffer and announces every reply, empty ones included, on
 * arrive_comb[peer][this rank] (units plus one, as in dispatch).  Call it once per
 * fl_moe_layout, after fl_moe_dispatch_recv. */
int fl_moe_combine_send(fl_moe_ctx *ctx, int rank_begin, int rank_count, const void *expert_y,
                        void *stream);

/* Step 5 (section Combine: weighted average computed locally; fp32 accumulation
 * in a fixed order, section Comparison with DeepEP).  weights [N][T][K] fp32,
 * out [N][T][H] bf16:
 *   out[s][t] = bf16( sum_{k=0..K-1} weights[s][t][k] * float(y of pair (s,t,k)) )
 * fp32 accumulator starting at +0, fused multiply-add, k ascending, one final
 * round-to-nearest-even; no division by the weight sum.  Rows t >= num_tokens[s]
 * are not written. */
int fl_moe_combine_reduce(fl_moe_ctx *ctx, int rank_begin, int rank_count, const float *weights,
                          void *out, void *stream);

/* Reads and clears the device status word (synchronises the stream). */
int fl_moe_status(fl_moe_ctx *ctx, int32_t *host_out /*host*/, void *stream);

/* What to do about FL_STATUS_CAPACITY (capacities are the caller's choice; the paper
 * sizes its buffers for the worst case, section Dispatch).  After the layout calls of
 * a step have covered all N ranks, this call returns the smallest recv_capacity_rows
 * and expert_capacity_rows with which that same step fits on every rank: the maxima
 * over ranks of the rows a rank receives beyond the private slots, and of the rows of
 * its expert-major layout with the padding of expert_align.  A caller whose step was
 * skipped for capacity creates a context with at least these values (and its own
 * margin) and repeats the step.  It reads the per-source count tables of the last
 * layout call (N*E + N*N ints), which the sources write whether or not the plan was
 * valid; after FL_STATUS_BAD_INDEX or a time-out of the layout call the result is
 * meaningless.  Set-up work: synchronises `stream`, copies to the host, allocates host
 * memory; it neither reads nor clears the status word. */
int fl_moe_required_capacities(fl_moe_ctx *ctx, int64_t *recv_capacity_rows /*host*/,
                               int64_t *expert_capacity_rows /*host*/, void *stream);

/* After FL_STATUS_TIMEOUT the counters of a context can be out of step for good: a
 * layout call whose peers never ran has advanced its own ranks' epochs and message
 * counters but not theirs, and a payload wait that gave up leaves its expectation ahead
 * of what was delivered.  Once every stream that carries calls of this context has
 * drained, fl_moe_reset zeroes the status word, the route epochs and message counters
 * and the payload counters (set-up work: a memset and a synchronisation of `stream`),
 * after which the next step starts as on a new context.  Not to be recorded in a graph. */
int fl_moe_reset(fl_moe_ctx *ctx, void *stream);

const char *fl_moe_strerror(int code);

int fl_moe_debug_views(fl_moe_ctx *ctx, fl_moe_debug_view *out /*host*/);

/* Diagnostic: overrides a launch-shape knob of the copy kernels (results never
 * change).  knob 0 = rows per workgroup of the unpack / combine-pack kernels
 * (0 = chosen from the row size, at most 64), knob 1 = row loads issued together
 * per thread in combine_reduce (0 = all K, at most 8), knob 2 = waves per row in
 * the fabric kernel (0 = chosen from the row size, else 1..16), knob 3 =
 * workgroups per token in the pack kernel (0 = chosen from the row size, at
 * most 16), knob 4 = size in MiB of the receive buffers a fabric launch may
 * write above which it uses streaming instead of cached stores (default 2560),
 * knob 5 = percentage of the rows uniform routing would bring to a rank that the
 * grids of the receive-side and reply kernels are sized for (default 200; 0 = the
 * whole capacity; a rank that holds more is served by the kernels' row loops),
 * knob 6 = payload in MiB one launch should move per direction: a call whose ranks
 * move more than three times as much is issued as several launches over rank
 * groups of about this size (default 860; 0 = always one launch per kernel;
 * contexts with FL_FLAG_PROGRESSIVE_RECV are never cut), knob 7 = eighths of the
 * machine's resident-workgroup slots the polling receive kernels of
 * FL_FLAG_PROGRESSIVE_RECV may take (default 3), knob 8 = order in which the fabric kernel
 * takes the destinations of a sender (0 = ascending, 1 = descending, 2 = starting with
 * the sender's right-hand neighbour and wrapping round; a test switch: nothing may depend
 * on the order in which transfers are carried out), knob 9 = workgroups that share one
 * token in combine_reduce, each summing a slice of the row (0 = chosen from the row
 * size).  A value of -1 restores a knob's default. */
int fl_moe_debug_tune(fl_moe_ctx *ctx, int knob, int value);

/* Diagnostic, host only (no GPU needed): how a payload call over `rank_count` ranks of
 * this configuration is cut into launches.  launch_mb as knob 6 above (-1 = the
 * default).  *ranks_per_group receives the ranks one launch serves (rank_count
 * when the call is not cut; the last group may be smaller). */
int fl_moe_debug_launch_groups(const fl_moe_config *cfg /*host*/, int rank_count, int launch_mb,
                               int *ranks_per_group /*host*/);

/* Diagnostic: plain linear device copy of `bytes` bytes with 16-byte accesses
 * (multiple of 16, both pointers 16-byte aligned), in the launch shape that measured
 * fastest for a linear copy on this part.  Used to measure the copy ceiling of the
 * machine and to calibrate hardware byte counters against a known size. */
int fl_moe_debug_copy(void *dst, const void *src, size_t bytes, void *stream);

/* Diagnostic: the write-only and read-only counterparts of fl_moe_debug_copy, each in its
 * own fastest launch shape (fill: 16-byte streaming stores of a constant; read: 16-byte
 * streaming loads whose values are folded and, practically never, written to the 4-byte
 * word `sink`).  They
 * measure the machine's one-directional ceilings, against which kernels that mostly
 * write (dispatch pack) or mostly read (combine reduce) are judged. */
int fl_moe_debug_fill(void *dst, size_t bytes, void *stream);
int fl_moe_debug_read(const void *src, size_t bytes, void *sink, void *stream);

/* Per-kernel timing with HIP events on the caller's stream.  While enabled,
 * every kernel launch of the shuffle calls is bracketed by an event pair;
 * fl_moe_profile_collect synchronises, adds the elapsed times of the launches
 * since the last collect to per-kernel totals, and fl_moe_profile_read returns
 * totals (ms) and launch counts for kernel ids 0..FL_KERNEL_COUNT-1.  At most
 * 512 launches between two collects are timed; further ones run untimed. */
#define FL_KERNEL_COUNT 14
int fl_moe_profile_enable(fl_moe_ctx *ctx, int on);
int fl_moe_profile_collect(fl_moe_ctx *ctx, void *stream);
int fl_moe_profile_read(fl_moe_ctx *ctx, double *total_ms /*host [FL_KERNEL_COUNT]*/,
                        int64_t *launches /*host [FL_KERNEL_COUNT]*/);
const char *fl_moe_kernel_name(int kernel_id);

/* Identifies the sources this binary was built from (a hash the build passes in; "unknown"
 * for a build that did not).  The Python binding refuses a library whose id differs from
 * the sources beside it, and stored profiler figures name the id they were measured with. */
const char *fl_moe_build_id(void);

#ifdef __cplusplus
}
#endif
#endif /* FLMOE_H */
