/*
 * libbls - one GPU's share of the distributed sparse-embedding lookup of
 * bounded-lag-synchronous (BLS) DLRM inference, for AMD MI355X (gfx950).
 *
 * P ranks are simulated inside one GPU's memory.  Rank s owns a contiguous block of
 * the global batch (its mini-batch); rank d owns a share of the embedding tables
 * (whole tables, or a block of rows of every table).  One iteration of the path is
 *
 *   bls_plan            which lookups go to which rank: alltoallv counts and
 *                       displacements, and the lookups laid out in owner order
 *   bls_embbag_pool     EmbeddingBag (sum) on every owner's local tables or shards
 *   bls_pack            pooled vectors into per-destination send regions S(d)
 *   bls_ring_advance    take the next of the k receive buffers, slot = iteration mod k
 *   bls_alltoallv_local the alltoallv itself: S(d) blocks into R(s, slot)
 *   bls_unpack          completion: copy R(s, slot) out as [B][T][D], free the slot
 * (bls_embbag_pool_put fuses pool, pack and the alltoallv: pooled vectors go straight into the slot.)
 *
 * Notation (used in every comment below): P ranks, T tables, B global batch, D vector
 * length, K = max(k, 1) ring slots, F = 1 (table-wise partition) or P (row-wise),
 * bag g = t*B + b, requester s(b) = rank whose mini-batch holds sample b, owner
 * d(t, idx), n_loc(d) = number of tables rank d serves, loc(t) = position of t among
 * its owner's tables in increasing t.  Mini-batch of rank s is samples
 * [first(s), first(s+1)); when P does not divide B the first B mod P ranks hold one
 * sample more.  Row-wise shards hold ceil(rows_t / P) rows (the last ones may be
 * short or empty): d = idx / ceil(rows_t / P).
 *
 * Segment order.  Owner-side data (ridx, segoff, send regions) is ordered by
 * (d, s, t_loc, b_loc), b_loc = b - first(s).  Receive regions are ordered by
 * (s, d, t_loc, b_loc).
 *
 * Conventions.  Every function returns BLS_OK or a negative code and never throws or
 * aborts.  Pointers named d_* are DEVICE memory owned by the caller and must stay
 * valid until the work enqueued on `hip_stream` has finished; all other pointers are
 * HOST memory.  `hip_stream` is a hipStream_t passed as void* (NULL = the null
 * stream).  Calls enqueue work and return without waiting.  Data-dependent errors
 * (an index outside its table, offsets that decrease) cannot be seen by the host at
 * call time: kernels raise a device-side flag that bls_check reports, and never touch
 * memory outside the buffers: a lookup with a bad index adds nothing to its bag's vector
 * (whether the alltoallv counts include it is unspecified), a bag with bad offsets is
 * treated as empty.  The library allocates no device memory: its small descriptor tables
 * live in a buffer the caller provides (bls_commit), scratch memory comes from the caller
 * (d_ws).  No path call allocates, frees or waits for the device.  A context is not thread
 * safe.
 */
#ifndef BLS_H
#define BLS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct bls_ctx bls_ctx; /* opaque; host memory owned by the library */

enum {
    BLS_OK = 0,
    BLS_EINVAL = -1,      /* bad argument, missing shard, NULL pointer                       */
    BLS_ERANGE = -2,      /* an index outside [0, rows_t) or non-monotone offsets (device)   */
    BLS_ENOSPC = -3,      /* a caller buffer (workspace, ring) is too small                  */
    BLS_ERING_FULL = -4,  /* K iterations already in flight                                  */
    BLS_ERING_EMPTY = -5, /* completion asked for with nothing in flight                     */
    BLS_EORDER = -6,      /* completion out of FIFO order, or exchange into a wrong slot     */
    BLS_EHIP = -7         /* a HIP runtime call failed; text in bls_last_error               */
};

/* Table storage; accumulation and output are fp32.
 * BLS_U8_ROWQ (an extension, not in the paper): a row is bls_row_bytes(D) = D + 8 rounded up
 * to a multiple of 16 bytes: D unsigned 8-bit codes, the row's fp32 scale, its fp32 bias,
 * padding (ignored).  Element c of the row stands for the fp32 number
 * fl(fl((float)code[c] * scale) + bias) - product and sum rounded separately, no fused
 * multiply-add - and the bag sum adds these numbers like any other fp32 row.
 * BLS_F8_ROWQ: the same row layout with 8-bit float codes (E4M3: 1 sign, 4 exponent bits with
 * bias 7, 3 mantissa bits, no infinities; NaN codes give NaN) in place of the integers. */
enum { BLS_FP32 = 0, BLS_FP16 = 1, BLS_U8_ROWQ = 2, BLS_F8_ROWQ = 3 };
enum { BLS_TABLE_WISE = 0, BLS_ROW_WISE = 1 };

typedef struct bls_config {
    int32_t P, T, D, k;          /* 1 <= P <= 64; k >= 0 is the paper's bound, K = max(k,1) slots   */
    int64_t B;                   /* global batch, B >= P                                             */
    int32_t table_dtype;         /* BLS_FP32 | BLS_FP16 | BLS_U8_ROWQ | BLS_F8_ROWQ                  */
    int32_t part_kind;           /* BLS_TABLE_WISE | BLS_ROW_WISE                                    */
    const int64_t *rows;         /* host [T], rows per table (global), each >= 1                     */
    const int32_t *table_owner;  /* host [T], owner rank of each table; read for table-wise only     */
} bls_config;

/* Lifecycle.  bls_create copies the configuration (rows / table_owner are not kept).
 * Touches no GPU. */
int bls_create(const bls_config *cfg, bls_ctx **out);
int bls_destroy(bls_ctx *ctx);

/* Hand the library one table shard: row-major [rows_in_shard][D] in the configured
 * storage dtype ([rows_in_shard][D + 8 rounded up to 16] bytes for the row-quantised ones), device
 * memory, 16-byte aligned, borrowed until bls_destroy.
 * Table-wise: rank must be table_owner[t] and rows_in_shard = rows[t].  Row-wise: one
 * call per (t, rank), rows_in_shard = number of rows of table t that fall in the
 * rank's block (may be 0, then d_rows may be NULL). */
int bls_set_shard(bls_ctx *ctx, int32_t t, int32_t rank, const void *d_rows, int64_t rows_in_shard);

/* Row-wise block partition made visible: rows [first_row, first_row + rows_in_shard) of table t
 * are the shard of `rank` (block size ceil(rows_t / P); trailing shards may be empty).  Table-wise:
 * the owner holds (0, rows_t), every other rank (0, 0).  Host outputs, either may be NULL. */
int bls_shard_range(const bls_ctx *ctx, int32_t t, int32_t rank, int64_t *first_row, int64_t *rows_in_shard);

/* The library's descriptor tables (mini-batch starts, tables per rank, shard pointers and sizes,
 * the error flag) live in device memory of the caller: bls_desc_bytes gives the size (a few KB),
 * bls_commit checks that every shard has been set and uploads the tables into d_desc (16-byte
 * aligned, borrowed until bls_destroy) with an asynchronous copy on `hip_stream`; path calls on
 * other streams must be ordered after it by the caller.  Every call that launches kernels returns
 * BLS_EINVAL until bls_commit has been called, and again after a later bls_set_shard until the next
 * bls_commit (which then waits for the device first: kernels in flight may still read the old
 * tables; the error flag is kept).  Not allowed while iterations are in flight (BLS_EORDER). */
int bls_desc_bytes(const bls_ctx *ctx, size_t *bytes);
int bls_commit(bls_ctx *ctx, void *d_desc, size_t bytes, void *hip_stream);

/* Popular rows of a shard (a hint; Related Work: systems for these models keep frequently used
 * embedding rows in faster memory).  rows[0 .. n): local row numbers of shard (t, rank), most
 * popular first, host memory, copied; at most BLS_HOT_ROWS_MAX are kept, repeats are dropped, a
 * row outside the shard is BLS_EINVAL, n = 0 clears the list.  When lists are set the pooling
 * calls may run workgroups that stay on a compute unit, copy the listed rows of the table they work
 * on to LDS once and serve lookups of them from there; every result is the same bit for bit with or
 * without lists, whatever they name.  Where the rows come from (counts over earlier batches, say)
 * is the caller's business.  Takes effect with the next bls_commit (bls_desc_bytes grows by four
 * bytes per listed row). */
enum { BLS_HOT_ROWS_MAX = 256 };
int bls_set_hot_rows(bls_ctx *ctx, int32_t t, int32_t rank, const int64_t *rows, int32_t n);

/* Launch shape of the pooling kernels, for tests and experiments; results are the same bit for
 * bit under every setting.  lane_bytes: table bytes one lane holds of a row (4, 8, 16; 0 = the
 * library's choice); segments_per_group: consecutive segments one lane group streams (1..63, capped
 * at lanes - 1; 0 = chosen from the mean bag length); xcd_map: 1 deals workgroups so that one XCD
 * works on the same tables, 0 plain grid (-1 = library's choice); wide_positions: 1 forces 64-bit
 * row positions (-1 / 0 = only when a shard needs them). */
int bls_set_pool_tuning(bls_ctx *ctx, int32_t lane_bytes, int32_t segments_per_group, int32_t xcd_map,
                        int32_t wide_positions);

/* Form of bls_plan, for tests and experiments; results are the same bit for bit.
 * scan_while_placing = 0: always three launches (count, scan, place).  -1 or 1: fewer where the
 * problem allows it.  Table-wise with at most 2048 runs (pairs of an (owner, table) and a
 * requester) and at most 2^22 lookups: one launch, every workgroup works the run starts out for
 * itself from the offsets at the run edges.  Row-wise with at most eight ranks and batches below 2^32 lookups: two launches,
 * every placing workgroup adds the tile counts up for itself instead of reading a scanned array. */
int bls_set_plan_tuning(bls_ctx *ctx, int32_t scan_while_placing);

/* Buffer sizes in bytes for a batch of at most max_nnz lookups: plan workspace, the
 * pooled buffer Y, the send buffer S, and one ring slot (all three F*T*B*D fp32). */
int bls_sizes(const bls_ctx *ctx, int64_t max_nnz, size_t *plan_ws_bytes, size_t *pooled_bytes,
              size_t *send_bytes, size_t *slot_bytes);

/* Counts and displacements of the pooled-vector alltoallv (the exchange of Listing 1,
 * alltoall(ly, n_emb_per_rank)), in fp32 elements, closed-form from the configuration:
 * pcount[d][s] = n_loc(d) * B_loc(s) * D.  Host outputs, [P*P] each, any may be NULL:
 * pcount / psdispl row-major [d][s] (send side), prcount / prdispl row-major [s][d]. */
int bls_pooled_counts(const bls_ctx *ctx, int64_t *pcount, int64_t *psdispl, int64_t *prcount, int64_t *prdispl);

/*
 * Index bucketing (Introduction: every process works out which vector IDs it needs
 * from which process; the irregular per-peer counts are what make the exchange an
 * alltoallv).  Inputs: d_indices[nnz] global row ids, d_offsets[T*B+1] with
 * offsets[0] = 0 and offsets[T*B] = nnz, bag g = t*B + b.
 * Outputs, all int64 device arrays:
 *   d_sendcounts, d_sdispls [P*P] row-major [s][d]: lookups rank s asks of rank d and
 *       their exclusive running sum over d;
 *   d_recvcounts, d_rdispls [P*P] row-major [d][s]: the transpose and its running sum;
 *   d_ridx[nnz]: row inside the owner's shard of every lookup, in owner order
 *       (d, then s, then input order - placement inside a bucket is stable);
 *   d_segoff[F*T*B+1]: start in d_ridx of every (d, s, t_loc, b_loc) segment, last
 *       entry nnz;
 *   d_perm[nnz] or NULL: requester-side position (s, then d, then input order) of
 *       every lookup, i.e. where it sits in rank s's send region of the index exchange.
 * d_ws / ws_bytes: scratch of at least bls_sizes' plan_ws_bytes, 8-byte aligned.
 */
int bls_plan(bls_ctx *ctx, const int64_t *d_indices, const int64_t *d_offsets, int64_t nnz,
             int64_t *d_sendcounts, int64_t *d_sdispls, int64_t *d_recvcounts, int64_t *d_rdispls,
             int64_t *d_ridx, int64_t *d_segoff, int64_t *d_perm, void *d_ws, size_t ws_bytes, void *hip_stream);

/*
 * bls_plan for callers that cannot allocate device memory (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): the same work and the same outputs, bit for bit,
 * with the scratch taken from a 1 MiB array that is part of the library's device code (one copy
 * per GPU, held until the process ends) instead of d_ws.  Calls nothing that allocates or frees.
 * BLS_ENOSPC when the problem needs more than that (bls_sizes' plan_ws_bytes > 1 MiB, i.e. beyond
 * about 10^8 segments F*T*B): use bls_plan then.  All calls on one GPU share the one array, from
 * every context and stream: two calls that may run at the same time on one GPU race - order them
 * (one stream, or events).  The array needs no clearing between calls: every word a call reads it
 * has written first.  The first call on a device looks the array's address up (no allocation, but
 * not a stream operation): make it before starting a capture.
 */
int bls_plan_noalloc(bls_ctx *ctx, const int64_t *d_indices, const int64_t *d_offsets, int64_t nnz,
                     int64_t *d_sendcounts, int64_t *d_sdispls, int64_t *d_recvcounts, int64_t *d_rdispls,
                     int64_t *d_ridx, int64_t *d_segoff, int64_t *d_perm, void *hip_stream);

/*
 * EmbeddingBag, sum mode (Listing 1: apply_emb over offsets and indices; the paper's
 * profile shows it dominating the run).  For owner d, local table t_loc and sample b:
 *   Y_d[t_loc][b][:] = sum over the segment's rows of W_{t,d}[ridx[.]][:]
 * fp32 accumulation from +0 in segment order (bit-exact against an ordered CPU sum).
 * d_pooled is Y_0 .. Y_{P-1} back to back, Y_d = [n_loc(d)][B][D] fp32.  nnz is the
 * extent of d_ridx; segments that reach past it are skipped and flagged.
 */
int bls_embbag_pool(bls_ctx *ctx, const int64_t *d_ridx, const int64_t *d_segoff, int64_t nnz,
                    float *d_pooled, void *hip_stream);

/* Send buffer S(p) of the alltoallv figure: S_d[s][t_loc][b_loc][:] =
 * Y_d[t_loc][first(s)+b_loc][:], regions of d = 0..P-1 back to back (segment order). */
int bls_pack(bls_ctx *ctx, const float *d_pooled, float *d_send, void *hip_stream);

/* Ring of K receive buffers R(*, i) (BLS backend initialisation: k buffers created
 * once and reused circularly).  d_slots is caller-owned, bytes >= K * slot_bytes,
 * 16-byte aligned. */
int bls_set_ring(bls_ctx *ctx, void *d_slots, size_t bytes);

/* Start iteration j = number of earlier successful calls: slot = j mod K (Alltoallv
 * initiation).  Fails with BLS_ERING_FULL when K iterations are in flight (section on
 * the bound: a process that has issued k iterations must complete the oldest first).
 * Makes `hip_stream` wait until the slot's previous contents have been copied out. */
int bls_ring_advance(bls_ctx *ctx, int64_t *iter_out, int32_t *slot_out, void *hip_stream);

/* The alltoallv on one device (Alltoallv initiation: each source writes its block into
 * the destination's receive buffer R(dst, slot); with k = 0 this is MPI_Alltoallv):
 * R_s(slot)[d][t_loc][b_loc][:] = S_d[s][t_loc][b_loc][:] for all P*P (d, s) blocks.
 * `slot` must be the slot of the youngest iteration started and not yet exchanged. */
int bls_alltoallv_local(bls_ctx *ctx, const float *d_send, int32_t slot, void *hip_stream);

/* The owner side in one pass: EmbeddingBag sum whose results are put straight into the
 * receive regions of ring slot `slot` (Alltoallv initiation is a sequence of one-sided puts
 * into R(dst, slot); here the source of each put is the pooling kernel's accumulator rather
 * than a send buffer, so neither Y nor S is written).  Leaves R(*, slot) exactly as
 * bls_embbag_pool + bls_pack + bls_alltoallv_local would, bit for bit.  `slot` as for
 * bls_alltoallv_local; arguments as for bls_embbag_pool. */
int bls_embbag_pool_put(bls_ctx *ctx, const int64_t *d_ridx, const int64_t *d_segoff, int64_t nnz,
                        int32_t slot, void *hip_stream);

/*
 * Per-sample weights (Listing 1 hands them to apply_emb as v_W_l).  bls_plan_weighted is
 * bls_plan that also carries the weight of every lookup along: d_weights[nnz] in input order,
 * d_rweights[nnz] out in the order of d_ridx.  The weighted pooling calls then compute
 *   Y_d[t_loc][b][:] = sum over the segment of  w * row,
 * each product rounded to fp32 and then added (no fused multiply-add), otherwise exactly as
 * bls_embbag_pool / bls_embbag_pool_put.
 */
int bls_plan_weighted(bls_ctx *ctx, const int64_t *d_indices, const int64_t *d_offsets, const float *d_weights,
                      int64_t nnz, int64_t *d_sendcounts, int64_t *d_sdispls, int64_t *d_recvcounts,
                      int64_t *d_rdispls, int64_t *d_ridx, float *d_rweights, int64_t *d_segoff, int64_t *d_perm,
                      void *d_ws, size_t ws_bytes, void *hip_stream);
int bls_embbag_pool_weighted(bls_ctx *ctx, const int64_t *d_ridx, const float *d_rweights, const int64_t *d_segoff,
                             int64_t nnz, float *d_pooled, void *hip_stream);
int bls_embbag_pool_put_weighted(bls_ctx *ctx, const int64_t *d_ridx, const float *d_rweights,
                                 const int64_t *d_segoff, int64_t nnz, int32_t slot, void *hip_stream);

/*
 * A whole synchronous iteration of a TABLE-WISE partition in one launch: bls_plan, bls_embbag_pool,
 * bls_pack, bls_ring_advance, bls_alltoallv_local and bls_unpack in that order with no other
 * iteration in flight (the k = 0 case of section "A zero-bound parameter": issue and completion
 * back to back).  Small batches are bound by the hand-over between the staged calls' kernels, not by
 * the kernels; with whole tables per rank every output has a closed-form place given the lengths
 * of the (table, mini-batch) runs, so one kernel writes them all.  Every output - counts and
 * displacements, d_ridx, d_segoff, d_perm (or NULL), d_pooled, d_send, the receive regions of ring
 * slot (iteration mod K) and d_out - is bit for bit what the staged calls leave.  Counts as one
 * iteration of the ring (*iter_out, may be NULL, receives its number).  BLS_EORDER while iterations
 * are in flight; BLS_EINVAL for a row-wise partition, for rows that are not a multiple of 16 bytes
 * or longer than 1 KB, and for more than 2048 (table, rank) runs: use the staged calls there.
 * Unweighted sum pooling only.  No workspace is needed.
 */
int bls_step_tablewise(bls_ctx *ctx, const int64_t *d_indices, const int64_t *d_offsets, int64_t nnz,
                       int64_t *d_sendcounts, int64_t *d_sdispls, int64_t *d_recvcounts, int64_t *d_rdispls,
                       int64_t *d_ridx, int64_t *d_segoff, int64_t *d_perm, float *d_pooled, float *d_send,
                       float *d_out, int64_t *iter_out, void *hip_stream);

/* Alltoallv completion for iteration `iter`, which must be the oldest in flight
 * (wait() completes the tail request and pops it): copy the receive regions of its
 * slot to d_out[B][T][D] fp32 and free the slot.  Table-wise: a copy.  Row-wise: the P
 * partial sums of every (b, t) are added from +0 in increasing owner rank. */
int bls_unpack(bls_ctx *ctx, int64_t iter, float *d_out, void *hip_stream);

/* Completion with mean pooling: as bls_unpack, and every vector of a non-empty bag is then
 * divided (one fp32 division per element) by the bag's length offsets[g+1] - offsets[g];
 * d_offsets is the iteration's offsets array, device memory. */
int bls_unpack_mean(bls_ctx *ctx, int64_t iter, const int64_t *d_offsets, float *d_out, void *hip_stream);

/*
 * Per-rank issue and completion: the work of bls_embbag_pool_put and bls_unpack split by
 * rank, so that every simulated rank can run on a stream of its own and fall behind the others
 * by up to K iterations (section "Bound": the fastest and the slowest process are at most
 * k iterations apart; Listing 2: the loop that keeps up to `bound` requests unfinished).
 *
 * bls_rank_put: owner `rank` pools its local tables (or shards) for every requester and puts the
 *   vectors into R(*, iter mod K) - the puts of Alltoallv initiation.  `iter` must be this
 *   rank's next iteration (0, 1, 2, ...).  The call makes the stream wait until every requester
 *   has copied iteration iter - K out of the slot, and records the arrival of this owner's
 *   blocks (one event per slot and owner: the role of the paper's tag counters).  BLS_ERING_FULL
 *   if some requester has not yet been asked to complete iteration iter - K.  d_rweights may
 *   be NULL (no per-sample weights).  d_ridx / d_segoff as produced by bls_plan for that iteration.
 * bls_rank_complete: requester `rank` completes its oldest iteration `iter`: the stream waits
 *   for the arrival of all P owners' blocks (every owner must already have been asked to put
 *   `iter`, else BLS_EORDER), then rows [first(rank), first(rank+1)) of d_out[B][T][D] are
 *   written (divided by the bag length if d_mean_offsets is not NULL) and the rank's share of
 *   the slot is released.
 * Do not interleave these with bls_ring_advance / bls_unpack while iterations are in flight, and let the
 * device go idle (bls_check) before switching from one style to the other: the two keep separate events.
 * bls_rank_delay keeps a stream busy for about `microseconds` (at most 1 s; a bounded sleep
 * loop in one lane): the injected delays of the paper's Setting 2, for experiments.
 */
int bls_rank_put(bls_ctx *ctx, int32_t rank, const int64_t *d_ridx, const float *d_rweights, const int64_t *d_segoff,
                 int64_t nnz, int64_t iter, void *hip_stream);
int bls_rank_complete(bls_ctx *ctx, int32_t rank, int64_t iter, const int64_t *d_mean_offsets, float *d_out,
                      void *hip_stream);
int bls_rank_delay(bls_ctx *ctx, uint32_t microseconds, void *hip_stream);

/*
 * The dense part of the model around the lookup (Introduction: dense features go through the
 * bottom MLP, the pooled vectors and its output through a dot-product interaction layer and
 * the top MLP; Listings 1 and 2: apply_mlp, interact_features).  fp32 in, fp32 out, products
 * accumulated in fp32 on the matrix cores; the summation order is the hardware's, so results
 * match a double-precision evaluation to within (K + 3) * 2^-24 * (|bias| + sum |x||w|).
 *
 * bls_mlp_layer: d_y[M][N] = act(d_x[M][K] * d_W[N][K]^T + d_bias[N]); d_bias may be NULL;
 *   act is BLS_ACT_NONE, BLS_ACT_RELU or BLS_ACT_SIGMOID.  All arrays row-major device memory,
 *   d_y must not overlap the inputs.  M >= 0, 1 <= K, N < 2^31 / 128.
 * bls_interact: for samples b0 .. b0+bn-1 (b0 + bn <= B), with Z = [d_x[b]; d_emb[b][0..T-1]]
 *   ((T+1) vectors of length D): d_z[b] = d_x[b] followed by Z_i . Z_j for all pairs i > j in
 *   the order i = 1..T, j = 0..i-1.  d_x is [B][D], d_emb is [B][T][D] (the output of
 *   bls_unpack), d_z is [B][D + T(T+1)/2].  BLS_EINVAL if the T vectors of a sample do not
 *   fit in 64 KB of LDS (about T * D <= 16000).
 * bls_unpack_interact: completion of iteration `iter` (the oldest in flight, as for bls_unpack)
 *   folded into the interaction: the pooled vectors are read from the iteration's ring slot where
 *   their owners put them (row-wise: the P partial vectors added in increasing owner rank, as
 *   bls_unpack does) and d_z[B][D + T(T+1)/2] is written for the whole batch; no [B][T][D] output
 *   is produced.  The slot is released as by bls_unpack.  Same results, bit for bit, as
 *   bls_unpack followed by bls_interact.
 */
enum { BLS_ACT_NONE = 0, BLS_ACT_RELU = 1, BLS_ACT_SIGMOID = 2 };
int bls_mlp_layer(bls_ctx *ctx, const float *d_x, int64_t M, int32_t K, const float *d_W, const float *d_bias,
                  int32_t N, int32_t act, float *d_y, void *hip_stream);
int bls_interact(bls_ctx *ctx, const float *d_x, const float *d_emb, float *d_z, int64_t b0, int64_t bn,
                 void *hip_stream);
int bls_unpack_interact(bls_ctx *ctx, int64_t iter, const float *d_x, float *d_z, void *hip_stream);

/* Ring state for callers and tests: next iteration number, oldest in flight, K. */
int bls_ring_state(const bls_ctx *ctx, int64_t *head, int64_t *tail, int32_t *K);

/* Wait for `hip_stream`, then return BLS_ERANGE if any kernel since the last
 * bls_check saw a bad index / offset / segment (and clear the flag), else BLS_OK. */
int bls_check(bls_ctx *ctx, void *hip_stream);

/* Text of the last error on this context (never NULL). */
const char *bls_last_error(const bls_ctx *ctx);

#ifdef __cplusplus
}
#endif
#endif /* BLS_H */
