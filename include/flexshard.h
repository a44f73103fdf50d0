/*
 * flexshard.h -- C ABI of libflexshard_hip.so
 *
 * The tiered sequence-embedding lookup behind FlexShard's per-row sharding
 * (arXiv 2301.02959), taken at one GPU's share of the work:
 *
 *   jagged ids -> per-row placement (tier, owner) -> stable bucketize by owner
 *   -> unpooled sequence gather -> duplicate-row gradient accumulation,
 *   plus the row-frequency histogram and top-k-under-budget choice of the
 *   rows to replicate.
 *
 * The paper describes the placement (Sections 3.1, 4.3-4.6) and the cost of
 * each stage (Section 3.2, the six per-GPU metrics and the two cost tables);
 * it describes no kernel.  The operations below are the stages those metrics
 * name, written as plain array operations.
 *
 * Conventions for every entry point
 *   - Every pointer is DEVICE memory owned by the caller unless the comment
 *     says "host".  The library allocates nothing, frees nothing and keeps no
 *     state between calls (the opt-in profiling hooks at the end and the
 *     static scratch array of fs_route_bucketize_noalloc excepted).
 *   - All work is enqueued on `stream` (a hipStream_t passed as void*; NULL is
 *     the default stream).  No entry point synchronises with the host.
 *   - `workspace == NULL`: the required scratch size is written to
 *     `*workspace_bytes` (host), nothing is launched, FS_OK is returned.
 *     Otherwise `*workspace_bytes` is the size of the buffer passed in and
 *     must be at least the required size (else FS_ERR_WORKSPACE).  The
 *     workspace must be 256-byte aligned.
 *   - Faults the host can see return an fs_status at once and launch nothing.
 *     Faults only the data shows OR a bit into `*dev_status` (a caller-owned
 *     int32 in device memory that the library never clears) and keep every
 *     access in bounds.  `dev_status` may be NULL: then nothing is reported.
 *   - n == 0 (or an empty [j0, j1) range) is legal everywhere.
 *   - 0 <= n < 2^31, 0 < R < 2^32 - 1.
 */
#ifndef FLEXSHARD_H
#define FLEXSHARD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    FS_OK = 0,
    FS_ERR_NULL = 1,      /* a required pointer is NULL */
    FS_ERR_SIZE = 2,      /* negative / overflowing / inconsistent size */
    FS_ERR_DTYPE = 3,     /* unknown fs_dtype */
    FS_ERR_ALIGN = 4,     /* row bytes not a multiple of 16, or base not 16-B aligned */
    FS_ERR_WORKSPACE = 5, /* workspace too small or misaligned */
    FS_ERR_CONFIG = 6,    /* U, W, self, flags, variant out of range */
    FS_ERR_DEVICE = 7     /* a HIP call failed */
} fs_status;

typedef enum { FS_F32 = 0, FS_F16 = 1, FS_BF16 = 2 } fs_dtype;

/* Bits OR-ed into *dev_status. */
enum {
    FS_DEV_BAD_ID = 1,         /* id outside its table / row or pos outside range */
    FS_DEV_BAD_OFFSETS = 2,    /* offsets[0] != 0, decreasing, or offsets[T*B] != n */
    FS_DEV_BAD_PLACEMENT = 4,  /* tier 3, or owner outside its range */
    FS_DEV_COUNT_OVERFLOW = 8, /* a histogram count saturated at 2^32 - 1 */
    FS_DEV_UNIQUE_OVERFLOW = 16, /* more distinct rows than cap_unique */
    FS_DEV_POS_ORDER = 32,     /* bwd: equal rows whose pos is not ascending in j */
    FS_DEV_NOT_SORTED = 64     /* fs_seq_grad_bwd_sorted: rows not ascending */
};

/*
 * Placement entry, one uint32 per global row g (Sections 4.3-4.5: every row
 * is in exactly one of three tiers):
 *   bits 31..30  tier   0 replicated on every GPU        ("DP")
 *                       1 replicated once per group      ("Flex": sharded
 *                         over the W GPUs of a group, each shard replicated
 *                         across the U/W groups)
 *                       2 sharded over all U GPUs        ("RW")
 *                       3 invalid
 *   bits 29..0   owner  tier 2: bucket in [0, U); tier 1: index in [0, W)
 *                       inside the requester's group; tier 0: ignored by
 *                       fs_route_bucketize; fs_route_bucketize_slots reads
 *                       the row's replica slot there (FS_OWNER_MASK: none).
 */
#define FS_TIER_SHIFT 30
#define FS_OWNER_MASK 0x3FFFFFFFu
#define FS_TIER_GLOBAL 0u
#define FS_TIER_GROUP 1u
#define FS_TIER_SHARDED 2u

/* Number of sorted lookups per partial sum in the backward's canonical
 * summation order (see fs_seq_grad_bwd). */
#define FS_BWD_TILE 256

/* Most owner buckets a call admits.  The router's scatter keeps 12 bytes of LDS per bucket and
 * workgroup (an output base, and a running count per wave): 48 KB at 4096 buckets; the CU has 160 KB. */
#define FS_MAX_BUCKETS 4096

/*
 * fs_route_bucketize -- input-ID distribution (Section 3.2, metric 2 "input
 * data distribution": the ids that must reach their owners before any lookup;
 * tier semantics from Sections 3.1, 4.4, 4.5).
 *
 *   ids[n], offsets[T*B + 1]   jagged batch, table-major: segment t*B + b holds
 *                              sample b of table t; ids are table-local.
 *   row_base[T + 1]            row_base[t] = first global row of table t,
 *                              row_base[T] = R.
 *   placement[R]               see above.
 *   n                          host copy of offsets[T*B].
 *   U, W, self                 buckets, group width (U % W == 0), own bucket.
 *
 * For lookup i in table t:  g = row_base[t] + ids[i];
 *   dest = self                     (tier 0: served from the local replica)
 *        = (self / W) * W + owner   (tier 1: served inside the own group)
 *        = owner                    (tier 2)
 * Outputs: bucket_offsets[U + 1] (exclusive scan of per-bucket counts,
 * bucket_offsets[U] = n); out_rows[n] = g and out_pos[n] = i, bucket-major and
 * in ascending i inside a bucket (a stable counting sort by dest);
 * tier_counts[3] (may be NULL) = lookups per tier, overwritten.
 *
 * Data faults: an id outside [0, E_t) is routed as row row_base[t]
 * (FS_DEV_BAD_ID); a row_base that is not ascending, or row_base[T] outside
 * [1, 2^32 - 1): the lookups it takes out of [0, row_base[T]) are routed as
 * row 0 (FS_DEV_BAD_ID); tier 3, owner >= U (tier 2) or owner >= W (tier 1) is
 * routed to `self` (FS_DEV_BAD_PLACEMENT; tier 3 is counted under tier 0);
 * bad offsets set FS_DEV_BAD_OFFSETS and leave the outputs unspecified but
 * written in bounds.
 * Host faults: NULL -> FS_ERR_NULL; n < 0, n >= 2^31, T < 1, B < 1,
 * T*B >= 2^31 -> FS_ERR_SIZE; U < 1, U > FS_MAX_BUCKETS, W < 1, U % W != 0,
 * self outside [0, U) -> FS_ERR_CONFIG.
 */
fs_status fs_route_bucketize(
    const int64_t* ids, const int64_t* offsets, int32_t T, int32_t B,
    const int64_t* row_base, const uint32_t* placement,
    int64_t n, int32_t U, int32_t W, int32_t self,
    int64_t* bucket_offsets, int64_t* out_rows, int32_t* out_pos,
    int64_t* tier_counts,
    void* workspace, size_t* workspace_bytes /* host */,
    void* stream, int32_t* dev_status);

/*
 * fs_route_bucketize_noalloc -- fs_route_bucketize for callers that cannot
 * allocate device memory or bring a workspace: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same inputs, outputs,
 * faults and kernels; the workspace is a static device array inside the
 * library, FS_ROUTE_NOALLOC_SCRATCH_BYTES per GPU (held until the process ends).
 * A batch whose workspace would be larger (about 6 bytes per lookup plus
 * 4 * (U + 3) bytes per 2048 lookups: roughly 5 million lookups at U = 64)
 * returns FS_ERR_WORKSPACE and launches nothing.  The call allocates and
 * frees nothing.  The first call on a GPU looks up that GPU's address of the
 * array (a host-side query, no allocation); make that call outside a capture.
 * All calls on one GPU share the array: two calls that overlap in time on one
 * GPU (different streams) race; calls on one stream, or ordered by events, are
 * fine.  Nothing in the array has to survive from call to call or start at zero.
 */
#define FS_ROUTE_NOALLOC_SCRATCH_BYTES (32u << 20)

fs_status fs_route_bucketize_noalloc(
    const int64_t* ids, const int64_t* offsets, int32_t T, int32_t B,
    const int64_t* row_base, const uint32_t* placement,
    int64_t n, int32_t U, int32_t W, int32_t self,
    int64_t* bucket_offsets, int64_t* out_rows, int32_t* out_pos,
    int64_t* tier_counts, void* stream, int32_t* dev_status);

/*
 * fs_seq_gather_fwd -- unpooled sequence lookup (Section 2, "Embedding
 * Pooling": every looked-up row is materialised; Section 3.2 metrics 3 and 4,
 * "rows accessed" and "dynamic memory").
 *
 *   weights[R, D] row-major, `dtype`; rows[*], pos[*] as written by
 *   fs_route_bucketize; for j in [j0, j1): out[pos[j], :] = weights[rows[j], :]
 *   (a bit copy).  out is [n, D]; rows of out whose index is not in
 *   pos[j0..j1) are left untouched.
 *
 * Data faults: rows[j] outside [0, R) or pos[j] outside [0, n): that j is
 * skipped (FS_DEV_BAD_ID).
 * Host faults: NULL; R < 1, n < 0, D < 1, j0 < 0, j0 > j1 (FS_ERR_SIZE);
 * D * sizeof(dtype) not a multiple of 16 or weights/out not 16-byte aligned
 * (FS_ERR_ALIGN).
 */
fs_status fs_seq_gather_fwd(
    const void* weights, int64_t R, int32_t D, fs_dtype dtype,
    const int64_t* rows, const int32_t* pos, int64_t j0, int64_t j1,
    void* out, int64_t n, void* stream, int32_t* dev_status);

/*
 * The two halves of fs_seq_gather_fwd that sit either side of the row exchange
 * (Section 3.2 metric 5, "dynamic communication": the looked-up rows travel
 * from the GPU that owns them back to the GPU that asked, in the order the ids
 * arrived there; the communication-cost table, column "Dynamic Comms").
 *
 * fs_seq_gather_send -- owner side: send[j - j0, :] = weights[rows[j], :] for
 *   j in [j0, j1); send is [j1 - j0, D], contiguous, in bucket order.
 * fs_seq_unbucketize -- requester side: out[pos[j], :] = recv[j - j0, :] for
 *   j in [j0, j1); recv is [j1 - j0, D].
 * fs_seq_unbucketize(send of fs_seq_gather_send) writes the same bits as
 * fs_seq_gather_fwd over the same [j0, j1).
 *
 * Data faults: rows[j] outside [0, R): send row j - j0 is left untouched;
 * pos[j] outside [0, n): that j is skipped (both FS_DEV_BAD_ID).
 * Host faults: as fs_seq_gather_fwd; j1 - j0 >= 2^31 (FS_ERR_SIZE).
 */
fs_status fs_seq_gather_send(
    const void* weights, int64_t R, int32_t D, fs_dtype dtype,
    const int64_t* rows, int64_t j0, int64_t j1,
    void* send, void* stream, int32_t* dev_status);

fs_status fs_seq_unbucketize(
    const void* recv, int32_t D, fs_dtype dtype,
    const int32_t* pos, int64_t j0, int64_t j1,
    void* out, int64_t n, void* stream, int32_t* dev_status);

/*
 * Replica store (Section 3.1, data-parallel placement: a replicated row is
 * held by every GPU and its lookups are served locally; Section 4.3: the
 * replicated rows are the most popular ones, so a small dense array serves a
 * large share of the lookups).
 *
 * fs_replica_build -- copies the selected rows into a dense array and writes
 *   the map from row to slot:
 *     k' = k if num_selected == NULL else min(k, *num_selected)   (device scalar)
 *     store[s, :] = weights[sel_rows[s], :]          for s in [0, k')
 *     slot_of_row[r] = the smallest s < k' with sel_rows[s] == r, else -1,
 *                      for every r in [0, R)   (overwritten completely)
 *   store is [k, D]; rows k'.. of it are left untouched.  sel_rows / num_selected
 *   are what fs_plan_replication writes.
 *   Data faults: sel_rows[s] outside [0, R): store row s is left untouched and
 *   no slot points to it (FS_DEV_BAD_ID).
 *   Host faults: NULL; R < 1, D < 1, k < 0, k >= 2^31 (FS_ERR_SIZE); alignment
 *   as fs_seq_gather_fwd.
 *
 * fs_seq_gather_fwd_replica -- fs_seq_gather_fwd, except that a row r with
 *   slot_of_row[r] = s >= 0 is read from store[s, :] instead of weights[r, :].
 *   With a store built from the same weights the output bits are those of
 *   fs_seq_gather_fwd.  A slot >= k skips that lookup (FS_DEV_BAD_ID).
 */
fs_status fs_replica_build(
    const void* weights, int64_t R, int32_t D, fs_dtype dtype,
    const int64_t* sel_rows, int64_t k, const int64_t* num_selected,
    void* store, int32_t* slot_of_row, void* stream, int32_t* dev_status);

fs_status fs_seq_gather_fwd_replica(
    const void* weights, int64_t R, int32_t D, fs_dtype dtype,
    const void* store, int64_t k, const int32_t* slot_of_row,
    const int64_t* rows, const int32_t* pos, int64_t j0, int64_t j1,
    void* out, int64_t n, void* stream, int32_t* dev_status);

/*
 * Replica slots handed over by the router (Section 3.1: a replicated row has no
 * owner to name, every GPU holds it; Section 4.3: the replicated rows are the
 * few most popular ones, which most lookups ask for).  The owner bits of a
 * tier-0 placement entry are free, so they can carry the row's slot in the
 * replica store; the router reads the entry of every lookup anyway and can hand
 * each lookup's slot to the gather, which then needs no load of the slot map in
 * front of the load of the row.
 *
 * fs_replica_tag_slots -- for every row r in [0, R) whose placement entry is
 *   tier 0: owner bits = slot_of_row[r] if that is >= 0, else FS_OWNER_MASK
 *   ("no slot").  Entries of the other tiers are left as they are.
 *   slot_of_row is what fs_replica_build wrote.
 *   Data faults: a slot >= FS_OWNER_MASK cannot be carried: "no slot" is
 *   written (FS_DEV_BAD_ID).  Host faults: NULL; R < 1 (FS_ERR_SIZE).
 *
 * fs_route_bucketize_slots -- fs_route_bucketize (same arguments, same outputs,
 *   same faults), and in addition out_slots[j], j in [0, n): the slot that the
 *   placement entry of out_rows[j] carries if that entry is tier 0 and its
 *   owner bits are not FS_OWNER_MASK, else -1.  Meant for a placement whose
 *   tier-0 entries were written by fs_replica_tag_slots (fs_route_bucketize
 *   itself ignores those bits).  The workspace is larger by 4 n bytes; ask with
 *   workspace == NULL.
 *
 * fs_seq_gather_fwd_slots -- fs_seq_gather_fwd, except that lookup j with
 *   slots[j] = s >= 0 is read from store[s, :] instead of weights[rows[j], :]
 *   (slots is indexed like rows and pos).  With a store built from the same
 *   weights and slots from fs_route_bucketize_slots the output bits are those
 *   of fs_seq_gather_fwd.  A slot >= k skips that lookup (FS_DEV_BAD_ID); other
 *   faults as fs_seq_gather_fwd_replica.
 */
fs_status fs_replica_tag_slots(
    uint32_t* placement, int64_t R, const int32_t* slot_of_row, void* stream, int32_t* dev_status);

fs_status fs_route_bucketize_slots(
    const int64_t* ids, const int64_t* offsets, int32_t T, int32_t B,
    const int64_t* row_base, const uint32_t* placement,
    int64_t n, int32_t U, int32_t W, int32_t self,
    int64_t* bucket_offsets, int64_t* out_rows, int32_t* out_pos, int32_t* out_slots,
    int64_t* tier_counts,
    void* workspace, size_t* workspace_bytes /* host */,
    void* stream, int32_t* dev_status);

fs_status fs_seq_gather_fwd_slots(
    const void* weights, int64_t R, int32_t D, fs_dtype dtype,
    const void* store, int64_t k, const int64_t* rows, const int32_t* slots, const int32_t* pos,
    int64_t j0, int64_t j1, void* out, int64_t n, void* stream, int32_t* dev_status);

/*
 * fs_seq_grad_bwd -- backward of the sequence lookup (Section 3.2 metrics 4-6:
 * the gradient of every materialised row flows back to the row's owner, where
 * duplicates of one row are summed before the update).
 *
 *   grad_out[n, D] in `dtype`; for every distinct row r among rows[j0..j1):
 *       row_grads[u(r), :] = sum over {j : rows[j] == r} of f32(grad_out[pos[j], :])
 *   uniq_rows[u] ascending, u(r) its rank; *num_unique = number of distinct
 *   rows.  uniq_rows and row_grads hold cap_unique rows; if there are more
 *   distinct rows, the first cap_unique are written, *num_unique is still the
 *   true count and FS_DEV_UNIQUE_OVERFLOW is set.
 *
 * Summation order (fp32, round-to-nearest-even, no fused multiply-add,
 * subnormals kept).  Sort the lookups by (row asc, pos asc), k = 0 .. m-1 the
 * sorted index, m = j1 - j0.  A partial sum starts at the first k of each
 * row's run and at every k that is a multiple of FS_BWD_TILE; a partial is
 * accumulated left to right starting from its first term; the row's gradient
 * is the left-to-right sum of its partials.
 *   variant 0: exactly that order, bit for bit, on every run.
 *   variant 1: partials as above, combined with fp32 atomic adds in arbitrary
 *              order: within 1e-5 of the fp64 sum, relative to
 *              max(|sum|, 2-norm of the terms), per element.
 *
 * Precondition (true of every fs_route_bucketize output and any [j0, j1) of
 * it): lookups of one row appear with ascending pos in j order.  A violation
 * sets FS_DEV_POS_ORDER; uniq_rows and *num_unique are then still exact, and
 * every row's gradient is still the sum of its terms, but in an order that is
 * not the stated one (the terms of a row are taken in j order), so only the
 * bound of variant 1 holds for the values.
 *
 * Data faults: rows[j] outside [0, R) or pos[j] outside [0, n) is replaced by
 * row 0 / pos 0 (FS_DEV_BAD_ID), result unspecified but in bounds.
 * Host faults: as fs_seq_gather_fwd; R >= 2^32 - 1, cap_unique < 0
 * (FS_ERR_SIZE); variant not 0/1 (FS_ERR_CONFIG).
 */
fs_status fs_seq_grad_bwd(
    const void* grad_out, int64_t n, int32_t D, fs_dtype dtype,
    const int64_t* rows, const int32_t* pos, int64_t j0, int64_t j1, int64_t R,
    int32_t variant,
    int64_t* uniq_rows, float* row_grads, int64_t cap_unique, int64_t* num_unique,
    void* workspace, size_t* workspace_bytes /* host */,
    void* stream, int32_t* dev_status);

/*
 * The backward's sort as a step of its own, so that one sort per batch serves
 * every pass that wants the lookups in row order (Section 3.2, metrics 4-6: the
 * same lookups are touched by the forward and by the backward pass).
 *
 * fs_sort_lookups -- the lookups rows[j0..j1), pos[j0..j1) in (row asc, pos asc)
 *   order as 32-bit pairs: sorted_rows[k], sorted_pos[k], k in [0, j1 - j0).
 *   The sort is stable by row alone, so this is the stated order under
 *   fs_seq_grad_bwd's precondition (equal rows come with ascending pos in j).
 *   Data faults: rows[j] outside [0, R) / pos[j] outside [0, n) are replaced by
 *   row 0 / position 0 (FS_DEV_BAD_ID).  Host faults: as fs_seq_grad_bwd.
 *
 * fs_seq_grad_bwd_sorted -- fs_seq_grad_bwd on lookups already in that order
 *   (m pairs, e.g. as fs_sort_lookups wrote them): same outputs, same summation
 *   order, bit for bit; its workspace holds only the run counts and the
 *   carries.  Data faults: a position >= n reads row 0 of grad_out, a row >= R
 *   is passed through to uniq_rows (both FS_DEV_BAD_ID); rows that are not
 *   ascending set FS_DEV_NOT_SORTED: every maximal stretch of equal rows is then
 *   summed as if it were a row of its own, and everything stays in bounds.
 *
 * fs_seq_gather_fwd_sorted -- fs_seq_gather_fwd over such pairs:
 *   out[sorted_pos[k], :] = weights[sorted_rows[k], :] for k in [0, m).  In row
 *   order every distinct row is fetched from memory once and its repeats follow
 *   at once (where the repeated rows do not fit the caches in bucket order, this
 *   is the cheaper order; where they do, bucket order writes more densely).
 *   Data faults and host faults as fs_seq_gather_fwd.
 */
fs_status fs_sort_lookups(
    const int64_t* rows, const int32_t* pos, int64_t j0, int64_t j1, int64_t R, int64_t n,
    uint32_t* sorted_rows, uint32_t* sorted_pos,
    void* workspace, size_t* workspace_bytes /* host */,
    void* stream, int32_t* dev_status);

fs_status fs_seq_grad_bwd_sorted(
    const void* grad_out, int64_t n, int32_t D, fs_dtype dtype,
    const uint32_t* sorted_rows, const uint32_t* sorted_pos, int64_t m, int64_t R,
    int32_t variant,
    int64_t* uniq_rows, float* row_grads, int64_t cap_unique, int64_t* num_unique,
    void* workspace, size_t* workspace_bytes /* host */,
    void* stream, int32_t* dev_status);

fs_status fs_seq_gather_fwd_sorted(
    const void* weights, int64_t R, int32_t D, fs_dtype dtype,
    const uint32_t* sorted_rows, const uint32_t* sorted_pos, int64_t m,
    void* out, int64_t n, void* stream, int32_t* dev_status);

/*
 * fs_plan_replication -- profile and choose the rows to replicate
 * (Section 4.1: per-row appearance counts; Section 4.3: rows are taken in
 * descending frequency order and, for a given amount of extra memory, the
 * best hybrid is the prefix that fits; Section 4.6: several tables are merged
 * into one distribution).
 *
 *   flags & FS_PLAN_ACCUMULATE  counts[row_base[t] + ids[i]] += 1 for every
 *                               lookup of the jagged sample (ids, offsets, T, B
 *                               as in fs_route_bucketize; counts is in/out, so
 *                               calls accumulate).  A count that would pass
 *                               2^32 - 1 stays there (FS_DEV_COUNT_OVERFLOW).
 *   flags & FS_PLAN_SELECT      order rows by (count desc, g asc); candidates
 *                               are rows with count > 0 (all rows with
 *                               FS_PLAN_ALLOW_ZERO);
 *                               k = min(budget_bytes / bytes_per_row, #candidates);
 *                               sel_rows[0..k) = the first k in that order,
 *                               *num_selected = k.  sel_rows holds
 *                               min(R, budget_bytes / bytes_per_row) entries.
 *   flags & FS_PLAN_TAG         (with SELECT) the tier bits of placement[g]
 *                               are set to 0 for the k selected rows.
 * Pointers a flag does not use may be NULL.
 * Data faults: an id outside its table is counted as the table's first row,
 * a row_base that takes a lookup outside [0, R) drops it (both FS_DEV_BAD_ID);
 * bad offsets (FS_DEV_BAD_OFFSETS) count nothing.
 * Host faults: NULL; n, R, T, B as above; budget_bytes < 0 or
 * bytes_per_row < 1 (FS_ERR_SIZE); unknown flag bits, TAG without SELECT
 * (FS_ERR_CONFIG); with ACCUMULATE, ids not 8-byte or counts not 4-byte
 * aligned (FS_ERR_ALIGN).
 */
#define FS_PLAN_ACCUMULATE 1
#define FS_PLAN_SELECT 2
#define FS_PLAN_TAG 4
#define FS_PLAN_ALLOW_ZERO 8

fs_status fs_plan_replication(
    const int64_t* ids, const int64_t* offsets, int32_t T, int32_t B,
    const int64_t* row_base, int64_t n, int64_t R,
    uint32_t* counts, int32_t flags,
    int64_t budget_bytes, int64_t bytes_per_row,
    int64_t* sel_rows, int64_t* num_selected,
    uint32_t* placement,
    void* workspace, size_t* workspace_bytes /* host */,
    void* stream, int32_t* dev_status);

/*
 * fs_plan_tiers -- the tier planner (Section 4.2: per-row costs are the cost
 * tables of Section 3.2 with E = 1 and L = p, and the row probability at which
 * two strategies cost the same is a breakpoint; Section 4.3: rows are walked in
 * descending frequency order and the points A, B, C of the cost curve are where
 * the walk crosses the breakpoints; Section 4.5: three tiers).
 *
 * p_i = counts[i] / num_samples.  Per row, in units of D * sizeof(dtype):
 *   replicated (DP) instead of row-wise:  memory  dp_multiplier - 1/U - B p
 *                                         traffic 1/ar_global - 2 B p / a2a_global
 *   Flex instead of row-wise:             memory  dp_multiplier/W - 1/U
 *                                         traffic 2 B p / a2a_intra + 1/(W ar_cross) - 2 B p / a2a_global
 * Candidates are the rows with counts > 0 in (count desc, row asc) order, K of
 * them.  All comparisons are exact (integers, cross-multiplied).
 *   cuts[FS_CUT_CANDIDATES] = K
 *   cuts[FS_CUT_A]     rows whose DP memory term is <= 0            (most memory saved)
 *   cuts[FS_CUT_B]     longest prefix whose DP memory terms sum to <= 0 (memory neutral)
 *   cuts[FS_CUT_C]     rows whose DP traffic term is <= 0           (least traffic)
 *   cuts[FS_CUT_FLEX]  rows whose Flex traffic term is <= 0
 *   tiers == 2:  n_dp = B rounded down to a multiple of granule, n_flex = 0
 *   tiers == 3:  n_dp = A rounded down; n_flex = the most rows after them that
 *                the memory saved by the n_dp rows pays for, not beyond
 *                cuts[FS_CUT_FLEX], rounded down to a multiple of granule
 *   cuts[FS_CUT_N_DP], cuts[FS_CUT_N_FLEX]; cuts[FS_CUT_SUM_ALL / _DP / _FLEX] =
 *   the counts summed over all candidates / the DP tier / the Flex tier (their
 *   ratios are the predicted share of lookups each tier serves).
 * sorted_rows[i], i < min(cap, n_dp + n_flex): the chosen rows in that order
 * (may be NULL with cap = 0).  placement (may be NULL): the n_dp rows get tier
 * 0 (owner bits kept), Flex row number j gets tier 1 with owner j % W; other
 * entries are left as they are.  cuts is device memory, FS_TIER_CUTS entries.
 *
 * Host faults: NULL; R < 1, R >= 2^32 - 1, cap < 0 (FS_ERR_SIZE); tiers not 2
 * or 3, num_samples outside [1, 2^40), B outside [1, 2^31), U outside
 * [1, FS_MAX_BUCKETS], W < 1, U % W != 0, dp_multiplier outside [1, 1024],
 * granule outside [1, 2^20], a bandwidth outside [1, 2^20) (FS_ERR_CONFIG);
 * workspace as everywhere.
 */
typedef struct fs_tier_params {
    int64_t num_samples;   /* profiled samples behind counts (per table) */
    int64_t B;             /* local batch size per GPU */
    int32_t U, W;          /* GPUs, GPUs per group */
    int32_t dp_multiplier; /* static memory of a replicated row in row sizes (Table 2: 6) */
    int32_t granule;       /* tier sizes are multiples of this */
    int64_t a2a_global, a2a_intra, ar_global, ar_cross;   /* bandwidths, one common unit */
} fs_tier_params;

#define FS_CUT_CANDIDATES 0
#define FS_CUT_A 1
#define FS_CUT_B 2
#define FS_CUT_C 3
#define FS_CUT_FLEX 4
#define FS_CUT_N_DP 5
#define FS_CUT_N_FLEX 6
#define FS_CUT_SUM_ALL 7
#define FS_CUT_SUM_DP 8
#define FS_CUT_SUM_FLEX 9
#define FS_TIER_CUTS 10

fs_status fs_plan_tiers(
    const uint32_t* counts, int64_t R, const fs_tier_params* params /* host */, int32_t tiers,
    int64_t* sorted_rows, int64_t cap, int64_t* cuts, uint32_t* placement,
    void* workspace, size_t* workspace_bytes /* host */,
    void* stream, int32_t* dev_status);

/*
 * fs_sparse_update -- one optimizer step on the rows fs_seq_grad_bwd produced
 * gradients for (the step that follows the backward pass of Section 3.2; the
 * replicated strategy's static-memory factor in the memory-cost table is this
 * optimizer state and gradient memory).
 *
 *   for u < min(cap_unique, *num_unique) (cap_unique if num_unique == NULL), r = uniq_rows[u], g = row_grads[u, :]:
 *     FS_OPT_SGD              w[r, :] -= lr g
 *     FS_OPT_ADAGRAD          state[r, :] += g^2;            w[r, :] -= lr g / (sqrt(state[r, :]) + eps)
 *     FS_OPT_ADAGRAD_ROWWISE  state[r] += mean over the row of g^2;  w[r, :] -= lr g / (sqrt(state[r]) + eps)
 *   weights[R, D] in `dtype`, updated in place; state is float32, [R, D] or [R]
 *   (unused and may be NULL for SGD).  If store / slot_of_row (both or neither;
 *   as fs_replica_build wrote them) are given, a row with a slot gets its new
 *   values there as well.
 * Arithmetic: float32, one IEEE operation at a time, the new weight rounded
 * once to `dtype` (nearest even).  Against the same rules in double precision:
 * within one unit in the last place of `dtype`; state within 1e-6 relative.
 * uniq_rows must not name a row twice (true of fs_seq_grad_bwd's output):
 * duplicates race.
 * Data faults: uniq_rows[u] outside [0, R) is skipped, a slot >= k is not
 * mirrored (both FS_DEV_BAD_ID).
 * Host faults: NULL; R < 1, D < 1, cap_unique < 0, k < 0 (FS_ERR_SIZE); unknown
 * optimizer (FS_ERR_CONFIG); D * sizeof(dtype) not a multiple of 16 or a
 * pointer not 16-byte aligned (FS_ERR_ALIGN).
 */
#define FS_OPT_SGD 0
#define FS_OPT_ADAGRAD_ROWWISE 1
#define FS_OPT_ADAGRAD 2

fs_status fs_sparse_update(
    void* weights, int64_t R, int32_t D, fs_dtype dtype,
    const int64_t* uniq_rows, const float* row_grads, int64_t cap_unique, const int64_t* num_unique,
    int32_t optimizer, float lr, float eps, float* state,
    void* store, const int32_t* slot_of_row, int64_t k,
    void* stream, int32_t* dev_status);

/*
 * fs_seq_grad_bwd_update -- the backward pass and the optimizer step in one
 * call (the step that follows the backward pass of Section 3.2; most distinct
 * rows of a power-law batch are looked up once, and their gradient need not
 * travel through memory to be applied).  Takes the lookups in row order, as
 * fs_sort_lookups writes them.  Same result as
 *     fs_seq_grad_bwd_sorted(..., variant 0, ...) followed by
 *     fs_sparse_update(weights, ..., uniq_rows, row_grads, cap_unique, num_unique, ...)
 * bit for bit in weights, state and store, in uniq_rows and *num_unique, and
 * in row_grads[u, :] for every row looked up more than once; row_grads[u, :]
 * of a row looked up ONCE is left unwritten (its gradient is applied straight
 * from grad_out).  Only rows with u < cap_unique are updated.
 * Data faults: as the two calls; with FS_DEV_NOT_SORTED the result is
 * unspecified (a row that appears in two stretches is updated twice, possibly
 * at the same time), in bounds.
 * Host faults: those of the two calls.
 */
fs_status fs_seq_grad_bwd_update(
    const void* grad_out, int64_t n, int32_t D, fs_dtype dtype,
    const uint32_t* sorted_rows, const uint32_t* sorted_pos, int64_t m, int64_t R,
    void* weights, int32_t optimizer, float lr, float eps, float* state,
    void* store, const int32_t* slot_of_row, int64_t k,
    int64_t* uniq_rows, float* row_grads, int64_t cap_unique, int64_t* num_unique,
    void* workspace, size_t* workspace_bytes /* host */,
    void* stream, int32_t* dev_status);

/*
 * fs_cost_model -- the analytical per-GPU costs of one sequence embedding
 * table in one training iteration under a uniform strategy (Section 3.2: the
 * six metrics; the memory-cost and communication-cost tables, cell by cell).
 * Host arithmetic in double precision, no GPU work.
 *   out[FS_COST_STATIC_MEMORY]   bytes
 *   out[FS_COST_INPUT_DIST]      ids to communicate before the lookups
 *   out[FS_COST_ROWS_ACCESSED]   row elements looked up on this GPU
 *   out[FS_COST_DYNAMIC_MEMORY]  bytes (each pass)
 *   out[FS_COST_DYNAMIC_COMM]    bytes / bandwidth (each pass)
 *   out[FS_COST_STATIC_COMM]     bytes / bandwidth (backward pass only)
 * Cells the tables mark "N/A" are 0.  With E = 1 and L = p the same cells are
 * the per-row costs of Section 4.2.
 * Faults: NULL; a parameter that is not positive (E, L: negative), NaN, or an
 * unknown strategy (FS_ERR_CONFIG).
 *
 * fs_tier_traffic -- what the tiers of a routed batch mean for the row
 * exchange (Section 6.2 reports it as the reduction of the global all-to-all):
 * from tier_counts[3] as fs_route_bucketize writes them (copied to the host),
 *   out[0] bytes one direction of one pass would move if every row were sharded,
 *   out[1] bytes left in the global all-to-all (tier 2),
 *   out[2] bytes in the intra-group all-to-all (tier 1),
 *   out[3] share of the global all-to-all avoided, (tier 0 + tier 1) / all.
 */
typedef struct fs_cost_params {
    double E, D, dtype_bytes, L;          /* rows, dimension, bytes per scalar, average length */
    double W, N, B;                       /* GPUs per node, nodes (U = N * W), local batch */
    double a2a_global, a2a_intra, ar_global, ar_cross;   /* bytes per second */
    double dp_multiplier;                 /* static memory of a replicated row in row sizes (6) */
} fs_cost_params;

#define FS_STRATEGY_RW 0
#define FS_STRATEGY_CW 1
#define FS_STRATEGY_DP 2
#define FS_STRATEGY_FLEX 3
#define FS_COST_STATIC_MEMORY 0
#define FS_COST_INPUT_DIST 1
#define FS_COST_ROWS_ACCESSED 2
#define FS_COST_DYNAMIC_MEMORY 3
#define FS_COST_DYNAMIC_COMM 4
#define FS_COST_STATIC_COMM 5
#define FS_COST_METRICS 6

fs_status fs_cost_model(const fs_cost_params* params /* host */, int32_t strategy, double* out /* host, 6 */);
fs_status fs_tier_traffic(const int64_t* tier_counts /* host, 3 */, int32_t D, int32_t dtype_bytes,
                          double* out /* host, 4 */);

/* ---- helpers ---------------------------------------------------------- */

/* Library version, major * 1000 + minor. */
int32_t fs_version(void);

/* FS_BWD_TILE as compiled into the library. */
int32_t fs_bwd_tile(void);

/*
 * Plain 128-bit copy kernel, dst[0..bytes) = src[0..bytes).  Not part of the method: the
 * benchmark uses it as the measured copy bandwidth of the box and the profiles use it to
 * scale the HBM byte counters (a launch of known traffic).  bytes must be a multiple of 16,
 * both pointers 16-byte aligned (FS_ERR_ALIGN), bytes >= 0 (FS_ERR_SIZE).
 */
fs_status fs_util_copy(void* dst, const void* src, int64_t bytes, void* stream);

/*
 * Reference stream for the backward's traffic shape (not part of the method; the benchmark prints
 * its rate beside the kernels'): src is read once in 512-byte pieces by groups that each walk 256
 * consecutive pieces; with pieces_per_write = w > 0 a group writes its running 32-bit-integer sum
 * of the pieces so far as one 1 KB row of dst after every w pieces (16 columns of 32 bits repeated
 * over the row; group g's rows start at row g * ceil(256 / w), wrapping around dst).  w = 0 only
 * reads.  src_bytes a multiple of 512, dst_bytes of 1024, both 16-byte aligned (FS_ERR_ALIGN).
 */
fs_status fs_util_read_write_mix(const void* src, int64_t src_bytes, int32_t pieces_per_write,
                                 void* dst, int64_t dst_bytes, void* stream);

/*
 * Opt-in per-kernel timing.  fs_prof_begin(max_records) makes every later
 * kernel launch of this library (on any stream) bracketed by a pair of HIP
 * events; fs_prof_end() synchronises those events, writes up to `cap` records
 * (kernel name, NUL-terminated, 48 bytes each, into names; milliseconds into
 * ms; all host memory), returns the number of records taken and switches
 * timing off.  Not thread-safe; for benchmarks only.
 */
fs_status fs_prof_begin(int32_t max_records);
/* Restricts the timing to the kernels named in a comma-separated list ("gather_rows,bwd_segreduce");
 * NULL or "" = every kernel again.  The names are those fs_prof_end reports.  Each timed launch
 * costs two event records on its stream, so a benchmark that needs a few kernels only names them. */
fs_status fs_prof_only(const char* names /* host */);
int32_t fs_prof_end(char* names /* host, cap*48 */, float* ms /* host */, int32_t cap);

#ifdef __cplusplus
}
#endif
#endif /* FLEXSHARD_H */
