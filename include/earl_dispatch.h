/*
 * earl_dispatch.h - C ABI of the MI355X (gfx950) re-layout library for intermediate RL rollout
 * batches: the on-device part of the paper's Data Dispatcher (Section 2, "Data Dispatcher").
 *
 * The paper states the operation as "plan, then move": the dispatcher looks at the current data
 * layout and at the parallelism configuration of the consumer, decides which worker needs which
 * part of every sequence, and sends each part straight from where it was computed to where it is
 * needed (an all-to-all), instead of gathering the whole batch on one node and scattering it.
 * The two calls of this library are those two halves:
 *
 *   earl_plan_build(lengths, src_layout, dst_layout)   who reads what from where, and where it lands
 *   earl_dispatch(fields, plan)                        materialise every destination shard
 *
 * The batch (Section 1) is a set of per-token tensors ("fields": token ids, masks, log-probabilities,
 * advantages, auxiliary vectors) over N ragged sequences.  One GPU materialises all D*C destination
 * shards in its own HBM.
 *
 * Conventions for every function:
 *   - returns an earl_status (int32); never throws, never aborts;
 *   - "device" pointers are HIP device pointers on the current device, "host" pointers are ordinary
 *     host memory; the caller owns every buffer it passes, scratch included; the library allocates
 *     no device memory;
 *   - work is enqueued on the HIP stream passed as `void* hip_stream` (a hipStream_t; NULL = the
 *     default stream); device buffers must stay valid until that work has finished;
 *   - calls on the same plan must come from one thread at a time.
 */
#ifndef EARL_DISPATCH_H_
#define EARL_DISPATCH_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  EARL_OK = 0,
  EARL_INVALID_ARG = 1,        /* null pointer, size out of range, misaligned buffer, L[i] < 1,
                                  seq_group out of range (the last two are found on the device and
                                  reported by earl_plan_get_summary / earl_dispatch)              */
  EARL_SEQ_EXCEEDS_BUDGET = 2, /* some padded sequence is longer than mb_token_budget            */
  EARL_CAPACITY = 3,           /* workspace or a destination/source buffer is too small          */
  EARL_HIP_ERROR = 4,          /* a HIP runtime call failed; see earl_last_error_message()       */
  EARL_NO_FEASIBLE_CONFIG = 5  /* earl_selector.h: every configuration failed in this range      */
} earl_status;

/* Limits (EARL_INVALID_ARG beyond them). */
#define EARL_MAX_SEQS (1 << 20)       /* N                                   */
#define EARL_MAX_DP 1024              /* D                                   */
#define EARL_MAX_SP 64                /* C                                   */
#define EARL_MAX_SRC_SHARDS 4096      /* S = G*R                             */
#define EARL_MAX_FIELDS 32            /* fields per earl_dispatch call       */
#define EARL_MAX_ROW_BYTES (1 << 20)  /* scalar_bytes * width                */

/*
 * Where the batch lives now ("current data distribution layout", Section 2).  The N sequences are
 * stored in G groups; group g exists as R identical replicas (e.g. the R tensor-parallel workers of
 * one rollout engine all hold its outputs), i.e. S = G*R shard buffers per field, replica t of group
 * g being shard g*R + t.
 *   seq_group  device int32[N], group holding sequence i; NULL = groups own equal contiguous index
 *              ranges, g = floor(i*G/N).
 *   seq_row    device int64[N], first row of sequence i inside its group's buffers; NULL = the
 *              group's sequences are packed in index order (the library computes the offsets by a
 *              segmented prefix scan of the lengths).
 * The plan reads the k-th of a group's n sequences from replica floor(k*R/n), so every row is read
 * once and each replica serves one contiguous share.
 */
typedef struct {
  int32_t n_groups;     /* G >= 1 */
  int32_t replication;  /* R >= 1 */
  const int32_t* seq_group;
  const int64_t* seq_row;
} earl_src_layout;

/*
 * Where the batch has to go ("parallelism configuration", Section 2): dp data-parallel ranks, each
 * split over sp sequence-parallel ranks; destination shard q = r*sp + c.
 *   zigzag            1: a sequence is cut into 2*sp chunks and SP rank c holds chunks c and
 *                     2*sp-1-c (equal causal-attention work); 0: sp contiguous chunks.
 *   pad_multiple      every chunk is padded to a multiple of this many rows (>= 1).
 *   balance_policy    0 = longest-first list scheduling on padded lengths (ties: lower index, lower
 *                     rank); 1 = sorted snake deal: longest first in rounds of dp, left to right in
 *                     even rounds and right to left in odd ones (no serial chain; equal sequence
 *                     counts per rank, loads within one padded length of each other);
 *                     2 = as 0, but a rank's load grows by the SQUARE of the padded length (equal
 *                     causal-attention work instead of equal token counts); padded lengths must
 *                     not exceed 2^21 then (EARL_INVALID_ARG, reported like a bad length).
 *                     rank_load in the summary is in padded tokens under every policy.
 *   equal_mb          1: every DP rank reports n_mb_max micro-batches; ranks that need fewer get
 *                     empty ones appended (no sequence, no row; their entries in mb_seq_start /
 *                     mb_row_start repeat the rank's totals, their cu_seqlens array is the single
 *                     entry 0), so that all ranks run the same number of steps.  Needs
 *                     dp * (n_seqs + 1) <= 2^27.  0: each rank reports what next-fit produced.
 *   mb_token_budget   a micro-batch holds whole sequences whose padded lengths sum to at most this.
 */
typedef struct {
  int32_t dp, sp, zigzag, pad_multiple, balance_policy, equal_mb;
  int64_t mb_token_budget;
} earl_dst_layout;

/*
 * One field: `width` scalars of `scalar_bytes` (1, 2, 4 or 8) bytes per token, row-major, rows
 * contiguous.  All pointer arrays are HOST arrays of DEVICE pointers.
 *   pad_scalar          padding rows are filled with `width` copies of its low scalar_bytes bytes.
 *   src_shard_ptrs[S]   shard buffers in the source layout (aligned to scalar_bytes).  A pointer may
 *                       be NULL if the plan reads no row from that shard.
 *   dst_shard_ptrs[D*C] destination shards (16-byte aligned; NULL allowed for a shard of 0 rows).
 *   dst_capacity_rows   rows each destination buffer can hold; EARL_CAPACITY if fewer than needed.
 *   src_capacity_rows   rows each source buffer holds, or NULL to skip the check.
 *   per_sequence        0: the source holds one row per token (the normal case).  1: the source holds
 *                       ONE row per sequence (row k of a group's buffer = its k-th sequence in index
 *                       order, whatever seq_row says) and the dispatch broadcasts it to every real
 *                       token of the sequence while it copies (e.g. a sequence-level advantage or
 *                       reward, Section 5 of the paper); padding rows get pad_scalar.  Needs
 *                       scalar_bytes * width in {1, 2, 4, 8} and source buffers aligned to that;
 *                       not accepted by earl_dispatch_inverse.
 *   nonzero_counts      NULL, or device int64[D*C][n_mb_max] (8-byte aligned): while the field is
 *                       copied, entry [q][b] receives the number of non-zero scalars among the REAL
 *                       rows of destination shard q that lie in micro-batch b of its DP rank
 *                       (entries of micro-batches a rank does not have become 0; padding rows never
 *                       count).  For a 0/1 loss mask this is the token count every (shard,
 *                       micro-batch) normalises its loss by.  Needs a per-token field with
 *                       scalar_bytes * width < 16; not accepted by earl_dispatch_inverse.  The
 *                       array is cleared and filled on the stream by earl_dispatch.
 *   nonzero_counts_capacity  entries the array holds; EARL_CAPACITY if fewer than D*C*n_mb_max.
 * Source and destination buffers must not overlap.
 */
typedef struct {
  int32_t scalar_bytes;
  int32_t width;
  uint64_t pad_scalar;
  const void* const* src_shard_ptrs;
  void* const* dst_shard_ptrs;
  const int64_t* dst_capacity_rows;
  const int64_t* src_capacity_rows;
  int32_t per_sequence;
  int64_t* nonzero_counts;
  int64_t nonzero_counts_capacity;
} earl_field;

typedef struct earl_plan earl_plan; /* host object owned by the library */

/*
 * Host copy of the plan's totals.  The arrays belong to the plan and stay valid until
 * earl_plan_destroy.  Flat-array sizes are needed to size the buffers of earl_plan_export.
 */
typedef struct {
  int32_t n_seqs, n_src_shards, n_dst_shards, chunks_per_seq; /* N, S, D*C, K               */
  int32_t n_segments;        /* N*K                                                          */
  int32_t n_mb_max;          /* largest micro-batch count over DP ranks                      */
  int32_t cu_seqlens_len;    /* N + sum n_mb                                                 */
  int32_t mb_table_len;      /* sum (n_mb + 1)                                               */
  int64_t total_real_rows, total_dst_rows;
  int64_t rank_load_min, rank_load_max;  /* padded tokens on the least / most loaded DP rank */
  const int64_t* shard_rows;       /* [D*C] rows of every destination shard                  */
  const int64_t* src_rows_needed;  /* [S]   rows every source shard buffer must hold         */
  const int64_t* src_seqs_needed;  /* [S]   the same for per_sequence fields (rows = sequences) */
  const int32_t* n_seq;            /* [D]   sequences per DP rank                            */
  const int32_t* n_mb;             /* [D]   micro-batches per DP rank                        */
  const int64_t* rank_load;        /* [D]   padded tokens per DP rank                        */
  const int64_t* a2a_counts;       /* [S][D*C] real rows read from shard s for shard q: the split
                                      sizes of the all-to-all of Section 2                     */
} earl_plan_summary;

/* Bytes of device workspace earl_plan_build needs for n_seqs sequences and these layouts.
 * (This call, earl_plan_get_summary, the two exports, earl_plan_destroy and the status texts are
 * bookkeeping around the plan; no passage of the paper defines them.) */
int32_t earl_plan_workspace_bytes(int32_t n_seqs, const earl_src_layout* src,
                                  const earl_dst_layout* dst, size_t* out_bytes);

/*
 * Computes the dispatch plan on the device (asynchronously on the stream).  This is the decision
 * part of Section 2, "Data Dispatcher" (dispatch logic that follows the current data layout and the
 * consumer's parallelism configuration, every piece sent from where it was computed to where it is
 * needed); the paper gives no rules, the ones below are this library's:
 *   source row offsets (segmented scan of lengths per group) and the replica each sequence is read
 *   from; chunk length m = P*ceil(ceil(L/K)/P) with K = 2*sp (zigzag, sp > 1) or sp, padded length
 *   K*m; longest-first assignment of sequences to DP ranks (ties: lower index, lower rank);
 *   ascending-index order inside a rank; next-fit micro-batches under the budget; destination row
 *   offsets; one segment per (sequence, chunk); a2a_counts; cu_seqlens.
 * lengths_dev: device int32[n_seqs].  workspace_dev: device memory, 256-byte aligned, at least
 * earl_plan_workspace_bytes() bytes, owned by the caller and in use until earl_plan_destroy (and
 * until all dispatches of the plan have finished).  *out_plan receives the new plan on EARL_OK.
 * Errors in the data itself (a length < 1, a group out of range, a sequence over the budget) are
 * found on the device and reported by the first earl_plan_get_summary / earl_dispatch.
 */
int32_t earl_plan_build(const int32_t* lengths_dev, int32_t n_seqs, const earl_src_layout* src,
                        const earl_dst_layout* dst, void* workspace_dev, size_t workspace_bytes,
                        void* hip_stream, earl_plan** out_plan);

/* Waits for the plan's totals (once per plan), copies them to the host and returns the plan's
 * status (EARL_OK, EARL_INVALID_ARG, EARL_SEQ_EXCEEDS_BUDGET, EARL_HIP_ERROR).  The plan kernel
 * stores its totals into a mailbox in pinned host memory and the call polls it (for a quarter of
 * a millisecond, then it waits for the stream); the mailboxes are 1 MiB that the library allocates
 * at the first earl_plan_build of the process and keeps until the process ends.  A plan whose
 * totals exceed 16 KiB (large a2a_counts), or that finds all 64 mailboxes held by plans that
 * were built and not yet asked for their summary, is copied from the device instead. */
int32_t earl_plan_get_summary(earl_plan* plan, earl_plan_summary* out);

/*
 * Copies per-sequence and per-rank plan arrays to HOST buffers (any pointer may be NULL to skip).
 * Indexed by sequence i, length N: rank, slot (position inside its rank), mb (micro-batch inside
 * its rank), dst_row (first row in every shard of its rank), seq_shard (shard buffer it is read
 * from), seq_row (first source row).  seq_ids[N]: sequences of rank 0 in packing order, then rank
 * 1, ...  mb_seq_start / mb_row_start [mb_table_len]: per rank n_mb+1 entries, slot index / shard
 * row at which each micro-batch starts, closed by n_seq / shard rows.  cu_seqlens
 * [cu_seqlens_len]: per rank, per micro-batch, the n+1 cumulative LOCAL row counts (rows on one SP
 * rank), restarting at 0 in every micro-batch.
 */
int32_t earl_plan_export(earl_plan* plan, int32_t* rank, int32_t* slot, int32_t* mb,
                         int64_t* dst_row, int32_t* seq_shard, int64_t* seq_row, int32_t* seq_ids,
                         int32_t* mb_seq_start, int64_t* mb_row_start, int32_t* cu_seqlens);

/*
 * Copies the segment table to HOST buffers of n_segments entries each (NULL to skip).  Segments are
 * ordered by (destination shard, destination row).  Segment e copies n_real[e] rows from row
 * src_row[e] of shard buffer src_shard[e] to row dst_row[e] of destination shard dst_shard[e] and
 * fills the following n_rows[e]-n_real[e] rows with padding; pos0[e] is the logical position of its
 * first row.  shard_seg_start has D*C+1 entries.
 */
int32_t earl_plan_export_segments(earl_plan* plan, int32_t* src_shard, int64_t* src_row,
                                  int32_t* dst_shard, int64_t* dst_row, int32_t* n_real,
                                  int32_t* n_rows, int32_t* pos0, int32_t* shard_seg_start);

/*
 * Bytes of device scratch one earl_dispatch call with these fields needs: the call's parameter
 * block plus one 16-byte record per 4 KiB of destination (about 0.4 % of the bytes written).  The
 * size depends on the plan's shard sizes, so this call waits for the plan like
 * earl_plan_get_summary.  Only scalar_bytes, width and nonzero_counts (null or not) of every field
 * are read.
 */
int32_t earl_dispatch_workspace_bytes(earl_plan* plan, const earl_field* fields, int32_t n_fields,
                                      int32_t with_position_ids, int32_t with_cu_seqlens,
                                      size_t* out_bytes);

/*
 * Materialises every destination shard of every field (asynchronously on the stream; the first call
 * on a plan waits for the plan as earl_plan_get_summary does).  This is the data movement of
 * Section 2, "Data Dispatcher": every row goes straight from the buffer it was produced in to its
 * place in the training layout, with no gathered intermediate copy (Section 1: the volume of these
 * batches is the bottleneck).
 *   fields[n_fields]             0 <= n_fields <= EARL_MAX_FIELDS.
 *   position_ids_shard_ptrs      host array[D*C] of device int32 buffers (16-byte aligned, at least
 *                                shard_rows[q] entries), or NULL: logical position of every row,
 *                                padding rows included.
 *   cu_seqlens_dev               device int32[cu_seqlens_len] (16-byte aligned) or NULL.
 *   dispatch_ws_dev / _bytes     device scratch, 256-byte aligned, at least
 *                                earl_dispatch_workspace_bytes() bytes (EARL_CAPACITY otherwise);
 *                                in use until the call's work has finished on the stream.
 * Every check (plan status, alignment, capacities) happens before anything is enqueued: a failed
 * call writes nothing.  Calls that share a scratch buffer must be ordered on one stream.
 * The call's parameter block (about 100 bytes per field and destination shard) reaches the device
 * through a pinned host block of 8 MiB that the library allocates at the first dispatch call of the
 * process and keeps until the process ends; it is used in slots of 256 KiB, so a block above
 * 8 MiB (some 80000 (field, shard) pairs) makes the call wait on the host for the work that
 * precedes it on the stream.  The same holds for earl_dispatch_async and earl_dispatch_inverse.
 */
int32_t earl_dispatch(earl_plan* plan, const earl_field* fields, int32_t n_fields,
                      int32_t* const* position_ids_shard_ptrs, int32_t* cu_seqlens_dev,
                      void* dispatch_ws_dev, size_t dispatch_ws_bytes, void* hip_stream);

/*
 * earl_dispatch without the wait for the plan.  earl_dispatch needs the shard sizes on the host
 * (to size its launches exactly and to check every capacity before anything is enqueued), so its
 * first call on a plan synchronises with the plan kernel.  This variant sizes its launches by the
 * CAPACITIES the caller states and leaves the rest to the device: it can be enqueued right
 * behind earl_plan_build with no host synchronisation in between (a serving or training loop that
 * pre-allocates its buffers never stalls; the summary can be fetched afterwards).
 *   fields[n_fields]               as for earl_dispatch; dst_capacity_rows AND src_capacity_rows
 *                                  are required; nonzero_counts must be NULL.
 *   position_ids_shard_ptrs        host array[D*C] of device int32 buffers or NULL, with
 *   position_ids_capacity_rows     host array[D*C]: rows each of them holds (NULL iff the former is).
 *   cu_seqlens_dev / _capacity     device int32 buffer and the entries it holds, or NULL and 0.
 *   dispatch_ws_dev / _bytes       scratch of at least earl_dispatch_async_workspace_bytes() bytes.
 *   hip_stream                     the stream earl_plan_build was given, or one ordered behind it.
 * Buffers with capacity 0 may be NULL; the others must be aligned as for earl_dispatch.
 * What cannot be checked on the host is checked on the device before any byte is written: if the
 * plan failed (bad length, budget exceeded) or any destination, source, position-id or cu_seqlens
 * buffer is smaller than the plan needs, the call writes NOTHING and records the status, which
 * earl_dispatch_async_status returns (it waits for the stream): EARL_OK, the plan's status, or
 * EARL_CAPACITY.  Rows of a destination buffer beyond the shard's size are left untouched.
 */
int32_t earl_dispatch_async_workspace_bytes(earl_plan* plan, const earl_field* fields,
                                            int32_t n_fields,
                                            const int64_t* position_ids_capacity_rows,
                                            int64_t cu_seqlens_capacity, size_t* out_bytes);
int32_t earl_dispatch_async(earl_plan* plan, const earl_field* fields, int32_t n_fields,
                            int32_t* const* position_ids_shard_ptrs,
                            const int64_t* position_ids_capacity_rows, int32_t* cu_seqlens_dev,
                            int64_t cu_seqlens_capacity, void* dispatch_ws_dev,
                            size_t dispatch_ws_bytes, void* hip_stream);
int32_t earl_dispatch_async_status(earl_plan* plan, int32_t* status);

/*
 * earl_dispatch for callers that cannot allocate (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): same arguments without the scratch buffer, same result.
 * The scratch (parameter block and tile codes) lives in an array of EARL_NOALLOC_SCRATCH_BYTES
 * that is part of the library's device image: every GPU the library runs on holds one copy from
 * the first call there until the process ends.  The call allocates nothing, on the device or on
 * the host, waits for nothing and copies nothing through staging memory (the parameter block
 * travels as kernel arguments), so:
 *   - the plan's summary must already be on the host (earl_plan_get_summary has returned EARL_OK
 *     for this plan; EARL_INVALID_ARG otherwise);
 *   - a call whose parameter block exceeds 256 KiB or whose scratch need (what
 *     earl_dispatch_workspace_bytes reports) exceeds the array returns EARL_CAPACITY and enqueues
 *     nothing;
 *   - all calls on one GPU share the array, which keeps the previous call's contents (every part a
 *     call reads it has written first): calls whose work can overlap on the GPU, from different
 *     streams or processes' threads, race; order them on one stream or by events.
 */
#define EARL_NOALLOC_SCRATCH_BYTES (32u << 20)
int32_t earl_dispatch_noalloc(earl_plan* plan, const earl_field* fields, int32_t n_fields,
                              int32_t* const* position_ids_shard_ptrs, int32_t* cu_seqlens_dev,
                              void* hip_stream);

/*
 * Measurement hook (no passage of the paper: it serves the benchmark): the following
 * earl_dispatch / earl_dispatch_async / earl_dispatch_inverse calls on this plan record
 * `event_before` on the stream right before the first kernel that moves or decodes data and
 * `event_after` right after the last one (both hipEvent_t created by the caller with timing
 * enabled; NULL, NULL switches the hook off).  The interval covers every kernel of the re-layout
 * (decode pass and copy), without the upload of the call's parameter block.
 */
int32_t earl_plan_set_dispatch_events(earl_plan* plan, void* event_before, void* event_after);

/*
 * The reverse direction (training layout back to the rollout layout; Section 2 describes dispatches
 * between several stages of a step, so data also has to come back): every real row of every
 * destination shard is copied back to the source row it was read from.  Field descriptors as in earl_dispatch with the roles of the two pointer
 * arrays unchanged (dst_shard_ptrs is read, src_shard_ptrs is written; both only need alignment to
 * scalar_bytes).  Rows of the source buffers that the plan does not read are left untouched.
 * The scratch buffer holds the call's parameter block and one 16-byte record per tile of the
 * stream of real rows; earl_dispatch_workspace_bytes() with the same fields is always enough.
 * Any stream may be used: the first inverse call on a plan computes a per-segment prefix of real
 * rows on its stream, and later calls on other streams are ordered behind it by an event.
 */
int32_t earl_dispatch_inverse(earl_plan* plan, const earl_field* fields, int32_t n_fields,
                              void* dispatch_ws_dev, size_t dispatch_ws_bytes, void* hip_stream);

/* Frees the host object (device memory is the caller's). */
int32_t earl_plan_destroy(earl_plan* plan);

const char* earl_status_string(int32_t status);
/* Text of the last failure on this thread (static storage, overwritten by the next failure). */
const char* earl_last_error_message(void);

#ifdef __cplusplus
}
#endif
#endif /* EARL_DISPATCH_H_ */
