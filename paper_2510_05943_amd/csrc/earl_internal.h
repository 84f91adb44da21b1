// Internal definitions shared by the host API and the gfx950 kernels of the re-layout library.
// Nothing here is part of the C ABI (see include/earl_dispatch.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace earl {

constexpr int kWave = 64;            // CDNA wavefront width
constexpr int kPlanThreads = 1024;   // the plan runs in one workgroup of 16 wavefronts
constexpr int kPlanWaves = kPlanThreads / kWave;
constexpr int kMaxDp = 1024;         // one DP rank per plan thread

// Labels (source groups, DP ranks) whose per-wave scan tables fit the workgroup's LDS; larger
// label counts use the same code on tables in the workspace.
constexpr int kMaxQuadraticLp = 1 << 21;   // largest padded length under balance_policy 2
constexpr int kLdsLabels = 256;
// Sort keys kept in LDS up to this many (power of two); more go to the workspace.
constexpr int kLdsSortKeys = 8192;

constexpr int kVecBytes = 16;        // one global_load/store_dwordx4 per lane
constexpr int kTileShift = 12;       // log2 of kTileBytes
constexpr int kTileBytes = 4096;     // destination bytes described by one tile code
constexpr int kFineTileShift = 10;   // fields with rows under 16 bytes: 1 KiB per tile code
constexpr int kCopyThreads = 64;     // re-layout workgroup: one wavefront, 1 KiB of a tile
constexpr int kSubTiles = kTileBytes / (kCopyThreads * kVecBytes);   // workgroups per 4 KiB tile
constexpr int kTilesPerLane = 4;     // code kernels: consecutive tiles per lane (measured best among
                                     // 1, 2, 4, 8, 16 on the 12 M tiles of the largest workload)
constexpr int kCodeThreads = 256;    // tile-code kernel workgroup

constexpr int kStatusCapacity = 3;   // EARL_CAPACITY, for device code

// First bytes of the workspace; copied to the host together with the arrays that follow it.
struct PlanHeader {
  int32_t status;
  int32_t bad_index;       // a sequence index that caused status != 0 (diagnostic)
  int32_t n_segments;
  int32_t n_mb_max;
  int32_t cu_seqlens_len;
  int32_t mb_table_len;
  int32_t pad_[2];
  int64_t total_real_rows;
  int64_t total_dst_rows;
  int64_t rank_load_min;
  int64_t rank_load_max;
  int64_t async_status;    // written by the last earl_dispatch_async on this plan (0 = carried out)
  int64_t reserved_[9];
};
static_assert(sizeof(PlanHeader) == 144, "PlanHeader layout");

// One segment: n_rows destination rows starting at dst_row of its shard; the first n_real are
// copied from row src_row of shard buffer src_shard, the rest is padding; pos0 = logical
// position of the first row.  32 bytes, so a lane fetches a whole record with two loads.
struct SegRec {
  int64_t dst_row;
  int64_t src_row;
  int32_t n_real;
  int32_t n_rows;
  int32_t src_shard;
  int32_t pos0;
};
static_assert(sizeof(SegRec) == 32, "SegRec layout");

// Everything the plan kernel needs: problem sizes and pointers into the caller's workspace.
struct PlanDev {
  // inputs
  const int32_t* lengths;
  const int32_t* seq_group_in;   // may be null
  const int64_t* seq_row_in;     // may be null
  int32_t N, G, R, S, D, C, K, halves, P;
  int32_t n_pow2;                // N rounded up to a power of two (sort size)
  int32_t policy;                // 0 longest-first list scheduling, 1 sorted snake deal,
                                 // 2 list scheduling on squared padded lengths
  int32_t equal_mb;              // 1: every rank reports the largest micro-batch count
  int64_t B;
  // Mailbox in pinned host memory (null: none): the kernel copies the finished summary block
  // there and then stores host_token into the mailbox's last eight bytes, so that the host can
  // see the plan's totals without a copy command and a stream synchronisation.
  unsigned char* host_summary;
  uint64_t host_token;
  uint32_t summary_bytes;        // bytes of the summary block (a multiple of 256)
  uint32_t host_flag_offset;     // byte offset of the token inside the mailbox
  // summary block (contiguous, copied to the host in one piece)
  PlanHeader* hdr;
  int64_t* shard_rows;           // [D*C]
  int64_t* src_rows_needed;      // [S]
  int64_t* src_seqs_needed;      // [S]
  int32_t* n_seq;                // [D]
  int32_t* n_mb;                 // [D]
  int64_t* rank_load;            // [D]
  int64_t* a2a;                  // [S*D*C]
  // per sequence
  int32_t* seq_group;            // [N]
  int32_t* seq_shard;            // [N]
  int32_t* seq_k;                // [N] index of the sequence among its group's members
  int64_t* seq_row;              // [N]
  int32_t* m;                    // [N] chunk length
  int32_t* rank;                 // [N]
  int32_t* slot;                 // [N]
  int32_t* mb;                   // [N]
  int64_t* dst_row;              // [N]
  int64_t* seq_pre;              // [N+1] real rows of all sequences before i (written by the kernel
                                 // that keeps the batch in LDS only; entry N is the total)
  // per rank / packed order
  int32_t* seq_ids;              // [N]
  int32_t* next_start;           // [N] scratch: first slot of the following micro-batch
  int32_t* mb_tmp;               // [N+D] scratch
  int32_t* mb_seq_start;         // [N+D]
  int64_t* mb_row_start;         // [N+D]
  int32_t* cu_seqlens;           // [2N]
  int32_t* rank_seq_base;        // [D+1]
  int32_t* rank_mbt_base;        // [D+1]
  int32_t* rank_cu_base;         // [D+1]
  // segment table, ordered by (destination shard, destination row)
  SegRec* segs;                  // [N*K]
  int32_t* seg_dst_shard;        // [N*K]
  int32_t* seg_src_seq;          // [N*K] seq_k of the segment's sequence
  int32_t* seg_mb;               // [N*K] micro-batch (within its rank) of the segment's sequence
  int32_t* shard_seg_start;      // [D*C+1]
  // scratch
  uint64_t* sort_keys;           // [n_pow2]; reused as int64 row offsets in packed order
  int64_t* lab_sum;              // [2*kPlanWaves*Lmax + Lmax], Lmax = max(G, D)
  int32_t* lab_cnt;              // same shape
};

// What a tile of the re-layout kernel copies.
enum FieldKind : int32_t { kFieldCopy = 0, kFieldPositionIds = 1, kFieldLinear = 2 };

// One (field, destination shard) pair of a dispatch call, or one field of an inverse call:
// everything a workgroup needs besides the segment table, in one 64-byte record.
constexpr uint32_t kNoCounters = 0xffffffffu;

struct TileRec {
  int64_t tile_first;       // first tile of this record in the launch
  int64_t end_bytes;        // bytes of this destination shard (kFieldLinear: bytes to copy)
  void* dst;                // destination shard (forward only)
  uint64_t pad_scalar;      // padding scalar replicated to 8 bytes
  int32_t e_begin, e_end;   // segments of this destination shard
  int32_t row_bytes;
  int32_t scalar_bytes;
  int32_t kind;
  uint32_t src_ptr_index;   // first of the field's S source pointers in the pointer table
  uint32_t dst_ptr_index;   // inverse: first of the field's D*C destination pointers; forward:
                            // pointer-table slot of this shard's counter row, or kNoCounters
  int16_t per_sequence;     // source holds one row per sequence, broadcast to its tokens
  int16_t tile_shift;       // log2 of the bytes one tile code of this record describes
};
static_assert(sizeof(TileRec) == 64, "TileRec layout");

// Parameter block of one call, in device memory: header, tile_start, recs[n_recs], pointer
// table.  The first n_direct records are decoded inside the copy kernel (their tile_first counts
// jobs of 1 << tile_shift bytes), the others go through tile codes; tile_start holds tile_first of the direct
// records and their total (n_direct + 1 entries), then the same for the coded records.
struct DispatchDev {
  int32_t n_recs;
  int32_t n_fields;         // earl_dispatch_async only: rows of src_caps
  uint32_t tile_start_ofs;  // byte offsets from the start of the block
  uint32_t recs_ofs;
  uint32_t ptrs_ofs;
  uint32_t total_bytes;
  // earl_dispatch_async only: rec_caps[n_recs] rows (kFieldLinear: entries) each record's
  // buffer holds; src_caps[n_fields][S] rows each source buffer holds (-1 = not checked);
  // src_per_sequence[n_fields]
  uint32_t rec_caps_ofs;
  uint32_t src_caps_ofs;
  uint32_t src_per_sequence_ofs;
  int32_t n_direct;
};

struct CopyArgs {
  const DispatchDev* params;
  const SegRec* segs;
  const int32_t* seg_src_seq;
  int64_t n_direct_jobs; // jobs of the records that are decoded inside the copy kernel
  // the parts of the parameter block those records use, so that the kernel need not read the
  // block's header first
  const int64_t* direct_tile_start;
  const TileRec* direct_recs;
  const void* const* ptrs;
  int32_t n_direct;
  int32_t n_src_shards;
  int64_t n_tiles;       // tile codes in the launch
  const int32_t* seg_mb;  // micro-batch of every segment (fields that ask for non-zero counts)
};

// Returns true if the kernel that keeps the batch in LDS took the plan (it also writes seq_pre).
bool launch_plan(const PlanDev& p, hipStream_t stream);
// tile_codes: 16 bytes of scratch per tile
constexpr size_t kTileCodeBytes = 16;
void launch_tile_codes(const CopyArgs& a, void* tile_codes, hipStream_t stream);
void launch_copy(const CopyArgs& a, const void* tile_codes, hipStream_t stream);
void launch_direct(const CopyArgs& a, hipStream_t stream);
// seg_real_prefix[e] = real rows of the segments before e (n_seg+1 entries)
void launch_zero_counters(int64_t* counters, int64_t n, hipStream_t stream);
// writes a host-built parameter block to device memory through kernel arguments, in pieces
constexpr int kParamChunkBytes = 3072;
void launch_param_chunks(void* dev_dst, const unsigned char* host_block, size_t bytes,
                         hipStream_t stream);
// earl_dispatch_async: completes the records of a parameter block from the plan in device memory
void launch_async_resolve(DispatchDev* params, const PlanDev& plan, hipStream_t stream);
void launch_real_prefix(const SegRec* segs, int64_t* prefix, int n_seg, hipStream_t stream);
// seq_pre/prefix_out: if seq_pre is given, also writes the prefix of real rows over the
// source-ordered table (n_seg + 1 entries), which has a closed form there
void launch_source_order(const SegRec* segs, const int32_t* seg_dst_shard,
                         const int32_t* seg_src_seq, SegRec* out, int32_t* out_dst_shard, int n_seg,
                         int N, int G, int R, int K, const int64_t* seq_pre, int64_t* prefix_out,
                         hipStream_t stream);
void launch_copy_inverse(const CopyArgs& a, const int64_t* seg_real_prefix,
                         const int32_t* seg_dst_shard, int n_seg, int n_dst_shards,
                         void* tile_codes, hipEvent_t before, hipEvent_t after,
                         hipStream_t stream);

}  // namespace earl
