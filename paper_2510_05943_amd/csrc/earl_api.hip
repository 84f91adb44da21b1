// Host side of the C ABI declared in include/earl_dispatch.h: argument checks, workspace
// carve-up, kernel launches, and host copies of the plan.  No device memory is allocated here;
// the only allocations are small host objects and a few pinned staging slots used to hand the
// per-call parameter block to the re-layout kernel.
#include "earl_dispatch.h"

#include <atomic>
#include <chrono>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "earl_internal.h"

using namespace earl;

namespace {

thread_local char g_err[512] = "";

int32_t fail(int32_t status, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return status;
}

#define HIP_TRY(expr)                                                                  \
  do {                                                                                 \
    hipError_t e_ = (expr);                                                            \
    if (e_ != hipSuccess)                                                              \
      return fail(EARL_HIP_ERROR, "%s failed: %s", #expr, hipGetErrorString(e_));      \
  } while (0)

static_assert(kStatusCapacity == EARL_CAPACITY, "status codes of device code");

constexpr size_t kAlign = 256;
size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

size_t param_block_bytes(int n_fields, int n_src, int n_dst) {
  const size_t n_recs = (size_t)n_fields * n_dst;
  size_t b = align_up(sizeof(DispatchDev));
  b += align_up(sizeof(int64_t) * (n_recs + 2));
  b += align_up(sizeof(TileRec) * n_recs);
  // per field: S source pointers, D*C destination pointers, D*C counter rows
  b += align_up(sizeof(void*) * (size_t)n_fields * ((size_t)n_src + 2 * (size_t)n_dst));
  // earl_dispatch_async: capacities of every record and of every source buffer, field flags
  b += align_up(sizeof(int64_t) * n_recs);
  b += align_up(sizeof(int64_t) * (size_t)n_fields * (size_t)n_src);
  b += align_up(sizeof(int32_t) * (size_t)n_fields);
  return b;
}

// Byte offsets of every array inside the workspace.
struct Layout {
  size_t hdr, shard_rows, src_rows_needed, src_seqs_needed, n_seq, n_mb, rank_load, a2a, summary_end;
  size_t seq_group, seq_shard, seq_k, seq_row, m, rank, slot, mb, dst_row, seq_pre;
  size_t seq_ids, next_start, mb_tmp, mb_seq_start, mb_row_start, cu_seqlens;
  size_t rank_seq_base, rank_mbt_base, rank_cu_base;
  size_t segs, seg_dst_shard, seg_src_seq, seg_mb;
  size_t shard_seg_start, seg_real_prefix, segs_src, seg_dst_shard_src;
  size_t sort_keys, lab_sum, lab_cnt;
  size_t total;
};

struct Dims {
  int32_t N, G, R, S, D, C, K, halves, P, zigzag, n_pow2, policy, equal_mb;
  int64_t B, n_seg;
};

Layout make_layout(const Dims& d) {
  Layout l{};
  size_t off = 0;
  auto take = [&](size_t bytes) {
    size_t o = off;
    off += align_up(bytes);
    return o;
  };
  const size_t N = d.N, S = d.S, D = d.D, DC = (size_t)d.D * d.C, NK = (size_t)d.n_seg;
  l.hdr = take(sizeof(PlanHeader));
  l.shard_rows = take(8 * DC);
  l.src_rows_needed = take(8 * S);
  l.src_seqs_needed = take(8 * S);
  l.n_seq = take(4 * D);
  l.n_mb = take(4 * D);
  l.rank_load = take(8 * D);
  l.a2a = take(8 * S * DC);
  l.summary_end = off;
  l.seq_group = take(4 * N);
  l.seq_shard = take(4 * N);
  l.seq_k = take(4 * N);
  l.seq_row = take(8 * N);
  l.m = take(4 * N);
  l.rank = take(4 * N);
  l.slot = take(4 * N);
  l.mb = take(4 * N);
  l.dst_row = take(8 * N);
  l.seq_pre = take(8 * (N + 1));
  l.seq_ids = take(4 * N);
  l.next_start = take(4 * N);
  l.mb_tmp = take(4 * (N + D));
  // micro-batch tables: sum over ranks of (n_mb + 1) entries, cu_seqlens: N + sum of n_mb; a
  // rank has at most as many micro-batches as sequences, with equal_mb at most N each
  const size_t mb_entries = d.equal_mb ? D * (N + 1) : N + D;
  l.mb_seq_start = take(4 * mb_entries);
  l.mb_row_start = take(8 * mb_entries);
  l.cu_seqlens = take(4 * (N + mb_entries));
  l.rank_seq_base = take(4 * (D + 1));
  l.rank_mbt_base = take(4 * (D + 1));
  l.rank_cu_base = take(4 * (D + 1));
  l.segs = take(sizeof(SegRec) * NK);
  l.seg_dst_shard = take(4 * NK);
  l.seg_src_seq = take(4 * NK);
  l.seg_mb = take(4 * NK);
  l.shard_seg_start = take(4 * (DC + 1));
  l.seg_real_prefix = take(8 * (NK + 1));
  // the reverse direction's copy of the segment table in source order (see earl_dispatch_inverse)
  l.segs_src = take(sizeof(SegRec) * NK);
  l.seg_dst_shard_src = take(4 * NK);
  l.sort_keys = take(8 * (size_t)d.n_pow2);
  const size_t lmax = (size_t)(d.G > d.D ? d.G : d.D);
  const size_t tab = (2 * (size_t)kPlanWaves + 1) * lmax;
  l.lab_sum = take(8 * tab);
  l.lab_cnt = take(4 * tab);
  l.total = off;
  return l;
}

int32_t check_layouts(int32_t n_seqs, const earl_src_layout* src, const earl_dst_layout* dst,
                      Dims* out) {
  if (!src || !dst) return fail(EARL_INVALID_ARG, "null layout");
  if (n_seqs < 1 || n_seqs > EARL_MAX_SEQS)
    return fail(EARL_INVALID_ARG, "n_seqs %d outside [1, %d]", n_seqs, EARL_MAX_SEQS);
  if (src->n_groups < 1 || src->replication < 1 ||
      (int64_t)src->n_groups * src->replication > EARL_MAX_SRC_SHARDS)
    return fail(EARL_INVALID_ARG, "source layout: need 1 <= groups*replication <= %d",
                EARL_MAX_SRC_SHARDS);
  if (dst->dp < 1 || dst->dp > EARL_MAX_DP) return fail(EARL_INVALID_ARG, "dp out of range");
  if (dst->sp < 1 || dst->sp > EARL_MAX_SP) return fail(EARL_INVALID_ARG, "sp out of range");
  if (dst->zigzag != 0 && dst->zigzag != 1) return fail(EARL_INVALID_ARG, "zigzag must be 0 or 1");
  if (dst->pad_multiple < 1) return fail(EARL_INVALID_ARG, "pad_multiple must be >= 1");
  if (dst->balance_policy < 0 || dst->balance_policy > 2)
    return fail(EARL_INVALID_ARG, "unknown balance_policy");
  if (dst->equal_mb != 0 && dst->equal_mb != 1)
    return fail(EARL_INVALID_ARG, "equal_mb must be 0 or 1");
  if (dst->equal_mb && (int64_t)dst->dp * ((int64_t)n_seqs + 1) > (int64_t)1 << 27)
    return fail(EARL_INVALID_ARG, "equal_mb: dp * (n_seqs + 1) exceeds 2^27");
  if (dst->mb_token_budget < 1) return fail(EARL_INVALID_ARG, "mb_token_budget must be >= 1");
  Dims d{};
  d.N = n_seqs;
  d.G = src->n_groups;
  d.R = src->replication;
  d.S = d.G * d.R;
  d.D = dst->dp;
  d.C = dst->sp;
  d.zigzag = dst->zigzag;
  d.K = (dst->zigzag && dst->sp > 1) ? 2 * dst->sp : dst->sp;
  d.halves = d.K / d.C;
  d.P = dst->pad_multiple;
  d.B = dst->mb_token_budget;
  d.policy = dst->balance_policy;
  d.equal_mb = dst->equal_mb;
  d.n_seg = (int64_t)d.N * d.K;
  if (d.n_seg > (int64_t)1 << 27) return fail(EARL_INVALID_ARG, "n_seqs * chunks exceeds 2^27");
  if ((int64_t)d.S * d.D * d.C > (int64_t)1 << 24)
    return fail(EARL_INVALID_ARG, "source shards * destination shards exceeds 2^24");
  d.n_pow2 = 1;
  while (d.n_pow2 < d.N) d.n_pow2 <<= 1;
  *out = d;
  return EARL_OK;
}

// Pinned staging slots for the per-call parameter block (host -> workspace copy on the stream).
struct StageSlot {
  void* host = nullptr;
  hipEvent_t done = nullptr;
  bool in_flight = false;
};
constexpr int kStageSlots = 32;
constexpr size_t kStageBytes = 256 * 1024;
std::mutex g_stage_mu;
StageSlot g_stage[kStageSlots];
bool g_stage_ready = false;
int g_stage_next = 0;

// Mailboxes in pinned, coherent host memory: the plan kernel copies its summary block into one
// and then stores the plan's token into the mailbox's last eight bytes.  The host polls that
// word instead of enqueueing a device-to-host copy and synchronising the stream, which costs
// some 20 us more than the kernel itself on a small batch.  One allocation of 1 MiB at the first
// plan of the process, kept until the process ends.  A plan whose summary block is larger than
// a mailbox, or that finds none free, falls back to the copy.
constexpr size_t kMailboxBytes = 16 * 1024;
constexpr size_t kMailboxFlagOffset = kMailboxBytes - 8;
constexpr int kMailboxes = 64;
struct Mailboxes {
  std::mutex mu;
  unsigned char* base = nullptr;
  bool tried = false;
  // 0 free, 1 held by a plan, 2 abandoned before its kernel was seen to finish (draining)
  int state[kMailboxes] = {};
  uint64_t token[kMailboxes] = {};
  uint64_t next_token = 1;
};
Mailboxes g_mail;

volatile uint64_t* mailbox_flag(int slot) {
  return reinterpret_cast<volatile uint64_t*>(g_mail.base + (size_t)slot * kMailboxBytes +
                                              kMailboxFlagOffset);
}

// A free mailbox with its flag cleared, or -1.
int acquire_mailbox(size_t summary_bytes, uint64_t* token) {
  if (summary_bytes > kMailboxFlagOffset) return -1;
  std::lock_guard<std::mutex> lock(g_mail.mu);
  if (!g_mail.tried) {
    g_mail.tried = true;
    void* base = nullptr;
    if (hipHostMalloc(&base, kMailboxBytes * kMailboxes, hipHostMallocCoherent) == hipSuccess)
      g_mail.base = static_cast<unsigned char*>(base);
    else
      (void)hipGetLastError();   // no mailboxes: every plan takes the copy path
  }
  if (!g_mail.base) return -1;
  for (int k = 0; k < kMailboxes; ++k) {
    if (g_mail.state[k] == 2 && *mailbox_flag(k) == g_mail.token[k]) g_mail.state[k] = 0;
    if (g_mail.state[k] != 0) continue;
    g_mail.state[k] = 1;
    g_mail.token[k] = g_mail.next_token++;
    *mailbox_flag(k) = 0;
    std::atomic_thread_fence(std::memory_order_seq_cst);
    *token = g_mail.token[k];
    return k;
  }
  return -1;
}

// done: the kernel's token has been seen, nothing will write the mailbox any more.
void release_mailbox(int slot, bool done) {
  std::lock_guard<std::mutex> lock(g_mail.mu);
  g_mail.state[slot] = done ? 0 : 2;
}

}  // namespace

struct earl_plan {
  Dims d;
  Layout l;
  PlanDev dev;
  unsigned char* ws;
  hipStream_t stream;
  bool summary_ready;
  int mailbox;                          // pinned host mailbox the kernel reports to, or -1
  uint64_t mailbox_token;
  int32_t status;
  bool inverse_ready;
  bool source_order;                    // the reverse direction walks the segments by source position
  bool has_seq_pre = false;             // the plan kernel wrote seq_pre (see launch_plan)
  void* inverse_prefix_done;            // hipEvent_t recorded behind the prefix kernel
  hipStream_t inverse_stream;           // stream that kernel ran on
  void* ev_before;
  void* ev_after;
  hipStream_t async_stream;             // stream of the last earl_dispatch_async
  bool async_used;
  std::vector<int32_t> seg_starts;      // first segment of every destination shard (+ total)
  std::vector<unsigned char> summary;   // host copy of the workspace's summary block
  PlanHeader hdr;
};

namespace {

// Waits until the plan kernel's token shows in the mailbox: polls for up to a quarter of a
// millisecond (a plan kernel takes 10 to 150 us), then lets the runtime wait for the stream.
bool wait_for_mailbox(earl_plan* p) {
  volatile uint64_t* flag = mailbox_flag(p->mailbox);
  const auto t0 = std::chrono::steady_clock::now();
  for (unsigned spin = 0; *flag != p->mailbox_token; ++spin) {
    __builtin_ia32_pause();
    if ((spin & 255u) == 255u &&
        std::chrono::steady_clock::now() - t0 > std::chrono::microseconds(250)) {
      if (hipStreamSynchronize(p->stream) != hipSuccess) return false;
      break;
    }
  }
  std::atomic_thread_fence(std::memory_order_acquire);
  return *flag == p->mailbox_token;
}

int32_t ensure_summary(earl_plan* p) {
  if (p->summary_ready) return p->status;
  p->summary.resize(p->l.summary_end);
  bool have = false;
  if (p->mailbox >= 0) {
    have = wait_for_mailbox(p);
    if (have)
      std::memcpy(p->summary.data(), g_mail.base + (size_t)p->mailbox * kMailboxBytes,
                  p->l.summary_end);
    release_mailbox(p->mailbox, have);
    p->mailbox = -1;
  }
  if (!have) {
    HIP_TRY(hipMemcpyAsync(p->summary.data(), p->ws, p->l.summary_end, hipMemcpyDeviceToHost,
                           p->stream));
    HIP_TRY(hipStreamSynchronize(p->stream));
  }
  std::memcpy(&p->hdr, p->summary.data() + p->l.hdr, sizeof(PlanHeader));
  p->status = p->hdr.status;
  p->summary_ready = true;
  if (p->status == EARL_OK) {
    // Segments are ordered by (rank, SP rank, position in rank, half): the first segment of
    // every destination shard follows from the per-rank sequence counts.
    const int32_t* n_seq = reinterpret_cast<const int32_t*>(p->summary.data() + p->l.n_seq);
    const int D = p->d.D, C = p->d.C, halves = p->d.halves;
    p->seg_starts.resize((size_t)D * C + 1);
    int64_t base = 0;
    for (int r = 0; r < D; ++r) {
      for (int c = 0; c < C; ++c)
        p->seg_starts[(size_t)r * C + c] = (int32_t)(halves * (C * base + (int64_t)c * n_seq[r]));
      base += n_seq[r];
    }
    p->seg_starts[(size_t)D * C] = (int32_t)(halves * C * base);
  }
  if (p->status == EARL_INVALID_ARG)
    fail(p->status, "sequence %d: length < 1, group out of range or negative row offset",
         p->hdr.bad_index);
  else if (p->status == EARL_SEQ_EXCEEDS_BUDGET)
    fail(p->status, "sequence %d: padded length exceeds the micro-batch budget", p->hdr.bad_index);
  return p->status;
}

template <class Tv>
const Tv* summary_ptr(const earl_plan* p, size_t off) {
  return reinterpret_cast<const Tv*>(p->summary.data() + off);
}

// Copies a host-built parameter block into the workspace, ordered on the stream, in pieces of
// one staging slot each.  A slot is reused once the copy that last read it has finished, so a
// block larger than all slots together (8 MiB) makes the caller wait for earlier pieces, and
// with them for the work that precedes them on the stream.
int32_t upload_params(const unsigned char* block, size_t bytes, void* dev_dst, hipStream_t stream) {
  std::lock_guard<std::mutex> lock(g_stage_mu);
  if (!g_stage_ready) {
    // first use: one pinned allocation for all slots, kept until the process ends; the slots
    // are published only when every one of them is complete
    StageSlot fresh[kStageSlots];
    void* base = nullptr;
    HIP_TRY(hipHostMalloc(&base, kStageBytes * kStageSlots, hipHostMallocDefault));
    for (int k = 0; k < kStageSlots; ++k) {
      hipError_t e = hipEventCreateWithFlags(&fresh[k].done, hipEventDisableTiming);
      if (e != hipSuccess) {
        for (int j = 0; j < k; ++j) (void)hipEventDestroy(fresh[j].done);
        (void)hipHostFree(base);
        return fail(EARL_HIP_ERROR, "hipEventCreateWithFlags failed: %s", hipGetErrorString(e));
      }
      fresh[k].host = static_cast<unsigned char*>(base) + (size_t)k * kStageBytes;
    }
    for (int k = 0; k < kStageSlots; ++k) g_stage[k] = fresh[k];
    g_stage_ready = true;
  }
  for (size_t off = 0; off < bytes; off += kStageBytes) {
    const size_t n = bytes - off < kStageBytes ? bytes - off : kStageBytes;
    StageSlot& s = g_stage[g_stage_next];
    g_stage_next = (g_stage_next + 1) % kStageSlots;
    if (s.in_flight) HIP_TRY(hipEventSynchronize(s.done));
    std::memcpy(s.host, block + off, n);
    HIP_TRY(hipMemcpyAsync(static_cast<unsigned char*>(dev_dst) + off, s.host, n,
                           hipMemcpyHostToDevice, stream));
    HIP_TRY(hipEventRecord(s.done, stream));
    s.in_flight = true;
  }
  return EARL_OK;
}

// The parameter block of one call, built in host memory: the builder's own vector, or a buffer
// the caller lends (`fixed`, for the entry point that must not allocate).
struct BlockBuilder {
  std::vector<unsigned char> owned;
  unsigned char* data = nullptr;
  size_t size = 0;
  DispatchDev hd{};
  int64_t* tile_start() { return reinterpret_cast<int64_t*>(data + hd.tile_start_ofs); }
  TileRec* recs() { return reinterpret_cast<TileRec*>(data + hd.recs_ofs); }
  const void** ptrs() { return reinterpret_cast<const void**>(data + hd.ptrs_ofs); }
  int64_t* rec_caps() { return reinterpret_cast<int64_t*>(data + hd.rec_caps_ofs); }
  int64_t* src_caps() { return reinterpret_cast<int64_t*>(data + hd.src_caps_ofs); }
  int32_t* src_per_sequence() {
    return reinterpret_cast<int32_t*>(data + hd.src_per_sequence_ofs);
  }
  // false: the block does not fit the lent buffer
  bool init(int n_recs, int n_fields, int n_src, int n_dst, unsigned char* fixed = nullptr,
            size_t fixed_bytes = 0) {
    hd.n_recs = n_recs;
    size_t off = align_up(sizeof(DispatchDev));
    hd.tile_start_ofs = (uint32_t)off;
    off += align_up(sizeof(int64_t) * ((size_t)n_recs + 2));
    hd.recs_ofs = (uint32_t)off;
    off += align_up(sizeof(TileRec) * (size_t)n_recs);
    hd.ptrs_ofs = (uint32_t)off;
    off += align_up(sizeof(void*) * (size_t)n_fields * ((size_t)n_src + 2 * (size_t)n_dst));
    hd.n_fields = n_fields;
    hd.rec_caps_ofs = (uint32_t)off;
    off += align_up(sizeof(int64_t) * (size_t)n_recs);
    hd.src_caps_ofs = (uint32_t)off;
    off += align_up(sizeof(int64_t) * (size_t)n_fields * (size_t)n_src);
    hd.src_per_sequence_ofs = (uint32_t)off;
    off += align_up(sizeof(int32_t) * (size_t)n_fields);
    hd.total_bytes = (uint32_t)off;
    size = off;
    if (fixed) {
      if (off > fixed_bytes) return false;
      data = fixed;
      std::memset(data, 0, off);
    } else {
      owned.assign(off, 0);
      data = owned.data();
    }
    std::memcpy(data, &hd, sizeof(hd));
    return true;
  }
};

uint64_t replicate_scalar(uint64_t v, int sb) {
  if (sb >= 8) return v;
  const uint64_t mask = (1ull << (8 * sb)) - 1ull;
  uint64_t x = v & mask;
  for (int b = sb; b < 8; b *= 2) x |= x << (8 * b);
  return x;
}

int32_t check_field(const earl_plan* p, const earl_field& f, int idx, bool inverse) {
  const int sb = f.scalar_bytes;
  if (sb != 1 && sb != 2 && sb != 4 && sb != 8)
    return fail(EARL_INVALID_ARG, "field %d: scalar_bytes must be 1, 2, 4 or 8", idx);
  if (f.width < 1 || (int64_t)f.width * sb > EARL_MAX_ROW_BYTES)
    return fail(EARL_INVALID_ARG, "field %d: row bytes outside [1, %d]", idx, EARL_MAX_ROW_BYTES);
  if (!f.src_shard_ptrs || !f.dst_shard_ptrs || !f.dst_capacity_rows)
    return fail(EARL_INVALID_ARG, "field %d: null pointer array", idx);
  const int64_t* shard_rows = summary_ptr<int64_t>(p, p->l.shard_rows);
  if (f.per_sequence != 0 && f.per_sequence != 1)
    return fail(EARL_INVALID_ARG, "field %d: per_sequence must be 0 or 1", idx);
  if (f.per_sequence) {
    const int64_t w = (int64_t)sb * f.width;
    if (inverse) return fail(EARL_INVALID_ARG, "field %d: a per-sequence field has no inverse", idx);
    if (w != 1 && w != 2 && w != 4 && w != 8)
      return fail(EARL_INVALID_ARG, "field %d: a per-sequence field needs 1, 2, 4 or 8 row bytes", idx);
  }
  if (f.nonzero_counts) {
    if (inverse) return fail(EARL_INVALID_ARG, "field %d: nonzero_counts has no inverse", idx);
    if (f.per_sequence || (int64_t)sb * f.width >= kVecBytes)
      return fail(EARL_INVALID_ARG,
                  "field %d: nonzero_counts needs a per-token field with rows under 16 bytes", idx);
    if (reinterpret_cast<uintptr_t>(f.nonzero_counts) % 8)
      return fail(EARL_INVALID_ARG, "field %d: nonzero_counts is misaligned", idx);
    const int64_t entries = (int64_t)p->d.D * p->d.C * p->hdr.n_mb_max;
    if (f.nonzero_counts_capacity < entries)
      return fail(EARL_CAPACITY, "field %d: nonzero_counts holds %lld entries, %lld needed", idx,
                  (long long)f.nonzero_counts_capacity, (long long)entries);
  }
  const int64_t* need = summary_ptr<int64_t>(p, f.per_sequence ? p->l.src_seqs_needed
                                                               : p->l.src_rows_needed);
  const int n_dst = p->d.D * p->d.C;
  for (int q = 0; q < n_dst; ++q) {
    if (shard_rows[q] == 0) continue;
    if (!f.dst_shard_ptrs[q]) return fail(EARL_INVALID_ARG, "field %d: destination %d is null", idx, q);
    if (reinterpret_cast<uintptr_t>(f.dst_shard_ptrs[q]) % (inverse ? sb : kVecBytes))
      return fail(EARL_INVALID_ARG, "field %d: destination %d is misaligned", idx, q);
    if (f.dst_capacity_rows[q] < shard_rows[q])
      return fail(EARL_CAPACITY, "field %d: destination %d holds %lld rows, %lld needed", idx, q,
                  (long long)f.dst_capacity_rows[q], (long long)shard_rows[q]);
  }
  for (int s = 0; s < p->d.S; ++s) {
    if (need[s] == 0) continue;
    if (!f.src_shard_ptrs[s]) return fail(EARL_INVALID_ARG, "field %d: source %d is null", idx, s);
    // a per-sequence row is fetched as one scalar of row_bytes
    if (reinterpret_cast<uintptr_t>(f.src_shard_ptrs[s]) % (f.per_sequence ? sb * f.width : sb))
      return fail(EARL_INVALID_ARG, "field %d: source %d is misaligned", idx, s);
    if (f.src_capacity_rows && f.src_capacity_rows[s] < need[s])
      return fail(EARL_CAPACITY, "field %d: source %d holds %lld rows, %lld needed", idx, s,
                  (long long)f.src_capacity_rows[s], (long long)need[s]);
  }
  return EARL_OK;
}

CopyArgs copy_args(const earl_plan* p, const void* params_dev, int64_t n_tiles) {
  CopyArgs a{};
  a.params = static_cast<const DispatchDev*>(params_dev);
  a.n_src_shards = p->d.S;
  a.segs = p->dev.segs;
  a.seg_src_seq = p->dev.seg_src_seq;
  a.seg_mb = p->dev.seg_mb;
  a.n_tiles = n_tiles;
  return a;
}

}  // namespace

extern "C" {

int32_t earl_plan_workspace_bytes(int32_t n_seqs, const earl_src_layout* src,
                                  const earl_dst_layout* dst, size_t* out_bytes) {
  if (!out_bytes) return fail(EARL_INVALID_ARG, "out_bytes is null");
  Dims d;
  int32_t st = check_layouts(n_seqs, src, dst, &d);
  if (st != EARL_OK) return st;
  *out_bytes = make_layout(d).total;
  return EARL_OK;
}

int32_t earl_plan_build(const int32_t* lengths_dev, int32_t n_seqs, const earl_src_layout* src,
                        const earl_dst_layout* dst, void* workspace_dev, size_t workspace_bytes,
                        void* hip_stream, earl_plan** out_plan) {
  if (!out_plan) return fail(EARL_INVALID_ARG, "out_plan is null");
  *out_plan = nullptr;
  if (!lengths_dev || !workspace_dev) return fail(EARL_INVALID_ARG, "null device pointer");
  Dims d;
  int32_t st = check_layouts(n_seqs, src, dst, &d);
  if (st != EARL_OK) return st;
  if (reinterpret_cast<uintptr_t>(workspace_dev) % kAlign)
    return fail(EARL_INVALID_ARG, "workspace must be %zu-byte aligned", kAlign);
  const Layout l = make_layout(d);
  if (workspace_bytes < l.total)
    return fail(EARL_CAPACITY, "workspace has %zu bytes, %zu needed", workspace_bytes, l.total);

  earl_plan* p = new (std::nothrow) earl_plan();
  if (!p) return fail(EARL_HIP_ERROR, "out of host memory");
  p->d = d;
  p->l = l;
  p->ws = static_cast<unsigned char*>(workspace_dev);
  p->stream = static_cast<hipStream_t>(hip_stream);
  p->summary_ready = false;
  p->mailbox = acquire_mailbox(l.summary_end, &p->mailbox_token);
  p->status = EARL_OK;
  p->inverse_ready = false;
  // packed source layout with contiguous groups: sequence index order is source order
  p->source_order = src->seq_group == nullptr && src->seq_row == nullptr;
  p->inverse_prefix_done = nullptr;
  p->inverse_stream = nullptr;
  p->async_stream = nullptr;
  p->async_used = false;
  // host arrays the dispatch calls fill are sized here, so that those calls allocate nothing
  p->summary.resize(l.summary_end);
  p->seg_starts.resize((size_t)d.D * d.C + 1);
  p->ev_before = nullptr;
  p->ev_after = nullptr;

  PlanDev& v = p->dev;
  unsigned char* w = p->ws;
  v.lengths = lengths_dev;
  v.seq_group_in = src->seq_group;
  v.seq_row_in = src->seq_row;
  v.N = d.N; v.G = d.G; v.R = d.R; v.S = d.S; v.D = d.D; v.C = d.C; v.K = d.K;
  v.halves = d.halves; v.P = d.P; v.n_pow2 = d.n_pow2; v.B = d.B; v.policy = d.policy; v.equal_mb = d.equal_mb;
  v.host_summary = p->mailbox >= 0 ? g_mail.base + (size_t)p->mailbox * kMailboxBytes : nullptr;
  v.host_token = p->mailbox_token;
  v.summary_bytes = (uint32_t)l.summary_end;
  v.host_flag_offset = (uint32_t)kMailboxFlagOffset;
  v.hdr = reinterpret_cast<PlanHeader*>(w + l.hdr);
  v.shard_rows = reinterpret_cast<int64_t*>(w + l.shard_rows);
  v.src_rows_needed = reinterpret_cast<int64_t*>(w + l.src_rows_needed);
  v.src_seqs_needed = reinterpret_cast<int64_t*>(w + l.src_seqs_needed);
  v.n_seq = reinterpret_cast<int32_t*>(w + l.n_seq);
  v.n_mb = reinterpret_cast<int32_t*>(w + l.n_mb);
  v.rank_load = reinterpret_cast<int64_t*>(w + l.rank_load);
  v.a2a = reinterpret_cast<int64_t*>(w + l.a2a);
  v.seq_group = reinterpret_cast<int32_t*>(w + l.seq_group);
  v.seq_shard = reinterpret_cast<int32_t*>(w + l.seq_shard);
  v.seq_k = reinterpret_cast<int32_t*>(w + l.seq_k);
  v.seq_row = reinterpret_cast<int64_t*>(w + l.seq_row);
  v.m = reinterpret_cast<int32_t*>(w + l.m);
  v.rank = reinterpret_cast<int32_t*>(w + l.rank);
  v.slot = reinterpret_cast<int32_t*>(w + l.slot);
  v.mb = reinterpret_cast<int32_t*>(w + l.mb);
  v.dst_row = reinterpret_cast<int64_t*>(w + l.dst_row);
  v.seq_pre = reinterpret_cast<int64_t*>(w + l.seq_pre);
  v.seq_ids = reinterpret_cast<int32_t*>(w + l.seq_ids);
  v.next_start = reinterpret_cast<int32_t*>(w + l.next_start);
  v.mb_tmp = reinterpret_cast<int32_t*>(w + l.mb_tmp);
  v.mb_seq_start = reinterpret_cast<int32_t*>(w + l.mb_seq_start);
  v.mb_row_start = reinterpret_cast<int64_t*>(w + l.mb_row_start);
  v.cu_seqlens = reinterpret_cast<int32_t*>(w + l.cu_seqlens);
  v.rank_seq_base = reinterpret_cast<int32_t*>(w + l.rank_seq_base);
  v.rank_mbt_base = reinterpret_cast<int32_t*>(w + l.rank_mbt_base);
  v.rank_cu_base = reinterpret_cast<int32_t*>(w + l.rank_cu_base);
  v.segs = reinterpret_cast<SegRec*>(w + l.segs);
  v.seg_dst_shard = reinterpret_cast<int32_t*>(w + l.seg_dst_shard);
  v.seg_src_seq = reinterpret_cast<int32_t*>(w + l.seg_src_seq);
  v.seg_mb = reinterpret_cast<int32_t*>(w + l.seg_mb);
  v.shard_seg_start = reinterpret_cast<int32_t*>(w + l.shard_seg_start);
  v.sort_keys = reinterpret_cast<uint64_t*>(w + l.sort_keys);
  v.lab_sum = reinterpret_cast<int64_t*>(w + l.lab_sum);
  v.lab_cnt = reinterpret_cast<int32_t*>(w + l.lab_cnt);

  p->has_seq_pre = launch_plan(v, p->stream);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) {
    if (p->mailbox >= 0) release_mailbox(p->mailbox, true);   // nothing was launched
    delete p;
    return fail(EARL_HIP_ERROR, "plan kernel launch failed: %s", hipGetErrorString(e));
  }
  *out_plan = p;
  return EARL_OK;
}

int32_t earl_plan_get_summary(earl_plan* p, earl_plan_summary* out) {
  if (!p || !out) return fail(EARL_INVALID_ARG, "null argument");
  std::memset(out, 0, sizeof(*out));
  const int32_t st = ensure_summary(p);
  if (st != EARL_OK) return st;
  out->n_seqs = p->d.N;
  out->n_src_shards = p->d.S;
  out->n_dst_shards = p->d.D * p->d.C;
  out->chunks_per_seq = p->d.K;
  out->n_segments = p->hdr.n_segments;
  out->n_mb_max = p->hdr.n_mb_max;
  out->cu_seqlens_len = p->hdr.cu_seqlens_len;
  out->mb_table_len = p->hdr.mb_table_len;
  out->total_real_rows = p->hdr.total_real_rows;
  out->total_dst_rows = p->hdr.total_dst_rows;
  out->rank_load_min = p->hdr.rank_load_min;
  out->rank_load_max = p->hdr.rank_load_max;
  out->shard_rows = summary_ptr<int64_t>(p, p->l.shard_rows);
  out->src_rows_needed = summary_ptr<int64_t>(p, p->l.src_rows_needed);
  out->src_seqs_needed = summary_ptr<int64_t>(p, p->l.src_seqs_needed);
  out->n_seq = summary_ptr<int32_t>(p, p->l.n_seq);
  out->n_mb = summary_ptr<int32_t>(p, p->l.n_mb);
  out->rank_load = summary_ptr<int64_t>(p, p->l.rank_load);
  out->a2a_counts = summary_ptr<int64_t>(p, p->l.a2a);
  return EARL_OK;
}

int32_t earl_plan_export(earl_plan* p, int32_t* rank, int32_t* slot, int32_t* mb, int64_t* dst_row,
                         int32_t* seq_shard, int64_t* seq_row, int32_t* seq_ids,
                         int32_t* mb_seq_start, int64_t* mb_row_start, int32_t* cu_seqlens) {
  if (!p) return fail(EARL_INVALID_ARG, "null plan");
  const int32_t st = ensure_summary(p);
  if (st != EARL_OK) return st;
  const size_t N = p->d.N;
  auto get = [&](void* dst, const void* src, size_t bytes) -> hipError_t {
    if (!dst || bytes == 0) return hipSuccess;
    return hipMemcpy(dst, src, bytes, hipMemcpyDeviceToHost);
  };
  HIP_TRY(get(rank, p->dev.rank, 4 * N));
  HIP_TRY(get(slot, p->dev.slot, 4 * N));
  HIP_TRY(get(mb, p->dev.mb, 4 * N));
  HIP_TRY(get(dst_row, p->dev.dst_row, 8 * N));
  HIP_TRY(get(seq_shard, p->dev.seq_shard, 4 * N));
  HIP_TRY(get(seq_row, p->dev.seq_row, 8 * N));
  HIP_TRY(get(seq_ids, p->dev.seq_ids, 4 * N));
  HIP_TRY(get(mb_seq_start, p->dev.mb_seq_start, 4 * (size_t)p->hdr.mb_table_len));
  HIP_TRY(get(mb_row_start, p->dev.mb_row_start, 8 * (size_t)p->hdr.mb_table_len));
  HIP_TRY(get(cu_seqlens, p->dev.cu_seqlens, 4 * (size_t)p->hdr.cu_seqlens_len));
  return EARL_OK;
}

int32_t earl_plan_export_segments(earl_plan* p, int32_t* src_shard, int64_t* src_row,
                                  int32_t* dst_shard, int64_t* dst_row, int32_t* n_real,
                                  int32_t* n_rows, int32_t* pos0, int32_t* shard_seg_start) {
  if (!p) return fail(EARL_INVALID_ARG, "null plan");
  const int32_t st = ensure_summary(p);
  if (st != EARL_OK) return st;
  const size_t E = (size_t)p->hdr.n_segments;
  const size_t n_dst = (size_t)p->d.D * p->d.C;
  std::vector<SegRec> segs(E);
  std::vector<int32_t> starts(n_dst + 1);
  if (E) HIP_TRY(hipMemcpy(segs.data(), p->dev.segs, sizeof(SegRec) * E, hipMemcpyDeviceToHost));
  HIP_TRY(hipMemcpy(starts.data(), p->dev.shard_seg_start, 4 * (n_dst + 1), hipMemcpyDeviceToHost));
  if (dst_shard && E)
    HIP_TRY(hipMemcpy(dst_shard, p->dev.seg_dst_shard, 4 * E, hipMemcpyDeviceToHost));
  for (size_t e = 0; e < E; ++e) {
    if (src_shard) src_shard[e] = segs[e].src_shard;
    if (src_row) src_row[e] = segs[e].src_row;
    if (dst_row) dst_row[e] = segs[e].dst_row;
    if (n_real) n_real[e] = segs[e].n_real;
    if (n_rows) n_rows[e] = segs[e].n_rows;
    if (pos0) pos0[e] = segs[e].pos0;
  }
  if (shard_seg_start) std::memcpy(shard_seg_start, starts.data(), 4 * (n_dst + 1));
  return EARL_OK;
}

}  // extern "C"

namespace {

// Bytes per tile code: fields with rows under 16 bytes are cut into 1 KiB tiles (with several
// hundred rows per tile most tiles then lie inside one segment and are plain copies), all others
// into 4 KiB tiles (16 KiB tiles for wide rows measured slower: more bytes in edge tiles).
inline int tile_shift_of(int64_t row_bytes, int kind) {
  return kind != kFieldLinear && row_bytes < kVecBytes ? kFineTileShift : kTileShift;
}
inline int64_t tile_bytes_of(int64_t row_bytes, int kind) {
  return (int64_t)1 << tile_shift_of(row_bytes, kind);
}

// Tile codes of one dispatch call: sum over (field, shard) of ceil(bytes / tile bytes).
int64_t count_tiles(const earl_plan* p, const earl_field* fields, int32_t n_fields, bool with_pos,
                    bool with_cu) {
  const int n_dst = p->d.D * p->d.C;
  const int64_t* shard_rows = summary_ptr<int64_t>(p, p->l.shard_rows);
  int64_t tiles = 0;
  for (int f = 0; f < n_fields + (with_pos ? 1 : 0); ++f) {
    const int64_t w = f < n_fields ? (int64_t)fields[f].scalar_bytes * fields[f].width : 4;
    const int64_t tb = tile_bytes_of(w, kFieldCopy);
    for (int q = 0; q < n_dst; ++q) tiles += (shard_rows[q] * w + tb - 1) / tb;
  }
  if (with_cu) tiles += (4ll * p->hdr.cu_seqlens_len + kTileBytes - 1) / kTileBytes;
  return tiles;
}

int32_t check_field_shapes(const earl_field* fields, int32_t n_fields) {
  if (n_fields < 0 || n_fields > EARL_MAX_FIELDS || (n_fields > 0 && !fields))
    return fail(EARL_INVALID_ARG, "n_fields outside [0, %d] or null fields", EARL_MAX_FIELDS);
  for (int f = 0; f < n_fields; ++f) {
    const int sb = fields[f].scalar_bytes;
    if (sb != 1 && sb != 2 && sb != 4 && sb != 8)
      return fail(EARL_INVALID_ARG, "field %d: scalar_bytes must be 1, 2, 4 or 8", f);
    if (fields[f].width < 1 || (int64_t)fields[f].width * sb > EARL_MAX_ROW_BYTES)
      return fail(EARL_INVALID_ARG, "field %d: row bytes outside [1, %d]", f, EARL_MAX_ROW_BYTES);
  }
  return EARL_OK;
}


// The scratch of earl_dispatch_noalloc: one array per GPU the library runs on, held until the
// process ends.  In host code the name below is only a handle for hipGetSymbolAddress; the
// address the kernels get is looked up once per device and kept in g_scratch_dev.
constexpr size_t kStaticScratchBytes = EARL_NOALLOC_SCRATCH_BYTES;
constexpr int kMaxDevices = 64;
unsigned char* g_scratch_dev[kMaxDevices] = {};
std::mutex g_scratch_mu;
std::mutex g_noalloc_mu;
// host copy of the parameter block of the running earl_dispatch_noalloc call
alignas(256) unsigned char g_noalloc_block[256 * 1024];

}  // namespace

static __device__ __align__(256) unsigned char scratch[EARL_NOALLOC_SCRATCH_BYTES];

namespace {

int32_t static_scratch(unsigned char** out) {
  int dev = -1;
  HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return fail(EARL_INVALID_ARG, "device %d out of range", dev);
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_dev[dev]) {
    void* ptr = nullptr;
    HIP_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    if (!ptr) return fail(EARL_HIP_ERROR, "hipGetSymbolAddress returned a null address");
    g_scratch_dev[dev] = static_cast<unsigned char*>(ptr);
  }
  *out = g_scratch_dev[dev];
  return EARL_OK;
}

// Launches whose fields with rows of 16 bytes and more sum to less than this go through the
// direct kernel as a whole: below it the tile-code pass costs more than it saves.
constexpr int64_t kDirectMaxCoarseBytes = (int64_t)64 << 20;
constexpr int64_t kMaxLaunchTiles = 0x7fffffffll;
constexpr int kJobShiftHost = 12;   // log2 of the bytes of a direct job: 4 KiB ...
constexpr int kJobShiftMin = 10;    // ... down to 1 KiB in small launches (both directions)
constexpr int64_t kSmallLaunchBytes = (int64_t)8 << 20;   // direct records of a "small launch"
constexpr int64_t kSmallLaunchJobs = 1024;                // jobs a small launch is cut into, about

struct RecordOrder {
  int n_direct = 0;
  int64_t jobs = 0;    // jobs of the direct records (4 KiB each, less in small launches)
  int64_t tiles = 0;   // tile codes of the other records
};

// Writes the records of a forward call in launch order: first those that are decoded inside the
// copy kernel (fields with rows under 16 bytes, position ids, cu_seqlens; every field when the
// wide ones are small), then those that go through tile codes.  bytes_of(f, q): bytes of
// destination shard q of field f as the launch is sized; fill(rec, f, q, index): completes a
// record.  Returns false if one launch cannot hold the tiles.
template <class BytesF, class FillF>
bool order_records(BlockBuilder& b, const TileRec* protos, int F, int n_dst, BytesF bytes_of,
                   FillF fill, RecordOrder* out) {
  int64_t coarse_bytes = 0;
  for (int f = 0; f < F; ++f) {
    if (protos[f].tile_shift == kFineTileShift || protos[f].kind == kFieldLinear) continue;
    for (int q = 0; q < n_dst && coarse_bytes <= kDirectMaxCoarseBytes; ++q)
      coarse_bytes += bytes_of(f, q);
  }
  const bool all_direct = coarse_bytes <= kDirectMaxCoarseBytes;
  // Bytes of a direct job.  A launch of a few hundred jobs leaves every wavefront alone on its
  // compute unit, where it issues an instruction every six cycles or so, and the call waits for
  // the longest job: such launches use jobs of 1 or 2 KiB (more wavefronts, each with less to
  // do), and their fields with rows of one or two bytes, whose 4 KiB jobs would span the most
  // segments, jobs of at most 1024 rows.  (On launches that fill the chip smaller jobs measured
  // 5-8 % slower: every job pays the searches again.)
  int64_t direct_bytes = 0, direct_recs = 0;
  for (int f = 0; f < F; ++f) {
    const TileRec& proto = protos[f];
    if (!(all_direct || proto.tile_shift == kFineTileShift || proto.kind == kFieldLinear)) continue;
    for (int q = 0; q < n_dst && direct_bytes <= kSmallLaunchBytes; ++q, ++direct_recs)
      direct_bytes += bytes_of(f, q);
  }
  const bool small_launch = direct_bytes <= kSmallLaunchBytes;
  int small_job_shift = kJobShiftHost;
  if (small_launch) {
    small_job_shift = kJobShiftMin;
    while (small_job_shift < kJobShiftHost &&
           (direct_bytes >> small_job_shift) + direct_recs > kSmallLaunchJobs)
      ++small_job_shift;
  }
  int64_t* ts = b.tile_start();
  TileRec* recs = b.recs();
  RecordOrder o;
  size_t n_rec = 0;
  for (int pass = 0; pass < 2; ++pass) {
    int64_t count = 0;
    for (int f = 0; f < F; ++f) {
      const TileRec& proto = protos[f];
      const bool direct = all_direct || proto.tile_shift == kFineTileShift || proto.kind == kFieldLinear;
      if (direct != (pass == 0)) continue;
      int shift = kTileShift;
      if (direct) {
        shift = small_job_shift;
        if (small_launch && proto.kind != kFieldLinear && proto.row_bytes <= 2)
          shift = proto.row_bytes == 1 ? kJobShiftMin : (shift < kJobShiftMin + 1 ? shift : kJobShiftMin + 1);
      }
      for (int q = 0; q < n_dst; ++q) {
        TileRec& r = recs[n_rec];
        r = proto;
        r.tile_shift = (int16_t)shift;
        r.tile_first = count;
        fill(r, f, q, n_rec);
        ts[n_rec + pass] = count;
        ++n_rec;
        count += (bytes_of(f, q) + ((int64_t)1 << shift) - 1) >> shift;
        if (count > kMaxLaunchTiles) return false;   // (also keeps the running sum from overflowing)
      }
    }
    ts[n_rec + pass] = count;   // closes this part of the table
    if (pass == 0) {
      o.n_direct = (int)n_rec;
      o.jobs = count;
    } else {
      o.tiles = count;
    }
  }
  if (o.tiles * kSubTiles > kMaxLaunchTiles) return false;
  b.hd.n_direct = o.n_direct;
  std::memcpy(b.data, &b.hd, sizeof(b.hd));
  *out = o;
  return true;
}

// Where the direct records of a parameter block will sit in device memory.
void set_direct_view(CopyArgs& ca, const BlockBuilder& b, const RecordOrder& order, void* block_dev) {
  unsigned char* base = static_cast<unsigned char*>(block_dev);
  ca.n_direct_jobs = order.jobs;
  ca.n_direct = order.n_direct;
  ca.direct_tile_start = reinterpret_cast<const int64_t*>(base + b.hd.tile_start_ofs);
  ca.direct_recs = reinterpret_cast<const TileRec*>(base + b.hd.recs_ofs);
  ca.ptrs = reinterpret_cast<const void* const*>(base + b.hd.ptrs_ofs);
}

// earl_dispatch after the plan's summary is on the host.  fixed_block != null: the parameter
// block is built in that host buffer and travels to the device as kernel arguments (nothing is
// allocated, no staging memory is touched); else it is built in a vector and copied through a
// pinned staging slot.
int32_t dispatch_impl(earl_plan* p, const earl_field* fields, int32_t n_fields,
                      int32_t* const* position_ids_shard_ptrs, int32_t* cu_seqlens_dev,
                      void* dispatch_ws_dev, size_t dispatch_ws_bytes, hipStream_t stream,
                      unsigned char* fixed_block, size_t fixed_block_bytes) {
  int32_t st = EARL_OK;
  const int n_dst = p->d.D * p->d.C, S = p->d.S;
  const int64_t* shard_rows = summary_ptr<int64_t>(p, p->l.shard_rows);
  for (int f = 0; f < n_fields; ++f) {
    st = check_field(p, fields[f], f, false);
    if (st != EARL_OK) return st;
  }
  if (position_ids_shard_ptrs) {
    for (int q = 0; q < n_dst; ++q) {
      if (shard_rows[q] == 0) continue;
      if (!position_ids_shard_ptrs[q] ||
          reinterpret_cast<uintptr_t>(position_ids_shard_ptrs[q]) % kVecBytes)
        return fail(EARL_INVALID_ARG, "position ids of shard %d: null or misaligned", q);
    }
  }
  if (cu_seqlens_dev && reinterpret_cast<uintptr_t>(cu_seqlens_dev) % kVecBytes)
    return fail(EARL_INVALID_ARG, "cu_seqlens buffer is misaligned");

  const int extra = (position_ids_shard_ptrs ? 1 : 0) + (cu_seqlens_dev ? 1 : 0);
  const int F = n_fields + extra;
  if (F == 0) return EARL_OK;
  BlockBuilder b;
  if (!b.init(F * n_dst, F, S, n_dst, fixed_block, fixed_block_bytes))
    return fail(EARL_CAPACITY, "the parameter block of this call needs %zu bytes, %zu available",
                b.size, fixed_block_bytes);
  const void** ptrs = b.ptrs();
  // pointer tables and one prototype record per field
  TileRec protos[EARL_MAX_FIELDS + 2];
  uint32_t counter_slot[EARL_MAX_FIELDS + 2];   // first counter row pointer
  const int64_t n_mb_max = p->hdr.n_mb_max;
  bool counting = false;
  uint32_t pi = 0;
  for (int f = 0; f < F; ++f) {
    TileRec& proto = protos[f];
    proto = TileRec{};
    counter_slot[f] = kNoCounters;
    proto.src_ptr_index = pi;
    proto.dst_ptr_index = pi + S;
    if (f < n_fields) {
      const earl_field& uf = fields[f];
      proto.kind = kFieldCopy;
      proto.scalar_bytes = uf.scalar_bytes;
      proto.row_bytes = uf.scalar_bytes * uf.width;
      proto.pad_scalar = replicate_scalar(uf.pad_scalar, uf.scalar_bytes);
      proto.per_sequence = (int16_t)uf.per_sequence;
      for (int s = 0; s < S; ++s) ptrs[pi + s] = uf.src_shard_ptrs[s];
      for (int q = 0; q < n_dst; ++q) ptrs[pi + S + q] = uf.dst_shard_ptrs[q];
      if (uf.nonzero_counts) {
        counting = true;
        counter_slot[f] = pi + S + n_dst;
        for (int q = 0; q < n_dst; ++q) ptrs[pi + S + n_dst + q] = uf.nonzero_counts + q * n_mb_max;
      }
    } else if (position_ids_shard_ptrs && f == n_fields) {
      proto.kind = kFieldPositionIds;
      proto.scalar_bytes = 4;
      proto.row_bytes = 4;
      for (int q = 0; q < n_dst; ++q) ptrs[pi + S + q] = position_ids_shard_ptrs[q];
    } else {
      proto.kind = kFieldLinear;
      proto.scalar_bytes = 4;
      proto.row_bytes = 4;
      ptrs[pi] = p->dev.cu_seqlens;
      ptrs[pi + S] = cu_seqlens_dev;
    }
    proto.tile_shift = (int16_t)tile_shift_of(proto.row_bytes, proto.kind);
    pi += S + 2 * n_dst;
  }
  RecordOrder order;
  const bool fits = order_records(
      b, protos, F, n_dst,
      [&](int f, int q) -> int64_t {
        return protos[f].kind == kFieldLinear ? (q == 0 ? 4ll * p->hdr.cu_seqlens_len : 0)
                                              : shard_rows[q] * (int64_t)protos[f].row_bytes;
      },
      [&](TileRec& r, int f, int q, size_t) {
        r.dst = const_cast<void*>(ptrs[protos[f].dst_ptr_index + q]);
        r.dst_ptr_index = counter_slot[f] == kNoCounters ? kNoCounters : counter_slot[f] + q;
        r.e_begin = p->seg_starts[q];
        r.e_end = p->seg_starts[q + 1];
        r.end_bytes = protos[f].kind == kFieldLinear
                          ? (q == 0 ? 4ll * p->hdr.cu_seqlens_len : 0)
                          : shard_rows[q] * (int64_t)protos[f].row_bytes;
      },
      &order);
  if (!fits) return fail(EARL_INVALID_ARG, "too many tiles for one launch");
  if (order.jobs == 0 && order.tiles == 0) return EARL_OK;
  const size_t codes_off = b.size;
  const size_t need = codes_off + kTileCodeBytes * (size_t)order.tiles;
  if (!dispatch_ws_dev || reinterpret_cast<uintptr_t>(dispatch_ws_dev) % kAlign)
    return fail(EARL_INVALID_ARG, "dispatch scratch is null or not %zu-byte aligned", kAlign);
  if (dispatch_ws_bytes < need)
    return fail(EARL_CAPACITY, "dispatch scratch has %zu bytes, %zu needed", dispatch_ws_bytes, need);
  if (fixed_block) {
    launch_param_chunks(dispatch_ws_dev, b.data, b.size, stream);
  } else {
    st = upload_params(b.data, b.size, dispatch_ws_dev, stream);
    if (st != EARL_OK) return st;
  }
  CopyArgs ca = copy_args(p, dispatch_ws_dev, order.tiles);
  set_direct_view(ca, b, order, dispatch_ws_dev);
  if (counting) {
    for (int f = 0; f < n_fields; ++f)
      if (fields[f].nonzero_counts)
        launch_zero_counters(fields[f].nonzero_counts, n_mb_max * n_dst, stream);
  }
  void* codes = static_cast<unsigned char*>(dispatch_ws_dev) + codes_off;
  if (p->ev_before) HIP_TRY(hipEventRecord(static_cast<hipEvent_t>(p->ev_before), stream));
  launch_direct(ca, stream);
  launch_tile_codes(ca, codes, stream);
  launch_copy(ca, codes, stream);
  if (p->ev_after) HIP_TRY(hipEventRecord(static_cast<hipEvent_t>(p->ev_after), stream));
  hipError_t e = hipGetLastError();
  if (e != hipSuccess)
    return fail(EARL_HIP_ERROR, "re-layout kernel launch failed: %s", hipGetErrorString(e));
  return EARL_OK;
}

}  // namespace

extern "C" {

int32_t earl_dispatch_workspace_bytes(earl_plan* p, const earl_field* fields, int32_t n_fields,
                                      int32_t with_position_ids, int32_t with_cu_seqlens,
                                      size_t* out_bytes) {
  if (!p || !out_bytes) return fail(EARL_INVALID_ARG, "null argument");
  int32_t st = check_field_shapes(fields, n_fields);
  if (st != EARL_OK) return st;
  st = ensure_summary(p);
  if (st != EARL_OK) return st;
  const int F = n_fields + (with_position_ids ? 1 : 0) + (with_cu_seqlens ? 1 : 0);
  int64_t tiles = count_tiles(p, fields, n_fields, with_position_ids != 0, with_cu_seqlens != 0);
  // the same scratch must do for earl_dispatch_inverse with these fields
  int64_t inverse_tiles = 0;
  for (int f = 0; f < n_fields; ++f) {
    const int64_t w = (int64_t)fields[f].scalar_bytes * fields[f].width;
    const int64_t tb = tile_bytes_of(w, kFieldCopy);
    inverse_tiles += (p->hdr.total_real_rows * w + tb - 1) / tb;
  }
  if (inverse_tiles > tiles) tiles = inverse_tiles;
  // (an upper bound for the forward direction, where only the fields with rows of 16 bytes and
  // more of a large launch get tile codes)
  *out_bytes = param_block_bytes(F, p->d.S, p->d.D * p->d.C) + kTileCodeBytes * (size_t)tiles;
  return EARL_OK;
}

int32_t earl_dispatch(earl_plan* p, const earl_field* fields, int32_t n_fields,
                      int32_t* const* position_ids_shard_ptrs, int32_t* cu_seqlens_dev,
                      void* dispatch_ws_dev, size_t dispatch_ws_bytes, void* hip_stream) {
  if (!p) return fail(EARL_INVALID_ARG, "null plan");
  int32_t st = check_field_shapes(fields, n_fields);
  if (st != EARL_OK) return st;
  st = ensure_summary(p);
  if (st != EARL_OK) return st;
  return dispatch_impl(p, fields, n_fields, position_ids_shard_ptrs, cu_seqlens_dev,
                       dispatch_ws_dev, dispatch_ws_bytes, static_cast<hipStream_t>(hip_stream),
                       nullptr, 0);
}

int32_t earl_dispatch_noalloc(earl_plan* p, const earl_field* fields, int32_t n_fields,
                              int32_t* const* position_ids_shard_ptrs, int32_t* cu_seqlens_dev,
                              void* hip_stream) {
  if (!p) return fail(EARL_INVALID_ARG, "null plan");
  int32_t st = check_field_shapes(fields, n_fields);
  if (st != EARL_OK) return st;
  // no wait and no copy here: the caller has fetched the summary (it had to, to size its buffers)
  if (!p->summary_ready)
    return fail(EARL_INVALID_ARG, "earl_dispatch_noalloc needs a plan whose summary has been fetched "
                                  "(earl_plan_get_summary)");
  if (p->status != EARL_OK) return fail(p->status, "the plan failed");
  unsigned char* scratch_dev = nullptr;
  st = static_scratch(&scratch_dev);
  if (st != EARL_OK) return st;
  // one host block and one device array per process and GPU: calls are serialised on the host
  // here, and must not overlap on the device (see the header)
  std::lock_guard<std::mutex> lock(g_noalloc_mu);
  return dispatch_impl(p, fields, n_fields, position_ids_shard_ptrs, cu_seqlens_dev, scratch_dev,
                       kStaticScratchBytes, static_cast<hipStream_t>(hip_stream), g_noalloc_block,
                       sizeof(g_noalloc_block));
}

namespace {

// Tile codes of an asynchronous dispatch: as count_tiles, from buffer capacities; -1 if a capacity
// is out of range or the sum exceeds what one launch can hold.
int64_t count_tiles_by_capacity(const earl_plan* p, const earl_field* fields, int32_t n_fields,
                                const int64_t* position_ids_capacity_rows,
                                int64_t cu_seqlens_capacity) {
  const int n_dst = p->d.D * p->d.C;
  int64_t tiles = 0;
  for (int f = 0; f < n_fields + (position_ids_capacity_rows ? 1 : 0); ++f) {
    const int64_t w = f < n_fields ? (int64_t)fields[f].scalar_bytes * fields[f].width : 4;
    const int64_t* cap = f < n_fields ? fields[f].dst_capacity_rows : position_ids_capacity_rows;
    const int64_t tb = tile_bytes_of(w, kFieldCopy);
    for (int q = 0; q < n_dst; ++q) {
      // cap <= 2^40 rows of w <= 2^20 bytes: one term fits, the running sum is cut off here
      if (cap[q] < 0 || cap[q] > ((int64_t)1 << 40)) return -1;
      tiles += (cap[q] * w + tb - 1) / tb;
      if (tiles > kMaxLaunchTiles) return -1;
    }
  }
  if (cu_seqlens_capacity > 0) tiles += (4 * cu_seqlens_capacity + kTileBytes - 1) / kTileBytes;
  return tiles > kMaxLaunchTiles ? -1 : tiles;
}

// Host-side checks of an asynchronous dispatch: everything that does not need the plan's result.
int32_t check_async_args(const earl_plan* p, const earl_field* fields, int32_t n_fields,
                         int32_t* const* position_ids_shard_ptrs,
                         const int64_t* position_ids_capacity_rows, const int32_t* cu_seqlens_dev,
                         int64_t cu_seqlens_capacity) {
  int32_t st = check_field_shapes(fields, n_fields);
  if (st != EARL_OK) return st;
  const int n_dst = p->d.D * p->d.C, S = p->d.S;
  if ((position_ids_shard_ptrs == nullptr) != (position_ids_capacity_rows == nullptr))
    return fail(EARL_INVALID_ARG, "position ids need both pointers and capacities");
  if (cu_seqlens_capacity < 0 || (cu_seqlens_dev == nullptr) != (cu_seqlens_capacity == 0))
    return fail(EARL_INVALID_ARG, "cu_seqlens needs a buffer and a positive capacity, or neither");
  if (cu_seqlens_capacity > 0x7fffffffll)
    return fail(EARL_INVALID_ARG, "cu_seqlens capacity out of range");
  if (cu_seqlens_dev && reinterpret_cast<uintptr_t>(cu_seqlens_dev) % kVecBytes)
    return fail(EARL_INVALID_ARG, "cu_seqlens buffer is misaligned");
  for (int f = 0; f < n_fields; ++f) {
    const earl_field& uf = fields[f];
    const int64_t w = (int64_t)uf.scalar_bytes * uf.width;
    if (!uf.src_shard_ptrs || !uf.dst_shard_ptrs || !uf.dst_capacity_rows || !uf.src_capacity_rows)
      return fail(EARL_INVALID_ARG, "field %d: null pointer or capacity array", f);
    if (uf.per_sequence != 0 && uf.per_sequence != 1)
      return fail(EARL_INVALID_ARG, "field %d: per_sequence must be 0 or 1", f);
    if (uf.per_sequence && w != 1 && w != 2 && w != 4 && w != 8)
      return fail(EARL_INVALID_ARG, "field %d: a per-sequence field needs 1, 2, 4 or 8 row bytes", f);
    if (uf.nonzero_counts)
      return fail(EARL_INVALID_ARG, "field %d: nonzero_counts needs earl_dispatch", f);
    for (int q = 0; q < n_dst; ++q) {
      if (uf.dst_capacity_rows[q] < 0 || uf.dst_capacity_rows[q] > ((int64_t)1 << 40))
        return fail(EARL_INVALID_ARG, "field %d: capacity of destination %d out of range", f, q);
      if (uf.dst_capacity_rows[q] == 0) continue;
      if (!uf.dst_shard_ptrs[q] || reinterpret_cast<uintptr_t>(uf.dst_shard_ptrs[q]) % kVecBytes)
        return fail(EARL_INVALID_ARG, "field %d: destination %d is null or misaligned", f, q);
    }
    for (int s = 0; s < S; ++s) {
      if (uf.src_capacity_rows[s] < 0)
        return fail(EARL_INVALID_ARG, "field %d: capacity of source %d is negative", f, s);
      if (uf.src_capacity_rows[s] == 0) continue;
      if (!uf.src_shard_ptrs[s] ||
          reinterpret_cast<uintptr_t>(uf.src_shard_ptrs[s]) % (uf.per_sequence ? w : uf.scalar_bytes))
        return fail(EARL_INVALID_ARG, "field %d: source %d is null or misaligned", f, s);
    }
  }
  if (position_ids_shard_ptrs)
    for (int q = 0; q < n_dst; ++q) {
      if (position_ids_capacity_rows[q] < 0 || position_ids_capacity_rows[q] > ((int64_t)1 << 40))
        return fail(EARL_INVALID_ARG, "position ids: capacity of shard %d out of range", q);
      if (position_ids_capacity_rows[q] == 0) continue;
      if (!position_ids_shard_ptrs[q] ||
          reinterpret_cast<uintptr_t>(position_ids_shard_ptrs[q]) % kVecBytes)
        return fail(EARL_INVALID_ARG, "position ids of shard %d are null or misaligned", q);
    }
  return EARL_OK;
}

}  // namespace

int32_t earl_dispatch_async_workspace_bytes(earl_plan* p, const earl_field* fields,
                                            int32_t n_fields,
                                            const int64_t* position_ids_capacity_rows,
                                            int64_t cu_seqlens_capacity, size_t* out_bytes) {
  if (!p || !out_bytes) return fail(EARL_INVALID_ARG, "null argument");
  int32_t st = check_field_shapes(fields, n_fields);
  if (st != EARL_OK) return st;
  for (int f = 0; f < n_fields; ++f)
    if (!fields[f].dst_capacity_rows) return fail(EARL_INVALID_ARG, "field %d: no capacities", f);
  if (cu_seqlens_capacity < 0) return fail(EARL_INVALID_ARG, "negative cu_seqlens capacity");
  const int F = n_fields + (position_ids_capacity_rows ? 1 : 0) + (cu_seqlens_capacity ? 1 : 0);
  const int64_t tiles = count_tiles_by_capacity(p, fields, n_fields, position_ids_capacity_rows,
                                                cu_seqlens_capacity);
  if (tiles < 0) return fail(EARL_INVALID_ARG, "capacities out of range or too many tiles for one launch");
  *out_bytes = param_block_bytes(F, p->d.S, p->d.D * p->d.C) + kTileCodeBytes * (size_t)tiles;
  return EARL_OK;
}

int32_t earl_dispatch_async(earl_plan* p, const earl_field* fields, int32_t n_fields,
                            int32_t* const* position_ids_shard_ptrs,
                            const int64_t* position_ids_capacity_rows, int32_t* cu_seqlens_dev,
                            int64_t cu_seqlens_capacity, void* dispatch_ws_dev,
                            size_t dispatch_ws_bytes, void* hip_stream) {
  if (!p) return fail(EARL_INVALID_ARG, "null plan");
  int32_t st = check_async_args(p, fields, n_fields, position_ids_shard_ptrs,
                                position_ids_capacity_rows, cu_seqlens_dev, cu_seqlens_capacity);
  if (st != EARL_OK) return st;
  const int n_dst = p->d.D * p->d.C, S = p->d.S;
  const int F = n_fields + (position_ids_shard_ptrs ? 1 : 0) + (cu_seqlens_dev ? 1 : 0);
  if (F == 0) return EARL_OK;
  BlockBuilder b;
  b.init(F * n_dst, F, S, n_dst);
  const void** ptrs = b.ptrs();
  int64_t* rec_caps = b.rec_caps();
  int64_t* src_caps = b.src_caps();
  int32_t* src_per_sequence = b.src_per_sequence();
  std::vector<TileRec> protos((size_t)F);
  std::vector<const int64_t*> caps((size_t)F, nullptr);
  uint32_t pi = 0;
  for (int f = 0; f < F; ++f) {
    TileRec& proto = protos[f];
    proto = TileRec{};
    proto.src_ptr_index = pi;
    proto.dst_ptr_index = kNoCounters;
    src_per_sequence[f] = 0;
    for (int s = 0; s < S; ++s) src_caps[(size_t)f * S + s] = -1;
    if (f < n_fields) {
      const earl_field& uf = fields[f];
      proto.kind = kFieldCopy;
      proto.scalar_bytes = uf.scalar_bytes;
      proto.row_bytes = uf.scalar_bytes * uf.width;
      proto.pad_scalar = replicate_scalar(uf.pad_scalar, uf.scalar_bytes);
      proto.per_sequence = (int16_t)uf.per_sequence;
      src_per_sequence[f] = uf.per_sequence;
      caps[f] = uf.dst_capacity_rows;
      for (int s = 0; s < S; ++s) {
        ptrs[pi + s] = uf.src_shard_ptrs[s];
        src_caps[(size_t)f * S + s] = uf.src_capacity_rows[s];
      }
      for (int q = 0; q < n_dst; ++q) ptrs[pi + S + q] = uf.dst_shard_ptrs[q];
    } else if (position_ids_shard_ptrs && f == n_fields) {
      proto.kind = kFieldPositionIds;
      proto.scalar_bytes = 4;
      proto.row_bytes = 4;
      caps[f] = position_ids_capacity_rows;
      for (int q = 0; q < n_dst; ++q) ptrs[pi + S + q] = position_ids_shard_ptrs[q];
    } else {
      proto.kind = kFieldLinear;
      proto.scalar_bytes = 4;
      proto.row_bytes = 4;
      ptrs[pi] = p->dev.cu_seqlens;
      ptrs[pi + S] = cu_seqlens_dev;
    }
    proto.tile_shift = (int16_t)tile_shift_of(proto.row_bytes, proto.kind);
    pi += S + 2 * n_dst;
  }
  // records in launch order; e_begin carries the shard number until the resolve kernel replaces
  // it, end_bytes the capacity that sizes the grid
  auto cap_of = [&](int f, int q) -> int64_t {
    return protos[f].kind == kFieldLinear ? (q == 0 ? cu_seqlens_capacity : 0) : caps[f][q];
  };
  RecordOrder order;
  const bool fits = order_records(
      b, protos.data(), F, n_dst,
      [&](int f, int q) -> int64_t { return cap_of(f, q) * (int64_t)protos[f].row_bytes; },
      [&](TileRec& r, int f, int q, size_t index) {
        r.dst = const_cast<void*>(ptrs[protos[f].src_ptr_index + S + q]);
        r.e_begin = q;
        rec_caps[index] = cap_of(f, q);
        r.end_bytes = cap_of(f, q) * (int64_t)protos[f].row_bytes;
      },
      &order);
  if (!fits) return fail(EARL_INVALID_ARG, "too many tiles for one launch");
  const size_t codes_off = b.size;
  const size_t need = codes_off + kTileCodeBytes * (size_t)order.tiles;
  if (!dispatch_ws_dev || reinterpret_cast<uintptr_t>(dispatch_ws_dev) % kAlign)
    return fail(EARL_INVALID_ARG, "dispatch scratch is null or not %zu-byte aligned", kAlign);
  if (dispatch_ws_bytes < need)
    return fail(EARL_CAPACITY, "dispatch scratch has %zu bytes, %zu needed", dispatch_ws_bytes, need);
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  st = upload_params(b.data, b.size, dispatch_ws_dev, stream);
  if (st != EARL_OK) return st;
  launch_async_resolve(static_cast<DispatchDev*>(dispatch_ws_dev), p->dev, stream);
  p->async_stream = stream;
  p->async_used = true;
  if (order.jobs > 0 || order.tiles > 0) {
    CopyArgs ca = copy_args(p, dispatch_ws_dev, order.tiles);
    set_direct_view(ca, b, order, dispatch_ws_dev);
    void* codes = static_cast<unsigned char*>(dispatch_ws_dev) + codes_off;
    if (p->ev_before) HIP_TRY(hipEventRecord(static_cast<hipEvent_t>(p->ev_before), stream));
    launch_direct(ca, stream);
    launch_tile_codes(ca, codes, stream);
    launch_copy(ca, codes, stream);
    if (p->ev_after) HIP_TRY(hipEventRecord(static_cast<hipEvent_t>(p->ev_after), stream));
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess)
    return fail(EARL_HIP_ERROR, "kernel launch failed: %s", hipGetErrorString(e));
  return EARL_OK;
}

int32_t earl_dispatch_async_status(earl_plan* p, int32_t* status) {
  if (!p || !status) return fail(EARL_INVALID_ARG, "null argument");
  if (!p->async_used) return fail(EARL_INVALID_ARG, "no earl_dispatch_async call on this plan");
  int64_t word = 0;
  HIP_TRY(hipStreamSynchronize(p->async_stream));
  HIP_TRY(hipMemcpy(&word, reinterpret_cast<unsigned char*>(p->dev.hdr) + offsetof(PlanHeader, async_status),
                    sizeof(word), hipMemcpyDeviceToHost));
  *status = (int32_t)word;
  return EARL_OK;
}

int32_t earl_dispatch_inverse(earl_plan* p, const earl_field* fields, int32_t n_fields,
                              void* dispatch_ws_dev, size_t dispatch_ws_bytes, void* hip_stream) {
  if (!p) return fail(EARL_INVALID_ARG, "null plan");
  int32_t st = check_field_shapes(fields, n_fields);
  if (st != EARL_OK) return st;
  st = ensure_summary(p);
  if (st != EARL_OK) return st;
  const int n_dst = p->d.D * p->d.C, S = p->d.S;
  for (int f = 0; f < n_fields; ++f) {
    st = check_field(p, fields[f], f, true);
    if (st != EARL_OK) return st;
  }
  if (n_fields == 0 || p->hdr.total_real_rows == 0) return EARL_OK;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  int64_t* prefix = reinterpret_cast<int64_t*>(p->ws + p->l.seg_real_prefix);
  // the order the stream of real rows is cut in: by source position where the source layout is
  // the packed one (the launch then writes the rollout buffers front to back), else the segment
  // table's own
  const SegRec* segs = p->dev.segs;
  const int32_t* seg_dst_shard = p->dev.seg_dst_shard;
  if (p->source_order) {
    segs = reinterpret_cast<const SegRec*>(p->ws + p->l.segs_src);
    seg_dst_shard = reinterpret_cast<const int32_t*>(p->ws + p->l.seg_dst_shard_src);
  }
  BlockBuilder b;
  b.init(n_fields, n_fields, S, n_dst);
  int64_t* ts = b.tile_start();
  TileRec* recs = b.recs();
  const void** ptrs = b.ptrs();
  // one record per field: first the fields that are decoded inside the copy kernel (rows under
  // 16 bytes; all of them when the wide ones are small), then those that go through tile codes
  int64_t coarse_bytes = 0;
  for (int f = 0; f < n_fields; ++f) {
    const int64_t w = (int64_t)fields[f].scalar_bytes * fields[f].width;
    if (w >= kVecBytes && coarse_bytes <= kDirectMaxCoarseBytes) coarse_bytes += p->hdr.total_real_rows * w;
  }
  const bool all_direct = coarse_bytes <= kDirectMaxCoarseBytes;
  // job size of the direct records, as in the forward direction (order_records)
  int64_t direct_bytes = 0, direct_recs = 0;
  for (int f = 0; f < n_fields && direct_bytes <= kSmallLaunchBytes; ++f) {
    const int64_t w = (int64_t)fields[f].scalar_bytes * fields[f].width;
    if (all_direct || w < kVecBytes) {
      direct_bytes += p->hdr.total_real_rows * w;
      ++direct_recs;
    }
  }
  const bool small_launch = direct_bytes <= kSmallLaunchBytes;
  int small_job_shift = kJobShiftHost;
  if (small_launch) {
    small_job_shift = kJobShiftMin;
    while (small_job_shift < kJobShiftHost &&
           (direct_bytes >> small_job_shift) + direct_recs > kSmallLaunchJobs)
      ++small_job_shift;
  }
  RecordOrder order;
  int n_rec = 0;
  for (int pass = 0; pass < 2; ++pass) {
    int64_t count = 0;
    for (int f = 0; f < n_fields; ++f) {
      const earl_field& uf = fields[f];
      const int64_t w = (int64_t)uf.scalar_bytes * uf.width;
      const bool direct = all_direct || w < kVecBytes;
      if (direct != (pass == 0)) continue;
      int shift = kTileShift;
      if (direct) {
        shift = small_job_shift;
        if (small_launch && w <= 2)
          shift = w == 1 ? kJobShiftMin : (shift < kJobShiftMin + 1 ? shift : kJobShiftMin + 1);
      }
      const uint32_t pi = (uint32_t)f * (uint32_t)(S + n_dst);
      TileRec& r = recs[n_rec];
      r.kind = kFieldCopy;
      r.scalar_bytes = uf.scalar_bytes;
      r.row_bytes = (int32_t)w;
      r.src_ptr_index = pi;
      r.dst_ptr_index = pi + S;
      r.tile_shift = (int16_t)shift;
      for (int s2 = 0; s2 < S; ++s2) ptrs[pi + s2] = uf.src_shard_ptrs[s2];
      for (int q = 0; q < n_dst; ++q) ptrs[pi + S + q] = uf.dst_shard_ptrs[q];
      r.tile_first = count;
      r.end_bytes = p->hdr.total_real_rows * w;
      ts[n_rec + pass] = count;
      ++n_rec;
      count += (r.end_bytes + ((int64_t)1 << shift) - 1) >> shift;
      if (count > kMaxLaunchTiles) return fail(EARL_INVALID_ARG, "too many tiles for one launch");
    }
    ts[n_rec + pass] = count;
    if (pass == 0) {
      order.n_direct = n_rec;
      order.jobs = count;
    } else {
      order.tiles = count;
    }
  }
  if (order.tiles * kSubTiles > kMaxLaunchTiles)
    return fail(EARL_INVALID_ARG, "too many tiles for one launch");
  b.hd.n_direct = order.n_direct;
  std::memcpy(b.data, &b.hd, sizeof(b.hd));
  const size_t codes_off = b.size;
  const size_t need = codes_off + kTileCodeBytes * (size_t)order.tiles;
  if (!dispatch_ws_dev || reinterpret_cast<uintptr_t>(dispatch_ws_dev) % kAlign)
    return fail(EARL_INVALID_ARG, "dispatch scratch is null or not %zu-byte aligned", kAlign);
  if (dispatch_ws_bytes < need)
    return fail(EARL_CAPACITY, "dispatch scratch has %zu bytes, %zu needed", dispatch_ws_bytes, need);
  // The source-ordered copy of the segment table and the per-segment prefix of real rows are
  // computed once per plan, on the stream of the first inverse call; an event recorded behind
  // them orders every later call, whatever its stream.
  if (!p->inverse_ready) {
    hipEvent_t ev = nullptr;
    HIP_TRY(hipEventCreateWithFlags(&ev, hipEventDisableTiming));
    // (in source order the prefix has a closed form, given the plan kernel's scan of the lengths)
    const bool closed_form = p->source_order && p->has_seq_pre;
    if (p->source_order)
      launch_source_order(p->dev.segs, p->dev.seg_dst_shard, p->dev.seg_src_seq,
                          reinterpret_cast<SegRec*>(p->ws + p->l.segs_src),
                          reinterpret_cast<int32_t*>(p->ws + p->l.seg_dst_shard_src),
                          p->hdr.n_segments, p->d.N, p->d.G, p->d.R, p->d.K,
                          closed_form ? p->dev.seq_pre : nullptr, prefix, stream);
    if (!closed_form) launch_real_prefix(segs, prefix, p->hdr.n_segments, stream);
    hipError_t e = hipEventRecord(ev, stream);
    if (e != hipSuccess) {
      (void)hipEventDestroy(ev);
      return fail(EARL_HIP_ERROR, "hipEventRecord failed: %s", hipGetErrorString(e));
    }
    p->inverse_prefix_done = ev;
    p->inverse_stream = stream;
    p->inverse_ready = true;
  } else if (stream != p->inverse_stream) {
    HIP_TRY(hipStreamWaitEvent(stream, static_cast<hipEvent_t>(p->inverse_prefix_done), 0));
  }
  st = upload_params(b.data, b.size, dispatch_ws_dev, stream);
  if (st != EARL_OK) return st;
  CopyArgs ca = copy_args(p, dispatch_ws_dev, order.tiles);
  ca.segs = segs;
  set_direct_view(ca, b, order, dispatch_ws_dev);
  launch_copy_inverse(ca, prefix, seg_dst_shard, p->hdr.n_segments, n_dst,
                      static_cast<unsigned char*>(dispatch_ws_dev) + codes_off,
                      static_cast<hipEvent_t>(p->ev_before), static_cast<hipEvent_t>(p->ev_after),
                      stream);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess)
    return fail(EARL_HIP_ERROR, "inverse kernel launch failed: %s", hipGetErrorString(e));
  return EARL_OK;
}

int32_t earl_plan_set_dispatch_events(earl_plan* p, void* event_before, void* event_after) {
  if (!p) return fail(EARL_INVALID_ARG, "null plan");
  if ((event_before == nullptr) != (event_after == nullptr))
    return fail(EARL_INVALID_ARG, "pass two events or two NULLs");
  p->ev_before = event_before;
  p->ev_after = event_after;
  return EARL_OK;
}

int32_t earl_plan_destroy(earl_plan* p) {
  // a plan that was never waited for: its kernel may still write the mailbox
  if (p && p->mailbox >= 0) release_mailbox(p->mailbox, false);
  if (p && p->inverse_prefix_done)
    (void)hipEventDestroy(static_cast<hipEvent_t>(p->inverse_prefix_done));
  delete p;
  return EARL_OK;
}

const char* earl_status_string(int32_t status) {
  switch (status) {
    case EARL_OK: return "ok";
    case EARL_INVALID_ARG: return "invalid argument";
    case EARL_SEQ_EXCEEDS_BUDGET: return "a padded sequence exceeds the micro-batch token budget";
    case EARL_CAPACITY: return "a buffer is too small";
    case EARL_HIP_ERROR: return "HIP runtime error";
    case EARL_NO_FEASIBLE_CONFIG: return "no feasible configuration for this context length";
    default: return "unknown status";
  }
}

const char* earl_last_error_message(void) { return g_err; }

}  // extern "C"
