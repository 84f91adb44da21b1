// Multi-field ragged re-layout for gfx950: materialises every destination shard of every field.
//
// This is where the bytes of the paper's dispatch move (Section 2, "Data Dispatcher": data goes
// straight from the buffers it was computed into, to the layout the consumer needs; Section 1:
// the volume of these batches is the bottleneck).  The path is pure data movement, bound by HBM
// bandwidth, and its shape follows what was measured on MI355X for plain copies:
//   * the chip streams fastest when every lane does ONE 16-byte load and ONE 16-byte store and
//     the wavefront then ends: stores are fire-and-forget (nothing waits for their
//     acknowledgement) and the wavefronts in flight always cover one compact, advancing window
//     of addresses.  Loops over large tiles, persistent grids and deeper unrolling all measured
//     15-30 % slower, and one-wavefront workgroups beat larger ones.  So a workgroup is one
//     wavefront and owns exactly 1 KiB of one destination shard of one field;
//   * with so little work per wavefront, any search ("which field, which shard, which segment")
//     in front of the load costs more than the copy itself.  A first kernel therefore decodes
//     every tile ONCE, a few consecutive tiles per lane, into a 16-byte tile code per 4 KiB of
//     destination (1 KiB for fields whose rows are shorter than a vector, so that a tile seldom
//     crosses a segment edge): source pointer, destination pointer and what to do.
//     The copy kernel reads its code with one uniform load and, for a tile that lies inside the
//     real part of one segment (nearly all bytes of a wide field), does nothing but load and store;
//   * work is cut on the DESTINATION, every lane owns one whole 16-byte destination vector:
//     stores are aligned global_store_dwordx4 and no two workgroups share a cache line;
//   * a vector inside the real part of a segment is one (possibly unaligned)
//     global_load_dwordx4 from the source shard; padding vectors are stored without a load;
//     vectors that straddle a segment edge are moved scalar by scalar;
//   * loads and stores carry the non-temporal hint: every byte is touched once (the stores of
//     the hot paths system scope as well, see store16_sys);
//   * position ids and cu_seqlens are further "fields" of the same launch.
#include <cstring>

#include "earl_internal.h"

namespace earl {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef u32x4 u32x4_u __attribute__((aligned(1)));
typedef unsigned char u8;

// All field buffers are global (HBM) memory: say so, or pointers rebuilt from integers compile to
// FLAT instead of GLOBAL loads and stores.
#define EARL_GLOBAL __attribute__((address_space(1)))
__device__ __forceinline__ u32x4 load16(const u8* p) {
  return __builtin_nontemporal_load((const EARL_GLOBAL u32x4_u*)p);
}
__device__ __forceinline__ void store16(u8* p, u32x4 v) {
  __builtin_nontemporal_store(v, (EARL_GLOBAL u32x4*)p);
}
// The store of the hot paths: system scope on top of the non-temporal hint measured 0.6-1.1 %
// faster than the hint alone on the full-size workloads (0.8 % on a plain 8 GiB copy); the
// compiler has no builtin for this combination, hence the instruction by name.  Any alignment.
__device__ __forceinline__ void store16_sys(u8* p, u32x4 v) {
  asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1 nt"
               :: "v"((EARL_GLOBAL u32x4_u*)p), "v"(v) : "memory");
}
__device__ __forceinline__ void store16_any(u8* p, u32x4 v) {
  __builtin_nontemporal_store(v, (EARL_GLOBAL u32x4_u*)p);
}

// Between LDS writes of some lanes and LDS reads of other lanes of the SAME wavefront: without it
// the compiler may hoist a read above a write it can prove to be to a different address for the
// reading lane itself (seen in the ISA of an earlier kernel: the values then came out stale).
// Wavefront scope costs no instruction; the hardware already keeps a wavefront's LDS
// operations in order.
__device__ __forceinline__ void wave_exchange_fence() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

__device__ __forceinline__ uint64_t load_scalar(const u8* p, int sb) {
  switch (sb) {
    case 1: return *p;
    case 2: return *reinterpret_cast<const uint16_t*>(p);
    case 4: return *reinterpret_cast<const uint32_t*>(p);
    default: return *reinterpret_cast<const uint64_t*>(p);
  }
}
__device__ __forceinline__ void store_scalar(u8* p, uint64_t v, int sb) {
  switch (sb) {
    case 1: *p = (u8)v; break;
    case 2: *reinterpret_cast<uint16_t*>(p) = (uint16_t)v; break;
    case 4: *reinterpret_cast<uint32_t*>(p) = (uint32_t)v; break;
    default: *reinterpret_cast<uint64_t*>(p) = v; break;
  }
}

// Last record x in [lo, hi) of `table` with table[x] <= v, one lane on its own.
__device__ __forceinline__ int last_le(const int64_t* table, int lo, int hi, int64_t v) {
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (table[mid] <= v) lo = mid; else hi = mid;
  }
  return lo;
}

// Last segment e in [lo, hi) whose first destination byte (dst_row * w) is <= byte; requires
// that of segment lo to be.
__device__ __forceinline__ int find_segment(const SegRec* segs, int lo, int hi, int64_t byte,
                                            int64_t w) {
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (segs[mid].dst_row * w <= byte) lo = mid; else hi = mid;
  }
  return lo;
}

// A segment as destination byte ranges of its shard, plus where its bytes come from.
struct SegCursor {
  int64_t lo, real_hi, hi;   // [lo, real_hi) real rows, [real_hi, hi) padding rows
  const u8* src;             // source byte that lands on destination byte lo
  int32_t pos0;
  int e;
};

// seg_src_seq != null: a per-sequence field, whose source row is the sequence's row.
__device__ __forceinline__ void load_segment(const SegRec* segs, const int32_t* seg_src_seq,
                                             const void* const* src_ptrs, int64_t w, int e,
                                             SegCursor& sc) {
  const SegRec r = segs[e];
  sc.e = e;
  sc.lo = r.dst_row * w;
  sc.real_hi = (r.dst_row + r.n_real) * w;
  sc.hi = (r.dst_row + r.n_rows) * w;
  sc.pos0 = r.pos0;
  const int64_t src_row = seg_src_seq ? (int64_t)seg_src_seq[e] : r.src_row;
  sc.src = src_ptrs ? static_cast<const u8*>(src_ptrs[r.src_shard]) + src_row * w : nullptr;
}

// 8 bytes holding copies of the low w bytes of v (w in {1, 2, 4, 8}).
__device__ __forceinline__ uint64_t splat_scalar(uint64_t v, int w) {
  if (w >= 8) return v;
  v &= (1ull << (8 * w)) - 1ull;
  for (int b = w; b < 8; b *= 2) v |= v << (8 * b);
  return v;
}

// Non-zero scalars (of 1 << sb_log2 bytes) among the 16 bytes of v.
__device__ __forceinline__ int count_nonzero16(u32x4 v, int sb_log2) {
  int n = 0;
  if (sb_log2 == 3) {
    n = ((v.x | v.y) != 0) + ((v.z | v.w) != 0);
  } else if (sb_log2 == 2) {
    n = (v.x != 0) + (v.y != 0) + (v.z != 0) + (v.w != 0);
  } else {
    // per scalar: the top bit of (low bits + all-ones-below-top) | value is set iff it is non-zero
    const uint32_t low = sb_log2 == 1 ? 0x7fff7fffu : 0x7f7f7f7fu;
    for (int k = 0; k < 4; ++k) {
      const uint32_t x = v[k];
      n += __builtin_popcount((((x & low) + low) | x) & ~low);
    }
  }
  return n;
}

__device__ __forceinline__ void add_to_counter(int64_t* counter, int n) {
  if (n) atomicAdd(reinterpret_cast<unsigned long long*>(counter), (unsigned long long)n);
}

// Tile codes (fields with rows of 16 bytes and more, in launches large enough to pay for the code
// pass).  `b` holds the destination pointer of the tile's first byte (16-byte aligned) with the
// action in its low four bits; `a` depends on the action.
enum TileAction : uint64_t {
  kActCopy = 0,      // a = source pointer of the tile's first byte: the tile is a straight copy
  kActFill = 1,      // a = padding scalar replicated to 8 bytes: the whole tile repeats it
  kActGeneric = 3,   // a = record index << 32 | segment of the tile's first byte
  kActSkip = 5,      // nothing to do: the tile lies behind the end of its shard (a grid sized by
                     // buffer capacities, earl_dispatch_async)
};
struct TileCode {
  uint64_t a, b;
};

struct ParamView {
  const int64_t* tile_start;
  const TileRec* recs;
  const void* const* ptrs;
  int n_recs;
};
// The records that go through tile codes (all records of an inverse call).
__device__ __forceinline__ ParamView view_params(const DispatchDev* p) {
  const u8* base = reinterpret_cast<const u8*>(p);
  const DispatchDev hd = *p;
  ParamView v;
  v.tile_start = reinterpret_cast<const int64_t*>(base + hd.tile_start_ofs) + (hd.n_direct + 1);
  v.recs = reinterpret_cast<const TileRec*>(base + hd.recs_ofs) + hd.n_direct;
  v.ptrs = reinterpret_cast<const void* const*>(base + hd.ptrs_ofs);
  v.n_recs = hd.n_recs - hd.n_direct;
  return v;
}
// Pass 1: every lane writes the codes of kTilesPerLane consecutive tiles.
//
// The searches (which record, which segment) are chains of dependent loads, a few microseconds
// per wavefront whatever the number of tiles it covers, so the kernel's time is that latency times
// the number of wavefront rounds.  Two things shorten it: the 64 lanes of a wavefront cover
// consecutive tiles, so the search is done once for the first lane with uniform values (scalar
// loads) and every lane only checks whether the answer holds for its own first tile; and a lane
// carries record and segment from one of its tiles to the next, searching again only when the
// next tile has left them.
struct TileCursor {
  int x;            // record of the current tile
  TileRec rec;
  int64_t x_end;    // first tile of the next record
  int e;            // segment holding the tile's first byte (copy and position-id records)
  SegRec seg;
};

__device__ __forceinline__ void cursor_set_record(const ParamView& pv, TileCursor& cur, int x) {
  cur.x = x;
  cur.rec = pv.recs[x];
  cur.x_end = pv.tile_start[x + 1];
}

__device__ __forceinline__ TileCode code_of_tile(const CopyArgs& a, const ParamView& pv,
                                                 const TileCursor& cur, int64_t tile) {
  const TileRec& rec = cur.rec;
  const int64_t lo = (tile - rec.tile_first) << rec.tile_shift;
  const int64_t hi = lo + ((int64_t)1 << rec.tile_shift);
  const uint64_t dst = reinterpret_cast<uint64_t>(static_cast<u8*>(rec.dst) + lo);
  TileCode c;
  c.a = (uint64_t)(uint32_t)cur.x << 32;
  c.b = dst | kActGeneric;
  if (lo >= rec.end_bytes) {
    c.b = dst | kActSkip;
    return c;
  }
  const int64_t w = rec.row_bytes;
  const SegRec& r = cur.seg;
  const int64_t s_lo = r.dst_row * w;
  const int64_t s_real_hi = (r.dst_row + r.n_real) * w;
  const int64_t s_hi = (r.dst_row + r.n_rows) * w;
  c.a |= (uint32_t)cur.e;
  if (hi > rec.end_bytes) return c;
  if (hi <= s_real_hi) {
    const u8* shard = static_cast<const u8*>(pv.ptrs[rec.src_ptr_index + r.src_shard]);
    c.a = reinterpret_cast<uint64_t>(shard + r.src_row * w + (lo - s_lo));
    c.b = dst | kActCopy;
  } else if (lo >= s_real_hi && hi <= s_hi) {
    c.a = rec.pad_scalar;
    c.b = dst | kActFill;
  }
  return c;
}

// The codes of the kTilesPerLane tiles that start at `first` (first < n_tiles), written to out[0..].
__device__ __forceinline__ void tile_codes_of_lane(const CopyArgs& a, const int64_t first,
                                                   TileCode* out) {
  const ParamView pv = view_params(a.params);
  // the wavefront's first tile: uniform, searched with scalar loads
  const int64_t tile0 = ((int64_t)__builtin_amdgcn_readfirstlane((int)(first >> 32)) << 32) |
                        (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)first);
  const int x0 = last_le(pv.tile_start, 0, pv.n_recs, tile0);
  const TileRec rec0 = pv.recs[x0];
  // (a shard without segments has no rows: all its tiles, if a capacity-sized grid gave it any,
  // are skipped before a segment is looked at)
  int e_guess = rec0.e_begin;
  if (rec0.e_begin < rec0.e_end)
    e_guess = find_segment(a.segs, rec0.e_begin, rec0.e_end,
                           (tile0 - rec0.tile_first) << rec0.tile_shift, rec0.row_bytes);

  TileCursor cur;
  cursor_set_record(pv, cur, first < pv.tile_start[x0 + 1] ? x0
                                                             : last_le(pv.tile_start, x0, pv.n_recs, first));
  cur.e = cur.rec.e_begin;
  if (cur.rec.e_begin < cur.rec.e_end) {
    const int64_t w = cur.rec.row_bytes;
    const int64_t lo = (first - cur.rec.tile_first) << cur.rec.tile_shift;
    if (cur.x == x0) {
      const SegRec g = a.segs[e_guess];
      cur.e = lo < (g.dst_row + g.n_rows) * w ? e_guess
                                               : find_segment(a.segs, e_guess, cur.rec.e_end, lo, w);
    } else {
      cur.e = find_segment(a.segs, cur.rec.e_begin, cur.rec.e_end, lo, w);
    }
    cur.seg = a.segs[cur.e];
  }
  const int64_t last = first + kTilesPerLane < a.n_tiles ? first + kTilesPerLane : a.n_tiles;
  for (int64_t tile = first; tile < last; ++tile) {
    if (tile != first) {
      if (tile >= cur.x_end) {
        // next record (records without tiles are skipped by the search)
        cursor_set_record(pv, cur, last_le(pv.tile_start, cur.x, pv.n_recs, tile));
        cur.e = cur.rec.e_begin;
        if (cur.rec.e_begin < cur.rec.e_end) cur.seg = a.segs[cur.e];
      }
      if (cur.rec.e_begin < cur.rec.e_end) {
        const int64_t w = cur.rec.row_bytes;
        const int64_t lo = (tile - cur.rec.tile_first) << cur.rec.tile_shift;
        if (lo >= (cur.seg.dst_row + cur.seg.n_rows) * w) {
          cur.e = find_segment(a.segs, cur.e, cur.rec.e_end, lo, w);
          cur.seg = a.segs[cur.e];
        }
      }
    }
    out[tile - first] = code_of_tile(a, pv, cur, tile);
  }
}


__global__ __launch_bounds__(kCodeThreads) void tile_code_kernel(const CopyArgs a, TileCode* codes) {
  // A lane's kTilesPerLane codes are consecutive, so storing them straight from the lanes would
  // scatter 16-byte pieces at a 64-byte stride; they pass through LDS instead and leave as whole
  // 1 KiB rows of the wavefront's 256 codes.  Only lanes of one wavefront exchange data, and the
  // hardware completes a wavefront's LDS operations in order, so no s_barrier is needed; the
  // compiler, however, must be told not to move the reads above the other lanes' writes
  // (wave_exchange_fence).
  __shared__ TileCode s_codes[kCodeThreads / kWave][kWave * kTilesPerLane];
  const int lane = threadIdx.x & (kWave - 1);
  TileCode* mine = s_codes[threadIdx.x / kWave];
  const int64_t wave_first =
      ((int64_t)blockIdx.x * kCodeThreads + (threadIdx.x - lane)) * kTilesPerLane;
  if (wave_first >= a.n_tiles) return;   // uniform per wavefront
  const int64_t first = wave_first + (int64_t)lane * kTilesPerLane;
  if (first < a.n_tiles) tile_codes_of_lane(a, first, mine + lane * kTilesPerLane);
  wave_exchange_fence();
#pragma unroll
  for (int j = 0; j < kTilesPerLane; ++j) {
    const int64_t tile = wave_first + j * kWave + lane;
    if (tile < a.n_tiles) codes[tile] = mine[j * kWave + lane];
  }
}

// What the generic path needs about its tile.
struct TileInfo {
  u8* dst;                   // destination shard
  int64_t end;               // bytes of the destination shard
  uint64_t pad_scalar;
  const void* const* src_ptrs;
  const int32_t* seg_src_seq;   // non-null for a per-sequence field
  int64_t* counters;            // non-null for a counting field: this shard's counter row
  int32_t e_end;
  int32_t row_bytes;
  int32_t scalar_bytes;
  int32_t kind;
};

// Moves a lane's cursor to the segment that holds destination byte o >= sc.lo.
__device__ __forceinline__ void seek(const SegRec* segs, const TileInfo& t, int64_t o, SegCursor& sc) {
  if (o < sc.hi) return;
  const int64_t w = t.row_bytes;
  int e = sc.e + 1;
  if (e + 1 < t.e_end && segs[e + 1].dst_row * w <= o) e = find_segment(segs, e + 1, t.e_end, o, w);
  load_segment(segs, t.seg_src_seq, t.src_ptrs, w, e, sc);
}

// Places the 16-byte destination vector at byte o of the record's shard on its own: aligned
// 16-byte store and possibly unaligned 16-byte load when the whole vector lies in the real part
// of one segment, fill or position ids when it lies in padding / one segment, scalar-sized moves
// when it straddles a segment edge, the real/padding edge or the end of the shard.  e: a
// segment of the shard that starts at or before byte o.
__device__ __forceinline__ void place_vector(const CopyArgs& a, const ParamView& pv,
                                             const TileRec& rec, int e, const int64_t o) {
  if (o >= rec.end_bytes) return;
  u8* dst = static_cast<u8*>(rec.dst);
  const int64_t o_end = o + kVecBytes;
  TileInfo t;
  t.dst = dst;
  t.end = rec.end_bytes;
  t.pad_scalar = rec.pad_scalar;
  t.src_ptrs = rec.kind == kFieldPositionIds ? nullptr : pv.ptrs + rec.src_ptr_index;
  t.seg_src_seq = rec.per_sequence ? a.seg_src_seq : nullptr;
  t.counters = rec.kind == kFieldCopy && rec.dst_ptr_index != kNoCounters
                   ? static_cast<int64_t*>(const_cast<void*>(pv.ptrs[rec.dst_ptr_index]))
                   : nullptr;
  t.e_end = rec.e_end;
  t.row_bytes = rec.row_bytes;
  t.scalar_bytes = rec.scalar_bytes;
  t.kind = rec.kind;
  SegCursor sc;
  load_segment(a.segs, t.seg_src_seq, t.src_ptrs, rec.row_bytes, e, sc);
  seek(a.segs, t, o, sc);
  if (rec.kind == kFieldCopy) {
    if (o_end <= sc.real_hi) {
      if (t.seg_src_seq) {
        const uint64_t v = splat_scalar(load_scalar(sc.src, rec.row_bytes), rec.row_bytes);
        store16(dst + o, u32x4{(uint32_t)v, (uint32_t)(v >> 32), (uint32_t)v, (uint32_t)(v >> 32)});
      } else {
        const u32x4 v = load16(sc.src + (o - sc.lo));
        store16(dst + o, v);
        if (t.counters)
          add_to_counter(t.counters + a.seg_mb[sc.e],
                         count_nonzero16(v, 31 - __builtin_clz(rec.scalar_bytes)));
      }
      return;
    }
    if (o >= sc.real_hi && o_end <= sc.hi) {
      const uint64_t p = t.pad_scalar;
      store16(dst + o, u32x4{(uint32_t)p, (uint32_t)(p >> 32), (uint32_t)p, (uint32_t)(p >> 32)});
      return;
    }
  } else if (o_end <= sc.hi) {
    const uint32_t p0 = (uint32_t)(sc.pos0 + (int32_t)((o - sc.lo) >> 2));
    store16(dst + o, u32x4{p0, p0 + 1, p0 + 2, p0 + 3});
    return;
  }
  // the vector straddles a segment edge, the real/padding edge or the end of the shard
  const int sb = t.scalar_bytes;
  for (int64_t b = o; b < o_end && b < t.end; b += sb) {
    seek(a.segs, t, b, sc);
    if (t.kind == kFieldPositionIds) {
      store_scalar(dst + b, (uint64_t)(uint32_t)(sc.pos0 + (int32_t)((b - sc.lo) >> 2)), 4);
    } else if (b < sc.real_hi) {
      // a per-sequence row is at most 8 bytes: byte (b - lo) mod w of it
      const int64_t off = t.seg_src_seq ? (b - sc.lo) % t.row_bytes : (b - sc.lo);
      const uint64_t v = load_scalar(sc.src + off, sb);
      store_scalar(dst + b, v, sb);
      if (t.counters) add_to_counter(t.counters + a.seg_mb[sc.e], v != 0);
    } else {
      store_scalar(dst + b, t.pad_scalar, sb);
    }
  }
}

// A tile that is not one plain copy / fill / iota: every lane places its own 16-byte vector.
// `tile` is the tile's code index, `vec0` the first 16-byte vector of the tile this workgroup owns.
__device__ __forceinline__ void generic_tile(const CopyArgs a, const TileCode c, const int64_t tile,
                                          const uint32_t vec0) {
  const ParamView pv = view_params(a.params);
  const TileRec rec = pv.recs[(uint32_t)(c.a >> 32)];
  const int64_t lo = (tile - rec.tile_first) << rec.tile_shift;
  const int64_t o = lo + (int64_t)(vec0 + threadIdx.x) * kVecBytes;   // this lane's vector
  if (o >= rec.end_bytes) return;
  place_vector(a, pv, rec, (int)(uint32_t)c.a, o);
}

// Pass 2: one-wavefront workgroups, one 16-byte vector per lane, kSubTiles workgroups per 4 KiB
// tile code.  The second launch bound asks for 8 wavefronts per SIMD (at most 64 VGPRs): at 7
// the copy measured 2.5 % slower; every wavefront waits for its tile code and then for its data,
// so the bytes in flight, and with them the bandwidth, follow the number of resident wavefronts.
// The rare path is inlined: as a called function it kept its uniform arguments in vector
// registers and saved callee-saved registers to scratch memory, and a kernel that owns scratch
// memory starts about 9 us later.
__global__ __launch_bounds__(kCopyThreads, 8) void relayout_kernel(const CopyArgs a,
                                                                   const TileCode* __restrict__ codes) {
  // consecutive workgroups go to different XCDs; grouping a tile's workgroups on one XCD
  // measured 5-12 % slower, so the hardware order is kept
  const int64_t tile = blockIdx.x / kSubTiles;
  const uint32_t vec0 = (uint32_t)(blockIdx.x % kSubTiles) * kCopyThreads;
  const TileCode c = codes[tile];
  const uint64_t act = c.b & 15u;
  const uint32_t v = vec0 + threadIdx.x;   // vector in the tile
  u8* dst = reinterpret_cast<u8*>(c.b & ~(uint64_t)15) + v * kVecBytes;
  // the plain copy first and on its own: nearly every workgroup takes it
  if (__builtin_expect(act == kActCopy, 1)) {
    store16_sys(dst, load16(reinterpret_cast<const u8*>(c.a) + v * kVecBytes));
    return;
  }
  if (act == kActFill) {
    store16_sys(dst, u32x4{(uint32_t)c.a, (uint32_t)(c.a >> 32), (uint32_t)c.a, (uint32_t)(c.a >> 32)});
  } else if (act == kActGeneric) {
    generic_tile(a, c, tile, vec0);
  }
}

// ---------------------------------------------------------------------------------------
// Decode and copy in one kernel ("direct" records).
//
// The tile-code pass costs a second launch and, on a batch of narrow fields (a few scalars per
// token, the paper's usual payload: Section 3.3 dispatches log-probabilities), 70 % of the
// copy's time; and with rows shorter than a vector most tiles of such a field cross a segment
// edge, where the coded kernel falls back to a search per lane.  Here a one-wavefront workgroup
// owns a JOB of 4 KiB (less in small launches) of one destination shard and finds its way with
// the whole wavefront:
//   * which record, which first segment: 64-way searches (every lane probes one entry, a ballot
//     counts the entries at or below the target), two rounds for up to 4096 entries where a
//     binary search makes twelve dependent loads;
//   * lane l then fetches segment e + l, so the job's segments (rarely more than a handful) sit
//     in registers, as byte ranges relative to the job; for each of the job's four 1 KiB
//     sub-tiles a short uniform loop hands them out with v_readlane and every lane picks the one
//     its 16-byte vector lies in: plain copy, padding, position ids, or, for the few vectors that
//     straddle an edge, the scalar path of place_vector.
// Used for every field with rows under 16 bytes, position ids and cu_seqlens, and for all
// fields of launches too small to amortise a code pass.
// ---------------------------------------------------------------------------------------
constexpr int kJobShift = 12;
constexpr int kJobBytes = 1 << kJobShift;
constexpr int kJobSubTiles = kJobBytes / (kCopyThreads * kVecBytes);
constexpr int32_t kFar = 1 << 30;   // job-relative byte offsets are clamped to +-kFar

// Last x in [0, n) with key(x) <= v, for key ascending and key(0) <= v; all lanes take part and
// get the same answer.  Equal keys: the last one (entries without tiles are skipped).
template <class KeyF>
__device__ __forceinline__ int wave_last_le(int n, int64_t v, KeyF key) {
  int lo = 0, end = n;
  while (end - lo > 1) {
    const int step = (end - lo + kWave - 1) >> 6;
    const int idx = lo + (int)threadIdx.x * step;
    const bool ok = idx < end && key(idx) <= v;   // true on a prefix of the lanes, lane 0 included
    const int cnt = __builtin_popcountll(__ballot(ok));
    lo += (cnt - 1) * step;
    end = end < lo + step ? end : lo + step;
  }
  return lo;
}

__device__ __forceinline__ int32_t clamp_far(int64_t v) {
  return v < -(int64_t)kFar ? -kFar : (v > (int64_t)kFar ? kFar : (int32_t)v);
}
__device__ __forceinline__ uint64_t readlane_u64(uint64_t x, int l) {
  const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)x, l);
  const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(x >> 32), l);
  return ((uint64_t)hi << 32) | lo;
}

enum VecMode : int { kVecNone = 0, kVecPending, kVecCopy, kVecSplat, kVecPad, kVecIota, kVecSlow };

// A segment as the job sees it: byte ranges relative to the job's first byte.
struct SegView {
  int32_t lo, real_hi, hi;   // [lo, real_hi) real rows, [real_hi, hi) padding rows
  uint64_t src;              // copy: address of the source byte of the job's byte 0; per-sequence:
                             // the sequence's value replicated to 8 bytes
  int32_t pos;               // position id of the job's byte 0
};

// A record held by one lane, handed to all lanes.
__device__ __forceinline__ TileRec broadcast_record(const TileRec& mine, int from_lane) {
  union {
    TileRec rec;
    uint32_t word[sizeof(TileRec) / 4];
  } in, out;
  in.rec = mine;
#pragma unroll
  for (int k = 0; k < (int)(sizeof(TileRec) / 4); ++k)
    out.word[k] = (uint32_t)__builtin_amdgcn_readlane((int)in.word[k], from_lane);
  return out.rec;
}

// The last record with tile_first <= job (records without jobs share it with their successor),
// found by the whole wavefront and handed to all its lanes.
__device__ __forceinline__ TileRec record_of_job(const ParamView& pv, int64_t job) {
  const int lane = threadIdx.x;
  int lo = 0, end = pv.n_recs;
  while (end - lo > kWave) {
    const int step = (end - lo + kWave - 1) >> 6;
    const int idx = lo + lane * step;
    const bool ok = idx < end && pv.recs[idx].tile_first <= job;
    lo += (__builtin_popcountll(__ballot(ok)) - 1) * step;
    end = end < lo + step ? end : lo + step;
  }
  TileRec mine = {};
  const bool valid = lo + lane < end;
  if (valid) mine = pv.recs[lo + lane];
  const int holder = __builtin_popcountll(__ballot(valid && mine.tile_first <= job)) - 1;
  return broadcast_record(mine, holder);
}

// The same on the compact table of first jobs (8 bytes per record): one more dependent load, the
// record itself, but 512 bytes of probes per wavefront instead of 4 KiB of whole records.
__device__ __forceinline__ TileRec record_of_job_light(const ParamView& pv, int64_t job) {
  const int r = wave_last_le(pv.n_recs, job, [&](int x) { return pv.tile_start[x]; });
  return pv.recs[__builtin_amdgcn_readfirstlane(r)];
}

__global__ __launch_bounds__(kCopyThreads, 8) void relayout_direct_kernel(const CopyArgs a) {
  // Everything up to the first data load is a chain of dependent memory round trips (each about
  // two microseconds when the plan and the parameter block were written on another XCD), and on a
  // small batch the kernel's time is that chain: it is kept to three or four.  Record and first
  // segment are found by 64-way probes that narrow the range, and the last probe of each search
  // fetches whole entries, so that the lane that holds the answer hands the record to the
  // wavefront, and the lanes behind the first segment already hold the job's segments.  The
  // field's source pointers are fetched one per lane while the segments are searched.
  ParamView pv;
  pv.tile_start = a.direct_tile_start;
  pv.recs = a.direct_recs;
  pv.ptrs = a.ptrs;
  pv.n_recs = a.n_direct;
  const int lane = threadIdx.x;
  const int64_t job = blockIdx.x;
  // (a launch of few jobs is latency-bound and takes the search with one round trip less; a
  // launch that fills the chip takes the one that reads an eighth of the bytes: 7-10 % faster on
  // the narrow fields of the two large workloads)
  const TileRec rec = a.n_direct_jobs > 2048 ? record_of_job_light(pv, job) : record_of_job(pv, job);
  // a job is 4 KiB of the shard, or 1 or 2 KiB where the host chose that for the record (rows of
  // one or two bytes, whose jobs would otherwise span many segments)
  const int64_t lo0 = (job - rec.tile_first) << rec.tile_shift;   // first byte of the job in its shard
  if (lo0 >= rec.end_bytes) return;   // behind the shard's end (a grid sized by capacities)
  u8* const dst = static_cast<u8*>(rec.dst) + lo0;
  const int32_t job_bytes = 1 << rec.tile_shift;
  const int32_t job_len = rec.end_bytes - lo0 < job_bytes ? (int32_t)(rec.end_bytes - lo0) : job_bytes;

  if (rec.kind == kFieldLinear) {
    const u8* src = static_cast<const u8*>(pv.ptrs[rec.src_ptr_index]) + lo0;
#pragma unroll
    for (int t = 0; t < kJobSubTiles; ++t) {
      const int32_t o = (t * kCopyThreads + lane) * kVecBytes;
      if (o + kVecBytes <= job_len) {
        store16_sys(dst + o, load16(src + o));
      } else {
        for (int32_t b = o; b < job_len; b += 4)
          *reinterpret_cast<uint32_t*>(dst + b) = *reinterpret_cast<const uint32_t*>(src + b);
      }
    }
    return;
  }

  const int64_t w = rec.row_bytes;
  const bool is_pos = rec.kind == kFieldPositionIds;
  const bool per_seq = rec.per_sequence != 0;
  const bool counting = rec.kind == kFieldCopy && rec.dst_ptr_index != kNoCounters;
  // source pointers of the field, one per lane (up to 64 shards; more are looked up per segment)
  const bool ptrs_in_lanes = !is_pos && a.n_src_shards <= kWave;
  uint64_t lane_ptr = 0;
  if (ptrs_in_lanes && lane < a.n_src_shards)
    lane_ptr = reinterpret_cast<uint64_t>(pv.ptrs[rec.src_ptr_index + lane]);

  // the segment that holds the job's first byte: narrow to at most 8 candidates, then fetch 64
  // whole segments from the first candidate on
  const int n_seg = rec.e_end - rec.e_begin;
  int first = 0;
  {
    int end = n_seg;
    while (end - first > 8) {
      const int step = (end - first + kWave - 1) >> 6;
      const int idx = first + lane * step;
      const bool ok = idx < end && a.segs[rec.e_begin + idx].dst_row * w <= lo0;
      first += (__builtin_popcountll(__ballot(ok)) - 1) * step;
      end = end < first + step ? end : first + step;
    }
  }
  const int idx = rec.e_begin + first + lane;
  const bool fetched = first + lane < n_seg;
  SegRec r = {};
  int32_t seq_row = 0, seg_mb = 0;
  if (fetched) {
    r = a.segs[idx];
    if (per_seq) seq_row = a.seg_src_seq[idx];
    if (counting) seg_mb = a.seg_mb[idx];
  }
  const int64_t s_lo = r.dst_row * w;
  const int shift = __builtin_popcountll(__ballot(fetched && s_lo <= lo0)) - 1;   // lane of the job's first segment
  const int e0 = rec.e_begin + first + shift;
  SegView win;            // this lane's segment, as the job sees it
  win.lo = win.real_hi = win.hi = kFar;
  win.src = 0;
  win.pos = 0;
  {
    uint64_t shard_ptr = (uint64_t)__shfl((unsigned long long)lane_ptr, r.src_shard);
    if (fetched) {
      win.lo = clamp_far(s_lo - lo0);
      win.real_hi = clamp_far(s_lo + (int64_t)r.n_real * w - lo0);
      win.hi = clamp_far(s_lo + (int64_t)r.n_rows * w - lo0);
      if (is_pos) {
        win.pos = r.pos0 + (int32_t)((lo0 - s_lo) >> 2);
      } else if (r.n_real > 0) {
        if (!ptrs_in_lanes) shard_ptr = reinterpret_cast<uint64_t>(pv.ptrs[rec.src_ptr_index + r.src_shard]);
        const u8* shard = reinterpret_cast<const u8*>(shard_ptr);
        if (per_seq)
          win.src = splat_scalar(load_scalar(shard + (int64_t)seq_row * w, (int)w), (int)w);
        else
          win.src = reinterpret_cast<uint64_t>(shard + r.src_row * w + (lo0 - s_lo));
      }
    }
  }
  // move the window down so that lane k holds segment e0 + k
  {
    const int from = lane + shift;
    const bool in = from < kWave;
    const int32_t lo_ = __shfl(win.lo, from), rh_ = __shfl(win.real_hi, from), hi_ = __shfl(win.hi, from);
    const uint64_t src_ = (uint64_t)__shfl((unsigned long long)win.src, from);
    const int32_t pos_ = __shfl(win.pos, from), mb_ = __shfl(seg_mb, from);
    win.lo = in ? lo_ : kFar;
    win.real_hi = in ? rh_ : kFar;
    win.hi = in ? hi_ : kFar;
    win.src = src_;
    win.pos = pos_;
    seg_mb = mb_;
  }
  const int window_lanes = kWave - shift;   // segments the window can hold
  const int n_win = __builtin_popcountll(__ballot(win.lo < job_len));   // the job's segments in the window
  // The window misses some of the job's segments only when they average under 64 bytes; vectors
  // that reach beyond it (past window_hi) then take the per-lane path as a whole.
  const bool window_complete = n_win < window_lanes || e0 + window_lanes >= rec.e_end;
  const int32_t window_hi =
      window_complete ? kFar : __builtin_amdgcn_readlane(win.hi, window_lanes - 1);

  const int sb_log2 = 31 - __builtin_clz(rec.scalar_bytes);
  int64_t* const counters =
      counting ? static_cast<int64_t*>(const_cast<void*>(pv.ptrs[rec.dst_ptr_index])) : nullptr;
  const uint64_t pad = rec.pad_scalar;

  // ---- every vector of the job's four sub-tiles finds its segment ---------------------------
  // One pass over the job's segments; each is handed out once (v_readlane) and every sub-tile it
  // overlaps classifies its vectors against it.
  int mode[kJobSubTiles], my_k[kJobSubTiles], k_first[kJobSubTiles], k_last[kJobSubTiles];
  uint64_t my_src[kJobSubTiles];
#pragma unroll
  for (int t = 0; t < kJobSubTiles; ++t) {
    mode[t] = (t * kCopyThreads + lane) * kVecBytes < job_len ? kVecPending : kVecNone;
    my_k[t] = 0;
    my_src[t] = 0;
    k_first[t] = 0;
    k_last[t] = -1;
  }
  for (int k = 0; k < n_win; ++k) {
    const int32_t dl = __builtin_amdgcn_readlane(win.lo, k);
    const int32_t dh = __builtin_amdgcn_readlane(win.hi, k);
    const int32_t drh = __builtin_amdgcn_readlane(win.real_hi, k);
    const uint64_t sj = readlane_u64(win.src, k);
    const int32_t pj = __builtin_amdgcn_readlane(win.pos, k);
#pragma unroll
    for (int t = 0; t < kJobSubTiles; ++t) {
      const int32_t sub_lo = t * (kCopyThreads * kVecBytes);
      const int32_t sub_hi = sub_lo + kCopyThreads * kVecBytes < job_len
                                 ? sub_lo + kCopyThreads * kVecBytes : job_len;
      if (sub_lo >= job_len || dl >= sub_hi || dh <= sub_lo) continue;   // uniform
      const int32_t o = sub_lo + lane * kVecBytes;
      const int32_t o_end = o + kVecBytes;
      if (k_last[t] < 0) k_first[t] = k;
      k_last[t] = k;
      // the first segment this vector overlaps decides what becomes of it (selects, no branches:
      // as nested branches every case cost its own pair of exec-mask instructions)
      const bool first_hit = mode[t] == kVecPending && o < dh && o_end > dl;
      // stays pending: it needs segments the window does not hold, or the shard ends inside it
      // (one vector per shard at most): the per-lane path at the end takes it
      const bool stays = o_end > window_hi || o_end > job_len;
      const bool crosses = o < dl || o_end > dh || (!is_pos && o < drh && o_end > drh);
      const int whole = is_pos ? kVecIota : (o >= drh ? kVecPad : (per_seq ? kVecSplat : kVecCopy));
      const uint64_t from = is_pos ? (uint64_t)(uint32_t)(pj + (o >> 2))
                                   : (per_seq ? sj : sj + (uint64_t)(int64_t)o);
      mode[t] = first_hit ? (stays ? kVecPending : (crosses ? kVecSlow : whole)) : mode[t];
      my_k[t] = first_hit ? k : my_k[t];
      my_src[t] = first_hit ? from : my_src[t];
    }
  }

  // ---- all loads of plain-copy vectors ---------------------------------------------------------
  u32x4 v[kJobSubTiles];
#pragma unroll
  for (int t = 0; t < kJobSubTiles; ++t) {
    v[t] = u32x4{0, 0, 0, 0};
    if (mode[t] == kVecCopy) v[t] = load16(reinterpret_cast<const u8*>(my_src[t]));
  }

  // ---- vectors that straddle an edge: byte by byte, four vectors per round --------------------
  // There are few of them (two per segment of the job at most), so they are taken out of the
  // lanes that own them and spread over the wavefront: group g of 16 lanes moves the 16 bytes of
  // the (4*round + g)-th such vector, each lane looking up the segment of its own byte in the
  // window (rows start at scalar boundaries, so single bytes serve every scalar size; padding and
  // per-sequence values are 8-byte patterns in phase with the shard, and a job starts at a
  // multiple of 4096).  One load and one store instruction per round, whatever the scalar size.
  {
    const uint64_t m0 = __ballot(mode[0] == kVecSlow), m1 = __ballot(mode[1] == kVecSlow),
                   m2 = __ballot(mode[2] == kVecSlow), m3 = __ballot(mode[3] == kVecSlow);
    const int c0 = __builtin_popcountll(m0), c1 = c0 + __builtin_popcountll(m1),
              c2 = c1 + __builtin_popcountll(m2), n_slow = c2 + __builtin_popcountll(m3);
    for (int base = 0; base < n_slow; base += 4) {
      int32_t vec_o = -1;   // job-relative first byte of this group's vector
      int k = 0;            // window segment of its first byte
#pragma unroll
      for (int slot = 0; slot < 4; ++slot) {
        const int i = base + slot;
        if (i >= n_slow) break;
        const int t = i < c0 ? 0 : (i < c1 ? 1 : (i < c2 ? 2 : 3));
        uint64_t m = t == 0 ? m0 : (t == 1 ? m1 : (t == 2 ? m2 : m3));
        for (int q = i - (t == 0 ? 0 : (t == 1 ? c0 : (t == 2 ? c1 : c2))); q > 0; --q) m &= m - 1;
        const int owner = __builtin_ctzll(m);
        const int ks = t == 0 ? my_k[0] : (t == 1 ? my_k[1] : (t == 2 ? my_k[2] : my_k[3]));
        const int owner_k = __builtin_amdgcn_readlane(ks, owner);
        if ((lane >> 4) == slot) {
          vec_o = (t * kCopyThreads + owner) * kVecBytes;
          k = owner_k;
        }
      }
      const bool act = vec_o >= 0;
      const int32_t b = vec_o + (lane & 15);
      // the byte's segment: the vector's first one or a later one (all inside the window, or the
      // vector would have stayed pending)
      for (;;) {
        const int32_t h = __shfl(win.hi, k);
        const bool further = act && b >= h && k < kWave - 1;
        if (__ballot(further) == 0) break;
        if (further) ++k;
      }
      const int32_t g_real_hi = __shfl(win.real_hi, k);
      const uint64_t g_src = (uint64_t)__shfl((unsigned long long)win.src, k);
      const int32_t g_pos = __shfl(win.pos, k);
      const int g_mb = __shfl(seg_mb, k);
      uint32_t x = 0;
      bool real = false;
      if (act) {
        if (is_pos) {
          x = (uint32_t)(g_pos + (b >> 2)) >> (8 * (b & 3));
        } else if (b >= g_real_hi) {
          x = (uint32_t)(pad >> (8 * (b & 7)));
        } else if (per_seq) {
          x = (uint32_t)(g_src >> (8 * (b & 7)));
          real = true;
        } else {
          x = *reinterpret_cast<const u8*>(g_src + (uint64_t)(int64_t)b);
          real = true;
        }
        dst[b] = (u8)x;
      }
      if (counting) {
        // a scalar is non-zero if one of its bytes is; its first byte's lane reports it
        uint32_t nz = real && (x & 0xffu) != 0;
        if (sb_log2 >= 1) nz |= __shfl_xor(nz, 1);
        if (sb_log2 >= 2) nz |= __shfl_xor(nz, 2);
        if (sb_log2 >= 3) nz |= __shfl_xor(nz, 4);
        if (real && nz && (b & (rec.scalar_bytes - 1)) == 0) add_to_counter(counters + g_mb, 1);
      }
    }
  }

  // ---- stores ---------------------------------------------------------------------------------
#pragma unroll
  for (int t = 0; t < kJobSubTiles; ++t) {
    const int32_t o = (t * kCopyThreads + lane) * kVecBytes;
    const uint64_t ms = my_src[t];
    if (mode[t] == kVecCopy) {
      store16_sys(dst + o, v[t]);
    } else if (mode[t] == kVecSplat) {
      store16_sys(dst + o, u32x4{(uint32_t)ms, (uint32_t)(ms >> 32), (uint32_t)ms, (uint32_t)(ms >> 32)});
    } else if (mode[t] == kVecPad) {
      store16_sys(dst + o, u32x4{(uint32_t)pad, (uint32_t)(pad >> 32), (uint32_t)pad,
                                 (uint32_t)(pad >> 32)});
    } else if (mode[t] == kVecIota) {
      const uint32_t p0 = (uint32_t)ms;
      store16_sys(dst + o, u32x4{p0, p0 + 1, p0 + 2, p0 + 3});
    }
    if (counting && k_last[t] >= 0) {
      // plain-copy vectors: one sum per segment (a segment lies in one micro-batch), one atomic
      const int mine = mode[t] == kVecCopy ? count_nonzero16(v[t], sb_log2) : 0;
      for (int k = k_first[t]; k <= k_last[t]; ++k) {
        int n = mode[t] == kVecCopy && my_k[t] == k ? mine : 0;
        for (int d = kCopyThreads / 2; d > 0; d >>= 1) n += __shfl_xor(n, d);
        const int mb = __builtin_amdgcn_readlane(seg_mb, k);
        if (lane == 0) add_to_counter(counters + mb, n);
      }
    }
  }
  // vectors still pending (beyond the window, or holding the shard's last bytes): per lane
  if (__ballot(mode[0] == kVecPending || mode[1] == kVecPending || mode[2] == kVecPending ||
               mode[3] == kVecPending) != 0) {
#pragma nounroll
    for (int t = 0; t < kJobSubTiles; ++t) {
      const int mt = t == 0 ? mode[0] : (t == 1 ? mode[1] : (t == 2 ? mode[2] : mode[3]));
      if (mt == kVecPending)
        place_vector(a, pv, rec, e0, lo0 + (int64_t)(t * kCopyThreads + lane) * kVecBytes);
    }
  }
}

// earl_dispatch_async: the host built the records from buffer capacities, with the destination
// shard number in e_begin; one workgroup checks the plan's status and every capacity against the
// plan in device memory and completes the records (segment range, bytes of the shard).  If
// anything is wrong every record gets zero bytes, so the two passes that follow write nothing.
constexpr int kResolveThreads = 256;
__global__ __launch_bounds__(kResolveThreads) void async_resolve_kernel(DispatchDev* params,
                                                                        const PlanDev plan) {
  u8* base = reinterpret_cast<u8*>(params);
  const DispatchDev hd = *params;
  TileRec* recs = reinterpret_cast<TileRec*>(base + hd.recs_ofs);
  const int64_t* rec_caps = reinterpret_cast<const int64_t*>(base + hd.rec_caps_ofs);
  const int64_t* src_caps = reinterpret_cast<const int64_t*>(base + hd.src_caps_ofs);
  const int32_t* per_seq = reinterpret_cast<const int32_t*>(base + hd.src_per_sequence_ofs);
  const PlanHeader* ph = plan.hdr;
  const int tid = threadIdx.x;
  int fits = 1;
  for (int x = tid; x < hd.n_recs; x += kResolveThreads) {
    const int q = recs[x].e_begin;
    const int64_t rows = recs[x].kind == kFieldLinear ? (q == 0 ? ph->cu_seqlens_len : 0)
                                                      : plan.shard_rows[q];
    if (rows > rec_caps[x]) fits = 0;
  }
  for (int x = tid; x < hd.n_fields * plan.S; x += kResolveThreads) {
    const int f = x / plan.S, sh = x - f * plan.S;
    const int64_t need = per_seq[f] ? plan.src_seqs_needed[sh] : plan.src_rows_needed[sh];
    if (src_caps[x] >= 0 && need > src_caps[x]) fits = 0;
  }
  const int all_fit = __syncthreads_and(fits);
  const int32_t plan_status = ph->status;
  const bool go = plan_status == 0 && all_fit;
  for (int x = tid; x < hd.n_recs; x += kResolveThreads) {
    TileRec r = recs[x];
    const int q = r.e_begin;
    const int64_t rows = r.kind == kFieldLinear ? (q == 0 ? ph->cu_seqlens_len : 0)
                                                : plan.shard_rows[q];
    // a failed plan leaves no segment table behind: empty ranges, nothing is looked up
    r.e_begin = go ? plan.shard_seg_start[q] : 0;
    r.e_end = go ? plan.shard_seg_start[q + 1] : 0;
    r.end_bytes = go ? rows * (r.kind == kFieldLinear ? 4 : (int64_t)r.row_bytes) : 0;
    recs[x] = r;
  }
  if (tid == 0)
    plan.hdr->async_status = plan_status != 0 ? plan_status : (all_fit ? 0 : (int64_t)kStatusCapacity);
}

// A piece of a parameter block that travels as a kernel argument: no staging memory, no copy
// engine, nothing allocated (for the entry point that must not allocate).
struct ParamChunk {
  uint64_t words[kParamChunkBytes / 8];
};
__global__ __launch_bounds__(kWave) void param_chunk_kernel(uint64_t* dst, const ParamChunk c,
                                                            int n_words) {
  for (int x = threadIdx.x; x < n_words; x += kWave) dst[x] = c.words[x];
}

__global__ void zero_i64_kernel(int64_t* p, int64_t n) {
  const int64_t x = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (x < n) p[x] = 0;
}

// ---------------------------------------------------------------------------------------
// Reverse direction: every real row goes back to the source row it was read from.
//
// Work is cut on the stream of real rows in segment-table order: seg_real_prefix[e] rows
// precede segment e, so a tile of the stream finds its segments by search and the host only
// needs the total row count to size the grid.  Reads (destination shards) and writes (source
// shards) are both contiguous inside a segment; vectors that would cross a segment edge are
// moved scalar by scalar.  Same two passes and the same one-load-one-store-per-lane shape as
// the forward direction; the stores may be unaligned (rollout rows start anywhere).
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(kPlanThreads) void real_prefix_kernel(const SegRec* segs,
                                                                    int64_t* prefix, int n_seg) {
  // one workgroup: each thread sums a contiguous run, the runs are scanned, then written out
  __shared__ int64_t wave_tot[kPlanWaves];
  const int tid = threadIdx.x;
  const int per = (n_seg + kPlanThreads - 1) / kPlanThreads;
  const int b = (int64_t)tid * per < n_seg ? tid * per : n_seg;
  const int e = b + per < n_seg ? b + per : n_seg;
  int64_t s = 0;
#pragma unroll 8
  for (int x = b; x < e; ++x) s += segs[x].n_real;
  int64_t incl = s;
  for (int d = 1; d < kWave; d <<= 1) {
    const int64_t o = __shfl_up(incl, d);
    if ((tid & (kWave - 1)) >= d) incl += o;
  }
  if ((tid & (kWave - 1)) == kWave - 1) wave_tot[tid >> 6] = incl;
  __syncthreads();
  int64_t acc = incl - s;
  for (int wv = 0; wv < (tid >> 6); ++wv) acc += wave_tot[wv];
  for (int x = b; x < e; ++x) {
    prefix[x] = acc;
    acc += segs[x].n_real;
  }
  if (tid == kPlanThreads - 1) prefix[n_seg] = acc;
}

// Last segment of [lo, hi) whose stream prefix (in bytes) is <= byte; empty segments share a
// prefix with their successor, and taking the last one skips them.
__device__ __forceinline__ int find_stream_segment(const int64_t* prefix, int lo, int hi,
                                                   int64_t byte, int64_t w) {
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (prefix[mid] * w <= byte) lo = mid; else hi = mid;
  }
  return lo;
}

// c.segs, seg_dst_shard and seg_real_prefix describe the segments in the order the stream of
// real rows is cut in: by source position where the plan's source layout is the packed one (then
// a launch advances through the rollout buffers front to back and its WRITES are sequential, as
// the forward direction's are; with the reads sequential and the writes hopping from segment to
// segment the wide field of the largest workload measured 1.2 % slower), else the segment
// table's own order.
struct InverseArgs {
  CopyArgs c;
  const int64_t* seg_real_prefix;   // [n_seg+1]
  const int32_t* seg_dst_shard;     // [n_seg]
  int32_t n_seg;
  int32_t n_dst_shards;
};

// Copies the segment table into source order: segment (sequence i, chunk kappa) goes to entry
// i*K + kappa.  For the packed source layout with contiguous groups that is ascending (shard
// buffer, row).  i follows from the segment's source shard (its group's first sequence) and
// its sequence's rank inside the group; kappa from the position of its first row.
// In that order the real rows in front of an entry need no scan over the table: they are the
// rows of all earlier sequences (seq_pre, if the plan kernel left it) plus the sequence's own
// rows in front of the chunk, min(length, position of the chunk's first row).
__global__ __launch_bounds__(256) void source_order_kernel(const SegRec* segs,
                                                           const int32_t* seg_dst_shard,
                                                           const int32_t* seg_src_seq, SegRec* out,
                                                           int32_t* out_dst_shard, int n_seg, int N,
                                                           int G, int R, int K,
                                                           const int64_t* seq_pre,
                                                           int64_t* prefix_out) {
  const int e = blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= n_seg) return;
  const SegRec r = segs[e];
  const int64_t g = r.src_shard / R;
  const int64_t first = (g * N + G - 1) / G;
  const int64_t i = first + seg_src_seq[e];
  const int kappa = r.pos0 / r.n_rows;
  out[i * K + kappa] = r;
  out_dst_shard[i * K + kappa] = seg_dst_shard[e];
  if (seq_pre) {
    const int64_t before = seq_pre[i], length = seq_pre[i + 1] - before;
    prefix_out[i * K + kappa] = before + (r.pos0 < length ? r.pos0 : length);
    if (e == 0) prefix_out[n_seg] = seq_pre[N];
  }
}

// Inverse tile codes: a = training-layout pointer of the tile's first byte (0 = generic tile,
// then b = record << 32 | first segment), b = rollout-layout pointer (any alignment).
// Organised like tile_code_kernel: the wavefront's first tile is searched with uniform values,
// every lane writes kTilesPerLane consecutive codes and carries its segment along.
__device__ __forceinline__ void inverse_codes_of_lane(const InverseArgs& a, const int64_t first,
                                                      TileCode* out) {
  const ParamView pv = view_params(a.c.params);
  const int64_t tile0 = ((int64_t)__builtin_amdgcn_readfirstlane((int)(first >> 32)) << 32) |
                        (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)first);
  const int x0 = last_le(pv.tile_start, 0, pv.n_recs, tile0);   // one record per field
  const TileRec rec0 = pv.recs[x0];
  const int e_guess = find_stream_segment(a.seg_real_prefix, 0, a.n_seg,
                                          (tile0 - rec0.tile_first) << rec0.tile_shift,
                                          rec0.row_bytes);
  int x = first < pv.tile_start[x0 + 1] ? x0 : last_le(pv.tile_start, x0, pv.n_recs, first);
  TileRec rec = pv.recs[x];
  int64_t x_end = pv.tile_start[x + 1];
  int64_t w = rec.row_bytes;
  int64_t lo = (first - rec.tile_first) << rec.tile_shift;
  int e;
  if (x == x0 && lo < a.seg_real_prefix[e_guess + 1] * w) e = e_guess;
  else e = find_stream_segment(a.seg_real_prefix, x == x0 ? e_guess : 0, a.n_seg, lo, w);
  SegRec r = a.c.segs[e];
  int64_t s_lo = a.seg_real_prefix[e] * w;
  const int64_t last = first + kTilesPerLane < a.c.n_tiles ? first + kTilesPerLane : a.c.n_tiles;
  for (int64_t tile = first; tile < last; ++tile) {
    if (tile != first) {
      bool moved = false;
      if (tile >= x_end) {
        x = last_le(pv.tile_start, x, pv.n_recs, tile);
        rec = pv.recs[x];
        x_end = pv.tile_start[x + 1];
        w = rec.row_bytes;
        e = 0;
        moved = true;
      }
      lo = (tile - rec.tile_first) << rec.tile_shift;
      if (moved || lo >= s_lo + (int64_t)r.n_real * w) {
        e = find_stream_segment(a.seg_real_prefix, e, a.n_seg, lo, w);
        r = a.c.segs[e];
        s_lo = a.seg_real_prefix[e] * w;
      }
    }
    const int64_t tile_bytes = (int64_t)1 << rec.tile_shift;
    TileCode c;
    c.a = 0;
    c.b = (uint64_t)(uint32_t)x << 32 | (uint32_t)e;
    if (lo + tile_bytes <= s_lo + (int64_t)r.n_real * w) {
      c.a = reinterpret_cast<uint64_t>(
          static_cast<const u8*>(pv.ptrs[rec.dst_ptr_index + a.seg_dst_shard[e]]) + r.dst_row * w +
          (lo - s_lo));
      c.b = reinterpret_cast<uint64_t>(
          static_cast<const u8*>(pv.ptrs[rec.src_ptr_index + r.src_shard]) + r.src_row * w +
          (lo - s_lo));
    }
    out[tile - first] = c;
  }
}

__global__ __launch_bounds__(kCodeThreads) void inverse_code_kernel(const InverseArgs a,
                                                                   TileCode* codes) {
  // codes leave through LDS as whole rows of the wavefront's 256 codes, as in tile_code_kernel
  __shared__ TileCode s_codes[kCodeThreads / kWave][kWave * kTilesPerLane];
  const int lane = threadIdx.x & (kWave - 1);
  TileCode* mine = s_codes[threadIdx.x / kWave];
  const int64_t wave_first =
      ((int64_t)blockIdx.x * kCodeThreads + (threadIdx.x - lane)) * kTilesPerLane;
  if (wave_first >= a.c.n_tiles) return;   // uniform per wavefront
  const int64_t first = wave_first + (int64_t)lane * kTilesPerLane;
  if (first < a.c.n_tiles) inverse_codes_of_lane(a, first, mine + lane * kTilesPerLane);
  wave_exchange_fence();
#pragma unroll
  for (int j = 0; j < kTilesPerLane; ++j) {
    const int64_t tile = wave_first + j * kWave + lane;
    if (tile < a.c.n_tiles) codes[tile] = mine[j * kWave + lane];
  }
}

// The 16-byte piece at byte o of the record's stream of real rows, moved by its lane alone: one
// load and one (possibly unaligned) store when it lies in one segment, scalar by scalar when it
// crosses into the next.  e: a segment that starts at or before stream byte o.
__device__ __forceinline__ void inverse_place_vector(const InverseArgs& a, const ParamView& pv,
                                                     const TileRec& rec, int e, const int64_t o) {
  const int64_t w = rec.row_bytes;
  const int sb = rec.scalar_bytes;
  const int64_t total = rec.end_bytes;   // bytes of the real-row stream of this field
  if (o >= total) return;
  const void* const* src_ptrs = pv.ptrs + rec.src_ptr_index;
  const void* const* dst_ptrs = pv.ptrs + rec.dst_ptr_index;
  int64_t s_lo = 0, s_hi = 0;     // stream byte range of the cached segment
  const u8* from = nullptr;       // training-layout byte of stream byte s_lo
  u8* to = nullptr;               // rollout-layout byte of stream byte s_lo
  auto load_seg = [&]() {
    const SegRec r = a.c.segs[e];
    s_lo = a.seg_real_prefix[e] * w;
    s_hi = s_lo + (int64_t)r.n_real * w;
    from = static_cast<const u8*>(dst_ptrs[a.seg_dst_shard[e]]) + r.dst_row * w;
    to = static_cast<u8*>(const_cast<void*>(src_ptrs[r.src_shard])) + r.src_row * w;
  };
  auto seek_stream = [&](int64_t b) {
    if (b < s_hi) return;
    e = find_stream_segment(a.seg_real_prefix, e, a.n_seg, b, w);
    load_seg();
  };
  load_seg();
  seek_stream(o);
  if (o + kVecBytes <= s_hi) {
    store16_any(to + (o - s_lo), load16(from + (o - s_lo)));
  } else {
    for (int64_t b = o; b < o + kVecBytes && b < total; b += sb) {
      seek_stream(b);
      store_scalar(to + (b - s_lo), load_scalar(from + (b - s_lo), sb), sb);
    }
  }
}

__device__ __forceinline__ void generic_inverse_tile(const InverseArgs a, const TileCode c,
                                                  const int64_t tile, const uint32_t vec0) {
  const ParamView pv = view_params(a.c.params);
  const TileRec rec = pv.recs[(uint32_t)(c.b >> 32)];
  const int64_t lo = (tile - rec.tile_first) << rec.tile_shift;
  inverse_place_vector(a, pv, rec, (int)(uint32_t)c.b,
                       lo + (int64_t)(vec0 + threadIdx.x) * kVecBytes);
}

// The reverse direction decoded inside the copy kernel (narrow fields, small launches), built like
// relayout_direct_kernel: a wavefront owns 4 KiB of one field's stream of real rows, finds record
// and first segment with 64-way probes, keeps the job's segments one per lane (their stream byte
// range and the addresses of the job's first byte in the training and in the rollout layout),
// lets every lane pick the segment of each of its four vectors, issues all loads, and moves the
// pieces that cross a segment edge byte by byte, four pieces per round.
__global__ __launch_bounds__(kCopyThreads, 8) void inverse_direct_kernel(const InverseArgs a) {
  ParamView pv;
  pv.tile_start = a.c.direct_tile_start;
  pv.recs = a.c.direct_recs;
  pv.ptrs = a.c.ptrs;
  pv.n_recs = a.c.n_direct;
  const int lane = threadIdx.x;
  const int64_t job = blockIdx.x;
  const TileRec rec = a.c.n_direct_jobs > 2048 ? record_of_job_light(pv, job) : record_of_job(pv, job);
  const int64_t lo0 = (job - rec.tile_first) << rec.tile_shift;   // first stream byte of the job
  if (lo0 >= rec.end_bytes) return;
  const int32_t job_bytes = 1 << rec.tile_shift;   // 4 KiB, or the host's smaller choice
  const int32_t job_len = rec.end_bytes - lo0 < job_bytes ? (int32_t)(rec.end_bytes - lo0) : job_bytes;
  const int64_t w = rec.row_bytes;
  // the field's buffers in both layouts, one pointer per lane where there are at most 64
  const bool src_in_lanes = a.c.n_src_shards <= kWave, dst_in_lanes = a.n_dst_shards <= kWave;
  uint64_t lane_src = 0, lane_dst = 0;
  if (src_in_lanes && lane < a.c.n_src_shards)
    lane_src = reinterpret_cast<uint64_t>(pv.ptrs[rec.src_ptr_index + lane]);
  if (dst_in_lanes && lane < a.n_dst_shards)
    lane_dst = reinterpret_cast<uint64_t>(pv.ptrs[rec.dst_ptr_index + lane]);

  // the last segment whose stream prefix is at or before the job's first byte (empty segments
  // share their prefix with their successor, and the last one is taken)
  int first = 0;
  {
    int end = a.n_seg;
    while (end - first > 8) {
      const int step = (end - first + kWave - 1) >> 6;
      const int idx = first + lane * step;
      const bool ok = idx < end && a.seg_real_prefix[idx] * w <= lo0;
      first += (__builtin_popcountll(__ballot(ok)) - 1) * step;
      end = end < first + step ? end : first + step;
    }
  }
  const int idx = first + lane;
  const bool fetched = idx < a.n_seg;
  SegRec r = {};
  int64_t s_lo = 0;
  int32_t dshard = 0;
  if (fetched) {
    r = a.c.segs[idx];
    s_lo = a.seg_real_prefix[idx] * w;
    dshard = a.seg_dst_shard[idx];
  }
  const int shift = __builtin_popcountll(__ballot(fetched && s_lo <= lo0)) - 1;
  const int e0 = first + shift;
  int32_t win_lo = kFar, win_hi = kFar;   // the segment's real rows in the stream, relative to the job
  uint64_t win_from = 0, win_to = 0;      // training / rollout address of the job's byte 0
  {
    uint64_t src_ptr = (uint64_t)__shfl((unsigned long long)lane_src, r.src_shard);
    uint64_t dst_ptr = (uint64_t)__shfl((unsigned long long)lane_dst, dshard);
    if (fetched) {
      win_lo = clamp_far(s_lo - lo0);
      win_hi = clamp_far(s_lo + (int64_t)r.n_real * w - lo0);
      if (r.n_real > 0) {
        if (!src_in_lanes) src_ptr = reinterpret_cast<uint64_t>(pv.ptrs[rec.src_ptr_index + r.src_shard]);
        if (!dst_in_lanes) dst_ptr = reinterpret_cast<uint64_t>(pv.ptrs[rec.dst_ptr_index + dshard]);
        win_from = dst_ptr + (uint64_t)(r.dst_row * w + (lo0 - s_lo));
        win_to = src_ptr + (uint64_t)(r.src_row * w + (lo0 - s_lo));
      }
    }
  }
  {
    // move the window down so that lane k holds segment e0 + k
    const int from_lane = lane + shift;
    const bool in = from_lane < kWave;
    const int32_t lo_ = __shfl(win_lo, from_lane), hi_ = __shfl(win_hi, from_lane);
    const uint64_t f_ = (uint64_t)__shfl((unsigned long long)win_from, from_lane);
    const uint64_t t_ = (uint64_t)__shfl((unsigned long long)win_to, from_lane);
    win_lo = in ? lo_ : kFar;
    win_hi = in ? hi_ : kFar;
    win_from = f_;
    win_to = t_;
  }
  const int window_lanes = kWave - shift;
  const int n_win = __builtin_popcountll(__ballot(win_lo < job_len));
  const bool window_complete = n_win < window_lanes || e0 + window_lanes >= a.n_seg;
  const int32_t window_hi =
      window_complete ? kFar : __builtin_amdgcn_readlane(win_hi, window_lanes - 1);

  int mode[kJobSubTiles], my_k[kJobSubTiles];
  uint64_t my_from[kJobSubTiles], my_to[kJobSubTiles];
  int k0 = 0;
#pragma unroll
  for (int t = 0; t < kJobSubTiles; ++t) {
    const int32_t sub_lo = t * (kCopyThreads * kVecBytes);
    const int32_t sub_hi = sub_lo + kCopyThreads * kVecBytes < job_len
                               ? sub_lo + kCopyThreads * kVecBytes : job_len;
    const int32_t o = sub_lo + lane * kVecBytes;
    const int32_t o_end = o + kVecBytes;
    mode[t] = o < job_len ? kVecPending : kVecNone;
    my_k[t] = 0;
    my_from[t] = my_to[t] = 0;
    if (sub_lo >= job_len) continue;
    for (int k = k0; k < n_win; ++k) {
      const int32_t dl = __builtin_amdgcn_readlane(win_lo, k);
      if (dl >= sub_hi) break;
      const int32_t dh = __builtin_amdgcn_readlane(win_hi, k);
      if (dh <= sub_lo) { k0 = k + 1; continue; }
      const uint64_t fj = readlane_u64(win_from, k), tj = readlane_u64(win_to, k);
      if (mode[t] == kVecPending && o < dh && o_end > dl) {
        my_k[t] = k;
        if (o_end > window_hi || o_end > job_len) {
          // stays pending: beyond the window, or the stream ends inside it
        } else if (o < dl || o_end > dh) {
          mode[t] = kVecSlow;
        } else {
          mode[t] = kVecCopy;
          my_from[t] = fj + (uint64_t)(int64_t)o;
          my_to[t] = tj + (uint64_t)(int64_t)o;
        }
      }
    }
  }
  u32x4 v[kJobSubTiles];
#pragma unroll
  for (int t = 0; t < kJobSubTiles; ++t) {
    v[t] = u32x4{0, 0, 0, 0};
    if (mode[t] == kVecCopy) v[t] = load16(reinterpret_cast<const u8*>(my_from[t]));
  }
  {
    // pieces that cross a segment edge: group g of 16 lanes moves the 16 bytes of the
    // (4*round + g)-th of them, each lane looking up its own byte's segment in the window
    const uint64_t m0 = __ballot(mode[0] == kVecSlow), m1 = __ballot(mode[1] == kVecSlow),
                   m2 = __ballot(mode[2] == kVecSlow), m3 = __ballot(mode[3] == kVecSlow);
    const int c0 = __builtin_popcountll(m0), c1 = c0 + __builtin_popcountll(m1),
              c2 = c1 + __builtin_popcountll(m2), n_slow = c2 + __builtin_popcountll(m3);
    for (int base = 0; base < n_slow; base += 4) {
      int32_t vec_o = -1;
      int k = 0;
#pragma unroll
      for (int slot = 0; slot < 4; ++slot) {
        const int i = base + slot;
        if (i >= n_slow) break;
        const int t = i < c0 ? 0 : (i < c1 ? 1 : (i < c2 ? 2 : 3));
        uint64_t m = t == 0 ? m0 : (t == 1 ? m1 : (t == 2 ? m2 : m3));
        for (int q = i - (t == 0 ? 0 : (t == 1 ? c0 : (t == 2 ? c1 : c2))); q > 0; --q) m &= m - 1;
        const int owner = __builtin_ctzll(m);
        const int ks = t == 0 ? my_k[0] : (t == 1 ? my_k[1] : (t == 2 ? my_k[2] : my_k[3]));
        const int owner_k = __builtin_amdgcn_readlane(ks, owner);
        if ((lane >> 4) == slot) {
          vec_o = (t * kCopyThreads + owner) * kVecBytes;
          k = owner_k;
        }
      }
      const bool act = vec_o >= 0;
      const int32_t b = vec_o + (lane & 15);
      for (;;) {
        const int32_t h = __shfl(win_hi, k);
        const bool further = act && b >= h && k < kWave - 1;
        if (__ballot(further) == 0) break;
        if (further) ++k;
      }
      const uint64_t g_from = (uint64_t)__shfl((unsigned long long)win_from, k);
      const uint64_t g_to = (uint64_t)__shfl((unsigned long long)win_to, k);
      if (act)
        *reinterpret_cast<u8*>(g_to + (uint64_t)(int64_t)b) =
            *reinterpret_cast<const u8*>(g_from + (uint64_t)(int64_t)b);
    }
  }
#pragma unroll
  for (int t = 0; t < kJobSubTiles; ++t)
    if (mode[t] == kVecCopy) store16_any(reinterpret_cast<u8*>(my_to[t]), v[t]);
  if (__ballot(mode[0] == kVecPending || mode[1] == kVecPending || mode[2] == kVecPending ||
               mode[3] == kVecPending) != 0) {
#pragma nounroll
    for (int t = 0; t < kJobSubTiles; ++t) {
      const int mt = t == 0 ? mode[0] : (t == 1 ? mode[1] : (t == 2 ? mode[2] : mode[3]));
      if (mt == kVecPending)
        inverse_place_vector(a, pv, rec, e0, lo0 + (int64_t)(t * kCopyThreads + lane) * kVecBytes);
    }
  }
}

__global__ __launch_bounds__(kCopyThreads, 8) void inverse_kernel(const InverseArgs a,
                                                               const TileCode* __restrict__ codes) {
  // as in the forward kernel: kSubTiles workgroups per 4 KiB tile code
  const int64_t tile = blockIdx.x / kSubTiles;
  const uint32_t vec0 = (uint32_t)(blockIdx.x % kSubTiles) * kCopyThreads;
  const TileCode c = codes[tile];
  if (c.a != 0) {
    const uint32_t v = vec0 + threadIdx.x;
    store16_sys(reinterpret_cast<u8*>(c.b) + v * kVecBytes,
                load16(reinterpret_cast<const u8*>(c.a) + v * kVecBytes));
  } else {
    generic_inverse_tile(a, c, tile, vec0);
  }
}

}  // namespace

void launch_tile_codes(const CopyArgs& a, void* tile_codes, hipStream_t stream) {
  if (a.n_tiles <= 0) return;
  const int64_t per_group = (int64_t)kCodeThreads * kTilesPerLane;
  const unsigned grid = (unsigned)((a.n_tiles + per_group - 1) / per_group);
  hipLaunchKernelGGL(tile_code_kernel, dim3(grid), dim3(kCodeThreads), 0, stream, a,
                     static_cast<TileCode*>(tile_codes));
}

void launch_copy(const CopyArgs& a, const void* tile_codes, hipStream_t stream) {
  if (a.n_tiles <= 0) return;
  const int64_t grid = a.n_tiles * kSubTiles;
  hipLaunchKernelGGL(relayout_kernel, dim3((unsigned)grid), dim3(kCopyThreads), 0, stream, a,
                     static_cast<const TileCode*>(tile_codes));
}

void launch_direct(const CopyArgs& a, hipStream_t stream) {
  if (a.n_direct_jobs <= 0) return;
  hipLaunchKernelGGL(relayout_direct_kernel, dim3((unsigned)a.n_direct_jobs), dim3(kCopyThreads), 0,
                     stream, a);
}

void launch_zero_counters(int64_t* counters, int64_t n, hipStream_t stream) {
  if (n <= 0) return;
  hipLaunchKernelGGL(zero_i64_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream,
                     counters, n);
}

void launch_param_chunks(void* dev_dst, const unsigned char* host_block, size_t bytes,
                         hipStream_t stream) {
  // bytes is a multiple of 8 (every part of a parameter block is 256-byte aligned)
  for (size_t off = 0; off < bytes; off += kParamChunkBytes) {
    const size_t n = bytes - off < (size_t)kParamChunkBytes ? bytes - off : (size_t)kParamChunkBytes;
    ParamChunk c;
    std::memcpy(c.words, host_block + off, n);
    hipLaunchKernelGGL(param_chunk_kernel, dim3(1), dim3(kWave), 0, stream,
                       reinterpret_cast<uint64_t*>(static_cast<unsigned char*>(dev_dst) + off), c,
                       (int)(n / 8));
  }
}

void launch_async_resolve(DispatchDev* params, const PlanDev& plan, hipStream_t stream) {
  hipLaunchKernelGGL(async_resolve_kernel, dim3(1), dim3(kResolveThreads), 0, stream, params, plan);
}

void launch_real_prefix(const SegRec* segs, int64_t* prefix, int n_seg, hipStream_t stream) {
  hipLaunchKernelGGL(real_prefix_kernel, dim3(1), dim3(kPlanThreads), 0, stream, segs, prefix, n_seg);
}

void launch_source_order(const SegRec* segs, const int32_t* seg_dst_shard,
                         const int32_t* seg_src_seq, SegRec* out, int32_t* out_dst_shard, int n_seg,
                         int N, int G, int R, int K, const int64_t* seq_pre, int64_t* prefix_out,
                         hipStream_t stream) {
  if (n_seg <= 0) return;
  hipLaunchKernelGGL(source_order_kernel, dim3((unsigned)((n_seg + 255) / 256)), dim3(256), 0, stream,
                     segs, seg_dst_shard, seg_src_seq, out, out_dst_shard, n_seg, N, G, R, K, seq_pre,
                     prefix_out);
}

void launch_copy_inverse(const CopyArgs& a, const int64_t* seg_real_prefix,
                         const int32_t* seg_dst_shard, int n_seg, int n_dst_shards,
                         void* tile_codes, hipEvent_t before, hipEvent_t after,
                         hipStream_t stream) {
  InverseArgs ia{a, seg_real_prefix, seg_dst_shard, n_seg, n_dst_shards};
  if (before) (void)hipEventRecord(before, stream);
  if (a.n_direct_jobs > 0)
    hipLaunchKernelGGL(inverse_direct_kernel, dim3((unsigned)a.n_direct_jobs), dim3(kCopyThreads), 0,
                       stream, ia);
  if (a.n_tiles > 0) {
    TileCode* codes = static_cast<TileCode*>(tile_codes);
    const int64_t per_group = (int64_t)kCodeThreads * kTilesPerLane;
    const unsigned g1 = (unsigned)((a.n_tiles + per_group - 1) / per_group);
    hipLaunchKernelGGL(inverse_code_kernel, dim3(g1), dim3(kCodeThreads), 0, stream, ia, codes);
    hipLaunchKernelGGL(inverse_kernel, dim3((unsigned)(a.n_tiles * kSubTiles)), dim3(kCopyThreads), 0,
                       stream, ia, codes);
  }
  if (after) (void)hipEventRecord(after, stream);
}

}  // namespace earl
