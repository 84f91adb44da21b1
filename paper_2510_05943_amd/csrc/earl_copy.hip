// Multi-field ragged re-layout for gfx950: materialises every destination shard of every field.
//
// This is where the bytes of the paper's dispatch move (Section 2, "Data Dispatcher": data goes
// straight from the buffers it was computed into, to the layout the consumer needs; Section 1:
// the volume of these batches is the bottleneck).  The path is pure data movement, bound by HBM
// bandwidth, and its shape follows what was measured on MI355X for plain copies:
//   * the chip streams fastest when every wavefront does ONE 16-byte load and ONE 16-byte store
//     per lane and then ends: stores are fire-and-forget (nothing waits for their
//     acknowledgement) and the wavefronts in flight always cover one compact, advancing window
//     of addresses.  Loops over large tiles, persistent grids and deeper unrolling all measured
//     15-30 % slower.  So a wavefront owns exactly 1 KiB of one destination shard of one field;
//   * work is cut on the DESTINATION, every lane owns one whole 16-byte destination vector:
//     stores are aligned global_store_dwordx4 and no two wavefronts share a cache line;
//   * a vector inside the real part of a segment is one (possibly unaligned)
//     global_load_dwordx4 from the source shard; padding vectors are stored without a load;
//     vectors that straddle a segment edge are moved scalar by scalar;
//   * loads and stores carry the non-temporal hint: every byte is touched once;
//   * finding (field, shard, segment) for a wavefront is done by the 64 lanes together
//     (each lane probes one table entry, a ballot counts the hits), so the dependent chain is a
//     handful of cache-resident loads, which the measurements show to be free at this occupancy;
//   * position ids and cu_seqlens are further "fields" of the same launch.
#include "earl_internal.h"

namespace earl {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef u32x4 u32x4_u __attribute__((aligned(1)));
typedef unsigned char u8;

__device__ __forceinline__ u32x4 load16(const u8* p) {
  return __builtin_nontemporal_load(reinterpret_cast<const u32x4_u*>(p));
}
__device__ __forceinline__ void store16(u8* p, u32x4 v) {
  __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(p));
}
__device__ __forceinline__ void store16_any(u8* p, u32x4 v) {
  __builtin_nontemporal_store(v, reinterpret_cast<u32x4_u*>(p));
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

// Last index x in [lo, hi) with key[x] <= v (key ascending, key[lo] <= v); one lane on its own.
template <class Tk>
__device__ __forceinline__ int last_le(const Tk* key, int lo, int hi, Tk v) {
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (key[mid] <= v) lo = mid; else hi = mid;
  }
  return lo;
}

// The same search done by the 64 lanes of a wavefront together (v is wavefront-uniform): every
// round each lane probes one of 64 evenly spaced entries and a ballot narrows the range 64-fold.
__device__ __forceinline__ int wave_last_le(const int64_t* key, int lo, int hi, int64_t v, int lane) {
  int len = hi - lo;
  while (len > 1) {
    const int stride = (len + kWave - 1) / kWave;
    const int idx = lo + lane * stride;
    const bool hit = idx < lo + len && key[idx] <= v;
    const int cnt = __builtin_popcountll(__ballot(hit));   // >= 1: key[lo] <= v
    const int nlo = lo + (cnt - 1) * stride;
    len = (lo + len - nlo) < stride ? (lo + len - nlo) : stride;
    lo = nlo;
  }
  return lo;
}

// Number of entries of the ascending table t[0..n) that are <= v, n <= 256, counted by the
// wavefront: lane l looks at entries 4l..4l+3.
__device__ __forceinline__ int wave_count_le_256(const int64_t* t, int n, int64_t v, int lane) {
  int c = 0;
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const int idx = 4 * lane + k;
    if (idx < n && t[idx] <= v) ++c;
  }
  return __builtin_popcountll(__ballot(c >= 1)) + __builtin_popcountll(__ballot(c >= 2)) +
         __builtin_popcountll(__ballot(c >= 3)) + __builtin_popcountll(__ballot(c >= 4));
}

// The segment a lane is currently copying from, as destination byte ranges of its shard.
struct SegCursor {
  int64_t lo, real_hi, hi;   // [lo, real_hi) real rows, [real_hi, hi) padding rows
  const u8* src;             // source byte that lands on destination byte lo
  int64_t dst_row;
  int32_t pos0;
  int e;
};

struct TileCtx {
  const CopyArgs* a;
  const void* const* src_ptrs;   // this field's S source shard pointers (null for position ids)
  int64_t w;                     // row bytes
  int e_end;                     // end of this destination shard's segments
};

__device__ __forceinline__ void load_segment(const TileCtx& t, int e, SegCursor& sc) {
  const CopyArgs& a = *t.a;
  const int64_t d = a.seg_dst_row[e];
  sc.e = e;
  sc.dst_row = d;
  sc.lo = d * t.w;
  sc.real_hi = (d + a.seg_n_real[e]) * t.w;
  sc.hi = (d + a.seg_n_rows[e]) * t.w;
  sc.pos0 = a.seg_pos0[e];
  sc.src = t.src_ptrs
               ? static_cast<const u8*>(t.src_ptrs[a.seg_src_shard[e]]) + a.seg_src_row[e] * t.w
               : nullptr;
}

// Moves a lane's cursor to the segment that holds destination byte o >= sc.lo.
__device__ __forceinline__ void seek(const TileCtx& t, int64_t o, SegCursor& sc) {
  if (o < sc.hi) return;
  int e = sc.e + 1;
  if (e + 1 < t.e_end && (t.a->seg_dst_row[e + 1]) * t.w <= o)
    e = last_le<int64_t>(t.a->seg_dst_row, e + 1, t.e_end, o / t.w);
  load_segment(t, e, sc);
}

// One 16-byte destination vector that is not a plain copy or a plain fill: element by element.
__device__ void slow_vector(const TileCtx& t, const FieldDev& fd, u8* dst, int64_t o, int64_t end,
                            SegCursor sc) {
  const int sb = fd.scalar_bytes;
  for (int64_t b = o; b < o + kVecBytes && b < end; b += sb) {
    seek(t, b, sc);
    if (fd.kind == kFieldPositionIds) {
      const int64_t row = b / t.w;
      store_scalar(dst + b, (uint64_t)(uint32_t)(sc.pos0 + (int32_t)(row - sc.dst_row)), 4);
    } else if (b < sc.real_hi) {
      store_scalar(dst + b, load_scalar(sc.src + (b - sc.lo), sb), sb);
    } else {
      store_scalar(dst + b, fd.pad_scalar, sb);
    }
  }
}

// One wavefront = one tile of kTileBytes destination bytes; kWaves tiles per workgroup.
template <int kWaves>
__global__ __launch_bounds__(kWaves * kWave) void relayout_kernel(const CopyArgs a) {
  const int lane = threadIdx.x & (kWave - 1);
  const int64_t tile = (int64_t)blockIdx.x * kWaves + (threadIdx.x >> 6);
  if (tile >= a.n_tiles) return;

  const u8* params = reinterpret_cast<const u8*>(a.params);
  const DispatchDev hd = *a.params;
  const FieldDev* fields = reinterpret_cast<const FieldDev*>(params + hd.fields_ofs);
  const int64_t* tile_start = reinterpret_cast<const int64_t*>(params + hd.tile_start_ofs);
  const void* const* ptrs = reinterpret_cast<const void* const*>(params + hd.ptrs_ofs);

  // (field, shard) of this tile: last entry of tile_start that is <= tile
  const int n_fq = hd.n_fields * hd.n_dst;
  const int x = n_fq <= 256 ? wave_count_le_256(tile_start, n_fq, tile, lane) - 1
                            : last_le<int64_t>(tile_start, 0, n_fq, tile);
  const int f = x / hd.n_dst;
  const int q = x - f * hd.n_dst;
  const FieldDev fd = fields[f];
  const int64_t w = fd.row_bytes;
  u8* dst = static_cast<u8*>(const_cast<void*>(ptrs[fd.dst_ptr_index + q]));
  const int64_t lo = (tile - tile_start[x]) * (int64_t)kTileBytes;
  const int64_t o = lo + (int64_t)lane * kVecBytes;   // this lane's destination vector

  if (fd.kind == kFieldLinear) {
    // a flat copy (cu_seqlens): shard 0 only, pad_scalar = bytes to copy
    const u8* src = static_cast<const u8*>(ptrs[fd.src_ptr_index]);
    const int64_t end = (int64_t)fd.pad_scalar;
    if (o + kVecBytes <= end) {
      store16(dst + o, load16(src + o));
    } else {
      for (int64_t b = o; b < end; b += 4)
        *reinterpret_cast<uint32_t*>(dst + b) = *reinterpret_cast<const uint32_t*>(src + b);
    }
    return;
  }

  const int64_t end = a.shard_rows[q] * w;   // bytes of this destination shard
  TileCtx t;
  t.a = &a;
  t.src_ptrs = fd.kind == kFieldCopy ? ptrs + fd.src_ptr_index : nullptr;
  t.w = w;
  t.e_end = a.shard_seg_start[q + 1];
  const int e0 = wave_last_le(a.seg_dst_row, a.shard_seg_start[q], t.e_end, lo / w, lane);
  if (o >= end) return;

  SegCursor sc;
  load_segment(t, e0, sc);
  seek(t, o, sc);
  const int64_t o_end = o + kVecBytes;
  if (fd.kind == kFieldPositionIds) {
    if (o_end <= sc.hi) {
      const uint32_t p0 = (uint32_t)(sc.pos0 + (int32_t)(o / 4 - sc.dst_row));
      store16(dst + o, u32x4{p0, p0 + 1, p0 + 2, p0 + 3});
      return;
    }
  } else if (o_end <= sc.real_hi) {
    store16(dst + o, load16(sc.src + (o - sc.lo)));
    return;
  } else if (o >= sc.real_hi && o_end <= sc.hi) {
    const uint32_t p_lo = (uint32_t)fd.pad_scalar, p_hi = (uint32_t)(fd.pad_scalar >> 32);
    store16(dst + o, u32x4{p_lo, p_hi, p_lo, p_hi});
    return;
  }
  slow_vector(t, fd, dst, o, end, sc);
}

// ---------------------------------------------------------------------------------------
// Reverse direction: every real row goes back to the source row it was read from.
//
// Work is cut on the stream of real rows in segment-table order: seg_real_prefix[e] rows
// precede segment e, so a tile of the stream finds its segments by search and the host only
// needs the total row count to size the grid.  Reads (destination shards) and writes (source
// shards) are both contiguous inside a segment; vectors that would cross a segment edge are
// moved scalar by scalar.  Same one-load-one-store-per-lane shape as the forward kernel.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(kPlanThreads) void real_prefix_kernel(const int32_t* seg_n_real,
                                                                    int64_t* prefix, int n_seg) {
  // one workgroup: each thread sums a contiguous run, the runs are scanned, then written out
  __shared__ int64_t wave_tot[kPlanWaves];
  const int tid = threadIdx.x;
  const int per = (n_seg + kPlanThreads - 1) / kPlanThreads;
  const int b = (int64_t)tid * per < n_seg ? tid * per : n_seg;
  const int e = b + per < n_seg ? b + per : n_seg;
  int64_t s = 0;
  for (int x = b; x < e; ++x) s += seg_n_real[x];
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
    acc += seg_n_real[x];
  }
  if (tid == kPlanThreads - 1) prefix[n_seg] = acc;
}

template <int kWaves>
__global__ __launch_bounds__(kWaves * kWave) void inverse_kernel(const CopyArgs a,
                                                                 const int64_t* seg_real_prefix,
                                                                 const int32_t* seg_dst_shard,
                                                                 int n_seg) {
  const int lane = threadIdx.x & (kWave - 1);
  const int64_t tile = (int64_t)blockIdx.x * kWaves + (threadIdx.x >> 6);
  if (tile >= a.n_tiles) return;

  const u8* params = reinterpret_cast<const u8*>(a.params);
  const DispatchDev hd = *a.params;
  const FieldDev* fields = reinterpret_cast<const FieldDev*>(params + hd.fields_ofs);
  const int64_t* tile_start = reinterpret_cast<const int64_t*>(params + hd.tile_start_ofs);
  const void* const* ptrs = reinterpret_cast<const void* const*>(params + hd.ptrs_ofs);

  // one tile_start entry per field here (at most EARL_MAX_FIELDS of them)
  const int f = wave_count_le_256(tile_start, hd.n_fields, tile, lane) - 1;
  const FieldDev fd = fields[f];
  const int64_t w = fd.row_bytes;
  const int sb = fd.scalar_bytes;
  const int64_t total = seg_real_prefix[n_seg] * w;   // bytes of the real-row stream
  const int64_t lo = (tile - tile_start[f]) * (int64_t)kTileBytes;
  const int64_t o = lo + (int64_t)lane * kVecBytes;
  // last segment whose prefix <= first row of the tile; empty segments share a prefix with
  // their successor, and taking the last one skips them
  int e = wave_last_le(seg_real_prefix, 0, n_seg, lo / w, lane);
  if (o >= total) return;

  int64_t s_lo = 0, s_hi = 0;     // stream byte range of the cached segment
  const u8* from = nullptr;       // training-layout byte of stream byte s_lo
  u8* to = nullptr;               // rollout-layout byte of stream byte s_lo
  auto load_seg = [&]() {
    s_lo = seg_real_prefix[e] * w;
    s_hi = s_lo + (int64_t)a.seg_n_real[e] * w;
    from = static_cast<const u8*>(ptrs[fd.dst_ptr_index + seg_dst_shard[e]]) + a.seg_dst_row[e] * w;
    to = static_cast<u8*>(const_cast<void*>(ptrs[fd.src_ptr_index + a.seg_src_shard[e]])) +
         a.seg_src_row[e] * w;
  };
  auto seek_stream = [&](int64_t b) {
    if (b < s_hi) return;
    e = last_le<int64_t>(seg_real_prefix, e, n_seg, b / w);
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

constexpr int kCopyWaves = kCopyThreads / kWave;

}  // namespace

void launch_copy(const CopyArgs& a, hipStream_t stream) {
  if (a.n_tiles <= 0) return;
  const unsigned grid = (unsigned)((a.n_tiles + kCopyWaves - 1) / kCopyWaves);
  hipLaunchKernelGGL(relayout_kernel<kCopyWaves>, dim3(grid), dim3(kCopyThreads), 0, stream, a);
}

void launch_real_prefix(const int32_t* seg_n_real, int64_t* prefix, int n_seg, hipStream_t stream) {
  hipLaunchKernelGGL(real_prefix_kernel, dim3(1), dim3(kPlanThreads), 0, stream, seg_n_real, prefix,
                     n_seg);
}

void launch_copy_inverse(const CopyArgs& a, const int64_t* seg_real_prefix,
                         const int32_t* seg_dst_shard, int n_seg, hipStream_t stream) {
  if (a.n_tiles <= 0) return;
  const unsigned grid = (unsigned)((a.n_tiles + kCopyWaves - 1) / kCopyWaves);
  hipLaunchKernelGGL(inverse_kernel<kCopyWaves>, dim3(grid), dim3(kCopyThreads), 0, stream, a,
                     seg_real_prefix, seg_dst_shard, n_seg);
}

}  // namespace earl
