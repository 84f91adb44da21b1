// Multi-field ragged re-layout for gfx950: materialises every destination shard of every field.
//
// This is where the bytes of the paper's dispatch move (Section 2, "Data Dispatcher": data goes
// straight from the buffers it was computed into, to the layout the consumer needs; Section 1:
// the volume of these batches is the bottleneck).  The path is pure data movement, so it is
// bound by HBM bandwidth and is built around that:
//   * work is cut on the DESTINATION: a workgroup owns 64 KiB of one destination shard of one
//     field, every lane owns whole 16-byte destination vectors, so all stores are aligned
//     global_store_dwordx4 and no two workgroups ever touch the same cache line;
//   * a vector that lies inside the real part of one segment is one (possibly unaligned)
//     global_load_dwordx4 from the source shard; padding vectors are stored without any load;
//     only vectors that straddle a segment edge fall back to scalar-sized copies;
//   * loads and stores carry the non-temporal hint (the data is touched once), and four
//     vectors per lane are in flight before the first store;
//   * position ids and cu_seqlens are further "fields" of the same launch.
#include "earl_internal.h"

namespace earl {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef u32x4 u32x4_u __attribute__((aligned(1)));
typedef unsigned char u8;

constexpr int kUnroll = 4;   // 16-byte vectors in flight per lane

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

// Last index x in [lo, hi) with key[x] <= v (key ascending, key[lo] <= v).
template <class Tk>
__device__ __forceinline__ int last_le(const Tk* key, int lo, int hi, Tk v) {
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (key[mid] <= v) lo = mid; else hi = mid;
  }
  return lo;
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
  const void* const* src_ptrs;   // this field's S source shard pointers
  int64_t w;                     // row bytes
  int e_begin, e_end;            // segments of this destination shard
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

// Moves the cursor to the segment that holds destination byte o (o only grows per lane).
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

__global__ __launch_bounds__(kCopyThreads) void relayout_kernel(const CopyArgs a) {
  const u8* params = reinterpret_cast<const u8*>(a.params);
  const DispatchDev hd = *a.params;
  const FieldDev* fields = reinterpret_cast<const FieldDev*>(params + hd.fields_ofs);
  const int64_t* tile_start = reinterpret_cast<const int64_t*>(params + hd.tile_start_ofs);
  const void* const* ptrs = reinterpret_cast<const void* const*>(params + hd.ptrs_ofs);

  const int64_t tile = blockIdx.x;
  const int x = last_le<int64_t>(tile_start, 0, hd.n_fields * hd.n_dst, tile);
  const int f = x / hd.n_dst;
  const int q = x - f * hd.n_dst;
  const FieldDev fd = fields[f];
  const int64_t w = fd.row_bytes;
  u8* dst = static_cast<u8*>(const_cast<void*>(ptrs[fd.dst_ptr_index + q]));
  const int64_t lo = (tile - tile_start[x]) * (int64_t)kTileBytes;
  const int tid = threadIdx.x;

  if (fd.kind == kFieldLinear) {
    // a flat copy (cu_seqlens): shard 0 only, linear_bytes long
    const u8* src = static_cast<const u8*>(ptrs[fd.src_ptr_index]);
    const int64_t end = (int64_t)fd.pad_scalar;
    const int64_t hi = lo + kTileBytes < end ? lo + kTileBytes : end;
    for (int64_t o = lo + (int64_t)tid * kVecBytes; o < hi; o += (int64_t)kCopyThreads * kVecBytes) {
      if (o + kVecBytes <= hi) {
        store16(dst + o, load16(src + o));
      } else {
        for (int64_t b = o; b < hi; b += 4)
          *reinterpret_cast<uint32_t*>(dst + b) = *reinterpret_cast<const uint32_t*>(src + b);
      }
    }
    return;
  }

  const int64_t end = a.shard_rows[q] * w;   // bytes of this destination shard
  const int64_t hi = lo + kTileBytes < end ? lo + kTileBytes : end;

  TileCtx t;
  t.a = &a;
  t.src_ptrs = fd.kind == kFieldCopy ? ptrs + fd.src_ptr_index : nullptr;
  t.w = w;
  t.e_begin = a.shard_seg_start[q];
  t.e_end = a.shard_seg_start[q + 1];

  SegCursor sc;
  load_segment(t, last_le<int64_t>(a.seg_dst_row, t.e_begin, t.e_end, lo / w), sc);

  u32x4 pad;
  {
    const uint32_t p_lo = (uint32_t)fd.pad_scalar, p_hi = (uint32_t)(fd.pad_scalar >> 32);
    pad = u32x4{p_lo, p_hi, p_lo, p_hi};
  }
  const bool is_pos = fd.kind == kFieldPositionIds;

  constexpr int64_t kStep = (int64_t)kCopyThreads * kVecBytes;
  for (int64_t base = lo + (int64_t)tid * kVecBytes; base < hi; base += kUnroll * kStep) {
    u32x4 v[kUnroll];
    bool full[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const int64_t o = base + u * kStep;
      full[u] = false;
      if (o >= hi) continue;
      seek(t, o, sc);
      const int64_t o_end = o + kVecBytes;
      if (is_pos) {
        if (o_end <= sc.hi) {
          const uint32_t p0 = (uint32_t)(sc.pos0 + (int32_t)(o / 4 - sc.dst_row));
          v[u] = u32x4{p0, p0 + 1, p0 + 2, p0 + 3};
          full[u] = true;
        }
      } else if (o_end <= sc.real_hi) {
        v[u] = load16(sc.src + (o - sc.lo));
        full[u] = true;
      } else if (o >= sc.real_hi && o_end <= sc.hi) {
        v[u] = pad;
        full[u] = true;
      }
      if (!full[u]) slow_vector(t, fd, dst, o, hi, sc);
    }
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      if (full[u]) store16(dst + base + u * kStep, v[u]);
    }
  }
}

// ---------------------------------------------------------------------------------------
// Reverse direction: every real row goes back to the source row it was read from.
//
// Work is cut on the stream of real rows in segment-table order: seg_real_prefix[e] rows
// precede segment e, so a tile of the stream finds its segments by binary search and the host
// only needs the total row count to size the grid.  Reads (destination shards) and writes
// (source shards) are both contiguous inside a segment; vectors that would cross a segment
// edge are moved scalar by scalar.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(kPlanThreads) void real_prefix_kernel(const int32_t* seg_n_real,
                                                                    int64_t* prefix, int n_seg) {
  // one workgroup: each thread sums a contiguous run, the runs are scanned, then written out
  __shared__ int64_t wave_tot[kPlanWaves];
  const int tid = threadIdx.x;
  const int per = (n_seg + kPlanThreads - 1) / kPlanThreads;
  const int b = tid * per < n_seg ? tid * per : n_seg;
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

__global__ __launch_bounds__(kCopyThreads) void inverse_kernel(const CopyArgs a,
                                                               const int64_t* seg_real_prefix,
                                                               const int32_t* seg_dst_shard,
                                                               int n_seg) {
  const u8* params = reinterpret_cast<const u8*>(a.params);
  const DispatchDev hd = *a.params;
  const FieldDev* fields = reinterpret_cast<const FieldDev*>(params + hd.fields_ofs);
  const int64_t* tile_start = reinterpret_cast<const int64_t*>(params + hd.tile_start_ofs);
  const void* const* ptrs = reinterpret_cast<const void* const*>(params + hd.ptrs_ofs);

  // tile_start here has one entry per field (n_dst == 1 in the block)
  const int64_t tile = blockIdx.x;
  const int f = last_le<int64_t>(tile_start, 0, hd.n_fields, tile);
  const FieldDev fd = fields[f];
  const int64_t w = fd.row_bytes;
  const int sb = fd.scalar_bytes;
  const int64_t total = seg_real_prefix[n_seg] * w;   // bytes of the real-row stream
  const int64_t lo = (tile - tile_start[f]) * (int64_t)kTileBytes;
  const int64_t hi = lo + kTileBytes < total ? lo + kTileBytes : total;
  const int tid = threadIdx.x;

  int e = -1;
  int64_t s_lo = 0, s_hi = 0;     // stream byte range of the cached segment
  const u8* from = nullptr;       // training-layout byte of stream byte s_lo
  u8* to = nullptr;               // rollout-layout byte of stream byte s_lo
  auto seek_stream = [&](int64_t o) {
    if (e >= 0 && o >= s_lo && o < s_hi) return;
    // last segment whose prefix <= row; empty segments share a prefix with their successor,
    // and taking the last one skips them
    e = last_le<int64_t>(seg_real_prefix, 0, n_seg, o / w);
    s_lo = seg_real_prefix[e] * w;
    s_hi = s_lo + (int64_t)a.seg_n_real[e] * w;
    from = static_cast<const u8*>(ptrs[fd.dst_ptr_index + seg_dst_shard[e]]) + a.seg_dst_row[e] * w;
    to = static_cast<u8*>(const_cast<void*>(ptrs[fd.src_ptr_index + a.seg_src_shard[e]])) +
         a.seg_src_row[e] * w;
  };

  for (int64_t o = lo + (int64_t)tid * kVecBytes; o < hi; o += (int64_t)kCopyThreads * kVecBytes) {
    seek_stream(o);
    if (o + kVecBytes <= s_hi) {
      store16_any(to + (o - s_lo), load16(from + (o - s_lo)));
    } else {
      for (int64_t b = o; b < o + kVecBytes && b < hi; b += sb) {
        seek_stream(b);
        store_scalar(to + (b - s_lo), load_scalar(from + (b - s_lo), sb), sb);
      }
    }
  }
}

}  // namespace

void launch_copy(const CopyArgs& a, hipStream_t stream) {
  if (a.n_tiles <= 0) return;
  hipLaunchKernelGGL(relayout_kernel, dim3((unsigned)a.n_tiles), dim3(kCopyThreads), 0, stream, a);
}

void launch_real_prefix(const int32_t* seg_n_real, int64_t* prefix, int n_seg, hipStream_t stream) {
  hipLaunchKernelGGL(real_prefix_kernel, dim3(1), dim3(kPlanThreads), 0, stream, seg_n_real, prefix,
                     n_seg);
}

void launch_copy_inverse(const CopyArgs& a, const int64_t* seg_real_prefix,
                         const int32_t* seg_dst_shard, int n_seg, hipStream_t stream) {
  if (a.n_tiles <= 0) return;
  hipLaunchKernelGGL(inverse_kernel, dim3((unsigned)a.n_tiles), dim3(kCopyThreads), 0, stream, a,
                     seg_real_prefix, seg_dst_shard, n_seg);
}

}  // namespace earl
