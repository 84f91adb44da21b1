// Dispatch plan on the device: one workgroup of 16 wavefronts on gfx950.
//
// The paper's Data Dispatcher (Section 2) chooses, from the current data layout and the
// consumer's parallelism configuration, where every part of every sequence has to go, so that
// it can be sent there directly.  This kernel is that decision for one batch: source row
// offsets, replica choice, padded chunk geometry, length-balanced DP-rank assignment, packing
// order, micro-batches, destination offsets, the segment table and the all-to-all counts.
// Everything is integer arithmetic with explicit tie-breaks, so the result is unique.
//
// N is a few thousand at most in practice and the longest dependency chain (the list
// scheduling of N sequences) is serial by definition, so the whole plan runs in a single
// workgroup: phases are separated by workgroup barriers, wide phases use all 1024 lanes, the
// serial chain runs in wavefront 0 with the rank loads held one per lane and the arg-min taken
// by DPP cross-lane operations.
#include <cstdlib>
#include <cstring>
#include <utility>

#include "earl_internal.h"

namespace earl {
namespace {

constexpr int T = kPlanThreads;
constexpr int kLdsA2a = 2048;   // (source shard, destination shard) pairs counted in LDS

// ---------------------------------------------------------------------------------------
// wavefront primitives
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ int lane_id() { return threadIdx.x & (kWave - 1); }
__device__ __forceinline__ int wave_id() { return threadIdx.x >> 6; }

template <int kCtrl, int kRowMask>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t old, uint32_t src) {
  return (uint32_t)__builtin_amdgcn_update_dpp((int)old, (int)src, kCtrl, kRowMask, 0xf, false);
}

// DPP controls of the GFX9 family.
constexpr int kDppQuadXor1 = 0xB1;      // quad_perm:[1,0,3,2]
constexpr int kDppQuadXor2 = 0x4E;      // quad_perm:[2,3,0,1]
constexpr int kDppRowHalfMirror = 0x141;
constexpr int kDppRowMirror = 0x140;
constexpr int kDppRowBcast15 = 0x142;
constexpr int kDppRowBcast31 = 0x143;
constexpr int kDppRowShr = 0x110;       // + n
constexpr int kDppRowShl1 = 0x101;      // row_shl:1, lane i reads lane i+1 of its row of 16
constexpr int kDppWaveShl1 = 0x130;     // wave_shl:1, the same over all 64 lanes

// Inclusive prefix sum over the 64 lanes: Hillis-Steele inside each row of 16 lanes with
// row_shr, then the row totals are carried across rows with row_bcast.
template <int kCtrl, int kRowMask>
__device__ __forceinline__ int64_t dpp_add_i64(int64_t x) {
  uint32_t lo = dpp_u32<kCtrl, kRowMask>(0u, (uint32_t)x);
  uint32_t hi = dpp_u32<kCtrl, kRowMask>(0u, (uint32_t)((uint64_t)x >> 32));
  return x + (int64_t)(((uint64_t)hi << 32) | lo);
}
__device__ __forceinline__ int64_t wave_incl_scan_i64(int64_t x) {
  x = dpp_add_i64<kDppRowShr + 1, 0xf>(x);
  x = dpp_add_i64<kDppRowShr + 2, 0xf>(x);
  x = dpp_add_i64<kDppRowShr + 4, 0xf>(x);
  x = dpp_add_i64<kDppRowShr + 8, 0xf>(x);
  x = dpp_add_i64<kDppRowBcast15, 0xa>(x);
  x = dpp_add_i64<kDppRowBcast31, 0xc>(x);
  return x;
}
__device__ __forceinline__ uint32_t wave_incl_scan_u32(uint32_t x) {
  x += dpp_u32<kDppRowShr + 1, 0xf>(0u, x);
  x += dpp_u32<kDppRowShr + 2, 0xf>(0u, x);
  x += dpp_u32<kDppRowShr + 4, 0xf>(0u, x);
  x += dpp_u32<kDppRowShr + 8, 0xf>(0u, x);
  x += dpp_u32<kDppRowBcast15, 0xa>(0u, x);
  x += dpp_u32<kDppRowBcast31, 0xc>(0u, x);
  return x;
}
// number of set bits of mask below this lane
__device__ __forceinline__ int count_below(uint64_t mask) {
  return (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32),
                                        __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}
__device__ __forceinline__ int64_t readlane_i64(int64_t x, int l) {
  uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)x, l);
  uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)((uint64_t)x >> 32), l);
  return (int64_t)(((uint64_t)hi << 32) | lo);
}

// ---------------------------------------------------------------------------------------
// workgroup primitives (every thread of the workgroup must call them)
// ---------------------------------------------------------------------------------------
struct BlockScratch {
  int64_t wave_tot[kPlanWaves];
  int64_t total;
};

// Exclusive prefix sum of one value per thread; returns the prefix, writes the total.
// n_waves: wavefronts in the workgroup.
__device__ int64_t block_excl_scan(int64_t v, BlockScratch& s, int64_t* total,
                                   int n_waves = kPlanWaves) {
  int64_t incl = wave_incl_scan_i64(v);
  if (lane_id() == kWave - 1) s.wave_tot[wave_id()] = incl;
  __syncthreads();
  if (wave_id() == 0) {
    int64_t t = lane_id() < n_waves ? s.wave_tot[lane_id()] : 0;
    int64_t ti = wave_incl_scan_i64(t);
    if (lane_id() < n_waves) s.wave_tot[lane_id()] = ti - t;
    if (lane_id() == n_waves - 1) s.total = ti;
  }
  __syncthreads();
  int64_t r = incl - v + s.wave_tot[wave_id()];
  *total = s.total;
  __syncthreads();
  return r;
}

__device__ int64_t block_reduce_max(int64_t v, BlockScratch& s) {
  for (int d = 32; d > 0; d >>= 1) {
    int64_t o = __shfl_xor(v, d);
    v = o > v ? o : v;
  }
  if (lane_id() == 0) s.wave_tot[wave_id()] = v;
  __syncthreads();
  int64_t r = s.wave_tot[0];
  for (int w = 1; w < kPlanWaves; ++w) r = s.wave_tot[w] > r ? s.wave_tot[w] : r;
  __syncthreads();
  return r;
}

__device__ int64_t block_reduce_min(int64_t v, BlockScratch& s) {
  return -block_reduce_max(-v, s);
}

// Hands the finished summary block (the first bytes of the workspace, header included) to the
// host through its mailbox, if the plan has one.  Every thread of the workgroup calls it, after
// the header has been written.  copy: the block is read back from the workspace and copied;
// false where every entry went to the mailbox as it was stored (put_summary).
__device__ void publish_summary(const PlanDev& p, bool copy = true) {
  if (!p.host_summary) return;
  if (copy) {
    __syncthreads();   // the whole block is written and visible to this workgroup
    const uint4* from = reinterpret_cast<const uint4*>(p.hdr);
    uint4* to = reinterpret_cast<uint4*>(p.host_summary);
    for (uint32_t x = threadIdx.x; x < p.summary_bytes / 16; x += blockDim.x) to[x] = from[x];
  }
  __threadfence_system();
  __syncthreads();
  if (threadIdx.x == 0)
    __hip_atomic_store(reinterpret_cast<uint64_t*>(p.host_summary + p.host_flag_offset), p.host_token,
                       __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
}

// Stores one entry of the summary block: in the workspace and, if the plan has a mailbox, at the
// same offset there.
template <class Tv>
__device__ __forceinline__ void put_summary(const PlanDev& p, Tv* where, const Tv& value) {
  *where = value;
  if (p.host_summary)
    *reinterpret_cast<Tv*>(p.host_summary + (reinterpret_cast<const unsigned char*>(where) -
                                             reinterpret_cast<const unsigned char*>(p.hdr))) = value;
}

// ---------------------------------------------------------------------------------------
// Segmented prefix scan by label, in index order.
//
// For every i in [0, N): cnt(i) = #{ j < i : lab(j) == lab(i) } and
// sum(i) = sum of val(j) over the same j.  With lab = source group and val = length this gives
// the packed source row offset of every sequence; with lab = DP rank and val = rows per SP rank
// it gives the position of a sequence inside its rank and its destination row offset.
//
// A chunk of 1024 consecutive indices is handled per step: each wavefront loops over the
// distinct labels among its 64 lanes (ballot / readlane) and scans the matching lanes; the
// per-(wavefront, label) totals are combined through a table (LDS or workspace) and a running
// carry per label.  tab_* are [2][kPlanWaves][n_labels] (contribution, prefix) followed by the
// carry [n_labels]; all zero on entry, and the carry holds the per-label totals on exit.
// ---------------------------------------------------------------------------------------
template <class LabF, class ValF, class OutF>
__device__ void label_scan(int N, int n_labels, LabF lab, ValF val, OutF out, int64_t* tab_sum,
                           int32_t* tab_cnt) {
  const int lane = lane_id(), wave = wave_id();
  const size_t plane = (size_t)kPlanWaves * n_labels;
  int64_t* tot_sum = tab_sum;
  int64_t* pre_sum = tab_sum + plane;
  int64_t* carry_sum = tab_sum + 2 * plane;
  int32_t* tot_cnt = tab_cnt;
  int32_t* pre_cnt = tab_cnt + plane;
  int32_t* carry_cnt = tab_cnt + 2 * plane;

  for (int base = 0; base < N; base += T) {
    const int i = base + (int)threadIdx.x;
    const bool active = i < N;
    const int l = active ? lab(i) : -1;
    const int64_t v = active ? val(i) : 0;
    int32_t my_cnt = 0;
    int64_t my_sum = 0;
    uint64_t remaining = __ballot(active);
    while (remaining) {
      const int leader = __builtin_ctzll(remaining);
      const int cur = __builtin_amdgcn_readlane(l, leader);
      const bool mine = active && l == cur;
      const uint64_t mask = __ballot(mine);
      const int64_t incl = wave_incl_scan_i64(mine ? v : 0);
      if (mine) {
        my_cnt = __builtin_popcountll(mask & ((1ull << lane) - 1ull));
        my_sum = incl - v;
      }
      const int64_t wtot = readlane_i64(incl, kWave - 1);
      if (lane == leader) {
        tot_sum[(size_t)wave * n_labels + cur] = wtot;
        tot_cnt[(size_t)wave * n_labels + cur] = __builtin_popcountll(mask);
      }
      remaining &= ~mask;
    }
    __syncthreads();
    for (int c = threadIdx.x; c < n_labels; c += T) {
      int64_t as = carry_sum[c];
      int32_t ac = carry_cnt[c];
      for (int w = 0; w < kPlanWaves; ++w) {
        const size_t x = (size_t)w * n_labels + c;
        const int64_t s = tot_sum[x];
        const int32_t n = tot_cnt[x];
        pre_sum[x] = as;
        pre_cnt[x] = ac;
        tot_sum[x] = 0;
        tot_cnt[x] = 0;
        as += s;
        ac += n;
      }
      carry_sum[c] = as;
      carry_cnt[c] = ac;
    }
    __syncthreads();
    if (active) {
      const size_t x = (size_t)wave * n_labels + l;
      out(i, my_cnt + pre_cnt[x], my_sum + pre_sum[x]);
    }
  }
  __syncthreads();
}

// ---------------------------------------------------------------------------------------
// Bitonic sort of n (power of two) unique 64-bit keys, ascending.
// ---------------------------------------------------------------------------------------
// Stages whose partner distance j is at most 64 only touch aligned blocks of 128 keys, and the
// 64 compare-exchanges of a block all belong to one wavefront (thread t handles block t / 64), so
// those stages need no workgroup barrier, only program order inside the wavefront.
template <class KeyPtr, bool kLds>
__device__ void bitonic_sort_impl(KeyPtr keys, int n) {
  const int nt = blockDim.x;   // a multiple of 64
  for (int k = 2; k <= n; k <<= 1) {
    for (int j = k >> 1; j > 0; j >>= 1) {
      for (int t = threadIdx.x; t < (n >> 1); t += nt) {
        const int i = ((t & ~(j - 1)) << 1) | (t & (j - 1));
        const int x = i | j;
        const uint64_t a = keys[i], b = keys[x];
        const bool up = (i & k) == 0;
        if ((a > b) == up) {
          keys[i] = b;
          keys[x] = a;
        }
      }
      if (!kLds || j > kWave || (j == 1 && k > kWave)) {
        __syncthreads();   // the next stage crosses wavefront blocks
      } else {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      }
    }
  }
  __syncthreads();
}

__device__ void bitonic_sort(uint64_t* keys, int n, bool keys_in_lds) {
  if (keys_in_lds) {
    typedef __attribute__((address_space(3))) uint64_t* LdsKeys;
    bitonic_sort_impl<LdsKeys, true>((LdsKeys)keys, n);
  } else {
    bitonic_sort_impl<uint64_t*, false>(keys, n);
  }
}

// ---------------------------------------------------------------------------------------
// The same sort with the keys of a stage's partners exchanged between LANES where they are
// fewer than 64 apart: element x is always handled by lane x & 63 of the same thread, so the
// six stages with partner distance 32 .. 1 that end every merge run in registers on cross-lane
// moves, with one LDS read before and one LDS write after them, and all stages of the merges
// up to 64 keys run in registers in one go.  Only partner distances of 64 and more go through
// LDS with a workgroup barrier per stage (10 of the 55 stages of 1024 keys).
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ uint64_t exchange_with_lane(uint64_t key, int x, int j, int k) {
  const uint64_t other = (uint64_t)__shfl_xor((unsigned long long)key, j);
  const bool keep_smaller = ((x & j) == 0) == ((x & k) == 0);   // lower partner of an ascending run
  const bool smaller = key < other;
  return smaller == keep_smaller ? key : other;
}

__device__ void bitonic_sort_lanes(uint64_t* keys_generic, int n) {
  typedef __attribute__((address_space(3))) uint64_t* LdsKeys;
  LdsKeys keys = (LdsKeys)keys_generic;
  const int nt = blockDim.x;   // a multiple of 64
  // merges of up to 64 keys: all partners inside the wavefront
  for (int x = threadIdx.x; x < n; x += nt) {
    uint64_t key = keys[x];
    for (int k = 2; k <= kWave && k <= n; k <<= 1)
      for (int j = k >> 1; j > 0; j >>= 1) key = exchange_with_lane(key, x, j, k);
    keys[x] = key;
  }
  __syncthreads();
  for (int k = 2 * kWave; k <= n; k <<= 1) {
    for (int j = k >> 1; j >= kWave; j >>= 1) {
      for (int t = threadIdx.x; t < (n >> 1); t += nt) {
        const int i = ((t & ~(j - 1)) << 1) | (t & (j - 1));
        const int y = i | j;
        const uint64_t a = keys[i], b = keys[y];
        if ((a > b) == ((i & k) == 0)) {
          keys[i] = b;
          keys[y] = a;
        }
      }
      __syncthreads();
    }
    for (int x = threadIdx.x; x < n; x += nt) {
      uint64_t key = keys[x];
#pragma unroll
      for (int j = kWave >> 1; j > 0; j >>= 1) key = exchange_with_lane(key, x, j, k);
      keys[x] = key;
    }
    __syncthreads();
  }
}

// ---------------------------------------------------------------------------------------
// The same sort for 32-bit keys.  The partner at lane distance 1, 2, 4 or 8 is inside the
// lane's row of 16 and comes through a DPP move (distance 4 has no control of its own: two
// moves, each written in the two banks of four lanes whose partner lies on that side);
// distances 16 and 32 cross rows and go through ds_bpermute.
// ---------------------------------------------------------------------------------------
constexpr int kDppRowShl4 = 0x104, kDppRowShr4 = 0x114, kDppRowRor8 = 0x128;

template <int kJ>
__device__ __forceinline__ uint32_t from_lane_xor(uint32_t v) {
  if constexpr (kJ == 1) {
    return dpp_u32<kDppQuadXor1, 0xf>(v, v);
  } else if constexpr (kJ == 2) {
    return dpp_u32<kDppQuadXor2, 0xf>(v, v);
  } else if constexpr (kJ == 4) {
    const uint32_t t =
        (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, kDppRowShl4, 0xf, 0x5, false);
    return (uint32_t)__builtin_amdgcn_update_dpp((int)t, (int)v, kDppRowShr4, 0xf, 0xa, false);
  } else if constexpr (kJ == 8) {
    return dpp_u32<kDppRowRor8, 0xf>(v, v);
  } else {
    return (uint32_t)__shfl_xor((int)v, kJ);
  }
}

// Compare-exchange stages with partner distance kJ, kJ/2, .. 1 of the merge into runs of k keys.
template <int kJ>
__device__ __forceinline__ uint32_t lane_stages(uint32_t key, int x, int k) {
  const uint32_t other = from_lane_xor<kJ>(key);
  const bool keep_smaller = ((x & kJ) == 0) == ((x & k) == 0);   // lower partner of an ascending run
  const uint32_t lo = key < other ? key : other, hi = key < other ? other : key;
  key = keep_smaller ? lo : hi;
  if constexpr (kJ > 1) key = lane_stages<kJ / 2>(key, x, k);
  return key;
}

__device__ void bitonic_sort_lanes32(uint32_t* keys_generic, int n) {
  typedef __attribute__((address_space(3))) uint32_t* LdsKeys;
  LdsKeys keys = (LdsKeys)keys_generic;
  const int nt = blockDim.x;   // a multiple of 64
  for (int x = threadIdx.x; x < n; x += nt) {
    uint32_t key = keys[x];
    if (n >= 2) key = lane_stages<1>(key, x, 2);
    if (n >= 4) key = lane_stages<2>(key, x, 4);
    if (n >= 8) key = lane_stages<4>(key, x, 8);
    if (n >= 16) key = lane_stages<8>(key, x, 16);
    if (n >= 32) key = lane_stages<16>(key, x, 32);
    if (n >= 64) key = lane_stages<32>(key, x, 64);
    keys[x] = key;
  }
  __syncthreads();
  for (int k = 2 * kWave; k <= n; k <<= 1) {
    for (int j = k >> 1; j >= kWave; j >>= 1) {
      for (int t = threadIdx.x; t < (n >> 1); t += nt) {
        const int i = ((t & ~(j - 1)) << 1) | (t & (j - 1));
        const int y = i | j;
        const uint32_t a = keys[i], b = keys[y];
        if ((a > b) == ((i & k) == 0)) {
          keys[i] = b;
          keys[y] = a;
        }
      }
      __syncthreads();
    }
    for (int x = threadIdx.x; x < n; x += nt) keys[x] = lane_stages<32>(keys[x], x, k);
    __syncthreads();
  }
}

// ---------------------------------------------------------------------------------------
// Sort keys: (padded length descending, index ascending) in one word, all ones after the last
// sequence (a padded length is at least 1, so no sequence has that key).
// ---------------------------------------------------------------------------------------
struct Key64 {   // any padded length below 2^31, any index
  typedef uint64_t Word;
  static constexpr Word kLast = ~0ull;
  static __device__ __forceinline__ Word make(int64_t lp, int i) {
    return ((uint64_t)(0x7fffffffll - lp) << 32) | (uint32_t)i;
  }
  static __device__ __forceinline__ int32_t lp(Word k) { return 0x7fffffff - (int32_t)(k >> 32); }
  static __device__ __forceinline__ int32_t index(Word k) { return (int32_t)(k & 0xffffffffu); }
};
template <int kIndexBitsT>   // indices below 2^kIndexBitsT, padded lengths below 2^(32 - kIndexBitsT)
struct Key32 {
  typedef uint32_t Word;
  static constexpr Word kLast = ~0u;
  static constexpr int kIndexBits = kIndexBitsT, kLpBits = 32 - kIndexBitsT;
  static constexpr int32_t kLpMax = (int32_t)((1u << kLpBits) - 1u);
  static __device__ __forceinline__ Word make(int64_t lp, int i) {
    return ((uint32_t)(kLpMax - (int32_t)lp) << kIndexBits) | (uint32_t)i;
  }
  static __device__ __forceinline__ int32_t lp(Word k) { return kLpMax - (int32_t)(k >> kIndexBits); }
  static __device__ __forceinline__ int32_t index(Word k) {
    return (int32_t)(k & ((1u << kIndexBits) - 1u));
  }
};

// ---------------------------------------------------------------------------------------
// Longest-first list scheduling in wavefront 0.
//
// keys[] holds the sequences sorted by (padded length descending, index ascending), packed as
// Key64 or Key32 above (Kc names the packing).  The chain of N "give the next
// sequence to the least loaded rank" steps is serial by definition, so everything is about the
// latency of one step.  Up to 64 ranks the loads are never searched: the ranks are kept as a
// list SORTED by (load, rank) across the lanes, one word per lane, and a step removes the head
// and re-inserts it with its grown load by one max and one min against the neighbouring lane
// (lpt_sorted with 32-bit words, lpt_sorted64 with 64-bit words for large or squared loads).
// Only beyond 64 ranks (lpt_blocks) do the loads stay in place, in LDS, and the minimum is
// searched with a v_min_u32 DPP butterfly over 32-bit distances from the running minimum.
// ---------------------------------------------------------------------------------------

// Minimum over the first 2^kSteps lanes (kSteps <= 4) or over all 64 lanes (kSteps == 6).
template <int kCtrl>
__device__ __forceinline__ uint32_t dpp_min_all_rows(uint32_t x) {
  // every source lane of these controls exists, so bound_ctrl never takes effect; written this
  // way the compiler folds the move into one v_min_u32_dpp
  const uint32_t y = (uint32_t)__builtin_amdgcn_mov_dpp((int)x, kCtrl, 0xf, 0xf, true);
  return y < x ? y : x;
}
template <int kSteps>
__device__ __forceinline__ uint32_t wave_min_low(uint32_t x) {
  uint32_t y;
  if (kSteps >= 1) x = dpp_min_all_rows<kDppQuadXor1>(x);
  if (kSteps >= 2) x = dpp_min_all_rows<kDppQuadXor2>(x);
  if (kSteps >= 3) x = dpp_min_all_rows<kDppRowHalfMirror>(x);
  if (kSteps >= 4) x = dpp_min_all_rows<kDppRowMirror>(x);
  if (kSteps >= 5) {
    y = dpp_u32<kDppRowBcast15, 0xa>(x, x); x = y < x ? y : x;
    y = dpp_u32<kDppRowBcast31, 0xc>(x, x); x = y < x ? y : x;
  }
  return (uint32_t)__builtin_amdgcn_readlane((int)x, kSteps >= 5 ? 63 : 0);
}

// D <= 64, loads small enough that (load << 6 | rank) fits 32 bits for the whole run.
//
// The ranks are kept SORTED by that word across the lanes (lane 0 holds the least loaded rank,
// the lowest one among equals since the rank number sits in the low bits; lanes >= D hold all
// ones).  A step takes the head, adds the sequence's padded length and puts the word back in
// its place: with w'[i] = w[i+1] (the list without its head) the new list is
//     w_new[i] = min(w'[i], max(w[i], grown))
// (below the insertion point w'[i] < grown, so the min keeps w'[i]; at it w[i] < grown < w'[i]
// gives grown; above it w[i] > grown and w[i] < w'[i] keep w[i]).  That is one v_max and one
// v_min with a DPP lane shift, against a log2(D)-step butterfly plus compare and select when
// the loads stay in place and the minimum is searched; head and grown word travel through
// scalar registers, and the head word (the winner is its low six bits) is written into lane s
// of `heads`.  (The median of the three in one v_med3_u32, on a shifted copy of the list kept in
// a register of its own, shortens the dependency chain by one instruction and measured 8 %
// slower: the lone wavefront's time follows the bytes of code it runs through, 0.4 ns per byte,
// not the chain's length, and v_med3_u32 takes eight bytes where v_max_u32 takes four.)
// kShift: row_shl:1 when the ranks fit one row of 16 lanes, else wave_shl:1.
// Items past N have length 0 and come last: the head is put back where it was.
// Lanes >= D hold 0xffffffff; a real word stays below it because the caller only takes this
// path when every load is below 2^26 - 1 (the largest word is then (2^26 - 2) << 6 | 63).
template <int kLane>
__device__ __forceinline__ void writelane_const(uint32_t& v, uint32_t value) {
  // v_writelane_b32 has no builtin in this compiler; lane number is an immediate
  asm volatile("v_writelane_b32 %0, %1, %2" : "+v"(v) : "s"(value), "n"(kLane));
}

// Two steps of the chain, written out by hand: six instructions per step (length to a scalar
// register, head to a scalar register, scalar add, max, record the head, min with the
// neighbouring lane) against eight from the compiler, which masks the rank before recording it
// and fills the one wait state that reading a fresh result across lanes needs with a no-op,
// where here the read of the next length stands (measured: 21.7 -> 19 ns per step; a lone
// wavefront issues an instruction every six to seven cycles).  The list alternates between the
// registers a and b: the DPP min writes over its second operand, whose lanes without a
// right-hand neighbour (end of the row or of the wavefront) keep max(word, grown), as if they
// had read all ones.  kItem is even; `heads` receives in lane s the head word at step s, whose
// low six bits are the winning rank.
#define EARL_LPT_TWO_STEPS(SHIFT)                                                        \
  asm volatile(                                                                          \
      "v_readlane_b32 %[lp], %[lp6], %[k0]\n\t"                                          \
      "v_readfirstlane_b32 %[head], %[a]\n\t"                                            \
      "s_add_u32 %[grown], %[head], %[lp]\n\t"                                           \
      "v_max_u32 %[b], %[grown], %[a]\n\t"                                               \
      "v_writelane_b32 %[heads], %[head], %[k0]\n\t"                                     \
      "v_min_u32_dpp %[b], %[a], %[b] " SHIFT " row_mask:0xf bank_mask:0xf\n\t"          \
      "v_readlane_b32 %[lp], %[lp6], %[k1]\n\t"                                          \
      "v_readfirstlane_b32 %[head], %[b]\n\t"                                            \
      "s_add_u32 %[grown], %[head], %[lp]\n\t"                                           \
      "v_max_u32 %[a], %[grown], %[b]\n\t"                                               \
      "v_writelane_b32 %[heads], %[head], %[k1]\n\t"                                     \
      "v_min_u32_dpp %[a], %[b], %[a] " SHIFT " row_mask:0xf bank_mask:0xf\n\t"          \
      : [a] "+v"(a), [b] "=&v"(b), [heads] "+v"(heads), [lp] "=&s"(s_lp),                \
        [head] "=&s"(s_head), [grown] "=&s"(s_grown)                                     \
      : [lp6] "v"(lp6), [k0] "n"(kItem), [k1] "n"(kItem + 1)                             \
      : "scc")

template <int kShift, int kItem>
__device__ __forceinline__ void lpt_sorted_two_steps(uint32_t& a, uint32_t& heads, uint32_t lp6) {
  uint32_t b, s_lp, s_head, s_grown;
  if (kShift == kDppRowShl1) EARL_LPT_TWO_STEPS("row_shl:1");
  else EARL_LPT_TWO_STEPS("wave_shl:1");
}
#undef EARL_LPT_TWO_STEPS

template <int kShift, int... kPairs>
__device__ __forceinline__ void lpt_sorted_block(uint32_t& word, uint32_t& heads, uint32_t lp6,
                                                 std::integer_sequence<int, kPairs...>) {
  (lpt_sorted_two_steps<kShift, 2 * kPairs>(word, heads, lp6), ...);
}

template <class Kc, int kShift>
__device__ void lpt_sorted(const PlanDev& p, const typename Kc::Word* keys, int32_t* rank_out) {
  const int lane = lane_id();
  const int N = p.N;
  uint32_t word = lane < p.D ? (uint32_t)lane : 0xffffffffu;   // load << 6 | rank
  for (int start = 0; start < N; start += kWave) {
    const int i = start + lane;
    const typename Kc::Word key = i < N ? keys[i] : Kc::kLast;
    const uint32_t lp6 = i < N ? (uint32_t)Kc::lp(key) << 6 : 0u;
    const int32_t idx = Kc::index(key);
    uint32_t heads = 0;   // lane s: the list's head word when the s-th item of this block came
    lpt_sorted_block<kShift>(word, heads, lp6, std::make_integer_sequence<int, kWave / 2>{});
    if (i < N) rank_out[idx] = (int32_t)(heads & 63u);
  }
}

// Up to 16 ranks: the whole chain on the vector unit.  The list fits one row of 16 lanes, and
// every row holds its own identical copy; row_newbcast (a DPP control of this chip family that
// hands one lane of a row to all its lanes) replaces the trip through scalar registers that
// v_readfirstlane / s_add / scalar operand make, so a step is five vector instructions: the
// next length to all lanes (off the chain), head + length, max, min with the neighbouring lane,
// and a masked move that records head + length (its low six bits are the winner) in the four
// lanes of one (row, bank), item s ending up in lane s of register s mod 4.  Written by hand
// so that the two wait states a cross-lane read of a fresh result needs are always filled.
// lp_j: lane l holds the shifted padded length of item 16*j + (l & 15) of the block.
#define EARL_LPT16_STEP(A, B, H, BANK, NEXTREG, NEXTLANE)                                        \
  "v_add_u32_dpp %[g], %[" A "], %[lp] row_newbcast:0 row_mask:0xf bank_mask:0xf\n\t"            \
  "v_max_u32 %[" B "], %[g], %[" A "]\n\t"                                                       \
  "v_min_u32_dpp %[" B "], %[" A "], %[" B "] row_shl:1 row_mask:0xf bank_mask:0xf\n\t"          \
  "v_mov_b32_dpp %[" H "], %[g] quad_perm:[0,1,2,3] row_mask:%[rm] bank_mask:" BANK "\n\t"       \
  "v_mov_b32_dpp %[lp], %[" NEXTREG "] row_newbcast:" NEXTLANE " row_mask:0xf bank_mask:0xf\n\t"

// Sixteen steps on the items of one lp register (lane l of lpreg: item 16*kQuarter + (l & 15)).
// The list alternates between a and b and is back in a at the end.  lp holds the first item's
// length in all lanes on entry and the next sixteen's first (from lpnext) on exit: the length
// move and the record move are the two instructions that every cross-lane read of the list
// needs between it and the instruction that wrote the list, inside a block and from one block
// to the next.
template <int kQuarter>
__device__ __forceinline__ void lpt16_sixteen_steps(uint32_t& a, uint32_t& lp, uint32_t lpreg,
                                                    uint32_t lpnext, uint32_t& h0, uint32_t& h1,
                                                    uint32_t& h2, uint32_t& h3) {
  uint32_t b, g;
  asm volatile(
      EARL_LPT16_STEP("a", "b", "h0", "1", "lpreg", "1")
      EARL_LPT16_STEP("b", "a", "h1", "1", "lpreg", "2")
      EARL_LPT16_STEP("a", "b", "h2", "1", "lpreg", "3")
      EARL_LPT16_STEP("b", "a", "h3", "1", "lpreg", "4")
      EARL_LPT16_STEP("a", "b", "h0", "2", "lpreg", "5")
      EARL_LPT16_STEP("b", "a", "h1", "2", "lpreg", "6")
      EARL_LPT16_STEP("a", "b", "h2", "2", "lpreg", "7")
      EARL_LPT16_STEP("b", "a", "h3", "2", "lpreg", "8")
      EARL_LPT16_STEP("a", "b", "h0", "4", "lpreg", "9")
      EARL_LPT16_STEP("b", "a", "h1", "4", "lpreg", "10")
      EARL_LPT16_STEP("a", "b", "h2", "4", "lpreg", "11")
      EARL_LPT16_STEP("b", "a", "h3", "4", "lpreg", "12")
      EARL_LPT16_STEP("a", "b", "h0", "8", "lpreg", "13")
      EARL_LPT16_STEP("b", "a", "h1", "8", "lpreg", "14")
      EARL_LPT16_STEP("a", "b", "h2", "8", "lpreg", "15")
      EARL_LPT16_STEP("b", "a", "h3", "8", "lpnext", "0")
      : [a] "+v"(a), [b] "=&v"(b), [g] "=&v"(g), [lp] "+v"(lp), [h0] "+v"(h0), [h1] "+v"(h1),
        [h2] "+v"(h2), [h3] "+v"(h3)
      : [lpreg] "v"(lpreg), [lpnext] "v"(lpnext), [rm] "n"(1 << kQuarter));
}
#undef EARL_LPT16_STEP

template <class Kc>
__device__ void lpt_sorted16(const PlanDev& p, const typename Kc::Word* keys, int32_t* rank_out) {
  const int lane = lane_id();
  const int N = p.N;
  const int col = lane & 15;
  uint32_t word = col < p.D ? (uint32_t)col : 0xffffffffu;   // load << 6 | rank, one list per row
  for (int start = 0; start < N; start += kWave) {
    uint32_t lpreg[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int x = start + 16 * j + col;
      lpreg[j] = x < N ? (uint32_t)Kc::lp(keys[x]) << 6 : 0u;
    }
    uint32_t h0 = 0, h1 = 0, h2 = 0, h3 = 0;
    // item 0's length to all lanes; the blocks below keep it one item ahead
    uint32_t lp = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)lpreg[0], 0x150, 0xf, 0xf, false);
    lpt16_sixteen_steps<0>(word, lp, lpreg[0], lpreg[1], h0, h1, h2, h3);
    lpt16_sixteen_steps<1>(word, lp, lpreg[1], lpreg[2], h0, h1, h2, h3);
    lpt16_sixteen_steps<2>(word, lp, lpreg[2], lpreg[3], h0, h1, h2, h3);
    lpt16_sixteen_steps<3>(word, lp, lpreg[3], lpreg[3], h0, h1, h2, h3);
    const int i = start + lane;
    if (i < N) {
      const uint32_t mine = (lane & 2) ? ((lane & 1) ? h3 : h2) : ((lane & 1) ? h1 : h0);
      rank_out[Kc::index(keys[i])] = (int32_t)(mine & 63u);
    }
  }
}

// The same sorted list with 64-bit words (two registers per lane), for loads that do not fit 26
// bits: huge padded lengths, or the quadratic cost (kQuadratic: a rank's load grows by the
// square of the padded length).  D <= 64 and loads below 2^58.
template <bool kQuadratic, int kItem>
__device__ __forceinline__ void lpt_sorted64_step(uint64_t& word, uint32_t& ranks, uint32_t lp) {
  const uint32_t lp_s = (uint32_t)__builtin_amdgcn_readlane((int)lp, kItem);
  const uint64_t cost = kQuadratic ? (uint64_t)lp_s * lp_s : (uint64_t)lp_s;
  const uint32_t head_lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)word);
  const uint32_t head_hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(word >> 32));
  const uint64_t grown = (((uint64_t)head_hi << 32) | head_lo) + (cost << 6);
  const uint64_t t = word > grown ? word : grown;
  const uint32_t next_lo = (uint32_t)__builtin_amdgcn_update_dpp(
      (int)0xffffffffu, (int)(uint32_t)word, kDppWaveShl1, 0xf, 0xf, false);
  const uint32_t next_hi = (uint32_t)__builtin_amdgcn_update_dpp(
      (int)0xffffffffu, (int)(uint32_t)(word >> 32), kDppWaveShl1, 0xf, 0xf, false);
  const uint64_t next = ((uint64_t)next_hi << 32) | next_lo;
  word = next < t ? next : t;
  writelane_const<kItem>(ranks, head_lo & 63u);
}

template <bool kQuadratic, int... kItems>
__device__ __forceinline__ void lpt_sorted64_block(uint64_t& word, uint32_t& ranks, uint32_t lp,
                                                   std::integer_sequence<int, kItems...>) {
  (lpt_sorted64_step<kQuadratic, kItems>(word, ranks, lp), ...);
}

template <class Kc, bool kQuadratic>
__device__ void lpt_sorted64(const PlanDev& p, const typename Kc::Word* keys, int32_t* rank_out) {
  const int lane = lane_id();
  const int N = p.N;
  uint64_t word = lane < p.D ? (uint64_t)lane : ~0ull;   // load << 6 | rank
  for (int start = 0; start < N; start += kWave) {
    const int i = start + lane;
    const typename Kc::Word key = i < N ? keys[i] : Kc::kLast;
    const uint32_t lp = i < N ? (uint32_t)Kc::lp(key) : 0u;
    const int32_t idx = Kc::index(key);
    uint32_t ranks = 0;
    lpt_sorted64_block<kQuadratic>(word, ranks, lp, std::make_integer_sequence<int, kWave>{});
    if (i < N) rank_out[idx] = (int32_t)ranks;
  }
}

// Any D <= 1024: each lane owns the loads (in LDS) of a block of consecutive ranks, so a lower
// lane always means lower ranks and ties resolve to the lowest rank by taking the first lane
// that holds the minimum.  kQuadratic: a rank's load grows by the square of the padded length
// (padded lengths up to 2^21, so a load stays below 2^62); the distance of a load from the
// smallest one then needs 64 bits and is reduced in two 32-bit rounds, high words first.
template <class Kc, bool kQuadratic>
__device__ void lpt_blocks(const PlanDev& p, const typename Kc::Word* keys, int64_t* lds_load,
                           int32_t* rank_out) {
  const int lane = lane_id();
  const int D = p.D, N = p.N;
  const int kper = (D + kWave - 1) / kWave;
  const int r_lo = lane * kper;
  const int r_hi = min(D, r_lo + kper);
  const bool owner = r_lo < D;
  for (int r = r_lo; r < r_hi; ++r) lds_load[r] = 0;
  int64_t best = 0;     // smallest load among this lane's ranks
  int best_r = r_lo;    // the lowest rank that has it
  int64_t base = 0;     // uniform: the minimum load over all ranks before the current step

  for (int start = 0; start < N; start += kWave) {
    const int i = start + lane;
    const typename Kc::Word key = i < N ? keys[i] : Kc::kLast;
    const int32_t lp = Kc::lp(key);
    const int32_t idx = Kc::index(key);
    int my_rank = 0;
    const int cnt = min(kWave, N - start);
    for (int s = 0; s < cnt; ++s) {
      const int32_t lp_s = __builtin_amdgcn_readlane(lp, s);
      int wl;
      int64_t mn;
      if (kQuadratic) {
        const uint64_t rel = owner ? (uint64_t)(best - base) : ~0ull;
        const uint32_t hi = (uint32_t)(rel >> 32), lo = (uint32_t)rel;
        const uint32_t hi_mn = wave_min_low<6>(hi);
        const uint32_t lo_mn = wave_min_low<6>(hi == hi_mn ? lo : 0xffffffffu);
        wl = __builtin_ctzll(__ballot(hi == hi_mn && lo == lo_mn));
        mn = (int64_t)(((uint64_t)hi_mn << 32) | lo_mn);
      } else {
        const uint32_t rel = owner ? (uint32_t)(best - base) : 0xffffffffu;
        const uint32_t rel_mn = wave_min_low<6>(rel);
        wl = __builtin_ctzll(__ballot(rel == rel_mn));
        mn = rel_mn;
      }
      const int r = __builtin_amdgcn_readlane(best_r, wl);
      base += mn;
      if (lane == wl) {
        lds_load[r] += kQuadratic ? (int64_t)lp_s * lp_s : (int64_t)lp_s;
        best = lds_load[r_lo];
        best_r = r_lo;
        for (int q = r_lo + 1; q < r_hi; ++q) {
          const int64_t v = lds_load[q];
          if (v < best) { best = v; best_r = q; }
        }
      }
      if (lane == s) my_rank = r;
    }
    if (i < N) rank_out[idx] = my_rank;
  }
}

// rank_out: where rank[i] goes (the workspace array, or an LDS copy of it).  lds_load is only
// needed beyond 64 ranks or 2^58 load units.
template <class Kc>
__device__ void lpt_wave0(const PlanDev& p, const typename Kc::Word* keys, int64_t* lds_load,
                          int32_t* rank_out) {
  const int D = p.D;
  const int64_t max_lp = Kc::lp(keys[0]);   // keys are sorted
  const bool quadratic = p.policy == 2;
  // no load exceeds total / D + the largest cost (the bound of list scheduling)
  const int64_t max_cost = quadratic ? max_lp * max_lp : max_lp;      // <= 2^42, N * it <= 2^62
  const int64_t load_bound = (int64_t)p.N * max_cost / D + max_cost;
  if (D > kWave || load_bound >= (1ll << 58)) {
    if (quadratic) lpt_blocks<Kc, true>(p, keys, lds_load, rank_out);
    else lpt_blocks<Kc, false>(p, keys, lds_load, rank_out);
  } else if (quadratic) {
    lpt_sorted64<Kc, true>(p, keys, rank_out);
  } else if (load_bound >= (1 << 26) - 1) {
    lpt_sorted64<Kc, false>(p, keys, rank_out);
  } else if (D <= 16) {
    lpt_sorted16<Kc>(p, keys, rank_out);
  } else {
    lpt_sorted<Kc, kDppWaveShl1>(p, keys, rank_out);
  }
}

// LDS carve-up: the sort keys and the label-scan tables are never live at the same time.
constexpr size_t kLdsTabSumBytes = sizeof(int64_t) * (2 * kPlanWaves + 1) * kLdsLabels;
constexpr size_t kLdsTabCntBytes = sizeof(int32_t) * (2 * kPlanWaves + 1) * kLdsLabels;
constexpr size_t kLdsSortBytes = sizeof(uint64_t) * kLdsSortKeys;
constexpr size_t kLdsUnionBytes =
    (kLdsTabSumBytes + kLdsTabCntBytes) > kLdsSortBytes ? (kLdsTabSumBytes + kLdsTabCntBytes)
                                                        : kLdsSortBytes;

__device__ __forceinline__ void zero_tables(int64_t* tab_sum, int32_t* tab_cnt, int n_labels) {
  const size_t n = (size_t)(2 * kPlanWaves + 1) * n_labels;
  for (size_t x = threadIdx.x; x < n; x += T) {
    tab_sum[x] = 0;
    tab_cnt[x] = 0;
  }
  __syncthreads();
}

__global__ __launch_bounds__(kPlanThreads) void plan_kernel(const PlanDev p) {
  __shared__ __align__(16) unsigned char lds_union[kLdsUnionBytes];
  __shared__ int64_t lds_load[kMaxDp];
  __shared__ BlockScratch bs;
  __shared__ int s_invalid, s_exceeds, s_bad, s_bad_invalid;
  __shared__ unsigned long long s_a2a[kLdsA2a];

  const int tid = threadIdx.x;
  const int N = p.N, G = p.G, R = p.R, S = p.S, D = p.D, C = p.C, K = p.K, P = p.P;
  const int halves = p.halves;
  const int n_dst = D * C;
  const int64_t B = p.B;

  // ---- phase 0: clear accumulators --------------------------------------------------------
  if (tid == 0) { s_invalid = 0; s_exceeds = 0; s_bad = -1; s_bad_invalid = -1; }
  if (S * n_dst > kLdsA2a)
    for (int64_t x = tid; x < (int64_t)S * n_dst; x += T) p.a2a[x] = 0;
  for (int x = tid; x < S; x += T) { p.src_rows_needed[x] = 0; p.src_seqs_needed[x] = 0; }
  for (int x = tid; x < n_dst; x += T) p.shard_rows[x] = 0;
  for (int x = tid; x < D; x += T) { p.n_seq[x] = 0; p.n_mb[x] = 0; p.rank_load[x] = 0; }
  __syncthreads();

  // ---- phase 1: validation and padded chunk geometry --------------------------------------
  // K equal chunks per sequence, each the smallest multiple of P that covers ceil(L/K) rows.
  const int64_t lp_cap = B < 0x7fffffffll ? B : 0x7fffffffll;
  int64_t real_rows = 0;
  for (int i = tid; i < N; i += T) {
    int32_t L = p.lengths[i];
    bool invalid = false;
    if (L < 1) { invalid = true; L = 1; }
    int64_t g = p.seq_group_in ? (int64_t)p.seq_group_in[i] : ((int64_t)i * G) / N;
    if (g < 0 || g >= G) { invalid = true; g = 0; }
    if (p.seq_row_in && p.seq_row_in[i] < 0) invalid = true;
    const int64_t per = ((int64_t)L + K - 1) / K;
    int64_t m = (int64_t)P * ((per + P - 1) / P);
    const bool exceeds = m * K > lp_cap;
    if (exceeds) m = 1;
    if (p.policy == 2 && m * K > kMaxQuadraticLp) invalid = true;   // squared loads must fit
    p.seq_group[i] = (int32_t)g;
    p.m[i] = (int32_t)m;
    real_rows += L;
    // s_bad: the largest offending index (an invalid one counts before one over the budget)
    if (invalid) { s_invalid = 1; atomicMax(&s_bad_invalid, i); }
    else if (exceeds) { s_exceeds = 1; atomicMax(&s_bad, i); }
  }
  __syncthreads();
  if (s_invalid || s_exceeds) {
    if (tid == 0) {
      PlanHeader h = {};
      h.status = s_invalid ? 1 : 2;
      h.bad_index = s_invalid ? s_bad_invalid : s_bad;
      *p.hdr = h;
    }
    publish_summary(p);
    return;
  }
  {
    int64_t tot;
    block_excl_scan(real_rows, bs, &tot);
    real_rows = tot;
  }

  // Scan tables: LDS when the label count fits, else the workspace.
  const int lmax = G > D ? G : D;
  int64_t* tab_sum;
  int32_t* tab_cnt;
  if (lmax <= kLdsLabels) {
    tab_sum = reinterpret_cast<int64_t*>(lds_union);
    tab_cnt = reinterpret_cast<int32_t*>(lds_union + kLdsTabSumBytes);
  } else {
    tab_sum = p.lab_sum;
    tab_cnt = p.lab_cnt;
  }

  // ---- phase 2: source offsets and replica choice ------------------------------------------
  // Packed row offset = exclusive scan of L over the group's earlier members; the k-th of a
  // group's n members is read from replica floor(k*R/n) ("from their computation origins").
  zero_tables(tab_sum, tab_cnt, G);
  label_scan(
      N, G, [&](int i) { return p.seq_group[i]; }, [&](int i) { return (int64_t)p.lengths[i]; },
      [&](int i, int32_t k, int64_t row) {
        p.seq_k[i] = k;
        p.seq_row[i] = p.seq_row_in ? p.seq_row_in[i] : row;
      },
      tab_sum, tab_cnt);
  {
    const int32_t* group_cnt = tab_cnt + 2 * (size_t)kPlanWaves * G;
    const bool lds_max = 2 * S <= kLdsA2a;   // rows needed per shard: maxima taken in LDS
    if (lds_max) {
      for (int x = tid; x < 2 * S; x += T) s_a2a[x] = 0;
      __syncthreads();
    }
    for (int i = tid; i < N; i += T) {
      const int g = p.seq_group[i];
      const int k = p.seq_k[i];
      const int64_t t = R == 1 ? 0 : ((int64_t)k * R) / group_cnt[g];
      const int s = g * R + (int)t;
      p.seq_shard[i] = s;
      const unsigned long long need = (unsigned long long)(p.seq_row[i] + p.lengths[i]);
      const unsigned long long need_seqs = (unsigned long long)k + 1ull;
      if (lds_max) {
        atomicMax(&s_a2a[s], need);
        atomicMax(&s_a2a[S + s], need_seqs);
      } else {
        atomicMax(reinterpret_cast<unsigned long long*>(&p.src_rows_needed[s]), need);
        atomicMax(reinterpret_cast<unsigned long long*>(&p.src_seqs_needed[s]), need_seqs);
      }
    }
    if (lds_max) {
      __syncthreads();
      for (int x = tid; x < S; x += T) {
        p.src_rows_needed[x] = (int64_t)s_a2a[x];
        p.src_seqs_needed[x] = (int64_t)s_a2a[S + x];
      }
    }
  }
  __syncthreads();

  // ---- phase 3: sort by (padded length desc, index asc), then rank assignment --------------
  uint64_t* keys = p.n_pow2 <= kLdsSortKeys ? reinterpret_cast<uint64_t*>(lds_union) : p.sort_keys;
  for (int i = tid; i < p.n_pow2; i += T) {
    uint64_t key = ~0ull;
    if (i < N) {
      const int64_t lp = (int64_t)p.m[i] * K;
      key = ((uint64_t)(0x7fffffffll - lp) << 32) | (uint32_t)i;
    }
    keys[i] = key;
  }
  __syncthreads();
  bitonic_sort(keys, p.n_pow2, p.n_pow2 <= kLdsSortKeys);
  if (p.policy == 1) {
    // sorted snake deal: rounds of D, left to right in even rounds, right to left in odd ones
    for (int j = tid; j < N; j += T) {
      const int round = j / D, k = j - round * D;
      p.rank[(int32_t)(keys[j] & 0xffffffffu)] = (round & 1) ? D - 1 - k : k;
    }
  } else if (wave_id() == 0) {
    lpt_wave0<Key64>(p, keys, lds_load, p.rank);
  }
  __syncthreads();

  // ---- phase 4: packing order, destination offsets, micro-batches --------------------------
  zero_tables(tab_sum, tab_cnt, D);
  label_scan(
      N, D, [&](int i) { return p.rank[i]; },
      [&](int i) { return (int64_t)p.m[i] * halves; },
      [&](int i, int32_t k, int64_t row) {
        p.slot[i] = k;
        p.dst_row[i] = row;
      },
      tab_sum, tab_cnt);
  const int64_t* rank_rows = tab_sum + 2 * (size_t)kPlanWaves * D;
  const int32_t* rank_cnt = tab_cnt + 2 * (size_t)kPlanWaves * D;
  int64_t load_max = 0, load_min = 0;
  {
    // D <= 1024: one rank per thread.
    const int32_t ns = tid < D ? rank_cnt[tid] : 0;
    int64_t tot;
    const int64_t ex = block_excl_scan(ns, bs, &tot);
    if (tid < D) {
      p.rank_seq_base[tid] = (int32_t)ex;
      p.n_seq[tid] = ns;
      for (int c = 0; c < C; ++c) p.shard_rows[(size_t)tid * C + c] = rank_rows[tid];
    }
    if (tid == 0) p.rank_seq_base[D] = N;
    const int64_t ld = tid < D ? rank_rows[tid] * C : 0;   // padded tokens = C * rows per SP rank
    if (tid < D) p.rank_load[tid] = ld;
    load_max = block_reduce_max(tid < D ? ld : INT64_MIN, bs);
    load_min = block_reduce_min(tid < D ? ld : INT64_MAX, bs);
  }
  __syncthreads();
  // sequences of a rank in ascending index; row_packed[pos] = destination row of the pos-th
  int64_t* row_packed = reinterpret_cast<int64_t*>(p.sort_keys);
  for (int i = tid; i < N; i += T) {
    const int pos = p.rank_seq_base[p.rank[i]] + p.slot[i];
    p.seq_ids[pos] = i;
    row_packed[pos] = p.dst_row[i];
  }
  __syncthreads();
  // Next-fit: the micro-batch that starts at slot s ends before the first slot u whose
  // inclusive padded prefix exceeds prefix(s) + B.  Padded prefix = C * destination row.
  for (int pos = tid; pos < N; pos += T) {
    const int r = p.rank[p.seq_ids[pos]];
    const int base = p.rank_seq_base[r];
    const int n = rank_cnt[r];
    const int s = pos - base;
    const int64_t limit = row_packed[pos] * C + B;
    int lo = s + 1, hi = n + 1;   // smallest u in [s+1, n] with E(u) > limit, else n+1
    while (lo < hi) {
      const int mid = (lo + hi) >> 1;
      const int64_t e = (mid < n ? row_packed[base + mid] : rank_rows[r]) * C;
      if (e > limit) hi = mid; else lo = mid + 1;
    }
    const int nxt = lo <= n ? lo - 1 : n;
    p.next_start[pos] = nxt > s ? nxt : s + 1;   // a micro-batch always holds its first sequence
  }
  __syncthreads();
  for (int r = tid; r < D; r += T) {
    const int base = p.rank_seq_base[r];
    const int n = rank_cnt[r];
    int s = 0, b = 0;
    while (s < n) {
      p.mb_tmp[base + r + b] = s;
      s = p.next_start[base + s];
      ++b;
    }
    p.mb_tmp[base + r + b] = n;
    p.n_mb[r] = b;
  }
  __syncthreads();
  int n_mb_max = 0;
  int64_t mb_table_len = 0, cu_len = 0;
  {
    const int32_t nm_own = tid < D ? p.n_mb[tid] : 0;
    n_mb_max = (int)block_reduce_max(nm_own, bs);
    // equal_mb: every rank gets the micro-batch count of the rank that has most
    const int32_t nm = p.equal_mb && tid < D ? n_mb_max : nm_own;
    const int32_t ns = tid < D ? rank_cnt[tid] : 0;
    const int64_t ex1 = block_excl_scan(tid < D ? nm + 1 : 0, bs, &mb_table_len);
    const int64_t ex2 = block_excl_scan(tid < D ? nm + ns : 0, bs, &cu_len);
    if (tid < D) {
      p.rank_mbt_base[tid] = (int32_t)ex1;
      p.rank_cu_base[tid] = (int32_t)ex2;
    }
    if (tid == 0) {
      p.rank_mbt_base[D] = (int32_t)mb_table_len;
      p.rank_cu_base[D] = (int32_t)cu_len;
    }
  }
  __syncthreads();
  // compact the per-rank micro-batch tables
  for (int x = tid; x < N + D; x += T) {
    int lo = 0, hi = D;   // last rank r with rank_seq_base[r] + r <= x
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (p.rank_seq_base[mid] + mid <= x) lo = mid; else hi = mid;
    }
    const int r = lo;
    const int b = x - (p.rank_seq_base[r] + r);
    if (b <= p.n_mb[r]) {
      const int s = p.mb_tmp[x];
      const int n = rank_cnt[r];
      const int o = p.rank_mbt_base[r] + b;
      p.mb_seq_start[o] = s;
      p.mb_row_start[o] = s < n ? row_packed[p.rank_seq_base[r] + s] : rank_rows[r];
    }
  }
  if (p.equal_mb) {
    // the appended micro-batches are empty: they start at the rank's last sequence and last row
    for (int x = tid; x < (int)mb_table_len; x += T) {
      const int r = x / (n_mb_max + 1);
      const int b = x - r * (n_mb_max + 1);
      if (b > p.n_mb[r]) {
        p.mb_seq_start[x] = rank_cnt[r];
        p.mb_row_start[x] = rank_rows[r];
      }
    }
    __syncthreads();
    for (int r = tid; r < D; r += T) p.n_mb[r] = n_mb_max;
  }
  __syncthreads();
  // micro-batch of every sequence; cu_seqlens (local rows, restarting in every micro-batch)
  for (int pos = tid; pos < N; pos += T) {
    const int i = p.seq_ids[pos];
    const int r = p.rank[i];
    const int s = pos - p.rank_seq_base[r];
    const int32_t* starts = p.mb_seq_start + p.rank_mbt_base[r];
    int lo = 0, hi = p.n_mb[r];   // last b with starts[b] <= s
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (starts[mid] <= s) lo = mid; else hi = mid;
    }
    p.mb[i] = lo;
    p.cu_seqlens[p.rank_cu_base[r] + s + lo] =
        (int32_t)(row_packed[pos] - p.mb_row_start[p.rank_mbt_base[r] + lo]);
  }
  for (int x = tid; x < (int)mb_table_len; x += T) {
    int lo = 0, hi = D;   // last rank r with rank_mbt_base[r] <= x
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (p.rank_mbt_base[mid] <= x) lo = mid; else hi = mid;
    }
    const int r = lo;
    const int b = x - p.rank_mbt_base[r];
    if (b < p.n_mb[r]) {
      const int64_t rows = p.mb_row_start[x + 1] - p.mb_row_start[x];
      if (rows > 0x7fffffffll) s_invalid = 1;   // cu_seqlens entries are int32
      p.cu_seqlens[p.rank_cu_base[r] + p.mb_seq_start[x + 1] + b] = (int32_t)rows;
    }
  }

  // ---- phase 5: segment table and all-to-all counts ----------------------------------------
  // One segment per (sequence, chunk): m rows contiguous in both layouts.  SP rank c holds chunk
  // c and, with zigzag, chunk 2C-1-c right after it.
  const int64_t n_seg = (int64_t)N * K;
  const int n_pairs = S * n_dst;
  const bool lds_counts = n_pairs <= kLdsA2a;   // count in LDS, flush once
  if (lds_counts) {
    for (int x = tid; x < n_pairs; x += T) s_a2a[x] = 0;
    __syncthreads();
  }
  __syncthreads();   // mb[] of every sequence is complete
  for (int pos = tid; pos < N; pos += T) {
    const int i = p.seq_ids[pos];
    const int r = p.rank[i];
    const int base = p.rank_seq_base[r];
    const int n = rank_cnt[r];
    const int32_t mi = p.m[i];
    const int32_t mb_i = p.mb[i];
    const int64_t len = p.lengths[i];
    const int s = p.seq_shard[i];
    const int64_t src_row = p.seq_row[i];
    const int64_t dst_row = p.dst_row[i];
    const int32_t k_in_group = p.seq_k[i];
    for (int c = 0; c < C; ++c) {
      const int64_t e0 = (int64_t)halves * ((int64_t)C * base + (int64_t)c * n + (pos - base));
      int64_t real_rows = 0;
      for (int h = 0; h < halves; ++h) {
        const int kappa = h == 0 ? c : 2 * C - 1 - c;
        const int64_t p0 = (int64_t)kappa * mi;
        int64_t n_real = len - p0;
        n_real = n_real < 0 ? 0 : (n_real > mi ? mi : n_real);
        SegRec rec;
        rec.dst_row = dst_row + (int64_t)h * mi;
        rec.src_row = src_row + p0;
        rec.n_real = (int32_t)n_real;
        rec.n_rows = mi;
        rec.src_shard = s;
        rec.pos0 = (int32_t)p0;
        p.segs[e0 + h] = rec;
        p.seg_dst_shard[e0 + h] = r * C + c;
        p.seg_src_seq[e0 + h] = k_in_group;
        p.seg_mb[e0 + h] = mb_i;
        real_rows += n_real;
      }
      if (real_rows > 0) {
        const size_t x = (size_t)s * n_dst + r * C + c;
        if (lds_counts) atomicAdd(&s_a2a[x], (unsigned long long)real_rows);
        else atomicAdd(reinterpret_cast<unsigned long long*>(&p.a2a[x]), (unsigned long long)real_rows);
      }
    }
  }
  if (lds_counts) {
    __syncthreads();
    for (int x = tid; x < n_pairs; x += T) p.a2a[x] = (int64_t)s_a2a[x];
  }
  for (int q = tid; q <= n_dst; q += T) {
    int64_t v = n_seg;
    if (q < n_dst) {
      const int r = q / C, c = q - r * C;
      v = (int64_t)halves * ((int64_t)C * p.rank_seq_base[r] + (int64_t)c * rank_cnt[r]);
    }
    p.shard_seg_start[q] = (int32_t)v;
  }
  int64_t dst_rows = 0;
  {
    int64_t tot;
    block_excl_scan(tid < D ? rank_rows[tid] * C : 0, bs, &tot);
    dst_rows = tot;
  }
  if (tid == 0) {
    PlanHeader h = {};
    h.status = s_invalid ? 1 : 0;
    h.bad_index = -1;
    h.n_segments = (int32_t)n_seg;
    h.n_mb_max = n_mb_max;
    h.cu_seqlens_len = (int32_t)cu_len;
    h.mb_table_len = (int32_t)mb_table_len;
    h.total_real_rows = real_rows;
    h.total_dst_rows = dst_rows;
    h.rank_load_min = load_min;
    h.rank_load_max = load_max;
    *p.hdr = h;
  }
  publish_summary(p);
}

// ---------------------------------------------------------------------------------------
// The same plan for batches of up to 4096 sequences on up to 64 ranks (the paper gives no batch
// sizes; a few hundred to a few thousand sequences per step is what the synthetic workloads
// assume), with another data flow: nothing is read back from global memory (beyond 2048
// sequences: nothing but the per-sequence outputs, once, for the segment table).
//
// The kernel above keeps every intermediate array in the workspace, so each of its ~40
// barrier-separated phases pays a store -> barrier -> load round trip through the L2 cache
// (a microsecond each, more than the arithmetic).  Here a thread owns kIters CONSECUTIVE
// sequences and keeps what it computes for them (length, chunk length, source offset, shard,
// rank, slot, destination row) in registers until its place in the packed order is known; what
// other threads need (sort keys, ranks, the packed order with its row offsets and a copy of the
// per-sequence values, micro-batch starts) lives in LDS.  Global memory sees the input lengths
// once and the outputs once, the segment table in table order (neighbouring lanes write
// neighbouring records; written per sequence, 32-byte records scattered over the ranks' blocks,
// the table alone took 25 us for 2048 sequences in 8 chunks).
// The workgroup is as wide as the batch needs (64 sequences run in one wavefront, where
// barriers cost nothing).  Rules, tie-breaks and outputs are those of plan_kernel, which stays
// the general path (more sequences, ranks or groups, explicit group labels).
// ---------------------------------------------------------------------------------------
constexpr int kResStagedSeqs = 2048;   // up to here the segment table's inputs are staged in LDS
constexpr int kResMaxSeqs = 4096;      // up to here the rest of the batch still fits
constexpr int kResMaxGroups = 256;     // source groups, and source shards
constexpr int kResMaxRanks = 64;

// kCap: sequences the arrays hold.  kStaged: a packed-order copy of what the segment table needs
// about every sequence is kept in LDS (7 arrays; with 4096 sequences they do not fit, and the
// segment table reads the per-sequence outputs back from the workspace instead).
template <int kCap, bool kStaged>
struct ResidentLds {
  static constexpr int kStage = kStaged ? kCap : 1;
  union {
    uint64_t keys[kCap];        // sort keys, until the ranks are assigned
    uint32_t keys32[kCap];      // (the narrow packing, when every padded length allows it)
    int64_t row_packed[kCap];   // then: destination row of the pos-th sequence, packed order
  };
  int32_t rank[kCap];           // by sequence
  int32_t seq_ids[kCap];        // packed order -> sequence
  int32_t next_start[kCap];     // packed order: first slot of the following micro-batch
  int64_t rows_before[kCap];    // by sequence: real rows of all sequences before it
  // what the segment table needs about the pos-th sequence of the packed order
  int64_t st_src_row[kStage];
  int32_t st_len[kStage];
  int32_t st_m[kStage];
  int32_t st_shard[kStage];
  int32_t st_k[kStage];
  int32_t st_mb[kStage];
  int32_t mb_tmp[kCap + kResMaxRanks];   // per rank: start slot of each micro-batch, then n
  unsigned long long need[2 * kResMaxGroups];   // rows / sequences every source shard must hold
  union {
    struct {
      int64_t sum[kPlanWaves * kResMaxRanks];
      int32_t cnt[kPlanWaves * kResMaxRanks];
    } tab;                                        // per (wavefront, rank) totals of the rank scan
    unsigned long long a2a[kLdsA2a];
  };
  int64_t rank_rows[kResMaxRanks];
  int32_t n_seq[kResMaxRanks];
  int32_t seq_base[kResMaxRanks + 1];
  int32_t n_mb_own[kResMaxRanks];      // micro-batches next-fit gave the rank
  int32_t n_mb[kResMaxRanks];          // micro-batches it reports (equal_mb: the largest count)
  int32_t mbt_base[kResMaxRanks + 1];
  int32_t cu_base[kResMaxRanks + 1];
  BlockScratch bs;
  int64_t load_max, load_min, dst_rows;
  int32_t n_mb_max, mb_table_len, cu_len;
  int invalid, exceeds, bad, bad_invalid;
  int wide;   // some padded length needs the 64-bit sort keys
};

// Last r in [0, D) with base[r] + r * stride_one <= x (base ascending, base[0] == 0).
__device__ __forceinline__ int rank_of_entry(const int32_t* base, int D, int x, int stride_one) {
  int lo = 0, hi = D;
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (base[mid] + mid * stride_one <= x) lo = mid; else hi = mid;
  }
  return lo;
}

template <int kIters, int kCap, bool kStaged>
__global__ __launch_bounds__(kPlanThreads) void plan_resident_kernel(const PlanDev p) {
  typedef Key32<kCap == 4096 ? 12 : 11> K32;   // index bits for kCap sequences, the rest for the length
  static_assert(kCap <= (1 << K32::kIndexBits), "index bits of the narrow keys");
  __shared__ ResidentLds<kCap, kStaged> s;
  const int tid = threadIdx.x, nt = blockDim.x, nw = nt >> 6;
  const int lane = lane_id(), wave = wave_id();
  const int N = p.N, G = p.G, R = p.R, S = p.S, D = p.D, C = p.C, K = p.K, P = p.P;
  const int halves = p.halves, n_dst = D * C;
  const int64_t B = p.B;
  const int i0 = tid * kIters;   // this thread owns sequences i0 .. i0 + kIters - 1

  if (tid == 0) { s.invalid = 0; s.exceeds = 0; s.bad = -1; s.bad_invalid = -1; s.wide = 0; }
  for (int x = tid; x < 2 * S; x += nt) s.need[x] = 0;
  __syncthreads();

  // ---- validation and padded chunk geometry (as phase 1 of plan_kernel) --------------------
  const int64_t lp_cap = B < 0x7fffffffll ? B : 0x7fffffffll;
  int32_t len[kIters], m[kIters];
  int64_t own_rows = 0;
#pragma unroll
  for (int j = 0; j < kIters; ++j) {
    const int i = i0 + j;
    len[j] = 0;
    m[j] = 1;
    if (i < N) {
      int32_t L = p.lengths[i];
      bool invalid = false;
      if (L < 1) { invalid = true; L = 1; }
      if (p.seq_row_in && p.seq_row_in[i] < 0) invalid = true;
      // L, K and P are below 2^31, so the roundings fit unsigned 32-bit division
      const uint32_t per = ((uint32_t)L + (uint32_t)K - 1u) / (uint32_t)K;
      int64_t mm = (int64_t)P * (int64_t)((per + (uint32_t)P - 1u) / (uint32_t)P);
      const bool exceeds = mm * K > lp_cap;
      if (exceeds) mm = 1;
      if (mm * K >= ((int64_t)1 << K32::kLpBits)) s.wide = 1;
      if (p.policy == 2 && mm * K > kMaxQuadraticLp) invalid = true;
      len[j] = L;
      m[j] = (int32_t)mm;
      own_rows += L;
      if (invalid) { s.invalid = 1; atomicMax(&s.bad_invalid, i); }
      else if (exceeds) { s.exceeds = 1; atomicMax(&s.bad, i); }
    }
  }
  __syncthreads();
  if (s.invalid || s.exceeds) {
    if (tid == 0) {
      PlanHeader h = {};
      h.status = s.invalid ? 1 : 2;
      h.bad_index = s.invalid ? s.bad_invalid : s.bad;
      put_summary(p, p.hdr, h);
    }
    publish_summary(p, false);
    return;
  }

  // ---- real rows before every sequence (for the source offsets below) ----------------------
  int64_t real_rows = 0;
  int64_t pre[kIters];
  {
    int64_t acc = block_excl_scan(own_rows, s.bs, &real_rows, nw);
#pragma unroll
    for (int j = 0; j < kIters; ++j) {
      pre[j] = acc;
      if (i0 + j < N) {
        s.rows_before[i0 + j] = acc;
        p.seq_pre[i0 + j] = acc;
      }
      acc += len[j];
    }
    if (tid == 0) p.seq_pre[N] = real_rows;
  }

  // ---- sort by (padded length desc, index asc), rank assignment ------------------------------
  // With every padded length below 2^21 (2^20 beyond 2048 sequences) key and index fit 32 bits,
  // and so do the row offsets (fewer than 2^32 / largest padded length sequences).
  const bool narrow = s.wide == 0;
  if (narrow) {
#pragma unroll
    for (int j = 0; j < kIters; ++j)
      if (i0 + j < N) s.keys32[i0 + j] = K32::make((int64_t)m[j] * K, i0 + j);
    for (int x = N + tid; x < p.n_pow2; x += nt) s.keys32[x] = K32::kLast;
    __syncthreads();
    bitonic_sort_lanes32(s.keys32, p.n_pow2);
  } else {
#pragma unroll
    for (int j = 0; j < kIters; ++j)
      if (i0 + j < N) s.keys[i0 + j] = Key64::make((int64_t)m[j] * K, i0 + j);
    for (int x = N + tid; x < p.n_pow2; x += nt) s.keys[x] = Key64::kLast;
    __syncthreads();
    bitonic_sort_lanes(s.keys, p.n_pow2);
  }
  if (p.policy == 1) {
    for (int x = tid; x < N; x += nt) {
      const int round = x / D, k = x - round * D;
      const int i = narrow ? K32::index(s.keys32[x]) : Key64::index(s.keys[x]);
      s.rank[i] = (round & 1) ? D - 1 - k : k;
    }
  } else if (wave == 0) {
    // D <= 64 and N <= 4096: the LDS load table is never used
    if (narrow) lpt_wave0<K32>(p, s.keys32, nullptr, s.rank);
    else lpt_wave0<Key64>(p, s.keys, nullptr, s.rank);
  }

  // ---- source offsets and replica choice ----------------------------------------------------
  // Nothing here depends on the ranks: the other wavefronts do it while wavefront 0 walks the
  // chain above, and wavefront 0 follows for its own sequences.  Groups own contiguous index
  // ranges (g = floor(i*G/N)), so the segmented scan is the plain scan of the lengths minus its
  // value at the group's first sequence.  i, G, R and N are small enough for 32-bit products.
  int32_t shard[kIters], seq_k[kIters];
  int64_t src_row[kIters];
#pragma unroll
  for (int j = 0; j < kIters; ++j) {
    const uint32_t i = (uint32_t)(i0 + j);
    shard[j] = 0; seq_k[j] = 0; src_row[j] = 0;
    if ((int)i < N) {
      const uint32_t g = i * (uint32_t)G / (uint32_t)N;
      const uint32_t first = (g * (uint32_t)N + (uint32_t)G - 1u) / (uint32_t)G;   // smallest index of group g
      const uint32_t next_first = ((g + 1u) * (uint32_t)N + (uint32_t)G - 1u) / (uint32_t)G;
      const uint32_t k = i - first;
      const int64_t row = p.seq_row_in ? p.seq_row_in[i] : pre[j] - s.rows_before[first];
      const uint32_t t = R == 1 ? 0u : k * (uint32_t)R / (next_first - first);
      const int sh = (int)(g * (uint32_t)R + t);
      shard[j] = sh;
      seq_k[j] = (int32_t)k;
      src_row[j] = row;
      atomicMax(&s.need[sh], (unsigned long long)(row + len[j]));
      atomicMax(&s.need[S + sh], (unsigned long long)k + 1ull);
    }
  }
  __syncthreads();
  for (int x = tid; x < S; x += nt) {
    put_summary(p, &p.src_rows_needed[x], (int64_t)s.need[x]);
    put_summary(p, &p.src_seqs_needed[x], (int64_t)s.need[S + x]);
  }

  // ---- position inside the rank and destination row: scan by rank, in index order -----------
  // Per rank one wavefront scan of (count << 48 | rows); a lane's own sequences are consecutive,
  // so their order inside the lane is index order as well.
  int32_t rk[kIters], slot[kIters];
  int64_t dst_row[kIters];
#pragma unroll
  for (int j = 0; j < kIters; ++j) {
    rk[j] = i0 + j < N ? s.rank[i0 + j] : -1;
    slot[j] = 0;
    dst_row[j] = 0;
  }
  constexpr int64_t kRowsMask = ((int64_t)1 << 48) - 1;
  if (narrow) {
    // row offsets stay below N * 2^21 <= 2^32: one 32-bit scan of the rows per rank, and the
    // position from the lanes' vote
    for (int r = 0; r < D; ++r) {
      uint32_t mine = 0;
      uint64_t vote[kIters];
      int n_here = 0;
#pragma unroll
      for (int j = 0; j < kIters; ++j) {
        vote[j] = __ballot(rk[j] == r);
        n_here += __builtin_popcountll(vote[j]);
        if (rk[j] == r) mine += (uint32_t)(m[j] * halves);
      }
      uint32_t tot = 0;
      if (n_here != 0) {
        const uint32_t incl = wave_incl_scan_u32(mine);
        uint32_t ex = incl - mine;
        int before = 0;
#pragma unroll
        for (int j = 0; j < kIters; ++j) before += count_below(vote[j]);
#pragma unroll
        for (int j = 0; j < kIters; ++j)
          if (rk[j] == r) {
            slot[j] = before++;
            dst_row[j] = ex;
            ex += (uint32_t)(m[j] * halves);
          }
        tot = (uint32_t)__builtin_amdgcn_readlane((int)incl, kWave - 1);
      }
      if (lane == 0) {
        s.tab.cnt[wave * D + r] = n_here;
        s.tab.sum[wave * D + r] = tot;
      }
    }
  } else
  for (int r = 0; r < D; ++r) {
    int64_t mine = 0;
#pragma unroll
    for (int j = 0; j < kIters; ++j)
      if (rk[j] == r) mine += ((int64_t)1 << 48) + (int64_t)m[j] * halves;
    int64_t tot = 0;
    if (__ballot(mine != 0) != 0) {
      const int64_t incl = wave_incl_scan_i64(mine);
      int64_t ex = incl - mine;
#pragma unroll
      for (int j = 0; j < kIters; ++j)
        if (rk[j] == r) {
          slot[j] = (int32_t)(ex >> 48);
          dst_row[j] = ex & kRowsMask;
          ex += ((int64_t)1 << 48) + (int64_t)m[j] * halves;
        }
      tot = readlane_i64(incl, kWave - 1);
    }
    if (lane == 0) {
      s.tab.cnt[wave * D + r] = (int32_t)(tot >> 48);
      s.tab.sum[wave * D + r] = tot & kRowsMask;
    }
  }
  __syncthreads();
  if (wave == 0) {
    // lane r: prefix over the wavefronts, totals of rank r, then the scans over the ranks
    int32_t ac = 0;
    int64_t as = 0;
    if (lane < D) {
      for (int w = 0; w < nw; ++w) {
        const int x = w * D + lane;
        const int32_t c = s.tab.cnt[x];
        const int64_t v = s.tab.sum[x];
        s.tab.cnt[x] = ac;
        s.tab.sum[x] = as;
        ac += c;
        as += v;
      }
      s.n_seq[lane] = ac;
      s.rank_rows[lane] = as;
      put_summary(p, &p.n_seq[lane], ac);
      put_summary(p, &p.rank_load[lane], as * C);      // padded tokens = C * rows per SP rank
      for (int c = 0; c < C; ++c) put_summary(p, &p.shard_rows[(size_t)lane * C + c], as);
    }
    const int64_t incl = wave_incl_scan_i64(ac);
    if (lane < D) s.seq_base[lane] = (int32_t)(incl - ac);
    if (lane == 0) s.seq_base[D] = N;
    const int64_t ld = as * C;
    int64_t mx = lane < D ? ld : INT64_MIN, mn = lane < D ? ld : INT64_MAX;
    for (int d = 32; d > 0; d >>= 1) {
      const int64_t a = __shfl_xor(mx, d), b = __shfl_xor(mn, d);
      mx = a > mx ? a : mx;
      mn = b < mn ? b : mn;
    }
    const int64_t rows_incl = wave_incl_scan_i64(lane < D ? ld : 0);
    if (lane == kWave - 1) { s.load_max = mx; s.load_min = mn; s.dst_rows = rows_incl; }
  }
  __syncthreads();
#pragma unroll
  for (int j = 0; j < kIters; ++j) {
    const int i = i0 + j;
    if (i < N) {
      slot[j] += s.tab.cnt[wave * D + rk[j]];
      dst_row[j] += s.tab.sum[wave * D + rk[j]];
      const int pos = s.seq_base[rk[j]] + slot[j];
      s.seq_ids[pos] = i;
      s.row_packed[pos] = dst_row[j];   // the sort keys are no longer needed
      if (kStaged) {
        s.st_src_row[pos] = src_row[j];
        s.st_len[pos] = len[j];
        s.st_m[pos] = m[j];
        s.st_shard[pos] = shard[j];
        s.st_k[pos] = seq_k[j];
      } else {
        // the segment table reads these back (with seq_shard, seq_row and mb below)
        p.m[i] = m[j];
        p.seq_k[i] = seq_k[j];
      }
      // per-sequence outputs (the micro-batch follows from the packed order below)
      p.rank[i] = rk[j];
      p.slot[i] = slot[j];
      p.dst_row[i] = dst_row[j];
      p.seq_shard[i] = shard[j];
      p.seq_row[i] = src_row[j];
    }
  }
  __syncthreads();

  // ---- micro-batches: next-fit along the packed order (as phase 4 of plan_kernel) -----------
  const int n_pairs = S * n_dst;
  for (int x = tid; x < n_pairs; x += nt) s.a2a[x] = 0;   // the scan tables are no longer needed
#pragma unroll
  for (int j = 0; j < kIters; ++j) {
    const int pos = i0 + j;
    if (pos < N) {
      const int r = s.rank[s.seq_ids[pos]];
      const int base = s.seq_base[r];
      const int n = s.n_seq[r];
      const int sl = pos - base;
      const int64_t limit = s.row_packed[pos] * C + B;
      int lo = sl + 1, hi = n + 1;   // smallest u in [sl+1, n] whose padded prefix exceeds limit
      while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        const int64_t e = (mid < n ? s.row_packed[base + mid] : s.rank_rows[r]) * C;
        if (e > limit) hi = mid; else lo = mid + 1;
      }
      const int nxt = lo <= n ? lo - 1 : n;
      s.next_start[pos] = nxt > sl ? nxt : sl + 1;
    }
  }
  __syncthreads();
  if (wave == 0) {
    int b = 0;
    if (lane < D) {
      const int base = s.seq_base[lane];
      const int n = s.n_seq[lane];
      int sl = 0;
      while (sl < n) {
        s.mb_tmp[base + lane + b] = sl;
        sl = s.next_start[base + sl];
        ++b;
      }
      s.mb_tmp[base + lane + b] = n;
      s.n_mb_own[lane] = b;
    }
    int most = b;
    for (int d = 32; d > 0; d >>= 1) {
      const int o = __shfl_xor(most, d);
      most = o > most ? o : most;
    }
    const int nm = p.equal_mb ? most : b;
    const int ns = lane < D ? s.n_seq[lane] : 0;
    const int64_t t1 = lane < D ? nm + 1 : 0, t2 = lane < D ? nm + ns : 0;
    const int64_t i1 = wave_incl_scan_i64(t1), i2 = wave_incl_scan_i64(t2);
    if (lane < D) {
      s.n_mb[lane] = nm;
      put_summary(p, &p.n_mb[lane], nm);
      s.mbt_base[lane] = (int32_t)(i1 - t1);
      s.cu_base[lane] = (int32_t)(i2 - t2);
    }
    if (lane == kWave - 1) {
      s.mbt_base[D] = (int32_t)i1;
      s.cu_base[D] = (int32_t)i2;
      s.mb_table_len = (int32_t)i1;
      s.cu_len = (int32_t)i2;
      s.n_mb_max = most;
    }
  }
  __syncthreads();
  const int n_mb_max = s.n_mb_max, mb_table_len = s.mb_table_len;
  // micro-batch tables (flat, per rank n_mb + 1 entries)
  for (int x = tid; x < N + D; x += nt) {
    const int r = rank_of_entry(s.seq_base, D, x, 1);
    const int b = x - (s.seq_base[r] + r);
    if (b <= s.n_mb_own[r]) {
      const int sl = s.mb_tmp[x];
      const int o = s.mbt_base[r] + b;
      p.mb_seq_start[o] = sl;
      p.mb_row_start[o] = sl < s.n_seq[r] ? s.row_packed[s.seq_base[r] + sl] : s.rank_rows[r];
    }
  }
  if (p.equal_mb) {
    // the appended micro-batches are empty: they start at the rank's last sequence and last row
    for (int x = tid; x < mb_table_len; x += nt) {
      const int r = x / (n_mb_max + 1);
      const int b = x - r * (n_mb_max + 1);
      if (b > s.n_mb_own[r]) {
        p.mb_seq_start[x] = s.n_seq[r];
        p.mb_row_start[x] = s.rank_rows[r];
      }
    }
  }
  // micro-batch of every sequence; cu_seqlens (local rows, restarting in every micro-batch)
#pragma unroll
  for (int j = 0; j < kIters; ++j) {
    const int pos = i0 + j;
    if (pos < N) {
      const int i = s.seq_ids[pos];
      const int r = s.rank[i];
      const int base = s.seq_base[r];
      const int sl = pos - base;
      const int32_t* starts = s.mb_tmp + base + r;
      int lo = 0, hi = s.n_mb_own[r];   // last b with starts[b] <= sl
      while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (starts[mid] <= sl) lo = mid; else hi = mid;
      }
      if (kStaged) s.st_mb[pos] = lo;
      p.mb[i] = lo;
      p.cu_seqlens[s.cu_base[r] + sl + lo] =
          (int32_t)(s.row_packed[pos] - s.row_packed[base + starts[lo]]);
    }
  }
  for (int x = tid; x < mb_table_len; x += nt) {
    const int r = rank_of_entry(s.mbt_base, D, x, 0);
    const int b = x - s.mbt_base[r];
    if (b < s.n_mb[r]) {
      // the entry that closes micro-batch b: its rows (an appended empty one has none)
      const int base = s.seq_base[r], n = s.n_seq[r], own = s.n_mb_own[r];
      const int s0 = b <= own ? s.mb_tmp[base + r + b] : n;
      const int s1 = b + 1 <= own ? s.mb_tmp[base + r + b + 1] : n;
      const int64_t row0 = s0 < n ? s.row_packed[base + s0] : s.rank_rows[r];
      const int64_t row1 = s1 < n ? s.row_packed[base + s1] : s.rank_rows[r];
      if (row1 - row0 > 0x7fffffffll) s.invalid = 1;   // cu_seqlens entries are int32
      p.cu_seqlens[s.cu_base[r] + s1 + b] = (int32_t)(row1 - row0);
    }
  }
  for (int x = tid; x < N; x += nt) p.seq_ids[x] = s.seq_ids[x];
  __syncthreads();   // st_mb[] is complete (not staged: so are this workgroup's stores of mb[])

  // ---- segment table and all-to-all counts (as phase 5 of plan_kernel) ----------------------
  // In table order: entry u = C*base_r + c*n_r + slot stands for the `halves` segments of one
  // sequence on one SP rank.
  for (int u = tid; u < N * C; u += nt) {
    int lo = 0, hi = D;   // last rank r with C * seq_base[r] <= u
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (C * s.seq_base[mid] <= u) lo = mid; else hi = mid;
    }
    const int r = lo;
    const int base = s.seq_base[r];
    const int n = s.n_seq[r];
    const int rem = u - C * base;
    const int c = rem / n;
    const int pos = base + (rem - c * n);
    const int seq = kStaged ? 0 : s.seq_ids[pos];
    const int32_t mi = kStaged ? s.st_m[pos] : p.m[seq];
    const int64_t L = kStaged ? s.st_len[pos] : p.lengths[seq];
    const int64_t src0 = kStaged ? s.st_src_row[pos] : p.seq_row[seq];
    const int64_t dst0 = s.row_packed[pos];
    const int32_t sh = kStaged ? s.st_shard[pos] : p.seq_shard[seq];
    const int32_t k_in_group = kStaged ? s.st_k[pos] : p.seq_k[seq];
    const int32_t mb_i = kStaged ? s.st_mb[pos] : p.mb[seq];
    const int64_t e0 = (int64_t)halves * u;
    int64_t real = 0;
    for (int h = 0; h < halves; ++h) {
      const int kappa = h == 0 ? c : 2 * C - 1 - c;
      const int64_t p0 = (int64_t)kappa * mi;
      int64_t n_real = L - p0;
      n_real = n_real < 0 ? 0 : (n_real > mi ? mi : n_real);
      SegRec rec;
      rec.dst_row = dst0 + (int64_t)h * mi;
      rec.src_row = src0 + p0;
      rec.n_real = (int32_t)n_real;
      rec.n_rows = mi;
      rec.src_shard = sh;
      rec.pos0 = (int32_t)p0;
      p.segs[e0 + h] = rec;
      p.seg_dst_shard[e0 + h] = r * C + c;
      p.seg_src_seq[e0 + h] = k_in_group;
      p.seg_mb[e0 + h] = mb_i;
      real += n_real;
    }
    if (real > 0)
      atomicAdd(&s.a2a[(size_t)sh * n_dst + r * C + c], (unsigned long long)real);
  }
  for (int q = tid; q <= n_dst; q += nt) {
    int64_t v = (int64_t)N * K;
    if (q < n_dst) {
      const int r = q / C, c = q - r * C;
      v = (int64_t)halves * ((int64_t)C * s.seq_base[r] + (int64_t)c * s.n_seq[r]);
    }
    p.shard_seg_start[q] = (int32_t)v;
  }
  __syncthreads();
  for (int x = tid; x < n_pairs; x += nt) put_summary(p, &p.a2a[x], (int64_t)s.a2a[x]);
  if (tid == 0) {
    PlanHeader h = {};
    h.status = s.invalid ? 1 : 0;
    h.bad_index = -1;
    h.n_segments = N * K;
    h.n_mb_max = n_mb_max;
    h.cu_seqlens_len = s.cu_len;
    h.mb_table_len = mb_table_len;
    h.total_real_rows = real_rows;
    h.total_dst_rows = s.dst_rows;
    h.rank_load_min = s.load_min;
    h.rank_load_max = s.load_max;
    put_summary(p, p.hdr, h);
  }
  publish_summary(p, false);
}

// Batches the resident kernel takes (the LDS carve-up above bounds every term).
bool fits_resident(const PlanDev& p) {
  return p.N <= kResMaxSeqs && p.D <= kResMaxRanks && p.G <= kResMaxGroups &&
         p.S <= kResMaxGroups && (int64_t)p.S * p.D * p.C <= kLdsA2a && p.seq_group_in == nullptr;
}

}  // namespace

bool launch_plan(const PlanDev& p, hipStream_t stream) {
  // EARL_PLAN_KERNEL=general forces the general kernel (the parity tests run both on the same
  // inputs this way).
  const char* force = std::getenv("EARL_PLAN_KERNEL");
  const bool general = force && std::strcmp(force, "general") == 0;
  if (!general && fits_resident(p)) {
    const int k_iters = p.N <= kPlanThreads ? 1 : (p.N <= 2 * kPlanThreads ? 2 : 4);
    const int per = (p.N + k_iters - 1) / k_iters;
    const unsigned nt = (unsigned)((per + kWave - 1) / kWave * kWave);
    if (k_iters == 1)
      hipLaunchKernelGGL((plan_resident_kernel<1, kResStagedSeqs, true>), dim3(1), dim3(nt), 0, stream, p);
    else if (k_iters == 2)
      hipLaunchKernelGGL((plan_resident_kernel<2, kResStagedSeqs, true>), dim3(1), dim3(nt), 0, stream, p);
    else
      hipLaunchKernelGGL((plan_resident_kernel<4, kResMaxSeqs, false>), dim3(1), dim3(nt), 0, stream, p);
    return true;
  }
  hipLaunchKernelGGL(plan_kernel, dim3(1), dim3(kPlanThreads), 0, stream, p);
  return false;
}

}  // namespace earl
