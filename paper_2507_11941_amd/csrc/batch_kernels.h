// Batch-level kernels around the per-string encoder: length binning (which kernel variant encodes which
// string, longest strings first), the cutting of long strings into pieces at segment cuts, the marking of
// special-token occurrences, the scan of token counts into out_offsets, and the packing of the per-item id
// runs into the dense output (the paper only says that the result is an id tensor, section 2.2; the dense
// ids + offsets layout is this library's).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "table_format.h"

namespace bpe {

constexpr int kMaxTiers = 4;
constexpr int kLenBuckets = 64;                      // length classes inside a tier, longest first
constexpr int kBinKeys = kMaxTiers * kLenBuckets;

struct TierPlan {
  int n_tiers;
  int cap[kMaxTiers];                                // tier t takes strings with cap[t-1] < len <= cap[t]
};

// Control block at the start of the workspace.
struct Control {
  uint32_t tier_base[kMaxTiers + 1];                 // start of each tier's slice of the list
  uint32_t queue_head[kMaxTiers];                    // work-queue heads of the encode kernels
  uint32_t fallback_range[2];                        // {0, items the lane-per-segment kernel passed on}
  uint32_t fallback_queue;                           // work-queue head of the kernel that takes those
  // used only when strings are split into pieces:
  uint32_t n_slots;                                  // piece slots in the batch
  uint32_t hist[kBinKeys];                           // pieces per (tier, length bucket)
  uint32_t key_base[kBinKeys];                       // exclusive scan of hist
  uint32_t cursor[kBinKeys];                         // scatter cursors
};

__device__ inline int bin_key(int len, const TierPlan& plan) {
  int lo = 0;
  for (int t = 0; t < plan.n_tiers; ++t) {
    const int cap = plan.cap[t];
    if (len <= cap) {
      // bucket 0 holds the longest strings of the tier
      const int span = cap - lo;
      int b = span > 0 ? (int)(((uint32_t)(cap - len) * (uint32_t)kLenBuckets) / (uint32_t)span) : 0;
      if (b >= kLenBuckets) b = kLenBuckets - 1;
      return t * kLenBuckets + b;
    }
    lo = cap;
  }
  return -1;                                         // longer than any launched variant: skipped
}

// What a work item is, stored beside its place in the work list: all that an encode kernel needs to start on it.
struct ItemDesc {
  int64_t begin;                                     // first byte of the item in `bytes`
  int32_t len;                                       // its length in bytes
  int32_t item;                                      // string index, or slot index when strings are split
};

// One workgroup bins the whole batch: histogram of (class, length bucket) keys in LDS, exclusive scan of the
// 256 keys, then the scatter of string indices into the work list (class-major, longest bucket first).
// Also resets the work-queue heads.  A second pass over the offsets is cheaper than a second launch.
__global__ __launch_bounds__(1024) void bin_kernel(const int64_t* offsets, int batch, TierPlan plan, Control* c,
                                                   int32_t* list, ItemDesc* desc, int32_t* counts) {
  __shared__ uint32_t hist[kBinKeys], scan[kBinKeys], cursor[kBinKeys];
  const int t = threadIdx.x;
  if (t < kBinKeys) { hist[t] = 0; cursor[t] = 0; }
  __syncthreads();
  for (int s = t; s < batch; s += 1024) {
    const int64_t len = offsets[s + 1] - offsets[s];
    const int key = (len < 0 || len > 0x7FFFFFFF) ? -1 : bin_key((int)len, plan);
    if (key >= 0) atomicAdd(&hist[key], 1u);
    else counts[s] = 0;                              // never encoded: contributes no tokens
  }
  __syncthreads();
  if (t < kBinKeys) scan[t] = hist[t];
  __syncthreads();
  for (int step = 1; step < kBinKeys; step <<= 1) {  // inclusive scan, all threads reach the barriers
    uint32_t v = 0;
    if (t < kBinKeys && t >= step) v = scan[t - step];
    __syncthreads();
    if (t < kBinKeys) scan[t] += v;
    __syncthreads();
  }
  if (t <= kMaxTiers) c->tier_base[t] = t == 0 ? 0 : scan[(t <= plan.n_tiers ? t : plan.n_tiers) * kLenBuckets - 1];
  if (t < kMaxTiers) c->queue_head[t] = 0;
  if (t < 2) c->fallback_range[t] = 0;
  if (t == 2) c->fallback_queue = 0;
  for (int s = t; s < batch; s += 1024) {
    const int64_t len = offsets[s + 1] - offsets[s];
    const int key = (len < 0 || len > 0x7FFFFFFF) ? -1 : bin_key((int)len, plan);
    if (key < 0) continue;
    const uint32_t pos = (scan[key] - hist[key]) + atomicAdd(&cursor[key], 1u);
    list[pos] = s;
    desc[pos] = ItemDesc{offsets[s], (int32_t)len, s};
  }
}

// out_offsets[i] = sum of counts[0..i), out_offsets[batch] = total.  One workgroup walks the batch.
__global__ __launch_bounds__(1024) void offsets_scan_kernel(const int32_t* counts, int batch,
                                                            int64_t* out_offsets) {
  __shared__ int64_t wave_sum[16];
  __shared__ int64_t carry_s;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (tid == 0) { carry_s = 0; out_offsets[0] = 0; }
  __syncthreads();
  for (int base = 0; base < batch; base += 1024) {
    const int i = base + tid;
    int64_t v = i < batch ? (int64_t)counts[i] : 0;
    for (int step = 1; step < 64; step <<= 1) {
      int64_t o = __shfl_up(v, step, 64);
      if (lane >= step) v += o;
    }
    if (lane == 63) wave_sum[wave] = v;
    __syncthreads();
    int64_t before = carry_s;
    for (int w = 0; w < wave; ++w) before += wave_sum[w];
    if (i < batch) out_offsets[i + 1] = before + v;
    __syncthreads();
    if (tid == 1023) carry_s = before + v;
    __syncthreads();
  }
}

// The encode kernels number tokens their own way (byte b = b, row r creates 256 + r); a table built over a
// vocabulary carries the vocabulary's id of each, applied where the ids are written to the output.
__device__ inline int32_t vocabulary_id(const int32_t* id_map, int32_t token) {
  return id_map ? id_map[token] : token;
}

// Small batches: offsets and packing in one launch.  Workgroup s sums the counts before its string itself
// (the batch is at most a few thousand strings), writes out_offsets[s] and copies the string's ids.
__global__ __launch_bounds__(256) void scan_pack_kernel(const int32_t* tmp_ids, const int64_t* offsets,
                                                        const int32_t* counts, int batch, int64_t* out_offsets,
                                                        int32_t* out_ids, const int32_t* id_map) {
  __shared__ int64_t wave_sum[4];
  const int s = blockIdx.x;
  int64_t v = 0;
  for (int i = threadIdx.x; i < s; i += 256) v += counts[i];
  for (int step = 32; step >= 1; step >>= 1) v += __shfl_down(v, step, 64);
  if ((threadIdx.x & 63) == 0) wave_sum[threadIdx.x >> 6] = v;
  __syncthreads();
  const int64_t dst = wave_sum[0] + wave_sum[1] + wave_sum[2] + wave_sum[3];
  const int k = counts[s];
  if (threadIdx.x == 0) {
    out_offsets[s] = dst;
    if (s == batch - 1) out_offsets[batch] = dst + k;
  }
  const int64_t src = offsets[s];
  for (int i = threadIdx.x; i < k; i += 256) out_ids[dst + i] = vocabulary_id(id_map, tmp_ids[src + i]);
}

// One workgroup per string: copy its ids from the per-string staging area to the dense output.
__global__ __launch_bounds__(256) void pack_kernel(const int32_t* tmp_ids, const int64_t* offsets,
                                                   const int64_t* out_offsets, int batch, int32_t* out_ids,
                                                   const int32_t* id_map) {
  for (int s = blockIdx.x; s < batch; s += gridDim.x) {
    const int64_t src = offsets[s], dst = out_offsets[s];
    const int k = (int)(out_offsets[s + 1] - dst);
    for (int i = threadIdx.x; i < k; i += blockDim.x) out_ids[dst + i] = vocabulary_id(id_map, tmp_ids[src + i]);
  }
}

// ---------------------------------------------------------------------------------------------------
// Splitting long strings into pieces.
//
// No merge can cross a cut (a byte bigram that occurs at no merge junction, see table_format.h), so the two
// sides of a cut are encoded independently and their ids concatenated.  Strings longer than the piece target
// P are therefore cut near every multiple of P: the string gets ceil(len / P) "slots"; slot 0 starts at the
// string's first byte, slot i at the last cut within kCutWindow bytes before byte i*P, or is void if there is
// none (then the piece before it simply runs on).  Pieces, not strings, are what the encode kernels work on;
// their ids land in tmp_ids at the piece's own byte offset, so a string's ids are the concatenation of its
// slots' runs.

constexpr int kCutWindow = 128;

__device__ inline uint32_t slots_of_length(int64_t len, int piece_target, int max_string) {
  // (a 32-bit division: a valid length fits, and the 64-bit one is a long software routine)
  return (len <= 0 || len > max_string) ? 1u : ((uint32_t)len + (uint32_t)piece_target - 1u) / (uint32_t)piece_target;
}
__device__ inline uint32_t slots_of(const int64_t* offsets, int s, int piece_target, int max_string) {
  return slots_of_length(offsets[s + 1] - offsets[s], piece_target, max_string);
}

// Slots per string, their exclusive scan (slot_base), and the owner string of every slot.  Workgroup b owns
// strings [1024 b, 1024 b + 1024): it counts the slots of all strings before its tile itself (the lengths are
// 8 bytes per string and come from L2), scans its own tile, and fills the tile's stretch of slot_string by
// binary search in the tile's prefix sums, one slot per thread and step.
__global__ __launch_bounds__(1024) void slot_layout_kernel(const int64_t* offsets, int batch, int piece_target,
                                                           int max_string, Control* c, int32_t* slot_base,
                                                           int32_t* slot_string) {
  __shared__ uint32_t wave_sum[16];
  __shared__ uint32_t first_s[1025];                   // slot_base of the tile's strings, relative to the tile
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int base = blockIdx.x * 1024;
  if (blockIdx.x == 0) {
    if (tid < kBinKeys) { c->hist[tid] = 0; c->cursor[tid] = 0; }
    if (tid < kMaxTiers) c->queue_head[tid] = 0;
    if (tid < 2) c->fallback_range[tid] = 0;
    if (tid == 2) c->fallback_queue = 0;
  }
  // slots of all strings before the tile
  uint32_t before = 0;
  for (int s0 = tid; s0 < base; s0 += 8 * 1024) {      // eight strings' loads in flight per thread: the loads
    int64_t lo[8], hi[8];                              // are unconditional (index clamped), the test comes after
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int s = min(s0 + u * 1024, base - 1);
      lo[u] = offsets[s];
      hi[u] = offsets[s + 1];
    }
#pragma unroll
    for (int u = 0; u < 8; ++u)
      before += s0 + u * 1024 < base ? slots_of_length(hi[u] - lo[u], piece_target, max_string) : 0u;
  }
  for (int step = 32; step >= 1; step >>= 1) before += (uint32_t)__shfl_xor((int)before, step, 64);
  if (lane == 0) wave_sum[wave] = before;
  __syncthreads();
  uint32_t tile_first = 0;
  for (int w = 0; w < 16; ++w) tile_first += wave_sum[w];
  __syncthreads();
  // the tile itself
  const int s = base + tid;
  const uint32_t m = s < batch ? slots_of(offsets, s, piece_target, max_string) : 0u;
  uint32_t v = m;
  for (int step = 1; step < 64; step <<= 1) {
    const uint32_t o = (uint32_t)__shfl_up((int)v, step, 64);
    if (lane >= step) v += o;
  }
  if (lane == 63) wave_sum[wave] = v;
  __syncthreads();
  uint32_t in_tile = v - m;
  for (int w = 0; w < wave; ++w) in_tile += wave_sum[w];
  first_s[tid] = in_tile;
  if (tid == 1023) first_s[1024] = in_tile + m;
  if (s < batch) slot_base[s] = (int32_t)(tile_first + in_tile);
  __syncthreads();
  const uint32_t tile_total = first_s[1024];
  for (uint32_t g = tid; g < tile_total; g += 1024) {
    int lo = 0, hi = 1023;                             // the last string of the tile whose first slot is <= g
    while (lo < hi) {
      const int mid = (lo + hi + 1) >> 1;
      if (first_s[mid] <= g) lo = mid; else hi = mid - 1;
    }
    slot_string[tile_first + g] = base + lo;
  }
  if (blockIdx.x == gridDim.x - 1 && tid == 0) {
    slot_base[batch] = (int32_t)(tile_first + tile_total);
    c->n_slots = tile_first + tile_total;
  }
}

// Eight lanes per slot, eight slots per wave: where does the slot's piece start?  The candidates are the 128
// positions q = t, t-1, ..., t-127 below the slot's nominal start t (a cut "before q" lies between bytes q-1 and
// q); the largest one with a cut wins.  A group looks at eight candidates per round -- in text the first round
// nearly always finds one -- and the wave goes on while any of its groups is still looking.
constexpr int kCutSlotsPerWave = 4;
__global__ __launch_bounds__(256) void cut_search_kernel(const uint8_t* bytes, const int64_t* offsets,
                                                         const uint32_t* byte_pair, int piece_target,
                                                         int max_string, const Control* c, const int32_t* slot_base,
                                                         const int32_t* slot_string, int64_t* piece_begin,
                                                         const uint8_t* cover) {
  const int lane = threadIdx.x & 63, sub = lane & 15, group = lane >> 4;
  const uint32_t g = (blockIdx.x * 4 + (threadIdx.x >> 6)) * kCutSlotsPerWave + group;
  const bool valid = g < c->n_slots;
  int64_t start = -1;                                  // void unless a cut is found
  int64_t t = 0;
  bool searching = false;
  if (valid) {
    const int s = slot_string[g];
    const int i = (int)g - slot_base[s];
    const int64_t begin = offsets[s];
    const int64_t len = offsets[s + 1] - begin;
    if (len < 0 || len > max_string) {
      start = -1;                                      // not encodable: the string yields no tokens
    } else if (i == 0) {
      start = begin;
    } else {
      t = begin + (int64_t)i * piece_target;           // piece_target >= 2 * kCutWindow keeps q-1 inside the string
      searching = true;
    }
  }
  for (int round = 0; round < kCutWindow / 16; ++round) {
    if (!__ballot(searching)) break;                   // uniform
    bool cut = false;
    if (searching) {
      const int64_t q = t - 16 * round - sub;
      const uint32_t a = bytes[q - 1], b = bytes[q];
      cut = byte_pair[(a << 8) | b] == kCut;
      if (cover) {                                     // special tokens: their ends are cuts, their inside is not
        const uint32_t ma = cover[q - 1], mb = cover[q];
        cut = (cut || ma != 0 || mb != 0) && mb != kCoverRest;
      }
    }
    const uint32_t mine = (uint32_t)(__ballot(cut) >> (16 * group)) & 0xFFFFu;
    if (searching && mine) {
      start = t - 16 * round - __builtin_ctz(mine);    // the largest candidate of the round
      searching = false;
    }
  }
  if (valid && sub == 0) piece_begin[g] = start;
}

// One thread per slot: piece lengths, and the histogram of (tier, length bucket) keys.
__global__ __launch_bounds__(256) void piece_hist_kernel(const int64_t* offsets, TierPlan plan, Control* c,
                                                         const int32_t* slot_base, const int32_t* slot_string,
                                                         const int64_t* piece_begin, int32_t* piece_len,
                                                         int32_t* counts) {
  __shared__ uint32_t hist[kBinKeys];
  hist[threadIdx.x] = 0;                               // 256 threads, 256 keys
  __syncthreads();
  const uint32_t n_slots = c->n_slots;
  for (uint32_t g = blockIdx.x * 256 + threadIdx.x; g < n_slots; g += gridDim.x * 256) {
    const int64_t start = piece_begin[g];
    int32_t len = 0;
    int key = -1;
    if (start >= 0) {
      const int s = slot_string[g];
      int64_t next = offsets[s + 1];
      for (int h = (int)g + 1; h < slot_base[s + 1]; ++h)
        if (piece_begin[h] >= 0) { next = piece_begin[h]; break; }
      len = (int32_t)(next - start);
      key = bin_key(len, plan);
      if (key >= 0) atomicAdd(&hist[key], 1u);
    }
    piece_len[g] = len;
    if (key < 0) counts[g] = 0;                        // void slot, or too long for the launched variants
  }
  __syncthreads();
  if (hist[threadIdx.x]) atomicAdd(&c->hist[threadIdx.x], hist[threadIdx.x]);
}

// One workgroup of 256: exclusive scan of the key histogram, list bases of the tiers.
__global__ __launch_bounds__(256) void piece_scan_kernel(Control* c, int n_tiers) {
  __shared__ uint32_t scan[kBinKeys];
  const int t = threadIdx.x;
  const uint32_t mine = c->hist[t];
  scan[t] = mine;
  __syncthreads();
  for (int step = 1; step < kBinKeys; step <<= 1) {
    const uint32_t v = t >= step ? scan[t - step] : 0;
    __syncthreads();
    scan[t] += v;
    __syncthreads();
  }
  c->key_base[t] = scan[t] - mine;
  if (t <= kMaxTiers) c->tier_base[t] = t == 0 ? 0 : scan[(t <= n_tiers ? t : n_tiers) * kLenBuckets - 1];
}

// Scatter the pieces into the work list, tier-major, longest bucket first.  Pieces of a long text all have about
// the same length, hence the same key: a workgroup first ranks its pieces per key in LDS and then reserves each
// key's range of the list with one global atomic.  Those atomics land on a handful of addresses and are served
// one after the other, so a workgroup takes kScatterPer slots per thread: fewer workgroups, fewer atomics.
constexpr int kScatterPer = 4;
__global__ __launch_bounds__(256) void piece_scatter_kernel(TierPlan plan, Control* c, const int64_t* piece_begin,
                                                            const int32_t* piece_len, int32_t* list, ItemDesc* desc) {
  __shared__ uint32_t local[kBinKeys];                 // 256 threads, 256 keys
  local[threadIdx.x] = 0;
  __syncthreads();
  const uint32_t n_slots = c->n_slots;
  int key[kScatterPer];
  uint32_t rank[kScatterPer];
  int64_t begin[kScatterPer];
  int32_t len[kScatterPer];
#pragma unroll
  for (int j = 0; j < kScatterPer; ++j) {
    const uint32_t g = (blockIdx.x * kScatterPer + j) * 256 + threadIdx.x;
    key[j] = -1;
    rank[j] = 0;
    begin[j] = -1;
    len[j] = 0;
    if (g < n_slots) {
      begin[j] = piece_begin[g];
      len[j] = piece_len[g];
    }
  }
#pragma unroll
  for (int j = 0; j < kScatterPer; ++j) {
    if (begin[j] >= 0) {
      key[j] = bin_key(len[j], plan);
      if (key[j] >= 0) rank[j] = atomicAdd(&local[key[j]], 1u);
    }
  }
  __syncthreads();
  const uint32_t mine = local[threadIdx.x];
  __syncthreads();
  if (mine) local[threadIdx.x] = c->key_base[threadIdx.x] + atomicAdd(&c->cursor[threadIdx.x], mine);
  __syncthreads();
#pragma unroll
  for (int j = 0; j < kScatterPer; ++j) {
    if (key[j] >= 0) {
      const uint32_t g = (blockIdx.x * kScatterPer + j) * 256 + threadIdx.x;
      list[local[key[j]] + rank[j]] = (int32_t)g;
      desc[local[key[j]] + rank[j]] = ItemDesc{begin[j], len[j], (int32_t)g};
    }
  }
}

// piece_hist_kernel, piece_scan_kernel and piece_scatter_kernel in one workgroup, for batches of at most
// kSmallSlots slots (a launch costs more than the work of a small batch).  Thread t takes slots t, t + 1024, ...
constexpr int kSmallSlots = 4096;
__global__ __launch_bounds__(1024) void piece_list_small_kernel(const int64_t* offsets, TierPlan plan, Control* c,
                                                                const int32_t* slot_base, const int32_t* slot_string,
                                                                const int64_t* piece_begin, int32_t* piece_len,
                                                                int32_t* counts, int32_t* list, ItemDesc* desc) {
  __shared__ uint32_t hist[kBinKeys], scan[kBinKeys];
  const int t = threadIdx.x;
  if (t < kBinKeys) hist[t] = 0;
  __syncthreads();
  const uint32_t n_slots = c->n_slots;
  constexpr int kPer = kSmallSlots / 1024;
  int32_t len[kPer];
  int key[kPer];
  uint32_t rank[kPer];
  int64_t start[kPer];
#pragma unroll
  for (int j = 0; j < kPer; ++j) {
    const uint32_t g = (uint32_t)t + 1024u * j;
    len[j] = 0;
    key[j] = -1;
    rank[j] = 0;
    start[j] = -1;
    if (g < n_slots) {
      start[j] = piece_begin[g];
      if (start[j] >= 0) {
        const int s = slot_string[g];
        int64_t next = offsets[s + 1];
        for (int h = (int)g + 1; h < slot_base[s + 1]; ++h)
          if (piece_begin[h] >= 0) { next = piece_begin[h]; break; }
        len[j] = (int32_t)(next - start[j]);
        key[j] = bin_key(len[j], plan);
        if (key[j] >= 0) rank[j] = atomicAdd(&hist[key[j]], 1u);
      }
      piece_len[g] = len[j];
      if (key[j] < 0) counts[g] = 0;                   // void slot, or too long for the launched variants
    }
  }
  __syncthreads();
  if (t < kBinKeys) scan[t] = hist[t];
  __syncthreads();
  for (int step = 1; step < kBinKeys; step <<= 1) {    // inclusive scan, all threads reach the barriers
    uint32_t v = 0;
    if (t < kBinKeys && t >= step) v = scan[t - step];
    __syncthreads();
    if (t < kBinKeys) scan[t] += v;
    __syncthreads();
  }
  if (t <= kMaxTiers) c->tier_base[t] = t == 0 ? 0 : scan[(t <= plan.n_tiers ? t : plan.n_tiers) * kLenBuckets - 1];
#pragma unroll
  for (int j = 0; j < kPer; ++j) {
    if (key[j] >= 0) {
      const uint32_t pos = scan[key[j]] - hist[key[j]] + rank[j];
      list[pos] = (int32_t)((uint32_t)t + 1024u * j);
      desc[pos] = ItemDesc{start[j], len[j], (int32_t)((uint32_t)t + 1024u * j)};
    }
  }
}

// Token offsets of the slots: per-tile sums, scan of the tile sums, then the scan inside each tile.
constexpr int kScanTile = 4096;

__global__ __launch_bounds__(1024) void tile_sum_kernel(const int32_t* counts, const Control* c, int64_t* tile_sum) {
  __shared__ int64_t wave_sum[16];
  const uint32_t n_slots = c->n_slots;
  const uint32_t base = blockIdx.x * kScanTile;
  int64_t v = 0;
  for (int j = 0; j < kScanTile / 1024; ++j) {
    const uint32_t g = base + j * 1024 + threadIdx.x;
    if (g < n_slots) v += counts[g];
  }
  for (int step = 32; step >= 1; step >>= 1) v += __shfl_down(v, step, 64);
  if ((threadIdx.x & 63) == 0) wave_sum[threadIdx.x >> 6] = v;
  __syncthreads();
  if (threadIdx.x == 0) {
    int64_t t = 0;
    for (int w = 0; w < 16; ++w) t += wave_sum[w];
    tile_sum[blockIdx.x] = t;
  }
}

__global__ __launch_bounds__(64) void tile_scan_kernel(int64_t* tile_sum, int n_tiles, const Control* c,
                                                       int64_t* out_offsets, int batch) {
  // one wave walks the tiles (there are few: one per 4096 slots); tile_sum becomes the exclusive scan
  const int lane = threadIdx.x;
  const int used = (int)((c->n_slots + kScanTile - 1) / kScanTile);
  int64_t carry = 0;
  for (int base = 0; base < n_tiles; base += 64) {
    const int i = base + lane;
    const int64_t m = (i < n_tiles && i < used) ? tile_sum[i] : 0;
    int64_t v = m;
    for (int step = 1; step < 64; step <<= 1) {
      const int64_t o = __shfl_up(v, step, 64);
      if (lane >= step) v += o;
    }
    if (i < n_tiles) tile_sum[i] = carry + v - m;
    carry += __shfl(v, 63, 64);
  }
  if (lane == 0) out_offsets[batch] = carry;
}

__global__ __launch_bounds__(1024) void slot_offsets_kernel(const int32_t* counts, const Control* c,
                                                            const int64_t* tile_base, const int32_t* slot_base,
                                                            const int32_t* slot_string, int64_t* slot_out,
                                                            int64_t* out_offsets) {
  __shared__ int64_t wave_sum[16];
  __shared__ int64_t carry_s;
  const uint32_t n_slots = c->n_slots;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (tid == 0) carry_s = tile_base[blockIdx.x];
  __syncthreads();
  for (int j = 0; j < kScanTile / 1024; ++j) {
    const uint32_t g = blockIdx.x * kScanTile + j * 1024 + tid;
    const int64_t m = g < n_slots ? (int64_t)counts[g] : 0;
    int64_t v = m;
    for (int step = 1; step < 64; step <<= 1) {
      const int64_t o = __shfl_up(v, step, 64);
      if (lane >= step) v += o;
    }
    if (lane == 63) wave_sum[wave] = v;
    __syncthreads();
    int64_t before = carry_s;
    for (int w = 0; w < wave; ++w) before += wave_sum[w];
    if (g < n_slots) {
      const int64_t at = before + v - m;
      slot_out[g] = at;
      const int s = slot_string[g];
      if ((uint32_t)slot_base[s] == g) out_offsets[s] = at;   // a string starts at its first slot
    }
    __syncthreads();
    if (tid == 1023) carry_s = before + v;
    __syncthreads();
  }
}

// tile_sum_kernel, tile_scan_kernel and slot_offsets_kernel in one workgroup, for at most kSmallSlots slots.
__global__ __launch_bounds__(1024) void slot_offsets_small_kernel(const int32_t* counts, const Control* c,
                                                                  const int32_t* slot_base, const int32_t* slot_string,
                                                                  int64_t* slot_out, int64_t* out_offsets, int batch) {
  __shared__ int64_t wave_sum[16];
  __shared__ int64_t carry_s;
  const uint32_t n_slots = c->n_slots;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (tid == 0) carry_s = 0;
  __syncthreads();
  for (int j = 0; j < kSmallSlots / 1024; ++j) {
    const uint32_t g = (uint32_t)j * 1024u + (uint32_t)tid;
    const int64_t m = g < n_slots ? (int64_t)counts[g] : 0;
    int64_t v = m;
    for (int step = 1; step < 64; step <<= 1) {
      const int64_t o = __shfl_up(v, step, 64);
      if (lane >= step) v += o;
    }
    if (lane == 63) wave_sum[wave] = v;
    __syncthreads();
    int64_t before = carry_s;
    for (int w = 0; w < wave; ++w) before += wave_sum[w];
    if (g < n_slots) {
      const int64_t at = before + v - m;
      slot_out[g] = at;
      const int s = slot_string[g];
      if ((uint32_t)slot_base[s] == g) out_offsets[s] = at;   // a string starts at its first slot
    }
    __syncthreads();
    if (tid == 1023) carry_s = before + v;
    __syncthreads();
  }
  if (tid == 0) out_offsets[batch] = carry_s;
}

// ---------------------------------------------------------------------------------------------------
// Special tokens (section 4.1: special-character lookups before any merging).  The set is small (at most 64
// strings of at most 64 bytes) and, by construction of the set, occurrences cannot overlap, so every byte
// position can decide on its own whether an occurrence starts there: the longest special that matches.

constexpr int kMaxSpecials = 64, kMaxSpecialBytes = 64;

struct SpecialSet {
  uint32_t first_byte[8];                              // bit b: some special starts with byte b
  int32_t n;
  int32_t len[kMaxSpecials];
  uint8_t text[kMaxSpecials][kMaxSpecialBytes];
};

__global__ __launch_bounds__(256) void cover_clear_kernel(uint8_t* cover, int64_t total_bytes) {
  const int64_t words = (total_bytes + 3) / 4;         // the buffer is padded to whole words
  for (int64_t i = blockIdx.x * 256ll + threadIdx.x; i < words; i += gridDim.x * 256ll) ((uint32_t*)cover)[i] = 0u;
}

__global__ __launch_bounds__(256) void special_mark_kernel(const uint8_t* bytes, const int64_t* offsets, int batch,
                                                           int64_t total_bytes, const SpecialSet* set,
                                                           uint8_t* cover) {
  for (int64_t p = blockIdx.x * 256ll + threadIdx.x; p < total_bytes; p += gridDim.x * 256ll) {
    const uint32_t b = bytes[p];
    if (!((set->first_byte[b >> 5] >> (b & 31)) & 1u)) continue;
    int lo = 0, hi = batch - 1;                        // the string that holds p: last s with offsets[s] <= p
    while (lo < hi) {
      const int mid = (lo + hi + 1) >> 1;
      if (offsets[mid] <= p) lo = mid; else hi = mid - 1;
    }
    const int64_t room = offsets[lo + 1] - p;          // bytes from p to the end of its string
    int best = -1, best_len = 0;
    for (int i = 0; i < set->n; ++i) {
      const int len = set->len[i];
      if (len <= best_len || len > room || set->text[i][0] != b) continue;
      int j = 1;
      while (j < len && bytes[p + j] == set->text[i][j]) ++j;
      if (j == len) { best = i; best_len = len; }
    }
    if (best >= 0) {
      cover[p] = (uint8_t)(kCoverFirst | (uint32_t)best);
      for (int j = 1; j < best_len; ++j) cover[p + j] = (uint8_t)kCoverRest;
    }
  }
}

// Copy every piece's ids to their place in the dense output.  A piece has a few hundred ids, so what limits
// this kernel is how many loads are in flight: a wave takes two pieces at a time, reads the next two descriptors
// while it copies, and issues four rows of loads per piece before the first store.
struct PackItem {
  int k;
  int64_t src, dst;
};
__device__ inline PackItem pack_item(uint32_t g, uint32_t n_slots, const int64_t* piece_begin, const int32_t* counts,
                                     const int64_t* slot_out) {
  PackItem it{0, 0, 0};
  if (g < n_slots) {
    it.k = counts[g];
    it.src = piece_begin[g];
    it.dst = slot_out[g];
  }
  return it;
}
__global__ __launch_bounds__(256) void piece_pack_kernel(const int32_t* tmp_ids, const Control* c,
                                                         const int64_t* piece_begin, const int32_t* counts,
                                                         const int64_t* slot_out, int32_t* out_ids,
                                                         const int32_t* id_map) {
  const uint32_t n_slots = c->n_slots;
  const int lane = threadIdx.x & 63;
  const uint32_t stride = gridDim.x * 4;               // pieces one round of the grid takes: wave w takes w and w + stride
  uint32_t g = blockIdx.x * 4 + (threadIdx.x >> 6);
  PackItem a = pack_item(g, n_slots, piece_begin, counts, slot_out);
  PackItem b = pack_item(g + stride, n_slots, piece_begin, counts, slot_out);
  while (g < n_slots) {
    const uint32_t g_next = g + 2 * stride;
    const PackItem a_next = pack_item(g_next, n_slots, piece_begin, counts, slot_out);
    const PackItem b_next = pack_item(g_next + stride, n_slots, piece_begin, counts, slot_out);
    const int longest = max(a.k, b.k);                 // (per wave: uniform)
    for (int i0 = 0; i0 < longest; i0 += 256) {
      int32_t va[4], vb[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int i = i0 + 64 * u + lane;
        va[u] = i < a.k ? tmp_ids[a.src + i] : 0;
        vb[u] = i < b.k ? tmp_ids[b.src + i] : 0;
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int i = i0 + 64 * u + lane;
        if (i < a.k) out_ids[a.dst + i] = vocabulary_id(id_map, va[u]);
        if (i < b.k) out_ids[b.dst + i] = vocabulary_id(id_map, vb[u]);
      }
    }
    g = g_next;
    a = a_next;
    b = b_next;
  }
}

}  // namespace bpe
