// One lane per segment: the encoder for work items of up to 1 KiB whose segments are short.
//
// A string falls apart at its cuts -- byte bigrams that lie at no merge junction, see table_format.h -- into
// segments that Algorithm 1 processes without any interaction; with word-like text a segment is a word of a
// few bytes.  Inside so short a stretch there is nothing for 64 lanes to share, so here every lane takes a
// whole segment and runs Algorithm 1 on it literally: find the lowest-rank pair (left-most on ties), replace
// it by its merged token, look up the two pairs the new token forms (section 4.2's steps, one lane wide), until
// no pair of the segment is in the table.  The wave as a whole still works on one item (section 4.3: one block
// per string), and a lane that finishes its segment takes the item's next one, so the lanes stay busy whatever
// the mix of segment lengths.
//
//   load     position-parallel: lane t owns bytes [16 t, 16 t + 16) of the item (one 16-byte load), looks up its
//            16 initial pairs in the direct byte-pair table, and writes token words, pair values and the
//            bitmap of segment ends to LDS.
//   list     starts of the segments with at least two bytes, by a prefix sum over the lanes.
//   merge    segment-parallel, as above; a lane keeps its segment's liveness as a 32-bit mask, so a segment
//            may have at most 32 bytes.  An item with a longer segment is not encoded here: the kernel hands
//            it to the wave-per-item encoder of encode_segmented.h, which has no such limit.
//   emit     position-parallel again: prefix sum of the surviving tokens, compaction in LDS, one coalesced
//            store of the ids.
#pragma once
#include "encode_segmented.h"

namespace bpe {

constexpr int kLaneItemBytes = 1024;            // capacity of a work item: 64 lanes x 16 positions
constexpr int kLaneSegmentMax = 32;             // positions a lane's liveness mask covers
constexpr int kLanePad = 32;                    // words after the position arrays that a scan may read

// Pair values as the lanes keep them: rank in bits 12..31 as in the table, the two operand-capability flags
// moved up to bits 6 and 7, bits 0..4 clear so that a position can ride in them through the minimum.
constexpr uint32_t kLaneNoPair = 0xFFFFFFFFu;
constexpr uint32_t kLaneInvalid = 0xFFFFE000u;  // values from here on are no pair (ranks stay below 0xFFFFE)

__device__ inline uint32_t lane_value(uint32_t v) {
  return (v & 0xFFFFF000u) | ((v & (kFlagLeft | kFlagRight)) << 5);
}
__device__ inline uint32_t lane_merged_word(uint32_t lv) {
  static_assert((kFlagLeft << 5 << 24) == kTokCanLeft && (kFlagRight << 5 << 24) == kTokCanRight, "flag positions");
  return (256u + (lv >> kRankShift)) | ((lv & ((kFlagLeft | kFlagRight) << 5)) << 24);
}

// Per-wave LDS, in 32-bit words.
struct LaneLds {
  static constexpr int kT = 0;                                          // token word of every position
  static constexpr int kV = kT + kLaneItemBytes + kLanePad;             // pair value of every position
  static constexpr int kEnds = kV + kLaneItemBytes + kLanePad;          // bit p: position p ends its segment
  static constexpr int kSeg = kEnds + kLaneItemBytes / 32 + 4;          // uint16: first position of each segment
  static constexpr int kWords = kSeg + kLaneItemBytes / 4;
};

struct __attribute__((packed, aligned(1))) Unaligned16 { uint32_t x, y, z, w; };

// 16 bytes from p (any alignment), or the first `count` of them where the buffer ends before p + 16.
__device__ inline void load_bytes16(const uint8_t* p, int count, bool whole, uint32_t (&w)[5]) {
  w[0] = w[1] = w[2] = w[3] = 0;
  if (count <= 0) return;
  if (whole) {
    const Unaligned16 v = *(const Unaligned16*)p;
    w[0] = v.x; w[1] = v.y; w[2] = v.z; w[3] = v.w;
  } else {
#pragma unroll
    for (int j = 0; j < 16; ++j)
      if (j < count) w[j >> 2] |= (uint32_t)p[j] << (8 * (j & 3));
  }
}

__device__ inline uint32_t byte_of(const uint32_t (&w)[5], int j) { return (w[j >> 2] >> (8 * (j & 3))) & 0xFFu; }

// Encodes item s if all its segments fit a lane; returns false (and has written nothing to global memory) if
// one does not.  lds: this wave's LaneLds words; byte_word: the 256 token words of the bytes, in LDS.
template <bool SPECIAL>
__device__ bool encode_item_lanes(const EncodeParams& p, int s, uint32_t* lds, const uint32_t* byte_word) {
  const int lane = (int)threadIdx.x & 63;
  const DeviceTable& tab = p.table;
  uint32_t* const T = lds + LaneLds::kT;
  uint32_t* const V = lds + LaneLds::kV;
  uint32_t* const ends = lds + LaneLds::kEnds;
  uint16_t* const seg = (uint16_t*)(lds + LaneLds::kSeg);

  const int64_t begin = p.piece_begin ? p.piece_begin[s] : p.offsets[s];
  const int n = (int)uniform((uint32_t)(p.piece_len ? p.piece_len[s] : (int32_t)(p.offsets[s + 1] - begin)));
  if (n <= 0 || n > kLaneItemBytes) {                  // uniform; too long only if max_len was wrong
    if (lane == 63) p.counts[s] = 0;
    return true;
  }

  // ---- load: byte-level pre-tokenisation (section 4.1) and the initial pair values ----
  const int base = lane * 16;
  int c = n - base;                                    // my byte count
  c = c < 0 ? 0 : (c > 16 ? 16 : c);
  int np = n - 1 - base;                               // pairs that start at my positions
  np = np < 0 ? 0 : (np > 16 ? 16 : np);
  uint32_t w[5], mk[5];
  const bool whole = begin + base + 16 <= p.total_bytes;
  load_bytes16(p.bytes + begin + base, c, whole, w);
  w[4] = wave_shift_down(w[0], 0u);                    // the next lane's first byte is my 17th
  if constexpr (SPECIAL) {
    load_bytes16(p.cover + begin + base, c, whole, mk);
    mk[4] = wave_shift_down(mk[0], 0u);
  }
  uint32_t raw[16];
#pragma unroll
  for (int j = 0; j < 16; ++j) {
    // index (byte j) << 8 | (byte j + 1): two adjacent bytes, swapped, from the dword pair that holds them
    constexpr uint32_t kSel[4] = {0x0c0c0001u, 0x0c0c0102u, 0x0c0c0203u, 0x0c0c0304u};
    const uint32_t idx = __builtin_amdgcn_perm(w[(j >> 2) + 1], w[j >> 2], kSel[j & 3]) & 0xFFFFu;
    raw[j] = j < np ? tab.byte_pair[idx] : kCut;       // the item's last byte ends a segment
  }
  uint32_t cutmask = 0;                                // bit j: my position j is the last of its segment
  {
    uint32_t tv[16], tt[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      uint32_t v = raw[j];
      uint32_t word = j < c ? byte_word[byte_of(w, j)] : kTokNone;
      if constexpr (SPECIAL) {
        // an occurrence of a special token is one token on its first byte and nothing on the others; no pair
        // involves it, so there is a cut on both sides of every marked byte
        const uint32_t m0 = byte_of(mk, j), m1 = byte_of(mk, j + 1);
        if (j < c && m0) word = (m0 & kCoverFirst) ? p.special_base + (m0 & kCoverIndex) : kTokNone;
        if (m0 | m1) v = kCut;
      }
      cutmask |= (v == kCut ? 1u : 0u) << j;
      tv[j] = lane_value(v);
      tt[j] = word;
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      ((uint4*)(T + base))[q] = make_uint4(tt[4 * q], tt[4 * q + 1], tt[4 * q + 2], tt[4 * q + 3]);
      ((uint4*)(V + base))[q] = make_uint4(tv[4 * q], tv[4 * q + 1], tv[4 * q + 2], tv[4 * q + 3]);
    }
  }
  // 32 aligned positions without a segment end: some segment is longer than a lane can take
  const uint64_t no_end = __ballot(c == 16 && cutmask == 0);
  if (no_end & (no_end >> 1)) return false;
  {
    const uint32_t other = dpp<kDppQuadXor1>(cutmask);                   // the mask of the lane I pair up with
    if ((lane & 1) == 0) ends[lane >> 1] = cutmask | (other << 16);
    if (lane < 4) ends[kLaneItemBytes / 32 + lane] = 0xFFFFFFFFu;        // a window never runs past the item
  }

  // ---- list: first positions of the segments that have a pair to look at (two bytes or more) ----
  uint32_t n_segments;
  {
    const uint32_t before = wave_shift_up(cutmask >> 15, 1u);            // the item's first byte starts a segment
    const uint32_t starts = ((cutmask << 1) | before) & 0xFFFFu & ~cutmask;   // not those that end where they start
    const uint32_t count = (uint32_t)__builtin_popcount(starts);
    const uint32_t inc = wave_scan<OpAdd>(count, 0u);
    n_segments = (uint32_t)__builtin_amdgcn_readlane((int)inc, 63);
    uint32_t at = inc - count;
    for (uint32_t m = starts; m; m &= m - 1) seg[at++] = (uint16_t)(base + __builtin_ctz(m));
  }
  __syncthreads();                                     // one wave: orders the LDS traffic of the phases

  // ---- merge: Algorithm 1 on one segment per lane ----
  uint32_t dead = 0xFFFFFFFFu;     // bit o: position o of my segment holds no token; all ones: I have no segment
  uint32_t s4 = 0;                 // byte offset of my segment's first position in T and V
  uint32_t next = 0;               // first segment nobody has taken (uniform)
  bool too_long = false;
  // Every trip ends a segment or removes a token in each lane that has a segment, so 2 n trips cannot be needed;
  // the bound only guarantees that the loop ends whatever the memory contents.
  for (int trip = 0; trip < 2 * n + 64; ++trip) {
    {
      const bool idle = dead == 0xFFFFFFFFu;
      const uint64_t idle_lanes = __ballot(idle);
      if (idle_lanes && next < n_segments) {           // uniform
        const uint32_t mine = next + __builtin_amdgcn_mbcnt_hi((uint32_t)(idle_lanes >> 32),
                                                               __builtin_amdgcn_mbcnt_lo((uint32_t)idle_lanes, 0u));
        next += (uint32_t)__builtin_popcountll(idle_lanes);
        if (idle && mine < n_segments) {
          const uint32_t first = seg[mine];
          // the segment ends at the first set bit of the ends bitmap from `first` on
          const uint32_t window = __builtin_amdgcn_alignbit(ends[(first >> 5) + 1], ends[first >> 5], first & 31u);
          too_long |= window == 0;
          const uint32_t len = window ? (uint32_t)__builtin_ctz(window) + 1u : 1u;
          dead = len >= 32u ? 0u : 0xFFFFFFFFu << len;
          s4 = first * 4u;
        }
      }
    }
    if (__ballot(too_long)) return false;              // (nothing has left LDS yet)
    if (!__ballot(dead != 0xFFFFFFFFu)) break;         // every segment is done

    // the lowest value among my live pairs, left-most on ties: the position rides in the low bits
    const uint32_t* vp = (const uint32_t*)((const char*)V + s4);
    uint32_t best = 0xFFFFFFFFu;
#pragma unroll
    for (int g = 0; g < kLaneSegmentMax; g += 8) {
      if (g == 0 || __ballot((~dead >> g) != 0)) {     // uniform: some lane's segment reaches this far
#pragma unroll
        for (int o = g; o < g + 8; ++o)
          best = min(best, vp[o] | (uint32_t)o | (uint32_t)__builtin_amdgcn_sbfe((int)dead, o, 1));
      }
    }
    const bool merge = best < kLaneInvalid;
    if (!merge) dead = 0xFFFFFFFFu;                    // no pair left: my segment is finished
    if (__ballot(merge)) {
      uint32_t x1 = 0, y1 = kTokNone, x2 = 0, y2 = kTokNone;
      uint32_t* left_v = V;
      uint32_t* here_v = V;
      bool has_left = false;
      if (merge) {
        const uint32_t k = best & 31u;
        const uint32_t word = lane_merged_word(best);
        const uint32_t alive = ~dead;
        const uint32_t upper = alive & (0xFFFFFFFEu << k);         // not empty: the pair has a right token
        const uint32_t r = (uint32_t)__builtin_ctz(upper);
        const uint32_t after = upper & (upper - 1u);               // live positions beyond the right token
        const uint32_t lower = alive & ((1u << k) - 1u);
        uint32_t* const t0 = (uint32_t*)((char*)T + s4);
        uint32_t* const v0 = (uint32_t*)((char*)V + s4);
        dead |= 1u << r;
        t0[k] = word;
        t0[r] = kTokNone;
        v0[r] = kLaneNoPair;
        here_v = v0 + k;
        x2 = word;
        if (after) y2 = t0[__builtin_ctz(after)];
        if (lower) {
          const uint32_t l = 31u - (uint32_t)__builtin_clz(lower);
          has_left = true;
          left_v = v0 + l;
          x1 = t0[l];
          y1 = word;
        }
      }
      // the two pairs the merged token forms (none where it has no neighbour): both look-ups in flight
      ProbeInFlight f1, f2;
      probe_start(tab, x1, y1, has_left, f1);
      probe_start(tab, x2, y2, merge, f2);
      const uint32_t r1 = probe_finish(tab, f1), r2 = probe_finish(tab, f2);
      if (merge) {
        if (has_left) *left_v = lane_value(r1);
        *here_v = lane_value(r2);
      }
    }
  }
  __syncthreads();

  // ---- emit: prefix sum of the surviving tokens (section 4.3's compaction), ids packed in LDS, one store ----
  {
    uint32_t tok[16];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const uint4 t = ((const uint4*)(T + base))[q];
      tok[4 * q] = t.x; tok[4 * q + 1] = t.y; tok[4 * q + 2] = t.z; tok[4 * q + 3] = t.w;
    }
    uint32_t count = 0;
#pragma unroll
    for (int j = 0; j < 16; ++j) count += tok[j] != kTokNone ? 1u : 0u;
    const uint32_t inc = wave_scan<OpAdd>(count, 0u);
    const uint32_t total = (uint32_t)__builtin_amdgcn_readlane((int)inc, 63);
    uint32_t at = inc - count;
    uint32_t* const out = V;                           // the pair values are no longer needed
    __syncthreads();
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      if (tok[j] != kTokNone) out[at++] = tok[j] & kTokIdMask;
    }
    __syncthreads();
    int32_t* dst = p.tmp_ids + begin;
    for (uint32_t i = (uint32_t)lane; i < total; i += 64) dst[i] = (int32_t)out[i];
    if (lane == 63) p.counts[s] = (int32_t)total;
    __syncthreads();                                   // LDS is reused by the next item
  }
  return true;
}

// Persistent one-wave workgroups over the items of tier 0 (see encode_kernel for the work queue).  An item with
// a segment that no lane can take goes to the wave-per-item encoder: in this kernel when INLINE (the launch
// that has no work list and no kernel after it to pick such items up), else through p.fallback_list.
template <bool SPECIAL, bool INLINE>
__global__ __launch_bounds__(64) void encode_lanes_kernel(EncodeParams p) {
  extern __shared__ uint32_t smem[];
  uint32_t* const byte_word = smem;                    // [256], then the per-item arrays
  uint32_t* const arrays = smem + 256;
  for (int i = (int)threadIdx.x; i < 256; i += 64) byte_word[i] = p.table.byte_word[i];

  // warm this XCD's L2 with the merge table (see encode_kernel)
  if (p.prefetch_lines > 0) {
    constexpr uint32_t kXcds = 8;
    const uint32_t peers = (gridDim.x + kXcds - 1) / kXcds;
    const uint32_t me = blockIdx.x / kXcds;
    const uint32_t per = (p.prefetch_lines + peers - 1) / peers;
    const uint32_t lo = me * per, hi = min(lo + per, p.prefetch_lines);
    uint32_t sink = 0;
    for (uint32_t line = lo + threadIdx.x; line < hi; line += 64)
      sink |= __builtin_nontemporal_load((const uint32_t*)p.table.buckets + (size_t)line * 32);
    if (sink == 0x9E3779B9u && p.prefetch_lines == 0xFFFFFFFFu) byte_word[0] = sink;   // keeps the loads alive
  }
  __syncthreads();

  const uint32_t first = p.list ? p.tier_base[p.tier] : 0u;
  const uint32_t count = p.list ? p.tier_base[p.tier + 1] - first : p.direct_count;
  uint32_t item = blockIdx.x;
  while (item < count) {
    const int s = p.list ? (int)uniform((uint32_t)p.list[first + item]) : (int)item;
    const bool done = encode_item_lanes<SPECIAL>(p, s, arrays, byte_word);
    if (!done) {                                       // uniform
      if constexpr (INLINE) {
        __syncthreads();
        BlockShared<1> sh;
        uint32_t* cur = arrays + 3 * kLaneItemBytes;
        sh.rec = (WaveRecord*)cur; cur += 2 * 8;
        sh.first_tok = cur; cur += 2;
        sh.part = cur; cur += 2;
        sh.item = cur;
        sh.byte_word = byte_word;
        encode_string_segmented<1, 16, true, SPECIAL>(p, s, arrays, arrays + kLaneItemBytes,
                                                      arrays + 2 * kLaneItemBytes, sh);
      } else {
        // every lane takes part in the atomic (lane 0 adds 1): no lane-dependent branch at the loop's edge
        const uint32_t slot = uniform(atomicAdd(p.fallback_count, threadIdx.x == 0 ? 1u : 0u));
        if (threadIdx.x == 0) p.fallback_list[slot] = s;
      }
    }
    if (gridDim.x >= count) break;                     // uniform: one item per workgroup at most
    const uint32_t claimed = atomicAdd(p.queue_head + p.tier, threadIdx.x == 0 ? 1u : 0u);
    item = gridDim.x + uniform(claimed);               // lane 0's value, as a scalar
  }
}

template <bool INLINE>
constexpr size_t lanes_lds_bytes() {
  constexpr size_t own = 256 + LaneLds::kWords;
  constexpr size_t with_fallback = 256 + 3 * kLaneItemBytes + 24;
  return sizeof(uint32_t) * (INLINE && with_fallback > own ? with_fallback : own);
}

}  // namespace bpe
