// One lane per segment: the encoder for work items of up to 1 KiB whose segments are short.
//
// A string falls apart at its cuts -- byte bigrams that lie at no merge junction, see table_format.h -- into
// segments that Algorithm 1 processes without any interaction; with word-like text a segment is a word of a
// few bytes.  Inside so short a stretch there is nothing for 64 lanes to share, so here every lane takes a
// whole segment and runs Algorithm 1 on it literally: find the lowest-rank pair (left-most on ties), replace
// it by its merged token, look up the two pairs the new token forms (section 4.2's steps, one lane wide), until
// no pair of the segment is in the table.  The wave as a whole still works on one item (section 4.3: one block
// per string), and a lane that finishes its segment takes the item's next one, longer segments first, so the
// lanes stay busy whatever the mix of segment lengths.
//
//   load     position-parallel, one row of 64 consecutive bytes at a time: lane t holds byte 64 j + t of row j
//            (coalesced byte loads, conflict-free LDS traffic), looks its pair with the next byte up in the direct
//            byte-pair table, and a ballot of "this pair is a cut" is the row's piece of the segment-end bitmap.
//   list     the segments with at least two bytes (first position and length), from the same ballots, then sorted
//            by length, longest first: a counting sort with one LDS counter per length.  Handing the long
//            segments out first is what keeps the lanes level at the end of an item (a third fewer trips of the
//            merge loop than in text order).
//   merge    segment-parallel, as above; a lane keeps its segment's liveness as a 32-bit mask, so a segment
//            may have at most 32 bytes.  An item with a longer segment is not encoded here: the kernel hands
//            it to the wave-per-item encoder of encode_segmented.h, which has no such limit.
//   emit     row by row again: a ballot of the surviving tokens gives every lane its place in the output
//            (section 4.3's compaction, as a prefix count over the ballots), and the ids go out in order.
#pragma once
#include "encode_segmented.h"

namespace bpe {

constexpr int kLaneItemBytes = 1024;            // capacity of a work item
constexpr int kLaneRows = kLaneItemBytes / 64;
constexpr int kLaneSegmentMax = 32;             // positions a lane's liveness mask covers
constexpr uint32_t kLaneChunk = 4;              // work items a workgroup claims at a time (1: 3.4 ms on the
                                                // 270,000 pieces of the throughput workload, 2: 2.2, 4: 2.1, 8: 2.1);
                                                // twice as many when the list holds 32 or more items per workgroup

// Pair values as the lanes keep them: the table's value (rank in bits 12..31, the two operand-capability flags
// in bits 10 and 11) with the bits below cleared, so that a position can ride in them through the minimum.
constexpr uint32_t kLaneNoPair = 0xFFFFFFFFu;
constexpr uint32_t kLaneInvalid = 0xFFFFE000u;  // values from here on are no pair (ranks stay below 0xFFFFE)

__device__ inline uint32_t lane_value(uint32_t v) { return v & ~((1u << 10) - 1u); }
__device__ inline uint32_t lane_merged_word(uint32_t lv) {
  static_assert(kFlagLeft == 1u << 10 && kFlagRight == 1u << 11 && (kFlagLeft << 20) == kTokCanLeft &&
                (kFlagRight << 20) == kTokCanRight, "flag positions");
  return (256u + (lv >> kRankShift)) | ((lv & (kFlagLeft | kFlagRight)) << 20);
}

// Per-wave LDS, in 32-bit words.  (9.3 KB: sixteen workgroups per CU, four waves per SIMD.)
struct LaneLds {
  static constexpr int kFlags = 0;                                      // 2 bits per byte value: can be a left / right operand
  static constexpr int kT = kFlags + 16;                                // token word of every position
  static constexpr int kV = kT + kLaneItemBytes;                        // pair value of every position; a scan may
  static constexpr int kEnds = kV + kLaneItemBytes;                     //   read up to 31 words on (masked out)
  static constexpr int kSeg = kEnds + kLaneItemBytes / 32 + 4;          // bit p of kEnds: position p ends its segment
  static constexpr int kHist = kSeg + kLaneItemBytes / 4;               // kSeg: uint16 first position | (length - 1) << 10
  static constexpr int kWords = kHist + 32;                             // kHist: segments of each length, then list bases
};

__device__ inline uint32_t mbcnt64(uint64_t mask) {                     // set bits of mask below my lane
  return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

// Encodes item s -- n bytes from `begin` on (both uniform) -- if all its segments fit a lane; returns false (and
// has written nothing to global memory) if one does not.  lds: this wave's LaneLds words (kFlags filled in by the
// kernel).
template <bool SPECIAL>
__device__ __forceinline__ bool encode_item_lanes(const EncodeParams& p, int s, int64_t begin, int n, uint32_t* lds) {
  const int lane = (int)threadIdx.x & 63;
  const DeviceTable& tab = p.table;
  uint32_t* const T = lds + LaneLds::kT;
  uint32_t* const V = lds + LaneLds::kV;
  uint32_t* const ends = lds + LaneLds::kEnds;
  uint16_t* const seg = (uint16_t*)(lds + LaneLds::kSeg);
  uint32_t* const hist = lds + LaneLds::kHist;

  if (n <= 0 || n > kLaneItemBytes) {                  // uniform; too long only if max_len was wrong
    if (lane == 63) p.counts[s] = 0;
    return true;
  }
  const int rows = (n + 63) >> 6;                      // uniform
  __builtin_amdgcn_s_setprio(3);                       // (the load phase too is a chain of round trips, and the
                                                       // sooner its loads go out the better)

  // ---- load: byte-level pre-tokenisation (section 4.1), the initial pair values, segment ends and starts ----
  uint32_t n_segments = 0;                             // segments with a pair to look at (uniform)
  {
    const uint8_t* src = p.bytes + begin + lane;
    uint32_t b[kLaneRows + 1], mk[kLaneRows + 1];
#pragma unroll
    for (int j = 0; j < kLaneRows; ++j) {
      b[j] = 0;
      mk[j] = 0;
      if (j < rows && 64 * j + lane < n) {
        b[j] = src[64 * j];
        if constexpr (SPECIAL) mk[j] = p.cover[begin + lane + 64 * j];
      }
    }
    b[kLaneRows] = mk[kLaneRows] = 0;
    uint32_t raw[kLaneRows];
    uint32_t word[kLaneRows];
#pragma unroll
    for (int j = 0; j < kLaneRows; ++j) {
      raw[j] = kCut;
      word[j] = kTokNone;
      if (j < rows) {                                  // uniform
        // the byte after mine: the next lane's of this row, or for the last lane the first of the next row
        uint32_t nb = wave_shift_down(b[j], 0u);
        const uint32_t wrap = (uint32_t)__builtin_amdgcn_readlane((int)b[j + 1], 0);
        nb = lane == 63 ? wrap : nb;
        const bool has_pair = 64 * j + lane + 1 < n;
        if (has_pair) raw[j] = tab.byte_pair[(b[j] << 8) | nb];          // (the item's last byte ends a segment)
        // token word of a byte: its value and the two capability bits (bits 30 and 31) from the packed table
        word[j] = b[j] | (((lds[LaneLds::kFlags + (b[j] >> 4)] >> (2u * (b[j] & 15u))) & 3u) << 30);
        if constexpr (SPECIAL) {
          // an occurrence of a special token is one token on its first byte and nothing on the others; no
          // pair involves it, so there is a cut on both sides of every marked byte
          uint32_t nm = wave_shift_down(mk[j], 0u);
          const uint32_t wrap_m = (uint32_t)__builtin_amdgcn_readlane((int)mk[j + 1], 0);
          nm = lane == 63 ? wrap_m : nm;
          if (mk[j]) word[j] = (mk[j] & kCoverFirst) ? p.special_base + (mk[j] & kCoverIndex) : kTokNone;
          if (mk[j] | nm) raw[j] = kCut;
        }
      }
    }
    uint64_t carry = 1;                                // the item's first byte starts a segment
#pragma unroll
    for (int j = 0; j < kLaneRows; ++j) {
      if (j < rows) {                                  // uniform
        const int pos = 64 * j + lane;
        const uint64_t end_row = __ballot(raw[j] == kCut);               // positions >= n - 1 included
        T[pos] = pos < n ? word[j] : kTokNone;
        V[pos] = lane_value(raw[j]);
        if (lane == 0) *(uint64_t*)(ends + 2 * j) = end_row;
        // segments that start in this row and hold a pair: after an end, and not an end themselves
        const uint64_t start_row = ((end_row << 1) | carry) & ~end_row;
        carry = end_row >> 63;
        if ((start_row >> lane) & 1ull) seg[n_segments + mbcnt64(start_row)] = (uint16_t)pos;
        n_segments += (uint32_t)__builtin_popcountll(start_row);
      }
    }
    if (lane < 4) ends[2 * rows + lane] = 0xFFFFFFFFu;                   // a window never runs past the item
    if (lane < 32) hist[lane] = 0;
  }
  __syncthreads();                                     // one wave: orders the LDS traffic of the phases

  __builtin_amdgcn_s_setprio(0);
  // ---- list, sorted: longest segments first (counting sort over the 31 possible lengths) ----
  {
    constexpr int kRounds = kLaneItemBytes / 2 / 64;   // at most 512 segments of two bytes
    uint32_t entry[kRounds], place[kRounds];
    bool too_long = false;
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
      entry[r] = 0;
      place[r] = 0;
      if ((uint32_t)(64 * r) < n_segments) {           // uniform
        const uint32_t i = 64u * r + (uint32_t)lane;
        if (i < n_segments) {
          const uint32_t first = seg[i];
          // the segment ends at the first set bit of the ends bitmap from `first` on
          const uint32_t window = __builtin_amdgcn_alignbit(ends[(first >> 5) + 1], ends[first >> 5], first & 31u);
          too_long |= window == 0;
          const uint32_t len = window ? (uint32_t)__builtin_ctz(window) + 1u : 2u;      // 2..32
          entry[r] = first | ((len - 1u) << 10);
          place[r] = atomicAdd(&hist[32u - len], 1u);  // my place among the segments of my length
        }
      }
    }
    if (__ballot(too_long)) return false;              // a segment no lane can take (nothing has left LDS)
    __syncthreads();
    {
      const uint32_t mine = lane < 32 ? hist[lane] : 0u;
      const uint32_t inc = wave_scan<OpAdd>(mine, 0u);
      __syncthreads();
      if (lane < 32) hist[lane] = inc - mine;          // where the segments of length 32 - lane start
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
      if ((uint32_t)(64 * r) < n_segments) {           // uniform
        if (64u * r + (uint32_t)lane < n_segments)
          seg[hist[31u - (entry[r] >> 10)] + place[r]] = (uint16_t)entry[r];
      }
    }
  }
  __syncthreads();

  // ---- merge: Algorithm 1 on one segment per lane ----
  // The look-ups of the two pairs a merge creates stay in flight over the loop's edge: the next trip first scans
  // the pair values that did not change and only then takes the two new ones.
  uint32_t dead = 0xFFFFFFFFu;     // bit o: position o of my segment holds no token; all ones: I have no segment
  uint32_t* t0 = T;                // my segment's first position in T ...
  uint32_t* v0 = V;                // ... and in V
  uint32_t next = 0;               // first segment nobody has taken (uniform)
  ProbeInFlight f1, f2;            // (left token, merged token) and (merged token, token after it)
  f1.q = f2.q = make_uint4(0, 0, 0, 0);
  f1.pl.bucket = f1.pl.fingerprint = f2.pl.bucket = f2.pl.fingerprint = 0;
  f1.live = f2.live = false;
  bool pending = false, pending_left = false;          // look-ups of my last merge are in flight
  uint32_t hold = 0;               // positions whose pair value is being looked up
  uint32_t pk = 0, pl = 0;         // ... the merged token's position and its left neighbour's
  // Every trip ends a segment or removes a token in each lane that has a segment, so 2 n trips cannot be needed;
  // the bound only guarantees that the loop ends whatever the memory contents.
  // A lane without a segment takes the next one of the list.
  auto take_segments = [&]() {
    const bool idle = dead == 0xFFFFFFFFu;             // (an idle lane has nothing in flight)
    const uint64_t idle_lanes = __ballot(idle);
    if (idle_lanes && next < n_segments) {             // uniform
      const uint32_t mine = next + mbcnt64(idle_lanes);
      next += (uint32_t)__builtin_popcountll(idle_lanes);
      if (idle && mine < n_segments) {
        const uint32_t e = seg[mine];
        const uint32_t first = e & 1023u, len = (e >> 10) + 1u;
        dead = len >= 32u ? 0u : 0xFFFFFFFFu << len;
        t0 = T + first;
        v0 = V + first;
      }
    }
  };
  take_segments();
#pragma unroll 2                   // (measured: 1.5 % faster than the rolled loop; 3 and 4 are not)
  for (int trip = 0; trip < 2 * n + 64; ++trip) {
    if (!__ballot(dead != 0xFFFFFFFFu)) break;         // every segment is done

    // the lowest value among my live pairs, left-most on ties: the position rides in the low bits
    uint32_t best = 0xFFFFFFFFu;
    {
      const uint32_t skip = dead | hold;
#pragma unroll
      // (two halves: gating by eights or fours costs more in branches than it saves in positions, and no
      // gating at all costs 15 %: one trip in five has a lane with a token beyond position 16)
      for (int g = 0; g < kLaneSegmentMax; g += 16) {
        if (g == 0 || __ballot((~dead >> g) != 0)) {   // uniform: some lane's segment reaches this far
#pragma unroll
          for (int o = g; o < g + 16; ++o)
            best = min(best, v0[o] | (uint32_t)o | (uint32_t)__builtin_amdgcn_sbfe((int)skip, o, 1));
        }
      }
    }
    // From here to the issue of the new look-ups a wave is on its way to its next memory round trip: it goes
    // before the waves that are scanning or loading (measured: 1 % on the large workloads).
    __builtin_amdgcn_s_setprio(2);
    {                                                  // the two pairs my last merge created (no "if any lane":
                                                       // nearly every trip has one, and the branch costs more)
      const uint32_t r1 = probe_finish(tab, f1), r2 = probe_finish(tab, f2);
      if (pending) {
        const uint32_t here = lane_value(r2);
        v0[pk] = here;
        best = min(best, here | pk);
        if (pending_left) {
          const uint32_t left = lane_value(r1);
          v0[pl] = left;
          best = min(best, left | pl);
        }
      }
    }
    const bool merge = best < kLaneInvalid;
    if (!merge) dead = 0xFFFFFFFFu;                    // no pair left: my segment is finished
    pending = merge;
    pending_left = false;
    hold = 0;
    {
      uint32_t x1 = 0, y1 = kTokNone, x2 = 0, y2 = kTokNone;
      if (merge) {
        const uint32_t k = best & 31u;
        const uint32_t word = lane_merged_word(best);
        const uint32_t alive = ~dead;
        const uint32_t upper = alive & (0xFFFFFFFEu << k);         // not empty: the pair has a right token
        const uint32_t r = (uint32_t)__builtin_ctz(upper);
        const uint32_t after = upper & (upper - 1u);               // live positions beyond the right token
        const uint32_t lower = alive & ((1u << k) - 1u);
        dead |= 1u << r;
        t0[k] = word;
        t0[r] = kTokNone;
        pk = k;
        hold = 1u << k;
        x2 = word;
        if (after) y2 = t0[__builtin_ctz(after)];
        if (lower) {
          pl = 31u - (uint32_t)__builtin_clz(lower);
          pending_left = true;
          hold |= 1u << pl;
          x1 = t0[pl];
          y1 = word;
        }
        if (!(after | lower)) {                                    // the merged token is all that is left of the
          dead = 0xFFFFFFFFu;                                      // segment (two segments in three end like this):
          pending = false;                                         // finished, without a trip that finds no pair
          hold = 0;
        }
      }
      probe_start(tab, x1, y1, pending_left, f1);
      probe_start(tab, x2, y2, merge, f2);
    }
    take_segments();                                   // lanes whose segment just ended go on at once
    __builtin_amdgcn_s_setprio(0);
  }
  __syncthreads();

  // ---- emit: the surviving tokens in order; a ballot per row gives every lane its place ----
  {
    int32_t* const dst = p.tmp_ids + begin;
    uint32_t total = 0;                                // uniform
#pragma unroll
    for (int j = 0; j < kLaneRows; ++j) {
      if (j < rows) {                                  // uniform
        const uint32_t tok = T[64 * j + lane];         // (positions from n on hold "no token")
        const uint64_t live_row = __ballot(tok != kTokNone);
        if (tok != kTokNone) dst[total + mbcnt64(live_row)] = (int32_t)(tok & kTokIdMask);
        total += (uint32_t)__builtin_popcountll(live_row);
      }
    }
    if (lane == 63) p.counts[s] = (int32_t)total;
    __syncthreads();                                   // LDS is reused by the next item
  }
  return true;
}

// Persistent one-wave workgroups over the items of tier 0.  An item with a segment that no lane can take goes to
// the wave-per-item encoder: in this kernel when INLINE (the launch that has no work list and no
// kernel after it to pick such items up), else through p.fallback_list.
template <bool SPECIAL, bool INLINE>
__global__ __launch_bounds__(64) void encode_lanes_kernel(EncodeParams p) {
  extern __shared__ uint32_t smem[];
  uint32_t* const arrays = smem;                       // this wave's LaneLds
  const uint32_t first = p.list ? p.tier_base[p.tier] : 0u;
  const uint32_t count = p.list ? p.tier_base[p.tier + 1] - first : p.direct_count;
  // items per claim: as many as keep every workgroup of the grid busy, kLaneChunk at most
  // The workgroups that take part: as many as make the rounds even.  5,120 items on 4,096 resident workgroups
  // are two rounds of 2,560 -- the same two item times, with fewer waves sharing each SIMD.
  const uint32_t rounds = (count + gridDim.x - 1) / gridDim.x;
  const uint32_t g = rounds ? (count + rounds - 1) / rounds : 1u;
  const uint32_t per_claim = min(count / g >= 32u ? 2u * kLaneChunk : kLaneChunk, max(1u, count / g));
  if (blockIdx.x >= g || (uint64_t)blockIdx.x * per_claim >= count) return;   // uniform: nothing for this workgroup
  // the capability bits of the 256 byte tokens, packed 16 bytes to a word
  if (threadIdx.x < 16) arrays[LaneLds::kFlags + threadIdx.x] = 0;
  __syncthreads();
  {
    uint32_t bits = 0;
    for (int k = 0; k < 4; ++k) bits |= (p.table.byte_word[4 * threadIdx.x + k] >> 30) << (2 * k);
    atomicOr(&arrays[LaneLds::kFlags + (threadIdx.x >> 2)], bits << (8 * (threadIdx.x & 3)));
  }
  uint32_t* const byte_word = smem + LaneLds::kWords;  // INLINE only: the byte token words for the other encoder
  if constexpr (INLINE)
    for (int i = (int)threadIdx.x; i < 256; i += 64) byte_word[i] = p.table.byte_word[i];
  __syncthreads();

  // Items are claimed kLaneChunk at a time: the first chunk of a workgroup is its own index, later ones come from
  // the tier's queue head (which starts at zero).  One claim per item would make every wave wait for a round trip
  // to the one contended address after each item.  Lane i fetches the descriptor of the chunk's i-th item, so a
  // chunk costs one round trip for its claim and one for its descriptors.  (Claiming ahead does not pay: loads
  // return in order, so whatever is loaded after the claim waits for it.)
  const int lane = (int)threadIdx.x & 63;
  const ItemDesc* const descs = (const ItemDesc*)p.list_desc;
  auto load_chunk = [&](uint64_t first_item, uint32_t n_items, ItemDesc& d) {
    d.begin = 0;
    d.len = 0;
    d.item = 0;
    const uint64_t item = first_item + (uint32_t)lane;
    if ((uint32_t)lane < n_items) {
      if (descs) {
        d = descs[first + item];
      } else {                                         // no work list: item i is string i
        d.begin = p.offsets[item];
        d.len = (int32_t)(p.offsets[item + 1] - d.begin);
        d.item = (int32_t)item;
      }
    }
  };
  auto encode_chunk = [&](uint32_t here, const ItemDesc& cur) __attribute__((always_inline)) {
    for (uint32_t i = 0; i < here; ++i) {
      const int s = __builtin_amdgcn_readlane(cur.item, (int)i);
      const int n = __builtin_amdgcn_readlane(cur.len, (int)i);
      const int64_t begin = ((int64_t)__builtin_amdgcn_readlane((int)(cur.begin >> 32), (int)i) << 32) |
                            (uint32_t)__builtin_amdgcn_readlane((int)cur.begin, (int)i);
      const bool done = encode_item_lanes<SPECIAL>(p, s, begin, n, arrays);
      if (!done) {                                     // uniform
        if constexpr (INLINE) {
          __syncthreads();
          BlockShared<1> sh;
          uint32_t* const other = byte_word + 256;     // the other encoder's arrays lie behind this one's
          uint32_t* cur_word = other + 3 * kLaneItemBytes;
          sh.rec = (WaveRecord*)cur_word; cur_word += 2 * 8;
          sh.first_tok = cur_word; cur_word += 2;
          sh.part = cur_word; cur_word += 2;
          sh.item = cur_word;
          sh.byte_word = byte_word;
          encode_string_segmented<1, 16, true, SPECIAL>(p, s, other, other + kLaneItemBytes,
                                                        other + 2 * kLaneItemBytes, sh);
        } else {
          // every lane takes part in the atomic (lane 0 adds 1): no lane-dependent branch at the loop's edge
          const uint32_t slot = uniform(atomicAdd(p.fallback_count, threadIdx.x == 0 ? 1u : 0u));
          if (threadIdx.x == 0) p.fallback_list[slot] = s;
        }
      }
    }
  };
  // A workgroup's own first chunk: per_claim items, and when the list is long zero to three more, by block index,
  // so that the workgroups do not all come back for their first claim at the same moment (claims on one address
  // are served one after the other, some ten nanoseconds each).
  const uint32_t spread = per_claim >= kLaneChunk ? 1u : 0u;
  const uint32_t b = blockIdx.x;
  constexpr uint32_t kBefore[4] = {0, 0, 1, 3};        // extra items of the blocks before b within its group of four
  uint64_t first_item = (uint64_t)b * per_claim + spread * ((b >> 2) * 6u + kBefore[b & 3u]);
  const uint64_t own_items = (uint64_t)g * per_claim + spread * ((g >> 2) * 6u + kBefore[g & 3u]);
  if (first_item >= count) return;                     // uniform
  uint32_t here = (uint32_t)min((uint64_t)(per_claim + spread * (b & 3u)), count - first_item);
  ItemDesc cur;
  load_chunk(first_item, here, cur);
  for (;;) {
    encode_chunk(here, cur);
    if (own_items >= count) break;                     // uniform: the grid's own chunks cover the list
    // (lane 0 adds 1; every lane takes part, so that no lane-dependent branch sits at the loop's edge)
    const uint32_t claimed = atomicAdd(p.queue_head + p.tier, threadIdx.x == 0 ? 1u : 0u);
    first_item = own_items + (uint64_t)uniform(claimed) * per_claim;
    if (first_item >= count) break;                    // uniform
    here = (uint32_t)min((uint64_t)per_claim, count - first_item);
    load_chunk(first_item, here, cur);
  }
}

template <bool INLINE>
constexpr size_t lanes_lds_bytes() {
  return lds_blocks(sizeof(uint32_t) * (LaneLds::kWords + (INLINE ? 256 + 3 * kLaneItemBytes + 24 : 0)));
}

}  // namespace bpe
