// Per-string BPE merge kernel for gfx950 (wave64).
//
// One workgroup encodes one string (section 4.3: one block per string) and repeats merge passes until no
// adjacent pair is in the table (section 4.2): every adjacent pair's rank is known, a workgroup minimum
// decides what may merge, the occurrences are marked -- left-most first where they overlap -- and the
// merged tokens are written.
//
// What differs from the paper's kernel, and why it is still Algorithm 1's result:
//
//   * Many ranks per pass.  The paper applies the single lowest rank per pass.  Here a pass takes the
//     workgroup minimum E of limit() over all present pairs (see table_format.h): no pair that can still
//     appear has a rank below E, so the present pairs with rank < E ("candidates") can be settled among
//     themselves.  Algorithm 1 would take them in (rank, position) order, and a candidate is lost only
//     if an adjacent candidate with better priority is applied first.  Candidates form runs; inside a
//     run, going right while ranks do not decrease, the applied ones alternate starting with the run's
//     head (for a self pair such as (a,a) in "aaaa" this is the left-most-first rule).  A candidate whose
//     right neighbour has a strictly lower rank is left for the next pass: by then the neighbour has
//     either consumed it or been consumed itself.  Applying a subset of the merges Algorithm 1 is bound
//     to apply never changes the result, because merges of non-adjacent pairs commute.
//     Passes drop by 4-12x on the benchmark workloads; each pass is one reduction, not one per rank.
//   * No compaction per pass across the workgroup.  Lane `tid` owns the d = ceil(n / W) consecutive byte
//     positions [tid*d, tid*d + d) of its string for the whole encode and keeps its live tokens compacted
//     inside its own column (slot k of lane tid is word k*W + tid: conflict-free in LDS, coalesced in
//     HBM).  A merged token stays with the lane of its left operand.  The paper's prefix-sum compaction
//     (section 4.3) runs once, at the end, to emit the ids.
//   * Ranks are looked up when a pair is created (n-1 initial probes, at most two per merge), never
//     re-probed per pass.
//   * Lanes exchange only boundary data: the value of the previous lane's last pair and of the next
//     lane's first pair, the next lane's first token, and a 2-bit segmented-scan element that carries
//     the parity of a run across lanes.  Inside a wave these travel through ballots and lane permutes
//     (registers only); between waves through one small LDS record per wave.  A one-wave workgroup
//     therefore needs no barrier at all.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>

#include "table_format.h"

namespace bpe {

struct DeviceTable {
  const uint4* buckets;       // one uint4 per bucket
  const uint32_t* byte_word;  // [256] token word (id | capability bits) of each byte
  const uint32_t* byte_pair;  // [256*256] value of the pair (byte a, byte b) at a*256 + b, kNoRank if none
  int log2_buckets;
};

struct EncodeParams {
  DeviceTable table;
  const uint8_t* bytes;
  const int64_t* offsets;
  const int64_t* piece_begin; // when strings are split: first byte of each piece (absolute), else null
  const int32_t* piece_len;   //                         and its length
  const int32_t* list;        // work items (strings or pieces) of all tiers, tier-major, longest first inside a tier
  const uint32_t* tier_base;  // [tiers+1] start of each tier's slice of `list`
  uint32_t* queue_head;       // [tiers] next unclaimed item of each tier
  int32_t* tmp_ids;           // ids of an item are written at tmp_ids[first byte of the item ...]
  int32_t* counts;            // token count of each item
  const void* list_desc;      // ItemDesc of every entry of `list` (begin, length, item), in the same order
  uint32_t* staged;           // HBM staging for the variant whose strings exceed LDS (else null)
  uint32_t prefetch_lines;    // 128-byte lines of table memory to pull into L2 at kernel start (0 = none)
  uint32_t direct_count;      // when `list` is null: items are the strings 0..direct_count-1, one per workgroup
  int tier;
  const uint8_t* cover;       // null, or one mark per input byte: where the special tokens lie (see kCover*)
  uint32_t special_base;      // token number of special 0 (256 + rows)
  int64_t total_bytes;        // size of `bytes`: wide loads must not run past it
  uint32_t* fallback_count;   // lane-per-segment kernel: items it cannot take are counted here ...
  int32_t* fallback_list;     // ... and listed here, for the wave-per-item kernel that runs after it
};

// What the load phases make of them: "byte codes" above the byte values.  Any code >= 0x100 is no byte, so
// the pair on either side of it counts as a cut and is in no table.
constexpr uint32_t kCodeNone = 0x100u;      // outside the string
constexpr uint32_t kCodeRest = 0x200u;      // inside a special occurrence: no token here
constexpr uint32_t kCodeSpecial = 0x400u;   // | index: the occurrence's single token

__device__ inline uint32_t cover_code(uint32_t byte, uint32_t mark) {
  return mark == 0 ? byte : ((mark & kCoverFirst) ? (kCodeSpecial | (mark & kCoverIndex)) : kCodeRest);
}

// ---------------------------------------------------------------------------------------------------
// wave64 primitives

__device__ inline uint32_t uniform(uint32_t v) { return (uint32_t)__builtin_amdgcn_readfirstlane((int)v); }

template <int CTRL>
__device__ inline uint32_t dpp(uint32_t v) {
  return (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, CTRL, 0xF, 0xF, false);
}
constexpr int kDppQuadXor1 = 0xB1;      // quad_perm 1,0,3,2
constexpr int kDppQuadXor2 = 0x4E;      // quad_perm 2,3,0,1
constexpr int kDppHalfMirror = 0x141;   // row_half_mirror
constexpr int kDppRowMirror = 0x140;    // row_mirror

struct OpMin { __device__ static uint32_t apply(uint32_t a, uint32_t b) { return a < b ? a : b; } };
struct OpMax { __device__ static uint32_t apply(uint32_t a, uint32_t b) { return a > b ? a : b; } };

// Reduction over the 64 lanes, uniform (scalar) result.  All lanes must be active.
template <class Op>
__device__ inline uint32_t wave_reduce(uint32_t v) {
  v = Op::apply(v, dpp<kDppQuadXor1>(v));
  v = Op::apply(v, dpp<kDppQuadXor2>(v));
  v = Op::apply(v, dpp<kDppHalfMirror>(v));
  v = Op::apply(v, dpp<kDppRowMirror>(v));   // every lane of a 16-lane row now holds the row's result
  const uint32_t a = (uint32_t)__builtin_amdgcn_readlane((int)v, 0);
  const uint32_t b = (uint32_t)__builtin_amdgcn_readlane((int)v, 16);
  const uint32_t c = (uint32_t)__builtin_amdgcn_readlane((int)v, 32);
  const uint32_t d = (uint32_t)__builtin_amdgcn_readlane((int)v, 48);
  return Op::apply(Op::apply(a, b), Op::apply(c, d));
}

__device__ inline uint32_t lane_read(uint32_t v, int src_lane) { return (uint32_t)__shfl((int)v, src_lane, 64); }

// Inclusive scan over the wave in lane order with DPP row shifts and row broadcasts; `identity` fills the
// lanes a shift has no source for.  combine(left, right) need not commute.
constexpr int kDppRowShr1 = 0x111, kDppRowShr2 = 0x112, kDppRowShr4 = 0x114, kDppRowShr8 = 0x118;
constexpr int kDppRowBcast15 = 0x142, kDppRowBcast31 = 0x143;

template <int CTRL, int ROW_MASK>
__device__ inline uint32_t dpp_or(uint32_t identity, uint32_t v) {
  return (uint32_t)__builtin_amdgcn_update_dpp((int)identity, (int)v, CTRL, ROW_MASK, 0xF, false);
}

template <class Op>
__device__ inline uint32_t wave_scan(uint32_t v, uint32_t identity) {
  v = Op::apply(dpp_or<kDppRowShr1, 0xF>(identity, v), v);
  v = Op::apply(dpp_or<kDppRowShr2, 0xF>(identity, v), v);
  v = Op::apply(dpp_or<kDppRowShr4, 0xF>(identity, v), v);
  v = Op::apply(dpp_or<kDppRowShr8, 0xF>(identity, v), v);   // scan inside each 16-lane row
  v = Op::apply(dpp_or<kDppRowBcast15, 0xA>(identity, v), v); // rows 1 and 3 take the total of the row before
  v = Op::apply(dpp_or<kDppRowBcast31, 0xC>(identity, v), v); // rows 2 and 3 take the total of lanes 0..31
  return v;
}

// Plain unsigned minimum, as an inclusive scan in lane order and as one in reverse lane order (a lane gets the
// minimum over itself and all later lanes).  Each step is one v_min_u32 with a DPP operand, in place: a lane
// that the step has no source for (or whose row is masked off) is simply not written.  The two wait states a
// DPP read needs after the write of the same register are spelled out.
#define BPE_DPP_MIN(v, ctrl) \
  asm volatile("s_nop 1\n\tv_min_u32_dpp %0, %0, %0 " ctrl : "+v"(v))
__device__ inline uint32_t wave_min_prefix(uint32_t v) {
  BPE_DPP_MIN(v, "row_shr:1 row_mask:0xf bank_mask:0xf");
  BPE_DPP_MIN(v, "row_shr:2 row_mask:0xf bank_mask:0xf");
  BPE_DPP_MIN(v, "row_shr:4 row_mask:0xf bank_mask:0xf");
  BPE_DPP_MIN(v, "row_shr:8 row_mask:0xf bank_mask:0xf");    // prefix minima inside each 16-lane row
  BPE_DPP_MIN(v, "row_bcast:15 row_mask:0xa bank_mask:0xf");  // rows 1 and 3 take the total of the row before
  BPE_DPP_MIN(v, "row_bcast:31 row_mask:0xc bank_mask:0xf");  // rows 2 and 3 take the total of lanes 0..31
  return v;
}
// `not_row[r]` is 0 in the lanes of row r and all ones elsewhere (r = 0, 1, 2).
__device__ inline uint32_t wave_min_suffix(uint32_t v, const uint32_t (&not_row)[3]) {
  BPE_DPP_MIN(v, "row_shl:1 row_mask:0xf bank_mask:0xf");
  BPE_DPP_MIN(v, "row_shl:2 row_mask:0xf bank_mask:0xf");
  BPE_DPP_MIN(v, "row_shl:4 row_mask:0xf bank_mask:0xf");
  BPE_DPP_MIN(v, "row_shl:8 row_mask:0xf bank_mask:0xf");    // suffix minima inside each 16-lane row
  const uint32_t t1 = (uint32_t)__builtin_amdgcn_readlane((int)v, 16);   // whole rows 1, 2, 3
  const uint32_t t2 = (uint32_t)__builtin_amdgcn_readlane((int)v, 32);
  const uint32_t t3 = (uint32_t)__builtin_amdgcn_readlane((int)v, 48);
  const uint32_t s2 = min(t2, t3), s1 = min(t1, s2);         // what rows 1 and 0 still have to see
  return min(min(v, s1 | not_row[0]), min(s2 | not_row[1], t3 | not_row[2]));
}
// The value the lane after mine holds (lane 63 receives `identity`).
__device__ inline uint32_t wave_shift_down(uint32_t v, uint32_t identity) {
  return (uint32_t)__builtin_amdgcn_update_dpp((int)identity, (int)v, 0x130, 0xF, 0xF, false);  // wave_shl:1
}

struct OpAdd { __device__ static uint32_t apply(uint32_t a, uint32_t b) { return a + b; } };

// Run-parity element: bit 1 = "a run restarts inside", bit 0 = parity of the run length since the last
// restart (or of the whole span if none).  apply(left, right) is the element of the concatenation.
struct OpParity {
  __device__ static uint32_t apply(uint32_t left, uint32_t right) {
    return (right & 2u) ? right : ((left & 2u) | ((left ^ right) & 1u));
  }
};

// Exclusive scan of run-parity elements over the wave from two ballots instead of a DPP chain: the element of
// the lanes before mine is (some lane before me restarts, parity summed from the last such lane on -- or from
// lane 0 -- up to the lane before me).  *total receives the element of the whole wave.
__device__ inline uint32_t wave_parity_exclusive(uint32_t elem, int lane, uint32_t* total) {
  const uint64_t par = __ballot((elem & 1u) != 0), rst = __ballot((elem & 2u) != 0);
  const uint64_t below = (1ull << lane) - 1ull;
  const uint64_t rb = rst & below;
  const uint64_t from = rb ? (~0ull << (63 - __builtin_clzll(rb))) : ~0ull;
  const uint32_t exc = (uint32_t)(__builtin_popcountll(par & below & from) & 1) | (rb ? 2u : 0u);
  const uint64_t from_all = rst ? (~0ull << (63 - __builtin_clzll(rst))) : ~0ull;     // uniform
  *total = (uint32_t)(__builtin_popcountll(par & from_all) & 1) | (rst ? 2u : 0u);
  return exc;
}

// The value the lane before mine holds (lane 0 receives `identity`).
__device__ inline uint32_t wave_shift_up(uint32_t v, uint32_t identity) {
  return (uint32_t)__builtin_amdgcn_update_dpp((int)identity, (int)v, 0x138, 0xF, 0xF, false);  // wave_shr:1
}

// ---------------------------------------------------------------------------------------------------
// table probe

// The lookup is split in two so that a lane can have several in flight: start() issues the one 16-byte load of
// the home bucket, finish() inspects it (and reads on along the line in the overflow case).
struct ProbeInFlight {
  uint4 q;          // the home bucket: two slots of {value, tag}
  Placement pl;
  bool live;        // false: the capability bits or a missing neighbour already decided "no pair"
};

__device__ inline void probe_start(const DeviceTable& t, uint32_t xw, uint32_t yw, bool wanted, ProbeInFlight& f) {
  f.live = wanted && yw != kTokNone && (xw & kTokCanLeft) && (yw & kTokCanRight);
  if (f.live) {
    f.pl = place_pair(xw & kTokIdMask, yw & kTokIdMask, t.log2_buckets);
    f.q = t.buckets[f.pl.bucket];
  }
}

// Value of the slot whose tag matches, kNoRank if neither does (selects, not branches).
__device__ inline uint32_t match_bucket(const uint4& q, uint32_t tag) {
  uint32_t found = q.y == tag ? q.x : kNoRank;
  return q.w == tag ? q.z : found;
}

__device__ inline uint32_t probe_finish(const DeviceTable& t, const ProbeInFlight& f) {
  uint32_t found = match_bucket(f.q, slot_tag(f.pl.fingerprint, 0));
  if (!f.live) return kNoRank;
  if (found == kNoRank && f.q.w != 0xFFFFFFFFu) {
    // my home bucket is full: keys of it may have been displaced, and mine, if it exists, is then one of them
    const uint32_t reach = bucket_reach(f.q.x, f.q.z);
    for (uint32_t d = 1; d <= reach && found == kNoRank; ++d)
      found = match_bucket(t.buckets[f.pl.bucket ^ d], slot_tag(f.pl.fingerprint, d));
  }
  return found == kNoRank ? kNoRank : (found & ~kValueSpare);
}

// ---------------------------------------------------------------------------------------------------
// workgroup-level exchange (only used when the workgroup has more than one wave)

// What a wave tells the others after each pass.
struct WaveRecord {
  uint32_t limit;      // min limit() over the wave's pairs, kNoRank if it has none
  uint32_t first_val;  // pair value at the wave's first live token (kNoRank if none / wave empty)
  uint32_t last_val;   // pair value at the wave's last live token
  uint32_t first_tok;  // first live token word, kTokNone if the wave is empty
};

template <int NW>
struct BlockShared {
  WaveRecord* rec;       // [2][NW] double buffered by pass parity
  uint32_t* first_tok;   // [2][NW] first live token of each wave after the pass's merges
  uint32_t* part;        // [2][NW] scan partials, double buffered by pass parity
  uint32_t* item;        // [1] work item broadcast
  const uint32_t* byte_word;  // [256] LDS copy of the byte token words
};

template <int NW>
__device__ inline void block_sync() {
  if (NW > 1) __syncthreads();
}

// Exclusive prefix sum of v over the workgroup in lane order; *total receives the sum.
template <int NW>
__device__ inline uint32_t block_prefix_sum(uint32_t v, const BlockShared<NW>& sh, int lane, int wave,
                                            uint32_t* total) {
  const uint32_t inc = wave_scan<OpAdd>(v, 0u);
  const uint32_t wave_total = (uint32_t)__builtin_amdgcn_readlane((int)inc, 63);
  if (NW == 1) {
    *total = wave_total;
    return inc - v;
  }
  __syncthreads();                       // previous users of sh.part are done
  if (lane == 0) sh.part[wave] = wave_total;
  __syncthreads();
  uint32_t before = 0, all = 0;
#pragma unroll
  for (int w = 0; w < NW; ++w) {
    const uint32_t p = sh.part[w];
    if (w < wave) before += p;
    all += p;
  }
  *total = all;
  return before + inc - v;
}

// My wave's record for the coming pass (no-op for a one-wave workgroup).
template <int NW>
__device__ inline void publish_record(const BlockShared<NW>& sh, int buf, int wave, int lane, bool nonempty,
                                      uint32_t llim, uint32_t firstv, uint32_t lastv, uint32_t ftok) {
  if (NW == 1) return;
  const uint64_t ne = __ballot(nonempty);
  const uint32_t wlim = wave_reduce<OpMin>(llim);
  const int fl = ne ? __builtin_ctzll(ne) : 0, ll = ne ? 63 - __builtin_clzll(ne) : 0;
  const uint32_t fv = lane_read(firstv, fl), ft = lane_read(ftok, fl), lv = lane_read(lastv, ll);
  if (lane == 0) {
    WaveRecord r;
    r.limit = wlim;
    r.first_val = ne ? fv : kNoRank;
    r.last_val = ne ? lv : kNoRank;
    r.first_tok = ne ? ft : kTokNone;
    sh.rec[buf * NW + wave] = r;
  }
}

// ---------------------------------------------------------------------------------------------------
// Encode string s.
//
// T, V, L: token word, pair value and pair limit of every byte position of the string (L is kept only by
// the variants with LIMITS; the others decode the limit from V when they need it); position k of lane
// tid is word k*W + tid, in LDS or (strings that exceed LDS) in HBM.  Every word is read and written by its
// owning lane only.  A position is live while its token exists; a merge keeps the merged token at the left
// operand's position and kills the right one, so nothing ever moves.  V[k] is the value of the pair
// (token k, next live token of the string) and L[k] its limit(); dead positions hold kNoRank in both.
//
// A pass costs every lane one sweep over its values (to find the candidates) and then work only per
// candidate; loads are issued in chunks of kChunk positions, cut into groups of kGroup that are skipped
// (scalar branch) beyond the string's bytes-per-lane.

constexpr int kChunk = 16;
constexpr int kGroup = 4;
constexpr int kProbes = 2;     // table probes a lane keeps in flight (measured: 1 is slower; 3, 4 and 8 cost
                               // registers, and with them a wave of occupancy, for no shorter a string)

template <class M> __device__ inline int ctz_bits(M m);
template <> __device__ inline int ctz_bits<uint32_t>(uint32_t m) { return __builtin_ctz(m); }
template <> __device__ inline int ctz_bits<uint64_t>(uint64_t m) { return __builtin_ctzll(m); }
template <class M> __device__ inline int top_bit(M m);
template <> __device__ inline int top_bit<uint32_t>(uint32_t m) { return 31 - __builtin_clz(m); }
template <> __device__ inline int top_bit<uint64_t>(uint64_t m) { return 63 - __builtin_clzll(m); }
template <class M> __device__ inline int pop_bits(M m);
template <> __device__ inline int pop_bits<uint32_t>(uint32_t m) { return __builtin_popcount(m); }
template <> __device__ inline int pop_bits<uint64_t>(uint64_t m) { return __builtin_popcountll(m); }
template <class M> __device__ inline M bit_at(int k) { return (M)1 << k; }
template <class M> __device__ inline M bits_below(int k) { return ((M)1 << k) - 1; }            // k < width
template <class M> __device__ inline M bits_above(int k) { return ~((((M)2) << k) - 1); }        // k < width

template <int NW, int D, bool STAGED, bool LIMITS, bool SPECIAL>
__device__ void encode_string(const EncodeParams& p, int s, uint32_t* __restrict__ T, uint32_t* __restrict__ V,
                              uint32_t* __restrict__ L, const BlockShared<NW>& sh) {
  static_assert(D % kGroup == 0 && D <= 64, "groups must tile the column; positions are a 64-bit mask at most");
  using mask_t = typename std::conditional<(D <= 32), uint32_t, uint64_t>::type;
  constexpr int W = NW * 64;
  const int tid = (int)threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const DeviceTable& tab = p.table;

  // a work item is a whole string, or a piece of one between two cuts
  const int64_t begin = p.piece_begin ? p.piece_begin[s] : p.offsets[s];
  const int n = (int)uniform((uint32_t)(p.piece_len ? p.piece_len[s] : (int32_t)(p.offsets[s + 1] - begin)));
  if (n <= 0 || n > W * D) {                           // uniform branch; too long only if max_len was wrong
    if (tid == W - 1) p.counts[s] = 0;
    return;
  }
  const uint8_t* src = p.bytes + begin;
  const int d = (n + W - 1) / W;                       // bytes per lane, 1 <= d <= D (uniform)
  const int dpad = (d + kGroup - 1) / kGroup * kGroup; // the sweeps read whole groups: pad with dead positions
  int c0 = n - tid * d;                                // my byte count
  c0 = c0 < 0 ? 0 : (c0 > d ? d : c0);

  mask_t live = c0 >= (int)(8 * sizeof(mask_t)) ? ~(mask_t)0 : bits_below<mask_t>(c0);
  uint32_t ftok = kTokNone;                            // my first live token word
  uint32_t succ_tok = kTokNone;                        // the token my last pair is looked up against
  uint32_t firstv = kNoRank, lastv = kNoRank;          // pair values at my first / last live position
  uint32_t llim = kNoRank;                             // min of L over my positions

  // ---- load: byte-level pre-tokenisation (section 4.1), id = byte value; and the initial pair values,
  //      one lookup per adjacent byte pair in the direct 256 x 256 table ----
  {
    const int base = tid * d;
    for (int k0 = 0; k0 < d; k0 += kChunk) {           // d is uniform: no lane leaves the loop early
      uint32_t b[kChunk + 1];
#pragma unroll
      for (int j = 0; j <= kChunk; ++j) {
        const int i = base + k0 + j;
        b[j] = (k0 + j <= c0 && i < n) ? src[i] : 0x100u;   // 0x100: no such byte
      }
      if constexpr (SPECIAL) {                         // special tokens are configured: their marks
        const uint8_t* mark = p.cover + begin;
#pragma unroll
        for (int j = 0; j <= kChunk; ++j) {
          const int i = base + k0 + j;
          if (k0 + j <= c0 && i < n) b[j] = cover_code(b[j], mark[i]);
        }
      }
      uint32_t v[kChunk];
#pragma unroll
      for (int j = 0; j < kChunk; ++j)
        v[j] = (k0 + j < c0 && b[j] < 0x100u && b[j + 1] < 0x100u) ? tab.byte_pair[(b[j] << 8) | b[j + 1]] : kNoRank;
#pragma unroll
      for (int j = 0; j < kChunk; ++j) {
        const int k = k0 + j;
        if (v[j] == kCut) v[j] = kNoRank;              // this variant does not use the segment cuts
        if (k < dpad) {                                // positions from c0 on are dead from the start
          const uint32_t lim = v[j] != kNoRank ? limit_of(v[j]) : kNoRank;
          V[k * W + tid] = v[j];
          if (LIMITS) L[k * W + tid] = lim;
          llim = min(llim, lim);
          if (k < c0) {
            uint32_t w = sh.byte_word[b[j] & 0xFFu];
            if constexpr (SPECIAL) {
              if (b[j] & kCodeSpecial) w = p.special_base + (b[j] & kCoverIndex);
              if (b[j] & kCodeRest) live &= ~bit_at<mask_t>(k);
            }
            T[k * W + tid] = w;
            if (k == 0) { ftok = w; firstv = v[j]; }
            if (k == c0 - 1) {
              lastv = v[j];
              if (b[j + 1] < 0x100u) succ_tok = sh.byte_word[b[j + 1]];
            }
          }
        }
      }
    }
    if constexpr (SPECIAL) {                           // positions may be dead from the start: look again
      ftok = live ? T[ctz_bits<mask_t>(live) * W + tid] : kTokNone;
      firstv = live ? V[ctz_bits<mask_t>(live) * W + tid] : kNoRank;
      lastv = live ? V[top_bit<mask_t>(live) * W + tid] : kNoRank;
    }
  }

  int buf = 0;                                         // which half of the double-buffered exchange is current
  publish_record<NW>(sh, buf, wave, lane, live != 0, llim, firstv, lastv, ftok);

  // ---- merge passes ----
  // Every pass removes at least one token, so n passes can never be needed; the bound only guarantees
  // that the loop ends whatever the memory contents.
  for (int pass = 0; pass < n; ++pass) {
    // -- the horizon E of this pass and the boundary values from the neighbouring waves --
    uint32_t E, wave_in_val = kNoRank, wave_nxt_val = kNoRank;
    if (NW == 1) {
      E = wave_reduce<OpMin>(llim);
    } else {
      __syncthreads();                                 // records of all waves are in place
      const WaveRecord* rec = sh.rec + buf * NW;
      E = kNoRank;
#pragma unroll
      for (int w = 0; w < NW; ++w) E = min(E, rec[w].limit);
      E = uniform(E);
      for (int w = wave - 1; w >= 0; --w)              // nearest earlier non-empty wave
        if (rec[w].first_tok != kTokNone) { wave_in_val = rec[w].last_val; break; }
      for (int w = wave + 1; w < NW; ++w)              // nearest later non-empty wave
        if (rec[w].first_tok != kTokNone) { wave_nxt_val = rec[w].first_val; break; }
    }
    if (E == kNoRank) break;                           // no pair of the string is in the table
    // a pair is a candidate iff its value is below ev
    const uint32_t ev = E >= 0xFFFFFu ? 0xFFFFFFFEu : (E << kRankShift);

    // -- values just outside my column: the pair ending at my first token, the pair after my last --
    const uint64_t ne = __ballot(live != 0);
    const uint64_t below = ne & ((1ull << lane) - 1ull);
    const uint64_t above = lane == 63 ? 0ull : (ne >> (lane + 1)) << (lane + 1);
    uint32_t in_val = lane_read(lastv, below ? 63 - __builtin_clzll(below) : lane);
    uint32_t nxt_val = lane_read(firstv, above ? __builtin_ctzll(above) : lane);
    if (!below) in_val = wave_in_val;
    if (!above) nxt_val = wave_nxt_val;

    // -- sweep: which of my pairs are candidates --
    mask_t cm = 0;
    for (int k0 = 0; k0 < d; k0 += kChunk) {
      uint32_t v[kChunk];
#pragma unroll
      for (int g = 0; g < kChunk; g += kGroup) {
        if (g < D && k0 + g < d) {
#pragma unroll
          for (int j = g; j < g + kGroup; ++j) v[j] = V[(k0 + j) * W + tid];
        }
      }
#pragma unroll
      for (int g = 0; g < kChunk; g += kGroup) {
        if (g < D && k0 + g < d) {
#pragma unroll
          for (int j = g; j < g + kGroup; ++j) cm |= (mask_t)(v[j] < ev ? 1u : 0u) << (k0 + j);
        }
      }
    }

    // -- walk 1 over my candidates: which are beaten by a neighbour, and my element of the parity scan --
    // A candidate is "beaten by its left" if the pair before it is a candidate of lower or equal rank, and
    // "beaten by its right" if the pair after it is a candidate of strictly lower rank.  Going right along
    // a run of left-beaten candidates the applied ones alternate, starting with the run's unbeaten head.
    // e0: candidates at an even place of their run, counting as if the run that reaches my first position
    //     (mask lr) started there; nbr: candidates not beaten by their right.
    mask_t e0 = 0, lr = 0, nbr = 0;
    uint32_t elem = live ? 2u : 0u;                    // no trailing run: my last pair restarts the count
    if (__ballot(cm != 0)) {
      int prevc = -1;
      uint32_t prevv = 0, prev_dl = 0;
      bool prev_lead = false, prev_bl = false;
      for (mask_t m = cm; m; m &= m - 1) {
        const int k = ctz_bits<mask_t>(m);
        const uint32_t v = V[k * W + tid];
        const mask_t lower = live & bits_below<mask_t>(k);
        bool bl, lead;
        uint32_t dl;
        if (lower) {
          const bool adjacent = top_bit<mask_t>(lower) == prevc;   // the live position before k is a candidate
          bl = adjacent && prevv <= v;
          if (prevc >= 0 && !(adjacent && v < prevv)) nbr |= bit_at<mask_t>(prevc);
          dl = bl ? (prev_dl ^ 1u) : 0u;
          lead = bl && prev_lead;
        } else {                                       // k is my first live position
          bl = in_val <= v;                            // v is a candidate, so in_val is one too
          dl = bl ? 1u : 0u;
          lead = bl;
        }
        if (dl == 0) e0 |= bit_at<mask_t>(k);
        if (lead) lr |= bit_at<mask_t>(k);
        prevc = k;
        prevv = v;
        prev_dl = dl;
        prev_lead = lead;
        prev_bl = bl;
      }
      if (prevc >= 0) {
        const bool is_last = (live & bits_above<mask_t>(prevc)) == 0;
        if (!(is_last && nxt_val < prevv)) nbr |= bit_at<mask_t>(prevc);
        if (is_last && prev_bl) elem = (prev_lead ? 0u : 2u) | prev_dl;
      }
    }
    // parity of the run of left-beaten candidates that ends at the last live token before my column
    uint32_t pin;
    {
      const uint32_t inc = wave_scan<OpParity>(elem, 0u);
      uint32_t exc = wave_shift_up(inc, 0u);
      if (NW > 1) {
        const uint32_t wave_total = (uint32_t)__builtin_amdgcn_readlane((int)inc, 63);
        if (lane == 0) sh.part[buf * NW + wave] = wave_total;
        __syncthreads();
        uint32_t before = 0;
        for (int w = 0; w < wave; ++w) before = OpParity::apply(before, sh.part[buf * NW + w]);
        exc = OpParity::apply(before, exc);
      }
      pin = exc & 1u;
    }

    // -- walk 2 over the candidates that are applied: merge --
    const mask_t applied = cm & nbr & (pin ? (e0 ^ lr) : e0);
    // my first token is consumed if the pair ending at it is applied by the lane before me
    const bool skip_first = live != 0 && in_val < ev && !(firstv < in_val) && pin == 0;
    const bool touched = skip_first || applied != 0;
    mask_t dirty = 0;                                  // positions whose pair must be looked up again
    if (__ballot(touched)) {
      for (mask_t m = applied; m; m &= m - 1) {
        const int k = ctz_bits<mask_t>(m);
        T[k * W + tid] = merged_token_word(V[k * W + tid]);
        const mask_t upper = live & bits_above<mask_t>(k);
        if (upper) {                                   // the right operand is mine: it dies
          const int kn = ctz_bits<mask_t>(upper);
          live &= ~bit_at<mask_t>(kn);
          V[kn * W + tid] = kNoRank;
          if (LIMITS) L[kn * W + tid] = kNoRank;
        }                                              // else it is the next lane's first token (skip_first there)
        dirty |= bit_at<mask_t>(k);
        const mask_t lower = live & bits_below<mask_t>(k);
        if (lower) dirty |= bit_at<mask_t>(top_bit<mask_t>(lower));
      }
      if (skip_first) {
        const int f = ctz_bits<mask_t>(live);
        live &= ~bit_at<mask_t>(f);
        V[f * W + tid] = kNoRank;
        if (LIMITS) L[f * W + tid] = kNoRank;
      }
      dirty &= live;
      if (touched) ftok = live ? T[ctz_bits<mask_t>(live) * W + tid] : kTokNone;
    }

    // -- who follows me now, and did the token there change? --
    {
      const uint64_t ne2 = __ballot(live != 0);
      uint32_t next_wave_tok = kTokNone;
      if (NW > 1) {
        const uint32_t first = lane_read(ftok, ne2 ? __builtin_ctzll(ne2) : 0);
        if (lane == 0) sh.first_tok[buf * NW + wave] = ne2 ? first : kTokNone;
        __syncthreads();
        for (int w = wave + 1; w < NW; ++w) {
          const uint32_t t = sh.first_tok[buf * NW + w];
          if (t != kTokNone) { next_wave_tok = t; break; }
        }
      }
      const uint64_t above2 = lane == 63 ? 0ull : (ne2 >> (lane + 1)) << (lane + 1);
      uint32_t st = lane_read(ftok, above2 ? __builtin_ctzll(above2) : lane);
      if (!above2) st = next_wave_tok;
      if (live != 0 && st != succ_tok) {
        succ_tok = st;
        dirty |= bit_at<mask_t>(top_bit<mask_t>(live));
      }
    }

    // -- look up the pairs that changed, kProbes at a time; refresh my summary --
    const bool refresh = touched || dirty != 0;
    while (__ballot(dirty != 0)) {
      int k[kProbes];
      uint32_t x[kProbes], y[kProbes];
      ProbeInFlight f[kProbes];
#pragma unroll
      for (int j = 0; j < kProbes; ++j) {
        k[j] = -1;
        x[j] = 0;
        y[j] = kTokNone;
        if (dirty) {
          k[j] = ctz_bits<mask_t>(dirty);
          dirty &= dirty - 1;
          x[j] = T[k[j] * W + tid];
          const mask_t upper = live & bits_above<mask_t>(k[j]);
          y[j] = upper ? T[ctz_bits<mask_t>(upper) * W + tid] : succ_tok;
        }
      }
#pragma unroll
      for (int j = 0; j < kProbes; ++j) probe_start(tab, x[j], y[j], k[j] >= 0, f[j]);
#pragma unroll
      for (int j = 0; j < kProbes; ++j) {
        if (k[j] >= 0) {
          const uint32_t v = probe_finish(tab, f[j]);
          V[k[j] * W + tid] = v;
          if (LIMITS) L[k[j] * W + tid] = v != kNoRank ? limit_of(v) : kNoRank;
        }
      }
    }
    if (__ballot(refresh)) {
      uint32_t m = kNoRank;
      for (int k0 = 0; k0 < d; k0 += kChunk) {
        uint32_t l[kChunk];
#pragma unroll
        for (int g = 0; g < kChunk; g += kGroup) {
          if (g < D && k0 + g < d) {
#pragma unroll
            for (int j = g; j < g + kGroup; ++j) l[j] = LIMITS ? L[(k0 + j) * W + tid] : V[(k0 + j) * W + tid];
          }
        }
#pragma unroll
        for (int g = 0; g < kChunk; g += kGroup) {
          if (g < D && k0 + g < d) {
#pragma unroll
            for (int j = g; j < g + kGroup; ++j)
              m = min(m, LIMITS ? l[j] : (l[j] != kNoRank ? limit_of(l[j]) : kNoRank));
          }
        }
      }
      if (refresh) {
        llim = m;
        firstv = live ? V[ctz_bits<mask_t>(live) * W + tid] : kNoRank;
        lastv = live ? V[top_bit<mask_t>(live) * W + tid] : kNoRank;
      }
    }
    buf ^= 1;
    publish_record<NW>(sh, buf, wave, lane, live != 0, llim, firstv, lastv, ftok);
  }

  // ---- emit: prefix sum of live counts gives each lane's write index (section 4.3's compaction) ----
  uint32_t total;
  const uint32_t out0 = block_prefix_sum<NW>((uint32_t)pop_bits<mask_t>(live), sh, lane, wave, &total);
  int32_t* dst = p.tmp_ids + begin + out0;
  for (mask_t m = live; m; m &= m - 1) *dst++ = (int32_t)(T[ctz_bits<mask_t>(m) * W + tid] & kTokIdMask);
  if (tid == W - 1) p.counts[s] = (int32_t)total;
  block_sync<NW>();                                    // the LDS exchange arrays are reused by the next string
}

}  // namespace bpe
