// Per-string BPE merge kernel for gfx950 (wave64).
//
// One workgroup encodes one string (section 4.3: one block per string) and repeats merge passes until no
// adjacent pair is in the table (section 4.2): (1-2) every adjacent pair's rank is known, (3) workgroup
// minimum, (4) mark the occurrences of that rank, left-most first where they overlap, (5) write the merged
// token.  All occurrences of the pass's rank are applied in the same pass; because every row's operands
// are older than the row, this equals Algorithm 1's one-at-a-time order.
//
// How the passes are organised here (differs from the paper's compaction-per-pass):
//   * Lane `tid` owns the d = ceil(n / W) consecutive byte positions [tid*d, tid*d + d) of its string for
//     the whole encode.  A position holds a token word and the cached rank value of the pair (this token,
//     next live token).  Position e of lane tid lives at index e*W + tid, so a wave touches 64 consecutive
//     words whatever e each lane is at: no LDS bank conflicts, coalesced when the arrays are in HBM.
//   * A merge keeps the merged token at the left position and kills the right one; liveness is a bit mask
//     in a register.  Nothing moves, so a pass costs the reduction plus work only in lanes that hold the
//     minimum; the paper's prefix-sum compaction (section 4.3) runs once, at the end, to emit the ids.
//   * Ranks are looked up when a pair is created (n-1 initial probes, at most two per merge), never
//     re-probed per pass; a lane keeps the minimum of its cached ranks in a register.
//   * The only data that crosses lanes: each lane's first live token, so that the previous non-empty lane
//     can form its boundary pair; a "your first token was consumed" bit; and the reductions.  Inside a
//     wave these travel through ballots and lane permutes (registers only), between waves through a few
//     words of LDS per wave.  A one-wave workgroup therefore needs no barrier at all.
//   * Self pairs (left == right, e.g. runs "aaaa"): occurrences overlap, so the pass numbers the live
//     tokens (prefix sum), finds each run's start (prefix max) and keeps every second occurrence counted
//     from the run start.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>

#include "table_format.h"

namespace bpe {

struct DeviceTable {
  const uint4* buckets;       // 2 x uint4 per bucket
  const uint32_t* byte_word;  // [256] token word (id | capability bits) of each byte
  int log2_buckets;
  uint32_t bucket_mask;
};

struct EncodeParams {
  DeviceTable table;
  const uint8_t* bytes;
  const int64_t* offsets;
  const int32_t* list;        // string indices of all tiers, tier-major, longest first inside a tier
  const uint32_t* tier_base;  // [tiers+1] start of each tier's slice of `list`
  uint32_t* queue_head;       // [tiers] next unclaimed item of each tier
  int32_t* tmp_ids;           // ids of string s are written at tmp_ids[offsets[s] ...]
  int32_t* counts;            // [batch] token count of each string
  uint32_t* staged;           // HBM staging for the variant whose strings exceed LDS (else null)
  int tier;
};

// ---------------------------------------------------------------------------------------------------
// wave64 primitives

__device__ inline uint32_t dpp_quad_xor1(uint32_t v) {
  return (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0xB1, 0xF, 0xF, false);  // quad_perm 1,0,3,2
}
__device__ inline uint32_t dpp_quad_xor2(uint32_t v) {
  return (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x4E, 0xF, 0xF, false);  // quad_perm 2,3,0,1
}
__device__ inline uint32_t dpp_half_mirror(uint32_t v) {
  return (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x141, 0xF, 0xF, false);
}
__device__ inline uint32_t dpp_row_mirror(uint32_t v) {
  return (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x140, 0xF, 0xF, false);
}

// Minimum over the 64 lanes, returned in every lane.  All lanes must be active.
__device__ inline uint32_t wave_min(uint32_t v) {
  v = min(v, dpp_quad_xor1(v));
  v = min(v, dpp_quad_xor2(v));
  v = min(v, dpp_half_mirror(v));
  v = min(v, dpp_row_mirror(v));   // every lane of a 16-lane row now holds the row minimum
  uint32_t a = (uint32_t)__builtin_amdgcn_readlane((int)v, 0);
  uint32_t b = (uint32_t)__builtin_amdgcn_readlane((int)v, 16);
  uint32_t c = (uint32_t)__builtin_amdgcn_readlane((int)v, 32);
  uint32_t d = (uint32_t)__builtin_amdgcn_readlane((int)v, 48);
  return min(min(a, b), min(c, d));
}

struct OpAdd { __device__ static uint32_t apply(uint32_t a, uint32_t b) { return a + b; } };
struct OpMax { __device__ static uint32_t apply(uint32_t a, uint32_t b) { return a > b ? a : b; } };

// Inclusive scan over the wave (identity 0 for both operators).
template <class Op>
__device__ inline uint32_t wave_scan_inclusive(uint32_t v, int lane) {
#pragma unroll
  for (int step = 1; step < 64; step <<= 1) {
    uint32_t o = (uint32_t)__shfl_up((int)v, step, 64);
    if (lane >= step) v = Op::apply(v, o);
  }
  return v;
}

template <class T> __device__ inline int ctz_bits(T m);
template <> __device__ inline int ctz_bits<uint32_t>(uint32_t m) { return __builtin_ctz(m); }
template <> __device__ inline int ctz_bits<uint64_t>(uint64_t m) { return __builtin_ctzll(m); }
template <class T> __device__ inline int top_bit(T m);
template <> __device__ inline int top_bit<uint32_t>(uint32_t m) { return 31 - __builtin_clz(m); }
template <> __device__ inline int top_bit<uint64_t>(uint64_t m) { return 63 - __builtin_clzll(m); }
template <class T> __device__ inline int pop_bits(T m);
template <> __device__ inline int pop_bits<uint32_t>(uint32_t m) { return __builtin_popcount(m); }
template <> __device__ inline int pop_bits<uint64_t>(uint64_t m) { return __builtin_popcountll(m); }

// ---------------------------------------------------------------------------------------------------
// table probe

__device__ inline uint32_t probe_ids(const DeviceTable& t, uint32_t a, uint32_t b) {
  uint32_t h = bucket_of(a, b, t.log2_buckets);
  const uint32_t hi = slot_hi(a, b), lo8 = b & 0xFFu;
  for (;;) {
    const uint4* p = t.buckets + 2 * (size_t)h;
    const uint4 x = p[0], y = p[1];
    if (x.y == hi && (x.x >> 24) == lo8) return x.x & 0xFFFFFFu;
    if (x.w == hi && (x.z >> 24) == lo8) return x.z & 0xFFFFFFu;
    if (y.y == hi && (y.x >> 24) == lo8) return y.x & 0xFFFFFFu;
    if (y.w == hi && (y.z >> 24) == lo8) return y.z & 0xFFFFFFu;
    if (y.w == 0xFFFFFFFFu) return kNoRank;   // bucket not full: the key is nowhere else
    h = (h + 1) & t.bucket_mask;
  }
}

// Rank value of the pair of two token words, skipping the probe when the capability bits rule it out.
__device__ inline uint32_t probe_words(const DeviceTable& t, uint32_t x, uint32_t y) {
  if (!(x & kTokCanLeft) || !(y & kTokCanRight)) return kNoRank;
  return probe_ids(t, x & kTokIdMask, y & kTokIdMask);
}

// ---------------------------------------------------------------------------------------------------

template <int NW>
struct BlockShared {
  uint32_t* wave_tok;    // [2*NW] first live token word of each wave (kTokNone if empty), double buffered
  uint32_t* wave_cross;  // [NW] 1 if the wave's last non-empty lane merged across the wave boundary
  uint32_t* red;         // [2*NW] minimum partials, double buffered
  uint32_t* part;        // [NW] scan partials
  uint32_t* item;        // [1] work item broadcast
};

__device__ inline uint32_t uniform(uint32_t v) { return (uint32_t)__builtin_amdgcn_readfirstlane((int)v); }

// Workgroup barrier; a single-wave workgroup exchanges data through registers only and needs none.
template <int NW>
__device__ inline void block_sync() {
  if (NW > 1) __syncthreads();
}

// Minimum over the workgroup, uniform (scalar) result.
template <int NW>
__device__ inline uint32_t block_min(uint32_t v, const BlockShared<NW>& sh, int wave, int parity) {
  v = wave_min(v);
  if (NW == 1) return v;
  uint32_t* red = sh.red + parity * NW;
  if ((threadIdx.x & 63) == 0) red[wave] = v;
  __syncthreads();
  uint32_t r = red[0];
#pragma unroll
  for (int w = 1; w < NW; ++w) r = min(r, red[w]);
  return uniform(r);
}

// Exclusive scan of v over the workgroup in lane order; *total receives the full reduction.
template <int NW, class Op>
__device__ inline uint32_t block_scan_exclusive(uint32_t v, const BlockShared<NW>& sh, int lane, int wave,
                                                uint32_t* total) {
  uint32_t inc = wave_scan_inclusive<Op>(v, lane);
  uint32_t exc = (uint32_t)__shfl_up((int)inc, 1, 64);
  if (lane == 0) exc = 0;
  uint32_t wave_total = (uint32_t)__builtin_amdgcn_readlane((int)inc, 63);
  if (NW == 1) {
    *total = wave_total;
    return exc;
  }
  __syncthreads();                       // previous users of sh.part are done
  if (lane == 0) sh.part[wave] = wave_total;
  __syncthreads();
  uint32_t before = 0, all = 0;
#pragma unroll
  for (int w = 0; w < NW; ++w) {
    uint32_t p = sh.part[w];
    if (w < wave) before = Op::apply(before, p);
    all = Op::apply(all, p);
  }
  *total = all;
  return Op::apply(before, exc);
}

// Encode string s.  tok/rnk: token words and cached pair ranks, index e*W + tid, in LDS or (strings that
// exceed LDS) in HBM; every word is read and written by its owning lane only.  Lanes of one wave exchange
// data through ballots and lane permutes; waves exchange through the small LDS arrays of BlockShared.
template <int NW, int D, bool STAGED>
__device__ void encode_string(const EncodeParams& p, int s, uint32_t* __restrict__ tok,
                              uint32_t* __restrict__ rnk, const BlockShared<NW>& sh) {
  constexpr int W = NW * 64;
  using mask_t = typename std::conditional<(D <= 32), uint32_t, uint64_t>::type;
  constexpr int kBits = (int)sizeof(mask_t) * 8;
  const int tid = (int)threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const DeviceTable& tab = p.table;

  const int64_t begin = p.offsets[s];
  const int n = (int)uniform((uint32_t)(p.offsets[s + 1] - begin));
  if (n <= 0) {                                        // uniform branch
    if (tid == W - 1) p.counts[s] = 0;
    return;
  }
  const uint8_t* src = p.bytes + begin;
  const int d = (n + W - 1) / W;                       // positions per lane, 1 <= d <= D
  int my_n = n - tid * d;
  my_n = my_n < 0 ? 0 : (my_n > d ? d : my_n);

  mask_t mask = my_n >= kBits ? ~(mask_t)0 : (((mask_t)1 << my_n) - 1);

  // ---- load: byte-level pre-tokenisation (section 4.1), id = byte value ----
  for (int e = 0; e < my_n; ++e) tok[e * W + tid] = tab.byte_word[src[tid * d + e]];
  uint32_t ftok = my_n > 0 ? tok[tid] : kTokNone;      // my first live token word
  // token my last pair is probed against: first token of the lane that follows (lanes fill contiguously)
  uint32_t succ_tok = kTokNone;
  if (my_n > 0 && (tid + 1) * d < n) succ_tok = tab.byte_word[src[(tid + 1) * d]];

  // ---- initial ranks: one probe per adjacent pair ----
  uint32_t lmin = kNoRank;
  {
    uint32_t x = ftok;
    for (int e = 0; e < my_n; ++e) {
      uint32_t y = (e + 1 < my_n) ? tok[(e + 1) * W + tid] : succ_tok;
      uint32_t r = (y == kTokNone) ? kNoRank : probe_words(tab, x, y);
      rnk[e * W + tid] = r;
      lmin = min(lmin, r);
      x = y;
    }
  }
  int buf = 0;
  if (NW > 1) {
    if (lane == 0) sh.wave_tok[wave] = ftok;           // lane 0 is empty only if the whole wave is
    __syncthreads();
  }

  // ---- merge passes ----
  // Every pass removes at least one token, so n passes can never be needed; the bound only guarantees
  // that the loop ends whatever the memory contents.
  int parity = 0;
  for (int pass = 0; pass < n; ++pass) {
    const uint32_t r = block_min<NW>(lmin, sh, wave, parity);
    parity ^= 1;
    if (r == kNoRank) break;
    const uint32_t merged = merged_token_word(r);
    const bool self = (r & kFlagSelf) != 0;
    const uint64_t ne = __ballot(mask != 0);           // non-empty lanes of my wave before this pass

    uint32_t base = 0, start = 0;
    if (self) {
      // number the live tokens and find where the run that reaches each lane began
      uint32_t total;
      const uint32_t c = (uint32_t)pop_bits<mask_t>(mask);
      base = block_scan_exclusive<NW, OpAdd>(c, sh, lane, wave, &total);
      uint32_t z = c ? base + c : 0;                   // 1 + index of my last non-matching token
      if (lmin == r) {
        z = 0;
        uint32_t g = base;
        for (mask_t m = mask; m; m &= m - 1, ++g) {
          const int e = ctz_bits<mask_t>(m);
          if (rnk[e * W + tid] != r) z = g + 1;
        }
      }
      start = block_scan_exclusive<NW, OpMax>(z, sh, lane, wave, &total);
    }

    mask_t dirty = 0;                                  // positions whose pair must be probed again
    bool touched = false;                              // my tokens or liveness changed
    bool cross = false;                                // I merged my last token with the next lane's first
    if (lmin == r) {
      uint32_t g = base;
      const mask_t before = mask;
      for (mask_t m = before; m; m &= m - 1, ++g) {
        const int e = ctz_bits<mask_t>(m);
        if (rnk[e * W + tid] != r) { start = g + 1; continue; }
        if (self && ((g - start) & 1u)) continue;      // overlaps the occurrence to its left
        // merge (token e, next live token) -> merged, kept at e
        tok[e * W + tid] = merged;
        const mask_t above = before & ~((((mask_t)2) << e) - 1);
        if (above) mask &= ~((mask_t)1 << ctz_bits<mask_t>(above));
        else cross = true;                             // the pair exists, so a following lane does
        dirty |= (mask_t)1 << e;
        const mask_t below = before & ((((mask_t)1) << e) - 1);
        if (below) dirty |= (mask_t)1 << top_bit<mask_t>(below);
        touched = true;
      }
    }

    // ---- was my first live token merged into the lane before me? ----
    const uint64_t crossmask = __ballot(cross);
    uint32_t in_cross = 0;                             // the same question across the wave boundary
    if (NW > 1) {
      if (lane == 0) sh.wave_cross[wave] = ne ? (uint32_t)((crossmask >> (63 - __builtin_clzll(ne))) & 1) : 0u;
      __syncthreads();
      for (int w = wave - 1; w >= 0; --w) {            // nearest earlier wave that was non-empty
        if (sh.wave_tok[buf * NW + w] != kTokNone) { in_cross = sh.wave_cross[w]; break; }
      }
    }
    if (mask) {
      const uint64_t below = ne & ((1ull << lane) - 1);
      const uint32_t consumed = below ? (uint32_t)((crossmask >> (63 - __builtin_clzll(below))) & 1) : in_cross;
      if (consumed) {
        mask &= mask - 1;
        touched = true;
      }
    }
    if (touched) ftok = mask ? tok[ctz_bits<mask_t>(mask) * W + tid] : kTokNone;

    // ---- who follows me now, and did the token there change? ----
    const uint64_t ne2 = __ballot(mask != 0);
    uint32_t next_wave_tok = kTokNone;
    if (NW > 1) {
      buf ^= 1;
      const uint32_t first = (uint32_t)__shfl((int)ftok, ne2 ? __builtin_ctzll(ne2) : 0, 64);
      if (lane == 0) sh.wave_tok[buf * NW + wave] = ne2 ? first : kTokNone;
      __syncthreads();
      for (int w = wave + 1; w < NW; ++w) {
        const uint32_t t = sh.wave_tok[buf * NW + w];
        if (t != kTokNone) { next_wave_tok = t; break; }
      }
    }
    {
      const uint64_t above = lane == 63 ? 0ull : (ne2 >> (lane + 1)) << (lane + 1);
      uint32_t st = (uint32_t)__shfl((int)ftok, above ? __builtin_ctzll(above) : lane, 64);
      if (!above) st = next_wave_tok;
      if (mask && st != succ_tok) {
        succ_tok = st;
        dirty |= (mask_t)1 << top_bit<mask_t>(mask);
      }
    }

    // ---- probe the pairs that changed; refresh my minimum ----
    if (dirty || touched) {
      for (mask_t m = dirty & mask; m; m &= m - 1) {
        const int e = ctz_bits<mask_t>(m);
        const uint32_t x = tok[e * W + tid];
        const mask_t above = mask & ~((((mask_t)2) << e) - 1);
        const uint32_t y = above ? tok[ctz_bits<mask_t>(above) * W + tid] : succ_tok;
        rnk[e * W + tid] = (y == kTokNone) ? kNoRank : probe_words(tab, x, y);
      }
      lmin = kNoRank;
      for (mask_t m = mask; m; m &= m - 1) lmin = min(lmin, rnk[ctz_bits<mask_t>(m) * W + tid]);
    }
  }

  // ---- emit: prefix sum of live counts gives each lane's write index (section 4.3's compaction) ----
  uint32_t total;
  const uint32_t c = (uint32_t)pop_bits<mask_t>(mask);
  const uint32_t out0 = block_scan_exclusive<NW, OpAdd>(c, sh, lane, wave, &total);
  int32_t* dst = p.tmp_ids + begin + out0;
  for (mask_t m = mask; m; m &= m - 1) *dst++ = (int32_t)(tok[ctz_bits<mask_t>(m) * W + tid] & kTokIdMask);
  if (tid == W - 1) p.counts[s] = (int32_t)total;
  block_sync<NW>();                                    // the LDS exchange arrays are reused by the next string
}

// Persistent workgroups: each claims the next string of its tier until the tier's list is exhausted.
template <int NW, int D, bool STAGED>
__global__ __launch_bounds__(NW * 64) void encode_kernel(EncodeParams p) {
  constexpr int W = NW * 64;
  extern __shared__ uint32_t smem[];
  uint32_t* cur = smem;
  uint32_t *tok, *rnk;
  if (STAGED) {
    tok = p.staged + (size_t)blockIdx.x * (2u * W * D);
    rnk = tok + W * D;
  } else {
    tok = cur; cur += W * D;
    rnk = cur; cur += W * D;
  }
  BlockShared<NW> sh;
  sh.wave_tok = cur; cur += 2 * NW;
  sh.wave_cross = cur; cur += NW;
  sh.red = cur; cur += 2 * NW;
  sh.part = cur; cur += NW;
  sh.item = cur;

  const uint32_t first = p.tier_base[p.tier], end = p.tier_base[p.tier + 1];
  for (;;) {
    // Claim the next item.  Every lane of the first wave takes part in the atomic (lane 0 adds 1, the
    // others 0) so that no lane-dependent branch sits at the loop boundary: a branch on "thread 0" here,
    // next to the "thread 0" store that ends the previous string, lets the compiler send the other lanes
    // round the loop on their own, past the lane-0 broadcast below.
    uint32_t claimed = 0;
    if (NW == 1) {
      claimed = first + atomicAdd(p.queue_head + p.tier, threadIdx.x == 0 ? 1u : 0u);
    } else {
      if (threadIdx.x < 64) claimed = first + atomicAdd(p.queue_head + p.tier, threadIdx.x == 0 ? 1u : 0u);
      if (threadIdx.x == 0) *sh.item = claimed;
      __syncthreads();
      claimed = *sh.item;
      __syncthreads();
    }
    const uint32_t item = uniform(claimed);            // lane 0's value, as a scalar
    if (item >= end) break;
    encode_string<NW, D, STAGED>(p, (int)uniform((uint32_t)p.list[item]), tok, rnk, sh);
  }
}

template <int NW, int D, bool STAGED>
constexpr size_t encode_lds_bytes() {
  return sizeof(uint32_t) * ((STAGED ? 0 : 2 * NW * 64 * D) + 6 * NW + 4);
}

}  // namespace bpe
