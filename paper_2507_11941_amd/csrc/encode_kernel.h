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

// Inclusive prefix sum over the wave.
__device__ inline uint32_t wave_prefix_sum(uint32_t v, int lane) {
#pragma unroll
  for (int step = 1; step < 64; step <<= 1) {
    const uint32_t o = (uint32_t)__shfl_up((int)v, step, 64);
    if (lane >= step) v += o;
  }
  return v;
}

// Run-parity element: bit 1 = "a run restarts inside", bit 0 = parity of the run length since the last
// restart (or of the whole span if none).  combine(left, right) is the element of the concatenation.
__device__ inline uint32_t parity_combine(uint32_t left, uint32_t right) {
  return (right & 2u) ? right : ((left & 2u) | ((left ^ right) & 1u));
}
__device__ inline uint32_t wave_parity_scan(uint32_t v, int lane) {   // inclusive
#pragma unroll
  for (int step = 1; step < 64; step <<= 1) {
    const uint32_t o = (uint32_t)__shfl_up((int)v, step, 64);
    if (lane >= step) v = parity_combine(o, v);
  }
  return v;
}

// ---------------------------------------------------------------------------------------------------
// table probe

__device__ inline uint32_t probe_ids(const DeviceTable& t, uint32_t a, uint32_t b) {
  const Placement pl = place_pair(a, b, t.log2_buckets);
  for (uint32_t step = 0; step <= kMaxDisplacement; ++step) {
    const uint4* p = t.buckets + 2 * (size_t)((pl.bucket + step) & t.bucket_mask);
    const uint4 x = p[0], y = p[1];
    const uint32_t tag = slot_tag(pl.fingerprint, step);
    if (x.y == tag) return x.x;
    if (x.w == tag) return x.z;
    if (y.y == tag) return y.x;
    if (y.w == tag) return y.z;
    if (y.w == 0xFFFFFFFFu) break;            // bucket not full: the key is nowhere else
  }
  return kNoRank;
}

// Value of the pair of two token words, skipping the probe when the capability bits rule it out.
__device__ inline uint32_t probe_words(const DeviceTable& t, uint32_t x, uint32_t y) {
  if (!(x & kTokCanLeft) || !(y & kTokCanRight)) return kNoRank;
  return probe_ids(t, x & kTokIdMask, y & kTokIdMask);
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
  uint32_t* part;        // [NW] scan partials
  uint32_t* item;        // [1] work item broadcast
};

template <int NW>
__device__ inline void block_sync() {
  if (NW > 1) __syncthreads();
}

// Exclusive prefix sum of v over the workgroup in lane order; *total receives the sum.
template <int NW>
__device__ inline uint32_t block_prefix_sum(uint32_t v, const BlockShared<NW>& sh, int lane, int wave,
                                            uint32_t* total) {
  const uint32_t inc = wave_prefix_sum(v, lane);
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
__device__ inline void publish_record(const BlockShared<NW>& sh, int buf, int wave, int lane, int c,
                                      uint32_t llim, uint32_t firstv, uint32_t lastv, uint32_t ftok) {
  if (NW == 1) return;
  const uint64_t ne = __ballot(c != 0);
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
// Encode string s.  T/V: token words and pair values of each lane's live tokens, slot k of lane tid at
// index k*W + tid, in LDS or (strings that exceed LDS) in HBM; every word is read and written by its
// owning lane only.  V[k] is the value of the pair (token k, next live token of the string) -- for a
// lane's last slot the next token is the first token of the next non-empty lane.

template <int NW, int D, bool STAGED>
__device__ void encode_string(const EncodeParams& p, int s, uint32_t* __restrict__ T, uint32_t* __restrict__ V,
                              const BlockShared<NW>& sh) {
  constexpr int W = NW * 64;
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
  const int d = (n + W - 1) / W;                       // bytes per lane, 1 <= d <= D
  int c = n - tid * d;                                 // my live token count
  c = c < 0 ? 0 : (c > d ? d : c);

  // ---- load: byte-level pre-tokenisation (section 4.1), id = byte value ----
  for (int k = 0; k < c; ++k) T[k * W + tid] = tab.byte_word[src[tid * d + k]];
  uint32_t ftok = c > 0 ? T[tid] : kTokNone;           // my first live token word
  // token my last pair is probed against: first token of the lane that follows (lanes fill contiguously)
  uint32_t succ_tok = kTokNone;
  if (c > 0 && (tid + 1) * d < n) succ_tok = tab.byte_word[src[(tid + 1) * d]];

  // ---- initial pair values: one probe per adjacent pair ----
  uint32_t llim = kNoRank;                             // min limit() over my pairs
  uint32_t lminv = kNoRank;                            // min value over my pairs
  uint32_t firstv = kNoRank, lastv = kNoRank;          // values at my first / last slot
  {
    uint32_t x = ftok;
    for (int k = 0; k < c; ++k) {
      const uint32_t y = (k + 1 < c) ? T[(k + 1) * W + tid] : succ_tok;
      const uint32_t v = (y == kTokNone) ? kNoRank : probe_words(tab, x, y);
      V[k * W + tid] = v;
      if (v != kNoRank) llim = min(llim, limit_of(v));
      lminv = min(lminv, v);
      if (k == 0) firstv = v;
      lastv = v;
      x = y;
    }
  }

  int buf = 0;                                         // which half of the double-buffered records is current
  publish_record<NW>(sh, buf, wave, lane, c, llim, firstv, lastv, ftok);

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
    const uint64_t ne = __ballot(c != 0);
    const uint64_t below = ne & ((1ull << lane) - 1ull);
    const uint64_t above = lane == 63 ? 0ull : (ne >> (lane + 1)) << (lane + 1);
    uint32_t in_val = lane_read(lastv, below ? 63 - __builtin_clzll(below) : lane);
    uint32_t nxt_val = lane_read(firstv, above ? __builtin_ctzll(above) : lane);
    if (!below) in_val = wave_in_val;
    if (!above) nxt_val = wave_nxt_val;

    // A lane takes part in the pass if it holds a candidate or may lose its first token to one.
    const bool active = c > 0 && (lminv < ev || in_val < ev);
    const uint64_t active_lanes = __ballot(active);
    const int kmax = (int)wave_reduce<OpMax>(active ? (uint32_t)c : 0u);

    // -- walk 1: my element of the run-parity scan --
    // A candidate is "beaten by its left" if the pair before it is a candidate of lower or equal rank.
    uint32_t elem = c > 0 ? 2u : 0u;                   // inactive lane: its last pair restarts any run
    if (active_lanes) {
      if (active) {
        uint32_t prev = in_val, par = 0, restart = 0;
        for (int k = 0; k < kmax; ++k) {
          if (k < c) {
            const uint32_t cur = V[k * W + tid];
            if (cur < ev && prev <= cur) par ^= 1u;
            else { restart = 2u; par = 0; }
            prev = cur;
          }
        }
        elem = restart | par;
      }
    }
    // parity of the run of beaten candidates that ends at the last live token before my column
    uint32_t pin;
    {
      const uint32_t inc = wave_parity_scan(elem, lane);
      uint32_t exc = (uint32_t)__shfl_up((int)inc, 1, 64);
      if (lane == 0) exc = 0;
      if (NW > 1) {
        const uint32_t wave_total = (uint32_t)__builtin_amdgcn_readlane((int)inc, 63);
        __syncthreads();                               // previous users of sh.part are done
        if (lane == 0) sh.part[wave] = wave_total;
        __syncthreads();
        uint32_t before = 0;
        for (int w = 0; w < wave; ++w) before = parity_combine(before, sh.part[w]);
        exc = parity_combine(before, exc);
      }
      pin = exc & 1u;
    }

    // -- walk 2: decide, merge, and compact my column in place --
    bool touched = false;                              // my tokens or my pair values changed
    if (active_lanes) {
      if (active) {
        uint32_t prev = in_val, dlpar = pin;
        uint32_t cur = V[tid];
        // my first token is consumed if the pair ending at it is applied by the lane before me
        bool skip = in_val < ev && !(cur < in_val) && pin == 0;
        int o = 0;
        bool prev_changed = false;
        uint32_t prev_val = kNoRank;
        for (int k = 0; k < kmax; ++k) {
          if (k < c) {
            const uint32_t nxt = (k + 1 < c) ? V[(k + 1) * W + tid] : nxt_val;
            const bool cand = cur < ev;
            dlpar = (cand && prev <= cur) ? (dlpar ^ 1u) : 0u;
            const bool apply = cand && !(nxt < cur) && dlpar == 0;   // not beaten by its right, even place
            if (!skip) {
              const uint32_t t = apply ? merged_token_word(cur) : T[k * W + tid];
              if (o > 0) V[(o - 1) * W + tid] = (prev_changed || apply) ? kDirty : prev_val;
              T[o * W + tid] = t;
              prev_changed = apply;
              prev_val = cur;
              ++o;
            }
            touched = touched || skip || apply;
            skip = apply;                              // the right operand is consumed
            prev = cur;
            cur = nxt;
          }
        }
        if (o > 0) V[(o - 1) * W + tid] = prev_changed ? kDirty : prev_val;
        c = o;
        if (touched) ftok = c > 0 ? T[tid] : kTokNone;
      }
    }

    // -- who follows me now, and did the token there change? --
    {
      const uint64_t ne2 = __ballot(c != 0);
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
      if (c > 0 && st != succ_tok) {
        succ_tok = st;
        V[(c - 1) * W + tid] = kDirty;
        touched = true;
      }
    }

    // -- look up the pairs that changed; refresh my summary --
    if (__ballot(touched)) {
      if (touched) {
        llim = kNoRank;
        lminv = kNoRank;
        firstv = kNoRank;
        lastv = kNoRank;
        uint32_t x = ftok;
        for (int k = 0; k < c; ++k) {
          const uint32_t y = (k + 1 < c) ? T[(k + 1) * W + tid] : succ_tok;
          uint32_t v = V[k * W + tid];
          if (v == kDirty) {
            v = (y == kTokNone) ? kNoRank : probe_words(tab, x, y);
            V[k * W + tid] = v;
          }
          if (v != kNoRank) llim = min(llim, limit_of(v));
          lminv = min(lminv, v);
          if (k == 0) firstv = v;
          lastv = v;
          x = y;
        }
      }
    }
    buf ^= 1;
    publish_record<NW>(sh, buf, wave, lane, c, llim, firstv, lastv, ftok);
  }

  // ---- emit: prefix sum of live counts gives each lane's write index (section 4.3's compaction) ----
  uint32_t total;
  const uint32_t out0 = block_prefix_sum<NW>((uint32_t)c, sh, lane, wave, &total);
  int32_t* dst = p.tmp_ids + begin + out0;
  for (int k = 0; k < c; ++k) dst[k] = (int32_t)(T[k * W + tid] & kTokIdMask);
  if (tid == W - 1) p.counts[s] = (int32_t)total;
  block_sync<NW>();                                    // the LDS exchange arrays are reused by the next string
}

// Persistent workgroups: each claims the next string of its tier until the tier's list is exhausted.
template <int NW, int D, bool STAGED>
__global__ __launch_bounds__(NW * 64) void encode_kernel(EncodeParams p) {
  constexpr int W = NW * 64;
  extern __shared__ uint32_t smem[];
  uint32_t* cur = smem;
  uint32_t *T, *V;
  if (STAGED) {
    T = p.staged + (size_t)blockIdx.x * (2u * W * D);
    V = T + W * D;
  } else {
    T = cur; cur += W * D;
    V = cur; cur += W * D;
  }
  BlockShared<NW> sh;
  sh.rec = (WaveRecord*)cur; cur += 2 * NW * (sizeof(WaveRecord) / sizeof(uint32_t));
  sh.first_tok = cur; cur += 2 * NW;
  sh.part = cur; cur += NW;
  sh.item = cur;

  const uint32_t first = p.tier_base[p.tier], end = p.tier_base[p.tier + 1];
  for (;;) {
    // Claim the next item.  Every lane of the first wave takes part in the atomic (lane 0 adds 1, the
    // others 0) so that no lane-dependent branch sits at the loop boundary: a branch on "thread 0" here,
    // next to a single-lane store that ends the previous string, lets the compiler send the other lanes
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
    encode_string<NW, D, STAGED>(p, (int)uniform((uint32_t)p.list[item]), T, V, sh);
  }
}

template <int NW, int D, bool STAGED>
constexpr size_t encode_lds_bytes() {
  return sizeof(uint32_t) * ((STAGED ? 0 : 2 * NW * 64 * D) + 11 * NW + 4);
}

}  // namespace bpe
