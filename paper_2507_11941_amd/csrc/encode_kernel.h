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
  const uint32_t* byte_pair;  // [256*256] value of the pair (byte a, byte b) at a*256 + b, kNoRank if none
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

struct OpAdd { __device__ static uint32_t apply(uint32_t a, uint32_t b) { return a + b; } };

// Run-parity element: bit 1 = "a run restarts inside", bit 0 = parity of the run length since the last
// restart (or of the whole span if none).  apply(left, right) is the element of the concatenation.
struct OpParity {
  __device__ static uint32_t apply(uint32_t left, uint32_t right) {
    return (right & 2u) ? right : ((left & 2u) | ((left ^ right) & 1u));
  }
};

// The value the lane before mine holds (lane 0 receives `identity`).
__device__ inline uint32_t wave_shift_up(uint32_t v, uint32_t identity) {
  return (uint32_t)__builtin_amdgcn_update_dpp((int)identity, (int)v, 0x138, 0xF, 0xF, false);  // wave_shr:1
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

// The same lookup split in two so that a lane can have several probes in flight: start() issues the two
// 16-byte loads of the home bucket, finish() inspects them (and walks on in the rare displaced case).
struct ProbeInFlight {
  uint4 x, y;
  Placement pl;
  bool live;        // false: the capability bits or a missing neighbour already decided "no pair"
};

__device__ inline void probe_start(const DeviceTable& t, uint32_t xw, uint32_t yw, bool wanted, ProbeInFlight& f) {
  f.live = wanted && yw != kTokNone && (xw & kTokCanLeft) && (yw & kTokCanRight);
  if (f.live) {
    f.pl = place_pair(xw & kTokIdMask, yw & kTokIdMask, t.log2_buckets);
    const uint4* p = t.buckets + 2 * (size_t)f.pl.bucket;
    f.x = p[0];
    f.y = p[1];
  }
}

__device__ inline uint32_t probe_finish(const DeviceTable& t, const ProbeInFlight& f) {
  if (!f.live) return kNoRank;
  const uint32_t tag = slot_tag(f.pl.fingerprint, 0);
  if (f.x.y == tag) return f.x.x;
  if (f.x.w == tag) return f.x.z;
  if (f.y.y == tag) return f.y.x;
  if (f.y.w == tag) return f.y.z;
  if (f.y.w == 0xFFFFFFFFu) return kNoRank;
  for (uint32_t step = 1; step <= kMaxDisplacement; ++step) {   // home bucket full: the key may be displaced
    const uint4* p = t.buckets + 2 * (size_t)((f.pl.bucket + step) & t.bucket_mask);
    const uint4 x = p[0], y = p[1];
    const uint32_t tg = slot_tag(f.pl.fingerprint, step);
    if (x.y == tg) return x.x;
    if (x.w == tg) return x.z;
    if (y.y == tg) return y.x;
    if (y.w == tg) return y.z;
    if (y.w == 0xFFFFFFFFu) break;
  }
  return kNoRank;
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
//
// The per-lane loops run over chunks of kChunk slots: all loads of a chunk are issued before any is used,
// so a lane pays one LDS (or L2) latency per chunk instead of one per slot; the work on a chunk is cut into
// groups of kGroup slots that are skipped (scalar branch) once past the longest column of the wave.  D is a
// multiple of kChunk, so a chunk never reads outside the arrays; slots at or beyond the lane's count hold
// stale words that are loaded but never used.

#ifdef BPE_TRACE
__device__ unsigned long long g_trace[32];
#define TRACE_T(var) const unsigned long long var = (blockIdx.x == 0) ? __builtin_readcyclecounter() : 0ull
#define TRACE_ADD(slot, t0, t1) do { if (blockIdx.x == 0 && threadIdx.x == 0) g_trace[slot] += (t1) - (t0); } while (0)
#else
#define TRACE_T(var)
#define TRACE_ADD(slot, t0, t1)
#endif

constexpr int kChunk = 16;
constexpr int kGroup = 4;
constexpr int kProbes = 4;     // table probes a lane keeps in flight

// Per-lane summary of its column, kept in registers between passes.
struct LaneState {
  int c = 0;                         // live tokens
  uint32_t ftok = kTokNone;          // first live token word
  uint32_t succ_tok = kTokNone;      // the token my last pair is looked up against
  uint32_t firstv = kNoRank;         // pair value at slot 0
  uint32_t lastv = kNoRank;          // pair value at slot c-1
  uint32_t rest_lim = kNoRank;       // min limit() over slots 0..c-2
  uint32_t rest_minv = kNoRank;      // min value over slots 0..c-2
  __device__ uint32_t lim() const {
    return min(rest_lim, (c > 0 && lastv != kNoRank) ? limit_of(lastv) : kNoRank);
  }
  __device__ uint32_t minv() const { return c > 0 ? min(rest_minv, lastv) : kNoRank; }
};

template <int NW, int D, bool STAGED>
__device__ void encode_string(const EncodeParams& p, int s, uint32_t* __restrict__ T, uint32_t* __restrict__ V,
                              const BlockShared<NW>& sh) {
  static_assert(D % kChunk == 0 && D <= 64, "chunks must tile the column; dirty slots are a 64-bit mask");
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
  TRACE_T(t_start);
  LaneState me;
  me.c = n - tid * d;
  me.c = me.c < 0 ? 0 : (me.c > d ? d : me.c);

  // ---- load: byte-level pre-tokenisation (section 4.1), id = byte value; and the initial pair values,
  //      one lookup per adjacent byte pair in the direct 256 x 256 table ----
  {
    const int base = tid * d;
    const int c = me.c;
    for (int k0 = 0; k0 < d; k0 += kChunk) {           // d is uniform: no lane leaves the loop early
      uint32_t b[kChunk + 1];
#pragma unroll
      for (int j = 0; j <= kChunk; ++j) {
        const int i = base + k0 + j;
        b[j] = (k0 + j <= c && i < n) ? src[i] : 0x100u;   // 0x100: no such byte
      }
      uint32_t v[kChunk];
#pragma unroll
      for (int j = 0; j < kChunk; ++j)
        v[j] = (k0 + j < c && b[j + 1] < 0x100u) ? tab.byte_pair[(b[j] << 8) | b[j + 1]] : kNoRank;
#pragma unroll
      for (int j = 0; j < kChunk; ++j) {
        const int k = k0 + j;
        if (k < c) {
          const uint32_t w = sh.byte_word[b[j]];
          T[k * W + tid] = w;
          V[k * W + tid] = v[j];
          if (k == 0) { me.ftok = w; me.firstv = v[j]; }
          if (k == c - 1) {
            me.lastv = v[j];
            if (b[j + 1] < 0x100u) me.succ_tok = sh.byte_word[b[j + 1]];
          } else {
            if (v[j] != kNoRank) me.rest_lim = min(me.rest_lim, limit_of(v[j]));
            me.rest_minv = min(me.rest_minv, v[j]);
          }
        }
      }
    }
  }

  int buf = 0;                                         // which half of the double-buffered exchange is current
  publish_record<NW>(sh, buf, wave, lane, me.c, me.lim(), me.firstv, me.lastv, me.ftok);
  TRACE_T(t_loaded);
  TRACE_ADD(0, t_start, t_loaded);

  // ---- merge passes ----
  // Every pass removes at least one token, so n passes can never be needed; the bound only guarantees
  // that the loop ends whatever the memory contents.
  for (int pass = 0; pass < n; ++pass) {
    TRACE_T(t0);
    // -- the horizon E of this pass and the boundary values from the neighbouring waves --
    uint32_t E, wave_in_val = kNoRank, wave_nxt_val = kNoRank;
    if (NW == 1) {
      E = wave_reduce<OpMin>(me.lim());
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
    const uint64_t ne = __ballot(me.c != 0);
    const uint64_t below = ne & ((1ull << lane) - 1ull);
    const uint64_t above = lane == 63 ? 0ull : (ne >> (lane + 1)) << (lane + 1);
    uint32_t in_val = lane_read(me.lastv, below ? 63 - __builtin_clzll(below) : lane);
    uint32_t nxt_val = lane_read(me.firstv, above ? __builtin_ctzll(above) : lane);
    if (!below) in_val = wave_in_val;
    if (!above) nxt_val = wave_nxt_val;

    // A lane takes part in the pass if it holds a candidate or may lose its first token to one.
    const bool active = me.c > 0 && (me.minv() < ev || in_val < ev);
    const uint64_t active_lanes = __ballot(active);
    const int kmax = (int)wave_reduce<OpMax>(active ? (uint32_t)me.c : 0u);

    uint64_t dirty = 0;                                // slots whose pair must be looked up again
    uint32_t pin = 0;
    TRACE_T(t1);
    TRACE_ADD(1, t0, t1);
    // -- walk 1: my element of the run-parity scan --
    // A candidate is "beaten by its left" if the pair before it is a candidate of lower or equal rank.
    uint32_t elem = me.c > 0 ? 2u : 0u;                // inactive lane: its last pair restarts any run
    if (active_lanes) {
      uint32_t prev = in_val, par = 0, restart = 0;
      for (int k0 = 0; k0 < kmax; k0 += kChunk) {
        uint32_t v[kChunk];
#pragma unroll
        for (int g = 0; g < kChunk; g += kGroup) {
          if (k0 + g < kmax) {
#pragma unroll
            for (int j = g; j < g + kGroup; ++j) v[j] = V[(k0 + j) * W + tid];
          }
        }
#pragma unroll
        for (int g = 0; g < kChunk; g += kGroup) {
          if (k0 + g < kmax) {
#pragma unroll
            for (int j = g; j < g + kGroup; ++j) {
              if (active && k0 + j < me.c) {
                if (v[j] < ev && prev <= v[j]) par ^= 1u;
                else { restart = 2u; par = 0; }
                prev = v[j];
              }
            }
          }
        }
      }
      if (active) elem = restart | par;
    }
    TRACE_T(t2);
    TRACE_ADD(2, t1, t2);
    // parity of the run of beaten candidates that ends at the last live token before my column
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

    TRACE_T(t3);
    TRACE_ADD(3, t2, t3);
    // -- walk 2: decide, merge, and compact my column in place --
    if (active_lanes) {
      const int c = me.c;
      uint32_t prev = in_val, dlpar = pin;
      uint32_t cur = active ? V[tid] : kNoRank;
      // my first token is consumed if the pair ending at it is applied by the lane before me
      bool skip = active && in_val < ev && !(cur < in_val) && pin == 0;
      int o = 0;
      bool prev_changed = false, touched = false;
      uint32_t prev_val = kNoRank;
      uint32_t rest_lim = kNoRank, rest_minv = kNoRank, firstv = kNoRank;
      for (int k0 = 0; k0 < kmax; k0 += kChunk) {
        uint32_t vn[kChunk], tk[kChunk];
#pragma unroll
        for (int g = 0; g < kChunk; g += kGroup) {
          if (k0 + g < kmax) {
#pragma unroll
            for (int j = g; j < g + kGroup; ++j) {
              const int kn = k0 + j + 1;
              vn[j] = V[(kn < D ? kn : D - 1) * W + tid];
              tk[j] = T[(k0 + j) * W + tid];
            }
          }
        }
#pragma unroll
        for (int g = 0; g < kChunk; g += kGroup) {
          if (k0 + g < kmax) {
#pragma unroll
            for (int j = g; j < g + kGroup; ++j) {
              const int k = k0 + j;
              if (active && k < c) {
                const uint32_t nxt = (k + 1 < c) ? vn[j] : nxt_val;
                const bool cand = cur < ev;
                dlpar = (cand && prev <= cur) ? (dlpar ^ 1u) : 0u;
                const bool apply = cand && !(nxt < cur) && dlpar == 0;   // not beaten by its right, even place
                if (!skip) {
                  if (o > 0) {                         // the slot before is now known not to be the last
                    const bool dty = prev_changed || apply;
                    V[(o - 1) * W + tid] = dty ? kDirty : prev_val;
                    if (dty) {
                      dirty |= 1ull << (o - 1);
                    } else {
                      if (prev_val != kNoRank) rest_lim = min(rest_lim, limit_of(prev_val));
                      rest_minv = min(rest_minv, prev_val);
                    }
                    if (o == 1) firstv = dty ? kDirty : prev_val;
                  }
                  T[o * W + tid] = apply ? merged_token_word(cur) : tk[j];
                  prev_changed = apply;
                  prev_val = cur;
                  ++o;
                }
                touched = touched || skip || apply;
                skip = apply;                          // the right operand is consumed
                prev = cur;
                cur = nxt;
              }
            }
          }
        }
      }
      if (active) {
        if (o > 0) {                                   // the last slot: its pair crosses into the next lane
          V[(o - 1) * W + tid] = prev_changed ? kDirty : prev_val;
          if (prev_changed) dirty |= 1ull << (o - 1);
          me.lastv = prev_changed ? kDirty : prev_val;
          if (o == 1) firstv = me.lastv;
        } else {
          me.lastv = kNoRank;
        }
        me.c = o;
        me.firstv = firstv;
        me.rest_lim = rest_lim;
        me.rest_minv = rest_minv;
        if (touched) me.ftok = o > 0 ? T[tid] : kTokNone;
      }
    }

    TRACE_T(t4);
    TRACE_ADD(4, t3, t4);
    // -- who follows me now, and did the token there change? --
    {
      const uint64_t ne2 = __ballot(me.c != 0);
      uint32_t next_wave_tok = kTokNone;
      if (NW > 1) {
        const uint32_t first = lane_read(me.ftok, ne2 ? __builtin_ctzll(ne2) : 0);
        if (lane == 0) sh.first_tok[buf * NW + wave] = ne2 ? first : kTokNone;
        __syncthreads();
        for (int w = wave + 1; w < NW; ++w) {
          const uint32_t t = sh.first_tok[buf * NW + w];
          if (t != kTokNone) { next_wave_tok = t; break; }
        }
      }
      const uint64_t above2 = lane == 63 ? 0ull : (ne2 >> (lane + 1)) << (lane + 1);
      uint32_t st = lane_read(me.ftok, above2 ? __builtin_ctzll(above2) : lane);
      if (!above2) st = next_wave_tok;
      if (me.c > 0 && st != me.succ_tok) {
        me.succ_tok = st;
        dirty |= 1ull << (me.c - 1);
      }
    }

    TRACE_T(t5);
    TRACE_ADD(5, t4, t5);
    // -- look up the pairs that changed, kProbes at a time --
    while (__ballot(dirty != 0)) {
      TRACE_ADD(9, 0ull, 1ull);
      int k[kProbes];
      uint32_t x[kProbes], y[kProbes];
      ProbeInFlight f[kProbes];
#pragma unroll
      for (int j = 0; j < kProbes; ++j) {
        k[j] = -1;
        if (dirty) {
          k[j] = __builtin_ctzll(dirty);
          dirty &= dirty - 1;
          x[j] = T[k[j] * W + tid];
          y[j] = T[(k[j] + 1 < D ? k[j] + 1 : D - 1) * W + tid];
        }
      }
#pragma unroll
      for (int j = 0; j < kProbes; ++j) {
        const uint32_t yy = (k[j] + 1 < me.c) ? y[j] : me.succ_tok;
        probe_start(tab, x[j], yy, k[j] >= 0, f[j]);
      }
#pragma unroll
      for (int j = 0; j < kProbes; ++j) {
        if (k[j] >= 0) {
          const uint32_t v = probe_finish(tab, f[j]);
          V[k[j] * W + tid] = v;
          if (k[j] == 0) me.firstv = v;
          if (k[j] == me.c - 1) {
            me.lastv = v;
          } else {
            if (v != kNoRank) me.rest_lim = min(me.rest_lim, limit_of(v));
            me.rest_minv = min(me.rest_minv, v);
          }
        }
      }
    }
    buf ^= 1;
    publish_record<NW>(sh, buf, wave, lane, me.c, me.lim(), me.firstv, me.lastv, me.ftok);
    TRACE_T(t6);
    TRACE_ADD(6, t5, t6);
    TRACE_ADD(8, 0ull, 1ull);
  }
  TRACE_T(t_passes);

  // ---- emit: prefix sum of live counts gives each lane's write index (section 4.3's compaction) ----
  uint32_t total;
  const uint32_t out0 = block_prefix_sum<NW>((uint32_t)me.c, sh, lane, wave, &total);
  int32_t* dst = p.tmp_ids + begin + out0;
  const int cmax = (int)wave_reduce<OpMax>((uint32_t)me.c);
  for (int k0 = 0; k0 < cmax; k0 += kChunk) {
    uint32_t t[kChunk];
#pragma unroll
    for (int g = 0; g < kChunk; g += kGroup) {
      if (k0 + g < cmax) {
#pragma unroll
        for (int j = g; j < g + kGroup; ++j) t[j] = T[(k0 + j) * W + tid];
      }
    }
#pragma unroll
    for (int g = 0; g < kChunk; g += kGroup) {
      if (k0 + g < cmax) {
#pragma unroll
        for (int j = g; j < g + kGroup; ++j)
          if (k0 + j < me.c) dst[k0 + j] = (int32_t)(t[j] & kTokIdMask);
      }
    }
  }
  if (tid == W - 1) p.counts[s] = (int32_t)total;
  block_sync<NW>();                                    // the LDS exchange arrays are reused by the next string
  TRACE_T(t_end);
  TRACE_ADD(7, t_passes, t_end);
  TRACE_ADD(10, t_start, t_end);
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
  sh.part = cur; cur += 2 * NW;
  sh.item = cur; cur += 4;
  uint32_t* byte_word = cur;
  sh.byte_word = byte_word;
  for (int i = (int)threadIdx.x; i < 256; i += W) byte_word[i] = p.table.byte_word[i];
  __syncthreads();

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
  return sizeof(uint32_t) * ((STAGED ? 0 : 2 * NW * 64 * D) + 12 * NW + 4 + 256);
}

}  // namespace bpe
