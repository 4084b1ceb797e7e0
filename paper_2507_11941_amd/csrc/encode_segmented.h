// Segment-local horizons: the encoder used for strings whose per-position state fits LDS.
//
// Same pass structure as encode_string() in encode_kernel.h (candidates below a horizon, run-parity scan,
// merge in place, look up the changed pairs), with one difference that cuts the number of passes by another
// order of magnitude: the horizon is taken per SEGMENT of the string instead of over the whole string.
//
// A merge joins a token that ends at byte i with a token that starts at byte i+1, so the bigram
// (byte i, byte i+1) then lies inside a vocabulary token.  The table builder marks every byte bigram that
// occurs at no row's junction (last byte of the left operand, first byte of the right operand); between two
// such bytes no merge can ever happen, whatever the rest of the string holds.  These "cuts" split a string
// into segments that Algorithm 1 processes without any interaction, so each segment may use its own horizon
// E = min limit() over its own pairs.  With word-like text a segment is a word, its merges take 5-10
// fused passes, and all segments of the string advance in the same passes.  Nothing here is a heuristic: a
// table without such bigrams simply yields one segment per string and the whole-string horizon.
//
// Per pass a lane (a) sweeps its limits and values: running minima forward and backward inside its segments
// give every position its segment minimum, except for the segment that enters the lane from the left and
// the one that leaves it to the right; (b) those two are completed by a prefix and a suffix minimum over the
// lanes, made segment-aware by putting the number of cut-holding lanes so far above the limit in the key
// (plain DPP minima; between waves through the LDS records); (c) compares each value with its segment's
// horizon to get the candidate mask.  The rest of the pass is the same as in encode_string().
#pragma once
#include "encode_kernel.h"

namespace bpe {

// Horizons are limits in rank units, 20 bits: a pair (value v) is a candidate iff (v >> kRankShift) < horizon.
constexpr uint32_t kInf20 = 0xFFFFFu;       // "no pair": equals kNoRank >> kRankShift, so it admits nothing
constexpr uint32_t kAll20 = 0xFFFFEu;       // horizon above every rank (ranks stay below BPE_MAX_MERGES)
constexpr uint32_t kInf31 = 0x7FFFFFFFu;    // identity of the cross-wave segmented minimum
constexpr uint32_t kReset31 = 0x80000000u;  // cross-wave element flag: a cut lies inside this span

// (Straight-line on purpose: it runs once per position at load and once per look-up.)
__device__ inline uint32_t limit20_of(uint32_t value) {
  const uint32_t code = (value >> kHorizonShift) & 0xFFu;
  const uint32_t e = code >> 4, m = code & 15u;
  const uint32_t span = e ? ((16u | m) << (e - 1u)) : m;                  // horizon_decode(code)
  uint32_t lim = min((value >> kRankShift) + 1u + span, kAll20);
  lim = code == 255u ? kAll20 : lim;                                     // the token is never an operand
  return value == kNoRank ? kInf20 : lim;
}

// Segmented minimum: apply(left, right) = right if a cut lies inside right, else the minimum of the two with
// left's flag.  Bit 31 is the flag, bits 0..30 the value; kInf31 (flag clear) is the identity.
struct OpSegMin {
  __device__ static uint32_t apply(uint32_t left, uint32_t right) {
    const uint32_t m = min(left & kInf31, right & kInf31) | (left & kReset31);
    return (right & kReset31) ? right : m;
  }
};

// What a wave tells the others at the start of each pass.
struct SegRecord {
  uint32_t fwd;        // segmented-min element of the whole wave, left to right (tail minima)
  uint32_t bwd;        // the same right to left (head minima)
  uint32_t first_val;  // pair value at the wave's first live token
  uint32_t last_val;   // pair value at the wave's last live token
  uint32_t first_tok;  // first live token word, kTokNone if the wave is empty
  uint32_t any_pair;   // 1 if any pair of the wave is in the table
  uint32_t pad0, pad1;
};

template <int NW, int D, bool LIMITS, bool SPECIAL>
__device__ void encode_string_segmented(const EncodeParams& p, int s, uint32_t* __restrict__ T,
                                        uint32_t* __restrict__ V, uint32_t* __restrict__ L,
                                        const BlockShared<NW>& sh) {
  static_assert(D % kGroup == 0 && D <= 16, "the per-position registers of the sweep are sized for 16");
  using mask_t = uint32_t;
  constexpr int W = NW * 64;
  const int tid = (int)threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const DeviceTable& tab = p.table;
  SegRecord* const rec_base = (SegRecord*)sh.rec;

  // a work item is a whole string, or a piece of one between two cuts
  const int64_t begin = p.piece_begin ? p.piece_begin[s] : p.offsets[s];
  const int n = (int)uniform((uint32_t)(p.piece_len ? p.piece_len[s] : (int32_t)(p.offsets[s + 1] - begin)));
  if (n <= 0 || n > W * D) {                           // uniform branch; too long only if max_len was wrong
    if (tid == W - 1) p.counts[s] = 0;
    return;
  }
  const uint8_t* src = p.bytes + begin;
  const int d = (n + W - 1) / W;                       // bytes per lane, 1 <= d <= D (uniform)
  const int dpad = (d + kGroup - 1) / kGroup * kGroup; // the sweeps work on whole groups: pad with dead positions
  int c0 = n - tid * d;                                // my byte count
  c0 = c0 < 0 ? 0 : (c0 > d ? d : c0);

  mask_t live = bits_below<mask_t>(c0);                // c0 <= 16
  mask_t cuts = 0;                                     // positions that start a segment (they never die)
  uint32_t ftok = kTokNone;                            // my first live token word
  uint32_t succ_tok = kTokNone;                        // the token my last pair is looked up against
  uint32_t firstv = kNoRank, lastv = kNoRank;          // pair values at my first / last live position

  // ---- load: byte-level pre-tokenisation (section 4.1), id = byte value; the initial pair values, one
  //      lookup per adjacent byte pair in the direct 256 x 256 table; and the cuts ----
  {
    const int base = tid * d;
    uint32_t b[D + 2];                                 // b[j] = byte (base - 1 + j) of the string, 0x100 = none
#pragma unroll
    for (int j = 0; j < D + 2; ++j) {
      const int i = base - 1 + j;
      b[j] = (j <= c0 + 1 && c0 > 0 && i >= 0 && i < n) ? src[i] : 0x100u;
    }
    if constexpr (SPECIAL) {                           // special tokens are configured: their marks
      const uint8_t* mark = p.cover + begin;
#pragma unroll
      for (int j = 0; j < D + 2; ++j) {
        const int i = base - 1 + j;
        if (j <= c0 + 1 && c0 > 0 && i >= 0 && i < n) b[j] = cover_code(b[j], mark[i]);
      }
    }
    uint32_t raw[D + 1];                               // raw[j]: table entry of the pair (b[j], b[j+1])
#pragma unroll
    for (int j = 0; j < D + 1; ++j)
      raw[j] = (j <= c0 && b[j] < 0x100u && b[j + 1] < 0x100u) ? tab.byte_pair[(b[j] << 8) | b[j + 1]] : kCut;
    // raw[0] is the pair that ends at my first byte; the start of the string counts as a cut
    if (c0 > 0 && raw[0] == kCut) cuts |= 1u;
#pragma unroll
    for (int k = 0; k < D; ++k) {
      if (k < dpad) {                                  // positions from c0 on are dead from the start
        uint32_t v = k < c0 ? raw[k + 1] : kNoRank;
        if (v == kCut) {
          v = kNoRank;
          if (k + 1 < c0) cuts |= bit_at<mask_t>(k + 1);
        }
        V[k * W + tid] = v;
        if (LIMITS) L[k * W + tid] = limit20_of(v);
        // (no lane-dependent branches here: positions from c0 on just get a token word nobody reads)
        const uint32_t code = b[k + 1];
        uint32_t w = sh.byte_word[code & 0xFFu];
        if constexpr (SPECIAL) {
          w = (code & kCodeSpecial) ? p.special_base + (code & kCoverIndex) : w;
          live &= (code & kCodeRest) ? ~bit_at<mask_t>(k) : ~(mask_t)0;
        }
        T[k * W + tid] = w;
        if (k == 0) { ftok = c0 > 0 ? w : ftok; firstv = c0 > 0 ? v : firstv; }
        const bool last = k == c0 - 1;
        lastv = last ? v : lastv;
        const uint32_t after = sh.byte_word[b[k + 2] & 0xFFu];
        succ_tok = (last && b[k + 2] < 0x100u) ? after : succ_tok;
      }
    }
    if constexpr (SPECIAL) {                           // positions may be dead from the start
      cuts &= live;                                    // a segment starts at a token
      ftok = live ? T[ctz_bits<mask_t>(live) * W + tid] : kTokNone;
      firstv = live ? V[ctz_bits<mask_t>(live) * W + tid] : kNoRank;
      lastv = live ? V[top_bit<mask_t>(live) * W + tid] : kNoRank;
    }
  }
  const uint64_t cut_first = __ballot((cuts & 1u) != 0);   // lanes whose column starts a segment (for good)
  // cuts never move, so the grouping of the lanes for the horizon scans is fixed for the whole string
  const uint64_t cut_lanes = __ballot(cuts != 0);
  const uint32_t cuts_below = __builtin_amdgcn_mbcnt_hi((uint32_t)(cut_lanes >> 32),
                                                        __builtin_amdgcn_mbcnt_lo((uint32_t)cut_lanes, 0u));
  const uint32_t cuts_upto = cuts_below + (cuts ? 1u : 0u);                      // lanes <= me that hold a cut
  const uint32_t cuts_from = (uint32_t)__builtin_popcountll(cut_lanes) - cuts_below;   // lanes >= me
  const uint32_t fwd_group = (64u - cuts_upto) << 20, bwd_group = (64u - cuts_from) << 20;
  uint32_t not_row[3];                                 // lane constants of the suffix scan, kept in registers
  for (int r = 0; r < 3; ++r) {
    not_row[r] = (lane >> 4) == r ? 0u : 0xFFFFFFFFu;
    asm volatile("" : "+v"(not_row[r]));
  }
  const uint32_t cut_before = cuts_below ? kReset31 : 0u;                        // some lane before me has a cut
  const uint32_t cut_after = cuts_from - (cuts ? 1u : 0u) ? kReset31 : 0u;       // some lane after me
  const int first_cut = cuts ? ctz_bits<mask_t>(cuts) : 32;
  const int last_cut = cuts ? top_bit<mask_t>(cuts) : 32;   // 32: none, every position belongs to the head

  // ---- merge passes ----
  // Every pass removes at least one token, so n passes can never be needed; the bound only guarantees
  // that the loop ends whatever the memory contents.
  int buf = 0;                                         // which half of the double-buffered exchange is current
  for (int pass = 0; pass < n; ++pass) {
    // -- sweep: values and limits of my positions; minima inside my segments --
    // Per-position conditions are taken as 0 / all-ones words with bit-field extracts so that the running
    // minima are three or four vector instructions per position and no lane mask has to stay live.
    uint32_t v[D], e[D], f[D];                         // e[k]: limit of k, later the horizon of k's segment
#pragma unroll
    for (int g = 0; g < D; g += kGroup) {
      if (g < d) {
#pragma unroll
        for (int k = g; k < g + kGroup; ++k) {
          v[k] = V[k * W + tid];
          if (LIMITS) e[k] = L[k * W + tid];
        }
      }
    }
    uint32_t run = kInf20;                             // forward: minimum since my last cut so far
#pragma unroll
    for (int g = 0; g < D; g += kGroup) {
      if (g < d) {
#pragma unroll
        for (int k = g; k < g + kGroup; ++k) {
          if (!LIMITS) {                               // decoded on the fly; most positions hold no pair
            e[k] = kInf20;
            if (__ballot(v[k] != kNoRank)) e[k] = limit20_of(v[k]);
          }
          const uint32_t at_cut = (uint32_t)__builtin_amdgcn_sbfe((int)cuts, k, 1);   // all ones at a cut
          run = min(run | at_cut, e[k]);               // a cut restarts the minimum
          f[k] = run;
        }
      }
    }
    const uint32_t tail_min = run;                     // over my positions from my last cut on (all, if none)
    run = kInf20;                                      // backward: minimum up to the end of the segment
#pragma unroll
    for (int g = D - kGroup; g >= 0; g -= kGroup) {
      if (g < d) {
#pragma unroll
        for (int k = g + kGroup - 1; k >= g; --k) {
          const uint32_t at_cut = (uint32_t)__builtin_amdgcn_sbfe((int)cuts, k, 1);
          run = min(run, e[k]);
          e[k] = min(f[k], run);                       // minimum of the part of k's segment that is mine
          run |= at_cut;                               // the segment starts here: restart for the one before
        }
      }
    }
    const uint32_t head_min = min(run, kInf20);        // over my positions before my first cut (all, if none)

    // -- complete the segments that cross lanes: forward and backward segmented min-scans --
    // A lane's key is (64 - number of lanes with a cut up to it) above the minimum: a plain minimum over the
    // lanes before me then lands in the nearest group of lanes that share my segment, and picks its smallest.
    const uint32_t fwd_inc = wave_min_prefix(fwd_group | tail_min);
    const uint32_t bwd_inc = wave_min_suffix(bwd_group | head_min, not_row);
    uint32_t in_fwd = (wave_shift_up(fwd_inc, 0xFFFFFFFFu) & kInf20) | cut_before;
    uint32_t in_bwd = (wave_shift_down(bwd_inc, 0xFFFFFFFFu) & kInf20) | cut_after;

    // -- values just outside my column: the pair ending at my first token, the pair after my last --
    const uint64_t ne = __ballot(live != 0);
    const uint64_t below = ne & ((1ull << lane) - 1ull);
    const uint64_t above = lane == 63 ? 0ull : (ne >> (lane + 1)) << (lane + 1);
    uint32_t in_val = lane_read(lastv, below ? 63 - __builtin_clzll(below) : lane);
    uint32_t nxt_val = lane_read(firstv, above ? __builtin_ctzll(above) : lane);
    if (!below) in_val = kNoRank;
    if (!above) nxt_val = kNoRank;

    bool any_pair;
    if (NW == 1) {
      any_pair = true;                                 // decided below from the candidate masks
    } else {
      // any pair in my wave: some position has a finite limit
      uint32_t mine = kInf20;
#pragma unroll
      for (int g = 0; g < D; g += kGroup) {
        if (g < d) {
#pragma unroll
          for (int k = g; k < g + kGroup; ++k) mine = min(mine, e[k]);
        }
      }
      const uint64_t havep = __ballot(mine != kInf20);
      const int fl = ne ? __builtin_ctzll(ne) : 0, ll = ne ? 63 - __builtin_clzll(ne) : 0;
      const uint32_t fv = lane_read(firstv, fl), ft = lane_read(ftok, fl), lv = lane_read(lastv, ll);
      const uint32_t wave_flag = cut_lanes ? kReset31 : 0u;
      const uint32_t fwd_total = ((uint32_t)__builtin_amdgcn_readlane((int)fwd_inc, 63) & kInf20) | wave_flag;
      const uint32_t bwd_total = ((uint32_t)__builtin_amdgcn_readlane((int)bwd_inc, 0) & kInf20) | wave_flag;
      if (lane == 0) {
        SegRecord r;
        r.fwd = fwd_total;
        r.bwd = bwd_total;
        r.first_val = ne ? fv : kNoRank;
        r.last_val = ne ? lv : kNoRank;
        r.first_tok = ne ? ft : kTokNone;
        r.any_pair = havep ? 1u : 0u;
        r.pad0 = r.pad1 = 0;
        rec_base[buf * NW + wave] = r;
      }
      __syncthreads();                                 // records of all waves are in place
      const SegRecord* rec = rec_base + buf * NW;
      uint32_t anyp = 0, pre = kInf31, suf = kInf31;
#pragma unroll
      for (int w = 0; w < NW; ++w) anyp |= rec[w].any_pair;
      for (int w = 0; w < wave; ++w) pre = OpSegMin::apply(pre, rec[w].fwd);          // left to right
      for (int w = NW - 1; w > wave; --w) suf = OpSegMin::apply(suf, rec[w].bwd);      // right to left
      in_fwd = OpSegMin::apply(pre, in_fwd);
      in_bwd = OpSegMin::apply(suf, in_bwd);
      any_pair = uniform(anyp) != 0;
      if (!below) {
        for (int w = wave - 1; w >= 0; --w)            // nearest earlier non-empty wave
          if (rec[w].first_tok != kTokNone) { in_val = rec[w].last_val; break; }
      }
      if (!above) {
        for (int w = wave + 1; w < NW; ++w)            // nearest later non-empty wave
          if (rec[w].first_tok != kTokNone) { nxt_val = rec[w].first_val; break; }
      }
    }
    if (NW > 1 && !any_pair) break;                    // uniform: every wave read the same records

    // horizons of the segment that enters my column and of the one that leaves it
    const bool through = cuts == 0;
    const uint32_t e_head = min(min(in_fwd & kInf31, head_min), through ? (in_bwd & kInf31) : kInf31);
    const uint32_t e_tail = min(min(in_bwd & kInf31, tail_min), through ? (in_fwd & kInf31) : kInf31);

    // -- candidates: pairs whose rank is below their segment's horizon --
    // positions before my first cut take the entering segment's horizon, positions from my last cut on the
    // leaving segment's, the others the minimum found inside my column
    const mask_t head_pos = first_cut >= 32 ? ~(mask_t)0 : bits_below<mask_t>(first_cut);
    const mask_t tail_pos = last_cut >= 32 ? (mask_t)0 : ~bits_below<mask_t>(last_cut);
    mask_t cm = 0;
#pragma unroll
    for (int g = 0; g < D; g += kGroup) {
      if (g < d) {
#pragma unroll
        for (int k = g; k < g + kGroup; ++k) {
          const uint32_t in_head = (uint32_t)__builtin_amdgcn_sbfe((int)head_pos, k, 1);
          const uint32_t in_tail = (uint32_t)__builtin_amdgcn_sbfe((int)tail_pos, k, 1);
          uint32_t ek = (e_head & in_head) | (e[k] & ~in_head);
          ek = (e_tail & in_tail) | (ek & ~in_tail);
          // both sides are below 2^31, so the sign of the difference is the comparison
          cm |= (((v[k] >> kRankShift) - ek) >> 31) << k;
        }
      }
    }
    if (NW == 1 && !__ballot(cm != 0)) break;          // a segment with pairs always has a candidate

    // -- walk 1 over my candidates: which are beaten by a neighbour, and my element of the parity scan --
    // (see encode_string(); a candidate and the neighbour that beats it are always in the same segment,
    //  because the pair across a cut is not in the table)
    mask_t e0 = 0, lr = 0, nbr = 0;
    uint32_t elem = live ? 2u : 0u;                    // no trailing run: my last pair restarts the count
    if (__ballot(cm != 0)) {
      int prevc = -1;
      uint32_t prevv = 0, prev_dl = 0;
      bool prev_lead = false, prev_bl = false;
      for (mask_t m = cm; m; m &= m - 1) {
        const int k = ctz_bits<mask_t>(m);
        const uint32_t vk = V[k * W + tid];
        const mask_t lower = live & bits_below<mask_t>(k);
        bool bl, lead;
        uint32_t dl;
        if (lower) {
          const bool adjacent = top_bit<mask_t>(lower) == prevc;   // the live position before k is a candidate
          bl = adjacent && prevv <= vk;
          if (prevc >= 0 && !(adjacent && vk < prevv)) nbr |= bit_at<mask_t>(prevc);
          dl = bl ? (prev_dl ^ 1u) : 0u;
          lead = bl && prev_lead;
        } else {                                       // k is my first live position
          bl = in_val <= vk;                           // same segment and lower rank: a candidate too
          dl = bl ? 1u : 0u;
          lead = bl;
        }
        if (dl == 0) e0 |= bit_at<mask_t>(k);
        if (lead) lr |= bit_at<mask_t>(k);
        prevc = k;
        prevv = vk;
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
      uint32_t wave_total;
      uint32_t exc = wave_parity_exclusive(elem, lane, &wave_total);
      if (NW > 1) {
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
    // my first token is consumed if the pair ending at it is a candidate applied by the lane before me;
    // that pair belongs to the segment that enters my column
    const bool skip_first = live != 0 && (in_val >> kRankShift) < e_head && !(firstv < in_val) && pin == 0 && !(cuts & 1u);
    const bool touched = skip_first || applied != 0;
    mask_t dirty = 0;                                  // positions whose pair must be looked up again
    if (__ballot(touched)) {
      for (mask_t m = applied; m; m &= m - 1) {
        const int k = ctz_bits<mask_t>(m);
        T[k * W + tid] = merged_token_word(V[k * W + tid]);
        V[k * W + tid] = kNoRank;                      // until the new pair is looked up (if it needs to be)
        if (LIMITS) L[k * W + tid] = kInf20;
        const mask_t upper = live & bits_above<mask_t>(k);
        if (upper) {                                   // the right operand is mine: it dies
          const int kn = ctz_bits<mask_t>(upper);
          live &= ~bit_at<mask_t>(kn);
          V[kn * W + tid] = kNoRank;
          if (LIMITS) L[kn * W + tid] = kInf20;
        }                                              // else it is the next lane's first token (skip_first there)
        dirty |= bit_at<mask_t>(k);
        const mask_t lower = live & bits_below<mask_t>(k);
        if (lower) dirty |= bit_at<mask_t>(top_bit<mask_t>(lower));
      }
      if (skip_first) {
        const int fk = ctz_bits<mask_t>(live);
        live &= ~bit_at<mask_t>(fk);
        V[fk * W + tid] = kNoRank;
        if (LIMITS) L[fk * W + tid] = kInf20;
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
      // A pair that straddles a cut is in no table, so it needs no look-up (its value is "none" already).
      // In reversed bit order the live position before each cut is the first live bit above the cut, which
      // a carry finds for all cuts at once: add the cuts, shifted up, to the dead positions.
      const uint32_t rl = __builtin_bitreverse32(live), rc = __builtin_bitreverse32(cuts);
      mask_t cross = __builtin_bitreverse32((~rl + (rc << 1)) & rl);
      if (above2 && live != 0 && ((cut_first >> __builtin_ctzll(above2)) & 1ull))
        cross |= bit_at<mask_t>(top_bit<mask_t>(live));                // my last token and the next lane's first
      dirty &= ~cross;
    }

    // -- look up the pairs that changed, kProbes at a time --
    const bool refresh = touched || dirty != 0;
    while (__ballot(dirty != 0)) {
      int k[kProbes];
      uint32_t x[kProbes], y[kProbes];
      ProbeInFlight pf[kProbes];
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
      for (int j = 0; j < kProbes; ++j) probe_start(tab, x[j], y[j], k[j] >= 0, pf[j]);
#pragma unroll
      for (int j = 0; j < kProbes; ++j) {
        if (k[j] >= 0) {
          const uint32_t nv = probe_finish(tab, pf[j]);
          V[k[j] * W + tid] = nv;
          if (LIMITS) L[k[j] * W + tid] = limit20_of(nv);
        }
      }
    }
    if (refresh) {
      firstv = live ? V[ctz_bits<mask_t>(live) * W + tid] : kNoRank;
      lastv = live ? V[top_bit<mask_t>(live) * W + tid] : kNoRank;
    }
    buf ^= 1;
  }

  // ---- emit: prefix sum of live counts gives each lane's write index (section 4.3's compaction) ----
  uint32_t total;
  const uint32_t out0 = block_prefix_sum<NW>((uint32_t)pop_bits<mask_t>(live), sh, lane, wave, &total);
  int32_t* dst = p.tmp_ids + begin + out0;
  for (mask_t m = live; m; m &= m - 1) *dst++ = (int32_t)(T[ctz_bits<mask_t>(m) * W + tid] & kTokIdMask);
  if (tid == W - 1) p.counts[s] = (int32_t)total;
  block_sync<NW>();                                    // the LDS exchange arrays are reused by the next string
}

// Persistent workgroups: each claims the next string of its tier until the tier's list is exhausted.
// SEGMENTED selects encode_string_segmented() (LDS variants with at most 16 positions per lane); SPECIAL
// compiles in the reading of the special-token marks (EncodeParams::cover must then be set).
template <int NW, int D, bool STAGED, bool LIMITS, bool SEGMENTED, bool SPECIAL>
__global__ __launch_bounds__(NW * 64) void encode_kernel(EncodeParams p) {
  static_assert(!(SEGMENTED && STAGED), "the segmented encoder keeps its arrays in LDS");
  constexpr int W = NW * 64;
  extern __shared__ uint32_t smem[];
  uint32_t* cur = smem;
  uint32_t *T, *V, *L;
  if (STAGED) {
    T = p.staged + (size_t)blockIdx.x * ((LIMITS ? 3u : 2u) * W * D);
    V = T + W * D;
    L = V + W * D;
  } else {
    T = cur; cur += W * D;
    V = cur; cur += W * D;
    L = cur;
    if (LIMITS) cur += W * D;
  }
  // Work items: the first one is my workgroup index, later ones come from the tier's atomic counter (which
  // starts at zero and is offset by the grid size).  When the grid covers the whole list no atomic is needed.
  // (With a single variant in use and a grid that covers the batch there is no list at all: item = string.)
  const uint32_t first = p.list ? p.tier_base[p.tier] : 0u;
  const uint32_t count = p.list ? p.tier_base[p.tier + 1] - first : p.direct_count;
  if (blockIdx.x >= count) return;                     // uniform: nothing for this workgroup (often: an empty tier)
  BlockShared<NW> sh;
  sh.rec = (WaveRecord*)cur; cur += 2 * NW * 8;        // room for either record type
  sh.first_tok = cur; cur += 2 * NW;
  sh.part = cur; cur += 2 * NW;
  sh.item = cur; cur += 4;
  uint32_t* byte_word = cur;
  sh.byte_word = byte_word;
  for (int i = (int)threadIdx.x; i < 256; i += W) byte_word[i] = p.table.byte_word[i];

  // Warm this XCD's L2 with the merge table.  L2 contents do not survive a kernel boundary, so without this
  // every first probe of a bucket pays a trip to the Infinity Cache in the middle of a merge pass; here the
  // same lines come in as one bandwidth-bound stream while the first strings are still being loaded.
  // Workgroups are dealt to the 8 XCDs round robin, so workgroups b, b+8, b+16, ... share an L2 and split
  // the table between them.  (Only a hint: a different placement just makes it less effective.)
  if (p.prefetch_lines > 0) {
    constexpr uint32_t kXcds = 8;
    const uint32_t peers = (gridDim.x + kXcds - 1) / kXcds;            // workgroups that share my L2
    const uint32_t me = blockIdx.x / kXcds;
    const uint32_t per = (p.prefetch_lines + peers - 1) / peers;        // 128-byte lines for each of them
    const uint32_t lo = me * per, hi = min(lo + per, p.prefetch_lines);
    uint32_t sink = 0;
    for (uint32_t line = lo + threadIdx.x; line < hi; line += W)
      sink |= __builtin_nontemporal_load((const uint32_t*)p.table.buckets + (size_t)line * 32);
    if (sink == 0x9E3779B9u && p.prefetch_lines == 0xFFFFFFFFu) byte_word[0] = sink;   // keeps the loads alive
  }
  __syncthreads();

  uint32_t item = blockIdx.x;
  while (item < count) {
    const int s = p.list ? (int)uniform((uint32_t)p.list[first + item]) : (int)item;
    if constexpr (SEGMENTED) encode_string_segmented<NW, D, LIMITS, SPECIAL>(p, s, T, V, L, sh);
    else encode_string<NW, D, STAGED, LIMITS, SPECIAL>(p, s, T, V, L, sh);
    if (gridDim.x >= count) break;                     // uniform: one item per workgroup at most
    // Claim the next item.  Every lane of the first wave takes part in the atomic (lane 0 adds 1, the
    // others 0) so that no lane-dependent branch sits at the loop boundary: a branch on "thread 0" here,
    // next to a single-lane store that ends the previous string, lets the compiler send the other lanes
    // round the loop on their own, past the lane-0 broadcast below.
    uint32_t claimed = 0;
    if (NW == 1) {
      claimed = atomicAdd(p.queue_head + p.tier, threadIdx.x == 0 ? 1u : 0u);
    } else {
      if (threadIdx.x < 64) claimed = atomicAdd(p.queue_head + p.tier, threadIdx.x == 0 ? 1u : 0u);
      if (threadIdx.x == 0) *sh.item = claimed;
      __syncthreads();
      claimed = *sh.item;
      __syncthreads();
    }
    item = gridDim.x + uniform(claimed);               // lane 0's value, as a scalar
  }
}

// LDS is handed out in blocks, and the occupancy the runtime reports is for the bytes asked for: for 9,552 bytes it
// says seventeen workgroups per CU where sixteen are resident.  The seventeenth of every CU then starts when
// another one exits -- for persistent workgroups, when the work list is empty -- and runs its own first items
// alone at the end (measured: 6 % of the call on 8,192 strings of 4 KiB).  So the kernels ask for whole blocks,
// and the reported figure is the true one.
constexpr size_t kLdsBlockBytes = 1280;
constexpr size_t lds_blocks(size_t bytes) { return (bytes + kLdsBlockBytes - 1) / kLdsBlockBytes * kLdsBlockBytes; }

template <int NW, int D, bool STAGED, bool LIMITS>
constexpr size_t encode_lds_bytes() {
  return lds_blocks(sizeof(uint32_t) * ((STAGED ? 0 : (LIMITS ? 3 : 2) * NW * 64 * D) + 20 * NW + 4 + 256));
}

}  // namespace bpe
