// Layout of the GPU-resident merge table (the pair -> rank map of Algorithm 1; section 4.3's hashmap).
//
// The table is static after it is built, so it needs no concurrent insert: it is a bucketed array tuned for
// the probe the merge passes issue -- one pair per lane, usually absent, 64 lanes at once, and the wave waits
// for the slowest lane.  What counts is therefore that a lookup is ONE memory round trip for (nearly) every
// lane, whether the pair is present or not.
//
//   * Placement.  The pair (a, b), ids < 2^20, goes through a two-round Feistel permutation of its 40 bits
//     (any round function gives a bijection; the rounds use 24-bit multiplies, which run at full rate).  The
//     low log2(buckets) bits of the result choose the bucket, the remaining 40 - log2(buckets) bits are the
//     fingerprint stored in the slot; bucket and fingerprint together identify the pair exactly, so a
//     fingerprint match is never a false positive.
//   * A slot is 8 bytes:  hi = tag = fingerprint (< 2^27) | displacement << 28,  lo = value.  An empty slot is
//     all ones.
//   * A bucket is 2 slots = 16 bytes: ONE 16-byte load per lane.  (The kernels that use the table are bound by
//     the number of accesses the L1 has to process, not by the bytes.)  Eight buckets share a 128-byte line.  A
//     key that finds its home bucket full goes to bucket ^ 1, ^ 2, ... ^ 15 -- the first of the line's other
//     buckets that has room, then of the neighbouring line's -- with that displacement recorded in its tag, so
//     that it cannot be mistaken for a key at home there; the largest displacement any key of a bucket has is
//     kept in spare value bits of the bucket's own two slots (bits 0..1 of each).  The builder doubles the
//     table in the (unseen) case that both lines are full.  A lookup reads the home bucket and, only if the key
//     is not there and that number is not zero, the buckets up to that displacement: those reads mostly hit
//     the L1, which the first read has filled with the line.
//   * Load is kept <= 0.4 (2 * buckets >= 2.5 * rows), so for 100,000 rows the table is 2 MiB and stays
//     resident in each XCD's 4 MiB L2; one lookup in twenty needs a second read.
//
// The value describes the row and the token it creates, so a merge pass needs no second lookup:
//   bits 12..31  rank (row index); the merged token id is 256 + rank
//   bit  10      the merged token occurs as the LEFT operand of some later row
//   bit  11      the merged token occurs as the RIGHT operand of some later row
//   bits  2..9   horizon code: a lower bound, as a floating-point-like 8-bit code, on how many ranks lie
//                between this row and the first later row that uses the merged token as an operand
//                (255 = the merged token is never an operand)
//   bits  0..1   spare: the bucket's largest displacement, see above
// Rank sits on top, so comparing values orders pairs by rank, and equal values mean equal rows (lookups return
// the value with bits 0..1 cleared).
//
// The horizon is what lets one pass apply many ranks at once.  Let limit(row) = rank + 1 + decode(code)
// <= the first rank at which the row's token can take part in a merge.  If E is the minimum of limit()
// over all pairs currently present in a string, every pair that can still be created has rank >= E (it
// contains a token made by a present or later pair, and rows only use older tokens), so all present pairs
// with rank < E can be resolved among themselves in one pass.
#pragma once
#include <stdint.h>

#if defined(__HIPCC__)
#define BPE_HD __host__ __device__ inline
#else
#define BPE_HD inline
#endif

namespace bpe {

constexpr uint32_t kNoRank = 0xFFFFFFFFu;     // "pair not in table"; larger than any value
constexpr uint32_t kCut = 0xFFFFFFFDu;        // byte-pair table only: not a pair, and no token spans this bigram
constexpr uint32_t kNoLimit = 0xFFFFFFFEu;    // limit of a row whose token is never an operand
constexpr uint32_t kFlagLeft = 1u << 10;
constexpr uint32_t kFlagRight = 1u << 11;
constexpr int kRankShift = 12;
constexpr int kHorizonShift = 2;
constexpr uint32_t kValueSpare = 3u;          // value bits that hold a bucket's largest displacement
constexpr int kSlotsPerBucket = 2;
constexpr int kMinLog2Buckets = 13;           // fingerprints must fit 27 bits (a tag can then never be all ones)
constexpr int kMaxLog2Buckets = 22;
constexpr uint32_t kMaxDisplacement = 15;     // the buckets of two adjacent 128-byte lines
constexpr int kTagDisplacementShift = 28;

// Token word kept per position by the kernels: id in the low 20 bits plus two capability bits that let a
// probe be skipped when the left token is never a left operand or the right token never a right operand.
constexpr uint32_t kTokIdMask = 0xFFFFFu;
constexpr uint32_t kTokCanLeft = 1u << 30;
constexpr uint32_t kTokCanRight = 1u << 31;
constexpr uint32_t kTokNone = 0xFFFFFFFFu;    // "no token" marker (id field all ones is never a valid id)

// Marks of the special-token pass (section 4.1's special-character lookup), one per input byte: 0 for ordinary
// text, kCoverFirst | index on the first byte of an occurrence of special `index`, kCoverRest on its other bytes.
constexpr uint32_t kCoverRest = 0x40u, kCoverFirst = 0x80u, kCoverIndex = 0x3Fu;

struct Placement {
  uint32_t bucket;
  uint32_t fingerprint;
};

// Low 32 bits of the product of two 24-bit numbers (one full-rate instruction on the GPU).
BPE_HD uint32_t mul24(uint32_t x, uint32_t y) {
#if defined(__HIP_DEVICE_COMPILE__)
  return __umul24(x, y);
#else
  return (uint32_t)((uint64_t)(x & 0xFFFFFFu) * (uint64_t)(y & 0xFFFFFFu));
#endif
}

BPE_HD Placement place_pair(uint32_t a, uint32_t b, int log2_buckets) {
  const uint32_t b2 = b ^ (mul24(a, 0x9E3779u) >> 12);        // 20 bits
  const uint32_t a2 = a ^ (mul24(b2, 0x85EBCBu) >> 12);       // 20 bits
  Placement p;
  p.bucket = a2 & ((1u << log2_buckets) - 1u);
  p.fingerprint = ((a2 >> log2_buckets) << 20) | b2;
  return p;
}

BPE_HD uint32_t slot_tag(uint32_t fingerprint, uint32_t displacement) {
  return fingerprint | (displacement << kTagDisplacementShift);
}
// Largest displacement among the keys whose home is the bucket with these two slot values (a full bucket).
BPE_HD uint32_t bucket_reach(uint32_t value0, uint32_t value1) { return (value0 & 3u) | ((value1 & 3u) << 2); }

// Horizon code: e = code >> 4, m = code & 15; decode = m for e == 0, else (16 + m) << (e - 1).
BPE_HD uint32_t horizon_decode(uint32_t code) {
  const uint32_t e = code >> 4, m = code & 15u;
  return e ? ((16u | m) << (e - 1u)) : m;
}
// Largest code in 0..254 whose decoded value does not exceed delta.
BPE_HD uint32_t horizon_encode(uint32_t delta) {
  uint32_t lo = 0, hi = 254;
  while (lo < hi) {
    const uint32_t mid = (lo + hi + 1) / 2;
    if (horizon_decode(mid) <= delta) lo = mid; else hi = mid - 1;
  }
  return lo;
}

BPE_HD uint32_t make_value(uint32_t rank, uint32_t horizon_code, bool can_left, bool can_right) {
  return (rank << kRankShift) | (horizon_code << kHorizonShift) | (can_left ? kFlagLeft : 0u) |
         (can_right ? kFlagRight : 0u);
}

// First rank at which the token made by this row can be merged again (a lower bound), kNoLimit if never.
BPE_HD uint32_t limit_of(uint32_t value) {
  const uint32_t code = (value >> kHorizonShift) & 0xFFu;
  return code == 255u ? kNoLimit : (value >> kRankShift) + 1u + horizon_decode(code);
}

// Token word of the token a row creates, from the row's value.
BPE_HD uint32_t merged_token_word(uint32_t value) {
  return (256u + (value >> kRankShift)) | ((value & kFlagLeft) ? kTokCanLeft : 0u) |
         ((value & kFlagRight) ? kTokCanRight : 0u);
}

}  // namespace bpe
