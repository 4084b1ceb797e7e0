// Layout of the GPU-resident merge table (the pair -> rank map of Algorithm 1; section 4.3's hashmap).
//
// The table is static after it is built, so it needs no concurrent insert: it is a bucketed
// open-addressing array tuned for the probe the merge passes issue -- one pair, usually absent.
//
//   * Placement.  The pair (a, b), ids < 2^20, goes through a two-round Feistel permutation of its 40 bits
//     (any round function gives a bijection).  The low log2(buckets) bits of the result choose the bucket,
//     the remaining 40 - log2(buckets) bits are the fingerprint stored in the slot; bucket and fingerprint
//     together identify the pair exactly, so a fingerprint match is never a false positive.
//   * A slot is 8 bytes:  hi = tag = fingerprint (< 2^30) | displacement << 30,  lo = value.  An empty slot
//     is all ones.
//   * A bucket is 4 slots = 32 bytes, fetched with two 16-byte loads issued together, so a probe costs one
//     memory round trip.  Slots fill a bucket front to back; a key that finds its home bucket full goes to
//     the next bucket or the one after (displacement 1 or 2, recorded in the tag so that a displaced key
//     cannot be mistaken for a key at home there); the builder grows the table if that is not enough.
//     A lookup stops at the first bucket whose last slot is empty, or after displacement 2.
//   * Load is kept <= 0.4 (4 * buckets >= 2.5 * rows), so for 100,000 rows the table is 2 MiB and stays
//     resident in each XCD's 4 MiB L2.
//
// The value describes the row and the token it creates, so a merge pass needs no second lookup:
//   bits 12..31  rank (row index); the merged token id is 256 + rank
//   bits  4..11  horizon code: a lower bound, as a floating-point-like 8-bit code, on how many ranks lie
//                between this row and the first later row that uses the merged token as an operand
//                (255 = the merged token is never an operand)
//   bit  1       the merged token occurs as the LEFT operand of some later row
//   bit  2       the merged token occurs as the RIGHT operand of some later row
// Rank sits on top, so comparing values orders pairs by rank, and equal values mean equal rows.
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
constexpr uint32_t kFlagLeft = 2u;
constexpr uint32_t kFlagRight = 4u;
constexpr int kRankShift = 12;
constexpr int kHorizonShift = 4;
constexpr int kSlotsPerBucket = 4;
constexpr int kMinLog2Buckets = 10;           // fingerprints must fit 30 bits
constexpr int kMaxLog2Buckets = 20;
constexpr uint32_t kMaxDisplacement = 2;      // tag value 3 << 30 is left to the empty marker

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

BPE_HD Placement place_pair(uint32_t a, uint32_t b, int log2_buckets) {
  const uint32_t b2 = b ^ ((a * 0x9E3779B1u) >> 12);          // 20 bits
  const uint32_t a2 = a ^ ((b2 * 0x85EBCA77u) >> 12);         // 20 bits
  Placement p;
  p.bucket = a2 & ((1u << log2_buckets) - 1u);
  p.fingerprint = ((a2 >> log2_buckets) << 20) | b2;
  return p;
}

BPE_HD uint32_t slot_tag(uint32_t fingerprint, uint32_t displacement) { return fingerprint | (displacement << 30); }

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
