// Layout of the GPU-resident merge table (the pair -> rank map of Algorithm 1; section 4.3's hashmap).
//
// The table is static after it is built, so it needs no concurrent insert: it is a bucketed
// open-addressing array tuned for the probe the merge passes issue -- one pair, usually absent.
//
//   * A slot is 8 bytes:  hi = left_id << 12 | right_id >> 8,   lo = (right_id & 0xFF) << 24 | value,
//     ids are < 2^20 - 1, value = rank << 4 | flags (24 bits).  An empty slot is all ones (no valid key
//     has hi == 0xFFFFFFFF).
//   * A bucket is 4 slots = 32 bytes, fetched with two 16-byte loads issued together, so a probe costs one
//     memory round trip.  Slots fill a bucket front to back; a key that finds its home bucket full goes to
//     the next bucket.  A lookup stops at the first bucket whose last slot is empty.
//   * Load is kept <= 0.4 (4 * buckets >= 2.5 * rows), so for 100,000 rows the table is 2 MiB and stays
//     resident in each XCD's 4 MiB L2.
//
// The value's low bits describe the merged token so a pass needs no second lookup:
//   bit 0  the pair is a self pair (left == right): overlapping occurrences must be resolved
//   bit 1  the merged token occurs as the LEFT operand of some later row
//   bit 2  the merged token occurs as the RIGHT operand of some later row
// Because flags sit below the rank, comparing values orders pairs by rank, and equal values mean equal rows.
#pragma once
#include <stdint.h>

#if defined(__HIPCC__)
#define BPE_HD __host__ __device__ inline
#else
#define BPE_HD inline
#endif

namespace bpe {

constexpr uint32_t kNoRank = 0xFFFFFFFFu;     // "pair not in table"; larger than any value
constexpr uint32_t kFlagSelf = 1u;
constexpr uint32_t kFlagLeft = 2u;
constexpr uint32_t kFlagRight = 4u;
constexpr int kFlagBits = 4;
constexpr int kSlotsPerBucket = 4;

// Token word kept per position by the kernels: id in the low 20 bits plus two capability bits that let a
// probe be skipped when the left token is never a left operand or the right token never a right operand.
constexpr uint32_t kTokIdMask = 0xFFFFFu;
constexpr uint32_t kTokCanLeft = 1u << 30;
constexpr uint32_t kTokCanRight = 1u << 31;
constexpr uint32_t kTokNone = 0xFFFFFFFFu;    // "no token" marker (id field all ones is never a valid id)

BPE_HD uint32_t hash_pair(uint32_t a, uint32_t b) { return a * 0x9E3779B1u + b * 0x85EBCA77u; }
BPE_HD uint32_t bucket_of(uint32_t a, uint32_t b, int log2_buckets) {
  uint32_t h = hash_pair(a, b);
  h ^= h >> 15;
  return (h * 0x2C1B3C6Du) >> (32 - log2_buckets);
}
BPE_HD uint32_t slot_hi(uint32_t a, uint32_t b) { return (a << 12) | (b >> 8); }
BPE_HD uint32_t slot_lo(uint32_t b, uint32_t value) { return ((b & 0xFFu) << 24) | value; }

// Token word of the token a row creates, from the row's value.
BPE_HD uint32_t merged_token_word(uint32_t value) {
  return (256u + (value >> kFlagBits)) | ((value & kFlagLeft) ? kTokCanLeft : 0u) |
         ((value & kFlagRight) ? kTokCanRight : 0u);
}

}  // namespace bpe
