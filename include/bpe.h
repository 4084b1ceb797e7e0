/* Byte-level BPE encoding of a batch of strings on one AMD MI355X (gfx950).
 *
 * C ABI of the hot path of BlockBPE (arXiv 2507.11941): given a merge table M (a list of token pairs, the
 * row index being the pair's rank -- Algorithm 1, "Require") and a batch of byte strings, return for every
 * string the token list T that Algorithm 1 ends with: start from the bytes, repeatedly replace the left-most
 * occurrence of the lowest-rank adjacent pair by its merged token, stop when no adjacent pair is in M.
 * A string -- or, for a long string, a piece of it cut where no merge can cross -- is encoded by one workgroup
 * (section 4.3: one block per string) that repeats section 4.2's steps (look up pair ranks, take the minimum,
 * merge, look up the new pairs) until no pair is left, independently for every stretch of the string that no
 * merge can leave.
 *
 * Token ids: a byte b is token b (byte-level pre-tokenisation, section 4.1); the token created by row r is
 * 256 + r.  Results are exact integers; there is nothing approximate in this interface.
 *
 * Every function returns one of the BPE_* codes below (0 = success) and none throws.  The library's only
 * process-wide state is a cache of kernel attributes, filled on the first encode, and the optional kernel
 * timing of bpe_set_profiling (off unless the caller switches it on).  Pointers are marked HOST or DEVICE; all
 * DEVICE pointers must belong to the device that was current when the table was built.
 */
#ifndef BPE_H_
#define BPE_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct bpe_table bpe_table; /* opaque; owns its device memory */

enum {
  BPE_OK = 0,
  BPE_EINVAL = -1,    /* null pointer, negative size, workspace too small, string longer than the maximum */
  BPE_EBADMERGE = -2, /* a row uses an id that does not exist before that row (id >= 256 + row) or < 0 */
  BPE_EDUPPAIR = -3,  /* the same (left,right) pair appears in two rows */
  BPE_ENOMEM = -4,    /* host or device allocation failed */
  BPE_EHIP = -5,      /* a HIP runtime call failed */
  BPE_ETOOBIG = -6,   /* more merges than the table format holds */
  BPE_EDUPID = -7,    /* bpe_build_table_vocab: two tokens of the vocabulary share an id */
  BPE_ESPECIAL = -8   /* bpe_table_set_specials: two special tokens could overlap in a text, or are the same */
};

/* Largest string (bytes) bpe_encode_batch accepts, and largest number of merge rows a table holds. */
#define BPE_MAX_STRING_BYTES 65536
#define BPE_MAX_MERGES 1048318 /* ids stay below 2^20 - 1 */
#define BPE_MAX_SPECIALS 64
#define BPE_MAX_SPECIAL_BYTES 64

/* Build the GPU-resident merge table (the map R of Algorithm 1: pair -> rank, O(1) lookup; section 4.3's
 * GPU hashmap).
 *   merges   HOST, int32[n_merges][2]: row r = (left_id, right_id), rank r, merged id 256 + r.
 *   n_merges >= 0.
 *   out      HOST, receives the table handle (NULL on error).
 *   bad_row  HOST, may be NULL; receives the first offending row on BPE_EBADMERGE / BPE_EDUPPAIR, else -1.
 * Validates that every row's operands are in [0, 256 + r) -- the property of any trained table under which
 * "apply every occurrence of the lowest rank per pass" equals Algorithm 1's one-at-a-time order -- and that
 * no pair repeats.  The rows are copied; the caller keeps `merges`.  Allocates device memory on the current
 * device and copies synchronously (this call is set-up, not hot path).
 */
int bpe_build_table(const int32_t* merges, int32_t n_merges, bpe_table** out, int32_t* bad_row);

/* The table bpe_build_table would upload, built in HOST memory instead (no device is touched): for callers
 * that want to inspect or cache it, and for tests of the builder.  Layout, in uint32 words:
 *   [buckets: 2^log2_buckets x 2 slots x {value, tag}] [token word of each byte: 256] [byte-pair table: 65536]
 * (section 4.3's hashmap; the format is described in paper_2507_11941_amd/csrc/table_format.h).
 *   merges, n_merges, bad_row  as for bpe_build_table (same validation, same codes).
 *   words         HOST, uint32[capacity]; may be NULL when capacity is 0 (size query).
 *   log2_buckets  HOST, may be NULL; receives log2 of the number of buckets.
 * Returns the number of words of the image (written only if it fits `capacity`), or a negative BPE_* code. */
int64_t bpe_table_image(const int32_t* merges, int32_t n_merges, uint32_t* words, int64_t capacity,
                        int32_t* log2_buckets, int32_t* bad_row);

/* Build the table over a vocabulary's own token ids (section 4.1: bytes are mapped to their initial token ids
 * by lookup; section 5.1 runs a pretrained tokenizer's vocabulary, whose ids are not "byte value" and
 * "256 + rank").  Same table, same encoding; only the numbering of the tokens differs:
 *   byte_ids    HOST, int32[256]: id of the single-byte token of each byte value; all distinct, >= 0.
 *   merges      HOST, int32[n_merges][2]: row r = (left_id, right_id) in vocabulary ids, rank r.  Each operand
 *               must be a byte id or the merged id of an EARLIER row (else BPE_EBADMERGE, bad_row = r).
 *   merged_ids  HOST, int32[n_merges]: id of the token row r creates; >= 0 and different from every byte id
 *               and every other row's merged id (else BPE_EDUPID, bad_row = r; -1 if two bytes collide).
 *   n_merges, out, bad_row: as for bpe_build_table.
 * bpe_encode_batch on such a table writes vocabulary ids to out_ids.  The arrays are copied. */
int bpe_build_table_vocab(const int32_t* byte_ids, const int32_t* merges, const int32_t* merged_ids,
                          int32_t n_merges, bpe_table** out, int32_t* bad_row);

/* Special tokens (section 4.1: special-character lookups identify BOS, EOS and the other reserved strings
 * before any merging).  After this call bpe_encode_batch treats every occurrence of one of the given byte
 * strings as a single token with the given id: the string is read left to right, where several specials match
 * the longest is taken, reading goes on after it, and the stretches in between are encoded by Algorithm 1 on
 * their own (no merge involves or crosses a special token).
 *   text          HOST, uint8: the specials' byte strings back to back.
 *   text_offsets  HOST, int32[n+1]: special i is text[text_offsets[i] .. text_offsets[i+1]), 1..64 bytes.
 *   ids           HOST, int32[n], >= 0: written to out_ids as given (they are not looked up in a vocabulary).
 *   n             0..BPE_MAX_SPECIALS; 0 removes the special tokens.
 * The set must be such that two occurrences can never overlap in any text: no special may contain, from an
 * offset > 0 on, another special or the beginning of one that runs past its end (BPE_ESPECIAL otherwise; the
 * usual reserved strings, bracketed by characters that occur nowhere inside them, satisfy this).  A special may
 * be the beginning of a longer one.  Set-up call: copies the arrays, allocates device memory, synchronous; the
 * caller must not run it while an encode that uses the table is enqueued or running. */
int bpe_table_set_specials(bpe_table* table, const uint8_t* text, const int32_t* text_offsets, const int32_t* ids,
                           int32_t n);

/* Release a table.  NULL is allowed.  The caller must have drained every stream that uses it. */
void bpe_free_table(bpe_table* table);

/* Number of merge rows of a table (0 for NULL). */
int32_t bpe_table_n_merges(const bpe_table* table);

/* Bytes of DEVICE workspace bpe_encode_batch needs for a batch of `batch` strings, `total_bytes` input
 * bytes in all, longest string `max_len` bytes.  Returns 0 for invalid arguments (negative sizes, max_len
 * above BPE_MAX_STRING_BYTES). */
size_t bpe_workspace_bytes(int32_t batch, int64_t total_bytes, int32_t max_len);

/* Encode a batch (Algorithm 1 per string; sections 4.2-4.3 for the parallel form).
 *   table        from bpe_build_table; read-only here, so concurrent calls on different streams are safe
 *                as long as each has its own workspace and outputs.
 *   bytes        DEVICE, uint8[total_bytes]: the strings back to back.
 *   offsets      DEVICE, int64[batch+1]: string i is bytes[offsets[i] .. offsets[i+1]); offsets[0] = 0,
 *                non-decreasing, offsets[batch] = total_bytes.  Any byte sequence is valid input.
 *   batch        number of strings, >= 0.
 *   total_bytes  offsets[batch], passed by the host so that the call needs no device-to-host read.
 *   max_len      an upper bound on the longest string, <= BPE_MAX_STRING_BYTES, passed by the host for the
 *                same reason.  It selects which kernel variants are launched.  Pass the true maximum: for a
 *                string longer than max_len the output is unspecified (it may be encoded, or contribute
 *                zero tokens); the other strings are unaffected and no out-of-bounds access happens.
 *   out_ids      DEVICE, int32, capacity >= total_bytes ids (a string never has more tokens than bytes).
 *   out_offsets  DEVICE, int64[batch+1].
 *   workspace    DEVICE, >= bpe_workspace_bytes(batch, total_bytes, max_len) bytes, 256-byte aligned,
 *                caller-owned; contents need not be initialised and are garbage afterwards.
 *   stream       a hipStream_t passed as void* (NULL = the default stream).
 * Only enqueues work on `stream`: no synchronisation, no allocation, no host reads of device data.  Once the
 * stream has drained: out_offsets[0] = 0 and out_ids[out_offsets[i] .. out_offsets[i+1]) is the encoding of
 * string i, dense and in batch order.  An empty string yields zero tokens.
 * Errors: BPE_EINVAL for null pointers with non-zero sizes, negative sizes, a short or misaligned workspace,
 * max_len out of range or a table of another device -- detected before anything is enqueued.  BPE_EHIP if the
 * runtime refuses a launch or an event record: kernels launched before the failing one may already be queued,
 * so the outputs and the workspace are then unspecified.
 */
int bpe_encode_batch(const bpe_table* table, const uint8_t* bytes, const int64_t* offsets, int32_t batch,
                     int64_t total_bytes, int32_t max_len, int32_t* out_ids, int64_t* out_offsets,
                     void* workspace, size_t workspace_bytes, void* stream);

/* bpe_encode_batch for callers that cannot allocate device memory or bring a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same result and same error
 * codes as bpe_encode_batch, without `workspace`: the kernels' scratch is a 24 MiB array that is part of the
 * library's device code (every GPU the library runs on holds one copy until the process ends).  Limits, beyond
 * which the call returns BPE_ETOOBIG and enqueues nothing: */
#define BPE_STATIC_MAX_BATCH 4096
#define BPE_STATIC_MAX_TOTAL_BYTES (4 << 20)
#define BPE_STATIC_MAX_STRING_BYTES 16384
/* The call allocates nothing and frees nothing (its first call on a device asks the runtime for the array's
 * address on that device).  All calls on one GPU share that GPU's array, so two such calls must not overlap in
 * time on one GPU -- enqueue them on one stream, or order the streams with events; calls that overlap race on
 * the scratch and their outputs are unspecified.  Nothing in the array has to survive from call to call: the
 * kernels reset the counters they use. */
int bpe_encode_batch_static(const bpe_table* table, const uint8_t* bytes, const int64_t* offsets, int32_t batch,
                            int64_t total_bytes, int32_t max_len, int32_t* out_ids, int64_t* out_offsets,
                            void* stream);

/* Timing of the per-string encode kernels alone (not the binning, offset-scan or packing kernels), for
 * roofline accounting.  bpe_set_profiling(1) is a set-up call: it creates 512 pairs of HIP events (once per
 * process), clears the record and switches the timing on; from then on every bpe_encode_batch, up to 512 calls,
 * records one of those pairs on its own stream around its encode kernels (nothing is created or allocated in
 * bpe_encode_batch).  bpe_set_profiling(0) switches it off, which is the default.  This state is process-wide
 * and guarded by a mutex; switch it on only while measuring.  Returns BPE_EHIP if the events cannot be made. */
int bpe_set_profiling(int enabled);

/* Sum of the recorded encode-kernel durations in milliseconds and the number of calls recorded since
 * profiling was switched on.  total_ms, calls: HOST.  Waits for the recorded events to complete. */
int bpe_read_profile(float* total_ms, int32_t* calls);

/* Human-readable text for a BPE_* code. */
const char* bpe_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* BPE_H_ */
