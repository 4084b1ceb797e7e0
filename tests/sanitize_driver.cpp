// Exercises every entry point of the CPU oracle and of the workload generators in one process, for a build with
// AddressSanitizer and UndefinedBehaviorSanitizer (tests/test_sanitizers.py compiles this file together with
// oracle/bpe_oracle.cpp and workloads/gen.cpp and runs it).  Prints a checksum; any sanitizer report aborts.
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <vector>

extern "C" {
void* orc_table_new(const int32_t* merges, int32_t n_merges);
void* orc_table_new_vocab(const int32_t* byte_ids, const int32_t* merges, const int32_t* merged_ids, int32_t n_merges);
void orc_table_free(void* h);
void orc_table_set_specials(void* h, const uint8_t* text, const int32_t* offsets, const int32_t* ids, int32_t n);
int64_t orc_encode(const void* h, int tier, const uint8_t* s, int64_t n, int32_t* out, int64_t* stats);
int64_t orc_pass_trace(const void* h, const uint8_t* s, int64_t n, int64_t* trace, int64_t capacity);
int64_t orc_encode_batch(const void* h, int tier, const uint8_t* bytes, const int64_t* offsets, int64_t batch,
                         int nthreads, int32_t* out_ids, int64_t* out_offsets, int64_t* stats);
int64_t orc_decode(const void* h, const int32_t* ids, int64_t k, uint8_t* out, int64_t cap);
int64_t orc_train(const uint8_t* corpus, int64_t n, int32_t n_merges, int32_t* out, int naive);
int wl_text(int style, uint64_t seed, uint8_t* out, int64_t nbytes);
int wl_adversarial(uint64_t seed, uint8_t* out, int64_t nstrings, int64_t len);
int wl_lognormal_lengths(uint64_t seed, int64_t* out, int64_t count, double median, double sigma, int64_t lo,
                         int64_t hi);
}

int main() {
  uint64_t sum = 0;
  // generators: every text style, the adversarial strings, the length mix
  std::vector<uint8_t> corpus(96 * 1024);
  for (int style = 1; style <= 3; ++style) {
    if (wl_text(style, 1000 + (uint64_t)style, corpus.data(), (int64_t)corpus.size()) != 0) return 2;
    for (uint8_t b : corpus) sum = sum * 31 + b;
  }
  std::vector<uint8_t> adv(8 * 2048);
  if (wl_adversarial(0, adv.data(), 8, 2048) != 0) return 2;
  std::vector<int64_t> lens(500);
  if (wl_lognormal_lengths(0, lens.data(), 500, 2048.0, 1.0, 64, 65536) != 0) return 2;
  for (int64_t l : lens) sum = sum * 31 + (uint64_t)l;

  // trainer, both ways, on a small corpus
  if (wl_text(2, 7, corpus.data(), 32 * 1024) != 0) return 2;
  std::vector<int32_t> rows(2 * 300), rows_naive(2 * 40);
  const int64_t n_rows = orc_train(corpus.data(), 32 * 1024, 300, rows.data(), 0);
  const int64_t n_naive = orc_train(corpus.data(), 4 * 1024, 40, rows_naive.data(), 1);
  if (n_rows <= 0 || n_naive <= 0) return 3;
  void* table = orc_table_new(rows.data(), (int32_t)n_rows);

  // all four encoders, the pass trace, the decoder; empty, one-byte and ragged strings
  std::vector<int32_t> ids(4096), ref(4096);
  std::vector<uint8_t> back(4096);
  std::vector<int64_t> trace(3 * 4096);
  for (int64_t n : {0, 1, 2, 17, 300, 1500}) {
    int64_t stats[3];
    const int64_t k = orc_encode(table, 1, corpus.data() + 5, n, ref.data(), nullptr);
    for (int tier : {0, 2, 3}) {
      if (n > 300 && tier == 0) continue;          // the brute force is cubic
      const int64_t kk = orc_encode(table, tier, corpus.data() + 5, n, ids.data(), stats);
      if (kk != k || std::memcmp(ids.data(), ref.data(), (size_t)k * 4) != 0) return 4;
    }
    if (orc_pass_trace(table, corpus.data() + 5, n, trace.data(), 4096) < 0) return 4;
    if (orc_decode(table, ref.data(), k, back.data(), 4096) != n || std::memcmp(back.data(), corpus.data() + 5, (size_t)n))
      return 5;
    sum = sum * 31 + (uint64_t)k;
  }
  // batch entry point on several threads, on text and on the adversarial strings
  {
    std::vector<int64_t> off = {0, 0, 1, 700, 700, 2048, 4096, 16384};
    std::vector<int32_t> out(16384);
    std::vector<int64_t> out_off(off.size());
    int64_t stats[3];
    for (int tier : {1, 2, 3})
      sum = sum * 31 + (uint64_t)orc_encode_batch(table, tier, adv.data(), off.data(), (int64_t)off.size() - 1, 4,
                                                  out.data(), out_off.data(), stats);
  }
  // special tokens and a vocabulary with its own ids
  {
    const uint8_t text[] = "<|eot|><|pad|>";
    const int32_t offs[] = {0, 7, 14}, sids[] = {9000, 9001};
    orc_table_set_specials(table, text, offs, sids, 2);
    const uint8_t s[] = "ab<|eot|>cd<|pad|><|eot|";
    sum = sum * 31 + (uint64_t)orc_encode(table, 1, s, (int64_t)sizeof(s) - 1, ids.data(), nullptr);
    orc_table_set_specials(table, nullptr, offs, nullptr, 0);
    int32_t byte_ids[256], merged[2] = {5, 3};
    for (int b = 0; b < 256; ++b) byte_ids[b] = 1000 + 255 - b;
    const int32_t vrows[4] = {1000 + 255 - 'a', 1000 + 255 - 'b', 5, 1000 + 255 - 'c'};
    void* vocab = orc_table_new_vocab(byte_ids, vrows, merged, 2);
    const uint8_t t[] = "abcab";
    const int64_t k = orc_encode(vocab, 3, t, 5, ids.data(), nullptr);
    if (k != 2 || ids[0] != 3 || ids[1] != 5) return 6;
    if (orc_decode(vocab, ids.data(), k, back.data(), 4096) != 5 || std::memcmp(back.data(), t, 5)) return 6;
    orc_table_free(vocab);
  }
  orc_table_free(table);
  std::printf("sanitize_driver ok %llu\n", (unsigned long long)sum);
  return 0;
}
