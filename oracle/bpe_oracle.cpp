// CPU ORACLE for byte-level BPE encoding -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
//
// Plain, slow, obviously-correct implementations of what the GPU path must compute, written from the
// paper (BlockBPE, arXiv 2507.11941).  Nothing here is shared with, included by, or linked into the HIP
// library; only the tests, the smoke check and the benchmark's cpu-baseline leg may call it.
//
// What is defined where:
//   * encode_bruteforce  -- Algorithm 1 ("BPE Tokenization with Merge Table", section 3.1) step by step:
//                           rebuild the list of adjacent pairs, take the pair with the lowest rank, replace
//                           its left-most occurrence, repeat until no adjacent pair is in the table.
//                           O(n^2 log) -- tiny inputs only.  THE DEFINITION.
//   * encode_textbook    -- the same result with the pair ranks cached per position: linear scan for the
//                           minimum (first index on ties), merge that one occurrence, recompute the two
//                           neighbouring ranks (section 3.1's O(n^2) procedure).
//   * encode_passes      -- section 4.2's pass view: per pass find the lowest rank present, then sweep left
//                           to right merging every occurrence of that pair and skipping the token just
//                           consumed.  Also counts passes and live-token visits (the work model O(n d) of
//                           section 4.2 needs them).
//   * encode_heap        -- the priority-queue scheme section 3.2 attributes to CPU libraries
//                           (O(n log n)): heap of (rank, position) over a doubly linked token list.  Used
//                           only where the quadratic encoders are too slow; admitted by agreeing with them.
//   * decode             -- expands ids back to bytes (a byte's id is a byte, a row's id is the row's pair).
//   * train / train_naive-- greedy most-frequent-pair trainer.  The paper uses pretrained tables
//                           (sections 5.1, 5.2), so the trainer is this build's own definition:
//                           chunk the corpus before every whitespace byte (space, tab, LF, CR), count
//                           distinct chunks; repeat: count every adjacent pair position in every chunk
//                           weighted by chunk frequency, take the highest count (ties: smallest
//                           (left,right) lexicographically), append it as the next row (rank = row index,
//                           merged id = 256 + rank), apply it in every chunk left to right without overlap.
//
// Conventions: a merge table is n rows of (left_id, right_id) int32; token ids are int32; a string is any
// byte sequence (byte-level pre-tokenisation, section 4.1: initial id = the vocabulary's id of the byte, the
// byte value itself unless a vocabulary is given; a row's merged token is 256 + rank unless a vocabulary
// names it).
//
// Parity pins (tests/test_oracle_*.py): hand-worked examples, closed forms for doubling chains and
// alternating pairs, brute force on exhaustive small alphabets, round trip and fixed-point invariants.
// The trainer has no external pin beyond its own definition (naive recount == incremental, first row ==
// most frequent pair by direct count): its "parity" is unpinned by the paper, and it only selects which
// table is used -- it never enters the GPU-vs-oracle comparison.

#include <algorithm>
#include <atomic>
#include <cstdint>
#include <cstring>
#include <map>
#include <queue>
#include <string>
#include <thread>
#include <unordered_map>
#include <utility>
#include <vector>

namespace {

constexpr int32_t kNoRank = INT32_MAX;

inline uint64_t pair_key(int32_t a, int32_t b) { return ((uint64_t)(uint32_t)a << 32) | (uint32_t)b; }

struct Table {
  std::vector<std::pair<int32_t, int32_t>> rows;   // row index = rank
  std::unordered_map<uint64_t, int32_t> rank;      // (a,b) -> rank     (map R of Algorithm 1)
  std::map<std::pair<int32_t, int32_t>, int32_t> rank_ordered;  // same content, used by the brute force
  // Vocabulary (section 4.1: bytes are mapped to their initial token ids by lookup; a merge yields the id the
  // vocabulary gives the merged token).  Default: byte b has id b, row r creates id 256 + r.
  int32_t byte_id[256];
  std::vector<int32_t> merged_id;                  // [rows]
  std::unordered_map<int32_t, int32_t> byte_of_id, row_of_id;   // inverse, for decode

  // Special tokens (section 4.1: special-character lookups identify BOS / EOS and the other reserved strings
  // before any merging): byte strings that become one token each.
  std::vector<std::string> special_text;
  std::vector<int32_t> special_id;

  std::vector<int32_t> initial(const uint8_t* s, int64_t n) const {   // "split S into a list of bytes"
    std::vector<int32_t> T((size_t)n);
    for (int64_t i = 0; i < n; ++i) T[(size_t)i] = byte_id[s[i]];
    return T;
  }

  int32_t lookup(int32_t a, int32_t b) const {
    auto it = rank.find(pair_key(a, b));
    return it == rank.end() ? kNoRank : it->second;
  }
};

// ---------------------------------------------------------------------------------------------------
// Algorithm 1, literally.
std::vector<int32_t> encode_bruteforce(const Table& t, const uint8_t* s, int64_t n) {
  std::vector<int32_t> T = t.initial(s, n);               // split S into a list of bytes
  while (true) {
    int32_t best = kNoRank;
    std::pair<int32_t, int32_t> best_pair{0, 0};
    for (size_t i = 0; i + 1 < T.size(); ++i) {           // all adjacent pairs
      auto it = t.rank_ordered.find({T[i], T[i + 1]});
      if (it != t.rank_ordered.end() && it->second < best) {
        best = it->second;
        best_pair = it->first;
      }
    }
    if (best == kNoRank) break;                            // no pair of T is in the table
    for (size_t i = 0; i + 1 < T.size(); ++i) {           // left-most occurrence of (a,b)
      if (T[i] == best_pair.first && T[i + 1] == best_pair.second) {
        T[i] = t.merged_id[(size_t)best];
        T.erase(T.begin() + (std::ptrdiff_t)i + 1);
        break;
      }
    }
  }
  return T;
}

// Textbook sequential encoder: cached ranks, one merge per iteration.
std::vector<int32_t> encode_textbook(const Table& t, const uint8_t* s, int64_t n) {
  std::vector<int32_t> T = t.initial(s, n);
  std::vector<int32_t> R;                                  // R[i] = rank of (T[i], T[i+1])
  for (size_t i = 0; i + 1 < T.size(); ++i) R.push_back(t.lookup(T[i], T[i + 1]));
  while (true) {
    int32_t best = kNoRank;
    size_t at = 0;
    for (size_t i = 0; i < R.size(); ++i) {
      if (R[i] < best) { best = R[i]; at = i; }            // strict <: first index wins ties
    }
    if (best == kNoRank) break;
    T[at] = t.merged_id[(size_t)best];
    T.erase(T.begin() + (std::ptrdiff_t)at + 1);
    R.erase(R.begin() + (std::ptrdiff_t)at);               // the pair that was merged
    if (at > 0) R[at - 1] = t.lookup(T[at - 1], T[at]);
    if (at + 1 < T.size()) R[at] = t.lookup(T[at], T[at + 1]);
  }
  return T;
}

struct PassStats {
  int64_t passes = 0;        // number of merge passes (distinct ranks applied)
  int64_t visits = 0;        // sum over passes of the live token count at the start of the pass
  int64_t merges = 0;        // total merges applied
  // what each pass did, for the checks of the pass invariants (kept only when asked for):
  bool keep_trace = false;
  std::vector<int64_t> trace;   // per pass: rank applied, live tokens at its start, merges it applied
};

// Pass view of section 4.2: one rank per pass, every non-overlapping occurrence, left-most first.
std::vector<int32_t> encode_passes(const Table& t, const uint8_t* s, int64_t n, PassStats* st) {
  std::vector<int32_t> T = t.initial(s, n);
  while (true) {
    int32_t best = kNoRank;
    for (size_t i = 0; i + 1 < T.size(); ++i) best = std::min(best, t.lookup(T[i], T[i + 1]));
    if (best == kNoRank) break;
    const int32_t a = t.rows[(size_t)best].first, b = t.rows[(size_t)best].second;
    if (st) { st->passes += 1; st->visits += (int64_t)T.size(); }
    const size_t live_before = T.size();
    int64_t merges_before = st ? st->merges : 0;
    std::vector<int32_t> next;
    next.reserve(T.size());
    size_t i = 0;
    while (i < T.size()) {
      if (i + 1 < T.size() && T[i] == a && T[i + 1] == b) {
        next.push_back(t.merged_id[(size_t)best]);
        i += 2;                                            // the right token is consumed
        if (st) st->merges += 1;
      } else {
        next.push_back(T[i]);
        i += 1;
      }
    }
    if (st && st->keep_trace) {
      st->trace.push_back(best);
      st->trace.push_back((int64_t)live_before);
      st->trace.push_back(st->merges - merges_before);
    }
    T.swap(next);
  }
  return T;
}

// Priority-queue encoder (section 3.2): heap ordered by (rank, position of the left token).
std::vector<int32_t> encode_heap(const Table& t, const uint8_t* s, int64_t n) {
  struct Entry {
    int32_t rank; int64_t left; int64_t right; int32_t a; int32_t b;
    bool operator>(const Entry& o) const { return rank != o.rank ? rank > o.rank : left > o.left; }
  };
  std::vector<int32_t> tok = t.initial(s, n);
  std::vector<int64_t> prev((size_t)n), next((size_t)n);
  std::vector<uint8_t> alive((size_t)n, 1);
  for (int64_t i = 0; i < n; ++i) { prev[(size_t)i] = i - 1; next[(size_t)i] = i + 1 < n ? i + 1 : -1; }
  std::priority_queue<Entry, std::vector<Entry>, std::greater<Entry>> heap;
  auto push = [&](int64_t l) {
    if (l < 0) return;
    int64_t r = next[(size_t)l];
    if (r < 0) return;
    int32_t rk = t.lookup(tok[(size_t)l], tok[(size_t)r]);
    if (rk != kNoRank) heap.push({rk, l, r, tok[(size_t)l], tok[(size_t)r]});
  };
  for (int64_t i = 0; i + 1 < n; ++i) push(i);
  while (!heap.empty()) {
    Entry e = heap.top();
    heap.pop();
    // stale if either token died, changed, or they are no longer neighbours
    if (!alive[(size_t)e.left] || !alive[(size_t)e.right]) continue;
    if (next[(size_t)e.left] != e.right) continue;
    if (tok[(size_t)e.left] != e.a || tok[(size_t)e.right] != e.b) continue;
    tok[(size_t)e.left] = t.merged_id[(size_t)e.rank];
    alive[(size_t)e.right] = 0;
    int64_t rr = next[(size_t)e.right];
    next[(size_t)e.left] = rr;
    if (rr >= 0) prev[(size_t)rr] = e.left;
    push(prev[(size_t)e.left]);
    push(e.left);
  }
  std::vector<int32_t> out;
  for (int64_t i = 0; i < n; ++i) if (alive[(size_t)i]) out.push_back(tok[(size_t)i]);
  return out;
}

void decode_id(const Table& t, int32_t id, std::string& out) {
  for (size_t i = 0; i < t.special_id.size(); ++i)
    if (t.special_id[i] == id) { out += t.special_text[i]; return; }
  auto b = t.byte_of_id.find(id);
  if (b != t.byte_of_id.end()) { out.push_back((char)b->second); return; }
  const auto& row = t.rows[(size_t)t.row_of_id.at(id)];
  decode_id(t, row.first, out);
  decode_id(t, row.second, out);
}

std::vector<int32_t> encode_plain(const Table& t, int tier, const uint8_t* s, int64_t n, PassStats* st);

// With special tokens: read the string left to right; where one or more specials match, the longest one
// becomes a single token with its id and reading goes on after it; the stretches in between are encoded by
// Algorithm 1 on their own (no merge involves a special token or crosses one).
std::vector<int32_t> encode_tier(const Table& t, int tier, const uint8_t* s, int64_t n, PassStats* st) {
  if (t.special_text.empty()) return encode_plain(t, tier, s, n, st);
  std::vector<int32_t> out;
  int64_t stretch = 0, p = 0;
  auto flush = [&](int64_t end) {
    if (end > stretch) {
      std::vector<int32_t> ids = encode_plain(t, tier, s + stretch, end - stretch, st);
      out.insert(out.end(), ids.begin(), ids.end());
    }
  };
  while (p < n) {
    int best = -1;
    for (size_t i = 0; i < t.special_text.size(); ++i) {
      const std::string& w = t.special_text[i];
      if ((int64_t)w.size() <= n - p && std::memcmp(w.data(), s + p, w.size()) == 0 &&
          (best < 0 || w.size() > t.special_text[(size_t)best].size()))
        best = (int)i;
    }
    if (best < 0) { ++p; continue; }
    flush(p);
    out.push_back(t.special_id[(size_t)best]);
    p += (int64_t)t.special_text[(size_t)best].size();
    stretch = p;
  }
  flush(n);
  return out;
}

std::vector<int32_t> encode_plain(const Table& t, int tier, const uint8_t* s, int64_t n, PassStats* st) {
  switch (tier) {
    case 0: return encode_bruteforce(t, s, n);
    case 1: return encode_textbook(t, s, n);
    case 2: return encode_passes(t, s, n, st);
    default: return encode_heap(t, s, n);
  }
}

// ---------------------------------------------------------------------------------------------------
// Trainer.

inline bool is_space(uint8_t c) { return c == 0x20 || c == 0x09 || c == 0x0A || c == 0x0D; }

// Distinct chunks with their frequencies.  A chunk starts at every whitespace byte (and at byte 0), so a
// separator stays attached to the front of the word that follows it.
void chunk_corpus(const uint8_t* c, int64_t n, std::vector<std::vector<int32_t>>& chunks,
                  std::vector<int64_t>& freq) {
  std::unordered_map<std::string, int64_t> seen;
  int64_t start = 0;
  for (int64_t i = 1; i <= n; ++i) {
    if (i == n || is_space(c[i])) {
      if (i > start) seen[std::string((const char*)c + start, (size_t)(i - start))] += 1;
      start = i;
    }
  }
  std::vector<std::pair<std::string, int64_t>> ordered(seen.begin(), seen.end());
  std::sort(ordered.begin(), ordered.end());               // order must not depend on the hash function
  for (auto& kv : ordered) {
    std::vector<int32_t> toks;
    for (unsigned char ch : kv.first) toks.push_back((int32_t)ch);
    chunks.push_back(std::move(toks));
    freq.push_back(kv.second);
  }
}

void apply_merge(std::vector<int32_t>& w, int32_t a, int32_t b, int32_t merged) {
  size_t o = 0;
  for (size_t i = 0; i < w.size();) {
    if (i + 1 < w.size() && w[i] == a && w[i + 1] == b) { w[o++] = merged; i += 2; }
    else { w[o++] = w[i]; i += 1; }
  }
  w.resize(o);
}

// Recount everything at every step: the definition of the trainer, for tiny corpora.
int64_t train_naive(const uint8_t* c, int64_t n, int32_t n_merges, int32_t* out) {
  std::vector<std::vector<int32_t>> chunks;
  std::vector<int64_t> freq;
  chunk_corpus(c, n, chunks, freq);
  int32_t done = 0;
  for (; done < n_merges; ++done) {
    std::map<std::pair<int32_t, int32_t>, int64_t> counts;
    for (size_t k = 0; k < chunks.size(); ++k)
      for (size_t i = 0; i + 1 < chunks[k].size(); ++i) counts[{chunks[k][i], chunks[k][i + 1]}] += freq[k];
    if (counts.empty()) break;
    std::pair<int32_t, int32_t> best{0, 0};
    int64_t best_count = 0;
    for (auto& kv : counts)                                // ascending (left,right): first maximum wins ties
      if (kv.second > best_count) { best_count = kv.second; best = kv.first; }
    out[2 * done] = best.first;
    out[2 * done + 1] = best.second;
    for (auto& w : chunks) apply_merge(w, best.first, best.second, 256 + done);
  }
  return done;
}

// Same result with incremental pair counts, a pair -> chunks index and a lazily cleaned max-heap.
int64_t train(const uint8_t* c, int64_t n, int32_t n_merges, int32_t* out) {
  std::vector<std::vector<int32_t>> chunks;
  std::vector<int64_t> freq;
  chunk_corpus(c, n, chunks, freq);

  std::unordered_map<uint64_t, int64_t> counts;
  std::unordered_map<uint64_t, std::vector<int32_t>> where;  // chunks that (may) contain the pair
  struct HeapEntry {
    int64_t count; uint64_t key;
    bool operator<(const HeapEntry& o) const {             // max-heap: high count first, then small key
      return count != o.count ? count < o.count : key > o.key;
    }
  };
  std::priority_queue<HeapEntry> heap;

  for (size_t k = 0; k < chunks.size(); ++k) {
    for (size_t i = 0; i + 1 < chunks[k].size(); ++i) {
      uint64_t key = pair_key(chunks[k][i], chunks[k][i + 1]);
      counts[key] += freq[k];
      auto& lst = where[key];
      if (lst.empty() || lst.back() != (int32_t)k) lst.push_back((int32_t)k);
    }
  }
  for (auto& kv : counts) heap.push({kv.second, kv.first});

  std::vector<uint64_t> touched;
  int32_t done = 0;
  while (done < n_merges) {
    // highest current count; entries whose count is out of date are refreshed and retried
    bool found = false;
    HeapEntry top{0, 0};
    while (!heap.empty()) {
      top = heap.top();
      heap.pop();
      auto it = counts.find(top.key);
      int64_t cur = it == counts.end() ? 0 : it->second;
      if (cur == top.count && cur > 0) { found = true; break; }
      if (cur > 0) heap.push({cur, top.key});
    }
    if (!found) break;
    const int32_t a = (int32_t)(top.key >> 32), b = (int32_t)(top.key & 0xFFFFFFFFu);
    const int32_t merged = 256 + done;
    out[2 * done] = a;
    out[2 * done + 1] = b;
    ++done;

    std::vector<int32_t> lst;
    lst.swap(where[top.key]);
    where.erase(top.key);
    std::sort(lst.begin(), lst.end());
    lst.erase(std::unique(lst.begin(), lst.end()), lst.end());
    touched.clear();
    for (int32_t k : lst) {
      auto& w = chunks[(size_t)k];
      bool has = false;
      for (size_t i = 0; i + 1 < w.size(); ++i) if (w[i] == a && w[i + 1] == b) { has = true; break; }
      if (!has) continue;
      for (size_t i = 0; i + 1 < w.size(); ++i) {          // retire the chunk's old pair counts
        uint64_t key = pair_key(w[i], w[i + 1]);
        counts[key] -= freq[(size_t)k];
        touched.push_back(key);
      }
      apply_merge(w, a, b, merged);
      for (size_t i = 0; i + 1 < w.size(); ++i) {          // and enter its new ones
        uint64_t key = pair_key(w[i], w[i + 1]);
        counts[key] += freq[(size_t)k];
        touched.push_back(key);
        if (w[i] == merged || w[i + 1] == merged) where[key].push_back(k);
      }
    }
    std::sort(touched.begin(), touched.end());
    touched.erase(std::unique(touched.begin(), touched.end()), touched.end());
    for (uint64_t key : touched) {
      auto it = counts.find(key);
      if (it->second > 0) heap.push({it->second, key});
      else counts.erase(it);
    }
  }
  return done;
}

}  // namespace

// ---------------------------------------------------------------------------------------------------
// C entry points (host pointers only).

extern "C" {

// Table over a vocabulary: byte_ids[256] are the ids of the single bytes, row r = (left id, right id) in
// vocabulary ids, merged_ids[r] the id of the token it creates.  Null byte_ids / merged_ids mean the default
// numbering (byte b -> b, row r -> 256 + r).
void* orc_table_new_vocab(const int32_t* byte_ids, const int32_t* merges, const int32_t* merged_ids,
                          int32_t n_merges) {
  Table* t = new Table();
  for (int b = 0; b < 256; ++b) {
    t->byte_id[b] = byte_ids ? byte_ids[b] : b;
    t->byte_of_id.emplace(t->byte_id[b], b);
  }
  for (int32_t r = 0; r < n_merges; ++r) {
    int32_t a = merges[2 * r], b = merges[2 * r + 1];
    t->rows.push_back({a, b});
    t->rank.emplace(pair_key(a, b), r);                    // first row wins if a pair repeats
    t->rank_ordered.emplace(std::make_pair(a, b), r);
    t->merged_id.push_back(merged_ids ? merged_ids[r] : 256 + r);
    t->row_of_id.emplace(t->merged_id.back(), r);
  }
  return t;
}

void* orc_table_new(const int32_t* merges, int32_t n_merges) {
  return orc_table_new_vocab(nullptr, merges, nullptr, n_merges);
}

void orc_table_free(void* h) { delete (Table*)h; }

// Special tokens: n byte strings (text[offsets[i] .. offsets[i+1])) with their ids; n = 0 removes them.
void orc_table_set_specials(void* h, const uint8_t* text, const int32_t* offsets, const int32_t* ids, int32_t n) {
  Table* t = (Table*)h;
  t->special_text.clear();
  t->special_id.clear();
  for (int32_t i = 0; i < n; ++i) {
    t->special_text.emplace_back((const char*)text + offsets[i], (size_t)(offsets[i + 1] - offsets[i]));
    t->special_id.push_back(ids[i]);
  }
}

// Encode one string with encoder `tier` (0 brute force, 1 textbook, 2 passes, 3 heap).
// out must hold n ids.  stats (may be null) = {passes, visits, merges}, filled by tier 2 only.
int64_t orc_encode(const void* h, int tier, const uint8_t* s, int64_t n, int32_t* out, int64_t* stats) {
  PassStats st;
  std::vector<int32_t> ids = encode_tier(*(const Table*)h, tier, s, n, &st);
  if (!ids.empty()) std::memcpy(out, ids.data(), ids.size() * sizeof(int32_t));
  if (stats) { stats[0] = st.passes; stats[1] = st.visits; stats[2] = st.merges; }
  return (int64_t)ids.size();
}

// What each pass of the pass view (tier 2) did on one string: trace receives, per pass, the rank applied, the
// number of live tokens at the start of the pass and the number of merges the pass applied (3 values per pass, at
// most `capacity` passes are written).  Returns the number of passes.
int64_t orc_pass_trace(const void* h, const uint8_t* s, int64_t n, int64_t* trace, int64_t capacity) {
  PassStats st;
  st.keep_trace = true;
  encode_passes(*(const Table*)h, s, n, &st);
  const int64_t passes = (int64_t)st.trace.size() / 3;
  for (int64_t i = 0; i < passes && i < capacity; ++i)
    for (int k = 0; k < 3; ++k) trace[3 * i + k] = st.trace[(size_t)(3 * i + k)];
  return passes;
}

// Encode a batch on `nthreads` host threads.  out_ids (capacity offsets[batch]) receives the dense
// concatenation, out_offsets[batch+1] the token offsets.  stats as above, summed over the batch.
int64_t orc_encode_batch(const void* h, int tier, const uint8_t* bytes, const int64_t* offsets, int64_t batch,
                         int nthreads, int32_t* out_ids, int64_t* out_offsets, int64_t* stats) {
  const Table& t = *(const Table*)h;
  std::vector<std::vector<int32_t>> results((size_t)batch);
  std::vector<PassStats> per((size_t)batch);
  std::atomic<int64_t> cursor{0};
  auto worker = [&]() {
    for (;;) {
      int64_t i = cursor.fetch_add(1);
      if (i >= batch) return;
      results[(size_t)i] = encode_tier(t, tier, bytes + offsets[i], offsets[i + 1] - offsets[i], &per[(size_t)i]);
    }
  };
  if (nthreads < 1) nthreads = 1;
  std::vector<std::thread> pool;
  for (int k = 1; k < nthreads; ++k) pool.emplace_back(worker);
  worker();
  for (auto& th : pool) th.join();
  int64_t pos = 0;
  PassStats sum;
  out_offsets[0] = 0;
  for (int64_t i = 0; i < batch; ++i) {
    auto& r = results[(size_t)i];
    if (!r.empty()) std::memcpy(out_ids + pos, r.data(), r.size() * sizeof(int32_t));
    pos += (int64_t)r.size();
    out_offsets[i + 1] = pos;
    sum.passes += per[(size_t)i].passes;
    sum.visits += per[(size_t)i].visits;
    sum.merges += per[(size_t)i].merges;
  }
  if (stats) { stats[0] = sum.passes; stats[1] = sum.visits; stats[2] = sum.merges; }
  return pos;
}

// ids -> bytes.  Returns the byte count; writes at most cap bytes.
int64_t orc_decode(const void* h, const int32_t* ids, int64_t k, uint8_t* out, int64_t cap) {
  std::string s;
  for (int64_t i = 0; i < k; ++i) decode_id(*(const Table*)h, ids[i], s);
  int64_t n = (int64_t)s.size();
  std::memcpy(out, s.data(), (size_t)std::min(n, cap));
  return n;
}

// Train up to n_merges rows on the corpus; returns the number of rows written to out (2 ints per row).
int64_t orc_train(const uint8_t* corpus, int64_t n, int32_t n_merges, int32_t* out, int naive) {
  return naive ? train_naive(corpus, n, n_merges, out) : train(corpus, n, n_merges, out);
}

}  // extern "C"
