// Seeded synthetic text generators for the byte-level BPE workloads.
//
// This file only produces INPUT bytes (corpora to train a merge table on, and batches of strings to
// encode).  It contains none of the method's arithmetic: no pair ranking, no merging, no table.  Both the
// CPU oracle's callers and the GPU path's callers draw their inputs from here so that they see the same
// bytes; neither of them is imported by, or imports, this module.
//
// Everything is derived from one counter-free PRNG implemented below (splitmix64 seeding a xoshiro256**
// state), never from rand() or <random> distributions, so a (style, seed, size) triple names the same
// bytes on every machine.
//
// Text styles (the paper tokenises excerpts of a novel with a pretrained vocabulary, section 5.1; neither
// is available offline, so Zipf-distributed word streams stand in for natural text's skewed pair
// statistics):
//   style 1: words over 'a'-'z', length uniform 1..12, word vocabulary 2^15, Zipf(s=1.1) over vocabulary
//            rank, single spaces between words.
//   style 2: word vocabulary 2^18 of three kinds (80 % lower-case alphabetic 1..12, 10 % digit strings
//            1..6, 10 % words with punctuation); ~15 % of emitted alphabetic words get a capital first
//            letter; the separator is '\n' instead of ' ' once the current line has reached 80 bytes.
//   style 3: as style 2 with a 2^20 vocabulary, but 15 % of emitted words are fresh random multibyte
//            UTF-8 words: 1..6 code points, all of one byte-length class drawn uniformly from {2,3,4},
//            code points uniform in that class's valid range (surrogates excluded).
//
// C ABI (all pointers are host memory owned by the caller):
//   wl_text(style, seed, out, nbytes)            fill out[0..nbytes) with the text stream
//   wl_adversarial(seed, out, nstrings, len)     nstrings strings of len bytes, repeated-byte runs
//                                                interleaved with repeated 2..8 byte motifs
//   wl_lognormal_lengths(seed, out, count, median, sigma, lo, hi)

#include <cmath>
#include <cstdint>
#include <cstring>
#include <string>
#include <vector>

namespace {

struct Rng {
  uint64_t s[4];
  explicit Rng(uint64_t seed) {
    uint64_t x = seed;
    for (int i = 0; i < 4; ++i) {  // splitmix64
      x += 0x9E3779B97F4A7C15ull;
      uint64_t z = x;
      z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
      z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
      s[i] = z ^ (z >> 31);
    }
  }
  static uint64_t rotl(uint64_t v, int k) { return (v << k) | (v >> (64 - k)); }
  uint64_t next() {  // xoshiro256**
    uint64_t r = rotl(s[1] * 5, 7) * 9;
    uint64_t t = s[1] << 17;
    s[2] ^= s[0];
    s[3] ^= s[1];
    s[1] ^= s[2];
    s[0] ^= s[3];
    s[2] ^= t;
    s[3] = rotl(s[3], 45);
    return r;
  }
  double uniform() { return (double)(next() >> 11) * (1.0 / 9007199254740992.0); }  // [0,1)
  // integer in [lo, hi], both inclusive
  int64_t range(int64_t lo, int64_t hi) {
    uint64_t span = (uint64_t)(hi - lo) + 1;
    return lo + (int64_t)(next() % span);
  }
};

const char kLower[] = "abcdefghijklmnopqrstuvwxyz";
const char kDigits[] = "0123456789";
const char kPunct[] = ".,;:!?'\"()-_/&%$#@*+=<>[]{}";

struct Vocab {
  std::vector<std::string> words;
  std::vector<uint8_t> alphabetic;  // 1 if the word may be capitalised
  std::vector<double> cdf;          // cumulative Zipf mass over vocabulary rank

  Vocab(int style) {
    size_t n = style == 1 ? (1u << 15) : style == 2 ? (1u << 18) : (1u << 20);
    Rng rng(0xB10CB9E0ull + (uint64_t)style);  // vocabulary depends on the style only
    words.reserve(n);
    alphabetic.reserve(n);
    for (size_t i = 0; i < n; ++i) {
      std::string w;
      bool alpha = true;
      double kind = style == 1 ? 0.0 : rng.uniform();
      if (kind < 0.80) {
        int len = (int)rng.range(1, 12);
        for (int k = 0; k < len; ++k) w.push_back(kLower[rng.range(0, 25)]);
      } else if (kind < 0.90) {
        alpha = false;
        int len = (int)rng.range(1, 6);
        for (int k = 0; k < len; ++k) w.push_back(kDigits[rng.range(0, 9)]);
      } else {
        alpha = false;
        int np = (int)sizeof(kPunct) - 2;
        int form = (int)rng.range(0, 2);
        if (form == 0) {  // pure punctuation, 1..3 characters
          int len = (int)rng.range(1, 3);
          for (int k = 0; k < len; ++k) w.push_back(kPunct[rng.range(0, np)]);
        } else {  // alphabetic word with one punctuation mark after it (form 1) or before it (form 2)
          int len = (int)rng.range(1, 10);
          std::string core;
          for (int k = 0; k < len; ++k) core.push_back(kLower[rng.range(0, 25)]);
          char p = kPunct[rng.range(0, np)];
          w = form == 1 ? core + p : p + core;
        }
      }
      words.push_back(w);
      alphabetic.push_back(alpha ? 1 : 0);
    }
    cdf.resize(n);
    double acc = 0.0;
    for (size_t i = 0; i < n; ++i) {
      acc += std::pow((double)(i + 1), -1.1);
      cdf[i] = acc;
    }
    for (size_t i = 0; i < n; ++i) cdf[i] /= acc;
    cdf[n - 1] = 1.0;
  }

  size_t draw(Rng& rng) const {
    double u = rng.uniform();
    size_t lo = 0, hi = cdf.size() - 1;
    while (lo < hi) {  // first index with cdf >= u
      size_t mid = (lo + hi) / 2;
      if (cdf[mid] >= u) hi = mid; else lo = mid + 1;
    }
    return lo;
  }
};

const Vocab& vocab_for(int style) {
  static Vocab* cache[4] = {nullptr, nullptr, nullptr, nullptr};
  if (!cache[style]) cache[style] = new Vocab(style);
  return *cache[style];
}

void append_utf8(std::string& w, uint32_t cp) {
  if (cp < 0x800) {
    w.push_back((char)(0xC0 | (cp >> 6)));
    w.push_back((char)(0x80 | (cp & 0x3F)));
  } else if (cp < 0x10000) {
    w.push_back((char)(0xE0 | (cp >> 12)));
    w.push_back((char)(0x80 | ((cp >> 6) & 0x3F)));
    w.push_back((char)(0x80 | (cp & 0x3F)));
  } else {
    w.push_back((char)(0xF0 | (cp >> 18)));
    w.push_back((char)(0x80 | ((cp >> 12) & 0x3F)));
    w.push_back((char)(0x80 | ((cp >> 6) & 0x3F)));
    w.push_back((char)(0x80 | (cp & 0x3F)));
  }
}

std::string multibyte_word(Rng& rng) {
  std::string w;
  int ncp = (int)rng.range(1, 6);
  int cls = (int)rng.range(2, 4);
  for (int k = 0; k < ncp; ++k) {
    uint32_t cp;
    if (cls == 2) {
      cp = (uint32_t)rng.range(0x80, 0x7FF);
    } else if (cls == 3) {
      // 0x800..0xFFFF without the surrogate block 0xD800..0xDFFF
      cp = (uint32_t)rng.range(0x800, 0xFFFF - 0x800);
      if (cp >= 0xD800) cp += 0x800;
    } else {
      cp = (uint32_t)rng.range(0x10000, 0x10FFFF);
    }
    append_utf8(w, cp);
  }
  return w;
}

}  // namespace

extern "C" {

// Fill out[0..nbytes) with the style's text stream for this seed (the last word may be cut short).
int wl_text(int style, uint64_t seed, uint8_t* out, int64_t nbytes) {
  if (style < 1 || style > 3 || nbytes < 0 || (nbytes > 0 && !out)) return -1;
  const Vocab& v = vocab_for(style);
  Rng rng(seed * 0x2545F4914F6CDD1Dull + (uint64_t)style);
  int64_t pos = 0;
  int64_t line = 0;
  bool first = true;
  std::string w;
  while (pos < nbytes) {
    if (!first) {
      char sep = ' ';
      if (style != 1 && line >= 80) { sep = '\n'; line = 0; }
      out[pos++] = (uint8_t)sep;
      ++line;
      if (pos >= nbytes) break;
    }
    first = false;
    if (style == 3 && rng.uniform() < 0.15) {
      w = multibyte_word(rng);
    } else {
      size_t idx = v.draw(rng);
      w = v.words[idx];
      if (style != 1 && v.alphabetic[idx] && rng.uniform() < 0.15) w[0] = (char)(w[0] - 'a' + 'A');
    }
    int64_t take = (int64_t)w.size();
    if (take > nbytes - pos) take = nbytes - pos;
    std::memcpy(out + pos, w.data(), (size_t)take);
    pos += take;
    line += take;
  }
  return 0;
}

// nstrings strings of exactly len bytes each, written back to back.  Each string alternates
//   (i)  a run of one byte, the byte from {'a','0',' ', a random letter or digit}, length uniform 16..1024
//   (ii) a 2..8 byte motif repeated until 16..512 bytes are filled; half of the motifs are random
//        letters/digits/punctuation, half are prefixes of one of the 1000 most frequent style-3 words
//        (padded with random lower-case letters when the word is shorter than the motif).
int wl_adversarial(uint64_t seed, uint8_t* out, int64_t nstrings, int64_t len) {
  if (nstrings < 0 || len < 0 || (nstrings * len > 0 && !out)) return -1;
  const Vocab& v = vocab_for(3);
  Rng rng(seed ^ 0xAD7E25A21A1ull);
  const std::string alnum = std::string(kLower) + kDigits;
  const std::string all = std::string(kLower) + kDigits + kPunct;
  for (int64_t s = 0; s < nstrings; ++s) {
    uint8_t* dst = out + s * len;
    int64_t pos = 0;
    bool run = rng.uniform() < 0.5;
    while (pos < len) {
      if (run) {
        int64_t n = rng.range(16, 1024);
        int pick = (int)rng.range(0, 3);
        uint8_t b = pick == 0 ? 'a' : pick == 1 ? '0' : pick == 2 ? ' '
                                                  : (uint8_t)alnum[rng.range(0, (int64_t)alnum.size() - 1)];
        for (int64_t k = 0; k < n && pos < len; ++k) dst[pos++] = b;
      } else {
        int m = (int)rng.range(2, 8);
        std::string motif;
        if (rng.uniform() < 0.5) {
          for (int k = 0; k < m; ++k) motif.push_back(all[rng.range(0, (int64_t)all.size() - 1)]);
        } else {
          motif = v.words[rng.range(0, 999)].substr(0, (size_t)m);
          while ((int)motif.size() < m) motif.push_back(kLower[rng.range(0, 25)]);
        }
        int64_t n = rng.range(16, 512);
        for (int64_t k = 0; k < n && pos < len; ++k) dst[pos++] = (uint8_t)motif[(size_t)(k % m)];
      }
      run = !run;
    }
  }
  return 0;
}

// out[i] = clip(round(median * exp(sigma * z_i)), lo, hi), z_i standard normal (Box-Muller on the PRNG).
int wl_lognormal_lengths(uint64_t seed, int64_t* out, int64_t count, double median, double sigma,
                         int64_t lo, int64_t hi) {
  if (count < 0 || (count > 0 && !out) || lo > hi) return -1;
  Rng rng(seed ^ 0x106A0A11ull);
  const double two_pi = 6.283185307179586476925286766559;
  for (int64_t i = 0; i < count; ++i) {
    double u1 = 1.0 - rng.uniform();  // (0,1]
    double u2 = rng.uniform();
    double z = std::sqrt(-2.0 * std::log(u1)) * std::cos(two_pi * u2);
    double x = std::floor(median * std::exp(sigma * z) + 0.5);
    int64_t n = x < (double)lo ? lo : x > (double)hi ? hi : (int64_t)x;
    out[i] = n;
  }
  return 0;
}

}  // extern "C"
