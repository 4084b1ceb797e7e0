// Host side of the C ABI declared in include/bpe.h: merge-table construction and the enqueue of one
// batch encode.  Everything numeric happens in the kernels of encode_kernel.h / batch_kernels.h.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <unordered_map>
#include <vector>

#include "../../include/bpe.h"
#include "batch_kernels.h"
#include "encode_kernel.h"
#include "encode_lanes.h"
#include "encode_segmented.h"
#include "table_format.h"

using namespace bpe;

struct bpe_table {
  int device = 0;
  int32_t n_merges = 0;
  int log2_buckets = 0;
  void* d_mem = nullptr;          // buckets, then the 256 byte token words, then the 256 x 256 byte-pair values,
                                  // then (tables over a vocabulary only) the id of every token, int32[256 + rows]
  size_t bucket_bytes = 0;
  const int32_t* d_id_map = nullptr;   // null: byte b is id b, row r creates id 256 + r.  Inside d_mem, or
                                       // d_special_mem once special tokens are set
  std::vector<int32_t> id_map_host;    // the vocabulary ids of the 256 + rows tokens (empty: the default)
  void* d_special_mem = nullptr;       // SpecialSet, then the id map extended by the specials' ids
  const SpecialSet* d_specials = nullptr;
};

// Scratch of bpe_encode_batch_static: what the caller's workspace is to bpe_encode_batch, for callers that
// cannot allocate.  One copy per GPU the library runs on, held until the process ends; every call on a GPU
// shares that GPU's copy.
constexpr size_t kStaticScratchBytes = (size_t)24 << 20;
static __device__ __align__(256) unsigned char g_static_scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
static void* g_scratch_ptr[kMaxDevices];       // device address of the array on each GPU, filled on first use
static std::mutex g_scratch_mutex;

namespace {

// ---- kernel variants ------------------------------------------------------------------------------
// A variant is (waves per workgroup, positions per lane, tokens staged in HBM or LDS); it encodes
// strings of up to 64 * waves * positions bytes.

struct Variant {
  int waves, depth;
  bool staged, limits;            // per-position arrays in HBM instead of LDS; a third array holds the pair limits
  int capacity;                   // bytes
  size_t lds;
  const void* fn;
  void (*launch)(const EncodeParams&, int grid, hipStream_t);
  int max_grid = 0;               // resident workgroups on the whole device (filled on first use)
};

template <int NW, int D, bool ST, bool LIM, bool SEG, bool SPC>
void launch_variant(const EncodeParams& p, int grid, hipStream_t stream) {
  constexpr size_t lds = encode_lds_bytes<NW, D, ST, LIM>();
  encode_kernel<NW, D, ST, LIM, SEG, SPC><<<dim3(grid), dim3(NW * 64), lds, stream>>>(p);
}

template <int NW, int D, bool ST, bool LIM, bool SEG, bool SPC>
Variant make_variant() {
  Variant v;
  v.waves = NW;
  v.depth = D;
  v.staged = ST;
  v.limits = LIM;
  v.capacity = 64 * NW * D;
  v.lds = encode_lds_bytes<NW, D, ST, LIM>();
  v.fn = (const void*)&encode_kernel<NW, D, ST, LIM, SEG, SPC>;
  v.launch = &launch_variant<NW, D, ST, LIM, SEG, SPC>;
  return v;
}

// Default plan: <= 1 KiB one wave, <= 4 KiB four waves, <= 16 KiB sixteen waves (all LDS-resident),
// <= 64 KiB sixteen waves with the per-position arrays staged in HBM.  Second family: the same kernels with
// the reading of special-token marks compiled in (tables that have special tokens set).
Variant g_variant_families[2][kMaxTiers] = {
    {make_variant<1, 16, false, true, true, false>(), make_variant<4, 16, false, true, true, false>(),
     make_variant<16, 16, false, false, true, false>(),   // three arrays of 16 Ki words would not fit the 160 KB of LDS
     make_variant<16, 64, true, true, false, false>()},   // whole-string horizon; arrays in HBM
    {make_variant<1, 16, false, true, true, true>(), make_variant<4, 16, false, true, true, true>(),
     make_variant<16, 16, false, false, true, true>(), make_variant<16, 64, true, true, false, true>()},
};
Variant (&g_variants)[kMaxTiers] = g_variant_families[0];   // sizes and capacities are those of either family

// Items of up to 1 KiB go to the lane-per-segment kernel first; the one-wave variant above then takes those that
// kernel passes on (items with a segment of more than 32 bytes).  [family][0]: passes them on through the
// fallback list; [family][1]: encodes them itself (the launch without a work list).
template <bool SPC, bool INL>
void launch_lanes(const EncodeParams& p, int grid, hipStream_t stream) {
  encode_lanes_kernel<SPC, INL><<<dim3(grid), dim3(64), lanes_lds_bytes<INL>(), stream>>>(p);
}
template <bool SPC, bool INL>
Variant make_lanes_variant() {
  Variant v;
  v.waves = 1;
  v.depth = 16;
  v.staged = false;
  v.limits = false;
  v.capacity = kLaneItemBytes;
  v.lds = lanes_lds_bytes<INL>();
  v.fn = (const void*)&encode_lanes_kernel<SPC, INL>;
  v.launch = &launch_lanes<SPC, INL>;
  return v;
}
Variant g_lanes_variants[2][2] = {
    {make_lanes_variant<false, false>(), make_lanes_variant<false, true>()},
    {make_lanes_variant<true, false>(), make_lanes_variant<true, true>()},
};
std::once_flag g_variants_once;
int g_variants_status = BPE_OK;
int g_num_cus = 0;

void init_variants() {
  int dev = 0;
  hipDeviceProp_t prop;
  if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) {
    g_variants_status = BPE_EHIP;
    return;
  }
  g_num_cus = prop.multiProcessorCount;
  std::vector<Variant*> all;
  for (auto& family : g_variant_families) for (auto& v : family) all.push_back(&v);
  for (auto& family : g_lanes_variants) for (auto& v : family) all.push_back(&v);
  for (Variant* vp : all) {
    Variant& v = *vp;
    if (v.lds > 48 * 1024) {
      if (hipFuncSetAttribute(v.fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)v.lds) != hipSuccess) {
        g_variants_status = BPE_EHIP;
        return;
      }
    }
    int per_cu = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, v.fn, v.waves * 64, v.lds) != hipSuccess ||
        per_cu < 1) {
      g_variants_status = BPE_EHIP;
      return;
    }
    v.max_grid = per_cu * g_num_cus;
  }
}

// Variants that a batch with strings of up to max_len bytes can need.
int n_tiers_for(int32_t max_len) {
  int n = 1;
  while (n < kMaxTiers && g_variants[n - 1].capacity < max_len) ++n;
  return n;
}

// Staged variant: resident workgroups each own one staging slab; the grid is capped so that the slabs
// stay modest (each is 768 KiB for 64 KiB strings).
constexpr int kMaxStagedGrid = 256;
size_t staged_slab_bytes(const Variant& v) {
  return (size_t)(v.limits ? 3 : 2) * 64 * v.waves * v.depth * sizeof(uint32_t);
}

constexpr size_t align_up(size_t x) { return (x + 255) & ~(size_t)255; }

// Strings longer than this are cut into pieces at segment cuts (see batch_kernels.h).  A piece starts at most
// kCutWindow - 1 bytes before a multiple of the target, so pieces stay within the one-wave variant's 1 KiB.
constexpr int kPieceTarget = 1024 - kCutWindow;

struct WorkspaceLayout {
  bool split;                        // strings are cut into pieces
  int64_t max_slots;                 // upper bound on the number of work items (strings or piece slots)
  int n_tiles;                       // scan tiles over the slots
  size_t control, list, list_desc, fallback, counts, tmp_ids, cover, staged;
  size_t slot_base, slot_string, piece_begin, piece_len, slot_out, tile_sum;   // split only
  size_t total;
};

WorkspaceLayout layout_for(int32_t batch, int64_t total_bytes, int32_t max_len) {
  WorkspaceLayout w;
  w.split = max_len > g_variants[0].capacity;   // everything already fits the one-wave variant otherwise
  w.max_slots = w.split ? (int64_t)batch + total_bytes / kPieceTarget : (int64_t)batch;
  w.n_tiles = (int)((w.max_slots + kScanTile - 1) / kScanTile);
  size_t at = 0;
  w.control = at; at += align_up(sizeof(Control));
  w.list = at; at += align_up((size_t)w.max_slots * sizeof(int32_t));
  w.list_desc = at; at += align_up((size_t)w.max_slots * sizeof(ItemDesc));
  w.fallback = at; at += align_up((size_t)w.max_slots * sizeof(int32_t));
  w.counts = at; at += align_up((size_t)w.max_slots * sizeof(int32_t));
  w.tmp_ids = at; at += align_up((size_t)total_bytes * sizeof(int32_t));
  w.cover = at; at += align_up((size_t)total_bytes + 4);      // special-token marks, one per byte
  w.slot_base = w.slot_string = w.piece_begin = w.piece_len = w.slot_out = w.tile_sum = 0;
  if (w.split) {
    w.slot_base = at; at += align_up(((size_t)batch + 1) * sizeof(int32_t));
    w.slot_string = at; at += align_up((size_t)w.max_slots * sizeof(int32_t));
    w.piece_begin = at; at += align_up((size_t)w.max_slots * sizeof(int64_t));
    w.piece_len = at; at += align_up((size_t)w.max_slots * sizeof(int32_t));
    w.slot_out = at; at += align_up((size_t)w.max_slots * sizeof(int64_t));
    w.tile_sum = at; at += align_up((size_t)(w.n_tiles + 1) * sizeof(int64_t));
  }
  w.staged = at;
  const int nt = n_tiers_for(max_len);
  for (int t = 0; t < nt; ++t)
    if (g_variants[t].staged) at += align_up(staged_slab_bytes(g_variants[t]) * kMaxStagedGrid);
  w.total = at;
  return w;
}

// Optional timing of the encode kernels alone: a ring of event pairs recorded on the caller's stream.
constexpr int kProfileRing = 512;
struct ProfileRing {
  hipEvent_t begin[kProfileRing], end[kProfileRing];
  int created = 0;   // event pairs that exist (all of them once profiling has been switched on)
  int used = 0;      // pairs recorded since profiling was switched on
};
ProfileRing g_prof;
std::mutex g_prof_mutex;
bool g_profiling = false;

// The table as it lies in device memory, built in host memory: [buckets | byte_word[256] | byte_pair[65536]].
int build_image(const int32_t* merges, int32_t n_merges, std::vector<uint32_t>& host, int& log2_buckets_out,
                int32_t* bad_row) {
  // operands must exist before the row that uses them
  for (int32_t r = 0; r < n_merges; ++r) {
    const int32_t a = merges[2 * r], b = merges[2 * r + 1];
    if (a < 0 || b < 0 || a >= 256 + r || b >= 256 + r) {
      if (bad_row) *bad_row = r;
      return BPE_EBADMERGE;
    }
  }

  std::vector<int32_t> first_left, first_right;                // first row that uses a token as left / right
  try {
    first_left.assign((size_t)n_merges + 256, -1);
    first_right.assign((size_t)n_merges + 256, -1);
  } catch (const std::bad_alloc&) {
    return BPE_ENOMEM;
  }
  for (int32_t r = 0; r < n_merges; ++r) {
    int32_t& fl = first_left[(size_t)merges[2 * r]];
    int32_t& fr = first_right[(size_t)merges[2 * r + 1]];
    if (fl < 0) fl = r;
    if (fr < 0) fr = r;
  }

  // Byte bigrams that can lie at the junction of a merge: (last byte of the left operand, first byte of the
  // right operand) of some row.  Between two bytes whose bigram is not among them no merge can ever happen.
  std::vector<uint8_t> first_byte, last_byte, junction;
  try {
    first_byte.resize((size_t)n_merges + 256);
    last_byte.resize((size_t)n_merges + 256);
    junction.assign(65536, 0);
  } catch (const std::bad_alloc&) {
    return BPE_ENOMEM;
  }
  for (int b = 0; b < 256; ++b) first_byte[(size_t)b] = last_byte[(size_t)b] = (uint8_t)b;
  for (int32_t r = 0; r < n_merges; ++r) {
    const size_t a = (size_t)merges[2 * r], b = (size_t)merges[2 * r + 1];
    junction[(size_t)last_byte[a] << 8 | first_byte[b]] = 1;
    first_byte[256 + (size_t)r] = first_byte[a];
    last_byte[256 + (size_t)r] = last_byte[b];
  }

  int log2_buckets = kMinLog2Buckets;
  while ((int64_t)kSlotsPerBucket * ((int64_t)1 << log2_buckets) * 2 < (int64_t)n_merges * 5) ++log2_buckets;
  size_t n_words = 0;
  for (;; ++log2_buckets) {                                    // grow until every key sits close to home
    if (log2_buckets > kMaxLog2Buckets) return BPE_ETOOBIG;
    const size_t n_buckets = (size_t)1 << log2_buckets;
    n_words = n_buckets * kSlotsPerBucket * 2;                 // uint32 words
    try {
      host.assign(n_words + 256 + 65536, 0xFFFFFFFFu);
    } catch (const std::bad_alloc&) {
      return BPE_ENOMEM;
    }
    bool fits = true;
    for (int32_t r = 0; r < n_merges && fits; ++r) {
      const uint32_t a = (uint32_t)merges[2 * r], b = (uint32_t)merges[2 * r + 1];
      const int32_t fl = first_left[256 + (size_t)r], fr = first_right[256 + (size_t)r];
      // horizon: ranks between this row and the first later row that uses its token (rows only use
      // older tokens, so that row comes after this one)
      uint32_t code = 255;
      if (fl >= 0 || fr >= 0) {
        const int32_t first_use = fl < 0 ? fr : (fr < 0 ? fl : (fl < fr ? fl : fr));
        code = horizon_encode((uint32_t)(first_use - r - 1));
      }
      const uint32_t value = make_value((uint32_t)r, code, fl >= 0, fr >= 0);
      if (a < 256 && b < 256) host[n_words + 256 + (a << 8 | b)] = value;   // direct table for byte pairs
      const Placement pl = place_pair(a, b, log2_buckets);
      bool placed = false;
      uint32_t* const home = host.data() + (size_t)pl.bucket * kSlotsPerBucket * 2;
      for (uint32_t d = 0; d <= kMaxDisplacement && !placed; ++d) {       // home bucket, then the rest of its line
        uint32_t* bucket = host.data() + (size_t)(pl.bucket ^ d) * kSlotsPerBucket * 2;
        const uint32_t tag = slot_tag(pl.fingerprint, d);
        for (int k = 0; k < kSlotsPerBucket; ++k) {
          uint32_t& slo = bucket[2 * k];
          uint32_t& shi = bucket[2 * k + 1];
          if (shi == 0xFFFFFFFFu) {                            // first empty slot of the bucket
            slo = value;
            shi = tag;
            placed = true;
            break;
          }
          if (shi == tag) {                                    // same home bucket, same fingerprint: same pair
            if (bad_row) *bad_row = r;
            return BPE_EDUPPAIR;
          }
        }
        // the home bucket is full (else the key would be in it): its spare bits say how far its keys reach
        if (placed && d > bucket_reach(home[0], home[2])) {
          home[0] = (home[0] & ~3u) | (d & 3u);
          home[2] = (home[2] & ~3u) | (d >> 2);
        }
      }
      fits = placed;
    }
    if (fits) break;
  }
  for (size_t i = 0; i < 65536; ++i)                           // byte pairs that are no row: cut or plain miss
    if (host[n_words + 256 + i] == 0xFFFFFFFFu && !junction[i]) host[n_words + 256 + i] = kCut;
  uint32_t* byte_word = host.data() + n_words;
  for (uint32_t b = 0; b < 256; ++b)
    byte_word[b] = b | (first_left[b] >= 0 ? kTokCanLeft : 0u) | (first_right[b] >= 0 ? kTokCanRight : 0u);
  log2_buckets_out = log2_buckets;
  return BPE_OK;
}

// merges: rows in the library's own numbering (byte b = b, row r creates 256 + r); id_map: null, or the
// vocabulary id of each of the 256 + n_merges tokens, which the packing kernels then write instead.
int build_table(const int32_t* merges, int32_t n_merges, const int32_t* id_map, bpe_table** out,
                int32_t* bad_row) {
  std::vector<uint32_t> host;
  int log2_buckets = 0;
  const int status = build_image(merges, n_merges, host, log2_buckets, bad_row);
  if (status != BPE_OK) return status;
  bpe_table* t = new (std::nothrow) bpe_table();
  if (!t) return BPE_ENOMEM;
  t->n_merges = n_merges;
  t->log2_buckets = log2_buckets;
  t->bucket_bytes = (host.size() - 256 - 65536) * sizeof(uint32_t);
  if (hipGetDevice(&t->device) != hipSuccess) { delete t; return BPE_EHIP; }
  const size_t map_words = id_map ? (size_t)n_merges + 256 : 0;
  hipError_t e = hipMalloc(&t->d_mem, (host.size() + map_words) * sizeof(uint32_t));
  if (e != hipSuccess) { delete t; return e == hipErrorOutOfMemory ? BPE_ENOMEM : BPE_EHIP; }
  bool ok = hipMemcpy(t->d_mem, host.data(), host.size() * sizeof(uint32_t), hipMemcpyHostToDevice) == hipSuccess;
  if (ok && id_map) {
    int32_t* d_map = (int32_t*)((uint32_t*)t->d_mem + host.size());
    ok = hipMemcpy(d_map, id_map, map_words * sizeof(int32_t), hipMemcpyHostToDevice) == hipSuccess;
    t->d_id_map = d_map;
    try {
      t->id_map_host.assign(id_map, id_map + map_words);
    } catch (const std::bad_alloc&) {
      ok = false;
    }
  }
  if (!ok) {
    (void)hipFree(t->d_mem);
    delete t;
    return BPE_EHIP;
  }
  *out = t;
  return BPE_OK;
}

}  // namespace

extern "C" {

int bpe_build_table(const int32_t* merges, int32_t n_merges, bpe_table** out, int32_t* bad_row) {
  if (bad_row) *bad_row = -1;
  if (!out) return BPE_EINVAL;
  *out = nullptr;
  if (n_merges < 0 || (n_merges > 0 && !merges)) return BPE_EINVAL;
  if (n_merges > BPE_MAX_MERGES) return BPE_ETOOBIG;
  return build_table(merges, n_merges, nullptr, out, bad_row);
}

int64_t bpe_table_image(const int32_t* merges, int32_t n_merges, uint32_t* words, int64_t capacity,
                        int32_t* log2_buckets, int32_t* bad_row) {
  if (bad_row) *bad_row = -1;
  if (n_merges < 0 || (n_merges > 0 && !merges) || capacity < 0 || (capacity > 0 && !words)) return BPE_EINVAL;
  if (n_merges > BPE_MAX_MERGES) return BPE_ETOOBIG;
  std::vector<uint32_t> host;
  int log2 = 0;
  const int status = build_image(merges, n_merges, host, log2, bad_row);
  if (status != BPE_OK) return status;
  if (log2_buckets) *log2_buckets = log2;
  if ((int64_t)host.size() <= capacity) std::memcpy(words, host.data(), host.size() * sizeof(uint32_t));
  return (int64_t)host.size();
}

int bpe_build_table_vocab(const int32_t* byte_ids, const int32_t* merges, const int32_t* merged_ids,
                          int32_t n_merges, bpe_table** out, int32_t* bad_row) {
  if (bad_row) *bad_row = -1;
  if (!out) return BPE_EINVAL;
  *out = nullptr;
  if (!byte_ids || n_merges < 0 || (n_merges > 0 && (!merges || !merged_ids))) return BPE_EINVAL;
  if (n_merges > BPE_MAX_MERGES) return BPE_ETOOBIG;
  // vocabulary id -> the library's own number of the token (byte b = b, row r = 256 + r), filled row by row
  // so that a row can only name tokens that exist before it
  std::vector<int32_t> id_map, own;
  std::unordered_map<int32_t, int32_t> number_of;
  try {
    id_map.resize((size_t)n_merges + 256);
    own.resize((size_t)n_merges * 2);
    number_of.reserve((size_t)n_merges + 256);
    for (int b = 0; b < 256; ++b) {
      if (byte_ids[b] < 0) return BPE_EINVAL;
      if (!number_of.emplace(byte_ids[b], b).second) return BPE_EDUPID;     // two bytes share an id
      id_map[(size_t)b] = byte_ids[b];
    }
    for (int32_t r = 0; r < n_merges; ++r) {
      for (int side = 0; side < 2; ++side) {
        const auto it = number_of.find(merges[2 * r + side]);
        if (it == number_of.end()) {                           // not a byte, not created by an earlier row
          if (bad_row) *bad_row = r;
          return BPE_EBADMERGE;
        }
        own[(size_t)(2 * r + side)] = it->second;
      }
      if (merged_ids[r] < 0 || !number_of.emplace(merged_ids[r], 256 + r).second) {
        if (bad_row) *bad_row = r;
        return merged_ids[r] < 0 ? BPE_EINVAL : BPE_EDUPID;    // the id already names another token
      }
      id_map[(size_t)(256 + r)] = merged_ids[r];
    }
  } catch (const std::bad_alloc&) {
    return BPE_ENOMEM;
  }
  return build_table(own.data(), n_merges, id_map.data(), out, bad_row);
}

int bpe_table_set_specials(bpe_table* table, const uint8_t* text, const int32_t* text_offsets, const int32_t* ids,
                           int32_t n) {
  if (!table || n < 0 || n > BPE_MAX_SPECIALS || (n > 0 && (!text || !text_offsets || !ids))) return BPE_EINVAL;
  if (256 + (int64_t)table->n_merges + n > 0xFFFFE) return BPE_ETOOBIG;      // token numbers stay below 2^20 - 1
  int device = -1;
  if (hipGetDevice(&device) != hipSuccess) return BPE_EHIP;
  if (device != table->device) return BPE_EINVAL;
  void* fresh = nullptr;
  const SpecialSet* d_set = nullptr;
  const int32_t* d_map = nullptr;
  if (n > 0) {
    SpecialSet set;
    std::memset(&set, 0, sizeof(set));
    set.n = n;
    for (int32_t i = 0; i < n; ++i) {
      const int32_t len = text_offsets[i + 1] - text_offsets[i];
      if (len < 1 || len > BPE_MAX_SPECIAL_BYTES || ids[i] < 0) return BPE_EINVAL;
      set.len[i] = len;
      std::memcpy(set.text[i], text + text_offsets[i], (size_t)len);
      set.first_byte[set.text[i][0] >> 5] |= 1u << (set.text[i][0] & 31);
    }
    // Occurrences must not be able to overlap: no special may hold, from some offset > 0 on, the beginning
    // of a special (be it all of that special, or as much of it as fits before the first one ends).
    for (int32_t a = 0; a < n; ++a)
      for (int32_t b = 0; b < n; ++b)
        for (int32_t o = 1; o < set.len[a]; ++o) {
          const int32_t m = std::min(set.len[b], set.len[a] - o);
          if (std::memcmp(set.text[a] + o, set.text[b], (size_t)m) == 0) return BPE_ESPECIAL;
        }
    for (int32_t a = 0; a < n; ++a)                       // two specials with the same text
      for (int32_t b = a + 1; b < n; ++b)
        if (set.len[a] == set.len[b] && std::memcmp(set.text[a], set.text[b], (size_t)set.len[a]) == 0)
          return BPE_ESPECIAL;
    // ids of all tokens: the table's (default or vocabulary), then the specials'
    const size_t n_tokens = 256 + (size_t)table->n_merges;
    std::vector<int32_t> map;
    try {
      map.resize(n_tokens + (size_t)n);
    } catch (const std::bad_alloc&) {
      return BPE_ENOMEM;
    }
    for (size_t t = 0; t < n_tokens; ++t) map[t] = table->id_map_host.empty() ? (int32_t)t : table->id_map_host[t];
    for (int32_t i = 0; i < n; ++i) map[n_tokens + (size_t)i] = ids[i];
    const size_t set_bytes = (sizeof(SpecialSet) + 255) & ~(size_t)255;
    hipError_t e = hipMalloc(&fresh, set_bytes + map.size() * sizeof(int32_t));
    if (e != hipSuccess) return e == hipErrorOutOfMemory ? BPE_ENOMEM : BPE_EHIP;
    if (hipMemcpy(fresh, &set, sizeof(set), hipMemcpyHostToDevice) != hipSuccess ||
        hipMemcpy((char*)fresh + set_bytes, map.data(), map.size() * sizeof(int32_t), hipMemcpyHostToDevice) !=
            hipSuccess) {
      (void)hipFree(fresh);
      return BPE_EHIP;
    }
    d_set = (const SpecialSet*)fresh;
    d_map = (const int32_t*)((char*)fresh + set_bytes);
  } else if (!table->id_map_host.empty()) {
    d_map = (const int32_t*)((const uint32_t*)table->d_mem + table->bucket_bytes / sizeof(uint32_t) + 256 + 65536);
  }
  if (table->d_special_mem) (void)hipFree(table->d_special_mem);
  table->d_special_mem = fresh;
  table->d_specials = d_set;
  table->d_id_map = d_map;
  return BPE_OK;
}

void bpe_free_table(bpe_table* table) {
  if (!table) return;
  if (table->d_special_mem) (void)hipFree(table->d_special_mem);
  if (table->d_mem) (void)hipFree(table->d_mem);
  delete table;
}

int32_t bpe_table_n_merges(const bpe_table* table) { return table ? table->n_merges : 0; }

size_t bpe_workspace_bytes(int32_t batch, int64_t total_bytes, int32_t max_len) {
  if (batch < 0 || total_bytes < 0 || max_len < 0 || max_len > BPE_MAX_STRING_BYTES) return 0;
  return layout_for(batch, total_bytes, max_len).total;
}

// Argument checks shared by the encode entry points, then the enqueue.  `workspace` is device memory of at
// least layout_for(...).total bytes, 256-byte aligned: the caller's, or this device's static scratch array.
static int encode_enqueue(const bpe_table* table, const uint8_t* bytes, const int64_t* offsets, int32_t batch,
                          int64_t total_bytes, int32_t max_len, int32_t* out_ids, int64_t* out_offsets,
                          void* workspace, const WorkspaceLayout& w, void* stream_ptr) {

  std::call_once(g_variants_once, init_variants);
  if (g_variants_status != BPE_OK) return g_variants_status;

  hipStream_t stream = (hipStream_t)stream_ptr;
  char* ws = (char*)workspace;
  Control* ctrl = (Control*)(ws + w.control);
  int32_t* list = (int32_t*)(ws + w.list);
  int32_t* counts = (int32_t*)(ws + w.counts);
  int32_t* tmp_ids = (int32_t*)(ws + w.tmp_ids);

  TierPlan plan;
  plan.n_tiers = n_tiers_for(max_len);
  for (int t = 0; t < kMaxTiers; ++t) plan.cap[t] = g_variants[t].capacity;

  const uint8_t* cover = nullptr;                        // special tokens: mark their occurrences first
  if (table->d_specials && batch > 0 && total_bytes > 0) {
    uint8_t* marks = (uint8_t*)(ws + w.cover);
    const int grid = (int)std::min<int64_t>((total_bytes + 255) / 256, 16384);
    hipLaunchKernelGGL(cover_clear_kernel, dim3(grid), dim3(256), 0, stream, marks, total_bytes);
    hipLaunchKernelGGL(special_mark_kernel, dim3(grid), dim3(256), 0, stream, bytes, offsets, batch, total_bytes,
                       table->d_specials, marks);
    cover = marks;
  }
  const int64_t* piece_begin = nullptr;
  const int32_t* piece_len = nullptr;
  const int32_t* slot_base = nullptr;
  const int32_t* slot_string = nullptr;
  const int n_items_max = (int)w.max_slots;              // grid bound for the encode kernels
  // A batch that one variant's resident grid covers needs no work list: workgroup i encodes string i.
  const Variant* family = g_variant_families[cover ? 1 : 0];
  const Variant* lanes = g_lanes_variants[cover ? 1 : 0];
  const bool direct = !w.split && plan.n_tiers == 1 && batch <= lanes[1].max_grid;
  if (batch > 0) {
    if (direct) {
      list = nullptr;
    } else if (!w.split) {
      hipLaunchKernelGGL(bin_kernel, dim3(1), dim3(1024), 0, stream, offsets, batch, plan, ctrl, list,
                         (ItemDesc*)(ws + w.list_desc), counts);
    } else {
      int32_t* sb = (int32_t*)(ws + w.slot_base);
      int32_t* ss = (int32_t*)(ws + w.slot_string);
      int64_t* pb = (int64_t*)(ws + w.piece_begin);
      int32_t* pl = (int32_t*)(ws + w.piece_len);
      const uint32_t* byte_pair =
          (const uint32_t*)((const char*)table->d_mem + table->bucket_bytes) + 256;
      const int per_slot_grid = (int)std::min<int64_t>((w.max_slots + 255) / 256, 256);   // (each workgroup ends with a few global atomics)
      hipLaunchKernelGGL(slot_layout_kernel, dim3((unsigned)((batch + 1023) / 1024)), dim3(1024), 0, stream, offsets, batch, kPieceTarget,
                         BPE_MAX_STRING_BYTES, ctrl, sb, ss);
      hipLaunchKernelGGL(cut_search_kernel, dim3((unsigned)((w.max_slots + 4 * kCutSlotsPerWave - 1) / (4 * kCutSlotsPerWave))), dim3(256), 0, stream, bytes,
                         offsets, byte_pair, kPieceTarget, BPE_MAX_STRING_BYTES, ctrl, sb, ss, pb, cover);
      if (w.max_slots <= kSmallSlots) {
        hipLaunchKernelGGL(piece_list_small_kernel, dim3(1), dim3(1024), 0, stream, offsets, plan, ctrl, sb, ss, pb, pl,
                           counts, list, (ItemDesc*)(ws + w.list_desc));
      } else {
        hipLaunchKernelGGL(piece_hist_kernel, dim3(per_slot_grid), dim3(256), 0, stream, offsets, plan, ctrl, sb, ss,
                           pb, pl, counts);
        hipLaunchKernelGGL(piece_scan_kernel, dim3(1), dim3(256), 0, stream, ctrl, plan.n_tiers);
        hipLaunchKernelGGL(piece_scatter_kernel, dim3((unsigned)((w.max_slots + 256 * kScatterPer - 1) / (256 * kScatterPer))), dim3(256), 0, stream, plan,
                           ctrl, pb, pl, list, (ItemDesc*)(ws + w.list_desc));
      }
      piece_begin = pb;
      piece_len = pl;
      slot_base = sb;
      slot_string = ss;
    }

    EncodeParams p;
    p.table.buckets = (const uint4*)table->d_mem;
    p.table.byte_word = (const uint32_t*)((const char*)table->d_mem + table->bucket_bytes);
    p.table.byte_pair = p.table.byte_word + 256;
    p.table.log2_buckets = table->log2_buckets;
    p.bytes = bytes;
    p.offsets = offsets;
    p.piece_begin = piece_begin;
    p.piece_len = piece_len;
    p.list = list;
    p.list_desc = list ? (const void*)(ws + w.list_desc) : nullptr;
    p.tier_base = ctrl->tier_base;
    p.queue_head = ctrl->queue_head;
    p.tmp_ids = tmp_ids;
    p.counts = counts;
    p.direct_count = (uint32_t)batch;
    p.cover = cover;
    p.special_base = 256u + (uint32_t)table->n_merges;
    p.total_bytes = total_bytes;
    p.fallback_count = &ctrl->fallback_range[1];
    p.fallback_list = (int32_t*)(ws + w.fallback);
    // Warming L2 pays once the batch probes the table more often than it has lines: ~1 probe per input byte.
    const size_t table_bytes = table->bucket_bytes + (256 + 65536) * sizeof(uint32_t);
    p.prefetch_lines = (size_t)total_bytes >= table_bytes / 4 ? (uint32_t)(table_bytes / 128) : 0u;

    int prof_slot = -1;
    if (g_profiling) {                                   // the event pairs exist already: nothing is created here
      std::lock_guard<std::mutex> lock(g_prof_mutex);
      if (g_profiling && g_prof.used < g_prof.created) {
        prof_slot = g_prof.used++;
        if (hipEventRecord(g_prof.begin[prof_slot], stream) != hipSuccess) return BPE_EHIP;
      }
    }
    size_t staged_at = w.staged;
    for (int t = 0; t < plan.n_tiers; ++t) {
      const Variant& v = family[t];
      int grid = v.max_grid < n_items_max ? v.max_grid : n_items_max;
      p.tier = t;
      p.staged = nullptr;
      if (v.staged) {
        if (grid > kMaxStagedGrid) grid = kMaxStagedGrid;
        p.staged = (uint32_t*)(ws + staged_at);
        staged_at += align_up(staged_slab_bytes(v) * kMaxStagedGrid);
      }
      if (t == 0) {
        // one lane per segment; what it cannot take (a segment of more than 32 bytes) it encodes itself when
        // there is no work list, and else leaves on the fallback list for the wave-per-item variant
        const Variant& lv = lanes[direct ? 1 : 0];
        lv.launch(p, lv.max_grid < n_items_max ? lv.max_grid : n_items_max, stream);
        if (direct) continue;
        EncodeParams rest = p;
        rest.list = p.fallback_list;
        rest.tier_base = ctrl->fallback_range;
        rest.queue_head = &ctrl->fallback_queue;
        rest.prefetch_lines = 0;
        v.launch(rest, grid, stream);
        continue;
      }
      v.launch(p, grid, stream);
    }
    if (prof_slot >= 0 && hipEventRecord(g_prof.end[prof_slot], stream) != hipSuccess) return BPE_EHIP;
  }
  if (!w.split && batch > 0 && batch <= 4096) {
    hipLaunchKernelGGL(scan_pack_kernel, dim3(batch), dim3(256), 0, stream, tmp_ids, offsets, counts, batch,
                       out_offsets, out_ids, table->d_id_map);
  } else if (!w.split) {
    hipLaunchKernelGGL(offsets_scan_kernel, dim3(1), dim3(1024), 0, stream, counts, batch, out_offsets);
    if (batch > 0) {
      const int grid = batch < 65536 ? batch : 65536;
      hipLaunchKernelGGL(pack_kernel, dim3(grid), dim3(256), 0, stream, tmp_ids, offsets, out_offsets, batch, out_ids,
                         table->d_id_map);
    }
  } else {
    int64_t* tile_sum = (int64_t*)(ws + w.tile_sum);
    int64_t* slot_out = (int64_t*)(ws + w.slot_out);
    if (w.max_slots <= kSmallSlots) {
      hipLaunchKernelGGL(slot_offsets_small_kernel, dim3(1), dim3(1024), 0, stream, counts, ctrl, slot_base, slot_string,
                         slot_out, out_offsets, batch);
    } else {
      hipLaunchKernelGGL(tile_sum_kernel, dim3(w.n_tiles), dim3(1024), 0, stream, counts, ctrl, tile_sum);
      hipLaunchKernelGGL(tile_scan_kernel, dim3(1), dim3(64), 0, stream, tile_sum, w.n_tiles, ctrl, out_offsets, batch);
      hipLaunchKernelGGL(slot_offsets_kernel, dim3(w.n_tiles), dim3(1024), 0, stream, counts, ctrl, tile_sum, slot_base,
                         slot_string, slot_out, out_offsets);
    }
    const int grid = (int)std::min<int64_t>((w.max_slots + 7) / 8, 32768);   // two pieces per wave and round
    hipLaunchKernelGGL(piece_pack_kernel, dim3(grid), dim3(256), 0, stream, tmp_ids, ctrl, piece_begin, counts,
                       slot_out, out_ids, table->d_id_map);
  }
  return hipGetLastError() == hipSuccess ? BPE_OK : BPE_EHIP;
}

static int check_encode_args(const bpe_table* table, const uint8_t* bytes, const int64_t* offsets, int32_t batch,
                             int64_t total_bytes, int32_t max_len, const int32_t* out_ids,
                             const int64_t* out_offsets, int* device) {
  if (!table || batch < 0 || total_bytes < 0 || max_len < 0 || max_len > BPE_MAX_STRING_BYTES)
    return BPE_EINVAL;
  if (!offsets || !out_offsets) return BPE_EINVAL;
  if (total_bytes > 0 && (!bytes || !out_ids)) return BPE_EINVAL;
  if (hipGetDevice(device) != hipSuccess) return BPE_EHIP;
  if (*device != table->device) return BPE_EINVAL;
  return BPE_OK;
}

int bpe_encode_batch(const bpe_table* table, const uint8_t* bytes, const int64_t* offsets, int32_t batch,
                     int64_t total_bytes, int32_t max_len, int32_t* out_ids, int64_t* out_offsets,
                     void* workspace, size_t workspace_bytes, void* stream_ptr) {
  int device = -1;
  const int status = check_encode_args(table, bytes, offsets, batch, total_bytes, max_len, out_ids, out_offsets,
                                       &device);
  if (status != BPE_OK) return status;
  if (!workspace || ((uintptr_t)workspace & 255) != 0) return BPE_EINVAL;
  const WorkspaceLayout w = layout_for(batch, total_bytes, max_len);
  if (workspace_bytes < w.total) return BPE_EINVAL;
  return encode_enqueue(table, bytes, offsets, batch, total_bytes, max_len, out_ids, out_offsets, workspace, w,
                        stream_ptr);
}

int bpe_encode_batch_static(const bpe_table* table, const uint8_t* bytes, const int64_t* offsets, int32_t batch,
                            int64_t total_bytes, int32_t max_len, int32_t* out_ids, int64_t* out_offsets,
                            void* stream_ptr) {
  int device = -1;
  const int status = check_encode_args(table, bytes, offsets, batch, total_bytes, max_len, out_ids, out_offsets,
                                       &device);
  if (status != BPE_OK) return status;
  if (batch > BPE_STATIC_MAX_BATCH || total_bytes > BPE_STATIC_MAX_TOTAL_BYTES ||
      max_len > BPE_STATIC_MAX_STRING_BYTES)
    return BPE_ETOOBIG;
  const WorkspaceLayout w = layout_for(batch, total_bytes, max_len);
  if (w.total > kStaticScratchBytes) return BPE_ETOOBIG;           // cannot happen within the three limits
  if (device < 0 || device >= kMaxDevices) return BPE_EINVAL;
  void* scratch = nullptr;
  {
    // The array's name is only a host-side handle: its device address, different on every GPU, comes from the
    // runtime, once per device, with that device current (it is: `device` is the current one).
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[device]) {
      void* p = nullptr;
      if (hipGetSymbolAddress(&p, HIP_SYMBOL(g_static_scratch)) != hipSuccess || !p) return BPE_EHIP;
      g_scratch_ptr[device] = p;
    }
    scratch = g_scratch_ptr[device];
  }
  return encode_enqueue(table, bytes, offsets, batch, total_bytes, max_len, out_ids, out_offsets, scratch, w,
                        stream_ptr);
}

int bpe_set_profiling(int enabled) {
  std::lock_guard<std::mutex> lock(g_prof_mutex);
  g_prof.used = 0;
  g_profiling = false;
  if (!enabled) return BPE_OK;
  while (g_prof.created < kProfileRing) {                // set-up: the only place where events are created
    if (hipEventCreate(&g_prof.begin[g_prof.created]) != hipSuccess) return BPE_EHIP;
    if (hipEventCreate(&g_prof.end[g_prof.created]) != hipSuccess) {
      (void)hipEventDestroy(g_prof.begin[g_prof.created]);
      return BPE_EHIP;
    }
    ++g_prof.created;
  }
  g_profiling = true;
  return BPE_OK;
}

int bpe_read_profile(float* total_ms, int32_t* calls) {
  if (!total_ms || !calls) return BPE_EINVAL;
  std::lock_guard<std::mutex> lock(g_prof_mutex);
  float sum = 0.0f;
  for (int i = 0; i < g_prof.used; ++i) {
    float ms = 0.0f;
    if (hipEventSynchronize(g_prof.end[i]) != hipSuccess ||
        hipEventElapsedTime(&ms, g_prof.begin[i], g_prof.end[i]) != hipSuccess)
      return BPE_EHIP;
    sum += ms;
  }
  *total_ms = sum;
  *calls = g_prof.used;
  return BPE_OK;
}

const char* bpe_strerror(int code) {
  switch (code) {
    case BPE_OK: return "ok";
    case BPE_EINVAL: return "invalid argument";
    case BPE_EBADMERGE: return "merge row uses a token id that does not exist before that row";
    case BPE_EDUPPAIR: return "the same pair appears in two merge rows";
    case BPE_ENOMEM: return "out of memory";
    case BPE_EHIP: return "HIP runtime call failed";
    case BPE_ETOOBIG: return "too many merge rows for the table format";
    case BPE_EDUPID: return "two tokens of the vocabulary share an id";
    case BPE_ESPECIAL: return "occurrences of the special tokens could overlap";
    default: return "unknown error";
  }
}

}  // extern "C"
