// Host-side encoder of libtq (off the hot path): per-row int8 quantization (paper section 3, 8-bit setting),
// segmentation of the rows, and LZW with a size-capped, frozen dictionary (paper Background "Compression"),
// laid out as interleaved lane streams per unit of 16 rows x 4 segments.
#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <new>
#include <thread>
#include <vector>

#include "../../include/tq.h"
#include "tq_format.h"

namespace tq {

namespace {

constexpr uint32_t kNone = 0xFFFFFFFFu;

unsigned pick_threads(uint32_t asked) {
  unsigned hw = std::thread::hardware_concurrency();
  if (hw == 0) hw = 1;
  unsigned n = asked ? asked : hw;
  return std::max(1u, std::min(n, 16u));
}

template <typename F>
void parallel_for(uint64_t n, unsigned n_threads, F&& body) {  // body(begin, end, thread_index)
  n_threads = (unsigned)std::min<uint64_t>(n_threads, std::max<uint64_t>(n, 1));
  if (n_threads <= 1) {
    body(0, n, 0);
    return;
  }
  std::vector<std::thread> th;
  uint64_t per = (n + n_threads - 1) / n_threads;
  for (unsigned t = 0; t < n_threads; ++t) {
    uint64_t b = std::min<uint64_t>(n, t * per), e = std::min<uint64_t>(n, b + per);
    th.emplace_back([=, &body] { body(b, e, t); });
  }
  for (auto& x : th) x.join();
}

// Dictionary of runs of up to 4 bytes, in the order LZW creates them (the container's code space is that order sorted by
// run length: final_codes()).  Codes 0..255 are the single bytes; a two-byte run is found through a direct table over
// the byte pair, a longer one through a hash table over (code of the run it extends, next byte).
class RunDict {
 public:
  RunDict(uint32_t max_entries, uint32_t lmax, uint32_t unit_budget)
      : max_(max_entries), lmax_(lmax), budget_(unit_budget), units_(256), pair_(65536, kNone) {
    bytes_.reserve(max_entries + 1);
    len_.reserve(max_entries + 1);
    for (uint32_t b = 0; b < 256; ++b) {
      bytes_.push_back(b);
      len_.push_back(1);
    }
    if (lmax > 2) {
      mask_ = 1u << 17;
      while (mask_ < 4u * max_entries) mask_ <<= 1;
      key_.assign(mask_, kNone);
      val_.assign(mask_, 0);
      --mask_;
    }
  }
  uint32_t size() const { return (uint32_t)bytes_.size(); }
  uint32_t length(uint32_t code) const { return len_[code]; }
  uint32_t word(uint32_t code) const { return bytes_[code]; }
  // no further entry can be added (count reached, or not even a two-byte run fits the unit budget)
  bool full() const { return size() >= max_ || lmax_ < 2 || (budget_ && units_ + 1 > budget_); }

  // The run (entry `parent` + byte b) as a new entry; false when it exists, is too long or does not fit.
  bool add(uint32_t parent, uint32_t b) {
    const uint32_t len = len_[parent] + 1, cost = len <= 2 ? 1u : 2u;
    if (len > lmax_ || size() >= max_ || (budget_ && units_ + cost > budget_) || child(parent, b) != kNone) return false;
    const uint32_t code = size();
    if (len == 2) {
      pair_[parent << 8 | b] = code;
    } else {
      uint32_t h = hash(parent << 8 | b);
      while (key_[h] != kNone) h = (h + 1) & mask_;
      key_[h] = parent << 8 | b;
      val_[h] = code;
    }
    bytes_.push_back(bytes_[parent] | b << (8 * len_[parent]));
    len_.push_back((uint8_t)len);
    units_ += cost;
    return true;
  }
  uint32_t child(uint32_t parent, uint32_t b) const {
    if (parent < 256) return pair_[parent << 8 | b];
    if (lmax_ <= 2) return kNone;
    const uint32_t k = parent << 8 | b;
    for (uint32_t h = hash(k); key_[h] != kNone; h = (h + 1) & mask_)
      if (key_[h] == k) return val_[h];
    return kNone;
  }
  // Continue from the dictionary section of another container: its entries from 256 on, which come sorted by length,
  // so each follows the run it extends.  lens[e] = length of entry e.
  bool adopt(const uint32_t* words, const std::vector<uint8_t>& lens, uint32_t n) {
    for (uint32_t e = 256; e < n; ++e) {
      const uint32_t w = words[e], len = lens[e];
      if (len < 2 || len > lmax_) return false;
      uint32_t parent = w & 0xFFu;
      for (uint32_t k = 1; k + 1 < len && parent != kNone; ++k) parent = child(parent, w >> (8 * k) & 0xFFu);
      if (parent == kNone || !add(parent, w >> (8 * (len - 1)) & 0xFFu)) return false;
    }
    return true;
  }

  // Greedy parse of S[gs, ge): longest entry at each position, never crossing ge.  While `kGrow`, the matched run plus
  // the following byte becomes a new entry if it fits.  Codes are written in creation order.
  template <bool kGrow>
  void parse(const uint8_t* S, uint64_t gs, uint64_t ge, std::vector<uint16_t>& out) {
    uint64_t i = gs;
    if (lmax_ <= 2) {   // the common case: one table lookup per position
      while (i < ge) {
        uint32_t code = S[i], m = 1;
        if (lmax_ == 2 && i + 1 < ge) {
          const uint32_t pc = pair_[(uint32_t)S[i] << 8 | S[i + 1]];
          if (pc != kNone) {
            code = pc;
            m = 2;
          }
        }
        out.push_back((uint16_t)code);
        if (kGrow && m < lmax_ && i + m < ge) add(code, S[i + 1]);   // m == 1 here: the new entry is a pair
        i += m;
      }
      return;
    }
    while (i < ge) {
      uint32_t code = S[i], m = 1;
      while (m < lmax_ && i + m < ge) {
        const uint32_t c = child(code, S[i + m]);
        if (c == kNone) break;
        code = c;
        ++m;
      }
      out.push_back((uint16_t)code);
      if (kGrow && m < lmax_ && i + m < ge) add(code, S[i + m]);
      i += m;
    }
  }

  // The container's numbering: entries in order of run length, equal lengths in order of creation.
  // final_of[creation code] = container code; class_end[k] = entries of at most k + 1 bytes.
  void final_codes(std::vector<uint16_t>* final_of, std::vector<uint32_t>* words, uint32_t class_end[4]) const {
    const uint32_t n = size();
    uint32_t count[5] = {0, 0, 0, 0, 0};
    for (uint32_t e = 0; e < n; ++e) ++count[len_[e]];
    uint32_t next[5] = {0, 0, count[1], count[1] + count[2], count[1] + count[2] + count[3]};
    for (int k = 0; k < 4; ++k) class_end[k] = next[k + 1] + count[k + 1];
    final_of->assign(n + 1, 0);
    words->assign(n, 0);
    for (uint32_t e = 0; e < n; ++e) {
      const uint32_t f = next[len_[e]]++;
      (*final_of)[e] = (uint16_t)f;
      (*words)[f] = bytes_[e];
    }
    (*final_of)[n] = (uint16_t)n;   // the pad code
  }

 private:
  uint32_t hash(uint32_t k) const { return (k * 2654435761u) >> 7 & mask_; }
  uint32_t max_, lmax_, budget_, units_, mask_ = 0;
  std::vector<uint32_t> pair_, bytes_, key_, val_;
  std::vector<uint8_t> len_;
};

int check_opts(const tq_encode_opts* o, uint32_t* max_entries, uint32_t* lmax, uint32_t* seg_cols, unsigned* n_threads) {
  *max_entries = (o && o->max_entries) ? o->max_entries : TQ_MAX_ENTRIES_DEVICE;
  *lmax = (o && o->lmax) ? o->lmax : TQ_DEFAULT_LMAX;
  // (packed values: the same number of weights per segment by default)
  *seg_cols = (o && o->seg_cols) ? o->seg_cols : (o && o->packing == TQ_PACK_NIBBLES) ? TQ_DEFAULT_SEG_COLS / 2 : TQ_DEFAULT_SEG_COLS;
  *n_threads = pick_threads(o ? o->n_threads : 0);
  if (*lmax < 1 || *lmax > TQ_MAX_LMAX) {
    set_error("tq_encode: lmax must be 0 (default) or in [1, " + std::to_string(TQ_MAX_LMAX) + "]");
    return TQ_E_INVALID_ARG;
  }
  if (*max_entries < 256 || *max_entries > TQ_MAX_ENTRIES_DEVICE) {
    set_error("tq_encode: max_entries must be 0 or in [256, " + std::to_string(TQ_MAX_ENTRIES_DEVICE) + "]");
    return TQ_E_INVALID_ARG;
  }
  if (*seg_cols < kMinSegCols || *seg_cols > kMaxSegCols || *seg_cols % 16) {
    set_error("tq_encode: seg_cols must be a multiple of 16 in [16, 1024]");
    return TQ_E_INVALID_ARG;
  }
  if (o && (o->dict_from != nullptr) != (o->dict_from_bytes != 0)) {
    set_error("tq_encode: dict_from and dict_from_bytes must be given together");
    return TQ_E_INVALID_ARG;
  }
  if (o && o->dictionary != TQ_DICT_LZW && o->dictionary != TQ_DICT_FREQUENCY) {
    set_error("tq_encode: dictionary must be TQ_DICT_LZW or TQ_DICT_FREQUENCY");
    return TQ_E_INVALID_ARG;
  }
  if (o && o->dictionary == TQ_DICT_FREQUENCY && *lmax > 2) {
    set_error("tq_encode: TQ_DICT_FREQUENCY picks runs of 2 bytes; use lmax 1 or 2 with it");
    return TQ_E_INVALID_ARG;
  }
  if (o && o->bits != 0 && (o->bits < 2 || o->bits > 8)) {
    set_error("tq_encode: bits must be 0 (= 8) or in [2, 8]");
    return TQ_E_INVALID_ARG;
  }
  if (o && o->packing > TQ_PACK_NIBBLES) {
    set_error("tq_encode: packing must be TQ_PACK_NONE or TQ_PACK_NIBBLES");
    return TQ_E_INVALID_ARG;
  }
  return TQ_OK;
}

// Codes of a contiguous range of units, concatenated in (unit, lane) order; cnt[(u - u_begin) * 64 + lane] codes each.
struct UnitRange {
  uint64_t u_begin = 0, u_end = 0;
  std::vector<uint16_t> codes;
  std::vector<uint16_t> cnt;
};

// Two 4-bit values per byte (low nibble: the even column).  false if a value does not fit or the column count is odd.
bool pack_nibbles(const std::vector<uint8_t>& Q, uint32_t rows, uint32_t cols, std::vector<uint8_t>* out) {
  if (cols % 2) {
    set_error("tq_encode: packing needs an even number of columns");
    return false;
  }
  out->assign((size_t)rows * (cols / 2), 0);
  for (size_t i = 0; i < out->size(); ++i) {
    const int a = (int8_t)Q[2 * i], b = (int8_t)Q[2 * i + 1];
    if (a < -8 || a > 7 || b < -8 || b > 7) {
      set_error("tq_encode: packing takes values in [-8, 7]");
      return false;
    }
    (*out)[i] = (uint8_t)((a & 15) | (b & 15) << 4);
  }
  return true;
}

// Q: the byte matrix rows x cols that is coded (for packing 1 the packed one).
int encode_quantized_matrix(const std::vector<uint8_t>& Q, const std::vector<float>& scales_pad, uint32_t rows, uint32_t cols,
                            const tq_encode_opts* opts, void** blob_out, size_t* bytes_out) {
  uint32_t max_entries, lmax, seg_cols;
  unsigned n_threads;
  if (int rc = check_opts(opts, &max_entries, &lmax, &seg_cols, &n_threads)) return rc;
  Header h;
  std::memset(&h, 0, sizeof h);
  std::memcpy(h.magic, kMagic, 8);
  h.version = kVersion;
  h.header_bytes = kHeaderBytes;
  h.rows = rows;
  h.cols = cols;
  h.seg_cols = seg_cols;
  h.unit_rows = kUnitRows;
  h.unit_panels = kUnitPanels;
  h.chunk_codes = kChunkCodes;
  h.n_bands = (rows + kUnitRows - 1) / kUnitRows;
  h.n_panels = (cols + seg_cols - 1) / seg_cols;
  h.n_quads = (h.n_panels + kUnitPanels - 1) / kUnitPanels;
  h.n_units = (uint64_t)h.n_bands * h.n_quads;
  h.lmax = lmax;
  h.max_entries = max_entries;
  h.packing = opts ? opts->packing : 0;
  const uint64_t n_units = h.n_units;

  // (runs longer than 2 bytes take two units of the device's dictionary storage each: the unit budget then applies)
  RunDict dict(max_entries, lmax, lmax > 2 ? kUnitBudget : 0u);
  if (opts && opts->dict_from) {
    // One LZW dictionary over a sequence of matrices: start from the entries the earlier container ended with.
    Header fh;
    if (int rc = validate_blob(opts->dict_from, (size_t)opts->dict_from_bytes, &fh, nullptr, n_threads)) return rc;
    std::vector<uint8_t> lens(fh.n_entries);
    for (uint32_t e = 0; e < fh.n_entries; ++e) lens[e] = (uint8_t)run_length(fh, e);
    if (fh.lmax > lmax || fh.n_entries > max_entries ||
        !dict.adopt((const uint32_t*)((const uint8_t*)opts->dict_from + fh.off_dict), lens, fh.n_entries)) {
      set_error("tq_encode: the dictionary of dict_from does not fit this lmax / max_entries");
      return TQ_E_INVALID_ARG;
    }
  }
  auto parse_unit = [&](uint64_t u, bool grow, UnitRange& out) {
    const uint32_t band = (uint32_t)(u / h.n_quads), quad = (uint32_t)(u % h.n_quads);
    for (uint32_t lane = 0; lane < 64; ++lane) {
      const uint32_t len = segment_len(h, band, quad, lane);
      const size_t before = out.codes.size();
      if (len) {
        const uint64_t start = (uint64_t)(band * kUnitRows + (lane & 15)) * cols + (uint64_t)(quad * kUnitPanels + (lane >> 4)) * seg_cols;
        if (grow) dict.parse<true>(Q.data(), start, start + len, out.codes);
        else dict.parse<false>(Q.data(), start, start + len, out.codes);
      }
      out.cnt.push_back((uint16_t)(out.codes.size() - before));
    }
  };

  const bool by_frequency = opts && opts->dictionary == TQ_DICT_FREQUENCY;
  if (by_frequency && !(opts && opts->dict_from) && lmax >= 2 && max_entries > 256) {
    // The most frequent pairs of neighbouring bytes, counted at every offset inside a segment, segments in the order
    // they are parsed in; ties go to the pair seen first.
    std::vector<uint64_t> count(65536, 0), first(65536, 0);
    uint64_t seen = 0;
    for (uint64_t uu = 0; uu < n_units; ++uu) {
      const uint32_t band = (uint32_t)(uu / h.n_quads), quad = (uint32_t)(uu % h.n_quads);
      for (uint32_t lane = 0; lane < 64; ++lane) {
        const uint32_t len = segment_len(h, band, quad, lane);
        if (len < 2) continue;
        const uint8_t* seg = Q.data() + (uint64_t)(band * kUnitRows + (lane & 15)) * cols + (uint64_t)(quad * kUnitPanels + (lane >> 4)) * seg_cols;
        for (uint32_t i = 0; i + 1 < len; ++i) {
          const uint32_t key = (uint32_t)seg[i] << 8 | seg[i + 1];
          if (count[key]++ == 0) first[key] = seen;
          ++seen;
        }
      }
    }
    std::vector<uint32_t> keys;
    for (uint32_t k = 0; k < 65536; ++k)
      if (count[k]) keys.push_back(k);
    std::sort(keys.begin(), keys.end(), [&](uint32_t a, uint32_t b) { return count[a] != count[b] ? count[a] > count[b] : first[a] < first[b]; });
    for (uint32_t k : keys)
      if (!dict.add(k >> 8, k & 0xFF)) break;
  }

  // Phase 1 (sequential): units in order while the dictionary can still grow.
  std::vector<UnitRange> ranges(1 + n_threads);
  uint64_t u = 0;
  for (; !by_frequency && u < n_units && !dict.full(); ++u) parse_unit(u, true, ranges[0]);
  ranges[0].u_end = u;
  const uint64_t u_frozen = u;
  const uint32_t n_entries = dict.size();
  const uint16_t pad = (uint16_t)n_entries;
  // The container's code space is sorted by run length; the parse above and below numbers entries as they were created.
  std::vector<uint16_t> final_of;
  std::vector<uint32_t> words;
  dict.final_codes(&final_of, &words, h.class_end);

  // Phase 2 (parallel): the dictionary no longer changes, units are independent.
  {
    const uint64_t rest = n_units - u_frozen, per = (rest + n_threads - 1) / std::max(1u, n_threads);
    std::vector<std::thread> th;
    for (unsigned t = 0; t < n_threads; ++t) {
      UnitRange& r = ranges[1 + t];
      r.u_begin = std::min<uint64_t>(n_units, u_frozen + t * per);
      r.u_end = std::min<uint64_t>(n_units, r.u_begin + per);
      if (r.u_begin >= r.u_end) continue;
      th.emplace_back([&, t] {
        UnitRange& rr = ranges[1 + t];
        rr.codes.reserve((rr.u_end - rr.u_begin) * 64 * (seg_cols / 2 + 8));
        for (uint64_t uu = rr.u_begin; uu < rr.u_end; ++uu) parse_unit(uu, false, rr);
      });
    }
    for (auto& x : th) x.join();
  }

  // Unit lengths in chunks: the longest lane stream, rounded up to whole chunks.
  std::vector<uint32_t> uoff(n_units + 1, 0);
  uint64_t acc = 0, n_real = 0;
  for (const UnitRange& r : ranges)
    for (uint64_t uu = r.u_begin; uu < r.u_end; ++uu) {
      const uint16_t* c = r.cnt.data() + (uu - r.u_begin) * 64;
      uint32_t mx = 0;
      for (int l = 0; l < 64; ++l) {
        mx = std::max<uint32_t>(mx, c[l]);
        n_real += c[l];
      }
      uoff[uu] = (uint32_t)acc;
      acc += (mx + kChunkCodes - 1) / kChunkCodes;
      if (acc >= 0xFFFFFFFFull / kChunkWords) {
        set_error("tq_encode: code stream exceeds 2^32 codes");
        return TQ_E_UNSUPPORTED;
      }
    }
  uoff[n_units] = (uint32_t)acc;

  h.n_entries = n_entries;
  h.pad_code = n_entries;
  h.n_chunks = acc;
  h.n_real_codes = n_real;
  h.dict_bytes = (uint64_t)(n_entries + 1) * 4;
  h.uoff_bytes = (n_units + 1) * 4;
  h.code_bytes = h.n_chunks * kChunkWords * 2;
  h.scale_bytes = (uint64_t)h.n_bands * kUnitRows * 4;
  h.off_dict = kHeaderBytes;
  h.off_uoff = round_up(h.off_dict + h.dict_bytes, kSectionAlign);
  h.off_codes = round_up(h.off_uoff + h.uoff_bytes, kSectionAlign);
  h.off_scales = round_up(h.off_codes + h.code_bytes, kSectionAlign);
  h.total_bytes = round_up(h.off_scales + h.scale_bytes, kSectionAlign);

  uint8_t* blob = (uint8_t*)std::calloc(1, h.total_bytes);
  if (!blob) {
    set_error("tq_encode: out of host memory");
    return TQ_E_OOM;
  }
  std::memcpy(blob, &h, sizeof h);
  std::memcpy(blob + h.off_dict, words.data(), (size_t)n_entries * 4);  // pad entry stays zero
  std::memcpy(blob + h.off_uoff, uoff.data(), uoff.size() * 4);
  uint16_t* codes = (uint16_t*)(blob + h.off_codes);
  {
    // Interleave: code k of lane l of unit u -> codes[(uoff[u] + k / 4) * 256 + l * 4 + k % 4]; pad the rest.
    auto fill = [&](const UnitRange& r) {
      const uint16_t* src = r.codes.data();
      for (uint64_t uu = r.u_begin; uu < r.u_end; ++uu) {
        const uint16_t* c = r.cnt.data() + (uu - r.u_begin) * 64;
        const uint32_t len = (uoff[uu + 1] - uoff[uu]) * kChunkCodes;
        uint16_t* base = codes + (uint64_t)uoff[uu] * kChunkWords;
        for (uint32_t l = 0; l < 64; ++l) {
          for (uint32_t k = 0; k < len; ++k) base[(uint64_t)(k / kChunkCodes) * kChunkWords + l * kChunkCodes + k % kChunkCodes] = k < c[l] ? final_of[src[k]] : pad;
          src += c[l];
        }
      }
    };
    std::vector<std::thread> th;
    for (size_t i = 1; i < ranges.size(); ++i)
      if (ranges[i].u_begin < ranges[i].u_end) th.emplace_back([&, i] { fill(ranges[i]); });
    fill(ranges[0]);
    for (auto& x : th) x.join();
  }
  std::memcpy(blob + h.off_scales, scales_pad.data(), (size_t)h.n_bands * kUnitRows * 4);
  *blob_out = blob;
  *bytes_out = (size_t)h.total_bytes;
  return TQ_OK;
}

}  // namespace
}  // namespace tq

using namespace tq;

extern "C" int tq_encode(const float* w, uint32_t rows, uint32_t cols, const tq_encode_opts* opts, void** blob,
                         size_t* blob_bytes) {
  try {
    if (!w || !blob || !blob_bytes || rows == 0 || cols == 0) {
      set_error("tq_encode: null pointer or empty matrix");
      return TQ_E_INVALID_ARG;
    }
    const unsigned nt = pick_threads(opts ? opts->n_threads : 0);
    const uint32_t rows_pad = (uint32_t)round_up(rows, kUnitRows);
    std::vector<uint8_t> Q((size_t)rows * cols, 0);
    std::vector<float> scales(rows_pad, 0.f);
    // Per row, in IEEE fp32 and in this order: amax = max|w|, s = amax / qmax, q = clamp(rne(w / s), -qmax, qmax),
    // qmax = 2^(bits - 1) - 1 (paper section 3: a fixed range of levels set by the number of bits; 127 at 8 bits).
    if (opts && opts->bits != 0 && (opts->bits < 2 || opts->bits > 8)) {
      set_error("tq_encode: bits must be 0 (= 8) or in [2, 8]");
      return TQ_E_INVALID_ARG;
    }
    const bool packed = opts && opts->packing == TQ_PACK_NIBBLES;
    if (packed && (opts->bits < 2 || opts->bits > 4)) {
      set_error("tq_encode: TQ_PACK_NIBBLES takes bits 2..4");
      return TQ_E_INVALID_ARG;
    }
    const float qmax = (float)((1u << ((opts && opts->bits ? opts->bits : 8u) - 1)) - 1u);
    parallel_for(rows, nt, [&](uint64_t rb, uint64_t re, unsigned) {
      for (uint64_t r = rb; r < re; ++r) {
        const float* row = w + r * cols;
        float amax = 0.f;
        for (uint32_t c = 0; c < cols; ++c) amax = std::max(amax, std::fabs(row[c]));
        const float s = amax / qmax;
        scales[r] = s;
        if (!(s > 0.f)) continue;  // all-zero row: bytes stay 0
        for (uint32_t c = 0; c < cols; ++c) {
          float t = std::nearbyintf(row[c] / s);  // default rounding mode: to nearest, ties to even
          t = std::min(qmax, std::max(-qmax, t));
          Q[r * cols + c] = (uint8_t)(int8_t)(int)t;
        }
      }
    });
    if (packed) {
      std::vector<uint8_t> P;
      if (!pack_nibbles(Q, rows, cols, &P)) return TQ_E_INVALID_ARG;
      return encode_quantized_matrix(P, scales, rows, cols / 2, opts, blob, blob_bytes);
    }
    return encode_quantized_matrix(Q, scales, rows, cols, opts, blob, blob_bytes);
  } catch (const std::bad_alloc&) {
    set_error("tq_encode: out of host memory");
    return TQ_E_OOM;
  }
}

extern "C" int tq_encode_quantized(const int8_t* q, const float* scales_in, uint32_t rows, uint32_t cols,
                                   const tq_encode_opts* opts, void** blob, size_t* blob_bytes) {
  try {
    if (!q || !scales_in || !blob || !blob_bytes || rows == 0 || cols == 0) {
      set_error("tq_encode_quantized: null pointer or empty matrix");
      return TQ_E_INVALID_ARG;
    }
    const uint32_t rows_pad = (uint32_t)round_up(rows, kUnitRows);
    std::vector<uint8_t> Q((const uint8_t*)q, (const uint8_t*)q + (size_t)rows * cols);
    std::vector<float> scales(rows_pad, 0.f);
    std::copy(scales_in, scales_in + rows, scales.begin());
    if (opts && opts->packing == TQ_PACK_NIBBLES) {
      std::vector<uint8_t> P;
      if (!pack_nibbles(Q, rows, cols, &P)) return TQ_E_INVALID_ARG;
      return encode_quantized_matrix(P, scales, rows, cols / 2, opts, blob, blob_bytes);
    }
    return encode_quantized_matrix(Q, scales, rows, cols, opts, blob, blob_bytes);
  } catch (const std::bad_alloc&) {
    set_error("tq_encode_quantized: out of host memory");
    return TQ_E_OOM;
  }
}

extern "C" int tq_encode_gate_up(const float* w_gate, const float* w_up, uint32_t rows, uint32_t cols, const tq_encode_opts* opts,
                                 void** blob, size_t* blob_bytes) {
  if (!w_gate || !w_up || !blob || !blob_bytes || rows == 0 || cols == 0 || rows > 0x7FFFFFFFu) {
    set_error("tq_encode_gate_up: null pointer or empty shape");
    return TQ_E_INVALID_ARG;
  }
  try {
    std::vector<float> w((size_t)2 * rows * cols);   // row 2r = gate row r, row 2r + 1 = up row r
    for (uint32_t r = 0; r < rows; ++r) {
      std::memcpy(w.data() + (size_t)(2 * r) * cols, w_gate + (size_t)r * cols, (size_t)cols * 4);
      std::memcpy(w.data() + (size_t)(2 * r + 1) * cols, w_up + (size_t)r * cols, (size_t)cols * 4);
    }
    return tq_encode(w.data(), 2 * rows, cols, opts, blob, blob_bytes);
  } catch (const std::bad_alloc&) {
    set_error("tq_encode_gate_up: out of host memory");
    return TQ_E_OOM;
  }
}

extern "C" void tq_free_blob(void* blob) { std::free(blob); }
