// Host-side encoder of libtq (off the hot path): per-row int8 quantization (paper section 3, 8-bit setting),
// micro-tile serialization, and LZW with a size-capped, frozen dictionary (paper Background "Compression").
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

// Dictionary for runs of at most 3 bytes.  Codes 0..255 are the single bytes.  Two-byte runs are found through a
// direct table over the byte pair; three-byte runs through an open-addressing table keyed by (pair code, byte).
class Dict3 {
 public:
  Dict3(uint32_t max_entries, uint32_t lmax) : max_(max_entries), lmax_(lmax), pair_(65536, kNone) {
    uint32_t cap = 1;
    while (cap < 2 * max_entries) cap <<= 1;
    tmask_ = cap - 1;
    tkey_.assign(cap, kNone);
    tval_.assign(cap, 0);
    slot_.reserve(max_entries + 1);
    for (uint32_t b = 0; b < 256; ++b) slot_.push_back(b | (8u << 24));   // top byte: run length in bits
  }
  uint32_t size() const { return (uint32_t)slot_.size(); }
  bool full() const { return size() >= max_; }
  const std::vector<uint32_t>& slots() const { return slot_; }

  // Greedy parse of S[gs, ge): longest entry at each position, never crossing ge.  While `grow` and the
  // dictionary is not full, the matched run plus the following byte becomes a new entry.
  template <bool kGrow>
  void parse(const uint8_t* S, uint64_t gs, uint64_t ge, std::vector<uint16_t>& out) {
    uint64_t i = gs;
    while (i < ge) {
      uint32_t code = S[i];
      uint32_t m = 1;
      if (lmax_ >= 2 && i + 1 < ge) {
        uint32_t pc = pair_[(uint32_t)S[i] << 8 | S[i + 1]];
        if (pc != kNone) {
          code = pc;
          m = 2;
          if (lmax_ >= 3 && i + 2 < ge) {
            uint32_t tc = find3(pc, S[i + 2]);
            if (tc != kNone) {
              code = tc;
              m = 3;
            }
          }
        }
      }
      out.push_back((uint16_t)code);
      if (kGrow && !full() && m < lmax_ && i + m < ge) {
        uint32_t nb = S[i + m];
        uint32_t id = size();
        if (m == 1) {
          pair_[code << 8 | nb] = id;
          slot_.push_back(code | nb << 8 | 16u << 24);
        } else {
          insert3(code, nb, id);
          slot_.push_back((slot_[code] & 0xFFFFu) | nb << 16 | 24u << 24);
        }
      }
      i += m;
    }
  }

 private:
  static uint32_t hash(uint32_t k) { return (k * 2654435761u) >> 7; }
  uint32_t find3(uint32_t pc, uint32_t b) const {
    uint32_t key = pc << 8 | b;
    for (uint32_t h = hash(key) & tmask_;; h = (h + 1) & tmask_) {
      if (tkey_[h] == key) return tval_[h];
      if (tkey_[h] == kNone) return kNone;
    }
  }
  void insert3(uint32_t pc, uint32_t b, uint32_t id) {
    uint32_t key = pc << 8 | b;
    uint32_t h = hash(key) & tmask_;
    while (tkey_[h] != kNone) h = (h + 1) & tmask_;
    tkey_[h] = key;
    tval_[h] = id;
  }
  uint32_t max_, lmax_;
  std::vector<uint32_t> pair_;
  uint32_t tmask_;
  std::vector<uint32_t> tkey_, tval_;
  std::vector<uint32_t> slot_;
};

int check_opts(const tq_encode_opts* o, uint32_t* max_entries, uint32_t* lmax, unsigned* n_threads) {
  *max_entries = (o && o->max_entries) ? o->max_entries : TQ_DEFAULT_MAX_ENTRIES;
  *lmax = (o && o->lmax) ? o->lmax : TQ_DEFAULT_LMAX;
  *n_threads = pick_threads(o ? o->n_threads : 0);
  if (*max_entries < 256 || *max_entries > TQ_MAX_ENTRIES_DEVICE) {
    set_error("tq_encode: max_entries must be in [256, " + std::to_string(TQ_MAX_ENTRIES_DEVICE) + "]");
    return TQ_E_INVALID_ARG;
  }
  if (*lmax > 3) {
    set_error("tq_encode: lmax must be 0 (auto), 1, 2 or 3");
    return TQ_E_INVALID_ARG;
  }
  return TQ_OK;
}

// Serialized position of element (r, c) of the padded matrix.
inline uint64_t ser_index(uint64_t r, uint64_t c, uint64_t cols_pad) {
  return (r / kTileRows) * (kTileRows * cols_pad) + (c / kMtCols) * (kTileRows * kMtCols) + (r % kTileRows) * kMtCols +
         (c % kMtCols);
}

int encode_with_lmax(const std::vector<uint8_t>& S, const std::vector<float>& scales_pad, uint32_t rows, uint32_t cols,
                     uint32_t rows_pad, uint32_t cols_pad, uint32_t max_entries, uint32_t lmax, unsigned n_threads,
                     void** blob_out, size_t* bytes_out);

// lmax == 0: encode with runs of at most 3 and of at most 2 bytes and keep the smaller container (3 on a tie).
int encode_serialized(const std::vector<uint8_t>& S, const std::vector<float>& scales_pad, uint32_t rows, uint32_t cols,
                      uint32_t rows_pad, uint32_t cols_pad, uint32_t max_entries, uint32_t lmax, unsigned n_threads,
                      void** blob_out, size_t* bytes_out) {
  if (lmax != 0)
    return encode_with_lmax(S, scales_pad, rows, cols, rows_pad, cols_pad, max_entries, lmax, n_threads, blob_out, bytes_out);
  void *b3 = nullptr, *b2 = nullptr;
  size_t n3 = 0, n2 = 0;
  int rc = encode_with_lmax(S, scales_pad, rows, cols, rows_pad, cols_pad, max_entries, 3, n_threads, &b3, &n3);
  if (rc != TQ_OK) return rc;
  rc = encode_with_lmax(S, scales_pad, rows, cols, rows_pad, cols_pad, max_entries, 2, n_threads, &b2, &n2);
  if (rc != TQ_OK) {
    std::free(b3);
    return rc;
  }
  const bool take2 = n2 < n3;
  std::free(take2 ? b3 : b2);
  *blob_out = take2 ? b2 : b3;
  *bytes_out = take2 ? n2 : n3;
  return TQ_OK;
}

int encode_with_lmax(const std::vector<uint8_t>& S, const std::vector<float>& scales_pad, uint32_t rows, uint32_t cols,
                     uint32_t rows_pad, uint32_t cols_pad, uint32_t max_entries, uint32_t lmax, unsigned n_threads,
                     void** blob_out, size_t* bytes_out) {
  const uint64_t n_groups = (uint64_t)(rows_pad / kTileRows) * (cols_pad / kGroupCols);
  Dict3 dict(max_entries, lmax);

  // Phase 1 (sequential): groups in order while the dictionary can still grow.
  std::vector<uint16_t> head;
  std::vector<uint32_t> count(n_groups, 0);
  uint64_t g = 0;
  for (; g < n_groups && !dict.full(); ++g) {
    size_t before = head.size();
    dict.parse<true>(S.data(), g * kGroupBytes, (g + 1) * kGroupBytes, head);
    count[g] = (uint32_t)(head.size() - before);
  }
  const uint64_t g_frozen = g;
  const uint32_t n_entries = dict.size();
  const uint16_t pad = (uint16_t)n_entries;

  // Phase 2 (parallel): the dictionary no longer changes, groups are independent.
  unsigned nt = n_threads;
  std::vector<std::vector<uint16_t>> part(nt);
  std::vector<uint64_t> part_begin(nt + 1, n_groups);
  {
    uint64_t rest = n_groups - g_frozen;
    uint64_t per = (rest + nt - 1) / std::max(1u, nt);
    for (unsigned t = 0; t <= nt; ++t) part_begin[t] = std::min<uint64_t>(n_groups, g_frozen + t * per);
    std::vector<std::thread> th;
    for (unsigned t = 0; t < nt; ++t) {
      if (part_begin[t] >= part_begin[t + 1]) continue;
      th.emplace_back([&, t] {
        std::vector<uint16_t>& out = part[t];
        out.reserve((part_begin[t + 1] - part_begin[t]) * (kGroupBytes / 2 + 64));
        for (uint64_t gg = part_begin[t]; gg < part_begin[t + 1]; ++gg) {
          size_t before = out.size();
          dict.parse<false>(S.data(), gg * kGroupBytes, (gg + 1) * kGroupBytes, out);
          count[gg] = (uint32_t)(out.size() - before);
          while ((out.size() - before) % kCodeAlign) out.push_back(pad);
        }
      });
    }
    for (auto& x : th) x.join();
  }

  // Offsets (in codes) of the padded runs.
  std::vector<uint32_t> goff(n_groups + 1, 0);
  uint64_t acc = 0;
  for (uint64_t i = 0; i < n_groups; ++i) {
    goff[i] = (uint32_t)acc;
    acc += round_up(count[i], kCodeAlign);
    if (acc >= 0xFFFFFFFFull) {
      set_error("tq_encode: code stream exceeds 2^32 codes");
      return TQ_E_UNSUPPORTED;
    }
  }
  goff[n_groups] = (uint32_t)acc;
  const uint64_t n_codes = acc;

  Header h;
  std::memset(&h, 0, sizeof h);
  std::memcpy(h.magic, kMagic, 8);
  h.version = kVersion;
  h.header_bytes = kHeaderBytes;
  h.rows = rows;
  h.cols = cols;
  h.rows_pad = rows_pad;
  h.cols_pad = cols_pad;
  h.tile_rows = kTileRows;
  h.mt_cols = kMtCols;
  h.group_cols = kGroupCols;
  h.group_bytes = kGroupBytes;
  h.n_entries = n_entries;
  h.lmax = lmax;
  h.max_entries = max_entries;
  h.pad_code = n_entries;
  h.n_groups = n_groups;
  h.n_codes = n_codes;
  h.dict_bytes = (uint64_t)(n_entries + 1) * 4;
  h.goff_bytes = (n_groups + 1) * 4;
  h.code_bytes = n_codes * 2;
  h.scale_bytes = (uint64_t)rows_pad * 4;
  h.off_dict = kHeaderBytes;
  h.off_goff = round_up(h.off_dict + h.dict_bytes, kSectionAlign);
  h.off_codes = round_up(h.off_goff + h.goff_bytes, kSectionAlign);
  h.off_scales = round_up(h.off_codes + h.code_bytes, kSectionAlign);
  h.total_bytes = round_up(h.off_scales + h.scale_bytes, kSectionAlign);
  h.code_align = kCodeAlign;

  uint8_t* blob = (uint8_t*)std::calloc(1, h.total_bytes);
  if (!blob) {
    set_error("tq_encode: out of host memory");
    return TQ_E_OOM;
  }
  std::memcpy(blob, &h, sizeof h);
  std::memcpy(blob + h.off_dict, dict.slots().data(), (size_t)n_entries * 4);  // pad entry stays zero
  std::memcpy(blob + h.off_goff, goff.data(), goff.size() * 4);
  uint16_t* codes = (uint16_t*)(blob + h.off_codes);
  {
    size_t src = 0;
    for (uint64_t i = 0; i < g_frozen; ++i) {
      uint16_t* dst = codes + goff[i];
      std::memcpy(dst, head.data() + src, (size_t)count[i] * 2);
      for (uint32_t k = count[i]; k < goff[i + 1] - goff[i]; ++k) dst[k] = pad;
      src += count[i];
    }
    for (unsigned t = 0; t < nt; ++t)
      if (!part[t].empty()) std::memcpy(codes + goff[part_begin[t]], part[t].data(), part[t].size() * 2);
  }
  std::memcpy(blob + h.off_scales, scales_pad.data(), (size_t)rows_pad * 4);
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
    uint32_t max_entries, lmax;
    unsigned nt;
    if (int rc = check_opts(opts, &max_entries, &lmax, &nt)) return rc;
    const uint32_t rows_pad = (uint32_t)round_up(rows, kTileRows), cols_pad = (uint32_t)round_up(cols, kGroupCols);
    std::vector<uint8_t> S((size_t)rows_pad * cols_pad, 0);
    std::vector<float> scales(rows_pad, 0.f);
    // Per row, in IEEE fp32 and in this order: amax = max|w|, s = amax / 127, q = clamp(rne(w / s), -127, 127).
    parallel_for(rows, nt, [&](uint64_t rb, uint64_t re, unsigned) {
      for (uint64_t r = rb; r < re; ++r) {
        const float* row = w + r * cols;
        float amax = 0.f;
        for (uint32_t c = 0; c < cols; ++c) amax = std::max(amax, std::fabs(row[c]));
        const float s = amax / 127.0f;
        scales[r] = s;
        if (!(s > 0.f)) continue;  // all-zero row: bytes stay 0
        for (uint32_t c = 0; c < cols; ++c) {
          float t = std::nearbyintf(row[c] / s);  // default rounding mode: to nearest, ties to even
          t = std::min(127.0f, std::max(-127.0f, t));
          S[ser_index(r, c, cols_pad)] = (uint8_t)(int8_t)(int)t;
        }
      }
    });
    return encode_serialized(S, scales, rows, cols, rows_pad, cols_pad, max_entries, lmax, nt, blob, blob_bytes);
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
    uint32_t max_entries, lmax;
    unsigned nt;
    if (int rc = check_opts(opts, &max_entries, &lmax, &nt)) return rc;
    const uint32_t rows_pad = (uint32_t)round_up(rows, kTileRows), cols_pad = (uint32_t)round_up(cols, kGroupCols);
    std::vector<uint8_t> S((size_t)rows_pad * cols_pad, 0);
    std::vector<float> scales(rows_pad, 0.f);
    parallel_for(rows, nt, [&](uint64_t rb, uint64_t re, unsigned) {
      for (uint64_t r = rb; r < re; ++r) {
        scales[r] = scales_in[r];
        for (uint32_t c = 0; c < cols; ++c) S[ser_index(r, c, cols_pad)] = (uint8_t)q[r * cols + c];
      }
    });
    return encode_serialized(S, scales, rows, cols, rows_pad, cols_pad, max_entries, lmax, nt, blob, blob_bytes);
  } catch (const std::bad_alloc&) {
    set_error("tq_encode_quantized: out of host memory");
    return TQ_E_OOM;
  }
}

extern "C" void tq_free_blob(void* blob) { std::free(blob); }
