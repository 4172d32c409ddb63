// Container validation (host only) and the thread-local error text of libtq.
#include <algorithm>
#include <atomic>
#include <cstring>
#include <string>
#include <thread>
#include <vector>

#include "../../include/tq.h"
#include "tq_format.h"

namespace tq {

static thread_local std::string g_err;
void set_error(const std::string& msg) { g_err = msg; }

static int bad(const std::string& why) {
  set_error("bad container: " + why);
  return TQ_E_BAD_BLOB;
}

int validate_blob(const void* blob, size_t bytes, Header* hdr_out, unsigned n_threads) {
  if (!blob) {
    set_error("null container pointer");
    return TQ_E_INVALID_ARG;
  }
  if (bytes < kHeaderBytes) return bad("shorter than the header");
  Header h;
  std::memcpy(&h, blob, sizeof h);
  if (std::memcmp(h.magic, kMagic, 8) != 0) return bad("magic");
  if (h.version != kVersion || h.header_bytes != kHeaderBytes) return bad("version");
  if (h.tile_rows != kTileRows || h.mt_cols != kMtCols || h.group_cols != kGroupCols || h.group_bytes != kGroupBytes ||
      h.code_align != kCodeAlign)
    return bad("tiling constants");
  if (h.rows == 0 || h.cols == 0) return bad("empty shape");
  if (h.rows_pad != round_up(h.rows, kTileRows) || h.cols_pad != round_up(h.cols, kGroupCols)) return bad("padded shape");
  if (h.n_entries < 256 || h.n_entries > TQ_MAX_ENTRIES_DEVICE) return bad("entry count");
  if (h.lmax < 1 || h.lmax > 3) return bad("lmax");
  if (h.pad_code != h.n_entries) return bad("pad code");
  const uint64_t n_groups = (uint64_t)(h.rows_pad / kTileRows) * (h.cols_pad / kGroupCols);
  if (h.n_groups != n_groups) return bad("group count");
  if (h.total_bytes != bytes) return bad("total size");
  if (h.n_codes >= 0xFFFFFFFFull) return bad("code count");
  if (h.dict_bytes != (uint64_t)(h.n_entries + 1) * 4 || h.goff_bytes != (n_groups + 1) * 4 || h.code_bytes != h.n_codes * 2 ||
      h.scale_bytes != (uint64_t)h.rows_pad * 4)
    return bad("section sizes");
  const uint64_t offs[4] = {h.off_dict, h.off_goff, h.off_codes, h.off_scales};
  const uint64_t lens[4] = {h.dict_bytes, h.goff_bytes, h.code_bytes, h.scale_bytes};
  uint64_t prev_end = kHeaderBytes;
  for (int i = 0; i < 4; ++i) {
    if (offs[i] % kSectionAlign || offs[i] < prev_end || offs[i] > bytes || lens[i] > bytes - offs[i]) return bad("section bounds");
    prev_end = offs[i] + lens[i];
  }
  const uint8_t* base = (const uint8_t*)blob;
  const uint32_t* slot = (const uint32_t*)(base + h.off_dict);
  const uint32_t* goff = (const uint32_t*)(base + h.off_goff);
  const uint16_t* codes = (const uint16_t*)(base + h.off_codes);

  // Dictionary: codes 0..255 are the single bytes; every entry has length 1..lmax and zero bytes past its length;
  // the pad entry is all zero (length 0).
  for (uint32_t e = 0; e < h.n_entries; ++e) {
    uint32_t w = slot[e], bits = w >> 24, len = bits / 8;   // the top byte holds the run length in bits
    if (bits % 8 || len < 1 || len > h.lmax) return bad("dictionary entry length");
    if (len < 3 && (w & 0xFFFFFFu) >> (8 * len)) return bad("dictionary entry has bytes past its length");
    if (e < 256 && w != (e | 8u << 24)) return bad("codes 0..255 must be the single bytes");
  }
  if (slot[h.n_entries] != 0) return bad("pad entry");

  // Offsets.
  if (goff[0] != 0 || goff[n_groups] != h.n_codes) return bad("first/last group offset");
  for (uint64_t g = 0; g < n_groups; ++g)
    if (goff[g + 1] < goff[g] || goff[g] % kCodeAlign || goff[g + 1] > h.n_codes) return bad("group offsets");
  if (h.n_codes % kCodeAlign) return bad("code count alignment");

  // Codes: in range, pads only as a tail of fewer than kCodeAlign codes, runs sum to the group size.
  std::atomic<uint64_t> first_bad(UINT64_MAX);
  n_threads = std::max(1u, std::min(n_threads, 16u));
  n_threads = (unsigned)std::min<uint64_t>(n_threads, n_groups);
  auto work = [&](uint64_t gb, uint64_t ge) {
    for (uint64_t g = gb; g < ge && first_bad.load(std::memory_order_relaxed) == UINT64_MAX; ++g) {
      uint32_t b = goff[g], e = goff[g + 1];
      uint32_t sum = 0, pads = 0;
      bool ok = true;
      for (uint32_t p = b; p < e; ++p) {
        uint32_t c = codes[p];
        if (c > h.n_entries) { ok = false; break; }
        if (c == h.n_entries) { ++pads; continue; }
        if (pads) { ok = false; break; }   // a real code after a pad
        sum += slot[c] >> 27;   // bits / 8
      }
      if (!ok || sum != kGroupBytes || pads >= kCodeAlign) {
        uint64_t cur = first_bad.load();
        while (g < cur && !first_bad.compare_exchange_weak(cur, g)) {}
      }
    }
  };
  if (n_threads <= 1) {
    work(0, n_groups);
  } else {
    std::vector<std::thread> th;
    uint64_t per = (n_groups + n_threads - 1) / n_threads;
    for (unsigned t = 0; t < n_threads; ++t) {
      uint64_t b = std::min(n_groups, t * per), e = std::min(n_groups, b + per);
      if (b < e) th.emplace_back(work, b, e);
    }
    for (auto& x : th) x.join();
  }
  if (first_bad.load() != UINT64_MAX) return bad("code stream of group " + std::to_string(first_bad.load()));
  if (hdr_out) *hdr_out = h;
  return TQ_OK;
}

void fill_info(const Header& h, tq_info* o) {
  std::memset(o, 0, sizeof *o);
  o->rows = h.rows;
  o->cols = h.cols;
  o->rows_pad = h.rows_pad;
  o->cols_pad = h.cols_pad;
  o->n_entries = h.n_entries;
  o->lmax = h.lmax;
  o->n_groups = h.n_groups;
  o->n_codes = h.n_codes;
  o->dict_bytes = h.dict_bytes;
  o->offset_bytes = h.goff_bytes;
  o->code_bytes = h.code_bytes;
  o->scale_bytes = h.scale_bytes;
  o->compressed_bytes = h.dict_bytes + h.goff_bytes + h.code_bytes + h.scale_bytes;
}

}  // namespace tq

extern "C" const char* tq_last_error_string(void) { return tq::g_err.c_str(); }

extern "C" int tq_validate_blob(const void* blob, size_t blob_bytes, tq_info* info) {
  tq::Header h;
  unsigned hw = std::thread::hardware_concurrency();
  int rc = tq::validate_blob(blob, blob_bytes, &h, hw ? hw : 1);
  if (rc == TQ_OK && info) tq::fill_info(h, info);
  return rc;
}
