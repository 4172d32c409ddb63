// Container validation (host only) and the thread-local error text of libtq.
#include <algorithm>
#include <atomic>
#include <cstring>
#include <new>
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

int validate_blob(const void* blob, size_t bytes, Header* hdr_out, BlobFacts* facts_out, unsigned n_threads) {
  if (!blob) {
    set_error("null container pointer");
    return TQ_E_INVALID_ARG;
  }
  if (bytes < kHeaderBytes) return bad("shorter than the header");
  Header h;
  std::memcpy(&h, blob, sizeof h);
  if (std::memcmp(h.magic, kMagic, 8) != 0) return bad("magic");
  if (h.version != kVersion || h.header_bytes != kHeaderBytes) return bad("version");
  if (h.unit_rows != kUnitRows || h.unit_panels != kUnitPanels || h.chunk_codes != kChunkCodes) return bad("layout constants");
  if (h.seg_cols < kMinSegCols || h.seg_cols > kMaxSegCols || h.seg_cols % 16) return bad("segment width");
  if (h.rows == 0 || h.cols == 0) return bad("empty shape");
  if (h.n_bands != (h.rows + kUnitRows - 1) / kUnitRows || h.n_panels != (h.cols + h.seg_cols - 1) / h.seg_cols ||
      h.n_quads != (h.n_panels + kUnitPanels - 1) / kUnitPanels)
    return bad("band / panel / quad counts");
  if (h.lmax < 1 || h.lmax > TQ_MAX_LMAX) return bad("lmax");
  if (h.packing > TQ_PACK_NIBBLES) return bad("packing");
  if (h.packing && h.cols > 0x7FFFFFFFu) return bad("packed width");
  if (h.n_entries < 256 || h.n_entries > TQ_MAX_ENTRIES_DEVICE || h.n_entries > h.max_entries) return bad("entry count");
  if (h.pad_code != h.n_entries) return bad("pad code");
  const uint64_t n_units = (uint64_t)h.n_bands * h.n_quads;
  if (h.n_units != n_units) return bad("unit count");
  if (h.total_bytes != bytes) return bad("total size");
  if (h.n_chunks >= 0xFFFFFFFFull / kChunkWords) return bad("chunk count");
  if (h.dict_bytes != (uint64_t)(h.n_entries + 1) * 4 || h.uoff_bytes != (n_units + 1) * 4 ||
      h.code_bytes != h.n_chunks * kChunkWords * 2 || h.scale_bytes != (uint64_t)h.n_bands * kUnitRows * 4)
    return bad("section sizes");
  const uint64_t offs[4] = {h.off_dict, h.off_uoff, h.off_codes, h.off_scales};
  const uint64_t lens[4] = {h.dict_bytes, h.uoff_bytes, h.code_bytes, h.scale_bytes};
  uint64_t prev_end = kHeaderBytes;
  for (int i = 0; i < 4; ++i) {
    if (offs[i] % kSectionAlign || offs[i] < prev_end || offs[i] > bytes || lens[i] > bytes - offs[i]) return bad("section bounds");
    prev_end = offs[i] + lens[i];
  }
  const uint8_t* base = (const uint8_t*)blob;
  const uint32_t* slot = (const uint32_t*)(base + h.off_dict);
  const uint32_t* uoff = (const uint32_t*)(base + h.off_uoff);
  const uint16_t* codes = (const uint16_t*)(base + h.off_codes);

  // Dictionary: codes 0..255 are the single bytes; the code space is sorted by run length (class_end), an entry's word
  // holds exactly as many bytes as its place says (zero above them); the pad entry is all zero; the entries fit the
  // device's dictionary storage.  The kernels take a run's length from the code alone, never from the entry.
  if (h.class_end[0] != 256 || h.class_end[1] < h.class_end[0] || h.class_end[2] < h.class_end[1] || h.class_end[3] < h.class_end[2] ||
      h.class_end[3] != h.n_entries || h.class_end[h.lmax - 1] != h.n_entries)
    return bad("code space classes");
  if (h.lmax > 2 && (uint64_t)h.class_end[1] + 2ull * (h.n_entries - h.class_end[1]) > kUnitBudget) return bad("dictionary exceeds the unit budget");
  for (uint32_t e = 0; e < h.n_entries; ++e) {
    const uint32_t w = slot[e], len = run_length(h, e);
    if (len < 4 && w >> (8 * len)) return bad("dictionary entry has bytes past its length");
    if (e < 256 && w != e) return bad("codes 0..255 must be the single bytes");
  }
  if (slot[h.n_entries] != 0) return bad("pad entry");

  // Offsets.
  if (uoff[0] != 0 || uoff[n_units] != h.n_chunks) return bad("first/last unit offset");
  for (uint64_t u = 0; u < n_units; ++u)
    if (uoff[u + 1] <= uoff[u] || uoff[u + 1] > h.n_chunks) return bad("unit offsets");

  // Codes: in range, pads only at the end of a lane stream, every lane stream's runs sum to its segment's length.
  std::atomic<uint64_t> first_bad(UINT64_MAX), real_codes(0);
  std::atomic<uint32_t> overrun(0), spread(0);
  n_threads = std::max(1u, std::min(n_threads, 16u));
  n_threads = (unsigned)std::min<uint64_t>(n_threads, n_units);
  const uint32_t pad_advance = h.lmax > 2 ? 4u : 2u;   // columns a pad code moves a lane's activation index in the product kernel
  auto work = [&](uint64_t ub, uint64_t ue) {
    uint64_t real = 0;
    uint32_t over = 0, wide = 0;
    std::vector<uint32_t> reach_lo, reach_hi;   // per chunk count: least / greatest column reached by an unfinished lane
    for (uint64_t u = ub; u < ue && first_bad.load(std::memory_order_relaxed) == UINT64_MAX; ++u) {
      const uint32_t band = (uint32_t)(u / h.n_quads), quad = (uint32_t)(u % h.n_quads);
      const uint32_t steps = (uoff[u + 1] - uoff[u]) * kChunkCodes;
      const uint16_t* cb = codes + (uint64_t)uoff[u] * kChunkWords;
      bool ok = true;
      reach_lo.assign(steps / kChunkCodes, UINT32_MAX);
      reach_hi.assign(steps / kChunkCodes, 0);
      for (uint32_t l = 0; l < 64 && ok; ++l) {
        const uint32_t want = segment_len(h, band, quad, l);
        uint32_t sum = 0, pads = 0;
        for (uint32_t k = 0; k < steps; ++k) {
          const uint32_t c = cb[(uint64_t)(k / kChunkCodes) * kChunkWords + l * kChunkCodes + k % kChunkCodes];
          if (c > h.n_entries) { ok = false; break; }
          if (c == h.n_entries) { ++pads; continue; }
          if (pads) { ok = false; break; }   // a real code after a pad
          sum += run_length(h, c);
          if (k % kChunkCodes == kChunkCodes - 1 && sum < want) {   // a whole chunk taken, segment not complete
            reach_lo[k / kChunkCodes] = std::min(reach_lo[k / kChunkCodes], sum);
            reach_hi[k / kChunkCodes] = std::max(reach_hi[k / kChunkCodes], sum);
          }
        }
        if (sum != want) ok = false;
        real += steps - pads;
        over = std::max(over, want + pad_advance * pads);
      }
      for (size_t k = 0; ok && k < reach_lo.size(); ++k)
        if (reach_hi[k] > reach_lo[k] && reach_lo[k] != UINT32_MAX) wide = std::max(wide, reach_hi[k] - reach_lo[k]);
      if (!ok) {
        uint64_t cur = first_bad.load();
        while (u < cur && !first_bad.compare_exchange_weak(cur, u)) {}
      }
    }
    real_codes += real;
    uint32_t cur = overrun.load();
    while (over > cur && !overrun.compare_exchange_weak(cur, over)) {}
    cur = spread.load();
    while (wide > cur && !spread.compare_exchange_weak(cur, wide)) {}
  };
  if (n_threads <= 1) {
    work(0, n_units);
  } else {
    std::vector<std::thread> th;
    uint64_t per = (n_units + n_threads - 1) / n_threads;
    for (unsigned t = 0; t < n_threads; ++t) {
      uint64_t b = std::min(n_units, t * per), e = std::min(n_units, b + per);
      if (b < e) th.emplace_back(work, b, e);
    }
    for (auto& x : th) x.join();
  }
  if (first_bad.load() != UINT64_MAX) return bad("code stream of unit " + std::to_string(first_bad.load()));
  if (real_codes.load() != h.n_real_codes) return bad("count of non-padding codes");
  if (hdr_out) *hdr_out = h;
  if (facts_out) {
    facts_out->max_lane_reach = overrun.load();
    facts_out->max_lane_spread = spread.load();
  }
  return TQ_OK;
}

void fill_info(const Header& h, const BlobFacts& facts, tq_info* o) {
  std::memset(o, 0, sizeof *o);
  o->rows = h.rows;
  o->cols = h.packing ? 2 * h.cols : h.cols;
  o->packing = h.packing;
  o->seg_cols = h.seg_cols;
  o->n_panels = h.n_panels;
  o->n_entries = h.n_entries;
  o->lmax = h.lmax;
  o->n_units = h.n_units;
  o->n_codes = h.n_chunks * kChunkWords;
  o->n_real_codes = h.n_real_codes;
  o->dict_bytes = h.dict_bytes;
  o->offset_bytes = h.uoff_bytes;
  o->code_bytes = h.code_bytes;
  o->scale_bytes = h.scale_bytes;
  o->compressed_bytes = h.dict_bytes + h.uoff_bytes + h.code_bytes + h.scale_bytes;
  o->lane_spread = facts.max_lane_spread;
}

}  // namespace tq

extern "C" const char* tq_last_error_string(void) { return tq::g_err.c_str(); }

extern "C" int tq_validate_blob(const void* blob, size_t blob_bytes, tq_info* info) {
  tq::Header h;
  tq::BlobFacts facts;
  try {   // no C++ exception leaves the library
    unsigned hw = std::thread::hardware_concurrency();
    int rc = tq::validate_blob(blob, blob_bytes, &h, &facts, hw ? hw : 1);
    if (rc == TQ_OK && info) tq::fill_info(h, facts, info);
    return rc;
  } catch (const std::bad_alloc&) {
    tq::set_error("tq_validate_blob: out of host memory");
    return TQ_E_OOM;
  } catch (...) {
    tq::set_error("tq_validate_blob: unexpected internal error (could a thread not be started?)");
    return TQ_E_HIP;
  }
}
