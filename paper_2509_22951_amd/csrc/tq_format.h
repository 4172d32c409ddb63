// Container layout shared by the host encoder, the validator and the device code of libtq.
// All integers little-endian; every section starts on a 256-byte boundary.
#pragma once
#include <cstddef>
#include <cstdint>
#include <string>

struct tq_info;

namespace tq {

constexpr uint32_t kTileRows = 16;      // rows of a micro-tile (= M of the 16x16x32 MFMA)
constexpr uint32_t kMtCols = 8;         // columns of a micro-tile (= the 8 k-values one lane feeds the MFMA)
constexpr uint32_t kGroupCols = 256;    // columns of a restart group: 32 micro-tiles, 8 MFMA steps
constexpr uint32_t kGroupBytes = kTileRows * kGroupCols;
constexpr uint32_t kCodeAlign = 8;      // codes per 16-byte lane load; each group's run is padded to this
constexpr uint32_t kSectionAlign = 256;
constexpr uint32_t kHeaderBytes = 256;
constexpr uint32_t kVersion = 1;
constexpr char kMagic[8] = {'T', 'Q', 'M', 'O', 'E', 'v', '1', '\0'};

#pragma pack(push, 1)
struct Header {
  char magic[8];
  uint32_t version, header_bytes;
  uint32_t rows, cols;
  uint32_t rows_pad, cols_pad;
  uint32_t tile_rows, mt_cols, group_cols, group_bytes;
  uint32_t n_entries, lmax, max_entries, pad_code;
  uint64_t n_groups, n_codes;
  uint64_t off_dict, dict_bytes;      // uint32 slot[n_entries + 1]: run bytes in bits 0..23, run length in BITS (8/16/24) in bits 24..31
  uint64_t off_goff, goff_bytes;      // uint32 goff[n_groups + 1], in codes
  uint64_t off_codes, code_bytes;     // uint16 codes[n_codes]
  uint64_t off_scales, scale_bytes;   // float scale[rows_pad]
  uint64_t total_bytes;
  uint32_t code_align;
  uint8_t zero[kHeaderBytes - 156];
};
#pragma pack(pop)
static_assert(sizeof(Header) == kHeaderBytes, "header size");

inline uint64_t round_up(uint64_t v, uint64_t a) { return (v + a - 1) / a * a; }

void set_error(const std::string& msg);   // thread-local last-error text

// Host-side structural validation; fills *hdr_out with a copy of the header on success.
int validate_blob(const void* blob, size_t bytes, Header* hdr_out, unsigned n_threads);
void fill_info(const Header& h, ::tq_info* out);

}  // namespace tq
