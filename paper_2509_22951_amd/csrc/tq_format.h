// Container layout (version 3) shared by the host encoder, the validator and the device code of libtq.
// All integers little-endian; every section starts on a 256-byte boundary.
//
// The quantized matrix Q (int8, rows x cols, row-major) is cut into *segments*: seg_cols consecutive columns of one
// row (the last panel of a row may be shorter).  A *unit* is the 64 segments one wavefront decodes in lockstep:
// 16 consecutive rows (a band) x 4 consecutive column panels (a quad); lane l of the wavefront owns row
// 16*band + (l & 15), panel 4*quad + (l >> 4).  Units are ordered band-major, quad-minor.  Segments past the matrix
// edge are empty.  The LZW parse (paper Background "Compression") visits the segments in (unit, lane) order with one
// dictionary per matrix; a run never crosses a segment boundary, so every lane's code stream can be decoded
// independently of the others (per-tile stream offsets).
//
// Dictionary: entries 0..255 are the single bytes (code == byte); the code space is sorted by run length - all runs of
// 2 bytes, then those of 3, then those of 4 (class_end[k] = number of entries of at most k + 1 bytes) - so a code's
// place tells its length, and entries of equal length keep the order LZW created them in.  An entry's word holds its
// bytes, first byte lowest, unused bytes zero.  Storage on the device: one unit per entry of up to 2 bytes, two per
// longer entry (kUnitBudget units when runs may be longer than 2; at most TQ_MAX_ENTRIES_DEVICE entries otherwise).
//
// packing 1 (values of at most 4 bits): byte j of a row holds the values of columns 2j (bits 0..3) and 2j + 1 (bits 4..7)
// in 4-bit two's complement; rows, cols, seg_cols and everything below describe that byte matrix, half as wide as the
// weight matrix.
//
// Code section: for unit u the codes of its 64 lane streams are interleaved in chunks of 4 codes per lane:
//   code k of lane l of unit u  ->  codes[(uoff[u] + k / 4) * 256 + l * 4 + k % 4]
// Every lane stream of a unit is padded with pad codes (index n_entries, an empty entry) to the unit's length,
// which is the longest lane stream rounded up to a multiple of 4.  One chunk is 512 contiguous bytes: a wavefront
// reads it with one coalesced 8-byte load per lane.
#pragma once
#include <cstddef>
#include <cstdint>
#include <string>

struct tq_info;

namespace tq {

constexpr uint32_t kUnitRows = 16;      // rows of a unit (lanes l & 15)
constexpr uint32_t kUnitPanels = 4;     // column panels of a unit (lanes l >> 4)
constexpr uint32_t kChunkCodes = 4;     // codes per lane and chunk (one 8-byte load)
constexpr uint32_t kChunkWords = 64 * kChunkCodes;   // 16-bit codes per chunk
constexpr uint32_t kMinSegCols = 16, kMaxSegCols = 1024, kDefaultSegCols = 256;
constexpr uint32_t kSectionAlign = 256;
constexpr uint32_t kHeaderBytes = 256;
constexpr uint32_t kVersion = 3;
constexpr char kMagic[8] = {'T', 'Q', 'M', 'O', 'E', 'v', '3', '\0'};
constexpr uint32_t kUnitBudget = 30716;   // units a dictionary with runs of 3 or 4 bytes may take (four more hold its pad entry and alignment)

#pragma pack(push, 1)
struct Header {
  char magic[8];
  uint32_t version, header_bytes;
  uint32_t rows, cols;
  uint32_t seg_cols;                      // columns per segment (multiple of 16)
  uint32_t unit_rows, unit_panels, chunk_codes;
  uint32_t n_bands, n_panels, n_quads;    // ceil(rows / 16), ceil(cols / seg_cols), ceil(n_panels / 4)
  uint32_t n_entries, lmax, max_entries, pad_code;
  uint32_t packing;                       // 0: one value per byte; 1: two 4-bit values per byte (the matrix has 2 * cols columns)
  uint64_t n_units, n_chunks;             // n_bands * n_quads; total chunks of the code section
  uint64_t n_real_codes;                  // codes that are not padding
  uint64_t off_dict, dict_bytes;          // uint32 slot[n_entries + 1]: the run's bytes, first byte lowest, unused bytes zero
  uint64_t off_uoff, uoff_bytes;          // uint32 uoff[n_units + 1], in chunks
  uint64_t off_codes, code_bytes;         // uint16 codes[n_chunks * 256]
  uint64_t off_scales, scale_bytes;       // float scale[n_bands * 16]
  uint64_t total_bytes;
  uint32_t class_end[4];                  // entries of at most 1, 2, 3, 4 bytes: 256 <= .. <= n_entries; [lmax - 1] == n_entries
  uint8_t zero[kHeaderBytes - 184];
};
#pragma pack(pop)
static_assert(sizeof(Header) == kHeaderBytes, "header size");

inline uint64_t round_up(uint64_t v, uint64_t a) { return (v + a - 1) / a * a; }

// Run length of a code by its place in the sorted code space (the pad code, n_entries, counts as the longest class).
inline uint32_t run_length(const Header& h, uint32_t code) {
  return 1u + (code >= h.class_end[0]) + (code >= h.class_end[1]) + (code >= h.class_end[2]);
}

// Length in bytes of the segment lane `lane` of unit (band, quad) owns.
inline uint32_t segment_len(const Header& h, uint32_t band, uint32_t quad, uint32_t lane) {
  const uint32_t row = band * kUnitRows + (lane & 15), panel = quad * kUnitPanels + (lane >> 4);
  if (row >= h.rows || panel >= h.n_panels) return 0;
  const uint32_t c0 = panel * h.seg_cols;
  return c0 + h.seg_cols <= h.cols ? h.seg_cols : h.cols - c0;
}

void set_error(const std::string& msg);   // thread-local last-error text

// What validation learns about a container beyond the header.
struct BlobFacts {
  uint32_t max_lane_reach;   // largest (segment length + 2 * pad codes) of any lane stream: how many columns past the start
                             // of its segment a lane's activation index can get when every pad code advances it by two
                             // (by four in containers whose runs may be longer than 2: what the pad code's place says)
  uint32_t max_lane_spread;  // the 64 lanes of a unit take their chunks in step; after any number of chunks, the lanes whose
                             // segment is not yet complete have reached different columns of it: the largest difference
                             // between two of them, over all units and all chunk counts
};

// Host-side structural validation; fills *hdr_out with a copy of the header on success.
int validate_blob(const void* blob, size_t bytes, Header* hdr_out, BlobFacts* facts_out, unsigned n_threads);
void fill_info(const Header& h, const BlobFacts& facts, ::tq_info* out);

}  // namespace tq
