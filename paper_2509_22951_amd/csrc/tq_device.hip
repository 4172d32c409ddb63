// Device side of libtq for gfx950 (MI355X): handle management and the hot-path kernels.
//
// Work decomposition.  The container stores the matrix as lane streams: a unit is 16 rows x 4 column panels, one
// (row, panel) segment per lane of a wavefront, and the 16-bit codes of the 64 segments are interleaved in chunks of
// 4 codes per lane.  A wavefront therefore reads one coalesced 512-byte chunk per step and every lane decodes its own
// segment, in lockstep with the others, with no cross-lane dependency:
//   1. code -> dictionary word by an LDS lookup (the dictionary is staged once per workgroup; for the product it is
//      held as two bf16 weights per entry, the second one zero for single-byte entries),
//   2. the lane's column position advances by the run length, which is 1 + (code >= 256) for runs of at most 2,
//   3. tq_matvec gathers the activation pair (x[col], x[col+1]) from an LDS image of x and issues one
//      v_dot2_f32_bf16 per code; the per-lane sums of the 4 panels of a row are added at the end of a band of 16
//      rows, multiplied by the row scale and stored,
//      (two activation rows are handled the same way, with both rows in the image and one dot product per row;
//      packed 4-bit weights: four weights per entry as fp8, two conversions and two dot products per code and row),
//   4. for batches of 3..16 rows and for tq_decompress the lanes append their run bytes to per-lane storage in LDS
//      instead - a ring of 128 bytes (k_matvec_ring: multiplied by bf16 MFMA, batch = N, while the decode goes on) or
//      a strip holding the whole segment (k_matvec_mfma: multiplied when the unit is complete; k_decompress: copied
//      out row-major).
// The expanded matrix never exists in HBM on the tq_matvec path.
// Containers of packed 4-bit weights (two per stored byte) take the same decode; what changes is the dequantization:
// four fp8 weights per dictionary word and two dot products per code at batch 1, nibbles expanded to bf16 ahead of the
// MFMA in the batched kernels, nibbles expanded to int8 in the copy-out of tq_decompress.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <thread>
#include <utility>
#include <vector>

#include "../../include/tq.h"
#include "tq_format.h"
#include "tq_kernels_common.h"
#include "tq_kernel_dot.h"
#include "tq_strip_decode.h"
#include "tq_kernel_ring.h"
#include "tq_kernel_strip.h"

using namespace tq;

// Job table of tq_matvec_multi_static: device memory that belongs to the library image, so that the call needs no
// allocation.  Every GPU the library runs on holds its own copy at its own address (looked up once per device, see
// static_table_of); all calls on a GPU share it.
constexpr size_t kStaticTableBytes = (size_t)kMaxStep * sizeof(StepEntry);
static __device__ __align__(256) unsigned char scratch[kStaticTableBytes];

namespace {

// What the table writer needs per job: where the matrix description lives in device memory, and the buffers.
struct JobRef {
  const DevMat* m;
  const uint16_t* x;
  float* y;
};
constexpr int kWriterJobs = 160;   // per launch of the writer (its arguments stay below 4 KB)
struct TableWrite {
  StepEntry* table;   // first entry to write
  int n;
  JobRef j[kWriterJobs];
};
static_assert(sizeof(TableWrite) <= 4096, "kernel arguments");

// The stage counters of a staged step start every launch at zero (a fill kernel, not a memset node: the launch may be
// captured in a HIP graph).
__global__ __launch_bounds__(256) void k_zero_words(uint32_t* p, uint32_t n) {
  for (uint32_t i = threadIdx.x; i < n; i += 256) p[i] = 0u;
}

// Entry t of the table = (description of job t copied from device memory, x, y).  One thread per dword of an entry.
__global__ __launch_bounds__(64) void k_write_table(TableWrite w) {
  constexpr int kDescDwords = sizeof(DevMat) / 4;
  const int t = blockIdx.x, k = threadIdx.x;
  if (t >= w.n) return;
  uint32_t* dst = (uint32_t*)(w.table + t);
  static_assert(offsetof(StepEntry, m) == 0 && sizeof(StepEntry) == sizeof(DevMat) + 16 && sizeof(DevMat) % 8 == 0, "entry layout");
  if (k < kDescDwords) {
    dst[k] = ((const uint32_t*)w.j[t].m)[k];
  } else if (k < kDescDwords + 4) {
    const uint64_t px = (uint64_t)w.j[t].x, py = (uint64_t)w.j[t].y;
    const uint32_t tail[4] = {(uint32_t)px, (uint32_t)(px >> 32), (uint32_t)py, (uint32_t)(py >> 32)};
    dst[k] = tail[k - kDescDwords];
  }
}

int hip_fail(const char* what, hipError_t e) {
  set_error(std::string(what) + ": " + hipGetErrorString(e));
  return TQ_E_HIP;
}

// Device copies of dictionaries, shared by every matrix whose container holds the same dictionary bytes (matrices
// encoded one after the other with dict_from do once the dictionary is full).  The kernels compare pointers to see
// that the dictionary staged in LDS is still the right one.
struct DictCopy {
  int device;
  std::vector<uint32_t> words;   // host copy for the comparison
  uint32_t* dev;        // container words
  uint32_t* dev_bf16;   // (bf16(b0), bf16(b1)) per entry; a single-byte entry has a zero second weight, the pad entry two.
                        // Packed 4-bit weights: the four nibbles of (b0, b1) as fp8 e4m3, in column order.
  uint32_t packing;
  uint32_t long_runs, class2, class3;   // containers with runs of 3 and 4 bytes: dev and dev_bf16 are slot images (long_slot)
  uint32_t image_bytes;                 // long_runs: size of the byte image at dev
  uint32_t dict_words_bf16;             // dwords of the image at dev_bf16 (a multiple of 4)
  int refs;
};

// int8 -> bf16 bit pattern (exact: |v| <= 128 needs 8 significant bits); bf16 = upper half of the fp32 encoding.
uint32_t i8_to_bf16_bits(uint32_t byte) {
  const float f = (float)(int8_t)byte;
  uint32_t u;
  std::memcpy(&u, &f, 4);
  return u >> 16;
}
// 4-bit two's complement -> fp8 e4m3 (1 sign, 4 exponent bits with bias 7, 3 mantissa bits): -8..7 are all exact.
uint32_t nibble_to_fp8_bits(uint32_t nibble) {
  const int v = (int)(nibble & 7u) - (int)(nibble & 8u);
  const uint32_t mag = (uint32_t)(v < 0 ? -v : v), sign = v < 0 ? 0x80u : 0u;
  if (mag == 0) return 0;
  uint32_t e = 0;
  while ((mag >> (e + 1)) != 0) ++e;                       // mag = 2^e * (1 + mantissa / 8)
  const uint32_t mant = ((mag << 3) >> e) & 7u;
  return sign | (e + 7) << 3 | mant;
}
std::mutex g_dict_mutex;
std::vector<DictCopy*> g_dicts;

// words: the container's dictionary section (n_words = entries + the pad entry).  hdr tells the code space classes.
int acquire_dictionary(int device, const uint32_t* words, uint32_t n_words, const Header& hdr, DictCopy** out) {
  const uint32_t packing = hdr.packing, long_runs = hdr.lmax > 2 ? 1u : 0u, class2 = hdr.class_end[1], class3 = hdr.class_end[2];
  std::lock_guard<std::mutex> lock(g_dict_mutex);
  for (DictCopy* d : g_dicts)
    if (d->device == device && d->packing == packing && d->long_runs == long_runs && d->class2 == class2 && d->class3 == class3 &&
        d->words.size() == n_words && std::memcmp(d->words.data(), words, (size_t)n_words * 4) == 0) {
      ++d->refs;
      *out = d;
      return TQ_OK;
    }
  DictCopy* d = new (std::nothrow) DictCopy;
  if (!d) {
    set_error("out of host memory");
    return TQ_E_OOM;
  }
  d->device = device;
  d->words.assign(words, words + n_words);
  d->refs = 1;
  d->packing = packing;
  d->long_runs = long_runs;
  d->class2 = class2;
  d->class3 = class3;
  d->image_bytes = 0;
  d->dev = d->dev_bf16 = nullptr;
  // bytes past an entry's length are zero in the container, so the conversions need no length test
  std::vector<uint32_t> first, second;   // what dev and dev_bf16 will hold
  if (!long_runs) {
    // dev: the container words (the kernels take the low 16 bits); dev_bf16: one dword per entry
    const uint32_t n_pad = (uint32_t)round_up(n_words, 4);
    first.assign(n_pad, 0u);
    second.assign(n_pad, 0u);
    for (uint32_t i = 0; i < n_words; ++i) {
      first[i] = words[i];
      if (packing) {
        for (uint32_t k = 0; k < 4; ++k) second[i] |= nibble_to_fp8_bits(words[i] >> (4 * k) & 15u) << (8 * k);
      } else {
        second[i] = i8_to_bf16_bits(words[i] & 0xFFu) | i8_to_bf16_bits(words[i] >> 8 & 0xFFu) << 16;
      }
    }
  } else {
    // Slot images: entry e sits at slot e + max(e - even(class2), 0); an entry below class2 takes one slot, the others
    // (the pad entry among them) two, starting on an even slot.  dev: 2 bytes per slot (the run's bytes as they are);
    // dev_bf16: one dword per slot (two bf16 weights).
    const uint32_t even = class2 & ~1u;
    auto slot_of = [&](uint32_t e) { return e + (e > even ? e - even : 0u); };
    const uint32_t n_slots = slot_of(n_words - 1) + 2;
    std::vector<uint16_t> bytes_img(round_up(n_slots, 8), 0);
    second.assign(round_up(n_slots, 4), 0u);
    for (uint32_t e = 0; e < n_words; ++e) {
      const uint32_t s0 = slot_of(e), w = words[e];
      bytes_img[s0] = (uint16_t)w;
      second[s0] = i8_to_bf16_bits(w & 0xFFu) | i8_to_bf16_bits(w >> 8 & 0xFFu) << 16;
      if (e >= class2) {
        bytes_img[s0 + 1] = (uint16_t)(w >> 16);
        second[s0 + 1] = i8_to_bf16_bits(w >> 16 & 0xFFu) | i8_to_bf16_bits(w >> 24) << 16;
      }
    }
    first.assign(bytes_img.size() / 2, 0u);
    std::memcpy(first.data(), bytes_img.data(), bytes_img.size() * 2);
    d->image_bytes = (uint32_t)(bytes_img.size() * 2);
  }
  hipError_t e = hipMalloc((void**)&d->dev, first.size() * 4);
  if (e == hipSuccess) e = hipMalloc((void**)&d->dev_bf16, second.size() * 4);
  if (e == hipSuccess) e = hipMemcpy(d->dev, first.data(), first.size() * 4, hipMemcpyHostToDevice);
  if (e == hipSuccess) e = hipMemcpy(d->dev_bf16, second.data(), second.size() * 4, hipMemcpyHostToDevice);
  if (e != hipSuccess) {
    if (d->dev) (void)hipFree(d->dev);
    if (d->dev_bf16) (void)hipFree(d->dev_bf16);
    delete d;
    return hip_fail("dictionary upload", e);
  }
  d->dict_words_bf16 = (uint32_t)second.size();
  g_dicts.push_back(d);
  *out = d;
  return TQ_OK;
}

hipError_t release_dictionary(DictCopy* d) {
  std::lock_guard<std::mutex> lock(g_dict_mutex);
  if (--d->refs > 0) return hipSuccess;
  g_dicts.erase(std::find(g_dicts.begin(), g_dicts.end(), d));
  hipError_t e = hipFree(d->dev);
  hipError_t e2 = hipFree(d->dev_bf16);
  delete d;
  return e != hipSuccess ? e : e2;
}

constexpr uint32_t kSlotBytes = 2 * kDotWavesMax * 2 * 16 * 4 + 2 * kDotWavesMax * 4;   // (two activation rows at most)

// LDS plan of the product kernel for a set of matrices: dictionary | activation image | partial-sum slots.
bool plan_matvec_lds(uint32_t dict_words_max, uint32_t x_dwords_max, uint32_t* x_off, uint32_t* slot_off, size_t* total) {
  *x_off = (uint32_t)round_up((uint64_t)dict_words_max * 4, 16);
  *slot_off = (uint32_t)round_up((uint64_t)*x_off + (uint64_t)x_dwords_max * 4, 16);
  *total = (size_t)*slot_off + kSlotBytes;
  return *total <= kLdsLimit;
}

// Whether the dot-product kernel takes a product: one activation row, two rows of one-weight-per-byte matrices (same
// image size), or two rows of packed matrices (the image is twice as large there) - and in every case only if the
// image fits the LDS beside the dictionary.  Everything else goes to the batched kernels.
bool dot_kernel_takes(int batch, bool packed, bool long_runs, uint32_t dict_words_max, uint32_t x_dwords_max) {
  if (batch > 2) return false;
  if (long_runs && (batch != 1 || packed)) return false;   // runs of 3 and 4 bytes: the dot-product kernel has a one-row form only
  uint32_t x_off, slot_off;
  size_t total;
  return plan_matvec_lds(dict_words_max, (batch == 2 && packed ? 2u : 1u) * x_dwords_max, &x_off, &slot_off, &total);
}

// Address of `scratch` on each device.  In host code the array's name is only a handle for the runtime: the address a
// kernel can use comes from hipGetSymbolAddress, asked once per device with that device current.
constexpr int kMaxDevices = 64;
std::mutex g_static_mutex;
StepEntry* g_static_table[kMaxDevices];   // null until looked up
int static_table_of(int device, StepEntry** out) {   // `device` is the current device
  if (device < 0 || device >= kMaxDevices) {
    set_error("device index " + std::to_string(device) + " is beyond what the library keeps a static table for");
    return TQ_E_UNSUPPORTED;
  }
  std::lock_guard<std::mutex> lock(g_static_mutex);
  if (!g_static_table[device]) {
    void* p = nullptr;
    hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) return hip_fail("hipGetSymbolAddress(static job table)", e);
    g_static_table[device] = (StepEntry*)p;
  }
  *out = g_static_table[device];
  return TQ_OK;
}

// Every kernel of the library that takes its dictionary at LDS address 0.
const void* const kLdsKernels[] = {
    (const void*)k_matvec<kDotPiece, kDotWaves, false, 1>,
    (const void*)k_matvec<kDotPiece, kDotWaves, false, 2>,
    (const void*)k_matvec<kDotPiecePacked, kDotWavesPacked, true, 1>,
    (const void*)k_matvec<kDotPiecePacked, kDotWavesPacked, true, 2>,
    (const void*)k_matvec<kDotPiece, kDotWaves, false, 1, true>,
    (const void*)k_matvec<kDotPiece, kDotWavesStaged, false, 1, false, true>,
    (const void*)k_matvec<kDotPiece, kDotWavesStaged, false, 2, false, true>,
    (const void*)k_matvec<kDotPiecePacked, kDotWavesPacked, true, 1, false, true>,
    (const void*)k_matvec<kDotPiecePacked, kDotWavesPacked, true, 2, false, true>,
    (const void*)k_decompress<false>,
    (const void*)k_decompress<true>,
    (const void*)k_matvec_mfma<true, false>,
    (const void*)k_matvec_mfma<false, false>,
    (const void*)k_matvec_mfma<true, true>,
    (const void*)k_matvec_mfma<false, true>,
    (const void*)k_matvec_mfma<true, false, true>,
    (const void*)k_matvec_mfma<false, false, true>,
    (const void*)k_matvec_mfma<true, true, true>,
    (const void*)k_matvec_mfma<false, true, true>,
    (const void*)k_matvec_ring<kRingWaves, 16, false>,
    (const void*)k_matvec_ring<kRingWavesHalf, 8, false>,
    (const void*)k_matvec_ring<kRingWaves, 16, true>,
    (const void*)k_matvec_ring<kRingWavesHalf, 8, true>,
    (const void*)k_matvec_ring<kRingWavesMore, 8, false>,
    (const void*)k_matvec_ring<kRingWavesMore, 8, true>,
    (const void*)k_matvec_ring<kRingWavesQuarter, 4, false>,
    (const void*)k_matvec_ring<kRingWavesQuarter, 4, true>,
};

// Once per matrix creation (cheap): dynamic LDS above 64 KB has to be allowed per kernel function, and the kernels'
// code -> entry lookup takes the dictionary to start at LDS address 0, which holds exactly when a kernel has no
// statically allocated LDS ahead of its dynamic segment.  That is checked here, on the host, so that no launch can
// run with a dictionary somewhere else.
int prepare_kernels() {
  for (const void* k : kLdsKernels) {
    hipFuncAttributes attr;
    hipError_t e = hipFuncGetAttributes(&attr, k);
    if (e != hipSuccess) return hip_fail("hipFuncGetAttributes", e);
    if (attr.sharedSizeBytes != 0) {
      set_error("internal: a kernel was built with static LDS, so its dictionary would not start at LDS address 0");
      return TQ_E_UNSUPPORTED;
    }
    e = hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsLimit);
    if (e != hipSuccess) return hip_fail("hipFuncSetAttribute(MaxDynamicSharedMemorySize)", e);
  }
  return TQ_OK;
}

// Runs the body of an entry point; no C++ exception leaves the library.
template <typename F>
int guarded(const char* who, F&& body) {
  try {
    return body();
  } catch (const std::bad_alloc&) {
    set_error(std::string(who) + ": out of host memory");
    return TQ_E_OOM;
  } catch (...) {
    set_error(std::string(who) + ": unexpected internal error");
    return TQ_E_HIP;
  }
}

}  // namespace

struct tq_matrix {
  Header h;
  BlobFacts facts;
  DevMat m;
  const DevMat* m_dev;   // the same description in device memory, for launches that serve many matrices
  DictCopy* dict;
  void* dev_base;
  uint32_t lds_dict16;   // bytes of LDS the byte image of the dictionary takes in the strip and ring kernels
  int device;
  int n_cu;
};

static int tq_create_from_encoded_impl(const void* blob, size_t blob_bytes, tq_handle* out) {
  if (!out) {
    set_error("tq_create_from_encoded: null output pointer");
    return TQ_E_INVALID_ARG;
  }
  *out = nullptr;
  Header h;
  BlobFacts facts;
  unsigned hw = std::thread::hardware_concurrency();
  if (int rc = validate_blob(blob, blob_bytes, &h, &facts, hw ? hw : 1)) return rc;

  DevMat m;
  std::memset(&m, 0, sizeof m);
  m.rows = h.rows;
  m.cols = h.cols;
  m.seg_cols = h.seg_cols;
  m.n_bands = h.n_bands;
  m.n_quads = h.n_quads;
  const bool long_runs = h.lmax > 2;
  m.dict_words = (uint32_t)round_up(h.n_entries + 1, 4);   // (containers with runs of 3 and 4 bytes: set below, from the slot image)
  // Panels of one unit are seg_cols columns apart; a gap of 16 dwords after every panel keeps their activation reads
  // on different LDS banks when seg_cols is a multiple of 32.
  m.x_span = h.seg_cols + (h.seg_cols % 32 == 0 ? 16u : 0u);
  m.seg_magic = (uint32_t)((1ull << 32) / h.seg_cols) + 1;   // exact quotient while col * seg_cols < 2^32
  m.reserved = long_runs ? 0u : facts.max_lane_spread <= kRingSpread ? 1u : facts.max_lane_spread <= kRingSpreadCareful ? 2u : 0u;
  m.packing = h.packing;
  m.long_runs = long_runs ? 1u : 0u;
  m.class2 = h.class_end[1];
  m.class3 = h.class_end[2];
  if (h.cols > (1u << 20)) {
    set_error("more than 2^20 columns are not supported");
    return TQ_E_UNSUPPORTED;
  }
  const uint64_t n_slots = (uint64_t)h.n_quads * kUnitPanels;
  // (a code of a long-run container also reads the activation pair two columns further on, against weights that are
  // zero when its run is shorter: two more dwords behind the furthest column a lane reaches)
  m.x_dwords = (uint32_t)((n_slots - 1) * m.x_span + std::max<uint64_t>(m.x_span + (long_runs ? 2u : 0u), (uint64_t)facts.max_lane_reach + (long_runs ? 3u : 1u)));
  // (A row whose activation image does not fit the LDS beside the dictionary is not refused: its products run on the
  // batched kernels, which take their activations from global memory or a tile of one quad, at any batch.)
  // tq_decompress and the batched product: byte image of the dictionary (2 bytes per slot, at most 30,720 slots) plus one
  // tile of 64 strips per wavefront.
  if (round_up((uint64_t)(long_runs ? 30720u : m.dict_words) * 2, 16) + (size_t)64 * (h.seg_cols + 8) > kLdsLimit) {
    set_error("segments of " + std::to_string(h.seg_cols) + " columns do not fit the LDS tile");
    return TQ_E_UNSUPPORTED;
  }

  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_fail("hipGetDevice (is a GPU present?)", e);
  hipDeviceProp_t prop;
  e = hipGetDeviceProperties(&prop, dev);
  if (e != hipSuccess) return hip_fail("hipGetDeviceProperties", e);
  if (prop.sharedMemPerBlock < kLdsLimit && (size_t)prop.maxSharedMemoryPerMultiProcessor < kLdsLimit) {
    set_error("device offers less LDS per workgroup than this library needs (built for gfx950, 160 KB)");
    return TQ_E_UNSUPPORTED;
  }
  if (int rc = prepare_kernels()) return rc;
  {
    StepEntry* table = nullptr;   // the static job table of this device, for tq_matvec_multi_static
    if (int rc = static_table_of(dev, &table)) return rc;
  }

  const uint8_t* src = (const uint8_t*)blob;
  DictCopy* dict = nullptr;
  if (int rc = acquire_dictionary(dev, (const uint32_t*)(src + h.off_dict), h.n_entries + 1, h, &dict)) return rc;
  if (long_runs) {
    m.dict_words = dict->dict_words_bf16;
    m.dict16_bytes = dict->image_bytes;
  }

  const uint64_t sz_uoff = round_up(h.uoff_bytes, kSectionAlign), sz_codes = round_up(h.code_bytes, kSectionAlign),
                 sz_scales = round_up(h.scale_bytes, kSectionAlign);
  const uint64_t o_uoff = 0, o_codes = o_uoff + sz_uoff, o_scales = o_codes + sz_codes, o_desc = o_scales + sz_scales,
                 total = o_desc + round_up(sizeof(DevMat), kSectionAlign);
  uint8_t* base = nullptr;
  e = hipMalloc((void**)&base, total);
  if (e != hipSuccess) {
    (void)release_dictionary(dict);
    set_error(std::string("hipMalloc of ") + std::to_string(total) + " bytes: " + hipGetErrorString(e));
    return e == hipErrorOutOfMemory ? TQ_E_OOM : TQ_E_HIP;
  }
  e = hipMemcpy(base + o_uoff, src + h.off_uoff, h.uoff_bytes, hipMemcpyHostToDevice);
  if (e == hipSuccess) e = hipMemcpy(base + o_codes, src + h.off_codes, h.code_bytes, hipMemcpyHostToDevice);
  if (e == hipSuccess) e = hipMemcpy(base + o_scales, src + h.off_scales, h.scale_bytes, hipMemcpyHostToDevice);
  m.dict = dict->dev;
  m.dict_bf16 = dict->dev_bf16;
  m.uoff = (const uint32_t*)(base + o_uoff);
  m.codes = (const uint2*)(base + o_codes);
  m.scales = (const float*)(base + o_scales);
  if (e == hipSuccess) e = hipMemcpy(base + o_desc, &m, sizeof m, hipMemcpyHostToDevice);
  if (e == hipSuccess) e = hipDeviceSynchronize();
  tq_matrix* t = e == hipSuccess ? new (std::nothrow) tq_matrix : nullptr;
  if (!t) {
    (void)hipFree(base);
    (void)release_dictionary(dict);
    if (e != hipSuccess) return hip_fail("upload", e);
    set_error("out of host memory");
    return TQ_E_OOM;
  }
  t->h = h;
  t->facts = facts;
  t->m = m;
  t->m_dev = (const DevMat*)(base + o_desc);
  t->dict = dict;
  t->dev_base = base;
  t->lds_dict16 = long_runs ? dict->image_bytes : (uint32_t)round_up((uint64_t)m.dict_words * 2, 16);
  t->device = dev;
  t->n_cu = prop.multiProcessorCount;
  *out = t;
  return TQ_OK;
}

namespace {

enum class Op { kMatvec, kDecompress };

// A kernel launch with everything but the stream decided.
struct PreparedLaunch {
  MatvecArgs a;
  const void* kernel;
  unsigned grid, block;
  size_t lds;
  size_t table_first;   // prepared steps: index of the launch's first job in the step's table
  const char* what;
};

// Launches recorded for a prepared step instead of being started, and the jobs they will read from device memory.
struct Recorder {
  std::vector<PreparedLaunch> launches;
  std::vector<StepEntry> entries;
  std::vector<JobRef> refs;   // the same jobs by the device address of their description (for the table writer)
};

int fire(const PreparedLaunch& p, hipStream_t stream) {
  MatvecArgs a = p.a;
  void* args[] = {&a};
  hipError_t e = hipLaunchKernel(p.kernel, dim3(p.grid), dim3(p.block), args, p.lds, stream);
  if (e == hipSuccess) e = hipGetLastError();
  if (e != hipSuccess) return hip_fail(p.what, e);
  return TQ_OK;
}

// One kernel launch for hs[0..n), all on one device, total cost below 2^32; n <= kMaxMulti, or n <= kMaxStep when the
// launch is recorded for a prepared step (rec: its jobs then go to the step's device table, not into the arguments).
// kMatvec: xs/ys are the activations and outputs; kDecompress: ys are the int8 output matrices, xs is not used.
// ring: the batched product with a ring per lane (every matrix of the call has passed ring_eligible).
int launch(Op op, int n, const tq_handle* hs, const void* const* xs, void* const* ys, int batch, hipStream_t stream, bool ring = false,
           bool gate_up = false, Recorder* rec = nullptr) {
  PreparedLaunch p;
  MatvecArgs& a = p.a;
  std::memset(&a, 0, sizeof a);
  a.n = n;
  a.batch = batch;
  a.tile_area = 0;
  a.gate_up = gate_up ? 1u : 0u;
  p.table_first = rec ? rec->entries.size() : 0;
  p.what = op == Op::kDecompress ? "tq_decompress launch" : "tq_matvec launch";
  a.table = rec ? (const StepEntry*)(uintptr_t)8 : nullptr;   // (the address follows when the step's table is in device memory)
  uint32_t dict_words_max = 0, x_dwords_max = 0, seg_max = 0, dict16_max = 0;
  uint64_t cost = 0, bands = 0, band_cost_max = 1;
  bool x_fast = true;
  for (int i = 0; i < n; ++i) {
    const tq_matrix* t = hs[i];
    if (rec) {
      rec->entries.push_back(StepEntry{t->m, xs ? (const uint16_t*)xs[i] : nullptr, (float*)ys[i]});
      rec->refs.push_back(JobRef{t->m_dev, xs ? (const uint16_t*)xs[i] : nullptr, (float*)ys[i]});
    } else {
      a.u.in.j[i].m = t->m_dev;
      if (i < kInlineDescriptions) a.u.in.first[i] = t->m;
      a.u.in.j[i].x = xs ? (const uint16_t*)xs[i] : nullptr;
      a.u.in.j[i].y = (float*)ys[i];
    }
    a.u.cost_long[i] = (uint32_t)cost;
    cost += (uint64_t)t->m.n_bands * t->m.cols;   // a band costs its 16 x cols weights, counted in units of 16
    bands += t->m.n_bands;
    band_cost_max = std::max<uint64_t>(band_cost_max, t->m.cols);
    dict_words_max = std::max(dict_words_max, t->m.dict_words);
    dict16_max = std::max(dict16_max, t->lds_dict16);
    x_dwords_max = std::max(x_dwords_max, t->m.x_dwords);
    seg_max = std::max(seg_max, t->m.seg_cols);
    x_fast = x_fast && (t->m.packing ? 2 : 1) * t->m.cols % 8 == 0 && xs && (uintptr_t)xs[i] % 16 == 0;
  }
  a.u.cost_long[n] = (uint32_t)cost;
  if (cost > 0xFFFFFFFFull) {
    set_error("more than 2^36 weights in one launch are not supported");
    return TQ_E_UNSUPPORTED;
  }
  // Every workgroup's share of the cost line is at least one band of the most expensive kind, and there is one
  // workgroup per CU at most.
  p.grid = (unsigned)std::max<uint64_t>(1, std::min<uint64_t>({(uint64_t)hs[0]->n_cu, bands, cost / band_cost_max}));
  const bool packed = hs[0]->m.packing != 0;   // (all matrices of a product launch hold their weights the same way: launch_all sees to that)
  const bool long_runs = hs[0]->m.long_runs != 0;   // (likewise)
  if (op == Op::kMatvec && dot_kernel_takes(batch, packed, long_runs, dict_words_max, x_dwords_max)) {
    // the dot-product kernel: one activation row or two
    if (!plan_matvec_lds(dict_words_max, (packed && batch == 2 ? 2 : 1) * x_dwords_max, &a.x_off, &a.slot_off, &p.lds)) {
      set_error("the matrices of this call together need " + std::to_string(p.lds) + " bytes of LDS (largest dictionary plus longest row)");
      return TQ_E_UNSUPPORTED;
    }
    p.kernel = long_runs ? (const void*)k_matvec<kDotPiece, kDotWaves, false, 1, true>
               : packed ? (batch == 2 ? (const void*)k_matvec<kDotPiecePacked, kDotWavesPacked, true, 2> : (const void*)k_matvec<kDotPiecePacked, kDotWavesPacked, true, 1>)
               : batch == 2 ? (const void*)k_matvec<kDotPiece, kDotWaves, false, 2> : (const void*)k_matvec<kDotPiece, kDotWaves, false, 1>;
    p.block = (packed ? kDotWavesPacked : kDotWaves) * 64;
  } else if (ring) {
    // LDS: 16-bit dictionary image | one ring per lane (aligned to its size: the kernel ORs piece offsets into its
    // address) | the activation tile of one quad.
    const size_t dict16 = round_up((uint64_t)dict_words_max * 2, kRingBytes);
    a.x_off = (uint32_t)dict16;
    a.tile_area = 64 * kRingBytes;
    const bool half = batch <= 8;   // 8 batch rows in the tile: room for two more wavefronts
    const bool more = half && dict16 + (size_t)kRingWavesMore * a.tile_area + ring_x_tile(8) + 128 <= kLdsLimit;   // a smaller dictionary leaves room
    // batches up to 4 beside a dictionary too large for that: a tile of 4 rows leaves room for one wavefront more
    const bool quarter = !more && batch <= 4 && dict16 + (size_t)kRingWavesQuarter * a.tile_area + ring_x_tile(4) + 128 <= kLdsLimit;
    const int waves = more ? kRingWavesMore : quarter ? kRingWavesQuarter : half ? kRingWavesHalf : kRingWaves;
    a.slot_off = (uint32_t)(dict16 + (size_t)waves * a.tile_area);
    p.lds = a.slot_off + ring_x_tile(quarter ? 4 : half ? 8 : 16) + 128;   // + the band counter
    if (p.lds > kLdsLimit || !x_fast) {
      set_error("internal: ring launch with a dictionary or activations that do not fit it");
      return TQ_E_UNSUPPORTED;
    }
    if (more) p.kernel = packed ? (const void*)k_matvec_ring<kRingWavesMore, 8, true> : (const void*)k_matvec_ring<kRingWavesMore, 8, false>;
    else if (quarter) p.kernel = packed ? (const void*)k_matvec_ring<kRingWavesQuarter, 4, true> : (const void*)k_matvec_ring<kRingWavesQuarter, 4, false>;
    else if (half) p.kernel = packed ? (const void*)k_matvec_ring<kRingWavesHalf, 8, true> : (const void*)k_matvec_ring<kRingWavesHalf, 8, false>;
    else p.kernel = packed ? (const void*)k_matvec_ring<kRingWaves, 16, true> : (const void*)k_matvec_ring<kRingWaves, 16, false>;
    p.block = (unsigned)waves * 64;
  } else {
    // Tile decode.  LDS: 16-bit dictionary image | one tile (64 strips) per wavefront, which the batched product reuses
    // for its partial sums (per wavefront two slots of 1 KB and their two band numbers).
    const size_t dict16 = round_up((uint64_t)dict16_max, 16);
    const size_t area = std::max<size_t>((size_t)64 * (seg_max + 8), 2048 + 8);
    const size_t waves = std::min<size_t>(kWaves, (kLdsLimit - dict16) / area);
    if (waves == 0) {
      set_error("segments of " + std::to_string(seg_max) + " columns do not fit the LDS tile");
      return TQ_E_UNSUPPORTED;
    }
    a.x_off = (uint32_t)dict16;
    a.tile_area = (uint32_t)area;
    a.slot_off = 0;
    p.lds = dict16 + waves * area;
    p.block = (unsigned)waves * 64;
    if (op == Op::kDecompress) p.kernel = long_runs ? (const void*)k_decompress<true> : (const void*)k_decompress<false>;
    else if (long_runs && packed) p.kernel = x_fast ? (const void*)k_matvec_mfma<true, true, true> : (const void*)k_matvec_mfma<false, true, true>;
    else if (long_runs) p.kernel = x_fast ? (const void*)k_matvec_mfma<true, false, true> : (const void*)k_matvec_mfma<false, false, true>;
    else if (packed) p.kernel = x_fast ? (const void*)k_matvec_mfma<true, true> : (const void*)k_matvec_mfma<false, true>;
    else p.kernel = x_fast ? (const void*)k_matvec_mfma<true, false> : (const void*)k_matvec_mfma<false, false>;
  }
  if (rec) {
    rec->launches.push_back(p);
    return TQ_OK;
  }
  return fire(p, stream);
}

// Whether the batched product of this matrix can keep a ring per lane instead of the whole strip.
// Bands per CU a launch needs for the ring kernel; tq_set_ring_min_bands_per_cu changes it (tests use 0 to put small
// matrices through that kernel).
std::atomic<uint64_t> g_ring_min_bands{kRingMinBandsPerCu};
uint64_t ring_min_bands_per_cu() { return g_ring_min_bands.load(std::memory_order_relaxed); }

bool ring_eligible(const tq_matrix* t, const void* x) {
  const DevMat& m = t->m;
  const uint32_t seg_weights = (m.packing ? 2u : 1u) * m.seg_cols;   // what the activation tile of a quad is sized by
  return m.reserved != 0 && m.cols % (kUnitPanels * m.seg_cols) == 0 && m.seg_cols % (8 * kRingGroup) == 0 &&
         seg_weights <= kRingMaxSeg && (uintptr_t)x % 16 == 0 &&
         round_up((uint64_t)m.dict_words * 2, kRingBytes) + (size_t)kRingWaves * 64 * kRingBytes + ring_x_tile(16) + 128 <= kLdsLimit;
}

// As few launches as the kernel-argument size and the 32-bit cost line allow.
int launch_all(Op op, int n, const tq_handle* hs, const void* const* xs, void* const* ys, int batch, hipStream_t stream, bool ring = false,
               bool gate_up = false, Recorder* rec = nullptr) {
  const int per_launch = rec ? kMaxStep : kMaxMulti;
  {
    // The kernels are built once per weight format: matrices of packed 4-bit weights, matrices with runs of 3 and 4
    // bytes and the others take separate launches.  (The expansion does not care about packing, only about the runs.)
    auto kind = [&](const tq_matrix* t) { return (op == Op::kMatvec && t->m.packing ? 1u : 0u) | (t->m.long_runs ? 2u : 0u); };
    uint32_t seen = 0;
    for (int i = 0; i < n; ++i) seen |= 1u << kind(hs[i]);
    if (seen & (seen - 1)) {   // more than one kind
      for (uint32_t want = 0; want < 4; ++want) {
        if (!(seen >> want & 1u)) continue;
        std::vector<tq_handle> h2;
        std::vector<const void*> x2;
        std::vector<void*> y2;
        for (int i = 0; i < n; ++i)
          if (kind(hs[i]) == want) {
            h2.push_back(hs[i]);
            x2.push_back(xs ? xs[i] : nullptr);
            y2.push_back(ys[i]);
          }
        if (int rc = launch_all(op, (int)h2.size(), h2.data(), xs ? x2.data() : nullptr, y2.data(), batch, stream, ring, gate_up, rec)) return rc;
      }
      return TQ_OK;
    }
  }
  // (one packing per call from here on)  The dot-product kernel takes the matrices whose activation image fits the LDS
  // beside the call's largest dictionary; the decision is taken here for the whole call, so that every launch cut from
  // it decides the same.  A call with both kinds is split.
  bool dot_call = false;
  if (op == Op::kMatvec && batch <= 2) {
    const bool packed = hs[0]->m.packing != 0, long_runs = hs[0]->m.long_runs != 0;
    uint32_t dict_words_max = 0;
    for (int i = 0; i < n; ++i) dict_words_max = std::max(dict_words_max, hs[i]->m.dict_words);
    int n_dot = 0;
    for (int i = 0; i < n; ++i) n_dot += dot_kernel_takes(batch, packed, long_runs, dict_words_max, hs[i]->m.x_dwords) ? 1 : 0;
    dot_call = n_dot == n;
    if (n_dot != 0 && n_dot != n) {
      for (int want = 1; want >= 0; --want) {
        std::vector<tq_handle> h2;
        std::vector<const void*> x2;
        std::vector<void*> y2;
        for (int i = 0; i < n; ++i)
          if ((dot_kernel_takes(batch, packed, long_runs, dict_words_max, hs[i]->m.x_dwords) ? 1 : 0) == want) {
            h2.push_back(hs[i]);
            x2.push_back(xs[i]);
            y2.push_back(ys[i]);
          }
        if (int rc = launch_all(op, (int)h2.size(), h2.data(), x2.data(), y2.data(), batch, stream, ring, gate_up, rec)) return rc;
      }
      return TQ_OK;
    }
  }
  if (op == Op::kMatvec && !dot_call && !ring && !gate_up) {   // (the ring kernel adds partial sums to y: no place for silu)
    // The matrices that can take the ring kernel go there, the others to the whole-strip kernel; the products are
    // independent, so regrouping them changes nothing but the launches.
    // The ring kernel gives whole bands to wavefronts, a quad at a time: it needs many bands per workgroup to keep its
    // wavefronts busy (the whole-strip kernel splits single units between them).
    int n_ring = 0;
    uint64_t ring_bands = 0;
    for (int i = 0; i < n; ++i)
      if (ring_eligible(hs[i], xs[i])) {
        ++n_ring;
        ring_bands += hs[i]->m.n_bands;
      }
    if (ring_bands < ring_min_bands_per_cu() * hs[0]->n_cu) n_ring = 0;
    if (n_ring == n) return launch_all(op, n, hs, xs, ys, batch, stream, true, false, rec);
    if (n_ring > 0) {
      std::vector<tq_handle> h2[2];
      std::vector<const void*> x2[2];
      std::vector<void*> y2[2];
      for (int i = 0; i < n; ++i) {
        const int g = ring_eligible(hs[i], xs[i]) ? 1 : 0;   // n_ring > 0: the eligible ones have enough bands together
        h2[g].push_back(hs[i]);
        x2[g].push_back(xs[i]);
        y2[g].push_back(ys[i]);
      }
      if (int rc = launch_all(op, (int)h2[1].size(), h2[1].data(), x2[1].data(), y2[1].data(), batch, stream, true, false, rec)) return rc;
      n = (int)h2[0].size();
      for (int i = 0; i < n;) {   // the rest, below, with the vectors alive
        int k = 0;
        uint64_t cost = 0;
        while (i + k < n && k < per_launch) {
          const uint64_t c = (uint64_t)h2[0][i + k]->m.n_bands * h2[0][i + k]->m.cols;
          if (k > 0 && cost + c > 0xFFFFFFFFull) break;
          cost += c;
          ++k;
        }
        if (int rc = launch(op, k, h2[0].data() + i, x2[0].data() + i, y2[0].data() + i, batch, stream, false, false, rec)) return rc;
        i += k;
      }
      return TQ_OK;
    }
  }
  for (int i = 0; i < n;) {
    int k = 0;
    uint64_t cost = 0;
    while (i + k < n && k < per_launch) {
      const uint64_t c = (uint64_t)hs[i + k]->m.n_bands * hs[i + k]->m.cols;
      if (k > 0 && cost + c > 0xFFFFFFFFull) break;
      cost += c;
      ++k;
    }
    if (int rc = launch(op, k, hs + i, xs ? xs + i : nullptr, ys + i, batch, stream, ring, gate_up, rec)) return rc;
    i += k;
  }
  return TQ_OK;
}

int check_call(const char* who, int n, const tq_handle* hs, const void* const* xs, void* const* ys, int batch) {
  if (batch < 1 || batch > TQ_MAX_BATCH) {
    set_error(std::string(who) + ": batch must be in [1, " + std::to_string(TQ_MAX_BATCH) + "]");
    return TQ_E_UNSUPPORTED;
  }
  for (int i = 0; i < n; ++i) {
    if (!hs[i] || !xs[i] || !ys[i]) {
      set_error(std::string(who) + ": null handle or pointer at index " + std::to_string(i));
      return TQ_E_INVALID_ARG;
    }
    if ((uintptr_t)xs[i] % 2 || (uintptr_t)ys[i] % 4) {
      set_error(std::string(who) + ": x must be 2-byte and y 4-byte aligned");
      return TQ_E_INVALID_ARG;
    }
    if (hs[i]->device != hs[0]->device) {
      set_error(std::string(who) + ": all matrices of a call must live on one device");
      return TQ_E_INVALID_ARG;
    }
  }
  return TQ_OK;
}

}  // namespace

static int tq_matvec_impl(tq_handle h, const void* x, void* y, int batch, void* stream) {
  if (!h || !x || !y) {
    set_error("tq_matvec: null argument");
    return TQ_E_INVALID_ARG;
  }
  if (int rc = check_call("tq_matvec", 1, &h, &x, &y, batch)) return rc;
  return launch(Op::kMatvec, 1, &h, &x, &y, batch, (hipStream_t)stream,
                !dot_kernel_takes(batch, h->m.packing != 0, h->m.long_runs != 0, h->m.dict_words, h->m.x_dwords) && ring_eligible(h, x) &&
                    h->m.n_bands >= ring_min_bands_per_cu() * h->n_cu);
}

static int tq_matvec_multi_impl(int n, const tq_handle* hs, const void* const* xs, void* const* ys, int batch, void* stream) {
  if (n < 1 || !hs || !xs || !ys) {
    set_error("tq_matvec_multi: null argument or n < 1");
    return TQ_E_INVALID_ARG;
  }
  if (int rc = check_call("tq_matvec_multi", n, hs, xs, ys, batch)) return rc;
  return launch_all(Op::kMatvec, n, hs, xs, ys, batch, (hipStream_t)stream);
}

static int tq_matvec_gate_up_multi_impl(int n, const tq_handle* hs, const void* const* xs, void* const* ys, int batch, void* stream) {
  if (n < 1 || !hs || !xs || !ys) {
    set_error("tq_matvec_gate_up_multi: null argument or n < 1");
    return TQ_E_INVALID_ARG;
  }
  if (int rc = check_call("tq_matvec_gate_up_multi", n, hs, xs, ys, batch)) return rc;
  for (int i = 0; i < n; ++i)
    if (hs[i]->m.rows % 2) {
      set_error("tq_matvec_gate_up_multi: the matrix at index " + std::to_string(i) + " has an odd number of rows");
      return TQ_E_INVALID_ARG;
    }
  return launch_all(Op::kMatvec, n, hs, xs, ys, batch, (hipStream_t)stream, false, true);
}

static int tq_matvec_gate_up_impl(tq_handle h, const void* x, void* y, int batch, void* stream) {
  if (!h || !x || !y) {
    set_error("tq_matvec_gate_up: null argument");
    return TQ_E_INVALID_ARG;
  }
  return tq_matvec_gate_up_multi(1, &h, &x, &y, batch, stream);
}

// A prepared step: the launches tq_matvec_multi (or tq_matvec_gate_up_multi) would make for these matrices and buffers,
// decided once, with the jobs in a device table so that one launch can serve up to kMaxStep matrices.
struct tq_step {
  std::vector<PreparedLaunch> launches;
  StepEntry* table_dev;
  size_t n_entries;
  int n_matrices;
  // staged steps that run as one launch (all stages in one persistent kernel):
  uint32_t n_stages = 0;
  bool persistent = false;
  uint32_t* stage_dev = nullptr;    // stage_first[n_stages + 1] | sync[n_stages + 1]
  uint32_t* fault_host = nullptr;   // pinned host word the kernel sets when a hand-over wait gave up
};

constexpr uint32_t kDefaultSpinLimit = 1u << 20;   // polls of a stage counter (a microsecond or two each) before a workgroup gives up

static int tq_step_create_impl(int n, const tq_handle* hs, const void* const* xs, void* const* ys, int batch, uint32_t flags,
                              tq_step_handle* out) {
  if (!out) {
    set_error("tq_step_create: null output pointer");
    return TQ_E_INVALID_ARG;
  }
  *out = nullptr;
  const bool expand = (flags & TQ_STEP_DECOMPRESS) != 0, gate_up = (flags & TQ_STEP_GATE_UP) != 0;
  if (n < 1 || !hs || !ys || (!xs && !expand) || (flags & ~(TQ_STEP_GATE_UP | TQ_STEP_DECOMPRESS)) || (expand && gate_up)) {
    set_error("tq_step_create: null argument, n < 1 or unknown combination of flags");
    return TQ_E_INVALID_ARG;
  }
  if (expand) {   // tq_decompress_multi prepared: ys are the int8 matrices, xs and batch are not used
    for (int i = 0; i < n; ++i) {
      if (!hs[i] || !ys[i]) {
        set_error("tq_step_create: null handle or pointer at index " + std::to_string(i));
        return TQ_E_INVALID_ARG;
      }
      if (hs[i]->device != hs[0]->device) {
        set_error("tq_step_create: all matrices of a step must live on one device");
        return TQ_E_INVALID_ARG;
      }
    }
  } else if (int rc = check_call("tq_step_create", n, hs, xs, ys, batch)) {
    return rc;
  }
  if (gate_up)
    for (int i = 0; i < n; ++i)
      if (hs[i]->m.rows % 2) {
        set_error("tq_step_create: the matrix at index " + std::to_string(i) + " has an odd number of rows");
        return TQ_E_INVALID_ARG;
      }
  try {
    Recorder rec;
    if (int rc = expand ? launch_all(Op::kDecompress, n, hs, nullptr, ys, 1, nullptr, false, false, &rec)
                        : launch_all(Op::kMatvec, n, hs, xs, ys, batch, nullptr, false, gate_up, &rec))
      return rc;
    tq_step* s = new tq_step;
    s->launches = std::move(rec.launches);
    s->n_entries = rec.entries.size();
    s->n_matrices = n;
    s->table_dev = nullptr;
    hipError_t e = hipMalloc((void**)&s->table_dev, rec.entries.size() * sizeof(StepEntry));
    if (e == hipSuccess) e = hipMemcpy(s->table_dev, rec.entries.data(), rec.entries.size() * sizeof(StepEntry), hipMemcpyHostToDevice);
    if (e != hipSuccess) {
      if (s->table_dev) (void)hipFree(s->table_dev);
      delete s;
      if (e == hipErrorOutOfMemory) {
        set_error("tq_step_create: out of device memory");
        return TQ_E_OOM;
      }
      return hip_fail("tq_step_create", e);
    }
    for (PreparedLaunch& p : s->launches) p.a.table = s->table_dev + p.table_first;
    *out = s;
    return TQ_OK;
  } catch (const std::bad_alloc&) {
    set_error("tq_step_create: out of host memory");
    return TQ_E_OOM;
  }
}

// A staged step: products that depend on each other in one prepared step.  When every matrix takes the dot-product
// kernel (batch 1 or 2, ordinary or packed weights, rows that fit its activation image) the whole step is ONE launch of
// that kernel's staged form, one workgroup per compute unit, with a grid-wide hand-over between stages; otherwise
// every stage gets the launches tq_matvec_multi would make for it, in stage order on the stream.
static int tq_step_create_staged_impl(int n, const tq_handle* hs, const void* const* xs, void* const* ys, const int* stage, int batch,
                                      uint32_t flags, tq_step_handle* out) {
  if (!out) {
    set_error("tq_step_create_staged: null output pointer");
    return TQ_E_INVALID_ARG;
  }
  *out = nullptr;
  if (n < 1 || !hs || !xs || !ys || !stage || flags != 0) {
    set_error("tq_step_create_staged: null argument, n < 1 or flags (none are defined for staged steps)");
    return TQ_E_INVALID_ARG;
  }
  if (int rc = check_call("tq_step_create_staged", n, hs, xs, ys, batch)) return rc;
  if (stage[0] != 0) {
    set_error("tq_step_create_staged: stages are numbered from 0");
    return TQ_E_INVALID_ARG;
  }
  for (int i = 1; i < n; ++i)
    if (stage[i] != stage[i - 1] && stage[i] != stage[i - 1] + 1) {
      set_error("tq_step_create_staged: stage numbers must not decrease and must not skip (index " + std::to_string(i) + ")");
      return TQ_E_INVALID_ARG;
    }
  const uint32_t n_stages = (uint32_t)stage[n - 1] + 1;
  std::vector<uint32_t> first(n_stages + 1, (uint32_t)n);
  for (int i = n - 1; i >= 0; --i) first[stage[i]] = (uint32_t)i;

  const bool packed = hs[0]->m.packing != 0;
  uint32_t dict_words_max = 0, x_dwords_max = 0;
  uint64_t cost = 0;
  bool one_kind = n <= kMaxStep;
  for (int i = 0; i < n; ++i) {
    one_kind = one_kind && (hs[i]->m.packing != 0) == packed && !hs[i]->m.long_runs;
    dict_words_max = std::max(dict_words_max, hs[i]->m.dict_words);
    x_dwords_max = std::max(x_dwords_max, hs[i]->m.x_dwords);
    cost += (uint64_t)hs[i]->m.n_bands * hs[i]->m.cols;
  }
  const bool persistent = one_kind && cost <= 0xFFFFFFFFull && dot_kernel_takes(batch, packed, false, dict_words_max, x_dwords_max);

  tq_step* s = new tq_step;
  s->table_dev = nullptr;
  s->n_matrices = n;
  s->n_stages = n_stages;
  s->persistent = persistent;
  auto fail = [&](int rc) {
    if (s->table_dev) (void)hipFree(s->table_dev);
    if (s->stage_dev) (void)hipFree(s->stage_dev);
    if (s->fault_host) (void)hipHostFree(s->fault_host);
    delete s;
    return rc;
  };
  Recorder rec;
  if (!persistent) {
    for (uint32_t k = 0; k < n_stages; ++k)
      if (int rc = launch_all(Op::kMatvec, (int)(first[k + 1] - first[k]), hs + first[k], xs + first[k], ys + first[k], batch, nullptr, false,
                              false, &rec))
        return fail(rc);
  } else {
    PreparedLaunch p;
    MatvecArgs& a = p.a;
    std::memset(&a, 0, sizeof a);
    a.n = n;
    a.batch = batch;
    a.n_stages = n_stages;
    a.spin_limit = kDefaultSpinLimit;
    a.table = (const StepEntry*)(uintptr_t)8;   // (the address follows below)
    p.table_first = 0;
    p.what = "tq_step_launch (staged)";
    uint64_t c = 0;
    for (int i = 0; i < n; ++i) {
      rec.entries.push_back(StepEntry{hs[i]->m, (const uint16_t*)xs[i], (float*)ys[i]});
      a.u.cost_long[i] = (uint32_t)c;
      c += (uint64_t)hs[i]->m.n_bands * hs[i]->m.cols;
    }
    a.u.cost_long[n] = (uint32_t)c;
    if (!plan_matvec_lds(dict_words_max, (packed && batch == 2 ? 2 : 1) * x_dwords_max, &a.x_off, &a.slot_off, &p.lds)) {
      set_error("tq_step_create_staged: internal: LDS plan");
      return fail(TQ_E_UNSUPPORTED);
    }
    p.kernel = packed ? (batch == 2 ? (const void*)k_matvec<kDotPiecePacked, kDotWavesPacked, true, 2, false, true>
                                    : (const void*)k_matvec<kDotPiecePacked, kDotWavesPacked, true, 1, false, true>)
               : batch == 2 ? (const void*)k_matvec<kDotPiece, kDotWavesStaged, false, 2, false, true>
                            : (const void*)k_matvec<kDotPiece, kDotWavesStaged, false, 1, false, true>;
    p.block = (packed ? kDotWavesPacked : kDotWavesStaged) * 64;
    p.grid = (unsigned)hs[0]->n_cu;   // one workgroup per compute unit (each takes the whole LDS): all resident together
    rec.launches.push_back(p);
  }
  s->launches = std::move(rec.launches);
  s->n_entries = rec.entries.size();
  hipError_t e = hipMalloc((void**)&s->table_dev, rec.entries.size() * sizeof(StepEntry));
  if (e == hipSuccess) e = hipMemcpy(s->table_dev, rec.entries.data(), rec.entries.size() * sizeof(StepEntry), hipMemcpyHostToDevice);
  if (e == hipSuccess && persistent) {
    e = hipMalloc((void**)&s->stage_dev, (size_t)2 * (n_stages + 1) * 4);
    if (e == hipSuccess) e = hipMemset(s->stage_dev, 0, (size_t)2 * (n_stages + 1) * 4);
    if (e == hipSuccess) e = hipMemcpy(s->stage_dev, first.data(), (size_t)(n_stages + 1) * 4, hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipHostMalloc((void**)&s->fault_host, 64, hipHostMallocMapped);
    if (e == hipSuccess) *s->fault_host = 0;
  }
  if (e != hipSuccess) {
    const bool oom = e == hipErrorOutOfMemory;
    if (oom) set_error("tq_step_create_staged: out of device memory");
    return fail(oom ? TQ_E_OOM : hip_fail("tq_step_create_staged", e));
  }
  for (PreparedLaunch& p : s->launches) {
    p.a.table = s->table_dev + p.table_first;
    if (persistent) {
      p.a.stage_first = s->stage_dev;
      p.a.sync = s->stage_dev + n_stages + 1;
      void* dp = nullptr;
      e = hipHostGetDevicePointer(&dp, s->fault_host, 0);
      if (e != hipSuccess) return fail(hip_fail("hipHostGetDevicePointer", e));
      p.a.fault_host = (uint32_t*)dp;
    }
  }
  *out = s;
  return TQ_OK;
}

static int tq_step_launch_impl(tq_step_handle s, void* stream) {
  if (!s) {
    set_error("tq_step_launch: null step");
    return TQ_E_INVALID_ARG;
  }
  if (s->persistent) {
    if (*(volatile uint32_t*)s->fault_host != 0) {
      set_error("tq_step_launch: an earlier launch of this staged step gave up waiting at a stage hand-over (were all its workgroups "
                "resident together?); its results must not be used");
      return TQ_E_HIP;
    }
    hipLaunchKernelGGL(k_zero_words, dim3(1), dim3(256), 0, (hipStream_t)stream, s->stage_dev + s->n_stages + 1, s->n_stages + 1);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail("tq_step_launch: counter reset", e);
  }
  for (const PreparedLaunch& p : s->launches)
    if (int rc = fire(p, (hipStream_t)stream)) return rc;
  return TQ_OK;
}

extern "C" int tq_step_get_info(tq_step_handle s, tq_step_info* out) {
  if (!s || !out) {
    set_error("tq_step_get_info: null argument");
    return TQ_E_INVALID_ARG;
  }
  out->n_matrices = (uint32_t)s->n_matrices;
  out->n_launches = (uint32_t)s->launches.size();
  out->table_bytes = (uint64_t)s->n_entries * sizeof(StepEntry) + (s->stage_dev ? (uint64_t)(2 * (s->n_stages + 1)) * 4 : 0);
  out->n_stages = s->n_stages;
  out->persistent = s->persistent ? 1u : 0u;
  out->fault = s->fault_host ? *(volatile uint32_t*)s->fault_host : 0u;
  return TQ_OK;
}

static int tq_step_destroy_impl(tq_step_handle s) {
  if (!s) return TQ_OK;
  hipError_t e = hipFree(s->table_dev);
  if (s->stage_dev) (void)hipFree(s->stage_dev);
  if (s->fault_host) (void)hipHostFree(s->fault_host);
  delete s;
  if (e != hipSuccess) return hip_fail("tq_step_destroy", e);
  return TQ_OK;
}

static int tq_decompress_impl(tq_handle h, void* out, void* stream) {
  if (!h || !out) {
    set_error("tq_decompress: null argument");
    return TQ_E_INVALID_ARG;
  }
  return launch(Op::kDecompress, 1, &h, nullptr, &out, 1, (hipStream_t)stream);
}

static int tq_decompress_multi_impl(int n, const tq_handle* hs, void* const* outs, void* stream) {
  if (n < 1 || !hs || !outs) {
    set_error("tq_decompress_multi: null argument or n < 1");
    return TQ_E_INVALID_ARG;
  }
  for (int i = 0; i < n; ++i) {
    if (!hs[i] || !outs[i]) {
      set_error("tq_decompress_multi: null handle or pointer at index " + std::to_string(i));
      return TQ_E_INVALID_ARG;
    }
    if (hs[i]->device != hs[0]->device) {
      set_error("tq_decompress_multi: all matrices of a call must live on one device");
      return TQ_E_INVALID_ARG;
    }
  }
  return launch_all(Op::kDecompress, n, hs, nullptr, outs, 1, (hipStream_t)stream);
}

extern "C" int tq_get_info(tq_handle h, tq_info* out) {
  if (!h || !out) {
    set_error("tq_get_info: null argument");
    return TQ_E_INVALID_ARG;
  }
  fill_info(h->h, h->facts, out);
  return TQ_OK;
}

static int tq_destroy_impl(tq_handle h) {
  if (!h) return TQ_OK;
  hipError_t e = hipFree(h->dev_base);
  hipError_t e2 = release_dictionary(h->dict);
  delete h;
  if (e != hipSuccess) return hip_fail("hipFree", e);
  if (e2 != hipSuccess) return hip_fail("hipFree", e2);
  return TQ_OK;
}

// tq_matvec_multi with the job table of a prepared step, but in the library's static device array instead of memory
// allocated for the step: the plan is made as for tq_step_create, small writer launches fill the table on `stream`
// (the jobs travel in their kernel arguments), and the product launches that follow on the same stream read it.
static int tq_matvec_multi_static_impl(int n, const tq_handle* hs, const void* const* xs, void* const* ys, int batch, void* stream) {
  if (n < 1 || !hs || !xs || !ys) {
    set_error("tq_matvec_multi_static: null argument or n < 1");
    return TQ_E_INVALID_ARG;
  }
  if (n > kMaxStep) {
    set_error("tq_matvec_multi_static: " + std::to_string(n) + " matrices do not fit the static job table (at most " +
              std::to_string(kMaxStep) + " per call)");
    return TQ_E_UNSUPPORTED;
  }
  if (int rc = check_call("tq_matvec_multi_static", n, hs, xs, ys, batch)) return rc;
  StepEntry* table = nullptr;
  {
    std::lock_guard<std::mutex> lock(g_static_mutex);
    const int dev = hs[0]->device;
    table = dev >= 0 && dev < kMaxDevices ? g_static_table[dev] : nullptr;   // looked up when the first matrix was created there
  }
  if (!table) {
    set_error("tq_matvec_multi_static: no static table is known for the matrices' device");
    return TQ_E_HIP;
  }
  Recorder rec;
  if (int rc = launch_all(Op::kMatvec, n, hs, xs, ys, batch, nullptr, false, false, &rec)) return rc;
  if (rec.refs.size() > (size_t)kMaxStep) {   // (cannot happen: one entry per matrix)
    set_error("tq_matvec_multi_static: internal: more jobs than matrices");
    return TQ_E_UNSUPPORTED;
  }
  for (size_t first = 0; first < rec.refs.size(); first += kWriterJobs) {
    TableWrite w;
    w.table = table + first;
    w.n = (int)std::min<size_t>(kWriterJobs, rec.refs.size() - first);
    std::memcpy(w.j, rec.refs.data() + first, (size_t)w.n * sizeof(JobRef));
    hipLaunchKernelGGL(k_write_table, dim3((unsigned)w.n), dim3(64), 0, (hipStream_t)stream, w);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail("tq_matvec_multi_static: table writer launch", e);
  }
  for (PreparedLaunch& p : rec.launches) {
    p.a.table = table + p.table_first;
    if (int rc = fire(p, (hipStream_t)stream)) return rc;
  }
  return TQ_OK;
}

// The entry points proper: argument checks and work above, behind a wrapper that lets no C++ exception out.
extern "C" int tq_create_from_encoded(const void* blob, size_t blob_bytes, tq_handle* out) {
  return guarded("tq_create_from_encoded", [&] { return tq_create_from_encoded_impl(blob, blob_bytes, out); });
}

extern "C" int tq_matvec(tq_handle h, const void* x, void* y, int batch, void* stream) {
  return guarded("tq_matvec", [&] { return tq_matvec_impl(h, x, y, batch, stream); });
}

extern "C" int tq_matvec_multi(int n, const tq_handle* hs, const void* const* xs, void* const* ys, int batch, void* stream) {
  return guarded("tq_matvec_multi", [&] { return tq_matvec_multi_impl(n, hs, xs, ys, batch, stream); });
}

extern "C" int tq_matvec_gate_up_multi(int n, const tq_handle* hs, const void* const* xs, void* const* ys, int batch, void* stream) {
  return guarded("tq_matvec_gate_up_multi", [&] { return tq_matvec_gate_up_multi_impl(n, hs, xs, ys, batch, stream); });
}

extern "C" int tq_matvec_gate_up(tq_handle h, const void* x, void* y, int batch, void* stream) {
  return guarded("tq_matvec_gate_up", [&] { return tq_matvec_gate_up_impl(h, x, y, batch, stream); });
}

extern "C" int tq_step_create(int n, const tq_handle* hs, const void* const* xs, void* const* ys, int batch, uint32_t flags, tq_step_handle* out) {
  return guarded("tq_step_create", [&] { return tq_step_create_impl(n, hs, xs, ys, batch, flags, out); });
}

extern "C" int tq_step_launch(tq_step_handle s, void* stream) {
  return guarded("tq_step_launch", [&] { return tq_step_launch_impl(s, stream); });
}

extern "C" int tq_decompress(tq_handle h, void* out, void* stream) {
  return guarded("tq_decompress", [&] { return tq_decompress_impl(h, out, stream); });
}

extern "C" int tq_decompress_multi(int n, const tq_handle* hs, void* const* outs, void* stream) {
  return guarded("tq_decompress_multi", [&] { return tq_decompress_multi_impl(n, hs, outs, stream); });
}

extern "C" int tq_destroy(tq_handle h) {
  return guarded("tq_destroy", [&] { return tq_destroy_impl(h); });
}

extern "C" int tq_step_destroy(tq_step_handle s) {
  return guarded("tq_step_destroy", [&] { return tq_step_destroy_impl(s); });
}

extern "C" int tq_step_create_staged(int n, const tq_handle* hs, const void* const* xs, void* const* ys, const int* stage, int batch,
                                     uint32_t flags, tq_step_handle* out) {
  return guarded("tq_step_create_staged", [&] { return tq_step_create_staged_impl(n, hs, xs, ys, stage, batch, flags, out); });
}

extern "C" int tq_step_set_spin_limit(tq_step_handle s, uint32_t polls) {
  if (!s) {
    set_error("tq_step_set_spin_limit: null step");
    return TQ_E_INVALID_ARG;
  }
  for (PreparedLaunch& p : s->launches) p.a.spin_limit = polls;
  return TQ_OK;
}

extern "C" int tq_matvec_multi_static(int n, const tq_handle* hs, const void* const* xs, void* const* ys, int batch, void* stream) {
  return guarded("tq_matvec_multi_static", [&] { return tq_matvec_multi_static_impl(n, hs, xs, ys, batch, stream); });
}

extern "C" int tq_set_ring_min_bands_per_cu(uint32_t bands_per_cu) {
  g_ring_min_bands.store(bands_per_cu, std::memory_order_relaxed);
  return TQ_OK;
}
