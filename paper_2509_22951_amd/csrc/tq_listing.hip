// The stream format of the paper's section 4 listings ("Finding Frequent Sequences", "Compressing Model Weights",
// "Decompressing Model Weights"), taken literally: a table of the most frequent windows of 4 consecutive byte values,
// and per parameter a sequence of 16-bit words in which a group of 4 values is either its table codeword (1, 2, ...) or
// the marker 0xFFFF followed by the values themselves, one word each.  Host side: table, compression, validation.
// Device side: decompression (gfx950).
//
// How the sequential reader of the third listing becomes a parallel one.  A raw value is at most 255, so every word
// 0xFFFF in a valid stream is a marker, and the words a marker covers are the up to 4 words after it: whether a word
// starts a token (codeword, or marker with its values) is decided by the 4 words before it alone.  Every token yields
// exactly 4 values (the last one of a stream possibly fewer), so token t writes values [4 t, 4 t + 4): all that is
// missing is the number of tokens before a word.  That count is a property of the stream, not of a call: the host
// takes it once per block of kBlockWords words while it validates the stream, and the kernel adds a prefix count
// within the block (one ballot per word position of a thread + one pass over the wave totals in LDS).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdlib>
#include <cstring>
#include <new>
#include <string>
#include <unordered_map>
#include <vector>

#include "../../include/tq.h"
#include "tq_format.h"

namespace tq {
namespace {

constexpr uint32_t kSeq = TQ_LISTING_SEQ;
constexpr uint32_t kMarker = 0xFFFFu;
constexpr int kThreadWords = 8;     // words per thread: one 16-byte load
constexpr int kListingThreads = 256;
constexpr int kBlockWords = kListingThreads * kThreadWords;   // words per workgroup

int hip_fail(const char* what, hipError_t e) {
  set_error(std::string(what) + ": " + hipGetErrorString(e));
  return TQ_E_HIP;
}

inline uint32_t pack4(const uint8_t* v) { return v[0] | (uint32_t)v[1] << 8 | (uint32_t)v[2] << 16 | (uint32_t)v[3] << 24; }

// Thread t of a workgroup takes the 8 words [8 t, 8 t + 8) of the workgroup's kBlockWords words, plus the 4 words before
// them (to know which of its words are raw values) and the 4 after them (the raw values of a marker near its end).
// words: n_words 16-bit words, 16-byte aligned; table[c - 1]: the 4 values of codeword c, first value in the low byte;
// block_base[b]: tokens that start before word b * kBlockWords; out: n_values bytes.
__global__ __launch_bounds__(kListingThreads) void k_listing_decompress(const uint16_t* __restrict__ words, uint64_t n_words,
                                                                        const uint32_t* __restrict__ table,
                                                                        const uint32_t* __restrict__ block_base, uint8_t* __restrict__ out) {
  __shared__ uint32_t wave_tokens[kListingThreads / 64];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const uint64_t i0 = ((uint64_t)blockIdx.x * kListingThreads + tid) * kThreadWords;   // this thread's first word
  // w[4 + j] = word i0 + j for j = -4 .. 11; words outside the stream read as 0, which is neither marker nor codeword
  uint32_t w[kThreadWords + 2 * kSeq];
  {
    uint2 before = make_uint2(0u, 0u), after = make_uint2(0u, 0u);
    uint4 mine = make_uint4(0u, 0u, 0u, 0u);
    if (i0 >= kSeq && i0 <= n_words) before = *(const uint2*)(words + i0 - kSeq);
    if (i0 + kThreadWords <= n_words) {
      mine = *(const uint4*)(words + i0);
    } else {
      uint32_t h[kThreadWords];
      for (int j = 0; j < kThreadWords; ++j) h[j] = i0 + j < n_words ? words[i0 + j] : 0u;
      mine = make_uint4(h[0] | h[1] << 16, h[2] | h[3] << 16, h[4] | h[5] << 16, h[6] | h[7] << 16);
    }
    if (i0 + kThreadWords + kSeq <= n_words) {
      after = *(const uint2*)(words + i0 + kThreadWords);
    } else {
      uint32_t h[kSeq];
      for (int j = 0; j < (int)kSeq; ++j) h[j] = i0 + kThreadWords + j < n_words ? words[i0 + kThreadWords + j] : 0u;
      after = make_uint2(h[0] | h[1] << 16, h[2] | h[3] << 16);
    }
    const uint32_t packed[8] = {before.x, before.y, mine.x, mine.y, mine.z, mine.w, after.x, after.y};
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      w[2 * k] = packed[k] & 0xFFFFu;
      w[2 * k + 1] = packed[k] >> 16;
    }
  }
  // which of the thread's words start a token
  uint32_t starts = 0;
#pragma unroll
  for (int j = 0; j < kThreadWords; ++j) {
    const bool covered = w[kSeq + j - 1] == kMarker || w[kSeq + j - 2] == kMarker || w[kSeq + j - 3] == kMarker || w[kSeq + j - 4] == kMarker;
    if (i0 + j < n_words && !covered) starts |= 1u << j;
  }
  // tokens that start in the workgroup before this thread's words: threads of lower lanes, then lower wavefronts
  uint32_t lower = 0, in_wave = 0;
#pragma unroll
  for (int j = 0; j < kThreadWords; ++j) {
    const uint64_t ballot = __builtin_amdgcn_ballot_w64((starts >> j) & 1u);
    lower += (uint32_t)__builtin_popcountll(ballot & ((1ull << lane) - 1));
    in_wave += (uint32_t)__builtin_popcountll(ballot);
  }
  if (lane == 0) wave_tokens[wave] = in_wave;
  __syncthreads();
  for (int v = 0; v < wave; ++v) lower += wave_tokens[v];
  uint64_t token = (uint64_t)block_base[blockIdx.x] + lower;
  const bool aligned = ((uintptr_t)out & 3) == 0;
#pragma unroll
  for (int j = 0; j < kThreadWords; ++j) {
    if (!((starts >> j) & 1u)) continue;
    const uint32_t c = w[kSeq + j];
    uint32_t v4, n = kSeq;
    if (c == kMarker) {
      v4 = (w[kSeq + j + 1] & 0xFF) | (w[kSeq + j + 2] & 0xFF) << 8 | (w[kSeq + j + 3] & 0xFF) << 16 | (w[kSeq + j + 4] & 0xFF) << 24;
      const uint64_t left = n_words - 1 - (i0 + j);   // the last marker of a stream may have fewer values
      if (left < kSeq) n = (uint32_t)left;
    } else {
      v4 = table[c - 1];
    }
    const uint64_t o = token * kSeq;   // first value of this token
    if (n == kSeq && aligned) {
      *(uint32_t*)(out + o) = v4;
    } else {
      for (uint32_t b = 0; b < n; ++b) out[o + b] = (uint8_t)(v4 >> (8 * b));
    }
    ++token;
  }
}

}  // namespace
}  // namespace tq

using namespace tq;

struct tq_listing_s {
  uint16_t* words;        // device
  uint32_t* table;        // device, one packed word per entry
  uint32_t* block_base;   // device
  tq_listing_info info;
  uint64_t n_blocks;
  int device;
};

extern "C" int tq_listing_build_table(const uint8_t* const* params, const uint64_t* lens, uint32_t n_params, uint32_t top_k,
                                      uint8_t** table, uint32_t* n_table) {
  if (!table || !n_table || (n_params && (!params || !lens))) {
    set_error("tq_listing_build_table: null argument");
    return TQ_E_INVALID_ARG;
  }
  *table = nullptr;
  *n_table = 0;
  if (top_k > TQ_LISTING_MAX_TOP_K) {
    set_error("tq_listing_build_table: top_k above " + std::to_string(TQ_LISTING_MAX_TOP_K) + " would give a codeword the marker's value");
    return TQ_E_UNSUPPORTED;
  }
  uint64_t n_windows = 0;
  for (uint32_t p = 0; p < n_params; ++p) {
    if (lens[p] && !params[p]) {
      set_error("tq_listing_build_table: null parameter");
      return TQ_E_INVALID_ARG;
    }
    if (lens[p] >= kSeq) n_windows += lens[p] - kSeq + 1;
  }
  if (n_windows >= (1ull << 32)) {
    set_error("tq_listing_build_table: 2^32 windows or more are not supported");
    return TQ_E_UNSUPPORTED;
  }
  if (n_windows == 0 || top_k == 0) return TQ_OK;
  try {
    // (window value, order of appearance) for every window of every parameter; sorted, equal windows are adjacent and
    // the first of them is the first appearance.
    std::vector<uint64_t> items;
    items.reserve(n_windows);
    uint64_t seen = 0;
    for (uint32_t p = 0; p < n_params; ++p) {
      if (lens[p] < kSeq) continue;
      const uint8_t* v = params[p];
      uint32_t key = pack4(v);
      items.push_back((uint64_t)key << 32 | seen++);
      for (uint64_t i = kSeq; i < lens[p]; ++i) {
        key = key >> 8 | (uint32_t)v[i] << 24;
        items.push_back((uint64_t)key << 32 | seen++);
      }
    }
    std::sort(items.begin(), items.end());
    struct Ranked {
      uint32_t count, first, key;
    };
    std::vector<Ranked> distinct;
    for (size_t i = 0; i < items.size();) {
      size_t j = i + 1;
      const uint32_t key = (uint32_t)(items[i] >> 32);
      while (j < items.size() && (uint32_t)(items[j] >> 32) == key) ++j;
      distinct.push_back({(uint32_t)(j - i), (uint32_t)items[i], key});
      i = j;
    }
    items.clear();
    items.shrink_to_fit();
    const size_t n = std::min<size_t>(top_k, distinct.size());
    auto better = [](const Ranked& a, const Ranked& b) { return a.count != b.count ? a.count > b.count : a.first < b.first; };
    std::partial_sort(distinct.begin(), distinct.begin() + n, distinct.end(), better);
    uint8_t* t = (uint8_t*)std::malloc(std::max<size_t>(n * kSeq, 1));
    if (!t) throw std::bad_alloc();
    for (size_t i = 0; i < n; ++i)
      for (uint32_t b = 0; b < kSeq; ++b) t[i * kSeq + b] = (uint8_t)(distinct[i].key >> (8 * b));
    *table = t;
    *n_table = (uint32_t)n;
  } catch (const std::bad_alloc&) {
    set_error("tq_listing_build_table: out of host memory");
    return TQ_E_OOM;
  }
  return TQ_OK;
}

extern "C" int tq_listing_compress(const uint8_t* values, uint64_t n_values, const uint8_t* table, uint32_t n_table, uint16_t** words,
                                   uint64_t* n_words) {
  if (!words || !n_words || (n_values && !values) || (n_table && !table)) {
    set_error("tq_listing_compress: null argument");
    return TQ_E_INVALID_ARG;
  }
  *words = nullptr;
  *n_words = 0;
  if (n_table > TQ_LISTING_MAX_TOP_K) {
    set_error("tq_listing_compress: table larger than " + std::to_string(TQ_LISTING_MAX_TOP_K) + " entries");
    return TQ_E_UNSUPPORTED;
  }
  try {
    std::unordered_map<uint32_t, uint16_t> code_of;
    code_of.reserve(n_table * 2);
    for (uint32_t c = 0; c < n_table; ++c)
      if (!code_of.emplace(pack4(table + (size_t)c * kSeq), (uint16_t)(c + 1)).second) {
        set_error("tq_listing_compress: table entries must be distinct");
        return TQ_E_INVALID_ARG;
      }
    std::vector<uint16_t> out;
    out.reserve(n_values / kSeq + 16);
    uint64_t i = 0;
    for (; i + kSeq <= n_values; i += kSeq) {
      auto it = code_of.find(pack4(values + i));
      if (it != code_of.end()) {
        out.push_back(it->second);
      } else {
        out.push_back((uint16_t)kMarker);
        for (uint32_t b = 0; b < kSeq; ++b) out.push_back(values[i + b]);
      }
    }
    if (i < n_values) {
      out.push_back((uint16_t)kMarker);
      for (; i < n_values; ++i) out.push_back(values[i]);
    }
    uint16_t* w = (uint16_t*)std::malloc(std::max<size_t>(out.size() * 2, 1));
    if (!w) throw std::bad_alloc();
    std::memcpy(w, out.data(), out.size() * 2);
    *words = w;
    *n_words = out.size();
  } catch (const std::bad_alloc&) {
    set_error("tq_listing_compress: out of host memory");
    return TQ_E_OOM;
  }
  return TQ_OK;
}

static int listing_create_impl(const uint16_t* words, uint64_t n_words, const uint8_t* table, uint32_t n_table, tq_listing* out) {
  if (!out || (n_words && !words) || (n_table && !table)) {
    set_error("tq_listing_create: null argument");
    return TQ_E_INVALID_ARG;
  }
  *out = nullptr;
  if (n_table > TQ_LISTING_MAX_TOP_K) {
    set_error("tq_listing_create: table larger than " + std::to_string(TQ_LISTING_MAX_TOP_K) + " entries");
    return TQ_E_UNSUPPORTED;
  }
  // Validation, and the token count ahead of every block.
  const uint64_t n_blocks = (n_words + kBlockWords - 1) / kBlockWords;
  if (n_blocks >= (1ull << 31)) {
    set_error("tq_listing_create: stream too long");
    return TQ_E_UNSUPPORTED;
  }
  std::vector<uint32_t> base(std::max<uint64_t>(n_blocks, 1));   // base[b]: tokens that start before word b * kBlockWords
  uint64_t tokens = 0, escapes = 0, values = 0, next_block = 0;
  for (uint64_t i = 0; i < n_words;) {   // a token starts at word i
    while (next_block < n_blocks && next_block * kBlockWords <= i) base[next_block++] = (uint32_t)tokens;
    const uint32_t c = words[i];
    uint64_t len = 1;
    if (c == kMarker) {
      const uint64_t raw = std::min<uint64_t>(kSeq, n_words - 1 - i);
      if (raw == 0) {
        set_error("bad listing stream: marker without values at the end");
        return TQ_E_BAD_BLOB;
      }
      for (uint64_t r = 1; r <= raw; ++r)
        if (words[i + r] > 0xFF) {
          set_error("bad listing stream: raw value above 255 at word " + std::to_string(i + r));
          return TQ_E_BAD_BLOB;
        }
      len = 1 + raw;   // fewer than 4 values only where the stream ends
      values += raw;
      ++escapes;
    } else {
      if (c == 0 || c > n_table) {
        set_error("bad listing stream: codeword " + std::to_string(c) + " at word " + std::to_string(i) + " is not in the table");
        return TQ_E_BAD_BLOB;
      }
      values += kSeq;
    }
    if (++tokens >= (1ull << 32)) {
      set_error("tq_listing_create: 2^32 tokens or more are not supported");
      return TQ_E_UNSUPPORTED;
    }
    i += len;
  }
  while (next_block < n_blocks) base[next_block++] = (uint32_t)tokens;

  std::vector<uint32_t> packed(std::max<uint32_t>(n_table, 1));
  for (uint32_t c = 0; c < n_table; ++c) packed[c] = pack4(table + (size_t)c * kSeq);
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_fail("hipGetDevice (is a GPU present?)", e);
  tq_listing_s* h = new (std::nothrow) tq_listing_s;
  if (!h) {
    set_error("out of host memory");
    return TQ_E_OOM;
  }
  std::memset(h, 0, sizeof *h);
  h->device = dev;
  h->n_blocks = n_blocks;
  h->info.n_values = values;
  h->info.n_words = n_words;
  h->info.n_tokens = tokens;
  h->info.n_escapes = escapes;
  h->info.n_table = n_table;
  e = hipMalloc((void**)&h->words, std::max<uint64_t>(n_words * 2, 4));
  if (e == hipSuccess) e = hipMalloc((void**)&h->table, packed.size() * 4);
  if (e == hipSuccess) e = hipMalloc((void**)&h->block_base, base.size() * 4);
  if (e == hipSuccess && n_words) e = hipMemcpy(h->words, words, n_words * 2, hipMemcpyHostToDevice);
  if (e == hipSuccess) e = hipMemcpy(h->table, packed.data(), packed.size() * 4, hipMemcpyHostToDevice);
  if (e == hipSuccess) e = hipMemcpy(h->block_base, base.data(), base.size() * 4, hipMemcpyHostToDevice);
  if (e != hipSuccess) {
    (void)hipFree(h->words);
    (void)hipFree(h->table);
    (void)hipFree(h->block_base);
    delete h;
    if (e == hipErrorOutOfMemory) {
      set_error("tq_listing_create: out of device memory");
      return TQ_E_OOM;
    }
    return hip_fail("tq_listing_create upload", e);
  }
  *out = h;
  return TQ_OK;
}

extern "C" int tq_listing_create(const uint16_t* words, uint64_t n_words, const uint8_t* table, uint32_t n_table, tq_listing* out) {
  try {   // no C++ exception leaves the library
    return listing_create_impl(words, n_words, table, n_table, out);
  } catch (const std::bad_alloc&) {
    set_error("tq_listing_create: out of host memory");
    return TQ_E_OOM;
  } catch (...) {
    set_error("tq_listing_create: unexpected internal error");
    return TQ_E_HIP;
  }
}

extern "C" int tq_listing_decompress(tq_listing h, void* out, void* stream) {
  if (!h || (!out && h->info.n_values)) {
    set_error("tq_listing_decompress: null argument");
    return TQ_E_INVALID_ARG;
  }
  if (h->n_blocks == 0) return TQ_OK;
  hipLaunchKernelGGL(k_listing_decompress, dim3((unsigned)h->n_blocks), dim3(kListingThreads), 0, (hipStream_t)stream, h->words,
                     h->info.n_words, h->table, h->block_base, (uint8_t*)out);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return hip_fail("tq_listing_decompress launch", e);
  return TQ_OK;
}

extern "C" int tq_listing_get_info(tq_listing h, tq_listing_info* out) {
  if (!h || !out) {
    set_error("tq_listing_get_info: null argument");
    return TQ_E_INVALID_ARG;
  }
  *out = h->info;
  return TQ_OK;
}

extern "C" int tq_listing_destroy(tq_listing h) {
  if (!h) return TQ_OK;
  hipError_t e = hipFree(h->words);
  hipError_t e2 = hipFree(h->table);
  hipError_t e3 = hipFree(h->block_base);
  delete h;
  if (e == hipSuccess) e = e2;
  if (e == hipSuccess) e = e3;
  if (e != hipSuccess) return hip_fail("tq_listing_destroy", e);
  return TQ_OK;
}
