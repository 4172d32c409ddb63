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
//   4. for batches of 2..16 rows and for tq_decompress the lanes append their run bytes to per-lane storage in LDS
//      instead - a ring of 128 bytes (k_matvec_ring: multiplied by bf16 MFMA, batch = N, while the decode goes on) or
//      a strip holding the whole segment (k_matvec_mfma: multiplied when the unit is complete; k_decompress: copied
//      out row-major).
// The expanded matrix never exists in HBM on the tq_matvec path.
// Containers of packed 4-bit weights (two per stored byte) take the same decode; what changes is the dequantization:
// four fp8 weights per dictionary word and two dot products per code at batch 1, nibbles expanded to bf16 ahead of the
// MFMA in the batched kernels, nibbles expanded to int8 in the copy-out of tq_decompress.
#include <hip/hip_runtime.h>

#include <algorithm>
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

namespace tq {

constexpr int kWaves = 8;            // most wavefronts per workgroup of the tile kernels (one workgroup per CU: LDS-bound)
constexpr int kThreads = kWaves * 64;
constexpr int kDotWavesPacked = 12;  // the same kernel for packed 4-bit weights: more work per byte read, more wavefronts to
                                     // hide it (config 4, ms per step: 8 wavefronts 0.379, 12 0.370, 16 0.379)
constexpr int kDotWavesMax = 12;
constexpr int kDotPiecePacked = 6;   // its units are half as long (segments of 128 bytes: 17 chunks, three pieces of 5 or 6)
constexpr int kDotWaves = 8;         // wavefronts per workgroup of the batch-1 kernel (measured on the 3B sweep, TB/s:
                                     // 6 waves 4.61, 8 waves 5.12, 10 waves 4.64, 12 waves 4.90, 16 waves 4.28)
constexpr int kDotPiece = 8;         // chunks per piece in the batch-1 kernel: two pieces (16 x 512 bytes) are in flight per
                                     // wavefront (measured on the 3B sweep, TB/s: 4 chunks 5.30, 6 5.48, 8 5.47, 12 5.41, 18 5.24)
constexpr uint32_t kLdsLimit = 160 * 1024;
constexpr int kPiece = 12;           // code chunks fetched together by a wavefront (units of 256-column segments are
                                     // 33..36 chunks long: three pieces with little repetition)
constexpr int kMaxMulti = 128;       // matrices one launch can serve (bounded by the 4 KB of kernel arguments)
constexpr int kInlineDescriptions = 4;

// What the kernels need to know about one matrix.
struct DevMat {
  const uint32_t* dict;    // container dictionary words (run bytes + length), dict_words of them, zero filled past the pad entry
  const uint32_t* dict_bf16;   // the same entries as two bf16 weights each (second one zero for a single byte): the form the
                               // batch-1 kernel keeps in LDS, made once when the dictionary is uploaded
  const uint32_t* uoff;    // n_units + 1 unit offsets, in chunks
  const uint2* codes;      // chunk c, lane l -> codes[c * 64 + l] (4 codes)
  const float* scales;     // n_bands * 16 row scales
  uint32_t rows, cols, seg_cols;
  uint32_t n_bands, n_quads;
  uint32_t dict_words;     // multiple of 4
  uint32_t x_span;         // dwords per panel in the LDS image of x: seg_cols plus a gap that spreads the 4 panels of a unit over the banks
  uint32_t x_dwords;       // size of that image, including the columns lanes can reach while they consume pad codes
  uint32_t seg_magic;      // floor(2^32 / seg_cols) + 1: col / seg_cols == mulhi(col, seg_magic) for every column index in use
  uint32_t reserved;       // how the ring kernel may decode the matrix: 0 not at all, 1 in groups of windows, 2 window by window
  uint32_t packing;        // 1: every byte holds two 4-bit weights (columns 2j and 2j + 1 of a matrix of 2 * cols columns); rows,
                           // cols and seg_cols describe the byte matrix, and dict_bf16 holds four fp8 (e4m3) weights per entry
};

struct Job {
  const DevMat* m;         // device copy of the matrix description
  const uint16_t* x;       // bf16 [batch][cols]
  float* y;                // fp32 [batch][rows]
};

// A job together with its matrix description, as a prepared step keeps them in device memory.
struct StepEntry {
  DevMat m;
  const uint16_t* x;
  float* y;
};
constexpr int kMaxStep = 896;        // matrices one launch can serve when the jobs come from a device table

// The launch's cost line: matrix i covers [cost[i], cost[i + 1]), one band of it costs its number of columns.
// The jobs travel in the kernel arguments (up to kMaxMulti of them) or, for a prepared step, sit in a table in device
// memory (up to kMaxStep); the cost line is in the arguments either way, at the same place.
struct MatvecArgs {
  int n, batch;
  uint32_t x_off, slot_off;   // byte offsets in LDS of the activation image (or of the tiles) and of the partial-sum slots
  uint32_t tile_area;         // bytes of LDS per wavefront in the tile kernels (the same for every matrix of the launch)
  uint32_t gate_up;           // 1: rows 2r and 2r + 1 are a gate and an up projection; y[b][r] = silu(row 2r) * (row 2r + 1)
  const StepEntry* table;     // device table of the n jobs, or null: then j and first below hold them
  union {
    struct {
      uint32_t cost[kMaxMulti + 1];
      Job j[kMaxMulti];
      DevMat first[kInlineDescriptions];   // descriptions of the first matrices by value: a launch of one matrix (or of a
                                           // few) does not wait for a read of device memory before it can start loading
    } in;
    uint32_t cost_long[kMaxStep + 1];
  } u;
};
static_assert(sizeof(MatvecArgs) <= 4096, "kernel arguments");

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(3))) const uint32_t lds_cu32;
typedef __attribute__((address_space(3))) const uint16_t lds_cu16;
typedef __attribute__((address_space(3))) uint8_t lds_u8;
typedef __attribute__((address_space(4))) const uint32_t const_u32;

template <int... I, typename F>
__device__ __forceinline__ void static_for_impl(std::integer_sequence<int, I...>, F&& f) {
  (f(std::integral_constant<int, I>{}), ...);
}
template <int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  static_for_impl(std::make_integer_sequence<int, N>{}, f);
}

// Unit offsets are wave-uniform and never written while a kernel runs: reading them through the constant address
// space makes them scalar loads, which do not share a counter with the vector loads of the code stream.
__device__ __forceinline__ uint32_t unit_offset(const DevMat& m, uint32_t u) { return ((const_u32*)m.uoff)[u]; }

// Loads and stores of device memory through the global address space.  Pointers that come out of a matrix description
// read from memory are generic to the compiler; a generic access is a flat instruction, which counts on the LDS counter
// as well as on the vector-memory one and so would make every LDS wait a wait for the code stream too.
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
// Chunk `chunk` of the code stream, lane's 4 codes: a wave-uniform base in scalar registers plus the lane's offset, so
// that no vector arithmetic goes into the address.
__device__ __forceinline__ uint2 load_chunk(const uint2* codes, uint32_t chunk, int lane) {
  const uint64_t base = (uint64_t)codes + (uint64_t)chunk * (64 * sizeof(uint2));
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)base), hi = __builtin_amdgcn_readfirstlane((uint32_t)(base >> 32));
  const u32x2 v = ((__attribute__((address_space(1))) const u32x2*)((uint64_t)hi << 32 | lo))[(uint32_t)lane];
  return make_uint2(v.x, v.y);
}

__device__ __forceinline__ uint2 global_load(const uint2* p) {
  const u32x2 v = *(__attribute__((address_space(1))) const u32x2*)p;
  return make_uint2(v.x, v.y);
}
__device__ __forceinline__ uint4 global_load(const uint4* p) {
  const u32x4 v = *(__attribute__((address_space(1))) const u32x4*)p;
  return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ uint32_t global_load(const uint32_t* p) { return *(__attribute__((address_space(1))) const uint32_t*)p; }
__device__ __forceinline__ uint32_t global_load(const uint16_t* p) { return *(__attribute__((address_space(1))) const uint16_t*)p; }
__device__ __forceinline__ float global_load(const float* p) { return *(__attribute__((address_space(1))) const float*)p; }
__device__ __forceinline__ void global_store(float* p, float v) { *(__attribute__((address_space(1))) float*)p = v; }

// A matrix description from device memory, through scalar loads.
__device__ __forceinline__ DevMat load_description(const DevMat* p) {
  static_assert(sizeof(DevMat) % 4 == 0, "whole dwords");
  uint32_t w[sizeof(DevMat) / 4];
#pragma unroll
  for (size_t k = 0; k < sizeof(DevMat) / 4; ++k) w[k] = ((const_u32*)p)[k];
  DevMat m;
  __builtin_memcpy(&m, w, sizeof m);
  return m;
}

// Point i of the launch's cost line (the two forms of the arguments keep it at the same place).
__device__ __forceinline__ uint32_t cost_at(const MatvecArgs& a, int i) { return a.u.cost_long[i]; }

// Job i of the launch and the description of its matrix: from the kernel arguments, or from the step's device table
// (scalar loads, like the descriptions the arguments do not hold by value).
__device__ __forceinline__ void fetch_job(const MatvecArgs& a, int i, Job& job, DevMat& m) {
  if (a.table) {
    const StepEntry* e = a.table + i;
    static_assert(sizeof(StepEntry) % 4 == 0, "whole dwords");
    uint32_t w[sizeof(StepEntry) / 4];
#pragma unroll
    for (size_t k = 0; k < sizeof(StepEntry) / 4; ++k) w[k] = ((const_u32*)e)[k];
    StepEntry v;
    __builtin_memcpy(&v, w, sizeof v);
    m = v.m;
    job.m = &e->m;
    job.x = v.x;
    job.y = v.y;
  } else {
    job = a.u.in.j[i];
    m = i < kInlineDescriptions ? a.u.in.first[i] : load_description(job.m);
  }
}

// Byte address inside LDS of a pointer into the workgroup's dynamic shared memory.
__device__ __forceinline__ uint32_t lds_address(const void* p) { return (uint32_t)(size_t)(const lds_u8*)p; }

// Pointer forms on purpose: the compiler tracks the outstanding LDS read and places the wait before the first use.
__device__ __forceinline__ uint32_t lds_read32(uint32_t addr) { return *(lds_cu32*)(size_t)addr; }
template <int kOff>
__device__ __forceinline__ uint32_t lds_read32_off(uint32_t addr) { return *(lds_cu32*)(size_t)(addr + kOff); }

// Byte offset of dictionary word `code` for the code in the low / high half of a packed code pair: one SDWA shift
// (selects the 16-bit half, zero-extends, multiplies by 4) instead of a mask and a shift.
__device__ __forceinline__ uint32_t word_offset_lo(uint32_t pair) {
  uint32_t a;
  const uint32_t two = 2;
  asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_0" : "=v"(a) : "v"(two), "v"(pair));
  return a;
}
__device__ __forceinline__ uint32_t word_offset_hi(uint32_t pair) {
  uint32_t a;
  const uint32_t two = 2;
  asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_1" : "=v"(a) : "v"(two), "v"(pair));
  return a;
}
// min(1, high byte of the low / high code): 1 for a two-weight entry (code >= 256, the pad code included), 0 for a single
__device__ __forceinline__ uint32_t is_pair_lo(uint32_t pair) {
  uint32_t a;
  const uint32_t one = 1;
  asm("v_min_u32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_1" : "=v"(a) : "v"(one), "v"(pair));
  return a;
}
__device__ __forceinline__ uint32_t is_pair_hi(uint32_t pair) {
  uint32_t a;
  const uint32_t one = 1;
  asm("v_min_u32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_3" : "=v"(a) : "v"(one), "v"(pair));
  return a;
}
__device__ __forceinline__ float dot2(uint32_t w, uint32_t x, float acc) {
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, w), __builtin_bit_cast(bf16x2, x), acc, false);
}

// Staging is split in two so that the loads of the dictionary, of the activations and of the first code chunks are
// all in flight together before anything waits: issue_* only loads into registers, commit_* writes LDS.
constexpr int kDictRegs = 16;   // uint4 per thread per round of the tile kernels' dictionary staging

template <int kThreads, int kDictRegs>   // kDictRegs x kThreads x 16 bytes per round (128 KB: the whole dictionary in one)
__device__ __forceinline__ void issue_dictionary(const DevMat& m, uint32_t base, int tid, uint4 (&v)[kDictRegs]) {
  const uint4* src = (const uint4*)m.dict_bf16;
  const uint32_t n4 = m.dict_words / 4;
#pragma unroll
  for (int k = 0; k < kDictRegs; ++k) v[k] = global_load(src + min(base + k * kThreads + tid, n4 - 1));
}
template <int kThreads, int kDictRegs>
__device__ __forceinline__ void commit_dictionary(const DevMat& m, uint32_t base, int tid, const uint4 (&v)[kDictRegs], uint32_t* lds_dict) {
  uint4* dst = (uint4*)lds_dict;
  const uint32_t n4 = m.dict_words / 4;
#pragma unroll
  for (int k = 0; k < kDictRegs; ++k) {
    const uint32_t i = base + k * kThreads + tid;
    if (i < n4) dst[i] = v[k];
  }
}

// LDS image of one activation row: dword (panel * x_span + c) = (x[panel * seg_cols + c], x[panel * seg_cols + c + 1])
// as two bf16, zero past the end of the row; the gap dwords between panels and the tail are zero.
// Thread t of a round handles the column pair (2 j, 2 j + 1), j = first_pair + k * 512 + t: it loads x[2j .. 2j+2].
template <bool kAligned, int kThreads, int kXRegs>   // kXRegs x kThreads x 2 columns per round (8192)
__device__ __forceinline__ void issue_activations(const DevMat& m, const uint16_t* __restrict__ x, uint32_t first_pair, int tid,
                                                  uint32_t (&lo)[kXRegs], uint32_t (&hi)[kXRegs]) {
#pragma unroll
  for (int k = 0; k < kXRegs; ++k) {
    const uint32_t j = first_pair + k * kThreads + tid, col = 2 * j;
    if (kAligned) {   // x is 4-byte aligned and cols is even
      lo[k] = col < m.cols ? global_load((const uint32_t*)x + j) : 0u;
      hi[k] = col + 2 < m.cols ? global_load((const uint32_t*)x + j + 1) : 0u;
    } else {
      lo[k] = (col < m.cols ? global_load(x + col) : 0u) | (col + 1 < m.cols ? global_load(x + col + 1) << 16 : 0u);
      hi[k] = col + 2 < m.cols ? global_load(x + col + 2) : 0u;
    }
  }
}
template <int kThreads, int kXRegs>
__device__ __forceinline__ void commit_activations(const DevMat& m, uint32_t first_pair, int tid, const uint32_t (&lo)[kXRegs],
                                                   const uint32_t (&hi)[kXRegs], uint32_t* lds_x, uint32_t image_cols) {
  const uint32_t gap = m.x_span - m.seg_cols;
#pragma unroll
  for (int k = 0; k < kXRegs; ++k) {
    const uint32_t col = 2 * (first_pair + k * kThreads + tid);
    if (col < image_cols) {   // image_cols and seg_cols are even: both dwords of the pair lie in one panel
      const uint32_t i = col + gap * __umulhi(col, m.seg_magic);
      lds_x[i] = lo[k];
      lds_x[i + 1] = lo[k] >> 16 | hi[k] << 16;
    }
  }
}
template <int kThreads>
__device__ __forceinline__ void zero_activation_gaps(const DevMat& m, int tid, uint32_t* lds_x, uint32_t n_slots) {
  const uint32_t gap = m.x_span - m.seg_cols;
  if (gap)   // gap is 16 dwords
    for (uint32_t i = tid; i < n_slots * 16; i += kThreads) lds_x[(i >> 4) * m.x_span + m.seg_cols + (i & 15)] = 0u;
  for (uint32_t i = n_slots * m.x_span + tid; i < m.x_dwords; i += kThreads) lds_x[i] = 0u;
}

// One chunk = 4 codes per lane.  xa = LDS byte address of the activation pair of the lane's next code, minus 4 bytes
// per code consumed since the start of the piece; code k of the piece therefore reads at xa + 4 k, and the constant
// part goes into the instruction's offset field.  A single advances the lane by one column (already counted by the
// 4 k), a pair by one more.  The dictionary sits at LDS address 0, so a code's word offset is its address.
// Per chunk and lane: 4 dictionary words, 4 activation pairs, 4 v_dot2_f32_bf16 into two accumulators.
// xa + 4 * pair as one instruction.  Written out because the compiler otherwise keeps a running count of the pairs and
// forms every address from it with a second instruction: a shorter dependency chain, but a quarter more vector
// instructions per code.
__device__ __forceinline__ uint32_t advance_by_pair(uint32_t pair, uint32_t xa) {
  uint32_t r;
  asm("v_lshl_add_u32 %0, %1, 2, %2" : "=v"(r) : "v"(pair), "v"(xa));
  return r;
}

// In two halves, so that the reads of the next chunk can be issued ahead of the dot products of this one (left to
// itself the compiler finishes a chunk before it requests anything of the next: one LDS round trip per chunk that a
// wavefront with few neighbours cannot hide).
template <int kCode0>
__device__ __forceinline__ void chunk4_read(uint2 c, uint32_t& xa, uint32_t (&w)[4], uint32_t (&x)[8]) {
  w[0] = lds_read32(word_offset_lo(c.x));
  w[1] = lds_read32(word_offset_hi(c.x));
  w[2] = lds_read32(word_offset_lo(c.y));
  w[3] = lds_read32(word_offset_hi(c.y));
  x[0] = lds_read32_off<4 * kCode0>(xa);
  xa = advance_by_pair(is_pair_lo(c.x), xa);
  x[1] = lds_read32_off<4 * kCode0 + 4>(xa);
  xa = advance_by_pair(is_pair_hi(c.x), xa);
  x[2] = lds_read32_off<4 * kCode0 + 8>(xa);
  xa = advance_by_pair(is_pair_lo(c.y), xa);
  x[3] = lds_read32_off<4 * kCode0 + 12>(xa);
  xa = advance_by_pair(is_pair_hi(c.y), xa);
}
__device__ __forceinline__ void chunk4_dot(const uint32_t (&w)[4], const uint32_t (&x)[8], float& a0, float& a1) {
  a0 = dot2(w[0], x[0], a0);
  a1 = dot2(w[1], x[1], a1);
  a0 = dot2(w[2], x[2], a0);
  a1 = dot2(w[3], x[3], a1);
}

// The same for a matrix of packed 4-bit weights.  A dictionary word holds the entry's four weights as fp8 (e4m3 holds
// -8..7 exactly; two zeros after a single byte), one activation dword holds the two columns of a byte: code k reads the
// dwords at xa + 4 k and the next one, and two conversions give the bf16 pairs for two dot products.
__device__ __forceinline__ float dot2_fp8(uint32_t w, bool high, uint32_t x, float acc) {
  const bf16x2 wb = high ? __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w, 1.0f, true) : __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w, 1.0f, false);
  return __builtin_amdgcn_fdot2_f32_bf16(wb, __builtin_bit_cast(bf16x2, x), acc, false);
}
template <int kCode0>
__device__ __forceinline__ void chunk4_packed_read(uint2 c, uint32_t& xa, uint32_t (&w)[4], uint32_t (&x)[8]) {
  w[0] = lds_read32(word_offset_lo(c.x));
  w[1] = lds_read32(word_offset_hi(c.x));
  w[2] = lds_read32(word_offset_lo(c.y));
  w[3] = lds_read32(word_offset_hi(c.y));
  x[0] = lds_read32_off<4 * kCode0>(xa);
  x[1] = lds_read32_off<4 * kCode0 + 4>(xa);
  xa = advance_by_pair(is_pair_lo(c.x), xa);
  x[2] = lds_read32_off<4 * kCode0 + 4>(xa);
  x[3] = lds_read32_off<4 * kCode0 + 8>(xa);
  xa = advance_by_pair(is_pair_hi(c.x), xa);
  x[4] = lds_read32_off<4 * kCode0 + 8>(xa);
  x[5] = lds_read32_off<4 * kCode0 + 12>(xa);
  xa = advance_by_pair(is_pair_lo(c.y), xa);
  x[6] = lds_read32_off<4 * kCode0 + 12>(xa);
  x[7] = lds_read32_off<4 * kCode0 + 16>(xa);
  xa = advance_by_pair(is_pair_hi(c.y), xa);
}
__device__ __forceinline__ void chunk4_packed_dot(const uint32_t (&w)[4], const uint32_t (&x)[8], float& a0, float& a1) {
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    a0 = dot2_fp8(w[k], false, x[2 * k], a0);
    a1 = dot2_fp8(w[k], true, x[2 * k + 1], a1);
  }
}

// LDS image of one activation row for packed weights: dword (panel * x_span + c) = the two activations of byte column
// panel * seg_cols + c, zero past the end of the row.  Thread t of a round handles dword first + k * kThreads + t.
template <bool kAligned, int kThreads, int kXRegs>
__device__ __forceinline__ void issue_activations_packed(const DevMat& m, const uint16_t* __restrict__ x, uint32_t first, int tid,
                                                         uint32_t (&v)[kXRegs]) {
#pragma unroll
  for (int k = 0; k < kXRegs; ++k) {
    const uint32_t j = first + k * kThreads + tid;
    if (kAligned) v[k] = j < m.cols ? global_load((const uint32_t*)x + j) : 0u;   // x is 4-byte aligned
    else v[k] = j < m.cols ? global_load(x + 2 * j) | global_load(x + 2 * j + 1) << 16 : 0u;
  }
}
template <int kThreads, int kXRegs>
__device__ __forceinline__ void commit_activations_packed(const DevMat& m, uint32_t first, int tid, const uint32_t (&v)[kXRegs], uint32_t* lds_x,
                                                          uint32_t image_cols) {
  const uint32_t gap = m.x_span - m.seg_cols;
#pragma unroll
  for (int k = 0; k < kXRegs; ++k) {
    const uint32_t j = first + k * kThreads + tid;
    if (j < image_cols) lds_x[j + gap * __umulhi(j, m.seg_magic)] = v[k];
  }
}

// Sum of the four panel lanes of each row: afterwards every lane l holds the sum over lanes l % 16 + {0, 16, 32, 48}.
__device__ __forceinline__ float sum_over_panels(float v) {
  v += __shfl_xor(v, 16);
  v += __shfl_xor(v, 32);
  return v;
}

// The gated product of a feed-forward block: silu(gate) * up, silu(g) = g / (1 + exp(-g)).
__device__ __forceinline__ float silu_times(float gate, float up) { return gate / (1.f + __expf(-gate)) * up; }

// Fused decode + dequantize + matrix-vector product for one activation row and up to kMaxMulti matrices.
//
// The launch's work is the line of all bands (16 rows each) of all matrices, each band weighted by its number of
// weights; workgroup g takes the bands whose middle lies in the g-th equal share of that line, so a workgroup serves a
// contiguous range of whole bands of one matrix after the other.  Inside a matrix the units of those bands are
// contiguous in the code stream and are cut into one contiguous run per wavefront.  A wavefront owns every band that
// lies entirely inside its run (it scales and stores those rows itself); a band it shares with its neighbours goes to
// one of two partial-sum slots in LDS, and after a workgroup barrier the slots of a band are added in wavefront order,
// so the result does not depend on timing.
template <int kPiece, int kWaves, bool kPacked>
__global__ __launch_bounds__(kWaves * 64, 1) void k_matvec(MatvecArgs a) {
  constexpr int kThreads = kWaves * 64, kDictRegs = 128 / kWaves, kXRegs = 64 / kWaves;
  extern __shared__ uint4 lds4[];
  uint32_t* lds_dict = (uint32_t*)lds4;
  uint32_t* lds_x = (uint32_t*)((uint8_t*)lds4 + a.x_off);
  float* slot_val = (float*)((uint8_t*)lds4 + a.slot_off);           // [2 * kWaves][16]
  int* slot_band = (int*)(slot_val + 2 * kWaves * 16);               // [2 * kWaves]
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  if (lds_address(lds4) != 0) return;   // the code -> word lookup takes the dictionary to start at LDS address 0 (no static LDS here)
  const uint64_t total = cost_at(a, a.n);
  const uint32_t lo = (uint32_t)(total * blockIdx.x / gridDim.x), hi = (uint32_t)(total * (blockIdx.x + 1) / gridDim.x);
  const uint32_t* staged = nullptr;
  for (int i = 0; i < a.n; ++i) {
    const uint32_t cb = cost_at(a, i), ce = cost_at(a, i + 1);
    if (hi <= cb || lo >= ce) continue;
    Job job;
    DevMat m;
    fetch_job(a, i, job, m);
    // a band goes to the share that holds its middle
    const uint32_t bc = m.cols;
    const uint32_t band_lo = lo <= cb ? 0u : (lo - cb + bc / 2) / bc;
    const uint32_t band_hi = hi >= ce ? m.n_bands : min(m.n_bands, (hi - cb + bc / 2) / bc);
    if (band_lo >= band_hi) continue;
    const bool new_dict = m.dict_bf16 != staged;
    staged = m.dict_bf16;
    const uint32_t nq = m.n_quads, n_slots = nq * kUnitPanels, image_cols = n_slots * m.seg_cols;
    const uint32_t unit_lo = band_lo * nq, n_units = (band_hi - band_lo) * nq;
    const uint32_t u0 = unit_lo + (uint32_t)((uint64_t)n_units * wave / kWaves);
    const uint32_t u1 = unit_lo + (uint32_t)((uint64_t)n_units * (wave + 1) / kWaves);
    // lane's panel inside a unit is lane >> 4; quad q adds 4 q panels
    const uint32_t xa_lane = lds_address(lds_x) + 4u * m.x_span * (uint32_t)(lane >> 4);
    const uint32_t xa_quad = 16u * m.x_span;
    const bool x_aligned = (kPacked || m.cols % 2 == 0) && ((uintptr_t)job.x % 4 == 0);
    const uint32_t c0 = u0 < u1 ? unit_offset(m, u0) : 0u, n_chunks = u0 < u1 ? unit_offset(m, u1) - c0 : 0u;
    {   // one activation row: larger batches run the MFMA kernel
      const uint16_t* xb = job.x;
      float* yb = job.y;
      __syncthreads();   // the previous dictionary, activation image and slots are no longer in use
      {
        uint4 dv[kDictRegs];
        uint32_t xlo[kXRegs], xhi[kXRegs];
        const bool dict_now = new_dict;
        if (dict_now) issue_dictionary<kThreads, kDictRegs>(m, 0, tid, dv);
        if constexpr (kPacked) {
          if (x_aligned) issue_activations_packed<true, kThreads, kXRegs>(m, xb, 0, tid, xlo);
          else issue_activations_packed<false, kThreads, kXRegs>(m, xb, 0, tid, xlo);
        } else {
          if (x_aligned) issue_activations<true, kThreads, kXRegs>(m, xb, 0, tid, xlo, xhi);
          else issue_activations<false, kThreads, kXRegs>(m, xb, 0, tid, xlo, xhi);
        }
        zero_activation_gaps<kThreads>(m, tid, lds_x, n_slots);
        if (tid < 2 * kWaves) slot_band[tid] = -1;
        if (dict_now) {
          commit_dictionary<kThreads, kDictRegs>(m, 0, tid, dv, lds_dict);
          for (uint32_t base = kDictRegs * kThreads; base < m.dict_words / 4; base += kDictRegs * kThreads) {
            issue_dictionary<kThreads, kDictRegs>(m, base, tid, dv);
            commit_dictionary<kThreads, kDictRegs>(m, base, tid, dv, lds_dict);
          }
        }
        if constexpr (kPacked) {
          commit_activations_packed<kThreads, kXRegs>(m, 0, tid, xlo, lds_x, image_cols);
          for (uint32_t first = kXRegs * kThreads; first < image_cols; first += kXRegs * kThreads) {
            if (x_aligned) issue_activations_packed<true, kThreads, kXRegs>(m, xb, first, tid, xlo);
            else issue_activations_packed<false, kThreads, kXRegs>(m, xb, first, tid, xlo);
            commit_activations_packed<kThreads, kXRegs>(m, first, tid, xlo, lds_x, image_cols);
          }
        } else {
          commit_activations<kThreads, kXRegs>(m, 0, tid, xlo, xhi, lds_x, image_cols);
          for (uint32_t first = kXRegs * kThreads; 2 * first < image_cols; first += kXRegs * kThreads) {
            if (x_aligned) issue_activations<true, kThreads, kXRegs>(m, xb, first, tid, xlo, xhi);
            else issue_activations<false, kThreads, kXRegs>(m, xb, first, tid, xlo, xhi);
            commit_activations<kThreads, kXRegs>(m, first, tid, xlo, xhi, lds_x, image_cols);
          }
        }
      }
      __syncthreads();
      if (u0 < u1) {
        uint32_t q = u0 % nq, band = u0 / nq;
        bool whole = q == 0;                             // the current band started inside this wavefront's run
        float a0 = 0.f, a1 = 0.f;
        uint32_t xa = xa_lane + q * xa_quad;
        // the scales of the band in work are requested when the band starts (the array is padded to whole bands)
        float scale = global_load(m.scales + band * kUnitRows + (lane & 15));
        auto finish_band = [&](bool complete) {
          const float v = sum_over_panels(a0 + a1);
          if (complete) {
            const uint32_t row = band * kUnitRows + lane;
            if (a.gate_up) {   // lanes 2r, 2r + 1 hold the gate and the up row of output r
              const float t = v * scale, other = __shfl_xor(t, 1);
              if (lane < 16 && !(lane & 1) && row + 1 < m.rows) global_store(yb + row / 2, silu_times(t, other));
            } else if (lane < 16 && row < m.rows) {
              global_store(yb + row, v * scale);
            }
          } else {
            const int s = 2 * wave + (whole ? 1 : 0);   // slot 2w: band begun by an earlier wavefront; 2w + 1: band left unfinished
            if (lane < 16) slot_val[s * 16 + lane] = v;
            if (lane == 0) slot_band[s] = (int)band;
          }
        };
        // The chunks of the run come in pieces of at most kPiece that never straddle a unit (a unit is cut into equal
        // pieces); two register sets alternate and every piece issues exactly kPiece loads (those past its end repeat
        // its last chunk), so the loads of the next piece are in flight while this one is worked on.  A piece of kPiece
        // or kPiece - 1 chunks (all pieces of a unit of 256-column segments) runs as straight-line code: the LDS reads
        // of later chunks overlap the dot products of earlier ones.
        uint32_t wu = u0, wc = c0, w_left = 0, w_base = 0, w_rem = 0;
        auto next_piece = [&](uint32_t& start, uint32_t& n, bool& ends) {
          if (w_left == 0) {
            if (wu == u1) {
              n = 0;
              ends = false;
              start = wc;
              return;
            }
            const uint32_t len = unit_offset(m, wu + 1) - wc;
            w_left = (len + kPiece - 1) / kPiece;
            w_base = len / w_left;
            w_rem = len - w_base * w_left;
            ++wu;
          }
          n = w_base + (w_rem ? 1u : 0u);
          if (w_rem) --w_rem;
          start = wc;
          wc += n;
          ends = --w_left == 0;
        };
        const uint32_t run_last = c0 + n_chunks - 1;
        auto load_piece = [&](uint2 (&cw)[kPiece], uint32_t start, uint32_t n) {
          const uint32_t last = min(start + max(n, 1u) - 1, run_last);
#pragma unroll
          for (int k = 0; k < kPiece; ++k) cw[k] = load_chunk(m.codes, min(start + k, last), lane);
        };
        auto run_piece = [&](const uint2 (&cw)[kPiece], uint32_t n, bool ends) {
          uint32_t w[2][4], x[2][8];   // two register sets: one chunk's operands are read while the one before is multiplied
          auto read = [&](auto kk) {
            constexpr int k = decltype(kk)::value;
            if constexpr (kPacked) chunk4_packed_read<4 * k>(cw[k], xa, w[k & 1], x[k & 1]);
            else chunk4_read<4 * k>(cw[k], xa, w[k & 1], x[k & 1]);
          };
          auto dot = [&](auto kk) {
            constexpr int k = decltype(kk)::value;
            if constexpr (kPacked) chunk4_packed_dot(w[k & 1], x[k & 1], a0, a1);
            else chunk4_dot(w[k & 1], x[k & 1], a0, a1);
          };
          auto straight = [&](auto nn) {   // a piece of nn chunks as straight-line code
            constexpr int kN = decltype(nn)::value;
            read(std::integral_constant<int, 0>{});
            static_for<kN>([&](auto kk) {
              constexpr int k = decltype(kk)::value;
              if constexpr (k + 1 < kN) read(std::integral_constant<int, k + 1>{});
              dot(kk);
            });
          };
          if (n == kPiece) {
            straight(std::integral_constant<int, kPiece>{});
          } else if (n == kPiece - 1) {
            straight(std::integral_constant<int, kPiece - 1>{});
          } else if (n == kPiece - 2) {
            straight(std::integral_constant<int, kPiece - 2>{});
          } else {
            static_for<kPiece>([&](auto kk) {
              if ((uint32_t)decltype(kk)::value < n) {
                read(kk);
                dot(kk);
              }
            });
          }
          xa += 16 * n;
          if (ends) {   // every lane restarts at the first column of its next segment
            if (++q == nq) {
              const bool more = band * nq + nq < u1;
              finish_band(whole);
              q = 0;
              ++band;
              if (more) scale = global_load(m.scales + band * kUnitRows + (lane & 15));
              whole = true;
              a0 = 0.f;
              a1 = 0.f;
            }
            xa = xa_lane + q * xa_quad;
          }
        };
        uint2 cwa[kPiece], cwb[kPiece];
        uint32_t sa, na, sb, nb;
        bool ea, eb;
        next_piece(sa, na, ea);
        load_piece(cwa, sa, na);
        while (na) {
          next_piece(sb, nb, eb);
          load_piece(cwb, sb, nb);
          run_piece(cwa, na, ea);
          next_piece(sa, na, ea);
          load_piece(cwa, sa, na);
          run_piece(cwb, nb, eb);
        }
        if (u1 % nq) finish_band(false);   // the run ends inside a band (a band that ends with the run was finished above)
      }
      __syncthreads();
      // Combine the shared bands: the first slot of a band adds the later slots of the same band in slot order.
      if (tid < 2 * kWaves * 16) {
        const int s = tid >> 4, r16 = tid & 15;
        const int bnd = slot_band[s];
        bool first = bnd >= 0;
        for (int t = 0; t < s; ++t) first = first && slot_band[t] != bnd;
        if (first) {
          float sum = slot_val[s * 16 + r16];
          for (int t = s + 1; t < 2 * kWaves; ++t)
            if (slot_band[t] == bnd) sum += slot_val[t * 16 + r16];
          const uint32_t row = (uint32_t)bnd * kUnitRows + r16;
          if (a.gate_up) {   // the two threads of a pair of rows are neighbours and take this branch together
            const float t = sum * global_load(m.scales + min(row, m.rows - 1)), other = __shfl_xor(t, 1);
            if (!(r16 & 1) && row + 1 < m.rows) global_store(yb + row / 2, silu_times(t, other));
          } else if (row < m.rows) {
            global_store(yb + row, sum * global_load(m.scales + row));
          }
        }
      }
    }
  }
}

// ---------------------------------------------------------------------------------------------------------------
// Product for batches of 2..16 activation rows, whole-strip form: decode a unit into an LDS tile, then bf16 MFMA with
// the batch as N.  (Large launches of well-behaved matrices take the ring form further down instead.)
//
// A lane's segment is (row l & 15, panel l >> 4) of its unit, which is exactly the A-operand layout of
// v_mfma_f32_16x16x32_bf16: lane l supplies row l % 16 and the 8 k-values of group l / 16.  Taking those 8 values as
// 8 consecutive columns of the lane's own segment makes every lane read back only what it wrote itself: the tile is a
// per-lane strip of seg_cols (+8) bytes, a lane appends the bytes of its runs (packed in registers, one aligned 8-byte
// store per chunk), and after the unit's last chunk window w of
// the unit is one MFMA: A = bytes [8 w, 8 w + 8) of every strip converted to bf16 (exact), B = the activations of the
// 4 x 8 columns those bytes stand for, one batch row per lane % 16.  Strips of shorter or empty segments hold stale
// (finite) values past their end; they meet activations that are zero there because B is loaded with bounds checks.

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) const u32x2 lds_cu64;

// Byte offset of the 16-bit dictionary entry of the code in the low / high half of a packed code pair.
__device__ __forceinline__ uint32_t half_offset_lo(uint32_t pair) {
  uint32_t a;
  const uint32_t one = 1;
  asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_0" : "=v"(a) : "v"(one), "v"(pair));
  return a;
}
__device__ __forceinline__ uint32_t half_offset_hi(uint32_t pair) {
  uint32_t a;
  const uint32_t one = 1;
  asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_1" : "=v"(a) : "v"(one), "v"(pair));
  return a;
}
__device__ __forceinline__ uint32_t lds_read16(uint32_t addr) { return *(lds_cu16*)(size_t)addr; }

// 8 int8 -> 8 bf16 (exact: |v| <= 128 needs 8 significant bits).  bf16 = upper half of the fp32 encoding.
__device__ __forceinline__ bf16x8 i8x8_to_bf16x8(uint2 w) {
  uint4 r;
  {
    float f0 = (float)(int8_t)(w.x), f1 = (float)(int8_t)(w.x >> 8), f2 = (float)(int8_t)(w.x >> 16), f3 = (float)(int8_t)(w.x >> 24);
    r.x = __builtin_amdgcn_perm(__float_as_uint(f1), __float_as_uint(f0), 0x07060302u);
    r.y = __builtin_amdgcn_perm(__float_as_uint(f3), __float_as_uint(f2), 0x07060302u);
  }
  {
    float f0 = (float)(int8_t)(w.y), f1 = (float)(int8_t)(w.y >> 8), f2 = (float)(int8_t)(w.y >> 16), f3 = (float)(int8_t)(w.y >> 24);
    r.z = __builtin_amdgcn_perm(__float_as_uint(f1), __float_as_uint(f0), 0x07060302u);
    r.w = __builtin_amdgcn_perm(__float_as_uint(f3), __float_as_uint(f2), 0x07060302u);
  }
  return __builtin_bit_cast(bf16x8, r);
}

// 8 packed 4-bit weights (a dword: byte j holds columns 2j in bits 0..3 and 2j + 1 in bits 4..7, two's complement)
// -> 8 bf16 in column order (exact).
__device__ __forceinline__ bf16x8 nib8_to_bf16x8(uint32_t d) {
  uint32_t r[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    // (the builtin's result type is unsigned: without the casts -1 would convert as 2^32 - 1)
    const float lo = (float)(int)__builtin_amdgcn_sbfe(d, 8 * j, 4), hi = (float)(int)__builtin_amdgcn_sbfe(d, 8 * j + 4, 4);
    r[j] = __builtin_amdgcn_perm(__float_as_uint(hi), __float_as_uint(lo), 0x07060302u);
  }
  return __builtin_bit_cast(bf16x8, make_uint4(r[0], r[1], r[2], r[3]));
}

// Append the runs of one chunk (4 codes) to the lane's strip.  The 4 entries (1 or 2 bytes each; the length follows
// from the code) are packed into one string of up to 8 bytes in registers, joined to the bytes the lane has not
// written yet (`carry`: the pos % 8 bytes after its last complete 8-byte piece), and one aligned 8-byte piece goes to
// LDS when it is complete: one store per chunk instead of one per byte.  pos = bytes of the segment appended so far.
// Pad codes (entry 0, counted as 2 bytes by the code test) only follow a complete segment: the clamp against the
// bytes still missing drops them.
typedef __attribute__((address_space(3))) uint64_t lds_u64;
__device__ __forceinline__ void append_chunk(uint2 c, uint32_t strip, uint32_t seg_len, uint32_t& pos, uint64_t& carry) {
  const uint32_t e0 = lds_read16(half_offset_lo(c.x)), e1 = lds_read16(half_offset_hi(c.x));
  const uint32_t e2 = lds_read16(half_offset_lo(c.y)), e3 = lds_read16(half_offset_hi(c.y));
  const uint32_t p0 = is_pair_lo(c.x), p1 = is_pair_hi(c.x), p2 = is_pair_lo(c.y), p3 = is_pair_hi(c.y);
  const uint32_t a01 = e1 << ((p0 << 3) + 8) | e0, n01 = p0 + p1 + 2;   // codes 0, 1: n01 = 2..4 bytes
  const uint32_t a23 = e3 << ((p2 << 3) + 8) | e2, n23 = p2 + p3 + 2;   // codes 2, 3
  const uint32_t t = (n01 << 3) - 8;                                    // 8, 16, 24: a23 starts 8 + t bits into the string
  const uint32_t s0 = (a23 << t) << 8 | a01, s1 = a23 >> (24 - t);
  const uint64_t str = (uint64_t)s1 << 32 | s0;
  const uint32_t n = min(n01 + n23, seg_len - pos);
  const uint32_t f = pos & 7u, sh = f << 3;
  const uint64_t lo = carry | str << sh, hi = (str >> 1) >> (63 - sh);  // the 16 bytes carry + string; hi is 0 for f == 0
  const bool full = f + n >= 8;
  if (full) *(lds_u64*)(size_t)(strip + (pos & ~7u)) = lo;
  carry = full ? hi : lo;
  pos += n;
}
// The bytes after the last complete 8-byte piece (a segment whose length is not a multiple of 8).
__device__ __forceinline__ void flush_carry(uint32_t strip, uint32_t pos, uint64_t carry) {
  if (pos & 7u) *(lds_u64*)(size_t)(strip + (pos & ~7u)) = carry;
}

// Decode the units [u0, u1) of a matrix, one after the other, into the strips of this wavefront's tile and call
// on_unit(band, quad) each time the tile holds a complete unit; before_last_piece(band, quad) is called ahead of the
// unit's last piece of chunks, a few thousand clocks earlier (the place to request what on_unit will need).  The code chunks of the run are contiguous in memory.
// They are fetched in pieces of at most kPiece chunks that never straddle a unit (a unit is cut into equal pieces);
// two register sets alternate, so the loads of the next piece are in flight while the current one is decoded.
// Every piece issues exactly kPiece loads (those past its end repeat its last chunk): a fixed number of loads in flight
// is what lets the compiler wait for the current piece only and not for the one just requested.

template <typename BeforeLast, typename OnUnit>
__device__ __forceinline__ void decode_run_to_tile(const DevMat& m, uint32_t u0, uint32_t u1, int lane, uint32_t my_strip,
                                                   BeforeLast&& before_last_piece, OnUnit&& on_unit) {
  if (u0 >= u1) return;
  const uint32_t nq = m.n_quads, n_panels = (m.cols + m.seg_cols - 1) / m.seg_cols;
  // walker over the pieces of the run: unit, pieces left in it, next chunk
  uint32_t wu = u0, wc = unit_offset(m, u0), w_left = 0, w_base = 0, w_rem = 0;
  auto next_piece = [&](uint32_t& start, uint32_t& n, bool& ends) {
    if (w_left == 0) {
      if (wu == u1) {
        n = 0;
        ends = false;
        start = wc;
        return;
      }
      const uint32_t len = unit_offset(m, wu + 1) - wc;
      w_left = (len + kPiece - 1) / kPiece;
      w_base = len / w_left;
      w_rem = len - w_base * w_left;
      ++wu;
    }
    n = w_base + (w_rem ? 1u : 0u);
    if (w_rem) --w_rem;
    start = wc;
    wc += n;
    ends = --w_left == 0;
  };
  const uint32_t run_last = unit_offset(m, u1) - 1;   // last chunk of the run
  auto load_piece = [&](uint2 (&cw)[kPiece], uint32_t start, uint32_t n) {
    const uint32_t last = min(start + max(n, 1u) - 1, run_last);
#pragma unroll
    for (int k = 0; k < kPiece; ++k) cw[k] = load_chunk(m.codes, min(start + k, last), lane);
  };
  // decoder state: the unit being filled
  uint32_t band = u0 / nq, quad = u0 - band * nq;
  auto segment_length = [&]() {   // of the lane's segment in the unit (band, quad)
    const uint32_t row = band * kUnitRows + (lane & 15), panel = quad * kUnitPanels + (lane >> 4);
    uint32_t len = 0;
    if (row < m.rows && panel < n_panels) len = min(m.seg_cols, m.cols - panel * m.seg_cols);
    return len;
  };
  uint32_t pos = 0, seg_len = segment_length();
  uint64_t carry = 0;
  auto decode_piece = [&](const uint2 (&cw)[kPiece], uint32_t n, bool ends) {
    if (ends) before_last_piece(band, quad);
    if (n == kPiece) {   // whole pieces as straight-line code: the dictionary reads of later chunks overlap the packing of earlier ones
#pragma unroll
      for (int k = 0; k < kPiece; ++k) append_chunk(cw[k], my_strip, seg_len, pos, carry);
    } else if (n == kPiece - 1) {
#pragma unroll
      for (int k = 0; k < kPiece - 1; ++k) append_chunk(cw[k], my_strip, seg_len, pos, carry);
    } else {
#pragma unroll
      for (int k = 0; k < kPiece; ++k)
        if ((uint32_t)k < n) append_chunk(cw[k], my_strip, seg_len, pos, carry);
    }
    if (ends) {
      flush_carry(my_strip, pos, carry);
      on_unit(band, quad);
      if (++quad == nq) {
        quad = 0;
        ++band;
      }
      pos = 0;
      carry = 0;
      seg_len = segment_length();
    }
  };
  uint2 cwa[kPiece], cwb[kPiece];
  uint32_t sa, na, sb, nb;
  bool ea, eb;
  next_piece(sa, na, ea);
  load_piece(cwa, sa, na);
  while (na) {
    next_piece(sb, nb, eb);
    load_piece(cwb, sb, nb);
    decode_piece(cwa, na, ea);
    next_piece(sa, na, ea);
    load_piece(cwa, sa, na);
    decode_piece(cwb, nb, eb);
  }
}

typedef __attribute__((address_space(1))) const uint16_t global_cu16;
typedef __attribute__((address_space(1))) const u32x4 global_cu128;

// Activation fragment of one MFMA step: 8 consecutive bf16 of one batch row starting at column col.  The load is
// unconditional (columns past the end of the row are clamped into it) so that several of them can be in flight without
// the compiler waiting for each; mask_x_fragment zeroes what lies past the row's end before use.
template <bool kFast>
__device__ __forceinline__ uint4 load_x_fragment(global_cu16* xrow, uint32_t cols, uint32_t col) {
  if (kFast) {   // cols % 8 == 0 and x 16-byte aligned
    const u32x4 v = *(global_cu128*)(xrow + min(col, cols - 8));
    return make_uint4(v.x, v.y, v.z, v.w);
  }
  uint32_t e[8];
#pragma unroll
  for (int k = 0; k < 8; ++k) e[k] = xrow[min(col + k, cols - 1)];
  return make_uint4(e[0] | e[1] << 16, e[2] | e[3] << 16, e[4] | e[5] << 16, e[6] | e[7] << 16);
}
template <bool kFast>
__device__ __forceinline__ uint4 mask_x_fragment(uint4 v, uint32_t cols, uint32_t col) {
  if (kFast) return col < cols ? v : make_uint4(0, 0, 0, 0);
  uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
  for (int k = 0; k < 8; ++k)
    if (col + k >= cols) w[k >> 1] &= (k & 1) ? 0x0000FFFFu : 0xFFFF0000u;
  return make_uint4(w[0], w[1], w[2], w[3]);
}

constexpr int kMfmaGroup = 8;   // MFMA steps per group: the activation fragments of the next group load while this one runs

// The MFMA steps of one decoded unit: step w multiplies bytes [8 w, 8 w + 8) of every lane's strip (16 rows x 4 panels
// x 8 columns, converted to bf16) with the activations of those 32 columns.  n_win is wave-uniform.
// Four accumulators so that consecutive MFMAs do not wait for each other; groups of kMfmaGroup steps whose weight
// reads are all issued before the first conversion and whose activation fragments were requested a group earlier
// (the first group by the caller, into xa).
// kPacked: the strips hold packed 4-bit weights; a step then takes 4 bytes of every strip (8 columns again), n_win counts
// those steps, and cols and xcol are columns of the weight matrix (twice the byte columns).
template <bool kFast, bool kRagged, bool kPacked>
__device__ __forceinline__ f32x4 multiply_unit(f32x4 acc, uint32_t my_strip, global_cu16* xrow, uint32_t cols, uint32_t xcol, uint32_t n_win,
                                               uint4 (&xa)[kMfmaGroup]) {
  f32x4 part[4] = {acc, {0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
  uint4 xb[kMfmaGroup];
  auto request = [&](uint4 (&xf)[kMfmaGroup], uint32_t w0) {
#pragma unroll
    for (int k = 0; k < kMfmaGroup; ++k) xf[k] = load_x_fragment<kFast>(xrow, cols, xcol + 8 * (w0 + k));
  };
  auto weights = [&](uint32_t w) {   // the 8 weights of step w as bf16
    if constexpr (kPacked) {
      return nib8_to_bf16x8(*(lds_cu32*)(size_t)(my_strip + 4 * w));
    } else {
      const u32x2 a8 = *(lds_cu64*)(size_t)(my_strip + 8 * w);
      return i8x8_to_bf16x8(make_uint2(a8.x, a8.y));
    }
  };
  auto run_group = [&](const uint4 (&xf)[kMfmaGroup], uint32_t w0) {
    if (w0 + kMfmaGroup <= n_win) {   // whole group
      bf16x8 a8[kMfmaGroup];
      if constexpr (kPacked) {
#pragma unroll
        for (int k = 0; k < kMfmaGroup; ++k) a8[k] = weights(w0 + k);
      } else {
        u32x2 raw[kMfmaGroup];
#pragma unroll
        for (int k = 0; k < kMfmaGroup; ++k) raw[k] = *(lds_cu64*)(size_t)(my_strip + 8 * (w0 + k));
#pragma unroll
        for (int k = 0; k < kMfmaGroup; ++k) a8[k] = i8x8_to_bf16x8(make_uint2(raw[k].x, raw[k].y));
      }
#pragma unroll
      for (int k = 0; k < kMfmaGroup; ++k) {
        const uint4 x8 = kRagged ? mask_x_fragment<kFast>(xf[k], cols, xcol + 8 * (w0 + k)) : xf[k];
        part[k & 3] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a8[k], __builtin_bit_cast(bf16x8, x8), part[k & 3], 0, 0, 0);
      }
    } else {
#pragma unroll
      for (int k = 0; k < kMfmaGroup; ++k) {
        if (w0 + k < n_win) {
          const uint4 x8 = kRagged ? mask_x_fragment<kFast>(xf[k], cols, xcol + 8 * (w0 + k)) : xf[k];
          part[k & 3] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(weights(w0 + k), __builtin_bit_cast(bf16x8, x8), part[k & 3], 0, 0, 0);
        }
      }
    }
  };
  // xa holds the first group already: it was requested before the unit's last piece of chunks was decoded
  for (uint32_t w = 0; w < n_win; w += 2 * kMfmaGroup) {
    request(xb, w + kMfmaGroup);
    run_group(xa, w);
    request(xa, w + 2 * kMfmaGroup);
    run_group(xb, w + kMfmaGroup);
  }
  return (part[0] + part[1]) + (part[2] + part[3]);
}

// ---------------------------------------------------------------------------------------------------------------
// The batched product with a ring of kRingBytes per lane in place of the whole strip, and the activations in LDS.
//
// The 16 rows of a band take their codes in step but reach different columns, so some per-lane storage has to bring
// them back into line before an MFMA can take 8 columns of all of them; what it has to hold is only the distance
// between the slowest and the fastest lane, not the segment.  Every kRingStep chunks the wavefront asks whether every
// unfinished lane has passed the next kRingGroup windows (one compare and a look at the condition mask) and, if so,
// multiplies them; a lane advances by at most 8 columns per chunk, so one group per look keeps up.  Bytes of the ring
// are reused kRingBytes columns later: a lane writes 8-byte piece q only when q + 8 - kRingBytes <= done, which holds
// whenever no two unfinished lanes are ever more than kRingSpread columns apart; the host checks that for every unit
// when the container is loaded.  A matrix that does not keep it is decoded in a careful mode - a look after every chunk
// and one MFMA step at a time, which absorbs a distance of kRingSpreadCareful columns (the first units of a matrix that
// starts a dictionary, where early segments are still all single bytes, need that) - or, beyond that, goes to the
// whole-strip kernel.
// Piece p (8 bytes) of lane l lives at p ^ (l & 15) within the lane's ring: when the 64 lanes read the same window, the
// 16 lanes served together hit different banks.
//
// With 8 KB of ring per wavefront, 8 wavefronts leave room for the activations of one quad (4 panels) in LDS, laid out
// as the B operands the MFMA steps take: [panel][window][batch row 0..15][8 columns], 16 bytes per lane and step, read
// with one ds_read_b128.  (Taken from global memory, every step's fragment load touches 4 panels x batch rows
// different cache lines; that, not the decode, then bounds the kernel.)  All wavefronts of a workgroup therefore work
// on the same quad at a time: the workgroup walks the quads of its bands in the outer loop, wavefront w takes the
// whole bands, and a band's sums go to y once per quad: a plain store for the first quad, an atomic add (no return
// value, so nothing waits for it) for the others.  The stores and adds to a given y element are issued in quad order,
// one workgroup barrier apart from each other, so the result does not depend on timing.
// Needs rows of a whole number of units (a multiple of 4 * seg_cols columns), segments of 32..256 columns in
// multiples of 32 (packed 4-bit weights: 32..128 bytes), and 16-byte aligned activations.
constexpr int kRingBytes = 128;
constexpr int kRingWaves = 8;       // with an activation tile of 16 batch rows
constexpr int kRingWavesHalf = 10;  // with one of 8 batch rows (batches up to 8): more wavefronts fit next to the smaller tile
constexpr int kRingWavesMore = 12;  // the same beside a dictionary of at most 24,512 entries
constexpr int kRingPiece = 12;    // chunks per piece of the code stream (two register sets)
constexpr int kRingStep = 4;      // chunks between two looks at the lanes' progress
constexpr int kRingGroup = 4;     // MFMA steps per group
constexpr uint32_t kRingSpread = kRingBytes - 8 * kRingStep - 8 * kRingGroup + 1;
constexpr uint32_t kRingSpreadCareful = kRingBytes - 8 - 8 + 1;   // looking after every chunk, one MFMA step at a time
constexpr uint32_t kRingMaxSeg = 256;
constexpr int kRingMinBandsPerCu = 24;   // below that many bands per CU in a launch the whole-strip kernel is used
constexpr uint32_t ring_x_tile(int rows) { return kUnitPanels * kRingMaxSeg * rows * 2; }   // bytes: 4 panels x 256 columns x batch rows of bf16
static_assert(kRingPiece % kRingStep == 0 && kRingGroup == 4 && kRingStep <= kRingGroup, "ring schedule");

// append_chunk for the ring: the complete 8-byte piece goes to its swizzled place; sw8 = 8 * (lane & 15).
// pos never passes seg_len (pad codes fall off the end), and a piece is complete when pos crosses a multiple of 8.
__device__ __forceinline__ void append_chunk_ring(uint2 c, uint32_t ring, uint32_t sw8, uint32_t seg_len, uint32_t& pos, uint64_t& carry) {
  const uint32_t e0 = lds_read16(half_offset_lo(c.x)), e1 = lds_read16(half_offset_hi(c.x));
  const uint32_t e2 = lds_read16(half_offset_lo(c.y)), e3 = lds_read16(half_offset_hi(c.y));
  const uint32_t p0 = is_pair_lo(c.x), p1 = is_pair_hi(c.x), p2 = is_pair_lo(c.y), p3 = is_pair_hi(c.y);
  const uint32_t a01 = e1 << ((p0 << 3) + 8) | e0, n01 = p0 + p1 + 2;   // codes 0, 1: n01 = 2..4 bytes
  const uint32_t a23 = e3 << ((p2 << 3) + 8) | e2, n23 = p2 + p3 + 2;   // codes 2, 3
  const uint64_t str = (uint64_t)a23 << (n01 << 3) | a01;               // the 4..8 bytes of the chunk
  const uint32_t after = min(pos + n01 + n23, seg_len);
  const uint32_t sh = (pos & 7u) << 3;
  const uint64_t lo = carry | str << sh, hi = (str >> 1) >> (63 - sh);  // the 16 bytes carry + string; hi is 0 when pos % 8 == 0
  const bool full = (after ^ pos) >= 8;
  if (full) *(lds_u64*)(size_t)(ring | ((pos ^ sw8) & 0x78u)) = lo;
  carry = full ? hi : lo;
  pos = after;
}

typedef __attribute__((address_space(3))) const u32x4 lds_cu128;

// Decode and multiply units of quad `quad`, one band after the other (every unit has 4 whole panels of seg_cols
// columns): first the one of band first_band, then those of the bands claim() hands out, until it returns kNoBand.
// ring: LDS address of the lane's ring; xfrag: LDS address of the lane's 16 bytes of window 0 in the activation tile
// (window w is 16 kRows w bytes further).  on_unit(band, next_band, sums) is called with a unit's 16 x 16 sums after its
// last MFMA step; next_band is the band that follows (claimed a piece of chunks ahead), or kNoBand.
constexpr uint32_t kNoBand = 0xFFFFFFFFu;
// kPacked: the ring holds packed 4-bit weights; an 8-byte piece is then two MFMA steps (16 columns), and the activation
// tile has two windows per piece.
template <bool kCareful, int kRows, bool kPacked, typename Claim, typename OnUnit>
__device__ __forceinline__ void decode_units_ring(const DevMat& m, uint32_t quad, uint32_t first_band, Claim&& claim, int lane, uint32_t ring,
                                                  uint32_t xfrag, OnUnit&& on_unit) {
  if (first_band == kNoBand) return;
  constexpr int kP = kRingPiece, kG = kCareful ? 1 : kRingGroup, kLook = kCareful ? 1 : kRingStep;
  const uint32_t sw8 = (uint32_t)(lane & 15) << 3;
  const uint32_t n_win8 = m.seg_cols;
  // a row past the end of the matrix has no segment: its lane decodes nothing
  auto segment_length = [&](uint32_t band) { return band != kNoBand && band * kUnitRows + (lane & 15) < m.rows ? m.seg_cols : 0u; };
  uint32_t cur_band = first_band, seg_len = segment_length(first_band);
  // walker over the pieces: the band it is in (the decoder is at most one band behind), pieces left in it, next chunk
  uint32_t w_band = kNoBand, wc = 0, w_left = 0, w_base = 0, w_rem = 0;
  bool w_started = false;
  auto next_piece = [&](uint32_t& start, uint32_t& n, bool& ends) {
    if (w_left == 0) {
      if (w_started && w_band == kNoBand) {   // nothing left to claim
        n = 0;
        ends = false;
        start = wc;
        return;
      }
      w_band = w_started ? claim() : first_band;
      w_started = true;
      if (w_band == kNoBand) {
        n = 0;
        ends = false;
        start = wc;
        return;
      }
      const uint32_t u = w_band * m.n_quads + quad;
      wc = unit_offset(m, u);
      const uint32_t len = unit_offset(m, u + 1) - wc;
      w_left = (len + kP - 1) / kP;
      w_base = len / w_left;
      w_rem = len - w_base * w_left;
    }
    n = w_base + (w_rem ? 1u : 0u);
    if (w_rem) --w_rem;
    start = wc;
    wc += n;
    ends = --w_left == 0;
  };
  // Every piece issues exactly kP loads (those past its end repeat its last chunk), kRingStep of them at a time.
  auto load_part = [&](uint2 (&cw)[kP], uint32_t start, uint32_t n, int part) {
    const uint32_t last = n ? start + n - 1 : start - 1;   // n == 0 (past the last unit, start >= 1): the chunk before, never used
#pragma unroll
    for (int k = part * kRingStep; k < (part + 1) * kRingStep; ++k) cw[k] = load_chunk(m.codes, min(start + k, last), lane);
  };
  uint32_t pos = 0, done = 0;
  uint64_t carry = 0;
  f32x4 part[4] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
  // One group of MFMA steps if every lane that is still decoding has written the columns [done, done + 8 kG).
  // The operands are read before it is known whether the group is ready (volatile: the reads stay ahead of the test),
  // so that their latency overlaps the test; an unready group just reads them again at the next look.
  auto multiply_ready = [&]() {
    const uint32_t at = min(done, n_win8 - 8 * kG);   // at the unit's end: any place inside the ring and the tile
    const uint32_t base = at ^ sw8;
    constexpr int kX = kPacked ? 2 : 1;             // activation windows per 8-byte piece of the ring
    const uint32_t xa = xfrag + at * (2 * kRows * kX);   // 16 kRows bytes per window
    u32x2 a8[kG];
    u32x4 x8[kG * kX];
#pragma unroll
    for (int k = 0; k < kG; ++k) {
      a8[k] = *(volatile lds_cu64*)(size_t)(ring | ((base ^ (8u * k)) & 0x78u));
#pragma unroll
      for (int h = 0; h < kX; ++h) x8[k * kX + h] = *(volatile lds_cu128*)(size_t)(xa + 16 * kRows * (k * kX + h));
    }
    const uint32_t next = done + 8 * kG;
    if (next > n_win8) return;
    if (__builtin_amdgcn_ballot_w64(pos < min(seg_len, next)) != 0) return;
#pragma unroll
    for (int k = 0; k < kG; ++k) {
      if constexpr (kPacked) {
        part[k] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(nib8_to_bf16x8(a8[k].x), __builtin_bit_cast(bf16x8, x8[2 * k]), part[k], 0, 0, 0);
        part[k] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(nib8_to_bf16x8(a8[k].y), __builtin_bit_cast(bf16x8, x8[2 * k + 1]), part[k], 0, 0, 0);
      } else {
        part[k] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(i8x8_to_bf16x8(make_uint2(a8[k].x, a8[k].y)), __builtin_bit_cast(bf16x8, x8[k]), part[k], 0, 0, 0);
      }
    }
    done = next;
  };
  auto decode_piece = [&](const uint2 (&cw)[kP], uint32_t n, bool ends, uint2 (&cw_next)[kP], uint32_t next_start, uint32_t next_n) {
    if (n == 0) return;
    if (n >= kP - 1) {
#pragma unroll
      for (int k = 0; k < kP - 1; ++k) {
        append_chunk_ring(cw[k], ring, sw8, seg_len, pos, carry);
        if (k % kLook == kLook - 1) multiply_ready();
        if (k % kRingStep == kRingStep - 1) load_part(cw_next, next_start, next_n, k / kRingStep);
      }
      if (n == kP) append_chunk_ring(cw[kP - 1], ring, sw8, seg_len, pos, carry);
    } else {
#pragma unroll
      for (int k = 0; k < kP - 2; ++k) {
        if ((uint32_t)k < n) append_chunk_ring(cw[k], ring, sw8, seg_len, pos, carry);
        if (k % kLook == kLook - 1 && (uint32_t)k + 1 < n) multiply_ready();
        if (k % kRingStep == kRingStep - 1) load_part(cw_next, next_start, next_n, k / kRingStep);
      }
    }
    multiply_ready();
    load_part(cw_next, next_start, next_n, kP / kRingStep - 1);
    if (ends) {   // every lane is complete and at most one whole group was left: the unit has been multiplied
      // the walker is one piece ahead: w_band is the band of the unit that follows, if there is one
      const uint32_t next_band = w_band == cur_band ? kNoBand : w_band;
      on_unit(cur_band, next_band, (part[0] + part[1]) + (part[2] + part[3]));
#pragma unroll
      for (int k = 0; k < 4; ++k) part[k] = f32x4{0.f, 0.f, 0.f, 0.f};
      cur_band = next_band;
      seg_len = segment_length(cur_band);
      pos = 0;
      carry = 0;
      done = 0;
    }
  };
  uint2 cwa[kP], cwb[kP];
  uint32_t sa, na, sb, nb;
  bool ea, eb;
  next_piece(sa, na, ea);
#pragma unroll
  for (int j = 0; j < kP / kRingStep; ++j) load_part(cwa, sa, na, j);
  while (na) {   // two register sets: one is decoded while the other is filled
    next_piece(sb, nb, eb);
    decode_piece(cwa, na, ea, cwb, sb, nb);
    next_piece(sa, na, ea);
    decode_piece(cwb, nb, eb, cwa, sa, na);
  }
}

template <int kWaves, int kRows, bool kPacked>
__global__ __launch_bounds__(kWaves * 64, 1) void k_matvec_ring(MatvecArgs a) {
  constexpr int kRingThreads = kWaves * 64;
  constexpr uint32_t kRingXTile = ring_x_tile(kRows);
  extern __shared__ uint4 lds4[];
  uint16_t* lds_dict = (uint16_t*)lds4;
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  if (lds_address(lds4) != 0) return;   // the code -> entry lookup takes the dictionary to start at LDS address 0
  const uint32_t rings = a.x_off, xtile = a.slot_off;   // LDS addresses (the LDS segment starts at 0)
  const uint64_t total = cost_at(a, a.n);
  const uint32_t lo = (uint32_t)(total * blockIdx.x / gridDim.x), hi = (uint32_t)(total * (blockIdx.x + 1) / gridDim.x);
  const uint32_t* staged = nullptr;
  const int bn = lane & 15, kg = lane >> 4;   // B operand: batch row and k-group (panel) of this lane
  const uint32_t ring = rings + (uint32_t)wave * (64 * kRingBytes) + (uint32_t)lane * kRingBytes;
  for (int i = 0; i < a.n; ++i) {
    const uint32_t cb = cost_at(a, i), ce = cost_at(a, i + 1);
    if (hi <= cb || lo >= ce) continue;
    Job job;
    DevMat m;
    fetch_job(a, i, job, m);
    const uint32_t bc = m.cols;
    const uint32_t band_lo = lo <= cb ? 0u : (lo - cb + bc / 2) / bc;
    const uint32_t band_hi = hi >= ce ? m.n_bands : min(m.n_bands, (hi - cb + bc / 2) / bc);
    if (band_lo >= band_hi) continue;
    constexpr uint32_t pk = kPacked ? 2u : 1u;             // columns of the weight matrix per stored byte
    const uint32_t nq = m.n_quads, n_win = pk * m.seg_cols / 8;   // activation windows (8 columns) per segment
    __syncthreads();   // the previous matrix's dictionary and activation tile are no longer in use
    if (m.dict != staged) {
      // 16-bit image of the dictionary: the run bytes of every entry (the length follows from the code)
      const uint4* src = (const uint4*)m.dict;
      uint2* dst = (uint2*)lds_dict;
      const uint32_t n4 = m.dict_words / 4;
      for (uint32_t base = 0; base < n4; base += kDictRegs * kRingThreads) {
        uint4 v[kDictRegs];
#pragma unroll
        for (int k = 0; k < kDictRegs; ++k) v[k] = global_load(src + min(base + k * kRingThreads + tid, n4 - 1));
#pragma unroll
        for (int k = 0; k < kDictRegs; ++k) {
          const uint32_t idx = base + k * kRingThreads + tid;
          if (idx < n4) dst[idx] = make_uint2((v[k].x & 0xFFFFu) | v[k].y << 16, (v[k].z & 0xFFFFu) | v[k].w << 16);
        }
      }
      staged = m.dict;
    }
    // Bands are handed out one at a time, per quad, through a counter in LDS: wavefront w starts with band w of the
    // workgroup's range and claims the next free one while it decodes the last piece of chunks of the one in work.
    // (An even split up front leaves wavefronts waiting at the end of every quad: for the slowest, and for the one more
    // band that some of them have.)
    const uint32_t n_bands = band_hi - band_lo;
    typedef __attribute__((address_space(3))) uint32_t lds_u32;
    lds_u32* next_band_counter = (lds_u32*)(size_t)(xtile + kRingXTile);
    auto claim = [&]() {
      uint32_t b = 0;
      if (lane == 0) b = __hip_atomic_fetch_add(next_band_counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
      b = __builtin_amdgcn_readfirstlane(b);
      return b < n_bands ? band_lo + b : kNoBand;
    };
    const uint32_t xfrag = xtile + ((uint32_t)kg * n_win * kRows + (bn & (kRows - 1))) * 16;   // lanes past kRows repeat a row: their sums are not stored
    // Activation tile of a quad: piece ((panel * n_win + w) * kRows + batch row) holds 8 columns; rows past the batch are
    // zero.  The pieces of the next quad's tile are requested into registers before this quad is decoded and written
    // to LDS when everybody has finished it, so that nobody waits for device memory between two quads.
    constexpr int kTileRegs = (kRingXTile / 16 + kRingThreads - 1) / kRingThreads;
    const uint32_t pieces = kUnitPanels * n_win * kRows, per_row = kUnitPanels * n_win;
    u32x4 tile[kTileRegs];
    auto request_tile = [&](uint32_t q) {
      const uint32_t col0 = q * kUnitPanels * pk * m.seg_cols;
#pragma unroll
      for (int k = 0; k < kTileRegs; ++k) {
        const uint32_t o = min((uint32_t)tid + k * kRingThreads, pieces - 1);
        const uint32_t r = o / per_row, c = o - r * per_row;   // batch row, 8-column piece of the quad
        tile[k] = *(global_cu128*)((global_cu16*)job.x + (size_t)min(r, (uint32_t)a.batch - 1) * (pk * m.cols) + col0 + 8 * c);
      }
    };
    auto commit_tile = [&]() {
#pragma unroll
      for (int k = 0; k < kTileRegs; ++k) {
        const uint32_t o = (uint32_t)tid + k * kRingThreads;
        const uint32_t r = o / per_row, c = o - r * per_row;
        u32x4 v = tile[k];
        if (r >= (uint32_t)a.batch) v = u32x4{0u, 0u, 0u, 0u};
        if (o < pieces) *(__attribute__((address_space(3))) u32x4*)(size_t)(xtile + (c * kRows + r) * 16) = v;   // c = panel * n_win + w
      }
    };
    request_tile(0);
    for (uint32_t q = 0; q < nq; ++q) {
      if (q) __syncthreads();   // everybody has finished the previous quad: its activation tile can go
      if (tid == 0) *next_band_counter = kWaves;   // bands 0 .. kWaves - 1 are the wavefronts' first ones
      commit_tile();
      if (q + 1 < nq) request_tile(q + 1);
      __syncthreads();
      // Sums of lane l: rows 4 * (l / 16) + v of the band, batch row l % 16.  The scales of the next band are requested
      // when this one's have been used, a unit ahead of their use: waiting for them is then not a wait for the code
      // chunks requested in between.
      const uint32_t band0 = (uint32_t)wave < n_bands ? band_lo + wave : kNoBand;
      float scale[4];
      auto request_scales = [&](uint32_t band) {
#pragma unroll
        for (int v = 0; v < 4; ++v) scale[v] = global_load(m.scales + min(band, m.n_bands - 1) * kUnitRows + 4 * kg + v);
      };
      request_scales(band0);
      auto finish_unit = [&](uint32_t band, uint32_t next_band, f32x4 sums) {
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          const uint32_t row = band * kUnitRows + 4 * kg + v;
          if (bn < a.batch && row < m.rows) {
            float* y = job.y + (size_t)bn * m.rows + row;
            if (q == 0) global_store(y, sums[v] * scale[v]);
            else (void)__builtin_amdgcn_global_atomic_fadd_f32((__attribute__((address_space(1))) float*)y, sums[v] * scale[v]);
          }
        }
        request_scales(next_band);
      };
      if (m.reserved == 2) decode_units_ring<true, kRows, kPacked>(m, q, band0, claim, lane, ring, xfrag, finish_unit);
      else decode_units_ring<false, kRows, kPacked>(m, q, band0, claim, lane, ring, xfrag, finish_unit);
    }
  }
}

template <bool kXFast, bool kPacked>
__global__ __launch_bounds__(kThreads, 1) void k_matvec_mfma(MatvecArgs a) {
  extern __shared__ uint4 lds4[];
  uint16_t* lds_dict = (uint16_t*)lds4;
  uint8_t* tiles = (uint8_t*)lds4 + a.x_off;
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n_threads = blockDim.x, n_waves = n_threads >> 6;
  if (lds_address(lds4) != 0) return;   // the code -> entry lookup takes the dictionary to start at LDS address 0
  const uint64_t total = cost_at(a, a.n);
  const uint32_t lo = (uint32_t)(total * blockIdx.x / gridDim.x), hi = (uint32_t)(total * (blockIdx.x + 1) / gridDim.x);
  const uint32_t* staged = nullptr;
  const int bn = lane & 15, kg = lane >> 4;   // B operand: batch row and k-group of this lane
  for (int i = 0; i < a.n; ++i) {
    const uint32_t cb = cost_at(a, i), ce = cost_at(a, i + 1);
    if (hi <= cb || lo >= ce) continue;
    Job job;
    DevMat m;
    fetch_job(a, i, job, m);
    const uint32_t bc = m.cols;
    const uint32_t band_lo = lo <= cb ? 0u : (lo - cb + bc / 2) / bc;
    const uint32_t band_hi = hi >= ce ? m.n_bands : min(m.n_bands, (hi - cb + bc / 2) / bc);
    if (band_lo >= band_hi) continue;
    const uint32_t nq = m.n_quads;
    const uint32_t unit_lo = band_lo * nq, n_units = (band_hi - band_lo) * nq;
    const uint32_t u0 = unit_lo + (uint32_t)((uint64_t)n_units * wave / n_waves);
    const uint32_t u1 = unit_lo + (uint32_t)((uint64_t)n_units * (wave + 1) / n_waves);
    __syncthreads();   // the previous matrix's dictionary and partial sums are no longer in use
    if (m.dict != staged) {
      // 16-bit image of the dictionary: the run bytes of every entry (the length follows from the code)
      const uint4* src = (const uint4*)m.dict;
      uint2* dst = (uint2*)lds_dict;
      const uint32_t n4 = m.dict_words / 4;
      for (uint32_t base = 0; base < n4; base += kDictRegs * n_threads) {
        uint4 v[kDictRegs];
#pragma unroll
        for (int k = 0; k < kDictRegs; ++k) v[k] = global_load(src + min(base + k * n_threads + tid, n4 - 1));
#pragma unroll
        for (int k = 0; k < kDictRegs; ++k) {
          const uint32_t idx = base + k * n_threads + tid;
          if (idx < n4) dst[idx] = make_uint2((v[k].x & 0xFFFFu) | v[k].y << 16, (v[k].z & 0xFFFFu) | v[k].w << 16);
        }
      }
      staged = m.dict;
    }
    __syncthreads();
    f32x4 acc = {0.f, 0.f, 0.f, 0.f}, head_acc = {0.f, 0.f, 0.f, 0.f}, tail_acc = {0.f, 0.f, 0.f, 0.f};
    int head_band = -1, tail_band = -1;
    // lanes past the batch repeat its last row: their output columns are never stored
    constexpr uint32_t pk = kPacked ? 2u : 1u;   // columns of the weight matrix per stored byte
    const uint32_t x_cols = pk * m.cols;
    global_cu16* xrow = (global_cu16*)job.x + (size_t)min(bn, a.batch - 1) * x_cols;
    const uint32_t first_band = u0 / nq;
    const bool first_whole = u0 % nq == 0;
    // acc holds the sums of the band in work when its last unit (or the run's) has been multiplied
    auto finish_unit = [&](uint32_t band, uint32_t quad) {
      const bool band_ends = quad + 1 == nq, run_ends = band * nq + quad + 1 == u1;
      if (band_ends || run_ends) {
        if (band_ends && (band != first_band || first_whole)) {
          // the whole band lies in this wavefront's run.  Accumulator register v of lane l: row 4 * (l / 16) + v, batch row l % 16
          if (a.gate_up) {   // registers 0, 1 and 2, 3 of a lane are gate and up row of two outputs
#pragma unroll
            for (int v = 0; v < 4; v += 2) {
              const uint32_t row = band * kUnitRows + 4 * kg + v;
              if (bn < a.batch && row + 1 < m.rows)
                global_store(job.y + (size_t)bn * (m.rows / 2) + row / 2,
                             silu_times(acc[v] * global_load(m.scales + row), acc[v + 1] * global_load(m.scales + row + 1)));
            }
          } else {
#pragma unroll
            for (int v = 0; v < 4; ++v) {
              const uint32_t row = band * kUnitRows + 4 * kg + v;
              if (bn < a.batch && row < m.rows) global_store(job.y + (size_t)bn * m.rows + row, acc[v] * global_load(m.scales + row));
            }
          }
        } else if (band == first_band && !first_whole) {   // band begun by an earlier wavefront
          head_acc = acc;
          head_band = (int)band;
        } else {                                           // band left unfinished
          tail_acc = acc;
          tail_band = (int)band;
        }
        acc = f32x4{0.f, 0.f, 0.f, 0.f};
      }
    };
    {
      const uint32_t strip = m.seg_cols + 8;   // bytes between the strips of two lanes
      const uint32_t my_strip = lds_address(tiles) + (uint32_t)wave * a.tile_area + (uint32_t)lane * strip;
      uint4 xa[kMfmaGroup];   // activation fragments of the first MFMA group of the unit being decoded
      decode_run_to_tile(m, u0, u1, lane, my_strip, [&](uint32_t, uint32_t quad) {
#pragma unroll
        for (int k = 0; k < kMfmaGroup; ++k)
          xa[k] = load_x_fragment<kXFast>(xrow, x_cols, pk * (quad * kUnitPanels + (uint32_t)kg) * m.seg_cols + 8 * k);
      }, [&](uint32_t band, uint32_t quad) {
        const uint32_t col0 = quad * kUnitPanels * m.seg_cols;                            // first (byte) column of the unit
        const uint32_t width = min(m.seg_cols, m.cols - col0);                            // its widest segment is the first panel's
        const uint32_t n_win = (pk * width + 7) / 8;
        const uint32_t xcol = pk * (col0 + (uint32_t)kg * m.seg_cols);
        const bool ragged = !kXFast || col0 + kUnitPanels * m.seg_cols > m.cols;          // some fragment reaches past the row's end
        if (ragged) acc = multiply_unit<kXFast, true, kPacked>(acc, my_strip, xrow, x_cols, xcol, n_win, xa);
        else acc = multiply_unit<kXFast, false, kPacked>(acc, my_strip, xrow, x_cols, xcol, n_win, xa);
        finish_unit(band, quad);
      });
    }
    __syncthreads();   // every wavefront is done with its tile: the partial sums go over the tile area
    float* slot_val = (float*)tiles;                                 // [2 * n_waves][256]
    int* slot_band = (int*)(slot_val + 2 * n_waves * 256);           // [2 * n_waves], also inside the tile area
    if (lane == 0) {
      slot_band[2 * wave] = head_band;
      slot_band[2 * wave + 1] = tail_band;
    }
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      slot_val[(2 * wave) * 256 + v * 64 + lane] = head_acc[v];
      slot_val[(2 * wave + 1) * 256 + v * 64 + lane] = tail_acc[v];
    }
    __syncthreads();
    for (int o = tid; o < 2 * n_waves * 256; o += n_threads) {
      const int s = o >> 8, e = o & 255;
      const int bnd = slot_band[s];
      bool first = bnd >= 0;
      for (int t = 0; t < s; ++t) first = first && slot_band[t] != bnd;
      if (first) {
        auto slot_sum = [&](int el) {
          float sum = slot_val[s * 256 + el];
          for (int t = s + 1; t < 2 * n_waves; ++t)
            if (slot_band[t] == bnd) sum += slot_val[t * 256 + el];
          return sum;
        };
        const int v = e >> 6, l = e & 63;
        const uint32_t row = (uint32_t)bnd * kUnitRows + 4 * (l >> 4) + v;
        const int b = l & 15;
        if (a.gate_up) {   // element e + 64 is the up row that belongs to this gate row
          if (!(v & 1) && b < a.batch && row + 1 < m.rows)
            global_store(job.y + (size_t)b * (m.rows / 2) + row / 2,
                         silu_times(slot_sum(e) * global_load(m.scales + row), slot_sum(e + 64) * global_load(m.scales + row + 1)));
        } else if (b < a.batch && row < m.rows) {
          global_store(job.y + (size_t)b * m.rows + row, slot_sum(e) * global_load(m.scales + row));
        }
      }
    }
  }
}

// Expansion to the row-major int8 matrices (the paper's own online step: every codeword is replaced by its table
// sequence).  Same work split and same tile decode as the batched product; a finished unit is copied out in 16-byte
// pieces, consecutive lanes taking consecutive pieces of a row (4 panels x seg_cols contiguous bytes per row).
// The y pointer of a job is the int8 output matrix here; the activation pointer is not used.
__global__ __launch_bounds__(kThreads, 1) void k_decompress(MatvecArgs a) {
  extern __shared__ uint4 lds4[];
  uint16_t* lds_dict = (uint16_t*)lds4;
  uint8_t* tiles = (uint8_t*)lds4 + a.x_off;
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n_threads = blockDim.x, n_waves = n_threads >> 6;
  if (lds_address(lds4) != 0) return;   // the code -> entry lookup takes the dictionary to start at LDS address 0
  const uint64_t total = cost_at(a, a.n);
  const uint32_t lo = (uint32_t)(total * blockIdx.x / gridDim.x), hi = (uint32_t)(total * (blockIdx.x + 1) / gridDim.x);
  const uint32_t* staged = nullptr;
  for (int i = 0; i < a.n; ++i) {
    const uint32_t cb = cost_at(a, i), ce = cost_at(a, i + 1);
    if (hi <= cb || lo >= ce) continue;
    Job job;
    DevMat m;
    fetch_job(a, i, job, m);
    const uint32_t bc = m.cols;
    const uint32_t band_lo = lo <= cb ? 0u : (lo - cb + bc / 2) / bc;
    const uint32_t band_hi = hi >= ce ? m.n_bands : min(m.n_bands, (hi - cb + bc / 2) / bc);
    if (band_lo >= band_hi) continue;
    const uint32_t nq = m.n_quads;
    const uint32_t unit_lo = band_lo * nq, n_units = (band_hi - band_lo) * nq;
    const uint32_t u0 = unit_lo + (uint32_t)((uint64_t)n_units * wave / n_waves);
    const uint32_t u1 = unit_lo + (uint32_t)((uint64_t)n_units * (wave + 1) / n_waves);
    if (m.dict != staged) {
      __syncthreads();   // nobody reads the previous dictionary any more
      const uint4* src = (const uint4*)m.dict;
      uint2* dst = (uint2*)lds_dict;
      const uint32_t n4 = m.dict_words / 4;
      for (uint32_t base = 0; base < n4; base += kDictRegs * n_threads) {
        uint4 v[kDictRegs];
#pragma unroll
        for (int k = 0; k < kDictRegs; ++k) v[k] = global_load(src + min(base + k * n_threads + tid, n4 - 1));
#pragma unroll
        for (int k = 0; k < kDictRegs; ++k) {
          const uint32_t idx = base + k * n_threads + tid;
          if (idx < n4) dst[idx] = make_uint2((v[k].x & 0xFFFFu) | v[k].y << 16, (v[k].z & 0xFFFFu) | v[k].w << 16);
        }
      }
      staged = m.dict;
      __syncthreads();
    }
    const uint32_t strip = m.seg_cols + 8;
    const uint32_t tile_lds = lds_address(tiles) + (uint32_t)wave * a.tile_area;   // matrices of different segment width may be in work at once
    int8_t* out = (int8_t*)job.y;
    const bool aligned = ((m.packing ? 2 * m.cols : m.cols) % 16 == 0) && ((uintptr_t)out % 16 == 0);
    const uint32_t ppp = m.seg_cols / 16;   // 16-byte pieces per segment
    decode_run_to_tile(m, u0, u1, lane, tile_lds + (uint32_t)lane * strip, [](uint32_t, uint32_t) {}, [&](uint32_t band, uint32_t quad) {
      for (uint32_t pc = lane; pc < 64 * ppp; pc += 64) {
        const uint32_t seg = pc / ppp, part = pc - seg * ppp;            // segment (row seg / 4, panel seg % 4) of the unit
        const uint32_t row = band * kUnitRows + (seg >> 2), col = (quad * kUnitPanels + (seg & 3)) * m.seg_cols + part * 16;
        if (row >= m.rows || col >= m.cols) continue;
        const uint32_t src = tile_lds + ((seg >> 2) + 16 * (seg & 3)) * strip + part * 16;   // strip of lane (row, panel)
        const u32x2 lo8 = *(lds_cu64*)(size_t)src, hi8 = *(lds_cu64*)(size_t)(src + 8);
        if (m.packing) {   // 16 bytes -> 32 int8: columns 2 col .. 2 col + 31 of a row of 2 cols values
          int8_t* dst2 = out + ((size_t)row * m.cols + col) * 2;
          const uint32_t w[4] = {lo8.x, lo8.y, hi8.x, hi8.y};
          uint32_t e[8];
#pragma unroll
          for (int k = 0; k < 4; ++k) {   // nibbles to bytes with their sign (8 -> 0xF8 inside its own byte), then in column order
            uint32_t even = w[k] & 0x0F0F0F0Fu, odd = (w[k] >> 4) & 0x0F0F0F0Fu;
            even |= (even & 0x08080808u) * 0x1Eu;
            odd |= (odd & 0x08080808u) * 0x1Eu;
            e[2 * k] = __builtin_amdgcn_perm(odd, even, 0x05010400u);
            e[2 * k + 1] = __builtin_amdgcn_perm(odd, even, 0x07030602u);
          }
          if (aligned && col + 16 <= m.cols) {
            *(__attribute__((address_space(1))) u32x4*)dst2 = u32x4{e[0], e[1], e[2], e[3]};
            *(__attribute__((address_space(1))) u32x4*)(dst2 + 16) = u32x4{e[4], e[5], e[6], e[7]};
          } else {
#pragma unroll
            for (int k = 0; k < 32; ++k)
              if (col + k / 2 < m.cols) *(__attribute__((address_space(1))) int8_t*)(dst2 + k) = (int8_t)(e[k >> 2] >> (8 * (k & 3)));
          }
          continue;
        }
        int8_t* dst = out + (size_t)row * m.cols + col;
        if (aligned && col + 16 <= m.cols) {
          u32x4 v = {lo8.x, lo8.y, hi8.x, hi8.y};
          *(__attribute__((address_space(1))) u32x4*)dst = v;
        } else {
          const uint32_t w[4] = {lo8.x, lo8.y, hi8.x, hi8.y};
#pragma unroll
          for (int k = 0; k < 16; ++k)
            if (col + k < m.cols) *(__attribute__((address_space(1))) int8_t*)(dst + k) = (int8_t)(w[k >> 2] >> (8 * (k & 3)));
        }
      }
    });
  }
}

}  // namespace tq

using namespace tq;

namespace {

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

int acquire_dictionary(int device, const uint32_t* words, uint32_t n_words, uint32_t n_words_pad, uint32_t packing, DictCopy** out) {
  std::lock_guard<std::mutex> lock(g_dict_mutex);
  for (DictCopy* d : g_dicts)
    if (d->device == device && d->packing == packing && d->words.size() == n_words && std::memcmp(d->words.data(), words, (size_t)n_words * 4) == 0) {
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
  d->dev = d->dev_bf16 = nullptr;
  // bytes past an entry's length are zero in the container, so the conversion needs no length test
  std::vector<uint32_t> pairs(n_words_pad, 0u);
  for (uint32_t i = 0; i < n_words; ++i) {
    if (packing) {
      for (uint32_t k = 0; k < 4; ++k) pairs[i] |= nibble_to_fp8_bits(words[i] >> (4 * k) & 15u) << (8 * k);
    } else {
      pairs[i] = i8_to_bf16_bits(words[i] & 0xFFu) | i8_to_bf16_bits(words[i] >> 8 & 0xFFu) << 16;
    }
  }
  hipError_t e = hipMalloc((void**)&d->dev, (size_t)n_words_pad * 4);
  if (e == hipSuccess) e = hipMalloc((void**)&d->dev_bf16, (size_t)n_words_pad * 4);
  if (e == hipSuccess) e = hipMemset(d->dev, 0, (size_t)n_words_pad * 4);
  if (e == hipSuccess) e = hipMemcpy(d->dev, words, (size_t)n_words * 4, hipMemcpyHostToDevice);
  if (e == hipSuccess) e = hipMemcpy(d->dev_bf16, pairs.data(), (size_t)n_words_pad * 4, hipMemcpyHostToDevice);
  if (e != hipSuccess) {
    if (d->dev) (void)hipFree(d->dev);
    if (d->dev_bf16) (void)hipFree(d->dev_bf16);
    delete d;
    return hip_fail("dictionary upload", e);
  }
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

constexpr uint32_t kSlotBytes = 2 * kDotWavesMax * 16 * 4 + 2 * kDotWavesMax * 4;

// LDS plan of the product kernel for a set of matrices: dictionary | activation image | partial-sum slots.
bool plan_matvec_lds(uint32_t dict_words_max, uint32_t x_dwords_max, uint32_t* x_off, uint32_t* slot_off, size_t* total) {
  *x_off = (uint32_t)round_up((uint64_t)dict_words_max * 4, 16);
  *slot_off = (uint32_t)round_up((uint64_t)*x_off + (uint64_t)x_dwords_max * 4, 16);
  *total = (size_t)*slot_off + kSlotBytes;
  return *total <= kLdsLimit;
}

}  // namespace

struct tq_matrix {
  Header h;
  BlobFacts facts;
  DevMat m;
  const DevMat* m_dev;   // the same description in device memory, for launches that serve many matrices
  DictCopy* dict;
  void* dev_base;
  int device;
  int n_cu;
};

extern "C" int tq_create_from_encoded(const void* blob, size_t blob_bytes, tq_handle* out) {
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
  m.dict_words = (uint32_t)round_up(h.n_entries + 1, 4);
  // Panels of one unit are seg_cols columns apart; a gap of 16 dwords after every panel keeps their activation reads
  // on different LDS banks when seg_cols is a multiple of 32.
  m.x_span = h.seg_cols + (h.seg_cols % 32 == 0 ? 16u : 0u);
  m.seg_magic = (uint32_t)((1ull << 32) / h.seg_cols) + 1;   // exact quotient while col * seg_cols < 2^32
  m.reserved = facts.max_lane_spread <= kRingSpread ? 1u : facts.max_lane_spread <= kRingSpreadCareful ? 2u : 0u;
  m.packing = h.packing;
  if (h.cols > (1u << 20)) {
    set_error("more than 2^20 columns are not supported");
    return TQ_E_UNSUPPORTED;
  }
  const uint64_t n_slots = (uint64_t)h.n_quads * kUnitPanels;
  m.x_dwords = (uint32_t)((n_slots - 1) * m.x_span + std::max<uint64_t>(m.x_span, (uint64_t)facts.max_lane_reach + 1));
  uint32_t x_off, slot_off;
  size_t lds_total;
  if (!plan_matvec_lds(m.dict_words, m.x_dwords, &x_off, &slot_off, &lds_total)) {
    set_error("a dictionary of " + std::to_string(h.n_entries) + " entries and a row of " + std::to_string(h.cols) +
              " activations (segments of " + std::to_string(h.seg_cols) + " columns) need " + std::to_string(lds_total) +
              " bytes of LDS; the device has " + std::to_string(kLdsLimit));
    return TQ_E_UNSUPPORTED;
  }
  // tq_decompress and the batched product: 16-bit dictionary image plus one tile of 64 strips per wavefront.
  if (round_up((uint64_t)m.dict_words * 2, 16) + (size_t)64 * (h.seg_cols + 8) > kLdsLimit) {
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
  // Dynamic LDS above 64 KB has to be allowed per kernel function.
  e = hipFuncSetAttribute((const void*)k_matvec<kDotPiece, kDotWaves, false>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsLimit);
  if (e == hipSuccess) e = hipFuncSetAttribute((const void*)k_matvec<kDotPiecePacked, kDotWavesPacked, true>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsLimit);
  if (e == hipSuccess) e = hipFuncSetAttribute((const void*)k_decompress, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsLimit);
  if (e == hipSuccess) e = hipFuncSetAttribute((const void*)k_matvec_mfma<true, false>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsLimit);
  if (e == hipSuccess) e = hipFuncSetAttribute((const void*)k_matvec_mfma<false, false>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsLimit);
  if (e == hipSuccess) e = hipFuncSetAttribute((const void*)k_matvec_mfma<true, true>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsLimit);
  if (e == hipSuccess) e = hipFuncSetAttribute((const void*)k_matvec_mfma<false, true>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsLimit);
  if (e == hipSuccess) e = hipFuncSetAttribute((const void*)k_matvec_ring<kRingWaves, 16, false>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsLimit);
  if (e == hipSuccess) e = hipFuncSetAttribute((const void*)k_matvec_ring<kRingWavesHalf, 8, false>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsLimit);
  if (e == hipSuccess) e = hipFuncSetAttribute((const void*)k_matvec_ring<kRingWaves, 16, true>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsLimit);
  if (e == hipSuccess) e = hipFuncSetAttribute((const void*)k_matvec_ring<kRingWavesHalf, 8, true>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsLimit);
  if (e == hipSuccess) e = hipFuncSetAttribute((const void*)k_matvec_ring<kRingWavesMore, 8, false>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsLimit);
  if (e == hipSuccess) e = hipFuncSetAttribute((const void*)k_matvec_ring<kRingWavesMore, 8, true>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsLimit);
  if (e != hipSuccess) return hip_fail("hipFuncSetAttribute(MaxDynamicSharedMemorySize)", e);

  const uint8_t* src = (const uint8_t*)blob;
  DictCopy* dict = nullptr;
  if (int rc = acquire_dictionary(dev, (const uint32_t*)(src + h.off_dict), h.n_entries + 1, m.dict_words, h.packing, &dict)) return rc;

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
  uint32_t dict_words_max = 0, x_dwords_max = 0, seg_max = 0;
  uint64_t cost = 0, bands = 0, band_cost_max = 1;
  bool x_fast = true;
  for (int i = 0; i < n; ++i) {
    const tq_matrix* t = hs[i];
    if (rec) {
      rec->entries.push_back(StepEntry{t->m, xs ? (const uint16_t*)xs[i] : nullptr, (float*)ys[i]});
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
  if (op == Op::kMatvec && batch == 1) {
    if (!plan_matvec_lds(dict_words_max, x_dwords_max, &a.x_off, &a.slot_off, &p.lds)) {
      set_error("the matrices of this call together need " + std::to_string(p.lds) + " bytes of LDS (largest dictionary plus longest row)");
      return TQ_E_UNSUPPORTED;
    }
    p.kernel = packed ? (const void*)k_matvec<kDotPiecePacked, kDotWavesPacked, true> : (const void*)k_matvec<kDotPiece, kDotWaves, false>;
    p.block = (packed ? kDotWavesPacked : kDotWaves) * 64;
  } else if (ring) {
    // LDS: 16-bit dictionary image | one ring per lane (aligned to its size: the kernel ORs piece offsets into its
    // address) | the activation tile of one quad.
    const size_t dict16 = round_up((uint64_t)dict_words_max * 2, kRingBytes);
    a.x_off = (uint32_t)dict16;
    a.tile_area = 64 * kRingBytes;
    const bool half = batch <= 8;   // 8 batch rows in the tile: room for two more wavefronts
    const bool more = half && dict16 + (size_t)kRingWavesMore * a.tile_area + ring_x_tile(8) + 128 <= kLdsLimit;   // a smaller dictionary leaves room
    const int waves = more ? kRingWavesMore : half ? kRingWavesHalf : kRingWaves;
    a.slot_off = (uint32_t)(dict16 + (size_t)waves * a.tile_area);
    p.lds = a.slot_off + ring_x_tile(half ? 8 : 16) + 128;   // + the band counter
    if (p.lds > kLdsLimit || !x_fast) {
      set_error("internal: ring launch with a dictionary or activations that do not fit it");
      return TQ_E_UNSUPPORTED;
    }
    if (more) p.kernel = packed ? (const void*)k_matvec_ring<kRingWavesMore, 8, true> : (const void*)k_matvec_ring<kRingWavesMore, 8, false>;
    else if (half) p.kernel = packed ? (const void*)k_matvec_ring<kRingWavesHalf, 8, true> : (const void*)k_matvec_ring<kRingWavesHalf, 8, false>;
    else p.kernel = packed ? (const void*)k_matvec_ring<kRingWaves, 16, true> : (const void*)k_matvec_ring<kRingWaves, 16, false>;
    p.block = (unsigned)waves * 64;
  } else {
    // Tile decode.  LDS: 16-bit dictionary image | one tile (64 strips) per wavefront, which the batched product reuses
    // for its partial sums (per wavefront two slots of 1 KB and their two band numbers).
    const size_t dict16 = round_up((uint64_t)dict_words_max * 2, 16);
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
    if (op == Op::kDecompress) p.kernel = (const void*)k_decompress;
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
// Bands per CU a launch needs for the ring kernel; TQ_RING_MIN_BANDS_PER_CU overrides it (tests use 0 to put small
// matrices through that kernel).
uint64_t ring_min_bands_per_cu() {
  if (const char* e = std::getenv("TQ_RING_MIN_BANDS_PER_CU")) return std::strtoull(e, nullptr, 10);
  return kRingMinBandsPerCu;
}

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
  if (op == Op::kMatvec) {
    // The product kernels are built once per weight format: matrices of packed 4-bit weights and the others take
    // separate launches.
    int n_packed = 0;
    for (int i = 0; i < n; ++i) n_packed += hs[i]->m.packing ? 1 : 0;
    if (n_packed != 0 && n_packed != n) {
      for (uint32_t want = 0; want < 2; ++want) {
        std::vector<tq_handle> h2;
        std::vector<const void*> x2;
        std::vector<void*> y2;
        for (int i = 0; i < n; ++i)
          if ((hs[i]->m.packing ? 1u : 0u) == want) {
            h2.push_back(hs[i]);
            x2.push_back(xs[i]);
            y2.push_back(ys[i]);
          }
        if (int rc = launch_all(op, (int)h2.size(), h2.data(), x2.data(), y2.data(), batch, stream, ring, gate_up, rec)) return rc;
      }
      return TQ_OK;
    }
  }
  if (op == Op::kMatvec && batch > 1 && !ring && !gate_up) {   // (the ring kernel adds partial sums to y: no place for silu)
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

extern "C" int tq_matvec(tq_handle h, const void* x, void* y, int batch, void* stream) {
  if (!h || !x || !y) {
    set_error("tq_matvec: null argument");
    return TQ_E_INVALID_ARG;
  }
  if (int rc = check_call("tq_matvec", 1, &h, &x, &y, batch)) return rc;
  return launch(Op::kMatvec, 1, &h, &x, &y, batch, (hipStream_t)stream,
                batch > 1 && ring_eligible(h, x) && h->m.n_bands >= ring_min_bands_per_cu() * h->n_cu);
}

extern "C" int tq_matvec_multi(int n, const tq_handle* hs, const void* const* xs, void* const* ys, int batch, void* stream) {
  if (n < 1 || !hs || !xs || !ys) {
    set_error("tq_matvec_multi: null argument or n < 1");
    return TQ_E_INVALID_ARG;
  }
  if (int rc = check_call("tq_matvec_multi", n, hs, xs, ys, batch)) return rc;
  return launch_all(Op::kMatvec, n, hs, xs, ys, batch, (hipStream_t)stream);
}

extern "C" int tq_matvec_gate_up_multi(int n, const tq_handle* hs, const void* const* xs, void* const* ys, int batch, void* stream) {
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

extern "C" int tq_matvec_gate_up(tq_handle h, const void* x, void* y, int batch, void* stream) {
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
};

extern "C" int tq_step_create(int n, const tq_handle* hs, const void* const* xs, void* const* ys, int batch, uint32_t flags,
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

extern "C" int tq_step_launch(tq_step_handle s, void* stream) {
  if (!s) {
    set_error("tq_step_launch: null step");
    return TQ_E_INVALID_ARG;
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
  out->table_bytes = (uint64_t)s->n_entries * sizeof(StepEntry);
  return TQ_OK;
}

extern "C" int tq_step_destroy(tq_step_handle s) {
  if (!s) return TQ_OK;
  hipError_t e = hipFree(s->table_dev);
  delete s;
  if (e != hipSuccess) return hip_fail("tq_step_destroy", e);
  return TQ_OK;
}

extern "C" int tq_decompress(tq_handle h, void* out, void* stream) {
  if (!h || !out) {
    set_error("tq_decompress: null argument");
    return TQ_E_INVALID_ARG;
  }
  return launch(Op::kDecompress, 1, &h, nullptr, &out, 1, (hipStream_t)stream);
}

extern "C" int tq_decompress_multi(int n, const tq_handle* hs, void* const* outs, void* stream) {
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

extern "C" int tq_destroy(tq_handle h) {
  if (!h) return TQ_OK;
  hipError_t e = hipFree(h->dev_base);
  hipError_t e2 = release_dictionary(h->dict);
  delete h;
  if (e != hipSuccess) return hip_fail("hipFree", e);
  if (e2 != hipSuccess) return hip_fail("hipFree", e2);
  return TQ_OK;
}
