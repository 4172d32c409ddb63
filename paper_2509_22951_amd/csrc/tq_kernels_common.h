// Device side of libtq: constants, kernel-argument structures and the small device helpers every kernel uses.
#pragma once
#include <hip/hip_runtime.h>

#include <cstddef>
#include <cstdint>
#include <utility>

#include "../../include/tq.h"
#include "tq_format.h"

namespace tq {

constexpr int kWaves = 8;            // most wavefronts per workgroup of the tile kernels (one workgroup per CU: LDS-bound)
constexpr int kThreads = kWaves * 64;
constexpr int kDotWavesPacked = 12;  // the same kernel for packed 4-bit weights: more work per byte read, more wavefronts to
                                     // hide it (config 4, ms per step: 8 wavefronts 0.379, 12 0.370, 16 0.379)
#ifndef TQ_STAGED_WAVES
#define TQ_STAGED_WAVES 8
#endif
constexpr int kDotWavesStaged = TQ_STAGED_WAVES;   // the staged form of the batch-1 and batch-2 kernel (the 113 dependent stages
                                                   // of the 3B sweep, ms per step: 8 wavefronts 1.59, 12 1.87, 16 1.88)
constexpr int kDotWavesMax = kDotWavesStaged > 12 ? kDotWavesStaged : 12;
constexpr int kDotPiecePacked = 6;   // its units are half as long (segments of 128 bytes: 17 chunks, three pieces of 5 or 6)
constexpr int kDotWaves = 8;         // wavefronts per workgroup of the batch-1 kernel (measured on the 3B sweep, TB/s:
                                     // 6 waves 4.61, 8 waves 5.12, 10 waves 4.64, 12 waves 4.90, 16 waves 4.28)
constexpr int kDotPiece = 8;         // chunks per piece in the batch-1 kernel: two pieces (16 x 512 bytes) are in flight per
                                     // wavefront (measured on the 3B sweep, TB/s: 4 chunks 5.30, 6 5.48, 8 5.47, 12 5.41, 18 5.24)
#ifndef TQ_DOT_SETS
#define TQ_DOT_SETS 2
#endif
constexpr int kDotSets = TQ_DOT_SETS;   // register sets of the batch-1 kernel's chunk pipeline (operands read kDotSets - 1 chunks ahead)
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
  uint32_t long_runs;      // 1: runs of 3 and 4 bytes exist (lmax > 2): the code space classes below apply, and dict / dict_bf16
                           // point to images with two slots for every entry from `class2` on (see long_slot)
  uint32_t class2, class3; // codes from class2 on are runs of at least 3 bytes, from class3 on of 4 (sorted code space)
  uint32_t dict16_bytes;   // long_runs: size of the byte image at `dict` (a multiple of 16)
};
static_assert(sizeof(DevMat) % 8 == 0, "copied as whole dwords, kept 8-byte aligned in tables");

// Containers with runs of up to 4 bytes keep a dictionary image with one slot for an entry of up to 2 bytes and two
// slots for a longer one, the long ones starting on an even slot: slot index of a code.
__device__ __forceinline__ uint32_t long_slot(uint32_t code, uint32_t class2) {
  const uint32_t even = class2 & ~1u;
  return code + (code > even ? code - even : 0u);   // codes below class2 never exceed `even` by more than 0: class2 - 1 <= even
}
// Run length of a code by its place in the sorted code space (the pad code, past the last entry, counts as 4).
__device__ __forceinline__ uint32_t long_run_length(uint32_t code, uint32_t class2, uint32_t class3) {
  return 1u + (code >= 256u ? 1u : 0u) + (code >= class2 ? 1u : 0u) + (code >= class3 ? 1u : 0u);
}

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
  // A staged step (one launch for products that depend on each other): the jobs come in n_stages groups, jobs
  // stage_first[s] .. stage_first[s + 1] - 1 form stage s, and no workgroup starts a stage before every workgroup has
  // stored the results of the one before (grid-wide hand-over through sync[s]; sync[n_stages] is set when a wait gave up).
  const uint32_t* stage_first;   // device, n_stages + 1 entries; null: not staged
  uint32_t* sync;                // device, n_stages + 1 words, zero at launch
  uint32_t* fault_host;          // host memory the device can write: set to 1 when a wait gave up
  uint32_t n_stages;
  uint32_t spin_limit;           // polls of a stage counter before a workgroup gives up
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
typedef __attribute__((address_space(3))) const uint64_t lds_cq64;
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

// The same accesses, coherent across the whole device without any cache maintenance: relaxed atomics at device scope
// are served at the level all compute units share.  A staged step stores its outputs and loads its activations this
// way, so that a hand-over between stages needs no write-back or invalidation of caches (those cost microseconds).
template <bool kCoherent>
__device__ __forceinline__ uint32_t x_load(const uint32_t* p) {
  if constexpr (kCoherent) return __hip_atomic_load((__attribute__((address_space(1))) const uint32_t*)p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  else return global_load(p);
}
template <bool kCoherent>
__device__ __forceinline__ uint32_t x_load(const uint16_t* p) {
  if constexpr (kCoherent) return __hip_atomic_load((__attribute__((address_space(1))) const uint16_t*)p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  else return global_load(p);
}
template <bool kCoherent>
__device__ __forceinline__ void y_store(float* p, float v) {
  if constexpr (kCoherent) __hip_atomic_store((__attribute__((address_space(1))) float*)p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  else global_store(p, v);
}

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

// Grid-wide hand-over between two stages of a staged step.  The stage's outputs were stored with device-coherent
// stores (y_store<true>); every wavefront waits until its own stores have been acknowledged, the workgroup meets at a
// barrier, one thread announces the workgroup at the stage's counter and polls it until all gridDim.x workgroups have
// arrived (relaxed device-scope atomics throughout: the counter and the data are coherent by the way they are accessed,
// so no cache is written back or invalidated).  The next stage loads its activations coherently too (x_load<true>).
// All workgroups of the launch must be resident together (the host launches at most one per compute unit).  The wait is
// bounded: after spin_limit polls, or when another workgroup has given up, the workgroup sets the fault words and
// goes on without waiting - the launch then ends with results that must not be used, and the host reports it.
// The hand-over comes in two halves so that a workgroup can fetch what its next stage needs and what no other workgroup
// writes (matrix descriptions, unit offsets, the first code chunks) between the two, while the others still finish.
// stage_arrive: this workgroup's outputs of `stage` are out.  stage_wait: every workgroup's are; it ends with a
// workgroup barrier.  A workgroup that has no share of a stage goes on to the next arrive without waiting: it reads
// and writes nothing there, and whatever it does later comes after a wait on a later stage.
__device__ __forceinline__ void stage_arrive(const MatvecArgs& a, uint32_t stage) {
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this wavefront's stores have reached the level the device shares
  __syncthreads();
  if (threadIdx.x == 0) __hip_atomic_fetch_add(a.sync + stage, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void stage_wait(const MatvecArgs& a, uint32_t stage) {
  if (threadIdx.x == 0) {
    uint32_t* counter = a.sync + stage;
    uint32_t* fault = a.sync + a.n_stages;
    uint32_t polls = 0;
    while (__hip_atomic_load(counter, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < gridDim.x) {
      if (++polls > a.spin_limit || __hip_atomic_load(fault, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) {
        __hip_atomic_store(fault, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(a.fault_host, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
        break;
      }
      __builtin_amdgcn_s_sleep(2);
    }
  }
  __syncthreads();
}

// Byte address inside LDS of a pointer into the workgroup's dynamic shared memory.
__device__ __forceinline__ uint32_t lds_address(const void* p) { return (uint32_t)(size_t)(const lds_u8*)p; }

// Pointer forms on purpose: the compiler tracks the outstanding LDS read and places the wait before the first use.
__device__ __forceinline__ uint32_t lds_read32(uint32_t addr) { return *(lds_cu32*)(size_t)addr; }
template <int kOff>
__device__ __forceinline__ uint32_t lds_read32_off(uint32_t addr) { return *(lds_cu32*)(size_t)(addr + kOff); }
template <int kOff>   // addr + kOff is 8-byte aligned
__device__ __forceinline__ uint64_t lds_read64_off(uint32_t addr) { return *(lds_cq64*)(size_t)(addr + kOff); }

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

}  // namespace tq
