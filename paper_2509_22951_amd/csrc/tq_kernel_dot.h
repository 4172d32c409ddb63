// Device side of libtq: the dot-product kernel for one or two activation rows (dictionary lookup, activation gather,
// one dot product per code and row).
#pragma once
#include "tq_kernels_common.h"

namespace tq {
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
template <bool kAligned, int kThreads, int kXRegs, bool kCoherent = false>   // kXRegs x kThreads x 2 columns per round (8192)
__device__ __forceinline__ void issue_activations(const DevMat& m, const uint16_t* __restrict__ x, uint32_t first_pair, int tid,
                                                  uint32_t (&lo)[kXRegs], uint32_t (&hi)[kXRegs]) {
#pragma unroll
  for (int k = 0; k < kXRegs; ++k) {
    const uint32_t j = first_pair + k * kThreads + tid, col = 2 * j;
    if (kAligned) {   // x is 4-byte aligned and cols is even
      lo[k] = col < m.cols ? x_load<kCoherent>((const uint32_t*)x + j) : 0u;
      hi[k] = col + 2 < m.cols ? x_load<kCoherent>((const uint32_t*)x + j + 1) : 0u;
    } else {
      lo[k] = (col < m.cols ? x_load<kCoherent>(x + col) : 0u) | (col + 1 < m.cols ? x_load<kCoherent>(x + col + 1) << 16 : 0u);
      hi[k] = col + 2 < m.cols ? x_load<kCoherent>(x + col + 2) : 0u;
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
template <int kThreads, int kDwords = 1>   // kDwords: dwords per column of the image (2: two rows of packed weights)
__device__ __forceinline__ void zero_activation_gaps(const DevMat& m, int tid, uint32_t* lds_x, uint32_t n_slots) {
  const uint32_t gap = m.x_span - m.seg_cols;
  constexpr uint32_t kGap = 16 * kDwords;
  if (gap)   // gap is 16 columns
    for (uint32_t i = tid; i < n_slots * kGap; i += kThreads) lds_x[kDwords * ((i / kGap) * m.x_span + m.seg_cols) + i % kGap] = 0u;
  for (uint32_t i = kDwords * n_slots * m.x_span + tid; i < kDwords * m.x_dwords; i += kThreads) lds_x[i] = 0u;
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
__device__ __forceinline__ uint32_t advance_by_wide_pair(uint32_t pair, uint32_t xa) {   // xa + 8 * pair: an image of 8 bytes per column
  uint32_t r;
  asm("v_lshl_add_u32 %0, %1, 3, %2" : "=v"(r) : "v"(pair), "v"(xa));
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
template <bool kAligned, int kThreads, int kXRegs, bool kCoherent = false>
__device__ __forceinline__ void issue_activations_packed(const DevMat& m, const uint16_t* __restrict__ x, uint32_t first, int tid,
                                                         uint32_t (&v)[kXRegs]) {
#pragma unroll
  for (int k = 0; k < kXRegs; ++k) {
    const uint32_t j = first + k * kThreads + tid;
    if (kAligned) v[k] = j < m.cols ? x_load<kCoherent>((const uint32_t*)x + j) : 0u;   // x is 4-byte aligned
    else v[k] = j < m.cols ? x_load<kCoherent>(x + 2 * j) | x_load<kCoherent>(x + 2 * j + 1) << 16 : 0u;
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

// Two activation rows of packed weights.  The image holds two dwords per byte column: the two activations of that byte
// in row 0, then those in row 1; a code reads the 16 bytes of its byte column and the next one at xa + 8 k, and each
// half of the dictionary word, converted once, meets the dword of either row: a0 collects row 0, a1 row 1.
template <int kCode0>
__device__ __forceinline__ void chunk4_packed_two_read(uint2 c, uint32_t& xa, uint32_t (&w)[4], uint64_t (&x)[8]) {
  w[0] = lds_read32(word_offset_lo(c.x));
  w[1] = lds_read32(word_offset_hi(c.x));
  w[2] = lds_read32(word_offset_lo(c.y));
  w[3] = lds_read32(word_offset_hi(c.y));
  x[0] = lds_read64_off<8 * kCode0>(xa);
  x[1] = lds_read64_off<8 * kCode0 + 8>(xa);
  xa = advance_by_wide_pair(is_pair_lo(c.x), xa);
  x[2] = lds_read64_off<8 * kCode0 + 8>(xa);
  x[3] = lds_read64_off<8 * kCode0 + 16>(xa);
  xa = advance_by_wide_pair(is_pair_hi(c.x), xa);
  x[4] = lds_read64_off<8 * kCode0 + 16>(xa);
  x[5] = lds_read64_off<8 * kCode0 + 24>(xa);
  xa = advance_by_wide_pair(is_pair_lo(c.y), xa);
  x[6] = lds_read64_off<8 * kCode0 + 24>(xa);
  x[7] = lds_read64_off<8 * kCode0 + 32>(xa);
  xa = advance_by_wide_pair(is_pair_hi(c.y), xa);
}
__device__ __forceinline__ void chunk4_packed_two_dot(const uint32_t (&w)[4], const uint64_t (&x)[8], float& a0, float& a1) {
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const bf16x2 first = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w[k], 1.0f, false);   // the weights of the code's first byte
    const bf16x2 second = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w[k], 1.0f, true);   // of its second byte (zeros after a single)
    a0 = __builtin_amdgcn_fdot2_f32_bf16(first, __builtin_bit_cast(bf16x2, (uint32_t)x[2 * k]), a0, false);
    a1 = __builtin_amdgcn_fdot2_f32_bf16(first, __builtin_bit_cast(bf16x2, (uint32_t)(x[2 * k] >> 32)), a1, false);
    a0 = __builtin_amdgcn_fdot2_f32_bf16(second, __builtin_bit_cast(bf16x2, (uint32_t)x[2 * k + 1]), a0, false);
    a1 = __builtin_amdgcn_fdot2_f32_bf16(second, __builtin_bit_cast(bf16x2, (uint32_t)(x[2 * k + 1] >> 32)), a1, false);
  }
}
template <int kThreads, int kXRegs>
__device__ __forceinline__ void commit_activations_packed_two(const DevMat& m, uint32_t first, int tid, const uint32_t (&r0)[kXRegs],
                                                              const uint32_t (&r1)[kXRegs], uint32_t* lds_x, uint32_t image_cols) {
  const uint32_t gap = m.x_span - m.seg_cols;
#pragma unroll
  for (int k = 0; k < kXRegs; ++k) {
    const uint32_t j = first + k * kThreads + tid;
    if (j < image_cols) {
      const uint32_t i = 2 * (j + gap * __umulhi(j, m.seg_magic));
      lds_x[i] = r0[k];
      lds_x[i + 1] = r1[k];
    }
  }
}

// Two activation rows (batch 2).  The image holds one dword per column, (x0[c], x1[c]); a code reads the dwords of its
// column and of the next one (the reads of chunk4_packed_read), two byte permutes put each row's pair together, and one
// dot product per row follows: a0 collects row 0, a1 row 1.
__device__ __forceinline__ void chunk4_two_dot(const uint32_t (&w)[4], const uint32_t (&x)[8], float& a0, float& a1) {
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    a0 = dot2(w[k], __builtin_amdgcn_perm(x[2 * k + 1], x[2 * k], 0x05040100u), a0);   // (x0[c], x0[c + 1])
    a1 = dot2(w[k], __builtin_amdgcn_perm(x[2 * k + 1], x[2 * k], 0x07060302u), a1);   // (x1[c], x1[c + 1])
  }
}
// Thread t of a round handles the columns (2 j, 2 j + 1), j = first_pair + k * kThreads + t, of both rows.
template <bool kAligned, int kThreads, int kXRegs, bool kCoherent = false>   // kAligned: both rows start 4-byte aligned and cols is even
__device__ __forceinline__ void issue_activations_two(const DevMat& m, const uint16_t* __restrict__ x, uint32_t first_pair, int tid,
                                                      uint32_t (&r0)[kXRegs], uint32_t (&r1)[kXRegs]) {
  const uint16_t* x1 = x + m.cols;
#pragma unroll
  for (int k = 0; k < kXRegs; ++k) {
    const uint32_t j = first_pair + k * kThreads + tid, col = 2 * j;
    if (kAligned) {
      r0[k] = col < m.cols ? x_load<kCoherent>((const uint32_t*)x + j) : 0u;
      r1[k] = col < m.cols ? x_load<kCoherent>((const uint32_t*)x1 + j) : 0u;
    } else {
      r0[k] = (col < m.cols ? x_load<kCoherent>(x + col) : 0u) | (col + 1 < m.cols ? x_load<kCoherent>(x + col + 1) << 16 : 0u);
      r1[k] = (col < m.cols ? x_load<kCoherent>(x1 + col) : 0u) | (col + 1 < m.cols ? x_load<kCoherent>(x1 + col + 1) << 16 : 0u);
    }
  }
}
template <int kThreads, int kXRegs>
__device__ __forceinline__ void commit_activations_two(const DevMat& m, uint32_t first_pair, int tid, const uint32_t (&r0)[kXRegs],
                                                       const uint32_t (&r1)[kXRegs], uint32_t* lds_x, uint32_t image_cols) {
  const uint32_t gap = m.x_span - m.seg_cols;
#pragma unroll
  for (int k = 0; k < kXRegs; ++k) {
    const uint32_t col = 2 * (first_pair + k * kThreads + tid);
    if (col < image_cols) {   // image_cols and seg_cols are even: both columns lie in one panel
      const uint32_t i = col + gap * __umulhi(col, m.seg_magic);
      lds_x[i] = (r0[k] & 0xFFFFu) | r1[k] << 16;
      lds_x[i + 1] = r0[k] >> 16 | (r1[k] & 0xFFFF0000u);
    }
  }
}

// Containers with runs of up to 4 bytes (one activation row).  The dictionary image has one dword (two bf16 weights) per
// slot; an entry of 3 or 4 bytes takes two slots, so a code reads the two dwords at its slot (for a shorter entry the
// second one belongs to the next entry and is dropped), the activation pairs of its column and of the column two
// further on, and multiplies both; its run length follows from the code's place in the sorted code space.
// xa = LDS byte address of the activation pair of the lane's next column.
struct LongClasses {
  uint32_t class2, class3;
};
__device__ __forceinline__ void code_long_dot(uint32_t code, const LongClasses& cl, uint32_t& xa, float& a0, float& a1) {
  const uint32_t da = long_slot(code, cl.class2) << 2;
  const uint32_t w0 = lds_read32(da), w1 = lds_read32_off<4>(da);
  const uint32_t x0 = lds_read32(xa), x1 = lds_read32_off<8>(xa);
  a0 = dot2(w0, x0, a0);
  a1 = dot2(code >= cl.class2 ? w1 : 0u, x1, a1);
  xa += 4u * long_run_length(code, cl.class2, cl.class3);
}
__device__ __forceinline__ void chunk4_long(uint2 c, const LongClasses& cl, uint32_t& xa, float& a0, float& a1) {
  code_long_dot(c.x & 0xFFFFu, cl, xa, a0, a1);
  code_long_dot(c.x >> 16, cl, xa, a0, a1);
  code_long_dot(c.y & 0xFFFFu, cl, xa, a0, a1);
  code_long_dot(c.y >> 16, cl, xa, a0, a1);
}

// Sum of the four panel lanes of each row: afterwards every lane l holds the sum over lanes l % 16 + {0, 16, 32, 48}.
__device__ __forceinline__ float sum_over_panels(float v) {
  v += __shfl_xor(v, 16);
  v += __shfl_xor(v, 32);
  return v;
}

// The gated product of a feed-forward block: silu(gate) * up, silu(g) = g / (1 + exp(-g)).
__device__ __forceinline__ float silu_times(float gate, float up) { return gate / (1.f + __expf(-gate)) * up; }

// Fused decode + dequantize + matrix-vector product for one or two activation rows (kB) and up to kMaxMulti matrices
// (kMaxStep when the jobs come from a prepared step's table).
//
// The launch's work is the line of all bands (16 rows each) of all matrices, each band weighted by its number of
// weights; workgroup g takes the bands whose middle lies in the g-th equal share of that line, so a workgroup serves a
// contiguous range of whole bands of one matrix after the other.  Inside a matrix the units of those bands are
// contiguous in the code stream and are cut into one contiguous run per wavefront.  A wavefront owns every band that
// lies entirely inside its run (it scales and stores those rows itself); a band it shares with its neighbours goes to
// one of two partial-sum slots in LDS, and after a workgroup barrier the slots of a band are added in wavefront order,
// so the result does not depend on timing.
// kStaged: the jobs form stages (MatvecArgs::stage_first); the workgroups take the stages in turn, each one's bands cut
// into equal shares as above, with a grid-wide hand-over between two stages; the dictionary stays in LDS across them.
template <int kPiece, int kWaves, bool kPacked, int kB, bool kLong = false, bool kStaged = false>
__global__ __launch_bounds__(kWaves * 64, 1) void k_matvec(MatvecArgs a) {
  static_assert(kB == 1 || kB == 2, "one activation row or two");
  static_assert(!kLong || (kB == 1 && !kPacked), "runs of 3 and 4 bytes: one activation row of one-weight-per-byte matrices");
  constexpr int kImage = kPacked && kB == 2 ? 2 : 1;   // dwords of the activation image per column
  constexpr int kThreads = kWaves * 64, kDictRegs = 128 / kWaves, kXRegs = 64 / kWaves;
  extern __shared__ uint4 lds4[];
  uint32_t* lds_dict = (uint32_t*)lds4;
  uint32_t* lds_x = (uint32_t*)((uint8_t*)lds4 + a.x_off);
  float* slot_val = (float*)((uint8_t*)lds4 + a.slot_off);           // [2 * kWaves][kB][16]
  int* slot_band = (int*)(slot_val + 2 * kWaves * kB * 16);          // [2 * kWaves]
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const uint32_t* staged = nullptr;
  const uint32_t n_stages = kStaged ? a.n_stages : 1u;
  constexpr uint32_t kNoStage = 0xFFFFFFFFu;
  uint32_t wait_for = kNoStage;   // staged: the stage whose outputs this workgroup has yet to wait for
  for (uint32_t stage = 0; stage < n_stages; ++stage) {
  const int job_first = kStaged ? (int)((const_u32*)a.stage_first)[stage] : 0, job_end = kStaged ? (int)((const_u32*)a.stage_first)[stage + 1] : a.n;
  const uint32_t cost_first = cost_at(a, job_first);
  const uint64_t total = cost_at(a, job_end) - cost_first;
  const uint32_t lo = cost_first + (uint32_t)(total * blockIdx.x / gridDim.x), hi = cost_first + (uint32_t)(total * (blockIdx.x + 1) / gridDim.x);
  for (int i = job_first; i < job_end; ++i) {
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
    const uint32_t xa_lane = lds_address(lds_x) + 4u * kImage * m.x_span * (uint32_t)(lane >> 4);
    const uint32_t xa_quad = 16u * kImage * m.x_span;
    const bool x_aligned = (kPacked || m.cols % 2 == 0) && ((uintptr_t)job.x % 4 == 0);   // (cols even: a second row is aligned like the first)
    const uint32_t c0 = u0 < u1 ? unit_offset(m, u0) : 0u, n_chunks = u0 < u1 ? unit_offset(m, u1) - c0 : 0u;
    {   // one activation row, or two: larger batches run the MFMA kernels
      const uint16_t* xb = job.x;
      float* yb = job.y;
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
      // The first piece of code chunks is requested here, ahead of the staging of dictionary and activations: the
      // chunks then arrive while the workgroup stages, and a small launch does not wait for device memory twice in a row.
      uint2 cwa[kPiece], cwb[kPiece];
      uint32_t sa = c0, na = 0, sb, nb;
      bool ea = false, eb;
      if (u0 < u1) {
        next_piece(sa, na, ea);
        load_piece(cwa, sa, na);
      }
      // the previous dictionary, activation image and slots are no longer in use; staged: nor is anyone still writing
      // the activations (the wait ends with the same barrier)
      if (kStaged && wait_for != kNoStage) {
        stage_wait(a, wait_for);
        wait_for = kNoStage;
      } else {
        __syncthreads();
      }
      {
        uint4 dv[kDictRegs];
        uint32_t xlo[kXRegs], xhi[kXRegs];
        const bool dict_now = new_dict;
        if (dict_now) issue_dictionary<kThreads, kDictRegs>(m, 0, tid, dv);
        if constexpr (kPacked) {
          if (x_aligned) issue_activations_packed<true, kThreads, kXRegs, kStaged>(m, xb, 0, tid, xlo);
          else issue_activations_packed<false, kThreads, kXRegs, kStaged>(m, xb, 0, tid, xlo);
          if constexpr (kB == 2) {   // the second row starts 2 * cols activations later, aligned like the first
            if (x_aligned) issue_activations_packed<true, kThreads, kXRegs, kStaged>(m, xb + 2 * m.cols, 0, tid, xhi);
            else issue_activations_packed<false, kThreads, kXRegs, kStaged>(m, xb + 2 * m.cols, 0, tid, xhi);
          }
        } else if constexpr (kB == 2) {
          if (x_aligned) issue_activations_two<true, kThreads, kXRegs, kStaged>(m, xb, 0, tid, xlo, xhi);
          else issue_activations_two<false, kThreads, kXRegs, kStaged>(m, xb, 0, tid, xlo, xhi);
        } else {
          if (x_aligned) issue_activations<true, kThreads, kXRegs, kStaged>(m, xb, 0, tid, xlo, xhi);
          else issue_activations<false, kThreads, kXRegs, kStaged>(m, xb, 0, tid, xlo, xhi);
        }
        zero_activation_gaps<kThreads, kImage>(m, tid, lds_x, n_slots);
        if (tid < 2 * kWaves) slot_band[tid] = -1;
        if (dict_now) {
          commit_dictionary<kThreads, kDictRegs>(m, 0, tid, dv, lds_dict);
          for (uint32_t base = kDictRegs * kThreads; base < m.dict_words / 4; base += kDictRegs * kThreads) {
            issue_dictionary<kThreads, kDictRegs>(m, base, tid, dv);
            commit_dictionary<kThreads, kDictRegs>(m, base, tid, dv, lds_dict);
          }
        }
        if constexpr (kPacked && kB == 2) {
          commit_activations_packed_two<kThreads, kXRegs>(m, 0, tid, xlo, xhi, lds_x, image_cols);
          for (uint32_t first = kXRegs * kThreads; first < image_cols; first += kXRegs * kThreads) {
            if (x_aligned) {
              issue_activations_packed<true, kThreads, kXRegs, kStaged>(m, xb, first, tid, xlo);
              issue_activations_packed<true, kThreads, kXRegs, kStaged>(m, xb + 2 * m.cols, first, tid, xhi);
            } else {
              issue_activations_packed<false, kThreads, kXRegs, kStaged>(m, xb, first, tid, xlo);
              issue_activations_packed<false, kThreads, kXRegs, kStaged>(m, xb + 2 * m.cols, first, tid, xhi);
            }
            commit_activations_packed_two<kThreads, kXRegs>(m, first, tid, xlo, xhi, lds_x, image_cols);
          }
        } else if constexpr (kPacked) {
          commit_activations_packed<kThreads, kXRegs>(m, 0, tid, xlo, lds_x, image_cols);
          for (uint32_t first = kXRegs * kThreads; first < image_cols; first += kXRegs * kThreads) {
            if (x_aligned) issue_activations_packed<true, kThreads, kXRegs, kStaged>(m, xb, first, tid, xlo);
            else issue_activations_packed<false, kThreads, kXRegs, kStaged>(m, xb, first, tid, xlo);
            commit_activations_packed<kThreads, kXRegs>(m, first, tid, xlo, lds_x, image_cols);
          }
        } else if constexpr (kB == 2) {
          commit_activations_two<kThreads, kXRegs>(m, 0, tid, xlo, xhi, lds_x, image_cols);
          for (uint32_t first = kXRegs * kThreads; 2 * first < image_cols; first += kXRegs * kThreads) {
            if (x_aligned) issue_activations_two<true, kThreads, kXRegs, kStaged>(m, xb, first, tid, xlo, xhi);
            else issue_activations_two<false, kThreads, kXRegs, kStaged>(m, xb, first, tid, xlo, xhi);
            commit_activations_two<kThreads, kXRegs>(m, first, tid, xlo, xhi, lds_x, image_cols);
          }
        } else {
          commit_activations<kThreads, kXRegs>(m, 0, tid, xlo, xhi, lds_x, image_cols);
          for (uint32_t first = kXRegs * kThreads; 2 * first < image_cols; first += kXRegs * kThreads) {
            if (x_aligned) issue_activations<true, kThreads, kXRegs, kStaged>(m, xb, first, tid, xlo, xhi);
            else issue_activations<false, kThreads, kXRegs, kStaged>(m, xb, first, tid, xlo, xhi);
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
          // one activation row: a0 and a1 are two chains of the same sum; two rows: one sum each
          float v[kB];
          if constexpr (kB == 1) {
            v[0] = sum_over_panels(a0 + a1);
          } else {
            v[0] = sum_over_panels(a0);
            v[1] = sum_over_panels(a1);
          }
          if (complete) {
            const uint32_t row = band * kUnitRows + lane;
#pragma unroll
            for (int b = 0; b < kB; ++b) {
              if (a.gate_up) {   // lanes 2r, 2r + 1 hold the gate and the up row of output r
                const float t = v[b] * scale, other = __shfl_xor(t, 1);
                if (lane < 16 && !(lane & 1) && row + 1 < m.rows) y_store<kStaged>(yb + (size_t)b * (m.rows / 2) + row / 2, silu_times(t, other));
              } else if (lane < 16 && row < m.rows) {
                y_store<kStaged>(yb + (size_t)b * m.rows + row, v[b] * scale);
              }
            }
          } else {
            const int s = 2 * wave + (whole ? 1 : 0);   // slot 2w: band begun by an earlier wavefront; 2w + 1: band left unfinished
#pragma unroll
            for (int b = 0; b < kB; ++b)
              if (lane < 16) slot_val[(s * kB + b) * 16 + lane] = v[b];
            if (lane == 0) slot_band[s] = (int)band;
          }
        };
        auto run_piece = [&](const uint2 (&cw)[kPiece], uint32_t n, bool ends) {
          // kSets register sets: the operands of the next kSets - 1 chunks are read while one chunk is multiplied, so a
          // wavefront that works alone (a small launch, the tail of a stage) does not sit out an LDS round trip per chunk
          constexpr int kSets = kDotSets;
          uint32_t w[kSets][4];
          std::conditional_t<kImage == 2, uint64_t, uint32_t> x[kSets][8];
          auto read = [&](auto kk) {
            constexpr int k = decltype(kk)::value;
            if constexpr (kImage == 2) chunk4_packed_two_read<4 * k>(cw[k], xa, w[k % kSets], x[k % kSets]);
            else if constexpr (kPacked || kB == 2) chunk4_packed_read<4 * k>(cw[k], xa, w[k % kSets], x[k % kSets]);   // this dword and the next
            else chunk4_read<4 * k>(cw[k], xa, w[k % kSets], x[k % kSets]);
          };
          auto dot = [&](auto kk) {
            constexpr int k = decltype(kk)::value;
            if constexpr (kImage == 2) chunk4_packed_two_dot(w[k % kSets], x[k % kSets], a0, a1);
            else if constexpr (kPacked) chunk4_packed_dot(w[k % kSets], x[k % kSets], a0, a1);
            else if constexpr (kB == 2) chunk4_two_dot(w[k % kSets], x[k % kSets], a0, a1);
            else chunk4_dot(w[k % kSets], x[k % kSets], a0, a1);
          };
          auto straight = [&](auto nn) {   // a piece of nn chunks as straight-line code
            constexpr int kN = decltype(nn)::value;
            static_for<(kSets - 1 < kN ? kSets - 1 : kN)>([&](auto kk) { read(kk); });
            static_for<kN>([&](auto kk) {
              constexpr int k = decltype(kk)::value;
              if constexpr (k + kSets - 1 < kN) read(std::integral_constant<int, k + kSets - 1>{});
              dot(kk);
            });
          };
          if constexpr (kLong) {
            const LongClasses cl = {m.class2, m.class3};
            static_for<kPiece>([&](auto kk) {
              if ((uint32_t)decltype(kk)::value < n) chunk4_long(cw[decltype(kk)::value], cl, xa, a0, a1);
            });
          } else if (n == kPiece) {
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
          if constexpr (!kLong) xa += 16 * kImage * n;   // (the long form keeps xa at the lane's column itself)
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
      if (tid < 2 * kWaves * kB * 16) {   // one thread per slot, activation row and row of the band
        const int s = tid / (16 * kB), b = (tid >> 4) % kB, r16 = tid & 15;
        const int bnd = slot_band[s];
        bool first = bnd >= 0;
        for (int t = 0; t < s; ++t) first = first && slot_band[t] != bnd;
        if (first) {
          float sum = slot_val[(s * kB + b) * 16 + r16];
          for (int t = s + 1; t < 2 * kWaves; ++t)
            if (slot_band[t] == bnd) sum += slot_val[(t * kB + b) * 16 + r16];
          const uint32_t row = (uint32_t)bnd * kUnitRows + r16;
          if (a.gate_up) {   // the two threads of a pair of rows are neighbours and take this branch together
            const float t = sum * global_load(m.scales + min(row, m.rows - 1)), other = __shfl_xor(t, 1);
            if (!(r16 & 1) && row + 1 < m.rows) y_store<kStaged>(yb + (size_t)b * (m.rows / 2) + row / 2, silu_times(t, other));
          } else if (row < m.rows) {
            y_store<kStaged>(yb + (size_t)b * m.rows + row, sum * global_load(m.scales + row));
          }
        }
      }
    }
  }
  if (kStaged && stage + 1 < n_stages) {
    stage_arrive(a, stage);
    wait_for = stage;
  }
  }
}

}  // namespace tq
