// Device side of libtq for gfx950 (MI355X): handle management and the two hot-path kernels.
//
// Work decomposition.  The container stores the matrix as restart groups of 16 rows x 256 columns (4096 bytes,
// 32 micro-tiles of 16x8 in MFMA operand order).  One wavefront decodes one group at a time into a private 4 KB
// LDS tile, streaming the 16-bit codes in rounds of 512:
//   1. 64 lanes load 8 consecutive codes each (one coalesced 1 KB read per round, six rounds in flight),
//   2. look each code up in the LDS-resident dictionary (one 32-bit word: 3 run bytes + length in bits),
//   3. get the byte position of the lane's runs from a DPP wave scan of the lane totals,
//   4. pack the lane's 8 runs into one byte string in registers (v_alignbit funnel) and OR it into the zeroed tile
//      as a few aligned dwords (ds_or_b32), instead of one LDS byte store per decoded byte.
// The tile then holds 8 MFMA A-operand blocks (16 rows x 32 k).  tq_matvec converts each lane's 8 int8 values to
// bf16 (exact) and issues v_mfma_f32_16x16x32_bf16 against the activations (batch is the N dimension, up to 16);
// tq_decompress copies the tile out to the row-major int8 matrix with 16-byte stores.
// The expanded matrix never exists in HBM on the tq_matvec path.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstring>
#include <new>
#include <string>
#include <thread>

#include "../../include/tq.h"
#include "tq_format.h"

namespace tq {

constexpr int kWaves = 8;                      // wavefronts per workgroup (one workgroup per CU: LDS-bound occupancy)
constexpr int kThreads = kWaves * 64;
constexpr uint32_t kTileStride = kGroupBytes + 16;
constexpr uint32_t kLdsLimit = 160 * 1024;

struct DevMat {
  const uint32_t* dict;
  const uint32_t* goff;
  const uint16_t* codes;
  const float* scales;
  uint32_t rows, cols;
  uint32_t n_bands, n_strips;
  uint32_t dict_words_pad;   // dictionary words staged into LDS (multiple of 4, zero filled past n_entries + 1)
  uint32_t pad_word;         // two pad codes in one dword
  uint64_t n_groups;
};

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

template <int kCtrl, int kRowMask>
__device__ __forceinline__ uint32_t dpp_add(uint32_t x) {
  return x + (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, kCtrl, kRowMask, 0xf, true);
}

// Inclusive prefix sum over the 64 lanes of a wavefront (row shifts inside rows of 16, then row broadcasts).
__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t x) {
  x = dpp_add<0x111, 0xf>(x);   // row_shr:1
  x = dpp_add<0x112, 0xf>(x);   // row_shr:2
  x = dpp_add<0x114, 0xf>(x);   // row_shr:4
  x = dpp_add<0x118, 0xf>(x);   // row_shr:8
  x = dpp_add<0x142, 0xa>(x);   // row_bcast:15 into rows 1 and 3
  x = dpp_add<0x143, 0xc>(x);   // row_bcast:31 into rows 2 and 3
  return x;
}

// Copy the dictionary into LDS.  The loads of a batch of 8 x 8 KB are all issued before the first LDS write, so the
// whole copy exposes two memory latencies instead of one per 8 KB.
__device__ __forceinline__ void stage_dictionary(const DevMat& m, uint4* lds4, int tid) {
  const uint4* src = (const uint4*)m.dict;
  const uint32_t n4 = m.dict_words_pad / 4;
  constexpr int kBatch = 8;
  for (uint32_t base = 0; base < n4; base += kBatch * kThreads) {
    uint4 v[kBatch];
#pragma unroll
    for (int k = 0; k < kBatch; ++k) {
      const uint32_t i = base + k * kThreads + tid;
      v[k] = src[min(i, n4 - 1)];
    }
#pragma unroll
    for (int k = 0; k < kBatch; ++k) {
      const uint32_t i = base + k * kThreads + tid;
      if (i < n4) lds4[i] = v[k];
    }
  }
  __syncthreads();
}

typedef __attribute__((address_space(3))) uint8_t lds_u8;
typedef __attribute__((address_space(4))) const uint32_t const_u32;

// Group offsets are wave-uniform and never written while a kernel runs: reading them through the constant address
// space makes them scalar loads, which do not share a counter with the vector loads of the code stream.
__device__ __forceinline__ uint32_t group_offset(const DevMat& m, uint32_t g) { return ((const_u32*)m.goff)[g]; }

// Byte address inside LDS of a pointer into the workgroup's dynamic shared memory.
__device__ __forceinline__ uint32_t lds_address(const void* p) { return (uint32_t)(size_t)(const lds_u8*)p; }

typedef __attribute__((address_space(3))) const uint32_t lds_cu32;

// LDS byte address of dictionary word `code`, for the code in the low / high half of a packed code pair:
// one SDWA shift (selects the 16-bit half, zero-extends, multiplies by 4) instead of a mask and a shift.
__device__ __forceinline__ uint32_t dict_address_lo(uint32_t pair, uint32_t two, uint32_t dict_base) {
  uint32_t a;
  asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_0" : "=v"(a) : "v"(two), "v"(pair));
  return a + dict_base;
}
__device__ __forceinline__ uint32_t dict_address_hi(uint32_t pair, uint32_t two, uint32_t dict_base) {
  uint32_t a;
  asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_1" : "=v"(a) : "v"(two), "v"(pair));
  return a + dict_base;
}
__device__ __forceinline__ uint32_t lds_read32(uint32_t addr) { return *(lds_cu32*)(size_t)addr; }

__device__ __forceinline__ void compiler_barrier() { asm volatile("" ::: "memory"); }

constexpr int kRoundCodes = 512;   // 64 lanes x 8 consecutive codes (one 16-byte load per lane)
constexpr int kDepth = 6;          // rounds of code loads kept in flight per wavefront (6 x 1 KB)

// The 8 runs of a lane are consecutive in the output, so they are first packed into one contiguous byte string in
// registers.  A dictionary word holds the run bytes in bits 0..23 and the run length in bits (8/16/24) in its top
// byte; v_alignbit(word, acc, len) shifts the accumulator right by the run length and inserts exactly the run's
// bytes at the top, whatever sits above them in the word.  After the 8 steps the string is top-justified in
// A[0 .. 2*kLmax).  Only the dwords that can be non-zero after each step are touched.
template <int kLmax>
__device__ __forceinline__ void pack_runs(const uint32_t (&s)[8], uint32_t (&A)[2 * kLmax]) {
  constexpr int ND = 2 * kLmax;
#pragma unroll
  for (int k = 0; k < ND; ++k) A[k] = 0;
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const uint32_t len = s[j] >> 24;
    const int live = (kLmax * (j + 1) + 3) / 4 < ND ? (kLmax * (j + 1) + 3) / 4 : ND;   // dwords in use after this step
#pragma unroll
    for (int k = ND - live; k < ND - 1; ++k) A[k] = __builtin_amdgcn_alignbit(A[k + 1], A[k], len);
    A[ND - 1] = __builtin_amdgcn_alignbit(s[j], A[ND - 1], len);
  }
}

// OR the lane's packed string into the tile.  `end_bits` = bit position (from the tile start) one past the lane's
// last byte.  The string is shifted so that its end falls on a dword boundary of the tile, which makes every store
// an aligned dword; dwords shared with a neighbouring lane combine through the OR (the tile is zero before a group
// is decoded).  Window dword k lies at `base + 4 k`; dwords that are zero in every lane are skipped.
template <int kLmax>
__device__ __forceinline__ void or_into_tile(const uint32_t (&A)[2 * kLmax], uint32_t end_bits, uint32_t tile_lds, int32_t rebase) {
  constexpr int ND = 2 * kLmax;
  const uint32_t r = (0u - end_bits) & 24u;                      // bits up to the next dword boundary (0, 8, 16, 24)
  uint32_t B[ND + 1];
  B[0] = __builtin_amdgcn_alignbit(A[0], 0u, r);
#pragma unroll
  for (int k = 1; k < ND; ++k) B[k] = __builtin_amdgcn_alignbit(A[k], A[k - 1], r);
  B[ND] = A[ND - 1] >> r;
  // address of window dword 0: (ceil(end / 4) - (ND + 1)) dwords from the tile start
  const uint32_t base = tile_lds + (((end_bits + 24u) >> 5) << 2) - 4u * (ND + 1) + (uint32_t)rebase;
#pragma unroll
  for (int k = 0; k <= ND; ++k) {
    // the upper half of the window is in use in nearly every round; the lower half only for long lanes
    if (k >= (ND + 1) / 2 || __builtin_amdgcn_ballot_w64(B[k] != 0) != 0)
      asm volatile("ds_or_b32 %0, %1 offset:%2" ::"v"(base), "v"(B[k]), "n"(4 * k));
  }
}

// Decode the groups [g_lo, g_hi) one after the other into the wave's LDS tile and hand each decoded tile to
// `consume(g)`, which must leave the tile zero-filled again.  The groups' codes are contiguous in memory, so the
// wavefront streams codes[goff[g_lo], goff[g_hi]) in rounds of 512 codes through a rolling window of kDepth
// outstanding loads, issued unconditionally from a clamped index.  Per round: 8 dictionary lookups per lane, one DPP
// wave scan of the lane totals, register packing, a handful of aligned ds_or_b32.  A group ends somewhere inside a
// round, at a lane boundary because every group's run is padded to 8 codes: the lanes before the boundary store into
// the tile, the tile is consumed, and the lanes after it store 4096 bytes lower, i.e. at the start of the next group.
template <int kLmax, typename Consume>
__device__ __forceinline__ void decode_chunk(const uint32_t* dict, const DevMat& m, uint32_t g_lo, uint32_t g_hi,
                                             uint32_t tile_lds, int lane, Consume&& consume) {
  if (g_lo >= g_hi) return;
  const uint32_t cbeg = group_offset(m, g_lo), cend = group_offset(m, g_hi);
  const uint32_t lane_off = 8 * lane;
  const uint32_t dict_base = lds_address(dict);
  const uint32_t two = 2;
  auto load = [&](uint32_t round_start) -> uint4 { return *(const uint4*)(m.codes + min(round_start + lane_off, cend - 8)); };
  uint4 cw[kDepth];
#pragma unroll
  for (int d = 0; d < kDepth; ++d) {
    cw[d] = load(cbeg + kRoundCodes * d);
    __builtin_amdgcn_sched_barrier(0);   // issue in consumption order: loads return in order, the loop waits per slot
  }
  uint32_t g = g_lo, gend = group_offset(m, g_lo + 1);
  uint32_t pos = 0;                                  // bits decoded so far in group g (wave-uniform)
  for (uint32_t rs = cbeg; rs < cend; rs += kRoundCodes * kDepth) {
#pragma unroll
    for (int d = 0; d < kDepth; ++d) {
      const uint32_t r0 = rs + kRoundCodes * d;     // first code of this round (wave-uniform)
      if (r0 < cend) {
        uint4 c = cw[d];
        if (r0 + kRoundCodes > cend && r0 + lane_off >= cend)   // last round of the chunk: lanes past the end decode nothing
          c = make_uint4(m.pad_word, m.pad_word, m.pad_word, m.pad_word);
        uint32_t s[8];
        s[0] = lds_read32(dict_address_lo(c.x, two, dict_base));
        s[1] = lds_read32(dict_address_hi(c.x, two, dict_base));
        s[2] = lds_read32(dict_address_lo(c.y, two, dict_base));
        s[3] = lds_read32(dict_address_hi(c.y, two, dict_base));
        s[4] = lds_read32(dict_address_lo(c.z, two, dict_base));
        s[5] = lds_read32(dict_address_hi(c.z, two, dict_base));
        s[6] = lds_read32(dict_address_lo(c.w, two, dict_base));
        s[7] = lds_read32(dict_address_hi(c.w, two, dict_base));
        uint32_t tot = s[0] >> 24;
#pragma unroll
        for (int i = 1; i < 8; ++i) tot += s[i] >> 24;
        const uint32_t incl = wave_inclusive_scan(tot);
        const uint32_t round_bits = (uint32_t)__builtin_amdgcn_readlane((int)incl, 63);
        uint32_t A[2 * kLmax];
        pack_runs<kLmax>(s, A);
        const uint32_t end_bits = pos + incl;
        if (r0 + kRoundCodes < gend) {               // the whole round lies inside group g
          or_into_tile<kLmax>(A, end_bits, tile_lds, 0);
          pos += round_bits;
        } else {                                    // group g ends at lane `cut` of this round (cut in 1..64)
          const uint32_t cut = (gend - r0) >> 3;
          if ((uint32_t)lane < cut) or_into_tile<kLmax>(A, end_bits, tile_lds, 0);
          compiler_barrier();
          consume(g);
          compiler_barrier();
          ++g;
          pos = pos + round_bits - 8u * kGroupBytes;   // group g ended exactly at byte 4096
          if (g < g_hi) {
            gend = group_offset(m, g + 1);
            if ((uint32_t)lane >= cut) or_into_tile<kLmax>(A, end_bits, tile_lds, -(int32_t)kGroupBytes);
          }
        }
      }
      cw[d] = load(r0 + kRoundCodes * kDepth);   // refill the slot only after its last use, so it stays in the same registers
    }
  }
}

// Zero a wave's 4 KB tile (64 lanes x 64 bytes).
__device__ __forceinline__ void zero_tile(uint8_t* tile, int lane) {
#pragma unroll
  for (int k = 0; k < 4; ++k) *(uint4*)(tile + (k * 64 + lane) * 16) = make_uint4(0, 0, 0, 0);
}

// Whole-group decode without the cross-group pipeline (used by the general-alignment matvec path).
template <int kLmax>
__device__ __forceinline__ void decode_group(const uint32_t* dict, const DevMat& m, uint32_t g, uint32_t tile_lds, int lane) {
  decode_chunk<kLmax>(dict, m, g, g + 1, tile_lds, lane, [](uint32_t) {});
}

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

constexpr int kMaxBandsPerPass = 4;   // partial accumulators of one pass must fit the tile area: 4 x 8 waves x 1 KB
constexpr int kMaxSlots = 4;          // groups per wavefront and pass whose activation fragments stay in registers

// The 8 MFMA steps of one decoded tile: A = 16 rows x 32 k of int8 weights from the tile (converted to bf16),
// B = the matching 32 k x 16 batch activation fragment held in registers.
__device__ __forceinline__ f32x4 mfma_tile(uint8_t* tile, int lane, const uint4 (&xf)[8], f32x4 acc) {
#pragma unroll
  for (int t = 0; t < 8; ++t) {
    uint2* p = (uint2*)(tile + t * 512 + lane * 8);
    const uint2 a8 = *p;
    *p = make_uint2(0, 0);   // leave the tile zero-filled for the next group (the decoder ORs into it)
    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(i8x8_to_bf16x8(a8), __builtin_bit_cast(bf16x8, xf[t]), acc, 0, 0, 0);
  }
  return acc;
}

// Fused decode + dequantize + matrix-vector product, 16-byte aligned activations.
// A workgroup takes `nb` consecutive bands (16 rows each) per pass.  The nb * n_strips groups of a pass are
// contiguous in the code stream; wavefront w owns the kS consecutive group slots [kS*w, kS*w + kS) of every pass.
// Slot -> column strip is the same in every pass, so the activation fragments of the wave's kS strips are loaded
// once and stay in registers (kS * 32 VGPRs) and the decode loop issues no vector load but the code stream's.
// A slot range touches at most two bands, so a wavefront carries two 16 x 16 fp32 accumulators (rows x batch).
// After the pass the partial accumulators are summed through LDS in wave order (deterministic), scaled and stored.
template <int kLmax, int kS>
__device__ __forceinline__ void matvec_body(const DevMat& m, const uint16_t* __restrict__ x, float* __restrict__ y, int batch,
                                            uint32_t nb, uint32_t slots, uint32_t block, uint32_t n_blocks) {
  extern __shared__ uint4 lds4[];
  uint32_t* dict = (uint32_t*)lds4;
  uint8_t* tiles = (uint8_t*)(dict + m.dict_words_pad);
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int j = lane & 15, kg = lane >> 4;
  // activation fragments: lane (batch row j, k-group kg) holds x[j][strip*256 + 32 t + 8 kg .. + 8), zero past batch / cols
  uint4 xf[kS][8];
  {
    const bool x_lane = j < batch;
    const uint16_t* xlane = x + (size_t)(x_lane ? j : 0) * m.cols + kg * 8;
#pragma unroll
    for (int i = 0; i < kS; ++i) {
      const uint32_t strip = (slots * wave + i) % m.n_strips;
#pragma unroll
      for (int t = 0; t < 8; ++t) {
        const uint32_t col = strip * kGroupCols + t * 32;
        xf[i][t] = (x_lane && col + kg * 8 < m.cols) ? *(const uint4*)(xlane + col) : make_uint4(0, 0, 0, 0);
      }
    }
  }
  uint8_t* tile = tiles + wave * kTileStride;
  const uint32_t tile_lds = lds_address(tile);
  zero_tile(tile, lane);
  stage_dictionary(m, lds4, tid);
  const uint32_t n_pass = (m.n_bands + nb - 1) / nb;
  for (uint32_t pass = block; pass < n_pass; pass += n_blocks) {
    const uint32_t band0 = pass * nb, nbh = min(nb, m.n_bands - band0), ng = nbh * m.n_strips;
    const uint32_t f_lo = min(slots * wave, ng), f_hi = min(slots * wave + slots, ng);
    const uint32_t g_lo = band0 * m.n_strips + f_lo, g_hi = band0 * m.n_strips + f_hi;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f}, acc_first = {0.f, 0.f, 0.f, 0.f};
    const uint32_t band_first = g_lo / m.n_strips;
    uint32_t st = g_lo % m.n_strips;
    decode_chunk<kLmax>(dict, m, g_lo, g_hi, tile_lds, lane, [&](uint32_t g) {
      const uint32_t slot = g - g_lo;
      if (kS == 1 || slot == 0) acc = mfma_tile(tile, lane, xf[0], acc);
      else if (kS == 2 || slot == 1) acc = mfma_tile(tile, lane, xf[kS > 1 ? 1 : 0], acc);
      else if (kS == 3 || slot == 2) acc = mfma_tile(tile, lane, xf[kS > 2 ? 2 : 0], acc);
      else acc = mfma_tile(tile, lane, xf[kS > 3 ? 3 : 0], acc);
      if (++st == m.n_strips) {
        st = 0;
        if (g + 1 < g_hi) {   // the slot range moves on to its second band
          acc_first = acc;
          acc = f32x4{0.f, 0.f, 0.f, 0.f};
        }
      }
    });
    // If the slot range stayed inside one band, everything is in `acc`: file it under the first band.
    const bool two = (g_lo < g_hi) && ((g_hi - 1) / m.n_strips != band_first);
    if (!two) {
      acc_first = acc;
      acc = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    // Partial sums: red[band_local][wave][256].  The tiles are free once every wave has finished its chunk.
    __syncthreads();
    float* red = (float*)tiles;
    for (uint32_t bl = 0; bl < nbh; ++bl) {
      const uint32_t bnd = band0 + bl;
      const bool is_first = (g_lo < g_hi) && bnd == band_first, is_second = two && bnd == band_first + 1;
#pragma unroll
      for (int v = 0; v < 4; ++v)
        red[(bl * kWaves + wave) * 256 + v * 64 + lane] = is_first ? acc_first[v] : (is_second ? acc[v] : 0.f);
    }
    __syncthreads();
    for (uint32_t o = tid; o < nbh * 256; o += kThreads) {
      const uint32_t bl = o >> 8, e = o & 255;
      float s = 0.f;
#pragma unroll
      for (int w = 0; w < kWaves; ++w) s += red[(bl * kWaves + w) * 256 + e];
      const uint32_t v = e >> 6, l = e & 63;
      const uint32_t row = (band0 + bl) * kTileRows + 4 * (l >> 4) + v;   // accumulator register v of lane l: row 4*(l/16)+v
      const uint32_t b = l & 15;                                          // batch column l%16
      if (b < (uint32_t)batch && row < m.rows) y[(size_t)b * m.rows + row] = s * m.scales[row];
    }
    __syncthreads();
    zero_tile(tile, lane);   // the partial sums lay over the tiles; the decoder needs them zero
  }
}

template <int kLmax, int kS>
__global__ __launch_bounds__(kThreads, 1) void k_matvec(DevMat m, const uint16_t* __restrict__ x, float* __restrict__ y,
                                                        int batch, uint32_t nb) {
  matvec_body<kLmax, kS>(m, x, y, batch, nb, kS, blockIdx.x, gridDim.x);
}

// Several independent matrices in one launch (e.g. the q, k, v projections of a layer): the grid is the
// concatenation of each matrix's own grid, every workgroup serves exactly one matrix, so small matrices run side by
// side instead of leaving most CUs idle one launch after the other.
constexpr int kMaxMulti = 8;
struct MultiArgs {
  DevMat m[kMaxMulti];
  const uint16_t* x[kMaxMulti];
  float* y[kMaxMulti];
  uint32_t nb[kMaxMulti], slots[kMaxMulti];
  uint32_t first_block[kMaxMulti + 1];
  int n, batch;
};

template <int kLmax, int kS>
__global__ __launch_bounds__(kThreads, 1) void k_matvec_multi(MultiArgs a) {
  int i = 0;
  while (i + 1 < a.n && blockIdx.x >= a.first_block[i + 1]) ++i;
  matvec_body<kLmax, kS>(a.m[i], a.x[i], a.y[i], a.batch, a.nb[i], a.slots[i], blockIdx.x - a.first_block[i],
                         a.first_block[i + 1] - a.first_block[i]);
}

// General-alignment fallback of the same product (activation pointer not 16-byte aligned or cols % 8 != 0):
// one band per pass, strips round-robin over the wavefronts, element-wise bounds-checked activation loads.
template <int kLmax>
__global__ __launch_bounds__(kThreads, 1) void k_matvec_anyalign(DevMat m, const uint16_t* __restrict__ x,
                                                                 float* __restrict__ y, int batch) {
  extern __shared__ uint4 lds4[];
  uint32_t* dict = (uint32_t*)lds4;
  uint8_t* tiles = (uint8_t*)(dict + m.dict_words_pad);
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  uint8_t* tile = tiles + wave * kTileStride;
  const uint32_t tile_lds = lds_address(tile);
  zero_tile(tile, lane);
  stage_dictionary(m, lds4, tid);
  const int j = lane & 15, kg = lane >> 4;
  for (uint32_t band = blockIdx.x; band < m.n_bands; band += gridDim.x) {
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    for (uint32_t st = wave; st < m.n_strips; st += kWaves) {
      decode_group<kLmax>(dict, m, band * m.n_strips + st, tile_lds, lane);
#pragma unroll
      for (int t = 0; t < 8; ++t) {
        uint2* ap = (uint2*)(tile + t * 512 + lane * 8);
        const uint2 a8 = *ap;
        *ap = make_uint2(0, 0);
        const uint32_t col = st * kGroupCols + t * 32 + kg * 8;
        uint32_t e[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) e[k] = (j < batch && col + k < m.cols) ? x[(size_t)j * m.cols + col + k] : 0u;
        const uint4 xb = make_uint4(e[0] | e[1] << 16, e[2] | e[3] << 16, e[4] | e[5] << 16, e[6] | e[7] << 16);
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(i8x8_to_bf16x8(a8), __builtin_bit_cast(bf16x8, xb), acc, 0, 0, 0);
      }
    }
    __syncthreads();
    float* red = (float*)tiles;
#pragma unroll
    for (int v = 0; v < 4; ++v) red[wave * 256 + v * 64 + lane] = acc[v];
    __syncthreads();
    if (tid < 256) {
      float s = 0.f;
#pragma unroll
      for (int w = 0; w < kWaves; ++w) s += red[w * 256 + tid];
      const int v = tid >> 6, l = tid & 63;
      const uint32_t row = band * kTileRows + 4 * (l >> 4) + v;
      const int b = l & 15;
      if (b < batch && row < m.rows) y[(size_t)b * m.rows + row] = s * m.scales[row];
    }
    __syncthreads();
    zero_tile(tile, lane);
  }
}

// Expansion to the row-major int8 matrix.  The groups are split into one contiguous chunk per wavefront of the
// grid; each decoded 16 x 256 tile is copied out with 16-byte stores (byte stores on the general-alignment path).
template <int kLmax, bool kFastOut>
__global__ __launch_bounds__(kThreads, 1) void k_decompress(DevMat m, int8_t* __restrict__ out) {
  extern __shared__ uint4 lds4[];
  uint32_t* dict = (uint32_t*)lds4;
  uint8_t* tiles = (uint8_t*)(dict + m.dict_words_pad);
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  uint8_t* tile = tiles + wave * kTileStride;
  const uint32_t tile_lds = lds_address(tile);
  zero_tile(tile, lane);
  stage_dictionary(m, lds4, tid);
  const uint64_t n_waves = (uint64_t)gridDim.x * kWaves, wid = (uint64_t)blockIdx.x * kWaves + wave;
  const uint32_t g_lo = (uint32_t)(m.n_groups * wid / n_waves), g_hi = (uint32_t)(m.n_groups * (wid + 1) / n_waves);
  uint32_t band = g_lo / m.n_strips, st = g_lo % m.n_strips;
  decode_chunk<kLmax>(dict, m, g_lo, g_hi, tile_lds, lane, [&](uint32_t) {
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const int q = lane + 64 * t, i = q >> 4, pc = q & 15;   // row i of the band, 16-byte piece pc of its 256 columns
      uint2* plo = (uint2*)(tile + (2 * pc) * 128 + i * 8);
      uint2* phi = (uint2*)(tile + (2 * pc + 1) * 128 + i * 8);
      const uint2 lo = *plo, hi = *phi;
      *plo = make_uint2(0, 0);   // leave the tile zero-filled for the next group
      *phi = make_uint2(0, 0);
      const uint32_t row = band * kTileRows + i, col = st * kGroupCols + pc * 16;
      if (row >= m.rows || col >= m.cols) continue;
      int8_t* dst = out + (size_t)row * m.cols + col;
      if (kFastOut) {
        *(uint4*)dst = make_uint4(lo.x, lo.y, hi.x, hi.y);
      } else {
        const uint32_t w[4] = {lo.x, lo.y, hi.x, hi.y};
#pragma unroll
        for (int k = 0; k < 16; ++k)
          if (col + k < m.cols) dst[k] = (int8_t)(w[k >> 2] >> (8 * (k & 3)));
      }
    }
    if (++st == m.n_strips) {
      st = 0;
      ++band;
    }
  });
}

}  // namespace tq

using namespace tq;

struct tq_matrix {
  Header h;
  DevMat m;
  void* dev_base;
  int device;
  int n_cu;
  size_t lds_bytes;
  uint32_t bands_per_pass, slots;   // launch shape of the aligned matvec kernel (0 bands: use the general kernel)
};

namespace {

int hip_fail(const char* what, hipError_t e) {
  set_error(std::string(what) + ": " + hipGetErrorString(e));
  return TQ_E_HIP;
}

typedef void (*matvec_fn)(DevMat, const uint16_t*, float*, int, uint32_t);
typedef void (*matvec_any_fn)(DevMat, const uint16_t*, float*, int);
typedef void (*decompress_fn)(DevMat, int8_t*);

template <int kLmax>
matvec_fn pick_matvec_slots(uint32_t slots) {
  switch (slots) {
    case 1: return k_matvec<kLmax, 1>;
    case 2: return k_matvec<kLmax, 2>;
    case 3: return k_matvec<kLmax, 3>;
    default: return k_matvec<kLmax, 4>;
  }
}
matvec_fn pick_matvec(uint32_t lmax, uint32_t slots) {
  return lmax == 1 ? pick_matvec_slots<1>(slots) : lmax == 2 ? pick_matvec_slots<2>(slots) : pick_matvec_slots<3>(slots);
}
typedef void (*matvec_multi_fn)(MultiArgs);
template <int kLmax>
matvec_multi_fn pick_multi_slots(uint32_t slots) {
  switch (slots) {
    case 1: return k_matvec_multi<kLmax, 1>;
    case 2: return k_matvec_multi<kLmax, 2>;
    case 3: return k_matvec_multi<kLmax, 3>;
    default: return k_matvec_multi<kLmax, 4>;
  }
}
matvec_multi_fn pick_matvec_multi(uint32_t lmax, uint32_t slots) {
  return lmax == 1 ? pick_multi_slots<1>(slots) : lmax == 2 ? pick_multi_slots<2>(slots) : pick_multi_slots<3>(slots);
}
matvec_any_fn pick_matvec_any(uint32_t lmax) {
  return lmax == 1 ? k_matvec_anyalign<1> : lmax == 2 ? k_matvec_anyalign<2> : k_matvec_anyalign<3>;
}
decompress_fn pick_decompress(uint32_t lmax, bool fast) {
  switch (lmax) {
    case 1: return fast ? k_decompress<1, true> : k_decompress<1, false>;
    case 2: return fast ? k_decompress<2, true> : k_decompress<2, false>;
    default: return fast ? k_decompress<3, true> : k_decompress<3, false>;
  }
}

// Dynamic LDS above 64 KB has to be allowed per kernel function.
int allow_lds(uint32_t lmax, size_t bytes) {
  const void* fns[11] = {(const void*)pick_matvec(lmax, 1), (const void*)pick_matvec(lmax, 2), (const void*)pick_matvec(lmax, 3),
                         (const void*)pick_matvec(lmax, 4), (const void*)pick_matvec_multi(lmax, 1),
                         (const void*)pick_matvec_multi(lmax, 2), (const void*)pick_matvec_multi(lmax, 3),
                         (const void*)pick_matvec_multi(lmax, 4), (const void*)pick_matvec_any(lmax),
                         (const void*)pick_decompress(lmax, false), (const void*)pick_decompress(lmax, true)};
  for (const void* f : fns) {
    hipError_t e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e != hipSuccess) return hip_fail("hipFuncSetAttribute(MaxDynamicSharedMemorySize)", e);
  }
  return TQ_OK;
}

// Bands per pass for the aligned matvec kernel: the value in {1, 2, 4} with the fewest sequential group decodes per
// wavefront, ceil(passes / CUs) * slots with slots = ceil(nb * n_strips / 8).  Returns 0 when even one band needs
// more than kMaxSlots slots (very wide matrices): those use the general kernel.
uint32_t pick_bands_per_pass(uint32_t n_bands, uint32_t n_strips, uint32_t n_cu, uint32_t* slots_out) {
  uint32_t best = 0;
  uint64_t best_cost = UINT64_MAX;
  for (uint32_t nb = 1; nb <= (uint32_t)kMaxBandsPerPass; nb *= 2) {
    const uint64_t slots = ((uint64_t)nb * n_strips + kWaves - 1) / kWaves;
    if (slots > (uint64_t)kMaxSlots) break;
    const uint64_t passes = (n_bands + nb - 1) / nb;
    const uint64_t cost = ((passes + n_cu - 1) / n_cu) * slots;
    if (cost < best_cost) {
      best_cost = cost;
      best = nb;
      *slots_out = (uint32_t)slots;
    }
  }
  return best;
}

}  // namespace

extern "C" int tq_create_from_encoded(const void* blob, size_t blob_bytes, tq_handle* out) {
  if (!out) {
    set_error("tq_create_from_encoded: null output pointer");
    return TQ_E_INVALID_ARG;
  }
  *out = nullptr;
  Header h;
  unsigned hw = std::thread::hardware_concurrency();
  if (int rc = validate_blob(blob, blob_bytes, &h, hw ? hw : 1)) return rc;

  const uint32_t dict_words_pad = (uint32_t)round_up(h.n_entries + 1, 4);
  const size_t lds_bytes = (size_t)dict_words_pad * 4 + (size_t)kWaves * kTileStride;
  if (lds_bytes > kLdsLimit) {
    set_error("dictionary with " + std::to_string(h.n_entries) + " entries does not fit the 160 KB LDS next to the decode tiles");
    return TQ_E_UNSUPPORTED;
  }
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_fail("hipGetDevice (is a GPU present?)", e);
  hipDeviceProp_t prop;
  e = hipGetDeviceProperties(&prop, dev);
  if (e != hipSuccess) return hip_fail("hipGetDeviceProperties", e);
  if (prop.sharedMemPerBlock < lds_bytes && (size_t)prop.maxSharedMemoryPerMultiProcessor < lds_bytes) {
    set_error("device offers less LDS per workgroup than this library needs (built for gfx950, 160 KB)");
    return TQ_E_UNSUPPORTED;
  }

  const uint64_t sz_dict = round_up((uint64_t)dict_words_pad * 4, kSectionAlign), sz_goff = round_up(h.goff_bytes, kSectionAlign),
                 sz_codes = round_up(h.code_bytes, kSectionAlign), sz_scales = round_up(h.scale_bytes, kSectionAlign);
  const uint64_t o_dict = 0, o_goff = o_dict + sz_dict, o_codes = o_goff + sz_goff, o_scales = o_codes + sz_codes;
  const uint64_t total = o_scales + sz_scales;
  uint8_t* base = nullptr;
  e = hipMalloc((void**)&base, total);
  if (e != hipSuccess) {
    set_error(std::string("hipMalloc of ") + std::to_string(total) + " bytes: " + hipGetErrorString(e));
    return e == hipErrorOutOfMemory ? TQ_E_OOM : TQ_E_HIP;
  }
  const uint8_t* src = (const uint8_t*)blob;
  e = hipMemset(base + o_dict, 0, sz_dict);
  if (e == hipSuccess) e = hipMemcpy(base + o_dict, src + h.off_dict, h.dict_bytes, hipMemcpyHostToDevice);
  if (e == hipSuccess) e = hipMemcpy(base + o_goff, src + h.off_goff, h.goff_bytes, hipMemcpyHostToDevice);
  if (e == hipSuccess) e = hipMemcpy(base + o_codes, src + h.off_codes, h.code_bytes, hipMemcpyHostToDevice);
  if (e == hipSuccess) e = hipMemcpy(base + o_scales, src + h.off_scales, h.scale_bytes, hipMemcpyHostToDevice);
  if (e == hipSuccess) e = hipDeviceSynchronize();
  if (e != hipSuccess) {
    (void)hipFree(base);
    return hip_fail("upload", e);
  }
  int rc = allow_lds(h.lmax, lds_bytes);
  if (rc != TQ_OK) {
    (void)hipFree(base);
    return rc;
  }
  tq_matrix* t = new (std::nothrow) tq_matrix;
  if (!t) {
    (void)hipFree(base);
    set_error("out of host memory");
    return TQ_E_OOM;
  }
  t->h = h;
  t->dev_base = base;
  t->device = dev;
  t->n_cu = prop.multiProcessorCount;
  t->lds_bytes = lds_bytes;
  t->slots = 0;
  t->bands_per_pass = pick_bands_per_pass(h.rows_pad / kTileRows, h.cols_pad / kGroupCols, (uint32_t)prop.multiProcessorCount, &t->slots);
  t->m.dict = (const uint32_t*)(base + o_dict);
  t->m.goff = (const uint32_t*)(base + o_goff);
  t->m.codes = (const uint16_t*)(base + o_codes);
  t->m.scales = (const float*)(base + o_scales);
  t->m.rows = h.rows;
  t->m.cols = h.cols;
  t->m.n_bands = h.rows_pad / kTileRows;
  t->m.n_strips = h.cols_pad / kGroupCols;
  t->m.dict_words_pad = dict_words_pad;
  t->m.pad_word = h.pad_code | h.pad_code << 16;
  t->m.n_groups = h.n_groups;
  *out = t;
  return TQ_OK;
}

extern "C" int tq_matvec(tq_handle h, const void* x, void* y, int batch, void* stream) {
  if (!h || !x || !y) {
    set_error("tq_matvec: null argument");
    return TQ_E_INVALID_ARG;
  }
  if (batch < 1 || batch > TQ_MAX_BATCH) {
    set_error("tq_matvec: batch must be in [1, " + std::to_string(TQ_MAX_BATCH) + "]");
    return TQ_E_UNSUPPORTED;
  }
  if ((uintptr_t)x % 2 || (uintptr_t)y % 4) {
    set_error("tq_matvec: x must be 2-byte and y 4-byte aligned");
    return TQ_E_INVALID_ARG;
  }
  const bool x_fast = (h->m.cols % 8 == 0) && ((uintptr_t)x % 16 == 0);
  if (x_fast && h->bands_per_pass) {
    const uint32_t nb = h->bands_per_pass, passes = (h->m.n_bands + nb - 1) / nb;
    const unsigned grid = (unsigned)std::min<uint32_t>(passes, (uint32_t)h->n_cu);
    hipLaunchKernelGGL(pick_matvec(h->h.lmax, h->slots), dim3(grid), dim3(kThreads), h->lds_bytes, (hipStream_t)stream,
                       h->m, (const uint16_t*)x, (float*)y, batch, nb);
  } else {
    const unsigned grid = (unsigned)std::min<uint32_t>(h->m.n_bands, (uint32_t)h->n_cu);
    hipLaunchKernelGGL(pick_matvec_any(h->h.lmax), dim3(grid), dim3(kThreads), h->lds_bytes, (hipStream_t)stream, h->m,
                       (const uint16_t*)x, (float*)y, batch);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return hip_fail("tq_matvec launch", e);
  return TQ_OK;
}

extern "C" int tq_matvec_multi(int n, const tq_handle* hs, const void* const* xs, void* const* ys, int batch, void* stream) {
  if (n < 1 || !hs || !xs || !ys) {
    set_error("tq_matvec_multi: null argument or n < 1");
    return TQ_E_INVALID_ARG;
  }
  if (batch < 1 || batch > TQ_MAX_BATCH) {
    set_error("tq_matvec_multi: batch must be in [1, " + std::to_string(TQ_MAX_BATCH) + "]");
    return TQ_E_UNSUPPORTED;
  }
  for (int i = 0; i < n; ++i) {
    if (!hs[i] || !xs[i] || !ys[i]) {
      set_error("tq_matvec_multi: null handle or pointer at index " + std::to_string(i));
      return TQ_E_INVALID_ARG;
    }
    if ((uintptr_t)xs[i] % 2 || (uintptr_t)ys[i] % 4) {
      set_error("tq_matvec_multi: x must be 2-byte and y 4-byte aligned");
      return TQ_E_INVALID_ARG;
    }
  }
  // One fused launch needs: at most kMaxMulti matrices, one dictionary run-length cap, one LDS size class, and the
  // aligned kernel for every member.  Anything else is served by consecutive single launches (same results).
  bool fuse = n >= 2 && n <= kMaxMulti;
  for (int i = 0; i < n && fuse; ++i)
    fuse = hs[i]->bands_per_pass != 0 && hs[i]->h.lmax == hs[0]->h.lmax && hs[i]->device == hs[0]->device &&
           (hs[i]->m.cols % 8 == 0) && ((uintptr_t)xs[i] % 16 == 0);
  if (!fuse) {
    for (int i = 0; i < n; ++i)
      if (int rc = tq_matvec(hs[i], xs[i], ys[i], batch, stream)) return rc;
    return TQ_OK;
  }
  MultiArgs a;
  std::memset(&a, 0, sizeof a);
  a.n = n;
  a.batch = batch;
  uint32_t slots = 1, blocks = 0;
  size_t lds = 0;
  for (int i = 0; i < n; ++i) {
    const tq_matrix* t = hs[i];
    a.m[i] = t->m;
    a.x[i] = (const uint16_t*)xs[i];
    a.y[i] = (float*)ys[i];
    a.nb[i] = t->bands_per_pass;
    a.slots[i] = t->slots;
    a.first_block[i] = blocks;
    const uint32_t passes = (t->m.n_bands + t->bands_per_pass - 1) / t->bands_per_pass;
    blocks += std::min<uint32_t>(passes, (uint32_t)t->n_cu);
    slots = std::max(slots, t->slots);
    lds = std::max(lds, t->lds_bytes);
  }
  a.first_block[n] = blocks;
  hipLaunchKernelGGL(pick_matvec_multi(hs[0]->h.lmax, slots), dim3(blocks), dim3(kThreads), lds, (hipStream_t)stream, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return hip_fail("tq_matvec_multi launch", e);
  return TQ_OK;
}

extern "C" int tq_decompress(tq_handle h, void* out, void* stream) {
  if (!h || !out) {
    set_error("tq_decompress: null argument");
    return TQ_E_INVALID_ARG;
  }
  const bool out_fast = (h->m.cols % 16 == 0) && ((uintptr_t)out % 16 == 0);
  const uint64_t wg_needed = (h->m.n_groups + kWaves - 1) / kWaves;
  const unsigned grid = (unsigned)std::min<uint64_t>(wg_needed, (uint64_t)h->n_cu);
  hipLaunchKernelGGL(pick_decompress(h->h.lmax, out_fast), dim3(grid), dim3(kThreads), h->lds_bytes, (hipStream_t)stream,
                     h->m, (int8_t*)out);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return hip_fail("tq_decompress launch", e);
  return TQ_OK;
}

extern "C" int tq_get_info(tq_handle h, tq_info* out) {
  if (!h || !out) {
    set_error("tq_get_info: null argument");
    return TQ_E_INVALID_ARG;
  }
  fill_info(h->h, out);
  return TQ_OK;
}

extern "C" int tq_destroy(tq_handle h) {
  if (!h) return TQ_OK;
  hipError_t e = hipFree(h->dev_base);
  delete h;
  if (e != hipSuccess) return hip_fail("hipFree", e);
  return TQ_OK;
}
