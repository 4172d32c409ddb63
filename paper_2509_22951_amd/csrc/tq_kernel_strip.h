// Device side of libtq: the whole-strip batched product and the expansion to int8 matrices.
#pragma once
#include "tq_kernels_common.h"
#include "tq_strip_decode.h"

namespace tq {
// Stage a dictionary image that is already laid out the way the kernel reads it (containers with runs of 3 and 4 bytes).
__device__ __forceinline__ void stage_image(const uint32_t* image, uint32_t bytes, uint16_t* lds_dict, int tid, int n_threads) {
  const uint4* src = (const uint4*)image;
  uint4* dst = (uint4*)lds_dict;
  for (uint32_t i = tid; i < bytes / 16; i += n_threads) dst[i] = global_load(src + i);
}

// kLong: the matrices of the launch hold runs of up to 4 bytes (append_chunk_long).
template <bool kXFast, bool kPacked, bool kLong = false>
__global__ __launch_bounds__(kThreads, 1) void k_matvec_mfma(MatvecArgs a) {
  extern __shared__ uint4 lds4[];
  uint16_t* lds_dict = (uint16_t*)lds4;
  uint8_t* tiles = (uint8_t*)lds4 + a.x_off;
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n_threads = blockDim.x, n_waves = n_threads >> 6;
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
    if (kLong && m.dict != staged) {
      stage_image(m.dict, m.dict16_bytes, lds_dict, tid, n_threads);
      staged = m.dict;
    }
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
      decode_run_to_tile<kLong>(m, u0, u1, lane, my_strip, [&](uint32_t, uint32_t quad) {
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
template <bool kLong = false>
__global__ __launch_bounds__(kThreads, 1) void k_decompress(MatvecArgs a) {
  extern __shared__ uint4 lds4[];
  uint16_t* lds_dict = (uint16_t*)lds4;
  uint8_t* tiles = (uint8_t*)lds4 + a.x_off;
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n_threads = blockDim.x, n_waves = n_threads >> 6;
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
    if (kLong && m.dict != staged) {
      __syncthreads();   // nobody reads the previous dictionary any more
      stage_image(m.dict, m.dict16_bytes, lds_dict, tid, n_threads);
      staged = m.dict;
      __syncthreads();
    }
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
    decode_run_to_tile<kLong>(m, u0, u1, lane, tile_lds + (uint32_t)lane * strip, [](uint32_t, uint32_t) {}, [&](uint32_t band, uint32_t quad) {
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
