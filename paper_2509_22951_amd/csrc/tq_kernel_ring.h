// Device side of libtq: the batched product with a ring per lane (decode and MFMA interleaved).
#pragma once
#include "tq_kernels_common.h"
#include "tq_strip_decode.h"

namespace tq {
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
constexpr int kRingWavesQuarter = 11;   // with a tile of 4 batch rows (batches up to 4) beside a full dictionary
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
  uint32_t s0, s1, n;
  chunk_string(c, s0, s1, n);                                           // the 4..8 bytes of the chunk, zero above them
  const uint64_t str = (uint64_t)s1 << 32 | s0;
  const uint32_t after = min(pos + n, seg_len);
  const uint32_t sh = (pos & 7u) << 3;
  const uint64_t lo = carry | str << sh, hi = (str >> 1) >> (63 - sh);  // the 16 bytes carry + string; hi is 0 when pos % 8 == 0
  const bool full = (after ^ pos) >= 8;
  // stored whether the piece is complete or not (an incomplete one holds zeros above its bytes and is stored again,
  // complete, by a later chunk; nobody reads a piece before every lane has passed it): no branch in the chunk's code
  *(lds_u64*)(size_t)(ring | ((pos ^ sw8) & 0x78u)) = lo;
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

}  // namespace tq
