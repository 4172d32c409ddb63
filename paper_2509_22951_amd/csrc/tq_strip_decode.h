// Device side of libtq: decode of a unit into per-lane strips in LDS, and the MFMA steps over a decoded unit.
#pragma once
#include "tq_kernels_common.h"
#include "tq_kernel_dot.h"

namespace tq {
// ---------------------------------------------------------------------------------------------------------------
// Product for the batches the dot-product kernel does not take (3..16 activation rows; 1 or 2 when a row is too long
// for that kernel's LDS image), whole-strip form: decode a unit into an LDS tile, then bf16 MFMA with the batch as N.
// (Large launches of well-behaved matrices take the ring form instead.)
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

// The runs of one chunk (4 codes) as one string of 4..8 bytes in (s0, s1), n = its length.  The 4 entries (1 or 2 bytes
// each; the length follows from the code; the byte after a single is zero in the dictionary image) are joined with
// byte-granular funnel shifts.  Bytes of the string past n are not zero in general.
__device__ __forceinline__ void chunk_string(uint2 c, uint32_t& s0, uint32_t& s1, uint32_t& n) {
  const uint32_t e0 = lds_read16(half_offset_lo(c.x)), e1 = lds_read16(half_offset_hi(c.x));
  const uint32_t e2 = lds_read16(half_offset_lo(c.y)), e3 = lds_read16(half_offset_hi(c.y));
  const uint32_t p0 = is_pair_lo(c.x), p1 = is_pair_hi(c.x), p2 = is_pair_lo(c.y), p3 = is_pair_hi(c.y);
  const uint32_t a01 = e1 << ((p0 << 3) + 8) | e0, q01 = p0 + p1;   // codes 0, 1: 2 + q01 bytes
  const uint32_t a23 = e3 << ((p2 << 3) + 8) | e2, q23 = p2 + p3;   // codes 2, 3
  const uint32_t k = 2u - q01;                                      // bytes of a23 that still fit the first dword: 0..2
  s0 = a01 | __builtin_amdgcn_alignbyte(a23, 0u, k);               // a23 << 8 (4 - k), nothing for k == 0
  s1 = __builtin_amdgcn_alignbyte(0u, a23, k);                      // a23 >> 8 k
  n = q01 + q23 + 4u;
}

typedef uint64_t lds_u64_any __attribute__((address_space(3), aligned(1)));
typedef __attribute__((address_space(3))) uint64_t lds_u64;

// Append the runs of one chunk to the lane's strip: the string goes to LDS as it is, with one 8-byte store at the
// byte the lane has reached (LDS stores need no alignment on this target); what it writes past its own n bytes is
// overwritten by the chunks that follow, or falls into the 8 spare bytes every strip has after its segment.
// wpos = LDS address of the next byte of the segment, limit = address of the segment's end.  Pad codes (entry 0,
// counted as 2 bytes by the code test) only follow a complete segment: the clamp keeps the lane at its end.
__device__ __forceinline__ void append_chunk(uint2 c, uint32_t limit, uint32_t& wpos) {
  uint32_t s0, s1, n;
  chunk_string(c, s0, s1, n);
  *(lds_u64_any*)(size_t)wpos = (uint64_t)s1 << 32 | s0;
  wpos = min(wpos + n, limit);
}

// The same for containers with runs of up to 4 bytes.  The byte image of the dictionary has one 2-byte slot per entry
// of up to 2 bytes and two slots (4 bytes, 4-byte aligned) per longer entry; a code reads the aligned dword its slot lies
// in, moves its bytes down, and stores them as one dword at the byte the lane has reached (bytes past the run's length
// are overwritten by the next code or fall into the strip's spare bytes).  One store per code: this form is the general
// one, not the fast one.
typedef uint32_t lds_u32_any __attribute__((address_space(3), aligned(1)));
__device__ __forceinline__ void append_code_long(uint32_t code, uint32_t class2, uint32_t class3, uint32_t limit, uint32_t& wpos) {
  const uint32_t ba = long_slot(code, class2) << 1;                    // byte address of the entry in the image
  const uint32_t e = lds_read32(ba & ~3u) >> ((ba & 2u) << 3);
  *(lds_u32_any*)(size_t)wpos = e;
  wpos = min(wpos + long_run_length(code, class2, class3), limit);
}
__device__ __forceinline__ void append_chunk_long(uint2 c, uint32_t class2, uint32_t class3, uint32_t limit, uint32_t& wpos) {
  append_code_long(c.x & 0xFFFFu, class2, class3, limit, wpos);
  append_code_long(c.x >> 16, class2, class3, limit, wpos);
  append_code_long(c.y & 0xFFFFu, class2, class3, limit, wpos);
  append_code_long(c.y >> 16, class2, class3, limit, wpos);
}

// Decode the units [u0, u1) of a matrix, one after the other, into the strips of this wavefront's tile and call
// on_unit(band, quad) each time the tile holds a complete unit; before_last_piece(band, quad) is called ahead of the
// unit's last piece of chunks, a few thousand clocks earlier (the place to request what on_unit will need).  The code chunks of the run are contiguous in memory.
// They are fetched in pieces of at most kPiece chunks that never straddle a unit (a unit is cut into equal pieces);
// two register sets alternate, so the loads of the next piece are in flight while the current one is decoded.
// Every piece issues exactly kPiece loads (those past its end repeat its last chunk): a fixed number of loads in flight
// is what lets the compiler wait for the current piece only and not for the one just requested.

template <bool kLong = false, typename BeforeLast, typename OnUnit>
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
  uint32_t wpos = my_strip, limit = my_strip + segment_length();   // next byte of the lane's segment in its strip, and its end
  auto decode_piece = [&](const uint2 (&cw)[kPiece], uint32_t n, bool ends) {
    if (ends) before_last_piece(band, quad);
    if constexpr (kLong) {
#pragma unroll
      for (int k = 0; k < kPiece; ++k)
        if ((uint32_t)k < n) append_chunk_long(cw[k], m.class2, m.class3, limit, wpos);
    } else if (n == kPiece) {   // whole pieces as straight-line code: the dictionary reads of later chunks overlap the packing of earlier ones
#pragma unroll
      for (int k = 0; k < kPiece; ++k) append_chunk(cw[k], limit, wpos);
    } else if (n == kPiece - 1) {
#pragma unroll
      for (int k = 0; k < kPiece - 1; ++k) append_chunk(cw[k], limit, wpos);
    } else {
#pragma unroll
      for (int k = 0; k < kPiece; ++k)
        if ((uint32_t)k < n) append_chunk(cw[k], limit, wpos);
    }
    if (ends) {
      on_unit(band, quad);
      if (++quad == nq) {
        quad = 0;
        ++band;
      }
      wpos = my_strip;
      limit = my_strip + segment_length();
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

}  // namespace tq
