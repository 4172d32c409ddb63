// Device side of libtq for gfx950 (MI355X): handle management and the two hot-path kernels.
//
// Work decomposition.  The container stores the matrix as restart groups of 16 rows x 256 columns (4096 bytes,
// 32 micro-tiles of 16x8 in MFMA operand order).  One wavefront decodes one group at a time:
//   1. 64 lanes load 4 consecutive 16-bit codes each (one coalesced 512-byte read per round),
//   2. look each code up in the LDS-resident dictionary (one 32-bit word: 3 run bytes + length),
//   3. get every run's byte position from a lane-local prefix plus a DPP wave scan of the lane totals,
//   4. scatter the run bytes into the wave's private 4 KB LDS tile.  Every code writes all three byte slots
//      unconditionally, highest byte index first: a slot past a run's length lands on a position owned by a later
//      run at a smaller byte index, so the owner's later write wins and no lane needs predication.
// The tile then holds 8 MFMA A-operand blocks (16 rows x 32 k).  tq_matvec converts each lane's 8 int8 values to
// bf16 (exact) and issues v_mfma_f32_16x16x32_bf16 against the activations (batch is the N dimension, up to 16);
// tq_decompress copies the tile out to the row-major int8 matrix with 16-byte stores.
// The expanded matrix never exists in HBM on the tq_matvec path.
#include <hip/hip_runtime.h>

#include <cstring>
#include <new>
#include <string>
#include <thread>

#include "../../include/tq.h"
#include "tq_format.h"

namespace tq {

constexpr int kWaves = 8;                      // wavefronts per workgroup (one workgroup per CU: LDS-bound occupancy)
constexpr int kThreads = kWaves * 64;
constexpr uint32_t kTileStride = kGroupBytes + 16;   // slack absorbs the over-writes of the last run and of pad codes
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

__device__ __forceinline__ void stage_dictionary(const DevMat& m, uint4* lds4, int tid) {
  const uint4* src = (const uint4*)m.dict;
  for (uint32_t i = tid; i < m.dict_words_pad / 4; i += kThreads) lds4[i] = src[i];
  __syncthreads();
}

// Decode codes[begin, end) (a whole group; begin and end are multiples of 4) into tile[0, 4096).
template <int kLmax>
__device__ __forceinline__ void decode_group(const uint32_t* dict, const uint16_t* __restrict__ codes, uint32_t begin,
                                             uint32_t end, uint32_t pad_word, volatile uint8_t* tile, int lane) {
  uint32_t pos = 0;
  for (uint32_t base = begin; base < end; base += 256) {
    const uint32_t idx = base + 4 * lane;
    uint2 cw = make_uint2(pad_word, pad_word);
    if (idx < end) cw = *(const uint2*)(codes + idx);
    const uint32_t s0 = dict[cw.x & 0xFFFFu], s1 = dict[cw.x >> 16], s2 = dict[cw.y & 0xFFFFu], s3 = dict[cw.y >> 16];
    const uint32_t t1 = s0 >> 24, t2 = t1 + (s1 >> 24), t3 = t2 + (s2 >> 24), tot = t3 + (s3 >> 24);
    const uint32_t incl = wave_inclusive_scan(tot);
    const uint32_t p0 = pos + incl - tot, p1 = p0 + t1, p2 = p0 + t2, p3 = p0 + t3;
    if (kLmax >= 3) {
      tile[p0 + 2] = (uint8_t)(s0 >> 16);
      tile[p1 + 2] = (uint8_t)(s1 >> 16);
      tile[p2 + 2] = (uint8_t)(s2 >> 16);
      tile[p3 + 2] = (uint8_t)(s3 >> 16);
    }
    if (kLmax >= 2) {
      tile[p0 + 1] = (uint8_t)(s0 >> 8);
      tile[p1 + 1] = (uint8_t)(s1 >> 8);
      tile[p2 + 1] = (uint8_t)(s2 >> 8);
      tile[p3 + 1] = (uint8_t)(s3 >> 8);
    }
    tile[p0] = (uint8_t)s0;
    tile[p1] = (uint8_t)s1;
    tile[p2] = (uint8_t)s2;
    tile[p3] = (uint8_t)s3;
    pos += (uint32_t)__builtin_amdgcn_readlane((int)incl, 63);
  }
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

// One workgroup per band of 16 rows at a time; its wavefronts take the band's column strips round-robin, keep a
// 16 x 16 fp32 accumulator each (rows x batch), and the partial accumulators are summed through LDS in wave order.
template <int kLmax>
__global__ __launch_bounds__(kThreads, 1) void k_matvec(DevMat m, const uint16_t* __restrict__ x, float* __restrict__ y,
                                                        int batch, int x_fast) {
  extern __shared__ uint4 lds4[];
  uint32_t* dict = (uint32_t*)lds4;
  uint8_t* tiles = (uint8_t*)(dict + m.dict_words_pad);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  stage_dictionary(m, lds4, tid);
  uint8_t* tile = tiles + wave * kTileStride;
  const int j = lane & 15, kg = lane >> 4;
  for (uint32_t band = blockIdx.x; band < m.n_bands; band += gridDim.x) {
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    for (uint32_t st = wave; st < m.n_strips; st += kWaves) {
      const uint32_t g = band * m.n_strips + st;
      decode_group<kLmax>(dict, m.codes, m.goff[g], m.goff[g + 1], m.pad_word, tile, lane);
#pragma unroll
      for (int t = 0; t < 8; ++t) {
        const uint2 a8 = *(const uint2*)(tile + t * 512 + lane * 8);
        const uint32_t col = st * kGroupCols + t * 32 + kg * 8;
        uint4 xb = make_uint4(0, 0, 0, 0);
        if (j < batch) {
          const uint16_t* xr = x + (size_t)j * m.cols;
          if (x_fast) {
            if (col < m.cols) xb = *(const uint4*)(xr + col);
          } else {
            uint32_t e[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) e[k] = (col + k < m.cols) ? xr[col + k] : 0u;
            xb = make_uint4(e[0] | e[1] << 16, e[2] | e[3] << 16, e[4] | e[5] << 16, e[6] | e[7] << 16);
          }
        }
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(i8x8_to_bf16x8(a8), __builtin_bit_cast(bf16x8, xb), acc, 0, 0, 0);
      }
    }
    // Cross-wave sum in fixed order.  The tiles are free once every wave has finished its strips.
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
      const uint32_t row = band * kTileRows + 4 * (l >> 4) + v;   // accumulator register v of lane l holds row 4*(l/16)+v
      const int b = l & 15;                                       // and batch column l%16
      if (b < batch && row < m.rows) y[(size_t)b * m.rows + row] = s * m.scales[row];
    }
    __syncthreads();
  }
}

// Every wavefront takes whole groups (grid-stride), decodes into its LDS tile and copies the 16 x 256 block out.
template <int kLmax>
__global__ __launch_bounds__(kThreads, 1) void k_decompress(DevMat m, int8_t* __restrict__ out, int out_fast) {
  extern __shared__ uint4 lds4[];
  uint32_t* dict = (uint32_t*)lds4;
  uint8_t* tiles = (uint8_t*)(dict + m.dict_words_pad);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  stage_dictionary(m, lds4, tid);
  uint8_t* tile = tiles + wave * kTileStride;
  for (uint64_t g = (uint64_t)blockIdx.x * kWaves + wave; g < m.n_groups; g += (uint64_t)gridDim.x * kWaves) {
    decode_group<kLmax>(dict, m.codes, m.goff[g], m.goff[g + 1], m.pad_word, tile, lane);
    const uint32_t band = (uint32_t)(g / m.n_strips), st = (uint32_t)(g % m.n_strips);
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const int q = lane + 64 * t, i = q >> 4, pc = q & 15;   // row i of the band, 16-byte piece pc of its 256 columns
      const uint2 lo = *(const uint2*)(tile + (2 * pc) * 128 + i * 8);
      const uint2 hi = *(const uint2*)(tile + (2 * pc + 1) * 128 + i * 8);
      const uint32_t row = band * kTileRows + i, col = st * kGroupCols + pc * 16;
      if (row >= m.rows || col >= m.cols) continue;
      int8_t* dst = out + (size_t)row * m.cols + col;
      if (out_fast) {
        *(uint4*)dst = make_uint4(lo.x, lo.y, hi.x, hi.y);
      } else {
        const uint32_t w[4] = {lo.x, lo.y, hi.x, hi.y};
#pragma unroll
        for (int k = 0; k < 16; ++k)
          if (col + k < m.cols) dst[k] = (int8_t)(w[k >> 2] >> (8 * (k & 3)));
      }
    }
  }
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
};

namespace {

int hip_fail(const char* what, hipError_t e) {
  set_error(std::string(what) + ": " + hipGetErrorString(e));
  return TQ_E_HIP;
}

template <int kLmax>
int allow_lds(size_t bytes) {
  hipError_t e = hipFuncSetAttribute((const void*)k_matvec<kLmax>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
  if (e != hipSuccess) return hip_fail("hipFuncSetAttribute(matvec)", e);
  e = hipFuncSetAttribute((const void*)k_decompress<kLmax>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
  if (e != hipSuccess) return hip_fail("hipFuncSetAttribute(decompress)", e);
  return TQ_OK;
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
  int rc = allow_lds<1>(lds_bytes);
  if (rc == TQ_OK) rc = allow_lds<2>(lds_bytes);
  if (rc == TQ_OK) rc = allow_lds<3>(lds_bytes);
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
  const int x_fast = (h->m.cols % 8 == 0) && ((uintptr_t)x % 16 == 0);
  const unsigned grid = (unsigned)std::min<uint32_t>(h->m.n_bands, (uint32_t)h->n_cu);
  hipStream_t s = (hipStream_t)stream;
  switch (h->h.lmax) {
    case 1: hipLaunchKernelGGL(k_matvec<1>, dim3(grid), dim3(kThreads), h->lds_bytes, s, h->m, (const uint16_t*)x, (float*)y, batch, x_fast); break;
    case 2: hipLaunchKernelGGL(k_matvec<2>, dim3(grid), dim3(kThreads), h->lds_bytes, s, h->m, (const uint16_t*)x, (float*)y, batch, x_fast); break;
    default: hipLaunchKernelGGL(k_matvec<3>, dim3(grid), dim3(kThreads), h->lds_bytes, s, h->m, (const uint16_t*)x, (float*)y, batch, x_fast); break;
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return hip_fail("tq_matvec launch", e);
  return TQ_OK;
}

extern "C" int tq_decompress(tq_handle h, void* out, void* stream) {
  if (!h || !out) {
    set_error("tq_decompress: null argument");
    return TQ_E_INVALID_ARG;
  }
  const int out_fast = (h->m.cols % 16 == 0) && ((uintptr_t)out % 16 == 0);
  const uint64_t wg_needed = (h->m.n_groups + kWaves - 1) / kWaves;
  const unsigned grid = (unsigned)std::min<uint64_t>(wg_needed, (uint64_t)h->n_cu);
  hipStream_t s = (hipStream_t)stream;
  switch (h->h.lmax) {
    case 1: hipLaunchKernelGGL(k_decompress<1>, dim3(grid), dim3(kThreads), h->lds_bytes, s, h->m, (int8_t*)out, out_fast); break;
    case 2: hipLaunchKernelGGL(k_decompress<2>, dim3(grid), dim3(kThreads), h->lds_bytes, s, h->m, (int8_t*)out, out_fast); break;
    default: hipLaunchKernelGGL(k_decompress<3>, dim3(grid), dim3(kThreads), h->lds_bytes, s, h->m, (int8_t*)out, out_fast); break;
  }
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
