/*
 * CPU oracle for the dictionary codec and the matrix-vector product.  TEST INFRASTRUCTURE ONLY:
 * nothing in the product library includes, links or calls this file, and it shares no code with it.
 * Plain, slow and written to be checked against the paper by eye.
 *
 *   tqo_lzw_encode  - the LZW scheme of the paper's Background, section "Compression": start from
 *                     the 256 single-byte strings, repeatedly take the longest string already in the
 *                     dictionary, output its code, and add that string plus the following byte as a
 *                     new entry.  Two bounded-resource rules are added (the paper gives none):
 *                     entries stop being added once `max_entries` exist (the dictionary is then
 *                     frozen, never reset), and a match is at most `lmax` bytes and never crosses a
 *                     restart boundary (every `group_bytes` bytes of input).
 *   tqo_lzw_decode  - the decompression step of section 4 ("8-bit Quantization Compression"): each
 *                     codeword is replaced by its table sequence, reproducing the input exactly.
 *                     There is no escape/raw branch because the single bytes are always entries.
 *   tqo_gemv_f64    - the plain definition y[b][r] = s[r] * sum_j Q[r][j] * x[b][j] in float64,
 *                     summed in natural j order, scale applied last.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define TQO_LCAP 16 /* storage per entry; lmax may not exceed it */

/*
 * in:  S[n] bytes; restart boundary every group_bytes (last group may be short)
 * out: codes[] (capacity n), group_ncodes[n_groups] = codes emitted per group,
 *      ent_bytes[max_entries*TQO_LCAP], ent_len[max_entries], *n_entries
 * returns number of codes, or -1 on bad arguments / allocation failure.
 */
long long tqo_lzw_encode(const uint8_t *S, long long n, long long group_bytes, int max_entries, int lmax,
                         uint16_t *codes, uint32_t *group_ncodes, uint8_t *ent_bytes, uint8_t *ent_len,
                         int *n_entries_out) {
  if (max_entries < 256 || max_entries > 65536 || lmax < 1 || lmax > TQO_LCAP || group_bytes < 1) return -1;
  /* child[e*256 + b] = entry equal to (entry e followed by byte b), or -1 */
  int32_t *child = (int32_t *)malloc((size_t)max_entries * 256 * sizeof(int32_t));
  if (!child) return -1;
  for (size_t i = 0; i < (size_t)max_entries * 256; ++i) child[i] = -1;
  int n_entries = 256;
  for (int b = 0; b < 256; ++b) {
    ent_len[b] = 1;
    ent_bytes[(size_t)b * TQO_LCAP] = (uint8_t)b;
  }
  long long n_codes = 0;
  long long g = 0;
  for (long long gs = 0; gs < n; gs += group_bytes, ++g) {
    long long ge = gs + group_bytes < n ? gs + group_bytes : n;
    uint32_t emitted = 0;
    long long i = gs;
    while (i < ge) {
      int e = S[i];
      int m = 1;
      while (m < lmax && i + m < ge) {
        int c = child[(size_t)e * 256 + S[i + m]];
        if (c < 0) break;
        e = c;
        ++m;
      }
      codes[n_codes++] = (uint16_t)e;
      ++emitted;
      if (n_entries < max_entries && m < lmax && i + m < ge) {
        /* by construction (entry e, next byte) is not in the dictionary yet */
        int ne = n_entries++;
        child[(size_t)e * 256 + S[i + m]] = ne;
        memcpy(ent_bytes + (size_t)ne * TQO_LCAP, ent_bytes + (size_t)e * TQO_LCAP, (size_t)m);
        ent_bytes[(size_t)ne * TQO_LCAP + m] = S[i + m];
        ent_len[ne] = (uint8_t)(m + 1);
      }
      i += m;
    }
    group_ncodes[g] = emitted;
  }
  free(child);
  *n_entries_out = n_entries;
  return n_codes;
}

/*
 * Decodes groups [0, n_groups): group g uses codes[goff[g] .. goff[g+1]) and must produce exactly
 * min(group_bytes, n - g*group_bytes) bytes.  A code equal to pad_code produces nothing.
 * returns 0, or -(g+1) for the first group that is inconsistent (bad code, wrong length).
 */
long long tqo_lzw_decode(const uint16_t *codes, const uint32_t *goff, long long n_groups, long long group_bytes,
                         long long n, const uint8_t *ent_bytes, const uint8_t *ent_len, int n_entries, int pad_code,
                         uint8_t *S_out) {
  for (long long g = 0; g < n_groups; ++g) {
    long long gs = g * group_bytes;
    long long want = gs + group_bytes < n ? group_bytes : n - gs;
    long long c = 0;
    for (uint32_t p = goff[g]; p < goff[g + 1]; ++p) {
      int e = codes[p];
      if (e == pad_code) continue;
      if (e >= n_entries) return -(g + 1);
      int len = ent_len[e];
      if (c + len > want) return -(g + 1);
      memcpy(S_out + gs + c, ent_bytes + (size_t)e * TQO_LCAP, (size_t)len);
      c += len;
    }
    if (c != want) return -(g + 1);
  }
  return 0;
}

/* Q int8 [R][K] row-major, s fp32 [R], x fp32 [B][K] (bf16-representable values), y double [B][R] */
void tqo_gemv_f64(const int8_t *Q, const float *s, const float *x, long long R, long long K, long long B, double *y) {
  for (long long b = 0; b < B; ++b)
    for (long long r = 0; r < R; ++r) {
      double acc = 0.0;
      for (long long j = 0; j < K; ++j) acc += (double)Q[r * K + j] * (double)x[b * K + j];
      y[b * R + r] = (double)s[r] * acc;
    }
}
