/*
 * CPU oracle for the dictionary codec and the matrix-vector product.  TEST INFRASTRUCTURE ONLY:
 * nothing in the product library includes, links or calls this file, and it shares no code with it.
 * Plain, slow and written to be checked against the paper by eye.
 *
 *   tqo_lzw_encode  - the LZW scheme of the paper's Background, section "Compression": start from
 *                     the 256 single-byte strings, repeatedly take the longest string already in the
 *                     dictionary, output its code, and add that string plus the following byte as a
 *                     new entry.  Bounded-resource rules are added (the paper gives none):
 *                     entries stop being added once `max_entries` exist (the dictionary is then
 *                     frozen, never reset); a match is at most `lmax` bytes and never crosses a
 *                     restart boundary (the input is a sequence of segments of given lengths); and,
 *                     when a unit budget is given, an entry is added only while the dictionary's
 *                     storage stays inside it, an entry of up to 2 bytes costing 1 unit and a longer
 *                     one 2 (an entry that does not fit is skipped; the parse goes on unchanged).
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
 * in:  S[n] bytes = n_segs segments back to back, segment g has seg_len[g] bytes (may be 0)
 *      unit_budget: 0 for none, else the most units the dictionary may take (entries of 1..2 bytes: 1 unit each, longer: 2)
 *      n_init: 0 to start from the 256 single bytes, or the number of entries (>= 256) already present in
 *      ent_bytes / ent_len: the dictionary a previous call left behind, so that one LZW dictionary runs over a
 *      sequence of inputs (section 4 of the paper builds its table over all parameters of the model)
 * out: codes[] (capacity n), seg_ncodes[n_segs] = codes emitted per segment,
 *      ent_bytes[max_entries*TQO_LCAP], ent_len[max_entries], *n_entries
 * returns number of codes, or -1 on bad arguments / allocation failure.
 */
long long tqo_lzw_encode(const uint8_t *S, long long n, const uint32_t *seg_len, long long n_segs, int max_entries,
                         int lmax, long long unit_budget, int n_init, uint16_t *codes, uint32_t *seg_ncodes,
                         uint8_t *ent_bytes, uint8_t *ent_len, int *n_entries_out) {
  if (max_entries < 256 || max_entries > 65536 || lmax < 1 || lmax > TQO_LCAP || n_segs < 0) return -1;
  if (n_init != 0 && (n_init < 256 || n_init > max_entries)) return -1;
  long long total = 0;
  for (long long g = 0; g < n_segs; ++g) total += seg_len[g];
  if (total != n) return -1;
  /* child[e*256 + b] = entry equal to (entry e followed by byte b), or -1 */
  int32_t *child = (int32_t *)malloc((size_t)max_entries * 256 * sizeof(int32_t));
  if (!child) return -1;
  for (size_t i = 0; i < (size_t)max_entries * 256; ++i) child[i] = -1;
  int n_entries = 256;
  long long units = 256; /* the single bytes */
  for (int b = 0; b < 256; ++b) {
    ent_len[b] = 1;
    ent_bytes[(size_t)b * TQO_LCAP] = (uint8_t)b;
  }
  /* carried-over entries: each is (an earlier entry) + one byte, because LZW only ever adds such strings */
  for (int e = 256; e < n_init; ++e) {
    int len = ent_len[e], par = ent_bytes[(size_t)e * TQO_LCAP];
    if (len < 2 || len > lmax) { free(child); return -1; }
    for (int k = 1; k < len - 1 && par >= 0; ++k) par = child[(size_t)par * 256 + ent_bytes[(size_t)e * TQO_LCAP + k]];
    if (par < 0 || child[(size_t)par * 256 + ent_bytes[(size_t)e * TQO_LCAP + len - 1]] >= 0) { free(child); return -1; }
    child[(size_t)par * 256 + ent_bytes[(size_t)e * TQO_LCAP + len - 1]] = e;
    n_entries = e + 1;
    units += len <= 2 ? 1 : 2;
  }
  long long n_codes = 0;
  long long gs = 0;
  for (long long g = 0; g < n_segs; ++g) {
    long long ge = gs + seg_len[g];
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
      int cost = m + 1 <= 2 ? 1 : 2; /* units the new entry (m + 1 bytes) would take */
      if (n_entries < max_entries && m < lmax && i + m < ge && (unit_budget <= 0 || units + cost <= unit_budget)) {
        /* by construction (entry e, next byte) is not in the dictionary yet */
        int ne = n_entries++;
        units += cost;
        child[(size_t)e * 256 + S[i + m]] = ne;
        memcpy(ent_bytes + (size_t)ne * TQO_LCAP, ent_bytes + (size_t)e * TQO_LCAP, (size_t)m);
        ent_bytes[(size_t)ne * TQO_LCAP + m] = S[i + m];
        ent_len[ne] = (uint8_t)(m + 1);
      }
      i += m;
    }
    seg_ncodes[g] = emitted;
    gs = ge;
  }
  free(child);
  *n_entries_out = n_entries;
  return n_codes;
}

/*
 * Decodes segments [0, n_segs) from the interleaved layout: the segments come in units of 64 (segment g is lane
 * g % 64 of unit g / 64); code k of lane l of unit u sits at codes[(uoff[u] + k / 4) * 256 + l * 4 + k % 4] and a
 * lane's stream has (uoff[u+1] - uoff[u]) * 4 codes.  Segment g must produce exactly seg_len[g] bytes, written
 * back to back to S_out.  A code equal to pad_code produces nothing and may only be followed by pad codes.
 * returns 0, or -(g+1) for the first segment that is inconsistent (bad code, wrong length, code after a pad).
 */
long long tqo_lzw_decode(const uint16_t *codes, const uint32_t *uoff, const uint32_t *seg_len, long long n_segs,
                         const uint8_t *ent_bytes, const uint8_t *ent_len, int n_entries, int pad_code, uint8_t *S_out) {
  long long pos = 0;
  for (long long g = 0; g < n_segs; ++g) {
    long long u = g / 64, l = g % 64;
    long long steps = ((long long)uoff[u + 1] - (long long)uoff[u]) * 4;
    long long want = seg_len[g];
    long long c = 0;
    int seen_pad = 0;
    for (long long k = 0; k < steps; ++k) {
      int e = codes[((long long)uoff[u] + k / 4) * 256 + l * 4 + k % 4];
      if (e == pad_code) {
        seen_pad = 1;
        continue;
      }
      if (seen_pad || e >= n_entries) return -(g + 1);
      int len = ent_len[e];
      if (c + len > want) return -(g + 1);
      memcpy(S_out + pos + c, ent_bytes + (size_t)e * TQO_LCAP, (size_t)len);
      c += len;
    }
    if (c != want) return -(g + 1);
    pos += want;
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
