/*
 * tq - dictionary-coded int8 weight matrices kept compressed in HBM, with a fused
 *      decode + dequantize + matrix-vector product for AMD MI355X (gfx950).
 *
 * Method (Tiny-QMoE): weights are quantized to 8 bits (paper section 3) and stored through a
 * dictionary code (paper Background "Compression": LZW - longest dictionary string, emit its code,
 * add string + next byte; section 4: 16-bit codewords, table lookup decompression that restores the
 * quantized parameters exactly).  At inference the parameters stay compressed and are expanded
 * layer by layer (Background "Inference"); here the expansion is fused into the matrix-vector
 * product so the expanded matrix is never written to memory.
 *
 * Plain C ABI.  Every function returns TQ_OK (0) or a negative TQ_E_* code; after a failure
 * tq_last_error_string() (thread-local) describes it.  No function throws.  "host" / "device" on a
 * pointer says which memory it must point to.
 */
#ifndef TQ_H
#define TQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define TQ_OK 0
#define TQ_E_INVALID_ARG (-1) /* null pointer, zero size, misaligned device pointer */
#define TQ_E_BAD_BLOB (-2)    /* container fails validation */
#define TQ_E_UNSUPPORTED (-3) /* e.g. batch > TQ_MAX_BATCH, dictionary too large for LDS */
#define TQ_E_OOM (-4)
#define TQ_E_HIP (-5)         /* a HIP runtime call or kernel launch failed */

#define TQ_MAX_BATCH 16
/* Dictionary entries (incl. the 256 single bytes) that fit the 120 KB of LDS the kernels give the dictionary:
 * an entry holds at most 2 weights and takes one 32-bit word there (two bf16 values); one more word is the pad entry. */
#define TQ_MAX_ENTRIES_DEVICE 30719
#define TQ_MAX_LMAX 4
#define TQ_DEFAULT_LMAX 2
#define TQ_DEFAULT_SEG_COLS 256

typedef struct tq_matrix *tq_handle;

#define TQ_DICT_LZW 0
#define TQ_DICT_FREQUENCY 1
#define TQ_PACK_NONE 0u
#define TQ_PACK_NIBBLES 1u

/* Encoder options; zero-initialise and set what you need (0 = default). */
typedef struct tq_encode_opts {
  uint32_t max_entries; /* dictionary size cap incl. the 256 single bytes; 256..TQ_MAX_ENTRIES_DEVICE;
                           0 = TQ_MAX_ENTRIES_DEVICE */
  uint32_t lmax;        /* longest run a dictionary entry may hold, 1..TQ_MAX_LMAX; 0 = TQ_DEFAULT_LMAX */
  uint32_t n_threads;   /* host threads for the frozen-dictionary part of the parse; 0 = all cores (max 16) */
  uint32_t seg_cols;    /* columns per independently decodable segment (the tile width of the per-tile stream offsets):
                           multiple of 16 in 16..1024; 0 = TQ_DEFAULT_SEG_COLS (half of it with TQ_PACK_NIBBLES) */
  const void *dict_from;    /* NULL, or a container made earlier: its dictionary is taken over and LZW goes on from
                               there (one dictionary over a sequence of matrices, as the table of paper section 4 is
                               built over all parameters of the model).  Once the dictionary is full every later
                               matrix of the sequence gets byte-identical dictionaries, which the device side stores
                               and stages once. */
  uint64_t dict_from_bytes; /* size of that container */
  uint32_t dictionary;      /* TQ_DICT_LZW (0, default): LZW growth with freeze, the paper's Background "Compression".
                               TQ_DICT_FREQUENCY: the dictionary is fixed before the parse - dict_from's if given, else
                               the 256 single bytes plus the most frequent pairs of neighbouring bytes of this matrix
                               (counted at every offset inside a segment; most frequent first, equally frequent ones in
                               order of first appearance: how the paper's section 4 picks its table), as many as
                               max_entries leaves room for - and the parse is the same greedy longest match.  Same
                               container, same kernels. */
  uint32_t bits;            /* tq_encode only: quantization width b, 2..8; 0 = 8.  Levels -qmax..qmax with
                               qmax = 2^(b-1) - 1 (8: 127, 6: 31, 4: 7, 2: 1, the ternary case): the widths the paper's
                               section 3 tried.  The values stay one per byte, so container and kernels are the same;
                               with fewer distinct bytes more of the pairs get a dictionary entry. */
  uint32_t packing;         /* TQ_PACK_NONE (0, default): one value per byte.  TQ_PACK_NIBBLES (widths of at most 4 bits;
                               tq_encode: bits 2..4, tq_encode_quantized: values in [-8, 7]; an even number of columns):
                               two values share a byte - column 2j in bits 0..3, column 2j + 1 in bits 4..7, 4-bit two's
                               complement - and that byte matrix, half as wide, is what the dictionary codes; seg_cols
                               then counts bytes.  A code stands for up to four weights.  The kernels expand the
                               nibbles where they dequantize; x, y and the output of tq_decompress keep their shapes. */
  uint32_t reserved;
} tq_encode_opts;

typedef struct tq_info {
  uint32_t rows, cols;         /* logical shape R x K, y = W x */
  uint32_t seg_cols, n_panels; /* stored bytes per segment (= columns, or two columns each with TQ_PACK_NIBBLES); segments per row */
  uint32_t n_entries, lmax;
  uint64_t n_units, n_codes;   /* units of 16 rows x 4 segments; 16-bit codes stored, incl. padding codes */
  uint64_t n_real_codes;       /* codes of the LZW parse itself (n_codes minus padding) */
  uint64_t dict_bytes, offset_bytes, code_bytes, scale_bytes;
  uint64_t compressed_bytes; /* sum of the four sections = bytes the kernels must read from HBM */
  uint32_t lane_spread;      /* the 64 segments of a unit are decoded in step, 4 codes of each at a time: the largest
                                difference, in columns, between two of them that are both still incomplete.  The batched
                                product keeps only a window of every segment in LDS when this stays small (see tq_matvec). */
  uint32_t packing;          /* TQ_PACK_NONE or TQ_PACK_NIBBLES (see tq_encode_opts) */
} tq_info;

/*
 * Host-side encoder (off the hot path).  w: host, fp32 [rows][cols] row-major.
 * Quantizes each row to int8 (symmetric, scale = absmax/127, round-half-to-even: the 8-bit setting
 * of paper section 3 at per-row granularity), cuts the rows into segments of seg_cols columns, runs LZW
 * with a frozen, size-capped dictionary over the segments (paper Background "Compression"; a run never
 * crosses a segment boundary), and lays out the container: header, dictionary, per-unit code offsets,
 * 16-bit code stream with the 64 lane streams of a unit interleaved, per-row scales.
 * *blob is allocated by the library; release it with tq_free_blob.  Deterministic for any n_threads.
 */
int tq_encode(const float *w, uint32_t rows, uint32_t cols, const tq_encode_opts *opts, void **blob, size_t *blob_bytes);

/* Same, from already quantized weights.  q: host int8 [rows][cols]; scales: host fp32 [rows].
 * Any byte value (including -128) is allowed. */
int tq_encode_quantized(const int8_t *q, const float *scales, uint32_t rows, uint32_t cols, const tq_encode_opts *opts,
                        void **blob, size_t *blob_bytes);

void tq_free_blob(void *blob);

/* Full host-side validation of a container (no GPU needed): header, section bounds, every dictionary
 * entry, monotone unit offsets, every code in range, padding codes only at the end of a lane stream, and
 * every lane stream's runs summing to exactly its segment's length.  info may be NULL. */
int tq_validate_blob(const void *blob, size_t blob_bytes, tq_info *info);

/*
 * blob: host.  Validates as tq_validate_blob does (so the kernels need no bounds checks on codes),
 * copies dictionary, offsets, codes and scales into device memory owned by the handle, on the
 * current HIP device.  Synchronous.  The caller may free blob on return.
 * This is the "parameters stay compressed in memory" state of the paper's Background "Inference".
 */
int tq_create_from_encoded(const void *blob, size_t blob_bytes, tq_handle *out);

/*
 * Fused decode + dequantize + matrix-vector product (paper section 4 decompression feeding the
 * layer's product, Background "Inference"), y[b][r] = scale[r] * sum_j Q[r][j] * x[b][j].
 *   x: device, bf16 [batch][cols] row-major contiguous.
 *   y: device, fp32 [batch][rows] row-major, fully overwritten.
 *   stream: a hipStream_t (NULL = default stream).
 * Asynchronous: returns after the launch; no host synchronisation, no allocation, no change to the
 * handle, so it may be captured in a HIP graph and called concurrently on different streams.
 * 1 <= batch <= TQ_MAX_BATCH, else TQ_E_UNSUPPORTED.  x and y must stay alive until the stream passes
 * the kernel.  The result is deterministic (fixed summation order).  x values must be finite: a lane that has
 * run out of codes multiplies activations of later columns by zero, so an infinity or NaN anywhere in x can make
 * any output of that batch row non-finite (the plain definition does the same wherever a weight is zero).
 * batch 1 and batch 2 run the dot-product kernel (activations gathered from an LDS image of x, which holds both rows
 * at batch 2; a matrix whose rows are too long for that image to fit the LDS beside the dictionary - more than 8192
 * columns with a full dictionary, more with a smaller one - goes on as batch 3 does, slower but to the same result);
 * batch 3..16 run an MFMA kernel (the batch is the N dimension).  Of those there are two.  The ring kernel keeps 128 bytes of every segment in LDS
 * and multiplies while it decodes; it takes matrices whose lane_spread (tq_info) is at most 113 columns, whose rows
 * are a whole number of units (cols a multiple of 4 * seg_cols), with seg_cols a multiple of 32 up to 256 and x
 * 16-byte aligned, in calls that bring at least 24 bands of 16 rows per compute unit (tq_set_ring_min_bands_per_cu
 * changes that number).  Everything else goes through the
 * whole-strip kernel, which decodes a unit into an LDS tile before it multiplies it.  The ring kernel adds the partial
 * sums of a row's later quads (groups of 4 segments) to y with atomic adds, always in the same order; y must not be
 * read or written by anything else on the device while the call runs (true of any output buffer).
 * Containers of packed 4-bit weights (TQ_PACK_NIBBLES): cols is the number of weights per row, twice the stored bytes;
 * batch 1 and 2 run the dot-product kernel with four weights per dictionary entry, batch 3..16 the same two MFMA
 * kernels (the ring kernel then takes segments of at most 128 bytes).
 */
int tq_matvec(tq_handle h, const void *x, void *y, int batch, void *stream);

/* Tuning knob of the choice between the two MFMA kernels of tq_matvec (see there): the ring kernel hands whole bands
 * of 16 rows to its wavefronts and is taken by launches that bring at least this many bands per compute unit
 * (default 24; 0 = whenever a matrix allows it).  Process-wide, atomic; affects the calls and the prepared steps made
 * after it returns.  Results stay within the tolerance either way (the two kernels add in different orders). */
int tq_set_ring_min_bands_per_cu(uint32_t bands_per_cu);

/*
 * tq_matvec for n independent matrices in as few launches as possible (for instance the q, k and v projections of a
 * layer, or gate and up, or every product of a step when their inputs are all known: products that do not depend on
 * each other; the paper's layer-by-layer expansion, Background "Inference", leaves their order free).
 * hs, xs, ys: host arrays of n handles / device x pointers / device y pointers, with the meaning they have in
 * tq_matvec; all share `batch`.  One kernel launch serves up to 128 matrices: the rows of all of them are cut into
 * equal shares of work, one per compute unit, so small matrices fill the GPU side by side, and a workgroup stages a
 * dictionary again only when the next matrix holds a different one (matrices encoded with dict_from share theirs).
 * Each output is a deterministic function of its matrix, x and the set of matrices in the call (the split of the rows
 * over workgroups, hence the summation order across a row's segments, depends on that set); it equals what tq_matvec
 * returns up to that reordering of fp32 additions.  Same asynchrony rules as tq_matvec.
 */
int tq_matvec_multi(int n, const tq_handle *hs, const void *const *xs, void *const *ys, int batch, void *stream);

/*
 * The gated pair of a feed-forward block in one pass (the products of the gate and the up projection read the same x;
 * their elementwise combination is fused into the kernel that produces them instead of costing two more passes over
 * their outputs): a container made by tq_encode_gate_up holds the two R x K matrices row-interleaved (row 2r = gate
 * row r, row 2r + 1 = up row r; each row keeps its own scale), and
 *   y[b][r] = silu(g) * u,  g = scale[2r] * sum_j Q[2r][j] x[b][j],  u = scale[2r+1] * sum_j Q[2r+1][j] x[b][j],
 *   silu(g) = g / (1 + exp(-g)) in fp32.
 * y: device, fp32 [batch][rows / 2].  Works on any handle with an even number of rows; otherwise as tq_matvec /
 * tq_matvec_multi (batch 1 and 2: dot-product kernel; batch 3..16: the whole-strip MFMA kernel).
 */
int tq_encode_gate_up(const float *w_gate, const float *w_up, uint32_t rows, uint32_t cols, const tq_encode_opts *opts,
                      void **blob, size_t *blob_bytes);
int tq_matvec_gate_up(tq_handle h, const void *x, void *y, int batch, void *stream);
int tq_matvec_gate_up_multi(int n, const tq_handle *hs, const void *const *xs, void *const *ys, int batch, void *stream);

/*
 * A prepared step: tq_matvec_multi (flags 0), tq_matvec_gate_up_multi (TQ_STEP_GATE_UP) or tq_decompress_multi
 * (TQ_STEP_DECOMPRESS) for a fixed set of matrices and
 * buffers, with everything but the stream decided once - for a decode loop that runs the same products on the same
 * buffers token after token (the layer-by-layer use of the compressed parameters in the paper's Background "Inference").
 * tq_step_create does what those calls do before they launch (argument checks, which kernel takes which matrix, the
 * split of the work) and copies the list of (matrix description, x, y) to device memory, which it allocates
 * (n * 104 bytes; synchronous, not for the hot path).  A launch that reads its matrices from that table serves up to
 * 896 of them where the kernel arguments hold 128: a whole decode step of a model becomes one kernel launch.
 * tq_step_launch only launches: no allocation, no synchronisation, nothing of the step is changed, so it may be
 * captured in a HIP graph and the same step may run on several streams (they write the same y).  Results are those of
 * the calls it stands for, up to the order of fp32 additions where the work is split differently.
 * The matrices, x and y must outlive the step and keep their addresses; x and y are read and written at every launch.
 * Errors as for tq_matvec_multi; tq_step_destroy(NULL) is a no-op; no launch of the step may be in flight when it is
 * destroyed.
 */
#define TQ_STEP_GATE_UP 1u
#define TQ_STEP_DECOMPRESS 2u /* the step stands for tq_decompress_multi: ys are the int8 output matrices, xs may be
                                 NULL and batch is not used */
typedef struct tq_step *tq_step_handle;
typedef struct tq_step_info {
  uint32_t n_matrices, n_launches; /* kernel launches one tq_step_launch makes (a staged step that runs as one kernel: 1,
                                      not counting the small launch that clears its stage counters) */
  uint64_t table_bytes;            /* device memory the step holds */
  uint32_t n_stages;               /* staged steps: number of stages, else 0 */
  uint32_t persistent;             /* 1: all stages run in one kernel launch with device-side hand-over between them */
  uint32_t fault;                  /* 1: a launch of the staged step gave up waiting at a hand-over (see tq_step_create_staged) */
  uint32_t reserved;
} tq_step_info;
int tq_step_create(int n, const tq_handle *hs, const void *const *xs, void *const *ys, int batch, uint32_t flags,
                   tq_step_handle *out);
/*
 * A staged step: the products of a decode step that DEPEND on each other, prepared once and run in order - the paper's
 * layer-by-layer use of the compressed parameters (Background "Inference"; section 5: the model's linear layers are
 * replaced by compressed counterparts): within a transformer layer q, k and v can run side by side, the output
 * projection needs their result, gate and up need the output projection's, down needs theirs, and the next layer needs
 * down's.  stage[i] (host array, n entries, starting at 0, never decreasing, never skipping) says which stage product i
 * belongs to; the products of one stage are independent of each other; no product of stage s + 1 reads its x before
 * every y of stage s has been stored and made visible (so whatever produces that x from those y on the same stream
 * order - or the caller's own kernels between two steps - finds them).  The activations x and outputs y are the
 * caller's, as in tq_step_create; this call only orders the products.
 * When every matrix takes the dot-product kernel (batch 1 or 2; ordinary or packed weights; rows that fit its LDS image;
 * no runs longer than 2 bytes) the whole step is one kernel launch: one workgroup per compute unit walks the stages, the
 * dictionary stays in LDS across them, and between two stages the workgroups hand over through a counter in device
 * memory (outputs and activations of such a step are stored and loaded device-coherently).  That needs all workgroups resident together, which holds when nothing
 * else occupies the GPU's compute units while the step runs; a wait is bounded (tq_step_set_spin_limit; about two
 * seconds by default): a workgroup that gives up sets a fault flag, every other wait of that launch ends at once, the
 * results must not be used, tq_step_get_info reports fault = 1 and later launches return TQ_E_HIP.
 * Otherwise (larger batches, long runs, mixed kinds) each stage gets the launches tq_matvec_multi would make, in order
 * on the stream.  Results equal tq_matvec_multi's for the same products up to the order of fp32 additions.
 * flags: none defined yet, pass 0.  Launch with tq_step_launch, release with tq_step_destroy.
 */
int tq_step_create_staged(int n, const tq_handle *hs, const void *const *xs, void *const *ys, const int *stage, int batch,
                          uint32_t flags, tq_step_handle *out);
/* Polls of a stage counter (a microsecond or two each) after which a workgroup of a staged step gives up waiting. */
int tq_step_set_spin_limit(tq_step_handle s, uint32_t polls);
int tq_step_launch(tq_step_handle s, void *stream);
int tq_step_get_info(tq_step_handle s, tq_step_info *out);
int tq_step_destroy(tq_step_handle s);

/*
 * For callers that cannot allocate device memory where they call the library - code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc: tq_matvec_multi for up to TQ_STATIC_MAX_MATRICES matrices with the
 * job table of a prepared step, so one kernel launch serves them all, but the table lives in a fixed array of
 * TQ_STATIC_MAX_MATRICES * 120 bytes that is part of the library's device image (each GPU the library runs on holds
 * it until the process ends) instead of memory a tq_step_create allocates.  The call plans the launches as
 * tq_step_create does, fills the table through small writer launches on `stream` (ahead of the product launches, on
 * the same stream; n / 160 of them, rounded up) and launches the products.  It makes no hipMalloc, hipFree or other
 * allocating HIP call; the planning on the host may use the C++ heap.  n > TQ_STATIC_MAX_MATRICES: TQ_E_UNSUPPORTED.
 * Arguments, results and asynchrony as for tq_matvec_multi; results are those of a prepared step for the same
 * matrices and buffers.  All calls on one GPU share the one table, which keeps the entries of the last call: two
 * calls whose execution overlaps on one GPU (different streams, or a captured graph replayed while another call
 * runs) race on it and must be ordered by the caller; calls on one stream are ordered by the stream.
 */
#define TQ_STATIC_MAX_MATRICES 896
int tq_matvec_multi_static(int n, const tq_handle *hs, const void *const *xs, void *const *ys, int batch, void *stream);

/*
 * Un-fused form: expand the whole matrix (paper section 4, Listing "Decompressing Model Weights").
 *   out: device, int8 [rows][cols] row-major, fully overwritten, bit-exact quantized weights.
 * Same asynchrony rules as tq_matvec.
 */
int tq_decompress(tq_handle h, void *out, void *stream);

/* tq_decompress for n matrices in as few launches as possible (up to 128 matrices per launch; the work is shared out
 * as in tq_matvec_multi).  outs: host array of n device pointers, outs[i] as `out` of tq_decompress for hs[i]. */
int tq_decompress_multi(int n, const tq_handle *hs, void *const *outs, void *stream);

int tq_get_info(tq_handle h, tq_info *out);

/* Frees the device memory.  The caller guarantees no work using the handle is in flight.  NULL is a no-op. */
int tq_destroy(tq_handle h);

const char *tq_last_error_string(void);

/*
 * The stream format of the paper's section 4 listings, taken literally (the container above is this library's own
 * reading of the method; this is the format the paper prints).
 *
 * Table (Listing "Finding Frequent Sequences"): every window of TQ_LISTING_SEQ = 4 consecutive byte values of every
 * parameter, at every offset, never across two parameters, is counted; the top_k most frequent windows, most frequent
 * first and among equally frequent ones in order of first appearance, get the codewords 1, 2, ...
 * Stream (Listing "Compressing Model Weights"), per parameter, 16-bit words: the values are cut into groups of 4 from
 * the start; a group in the table becomes its codeword, any other group the marker 0xFFFF followed by its 4 values,
 * one word each; fewer than 4 values left at the end follow a marker likewise.
 * top_k is at most TQ_LISTING_MAX_TOP_K = 65534: with the 65535 the listing prints as default, the last codeword
 * would have the marker's value.  Codeword 0 is never assigned.
 */
#define TQ_LISTING_SEQ 4
#define TQ_LISTING_MAX_TOP_K 65534u

typedef struct tq_listing_s *tq_listing;

typedef struct tq_listing_info {
  uint64_t n_values;  /* byte values the stream stands for */
  uint64_t n_words;   /* 16-bit words of the stream */
  uint64_t n_tokens;  /* codewords + markers */
  uint64_t n_escapes; /* markers */
  uint32_t n_table;   /* table entries */
  uint32_t reserved;
} tq_listing_info;

/* Host.  params[i]: lens[i] byte values.  *table: n_table x 4 values, entry i = codeword i + 1; allocated by the
 * library, release with tq_free_blob.  Fewer than top_k entries when there are fewer distinct windows. */
int tq_listing_build_table(const uint8_t *const *params, const uint64_t *lens, uint32_t n_params, uint32_t top_k,
                           uint8_t **table, uint32_t *n_table);

/* Host.  One parameter -> its words (allocated by the library, release with tq_free_blob).  Table entries must be
 * distinct. */
int tq_listing_compress(const uint8_t *values, uint64_t n_values, const uint8_t *table, uint32_t n_table,
                        uint16_t **words, uint64_t *n_words);

/* words, table: host.  Validates the stream (every codeword in the table, raw values at most 255, a marker followed by
 * 4 values except at the very end, where 1..3 are allowed), copies stream and table into device memory the handle
 * owns, on the current HIP device, and keeps the number of tokens ahead of every block of words, which is what lets
 * the device expand the stream in parallel.  Synchronous; the caller may free words and table on return. */
int tq_listing_create(const uint16_t *words, uint64_t n_words, const uint8_t *table, uint32_t n_table, tq_listing *out);

/* Listing "Decompressing Model Weights" on the device.  out: device, n_values bytes (tq_listing_get_info), fully
 * overwritten with exactly the values that were compressed.  Asynchronous on `stream` (a hipStream_t, NULL = default
 * stream); no allocation, no change to the handle. */
int tq_listing_decompress(tq_listing h, void *out, void *stream);

int tq_listing_get_info(tq_listing h, tq_listing_info *out);

/* Frees the device memory; no work of the handle may be in flight.  NULL is a no-op. */
int tq_listing_destroy(tq_listing h);

#ifdef __cplusplus
}
#endif
#endif /* TQ_H */
