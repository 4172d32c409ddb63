"""pytest plugin that plants ONE mistake in the CPU oracle, named by the environment variable TQ_PLANTED_MISTAKE.

Used only by test_oracle_pins_catch_mistakes.py, which runs the oracle's pin tests in a child process with this plugin
loaded and expects them to fail: a pin that lets a plausible mistake through pins nothing.  Every mistake is planted
in the oracle (Python: by replacing a function of the module; C: by compiling an edited copy of tq_oracle.c into a
temporary folder), on the CPU; the product library is never touched.
"""
import os
import subprocess
import sys
import tempfile

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _edited_c_library(O, old: str, new: str):
    """Compile oracle/tq_oracle.c with `old` replaced by `new` (exactly one occurrence) and make the oracle load it."""
    src = open(os.path.join(ROOT, "oracle", "tq_oracle.c")).read()
    assert src.count(old) == 1, f"the text to edit occurs {src.count(old)} times"
    folder = tempfile.mkdtemp(prefix="tq_planted_")
    c_file, so_file = os.path.join(folder, "tq_oracle_edited.c"), os.path.join(folder, "libtqoracle_edited.so")
    open(c_file, "w").write(src.replace(old, new))
    subprocess.check_call(["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-o", so_file, c_file])
    O.build_oracle_lib = lambda force=False: so_file
    O._LIB = None


def _plant(name: str):
    if ROOT not in sys.path:
        sys.path.insert(0, ROOT)
    from oracle import listing_oracle as L
    from oracle import oracle as O

    # ---- quantizer
    if name.startswith("quantize_"):
        def quantize_rows(W, bits=8):
            qmax = np.float32((1 << (bits - 1)) - 1)
            W = np.ascontiguousarray(W, dtype=np.float32)
            amax = np.max(np.abs(W), axis=1).astype(np.float32)
            if name == "quantize_one_scale_for_the_matrix":
                amax = np.full_like(amax, amax.max())
            s = (amax / (qmax + 1 if name == "quantize_divides_by_two_to_the_bits_minus_one" else qmax)).astype(np.float32)
            safe = np.where(s > 0, s, np.float32(1.0)).astype(np.float32)
            t = (W / safe[:, None]).astype(np.float32)
            r = {"quantize_rounds_half_up": lambda v: np.floor(v + np.float32(0.5)),
                 "quantize_truncates": np.trunc}.get(name, np.rint)(t)
            q = np.where(s[:, None] > 0, np.clip(r, -qmax, qmax), 0.0)
            return q.astype(np.int8), s
        assert name in ("quantize_one_scale_for_the_matrix", "quantize_divides_by_two_to_the_bits_minus_one",
                        "quantize_rounds_half_up", "quantize_truncates"), name
        O.quantize_rows = quantize_rows

    # ---- byte order of the matrix in the codec's input
    elif name in ("segments_lane_bits_swapped", "segments_quad_major"):
        def segment_table(rows, cols, seg_cols=O.DEFAULT_SEG_COLS):
            n_bands, n_panels, n_quads = O.geometry(rows, cols, seg_cols)
            if name == "segments_quad_major":
                quad, band, lane = np.meshgrid(np.arange(n_quads), np.arange(n_bands), np.arange(64), indexing="ij")
                r, p = 16 * band + (lane & 15), 4 * quad + (lane >> 4)
            else:
                band, quad, lane = np.meshgrid(np.arange(n_bands), np.arange(n_quads), np.arange(64), indexing="ij")
                r, p = 16 * band + (lane >> 2), 4 * quad + (lane & 3)
            row, panel = r.reshape(-1).astype(np.int64), p.reshape(-1).astype(np.int64)
            col0 = panel * seg_cols
            length = np.where((row < rows) & (panel < n_panels), np.minimum(seg_cols, cols - col0), 0)
            return row, col0, np.maximum(length, 0).astype(np.int64)
        O.segment_table = segment_table

    elif name == "bytes_offset_binary":
        real_serialize, real_deserialize = O.serialize, O.deserialize

        def serialize(Q, seg_cols=O.DEFAULT_SEG_COLS):
            S, length = real_serialize(Q, seg_cols)
            return S ^ np.uint8(0x80), length          # value + 128 instead of two's complement

        def deserialize(S, rows, cols, seg_cols=O.DEFAULT_SEG_COLS):
            return real_deserialize(np.asarray(S, np.uint8) ^ np.uint8(0x80), rows, cols, seg_cols)
        O.serialize, O.deserialize = serialize, deserialize   # consistent with each other

    elif name == "chunk_layout_lane_minor":
        def interleave(codes, seg_ncodes, pad_code):
            n_segs = int(seg_ncodes.size)
            n_units = -(-n_segs // 64)
            cnt = np.zeros(n_units * 64, np.int64)
            cnt[:n_segs] = seg_ncodes
            unit_chunks = -(-cnt.reshape(n_units, 64).max(axis=1) // 4) if n_units else np.zeros(0, np.int64)
            uoff = np.zeros(n_units + 1, np.int64)
            np.cumsum(unit_chunks, out=uoff[1:])
            stream = np.full(int(uoff[-1]) * 256, pad_code, dtype=np.uint16)
            src = np.zeros(cnt.size + 1, np.int64)
            np.cumsum(cnt, out=src[1:])
            seg = np.repeat(np.arange(cnt.size), cnt)
            k = np.arange(codes.size, dtype=np.int64) - src[seg]
            stream[(uoff[seg // 64] + k // 4) * 256 + (k % 4) * 64 + seg % 64] = codes
            return stream, uoff.astype(np.uint32)
        O.interleave = interleave
        _edited_c_library(O, "k / 4) * 256 + l * 4 + k % 4];", "k / 4) * 256 + (k % 4) * 64 + l];")   # reader agrees

    # ---- packed 4-bit values
    elif name == "nibbles_high_first":
        def pack_nibbles(Q):
            Q = np.asarray(Q, dtype=np.int64)
            if Q.shape[1] % 2 or Q.min(initial=0) < -8 or Q.max(initial=0) > 7:
                raise ValueError("pack_nibbles: an even number of columns of values in [-8, 7]")
            return (16 * (Q[:, 0::2] % 16) + Q[:, 1::2] % 16).astype(np.uint8).view(np.int8)

        def unpack_nibbles(P):
            b = np.asarray(P).view(np.uint8).astype(np.int64)
            lo, hi = b % 16, b // 16
            Q = np.empty((b.shape[0], 2 * b.shape[1]), np.int64)
            Q[:, 0::2] = np.where(hi >= 8, hi - 16, hi)
            Q[:, 1::2] = np.where(lo >= 8, lo - 16, lo)
            return Q.astype(np.int8)
        O.pack_nibbles, O.unpack_nibbles = pack_nibbles, unpack_nibbles   # consistent with each other, wrong order
    elif name == "nibbles_not_sign_extended":
        def unpack_nibbles(P):
            b = np.asarray(P).view(np.uint8).astype(np.int64)
            Q = np.empty((b.shape[0], 2 * b.shape[1]), np.int64)
            Q[:, 0::2], Q[:, 1::2] = b % 16, b // 16
            return Q.astype(np.int8)
        O.unpack_nibbles = unpack_nibbles

    # ---- dictionary picked by frequency
    elif name in ("frequency_ties_by_value", "frequency_counts_across_segments"):
        def frequency_dictionary(S, seg_len, max_entries=30719, lmax=2):
            S = np.ascontiguousarray(S, dtype=np.uint8)
            eb = np.zeros((256, O.LCAP), np.uint8)
            eb[:, 0] = np.arange(256)
            el = np.ones(256, np.uint8)
            room = max_entries - 256
            if lmax < 2 or room <= 0 or S.size < 2:
                return O.Dictionary(eb, el)
            inside = np.ones(S.size - 1, bool)
            if name != "frequency_counts_across_segments":
                ends = np.cumsum(np.asarray(seg_len, dtype=np.int64))
                inside[ends[(ends > 0) & (ends < S.size)] - 1] = False
            keys = (S[:-1].astype(np.uint32) << 8 | S[1:])[inside]
            if keys.size == 0:
                return O.Dictionary(eb, el)
            uniq, first, count = np.unique(keys, return_index=True, return_counts=True)
            tie = uniq if name == "frequency_ties_by_value" else first
            order = np.lexsort((tie, -count.astype(np.int64)))[:room]
            pairs = np.zeros((order.size, O.LCAP), np.uint8)
            pairs[:, 0], pairs[:, 1] = uniq[order] >> 8, uniq[order] & 0xFF
            return O.Dictionary(np.concatenate([eb, pairs]), np.concatenate([el, np.full(order.size, 2, np.uint8)]))
        O.frequency_dictionary = frequency_dictionary

    # ---- the C part: LZW and the matrix-vector product
    elif name == "lzw_match_crosses_segment_end":
        _edited_c_library(O, "while (m < lmax && i + m < ge) {", "while (m < lmax && i + m < n) {")
    elif name == "lzw_match_stops_at_two_bytes":
        _edited_c_library(O, "while (m < lmax && i + m < ge) {", "while (m < lmax && m < 2 && i + m < ge) {")
    elif name == "lzw_new_entry_repeats_first_byte":
        _edited_c_library(O, "ent_bytes[(size_t)ne * TQO_LCAP + m] = S[i + m];", "ent_bytes[(size_t)ne * TQO_LCAP + m] = S[i];")
    elif name == "lzw_restarts_when_full":
        _edited_c_library(O, "      i += m;\n",
                          "      i += m;\n      if (n_entries == max_entries && n_init == 0) {\n"
                          "        n_entries = 256;\n"
                          "        for (size_t z = 0; z < (size_t)max_entries * 256; ++z) child[z] = -1;\n      }\n")
    elif name == "decode_ignores_codes_after_padding":
        _edited_c_library(O, "if (seen_pad || e >= n_entries) return -(g + 1);", "if (e >= n_entries) return -(g + 1);")
    elif name == "gemv_scale_dropped":
        _edited_c_library(O, "y[b * R + r] = (double)s[r] * acc;", "y[b * R + r] = acc;")
    elif name == "gemv_weights_read_transposed":
        _edited_c_library(O, "(double)Q[r * K + j] * (double)x[b * K + j]", "(double)Q[j * R + r] * (double)x[b * K + j]")
    elif name == "gemv_weights_read_unsigned":
        _edited_c_library(O, "(double)Q[r * K + j] * (double)x[b * K + j]", "(double)(uint8_t)Q[r * K + j] * (double)x[b * K + j]")
    elif name == "gemv_activations_read_transposed":
        _edited_c_library(O, "(double)Q[r * K + j] * (double)x[b * K + j]", "(double)Q[r * K + j] * (double)x[j * B + b]")
    elif name == "lzw_unit_budget_ignored":
        _edited_c_library(O, "(unit_budget <= 0 || units + cost <= unit_budget)) {", "1) {")
    elif name == "lzw_long_entries_cost_one_unit":
        _edited_c_library(O, "int cost = m + 1 <= 2 ? 1 : 2;", "int cost = 1;")
    elif name in ("sorted_codes_not_renumbered", "sorted_order_not_stable"):
        def sort_code_space(codes, d):
            kind = "stable" if name == "sorted_codes_not_renumbered" else None
            key = d.ent_len if kind else d.ent_len.astype(np.int64) * 100000 - np.arange(d.ent_len.size)   # equal lengths reversed
            order = np.argsort(key, kind="stable")
            new_of_old = np.empty(order.size, np.int64)
            new_of_old[order] = np.arange(order.size)
            sorted_len = d.ent_len[order]
            class_end = np.array([int((sorted_len <= k + 1).sum()) for k in range(4)], np.uint32)
            out = codes if name == "sorted_codes_not_renumbered" else new_of_old[codes].astype(np.uint16)
            return out, O.Dictionary(d.ent_bytes[order].copy(), sorted_len.copy()), class_end
        O.sort_code_space = sort_code_space
    elif name == "dictionary_words_high_byte_first":
        def dict_slots(d):
            eb = d.ent_bytes.astype(np.uint32)
            w = eb[:, 3] | (eb[:, 2] << 8) | (eb[:, 1] << 16) | (eb[:, 0] << 24)
            return np.concatenate([w, np.zeros(1, np.uint32)]).astype(np.uint32)
        O.dict_slots = dict_slots
    elif name == "lzw_carried_dictionary_ignored":
        _edited_c_library(O, "for (int e = 256; e < n_init; ++e) {", "for (int e = 256; e < n_init && e < 256; ++e) {")
    elif name == "gemv_output_transposed":
        _edited_c_library(O, "y[b * R + r] = (double)s[r] * acc;", "y[r * B + b] = (double)s[r] * acc;")
    elif name == "gate_up_sigmoid_sign":
        O.gate_up_f64 = lambda Qg, sg, Qu, su, x: (lambda g, u: g / (1.0 + np.exp(g)) * u)(O.gemv_f64(Qg, sg, x), O.gemv_f64(Qu, su, x))
    elif name == "gate_up_operands_swapped":
        O.gate_up_f64 = lambda Qg, sg, Qu, su, x: (lambda g, u: u / (1.0 + np.exp(-u)) * g)(O.gemv_f64(Qg, sg, x), O.gemv_f64(Qu, su, x))

    # ---- the stream format of the section 4 listings
    elif name == "listing_table_counts_stride_four":
        def _keys(values):
            v = np.ascontiguousarray(values, dtype=np.uint8).astype(np.uint32)
            n = v.size // 4
            g = v[: 4 * n].reshape(n, 4)
            return g[:, 0] | g[:, 1] << 8 | g[:, 2] << 16 | g[:, 3] << 24
        L._keys = _keys
    elif name == "listing_table_ties_by_value":
        def build_table(params, top_k=L.MAX_TOP_K):
            keys = np.concatenate([L._keys(p) for p in params]) if len(params) else np.zeros(0, np.uint32)
            if keys.size == 0 or top_k == 0:
                return np.zeros((0, 4), np.uint8)
            uniq, count = np.unique(keys, return_counts=True)
            chosen = uniq[np.lexsort((uniq, -count.astype(np.int64)))[:top_k]]
            return np.stack([(chosen >> (8 * k)) & 0xFF for k in range(4)], axis=1).astype(np.uint8)
        L.build_table = build_table
    elif name == "listing_codewords_from_zero":
        real_compress, real_decompress = L.compress, L.decompress

        def compress(values, table):
            w = real_compress(values, table).astype(np.int64)
            out, i = [], 0
            while i < w.size:                      # shift every codeword down by one, leave markers and raw values
                if w[i] == L.MARKER:
                    out.extend(w[i: i + 5])
                    i += 5
                else:
                    out.append(w[i] - 1)
                    i += 1
            return np.array(out, dtype=np.uint16)

        def decompress(words, table):
            w = np.ascontiguousarray(words, dtype=np.uint16).astype(np.int64)
            out, i = [], 0
            while i < w.size:
                if w[i] == L.MARKER:
                    out.extend(w[i: i + 5])
                    i += 5
                else:
                    out.append(w[i] + 1)
                    i += 1
            return real_decompress(np.array(out, dtype=np.uint16), table)
        L.compress, L.decompress = compress, decompress   # consistent with each other, not with the listings
    elif name == "listing_tail_dropped":
        real_compress = L.compress
        L.compress = lambda values, table: real_compress(np.asarray(values)[: np.asarray(values).size // 4 * 4], table)
    else:
        raise ValueError(f"unknown planted mistake {name!r}")


def pytest_configure(config):
    name = os.environ.get("TQ_PLANTED_MISTAKE")
    if name:
        _plant(name)
