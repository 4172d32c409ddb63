"""The oracle's pins must fail when the oracle is wrong.

Each case plants one plausible mistake in the CPU oracle (a dropped term, a wrong sign or index, a transposed operand,
a tie broken the other way: see planted_mistakes.py) and runs the pin tests of the part concerned in a child process.
The child must FAIL; with nothing planted it must pass.  Nothing here touches the GPU or the product library.
"""
import os
import subprocess
import sys

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)

QUANT = "test_oracle_quantize.py"
CODEC = "test_oracle_codec.py"
GEMV = "test_oracle_gemv_container.py"
LISTING = "test_listing_format.py"

MISTAKES = [
    ("quantize_rounds_half_up", QUANT),
    ("quantize_truncates", QUANT),
    ("quantize_divides_by_two_to_the_bits_minus_one", QUANT),
    ("quantize_one_scale_for_the_matrix", QUANT),
    ("segments_lane_bits_swapped", GEMV),
    ("segments_quad_major", GEMV),
    ("bytes_offset_binary", GEMV),
    ("chunk_layout_lane_minor", CODEC),
    ("nibbles_high_first", GEMV),
    ("nibbles_not_sign_extended", GEMV),
    ("frequency_ties_by_value", CODEC),
    ("frequency_counts_across_segments", CODEC),
    ("lzw_match_crosses_segment_end", CODEC),
    ("lzw_match_stops_at_two_bytes", CODEC),
    ("lzw_new_entry_repeats_first_byte", CODEC),
    ("lzw_restarts_when_full", CODEC),
    ("lzw_carried_dictionary_ignored", CODEC),
    ("lzw_unit_budget_ignored", CODEC),
    ("lzw_long_entries_cost_one_unit", CODEC),
    ("sorted_codes_not_renumbered", CODEC),
    ("sorted_order_not_stable", CODEC),
    ("dictionary_words_high_byte_first", GEMV),
    ("decode_ignores_codes_after_padding", CODEC),
    ("gemv_scale_dropped", GEMV),
    ("gemv_weights_read_transposed", GEMV),
    ("gemv_weights_read_unsigned", GEMV),
    ("gemv_output_transposed", GEMV),
    ("gemv_activations_read_transposed", GEMV),
    ("gate_up_sigmoid_sign", GEMV),
    ("gate_up_operands_swapped", GEMV),
    ("listing_table_counts_stride_four", LISTING),
    ("listing_table_ties_by_value", LISTING),
    ("listing_codewords_from_zero", LISTING),
    ("listing_tail_dropped", LISTING),
]


def run_pins(test_file: str, mistake: "str | None"):
    env = dict(os.environ)
    env["PYTHONPATH"] = os.pathsep.join([HERE, ROOT, env.get("PYTHONPATH", "")])
    env.pop("TQ_PLANTED_MISTAKE", None)
    if mistake:
        env["TQ_PLANTED_MISTAKE"] = mistake
    cmd = [sys.executable, "-m", "pytest", os.path.join(HERE, test_file), "-q", "-x", "-m", "not gpu", "--no-header",
           "-p", "no:cacheprovider", "-p", "planted_mistakes"]
    return subprocess.run(cmd, cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=600)


@pytest.mark.parametrize("test_file", [QUANT, CODEC, GEMV, LISTING])
def test_pins_pass_with_nothing_planted(test_file):
    r = run_pins(test_file, None)
    assert r.returncode == 0, r.stdout[-3000:]


@pytest.mark.parametrize("mistake,test_file", MISTAKES, ids=[m for m, _ in MISTAKES])
def test_planted_mistake_is_caught(mistake, test_file):
    r = run_pins(test_file, mistake)
    # 1 = some test failed.  Anything else (0: all passed; 2..5: interrupted, internal or usage error, nothing collected)
    # means the pins did not do their job or the mistake was not planted.
    assert r.returncode == 1, f"planted mistake {mistake!r} was not caught by {test_file} (exit {r.returncode}):\n{r.stdout[-3000:]}"
    assert " failed" in r.stdout and "planted_" not in r.stdout.split("short test summary")[-1], r.stdout[-3000:]
