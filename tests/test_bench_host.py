"""Host-side checks of the benchmark's own arithmetic (no GPU): the round roofline that every fraction in the report is
taken against must reproduce the figures derived for the five workloads when they were defined -- weights once per
forward, the target's KV cache once, fp32 logits written once, at 8 TB/s and 2.5 PFLOP/s (bf16)."""
import pytest

import bench
from paper_2408_05636_amd import synth

# (workload, target pass us, drafter step us, round us) as derived with the workload definitions
EXPECTED = [
    ("gpt2s", 32.5, 31.3, 283.0),
    ("gpt2xl", 408.8, 40.5, 733.0),
    ("llama8b", 1895.0, 90.7, 2621.0),
    ("llama8b_b8", 2027.0, 726.0, 7833.0),
]


@pytest.mark.parametrize("name,target_us,drafter_us,round_us", EXPECTED)
def test_round_roofline_matches_the_derived_figures(name, target_us, drafter_us, round_us):
    w = synth.workload(name)
    lens = [w["prefix_len"]] * w["batch"]
    us, parts = bench.round_roofline(w, lens)
    assert parts["target_us"] == pytest.approx(target_us, rel=2e-3)
    assert parts["drafter_step_us"] == pytest.approx(drafter_us, rel=5e-3)
    assert us == pytest.approx(round_us, rel=2e-3)
    assert us == pytest.approx(w["T"] * parts["drafter_step_us"] + parts["target_us"], rel=1e-12)


def test_round_roofline_bounds():
    """Few rows against large weights are bound by HBM; a thousand drafter rows against 85 M parameters by the matrix
    cores; the fp32 workload is priced at the fp32 peak."""
    _, p = bench.round_roofline(synth.workload("llama8b"), [1024])
    assert p["target_bound"] == "hbm" and p["drafter_bound"] == "mfma"
    _, p = bench.round_roofline(synth.workload("gpt2s"), [256])
    assert p["target_bound"] == "hbm" and p["drafter_bound"] == "hbm"
    us, _ = bench.round_roofline(synth.workload("tiny"), [32])
    assert 0.5 < us < 5.0


def test_ragged_batch_roofline_counts_every_sequence():
    w = synth.workload("gpt2xl_b16")
    lens = [int(x) for x in synth.gen_prefix_lengths(w["batch"], w["prefix_len"][0], w["prefix_len"][1], 3)]
    us, _ = bench.round_roofline(w, lens)
    us_short, _ = bench.round_roofline(w, [min(lens)] * len(lens))
    us_long, _ = bench.round_roofline(w, [max(lens)] * len(lens))
    assert us_short < us < us_long
