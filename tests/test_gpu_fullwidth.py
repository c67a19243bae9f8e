"""GPU parity at the real layer widths of the large configurations, with the depth cut to one or two layers so
that the fp64 oracle stays fast: GPT-2-XL width (d = 1600, 25 heads, MLP 6400) and Llama-3-8B width (d = 4096,
32 query / 8 KV heads of 128, SwiGLU 14336, RoPE, RMSNorm).  These shapes select kernel paths that the small
test models never reach: K split over workgroups, the 64-row few-row tile (gamma + 1 = 33 rows), the
workgroup-shared tiles on 272-row target batches, 128-wide attention heads, grouped-query attention."""
import numpy as np
import pytest

from paper_2408_05636_amd import synth
from tests.test_gpu_forward import check_forwards
from tests.test_gpu_round import check_rounds

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def xl_pair():
    w = synth.workload("gpt2xl")
    return synth.shrink(w["target"], n_layer=2, n_ctx=256), synth.shrink(w["drafter"], n_layer=2, n_ctx=256)


def llama_pair():
    w = synth.workload("llama8b")
    return (synth.shrink(w["target"], n_layer=1, n_ctx=256, vocab=32064),
            synth.shrink(w["drafter"], n_layer=1, n_ctx=256, vocab=32064))


def test_xl_width_forwards_single_and_batched():
    t, d = xl_pair()
    check_forwards(t, d, [200], 16, 8, seed=31, steps=[8, 3])                       # 17 query rows: few-row kernels, K split
    lens = [int(x) for x in synth.gen_prefix_lengths(16, 20, 90, 5)]
    check_forwards(t, d, lens, 16, 4, seed=32, steps=[2])                           # 272 query rows: shared 64-row tiles


def test_xl_width_round():
    from paper_2408_05636_amd import binding
    t, d = xl_pair()
    Wt, Wd = synth.gen_weights(t, 41), synth.gen_weights(d, 42)
    sd = binding.SpecDiff(t, d, Wt, Wd, max_batch=2, gamma_max=16)
    prefixes = [synth.gen_prefix(t.vocab, L, 50 + L) for L in (120, 77)]
    check_rounds(sd, prefixes, 16, 4, seeds=[1, 2])
    sd.close()


def test_llama_width_forwards_and_round():
    from paper_2408_05636_amd import binding
    t, d = llama_pair()
    check_forwards(t, d, [96], 32, 8, seed=33, steps=[8, 1])                        # 33 query rows
    check_forwards(t, d, [40, 96, 63, 71, 88, 52, 90, 35], 32, 4, seed=34, steps=[2])   # 264 query rows
    Wt, Wd = synth.gen_weights(t, 43), synth.gen_weights(d, 44)
    sd = binding.SpecDiff(t, d, Wt, Wd, max_batch=1, gamma_max=32)
    check_rounds(sd, [synth.gen_prefix(t.vocab, 100, 9)], 32, 4, seeds=[3])
    sd.close()
