"""GPU parity at the FULL shapes of the large configurations -- every layer, the real prefix lengths (the KV-cache
tails the configurations use) and the real vocabularies -- against the pure fp64 oracle:

  * GPT-2-XL-shaped target, 48 layers, prefix 512, gamma 32 and 16, with the 12-layer drafter at 544 rows;
  * the batched configuration: 16 sequences with prefixes drawn from U[128, 768] (the workload's own lengths), the
    whole batch on the GPU, three of its sequences (shortest, median, longest) through the oracle;
  * Llama-3-8B-shaped target, 32 layers, vocabulary 128256, prefix 1024, gamma 32, and its drafter at 1056 rows,
    plus one whole round replayed by the oracle's Algorithm 1 on the GPU's logits.

The bf16 bound comes from the storage model on the same inputs (tests/helpers.py); measured maxima, rms errors and the
model's sigma are written to fulldepth_errors.json in the folder that SD_TEST_OUT names, when it is set.  These tests take minutes of
host time (fp64 forwards of 1.5 and 8 billion parameters); they print a progress line per phase.
"""
import json
import os
import time

import numpy as np
import pytest

from oracle import transformer as otf
from paper_2408_05636_amd import synth
from tests import bf16_model as bm
from tests.helpers import assert_logits_close

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(1500)]
torch = pytest.importorskip("torch")

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
_T0 = time.perf_counter()


class Progress:
    """Progress lines past pytest's capture (a quiet minute-long test looks hung from outside) and a record of the
    measured errors."""
    def __init__(self, capsys, test):
        self.capsys, self.test = capsys, test

    def __call__(self, msg):
        line = f"[fulldepth {time.perf_counter() - _T0:7.1f}s] {self.test}: {msg}"
        with self.capsys.disabled():
            print(line, flush=True)
        d = os.environ.get("SD_TEST_OUT", "")
        if d and os.path.isdir(d):
            with open(os.path.join(d, "fulldepth_progress.log"), "a") as f:
                f.write(line + "\n")

    def record(self, stats):
        self(f"{stats['what']}: logit rms {stats['logit_rms']:.3f}, max err {stats['max_err']:.4f}, rms err {stats['rms_err']:.5f}, "
             f"storage-model sigma {stats['sigma_model']:.5f}, bound {stats['tol']:.4f}")
        d = os.environ.get("SD_TEST_OUT", "")
        if d and os.path.isdir(d):
            path = os.path.join(d, "fulldepth_errors.json")
            all_ = json.load(open(path)) if os.path.exists(path) else {}
            all_[f"{self.test}/{stats['what']}"] = stats
            json.dump(all_, open(path, "w"), indent=1)


@pytest.fixture
def progress(capsys, request):
    return Progress(capsys, request.node.name)


def build(progress, name, max_batch, gamma_max, seed=1):
    from paper_2408_05636_amd import binding
    w = synth.workload(name)
    t, d = w["target"], w["drafter"]
    Wt, Wd = synth.gen_weights(t, seed, threads=16), synth.gen_weights(d, seed + 1, threads=16)
    progress(f"weights generated ({t.n_layer} + {d.n_layer} layers)")
    sd = binding.SpecDiff(t, d, Wt, Wd, max_batch=max_batch, gamma_max=gamma_max)
    progress("uploaded")
    return sd, w, t, d, Wt, Wd


def check(progress, got, ref_fn, model_fn, what, dtype="bf16"):
    ref = ref_fn()
    progress(f"{what}: oracle forward done")
    model = model_fn()
    progress(f"{what}: storage model done")
    stats = {}
    try:
        assert_logits_close(got, ref, dtype, what, model, stats)
    finally:
        if stats:
            progress.record(stats)


def masked_block(rng, V, gamma, frac):
    blk = rng.integers(0, V, gamma)
    blk[rng.random(gamma) < frac] = V
    return blk


def test_gpt2xl_48_layers_prefix_512(progress):
    sd, w, t, d, Wt, Wd = build(progress, "gpt2xl", 1, 32)
    V, L = t.vocab, 512
    rng = np.random.default_rng(101)
    prefix = synth.gen_prefix(V, L, 11)
    draft = rng.integers(0, V, (1, 32)).astype(np.int32)
    sd.sd_prefill([prefix])
    got32 = sd.sd_target_logits([prefix], draft).cpu().numpy()[:, :V].copy()
    got16 = sd.sd_target_logits([prefix], draft[:, :16]).cpu().numpy()[:, :V].copy()
    progress("GPU target passes done (gamma 32 and 16)")
    toks, rows = np.concatenate([prefix, draft[0]]), np.arange(L - 1, L + 32)
    ref = otf.logits_at(Wt, t, toks, rows)
    progress("oracle target forward done")
    model = bm.logits_at(Wt, t, toks, rows)
    progress("storage model done")
    for got, g in ((got32, 32), (got16, 16)):           # causal: the first 17 rows do not see draft[16:]
        stats = {}
        try:
            assert_logits_close(got, ref[:g + 1], "bf16", f"target gamma {g}", model[:g + 1], stats)
        finally:
            progress.record(stats)
    # the drafter of this configuration at its real row count (prefix 512 + 32 slots), a late and an early step
    for j, T in ((8, 8), (2, 8)):
        seq = np.concatenate([prefix, masked_block(rng, V, 32, j / T)]).astype(np.int32)
        got = sd.sd_drafter_logits([seq], 32, j, T).cpu().numpy()[:, :V].copy()
        r = np.arange(L, L + 32)
        check(progress, got, lambda: otf.logits_at(Wd, d, seq, r, j / T), lambda: bm.logits_at(Wd, d, seq, r, j / T), f"drafter step {j}/{T}")
    sd.close()


def test_gpt2xl_batch_16_prefixes_128_to_768(progress):
    sd, w, t, d, Wt, Wd = build(progress, "gpt2xl_b16", 16, 16)
    V, gamma = t.vocab, 16
    lens = [int(x) for x in synth.gen_prefix_lengths(16, 128, 768, 3)]
    assert min(lens) >= 128 and max(lens) <= 768
    prefixes = [synth.gen_prefix(V, L, 4 + i) for i, L in enumerate(lens)]
    rng = np.random.default_rng(102)
    draft = rng.integers(0, V, (16, gamma)).astype(np.int32)
    sd.sd_prefill(prefixes)
    got_t = sd.sd_target_logits(prefixes, draft).cpu().numpy()[:, :V].copy()
    seqs = [np.concatenate([p, masked_block(rng, V, gamma, 0.5)]).astype(np.int32) for p in prefixes]
    got_d = sd.sd_drafter_logits(seqs, gamma, 2, 4).cpu().numpy()[:, :V].copy()
    progress(f"GPU batch passes done, prefix lengths {lens}")
    order = np.argsort(lens)
    for b in (int(order[0]), int(order[8]), int(order[-1])):
        L = lens[b]
        toks, rows = np.concatenate([prefixes[b], draft[b]]), np.arange(L - 1, L + gamma)
        check(progress, got_t[b * (gamma + 1):(b + 1) * (gamma + 1)], lambda: otf.logits_at(Wt, t, toks, rows),
              lambda: bm.logits_at(Wt, t, toks, rows), f"target seq {b} (prefix {L})")
        r = np.arange(L, L + gamma)
        check(progress, got_d[b * gamma:(b + 1) * gamma], lambda: otf.logits_at(Wd, d, seqs[b], r, 0.5),
              lambda: bm.logits_at(Wd, d, seqs[b], r, 0.5), f"drafter seq {b} (prefix {L})")
    sd.close()


def test_llama8b_32_layers_vocab_128256_prefix_1024(progress):
    from tests.test_gpu_round import check_rounds
    sd, w, t, d, Wt, Wd = build(progress, "llama8b", 1, 32)
    V, L, gamma = t.vocab, 1024, 32
    assert V == 128256 and t.n_layer == 32
    rng = np.random.default_rng(103)
    prefix = synth.gen_prefix(V, L, 12)
    draft = rng.integers(0, V, (1, gamma)).astype(np.int32)
    sd.sd_prefill([prefix])
    progress("prefill done")
    got = sd.sd_target_logits([prefix], draft).cpu().numpy()[:, :V].copy()
    seq = np.concatenate([prefix, masked_block(rng, V, gamma, 0.5)]).astype(np.int32)
    got_d = sd.sd_drafter_logits([seq], gamma, 4, 8).cpu().numpy()[:, :V].copy()
    progress("GPU passes done")
    # one whole round at full size: the oracle's Algorithm 1 on the GPU's own logits must reproduce draft, q, n and token
    check_rounds(sd, [prefix], gamma, 4, seeds=[5])
    progress("round replayed by the oracle on the GPU's logits")
    sd.close()
    r = np.arange(L, L + gamma)
    check(progress, got_d, lambda: otf.logits_at(Wd, d, seq, r, 0.5), lambda: bm.logits_at(Wd, d, seq, r, 0.5), "drafter step 4/8 (1056 rows)")
    del Wd
    toks, rows = np.concatenate([prefix, draft[0]]), np.arange(L - 1, L + gamma)
    check(progress, got, lambda: otf.logits_at(Wt, t, toks, rows), lambda: bm.logits_at(Wt, t, toks, rows), "target 32 layers")
