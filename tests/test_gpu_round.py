"""GPU parity of whole rounds (sd_draft, sd_verify, sd_round) against the oracle's Algorithm 1.

Two comparisons per workload:
 (a) the oracle's algorithm fed with the GPU's own forward passes (sd_drafter_logits /
     sd_target_logits) must reproduce the GPU round exactly -- tokens, q, accepted count,
     correction token; the forwards themselves are compared in test_gpu_forward.py;
 (b) for the fp32 workload, the oracle running entirely on its own fp64 forwards must agree
     wherever its decision margins exceed the logit tolerance.
"""
import numpy as np
import pytest

from oracle import specdiff as osd
from oracle import transformer as otf
from oracle.transformer import softmax_rows
from paper_2408_05636_amd import synth
from tests.helpers import MARGIN_EXACT, oracle_drafter_fn, oracle_target_fn

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def make(workload, seed, shrink_t=None, shrink_d=None, max_batch=1, gamma_max=16):
    from paper_2408_05636_amd import binding
    w = synth.workload(workload)
    t = synth.shrink(w["target"], **(shrink_t or {}))
    d = synth.shrink(w["drafter"], **(shrink_d or {}))
    Wt, Wd = synth.gen_weights(t, seed), synth.gen_weights(d, seed + 1)
    return binding.SpecDiff(t, d, Wt, Wd, max_batch=max_batch, gamma_max=gamma_max), t, d, Wt, Wd


def replay_with_gpu_forwards(sd, prefixes, gamma, T, seed):
    """Oracle algorithm, GPU forwards.  Returns per sequence (z, q, n, tok, margins)."""
    V = sd.target.vocab
    out = []
    for b, p in enumerate(prefixes):
        def dl(tokens, t, b=b):
            # the library evaluates the whole batch; rebuild the batch with this sequence's block
            seqs = [np.concatenate([pp, np.full(gamma, V)]).astype(np.int32) for pp in prefixes]
            seqs[b] = tokens.astype(np.int32)
            lg = sd.sd_drafter_logits(seqs, gamma, int(round(t * T)), T).cpu().numpy()
            return lg[b * gamma:(b + 1) * gamma, :V]
        z, q, dm, nf = osd.oracle_draft(dl, p, gamma, T, seed, V, batch=b)
        out.append([z, q, dm])
    draft = np.stack([o[0] for o in out]).astype(np.int32)
    lt = sd.sd_target_logits(prefixes, draft).cpu().numpy()
    for b, p in enumerate(prefixes):
        P = softmax_rows(lt[b * (gamma + 1):(b + 1) * (gamma + 1), :V].astype(np.float64))
        r, u = osd.verify_uniforms(seed, b, gamma)
        n, tok, vm, fb = osd.verify_with_uniforms(P, out[b][1], out[b][0], r, u)
        am = osd.accept_margins(P, out[b][1], out[b][0], r)
        out[b] += [n, tok, vm, am]
    return out


def check_rounds(sd, prefixes, gamma, T, seeds):
    V = sd.target.vocab
    B = len(prefixes)
    for seed in seeds:
        draft, qtok, q_dev = sd.sd_draft(prefixes, gamma, T, seed)
        q_gpu = q_dev.cpu().numpy().copy()
        n_v, tok_v = sd.sd_verify(prefixes, draft, q_dev, seed)
        draft_r, n_r, tok_r = sd.sd_round(prefixes, gamma, T, seed)
        assert np.array_equal(draft, draft_r) and np.array_equal(n_v, n_r) and np.array_equal(tok_v, tok_r)
        assert ((draft >= 0) & (draft < V)).all() and ((n_v >= 0) & (n_v <= gamma)).all() and ((tok_v >= 0) & (tok_v < V)).all()
        ref = replay_with_gpu_forwards(sd, prefixes, gamma, T, seed)
        for b in range(B):
            z, q, dm, n, tok, vm, am = ref[b]
            if not np.array_equal(draft[b], z):
                # a sampling decision on a CDF edge: everything downstream legitimately differs
                k = int(np.flatnonzero(draft[b] != z)[0])
                assert dm[k] < MARGIN_EXACT, (seed, b, k, dm[k])
                continue
            qg = q_gpu[b * gamma:(b + 1) * gamma, :V]
            np.testing.assert_allclose(qg, q, rtol=2.5e-7, atol=0)
            np.testing.assert_array_equal(qtok[b], qg[np.arange(gamma), z])
            # the verify replay used the oracle's q; the GPU used its own (<= 1 ulp apart)
            if n_v[b] != n:
                assert am[min(n, n_v[b])] < 1e-6, (seed, b, n, n_v[b], am)
                continue
            assert tok_v[b] == tok or vm < 1e-7, (seed, b, tok, tok_v[b], vm)


def test_tiny_fp32_64_rounds():
    sd, t, d, Wt, Wd = make("tiny", seed=1, gamma_max=8)
    prefix = synth.gen_prefix(t.vocab, 32, 2)
    check_rounds(sd, [prefix], 8, 4, seeds=[1000 + i for i in range(64)])
    sd.close()


def test_tiny_fp32_rounds_against_pure_oracle():
    """(b): oracle on its own fp64 forwards.  A mismatch is allowed only at a decision whose
    margin is within reach of the 1e-4 logit tolerance; after one, the round is not compared further."""
    sd, t, d, Wt, Wd = make("tiny", seed=1, gamma_max=8)
    prefix = synth.gen_prefix(t.vocab, 32, 2)
    gamma, T, tau = 8, 4, 1e-5
    exact = weak = 0
    accepted = []
    for i in range(64):
        seed = 1000 + i
        draft, n_g, tok_g = sd.sd_round([prefix], gamma, T, seed)
        z, q, dm, nf = osd.oracle_draft(oracle_drafter_fn(Wd, d, gamma), prefix, gamma, T, seed, t.vocab)
        assert nf <= T
        if not np.array_equal(draft[0], z):
            k = int(np.flatnonzero(draft[0] != z)[0])
            assert dm[k] < tau, (seed, k, dm[k])
            weak += 1
            continue
        n, tok, vm, fb = osd.oracle_verify(oracle_target_fn(Wt, t), prefix, z, q, seed)
        assert not fb
        if n != n_g[0]:
            # only an acceptance test sitting on its threshold (within reach of the logit tolerance) may differ
            rows = np.arange(len(prefix) - 1, len(prefix) + gamma)
            P = softmax_rows(oracle_target_fn(Wt, t)(np.concatenate([prefix, z]), rows))
            r, _ = osd.verify_uniforms(seed, 0, gamma)
            am = osd.accept_margins(P, q, z, r)
            assert am[min(n, int(n_g[0]))] < 1e-3, (seed, n, n_g[0], am)
            weak += 1
            continue
        if tok != tok_g[0]:
            assert vm < tau, (seed, n, tok, tok_g[0], vm)
            weak += 1
            continue
        exact += 1
        accepted.append(n)
    assert exact >= 60 and weak <= 4
    assert 0 <= min(accepted) and max(accepted) <= gamma


def test_tiny_fp32_ragged_batch_rounds():
    sd, t, d, Wt, Wd = make("tiny", seed=3, max_batch=3, gamma_max=8)
    prefixes = [synth.gen_prefix(t.vocab, L, 20 + L) for L in (9, 40, 1)]
    check_rounds(sd, prefixes, 5, 3, seeds=[7, 8, 9])
    check_rounds(sd, prefixes[:2], 8, 1, seeds=[10])          # T = 1: everything revealed in one step
    sd.close()


def test_bf16_small_rounds():
    sd, t, d, Wt, Wd = make("gpt2s", seed=4, shrink_t=dict(n_layer=2, vocab=5003, n_ctx=128),
                            shrink_d=dict(n_layer=2, vocab=5003, n_ctx=128), max_batch=2, gamma_max=16)
    prefixes = [synth.gen_prefix(t.vocab, L, 30 + L) for L in (50, 21)]
    check_rounds(sd, prefixes, 16, 8, seeds=[1, 2, 3])
    sd.close()


def test_llama_target_rounds():
    w = synth.workload("llama8b")
    from paper_2408_05636_amd import binding
    t = synth.shrink(w["target"], n_layer=2, d_model=512, n_head=4, n_kv_head=2, d_ff=1408, vocab=2000, n_ctx=128)
    d = synth.shrink(w["drafter"], n_layer=1, d_model=256, n_head=4, n_kv_head=4, d_ff=512, vocab=2000, n_ctx=128)
    sd = binding.SpecDiff(t, d, synth.gen_weights(t, 8), synth.gen_weights(d, 9), max_batch=2, gamma_max=8)
    prefixes = [synth.gen_prefix(t.vocab, L, 40 + L) for L in (30, 12)]
    check_rounds(sd, prefixes, 8, 2, seeds=[5, 6])
    sd.close()


def test_gpt2_small_full_size_round():
    sd, t, d, Wt, Wd = make("gpt2s", seed=6, gamma_max=16)
    prefix = synth.gen_prefix(t.vocab, 256, 7)
    check_rounds(sd, [prefix], 16, 8, seeds=[11])
    sd.close()


def test_argument_errors_are_reported():
    from paper_2408_05636_amd import binding
    sd, t, d, Wt, Wd = make("tiny", seed=1, gamma_max=8)
    prefix = synth.gen_prefix(t.vocab, 32, 2)
    for bad_call, code in [
        (lambda: sd.sd_round([prefix], 9, 4, 1), 2),                       # gamma > gamma_max
        (lambda: sd.sd_round([prefix], 8, 0, 1), 2),                       # T < 1
        (lambda: sd.sd_round([prefix, prefix], 8, 4, 1), 2),               # batch > max_batch
        (lambda: sd.sd_round([np.array([t.vocab], dtype=np.int32)], 8, 4, 1), 3),   # token id out of range
        (lambda: sd.sd_round([synth.gen_prefix(t.vocab, 1020, 1)], 8, 4, 1), 2),    # prefix + gamma > n_ctx
    ]:
        with pytest.raises(binding.SdError) as e:
            bad_call()
        assert e.value.code == code
    draft, n, tok = sd.sd_round([prefix], 8, 4, 1)                         # the handle still works
    assert draft.shape == (1, 8)
    sd.close()


def test_graph_replay_equals_eager_launches():
    """Captured launch sequences are replayed with new seeds and new prefixes of the same shape;
    every replay must equal the eager result, with eager work and synchronisations in between."""
    sd, t, d, Wt, Wd = make("gpt2s", seed=4, shrink_t=dict(n_layer=2, vocab=5003, n_ctx=128),
                            shrink_d=dict(n_layer=2, vocab=5003, n_ctx=128), max_batch=2, gamma_max=16)
    for trial in range(3):
        prefixes = [synth.gen_prefix(t.vocab, L, 100 * trial + L) for L in (50, 21)]
        for seed in (1, 2, 3):
            sd.sd_set_graph_replay(True)
            a = sd.sd_round(prefixes, 16, 8, seed)
            d1, qt1, q1 = sd.sd_draft(prefixes, 16, 8, seed)
            n1, t1 = sd.sd_verify(prefixes, d1, q1, seed)
            sd.sd_set_graph_replay(False)
            b = sd.sd_round(prefixes, 16, 8, seed)
            d2, qt2, q2 = sd.sd_draft(prefixes, 16, 8, seed)
            n2, t2 = sd.sd_verify(prefixes, d2, q2, seed)
            for x, y in zip(a, b):
                assert np.array_equal(x, y), (trial, seed)
            assert np.array_equal(d1, d2) and np.array_equal(qt1, qt2) and np.array_equal(n1, n2) and np.array_equal(t1, t2)
            assert np.array_equal(a[0], d1) and np.array_equal(a[1], n1) and np.array_equal(a[2], t1)
    sd.close()
