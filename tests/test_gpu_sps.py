"""GPU parity of standard speculative decoding (the paper's SpS baseline: an autoregressive drafter producing the gamma
draft tokens one after the other) and of the sequence-initialisation hybrid, against the oracle:

 (a) the drafter's forward (sd_sps_logits, with its incremental KV cache) against the fp64 oracle;
 (b) the oracle's algorithm fed with the GPU's own logits reproduces sd_sps_draft / sd_verify / sd_sps_round exactly;
 (c) fp32: whole rounds against the pure oracle; a drafter that is the target gets everything accepted;
 (d) hybrid generation at temperature 0 emits the target's own greedy string and the oracle's accepted counts.
"""
import numpy as np
import pytest

from oracle import specdiff as osd
from oracle import transformer as otf
from oracle.transformer import softmax_rows
from paper_2408_05636_amd import synth
from tests import bf16_model as bm
from tests.helpers import MARGIN_EXACT, assert_logits_close

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def make(workload, seed, shrink_t=None, shrink_d=None, shrink_s=None, max_batch=1, gamma_max=8, sps_is_target=False):
    from paper_2408_05636_amd import binding
    w = synth.workload(workload)
    t = synth.shrink(w["target"], **(shrink_t or {}))
    d = synth.shrink(w["drafter"], **(shrink_d or {}))
    s = t if sps_is_target else synth.shrink(w["target"], **(shrink_s or {}))
    Wt, Wd = synth.gen_weights(t, seed), synth.gen_weights(d, seed + 1)
    Ws = Wt if sps_is_target else synth.gen_weights(s, seed + 2)
    sd = binding.SpecDiff(t, d, Wt, Wd, max_batch=max_batch, gamma_max=gamma_max)
    sd.sd_sps_attach(s, Ws)
    return sd, t, d, s, Wt, Wd, Ws


def test_sps_drafter_forward_and_incremental_cache():
    sd, t, d, s, Wt, Wd, Ws = make("tiny", 31, shrink_s=dict(n_layer=1), max_batch=3)
    V = t.vocab
    seqs = [synth.gen_prefix(V, L, 40 + L) for L in (33, 7, 1)]
    for step in range(4):                              # the same sequences growing: only new rows are computed
        got = sd.sd_sps_logits(seqs).cpu().numpy()[:, :V]
        for b, q in enumerate(seqs):
            ref = otf.logits_at(Ws, s, q, [len(q) - 1])
            assert_logits_close(got[b:b + 1], ref, "f32", f"step {step} seq {b}")
        seqs = [np.append(q, synth.gen_prefix(V, 1 + b, 90 + step)) for b, q in enumerate(seqs)]
    # a different string of the same length: the cache must notice and start over
    other = [synth.gen_prefix(V, len(q), 500 + b) for b, q in enumerate(seqs)]
    got = sd.sd_sps_logits(other).cpu().numpy()[:, :V]
    for b, q in enumerate(other):
        assert_logits_close(got[b:b + 1], otf.logits_at(Ws, s, q, [len(q) - 1]), "f32", f"other seq {b}")
    sd.close()


def test_sps_drafter_forward_bf16():
    sd, t, d, s, Wt, Wd, Ws = make("gpt2s", 33, shrink_t=dict(n_layer=2, vocab=3001, n_ctx=256), shrink_d=dict(n_layer=1, vocab=3001, n_ctx=256),
                                   shrink_s=dict(n_layer=2, d_model=256, n_head=4, n_kv_head=4, d_ff=1024, vocab=3001, n_ctx=256), max_batch=2)
    V = t.vocab
    seqs = [synth.gen_prefix(V, L, 60 + L) for L in (120, 45)]
    for step in range(2):
        got = sd.sd_sps_logits(seqs).cpu().numpy()[:, :V]
        for b, q in enumerate(seqs):
            rows = [len(q) - 1]
            assert_logits_close(got[b:b + 1], otf.logits_at(Ws, s, q, rows), "bf16", f"step {step} seq {b}", bm.logits_at(Ws, s, q, rows))
        seqs = [np.append(q, synth.gen_prefix(V, 2, 70 + step)) for q in seqs]
    sd.close()


def replay_with_gpu_logits(sd, prefixes, gamma, seed, greedy=False):
    V = sd.target.vocab
    out = []
    for b, p in enumerate(prefixes):
        def dl(tokens, rows, b=b):
            assert list(rows) == [len(tokens) - 1]
            seqs = [np.asarray(pp, dtype=np.int32) for pp in prefixes]
            seqs[b] = np.asarray(tokens, dtype=np.int32)
            return sd.sd_sps_logits(seqs).cpu().numpy()[b:b + 1, :V]
        z, q, dm, nf = osd.sps_draft_with_uniforms(dl, p, gamma, osd.sps_uniforms(seed, b, gamma), greedy)
        assert nf == gamma
        out.append([z, q, dm])
    draft = np.stack([o[0] for o in out]).astype(np.int32)
    lt = sd.sd_target_logits(prefixes, draft).cpu().numpy()
    for b in range(len(prefixes)):
        lg = lt[b * (gamma + 1):(b + 1) * (gamma + 1), :V].astype(np.float64)
        if greedy:
            n, tok, gaps = osd.verify_greedy(lg, out[b][0])
            out[b] += [n, tok, gaps, None]
        else:
            P = softmax_rows(lg)
            r, u = osd.verify_uniforms(seed, b, gamma)
            n, tok, vm, fb = osd.verify_with_uniforms(P, out[b][1], out[b][0], r, u)
            out[b] += [n, tok, vm, osd.accept_margins(P, out[b][1], out[b][0], r)]
    return out


def check_sps_rounds(sd, prefixes, gamma, seeds):
    V = sd.target.vocab
    for seed in seeds:
        draft, qtok, q_dev = sd.sd_sps_draft(prefixes, gamma, seed)
        q_gpu = q_dev.cpu().numpy().copy()
        n_v, tok_v = sd.sd_verify(prefixes, draft, q_dev, seed)
        draft_r, n_r, tok_r = sd.sd_sps_round(prefixes, gamma, seed)
        assert np.array_equal(draft, draft_r) and np.array_equal(n_v, n_r) and np.array_equal(tok_v, tok_r)
        assert ((draft >= 0) & (draft < V)).all() and ((n_v >= 0) & (n_v <= gamma)).all() and ((tok_v >= 0) & (tok_v < V)).all()
        ref = replay_with_gpu_logits(sd, prefixes, gamma, seed)
        for b in range(len(prefixes)):
            z, q, dm, n, tok, vm, am = ref[b]
            if not np.array_equal(draft[b], z):
                k = int(np.flatnonzero(draft[b] != z)[0])
                assert dm[k] < MARGIN_EXACT, (seed, b, k, dm[k])
                continue
            qg = q_gpu[b * gamma:(b + 1) * gamma, :V]
            np.testing.assert_allclose(qg, q, rtol=2.5e-7, atol=0)
            np.testing.assert_array_equal(qtok[b], qg[np.arange(gamma), z])
            if n_v[b] != n:
                assert am[min(n, n_v[b])] < 1e-6, (seed, b, n, n_v[b], am)
                continue
            assert tok_v[b] == tok or vm < 1e-7, (seed, b, tok, tok_v[b], vm)


def test_sps_rounds_tiny_fp32_single_and_ragged_batch():
    sd, t, d, s, Wt, Wd, Ws = make("tiny", 35, shrink_s=dict(n_layer=1), max_batch=3, gamma_max=8)
    check_sps_rounds(sd, [synth.gen_prefix(t.vocab, 32, 2)], 8, seeds=range(1000, 1012))
    check_sps_rounds(sd, [synth.gen_prefix(t.vocab, L, 20 + L) for L in (9, 40, 1)], 5, seeds=[7, 8, 9])
    check_sps_rounds(sd, [synth.gen_prefix(t.vocab, 17, 3)], 1, seeds=[4, 5])          # gamma = 1
    sd.close()


def test_sps_rounds_bf16_and_llama_shapes():
    sd, t, d, s, Wt, Wd, Ws = make("gpt2s", 37, shrink_t=dict(n_layer=2, vocab=5003, n_ctx=128), shrink_d=dict(n_layer=1, vocab=5003, n_ctx=128),
                                   shrink_s=dict(n_layer=1, vocab=5003, n_ctx=128), max_batch=2, gamma_max=8)
    check_sps_rounds(sd, [synth.gen_prefix(t.vocab, L, 30 + L) for L in (50, 21)], 8, seeds=[1, 2])
    sd.close()
    sd, t, d, s, Wt, Wd, Ws = make("llama8b", 39, shrink_t=dict(n_layer=2, d_model=512, n_head=4, n_kv_head=2, d_ff=1408, vocab=2000, n_ctx=128),
                                   shrink_d=dict(n_layer=1, d_model=256, n_head=4, n_kv_head=4, d_ff=512, vocab=2000, n_ctx=128),
                                   shrink_s=dict(n_layer=1, d_model=256, n_head=2, n_kv_head=1, d_ff=512, vocab=2000, n_ctx=128), max_batch=2, gamma_max=6)
    check_sps_rounds(sd, [synth.gen_prefix(t.vocab, L, 40 + L) for L in (30, 12)], 6, seeds=[5, 6])
    sd.close()


def test_sps_rounds_against_the_pure_oracle_and_self_drafting():
    sd, t, d, s, Wt, Wd, Ws = make("tiny", 41, shrink_s=dict(n_layer=1), gamma_max=6)
    prefix = synth.gen_prefix(t.vocab, 24, 6)
    sl = lambda tokens, rows: otf.logits_at(Ws, s, tokens, rows)
    tl = lambda tokens, rows: otf.logits_at(Wt, t, tokens, rows)
    exact = 0
    for seed in range(2000, 2024):
        draft, n_g, tok_g = sd.sd_sps_round([prefix], 6, seed)
        z, q, dm, _ = osd.oracle_sps_draft(sl, prefix, 6, seed)
        if not np.array_equal(draft[0], z):
            k = int(np.flatnonzero(draft[0] != z)[0])
            assert dm[k] < 1e-5, (seed, k, dm[k])
            continue
        n, tok, vm, fb = osd.oracle_verify(tl, prefix, z, q, seed)
        if n != n_g[0] or tok != tok_g[0]:
            continue
        exact += 1
    assert exact >= 21
    sd.close()
    # the target as its own drafter: p == q up to rounding, every token accepted
    sd, t, d, s, Wt, Wd, Ws = make("tiny", 43, sps_is_target=True, gamma_max=6)
    for seed in range(10):
        draft, n, tok = sd.sd_sps_round([prefix], 6, seed)
        assert n[0] == 6
    sd.close()


def test_hybrid_generation_greedy_is_lossless_and_matches_the_oracle():
    sd, t, d, s, Wt, Wd, Ws = make("tiny", 45, shrink_s=dict(n_layer=1), max_batch=2, gamma_max=6)
    sd.close()
    from paper_2408_05636_amd import binding
    Wt = {k: v * (40.0 if k == "w_head" else 1.0) for k, v in Wt.items()}          # distinct argmaxima
    sd = binding.SpecDiff(t, d, Wt, Wd, max_batch=2, gamma_max=6)
    sd.sd_sps_attach(s, Ws)
    sd.sd_set_greedy(True)
    prefixes = [synth.gen_prefix(t.vocab, 20, 1), synth.gen_prefix(t.vocab, 13, 2)]
    new, accepted, n_sps = sd.generate_hybrid(prefixes, 20, 3, 6, 2, 700, 8)
    tl = lambda tokens, rows: otf.logits_at(Wt, t, tokens, rows)
    for b, p in enumerate(prefixes):
        assert np.array_equal(new[b], osd.target_greedy_decode(tl, p, len(new[b]))), b
    assert 1 <= n_sps < len(accepted)
    # sequence 0 alone, as the pure oracle runs it
    sl = lambda tokens, rows: otf.logits_at(Ws, s, tokens, rows)
    dl = lambda tokens, tt: otf.logits_at(Wd, d, tokens, np.arange(len(tokens) - 6, len(tokens)), tt)
    new1, acc1, n1 = sd.generate_hybrid(prefixes[:1], 20, 3, 6, 2, 700, 8)
    toks_o, acc_o, n_o = osd.generate_hybrid(sl, dl, tl, prefixes[0], 20, 3, 6, 2, 700, t.vocab, 8, greedy=True)
    assert n1 == n_o and np.array_equal(np.array([a[0] for a in acc1]), acc_o) and np.array_equal(new1[0], toks_o)
    sd.close()


def test_sps_argument_and_state_errors():
    from paper_2408_05636_amd import binding
    w = synth.workload("tiny")
    t, d = w["target"], w["drafter"]
    sd = binding.SpecDiff(t, d, synth.gen_weights(t, 1), synth.gen_weights(d, 2), max_batch=1, gamma_max=4)
    prefix = synth.gen_prefix(t.vocab, 10, 1)
    with pytest.raises(binding.SdError) as e:
        sd.sd_sps_round([prefix], 4, 1)                                  # nothing attached
    assert e.value.code == 4
    with pytest.raises(binding.SdError):
        sd.sd_sps_attach(d, synth.gen_weights(d, 2))                     # a bidirectional model is no autoregressive drafter
    with pytest.raises(binding.SdError):
        sd.sd_sps_attach(synth.shrink(t, d_model=256), synth.gen_weights(synth.shrink(t, d_model=256), 3))   # wider than the buffers
    s = synth.shrink(t, n_layer=1)
    sd.sd_sps_attach(s, synth.gen_weights(s, 3))
    with pytest.raises(binding.SdError) as e:
        sd.sd_sps_attach(s, synth.gen_weights(s, 3))                     # already attached
    assert e.value.code == 4
    with pytest.raises(binding.SdError) as e:
        sd.sd_sps_round([prefix], 5, 1)                                  # gamma > gamma_max
    assert e.value.code == 2
    draft, n, tok = sd.sd_sps_round([prefix], 4, 1)
    assert draft.shape == (1, 4)
    sd.close()
