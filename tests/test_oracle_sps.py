"""Pins of the oracle's standard speculative decoding (the paper's SpS baseline: Section 3 "Speculative decoding",
Table 1 row SpS) and of the sequence-initialisation hybrid (Section 4, "Sequence initialization").

* The autoregressive drafter samples x_k ~ q_k(. | prefix, x_<k): the joint law of the draft is the chain product,
  checked by exact integration over grids of the uniforms.
* Lossless for whole strings (unlike the diffusion drafter at T > 1, the draft tokens are sampled conditionally, so
  token-level verification is exact for every emitted token): with table-driven toy models, the law of the first two
  emitted tokens equals p(y1) p(y2 | y1) exactly.
* A drafter identical to the target gets every token accepted, whatever the uniforms; gamma drafter evaluations per round
  (depth D_p + gamma D_q).
* Hybrid: SpS rounds until n_init tokens exist, then SpecDiff rounds; at temperature 0 the emitted string is the
  target's own greedy continuation whatever either drafter proposes.
"""
import itertools
from collections import defaultdict

import numpy as np
import pytest

from oracle import philox
from oracle import specdiff as sd
from oracle import transformer as otf
from paper_2408_05636_amd import synth

V = 3


def table_model(seed, sharp=1.5):
    """A causal toy model: next-token logits depend on the last two tokens of the sequence."""
    rng = np.random.default_rng(seed)
    tab = rng.standard_normal((V + 1, V + 1, V)) * sharp

    def logits(tokens, rows):
        out = []
        for r in rows:
            a = int(tokens[r])
            b = int(tokens[r - 1]) if r >= 1 else V
            out.append(tab[b, a])
        return np.array(out)
    return logits


def law(model, tokens):
    return otf.softmax_rows(model(np.array(tokens), np.array([len(tokens) - 1])))[0]


def midgrid(n):
    return (np.arange(n) + 0.5) / n


def test_sps_draft_follows_the_drafters_chain_law():
    q = table_model(1)
    prefix = [0, 2]
    N = 240
    counts = defaultdict(float)
    for u0, u1 in itertools.product(midgrid(N), repeat=2):
        z, qs, _, nf = sd.sps_draft_with_uniforms(q, prefix, 2, np.array([u0, u1]))
        assert nf == 2
        counts[tuple(z)] += 1.0 / N ** 2
    for y0 in range(V):
        for y1 in range(V):
            expect = law(q, prefix)[y0] * law(q, prefix + [y0])[y1]
            assert counts[(y0, y1)] == pytest.approx(expect, abs=2.0 / N)
    # q_k is the row x_k was drawn from: the conditional given the tokens drafted so far
    z, qs, _, _ = sd.sps_draft_with_uniforms(q, prefix, 2, np.array([0.3, 0.9]))
    np.testing.assert_allclose(qs[0], law(q, prefix), rtol=1e-6)
    np.testing.assert_allclose(qs[1], law(q, prefix + [int(z[0])]), rtol=1e-6)


def emitted_pair_law(p, q, prefix, gamma, N):
    """Law of the first two emitted tokens of SpS generation, by integrating the oracle's code path over a grid of all
    uniforms of the first round (and, when the first round emits only one token, of a second round)."""
    out = defaultdict(float)
    grid = midgrid(N)

    def run_round(seq, weight, depth, first):
        # enumerate the uniforms of one round: gamma draft samples, gamma acceptance tests, one final sample
        for us in itertools.product(grid, repeat=gamma):
            z, qs, _, _ = sd.sps_draft_with_uniforms(q, seq, gamma, np.array(us))
            rows = np.arange(len(seq) - 1, len(seq) + gamma)
            P = otf.softmax_rows(p(np.array(list(seq) + [int(t) for t in z]), rows))
            for rs in itertools.product(grid, repeat=gamma):
                for uf in grid:
                    n, tok, _, fb = sd.verify_with_uniforms(P, qs, z, np.array(rs), np.full(gamma + 1, uf))
                    assert not fb
                    emitted = first + [int(t) for t in z[:n]] + [int(tok)]
                    w = weight / N ** (2 * gamma + 1)
                    if len(emitted) >= 2:
                        out[tuple(emitted[:2])] += w
                    else:
                        assert depth == 0
                        second[tuple(emitted)] += w
    second = defaultdict(float)
    run_round(list(prefix), 1.0, 0, [])
    for (y0,), w in list(second.items()):               # one token so far: the second comes from the next round's first token
        sub = defaultdict(float)
        seq = list(prefix) + [y0]
        for us in itertools.product(grid, repeat=gamma):
            z, qs, _, _ = sd.sps_draft_with_uniforms(q, seq, gamma, np.array(us))
            rows = np.arange(len(seq) - 1, len(seq) + gamma)
            P = otf.softmax_rows(p(np.array(seq + [int(t) for t in z]), rows))
            for rs in itertools.product(grid, repeat=gamma):
                for uf in grid:
                    n, tok, _, _ = sd.verify_with_uniforms(P, qs, z, np.array(rs), np.full(gamma + 1, uf))
                    first_tok = int(z[0]) if n >= 1 else int(tok)
                    sub[first_tok] += 1.0 / N ** (2 * gamma + 1)
        for y1, w1 in sub.items():
            out[(y0, y1)] += w * w1
    return out


def test_sps_rounds_emit_strings_with_the_targets_law():
    p, q = table_model(2), table_model(3)
    prefix = [1, 0]
    N = 30                                                     # gamma = 1: three uniforms per round
    got = emitted_pair_law(p, q, prefix, 1, N)
    for y0 in range(V):
        for y1 in range(V):
            expect = law(p, prefix)[y0] * law(p, prefix + [y0])[y1]
            assert got[(y0, y1)] == pytest.approx(expect, abs=1.5 / N)
    assert sum(got.values()) == pytest.approx(1.0)


def test_sps_first_token_law_with_two_draft_tokens():
    """gamma = 2: P(first emitted = y) = p(y | prefix), by integration over the five uniforms that matter."""
    p, q = table_model(4), table_model(5, sharp=2.5)
    prefix = [2, 2]
    N = 60
    grid = midgrid(N)
    got = np.zeros(V)
    for u0 in grid:                                            # the second draft sample never changes the first emitted token
        z, qs, _, _ = sd.sps_draft_with_uniforms(q, prefix, 2, np.array([u0, 0.37]))
        rows = np.arange(len(prefix) - 1, len(prefix) + 2)
        P = otf.softmax_rows(p(np.array(prefix + [int(t) for t in z]), rows))
        for r0 in grid:
            for uf in grid:
                n, tok, _, _ = sd.verify_with_uniforms(P, qs, z, np.array([r0, 0.5]), np.full(3, uf))
                got[int(z[0]) if n >= 1 else int(tok)] += 1.0 / N ** 3
    np.testing.assert_allclose(got, law(p, prefix), atol=2.0 / N)


@pytest.mark.parametrize("seed", range(4))
def test_a_drafter_equal_to_the_target_gets_everything_accepted(seed):
    m = table_model(10 + seed)
    rng = np.random.default_rng(seed)
    gamma = 5
    prefix = [0, 1]
    for _ in range(30):
        z, qs, _, nf = sd.sps_draft_with_uniforms(m, prefix, gamma, rng.random(gamma))
        assert nf == gamma
        rows = np.arange(len(prefix) - 1, len(prefix) + gamma)
        P = otf.softmax_rows(m(np.array(prefix + [int(t) for t in z]), rows))
        n, tok, _, fb = sd.verify_with_uniforms(P, qs, z, rng.random(gamma), rng.random(gamma + 1))
        assert n == gamma and not fb


def test_sps_uniforms_come_from_their_own_stream():
    u = sd.sps_uniforms(77, 3, 6)
    ref = philox.uniforms(77, philox.STREAM_SPS, 3, 0, np.arange(6))[1]
    assert np.array_equal(u, ref) and philox.STREAM_SPS not in (philox.STREAM_DRAFT, philox.STREAM_VERIFY)
    z1, *_ = sd.oracle_sps_draft(table_model(1), [0, 1], 6, 77, batch=3)
    z2, *_ = sd.sps_draft_with_uniforms(table_model(1), [0, 1], 6, ref)
    assert np.array_equal(z1, z2)


def tiny_models():
    w = synth.workload("tiny")
    t, d = w["target"], w["drafter"]
    s = synth.shrink(w["target"], n_layer=1)                    # the autoregressive drafter: a smaller causal model
    Wt, Wd, Ws = synth.gen_weights(t, 21), synth.gen_weights(d, 22), synth.gen_weights(s, 23)
    Wt = {k: v * (40.0 if k == "w_head" else 1.0) for k, v in Wt.items()}       # a sharper target: distinct argmaxima
    tl = lambda tokens, rows: otf.logits_at(Wt, t, tokens, rows)
    sl = lambda tokens, rows: otf.logits_at(Ws, s, tokens, rows)
    return t, tl, sl, (Wd, d)


def test_hybrid_generation_bookkeeping_and_greedy_losslessness():
    t, tl, sl, (Wd, d) = tiny_models()
    gamma, T, gs = 4, 2, 3
    dl = lambda tokens, tt: otf.logits_at(Wd, d, tokens, np.arange(len(tokens) - gamma, len(tokens)), tt)
    prefix = synth.gen_prefix(t.vocab, 12, 5)
    toks, acc, n_sps = sd.generate_hybrid(sl, dl, tl, prefix, 14, gs, gamma, T, 300, t.vocab, 6, greedy=True)
    ref = sd.target_greedy_decode(tl, prefix, len(toks))
    assert np.array_equal(toks, ref)                                     # lossless whatever either drafter proposes
    # SpS rounds run exactly until six tokens exist, SpecDiff rounds afterwards
    emitted = np.cumsum(acc + 1)
    assert n_sps == int(np.searchsorted(emitted, 6)) + 1 and 1 <= n_sps < len(acc)
    assert (acc[:n_sps] <= gs).all() and (acc[n_sps:] <= gamma).all() and len(toks) == emitted[-1] >= 14
    # stochastic rule: same bookkeeping, every round consumes seed + round index
    toks2, acc2, n2 = sd.generate_hybrid(sl, dl, tl, prefix, 10, gs, gamma, T, 300, t.vocab, 4, greedy=False)
    assert len(toks2) == int((acc2 + 1).sum()) >= 10 and n2 >= 1
    z0, q0, _, _ = sd.oracle_sps_draft(sl, prefix, gs, 300)
    n0, tok0, _, _ = sd.oracle_verify(tl, prefix, z0, q0, 300)
    assert acc2[0] == n0 and np.array_equal(toks2[:n0 + 1], np.append(z0[:n0], tok0))
