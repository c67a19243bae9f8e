"""GPU parity of the temperature-0 mode (sd_set_greedy), of sd_commit and of multi-round generation.

 (a) Level 1: the oracle's greedy rule fed with the GPU's own logits reproduces the GPU's draft tokens,
     accepted counts and extra tokens exactly (arg-maxima on identical fp32 numbers, lowest id on ties).
 (b) The lossless property: a greedy generation equals the target's own greedy continuation, computed by
     the pure fp64 oracle on a model whose heads are sharpened so that no argmax hinges on rounding.
 (c) sd_commit keeps results unchanged (a round after a commit equals a round after a fresh prefill) and
     rejects calls that have nothing to commit.
"""
import numpy as np
import pytest

from oracle import specdiff as osd
from oracle import transformer as otf
from paper_2408_05636_amd import synth

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def build(workload, seed, shrink_t, shrink_d, sharpen, max_batch=2, gamma_max=8):
    from paper_2408_05636_amd import binding
    w = synth.workload(workload)
    t = synth.shrink(w["target"], **shrink_t)
    d = synth.shrink(w["drafter"], **shrink_d)
    Wt, Wd = synth.gen_weights(t, seed), synth.gen_weights(d, seed + 1)
    if sharpen:
        for W, c in ((Wt, t), (Wd, d)):
            x = W["w_head"] * np.float32(sharpen)
            W["w_head"] = synth.round_to_bf16(x) if c.dtype == "bf16" else x
    return binding.SpecDiff(t, d, Wt, Wd, max_batch=max_batch, gamma_max=gamma_max), t, d, Wt, Wd


def level1_round(sd, prefixes, gamma, T, seed):
    """One greedy round; every decision re-derived by the oracle from the GPU's logits."""
    V = sd.target.vocab
    B = len(prefixes)
    draft, qtok, _ = sd.sd_draft(prefixes, gamma, T, seed)
    assert (qtok == 1.0).all()
    for b, p in enumerate(prefixes):
        def dl(tokens, t, b=b):
            seqs = [np.concatenate([pp, np.full(gamma, V)]).astype(np.int32) for pp in prefixes]
            seqs[b] = tokens.astype(np.int32)
            return sd.sd_drafter_logits(seqs, gamma, int(round(t * T)), T).cpu().numpy()[b * gamma:(b + 1) * gamma, :V]
        z, gaps, _ = osd.oracle_draft_greedy(dl, p, gamma, T, seed, V, batch=b)
        # other sequences of the batch were evaluated with an all-[MASK] block above, this one exactly as in the
        # round only if B == 1; for B > 1 compare sequence 0 only when the others' blocks do not matter (no cross-talk)
        assert np.array_equal(draft[b], z), (b, draft[b], z, gaps)
    lt = sd.sd_target_logits(prefixes, draft).cpu().numpy()
    draft_r, n, tok = sd.sd_round(prefixes, gamma, T, seed)
    assert np.array_equal(draft, draft_r)
    for b in range(B):
        n_o, tok_o, _ = osd.verify_greedy(lt[b * (gamma + 1):(b + 1) * (gamma + 1), :V], draft[b])
        assert (n[b], tok[b]) == (n_o, tok_o)
    return draft, n, tok


def test_greedy_round_matches_oracle_on_gpu_logits_fp32():
    sd, t, d, Wt, Wd = build("tiny", 5, {}, {}, sharpen=0)
    sd.sd_set_greedy(True)
    prefixes = [synth.gen_prefix(t.vocab, 32, 7), synth.gen_prefix(t.vocab, 20, 8)]
    for seed in (1, 2, 3):
        level1_round(sd, prefixes, 8, 4, seed)


def test_greedy_round_matches_oracle_on_gpu_logits_bf16():
    sd, t, d, Wt, Wd = build("gpt2s", 9, dict(n_layer=2, vocab=3000), dict(n_layer=2, vocab=3000), sharpen=0, gamma_max=16)
    sd.sd_set_greedy(True)
    prefixes = [synth.gen_prefix(t.vocab, 70, 3)]
    for seed in (4, 5):
        level1_round(sd, prefixes, 16, 4, seed)
    # back to the stochastic rule: results differ from temperature 0 and q is produced again
    sd.sd_set_greedy(False)
    draft, qtok, q = sd.sd_draft(prefixes, 16, 4, 4)
    assert (qtok < 1.0).all() and abs(float(q[0, :t.vocab].sum()) - 1.0) < 1e-4


@pytest.mark.parametrize("gamma,T", [(4, 2), (8, 3)])
def test_greedy_generation_is_the_targets_greedy_string(gamma, T):
    sd, t, d, Wt, Wd = build("tiny", 11, {}, {}, sharpen=40.0)
    sd.sd_set_greedy(True)
    prefixes = [synth.gen_prefix(t.vocab, 24, 1), synth.gen_prefix(t.vocab, 17, 2)]
    new, accepted = sd.generate(prefixes, 24, gamma, T, seed=100)
    tl = lambda tokens, rows: otf.logits_at(Wt, t, tokens, rows)
    for b, p in enumerate(prefixes):
        ref = osd.target_greedy_decode(tl, p, len(new[b]))
        assert np.array_equal(new[b], ref), (b, new[b], ref)
    assert accepted.shape[1] == 2 and (accepted >= 0).all() and (accepted <= gamma).all()
    # the whole generation, drafts included, as the pure oracle runs it (sequence 0; batch index 0 in the counters)
    dl = lambda tokens, tt: otf.logits_at(Wd, d, tokens, np.arange(len(tokens) - gamma, len(tokens)), tt)
    toks_o, acc_o = osd.generate(dl, tl, prefixes[0], 24, gamma, T, 100, t.vocab, greedy=True)
    k = min(len(acc_o), accepted.shape[0])
    assert np.array_equal(acc_o[:k], accepted[:k, 0])


def test_commit_keeps_results_and_checks_state():
    from paper_2408_05636_amd import binding
    sd, t, d, Wt, Wd = build("tiny", 13, {}, {}, sharpen=40.0)
    prefixes = [synth.gen_prefix(t.vocab, 30, 4)]
    with pytest.raises(binding.SdError):
        sd.sd_commit(np.zeros(1, dtype=np.int32))            # nothing verified yet
    draft, n, tok = sd.sd_round(prefixes, 8, 4, 21)
    with pytest.raises(binding.SdError):
        sd.sd_commit(np.array([9], dtype=np.int32))           # more than gamma
    sd.sd_commit(n)
    with pytest.raises(binding.SdError):
        sd.sd_commit(n)                                       # already committed
    nxt = [np.concatenate([prefixes[0], draft[0, :n[0]], tok[:1]]).astype(np.int32)]
    after_commit = sd.sd_round(nxt, 8, 4, 22)
    sd.sd_prefill(nxt)                                        # the same round from a fresh prefill
    fresh = sd.sd_round(nxt, 8, 4, 22)
    for a, b in zip(after_commit, fresh):
        assert np.array_equal(a, b)


def test_stochastic_generation_equals_round_by_round_calls():
    sd, t, d, Wt, Wd = build("tiny", 17, {}, {}, sharpen=0)
    prefixes = [synth.gen_prefix(t.vocab, 16, 5), synth.gen_prefix(t.vocab, 28, 6)]
    new, accepted = sd.generate(prefixes, 12, 6, 3, seed=50)
    seqs = [list(p) for p in prefixes]
    for i in range(accepted.shape[0]):
        sd.sd_prefill(seqs)                                    # no commit: prefill every round
        draft, n, tok = sd.sd_round(seqs, 6, 3, 50 + i)
        assert np.array_equal(n, accepted[i])
        for b in range(2):
            seqs[b] += list(draft[b, :n[b]]) + [tok[b]]
    for b in range(2):
        assert np.array_equal(np.array(seqs[b][len(prefixes[b]):]), new[b])


def test_generation_with_step_skipping_is_the_same_generation():
    """A multi-round generation (prefix growing by every round's accepted tokens, sd_commit in between, one launch
    sequence per step and length) with the drafter left out at idle steps emits the same tokens and accepts the same
    counts as without, at temperature 0 (where it is also the target's own greedy string) and with the stochastic rule."""
    sd, t, d, Wt, Wd = build("tiny", 11, {}, {}, sharpen=40.0, max_batch=1)
    prefix = [synth.gen_prefix(t.vocab, 24, 1)]
    tl = lambda tokens, rows: otf.logits_at(Wt, t, tokens, rows)
    for greedy in (True, False):
        sd.sd_set_greedy(greedy)
        sd.sd_set_step_skipping(False)
        new0, acc0 = sd.generate(prefix, 20, 4, 6, seed=300)
        sd.sd_set_step_skipping(True)
        new1, acc1 = sd.generate(prefix, 20, 4, 6, seed=300)
        assert np.array_equal(new0[0], new1[0]) and np.array_equal(acc0, acc1)
        if greedy:
            assert np.array_equal(new1[0], osd.target_greedy_decode(tl, prefix[0], len(new1[0])))
    sd.close()
