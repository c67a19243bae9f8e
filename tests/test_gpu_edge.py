"""Degenerate and limiting shapes of a round on the GPU, each replayed by the oracle's Algorithm 1 on the
GPU's own forwards (exact decisions): a single draft slot, more diffusion steps than slots, a context filled
to the last position, the largest step count, and the limits that must be refused."""
import numpy as np
import pytest

from paper_2408_05636_amd import synth
from tests.test_gpu_round import check_rounds, make

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def test_single_slot_and_more_steps_than_slots():
    sd, t, d, Wt, Wd = make("tiny", seed=21, max_batch=2, gamma_max=8)
    prefixes = [synth.gen_prefix(t.vocab, L, 40 + L) for L in (12, 3)]
    check_rounds(sd, prefixes, 1, 1, seeds=[1, 2])            # gamma = 1, T = 1
    check_rounds(sd, prefixes, 1, 5, seeds=[3])               # one slot, five steps
    check_rounds(sd, prefixes[:1], 2, 16, seeds=[4, 5])       # T >> gamma: most steps reveal nothing
    sd.close()


def test_context_filled_to_the_last_position_and_limits():
    from paper_2408_05636_amd import binding
    sd, t, d, Wt, Wd = make("tiny", seed=22, max_batch=1, gamma_max=8)
    n_ctx = min(t.n_ctx, d.n_ctx)
    full = [synth.gen_prefix(t.vocab, n_ctx - 8, 5)]
    check_rounds(sd, full, 8, 2, seeds=[6])                   # prefix + gamma == n_ctx
    with pytest.raises(binding.SdError):
        sd.sd_round([synth.gen_prefix(t.vocab, n_ctx - 7, 5)], 8, 2, 6)     # one position too many
    with pytest.raises(binding.SdError):
        sd.sd_round(full, 9, 2, 6)                            # gamma > gamma_max
    with pytest.raises(binding.SdError):
        sd.sd_round(full, 8, 257, 6)                          # T beyond the step limit
    with pytest.raises(binding.SdError):
        sd.sd_round([full[0], full[0]], 8, 2, 6)              # batch > max_batch
    sd.close()


def test_largest_step_count():
    sd, t, d, Wt, Wd = make("tiny", seed=23, max_batch=1, gamma_max=8)
    prefix = [synth.gen_prefix(t.vocab, 10, 9)]
    draft, n, tok = sd.sd_round(prefix, 3, 256, 77)
    assert ((draft >= 0) & (draft < t.vocab)).all() and 0 <= n[0] <= 3
    check_rounds(sd, prefix, 3, 64, seeds=[8])
    sd.close()


def test_step_count_changes_back_and_forth():
    """The timestep-embedding table is kept between calls and rebuilt when T changes: T = 4, 8, 4 on one handle
    (and one eager, one captured and one replayed launch sequence per T) each reproduce Algorithm 1."""
    sd, t, d, Wt, Wd = make("tiny", seed=24, max_batch=1, gamma_max=8)
    prefix = [synth.gen_prefix(t.vocab, 20, 11)]
    for T in (4, 8, 4, 8):
        check_rounds(sd, prefix, 6, T, seeds=[30 + T, 31 + T])
    sd.close()


def test_profile_entries_name_the_part_of_the_round():
    sd, t, d, Wt, Wd = make("tiny", seed=25, max_batch=1, gamma_max=8)
    prefix = [synth.gen_prefix(t.vocab, 16, 12)]
    sd.sd_round(prefix, 4, 3, 1)
    sd.sd_profile_begin()
    sd.sd_round(prefix, 4, 3, 2)
    prof = sd.sd_profile_end()
    parts = {e["name"].split(":")[0] for e in prof}
    assert parts == {"draft", "verify", "accept"}, parts
    launches = {p: sum(e["launches"] for e in prof if e["name"].startswith(p + ":")) for p in parts}
    # the draft part is T forwards (every layer kernel T times), the verify part one forward
    assert launches["draft"] > 2 * launches["verify"] and launches["accept"] >= 1
    assert all(e["ms"] > 0 for e in prof)
    sd.close()


def test_step_skipping_changes_nothing_but_the_number_of_forwards():
    """sd_set_step_skipping: the drafter runs only at the steps that reveal a slot.  Draft, q, q(x), accepted counts
    and extra tokens are bit-identical with the option on and off (stochastic and temperature-0 rule, single
    sequence and batch, each launch sequence eager, captured and replayed), the number of forwards is the number of
    distinct reveal steps of the oracle's reveal rule, and with the option on the rounds still reproduce Algorithm 1."""
    from oracle import specdiff as osd
    sd, t, d, Wt, Wd = make("tiny", seed=26, max_batch=3, gamma_max=8)
    V = t.vocab
    saved = 0
    for prefixes, gamma, T in (([synth.gen_prefix(V, 24, 13)], 4, 8), ([synth.gen_prefix(V, 9, 14), synth.gen_prefix(V, 30, 15), synth.gen_prefix(V, 17, 16)], 3, 6)):
        for greedy in (False, True):
            sd.sd_set_greedy(greedy)
            for seed in range(500, 512):
                sd.sd_set_step_skipping(False)
                d0, qt0, q0 = sd.sd_draft(prefixes, gamma, T, seed)
                assert (q0 is None) == greedy                      # temperature 0 produces no q
                q0 = None if greedy else q0.cpu().numpy().copy()
                assert sd.sd_steps_run() == T
                r0 = sd.sd_round(prefixes, gamma, T, seed)
                sd.sd_set_step_skipping(True)
                d1, qt1, q1 = sd.sd_draft(prefixes, gamma, T, seed)
                q1 = None if greedy else q1.cpu().numpy().copy()
                steps = set()
                for b in range(len(prefixes)):
                    ua, _ = osd.draft_uniforms(seed, b, gamma, T)
                    steps |= {next(j for j in range(T, 0, -1) if j == 1 or ua[j, k] * j < 1.0) for k in range(gamma)}
                assert sd.sd_steps_run() == len(steps)
                saved += T - len(steps)
                r1 = sd.sd_round(prefixes, gamma, T, seed)
                assert sd.sd_steps_run() == len(steps)
                assert np.array_equal(d0, d1) and np.array_equal(qt0, qt1)
                if not greedy:
                    assert np.array_equal(q0[:, :V], q1[:, :V])
                assert all(np.array_equal(a, b) for a, b in zip(r0, r1))
    assert saved > 0
    sd.sd_set_greedy(False)
    check_rounds(sd, [synth.gen_prefix(V, 24, 13)], 4, 8, seeds=[601, 602, 603])     # with the option still on
    sd.close()
    # bf16 pair at GPT-2 width (matrix-core kernels, folded normalisations, direct KV-cache writes)
    sd, t, d, Wt, Wd = make("gpt2s", seed=27, shrink_t=dict(n_layer=2, vocab=3001, n_ctx=256), shrink_d=dict(n_layer=2, vocab=3001, n_ctx=256),
                            max_batch=1, gamma_max=8)
    prefix = [synth.gen_prefix(t.vocab, 200, 17)]
    for seed in range(700, 706):
        sd.sd_set_step_skipping(False)
        r0 = sd.sd_round(prefix, 8, 8, seed)
        sd.sd_set_step_skipping(True)
        r1 = sd.sd_round(prefix, 8, 8, seed)
        assert all(np.array_equal(a, b) for a, b in zip(r0, r1)) and 1 <= sd.sd_steps_run() <= 8
    sd.close()
