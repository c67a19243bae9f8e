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
