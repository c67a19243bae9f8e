"""The allocation-free entry point sd_accept_resample_static against sd_accept_resample: same inputs, same
integer results (bit-exact: accepted counts and tokens), on two calls in a row, the second with a smaller input
(the fixed scratch buffer keeps the first call's partials), and an oversized shape is refused."""
import numpy as np
import pytest

from paper_2408_05636_amd import synth
from tests.test_gpu_sampling import dev, make_case, padded

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def run_both(binding, vocab, batch, gamma, seed, mode):
    ld = binding.sd_vocab_pad(vocab)
    p_logits, P, q, draft = make_case(vocab, batch, gamma, seed, mode)
    qp = np.zeros((batch * gamma, ld), dtype=np.float32)
    qp[:, :vocab] = q.reshape(batch * gamma, vocab)
    pl_d, q_d, dr_d = dev(padded(p_logits, ld)), dev(qp), dev(draft)
    n_ref, tok_ref = binding.sd_accept_resample(pl_d, q_d, dr_d, batch, gamma, vocab, seed)
    n = torch.full((batch,), -7, dtype=torch.int32, device="cuda:0")
    tok = torch.full((batch,), -7, dtype=torch.int32, device="cuda:0")
    binding.sd_accept_resample_static(pl_d, q_d, dr_d, batch, gamma, vocab, seed, n, tok)
    assert torch.equal(n, n_ref) and torch.equal(tok, tok_ref), (vocab, batch, gamma, seed, mode, n, n_ref, tok, tok_ref)
    return n_ref.cpu().numpy()


def test_static_scratch_entry_point_matches_the_workspace_one():
    from paper_2408_05636_amd import binding
    assert binding.lib().sd_static_scratch_bytes() == 4 << 20
    seen = set()
    # large call first, then smaller ones on the same buffer (stale partials of the large call lie behind them)
    for vocab, batch, gamma, mode in [(50257, 2, 16, "far"), (1000, 3, 5, "close"), (50257, 1, 4, "close"),
                                      (512, 4, 8, "equal"), (128256, 1, 8, "far"), (777, 1, 1, "onehot")]:
        for seed in (11, 12):
            seen |= set(run_both(binding, vocab, batch, gamma, seed, mode).tolist())
    assert len(seen) > 2


def test_static_scratch_entry_point_refuses_what_does_not_fit():
    from paper_2408_05636_amd import binding
    lib = binding.lib()
    batch, gamma, vocab = 64, 64, 128256          # 4160 rows x 126 chunks of partials: far beyond 4 MiB
    assert binding.sd_sampling_scratch_bytes(batch * (gamma + 1), vocab) > lib.sd_static_scratch_bytes()
    x = torch.zeros(8, device="cuda:0")
    i = torch.zeros(8, dtype=torch.int32, device="cuda:0")
    st = torch.cuda.current_stream().cuda_stream
    rc = lib.sd_accept_resample_static(x.data_ptr(), x.data_ptr(), i.data_ptr(), batch, gamma, vocab, 1, i.data_ptr(), i.data_ptr(), st)
    assert rc == 5 and b"fixed buffer" in lib.sd_last_error(None)
    assert lib.sd_accept_resample_static(None, x.data_ptr(), i.data_ptr(), 1, 1, 10, 1, i.data_ptr(), i.data_ptr(), st) == 1
    torch.cuda.synchronize()
    assert int(i.sum()) == 0                     # nothing was launched
