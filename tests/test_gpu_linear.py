"""GPU parity of the dense contraction y = epilogue(x W^T + bias) (QKV / MLP / LM-head layers)
against the fp64 oracle, over shapes that cover every kernel variant, ragged tile edges and
all four epilogues."""
import numpy as np
import pytest

from oracle import transformer as otf
from paper_2408_05636_amd import synth

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")

SHAPES = [  # (m, n, k)
    (17, 768, 768), (16, 50257, 768), (17, 2304, 768), (17, 768, 3072),      # target / LM-head rows of the bench workload
    (272, 2304, 768), (272, 768, 768), (272, 3072, 768), (272, 768, 3072),   # drafter rows
    (1, 64, 64), (33, 100, 128), (65, 33, 192), (130, 4801, 1600), (700, 1000, 256), (3000, 1100, 128),
    (17, 1600, 6400), (17, 1600, 1600), (33, 1024, 4096), (64, 200, 2048), (40, 100, 1024),   # K split over workgroups
]


def run_case(dtype, m, n, k, epi, seed):
    from paper_2408_05636_amd import binding
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((m, k)).astype(np.float32)
    w = (rng.standard_normal((n, k)) * 0.05).astype(np.float32)
    b = rng.standard_normal(n).astype(np.float32) * 0.1
    y0 = rng.standard_normal((m, n)).astype(np.float32)            # previous content (residual epilogue adds to it)
    if dtype == "bf16":
        x, w = synth.round_to_bf16(x), synth.round_to_bf16(w)
    td = torch.bfloat16 if dtype == "bf16" else torch.float32
    xd, wd = torch.from_numpy(x).to("cuda:0").to(td), torch.from_numpy(w).to("cuda:0").to(td)
    bd = torch.from_numpy(b).to("cuda:0")
    out_f32 = epi in (2, 3)
    ld = n + 5 if n % 2 else n                                      # a leading dimension larger than n
    yd = torch.zeros(m, ld, dtype=torch.float32 if out_f32 else td, device="cuda:0")
    yd[:, :n] = torch.from_numpy(y0).to("cuda:0").to(yd.dtype)
    binding.sd_linear(dtype, xd, wd, bd, yd, epi)
    got = yd.float().cpu().numpy()
    ref = otf.linear(x, w, b)
    if epi == 1:
        ref = otf.gelu_tanh(ref)
    if epi == 2:
        ref = ref + y0.astype(np.float64)
    assert np.array_equal(got[:, n:], np.zeros((m, ld - n), dtype=np.float32))   # nothing written past column n
    scale = np.sqrt((ref ** 2).mean())
    err = np.abs(got[:, :n] - ref).max()
    # fp32 accumulation of exact products; outputs rounded to bf16 (2^-9 relative) for epilogues 0, 1
    tol = 2e-5 * scale * max(1.0, np.sqrt(k / 256)) if dtype == "f32" or out_f32 else 6e-3 * max(scale, np.abs(ref).max())
    assert err <= tol, (dtype, m, n, k, epi, err, tol)


@pytest.mark.parametrize("m,n,k", SHAPES)
def test_linear_bf16_all_epilogues(m, n, k):
    for epi in range(4):
        run_case("bf16", m, n, k, epi, seed=m + n + k + epi)


@pytest.mark.parametrize("m,n,k", [(9, 512, 128), (40, 384, 128), (40, 128, 512), (8, 512, 128), (70, 130, 72)])
def test_linear_fp32_all_epilogues(m, n, k):
    for epi in range(4):
        run_case("f32", m, n, k, epi, seed=m + n + k + epi)


@pytest.mark.parametrize("m,n,k", [(130, 4801, 1600), (700, 1000, 256), (1056, 2304, 768), (300, 130, 64), (1, 64, 64), (2100, 768, 3072),
                                   (70, 200, 128), (70, 200, 192), (257, 129, 320), (64, 128, 384)])     # K around the ring lengths (2 to 6 chunks)
@pytest.mark.parametrize("variant", [7, 8, 10, 11, 12, 13, 14, 15])
def test_linear_shared_tile_kernel(m, n, k, variant):
    """The workgroup-shared tile kernels (7, 8: 128 / 64 rows, prefetch through registers; 10-13: 64 x 64 to 256 x 128
    tiles fed straight into a ring of LDS stages, 14, 15: the 64-row ones with two chunks of K per stage; a K shorter
    than the ring or not a multiple of the stage width falls back to the default choice), forced on ragged shapes."""
    from paper_2408_05636_amd import binding
    binding.lib().sd_set_linear_variant(variant)
    try:
        for epi in range(4):
            run_case("bf16", m, n, k, epi, seed=7 + m + n + k + epi)
    finally:
        binding.lib().sd_set_linear_variant(-1)


@pytest.mark.parametrize("split", [-1, 3, 64])
@pytest.mark.parametrize("m,n,k", [(17, 768, 768), (16, 50257, 768), (33, 2304, 1024), (64, 200, 2048), (40, 100, 4096), (1, 64, 64),
                                   (33, 4100, 4096), (17, 1600, 6400), (31, 130, 2304)])
def test_linear_streaming_kernel(m, n, k, split):
    """The weight-streaming kernel for up to 64 rows (x parked in LDS; normally chosen for long weight streams only),
    forced on small and ragged shapes, with the K range in one piece and split over workgroups, twice in a row."""
    from paper_2408_05636_amd import binding
    binding.lib().sd_set_linear_variant(9)
    binding.lib().sd_set_linear_split(split)
    try:
        for epi in range(4):
            run_case("bf16", m, n, k, epi, seed=11 + m + n + k + epi)
        run_case("bf16", m, n, k, 2, seed=12 + m + n + k)
    finally:
        binding.lib().sd_set_linear_variant(-1)
        binding.lib().sd_set_linear_split(-1)


@pytest.mark.parametrize("split", [2, 3, 7, 64])
def test_linear_forced_split(split):
    """Every split count gives the same contraction (up to fp32 summation order), twice in a row on
    the same workspace, and agrees with the unsplit kernel."""
    from paper_2408_05636_amd import binding
    binding.lib().sd_set_linear_split(split)
    try:
        for m, n, k in [(17, 1600, 6400), (50, 300, 1024), (5, 96, 4096)]:
            for epi in (2, 0):
                run_case("bf16", m, n, k, epi, seed=split + m)
                run_case("bf16", m, n, k, epi, seed=split + m + 1)
    finally:
        binding.lib().sd_set_linear_split(-1)


@pytest.mark.parametrize("m,n,k", [(17, 2304, 768), (272, 2304, 768), (301, 3072, 768), (33, 100, 128), (65, 4801, 1600), (700, 1000, 256),
                                   (17, 4800, 1600), (33, 512, 4096), (60, 96, 2048), (2100, 2304, 768)])
@pytest.mark.parametrize("norm_kind", [1, 2])
@pytest.mark.parametrize("variant", [-1, 9, 10, 11, 12, 13, 14, 15])
def test_norm_folded_linear(m, n, k, norm_kind, variant):
    """LayerNorm / RMSNorm folded into the contraction vs. the oracle's norm followed by its linear
    (variant 9: the weight-streaming kernel, up to 64 rows)."""
    from paper_2408_05636_amd import binding
    if variant == 9 and m > 64:
        pytest.skip("the streaming kernel takes up to 64 rows")
    binding.lib().sd_set_linear_variant(variant)
    try:
        norm_folded_case(m, n, k, norm_kind)
    finally:
        binding.lib().sd_set_linear_variant(-1)


def norm_folded_case(m, n, k, norm_kind):
    from paper_2408_05636_amd import binding
    rng = np.random.default_rng(m + n + k + norm_kind)
    # residual-stream-like rows: a common offset pattern plus row-specific parts, non-zero mean
    h = (rng.standard_normal((1, k)) * 0.3 + rng.standard_normal((m, k)) * 0.2 + 0.05).astype(np.float32)
    w = synth.round_to_bf16((rng.standard_normal((n, k)) * 0.05).astype(np.float32))
    gain = (1 + rng.standard_normal(k) * 0.1).astype(np.float32)
    beta = (rng.standard_normal(k) * 0.1).astype(np.float32)
    bias = (rng.standard_normal(n) * 0.1).astype(np.float32)
    eps = 1e-5
    for epi in (0, 1, 3):
        hd, wd = torch.from_numpy(h).to("cuda:0"), torch.from_numpy(w).to("cuda:0").bfloat16()
        yd = torch.zeros(m, n, dtype=torch.float32 if epi == 3 else torch.bfloat16, device="cuda:0")
        binding.sd_norm_linear(norm_kind, hd, wd, torch.from_numpy(gain).to("cuda:0"), torch.from_numpy(beta).to("cuda:0"),
                               torch.from_numpy(bias).to("cuda:0"), yd, epi, eps)
        x = otf.layer_norm(h.astype(np.float64), gain, beta, eps) if norm_kind == 1 else otf.rms_norm(h.astype(np.float64), gain, eps)
        ref = otf.linear(x, w, bias)
        if epi == 1:
            ref = otf.gelu_tanh(ref)
        got = yd.float().cpu().numpy()
        scale = np.sqrt((ref ** 2).mean())
        err = np.abs(got - ref).max()
        # the A operand is rounded to bf16 (2^-9 relative per element): error ~ 2^-9 * scale / sqrt(3) * few sigma
        assert err <= 0.012 * scale + (0.006 * np.abs(ref).max() if epi != 3 else 0), (m, n, k, norm_kind, epi, err, scale)


@pytest.mark.parametrize("variant", [-1, 5, 7, 8, 9, 10, 11, 12, 13, 14, 15])
@pytest.mark.parametrize("m,n,k", [(17, 768, 768), (272, 768, 3072), (40, 100, 1024), (17, 1600, 6400), (300, 1601, 128), (1056, 768, 3072)])
def test_residual_epilogue_prepares_the_next_normalisation(m, n, k, variant):
    """Producer side of a folded normalisation: h += x W^T + b, xg = bf16(h * gain), per-tile row sums of h and h^2
    (every kernel family: few-row with K split, wave-private 64 x 64, workgroup-shared tiles, weight streaming)."""
    from paper_2408_05636_amd import binding
    if variant == 9 and m > 64:
        pytest.skip("the streaming kernel takes up to 64 rows")
    rng = np.random.default_rng(m + n + k)
    x = synth.round_to_bf16(rng.standard_normal((m, k)).astype(np.float32))
    w = synth.round_to_bf16((rng.standard_normal((n, k)) * 0.05).astype(np.float32))
    b = (rng.standard_normal(n) * 0.1).astype(np.float32)
    h0 = (rng.standard_normal((m, n)) + 0.3).astype(np.float32)
    gain = (1 + rng.standard_normal(n) * 0.1).astype(np.float32)
    binding.lib().sd_set_linear_variant(variant)
    try:
        yd = torch.from_numpy(h0.copy()).to("cuda:0")
        xg, stats = binding.sd_linear_resid_norm(torch.from_numpy(x).to("cuda:0").bfloat16(), torch.from_numpy(w).to("cuda:0").bfloat16(),
                                                 torch.from_numpy(b).to("cuda:0"), yd, torch.from_numpy(gain).to("cuda:0"))
    finally:
        binding.lib().sd_set_linear_variant(-1)
    ref = otf.linear(x, w, b) + h0.astype(np.float64)
    got = yd.cpu().numpy().astype(np.float64)
    scale = np.sqrt((ref ** 2).mean())
    assert np.abs(got - ref).max() <= 2e-5 * scale * max(1.0, np.sqrt(k / 256))
    # xg is the bf16 rounding of the fp32 product the kernel formed from its own y
    want_xg = synth.round_to_bf16((got.astype(np.float32) * gain[None, :]).astype(np.float32))
    got_xg = xg.float().cpu().numpy()
    assert np.abs(got_xg - want_xg).max() <= 2.0 ** -7 * np.abs(want_xg).max()      # at most one bf16 ulp apart
    assert (got_xg == want_xg).mean() > 0.999
    parts = (n + 31) // 32
    pad = np.zeros((m, parts * 32))
    pad[:, :n] = got
    tiles = pad.reshape(m, parts, 32)
    st = stats.cpu().numpy().astype(np.float64)
    assert np.abs(st[:, :, 0] - tiles.sum(axis=2)).max() <= 1e-5 * 32 * np.abs(got).max()
    assert np.abs(st[:, :, 1] - (tiles ** 2).sum(axis=2)).max() <= 1e-5 * 32 * (got ** 2).max()
