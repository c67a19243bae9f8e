"""Pins for oracle/transformer.py.

The oracle's forwards are checked against an independent composition of torch CPU library
routines in fp64 (layer_norm, scaled_dot_product_attention, gelu(tanh), silu, complex
rotation for RoPE) written here, and against structural properties a mistake would break:
causal / bidirectional dependence, GQA == MHA when every query head has its own kv head,
RoPE's shift invariance, a time-embedding that matters.
"""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import transformer as otf
from paper_2408_05636_amd import synth

torch.set_grad_enabled(False)
T64 = lambda a: torch.tensor(np.asarray(a, dtype=np.float64))


def small(arch, bidirectional, n_kv_head=4, dtype="f32"):
    return synth.ModelConfig(arch, dtype, 2, 64, 4, n_kv_head, 160, 97, 64, bidirectional, 1e-5, 10000.0)


def torch_forward(W, cfg, tokens, t=None):
    """Independent fp64 reference out of torch library ops (batch-free, one sequence)."""
    tok = torch.tensor(np.asarray(tokens, dtype=np.int64))
    S, d, H, Hkv = tok.numel(), cfg.d_model, cfg.n_head, cfg.n_kv_head
    dh = d // H
    h = T64(W["wte"])[tok]
    if cfg.arch == "gpt2":
        h = h + T64(W["wpe"])[:S]
    if cfg.bidirectional:
        i = torch.arange(d // 2, dtype=torch.float64)
        ang = 1000.0 * t * torch.exp(-np.log(10000.0) * 2.0 * i / d)
        s = torch.cat([torch.sin(ang), torch.cos(ang)])
        h = h + F.linear(F.silu(F.linear(s, T64(W["t_w1"]), T64(W["t_b1"]))), T64(W["t_w2"]), T64(W["t_b2"]))

    def norm(x, g, b):
        if cfg.arch == "gpt2":
            return F.layer_norm(x, (d,), T64(W[g]), T64(W[b]), cfg.norm_eps)
        return x * torch.rsqrt((x * x).mean(-1, keepdim=True) + cfg.norm_eps) * T64(W[g])

    def rot(x):      # x: [S, heads, dh]; complex rotation of (x_i, x_{i+dh/2})
        half = dh // 2
        inv = cfg.rope_theta ** (-torch.arange(half, dtype=torch.float64) * 2.0 / dh)
        ph = torch.polar(torch.ones(S, half, dtype=torch.float64), torch.arange(S, dtype=torch.float64)[:, None] * inv)
        zc = torch.complex(x[..., :half], x[..., half:]) * ph[:, None, :]
        return torch.cat([zc.real, zc.imag], dim=-1)

    for l in range(cfg.n_layer):
        p = f"l{l}."
        x = norm(h, p + "ln1_g", p + "ln1_b")
        qkv = F.linear(x, T64(W[p + "w_qkv"]), T64(W[p + "b_qkv"]) if cfg.arch == "gpt2" else None)
        q, k, v = torch.split(qkv, [H * dh, Hkv * dh, Hkv * dh], dim=-1)
        q, k, v = q.view(S, H, dh), k.view(S, Hkv, dh), v.view(S, Hkv, dh)
        if cfg.arch == "llama":
            q, k = rot(q), rot(k)
        k = k.repeat_interleave(H // Hkv, dim=1)
        v = v.repeat_interleave(H // Hkv, dim=1)
        a = F.scaled_dot_product_attention(q.transpose(0, 1), k.transpose(0, 1), v.transpose(0, 1),
                                           is_causal=not cfg.bidirectional)
        a = a.transpose(0, 1).reshape(S, d)
        if cfg.arch == "gpt2":
            h = h + F.linear(a, T64(W[p + "w_o"]), T64(W[p + "b_o"]))
            x = norm(h, p + "ln2_g", p + "ln2_b")
            m = F.gelu(F.linear(x, T64(W[p + "w_fc"]), T64(W[p + "b_fc"])), approximate="tanh")
            h = h + F.linear(m, T64(W[p + "w_proj"]), T64(W[p + "b_proj"]))
        else:
            h = h + F.linear(a, T64(W[p + "w_o"]))
            x = norm(h, p + "ln2_g", None)
            m = F.silu(F.linear(x, T64(W[p + "w_gate"]))) * F.linear(x, T64(W[p + "w_up"]))
            h = h + F.linear(m, T64(W[p + "w_proj"]))
    h = norm(h, "lnf_g", "lnf_b")
    return F.linear(h, T64(W["w_head"])).numpy()


def scaled_weights(cfg, seed, scale=8.0):
    """N(0, 0.02) weights make every layer nearly linear; scale the matrices up so that
    softmax, GELU and the norms are exercised away from their linear regime."""
    W = synth.gen_weights(cfg, seed)
    for name, _, role in synth.weight_specs(cfg):
        if role in ("matrix", "embed", "bias"):
            W[name] = W[name] * np.float32(scale)
    return W


@pytest.mark.parametrize("arch,bidir,kv", [("gpt2", False, 4), ("gpt2", True, 4), ("llama", False, 2), ("llama", False, 4)])
def test_forward_matches_torch_library_composition(arch, bidir, kv):
    cfg = small(arch, bidir, kv)
    W = scaled_weights(cfg, 11)
    tokens = synth.gen_prefix(cfg.vocab, 23, 5).astype(np.int64)
    if bidir:
        tokens[-5:] = cfg.vocab                       # mask ids
    t = 0.75 if bidir else None
    got = otf.logits_at(W, cfg, tokens, np.arange(tokens.size), t)
    ref = torch_forward(W, cfg, tokens, t)
    assert got.shape == (23, cfg.vocab)
    assert np.abs(ref).max() > 0.5                    # not a degenerate comparison
    np.testing.assert_allclose(got, ref, rtol=1e-10, atol=1e-11)


def test_causal_target_ignores_the_future_and_drafter_does_not():
    tokens = synth.gen_prefix(97, 20, 8).astype(np.int64)
    other = tokens.copy()
    other[12] = (other[12] + 1) % 97
    for arch in ("gpt2", "llama"):
        cfg = small(arch, False)
        W = scaled_weights(cfg, 3)
        a = otf.logits_at(W, cfg, tokens, np.arange(20))
        b = otf.logits_at(W, cfg, other, np.arange(20))
        assert np.array_equal(a[:12], b[:12])          # positions before the change: identical
        assert np.abs(a[12:] - b[12:]).max() > 1e-3
    cfg = small("gpt2", True)
    W = scaled_weights(cfg, 3)
    a = otf.logits_at(W, cfg, tokens, np.arange(20), 0.5)
    b = otf.logits_at(W, cfg, other, np.arange(20), 0.5)
    assert np.abs(a[:12] - b[:12]).max() > 1e-4        # bidirectional: earlier rows see it


def test_prefix_of_causal_forward_equals_forward_of_prefix():
    """What a KV cache relies on: rows of the long forward equal the short forward's rows."""
    cfg = small("llama", False, 2)
    W = scaled_weights(cfg, 4)
    tokens = synth.gen_prefix(97, 18, 9).astype(np.int64)
    full = otf.logits_at(W, cfg, tokens, np.arange(18))
    part = otf.logits_at(W, cfg, tokens[:11], np.arange(11))
    np.testing.assert_allclose(full[:11], part, rtol=1e-12, atol=1e-13)


def test_timestep_changes_drafter_output_and_mask_row_is_used():
    cfg = small("gpt2", True)
    W = scaled_weights(cfg, 6)
    tokens = synth.gen_prefix(97, 16, 2).astype(np.int64)
    tokens[-4:] = cfg.vocab
    a = otf.logits_at(W, cfg, tokens, np.arange(12, 16), 1.0)
    b = otf.logits_at(W, cfg, tokens, np.arange(12, 16), 0.25)
    assert np.abs(a - b).max() > 1e-4
    W2 = dict(W)
    W2["wte"] = W["wte"].copy()
    W2["wte"][cfg.vocab, ::2] += 1.0            # (a constant shift of the whole row is removed by LayerNorm)
    c = otf.logits_at(W2, cfg, tokens, np.arange(12, 16), 1.0)
    assert np.abs(a - c).max() > 1e-3
    assert a.shape[1] == cfg.vocab                     # no output class for the mask token


def test_gqa_with_duplicated_kv_heads_equals_mha():
    g = small("llama", False, 2)
    m = small("llama", False, 4)
    Wg = scaled_weights(g, 12)
    Wm = dict(Wg)
    dh, d = g.d_model // g.n_head, g.d_model
    for l in range(g.n_layer):
        w = Wg[f"l{l}.w_qkv"]
        q, k, v = w[:d], w[d:d + 2 * dh], w[d + 2 * dh:]
        rep = lambda x: np.repeat(x.reshape(2, dh, d), 2, axis=0).reshape(4 * dh, d)
        Wm[f"l{l}.w_qkv"] = np.concatenate([q, rep(k), rep(v)], axis=0)
    tokens = synth.gen_prefix(97, 14, 1)
    np.testing.assert_allclose(otf.logits_at(Wg, g, tokens, np.arange(14)),
                               otf.logits_at(Wm, m, tokens, np.arange(14)), rtol=1e-12, atol=1e-13)


def test_rope_scores_depend_on_relative_position_only():
    rng = np.random.default_rng(0)
    q = rng.standard_normal((6, 2, 16))
    k = rng.standard_normal((6, 2, 16))
    pos = np.arange(6)
    s0 = np.einsum("ihd,jhd->hij", otf.rope(q, pos, 10000.0), otf.rope(k, pos, 10000.0))
    s1 = np.einsum("ihd,jhd->hij", otf.rope(q, pos + 37, 10000.0), otf.rope(k, pos + 37, 10000.0))
    np.testing.assert_allclose(s0, s1, rtol=1e-10, atol=1e-10)
    assert np.allclose(otf.rope(q, np.zeros(6), 10000.0), q)      # position 0 is the identity
    x = np.zeros((1, 1, 4)); x[0, 0, 0] = 1.0                     # quarter turn of pair (0, 2) at angle pi/2
    y = otf.rope(x, np.array([np.pi / 2]), 1.0)
    np.testing.assert_allclose(y[0, 0], [0, 0, 1, 0], atol=1e-12)


def test_elementwise_closed_forms():
    x = np.linspace(-6, 6, 101)
    from scipy.special import erf, softmax as sp_softmax
    assert np.abs(otf.gelu_tanh(x) - 0.5 * x * (1 + erf(x / np.sqrt(2)))).max() < 2.5e-3  # tanh form approximates erf form
    assert otf.gelu_tanh(np.array([0.0]))[0] == 0.0
    np.testing.assert_allclose(otf.gelu_tanh(np.array([1.0])), [0.8411919906082768], rtol=1e-12)
    np.testing.assert_allclose(otf.silu(np.array([1.0, -2.0])), [1 / (1 + np.exp(-1.0)), -2 / (1 + np.exp(2.0))], rtol=1e-14)
    r = np.random.default_rng(1).standard_normal((5, 33)) * 4
    np.testing.assert_allclose(otf.softmax_rows(r), sp_softmax(r, axis=-1), rtol=1e-13)
    ln = otf.layer_norm(r, np.ones(33), np.zeros(33), 0.0)
    np.testing.assert_allclose(ln.mean(-1), 0, atol=1e-13)
    np.testing.assert_allclose((ln ** 2).mean(-1), 1, rtol=1e-12)
    np.testing.assert_allclose((otf.rms_norm(r, np.ones(33), 0.0) ** 2).mean(-1), 1, rtol=1e-12)


def test_linear_matches_library_routine():
    rng = np.random.default_rng(3)
    x, W, b = rng.standard_normal((5, 7)), rng.standard_normal((4, 7)), rng.standard_normal(4)
    np.testing.assert_allclose(otf.linear(x, W, b), F.linear(T64(x), T64(W), T64(b)).numpy(), rtol=1e-13)
    assert otf.linear(np.eye(3), np.arange(6.0).reshape(2, 3)).tolist() == [[0, 3], [1, 4], [2, 5]]   # W is [out, in]
