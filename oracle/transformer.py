"""The two networks of Algorithm 1 -- causal target M_p and bidirectional, time-conditioned
diffusion drafter M_q -- as plain fp64 numpy.  Test infrastructure only.

The paper names the models (GPT-2 XL / GPT-Neo / Vicuna targets, MDLM drafter; Section
"Experimental Setup") but not their arithmetic, so the shapes follow the benchmark
configurations and the arithmetic follows the public definitions of those families:

  gpt2 : h = wte[tok] + wpe[pos] (+ temb(t) for the drafter);  per layer
         h += W_o attn(LN1 h) + b_o ;  h += W_proj gelu_tanh(W_fc LN2 h + b_fc) + b_proj ;
         logits = W_head LN_f h.     LayerNorm with biased variance, eps inside the sqrt.
  llama: h = wte[tok]; per layer h += W_o attn(rope(RMS1 h)); h += W_proj(silu(W_gate x) * W_up x),
         x = RMS2 h; grouped-query attention; rotary pairs (i, i + d_head/2).
  drafter timestep embedding: s_i = sin(1000 t f_i), s_{i+d/2} = cos(1000 t f_i),
         f_i = 10000^(-2i/d), temb = W_t2 silu(W_t1 s + b_t1) + b_t2, added to every row.

All weights arrive as the stored values (already rounded to the storage type) and are
promoted to fp64; every product, statistic and softmax is fp64.  One sequence at a time,
full recompute, no cache, no blocking.
"""
import numpy as np


def f64(x):
    return np.asarray(x, dtype=np.float64)


def layer_norm(x, gain, bias, eps):
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    return (x - mu) / np.sqrt(var + eps) * f64(gain) + f64(bias)


def rms_norm(x, gain, eps):
    ms = (x ** 2).mean(axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * f64(gain)


def gelu_tanh(x):
    return 0.5 * x * (1.0 + np.tanh(np.sqrt(2.0 / np.pi) * (x + 0.044715 * x ** 3)))


def silu(x):
    return x / (1.0 + np.exp(-x))


def softmax_rows(x):
    z = x - x.max(axis=-1, keepdims=True)
    e = np.exp(z)
    return e / e.sum(axis=-1, keepdims=True)


def linear(x, W, bias=None):
    """y = x W^T + bias with W stored [out_features, in_features]."""
    y = f64(x) @ f64(W).T
    return y if bias is None else y + f64(bias)


def rope(x, positions, theta):
    """x: [S, n_head, d_head]; rotates the pair (i, i + d_head/2) by positions * theta^(-2i/d_head)."""
    half = x.shape[-1] // 2
    inv = theta ** (-np.arange(half, dtype=np.float64) * 2.0 / x.shape[-1])
    ang = f64(positions)[:, None] * inv[None, :]            # [S, half]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    a, b = x[..., :half], x[..., half:]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


def attention(q, k, v, causal):
    """q: [S, H, dh]; k, v: [S, Hkv, dh] -> [S, H*dh].  Query head h uses kv head h // (H/Hkv)."""
    S, H, dh = q.shape
    group = H // k.shape[1]
    out = np.empty((S, H, dh), dtype=np.float64)
    for h in range(H):
        kh, vh = k[:, h // group, :], v[:, h // group, :]
        scores = q[:, h, :] @ kh.T / np.sqrt(dh)
        if causal:
            scores = np.where(np.tril(np.ones((S, S), dtype=bool)), scores, -np.inf)
        out[:, h, :] = softmax_rows(scores) @ vh
    return out.reshape(S, H * dh)


def timestep_embedding(W, cfg, t):
    d = cfg.d_model
    half = d // 2
    freq = 10000.0 ** (-2.0 * np.arange(half, dtype=np.float64) / d)
    s = np.concatenate([np.sin(1000.0 * t * freq), np.cos(1000.0 * t * freq)])
    hid = silu(f64(W["t_w1"]) @ s + f64(W["t_b1"]))
    return f64(W["t_w2"]) @ hid + f64(W["t_b2"])


def hidden_states(W, cfg, tokens, t=None):
    """Final-norm hidden states [S, d] of one sequence.  tokens may contain the mask id
    (== cfg.vocab) when cfg.bidirectional.  t in (0, 1] is the drafter's diffusion time."""
    tokens = np.asarray(tokens, dtype=np.int64)
    S = tokens.size
    pos = np.arange(S)
    H, Hkv, dh = cfg.n_head, cfg.n_kv_head, cfg.d_model // cfg.n_head
    causal = not cfg.bidirectional
    h = f64(W["wte"])[tokens]
    if cfg.arch == "gpt2":
        h = h + f64(W["wpe"])[pos]
    if cfg.bidirectional:
        h = h + timestep_embedding(W, cfg, t)[None, :]
    for i in range(cfg.n_layer):
        p = f"l{i}."
        if cfg.arch == "gpt2":
            x = layer_norm(h, W[p + "ln1_g"], W[p + "ln1_b"], cfg.norm_eps)
            qkv = x @ f64(W[p + "w_qkv"]).T + f64(W[p + "b_qkv"])
        else:
            x = rms_norm(h, W[p + "ln1_g"], cfg.norm_eps)
            qkv = x @ f64(W[p + "w_qkv"]).T
        dq, dkv = H * dh, Hkv * dh
        q = qkv[:, :dq].reshape(S, H, dh)
        k = qkv[:, dq:dq + dkv].reshape(S, Hkv, dh)
        v = qkv[:, dq + dkv:].reshape(S, Hkv, dh)
        if cfg.arch == "llama":
            q, k = rope(q, pos, cfg.rope_theta), rope(k, pos, cfg.rope_theta)
        a = attention(q, k, v, causal)
        if cfg.arch == "gpt2":
            h = h + a @ f64(W[p + "w_o"]).T + f64(W[p + "b_o"])
            x = layer_norm(h, W[p + "ln2_g"], W[p + "ln2_b"], cfg.norm_eps)
            m = gelu_tanh(x @ f64(W[p + "w_fc"]).T + f64(W[p + "b_fc"]))
            h = h + m @ f64(W[p + "w_proj"]).T + f64(W[p + "b_proj"])
        else:
            h = h + a @ f64(W[p + "w_o"]).T
            x = rms_norm(h, W[p + "ln2_g"], cfg.norm_eps)
            m = silu(x @ f64(W[p + "w_gate"]).T) * (x @ f64(W[p + "w_up"]).T)
            h = h + m @ f64(W[p + "w_proj"]).T
    if cfg.arch == "gpt2":
        return layer_norm(h, W["lnf_g"], W["lnf_b"], cfg.norm_eps)
    return rms_norm(h, W["lnf_g"], cfg.norm_eps)


def logits_at(W, cfg, tokens, rows, t=None):
    """Logits [len(rows), vocab] at the given positions of one sequence."""
    hs = hidden_states(W, cfg, tokens, t)
    return hs[np.asarray(rows, dtype=np.int64)] @ f64(W["w_head"]).T
