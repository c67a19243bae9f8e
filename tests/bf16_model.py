"""Test-side model of what bf16 storage does to the two networks: the oracle's forward with every activation that a
bf16 pipeline keeps in memory rounded to bf16 at that point, and fp32 arithmetic in between.

Why it exists.  The workload definition states the bf16 logit tolerance as an absolute number (2e-2), which fits the
logit scale of the GPT-2-small-shaped pair (random-init logit rms about 0.55).  The error of a pipeline that stores
its activations in bf16 is a *relative* error (2^-9 per stored value) that propagates to the logits in proportion to
their scale and grows with depth, so wide and deep random-init models (logit rms 0.8 at d = 1600, 1.3 at d = 4096)
exceed 2e-2 by construction, not by a defect.  This module predicts that error from first principles -- independent of
the HIP kernels -- so that the GPU tests can hold the kernels to `what bf16 storage costs` instead of to a blanket
percentage: a test computes sigma = rms(model - oracle) on the very inputs it runs and requires
rms(gpu - oracle) <= 1.3 sigma and max |gpu - oracle| <= max(2e-2, 6.5 sigma) (6.5 sigma: the largest of 10^6 - 10^7
near-Gaussian errors sits at 5 - 5.5 sigma).

Storage points (where a value is rounded to bf16), per layer: the operand of a normalised contraction
x = bf16(h * gain) -- the normalisation's mean and variance are taken from the fp32 residual stream h and applied after
the contraction: y = rstd (x W^T - mu (W gain)) + (W beta + bias) --, the QKV output, rotated q and k (rotary models), the
softmax numerators exp(s - max), the attention output, the MLP hidden activation (after GELU; gate/up and silu(gate) * up
for SwiGLU), and once more the operand of the LM head after the final normalisation.  The residual stream, the
accumulators and the logits are fp32.  With `rounding=False` nothing is rounded and the model is the oracle's network in
fp32 (pinned against the oracle in the CPU tests).

Uses numpy only; shares no code with the library and none with the oracle.
"""
import numpy as np


def bf16(x):
    """Round fp32 values to the nearest bf16 (ties to even), returned as fp32."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + r) & np.uint32(0xFFFF0000)).view(np.float32)


class Bf16Model:
    def __init__(self, W, cfg, rounding=True):
        self.W, self.c = W, cfg
        self.rd = bf16 if (rounding and cfg.dtype == "bf16") else (lambda x: np.asarray(x, dtype=np.float32))
        self.count = 0          # storage points passed (for the tests)

    def store(self, x):
        self.count += 1
        return self.rd(x)

    def w(self, name):
        return np.asarray(self.W[name], dtype=np.float32)

    def attention(self, q, k, v, causal):
        S, H, dh = q.shape
        group = H // k.shape[1]
        out = np.empty((S, H, dh), dtype=np.float32)
        mask = np.tril(np.ones((S, S), dtype=bool)) if causal else None
        for hh in range(H):
            kh, vh = k[:, hh // group], v[:, hh // group]
            s = (q[:, hh] @ kh.T) * np.float32(1.0 / np.sqrt(dh))
            if causal:
                s = np.where(mask, s, -np.inf)
            e = np.exp(s - s.max(axis=1, keepdims=True))
            out[:, hh] = (self.store(e) @ vh) / e.sum(axis=1, keepdims=True)
        return out.reshape(S, H * dh)

    def hidden(self, tokens, t=None):
        c, W = self.c, self.W
        tokens = np.asarray(tokens, dtype=np.int64)
        S = tokens.size
        pos = np.arange(S)
        H, Hkv, dh, F = c.n_head, c.n_kv_head, c.d_model // c.n_head, c.d_ff
        dq, dkv = H * dh, Hkv * dh
        h = self.w("wte")[tokens]
        if c.arch == "gpt2":
            h = h + self.w("wpe")[pos]
        if c.bidirectional:
            d = c.d_model
            f = 10000.0 ** (-2.0 * np.arange(d // 2, dtype=np.float64) / d)
            s = np.concatenate([np.sin(1000.0 * t * f), np.cos(1000.0 * t * f)])
            a = self.w("t_w1").astype(np.float64) @ s + self.w("t_b1")
            hid = a / (1.0 + np.exp(-a))
            h = h + (self.w("t_w2").astype(np.float64) @ hid + self.w("t_b2")).astype(np.float32)[None, :]
        h = h.astype(np.float32)
        if c.arch == "llama":
            inv = c.rope_theta ** (-np.arange(dh // 2, dtype=np.float64) * 2.0 / dh)
            ang = pos[:, None] * inv[None, :]
            cs, sn = np.cos(ang)[:, None, :].astype(np.float32), np.sin(ang)[:, None, :].astype(np.float32)

            def rope(x):
                a, b = x[..., :dh // 2], x[..., dh // 2:]
                return self.store(np.concatenate([a * cs - b * sn, b * cs + a * sn], axis=-1))
        for i in range(c.n_layer):
            p = f"l{i}."
            gpt2 = c.arch == "gpt2"
            qkv = self.store(self.normed_linear(h, p + "ln1_g", p + "ln1_b" if gpt2 else None, p + "w_qkv", p + "b_qkv" if gpt2 else None))
            q = qkv[:, :dq].reshape(S, H, dh)
            k = qkv[:, dq:dq + dkv].reshape(S, Hkv, dh)
            v = qkv[:, dq + dkv:].reshape(S, Hkv, dh)
            if not gpt2:
                q, k = rope(q), rope(k)
            att = self.store(self.attention(q, k, v, not c.bidirectional))
            h = h + att @ self.w(p + "w_o").T + (self.w(p + "b_o") if gpt2 else np.float32(0))
            if gpt2:
                m = self.normed_linear(h, p + "ln2_g", p + "ln2_b", p + "w_fc", p + "b_fc")
                m = self.store(0.5 * m * (1.0 + np.tanh(np.float32(np.sqrt(2.0 / np.pi)) * (m + np.float32(0.044715) * m ** 3))))
                h = h + m @ self.w(p + "w_proj").T + self.w(p + "b_proj")
            else:
                g = self.store(self.normed_linear(h, p + "ln2_g", None, p + "w_gate", None))
                up = self.store(self.normed_linear_reuse(p + "w_up"))
                act = self.store(g / (1.0 + np.exp(-g)) * up)
                h = h + act @ self.w(p + "w_proj").T
            h = h.astype(np.float32)
        return h

    def normed_linear(self, h, gain, beta, Wm, bias):
        """y = W norm(h) + bias with the operand x = bf16(h gain) and the statistics applied after the contraction."""
        y, self._last = self._normed_linear(h, gain, beta, Wm, bias)
        return y

    # the gate and up projections share their operand and statistics (one contraction in the pipeline)
    def normed_linear_reuse(self, Wm):
        x, rstd = self._last
        return ((x @ self.w(Wm).T).astype(np.float64) * rstd).astype(np.float32)

    def _normed_linear(self, h, gain, beta, Wm, bias):
        c = self.c
        g = self.w(gain)
        x = self.store(h * g)
        h64 = h.astype(np.float64)
        if c.arch == "gpt2":
            mu = h64.mean(axis=1, keepdims=True)
            var = np.maximum((h64 ** 2).mean(axis=1, keepdims=True) - mu ** 2, 0.0)
            rstd = 1.0 / np.sqrt(var + c.norm_eps)
            Wf = self.w(Wm)
            u = Wf.astype(np.float64) @ g.astype(np.float64)
            v = Wf.astype(np.float64) @ self.w(beta).astype(np.float64)
            if bias is not None:
                v = v + self.w(bias)
            acc = (x @ Wf.T).astype(np.float64)
            return (rstd * (acc - mu * u[None, :]) + v[None, :]).astype(np.float32), (x, rstd)
        rstd = 1.0 / np.sqrt((h64 ** 2).mean(axis=1, keepdims=True) + c.norm_eps)
        return ((x @ self.w(Wm).T).astype(np.float64) * rstd).astype(np.float32), (x, rstd)

    def logits_at(self, tokens, rows, t=None):
        c = self.c
        h = self.hidden(tokens, t)[np.asarray(rows, dtype=np.int64)]
        return self.normed_linear(h, "lnf_g", "lnf_b" if c.arch == "gpt2" else None, "w_head", None)


def logits_at(W, cfg, tokens, rows, t=None, rounding=True):
    return Bf16Model(W, cfg, rounding).logits_at(tokens, rows, t).astype(np.float64)


def predicted_sigma(model_logits, oracle_logits):
    e = np.asarray(model_logits, dtype=np.float64) - np.asarray(oracle_logits, dtype=np.float64)
    return float(np.sqrt((e ** 2).mean()))
