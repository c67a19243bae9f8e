"""Benchmark of one SpecDiff draft-then-verify round on one MI355X.

A step is one whole round (sd_round): T drafter evaluations with their vocabulary softmax and
reveal/sampling step, one target evaluation against its KV cache, acceptance and residual
resampling.  Inputs (weights, KV cache of the prefix, prefix tokens) are resident in HBM before
the timed region; each step uploads ~1 KB of token ids / row maps and reads back gamma + 2 ints.

The headline workload is the largest single-GPU configuration (`llama8b`: Llama-3-8B-shaped target,
12-layer d=768 drafter, vocabulary 128256, prefix 1024, gamma 32, T 8, one sequence).  Prints ONE
JSON line: verified tokens/s of that workload, the roofline fraction of its dominant kernel (kernel
execution times from HIP events stamped by the launches themselves, in an instrumented pass over the
same steps), the CPU oracle's rate on a bounded sample of the same workload, and -- under
`configs` -- round latency, tokens/s, acceptance and round-roofline fraction of the other workloads.
"""
import argparse
import json
import os
import platform
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0
PEAK_MFMA_TFLOPS = {"bf16": 2500.0, "f32": 157.3}
EXTRA_WORKLOADS = ["tiny", "gpt2s", "gpt2xl", "gpt2xl_b16", "llama8b_b8"]


def log(msg):
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def prefixes_for(w, seed):
    from paper_2408_05636_amd import synth
    V = w["target"].vocab
    if isinstance(w["prefix_len"], tuple):
        lens = synth.gen_prefix_lengths(w["batch"], w["prefix_len"][0], w["prefix_len"][1], seed)
    else:
        lens = [w["prefix_len"]] * w["batch"]
    return [synth.gen_prefix(V, int(L), seed + 1 + i) for i, L in enumerate(lens)]


def layer_params(c):
    d, F, dkv = c.d_model, c.d_ff, c.d_kv
    return d * (d + 2 * dkv) + d * d + (3 if c.arch == "llama" else 2) * d * F


def round_roofline(w, lens):
    """Time of one round at the peaks: T x max(HBM, matrix cores) of a drafter step + the same for the target pass.
    Bytes: weights once (2 B per parameter, 4 B for the fp32 workload), the target's KV cache once, fp32 logits
    written; flops: 2 x rows x parameters + 4 x rows x keys x d per attention layer.  Returns microseconds."""
    t, d, gamma, T = w["target"], w["drafter"], w["gamma"], w["T"]
    ew = 2 if t.dtype == "bf16" else 4
    peak = PEAK_MFMA_TFLOPS[t.dtype] * 1e12
    B = len(lens)
    rows_t = B * (gamma + 1)
    p_t = layer_params(t) * t.n_layer
    by_t = ew * (p_t + t.vocab * t.d_model) + sum(2 * L * t.d_kv * ew * t.n_layer for L in lens) + rows_t * t.vocab * 4
    fl_t = 2 * rows_t * (p_t + t.vocab * t.d_model) + sum(4 * (gamma + 1) * (L + gamma) * t.d_model * t.n_layer for L in lens)
    rows_d = sum(L + gamma for L in lens)
    p_d = layer_params(d) * d.n_layer
    by_d = ew * (p_d + d.vocab * d.d_model) + B * gamma * d.vocab * 4
    fl_d = 2 * rows_d * p_d + 2 * B * gamma * d.vocab * d.d_model + sum(4 * (L + gamma) ** 2 * d.d_model * d.n_layer for L in lens)
    t_t = max(by_t / (PEAK_HBM_GBS * 1e9), fl_t / peak)
    t_d = max(by_d / (PEAK_HBM_GBS * 1e9), fl_d / peak)
    return (T * t_d + t_t) * 1e6, {"target_us": t_t * 1e6, "target_bound": "hbm" if by_t / (PEAK_HBM_GBS * 1e9) >= fl_t / peak else "mfma",
                                   "drafter_step_us": t_d * 1e6, "drafter_bound": "hbm" if by_d / (PEAK_HBM_GBS * 1e9) >= fl_d / peak else "mfma"}


def accept_micro(torch, binding, vocab, gamma, batch):
    """The accept / residual-sampling kernels alone, on synthetic rows whose agreement is controlled:
    q = (1 - lam) p + lam noise, x_k ~ q_k.  lam = 0.15: most positions accepted; lam = 1: early rejections.
    Returns per lam: mean accepted count, microseconds per call (HIP events around 20 calls on one stream) and the
    algorithmic bytes behind them ((gamma + 1) V fp32 for the row statistics and the tests, 4 V fp32 for the two passes
    over row n of p and q)."""
    ld = binding.sd_vocab_pad(vocab)
    rows = batch * (gamma + 1)
    g = torch.Generator(device="cuda:0").manual_seed(7)
    p_logits = torch.zeros(rows, ld, device="cuda:0")
    p_logits[:, :vocab] = torch.randn(rows, vocab, device="cuda:0", generator=g) * 1.5
    P = torch.softmax(p_logits[:, :vocab].double(), dim=1).view(batch, gamma + 1, vocab)
    out = {}
    for lam in (0.15, 1.0):
        noise = torch.softmax(torch.randn(batch, gamma, vocab, device="cuda:0", generator=g).double() * 1.5, dim=2)
        q = ((1 - lam) * P[:, :gamma] + lam * noise).float()
        draft = torch.multinomial(q.view(-1, vocab), 1, generator=g).view(batch, gamma).int()
        qp = torch.zeros(batch * gamma, ld, device="cuda:0")
        qp[:, :vocab] = q.view(-1, vocab)
        nb = binding.sd_sampling_scratch_bytes(rows, vocab)
        scratch = torch.empty(nb, dtype=torch.uint8, device="cuda:0")
        n = torch.zeros(batch, dtype=torch.int32, device="cuda:0")
        tok = torch.zeros(batch, dtype=torch.int32, device="cuda:0")
        st = torch.cuda.current_stream().cuda_stream
        call = lambda seed: binding.lib().sd_accept_resample(p_logits.data_ptr(), qp.data_ptr(), draft.data_ptr(), batch, gamma, vocab,
                                                             seed, n.data_ptr(), tok.data_ptr(), scratch.data_ptr(), nb, st)
        acc = 0
        for seed in range(3):
            assert call(seed) == 0
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for seed in range(20):
            assert call(100 + seed) == 0
        e1.record()
        torch.cuda.synchronize()
        for seed in range(20):                                    # accepted counts (outside the timed calls)
            call(100 + seed)
            torch.cuda.synchronize()
            acc += int(n.sum())
        us = e0.elapsed_time(e1) * 1e3 / 20
        nbytes = batch * ((gamma + 1) * vocab * 4 + 4 * vocab * 4)
        out[f"lam={lam}"] = {"mean_accepted": acc / (20 * batch), "us_per_call": round(us, 2), "algorithmic_MB": round(nbytes / 1e6, 2),
                             "GB_per_s": round(nbytes / us / 1e3, 1)}
    return out


def cpu_info():
    model = platform.processor() or ""
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                model = line.split(":", 1)[1].strip()
                break
    except OSError:
        pass
    try:
        usable = len(os.sched_getaffinity(0))
    except AttributeError:
        usable = os.cpu_count() or 1
    return model, usable


def cpu_baseline(w, Wt, Wd, prefixes, seed, tokens_per_round):
    """The oracle as it stands on a bounded sample of the same workload.  Small models: one whole round of sequence 0.
    Large targets (more than 8 layers): ONE of the T drafter evaluations and the target evaluation cut to its first
    2 layers (full width, full rows, full LM head) are timed, and the round is put together as
    T x drafter + (n_layer / 2) x two-layer time + embedding/head time; tokens per round are the ones the timed GPU
    rounds of this workload produced."""
    from threadpoolctl import threadpool_info
    from oracle import specdiff as osd
    from oracle import transformer as otf
    from paper_2408_05636_amd import synth
    t, d, gamma, T = w["target"], w["drafter"], w["gamma"], w["T"]
    p = prefixes[0]
    model, usable = cpu_info()
    if t.n_layer <= 12:
        t0 = time.perf_counter()
        dl = lambda tokens, tt: otf.logits_at(Wd, d, tokens, np.arange(len(tokens) - gamma, len(tokens)), tt)
        z, q, _, nf = osd.oracle_draft(dl, p, gamma, T, seed, t.vocab)
        tl = lambda tokens, rows: otf.logits_at(Wt, t, tokens, rows)
        n, tok, _, _ = osd.oracle_verify(tl, p, z, q, seed)
        dt = time.perf_counter() - t0
        value = (n + 1) / dt
        sample = (f"1 round of sequence 0 ({nf} drafter + 1 target fp64 forwards over {len(p) + gamma} tokens), "
                  f"{dt:.1f} s, {n + 1} tokens")
    else:
        block = np.full(gamma, t.vocab, dtype=np.int64)
        seq = np.concatenate([np.asarray(p, dtype=np.int64), block])
        t0 = time.perf_counter()
        lg = otf.logits_at(Wd, d, seq, np.arange(len(seq) - gamma, len(seq)), 1.0)
        osd.softmax_rows(lg)
        t_d = time.perf_counter() - t0
        toks = np.concatenate([np.asarray(p, dtype=np.int64), np.zeros(gamma, dtype=np.int64)])
        rows = np.arange(len(p) - 1, len(p) + gamma)
        cut0 = synth.shrink(t, n_layer=0)
        t0 = time.perf_counter()
        otf.logits_at(Wt, cut0, toks, rows)
        t_head = time.perf_counter() - t0                  # embedding, final norm, LM head on gamma + 1 rows
        cut2 = synth.shrink(t, n_layer=2)
        t0 = time.perf_counter()
        otf.hidden_states(Wt, cut2, toks)
        t_2 = time.perf_counter() - t0                     # embedding + 2 layers + final norm over all L + gamma rows
        est = T * t_d + t.n_layer / 2.0 * t_2 + t_head
        value = tokens_per_round / est
        sample = (f"sequence 0: one of the {T} drafter forwards ({t_d:.1f} s) + target cut to 2 of {t.n_layer} layers over "
                  f"{len(toks)} tokens ({t_2:.1f} s) + embedding/final norm/LM head on {gamma + 1} rows ({t_head:.1f} s); round put "
                  f"together as {T} x drafter + {t.n_layer}/2 x two-layer time + head = {est:.0f} s, {tokens_per_round:.2f} tokens per "
                  f"round as the timed GPU rounds produced")
    threads = max([i.get("num_threads", 1) for i in threadpool_info()] or [1])
    return {"value": value, "unit": "tokens/s", "cores": int(threads), "kind": "oracle", "sample": sample,
            "cpu_model": model, "cpus_usable": usable}


class Pair:
    """Weights of one (target, drafter) pair on the host (for the oracle) and on the device (kept across handles)."""
    cache = {}

    def __init__(self, synth, binding, torch, t, d, keep_host):
        self.t, self.d = t, d
        t0 = time.perf_counter()
        Wt, Wd = synth.gen_weights(t, 1, threads=16), synth.gen_weights(d, 2, threads=16)
        log(f"weights of {t.n_layer}L d={t.d_model} target + drafter generated in {time.perf_counter() - t0:.1f} s; packing and uploading")
        dev = torch.device("cuda:0")
        self.tw = torch.from_numpy(binding.pack_weights(t, Wt)).to(dev)
        self.dw = torch.from_numpy(binding.pack_weights(d, Wd)).to(dev)
        self.Wt, self.Wd = (Wt, Wd) if keep_host else (None, None)

    @classmethod
    def get(cls, synth, binding, torch, t, d, keep_host=False):
        key = (t, d)
        if key not in cls.cache:
            cls.cache.clear()                              # one pair resident at a time
            cls.cache[key] = cls(synth, binding, torch, t, d, keep_host)
        return cls.cache[key]


def time_rounds(sd, flat, lens, gamma, T, B, steps, warmup, torch):
    for i in range(warmup):
        sd.sd_round_flat(flat, lens, gamma, T, 100 + i)
    torch.cuda.synchronize()
    g0 = sd.sd_graph_stats()
    tokens = accepted = 0
    n_hist = []
    t0 = time.perf_counter()
    for i in range(steps):
        _, n, _ = sd.sd_round_flat(flat, lens, gamma, T, 1000 + i)
        tokens += int(n.sum()) + B
        accepted += int(n.sum())
        n_hist.extend(n.tolist())
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    g1 = sd.sd_graph_stats()
    # the timed rounds must have run as graph replays: a failed capture falls back to eager launches, which are
    # correct but several times slower
    assert g1["failures"] == 0 and g1["replays"] - g0["replays"] == steps, f"timed rounds did not run as graph replays: {g0} -> {g1}"
    tested = sum(min(int(x) + 1, gamma) for x in n_hist)
    return dict(dt=dt, tokens=tokens, accepted=accepted, alpha_hat=accepted / max(tested, 1))


def run_workload(name, a, torch, binding, synth, headline):
    w = synth.workload(name)
    if headline and a.gamma:
        w["gamma"] = a.gamma
    if headline and a.T:
        w["T"] = a.T
    t, d, gamma, T, B = w["target"], w["drafter"], w["gamma"], w["T"], w["batch"]
    steps = a.steps if headline else min(a.steps, 12)
    warmup = a.warmup if headline else min(a.warmup, 3)
    pair = Pair.get(synth, binding, torch, t, d, keep_host=headline and not a.no_cpu_baseline)
    sd = binding.SpecDiff(t, d, None, None, max_batch=B, gamma_max=gamma, device_weights=(pair.tw, pair.dw))
    if headline and a.greedy:
        sd.sd_set_greedy(True)
    prefixes = prefixes_for(w, 3)
    flat, lens = binding._ragged(prefixes)
    sd.sd_prefill(prefixes)                       # prompt processing: outside the round
    log(f"{name}: prefill done; timing {steps} rounds")
    r = time_rounds(sd, flat, lens, gamma, T, B, steps, warmup, torch)
    ms = r["dt"] / steps * 1e3
    roof_us, roof_parts = round_roofline(w, [int(x) for x in lens])
    alpha_paper = 0.78
    per_round = (1.0 - alpha_paper ** (gamma + 1)) / (1.0 - alpha_paper)
    res = {
        "workload": f"{name}: one SpecDiff round, target {t.n_layer}L d={t.d_model} V={t.vocab}, drafter {d.n_layer}L d={d.d_model}, "
                    f"prefix {[int(x) for x in lens][:4]}{'...' if B > 4 else ''}, gamma={gamma}, T={T}, batch={B}, random-init weights"
                    + (", temperature 0" if headline and a.greedy else ""),
        "dtype": t.dtype, "steps": steps, "round_latency_us": ms * 1e3, "tokens_per_s": r["tokens"] / r["dt"],
        "mean_accepted_per_round": r["accepted"] / (steps * B), "alpha_hat": r["alpha_hat"],
        "round_roofline_us": roof_us, "roofline_parts": roof_parts,
        "frac_of_round_roofline": None if name == "tiny" else roof_us / (ms * 1e3),
    }
    log(f"{name}: {ms:.3f} ms per round, {res['tokens_per_s']:.1f} tok/s, roofline {roof_us:.0f} us")
    if name == "gpt2xl" and not (headline and a.greedy):
        res["sps"] = sps_comparison(sd, synth, binding, torch, w, flat, lens, steps, warmup, res)
    if B == 1 and name != "tiny" and not a.no_autoregressive:
        res["autoregressive"] = autoregressive_baseline(binding, torch, pair, w, prefixes, steps, warmup, res, alpha_paper, per_round)
    if not headline:
        sd.close()
        return res, None
    res["acceptance"] = {"alpha_hat": r["alpha_hat"], "mean_tokens_per_round": r["tokens"] / (steps * B),
                         # context only: the rate this latency would give at an acceptance rate the paper reports for a trained
                         # pair (vanilla SpecDiff, GPT-2 XL / MDLM on OpenWebText: alpha = 0.78), expected tokens by Appendix A Eq. (2)
                         "context_only": {"alpha": alpha_paper, "expected_tokens_per_round": per_round,
                                          "tokens_per_s_at_this_latency": B * per_round / (ms * 1e-3)}}
    if a.copy_probe:
        src = torch.ones(16 << 20, dtype=torch.float32, device="cuda:0")     # 64 MiB read, 64 MiB written
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        torch.neg(src, out=dst)                                              # one elementwise kernel ("neg")
        torch.cuda.synchronize()
    ctx = dict(sd=sd, w=w, pair=pair, prefixes=prefixes, flat=flat, lens=lens, steps=steps, warmup=warmup, tokens=r["tokens"], ms=ms)
    return res, ctx


def autoregressive_baseline(binding, torch, pair, w, prefixes, steps, warmup, res, alpha_paper, per_round_paper):
    """Plain autoregressive decoding with the target alone, on the same kernels: the target is attached to a second handle
    as the one-token-per-step model of sd_sps_draft (causal, incremental KV cache), which then produces tokens one forward
    at a time from the same prefix.  The paper's speed-ups (Tables 2, 3) are quoted against this; reported here: time per
    token, SpecDiff's tokens/s over it at the acceptance the random-init pair happens to have, and -- context only -- at an
    acceptance rate the paper reports for a trained pair."""
    t, d, gamma = w["target"], w["drafter"], w["gamma"]
    n_tok = min(gamma, 16)
    ar = binding.SpecDiff(t, d, None, None, max_batch=1, gamma_max=n_tok, device_weights=(pair.tw, pair.dw))
    ar.sd_sps_attach(t, device_weights=pair.tw)
    for i in range(warmup):
        ar.sd_sps_draft(prefixes, n_tok, 100 + i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        ar.sd_sps_draft(prefixes, n_tok, 1000 + i)
    torch.cuda.synchronize()
    us = (time.perf_counter() - t0) / (steps * n_tok) * 1e6
    ar.close()
    out = {"us_per_token": us, "tokens_per_s": 1e6 / us, "tokens_per_call": n_tok,
           "specdiff_over_autoregressive": res["tokens_per_s"] * us * 1e-6,
           "context_only": {"alpha": alpha_paper, "specdiff_over_autoregressive": per_round_paper / (res["round_latency_us"] / us),
                            "paper": "speed-ups over autoregressive decoding of 3.8-7.2x (T = 2, gamma 10-20, trained pairs, 2x A100-80GB)"}}
    log(f"autoregressive decoding with the target alone: {us:.0f} us per token; SpecDiff / autoregressive = {out['specdiff_over_autoregressive']:.2f}")
    return out


def sps_comparison(sd, synth, binding, torch, w, flat, lens, steps, warmup, res):
    """Standard speculative decoding on the same target and prefix: an autoregressive GPT-2-small-shaped drafter (12
    layers, d = 768, causal, random-init) produces the draft tokens one after the other (sd_sps_round).  Reported: round
    latency and verified tokens/s at the draft length the paper's SpS rows use for this target (gamma = 8) and at the
    SpecDiff round's own gamma, and the ratio of SpecDiff's tokens/s to SpS's best.  Both drafters are random-init, so the
    acceptance rates are whatever they are; the paper's 1.45-1.75x is for trained pairs (context only)."""
    t, gamma, T, B = w["target"], w["gamma"], w["T"], w["batch"]
    s_cfg = synth.gpt2_shape(t.dtype, 12, 768, 12, 3072, t.vocab, t.n_ctx, False)
    sd.sd_sps_attach(s_cfg, synth.gen_weights(s_cfg, 4, threads=16))
    out = {}
    for g in sorted({min(8, gamma), gamma}):
        for i in range(warmup):
            sd.sd_sps_round_flat(flat, lens, g, 100 + i)
        torch.cuda.synchronize()
        tokens = 0
        t0 = time.perf_counter()
        for i in range(steps):
            _, n, _ = sd.sd_sps_round_flat(flat, lens, g, 1000 + i)
            tokens += int(n.sum()) + B
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        out[f"gamma={g}"] = {"round_latency_us": dt / steps * 1e6, "tokens_per_s": tokens / dt, "mean_tokens_per_round": tokens / (steps * B)}
    best = max(v["tokens_per_s"] for v in out.values())
    out["specdiff_over_sps_tokens_per_s"] = res["tokens_per_s"] / best
    out["specdiff_over_sps_round_latency_at_equal_gamma"] = out[f"gamma={gamma}"]["round_latency_us"] / res["round_latency_us"]
    out["paper_context"] = "SpecDiff 1.45-1.75x over SpS with trained drafters on 2x A100-80GB (Table 2)"
    log(f"SpS on the same target: {out}")
    return out


def step_skipping_pass(ctx, torch):
    sd, w, flat, lens, steps, warmup = ctx["sd"], ctx["w"], ctx["flat"], ctx["lens"], ctx["steps"], ctx["warmup"]
    gamma, T, B = w["gamma"], w["T"], w["batch"]
    sd.sd_set_step_skipping(True)
    for i in range(warmup):
        sd.sd_round_flat(flat, lens, gamma, T, 100 + i)
    for i in range(steps):                              # every step's launch sequence seen, captured and replayed
        sd.sd_round_flat(flat, lens, gamma, T, 1000 + i)
    torch.cuda.synchronize()
    tok2 = steps_run = 0
    t1 = time.perf_counter()
    for i in range(steps):
        _, n, _ = sd.sd_round_flat(flat, lens, gamma, T, 1000 + i)
        tok2 += int(n.sum()) + B
        steps_run += sd.sd_steps_run()
    torch.cuda.synchronize()
    dt2 = time.perf_counter() - t1
    sd.sd_set_step_skipping(False)
    assert tok2 == ctx["tokens"], "step skipping changed the outcome of a round"
    return {"value": tok2 / dt2, "unit": "tokens/s", "ms_per_step": dt2 / steps * 1e3,
            "mean_drafter_forwards_per_round": steps_run / steps, "of": T}


def profile_pass(ctx, dtype):
    """Kernel execution times per kernel name (HIP events stamped with each kernel's own start and end), the roofline
    of the dominant kernel, and the parts of the round -- which, with the time the GPU spent between kernels, add up
    to the timed round."""
    sd, w, flat, lens, steps = ctx["sd"], ctx["w"], ctx["flat"], ctx["lens"], ctx["steps"]
    gamma, T = w["gamma"], w["T"]
    sd.sd_profile_begin()
    for i in range(steps):
        sd.sd_round_flat(flat, lens, gamma, T, 1000 + i)
    prof = sd.sd_profile_end()
    prof.sort(key=lambda e: -e["ms"])
    total = sum(e["ms"] for e in prof)
    for e in prof:                                    # entry names are "<part of the round>:<kernel>"
        e["phase"], _, e["name"] = e["name"].rpartition(":")
    kernels = [{"phase": e["phase"], "kernel": e["name"], "launches_per_step": e["launches"] / steps,
                "us_per_launch": round(1e3 * e["ms"] / e["launches"], 3), "share": round(e["ms"] / total, 4)} for e in prof]
    peak_f = PEAK_MFMA_TFLOPS[dtype]
    phases = {}
    for ph in ("draft", "verify", "accept"):
        es = [e for e in prof if e["phase"] == ph]
        if not es:
            continue
        us = 1e3 * sum(e["ms"] for e in es) / steps
        by = sum(e["bytes"] for e in es) / steps
        fl = sum(e["flops"] for e in es) / steps
        t_hbm, t_mfma = by / (PEAK_HBM_GBS * 1e9) * 1e6, fl / (peak_f * 1e12) * 1e6
        phases[ph] = {"kernel_us": round(us, 1), "launches": sum(e["launches"] for e in es) / steps, "algorithmic_MB": round(by / 1e6, 1),
                      "GFLOP": round(fl / 1e9, 2), "us_at_hbm_peak": round(t_hbm, 1), "us_at_mfma_peak": round(t_mfma, 1),
                      "bound": "hbm" if t_hbm >= t_mfma else "mfma", "frac_of_roofline": round(max(t_hbm, t_mfma) / us, 4)}
    kernel_us = sum(p["kernel_us"] for p in phases.values())
    # what is left of the timed (graph-replayed) round: the gaps between dependent kernels, the uploads and the read-back
    phases["between_kernels_and_host"] = {"us": round(ctx["ms"] * 1e3 - kernel_us, 1)}
    phases["sum_us"] = round(ctx["ms"] * 1e3, 1)
    # Dominant kernel = largest share of the kernel time; a launcher that starts several kernels counts as one entry.
    e = prof[0]
    us = 1e3 * e["ms"] / e["launches"]
    gbs = e["bytes"] / e["launches"] / (us * 1e-6) / 1e9
    tfl = e["flops"] / e["launches"] / (us * 1e-6) / 1e12
    if gbs / PEAK_HBM_GBS >= tfl / peak_f:
        roof = {"kernel": e["name"], "bound": "hbm", "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "frac": gbs / PEAK_HBM_GBS, "traffic": None}
    else:
        roof = {"kernel": e["name"], "bound": "mfma", "achieved": tfl, "peak": peak_f, "unit": "TFLOP/s",
                "frac": tfl / peak_f, "traffic": None}
    roof["part_of_round"] = e["phase"]
    roof["us_per_launch"] = us
    roof["algorithmic_bytes_per_launch"] = e["bytes"] / e["launches"]
    roof["flops_per_launch"] = e["flops"] / e["launches"]
    roof["timing"] = "kernel start/end time stamps (hipExtLaunchKernelGGL events) over the timed steps, eager launches"
    tr = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(tr):
        roof["traffic"] = json.load(open(tr)).get(ctx["name"], {}).get(e["name"])
    return roof, phases, kernels


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="llama8b")
    ap.add_argument("--gamma", type=int, default=0)
    ap.add_argument("--T", type=int, default=0)
    ap.add_argument("--greedy", action="store_true", help="temperature 0 (sd_set_greedy) instead of the stochastic rule")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-profile", action="store_true")
    ap.add_argument("--no-accept-micro", action="store_true", help="leave out the micro-benchmark of the accept / residual-sampling kernels")
    ap.add_argument("--no-step-skipping", action="store_true", help="leave out the extra timed pass with sd_set_step_skipping")
    ap.add_argument("--no-extras", action="store_true", help="only the headline workload, not the other configurations")
    ap.add_argument("--no-autoregressive", action="store_true", help="leave out the autoregressive-decoding reference (target alone, one token per forward)")
    ap.add_argument("--extras", default=",".join(EXTRA_WORKLOADS), help="comma-separated workloads reported under `configs`")
    ap.add_argument("--copy-probe", action="store_true", help="also launch one 64 MiB elementwise copy kernel, torch.neg (calibrates rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE)")
    a = ap.parse_args()
    if a.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2408_05636_amd import binding, synth

    t_start = time.perf_counter()
    res, ctx = run_workload(a.workload, a, torch, binding, synth, headline=True)
    ctx["name"] = a.workload
    sd, w = ctx["sd"], ctx["w"]
    t, gamma, B = w["target"], w["gamma"], w["batch"]

    skipping = None
    if not a.no_step_skipping:
        skipping = step_skipping_pass(ctx, torch)
        log(f"with step skipping: {skipping['ms_per_step']:.3f} ms per round, {skipping['mean_drafter_forwards_per_round']:.2f} of {w['T']} forwards")
    roof = phases = kernels = None
    if not a.no_profile:
        roof, phases, kernels = profile_pass(ctx, t.dtype)
        log(f"dominant kernel {roof['kernel']}: {roof['us_per_launch']:.2f} us per launch, {roof['frac']:.3f} of the {roof['bound']} peak")
    graphs = sd.sd_graph_stats()
    sd.close()

    cpu = None
    if not a.no_cpu_baseline and not a.greedy:
        cpu = cpu_baseline(w, ctx["pair"].Wt, ctx["pair"].Wd, ctx["prefixes"], 1000, ctx["tokens"] / (ctx["steps"] * B))
        log(f"cpu baseline: {cpu['value']:.4f} tok/s ({cpu['sample']})")
        ctx["pair"].Wt = ctx["pair"].Wd = None

    micro = None
    if not a.no_accept_micro:
        micro = accept_micro(torch, binding, t.vocab, gamma, B)
        log(f"accept kernels alone: {micro}")

    configs = {a.workload: {k: res[k] for k in ("round_latency_us", "tokens_per_s", "alpha_hat", "mean_accepted_per_round",
                                                "round_roofline_us", "frac_of_round_roofline")}}
    if not a.no_extras:
        for name in [x for x in a.extras.split(",") if x and x != a.workload]:
            if time.perf_counter() - t_start > 420:      # the whole run stays within minutes
                configs[name] = {"skipped": "time budget of the run"}
                continue
            r2, _ = run_workload(name, a, torch, binding, synth, headline=False)
            configs[name] = {k: r2[k] for k in ("workload", "round_latency_us", "tokens_per_s", "alpha_hat", "mean_accepted_per_round",
                                                 "round_roofline_us", "roofline_parts", "frac_of_round_roofline", "sps", "autoregressive") if k in r2}

    out = {
        "metric": "verified tokens/s", "value": res["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": ctx["steps"],
        "warmup": ctx["warmup"], "ms_per_step": ctx["ms"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": t.dtype, "data": "synthetic",
        "config": {"workload": res["workload"]},
        "round_latency_us": res["round_latency_us"],
        "mean_accepted_per_round": res["mean_accepted_per_round"],
        "acceptance": res["acceptance"],
        "round_roofline_us": res["round_roofline_us"], "roofline_parts": res["roofline_parts"],
        "frac_of_round_roofline": res["frac_of_round_roofline"],
        "autoregressive": res.get("autoregressive"),
        "roofline": roof, "cpu_baseline": cpu, "step_skipping": skipping, "accept_micro": micro, "phases": phases,
        "graph_replay": graphs, "configs": configs, "kernels": kernels,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
