"""One SpecDiff round -- Algorithm 1 of the paper -- as plain fp64 numpy / Python loops.
Test infrastructure only.

Algorithm 1 in the paper's order: (1) start the gamma-slot block from noise, (2) T reverse
diffusion steps t = T..1, each one evaluation of M_q on prefix o block, (3) the draft
tokens are sampled from q and q is kept, (4) M_p scores the gamma+1 prefixes in parallel,
(5) uniforms r are drawn and n = number of leading accepted tokens (reject when
r > p(x)/q(x)), (6) p' = p_{n+1}, replaced by norm(max(0, p_{n+1} - q_{n+1})) when a
rejection happened, (7) one token from p', return n draft tokens + that token.

Readings where the paper is silent or inconsistent (each also listed in the design notes):
  * the drafter is a *masked* diffusion model (Section 4.1), so the start state is an
    all-[MASK] block, not Gaussian noise;
  * reverse step j (time t = j/T, linear schedule alpha_t = 1 - t): every still-masked slot
    is revealed with probability 1/j, independently; a revealed slot draws its token from
    the softmax row M_q gives it at that step; revealed slots never change again
    (absorbing-state reverse process of masked diffusion); step j = 1 reveals all;
  * q_k is the row token k was drawn from (so that x_k ~ q_k, which the acceptance
    identity needs); q crosses the draft/verify boundary as fp32;
  * indices are relative: P[0..gamma], n in [0, gamma], residual iff n < gamma;
  * accept iff r * q(x) <= p(x), the product and the comparison in fp32;
  * sampling = inverse CDF over ascending token id with a strict '>' crossing;
  * a residual whose mass is zero (impossible in exact arithmetic) falls back to p.
"""
import numpy as np

from . import philox
from .transformer import softmax_rows


def invcdf(w, u):
    """Smallest v with sum_{v'<=v} w[v'] > u * sum(w).  Returns (v, margin): margin is the
    distance of u*sum(w) from the nearer edge of v's CDF interval, divided by sum(w) --
    how far the decision is from flipping to a neighbouring token."""
    c = np.cumsum(np.asarray(w, dtype=np.float64))
    total = c[-1]
    target = u * total
    v = int(np.searchsorted(c, target, side="right"))     # first index with c[v] > target
    if v >= c.size:                                        # rounding only
        v = int(np.flatnonzero(np.asarray(w) > 0)[-1])
    lo = c[v - 1] if v > 0 else 0.0
    margin = min(target - lo, c[v] - target) / total
    return v, float(margin)


def draft_with_uniforms(drafter_logits, prefix, gamma, T, ua, ub, mask_id, skip_when_done=True, skip_idle_steps=False):
    """Steps (1)-(3).  drafter_logits(tokens, t) -> [gamma, V] logits of the block rows for the
    sequence prefix o block.  ua, ub: [T+1, gamma] uniforms indexed [j, k] (row 0 unused).
    skip_idle_steps: also leave out the forward of a step at which no masked slot is revealed -- which
    slots a step reveals is decided by the uniforms alone, and the output of a step's forward is read
    by nothing but the slots revealed at that step, so z and q cannot depend on it.
    Returns (z int64[gamma], q fp32[gamma, V], margins fp64[gamma], n_forwards)."""
    prefix = np.asarray(prefix, dtype=np.int64)
    z = np.full(gamma, mask_id, dtype=np.int64)
    q = None
    margins = np.zeros(gamma)
    n_forwards = 0
    for j in range(T, 0, -1):
        masked = np.flatnonzero(z == mask_id)
        if masked.size == 0 and skip_when_done:
            continue                                   # nothing left to reveal: the step is a no-op
        if skip_idle_steps and not any(j == 1 or ua[j, k] * j < 1.0 for k in masked):
            continue                                   # nobody looks at this step's logits
        logits = np.asarray(drafter_logits(np.concatenate([prefix, z]), j / T), dtype=np.float64)
        n_forwards += 1
        if q is None:
            q = np.zeros((gamma, logits.shape[1]), dtype=np.float64)
        for k in masked:
            if j == 1 or ua[j, k] * j < 1.0:           # reveal with probability 1/j
                pi = softmax_rows(logits[k])
                z[k], margins[k] = invcdf(pi, ub[j, k])
                q[k] = pi
    return z, q.astype(np.float32), margins, n_forwards


def accept_flags(P, q, draft, r):
    """Step (5), per position: accept iff fl32(r * q_k(x_k)) <= fl32(p_k(x_k))."""
    gamma = len(draft)
    flags = np.zeros(gamma, dtype=bool)
    for k in range(gamma):
        px = np.float32(P[k][draft[k]])
        qx = np.float32(q[k][draft[k]])
        flags[k] = (np.float32(r[k]) * qx) <= px
    return flags


def accept_margins(P, q, draft, r):
    """Relative distance |r*q(x) - p(x)| / p(x) of every acceptance test from flipping."""
    out = np.zeros(len(draft))
    for k in range(len(draft)):
        px, qx = float(P[k][draft[k]]), float(q[k][draft[k]])
        out[k] = abs(r[k] * qx - px) / px if px > 0 else np.inf
    return out


def residual(p_row, q_row):
    """Step (6): unnormalised max(0, p - q); falls back to p if nothing is left."""
    R = np.maximum(0.0, np.asarray(p_row, dtype=np.float64) - np.asarray(q_row, dtype=np.float64))
    return (R, False) if R.sum() > 0.0 else (np.asarray(p_row, dtype=np.float64), True)


def verify_with_uniforms(P, q, draft, r, u_final):
    """Steps (5)-(7).  P: [gamma+1, V] target probabilities (row k = next-token law after
    prefix o draft[:k]); q: [gamma, V]; r: [gamma]; u_final: [gamma+1], entry n is used.
    Returns (n, token, margin, fell_back)."""
    gamma = len(draft)
    flags = accept_flags(P, q, draft, r)
    rejected = np.flatnonzero(~flags)
    n = int(rejected[0]) if rejected.size else gamma
    if n < gamma:
        w, fell_back = residual(P[n], q[n])
    else:
        w, fell_back = np.asarray(P[gamma], dtype=np.float64), False
    tok, margin = invcdf(w, u_final[n])
    return n, tok, margin, fell_back


# ---------------------------------------------------------------------------------------
# The two boundary calls, with uniforms taken from the counter-based generator.
# ---------------------------------------------------------------------------------------
def draft_uniforms(seed, batch, gamma, T):
    ua = np.zeros((T + 1, gamma))
    ub = np.zeros((T + 1, gamma))
    for j in range(1, T + 1):
        ua[j], ub[j] = philox.uniforms(seed, philox.STREAM_DRAFT, batch, j, np.arange(gamma))
    return ua, ub


def verify_uniforms(seed, batch, gamma):
    r, u = philox.uniforms(seed, philox.STREAM_VERIFY, batch, 0, np.arange(gamma + 1))
    return r[:gamma], u


def oracle_draft(drafter_logits, prefix, gamma, T, seed, mask_id, batch=0):
    ua, ub = draft_uniforms(seed, batch, gamma, T)
    return draft_with_uniforms(drafter_logits, prefix, gamma, T, ua, ub, mask_id)


def oracle_verify(target_logits, prefix, draft, q, seed, batch=0):
    """target_logits(tokens, rows) -> logits [len(rows), V] of the causal model at those
    positions of `tokens`.  Rows L-1 .. L-1+gamma of prefix o draft give P[0..gamma]."""
    prefix = np.asarray(prefix, dtype=np.int64)
    draft = np.asarray(draft, dtype=np.int64)
    L, gamma = prefix.size, draft.size
    rows = np.arange(L - 1, L + gamma)
    P = softmax_rows(np.asarray(target_logits(np.concatenate([prefix, draft]), rows), dtype=np.float64))
    r, u = verify_uniforms(seed, batch, gamma)
    return verify_with_uniforms(P, q, draft, r, u)


def expected_tokens(alpha, gamma):
    """Appendix A, Eq. (2): expected tokens per round for i.i.d. acceptance rate alpha."""
    return (1.0 - alpha ** (gamma + 1)) / (1.0 - alpha) if alpha < 1.0 else gamma + 1.0


# ---------------------------------------------------------------------------------------
# Temperature 0 (the setting of the paper's experiments, Section 4.1) and multi-round
# generation.  At temperature 0 both laws are one-hot on their argmax, and Algorithm 1
# degenerates: p(x)/q(x) is 1 when the drafted token is the target's argmax and 0 otherwise,
# so a token is accepted iff it equals the target's argmax there, and the residual
# norm(max(0, p - q)) after a rejection is p itself, i.e. the target's argmax.  No uniforms
# are consumed by verification; the drafter still reveals slots by the same 1/j rule.
# ---------------------------------------------------------------------------------------
def argmax_f32(row):
    """Index of the largest logit after rounding to fp32 (the precision the path stores
    logits in), lowest index on ties.  Returns (index, gap to the runner-up)."""
    x = np.asarray(row, dtype=np.float32)
    v = int(np.argmax(x))
    if x.size == 1:
        return v, np.inf
    rest = np.delete(x, v)
    return v, float(x[v] - rest.max())


def draft_greedy_with_uniforms(drafter_logits, prefix, gamma, T, ua, mask_id):
    """Steps (1)-(3) at temperature 0: a slot revealed at step j takes the argmax of its row.
    Returns (z, gaps, n_forwards)."""
    prefix = np.asarray(prefix, dtype=np.int64)
    z = np.full(gamma, mask_id, dtype=np.int64)
    gaps = np.full(gamma, np.inf)
    n_forwards = 0
    for j in range(T, 0, -1):
        masked = np.flatnonzero(z == mask_id)
        if masked.size == 0:
            continue
        logits = np.asarray(drafter_logits(np.concatenate([prefix, z]), j / T), dtype=np.float64)
        n_forwards += 1
        for k in masked:
            if j == 1 or ua[j, k] * j < 1.0:
                z[k], gaps[k] = argmax_f32(logits[k])
    return z, gaps, n_forwards


def verify_greedy(logits, draft):
    """Steps (4)-(7) at temperature 0.  logits: [gamma+1, V] target logits (row k follows
    prefix o draft[:k]).  Returns (n, token, gaps[gamma+1])."""
    gamma = len(draft)
    top = [argmax_f32(logits[k]) for k in range(gamma + 1)]
    n = gamma
    for k in range(gamma):
        if int(draft[k]) != top[k][0]:
            n = k
            break
    return n, top[n][0], np.array([g for _, g in top])


def oracle_draft_greedy(drafter_logits, prefix, gamma, T, seed, mask_id, batch=0):
    ua, _ = draft_uniforms(seed, batch, gamma, T)
    return draft_greedy_with_uniforms(drafter_logits, prefix, gamma, T, ua, mask_id)


def oracle_verify_greedy(target_logits, prefix, draft):
    prefix = np.asarray(prefix, dtype=np.int64)
    draft = np.asarray(draft, dtype=np.int64)
    rows = np.arange(prefix.size - 1, prefix.size + draft.size)
    logits = np.asarray(target_logits(np.concatenate([prefix, draft]), rows), dtype=np.float64)
    return verify_greedy(logits, draft)


def generate(drafter_logits, target_logits, prefix, n_new, gamma, T, seed, mask_id, greedy):
    """Rounds of Algorithm 1 until at least n_new tokens were emitted; round i uses seed + i and
    appends its n accepted draft tokens and the extra token to the prefix.
    Returns (tokens emitted [>= n_new], accepted count of every round)."""
    seq = [int(t) for t in prefix]
    start = len(seq)
    accepted = []
    rnd = 0
    while len(seq) - start < n_new:
        if greedy:
            z, _, _ = oracle_draft_greedy(drafter_logits, seq, gamma, T, seed + rnd, mask_id)
            n, tok, _ = oracle_verify_greedy(target_logits, seq, z)
        else:
            z, q, _, _ = oracle_draft(drafter_logits, seq, gamma, T, seed + rnd, mask_id)
            n, tok, _, _ = oracle_verify(target_logits, seq, z, q, seed + rnd)
        seq += [int(t) for t in z[:n]] + [int(tok)]
        accepted.append(n)
        rnd += 1
    return np.array(seq[start:], dtype=np.int64), np.array(accepted, dtype=np.int64)


def target_greedy_decode(target_logits, prefix, n_new):
    """Plain autoregressive decoding of the target at temperature 0 (what SpecDiff must reproduce)."""
    seq = [int(t) for t in prefix]
    for _ in range(n_new):
        logits = np.asarray(target_logits(np.array(seq), np.array([len(seq) - 1])), dtype=np.float64)
        seq.append(argmax_f32(logits[0])[0])
    return np.array(seq[len(prefix):], dtype=np.int64)


# ---------------------------------------------------------------------------------------
# Standard speculative decoding (SpS), the paper's baseline (Section 3, "Speculative decoding"; Table 1, row
# SpS: depth D_p + gamma D_q): the drafter is a small *autoregressive* model that produces the gamma draft
# tokens one after the other, x_k ~ q_k = M_q(prefix o x_0 .. x_{k-1}); verification is the same
# (verify_with_uniforms).  And the paper's "sequence initialisation" (Section 4): the first tokens of a
# generation are produced with SpS, the rest with the diffusion drafter.
# ---------------------------------------------------------------------------------------
def sps_draft_with_uniforms(drafter_logits, prefix, gamma, u, greedy=False):
    """gamma sequential evaluations of a causal drafter.  drafter_logits(tokens, rows) -> logits [len(rows), V]
    of the causal model at those positions; u: [gamma] uniforms (step k uses u[k]; unused when greedy).
    Returns (z int64[gamma], q fp32[gamma, V], margins fp64[gamma], n_forwards)."""
    seq = [int(t) for t in prefix]
    z = np.zeros(gamma, dtype=np.int64)
    q = None
    margins = np.zeros(gamma)
    for k in range(gamma):
        logits = np.asarray(drafter_logits(np.array(seq), np.array([len(seq) - 1])), dtype=np.float64)[0]
        if q is None:
            q = np.zeros((gamma, logits.size), dtype=np.float64)
        if greedy:
            z[k], margins[k] = argmax_f32(logits)
            q[k, z[k]] = 1.0
        else:
            pi = softmax_rows(logits)
            z[k], margins[k] = invcdf(pi, u[k])
            q[k] = pi
        seq.append(int(z[k]))
    return z, q.astype(np.float32), margins, gamma


def sps_uniforms(seed, batch, gamma):
    return philox.uniforms(seed, philox.STREAM_SPS, batch, 0, np.arange(gamma))[1]


def oracle_sps_draft(drafter_logits, prefix, gamma, seed, batch=0):
    return sps_draft_with_uniforms(drafter_logits, prefix, gamma, sps_uniforms(seed, batch, gamma))


def generate_hybrid(sps_logits, drafter_logits, target_logits, prefix, n_new, gamma_sps, gamma, T, seed, mask_id, n_init, greedy):
    """Sequence initialisation: rounds of SpS (draft length gamma_sps) until at least n_init tokens were emitted, then
    rounds of SpecDiff (gamma, T) until n_new in all; round i uses seed + i whichever drafter runs it.
    Returns (tokens emitted, accepted count per round, number of SpS rounds)."""
    seq = [int(t) for t in prefix]
    start = len(seq)
    accepted = []
    rnd = sps_rounds = 0
    while len(seq) - start < n_new:
        use_sps = len(seq) - start < n_init
        if use_sps:
            z, q, _, _ = sps_draft_with_uniforms(sps_logits, seq, gamma_sps, sps_uniforms(seed + rnd, 0, gamma_sps), greedy)
            sps_rounds += 1
        elif greedy:
            z, _, _ = oracle_draft_greedy(drafter_logits, seq, gamma, T, seed + rnd, mask_id)
        else:
            z, q, _, _ = oracle_draft(drafter_logits, seq, gamma, T, seed + rnd, mask_id)
        if greedy:
            n, tok, _ = oracle_verify_greedy(target_logits, seq, z)
        else:
            n, tok, _, _ = oracle_verify(target_logits, seq, z, q, seed + rnd)
        seq += [int(t) for t in z[:n]] + [int(tok)]
        accepted.append(n)
        rnd += 1
    return np.array(seq[start:], dtype=np.int64), np.array(accepted, dtype=np.int64), sps_rounds
