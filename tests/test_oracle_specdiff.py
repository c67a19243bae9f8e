"""Pins for oracle/specdiff.py: what the paper and the mathematics fix about Algorithm 1.

* losslessness (Sections 1, 3): the law of the emitted token equals the target law p,
  checked by integrating the oracle's own code path over exact grids of its uniforms;
* acceptance rule special cases (Section 3): p == q accepts everything, a one-hot q is
  accepted with probability p(x), the residual never returns the rejected token;
* alpha = sum min(p, q) (Appendix A, Corollary) and the expected tokens per round
  (Appendix A, Eq. 2) by Monte-Carlo over Philox seeds;
* the masked-diffusion schedule: each slot is revealed at step j with probability 1/T,
  everything is revealed after step 1, revealed slots are a fixed point, the drafter is
  evaluated T times (Section 4, "Drafter's evaluations"; Table 1 depth D_p + T D_q);
* a complete round with table-driven toy models, enumerated exactly: the first emitted
  token follows p_1 for T in {1, 2}; for T = 1 the second one follows p_2(. | first).
"""
import itertools
from collections import defaultdict
from fractions import Fraction

import numpy as np
import pytest

from oracle import specdiff as sd
from oracle import philox


def midgrid(n):
    return (np.arange(n) + 0.5) / n


# ------------------------------------------------------------------ invcdf
def test_invcdf_textbook_cases():
    assert sd.invcdf([0, 0, 1, 0], 0.0)[0] == 2           # one-hot, any u
    assert sd.invcdf([0, 0, 1, 0], 1 - 2.0 ** -24)[0] == 2
    w = [0.25, 0.25, 0.25, 0.25]
    assert [sd.invcdf(w, u)[0] for u in (0.0, 0.2499, 0.25, 0.5, 0.75, 1 - 2.0 ** -24)] == [0, 0, 1, 2, 3, 3]
    assert sd.invcdf([0, 2, 0, 6, 0], 0.0)[0] == 1         # leading zeros are skipped (strict '>')
    assert sd.invcdf([0, 2, 0, 6, 0], 0.25)[0] == 3        # boundary value belongs to the next token
    assert sd.invcdf([0, 2, 0, 6, 0], 0.9999999)[0] == 3   # trailing zeros never chosen
    v, m = sd.invcdf([1, 1, 2], 0.375)                     # target 1.5 in [1, 2): margin .5/4
    assert v == 1 and abs(m - 0.125) < 1e-15


def test_invcdf_frequencies_match_weights():
    w = np.array([3, 0, 1, 4, 0, 2], dtype=float)
    counts = np.bincount([sd.invcdf(w, u)[0] for u in midgrid(1000)], minlength=6)
    assert (counts == w * 100).all()


# ------------------------------------------------------------------ accept + residual, brute force
GRID12 = [Fraction(a, 12) for a in range(13)]


def dists(V, denom):
    for c in itertools.product(range(denom + 1), repeat=V):
        if sum(c) == denom:
            yield np.array(c, dtype=np.float64) / denom


def round_output_law(p0, p1, q0, N=240):
    """Law of the first emitted token of a gamma = 1 round, by sweeping the oracle's
    verify path over exact mid-point grids of r and u (N divisible by every denominator)."""
    V = len(p0)
    law = np.zeros(V)
    P = np.stack([p0, p1])
    for x in range(V):
        if q0[x] == 0:
            continue
        acc = 0
        for r in midgrid(N):
            n, _, _, _ = sd.verify_with_uniforms(P, q0[None, :], [x], [r], [0.5, 0.5])
            acc += n
        a = acc / N
        law[x] += q0[x] * a
        if a < 1:                         # law of the correction token given a rejection
            res = np.zeros(V)
            for u in midgrid(N):
                n, tok, _, fb = sd.verify_with_uniforms(P, q0[None, :], [x], [1 - 1e-9], [u, u])
                assert n == 0 and not fb
                res[tok] += 1.0 / N
            assert res[x] == 0            # the rejected token is never resampled
            law += q0[x] * (1 - a) * res
    return law


def test_emitted_token_follows_target_law_exactly():
    p1 = np.array([0.5, 0.25, 0.25])
    n_cases = 0
    for p0 in dists(3, 4):
        for q0 in dists(3, 4):
            law = round_output_law(p0, p1, q0)
            np.testing.assert_allclose(law, p0, atol=1e-12)
            n_cases += 1
    assert n_cases == 15 * 15             # includes p == q, one-hot q, one-hot p, disjoint supports


def test_bonus_token_after_full_acceptance_follows_last_target_row():
    P = np.array([[0.5, 0.5, 0.0], [0.25, 0.5, 0.25]])
    q = np.array([[0.5, 0.5, 0.0]])
    counts = np.zeros(3)
    for u in midgrid(8):
        n, tok, _, _ = sd.verify_with_uniforms(P, q, [1], [0.999], [0.123, u])
        assert n == 1
        counts[tok] += 1
    assert (counts == [2, 4, 2]).all()


def test_p_equal_q_accepts_everything():
    rng = np.random.default_rng(0)
    for seed in range(50):
        gamma, V = 6, 11
        P = rng.dirichlet(np.ones(V), size=gamma + 1)
        q = P[:gamma].astype(np.float32)
        P[:gamma] = q                                  # identical numbers on both sides
        draft = rng.integers(0, V, gamma)
        r, u = sd.verify_uniforms(seed, 0, gamma)
        n, tok, _, _ = sd.verify_with_uniforms(P, q, draft, r, u)
        assert n == gamma
    # also at the largest uniform the generator can emit
    assert sd.accept_flags(P, q, draft, np.full(gamma, 1 - 2.0 ** -24)).all()


def test_one_hot_q_is_accepted_with_probability_p():
    p = np.array([[0.25, 0.75], [0.5, 0.5]])
    q = np.array([[1.0, 0.0]])
    acc = sum(sd.verify_with_uniforms(p, q, [0], [r], [0.5, 0.5])[0] for r in midgrid(64))
    assert acc == 16
    # rejected => residual is p with the drafted token removed
    assert all(sd.verify_with_uniforms(p, q, [0], [0.99], [u, u])[1] == 1 for u in midgrid(16))


def test_first_rejection_discards_the_rest_and_picks_the_uniform_of_that_position():
    V, gamma = 4, 5
    P = np.full((gamma + 1, V), 0.25)
    q = np.full((gamma, V), 0.25)
    q[2] = [0.7, 0.1, 0.1, 0.1]                        # token 0 at position 2: ratio .25/.7
    q[4] = [0.7, 0.1, 0.1, 0.1]
    draft = [0, 0, 0, 0, 0]
    r = np.array([0.9, 0.9, 0.9, 0.0, 0.9])
    u = np.array([0.0, 0.0, 0.999, 0.0, 0.0, 0.0])     # only entry n = 2 may be consumed
    n, tok, _, _ = sd.verify_with_uniforms(P, q, draft, r, u)
    assert n == 2 and tok == 3                          # residual (0, .15, .15, .15): u = .999 -> last
    r[2] = 0.3                                          # now position 2 passes; position 4 fails
    n, tok, _, _ = sd.verify_with_uniforms(P, q, draft, r, u)
    assert n == 4 and tok == 1                          # u[4] = 0 -> first token with residual mass


def test_residual_properties():
    rng = np.random.default_rng(5)
    for _ in range(100):
        p, q = rng.dirichlet(np.ones(9)), rng.dirichlet(np.ones(9)).astype(np.float32)
        R, fb = sd.residual(p, q)
        assert not fb and (R >= 0).all() and R.sum() > 0
        assert ((R > 0) == (p > q)).all()
        # closed form of the normaliser: sum max(0, p - q) = 1 - sum min(p, q)   (both sum to 1)
        assert abs(R.sum() - (1 - np.minimum(p, q).sum()) - (q.astype(np.float64).sum() - 1) * 0) < 1e-6
    R, fb = sd.residual(np.array([0.5, 0.5]), np.array([0.5, 0.5]))
    assert fb and (R == [0.5, 0.5]).all()              # zero-mass fallback: p itself


# ------------------------------------------------------------------ alpha and expected tokens (Monte-Carlo)
def test_acceptance_rate_and_expected_tokens_match_closed_forms():
    V, gamma, N = 8, 5, 20000
    rng = np.random.default_rng(42)
    p = rng.dirichlet(np.ones(V))
    qrow = rng.dirichlet(np.ones(V))
    P = np.tile(p, (gamma + 1, 1))
    q = np.tile(qrow, (gamma, 1)).astype(np.float32)
    alpha = np.minimum(p, q[0].astype(np.float64)).sum()
    acc_first, tokens, out_first = 0, 0, np.zeros(V)
    for seed in range(N):
        ua, ub = philox.uniforms(seed, 7, 0, 0, np.arange(gamma))      # draft tokens x_k ~ q, i.i.d.
        draft = [sd.invcdf(q[0], u)[0] for u in ub]
        r, u = sd.verify_uniforms(seed, 0, gamma)
        n, tok, _, _ = sd.verify_with_uniforms(P, q, draft, r, u)
        acc_first += n >= 1
        tokens += n + 1
        out_first[draft[0] if n >= 1 else tok] += 1
    se = np.sqrt(alpha * (1 - alpha) / N)
    assert abs(acc_first / N - alpha) < 4 * se                          # alpha = sum_x min(p, q)
    expect = sd.expected_tokens(alpha, gamma)
    assert abs(expect - sum(alpha ** i for i in range(gamma + 1))) < 1e-12   # Eq. (2) is the geometric sum
    assert abs(tokens / N - expect) < 4 * 1.6 / np.sqrt(N)
    assert np.abs(out_first / N - p).max() < 4 * 0.5 / np.sqrt(N)       # first emitted token ~ p


def test_expected_tokens_limits():
    assert sd.expected_tokens(0.0, 7) == 1.0
    assert sd.expected_tokens(1.0, 7) == 8.0
    assert abs(sd.expected_tokens(0.5, 1) - 1.5) < 1e-15
    assert abs(sd.expected_tokens(0.9, 15) - (1 - 0.9 ** 16) / 0.1) < 1e-12


# ------------------------------------------------------------------ table-driven toy models
class ToyDrafter:
    """logits = log of a table row chosen by (t, the other slot's state); probabilities are
    multiples of 1/4 so that mid-point grids of 4 integrate the sampler exactly."""
    rows = [np.array(r) / 4.0 for r in ([2, 1, 1], [1, 2, 1], [1, 1, 2], [2, 2, 0], [0, 1, 3], [4, 0, 0], [1, 3, 0])]

    def __init__(self, V=3, gamma=2):
        self.V, self.gamma, self.calls = V, gamma, 0

    def __call__(self, tokens, t):
        self.calls += 1
        block = tokens[-self.gamma:]
        out = np.zeros((self.gamma, self.V))
        for k in range(self.gamma):
            other = int(block[1 - k])
            idx = (3 * k + other + int(round(4 * t))) % len(self.rows)
            with np.errstate(divide="ignore"):
                out[k] = np.log(self.rows[idx]) + 0.37 * (k + 1)        # softmax removes the shift
        return out


def toy_target(draft):
    """Causal toy: row k depends on draft[:k] only.  Multiples of 1/4."""
    base = [np.array(r) / 4.0 for r in ([1, 2, 1], [2, 0, 2], [0, 3, 1], [1, 1, 2])]
    P0 = base[0]
    P1 = base[1 + draft[0] % 3]
    P2 = base[(2 * draft[0] + draft[1]) % 4]
    return np.stack([P0, P1, P2])


def enumerate_drafts(T):
    """Exact law of (draft tokens, q) for the toy drafter: all combinations of representative
    uniforms, each with equal weight."""
    gamma, MASK = 2, 3
    outcomes = defaultdict(float)
    ua_vals = {j: ([0.5] if j == 1 else list(midgrid(2 * j))) for j in range(1, T + 1)}  # 1/j is a grid edge
    ub_vals = list(midgrid(4))
    slots = [(j, k) for j in range(1, T + 1) for k in range(gamma)]
    total = 0
    for ua_c in itertools.product(*[ua_vals[j] for j, _ in slots]):
        for ub_c in itertools.product(ub_vals, repeat=len(slots)):
            ua = np.zeros((T + 1, gamma)); ub = np.zeros((T + 1, gamma))
            for (j, k), a, b in zip(slots, ua_c, ub_c):
                ua[j, k], ub[j, k] = a, b
            z, q, _, _ = sd.draft_with_uniforms(ToyDrafter(), [0, 1], gamma, T, ua, ub, MASK)
            assert (z != MASK).all()
            outcomes[(tuple(int(v) for v in z), q.tobytes())] += 1.0
            total += 1
    return {k: w / total for k, w in outcomes.items()}


def round_law(T):
    """Joint law of (n, first emitted, second emitted or -1) of one full toy round."""
    law = defaultdict(float)
    g = midgrid(12)
    for (z, qb), w in enumerate_drafts(T).items():
        q = np.frombuffer(qb, dtype=np.float32).reshape(2, 3)
        P = toy_target(z)
        for r0, r1, u in itertools.product(g, g, g):
            n, tok, _, fb = sd.verify_with_uniforms(P, q, list(z), [r0, r1], [u, u, u])
            assert not fb
            emitted = list(z[:n]) + [tok]
            law[(n, emitted[0], emitted[1] if len(emitted) > 1 else -1)] += w / 12 ** 3
    return law


@pytest.mark.parametrize("T", [1, 2])
def test_full_round_first_token_follows_target(T):
    law = round_law(T)
    first = np.zeros(3)
    for (n, a, b), w in law.items():
        first[a] += w
    np.testing.assert_allclose(first, toy_target([0, 0])[0], atol=1e-12)
    assert abs(sum(law.values()) - 1) < 1e-12


def test_full_round_T1_second_token_follows_target_conditional():
    """With one diffusion step the drafted tokens are independent given the prefix, and the
    round is lossless beyond the first token: P(first = a accepted, second = b) =
    P(first = a accepted) * p_2(b | a)."""
    law = round_law(1)
    for a in range(3):
        pa = sum(w for (n, x, y), w in law.items() if n >= 1 and x == a)
        if pa == 0:
            continue
        cond = toy_target([a, 0])[1]
        for b in range(3):
            pab = sum(w for (n, x, y), w in law.items() if n >= 1 and x == a and y == b)
            assert abs(pab - pa * cond[b]) < 1e-12


# ------------------------------------------------------------------ the reverse-diffusion schedule
@pytest.mark.parametrize("T", [1, 2, 3, 4])
def test_each_slot_is_revealed_at_step_j_with_probability_one_over_T(T):
    """Telescoping of the 1/j reveal probabilities, integrated exactly through the code."""
    MASK, gamma = 3, 1
    N = 12                                           # divisible by 1..4: thresholds 1/j are grid edges
    reveal = defaultdict(int)

    class Rec(ToyDrafter):
        pass

    for ua_c in itertools.product(midgrid(N), repeat=T):
        ua = np.zeros((T + 1, gamma)); ub = np.full((T + 1, gamma), 0.5)
        for j in range(1, T + 1):
            ua[j, 0] = ua_c[j - 1]
        seen = []

        def logits(tokens, t, seen=seen):
            seen.append((t, int(tokens[-1])))
            return np.zeros((1, 3))

        z, q, _, nf = sd.draft_with_uniforms(logits, [0], gamma, T, ua, ub, MASK)
        assert z[0] != MASK and abs(q.sum() - 1) < 1e-6
        # the step after which the slot stopped being MASK = number of forwards that saw MASK
        j_reveal = T - sum(1 for _, tok in seen if tok == MASK) + 1
        reveal[j_reveal] += 1
        assert nf == len(seen) == T - j_reveal + 1    # later steps are skipped once nothing is masked
        assert [round(t * T) for t, _ in seen] == list(range(T, j_reveal - 1, -1))   # t = j / T, descending
    assert all(reveal[j] == N ** T // T for j in range(1, T + 1))


def test_revealed_block_is_a_fixed_point_and_skipping_is_harmless():
    MASK, gamma, T = 3, 2, 4
    for seed in range(40):
        ua, ub = sd.draft_uniforms(seed, 0, gamma, T)
        d1, d2 = ToyDrafter(), ToyDrafter()
        z1, q1, _, n1 = sd.draft_with_uniforms(d1, [2, 2, 1], gamma, T, ua, ub, MASK, skip_when_done=True)
        z2, q2, _, n2 = sd.draft_with_uniforms(d2, [2, 2, 1], gamma, T, ua, ub, MASK, skip_when_done=False)
        assert (z1 == z2).all() and np.array_equal(q1, q2)
        assert n2 == T and n1 <= T and d2.calls == T           # exactly T drafter evaluations
        assert np.allclose(q1.sum(axis=1), 1, atol=1e-6)
        assert all(q1[k, z1[k]] > 0 for k in range(gamma))     # a token is drawn from its own row


def test_steps_that_reveal_nothing_can_be_left_out():
    """Which slots a step reveals is decided by the uniforms alone and a step's logits are read by nothing but
    the slots revealed at it: leaving out the forwards of steps that reveal nothing changes neither z nor q, for
    a drafter whose logits depend on the time and on the state of the block.  The forwards that remain are those
    of the distinct reveal steps (each slot's reveal step is uniform on 1..T: Algorithm 1's 1/j rule)."""
    MASK, gamma, T = 3, 2, 6
    saved = 0
    for seed in range(60):
        ua, ub = sd.draft_uniforms(seed, 0, gamma, T)
        d1, d2 = ToyDrafter(), ToyDrafter()
        z1, q1, m1, n1 = sd.draft_with_uniforms(d1, [2, 2, 1], gamma, T, ua, ub, MASK)
        z2, q2, m2, n2 = sd.draft_with_uniforms(d2, [2, 2, 1], gamma, T, ua, ub, MASK, skip_idle_steps=True)
        assert (z1 == z2).all() and np.array_equal(q1, q2) and np.array_equal(m1, m2)
        # reveal step of slot k: the first j, counting down from T, with ua[j, k] * j < 1 (j = 1 always)
        steps = {next(j for j in range(T, 0, -1) if j == 1 or ua[j, k] * j < 1.0) for k in range(gamma)}
        assert n2 == d2.calls == len(steps) <= n1
        saved += n1 - n2
    assert saved > 0                                           # the option does leave forwards out


def test_draft_uses_the_documented_counters():
    gamma, T = 3, 2
    ua, ub = sd.draft_uniforms(77, 4, gamma, T)
    for j in (1, 2):
        a, b = philox.uniforms(77, philox.STREAM_DRAFT, 4, j, [0, 1, 2])
        assert (ua[j] == a).all() and (ub[j] == b).all()
    r, u = sd.verify_uniforms(77, 4, gamma)
    a, b = philox.uniforms(77, philox.STREAM_VERIFY, 4, 0, [0, 1, 2, 3])
    assert (r == a[:3]).all() and (u == b).all()


def test_oracle_verify_reads_the_right_rows_of_the_target():
    """P[k] must be the target's law after prefix o draft[:k]: rows L-1 .. L-1+gamma."""
    prefix, draft = [5, 6, 7], [1, 0]

    def target_logits(tokens, rows):
        assert list(tokens) == prefix + draft and list(rows) == [2, 3, 4]
        with np.errstate(divide="ignore"):
            return np.log(toy_target(draft))

    q = np.array([[0.25, 0.5, 0.25], [0.5, 0.25, 0.25]], dtype=np.float32)
    n, tok, _, _ = sd.oracle_verify(target_logits, prefix, draft, q, seed=3)
    r, u = sd.verify_uniforms(3, 0, 2)
    assert (n, tok) == sd.verify_with_uniforms(toy_target(draft), q, draft, r, u)[:2]


# ------------------------------------------------------------------ accept_margins
def test_accept_margins_hand_computed_cases():
    """The margin of acceptance test k is |r_k q_k(x_k) - p_k(x_k)| / p_k(x_k) (Section 3: the test compares
    r with p(x)/q(x)).  Hand-computed cases: an exact tie gives 0, a known ratio gives its distance from 1,
    p(x) = 0 gives infinity, and the margin is small exactly where flipping r across p/q flips accept_flags."""
    P = np.array([[0.5, 0.5, 0.0], [0.2, 0.3, 0.5], [0.0, 1.0, 0.0], [0.25, 0.25, 0.5]])
    q = np.array([[0.25, 0.75, 0.0], [0.4, 0.4, 0.2], [0.5, 0.5, 0.0], [0.5, 0.25, 0.25]])
    draft = np.array([0, 0, 0, 0])
    r = np.array([0.5, 0.5, 0.3, 0.75])
    m = sd.accept_margins(P, q, draft, r)
    # k = 0: r q = 0.125 vs p = 0.5 -> |0.125 - 0.5| / 0.5 = 0.75
    # k = 1: r q = 0.2 vs p = 0.2 -> exact tie (0.5 * 0.4 is exact in binary up to the rounding of 0.4 and 0.2)
    # k = 2: p(x) = 0 -> inf (always rejected, never close)
    # k = 3: r q = 0.375 vs p = 0.25 -> 0.5
    assert m[0] == pytest.approx(0.75, abs=1e-15)
    assert m[1] < 1e-15
    assert np.isinf(m[2])
    assert m[3] == pytest.approx(0.5, abs=1e-15)
    # only x_k's entries matter: other columns may change freely
    P2, q2 = P.copy(), q.copy()
    P2[:, 1:] += 0.125
    q2[:, 1:] *= 0.5
    np.testing.assert_array_equal(sd.accept_margins(P2, q2, draft, r), m)
    # the draft index is honoured (not always column 0)
    m1 = sd.accept_margins(P, q, np.array([1, 2, 1, 2]), r)
    assert m1[0] == pytest.approx(abs(0.5 * 0.75 - 0.5) / 0.5) and m1[1] == pytest.approx(abs(0.5 * 0.2 - 0.5) / 0.5)
    assert m1[2] == pytest.approx(abs(0.3 * 0.5 - 1.0)) and m1[3] == pytest.approx(abs(0.75 * 0.25 - 0.5) / 0.5)


def test_accept_margin_is_small_exactly_where_the_flag_can_flip():
    """Sweep r across the threshold p/q: accept_flags changes sign where the margin passes through 0, and a
    relative perturbation of p(x) smaller than the margin never changes the flag."""
    rng = np.random.default_rng(5)
    for _ in range(200):
        V = 6
        p = rng.dirichlet(np.ones(V))
        q = rng.dirichlet(np.ones(V))
        x = int(rng.integers(V))
        r = float(rng.random())
        P, Q, d, rr = p[None], q[None], np.array([x]), np.array([r])
        m = sd.accept_margins(P, Q, d, rr)[0]
        flag = sd.accept_flags(P, Q, d, rr)[0]
        assert flag == (r * q[x] <= p[x]) or m < 1e-6          # the flag is the fp32 form of the same comparison
        for eps in (0.5 * m, -0.5 * m):                        # p(x) moved by less than the margin: same decision
            if m < 1e-5:
                continue
            P2 = P.copy()
            P2[0, x] *= 1.0 + eps
            assert sd.accept_flags(P2, Q, d, rr)[0] == flag
        if np.isfinite(m):                                     # moved past the margin: the decision flips
            P3 = P.copy()
            P3[0, x] *= (1.0 + 2.0 * m + 1e-3) if not flag else max(0.0, 1.0 - 2.0 * m - 1e-3)
            if P3[0, x] > 0:
                assert sd.accept_flags(P3, Q, d, rr)[0] != flag
