"""Pins of the speculative-sampling oracle (oracle/sampling.py) to things other than itself: hand-worked cases,
the identity the rule exists for (emitted tokens are distributed as plain sampling from the target), and the
special cases that reduce to something simpler.  CPU only."""
import os

import numpy as np
import pytest

from oracle import sampling as osm

HERE = os.path.dirname(os.path.abspath(__file__))


def _rows(txt):
    return [np.log(np.array([float(x) for x in r.split(",")])) for r in txt.split(";")]


def _golden():
    cases = []
    for line in open(os.path.join(HERE, "golden", "spec_sampling_cases.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        f = [x.strip() for x in line.split("|")]
        s = int(f[0])
        tgt = _rows(f[1])
        drf = None if f[2] in ("point", "-") else _rows(f[2])
        lst = lambda t, conv: [] if t == "-" else [conv(x) for x in t.split(",")]
        cases.append((s, tgt, drf, lst(f[3], int), lst(f[4], float), lst(f[5], float), int(f[6]), lst(f[7], int)))
    return cases


@pytest.mark.parametrize("case", _golden())
def test_hand_worked_cases(case):
    s, tgt, drf, props, ua, us, l, emitted = case
    assert len(tgt) == s + 1 and len(props) == s and len(ua) == s and len(us) == s + 1
    got_l, got_e, _ = osm.spec_sample_round(tgt, drf, props, ua, us, 1.0)
    assert (got_l, got_e) == (l, emitted)


def test_draw_is_the_inverse_cdf_on_dyadic_weights():
    # weights 1/2, 1/4, 1/8, 1/8: every boundary is exact in binary, so the intervals are [0,.5) [.5,.75) [.75,.875) [.875,1)
    w = [4.0, 2.0, 1.0, 1.0]
    for u, want in [(0.0, 0), (0.49999, 0), (0.5, 1), (0.74999, 1), (0.75, 2), (0.875, 3), (0.99999, 3)]:
        assert osm.draw(w, u)[0] == want
    # zero-weight entries are never drawn, whatever u
    w = [0.0, 1.0, 0.0, 1.0, 0.0]
    assert {osm.draw(w, u)[0] for u in np.linspace(0, 0.999999, 1001)} == {1, 3}
    # margin: distance to the nearest boundary that has a token on its other side
    assert abs(osm.draw([1.0, 1.0], 0.45)[1] - 0.05) < 1e-12
    assert abs(osm.draw([1.0, 1.0], 0.05)[1] - 0.45) < 1e-12   # nothing below index 0: only the upper boundary counts


def test_softmax_temperature():
    z = np.array([0.3, -1.2, 2.0, 0.0])
    p = osm.softmax_t(z, 0.5)
    assert abs(p.sum() - 1) < 1e-15
    # ratios of probabilities are exp of logit differences over T
    assert abs(p[2] / p[0] - np.exp((2.0 - 0.3) / 0.5)) < 1e-12
    # T -> 0: the arg-max takes everything
    assert osm.softmax_t(z, 1e-3)[2] > 1 - 1e-12


def _tiny_models(rng, V):
    """Conditional distributions of a target and a draft 'model' over all prefixes of length < 3, as logits."""
    tgt, drf = {}, {}
    for n in range(3):
        for prefix in np.ndindex(*([V] * n)):
            tgt[prefix] = rng.normal(size=V) * 1.5
            drf[prefix] = tgt[prefix] + rng.normal(size=V) * 1.0    # a draft that is near, not equal
    return tgt, drf


@pytest.mark.parametrize("point_mass", [False, True])
def test_emitted_tokens_are_distributed_as_plain_target_sampling(point_mass):
    """The identity the rule exists for, by simulation on a 3-token vocabulary with conditional distributions that
    depend on the prefix: the first two generated tokens (over as many rounds as that takes, s = 2) must have the
    joint distribution p(y1) p(y2 | y1) of the target alone.  A wrong ratio, a residual without the clamp or the
    normalisation, a bonus row off by one, or the wrong row for a rejected position all move it by many sigma."""
    rng = np.random.default_rng(7)
    V, s, T, N = 3, 2, 0.8, 40000
    tgt, drf = _tiny_models(rng, V)
    counts = np.zeros((V, V))
    for _ in range(N):
        out = []
        while len(out) < 2:
            k = min(s, 2 - len(out))           # never look further than the two tokens wanted
            props, dl, prefix = [], [], tuple(out)
            for j in range(k):
                cur = prefix + tuple(props)
                if point_mass:
                    props.append(int(rng.integers(V)))    # any fixed proposal is valid for a point-mass drafter
                else:
                    dl.append(drf[cur])
                    props.append(osm.sample_token(drf[cur], T, rng.random())[0])
            tl = [tgt[prefix + tuple(props[:j])] for j in range(k + 1)]
            l, em, _ = osm.spec_sample_round(tl, None if point_mass else dl, props, rng.random(k), rng.random(k + 1), T)
            out += em
        counts[out[0], out[1]] += 1
    want = np.zeros((V, V))
    for a in range(V):
        for b in range(V):
            want[a, b] = osm.softmax_t(tgt[()], T)[a] * osm.softmax_t(tgt[(a,)], T)[b]
    got = counts / N
    sigma = np.sqrt(want * (1 - want) / N)
    assert np.all(np.abs(got - want) < 5 * sigma + 1e-9), (got, want)


def test_planted_mistakes_move_the_distribution():
    """The simulation above is a pin only if it catches the plausible mistakes: here two of them, planted in a copy
    of the rule, fail the same check on the first token."""
    rng = np.random.default_rng(11)
    V, T, N = 3, 1.0, 20000
    p_log, q_log = np.log([0.6, 0.3, 0.1]), np.log([0.2, 0.3, 0.5])
    p = osm.softmax_t(p_log, T)

    def first_token(rule):
        c = np.zeros(V)
        for _ in range(N):
            t = osm.sample_token(q_log, T, rng.random())[0]
            c[rule(t, rng.random(), rng.random())] += 1
        return c / N

    def right(t, ua, us):
        return osm.spec_sample_round([p_log, p_log], [q_log], [t], [ua], [us, 0.0], T)[1][0]

    def no_clamp(t, ua, us):       # residual |p - q| instead of max(0, p - q)
        q = osm.softmax_t(q_log, T)
        return t if ua * q[t] < p[t] else osm.draw(np.abs(p - q), us)[0]

    def inverse_ratio(t, ua, us):  # q / p instead of p / q
        q = osm.softmax_t(q_log, T)
        return t if ua * p[t] < q[t] else osm.draw(np.maximum(p - q, 0), us)[0]

    sigma = np.sqrt(p * (1 - p) / N)
    assert np.all(np.abs(first_token(right) - p) < 5 * sigma)
    assert np.any(np.abs(first_token(no_clamp) - p) > 8 * sigma)
    assert np.any(np.abs(first_token(inverse_ratio) - p) > 8 * sigma)


def test_draft_equal_to_target_keeps_every_proposal():
    rng = np.random.default_rng(3)
    V, s = 50, 5
    z = rng.normal(size=(s + 1, V)) * 2
    for _ in range(200):
        props = [osm.sample_token(z[j], 0.9, rng.random())[0] for j in range(s)]
        l, em, _ = osm.spec_sample_round(z, z[:s], props, rng.random(s), rng.random(s + 1), 0.9)
        assert l == s and em[:s] == props


def test_low_temperature_reduces_to_the_greedy_rule():
    """T -> 0 with point-mass proposals: a proposal survives exactly when it is the target's arg-max, and the token
    emitted behind the survivors is the arg-max of its row -- the acceptance rule of Sec. 2 / Alg. 1."""
    rng = np.random.default_rng(5)
    V, s = 40, 4
    for _ in range(200):
        z = rng.normal(size=(s + 1, V)) * 3
        am = z.argmax(-1)
        props = [int(am[j]) if rng.random() < 0.7 else int(rng.integers(V)) for j in range(s)]
        l_greedy = 0
        while l_greedy < s and props[l_greedy] == am[l_greedy]:
            l_greedy += 1
        l, em, _ = osm.spec_sample_round(z, None, props, rng.random(s) * 0.98 + 0.01, rng.random(s + 1) * 0.98 + 0.01, 1e-3)
        srt = np.sort(z, -1)
        if np.min(srt[:, -1] - srt[:, -2]) < 0.05:
            continue  # a near-tie: at T = 1e-3 a gap of 0.05 is still a factor e^50
        assert l == l_greedy and em == props[:l] + [int(am[l])]


def test_no_proposals_is_plain_sampling():
    rng = np.random.default_rng(9)
    z = rng.normal(size=(1, 30))
    for u in rng.random(50):
        l, em, _ = osm.spec_sample_round(z, None, [], [], [u], 1.3)
        assert l == 0 and em == [osm.sample_token(z[0], 1.3, u)[0]]
