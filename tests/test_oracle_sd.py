"""Pins of the CPU checker's speculative-decoding regeneration of rejected steps
(Section 5, "Combine RSD with SD"): the law of the emitted tokens, the expected
number of kept proposals, and - for greedy decoding, the paper's SD setting
(Section 3, "Default Setting") - identity with plain target decoding."""
from dataclasses import replace

import numpy as np
import pytest

from oracle import rsd_oracle as O
from test_oracle_rsd import params, run, GREEDY_MIX


def _dist(r, V, zeros=0):
    p = r.random(V) ** 2
    if zeros:
        p[r.choice(V, zeros, replace=False)] = 0.0
    return p / p.sum()


def test_verification_emits_the_target_law_and_keeps_the_overlap():
    """Two proposals whose second distribution depends on the first token.  The
    first emitted token must follow p_0 whatever q_0 is, the pair (when two or
    more tokens are emitted) p_0(x) p_1(y | x), and the first proposal is kept
    with probability sum_x min(p_0, q_0)."""
    V = 5
    r = np.random.default_rng(11)
    p0, q0 = _dist(r, V, zeros=1), _dist(r, V)
    p1 = [_dist(r, V) for _ in range(V)]
    q1 = [_dist(r, V, zeros=1) for _ in range(V)]
    p2 = _dist(r, V)
    n = 60000
    first = np.zeros(V)
    pair = np.zeros((V, V))
    kept0 = 0
    for _ in range(n):
        u = r.random(7)
        x0 = O.draw(q0, u[0])
        x1 = O.draw(q1[x0], u[1])
        out, kept = O.sd_verify([q0, q1[x0]], [p0, p1[x0], p2], [x0, x1], u[2:4], u[4:7])
        assert len(out) == kept + 1
        first[out[0]] += 1
        kept0 += kept >= 1
        if len(out) >= 2:
            pair[out[0], out[1]] += 1
    live = p0 > 0
    assert first[~live].sum() == 0
    chi2 = np.sum((first[live] - n * p0[live]) ** 2 / (n * p0[live]))
    assert chi2 < 30.0                                    # 3 dof
    overlap = np.minimum(p0, q0).sum()
    assert abs(kept0 / n - overlap) < 5 * np.sqrt(overlap * (1 - overlap) / n)
    # a second token is emitted exactly when the first proposal was kept, which happens with
    # probability min(p0, q0)(x) for first token x; given that, it follows p_1(. | x)
    for x in range(V):
        m = pair[x].sum()
        if m < 2000:
            continue
        chi2 = np.sum((pair[x] - m * p1[x]) ** 2 / (m * p1[x]))
        assert chi2 < 35.0                                # 4 dof
        assert abs(m / n - min(p0[x], q0[x])) < 5 * np.sqrt(0.25 / n)


def test_verification_special_cases():
    p = np.array([0.1, 0.2, 0.7])
    # identical distributions: every proposal kept, then one more target draw
    out, kept = O.sd_verify([p, p], [p, p, p], [2, 0], [0.999, 0.999], [0.0, 0.0, 0.25])
    assert (out, kept) == ([2, 0, 1], 2)
    # disjoint supports: nothing kept, the replacement follows p (residual = p)
    q = np.array([1.0, 0.0, 0.0]); pp = np.array([0.0, 0.5, 0.5])
    assert O.sd_verify([q], [pp, p], [0], [0.0], [0.6, 0.0]) == ([2], 0)
    # greedy rows are one-hot: kept iff equal to the target's choice, else that choice
    e = np.eye(3)
    assert O.sd_verify([e[1], e[2]], [e[1], e[0], e[2]], [1, 2], [0.0, 0.0], [0.0, 0.0, 0.0]) == ([1, 0], 1)
    # no proposals: a plain target draw
    assert O.sd_verify([], [p], [], [], [0.31]) == ([2], 0)


def test_token_distribution_is_what_sample_draws_from():
    r = np.random.default_rng(5)
    for _ in range(50):
        lg = r.normal(size=40) * 2
        for T, tp in [(0.0, 1.0), (0.7, 0.9), (1.0, 1.0), (1.3, 0.5)]:
            d = O.token_distribution(lg, T, tp)
            assert abs(d.sum() - 1) < 1e-12
            for u in r.random(6):
                assert O.draw(d, u) == O.sample(lg, u, T, tp)


@pytest.mark.parametrize("k", [1, 3, 7])
def test_greedy_speculation_reproduces_plain_target_steps(tiny, k):
    """Greedy decoding: whatever the draft proposes, the committed tokens are the
    target's own greedy continuation, so the whole run equals the run without
    speculation; afterwards neither model holds the newest token."""
    P = params(tiny["w"], **GREEDY_MIX)
    n_rej = 0
    for b in range(4):
        a = run(tiny, b, P)
        s = run(tiny, b, replace(P, sd_k=k))
        assert a["tokens"] == s["tokens"]
        for ra, rs in zip(a["records"], s["records"]):
            assert ra["accepted"] == rs["accepted"] and ra["final_tokens"] == rs["final_tokens"]
            if rs["accepted"]:
                assert rs["sd_rounds"] == []
                continue
            n_rej += 1
            ctx = rs["ctx_len"]
            assert rs["kv_len"][1] == ctx - 1 and rs["kv_len"][0] <= ctx - 1 and rs["kv_len"][2] == rs["ctx_pre"]
            emitted = sum(kept + 1 for _, kept in rs["sd_rounds"])
            assert emitted >= len(rs["final_tokens"])          # tokens after a step end are dropped
            used = 0
            for prop, kept in rs["sd_rounds"]:       # a round never proposes more than the step has room for
                assert 0 <= kept <= prop <= min(k, P.step_cap - used - 1)
                used += kept + 1
            # the cache-free run takes the same decisions
        c = run(tiny, b, replace(P, sd_k=k), use_cache=False)
        assert c["tokens"] == s["tokens"]
        assert [r["sd_rounds"] for r in c["records"]] == [r["sd_rounds"] for r in s["records"]]
    assert n_rej >= 3


def test_a_draft_equal_to_the_target_has_every_proposal_kept(tiny):
    d, t, p = tiny["models"]
    P = params(tiny["w"], delta=1.01, sd_k=3, sep_logit_bias=0.6)       # every step rejected
    out = run(tiny, 0, P, models=(t, t, p), max_steps=2)
    for rec in out["records"]:
        n = len(rec["final_tokens"])
        assert all(prop == kept for prop, kept in rec["sd_rounds"])
        # full rounds commit 4 tokens each; the last round may end the step early
        assert len(rec["sd_rounds"]) == -(-n // 4)


def _restricted(m, ids, scale=8.0):
    wv = dict(m._w)
    wv["lm_head"] = m._w["lm_head"][ids] * scale              # sharper, distinct distributions
    wv["embed"] = np.array(m._w["embed"], copy=True)
    wv["embed"][:len(ids)] = m._w["embed"][ids]
    return O.OracleModel(m.s, wv)


def test_each_proposal_is_judged_with_the_uniform_of_its_own_position(tiny):
    d, t, p = tiny["models"]
    ids = np.arange(8) * 100 + 3
    dm, tm = _restricted(d, ids), _restricted(t, ids)
    prompt = [int(x) for x in tiny["tokens"][1, :5]]
    n = len(prompt)
    P = O.Params(delta=2.0, sep_id=-1, step_cap=6, max_steps=1, max_ctx=n + 6, temperature=1.0, top_p=1.0, sd_k=3)
    r = np.random.default_rng(9)
    found = 0
    for trial in range(20):
        u_prop, u_t = r.random(n + 6), r.random(n + 6)
        def rounds(u_acc):
            out = O.generate_sequence(dm, tm, p, prompt, r.random(n + 6), u_t, np.zeros(1), P, u_prop=u_prop, u_acc=u_acc)
            return out["records"][0]["sd_rounds"], out["tokens"]
        base, toks = rounds(np.zeros(n + 6))
        assert base[0] == (3, 3)                                  # u = 0 keeps every proposal of positive target mass
        x = toks[n + 1]                                           # the second proposal and the distributions it met
        pq = [O.softmax(O.lm_logits(m, O.forward_full(m, toks[:n + 1])[-1])) for m in (tm, dm)]
        ratio = pq[0][x] / pq[1][x]
        if ratio >= 0.9:
            continue
        u = np.zeros(n + 6)
        u[n + 1] = 0.95
        assert rounds(u)[0][0] == (3, 1)                          # refused at the second proposal only
        u = np.zeros(n + 6)
        pq0 = [O.softmax(O.lm_logits(m, O.forward_full(m, toks[:n])[-1])) for m in (tm, dm)]
        u[n] = 0.95 * min(1.0, pq0[0][toks[n]] / pq0[1][toks[n]])  # still below the first proposal's ratio
        assert rounds(u)[0][0] == (3, 3)
        found += 1
    assert found >= 3


def test_sampled_speculation_follows_the_target_law(tiny):
    """One rejected two-token step with an 8-token vocabulary, sampled: the law of
    the regenerated step must be the target's, p(x) p(y | x), although the draft
    makes the proposals."""
    d, t, p = tiny["models"]
    ids = np.arange(8) * 100 + 3
    prompt = [int(x) for x in tiny["tokens"][0, :5]]

    dm, tm = _restricted(d, ids), _restricted(t, ids)
    T = 1.0
    px = O.softmax(O.lm_logits(tm, O.forward_full(tm, prompt)[-1]) / T)
    pyx = np.array([O.softmax(O.lm_logits(tm, O.forward_full(tm, prompt + [x])[-1]) / T) for x in range(8)])
    qx = O.softmax(O.lm_logits(dm, O.forward_full(dm, prompt)[-1]) / T)
    assert np.abs(px - qx).sum() > 0.2                         # the two models do differ
    expect = px[:, None] * pyx
    P = O.Params(delta=2.0, sep_id=-1, step_cap=2, max_steps=1, max_ctx=len(prompt) + 2,
                 temperature=T, top_p=1.0, sd_k=3)
    n = 4000
    r = np.random.default_rng(3)
    counts = np.zeros((8, 8))
    kept = 0
    L = len(prompt) + 2
    for _ in range(n):
        out = O.generate_sequence(dm, tm, p, prompt, r.random(L), r.random(L), np.zeros(1), P,
                                  u_prop=r.random(L), u_acc=r.random(L))
        x, y = out["tokens"][-2:]
        counts[x, y] += 1
        kept += out["records"][0]["sd_rounds"][0][1]
        assert out["records"][0]["sd_rounds"][0][0] == 1       # room for one proposal in a two-token step
    big = expect * n >= 5
    chi2 = np.sum((counts[big] - n * expect[big]) ** 2 / (n * expect[big]))
    dof = int(big.sum()) - 1
    assert chi2 < dof + 6 * np.sqrt(2 * dof)
    overlap = np.minimum(px, qx).sum()
    assert abs(kept / n - overlap) < 5 * np.sqrt(overlap * (1 - overlap) / n)
