"""Pins of the CPU checker's process Best-of-N procedure (Section 3, "Baselines":
sample N candidate steps, commit the one with the highest reward): reductions to
plain decoding, brute force on the candidates, invariance under a permutation of
the candidate streams, and the closed-form law of the maximum of N draws."""
import numpy as np
import pytest

from oracle import rsd_oracle as O

MIX = dict(temperature=0.7, top_p=0.8, sep_logit_bias=3.5)      # the paper's sampling setting for this procedure


def params(w, **kw):
    base = dict(delta=0.0, sep_id=w.sep_id, step_cap=w.step_cap, max_steps=w.max_steps, max_ctx=w.max_ctx,
                eos_id=w.eos_id, temperature=w.temperature, top_p=w.top_p, sep_logit_bias=w.sep_logit_bias)
    base.update(kw)
    return O.Params(**base)


def streams(tiny, b, n):
    """Candidate uniform streams of sequence b: n rows of per-position uniforms."""
    from rsd_inputs import uniforms
    from dataclasses import replace
    w = replace(tiny["w"], batch=tiny["w"].batch * n)
    return uniforms(w, "U_DRAFT", w.max_ctx)[b * n:(b + 1) * n]


def test_one_candidate_is_plain_decoding_with_the_base_model(tiny):
    d, t, p = tiny["models"]
    w = tiny["w"]
    for b in range(2):
        prompt = tiny["tokens"][b, :tiny["lens"][b]]
        u = streams(tiny, b, 1)
        P = params(w, **MIX)
        out = O.generate_sequence_bon(d, p, prompt, u, P, 1)
        n_new = len(out["tokens"]) - len(prompt)
        assert n_new > w.step_cap                         # several steps were taken
        plain = O.decode_plain(d, prompt, u[0], P, n_new)
        assert out["tokens"][len(prompt):] == plain
        assert all(r["chosen"] == 0 for r in out["records"])
        # and it is the RSD loop with a gate that accepts everything (delta <= 0)
        rsd = O.generate_sequence(d, t, p, prompt, u[0], u[0], np.zeros(w.max_steps), params(w, delta=-1.0, **MIX))
        assert rsd["tokens"] == out["tokens"]


def test_equal_rewards_take_the_first_candidate(tiny):
    """A reward model with a zero head scores everything 1/2: candidate 0 wins every step, so the
    run equals the one-candidate run on stream 0."""
    d, _, p = tiny["models"]
    w = tiny["w"]
    wz = dict(p._w)
    wz["w_r"] = np.zeros_like(p._w["w_r"])
    pz = O.OracleModel(p.s, wz)
    prompt = tiny["tokens"][1, :tiny["lens"][1]]
    u = streams(tiny, 1, 4)
    P = params(w, **MIX)
    out = O.generate_sequence_bon(d, pz, prompt, u, P, 4)
    one = O.generate_sequence_bon(d, pz, prompt, u[:1], P, 1)
    assert out["tokens"] == one["tokens"]
    assert all(r["chosen"] == 0 and np.allclose(r["rewards"], 0.5, atol=0, rtol=0) for r in out["records"])


def test_candidates_are_independent_continuations_and_the_best_is_committed(tiny):
    """Brute force: candidate n of a step is what plain decoding with stream n produces from the
    committed context (cut at the step's end), its reward is the reward model's score of context +
    candidate, and the committed step is the arg max."""
    d, _, p = tiny["models"]
    w = tiny["w"]
    N = 3
    prompt = [int(x) for x in tiny["tokens"][2, :tiny["lens"][2]]]
    u = streams(tiny, 2, N)
    P = params(w, **MIX)
    out = O.generate_sequence_bon(d, p, prompt, u, P, N)
    ctx = list(prompt)
    chosen = []
    for r in out["records"]:
        assert r["ctx_pre"] == len(ctx)
        for n in range(N):
            cand = r["candidates"][n]
            assert O.decode_plain(d, ctx, u[n], P, len(cand)) == cand
            ends = [t == P.sep_id or t == P.eos_id for t in cand]
            assert not any(ends[:-1]) and (ends[-1] or len(cand) == P.step_cap or len(ctx) + len(cand) == P.max_ctx)
            assert r["rewards"][n] == O.reward(p, O.forward_full(p, ctx + cand)[-1])
        best = max(range(N), key=lambda n: (np.float32(r["rewards"][n]), -n))
        assert r["chosen"] == best and r["final_tokens"] == r["candidates"][best]
        chosen.append(best)
        ctx += r["final_tokens"]
        assert r["ctx_len"] == len(ctx) and r["kv_len"] == [len(ctx) - 1, 0, len(ctx)]
    assert ctx == out["tokens"]
    assert len(set(chosen)) > 1                           # not always the same candidate
    assert len(set(tuple(c) for c in out["records"][0]["candidates"])) == N      # the candidates differ


def test_permuting_the_candidate_streams_permutes_the_candidates_only(tiny):
    d, _, p = tiny["models"]
    w = tiny["w"]
    N = 4
    prompt = tiny["tokens"][0, :tiny["lens"][0]]
    u = streams(tiny, 0, N)
    P = params(w, **MIX)
    a = O.generate_sequence_bon(d, p, prompt, u, P, N)
    perm = np.array([2, 0, 3, 1])
    b = O.generate_sequence_bon(d, p, prompt, u[perm], P, N)
    assert a["tokens"] == b["tokens"]
    for ra, rb in zip(a["records"], b["records"]):
        r32 = np.float32(ra["rewards"])
        assert int((r32 == r32.max()).sum()) == 1                       # the arg max is unique (no tie to break by index)
        assert [ra["candidates"][perm[i]] for i in range(N)] == rb["candidates"]
        assert perm[rb["chosen"]] == ra["chosen"]


def test_eos_and_limits(tiny):
    """EOS ends the sequence only when the committed step holds it (a candidate that was not chosen
    may hold it without effect); the context and step limits end it as in the RSD loop."""
    d, _, p = tiny["models"]
    w = tiny["w"]
    prompt = tiny["tokens"][3, :tiny["lens"][3]]
    u = streams(tiny, 3, 2)
    base = O.generate_sequence_bon(d, p, prompt, u, params(w, **MIX), 2)
    assert base["finished"] == O.FIN_MAX_STEPS and len(base["records"]) == w.max_steps
    seen_end = seen_ignored = False
    tried = sorted({t for r in base["records"] for c in r["candidates"] for t in c if t != w.sep_id})[:40]
    for eos in tried:
        out = O.generate_sequence_bon(d, p, prompt, u, params(w, eos_id=int(eos), **MIX), 2)
        for i, r in enumerate(out["records"]):
            last = i == len(out["records"]) - 1
            for c in r["candidates"]:
                assert eos not in c[:-1]                   # a candidate stops right after EOS
            if eos in r["final_tokens"]:
                assert last and out["finished"] == O.FIN_EOS and r["final_tokens"][-1] == eos
                seen_end = True
            else:
                assert not (last and out["finished"] == O.FIN_EOS)
                if any(eos in c for c in r["candidates"]) and not last:
                    seen_ignored = True
    assert seen_end and seen_ignored
    short = O.generate_sequence_bon(d, p, prompt, u, params(w, max_ctx=len(prompt) + 5, **MIX), 2)
    assert short["finished"] == O.FIN_MAX_CTX and len(short["tokens"]) == len(prompt) + 5


@pytest.mark.parametrize("N", [1, 3])
def test_one_token_steps_follow_the_law_of_the_best_of_n_draws(tiny, N):
    """With one-token steps the committed token is the best-scored of N independent draws from P_m:
    with the outcomes ordered by reward and F the distribution function of P_m in that order,
    P(committed = y) = F(y)^N - F(y-)^N.  (Vocabulary cut to 8 ids as in the RSD loop's test.)"""
    d, _, p = tiny["models"]
    ids = np.arange(8) * 100 + 3
    prompt = [int(x) for x in tiny["tokens"][0, :6]]
    wv = dict(d._w)
    wv["lm_head"] = d._w["lm_head"][ids]
    dm = O.OracleModel(d.s, wv)
    wp = dict(p._w)
    emb = np.array(p._w["embed"], copy=True)
    emb[:len(ids)] = p._w["embed"][ids]
    wp["embed"] = emb
    pm = O.OracleModel(p.s, wp)
    p_m = O.softmax(O.lm_logits(dm, O.forward_full(dm, prompt)[-1]))
    rew = np.array([O.reward(p, O.forward_full(p, prompt + [int(i)])[-1]) for i in ids])
    assert len(set(np.float32(rew))) == len(ids)
    order = np.argsort(rew)
    F = np.cumsum(p_m[order])
    expect = np.empty(len(ids))
    expect[order] = F ** N - np.concatenate([[0.0], F[:-1]]) ** N
    assert abs(expect.sum() - 1) < 1e-12
    P = O.Params(delta=0.0, sep_id=0, step_cap=1, max_steps=1, max_ctx=len(prompt) + 1, temperature=1.0, top_p=1.0)
    n = 2500
    r = np.random.default_rng(6)
    counts = np.zeros(len(ids))
    for _ in range(n):
        out = O.generate_sequence_bon(dm, pm, prompt, r.random((N, len(prompt) + 1)), P, N)
        counts[out["tokens"][-1]] += 1
    chi2 = np.sum((counts - n * expect) ** 2 / (n * expect))
    assert chi2 < 35.0                                   # 7 dof: P(chi2 > 35) ~ 1e-5
