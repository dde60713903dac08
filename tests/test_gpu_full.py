"""GPU checks at the full size of configuration 1 (bf16, batch 1, 28-layer
1.5B draft / 7B target / 1.5B reward model, vocabulary 151936), in the launch
configuration bench.py times.

The fp64 CPU checker can still evaluate the full-depth 1.5B shapes on the
256-token prompt (about 14 GB as fp64), so the draft's next-token logits and
the reward model's score are compared with it directly; the 7B target does not
fit and is covered by properties that hold at any size."""
import gc

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

TOL = 2e-2


@pytest.fixture(scope="module")
def full():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from rsd_inputs import workload
    from paper_2501_19324_amd import binding as R
    from paper_2501_19324_amd.harness import Session
    w = workload("cfg1")
    s = Session(w)
    yield dict(R=R, s=s, w=w, torch=torch)
    s.close()


@pytest.mark.parametrize("which", [0, 2])
def test_full_depth_prompt_against_checker(full, which):
    """Last-position logits of the draft (which = 0) and the reward of the
    reward model (which = 2) on the 256-token prompt, through the chunked
    prefill kernels and through 256 single-token iterations."""
    from oracle import rsd_oracle as O
    from rsd_inputs import model_weights_np
    R, s, w = full["R"], full["s"], full["w"]
    shape = w.shapes[which]
    n = int(s.prompt_len[0])
    toks = s.tokens_host[:, :n].copy()
    lens = np.array([n], np.int32)
    m = O.OracleModel(shape, model_weights_np(w.seed, which, shape, threads=16))
    y = O.forward_full(m, [int(t) for t in toks[0]], "bf16")
    ref = O.lm_logits(m, y[-1]) if which == 0 else np.array(O.reward(m, y[-1]))
    del m, y
    gc.collect()
    for chunk in (n, 1):
        out = R.rsd_forward(s.ctx, which, toks, lens, chunk)
        got = out[0, n - 1].cpu().numpy()
        err = float(np.max(np.abs(got - ref)))
        print(f"model {which} chunk {chunk}: max abs error {err:.2e}")
        assert err < (TOL if which == 0 else 1e-3), (which, chunk, err)
    s.reset()


def test_full_size_steps_properties(full):
    """Three reasoning steps at full size, twice: identical results, offsets and
    page tables consistent with the decisions, rewards inside (0, 1)."""
    R, s, w = full["R"], full["s"], full["w"]
    runs = []
    for _ in range(2):
        s.reset()
        recs, states = [], []
        for _i in range(3):
            recs.append(R.rsd_step(s.ctx))
            states.append(R.rsd_export_state(s.ctx, want_tokens=False))
        runs.append((recs, states, R.rsd_export_state(s.ctx)["tokens"].copy()))
    (ra, sa, ta), (rb, sb, tb) = runs
    assert np.array_equal(ta, tb)
    for x, y in zip(ra, rb):
        for k in x:
            assert np.array_equal(x[k], y[k]), k
    kv_t_prev = 0
    ctx = int(s.prompt_len[0])
    for g, st in zip(ra, sa):
        assert 0.0 < g["reward"][0] < 1.0
        assert g["accepted"][0] == g["own_accept"][0] == int(g["reward"][0] >= np.float32(w.delta))
        assert 1 <= g["draft_len"][0] <= w.step_cap and 1 <= g["final_len"][0] <= w.step_cap
        pre, ctx = ctx, ctx + int(g["final_len"][0])
        kd, kt, kp = (int(v) for v in st["kv_len"][:, 0])
        assert st["ctx_len"][0] == ctx
        if g["accepted"][0]:
            assert (kd, kt, kp) == (ctx - 1, kv_t_prev, ctx)
            assert np.array_equal(g["draft_tokens"], g["final_tokens"])
        else:
            assert (kd, kt, kp) == (pre, ctx - 1, pre)
        assert list(st["n_pages"][:, 0]) == [-(-v // 16) for v in (kd, kt, kp)]
        kv_t_prev = kt
    for mdl in range(3):
        pg = R.rsd_export_pages(s.ctx, mdl)
        used = pg["block_table"][pg["block_table"] >= 0]
        assert len(set(used.tolist())) == used.size and used.size + pg["free_pages"] == pg["pool_pages"]
