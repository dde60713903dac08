"""The timing probes bench.py reports from (rsd_probe_start / rsd_probe_read / rsd_probe_clock): the accounting of
algorithmic flops and bytes is exact, the times are positive, and the shader clock read inside the probed
many-row GEMM is a plausible clock of this part.  No numerics here: the same passes are compared with the
checker in test_gpu_bf16.py."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

PREFILL, DECODE = 1, 0
OP_GATE_UP, OP_DOWN = 2, 3


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2501_19324_amd import binding as R
    from paper_2501_19324_amd.harness import Session
    return dict(R=R, Session=Session)


def small_workload(batch):
    from rsd_inputs import workload
    return workload("cfg1", n_layers=2, vocab=4096, batch=batch, prompt_len_min=20, prompt_len_max=70, step_cap=8,
                    max_steps=3, temperature=0.0, top_p=1.0, deltas=(0.6,))


def test_chunked_pass_probe_counts_flops_and_reads_the_clock(gpu):
    R = gpu["R"]
    w = small_workload(4)
    s = gpu["Session"](w)
    T = 80
    lens = np.full(4, T, dtype=np.int32)
    toks = np.random.default_rng(5).integers(0, w.draft.vocab, size=(4, T)).astype(np.int32)
    prm = 2
    shape = w.shapes[prm]
    R.rsd_probe_start(s.ctx, 0, prm, PREFILL, OP_GATE_UP, 64, 1)
    R.rsd_probe_start(s.ctx, 1, prm, PREFILL, OP_DOWN, 64, 1)
    R.rsd_forward(s.ctx, prm, toks, lens, T)        # one chunked pass of 4 x 80 = 320 rows: the many-row GEMM
    clk = [R.rsd_probe_clock(s.ctx, slot) for slot in (0, 1)]
    rec = [R.rsd_probe_read(s.ctx, slot) for slot in (0, 1)]
    rows, d, F, L = 4 * T, shape.d_model, shape.d_ffn, shape.n_layers
    assert rec[0]["n"] == L and rec[1]["n"] == L
    assert rec[0]["total_flops"] == L * 2 * rows * (2 * F) * d
    assert rec[1]["total_flops"] == L * 2 * rows * d * F
    for r, c in zip(rec, clk):
        assert r["total_ms"] > 0
        assert c["launches"] == r["n"]
        mhz = c["shader_ticks"] / c["ref_ticks"] * 100.0
        print(f"shader clock inside the probed GEMM: {mhz:.0f} MHz over {c['launches']} launches")
        assert 50.0 < mhz < 3000.0          # a clock, not garbage; the value itself is a measurement, not a contract
    # a second arming starts from zero, and a pass of few rows (the weight-streaming kernels) reports no clock
    R.rsd_probe_start(s.ctx, 0, prm, PREFILL, OP_GATE_UP, 64, 1)
    R.rsd_forward(s.ctx, prm, toks[:, :8].copy(), np.full(4, 8, dtype=np.int32), 8)       # 32 rows
    c = R.rsd_probe_clock(s.ctx, 0)
    r = R.rsd_probe_read(s.ctx, 0)
    assert r["n"] == L and c["launches"] == 0 and c["shader_ticks"] == 0
    s.close()
