"""The seeded input generators: determinism, ranges, and agreement of the NumPy
and torch implementations bit for bit."""
import numpy as np
import torch

from rsd_inputs import (workload, blob_layout, hash32_np, model_blob_np, model_blob_torch,
                        model_weights_np, prompt_lengths, prompt_tokens, uniforms,
                        bf16_bits_to_f32, f32_to_bf16_bits, normal_table)
from rsd_inputs.generate import hash32_int, _key


def test_hash_vector_matches_scalar():
    key = _key(123, 2, 7)
    idx = np.array([0, 1, 2, 65535, 2**31, 2**32 - 1, 1234567], dtype=np.uint64)
    got = hash32_np(idx, key)
    for i, g in zip(idx, got):
        assert int(g) == hash32_int(int(i), key)


def test_bf16_rounding_nearest_even():
    x = np.array([1.0, 1.0 + 2**-8, 1.0 + 2**-7, 1.0 + 3 * 2**-8, -0.3], dtype=np.float32)
    r = bf16_bits_to_f32(f32_to_bf16_bits(x))
    ref = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(r, ref)


def test_blob_numpy_equals_torch_bitwise():
    for name in ("cfg0",):
        w = workload(name)
        for which, s in enumerate(w.shapes):
            a = model_blob_np(w.seed, which, s)
            b = model_blob_torch(w.seed, which, s, "cpu", chunk=50000)
            assert np.array_equal(a, b.numpy())
    w = workload("cfg1", n_layers=1, vocab=512)
    s = w.draft
    a = model_blob_np(w.seed, 0, s)
    b = model_blob_torch(w.seed, 0, s, "cpu")
    assert np.array_equal(a, b.view(torch.int16).numpy().view(np.uint16))


def test_layout_is_contiguous_and_aligned():
    for name in ("cfg0", "cfg1", "cfg3"):
        for s in workload(name).shapes:
            layout, total = blob_layout(s)
            off = 0
            for _n, rows, cols, o in layout:
                assert o == off and (o * s.elt_bytes) % 16 == 0
                off += rows * cols
            assert off == total
    # wq, wk, wv follow one another, and so do w_gate, w_up: each group can be
    # read as one [out, in] matrix
    layout, _ = blob_layout(workload("cfg1").target)
    d = {n: (r, c, o) for n, r, c, o in layout}
    assert d["l0.wk"][2] == d["l0.wq"][2] + d["l0.wq"][0] * d["l0.wq"][1]
    assert d["l0.wv"][2] == d["l0.wk"][2] + d["l0.wk"][0] * d["l0.wk"][1]
    assert d["l0.w_up"][2] == d["l0.w_gate"][2] + d["l0.w_gate"][0] * d["l0.w_gate"][1]


def test_param_counts_match_model_sizes():
    w1, w3 = workload("cfg1"), workload("cfg3")
    assert abs(w1.draft.n_params() / 1e9 - 1.777) < 0.01      # 1.310 B + 2 x 0.233 B
    assert abs(w1.target.n_params() / 1e9 - 7.615) < 0.01
    assert abs(w3.target.n_params() / 1e9 - 72.70) < 0.05
    assert abs(w1.draft.decode_weight_bytes() / 1e9 - 3.09) < 0.01
    assert abs(w1.target.decode_weight_bytes() / 1e9 - 14.14) < 0.01
    assert w1.draft.kv_bytes_per_token == 28672 and w1.target.kv_bytes_per_token == 57344


def test_weight_distribution():
    w = workload("cfg0")
    ws = model_weights_np(w.seed, 1, w.target)
    a = ws["l0.w_gate"].astype(np.float64).ravel()
    assert abs(a.mean()) < 3 * 0.02 / np.sqrt(a.size) + 1e-5
    assert abs(a.std() - 0.02) < 2e-4
    assert abs(np.mean(np.abs(a) < 0.02) - 0.6827) < 0.01
    assert np.all(ws["l0.attn_norm"] == 1.0) and np.all(ws["final_norm"] == 1.0)
    t = normal_table("bf16")
    assert np.array_equal(t, bf16_bits_to_f32(f32_to_bf16_bits(t)))
    # different tensors and different models are different draws
    assert not np.array_equal(ws["l0.w_gate"], ws["l0.w_up"])
    assert not np.array_equal(ws["l0.w_gate"], ws["l1.w_gate"])


def test_prompts_and_uniforms():
    w = workload("cfg2")
    lens = prompt_lengths(w)
    assert lens.shape == (64,) and lens.min() >= 128 and lens.max() <= 1024 and len(set(lens.tolist())) > 32
    w0 = workload("cfg0", eos_id=1022)
    toks = prompt_tokens(w0)
    assert toks.shape == (4, w0.max_ctx)
    body = toks[:, :32]
    assert body.min() >= 0 and body.max() < 1022 and np.all(toks[:, 32:] == -1)
    u = uniforms(w, "U_DRAFT", 4096)
    assert u.dtype == np.float32 and u.min() >= 0.0 and u.max() < 1.0
    assert abs(u.mean() - 0.5) < 0.005
    assert np.array_equal(u, uniforms(w, "U_DRAFT", 4096))
    assert not np.array_equal(u, uniforms(w, "U_TARGET", 4096))
