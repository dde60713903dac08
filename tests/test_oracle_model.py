"""Pins of the CPU checker's transformer pieces against library routines,
identities and invariants (none of them its own formulas retyped)."""
import copy

import numpy as np
import pytest
import torch
import torch.nn.functional as TF

from oracle import rsd_oracle as O
from rsd_inputs import workload, model_weights_np

rng = np.random.default_rng(7)


def t64(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(torch.float64)


# ---------------------------------------------------------------- norm / mlp
def test_rmsnorm_matches_library_and_is_scale_invariant():
    x = rng.normal(size=(5, 96))
    g = rng.normal(size=96)
    got = O.rmsnorm(x, g, 1e-6)
    ref = TF.rms_norm(t64(x), (96,), weight=t64(g), eps=1e-6).numpy()
    assert np.allclose(got, ref, rtol=0, atol=1e-13)
    assert np.allclose(O.rmsnorm(37.0 * x, g, 0.0), O.rmsnorm(x, g, 0.0), atol=1e-12)
    # unit gain => unit root-mean-square
    y = O.rmsnorm(x, np.ones(96), 0.0)
    assert np.allclose(np.sqrt(np.mean(y * y, axis=-1)), 1.0, atol=1e-12)


def test_silu_and_softmax_match_library():
    x = rng.normal(size=1000) * 4
    assert np.allclose(O.silu(x), TF.silu(t64(x)).numpy(), atol=1e-14)
    assert O.silu(np.zeros(1))[0] == 0.0
    z = rng.normal(size=(7, 33)) * 10
    p = O.softmax(z)
    assert np.allclose(p.sum(-1), 1.0, atol=1e-14)
    assert np.allclose(p, torch.softmax(t64(z), -1).numpy(), atol=1e-15)


# ---------------------------------------------------------------- rope
def test_rope_is_a_complex_rotation():
    T, H, hd, theta = 6, 3, 16, 1e4
    x = rng.normal(size=(T, H, hd))
    pos = np.array([0, 1, 5, 17, 300, 4095])
    y = O.rope(x, pos, theta)
    # pair (i, i+hd/2) as a complex number, multiply by exp(i * pos * theta^(-2i/hd))
    zc = x[..., :hd // 2] + 1j * x[..., hd // 2:]
    freq = theta ** (-np.arange(hd // 2) * 2.0 / hd)
    rot = zc * np.exp(1j * pos[:, None, None] * freq[None, None, :])
    assert np.allclose(y[..., :hd // 2], rot.real, atol=1e-12)
    assert np.allclose(y[..., hd // 2:], rot.imag, atol=1e-12)
    assert np.allclose(O.rope(x, np.zeros(T, dtype=int), theta), x)
    assert np.allclose(np.linalg.norm(y, axis=-1), np.linalg.norm(x, axis=-1))


def test_rope_scores_depend_on_relative_position_only():
    hd = 32
    q = rng.normal(size=(1, 1, hd))
    k = rng.normal(size=(1, 1, hd))
    def score(pq, pk):
        return float(np.sum(O.rope(q, np.array([pq]), 1e4) * O.rope(k, np.array([pk]), 1e4)))
    assert abs(score(10, 3) - score(110, 103)) < 1e-10
    assert abs(score(10, 3) - score(10, 4)) > 1e-6


# ---------------------------------------------------------------- attention
def test_attention_rows_sum_to_one_and_are_causal():
    q = rng.normal(size=(4, 16))
    k = rng.normal(size=(10, 16))
    pos = np.array([6, 7, 8, 9])
    p = O.attention_probs(q, k, pos)
    assert np.allclose(p.sum(-1), 1.0, atol=1e-14)
    for i, pq in enumerate(pos):
        assert np.all(p[i, pq + 1:] == 0.0) and np.all(p[i, :pq + 1] > 0.0)


@pytest.mark.parametrize("H,Hkv", [(4, 4), (8, 2), (6, 1)])
def test_gqa_matches_library_attention(H, Hkv):
    T, hd = 9, 16
    q = rng.normal(size=(T, H, hd))
    k = rng.normal(size=(T, Hkv, hd))
    v = rng.normal(size=(T, Hkv, hd))
    got = O.gqa_attention(q, k, v, np.arange(T))
    # library routine: multi-head attention with each KV head repeated H/Hkv times
    kk = t64(k).repeat_interleave(H // Hkv, dim=1)
    vv = t64(v).repeat_interleave(H // Hkv, dim=1)
    ref = TF.scaled_dot_product_attention(t64(q).transpose(0, 1), kk.transpose(0, 1),
                                          vv.transpose(0, 1), is_causal=True).transpose(0, 1).numpy()
    assert np.allclose(got, ref, atol=1e-12)


def test_gqa_with_cached_prefix_matches_library():
    S, T, H, Hkv, hd = 13, 4, 4, 2, 8
    q = rng.normal(size=(T, H, hd))
    k = rng.normal(size=(S, Hkv, hd))
    v = rng.normal(size=(S, Hkv, hd))
    pos = np.arange(S - T, S)
    got = O.gqa_attention(q, k, v, pos)
    mask = torch.from_numpy(np.arange(S)[None, :] <= pos[:, None])
    kk = t64(k).repeat_interleave(2, dim=1).transpose(0, 1)
    vv = t64(v).repeat_interleave(2, dim=1).transpose(0, 1)
    ref = TF.scaled_dot_product_attention(t64(q).transpose(0, 1), kk, vv, attn_mask=mask).transpose(0, 1).numpy()
    assert np.allclose(got, ref, atol=1e-12)


# ---------------------------------------------------------------- whole forward
def torch_forward(s, w, tokens):
    """Independent evaluation with torch library ops (fp64): nn.functional
    linear / rms_norm / silu / scaled_dot_product_attention, rotary embedding
    through complex multiplication."""
    W = {k: t64(v) for k, v in w.items()}
    T = len(tokens)
    H, Hkv, hd = s.n_heads, s.n_kv_heads, s.head_dim
    h = TF.embedding(torch.tensor(tokens, dtype=torch.long), W["embed"])
    freq = torch.tensor(s.rope_theta, dtype=torch.float64) ** (-torch.arange(hd // 2, dtype=torch.float64) * 2 / hd)
    cis = torch.polar(torch.ones(T, hd // 2, dtype=torch.float64), torch.arange(T, dtype=torch.float64)[:, None] * freq)

    def rot(x):                       # x [T, heads, hd], pairs (i, i + hd/2)
        zc = torch.complex(x[..., :hd // 2], x[..., hd // 2:]) * cis[:, None, :]
        return torch.cat([zc.real, zc.imag], dim=-1)

    for l in range(s.n_layers):
        p = f"l{l}."
        a = TF.rms_norm(h, (s.d_model,), W[p + "attn_norm"], s.rms_eps)
        q = rot(TF.linear(a, W[p + "wq"]).view(T, H, hd)).transpose(0, 1)
        k = rot(TF.linear(a, W[p + "wk"]).view(T, Hkv, hd)).transpose(0, 1)
        v = TF.linear(a, W[p + "wv"]).view(T, Hkv, hd).transpose(0, 1)
        o = TF.scaled_dot_product_attention(q, k, v, is_causal=True, enable_gqa=True)
        h = h + TF.linear(o.transpose(0, 1).reshape(T, H * hd), W[p + "wo"])
        b = TF.rms_norm(h, (s.d_model,), W[p + "ffn_norm"], s.rms_eps)
        h = h + TF.linear(TF.silu(TF.linear(b, W[p + "w_gate"])) * TF.linear(b, W[p + "w_up"]), W[p + "w_down"])
    return TF.rms_norm(h, (s.d_model,), W["final_norm"], s.rms_eps)


@pytest.mark.parametrize("which", [0, 1, 2])
def test_forward_matches_library_built_transformer(tiny, which):
    m = tiny["models"][which]
    toks = [int(t) for t in tiny["tokens"][1, :24]]
    got = O.forward_full(m, toks)
    y = torch_forward(m.s, m._w, toks)
    assert np.allclose(got, y.numpy(), atol=1e-11)
    if m.s.head_kind == "lm":
        ref = TF.linear(y, t64(m._w["lm_head"])).numpy()
        assert np.allclose(O.lm_logits(m, got), ref, atol=1e-11)
    else:
        z = TF.linear(y[-1], t64(m._w["w_r"])[None, :]) + float(m._w["b_r"][0])
        assert abs(O.reward(m, got[-1]) - float(torch.sigmoid(z))) < 1e-13
        assert 0.0 < O.reward(m, got[-1]) < 1.0


def test_non_unit_gains_and_bias_are_used(tiny):
    """Random init has gains 1 and bias 0, which would hide a dropped gain or
    bias; perturb them and compare with the library-built model again."""
    m0 = tiny["models"][2]
    w = {k: np.array(v, copy=True) for k, v in m0._w.items()}
    r = np.random.default_rng(3)
    for k in w:
        if k.endswith("norm"):
            w[k] = (1.0 + 0.3 * r.normal(size=w[k].shape)).astype(np.float32)
    w["b_r"][0] = 0.37
    m = O.OracleModel(m0.s, w)
    toks = [int(t) for t in tiny["tokens"][0, :12]]
    got = O.forward_full(m, toks)
    y = torch_forward(m.s, w, toks)
    assert np.allclose(got, y.numpy(), atol=1e-11)
    z = TF.linear(y[-1], t64(w["w_r"])[None, :]) + float(w["b_r"][0])
    assert abs(O.reward(m, got[-1]) - float(torch.sigmoid(z))) < 1e-13


def test_incremental_cache_equals_full_recompute(tiny):
    m = tiny["models"][1]
    toks = [int(t) for t in tiny["tokens"][2, :32]]
    full = O.forward_full(m, toks)
    kv = O.KVCache(m.s, 64)
    parts = [O.forward_chunk(m, kv, toks[:5]), O.forward_chunk(m, kv, toks[5:6]),
             O.forward_chunk(m, kv, toks[6:20])]
    for t in toks[20:]:
        parts.append(O.forward_chunk(m, kv, [t]))
    assert np.max(np.abs(np.concatenate(parts) - full)) < 1e-12
    # truncate, then feed different tokens: equals a fresh run on the new sequence
    kv.truncate(10)
    alt = toks[:10] + [5, 6, 7]
    y = O.forward_chunk(m, kv, alt[10:])
    assert np.max(np.abs(y - O.forward_full(m, alt)[10:])) < 1e-12


def test_causality(tiny):
    m = tiny["models"][0]
    toks = [int(t) for t in tiny["tokens"][0, :16]]
    a = O.forward_full(m, toks)
    toks2 = list(toks)
    toks2[9] = (toks2[9] + 1) % 1000
    b = O.forward_full(m, toks2)
    assert np.array_equal(a[:9], b[:9]) and not np.allclose(a[9:], b[9:])


def test_zeroed_projections_leave_the_residual_alone(tiny):
    m0 = tiny["models"][0]
    w = {k: np.array(v, copy=True) for k, v in m0._w.items()}
    for l in range(m0.s.n_layers):
        w[f"l{l}.w_down"][:] = 0
        w[f"l{l}.wo"][:] = 0
    m = O.OracleModel(m0.s, w)
    toks = [3, 1, 4, 1, 5]
    e = w["embed"][toks].astype(np.float64)
    assert np.allclose(O.forward_full(m, toks), O.rmsnorm(e, np.ones(m0.s.d_model), m0.s.rms_eps), atol=1e-14)
    # zero only the MLP output: a one-token sequence attends to itself alone, so
    # each layer adds exactly wo @ (wv @ norm(h))
    w2 = {k: np.array(v, copy=True) for k, v in m0._w.items()}
    for l in range(m0.s.n_layers):
        w2[f"l{l}.w_down"][:] = 0
    m2 = O.OracleModel(m0.s, w2)
    h = w2["embed"][[7]].astype(np.float64)
    for l in range(m0.s.n_layers):
        a = TF.rms_norm(t64(h), (m0.s.d_model,), eps=m0.s.rms_eps).numpy()
        v = a @ w2[f"l{l}.wv"].astype(np.float64).T                       # [1, Hkv*hd]
        grp = m0.s.n_heads // m0.s.n_kv_heads
        o = v.reshape(m0.s.n_kv_heads, 1, m0.s.head_dim).repeat(grp, axis=1).reshape(1, -1)
        h = h + o @ w2[f"l{l}.wo"].astype(np.float64).T
    ref = TF.rms_norm(t64(h), (m0.s.d_model,), eps=m0.s.rms_eps).numpy()
    assert np.allclose(O.forward_full(m2, [7]), ref, atol=1e-13)


def test_bf16_weights_are_used_exactly():
    w = workload("cfg1", n_layers=1, vocab=256)
    ws = model_weights_np(w.seed, 0, w.draft)
    m = O.OracleModel(w.draft, ws)
    a = m.mat("l0.wq")
    assert a.dtype == np.float64
    assert np.array_equal(a.astype(np.float32), ws["l0.wq"])
    b = torch.from_numpy(ws["l0.wq"]).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(b, ws["l0.wq"])


def test_bf16_storage_rounding_is_nearest_even():
    r = np.random.default_rng(12)
    x = np.concatenate([r.normal(size=20000) * 1.3, r.normal(size=2000) * 1e-3, [0.0, 1.0, -2.5]])
    got = O.round_to_bf16(x)
    ref = torch.from_numpy(x).to(torch.float32).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(got, ref)
    # ties go to the even neighbour: 1 + 2^-8 lies halfway between 1 and 1 + 2^-7
    assert O.round_to_bf16(np.array([1.0 + 2.0 ** -8]))[0] == 1.0
    assert O.round_to_bf16(np.array([1.0 + 3 * 2.0 ** -8]))[0] == 1.0 + 2.0 ** -6
    assert np.max(np.abs(got - x) / np.maximum(np.abs(x), 1e-30)) <= 2.0 ** -8


def test_bf16_cache_rounds_what_is_stored_and_nothing_else(tiny):
    m = tiny["models"][1]
    toks = [int(t) for t in tiny["tokens"][1, :20]]
    kv = O.KVCache(m.s, 32, "bf16")
    y = O.forward_chunk(m, kv, toks[:12])
    for t in toks[12:]:
        y = np.concatenate([y, O.forward_chunk(m, kv, [t])])
    # every stored entry is a bf16 value, the result differs from the exact run by a bf16-sized amount,
    # and chunking does not matter (cache and recompute agree to fp64 rounding)
    assert np.array_equal(kv.k[:, :20], O.round_to_bf16(kv.k[:, :20]))
    assert np.array_equal(kv.v[:, :20], O.round_to_bf16(kv.v[:, :20]))
    exact = O.forward_full(m, toks)
    full = O.forward_full(m, toks, "bf16")
    assert np.max(np.abs(y - full)) < 1e-12
    d = np.max(np.abs(full - exact))
    assert 1e-5 < d < 5e-2
