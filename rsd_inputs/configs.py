"""Workload definitions: model shapes and decoding limits of the five synthetic
configurations, plus the canonical weight-blob layout shared by every consumer.

All models are decoder-only transformers with RMSNorm, rotary embeddings
(rotate-half pairing), grouped-query attention, a SwiGLU MLP and an untied
output head; the reward model replaces the vocabulary head by one row and a
bias.  Nothing here evaluates a model.
"""
from __future__ import annotations

from dataclasses import dataclass, replace, field
from typing import Dict, List, Tuple

SEED_BASE = 25011932400


@dataclass(frozen=True)
class ModelShape:
    n_layers: int
    d_model: int
    n_heads: int
    n_kv_heads: int
    d_ffn: int
    vocab: int
    dtype: str = "bf16"          # "f32" | "bf16": storage type of weights and KV
    head_kind: str = "lm"        # "lm": lm_head[V,d] | "reward": w_r[d], b_r[1]
    rope_theta: float = 1.0e4
    rms_eps: float = 1.0e-6

    @property
    def head_dim(self) -> int:
        return self.d_model // self.n_heads

    @property
    def q_dim(self) -> int:
        return self.n_heads * self.head_dim

    @property
    def kv_dim(self) -> int:
        return self.n_kv_heads * self.head_dim

    @property
    def elt_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2

    @property
    def kv_bytes_per_token(self) -> int:
        return self.n_layers * 2 * self.kv_dim * self.elt_bytes

    def n_params(self) -> int:
        return blob_layout(self)[1]

    def decode_weight_bytes(self) -> int:
        """Bytes of weights one decode iteration has to read: everything but the
        embedding table (one row of it is read per token)."""
        emb = self.vocab * self.d_model
        return (self.n_params() - emb) * self.elt_bytes


def blob_layout(s: ModelShape) -> Tuple[List[Tuple[str, int, int, int]], int]:
    """Canonical order of the tensors of one model inside its weight blob.

    Returns ``([(name, rows, cols, offset_in_elements), ...], total_elements)``.
    Matrices are row-major ``[out, in]``; vectors have ``rows == 1``.
    """
    d, hd = s.d_model, s.head_dim
    out: List[Tuple[str, int, int, int]] = []
    off = 0

    def add(name: str, rows: int, cols: int) -> None:
        nonlocal off
        out.append((name, rows, cols, off))
        off += rows * cols

    add("embed", s.vocab, d)
    for l in range(s.n_layers):
        p = f"l{l}."
        add(p + "attn_norm", 1, d)
        add(p + "wq", s.n_heads * hd, d)
        add(p + "wk", s.n_kv_heads * hd, d)
        add(p + "wv", s.n_kv_heads * hd, d)
        add(p + "wo", d, s.n_heads * hd)
        add(p + "ffn_norm", 1, d)
        add(p + "w_gate", s.d_ffn, d)
        add(p + "w_up", s.d_ffn, d)
        add(p + "w_down", d, s.d_ffn)
    add("final_norm", 1, d)
    if s.head_kind == "lm":
        add("lm_head", s.vocab, d)
    else:
        add("w_r", 1, d)
        add("b_r", 1, 8)   # one bias value, padded to 8 elements to keep 16-byte alignment
    return out, off


@dataclass(frozen=True)
class Workload:
    name: str
    seed: int
    batch: int
    draft: ModelShape
    target: ModelShape
    prm: ModelShape
    prompt_len_min: int
    prompt_len_max: int
    step_cap: int
    max_steps: int
    temperature: float          # 0 => greedy
    top_p: float
    deltas: Tuple[float, ...]
    sep_id: int
    eos_id: int = -1
    sep_logit_bias: float = 0.0
    page_tokens: int = 16
    omega_kind: int = 0         # 0 binary step (Table 1, row 2)
    omega_a: float = 0.0
    omega_b: float = 0.0

    @property
    def max_ctx(self) -> int:
        return self.prompt_len_max + self.step_cap * self.max_steps

    @property
    def shapes(self) -> Tuple[ModelShape, ModelShape, ModelShape]:
        return (self.draft, self.target, self.prm)

    @property
    def delta(self) -> float:
        return self.deltas[0]


def _tiny(L, d, H, Hkv, F, head="lm"):
    return ModelShape(L, d, H, Hkv, F, 1024, dtype="f32", head_kind=head)


V_BIG = 151936
M_1P5B = ModelShape(28, 1536, 12, 2, 8960, V_BIG)
M_7B = ModelShape(28, 3584, 28, 4, 18944, V_BIG)
M_72B = ModelShape(80, 8192, 64, 8, 29568, V_BIG)


def _prm(s: ModelShape) -> ModelShape:
    return replace(s, head_kind="reward")


WORKLOADS: Dict[str, Workload] = {
    # config 0: tiny fp32, greedy, delta 0.5
    "cfg0": Workload("cfg0", SEED_BASE + 0, 4,
                     _tiny(2, 128, 4, 2, 512), _tiny(4, 256, 8, 2, 1024),
                     _tiny(2, 128, 4, 2, 512, "reward"),
                     32, 32, 16, 4, 0.0, 1.0, (0.5,), sep_id=1023),
    # config 1: bf16, batch 1, 1.5B / 7B / 1.5B-PRM, top-p 0.95 at T=0.7
    "cfg1": Workload("cfg1", SEED_BASE + 1, 1, M_1P5B, M_7B, _prm(M_1P5B),
                     256, 256, 64, 16, 0.7, 0.95, (0.7,), sep_id=V_BIG - 1),
    # config 2: batch 64, ragged prompts, delta sweep, greedy
    "cfg2": Workload("cfg2", SEED_BASE + 2, 64, M_1P5B, M_7B, _prm(M_1P5B),
                     128, 1024, 128, 32, 0.0, 1.0, (0.7, 0.0, 0.5, 0.9, 1.01),
                     sep_id=V_BIG - 1),
    # config 3: batch 16, 1.5B / 72B / 7B-PRM all resident
    "cfg3": Workload("cfg3", SEED_BASE + 3, 16, M_1P5B, M_72B, _prm(M_7B),
                     512, 512, 128, 16, 0.0, 1.0, (0.7,), sep_id=V_BIG - 1),
    # config 4: long context, batch 256, paged KV
    "cfg4": Workload("cfg4", SEED_BASE + 4, 256, M_1P5B, M_7B, _prm(M_1P5B),
                     1024, 1024, 128, 64, 0.0, 1.0, (0.5, 0.9), sep_id=V_BIG - 1),
}


def workload(name: str, **overrides) -> Workload:
    """Look a workload up; keyword overrides build a reduced variant, e.g.
    ``workload("cfg1", n_layers=2)`` keeps every width but uses two layers in
    each model (used by parity tests the CPU checker can finish quickly)."""
    w = WORKLOADS[name]
    n_layers = overrides.pop("n_layers", None)
    vocab = overrides.pop("vocab", None)
    if n_layers is not None or vocab is not None:
        def red(s: ModelShape) -> ModelShape:
            kw = {}
            if n_layers is not None:
                kw["n_layers"] = min(s.n_layers, n_layers)
            if vocab is not None:
                kw["vocab"] = vocab
            return replace(s, **kw)
        w = replace(w, draft=red(w.draft), target=red(w.target), prm=red(w.prm))
        if vocab is not None:
            w = replace(w, sep_id=vocab - 1)
    if overrides:
        w = replace(w, **overrides)
    return w
