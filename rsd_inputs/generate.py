"""Counter-based generators for weights, prompts and uniforms.

Every value is a pure function of ``(seed, stream, tensor/sequence id, index)``:

* a 32-bit integer mixing hash of ``index + key`` (two multiply/xor-shift
  rounds), where ``key`` folds seed, stream and id together;
* weights: the top 16 bits of the hash index a 65536-entry table holding the
  normal quantiles ``0.02 * Phi^-1((k + 1/2) / 65536)`` rounded once to the
  storage type (fp32 or bf16), so the values are N(0, 0.02) up to a 2^-16
  quantisation of the probability axis and are bit-identical wherever they are
  produced (NumPy on the host, integer torch ops on a device);
* prompt tokens and lengths: ``hash % range``; uniforms: top 24 bits * 2^-24.

Norm gains are 1 and the reward bias is 0, as at random initialisation.
"""
from __future__ import annotations

import numpy as np

from .configs import ModelShape, Workload, blob_layout

STREAMS = {"W_DRAFT": 1, "W_TARGET": 2, "W_PRM": 3, "PLEN": 4, "PTOK": 5,
           "U_DRAFT": 6, "U_TARGET": 7, "U_GATE": 8, "U_PROP": 9, "U_ACC": 10}
WEIGHT_STD = 0.02
_M32 = 0xFFFFFFFF


def _key(seed: int, stream: int, ident: int) -> int:
    """Fold seed, stream and id into one 32-bit key (splitmix64 finaliser)."""
    z = (seed * 0x9E3779B97F4A7C15 + stream * 0xBF58476D1CE4E5B9 + ident * 0x94D049BB133111EB) & 0xFFFFFFFFFFFFFFFF
    z ^= z >> 30
    z = (z * 0xBF58476D1CE4E5B9) & 0xFFFFFFFFFFFFFFFF
    z ^= z >> 27
    z = (z * 0x94D049BB133111EB) & 0xFFFFFFFFFFFFFFFF
    z ^= z >> 31
    return z & _M32


def hash32_np(index: np.ndarray, key: int) -> np.ndarray:
    """32-bit mixing hash of ``index + key`` (wrapping), elementwise."""
    x = (np.asarray(index).astype(np.uint64) + np.uint64(key)).astype(np.uint32)
    x ^= x >> np.uint32(16)
    x *= np.uint32(0x7FEB352D)
    x ^= x >> np.uint32(15)
    x *= np.uint32(0x846CA68B)
    x ^= x >> np.uint32(16)
    return x


def hash32_int(index: int, key: int) -> int:
    x = (index + key) & _M32
    x ^= x >> 16
    x = (x * 0x7FEB352D) & _M32
    x ^= x >> 15
    x = (x * 0x846CA68B) & _M32
    x ^= x >> 16
    return x


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest, ties to even); returns the 16-bit patterns."""
    b = np.asarray(x, dtype=np.float32).view(np.uint32)
    r = b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.asarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


_TABLE_CACHE = {}


def normal_table(dtype: str) -> np.ndarray:
    """65536 normal quantiles scaled by 0.02, as fp32 values exactly
    representable in ``dtype`` ("f32" or "bf16")."""
    if dtype not in _TABLE_CACHE:
        from scipy.special import ndtri
        q = ndtri((np.arange(65536, dtype=np.float64) + 0.5) / 65536.0) * WEIGHT_STD
        t = q.astype(np.float32)
        if dtype == "bf16":
            t = bf16_bits_to_f32(f32_to_bf16_bits(t))
        _TABLE_CACHE[dtype] = t
    return _TABLE_CACHE[dtype]


def _weight_stream(which: int) -> int:
    return (STREAMS["W_DRAFT"], STREAMS["W_TARGET"], STREAMS["W_PRM"])[which]


def weight_values_np(seed: int, which: int, tensor_idx: int, start: int, count: int, dtype: str,
                     out: np.ndarray = None) -> np.ndarray:
    """fp32 values (exact in ``dtype``) of elements ``[start, start+count)`` of
    tensor number ``tensor_idx`` (its position in the blob layout) of model
    ``which`` (0 draft, 1 target, 2 reward model)."""
    key = _key(seed, _weight_stream(which), tensor_idx)
    # index + key wraps modulo 2^32, exactly as in hash32_np
    x = np.arange(start, start + count, dtype=np.uint64).astype(np.uint32) if start + count > _M32 else \
        np.arange(start, start + count, dtype=np.uint32)
    x += np.uint32(key)
    x ^= x >> np.uint32(16)
    x *= np.uint32(0x7FEB352D)
    x ^= x >> np.uint32(15)
    x *= np.uint32(0x846CA68B)
    x ^= x >> np.uint32(16)
    x >>= np.uint32(16)
    return np.take(normal_table(dtype), x, out=out)


def fill_weights_np(seed: int, which: int, tensor_idx: int, dst: np.ndarray, dtype: str, threads: int = 1,
                    piece: int = 1 << 22) -> None:
    """Fill the flat fp32 array ``dst`` with a whole tensor, optionally with a
    pool of threads (NumPy releases the GIL inside its loops)."""
    n = dst.size
    spans = [(s, min(piece, n - s)) for s in range(0, n, piece)]
    if threads <= 1 or len(spans) == 1:
        for s, c in spans:
            weight_values_np(seed, which, tensor_idx, s, c, dtype, out=dst[s:s + c])
        return
    from concurrent.futures import ThreadPoolExecutor
    with ThreadPoolExecutor(threads) as ex:
        list(ex.map(lambda sc: weight_values_np(seed, which, tensor_idx, sc[0], sc[1], dtype, out=dst[sc[0]:sc[0] + sc[1]]), spans))


def _is_gain(name: str) -> bool:
    return name.endswith("norm")


def model_weights_np(seed: int, which: int, shape: ModelShape, threads: int = 1) -> dict:
    """All tensors of one model as a dict name -> fp32 array (values exact in
    the model's storage type)."""
    layout, _ = blob_layout(shape)
    out = {}
    for ti, (name, rows, cols, _off) in enumerate(layout):
        if _is_gain(name):
            a = np.ones(cols, dtype=np.float32)
        elif name == "b_r":
            a = np.zeros(cols, dtype=np.float32)
        else:
            a = np.empty(rows * cols, dtype=np.float32)
            fill_weights_np(seed, which, ti, a, shape.dtype, threads)
            a = a.reshape(cols) if rows == 1 else a.reshape(rows, cols)
        out[name] = a
    return out


def tensor_np(seed: int, which: int, shape: ModelShape, name: str) -> np.ndarray:
    """One named tensor (see :func:`blob_layout`) without building the rest."""
    layout, _ = blob_layout(shape)
    for ti, (n, rows, cols, _off) in enumerate(layout):
        if n == name:
            if _is_gain(n):
                return np.ones(cols, dtype=np.float32)
            if n == "b_r":
                return np.zeros(cols, dtype=np.float32)
            a = weight_values_np(seed, which, ti, 0, rows * cols, shape.dtype).reshape(rows, cols)
            return a.reshape(cols) if rows == 1 else a
    raise KeyError(name)


def model_blob_np(seed: int, which: int, shape: ModelShape) -> np.ndarray:
    """The weight blob of one model in canonical order: fp32 array for "f32"
    models, uint16 array of bf16 bit patterns for "bf16" models."""
    layout, total = blob_layout(shape)
    w = model_weights_np(seed, which, shape)
    flat = np.empty(total, dtype=np.float32)
    for name, rows, cols, off in layout:
        flat[off:off + rows * cols] = w[name].reshape(-1)
    if shape.dtype == "bf16":
        return f32_to_bf16_bits(flat)
    return flat


def model_blob_torch(seed: int, which: int, shape: ModelShape, device, chunk: int = 1 << 26):
    """Same blob as :func:`model_blob_np`, produced on ``device`` with integer
    torch ops (no host copy of the weights).  Returns a float32 or bfloat16
    tensor of ``total`` elements."""
    import torch

    layout, total = blob_layout(shape)
    tdtype = torch.float32 if shape.dtype == "f32" else torch.bfloat16
    blob = torch.empty(total, dtype=tdtype, device=device)
    table = torch.from_numpy(normal_table(shape.dtype)).to(device=device).to(tdtype)
    for ti, (name, rows, cols, off) in enumerate(layout):
        n = rows * cols
        dst = blob[off:off + n]
        if _is_gain(name):
            dst.fill_(1.0)
            continue
        if name == "b_r":
            dst.zero_()
            continue
        key = _key(seed, _weight_stream(which), ti)
        for s in range(0, n, chunk):
            c = min(chunk, n - s)
            x = torch.arange(s, s + c, dtype=torch.int64, device=device)
            x = (x + key) & _M32
            x = x ^ (x >> 16)
            x = (x * 0x7FEB352D) & _M32
            x = x ^ (x >> 15)
            x = (x * 0x846CA68B) & _M32
            x = x ^ (x >> 16)
            dst[s:s + c] = table[x >> 16]
            del x
    return blob


def prompt_lengths(w: Workload) -> np.ndarray:
    """Prompt length of every sequence: uniform integers in
    ``[prompt_len_min, prompt_len_max]``."""
    span = w.prompt_len_max - w.prompt_len_min + 1
    h = hash32_np(np.arange(w.batch, dtype=np.uint64), _key(w.seed, STREAMS["PLEN"], 0))
    return (w.prompt_len_min + (h % np.uint32(span))).astype(np.int32)


def prompt_tokens(w: Workload) -> np.ndarray:
    """``[batch, max_ctx]`` int32 token buffer: prompt tokens uniform over the
    vocabulary minus the separator and EOS ids, -1 beyond each prompt."""
    V = w.draft.vocab
    excluded = sorted({t for t in (w.sep_id, w.eos_id) if 0 <= t < V})
    lens = prompt_lengths(w)
    toks = np.full((w.batch, w.max_ctx), -1, dtype=np.int32)
    for b in range(w.batch):
        h = hash32_np(np.arange(int(lens[b]), dtype=np.uint64), _key(w.seed, STREAMS["PTOK"], b))
        t = (h % np.uint32(V - len(excluded))).astype(np.int64)
        for e in excluded:           # ascending: skip over each excluded id
            t = t + (t >= e)
        toks[b, :lens[b]] = t.astype(np.int32)
    return toks


def uniforms(w: Workload, stream: str, n_cols: int) -> np.ndarray:
    """``[batch, n_cols]`` fp32 uniforms in [0, 1) with 24 random bits each."""
    out = np.empty((w.batch, n_cols), dtype=np.float32)
    for b in range(w.batch):
        h = hash32_np(np.arange(n_cols, dtype=np.uint64), _key(w.seed, STREAMS[stream], b))
        out[b] = (h >> np.uint32(8)).astype(np.float32) * np.float32(2.0 ** -24)
    return out


def weights_from_blob(blob: np.ndarray, shape: ModelShape) -> dict:
    """Split a blob (fp32 array, or uint16 bf16 bit patterns) into the dict of
    fp32 tensors :func:`model_weights_np` returns (views where possible)."""
    layout, total = blob_layout(shape)
    assert blob.size == total
    out = {}
    for name, rows, cols, off in layout:
        a = blob[off:off + rows * cols]
        if a.dtype == np.uint16:
            a = bf16_bits_to_f32(a)
        out[name] = a.reshape(cols) if rows == 1 else a.reshape(rows, cols)
    return out
