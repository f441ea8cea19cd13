"""Seeded synthetic inputs for the denoise-step path: model shapes, weights, tokens, KV fill.

This module only draws and packs numbers.  It holds none of the method's arithmetic (no norm,
no attention, no softmax, no selection), so both the CPU oracle's tests and the HIP path's tests
and benchmark may take their inputs from it.  Everything is a pure function of (seed, tensor id).

Storage conventions
  * "f32" tensors are numpy float32 arrays.
  * "bf16" tensors are numpy uint16 arrays holding bfloat16 bit patterns (round-to-nearest-even of
    the float32 draw, done once here so that every consumer sees identical values).
  * Linear weights are [out_features, in_features], row-major (in_features contiguous).
"""
from __future__ import annotations

import dataclasses
from concurrent.futures import ThreadPoolExecutor

import numpy as np


@dataclasses.dataclass(frozen=True)
class ModelShape:
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ff: int
    vocab: int
    mask_id: int
    rms_eps: float = 1e-5
    rope_base: float = 10000.0
    dtype: str = "bf16"            # "f32" or "bf16": weights, activations handed between kernels, KV
    lm_head_scale: float = 1.0     # multiplies the N(0, 0.02) draw of the LM head
    name: str = ""

    def with_layers(self, n_layers: int) -> "ModelShape":
        return dataclasses.replace(self, n_layers=n_layers)


# The three architectures the workloads are quoted on.
TINY = ModelShape(2, 256, 4, 4, 64, 688, 4096, 4095, dtype="f32", lm_head_scale=8.0, name="tiny")
LLADA_8B = ModelShape(32, 4096, 32, 32, 128, 12288, 126464, 126463, name="llada8b")
DREAM_7B = ModelShape(28, 3584, 28, 4, 128, 18944, 152064, 152063, name="dream7b")

# tensor ids: global tensors use layer = -1
_GLOBAL_IDS = {"tok_emb": 1, "lm_head": 2}
_LAYER_IDS = {"wq": 1, "wk": 2, "wv": 3, "wo": 4, "w_gate": 5, "w_up": 6, "w_down": 7}


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    rounded = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns (uint16) to the float32 values they denote (exact)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_bf16(a: np.ndarray) -> np.ndarray:
    """Values of `a` after a round trip through bfloat16 (nearest even), as float64."""
    return bf16_bits_to_f32(_to_store(np.ascontiguousarray(a, dtype=np.float32), "bf16")).astype(np.float64)


def as_float(a: np.ndarray) -> np.ndarray:
    """Float view of a stored tensor: uint16 means bf16 bits, anything else is returned as is."""
    return bf16_bits_to_f32(a) if a.dtype == np.uint16 else a


def _rng(seed: int, layer: int, tid: int, chunk: int = 0) -> np.random.Generator:
    """Counter-based stream for (seed, layer, tensor id, chunk): Philox keyed by the first three,
    with the chunk number in the high word of its counter."""
    key = [int(seed), (int(layer) + 1) * 64 + int(tid)]
    return np.random.Generator(np.random.Philox(key=key, counter=[0, 0, int(chunk), 0]))


_CHUNK_ELEMS = 1 << 22
_POOL = ThreadPoolExecutor(max_workers=8)


def _to_store(w: np.ndarray, dtype: str) -> np.ndarray:
    if dtype != "bf16":
        return w
    import torch  # bf16 rounding (nearest even) of a float32 buffer; same bits as f32_to_bf16_bits
    return torch.from_numpy(w).to(torch.bfloat16).view(torch.uint16).numpy()


def _draw(seed, layer, tid, shape, std, dtype):
    """N(0, std) tensor, drawn in independent row chunks (so large tensors fill on several threads)."""
    rows = int(shape[0])
    per_row = int(np.prod(shape[1:], dtype=np.int64)) if len(shape) > 1 else 1
    rows_per_chunk = max(1, _CHUNK_ELEMS // per_row)
    w = np.empty(shape, dtype=np.float32)

    def fill(c):
        r0 = c * rows_per_chunk
        r1 = min(rows, r0 + rows_per_chunk)
        _rng(seed, layer, tid, c).standard_normal(out=w[r0:r1], dtype=np.float32)
        w[r0:r1] *= np.float32(std)

    n_chunks = (rows + rows_per_chunk - 1) // rows_per_chunk
    if n_chunks == 1:
        fill(0)
    else:
        list(_POOL.map(fill, range(n_chunks)))
    return _to_store(w, dtype)


def _ones(shape, dtype):
    return _to_store(np.ones(shape, dtype=np.float32), dtype)


def layer_tensor_shapes(ms: ModelShape) -> dict:
    d, hq, hkv, dh, f = ms.d_model, ms.n_q_heads, ms.n_kv_heads, ms.head_dim, ms.d_ff
    return {"wq": (hq * dh, d), "wk": (hkv * dh, d), "wv": (hkv * dh, d), "wo": (d, hq * dh),
            "w_gate": (f, d), "w_up": (f, d), "w_down": (d, f)}


def make_layer(ms: ModelShape, seed: int, layer: int) -> dict:
    """One transformer layer: matrices N(0, 0.02), norm gains 1."""
    out = {n: _draw(seed, layer, _LAYER_IDS[n], s, 0.02, ms.dtype)
           for n, s in layer_tensor_shapes(ms).items()}
    out["attn_norm"] = _ones((ms.d_model,), ms.dtype)
    out["mlp_norm"] = _ones((ms.d_model,), ms.dtype)
    return out


def make_globals(ms: ModelShape, seed: int) -> dict:
    """Embedding, final norm gain and (untied) LM head."""
    g = {"tok_emb": _draw(seed, -1, _GLOBAL_IDS["tok_emb"], (ms.vocab, ms.d_model), 0.02, ms.dtype),
         "lm_head": _draw(seed, -1, _GLOBAL_IDS["lm_head"], (ms.vocab, ms.d_model),
                          0.02 * ms.lm_head_scale, ms.dtype),
         "final_norm": _ones((ms.d_model,), ms.dtype)}
    return g


class Weights:
    """All tensors of a model, generated on first use and cached (or not, for 8B-scale shapes)."""

    def __init__(self, ms: ModelShape, seed: int, cache_layers: bool = True):
        self.ms, self.seed, self.cache_layers = ms, seed, cache_layers
        self._layers: dict[int, dict] = {}
        self._globals: dict | None = None

    def layer(self, l: int) -> dict:
        if l in self._layers:
            return self._layers[l]
        lw = {n: _draw(self.seed, l, _LAYER_IDS[n], shp, 0.02, self.ms.dtype)
              for n, shp in layer_tensor_shapes(self.ms).items()}
        lw["attn_norm"] = _ones((self.ms.d_model,), self.ms.dtype)
        lw["mlp_norm"] = _ones((self.ms.d_model,), self.ms.dtype)
        if self.cache_layers:
            self._layers[l] = lw
        return lw

    def globals(self) -> dict:
        if self._globals is None:
            self._globals = make_globals(self.ms, self.seed)
        return self._globals

    def __getitem__(self, name: str) -> np.ndarray:
        return self.globals()[name]


def random_tokens(ms: ModelShape, seed: int, n: int, stream: int = 0) -> np.ndarray:
    """n token ids uniform over 0..vocab-2 (never the mask id, which is vocab-1 in every shape here)."""
    hi = ms.vocab - 1 if ms.mask_id == ms.vocab - 1 else ms.vocab
    t = _rng(seed, -1, 16 + stream).integers(0, hi, size=n, dtype=np.int64).astype(np.int32)
    if ms.mask_id != ms.vocab - 1:
        t[t == ms.mask_id] = (ms.mask_id + 1) % ms.vocab
    return t


def masked_block(ms: ModelShape, seed: int, q: int, n_masked: int, stream: int = 0) -> np.ndarray:
    """A query block of q tokens: a seeded random subset of n_masked positions holds the mask id,
    the others hold uniform random ids."""
    blk = random_tokens(ms, seed, q, stream=32 + stream)
    pos = _rng(seed, -1, 48 + stream).permutation(q)[:n_masked]
    blk[pos] = ms.mask_id
    return blk


def random_kv(ms: ModelShape, seed: int, layer: int, seq: int, n_tokens: int) -> tuple[np.ndarray, np.ndarray]:
    """Directly drawn N(0,1) K and V for a prefix of n_tokens: [n_tokens, n_kv_heads, head_dim]
    (stands in for a prefilled cache where the prefill itself is too large for the CPU oracle)."""
    shape = (n_tokens, ms.n_kv_heads, ms.head_dim)
    out = []
    for which in (0, 1):
        key = [int(seed), (1 << 40) + (int(layer) << 24) + (int(seq) << 1) + which]
        a = np.random.Generator(np.random.Philox(key=key)).standard_normal(shape, dtype=np.float32)
        out.append(_to_store(a, ms.dtype))
    return out[0], out[1]


def device_weights(ms, torch, device, seed):
    """Random-init weights of the architecture, drawn on the device (never aliased between layers)."""
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    dt = torch.bfloat16 if ms.dtype == "bf16" else torch.float32

    def mat(rows, cols, std=0.02):
        return (torch.randn(rows, cols, generator=gen, device=device, dtype=torch.float32) * std).to(dt)

    d, dq, dkv, F = ms.d_model, ms.n_q_heads * ms.head_dim, ms.n_kv_heads * ms.head_dim, ms.d_ff
    ones = lambda: torch.ones(d, device=device, dtype=dt)
    g = {"tok_emb": mat(ms.vocab, d), "lm_head": mat(ms.vocab, d, 0.02 * ms.lm_head_scale), "final_norm": ones()}
    layers = []
    for _ in range(ms.n_layers):
        layers.append({"attn_norm": ones(), "wq": mat(dq, d), "wk": mat(dkv, d), "wv": mat(dkv, d),
                       "wo": mat(d, dq), "mlp_norm": ones(), "w_gate": mat(F, d), "w_up": mat(F, d),
                       "w_down": mat(d, F)})
    return g, layers
