"""Synthetic early-exit (EE) transformer: configuration and seeded weights.

The paper evaluates trained EE checkpoints (its Evaluation Methodology
section); none are available here, so a random-init model of the same
architecture stands in.  Weights come from a counter-based, integer-exact
generator so that a separately written device kernel can produce the very same
bits without any code being shared:

    GOLD      = 0x9E3779B97F4A7C15
    mix64(z)  : z ^= z >> 30; z *= 0xBF58476D1CE4E5B9;
                z ^= z >> 27; z *= 0x94D049BB133111EB; z ^= z >> 31
    key       = mix64(mix64(seed) ^ ((tensor_id << 32) | layer))
    word_j(e) = mix64(key + (3*e + j + 1) * GOLD)            j = 0, 1, 2
    s(e)      = sum of the twelve 16-bit lanes of word_0..2   (Irwin-Hall, n=12)
    n(e)      = float32(s(e) - 393210) * scale                (ONE fp32 multiply)
    scale     = float32(float32(sigma) * float32(gamma)) * 2**-16

`e` is the row-major element index in the tensor's logical shape.  The lane sum
has mean 393210 and standard deviation sqrt(65536**2 - 1) ~= 65536, so n(e) is
approximately N(0, (sigma*gamma)**2).  Norm gains are `1 + n(e)` (one fp32
add).  In bf16 configurations every value is then rounded to bf16 with
round-to-nearest-even on the bit pattern.  No transcendental function is used.
"""
from __future__ import annotations

import dataclasses
from concurrent.futures import ThreadPoolExecutor
from typing import Dict, Tuple

import numpy as np

GOLD = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_LANE_MEAN = 6 * 65535  # 393210

# tensor ids (part of the generator's key; the device generator uses the same numbers)
TENSOR_IDS: Dict[str, int] = {
    "emb": 0, "head": 1, "gfinal": 2,
    "g1": 3, "wq": 4, "wk": 5, "wv": 6, "wo": 7,
    "g2": 8, "wgate": 9, "wup": 10, "wdown": 11,
    "aux_g": 12, "aux_a": 13, "aux_b": 14,
}
GLOBAL_TENSORS = ("emb", "head", "gfinal")
LAYER_TENSORS = ("g1", "wq", "wk", "wv", "wo", "g2", "wgate", "wup", "wdown")
# auxiliary low-rank exit heads (cfg.head_rank > 0): one set per early exit, looked up with the exit
# index in the layer slot (0 = L_d, 1 = L_i, 2.. = the further verifier exits)
EXIT_TENSORS = ("aux_g", "aux_a", "aux_b")
GAIN_TENSORS = ("gfinal", "g1", "g2", "aux_g")
DAMPED_TENSORS = ("wo", "wdown")  # scaled by gamma[group of the layer]; aux_b by gamma[exit index]


@dataclasses.dataclass(frozen=True)
class EEConfig:
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    exit_draft: int          # L_d : layers 1..L_d form group G1
    exit_inter: int          # L_i : layers L_d+1..L_i form G2; L_i+1..L_f form G3
    rope_theta: float = 10000.0
    rms_eps: float = 1e-5
    dtype: str = "f32"       # "f32" | "bf16"
    sigma: float = 0.02
    gamma: Tuple[float, float, float] = (1.0, 1.0, 1.0)
    head_rank: int = 0       # > 0: every early exit carries a low-rank adapter of this rank in front of the shared head
    exit_extra: Tuple[int, ...] = ()   # further intermediate verifier exits between L_i and L_f (strictly increasing)

    def __post_init__(self):
        assert 0 < self.exit_draft < self.exit_inter < self.n_layers
        assert self.n_q_heads % self.n_kv_heads == 0
        assert self.head_dim % 2 == 0
        assert self.dtype in ("f32", "bf16")
        assert self.head_rank >= 0 and (self.dtype == "f32" or self.head_rank % 32 == 0)
        ex = (self.exit_inter,) + tuple(self.exit_extra) + (self.n_layers,)
        assert len(self.exit_extra) <= 4 and all(a < b for a, b in zip(ex, ex[1:]))

    @property
    def exit_full(self) -> int:
        return self.n_layers

    def group_of_layer(self, layer: int) -> int:
        """0-based layer index -> 0 (G1), 1 (G2) or 2 (G3)."""
        if layer < self.exit_draft:
            return 0
        if layer < self.exit_inter:
            return 1
        return 2

    def group_layers(self, g: int) -> range:
        bounds = (0, self.exit_draft, self.exit_inter, self.n_layers)
        return range(bounds[g], bounds[g + 1])


def tiny_config(**kw) -> EEConfig:
    base = dict(n_layers=4, d_model=256, n_q_heads=4, n_kv_heads=4, head_dim=64,
                d_ffn=688, vocab=1024, exit_draft=1, exit_inter=2,
                rope_theta=10000.0, dtype="f32")
    base.update(kw)
    return EEConfig(**base)


def llama8b_config(**kw) -> EEConfig:
    base = dict(n_layers=32, d_model=4096, n_q_heads=32, n_kv_heads=8, head_dim=128,
                d_ffn=14336, vocab=128256, exit_draft=4, exit_inter=16,
                rope_theta=500000.0, dtype="bf16")
    base.update(kw)
    return EEConfig(**base)


def llama70b_config(**kw) -> EEConfig:
    base = dict(n_layers=80, d_model=8192, n_q_heads=64, n_kv_heads=8, head_dim=128,
                d_ffn=28672, vocab=128256, exit_draft=8, exit_inter=40,
                rope_theta=500000.0, dtype="bf16")
    base.update(kw)
    return EEConfig(**base)


def tensor_shape(cfg: EEConfig, name: str) -> Tuple[int, ...]:
    d, hq, hkv, D, F, V = (cfg.d_model, cfg.n_q_heads, cfg.n_kv_heads,
                           cfg.head_dim, cfg.d_ffn, cfg.vocab)
    r = cfg.head_rank
    return {
        "aux_g": (d,), "aux_a": (r, d), "aux_b": (d, r),
        "emb": (V, d), "head": (V, d), "gfinal": (d,),
        "g1": (d,), "g2": (d,),
        "wq": (hq * D, d), "wk": (hkv * D, d), "wv": (hkv * D, d),
        "wo": (d, hq * D), "wgate": (F, d), "wup": (F, d), "wdown": (d, F),
    }[name]


# ----------------------------------------------------------------------------
# bit-level helpers
# ----------------------------------------------------------------------------

def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit pattern (uint16), round-to-nearest-even. Finite inputs only."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.asarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _mix64(z: np.ndarray) -> np.ndarray:
    z = z ^ (z >> np.uint64(30))
    z = z * _M1
    z = z ^ (z >> np.uint64(27))
    z = z * _M2
    return z ^ (z >> np.uint64(31))


def _mix64_scalar(z: int) -> int:
    m = (1 << 64) - 1
    z &= m
    z ^= z >> 30
    z = (z * 0xBF58476D1CE4E5B9) & m
    z ^= z >> 27
    z = (z * 0x94D049BB133111EB) & m
    return z ^ (z >> 31)


def stream_key(seed: int, tensor_id: int, layer: int) -> int:
    return _mix64_scalar(_mix64_scalar(seed) ^ ((tensor_id << 32) | layer))


def _lane_sum(key: int, e: np.ndarray) -> np.ndarray:
    """Centered Irwin-Hall(12) integer for element indices e (uint64) -> int32."""
    with np.errstate(over="ignore"):
        base = np.uint64(key) + (np.uint64(3) * e + np.uint64(1)) * GOLD
        s = np.zeros(e.shape, dtype=np.uint64)
        for j in range(3):
            w = _mix64(base + np.uint64(j) * GOLD)
            s += (w & np.uint64(0xFFFF)) + ((w >> np.uint64(16)) & np.uint64(0xFFFF)) \
                + ((w >> np.uint64(32)) & np.uint64(0xFFFF)) + (w >> np.uint64(48))
    return s.astype(np.int64).astype(np.int32) - np.int32(_LANE_MEAN)


def tensor_scale(cfg: EEConfig, name: str, layer: int) -> np.float32:
    gamma = cfg.gamma[cfg.group_of_layer(layer)] if name in DAMPED_TENSORS else 1.0
    if name == "aux_b":
        gamma = cfg.gamma[min(layer, 2)]
    s1 = np.float32(cfg.sigma) * np.float32(gamma)
    return np.float32(s1) * np.float32(2.0 ** -16)


def gen_flat(cfg: EEConfig, seed: int, name: str, layer: int, e0: int, count: int) -> np.ndarray:
    """`count` consecutive elements (row-major index e0..) of a tensor, as float32."""
    key = stream_key(seed, TENSOR_IDS[name], layer if name in LAYER_TENSORS + EXIT_TENSORS else 0)
    e = np.arange(e0, e0 + count, dtype=np.uint64)
    v = _lane_sum(key, e).astype(np.float32) * tensor_scale(cfg, name, layer)
    if name in GAIN_TENSORS:
        v = np.float32(1.0) + v
    if cfg.dtype == "bf16":
        v = bf16_bits_to_f32(f32_to_bf16_bits(v))
    return v.astype(np.float32, copy=False)


_CHUNK = 1 << 20
_POOL = None
_FAST = None     # the compiled generator (synth/gen_fast.c), False once found absent


def _fast_lib():
    """The C version of the recipe above, if it has been built (the build entry point compiles it); the numpy
    version serves otherwise.  Both give the same bits."""
    global _FAST
    if _FAST is None:
        import ctypes
        import os
        path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libsynthgen.so")
        try:
            lib = ctypes.CDLL(path)
            lib.synth_fill.argtypes = [ctypes.c_uint64, ctypes.c_uint64, ctypes.c_uint64, ctypes.c_float,
                                       ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_void_p]
            lib.synth_fill.restype = None
            _FAST = lib
        except OSError:
            _FAST = False
    return _FAST


def _pool() -> ThreadPoolExecutor:
    global _POOL
    if _POOL is None:
        import os
        _POOL = ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1))
    return _POOL


def gen_tensor_rows(cfg: EEConfig, seed: int, name: str, layer: int,
                    row0: int, nrows: int, use_fast: bool = True, dtype=np.float32) -> np.ndarray:
    """Rows [row0, row0+nrows) of a 2-D tensor (or elements of a 1-D tensor), float32 (or the same values
    widened to float64)."""
    shape = tensor_shape(cfg, name)
    cols = shape[1] if len(shape) == 2 else 1
    e0, count = row0 * cols, nrows * cols
    fast = _fast_lib() if use_fast else False
    if fast:
        key = stream_key(seed, TENSOR_IDS[name], layer if name in LAYER_TENSORS + EXIT_TENSORS else 0)
        flat = np.empty(count, dtype)
        fast.synth_fill(key, e0, count, float(tensor_scale(cfg, name, layer)), int(name in GAIN_TENSORS),
                        int(cfg.dtype == "bf16"), int(np.dtype(dtype) == np.float64), flat.ctypes.data)
    elif count <= _CHUNK:
        flat = gen_flat(cfg, seed, name, layer, e0, count)
    else:
        starts = list(range(0, count, _CHUNK))
        parts = _pool().map(
            lambda s: gen_flat(cfg, seed, name, layer, e0 + s, min(_CHUNK, count - s)), starts)
        flat = np.concatenate(list(parts))
    return flat.astype(dtype, copy=False).reshape((nrows, cols) if len(shape) == 2 else (nrows,))


def gen_tensor(cfg: EEConfig, seed: int, name: str, layer: int = 0, dtype=np.float32) -> np.ndarray:
    return gen_tensor_rows(cfg, seed, name, layer, 0, tensor_shape(cfg, name)[0], dtype=dtype)


class WeightStore:
    """Lazily generated weights, looked up as store.get(name, layer).

    Values are float32 arrays in the tensor's logical [out_features,
    in_features] layout (bf16-representable when cfg.dtype == "bf16").  With
    `cache=False` nothing is retained, so an 8B- or 70B-shaped model can be
    walked layer by layer within host memory.
    """

    def __init__(self, cfg: EEConfig, seed: int, cache: bool = True):
        self.cfg, self.seed, self.cache = cfg, seed, cache
        self._mem: Dict[Tuple[str, int], np.ndarray] = {}

    def get(self, name: str, layer: int = 0) -> np.ndarray:
        k = (name, layer if name in LAYER_TENSORS + EXIT_TENSORS else 0)
        if k in self._mem:
            return self._mem[k]
        t = gen_tensor(self.cfg, self.seed, name, k[1])
        if self.cache:
            self._mem[k] = t
        return t

    def override(self, name: str, layer: int, value: np.ndarray) -> None:
        """Replace a tensor (tests that need hand-made weights)."""
        assert tuple(value.shape) == tensor_shape(self.cfg, name)
        self._mem[(name, layer if name in LAYER_TENSORS + EXIT_TENSORS else 0)] = np.asarray(value, np.float32)
