"""ctypes binding of libhispec.so: argument marshalling only, every step runs in the library.

Module-level functions carry the names of the C entry points (include/hispec.h).  `Model` and
`Session` own the caller-side device arenas (torch uint8 tensors) the C ABI asks for.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence, Tuple

import numpy as np

__all__ = [
    "lib", "lib_path", "EEError", "ee_config", "make_config", "Model", "Session",
    "ee_model_bytes", "ee_model_load", "ee_model_set_tensor", "ee_model_get_tensor_rows", "ee_model_free",
    "ee_session_bytes", "ee_session_create", "ee_session_free", "ee_prefill", "ee_prefill_seq", "ee_seq_release", "ee_free_pages", "ee_decode_ar", "ee_draft", "ee_draft_inject",
    "ee_verify_intermediate", "ee_verify_intermediate_static", "ee_verify_full", "ee_verify_level", "ee_n_levels", "kv_rollback", "ee_sampling_bytes", "ee_sampling_attach",
    "ee_draft_sample", "ee_verify_intermediate_rs", "ee_verify_full_rs", "ee_verify_level_rs", "ee_debug_read_dist", "ee_get_lengths", "ee_get_counts", "ee_get_tokens",
    "ee_debug_enable_logits", "ee_debug_last_logits", "ee_debug_last_hidden", "ee_debug_read_kv", "ee_debug_write_kv",
    "ee_debug_poison_dead_kv", "ee_debug_time_kernels", "ee_debug_kernel_times", "ee_debug_gemm_row_blocks", "ee_debug_attention_split_pages", "ee_debug_stream_copy", "ee_debug_read_floor", "ee_last_error",
    "EE_F32", "EE_BF16", "TENSOR_IDS", "EXPORTED_SYMBOLS",
]

EE_F32, EE_BF16 = 0, 1
TENSOR_IDS = {"emb": 0, "head": 1, "gfinal": 2, "g1": 3, "wq": 4, "wk": 5, "wv": 6, "wo": 7,
              "g2": 8, "wgate": 9, "wup": 10, "wdown": 11,
              "aux_g": 12, "aux_a": 13, "aux_b": 14}   # auxiliary exit heads: `layer` = exit index (0 = L_d, 1 = L_i)

EXPORTED_SYMBOLS = [
    "ee_model_bytes", "ee_model_load", "ee_model_set_tensor", "ee_model_get_tensor_rows", "ee_model_free",
    "ee_session_bytes", "ee_session_create", "ee_session_free", "ee_prefill", "ee_prefill_seq", "ee_seq_release", "ee_free_pages", "ee_decode_ar", "ee_draft", "ee_draft_inject",
    "ee_verify_intermediate", "ee_verify_intermediate_static", "ee_verify_full", "ee_verify_level", "ee_n_levels", "kv_rollback", "ee_sampling_bytes", "ee_sampling_attach",
    "ee_draft_sample", "ee_verify_intermediate_rs", "ee_verify_full_rs", "ee_verify_level_rs", "ee_debug_read_dist", "ee_get_lengths", "ee_get_counts", "ee_get_tokens",
    "ee_debug_enable_logits", "ee_debug_last_logits", "ee_debug_last_hidden", "ee_debug_read_kv", "ee_debug_write_kv",
    "ee_debug_poison_dead_kv", "ee_debug_time_kernels", "ee_debug_kernel_times", "ee_debug_gemm_row_blocks", "ee_debug_attention_split_pages", "ee_debug_stream_copy", "ee_debug_read_floor", "ee_last_error",
]


class ee_config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_q_heads", "n_kv_heads", "head_dim", "d_ffn", "vocab",
                                         "exit_draft", "exit_inter")] + \
               [("rope_theta", C.c_float), ("rms_eps", C.c_float), ("dtype", C.c_int32),
                ("bonus_inter", C.c_int32), ("bonus_full", C.c_int32), ("sigma", C.c_float), ("gamma", C.c_float * 3),
                ("head_rank", C.c_int32), ("n_extra_exits", C.c_int32), ("extra_exits", C.c_int32 * 4)]


class EEError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"libhispec error {code}: {msg}")
        self.code = code


def lib_path() -> str:
    return os.path.join(os.path.dirname(os.path.abspath(__file__)), "libhispec.so")


def _load():
    path = lib_path()
    if not os.path.exists(path):
        raise ImportError(f"{path} is missing: build it with `python paper_2510_01336_amd/build.py` "
                          "(there is no fallback path)")
    # torch ships its own HIP runtime; it must be in the process before libhispec.so is mapped so
    # that both resolve the one libamdhip64.so.7 (two runtimes in a process do not share a device)
    import torch  # noqa: F401
    L = C.CDLL(path)
    vp, i32p, f32p = C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_float)
    sig = {
        "ee_model_bytes": (C.c_size_t, [C.POINTER(ee_config)]),
        "ee_model_load": (C.c_int, [C.POINTER(ee_config), vp, C.c_size_t, C.c_uint64, vp, C.POINTER(vp)]),
        "ee_model_set_tensor": (C.c_int, [vp, C.c_int, C.c_int, f32p]),
        "ee_model_get_tensor_rows": (C.c_int, [vp, C.c_int, C.c_int, C.c_int, C.c_int, f32p]),
        "ee_model_free": (None, [vp]),
        "ee_session_bytes": (C.c_size_t, [vp, C.c_int, C.c_int, C.c_int, C.c_int]),
        "ee_session_create": (C.c_int, [vp, C.c_int, C.c_int, C.c_int, C.c_int, vp, C.c_size_t, vp, C.POINTER(vp)]),
        "ee_session_free": (None, [vp]),
        "ee_prefill": (C.c_int, [vp, i32p, i32p, i32p]),
        "ee_decode_ar": (C.c_int, [vp, C.c_int, i32p]),
        "ee_prefill_seq": (C.c_int, [vp, C.c_int, i32p, C.c_int, i32p]),
        "ee_seq_release": (C.c_int, [vp, C.c_int]),
        "ee_free_pages": (C.c_int, [vp]),
        "ee_draft": (C.c_int, [vp, C.c_int, i32p]),
        "ee_draft_inject": (C.c_int, [vp, C.c_int, i32p]),
        "ee_verify_intermediate": (C.c_int, [vp, i32p, i32p]),
        "ee_verify_intermediate_static": (C.c_int, [vp, i32p, i32p]),
        "ee_verify_full": (C.c_int, [vp, C.POINTER(C.c_uint8), i32p, i32p, i32p, i32p]),
        "ee_verify_level": (C.c_int, [vp, C.c_int, C.POINTER(C.c_uint8), i32p, i32p, i32p, i32p]),
        "ee_n_levels": (C.c_int, [vp]),
        "kv_rollback": (C.c_int, [vp, C.c_int, C.c_int, C.c_int]),
        "ee_sampling_bytes": (C.c_size_t, [vp]),
        "ee_sampling_attach": (C.c_int, [vp, vp, C.c_size_t]),
        "ee_draft_sample": (C.c_int, [vp, C.c_int, f32p, i32p]),
        "ee_debug_read_dist": (C.c_int, [vp, C.c_int, C.c_int, C.c_int, C.c_int, f32p]),
        "ee_verify_intermediate_rs": (C.c_int, [vp, f32p, C.c_int, f32p, i32p, i32p]),
        "ee_verify_full_rs": (C.c_int, [vp, C.POINTER(C.c_uint8), f32p, C.c_int, f32p, i32p, i32p, i32p, i32p]),
        "ee_verify_level_rs": (C.c_int, [vp, C.c_int, C.POINTER(C.c_uint8), f32p, C.c_int, f32p, i32p, i32p, i32p, i32p]),
        "ee_get_lengths": (C.c_int, [vp, i32p]),
        "ee_get_counts": (C.c_int, [vp, i32p, i32p]),
        "ee_get_tokens": (C.c_int, [vp, C.c_int, i32p, C.c_int, i32p]),
        "ee_debug_enable_logits": (C.c_int, [vp, C.c_int]),
        "ee_debug_last_logits": (C.c_int, [vp, f32p, C.c_int, i32p]),
        "ee_debug_last_hidden": (C.c_int, [vp, f32p, C.c_int, i32p]),
        "ee_debug_read_kv": (C.c_int, [vp, C.c_int, C.c_int, C.c_int, C.c_int, f32p, f32p]),
        "ee_debug_write_kv": (C.c_int, [vp, C.c_int, C.c_int, C.c_int, C.c_int, f32p, f32p]),
        "ee_debug_poison_dead_kv": (C.c_int, [vp, C.c_int]),
        "ee_debug_time_kernels": (C.c_int, [vp, C.c_int]),
        "ee_debug_gemm_row_blocks": (C.c_int, [C.c_int]),
        "ee_debug_attention_split_pages": (C.c_int, [C.c_int]),
        "ee_debug_kernel_times": (C.c_int, [vp, i32p, C.POINTER(C.c_char_p), f32p, i32p]),
        "ee_debug_stream_copy": (C.c_int, [vp, vp, C.c_size_t, vp]),
        "ee_debug_read_floor": (C.c_int, [vp, C.POINTER(C.c_size_t), C.c_int, C.c_int, C.POINTER(C.c_float), vp]),
        "ee_last_error": (C.c_char_p, []),
    }
    for name, (res, args) in sig.items():
        fn = getattr(L, name)
        fn.restype, fn.argtypes = res, args
    return L


lib = _load()


def ee_last_error() -> str:
    return lib.ee_last_error().decode()


def _chk(rc: int) -> None:
    if rc != 0:
        raise EEError(rc, ee_last_error())


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _p_i32(a: np.ndarray):
    return a.ctypes.data_as(C.POINTER(C.c_int32))


def _p_f32(a: np.ndarray):
    return a.ctypes.data_as(C.POINTER(C.c_float))


def make_config(cfg, bonus_inter: int = 1, bonus_full: int = 1) -> ee_config:
    """Build the C config from any object carrying the architecture fields by name."""
    c = ee_config()
    for n in ("n_layers", "d_model", "n_q_heads", "n_kv_heads", "head_dim", "d_ffn", "vocab", "exit_draft", "exit_inter"):
        setattr(c, n, int(getattr(cfg, n)))
    c.rope_theta, c.rms_eps = float(cfg.rope_theta), float(cfg.rms_eps)
    c.dtype = EE_BF16 if getattr(cfg, "dtype", "f32") == "bf16" else EE_F32
    c.bonus_inter, c.bonus_full = int(bonus_inter), int(bonus_full)
    c.sigma = float(getattr(cfg, "sigma", 0.02))
    for i, g in enumerate(getattr(cfg, "gamma", (1.0, 1.0, 1.0))):
        c.gamma[i] = float(g)
    c.head_rank = int(getattr(cfg, "head_rank", 0))
    extra = tuple(getattr(cfg, "exit_extra", ()))
    c.n_extra_exits = len(extra)
    for i, e in enumerate(extra):
        c.extra_exits[i] = int(e)
    return c


def _stream_ptr(stream) -> int:
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return int(stream.cuda_stream)


def _arena(nbytes: int):
    import torch
    t = torch.empty(int(nbytes) + 256, dtype=torch.uint8, device="cuda")
    off = (-t.data_ptr()) % 256
    return t, t.data_ptr() + off


# ---- entry points (same names as the C ABI) -----------------------------------------------------

def ee_model_bytes(cfg: ee_config) -> int:
    n = lib.ee_model_bytes(C.byref(cfg))
    if n == 0:
        raise EEError(-1, ee_last_error())
    return n


def ee_model_load(cfg: ee_config, dev_ptr: int, nbytes: int, seed: int, stream_ptr: int) -> int:
    out = C.c_void_p()
    _chk(lib.ee_model_load(C.byref(cfg), dev_ptr, nbytes, seed, stream_ptr, C.byref(out)))
    return out.value


def ee_model_set_tensor(model: int, tensor_id: int, layer: int, values: np.ndarray) -> None:
    v = np.ascontiguousarray(values, dtype=np.float32)
    _chk(lib.ee_model_set_tensor(model, tensor_id, layer, _p_f32(v)))


def ee_model_get_tensor_rows(model: int, tensor_id: int, layer: int, row0: int, nrows: int, cols: int) -> np.ndarray:
    out = np.empty((nrows, cols), np.float32)
    _chk(lib.ee_model_get_tensor_rows(model, tensor_id, layer, row0, nrows, _p_f32(out)))
    return out


def ee_model_free(model: int) -> None:
    lib.ee_model_free(model)


def ee_session_bytes(model: int, batch: int, max_ctx: int, max_rows: int, total_pages: int = 0) -> int:
    n = lib.ee_session_bytes(model, batch, max_ctx, max_rows, total_pages)
    if n == 0:
        raise EEError(-1, ee_last_error())
    return n


def ee_session_create(model: int, batch: int, max_ctx: int, max_rows: int, total_pages: int, dev_ptr: int,
                      nbytes: int, stream_ptr: int) -> int:
    out = C.c_void_p()
    _chk(lib.ee_session_create(model, batch, max_ctx, max_rows, total_pages, dev_ptr, nbytes, stream_ptr, C.byref(out)))
    return out.value


def ee_session_free(session: int) -> None:
    lib.ee_session_free(session)


def ee_prefill(session: int, tokens: np.ndarray, lens: np.ndarray) -> np.ndarray:
    t, l = _i32(tokens), _i32(lens)
    first = np.empty(len(l), np.int32)
    _chk(lib.ee_prefill(session, _p_i32(t), _p_i32(l), _p_i32(first)))
    return first


def ee_seq_release(session: int, seq: int) -> None:
    _chk(lib.ee_seq_release(session, seq))


def ee_free_pages(session: int) -> int:
    return int(lib.ee_free_pages(session))


def ee_prefill_seq(session: int, seq: int, tokens: np.ndarray) -> int:
    t = _i32(tokens)
    out = np.empty(1, np.int32)
    _chk(lib.ee_prefill_seq(session, seq, _p_i32(t), len(t), _p_i32(out)))
    return int(out[0])


def ee_decode_ar(session: int, batch: int, n: int) -> np.ndarray:
    out = np.empty((batch, n), np.int32)
    _chk(lib.ee_decode_ar(session, n, _p_i32(out)))
    return out


def ee_draft(session: int, batch: int, k: int) -> np.ndarray:
    out = np.empty((batch, k), np.int32)
    _chk(lib.ee_draft(session, k, _p_i32(out)))
    return out


def ee_draft_inject(session: int, draft: np.ndarray) -> None:
    d = _i32(draft)
    assert d.ndim == 2
    _chk(lib.ee_draft_inject(session, d.shape[1], _p_i32(d)))


def ee_verify_intermediate(session: int, batch: int) -> Tuple[np.ndarray, np.ndarray]:
    a, n = np.empty(batch, np.int32), np.empty(batch, np.int32)
    _chk(lib.ee_verify_intermediate(session, _p_i32(a), _p_i32(n)))
    return a, n


def ee_verify_intermediate_static(session: int, batch: int) -> Tuple[np.ndarray, np.ndarray]:
    a, n = np.empty(batch, np.int32), np.empty(batch, np.int32)
    _chk(lib.ee_verify_intermediate_static(session, _p_i32(a), _p_i32(n)))
    return a, n


def ee_verify_full(session: int, batch: int, max_rows: int, active: Optional[Sequence[int]] = None):
    a, n, nc = np.empty(batch, np.int32), np.empty(batch, np.int32), np.empty(batch, np.int32)
    com = np.zeros((batch, max_rows + 1), np.int32)
    act = None
    if active is not None:
        act_arr = np.ascontiguousarray(active, dtype=np.uint8)
        act = act_arr.ctypes.data_as(C.POINTER(C.c_uint8))
    _chk(lib.ee_verify_full(session, act, _p_i32(a), _p_i32(n), _p_i32(com), _p_i32(nc)))
    return a, n, [com[b, :nc[b]].tolist() for b in range(batch)]


def ee_verify_level(session: int, level: int, batch: int, max_rows: int, active: Optional[Sequence[int]] = None):
    a, n, nc = np.empty(batch, np.int32), np.empty(batch, np.int32), np.empty(batch, np.int32)
    com = np.zeros((batch, max_rows + 1), np.int32)
    act = None
    if active is not None:
        act_arr = np.ascontiguousarray(active, dtype=np.uint8)
        act = act_arr.ctypes.data_as(C.POINTER(C.c_uint8))
    _chk(lib.ee_verify_level(session, level, act, _p_i32(a), _p_i32(n), _p_i32(com), _p_i32(nc)))
    return a, n, [com[b, :nc[b]].tolist() for b in range(batch)]


def ee_n_levels(session: int) -> int:
    return int(lib.ee_n_levels(session))


def _f32c(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def ee_sampling_bytes(session: int) -> int:
    return int(lib.ee_sampling_bytes(session))


def ee_sampling_attach(session: int, dev_ptr: int, nbytes: int) -> None:
    _chk(lib.ee_sampling_attach(session, dev_ptr, nbytes))


def ee_debug_read_dist(session: int, which: int, seq: int, row0: int, n: int, vocab: int) -> np.ndarray:
    out = np.empty((n, vocab), np.float32)
    _chk(lib.ee_debug_read_dist(session, which, seq, row0, n, _p_f32(out)))
    return out


def ee_draft_sample(session: int, batch: int, k: int, u: np.ndarray) -> np.ndarray:
    u = _f32c(u).reshape(batch, k)
    out = np.empty((batch, k), np.int32)
    _chk(lib.ee_draft_sample(session, k, _p_f32(u), _p_i32(out)))
    return out


def ee_verify_intermediate_rs(session: int, batch: int, u_acc: np.ndarray, u_res: np.ndarray):
    u_acc, u_res = _f32c(u_acc).reshape(batch, -1), _f32c(u_res).reshape(batch)
    a, n = np.empty(batch, np.int32), np.empty(batch, np.int32)
    _chk(lib.ee_verify_intermediate_rs(session, _p_f32(u_acc), u_acc.shape[1], _p_f32(u_res), _p_i32(a), _p_i32(n)))
    return a, n


def ee_verify_full_rs(session: int, batch: int, max_rows: int, u_acc: np.ndarray, u_res: np.ndarray,
                      active: Optional[Sequence[int]] = None):
    u_acc, u_res = _f32c(u_acc).reshape(batch, -1), _f32c(u_res).reshape(batch)
    a, n, nc = np.empty(batch, np.int32), np.empty(batch, np.int32), np.empty(batch, np.int32)
    com = np.zeros((batch, max_rows + 1), np.int32)
    act = None
    if active is not None:
        act_arr = np.ascontiguousarray(active, dtype=np.uint8)
        act = act_arr.ctypes.data_as(C.POINTER(C.c_uint8))
    _chk(lib.ee_verify_full_rs(session, act, _p_f32(u_acc), u_acc.shape[1], _p_f32(u_res), _p_i32(a), _p_i32(n), _p_i32(com),
                               _p_i32(nc)))
    return a, n, [com[b, :nc[b]].tolist() for b in range(batch)]


def ee_verify_level_rs(session: int, level: int, batch: int, max_rows: int, u_acc: np.ndarray, u_res: np.ndarray,
                       active: Optional[Sequence[int]] = None):
    u_acc, u_res = _f32c(u_acc).reshape(batch, -1), _f32c(u_res).reshape(batch)
    a, n, nc = np.empty(batch, np.int32), np.empty(batch, np.int32), np.empty(batch, np.int32)
    com = np.zeros((batch, max_rows + 1), np.int32)
    act = None
    if active is not None:
        act_arr = np.ascontiguousarray(active, dtype=np.uint8)
        act = act_arr.ctypes.data_as(C.POINTER(C.c_uint8))
    _chk(lib.ee_verify_level_rs(session, level, act, _p_f32(u_acc), u_acc.shape[1], _p_f32(u_res), _p_i32(a), _p_i32(n),
                                _p_i32(com), _p_i32(nc)))
    return a, n, [com[b, :nc[b]].tolist() for b in range(batch)]


def kv_rollback(session: int, seq: int, group_mask: int, new_len: int) -> None:
    _chk(lib.kv_rollback(session, seq, group_mask, new_len))


def ee_get_lengths(session: int, batch: int) -> np.ndarray:
    out = np.empty((batch, ee_n_levels(session) + 1), np.int32)
    _chk(lib.ee_get_lengths(session, _p_i32(out)))
    return out


def ee_get_counts(session: int, batch: int) -> Tuple[np.ndarray, np.ndarray]:
    a, b = np.empty(batch, np.int32), np.empty(batch, np.int32)
    _chk(lib.ee_get_counts(session, _p_i32(a), _p_i32(b)))
    return a, b


def ee_get_tokens(session: int, seq: int, cap: int = 1 << 20) -> np.ndarray:
    out, n = np.empty(cap, np.int32), C.c_int32()
    _chk(lib.ee_get_tokens(session, seq, _p_i32(out), cap, C.byref(n)))
    return out[:n.value].copy()


def ee_debug_enable_logits(session: int, on: bool) -> None:
    _chk(lib.ee_debug_enable_logits(session, int(on)))


def ee_debug_last_logits(session: int, max_rows: int, vocab: int) -> np.ndarray:
    out, n = np.empty((max_rows, vocab), np.float32), C.c_int32()
    _chk(lib.ee_debug_last_logits(session, _p_f32(out), max_rows, C.byref(n)))
    return out[:n.value]


def ee_debug_last_hidden(session: int, max_rows: int, d: int) -> np.ndarray:
    out, n = np.empty((max_rows, d), np.float32), C.c_int32()
    _chk(lib.ee_debug_last_hidden(session, _p_f32(out), max_rows, C.byref(n)))
    return out[:n.value]


def ee_debug_read_kv(session: int, seq: int, layer: int, pos0: int, n: int, n_kv: int, head_dim: int):
    k, v = np.empty((n, n_kv, head_dim), np.float32), np.empty((n, n_kv, head_dim), np.float32)
    _chk(lib.ee_debug_read_kv(session, seq, layer, pos0, n, _p_f32(k), _p_f32(v)))
    return k, v


def ee_debug_write_kv(session: int, seq: int, layer: int, pos0: int, k: np.ndarray, v: np.ndarray) -> None:
    k, v = np.ascontiguousarray(k, np.float32), np.ascontiguousarray(v, np.float32)
    assert k.shape == v.shape and k.ndim == 3
    _chk(lib.ee_debug_write_kv(session, seq, layer, pos0, k.shape[0], _p_f32(k), _p_f32(v)))


def ee_debug_poison_dead_kv(session: int, seq: int) -> None:
    _chk(lib.ee_debug_poison_dead_kv(session, seq))


def ee_debug_gemm_row_blocks(row_tiles: int) -> None:
    _chk(lib.ee_debug_gemm_row_blocks(int(row_tiles)))


def ee_debug_attention_split_pages(pages: int) -> None:
    _chk(lib.ee_debug_attention_split_pages(int(pages)))


def ee_debug_time_kernels(session: int, on: bool) -> None:
    _chk(lib.ee_debug_time_kernels(session, int(on)))


def ee_debug_kernel_times(session: int) -> dict:
    n = C.c_int32()
    names = (C.c_char_p * 16)()
    ms, cnt = np.zeros(16, np.float32), np.zeros(16, np.int32)
    _chk(lib.ee_debug_kernel_times(session, C.byref(n), names, _p_f32(ms), _p_i32(cnt)))
    return {names[i].decode(): (float(ms[i]), int(cnt[i])) for i in range(n.value)}


def ee_debug_stream_copy(dst_ptr: int, src_ptr: int, nbytes: int, stream_ptr: int) -> None:
    _chk(lib.ee_debug_stream_copy(dst_ptr, src_ptr, nbytes, stream_ptr))


def ee_debug_read_floor(buf_ptr: int, sizes, reps: int, stream_ptr: int) -> list:
    """Mean microseconds of a plain read of each region (sizes in bytes, laid out one after another from buf_ptr)."""
    n = len(sizes)
    arr = (C.c_size_t * n)(*[int(x) for x in sizes])
    out = (C.c_float * n)()
    _chk(lib.ee_debug_read_floor(buf_ptr, arr, n, int(reps), out, stream_ptr))
    return [float(x) for x in out]


# ---- arena owners ---------------------------------------------------------------------------------

class Model:
    """Owns the device arena of one EE model and its library handle."""

    def __init__(self, cfg, seed: int, bonus_inter: int = 1, bonus_full: int = 1, stream=None):
        self.cfg = cfg
        self.c = make_config(cfg, bonus_inter, bonus_full)
        self.nbytes = ee_model_bytes(self.c)
        self._buf, ptr = _arena(self.nbytes)
        self.stream = _stream_ptr(stream)
        self.handle = ee_model_load(self.c, ptr, self.nbytes, seed, self.stream)

    def tensor_rows(self, name: str, layer: int, row0: int, nrows: int, cols: int) -> np.ndarray:
        return ee_model_get_tensor_rows(self.handle, TENSOR_IDS[name], layer, row0, nrows, cols)

    def set_tensor(self, name: str, layer: int, values: np.ndarray) -> None:
        ee_model_set_tensor(self.handle, TENSOR_IDS[name], layer, values)

    def close(self) -> None:
        if self.handle:
            ee_model_free(self.handle)
            self.handle, self._buf = None, None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Session:
    """Owns the device arena of one session; methods forward to the C entry points."""

    def __init__(self, model: Model, batch: int, max_ctx: int, max_rows: int, total_pages: int = 0):
        self.model, self.batch, self.max_ctx, self.max_rows = model, batch, max_ctx, max_rows
        self.nbytes = ee_session_bytes(model.handle, batch, max_ctx, max_rows, total_pages)
        self._buf, ptr = _arena(self.nbytes)
        self.handle = ee_session_create(model.handle, batch, max_ctx, max_rows, total_pages, ptr, self.nbytes, model.stream)

    def prefill(self, prompts: Sequence[np.ndarray]) -> np.ndarray:
        lens = np.array([len(p) for p in prompts], np.int32)
        return ee_prefill(self.handle, np.concatenate([_i32(p) for p in prompts]), lens)

    def prefill_seq(self, seq: int, prompt: np.ndarray) -> int:
        return ee_prefill_seq(self.handle, seq, prompt)

    def release(self, seq: int) -> None:
        ee_seq_release(self.handle, seq)

    def free_pages(self) -> int:
        return ee_free_pages(self.handle)

    def decode_ar(self, n: int) -> np.ndarray:
        return ee_decode_ar(self.handle, self.batch, n)

    def draft(self, k: int) -> np.ndarray:
        return ee_draft(self.handle, self.batch, k)

    def draft_inject(self, draft: np.ndarray) -> None:
        ee_draft_inject(self.handle, np.asarray(draft).reshape(self.batch, -1))

    def verify_intermediate(self):
        return ee_verify_intermediate(self.handle, self.batch)

    def verify_intermediate_static(self):
        return ee_verify_intermediate_static(self.handle, self.batch)

    def verify_full(self, active=None):
        return ee_verify_full(self.handle, self.batch, self.max_rows, active)

    def verify_level(self, level: int, active=None):
        return ee_verify_level(self.handle, level, self.batch, self.max_rows, active)

    def n_levels(self) -> int:
        return ee_n_levels(self.handle)

    def enable_sampling(self) -> None:
        """Allocate and attach the buffers of the rejection-sampling calls."""
        n = ee_sampling_bytes(self.handle)
        self._sampling_buf, ptr = _arena(n)
        ee_sampling_attach(self.handle, ptr, n)

    def read_dist(self, which: int, seq: int, row0: int, n: int) -> np.ndarray:
        return ee_debug_read_dist(self.handle, which, seq, row0, n, self.model.cfg.vocab)

    def draft_sample(self, k: int, u: np.ndarray) -> np.ndarray:
        return ee_draft_sample(self.handle, self.batch, k, u)

    def verify_intermediate_rs(self, u_acc: np.ndarray, u_res: np.ndarray):
        return ee_verify_intermediate_rs(self.handle, self.batch, u_acc, u_res)

    def verify_full_rs(self, u_acc: np.ndarray, u_res: np.ndarray, active=None):
        return ee_verify_full_rs(self.handle, self.batch, self.max_rows, u_acc, u_res, active)

    def verify_level_rs(self, level: int, u_acc: np.ndarray, u_res: np.ndarray, active=None):
        return ee_verify_level_rs(self.handle, level, self.batch, self.max_rows, u_acc, u_res, active)

    def rollback(self, seq: int, group_mask: int, new_len: int) -> None:
        kv_rollback(self.handle, seq, group_mask, new_len)

    def lengths(self) -> np.ndarray:
        return ee_get_lengths(self.handle, self.batch)

    def counts(self):
        return ee_get_counts(self.handle, self.batch)

    def tokens(self, seq: int) -> np.ndarray:
        return ee_get_tokens(self.handle, seq)

    def enable_logits(self, on: bool = True) -> None:
        ee_debug_enable_logits(self.handle, on)

    def last_logits(self, max_rows: Optional[int] = None) -> np.ndarray:
        return ee_debug_last_logits(self.handle, max_rows or max(512, self.batch * self.max_rows), self.model.cfg.vocab)

    def last_hidden(self, max_rows: Optional[int] = None) -> np.ndarray:
        return ee_debug_last_hidden(self.handle, max_rows or max(512, self.batch * self.max_rows), self.model.cfg.d_model)

    def read_kv(self, seq: int, layer: int, pos0: int, n: int):
        return ee_debug_read_kv(self.handle, seq, layer, pos0, n, self.model.cfg.n_kv_heads, self.model.cfg.head_dim)

    def write_kv(self, seq: int, layer: int, pos0: int, k: np.ndarray, v: np.ndarray) -> None:
        ee_debug_write_kv(self.handle, seq, layer, pos0, k, v)

    def poison_dead_kv(self, seq: int) -> None:
        ee_debug_poison_dead_kv(self.handle, seq)

    def time_kernels(self, on: bool = True) -> None:
        ee_debug_time_kernels(self.handle, on)

    def kernel_times(self) -> dict:
        return ee_debug_kernel_times(self.handle)

    def close(self) -> None:
        if self.handle:
            ee_session_free(self.handle)
            self.handle, self._buf = None, None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
