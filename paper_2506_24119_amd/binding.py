"""ctypes binding of libspiral.so: same names as include/spiral.h, argument
marshalling only.  PyTorch is used for device memory and streams; every step of
the decode path runs inside the library's HIP kernels.  There is no CPU or
eager fallback: if the shared library is missing, loading raises."""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional, Sequence

import numpy as np

from . import inputs as _inputs

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("SPIRAL_LIB", os.path.join(_HERE, "libspiral.so"))

SPIRAL_OK = 0
SPIRAL_ERR_INVALID_ARG = -1
SPIRAL_ERR_SHAPE = -2
SPIRAL_ERR_OOM_KV = -3
SPIRAL_ERR_NOT_LOADED = -4
SPIRAL_ERR_HIP = -5
SPIRAL_MAX_BATCH = 1024
SPIRAL_LAYER_SLOTS = 14

EXPORTS = [
    "spiral_last_error", "spiral_version", "spiral_model_load", "spiral_model_free", "spiral_model_repack_bytes", "spiral_model_repack",
    "spiral_workspace_bytes", "spiral_kv_pool_bytes", "spiral_kv_pool_create", "spiral_kv_pool_free",
    "spiral_seq_reset", "spiral_seq_truncate", "spiral_profile_begin", "spiral_profile_end", "spiral_seq_len", "spiral_kv_free_pages", "spiral_prefill", "spiral_decode_step",
    "spiral_sample", "spiral_sample_truncated", "spiral_score", "spiral_policy_objective", "spiral_rae_create", "spiral_rae_update", "spiral_rae_get", "spiral_rae_set",
    "spiral_rae_free", "spiral_model_tune", "spiral_kv_pool_status_offset", "spiral_decode_sample_step",
    "spiral_decode_step_static", "spiral_static_workspace_bytes", "spiral_probe_stream_read",
    "spiral_sample_truncated_ws", "spiral_sample_truncated_workspace_bytes",
]


class spiral_model_config(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_q_heads", C.c_int32),
                ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("ffn_dim", C.c_int32),
                ("vocab", C.c_int32), ("rope_theta", C.c_float), ("rms_eps", C.c_float),
                ("qk_norm", C.c_int32), ("qkv_bias", C.c_int32), ("tie_lm_head", C.c_int32),
                ("weight_dtype", C.c_int32), ("kv_block_tokens", C.c_int32)]


class SpiralError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"spiral error {code}: {text}")
        self.code = code


_lib = None


def load_library(path: Optional[str] = None):
    """Loads libspiral.so (once) and declares the prototypes.  Raises OSError if
    the library has not been built (python -m paper_2506_24119_amd.build)."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    p = path or LIB_PATH
    # PyTorch ships its own HIP runtime under the same soname as the system one; importing torch
    # first makes the dynamic linker resolve libspiral's dependency to that copy, so that the
    # library and torch share one runtime (two runtimes in one process cannot both see the GPU).
    import torch  # noqa: F401
    if not os.path.exists(p):
        raise OSError(f"{p} not found: build it with `python -m paper_2506_24119_amd.build`; "
                      "there is no fallback path")
    lib = C.CDLL(p)
    vp, i32p, f32p, f64p = C.c_void_p, C.POINTER(C.c_int32), C.c_void_p, C.POINTER(C.c_double)
    lib.spiral_last_error.restype = C.c_char_p
    lib.spiral_last_error.argtypes = []
    lib.spiral_version.restype = C.c_char_p
    lib.spiral_version.argtypes = []
    lib.spiral_model_load.restype = C.c_int
    lib.spiral_model_load.argtypes = [C.POINTER(spiral_model_config), C.POINTER(C.c_void_p), C.c_int, C.POINTER(vp)]
    lib.spiral_model_repack_bytes.restype = C.c_size_t
    lib.spiral_model_repack_bytes.argtypes = [vp]
    lib.spiral_model_repack.restype = C.c_int
    lib.spiral_model_repack.argtypes = [vp, vp, C.c_size_t, vp]
    lib.spiral_model_free.restype = None
    lib.spiral_model_free.argtypes = [vp]
    lib.spiral_workspace_bytes.restype = C.c_size_t
    lib.spiral_workspace_bytes.argtypes = [vp, C.c_int, C.c_int]
    lib.spiral_kv_pool_bytes.restype = C.c_size_t
    lib.spiral_kv_pool_bytes.argtypes = [vp, C.c_int, C.c_int, C.c_int]
    lib.spiral_kv_pool_create.restype = C.c_int
    lib.spiral_kv_pool_create.argtypes = [vp, vp, C.c_size_t, C.c_int, C.c_int, C.c_int, i32p, vp, C.POINTER(vp)]
    lib.spiral_kv_pool_free.restype = None
    lib.spiral_kv_pool_free.argtypes = [vp]
    lib.spiral_seq_reset.restype = C.c_int
    lib.spiral_seq_reset.argtypes = [vp, i32p, C.c_int, vp]
    lib.spiral_seq_truncate.restype = C.c_int
    lib.spiral_seq_truncate.argtypes = [vp, i32p, i32p, C.c_int, vp]
    lib.spiral_profile_begin.restype = C.c_int
    lib.spiral_profile_begin.argtypes = [vp, C.c_int, C.c_int]
    lib.spiral_profile_end.restype = C.c_int
    lib.spiral_profile_end.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(C.c_int)]
    lib.spiral_seq_len.restype = C.c_int
    lib.spiral_seq_len.argtypes = [vp, C.c_int]
    lib.spiral_kv_free_pages.restype = C.c_int
    lib.spiral_kv_free_pages.argtypes = [vp]
    lib.spiral_prefill.restype = C.c_int
    lib.spiral_prefill.argtypes = [vp, vp, i32p, i32p, C.c_int, vp, vp, C.c_size_t, f32p, vp]
    lib.spiral_decode_step.restype = C.c_int
    lib.spiral_decode_step.argtypes = [vp, vp, i32p, C.c_int, vp, vp, C.c_size_t, f32p, vp]
    lib.spiral_decode_sample_step.restype = C.c_int
    lib.spiral_decode_sample_step.argtypes = [vp, vp, i32p, C.c_int, vp, vp, C.c_size_t, C.c_float, C.c_uint64, i32p, vp, vp]
    lib.spiral_decode_step_static.restype = C.c_int
    lib.spiral_decode_step_static.argtypes = [vp, vp, i32p, C.c_int, vp, f32p, vp]
    lib.spiral_static_workspace_bytes.restype = C.c_size_t
    lib.spiral_static_workspace_bytes.argtypes = []
    lib.spiral_probe_stream_read.restype = C.c_int
    lib.spiral_probe_stream_read.argtypes = [vp, C.c_size_t, C.c_int, C.POINTER(C.c_double), vp]
    lib.spiral_model_tune.restype = C.c_int
    lib.spiral_model_tune.argtypes = [vp, C.c_char_p]
    lib.spiral_kv_pool_status_offset.restype = C.c_longlong
    lib.spiral_kv_pool_status_offset.argtypes = [vp]
    lib.spiral_sample.restype = C.c_int
    lib.spiral_sample.argtypes = [f32p, C.c_int, C.c_int, C.c_float, C.c_uint64, i32p, i32p, vp, vp, vp]
    lib.spiral_score.restype = C.c_int
    lib.spiral_score.argtypes = [vp, vp, i32p, i32p, C.c_int, vp, vp, vp, C.c_size_t, vp, vp]
    lib.spiral_policy_objective.restype = C.c_int
    lib.spiral_policy_objective.argtypes = [vp, vp, vp, vp, C.c_longlong, C.c_float, vp, vp]
    lib.spiral_sample_truncated.restype = C.c_int
    lib.spiral_sample_truncated.argtypes = [f32p, C.c_int, C.c_int, C.c_float, C.c_int, C.c_float, C.c_uint64, i32p, i32p, vp, vp,
                                            vp, vp]
    lib.spiral_sample_truncated_workspace_bytes.restype = C.c_size_t
    lib.spiral_sample_truncated_workspace_bytes.argtypes = [C.c_int, C.c_int]
    lib.spiral_sample_truncated_ws.restype = C.c_int
    lib.spiral_sample_truncated_ws.argtypes = [f32p, C.c_int, C.c_int, C.c_float, C.c_int, C.c_float, C.c_uint64, i32p, i32p, vp, vp,
                                               vp, vp, C.c_size_t, vp]
    lib.spiral_rae_create.restype = C.c_int
    lib.spiral_rae_create.argtypes = [C.c_int, C.c_double, C.POINTER(vp)]
    lib.spiral_rae_update.restype = C.c_int
    lib.spiral_rae_update.argtypes = [vp, i32p, f64p, C.c_int, f64p]
    lib.spiral_rae_get.restype = C.c_int
    lib.spiral_rae_get.argtypes = [vp, f64p]
    lib.spiral_rae_set.restype = C.c_int
    lib.spiral_rae_set.argtypes = [vp, f64p]
    lib.spiral_rae_free.restype = None
    lib.spiral_rae_free.argtypes = [vp]
    if path is None:
        _lib = lib
    return lib


def _check(rc: int):
    if rc != SPIRAL_OK:
        raise SpiralError(rc, load_library().spiral_last_error().decode())


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.int32))


def _ip(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.POINTER(C.c_int32))


def _stream_handle(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    return getattr(stream, "cuda_stream", stream)


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


# ------------------------------------------------------------------------- plain functions
def spiral_version() -> str:
    return load_library().spiral_version().decode()


def spiral_last_error() -> str:
    return load_library().spiral_last_error().decode()


def make_config(g: _inputs.ModelGeometry) -> spiral_model_config:
    return spiral_model_config(g.n_layers, g.d_model, g.n_q_heads, g.n_kv_heads, g.head_dim, g.ffn_dim,
                               g.vocab, g.rope_theta, g.rms_eps, int(g.qk_norm), int(g.qkv_bias),
                               int(g.tie_lm_head), g.weight_dtype, g.kv_block_tokens)


def weight_pointer_table(g: _inputs.ModelGeometry, w: Dict[str, object]) -> List[Optional[int]]:
    """Device addresses in the order spiral_model_load expects (torch tensors on the GPU)."""
    ptrs: List[Optional[int]] = [w["embed"].data_ptr(), w["final_norm"].data_ptr(), w["lm_head"].data_ptr()]
    for lw in w["layers"]:
        for name in _inputs.LAYER_TENSORS:
            ptrs.append(lw[name].data_ptr() if name in lw else None)
    return ptrs


def spiral_model_load(cfg: spiral_model_config, dev_weight_ptrs: Sequence[Optional[int]]) -> int:
    lib = load_library()
    arr = (C.c_void_p * len(dev_weight_ptrs))(*[C.c_void_p(p) if p else None for p in dev_weight_ptrs])
    out = C.c_void_p()
    _check(lib.spiral_model_load(C.byref(cfg), arr, len(dev_weight_ptrs), C.byref(out)))
    return out.value


def spiral_model_free(model: int):
    load_library().spiral_model_free(model)


def spiral_workspace_bytes(model: int, max_rows: int, max_context: int) -> int:
    return load_library().spiral_workspace_bytes(model, max_rows, max_context)


def spiral_kv_pool_bytes(model: int, n_pages: int, max_seqs: int, max_blocks_per_seq: int) -> int:
    return load_library().spiral_kv_pool_bytes(model, n_pages, max_seqs, max_blocks_per_seq)


def spiral_kv_pool_create(model: int, dev_mem, n_pages: int, max_seqs: int, max_blocks_per_seq: int,
                          page_order=None, stream=None) -> int:
    out = C.c_void_p()
    po = None if page_order is None else _i32(page_order)
    _check(load_library().spiral_kv_pool_create(model, dev_mem.data_ptr(), dev_mem.numel() * dev_mem.element_size(),
                                                n_pages, max_seqs, max_blocks_per_seq, _ip(po),
                                                _stream_handle(stream), C.byref(out)))
    return out.value


def spiral_kv_pool_free(pool: int):
    load_library().spiral_kv_pool_free(pool)


def spiral_seq_reset(pool: int, seq_ids, stream=None):
    ids = _i32(seq_ids)
    _check(load_library().spiral_seq_reset(pool, _ip(ids), int(ids.shape[0]), _stream_handle(stream)))


def spiral_seq_truncate(pool: int, seq_ids, new_lens, stream=None):
    ids, ln = _i32(seq_ids), _i32(new_lens)
    _check(load_library().spiral_seq_truncate(pool, _ip(ids), _ip(ln), int(ids.shape[0]), _stream_handle(stream)))


KERNEL_CLASSES = ["attn_decode", "attn_combine", "attn_prefill", "gemm_qkv", "gemm_o", "gemm_gate_up",
                  "gemm_down", "gemm_lm_head", "norm", "qkv_post", "sample"]


def spiral_profile_begin(model: int, kernel_class: int, max_launches: int):
    _check(load_library().spiral_profile_begin(model, kernel_class, max_launches))


def spiral_profile_end(model: int):
    """-> (total milliseconds, launches timed)"""
    ms, n = C.c_double(0.0), C.c_int(0)
    _check(load_library().spiral_profile_end(model, C.byref(ms), C.byref(n)))
    return ms.value, n.value


def spiral_seq_len(pool: int, seq_id: int) -> int:
    n = load_library().spiral_seq_len(pool, seq_id)
    if n < 0:
        _check(n)
    return n


def spiral_kv_free_pages(pool: int) -> int:
    return load_library().spiral_kv_free_pages(pool)


def spiral_prefill(model: int, pool: int, seq_ids, lens, dev_tokens_packed, dev_ws, dev_logits, stream=None):
    ids, ln = _i32(seq_ids), _i32(lens)
    _check(load_library().spiral_prefill(model, pool, _ip(ids), _ip(ln), int(ids.shape[0]),
                                         _ptr(dev_tokens_packed), _ptr(dev_ws),
                                         0 if dev_ws is None else dev_ws.numel() * dev_ws.element_size(),
                                         _ptr(dev_logits), _stream_handle(stream)))


def spiral_decode_step(model: int, pool: int, seq_ids, dev_in_tokens, dev_ws, dev_logits, stream=None):
    ids = seq_ids if isinstance(seq_ids, np.ndarray) and seq_ids.dtype == np.int32 else _i32(seq_ids)
    _check(load_library().spiral_decode_step(model, pool, _ip(ids), int(ids.shape[0]), _ptr(dev_in_tokens),
                                             _ptr(dev_ws),
                                             0 if dev_ws is None else dev_ws.numel() * dev_ws.element_size(),
                                             _ptr(dev_logits), _stream_handle(stream)))


def spiral_decode_sample_step(model: int, pool: int, seq_ids, dev_in_tokens, dev_ws, temperature: float, seed: int, steps,
                              dev_out_tokens, stream=None):
    ids = seq_ids if isinstance(seq_ids, np.ndarray) and seq_ids.dtype == np.int32 else _i32(seq_ids)
    st = None if steps is None else (steps if isinstance(steps, np.ndarray) and steps.dtype == np.int32 else _i32(steps))
    _check(load_library().spiral_decode_sample_step(model, pool, _ip(ids), int(ids.shape[0]), _ptr(dev_in_tokens), _ptr(dev_ws),
                                                    0 if dev_ws is None else dev_ws.numel() * dev_ws.element_size(),
                                                    C.c_float(temperature), C.c_uint64(seed), _ip(st), _ptr(dev_out_tokens),
                                                    _stream_handle(stream)))


def spiral_decode_step_static(model: int, pool: int, seq_ids, dev_in_tokens, dev_logits, stream=None):
    ids = _i32(seq_ids)
    _check(load_library().spiral_decode_step_static(model, pool, _ip(ids), int(ids.shape[0]), _ptr(dev_in_tokens),
                                                    _ptr(dev_logits), _stream_handle(stream)))


def spiral_static_workspace_bytes() -> int:
    return load_library().spiral_static_workspace_bytes()


def spiral_probe_stream_read(dev_buf, nbytes: int, iters: int = 5, stream=None) -> float:
    """-> GB/s of a pure streaming read over the first nbytes of dev_buf"""
    ms = C.c_double(0.0)
    _check(load_library().spiral_probe_stream_read(_ptr(dev_buf), C.c_size_t(nbytes), iters, C.byref(ms), _stream_handle(stream)))
    return nbytes / (ms.value * 1e-3) / 1e9


def spiral_model_tune(model: int, spec: str):
    _check(load_library().spiral_model_tune(model, spec.encode()))


def spiral_kv_pool_status_offset(pool: int) -> int:
    off = load_library().spiral_kv_pool_status_offset(pool)
    if off < 0:
        _check(int(off))
    return int(off)


def spiral_sample(dev_logits, B: int, V: int, temperature: float, seed: int, seq_ids, steps, dev_noise,
                  dev_out_tokens, stream=None):
    ids = None if seq_ids is None else _i32(seq_ids)
    st = None if steps is None else _i32(steps)
    _check(load_library().spiral_sample(_ptr(dev_logits), B, V, float(temperature), C.c_uint64(seed), _ip(ids),
                                        _ip(st), _ptr(dev_noise), _ptr(dev_out_tokens), _stream_handle(stream)))


def spiral_score(model: int, pool: int, seq_ids, lens, dev_tokens_packed, dev_targets, ws, dev_logp, stream=None):
    ids, ln = _i32(seq_ids), _i32(lens)
    _check(load_library().spiral_score(model, pool, _ip(ids), _ip(ln), int(ids.shape[0]), _ptr(dev_tokens_packed),
                                       _ptr(dev_targets), _ptr(ws), C.c_size_t(ws.numel() * ws.element_size()),
                                       _ptr(dev_logp), _stream_handle(stream)))


def spiral_policy_objective(dev_logp_new, dev_logp_old, dev_advantage, dev_mask, n: int, clip_eps: float, dev_out2, stream=None):
    _check(load_library().spiral_policy_objective(_ptr(dev_logp_new), _ptr(dev_logp_old), _ptr(dev_advantage), _ptr(dev_mask),
                                                  C.c_longlong(n), C.c_float(clip_eps), _ptr(dev_out2), _stream_handle(stream)))


def spiral_sample_truncated(dev_logits, B: int, V: int, temperature: float, top_k: int, top_p: float, seed: int, seq_ids,
                            steps, dev_noise, dev_out_tokens, dev_threshold_out=None, stream=None):
    ids = None if seq_ids is None else _i32(seq_ids)
    st = None if steps is None else _i32(steps)
    _check(load_library().spiral_sample_truncated(_ptr(dev_logits), B, V, C.c_float(temperature), int(top_k), C.c_float(top_p),
                                                  C.c_uint64(seed), _ip(ids), _ip(st), _ptr(dev_noise), _ptr(dev_out_tokens),
                                                  _ptr(dev_threshold_out), _stream_handle(stream)))


def spiral_sample_truncated_workspace_bytes(B: int, V: int) -> int:
    return int(load_library().spiral_sample_truncated_workspace_bytes(B, V))


def spiral_sample_truncated_ws(dev_logits, B: int, V: int, temperature: float, top_k: int, top_p: float, seed: int, seq_ids,
                               steps, dev_noise, dev_out_tokens, dev_threshold_out, dev_workspace, workspace_bytes: int,
                               stream=None):
    ids = None if seq_ids is None else _i32(seq_ids)
    st = None if steps is None else _i32(steps)
    _check(load_library().spiral_sample_truncated_ws(_ptr(dev_logits), B, V, C.c_float(temperature), int(top_k), C.c_float(top_p),
                                                     C.c_uint64(seed), _ip(ids), _ip(st), _ptr(dev_noise), _ptr(dev_out_tokens),
                                                     _ptr(dev_threshold_out), _ptr(dev_workspace), C.c_size_t(workspace_bytes),
                                                     _stream_handle(stream)))


# ------------------------------------------------------------------------- RAE (host only)
def spiral_rae_create(n_games: int, alpha: float = 0.95) -> int:
    out = C.c_void_p()
    _check(load_library().spiral_rae_create(n_games, alpha, C.byref(out)))
    return out.value


def spiral_rae_update(rae: int, game_id, r0) -> np.ndarray:
    gid = _i32(game_id)
    r = np.ascontiguousarray(np.asarray(r0, dtype=np.float64))
    adv = np.empty((gid.shape[0], 2), dtype=np.float64)
    dp = C.POINTER(C.c_double)
    _check(load_library().spiral_rae_update(rae, _ip(gid), r.ctypes.data_as(dp), int(gid.shape[0]),
                                            adv.ctypes.data_as(dp)))
    return adv


def spiral_rae_get(rae: int, n_games: int) -> np.ndarray:
    b = np.empty((n_games, 2), dtype=np.float64)
    _check(load_library().spiral_rae_get(rae, b.ctypes.data_as(C.POINTER(C.c_double))))
    return b


def spiral_rae_set(rae: int, b):
    b = np.ascontiguousarray(np.asarray(b, dtype=np.float64))
    _check(load_library().spiral_rae_set(rae, b.ctypes.data_as(C.POINTER(C.c_double))))


def spiral_rae_free(rae: int):
    load_library().spiral_rae_free(rae)


# ------------------------------------------------------------------------- buffer holder
class Session:
    """Owns the device buffers one model needs (torch tensors) and forwards to the C ABI.
    It adds no computation of its own."""

    def __init__(self, g: _inputs.ModelGeometry, weights_dev: Dict[str, object], n_pages: int, max_seqs: int,
                 max_blocks_per_seq: int, max_rows: int, max_context: int, page_order=None, device="cuda:0",
                 repack: bool = True, tune: Optional[str] = None):
        import torch
        self.torch = torch
        self.g = g
        self.device = torch.device(device)
        self.weights = weights_dev                       # keeps the tensors alive
        self.model = spiral_model_load(make_config(g), weight_pointer_table(g, weights_dev))
        if tune:
            spiral_model_tune(self.model, tune)
        self.repacked = None
        nbytes = load_library().spiral_model_repack_bytes(self.model) if repack else 0
        if nbytes:
            self.repacked = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
            _check(load_library().spiral_model_repack(self.model, _ptr(self.repacked), C.c_size_t(nbytes), None))
        self.pool_mem = torch.empty(spiral_kv_pool_bytes(self.model, n_pages, max_seqs, max_blocks_per_seq),
                                    dtype=torch.uint8, device=self.device)
        self.pool = spiral_kv_pool_create(self.model, self.pool_mem, n_pages, max_seqs, max_blocks_per_seq, page_order)
        self.ws = torch.empty(spiral_workspace_bytes(self.model, max_rows, max_context), dtype=torch.uint8,
                              device=self.device)
        self.max_rows, self.max_context = max_rows, max_context

    def new_logits(self, batch: int):
        return self.torch.empty((batch, self.g.vocab), dtype=self.torch.float32, device=self.device)

    def prefill(self, seq_ids, prompts: Sequence[np.ndarray], logits=None):
        lens = [len(p) for p in prompts]
        toks = self.torch.from_numpy(np.concatenate([np.asarray(p, dtype=np.int32) for p in prompts])).to(self.device)
        logits = self.new_logits(len(lens)) if logits is None else logits
        spiral_prefill(self.model, self.pool, seq_ids, lens, toks, self.ws, logits)
        return logits

    def decode_step(self, seq_ids, dev_in_tokens, logits):
        spiral_decode_step(self.model, self.pool, seq_ids, dev_in_tokens, self.ws, logits)
        return logits

    def decode_sample_step(self, seq_ids, dev_in_tokens, temperature: float, seed: int, steps, out_tokens):
        spiral_decode_sample_step(self.model, self.pool, seq_ids, dev_in_tokens, self.ws, temperature, seed, steps, out_tokens)
        return out_tokens

    def saturation_count(self) -> int:
        """Activation values that did not fit the 16-bit format since the pool was created (synchronises)."""
        off = spiral_kv_pool_status_offset(self.pool)
        return int(self.pool_mem[off:off + 4].view(self.torch.int32).cpu().item())

    def sample(self, logits, temperature: float, seed: int, seq_ids, steps, out_tokens, noise=None):
        spiral_sample(logits, logits.shape[0], logits.shape[1], temperature, seed, seq_ids, steps, noise, out_tokens)
        return out_tokens

    def close(self):
        if self.pool:
            spiral_kv_pool_free(self.pool)
            self.pool = None
        if self.model:
            spiral_model_free(self.model)
            self.model = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def weights_to_device(w_host: Dict[str, object], device="cuda:0") -> Dict[str, object]:
    """make_weights() host arrays -> torch tensors on the device (uint16 bit patterns become bf16)."""
    import torch

    def conv(a):
        t = torch.from_numpy(np.ascontiguousarray(a))
        if a.dtype == np.uint16:
            t = t.view(torch.int16).view(torch.bfloat16)
        return t.to(device)

    out = {"embed": conv(w_host["embed"]), "final_norm": conv(w_host["final_norm"])}
    out["lm_head"] = out["embed"] if w_host["lm_head"] is w_host["embed"] else conv(w_host["lm_head"])
    out["layers"] = [{k: conv(v) for k, v in lw.items()} for lw in w_host["layers"]]
    return out
