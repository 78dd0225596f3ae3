"""Thin ctypes binding of ``liblshe.so`` -- argument marshalling only.

Function names and argument order follow ``include/lshe.h``.  Device buffers are
``torch`` tensors (used for memory and streams only); every step of the path runs in
the HIP kernels of the library.  There is no CPU fallback: if the library has not been
built, loading it raises.
"""
from __future__ import annotations

import ctypes as C
import os

LSHE_OK = 0
LSHE_INVALID_ARG = -1
LSHE_UNSUPPORTED = -2
LSHE_WORKSPACE_TOO_SMALL = -3
LSHE_HIP_ERROR = -4
LSHE_SCRATCH_EXCEEDED = -5
LSHE_BUILTIN_SCRATCH_BYTES = 2 << 20
LSHE_F32 = 0
LSHE_BF16 = 1
LSHE_POLICY_HASH = 0
LSHE_POLICY_L2NORM = 1
LSHE_STATUS_SELECT_TIMEOUT = 1
LSHE_PREFILL_HASH = 1
LSHE_PREFILL_EVICT = 2
LSHE_PREFILL_GATHER = 4

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblshe.so")

EXPORTS = ("lshe_strerror", "lshe_version", "lshe_check_config", "lshe_projection_bytes",
           "lshe_code_cache_bytes", "lshe_workspace_bytes", "lshe_decode_plan", "lshe_prefill_plan", "lshe_init_projection",
           "lshe_hash_keys", "lshe_key_norms", "lshe_prefill_compress", "lshe_prefill_phases", "lshe_decode_step", "lshe_decode_select",
           "lshe_decode_attend", "lshe_decode_step_noalloc", "lshe_debug_select_wait", "lshe_debug_prefill_ranges",
           "lshe_decode_select_unpacked")


class lshe_config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "head_dim", "hash_bits", "n_kv_heads", "gqa_group", "n_layers", "batch", "budget",
        "dtype", "n_sink", "n_recent", "policy")]


class LsheError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s failed: %s (%d)" % (where, strerror(status), status))


_lib = None


def lib():
    """Load the HIP library (built by ``paper_2412_16187_amd.build``); never falls back."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                "HIP library %s is missing: run `python -m paper_2412_16187_amd.build` "
                "(there is no CPU fallback)" % LIB_PATH)
        L = C.CDLL(LIB_PATH)
        vp, i32, i64, u64, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_uint64, C.c_size_t
        cfgp = C.POINTER(lshe_config)
        L.lshe_strerror.restype = C.c_char_p
        L.lshe_strerror.argtypes = [C.c_int]
        L.lshe_version.restype = C.c_char_p
        L.lshe_version.argtypes = []
        L.lshe_check_config.restype = C.c_int
        L.lshe_check_config.argtypes = [cfgp]
        for name in ("lshe_projection_bytes", "lshe_code_cache_bytes"):
            getattr(L, name).restype = sz
            getattr(L, name).argtypes = [cfgp]
        L.lshe_decode_plan.restype = C.c_char_p
        L.lshe_decode_plan.argtypes = [cfgp]
        L.lshe_prefill_plan.restype = C.c_char_p
        L.lshe_prefill_plan.argtypes = [cfgp, i32]
        L.lshe_workspace_bytes.restype = sz
        L.lshe_workspace_bytes.argtypes = [cfgp, i32]
        L.lshe_init_projection.restype = C.c_int
        L.lshe_init_projection.argtypes = [cfgp, u64, vp, vp, vp]
        L.lshe_hash_keys.restype = C.c_int
        L.lshe_hash_keys.argtypes = [cfgp, vp, vp, i64, vp, vp]
        L.lshe_key_norms.restype = C.c_int
        L.lshe_key_norms.argtypes = [cfgp, vp, i64, vp, vp]
        L.lshe_prefill_compress.restype = C.c_int
        L.lshe_prefill_compress.argtypes = [cfgp, vp, vp, vp, vp, i32, vp, vp, vp, vp, vp, vp,
                                            vp, sz, vp]
        L.lshe_prefill_phases.restype = C.c_int
        L.lshe_prefill_phases.argtypes = [cfgp, vp, vp, vp, vp, i32, vp, vp, vp, vp, vp, vp,
                                          vp, sz, vp, i32]
        L.lshe_decode_step.restype = C.c_int
        L.lshe_decode_step.argtypes = [cfgp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp,
                                       vp, vp, vp, sz, vp]
        L.lshe_decode_select_unpacked.restype = C.c_int
        L.lshe_decode_select_unpacked.argtypes = [cfgp] + [vp] * 9
        L.lshe_debug_select_wait.restype = None
        L.lshe_debug_select_wait.argtypes = [i32, i32]
        L.lshe_debug_prefill_ranges.restype = None
        L.lshe_debug_prefill_ranges.argtypes = [i32]
        L.lshe_decode_step_noalloc.restype = C.c_int
        L.lshe_decode_step_noalloc.argtypes = [cfgp] + [vp] * 16
        L.lshe_decode_select.restype = C.c_int
        L.lshe_decode_select.argtypes = [cfgp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp,
                                         vp, sz, vp]
        L.lshe_decode_attend.restype = C.c_int
        L.lshe_decode_attend.argtypes = [cfgp, vp, vp, vp, vp, vp, vp, sz, vp]
        _lib = L
    return _lib


def make_config(head_dim, hash_bits, n_kv_heads, gqa_group, n_layers, batch, budget, dtype,
                n_sink=0, n_recent=0, policy=LSHE_POLICY_HASH) -> lshe_config:
    if isinstance(dtype, str):
        dtype = {"f32": LSHE_F32, "bf16": LSHE_BF16}[dtype]
    if isinstance(policy, str):
        policy = {"hash": LSHE_POLICY_HASH, "l2": LSHE_POLICY_L2NORM}[policy]
    return lshe_config(head_dim, hash_bits, n_kv_heads, gqa_group, n_layers, batch, budget,
                       dtype, n_sink, n_recent, policy)


def _ptr(t):
    """Device (or host) address of a tensor / ndarray; None -> NULL."""
    if t is None:
        return None
    if hasattr(t, "data_ptr"):
        return C.c_void_p(t.data_ptr())
    return C.c_void_p(t.ctypes.data)


def _stream(stream):
    if stream is None:
        import torch
        return C.c_void_p(torch.cuda.current_stream().cuda_stream)
    if hasattr(stream, "cuda_stream"):
        return C.c_void_p(stream.cuda_stream)
    return C.c_void_p(int(stream))


def _check(status, where):
    if status != LSHE_OK:
        raise LsheError(status, where)


def strerror(status: int) -> str:
    return lib().lshe_strerror(int(status)).decode()


def version() -> str:
    return lib().lshe_version().decode()


def lshe_check_config(cfg) -> int:
    return int(lib().lshe_check_config(C.byref(cfg) if cfg is not None else None))


def lshe_projection_bytes(cfg) -> int:
    return int(lib().lshe_projection_bytes(C.byref(cfg)))


def lshe_code_cache_bytes(cfg) -> int:
    return int(lib().lshe_code_cache_bytes(C.byref(cfg)))


def lshe_decode_plan(cfg):
    p = lib().lshe_decode_plan(C.byref(cfg))
    return p.decode() if p else None


def lshe_prefill_plan(cfg, n_prompt: int):
    p = lib().lshe_prefill_plan(C.byref(cfg), int(n_prompt))
    return p.decode() if p else None


def lshe_workspace_bytes(cfg, n_prompt: int = 0) -> int:
    return int(lib().lshe_workspace_bytes(C.byref(cfg), int(n_prompt)))


def lshe_init_projection(cfg, seed, R_host, R_dev, stream=None, check=True) -> int:
    """R_host: float32 ndarray [d][r] or None; R_dev: device tensor of lshe_projection_bytes."""
    rc = lib().lshe_init_projection(C.byref(cfg), C.c_uint64(int(seed)), _ptr(R_host),
                                    _ptr(R_dev), _stream(stream))
    if check:
        _check(rc, "lshe_init_projection")
    return rc


def lshe_hash_keys(cfg, R_dev, X, n, codes, stream=None, check=True) -> int:
    rc = lib().lshe_hash_keys(C.byref(cfg), _ptr(R_dev), _ptr(X), C.c_int64(int(n)),
                              _ptr(codes), _stream(stream))
    if check:
        _check(rc, "lshe_hash_keys")
    return rc


def lshe_key_norms(cfg, X, n, norm2, stream=None, check=True) -> int:
    rc = lib().lshe_key_norms(C.byref(cfg), _ptr(X), C.c_int64(int(n)), _ptr(norm2), _stream(stream))
    if check:
        _check(rc, "lshe_key_norms")
    return rc


def lshe_prefill_compress(cfg, R_dev, K_prompt, V_prompt, Q_prompt, n_prompt, K_cache, V_cache,
                          code_cache, slot_pos, n_valid, evict_log, workspace, workspace_bytes=None,
                          stream=None, check=True) -> int:
    if workspace_bytes is None:
        workspace_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    rc = lib().lshe_prefill_compress(
        C.byref(cfg), _ptr(R_dev), _ptr(K_prompt), _ptr(V_prompt), _ptr(Q_prompt),
        C.c_int32(int(n_prompt)), _ptr(K_cache), _ptr(V_cache), _ptr(code_cache), _ptr(slot_pos),
        _ptr(n_valid), _ptr(evict_log), _ptr(workspace), C.c_size_t(int(workspace_bytes)),
        _stream(stream))
    if check:
        _check(rc, "lshe_prefill_compress")
    return rc


def lshe_prefill_phases(cfg, R_dev, K_prompt, V_prompt, Q_prompt, n_prompt, K_cache, V_cache,
                        code_cache, slot_pos, n_valid, evict_log, workspace, phases,
                        workspace_bytes=None, stream=None, check=True) -> int:
    if workspace_bytes is None:
        workspace_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    rc = lib().lshe_prefill_phases(
        C.byref(cfg), _ptr(R_dev), _ptr(K_prompt), _ptr(V_prompt), _ptr(Q_prompt),
        C.c_int32(int(n_prompt)), _ptr(K_cache), _ptr(V_cache), _ptr(code_cache), _ptr(slot_pos),
        _ptr(n_valid), _ptr(evict_log), _ptr(workspace), C.c_size_t(int(workspace_bytes)),
        _stream(stream), C.c_int32(int(phases)))
    if check:
        _check(rc, "lshe_prefill_phases")
    return rc


def lshe_decode_step(cfg, R_dev, q_new, k_new, v_new, pos, K_cache, V_cache, code_cache, slot_pos,
                     n_valid, out, evicted, scores_dbg, codes_dbg, evicted_mass, workspace,
                     workspace_bytes=None, stream=None, check=True) -> int:
    if workspace_bytes is None:
        workspace_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    rc = lib().lshe_decode_step(
        C.byref(cfg), _ptr(R_dev), _ptr(q_new), _ptr(k_new), _ptr(v_new), _ptr(pos),
        _ptr(K_cache), _ptr(V_cache), _ptr(code_cache), _ptr(slot_pos), _ptr(n_valid), _ptr(out),
        _ptr(evicted), _ptr(scores_dbg), _ptr(codes_dbg), _ptr(evicted_mass), _ptr(workspace),
        C.c_size_t(int(workspace_bytes)), _stream(stream))
    if check:
        _check(rc, "lshe_decode_step")
    return rc


def lshe_decode_step_noalloc(cfg, R_dev, q_new, k_new, v_new, pos, K_cache, V_cache, code_cache,
                             slot_pos, n_valid, out, evicted, scores_dbg, codes_dbg, evicted_mass,
                             stream=None, check=True) -> int:
    rc = lib().lshe_decode_step_noalloc(
        C.byref(cfg), _ptr(R_dev), _ptr(q_new), _ptr(k_new), _ptr(v_new), _ptr(pos),
        _ptr(K_cache), _ptr(V_cache), _ptr(code_cache), _ptr(slot_pos), _ptr(n_valid), _ptr(out),
        _ptr(evicted), _ptr(scores_dbg), _ptr(codes_dbg), _ptr(evicted_mass), _stream(stream))
    if check:
        _check(rc, "lshe_decode_step_noalloc")
    return rc


def lshe_decode_select_unpacked(cfg, R_dev, q_new, k_new, pos, code_bytes, slot_pos, n_valid, evicted,
                                stream=None, check=True) -> int:
    rc = lib().lshe_decode_select_unpacked(C.byref(cfg), _ptr(R_dev), _ptr(q_new), _ptr(k_new), _ptr(pos),
                                           _ptr(code_bytes), _ptr(slot_pos), _ptr(n_valid), _ptr(evicted),
                                           _stream(stream))
    if check:
        _check(rc, "lshe_decode_select_unpacked")
    return rc


def lshe_debug_select_wait(spin_limit: int, withhold_victim: int) -> None:
    lib().lshe_debug_select_wait(int(spin_limit), int(withhold_victim))


def lshe_debug_prefill_ranges(n: int) -> None:
    lib().lshe_debug_prefill_ranges(int(n))


def lshe_decode_select(cfg, R_dev, q_new, k_new, v_new, pos, K_cache, V_cache, code_cache,
                       slot_pos, n_valid, evicted, scores_dbg, codes_dbg, workspace,
                       workspace_bytes=None, stream=None, check=True) -> int:
    if workspace_bytes is None:
        workspace_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    rc = lib().lshe_decode_select(
        C.byref(cfg), _ptr(R_dev), _ptr(q_new), _ptr(k_new), _ptr(v_new), _ptr(pos),
        _ptr(K_cache), _ptr(V_cache), _ptr(code_cache), _ptr(slot_pos), _ptr(n_valid),
        _ptr(evicted), _ptr(scores_dbg), _ptr(codes_dbg), _ptr(workspace),
        C.c_size_t(int(workspace_bytes)), _stream(stream))
    if check:
        _check(rc, "lshe_decode_select")
    return rc


def lshe_decode_attend(cfg, q_new, K_cache, V_cache, n_valid, out, workspace,
                       workspace_bytes=None, stream=None, check=True) -> int:
    if workspace_bytes is None:
        workspace_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    rc = lib().lshe_decode_attend(
        C.byref(cfg), _ptr(q_new), _ptr(K_cache), _ptr(V_cache), _ptr(n_valid), _ptr(out),
        _ptr(workspace), C.c_size_t(int(workspace_bytes)), _stream(stream))
    if check:
        _check(rc, "lshe_decode_attend")
    return rc
