"""Thin ctypes binding of libcqa.so: argument marshalling only.

Function names mirror the C ABI in include/cqa.h (the product boundary) and
include/cqa_test.h (test hooks and measurement helpers).  Pointers are accepted as
Python ints, ctypes pointers or any object with a `data_ptr()` method (e.g. a
torch tensor used purely as device memory).  Every computation runs in the HIP
library; there is no CPU fallback: if the library is missing or fails to load,
importing this module raises.
"""
from __future__ import annotations

import ctypes as C
import math
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("CQA_LIB") or os.path.join(_HERE, "libcqa.so")

OK = 0
ERR_INVALID_ARG = -1
ERR_OOM_DEVICE = -2
ERR_OOM_PINNED = -3
ERR_NO_TIER2 = -4
ERR_CAPACITY = -5
ERR_HIP = -6
ERR_UNSUPPORTED = -7
ERR_SCRATCH = -8
STATIC_SCRATCH_BYTES = 4 * 1024 * 1024

TIER2_PINNED = 0
TIER2_NONE = 1

FLAG_KEY = 0x01
FLAG_VAL = 0x02
FLAG_RANK = 0x04
FLAG_PRECOND = 0x08
FLAG_TOTAL = 0x10
FLAG_ANY = 0x1F
RUNG_SHIFT = 8


class CacheDesc(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("batch", C.c_int32), ("n_q_heads", C.c_int32),
                ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("block_tokens", C.c_int32),
                ("v_group", C.c_int32), ("tier2_mode", C.c_int32), ("max_tokens", C.c_int64)]


class Tolerances(C.Structure):
    _fields_ = [("eps_total", C.c_float), ("eps_key", C.c_float), ("eps_val", C.c_float),
                ("v_tol", C.c_float), ("rank_min_mass", C.c_float), ("eps_guard", C.c_float),
                ("rank_depth", C.c_int32), ("mass_exp", C.c_int32), ("key_bound_mode", C.c_int32),
                ("rung4_min_groups", C.c_int32), ("force_flags", C.c_uint32), ("int8_query", C.c_int32)]

    def __init__(self, eps_total=math.inf, eps_key=math.inf, eps_val=math.inf, v_tol=math.inf,
                 rank_min_mass=0.0, eps_guard=1e-6, rank_depth=0, mass_exp=2, key_bound_mode=0,
                 rung4_min_groups=0, force_flags=0, int8_query=False):
        super().__init__(eps_total, eps_key, eps_val, v_tol, rank_min_mass, eps_guard, rank_depth,
                         mass_exp, key_bound_mode, rung4_min_groups, force_flags, 1 if int8_query else 0)


class Selector(C.Structure):
    """Parameters of the adaptive key-precision selector (cqa_selector)."""
    _fields_ = [("tau_cov", C.c_float), ("k_min", C.c_int32), ("k_max", C.c_int32),
                ("k_limit", C.c_int32), ("v_limit", C.c_int32), ("v_greedy", C.c_int32),
                ("canary", C.c_int32), ("explore_frac", C.c_float), ("explore_seed", C.c_uint32),
                ("per_head", C.c_int32)]

    def __init__(self, tau_cov=0.995, k_min=2, k_max=128, k_limit=None, v_limit=0, v_greedy=False,
                 canary=False, explore_frac=0.0, explore_seed=0, per_head=False):
        super().__init__(tau_cov, k_min, k_max, k_max if k_limit is None else k_limit, v_limit,
                         1 if v_greedy else 0, 1 if canary else 0, explore_frac,
                         explore_seed & 0xFFFFFFFF, 1 if per_head else 0)


MAX_K_LIMIT = 512


class HeadCert(C.Structure):
    _fields_ = [("E_key", C.c_float), ("E_val", C.c_float), ("delta_h", C.c_float),
                ("v_max", C.c_float), ("alpha_tail_hat", C.c_float), ("lse", C.c_float),
                ("max_block_contrib", C.c_float), ("rank_margin", C.c_float),
                ("top_block", C.c_int32), ("served_rung", C.c_int32)]


CERT_BYTES = C.sizeof(HeadCert)
# numpy structured dtype with the same layout, for reading certificates back
CERT_FIELDS = [("E_key", "<f4"), ("E_val", "<f4"), ("delta_h", "<f4"), ("v_max", "<f4"),
               ("alpha_tail_hat", "<f4"), ("lse", "<f4"), ("max_block_contrib", "<f4"),
               ("rank_margin", "<f4"), ("top_block", "<i4"), ("served_rung", "<i4")]


class CqaError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = _lib.cqa_strerror(status).decode() if _lib is not None else "?"
        hip = _lib.cqa_last_hip_error() if _lib is not None and status == ERR_HIP else 0
        super().__init__(f"{where}: {msg} (status {status}" + (f", hipError {hip})" if hip else ")"))


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2605_20868_amd.build` "
                          "(there is no CPU fallback)")
    try:
        # One HIP runtime per process: if torch is around, its bundled runtime must be the one
        # that gets loaded, and it must be loaded before this library resolves libamdhip64.
        import torch  # noqa: F401
    except ImportError:
        pass
    lib = C.CDLL(LIB_PATH)
    vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
    sig = {
        "cqa_cache_create": (i32, [C.POINTER(CacheDesc), C.POINTER(vp)]),
        "cqa_cache_create_caller_tier2": (i32, [C.POINTER(CacheDesc), vp, vp, i64, C.POINTER(vp)]),
        "cqa_cache_destroy": (i32, [vp]),
        "cqa_workspace_bytes": (i32, [C.POINTER(CacheDesc), C.POINTER(i64), C.POINTER(i64)]),
        "cqa_cache_append": (i32, [vp, i32, vp, vp, i64, vp]),
        "cqa_cache_length": (i32, [vp, i32, C.POINTER(i64)]),
        "cqa_cache_reset": (i32, [vp, i32]),
        "cqa_cache_export_block": (i32, [vp, i32, i32, i32, i64, vp, vp, vp, vp, vp, vp, vp, vp]),
        "cqa_certified_decode": (i32, [vp, i32, vp, C.POINTER(Tolerances), vp, vp, vp, vp, vp]),
        "cqa_certified_decode_noalloc": (i32, [vp, i32, vp, C.POINTER(Tolerances), vp, vp, vp, vp]),
        "cqa_dense_fallback": (i32, [vp, i32, vp, vp, i32, i32, vp, vp, vp, vp]),
        "cqa_decode_step": (i32, [vp, i32, vp, C.POINTER(Tolerances), vp, vp, vp, vp,
                                  C.POINTER(i32), vp]),
        "cqa_append_decode_step": (i32, [vp, i32, vp, vp, vp, C.POINTER(Tolerances), vp, vp, vp,
                                         C.POINTER(i32), vp]),
        "cqa_decode_step_enqueue": (i32, [vp, i32, vp, vp, vp, C.POINTER(Tolerances), vp, vp, vp, vp]),
        "cqa_ladder_counts": (i32, [vp, C.POINTER(i64), C.POINTER(i64)]),
        "cqa_adaptive_decode": (i32, [vp, i32, vp, C.POINTER(Tolerances), C.POINTER(Selector), vp, vp,
                                      vp, vp]),
        "cqa_adaptive_step": (i32, [vp, i32, vp, C.POINTER(Tolerances), C.POINTER(Selector), vp, vp,
                                    vp, C.POINTER(i32), vp]),
        "cqa_adaptive_step_enqueue": (i32, [vp, i32, vp, C.POINTER(Tolerances), C.POINTER(Selector), vp, vp,
                                            vp, vp]),
        "cqa_set_scratch_slots": (i32, [vp, i32]),
        "cqa_scratch_stats": (i32, [vp, C.POINTER(i32), C.POINTER(i64), C.POINTER(i64)]),
        "cqa_adaptive_state": (i32, [vp, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp]),
        "cqa_dense_attention": (i32, [vp, vp, vp, i32, i32, i32, i64, vp, vp, vp]),
        "cqa_dense_workspace_bytes": (i64, [i32, i32, i64]),
        "cqa_time_certified_decode": (i32, [vp, i32, vp, C.POINTER(Tolerances), vp, vp, vp, vp,
                                            i32, C.POINTER(C.c_float), vp]),
        "cqa_time_stream_read": (i32, [vp, i32, i32, C.POINTER(C.c_float), C.POINTER(i64), vp]),
        "cqa_profile_begin": (i32, [vp, i32]),
        "cqa_profile_end": (i32, [vp, C.POINTER(C.c_float), C.POINTER(C.c_float), C.POINTER(i32)]),
        "cqa_profile_durations": (i32, [vp, vp, i32, C.POINTER(i32)]),
        "cqa_decode_splits": (i32, [vp, i32, C.POINTER(i32)]),
        "cqa_set_splits": (i32, [vp, i32]),
        "cqa_set_stream_hint": (i32, [vp, i32]),
        "cqa_set_kernel_variant": (i32, [vp, i32]),
        "cqa_strerror": (C.c_char_p, [i32]),
        "cqa_version": (i32, []),
        "cqa_last_hip_error": (i32, []),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)      # raises AttributeError if the symbol is not exported
        fn.restype = res
        fn.argtypes = args
    return lib, sorted(sig)


_lib = None
_lib, EXPORTED = _load()


def _ptr(x):
    if x is None:
        return None
    if isinstance(x, int):
        return C.c_void_p(x)
    if hasattr(x, "data_ptr"):
        return C.c_void_p(x.data_ptr())
    if hasattr(x, "ctypes"):
        return C.c_void_p(x.ctypes.data)
    return x


def _check(status: int, where: str) -> None:
    if status != OK:
        raise CqaError(status, where)


def cqa_version() -> int:
    return _lib.cqa_version()


def cqa_strerror(status: int) -> str:
    return _lib.cqa_strerror(status).decode()


def cqa_last_hip_error() -> int:
    return _lib.cqa_last_hip_error()


def cqa_workspace_bytes(desc: CacheDesc):
    dev, pin = C.c_int64(0), C.c_int64(0)
    _check(_lib.cqa_workspace_bytes(C.byref(desc), C.byref(dev), C.byref(pin)), "cqa_workspace_bytes")
    return dev.value, pin.value


def cqa_cache_create(n_layers, batch, n_q_heads, n_kv_heads, max_tokens, tier2_mode=TIER2_PINNED,
                     head_dim=128, block_tokens=16, v_group=16):
    desc = CacheDesc(n_layers, batch, n_q_heads, n_kv_heads, head_dim, block_tokens, v_group,
                     tier2_mode, max_tokens)
    h = C.c_void_p(None)
    _check(_lib.cqa_cache_create(C.byref(desc), C.byref(h)), "cqa_cache_create")
    return h


def cqa_cache_create_caller_tier2(n_layers, batch, n_q_heads, n_kv_heads, max_tokens, t2_k_host, t2_v_host,
                                  bytes_each, head_dim=128, block_tokens=16, v_group=16):
    """t2_k_host / t2_v_host: pinned host memory (address, or an object with data_ptr())."""
    desc = CacheDesc(n_layers, batch, n_q_heads, n_kv_heads, head_dim, block_tokens, v_group,
                     TIER2_PINNED, max_tokens)
    h = C.c_void_p(None)
    _check(_lib.cqa_cache_create_caller_tier2(C.byref(desc), _ptr(t2_k_host), _ptr(t2_v_host), bytes_each,
                                              C.byref(h)), "cqa_cache_create_caller_tier2")
    return h


def cqa_cache_destroy(h) -> None:
    _check(_lib.cqa_cache_destroy(h), "cqa_cache_destroy")


def cqa_cache_append(h, layer, k_dev, v_dev, n_new, stream=None) -> None:
    _check(_lib.cqa_cache_append(h, layer, _ptr(k_dev), _ptr(v_dev), n_new, _ptr(stream)),
           "cqa_cache_append")


def cqa_cache_length(h, layer) -> int:
    n = C.c_int64(0)
    _check(_lib.cqa_cache_length(h, layer, C.byref(n)), "cqa_cache_length")
    return n.value


def cqa_cache_reset(h, layer) -> None:
    _check(_lib.cqa_cache_reset(h, layer), "cqa_cache_reset")


def cqa_cache_export_block(h, layer, batch, kv_head, block):
    """Returns numpy arrays (kcodes i8[16,128], sigma f32[128], z f32[128], vcodes u8[16,128],
    vscale f16[16,8], voffset f16[16,8], eta f32, nu f32) -- the canonical logical view."""
    import numpy as np
    kc = np.empty((16, 128), np.int8)
    sg = np.empty(128, np.float32)
    z = np.empty(128, np.float32)
    vc = np.empty((16, 128), np.uint8)
    vs = np.empty((16, 8), np.uint16)
    vo = np.empty((16, 8), np.uint16)
    eta = C.c_float(0)
    nu = C.c_float(0)
    _check(_lib.cqa_cache_export_block(h, layer, batch, kv_head, block, _ptr(kc), _ptr(sg), _ptr(z),
                                       _ptr(vc), _ptr(vs), _ptr(vo),
                                       C.cast(C.byref(eta), C.c_void_p),
                                       C.cast(C.byref(nu), C.c_void_p)), "cqa_cache_export_block")
    import numpy as _np
    return (kc, sg, z, vc, vs.view(_np.float16), vo.view(_np.float16),
            _np.float32(eta.value), _np.float32(nu.value))


def cqa_certified_decode(h, layer, q_dev, tol: Tolerances, O_dev, cert_dev, flags_dev,
                         blk_logmass_dev=None, stream=None) -> None:
    _check(_lib.cqa_certified_decode(h, layer, _ptr(q_dev), C.byref(tol), _ptr(O_dev),
                                     _ptr(cert_dev), _ptr(flags_dev), _ptr(blk_logmass_dev),
                                     _ptr(stream)), "cqa_certified_decode")


def cqa_certified_decode_noalloc(h, layer, q_dev, tol: Tolerances, O_dev, cert_dev, flags_dev,
                                 stream=None) -> None:
    _check(_lib.cqa_certified_decode_noalloc(h, layer, _ptr(q_dev), C.byref(tol), _ptr(O_dev),
                                             _ptr(cert_dev), _ptr(flags_dev), _ptr(stream)),
           "cqa_certified_decode_noalloc")


def cqa_dense_fallback(h, layer, q_dev, head_select_host, all_heads, rung, O_dev, cert_dev=None,
                       flags_dev=None, stream=None) -> None:
    _check(_lib.cqa_dense_fallback(h, layer, _ptr(q_dev), _ptr(head_select_host), int(all_heads),
                                   rung, _ptr(O_dev), _ptr(cert_dev), _ptr(flags_dev),
                                   _ptr(stream)), "cqa_dense_fallback")


def cqa_decode_step(h, layer, q_dev, tol: Tolerances, O_dev, cert_dev, flags_dev,
                    blk_logmass_dev=None, stream=None) -> int:
    rung = C.c_int32(0)
    _check(_lib.cqa_decode_step(h, layer, _ptr(q_dev), C.byref(tol), _ptr(O_dev), _ptr(cert_dev),
                                _ptr(flags_dev), _ptr(blk_logmass_dev), C.byref(rung),
                                _ptr(stream)), "cqa_decode_step")
    return rung.value


def cqa_append_decode_step(h, layer, k_dev, v_dev, q_dev, tol: Tolerances, O_dev, cert_dev, flags_dev,
                           stream=None) -> int:
    rung = C.c_int32(0)
    _check(_lib.cqa_append_decode_step(h, layer, _ptr(k_dev), _ptr(v_dev), _ptr(q_dev), C.byref(tol),
                                       _ptr(O_dev), _ptr(cert_dev), _ptr(flags_dev), C.byref(rung),
                                       _ptr(stream)), "cqa_append_decode_step")
    return rung.value


def cqa_decode_step_enqueue(h, layer, k_dev, v_dev, q_dev, tol: Tolerances, O_dev, cert_dev, flags_dev,
                            stream=None) -> None:
    _check(_lib.cqa_decode_step_enqueue(h, layer, _ptr(k_dev), _ptr(v_dev), _ptr(q_dev), C.byref(tol),
                                        _ptr(O_dev), _ptr(cert_dev), _ptr(flags_dev), _ptr(stream)),
           "cqa_decode_step_enqueue")


def cqa_ladder_counts(h):
    r3, r4 = C.c_int64(0), C.c_int64(0)
    _check(_lib.cqa_ladder_counts(h, C.byref(r3), C.byref(r4)), "cqa_ladder_counts")
    return r3.value, r4.value


def cqa_adaptive_decode(h, layer, q_dev, tol: Tolerances, sel: Selector, O_dev, cert_dev, flags_dev,
                        stream=None) -> None:
    _check(_lib.cqa_adaptive_decode(h, layer, _ptr(q_dev), C.byref(tol), C.byref(sel), _ptr(O_dev),
                                    _ptr(cert_dev), _ptr(flags_dev), _ptr(stream)),
           "cqa_adaptive_decode")


def cqa_adaptive_step(h, layer, q_dev, tol: Tolerances, sel: Selector, O_dev, cert_dev, flags_dev,
                      stream=None) -> int:
    rung = C.c_int32(0)
    _check(_lib.cqa_adaptive_step(h, layer, _ptr(q_dev), C.byref(tol), C.byref(sel), _ptr(O_dev),
                                  _ptr(cert_dev), _ptr(flags_dev), C.byref(rung), _ptr(stream)),
           "cqa_adaptive_step")
    return rung.value


def cqa_adaptive_step_enqueue(h, layer, q_dev, tol: Tolerances, sel: Selector, O_dev, cert_dev, flags_dev,
                              stream=None) -> None:
    _check(_lib.cqa_adaptive_step_enqueue(h, layer, _ptr(q_dev), C.byref(tol), C.byref(sel), _ptr(O_dev),
                                          _ptr(cert_dev), _ptr(flags_dev), _ptr(stream)),
           "cqa_adaptive_step_enqueue")


def cqa_set_scratch_slots(h, n_slots) -> None:
    _check(_lib.cqa_set_scratch_slots(h, n_slots), "cqa_set_scratch_slots")


def cqa_scratch_stats(h):
    """(slots per head in use, hits, misses)"""
    n, hit, miss = C.c_int32(0), C.c_int64(0), C.c_int64(0)
    _check(_lib.cqa_scratch_stats(h, C.byref(n), C.byref(hit), C.byref(miss)), "cqa_scratch_stats")
    return n.value, hit.value, miss.value


def cqa_adaptive_state(h, layer, batch, n_q_heads, n_kv_heads):
    """Returns (k_star i32[Bt,Hq], selected i32[Bt,Hq,512], promoted u16[Bt,Hkv,NB] (bit 0 keys,
    bit 1 values for some head of the group; bits 4-7 / 8-11: for which heads), logmass_int8 f32[Bt,Hq,NB], logmass_mixed f32[Bt,Hq,NB], v_count i32[Bt,Hq],
    v_selected i32[Bt,Hq,512], contrib f32[Bt,Hq,NB], score_dev f32[Bt,Hq]) of the last adaptive
    decode."""
    import numpy as np
    nb = cqa_cache_length(h, layer) // 16
    ks = np.zeros((batch, n_q_heads), np.int32)
    sel = np.zeros((batch, n_q_heads, MAX_K_LIMIT), np.int32)
    prom = np.zeros((batch, n_kv_heads, nb), np.uint16)
    l8 = np.zeros((batch, n_q_heads, nb), np.float32)
    lx = np.zeros((batch, n_q_heads, nb), np.float32)
    vc = np.zeros((batch, n_q_heads), np.int32)
    vsel = np.zeros((batch, n_q_heads, MAX_K_LIMIT), np.int32)
    contrib = np.zeros((batch, n_q_heads, nb), np.float32)
    dev = np.zeros((batch, n_q_heads), np.float32)
    _check(_lib.cqa_adaptive_state(h, layer, _ptr(ks), _ptr(sel), _ptr(prom), _ptr(l8), _ptr(lx),
                                   _ptr(vc), _ptr(vsel), _ptr(contrib), _ptr(dev)), "cqa_adaptive_state")
    return ks, sel, prom, l8, lx, vc, vsel, contrib, dev


def cqa_dense_workspace_bytes(batch, n_q_heads, n_tokens) -> int:
    return _lib.cqa_dense_workspace_bytes(batch, n_q_heads, n_tokens)


def cqa_dense_attention(q_dev, k_dev, v_dev, batch, n_q_heads, n_kv_heads, n_tokens, O_dev,
                        workspace_dev, stream=None) -> None:
    _check(_lib.cqa_dense_attention(_ptr(q_dev), _ptr(k_dev), _ptr(v_dev), batch, n_q_heads,
                                    n_kv_heads, n_tokens, _ptr(O_dev), _ptr(workspace_dev),
                                    _ptr(stream)), "cqa_dense_attention")


def cqa_time_certified_decode(h, layer, q_dev, tol: Tolerances, O_dev, cert_dev, flags_dev,
                              blk_logmass_dev=None, iters=1, stream=None) -> float:
    ms = C.c_float(0)
    _check(_lib.cqa_time_certified_decode(h, layer, _ptr(q_dev), C.byref(tol), _ptr(O_dev),
                                          _ptr(cert_dev), _ptr(flags_dev), _ptr(blk_logmass_dev),
                                          iters, C.byref(ms), _ptr(stream)),
           "cqa_time_certified_decode")
    return ms.value


def cqa_time_stream_read(h, layer, iters, stream=None):
    """(ms per launch, bytes per launch) of the load-only kernel with the split pass's access pattern."""
    ms, nbytes = C.c_float(0.0), C.c_int64(0)
    _check(_lib.cqa_time_stream_read(h, layer, iters, C.byref(ms), C.byref(nbytes), _ptr(stream)),
           "cqa_time_stream_read")
    return ms.value, nbytes.value


def cqa_profile_begin(h, max_launches) -> None:
    _check(_lib.cqa_profile_begin(h, max_launches), "cqa_profile_begin")


def cqa_profile_end(h):
    """Returns (mean_ms, min_ms, n_launches) of the split-K decode kernel since profile_begin."""
    mean, mn, n = C.c_float(0), C.c_float(0), C.c_int32(0)
    _check(_lib.cqa_profile_end(h, C.byref(mean), C.byref(mn), C.byref(n)), "cqa_profile_end")
    return mean.value, mn.value, n.value


def cqa_profile_durations(h):
    """numpy float32 array: duration in ms of every launch timed by the last begin / end pair."""
    import numpy as np
    n = C.c_int32(0)
    _check(_lib.cqa_profile_durations(h, None, 0, C.byref(n)), "cqa_profile_durations")
    out = np.zeros(max(n.value, 1), np.float32)
    _check(_lib.cqa_profile_durations(h, _ptr(out), n.value, C.byref(n)), "cqa_profile_durations")
    return out[:n.value]


def cqa_decode_splits(h, layer) -> int:
    n = C.c_int32(0)
    _check(_lib.cqa_decode_splits(h, layer, C.byref(n)), "cqa_decode_splits")
    return n.value


def cqa_set_kernel_variant(h, variant) -> None:
    _check(_lib.cqa_set_kernel_variant(h, variant), "cqa_set_kernel_variant")


def cqa_set_stream_hint(h, mode) -> None:
    _check(_lib.cqa_set_stream_hint(h, mode), "cqa_set_stream_hint")


def cqa_set_splits(h, n_splits) -> None:
    _check(_lib.cqa_set_splits(h, n_splits), "cqa_set_splits")
