"""ctypes binding of include/pop.h: same names, argument marshalling only.

Device buffers are torch tensors (or raw integer addresses); `None` is NULL.  The HIP stream defaults to
torch's current stream.  Nothing here computes: every step runs in the library's kernels.  If the
library is not built the import fails loudly -- there is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("POP_HIP_LIB") or os.path.join(_HERE, "libpop_hip.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2602_06822_amd.build` "
                      "(there is no CPU fallback)")

_lib = C.CDLL(LIB_PATH)

POP_F32, POP_BF16 = 0, 1
POP_OK, POP_EINVAL, POP_ESHAPE, POP_ENOMEM, POP_EHIP, POP_ESTATE, POP_EUNSUPPORTED = 0, -1, -2, -3, -4, -5, -6
POP_EDEVICE = -7
POP_REGION_RETAINED, POP_REGION_CANDIDATE, POP_REGION_PRUNED = 0, 1, 2
POP_MAX_BATCH = 8

_vp, _i, _dbl = C.c_void_p, C.c_int, C.c_double
_ip = C.POINTER(C.c_int)

_SIGS = {
    "pop_version": (C.c_int, []),
    "pop_strerror": (C.c_char_p, [_i]),
    "pop_last_hip_error": (C.c_char_p, []),
    "pop_region_counts": (_i, [_i, _dbl, _dbl, _ip, _ip, _ip]),
    "pop_k_for_ratio": (_i, [_i, _dbl, _i, _i, _ip]),
    "pop_strategy_counts": (_i, [_i, _i, _dbl, _dbl, _ip, _ip, _ip]),
    "pop_layer_set_strategy": (_i, [_vp, _i, _dbl, _dbl]),
    "pop_layer_create": (_i, [C.POINTER(_vp), _i, _i, _i, _vp, _vp, _vp, _i, _i, _vp]),
    "pop_layer_destroy": (_i, [_vp]),
    "pop_prefill_partition": (_i, [_vp, _vp, _i, _i, _i, _vp, _vp, _vp, _vp, _vp]),
    "pop_prefill_forward": (_i, [_vp, _vp, _i, _i, _i, _i, _vp, _i, _vp, _vp, _vp, _vp, _vp, _vp]),
    "pop_decode_mask": (_i, [_vp, _vp, _i, _ip, _vp, _vp, _vp, _vp, _vp]),
    "pop_decode_step": (_i, [_vp, _vp, _i, _ip, _vp, _i, _vp, _vp, _vp, _vp, _vp]),
    "pop_pruned_ffn": (_i, [_vp, _vp, _i, _vp, _i, _vp, _i, _vp]),
    "pop_partition_from_scores": (_i, [_vp, _i, _i, _i, _vp, _vp, _vp, _vp]),
    "pop_partition_top_from_scores": (_i, [_vp, _i, _i, _i, _i, _vp, _vp, _vp, _vp, _vp, _vp]),
    "pop_topk_from_scores": (_i, [_vp, _vp, _i, _i, _vp, _i, _vp, _vp, _vp]),
    "pop_importance_reduce": (_i, [_vp, _i, _i, _i, _vp, _vp, _vp]),
    "pop_importance_reduce_static": (_i, [_vp, _i, _i, _i, _vp, _vp, _vp]),
    "pop_layer_reserve_prompt": (_i, [_vp, _i, _vp]),
    "pop_probe_read": (_i, [_vp, C.c_size_t, _i, _vp, _vp]),
    "pop_probe_step_read": (_i, [_vp, _i, _i, _vp, _vp]),
    "pop_layer_get_norms": (_i, [_vp, _vp, _vp]),
    "pop_layer_get_hidden": (_i, [_vp, _vp, _i, _vp]),
    "pop_layer_sync_status": (_i, [_vp, _vp]),
    "pop_layer_step_kind": (_i, [_vp, _ip]),
    "pop_layer_set_wait_limit": (_i, [_vp, _i]),
    "pop_layer_set_shared_batch_mask": (_i, [_vp, _i]),
    "pop_layer_set_importance": (_i, [_vp, _i]),
}
for _name, (_res, _args) in _SIGS.items():
    _fn = getattr(_lib, _name)
    _fn.restype = _res
    _fn.argtypes = _args

EXPORTED = tuple(_SIGS)


class PopError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = _lib.pop_strerror(status).decode()
        if status == POP_EHIP:
            msg += ": " + _lib.pop_last_hip_error().decode()
        super().__init__(f"{where}: {msg} ({status})")


def _check(status: int, where: str):
    if status != POP_OK:
        raise PopError(status, where)


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if not t.is_cuda:
        raise ValueError("device tensor expected")
    if not t.is_contiguous():
        raise ValueError("contiguous tensor expected")
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def pop_version() -> int:
    return _lib.pop_version()


def pop_strerror(status: int) -> str:
    return _lib.pop_strerror(status).decode()


def pop_last_hip_error() -> str:
    return _lib.pop_last_hip_error().decode()


def pop_region_counts(m: int, f_ret: float, f_cand: float):
    a, b, c = C.c_int(), C.c_int(), C.c_int()
    _check(_lib.pop_region_counts(m, f_ret, f_cand, C.byref(a), C.byref(b), C.byref(c)), "pop_region_counts")
    return a.value, b.value, c.value


def pop_k_for_ratio(m: int, r: float, n_ret: int, n_cand: int) -> int:
    k = C.c_int()
    _check(_lib.pop_k_for_ratio(m, r, n_ret, n_cand, C.byref(k)), "pop_k_for_ratio")
    return k.value


POP_STRATEGY_POP, POP_STRATEGY_STATIC_MASK, POP_STRATEGY_RESCORE_ALL = 0, 1, 2


def pop_strategy_counts(strategy: int, m: int, r: float, gamma: float):
    """(n_ret, n_cand, k) of a decode strategy of the ablation."""
    a, b, c = C.c_int(), C.c_int(), C.c_int()
    _check(_lib.pop_strategy_counts(strategy, m, r, gamma, C.byref(a), C.byref(b), C.byref(c)), "pop_strategy_counts")
    return a.value, b.value, c.value


def pop_layer_create(d, m, wdtype, w_gate, w_up, w_down, max_tokens, max_batch, stream=None):
    h = C.c_void_p()
    _check(_lib.pop_layer_create(C.byref(h), d, m, wdtype, _ptr(w_gate), _ptr(w_up), _ptr(w_down),
                                 max_tokens, max_batch, _stream(stream)), "pop_layer_create")
    return h


def pop_layer_destroy(layer):
    _check(_lib.pop_layer_destroy(layer), "pop_layer_destroy")


def pop_prefill_partition(layer, x, T, n_ret, n_cand, scores=None, region=None, ret_idx=None, cand_idx=None,
                          stream=None):
    _check(_lib.pop_prefill_partition(layer, _ptr(x), T, n_ret, n_cand, _ptr(scores), _ptr(region),
                                      _ptr(ret_idx), _ptr(cand_idx), _stream(stream)), "pop_prefill_partition")


def pop_prefill_forward(layer, x, T, n_ret, n_cand, k0, y, ydtype, scores=None, region=None, ret_idx=None,
                        cand_idx=None, mask=None, stream=None):
    _check(_lib.pop_prefill_forward(layer, _ptr(x), T, n_ret, n_cand, k0, _ptr(y), ydtype, _ptr(scores), _ptr(region),
                                    _ptr(ret_idx), _ptr(cand_idx), _ptr(mask), _stream(stream)), "pop_prefill_forward")


def _k_array(k, B):
    if k is None:  # the layer's strategy decides (pop_layer_set_strategy)
        return None
    if isinstance(k, int):
        k = [k] * B
    return (C.c_int * len(k))(*k)


def pop_decode_mask(layer, x_t, B, k, cand_scores=None, mask=None, active_idx=None, n_active=None, stream=None):
    _check(_lib.pop_decode_mask(layer, _ptr(x_t), B, _k_array(k, B), _ptr(cand_scores), _ptr(mask),
                                _ptr(active_idx), _ptr(n_active), _stream(stream)), "pop_decode_mask")


def pop_decode_step(layer, x_t, B, k, y, ydtype, cand_scores=None, mask=None, active_idx=None, n_active=None,
                    stream=None):
    _check(_lib.pop_decode_step(layer, _ptr(x_t), B, _k_array(k, B), _ptr(y), ydtype, _ptr(cand_scores), _ptr(mask),
                                _ptr(active_idx), _ptr(n_active), _stream(stream)), "pop_decode_step")


def pop_pruned_ffn(layer, x, T, mask, mask_rows, y, ydtype, stream=None):
    _check(_lib.pop_pruned_ffn(layer, _ptr(x), T, _ptr(mask), mask_rows, _ptr(y), ydtype, _stream(stream)),
           "pop_pruned_ffn")


def pop_partition_from_scores(scores, m, n_ret, n_cand, region=None, ret_idx=None, cand_idx=None, stream=None):
    _check(_lib.pop_partition_from_scores(_ptr(scores), m, n_ret, n_cand, _ptr(region), _ptr(ret_idx),
                                          _ptr(cand_idx), _stream(stream)), "pop_partition_from_scores")


def pop_partition_top_from_scores(scores, m, n_ret, n_cand, n_top, region=None, ret_idx=None, cand_idx=None,
                                  top_mask=None, top_list=None, stream=None):
    _check(_lib.pop_partition_top_from_scores(_ptr(scores), m, n_ret, n_cand, n_top, _ptr(region), _ptr(ret_idx),
                                              _ptr(cand_idx), _ptr(top_mask), _ptr(top_list), _stream(stream)),
           "pop_partition_top_from_scores")


def pop_topk_from_scores(cand_scores, cand_idx, n_cand, k, region, m, mask=None, sel_idx=None, stream=None):
    _check(_lib.pop_topk_from_scores(_ptr(cand_scores), _ptr(cand_idx), n_cand, k, _ptr(region), m, _ptr(mask),
                                     _ptr(sel_idx), _stream(stream)), "pop_topk_from_scores")


def pop_importance_reduce(h, hdtype, T, m, nrm, scores, stream=None):
    _check(_lib.pop_importance_reduce(_ptr(h), hdtype, T, m, _ptr(nrm), _ptr(scores), _stream(stream)),
           "pop_importance_reduce")


def pop_importance_reduce_static(h, hdtype, T, m, nrm, scores, stream=None):
    _check(_lib.pop_importance_reduce_static(_ptr(h), hdtype, T, m, _ptr(nrm), _ptr(scores), _stream(stream)),
           "pop_importance_reduce_static")


def pop_layer_reserve_prompt(layer, T: int, stream=None):
    _check(_lib.pop_layer_reserve_prompt(layer, T, _stream(stream)), "pop_layer_reserve_prompt")


def pop_probe_read(buf, nbytes: int, workgroups: int, sink, stream=None):
    _check(_lib.pop_probe_read(_ptr(buf), nbytes, workgroups, _ptr(sink), _stream(stream)), "pop_probe_read")


def pop_probe_step_read(layer, k: int, workgroups: int, sink, stream=None):
    _check(_lib.pop_probe_step_read(layer, k, workgroups, _ptr(sink), _stream(stream)), "pop_probe_step_read")


def pop_layer_get_norms(layer, nrm, stream=None):
    _check(_lib.pop_layer_get_norms(layer, _ptr(nrm), _stream(stream)), "pop_layer_get_norms")


def pop_layer_get_hidden(layer, h, B, stream=None):
    _check(_lib.pop_layer_get_hidden(layer, _ptr(h), B, _stream(stream)), "pop_layer_get_hidden")


def pop_layer_sync_status(layer, stream=None):
    _check(_lib.pop_layer_sync_status(layer, _stream(stream)), "pop_layer_sync_status")


POP_FROM_STRATEGY = -1


def pop_layer_set_strategy(layer, strategy: int, r: float, gamma: float = 0.0):
    _check(_lib.pop_layer_set_strategy(layer, strategy, r, gamma), "pop_layer_set_strategy")


def pop_layer_set_wait_limit(layer, looks: int):
    _check(_lib.pop_layer_set_wait_limit(layer, looks), "pop_layer_set_wait_limit")


POP_IMPORTANCE_OUTPUT_SIDE, POP_IMPORTANCE_INPUT_SIDE = 0, 1


def pop_layer_set_importance(layer, reading: int):
    _check(_lib.pop_layer_set_importance(layer, reading), "pop_layer_set_importance")


def pop_layer_set_shared_batch_mask(layer, on: bool):
    _check(_lib.pop_layer_set_shared_batch_mask(layer, 1 if on else 0), "pop_layer_set_shared_batch_mask")


def pop_layer_step_kind(layer):
    """(kind, workgroups): kind 0 none, 1 fused kernel, 2 batch-general kernels."""
    wg = C.c_int()
    kind = _lib.pop_layer_step_kind(layer, C.byref(wg))
    if kind < 0:
        raise PopError(kind, "pop_layer_step_kind")
    return kind, wg.value


def raw():
    """The ctypes library object, for callers that pre-marshal arguments (tight decode loops)."""
    return _lib
