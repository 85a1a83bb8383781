"""ctypes access to the CPU oracle (oracle/pop_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  It marshals numpy arrays; all arithmetic is in
the C file.  It never imports the HIP package.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pop_oracle.c")
_LIB = os.path.join(_HERE, "libpop_oracle.so")

F32, BF16 = 0, 1


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (double precision, OpenMP over channels)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared",
                               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None

_TIMED_LIB = os.path.join(_HERE, "libpop_oracle_timed.so")
_TIMED_FLAGS = ["-O3", "-march=native", "-std=c11", "-fopenmp"]


def use_timed_build():
    """Switch this process to a build of the same source with -O3 -march=native (the benchmark's timed baseline leg;
    compiled on the machine it runs on).  Returns the flags."""
    global _lib
    subprocess.check_call(["gcc", *_TIMED_FLAGS, "-fPIC", "-shared", "-o", _TIMED_LIB, _SRC, "-lm"])
    _lib = C.CDLL(_TIMED_LIB)
    return list(_TIMED_FLAGS)


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _storage(a, dtype):
    want = np.float32 if dtype == F32 else np.uint16
    a = np.ascontiguousarray(a)
    assert a.dtype == want, (a.dtype, want)
    return a


def _check(rc, what):
    if rc != 0:
        raise ValueError(f"oracle {what} failed with status {rc}")


def num_threads() -> int:
    return int(lib().pop_oracle_num_threads())


def region_counts(m, f_ret, f_cand):
    a, b, c = C.c_int(), C.c_int(), C.c_int()
    _check(lib().pop_oracle_region_counts(C.c_int(m), C.c_double(f_ret), C.c_double(f_cand),
                                          C.byref(a), C.byref(b), C.byref(c)), "region_counts")
    return a.value, b.value, c.value


def k_for_ratio(m, r, n_ret, n_cand):
    return int(lib().pop_oracle_k_for_ratio(C.c_int(m), C.c_double(r), C.c_int(n_ret), C.c_int(n_cand)))


def hidden(x, w_gate, w_up, dtype, chan=None):
    x, w_gate, w_up = _storage(x, dtype), _storage(w_gate, dtype), _storage(w_up, dtype)
    T, d = x.shape
    m = w_gate.shape[0]
    assert w_gate.shape == (m, d) and w_up.shape == (m, d)
    H = np.zeros((T, m), dtype=np.float64)
    ch = None if chan is None else np.ascontiguousarray(chan, dtype=np.int32)
    _check(lib().pop_oracle_hidden(_p(x), _p(w_gate), _p(w_up), C.c_int(dtype), C.c_int(T), C.c_int(d),
                                   C.c_int(m), _p(ch), C.c_int(0 if ch is None else len(ch)), _p(H)),
           "hidden")
    return H


def importance(w_down, dtype, H, chan=None):
    w_down = _storage(w_down, dtype)
    d, m = w_down.shape
    H = np.ascontiguousarray(H, dtype=np.float64)
    T = H.shape[0]
    assert H.shape == (T, m)
    I = np.zeros(m, dtype=np.float64)
    ch = None if chan is None else np.ascontiguousarray(chan, dtype=np.int32)
    _check(lib().pop_oracle_importance(_p(w_down), C.c_int(dtype), C.c_int(d), C.c_int(m), _p(H), C.c_int(T),
                                       _p(ch), C.c_int(0 if ch is None else len(ch)), _p(I)), "importance")
    return I


def importance_input_side(x, w_gate, w_up, dtype, chan=None):
    """Importance under the input-side reading of Eq. 1-2: I_j = || [W_gate[j,:], W_up[j,:]] * s ||_2 with
    s_k = ||X[:,k]||_2 over the T rows of x."""
    x, w_gate, w_up = _storage(x, dtype), _storage(w_gate, dtype), _storage(w_up, dtype)
    T, d = x.shape
    m = w_gate.shape[0]
    assert w_gate.shape == (m, d) and w_up.shape == (m, d)
    I = np.zeros(m, dtype=np.float64)
    ch = None if chan is None else np.ascontiguousarray(chan, dtype=np.int32)
    _check(lib().pop_oracle_importance_input_side(_p(x), _p(w_gate), _p(w_up), C.c_int(dtype), C.c_int(T),
                                                  C.c_int(d), C.c_int(m), _p(ch), C.c_int(0 if ch is None else len(ch)),
                                                  _p(I)), "importance_input_side")
    return I


def down_norms(w_down, dtype):
    w_down = _storage(w_down, dtype)
    d, m = w_down.shape
    n = np.zeros(m, dtype=np.float64)
    _check(lib().pop_oracle_down_norms(_p(w_down), C.c_int(dtype), C.c_int(d), C.c_int(m), _p(n)), "down_norms")
    return n


def partition(scores, n_ret, n_cand):
    """scores: float32 or float64 [m] (float32 is widened exactly).  Returns region, ret_idx, cand_idx."""
    s = np.ascontiguousarray(scores).astype(np.float64)
    m = len(s)
    region = np.zeros(m, dtype=np.uint8)
    ret = np.zeros(n_ret, dtype=np.int32)
    cand = np.zeros(n_cand, dtype=np.int32)
    _check(lib().pop_oracle_partition(_p(s), C.c_int(m), C.c_int(n_ret), C.c_int(n_cand),
                                      _p(region), _p(ret), _p(cand)), "partition")
    return region, ret, cand


def select(region, cscore, cand_idx, k):
    """Returns mask[m], sel_idx[k], active_idx[n_ret+k]."""
    region = np.ascontiguousarray(region, dtype=np.uint8)
    m = len(region)
    cs = np.ascontiguousarray(cscore).astype(np.float64)
    cand_idx = np.ascontiguousarray(cand_idx, dtype=np.int32)
    n_cand = len(cand_idx)
    assert len(cs) == n_cand
    n_ret = int((region == 0).sum())
    mask = np.zeros(m, dtype=np.uint8)
    sel = np.zeros(k, dtype=np.int32)
    act = np.zeros(n_ret + k, dtype=np.int32)
    na = C.c_int()
    _check(lib().pop_oracle_select(_p(region), C.c_int(m), _p(cs), _p(cand_idx), C.c_int(n_cand), C.c_int(k),
                                   _p(mask), _p(sel), _p(act), C.byref(na)), "select")
    assert na.value == n_ret + k
    return mask, sel, act


def down(H, w_down, dtype, mask):
    w_down = _storage(w_down, dtype)
    d, m = w_down.shape
    H = np.ascontiguousarray(H, dtype=np.float64)
    T = H.shape[0]
    mask = np.ascontiguousarray(mask, dtype=np.uint8).reshape(-1, m)
    y = np.zeros((T, d), dtype=np.float64)
    _check(lib().pop_oracle_down(_p(H), _p(w_down), C.c_int(dtype), C.c_int(T), C.c_int(d), C.c_int(m),
                                 _p(mask), C.c_int(mask.shape[0]), _p(y)), "down")
    return y


def pruned_ffn(x, w_gate, w_up, w_down, dtype, mask):
    x, w_gate, w_up, w_down = (_storage(a, dtype) for a in (x, w_gate, w_up, w_down))
    T, d = x.shape
    m = w_gate.shape[0]
    mask = np.ascontiguousarray(mask, dtype=np.uint8).reshape(-1, m)
    y = np.zeros((T, d), dtype=np.float64)
    _check(lib().pop_oracle_pruned_ffn(_p(x), _p(w_gate), _p(w_up), _p(w_down), C.c_int(dtype), C.c_int(T),
                                       C.c_int(d), C.c_int(m), _p(mask), C.c_int(mask.shape[0]), _p(y)),
           "pruned_ffn")
    return y


def prefill(x, w_gate, w_up, w_down, dtype, n_ret, n_cand):
    """Returns scores[m] (float64), region[m], ret_idx, cand_idx."""
    x, w_gate, w_up, w_down = (_storage(a, dtype) for a in (x, w_gate, w_up, w_down))
    T, d = x.shape
    m = w_gate.shape[0]
    scores = np.zeros(m, dtype=np.float64)
    region = np.zeros(m, dtype=np.uint8)
    ret = np.zeros(n_ret, dtype=np.int32)
    cand = np.zeros(n_cand, dtype=np.int32)
    _check(lib().pop_oracle_prefill(_p(x), _p(w_gate), _p(w_up), _p(w_down), C.c_int(dtype), C.c_int(T),
                                    C.c_int(d), C.c_int(m), C.c_int(n_ret), C.c_int(n_cand),
                                    _p(scores), _p(region), _p(ret), _p(cand)), "prefill")
    return scores, region, ret, cand


def decode(x_t, w_gate, w_up, w_down, dtype, region, cand_idx, k, want_y=True):
    """One token.  Returns dict(h[m], cscore[n_cand], mask[m], sel_idx, active_idx, y[d])."""
    x_t = _storage(x_t, dtype).reshape(1, -1)
    w_gate, w_up, w_down = (_storage(a, dtype) for a in (w_gate, w_up, w_down))
    d = x_t.shape[1]
    m = w_gate.shape[0]
    region = np.ascontiguousarray(region, dtype=np.uint8)
    cand_idx = np.ascontiguousarray(cand_idx, dtype=np.int32)
    n_cand = len(cand_idx)
    n_ret = int((region == 0).sum())
    h = np.zeros(m, dtype=np.float64)
    cs = np.zeros(n_cand, dtype=np.float64)
    mask = np.zeros(m, dtype=np.uint8)
    sel = np.zeros(k, dtype=np.int32)
    act = np.zeros(n_ret + k, dtype=np.int32)
    na = C.c_int()
    y = np.zeros(d, dtype=np.float64) if want_y else None
    _check(lib().pop_oracle_decode(_p(x_t), _p(w_gate), _p(w_up), _p(w_down), C.c_int(dtype), C.c_int(d),
                                   C.c_int(m), _p(region), _p(cand_idx), C.c_int(n_cand), C.c_int(k),
                                   _p(h), _p(cs), _p(mask), _p(sel), _p(act), C.byref(na), _p(y)), "decode")
    return dict(h=h, cscore=cs, mask=mask, sel_idx=sel, active_idx=act, n_active=na.value, y=y)
