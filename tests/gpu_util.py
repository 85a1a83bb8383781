"""Helpers for the GPU parity tests: move seeded host arrays to the device and call the HIP path."""
import numpy as np
import torch

from paper_2602_06822_amd import synth


def dev(a: np.ndarray) -> torch.Tensor:
    """Host storage array -> device tensor holding the same bytes."""
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16).copy()).cuda()
    if a.dtype == np.uint8:
        return torch.from_numpy(a.copy()).cuda()
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t: torch.Tensor) -> np.ndarray:
    torch.cuda.synchronize()
    return t.cpu().numpy()


def bf16_out_to_f64(t: torch.Tensor) -> np.ndarray:
    """int16 tensor of bf16 bit patterns -> float64."""
    return synth.storage_to_f64(host(t).view(np.uint16), synth.BF16)


class GpuLayer:
    """A synthetic layer resident on the device plus its library handle."""

    def __init__(self, pop, layer: synth.Layer, max_tokens: int, max_batch: int = 1):
        self.pop = pop
        self.layer = layer
        cfg = layer.cfg
        self.d, self.m, self.dtype = cfg.d, cfg.m, cfg.dtype
        wg, wu, wd = dev(layer.w_gate), dev(layer.w_up), dev(layer.w_down)
        self.handle = pop.pop_layer_create(cfg.d, cfg.m, cfg.dtype, wg, wu, wd, max_tokens, max_batch)
        del wg, wu, wd
        self.n_ret = self.n_cand = None

    def close(self):
        if self.handle is not None:
            self.pop.pop_layer_destroy(self.handle)
            self.handle = None

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()

    def norms(self):
        n = torch.empty(self.m, dtype=torch.float32, device="cuda")
        self.pop.pop_layer_get_norms(self.handle, n)
        return host(n)

    def prefill(self, x: np.ndarray, n_ret: int, n_cand: int):
        T = x.shape[0]
        scores = torch.empty(self.m, dtype=torch.float32, device="cuda")
        region = torch.empty(self.m, dtype=torch.uint8, device="cuda")
        ret = torch.empty(max(n_ret, 1), dtype=torch.int32, device="cuda")
        cand = torch.empty(max(n_cand, 1), dtype=torch.int32, device="cuda")
        self.pop.pop_prefill_partition(self.handle, dev(x), T, n_ret, n_cand, scores, region, ret, cand)
        self.n_ret, self.n_cand = n_ret, n_cand
        return host(scores), host(region), host(ret)[:n_ret], host(cand)[:n_cand]

    def prefill_forward(self, x: np.ndarray, n_ret: int, n_cand: int, k0: int, ydtype=None):
        """pop_prefill_forward: returns (scores, region, ret_idx, cand_idx, mask, y as float64)."""
        T = x.shape[0]
        ydtype = self.dtype if ydtype is None else ydtype
        scores = torch.empty(self.m, dtype=torch.float32, device="cuda")
        region = torch.empty(self.m, dtype=torch.uint8, device="cuda")
        mask = torch.full((self.m,), 7, dtype=torch.uint8, device="cuda")
        ret = torch.empty(max(n_ret, 1), dtype=torch.int32, device="cuda")
        cand = torch.empty(max(n_cand, 1), dtype=torch.int32, device="cuda")
        y = torch.full((T, self.d), 12345, dtype=torch.float32 if ydtype == synth.F32 else torch.int16, device="cuda")
        self.pop.pop_prefill_forward(self.handle, dev(x), T, n_ret, n_cand, k0, y, ydtype, scores, region, ret, cand,
                                     mask)
        self.n_ret, self.n_cand = n_ret, n_cand
        yh = host(y).astype(np.float64) if ydtype == synth.F32 else bf16_out_to_f64(y)
        return host(scores), host(region), host(ret)[:n_ret], host(cand)[:n_cand], host(mask), yh

    def decode(self, x_t: np.ndarray, k, ydtype=None, one_call=False):
        """x_t: [B][d] storage.  Returns dict of host arrays (cscore, mask, active_idx, n_active, h, y).
        one_call: use pop_decode_step instead of pop_decode_mask + pop_pruned_ffn."""
        B = x_t.shape[0]
        ks = None if k is None else ([k] * B if isinstance(k, int) else list(k))  # None: the layer's strategy decides
        n_ret, n_cand, m, d = self.n_ret, self.n_cand, self.m, self.d
        cs = torch.empty((B, max(n_cand, 1)), dtype=torch.float32, device="cuda")
        mask = torch.empty((B, m), dtype=torch.uint8, device="cuda")
        act = torch.full((B, max(n_ret + n_cand, 1)), -1, dtype=torch.int32, device="cuda")
        na = torch.empty(B, dtype=torch.int32, device="cuda")
        ydtype = self.dtype if ydtype is None else ydtype
        y = torch.full((B, d), 12345, dtype=torch.float32 if ydtype == synth.F32 else torch.int16, device="cuda")
        if one_call:
            self.pop.pop_decode_step(self.handle, dev(x_t), B, ks, y, ydtype, cs if n_cand else None, mask,
                                     act if n_ret + n_cand else None, na)
        else:
            self.pop.pop_decode_mask(self.handle, dev(x_t), B, ks, cs if n_cand else None, mask,
                                     act if n_ret + n_cand else None, na)
            self.pop.pop_pruned_ffn(self.handle, None, B, None, 0, y, ydtype)
        h = torch.empty((B, m), dtype=torch.float32, device="cuda")
        self.pop.pop_layer_get_hidden(self.handle, h, B)
        yh = host(y).astype(np.float64) if ydtype == synth.F32 else bf16_out_to_f64(y)
        self.pop.pop_layer_sync_status(self.handle)  # raises if an in-kernel bounded wait expired
        return dict(cscore=host(cs)[:, :n_cand], mask=host(mask), active_idx=host(act), n_active=host(na),
                    h=host(h), y=yh)

    def ffn(self, x: np.ndarray, mask: np.ndarray, ydtype=None):
        T = x.shape[0]
        mask = np.ascontiguousarray(mask, dtype=np.uint8).reshape(-1, self.m)
        ydtype = self.dtype if ydtype is None else ydtype
        y = torch.empty((T, self.d), dtype=torch.float32 if ydtype == synth.F32 else torch.int16, device="cuda")
        self.pop.pop_pruned_ffn(self.handle, dev(x), T, dev(mask), mask.shape[0], y, ydtype)
        return host(y).astype(np.float64) if ydtype == synth.F32 else bf16_out_to_f64(y)


def score_rel_err(gpu: np.ndarray, ref: np.ndarray, eps: float = 1e-3) -> float:
    """max |gpu - ref| / max(|ref|, eps * max|ref|): relative error with a floor for near-zero scores."""
    ref = np.asarray(ref, dtype=np.float64)
    floor = eps * float(np.max(np.abs(ref))) if ref.size else 0.0
    den = np.maximum(np.abs(ref), floor if floor > 0 else 1.0)
    return float(np.max(np.abs(np.asarray(gpu, dtype=np.float64) - ref) / den)) if ref.size else 0.0


def max_abs_rel(y: np.ndarray, ref: np.ndarray) -> float:
    """max |y - ref| / max |ref|."""
    den = float(np.max(np.abs(ref)))
    return float(np.max(np.abs(y - ref)) / (den if den > 0 else 1.0))
