"""Helpers for the GPU parity tests: host arrays -> device buffers -> C ABI -> host arrays."""
from __future__ import annotations

import numpy as np
import torch

from paper_2510_16415_amd import binding as B

TOL = {"bf16": 2e-2, "f32": 1e-5}   # relative Frobenius error gates (bf16 in / fp32 acc; fp32 path)


def relerr(a, b) -> float:
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    den = np.linalg.norm(b)
    return float(np.linalg.norm(a - b) / den) if den > 0 else float(np.linalg.norm(a - b))


def up8(x: int) -> int:
    return (x + 7) // 8 * 8


def tdtype(dtype: str):
    return torch.bfloat16 if dtype == "bf16" else torch.float32


def dev(x: np.ndarray, dtype: str, ld: int | None = None, fill: float = float("nan")) -> torch.Tensor:
    """Host [rows x cols] -> device [rows x ld]; padding columns are poisoned with `fill`."""
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32))
    if t.ndim == 2 and ld is not None and ld != t.shape[1]:
        full = torch.full((t.shape[0], ld), fill, dtype=torch.float32)
        full[:, : t.shape[1]] = t
        t = full
    return t.to(tdtype(dtype)).cuda()


def poisoned_ws(nbytes: int) -> torch.Tensor:
    """Workspace for a library call with every byte 0xFF (NaN as bf16 and as fp32, -1 as an integer): a
    kernel that reads workspace bytes no earlier kernel of the same call has written shows up as a
    non-finite output instead of depending on what the allocator handed out."""
    return torch.full((max(int(nbytes), 1),), 255, dtype=torch.uint8, device="cuda")


def host(t: torch.Tensor, cols: int | None = None) -> np.ndarray:
    a = t.detach().float().cpu().numpy()
    return a if cols is None else a[:, :cols]


class Layer:
    """Device-resident weights / projections of one layer plus a descriptor and workspace."""

    def __init__(self, b, d, f, dtype, Wg, Wu, Wd, gamma, Pg, Pu, Pd, eps=1e-6, grad_dtype="f32",
                 side=B.SIDE_INPUT, pad_act_d=0, pad_w=0):
        self.b, self.d, self.f, self.dtype, self.side = b, d, f, dtype, side
        self.grad_dtype = grad_dtype
        al = 8 if dtype == "bf16" else 1
        rnd = (lambda x: (x + al - 1) // al * al)
        self.ld_act_d = rnd(d) + pad_act_d
        self.ld_act_f = rnd(f) + pad_act_d
        self.ld_w_fd = rnd(d) + pad_w
        self.ld_w_df = rnd(f) + pad_w
        self.Wg, self.Wu = dev(Wg, dtype, self.ld_w_fd), dev(Wu, dtype, self.ld_w_fd)
        self.Wd = dev(Wd, dtype, self.ld_w_df)
        self.gamma = None if gamma is None else dev(gamma, dtype)
        self.P = []
        for P in (Pg, Pu, Pd):
            if P is None:
                self.P.append(None)
            else:
                self.P.append(dev(P, dtype, rnd(P.shape[1]) + pad_w))
        self.r = [0 if P is None else P.shape[1] for P in (Pg, Pu, Pd)]
        self.desc = B.make_desc(b, d, f, B.BF16 if dtype == "bf16" else B.F32,
                                B.F32 if grad_dtype == "f32" else (B.BF16 if dtype == "bf16" else B.F32),
                                self.ld_act_d, self.ld_act_f, self.ld_w_fd, self.ld_w_df, eps)
        nbytes = B.mecefo_workspace_bytes(self.desc, *self.r)
        self.ws = poisoned_ws(nbytes)
        gt = torch.float32 if grad_dtype == "f32" else tdtype(dtype)
        self.dWg = torch.full((f, self.ld_w_fd), float("nan"), dtype=gt, device="cuda")
        self.dWu = torch.full((f, self.ld_w_fd), float("nan"), dtype=gt, device="cuda")
        self.dWd = torch.full((d, self.ld_w_df), float("nan"), dtype=gt, device="cuda")
        self.dgamma = torch.full((d,), float("nan"), dtype=gt, device="cuda")

    def projs(self):
        return [B.proj(P, r) for P, r in zip(self.P, self.r)]

    def act(self, x, wide=False):
        return dev(x, self.dtype, self.ld_act_f if wide else self.ld_act_d)

    def block_bwd_skip(self, H, dOut, accumulate=0, alias=False, want_dgamma=True):
        Hd, dOd = self.act(H), self.act(dOut)
        dX = dOd if alias else torch.full_like(dOd, float("nan"))
        B.mecefo_block_bwd_skip(self.desc, Hd, dOd, self.gamma, self.Wg, self.Wu, self.Wd, *self.projs(),
                                self.side, dX, self.dgamma if (want_dgamma and self.gamma is not None) else None,
                                self.dWg, self.dWu, self.dWd, accumulate, self.ws)
        torch.cuda.synchronize()
        return self.results(dX)

    def results(self, dX=None):
        out = dict(dWg=host(self.dWg, self.d), dWu=host(self.dWu, self.d), dWd=host(self.dWd, self.f),
                   dgamma=host(self.dgamma))
        if dX is not None:
            out["dX"] = host(dX, self.d)
        return out


def local_relerr(got, want) -> dict:
    """Localised error measures: for a matrix the largest per-row and per-column L2 error, for a vector the
    largest error of a block of 32 consecutive elements, each relative to that piece's own norm or, for
    pieces that are small themselves, to the root-mean-square piece norm of the whole tensor.  One wrong
    row, column or edge tile shows up here at order one even where it would move the Frobenius ratio of a
    large matrix by less than the gate.  Pieces shorter than 32 elements are not measured on their own
    (a single rounding error would dominate them); the Frobenius gate covers such small tensors."""
    g = np.asarray(got, dtype=np.float64)
    w = np.asarray(want, dtype=np.float64)
    if w.ndim == 1:
        n = w.shape[0] // 32 * 32
        if n < 64:
            return {}
        g, w = g[:n].reshape(-1, 32), w[:n].reshape(-1, 32)
        axes = ((1, "block"),)
    else:
        axes = ((1, "row"), (0, "col"))
    out = {}
    diff = g - w
    for axis, name in axes:
        if w.shape[axis] < 32 or w.shape[1 - axis] < 2:
            continue
        dn = np.sqrt((diff * diff).sum(axis=axis))
        wn = np.sqrt((w * w).sum(axis=axis))
        rms = float(np.sqrt((wn * wn).mean()))
        den = np.maximum(wn, rms)
        out[name] = float((dn / den).max()) if rms > 0 else float(dn.max())
    return out


LOCAL_FACTOR = 3.0   # worst piece vs whole tensor, see assert_close


def assert_close(got: dict, want: dict, tol: float, keys=None, label="", local=True):
    """Gate per output tensor: relative Frobenius error <= tol (the stated tolerance).  On top of it a defect
    detector: the worst row and column of a matrix / the worst 32-element block of a vector (local_relerr)
    must stay below LOCAL_FACTOR * tol.  The factor is not a looser parity gate: the worst of thousands of
    short pieces lies above the average of all of them even when every element carries the same rounding
    noise (rows of 64 to 128 elements, rows with a small norm of their own), while a wrong or missing row,
    column or tile reads 0.1 to 1 on this measure, whatever the size of the tensor."""
    errs = {}
    loc = {}
    for k in keys or want.keys():
        if want.get(k) is None:
            continue
        g = got[k]
        assert np.all(np.isfinite(g)), f"{label}{k}: non-finite values in GPU result"
        errs[k] = relerr(g, want[k])
        if local:
            loc[k] = local_relerr(g, want[k])
    bad = {k: e for k, e in errs.items() if not e <= tol}
    assert not bad, f"{label}relative Frobenius error above {tol}: {bad} (all: {errs})"
    bad_loc = {k: e for k, e in loc.items() if any(not v <= LOCAL_FACTOR * tol for v in e.values())}
    assert not bad_loc, f"{label}worst row / column error above {LOCAL_FACTOR * tol}: {bad_loc} (Frobenius: {errs})"
    return errs
