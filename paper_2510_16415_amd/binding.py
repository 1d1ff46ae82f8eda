"""ctypes binding of libmecefo.so: same names as the C ABI, argument marshalling only.

Tensors are torch CUDA tensors used as plain device buffers (torch is here for memory
and the stream handle); every arithmetic step runs inside the library's kernels.
There is no fallback: if the library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "lib", "libmecefo.so")

OK, ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_WORKSPACE_TOO_SMALL, ERR_LAUNCH = range(5)
F32, BF16 = 0, 1
SIDE_INPUT, SIDE_OUTPUT = 0, 1


class FfnDesc(C.Structure):
    _fields_ = [("tokens", C.c_int64), ("d_model", C.c_int32), ("d_ff", C.c_int32),
                ("ld_act_d", C.c_int64), ("ld_act_f", C.c_int64),
                ("ld_w_fd", C.c_int64), ("ld_w_df", C.c_int64),
                ("dtype", C.c_int), ("grad_dtype", C.c_int), ("rms_eps", C.c_float)]


class Proj(C.Structure):
    _fields_ = [("P", C.c_void_p), ("r", C.c_int32), ("ld", C.c_int64)]


class AttnDesc(C.Structure):
    _fields_ = [("batch", C.c_int32), ("seq", C.c_int32), ("heads", C.c_int32),
                ("rope_theta", C.c_float), ("ld_w_dd", C.c_int64)]


_BLOCK_IN = ["X", "H", "dOut", "g_attn", "g_ffn", "Wq", "Wk", "Wv", "Wo", "Wg", "Wu", "Wd", "Q", "K", "V", "O", "L"]
_BLOCK_OUT = ["dX", "dg_attn", "dg_ffn", "dWq", "dWk", "dWv", "dWo", "dWg", "dWu", "dWd"]


class BlockInputs(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in _BLOCK_IN]


class BlockGrads(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in _BLOCK_OUT]


_FWD_IN = ["X", "g_attn", "g_ffn", "Wq", "Wk", "Wv", "Wo", "Wg", "Wu", "Wd"]
_FWD_OUT = ["Out", "H", "Q", "K", "V", "O", "L"]


class BlockFwdInputs(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in _FWD_IN]


class BlockFwdOutputs(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in _FWD_OUT]


_LAYER_W = ["g_attn", "g_ffn", "Wq", "Wk", "Wv", "Wo", "Wg", "Wu", "Wd"]


class LayerWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in _LAYER_W]


class LayerLowrank(C.Structure):
    _fields_ = [("Pg", Proj), ("Pu", Proj), ("Pd", Proj), ("dg_ffn", C.c_void_p), ("dWg", C.c_void_p),
                ("dWu", C.c_void_p), ("dWd", C.c_void_p)]


class RefreshPolicy(C.Structure):
    _fields_ = [("tau", C.c_int64), ("power_iters", C.c_int32), ("cond_steps", C.c_int32), ("polish_steps", C.c_int32)]


MODE_STANDARD, MODE_NEIGHBOR = 0, 1


class SkipOptions(C.Structure):
    _fields_ = [("G", C.c_void_p), ("Z", C.c_void_p), ("exact_wgrad_mask", C.c_int32)]


class MecefoError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"mecefo status {status}: {message}")
        self.status = status


_lib = None
_vp = C.c_void_p


def lib() -> C.CDLL:
    """Loads the library (once).  Raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} not found: run `python -m paper_2510_16415_amd.build` first")
    L = C.CDLL(LIB_PATH)
    D = C.POINTER(FfnDesc)
    L.mecefo_last_error.restype = C.c_char_p
    L.mecefo_version.restype = C.c_char_p
    L.mecefo_workspace_bytes.argtypes = [D, C.c_int, C.c_int, C.c_int, C.POINTER(C.c_size_t)]
    L.mecefo_ffn_fwd_recompute.argtypes = [D] + [_vp] * 8 + [_vp, C.c_size_t, _vp]
    L.mecefo_ffn_bwd_exact.argtypes = [D] + [_vp] * 7 + [_vp] * 4 + [C.c_int, _vp, C.c_size_t, _vp]
    L.mecefo_ffn_bwd_lowrank.argtypes = ([D] + [_vp] * 5 + [Proj] * 3 + [C.c_int] + [_vp] * 4 +
                                         [C.c_int, _vp, C.c_size_t, _vp])
    L.mecefo_block_bwd_skip.argtypes = ([D] + [_vp] * 6 + [Proj] * 3 + [C.c_int] + [_vp] * 5 +
                                        [C.c_int, _vp, C.c_size_t, _vp])
    L.mecefo_block_bwd_skip_noalloc.argtypes = ([D] + [_vp] * 6 + [Proj] * 3 + [C.c_int] + [_vp] * 5 + [C.c_int, _vp])
    L.mecefo_block_bwd_skip_noalloc.restype = C.c_int
    L.mecefo_block_bwd_skip_ex.argtypes = ([D] + [_vp] * 6 + [Proj] * 3 + [C.c_int, C.POINTER(SkipOptions)] + [_vp] * 5 +
                                           [C.c_int, _vp, C.c_size_t, _vp])
    L.mecefo_block_full_workspace_bytes.argtypes = [D, C.POINTER(AttnDesc), C.POINTER(C.c_size_t)]
    L.mecefo_block_bwd_full.argtypes = [D, C.POINTER(AttnDesc), C.POINTER(BlockInputs), C.POINTER(BlockGrads),
                                        C.c_int, _vp, C.c_size_t, _vp]
    L.mecefo_block_fwd_workspace_bytes.argtypes = [D, C.POINTER(AttnDesc), C.POINTER(C.c_size_t)]
    L.mecefo_block_fwd.argtypes = [D, C.POINTER(AttnDesc), C.POINTER(BlockFwdInputs), C.POINTER(BlockFwdOutputs),
                                   _vp, C.c_size_t, _vp]
    L.mecefo_stack_workspace_bytes.argtypes = [D, C.POINTER(AttnDesc), C.c_int, C.c_int, C.c_int, C.POINTER(C.c_size_t)]
    L.mecefo_stack_fwd_neighbor.argtypes = [D, C.POINTER(AttnDesc), C.c_int, C.POINTER(LayerWeights), _vp,
                                            C.POINTER(C.c_void_p), _vp, _vp, C.c_size_t, _vp]
    L.mecefo_stack_bwd_skip.argtypes = [D, C.c_int, C.POINTER(LayerWeights), C.POINTER(C.c_void_p),
                                        C.POINTER(LayerLowrank), C.c_int, _vp, _vp, C.c_int, _vp, C.c_size_t, _vp]
    L.mecefo_grad_average.argtypes = [C.c_int, C.POINTER(C.c_void_p), C.POINTER(C.c_int32), C.c_int, _vp, C.c_int64, _vp]
    L.mecefo_adamw_step.argtypes = [C.c_int, C.c_int, _vp, _vp, _vp, _vp, C.c_int64, C.c_int64] + [C.c_float] * 5 + [_vp]
    L.mecefo_projection_workspace_bytes.argtypes = [C.c_int] * 5 + [C.POINTER(C.c_size_t)]
    L.mecefo_projection_refresh.argtypes = [C.c_int, _vp, C.c_int, C.c_int, C.c_int64, C.c_int, _vp, C.c_int64,
                                            C.c_int, C.c_int, C.c_int, C.c_int, _vp, C.c_int64, _vp, C.c_size_t, _vp]
    L.mecefo_profile_enable.argtypes = [C.c_int]
    L.mecefo_profile_collect.argtypes = [C.POINTER(C.c_double), C.POINTER(C.c_int)]
    L.mecefo_profile_enable.restype = C.c_int
    L.mecefo_profile_collect.restype = C.c_int
    L.mecefo_refresh_due.argtypes = [C.c_int64, C.c_int64]
    L.mecefo_refresh_due.restype = C.c_int
    L.mecefo_counters_reset.argtypes = [C.POINTER(C.c_int64), C.c_int]
    L.mecefo_counters_reset.restype = None
    L.mecefo_stack_mixed_workspace_bytes.argtypes = [D, C.POINTER(AttnDesc), C.c_int, C.c_int, C.c_int, C.POINTER(C.c_size_t)]
    L.mecefo_stack_mixed_workspace_bytes.restype = C.c_int
    L.mecefo_stack_bwd_mixed.argtypes = [D, C.POINTER(AttnDesc), C.c_int, C.POINTER(C.c_int), C.POINTER(BlockInputs),
                                         C.POINTER(BlockGrads), C.POINTER(LayerLowrank), C.c_int,
                                         C.POINTER(RefreshPolicy), C.POINTER(C.c_int64), _vp, _vp, C.c_int, _vp,
                                         C.c_size_t, _vp]
    L.mecefo_stack_bwd_mixed.restype = C.c_int
    L.mecefo_profile_clock_mhz.argtypes = [C.POINTER(C.c_double)]
    L.mecefo_profile_clock_mhz.restype = C.c_int
    L.mecefo_init.argtypes = []
    L.mecefo_init.restype = C.c_int
    L.mecefo_set_option.argtypes = [C.c_char_p, C.c_char_p]
    L.mecefo_set_option.restype = C.c_int
    for f in ("mecefo_workspace_bytes", "mecefo_ffn_fwd_recompute", "mecefo_ffn_bwd_exact",
              "mecefo_ffn_bwd_lowrank", "mecefo_block_bwd_skip", "mecefo_block_full_workspace_bytes",
              "mecefo_block_bwd_full", "mecefo_projection_workspace_bytes", "mecefo_projection_refresh",
              "mecefo_block_fwd_workspace_bytes", "mecefo_block_fwd", "mecefo_grad_average", "mecefo_adamw_step",
              "mecefo_stack_workspace_bytes", "mecefo_stack_fwd_neighbor", "mecefo_stack_bwd_skip",
              "mecefo_block_bwd_skip_ex"):
        getattr(L, f).restype = C.c_int
    _lib = L
    return L


def _check(st: int):
    if st != OK:
        raise MecefoError(st, lib().mecefo_last_error().decode())


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is not None:
        return C.c_void_p(stream if isinstance(stream, int) else stream.cuda_stream)
    import torch
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def make_desc(tokens, d_model, d_ff, dtype, grad_dtype=F32, ld_act_d=None, ld_act_f=None,
              ld_w_fd=None, ld_w_df=None, rms_eps=1e-6) -> FfnDesc:
    return FfnDesc(tokens, d_model, d_ff, ld_act_d or d_model, ld_act_f or d_ff,
                   ld_w_fd or d_model, ld_w_df or d_ff, dtype, grad_dtype, rms_eps)


def proj(P, r=None, ld=None) -> Proj:
    """Projection argument from a 2-D row-major tensor [dim x >=r].  The struct holds a raw device pointer;
    it also keeps a reference to the tensor, so that the memory cannot go back to the allocator while the
    argument is alive."""
    pr = Proj(P.data_ptr(), int(r if r is not None else P.shape[1]), int(ld if ld is not None else P.stride(0)))
    pr._tensor = P
    return pr


def mecefo_workspace_bytes(desc: FfnDesc, r_gate=0, r_up=0, r_down=0) -> int:
    out = C.c_size_t(0)
    _check(lib().mecefo_workspace_bytes(C.byref(desc), r_gate, r_up, r_down, C.byref(out)))
    return out.value


def _ws(ws):
    return (None, 0) if ws is None else (C.c_void_p(ws.data_ptr()), ws.numel() * ws.element_size())


def mecefo_ffn_fwd_recompute(desc, U, Wg, Wu, Wd, G, Z, A, Y, ws=None, stream=None):
    p, n = _ws(ws)
    _check(lib().mecefo_ffn_fwd_recompute(C.byref(desc), _ptr(U), _ptr(Wg), _ptr(Wu), _ptr(Wd), _ptr(G),
                                          _ptr(Z), _ptr(A), _ptr(Y), p, n, _stream(stream)))


def mecefo_ffn_bwd_exact(desc, U, dY, Wg, Wu, Wd, G, Z, dU, dWg, dWu, dWd, accumulate, ws, stream=None):
    p, n = _ws(ws)
    _check(lib().mecefo_ffn_bwd_exact(C.byref(desc), _ptr(U), _ptr(dY), _ptr(Wg), _ptr(Wu), _ptr(Wd), _ptr(G),
                                      _ptr(Z), _ptr(dU), _ptr(dWg), _ptr(dWu), _ptr(dWd), int(accumulate),
                                      p, n, _stream(stream)))


def mecefo_ffn_bwd_lowrank(desc, U, dY, Wg, Wu, Wd, Pg, Pu, Pd, side, dU, dWg, dWu, dWd, accumulate, ws,
                           stream=None):
    p, n = _ws(ws)
    _check(lib().mecefo_ffn_bwd_lowrank(C.byref(desc), _ptr(U), _ptr(dY), _ptr(Wg), _ptr(Wu), _ptr(Wd),
                                        Pg, Pu, Pd, int(side), _ptr(dU), _ptr(dWg), _ptr(dWu), _ptr(dWd),
                                        int(accumulate), p, n, _stream(stream)))


def mecefo_block_bwd_skip(desc, H, dOut, gamma, Wg, Wu, Wd, Pg, Pu, Pd, side, dX, dgamma, dWg, dWu, dWd,
                          accumulate, ws, stream=None):
    p, n = _ws(ws)
    _check(lib().mecefo_block_bwd_skip(C.byref(desc), _ptr(H), _ptr(dOut), _ptr(gamma), _ptr(Wg), _ptr(Wu),
                                       _ptr(Wd), Pg, Pu, Pd, int(side), _ptr(dX), _ptr(dgamma), _ptr(dWg),
                                       _ptr(dWu), _ptr(dWd), int(accumulate), p, n, _stream(stream)))


NOALLOC_SCRATCH_BYTES = 64 << 20


def mecefo_block_bwd_skip_noalloc(desc, H, dOut, gamma, Wg, Wu, Wd, Pg, Pu, Pd, side, dX, dgamma, dWg, dWu, dWd,
                                  accumulate, stream=None):
    _check(lib().mecefo_block_bwd_skip_noalloc(C.byref(desc), _ptr(H), _ptr(dOut), _ptr(gamma), _ptr(Wg), _ptr(Wu),
                                               _ptr(Wd), Pg, Pu, Pd, int(side), _ptr(dX), _ptr(dgamma), _ptr(dWg),
                                               _ptr(dWu), _ptr(dWd), int(accumulate), _stream(stream)))


def mecefo_block_bwd_skip_ex(desc, H, dOut, gamma, Wg, Wu, Wd, Pg, Pu, Pd, side, dX, dgamma, dWg, dWu, dWd,
                             accumulate, ws, G=None, Z=None, exact_wgrad_mask=0, stream=None):
    p, n = _ws(ws)
    opt = SkipOptions(None if G is None else G.data_ptr(), None if Z is None else Z.data_ptr(), exact_wgrad_mask)
    null = Proj(None, 0, 0)
    _check(lib().mecefo_block_bwd_skip_ex(C.byref(desc), _ptr(H), _ptr(dOut), _ptr(gamma), _ptr(Wg), _ptr(Wu),
                                          _ptr(Wd), Pg or null, Pu or null, Pd or null, int(side), C.byref(opt),
                                          _ptr(dX), _ptr(dgamma), _ptr(dWg), _ptr(dWu), _ptr(dWd), int(accumulate),
                                          p, n, _stream(stream)))


def make_attn_desc(batch, seq, heads, ld_w_dd, rope_theta=10000.0) -> AttnDesc:
    return AttnDesc(batch, seq, heads, rope_theta, ld_w_dd)


def mecefo_block_full_workspace_bytes(desc: FfnDesc, attn: AttnDesc) -> int:
    out = C.c_size_t(0)
    _check(lib().mecefo_block_full_workspace_bytes(C.byref(desc), C.byref(attn), C.byref(out)))
    return out.value


def mecefo_block_bwd_full(desc, attn, inputs: dict, grads: dict, accumulate, ws, stream=None):
    """inputs / grads: tensors by the field names of mecefo_block_inputs_t / mecefo_block_grads_t."""
    def table(cls, names, d):
        unknown = set(d) - set(names)
        if unknown:
            raise KeyError(f"unknown fields {sorted(unknown)}")
        return cls(*[None if d.get(n) is None else d[n].data_ptr() for n in names])
    p, n = _ws(ws)
    tin, tout = table(BlockInputs, _BLOCK_IN, inputs), table(BlockGrads, _BLOCK_OUT, grads)
    _check(lib().mecefo_block_bwd_full(C.byref(desc), C.byref(attn), C.byref(tin), C.byref(tout),
                                       int(accumulate), p, n, _stream(stream)))


def _table(cls, names, d):
    unknown = set(d) - set(names)
    if unknown:
        raise KeyError(f"unknown fields {sorted(unknown)}")
    return cls(*[None if d.get(n) is None else d[n].data_ptr() for n in names])


def mecefo_block_fwd_workspace_bytes(desc: FfnDesc, attn: AttnDesc) -> int:
    out = C.c_size_t(0)
    _check(lib().mecefo_block_fwd_workspace_bytes(C.byref(desc), C.byref(attn), C.byref(out)))
    return out.value


def mecefo_block_fwd(desc, attn, inputs: dict, outputs: dict, ws, stream=None):
    """inputs / outputs: tensors by the field names of mecefo_block_fwd_inputs_t / _outputs_t
    (omit Q, K, V, O, L for the neighbor-mode forward that keeps only H)."""
    p, n = _ws(ws)
    tin, tout = _table(BlockFwdInputs, _FWD_IN, inputs), _table(BlockFwdOutputs, _FWD_OUT, outputs)
    _check(lib().mecefo_block_fwd(C.byref(desc), C.byref(attn), C.byref(tin), C.byref(tout), p, n, _stream(stream)))


def mecefo_stack_workspace_bytes(desc, attn, r_gate=0, r_up=0, r_down=0) -> int:
    out = C.c_size_t(0)
    _check(lib().mecefo_stack_workspace_bytes(C.byref(desc), C.byref(attn), r_gate, r_up, r_down, C.byref(out)))
    return out.value


def layer_weights(layers):
    """layers: list of dicts of tensors by the field names of mecefo_layer_weights_t."""
    return (LayerWeights * len(layers))(*[_table(LayerWeights, _LAYER_W, d) for d in layers])


def layer_lowrank(layers):
    """layers: list of dicts with Pg, Pu, Pd (Proj) and dg_ffn, dWg, dWu, dWd (tensors)."""
    arr = (LayerLowrank * len(layers))()
    for a, d in zip(arr, layers):
        a.Pg, a.Pu, a.Pd = d["Pg"], d["Pu"], d["Pd"]
        for k in ("dg_ffn", "dWg", "dWu", "dWd"):
            setattr(a, k, None if d.get(k) is None else d[k].data_ptr())
    return arr


def _ptr_array(tensors):
    return (C.c_void_p * len(tensors))(*[t.data_ptr() for t in tensors])


def mecefo_stack_fwd_neighbor(desc, attn, layers, X0, H, X_out, ws, stream=None):
    p, n = _ws(ws)
    _check(lib().mecefo_stack_fwd_neighbor(C.byref(desc), C.byref(attn), len(layers), layers, _ptr(X0),
                                           _ptr_array(H), _ptr(X_out), p, n, _stream(stream)))


def mecefo_stack_bwd_skip(desc, layers, H, lowrank, side, dOut_top, dX_bottom, accumulate, ws, stream=None):
    p, n = _ws(ws)
    _check(lib().mecefo_stack_bwd_skip(C.byref(desc), len(layers), layers, _ptr_array(H), lowrank, int(side),
                                       _ptr(dOut_top), _ptr(dX_bottom), int(accumulate), p, n, _stream(stream)))


def mecefo_refresh_due(t: int, tau: int) -> bool:
    return bool(lib().mecefo_refresh_due(int(t), int(tau)))


def mecefo_counters_reset(counters):
    """counters: ctypes array of int64 (the per-layer step counters of one rank), set to zero in place."""
    lib().mecefo_counters_reset(counters, len(counters))


def mecefo_stack_mixed_workspace_bytes(desc, attn, r_gate=0, r_up=0, r_down=0) -> int:
    out = C.c_size_t(0)
    _check(lib().mecefo_stack_mixed_workspace_bytes(C.byref(desc), C.byref(attn), r_gate, r_up, r_down, C.byref(out)))
    return out.value


def mecefo_stack_bwd_mixed(desc, attn, modes, inputs, grads, lowrank, side, policy, counters, dOut_top, dX_bottom,
                           accumulate, ws, stream=None):
    """modes: list of MODE_*; inputs / grads: lists of dicts by the field names of mecefo_block_inputs_t /
    mecefo_block_grads_t (a neighbor-mode layer needs H, g_ffn, Wg, Wu, Wd only); lowrank: layer_lowrank(...)
    or None; policy: RefreshPolicy or None; counters: ctypes int64 array (updated in place) or None."""
    n = len(modes)
    p, nbytes = _ws(ws)
    m = (C.c_int * n)(*[int(x) for x in modes])
    tin = (BlockInputs * n)(*[_table(BlockInputs, _BLOCK_IN, d) for d in inputs])
    tout = (BlockGrads * n)(*[_table(BlockGrads, _BLOCK_OUT, d) for d in grads])
    _check(lib().mecefo_stack_bwd_mixed(C.byref(desc), C.byref(attn), n, m, tin, tout, lowrank, int(side),
                                        C.byref(policy) if policy is not None else None, counters, _ptr(dOut_top),
                                        _ptr(dX_bottom), int(accumulate), p, nbytes, _stream(stream)))


def mecefo_grad_average(grad_dtype, grads, contributes, out, n_elems, stream=None):
    """grads: list of tensors (None allowed for ranks that do not contribute)."""
    n = len(grads)
    ptrs = (C.c_void_p * n)(*[None if g is None else g.data_ptr() for g in grads])
    mask = (C.c_int32 * n)(*[int(bool(c)) for c in contributes])
    _check(lib().mecefo_grad_average(grad_dtype, ptrs, mask, n, _ptr(out), n_elems, _stream(stream)))


def mecefo_adamw_step(w_dtype, grad_dtype, W, G, M, V, n_elems, step, lr, beta1=0.9, beta2=0.999, eps=1e-8,
                      weight_decay=0.01, stream=None):
    _check(lib().mecefo_adamw_step(w_dtype, grad_dtype, _ptr(W), _ptr(G), _ptr(M), _ptr(V), n_elems, step, lr,
                                   beta1, beta2, eps, weight_decay, _stream(stream)))


def mecefo_projection_workspace_bytes(dtype, m, n, r, left=0) -> int:
    out = C.c_size_t(0)
    _check(lib().mecefo_projection_workspace_bytes(dtype, m, n, r, int(left), C.byref(out)))
    return out.value


def mecefo_projection_refresh(dtype, W, m, n, ldw, left, V0, ldv, r, power_iters, cond_steps, polish_steps,
                              P, ldp, ws, stream=None):
    p, nb = _ws(ws)
    _check(lib().mecefo_projection_refresh(dtype, _ptr(W), m, n, ldw, int(left), _ptr(V0), ldv, r, power_iters,
                                           cond_steps, polish_steps, _ptr(P), ldp, p, nb, _stream(stream)))


STAGES = ["norm_fwd", "dgrad_down", "recompute", "swiglu_bwd", "dgrad_gate_up", "project", "contract",
          "splitk_reduce", "expand", "norm_bwd", "wgrad_exact", "attn_out_bwd", "attn_rowdot", "attn_probs",
          "attn_dv", "attn_ds", "attn_dq", "attn_dk", "rope_bwd", "qkv_wgrad", "qkv_dgrad", "attn_fused_kv"]


def mecefo_profile_enable(max_stage_launches: int):
    _check(lib().mecefo_profile_enable(int(max_stage_launches)))


def mecefo_profile_collect():
    """Returns {stage name: (total milliseconds, launches)} for stages that ran."""
    n = len(STAGES)
    ms = (C.c_double * n)()
    cnt = (C.c_int * n)()
    _check(lib().mecefo_profile_collect(ms, cnt))
    return {STAGES[i]: (ms[i], cnt[i]) for i in range(n) if cnt[i]}


def mecefo_profile_clock_mhz():
    """After mecefo_profile_collect: {stage name: average shader clock in MHz} of the sampled GEMM launches."""
    n = len(STAGES)
    mhz = (C.c_double * n)()
    _check(lib().mecefo_profile_clock_mhz(mhz))
    return {STAGES[i]: mhz[i] for i in range(n) if mhz[i] > 0}


def mecefo_init():
    _check(lib().mecefo_init())


def mecefo_set_option(name: str, value: str):
    _check(lib().mecefo_set_option(name.encode(), value.encode()))


def mecefo_last_error() -> str:
    return lib().mecefo_last_error().decode()


def mecefo_version() -> str:
    return lib().mecefo_version().decode()
