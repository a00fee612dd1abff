"""Thin ctypes binding of libpbsa.so: argument marshalling only, same names as include/pbsa.h.

Tensor arguments are torch tensors living on the GPU (their data_ptr() is passed through) or plain
integers holding a device address.  Nothing is computed here and there is no fallback: if the HIP
library is missing the import of the library fails loudly.
"""
from __future__ import annotations

import ctypes
import os

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libpbsa.so")

PBSA_OK, PBSA_EINVAL, PBSA_ESHAPE, PBSA_EALIGN, PBSA_EWS, PBSA_EHIP = 0, -1, -2, -3, -4, -5
PBSA_MAX_N_LOC, PBSA_MAX_C, PBSA_MAX_C_ATTEND, PBSA_MAX_K = 672, 64, 336, 672
PBSA_MAX_N_LOC_AUX, PBSA_MAX_C_AUX, PBSA_MAX_K_AUX = 512, 192, 512
PBSA_STATIC_WS_BYTES = 4 << 20

EXPORTS = ("pbsa_workspace_bytes", "pbsa_pool_blocks", "pbsa_summary_view", "pbsa_select_blocks", "pbsa_attention_fwd",
           "pbsa_memory_update", "pbsa_memory_update_static", "pbsa_memory_update_plan", "pbsa_memory_update_apply", "pbsa_attention_fwd_plan",
           "pbsa_select_blocks_apply",
           "pbsa_attention_mass", "pbsa_mass_workspace_bytes", "pbsa_attention_fwd_mass",
           "pbsa_memory_update_fine", "pbsa_bwd_workspace_bytes", "pbsa_attention_bwd", "pbsa_blockify",
           "pbsa_unblockify", "pbsa_strerror", "pbsa_version")


class pbsa_params(ctypes.Structure):
    _fields_ = [("size", ctypes.c_uint32), ("H", ctypes.c_int32), ("d", ctypes.c_int32), ("B", ctypes.c_int32),
                ("Nq", ctypes.c_int32), ("nqb", ctypes.c_int32), ("n_loc", ctypes.c_int32),
                ("n_loc_cap", ctypes.c_int32), ("C", ctypes.c_int32), ("n_sink", ctypes.c_int32),
                ("k", ctypes.c_int32), ("causal", ctypes.c_int32), ("n_evict", ctypes.c_int32),
                ("pool_from", ctypes.c_int32), ("scale", ctypes.c_float),
                ("q_stride_h", ctypes.c_int64), ("q_stride_t", ctypes.c_int64),
                ("o_stride_h", ctypes.c_int64), ("o_stride_t", ctypes.c_int64)]


def make_params(H, d, B, Nq, n_loc, n_loc_cap, C, k, scale, n_sink=0, causal=1, n_evict=0, pool_from=0,
                q_strides=None, o_strides=None) -> pbsa_params:
    qs = q_strides or (Nq * d, d)
    os_ = o_strides or (Nq * d, d)
    return pbsa_params(ctypes.sizeof(pbsa_params), H, d, B, Nq, -(-Nq // B), n_loc, n_loc_cap, C, n_sink, k, causal,
                       n_evict, pool_from, scale, qs[0], qs[1], os_[0], os_[1])


class pbsa_grid(ctypes.Structure):
    _fields_ = [("size", ctypes.c_uint32), ("T", ctypes.c_int32), ("Hs", ctypes.c_int32), ("Ws", ctypes.c_int32),
                ("Bt", ctypes.c_int32), ("Bh", ctypes.c_int32), ("Bw", ctypes.c_int32), ("H", ctypes.c_int32),
                ("d", ctypes.c_int32), ("B", ctypes.c_int32)]


def make_grid(T, Hs, Ws, Bt, Bh, Bw, H, d, B) -> pbsa_grid:
    return pbsa_grid(ctypes.sizeof(pbsa_grid), T, Hs, Ws, Bt, Bh, Bw, H, d, B)


class PbsaError(RuntimeError):
    def __init__(self, code: int):
        self.code = code
        super().__init__(f"pbsa error {code}: {pbsa_strerror(code)}")


_lib = None


def lib() -> ctypes.CDLL:
    """Load libpbsa.so (built in-tree by paper_2604_21221_amd/build.py).  No fallback."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2604_21221_amd.build` "
                              "(there is no CPU fallback)")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
        pp = ctypes.POINTER(pbsa_params)
        L.pbsa_version.restype = ctypes.c_int
        L.pbsa_version.argtypes = []
        L.pbsa_strerror.restype = ctypes.c_char_p
        L.pbsa_strerror.argtypes = [ctypes.c_int]
        L.pbsa_workspace_bytes.argtypes = [pp, ctypes.POINTER(sz)]
        L.pbsa_pool_blocks.argtypes = [pp, vp, vp, i32, vp, vp]
        L.pbsa_summary_view.argtypes = [pp] + [vp] * 6
        L.pbsa_select_blocks.argtypes = [pp] + [vp] * 9 + [sz, vp]
        L.pbsa_attention_fwd.argtypes = [pp] + [vp] * 12 + [sz, vp]
        L.pbsa_memory_update.argtypes = [pp] + [vp] * 18 + [sz, vp]
        L.pbsa_memory_update_static.argtypes = [pp] + [vp] * 18
        L.pbsa_memory_update_plan.argtypes = [pp] + [vp] * 13 + [sz, vp]
        L.pbsa_memory_update_apply.argtypes = [pp] + [vp] * 8 + [sz, vp]
        L.pbsa_attention_fwd_plan.argtypes = [pp] + [vp] * 21 + [sz, vp]
        L.pbsa_select_blocks_apply.argtypes = [pp] + [vp] * 8 + [pp] + [vp] * 7 + [sz, vp]
        L.pbsa_attention_mass.argtypes = [pp] + [vp] * 10
        L.pbsa_mass_workspace_bytes.argtypes = [pp, ctypes.POINTER(sz)]
        L.pbsa_attention_fwd_mass.argtypes = [pp] + [vp] * 13 + [sz, vp]
        L.pbsa_memory_update_fine.argtypes = [pp] + [vp] * 17 + [sz, vp]
        L.pbsa_bwd_workspace_bytes.argtypes = [pp, ctypes.POINTER(sz)]
        L.pbsa_attention_bwd.argtypes = [pp] + [vp] * 18 + [sz, vp]
        pg = ctypes.POINTER(pbsa_grid)
        L.pbsa_blockify.argtypes = [pg, i32, ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.POINTER(ctypes.c_int64), vp]
        L.pbsa_unblockify.argtypes = [pg, vp, ctypes.c_int64, vp, vp]
        for name in ("pbsa_workspace_bytes", "pbsa_pool_blocks", "pbsa_summary_view", "pbsa_select_blocks", "pbsa_attention_fwd",
                     "pbsa_memory_update", "pbsa_memory_update_static", "pbsa_memory_update_plan", "pbsa_memory_update_apply",
                     "pbsa_attention_fwd_plan", "pbsa_select_blocks_apply", "pbsa_attention_mass", "pbsa_mass_workspace_bytes",
                     "pbsa_attention_fwd_mass", "pbsa_memory_update_fine", "pbsa_bwd_workspace_bytes",
                     "pbsa_attention_bwd", "pbsa_blockify", "pbsa_unblockify"):
            getattr(L, name).restype = ctypes.c_int
        _lib = L
    return _lib


def _ptr(x):
    """Device address of a tensor (must be on the GPU), or an int / None passed through."""
    if x is None:
        return None
    if isinstance(x, int):
        return ctypes.c_void_p(x)
    if not x.is_cuda:
        raise TypeError("pbsa: tensor arguments must live on the GPU")
    if not x.is_contiguous() and x.dim() < 3:
        raise TypeError("pbsa: small tensors must be contiguous")
    return ctypes.c_void_p(x.data_ptr())


def _stream(stream):
    if stream is None:
        import torch
        return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    if isinstance(stream, int):
        return ctypes.c_void_p(stream)
    return ctypes.c_void_p(stream.cuda_stream)


def _ws(ws):
    if ws is None:
        return None, 0
    if isinstance(ws, tuple):
        return ctypes.c_void_p(ws[0]), ws[1]
    return ctypes.c_void_p(ws.data_ptr()), ws.numel() * ws.element_size()


def _check(rc: int):
    if rc != PBSA_OK:
        raise PbsaError(rc)


def pbsa_version() -> int:
    return lib().pbsa_version()


def pbsa_strerror(code: int) -> str:
    return lib().pbsa_strerror(code).decode()


def pbsa_workspace_bytes(p: pbsa_params) -> int:
    out = ctypes.c_size_t(0)
    _check(lib().pbsa_workspace_bytes(ctypes.byref(p), ctypes.byref(out)))
    return out.value


def pbsa_pool_blocks(p, X, length, n_blocks, out, stream=None):
    _check(lib().pbsa_pool_blocks(ctypes.byref(p), _ptr(X), _ptr(length), n_blocks, _ptr(out), _stream(stream)))


def pbsa_summary_view(p, S_sum, S_cnt, Kp, Vp, p_len, stream=None):
    _check(lib().pbsa_summary_view(ctypes.byref(p), _ptr(S_sum), _ptr(S_cnt), _ptr(Kp), _ptr(Vp), _ptr(p_len), _stream(stream)))


def pbsa_select_blocks(p, Q, Kl, l_len, l_map, Kc_l, Qc, sel, Zl=None, ws=None, stream=None):
    w, wb = _ws(ws)
    _check(lib().pbsa_select_blocks(ctypes.byref(p), _ptr(Q), _ptr(Kl), _ptr(l_len), _ptr(l_map), _ptr(Kc_l),
                                    _ptr(Qc), _ptr(sel), _ptr(Zl), w, wb, _stream(stream)))


def pbsa_select_blocks_apply(p, Q, Kl, l_len, l_map, Kc_l, Qc, sel, Zl, p_upd, Kp, Vp, p_len, S_sum, S_cnt, Vl, ws,
                             stream=None):
    w, wb = _ws(ws)
    _check(lib().pbsa_select_blocks_apply(ctypes.byref(p), _ptr(Q), _ptr(Kl), _ptr(l_len), _ptr(l_map), _ptr(Kc_l),
                                          _ptr(Qc), _ptr(sel), _ptr(Zl), ctypes.byref(p_upd), _ptr(Kp), _ptr(Vp),
                                          _ptr(p_len), _ptr(S_sum), _ptr(S_cnt), _ptr(Vl), w, wb, _stream(stream)))


def pbsa_attention_fwd(p, Q, Kp, Vp, p_len, Kl, Vl, l_len, l_map, sel, O, lse=None, ws=None, stream=None):
    w, wb = _ws(ws)
    _check(lib().pbsa_attention_fwd(ctypes.byref(p), _ptr(Q), _ptr(Kp), _ptr(Vp), _ptr(p_len), _ptr(Kl), _ptr(Vl),
                                    _ptr(l_len), _ptr(l_map), _ptr(sel), _ptr(O), _ptr(lse), w, wb, _stream(stream)))


def pbsa_memory_update(p, Qc, Kc_l, Zl, Kp, Vp, Kc_p, p_len, p_id, S_sum, S_cnt, Kl, Vl, l_len, l_map, l_id, scores,
                       slot_src, ws, stream=None):
    w, wb = _ws(ws)
    _check(lib().pbsa_memory_update(ctypes.byref(p), _ptr(Qc), _ptr(Kc_l), _ptr(Zl), _ptr(Kp), _ptr(Vp), _ptr(Kc_p),
                                    _ptr(p_len), _ptr(p_id), _ptr(S_sum), _ptr(S_cnt), _ptr(Kl), _ptr(Vl),
                                    _ptr(l_len), _ptr(l_map), _ptr(l_id), _ptr(scores), _ptr(slot_src), w, wb,
                                    _stream(stream)))


def pbsa_memory_update_static(p, Qc, Kc_l, Zl, Kp, Vp, Kc_p, p_len, p_id, S_sum, S_cnt, Kl, Vl, l_len, l_map, l_id, scores,
                              slot_src, stream=None):
    _check(lib().pbsa_memory_update_static(ctypes.byref(p), _ptr(Qc), _ptr(Kc_l), _ptr(Zl), _ptr(Kp), _ptr(Vp),
                                           _ptr(Kc_p), _ptr(p_len), _ptr(p_id), _ptr(S_sum), _ptr(S_cnt), _ptr(Kl),
                                           _ptr(Vl), _ptr(l_len), _ptr(l_map), _ptr(l_id), _ptr(scores),
                                           _ptr(slot_src), _stream(stream)))


def pbsa_memory_update_plan(p, Qc, Kc_l, Zl, Kc_p, p_len, p_id, S_cnt, l_len, l_map, l_id, scores, slot_src, ws,
                            stream=None):
    w, wb = _ws(ws)
    _check(lib().pbsa_memory_update_plan(ctypes.byref(p), _ptr(Qc), _ptr(Kc_l), _ptr(Zl), _ptr(Kc_p), _ptr(p_len),
                                         _ptr(p_id), _ptr(S_cnt), _ptr(l_len), _ptr(l_map), _ptr(l_id), _ptr(scores),
                                         _ptr(slot_src), w, wb, _stream(stream)))


def pbsa_attention_fwd_plan(p, Q, Kp, Vp, p_len, Kl, Vl, l_len, l_map, sel, O, lse, Qc, Kc_l, Zl, Kc_p, p_id, S_cnt, l_id,
                            scores, slot_src, ws, stream=None):
    w, wb = _ws(ws)
    _check(lib().pbsa_attention_fwd_plan(ctypes.byref(p), _ptr(Q), _ptr(Kp), _ptr(Vp), _ptr(p_len), _ptr(Kl), _ptr(Vl),
                                         _ptr(l_len), _ptr(l_map), _ptr(sel), _ptr(O), _ptr(lse), _ptr(Qc), _ptr(Kc_l),
                                         _ptr(Zl), _ptr(Kc_p), _ptr(p_id), _ptr(S_cnt), _ptr(l_id), _ptr(scores),
                                         _ptr(slot_src), w, wb, _stream(stream)))


def pbsa_memory_update_apply(p, Kp, Vp, p_len, S_sum, S_cnt, Kl, Vl, ws, stream=None):
    w, wb = _ws(ws)
    _check(lib().pbsa_memory_update_apply(ctypes.byref(p), _ptr(Kp), _ptr(Vp), _ptr(p_len), _ptr(S_sum), _ptr(S_cnt),
                                          _ptr(Kl), _ptr(Vl), w, wb, _stream(stream)))


def pbsa_attention_mass(p, Q, Kp, p_len, Kl, l_len, l_map, sel, lse, Mt, stream=None):
    _check(lib().pbsa_attention_mass(ctypes.byref(p), _ptr(Q), _ptr(Kp), _ptr(p_len), _ptr(Kl), _ptr(l_len),
                                     _ptr(l_map), _ptr(sel), _ptr(lse), _ptr(Mt), _stream(stream)))


def pbsa_mass_workspace_bytes(p: pbsa_params) -> int:
    out = ctypes.c_size_t(0)
    _check(lib().pbsa_mass_workspace_bytes(ctypes.byref(p), ctypes.byref(out)))
    return out.value


def pbsa_attention_fwd_mass(p, Q, Kp, Vp, p_len, Kl, Vl, l_len, l_map, sel, O, lse, Mt, ws, stream=None):
    w, wb = _ws(ws)
    _check(lib().pbsa_attention_fwd_mass(ctypes.byref(p), _ptr(Q), _ptr(Kp), _ptr(Vp), _ptr(p_len), _ptr(Kl), _ptr(Vl),
                                         _ptr(l_len), _ptr(l_map), _ptr(sel), _ptr(O), _ptr(lse), _ptr(Mt), w, wb,
                                         _stream(stream)))


def pbsa_memory_update_fine(p, Mt, Kc_l, Kp, Vp, Kc_p, p_len, p_id, S_sum, S_cnt, Kl, Vl, l_len, l_map, l_id, scores,
                            slot_src, ws, stream=None):
    w, wb = _ws(ws)
    _check(lib().pbsa_memory_update_fine(ctypes.byref(p), _ptr(Mt), _ptr(Kc_l), _ptr(Kp), _ptr(Vp), _ptr(Kc_p),
                                         _ptr(p_len), _ptr(p_id), _ptr(S_sum), _ptr(S_cnt), _ptr(Kl), _ptr(Vl),
                                         _ptr(l_len), _ptr(l_map), _ptr(l_id), _ptr(scores), _ptr(slot_src), w, wb,
                                         _stream(stream)))


def pbsa_bwd_workspace_bytes(p: pbsa_params) -> int:
    out = ctypes.c_size_t(0)
    _check(lib().pbsa_bwd_workspace_bytes(ctypes.byref(p), ctypes.byref(out)))
    return out.value


def pbsa_attention_bwd(p, Q, Kp, Vp, p_len, Kl, Vl, l_len, l_map, sel, O, dO, lse, dQ, dKp, dVp, dKl, dVl, ws, stream=None):
    w, wb = _ws(ws)
    _check(lib().pbsa_attention_bwd(ctypes.byref(p), _ptr(Q), _ptr(Kp), _ptr(Vp), _ptr(p_len), _ptr(Kl), _ptr(Vl),
                                    _ptr(l_len), _ptr(l_map), _ptr(sel), _ptr(O), _ptr(dO), _ptr(lse), _ptr(dQ),
                                    _ptr(dKp), _ptr(dVp), _ptr(dKl), _ptr(dVl), w, wb, _stream(stream)))


def pbsa_blockify(g, X, Xblk, blk_stride_h, stream=None):
    """X, Xblk: sequences of tensors (or device addresses), blk_stride_h: sequence of ints, one per tensor."""
    n = len(X)
    xs = (ctypes.c_void_p * n)(*[_ptr(x) for x in X])
    bs = (ctypes.c_void_p * n)(*[_ptr(x) for x in Xblk])
    st = (ctypes.c_int64 * n)(*[int(v) for v in blk_stride_h])
    _check(lib().pbsa_blockify(ctypes.byref(g), n, xs, bs, st, _stream(stream)))


def pbsa_unblockify(g, Xblk, blk_stride_h, X, stream=None):
    _check(lib().pbsa_unblockify(ctypes.byref(g), _ptr(Xblk), int(blk_stride_h), _ptr(X), _stream(stream)))
