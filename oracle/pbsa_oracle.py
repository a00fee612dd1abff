"""ctypes binding of the CPU oracle (pbsa_oracle.c) -- TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this module; the
product package never does.  All arrays are host numpy arrays in the layouts documented at the
top of pbsa_oracle.c; bf16 tensors travel as uint16 bit patterns.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pbsa_oracle.c")
_LIB = os.path.join(_HERE, "libpbsa_oracle.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (strict fp32: no contraction, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off", "-fno-fast-math",
               "-mfma", "-mavx2", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


class _Cfg(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("H", "d", "B", "Nq", "nqb", "n_loc", "n_loc_cap", "C", "n_sink", "k", "causal", "n_evict",
                 "pool_from")] + [("scale", ctypes.c_float)]


@dataclass
class Cfg:
    H: int
    d: int
    B: int
    Nq: int
    n_loc: int
    n_loc_cap: int
    C: int
    k: int
    scale: float
    n_sink: int = 0
    causal: int = 1
    n_evict: int = 0
    pool_from: int = 0

    @property
    def nqb(self) -> int:
        return -(-self.Nq // self.B)

    def c(self) -> _Cfg:
        return _Cfg(self.H, self.d, self.B, self.Nq, self.nqb, self.n_loc, self.n_loc_cap, self.C, self.n_sink,
                    self.k, self.causal, self.n_evict, self.pool_from, np.float32(self.scale))


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.orc_pexp.restype = ctypes.c_float
        _lib.orc_pexp.argtypes = [ctypes.c_float]
    return _lib


def _p(a, dtype, shape=None):
    """Pointer to a C-contiguous numpy array after checking dtype (and shape)."""
    if a is None:
        return None
    if not isinstance(a, np.ndarray) or a.dtype != np.dtype(dtype) or not a.flags["C_CONTIGUOUS"]:
        raise TypeError(f"expected C-contiguous {np.dtype(dtype)} array, got {getattr(a, 'dtype', type(a))}")
    if shape is not None and tuple(a.shape) != tuple(shape):
        raise ValueError(f"expected shape {tuple(shape)}, got {tuple(a.shape)}")
    return a.ctypes.data_as(ctypes.c_void_p)


def num_threads() -> int:
    """Threads the OpenMP loops of the oracle use."""
    return int(lib().orc_num_threads())


def pexp(x: float) -> float:
    return float(lib().orc_pexp(ctypes.c_float(x)))


def pool_block(rows: np.ndarray, length: int) -> np.ndarray:
    """Average-pool the first `length` rows of a [*, d] bf16-bit block -> fp32 [d]."""
    d = rows.shape[-1]
    out = np.zeros(d, np.float32)
    lib().orc_pool_block(_p(np.ascontiguousarray(rows), np.uint16), ctypes.c_int(length), ctypes.c_int(d),
                         _p(out, np.float32))
    return out


def select(cfg: Cfg, Q, Kl, l_len, l_map, Kc_l, want_logits: bool = False):
    """Returns (Qc [H][nqb][d] f32, sel [H][nqb][k] i32, Z or None); updates Kc_l in place."""
    H, d, B, nqb = cfg.H, cfg.d, cfg.B, cfg.nqb
    Qc = np.zeros((H, nqb, d), np.float32)
    sel = np.full((H, nqb, max(cfg.k, 0)), -1, np.int32)
    Z = np.zeros((H, nqb, cfg.n_loc), np.float32) if want_logits else None
    c = cfg.c()
    rc = lib().orc_select(ctypes.byref(c), _p(Q, np.uint16, (H, cfg.Nq, d)),
                          _p(Kl, np.uint16, (H, cfg.n_loc_cap, B, d)), _p(l_len, np.int32, (cfg.n_loc,)),
                          _p(l_map, np.int32, (cfg.n_loc,)), _p(Kc_l, np.float32, (H, cfg.n_loc_cap, d)),
                          _p(Qc, np.float32), _p(sel, np.int32), _p(Z, np.float32))
    if rc:
        raise RuntimeError(f"orc_select failed: {rc}")
    return Qc, sel, Z


def attention_rows(cfg: Cfg, Q, Kp, Vp, p_len, Kl, Vl, l_len, l_map, sel, rows_h, rows_t):
    """fp64 outputs [n_rows][d] and log-sum-exp [n_rows] of the requested (head, token) rows."""
    H, d, B = cfg.H, cfg.d, cfg.B
    rows_h = np.ascontiguousarray(rows_h, np.int32)
    rows_t = np.ascontiguousarray(rows_t, np.int32)
    n = rows_h.shape[0]
    O = np.zeros((n, d), np.float64)
    lse = np.zeros(n, np.float64)
    c = cfg.c()
    rc = lib().orc_attention_rows(
        ctypes.byref(c), _p(Q, np.uint16, (H, cfg.Nq, d)), _p(Kp, np.uint16, (H, cfg.C + 1, B, d)),
        _p(Vp, np.uint16, (H, cfg.C + 1, B, d)), _p(p_len, np.int32, (H, cfg.C + 1)),
        _p(Kl, np.uint16, (H, cfg.n_loc_cap, B, d)), _p(Vl, np.uint16, (H, cfg.n_loc_cap, B, d)),
        _p(l_len, np.int32, (cfg.n_loc,)), _p(l_map, np.int32, (cfg.n_loc,)),
        _p(sel, np.int32, (H, cfg.nqb, cfg.k)), ctypes.c_int64(n), _p(rows_h, np.int32), _p(rows_t, np.int32),
        _p(O, np.float64), _p(lse, np.float64))
    if rc:
        raise RuntimeError(f"orc_attention_rows failed: {rc}")
    return O, lse


def attention(cfg: Cfg, Q, Kp, Vp, p_len, Kl, Vl, l_len, l_map, sel):
    """All rows: O [H][Nq][d] fp64, lse [H][Nq] fp64."""
    hh, tt = np.meshgrid(np.arange(cfg.H, dtype=np.int32), np.arange(cfg.Nq, dtype=np.int32), indexing="ij")
    O, lse = attention_rows(cfg, Q, Kp, Vp, p_len, Kl, Vl, l_len, l_map, sel, hh.ravel(), tt.ravel())
    return O.reshape(cfg.H, cfg.Nq, cfg.d), lse.reshape(cfg.H, cfg.Nq)


def scores(cfg: Cfg, Qc, Kc_l, l_map, Kc_p, p_len):
    """Persistence scores: s_p [H][C], s_l [H][n_loc] (fp32)."""
    H, d = cfg.H, cfg.d
    s_p = np.zeros((H, cfg.C), np.float32)
    s_l = np.zeros((H, cfg.n_loc), np.float32)
    c = cfg.c()
    rc = lib().orc_scores(ctypes.byref(c), _p(Qc, np.float32, (H, cfg.nqb, d)),
                          _p(Kc_l, np.float32, (H, cfg.n_loc_cap, d)), _p(l_map, np.int32, (cfg.n_loc,)),
                          _p(Kc_p, np.float32, (H, cfg.C, d)), _p(p_len, np.int32, (H, cfg.C + 1)),
                          _p(s_p, np.float32), _p(s_l, np.float32))
    if rc:
        raise RuntimeError(f"orc_scores failed: {rc}")
    return s_p, s_l


def memory_update(cfg: Cfg, Qc, Kc_l, Kp, Vp, Kc_p, p_len, p_id, S_sum, S_cnt, Kl, Vl, l_len, l_map, l_id):
    """In-place update of (Kp, Vp, Kc_p, p_len, p_id, S_sum, S_cnt); returns (scores, slot_src)."""
    H, d, B, C = cfg.H, cfg.d, cfg.B, cfg.C
    sc = np.zeros((H, C + cfg.n_evict), np.float32)
    src = np.full((H, C), -1, np.int32)
    c = cfg.c()
    rc = lib().orc_memory_update(
        ctypes.byref(c), _p(Qc, np.float32, (H, cfg.nqb, d)), _p(Kc_l, np.float32, (H, cfg.n_loc_cap, d)),
        _p(Kp, np.uint16, (H, C + 1, B, d)), _p(Vp, np.uint16, (H, C + 1, B, d)),
        _p(Kc_p, np.float32, (H, C, d)), _p(p_len, np.int32, (H, C + 1)), _p(p_id, np.int64, (H, C)),
        _p(S_sum, np.float32, (H, 2, B, d)) if S_sum is not None else None,
        _p(S_cnt, np.int32, (H, B)) if S_sum is not None else None,
        _p(Kl, np.uint16, (H, cfg.n_loc_cap, B, d)), _p(Vl, np.uint16, (H, cfg.n_loc_cap, B, d)),
        _p(l_len, np.int32, (cfg.n_loc,)), _p(l_map, np.int32, (cfg.n_loc,)), _p(l_id, np.int64, (cfg.n_loc,)),
        _p(sc, np.float32), _p(src, np.int32))
    if rc:
        raise RuntimeError(f"orc_memory_update failed: {rc}")
    return sc, src


def attention_mass(cfg: Cfg, Q, Kp, p_len, Kl, l_len, l_map, sel, qb_h=None, qb_i=None):
    """fp64 attention mass of every key block from the requested query blocks: [n][C+1+n_loc]
    (all H * nqb query blocks, head-major, when no list is given)."""
    H, d, B = cfg.H, cfg.d, cfg.B
    if qb_h is None:
        hh, ii = np.meshgrid(np.arange(H, dtype=np.int32), np.arange(cfg.nqb, dtype=np.int32), indexing="ij")
        qb_h, qb_i = hh.ravel(), ii.ravel()
    qb_h = np.ascontiguousarray(qb_h, np.int32)
    qb_i = np.ascontiguousarray(qb_i, np.int32)
    n = qb_h.shape[0]
    mass = np.zeros((n, cfg.C + 1 + cfg.n_loc), np.float64)
    c = cfg.c()
    rc = lib().orc_attention_mass(
        ctypes.byref(c), _p(Q, np.uint16, (H, cfg.Nq, d)), _p(Kp, np.uint16, (H, cfg.C + 1, B, d)),
        _p(p_len, np.int32, (H, cfg.C + 1)), _p(Kl, np.uint16, (H, cfg.n_loc_cap, B, d)),
        _p(l_len, np.int32, (cfg.n_loc,)), _p(l_map, np.int32, (cfg.n_loc,)),
        _p(sel, np.int32, (H, cfg.nqb, cfg.k)), ctypes.c_int64(n), _p(qb_h, np.int32), _p(qb_i, np.int32),
        _p(mass, np.float64))
    if rc:
        raise RuntimeError(f"orc_attention_mass failed: {rc}")
    return mass


def memory_update_fine(cfg: Cfg, Mt, Kc_l, Kp, Vp, Kc_p, p_len, p_id, S_sum, S_cnt, Kl, Vl, l_len, l_map, l_id):
    """Update ranked by fine attention mass Mt [H][C+1+n_loc][nqb] fp32; in place like memory_update;
    returns (scores, slot_src)."""
    H, d, B, C = cfg.H, cfg.d, cfg.B, cfg.C
    sc = np.zeros((H, C + cfg.n_evict), np.float32)
    src = np.full((H, C), -1, np.int32)
    c = cfg.c()
    rc = lib().orc_memory_update_fine(
        ctypes.byref(c), _p(Mt, np.float32, (H, C + 1 + cfg.n_loc, cfg.nqb)),
        _p(Kc_l, np.float32, (H, cfg.n_loc_cap, d)),
        _p(Kp, np.uint16, (H, C + 1, B, d)), _p(Vp, np.uint16, (H, C + 1, B, d)),
        _p(Kc_p, np.float32, (H, C, d)), _p(p_len, np.int32, (H, C + 1)), _p(p_id, np.int64, (H, C)),
        _p(S_sum, np.float32, (H, 2, B, d)) if S_sum is not None else None,
        _p(S_cnt, np.int32, (H, B)) if S_sum is not None else None,
        _p(Kl, np.uint16, (H, cfg.n_loc_cap, B, d)), _p(Vl, np.uint16, (H, cfg.n_loc_cap, B, d)),
        _p(l_len, np.int32, (cfg.n_loc,)), _p(l_map, np.int32, (cfg.n_loc,)), _p(l_id, np.int64, (cfg.n_loc,)),
        _p(sc, np.float32), _p(src, np.int32))
    if rc:
        raise RuntimeError(f"orc_memory_update_fine failed: {rc}")
    return sc, src


def attention_bwd(cfg: Cfg, Q, Kp, Vp, p_len, Kl, Vl, l_len, l_map, sel, dO, row_mask=None, want_kv=True):
    """fp64 gradients of the fine stage: (dQ [H][Nq][d], dKp, dVp [H][C+1][B][d], dKl, dVl [H][cap][B][d]);
    with row_mask ([H][Nq] bool) only those rows take part."""
    H, d, B = cfg.H, cfg.d, cfg.B
    dQ = np.zeros((H, cfg.Nq, d), np.float64)
    outs = [np.zeros((H, cfg.C + 1, B, d), np.float64), np.zeros((H, cfg.C + 1, B, d), np.float64),
            np.zeros((H, cfg.n_loc_cap, B, d), np.float64), np.zeros((H, cfg.n_loc_cap, B, d), np.float64)] if want_kv else [None] * 4
    mask = None if row_mask is None else np.ascontiguousarray(row_mask, np.uint8)
    c = cfg.c()
    rc = lib().orc_attention_bwd(
        ctypes.byref(c), _p(Q, np.uint16, (H, cfg.Nq, d)), _p(Kp, np.uint16, (H, cfg.C + 1, B, d)),
        _p(Vp, np.uint16, (H, cfg.C + 1, B, d)), _p(p_len, np.int32, (H, cfg.C + 1)),
        _p(Kl, np.uint16, (H, cfg.n_loc_cap, B, d)), _p(Vl, np.uint16, (H, cfg.n_loc_cap, B, d)),
        _p(l_len, np.int32, (cfg.n_loc,)), _p(l_map, np.int32, (cfg.n_loc,)),
        _p(sel, np.int32, (H, cfg.nqb, cfg.k)), _p(dO, np.uint16, (H, cfg.Nq, d)),
        _p(mask, np.uint8, (H, cfg.Nq)) if mask is not None else None,
        _p(dQ, np.float64), *[_p(a, np.float64) if a is not None else None for a in outs])
    if rc:
        raise RuntimeError(f"orc_attention_bwd failed: {rc}")
    return (dQ, *outs)
