"""Seeded synthetic inputs for the PBSA decode path (workload shapes + random tensors only).

This module is plumbing shared by the GPU harness and by the CPU checker: it draws the
random Q/K/V tensors, lays a chunk out block-major, and lists the workload shapes.  It holds
none of the method's arithmetic (no pooling, scoring, selection, softmax or retention).

Generator: counter-based.  Every element is a pure function of (seed, tensor tag, layer,
chunk, flat index): a splitmix64-style finaliser gives two 53-bit uniforms per pair of
outputs, Box-Muller (fp64) turns them into two standard normals, and the result is rounded
fp64 -> fp32 -> bf16 (round-to-nearest-even).  No library RNG stream is involved, so the
bits do not depend on numpy / torch versions.

Shapes stand in for Wan2.1-T2V-1.3B activations (Sec. 4.1 of the paper: 12 heads of 128,
chunks of 3 latent frames; 30x52 = 1560 tokens per latent frame at 832x480), which are not
available here.  Structure: a per-block low-rank bias whose coefficients follow an AR(1)
walk along the block index, so neighbouring blocks score alike (the "locally diagonal"
pattern of Sec. 3.2), plus optional heavy-tailed blocks.
"""
from __future__ import annotations

import functools
import math
import os
from dataclasses import dataclass

import numpy as np

_M64 = (1 << 64) - 1
_GOLD = 0x9E3779B97F4A7C15


def _mix_int(x: int) -> int:
    x &= _M64
    x = ((x ^ (x >> 30)) * 0xBF58476D1CE4E5B9) & _M64
    x = ((x ^ (x >> 27)) * 0x94D049BB133111EB) & _M64
    return x ^ (x >> 31)


def _mix_arr(x: np.ndarray) -> np.ndarray:
    x = x.copy()
    x ^= x >> np.uint64(30)
    x *= np.uint64(0xBF58476D1CE4E5B9)
    x ^= x >> np.uint64(27)
    x *= np.uint64(0x94D049BB133111EB)
    x ^= x >> np.uint64(31)
    return x


_TAGS = {"q": 1, "k": 2, "v": 3, "basis_qk": 4, "basis_v": 5, "coef": 6, "heavy": 7,
         "pk": 8, "pv": 9, "pcoef": 10, "summary": 11, "misc": 12}


def stream_key(seed: int, tag: str, *idx: int) -> int:
    """64-bit key of one random stream: a hash of (seed, tensor tag, integer indices)."""
    k = _mix_int(seed * _GOLD + _TAGS[tag])
    for i in idx:
        k = _mix_int(k + (int(i) + 0x632BE59BD9B4E019) * _GOLD)
    return k


def uniforms(key: int, n: int) -> np.ndarray:
    """n uniforms in [0, 1) (fp64, 53 bits), element i a pure function of (key, i)."""
    with np.errstate(over="ignore"):
        ctr = np.arange(n, dtype=np.uint64) * np.uint64(_GOLD) + np.uint64(key)
        bits = _mix_arr(ctr)
    return (bits >> np.uint64(11)).astype(np.float64) * (1.0 / (1 << 53))


def _normals_into(out: np.ndarray, key: int, s: int, e: int) -> None:
    """Fill out[2s:2e] with the normals of pair counters s..e-1."""
    with np.errstate(over="ignore"):
        ctr = np.arange(s, e, dtype=np.uint64)
        ctr *= np.uint64(2)
        ctr *= np.uint64(_GOLD)
        ctr += np.uint64(key)
        a = _mix_arr(ctr)
        ctr += np.uint64(_GOLD)
        b = _mix_arr(ctr)
    a >>= np.uint64(11)
    b >>= np.uint64(11)
    u1 = a.astype(np.float64)
    u1 += 1.0
    u1 *= 1.0 / (1 << 53)                  # (0, 1]
    th = b.astype(np.float64)
    th *= (2.0 * math.pi) / (1 << 53)      # 2 pi u2, u2 in [0, 1)
    np.log(u1, out=u1)
    u1 *= -2.0
    np.sqrt(u1, out=u1)
    out[2 * s:2 * e:2] = u1 * np.cos(th)
    np.sin(th, out=th)
    th *= u1
    out[2 * s + 1:2 * e:2] = th


_POOL = None
_N_THREADS = max(1, min(16, len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else 4))


def normals(key: int, n: int) -> np.ndarray:
    """n standard normals (fp64) by Box-Muller on pairs of counter-based uniforms.

    Element i depends only on (key, i); large requests are split over a few threads, which changes
    nothing in the result.
    """
    global _POOL
    npair = (n + 1) // 2
    out = np.empty(2 * npair, dtype=np.float64)
    step = 1 << 18
    spans = [(s, min(npair, s + step)) for s in range(0, npair, step)]
    if len(spans) <= 1 or _N_THREADS == 1:
        for s, e in spans:
            _normals_into(out, key, s, e)
    else:
        if _POOL is None:
            from concurrent.futures import ThreadPoolExecutor
            _POOL = ThreadPoolExecutor(max_workers=_N_THREADS)
        list(_POOL.map(lambda se: _normals_into(out, key, se[0], se[1]), spans))
    return out[:n]


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp64/fp32 values to bf16 (nearest even) and return the 16-bit patterns (uint16)."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns (uint16) exactly to fp32."""
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


@dataclass(frozen=True)
class Workload:
    """One synthetic workload: tensor shapes, cache geometry and the input recipe."""
    name: str
    H: int                 # attention heads
    d: int                 # head dim
    F: int                 # tokens per latent frame
    B: int                 # tokens per block
    chunk_frames: int      # latent frames per query chunk
    window_chunks: int     # whole chunks in the sliding local window
    C: int                 # persistent slots
    k: int                 # local blocks selected per query block
    seed: int
    bias_rank: int = 0
    bias_scale: float = 0.0
    heavy_prob: float = 0.0
    heavy_scale: float = 1.0
    n_layers: int = 1
    n_chunks: int = 1      # sequential chunks of the rollout this workload measures
    cold_start: bool = False
    summary_prefill: int = 0   # blocks already folded into the summary (0 = empty)
    rho: float = 0.9       # AR(1) coefficient of the block-bias walk

    @property
    def Nq(self) -> int:
        return self.F * self.chunk_frames

    @property
    def nqb(self) -> int:
        return -(-self.Nq // self.B)

    @property
    def n_win(self) -> int:
        return self.window_chunks * self.nqb

    @property
    def n_loc(self) -> int:
        return self.n_win + self.nqb

    @property
    def scale(self) -> float:
        return 1.0 / math.sqrt(self.d)


WORKLOADS = {
    "cfg1": Workload("cfg1", H=2, d=64, F=256, B=64, chunk_frames=1, window_chunks=3, C=2, k=4, seed=0),
    "cfg2": Workload("cfg2", H=12, d=128, F=1560, B=128, chunk_frames=3, window_chunks=2, C=8, k=16, seed=1,
                     bias_rank=4, bias_scale=2.0),
    "cfg3": Workload("cfg3", H=12, d=128, F=1560, B=128, chunk_frames=3, window_chunks=2, C=8, k=16, seed=1,
                     bias_rank=4, bias_scale=2.0, n_layers=30),
    "cfg4": Workload("cfg4", H=12, d=128, F=1560, B=128, chunk_frames=3, window_chunks=3, C=16, k=24, seed=2,
                     bias_rank=4, bias_scale=2.0, summary_prefill=946),
    "cfg5": Workload("cfg5", H=12, d=128, F=1560, B=64, chunk_frames=3, window_chunks=3, C=32, k=48, seed=3,
                     bias_rank=4, bias_scale=2.0, heavy_prob=0.10, heavy_scale=4.0, n_chunks=80,
                     cold_start=True),
}


def t7_workload(ratio_l: int, ratio_p: float, topk: float, B: int = 128, frames: int = 3) -> Workload:
    """A shape of the paper's kernel benchmark (App. kernel-level analysis, the forward columns of the
    latency table): 1792-token frames, query chunk N_C = 3 frames = 5376 tokens or 12 frames = 21504
    (blocks divide it exactly), local KV N_L = ratio_l * N_C (the chunk included), persistent KV N_P = ratio_p * N_L,
    top-k = topk * (number of local blocks); topk = 1 selects every block (the dense stand-in).
    Heads and head dim are not stated there: 12 x 128 as in the other workloads."""
    F = 1792
    nqb = F * frames // B
    n_loc = ratio_l * nqb
    C = int(round(ratio_p * n_loc))
    k = n_loc if topk >= 1.0 else max(1, int(round(topk * n_loc)))
    name = f"t7_C{frames}_L{ratio_l}_P{int(round(ratio_p * 100))}_K{int(round(topk * 10000))}_B{B}"
    return Workload(name, H=12, d=128, F=F, B=B, chunk_frames=frames, window_chunks=ratio_l - 1, C=C, k=k,
                    seed=7, bias_rank=4, bias_scale=2.0)


MAX_CHUNKS = 128   # the block-bias walk and heavy flags are drawn for this many chunks up front


def block_lens(w: Workload) -> np.ndarray:
    """Valid tokens of each of the chunk's nqb blocks (blocks tile the chunk from its first token)."""
    lens = np.full(w.nqb, w.B, dtype=np.int32)
    lens[-1] = w.Nq - (w.nqb - 1) * w.B
    return lens


@functools.lru_cache(maxsize=64)
def _block_coeffs(w: Workload, layer: int, n_blocks: int) -> np.ndarray:
    """AR(1) walk of the bias coefficients along the global block index: [H][n_blocks][rank], unit variance."""
    R = max(w.bias_rank, 1)
    eps = normals(stream_key(w.seed, "coef", layer), w.H * n_blocks * R).reshape(w.H, n_blocks, R)
    c = np.empty_like(eps)
    c[:, 0] = eps[:, 0]
    g = math.sqrt(1.0 - w.rho * w.rho)
    for b in range(1, n_blocks):
        c[:, b] = w.rho * c[:, b - 1] + g * eps[:, b]
    return c


def _basis(w: Workload, layer: int, tag: str) -> np.ndarray:
    """[H][rank][d] directions with entries N(0, 1/d)."""
    R = max(w.bias_rank, 1)
    return normals(stream_key(w.seed, tag, layer), w.H * R * w.d).reshape(w.H, R, w.d) / math.sqrt(w.d)


def _heavy_flags(w: Workload, layer: int, n_blocks: int) -> np.ndarray:
    u = uniforms(stream_key(w.seed, "heavy", layer), w.H * n_blocks).reshape(w.H, n_blocks)
    return u < w.heavy_prob


@functools.lru_cache(maxsize=6)
def chunk_qkv(w: Workload, layer: int, chunk: int):
    """bf16 bit patterns (uint16) of Q, K, V for global chunk index `chunk`: each [H][Nq][d], token-major.

    Q/K/V ~ N(0,1); with bias_rank > 0 every token of global block g gets
    bias_scale * sum_r c[g][r] u[r] added (Q and K share the basis u, V has its own); with
    heavy_prob > 0 a (head, block) is heavy with that probability and its Q and K tokens are
    multiplied by heavy_scale (V is left alone so outputs stay in bf16's fine range).
    The returned arrays are cached and read-only.
    """
    H, Nq, d, B, nqb = w.H, w.Nq, w.d, w.B, w.nqb
    if not 0 <= chunk < MAX_CHUNKS:
        raise ValueError("chunk index out of range")
    n = H * Nq * d
    out = []
    if w.bias_rank > 0:
        coef = _block_coeffs(w, layer, MAX_CHUNKS * nqb)[:, chunk * nqb:(chunk + 1) * nqb]  # [H][nqb][R]
        tok_blk = np.arange(Nq) // B
    if w.heavy_prob > 0:
        heavy = _heavy_flags(w, layer, MAX_CHUNKS * nqb)[:, chunk * nqb:(chunk + 1) * nqb]
    for tag in ("q", "k", "v"):
        x = normals(stream_key(w.seed, tag, layer, chunk), n).reshape(H, Nq, d)
        if w.bias_rank > 0:
            u = _basis(w, layer, "basis_v" if tag == "v" else "basis_qk")       # [H][R][d]
            blk_bias = w.bias_scale * np.einsum("hbr,hrd->hbd", coef, u)       # [H][nqb][d]
            x += blk_bias[:, tok_blk, :]
        if w.heavy_prob > 0 and tag != "v":
            mul = np.where(heavy, w.heavy_scale, 1.0)[:, np.arange(Nq) // B]     # [H][Nq]
            x *= mul[:, :, None]
        bits = to_bf16_bits(x)
        bits.setflags(write=False)
        out.append(bits)
    return tuple(out)


def to_blocks(x: np.ndarray, B: int) -> np.ndarray:
    """[H][Nq][d] token-major -> [H][nqb][B][d] block-major, the ragged last block zero-padded."""
    H, Nq, d = x.shape
    nqb = -(-Nq // B)
    out = np.zeros((H, nqb * B, d), dtype=x.dtype)
    out[:, :Nq] = x
    return out.reshape(H, nqb, B, d)


def persistent_init(w: Workload, layer: int):
    """Initial occupants of the C persistent slots, drawn like any block: (Kp, Vp) uint16 [H][C][B][d], all full."""
    H, C, B, d = w.H, w.C, w.B, w.d
    res = []
    if w.bias_rank > 0:
        coef = normals(stream_key(w.seed, "pcoef", layer), H * C * w.bias_rank).reshape(H, C, w.bias_rank)
    for tag, btag in (("pk", "basis_qk"), ("pv", "basis_v")):
        x = normals(stream_key(w.seed, tag, layer), H * C * B * d).reshape(H, C, B, d)
        if w.bias_rank > 0:
            u = _basis(w, layer, btag)
            x += (w.bias_scale * np.einsum("hcr,hrd->hcd", coef, u))[:, :, None, :]
        res.append(to_bf16_bits(x))
    return tuple(res)


def summary_init(w: Workload, layer: int):
    """Pre-filled compressed-history state: S_sum fp32 [H][2][B][d], S_cnt int32 [H][B].

    Stands for `summary_prefill` blocks folded earlier: the count is summary_prefill for positions every
    block has and proportionally fewer for positions only full blocks have; the running mean is
    N(0, 1/count) per element.
    """
    H, B, d = w.H, w.B, w.d
    cnt = np.zeros((H, B), dtype=np.int32)
    ssum = np.zeros((H, 2, B, d), dtype=np.float32)
    if w.summary_prefill > 0:
        tail = int(block_lens(w)[-1])
        full = w.summary_prefill
        part = full - full // w.nqb            # positions the ragged block lacks
        cnt[:, :tail] = full
        cnt[:, tail:] = part
        mean = normals(stream_key(w.seed, "summary", layer), H * 2 * B * d).reshape(H, 2, B, d)
        c = cnt.astype(np.float64)[:, None, :, None]
        ssum = (mean / np.sqrt(c) * c).astype(np.float32)
    return ssum, cnt
