"""Test infrastructure: how far the integer decisions of the method are from a tie, in fp64.

Selection (Eq. 6, 10-11) and retention (Eq. 7-9) both cut a sorted list of real scores at a fixed rank.  The
library and the oracle take those decisions in one pinned fp32 arithmetic, so they agree whatever the margin is;
this audit says how much the decisions depend on that arithmetic at all.  It recomputes the pooled vectors, the
block logits and the persistence scores in fp64 from the bf16 inputs (plain definitions: means, dot products, row
softmax, column mean) and reports, for every cut, the relative gap

    (last kept - first dropped) / max(|last kept|, |first dropped|)

between the two scores on either side of it, together with the cuts where the fp64 ranking and the pinned-fp32
ranking choose different sets.  numpy only; shares nothing with the library or with the C oracle.
"""
from __future__ import annotations

import numpy as np


def bf16_to_f64(bits: np.ndarray) -> np.ndarray:
    return (np.asarray(bits, np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def pooled_f64(block_bits: np.ndarray, length: int) -> np.ndarray:
    """Eq. 6: the mean of the first `length` rows of a [B][d] block (zero vector for an empty block)."""
    if length <= 0:
        return np.zeros(block_bits.shape[-1], np.float64)
    return bf16_to_f64(block_bits[:length]).mean(axis=0)


def rel_gap(kept: float, dropped: float) -> float:
    den = max(abs(kept), abs(dropped))
    return float("inf") if den == 0.0 and kept == dropped else (kept - dropped) / den if den > 0.0 else float("inf")


def _cut(values: np.ndarray, keep: int):
    """values sorted by (value desc, index asc): the kept index set and the relative gap at the cut (None when
    nothing is dropped or nothing is kept)."""
    order = np.lexsort((np.arange(len(values)), -values))
    kept = set(int(j) for j in order[:keep])
    if keep <= 0 or keep >= len(values):
        return kept, None
    return kept, rel_gap(float(values[order[keep - 1]]), float(values[order[keep]]))


def _local_pooled(st):
    l_map, l_len, _ = st._maps()
    Kc = np.zeros((st.H, st.n_loc, st.d), np.float64)
    for h in range(st.H):
        for l in range(st.n_loc):
            Kc[h, l] = pooled_f64(st.Kl[h, l_map[l]], int(l_len[l]))
    return Kc


def _query_pooled(st, Q):
    Qc = np.zeros((st.H, st.nqb, st.d), np.float64)
    for i in range(st.nqb):
        rows = bf16_to_f64(Q[:, i * st.B:min((i + 1) * st.B, st.Nq)])
        Qc[:, i] = rows.mean(axis=1)
    return Qc


def selection_gaps(st, Q, sel=None):
    """Cuts of Eq. 11 for the chunk whose queries are Q (bf16 bits [H][Nq][d]) against the state's local region.
    Returns dict(gaps=[(h, i, gap)], mismatches=[(h, i)] against `sel` [H][nqb][k] if given)."""
    Qc, Kc = _query_pooled(st, Q), _local_pooled(st)
    z = np.einsum("hid,hld->hil", Qc, Kc) * float(st.scale)
    gaps, mismatches = [], []
    for h in range(st.H):
        for i in range(st.nqb):
            nvis = st.n_loc - st.nqb + i + 1 if st.causal else st.n_loc
            kept, gap = _cut(z[h, i, :nvis], min(st.k, nvis))
            if gap is not None:
                gaps.append((h, i, gap))
            if sel is not None and kept != set(int(j) for j in sel[h, i] if j >= 0):
                mismatches.append((h, i))
    return dict(gaps=gaps, mismatches=mismatches)


def retention_gaps(st, Q, n_evict, slot_src=None, p_id_before=None):
    """The cut of Eq. 9 for the update that follows the chunk whose queries are Q: scores of Eq. 7-8 in fp64 over
    U = occupied slots then all local blocks, candidates = occupants of slots n_sink.. then the n_evict leading
    local blocks, the best C - n_sink kept.  Returns dict(gaps=[(h, gap)], kept=[set of candidate indices per head]),
    candidate index = slot for a slot, C + e for evicted block e."""
    Qc, Kc_l = _query_pooled(st, Q), _local_pooled(st)
    C = st.C
    gaps, kept_sets = [], []
    for h in range(st.H):
        occ = [s for s in range(C) if st.p_len[h, s] > 0]
        cols = [pooled_f64(st.Kp[h, s], int(st.p_len[h, s])) for s in occ] + [Kc_l[h, l] for l in range(st.n_loc)]
        U = np.stack(cols) if cols else np.zeros((0, st.d))
        z = (Qc[h] @ U.T) * float(st.scale)
        e = np.exp(z - z.max(axis=1, keepdims=True))
        s = (e / e.sum(axis=1, keepdims=True)).mean(axis=0)
        cand = [c for c in occ if c >= st.n_sink] + [C + ev for ev in range(n_evict)]
        score = np.array([s[occ.index(c)] if c < C else s[len(occ) + (c - C)] for c in cand], np.float64)
        kept, gap = _cut(score, min(C - st.n_sink, len(cand)))
        kept_sets.append(set(cand[j] for j in kept))
        if gap is not None:
            gaps.append((h, gap))
    return dict(gaps=gaps, kept=kept_sets)
