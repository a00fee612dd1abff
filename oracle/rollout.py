"""Host-side (numpy) cache state that drives the CPU oracle through a chunk-by-chunk rollout.

TEST INFRASTRUCTURE ONLY, like everything under oracle/.  It plays the caller of Alg. 1: it
writes each chunk's K/V blocks into the local ring, asks the oracle for the block sets
(Eq. 10-11), optionally the attention rows (Eq. 3-5), runs the persistent update (Eq. 7-9) on
the chunk's clean pass, and slides the window.
"""
from __future__ import annotations

import numpy as np

from . import pbsa_oracle as orc


class OracleState:
    def __init__(self, H, d, B, Nq, window_chunks, C, k, scale, n_sink=0, causal=1, fold=True):
        self.H, self.d, self.B, self.Nq, self.C, self.k = H, d, B, Nq, C, k
        self.w, self.scale, self.n_sink, self.causal = window_chunks, scale, n_sink, causal
        self.nqb = -(-Nq // B)
        self.cap = (window_chunks + 1) * self.nqb
        self.Kl = np.zeros((H, self.cap, B, d), np.uint16)
        self.Vl = np.zeros_like(self.Kl)
        self.Kc_l = np.zeros((H, self.cap, d), np.float32)
        self.Kp = np.zeros((H, C + 1, B, d), np.uint16)
        self.Vp = np.zeros_like(self.Kp)
        self.Kc_p = np.zeros((H, C, d), np.float32)
        self.p_len = np.zeros((H, C + 1), np.int32)
        self.p_id = np.full((H, C), -1, np.int64)
        self.S_sum = np.zeros((H, 2, B, d), np.float32) if fold else None
        self.S_cnt = np.zeros((H, B), np.int32) if fold else None
        self.chunks = []        # (ring position, lens, ids) of the chunks in the local region, oldest first
        self.n_appended = 0
        self.stale_from = 0     # logical blocks >= this need their pooled key (re)computed

    # -- local region bookkeeping -------------------------------------------------------------
    @property
    def n_loc(self):
        return len(self.chunks) * self.nqb

    def _maps(self):
        l_map = np.concatenate([np.arange(p * self.nqb, (p + 1) * self.nqb) for p, _, _ in self.chunks]).astype(np.int32)
        l_len = np.concatenate([ln for _, ln, _ in self.chunks]).astype(np.int32)
        l_id = np.concatenate([ids for _, _, ids in self.chunks]).astype(np.int64)
        return l_map, l_len, l_id

    def append_chunk(self, Kb, Vb, lens, ids):
        """Write a chunk's blocks ([H][nqb][B][d] bf16 bits) into the next ring position as the newest chunk."""
        assert len(self.chunks) <= self.w, "slide() before appending to a full local region"
        pos = self.n_appended % (self.w + 1)
        self.Kl[:, pos * self.nqb:(pos + 1) * self.nqb] = Kb
        self.Vl[:, pos * self.nqb:(pos + 1) * self.nqb] = Vb
        self.chunks.append((pos, np.asarray(lens, np.int32), np.asarray(ids, np.int64)))
        self.n_appended += 1
        self.stale_from = min(self.stale_from, self.n_loc - self.nqb)

    def rewrite_chunk(self, Kb, Vb):
        """Overwrite the newest chunk's blocks in place (the chunk's K/V change between the denoising passes
        of one chunk, Sec. 3.1); its pooled keys are recomputed by the next selection, the window's are kept."""
        pos = self.chunks[-1][0]
        self.Kl[:, pos * self.nqb:(pos + 1) * self.nqb] = Kb
        self.Vl[:, pos * self.nqb:(pos + 1) * self.nqb] = Vb
        self.stale_from = min(self.stale_from, self.n_loc - self.nqb)

    def set_persistent(self, Kp, Vp, lens, ids):
        """Seed the first C slots with given blocks ([H][C][B][d]); pooled keys by the oracle's own pooling."""
        C = Kp.shape[1]
        self.Kp[:, :C] = Kp
        self.Vp[:, :C] = Vp
        self.p_len[:, :C] = lens
        self.p_id[:, :C] = np.where(np.asarray(self.p_len[:, :C]) > 0, ids, -1)
        for h in range(self.H):
            for c in range(C):
                self.Kc_p[h, c] = orc.pool_block(self.Kp[h, c], int(self.p_len[h, c]))

    def set_summary(self, S_sum, S_cnt):
        """Seed the compressed-history sums/counts and the bf16 view in slot C (fp32 divide, round to nearest even)."""
        self.S_sum[...] = S_sum
        self.S_cnt[...] = S_cnt
        for h in range(self.H):
            nz = self.S_cnt[h] > 0
            mean = np.zeros((2, self.B, self.d), np.float32)
            mean[:, nz] = self.S_sum[h][:, nz] / self.S_cnt[h][nz].astype(np.float32)[None, :, None]
            bits = mean.view(np.uint32)
            bits = ((bits + np.uint32(0x7FFF) + ((bits >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)).astype(np.uint16)
            self.Kp[h, self.C][nz] = bits[0][nz]
            self.Vp[h, self.C][nz] = bits[1][nz]
            self.p_len[h, self.C] = int(nz.sum())

    def cfg(self, n_evict=0, pool_from=0):
        return orc.Cfg(H=self.H, d=self.d, B=self.B, Nq=self.Nq, n_loc=self.n_loc, n_loc_cap=self.cap, C=self.C,
                       k=self.k, scale=self.scale, n_sink=self.n_sink, causal=self.causal, n_evict=n_evict,
                       pool_from=pool_from)

    # -- the three calls ------------------------------------------------------------------------
    def select(self, Q, want_logits=False):
        l_map, l_len, _ = self._maps()
        cfg = self.cfg(pool_from=self.stale_from)
        self.Qc, self.sel, Z = orc.select(cfg, Q, self.Kl, l_len, l_map, self.Kc_l, want_logits)
        self.stale_from = self.n_loc
        return self.sel, Z

    def attention_rows(self, Q, rows_h, rows_t):
        l_map, l_len, _ = self._maps()
        return orc.attention_rows(self.cfg(), Q, self.Kp, self.Vp, self.p_len, self.Kl, self.Vl, l_len, l_map,
                                  self.sel, rows_h, rows_t)

    def attention(self, Q):
        l_map, l_len, _ = self._maps()
        return orc.attention(self.cfg(), Q, self.Kp, self.Vp, self.p_len, self.Kl, self.Vl, l_len, l_map, self.sel)

    def attention_mass(self, Q, qb_h=None, qb_i=None):
        """fp64 mass of every key block (slots 0..C, then the local blocks) from the given query blocks."""
        l_map, l_len, _ = self._maps()
        return orc.attention_mass(self.cfg(), Q, self.Kp, self.p_len, self.Kl, l_len, l_map, self.sel, qb_h, qb_i)

    def attention_bwd(self, Q, dO, row_mask=None, want_kv=True):
        """fp64 gradients (dQ, dKp, dVp, dKl, dVl) of the fine stage for the output gradient dO."""
        l_map, l_len, _ = self._maps()
        return orc.attention_bwd(self.cfg(), Q, self.Kp, self.Vp, self.p_len, self.Kl, self.Vl, l_len, l_map,
                                 self.sel, dO, row_mask, want_kv)

    def n_evict_now(self):
        return self.nqb if len(self.chunks) == self.w + 1 else 0

    def update(self):
        """Persistent update with E_t = the oldest chunk when the region is full; then slide the window."""
        l_map, l_len, l_id = self._maps()
        ne = self.n_evict_now()
        sc, src = orc.memory_update(self.cfg(n_evict=ne), self.Qc, self.Kc_l, self.Kp, self.Vp, self.Kc_p,
                                    self.p_len, self.p_id, self.S_sum, self.S_cnt, self.Kl, self.Vl, l_len, l_map,
                                    l_id)
        if ne:
            self.chunks.pop(0)
            self.stale_from = self.n_loc
        return sc, src

    def update_fine(self, Mt):
        """The same update ranked by fine attention mass Mt [H][C+1+n_loc][nqb] fp32; then slide the window."""
        l_map, l_len, l_id = self._maps()
        ne = self.n_evict_now()
        sc, src = orc.memory_update_fine(self.cfg(n_evict=ne), np.ascontiguousarray(Mt, np.float32), self.Kc_l,
                                         self.Kp, self.Vp, self.Kc_p, self.p_len, self.p_id, self.S_sum, self.S_cnt,
                                         self.Kl, self.Vl, l_len, l_map, l_id)
        if ne:
            self.chunks.pop(0)
            self.stale_from = self.n_loc
        return sc, src


def state_for_workload(w, layer=0, fold=True):
    """OracleState primed for a synth.Workload: warm workloads get their full window (global chunks
    0..w-1), C seeded persistent slots and the pre-filled summary; cold-start workloads get nothing.
    Returns (state, index of the first chunk to run)."""
    from harness import synth
    st = OracleState(w.H, w.d, w.B, w.Nq, w.window_chunks, w.C, w.k, np.float32(w.scale), fold=fold)
    if w.cold_start:
        return st, 0
    Kp, Vp = synth.persistent_init(w, layer)
    st.set_persistent(Kp, Vp, np.full((w.H, w.C), w.B, np.int32), -100 - np.arange(w.C)[None, :].repeat(w.H, 0))
    if w.summary_prefill:
        st.set_summary(*synth.summary_init(w, layer))
    lens = synth.block_lens(w)
    for g in range(w.window_chunks):
        _, K, V = synth.chunk_qkv(w, layer, g)
        st.append_chunk(synth.to_blocks(K, w.B), synth.to_blocks(V, w.B), lens, g * w.nqb + np.arange(w.nqb))
    return st, w.window_chunks


def run_chunk(st, w, layer, g, rows=None):
    """One layer-chunk step on global chunk g: append K/V, select, (attention rows), update. Returns dict."""
    from harness import synth
    Q, K, V = synth.chunk_qkv(w, layer, g)
    st.append_chunk(synth.to_blocks(K, w.B), synth.to_blocks(V, w.B), synth.block_lens(w), g * w.nqb + np.arange(w.nqb))
    sel, _ = st.select(Q)
    out = {"Q": Q, "sel": sel.copy(), "Qc": st.Qc.copy()}
    if rows is not None:
        out["O"], out["lse"] = st.attention_rows(Q, rows[0], rows[1]) if rows != "all" else st.attention(Q)
    out["scores"], out["slot_src"] = st.update()
    return out
