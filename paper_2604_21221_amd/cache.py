"""Device-resident KV memory M = P u L (Sec. 3.3, Eq. 2) and the caller side of one layer-chunk step.

PbsaCache owns the torch tensors (device memory only) and plays the caller of Alg. 1: it copies a
chunk's K/V into the local ring in block-major layout, then issues the three library calls
pbsa_select_blocks -> pbsa_attention_fwd -> pbsa_memory_update and slides the window.  All
arithmetic of the method happens inside libpbsa's kernels; this file only moves data and keeps the
ring bookkeeping (which physical slot holds which logical block).
"""
from __future__ import annotations

import torch

from . import pbsa


class PbsaCache:
    def __init__(self, H, d, B, Nq, window_chunks, C, k, scale, n_sink=0, causal=1, fold=True, device="cuda:0",
                 pass_logits=True, ring_chunks=None):
        self.H, self.d, self.B, self.Nq, self.C, self.k = H, d, B, Nq, C, k
        self.w, self.scale, self.n_sink, self.causal = window_chunks, float(scale), n_sink, causal
        self.nqb = -(-Nq // B)
        # ring positions: the window and the current chunk, or one more -- then the chunk that follows is written
        # to a position other than the one whose blocks the update of the current chunk still has to fold, and that
        # update's data movement can ride in the next selection call (defer_apply)
        self.ring = ring_chunks or window_chunks + 1
        assert self.ring >= window_chunks + 1
        self.cap = self.ring * self.nqb
        self._pending = None         # params of an update whose apply call has been deferred
        self.dev = torch.device(device)
        z = lambda *s, dt=torch.bfloat16: torch.zeros(*s, dtype=dt, device=self.dev)
        self.Kl, self.Vl = z(H, self.cap, B, d), z(H, self.cap, B, d)
        self.Kc_l = z(H, self.cap, d, dt=torch.float32)
        self.Kp, self.Vp = z(H, C + 1, B, d), z(H, C + 1, B, d)
        self.Kc_p = z(H, max(C, 1), d, dt=torch.float32)
        self.p_len = z(H, C + 1, dt=torch.int32)
        self.p_id = torch.full((H, max(C, 1)), -1, dtype=torch.int64, device=self.dev)
        self.S_sum = z(H, 2, B, d, dt=torch.float32) if fold else None
        self.S_cnt = z(H, B, dt=torch.int32) if fold else None
        self.Qc = z(H, self.nqb, d, dt=torch.float32)
        # coarse logits handed from the selection call to the update call (None: update recomputes them)
        self.Zl = z(H * self.nqb * self.cap, dt=torch.float32) if pass_logits else None
        self.sel = torch.full((H, self.nqb, max(k, 1)), -1, dtype=torch.int32, device=self.dev)
        self.slot_src = torch.full((H, max(C, 1)), -1, dtype=torch.int32, device=self.dev)
        self.scores = z(H, C + self.nqb, dt=torch.float32)
        full = pbsa.make_params(H, d, B, Nq, self.cap, self.cap, C, k, self.scale, n_sink, causal, n_evict=self.nqb)
        # with more slots than pbsa_memory_update maintains the cache can only be selected from and attended
        n_ws = pbsa.pbsa_workspace_bytes(full) if C <= pbsa.PBSA_MAX_C else 0
        self.ws = torch.empty(max(n_ws, 256), dtype=torch.uint8, device=self.dev)
        self.chunk_pos = []          # ring position of each chunk in the local region, oldest first
        self.chunk_ids = []          # global chunk index of each
        self.n_appended = 0
        self.stale_from = 0
        self._maps = {}
        self._arange64 = None
        lens = torch.full((self.nqb,), B, dtype=torch.int32)
        lens[-1] = Nq - (self.nqb - 1) * B
        self._chunk_lens = lens

    @property
    def n_loc(self):
        return len(self.chunk_pos) * self.nqb

    def _device_maps(self, want_ids=False):
        """l_map / l_len (and on request l_id) device tensors of the current ring arrangement.  The map
        and the lengths depend only on the ring positions and are cached per arrangement; ids of
        consecutive chunks are a window of one device-resident arange, so the steady state issues no
        copy and no kernel here."""
        key = tuple(self.chunk_pos)
        m = self._maps.get(key)
        if m is None:
            ar = torch.arange(self.nqb)
            l_map = torch.cat([p * self.nqb + ar for p in self.chunk_pos]).to(torch.int32)
            l_len = self._chunk_lens.repeat(len(self.chunk_pos))
            m = (l_map.to(self.dev), l_len.to(self.dev))
            self._maps[key] = m
        if not want_ids:
            return m[0], m[1], None
        ids = self.chunk_ids
        if ids[0] >= 0 and all(b == a + 1 for a, b in zip(ids, ids[1:])):
            lo, hi = ids[0] * self.nqb, (ids[-1] + 1) * self.nqb
            if self._arange64 is None or self._arange64.numel() < hi:
                self._arange64 = torch.arange(max(2 * hi, 64 * self.cap), dtype=torch.int64, device=self.dev)
            l_id = self._arange64[lo:hi]
        else:
            ar = torch.arange(self.nqb)
            l_id = torch.cat([g * self.nqb + ar for g in ids]).to(torch.int64).to(self.dev)
        return m[0], m[1], l_id

    def params(self, n_evict=0, pool_from=0, Q=None, O=None):
        qs = (Q.stride(0), Q.stride(1)) if Q is not None else None
        os_ = (O.stride(0), O.stride(1)) if O is not None else None
        return pbsa.make_params(self.H, self.d, self.B, self.Nq, self.n_loc, self.cap, self.C, self.k, self.scale,
                                self.n_sink, self.causal, n_evict, pool_from, qs, os_)

    # -- state seeding (data movement + the library's own pooling kernel) ----------------------------
    def set_persistent(self, Kp, Vp, lens, ids):
        """Install blocks ([H][c][B][d] bf16) in the first slots; pooled keys come from pbsa_pool_blocks."""
        c = Kp.shape[1]
        self.Kp[:, :c] = Kp
        self.Vp[:, :c] = Vp
        self.p_len[:, :c] = lens
        self.p_id[:, :c] = torch.where(self.p_len[:, :c] > 0, ids.to(self.dev), torch.full_like(ids, -1).to(self.dev))
        flat_len = self.p_len[:, :c].contiguous().view(-1)
        X = self.Kp[:, :c].contiguous()
        out = torch.empty(self.H * c, self.d, dtype=torch.float32, device=self.dev)
        pbsa.pbsa_pool_blocks(self.params(), X, flat_len, self.H * c, out)
        self.Kc_p[:, :c] = out.view(self.H, c, self.d)

    def set_summary(self, S_sum, S_cnt):
        """Install a pre-filled compressed-history state: sums and counts; pbsa_summary_view derives the bf16 view
        in slot C and its length."""
        self.S_sum.copy_(S_sum)
        self.S_cnt.copy_(S_cnt)
        pbsa.pbsa_summary_view(self.params(), self.S_sum, self.S_cnt, self.Kp, self.Vp, self.p_len)

    def append_chunk(self, K, V, chunk_id):
        """Copy a chunk's K/V ([H][Nq][d] bf16, token-major) into the next ring position, block-major."""
        assert len(self.chunk_pos) <= self.w, "update() slides the window before the next append"
        pos = self.n_appended % self.ring
        for dst, src in ((self.Kl, K), (self.Vl, V)):
            view = dst[:, pos * self.nqb:(pos + 1) * self.nqb].view(self.H, self.nqb * self.B, self.d)
            view[:, :self.Nq] = src
            if self.nqb * self.B > self.Nq:
                view[:, self.Nq:] = 0
        self.chunk_pos.append(pos)
        self.chunk_ids.append(chunk_id)
        self.n_appended += 1
        self.stale_from = min(self.stale_from, self.n_loc - self.nqb)

    def rewrite_chunk(self, K=None, V=None):
        """Between the denoising passes of one chunk (Sec. 3.1: each chunk is denoised in T passes over the
        same cache) only the newest chunk's own K/V change: overwrite them in place ([H][Nq][d] bf16), or
        with no arguments just note that the producer has.  The next selection then pools the chunk's
        blocks again; the pooled keys of the window stay cached."""
        assert self.chunk_pos, "no chunk to rewrite"
        pos = self.chunk_pos[-1]
        for dst, src in ((self.Kl, K), (self.Vl, V)):
            if src is not None:
                dst[:, pos * self.nqb:(pos + 1) * self.nqb].view(self.H, self.nqb * self.B, self.d)[:, :self.Nq] = src
        self.stale_from = min(self.stale_from, self.n_loc - self.nqb)

    def adopt_chunk(self, chunk_id):
        """Declare the next ring position to hold chunk `chunk_id` whose K/V the producer has already
        written there in block-major layout (zero-copy append)."""
        assert len(self.chunk_pos) <= self.w, "update() slides the window before the next append"
        self.chunk_pos.append(self.n_appended % self.ring)
        self.chunk_ids.append(chunk_id)
        self.n_appended += 1
        self.stale_from = min(self.stale_from, self.n_loc - self.nqb)

    # -- the three calls ---------------------------------------------------------------------------
    def select(self, Q):
        l_map, l_len, _ = self._device_maps()
        p = self.params(pool_from=self.stale_from, Q=Q)
        if self._pending is not None:            # with the data movement of the previous chunk's update in its pooling launch
            pbsa.pbsa_select_blocks_apply(p, Q, self.Kl, l_len, l_map, self.Kc_l, self.Qc, self.sel, self.Zl, self._pending,
                                          self.Kp, self.Vp, self.p_len, self.S_sum, self.S_cnt, self.Vl, self.ws)
            self._pending = None
        else:
            pbsa.pbsa_select_blocks(p, Q, self.Kl, l_len, l_map, self.Kc_l, self.Qc, self.sel, self.Zl)
        self.stale_from = self.n_loc
        return self.sel

    def attention(self, Q, O=None, lse=None):
        if O is None:
            O = torch.empty_like(Q)
        l_map, l_len, _ = self._device_maps()
        p = self.params(Q=Q, O=O)
        pbsa.pbsa_attention_fwd(p, Q, self.Kp, self.Vp, self.p_len, self.Kl, self.Vl, l_len, l_map, self.sel, O, lse)
        return O

    def _no_pending(self):
        # a deferred apply still owns the workspace and the slot lengths it will commit
        assert self._pending is None, "a deferred update is pending: select() or flush() completes it first"

    def n_evict_now(self):
        return self.nqb if len(self.chunk_pos) == self.w + 1 else 0

    def update(self, static_scratch=False):
        """pbsa_memory_update; static_scratch: through pbsa_memory_update_static (the library's own scratch, no workspace)."""
        self._no_pending()
        l_map, l_len, l_id = self._device_maps(want_ids=True)
        ne = self.n_evict_now()
        p = self.params(n_evict=ne)
        if static_scratch:
            pbsa.pbsa_memory_update_static(p, self.Qc, self.Kc_l, self.Zl, self.Kp, self.Vp, self.Kc_p, self.p_len, self.p_id,
                                           self.S_sum, self.S_cnt, self.Kl, self.Vl, l_len, l_map, l_id, self.scores,
                                           self.slot_src)
        else:
            pbsa.pbsa_memory_update(p, self.Qc, self.Kc_l, self.Zl, self.Kp, self.Vp, self.Kc_p, self.p_len, self.p_id,
                                    self.S_sum, self.S_cnt, self.Kl, self.Vl, l_len, l_map, l_id, self.scores,
                                    self.slot_src, self.ws)
        if ne:
            self.chunk_pos.pop(0)
            self.chunk_ids.pop(0)
            self.stale_from = self.n_loc
        return ne

    # -- the variant that ranks the persistent set by the attention actually paid --------------------
    def attention_mass(self, Q, lse, Mt=None):
        """Mass of every key block (slots 0..C, then the local blocks) from every query block:
        [H][C+1+n_loc][nqb rounded up to 4] fp32, from the log-sum-exp that attention() wrote."""
        if Mt is None:
            Mt = self._mass_buffer()
        l_map, l_len, _ = self._device_maps()
        pbsa.pbsa_attention_mass(self.params(Q=Q), Q, self.Kp, self.p_len, self.Kl, l_len, l_map, self.sel, lse, Mt)
        return Mt

    def _mass_buffer(self):
        n_u, pad = self.C + 1 + self.n_loc, (self.nqb + 3) & ~3
        if getattr(self, "_Mt", None) is None:
            self._Mt = torch.zeros(self.H * (self.C + 1 + self.cap) * pad, dtype=torch.float32, device=self.dev)
        return self._Mt[:self.H * n_u * pad].view(self.H, n_u, pad)

    def attention_with_mass(self, Q, O=None, lse=None):
        """Attention and the mass matrix in one call (the attention kernel records what the mass needs).
        Returns (O, Mt)."""
        if O is None:
            O = torch.empty_like(Q)
        if lse is None:
            if getattr(self, "_lse", None) is None:
                self._lse = torch.empty(self.H, self.Nq, dtype=torch.float32, device=self.dev)
            lse = self._lse
        if getattr(self, "_mass_ws", None) is None:
            full = pbsa.make_params(self.H, self.d, self.B, self.Nq, self.cap, self.cap, self.C, self.k, self.scale)
            self._mass_ws = torch.empty(pbsa.pbsa_mass_workspace_bytes(full), dtype=torch.uint8, device=self.dev)
        Mt = self._mass_buffer()
        l_map, l_len, _ = self._device_maps()
        p = self.params(Q=Q, O=O)
        pbsa.pbsa_attention_fwd_mass(p, Q, self.Kp, self.Vp, self.p_len, self.Kl, self.Vl, l_len, l_map, self.sel, O,
                                     lse, Mt, self._mass_ws)
        return O, Mt

    def update_fine(self, Mt):
        self._no_pending()
        l_map, l_len, l_id = self._device_maps(want_ids=True)
        ne = self.n_evict_now()
        pbsa.pbsa_memory_update_fine(self.params(n_evict=ne), Mt, self.Kc_l, self.Kp, self.Vp, self.Kc_p, self.p_len,
                                     self.p_id, self.S_sum, self.S_cnt, self.Kl, self.Vl, l_len, l_map, l_id,
                                     self.scores, self.slot_src, self.ws)
        if ne:
            self.chunk_pos.pop(0)
            self.chunk_ids.pop(0)
            self.stale_from = self.n_loc
        return ne

    def step_fine(self, Q, K, V, chunk_id, O=None, lse=None):
        """The step with the fine-mass score: append, select, attend (recording the mass), update."""
        self.append_chunk(K, V, chunk_id)
        self.select(Q)
        O, Mt = self.attention_with_mass(Q, O, lse)
        self.update_fine(Mt)
        return O

    def attention_bwd(self, Q, O, dO, lse, grads=None):
        """Gradients of attention(Q) for the output gradient dO (bf16, O's strides): returns the dict of fp32
        tensors dQ [H][Nq][d], dKp, dVp [H][C+1][B][d], dKl, dVl [H][cap][B][d] (allocated unless given)."""
        if grads is None:
            z = lambda *s: torch.zeros(*s, dtype=torch.float32, device=self.dev)
            grads = dict(dQ=z(self.H, self.Nq, self.d), dKp=z(self.H, self.C + 1, self.B, self.d),
                         dVp=z(self.H, self.C + 1, self.B, self.d), dKl=z(self.H, self.cap, self.B, self.d),
                         dVl=z(self.H, self.cap, self.B, self.d))
        p = self.params(Q=Q, O=O)
        if getattr(self, "_bwd_ws", None) is None:
            self._bwd_ws = torch.empty(pbsa.pbsa_bwd_workspace_bytes(p), dtype=torch.uint8, device=self.dev)
        l_map, l_len, _ = self._device_maps()
        pbsa.pbsa_attention_bwd(p, Q, self.Kp, self.Vp, self.p_len, self.Kl, self.Vl, l_len, l_map, self.sel, O, dO, lse,
                                grads["dQ"], grads["dKp"], grads["dVp"], grads["dKl"], grads["dVl"], self._bwd_ws)
        return grads

    def update_plan(self):
        """pbsa_memory_update_plan: the update's decisions alone (scores, retention, slot sources); update_apply()
        moves the data."""
        self._no_pending()
        l_map, l_len, l_id = self._device_maps(want_ids=True)
        self._plan_p = self.params(n_evict=self.n_evict_now())
        pbsa.pbsa_memory_update_plan(self._plan_p, self.Qc, self.Kc_l, self.Zl, self.Kc_p, self.p_len, self.p_id,
                                     self.S_cnt, l_len, l_map, l_id, self.scores, self.slot_src, self.ws)

    def update_apply(self):
        """After attention_with_plan() or update_plan(): fold, promote, commit; slides the window."""
        self._no_pending()
        pbsa.pbsa_memory_update_apply(self._plan_p, self.Kp, self.Vp, self.p_len, self.S_sum, self.S_cnt, self.Kl, self.Vl,
                                      self.ws)
        ne = self._plan_p.n_evict
        if ne:
            self.chunk_pos.pop(0)
            self.chunk_ids.pop(0)
            self.stale_from = self.n_loc
        return ne

    def attention_with_plan(self, Q, O=None, lse=None):
        """pbsa_attention_fwd_plan: the attention of the chunk and, by extra workgroups of the same launch, the
        decisions of the update that follows it (needs the logits the selection call left).  update_apply()
        completes the update."""
        self._no_pending()
        if O is None:
            O = torch.empty_like(Q)
        l_map, l_len, l_id = self._device_maps(want_ids=True)
        self._plan_p = self.params(n_evict=self.n_evict_now(), Q=Q, O=O)
        pbsa.pbsa_attention_fwd_plan(self._plan_p, Q, self.Kp, self.Vp, self.p_len, self.Kl, self.Vl, l_len, l_map, self.sel,
                                     O, lse, self.Qc, self.Kc_l, self.Zl, self.Kc_p, self.p_id, self.S_cnt, l_id,
                                     self.scores, self.slot_src, self.ws)
        return O

    def step_fused(self, Q, K=None, V=None, chunk_id=None, O=None, lse=None):
        """The step as two launches after the selection: attention with the update's decisions, then fold /
        promote.  K = V = None: the chunk has been adopted already."""
        if K is not None:
            self.append_chunk(K, V, chunk_id)
        self.select(Q)
        O = self.attention_with_plan(Q, O, lse)
        self.update_apply()
        return O

    def defer_apply(self):
        """After attention_with_plan(): slides the window now and leaves fold / promote to the next select() call, in
        whose pooling launch they ride (or to flush()).  Needs the spare ring position (ring_chunks = window + 2)."""
        assert self.ring >= self.w + 2, "the next chunk would overwrite the blocks that are still to be folded"
        assert self._pending is None
        self._pending = self._plan_p
        ne = self._plan_p.n_evict
        if ne:
            self.chunk_pos.pop(0)
            self.chunk_ids.pop(0)
            self.stale_from = self.n_loc
        return ne

    def flush(self):
        """Completes a deferred update now (pbsa_memory_update_apply)."""
        if self._pending is not None:
            pbsa.pbsa_memory_update_apply(self._pending, self.Kp, self.Vp, self.p_len, self.S_sum, self.S_cnt, self.Kl,
                                          self.Vl, self.ws)
            self._pending = None

    def step_chained(self, Q, K=None, V=None, chunk_id=None, O=None, lse=None):
        """Two library calls per step: selection (carrying the previous step's fold / promote), attention (carrying
        this step's decisions).  flush() after the last step.  K = V = None: the chunk has been adopted already."""
        if K is not None:
            self.append_chunk(K, V, chunk_id)
        self.select(Q)
        O = self.attention_with_plan(Q, O, lse)
        self.defer_apply()
        return O

    def step(self, Q, K, V, chunk_id, O=None, lse=None):
        """One layer-chunk step: append the chunk, select, attend, update (all enqueued, no sync)."""
        self.append_chunk(K, V, chunk_id)
        self.select(Q)
        O = self.attention(Q, O, lse)
        self.update()
        return O
