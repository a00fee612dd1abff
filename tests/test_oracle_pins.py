"""Pins of the CPU oracle against what the paper and the mathematics fix (no GPU needed).

The paper prints no worked numeric example for any PBSA step, so every pin below is a closed
form, an invariant, a special case that reduces to a textbook routine coded here independently
in numpy fp64, or brute force on tiny inputs.
"""
import math

import numpy as np
import pytest

from oracle.rollout import OracleState
from harness import synth


def bf(x):
    return synth.to_bf16_bits(x)


def f32(bits):
    return synth.bf16_bits_to_f32(bits)


def rnd(key, *shape):
    return synth.normals(synth.stream_key(1234, "misc", key), int(np.prod(shape))).reshape(shape)


def make_state(seed=0, H=2, d=16, B=8, Nq=20, w=2, C=3, k=2, n_sink=0, causal=1, p_lens=None, fill_chunks=None,
               fold=True):
    """Small random problem: window of `w` chunks + the current chunk, C persistent slots (ragged lens)."""
    st = OracleState(H, d, B, Nq, w, C, k, 1.0 / math.sqrt(d), n_sink=n_sink, causal=causal, fold=fold)
    nqb = st.nqb
    lens = np.full(nqb, B, np.int32)
    lens[-1] = Nq - (nqb - 1) * B
    if C > 0:
        Kp = bf(rnd(seed * 100 + 1, H, C, B, d))
        Vp = bf(rnd(seed * 100 + 2, H, C, B, d))
        pl = np.full((H, C), B, np.int32) if p_lens is None else np.asarray(p_lens, np.int32)
        st.set_persistent(Kp, Vp, pl, -100 - np.arange(C)[None, :].repeat(H, 0))
    n_chunks = (w + 1) if fill_chunks is None else fill_chunks
    Q = None
    for g in range(n_chunks):
        K = bf(rnd(seed * 100 + 10 + 3 * g, H, Nq, d))
        V = bf(rnd(seed * 100 + 11 + 3 * g, H, Nq, d))
        Q = bf(rnd(seed * 100 + 12 + 3 * g, H, Nq, d))
        st.append_chunk(synth.to_blocks(K, B), synth.to_blocks(V, B), lens, g * nqb + np.arange(nqb))
    return st, Q


# ------------------------------------------------------------------------------------------------
# independent numpy references
# ------------------------------------------------------------------------------------------------
def ref_pooled(st, Q):
    """fp64 pooled representatives: Qc [H][nqb][d], Kc [H][n_loc][d] (logical order)."""
    l_map, l_len, _ = st._maps()
    Qf = f32(Q).astype(np.float64)
    Qc = np.stack([[Qf[h, i * st.B:min((i + 1) * st.B, st.Nq)].mean(0) for i in range(st.nqb)] for h in range(st.H)])
    Kf = f32(st.Kl).astype(np.float64)
    Kc = np.stack([[Kf[h, l_map[l], :l_len[l]].mean(0) for l in range(st.n_loc)] for h in range(st.H)])
    return Qc, Kc


def ref_dense_attention(st, Q, sel):
    """softmax(Q K^T * scale + M) V with the mask matrix of Eq. 5 written out explicitly (fp64)."""
    l_map, l_len, _ = st._maps()
    out = np.zeros((st.H, st.Nq, st.d))
    wsum = np.zeros((st.H, st.Nq))
    for h in range(st.H):
        keys, vals, owner = [], [], []          # owner: -1 persistent, else logical local block
        for s in range(st.C + 1):
            n = st.p_len[h, s]
            keys.append(f32(st.Kp[h, s, :n])); vals.append(f32(st.Vp[h, s, :n])); owner += [-1] * n
        for l in range(st.n_loc):
            n = l_len[l]
            keys.append(f32(st.Kl[h, l_map[l], :n])); vals.append(f32(st.Vl[h, l_map[l], :n])); owner += [l] * n
        Kc = np.concatenate(keys).astype(np.float64)
        Vc = np.concatenate(vals).astype(np.float64)
        owner = np.array(owner)
        M = np.full((st.Nq, len(owner)), -np.inf)
        for t in range(st.Nq):
            vis = set(int(x) for x in sel[h, t // st.B] if x >= 0)
            M[t, (owner < 0) | np.isin(owner, list(vis))] = 0.0
        S = f32(Q[h]).astype(np.float64) @ Kc.T * st.scale + M
        P = np.exp(S - S.max(1, keepdims=True))
        P /= P.sum(1, keepdims=True)
        out[h] = P @ Vc
        wsum[h] = P.sum(1)
    return out, wsum


# ------------------------------------------------------------------------------------------------
# pinned exp
# ------------------------------------------------------------------------------------------------
def test_pexp_matches_exp(oracle):
    xs = np.concatenate([np.linspace(-64, 0, 4001), -np.logspace(-8, 1.8, 500)]).astype(np.float32)
    worst = 0.0
    for x in xs:
        got, want = oracle.pexp(float(x)), math.exp(float(x))
        worst = max(worst, abs(got - want) / want)
    assert worst < 4 * 2.0 ** -24          # a few ulp
    assert oracle.pexp(0.0) == 1.0
    assert oracle.pexp(-64.5) == 0.0 and oracle.pexp(-1e30) == 0.0
    ys = [oracle.pexp(float(x)) for x in np.linspace(-20, 0, 2001, dtype=np.float32)]
    assert all(b >= a for a, b in zip(ys, ys[1:]))


# ------------------------------------------------------------------------------------------------
# pooling + selection (Eq. 6, 10, 11)
# ------------------------------------------------------------------------------------------------
def test_pool_is_mean_of_valid_tokens(oracle):
    x = rnd(7, 8, 16) * 3
    bits = bf(x)
    for length in (1, 5, 8):
        got = oracle.pool_block(bits, length)
        np.testing.assert_allclose(got, f32(bits[:length]).astype(np.float64).mean(0), rtol=0, atol=2e-6)
    # padding rows are never trusted: garbage beyond len does not change the result
    junk = bits.copy(); junk[5:] = bf(np.full((3, 16), 1e6))
    assert np.array_equal(oracle.pool_block(junk, 5), oracle.pool_block(bits, 5))


@pytest.mark.parametrize("causal", [0, 1])
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_select_is_bruteforce_topk(oracle, seed, causal):
    st, Q = make_state(seed, H=3, d=16, B=8, Nq=28, w=2, C=1, k=3, causal=causal)
    sel, Z = st.select(Q, want_logits=True)
    Qc, Kc = ref_pooled(st, Q)
    n_win = st.n_loc - st.nqb
    for h in range(st.H):
        for i in range(st.nqb):
            nvis = n_win + i + 1 if causal else st.n_loc
            z = Kc[h, :nvis] @ Qc[h, i] * st.scale
            np.testing.assert_allclose(Z[h, i, :nvis], z, rtol=0, atol=1e-5)
            assert np.all(np.isneginf(Z[h, i, nvis:]))
            order = sorted(range(nvis), key=lambda l: (-z[l], l))           # full sort of (-z, l)
            want = sorted(order[:st.k])
            assert [int(x) for x in sel[h, i] if x >= 0] == want
            # Eq. 10-11 literally: top-k of the softmax probabilities picks the same set
            p = np.exp(z - z.max()); p /= p.sum()
            assert sorted(np.argsort(-p, kind="stable")[:st.k].tolist()) == want
            assert sel[h, i].max() <= (n_win + i if causal else st.n_loc - 1)


def test_select_ties_go_to_lowest_index_and_respect_visibility(oracle):
    st, Q = make_state(3, H=1, d=16, B=8, Nq=32, w=1, C=0, k=6)
    st.Kl[...] = st.Kl[0, 0, 0]            # every key token identical -> every block logit identical
    st.stale_from = 0
    sel, _ = st.select(Q)
    n_win = st.n_loc - st.nqb               # 4 window blocks, query block i sees n_win + i + 1
    for i in range(st.nqb):
        nvis = n_win + i + 1
        want = list(range(min(st.k, nvis))) + [-1] * max(0, st.k - nvis)
        assert sel[0, i].tolist() == want


def test_select_boosted_block_and_permutation(oracle):
    st, Q = make_state(4, H=2, d=16, B=8, Nq=24, w=2, C=0, k=2, causal=0)
    sel0, _ = st.select(Q)
    Qc, _ = ref_pooled(st, Q)
    # make local block 5 strongly aligned with every pooled query of head 0 -> selected by all rows
    direction = Qc[0].mean(0); direction /= np.linalg.norm(direction)
    for i in range(st.nqb):
        assert Qc[0, i] @ direction > 0
    l_map, _, _ = st._maps()
    st.Kl[0, l_map[5]] = bf(np.tile(60.0 * direction, (st.B, 1)))
    st.stale_from = 0
    sel1, _ = st.select(Q)
    assert all(5 in sel1[0, i] for i in range(st.nqb))
    assert np.array_equal(sel1[1], sel0[1])                      # heads are independent
    # reversing the order of the local blocks maps every set through the same permutation
    n = st.n_loc
    perm = l_map[::-1].copy()
    st2, _ = make_state(4, H=2, d=16, B=8, Nq=24, w=2, C=0, k=2, causal=0)
    st2.Kl[...] = st.Kl
    import oracle.pbsa_oracle as orc
    _, l_len, _ = st._maps()
    Kc = np.zeros_like(st.Kc_l)
    _, selp, _ = orc.select(st.cfg(), Q, st.Kl, l_len[::-1].copy(), perm, Kc)
    for h in range(st.H):
        for i in range(st.nqb):
            assert sorted(n - 1 - selp[h, i]) == sel1[h, i].tolist()


# ------------------------------------------------------------------------------------------------
# attention (Eq. 3-5)
# ------------------------------------------------------------------------------------------------
def test_attention_all_selected_is_dense_block_causal(oracle):
    st, Q = make_state(5, H=2, d=16, B=8, Nq=20, w=2, C=3, k=99, p_lens=[[8, 3, 0], [5, 8, 8]])
    st.k = st.n_loc
    sel, _ = st.select(Q)
    n_win = st.n_loc - st.nqb
    for i in range(st.nqb):                  # k >= n_vis: everything visible is selected
        assert [x for x in sel[0, i] if x >= 0] == list(range(n_win + i + 1))
    O, lse = st.attention(Q)
    ref, wsum = ref_dense_attention(st, Q, sel)
    np.testing.assert_allclose(O, ref, rtol=0, atol=1e-12)
    np.testing.assert_allclose(wsum, 1.0, atol=1e-12)


def test_attention_noncausal_no_memory_is_plain_attention(oracle):
    st, Q = make_state(6, H=1, d=16, B=8, Nq=24, w=1, C=0, k=6, causal=0)
    st.select(Q)
    O, lse = st.attention(Q)
    l_map, l_len, _ = st._maps()
    K = np.concatenate([f32(st.Kl[0, l_map[l], :l_len[l]]) for l in range(st.n_loc)]).astype(np.float64)
    V = np.concatenate([f32(st.Vl[0, l_map[l], :l_len[l]]) for l in range(st.n_loc)]).astype(np.float64)
    S = f32(Q[0]).astype(np.float64) @ K.T * st.scale
    P = np.exp(S - S.max(1, keepdims=True)); Z = P.sum(1, keepdims=True)
    np.testing.assert_allclose(O[0], (P / Z) @ V, rtol=0, atol=1e-12)
    np.testing.assert_allclose(lse[0], S.max(1) + np.log(Z[:, 0]), rtol=0, atol=1e-12)


def test_attention_sparse_mask_semantics(oracle):
    st, Q = make_state(7, H=2, d=16, B=8, Nq=20, w=2, C=2, k=2, p_lens=[[8, 6], [8, 8]])
    sel, _ = st.select(Q)
    O, _ = st.attention(Q)
    ref, _ = ref_dense_attention(st, Q, sel)
    np.testing.assert_allclose(O, ref, rtol=0, atol=1e-12)
    l_map, l_len, _ = st._maps()
    # convexity: every output row lies inside the per-dimension range of the values it can see
    for h in range(st.H):
        for t in range(st.Nq):
            vs = [f32(st.Vp[h, s, :st.p_len[h, s]]) for s in range(st.C + 1)]
            vs += [f32(st.Vl[h, l_map[l], :l_len[l]]) for l in sel[h, t // st.B] if l >= 0]
            vs = np.concatenate(vs)
            assert np.all(O[h, t] <= vs.max(0) + 1e-12) and np.all(O[h, t] >= vs.min(0) - 1e-12)
    # a local block nobody selected does not influence any output, bit for bit
    unused = sorted(set(range(st.n_loc)) - set(int(x) for x in sel[0].ravel() if x >= 0))
    assert unused
    Kl_saved, Vl_saved = st.Kl.copy(), st.Vl.copy()
    st.Kl[0, l_map[unused[0]]] = bf(rnd(99, st.B, st.d) * 5)
    st.Vl[0, l_map[unused[0]]] = bf(rnd(98, st.B, st.d) * 5)
    O2, _ = st.attention(Q)
    assert np.array_equal(O2, O)
    st.Kl[...] = Kl_saved; st.Vl[...] = Vl_saved
    # padding rows of ragged blocks are masked: garbage there changes nothing
    st.Kp[0, 1, 6:] = bf(np.full((2, st.d), 50.0)); st.Vp[0, 1, 6:] = bf(np.full((2, st.d), 50.0))
    tail = l_len[-1]
    st.Kl[:, l_map[-1], tail:] = bf(np.full((st.B - tail, st.d), 50.0))
    O3, _ = st.attention(Q)
    assert np.array_equal(O3, O)
    # persistent blocks are visible to every query row (zero block of Eq. 5)
    st.Vp[0, 0] = bf(f32(st.Vp[0, 0]) + 1.0)
    O4, _ = st.attention(Q)
    assert np.all(np.abs(O4[0] - O[0]).max(1) > 0) and np.array_equal(O4[1], O[1])


def test_attention_empty_memory_and_no_keys(oracle):
    st, Q = make_state(8, H=1, d=16, B=8, Nq=16, w=0, C=2, k=0, p_lens=[[0, 0]])
    st.select(Q)
    O, lse = st.attention(Q)
    assert np.all(O == 0) and np.all(np.isneginf(lse))


# ------------------------------------------------------------------------------------------------
# persistence scores (Eq. 7-8)
# ------------------------------------------------------------------------------------------------
def test_scores_closed_forms(oracle):
    st, Q = make_state(9, H=2, d=16, B=8, Nq=28, w=2, C=3, k=2, p_lens=[[8, 0, 4], [8, 8, 8]])
    st.select(Q)
    l_map, _, _ = st._maps()
    s_p, s_l = oracle.scores(st.cfg(), st.Qc, st.Kc_l, l_map, st.Kc_p, st.p_len)
    # a row-stochastic matrix averaged over rows sums to one; empty slots score 0
    np.testing.assert_allclose(s_p.sum(1) + s_l.sum(1), 1.0, atol=2e-6)
    assert s_p[0, 1] == 0.0
    # fp64 shadow from independently pooled representatives
    Qc, Kc = ref_pooled(st, Q)
    for h in range(st.H):
        occ = [s for s in range(st.C) if st.p_len[h, s] > 0]
        Kp_c = np.stack([f32(st.Kp[h, s, :st.p_len[h, s]]).astype(np.float64).mean(0) for s in occ])
        U = np.concatenate([Kp_c, Kc[h]])
        Zm = Qc[h] @ U.T * st.scale
        A = np.exp(Zm - Zm.max(1, keepdims=True)); A /= A.sum(1, keepdims=True)
        s = A.mean(0)
        np.testing.assert_allclose(s_p[h, occ], s[:len(occ)], rtol=0, atol=1e-6)
        np.testing.assert_allclose(s_l[h], s[len(occ):], rtol=0, atol=1e-6)
    # identical representatives everywhere -> uniform 1/|U|
    st.Kc_l[...] = st.Kc_l[0, 0]
    st.Kc_p[...] = st.Kc_l[0, 0]
    s_p, s_l = oracle.scores(st.cfg(), st.Qc, st.Kc_l, l_map, st.Kc_p, st.p_len)
    nU = [2 + st.n_loc, 3 + st.n_loc]
    for h in range(st.H):
        np.testing.assert_allclose(s_l[h], 1.0 / nU[h], rtol=1e-6)


# ------------------------------------------------------------------------------------------------
# retention, slots, summary (Eq. 9 + compressed history)
# ------------------------------------------------------------------------------------------------
def run_update(st):
    before = dict(Kp=st.Kp.copy(), Vp=st.Vp.copy(), p_len=st.p_len.copy(), p_id=st.p_id.copy(),
                  Kc_p=st.Kc_p.copy(), S_sum=None if st.S_sum is None else st.S_sum.copy(),
                  S_cnt=None if st.S_cnt is None else st.S_cnt.copy(), Kl=st.Kl.copy(), Vl=st.Vl.copy())
    before["maps"] = st._maps()
    before["n_evict"] = st.n_evict_now()
    sc, src = st.update()
    return before, sc, src


@pytest.mark.parametrize("seed,n_sink", [(10, 0), (11, 1), (12, 2)])
def test_retention_is_bruteforce_topc(oracle, seed, n_sink):
    st, Q = make_state(seed, H=3, d=16, B=8, Nq=28, w=2, C=4, k=2, n_sink=n_sink,
                       p_lens=[[8, 8, 5, 8], [8, 0, 8, 8], [8, 8, 8, 0]])
    st.select(Q)
    b, sc, src = run_update(st)
    l_map, l_len, l_id = b["maps"]
    ne, C = b["n_evict"], st.C
    assert ne == st.nqb
    for h in range(st.H):
        cands = [("p", s) for s in range(n_sink, C) if b["p_len"][h, s] > 0] + [("e", e) for e in range(ne)]
        val = [sc[h, s] if kind == "p" else sc[h, C + s] for kind, s in cands]
        order = sorted(range(len(cands)), key=lambda a: (-val[a], a))
        winners = set(order[:C - n_sink])
        # sinks never move
        for s in range(n_sink):
            assert src[h, s] == -1 and st.p_id[h, s] == b["p_id"][h, s]
            assert np.array_equal(st.Kp[h, s], b["Kp"][h, s])
        # winning occupants keep their slot, losers vacate, newcomers fill ascending
        free = [s for s in range(n_sink, C) if b["p_len"][h, s] == 0]
        free += [cands[a][1] for a in range(len(cands)) if cands[a][0] == "p" and a not in winners]
        free.sort()
        new = sorted(cands[a][1] for a in winners if cands[a][0] == "e")
        want_src = np.full(C, -1)
        for s, e in zip(free, new):
            want_src[s] = e
        assert src[h].tolist() == want_src.tolist()
        for s in range(n_sink, C):
            if want_src[s] >= 0:
                e = want_src[s]
                assert np.array_equal(st.Kp[h, s], b["Kl"][h, l_map[e]]) and np.array_equal(st.Vp[h, s], b["Vl"][h, l_map[e]])
                assert st.p_len[h, s] == l_len[e] and st.p_id[h, s] == l_id[e]
                assert np.array_equal(st.Kc_p[h, s], st.Kc_l[h, l_map[e]])
            elif b["p_len"][h, s] > 0:
                assert np.array_equal(st.Kp[h, s], b["Kp"][h, s]) and st.p_id[h, s] == b["p_id"][h, s]
        kept_ids = set(int(x) for x in st.p_id[h] if x != -1)
        assert kept_ids <= set(int(x) for x in b["p_id"][h]) | set(int(x) for x in l_id[:ne])
        # summary = position-wise mean of every loser (fp64 batch mean), counts integer-exact
        losers = [cands[a] for a in range(len(cands)) if a not in winners]
        cnt = np.zeros(st.B, np.int64); ks = np.zeros((st.B, st.d)); vs = np.zeros((st.B, st.d))
        for kind, s in losers:
            if kind == "p":
                n = b["p_len"][h, s]; kb, vb = b["Kp"][h, s], b["Vp"][h, s]
            else:
                n = l_len[s]; kb, vb = b["Kl"][h, l_map[s]], b["Vl"][h, l_map[s]]
            cnt[:n] += 1; ks[:n] += f32(kb[:n]); vs[:n] += f32(vb[:n])
        assert st.S_cnt[h].tolist() == cnt.tolist() and st.S_cnt[h].sum() == sum(
            (b["p_len"][h, s] if kind == "p" else l_len[s]) for kind, s in losers)
        nz = cnt > 0
        assert st.p_len[h, C] == nz.sum()
        np.testing.assert_allclose(st.S_sum[h, 0][nz] / st.S_cnt[h][nz, None], ks[nz] / cnt[nz, None], atol=1e-5)
        np.testing.assert_allclose(f32(st.Kp[h, C][nz]), ks[nz] / cnt[nz, None], rtol=2 ** -8, atol=1e-6)
        np.testing.assert_allclose(f32(st.Vp[h, C][nz]), vs[nz] / cnt[nz, None], rtol=2 ** -8, atol=1e-6)


def test_update_without_eviction_is_noop_and_room_for_all(oracle):
    st, Q = make_state(13, H=2, d=16, B=8, Nq=24, w=2, C=3, k=2, fill_chunks=2, p_lens=[[8, 8, 0], [0, 0, 0]])
    st.select(Q)
    b, sc, src = run_update(st)
    assert b["n_evict"] == 0 and np.all(src == -1)
    for name in ("Kp", "Vp", "p_len", "p_id", "S_sum", "S_cnt"):
        assert np.array_equal(getattr(st, name), b[name])
    # more places than candidates: nothing is dropped, summary untouched
    st2, Q2 = make_state(14, H=1, d=16, B=8, Nq=16, w=1, C=6, k=1, p_lens=[[8, 8, 0, 0, 0, 0]])
    st2.select(Q2)
    b2, _, src2 = run_update(st2)
    assert src2[0].tolist() == [-1, -1, 0, 1, -1, -1]
    assert st2.S_cnt.sum() == 0 and st2.p_len[0, 6] == 0 and st2.p_id[0, 4] == -1


def test_uniform_scores_keep_lowest_candidates(oracle):
    st, Q = make_state(15, H=1, d=16, B=8, Nq=24, w=1, C=2, k=1)
    st.select(Q)
    st.Kc_l[...] = 0.0; st.Kc_p[...] = 0.0            # all representatives equal -> all scores equal
    b, sc, src = run_update(st)
    assert len(set(sc[0].tolist())) == 1
    assert np.all(src == -1) and np.array_equal(st.p_id, b["p_id"])   # occupants are the lowest candidates
    assert st.S_cnt[0].tolist() == [3] * 8                            # the three evicted blocks were folded


def test_fold_of_constant_blocks_is_exact_and_drop_mode(oracle):
    st, Q = make_state(16, H=1, d=16, B=8, Nq=16, w=1, C=1, k=1)
    st.select(Q)
    const = bf(np.tile(np.linspace(-2, 2, 16), (8, 1)))
    l_map, _, _ = st._maps()
    st.Kl[0, l_map[:2]] = const; st.Vl[0, l_map[:2]] = const
    st.Kp[0, 0] = const; st.Vp[0, 0] = const
    st.update()
    assert st.S_cnt[0].tolist() == [2] * 8
    assert np.array_equal(st.Kp[0, 1], const) and np.array_equal(st.Vp[0, 1], const)
    # S_sum = NULL: losers are simply dropped (the paper's plain Top-C), slot C stays empty
    st3, Q3 = make_state(16, H=1, d=16, B=8, Nq=16, w=1, C=1, k=1, fold=False)
    st3.select(Q3)
    st3.update()
    assert st3.p_len[0, 1] == 0


# ------------------------------------------------------------------------------------------------
# fine attention mass and the update ranked by it
# ------------------------------------------------------------------------------------------------
def ref_block_mass(st, Q, sel):
    """Per (head, query block, key block) sums of the explicit masked softmax matrix (fp64), written
    independently of the oracle: the dense P of Eq. 3-5 first, then plain slicing by block owner."""
    l_map, l_len, _ = st._maps()
    nu = st.C + 1 + st.n_loc
    out = np.zeros((st.H, st.nqb, nu))
    for h in range(st.H):
        keys, owner = [], []
        for s in range(st.C + 1):
            n = st.p_len[h, s]
            keys.append(f32(st.Kp[h, s, :n])); owner += [s] * n
        for l in range(st.n_loc):
            n = l_len[l]
            keys.append(f32(st.Kl[h, l_map[l], :n])); owner += [st.C + 1 + l] * n
        Kc = np.concatenate(keys).astype(np.float64)
        owner = np.array(owner)
        M = np.full((st.Nq, len(owner)), -np.inf)
        for t in range(st.Nq):
            vis = [st.C + 1 + int(x) for x in sel[h, t // st.B] if x >= 0]
            M[t, (owner <= st.C) | np.isin(owner, vis)] = 0.0
        S = f32(Q[h]).astype(np.float64) @ Kc.T * st.scale + M
        P = np.exp(S - S.max(1, keepdims=True))
        P /= P.sum(1, keepdims=True)
        for i in range(st.nqb):
            rows = P[i * st.B:min((i + 1) * st.B, st.Nq)]
            for u in range(nu):
                out[h, i, u] = rows[:, owner == u].sum()
    return out


def test_attention_mass_is_the_block_sum_of_the_softmax_matrix(oracle):
    st, Q = make_state(20, H=2, d=16, B=8, Nq=20, w=2, C=3, k=3, p_lens=[[8, 0, 5], [8, 8, 8]])
    st.set_summary(np.abs(rnd(201, 2, 2, 8, 16)).astype(np.float32), np.tile(np.array([2, 2, 1, 1, 0, 0, 0, 0], np.int32), (2, 1)))
    sel, _ = st.select(Q)
    mass = st.attention_mass(Q).reshape(st.H, st.nqb, -1)
    np.testing.assert_allclose(mass, ref_block_mass(st, Q, sel), rtol=0, atol=1e-12)
    # every row of a softmax matrix adds 1: a query block's masses add up to its number of rows
    rows = np.array([8, 8, 4], np.float64)
    np.testing.assert_allclose(mass.sum(2), np.tile(rows, (st.H, 1)), rtol=0, atol=1e-12)
    # no mass where nothing is attended: the empty slot, the local blocks outside the row of sel
    assert np.all(mass[0, :, 1] == 0.0)
    for h in range(st.H):
        for i in range(st.nqb):
            off = sorted(set(range(st.n_loc)) - set(int(x) for x in sel[h, i] if x >= 0))
            assert np.all(mass[h, i, st.C + 1 + np.array(off)] == 0.0)
            on = [int(x) for x in sel[h, i] if x >= 0]
            assert np.all(mass[h, i, st.C + 1 + np.array(on)] > 0.0)
    assert np.all(mass[:, :, st.C] > 0.0)                    # the summary block is attended by every row
    # a list of query blocks gives the same numbers as the full run
    part = st.attention_mass(Q, np.array([1, 0], np.int32), np.array([2, 1], np.int32))
    assert np.array_equal(part[0], mass[1, 2]) and np.array_equal(part[1], mass[0, 1])


def test_attention_mass_closed_forms(oracle):
    # one persistent block and nothing else: all the mass of every row lands on it
    st, Q = make_state(21, H=1, d=16, B=8, Nq=12, w=0, C=1, k=0, p_lens=[[6]])
    st.select(Q)
    mass = st.attention_mass(Q).reshape(1, st.nqb, -1)
    np.testing.assert_allclose(mass[0, :, 0], [8.0, 4.0], rtol=1e-14)
    assert np.all(mass[0, :, 1:] == 0.0)
    # identical keys everywhere: the mass of a block is proportional to its valid tokens
    st, Q = make_state(22, H=1, d=16, B=8, Nq=16, w=1, C=2, k=4, causal=0, p_lens=[[8, 3]])
    l_map, l_len, _ = st._maps()
    row = bf(rnd(221, 1, 16))
    st.Kp[...] = row
    st.Kl[...] = row
    sel, _ = st.select(Q)
    st.sel = np.tile(np.arange(4, dtype=np.int32), (1, st.nqb, 1))       # everything attended, whatever the ties chose
    mass = st.attention_mass(Q).reshape(st.nqb, -1)
    tokens = np.array([8, 3, 0] + [8] * 4, np.float64)
    np.testing.assert_allclose(mass, np.tile(8.0 * tokens / tokens.sum(), (st.nqb, 1)), rtol=1e-12)
    # garbage in the padding rows of a ragged block carries no mass
    st.Kp[0, 1, 3:] = bf(np.full((5, 16), 40.0))
    np.testing.assert_array_equal(st.attention_mass(Q).reshape(st.nqb, -1), mass)


def fine_inputs(st, seed, ties=False):
    """A made-up mass matrix [H][C+1+n_loc][nqb] (the update only ranks it)."""
    nu = st.C + 1 + st.n_loc
    Mt = np.abs(rnd(seed, st.H, nu, st.nqb)).astype(np.float32)
    if ties:
        Mt = np.round(Mt).astype(np.float32)                           # few distinct sums: many equal scores
    return Mt


@pytest.mark.parametrize("seed,n_sink,ties", [(30, 0, False), (31, 1, False), (32, 0, True), (33, 2, True)])
def test_fine_retention_is_bruteforce_topc_of_the_column_sums(oracle, seed, n_sink, ties):
    st, Q = make_state(seed, H=3, d=16, B=8, Nq=28, w=2, C=4, k=2, n_sink=n_sink,
                       p_lens=[[8, 8, 5, 8], [8, 0, 8, 8], [8, 8, 8, 0]])
    st.select(Q)
    Mt = fine_inputs(st, seed, ties)
    b = dict(p_len=st.p_len.copy(), p_id=st.p_id.copy(), Kp=st.Kp.copy(), Kl=st.Kl.copy(), maps=st._maps())
    ne, C = st.n_evict_now(), st.C
    sc, src = st.update_fine(Mt)
    l_map, l_len, l_id = b["maps"]
    # the score is the mass per query token, summed over query blocks in ascending order in fp32
    want = np.zeros((st.H, C + 1 + len(l_map)), np.float32)
    for i in range(st.nqb):
        want = want + Mt[:, :, i]
    want = want / np.float32(st.Nq)
    n_tied = 0
    for h in range(st.H):
        occ = b["p_len"][h, :C] > 0
        assert sc[h, :C].tolist() == np.where(occ, want[h, :C], np.float32(0)).tolist()
        assert sc[h, C:].tolist() == want[h, C + 1:C + 1 + ne].tolist()
        cands = [("p", s) for s in range(n_sink, C) if occ[s]] + [("e", e) for e in range(ne)]
        val = [float(want[h, s]) if kind == "p" else float(want[h, C + 1 + s]) for kind, s in cands]
        order = sorted(range(len(cands)), key=lambda a: (-val[a], a))
        winners = set(order[:C - n_sink])
        n_tied += len(val) - len(set(val))
        free = [s for s in range(n_sink, C) if not occ[s]]
        free += [cands[a][1] for a in range(len(cands)) if cands[a][0] == "p" and a not in winners]
        free.sort()
        new = sorted(cands[a][1] for a in winners if cands[a][0] == "e")
        want_src = np.full(C, -1)
        for s, e in zip(free, new):
            want_src[s] = e
        assert src[h].tolist() == want_src.tolist()
        for s in range(C):
            if want_src[s] >= 0:
                e = want_src[s]
                assert np.array_equal(st.Kp[h, s], b["Kl"][h, l_map[e]]) and st.p_id[h, s] == l_id[e]
            elif occ[s] and s not in free:
                assert np.array_equal(st.Kp[h, s], b["Kp"][h, s]) and st.p_id[h, s] == b["p_id"][h, s]
        n_lost = len(cands) - len(winners)
        assert st.S_cnt[h].max() == n_lost or n_lost == 0
    assert (n_tied > 0) == ties


def test_fine_and_coarse_updates_share_everything_but_the_score(oracle):
    """Fed the coarse column scores as a one-query-block mass matrix, the fine update must do exactly what the
    coarse one does: retention, slots and fold are one piece of arithmetic with two sources of scores."""
    a, Q = make_state(34, H=2, d=16, B=8, Nq=8, w=2, C=3, k=2, p_lens=[[8, 8, 6], [8, 0, 8]])
    b2, _ = make_state(34, H=2, d=16, B=8, Nq=8, w=2, C=3, k=2, p_lens=[[8, 8, 6], [8, 0, 8]])
    a.select(Q); b2.select(Q)
    l_map, _, _ = a._maps()
    s_p, s_l = oracle.scores(a.cfg(), a.Qc, a.Kc_l, l_map, a.Kc_p, a.p_len)
    Mt = np.zeros((a.H, a.C + 1 + a.n_loc, 1), np.float32)
    Mt[:, :a.C, 0] = s_p * np.float32(a.Nq)                 # Nq = 8: scaling by a power of two and back is exact
    Mt[:, a.C + 1:, 0] = s_l * np.float32(a.Nq)
    sc_a, src_a = a.update()
    sc_b, src_b = b2.update_fine(Mt)
    assert np.array_equal(sc_a, sc_b) and np.array_equal(src_a, src_b)
    for name in ("Kp", "Vp", "p_len", "p_id", "Kc_p", "S_sum", "S_cnt"):
        assert np.array_equal(getattr(a, name), getattr(b2, name))


# ------------------------------------------------------------------------------------------------
# backward of the fine stage
# ------------------------------------------------------------------------------------------------
def gathered(st, h, sel):
    """Keys and values of head h as fp64 matrices, where each key lives (('p', slot, token) / ('l', physical
    slot, token)), and the visibility mask [Nq][n_keys] of Eq. 5."""
    l_map, l_len, _ = st._maps()
    keys, vals, where, owner = [], [], [], []
    for s in range(st.C + 1):
        for u in range(st.p_len[h, s]):
            keys.append(f32(st.Kp[h, s, u])); vals.append(f32(st.Vp[h, s, u])); where.append(("p", s, u)); owner.append(-1)
    for l in range(st.n_loc):
        for u in range(l_len[l]):
            keys.append(f32(st.Kl[h, l_map[l], u])); vals.append(f32(st.Vl[h, l_map[l], u]))
            where.append(("l", int(l_map[l]), u)); owner.append(l)
    owner = np.array(owner)
    M = np.full((st.Nq, len(owner)), -np.inf)
    for t in range(st.Nq):
        vis = [int(x) for x in sel[h, t // st.B] if x >= 0]
        M[t, (owner < 0) | np.isin(owner, vis)] = 0.0
    return np.array(keys, np.float64), np.array(vals, np.float64), where, M


def loss_of(Qh, K, V, M, G, scale):
    """sum(O * G) with O = softmax(Q K^T scale + M) V: the scalar whose gradient the backward pass is."""
    S = Qh @ K.T * scale + M
    P = np.exp(S - S.max(1, keepdims=True))
    P /= P.sum(1, keepdims=True)
    return float(((P @ V) * G).sum())


def test_backward_matches_finite_differences_of_the_forward(oracle):
    st, Q = make_state(40, H=2, d=16, B=8, Nq=20, w=2, C=3, k=2, p_lens=[[8, 0, 5], [8, 8, 8]])
    st.set_summary(np.abs(rnd(401, 2, 2, 8, 16)).astype(np.float32), np.tile(np.array([2, 2, 1, 0, 0, 0, 0, 0], np.int32), (2, 1)))
    sel, _ = st.select(Q)
    dO = bf(rnd(402, st.H, st.Nq, st.d))
    dQ, dKp, dVp, dKl, dVl = st.attention_bwd(Q, dO)
    eps = 1e-5
    for h in range(st.H):
        K, V, where, M = gathered(st, h, sel)
        Qh, G = f32(Q[h]).astype(np.float64), f32(dO[h]).astype(np.float64)

        def num(arr, idx):
            old = arr[idx]
            arr[idx] = old + eps; up = loss_of(Qh, K, V, M, G, st.scale)
            arr[idx] = old - eps; dn = loss_of(Qh, K, V, M, G, st.scale)
            arr[idx] = old
            return (up - dn) / (2 * eps)

        pick = (rnd(403 + h, 24) * 1e6).astype(np.int64)
        for n in range(8):
            t, x = abs(pick[n]) % st.Nq, abs(pick[n + 8]) % st.d
            np.testing.assert_allclose(dQ[h, t, x], num(Qh, (t, x)), rtol=1e-6, atol=1e-9)
        for n in range(12):                      # keys of every kind: persistent, summary, selected by some, by none
            j, x = abs(pick[n]) % len(where) if n > 3 else [0, len(where) - 1, st.p_len[h, :st.C].sum(), len(where) // 2][n], abs(pick[n + 12]) % st.d
            kind, slot, u = where[j]
            dK, dV = (dKp, dVp) if kind == "p" else (dKl, dVl)
            np.testing.assert_allclose(dK[h, slot, u, x], num(K, (j, x)), rtol=1e-6, atol=1e-9)
            np.testing.assert_allclose(dV[h, slot, u, x], num(V, (j, x)), rtol=1e-6, atol=1e-9)


def test_backward_invariants_and_special_cases(oracle):
    st, Q = make_state(41, H=2, d=16, B=8, Nq=28, w=2, C=2, k=2, p_lens=[[8, 6], [8, 8]])
    sel, _ = st.select(Q)
    dO = bf(rnd(412, st.H, st.Nq, st.d))
    dQ, dKp, dVp, dKl, dVl = st.attention_bwd(Q, dO)
    G = f32(dO).astype(np.float64)
    for h in range(st.H):
        # every row's probabilities add up to 1: the value gradients add up to the output gradients
        np.testing.assert_allclose(dVp[h].sum((0, 1)) + dVl[h].sum((0, 1)), G[h].sum(0), rtol=1e-12, atol=1e-12)
        # a softmax does not see a vector added to all its keys: the key gradients of a head add up to zero
        np.testing.assert_allclose(dKp[h].sum((0, 1)) + dKl[h].sum((0, 1)), 0.0, atol=1e-12)
    l_map, l_len, _ = st._maps()
    # nothing for keys that nobody attends: the padding of ragged blocks, the blocks in no row of sel
    assert np.all(dKp[0, 1, 6:] == 0) and np.all(dVp[0, 1, 6:] == 0)
    assert np.all(dKl[:, l_map[-1], l_len[-1]:] == 0)
    for h in range(st.H):
        unused = sorted(set(range(st.n_loc)) - set(int(x) for x in sel[h].ravel() if x >= 0))
        assert unused
        assert np.all(dKl[h, l_map[unused]] == 0) and np.all(dVl[h, l_map[unused]] == 0)
        used = sorted(set(int(x) for x in sel[h].ravel() if x >= 0))
        assert all(np.abs(dVl[h, l_map[l], :l_len[l]]).min() > 0 for l in used)
    # a subset of the rows: their dQ is that of the full run, the others get none; dK/dV are sums over rows
    mask = np.zeros((st.H, st.Nq), bool); mask[0, ::3] = True; mask[1, 5] = True
    dQ2, dKp2, dVp2, dKl2, dVl2 = st.attention_bwd(Q, dO, row_mask=mask)
    assert np.array_equal(dQ2[mask], dQ[mask]) and np.all(dQ2[~mask] == 0)
    dQ3, dKp3, dVp3, dKl3, dVl3 = st.attention_bwd(Q, dO, row_mask=~mask)
    np.testing.assert_allclose(dKp2 + dKp3, dKp, atol=1e-13); np.testing.assert_allclose(dVl2 + dVl3, dVl, atol=1e-13)
    # one key and nothing else: P = 1 whatever Q is, so dQ = dK = 0 and the key's value takes all of dO
    st1, Q1 = make_state(42, H=1, d=16, B=8, Nq=12, w=0, C=1, k=0, p_lens=[[1]])
    st1.select(Q1)
    dO1 = bf(rnd(421, 1, 12, 16))
    dQ1, dKp1, dVp1, _, _ = st1.attention_bwd(Q1, dO1)
    assert np.all(dQ1 == 0) and np.all(dKp1 == 0)
    np.testing.assert_allclose(dVp1[0, 0, 0], f32(dO1[0]).astype(np.float64).sum(0), rtol=1e-14)


def test_rollout_summary_counts(oracle):
    """Cold start over several chunks: window fills, then every update evicts one chunk; counts add up."""
    H, d, B, Nq, w, C = 1, 16, 8, 20, 2, 2
    st = OracleState(H, d, B, Nq, w, C, 2, 0.25)
    nqb = st.nqb
    lens = np.array([8, 8, 4], np.int32)
    folded = 0
    for g in range(7):
        K = bf(rnd(200 + 3 * g, H, Nq, d)); V = bf(rnd(201 + 3 * g, H, Nq, d)); Q = bf(rnd(202 + 3 * g, H, Nq, d))
        st.append_chunk(synth.to_blocks(K, B), synth.to_blocks(V, B), lens, g * nqb + np.arange(nqb))
        st.select(Q)
        occupied_before = int((st.p_len[0, :C] > 0).sum())
        ne = st.n_evict_now()
        assert ne == (nqb if g >= w else 0)
        st.update()
        occupied_after = int((st.p_len[0, :C] > 0).sum())
        if ne:
            folded += occupied_before + ne - occupied_after
    assert occupied_after == C
    assert st.S_cnt[0].max() == folded
    ids = [int(x) for x in st.p_id[0]]
    assert len(set(ids)) == C and all(0 <= x < 5 * nqb for x in ids)


def test_cfg1_rollout_matches_the_stored_fixture():
    """The oracle's results on cfg1 as frozen by tests/golden/make_cfg1_golden.py (which calls only the
    oracle): block sets, score bit patterns, slot assignments exactly; stored attention rows to 1e-5.
    Not a pin against the paper (it prints no intermediate values): a guard against silent drift."""
    import importlib.util
    import json
    import os
    here = os.path.dirname(os.path.abspath(__file__))
    spec = importlib.util.spec_from_file_location("make_cfg1_golden", os.path.join(here, "golden", "make_cfg1_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    now = mod.build()
    with open(os.path.join(here, "golden", "cfg1_rollout.json")) as f:
        ref = json.load(f)
    assert len(now["chunks"]) == len(ref["chunks"])
    for a, b in zip(now["chunks"], ref["chunks"]):
        for key in ("sel", "scores_bits", "slot_src", "p_id", "p_len", "S_cnt_sum"):
            assert a[key] == b[key], key
        assert np.allclose(a["O_rows"], b["O_rows"], atol=1e-5)
        assert np.allclose(a["lse_rows"], b["lse_rows"], atol=1e-5)


# ------------------------------------------------------------------------------------------------
# block rearrange (Alg. 3): pinned by a brute-force index walk and by what the layout promises
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("shape", [(3, 8, 12, 1, 4, 4), (3, 8, 8, 3, 4, 4), (2, 16, 8, 1, 8, 8), (4, 4, 6, 2, 2, 3)])
def test_blockify_is_the_box_walk(shape):
    from oracle import blockify as ob
    T, Hs, Ws, Bt, Bh, Bw = shape
    H, d = 2, 3
    X = np.arange(T * Hs * Ws * H * d, dtype=np.int64).reshape(T, Hs, Ws, H, d)
    Y = ob.blockify(X, Bt, Bh, Bw)
    Nt, Nh, Nw = T // Bt, Hs // Bh, Ws // Bw
    assert Y.shape == (H, Nt * Nh * Nw, Bt * Bh * Bw, d)
    # every block is one box of the grid, blocks and the tokens inside them in row-major order
    for tb in range(Nt):
        for hb in range(Nh):
            for wb in range(Nw):
                b = (tb * Nh + hb) * Nw + wb
                r = 0
                for dt in range(Bt):
                    for dh in range(Bh):
                        for dw in range(Bw):
                            for h in range(H):
                                assert np.array_equal(Y[h, b, r], X[tb * Bt + dt, hb * Bh + dh, wb * Bw + dw, h])
                            r += 1
    # a permutation (nothing lost, nothing doubled) and its inverse
    assert np.array_equal(np.sort(Y.ravel()), X.ravel())
    assert np.array_equal(ob.unblockify(Y, T, Hs, Ws, Bt, Bh, Bw), X)


def test_blockify_degenerate_shapes():
    from oracle import blockify as ob
    X = np.arange(2 * 4 * 6 * 1 * 2).reshape(2, 4, 6, 1, 2)
    # one block = the whole grid: token order unchanged; blocks of one token: token order unchanged too
    assert np.array_equal(ob.blockify(X, 2, 4, 6)[0, 0], X.reshape(-1, 2))
    assert np.array_equal(ob.blockify(X, 1, 1, 1)[0, :, 0], X.reshape(-1, 2))
    # blocks that are whole rows keep raster order
    assert np.array_equal(ob.blockify(X, 1, 1, 6)[0].reshape(-1, 2), X.reshape(-1, 2))
    with pytest.raises(AssertionError):
        ob.blockify(X, 1, 3, 6)
