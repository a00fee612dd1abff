"""GPU parity of the fine-mass variant: pbsa_attention_mass and pbsa_memory_update_fine against the CPU oracle.

Bar.  The mass matrix is floating point: every entry within MASS_RTOL of the fp64 oracle (a probability is
exp(s - lse); the kernel's lse is within 4e-3 of the exact one because its normaliser sums bf16-rounded
probabilities, the scores themselves are fp32 sums of exact bf16 products), and the masses of a query block
add up to its number of rows within the same bound.  The update ranked by a mass matrix is integer work
decided by fp32 sums in a fixed order: fed the SAME matrix (a seeded synthetic one, never the kernel's), the
GPU and the oracle must agree bit for bit on slots, ids, lengths, scores and the summary.  End to end (each
side ranking its own masses) the retained sets must be equal whenever the oracle's scores separate the last
block kept from the first one dropped by more than the mass tolerance, and valid otherwise.
"""
import math

import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle.rollout import OracleState, state_for_workload  # noqa: E402
from harness import synth  # noqa: E402
from tests.test_gpu_parity import DEV, check_attention, compare_select, compare_update, rnd  # noqa: E402

pytestmark = pytest.mark.gpu

MASS_RTOL, MASS_ATOL = 6e-3, 1e-6


@pytest.fixture(scope="module")
def gpu():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from harness import workloads
    from paper_2604_21221_amd import cache, pbsa
    pbsa.lib()
    return dict(cache=cache, pbsa=pbsa, wl=workloads)


def chunk_lens(st):
    lens = np.full(st.nqb, st.B, np.int32)
    lens[-1] = st.Nq - (st.nqb - 1) * st.B
    return lens


def attend_both(gpu, c, st, Q, K, V, g, what, qb=None):
    """Append, select and attend on both sides, then the masses: the GPU's for every query block, the oracle's
    for the listed (heads, blocks) or all.  The GPU computes them twice: by pbsa_attention_mass (checked here)
    and by pbsa_attention_fwd_mass, whose matrix is returned: (Mt device tensor, the same as [H][nqb][n_u] on
    the host, oracle masses in that shape with NaN where not computed)."""
    wl = gpu["wl"]
    print(f"[case] {what} chunk {g}", flush=True)
    st.append_chunk(synth.to_blocks(K, st.B), synth.to_blocks(V, st.B), chunk_lens(st), g * st.nqb + np.arange(st.nqb))
    Qd = wl.bf16_tensor(Q, DEV)
    c.append_chunk(wl.bf16_tensor(K, DEV), wl.bf16_tensor(V, DEV), g)
    st.select(Q)
    c.select(Qd)
    compare_select(c, st, what)
    lse = torch.empty(st.H, st.Nq, dtype=torch.float32, device=DEV)
    O = c.attention(Qd, lse=lse)
    n_u = st.C + 1 + st.n_loc
    # the separate pass over the keys ...
    Mt_pass = c.attention_mass(Qd, lse).clone()
    # ... and the attention call that records the masses as it goes: same O and lse, bit for bit
    lse2 = torch.empty_like(lse)
    O2, Mt = c.attention_with_mass(Qd, lse=lse2)
    torch.cuda.synchronize()
    assert torch.equal(O.view(torch.int16), O2.view(torch.int16)), f"{what}: the mass variant changed the output"
    assert torch.equal(lse.view(torch.int32), lse2.view(torch.int32)), f"{what}: the mass variant changed lse"
    assert tuple(Mt.shape) == (st.H, n_u, (st.nqb + 3) & ~3) == tuple(Mt_pass.shape)
    to_np = lambda M: M.cpu().numpy()[:, :, :st.nqb].transpose(0, 2, 1).astype(np.float64)   # [H][nqb][n_u]
    ref = np.full((st.H, st.nqb, n_u), np.nan)
    if qb is None:
        ref[...] = st.attention_mass(Q).reshape(st.H, st.nqb, n_u)
    else:
        ref[qb[0], qb[1]] = st.attention_mass(Q, qb[0], qb[1])
    check_mass(to_np(Mt_pass), ref, st, f"{what} chunk {g}, separate pass")
    return Mt, to_np(Mt), ref


def check_mass(got, ref, st, what):
    done = ~np.isnan(ref)
    err = np.abs(got[done] - ref[done])
    bound = MASS_RTOL * np.abs(ref[done]) + MASS_ATOL
    rel = (err / np.maximum(np.abs(ref[done]), 1e-3)).max() if err.size else 0.0
    print(f"{what}: mass entries {done.sum()}, worst err/bound {np.max(err / bound) if err.size else 0:.3f}, "
          f"worst relative (masses above 1e-3) {rel:.2e}", flush=True)
    assert np.isfinite(got).all(), what
    assert (err <= bound).all(), what
    # exactly zero where nothing is attended, positive where something is -- unless it is below what the kernels
    # hold: fp32 for the separate pass; in the attention kernel a probability is a bf16 number 2^80 below its
    # row's reference, so whatever lies more than 2^-46 under the score that set the reference is flushed to zero
    # (a block of 128 x 128 such entries stays below 2.4e-10, four orders of magnitude under MASS_ATOL)
    assert (got[done][ref[done] == 0.0] == 0.0).all(), what
    assert (got[done][ref[done] > 1e-9] > 0.0).all(), what
    rows = chunk_lens(st).astype(np.float64)
    np.testing.assert_allclose(got.sum(2), np.tile(rows, (st.H, 1)), rtol=MASS_RTOL, err_msg=what)


SMALL = [
    # name,           H, d,   B,   Nq,  w, C, k, n_sink, causal, p_lens
    ("d64_B64",       2, 64,  64,  200, 2, 3, 3, 0, 1, [64, 17, 0]),
    ("d128_B64",      2, 128, 64,  333, 2, 4, 5, 1, 1, [64, 64, 1, 40]),
    ("d128_B128",     2, 128, 128, 333, 2, 3, 4, 0, 1, [128, 70, 64]),
    ("d64_B128",      1, 64,  128, 300, 1, 2, 2, 1, 0, [100, 128]),
    ("noncausal_all", 2, 128, 64,  200, 1, 2, 64, 0, 0, [64, 64]),
    ("no_memory",     1, 128, 64,  130, 2, 0, 2, 0, 1, []),
    ("k_zero",        1, 64,  64,  100, 1, 2, 0, 0, 1, [64, 30]),
]


def small_pair(gpu, case):
    name, H, d, B, Nq, w, C, k, n_sink, causal, p_lens = case
    scale = np.float32(1.0 / math.sqrt(d))
    st = OracleState(H, d, B, Nq, w, C, k, scale, n_sink=n_sink, causal=causal)
    c = gpu["cache"].PbsaCache(H, d, B, Nq, w, C, k, scale, n_sink=n_sink, causal=causal, device=DEV)
    if C > 0:
        Kp, Vp = rnd(1, H, C, B, d), rnd(2, H, C, B, d)
        for s, n in enumerate(p_lens):           # non-finite patterns beyond the valid length must never matter
            Kp[:, s, n:] = 0x7FC0; Vp[:, s, n:] = 0x7F80
        pl = np.tile(np.array(p_lens, np.int32), (H, 1))
        ids = -100 - np.arange(C)[None, :].repeat(H, 0)
        st.set_persistent(Kp, Vp, pl, ids)
        c.set_persistent(gpu["wl"].bf16_tensor(Kp, DEV), gpu["wl"].bf16_tensor(Vp, DEV),
                         torch.from_numpy(pl).to(DEV), torch.from_numpy(ids))
    return st, c


@pytest.mark.parametrize("case", SMALL, ids=[c[0] for c in SMALL])
def test_mass_small_every_entry(gpu, case):
    """Cold start, fill, then evicting updates (the coarse ones, which keep both sides bit-identical): the mass
    matrix of every chunk, every entry."""
    st, c = small_pair(gpu, case)
    name, H, d, B, Nq, w = case[:6]
    for g in range(w + 3):
        Q, K, V = rnd(10 + 3 * g, H, Nq, d), rnd(11 + 3 * g, H, Nq, d, scale=1.5), rnd(12 + 3 * g, H, Nq, d)
        _, got, ref = attend_both(gpu, c, st, Q, K, V, g, name)
        check_mass(got, ref, st, f"{name} chunk {g}")
        ne = st.n_evict_now()
        sc_ref, src_ref = st.update()
        assert c.update() == ne
        compare_update(c, st, gpu["wl"], sc_ref, src_ref, ne, name)


def synthetic_mass(st, seed, ties):
    """A seeded mass-like matrix [H][C+1+n_loc][nqb] (the update only ranks it): positive, a few times the
    spread of real masses; with `ties` quantised so that many row sums are equal."""
    n_u = st.C + 1 + st.n_loc
    u = synth.uniforms(synth.stream_key(seed, "misc", 5), st.H * n_u * st.nqb).reshape(st.H, n_u, st.nqb)
    M = (u * 4.0).astype(np.float32)
    return np.round(M).astype(np.float32) if ties else M


@pytest.mark.parametrize("case", [SMALL[0], SMALL[1], SMALL[2], SMALL[3]], ids=[c[0] for c in SMALL[:4]])
@pytest.mark.parametrize("ties", [False, True], ids=["distinct", "ties"])
def test_fine_update_bit_exact_on_a_given_matrix(gpu, case, ties):
    """Both sides rank the same seeded matrix: slots, ids, lengths, scores, summary sums bit for bit, chunk
    after chunk (the states stay identical, so the rollout goes on)."""
    st, c = small_pair(gpu, case)
    name, H, d, B, Nq, w = case[:6]
    pad = (st.nqb + 3) & ~3
    for g in range(w + 4):
        Q, K, V = rnd(20 + 3 * g, H, Nq, d), rnd(21 + 3 * g, H, Nq, d), rnd(22 + 3 * g, H, Nq, d)
        print(f"[case] fine update {name} ties={ties} chunk {g}", flush=True)
        st.append_chunk(synth.to_blocks(K, B), synth.to_blocks(V, B), chunk_lens(st), g * st.nqb + np.arange(st.nqb))
        c.append_chunk(gpu["wl"].bf16_tensor(K, DEV), gpu["wl"].bf16_tensor(V, DEV), g)
        st.select(Q)
        c.select(gpu["wl"].bf16_tensor(Q, DEV))
        M = synthetic_mass(st, 100 * g + 7, ties)
        Md = torch.full((H, M.shape[1], pad), float("nan"), dtype=torch.float32, device=DEV)   # padding is never read
        Md[:, :, :st.nqb] = torch.from_numpy(M).to(DEV)
        ne = st.n_evict_now()
        sc_ref, src_ref = st.update_fine(M)
        assert c.update_fine(Md) == ne
        torch.cuda.synchronize()
        compare_update(c, st, gpu["wl"], sc_ref, src_ref, ne, f"{name} chunk {g}")
    if st.C > 0:
        assert (st.p_id[:, case[8]:] >= 0).any(), "some newcomer must have been promoted during the rollout"


def chain_step(gpu, c, st, Q, K, V, g, what):
    """select -> attention -> mass -> update ranked by the mass, each side on its own masses.  Returns True if
    the two sides took the same decisions (and are then compared in full), False if the oracle's scores were too
    close to call and the GPU's choice was only checked for validity."""
    Mt, got, ref = attend_both(gpu, c, st, Q, K, V, g, what)
    check_mass(got, ref, st, f"{what} chunk {g}")
    ne, C, n_sink = st.n_evict_now(), st.C, st.n_sink
    occ = st.p_len[:, :C] > 0
    Mo = np.ascontiguousarray(ref.transpose(0, 2, 1)).astype(np.float32)               # [H][n_u][nqb]
    sc_ref, src_ref = st.update_fine(Mo)
    assert c.update_fine(Mt) == ne
    torch.cuda.synchronize()
    sc = c.scores.view(-1)[:st.H * (C + ne)].view(st.H, C + ne).cpu().numpy()
    tol = MASS_RTOL * np.abs(sc_ref) + MASS_ATOL
    assert (np.abs(sc - sc_ref) <= tol).all(), f"{what}: scores differ by more than the mass tolerance"
    src = c.slot_src.cpu().numpy()[:, :C]
    clear = True
    for h in range(st.H):
        cand = [s for s in range(n_sink, C) if occ[h, s]] + [C + e for e in range(ne)]
        vals = sorted((float(sc_ref[h, x]) for x in cand), reverse=True)
        places = C - n_sink
        if len(vals) > places:
            gap = vals[places - 1] - vals[places]
            if gap <= 2 * (MASS_RTOL * vals[places - 1] + MASS_ATOL):
                clear = False
                # valid all the same: whatever the GPU kept scores at least the oracle's threshold, within tolerance
                kept = [s for s in range(n_sink, C) if occ[h, s] and src[h, s] < 0 and c.p_len[h, s].item() > 0]
                kept += [C + int(e) for e in src[h] if e >= 0]
                thr = vals[places - 1]
                assert all(sc_ref[h, x] >= thr - 2 * (MASS_RTOL * thr + MASS_ATOL) for x in kept), what
    if clear:
        assert np.array_equal(src, src_ref), f"{what}: slot assignment differs"
        assert np.array_equal(c.p_id.cpu().numpy()[:, :C], st.p_id) and np.array_equal(c.p_len.cpu().numpy(), st.p_len)
        assert np.array_equal(gpu["wl"].bits_of(c.Kp), st.Kp) and np.array_equal(gpu["wl"].bits_of(c.Vp), st.Vp)
        assert np.array_equal(c.S_cnt.cpu().numpy(), st.S_cnt)
        assert np.array_equal(c.S_sum.cpu().numpy().view(np.uint32), st.S_sum.view(np.uint32))
    return clear


@pytest.mark.parametrize("case", [SMALL[1], SMALL[2]], ids=[SMALL[1][0], SMALL[2][0]])
def test_fine_chain_small(gpu, case):
    st, c = small_pair(gpu, case)
    name, H, d, B, Nq, w = case[:6]
    n_clear = 0
    for g in range(w + 4):
        Q, K, V = rnd(30 + 3 * g, H, Nq, d), rnd(31 + 3 * g, H, Nq, d, scale=1.5), rnd(32 + 3 * g, H, Nq, d)
        if not chain_step(gpu, c, st, Q, K, V, g, f"chain {name}"):
            break                                 # the sides may hold different sets from here on
        n_clear += 1
    assert n_clear > w + 1, "at least one evicting update must have been compared in full"


def sample_blocks(H, nqb, per_head, seed):
    u = synth.uniforms(synth.stream_key(seed, "misc", 78), H * per_head).reshape(H, per_head)
    ii = (u * nqb).astype(np.int32)
    ii[:, 0] = 0; ii[:, 1] = nqb - 1; ii[:, 2] = nqb - 2
    return np.repeat(np.arange(H, dtype=np.int32), per_head), np.minimum(ii, nqb - 1).ravel().astype(np.int32)


def test_cfg2_full_size_chain(gpu):
    """Full size, B = 128: masses of every query block against the oracle, then the update each side ranks by
    its own."""
    w = synth.WORKLOADS["cfg2"]
    st, g0 = state_for_workload(w)
    c, _ = gpu["wl"].cache_for_workload(w, device=DEV)
    Q, K, V = synth.chunk_qkv(w, 0, g0)
    chain_step(gpu, c, st, Q, K, V, g0, "cfg2")


def test_cfg5_full_size_sampled_blocks(gpu):
    """The 1-minute shape (B = 64), cold start through the first evicting updates with the coarse update; from
    the first full window on, the masses of sampled query blocks of every head against the oracle, the row-sum
    property on all of them, and at the last chunk the whole chain."""
    w = synth.WORKLOADS["cfg5"]
    st, g0 = state_for_workload(w)
    c, _ = gpu["wl"].cache_for_workload(w, device=DEV)
    qb = sample_blocks(w.H, w.nqb, 4, 5)
    for g in range(5):
        Q, K, V = synth.chunk_qkv(w, 0, g)
        if g == 4:
            chain_step(gpu, c, st, Q, K, V, g, "cfg5")
            break
        _, got, ref = attend_both(gpu, c, st, Q, K, V, g, "cfg5", qb if g >= 2 else (qb[0][:4], qb[1][:4]))
        check_mass(got, ref, st, f"cfg5 chunk {g}")
        ne = st.n_evict_now()
        sc_ref, src_ref = st.update()
        assert c.update() == ne
        compare_update(c, st, gpu["wl"], sc_ref, src_ref, ne, "cfg5")


def test_mass_with_more_slots_than_the_update_maintains(gpu):
    """100 persistent slots of every length from empty to full (the attention calls and the mass calls take up to
    192; only the update stops at 64): every entry of the mass matrix from both routes."""
    H, d, B, Nq, w, C, k = 1, 64, 64, 150, 1, 100, 2
    scale = np.float32(1.0 / math.sqrt(d))
    st = OracleState(H, d, B, Nq, w, C, k, scale)
    c = gpu["cache"].PbsaCache(H, d, B, Nq, w, C, k, scale, device=DEV)
    Kp, Vp = rnd(801, H, C, B, d), rnd(802, H, C, B, d)
    pl = np.tile((np.arange(C, dtype=np.int32) * 7) % (B + 1), (H, 1))
    ids = -100 - np.arange(C)[None, :].repeat(H, 0)
    st.set_persistent(Kp, Vp, pl, ids)
    c.set_persistent(gpu["wl"].bf16_tensor(Kp, DEV), gpu["wl"].bf16_tensor(Vp, DEV), torch.from_numpy(pl).to(DEV),
                     torch.from_numpy(ids))
    for g in range(2):
        Q, K, V = rnd(810 + 3 * g, H, Nq, d), rnd(811 + 3 * g, H, Nq, d), rnd(812 + 3 * g, H, Nq, d)
        _, got, ref = attend_both(gpu, c, st, Q, K, V, g, "100 slots")
        check_mass(got, ref, st, f"100 slots chunk {g}")
