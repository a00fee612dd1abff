"""GPU parity of pbsa_attention_bwd against the fp64 oracle backward, through the C ABI.

Bar (floating point, no integer decisions): for each of dQ, dK, dV the error against the fp64 oracle is bounded,
element by element, relative to the size of the tensor's entries: max-abs <= GRAD_MAX * max|ref| and mean-abs <=
GRAD_MEAN * mean|ref|.  The kernel's roundings: P = exp(z - lse) inherits the forward's lse (within 4e-3 of exact,
so every probability of a row is off by the same factor up to 4e-3), P and dZ are rounded to bf16 (2^-9 relative)
before the second products, D = dO . O uses the forward's bf16 O; sums are fp32.  A gradient entry is a sum of
hundreds to thousands of such terms with mixed signs, so the systematic part (the lse factor, <= 4e-3 of the
entry's scale) plus the bf16 rounding (2e-3) bounds the mean at 6e-3 of the mean entry, and the max is allowed 1e-2
of the largest entry (worst seen: 5.7e-3 and 4.3e-3).
"""
import math

import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle.rollout import OracleState, state_for_workload  # noqa: E402
from harness import synth  # noqa: E402
from tests.test_gpu_parity import DEV, compare_select, compare_update, rnd  # noqa: E402
from tests.test_gpu_parity_fine_mass import SMALL, chunk_lens, small_pair  # noqa: E402

pytestmark = pytest.mark.gpu

GRAD_MAX, GRAD_MEAN = 1e-2, 6e-3
SENTINEL = 7.0


@pytest.fixture(scope="module")
def gpu():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from harness import workloads
    from paper_2604_21221_amd import cache, pbsa
    pbsa.lib()
    return dict(cache=cache, pbsa=pbsa, wl=workloads)


def check_grad(got, ref, what):
    got = got.astype(np.float64)
    assert np.isfinite(got).all(), what
    err = np.abs(got - ref)
    scale_max, scale_mean = np.abs(ref).max(), np.abs(ref).mean()
    if scale_max == 0.0:
        assert err.max() == 0.0, what
        return
    print(f"{what}: max-abs err {err.max():.3e} ({err.max() / scale_max:.2e} of max|ref| {scale_max:.3e}), "
          f"mean-abs err {err.mean():.3e} ({err.mean() / scale_mean:.2e} of mean|ref|)", flush=True)
    assert err.max() <= GRAD_MAX * scale_max, what
    assert err.mean() <= GRAD_MEAN * scale_mean, what


def backward_both(gpu, c, st, Q, K, V, g, what, heads=None):
    """Append, select, attend on both sides, then the backward pass for a seeded dO.  heads: compare only these
    (the oracle then runs on their rows alone); None = all.  Returns nothing; asserts."""
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
    dO = rnd(900 + g, st.H, st.Nq, st.d)
    z = lambda *s: torch.full(s, SENTINEL, dtype=torch.float32, device=DEV)
    grads = dict(dQ=z(st.H, st.Nq, st.d), dKp=z(st.H, st.C + 1, st.B, st.d), dVp=z(st.H, st.C + 1, st.B, st.d),
                 dKl=z(st.H, st.cap, st.B, st.d), dVl=z(st.H, st.cap, st.B, st.d))
    c.attention_bwd(Qd, O, wl.bf16_tensor(dO, DEV), lse, grads)
    torch.cuda.synchronize()
    got = {k: v.cpu().numpy() for k, v in grads.items()}
    hs = list(range(st.H)) if heads is None else list(heads)
    mask = None
    if heads is not None:
        mask = np.zeros((st.H, st.Nq), bool)
        mask[hs] = True
    ref = dict(zip(("dQ", "dKp", "dVp", "dKl", "dVl"), st.attention_bwd(Q, dO, row_mask=mask)))
    l_map, l_len, _ = st._maps()
    for name in ("dQ", "dKp", "dVp"):
        check_grad(got[name][hs], ref[name][hs], f"{what} chunk {g} {name}")
    for name in ("dKl", "dVl"):              # the slots of the logical blocks (the others are checked below)
        check_grad(got[name][hs][:, l_map], ref[name][hs][:, l_map], f"{what} chunk {g} {name}")
    # every row of a logical block's slot is written: zeros past its length and for blocks nobody selected ...
    for h in hs:
        for l in range(st.n_loc):
            assert np.all(got["dKl"][h, l_map[l], l_len[l]:] == 0.0) and np.all(got["dVl"][h, l_map[l], l_len[l]:] == 0.0)
        unused = sorted(set(range(st.n_loc)) - set(int(x) for x in st.sel[h].ravel() if x >= 0))
        if unused:
            assert np.all(got["dKl"][h, l_map[unused]] == 0.0) and np.all(got["dVl"][h, l_map[unused]] == 0.0)
        for s in range(st.C + 1):
            assert np.all(got["dKp"][h, s, st.p_len[h, s]:] == 0.0) and np.all(got["dVp"][h, s, st.p_len[h, s]:] == 0.0)
    # ... and the physical slots that hold no logical block are left alone
    free = sorted(set(range(st.cap)) - set(int(x) for x in l_map))
    if free:
        assert np.all(got["dKl"][:, free] == SENTINEL) and np.all(got["dVl"][:, free] == SENTINEL)


@pytest.mark.parametrize("case", SMALL, ids=[c[0] for c in SMALL])
def test_backward_small_every_element(gpu, case):
    st, c = small_pair(gpu, case)
    name, H, d, B, Nq, w = case[:6]
    for g in range(w + 2):
        Q, K, V = rnd(40 + 3 * g, H, Nq, d), rnd(41 + 3 * g, H, Nq, d, scale=1.5), rnd(42 + 3 * g, H, Nq, d)
        backward_both(gpu, c, st, Q, K, V, g, f"bwd {name}")
        ne = st.n_evict_now()
        sc_ref, src_ref = st.update()
        assert c.update() == ne
        compare_update(c, st, gpu["wl"], sc_ref, src_ref, ne, name)


def test_backward_strided_inputs(gpu):
    """Q and O / dO as slices of packed tensors (token stride 3 d): same gradients as from dense copies."""
    H, d, B, Nq, w, C, k = 2, 128, 64, 200, 1, 2, 2
    scale = np.float32(1.0 / math.sqrt(d))
    c = gpu["cache"].PbsaCache(H, d, B, Nq, w, C, k, scale, device=DEV)
    wl = gpu["wl"]
    c.set_persistent(wl.bf16_tensor(rnd(1, H, C, B, d), DEV), wl.bf16_tensor(rnd(2, H, C, B, d), DEV),
                     torch.full((H, C), B, dtype=torch.int32, device=DEV), -100 - torch.arange(C)[None, :].repeat(H, 1))
    packed = torch.zeros(H, Nq, 3 * d, dtype=torch.bfloat16, device=DEV)
    packed[:, :, :d] = wl.bf16_tensor(rnd(50, H, Nq, d), DEV)
    Qs = packed[:, :, :d]
    c.append_chunk(wl.bf16_tensor(rnd(51, H, Nq, d), DEV), wl.bf16_tensor(rnd(52, H, Nq, d), DEV), 0)
    c.select(Qs)
    lse = torch.empty(H, Nq, dtype=torch.float32, device=DEV)
    out = torch.zeros(H, Nq, 3 * d, dtype=torch.bfloat16, device=DEV)
    Os = c.attention(Qs, O=out[:, :, d:2 * d], lse=lse)
    gpk = torch.zeros(H, Nq, 3 * d, dtype=torch.bfloat16, device=DEV)
    gpk[:, :, d:2 * d] = wl.bf16_tensor(rnd(53, H, Nq, d), DEV)
    g1 = c.attention_bwd(Qs, Os, gpk[:, :, d:2 * d], lse)
    g2 = c.attention_bwd(Qs.contiguous(), Os.contiguous(), gpk[:, :, d:2 * d].contiguous(), lse)
    torch.cuda.synchronize()
    for name in g1:
        assert torch.equal(g1[name], g2[name]), name


@pytest.mark.parametrize("name,heads", [("cfg2", (0, 11)), ("cfg5", (3,))])
def test_backward_full_size_sampled_heads(gpu, name, heads):
    """Full BASELINE shapes (cfg5: cold start through the first evicting update, then the full window); the oracle
    runs the rows of the sampled heads, whose dQ, dK and dV are compared in full."""
    w = synth.WORKLOADS[name]
    st, g0 = state_for_workload(w)
    c, _ = gpu["wl"].cache_for_workload(w, device=DEV)
    last = g0 if name == "cfg2" else 4
    for g in range(g0, last + 1):
        Q, K, V = synth.chunk_qkv(w, 0, g)
        if g == last:
            backward_both(gpu, c, st, Q, K, V, g, f"bwd {name}", heads=heads)
            break
        st.append_chunk(synth.to_blocks(K, st.B), synth.to_blocks(V, st.B), chunk_lens(st), g * st.nqb + np.arange(st.nqb))
        c.append_chunk(gpu["wl"].bf16_tensor(K, DEV), gpu["wl"].bf16_tensor(V, DEV), g)
        st.select(Q)
        c.select(gpu["wl"].bf16_tensor(Q, DEV))
        ne = st.n_evict_now()
        sc_ref, src_ref = st.update()
        assert c.update() == ne
        compare_update(c, st, gpu["wl"], sc_ref, src_ref, ne, name)


def test_backward_with_many_slots_and_all_blocks_selected(gpu):
    """Edge shapes of the lists the two kernels build: 100 persistent slots of every length (dq walks them all, dkv
    has a workgroup for each), and k larger than the number of local blocks (every block attended by every query
    block it is visible to)."""
    H, d, B, Nq, w, C, k = 1, 64, 64, 150, 1, 100, 64
    scale = np.float32(1.0 / math.sqrt(d))
    st = OracleState(H, d, B, Nq, w, C, k, scale)
    c = gpu["cache"].PbsaCache(H, d, B, Nq, w, C, k, scale, device=DEV)
    Kp, Vp = rnd(821, H, C, B, d), rnd(822, H, C, B, d)
    pl = np.tile((np.arange(C, dtype=np.int32) * 7) % (B + 1), (H, 1))
    ids = -100 - np.arange(C)[None, :].repeat(H, 0)
    st.set_persistent(Kp, Vp, pl, ids)
    c.set_persistent(gpu["wl"].bf16_tensor(Kp, DEV), gpu["wl"].bf16_tensor(Vp, DEV), torch.from_numpy(pl).to(DEV),
                     torch.from_numpy(ids))
    for g in range(2):
        Q, K, V = rnd(830 + 3 * g, H, Nq, d), rnd(831 + 3 * g, H, Nq, d), rnd(832 + 3 * g, H, Nq, d)
        backward_both(gpu, c, st, Q, K, V, g, "bwd 100 slots")
