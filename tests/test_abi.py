"""C-ABI checks that need no GPU: the library loads, exports what include/pbsa.h declares, and
rejects bad arguments on the host before any launch."""
import ctypes
import os
import re

import pytest

from paper_2604_21221_amd import pbsa

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(pbsa.LIB_PATH):
        from paper_2604_21221_amd import build
        build.build()
    return pbsa.lib()


def good(**kw):
    a = dict(H=2, d=128, B=64, Nq=200, n_loc=16, n_loc_cap=16, C=4, k=3, scale=0.088)
    a.update(kw)
    return pbsa.make_params(**a)


def test_exports_match_header(L):
    text = open(os.path.join(ROOT, "include", "pbsa.h")).read()
    declared = set(re.findall(r"\b(pbsa_[a-z_]+)\s*\(", text))
    assert declared == set(pbsa.EXPORTS)
    for name in declared:
        assert hasattr(L, name)
    assert pbsa.pbsa_version() >= 1
    assert ctypes.sizeof(pbsa.pbsa_params) == 92 or ctypes.sizeof(pbsa.pbsa_params) == 96
    for code in (0, -1, -2, -3, -4, -5, -99):
        assert isinstance(pbsa.pbsa_strerror(code), str) and pbsa.pbsa_strerror(code)


def test_header_constants_match_binding():
    text = open(os.path.join(ROOT, "include", "pbsa.h")).read()
    for name in ("PBSA_MAX_N_LOC", "PBSA_MAX_C", "PBSA_MAX_C_ATTEND", "PBSA_MAX_K", "PBSA_MAX_N_LOC_AUX",
                 "PBSA_MAX_C_AUX", "PBSA_MAX_K_AUX"):
        assert int(re.search(rf"#define {name}\s+(\d+)", text).group(1)) == getattr(pbsa, name)
    for name in ("PBSA_EINVAL", "PBSA_ESHAPE", "PBSA_EALIGN", "PBSA_EWS", "PBSA_EHIP"):
        assert int(re.search(rf"#define {name}\s+\((-\d+)\)", text).group(1)) == getattr(pbsa, name)


def test_workspace_bytes(L):
    n = pbsa.pbsa_workspace_bytes(good(n_evict=4))
    assert n >= 2 * 4 * (4 + 16) * 4 and n % 256 == 0
    with pytest.raises(pbsa.PbsaError) as e:
        pbsa.pbsa_workspace_bytes(good(d=96))
    assert e.value.code == pbsa.PBSA_ESHAPE


P = 0x10000  # a fake, 16-byte aligned, non-NULL device address: validation must fail before it is touched


def call_select(p, Q=P, Kl=P, l_len=P, l_map=P, Kc_l=P, Qc=P, sel=P):
    pbsa.pbsa_select_blocks(p, Q, Kl, l_len, l_map, Kc_l, Qc, sel, None, None, stream=0)


def call_attn(p, Q=P, Kp=P, Vp=P, p_len=P, Kl=P, Vl=P, l_len=P, l_map=P, sel=P, O=P):
    pbsa.pbsa_attention_fwd(p, Q, Kp, Vp, p_len, Kl, Vl, l_len, l_map, sel, O, None, None, stream=0)


def call_update(p, ws=(0x10000, 1 << 30), S_sum=P, S_cnt=P, Qc=P):
    pbsa.pbsa_memory_update(p, Qc, P, None, P, P, P, P, P, S_sum, S_cnt, P, P, P, P, P, None, P, ws, stream=0)


@pytest.mark.parametrize("kw,code", [
    (dict(d=96), pbsa.PBSA_ESHAPE), (dict(B=32), pbsa.PBSA_ESHAPE), (dict(k=673), pbsa.PBSA_ESHAPE),
    (dict(C=337), pbsa.PBSA_ESHAPE), (dict(n_loc=673, n_loc_cap=673), pbsa.PBSA_ESHAPE),
    (dict(H=65536), pbsa.PBSA_ESHAPE), (dict(H=40000, n_loc_cap=256, n_loc=16), pbsa.PBSA_ESHAPE),
    (dict(n_loc=2), pbsa.PBSA_EINVAL),               # fewer local blocks than the chunk itself has
    (dict(n_loc=17), pbsa.PBSA_EINVAL),              # more than the physical capacity
    (dict(n_sink=5), pbsa.PBSA_EINVAL), (dict(n_evict=17), pbsa.PBSA_EINVAL), (dict(causal=2), pbsa.PBSA_EINVAL),
    (dict(scale=0.0), pbsa.PBSA_EINVAL), (dict(H=0), pbsa.PBSA_EINVAL), (dict(pool_from=17), pbsa.PBSA_EINVAL),
    (dict(q_strides=(200 * 128, 100)), pbsa.PBSA_EINVAL), (dict(q_strides=(200 * 132, 132)), pbsa.PBSA_EALIGN),
])
def test_bad_params_rejected_by_every_call(L, kw, code):
    p = good(**kw)
    for call in (call_select, call_attn):
        with pytest.raises(pbsa.PbsaError) as e:
            call(p)
        assert e.value.code == code
    if "q_strides" not in kw:
        with pytest.raises(pbsa.PbsaError) as e:
            call_update(p)
        assert e.value.code == code


def test_summary_view_validates_before_touching_memory(L):
    for kw, args, code in [(dict(d=96), (P, P, P, P, P), pbsa.PBSA_ESHAPE), (dict(B=32), (P, P, P, P, P), pbsa.PBSA_ESHAPE),
                           (dict(), (None, P, P, P, P), pbsa.PBSA_EINVAL), (dict(), (P, P, P, P, None), pbsa.PBSA_EINVAL),
                           (dict(), (P + 4, P, P, P, P), pbsa.PBSA_EALIGN), (dict(), (P, P, P, P + 8, P), pbsa.PBSA_EALIGN),
                           (dict(C=337), (P, P, P, P, P), pbsa.PBSA_ESHAPE)]:
        with pytest.raises(pbsa.PbsaError) as e:
            pbsa.pbsa_summary_view(good(**kw), *args, stream=0)
        assert e.value.code == code


def test_only_selection_and_plain_attention_take_the_largest_shapes(L):
    """Between the two sets of limits: every call but pbsa_select_blocks and pbsa_attention_fwd refuses (that those two
    accept is a GPU test: with valid parameters they launch)."""
    for kw in (dict(k=513), dict(C=193), dict(n_loc=513, n_loc_cap=513)):
        p = good(**kw)
        with pytest.raises(pbsa.PbsaError) as e:
            call_update(p)
        assert e.value.code == pbsa.PBSA_ESHAPE
        for fn in (pbsa.pbsa_mass_workspace_bytes, pbsa.pbsa_bwd_workspace_bytes):
            with pytest.raises(pbsa.PbsaError) as e:
                fn(p)
            assert e.value.code == pbsa.PBSA_ESHAPE


def test_update_maintains_fewer_slots_than_attention_attends(L):
    """65..192 persistent slots: the update and its workspace refuse them (that selection and attention accept
    them is a GPU test: with valid parameters those calls launch)."""
    p = good(C=65)
    with pytest.raises(pbsa.PbsaError) as e:
        call_update(p)
    assert e.value.code == pbsa.PBSA_ESHAPE
    with pytest.raises(pbsa.PbsaError) as e:
        pbsa.pbsa_workspace_bytes(p)
    assert e.value.code == pbsa.PBSA_ESHAPE


def test_wrong_struct_size_and_nqb(L):
    p = good()
    p.size = 8
    with pytest.raises(pbsa.PbsaError) as e:
        call_select(p)
    assert e.value.code == pbsa.PBSA_EINVAL
    p = good()
    p.nqb = 3
    with pytest.raises(pbsa.PbsaError) as e:
        call_attn(p)
    assert e.value.code == pbsa.PBSA_EINVAL


def test_null_and_misaligned_pointers(L):
    p = good()
    with pytest.raises(pbsa.PbsaError) as e:
        call_select(p, Q=None)
    assert e.value.code == pbsa.PBSA_EINVAL
    with pytest.raises(pbsa.PbsaError) as e:
        call_select(p, Kl=P + 2)
    assert e.value.code == pbsa.PBSA_EALIGN
    with pytest.raises(pbsa.PbsaError) as e:
        call_attn(p, O=None)
    assert e.value.code == pbsa.PBSA_EINVAL
    with pytest.raises(pbsa.PbsaError) as e:
        call_attn(p, Vl=P + 8)
    assert e.value.code == pbsa.PBSA_EALIGN
    with pytest.raises(pbsa.PbsaError) as e:
        call_update(p, S_cnt=None)                 # S_sum without S_cnt
    assert e.value.code == pbsa.PBSA_EINVAL


def test_workspace_checks(L):
    p = good(n_evict=4)
    need = pbsa.pbsa_workspace_bytes(p)
    for ws in (None, (0x10000, need - 1)):
        with pytest.raises(pbsa.PbsaError) as e:
            call_update(p, ws=ws)
        assert e.value.code == pbsa.PBSA_EWS
    with pytest.raises(pbsa.PbsaError) as e:
        call_update(p, ws=(0x10010, need))
    assert e.value.code == pbsa.PBSA_EALIGN


def test_fine_mass_argument_checks(L):
    """pbsa_attention_mass and pbsa_memory_update_fine validate like the calls they sit beside."""
    p = good(n_evict=4)
    need = pbsa.pbsa_workspace_bytes(p)

    def mass(p=p, Q=P, lse=P, Mt=P):
        pbsa.pbsa_attention_mass(p, Q, P, P, P, P, P, P, lse, Mt, stream=0)

    def fine(p=p, Mt=P, ws=(0x10000, 1 << 30), S_cnt=P):
        pbsa.pbsa_memory_update_fine(p, Mt, P, P, P, P, P, P, P, S_cnt, P, P, P, P, P, None, P, ws, stream=0)

    def fused(p=p, lse=P, Mt=P, ws=(0x10000, 1 << 40)):
        pbsa.pbsa_attention_fwd_mass(p, P, P, P, P, P, P, P, P, P, P, lse, Mt, ws, stream=0)

    need_m = pbsa.pbsa_mass_workspace_bytes(p)
    # per 128 query rows: two waves x (C + 1 + min(2k, n_loc)) records of 256 bytes, and the tile list
    assert need_m >= 2 * 2 * 2 * (5 + 6) * 256 and need_m % 256 == 0
    with pytest.raises(pbsa.PbsaError) as e:
        pbsa.pbsa_mass_workspace_bytes(good(B=32))
    assert e.value.code == pbsa.PBSA_ESHAPE
    for call, kw, code in [(fused, dict(lse=None), pbsa.PBSA_EINVAL), (fused, dict(Mt=None), pbsa.PBSA_EINVAL),
                           (fused, dict(ws=None), pbsa.PBSA_EWS), (fused, dict(ws=(0x10000, need_m - 1)), pbsa.PBSA_EWS),
                           (fused, dict(ws=(0x10010, need_m)), pbsa.PBSA_EALIGN), (fused, dict(Mt=P + 4), pbsa.PBSA_EALIGN),
                           (fused, dict(p=good(C=193)), pbsa.PBSA_ESHAPE),
                           (mass, dict(lse=None), pbsa.PBSA_EINVAL), (mass, dict(Mt=None), pbsa.PBSA_EINVAL),
                           (mass, dict(Mt=P + 4), pbsa.PBSA_EALIGN), (mass, dict(Q=P + 2), pbsa.PBSA_EALIGN),
                           (mass, dict(p=good(d=96)), pbsa.PBSA_ESHAPE), (mass, dict(p=good(C=193)), pbsa.PBSA_ESHAPE),
                           (fine, dict(Mt=None), pbsa.PBSA_EINVAL), (fine, dict(S_cnt=None), pbsa.PBSA_EINVAL),
                           (fine, dict(Mt=P + 8), pbsa.PBSA_EALIGN), (fine, dict(ws=None), pbsa.PBSA_EWS),
                           (fine, dict(ws=(0x10000, need - 1)), pbsa.PBSA_EWS),
                           (fine, dict(p=good(C=65)), pbsa.PBSA_ESHAPE), (fine, dict(p=good(n_evict=17)), pbsa.PBSA_EINVAL)]:
        with pytest.raises(pbsa.PbsaError) as e:
            call(**kw)
        assert e.value.code == code, (call.__name__, kw)


def test_backward_argument_checks(L):
    p = good()
    need = pbsa.pbsa_bwd_workspace_bytes(p)
    assert need >= 2 * 200 * 4 and need % 256 == 0

    def bwd(p=p, dO=P, lse=P, dQ=P, dVl=P, ws=(0x10000, 1 << 30)):
        pbsa.pbsa_attention_bwd(p, P, P, P, P, P, P, P, P, P, P, dO, lse, dQ, P, P, P, dVl, ws, stream=0)

    for kw, code in [(dict(dO=None), pbsa.PBSA_EINVAL), (dict(lse=None), pbsa.PBSA_EINVAL), (dict(dVl=None), pbsa.PBSA_EINVAL),
                     (dict(dQ=P + 4), pbsa.PBSA_EALIGN), (dict(dO=P + 2), pbsa.PBSA_EALIGN), (dict(ws=None), pbsa.PBSA_EWS),
                     (dict(ws=(0x10000, need - 1)), pbsa.PBSA_EWS), (dict(ws=(0x10040, need)), pbsa.PBSA_EALIGN),
                     (dict(p=good(d=96)), pbsa.PBSA_ESHAPE), (dict(p=good(causal=2)), pbsa.PBSA_EINVAL),
                     (dict(p=good(q_strides=(1 << 30, 1 << 24))), pbsa.PBSA_ESHAPE)]:
        with pytest.raises(pbsa.PbsaError) as e:
            bwd(**kw)
        assert e.value.code == code, kw


def test_plan_and_apply_argument_checks(L):
    p = good(n_evict=4)
    need = pbsa.pbsa_workspace_bytes(p)

    def plan(p=p, Qc=P, p_len=P, ws=(0x10000, 1 << 30)):
        pbsa.pbsa_memory_update_plan(p, Qc, P, None, P, p_len, P, P, P, P, P, None, P, ws, stream=0)

    def apply(p=p, Kp=P, S_sum=P, S_cnt=P, ws=(0x10000, 1 << 30)):
        pbsa.pbsa_memory_update_apply(p, Kp, P, P, S_sum, S_cnt, P, P, ws, stream=0)

    for call, kw, code in [(plan, dict(Qc=None), pbsa.PBSA_EINVAL), (plan, dict(p_len=None), pbsa.PBSA_EINVAL),
                           (plan, dict(Qc=P + 4), pbsa.PBSA_EALIGN), (plan, dict(ws=None), pbsa.PBSA_EWS),
                           (plan, dict(ws=(0x10000, need - 1)), pbsa.PBSA_EWS), (plan, dict(p=good(C=65)), pbsa.PBSA_ESHAPE),
                           (apply, dict(Kp=None), pbsa.PBSA_EINVAL), (apply, dict(S_cnt=None), pbsa.PBSA_EINVAL),
                           (apply, dict(S_sum=P + 8), pbsa.PBSA_EALIGN), (apply, dict(ws=None), pbsa.PBSA_EWS),
                           (apply, dict(ws=(0x10080, need)), pbsa.PBSA_EALIGN), (apply, dict(p=good(n_evict=17)), pbsa.PBSA_EINVAL)]:
        with pytest.raises(pbsa.PbsaError) as e:
            call(**kw)
        assert e.value.code == code, (call.__name__, kw)


def test_attention_with_plan_argument_checks(L):
    """pbsa_attention_fwd_plan validates like pbsa_attention_fwd and pbsa_memory_update_plan together, and wants
    the logits of the selection call."""
    p = good(n_evict=4)
    need = pbsa.pbsa_workspace_bytes(p)

    def fused(p=p, Q=P, O=P, Qc=P, Zl=P, l_id=P, slot_src=P, ws=(0x10000, 1 << 30)):
        pbsa.pbsa_attention_fwd_plan(p, Q, P, P, P, P, P, P, P, P, O, None, Qc, P, Zl, P, P, P, l_id, None, slot_src, ws,
                                     stream=0)

    for kw, code in [(dict(Q=None), pbsa.PBSA_EINVAL), (dict(O=None), pbsa.PBSA_EINVAL), (dict(Zl=None), pbsa.PBSA_EINVAL),
                     (dict(l_id=None), pbsa.PBSA_EINVAL), (dict(slot_src=None), pbsa.PBSA_EINVAL),
                     (dict(Q=P + 2), pbsa.PBSA_EALIGN), (dict(Qc=P + 4), pbsa.PBSA_EALIGN), (dict(ws=None), pbsa.PBSA_EWS),
                     (dict(ws=(0x10000, need - 1)), pbsa.PBSA_EWS), (dict(ws=(0x10010, need)), pbsa.PBSA_EALIGN),
                     (dict(p=good(C=65)), pbsa.PBSA_ESHAPE), (dict(p=good(n_evict=17)), pbsa.PBSA_EINVAL),
                     (dict(p=good(q_strides=(200 * 132, 132))), pbsa.PBSA_EALIGN)]:
        with pytest.raises(pbsa.PbsaError) as e:
            fused(**kw)
        assert e.value.code == code, kw


def test_select_with_pending_apply_argument_checks(L):
    """pbsa_select_blocks_apply validates both halves and that the two parameter blocks describe the same cache."""
    p, pu = good(), good(n_evict=4)
    need = pbsa.pbsa_workspace_bytes(pu)

    def both(p=p, pu=pu, Q=P, Kp=P, S_sum=P, S_cnt=P, Vl=P, ws=(0x10000, 1 << 30)):
        pbsa.pbsa_select_blocks_apply(p, Q, P, P, P, P, P, P, None, pu, Kp, P, P, S_sum, S_cnt, Vl, ws, stream=0)

    for kw, code in [(dict(Q=None), pbsa.PBSA_EINVAL), (dict(Kp=None), pbsa.PBSA_EINVAL), (dict(Vl=None), pbsa.PBSA_EINVAL),
                     (dict(S_cnt=None), pbsa.PBSA_EINVAL), (dict(Q=P + 2), pbsa.PBSA_EALIGN), (dict(S_sum=P + 8), pbsa.PBSA_EALIGN),
                     (dict(ws=None), pbsa.PBSA_EWS), (dict(ws=(0x10000, need - 1)), pbsa.PBSA_EWS),
                     (dict(ws=(0x10040, need)), pbsa.PBSA_EALIGN), (dict(pu=good(n_evict=4, C=3)), pbsa.PBSA_EINVAL),
                     (dict(pu=good(n_evict=4, H=3)), pbsa.PBSA_EINVAL), (dict(pu=good(C=65)), pbsa.PBSA_ESHAPE),
                     (dict(p=good(k=513)), pbsa.PBSA_ESHAPE), (dict(pu=good(n_evict=17)), pbsa.PBSA_EINVAL)]:
        with pytest.raises(pbsa.PbsaError) as e:
            both(**kw)
        assert e.value.code == code, kw


def test_binding_refuses_host_tensors(L):
    import torch
    with pytest.raises(TypeError):
        pbsa.pbsa_select_blocks(good(), torch.zeros(4), P, P, P, P, P, P, None, None, stream=0)


def test_blockify_argument_checks(L):
    """Grid and pointer validation of the rearrange calls; no GPU needed (validation precedes any HIP call)."""
    import ctypes
    vp = ctypes.c_void_p
    good = dict(T=3, Hs=8, Ws=8, Bt=1, Bh=8, Bw=8, H=2, d=128, B=64)
    X = (vp * 1)(0x1000)
    Y = (vp * 1)(0x2000)
    st = (ctypes.c_int64 * 1)(64 * 128 * 3)

    def call(**kw):
        g = pbsa.make_grid(**{**good, **kw})
        return L.pbsa_blockify(ctypes.byref(g), 1, X, Y, st, None)

    assert call(Bh=3) == pbsa.PBSA_ESHAPE            # block shape must divide the grid
    assert call(Bt=2) == pbsa.PBSA_ESHAPE
    assert call(B=63) == pbsa.PBSA_ESHAPE            # a slot must hold a block
    assert call(d=12) == pbsa.PBSA_ESHAPE
    assert call(T=0) == pbsa.PBSA_EINVAL
    g = pbsa.make_grid(**good)
    assert L.pbsa_blockify(ctypes.byref(g), 0, X, Y, st, None) == pbsa.PBSA_EINVAL
    assert L.pbsa_blockify(ctypes.byref(g), 5, X, Y, st, None) == pbsa.PBSA_EINVAL
    assert L.pbsa_blockify(ctypes.byref(g), 1, None, Y, st, None) == pbsa.PBSA_EINVAL
    bad = (vp * 1)(0x1004)
    assert L.pbsa_blockify(ctypes.byref(g), 1, bad, Y, st, None) == pbsa.PBSA_EALIGN
    st_bad = (ctypes.c_int64 * 1)(7)
    assert L.pbsa_blockify(ctypes.byref(g), 1, X, Y, st_bad, None) == pbsa.PBSA_EALIGN
    g.size = 4
    assert L.pbsa_blockify(ctypes.byref(g), 1, X, Y, st, None) == pbsa.PBSA_EINVAL
    g = pbsa.make_grid(**good)
    assert L.pbsa_unblockify(ctypes.byref(g), None, 0, vp(0x1000), None) == pbsa.PBSA_EINVAL
    assert L.pbsa_unblockify(ctypes.byref(g), vp(0x1008), 0, vp(0x1000), None) == pbsa.PBSA_EALIGN
