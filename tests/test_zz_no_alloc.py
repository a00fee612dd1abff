"""pbsa_memory_update_static (the update on the library's built-in scratch, for callers that cannot allocate) against
pbsa_memory_update with a caller workspace: the same kernels on another scratch address, so every output is compared bit
for bit.  Two roll-outs in a row through the C ABI, the second smaller than the first (what the first left in the
shared scratch must not matter)."""
import math

import numpy as np
import pytest

torch = pytest.importorskip("torch")

from harness import synth  # noqa: E402

DEV = "cuda:0"

STATE = ("Kp", "Vp", "Kc_p", "p_len", "p_id", "S_sum", "S_cnt", "scores", "slot_src")


def _bits(t):
    t = t.detach().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy()
    if t.dtype == torch.float32:
        return t.view(torch.int32).cpu().numpy()
    return t.cpu().numpy()


def _rollout(cache, pbsa, wl, H, d, B, Nq, w, C, k, n_chunks, seed):
    scale = np.float32(1.0 / math.sqrt(d))
    a = cache.PbsaCache(H, d, B, Nq, w, C, k, scale, device=DEV)     # workspace from the caller
    b = cache.PbsaCache(H, d, B, Nq, w, C, k, scale, device=DEV)     # the library's scratch
    full = pbsa.make_params(H, d, B, Nq, a.cap, a.cap, C, k, scale, n_evict=a.nqb)
    assert pbsa.pbsa_workspace_bytes(full) <= pbsa.PBSA_STATIC_WS_BYTES
    evictions = 0
    for g in range(n_chunks):
        print(f"[case] static scratch H={H} d={d} B={B} Nq={Nq} chunk {g}", flush=True)
        key = synth.stream_key(seed, "misc", 100 + g)
        x = synth.to_bf16_bits(synth.normals(key, 3 * H * Nq * d).reshape(3, H, Nq, d))
        Q, K, V = (wl.bf16_tensor(x[i], DEV) for i in range(3))
        for c in (a, b):
            c.append_chunk(K, V, g)
            c.select(Q)
        ne = a.update()
        assert b.update(static_scratch=True) == ne
        evictions += ne
        torch.cuda.synchronize()
        for name in STATE:
            ta, tb = getattr(a, name), getattr(b, name)
            assert np.array_equal(_bits(ta), _bits(tb)), f"{name} differs at chunk {g}"
    assert evictions > 0, "the roll-out must reach the steady state (evictions, fold, promote)"


@pytest.mark.gpu
def test_static_scratch_matches_workspace_twice_second_smaller():
    assert torch.cuda.is_available(), "this test needs the MI355X"
    from harness import workloads
    from paper_2604_21221_amd import cache, pbsa
    pbsa.lib()
    _rollout(cache, pbsa, workloads, H=3, d=128, B=64, Nq=333, w=2, C=4, k=5, n_chunks=5, seed=11)
    _rollout(cache, pbsa, workloads, H=1, d=64, B=64, Nq=130, w=1, C=2, k=2, n_chunks=4, seed=12)


def test_static_scratch_refuses_what_does_not_fit():
    from paper_2604_21221_amd import pbsa
    pbsa.lib()
    # 48 heads x (64 + 512) score columns x 128 query blocks of fp32 rows: far beyond the built-in scratch
    p = pbsa.make_params(48, 128, 64, 128 * 64, 512, 512, 64, 8, 0.1, n_evict=128)
    assert pbsa.pbsa_workspace_bytes(p) > pbsa.PBSA_STATIC_WS_BYTES
    fake = 1 << 20        # validation only looks at NULL-ness and alignment; nothing is enqueued
    with pytest.raises(pbsa.PbsaError) as e:
        pbsa.pbsa_memory_update_static(p, *([fake] * 17), stream=0)
    assert e.value.code == pbsa.PBSA_EWS
