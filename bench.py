#!/usr/bin/env python3
"""Benchmark of the PBSA layer-chunk step on one MI355X.

A step is one pass of the whole hot path over one chunk of synthetic input, all resident in HBM:
pbsa_select_blocks -> pbsa_attention_fwd -> pbsa_memory_update, enqueued back to back on one stream.
Prints ONE JSON line: effective TFLOP/s on the executed (sparse) attention FLOPs over the whole step,
ms per step, the roofline of the dominant kernel (attention, bf16 MFMA) from HIP events recorded
around that kernel inside the timed region, and the CPU oracle timed on a bounded sample.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E

def hbm_traffic_bytes(workload):
    """HBM-side bytes per attention launch from the hardware counters (rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE,
    KiB per dispatch, each scaled by what the same counter reads for a 1 GiB copy).  Counters cannot be read from
    inside this process, so the figure is taken from the committed summary of the profile runs of this same command,
    profiles/attention_<workload>_hbm_counters.txt (its line "-> F KiB * a + W KiB * b = ..."); None without one."""
    import re
    path = os.path.join(ROOT, "profiles", f"attention_{workload}_hbm_counters.txt")
    try:
        m = re.search(r"->\s*([\d,]+) KiB \* ([\d.]+) \+ ([\d,]+) KiB \* ([\d.]+)", open(path).read())
    except OSError:
        return None
    if not m:
        return None
    f, a, w, b = (float(x.replace(",", "")) for x in m.groups())
    return int((f * a + w * b) * 1024)


def executed_flops(sel, p_len, l_len_by_block, rows_per_qblock, d):
    """4 d sum_h sum_i rows_i (valid persistent tokens + valid tokens of the selected blocks)."""
    import torch
    persistent = p_len.to(torch.int64).sum(1)                                   # [H]
    ok = sel >= 0
    lens = l_len_by_block.to(torch.int64)[sel.clamp(min=0).to(torch.int64)] * ok
    per_qblock = lens.sum(2) + persistent[:, None]                              # [H][nqb]
    return int(4 * d * (per_qblock * rows_per_qblock[None, :].to(torch.int64)).sum().item())


def cpu_baseline(w, n_rows=1536):
    """The oracle on the host cores: one full selection and update plus attention on a sample of rows,
    attention scaled to the whole chunk.  Runs on a steady-state state reached by the oracle itself."""
    import numpy as np
    from oracle import rollout
    from harness import synth
    st, g0 = rollout.state_for_workload(w)
    lens = synth.block_lens(w)
    n_setup = (w.window_chunks + 2) if w.cold_start else 1
    for g in range(g0, g0 + n_setup):
        Q, K, V = synth.chunk_qkv(w, 0, g)
        st.append_chunk(synth.to_blocks(K, w.B), synth.to_blocks(V, w.B), lens, g * w.nqb + np.arange(w.nqb))
        st.select(Q)
        st.update()
    g = g0 + n_setup
    Q, K, V = synth.chunk_qkv(w, 0, g)
    st.append_chunk(synth.to_blocks(K, w.B), synth.to_blocks(V, w.B), lens, g * w.nqb + np.arange(w.nqb))
    t0 = time.perf_counter()
    st.select(Q)
    t_sel = time.perf_counter() - t0
    per_head = n_rows // w.H
    hh = np.repeat(np.arange(w.H, dtype=np.int32), per_head)
    tt = np.tile(np.linspace(0, w.Nq - 1, per_head).astype(np.int32), w.H)
    t0 = time.perf_counter()
    st.attention_rows(Q, hh, tt)
    t_att = (time.perf_counter() - t0) * (w.H * w.Nq) / len(hh)
    t0 = time.perf_counter()
    st.update()
    t_upd = time.perf_counter() - t0
    return t_sel, t_att, t_upd, len(hh)


def sweep_kernel_grid(dev, reps=20):
    """pbsa_attention_fwd alone (block sets from pbsa_select_blocks on the same synthetic inputs) on the
    kernel-benchmark shapes of the paper's appendix: N_C = 5376 or 21504 query tokens (3 or 12 frames of
    1792 tokens), local KV N_L = 2 or 4 N_C, persistent KV N_P = 0.25 or 0.5 N_L, 12 heads of 128 (the
    paper does not state heads), blocks of 128: all eight shapes of the table.  The dense stand-in is the same
    kernel with every visible block selected (block-causal within the chunk)."""
    import numpy as np
    import torch
    from harness import synth, workloads
    rows = []
    memo = {}
    gen_qkv, gen_pers = synth.chunk_qkv, synth.persistent_init

    def once(fn, tag):
        # the inputs do not depend on top-k: generate them once per shape
        def wrapped(w, *a):
            key = (tag, w.chunk_frames, w.window_chunks, w.C) + a
            if key not in memo:
                memo[key] = fn(w, *a)
            return memo[key]
        return wrapped
    synth.chunk_qkv, synth.persistent_init = once(gen_qkv, "qkv"), once(gen_pers, "pers")
    for frames, ratio_l, ratio_p in ((3, 2, 0.25), (3, 2, 0.5), (3, 4, 0.25), (3, 4, 0.5), (12, 2, 0.25), (12, 2, 0.5),
                                     (12, 4, 0.25), (12, 4, 0.5)):
        dense_us = None
        memo.clear()
        for topk in (1.0, 0.25, 0.125, 0.0625):
            w = synth.t7_workload(ratio_l, ratio_p, topk, frames=frames)
            c, g0 = workloads.cache_for_workload(w, device=dev, fold=False)
            Q, Kc, Vc = synth.chunk_qkv(w, 0, g0)
            Qd = workloads.bf16_tensor(Q, dev)
            c.append_chunk(workloads.bf16_tensor(Kc, dev), workloads.bf16_tensor(Vc, dev), g0)
            c.select(Qd)
            O = torch.empty_like(Qd)
            for _ in range(60):                # enough load for the GPU's clocks to settle
                c.attention(Qd, O)
            ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
            for a, b in ev:
                a.record()
                c.attention(Qd, O)
                b.record()
            torch.cuda.synchronize()
            us = float(np.median([a.elapsed_time(b) for a, b in ev])) * 1e3
            print(f"[sweep] {w.name}: {us:.1f} us", file=sys.stderr, flush=True)
            lens = torch.from_numpy(np.tile(synth.block_lens(w), w.window_chunks + 1)).to(dev)
            flops = executed_flops(c.sel, c.p_len, lens, torch.from_numpy(synth.block_lens(w)).to(dev), w.d)
            if topk >= 1.0:
                dense_us = us
            rows.append({"N_C": w.Nq, "N_L": w.n_loc * w.B, "N_P": w.C * w.B, "N_KV": (w.C + w.n_loc) * w.B,
                         "top_k_pct": 100 * topk, "k_blocks": w.k, "us": round(us, 1),
                         "tflops_executed": round(flops / us / 1e6, 1),
                         "speedup_vs_all_blocks": round(dense_us / us, 2)})
            del c
            torch.cuda.empty_cache()
    synth.chunk_qkv, synth.persistent_init = gen_qkv, gen_pers
    return {"metric": "pbsa_attention_fwd latency on the paper's kernel-benchmark shapes (forward)", "unit": "us",
            "config": {"workload": "N_C=5376 / 21504 (3 / 12 frames of 1792 tokens), H=12, d=128, B=128; synthetic bf16 inputs"},
            "data": "synthetic", "dtype": "bf16", "n_gpus": 1, "rows": rows}


def bench_blockify(dev, reps=50):
    """pbsa_blockify on a chunk of the paper's kernel-benchmark geometry (3 frames of 56 x 32 patches =
    5376 tokens, 12 heads of 128): Q, K and V rearranged in one launch, K and V straight into a ring
    position of a cache; then pbsa_unblockify of an output.  A permutation: algorithmic bytes = every
    byte read once and written once."""
    import numpy as np
    import torch
    from paper_2604_21221_amd import pbsa
    from oracle import blockify as ob
    T, Hs, Ws, H, d, B = 3, 56, 32, 12, 128, 64
    rows = []
    for Bt, Bh, Bw in ((1, 8, 8), (3, 4, 4)):
        g = pbsa.make_grid(T, Hs, Ws, Bt, Bh, Bw, H, d, B)
        nb = (T // Bt) * (Hs // Bh) * (Ws // Bw)
        X = [torch.randn(T, Hs, Ws, H, d, device=dev).to(torch.bfloat16) for _ in range(3)]
        cap = 4 * nb
        Kl = torch.zeros(H, cap, B, d, dtype=torch.bfloat16, device=dev)
        Vl = torch.zeros_like(Kl)
        Qb = torch.zeros(H, nb, B, d, dtype=torch.bfloat16, device=dev)
        O = torch.empty(T, Hs, Ws, H, d, dtype=torch.bfloat16, device=dev)
        fwd = lambda: pbsa.pbsa_blockify(g, X, [Qb, Kl[:, nb:], Vl[:, nb:]], [nb * B * d, cap * B * d, cap * B * d])
        inv = lambda: pbsa.pbsa_unblockify(g, Qb, nb * B * d, O)
        out = {}
        for name, fn, n_t in (("pbsa_blockify", fwd, 3), ("pbsa_unblockify", inv, 1)):
            for _ in range(100):
                fn()
            ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
            for a, b in ev:
                a.record()
                fn()
                b.record()
            torch.cuda.synchronize()
            us = float(np.median([a.elapsed_time(b) for a, b in ev])) * 1e3
            nbytes = 2 * n_t * T * Hs * Ws * H * d * 2
            out[name] = {"us": round(us, 2), "algorithmic_bytes": nbytes, "achieved": round(nbytes / us / 1e3, 1),
                         "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": round(nbytes / us / 1e3 / PEAK_HBM_GBS, 4)}
        assert torch.equal(O, X[0]), "rearrange and its inverse do not give the input back"
        xh = X[1].cpu().view(torch.int16).numpy()
        t0 = time.perf_counter()
        ref = ob.blockify(xh, Bt, Bh, Bw)
        t_cpu = time.perf_counter() - t0
        assert np.array_equal(Kl[:, nb:2 * nb, :Bt * Bh * Bw].cpu().view(torch.int16).numpy(), ref)
        out["cpu_oracle_us_per_tensor"] = round(t_cpu * 1e6, 1)
        rows.append({"block": [Bt, Bh, Bw], "n_blocks": nb, **out})
    return {"metric": "pbsa_blockify / pbsa_unblockify achieved HBM GB/s (bytes read + written)", "unit": "GB/s",
            "config": {"workload": "chunk of 3 x 56 x 32 tokens, H=12, d=128, block slots of 64 rows; Q, K, V in one launch"},
            "data": "synthetic", "dtype": "bf16", "n_gpus": 1, "rows": rows}


def bench_backward(w, c, Q_at, g_next, n_ring, dev, K, W, settle):
    """pbsa_attention_bwd on the steady-state cache of workload w: one selection + forward, then the backward
    call repeated on the same inputs (it changes nothing it reads)."""
    import numpy as np
    import torch
    from harness import synth, workloads
    c.adopt_chunk(g_next)
    Qd = Q_at[(c.n_appended - 1) % n_ring]
    c.select(Qd)
    lse = torch.empty(w.H, w.Nq, dtype=torch.float32, device=dev)
    O = c.attention(Qd, lse=lse)
    dO = workloads.bf16_tensor(synth.to_bf16_bits(synth.normals(synth.stream_key(w.seed, "misc", 99), w.H * w.Nq * w.d)
                                                  .reshape(w.H, w.Nq, w.d)), dev)
    grads = c.attention_bwd(Qd, O, dO, lse)
    stream = torch.cuda.current_stream()
    for _ in range(settle // 3 + W):
        c.attention_bwd(Qd, O, dO, lse, grads)
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(K)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for a, b in ev:
        a.record(stream)
        c.attention_bwd(Qd, O, dO, lse, grads)
        b.record(stream)
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) / K
    us = sum(a.elapsed_time(b) for a, b in ev) / K * 1e3
    rows = torch.from_numpy(synth.block_lens(w)).to(dev)
    l_len = torch.from_numpy(np.tile(synth.block_lens(w), n_ring)).to(dev)
    fwd = executed_flops(c.sel, c.p_len, l_len, rows, w.d)
    flops = 2.5 * fwd          # five products of the size of the forward's two: dV, dP, dQ, dK and the recomputed scores
    out_bytes = 4 * (w.H * w.Nq * w.d + 2 * w.H * (w.C + 1 + n_ring * w.nqb) * w.B * w.d)
    return {"metric": "pbsa_attention_bwd: effective TFLOP/s on 2.5 x the executed forward FLOPs", "value": round(flops / us / 1e6, 3),
            "unit": "TFLOP/s", "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": round(us / 1e3, 5),
            "wall_ms_per_call": round(wall * 1e3, 5), "higher_is_better": True, "dtype": "bf16", "data": "synthetic",
            "config": {"workload": f"{w.name} steady state, backward of one attention call: H={w.H} d={w.d} B={w.B} "
                                   f"Nq={w.Nq} C={w.C}+summary k={w.k}", "executed_gflop": round(flops / 1e9, 3),
                       "kernels": "bwd_prep_kernel, bwd_dq_kernel, bwd_dkv_kernel", "gradient_bytes_written": out_bytes},
            "roofline": {"bound": "mfma", "achieved": round(flops / us / 1e6, 3), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                         "frac": round(flops / us / 1e6 / PEAK_BF16_TFLOPS, 5), "traffic": None}}


def bench_steps(w, args, K, W, settle, dev, layers=None):
    """The step benchmark on workload w: K timed steps after `settle` + W untimed ones, on `layers` layers (the
    workload's own count unless given).  Returns the fields of the JSON line (no CPU baseline)."""
    import numpy as np
    import torch
    from harness import synth, workloads

    # ---- state: reach steady state (full window, full persistent set, non-empty summary) untimed ----
    # one cache and one set of inputs per layer; a step visits the layers in turn
    L, T = layers or w.n_layers, max(1, args.denoise_steps)
    n_ring = w.window_chunks + 1               # chunks in the local region during a step
    chained = not (args.three_launches or args.separate_update or args.fine_mass or args.backward)
    n_pos = n_ring + 1 if chained else n_ring  # ring positions
    n_setup = n_pos + 2 if w.cold_start else n_pos
    caches, Q_ats = [], []
    for layer in range(L):
        cl, g0 = workloads.cache_for_workload(w, layer=layer, device=dev, ring_chunks=n_pos)
        Q_at = {}              # ring position -> the query chunk that goes with the K/V sitting there
        for g in range(g0, g0 + n_setup):
            Q, Kc, Vc = synth.chunk_qkv(w, layer, g)
            Qd = workloads.bf16_tensor(Q, dev)
            cl.step(Qd, workloads.bf16_tensor(Kc, dev), workloads.bf16_tensor(Vc, dev), g)
            Q_at[(cl.n_appended - 1) % n_pos] = Qd
        caches.append(cl)
        Q_ats.append(Q_at)
    c = caches[0]
    g_next = g0 + n_setup
    torch.cuda.synchronize()

    if args.backward:
        return bench_backward(w, caches[0], Q_ats[0], g_next, n_ring, dev, K, W, settle)
    O = torch.empty(w.H, w.Nq, w.d, dtype=torch.bfloat16, device=dev)
    K2 = min(K, 20)            # extra steps after the timed region: per-call split of select and update
    n_total = W + K + K2
    sel_hist = torch.full((n_total,) + tuple(c.sel.shape), -1, dtype=torch.int32, device=dev)
    src_hist = torch.full((n_total,) + tuple(c.slot_src.shape), -1, dtype=torch.int32, device=dev)
    plen_hist = torch.zeros((n_total,) + tuple(c.p_len.shape), dtype=torch.int32, device=dev)
    new_ev = lambda n: [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
    ev, ev_sel, ev_upd, ev_mass = new_ev(K), new_ev(K2), new_ev(K2), new_ev(K2)
    lse = torch.empty(w.H, w.Nq, dtype=torch.float32, device=dev) if args.fine_mass else None
    Mt_pass = (torch.zeros(w.H, w.C + 1 + n_ring * w.nqb, (w.nqb + 3) & ~3, dtype=torch.float32, device=dev)
               if args.fine_mass else None)
    stream = torch.cuda.current_stream()

    n_done = [0]
    fused = not (args.separate_update or args.fine_mass)

    def one_step(i, attn_ev=None, sel_ev=None, upd_ev=None, mass_ev=None):
        # the producer has written the next chunk's K/V into the ring position that was just freed
        # (here: the data already there serves as the new chunk); its queries are the matching Q.
        # i is the row of the history buffers this step records into.
        g = g_next + n_done[0] // L
        c = caches[n_done[0] % L]
        n_done[0] += 1
        c.adopt_chunk(g)
        Qd = Q_ats[(n_done[0] - 1) % L][(c.n_appended - 1) % n_pos]
        c.sel, c.slot_src = sel_hist[i], src_hist[i]
        for _ in range(T - 1):
            # earlier denoising passes of this chunk: the chunk's own K/V (and so its pooled keys) change
            # from pass to pass, everything else in the cache stays
            c.select(Qd)
            c.attention(Qd, O)
            c.rewrite_chunk()
        if sel_ev is not None:
            sel_ev[0].record(stream)
        c.select(Qd)
        if sel_ev is not None:
            sel_ev[1].record(stream)
        plen_hist[i].copy_(c.p_len, non_blocking=True)
        if attn_ev is not None:
            attn_ev[0].record(stream)
        if args.fine_mass:
            _, Mt = c.attention_with_mass(Qd, O, lse)      # the attention kernel records the masses, a short kernel sums them
        elif fused:
            c.attention_with_plan(Qd, O)                   # scoring and retention by extra workgroups of this launch
        else:
            c.attention(Qd, O)
        if attn_ev is not None:
            attn_ev[1].record(stream)
        if args.fine_mass and mass_ev is not None:
            # for comparison only (the step does not need it): the same matrix by a separate pass over the keys
            mass_ev[0].record(stream)
            c.attention_mass(Qd, lse, Mt_pass)
            mass_ev[1].record(stream)
        if upd_ev is not None:
            upd_ev[0].record(stream)
        if args.fine_mass:
            c.update_fine(Mt)
        elif chained:
            c.defer_apply()                        # fold / promote ride in the next step's selection call
        elif fused:
            c.update_apply()
        else:
            c.update()
        if upd_ev is not None:
            upd_ev[1].record(stream)

    # The engine clock of an idle GPU takes some tens of milliseconds of load to settle (the first
    # ~50 steps run about 10 % slower): bring it there before the W warm-up steps, whatever W is.
    for _ in range(settle):
        one_step(0)
    for i in range(W):
        one_step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(K):
        one_step(W + i, attn_ev=ev[i])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for i in range(K2):
        one_step(W + K + i, sel_ev=ev_sel[i], upd_ev=ev_upd[i], mass_ev=ev_mass[i])
    for cl in caches:
        cl.flush()
    torch.cuda.synchronize()

    step_s = (t1 - t0) / K
    attn_ms = sum(a.elapsed_time(b) for a, b in ev) / K                 # the last pass's launch
    rows = torch.from_numpy(synth.block_lens(w)).to(dev)
    # lengths by logical block are the same for every arrangement (each chunk has the same block lens)
    l_len = torch.from_numpy(np.tile(synth.block_lens(w), n_ring)).to(dev)
    flops = [executed_flops(sel_hist[W + i], plen_hist[W + i], l_len, rows, w.d) for i in range(K)]
    mean_flops = float(np.mean(flops)) * T
    tflops_step = mean_flops / step_s / 1e12
    tflops_attn = mean_flops / T / (attn_ms * 1e-3) / 1e12

    # HBM-bound calls: algorithmic bytes over the event-bracketed duration.  Selection reads the chunk's
    # Q and K once and writes sel and the logits; the update reads the logits, reads K and V of every
    # folded block, reads and writes K and V of every promoted block and the summary sums and slot.
    sel_us = sum(a.elapsed_time(b) for a, b in ev_sel) / K2 * 1e3
    upd_us = sum(a.elapsed_time(b) for a, b in ev_upd) / K2 * 1e3
    blk = w.B * w.d * 2
    n_loc = n_ring * w.nqb
    sel_bytes = 2 * w.H * w.Nq * w.d * 2 + w.H * w.nqb * (w.k + n_loc) * 4
    upd_bytes = []
    for i in range(W + K, n_total):
        occupied = int((plen_hist[i][:, :w.C] > 0).sum().item())
        promoted = int((src_hist[i] >= 0).sum().item())
        folded = occupied + w.H * w.nqb - min(w.H * w.C, occupied + w.H * w.nqb)
        # what the ranking reads: the coarse logits, or the candidates' rows of the mass matrix
        ranked = (w.H * (w.C + w.nqb) * ((w.nqb + 3) & ~3) * 4 if args.fine_mass else
                  0 if fused else w.H * w.nqb * n_loc * 4)      # the apply call reads no scores
        upd_bytes.append(ranked + folded * 2 * blk + promoted * 4 * blk
                         + w.H * (2 * 2 * w.B * w.d * 4 + 2 * blk))
    upd_b = float(np.mean(upd_bytes))

    out = {
        "metric": "effective TFLOP/s on executed (sparse) attention FLOPs per layer-chunk step (select+attention+update)",
        "value": round(tflops_step, 3), "unit": "TFLOP/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": round(step_s * 1e3, 5), "us_per_layer_chunk": round(step_s * 1e6, 2),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "pct_bf16_mfma_peak_step": round(100 * tflops_step / PEAK_BF16_TFLOPS, 3),
        "config": {"workload": f"{w.name} steady state: H={w.H} d={w.d} B={w.B} Nq={w.Nq} C={w.C}+summary "
                               f"window={w.window_chunks} chunks ({w.n_win} blocks) k={w.k}",
                   "layers": L, "denoise_steps": T, "executed_gflop_per_step": round(mean_flops / 1e9, 3)},
        "roofline": {"kernel": "pbsa_attention_fwd", "bound": "mfma", "achieved": round(tflops_attn, 3),
                     "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(tflops_attn / PEAK_BF16_TFLOPS, 5),
                     "traffic": hbm_traffic_bytes(w.name), "traffic_unit": "bytes per launch",
                     "us_per_launch": round(attn_ms * 1e3, 2)},
        "hbm_bound_calls": {
            "pbsa_select_blocks": {"us_per_call": round(sel_us, 2), "algorithmic_bytes": sel_bytes,
                                   "achieved": round(sel_bytes / sel_us / 1e3, 1), "peak": PEAK_HBM_GBS,
                                   "unit": "GB/s", "frac": round(sel_bytes / sel_us / 1e3 / PEAK_HBM_GBS, 4)},
            "pbsa_memory_update": {"us_per_call": round(upd_us, 2), "algorithmic_bytes": int(upd_b),
                                   "achieved": round(upd_b / upd_us / 1e3, 1), "peak": PEAK_HBM_GBS,
                                   "unit": "GB/s", "frac": round(upd_b / upd_us / 1e3 / PEAK_HBM_GBS, 4)},
            "note": f"{K2} steps after the timed region, HIP events around each call"},
    }
    if fused:
        out["config"]["schedule"] = ("pbsa_select_blocks -> pbsa_attention_fwd_plan (attention + one workgroup per head taking the "
                                     "update's decisions, Eq. 7-9) -> pbsa_memory_update_apply (fold, promote)")
        out["roofline"]["kernel"] = ("pbsa_attention_fwd_plan: the attention kernel's launch, FLOPs of the attention only "
                                     "(the decision workgroups run on SIMDs the attention leaves free)")
        u = out["hbm_bound_calls"].pop("pbsa_memory_update")
        u["note"] = "the apply call alone; the decisions are taken inside the attention launch"
        out["hbm_bound_calls"]["pbsa_memory_update_apply"] = u
    if chained:
        out["config"]["schedule"] = ("pbsa_select_blocks_apply (selection + fold / promote of the previous step's update in its pooling "
                                     "launch; ring of window + 2 chunks) -> pbsa_attention_fwd_plan (attention + the update's decisions)")
        out["hbm_bound_calls"].pop("pbsa_memory_update_apply")
        u = out["hbm_bound_calls"].pop("pbsa_select_blocks")
        u["algorithmic_bytes"] += int(upd_b)
        u["achieved"] = round(u["algorithmic_bytes"] / u["us_per_call"] / 1e3, 1)
        u["frac"] = round(u["achieved"] / PEAK_HBM_GBS, 4)
        out["hbm_bound_calls"]["pbsa_select_blocks_apply"] = u
    if args.fine_mass:
        mass_us = sum(a.elapsed_time(b) for a, b in ev_mass) / K2 * 1e3
        qk_flops = mean_flops / T / 2          # the first product of the attention only
        out["metric"] = out["metric"].replace("select+attention+update", "select+attention with mass+update by mass")
        out["roofline"]["kernel"] = "pbsa_attention_fwd_mass (attention kernel recording row sums + the kernel that sums them)"
        out["hbm_bound_calls"]["pbsa_memory_update_fine"] = out["hbm_bound_calls"].pop("pbsa_memory_update")
        out["fine_mass"] = {"note": "the step uses pbsa_attention_fwd_mass; the separate pass below is timed beside it",
                            "pbsa_attention_mass": {
            "us_per_call": round(mass_us, 2), "executed_gflop": round(qk_flops / 1e9, 3),
            "achieved": round(qk_flops / mass_us / 1e6, 3), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
            "frac": round(qk_flops / mass_us / 1e6 / PEAK_BF16_TFLOPS, 5), "bound": "mfma"}}
    out["_mean_flops"], out["_T"] = mean_flops, T
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="cfg5", choices=["cfg2", "cfg3", "cfg4", "cfg5"],
                    help="cfg3: the shapes of cfg2 on 30 layers, each with its own cache and inputs, visited in turn")
    ap.add_argument("--denoise-steps", type=int, default=1,
                    help="T: selection + attention passes per layer-chunk; the cache (persistent set, window, pooled keys "
                         "of the window) is the same for all of them and the update follows the last one only")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--settle-steps", type=int, default=150,
                    help="untimed steps before the warm-up steps, so that the GPU's clocks have settled under load")
    ap.add_argument("--sweep-kernel-grid", action="store_true",
                    help="instead of the step benchmark: pbsa_attention_fwd alone on the shapes of the paper's "
                         "kernel benchmark (forward latency table of its appendix) that fit the interface limits, "
                         "at top-k 6.25 / 12.5 / 25 % and with every block selected (the dense stand-in)")
    ap.add_argument("--blockify", action="store_true",
                    help="instead of the step benchmark: the block rearrange of a chunk's Q, K, V and its inverse")
    ap.add_argument("--separate-update", action="store_true",
                    help="the step as the three plain calls, pbsa_select_blocks -> pbsa_attention_fwd -> pbsa_memory_update")
    ap.add_argument("--three-launches", action="store_true",
                    help="self-contained steps: pbsa_select_blocks -> pbsa_attention_fwd_plan (the attention launch with one more "
                         "workgroup per head that takes the update's decisions) -> pbsa_memory_update_apply, instead of the "
                         "default of two library calls per step: pbsa_select_blocks_apply (the selection, with the fold / "
                         "promote of the previous step's update riding in its pooling launch; the ring gets a spare position "
                         "so that the new chunk is not written over the blocks still to be folded) and pbsa_attention_fwd_plan")
    ap.add_argument("--no-per-config", action="store_true",
                    help="skip the short runs of cfg2, cfg3 and cfg4 that follow the timed region of cfg5")
    ap.add_argument("--per-config-layers", type=int, default=8,
                    help="layers of cfg3 in its short run (each needs its own synthetic inputs, generated on the host)")
    ap.add_argument("--fine-mass", action="store_true",
                    help="the step with the persistent set ranked by the attention actually paid: after the attention "
                         "call pbsa_attention_mass sums the probabilities per key block and pbsa_memory_update_fine "
                         "ranks by them (select + attention + mass + update per step)")
    ap.add_argument("--backward", action="store_true",
                    help="instead of the step benchmark: pbsa_attention_bwd (dQ, dK, dV) on the workload's steady-state "
                         "cache, after one forward call that supplies O and lse")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run three 1 GiB device copies and exit: the known-size kernel that the HBM byte "
                         "counters are scaled by")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (the path shards by head without exchange; "
                 "no multi-GPU figure is produced). Use --gpus 1.")
    import numpy as np
    import torch
    from harness import synth, workloads
    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    dev = "cuda:0"
    if args.calibrate_copy:
        a = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        b = torch.empty_like(a)
        for _ in range(3):
            b.copy_(a)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes_read": a.numel() * 4, "copy_bytes_written": b.numel() * 4, "copies": 3}))
        return
    if args.blockify:
        print(json.dumps(bench_blockify(dev)))
        return
    if args.sweep_kernel_grid:
        print(json.dumps(sweep_kernel_grid(dev, reps=max(args.steps, 10))))
        return
    w = synth.WORKLOADS[args.workload]
    out = bench_steps(w, args, args.steps, args.warmup, args.settle_steps, dev)
    if args.backward:
        print(json.dumps(out))
        return
    mean_flops, T = out.pop("_mean_flops"), out.pop("_T")
    if args.workload == "cfg5" and not (args.no_per_config or args.fine_mass or args.separate_update):
        # the other configurations, after the timed region of the headline one (the chip is warm: short settling)
        out["per_config"] = {}
        for name in ("cfg2", "cfg3", "cfg4"):
            w2 = synth.WORKLOADS[name]
            layers = min(w2.n_layers, args.per_config_layers)
            r = bench_steps(w2, args, max(args.steps, 3 * layers), 5, 40, dev, layers=layers)
            row = {"us_per_layer_chunk": r["us_per_layer_chunk"], "value": r["value"], "unit": "TFLOP/s",
                   "attention_us_per_launch": r["roofline"]["us_per_launch"], "frac": r["roofline"]["frac"],
                   "executed_gflop_per_step": r["config"]["executed_gflop_per_step"], "steps": r["steps"]}
            if w2.n_layers > 1:
                row["layers"] = layers
                row["note"] = (f"{layers} of the {w2.n_layers} independently seeded layers, visited in turn: their caches "
                               "(86 MB of K/V each) already exceed what the chip keeps between visits")
            out["per_config"][name] = row
    if not args.no_cpu_baseline:
        from oracle import pbsa_oracle as orc
        t_sel, t_att, t_upd, n_rows = cpu_baseline(w)
        cpu_s = T * (t_sel + t_att) + t_upd
        out["cpu_baseline"] = {
            "value": round(mean_flops / cpu_s / 1e12, 6), "unit": "TFLOP/s", "cores": orc.num_threads(),
            "kind": "oracle", "seconds_per_layer_chunk": round(cpu_s, 3),   # all T passes
            "sample": f"full selection ({t_sel:.3f} s) and update ({t_upd:.3f} s) of one {w.name} steady-state chunk; "
                      f"attention on {n_rows} of {w.H * w.Nq} rows, scaled to the chunk ({t_att:.2f} s)"}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
