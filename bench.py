#!/usr/bin/env python3
"""Benchmark of the S2-Attention / HHST hot path on one MI355X.

A step is one forward + backward pass of head-heterogeneous block-sparse causal
attention over one batch of synthetic bf16 tensors that are already resident in
HBM.  Prints ONE JSON line: effective (unmasked) TFLOP/s of forward+backward,
its fraction of the bf16 MFMA peak, the speed-up over the library's own dense
causal kernels, a roofline record for the dominant kernel (timed here with HIP
events, one kernel per launch) and the CPU oracle's rate on a bounded sample.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 7b_32k]
"""

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def sparse_pairs(nnz, H, B, S):
    """Unmasked (query, key) pairs of one batch element: diagonal blocks are triangular."""
    return (nnz - H * B) * S * S + H * B * S * (S + 1) // 2


def prewarm(fn, seconds=0.3):
    """Untimed: runs fn until the GPU has been busy for a while, so that what is measured next is
    at the sustained clocks of a long-running job rather than those of a device just woken up."""
    import torch
    t0 = time.perf_counter()
    while time.perf_counter() - t0 < seconds:
        for _ in range(8):
            fn()
        torch.cuda.synchronize()


def time_events(fn, steps, warmup):
    import torch
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / steps


def measured_traffic(workload, kernel):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 --pmc summary
    (profiles/traffic_<workload>.txt, lines `<kernel> <bytes>`), or None.  The file names the
    kernel sources it was measured on (`# sources <fingerprint>`, written by
    paper_2407_17678_amd/profile_summary.py); a file taken on other sources is refused, so that the
    figure cannot outlive the kernels it describes."""
    from paper_2407_17678_amd import profile_summary
    path = os.path.join(ROOT, "profiles", "traffic_%s.txt" % workload)
    try:
        with open(path) as f:
            lines = f.read().splitlines()
    except OSError:
        return None
    stamp = [l.split()[2] for l in lines if l.startswith("# sources ") and len(l.split()) >= 3]
    if not stamp or stamp[0] != profile_summary.source_fingerprint():
        log("[bench] %s was measured on other kernel sources: traffic not reported" % os.path.basename(path))
        return None
    for line in lines:
        parts = line.split()
        if len(parts) >= 2 and parts[0] == kernel:
            return float(parts[1])
    return None


def measured_ceilings():
    """What the chip sustains on a pure MFMA loop (alone, and with a softmax's vector work per MFMA)
    and on a pure read, timed like the kernels: the library's probe kernels (s2_probe_*), a few
    milliseconds per launch on random operands."""
    import torch
    from paper_2407_17678_amd import binding as B
    scratch = torch.empty(max(B.s2_probe_scratch_bytes(), 4 << 20), dtype=torch.uint8, device="cuda")
    out = {}
    for name, mix in (("mfma_bf16_tflops", 0), ("mfma_bf16_with_softmax_vector_work_tflops", 1)):
        flops = [0.0]

        def run():
            flops[0] = B.s2_probe_mfma(mix, 20000, scratch)
        prewarm(run, 0.2)
        ms = time_events(run, 5, 1)
        out[name] = flops[0] / (ms * 1e-3) / 1e12
    src = torch.empty(2 << 30, dtype=torch.uint8, device="cuda").random_(0, 255)
    rd = lambda: B.s2_probe_read(src, scratch)
    prewarm(rd, 0.2)
    ms = time_events(rd, 10, 2)
    out["hbm_read_gbs"] = (2 << 30) / (ms * 1e-3) / 1e9
    del src
    # what accumulating partial gradients with atomics would cost (a single-pass backward's dQ)
    acc = torch.zeros(128 << 20, dtype=torch.float32, device="cuda")
    added = [0.0]

    def at():
        added[0] = B.s2_probe_atomic_add(acc)
    ms = time_events(at, 3, 1)
    out["fp32_atomic_add_gbs"] = added[0] / (ms * 1e-3) / 1e9
    del acc
    torch.cuda.empty_cache()
    return out


def bench_train(w, steps, warmup, with_dense=True, with_bwd=True, dense_steps=3, hybrid_layers=None):
    """Times fwd(+bwd) of workload `w`; returns a dict of timings and derived rates."""
    import torch
    from paper_2407_17678_amd import binding as B
    from paper_2407_17678_amd import synth

    t0 = time.time()
    qb, kb, vb, gb = synth.train_inputs(w)
    q, k, v, g = (B.bf16_bits_to_device(x) for x in (qb, kb, vb, gb))
    log("[bench] %s: inputs %s generated in %.1fs" % (w.name, tuple(q.shape), time.time() - t0))
    Bt, H, N, D = q.shape
    S = w.block_size
    o = torch.empty_like(q)
    lse = torch.empty((Bt, H, N), dtype=torch.float32, device="cuda")
    dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
    ws = torch.empty(B.s2_attn_bwd_workspace_bytes(Bt, H, N, D), dtype=torch.uint8, device="cuda")
    t0 = time.time()
    lay = B.s2_layout_build(B.layout_params(H, N // S, S, w.local_blocks, w.stride, 0, w.window_blocks, 0))
    layout_ms = (time.time() - t0) * 1e3
    # The backward has two forms, chosen by the workspace the caller brings: the small one (delta and
    # LSE only: the dQ launch recomputes S and dP) and, where it applies, the one that also holds dS
    # between the dK/dV and dQ launches (2 bytes per kept block element; nothing is computed twice).
    keep_bytes = B.s2_attn_bwd_layout_workspace_bytes(lay, Bt, H, N, D) if with_bwd else 0
    ws_keep = torch.empty(keep_bytes, dtype=torch.uint8, device="cuda") if keep_bytes > ws.numel() else None
    nnz = B.s2_layout_get(lay)["nnz"]
    # KV-block loads of the forward: one per list entry of a merged 128-row query tile, against one
    # per kept block of every S-token mask row without merging (the reload accounting of section 3.2)
    merged = int(B.s2_layout_get_tiles(lay, B.TILES_FWD)["ptr"][-1])
    pairs = sparse_pairs(nnz, H, N // S, S) * Bt
    dense_pairs = H * N * (N + 1) // 2 * Bt

    fwd = lambda: B.s2_attn_fwd(lay, q, k, v, o, lse, w.scale)
    bwd_of = lambda wsp: (lambda: B.s2_attn_bwd(lay, q, k, v, o, lse, g, dq, dk, dv, w.scale, wsp))
    stage_of = lambda wsp, s: (lambda: B.s2_attn_bwd_stages(lay, q, k, v, o, lse, g, dq, dk, dv, w.scale, wsp, s))
    bwd = bwd_of(ws)
    stage = lambda s: stage_of(ws, s)

    def step():
        fwd()
        if with_bwd:
            bwd()

    # Untimed: bring the GPU to its sustained clocks first (whatever is measured in the first tens of
    # milliseconds after idle comes out 3-12 % slow), as it would be in a long-running job.
    prewarm(step)

    res = dict(workload=w.name, batch=Bt, heads=H, seqlen=N, head_dim=D, block_size=S,
               local_blocks=w.local_blocks, stride=w.stride, nnz_blocks=int(nnz),
               layout_build_ms=round(layout_ms, 2), kv_block_loads_per_head_set=dict(unmerged=int(nnz), merged=merged))
    # each kernel on its own (same stream, same inputs)
    res["ms_fwd"] = time_events(fwd, steps, 1)
    flops_fwd = 4.0 * D * pairs
    if with_bwd:
        # small workspace: the dQ launch (which also computes delta) followed by the dK/dV launch
        rec = dict(ms_dq=time_events(stage(B.BWD_DQ), steps, 1), ms_dkdv=time_events(stage(B.BWD_DKDV), steps, 1),
                   ms=time_events(bwd, steps, 1), workspace_bytes=ws.numel())
        res["backward_recomputing"] = rec
        res["backward_path"] = "recomputing"
        # the stand-alone delta kernel (with the small workspace only used when dK/dV is asked for without dQ)
        res["ms_delta_standalone"] = time_events(stage(B.BWD_DELTA), steps, 1)
        res["ms_bwd_dq"], res["ms_bwd_dkdv"], res["ms_bwd_delta"] = rec["ms_dq"], rec["ms_dkdv"], 0.0
        if ws_keep is not None:
            # larger workspace: delta kernel, dK/dV launch that leaves dS, dQ = dS K
            keep = dict(ms_delta=time_events(stage_of(ws_keep, B.BWD_DELTA), steps, 1),
                        ms_dkdv=time_events(stage_of(ws_keep, B.BWD_DKDV), steps, 1),
                        ms_dq=time_events(stage_of(ws_keep, B.BWD_DQ), steps, 1),
                        ms=time_events(bwd_of(ws_keep), steps, 1), workspace_bytes=ws_keep.numel())
            res["backward_keeping_ds"] = keep
            if keep["ms"] < rec["ms"]:   # a step uses the faster form, as a caller with the memory to spare would
                bwd = bwd_of(ws_keep)
                res["backward_path"] = "keeping dS"
                res["ms_bwd_dq"], res["ms_bwd_dkdv"], res["ms_bwd_delta"] = keep["ms_dq"], keep["ms_dkdv"], keep["ms_delta"]
        flops = 14.0 * D * pairs
    else:
        flops = flops_fwd
    # the timed region: `warmup` untimed steps, then exactly `steps` steps between two synchronisations
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    t_wall = time.perf_counter()
    marks[0].record()
    for i in range(steps):
        step()
        marks[i + 1].record()   # an event between steps costs nothing on the stream; gives median and min
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t_wall) * 1e3 / steps
    ms_step = marks[0].elapsed_time(marks[steps]) / steps
    each = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(steps))
    res["ms_step_median"] = each[len(each) // 2]
    res["ms_step_min"] = each[0]

    res["ms_per_step"] = ms_step
    res["wall_ms_per_step"] = wall_ms
    res["effective_gflop"] = flops / 1e9
    res["tflops"] = flops / (ms_step * 1e-3) / 1e12
    res["tflops_fwd"] = flops_fwd / (res["ms_fwd"] * 1e-3) / 1e12
    res["pct_mfma_peak"] = 100.0 * res["tflops"] / PEAK_BF16_TFLOPS
    res["pair_ratio_dense_over_sparse"] = dense_pairs / pairs

    if with_dense:
        dfwd = lambda: B.s2_dense_causal_fwd(q, k, v, o, lse, w.scale)
        dbwd = lambda: B.s2_dense_causal_bwd(q, k, v, o, lse, g, dq, dk, dv, w.scale, ws)

        def dstep():
            dfwd()
            if with_bwd:
                dbwd()
        res["dense_ms_per_step"] = time_events(dstep, dense_steps, 1)
        res["dense_ms_fwd"] = time_events(dfwd, dense_steps, 0)
        dflops = (14.0 if with_bwd else 4.0) * D * dense_pairs
        res["dense_tflops"] = dflops / (res["dense_ms_per_step"] * 1e-3) / 1e12
        res["speedup_vs_dense"] = res["dense_ms_per_step"] / ms_step
        if with_bwd:
            # the dense kernels have no form that keeps dS (it would be 2 bytes per causal pair): like for like,
            # both sides with the recomputing backward
            res["speedup_vs_dense_both_recomputing"] = res["dense_ms_per_step"] / (res["ms_fwd"] + res["backward_recomputing"]["ms"])
        res["speedup_vs_dense_fwd"] = res["dense_ms_fwd"] / res["ms_fwd"]
        if hybrid_layers:
            # Attention time of a whole layer stack that keeps a few layers dense (section 4.2's
            # hybrid architecture: dense attention in about 1/6 of the layers): every layer's
            # forward in order, then every layer's backward in reverse order, one launch set per
            # layer as a model would issue them.
            n_layers, n_dense = hybrid_layers
            every = n_layers / n_dense
            dense_at = {int(i * every) for i in range(n_dense)}

            def stack(all_dense):
                for l in range(n_layers):
                    (dfwd if all_dense or l in dense_at else fwd)()
                if with_bwd:
                    for l in reversed(range(n_layers)):
                        (dbwd if all_dense or l in dense_at else bwd)()
            ms_h = time_events(lambda: stack(False), 2, 1)
            ms_d = time_events(lambda: stack(True), 1, 0)
            frac = (n_dense * dense_pairs + (n_layers - n_dense) * pairs) / (n_layers * dense_pairs)
            res["hybrid_stack"] = dict(layers=n_layers, dense_layers=sorted(dense_at), ms=ms_h, all_dense_ms=ms_d,
                                       speedup=ms_d / ms_h, flop_fraction_of_dense=frac)
        step()  # leave the sparse path's outputs in place for the parity sample

    # roofline of the dominant kernel.  Flops attributed per kernel (sums to 14*D*pairs):
    # forward 4*D*pairs (QK^T, PV); dK/dV kernel 8*D*pairs (S, dP, dV, dK); dQ kernel 2*D*pairs.
    # (head_dim 128 with mask blocks of 64 tokens or more runs the hand-scheduled forward and dQ kernels)
    fast = D == 128 and S >= 64 and N % 128 == 0
    kernels = {"fwd_pipe_kernel" if fast else "fwd_kernel": (res["ms_fwd"], 4.0)}
    if with_bwd:
        kernels["dkdv_kernel"] = (res["ms_bwd_dkdv"], 8.0)
        dq_name = "dq_gemm_kernel" if res["backward_path"] == "keeping dS" else "dq_pipe_kernel" if fast else "dq_kernel"
        kernels[dq_name] = (res["ms_bwd_dq"], 2.0)
    dom = max(kernels, key=lambda n: kernels[n][0])
    ach = kernels[dom][1] * D * pairs / (kernels[dom][0] * 1e-3) / 1e12
    res["roofline"] = {"kernel": dom, "bound": "mfma", "achieved": ach, "peak": PEAK_BF16_TFLOPS,
                       "unit": "TFLOP/s", "frac": ach / PEAK_BF16_TFLOPS,
                       "traffic": measured_traffic(w.name, dom + ("_keeping_ds" if dom == "dkdv_kernel" and with_bwd and
                                                                  res["backward_path"] == "keeping dS" else "")),
                       "avg_launch_ms": kernels[dom][0],
                       "algorithmic_flops_per_launch": kernels[dom][1] * D * pairs}
    if with_bwd:
        # The attribution above is a convention (with the small workspace the dQ launch recomputes S and
        # dP, which it is not credited with); the whole backward against its 10 * D * pairs says what
        # the launches deliver together.
        t_bwd = res["ms_bwd_dq"] + res["ms_bwd_dkdv"] + res["ms_bwd_delta"]
        res["roofline"]["whole_backward"] = {"ms": t_bwd, "achieved": 10.0 * D * pairs / (t_bwd * 1e-3) / 1e12,
                                             "frac": 10.0 * D * pairs / (t_bwd * 1e-3) / 1e12 / PEAK_BF16_TFLOPS}
        res["roofline"]["forward"] = {"ms": res["ms_fwd"], "achieved": res["tflops_fwd"],
                                      "frac": res["tflops_fwd"] / PEAK_BF16_TFLOPS}
    tensors = dict(q=q, k=k, v=v, g=g, o=o, lse=lse, dq=dq, dk=dk, dv=dv, bits=(qb, kb, vb, gb))
    return res, tensors


def cpu_baseline_train(w, tensors, sample_tokens, with_bwd=True):
    """The oracle, untuned, on head 0 of batch 0 restricted to the first `sample_tokens` tokens
    (a causal prefix is self-contained); also compares the GPU's O / LSE / dQ on that prefix."""
    from oracle import s2_oracle as orc
    from paper_2407_17678_amd import synth
    qb, kb, vb, gb = tensors["bits"]
    n = min(sample_tokens, qb.shape[2])
    S = w.block_size
    f64 = lambda x: synth.bf16_bits_to_f32(x[0, 0, :n]).astype(np.float64)
    q, k, v, g = f64(qb), f64(kb), f64(vb), f64(gb)
    M = orc.block_mask(1, n // S, w.local_blocks, w.stride, window_blocks=w.window_blocks)
    pairs = orc.unmasked_pairs(M, S, n)
    t0 = time.perf_counter()
    if with_bwd:
        dQ, dK, dV, O, LSE = orc.attention_backward_head(q, k, v, g, M[0], S, w.scale)
    else:
        O, LSE = orc.attention_forward_head(q, k, v, M[0], S, w.scale)
    sec = time.perf_counter() - t0
    flops = (14.0 if with_bwd else 4.0) * w.head_dim * pairs
    try:
        cores = len(os.sched_getaffinity(0))
    except AttributeError:
        cores = os.cpu_count()
    threads = cores
    try:
        from threadpoolctl import threadpool_info
        blas = [i["num_threads"] for i in threadpool_info() if i.get("user_api") == "blas"]
        if blas:
            threads = max(blas)
    except Exception:
        pass
    go = tensors["o"][0, 0, :n].float().cpu().numpy().astype(np.float64)
    gl = tensors["lse"][0, 0, :n].cpu().numpy().astype(np.float64)
    # bound on O: 1e-2, or half a bf16 ulp of the reference value where that is larger (|O| >= 4 only)
    err = np.abs(go - O)
    half_ulp = np.exp2(np.floor(np.log2(np.maximum(np.abs(O), 2.0 ** -126))) - 8.0)
    excess = err - np.maximum(1e-2, half_ulp)
    worst = np.unravel_index(int(np.argmax(err)), err.shape)
    below4 = np.abs(O) < 4.0
    parity = {"o_max_abs": float(err.max()), "o_ref_at_worst": float(O[worst]),
              "o_max_abs_where_ref_below_4": float(err[below4].max()) if below4.any() else 0.0,
              "o_max_excess_over_bound": float(excess.max()),
              "lse_max_abs": float(np.abs(gl - LSE).max())}
    if with_bwd:
        gq = tensors["dq"][0, 0, :n].float().cpu().numpy().astype(np.float64)
        parity["dq_rel_l2"] = float(np.linalg.norm(gq - dQ) / np.linalg.norm(dQ))
        if n == qb.shape[2]:   # dK, dV need every query of the head
            for name, ref in (("dk", dK), ("dv", dV)):
                gg = tensors[name][0, 0].float().cpu().numpy().astype(np.float64)
                parity[name + "_rel_l2"] = float(np.linalg.norm(gg - ref) / np.linalg.norm(ref))
    return {"value": flops / sec / 1e12, "unit": "TFLOP/s", "cores": int(threads), "kind": "oracle",
            "sample": "head 0 of batch 0, first %d tokens, %s, fp64 numpy" % (n, "fwd+bwd" if with_bwd else "fwd"),
            "seconds": sec, "host_cores_visible": int(cores)}, parity


def bench_decode_paged(w, steps, warmup):
    """The decode workload with the cache held as pages behind a block table, each head keeping
    only the blocks some later query can still attend (section 4.1)."""
    import torch
    from paper_2407_17678_amd import binding as B
    from paper_2407_17678_amd import synth
    nseq, H, D, max_len, S = w.batch, w.heads, w.head_dim, w.max_len, w.block_size
    lens = synth.decode_lengths(w)
    p = B.layout_params(H, 1, S, w.local_blocks, w.stride, 0, w.window_blocks, 0)
    resident = [[B.s2_kv_resident_blocks(p, h, int(L)) for h in range(H)] for L in lens]
    max_blocks = max_len // S
    table, num_pages = synth.page_table(resident, max_blocks, index=w.index)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(synth.BASE_SEED + w.index)
    q = torch.randn((nseq, H, D), device="cuda", generator=gen).to(torch.bfloat16)
    kp = torch.empty((num_pages, S, D), dtype=torch.bfloat16, device="cuda")
    vp = torch.empty_like(kp)
    step = 4096
    for lo in range(0, num_pages, step):   # fill in slices so that the fp32 temporaries stay small
        n = min(step, num_pages - lo)
        kp[lo:lo + n] = torch.randn((n, S, D), device="cuda", generator=gen).to(torch.bfloat16)
        vp[lo:lo + n] = torch.randn((n, S, D), device="cuda", generator=gen).to(torch.bfloat16)
    tb = torch.from_numpy(table).cuda()
    sl = torch.from_numpy(lens).cuda()
    o = torch.empty_like(q)
    lse = torch.empty((nseq, H), dtype=torch.float32, device="cuda")
    missing = torch.zeros(1, dtype=torch.int32, device="cuda")
    splits = B.s2_attn_decode_default_splits(nseq, H, max_len)
    ws = torch.empty(B.s2_attn_decode_workspace_bytes(nseq, H, D, max_len, splits), dtype=torch.uint8,
                     device="cuda")
    run = lambda: B.s2_attn_decode_paged(p, q, kp, vp, tb, sl, o, lse, w.scale, ws, missing=missing,
                                         num_splits=splits)
    prewarm(run)
    ms = time_events(run, steps, warmup)
    if int(missing.item()) != 0:
        sys.exit("bench.py: the paged decode found kept blocks missing from its own table")
    tokens = 0
    for b, L in enumerate(lens.tolist()):
        i = (L - 1) // S
        for h in range(H):
            tokens += sum(min(S, L - j * S) for j in resident[b][h])
            assert resident[b][h][-1] == i
    kv_bytes = tokens * D * 2 * 2
    # q, o, split partials, and the table entries looked up
    partials = 0 if splits == 1 else 2 * nseq * H * splits * (D + 2) * 4   # one split writes the result itself
    other = nseq * H * D * 2 * 2 + partials + sum(len(r) for row in resident for r in row) * 4
    gbs = (kv_bytes + other) / (ms * 1e-3) / 1e9
    contiguous_gb = 2 * nseq * H * max_len * D * 2 / 1e9
    return dict(workload=w.name + "_paged", nseq=nseq, heads=H, head_dim=D, max_len=max_len, splits=int(splits),
                mean_len=float(lens.mean()), ms=ms, kept_tokens=int(tokens), pages=int(num_pages),
                cache_gb=2 * num_pages * S * D * 2 / 1e9, contiguous_cache_gb=contiguous_gb,
                algorithmic_gb=(kv_bytes + other) / 1e9, hbm_gbs=gbs, frac_hbm_peak=gbs / PEAK_HBM_GBS)


def bench_prefill_varlen(w, steps, warmup, nseq=12, min_len=1024):
    """A serving prefill batch: `nseq` prompts of different lengths packed into one tensor, one
    launch of the variable-length forward; beside it the same prompts padded to the longest."""
    import torch
    from paper_2407_17678_amd import binding as B
    from paper_2407_17678_amd import synth
    H, D, S = w.heads, w.head_dim, w.block_size
    lens = synth.prefill_lengths(w, nseq, min_len)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    total = int(cu[-1])
    lay = B.s2_layout_build(B.layout_params(H, w.num_blocks, S, w.local_blocks, w.stride, 0, w.window_blocks, 0))
    view = B.s2_layout_get(lay)
    # unmasked pairs: per block row, (kept blocks - 1) full blocks of S keys plus the causal diagonal
    row_blocks = np.diff(view["row_ptr"]).reshape(H, w.num_blocks).astype(np.int64)
    pairs = 0
    for L in lens.tolist():
        full, rem = divmod(L, S)
        pairs += int(((row_blocks[:, :full] - 1) * S * S + S * (S + 1) // 2).sum())
        if rem:
            pairs += int(((row_blocks[:, full] - 1) * S * rem + rem * (rem + 1) // 2).sum())
    gen = torch.Generator(device="cuda")
    gen.manual_seed(synth.BASE_SEED + w.index)
    q, k, v = (torch.randn((1, H, total, D), device="cuda", generator=gen).to(torch.bfloat16) for _ in range(3))
    o = torch.empty_like(q)
    lse = torch.empty((H, total), dtype=torch.float32, device="cuda")
    cud = torch.from_numpy(cu).cuda()
    run = lambda: B.s2_attn_fwd_varlen(lay, q, k, v, o, lse, cud, w.seqlen, w.scale)
    prewarm(run)
    ms = time_events(run, steps, warmup)
    # what a caller without the packed entry point does: every prompt padded to the longest one
    pad_len = -(-int(lens.max()) // 128) * 128
    lay_p = B.s2_layout_build(B.layout_params(H, pad_len // S, S, w.local_blocks, w.stride, 0, w.window_blocks, 0))
    qp, kp, vp = (torch.randn((nseq, H, pad_len, D), device="cuda", generator=gen).to(torch.bfloat16) for _ in range(3))
    op = torch.empty_like(qp)
    lsep = torch.empty((nseq, H, pad_len), dtype=torch.float32, device="cuda")
    run_p = lambda: B.s2_attn_fwd(lay_p, qp, kp, vp, op, lsep, w.scale)
    ms_pad = time_events(run_p, max(3, steps // 2), 2)
    # the same packed batch as a training step: forward + backward in two more launches
    g = torch.randn((1, H, total, D), device="cuda", generator=gen).to(torch.bfloat16)
    dq, dk, dv = torch.empty_like(q), torch.empty_like(q), torch.empty_like(q)
    wsb = torch.empty(B.s2_attn_bwd_varlen_workspace_bytes(H, total, D), dtype=torch.uint8, device="cuda")
    run_b = lambda: B.s2_attn_bwd_varlen(lay, q, k, v, o, lse, g, dq, dk, dv, cud, w.seqlen, w.scale, wsb)
    run()
    ms_bwd = time_events(run_b, steps, warmup)
    tf = 4.0 * D * pairs / (ms * 1e-3) / 1e12
    extra_bwd = dict(ms_bwd=ms_bwd, tflops_fwd_bwd=14.0 * D * pairs / ((ms + ms_bwd) * 1e-3) / 1e12)
    return dict(extra_bwd, workload=w.name + "_prefill_varlen", nseq=nseq, heads=H, head_dim=D, block_size=S,
                lengths=lens.tolist(), total_tokens=total, ms=ms, unmasked_pairs=pairs, tflops=tf,
                pct_mfma_peak=100.0 * tf / PEAK_BF16_TFLOPS, ms_padded_to_longest=ms_pad,
                speedup_vs_padded=ms_pad / ms)


def bench_decode(w, steps, warmup, auto_splits=False):
    """auto_splits: leave the split count to the library (it cuts the public default down where a row has
    few units of work); the workspace is sized for the public default either way."""
    import torch
    from paper_2407_17678_amd import binding as B
    from paper_2407_17678_amd import synth
    nseq, H, D, max_len = w.batch, w.heads, w.head_dim, w.max_len
    lens = synth.decode_lengths(w)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(synth.BASE_SEED + w.index)
    q = torch.randn((nseq, H, D), device="cuda", generator=gen).to(torch.bfloat16)
    kc = torch.empty((nseq, H, max_len, D), dtype=torch.bfloat16, device="cuda")
    vc = torch.empty_like(kc)
    for b in range(nseq):   # fill in slices so that the fp32 temporaries stay small
        kc[b] = torch.randn((H, max_len, D), device="cuda", generator=gen).to(torch.bfloat16)
        vc[b] = torch.randn((H, max_len, D), device="cuda", generator=gen).to(torch.bfloat16)
    sl = torch.from_numpy(lens).cuda()
    o = torch.empty_like(q)
    lse = torch.empty((nseq, H), dtype=torch.float32, device="cuda")
    p = B.layout_params(H, 1, w.block_size, w.local_blocks, w.stride, 0, w.window_blocks, 0)
    splits = B.s2_attn_decode_default_splits(nseq, H, max_len)
    ws = torch.empty(B.s2_attn_decode_workspace_bytes(nseq, H, D, max_len, splits), dtype=torch.uint8,
                     device="cuda")
    run = lambda: B.s2_attn_decode(p, q, kc, vc, sl, o, lse, w.scale, ws, max_len, num_splits=0 if auto_splits else splits)
    prewarm(run)
    ms = time_events(run, steps, warmup)
    # algorithmic bytes: K and V rows of the kept tokens, plus q, o and the split partials
    S = w.block_size
    tokens = 0
    for L in lens.tolist():
        i = (L - 1) // S
        for h in range(H):
            o_h = h % w.stride
            local_lo = max(0, i - w.local_blocks + 1)
            n_str = (local_lo - 1 - o_h) // w.stride + 1 if o_h < local_lo else 0
            tokens += n_str * S + (L - local_lo * S)
    kv_bytes = tokens * D * 2 * 2
    partials = 0 if splits == 1 and not auto_splits else 2 * nseq * H * splits * (D + 2) * 4   # one split writes the result itself
    other = nseq * H * D * 2 * 2 + partials
    dense_bytes = int(lens.astype(np.int64).sum()) * H * D * 2 * 2
    gbs = (kv_bytes + other) / (ms * 1e-3) / 1e9
    return dict(workload=w.name, nseq=nseq, heads=H, head_dim=D, max_len=max_len, block_size=w.block_size,
                splits="left to the library" if auto_splits else int(splits),
                mean_len=float(lens.mean()), ms=ms, kept_tokens=int(tokens), algorithmic_gb=(kv_bytes + other) / 1e9,
                dense_gb=dense_bytes / 1e9, hbm_gbs=gbs, frac_hbm_peak=gbs / PEAK_HBM_GBS)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="7b_32k", choices=["tiny", "1p3b_8k", "7b_32k", "7b_128k", "7b_decode", "7b_decode_paged",
                             "7b_prefill_varlen"])
    ap.add_argument("--cpu-sample-tokens", type=int, default=32768)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-dense", action="store_true")
    ap.add_argument("--extra", action="store_true", help="(default) also time the other workloads, reported under 'extra'")
    ap.add_argument("--no-extra", action="store_true", help="only the workload named by --workload")
    ap.add_argument("--no-ceilings", action="store_true", help="skip the MFMA / HBM ceiling probes")
    ap.add_argument("--hybrid-stack", default=None, metavar="LAYERS:DENSE",
                    help="also time the attention of a LAYERS-layer stack with DENSE of them dense, e.g. 32:5")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="first run a 1 GiB device-to-device copy, so that a rocprofv3 --pmc run has a kernel "
                         "of known traffic to scale FETCH_SIZE / WRITE_SIZE by")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU; --gpus %d is not supported (heads and batch "
                 "shard across GPUs without communication)" % args.gpus)
    if int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.exit("bench.py: launched with WORLD_SIZE > 1; this build runs on one GPU")

    import torch
    from paper_2407_17678_amd import binding as B
    from paper_2407_17678_amd import synth
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; the HIP library is the only path")
    B.lib()
    torch.cuda.set_device(0)
    paged = args.workload == "7b_decode_paged"
    varlen = args.workload == "7b_prefill_varlen"
    w = synth.WORKLOADS["7b_decode" if paged else "7b_32k" if varlen else args.workload]
    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    if varlen:
        d = bench_prefill_varlen(w, args.steps, args.warmup)
        # two launches per call: the pipelined kernel on each sequence's whole 128-row tiles, the plain one on
        # the partial last tiles
        parts = [measured_traffic(d["workload"], k) for k in ("fwd_pipe_kernel", "fwd_kernel")]
        traffic = None if any(t is None for t in parts) else sum(parts)
        out = {"metric": "effective sparse-attn TFLOP/s, forward on a packed variable-length prefill batch",
               "value": d["tflops"], "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
               "ms_per_step": d["ms"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
               "dtype": "bf16", "data": "synthetic", "config": d,
               "roofline": {"kernel": "fwd_pipe_kernel + fwd_kernel (variable-length)", "bound": "mfma",
                            "achieved": d["tflops"], "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                            "frac": d["tflops"] / PEAK_BF16_TFLOPS, "traffic": traffic},
               "cpu_baseline": None}
        print(json.dumps(out))
        return

    if w.kind == "decode":
        d = bench_decode_paged(w, args.steps, args.warmup) if paged else bench_decode(w, args.steps, args.warmup)
        out = {"metric": "decode HBM GB/s (algorithmic K+V bytes of kept blocks)", "value": d["hbm_gbs"],
               "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": d["ms"],
               "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
               "data": "synthetic", "config": d,
               "roofline": {"kernel": "decode_split_kernel", "bound": "hbm", "achieved": d["hbm_gbs"],
                            "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": d["frac_hbm_peak"],
                            "traffic": measured_traffic(d["workload"], "decode_split_kernel")},
               "cpu_baseline": None}
        print(json.dumps(out))
        return

    with_bwd = w.name != "7b_128k"
    extras_on = not args.no_extra
    if args.hybrid_stack is None and extras_on and w.name == "7b_32k":
        args.hybrid_stack = "32:5"   # section 4.2: about 1/6 of a 7B model's 32 layers stay dense
    hybrid = tuple(int(x) for x in args.hybrid_stack.split(":")) if args.hybrid_stack else None

    res, tensors = bench_train(w, args.steps, args.warmup, with_dense=not args.no_dense, with_bwd=with_bwd,
                               dense_steps=2 if w.seqlen > 40000 else 3, hybrid_layers=hybrid)
    roof = res.pop("roofline")
    cpu, parity = None, None
    if not args.no_cpu_baseline:
        log("[bench] timing the CPU oracle on a %d-token prefix of one head ..." % args.cpu_sample_tokens)
        cpu, parity = cpu_baseline_train(w, tensors, args.cpu_sample_tokens, with_bwd=with_bwd)
        log("[bench] oracle: %.1fs on %d threads; parity on the sample: %s" % (cpu["seconds"], cpu["cores"], parity))
    del tensors
    torch.cuda.empty_cache()

    extra = None
    if extras_on:
        extra = {}
        for name in ("tiny", "1p3b_8k", "7b_32k", "7b_128k"):
            if name == w.name:
                continue
            ww = synth.WORKLOADS[name]
            r, t = bench_train(ww, max(3, args.steps // 2), 2, with_dense=not args.no_dense,
                               with_bwd=name != "7b_128k", dense_steps=1 if name == "7b_128k" else 3)
            rf = r.pop("roofline")
            r["roofline_frac_dominant_kernel"] = {"kernel": rf["kernel"], "frac": rf["frac"]}
            extra[name] = r
            del t
            torch.cuda.empty_cache()
        extra["7b_decode"] = bench_decode(synth.WORKLOADS["7b_decode"], 20, 3)
        extra["7b_decode_paged"] = bench_decode_paged(synth.WORKLOADS["7b_decode"], 20, 3)
        # the same cache read through 16-token blocks (the finest shards the paper mentions; 64 local
        # blocks and a stripe every 64 keep the local window's tokens and a quarter of each stripe's),
        # and one sequence on its own (two launches of a few microseconds: bound by launch latency)
        import dataclasses
        dw = synth.WORKLOADS["7b_decode"]
        extra["7b_decode_16_token_blocks"] = bench_decode(dataclasses.replace(dw, block_size=16, local_blocks=64, stride=64), 20, 3)
        extra["7b_decode_one_sequence_32k"] = bench_decode(dataclasses.replace(dw, batch=1, min_len=dw.max_len), 50, 5, auto_splits=True)
        extra["7b_prefill_varlen"] = bench_prefill_varlen(synth.WORKLOADS["7b_32k"], 10, 2)

    # last, so that a second of pure MFMA load does not heat the chip under the numbers above
    ceilings = None if args.no_ceilings else measured_ceilings()
    if ceilings:
        log("[bench] measured ceilings: %s" % ceilings)
        roof["measured_peak"] = dict(ceilings, note="the library's probe kernels timed in this run: a pure MFMA loop on "
                                     "random operands with two wavefronts per SIMD, alone and with a softmax's vector "
                                     "work per MFMA beside it; a pure 2 GiB read; coalesced fp32 atomic adds into a 512 MiB buffer")
        roof["frac_of_measured_mfma"] = roof["achieved"] / ceilings["mfma_bf16_tflops"]
        if extra is not None:
            for name in ("7b_decode", "7b_decode_paged", "7b_decode_16_token_blocks", "7b_decode_one_sequence_32k"):
                extra[name]["frac_of_measured_read"] = extra[name]["hbm_gbs"] / ceilings["hbm_read_gbs"]
    out = {
        "metric": "effective sparse-attn TFLOP/s fwd+bwd (% MFMA peak) + speedup vs dense causal"
                  if with_bwd else "effective sparse-attn TFLOP/s fwd (% MFMA peak) + speedup vs dense causal",
        "value": res["tflops"], "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": res["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": w.name, "batch": res["batch"], "heads": res["heads"], "seq_len": res["seqlen"],
                   "head_dim": res["head_dim"], "block_size": res["block_size"],
                   "local_blocks": res["local_blocks"], "stride": res["stride"], "pass": "fwd+bwd" if with_bwd else "fwd"},
        "pct_mfma_peak": res["pct_mfma_peak"],
        "speedup_vs_dense": res.get("speedup_vs_dense"),
        "detail": res,
        "roofline": roof,
        "cpu_baseline": cpu,
        "parity_on_cpu_sample": parity,
    }
    if "hybrid_stack" in res:
        out["hybrid_stack"] = res["hybrid_stack"]
    if extra is not None:
        out["extra"] = extra
    print(json.dumps(out))


if __name__ == "__main__":
    main()
