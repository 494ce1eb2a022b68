#!/usr/bin/env python3
"""Benchmark of the MLRA-4 decode hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C3|C2|C4|C5|M2] [--no-cpu-baseline]

One "step" = mlra_append_kv + mlra_absorb_q + mlra_decode_attn over one batch of synthetic,
seeded inputs that are already resident in HBM (workload M2: the MLRA-2 entry points, Eq. (6)).  Successive steps read different copies of the
cache so that the 256 MB Infinity Cache cannot serve the reads.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)


def _args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=100,
                    help="untimed steps first (the first 30-50 steps after start-up run up to 15 %% slower)")
    ap.add_argument("--workload", default="C3", choices=["C2", "C3", "C4", "C5", "M2", "G2"])
    ap.add_argument("--copies", type=int, default=0, help="cache copies to rotate over (0 = enough for ~3 GB)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--parity", action="store_true",
                    help="(kept for old command lines: the comparison with the oracle is always made with the CPU baseline)")
    ap.add_argument("--baselines", action="store_true",
                    help="C5 only: also time the GQA and MLA decode baselines on the same lengths and page table")
    ap.add_argument("--pre-attention", action="store_true",
                    help="the step starts from hidden states: mlra_pre_attention (projections, RMSNorm, RoPE, cache "
                         "append; hidden size 7168, query latent 1536) replaces mlra_append_kv")
    ap.add_argument("--q-len", type=int, default=1,
                    help="query tokens per sequence (> 1: mlra_decode_attn_multi; the q_len newest rows are cached, "
                         "the step appends only the newest one)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run plain 1 GiB device copies (reference dispatches for rocprofv3 byte counters)")
    ap.add_argument("--max-settle", type=int, default=400,
                    help="upper bound of the untimed settle phase (steps run before --warmup until the decode "
                         "kernel's time has stopped falling: the chip raises its clocks over the first milliseconds "
                         "of load); 0 switches it off")
    ap.add_argument("--no-graph", action="store_true", help="skip the HIP-graph replay of the step")
    ap.add_argument("--no-probes", action="store_true",
                    help="skip the streaming-read ceiling and shader-clock probes (profiling runs)")
    return ap.parse_args()


def _cpu_baseline(inp, max_seconds=25.0):
    """The fp64 oracle, as it stands, timed on this host on a bounded sample of the same workload."""
    from oracle import mlra_oracle as orc
    from paper_2603_02188_amd import inputs as gen
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    wl = inp.wl
    lat = gen.to_f64(inp.latent_pool, wl.dtype)
    rope = gen.to_f64(inp.rope_pool, wl.dtype)
    qn, qr = gen.to_f64(inp.q_nope, wl.dtype), gen.to_f64(inp.q_rope, wl.dtype)
    wk, wv = gen.to_f64(inp.w_uk, wl.dtype), gen.to_f64(inp.w_uv, wl.dtype)
    done_tokens, done_seqs = 0, 0
    t0 = time.perf_counter()
    outs = []
    if wl.groups == 2 and wl.n_blocks == 2:
        decode_batch = orc.gla2_decode_batch
    else:
        decode_batch = orc.mlra2_decode_batch if wl.groups == 2 else orc.mlra_decode_batch
    for b in range(wl.batch):
        outs.append(decode_batch(lat, rope, inp.page_table, inp.seq_lens, qn, qr, wk, wv, wl.tau, seqs=[b])[0])
        done_tokens += int(inp.seq_lens[b])
        done_seqs += 1
        if time.perf_counter() - t0 > max_seconds:
            break
    dt = time.perf_counter() - t0
    total_tokens = int(inp.seq_lens.sum())
    est_step_us = dt * 1e6 * total_tokens / max(1, done_tokens)
    return {"value": est_step_us, "unit": "us/step", "cores": int(threads), "kind": "oracle",
            "sample": f"{done_seqs} of {wl.batch} sequences ({done_tokens} of {total_tokens} cached tokens), "
                      f"{dt:.1f} s of fp64 numpy, scaled to the whole batch by token count"}, np.stack(outs)


_DECODE_KERNEL_SOURCES = ("decode_mfma.hip", "mfma_tile.h", "proj_mfma.hip")


def _kernel_sources_digest():
    """sha256 over the code (comments and blank space stripped) of the kernels of one decode step (the streaming
    decode kernel, its tile helpers, the absorb and merge + up-projection kernels): what the counter profiles were
    measured on."""
    import hashlib
    import re
    h = hashlib.sha256()
    for name in _DECODE_KERNEL_SOURCES:
        text = open(os.path.join(ROOT, "paper_2603_02188_amd", "csrc", name)).read()
        text = re.sub(r"/\*.*?\*/", " ", text, flags=re.S)
        text = re.sub(r"//[^\n]*", " ", text)
        h.update(name.encode())
        h.update(" ".join(text.split()).encode())
    return h.hexdigest()[:16]


def _measured_traffic(workload):
    """HBM bytes per launch of the decode kernel from the committed rocprofv3 counter summary (FETCH_SIZE and
    WRITE_SIZE runs, scaled by a plain copy of known size).  The summary names the digest of the kernel
    sources it was measured on: (None, reason) if no summary covers this workload or the sources changed."""
    path = os.path.join(ROOT, "profiles", f"decode_step_{workload}_counters.md")
    value, digest = None, None
    try:
        for line in open(path):
            if line.startswith("kernel sources digest:"):
                digest = line.split(":", 1)[1].strip()
            cells = [c.strip() for c in line.strip().strip("|").split("|")]
            if len(cells) == 7 and cells[0].startswith("decode_mfma_kernel"):
                value = float(cells[6])
    except OSError:
        return None, "no counter profile for this workload"
    if value is None:
        return None, "no decode kernel row in the counter profile"
    if digest != _kernel_sources_digest():
        return None, "the counter profile was measured on other kernel sources (digest %s)" % digest
    return value, "profiles/decode_step_%s_counters.md" % workload


def _time_us(fn, iters):
    import torch
    fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(iters):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3 / iters


def _baselines(inp, mlra_decode_us):
    """Decode-attention latency of the paper's comparison methods on the same batch (lengths, page table):
    GQA with 8 KV heads (MFMA streaming kernel, HBM-bound), GLA-2 and MLRA-2 (forms of the MLRA decode
    kernel, HBM-bound at half the arithmetic of MLRA-4) and MLA with one 512-dim latent (a plain MFMA
    kernel, not software-pipelined like the MLRA one: its ratio reflects kernel maturity as much as the
    method; by bytes moved MLA and full MLRA-4 are equal on one GPU)."""
    import torch
    from paper_2603_02188_amd import binding as mlra
    from paper_2603_02188_amd import inputs as gen
    from paper_2603_02188_amd import roofline as rf
    wl = inp.wl
    dev = "cuda"

    def up(x, bf16=True):
        t = torch.from_numpy(np.ascontiguousarray(x))
        return (t.view(torch.bfloat16) if bf16 and t.dtype == torch.uint16 else t).to(dev)

    out = torch.empty((wl.batch, wl.h, wl.d_h), dtype=torch.bfloat16, device=dev)
    gi = gen.make_gqa_inputs(wl, poison=False, seq_lens=inp.seq_lens)
    kp, vp, q = up(gi.k_pool), up(gi.v_pool), up(gi.q)
    pt, sl = up(gi.page_table, False), up(gi.seq_lens, False)
    ws = torch.empty(mlra.gqa_decode_workspace_bytes(wl.batch, wl.h, wl.d_h, int(pt.shape[1]) * wl.page_size),
                     dtype=torch.uint8, device=dev)
    gqa_us = _time_us(lambda: mlra.gqa_decode_attn(kp, vp, pt, sl, q, gi.scale, out=out, workspace=ws), 20)
    gqa_bytes = rf.gqa_bytes(inp.seq_lens, wl.h, wl.d_h, wl.g)
    del kp, vp
    inp1 = gen.as_single_latent(inp)
    lat1, rope1 = up(inp1.latent_pool), up(inp1.rope_pool)
    cache1 = mlra.Cache(lat1, rope1, up(inp1.page_table, False), up(inp1.seq_lens, False))
    q_abs1 = mlra.mlra_absorb_q(up(inp1.q_nope), up(inp1.w_uk))
    ws1 = torch.empty(mlra.mlra_decode_workspace_bytes(wl.batch, wl.h, 1, inp1.wl.d_cb, cache1.max_seq_len),
                      dtype=torch.uint8, device=dev)
    w_uv1, q_rope1 = up(inp1.w_uv), up(inp1.q_rope)
    mla_us = _time_us(lambda: mlra.mla_decode_attn(cache1, q_abs1, q_rope1, w_uv1, wl.tau, out=out, workspace=ws1), 20)
    del lat1, cache1
    # GLA-2 and MLRA-2 on caches of the same size (two 256-channel / four 128-channel latent heads, each
    # serving half of the heads), same lengths and page table, their own seeded values
    two = {}
    for key, shape in (("gla2", dict(n_blocks=2, d_cb=2 * wl.d_cb, groups=2)), ("mlra2", dict(groups=2))):
        wg = wl.scaled(name=wl.name + "-" + key, **shape)
        ig = gen.make_decode_inputs(wg, poison=False, seq_lens=inp.seq_lens)
        cg = mlra.Cache(up(ig.latent_pool), up(ig.rope_pool), up(ig.page_table, False), up(ig.seq_lens, False))
        qa = mlra.mlra2_absorb_q(up(ig.q_nope), up(ig.w_uk))
        wsg = torch.empty(mlra.mlra2_decode_workspace_bytes(wg.batch, wg.h, wg.n_blocks, wg.d_cb, cg.max_seq_len),
                          dtype=torch.uint8, device=dev)
        w_uvg, q_ropeg = up(ig.w_uv), up(ig.q_rope)
        two[key] = _time_us(lambda: mlra.mlra2_decode_attn(cg, qa, q_ropeg, w_uvg, wg.tau, out=out, workspace=wsg), 20)
        del cg, ig
    # what the bytes moved predict for the ratios (Table 1, one GPU): MLA and full MLRA-4 read the same cache
    mlra4_bytes = rf.decode_bytes(inp.seq_lens, wl.h, wl.d_h, wl.n_blocks, wl.d_cb, wl.d_r)["total"]
    mla_bytes = rf.decode_bytes(inp.seq_lens, wl.h, wl.d_h, 1, wl.n_blocks * wl.d_cb, wl.d_r)["total"]
    return {"mlra4_decode_us": mlra_decode_us,
            "mla_over_mlra4_bytes_model": mla_bytes / mlra4_bytes,
            "gqa_over_mlra4_bytes_model": gqa_bytes["total"] / mlra4_bytes,
            "mla_over_mlra4_is": "kernel-limited: the MLA baseline kernel runs far below its own roofline, so the "
                                 "measured ratio says more about the two kernels than about the two methods; the "
                                 "bytes-model ratio beside it is what Table 1 predicts on one GPU",
            "mlra2_decode_us": two["mlra2"], "mlra2_over_mlra4": two["mlra2"] / mlra_decode_us,
            "gla2_decode_us": two["gla2"], "gla2_over_mlra4": two["gla2"] / mlra_decode_us,
            "gla2_kernel": "MFMA decode kernel, GLA form (channel halves of a latent head on two waves)",
            "two_group_note": "MLRA-2, GLA-2 and MLA give about one round of workgroups on this batch, so a planning "
                              "kernel cuts the long sequences into chunks and hands them out longest first; on a "
                              "uniform batch (workloads M2, G2) the two-group forms take about 0.7x the MLRA-4 time",
            "gqa_decode_us": gqa_us, "gqa_over_mlra4": gqa_us / mlra_decode_us,
            "gqa_gbps": gqa_bytes["total"] / (gqa_us * 1e-6) / 1e9,
            "gqa_kernel": "MFMA streaming kernel",
            "mla_decode_us": mla_us, "mla_over_mlra4": mla_us / mlra_decode_us,
            "mla_kernel": "MFMA kernel (32-token tiles; scores split by heads, values by channels; not pipelined across tiles)",
            "paper_context": "H100, Section 4.5: MLRA-4 1.05-1.26x faster than GQA, about 2.8x faster than MLA "
                             "(MLRA-4 measured as one 4-way-TP device's share)"}


def main():
    a = _args()
    if a.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (the 4-way tensor-parallel case is "
              "benchmarked as one device's share, workload C2). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2603_02188_amd import binding as mlra
    from paper_2603_02188_amd import inputs as gen
    from paper_2603_02188_amd import roofline as rf

    if not torch.cuda.is_available():
        print("bench.py needs a GPU (the MLRA decode path has no CPU fallback)", file=sys.stderr)
        sys.exit(2)
    mlra.load_library()
    wl = gen.WORKLOADS[a.workload]
    dev = "cuda"
    t_gen = time.perf_counter()
    inp = gen.make_decode_inputs(wl, poison=False, hole=False)
    t_gen = time.perf_counter() - t_gen

    def up(x, tag=None):
        t = torch.from_numpy(np.ascontiguousarray(x))
        if tag == "bf16":
            t = t.view(torch.bfloat16)
        return t.to(dev)

    cache_bytes = inp.latent_pool.nbytes + inp.rope_pool.nbytes
    copies = a.copies or max(2, min(32, int(np.ceil(3.0e9 / cache_bytes))))
    lat0, rope0 = up(inp.latent_pool, wl.dtype), up(inp.rope_pool, wl.dtype)
    page_table, seq_lens = up(inp.page_table), up(inp.seq_lens)
    caches = [mlra.Cache(lat0, rope0, page_table, seq_lens)]
    for _ in range(copies - 1):
        caches.append(mlra.Cache(lat0.clone(), rope0.clone(), page_table, seq_lens))
    q_nope, q_rope = up(inp.q_nope, wl.dtype), up(inp.q_rope, wl.dtype)
    w_uk, w_uv = up(inp.w_uk, wl.dtype), up(inp.w_uv, wl.dtype)
    c_new, k_new, positions = up(inp.c_kv_new), up(inp.k_rope_new), up(inp.positions)
    q_abs = torch.empty((wl.batch, wl.n_blocks, wl.h // wl.groups, wl.d_cb), dtype=q_nope.dtype, device=dev)
    out = torch.empty((wl.batch, wl.h, wl.d_h), dtype=torch.bfloat16, device=dev)
    # (the absorb call folds tau log2(e) into the queries, the decode call is told so)
    if wl.groups == 2:   # MLRA-2 (Eq. (6))
        absorb_q, decode_attn, ws_query = mlra.mlra2_absorb_q_folded, mlra.mlra2_decode_attn, mlra.mlra2_decode_workspace_bytes
    else:
        absorb_q, decode_attn, ws_query = mlra.mlra_absorb_q_folded, mlra.mlra_decode_attn, mlra.mlra_decode_workspace_bytes
    ws_bytes = ws_query(wl.batch, wl.h, wl.n_blocks, wl.d_cb, caches[0].max_seq_len)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)

    pre = None
    if a.pre_attention:
        # hidden size and head count of the paper's decode benchmark (Section 4.5); d_c' = 1536 is this
        # build's choice (the paper does not print it for that benchmark)
        pre = gen.make_pre_inputs(wl, d=7168, d_cq=1536, unit_gains=True)
        pw = mlra.PreWeights(up(pre.w_dq, wl.dtype), up(pre.w_dkv, wl.dtype), up(pre.w_kr, wl.dtype),
                             up(pre.w_uq, wl.dtype), up(pre.w_qr, wl.dtype), wl.h, pre.alpha_q, pre.alpha_kv,
                             None, None, pre.eps, pre.rope_base)
        hidden = up(pre.hidden, wl.dtype)
        pre_ws = torch.empty(mlra.mlra_pre_attention_workspace_bytes(wl.batch, pre.d, pre.d_cq, wl.n_blocks, wl.d_cb,
                                                                     wl.d_r, wl.h, wl.d_h, q_nope.dtype),
                             dtype=torch.uint8, device=dev)
        q_nope, q_rope = torch.empty_like(q_nope), torch.empty_like(q_rope)

    if a.q_len > 1:
        if wl.groups != 1 or a.pre_attention:
            print("--q-len > 1 applies to the MLRA-4 workloads without --pre-attention", file=sys.stderr)
            sys.exit(2)
        rng = np.random.default_rng([wl.seed, 0x4D7, a.q_len])
        q_nope = up(gen.to_storage(rng.standard_normal((wl.batch * a.q_len, wl.h, wl.d_h), dtype=np.float32), wl.dtype), wl.dtype)
        q_rope = up(gen.to_storage(rng.standard_normal((wl.batch, a.q_len, wl.h, wl.d_r), dtype=np.float32), wl.dtype), wl.dtype)
        q_abs = torch.empty((wl.batch * a.q_len, wl.n_blocks, wl.h, wl.d_cb), dtype=q_nope.dtype, device=dev)
        out = torch.empty((wl.batch, a.q_len, wl.h, wl.d_h), dtype=torch.bfloat16, device=dev)
        ws = torch.empty(mlra.mlra_decode_multi_workspace_bytes(wl.batch, a.q_len, wl.h, wl.n_blocks, wl.d_cb,
                                                                wl.page_size, caches[0].page_table.shape[1]),
                         dtype=torch.uint8, device=dev)
        q_abs5 = q_abs.view(wl.batch, a.q_len, wl.n_blocks, wl.h, wl.d_cb)

        def decode_attn(c, q_abs_, q_rope_, w_uv_, tau, out_scale, out=None, workspace=None):   # noqa: F811
            return mlra.mlra_decode_attn_multi(c, q_abs5, q_rope_, w_uv_, tau, out_scale, out=out, workspace=workspace)

    q_rope_s = torch.empty_like(q_rope)   # the RoPE queries times tau log2(e)

    def step(i):
        c = caches[i % copies]
        if pre is None:
            mlra.mlra_append_kv(c, c_new, k_new, positions)
        else:
            mlra.mlra_pre_attention(c, pw, hidden, positions, q_nope, q_rope, pre_ws)
        absorb_q(q_nope, w_uk, q_rope, wl.tau, q_abs, q_rope_s)
        decode_attn(c, q_abs, q_rope_s, w_uv, mlra.SCALE_FOLDED, 1.0, out=out, workspace=ws)

    def decode_only(i):
        decode_attn(caches[i % copies], q_abs, q_rope_s, w_uv, mlra.SCALE_FOLDED, 1.0, out=out, workspace=ws)

    if a.copy_calibration:
        # a plain copy of known size: 2^30 bytes read, 2^30 bytes written per dispatch
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # Untimed settle phase: the chip raises its clocks over the first milliseconds of load, so a run of a few
    # steps would time that transient.  Steps run in batches of 20 until the decode kernel's own time (events on
    # its launch) has not improved by 1 % for two batches in a row, or --max-settle steps have run.
    settle_steps, settle_trace = 0, []
    if a.max_settle > 0:
        best, stale, batch_n = float("inf"), 0, 20
        while settle_steps < a.max_settle:
            mlra.mlra_kernel_timing_begin(batch_n)
            for i in range(batch_n):
                step(settle_steps + i)
            torch.cuda.synchronize()
            batch_ms = mlra.mlra_kernel_timing_end()[0]
            settle_steps += batch_n
            settle_trace.append(round(batch_ms * 1e3, 1))
            if batch_ms < 0.99 * best:
                best, stale = batch_ms, 0
            else:
                stale += 1
                if stale >= 2:
                    break

    for i in range(a.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(a.steps):
        step(a.warmup + i)
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / a.steps

    # the same loop again with a start and a stop event on each decode kernel launch (inside the library,
    # on the launch stream: the kernel's own execution interval), for the roofline of the dominant kernel
    mlra.mlra_kernel_timing_begin(a.steps)
    for i in range(a.steps):
        step(a.warmup + a.steps + i)
    torch.cuda.synchronize()
    main_ms, epi_ms, calls = mlra.mlra_kernel_timing_end()

    # the same steps captured once in a HIP graph (one graph = one step on each rotated cache copy) and
    # replayed: what a serving loop that replays a captured step pays, without the per-call host work
    graph_us = None
    if not a.no_graph:
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for i in range(copies):
                step(i)
        n_replays = max(10, (2 * a.steps + copies - 1) // copies)
        g.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n_replays):
            g.replay()
        torch.cuda.synchronize()
        graph_us = (time.perf_counter() - t0) * 1e6 / (n_replays * copies)

    # shader clock under this load: one wavefront on a second stream (default priority) counts shader cycles
    # against the 100 MHz counter while a few more, untimed, steps run (it shares a SIMD with a decode
    # workgroup, so these steps are not part of any figure)
    shader_clock_ghz = None
    if not a.no_probes:
        clock_out = torch.zeros(2, dtype=torch.int64, device=dev)
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        n_probe = max(10, min(a.steps, 50))
        for i in range(n_probe):
            if i == 2:
                mlra.mlra_probe_shader_clock(clock_out, max(200, int(0.6 * (n_probe - 2) * ms_per_step * 1e3)), stream=side)
            step(i)
        torch.cuda.synchronize()
        cyc, ticks = [int(v) for v in clock_out.cpu().tolist()]
        shader_clock_ghz = cyc / (ticks * 10.0) if ticks > 0 else None

    # decode-attention-only latency (per-step samples with events on the launch stream)
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(a.steps)]
    for i, (e0, e1) in enumerate(evs):
        e0.record()
        decode_only(i)
        e1.record()
    torch.cuda.synchronize()
    dec = np.array([e0.elapsed_time(e1) for e0, e1 in evs]) * 1e3

    # streaming-read ceiling of this machine: a plain read of the rotated cache copies (>= 3 GB, so the
    # memory-side cache cannot serve it), best of three passes
    stream_gbps = None
    if not a.no_probes:
        sink = torch.zeros(4096, dtype=torch.int32, device=dev)
        bufs = [c.latent for c in caches]
        total = sum(b.numel() * b.element_size() for b in bufs)
        for _ in range(3):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for b in bufs:
                mlra.mlra_probe_stream_read(b, sink, 4096)
            e1.record()
            torch.cuda.synchronize()
            gbps = total / (e0.elapsed_time(e1) * 1e-3) / 1e9
            stream_gbps = gbps if stream_gbps is None else max(stream_gbps, gbps)

    bytes_decode = rf.decode_bytes(inp.seq_lens, wl.h, wl.d_h, wl.n_blocks, wl.d_cb, wl.d_r, groups=wl.groups)
    if a.q_len > 1:   # the cache is shared by the queries of a sequence; queries and outputs are not
        for k in ("q_abs", "q_rope", "out"):
            bytes_decode["total"] += (a.q_len - 1) * bytes_decode[k]
            bytes_decode[k] *= a.q_len
    bytes_step = (bytes_decode["total"] + rf.absorb_bytes(wl.batch, wl.h, wl.d_h, wl.n_blocks, wl.d_cb, groups=wl.groups)
                  + rf.append_bytes(wl.batch, wl.n_blocks, wl.d_cb, wl.d_r))
    flops = rf.decode_flops(inp.seq_lens, wl.h, wl.d_h, wl.n_blocks, wl.d_cb, wl.d_r, groups=wl.groups)
    if a.q_len > 1:
        flops = sum(rf.decode_flops(np.maximum(inp.seq_lens - (a.q_len - 1 - j), 0), wl.h, wl.d_h, wl.n_blocks,
                                    wl.d_cb, wl.d_r) for j in range(a.q_len))
    # dominant kernel: the context-streaming decode kernel; its algorithmic bytes are the cache rows of
    # every valid token plus the absorbed / RoPE queries (W^UV and the output belong to the epilogue)
    kernel_bytes = bytes_decode["cache"] + bytes_decode["q_abs"] + bytes_decode["q_rope"]
    achieved = kernel_bytes / (main_ms * 1e-3) / 1e9 if main_ms > 0 else 0.0

    traffic, traffic_note = _measured_traffic(a.workload)
    res = {
        "metric": "decode attention us/step, %s bf16 (append_kv + absorb_q + decode_attn)"
                  % ("GLA-2" if wl.groups == 2 and wl.n_blocks == 2 else "MLRA-2" if wl.groups == 2 else "MLRA-4"),
        "value": ms_per_step * 1e3, "unit": "us/step", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": wl.name, "batch": wl.batch, "context": [wl.n_min, wl.n_max], "n_blocks": wl.n_blocks,
                   "d_cb": wl.d_cb, "d_r": wl.d_r, "h": wl.h, "d_h": wl.d_h, "head_groups": wl.groups, "page_size": wl.page_size,
                   "cache_copies_rotated": copies, "seed": wl.seed, "q_len": a.q_len},
        "step_gbps": bytes_step / (ms_per_step * 1e-3) / 1e9,
        "step_frac_of_hbm_peak": bytes_step / (ms_per_step * 1e-3) / 1e9 / rf.HBM_PEAK_GBS,
        "decode_attn_us": {"median": float(np.median(dec)), "p10": float(np.percentile(dec, 10)),
                           "p90": float(np.percentile(dec, 90))},
        "decode_attn_gbps": bytes_decode["total"] / (float(np.median(dec)) * 1e-6) / 1e9,
        "decode_attn_tflops": flops / (float(np.median(dec)) * 1e-6) / 1e12,
        "kernels_us": {"decode_main": main_ms * 1e3, "merge_upproj": epi_ms * 1e3, "calls": calls},
        "graph_replay_us_per_step": graph_us,
        "settle_steps": settle_steps, "settle_decode_main_us": settle_trace,
        "shader_clock_ghz_under_load": shader_clock_ghz,
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": rf.HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / rf.HBM_PEAK_GBS, "traffic": traffic, "traffic_source": traffic_note,
                     "stream_ceiling_gbps": stream_gbps,
                     "frac_of_stream_ceiling": achieved / stream_gbps if stream_gbps else None,
                     "kernel": "mlra decode main kernel", "algorithmic_bytes": kernel_bytes,
                     "mfma_tflops": (flops - wl.batch * wl.h * 2.0 * (wl.n_blocks // wl.groups) * wl.d_cb * wl.d_h)
                     / (main_ms * 1e-3) / 1e12 if main_ms > 0 else 0.0},
        "input_gen_s": t_gen,
    }
    if pre is not None:
        pre_us = _time_us(lambda: mlra.mlra_pre_attention(caches[0], pw, hidden, positions, q_nope, q_rope, pre_ws), 50)
        pre_bytes = 2 * (pre.d * (pre.d_cq + wl.n_blocks * wl.d_cb + wl.d_r) + pre.d_cq * wl.h * (wl.d_h + wl.d_r)
                         + wl.batch * (pre.d + wl.h * (wl.d_h + wl.d_r)))
        res["metric"] = res["metric"].replace("append_kv", "pre_attention")
        res["pre_attention"] = {"us": pre_us, "weights_and_io_bytes": pre_bytes,
                                "gbps": pre_bytes / (pre_us * 1e-6) / 1e9,
                                "frac_of_hbm_peak": pre_bytes / (pre_us * 1e-6) / 1e9 / rf.HBM_PEAK_GBS,
                                "d": pre.d, "d_cq": pre.d_cq}
    if a.baselines:
        if a.workload != "C5":
            print("--baselines applies to workload C5 (the paged mixed batch)", file=sys.stderr)
            sys.exit(2)
        res["baselines"] = _baselines(inp, float(np.median(dec)))
    if a.q_len > 1:
        res["metric"] = res["metric"].replace("decode_attn)", "decode_attn_multi, %d query tokens per sequence)" % a.q_len)
        # the cache is streamed once for q_len queries, so the path is bound by the matrix pipe
        tf = res["roofline"]["mfma_tflops"]
        res["roofline"].update({"bound": "mfma", "achieved": tf, "peak": rf.MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                                "frac": tf / rf.MFMA_BF16_PEAK_TFLOPS, "traffic": None,
                                "hbm_gbps_algorithmic": achieved})
    if not a.no_cpu_baseline and a.q_len == 1:
        base, ref = _cpu_baseline(inp)
        res["cpu_baseline"] = base
        # the sequences the oracle got through, element by element against the last step's output
        got = out.to(torch.float64).cpu().numpy()[: ref.shape[0]]
        res["max_rel_err_vs_oracle"] = float(np.max(np.abs(got - ref)) / np.max(np.abs(ref)))
        res["max_rel_err_sequences"] = int(ref.shape[0])
    print(json.dumps(res))


if __name__ == "__main__":
    main()
