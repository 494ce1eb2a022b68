"""A decode step captured in a HIP graph gives, on every replay, exactly what the eager calls give."""
import numpy as np
import pytest
import torch

from paper_2603_02188_amd import binding as mlra
from paper_2603_02188_amd import inputs as gen

from gpu_util import device_cache, device_queries_weights

pytestmark = pytest.mark.gpu


def test_graph_replays_match_eager():
    wl = gen.WORKLOADS["C3"].scaled(batch=5, n_min=200, n_max=1500)
    inp = gen.make_decode_inputs(wl, poison=True, hole=True)
    cache = device_cache(inp)
    qn, qr, wk, wv = device_queries_weights(inp)
    dev = qn.device
    c_new = torch.from_numpy(inp.c_kv_new).to(dev)
    k_new = torch.from_numpy(inp.k_rope_new).to(dev)
    pos = torch.from_numpy(inp.positions).to(dev)
    q_abs = torch.empty((wl.batch, wl.n_blocks, wl.h, wl.d_cb), dtype=qn.dtype, device=dev)
    ws = torch.empty(mlra.mlra_decode_workspace_bytes(wl.batch, wl.h, wl.n_blocks, wl.d_cb, cache.max_seq_len),
                     dtype=torch.uint8, device=dev)
    out_eager = torch.empty((wl.batch, wl.h, wl.d_h), dtype=torch.float32, device=dev)
    out_graph = torch.empty_like(out_eager)

    def step(out):
        mlra.mlra_append_kv(cache, c_new, k_new, pos)
        mlra.mlra_absorb_q(qn, wk, q_abs)
        mlra.mlra_decode_attn(cache, q_abs, qr, wv, wl.tau, 1.0, out=out, workspace=ws)

    step(out_eager)                      # eager reference (also the warm-up the capture needs)
    torch.cuda.synchronize()
    ref = out_eager.cpu().numpy().copy()
    assert np.isfinite(ref).all()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step(out_graph)
    for replay in range(4):
        out_graph.fill_(float("nan"))
        q_abs.zero_()                    # eager work between the replays
        ws.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        got = out_graph.cpu().numpy()
        assert np.array_equal(got, ref), f"replay {replay} differs from the eager result"


def _replay_and_compare(g, outs_graph, refs, scratch):
    for replay in range(3):
        for o in outs_graph:
            o.fill_(float("nan"))
        for t in scratch:                # eager work between the replays
            t.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for o, ref in zip(outs_graph, refs):
            assert np.array_equal(o.float().cpu().numpy(), ref), f"replay {replay} differs from the eager result"


def test_graph_replays_match_eager_pre_attention_and_mlra2():
    """The step that starts from hidden states (pre-attention, absorb, MLRA-2 decode) captured as one graph."""
    wl = gen.WORKLOADS["M2"].scaled(batch=6, n_min=100, n_max=1200)
    inp = gen.make_decode_inputs(wl, poison=True, hole=True)
    pre = gen.make_pre_inputs(wl, 1024, 384)
    tag = wl.dtype
    cache = device_cache(inp)
    qn0, qr, wk, wv = device_queries_weights(inp)
    dev = qn0.device
    up = lambda a: (torch.from_numpy(np.ascontiguousarray(a)).view(torch.bfloat16) if a.dtype == np.uint16
                    else torch.from_numpy(np.ascontiguousarray(a))).to(dev)
    # the pre-attention produces queries for all h heads; MLRA-2 reads them as two groups of h / 2
    W = mlra.PreWeights(up(pre.w_dq), up(pre.w_dkv), up(pre.w_kr), up(pre.w_uq), up(pre.w_qr), wl.h, pre.alpha_q,
                        pre.alpha_kv, up(pre.gain_q), up(pre.gain_kv), pre.eps, pre.rope_base)
    hidden, pos = up(pre.hidden), up(inp.positions)
    q_nope = torch.empty((wl.batch, wl.h, wl.d_h), dtype=qn0.dtype, device=dev)
    q_rope = torch.empty((wl.batch, wl.h, wl.d_r), dtype=qn0.dtype, device=dev)
    pre_ws = torch.empty(mlra.mlra_pre_attention_workspace_bytes(wl.batch, pre.d, pre.d_cq, wl.n_blocks, wl.d_cb,
                                                                 wl.d_r, wl.h, wl.d_h, qn0.dtype),
                         dtype=torch.uint8, device=dev)
    q_abs = torch.empty((wl.batch, wl.n_blocks, wl.h // 2, wl.d_cb), dtype=qn0.dtype, device=dev)
    ws = torch.empty(mlra.mlra2_decode_workspace_bytes(wl.batch, wl.h, wl.n_blocks, wl.d_cb, cache.max_seq_len),
                     dtype=torch.uint8, device=dev)
    out_eager = torch.empty((wl.batch, wl.h, wl.d_h), dtype=torch.float32, device=dev)
    out_graph = torch.empty_like(out_eager)

    def step(out):
        mlra.mlra_pre_attention(cache, W, hidden, pos, q_nope, q_rope, pre_ws)
        mlra.mlra2_absorb_q(q_nope, wk, q_abs)
        mlra.mlra2_decode_attn(cache, q_abs, q_rope, wv, wl.tau, 1.0, out=out, workspace=ws)

    step(out_eager)
    torch.cuda.synchronize()
    ref = out_eager.cpu().numpy().copy()
    assert np.isfinite(ref).all()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step(out_graph)
    _replay_and_compare(g, [out_graph], [ref], [q_abs, ws, pre_ws, q_nope, q_rope])


def test_graph_replays_match_eager_multi_token():
    wl = gen.WORKLOADS["C3"].scaled(batch=3, n_min=300, n_max=1500)
    q_len = 3
    inp = gen.make_decode_inputs(wl, poison=True)
    cache = device_cache(inp)
    _, _, wk, wv = device_queries_weights(inp)
    dev = wk.device
    rng = np.random.default_rng(99)
    bf = lambda a: torch.from_numpy(gen.to_storage(a.astype(np.float32), wl.dtype)).view(torch.bfloat16).to(dev)
    q_nope = bf(rng.standard_normal((wl.batch * q_len, wl.h, wl.d_h)))
    q_rope = bf(rng.standard_normal((wl.batch, q_len, wl.h, wl.d_r)))
    q_abs = torch.empty((wl.batch * q_len, wl.n_blocks, wl.h, wl.d_cb), dtype=q_nope.dtype, device=dev)
    q_abs5 = q_abs.view(wl.batch, q_len, wl.n_blocks, wl.h, wl.d_cb)
    ws = torch.empty(mlra.mlra_decode_multi_workspace_bytes(wl.batch, q_len, wl.h, wl.n_blocks, wl.d_cb,
                                                            wl.page_size, cache.page_table.shape[1]),
                     dtype=torch.uint8, device=dev)
    out_eager = torch.empty((wl.batch, q_len, wl.h, wl.d_h), dtype=torch.float32, device=dev)
    out_graph = torch.empty_like(out_eager)

    def step(out):
        mlra.mlra_absorb_q(q_nope, wk, q_abs)
        mlra.mlra_decode_attn_multi(cache, q_abs5, q_rope, wv, wl.tau, 1.0, out=out, workspace=ws)

    step(out_eager)
    torch.cuda.synchronize()
    ref = out_eager.cpu().numpy().copy()
    assert np.isfinite(ref).all()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step(out_graph)
    _replay_and_compare(g, [out_graph], [ref], [q_abs, ws])
