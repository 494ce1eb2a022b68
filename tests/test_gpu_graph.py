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
