"""mlra_decode_attn_static (the entry point that allocates nothing) against mlra_decode_attn: same
kernels on the library's built-in scratch array instead of a caller workspace, so the outputs must agree
bit for bit, and both must meet the oracle bar.  Two calls in a row, the second with a smaller input
(the scratch array keeps what the first call left in it)."""
import ctypes
import sys

import numpy as np
import pytest
import torch

from oracle import mlra_oracle as orc
from paper_2603_02188_amd import binding as mlra
from paper_2603_02188_amd import inputs as gen

from gpu_util import device_cache, device_queries_weights, host, max_rel_err, oracle_views

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def _both_ways(inp, out_scale):
    wl = inp.wl
    _say(f"[case] static vs workspace: {wl.name} B={wl.batch} n=[{wl.n_min},{wl.n_max}] NB={wl.n_blocks} {wl.dtype}")
    cache = device_cache(inp)
    q_nope, q_rope, w_uk, w_uv = device_queries_weights(inp)
    q_abs = mlra.mlra_absorb_q(q_nope, w_uk)
    lse_a = torch.full((wl.batch, wl.n_blocks, wl.h), float("nan"), device="cuda")
    lse_b = torch.full_like(lse_a, float("nan"))
    out_a = mlra.mlra_decode_attn(cache, q_abs, q_rope, w_uv, wl.tau, out_scale, out_dtype=torch.float32, lse=lse_a)
    out_b = torch.full_like(out_a, float("nan"))
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    mlra.mlra_decode_attn_static(cache, q_abs, q_rope, w_uv, wl.tau, out_scale, out_b, lse=lse_b)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before          # nothing went through torch's allocator either
    a, b = host(out_a), host(out_b)
    assert np.array_equal(a, b)
    assert np.array_equal(host(lse_a), host(lse_b), equal_nan=True)
    v = oracle_views(inp)
    ref = orc.mlra_decode_batch(v["latent_pool"], v["rope_pool"], v["page_table"], v["seq_lens"], v["q_nope"],
                                v["q_rope"], v["w_uk"], v["w_uv"], wl.tau, out_scale)
    err = max_rel_err(b, ref)
    tol = 1e-2 if wl.dtype == "bf16" else 1e-5
    _say(f"       max rel err vs oracle {err:.3e} (tol {tol:g})")
    assert err <= tol


def test_static_scratch_two_calls_second_smaller():
    # first: split mode (few sequences, long context: fp32 partials of many chunks fill the scratch)
    big = gen.WORKLOADS["C2"].scaled(batch=3, n_min=3000, n_max=9000)
    _both_ways(gen.make_decode_inputs(big, seq_lens=np.array([9000, 3001, 6100], dtype=np.int32)), 1.0)
    # second, smaller: MLRA-4 with ragged, empty and one-token sequences on the same scratch
    small = gen.WORKLOADS["C3"].scaled(batch=4, n_min=0, n_max=700)
    _both_ways(gen.make_decode_inputs(small, seq_lens=np.array([700, 0, 1, 65], dtype=np.int32)), 0.5)
    # third: the generic fp32 kernels (workload C1) use the same scratch
    _both_ways(gen.make_decode_inputs(gen.WORKLOADS["C1"]), 1.0)


def test_static_scratch_rejects_shapes_beyond_its_size():
    """A call that claims 4096 sequences needs far more than the 40 MiB scratch array: it must be refused
    with MLRA_ERR_WORKSPACE and enqueue nothing (the tensors here are far too small for that shape, and
    the output stays untouched)."""
    wl = gen.WORKLOADS["C3"].scaled(batch=2, n_min=10, n_max=100)
    inp = gen.make_decode_inputs(wl)
    cache = device_cache(inp)
    q_nope, q_rope, w_uk, w_uv = device_queries_weights(inp)
    q_abs = mlra.mlra_absorb_q(q_nope, w_uk)
    lib = mlra.load_library()
    cs = cache.struct()
    cs.max_pages_per_seq = 8192          # claims 524288 tokens per sequence: nothing is read before the size check
    out = torch.zeros((wl.batch, wl.h, wl.d_h), dtype=torch.float32, device="cuda")
    need = mlra.mlra_decode_workspace_bytes(4096, wl.h, wl.n_blocks, wl.d_cb, 8192 * wl.page_size)
    assert need > 40 << 20
    st = lib.mlra_decode_attn_static(ctypes.byref(cs), 4096, wl.h, wl.d_h, mlra._ptr(q_abs), mlra._ptr(q_rope),
                                     mlra._ptr(w_uv), wl.tau, 1.0, mlra._ptr(out), mlra.MLRA_F32, None, None)
    assert st == -4, mlra.strerror(st)
    torch.cuda.synchronize()
    assert float(out.abs().max()) == 0.0
