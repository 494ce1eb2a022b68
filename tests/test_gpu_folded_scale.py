"""GPU parity of the calls that fold the softmax scale into the queries (mlra_absorb_q_folded /
mlra2_absorb_q_folded + decode with softmax_scale = MLRA_SCALE_FOLDED; Eq. (5): both score terms carry tau)
against the fp64 oracle, which applies tau to the scores as the equation writes it.  Bars as everywhere:
max|gpu - ref| / max|ref| <= 1e-2 (bf16), <= 1e-5 (fp32); log-sum-exp within 2e-2 / 1e-4."""
import sys

import numpy as np
import pytest
import torch

from oracle import mlra_oracle as orc
from paper_2603_02188_amd import binding as mlra
from paper_2603_02188_amd import inputs as gen

from gpu_util import device_cache, device_queries_weights, host, max_rel_err, oracle_views

pytestmark = pytest.mark.gpu

TOL = {"bf16": 1e-2, "f32": 1e-5}


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def _run(wl, lens, form):
    _say(f"[case] folded scale, {form}: {wl.name} B={wl.batch} h={wl.h} NB={wl.n_blocks} d_cb={wl.d_cb} {wl.dtype} "
         f"page={wl.page_size} lens={np.asarray(lens).tolist()}")
    inp = gen.make_decode_inputs(wl, poison=True, seq_lens=np.asarray(lens, dtype=np.int32))
    cache = device_cache(inp)
    q_nope, q_rope, w_uk, w_uv = device_queries_weights(inp)
    q_rope_before = q_rope.clone()
    v = oracle_views(inp)
    args = (v["latent_pool"], v["rope_pool"], v["page_table"], v["seq_lens"], v["q_nope"], v["q_rope"], v["w_uk"],
            v["w_uv"], wl.tau)
    if form == "mlra4":
        q_abs, q_rope_s = mlra.mlra_absorb_q_folded(q_nope, w_uk, q_rope, wl.tau)
        lse = torch.empty((wl.batch, wl.n_blocks, wl.h), dtype=torch.float32, device="cuda")
        out = mlra.mlra_decode_attn(cache, q_abs, q_rope_s, w_uv, mlra.SCALE_FOLDED, 1.0, out_dtype=torch.float32, lse=lse)
        ref, ref_lse = orc.mlra_decode_batch(*args, 1.0, return_lse=True)
    else:
        q_abs, q_rope_s = mlra.mlra2_absorb_q_folded(q_nope, w_uk, q_rope, wl.tau)
        lse = None
        out = mlra.mlra2_decode_attn(cache, q_abs, q_rope_s, w_uv, mlra.SCALE_FOLDED, 1.0, out_dtype=torch.float32)
        ref = orc.mlra2_decode_batch(*args, 1.0) if form == "mlra2" else orc.gla2_decode_batch(*args)
        ref_lse = None
    torch.cuda.synchronize()
    assert torch.equal(q_rope.view(torch.int16) if q_rope.dtype == torch.bfloat16 else q_rope,
                       q_rope_before.view(torch.int16) if q_rope.dtype == torch.bfloat16 else q_rope_before), \
        "the caller's q_rope was modified"
    # the folded RoPE queries are the stored ones times tau log2(e), rounded once
    want = host(q_rope_before) * (wl.tau * np.log2(np.e))
    assert max_rel_err(host(q_rope_s), want) <= (4e-3 if wl.dtype == "bf16" else 1e-6)
    err = max_rel_err(host(out), ref)
    _say(f"       max rel err {err:.3e} (tol {TOL[wl.dtype]:g})")
    assert err <= TOL[wl.dtype]
    if ref_lse is not None:
        got_lse = host(lse)
        live = np.isfinite(ref_lse)
        assert np.array_equal(np.isfinite(got_lse), live)
        if live.any():
            assert np.max(np.abs(got_lse[live] - ref_lse[live])) <= (2e-2 if wl.dtype == "bf16" else 1e-4)


def test_folded_fp32_generic_kernels():
    wl = gen.WORKLOADS["C1"].scaled(name="folded-fp32", batch=6)
    _run(wl, [0, 1, 64, 65, 200, 256], "mlra4")


def test_folded_fp32_odd_dims():
    wl = gen.WORKLOADS["C1"].scaled(name="folded-odd", batch=3, n_min=5, n_max=333, h=5, d_h=24, d_cb=40, d_r=12,
                                    n_blocks=3, page_size=16)
    _run(wl, [5, 333, 100], "mlra4")


def test_folded_bf16_mlra4_tiles_ragged_and_split():
    # one chunk per sequence with several tiles and a ragged tail, an empty sequence, and a context long
    # enough to be cut into chunks
    wl = gen.WORKLOADS["C3"].scaled(name="folded-bf16", batch=6, n_min=0, n_max=6000)
    _run(wl, [0, 1, 63, 700, 2049, 6000], "mlra4")


def test_folded_bf16_mlra2_and_gla2():
    wl = gen.WORKLOADS["M2"].scaled(name="folded-mlra2", batch=4, n_min=1, n_max=3000)
    _run(wl, [1, 64, 1500, 3000], "mlra2")
    wl = gen.WORKLOADS["G2"].scaled(name="folded-gla2", batch=4, n_min=1, n_max=3000)
    _run(wl, [65, 2, 3000, 1111], "gla2")


def test_folded_argument_errors():
    wl = gen.WORKLOADS["C1"].scaled(name="folded-errors", batch=2)
    inp = gen.make_decode_inputs(wl, seq_lens=np.array([3, 4], dtype=np.int32))
    q_nope, q_rope, w_uk, _ = device_queries_weights(inp)
    for bad in (0.0, -1.0, float("nan")):
        with pytest.raises(RuntimeError):
            mlra.mlra_absorb_q_folded(q_nope, w_uk, q_rope, bad)
