"""GPU parity at the full benchmark sizes (workloads C2..C5), in the launch configuration bench.py
times.  The fp64 oracle is fast enough to check every output element of every sequence."""
import sys

import numpy as np
import pytest
import torch

from oracle import mlra_oracle as orc
from paper_2603_02188_amd import binding as mlra
from paper_2603_02188_amd import inputs as gen

from gpu_util import (device_cache, device_queries_weights, host, max_rel_err, oracle_views, run_mlra_path,
                      to_device)

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


@pytest.mark.parametrize("key", ["C2", "C3", "C4", "C5"])
def test_full_size_mlra(key):
    wl = gen.WORKLOADS[key]
    _say(f"[case] full size {wl.name}: generating inputs")
    inp = gen.make_decode_inputs(wl, poison=True, hole=True)
    out, lse, _ = run_mlra_path(inp, out_dtype=torch.bfloat16, append=True)
    _say("       GPU done; running the oracle")
    full = gen.make_decode_inputs(wl, poison=True, hole=False)
    v = oracle_views(full)
    ref, ref_lse = orc.mlra_decode_batch(v["latent_pool"], v["rope_pool"], v["page_table"], v["seq_lens"],
                                         v["q_nope"], v["q_rope"], v["w_uk"], v["w_uv"], wl.tau, return_lse=True)
    err = max_rel_err(out, ref)
    lse_err = float(np.max(np.abs(lse - ref_lse)))
    _say(f"       max rel err {err:.3e} (tol 1e-2), max |lse - ref| {lse_err:.3e}, tokens {int(inp.seq_lens.sum())}")
    assert err <= 1e-2
    assert lse_err <= 2e-2


def test_full_size_c5_mla_and_gqa_baselines():
    wl = gen.WORKLOADS["C5"]
    _say("[case] full size C5 MLA baseline")
    inp = gen.as_single_latent(gen.make_decode_inputs(wl, poison=True))
    cache = device_cache(inp)
    q_nope, q_rope, w_uk, w_uv = device_queries_weights(inp)
    q_abs = mlra.mlra_absorb_q(q_nope, w_uk)
    out = host(mlra.mla_decode_attn(cache, q_abs, q_rope, w_uv, wl.tau, out_dtype=torch.float32))
    v = oracle_views(inp)
    ref = orc.mlra_decode_batch(v["latent_pool"], v["rope_pool"], v["page_table"], v["seq_lens"], v["q_nope"],
                                v["q_rope"], v["w_uk"], v["w_uv"], wl.tau)
    err = max_rel_err(out, ref)
    _say(f"       MLA max rel err {err:.3e}")
    assert err <= 1e-2
    del cache, inp, v
    torch.cuda.empty_cache()

    _say("[case] full size C5 GQA baseline (g = 8)")
    gi = gen.make_gqa_inputs(wl, poison=True)
    out = host(mlra.gqa_decode_attn(to_device(gi.k_pool, wl.dtype), to_device(gi.v_pool, wl.dtype),
                                    to_device(gi.page_table), to_device(gi.seq_lens), to_device(gi.q, wl.dtype),
                                    gi.scale, out_dtype=torch.float32))
    # every sequence (the GQA oracle walks heads one by one: about a minute)
    ref = orc.gqa_decode_batch(gen.to_f64(gi.k_pool, wl.dtype), gen.to_f64(gi.v_pool, wl.dtype), gi.page_table,
                               gi.seq_lens, gen.to_f64(gi.q, wl.dtype), gi.scale)
    err = max_rel_err(out, ref)
    _say(f"       GQA max rel err {err:.3e} on all {wl.batch} sequences")
    assert err <= 1e-2
