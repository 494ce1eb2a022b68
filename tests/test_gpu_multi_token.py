"""GPU parity of mlra_decode_attn_multi (several query tokens per sequence, causal tail of Eq. (5))
against the fp64 oracle.  Bars: 1e-2 (bf16), 1e-5 (fp32), max-abs-normalised."""
import sys

import numpy as np
import pytest
import torch

from oracle import mlra_oracle as orc
from paper_2603_02188_amd import binding as mlra
from paper_2603_02188_amd import inputs as gen

from gpu_util import device_cache, host, max_rel_err, oracle_views, to_device

pytestmark = pytest.mark.gpu

TOL = {"bf16": 1e-2, "f32": 1e-5}


def _queries(wl, q_len, seed):
    rng = np.random.default_rng([wl.seed, 0x4D7, seed])
    q_nope = gen.to_storage(rng.standard_normal((wl.batch, q_len, wl.h, wl.d_h), dtype=np.float32), wl.dtype)
    q_rope = gen.to_storage(rng.standard_normal((wl.batch, q_len, wl.h, wl.d_r), dtype=np.float32), wl.dtype)
    return q_nope, q_rope


def _check(wl, q_len, lens, seqs=None, out_dtype=torch.float32):
    print(f"[case] multi-token {wl.name} B={wl.batch} q_len={q_len} NB={wl.n_blocks} h={wl.h} {wl.dtype}", flush=True)
    sys.stdout.flush()
    inp = gen.make_decode_inputs(wl, poison=True, seq_lens=lens)
    q_nope, q_rope = _queries(wl, q_len, q_len)
    tag = wl.dtype
    cache = device_cache(inp)
    w_uk, w_uv = to_device(inp.w_uk, tag), to_device(inp.w_uv, tag)
    qn_dev = to_device(q_nope, tag)
    q_abs = mlra.mlra_absorb_q(qn_dev.view(wl.batch * q_len, wl.h, wl.d_h), w_uk)
    q_abs = q_abs.view(wl.batch, q_len, wl.n_blocks, wl.h, wl.d_cb)
    lse = torch.full((wl.batch, q_len, wl.n_blocks, wl.h), float("nan"), device="cuda")
    out = mlra.mlra_decode_attn_multi(cache, q_abs, to_device(q_rope, tag), w_uv, wl.tau, out_dtype=out_dtype, lse=lse)
    torch.cuda.synchronize()
    out = host(out)
    v = oracle_views(inp)
    seqs = list(range(wl.batch)) if seqs is None else seqs
    ref = orc.mlra_decode_multi_batch(v["latent_pool"], v["rope_pool"], v["page_table"], v["seq_lens"],
                                      gen.to_f64(q_nope, tag), gen.to_f64(q_rope, tag), v["w_uk"], v["w_uv"], wl.tau,
                                      seqs=seqs)
    err = max_rel_err(out[seqs], ref)
    print(f"       max rel err {err:.3e} (tol {TOL[tag]:g})", flush=True)
    assert err <= TOL[tag]
    # queries without a prefix: zero rows and lse = -inf
    lse = host(lse)
    for s in seqs:
        for j in range(q_len):
            if int(lens[s]) - (q_len - 1 - j) <= 0:
                assert np.all(out[s, j] == 0.0) and np.all(np.isneginf(lse[s, j]))


def test_multi_token_fp32_tiny_with_short_and_empty_sequences():
    wl = gen.WORKLOADS["C1"].scaled(name="mt-tiny", batch=6)
    _check(wl, 3, np.array([0, 1, 2, 3, 100, 256], dtype=np.int32))


@pytest.mark.parametrize("q_len", [2, 4])
def test_multi_token_bf16_fast_path(q_len):
    wl = gen.WORKLOADS["C5"].scaled(name="mt-bf16", batch=5, n_min=1, n_max=2000)
    _check(wl, q_len, np.array([2000, 64, 65, 3, 700], dtype=np.int32))
    _check(wl, q_len, np.array([2000, 64, 65, 3, 700], dtype=np.int32), out_dtype=torch.bfloat16)


def test_multi_token_dispatch_order_full_run_and_tail():
    """11 ragged sequences x 3 queries: the dispatch order that brings a sequence's queries together has one
    full run of 8 sequences and a tail of 3 (two different slot formulas), with ties and an empty sequence."""
    wl = gen.WORKLOADS["C5"].scaled(name="mt-order", batch=11, n_min=0, n_max=1500)
    _check(wl, 3, np.array([700, 1500, 0, 64, 700, 2, 1280, 65, 700, 1, 333], dtype=np.int32))


def test_multi_token_q_len_one_is_the_plain_decode():
    wl = gen.WORKLOADS["C3"].scaled(name="mt-one", batch=3, n_min=100, n_max=900)
    _check(wl, 1, np.array([900, 100, 513], dtype=np.int32))


def test_multi_token_full_size_every_sequence():
    wl = gen.WORKLOADS["C3"]
    _check(wl, 4, gen.draw_seq_lens(wl), out_dtype=torch.bfloat16)
