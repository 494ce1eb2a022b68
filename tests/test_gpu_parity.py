"""GPU parity: the HIP path (through the C ABI) against the fp64 CPU oracle on the same seeded
inputs.  Bars: max|gpu - ref| / max|ref| <= 1e-2 for bf16 caches and <= 1e-5 for fp32; cache
appends are bit-exact."""
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

TOL = {"bf16": 1e-2, "f32": 1e-5}


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def _oracle_out(inp, out_scale=1.0, seqs=None):
    v = oracle_views(inp)
    return orc.mlra_decode_batch(v["latent_pool"], v["rope_pool"], v["page_table"], v["seq_lens"], v["q_nope"],
                                 v["q_rope"], v["w_uk"], v["w_uv"], inp.wl.tau, out_scale, seqs=seqs,
                                 return_lse=True)


def _check_mlra(inp, out_dtype=torch.float32, out_scale=1.0, append=False, tol=None):
    wl = inp.wl
    _say(f"[case] {wl.name} B={wl.batch} n=[{wl.n_min},{wl.n_max}] NB={wl.n_blocks} d_cb={wl.d_cb} d_r={wl.d_r} "
         f"h={wl.h} d_h={wl.d_h} {wl.dtype} page={wl.page_size} out={out_dtype} append={append}")
    out, lse, _ = run_mlra_path(inp, out_dtype=out_dtype, out_scale=out_scale, append=append)
    ref_inp = gen.make_decode_inputs(wl, poison=True, hole=False, seq_lens=inp.seq_lens) if append else inp
    ref, ref_lse = _oracle_out(ref_inp, out_scale)
    tol = TOL[wl.dtype] if tol is None else tol
    err = max_rel_err(out, ref)
    _say(f"       max rel err {err:.3e} (tol {tol:g})")
    assert err <= tol
    live = np.isfinite(ref_lse)
    assert np.array_equal(np.isfinite(lse), live)
    if live.any():
        assert np.max(np.abs(lse[live] - ref_lse[live])) <= (2e-2 if wl.dtype == "bf16" else 1e-4)
    return out


# ---- workload C1 exactly: tiny MLRA-4, fp32 ------------------------------------------------------
def test_c1_tiny_fp32_full_path():
    inp = gen.make_decode_inputs(gen.WORKLOADS["C1"], poison=True, hole=True)
    _check_mlra(inp, append=True)


def test_c1_fp32_ragged_and_empty_sequences():
    wl = gen.WORKLOADS["C1"].scaled(batch=9)
    lens = np.array([0, 1, 2, 63, 64, 65, 127, 200, 256], dtype=np.int32)
    inp = gen.make_decode_inputs(wl, seq_lens=lens)
    out = _check_mlra(inp)
    assert np.all(out[0] == 0.0)            # empty context: zero row


def test_c1_fp32_many_splits_long_ragged():
    wl = gen.WORKLOADS["C1"].scaled(batch=2, n_min=1500, n_max=3000, shuffle_pages=True, spare_frac=0.2)
    _check_mlra(gen.make_decode_inputs(wl))


def test_fp32_odd_dims_and_pages():
    """Dims that are not multiples of the tile sizes; page size 16 and 48."""
    for ps in (16, 48):
        wl = gen.WORKLOADS["C1"].scaled(batch=3, n_min=5, n_max=333, h=5, d_h=24, d_cb=40, d_r=12, n_blocks=3,
                                        page_size=ps, shuffle_pages=True, spare_frac=0.3)
        _check_mlra(gen.make_decode_inputs(wl))


# ---- bf16, the shapes of C2 / C3 / C5 at sizes the oracle does in seconds -------------------------
def test_bf16_tp_share_shape_ragged():
    wl = gen.WORKLOADS["C2"].scaled(batch=3, n_min=700, n_max=2500)
    _check_mlra(gen.make_decode_inputs(wl), append=False)


def test_bf16_mlra4_shape_ragged_with_append():
    wl = gen.WORKLOADS["C3"].scaled(batch=4, n_min=1, n_max=1800)
    lens = np.array([1, 64, 1337, 1800], dtype=np.int32)
    inp = gen.make_decode_inputs(wl, hole=True, seq_lens=lens)
    _check_mlra(inp, append=True)


def test_bf16_paged_mixed_shape():
    wl = gen.WORKLOADS["C5"].scaled(batch=6, n_min=100, n_max=1500)
    _check_mlra(gen.make_decode_inputs(wl))


def test_bf16_out_and_out_scale():
    wl = gen.WORKLOADS["C3"].scaled(batch=2, n_min=300, n_max=900)
    inp = gen.make_decode_inputs(wl)
    o32 = _check_mlra(inp, out_dtype=torch.float32, out_scale=0.5)     # Eq. (10): alpha_attn = 1/2
    o16 = _check_mlra(inp, out_dtype=torch.bfloat16, out_scale=0.5)
    # the bf16 output is the fp32 output rounded once
    assert np.array_equal(o16, orc.round_bf16(o32.astype(np.float32)))


def test_bf16_large_page_size():
    wl = gen.WORKLOADS["C3"].scaled(batch=2, n_min=500, n_max=1300, page_size=256, shuffle_pages=True,
                                    spare_frac=0.5)
    _check_mlra(gen.make_decode_inputs(wl))


@pytest.mark.parametrize("page_size", [16, 32])
def test_bf16_pages_shorter_than_a_tile(page_size):
    """Pages of 16 and 32 tokens: the four waves of a 64-token tile read different pages, and at a ragged
    end the waves past it re-read the last valid row from a page that is not theirs (unmapped table
    entries and spare page slots hold poison)."""
    wl = gen.WORKLOADS["C3"].scaled(batch=9, n_min=1, n_max=2100, page_size=page_size, shuffle_pages=True,
                                    spare_frac=0.3)
    lens = np.array([1, 16, 17, 65, 81, 100, 1337, 2047, 2100], dtype=np.int32)
    _check_mlra(gen.make_decode_inputs(wl, hole=True, seq_lens=lens), append=True)
    # one block, few sequences: the context is split into chunks
    wl = gen.WORKLOADS["C2"].scaled(batch=2, n_min=3000, n_max=5000, page_size=page_size, shuffle_pages=True,
                                    spare_frac=0.2)
    _check_mlra(gen.make_decode_inputs(wl, seq_lens=np.array([4993, 3001], dtype=np.int32)))


def test_deterministic_bitwise():
    wl = gen.WORKLOADS["C5"].scaled(batch=3, n_min=900, n_max=2100)
    inp = gen.make_decode_inputs(wl)
    a, la, _ = run_mlra_path(inp)
    b, lb, _ = run_mlra_path(inp)
    assert np.array_equal(a, b) and np.array_equal(la, lb)


# ---- the steps on their own ------------------------------------------------------------------------
@pytest.mark.parametrize("key", ["C1", "C3"])
def test_append_kv_bit_exact(key):
    wl = gen.WORKLOADS[key].scaled(batch=5, n_min=1, n_max=300, shuffle_pages=True, spare_frac=0.2)
    holed = gen.make_decode_inputs(wl, hole=True)
    full = gen.make_decode_inputs(wl, hole=False)
    for src in ("f32", "bf16"):
        cache = device_cache(holed)
        c_new, k_new = to_device(gen.to_storage(holed.c_kv_new, src), src), to_device(
            gen.to_storage(holed.k_rope_new, src), src)
        pos = holed.positions.copy()
        pos[0] = -1                                              # skipped sequence keeps its hole
        mlra.mlra_append_kv(cache, c_new, k_new, to_device(pos))
        torch.cuda.synchronize()
        lat = gen.to_f64(holed.latent_pool, wl.dtype)
        rope = gen.to_f64(holed.rope_pool, wl.dtype)
        to_bf16 = wl.dtype == "bf16"
        c_src = gen.to_f64(gen.to_storage(holed.c_kv_new, src), src)
        k_src = gen.to_f64(gen.to_storage(holed.k_rope_new, src), src)
        orc.append_kv(lat, rope, holed.page_table, pos, c_src, k_src, to_bf16)
        assert np.array_equal(host(cache.latent), lat, equal_nan=True)
        assert np.array_equal(host(cache.rope), rope, equal_nan=True)
        if src == "f32":
            pos_all = holed.positions
            cache2 = device_cache(holed)
            mlra.mlra_append_kv(cache2, to_device(holed.c_kv_new), to_device(holed.k_rope_new), to_device(pos_all))
            assert np.array_equal(host(cache2.latent), gen.to_f64(full.latent_pool, wl.dtype), equal_nan=True)


@pytest.mark.parametrize("key,tol", [("C1", 1e-5), ("C3", 6e-3)])
def test_absorb_q_against_oracle(key, tol):
    wl = gen.WORKLOADS[key].scaled(batch=3)
    q_nope, q_rope, w_uk, w_uv = gen.draw_queries_weights(wl)
    got = host(mlra.mlra_absorb_q(to_device(q_nope, wl.dtype), to_device(w_uk, wl.dtype)))
    W = gen.to_f64(w_uk, wl.dtype).reshape(-1, wl.h * wl.d_h)
    ref = np.stack([orc.absorb_q(gen.to_f64(q_nope[b], wl.dtype), W, wl.n_blocks) for b in range(wl.batch)])
    assert max_rel_err(got, ref) <= tol


# ---- comparison kernels on the same harness -----------------------------------------------------------
def test_mla_baseline_bf16():
    wl = gen.WORKLOADS["C5"].scaled(batch=3, n_min=200, n_max=1100)
    inp = gen.as_single_latent(gen.make_decode_inputs(wl))
    cache = device_cache(inp)
    q_nope, q_rope, w_uk, w_uv = device_queries_weights(inp)
    q_abs = mlra.mlra_absorb_q(q_nope, w_uk)
    out = host(mlra.mla_decode_attn(cache, q_abs, q_rope, w_uv, wl.tau, out_dtype=torch.float32))
    v = oracle_views(inp)
    ref = np.stack([
        orc.mla_decode(v["q_nope"][b], v["q_rope"][b],
                       *orc.gather_sequence(v["latent_pool"], v["rope_pool"], v["page_table"][b], int(v["seq_lens"][b])),
                       v["w_uk"].reshape(-1, wl.h * wl.d_h), v["w_uv"].reshape(-1, wl.h * wl.d_h), wl.tau)
        for b in range(wl.batch)])
    err = max_rel_err(out, ref)
    _say(f"[case] MLA baseline max rel err {err:.3e}")
    assert err <= 1e-2


@pytest.mark.parametrize("dtype,tol", [("bf16", 1e-2), ("f32", 1e-5)])
def test_gqa_baseline(dtype, tol):
    wl = gen.WORKLOADS["C5"].scaled(batch=4, n_min=1, n_max=1500, dtype=dtype)
    lens = np.array([0, 1, 777, 1500], dtype=np.int32)
    gi = gen.make_gqa_inputs(wl, seq_lens=lens)
    out = host(mlra.gqa_decode_attn(to_device(gi.k_pool, dtype), to_device(gi.v_pool, dtype),
                                    to_device(gi.page_table), to_device(gi.seq_lens), to_device(gi.q, dtype),
                                    gi.scale, out_dtype=torch.float32))
    ref = orc.gqa_decode_batch(gen.to_f64(gi.k_pool, dtype), gen.to_f64(gi.v_pool, dtype), gi.page_table,
                               gi.seq_lens, gen.to_f64(gi.q, dtype), gi.scale)
    err = max_rel_err(out, ref)
    _say(f"[case] GQA baseline {dtype} max rel err {err:.3e}")
    assert err <= tol and np.all(out[0] == 0)


def _mla_reference(inp, seqs=None):
    wl = inp.wl
    v = oracle_views(inp)
    rows = []
    for b in (range(wl.batch) if seqs is None else seqs):
        n = int(v["seq_lens"][b])
        if n == 0:
            rows.append(np.zeros((wl.h, wl.d_h)))
            continue
        rows.append(orc.mla_decode(v["q_nope"][b], v["q_rope"][b],
                                   *orc.gather_sequence(v["latent_pool"], v["rope_pool"], v["page_table"][b], n),
                                   v["w_uk"].reshape(-1, wl.h * wl.d_h), v["w_uv"].reshape(-1, wl.h * wl.d_h), wl.tau))
    return np.stack(rows)


@pytest.mark.parametrize("h,lens,page_size", [
    (128, [0, 1, 31, 32, 33, 700], 64),          # empty, single token, around one 32-token tile
    (64, [95, 96, 97, 2050], 32),                # one head group; page = tile
    (96, [5000, 17], 256),                       # ragged head group; context split into chunks
])
def test_mla_baseline_edge_shapes(h, lens, page_size):
    lens = np.array(lens, dtype=np.int32)
    wl = gen.WORKLOADS["C5"].scaled(batch=len(lens), n_min=0, n_max=int(lens.max()), h=h, page_size=page_size)
    inp = gen.as_single_latent(gen.make_decode_inputs(wl, seq_lens=lens))
    cache = device_cache(inp)
    q_nope, q_rope, w_uk, w_uv = device_queries_weights(inp)
    q_abs = mlra.mlra_absorb_q(q_nope, w_uk)
    out = host(mlra.mla_decode_attn(cache, q_abs, q_rope, w_uv, wl.tau, out_dtype=torch.float32))
    ref = _mla_reference(inp)
    err = max_rel_err(out, ref)
    _say(f"[case] MLA baseline h={h} lens={lens.tolist()} page={page_size} max rel err {err:.3e}")
    assert np.isfinite(out).all() and err <= 1e-2
    for b in np.flatnonzero(lens == 0):
        assert np.all(out[b] == 0)


def test_mla_baseline_one_round_ragged_batch_is_cut_by_length():
    rng = np.random.default_rng(78)
    lens = rng.integers(1, 3001, size=140).astype(np.int32)
    lens[[3, 50]] = [0, 3000]
    wl = gen.WORKLOADS["C5"].scaled(batch=140, n_min=0, n_max=3000)
    inp = gen.as_single_latent(gen.make_decode_inputs(wl, seq_lens=lens))
    cache = device_cache(inp)
    q_nope, q_rope, w_uk, w_uv = device_queries_weights(inp)
    q_abs = mlra.mlra_absorb_q(q_nope, w_uk)
    out = host(mlra.mla_decode_attn(cache, q_abs, q_rope, w_uv, wl.tau, out_dtype=torch.float32))
    ref = _mla_reference(inp)
    err = max_rel_err(out, ref)
    _say(f"[case] MLA baseline, 140 ragged sequences: max rel err {err:.3e}")
    assert np.isfinite(out).all() and err <= 1e-2 and np.all(out[3] == 0)


@pytest.mark.parametrize("h,g,lens,page_size", [
    (128, 8, [1, 31, 32, 33, 127, 129, 900], 64),    # 16 query heads per KV head
    (128, 4, [64, 65, 2000], 32),                    # 32 per KV head; page = sub-tile
    (24, 8, [300, 1], 128),                          # 3 per KV head: mostly padding columns
])
def test_gqa_baseline_edge_shapes(h, g, lens, page_size):
    lens = np.array(lens, dtype=np.int32)
    wl = gen.WORKLOADS["C5"].scaled(batch=len(lens), n_min=1, n_max=int(lens.max()), h=h, g=g, page_size=page_size)
    gi = gen.make_gqa_inputs(wl, seq_lens=lens)
    out = host(mlra.gqa_decode_attn(to_device(gi.k_pool, "bf16"), to_device(gi.v_pool, "bf16"),
                                    to_device(gi.page_table), to_device(gi.seq_lens), to_device(gi.q, "bf16"),
                                    gi.scale, out_dtype=torch.float32))
    ref = orc.gqa_decode_batch(gen.to_f64(gi.k_pool, "bf16"), gen.to_f64(gi.v_pool, "bf16"), gi.page_table,
                               gi.seq_lens, gen.to_f64(gi.q, "bf16"), gi.scale)
    err = max_rel_err(out, ref)
    _say(f"[case] GQA baseline h={h} g={g} lens={lens.tolist()} page={page_size} max rel err {err:.3e}")
    assert np.isfinite(out).all() and err <= 1e-2


def test_longest_first_order_with_ties_and_empty_sequences():
    # more workgroups than CUs (80 sequences x 4 blocks), equal lengths and empty sequences in the batch
    lens = np.array(([0, 64, 64, 1000, 1, 513, 513, 130] * 10), dtype=np.int32)
    wl = gen.WORKLOADS["C5"].scaled(batch=len(lens), n_min=0, n_max=1000)
    inp = gen.make_decode_inputs(wl, seq_lens=lens)
    out = _check_mlra(inp)
    for b in np.flatnonzero(lens == 0):
        assert np.all(out[b] == 0)


def test_length_proportional_chunks_on_a_ragged_long_batch():
    # split mode with chunks of 128 tiles or more: chunk lengths follow the sequence lengths (one sequence
    # takes most of the chunk slots, one is shorter than a single chunk, one is empty)
    lens = np.array([131072, 40000, 300, 0], dtype=np.int32)
    wl = gen.WORKLOADS["C4"].scaled(batch=len(lens), n_min=0, n_max=int(lens.max()))
    inp = gen.make_decode_inputs(wl, seq_lens=lens)
    out = _check_mlra(inp)
    assert np.all(out[3] == 0)


@pytest.mark.parametrize("key,out_dtype", [("C1", torch.float32), ("C3", torch.float32), ("C3", torch.bfloat16)])
def test_gated_output(key, out_dtype):
    # Appendix E: the attention output times a gate G = sigmoid(...) in (0, 1), elementwise
    wl = gen.WORKLOADS[key].scaled(batch=3, n_min=40, n_max=700)
    inp = gen.make_decode_inputs(wl)
    rng = np.random.default_rng([wl.seed, 0x6A7E])
    gate = gen.to_storage((1.0 / (1.0 + np.exp(-rng.standard_normal((wl.batch, wl.h, wl.d_h))))).astype(np.float32),
                          wl.dtype)
    cache = device_cache(inp)
    q_nope, q_rope, w_uk, w_uv = device_queries_weights(inp)
    q_abs = mlra.mlra_absorb_q(q_nope, w_uk)
    out = host(mlra.mlra_decode_attn_gated(cache, q_abs, q_rope, w_uv, to_device(gate, wl.dtype), wl.tau, 0.5,
                                           out_dtype=out_dtype))
    ref, _ = _oracle_out(inp, 0.5)
    ref = orc.gated_output(ref, gen.to_f64(gate, wl.dtype))
    err = max_rel_err(out, ref)
    _say(f"[case] gated {wl.name} out={out_dtype}: max rel err {err:.3e}")
    assert err <= TOL[wl.dtype]


def test_workspace_too_small_is_refused_on_device_pointers():
    wl = gen.WORKLOADS["C1"]
    inp = gen.make_decode_inputs(wl)
    cache = device_cache(inp)
    q_nope, q_rope, w_uk, w_uv = device_queries_weights(inp)
    q_abs = mlra.mlra_absorb_q(q_nope, w_uk)
    ws = torch.empty(256, dtype=torch.uint8, device="cuda")
    with pytest.raises(RuntimeError, match="workspace"):
        mlra.mlra_decode_attn(cache, q_abs, q_rope, w_uv, wl.tau, workspace=ws)
