"""GPU parity of the MLRA-2 entry points (Eq. (6)) against the fp64 oracle, through the C ABI.
Bars as for MLRA-4: max|gpu - ref| / max|ref| <= 1e-2 (bf16) and <= 1e-5 (fp32)."""
import sys

import numpy as np
import pytest
import torch

from oracle import mlra_oracle as orc
from paper_2603_02188_amd import binding as mlra
from paper_2603_02188_amd import inputs as gen

from gpu_util import device_cache, device_queries_weights, host, max_rel_err, oracle_views, to_device

pytestmark = pytest.mark.gpu

TOL = {"bf16": 1e-2, "f32": 1e-5}


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def _run(inp, out_dtype=torch.float32, out_scale=1.0, append=False):
    wl = inp.wl
    cache = device_cache(inp)
    q_nope, q_rope, w_uk, w_uv = device_queries_weights(inp)
    if append:
        mlra.mlra_append_kv(cache, to_device(inp.c_kv_new), to_device(inp.k_rope_new), to_device(inp.positions))
    q_abs = mlra.mlra2_absorb_q(q_nope, w_uk)
    lse = torch.full((wl.batch, wl.n_blocks, wl.h // 2), float("nan"), device="cuda")
    out = mlra.mlra2_decode_attn(cache, q_abs, q_rope, w_uv, wl.tau, out_scale, out_dtype=out_dtype, lse=lse)
    torch.cuda.synchronize()
    return host(out), host(lse), host(q_abs)


def _check(inp, out_dtype=torch.float32, out_scale=1.0, append=False, seqs=None):
    wl = inp.wl
    _say(f"[case] {wl.name} MLRA-2 B={wl.batch} n=[{wl.n_min},{wl.n_max}] d_cb={wl.d_cb} d_r={wl.d_r} h={wl.h} "
         f"d_h={wl.d_h} {wl.dtype} out={out_dtype} append={append}")
    out, lse, q_abs = _run(inp, out_dtype, out_scale, append)
    ref_inp = gen.make_decode_inputs(wl, poison=True, hole=False, seq_lens=inp.seq_lens) if append else inp
    v = oracle_views(ref_inp)
    seqs = list(range(wl.batch)) if seqs is None else seqs
    ref, ref_lse = orc.mlra2_decode_batch(v["latent_pool"], v["rope_pool"], v["page_table"], v["seq_lens"],
                                          v["q_nope"], v["q_rope"], v["w_uk"], v["w_uv"], wl.tau, out_scale,
                                          seqs=seqs, return_lse=True)
    err = max_rel_err(out[seqs], ref)
    _say(f"       max rel err {err:.3e} (tol {TOL[wl.dtype]:g})")
    assert err <= TOL[wl.dtype]
    live = np.isfinite(ref_lse)
    assert np.array_equal(np.isfinite(lse[seqs]), live)
    if live.any():
        assert np.max(np.abs(lse[seqs][live] - ref_lse[live])) <= (2e-2 if wl.dtype == "bf16" else 1e-4)
    # Step 1 alone (absorbed queries of every block)
    W_UK_g = v["w_uk"].reshape(2, 2 * wl.d_cb, (wl.h // 2) * wl.d_h)
    for s in seqs[:2]:
        qa_ref = orc.mlra2_absorb_q(v["q_nope"][s], W_UK_g)
        assert max_rel_err(q_abs[s], qa_ref) <= (8e-3 if wl.dtype == "bf16" else 1e-5)


def test_mlra2_tiny_fp32_with_append_ragged_and_empty():
    wl = gen.WORKLOADS["C1"].scaled(name="C1-as-mlra2", batch=7, groups=2)
    lens = np.array([0, 1, 63, 64, 65, 200, 256], dtype=np.int32)
    _check(gen.make_decode_inputs(wl, poison=True, hole=True, seq_lens=lens), append=True)


def test_mlra2_fp32_odd_dims_out_scale():
    # the paper's output rescale for MLRA-2 is 1/sqrt(2) (Eq. (10)); 6 heads, dims off the fast path
    wl = gen.WORKLOADS["C1"].scaled(name="mlra2-odd", batch=3, h=6, d_h=24, d_cb=40, d_r=8, n_min=90, n_max=333,
                                    groups=2)
    _check(gen.make_decode_inputs(wl, poison=True), out_scale=2 ** -0.5)


@pytest.mark.parametrize("h", [128, 256])
def test_mlra2_bf16_fast_path_shapes(h):
    # h = 128: 64 heads per block (half of a workgroup's head range is idle); h = 256: 128 per block
    wl = gen.WORKLOADS["M2"].scaled(batch=5, h=h, n_min=100, n_max=1500, shuffle_pages=True, spare_frac=0.1)
    lens = np.array([1500, 64, 1, 777, 0], dtype=np.int32)
    _check(gen.make_decode_inputs(wl, poison=True, hole=True, seq_lens=lens), append=True)
    _check(gen.make_decode_inputs(wl, poison=True, seq_lens=lens), out_dtype=torch.bfloat16)


def test_mlra2_bf16_split_context():
    wl = gen.WORKLOADS["M2"].scaled(batch=2, n_min=5000, n_max=9000)
    _check(gen.make_decode_inputs(wl, poison=True))


def test_mlra2_length_proportional_chunks_on_a_ragged_long_batch():
    # two blocks per workgroup and chunk lengths that follow the sequence lengths (chunks of 128 tiles or more)
    lens = np.array([131072, 40000, 300, 0, 5000, 64, 9000, 70000], dtype=np.int32)
    wl = gen.WORKLOADS["M2"].scaled(batch=len(lens), n_min=0, n_max=int(lens.max()))
    _check(gen.make_decode_inputs(wl, poison=True, seq_lens=lens))


def test_mlra2_two_blocks_is_gla2_shape():
    # n_blocks = 2: one block per group (GLA-2, Eq. (3)); d_cb = 2 d_h runs on the generic kernels
    wl = gen.WORKLOADS["C1"].scaled(name="gla2-shape", batch=2, n_blocks=2, d_cb=64, d_h=32, h=8, d_r=16,
                                    n_min=50, n_max=300, groups=2, dtype="bf16")
    inp = gen.make_decode_inputs(wl, poison=True)
    out, lse, _ = _run(inp)
    v = oracle_views(inp)
    ref = orc.gla2_decode_batch(v["latent_pool"], v["rope_pool"], v["page_table"], v["seq_lens"], v["q_nope"],
                                v["q_rope"], v["w_uk"], v["w_uv"], wl.tau)
    assert max_rel_err(out, ref) <= 1e-2


def _check_gla2(wl, lens, seqs=None, append=False, out_dtype=torch.float32):
    print(f"[case] GLA-2 {wl.name} B={wl.batch} h={wl.h} d_cb={wl.d_cb} append={append} out={out_dtype}", flush=True)
    inp = gen.make_decode_inputs(wl, poison=True, hole=append, seq_lens=lens)
    out, lse, _ = _run(inp, out_dtype=out_dtype, append=append)
    ref_inp = gen.make_decode_inputs(wl, poison=True, hole=False, seq_lens=lens) if append else inp
    v = oracle_views(ref_inp)
    seqs = list(range(wl.batch)) if seqs is None else seqs
    ref = orc.gla2_decode_batch(v["latent_pool"], v["rope_pool"], v["page_table"], v["seq_lens"], v["q_nope"],
                                v["q_rope"], v["w_uk"], v["w_uv"], wl.tau, seqs=seqs)
    err = max_rel_err(out[seqs], ref)
    print(f"       max rel err {err:.3e}", flush=True)
    assert err <= 1e-2
    for s in seqs:
        assert np.all(np.isfinite(lse[s])) == (int(lens[s]) > 0)


@pytest.mark.parametrize("h", [128, 256, 48])
def test_gla2_bf16_fast_path_ragged(h):
    # 256-channel latent heads on the MFMA kernel: 64 heads per group (one workgroup), 128 (two), 24 (partial)
    wl = gen.WORKLOADS["G2"].scaled(batch=6, h=h, n_min=0, n_max=1500, shuffle_pages=True, spare_frac=0.1)
    lens = np.array([1500, 64, 1, 777, 0, 65], dtype=np.int32)
    _check_gla2(wl, lens, append=True)
    _check_gla2(wl, lens, out_dtype=torch.bfloat16)


@pytest.mark.parametrize("page_size", [16, 32])
def test_two_group_forms_with_pages_shorter_than_a_tile(page_size):
    # PAIRED (MLRA-2) and GLA forms of the decode kernel on pages of 16 / 32 tokens
    lens = np.array([1500, 65, 1, 81, 0, 17], dtype=np.int32)
    wl = gen.WORKLOADS["M2"].scaled(batch=6, n_min=0, n_max=1500, page_size=page_size, shuffle_pages=True,
                                    spare_frac=0.2)
    _check(gen.make_decode_inputs(wl, poison=True, hole=True, seq_lens=lens), append=True)
    wl = gen.WORKLOADS["G2"].scaled(batch=6, n_min=0, n_max=1500, page_size=page_size, shuffle_pages=True,
                                    spare_frac=0.2)
    _check_gla2(wl, lens, append=True)


@pytest.mark.parametrize("uniform", [False, True])
def test_two_group_forms_one_round_batches_are_cut_by_length(uniform):
    # about one round of workgroups (140 sequences x 2 block pairs): a ragged batch is cut into chunks that
    # follow the lengths and handed out longest first; a batch of nearly equal lengths is left uncut
    rng = np.random.default_rng(77)
    lens = (np.full(140, 2100) - rng.integers(0, 200, size=140) if uniform
            else rng.integers(1, 3001, size=140)).astype(np.int32)
    if not uniform:
        lens[[3, 50]] = [0, 3000]
    wl = gen.WORKLOADS["M2"].scaled(batch=140, n_min=0, n_max=3000, shuffle_pages=True, spare_frac=0.1)
    _check(gen.make_decode_inputs(wl, poison=True, seq_lens=lens))
    wl = gen.WORKLOADS["G2"].scaled(batch=140, n_min=0, n_max=3000, shuffle_pages=True, spare_frac=0.1)
    _check_gla2(wl, lens)


def test_two_group_forms_many_short_sequences_single_chunk():
    # several rounds of workgroups, one chunk per sequence: the decode kernel hands normalised bf16 rows
    # straight to the up-projection (PAIRED and GLA forms), sequences taken longest first
    rng = np.random.default_rng(79)
    lens = rng.integers(0, 201, size=520).astype(np.int32)
    lens[[0, 7]] = [200, 0]
    wl = gen.WORKLOADS["M2"].scaled(batch=520, n_min=0, n_max=200, shuffle_pages=True, spare_frac=0.1)
    info = mlra.mlra_decode_plan_info(wl.batch, wl.h, wl.d_h, 2, wl.n_blocks, wl.d_cb, wl.d_r, wl.page_size, 256,
                                      torch.bfloat16)
    assert info["kernel"] == "mfma-paired" and info["chunk_slots"] == 1 and info["target_chunks"] == 0
    _check(gen.make_decode_inputs(wl, poison=True, seq_lens=lens))
    wl = gen.WORKLOADS["G2"].scaled(batch=520, n_min=0, n_max=200, shuffle_pages=True, spare_frac=0.1)
    _check_gla2(wl, lens)


def test_gla2_bf16_split_context_and_full_size():
    wl = gen.WORKLOADS["G2"].scaled(batch=2, n_min=5000, n_max=9000)
    _check_gla2(wl, np.array([9000, 5000], dtype=np.int32))
    wl = gen.WORKLOADS["G2"]
    _check_gla2(wl, gen.draw_seq_lens(wl), out_dtype=torch.bfloat16)


def test_mlra2_full_size_every_sequence():
    wl = gen.WORKLOADS["M2"]
    _check(gen.make_decode_inputs(wl, poison=False), out_dtype=torch.bfloat16)
