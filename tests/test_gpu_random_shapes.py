"""Seeded random shapes through the decode entry points (MLRA-4, MLRA-2, GLA-2 form) against the fp64 oracle:
head counts, block counts, page sizes (16 to 192 tokens, shuffled, with poisoned spare slots), ragged and
empty sequences, contexts long enough to be split, append on or off, both output types.  The draws are
fixed by the seed, so every run tests the same shapes.  Bar: max|gpu - ref| / max|ref| <= 1e-2 (bf16)."""
import numpy as np
import pytest
import torch

from oracle import mlra_oracle as orc
from paper_2603_02188_amd import binding as mlra
from paper_2603_02188_amd import inputs as gen

from gpu_util import device_cache, device_queries_weights, host, max_rel_err, oracle_views, to_device

pytestmark = pytest.mark.gpu


def _draw_lens(rng, batch, nmax):
    """A mix of special lengths (empty, around page and tile edges), tile multiples +-1 and uniform draws."""
    lens = []
    for _ in range(batch):
        k = rng.integers(0, 6)
        if k == 0:
            n = int(rng.choice([0, 1, 2, 15, 16, 17, 63, 64, 65, 127, 128, 129]))
        elif k == 1:
            n = int(64 * rng.integers(1, max(2, nmax // 64)) + rng.integers(-1, 2))
        else:
            n = int(rng.integers(1, nmax + 1))
        lens.append(max(0, min(n, nmax)))
    return np.array(lens, dtype=np.int32)


def _one(seed):
    rng = np.random.default_rng(seed)
    form = rng.choice(["mlra4", "mlra4", "mlra2", "gla2"])
    ps = int(rng.choice([16, 32, 64, 128, 192]))
    batch = int(rng.integers(1, 10))
    nmax = int(rng.choice([300, 1500, 6000, 30000])) if batch <= 4 else int(rng.choice([300, 1500, 4000]))
    lens = _draw_lens(rng, batch, nmax)
    append = bool(rng.integers(0, 2))
    out_dtype = torch.float32 if rng.integers(0, 2) else torch.bfloat16
    out_scale = float(rng.choice([1.0, 0.5, 0.7071067811865476]))
    if form == "mlra4":
        nb = int(rng.choice([1, 2, 3, 4]))
        h = int(rng.choice([16, 64, 100, 128, 192, 256]))
        wl = gen.WORKLOADS["C3"].scaled(name=f"random-{seed}", batch=batch, n_min=0, n_max=nmax, n_blocks=nb, h=h,
                                        page_size=ps, shuffle_pages=True, spare_frac=0.2, index=1000 + seed)
    elif form == "mlra2":
        h = int(rng.choice([64, 128, 256]))
        wl = gen.WORKLOADS["M2"].scaled(name=f"random-{seed}", batch=batch, n_min=0, n_max=nmax, h=h, page_size=ps,
                                        shuffle_pages=True, spare_frac=0.2, index=1000 + seed)
    else:
        h = int(rng.choice([48, 128, 256]))
        wl = gen.WORKLOADS["G2"].scaled(name=f"random-{seed}", batch=batch, n_min=0, n_max=nmax, h=h, page_size=ps,
                                        shuffle_pages=True, spare_frac=0.2, index=1000 + seed)
    print(f"[case] random shape {seed}: {form} B={batch} h={wl.h} NB={wl.n_blocks} d_cb={wl.d_cb} page={ps} "
          f"lens={lens.tolist()} append={append} out={out_dtype} scale={out_scale}", flush=True)
    inp = gen.make_decode_inputs(wl, poison=True, hole=append, seq_lens=lens)
    cache = device_cache(inp)
    q_nope, q_rope, w_uk, w_uv = device_queries_weights(inp)
    if append:
        mlra.mlra_append_kv(cache, to_device(inp.c_kv_new), to_device(inp.k_rope_new), to_device(inp.positions))
    if form == "mlra4":
        q_abs = mlra.mlra_absorb_q(q_nope, w_uk)
        out = mlra.mlra_decode_attn(cache, q_abs, q_rope, w_uv, wl.tau, out_scale, out_dtype=out_dtype)
    else:
        q_abs = mlra.mlra2_absorb_q(q_nope, w_uk)
        out = mlra.mlra2_decode_attn(cache, q_abs, q_rope, w_uv, wl.tau, out_scale, out_dtype=out_dtype)
    torch.cuda.synchronize()
    got = host(out)
    ref_inp = gen.make_decode_inputs(wl, poison=True, hole=False, seq_lens=lens) if append else inp
    v = oracle_views(ref_inp)
    args = (v["latent_pool"], v["rope_pool"], v["page_table"], v["seq_lens"], v["q_nope"], v["q_rope"], v["w_uk"],
            v["w_uv"], wl.tau)
    if form == "mlra4":
        ref = orc.mlra_decode_batch(*args, out_scale)
    elif form == "mlra2":
        ref = orc.mlra2_decode_batch(*args, out_scale)
    else:
        ref = orc.gla2_decode_batch(*args) * out_scale
    err = max_rel_err(got, ref)
    print(f"           max rel err {err:.3e}", flush=True)
    return err


@pytest.mark.parametrize("first", [0, 16, 32, 48])
def test_random_shapes_match_the_oracle(first):
    for seed in range(first, first + 16):
        assert _one(seed) <= 1e-2, f"seed {seed}"


def test_eight_blocks_sixteen_chunks_epilogue_tables_exceed_lds():
    """8 blocks x 128 channels with 16 chunks per sequence: the MFMA epilogue's tables (1024 latent channels
    of z rows plus 128 merge weights per sequence) would need more than the 160 KiB of LDS, so the call has
    to take the generic merge + up-projection (and must not fail at launch)."""
    wl = gen.WORKLOADS["C3"].scaled(name="eight-blocks", batch=2, n_min=1500, n_max=2048, n_blocks=8, index=2001)
    lens = np.array([2048, 1501], dtype=np.int32)
    info = mlra.mlra_decode_plan_info(wl.batch, wl.h, wl.d_h, 1, wl.n_blocks, wl.d_cb, wl.d_r, wl.page_size, 2048,
                                      torch.bfloat16)
    assert info["kernel"] == "mfma" and info["chunk_slots"] == 16 and not info["merge_mfma"]
    inp = gen.make_decode_inputs(wl, poison=True, seq_lens=lens)
    assert inp.page_table.shape[1] * wl.page_size == 2048
    cache = device_cache(inp)
    q_nope, q_rope, w_uk, w_uv = device_queries_weights(inp)
    q_abs = mlra.mlra_absorb_q(q_nope, w_uk)
    out = mlra.mlra_decode_attn(cache, q_abs, q_rope, w_uv, wl.tau, 1.0, out_dtype=torch.float32)
    torch.cuda.synchronize()
    v = oracle_views(inp)
    ref = orc.mlra_decode_batch(v["latent_pool"], v["rope_pool"], v["page_table"], v["seq_lens"], v["q_nope"],
                                v["q_rope"], v["w_uk"], v["w_uv"], wl.tau, 1.0)
    err = max_rel_err(host(out), ref)
    print(f"[case] eight blocks, sixteen chunks: max rel err {err:.3e}", flush=True)
    assert err <= 1e-2
