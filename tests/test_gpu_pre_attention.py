"""GPU parity of mlra_pre_attention (projections of the appendix "Attention Mechanism", subsection
Multi-Head Latent Attention; RMSNorm, Eq. (9) scaling, RoPE, cache append) against the fp64 oracle.
Bars: max|gpu - ref| / max|ref| <= 1e-2 for bf16, <= 1e-5 for fp32, taken against the exact oracle (no
intermediate rounding on the oracle's side: the kernel's rounding of C^Q to the storage type is part of
what the budget covers).  As a diagnostic, the same outputs must also lie within half of the budget of
the oracle evaluated with C^Q rounded where the kernel rounds it."""
import sys

import numpy as np
import pytest
import torch

from oracle import mlra_oracle as orc
from paper_2603_02188_amd import binding as mlra
from paper_2603_02188_amd import inputs as gen

from gpu_util import device_cache, host, max_rel_err, to_device

pytestmark = pytest.mark.gpu

TOL = {"bf16": 1e-2, "f32": 1e-5}


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def _run_and_check(wl, d, d_cq, lens, unit_gains=False):
    _say(f"[case] pre-attention {wl.name} B={wl.batch} d={d} d_cq={d_cq} NB={wl.n_blocks} d_cb={wl.d_cb} "
         f"d_r={wl.d_r} h={wl.h} d_h={wl.d_h} {wl.dtype}")
    inp = gen.make_decode_inputs(wl, poison=True, hole=True, seq_lens=lens)
    pre = gen.make_pre_inputs(wl, d, d_cq, unit_gains=unit_gains)
    tag = wl.dtype
    cache = device_cache(inp)
    lat_before, rope_before = cache.latent.clone(), cache.rope.clone()
    W = mlra.PreWeights(to_device(pre.w_dq, tag), to_device(pre.w_dkv, tag), to_device(pre.w_kr, tag),
                        to_device(pre.w_uq, tag), to_device(pre.w_qr, tag), wl.h, pre.alpha_q, pre.alpha_kv,
                        None if unit_gains else to_device(pre.gain_q, tag),
                        None if unit_gains else to_device(pre.gain_kv, tag), pre.eps, pre.rope_base)
    q_nope, q_rope = mlra.mlra_pre_attention(cache, W, to_device(pre.hidden, tag), to_device(inp.positions))
    torch.cuda.synchronize()
    q_nope, q_rope = host(q_nope), host(q_rope)
    lat, rope = host(cache.latent), host(cache.rope)
    f = lambda a: gen.to_f64(a, tag)
    round_cq = orc.round_bf16 if tag == "bf16" else (lambda v: np.asarray(v, np.float32).astype(np.float64))
    ps = wl.page_size
    worst = worst_rounded = 0.0
    untouched_lat = np.ones(lat.shape, bool)
    untouched_rope = np.ones(rope.shape, bool)
    for s in range(wl.batch):
        pos = int(inp.positions[s])
        args = (f(pre.hidden)[s], max(pos, 0), f(pre.w_dq), f(pre.w_dkv), f(pre.w_kr), f(pre.w_uq), f(pre.w_qr),
                wl.h, pre.alpha_q, pre.alpha_kv, f(pre.gain_q), f(pre.gain_kv), pre.eps, pre.rope_base)
        c_kv, k_rope, qn, qr = orc.pre_attention(*args)                  # the exact definition
        worst = max(worst, max_rel_err(q_nope[s], qn), max_rel_err(q_rope[s], qr))
        _, _, qn_r, qr_r = orc.pre_attention(*args, round_cq=round_cq)   # diagnostic only
        worst_rounded = max(worst_rounded, max_rel_err(q_nope[s], qn_r), max_rel_err(q_rope[s], qr_r))
        if pos < 0:
            continue
        page, slot = int(inp.page_table[s, pos // ps]), pos % ps
        got_row = lat[page, :, slot, :].reshape(-1)
        worst = max(worst, max_rel_err(got_row, c_kv), max_rel_err(rope[page, slot], k_rope))
        untouched_lat[page, :, slot, :] = False
        untouched_rope[page, slot, :] = False
    _say(f"       max rel err {worst:.3e} (tol {TOL[tag]:g}); against the oracle with C^Q rounded to the "
         f"storage type {worst_rounded:.3e}")
    assert worst <= TOL[tag]
    assert worst_rounded <= 0.5 * TOL[tag]
    # nothing but the new rows was written (bitwise; NaN poison compares through the raw bits)
    raw = lambda t: t.view(torch.int16) if t.dtype == torch.bfloat16 else t.view(torch.int32)
    assert torch.equal(raw(cache.latent)[torch.from_numpy(untouched_lat).cuda()],
                       raw(lat_before)[torch.from_numpy(untouched_lat).cuda()])
    assert torch.equal(raw(cache.rope)[torch.from_numpy(untouched_rope).cuda()],
                       raw(rope_before)[torch.from_numpy(untouched_rope).cuda()])


def test_pre_attention_tiny_fp32_generic_path():
    wl = gen.WORKLOADS["C1"].scaled(name="pre-tiny", batch=5)
    _run_and_check(wl, d=96, d_cq=40, lens=np.array([0, 1, 64, 65, 256], dtype=np.int32))


def test_pre_attention_fp32_odd_dims():
    wl = gen.WORKLOADS["C1"].scaled(name="pre-odd", batch=3, h=6, d_h=24, d_cb=40, d_r=8, n_blocks=2, n_min=1, n_max=300)
    _run_and_check(wl, d=50, d_cq=28, lens=np.array([300, 17, 129], dtype=np.int32))


@pytest.mark.parametrize("batch", [1, 37, 64, 96, 130])
def test_pre_attention_bf16_mfma_path(batch):
    # K slices, a narrow last segment (d_r = 64 < one column tile) and a ragged one (17 heads x 64 RoPE
    # channels), ragged batch tiles (1..4 accumulator tiles, two batch tiles at 130), far positions
    wl = gen.WORKLOADS["C3"].scaled(name="pre-bf16", batch=batch, h=17, n_min=1, n_max=4000)
    rng = np.random.default_rng(5 + batch)
    lens = rng.integers(1, 4001, size=batch).astype(np.int32)
    lens[0] = 4000
    _run_and_check(wl, d=1024, d_cq=384, lens=lens)


def test_pre_attention_bf16_row_counts_off_the_chunk():
    # projection depths that are not multiples of the MFMA kernel's 128-row chunks: the plain kernel runs
    wl = gen.WORKLOADS["C3"].scaled(name="pre-bf16-odd", batch=9, h=16, n_min=1, n_max=4000)
    lens = np.array([4000, 1, 2, 63, 64, 65, 1000, 3999, 77], dtype=np.int32)
    _run_and_check(wl, d=1024 + 16, d_cq=384 + 8, lens=lens)


@pytest.mark.parametrize("batch", [3, 100, 130])
def test_pre_attention_bf16_single_slice_up_projection(batch):
    # enough column tiles that the up-projection keeps K in one slice: its GEMM writes q_nope and the rotated
    # q_rope itself (1, 4 and 4 + 1 accumulator tiles; 121 heads leave a ragged last column tile)
    wl = gen.WORKLOADS["C3"].scaled(name="pre-fused", batch=batch, h=121, n_min=1, n_max=3000)
    rng = np.random.default_rng(11 + batch)
    lens = rng.integers(1, 3001, size=batch).astype(np.int32)
    _run_and_check(wl, d=256, d_cq=256, lens=lens)


def test_pre_attention_bf16_paper_shape_unit_gains():
    # hidden size 7168 and 128 heads as in the paper's decode benchmark (Section 4.5); d_c' = 1536
    wl = gen.WORKLOADS["C3"].scaled(name="pre-paper-shape", batch=8, n_min=1, n_max=131072)
    lens = np.array([131072, 1, 70000, 8192, 4097, 64, 65, 100000], dtype=np.int32)
    _run_and_check(wl, d=7168, d_cq=1536, lens=lens, unit_gains=True)
