"""Helpers for the GPU parity tests: host arrays -> device tensors, oracle views, error metric."""
from __future__ import annotations

import numpy as np
import torch

from paper_2603_02188_amd import binding as mlra
from paper_2603_02188_amd import inputs as gen


def to_device(arr: np.ndarray, dtype_tag: str | None = None) -> torch.Tensor:
    """numpy -> cuda tensor; uint16 arrays tagged 'bf16' are reinterpreted as bfloat16."""
    t = torch.from_numpy(np.ascontiguousarray(arr))
    if dtype_tag == "bf16":
        assert arr.dtype == np.uint16
        t = t.view(torch.bfloat16)
    return t.to("cuda")


def device_cache(inp: gen.DecodeInputs) -> mlra.Cache:
    tag = inp.wl.dtype
    return mlra.Cache(to_device(inp.latent_pool, tag), to_device(inp.rope_pool, tag),
                      to_device(inp.page_table), to_device(inp.seq_lens))


def device_queries_weights(inp: gen.DecodeInputs):
    tag = inp.wl.dtype
    return (to_device(inp.q_nope, tag), to_device(inp.q_rope, tag), to_device(inp.w_uk, tag),
            to_device(inp.w_uv, tag))


def oracle_views(inp: gen.DecodeInputs):
    """float64 arrays holding exactly the stored values, in the oracle's argument order."""
    tag = inp.wl.dtype
    return dict(latent_pool=gen.to_f64(inp.latent_pool, tag), rope_pool=gen.to_f64(inp.rope_pool, tag),
                page_table=inp.page_table, seq_lens=inp.seq_lens, q_nope=gen.to_f64(inp.q_nope, tag),
                q_rope=gen.to_f64(inp.q_rope, tag), w_uk=gen.to_f64(inp.w_uk, tag), w_uv=gen.to_f64(inp.w_uv, tag))


def max_rel_err(got, ref) -> float:
    """max |got - ref| / max |ref| over the whole tensor (elementwise relative error is
    meaningless where the reference passes through zero)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    if not np.isfinite(got).all():
        return float("inf")
    denom = float(np.max(np.abs(ref)))
    if denom == 0.0:
        return float(np.max(np.abs(got)))
    return float(np.max(np.abs(got - ref)) / denom)


def host(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float64).cpu().numpy()


def run_mlra_path(inp: gen.DecodeInputs, out_dtype=torch.float32, out_scale=1.0, with_lse=True,
                  append=False):
    """append (optional) -> absorb -> decode through the C ABI; returns (out, lse, q_abs) on host."""
    wl = inp.wl
    cache = device_cache(inp)
    q_nope, q_rope, w_uk, w_uv = device_queries_weights(inp)
    if append:
        mlra.mlra_append_kv(cache, to_device(inp.c_kv_new), to_device(inp.k_rope_new), to_device(inp.positions))
    q_abs = mlra.mlra_absorb_q(q_nope, w_uk)
    lse = torch.full((wl.batch, wl.n_blocks, wl.h), float("nan"), device="cuda") if with_lse else None
    out = mlra.mlra_decode_attn(cache, q_abs, q_rope, w_uv, wl.tau, out_scale, out_dtype=out_dtype, lse=lse)
    torch.cuda.synchronize()
    return host(out), (host(lse) if with_lse else None), host(q_abs)
