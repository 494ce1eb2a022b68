"""Algorithmic byte / flop models of decode attention (host arithmetic only).

* kv_loading_per_token: Table 1 of the paper ("Loading Per Token Per Device"), in elements.
* arithmetic_intensity: Table 2 of the paper (flops per byte of 16-bit cache, long context).
* decode_bytes / decode_flops: the same models written out for a concrete batch, used by the
  benchmark to turn a measured kernel time into achieved GB/s and TFLOP/s.
"""
from __future__ import annotations

from math import ceil
from typing import Sequence

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 MFMA, published


def kv_loading_per_token(method: str, n_devices: int, d_h: int = 128, h: int = 64, g: int = 8,
                         d_c: int | None = None, d_r: int | None = None) -> float:
    """Cache elements one device must load per token under n_devices-way tensor parallelism
    (Table 1; Section 3.4 "KV Cache" uses h = 64, g = 8, d_c = 4 d_h, d_h^R = d_h / 2)."""
    d_c = 4 * d_h if d_c is None else d_c
    d_r = d_h // 2 if d_r is None else d_r
    m = method.upper()
    if m == "MHA":
        return 2.0 * d_h * ceil(h / n_devices)
    if m == "MQA":
        return 2.0 * d_h
    if m == "GQA":
        return 2.0 * d_h * ceil(g / min(n_devices, g))
    if m == "MLA":
        return float(d_c + d_r)                       # the single latent head cannot be sharded
    if m == "GLA-2":
        return (d_c / 2.0) * ceil(2 / min(n_devices, 2)) + d_r
    if m in ("MLRA-2", "MLRA-4"):
        return (d_c / 4.0) * ceil(4 / min(n_devices, 4)) + d_r
    raise ValueError(f"unknown method {method!r}")


def arithmetic_intensity(method: str, h: int, d_h: int = 128, g: int = 8,
                         d_c: int | None = None, d_r: int | None = None) -> float:
    """Decode flops per cache byte at long context (Table 2), 2-byte cache elements."""
    d_c = 4 * d_h if d_c is None else d_c
    d_r = d_h // 2 if d_r is None else d_r
    m = method.upper()
    if m == "MHA":
        return (4.0 * h * d_h) / (4.0 * h * d_h)
    if m == "MQA":
        return (4.0 * h * d_h) / (4.0 * d_h)
    if m == "GQA":
        return (4.0 * h * d_h) / (4.0 * g * d_h)
    if m == "MLA":
        return (4.0 * h * d_c + 2.0 * h * d_r) / (2.0 * (d_c + d_r))
    if m == "GLA-2":
        return (2.0 * h * d_c / 2 + h * d_r) / (2.0 * (d_c / 2 + d_r))
    if m == "MLRA-2":
        return (2.0 * h * d_c / 4 + h * d_r) / (2.0 * (d_c / 4 + d_r))
    if m == "MLRA-4":
        return (4.0 * h * d_c / 4 + 2.0 * h * d_r) / (2.0 * (d_c / 4 + d_r))
    raise ValueError(f"unknown method {method!r}")


def decode_bytes(seq_lens: Sequence[int], h: int, d_h: int, n_blocks: int, d_cb: int, d_r: int,
                 elt: int = 2, out_elt: int = 2, groups: int = 1) -> dict:
    """Bytes mlra_decode_attn must move once: the latent cache and the RoPE key of every valid
    token, the absorbed and RoPE queries, W^UV and the output.  Split-K partials, page-table
    reads and RoPE re-reads are overhead and deliberately not counted.  With head groups
    (MLRA-2, Eq. (6)) a block serves h/groups heads."""
    B = len(seq_lens)
    tokens = int(sum(int(n) for n in seq_lens))
    cache = tokens * (n_blocks * d_cb + d_r) * elt
    q_abs = B * n_blocks * (h // groups) * d_cb * elt
    q_rope = B * h * d_r * elt
    w_uv = n_blocks * d_cb * (h // groups) * d_h * elt
    out = B * h * d_h * out_elt
    return {"tokens": tokens, "cache": cache, "q_abs": q_abs, "q_rope": q_rope, "w_uv": w_uv,
            "out": out, "total": cache + q_abs + q_rope + w_uv + out}


def absorb_bytes(batch: int, h: int, d_h: int, n_blocks: int, d_cb: int, elt: int = 2, groups: int = 1) -> int:
    """Bytes of Step 1 (read q_nope and W^UK once, write the absorbed queries)."""
    hb = h // groups
    return (batch * h * d_h + n_blocks * d_cb * hb * d_h + batch * n_blocks * hb * d_cb) * elt


def append_bytes(batch: int, n_blocks: int, d_cb: int, d_r: int, src_elt: int = 4, elt: int = 2) -> int:
    return batch * (n_blocks * d_cb + d_r) * (src_elt + elt) + batch * 4


def decode_flops(seq_lens: Sequence[int], h: int, d_h: int, n_blocks: int, d_cb: int, d_r: int,
                 share_rope_score: bool = False, groups: int = 1) -> float:
    """Flops of Steps 2 and 3 per decode step: per token, head and block 2 d_cb (latent score)
    + 2 d_cb (PV) + 2 d_r (RoPE score; once per token and head if shared across blocks),
    i.e. Table 2's 4 n h d_c/4 + 2 n h d_h^R per block; plus the Step-3 up-projection.
    With head groups a head has n_blocks/groups branches (Table 2, MLRA-2 row)."""
    tokens = float(sum(int(n) for n in seq_lens))
    branches = n_blocks // groups
    rope_terms = 1 if share_rope_score else branches
    step2 = tokens * h * (branches * 4.0 * d_cb + rope_terms * 2.0 * d_r)
    step3 = len(seq_lens) * h * 2.0 * branches * d_cb * d_h
    return step2 + step3


def gqa_bytes(seq_lens: Sequence[int], h: int, d_h: int, g: int, elt: int = 2, out_elt: int = 2) -> dict:
    tokens = int(sum(int(n) for n in seq_lens))
    cache = tokens * 2 * g * d_h * elt
    q = len(seq_lens) * h * d_h * elt
    out = len(seq_lens) * h * d_h * out_elt
    return {"tokens": tokens, "cache": cache, "total": cache + q + out}


def gqa_flops(seq_lens: Sequence[int], h: int, d_h: int) -> float:
    return float(sum(int(n) for n in seq_lens)) * 4.0 * h * d_h
