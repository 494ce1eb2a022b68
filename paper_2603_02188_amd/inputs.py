"""Seeded synthetic inputs for MLRA / MLA / GQA decode attention.

This module only *draws and lays out* data: random numbers, dtype rounding of the
drawn values, page assignment and the physical cache layout.  It contains none of
the attention arithmetic and imports neither the HIP binding nor the CPU oracle, so
both sides can be fed from it.

Workload shapes follow the paper's decode benchmarks (Section 4.5, "Decoding
Efficiency": 128 heads, head dim 128, partial-RoPE dim 64, batch up to 128, contexts
from 1K to 16K and beyond 128K) and the KV-cache definition of Section 2.1: per token
a latent of d_c = 4 d_h channels, cut into n_blocks channel blocks of d_cb, plus one
RoPE key of d_r = d_h / 2 channels shared by all heads.

Physical cache layout (ours; the paper only fixes the logical concat [C^KV, K^RoPE]):
    latent_pool [num_pages][n_blocks][page_size][d_cb]
    rope_pool   [num_pages][page_size][d_r]
    page_table  [batch][max_pages_per_seq] int32  -> physical page id
    seq_lens    [batch] int32                      valid tokens (incl. the newest one)
bf16 arrays are carried as uint16 bit patterns (numpy has no bf16).
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, Optional

import numpy as np

BASE_SEED = 260302188
BF16_NAN_BITS = np.uint16(0x7FC0)


# --------------------------------------------------------------------------------------
# dtype helpers (storage only)
# --------------------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 values to bfloat16 (round-to-nearest-even); returns uint16 bits."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    nan = (u & np.uint32(0x7FFFFFFF)) > np.uint32(0x7F800000)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    r = ((u + bias) >> np.uint32(16)).astype(np.uint16)
    if nan.any():
        r = np.where(nan, BF16_NAN_BITS, r)
    return r


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bit patterns to float32."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def to_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    """float32 values -> storage array of the given dtype tag ('bf16' -> uint16 bits)."""
    if dtype == "bf16":
        return f32_to_bf16_bits(x)
    if dtype == "f32":
        return np.ascontiguousarray(x, dtype=np.float32)
    raise ValueError(f"unknown dtype tag {dtype!r}")


def to_f64(x: np.ndarray, dtype: str) -> np.ndarray:
    """Storage array -> float64 holding exactly the stored (already rounded) values."""
    if dtype == "bf16":
        return bf16_bits_to_f32(x).astype(np.float64)
    return np.asarray(x, dtype=np.float64)


# --------------------------------------------------------------------------------------
# workload registry
# --------------------------------------------------------------------------------------
@dataclass(frozen=True)
class Workload:
    """Problem shape, in the paper's notation (Appendix A) plus batch/paging terms."""

    name: str
    index: int            # 1-based workload number; seed = BASE_SEED + index
    batch: int
    n_min: int            # context length range, inclusive both ends
    n_max: int
    n_blocks: int         # latent channel blocks (4 = MLRA-4, 1 = one TP share / MLA)
    d_cb: int             # latent channels per block
    d_r: int              # RoPE key channels
    h: int                # query heads
    d_h: int              # head dim
    dtype: str            # 'bf16' or 'f32' (cache, queries and weights)
    page_size: int = 64
    shuffle_pages: bool = False
    spare_frac: float = 0.0
    g: int = 8            # KV heads of the GQA comparison
    groups: int = 1       # head groups: 1 = every block serves all h heads (MLRA-4, Eq. (5));
                          # 2 = MLRA-2 (Eq. (6)): block b serves the h/2 heads of group b // (n_blocks/2)

    @property
    def tau(self) -> float:
        """Softmax scale tau = 1/sqrt(d_h + d_h^R) (Section 2.1, Efficient Decoding)."""
        return 1.0 / float(np.sqrt(self.d_h + self.d_r))

    @property
    def seed(self) -> int:
        return BASE_SEED + self.index

    def scaled(self, **kw) -> "Workload":
        """Same shape family with some fields overridden (smaller parity cases)."""
        return replace(self, **kw)


WORKLOADS: Dict[str, Workload] = {
    "C1": Workload("C1-tiny-f32", 1, batch=1, n_min=256, n_max=256, n_blocks=4, d_cb=64,
                   d_r=32, h=8, d_h=64, dtype="f32"),
    "C2": Workload("C2-tp-share-bf16", 2, batch=16, n_min=16384, n_max=16384, n_blocks=1,
                   d_cb=128, d_r=64, h=128, d_h=128, dtype="bf16"),
    "C3": Workload("C3-mlra4-bf16", 3, batch=64, n_min=8192, n_max=8192, n_blocks=4,
                   d_cb=128, d_r=64, h=128, d_h=128, dtype="bf16"),
    "C4": Workload("C4-long-context-bf16", 4, batch=4, n_min=65536, n_max=131072,
                   n_blocks=4, d_cb=128, d_r=64, h=128, d_h=128, dtype="bf16"),
    "C5": Workload("C5-paged-mixed-bf16", 5, batch=128, n_min=512, n_max=8192, n_blocks=4,
                   d_cb=128, d_r=64, h=128, d_h=128, dtype="bf16", shuffle_pages=True,
                   spare_frac=0.10),
    # MLRA-2 (Eq. (6)) on the shape of C3: same cache, each block serves 64 of the 128 heads
    # GLA-2 baseline (Eq. (3)) on the same sizes: two latent heads of 2 d_h channels, each for half of the heads
    "G2": Workload("G2-gla2-bf16", 7, batch=64, n_min=8192, n_max=8192, n_blocks=2,
                   d_cb=256, d_r=64, h=128, d_h=128, dtype="bf16", groups=2),
    "M2": Workload("M2-mlra2-bf16", 6, batch=64, n_min=8192, n_max=8192, n_blocks=4,
                   d_cb=128, d_r=64, h=128, d_h=128, dtype="bf16", groups=2),
}


# --------------------------------------------------------------------------------------
# generators
# --------------------------------------------------------------------------------------
@dataclass
class DecodeInputs:
    """One decode step's inputs for the latent-cache path (MLRA / MLA)."""

    wl: Workload
    latent_pool: np.ndarray   # [P][NB][page][d_cb] storage dtype
    rope_pool: np.ndarray     # [P][page][d_r]
    page_table: np.ndarray    # [B][max_pages] int32
    seq_lens: np.ndarray      # [B] int32
    q_nope: np.ndarray        # [B][h][d_h]
    q_rope: np.ndarray        # [B][h][d_r]
    w_uk: np.ndarray          # [NB][d_cb][(h/groups)*d_h]
    w_uv: np.ndarray          # [NB][d_cb][(h/groups)*d_h]
    c_kv_new: np.ndarray      # [B][NB*d_cb] float32, the newest token's unrounded latent
    k_rope_new: np.ndarray    # [B][d_r]     float32, the newest token's unrounded RoPE key
    positions: np.ndarray     # [B] int32 = seq_lens - 1

    @property
    def num_pages(self) -> int:
        return int(self.latent_pool.shape[0])

    @property
    def max_pages_per_seq(self) -> int:
        return int(self.page_table.shape[1])


def draw_seq_lens(wl: Workload) -> np.ndarray:
    rng = np.random.default_rng([wl.seed, 0xA11])
    return rng.integers(wl.n_min, wl.n_max + 1, size=wl.batch).astype(np.int32)


def draw_page_table(wl: Workload, seq_lens: np.ndarray):
    """Returns (page_table [B][max_pages], num_pages).  Unused entries name a spare page that no sequence
    owns (poisoned in parity tests, so a read through an unmapped entry shows up), or page 0 if the pool
    has no spare page."""
    pages = (seq_lens.astype(np.int64) + wl.page_size - 1) // wl.page_size
    used = int(pages.sum())
    num_pages = max(1, int(np.ceil(used * (1.0 + wl.spare_frac))))
    if wl.shuffle_pages:
        rng = np.random.default_rng([wl.seed, 0xB22])
        order = rng.permutation(num_pages).astype(np.int32)
    else:
        order = np.arange(num_pages, dtype=np.int32)
    max_pages = max(1, int(pages.max()) if len(pages) else 1)
    table = np.full((wl.batch, max_pages), order[used] if num_pages > used else 0, dtype=np.int32)
    at = 0
    for b in range(wl.batch):
        k = int(pages[b])
        table[b, :k] = order[at:at + k]
        at += k
    return table, num_pages


def _seq_rng(wl: Workload, b: int) -> np.random.Generator:
    return np.random.default_rng([wl.seed, 0xC33, b])


def draw_sequence_rows(wl: Workload, b: int, n: int):
    """Unrounded float32 cache rows of sequence b: latent [n][NB*d_cb], rope [n][d_r]."""
    rng = _seq_rng(wl, b)
    latent = rng.standard_normal((n, wl.n_blocks * wl.d_cb), dtype=np.float32)
    rope = rng.standard_normal((n, wl.d_r), dtype=np.float32)
    return latent, rope


def draw_queries_weights(wl: Workload):
    """q_nope, q_rope ~ N(0,1); W^UK, W^UV ~ N(0, variance 1/d_cb), all rounded to wl.dtype.
    With head groups (MLRA-2) a block's weight rows have columns for the heads of its group only."""
    rng = np.random.default_rng([wl.seed, 0xD44])
    q_nope = rng.standard_normal((wl.batch, wl.h, wl.d_h), dtype=np.float32)
    q_rope = rng.standard_normal((wl.batch, wl.h, wl.d_r), dtype=np.float32)
    std = np.float32(1.0 / np.sqrt(wl.d_cb))
    cols = (wl.h // wl.groups) * wl.d_h
    w_uk = rng.standard_normal((wl.n_blocks, wl.d_cb, cols), dtype=np.float32) * std
    w_uv = rng.standard_normal((wl.n_blocks, wl.d_cb, cols), dtype=np.float32) * std
    return (to_storage(q_nope, wl.dtype), to_storage(q_rope, wl.dtype),
            to_storage(w_uk, wl.dtype), to_storage(w_uv, wl.dtype))


def make_decode_inputs(wl: Workload, poison: bool = True, hole: bool = False,
                       seq_lens: Optional[np.ndarray] = None) -> DecodeInputs:
    """Builds the paged latent cache and one decode step's queries and weights.

    poison: slots no sequence owns (tails of last pages, spare pages) hold NaN so a
            kernel that lets them leak into a result is caught; otherwise they hold 0.
    hole:   the newest row (position seq_len-1) of every sequence is left poisoned in the
            pools; mlra_append_kv is expected to fill it from c_kv_new / k_rope_new.
    """
    if seq_lens is None:
        seq_lens = draw_seq_lens(wl)
    seq_lens = np.asarray(seq_lens, dtype=np.int32)
    table, num_pages = draw_page_table(wl, seq_lens)
    ps, NB, dcb, dr = wl.page_size, wl.n_blocks, wl.d_cb, wl.d_r
    store = np.uint16 if wl.dtype == "bf16" else np.float32
    latent_pool = np.zeros((num_pages, NB, ps, dcb), dtype=store)
    rope_pool = np.zeros((num_pages, ps, dr), dtype=store)
    if poison:
        fill = BF16_NAN_BITS if wl.dtype == "bf16" else np.float32(np.nan)
        latent_pool[...] = fill
        rope_pool[...] = fill
    c_kv_new = np.zeros((wl.batch, NB * dcb), dtype=np.float32)
    k_rope_new = np.zeros((wl.batch, dr), dtype=np.float32)
    for b in range(wl.batch):
        n = int(seq_lens[b])
        if n == 0:
            continue
        latent, rope = draw_sequence_rows(wl, b, n)
        c_kv_new[b] = latent[n - 1]
        k_rope_new[b] = rope[n - 1]
        n_fill = n - 1 if hole else n
        lat_s = to_storage(latent[:n_fill], wl.dtype)
        rope_s = to_storage(rope[:n_fill], wl.dtype)
        full = n_fill // ps                      # whole pages in one scatter, then the ragged tail
        if full:
            phys = table[b, :full]
            latent_pool[phys] = lat_s[:full * ps].reshape(full, ps, NB, dcb).transpose(0, 2, 1, 3)
            rope_pool[phys] = rope_s[:full * ps].reshape(full, ps, dr)
        rem = n_fill - full * ps
        if rem:
            phys = int(table[b, full])
            latent_pool[phys, :, :rem, :] = lat_s[full * ps:].reshape(rem, NB, dcb).transpose(1, 0, 2)
            rope_pool[phys, :rem, :] = rope_s[full * ps:]
    q_nope, q_rope, w_uk, w_uv = draw_queries_weights(wl)
    return DecodeInputs(wl, latent_pool, rope_pool, table, seq_lens, q_nope, q_rope, w_uk, w_uv,
                        c_kv_new, k_rope_new, (seq_lens - 1).astype(np.int32))


def as_single_latent(inp: DecodeInputs) -> DecodeInputs:
    """The same logical cache and weights presented as one latent block of NB*d_cb channels
    (the MLA comparison: W^UK/W^UV are the row blocks stacked, Eq. (2))."""
    wl = inp.wl
    P, NB, ps, dcb = inp.latent_pool.shape
    pool = np.ascontiguousarray(inp.latent_pool.transpose(0, 2, 1, 3)).reshape(P, 1, ps, NB * dcb)
    wl1 = wl.scaled(name=wl.name + "-as-mla", n_blocks=1, d_cb=NB * dcb)
    hd = wl.h * wl.d_h
    return DecodeInputs(wl1, pool, inp.rope_pool, inp.page_table, inp.seq_lens, inp.q_nope,
                        inp.q_rope, inp.w_uk.reshape(1, NB * dcb, hd), inp.w_uv.reshape(1, NB * dcb, hd),
                        inp.c_kv_new, inp.k_rope_new, inp.positions)


@dataclass
class GqaInputs:
    """One decode step's inputs for the GQA comparison (Appendix C, MQA/GQA)."""

    wl: Workload
    k_pool: np.ndarray       # [P][g][page][d_h]
    v_pool: np.ndarray       # [P][g][page][d_h]
    page_table: np.ndarray   # [B][max_pages] int32
    seq_lens: np.ndarray     # [B] int32
    q: np.ndarray            # [B][h][d_h]

    @property
    def scale(self) -> float:
        return 1.0 / float(np.sqrt(self.wl.d_h))


def make_gqa_inputs(wl: Workload, poison: bool = True,
                    seq_lens: Optional[np.ndarray] = None) -> GqaInputs:
    """K, V ~ N(0,1) in [P][g][page][d_h]; lengths and page table as the latent path's."""
    if seq_lens is None:
        seq_lens = draw_seq_lens(wl)
    seq_lens = np.asarray(seq_lens, dtype=np.int32)
    table, num_pages = draw_page_table(wl, seq_lens)
    ps, g, dh = wl.page_size, wl.g, wl.d_h
    store = np.uint16 if wl.dtype == "bf16" else np.float32
    k_pool = np.zeros((num_pages, g, ps, dh), dtype=store)
    v_pool = np.zeros((num_pages, g, ps, dh), dtype=store)
    if poison:
        fill = BF16_NAN_BITS if wl.dtype == "bf16" else np.float32(np.nan)
        k_pool[...] = fill
        v_pool[...] = fill
    for b in range(wl.batch):
        n = int(seq_lens[b])
        if n == 0:
            continue
        rng = np.random.default_rng([wl.seed, 0xE55, b])
        k = to_storage(rng.standard_normal((n, g, dh), dtype=np.float32), wl.dtype)
        v = to_storage(rng.standard_normal((n, g, dh), dtype=np.float32), wl.dtype)
        full = n // ps
        if full:
            phys = table[b, :full]
            k_pool[phys] = k[:full * ps].reshape(full, ps, g, dh).transpose(0, 2, 1, 3)
            v_pool[phys] = v[:full * ps].reshape(full, ps, g, dh).transpose(0, 2, 1, 3)
        rem = n - full * ps
        if rem:
            phys = int(table[b, full])
            k_pool[phys, :, :rem, :] = k[full * ps:].transpose(1, 0, 2)
            v_pool[phys, :, :rem, :] = v[full * ps:].transpose(1, 0, 2)
    rng = np.random.default_rng([wl.seed, 0xF66])
    q = to_storage(rng.standard_normal((wl.batch, wl.h, dh), dtype=np.float32), wl.dtype)
    return GqaInputs(wl, k_pool, v_pool, table, seq_lens, q)


@dataclass
class PreInputs:
    """The new token's hidden states and the projection weights of Appendix C, subsection "Multi-Head Latent Attention (MLA)" (the form MLRA keeps)."""

    wl: Workload
    d: int                   # hidden size
    d_cq: int                # query latent dim d_c'
    hidden: np.ndarray       # [B][d]
    w_dq: np.ndarray         # [d][d_cq]
    w_dkv: np.ndarray        # [d][NB*d_cb]
    w_kr: np.ndarray         # [d][d_r]
    w_uq: np.ndarray         # [d_cq][h*d_h]
    w_qr: np.ndarray         # [d_cq][h*d_r]
    gain_q: np.ndarray       # [d_cq]
    gain_kv: np.ndarray      # [NB*d_cb]
    eps: float = 1e-6
    rope_base: float = 10000.0

    @property
    def alpha_q(self) -> float:
        """Eq. (9): sqrt(d / d_c')."""
        return float(np.sqrt(self.d / self.d_cq))

    @property
    def alpha_kv(self) -> float:
        """Eq. (9), MLRA: sqrt(4 d / d_c)."""
        return float(np.sqrt(4.0 * self.d / (self.wl.n_blocks * self.wl.d_cb)))


def make_pre_inputs(wl: Workload, d: int, d_cq: int, unit_gains: bool = False) -> PreInputs:
    """hidden ~ N(0,1); every projection matrix ~ N(0, variance 1/d) (a common variance, as the paper's
    variance analysis of Section 3.3 assumes: with the Eq. (9) scaling queries and keys then have about
    unit variance); RMSNorm gains 1 + 0.1 N(0,1) (or exactly 1).  All rounded to wl.dtype."""
    rng = np.random.default_rng([wl.seed, 0x977])
    d_c = wl.n_blocks * wl.d_cb
    std = np.float32(1.0 / np.sqrt(d))
    def mat(r, c):
        return to_storage(rng.standard_normal((r, c), dtype=np.float32) * std, wl.dtype)
    hidden = to_storage(rng.standard_normal((wl.batch, d), dtype=np.float32), wl.dtype)
    w_dq, w_dkv, w_kr = mat(d, d_cq), mat(d, d_c), mat(d, wl.d_r)
    w_uq, w_qr = mat(d_cq, wl.h * wl.d_h), mat(d_cq, wl.h * wl.d_r)
    if unit_gains:
        gq, gkv = np.ones(d_cq, np.float32), np.ones(d_c, np.float32)
    else:
        gq = 1.0 + 0.1 * rng.standard_normal(d_cq, dtype=np.float32)
        gkv = 1.0 + 0.1 * rng.standard_normal(d_c, dtype=np.float32)
    return PreInputs(wl, d, d_cq, hidden, w_dq, w_dkv, w_kr, w_uq, w_qr, to_storage(gq, wl.dtype),
                     to_storage(gkv, wl.dtype))
