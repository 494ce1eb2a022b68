"""CPU oracle for MLRA / MLA / GQA decode attention -- TEST INFRASTRUCTURE ONLY.

Plain, slow, float64 numpy written from the paper's definitions.  It shares no code with
the HIP library and must never be imported by the product path; only the tests, the
smoke check and the bench's cpu_baseline leg may call it.

What each function follows (all citations are to the MLRA paper):
  * mlra_decode_unabsorbed  -- Eq. (5) (MLRA-4) read for the single decode query at the
    last prefix position, as in Section 2.1 "Efficient Decoding": per block b the NoPE keys
    and values are materialised as C_(b) W^UK_(b),(i) and C_(b) W^UV_(b),(i).
  * absorb_q / latent_attention / up_project  -- Steps 1, 2 (Eq. (1)) and 3 of the
    three-step absorbed decode of Section 2.1, applied per block (d_c -> d_cb).
  * mlra_decode_absorbed    -- the three steps per block, block outputs summed (Eq. (5)),
    times the output rescale alpha_attn of Eq. (10).
  * mla_decode              -- the same with a single block of d_c channels (Section 2.1).
  * gla2_decode             -- GLA-2 (Section 2.3, Eq. (3)-(4)): head i attends through the latent head of its
    group, [C_(2g), C_(2g+1)], with that group's matrices; the absorbed three steps on 2 d_cb channels.
  * gated_output            -- Appendix E: the attention output times the gate G, elementwise.
  * mlra_decode_multi       -- Eq. (5) for the last q_len rows of a sequence at once: row n - q_len + j
    attends to its prefix {0..n - q_len + j} (Section 2.1 states attention for a position over its
    prefix), i.e. the causal tail of the n x n attention.
  * mlra2_decode_unabsorbed -- Eq. (6) (MLRA-2) with the group map gamma(i) and the group matrices
    W^(gamma),UK / W^(gamma),UV of Section 2.3 (GLA-2), for the single decode query.
  * mlra2_absorb_q / mlra2_decode_absorbed -- the three absorbed steps applied to each of
    the two branches of Eq. (6); each latent block serves the h/2 heads of its group.
  * gqa_decode              -- Appendix C, MQA/GQA: query head i reads KV head floor(i/r),
    r = h/g.
  * rms_norm / rope / pre_attention -- the projections that produce one new token's queries
    and cache row (Section 2.1 and Appendix C, subsection "Multi-Head Latent Attention (MLA)": C^Q = alpha_q RMSNorm(H W^DQ), Q^NoPE = C^Q W^UQ,
    Q^RoPE = RoPE(C^Q W^QR), C^KV = alpha_kv RMSNorm(H W^DKV), K^RoPE = RoPE(H W^KR); the scaling
    factors are those of Eq. (9)); RoPE rotates the 2-D blocks [2l, 2l+1] by t theta_l as in the
    proof of the paper's RoPE theorem (Appendix B).
  * round_bf16 / append_kv / gather_sequence -- storage conventions of this build (the paper
    is silent on dtype rounding and physical layout): round-to-nearest-even to bfloat16,
    and the paged pool layout [page][block][slot][channel].

Pins: every function above is pinned in tests/test_oracle_pins.py against something other
than itself (Eq. (2) identity, a library SDPA on materialised K/V, closed forms for n = 1,
two tokens, zero queries and constant caches, split/merge and permutation invariances,
brute-force Python loops on tiny inputs, hand-picked bf16 rounding cases; for MLRA-2 a
brute-force evaluation of Eq. (6), the GLA-2 value identity at n = 1, the head-group
independence and a library SDPA per branch).
The paper prints no numeric attention example, so there is no printed value to reproduce.
"""
from __future__ import annotations

import numpy as np


# --------------------------------------------------------------------------------------
# Section 2.1 "Block Multiplications": W_(b),(i) and C_(b)
# --------------------------------------------------------------------------------------
def w_block(W: np.ndarray, b: int, i: int, d_cb: int, d_h: int) -> np.ndarray:
    """W_(b),(i) = W[b*d_cb:(b+1)*d_cb, i*d_h:(i+1)*d_h] for W in R^{d_c x (h d_h)}."""
    return W[b * d_cb:(b + 1) * d_cb, i * d_h:(i + 1) * d_h]


def c_block(C: np.ndarray, b: int, d_cb: int) -> np.ndarray:
    """C_(b) = C[:, b*d_cb:(b+1)*d_cb] for C in R^{n x d_c}."""
    return C[:, b * d_cb:(b + 1) * d_cb]


def softmax_1d(s: np.ndarray) -> np.ndarray:
    s = np.asarray(s, dtype=np.float64)
    e = np.exp(s - np.max(s))
    return e / np.sum(e)


# --------------------------------------------------------------------------------------
# Eq. (5), unabsorbed: the definition.  Materialises K and V, so small inputs only.
# --------------------------------------------------------------------------------------
def mlra_decode_unabsorbed(q_nope, q_rope, C, KR, W_UK, W_UV, n_blocks, tau, out_scale=1.0):
    """O_i = out_scale * sum_b Softmax(tau q^N_i (C_b W^UK_(b),(i))^T + tau q^R_i KR^T) (C_b W^UV_(b),(i)).

    q_nope [h][d_h], q_rope [h][d_r], C [n][d_c], KR [n][d_r], W_UK/W_UV [d_c][h*d_h].
    Returns O [h][d_h] (zeros when n == 0).
    """
    q_nope = np.asarray(q_nope, np.float64)
    q_rope = np.asarray(q_rope, np.float64)
    C = np.asarray(C, np.float64)
    KR = np.asarray(KR, np.float64)
    W_UK = np.asarray(W_UK, np.float64)
    W_UV = np.asarray(W_UV, np.float64)
    h, d_h = q_nope.shape
    n, d_c = C.shape
    d_cb = d_c // n_blocks
    O = np.zeros((h, d_h))
    if n == 0:
        return O
    for i in range(h):
        acc = np.zeros(d_h)
        for b in range(n_blocks):
            K_bi = c_block(C, b, d_cb) @ w_block(W_UK, b, i, d_cb, d_h)     # [n][d_h]
            V_bi = c_block(C, b, d_cb) @ w_block(W_UV, b, i, d_cb, d_h)     # [n][d_h]
            s = tau * (K_bi @ q_nope[i]) + tau * (KR @ q_rope[i])            # [n]
            p = softmax_1d(s)
            acc = acc + p @ V_bi
        O[i] = out_scale * acc
    return O


# --------------------------------------------------------------------------------------
# Section 2.1, Steps 1-3, per block
# --------------------------------------------------------------------------------------
def absorb_q(q_nope, W_UK, n_blocks):
    """Step 1 per block: q~_b[i] = W^UK_(b),(i) q^N_i, i.e. einsum('hp,hpc->hc') with
    W~_i = (W^UK_(b),(i))^T.  Returns [n_blocks][h][d_cb]."""
    q_nope = np.asarray(q_nope, np.float64)
    W_UK = np.asarray(W_UK, np.float64)
    h, d_h = q_nope.shape
    d_c = W_UK.shape[0]
    d_cb = d_c // n_blocks
    out = np.zeros((n_blocks, h, d_cb))
    for b in range(n_blocks):
        W_b = W_UK[b * d_cb:(b + 1) * d_cb].reshape(d_cb, h, d_h)      # [c][h][p]
        out[b] = np.einsum("hp,chp->hc", q_nope, W_b)
    return out


def latent_attention(q_abs_b, q_rope, C_b, KR, tau):
    """Step 2 (Eq. (1)) on one block: shared key [C_b, KR], shared value C_b for all heads.

    Returns (Z [h][d_cb], lse [h]) with lse = log sum_t exp(s_t) of the scaled logits.
    n == 0 gives Z = 0 and lse = -inf.
    """
    q_abs_b = np.asarray(q_abs_b, np.float64)
    q_rope = np.asarray(q_rope, np.float64)
    C_b = np.asarray(C_b, np.float64)
    KR = np.asarray(KR, np.float64)
    h = q_abs_b.shape[0]
    n = C_b.shape[0]
    if n == 0:
        return np.zeros((h, C_b.shape[1])), np.full(h, -np.inf)
    S = tau * (q_abs_b @ C_b.T) + tau * (q_rope @ KR.T)                 # [h][n]
    m = S.max(axis=1, keepdims=True)
    E = np.exp(S - m)
    l = E.sum(axis=1, keepdims=True)
    Z = (E / l) @ C_b
    return Z, (m + np.log(l))[:, 0]


def up_project(Z_b, W_UV_b, h, d_h):
    """Step 3 on one block: o_b[i] = z_b[i] W^UV_(b),(i) (einsum 'hc,hcp->hp')."""
    W = np.asarray(W_UV_b, np.float64).reshape(-1, h, d_h)            # [c][h][p]
    return np.einsum("hc,chp->hp", np.asarray(Z_b, np.float64), W)


def mlra_decode_absorbed(q_nope, q_rope, C, KR, W_UK, W_UV, n_blocks, tau, out_scale=1.0,
                         return_lse=False):
    """Eq. (5) through the absorbed three-step form, blocks summed in order b = 0..n_blocks-1."""
    q_nope = np.asarray(q_nope, np.float64)
    C = np.asarray(C, np.float64)
    W_UV = np.asarray(W_UV, np.float64)
    h, d_h = q_nope.shape
    d_c = C.shape[1]
    d_cb = d_c // n_blocks
    q_abs = absorb_q(q_nope, W_UK, n_blocks)
    O = np.zeros((h, d_h))
    lse = np.zeros((n_blocks, h))
    for b in range(n_blocks):
        Z_b, lse[b] = latent_attention(q_abs[b], q_rope, c_block(C, b, d_cb), KR, tau)
        O = O + up_project(Z_b, W_UV[b * d_cb:(b + 1) * d_cb], h, d_h)
    O = out_scale * O
    return (O, lse) if return_lse else O


def mlra_decode_multi(q_nope, q_rope, C, KR, W_UK, W_UV, n_blocks, tau, out_scale=1.0):
    """Queries of the last q_len cached rows: q_nope [q_len][h][d_h], q_rope [q_len][h][d_r]; C, KR hold all
    n rows (the q_len newest included).  Query j sits at row n - q_len + j and attends to rows
    0 .. n - q_len + j.  Returns O [q_len][h][d_h]; a query whose prefix is empty (n < q_len) gives zeros."""
    q_nope = np.asarray(q_nope, np.float64)
    q_len, h, d_h = q_nope.shape
    n = np.asarray(C).shape[0]
    O = np.zeros((q_len, h, d_h))
    for j in range(q_len):
        n_eff = max(0, n - (q_len - 1 - j))
        O[j] = mlra_decode_absorbed(q_nope[j], np.asarray(q_rope)[j], np.asarray(C)[:n_eff], np.asarray(KR)[:n_eff],
                                    W_UK, W_UV, n_blocks, tau, out_scale)
    return O


def gla2_decode(q_nope, q_rope, C, KR, W_UK_g, W_UV_g, tau):
    """GLA-2: O_i = Softmax(tau q^N_i ([C_(2g), C_(2g+1)] W^(g),UK_:,(i))^T + tau q^R_i KR^T) [C_(2g), C_(2g+1)] W^(g),UV_:,(i),
    g = gamma(i).  q_nope [h][d_h], C [n][d_c] (two latent heads of d_c/2 channels side by side),
    W_UK_g / W_UV_g [2][d_c/2][(h/2)*d_h].  Returns O [h][d_h]."""
    q_nope = np.asarray(q_nope, np.float64)
    q_rope = np.asarray(q_rope, np.float64)
    C = np.asarray(C, np.float64)
    h, d_h = q_nope.shape
    hg, d_g = h // 2, C.shape[1] // 2
    O = np.zeros((h, d_h))
    for g in range(2):
        heads = slice(g * hg, (g + 1) * hg)
        O[heads] = mla_decode(q_nope[heads], q_rope[heads], C[:, g * d_g:(g + 1) * d_g], KR,
                              np.asarray(W_UK_g, np.float64)[g], np.asarray(W_UV_g, np.float64)[g], tau)
    return O


def gated_output(O, G):
    """Appendix E ("Gated Attention"): O^attn = Attention(H') (.) G, elementwise, with G = sigma(H W^G) given."""
    return np.asarray(O, np.float64) * np.asarray(G, np.float64)


def mla_decode(q_nope, q_rope, C, KR, W_UK, W_UV, tau):
    """MLA three-step decode (Section 2.1): one latent block of d_c channels."""
    return mlra_decode_absorbed(q_nope, q_rope, C, KR, W_UK, W_UV, 1, tau, 1.0)


# --------------------------------------------------------------------------------------
# Eq. (6), MLRA-2.  Group map and group matrices as in Section 2.3 (GLA-2): head i belongs to
# group gamma(i) = 0 for i < h/2, else 1, with in-group index i_bar = i - gamma(i) h/2; group
# gamma owns latent blocks 2 gamma and 2 gamma + 1 and matrices W^(gamma) in R^{2 d_cb x (h/2) d_h};
# W^(gamma)_(j),(i) = W^(gamma)[j d_cb:(j+1) d_cb, i_bar d_h:(i_bar+1) d_h].
# --------------------------------------------------------------------------------------
def gamma(i: int, h: int) -> int:
    return 0 if i < h // 2 else 1


def wg_block(W_g: np.ndarray, j: int, i_bar: int, d_cb: int, d_h: int) -> np.ndarray:
    """W^(gamma)_(j),(i) from one group's matrix W_g [2*d_cb][(h/2)*d_h]."""
    return W_g[j * d_cb:(j + 1) * d_cb, i_bar * d_h:(i_bar + 1) * d_h]


def mlra2_decode_unabsorbed(q_nope, q_rope, C, KR, W_UK_g, W_UV_g, tau, out_scale=1.0):
    """O_i = out_scale * sum_{j=0,1} Softmax(tau q^N_i (C_(2g+j) W^(g),UK_(j),(i))^T + tau q^R_i KR^T)
                                      (C_(2g+j) W^(g),UV_(j),(i)),   g = gamma(i).

    q_nope [h][d_h], q_rope [h][d_r], C [n][4*d_cb], KR [n][d_r], W_UK_g / W_UV_g [2][2*d_cb][(h/2)*d_h].
    Returns O [h][d_h] (zeros when n == 0).
    """
    q_nope = np.asarray(q_nope, np.float64)
    q_rope = np.asarray(q_rope, np.float64)
    C = np.asarray(C, np.float64)
    KR = np.asarray(KR, np.float64)
    W_UK_g = np.asarray(W_UK_g, np.float64)
    W_UV_g = np.asarray(W_UV_g, np.float64)
    h, d_h = q_nope.shape
    n, d_c = C.shape
    d_cb = d_c // 4
    O = np.zeros((h, d_h))
    if n == 0:
        return O
    for i in range(h):
        g = gamma(i, h)
        i_bar = i - g * (h // 2)
        acc = np.zeros(d_h)
        for j in range(2):
            C_b = c_block(C, 2 * g + j, d_cb)
            K_bi = C_b @ wg_block(W_UK_g[g], j, i_bar, d_cb, d_h)              # [n][d_h]
            V_bi = C_b @ wg_block(W_UV_g[g], j, i_bar, d_cb, d_h)
            s = tau * (K_bi @ q_nope[i]) + tau * (KR @ q_rope[i])
            acc = acc + softmax_1d(s) @ V_bi
        O[i] = out_scale * acc
    return O


def mlra2_absorb_q(q_nope, W_UK_g):
    """Step 1 on each branch of Eq. (6): q~_b[i_bar] = W^(g),UK_(j),(i) q^N_i for block b = 2g + j.
    Returns [4][h/2][d_cb] (rows of block b are the heads of group b // 2 in order)."""
    q_nope = np.asarray(q_nope, np.float64)
    W_UK_g = np.asarray(W_UK_g, np.float64)
    h, d_h = q_nope.shape
    hg = h // 2
    d_cb = W_UK_g.shape[1] // 2
    out = np.zeros((4, hg, d_cb))
    for g in range(2):
        for j in range(2):
            W = W_UK_g[g][j * d_cb:(j + 1) * d_cb].reshape(d_cb, hg, d_h)      # [c][i_bar][p]
            out[2 * g + j] = np.einsum("hp,chp->hc", q_nope[g * hg:(g + 1) * hg], W)
    return out


def mlra2_decode_absorbed(q_nope, q_rope, C, KR, W_UK_g, W_UV_g, tau, out_scale=1.0, return_lse=False):
    """Eq. (6) through the absorbed three-step form; branch j = 0 is added before j = 1.
    lse is [4][h/2], indexed like mlra2_absorb_q's result."""
    q_nope = np.asarray(q_nope, np.float64)
    q_rope = np.asarray(q_rope, np.float64)
    C = np.asarray(C, np.float64)
    W_UV_g = np.asarray(W_UV_g, np.float64)
    h, d_h = q_nope.shape
    hg = h // 2
    d_cb = C.shape[1] // 4
    q_abs = mlra2_absorb_q(q_nope, W_UK_g)
    O = np.zeros((h, d_h))
    lse = np.zeros((4, hg))
    for g in range(2):
        heads = slice(g * hg, (g + 1) * hg)
        for j in range(2):
            b = 2 * g + j
            Z_b, lse[b] = latent_attention(q_abs[b], q_rope[heads], c_block(C, b, d_cb), KR, tau)
            O[heads] = O[heads] + up_project(Z_b, W_UV_g[g][j * d_cb:(j + 1) * d_cb], hg, d_h)
    O = out_scale * O
    return (O, lse) if return_lse else O


# --------------------------------------------------------------------------------------
# Appendix C, MQA/GQA
# --------------------------------------------------------------------------------------
def gqa_decode(q, K, V, scale):
    """O_i = Softmax(scale * q_i K[:, floor(i/r), :]^T) V[:, floor(i/r), :], r = h/g.

    q [h][d_h], K and V [n][g][d_h].  Returns [h][d_h] (zeros when n == 0)."""
    q = np.asarray(q, np.float64)
    K = np.asarray(K, np.float64)
    V = np.asarray(V, np.float64)
    h, d_h = q.shape
    n, g, _ = K.shape
    r = h // g
    O = np.zeros((h, d_h))
    if n == 0:
        return O
    for i in range(h):
        j = i // r
        p = softmax_1d(scale * (K[:, j, :] @ q[i]))
        O[i] = p @ V[:, j, :]
    return O


# --------------------------------------------------------------------------------------
# Pre-attention of one new token per sequence (Section 2.1; Appendix C, subsection MLA; Eq. (9))
# --------------------------------------------------------------------------------------
def rms_norm(x, gain=None, eps=0.0):
    """RMSNorm over the last axis: x / sqrt(mean(x^2) + eps) * gain (the paper cites the standard
    definition; gain and eps are this build's arguments, 1 and a small constant in the workloads)."""
    x = np.asarray(x, np.float64)
    y = x / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps)
    return y if gain is None else y * np.asarray(gain, np.float64)


def rope_angles(d_r: int, base: float) -> np.ndarray:
    """theta_l = base^(-2l/d_r), l = 0..d_r/2-1 (the usual frequencies; the paper leaves them open)."""
    return np.asarray(base, np.float64) ** (-2.0 * np.arange(d_r // 2) / d_r)


def rope(x, t, base=10000.0):
    """Rotates each 2-D block x[..., 2l:2l+2] by the angle t * theta_l (x R_t in the paper's
    row-vector notation).  x [..., d_r], t scalar or broadcastable to x[..., 0]."""
    x = np.asarray(x, np.float64)
    d_r = x.shape[-1]
    ang = np.asarray(t, np.float64)[..., None] * rope_angles(d_r, base)     # [..., d_r/2]
    c, s = np.cos(ang), np.sin(ang)
    even, odd = x[..., 0::2], x[..., 1::2]
    out = np.empty_like(x)
    out[..., 0::2] = even * c - odd * s
    out[..., 1::2] = even * s + odd * c
    return out


def pre_attention(hidden, position, W_DQ, W_DKV, W_KR, W_UQ, W_QR, h, alpha_q, alpha_kv,
                  gain_q=None, gain_kv=None, eps=0.0, rope_base=10000.0, round_cq=None):
    """One token: hidden [d], position t.  Returns (c_kv [d_c], k_rope [d_r], q_nope [h][d_h],
    q_rope [h][d_r]).  round_cq, if given, is applied to C^Q before the up-projections (the
    storage rounding of the intermediate latent in a 16-bit pipeline; None = exact)."""
    x = np.asarray(hidden, np.float64)
    c_q = alpha_q * rms_norm(x @ np.asarray(W_DQ, np.float64), gain_q, eps)
    if round_cq is not None:
        c_q = round_cq(c_q)
    c_kv = alpha_kv * rms_norm(x @ np.asarray(W_DKV, np.float64), gain_kv, eps)
    k_rope = rope(x @ np.asarray(W_KR, np.float64), position, rope_base)
    q_nope = (c_q @ np.asarray(W_UQ, np.float64)).reshape(h, -1)
    q_rope = rope((c_q @ np.asarray(W_QR, np.float64)).reshape(h, -1), position, rope_base)
    return c_kv, k_rope, q_nope, q_rope


# --------------------------------------------------------------------------------------
# storage conventions of this build
# --------------------------------------------------------------------------------------
def round_bf16(x):
    """float32 -> nearest bfloat16 value (ties to even), returned as float64.

    bfloat16 keeps the top 16 bits of the IEEE binary32 pattern: 1 sign, 8 exponent and
    7 mantissa bits.  Rounding is done on the integer pattern: add half an ulp (0x7FFF)
    plus the lowest kept bit, then truncate.
    """
    x32 = np.asarray(x, dtype=np.float32)
    bits = x32.view(np.uint32).astype(np.uint64)
    keep_lsb = (bits >> np.uint64(16)) & np.uint64(1)
    rounded = ((bits + np.uint64(0x7FFF) + keep_lsb) >> np.uint64(16)) << np.uint64(16)
    out = rounded.astype(np.uint32).view(np.float32).astype(np.float64)
    return np.where(np.isnan(x32), np.nan, out)


def gather_sequence(latent_pool, rope_pool, page_table_row, n):
    """Logical rows of one sequence from the paged pools.

    latent_pool [P][NB][page][d_cb], rope_pool [P][page][d_r] (already float64),
    page_table_row [max_pages].  Returns C [n][NB*d_cb] (blocks side by side in order
    b = 0..NB-1, Section 2.1 "Block Multiplications") and KR [n][d_r].
    """
    P, NB, ps, d_cb = latent_pool.shape
    d_r = rope_pool.shape[2]
    C = np.zeros((n, NB * d_cb))
    KR = np.zeros((n, d_r))
    for t in range(0, n, ps):
        page = int(page_table_row[t // ps])
        k = min(ps, n - t)
        for b in range(NB):
            C[t:t + k, b * d_cb:(b + 1) * d_cb] = latent_pool[page, b, :k, :]
        KR[t:t + k] = rope_pool[page, :k, :]
    return C, KR


def gather_gqa_sequence(k_pool, v_pool, page_table_row, n):
    """K, V [n][g][d_h] of one sequence from pools laid out [P][g][page][d_h]."""
    P, g, ps, d_h = k_pool.shape
    K = np.zeros((n, g, d_h))
    V = np.zeros((n, g, d_h))
    for t in range(0, n, ps):
        page = int(page_table_row[t // ps])
        k = min(ps, n - t)
        K[t:t + k] = np.transpose(k_pool[page, :, :k, :], (1, 0, 2))
        V[t:t + k] = np.transpose(v_pool[page, :, :k, :], (1, 0, 2))
    return K, V


def append_kv(latent_pool, rope_pool, page_table, positions, c_kv_new, k_rope_new, to_bf16):
    """Stores each sequence's newest row at logical slot positions[b] (Section 2.1: both
    C^KV and K^RoPE are cached).  Values are rounded to bfloat16 first when to_bf16.
    Pools are float64 arrays holding storage values; they are modified in place."""
    P, NB, ps, d_cb = latent_pool.shape
    for b in range(len(positions)):
        pos = int(positions[b])
        if pos < 0:
            continue
        page = int(page_table[b, pos // ps])
        slot = pos % ps
        row = np.asarray(c_kv_new[b], np.float32)
        kr = np.asarray(k_rope_new[b], np.float32)
        if to_bf16:
            row, kr = round_bf16(row), round_bf16(kr)
        for blk in range(NB):
            latent_pool[page, blk, slot, :] = row[blk * d_cb:(blk + 1) * d_cb]
        rope_pool[page, slot, :] = kr
    return latent_pool, rope_pool


# --------------------------------------------------------------------------------------
# batch drivers
# --------------------------------------------------------------------------------------
def mlra_decode_batch(latent_pool, rope_pool, page_table, seq_lens, q_nope, q_rope, w_uk, w_uv,
                      tau, out_scale=1.0, seqs=None, return_lse=False):
    """Runs mlra_decode_absorbed for the listed sequences (default: all).

    w_uk / w_uv are [NB][d_cb][h*d_h]; stacking the blocks gives the paper's
    [d_c][h*d_h] matrices.  Returns O [len(seqs)][h][d_h] (and lse [len(seqs)][NB][h]).
    """
    NB = latent_pool.shape[1]
    h, d_h = q_nope.shape[1], q_nope.shape[2]
    W_UK = np.asarray(w_uk, np.float64).reshape(-1, h * d_h)
    W_UV = np.asarray(w_uv, np.float64).reshape(-1, h * d_h)
    seqs = list(range(len(seq_lens))) if seqs is None else list(seqs)
    O = np.zeros((len(seqs), h, d_h))
    L = np.zeros((len(seqs), NB, h))
    for k, b in enumerate(seqs):
        C, KR = gather_sequence(latent_pool, rope_pool, page_table[b], int(seq_lens[b]))
        O[k], L[k] = mlra_decode_absorbed(q_nope[b], q_rope[b], C, KR, W_UK, W_UV, NB, tau,
                                          out_scale, return_lse=True)
    return (O, L) if return_lse else O


def mlra_decode_multi_batch(latent_pool, rope_pool, page_table, seq_lens, q_nope, q_rope, w_uk, w_uv, tau,
                            out_scale=1.0, seqs=None):
    """q_nope [B][q_len][h][d_h], q_rope [B][q_len][h][d_r]; returns O [len(seqs)][q_len][h][d_h]."""
    NB = latent_pool.shape[1]
    q_len, h, d_h = q_nope.shape[1], q_nope.shape[2], q_nope.shape[3]
    W_UK = np.asarray(w_uk, np.float64).reshape(-1, h * d_h)
    W_UV = np.asarray(w_uv, np.float64).reshape(-1, h * d_h)
    seqs = list(range(len(seq_lens))) if seqs is None else list(seqs)
    O = np.zeros((len(seqs), q_len, h, d_h))
    for k, b in enumerate(seqs):
        C, KR = gather_sequence(latent_pool, rope_pool, page_table[b], int(seq_lens[b]))
        O[k] = mlra_decode_multi(q_nope[b], q_rope[b], C, KR, W_UK, W_UV, NB, tau, out_scale)
    return O


def mlra2_decode_batch(latent_pool, rope_pool, page_table, seq_lens, q_nope, q_rope, w_uk, w_uv,
                       tau, out_scale=1.0, seqs=None, return_lse=False):
    """Runs mlra2_decode_absorbed for the listed sequences (default: all).

    w_uk / w_uv are [4][d_cb][(h/2)*d_h]: blocks 2g and 2g+1 stacked are group g's matrix
    W^(g) of Section 2.3.  Returns O [len(seqs)][h][d_h] (and lse [len(seqs)][4][h/2]).
    """
    NB, d_cb = latent_pool.shape[1], latent_pool.shape[3]
    assert NB == 4
    h, d_h = q_nope.shape[1], q_nope.shape[2]
    W_UK_g = np.asarray(w_uk, np.float64).reshape(2, 2 * d_cb, (h // 2) * d_h)
    W_UV_g = np.asarray(w_uv, np.float64).reshape(2, 2 * d_cb, (h // 2) * d_h)
    seqs = list(range(len(seq_lens))) if seqs is None else list(seqs)
    O = np.zeros((len(seqs), h, d_h))
    L = np.zeros((len(seqs), NB, h // 2))
    for k, b in enumerate(seqs):
        C, KR = gather_sequence(latent_pool, rope_pool, page_table[b], int(seq_lens[b]))
        O[k], L[k] = mlra2_decode_absorbed(q_nope[b], q_rope[b], C, KR, W_UK_g, W_UV_g, tau,
                                           out_scale, return_lse=True)
    return (O, L) if return_lse else O


def gla2_decode_batch(latent_pool, rope_pool, page_table, seq_lens, q_nope, q_rope, w_uk, w_uv, tau, seqs=None):
    """GLA-2 on a cache of two latent heads (pool [P][2][page][d_c/2]); w_uk / w_uv [2][d_c/2][(h/2)*d_h]."""
    assert latent_pool.shape[1] == 2
    seqs = list(range(len(seq_lens))) if seqs is None else list(seqs)
    h, d_h = q_nope.shape[1], q_nope.shape[2]
    O = np.zeros((len(seqs), h, d_h))
    for k, b in enumerate(seqs):
        C, KR = gather_sequence(latent_pool, rope_pool, page_table[b], int(seq_lens[b]))
        O[k] = gla2_decode(q_nope[b], q_rope[b], C, KR, w_uk, w_uv, tau)
    return O


def gqa_decode_batch(k_pool, v_pool, page_table, seq_lens, q, scale, seqs=None):
    seqs = list(range(len(seq_lens))) if seqs is None else list(seqs)
    h, d_h = q.shape[1], q.shape[2]
    O = np.zeros((len(seqs), h, d_h))
    for k, b in enumerate(seqs):
        K, V = gather_gqa_sequence(k_pool, v_pool, page_table[b], int(seq_lens[b]))
        O[k] = gqa_decode(q[b], K, V, scale)
    return O
