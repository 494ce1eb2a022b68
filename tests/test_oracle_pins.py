"""Pins for the CPU oracle: each check compares an oracle function with something other
than itself -- the paper's Eq. (2) identity, a library attention routine on materialised
keys/values, closed forms, invariances, scalar brute force, a library bf16 cast.
All CPU, float64."""
import math

import numpy as np
import pytest
import torch

from oracle import mlra_oracle as orc


def _rand_case(seed, n, h, d_h, NB, d_cb, d_r):
    rng = np.random.default_rng(seed)
    d_c = NB * d_cb
    return dict(
        q_nope=rng.standard_normal((h, d_h)),
        q_rope=rng.standard_normal((h, d_r)),
        C=rng.standard_normal((n, d_c)),
        KR=rng.standard_normal((n, d_r)),
        W_UK=rng.standard_normal((d_c, h * d_h)) / math.sqrt(d_cb),
        W_UV=rng.standard_normal((d_c, h * d_h)) / math.sqrt(d_cb),
        tau=1.0 / math.sqrt(d_h + d_r),
    )


def _sdpa(q, K, V, scale):
    """Library attention on explicit per-head keys/values: q [h][D], K [h][n][D], V [h][n][Dv]."""
    out = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q)[None, :, None, :], torch.from_numpy(K)[None], torch.from_numpy(V)[None],
        scale=scale)
    return out[0, :, 0, :].numpy()


# ---- Eq. (2): block-sum identity -------------------------------------------------------
def test_eq2_block_sum_identity():
    n, h, d_h, NB, d_cb = 19, 5, 8, 4, 8
    c = _rand_case(1, n, h, d_h, NB, d_cb, 4)
    for W in (c["W_UK"], c["W_UV"]):
        full = c["C"] @ W                                            # [n][h*d_h]
        for i in range(h):
            blocks = sum(orc.c_block(c["C"], b, d_cb) @ orc.w_block(W, b, i, d_cb, d_h)
                         for b in range(NB))
            assert np.max(np.abs(blocks - full[:, i * d_h:(i + 1) * d_h])) <= 1e-10


# ---- absorbed == unabsorbed (associativity, Section 2.1 Steps 1-3) ----------------------
@pytest.mark.parametrize("NB", [1, 2, 4])
def test_absorbed_equals_unabsorbed(NB):
    n, h, d_h, d_cb, d_r = 37, 3, 8, 8, 4
    c = _rand_case(2 + NB, n, h, d_h, NB, d_cb, d_r)
    a = orc.mlra_decode_absorbed(c["q_nope"], c["q_rope"], c["C"], c["KR"], c["W_UK"], c["W_UV"], NB, c["tau"])
    u = orc.mlra_decode_unabsorbed(c["q_nope"], c["q_rope"], c["C"], c["KR"], c["W_UK"], c["W_UV"], NB, c["tau"])
    assert np.max(np.abs(a - u)) <= 1e-10 * max(1.0, np.max(np.abs(u)))


# ---- brute force: Eq. (5) in scalar Python loops ----------------------------------------
def test_unabsorbed_vs_scalar_loops():
    n, h, d_h, NB, d_cb, d_r = 5, 2, 3, 2, 2, 2
    c = _rand_case(11, n, h, d_h, NB, d_cb, d_r)
    C, KR, WK, WV, qn, qr, tau = (c[k] for k in ("C", "KR", "W_UK", "W_UV", "q_nope", "q_rope", "tau"))
    expect = [[0.0] * d_h for _ in range(h)]
    for i in range(h):
        for b in range(NB):
            logits = []
            for t in range(n):
                s = 0.0
                for p in range(d_h):                 # q^NoPE . (C_b W^UK_(b),(i))[t]
                    k_tp = sum(C[t][b * d_cb + cc] * WK[b * d_cb + cc][i * d_h + p] for cc in range(d_cb))
                    s += qn[i][p] * k_tp
                for u in range(d_r):                 # q^RoPE . K^RoPE[t]
                    s += qr[i][u] * KR[t][u]
                logits.append(tau * s)
            mx = max(logits)
            w = [math.exp(x - mx) for x in logits]
            tot = sum(w)
            for p in range(d_h):
                for t in range(n):
                    v_tp = sum(C[t][b * d_cb + cc] * WV[b * d_cb + cc][i * d_h + p] for cc in range(d_cb))
                    expect[i][p] += (w[t] / tot) * v_tp
    got = orc.mlra_decode_unabsorbed(qn, qr, C, KR, WK, WV, NB, tau)
    assert np.max(np.abs(got - np.array(expect))) <= 1e-12
    got_a = orc.mlra_decode_absorbed(qn, qr, C, KR, WK, WV, NB, tau)
    assert np.max(np.abs(got_a - np.array(expect))) <= 1e-12


# ---- NB = 1 is MLA is textbook attention on K = [C W^UK || K^R], V = C W^UV ---------------
def test_mla_equals_library_sdpa():
    n, h, d_h, d_c, d_r = 53, 4, 8, 32, 4
    c = _rand_case(21, n, h, d_h, 1, d_c, d_r)
    Kn = (c["C"] @ c["W_UK"]).reshape(n, h, d_h).transpose(1, 0, 2)
    V = (c["C"] @ c["W_UV"]).reshape(n, h, d_h).transpose(1, 0, 2)
    K = np.concatenate([Kn, np.broadcast_to(c["KR"][None], (h, n, d_r))], axis=2)
    q = np.concatenate([c["q_nope"], c["q_rope"]], axis=1)
    ref = _sdpa(q, np.ascontiguousarray(K), np.ascontiguousarray(V), c["tau"])
    got = orc.mla_decode(c["q_nope"], c["q_rope"], c["C"], c["KR"], c["W_UK"], c["W_UV"], c["tau"])
    assert np.max(np.abs(got - ref)) <= 1e-10


# ---- Eq. (5) with a library attention per block ------------------------------------------
@pytest.mark.parametrize("NB", [2, 4])
def test_mlra_equals_sum_of_block_sdpa(NB):
    n, h, d_h, d_cb, d_r = 41, 4, 8, 8, 4
    c = _rand_case(31 + NB, n, h, d_h, NB, d_cb, d_r)
    q = np.concatenate([c["q_nope"], c["q_rope"]], axis=1)
    ref = np.zeros((h, d_h))
    for b in range(NB):
        Cb = c["C"][:, b * d_cb:(b + 1) * d_cb]
        Kn = (Cb @ c["W_UK"][b * d_cb:(b + 1) * d_cb]).reshape(n, h, d_h).transpose(1, 0, 2)
        V = (Cb @ c["W_UV"][b * d_cb:(b + 1) * d_cb]).reshape(n, h, d_h).transpose(1, 0, 2)
        K = np.concatenate([Kn, np.broadcast_to(c["KR"][None], (h, n, d_r))], axis=2)
        ref += _sdpa(q, np.ascontiguousarray(K), np.ascontiguousarray(V), c["tau"])
    for fn in (orc.mlra_decode_absorbed, orc.mlra_decode_unabsorbed):
        got = fn(c["q_nope"], c["q_rope"], c["C"], c["KR"], c["W_UK"], c["W_UV"], NB, c["tau"])
        assert np.max(np.abs(got - ref)) <= 1e-10
    # MLRA-4 is not MLA: the softmax is taken per block.
    mla = orc.mla_decode(c["q_nope"], c["q_rope"], c["C"], c["KR"], c["W_UK"], c["W_UV"], c["tau"])
    assert np.max(np.abs(mla - ref)) > 1e-3


# ---- closed forms where every softmax is known -------------------------------------------
def test_closed_form_single_token():
    h, d_h, NB, d_cb, d_r = 3, 8, 4, 8, 4
    c = _rand_case(41, 1, h, d_h, NB, d_cb, d_r)
    expect = (c["C"] @ c["W_UV"]).reshape(h, d_h)       # softmax over one token is 1; Eq. (2)
    got = orc.mlra_decode_absorbed(c["q_nope"], c["q_rope"], c["C"], c["KR"], c["W_UK"], c["W_UV"], NB, c["tau"])
    assert np.max(np.abs(got - expect)) <= 1e-12
    mla = orc.mla_decode(c["q_nope"], c["q_rope"], c["C"], c["KR"], c["W_UK"], c["W_UV"], c["tau"])
    assert np.max(np.abs(mla - expect)) <= 1e-12


def test_closed_form_zero_queries_gives_mean():
    n, h, d_h, NB, d_cb, d_r = 29, 3, 8, 4, 8, 4
    c = _rand_case(42, n, h, d_h, NB, d_cb, d_r)
    z = np.zeros_like
    expect = (c["C"].mean(axis=0) @ c["W_UV"]).reshape(h, d_h)
    got, lse = orc.mlra_decode_absorbed(z(c["q_nope"]), z(c["q_rope"]), c["C"], c["KR"], c["W_UK"], c["W_UV"],
                                        NB, c["tau"], return_lse=True)
    assert np.max(np.abs(got - expect)) <= 1e-12
    assert np.max(np.abs(lse - math.log(n))) <= 1e-12      # log sum_t exp(0)


def test_closed_form_constant_cache():
    n, h, d_h, NB, d_cb, d_r = 17, 2, 8, 4, 8, 4
    c = _rand_case(43, n, h, d_h, NB, d_cb, d_r)
    C = np.broadcast_to(c["C"][:1], c["C"].shape).copy()
    expect = (C[0] @ c["W_UV"]).reshape(h, d_h)           # any weights average equal rows
    got = orc.mlra_decode_absorbed(c["q_nope"], c["q_rope"], C, c["KR"], c["W_UK"], c["W_UV"], NB, c["tau"])
    assert np.max(np.abs(got - expect)) <= 1e-12


def test_closed_form_two_tokens_sigmoid():
    """One head, one channel everywhere: the two-token softmax is a logistic function."""
    qn, qr = 0.7, -1.3
    C = np.array([[0.5, -2.0], [1.5, 0.25]])               # n = 2, two blocks of one channel
    KR = np.array([[0.3], [-0.9]])
    WK = np.array([[1.1], [-0.6]])                          # d_c x (h d_h) = 2 x 1
    WV = np.array([[0.8], [2.0]])
    tau = 1.0 / math.sqrt(1 + 1)
    expect = 0.0
    for b in range(2):
        s0 = tau * (qn * C[0, b] * WK[b, 0] + qr * KR[0, 0])
        s1 = tau * (qn * C[1, b] * WK[b, 0] + qr * KR[1, 0])
        p1 = 1.0 / (1.0 + math.exp(s0 - s1))
        expect += ((1 - p1) * C[0, b] + p1 * C[1, b]) * WV[b, 0]
    for fn in (orc.mlra_decode_absorbed, orc.mlra_decode_unabsorbed):
        got = fn(np.array([[qn]]), np.array([[qr]]), C, KR, WK, WV, 2, tau)
        assert abs(got[0, 0] - expect) <= 1e-14
    half = orc.mlra_decode_absorbed(np.array([[qn]]), np.array([[qr]]), C, KR, WK, WV, 2, tau, out_scale=0.5)
    assert abs(half[0, 0] - 0.5 * expect) <= 1e-14       # Eq. (10), alpha_attn = 1/2


def test_rope_term_and_scale_matter():
    """Dropping the RoPE score, using 1/sqrt(d_h) or skipping tau must change the result
    (guards the checks above against being insensitive to those terms)."""
    n, h, d_h, NB, d_cb, d_r = 23, 2, 8, 4, 8, 4
    c = _rand_case(44, n, h, d_h, NB, d_cb, d_r)
    args = (c["C"], c["KR"], c["W_UK"], c["W_UV"], NB)
    base = orc.mlra_decode_absorbed(c["q_nope"], c["q_rope"], *args, c["tau"])
    no_rope = orc.mlra_decode_absorbed(c["q_nope"], 0 * c["q_rope"], *args, c["tau"])
    other_scale = orc.mlra_decode_absorbed(c["q_nope"], c["q_rope"], *args, 1 / math.sqrt(d_h))
    assert np.max(np.abs(base - no_rope)) > 1e-3
    assert np.max(np.abs(base - other_scale)) > 1e-4


def test_tau_values():
    from paper_2603_02188_amd.inputs import WORKLOADS
    assert abs(WORKLOADS["C1"].tau - 0.10206207261596575) < 1e-15      # 1/sqrt(64+32)
    for k in ("C2", "C3", "C4", "C5"):
        assert abs(WORKLOADS[k].tau - 0.07216878364870323) < 1e-15    # 1/sqrt(128+64)


# ---- split / merge invariance of Step 2 (pins lse as well) --------------------------------
def test_split_merge_invariance():
    n, h, d_cb, d_r = 101, 3, 8, 4
    rng = np.random.default_rng(51)
    qa, qr = rng.standard_normal((h, d_cb)), rng.standard_normal((h, d_r))
    Cb, KR = rng.standard_normal((n, d_cb)), rng.standard_normal((n, d_r))
    tau = 0.3
    Z, lse = orc.latent_attention(qa, qr, Cb, KR, tau)
    cuts = [0, 7, 7, 40, 100, 101]                        # includes an empty part
    parts = [orc.latent_attention(qa, qr, Cb[a:b], KR[a:b], tau) for a, b in zip(cuts[:-1], cuts[1:])]
    lses = np.stack([p[1] for p in parts])                 # [parts][h]
    m = lses.max(axis=0)
    w = np.exp(lses - m)                                   # empty part: exp(-inf) = 0
    merged = sum(w[k][:, None] * parts[k][0] for k in range(len(parts))) / w.sum(axis=0)[:, None]
    assert np.max(np.abs(merged - Z)) <= 1e-12
    assert np.max(np.abs(m + np.log(w.sum(axis=0)) - lse)) <= 1e-12


def test_lse_matches_scipy_logsumexp():
    from scipy.special import logsumexp
    n, h, d_cb, d_r = 33, 2, 8, 4
    rng = np.random.default_rng(52)
    qa, qr = rng.standard_normal((h, d_cb)), rng.standard_normal((h, d_r))
    Cb, KR = rng.standard_normal((n, d_cb)), rng.standard_normal((n, d_r))
    _, lse = orc.latent_attention(qa, qr, Cb, KR, 0.25)
    S = 0.25 * (np.concatenate([qa, qr], 1) @ np.concatenate([Cb, KR], 1).T)
    assert np.max(np.abs(lse - logsumexp(S, axis=1))) <= 1e-12


def test_empty_context():
    h, d_h, NB, d_cb, d_r = 2, 8, 4, 8, 4
    c = _rand_case(53, 0, h, d_h, NB, d_cb, d_r)
    got, lse = orc.mlra_decode_absorbed(c["q_nope"], c["q_rope"], c["C"], c["KR"], c["W_UK"], c["W_UV"],
                                        NB, c["tau"], return_lse=True)
    assert np.all(got == 0) and np.all(np.isneginf(lse))
    assert np.all(orc.mlra_decode_unabsorbed(c["q_nope"], c["q_rope"], c["C"], c["KR"], c["W_UK"],
                                             c["W_UV"], NB, c["tau"]) == 0)


# ---- the kernel never sees positions: row permutations and page tables ---------------------
def test_token_permutation_invariance():
    n, h, d_h, NB, d_cb, d_r = 31, 3, 8, 4, 8, 4
    c = _rand_case(61, n, h, d_h, NB, d_cb, d_r)
    perm = np.random.default_rng(62).permutation(n)
    a = orc.mlra_decode_absorbed(c["q_nope"], c["q_rope"], c["C"], c["KR"], c["W_UK"], c["W_UV"], NB, c["tau"])
    b = orc.mlra_decode_absorbed(c["q_nope"], c["q_rope"], c["C"][perm], c["KR"][perm], c["W_UK"], c["W_UV"],
                                 NB, c["tau"])
    assert np.max(np.abs(a - b)) <= 1e-12


def test_paged_gather_matches_contiguous_rows():
    """gather_sequence on a shuffled page table returns exactly the rows that were drawn."""
    from paper_2603_02188_amd import inputs as gen
    wl = gen.WORKLOADS["C5"].scaled(batch=3, n_min=1, n_max=200, h=2, d_h=8, d_cb=8, d_r=4, page_size=16)
    inp = gen.make_decode_inputs(wl, poison=True)
    lat = gen.to_f64(inp.latent_pool, wl.dtype)
    rope = gen.to_f64(inp.rope_pool, wl.dtype)
    for b in range(wl.batch):
        n = int(inp.seq_lens[b])
        C, KR = orc.gather_sequence(lat, rope, inp.page_table[b], n)
        rows, rrows = gen.draw_sequence_rows(wl, b, n)
        assert np.array_equal(C, gen.to_f64(gen.to_storage(rows, wl.dtype), wl.dtype))
        assert np.array_equal(KR, gen.to_f64(gen.to_storage(rrows, wl.dtype), wl.dtype))
        assert not np.isnan(C).any() and not np.isnan(KR).any()


def test_append_kv_fills_the_hole():
    from paper_2603_02188_amd import inputs as gen
    wl = gen.WORKLOADS["C5"].scaled(batch=4, n_min=1, n_max=90, h=2, d_h=8, d_cb=8, d_r=4, page_size=16)
    full = gen.make_decode_inputs(wl, poison=True, hole=False)
    holed = gen.make_decode_inputs(wl, poison=True, hole=True)
    lat, rope = gen.to_f64(holed.latent_pool, wl.dtype), gen.to_f64(holed.rope_pool, wl.dtype)
    assert np.isnan(lat).sum() > np.isnan(gen.to_f64(full.latent_pool, wl.dtype)).sum()
    orc.append_kv(lat, rope, holed.page_table, holed.positions, holed.c_kv_new, holed.k_rope_new, to_bf16=True)
    assert np.array_equal(lat, gen.to_f64(full.latent_pool, wl.dtype), equal_nan=True)
    assert np.array_equal(rope, gen.to_f64(full.rope_pool, wl.dtype), equal_nan=True)


# ---- GQA (Appendix C) ---------------------------------------------------------------------
@pytest.mark.parametrize("g", [1, 2, 8])
def test_gqa_equals_mha_after_repeat_interleave(g):
    n, h, d_h = 47, 8, 16
    rng = np.random.default_rng(70 + g)
    q = rng.standard_normal((h, d_h))
    K, V = rng.standard_normal((n, g, d_h)), rng.standard_normal((n, g, d_h))
    scale = 1 / math.sqrt(d_h)
    Kr = np.repeat(K, h // g, axis=1).transpose(1, 0, 2)      # RepeatInterleave along heads
    Vr = np.repeat(V, h // g, axis=1).transpose(1, 0, 2)
    ref = _sdpa(q, np.ascontiguousarray(Kr), np.ascontiguousarray(Vr), scale)
    assert np.max(np.abs(orc.gqa_decode(q, K, V, scale) - ref)) <= 1e-12


def test_gqa_paged_gather():
    from paper_2603_02188_amd import inputs as gen
    wl = gen.WORKLOADS["C5"].scaled(batch=2, n_min=1, n_max=70, h=4, d_h=8, g=2, page_size=16)
    gi = gen.make_gqa_inputs(wl)
    k, v = gen.to_f64(gi.k_pool, wl.dtype), gen.to_f64(gi.v_pool, wl.dtype)
    for b in range(wl.batch):
        n = int(gi.seq_lens[b])
        K, V = orc.gather_gqa_sequence(k, v, gi.page_table[b], n)
        assert K.shape == (n, 2, 8) and not np.isnan(K).any() and not np.isnan(V).any()
        # slot t of KV head j lives at pool[page][j][t % page][:]
        t = n - 1
        page = gi.page_table[b, t // 16]
        assert np.array_equal(K[t, 1], k[page, 1, t % 16]) and np.array_equal(V[t, 0], v[page, 0, t % 16])


# ---- bf16 rounding ---------------------------------------------------------------------
def test_round_bf16_hand_cases():
    cases = {
        1.0: 1.0,
        1.0 + 2.0 ** -8: 1.0,                        # tie, even mantissa stays
        1.0 + 2.0 ** -7 + 2.0 ** -8: 1.0 + 2.0 ** -6,  # tie, odd mantissa rounds up
        1.0 + 2.0 ** -8 + 2.0 ** -20: 1.0 + 2.0 ** -7,  # just above the tie
        -(1.0 + 2.0 ** -8 + 2.0 ** -20): -(1.0 + 2.0 ** -7),
        0.0: 0.0,
        257.0: 256.0,                                  # 8 significant bits: tie to even
        259.0: 260.0,                                  # tie, odd neighbour rounds away
        -0.3: -0.30078125,                             # 0.3 = 1.0011001|1001...b x 2^-2 rounds up
    }
    for x, want in cases.items():
        got = float(orc.round_bf16(np.float32(x)))
        assert got == want, (x, got, want)


def test_round_bf16_matches_library_cast():
    from paper_2603_02188_amd import inputs as gen
    x = np.random.default_rng(81).standard_normal(20000).astype(np.float32) * 37.0
    lib = torch.from_numpy(x).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(orc.round_bf16(x), lib)
    assert np.array_equal(gen.bf16_bits_to_f32(gen.f32_to_bf16_bits(x)).astype(np.float64), lib)


# ---- mutation guard: the pins above must notice plausible mistakes ---------------------------
def test_pins_detect_planted_mistakes(monkeypatch):
    n, h, d_h, NB, d_cb, d_r = 13, 3, 8, 4, 8, 4
    c = _rand_case(91, n, h, d_h, NB, d_cb, d_r)
    good = orc.mlra_decode_unabsorbed(c["q_nope"], c["q_rope"], c["C"], c["KR"], c["W_UK"], c["W_UV"], NB, c["tau"])

    def run():
        return orc.mlra_decode_absorbed(c["q_nope"], c["q_rope"], c["C"], c["KR"], c["W_UK"], c["W_UV"], NB, c["tau"])

    real_absorb, real_up, real_att = orc.absorb_q, orc.up_project, orc.latent_attention
    mistakes = {
        "absorb uses a neighbouring head's columns":
            ("absorb_q", lambda q, W, nb: np.roll(real_absorb(q, W, nb), 1, axis=1)),
        "blocks swapped in the up-projection":
            ("up_project", lambda Z, W, hh, dd: real_up(Z, W[::-1], hh, dd)),
        "rope score dropped":
            ("latent_attention", lambda qa, qr, Cb, KR, tau: real_att(qa, 0 * qr, Cb, KR, tau)),
        "scale applied to the latent term only":
            ("latent_attention", lambda qa, qr, Cb, KR, tau: real_att(qa, qr / tau, Cb, KR, tau)),
    }
    assert np.max(np.abs(run() - good)) <= 1e-10
    for why, (name, bad) in mistakes.items():
        monkeypatch.setattr(orc, name, bad)
        assert np.max(np.abs(run() - good)) > 1e-4, why
        monkeypatch.undo()


# =========================================================================================
# MLRA-2 (Eq. (6)): group map gamma(i), group matrices W^(gamma) of Section 2.3
# =========================================================================================
def _rand_case2(seed, n, h, d_h, d_cb, d_r):
    rng = np.random.default_rng(seed)
    return dict(
        q_nope=rng.standard_normal((h, d_h)),
        q_rope=rng.standard_normal((h, d_r)),
        C=rng.standard_normal((n, 4 * d_cb)),
        KR=rng.standard_normal((n, d_r)),
        W_UK_g=rng.standard_normal((2, 2 * d_cb, (h // 2) * d_h)) / math.sqrt(d_cb),
        W_UV_g=rng.standard_normal((2, 2 * d_cb, (h // 2) * d_h)) / math.sqrt(d_cb),
        tau=1.0 / math.sqrt(d_h + d_r),
    )


def _m2_args(c):
    return (c["q_nope"], c["q_rope"], c["C"], c["KR"], c["W_UK_g"], c["W_UV_g"], c["tau"])


def test_mlra2_unabsorbed_vs_scalar_loops():
    """Eq. (6) written out with scalar sums: head i uses latent blocks 2 gamma(i) and 2 gamma(i) + 1, rows
    j d_cb.. of its group's matrices, columns i_bar d_h.. ."""
    n, h, d_h, d_cb, d_r = 4, 4, 3, 2, 2
    c = _rand_case2(61, n, h, d_h, d_cb, d_r)
    qn, qr, C, KR, WK, WV, tau = _m2_args(c)
    expect = [[0.0] * d_h for _ in range(h)]
    for i in range(h):
        grp = 0 if i < h // 2 else 1
        ib = i - grp * (h // 2)
        for j in range(2):
            blk = 2 * grp + j
            logits = []
            for t in range(n):
                s = 0.0
                for p in range(d_h):
                    k_tp = sum(C[t][blk * d_cb + cc] * WK[grp][j * d_cb + cc][ib * d_h + p] for cc in range(d_cb))
                    s += qn[i][p] * k_tp
                for u in range(d_r):
                    s += qr[i][u] * KR[t][u]
                logits.append(tau * s)
            mx = max(logits)
            w = [math.exp(x - mx) for x in logits]
            tot = sum(w)
            for p in range(d_h):
                for t in range(n):
                    v_tp = sum(C[t][blk * d_cb + cc] * WV[grp][j * d_cb + cc][ib * d_h + p] for cc in range(d_cb))
                    expect[i][p] += w[t] / tot * v_tp
    got = orc.mlra2_decode_unabsorbed(*_m2_args(c))
    assert np.max(np.abs(got - np.array(expect))) <= 1e-12


def test_mlra2_absorbed_equals_unabsorbed():
    c = _rand_case2(62, 29, 6, 8, 8, 4)
    a, lse = orc.mlra2_decode_absorbed(*_m2_args(c), return_lse=True)
    u = orc.mlra2_decode_unabsorbed(*_m2_args(c))
    assert np.max(np.abs(a - u)) <= 1e-10 * max(1.0, np.max(np.abs(u)))
    assert lse.shape == (4, 3) and np.all(np.isfinite(lse))


def test_mlra2_single_token_is_the_gla2_value():
    """n = 1: every softmax is 1, so O_i = C_(2g) W^(g),UV_(0),(i) + C_(2g+1) W^(g),UV_(1),(i), which by
    Eq. (4) is GLA-2's value row [C_(2g), C_(2g+1)] W^(g),UV_(:),(i)."""
    h, d_h, d_cb, d_r = 6, 5, 4, 2
    c = _rand_case2(63, 1, h, d_h, d_cb, d_r)
    got = orc.mlra2_decode_unabsorbed(*_m2_args(c))
    for i in range(h):
        grp = i // (h // 2)
        ib = i % (h // 2)
        latent_g = c["C"][0, 2 * grp * d_cb:(2 * grp + 2) * d_cb]                     # [2 d_cb]
        v = latent_g @ c["W_UV_g"][grp][:, ib * d_h:(ib + 1) * d_h]
        assert np.max(np.abs(got[i] - v)) <= 1e-12


def test_mlra2_branches_against_library_sdpa():
    """Each branch is ordinary attention with keys [C_b W^UK | K^RoPE] and values C_b W^UV (Eq. (6))."""
    n, h, d_h, d_cb, d_r = 23, 4, 8, 8, 4
    c = _rand_case2(64, n, h, d_h, d_cb, d_r)
    q = np.concatenate([c["q_nope"], c["q_rope"]], axis=1)                            # [h][d_h + d_r]
    total = np.zeros((h, d_h))
    for j in range(2):
        K = np.zeros((h, n, d_h + d_r))
        V = np.zeros((h, n, d_h))
        for i in range(h):
            grp, ib = i // (h // 2), i % (h // 2)
            C_b = c["C"][:, (2 * grp + j) * d_cb:(2 * grp + j + 1) * d_cb]
            K[i, :, :d_h] = C_b @ c["W_UK_g"][grp][j * d_cb:(j + 1) * d_cb, ib * d_h:(ib + 1) * d_h]
            K[i, :, d_h:] = c["KR"]
            V[i] = C_b @ c["W_UV_g"][grp][j * d_cb:(j + 1) * d_cb, ib * d_h:(ib + 1) * d_h]
        total += _sdpa(q, K, V, c["tau"])
    got = orc.mlra2_decode_unabsorbed(*_m2_args(c), out_scale=0.5)
    assert np.max(np.abs(got - 0.5 * total)) <= 1e-10


def test_mlra2_groups_do_not_interact():
    """Heads of group 0 never see blocks 2, 3 or group 1's matrices, and vice versa."""
    c = _rand_case2(65, 17, 4, 4, 4, 2)
    base = orc.mlra2_decode_absorbed(*_m2_args(c))
    d = dict(c)
    d["C"] = c["C"].copy()
    d["C"][:, 2 * 4:] = 7.0                                   # blocks 2 and 3
    d["W_UK_g"] = c["W_UK_g"].copy(); d["W_UK_g"][1] *= -3.0
    d["W_UV_g"] = c["W_UV_g"].copy(); d["W_UV_g"][1] += 1.0
    other = orc.mlra2_decode_absorbed(*_m2_args(d))
    assert np.array_equal(base[:2], other[:2])
    assert not np.allclose(base[2:], other[2:])


def test_mlra2_reduces_to_two_block_mlra_per_group():
    """Group g alone is Eq. (5) with two branches: heads of the group, blocks 2g and 2g+1, W^(g)."""
    n, h, d_h, d_cb, d_r = 13, 6, 4, 4, 2
    c = _rand_case2(66, n, h, d_h, d_cb, d_r)
    got = orc.mlra2_decode_absorbed(*_m2_args(c))
    hg = h // 2
    for grp in range(2):
        sub = orc.mlra_decode_unabsorbed(c["q_nope"][grp * hg:(grp + 1) * hg], c["q_rope"][grp * hg:(grp + 1) * hg],
                                         c["C"][:, 2 * grp * d_cb:(2 * grp + 2) * d_cb], c["KR"],
                                         c["W_UK_g"][grp], c["W_UV_g"][grp], 2, c["tau"])
        assert np.max(np.abs(got[grp * hg:(grp + 1) * hg] - sub)) <= 1e-10


def test_mlra2_zero_query_gives_the_mean_value_and_empty_context_zero():
    n, h, d_h, d_cb, d_r = 9, 4, 3, 4, 2
    c = _rand_case2(67, n, h, d_h, d_cb, d_r)
    c["q_nope"][:] = 0.0
    c["q_rope"][:] = 0.0
    got = orc.mlra2_decode_absorbed(*_m2_args(c))
    for i in range(h):
        grp, ib = i // (h // 2), i % (h // 2)
        mean_latent = c["C"][:, 2 * grp * d_cb:(2 * grp + 2) * d_cb].mean(axis=0)
        assert np.max(np.abs(got[i] - mean_latent @ c["W_UV_g"][grp][:, ib * d_h:(ib + 1) * d_h])) <= 1e-12
    e = dict(c); e["C"] = c["C"][:0]; e["KR"] = c["KR"][:0]
    out, lse = orc.mlra2_decode_absorbed(*_m2_args(e), return_lse=True)
    assert np.all(out == 0.0) and np.all(np.isneginf(lse))


# =========================================================================================
# Pre-attention of the new token: RMSNorm, RoPE, projections (Section 2.1, Appendix B, Eq. (9))
# =========================================================================================
def test_rope_matches_the_complex_form_of_the_papers_theorem():
    """<RoPE(q, tq), RoPE(k, tk)> = Re sum_l q_l conj(k_l) e^{i (tq - tk) theta_l} with q_l = q[2l] + i q[2l+1]
    (proof of the RoPE theorem in Appendix B), hence translation invariance."""
    rng = np.random.default_rng(71)
    d_r, base = 16, 10000.0
    q, k = rng.standard_normal(d_r), rng.standard_normal(d_r)
    theta = base ** (-2.0 * np.arange(d_r // 2) / d_r)
    qc, kc = q[0::2] + 1j * q[1::2], k[0::2] + 1j * k[1::2]
    for tq, tk in [(0, 0), (5, 2), (1000, 993), (17, 4000)]:
        lhs = float(orc.rope(q, tq, base) @ orc.rope(k, tk, base))
        rhs = float(np.real(np.sum(qc * np.conj(kc) * np.exp(1j * (tq - tk) * theta))))
        assert abs(lhs - rhs) <= 1e-9
        shifted = float(orc.rope(q, tq + 321, base) @ orc.rope(k, tk + 321, base))
        assert abs(lhs - shifted) <= 1e-9
    # position 0 is the identity, the rotation preserves the norm, and blocks do not mix
    assert np.array_equal(orc.rope(q, 0, base), q)
    assert abs(np.linalg.norm(orc.rope(q, 77, base)) - np.linalg.norm(q)) <= 1e-12
    e0 = np.zeros(d_r); e0[0] = 1.0
    r = orc.rope(e0, 3, base)
    assert abs(r[0] - math.cos(3.0)) <= 1e-12 and abs(r[1] - math.sin(3.0)) <= 1e-12 and np.all(r[2:] == 0.0)


def test_rope_frequencies_hand_values_and_read_back_angles():
    """The frequency law theta_l = base^(-2l/d_r) (the usual reading; the paper leaves the constants open)
    pinned by hand-computed values, not by its own expression: base 100 makes every frequency a power of
    sqrt(10).  The angles are also read back from rope() itself: unit vector e_{2l} at t = 1 is rotated
    to (cos theta_l, sin theta_l) in its 2-D block, so atan2 recovers theta_l, and consecutive
    frequencies keep the constant ratio base^(-2/d_r)."""
    # d_r = 4: theta = 100^0, 100^(-1/2);  d_r = 8: 100^0, 100^(-1/4), 100^(-1/2), 100^(-3/4)
    hand = {4: [1.0, 0.1], 8: [1.0, 0.31622776601683794, 0.1, 0.031622776601683794]}
    for d_r, want in hand.items():
        got = orc.rope_angles(d_r, 100.0)
        assert got.shape == (d_r // 2,)
        assert np.max(np.abs(got - np.array(want))) <= 1e-15
        for l in range(d_r // 2):
            e = np.zeros(d_r); e[2 * l] = 1.0
            r = orc.rope(e, 1, 100.0)
            assert abs(math.atan2(r[2 * l + 1], r[2 * l]) - want[l]) <= 1e-15      # the angle of block l at t = 1
            assert np.all(np.delete(r, [2 * l, 2 * l + 1]) == 0.0)                 # nothing leaks into other blocks
            e = np.zeros(d_r); e[2 * l + 1] = 1.0                                   # second axis of the block: +90 degrees
            r = orc.rope(e, 1, 100.0)
            assert abs(math.atan2(-r[2 * l], r[2 * l + 1]) - want[l]) <= 1e-15
    # the default base 10000 at d_r = 64 (the benchmark shape): first, middle and last frequency by hand:
    # 10000^0, 10000^(-32/64) = 0.01, 10000^(-62/64) = 10^(-3.875)
    th = orc.rope_angles(64, 10000.0)
    assert th[0] == 1.0 and abs(th[16] - 0.01) <= 1e-17 and abs(th[31] - 1.3335214321633240e-4) <= 1e-18
    ratios = th[1:] / th[:-1]
    assert np.max(np.abs(ratios - 0.74989420933245582)) <= 1e-14                    # 10^(-1/8), constant
    # angles add up over positions: t = 7 is seven times the t = 1 rotation (read back below one turn)
    e = np.zeros(8); e[2] = 1.0
    r = orc.rope(e, 7, 100.0)
    assert abs(math.atan2(r[3], r[2]) - 7 * 0.31622776601683794) <= 1e-14


def test_rms_norm_against_library_and_invariants():
    rng = np.random.default_rng(72)
    x = rng.standard_normal((5, 48)) * 3.0
    g = rng.standard_normal(48)
    lib = torch.nn.functional.rms_norm(torch.from_numpy(x), (48,), torch.from_numpy(g), eps=1e-6).numpy()
    assert np.max(np.abs(orc.rms_norm(x, g, 1e-6) - lib)) <= 1e-12
    y = orc.rms_norm(x)
    assert np.max(np.abs(np.sqrt(np.mean(y * y, axis=-1)) - 1.0)) <= 1e-12          # unit RMS
    assert np.max(np.abs(orc.rms_norm(7.5 * x) - y)) <= 1e-12                       # scale invariance


def test_pre_attention_scalar_loops_and_scaling():
    """The MLA projections of Appendix C (subsection "Multi-Head Latent Attention (MLA)") written out with scalar sums on a tiny case; alpha factors are those of Eq. (9)."""
    rng = np.random.default_rng(73)
    d, d_cq, d_c, d_r, h, d_h = 6, 4, 8, 4, 2, 3
    x = rng.standard_normal(d)
    W_DQ, W_DKV, W_KR = rng.standard_normal((d, d_cq)), rng.standard_normal((d, d_c)), rng.standard_normal((d, d_r))
    W_UQ, W_QR = rng.standard_normal((d_cq, h * d_h)), rng.standard_normal((d_cq, h * d_r))
    a_q, a_kv, t, base = math.sqrt(d / d_cq), math.sqrt(4 * d / d_c), 9, 100.0
    c_kv, k_rope, q_nope, q_rope = orc.pre_attention(x, t, W_DQ, W_DKV, W_KR, W_UQ, W_QR, h, a_q, a_kv,
                                                     rope_base=base)
    def down(W, n):
        return [sum(x[i] * W[i][j] for i in range(d)) for j in range(n)]
    def norm(v):
        ms = sum(e * e for e in v) / len(v)
        return [e / math.sqrt(ms) for e in v]
    def rot(v):
        out = list(v)
        for l in range(len(v) // 2):
            th = t * base ** (-2.0 * l / len(v))
            out[2 * l] = v[2 * l] * math.cos(th) - v[2 * l + 1] * math.sin(th)
            out[2 * l + 1] = v[2 * l] * math.sin(th) + v[2 * l + 1] * math.cos(th)
        return out
    cq = [a_q * e for e in norm(down(W_DQ, d_cq))]
    assert np.max(np.abs(c_kv - np.array([a_kv * e for e in norm(down(W_DKV, d_c))]))) <= 1e-12
    assert np.max(np.abs(k_rope - np.array(rot(down(W_KR, d_r))))) <= 1e-12
    for i in range(h):
        qn = [sum(cq[c] * W_UQ[c][i * d_h + p] for c in range(d_cq)) for p in range(d_h)]
        qr = rot([sum(cq[c] * W_QR[c][i * d_r + u] for c in range(d_cq)) for u in range(d_r)])
        assert np.max(np.abs(q_nope[i] - np.array(qn))) <= 1e-12
        assert np.max(np.abs(q_rope[i] - np.array(qr))) <= 1e-12
    # after the Eq. (9) scaling the latents have RMS alpha (unit-RMS RMSNorm output times alpha)
    assert abs(np.sqrt(np.mean(c_kv * c_kv)) - a_kv) <= 1e-12


def test_pre_attention_scores_depend_on_relative_position_only():
    """The RoPE part of the logit between a query made at position tq and a key made at position tk
    depends on tq - tk only (semi-translation equivariance: the remark that closes the MLA subsection of Appendix C, by the RoPE theorem of Appendix B)."""
    rng = np.random.default_rng(74)
    d, d_cq, d_c, d_r, h, d_h = 12, 6, 8, 8, 3, 4
    Ws = [rng.standard_normal(s) for s in ((d, d_cq), (d, d_c), (d, d_r), (d_cq, h * d_h), (d_cq, h * d_r))]
    xq, xk = rng.standard_normal(d), rng.standard_normal(d)
    def logit(tq, tk):
        _, _, _, q_rope = orc.pre_attention(xq, tq, *Ws, h, 1.3, 0.7)
        _, k_rope, _, _ = orc.pre_attention(xk, tk, *Ws, h, 1.3, 0.7)
        return q_rope @ k_rope
    assert np.max(np.abs(logit(40, 33) - logit(1040, 1033))) <= 1e-9
    assert np.max(np.abs(logit(40, 33) - logit(41, 33))) > 1e-6


# =========================================================================================
# Several query tokens per sequence (the causal tail of Eq. (5))
# =========================================================================================
def test_multi_token_decode_against_causal_library_sdpa():
    """The last q_len rows of causal attention over all n rows, per block, with keys [C_b W^UK | K^RoPE] and
    values C_b W^UV, computed by the library routine with an explicit lower-triangular mask."""
    n, q_len, h, d_h, NB, d_cb, d_r = 21, 4, 3, 8, 4, 8, 4
    c = _rand_case(81, n, h, d_h, NB, d_cb, d_r)
    rng = np.random.default_rng(82)
    qn, qr = rng.standard_normal((q_len, h, d_h)), rng.standard_normal((q_len, h, d_r))
    got = orc.mlra_decode_multi(qn, qr, c["C"], c["KR"], c["W_UK"], c["W_UV"], NB, c["tau"])
    mask = torch.zeros(q_len, n, dtype=torch.bool)
    for j in range(q_len):
        mask[j, :n - q_len + j + 1] = True
    total = np.zeros((q_len, h, d_h))
    for b in range(NB):
        K = np.zeros((h, n, d_h + d_r)); V = np.zeros((h, n, d_h))
        for i in range(h):
            C_b = c["C"][:, b * d_cb:(b + 1) * d_cb]
            K[i, :, :d_h] = C_b @ c["W_UK"][b * d_cb:(b + 1) * d_cb, i * d_h:(i + 1) * d_h]
            K[i, :, d_h:] = c["KR"]
            V[i] = C_b @ c["W_UV"][b * d_cb:(b + 1) * d_cb, i * d_h:(i + 1) * d_h]
        q = np.concatenate([qn, qr], axis=2).transpose(1, 0, 2)                      # [h][q_len][D]
        out = torch.nn.functional.scaled_dot_product_attention(
            torch.from_numpy(q)[None], torch.from_numpy(K)[None], torch.from_numpy(V)[None],
            attn_mask=mask, scale=c["tau"])[0].numpy()                               # [h][q_len][d_h]
        total += out.transpose(1, 0, 2)
    assert np.max(np.abs(got - total)) <= 1e-10


def test_multi_token_decode_causality_and_single_token_case():
    n, q_len, h, d_h, NB, d_cb, d_r = 12, 3, 2, 4, 2, 4, 2
    c = _rand_case(83, n, h, d_h, NB, d_cb, d_r)
    rng = np.random.default_rng(84)
    qn, qr = rng.standard_normal((q_len, h, d_h)), rng.standard_normal((q_len, h, d_r))
    args = (c["W_UK"], c["W_UV"], NB, c["tau"])
    base = orc.mlra_decode_multi(qn, qr, c["C"], c["KR"], *args)
    # the last query is the ordinary decode query
    assert np.array_equal(base[-1], orc.mlra_decode_absorbed(qn[-1], qr[-1], c["C"], c["KR"], *args))
    # changing the newest row changes only the newest query's output
    C2, KR2 = c["C"].copy(), c["KR"].copy()
    C2[-1] += 5.0; KR2[-1] -= 3.0
    other = orc.mlra_decode_multi(qn, qr, C2, KR2, *args)
    assert np.array_equal(base[:-1], other[:-1]) and not np.allclose(base[-1], other[-1])
    # fewer cached rows than queries: the queries without a prefix give zeros
    short = orc.mlra_decode_multi(qn, qr, c["C"][:2], c["KR"][:2], *args)
    assert np.all(short[0] == 0.0) and np.any(short[1] != 0.0)
    assert np.array_equal(short[1], orc.mlra_decode_absorbed(qn[1], qr[1], c["C"][:1], c["KR"][:1], *args))


def test_gated_output_is_the_elementwise_product():
    """Appendix E: the gate multiplies the attention output element by element.  Pinned by hand values, by
    the cases that have closed forms (all-ones gate, zero gate, one-hot gate, sigmoid of zero), by
    linearity in each argument, and by a library product; a matrix product or a broadcast over the wrong
    axis fails the one-hot and the shape cases."""
    got = orc.gated_output([[2.0, -3.0, 0.5], [4.0, 8.0, -1.0]], [[0.5, 0.25, 1.0], [0.0, 0.125, 2.0]])
    assert np.array_equal(got, np.array([[1.0, -0.75, 0.5], [0.0, 1.0, -2.0]]))
    rng = np.random.default_rng(91)
    O, G = rng.standard_normal((3, 4)), 1.0 / (1.0 + np.exp(-rng.standard_normal((3, 4))))
    assert np.array_equal(orc.gated_output(O, np.ones_like(O)), O)
    assert np.all(orc.gated_output(O, np.zeros_like(O)) == 0.0)
    assert np.array_equal(orc.gated_output(O, np.full_like(O, 0.5)), 0.5 * O)      # sigma(0) = 1/2 everywhere
    onehot = np.zeros_like(O); onehot[1, 2] = 1.0
    picked = orc.gated_output(O, onehot)
    assert picked[1, 2] == O[1, 2] and np.count_nonzero(picked) == 1                # (head 1, channel 2) only
    G2 = rng.standard_normal((3, 4))
    assert np.max(np.abs(orc.gated_output(O, G + G2) - orc.gated_output(O, G) - orc.gated_output(O, G2))) <= 1e-15
    assert np.max(np.abs(orc.gated_output(O + G2, G) - orc.gated_output(O, G) - orc.gated_output(G2, G))) <= 1e-15
    lib = torch.mul(torch.from_numpy(O), torch.from_numpy(G)).numpy()
    assert np.array_equal(orc.gated_output(O, G), lib)
    assert orc.gated_output(O, G).shape == (3, 4)


def test_gla2_against_library_sdpa_on_materialised_keys_and_values():
    """Eq. (3)-(4): K_i = [C_(2g), C_(2g+1)] W^(g),UK_:,(i) and V_i likewise; plain attention on them."""
    rng = np.random.default_rng(92)
    n, h, d_h, d_g, d_r = 19, 4, 8, 16, 4
    qn, qr = rng.standard_normal((h, d_h)), rng.standard_normal((h, d_r))
    C, KR = rng.standard_normal((n, 2 * d_g)), rng.standard_normal((n, d_r))
    WK, WV = rng.standard_normal((2, d_g, (h // 2) * d_h)), rng.standard_normal((2, d_g, (h // 2) * d_h))
    tau = 1.0 / math.sqrt(d_h + d_r)
    K = np.zeros((h, n, d_h + d_r)); V = np.zeros((h, n, d_h))
    for i in range(h):
        g, ib = i // (h // 2), i % (h // 2)
        K[i, :, :d_h] = C[:, g * d_g:(g + 1) * d_g] @ WK[g][:, ib * d_h:(ib + 1) * d_h]
        K[i, :, d_h:] = KR
        V[i] = C[:, g * d_g:(g + 1) * d_g] @ WV[g][:, ib * d_h:(ib + 1) * d_h]
    ref = _sdpa(np.concatenate([qn, qr], axis=1), K, V, tau)
    assert np.max(np.abs(orc.gla2_decode(qn, qr, C, KR, WK, WV, tau) - ref)) <= 1e-10
