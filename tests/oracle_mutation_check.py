"""Mutation check of the oracle pins (CPU only, not collected by pytest; run `python tests/oracle_mutation_check.py`).

One small, plausible mistake at a time (a dropped term, a wrong sign, a wrong block or head slab, a transposed
operand, an index off by one) is planted in a temporary copy of oracle/mlra_oracle.py, and the pin tests
(tests/test_oracle_pins.py, tests/test_models_golden.py) are run against that copy.  Every mutant has to make
at least one pin fail; the script exits non-zero if one survives."""
import os
import re
import shutil
import subprocess
import sys
import tempfile

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
src = open(os.path.join(ROOT, "oracle", "mlra_oracle.py")).read()
MUTS = [
 ("unabsorbed: drop rope term", "s = tau * (K_bi @ q_nope[i]) + tau * (KR @ q_rope[i])            # [n]", "s = tau * (K_bi @ q_nope[i])            # [n]"),
 ("unabsorbed: sign of rope term", "s = tau * (K_bi @ q_nope[i]) + tau * (KR @ q_rope[i])            # [n]", "s = tau * (K_bi @ q_nope[i]) - tau * (KR @ q_rope[i])            # [n]"),
 ("absorbed: drop tau on rope", "S = tau * (q_abs_b @ C_b.T) + tau * (q_rope @ KR.T)", "S = tau * (q_abs_b @ C_b.T) + (q_rope @ KR.T)"),
 ("absorbed: drop rope", "S = tau * (q_abs_b @ C_b.T) + tau * (q_rope @ KR.T)", "S = tau * (q_abs_b @ C_b.T)"),
 ("w_block: wrong block rows", "return W[b * d_cb:(b + 1) * d_cb, i * d_h:(i + 1) * d_h]", "return W[((b + 1) % 2) * d_cb:(((b + 1) % 2) + 1) * d_cb, i * d_h:(i + 1) * d_h]"),
 ("w_block: wrong head cols", "return W[b * d_cb:(b + 1) * d_cb, i * d_h:(i + 1) * d_h]", "return W[b * d_cb:(b + 1) * d_cb, 0:d_h]"),
 ("c_block: always block 0", "return C[:, b * d_cb:(b + 1) * d_cb]", "return C[:, 0:d_cb]"),
 ("softmax: no normalisation", "return e / np.sum(e)", "return e"),
 ("lse: m - log l", "return Z, (m + np.log(l))[:, 0]", "return Z, (m - np.log(l))[:, 0]"),
 ("gamma: swapped groups", "return 0 if i < h // 2 else 1", "return 1 if i < h // 2 else 0"),
 ("wg_block: j ignored", "return W_g[j * d_cb:(j + 1) * d_cb, i_bar * d_h:(i_bar + 1) * d_h]", "return W_g[0:d_cb, i_bar * d_h:(i_bar + 1) * d_h]"),
 ("mlra2 unabsorbed: drop rope", "            s = tau * (K_bi @ q_nope[i]) + tau * (KR @ q_rope[i])\n", "            s = tau * (K_bi @ q_nope[i])\n"),
 ("rope_angles: +2l/d_r", "** (-2.0 * np.arange(d_r // 2) / d_r)", "** (2.0 * np.arange(d_r // 2) / d_r)"),
 ("rope_angles: l/d_r", "** (-2.0 * np.arange(d_r // 2) / d_r)", "** (-1.0 * np.arange(d_r // 2) / d_r)"),
 ("rope_angles: starts at l = 1", "** (-2.0 * np.arange(d_r // 2) / d_r)", "** (-2.0 * (np.arange(d_r // 2) + 1) / d_r)"),
 ("rope_angles: 2l/(d_r/2)", "** (-2.0 * np.arange(d_r // 2) / d_r)", "** (-2.0 * np.arange(d_r // 2) / (d_r // 2))"),
 ("gated: divide instead of multiply", "return np.asarray(O, np.float64) * np.asarray(G, np.float64)", "return np.asarray(O, np.float64) / np.asarray(G, np.float64)"),
 ("gated: add instead of multiply", "return np.asarray(O, np.float64) * np.asarray(G, np.float64)", "return np.asarray(O, np.float64) + np.asarray(G, np.float64)"),
 ("mla: out_scale 0.5", "return mlra_decode_absorbed(q_nope, q_rope, C, KR, W_UK, W_UV, 1, tau, 1.0)", "return mlra_decode_absorbed(q_nope, q_rope, C, KR, W_UK, W_UV, 1, tau, 0.5)"),
]

MUTS += [
 ("absorb: transposed contraction", 'out[b] = np.einsum("hp,chp->hc", q_nope, W_b)', 'out[b] = np.einsum("hp,chp->hc", q_nope[::-1], W_b)'),
 ("absorb: wrong block slab", "W_b = W_UK[b * d_cb:(b + 1) * d_cb].reshape(d_cb, h, d_h)", "W_b = W_UK[0:d_cb].reshape(d_cb, h, d_h)"),
 ("up_project: head/channel swapped reshape", "W = np.asarray(W_UV_b, np.float64).reshape(-1, h, d_h)", "W = np.asarray(W_UV_b, np.float64).reshape(-1, d_h, h).transpose(0, 2, 1)"),
 ("rope: sin sign", "out[..., 0::2] = even * c - odd * s", "out[..., 0::2] = even * c + odd * s"),
 ("rope: second row sign", "out[..., 1::2] = even * s + odd * c", "out[..., 1::2] = -even * s + odd * c"),
 ("pre: k_rope not rotated", "k_rope = rope(x @ np.asarray(W_KR, np.float64), position, rope_base)", "k_rope = x @ np.asarray(W_KR, np.float64)"),
 ("pre: q_rope uses position+1", "q_rope = rope((c_q @ np.asarray(W_QR, np.float64)).reshape(h, -1), position, rope_base)", "q_rope = rope((c_q @ np.asarray(W_QR, np.float64)).reshape(h, -1), position + 1, rope_base)"),
 ("pre: c_kv from W_DQ-normalised x", "c_kv = alpha_kv * rms_norm(x @ np.asarray(W_DKV, np.float64), gain_kv, eps)", "c_kv = alpha_kv * (x @ np.asarray(W_DKV, np.float64))"),
 ("gather: page index off", "page = int(page_table_row[t // ps])\n        k = min(ps, n - t)\n        for b in range(NB):", "page = int(page_table_row[0])\n        k = min(ps, n - t)\n        for b in range(NB):"),
 ("gather: block order reversed", "C[t:t + k, b * d_cb:(b + 1) * d_cb] = latent_pool[page, b, :k, :]", "C[t:t + k, b * d_cb:(b + 1) * d_cb] = latent_pool[page, NB - 1 - b, :k, :]"),
 ("append: slot off by one", "slot = pos % ps", "slot = (pos + 1) % ps"),
 ("append: block slab", "latent_pool[page, blk, slot, :] = row[blk * d_cb:(blk + 1) * d_cb]", "latent_pool[page, blk, slot, :] = row[0:d_cb]"),
 ("gqa gather: no transpose", "K[t:t + k] = np.transpose(k_pool[page, :, :k, :], (1, 0, 2))", "K[t:t + k] = np.transpose(k_pool[page, ::-1, :k, :], (1, 0, 2))"),
]
# a few regex-based ones on functions whose body is not quoted above
RE_MUTS = [
 ("rms_norm: mean -> sum", r"np\.mean\(", "np.sum("),
 ("pre_attention: alpha_q dropped", r"alpha_q \* ", ""),
 ("pre_attention: alpha_kv dropped", r"alpha_kv \* ", ""),
 ("multi: causal offset", r"n - \(q_len - 1 - j\)", "n - (q_len - j)"),
 ("gqa: group map", r"i // r\b", "i % g"),
]
def run(mut_src):
    d = tempfile.mkdtemp(prefix="oracle_mutant_")
    for sub in ("oracle", "tests", "paper_2603_02188_amd", "include"):
        shutil.copytree(os.path.join(ROOT, sub), os.path.join(d, sub), ignore=shutil.ignore_patterns("_build", "__pycache__", "csrc"))
    open(os.path.join(d, "oracle", "mlra_oracle.py"), "w").write(mut_src)
    r = subprocess.run([sys.executable, "-m", "pytest", "tests/test_oracle_pins.py", "tests/test_models_golden.py", "-x", "-q", "-p", "no:cacheprovider"],
                       cwd=d, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    shutil.rmtree(d, ignore_errors=True)
    return r.returncode, r.stdout.strip().splitlines()[-1]
def main():
    rc0, last = run(src)
    print("unmodified oracle:", rc0, last)
    surv = []
    for name, a, b in MUTS:
        if a not in src: print("SKIP (pattern not found):", name); continue
        rc, last = run(src.replace(a, b, 1))
        print(("killed  " if rc != 0 else "SURVIVED"), name, "|", last[:80])
        if rc == 0: surv.append(name)
    for name, pat, rep in RE_MUTS:
        if not re.search(pat, src): print("SKIP (pattern not found):", name); continue
        rc, last = run(re.sub(pat, rep, src, count=1))
        print(("killed  " if rc != 0 else "SURVIVED"), name, "|", last[:80])
        if rc == 0: surv.append(name)
    print("survivors:", surv)
    sys.exit(1 if surv or rc0 != 0 else 0)


if __name__ == "__main__":
    main()
