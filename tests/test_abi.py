"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, and turns host-visible mistakes into error codes without launching anything."""
import ctypes
import os
import re

import pytest

from paper_2603_02188_amd import binding as mlra

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "mlra.h")).read()
    return sorted(set(re.findall(r"MLRA_API\s+[\w\s\*]+?\b(\w+)\s*\(", text)))


def test_header_and_binding_agree_on_exports():
    assert sorted(mlra.EXPORTS) == _declared()


def test_library_exports_every_declared_symbol():
    lib = mlra.load_library()
    for name in _declared():
        assert hasattr(lib, name), name


def test_strerror_texts():
    assert mlra.strerror(0) == "ok"
    for code in (-1, -2, -3, -4, -5):
        assert mlra.strerror(code) not in ("ok", "unknown status")
    assert mlra.strerror(-99) == "unknown status"


def test_null_and_shape_errors_are_reported_on_the_host():
    lib = mlra.load_library()
    cs = mlra._CacheStruct(0, 0, 0, 0, 1, 64, 1, 4, 128, 64, 0)
    null = ctypes.c_void_p(None)
    assert lib.mlra_append_kv(ctypes.byref(cs), 1, null, null, 1, null, null) == -1
    assert lib.mlra_absorb_q(1, 8, 64, 4, 64, null, null, null, 1, null) == -1
    one = ctypes.c_void_p(256)   # never dereferenced: the shape/dtype checks come first
    assert lib.mlra_absorb_q(0, 8, 64, 4, 64, one, one, one, 1, null) == -2
    assert lib.mlra_absorb_q(1, 8, 64, 4, 64, one, one, one, 7, null) == -3
    assert lib.mlra_decode_attn(None, 1, 8, 64, one, one, one, 0.1, 1.0, one, 1, null, one, 1 << 30, null) == -1
    cs2 = mlra._CacheStruct(256, 256, 256, 256, 4, 64, 4, 4, 64, 32, 1)
    assert lib.mlra_decode_attn(ctypes.byref(cs2), 1, 8, 64, one, one, one, 0.1, 1.0, one, 5, null, one, 1 << 30,
                                null) == -3
    assert lib.mlra_decode_attn(ctypes.byref(cs2), 0, 8, 64, one, one, one, 0.1, 1.0, one, 1, null, one, 1 << 30,
                                null) == -2
    # workspace: missing, too small, misaligned
    assert lib.mlra_decode_attn(ctypes.byref(cs2), 1, 8, 64, one, one, one, 0.1, 1.0, one, 1, null, null, 0,
                                null) == -4
    assert lib.mlra_decode_attn(ctypes.byref(cs2), 1, 8, 64, one, one, one, 0.1, 1.0, one, 1, null, one, 16,
                                null) == -4
    assert lib.mlra_decode_attn(ctypes.byref(cs2), 1, 8, 64, one, one, one, 0.1, 1.0, one, 1, null,
                                ctypes.c_void_p(264), 1 << 30, null) == -4
    # MLA entry point insists on a single latent block
    assert lib.mla_decode_attn(ctypes.byref(cs2), 1, 8, 64, one, one, one, 0.1, one, 1, null, one, 1 << 30,
                               null) == -2
    # MLRA-2 wants an even number of heads and of blocks
    assert lib.mlra2_absorb_q(1, 7, 64, 4, 64, one, one, one, 1, null) == -2
    assert lib.mlra2_absorb_q(1, 8, 64, 3, 64, one, one, one, 1, null) == -2
    assert lib.mlra2_absorb_q(1, 8, 64, 4, 64, null, one, one, 1, null) == -1
    assert lib.mlra2_decode_attn(ctypes.byref(cs2), 1, 7, 64, one, one, one, 0.1, 1.0, one, 1, null, one, 1 << 30,
                                 null) == -2
    cs3 = mlra._CacheStruct(256, 256, 256, 256, 4, 64, 4, 3, 64, 32, 1)
    assert lib.mlra2_decode_attn(ctypes.byref(cs3), 1, 8, 64, one, one, one, 0.1, 1.0, one, 1, null, one, 1 << 30,
                                 null) == -2
    assert lib.mlra2_decode_attn(ctypes.byref(cs2), 1, 8, 64, one, one, one, 0.1, 1.0, one, 1, null, null, 0,
                                 null) == -4
    # gated output needs its gate
    assert lib.mlra_decode_attn_gated(ctypes.byref(cs2), 1, 8, 64, one, one, one, null, 0.1, 1.0, one, 1, null, one,
                                      1 << 30, null) == -1
    # several query tokens: bad q_len, workspace too small, null cache
    assert lib.mlra_decode_attn_multi(ctypes.byref(cs2), 1, 0, 8, 64, one, one, one, 0.1, 1.0, one, 1, null, one,
                                      1 << 30, null) == -2
    assert lib.mlra_decode_attn_multi(ctypes.byref(cs2), 1, 3, 8, 64, one, one, one, 0.1, 1.0, one, 1, null, one,
                                      64, null) == -4
    assert lib.mlra_decode_attn_multi(None, 1, 3, 8, 64, one, one, one, 0.1, 1.0, one, 1, null, one, 1 << 30,
                                      null) == -1
    assert lib.mlra_decode_attn_multi(ctypes.byref(cs2), 1, 3, 8, 64, null, one, one, 0.1, 1.0, one, 1, null, one,
                                      1 << 30, null) == -1
    # pre-attention: null weights, odd RoPE dim, workspace too small
    pw = mlra._PreWeightsStruct(256, 256, 256, 256, 256, None, None, 96, 40, 8, 64, 1, 1.0, 1.0, 1e-6, 1e4)
    pw_null = mlra._PreWeightsStruct(None, 256, 256, 256, 256, None, None, 96, 40, 8, 64, 1, 1.0, 1.0, 1e-6, 1e4)
    assert lib.mlra_pre_attention(ctypes.byref(cs2), ctypes.byref(pw_null), 2, one, one, one, one, one, 1 << 30,
                                  null) == -1
    assert lib.mlra_pre_attention(ctypes.byref(cs2), None, 2, one, one, one, one, one, 1 << 30, null) == -1
    cs_odd = mlra._CacheStruct(256, 256, 256, 256, 4, 64, 4, 4, 64, 31, 1)
    assert lib.mlra_pre_attention(ctypes.byref(cs_odd), ctypes.byref(pw), 2, one, one, one, one, one, 1 << 30,
                                  null) == -2
    assert lib.mlra_pre_attention(ctypes.byref(cs2), ctypes.byref(pw), 2, one, one, one, one, one, 16, null) == -4
    pw_dt = mlra._PreWeightsStruct(256, 256, 256, 256, 256, None, None, 96, 40, 8, 64, 9, 1.0, 1.0, 1e-6, 1e4)
    assert lib.mlra_pre_attention(ctypes.byref(cs2), ctypes.byref(pw_dt), 2, one, one, one, one, one, 1 << 30,
                                  null) == -3
    assert lib.gqa_decode_attn(one, one, one, one, 4, 64, 4, 1, 8, 3, 64, 0, one, 0.1, one, 1, one, 1 << 30,
                               null) == -2   # h % g != 0
    assert lib.gqa_decode_attn(null, one, one, one, 4, 64, 4, 1, 8, 2, 64, 0, one, 0.1, one, 1, one, 1 << 30,
                               null) == -1


def test_workspace_sizing():
    assert mlra.mlra_decode_workspace_bytes(0, 8, 4, 64, 256) == 0
    small = mlra.mlra_decode_workspace_bytes(1, 8, 4, 64, 256)
    # at least one partial (z, m, l) per (sequence, block, head)
    assert small >= 1 * 4 * 8 * (64 + 2) * 4
    big = mlra.mlra_decode_workspace_bytes(64, 128, 4, 128, 8192)
    assert big >= 64 * 4 * 128 * (128 + 2) * 4 and big % 256 == 0
    assert mlra.gqa_decode_workspace_bytes(2, 16, 128, 4096) >= 2 * 16 * 130 * 4
    assert mlra.mlra_pre_attention_workspace_bytes(64, 7168, 1536, 4, 128, 64, 128, 128, __import__("torch").bfloat16) \
        >= 64 * (1536 + 512 + 64) * 4 + 64 * 1536 * 2 + 64 * 128 * 192 * 4
    assert mlra.mlra_pre_attention_workspace_bytes(64, 7168, 1536, 4, 128, 63, 128, 128, __import__("torch").bfloat16) == 0
    assert mlra.mlra_decode_multi_workspace_bytes(2, 0, 8, 4, 64, 64, 4) == 0
    assert mlra.mlra_decode_multi_workspace_bytes(2, 3, 8, 4, 64, 64, 4) > mlra.mlra_decode_workspace_bytes(6, 8, 4, 64, 256)
    # MLRA-2: each block holds partials for h/2 heads
    assert mlra.mlra2_decode_workspace_bytes(1, 7, 4, 64, 256) == 0
    m2 = mlra.mlra2_decode_workspace_bytes(64, 128, 4, 128, 8192)
    assert 64 * 4 * 64 * (128 + 2) * 4 <= m2 <= big + 4096   # two chunks of 64 heads per (sequence, block)


def test_binding_fails_loudly_without_the_library(monkeypatch, tmp_path):
    monkeypatch.setattr(mlra, "_lib", None)
    monkeypatch.setattr(mlra, "_LIB_PATH", str(tmp_path / "libmlra.so"))
    with pytest.raises(RuntimeError, match="no CPU or PyTorch fallback"):
        mlra.load_library()


def test_workload_shapes_take_the_fast_paths():
    """Host logic: the benchmark shapes run on the MFMA kernels with the context split they were tuned with
    (a shape that silently fell back to a generic kernel, or lost its planning mode, would still pass
    parity)."""
    import numpy as np
    import torch
    from paper_2603_02188_amd import inputs as gen

    def info(key, **kw):
        wl = gen.WORKLOADS[key]
        lens = gen.draw_seq_lens(wl)
        max_seq_len = int(-(-int(lens.max()) // wl.page_size) * wl.page_size)
        dt = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
        args = dict(batch=wl.batch, h=wl.h, d_h=wl.d_h, groups=wl.groups, n_blocks=wl.n_blocks, d_cb=wl.d_cb,
                    d_r=wl.d_r, page_size=wl.page_size, max_seq_len=max_seq_len, dtype=dt)
        args.update(kw)
        return mlra.mlra_decode_plan_info(**args)

    assert info("C1")["kernel"] == "generic"                         # fp32 cache
    c2 = info("C2")
    assert (c2["kernel"], c2["chunk_slots"], c2["chunk_tokens"], c2["merge_mfma"]) == ("mfma", 16, 1024, True)
    c3 = info("C3")
    assert (c3["kernel"], c3["chunk_slots"], c3["target_chunks"], c3["merge_mfma"]) == ("mfma", 1, 0, True)
    c4 = info("C4")                                                  # long ragged contexts: planned chunks
    assert c4["kernel"] == "mfma" and c4["target_chunks"] == 64 and c4["chunk_slots"] == 32 and c4["merge_mfma"]
    c5 = info("C5")
    assert (c5["kernel"], c5["chunk_slots"], c5["target_chunks"]) == ("mfma", 1, 0)
    assert info("C5", page_size=16)["kernel"] == "mfma" and info("C5", page_size=48)["kernel"] == "generic"
    m2, g2 = info("M2"), info("G2")
    assert (m2["kernel"], m2["chunk_slots"], m2["target_chunks"]) == ("mfma-paired", 2, 0)
    assert (g2["kernel"], g2["chunk_slots"], g2["target_chunks"]) == ("mfma-gla", 2, 0)
    # the comparison kernels on the C5 batch: about one round of workgroups, so chunks are planned
    mla = info("C5", groups=1, n_blocks=1, d_cb=512, max_seq_len=8192)
    assert mla["kernel"] == "mfma-mla" and mla["target_chunks"] == 256 and mla["single_if_uniform"]
    two = info("M2", batch=128, max_seq_len=8192)
    assert two["kernel"] == "mfma-paired" and two["chunk_slots"] == 4 and two["single_if_uniform"]
    # 8 blocks x 16 chunks: the MFMA epilogue's LDS tables would exceed 160 KiB, so the generic epilogue runs
    big = info("C3", batch=2, n_blocks=8, max_seq_len=2048)
    assert (big["kernel"], big["chunk_slots"], big["merge_mfma"]) == ("mfma", 16, False)
    assert info("C3", batch=2, n_blocks=4, max_seq_len=2048)["merge_mfma"]


def test_static_entry_point_refuses_what_its_scratch_cannot_hold():
    """mlra_decode_attn_static checks sizes before it touches the device: a shape whose workspace exceeds the
    built-in 40 MiB returns MLRA_ERR_WORKSPACE, invalid sizes MLRA_ERR_SHAPE, a null cache MLRA_ERR_NULL."""
    import ctypes
    lib = mlra.load_library()
    cs = mlra._CacheStruct(1, 1, 1, 1, 1 << 20, 64, 256, 4, 128, 64, 0)       # dummy non-null pointers, 16384 tokens
    assert mlra.mlra_decode_workspace_bytes(512, 128, 4, 128, 16384) > 40 << 20
    st = lib.mlra_decode_attn_static(ctypes.byref(cs), 512, 128, 128, None, None, None, 0.07, 1.0, None, 0, None, None)
    assert st == -4
    assert lib.mlra_decode_attn_static(ctypes.byref(cs), 0, 128, 128, None, None, None, 0.07, 1.0, None, 0, None, None) == -2
    assert lib.mlra_decode_attn_static(None, 4, 128, 128, None, None, None, 0.07, 1.0, None, 0, None, None) == -1


def test_plan_info_errors():
    import ctypes
    import torch
    lib = mlra.load_library()
    buf = (ctypes.c_int32 * 6)()
    assert lib.mlra_decode_plan_info(4, 128, 128, 1, 4, 128, 64, 64, 8192, 0, None) == -1
    assert lib.mlra_decode_plan_info(0, 128, 128, 1, 4, 128, 64, 64, 8192, 0, buf) == -2
    assert lib.mlra_decode_plan_info(4, 127, 128, 2, 4, 128, 64, 64, 8192, 0, buf) == -2      # heads do not split into groups
    assert lib.mlra_decode_plan_info(4, 128, 128, 1, 4, 128, 64, 64, 8192, 7, buf) == -3
    assert mlra.mlra_decode_plan_info(4, 128, 128, 1, 4, 128, 64, 64, 8192, torch.bfloat16)["kernel"] == "mfma"
