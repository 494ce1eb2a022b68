"""The measurement probes of the library: the streaming read really reads (its per-workgroup XOR words fold
to the XOR of the whole buffer), and the shader-clock probe reports a plausible clock."""
import numpy as np
import pytest
import torch

from paper_2603_02188_amd import binding as mlra

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("nbytes,workgroups", [(16, 1), (4096 * 5 + 16 * 7, 3), (1 << 22, 64), ((1 << 22) + 4080, 2048)])
def test_stream_read_probe_folds_every_dword(nbytes, workgroups):
    rng = np.random.default_rng(nbytes)
    data = rng.integers(0, 2 ** 32, size=nbytes // 4, dtype=np.uint32)
    src = torch.from_numpy(data.view(np.int32)).cuda()
    sink = torch.zeros(workgroups, dtype=torch.int32, device="cuda")
    print(f"[case] stream read probe {nbytes} bytes, {workgroups} workgroups", flush=True)
    mlra.mlra_probe_stream_read(src, sink, workgroups)
    torch.cuda.synchronize()
    got = np.bitwise_xor.reduce(sink.cpu().numpy().view(np.uint32))
    want = np.bitwise_xor.reduce(data)
    assert got == want


def test_shader_clock_probe_is_plausible():
    out = torch.zeros(2, dtype=torch.int64, device="cuda")
    mlra.mlra_probe_shader_clock(out, 500)
    torch.cuda.synchronize()
    cycles, ticks = [int(v) for v in out.cpu().tolist()]
    assert 45000 <= ticks <= 200000            # about 500 us in 10 ns ticks
    ghz = cycles / (ticks * 10.0)
    print(f"[case] shader clock probe: {ghz:.3f} GHz", flush=True)
    assert 0.05 <= ghz <= 3.0


def test_probe_argument_checks():
    lib = mlra.load_library()
    assert lib.mlra_probe_stream_read(None, 64, None, 1, None) == -1
    x = torch.zeros(64, dtype=torch.uint8, device="cuda")
    s = torch.zeros(1, dtype=torch.int32, device="cuda")
    assert lib.mlra_probe_stream_read(mlra._ptr(x), 8, mlra._ptr(s), 1, None) == -2
    assert lib.mlra_probe_stream_read(mlra._ptr(x), 64, mlra._ptr(s), 0, None) == -2
    assert lib.mlra_probe_shader_clock(None, 10, None) == -1
    o = torch.zeros(2, dtype=torch.int64, device="cuda")
    assert lib.mlra_probe_shader_clock(mlra._ptr(o), 0, None) == -2
