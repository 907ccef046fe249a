"""GPU: the unified-tensor convenience (Section 3.1, Listing 1 usage) returns what torch indexing
of the CPU tensor returns, bit for bit, for every element size."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
z = pytest.importorskip("paper_2103_03330_amd")


@pytest.mark.parametrize("dtype", [torch.float32, torch.float16, torch.bfloat16, torch.int8, torch.float64,
                                   torch.int32])
def test_indexing_a_unified_tensor_matches_cpu_indexing(dtype):
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU")
    torch.cuda.set_device(0)
    g = torch.Generator().manual_seed(5)
    cpu = (torch.randn((4000, 100), generator=g) * 50).to(dtype)
    idx = torch.randint(0, 4000, (12345,), generator=g)
    with z.to_unified(cpu) as u:
        got = u[idx.cuda()]
        torch.cuda.synchronize()
        assert got.dtype == dtype and got.device.type == "cuda"
        want = cpu[idx]
        assert got.cpu().view(torch.uint8).numpy().tobytes() == want.view(torch.uint8).numpy().tobytes()
        out = torch.empty((idx.numel(), 100), dtype=dtype, device="cuda")
        order = torch.argsort(idx.cuda())
        assert u.gather(idx.cuda(), out=out, ordered_by=order) is out
        torch.cuda.synchronize()
        assert out.cpu().view(torch.uint8).numpy().tobytes() == want.view(torch.uint8).numpy().tobytes()
        with pytest.raises(ValueError):
            u.gather(idx.cuda(), out=out[:10])
    with pytest.raises(ValueError):
        z.to_unified(cpu[:, ::2])


def test_short_row_unified_tensor_lends_its_own_workspace():
    """Rows of at most a line and a long dense list: indexing goes through the ordered walk with
    scratch memory the tensor owns; the result is torch's."""
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU")
    torch.cuda.set_device(0)
    g = torch.Generator().manual_seed(9)
    cpu = torch.randn((300_000, 16), generator=g).to(torch.float16)
    with z.to_unified(cpu) as u:
        for n in (250_000, 40_000, 1000):
            idx = torch.randint(0, cpu.shape[0], (n,), generator=g)
            got = u[idx.cuda()]
            torch.cuda.synchronize()
            assert got.cpu().view(torch.uint8).numpy().tobytes() == cpu[idx].view(torch.uint8).numpy().tobytes()
        assert u._workspace is not None and u._workspace.numel() >= z.gather_workspace_bytes(250_000)
