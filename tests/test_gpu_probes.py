"""The two streaming yardsticks of the benchmark (no part of the method): the
read probe reports the bytes it covers and writes nothing, the mixed probe
writes a ^ b over exactly the slices it reports and nothing beyond."""
import pytest
import torch

from paper_2601_21686_amd import binding as B

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("streaming", [False, True])
@pytest.mark.parametrize("n_bytes,workgroups", [(1 << 22, 64), ((1 << 22) + 40000, 100), (16384 * 7, 7)])
def test_read_probe_covers_whole_slices_and_writes_nothing(n_bytes, workgroups, streaming):
    src = torch.ones(n_bytes // 4, dtype=torch.int32, device="cuda")
    sink = torch.full((workgroups,), -7.0, dtype=torch.float32, device="cuda")
    n = B.skv_probe_stream_read(src, workgroups, sink, streaming)
    torch.cuda.synchronize()
    assert 0 < n <= n_bytes and n % (workgroups * 16384) == 0 and n_bytes - n < workgroups * 16384
    assert bool((sink == -7.0).all())


@pytest.mark.parametrize("n_bytes,workgroups", [(1 << 22, 64), ((1 << 22) + 40000, 100), (16384 * 7, 7)])
def test_mix_probe_writes_the_xor_of_its_slices_only(n_bytes, workgroups):
    g = torch.Generator(device="cpu").manual_seed(5)
    a = torch.randint(-2**31, 2**31 - 1, (n_bytes // 4,), dtype=torch.int32, generator=g).cuda()
    b = torch.randint(-2**31, 2**31 - 1, (n_bytes // 4,), dtype=torch.int32, generator=g).cuda()
    c = torch.full_like(a, 0x5A5A5A5A)
    n = B.skv_probe_stream_mix(a, b, c, workgroups)
    torch.cuda.synchronize()
    assert 0 < n <= n_bytes and n % (workgroups * 16384) == 0
    assert torch.equal(c[: n // 4], a[: n // 4] ^ b[: n // 4])
    assert bool((c[n // 4:] == 0x5A5A5A5A).all())
