"""The streaming probes (measurement aids of the library): the copy moves exactly the bytes it is asked to, the
mixed probe writes exactly its write share, and both refuse sizes and addresses they cannot serve."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available()
    from paper_2311_17410_amd import binding as B
    B.lib()
    return B


def test_copy_read_write_probes(B):
    import torch
    dev = torch.device("cuda", 0)
    n = (1 << 20) + 4096 + 16          # several workgroups and a ragged tail
    src = torch.randint(0, 255, (n,), dtype=torch.uint8, device=dev)
    for nt in (False, True):
        dst = torch.zeros(n + 64, dtype=torch.uint8, device=dev)
        B.tns_hbm_probe(0, nt, dst.data_ptr(), src.data_ptr(), n)
        torch.cuda.synchronize()
        assert torch.equal(dst[:n], src) and int(dst[n:].sum()) == 0
        B.tns_hbm_probe(1, nt, 0, src.data_ptr(), n)          # read only: no destination needed
        B.tns_hbm_probe(2, nt, dst.data_ptr(), 0, n)          # write only
        torch.cuda.synchronize()
        assert int(dst[n:].sum()) == 0
    with pytest.raises(B.TnsError):
        B.tns_hbm_probe(0, True, dst.data_ptr(), src.data_ptr(), n + 8)       # not a multiple of 16
    with pytest.raises(B.TnsError):
        B.tns_hbm_probe(3, True, dst.data_ptr(), src.data_ptr(), n)           # no such mode
    with pytest.raises(B.TnsError):
        B.tns_hbm_probe(0, True, 0, src.data_ptr(), n)                        # copy without a destination


@pytest.mark.parametrize("read_bytes,write_bytes", [(1 << 20, 1 << 20), (1 << 20, 1 << 18), (1 << 18, 1 << 20), ((1 << 20) + 48, 4096 + 16),
                                                    (16, 1 << 16)])
def test_mixed_probe_writes_its_share_only(B, read_bytes, write_bytes):
    import torch
    dev = torch.device("cuda", 0)
    src = torch.randint(1, 255, (read_bytes,), dtype=torch.uint8, device=dev)
    dst = torch.zeros(write_bytes + 256, dtype=torch.uint8, device=dev)
    B.tns_hbm_probe_mix(True, dst.data_ptr(), write_bytes, src.data_ptr(), read_bytes)
    torch.cuda.synchronize()
    assert int(dst[write_bytes:].sum()) == 0                   # nothing beyond the write share
    written = dst[:write_bytes].view(-1, 16).any(dim=1)
    assert bool(written.all())                                 # every 16-byte vector of the share was stored
    with pytest.raises(B.TnsError):
        B.tns_hbm_probe_mix(True, dst.data_ptr(), write_bytes + 4, src.data_ptr(), read_bytes)
    with pytest.raises(B.TnsError):
        B.tns_hbm_probe_mix(True, dst.data_ptr(), 0, src.data_ptr(), read_bytes)
