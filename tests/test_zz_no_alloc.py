"""zvc_compress_static (the entry point that allocates nothing: its scan state
lives in an array inside the library) against zvc_compress, through the C ABI,
bit for bit: two calls in a row, the second with a smaller input, then a third
at the size limit's error path."""
import numpy as np
import pytest
import torch

from paper_1705_01626_amd import zvc
from tests.gpu_util import say
from tests.test_gpu_parity import random_tensor

pytestmark = pytest.mark.gpu


def both_streams(x):
    n, w = x.numel(), x.element_size()
    ws = zvc.new_workspace(n, w, x.device)
    ref = zvc.new_compressed_buffer(n, w, x.device)
    ref.fill_(0xCD)
    ref_bytes = torch.full((1,), -1, dtype=torch.int64, device=x.device)
    zvc.zvc_compress(x, ref, ref_bytes, ws)
    got = zvc.new_compressed_buffer(n, w, x.device)
    got.fill_(0xCD)
    got_bytes = torch.full((1,), -1, dtype=torch.int64, device=x.device)
    zvc.zvc_compress_static(x, got, got_bytes)
    torch.cuda.synchronize()
    return ref, int(ref_bytes.item()), got, int(got_bytes.item())


@pytest.mark.parametrize("w", [4, 2])
def test_static_scratch_matches_workspace_call(w):
    # 70 MB then 5 MB at w = 4 (32 KB then 16 KB tiles), half that at w = 2; ragged sizes
    for k, n in enumerate((17_500_003, 1_300_021)):
        x = random_tensor(n, w, (0.35, 0.7)[k], seed=1000 + n + w)
        say("zvc_compress_static n=%d w=%d" % (n, w))
        ref, ref_bytes, got, got_bytes = both_streams(x)
        assert got_bytes == ref_bytes
        assert torch.equal(got[:got_bytes], ref[:ref_bytes]), "stream differs from zvc_compress's"
        # and it decodes back to the input
        out = torch.empty_like(x)
        ws = zvc.new_workspace(n, w, x.device)
        zvc.zvc_decompress(got, got_bytes, out, ws)
        torch.cuda.synchronize()
        assert torch.equal(out, x)


def test_static_scratch_size_limit():
    x = torch.zeros(16, dtype=torch.int32, device="cuda")
    out = torch.empty(4096, dtype=torch.uint8, device="cuda")
    nbytes = torch.zeros(1, dtype=torch.int64, device="cuda")
    with pytest.raises(zvc.ZvcError) as err:
        zvc.zvc_compress_static(x, out, nbytes, n=zvc.STATIC_MAX_BYTES // 4 + 1)
    assert err.value.status == zvc.ZVC_E_WORKSPACE
    # the largest tile count the scratch must hold: the limit itself is accepted by the size check
    # (it then fails on the output capacity, before anything is enqueued)
    with pytest.raises(zvc.ZvcError) as err:
        zvc.zvc_compress_static(x, out, nbytes, n=zvc.STATIC_MAX_BYTES // 4)
    assert err.value.status == zvc.ZVC_E_CAPACITY
