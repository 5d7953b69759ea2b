"""Two things the small parity cases cannot show: the calls can be captured in
a HIP graph and replayed (no hidden allocation, memset or host wait; the
workspace is left ready by every call), and 64-bit indexing holds past 2^32
elements."""
import numpy as np
import pytest
import torch

from paper_1705_01626_amd import zvc
from tests.gpu_util import raw_bytes, say

pytestmark = pytest.mark.gpu
DEV = "cuda"


def sparse_floats(n, density, seed):
    g = torch.Generator(device=DEV).manual_seed(seed)
    x = torch.randn(n, generator=g, device=DEV)
    keep = torch.rand(n, generator=g, device=DEV) < density
    return torch.where(keep, x, torch.zeros_like(x))


def test_graph_replays_match_eager(oracle):
    """compress + decompress + windowed compress captured once, replayed on changing inputs, with the
    program's own eager work and synchronisations between the replays."""
    n, w = 3 * (1 << 20) + 4321, 4
    x = torch.empty(n, dtype=torch.float32, device=DEV)
    ws = zvc.new_workspace(n, w, DEV)
    comp = zvc.new_compressed_buffer(n, w, DEV)
    wcomp = zvc.new_compressed_buffer(n, w, DEV)
    offsets = torch.zeros(zvc.zvc_window_count(n, w) + 1, dtype=torch.int64, device=DEV)
    d_bytes = torch.zeros(1, dtype=torch.int64, device=DEV)
    w_bytes = torch.zeros(1, dtype=torch.int64, device=DEV)
    out = torch.empty_like(x)
    side = torch.cuda.Stream()
    x.copy_(sparse_floats(n, 0.5, 1))
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    say("capturing compress + decompress + window compress")
    with torch.cuda.graph(graph, stream=side):
        zvc.zvc_compress(x, comp, d_bytes, ws)
        # the decoder reads exactly the bytes a stream of this size has; capture uses the worst case
        zvc.zvc_decompress(comp, comp.numel(), out, ws)
        zvc.zvc_window_compress(x, wcomp, offsets, w_bytes, ws)
    for rep, density in enumerate((0.5, 0.1, 0.9, 0.0, 1.0)):
        x.copy_(sparse_floats(n, density, 10 + rep) if density < 1.0 else torch.randn(n, device=DEV).abs_() + 1)
        out.fill_(7.0)
        torch.cuda.synchronize()
        say("replay %d density %.1f" % (rep, density))
        graph.replay()
        torch.cuda.synchronize()
        host = raw_bytes(x)
        expect = oracle.compress_stream(host, w)
        nbytes = int(d_bytes.item())
        assert nbytes == expect.size
        assert np.array_equal(comp[:nbytes].cpu().numpy(), expect)
        assert torch.equal(out, x)
        wexpect, woffsets = oracle.window_compress(host, w, zvc.WINDOW_PAPER_BYTES // w)
        assert int(w_bytes.item()) == wexpect.size
        assert np.array_equal(wcomp[: wexpect.size].cpu().numpy(), wexpect)
        assert offsets.cpu().numpy().astype(np.uint64).tolist() == woffsets.tolist()
        # eager work on the same workspace between replays
        eager = zvc.new_compressed_buffer(n, w, DEV)
        zvc.zvc_compress(x, eager, d_bytes, ws)
        torch.cuda.synchronize()
        assert torch.equal(eager[:nbytes], comp[:nbytes])


def test_past_two_to_the_32_elements():
    """n = 2^32 + 70,001 16-bit elements (8.6 GB): sizes, sampled masks and values against
    what torch computes on the same bytes, and the full round trip."""
    n = (1 << 32) + 70001
    free, _ = torch.cuda.mem_get_info()
    if free < 40 * (1 << 30):
        pytest.skip("needs about 36 GB of free GPU memory")
    w = 2
    say("building %d elements" % n)
    x = torch.empty(n, dtype=torch.int16, device=DEV)
    chunk = 1 << 28
    g = torch.Generator(device=DEV).manual_seed(5)
    for lo in range(0, n, chunk):
        m = min(chunk, n - lo)
        v = torch.randint(1, 30000, (m,), generator=g, device=DEV, dtype=torch.int16)
        keep = torch.rand(m, generator=g, device=DEV) < 0.25
        x[lo: lo + m] = torch.where(keep, v, torch.zeros_like(v))
        del v, keep
    nnz = 0
    for lo in range(0, n, chunk):
        nnz += int(torch.count_nonzero(x[lo: lo + chunk]).item())
    groups = (n + 31) // 32
    ws = zvc.new_workspace(n, w, DEV)
    comp = zvc.new_compressed_buffer(n, w, DEV)
    d_bytes = torch.zeros(1, dtype=torch.int64, device=DEV)
    say("compress")
    zvc.zvc_compress(x, comp, d_bytes, ws)
    torch.cuda.synchronize()
    nbytes = int(d_bytes.item())
    assert nbytes == 4 * groups + w * nnz
    say("count-only")
    d2 = torch.zeros(1, dtype=torch.int64, device=DEV)
    zvc.zvc_compressed_size(x, d2, ws)
    assert int(d2.item()) == nbytes
    # sampled groups around the 2^32 element boundary and at both ends: mask and values
    masks = comp[: 4 * groups].view(torch.int32)
    values = comp[4 * groups: nbytes].view(torch.int16)
    weights = (1 << torch.arange(32, device=DEV, dtype=torch.int64))
    for g0 in (0, 1, (1 << 27) - 1, 1 << 27, (1 << 27) + 1, groups - 2, groups - 1):
        lo, hi = g0 * 32, min(n, g0 * 32 + 32)
        seg = x[lo:hi]
        bits = (seg != 0).to(torch.int64)
        expect_mask = int((bits * weights[: hi - lo]).sum().item())
        got_mask = int(masks[g0].item()) & 0xFFFFFFFF
        assert got_mask == expect_mask, "mask of group %d" % g0
        before = 0
        for lo2 in range(0, lo, chunk):
            before += int(torch.count_nonzero(x[lo2: min(lo, lo2 + chunk)]).item())
        kept = seg[seg != 0]
        assert torch.equal(values[before: before + kept.numel()], kept), "values of group %d" % g0
    say("decompress")
    out = torch.empty_like(x)
    zvc.zvc_decompress(comp, nbytes, out, ws)
    torch.cuda.synchronize()
    for lo in range(0, n, chunk):
        assert torch.equal(out[lo: lo + chunk], x[lo: lo + chunk]), "round trip near element %d" % lo
    say("self-help events: %d" % zvc.zvc_workspace_self_help_count(ws))


def test_calls_on_two_streams_overlap(oracle):
    """Calls with their own workspaces on two streams may run at the same time:
    the library keeps no state outside the buffers it is given."""
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    sets = []
    for k, (n, w, density) in enumerate(((6 * (1 << 20) + 123, 4, 0.4), (9 * (1 << 20) + 77, 2, 0.15))):
        x = sparse_floats(n, density, 40 + k)
        x = x if w == 4 else x.to(torch.bfloat16)
        sets.append(dict(x=x, n=n, w=w, ws=zvc.new_workspace(n, w, DEV), comp=zvc.new_compressed_buffer(n, w, DEV),
                         d_bytes=torch.zeros(1, dtype=torch.int64, device=DEV), out=torch.empty_like(x)))
    torch.cuda.synchronize()
    say("two streams, interleaved launches")
    for rep in range(6):
        for s, t in zip(streams, sets):
            with torch.cuda.stream(s):
                zvc.zvc_compress(t["x"], t["comp"], t["d_bytes"], t["ws"], stream=s)
        for s, t in zip(streams, sets):
            with torch.cuda.stream(s):
                # worst-case size: the decoder reads no stored element the masks do not ask for
                zvc.zvc_decompress(t["comp"], t["comp"].numel(), t["out"], t["ws"], stream=s)
    torch.cuda.synchronize()
    for t in sets:
        expect = oracle.compress_stream(raw_bytes(t["x"]), t["w"])
        assert int(t["d_bytes"].item()) == expect.size
        assert np.array_equal(t["comp"][:expect.size].cpu().numpy(), expect)
        assert torch.equal(t["out"].view(torch.int16 if t["w"] == 2 else torch.int32),
                           t["x"].view(torch.int16 if t["w"] == 2 else torch.int32))
        say("self-help events: %d" % zvc.zvc_workspace_self_help_count(t["ws"]))
