"""The measurement aids move the bytes they say they move: the figures bench.py and the ceiling sweep derive from
their run times count exactly these bytes."""
import numpy as np
import pytest
import torch

import paper_2605_01708_amd as sz

pytestmark = pytest.mark.gpu

RUN = 4096  # bytes a workgroup moves per access of all its threads


def expected(src, write_bytes, r, w):
    """what splitzip_traffic_probe_shape leaves in the first write_bytes of the written buffer: the i-th written run
    of step s holds the (i mod r)-th run the step read; runs that start beyond the read bytes read as zero"""
    nread = len(src) // 16 * 16
    nwrite = write_bytes // 16 * 16
    padded = np.zeros(nread + 64 * RUN * max(r, 1) + nwrite * max(r, 1) // max(w, 1) + RUN * r, dtype=np.uint8)
    padded[:nread] = src[:nread]
    out = np.zeros(nwrite, dtype=np.uint8)
    steps = (nwrite + w * RUN - 1) // (w * RUN)
    for s in range(steps):
        for i in range(w):
            o = (w * s + i) * RUN
            if o >= nwrite:
                break
            a = (r * s + i % r) * RUN
            k = min(RUN, nwrite - o)
            out[o:o + k] = padded[a:a + k]
    return out


@pytest.mark.parametrize("r,w", [(4, 3), (8, 6), (16, 12), (3, 4), (6, 8), (12, 16), (1, 1), (4, 4)])
@pytest.mark.parametrize("wgs,flags", [(0, 0), (0, 3), (2, 3), (3, 7), (1, 15)])
def test_probe_shape_writes_the_runs_it_read(r, w, wgs, flags):
    steps = 37
    read_bytes = r * RUN * steps - 5 * 16          # the last step is ragged on both sides
    write_bytes = w * RUN * steps - RUN - 7 * 16
    g = torch.Generator().manual_seed(r * 100 + w)
    src_h = torch.randint(0, 256, (read_bytes,), dtype=torch.uint8, generator=g)
    src = src_h.cuda()
    dst = torch.full((write_bytes + 4096,), 0xA5, dtype=torch.uint8, device="cuda")
    sz.traffic_probe_shape(src, read_bytes, dst, write_bytes, r, w, wgs, flags)
    torch.cuda.synchronize()
    got = dst.cpu().numpy()
    want = expected(src_h.numpy(), write_bytes, r, w)
    assert np.array_equal(got[:len(want)], want)
    assert (got[len(want):] == 0xA5).all(), "wrote beyond the bytes it was given"


def test_probe_shape_rejects_what_it_does_not_know():
    src = torch.zeros(1 << 16, dtype=torch.uint8, device="cuda")
    dst = torch.zeros(1 << 16, dtype=torch.uint8, device="cuda")
    for r, w, wgs, flags in [(5, 3, 0, 0), (4, 3, 33, 0), (4, 3, 0, 64), (4, 3, 0, 8), (4, 3, 0, 20)]:
        with pytest.raises(sz.SplitZipError):
            sz.traffic_probe_shape(src, 1 << 16, dst, 1 << 16, r, w, wgs, flags)


@pytest.mark.parametrize("steps,cut", [(1, 0), (37, 0), (37, 5), (2100, 3)])
def test_fixed_probe_writes_three_of_the_four_runs_it_read(steps, cut):
    """splitzip_traffic_probe: per step four 4 KB runs read, three written; thread by thread the written 16 bytes are the
    read ones with words of the fourth run mixed in (so that the fourth run's loads cannot be dropped)"""
    read_bytes = 4 * RUN * steps - cut * 16
    write_bytes = 3 * RUN * steps - cut * 16 - (RUN if cut else 0)
    g = torch.Generator().manual_seed(steps)
    src_h = torch.randint(0, 256, (read_bytes,), dtype=torch.uint8, generator=g)
    dst = torch.full((write_bytes + 4096,), 0xA5, dtype=torch.uint8, device="cuda")
    sz.traffic_probe(src_h.cuda(), read_bytes, dst, write_bytes)
    torch.cuda.synchronize()
    got = dst.cpu().numpy()
    padded = np.zeros(4 * RUN * steps, dtype=np.uint8)
    padded[:read_bytes] = src_h.numpy()
    v = padded.view(np.uint32).reshape(steps, 4, RUN // 16, 4).copy()   # step, run, thread, word
    v[:, 0, :, 0] ^= v[:, 3, :, 0]
    v[:, 1, :, 1] ^= v[:, 3, :, 1]
    v[:, 2, :, 2] ^= v[:, 3, :, 2]
    v[:, 0, :, 3] ^= v[:, 3, :, 3]
    want = np.ascontiguousarray(v[:, :3]).view(np.uint8).reshape(-1)[:write_bytes]
    assert np.array_equal(got[:write_bytes], want)
    assert (got[write_bytes:] == 0xA5).all(), "wrote beyond the bytes it was given"
