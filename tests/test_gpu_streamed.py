"""Keys held in pinned host memory and imported chunk by chunk while the previous chunk is
evaluated (fss_cmp_eval_streamed): same shares as the resident path and as the oracle."""
import numpy as np
import pytest

import oracle
import paper_2006_04593_amd as fss
from paper_2006_04593_amd import workloads as W

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def to_dev(a):
    if a.dtype == np.uint32:
        a = a.view(np.int32)
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def chunked_host_keys(n, g, chunk):
    """Generate keys chunk by chunk on the device and park them in pinned host memory."""
    batch = g.batch
    total = fss.cmp_chunked_key_bytes(n, batch, chunk)
    host = [torch.empty(total, dtype=torch.uint8, pin_memory=True) for _ in range(2)]
    off = 0
    for first in range(0, batch, chunk):
        sl = slice(first, min(first + chunk, batch))
        ln = sl.stop - sl.start
        nb = fss.cmp_key_bytes(n, ln)
        k = [torch.empty(nb, dtype=torch.uint8, device="cuda:0") for _ in range(2)]
        fss.cmp_gen(n, ln, to_dev(g.alpha[sl]), to_dev(g.r[sl]), to_dev(g.seed0[sl]), to_dev(g.seed1[sl]), k[0], k[1])
        torch.cuda.synchronize()
        for j in (0, 1):
            host[j][off:off + nb].copy_(k[j])
        off += nb
    assert off == total
    return host


@pytest.mark.parametrize("batch,chunk", [(1000, 256), (64 * 50, 64 * 50), (10_000, 4096), (300_000, 65536)])
def test_streamed_eval_matches_resident_and_oracle(batch, chunk):
    print(f"case streamed batch={batch} chunk={chunk}", flush=True)
    n = 32
    w = W.uniform_workload("cmp", n, batch, seed=batch + chunk)
    g = w.gen
    host = chunked_host_keys(n, g, chunk)
    xd = to_dev(w.x)
    staging = torch.empty(2 * fss.cmp_key_bytes(n, chunk), dtype=torch.uint8, device="cuda:0")
    copy_stream = torch.cuda.Stream()
    outs = []
    for j in (0, 1):
        out = torch.full((batch,), -1, dtype=torch.int32, device="cuda:0")
        fss.cmp_eval_streamed(j, n, batch, chunk, host[j], xd, out, staging, copy_stream)
        outs.append(out.cpu().numpy().view(np.uint32))
    assert np.array_equal(outs[0] + outs[1], (w.x <= g.alpha).astype(np.uint32))
    # oracle, chunk by chunk on the very bytes that were streamed
    off = 0
    for first in range(0, batch, chunk):
        ln = min(chunk, batch - first)
        nb = fss.cmp_key_bytes(n, ln)
        if first in (0, (batch - 1) // chunk * chunk):                 # first and last chunk
            for j in (0, 1):
                kb = host[j][off:off + nb].numpy()
                assert np.array_equal(outs[j][first:first + ln], oracle.eval_("cmp", j, n, kb, w.x[first:first + ln]))
        off += nb


def test_streamed_bad_arguments():
    s = torch.cuda.Stream()
    with pytest.raises(fss.FssError):
        fss.cmp_eval_streamed(0, 32, 100, 100, None, None, None, None, s)          # chunk not a multiple of 64
    assert fss.cmp_chunked_key_bytes(32, 1000, 100) == 0
    assert fss.cmp_chunked_key_bytes(32, 1000, 256) == 808 * (3 * 256 + 256)       # 232 padded to 256
