"""The streamed evaluation with the library's built-in staging memory
(fss_cmp_eval_streamed_static, for callers that cannot allocate) against the existing entry point
with a caller-provided staging buffer (fss_cmp_eval_streamed): same shares bit for bit, on two calls
in a row, the second with a smaller input, which must not see what the first left in the array."""
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
    """Keys generated chunk by chunk on the device and parked in pinned host memory."""
    total = fss.cmp_chunked_key_bytes(n, g.batch, chunk)
    host = [torch.empty(total, dtype=torch.uint8, pin_memory=True) for _ in range(2)]
    off = 0
    for first in range(0, g.batch, chunk):
        sl = slice(first, min(first + chunk, g.batch))
        nb = fss.cmp_key_bytes(n, sl.stop - sl.start)
        k = [torch.empty(nb, dtype=torch.uint8, device="cuda:0") for _ in range(2)]
        fss.cmp_gen(n, sl.stop - sl.start, to_dev(g.alpha[sl]), to_dev(g.r[sl]), to_dev(g.seed0[sl]), to_dev(g.seed1[sl]), k[0], k[1])
        torch.cuda.synchronize()
        for j in (0, 1):
            host[j][off:off + nb].copy_(k[j])
        off += nb
    assert off == total
    return host


def test_static_staging_matches_the_caller_provided_staging():
    fss.prepare()
    limit = fss.static_staging_bytes()
    assert limit == 32 << 20
    copy_stream = torch.cuda.Stream()
    # second call: fewer elements, smaller chunks, a shorter ring, a ragged last chunk
    for n, batch, chunk in ((32, 50_000, 16_384), (24, 3_001, 1_024)):
        print(f"case static staging n={n} batch={batch} chunk={chunk}", flush=True)
        assert 2 * fss.cmp_key_bytes(n, chunk) <= limit
        w = W.uniform_workload("cmp", n, batch, seed=7 * batch + chunk)
        host = chunked_host_keys(n, w.gen, chunk)
        xd = to_dev(w.x)
        staging = torch.empty(2 * fss.cmp_key_bytes(n, chunk), dtype=torch.uint8, device="cuda:0")
        shares = []
        for j in (0, 1):
            want = torch.full((batch,), -1, dtype=torch.int32, device="cuda:0")
            got = torch.full((batch,), -2, dtype=torch.int32, device="cuda:0")
            fss.cmp_eval_streamed(j, n, batch, chunk, host[j], xd, want, staging, copy_stream)
            fss.cmp_eval_streamed_static(j, n, batch, chunk, host[j], xd, got, copy_stream)
            torch.cuda.synchronize()
            assert torch.equal(got, want), f"party {j}: static staging differs from caller-provided staging"
            shares.append(got.cpu().numpy().view(np.uint32))
        mask = np.uint32(W.ring_mask(n))
        assert np.array_equal((shares[0] + shares[1]) & mask, (w.x <= w.gen.alpha).astype(np.uint32))
        # and the oracle on the first chunk of the very bytes that were streamed
        ln = min(chunk, batch)
        for j in (0, 1):
            kb = host[j][:fss.cmp_key_bytes(n, ln)].numpy()
            assert np.array_equal(shares[j][:ln], oracle.eval_("cmp", j, n, kb, w.x[:ln]))


def test_static_staging_rejects_chunks_beyond_its_limit():
    n = 32
    too_big = 20_736 + 64                       # 2 * 808 * 20,800 bytes > 32 MiB
    assert 2 * fss.cmp_key_bytes(n, too_big) > fss.static_staging_bytes() >= 2 * fss.cmp_key_bytes(n, 20_736)
    batch = 100
    host = torch.zeros(fss.cmp_chunked_key_bytes(n, batch, too_big), dtype=torch.uint8, pin_memory=True)
    x = torch.zeros(batch, dtype=torch.int32, device="cuda:0")
    out = torch.full((batch,), 5, dtype=torch.int32, device="cuda:0")
    with pytest.raises(fss.FssError) as err:
        fss.cmp_eval_streamed_static(0, n, batch, too_big, host, x, out, torch.cuda.Stream())
    assert err.value.code == -4 and "limit" in str(err.value)
    torch.cuda.synchronize()
    assert (out == 5).all()                     # a rejected call does nothing
