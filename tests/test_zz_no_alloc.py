"""pk_search_noalloc (the search whose workspace is a fixed device array of the library, for
callers that cannot call hipMalloc) against pk_search: two calls in a row, the second with a
smaller input, bit for bit; then the size limit.  Collected last: it shares one device array
with nothing else, but a failure here must not hide the tests before it."""
import ctypes as C

import numpy as np
import pytest
import torch

import training
from gpu_util import dev
from paper_2602_21477_amd import binding as B
from paper_2602_21477_amd import workload as W

pytestmark = pytest.mark.gpu


def say(msg):
    print(f"[no_alloc] {msg}", flush=True)


@pytest.mark.parametrize("storage,metric", [(B.PK_F32, B.PK_METRIC_IP), (B.PK_F16, B.PK_METRIC_L2)])
def test_noalloc_search_equals_pk_search_on_two_calls_in_a_row(gpu_device, storage, metric):
    cfg = W.scaled(W.C1, n=12000)
    x = W.vectors(cfg, 0, cfg.n)
    if storage == B.PK_F16:
        x = x.astype(np.float16).astype(np.float32)
    cent = training.train_centroids(cfg, x)
    ix = B.Index(dev(cent), dev(x), metric=metric, storage=storage, insert_reserve=2048)
    try:
        ix.insert(dev(W.inserts(cfg, 0, 300)))  # delta pages take part
        big, small = dev(W.queries(cfg, 0, 200)), dev(W.queries(cfg, 1, 37))
        # the reference rows first (pk_search may grow the handle's workspace: that is its business)
        want = [ix.search(big, 10, 8), ix.search(small, 7, 5)]
        torch.cuda.synchronize()
        assert 0 < B.pk_search_noalloc_bytes(ix.handle, 200, 10, 8) <= B.PK_NOALLOC_WORKSPACE_BYTES
        out = []
        for q, k, nprobe in ((big, 10, 8), (small, 7, 5)):
            ids = torch.full((q.shape[0], k), -7, dtype=torch.int64, device="cuda")
            dist = torch.full((q.shape[0], k), float("nan"), dtype=torch.float32, device="cuda")
            out.append((ids, dist))
        torch.cuda.synchronize()
        free0, _ = torch.cuda.mem_get_info()
        say(f"two calls in a row, storage={storage} metric={metric}")
        B.pk_search_noalloc(ix.handle, big, 10, 8, *out[0])
        B.pk_search_noalloc(ix.handle, small, 7, 5, *out[1])  # smaller input, same array, no wait between
        torch.cuda.synchronize()
        free1, _ = torch.cuda.mem_get_info()
        assert free1 >= free0, "device memory was allocated during pk_search_noalloc"
        for (gi, gd), (wi, wd) in zip(out, want):
            assert torch.equal(gi, wi)
            assert torch.equal(gd, wd)
        # and again the large one after the small one: stale contents of the array do not leak
        B.pk_search_noalloc(ix.handle, big, 10, 8, *out[0])
        torch.cuda.synchronize()
        assert torch.equal(out[0][0], want[0][0]) and torch.equal(out[0][1], want[0][1])
        assert ix.stats().device_error == 0
    finally:
        ix.close()


def test_noalloc_search_rejects_what_does_not_fit(gpu_device):
    cfg = W.scaled(W.C1, n=12000)
    x = W.vectors(cfg, 0, cfg.n)
    cent = training.train_centroids(cfg, x)
    ix = B.Index(dev(cent), dev(x), metric=B.PK_METRIC_IP)
    try:
        nq = 1
        while B.pk_search_noalloc_bytes(ix.handle, nq, 10, 64) <= B.PK_NOALLOC_WORKSPACE_BYTES:
            nq *= 2
            assert nq < 1 << 24
        q = torch.zeros((nq, cfg.d), dtype=torch.float32, device="cuda")
        ids = torch.empty((nq, 10), dtype=torch.int64, device="cuda")
        dist = torch.empty((nq, 10), dtype=torch.float32, device="cuda")
        say(f"rejection at nq={nq}")
        with pytest.raises(B.PancakeError) as e:
            B.pk_search_noalloc(ix.handle, q, 10, 64, ids, dist)
        assert e.value.status == B.PK_ERR_WORKSPACE
        assert "workspace" in B.strerror(B.PK_ERR_WORKSPACE)
        # argument errors as in pk_search
        assert B.lib().pk_search_noalloc(None, None, 1, 1, 1, None, None, None) == B.PK_ERR_BAD_HANDLE
        assert B.pk_search_noalloc_bytes(ix.handle, 0, 10, 8) == 0
    finally:
        ix.close()
