"""Caller-owned buffers with guard words on both sides: a search must write its outputs and nothing around them, and
must leave its inputs as they were.  (A kernel that writes a row too many, or pads with the wrong stride, passes a
parity test that only looks at the rows it expects.)"""
import numpy as np
import pytest
import torch

import synth
from gpu_common import dev_index
from helpers import to_np

pytestmark = pytest.mark.gpu
GUARD = 1024          # elements on either side


@pytest.fixture(scope="module")
def rb():
    from paper_2503_14649_amd import binding
    return binding


def guarded(shape, dtype, fill):
    n = int(np.prod(shape))
    buf = torch.full((n + 2 * GUARD,), fill, dtype=dtype, device="cuda")
    return buf, buf[GUARD:GUARD + n].view(*shape)


def guards_intact(buf, fill):
    return bool((buf[:GUARD] == fill).all()) and bool((buf[-GUARD:] == fill).all())


@pytest.mark.parametrize("kernel", ["auto", "wide", "narrow", "wave"])
@pytest.mark.parametrize("nq,nprobe,k", [(1, 6, 10), (5, 3, 128), (40, 9, 7)])
def test_ivfpq_search_writes_only_its_outputs(rb, kernel, nq, nprobe, k):
    ix = to_np(synth.random_index(n=6000, d=64, m=16, nlist=9, seed=5, empty_lists=(2,)))
    h = rb.rago_index_wrap(dev_index(ix))
    rb.rago_debug_force_scan_kernel(kernel)
    try:
        g = torch.Generator().manual_seed(3)
        qbuf, Q = guarded((nq, 64), torch.float32, 7.0)
        Q.copy_(torch.nn.functional.normalize(torch.randn(nq, 64, generator=g), dim=1))
        q_before = Q.clone()
        b_ids, ids = guarded((nq, k), torch.int64, -77)
        b_sc, sc = guarded((nq, k), torch.float32, 123.5)
        b_is, isc = guarded((nq, k), torch.int32, -99)
        ref = rb.rago_ivfpq_search(h, Q.clone(), nprobe, k)
        rb.rago_ivfpq_search(h, Q, nprobe, k, out=(ids, sc, isc))
        torch.cuda.synchronize()
        assert guards_intact(b_ids, -77) and guards_intact(b_sc, 123.5) and guards_intact(b_is, -99)
        assert guards_intact(qbuf, 7.0) and torch.equal(Q, q_before)
        assert torch.equal(ids, ref[0]) and torch.equal(isc, ref[2])
        assert not bool((ids == -77).any()) and not bool((isc == -99).any())        # every output element was written
    finally:
        rb.rago_debug_force_scan_kernel("auto")
        rb.rago_index_free(h)


@pytest.mark.parametrize("fmt", [torch.bfloat16, torch.float16])
@pytest.mark.parametrize("R,n,nqr,k", [(1, 17, 3, 5), (3, 1000, 16, 32), (2, 40, 1, 128)])
def test_flat_search_writes_only_its_outputs(rb, fmt, R, n, nqr, k):
    g = torch.Generator().manual_seed(4)
    cbuf, C = guarded((R, n, 128), fmt, 3.0)
    C.copy_(torch.nn.functional.normalize(torch.randn(R, n, 128, generator=g), dim=2).to(fmt))
    qbuf, Q = guarded((R, nqr, 128), fmt, 3.0)
    Q.copy_(torch.nn.functional.normalize(torch.randn(R, nqr, 128, generator=g), dim=2).to(fmt))
    c_before, q_before = C.clone(), Q.clone()
    b_ids, ids = guarded((R, nqr, k), torch.int64, -77)
    b_sc, sc = guarded((R, nqr, k), torch.float32, 123.5)
    fn = rb.rago_flat_search_f16 if fmt == torch.float16 else rb.rago_flat_search
    ref = fn(C.clone(), Q.clone(), k)
    fn(C, Q, k, out=(ids, sc))
    torch.cuda.synchronize()
    assert guards_intact(b_ids, -77) and guards_intact(b_sc, 123.5)
    assert guards_intact(cbuf, 3.0) and guards_intact(qbuf, 3.0) and torch.equal(C, c_before) and torch.equal(Q, q_before)
    assert torch.equal(ids, ref[0])
    assert not bool((ids == -77).any())
