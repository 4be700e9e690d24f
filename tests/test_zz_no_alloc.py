"""GPU: the flat search that allocates nothing (rago_flat_search_static) against rago_flat_search, through
the C ABI: two calls in a row, the second with a smaller input, before and after the ordinary entry point
has run, in both number formats; no device allocation by the library during the static calls."""
import pytest
import torch

import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def rb():
    from paper_2503_14649_amd import binding
    return binding


def _inputs(R, n, d, nq, seed, dtype):
    g = torch.Generator(device="cuda").manual_seed(seed)
    X = torch.nn.functional.normalize(torch.randn(R, n, d, device="cuda", generator=g), dim=2)
    X[:, n // 2] = X[:, n // 3]                                   # an exact duplicate row: ties by lower index
    Q = torch.nn.functional.normalize(X[:, :nq] + 0.3 * torch.randn(R, nq, d, device="cuda", generator=g), dim=2)
    return X.to(dtype).contiguous(), Q.to(dtype).contiguous()


def _out(R, nq, k):
    return (torch.full((R, nq, k), -7, dtype=torch.int64, device="cuda"), torch.full((R, nq, k), float("nan"), dtype=torch.float32, device="cuda"))


def _same(a, b):
    return torch.equal(a[0], b[0]) and torch.equal(a[1].view(torch.int32), b[1].view(torch.int32))


def test_static_flat_search_equals_the_allocating_one(rb):
    k = 32
    big = _inputs(6, 30000, 768, 16, 1, torch.bfloat16)
    small = _inputs(2, 1777, 768, 5, 2, torch.bfloat16)             # ragged tail, fewer queries, fewer requests
    before = rb.rago_debug_allocations()
    o1, o2 = _out(6, 16, k), _out(2, 5, k)
    rb.rago_flat_search_static(*big, k, o1)                         # first use of the static scratch on this device
    rb.rago_flat_search_static(*small, k, o2)                       # smaller input right after: stale keys and counts stay unused
    torch.cuda.synchronize()
    assert rb.rago_debug_allocations() == before
    r1 = rb.rago_flat_search(*big, k)
    r2 = rb.rago_flat_search(*small, k)
    torch.cuda.synchronize()
    assert _same(o1, r1) and _same(o2, r2)
    # again after the ordinary entry point has run, other sizes and the other format, results into fresh buffers
    h_big = _inputs(3, 9000, 256, 16, 3, torch.float16)
    h_small = _inputs(1, 255, 256, 1, 4, torch.float16)
    before = rb.rago_debug_allocations()
    o3, o4, o5 = _out(3, 16, 100), _out(1, 1, 100), _out(6, 16, k)
    rb.rago_flat_search_static(*h_big, 100, o3)
    rb.rago_flat_search_static(*h_small, 100, o4)
    rb.rago_flat_search_static(*big, k, o5)
    torch.cuda.synchronize()
    assert rb.rago_debug_allocations() == before
    assert _same(o3, rb.rago_flat_search_f16(*h_big, 100)) and _same(o4, rb.rago_flat_search_f16(*h_small, 100))
    assert _same(o5, r1)
    assert int(o4[0][0, 0, 99]) >= 0 and int((o4[0] < 0).sum()) == 0          # 255 rows >= k = 100: no padding


def test_static_flat_search_limits(rb):
    X, Q = _inputs(1, 64, 64, 2, 5, torch.bfloat16)
    Xm = X.expand(257, 64, 64).contiguous()
    Qm = Q.expand(257, 2, 64).contiguous()
    with pytest.raises(rb.RagoError) as e:
        rb.rago_flat_search_static(Xm, Qm, 4, _out(257, 2, 4))
    assert e.value.code == -6 and "256" in str(e.value)
    o = _out(256, 2, 4)
    rb.rago_flat_search_static(Xm[:256].contiguous(), Qm[:256].contiguous(), 4, o)      # the largest batch it takes
    torch.cuda.synchronize()
    assert _same(o, rb.rago_flat_search(Xm[:256].contiguous(), Qm[:256].contiguous(), 4))
