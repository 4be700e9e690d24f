"""GPU parity: exact bf16 flat search (HIP, MFMA) against the CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def rb():
    from paper_2503_14649_amd import binding
    return binding


def _bits(t):
    return t.cpu().view(torch.int16).numpy().view(np.uint16)


def _check(rb, corpus, queries, k):
    """bf16 tensors go through rago_flat_search, fp16 tensors through rago_flat_search_f16."""
    half = corpus.dtype == torch.float16
    fn = rb.rago_flat_search_f16 if half else rb.rago_flat_search
    gi, gs = fn(corpus.cuda(), queries.cuda(), k)
    torch.cuda.synchronize()
    gi, gs = gi.cpu().numpy(), gs.cpu().numpy()
    oi, osc = oracle.flat_search(_bits(corpus), _bits(queries), k, fmt="f16" if half else "bf16")
    R, nq = queries.shape[:2]
    n = corpus.shape[1]
    kk = min(k, n)
    assert np.all(gi[:, :, kk:] == -1) and np.all(np.isneginf(gs[:, :, kk:]))
    # scores: bf16 (and fp16) products are exact in fp32, only the accumulation order differs; |q||x| ~ 1
    assert np.max(np.abs(gs[:, :, :kk] - osc[:, :, :kk])) < 1e-4
    ov = np.mean([len(set(gi[r, q, :kk].tolist()) & set(oi[r, q, :kk].tolist())) / kk for r in range(R) for q in range(nq)])
    assert ov >= 0.999, ov
    # each returned score is the true score of the returned row (fp64 reference), order is non-increasing
    ref = torch.einsum("rqd,rnd->rqn", queries.double(), corpus.double()).numpy()
    for r in range(R):
        for q in range(nq):
            assert np.max(np.abs(ref[r, q][gi[r, q, :kk]] - gs[r, q, :kk])) < 1e-5
            assert np.all(np.diff(gs[r, q, :kk]) <= 0)
            same = np.diff(gs[r, q, :kk]) == 0
            assert np.all(np.diff(gi[r, q, :kk])[same] > 0)          # equal scores: lower row first
    return gi, gs, oi, osc


@pytest.mark.parametrize("R,n,nq,k", [(2, 700, 16, 32), (3, 5000, 5, 128), (1, 20, 16, 32), (2, 1, 3, 4), (2, 30000, 16, 32)])
def test_flat_matches_oracle(rb, R, n, nq, k):
    print(f"[flat] R={R} n={n} nq={nq} k={k}", flush=True)
    cfg = synth.FLAT
    corpus, queries = synth.make_flat(cfg, requests=R, n=n)
    queries = queries[:, :nq].contiguous()
    _check(rb, corpus, queries, k)


def test_flat_duplicate_rows_tie_by_lower_index(rb):
    cfg = synth.FLAT
    corpus, queries = synth.make_flat(cfg, requests=1, n=3000)
    for i in (17, 300, 301, 1700, 2999):
        corpus[0, i] = corpus[0, 5]
    queries[0, 0] = corpus[0, 5]
    gi, gs, oi, osc = _check(rb, corpus, queries, 32)
    assert gi[0, 0, :6].tolist() == [5, 17, 300, 301, 1700, 2999]
    assert np.array_equal(gi[0, 0, :6], oi[0, 0, :6])


def test_flat_other_dims_and_errors(rb):
    g = torch.Generator().manual_seed(3)
    for d in (64, 128, 256, 1024):
        corpus = torch.nn.functional.normalize(torch.randn(2, 900, d, generator=g), dim=2).to(torch.bfloat16)
        queries = torch.nn.functional.normalize(torch.randn(2, 7, d, generator=g), dim=2).to(torch.bfloat16)
        _check(rb, corpus, queries, 10)
    c = torch.zeros(1, 10, 96, dtype=torch.bfloat16).cuda()
    q = torch.zeros(1, 2, 96, dtype=torch.bfloat16).cuda()
    with pytest.raises(rb.RagoError) as e:
        rb.rago_flat_search(c, q, 4)
    assert e.value.code == -6
    c = torch.zeros(1, 10, 128, dtype=torch.bfloat16).cuda()
    q = torch.zeros(1, 17, 128, dtype=torch.bfloat16).cuda()
    with pytest.raises(rb.RagoError) as e:
        rb.rago_flat_search(c, q, 4)
    assert e.value.code == -1
    gi, gs = rb.rago_flat_search(c[:, :0].contiguous(), q[:, :4].contiguous(), 4)   # empty corpus: all padding
    assert torch.all(gi == -1)


# ------------------------------------------------------------------ IEEE binary16 embeddings
@pytest.mark.parametrize("R,n,nq,k", [(2, 700, 16, 32), (3, 5000, 5, 128), (1, 20, 16, 32), (2, 1, 3, 4), (2, 30000, 16, 32)])
def test_flat_f16_matches_oracle(rb, R, n, nq, k):
    print(f"[flat f16] R={R} n={n} nq={nq} k={k}", flush=True)
    corpus, queries = synth.make_flat(synth.FLAT, requests=R, n=n)
    corpus, queries = corpus.float().half(), queries[:, :nq].float().half().contiguous()
    _check(rb, corpus, queries, k)


def test_flat_f16_ties_subnormals_and_dims(rb):
    corpus, queries = synth.make_flat(synth.FLAT, requests=1, n=3000)
    corpus, queries = corpus.float().half(), queries.float().half()
    for i in (17, 300, 301, 1700, 2999):
        corpus[0, i] = corpus[0, 5]
    queries[0, 0] = corpus[0, 5]
    gi, gs, oi, osc = _check(rb, corpus, queries, 32)
    assert gi[0, 0, :6].tolist() == [5, 17, 300, 301, 1700, 2999]
    # a corpus scaled by 2^-12: nearly every entry is a subnormal fp16 number and must keep its value
    g = torch.Generator().manual_seed(11)
    for d in (64, 256, 768, 1024):
        c = (torch.nn.functional.normalize(torch.randn(2, 900, d, generator=g), dim=2) * 2.0 ** -12).half()
        q = (torch.nn.functional.normalize(torch.randn(2, 7, d, generator=g), dim=2) * 2.0 ** 10).half()
        bits = _bits(c)
        assert np.mean(((bits >> 10) & 31) == 0) > 0.5
        gi, gs, oi, osc = _check(rb, c, q, 10)
        assert np.all(np.abs(gs[:, :, 0]) > 1e-3)                       # scores of order 2^-2 cos: nothing was flushed to zero
    with pytest.raises(AssertionError):                                  # the binding refuses the wrong number format
        rb.rago_flat_search_f16(torch.zeros(1, 10, 128, dtype=torch.bfloat16).cuda(), torch.zeros(1, 2, 128, dtype=torch.bfloat16).cuda(), 4)


@pytest.mark.parametrize("kind", ["large_scores", "ascending_scores", "all_equal"])
def test_flat_scores_outside_the_histogram_range(rb, kind):
    """The selection's histogram covers scores in [-1, 1]; embeddings that are not normalised fall outside it, where
    the filter passes everything and the candidate areas are cut back again and again.  Results must not change.
    `ascending_scores`: every row beats all rows before it (every row is a candidate in any case);
    `all_equal`: one score for the whole corpus (ties by row)."""
    g = torch.Generator().manual_seed(21)
    R, n, d, nq, k = 2, 20000, 128, 16, 32
    if kind == "large_scores":
        corpus = (torch.randn(R, n, d, generator=g) * 3.0).to(torch.bfloat16)
        queries = (torch.randn(R, nq, d, generator=g) * 3.0).to(torch.bfloat16)
    elif kind == "ascending_scores":
        base = torch.nn.functional.normalize(torch.randn(R, 1, d, generator=g), dim=2)
        corpus = (base * torch.linspace(0.5, 40.0, n).view(1, n, 1)).to(torch.bfloat16)
        queries = base.expand(R, nq, d).contiguous().to(torch.bfloat16)
    else:
        base = torch.nn.functional.normalize(torch.randn(R, 1, d, generator=g), dim=2)
        corpus = base.expand(R, n, d).contiguous().to(torch.bfloat16)
        queries = base.expand(R, nq, d).contiguous().to(torch.bfloat16)
    gi, gs = rb.rago_flat_search(corpus.cuda(), queries.cuda(), k)
    torch.cuda.synchronize()
    gi, gs = gi.cpu().numpy(), gs.cpu().numpy()
    oi, osc = oracle.flat_search(_bits(corpus), _bits(queries), k)
    scale = float(np.abs(osc).max())
    assert np.max(np.abs(gs - osc)) <= 1e-4 * max(scale, 1.0)
    if kind == "all_equal":
        assert np.array_equal(gi, oi)                          # rows 0 .. k-1
    else:
        ov = np.mean([len(set(gi[r, q].tolist()) & set(oi[r, q].tolist())) / k for r in range(R) for q in range(nq)])
        assert ov >= 0.999, ov


def test_flat_search_replayed_from_a_hip_graph(rb):
    """After one call that sizes the library's workspace the flat search only enqueues kernels, so a caller may capture
    it; every replay (with eager calls and synchronisation in between) must equal the eager call on the same data."""
    cfg = synth.FLAT
    corpus, queries = synth.make_flat(cfg, requests=3, n=9000)
    c_static, q_static = corpus.cuda(), queries.cuda()
    k = 20
    out = (torch.empty(3, cfg.nq, k, dtype=torch.int64, device="cuda"), torch.empty(3, cfg.nq, k, dtype=torch.float32, device="cuda"))
    rb.rago_flat_search(c_static, q_static, k, out=out)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        rb.rago_flat_search(c_static, q_static, k, out=out)
    g = torch.Generator().manual_seed(5)
    for rep in range(4):
        perm = torch.randperm(9000, generator=g)
        c_new = corpus[:, perm].contiguous()                           # the same rows in another order
        c_static.copy_(c_new.cuda())
        graph.replay()
        torch.cuda.synchronize()
        gi, gs = out[0].cpu().numpy().copy(), out[1].cpu().numpy().copy()
        ei, es = rb.rago_flat_search(c_new.cuda(), q_static, k)        # eager work between replays
        torch.cuda.synchronize()
        assert np.array_equal(ei.cpu().numpy(), gi) and np.array_equal(es.cpu().numpy(), gs), rep
        oi, osc = oracle.flat_search(_bits(c_new), _bits(queries), k)
        assert np.max(np.abs(gs - osc)) < 1e-4
