"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times.

The hyperscale shard (1e9 x 96-byte codes, nlist 65536) is generated on the GPU (~30 s); the
oracle recomputes sampled queries one by one over the lists they probe (copied to the host),
and properties that hold at any size are checked on every query of the batch.
"""
import numpy as np
import pytest
import torch

import oracle
import synth
from bench import host_subindex

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def rb():
    from paper_2503_14649_amd import binding
    return binding


@pytest.fixture(scope="module")
def hyper(rb):
    cfg = synth.HYPER
    print(f"[fullsize] building {cfg.name}: n={cfg.n} nlist={cfg.nlist}", flush=True)
    index = synth.build_index(cfg, device="cuda:0", keep_vectors=False)
    Q = synth.make_queries(cfg, cfg.nq, device="cuda:0")
    Qi = synth.make_queries(cfg, 16, device="cuda:0", stream=7)
    # oracle inputs for the sampled queries, taken from the generator's plain arrays
    cen = index["centroids"].cpu().numpy()
    samples = {}
    for name, qs, nprobe in (("batch", Q[:32], cfg.nprobe), ("iter", Qi[:16], synth.ITER_NPROBE)):
        qn = qs.cpu().numpy()
        pr = oracle.select(oracle.coarse(qn, cen), nprobe)
        samples[name] = (qn, host_subindex(index, pr))
    torch.cuda.empty_cache()
    h = rb.rago_index_wrap(index, 0)
    print("[fullsize] index wrapped", flush=True)
    # (the generator's plain arrays stay: the Euclidean test at the end of this file wraps them once more, after
    # freeing this handle - two laid-out copies of the codes would not fit beside them)
    state = {"h": h, "index": index, "cen": cen}
    _HYPER_STATE.update(state=state)
    yield cfg, h, Q, Qi, samples
    if state["h"] is not None:
        rb.rago_index_free(state["h"])
    _HYPER_STATE.clear()


_HYPER_STATE = {}


def test_hyperscale_batch_matches_oracle_on_samples(hyper, rb):
    cfg, h, Q, Qi, samples = hyper
    ids, scores, isc = rb.rago_ivfpq_search(h, Q, cfg.nprobe, cfg.k)       # the timed configuration: 1024 x 128 x 100
    torch.cuda.synchronize()
    ids, scores, isc = ids.cpu().numpy(), scores.cpu().numpy(), isc.cpu().numpy()
    qn, sub = samples["batch"]
    ref = oracle.ivfpq_search(qn, sub, cfg.nprobe, cfg.k)
    n = len(qn)
    overlap = np.mean([len(set(ids[q].tolist()) & set(ref["ids"][q].tolist())) / cfg.k for q in range(n)])
    assert overlap >= 0.999
    assert np.array_equal(ids[:n], ref["ids"]) and np.array_equal(isc[:n], ref["iscores"])
    assert np.array_equal(scores[:n], ref["scores"])
    # properties of every query of the batch
    assert ids.min() >= 0 and ids.max() < cfg.n
    assert all(len(set(row.tolist())) == cfg.k for row in ids)
    d_isc = np.diff(isc.astype(np.int64), axis=1)
    assert np.all(d_isc <= 0)
    assert np.all(np.diff(ids, axis=1)[d_isc == 0] > 0)                       # equal scores: ascending ids
    ratio = scores / isc
    assert np.allclose(ratio, ratio[:, :1], rtol=1e-6)                         # score = integer score x per-query step
    cnt = rb.rago_debug_counters(h)
    assert cnt[3] == 0 and cnt[5] == 0
    assert cnt[2] > 0.5 * cfg.n * cfg.m * cfg.nprobe / cfg.nlist * cfg.nq      # algorithmic bytes ~ N m nprobe/nlist per query


def test_iterative_rounds_match_oracle(hyper, rb):
    cfg, h, Q, Qi, samples = hyper
    qn, sub = samples["iter"]
    for b in synth.ITER_BATCHES:                 # 1, 4, 16
        ids, scores, isc = rb.rago_ivfpq_search(h, Qi[:b].contiguous(), synth.ITER_NPROBE, synth.ITER_K)
        torch.cuda.synchronize()
        ref = oracle.ivfpq_search(qn[:b], sub, synth.ITER_NPROBE, synth.ITER_K)
        assert np.array_equal(ids.cpu().numpy(), ref["ids"]) and np.array_equal(isc.cpu().numpy(), ref["iscores"])


def test_hyperscale_batch_is_deterministic(hyper, rb):
    """The grouping of (query, list) pairs uses atomics, so which workgroup scans what differs from run to run:
    the outputs must not (integer scores and a total order leave one answer)."""
    cfg, h, Q, Qi, samples = hyper
    a = [t.clone() for t in rb.rago_ivfpq_search(h, Q, cfg.nprobe, cfg.k)]
    b = rb.rago_ivfpq_search(h, Q, cfg.nprobe, cfg.k)
    torch.cuda.synchronize()
    for x, y in zip(a, b):
        assert torch.equal(x.view(torch.uint8), y.view(torch.uint8))


def test_tiny_config_every_query(rb):
    """1M x 128, m 16, nlist 1024; 64 queries, nprobe 16, k 10: the whole batch against the oracle."""
    cfg = synth.TINY
    index = synth.build_index(cfg, device="cuda:0", keep_vectors=False)
    Q = synth.make_queries(cfg, cfg.nq, device="cuda:0")
    h = rb.rago_index_wrap(index, 0)
    ids, scores, isc = rb.rago_ivfpq_search(h, Q, cfg.nprobe, cfg.k)
    torch.cuda.synchronize()
    ref = oracle.ivfpq_search(Q.cpu().numpy(), {k: v.cpu().numpy() for k, v in index.items()}, cfg.nprobe, cfg.k)
    assert np.array_equal(ids.cpu().numpy(), ref["ids"]) and np.array_equal(isc.cpu().numpy(), ref["iscores"])
    assert np.array_equal(scores.cpu().numpy(), ref["scores"])
    rb.rago_index_free(h)


def test_mid_config_samples(rb):
    """10M x 768, m 96, nlist 16384; 256 queries, nprobe 64, k 100: 24 sampled queries against the oracle."""
    cfg = synth.MID
    index = synth.build_index(cfg, device="cuda:0", keep_vectors=False)
    Q = synth.make_queries(cfg, cfg.nq, device="cuda:0")
    qn = Q[:24].cpu().numpy()
    sub = host_subindex(index, oracle.select(oracle.coarse(qn, index["centroids"].cpu().numpy()), cfg.nprobe))
    h = rb.rago_index_wrap(index, 0)
    ids, scores, isc = rb.rago_ivfpq_search(h, Q, cfg.nprobe, cfg.k)
    torch.cuda.synchronize()
    ref = oracle.ivfpq_search(qn, sub, cfg.nprobe, cfg.k)
    assert np.array_equal(ids.cpu().numpy()[:24], ref["ids"]) and np.array_equal(isc.cpu().numpy()[:24], ref["iscores"])
    assert rb.rago_debug_counters(h)[3] == 0
    rb.rago_index_free(h)


@pytest.mark.parametrize("variant", ["l2", "pq4", "pq4_l2"])
def test_mid_config_other_metrics_and_code_widths(rb, variant):
    """The mid configuration under the Euclidean metric, with 4-bit codes (192 sub-quantisers of 16 codewords =
    96 code bytes), and both: 12 sampled queries against the oracle."""
    metric = "l2" if variant.endswith("l2") else "ip"
    cfg = synth.MID if variant == "l2" else synth.MID.scaled(m=192, ksub=16)
    print(f"[fullsize] mid {variant}: m={cfg.m} ksub={cfg.ksub} metric={metric}", flush=True)
    index = synth.build_index(cfg, device="cuda:0", keep_vectors=False)
    Q = synth.make_queries(cfg, cfg.nq, device="cuda:0")
    qn = Q[:12].cpu().numpy()
    sub = host_subindex(index, oracle.select(oracle.coarse(qn, index["centroids"].cpu().numpy(), metric=metric), cfg.nprobe))
    h = rb.rago_index_wrap(index, 0, metric=metric)
    ids, scores, isc = rb.rago_ivfpq_search(h, Q, cfg.nprobe, cfg.k)
    torch.cuda.synchronize()
    ref = oracle.ivfpq_search(qn, sub, cfg.nprobe, cfg.k, metric=metric)
    assert np.array_equal(ids.cpu().numpy()[:12], ref["ids"]) and np.array_equal(isc.cpu().numpy()[:12], ref["iscores"])
    assert np.array_equal(scores.cpu().numpy()[:12], ref["scores"])
    cnt = rb.rago_debug_counters(h)
    assert cnt[3] == 0
    if metric == "l2":
        assert cnt[5] == 0 and cnt[4] < 0.02 * 2 * cfg.nq * cfg.nprobe * 96 * 256   # fp32 decided all but a few entries
    rb.rago_index_free(h)


def test_flat_full_size_matches_oracle_on_samples(rb):
    cfg = synth.FLAT
    corpus, queries = synth.make_flat(cfg, device="cuda:0")                   # 32 x 100000 x 768 bf16
    gi, gs = rb.rago_flat_search(corpus, queries, cfg.k)
    torch.cuda.synchronize()
    gi, gs = gi.cpu().numpy(), gs.cpu().numpy()
    for r in (0, 17):
        cb = corpus[r:r + 1].cpu().view(torch.int16).numpy().view(np.uint16)
        qb = queries[r:r + 1].cpu().view(torch.int16).numpy().view(np.uint16)
        oi, osc = oracle.flat_search(cb, qb, cfg.k)
        assert np.max(np.abs(gs[r] - osc[0])) < 1e-4
        ov = np.mean([len(set(gi[r, q].tolist()) & set(oi[0, q].tolist())) / cfg.k for q in range(cfg.nq)])
        assert ov >= 0.999, ov
    assert gi.min() >= 0 and gi.max() < cfg.n
    assert np.all(np.diff(gs, axis=2) <= 0)
    # the same embeddings as IEEE binary16
    ch, qh = corpus.to(torch.float16), queries.to(torch.float16)
    hi, hs = rb.rago_flat_search_f16(ch, qh, cfg.k)
    torch.cuda.synchronize()
    hi, hs = hi.cpu().numpy(), hs.cpu().numpy()
    r = 5
    cb = ch[r:r + 1].cpu().view(torch.int16).numpy().view(np.uint16)
    qb = qh[r:r + 1].cpu().view(torch.int16).numpy().view(np.uint16)
    oi, osc = oracle.flat_search(cb, qb, cfg.k, fmt="f16")
    assert np.max(np.abs(hs[r] - osc[0])) < 1e-4
    assert np.mean([len(set(hi[r, q].tolist()) & set(oi[0, q].tolist())) / cfg.k for q in range(cfg.nq)]) >= 0.999


def test_hyperscale_batch_under_the_euclidean_metric(hyper, rb):
    """The same billion-vector arrays wrapped with the Euclidean metric (per-pair tables built on the matrix cores, the
    wide scan fed full tables): 8 sampled queries of the 1024 x 128 x 100 batch against the oracle.  Runs last in this
    file: it frees the inner-product handle first."""
    cfg, h, Q, Qi, samples = hyper
    state = _HYPER_STATE["state"]
    rb.rago_index_free(state["h"])
    state["h"] = None
    torch.cuda.empty_cache()
    h2 = rb.rago_index_wrap(state["index"], 0, metric="l2")
    try:
        ns = 8
        qn = Q[:ns].cpu().numpy()
        pr = oracle.select(oracle.coarse(qn, state["cen"], metric="l2"), cfg.nprobe)
        sub = host_subindex(state["index"], pr)
        ids, scores, isc = rb.rago_ivfpq_search(h2, Q, cfg.nprobe, cfg.k)
        torch.cuda.synchronize()
        ref = oracle.ivfpq_search(qn, sub, cfg.nprobe, cfg.k, metric="l2")
        assert np.array_equal(ids[:ns].cpu().numpy(), ref["ids"]) and np.array_equal(isc[:ns].cpu().numpy(), ref["iscores"])
        assert np.array_equal(scores[:ns].cpu().numpy(), ref["scores"])
        assert bool((scores <= 0).all())                     # similarities are minus squared distances
        assert rb.rago_debug_counters(h2)[3] == 0
    finally:
        rb.rago_index_free(h2)


def test_hyperscale_batch_with_4bit_codes(hyper, rb):
    """A billion-vector index with 4-bit codes (192 sub-quantisers of 16 codewords = the same 96 bytes per vector):
    8 sampled queries of the 1024 x 128 x 100 batch against the oracle.  Frees what the tests before it hold first
    (two billion-vector indexes do not fit side by side)."""
    state = _HYPER_STATE["state"]
    if state["h"] is not None:
        rb.rago_index_free(state["h"])
        state["h"] = None
    state["index"].clear()
    torch.cuda.empty_cache()
    cfg = synth.HYPER.scaled(m=192, ksub=16)
    print(f"[fullsize] building {cfg.name} with 4-bit codes: n={cfg.n} nlist={cfg.nlist}", flush=True)
    index = synth.build_index(cfg, device="cuda:0", keep_vectors=False)
    Q = synth.make_queries(cfg, cfg.nq, device="cuda:0")
    ns = 8
    qn = Q[:ns].cpu().numpy()
    sub = host_subindex(index, oracle.select(oracle.coarse(qn, index["centroids"].cpu().numpy()), cfg.nprobe))
    torch.cuda.empty_cache()
    h = rb.rago_index_wrap(index, 0)
    try:
        ids, scores, isc = rb.rago_ivfpq_search(h, Q, cfg.nprobe, cfg.k)
        torch.cuda.synchronize()
        ref = oracle.ivfpq_search(qn, sub, cfg.nprobe, cfg.k)
        assert np.array_equal(ids[:ns].cpu().numpy(), ref["ids"]) and np.array_equal(isc[:ns].cpu().numpy(), ref["iscores"])
        assert np.array_equal(scores[:ns].cpu().numpy(), ref["scores"])
        assert rb.rago_debug_counters(h)[3] == 0
    finally:
        rb.rago_index_free(h)
