"""CPU-only pins of the oracle against closed forms, identities, library routines and brute force."""
import os

import numpy as np
import pytest
import torch

import oracle
import synth
from helpers import list_of, reconstruct, to_np, topk_desc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


@pytest.fixture(scope="module")
def rnd():
    ix = to_np(synth.random_index(n=1500, d=16, m=4, nlist=8, seed=11, empty_lists=(3,), dup_codes=40,
                                  shuffle_ids=True))
    g = torch.Generator().manual_seed(5)
    Q = torch.nn.functional.normalize(torch.randn(6, 16, generator=g), dim=1).numpy()
    return ix, Q


@pytest.fixture(scope="module")
def trained():
    cfg = synth.TINY.scaled(n=20000, d=32, m=8, nlist=32, components=32, train_n=8000, pq_train_n=4096,
                            kmeans_iters=5)
    ix = to_np(synth.build_index(cfg))
    Q = synth.make_queries(cfg, 12).numpy()
    return cfg, ix, Q


# ------------------------------------------------------------------ step 1: coarse = a plain matmul
def test_coarse_equals_fp64_matmul(rnd):
    ix, Q = rnd
    S = oracle.coarse(Q, ix["centroids"])
    ref = (Q.astype(np.float64) @ ix["centroids"].astype(np.float64).T)
    assert S.shape == ref.shape and S.dtype == np.float32
    assert np.max(np.abs(S - ref)) <= 2 ** -24 * np.max(np.abs(ref)) * 1.01
    # a transposed operand or a wrong stride would break the per-entry dot product
    assert abs(S[2, 5] - float(np.dot(Q[2].astype(np.float64), ix["centroids"][5].astype(np.float64)))) < 1e-7


# ------------------------------------------------------------------ step 2: selection with forced ties
def test_select_order_and_ties():
    S = np.array([[0.5, 0.9, 0.9, -1.0, 0.5, 0.9, 0.1],
                  [0.0, 0.0, 0.0, 0.0, 0.0, 0.0, 0.0]], np.float32)
    p = oracle.select(S, 4)
    assert p.tolist() == [[1, 2, 5, 0], [0, 1, 2, 3]]
    g = np.random.default_rng(0)
    S = g.integers(0, 6, size=(5, 40)).astype(np.float32)      # many exact ties
    p = oracle.select(S, 9)
    for q in range(5):
        ref, _ = topk_desc(S[q].astype(np.float64), np.arange(40), 9)
        assert p[q].tolist() == ref.tolist()
    with pytest.raises(RuntimeError):
        oracle.select(S, 41)                                   # nprobe > nlist is an error


# ------------------------------------------------------------------ step 3: table identities
def test_lut_sum_identity_is_score_of_reconstruction(rnd):
    ix, Q = rnd
    probes = np.tile(np.arange(8, dtype=np.int32), (Q.shape[0], 1))     # every list, in list order
    L = oracle.lut_f32(Q, ix["centroids"], ix["codebooks"], probes)
    xhat, lst, codes = reconstruct(ix), list_of(ix), ix["codes"]
    ref = Q.astype(np.float64) @ xhat.T                                  # [nq][n]
    m = codes.shape[1]
    for q in range(Q.shape[0]):
        got = sum(L[q, lst, j, codes[:, j]].astype(np.float64) for j in range(m))
        assert np.max(np.abs(got - ref[q])) < 1e-6


def test_lut_difference_between_lists_is_constant_in_c(rnd):
    ix, Q = rnd
    probes = np.tile(np.array([0, 5, 7], np.int32), (Q.shape[0], 1))
    L = oracle.lut_f32(Q, ix["centroids"], ix["codebooks"], probes).astype(np.float64)
    dsub = 16 // 4
    for a, b in ((0, 1), (1, 2)):
        diff = L[:, a] - L[:, b]                                         # [nq][m][256]
        assert np.max(diff.max(axis=2) - diff.min(axis=2)) < 1e-6
        la, lb = probes[0, a], probes[0, b]
        for j in range(4):                                               # and equals <q_j, C[la]_j - C[lb]_j>
            sl = slice(j * dsub, (j + 1) * dsub)
            ref = Q[:, sl].astype(np.float64) @ (ix["centroids"][la, sl] - ix["centroids"][lb, sl]).astype(np.float64)
            assert np.max(np.abs(diff[:, j, 17] - ref)) < 1e-6


# ------------------------------------------------------------------ steps 3-6: integer-exact worked case
def _read_golden():
    vals = {}
    for line in open(os.path.join(GOLDEN, "integer_case.txt")):
        if line.startswith("#") or "=" not in line:
            continue
        k, v = line.split("=")
        vals[k.strip()] = np.array([float(t) for t in v.split()], np.float32)
    return vals


def test_integer_exact_case():
    v = _read_golden()
    q = v["q"][None, :]
    C = np.stack([v["C0"], v["C1"]])
    CB = np.zeros((2, 256, 2), np.float32)
    c = np.arange(256)
    CB[0, :, 0] = c
    CB[1, :, 0] = (c % 16) - 8
    CB[1, :, 1] = (c // 16) - 8
    g = np.random.default_rng(3)
    n0, n1 = 300, 200
    codes = g.integers(0, 256, size=(n0 + n1, 2)).astype(np.uint8)
    codes[0] = (255, 0)
    codes[1] = (0, 255)
    off = np.array([0, n0, n0 + n1], np.int64)
    ids = np.arange(n0 + n1, dtype=np.int64)
    probes = np.array([[1, 0]], np.int32)
    L = oracle.lut_f32(q, C, CB, probes)
    LUT8, B, delta = oracle.quantise(L)
    assert delta[0] == 1.0
    assert LUT8[0, :, 0].min() == 0 and LUT8[0, :, 0].max() == 255 and LUT8[0, :, 1].max() == 75
    k = n0 + n1
    oi, ois, osc = oracle.scan_topk(probes, LUT8, B, delta, off, codes, ids, k)
    # closed form: exact integer inner product with the reconstruction
    lst = np.repeat([0, 1], [n0, n1])
    xhat = C[lst].astype(np.int64)
    xhat[:, 0] += codes[:, 0]
    xhat[:, 2] += (codes[:, 1] % 16).astype(np.int64) - 8
    xhat[:, 3] += (codes[:, 1] // 16).astype(np.int64) - 8
    exact = xhat @ v["q"].astype(np.int64)
    rid, rkey = topk_desc(exact, ids, k)
    assert oi[0].tolist() == rid.tolist()
    assert ois[0].tolist() == rkey.tolist()
    assert osc[0].tolist() == rkey.astype(np.float32).tolist()


# ------------------------------------------------------------------ step 4: quantisation invariants
def test_quantisation_endpoints_and_error_bound(trained):
    cfg, ix, Q = trained
    S = oracle.coarse(Q, ix["centroids"])
    probes = oracle.select(S, 6)
    L = oracle.lut_f32(Q, ix["centroids"], ix["codebooks"], probes)
    LUT8, B, delta = oracle.quantise(L)
    m = cfg.m
    rng = L.max(axis=3) - L.min(axis=3)                                   # [nq][np][m]
    assert np.array_equal(delta, (rng.reshape(len(Q), -1).max(axis=1) / np.float32(255.0)).astype(np.float32))
    amin = L.argmin(axis=3)
    assert np.all(np.take_along_axis(LUT8, amin[..., None], axis=3) == 0)
    for q in range(len(Q)):                                               # widest sub-table reaches 255
        p, j = np.unravel_index(rng[q].argmax(), rng[q].shape)
        assert LUT8[q, p, j, L[q, p, j].argmax()] == 255
    # table values are the rounded affine map of L, and monotone in L
    recon = L.min(axis=3, keepdims=True).astype(np.float64) + LUT8 * delta[:, None, None, None].astype(np.float64)
    assert np.max(np.abs(recon - L) / delta[:, None, None, None]) <= 0.5 + 1e-3
    # |delta*I - F| <= delta*(m+1)/2 for every scanned vector (F = unquantised ADC score)
    k = 50
    oi, ois, osc = oracle.scan_topk(probes, LUT8, B, delta, ix["list_offsets"], ix["codes"], ix["ids"], k)
    row_of_id = np.empty(cfg.n, np.int64)
    row_of_id[ix["ids"]] = np.arange(cfg.n)
    xhat = reconstruct(ix)
    for q in range(len(Q)):
        F = xhat[row_of_id[oi[q]]] @ Q[q].astype(np.float64)
        assert np.max(np.abs(osc[q] - F)) <= delta[q] * (m + 1) / 2 * (1 + 1e-4)
        assert np.array_equal(osc[q], ois[q].astype(np.float32) * delta[q])


def test_zero_range_tables_give_unit_step():
    Q = np.zeros((1, 8), np.float32)                                      # every table entry is 0
    C = np.ones((2, 8), np.float32)
    CB = np.ones((2, 256, 4), np.float32)
    L = oracle.lut_f32(Q, C, CB, np.array([[0, 1]], np.int32))
    LUT8, B, delta = oracle.quantise(L)
    assert delta[0] == 1.0 and not LUT8.any() and not B.any()


# ------------------------------------------------------------------ steps 5-6: brute force, ties, padding
def _brute_integer(ix, probes, LUT8, B, k):
    off, codes, ids = ix["list_offsets"], ix["codes"], ix["ids"]
    out = []
    for q in range(probes.shape[0]):
        cand = []
        for p, l in enumerate(probes[q]):
            for i in range(off[l], off[l + 1]):
                I = int(B[q, p]) + sum(int(LUT8[q, p, j, codes[i, j]]) for j in range(codes.shape[1]))
                cand.append((-I, int(ids[i])))
        cand.sort()
        out.append(cand[:k])
    return out


def test_integer_scan_vs_python_brute_force_with_ties(rnd):
    ix, Q = rnd
    S = oracle.coarse(Q, ix["centroids"])
    probes = oracle.select(S, 4)
    L = oracle.lut_f32(Q, ix["centroids"], ix["codebooks"], probes)
    LUT8, B, delta = oracle.quantise(L)
    LUT8 = (LUT8 // 32).astype(np.uint8)            # coarse tables: massive exact ties, id order decides
    k = 25
    oi, ois, _ = oracle.scan_topk(probes, LUT8, B, delta, ix["list_offsets"], ix["codes"], ix["ids"], k)
    ref = _brute_integer(ix, probes, LUT8, B, k)
    ties = 0
    for q in range(len(Q)):
        assert [(-int(s), int(i)) for s, i in zip(ois[q], oi[q])] == ref[q]
        ties += len(ois[q]) - len(set(ois[q].tolist()))
    assert ties > 20


def test_padding_when_fewer_candidates_than_k(rnd):
    ix, Q = rnd
    probes = np.tile(np.array([[3]], np.int32), (len(Q), 1))             # list 3 is empty
    L = oracle.lut_f32(Q, ix["centroids"], ix["codebooks"], probes)
    LUT8, B, delta = oracle.quantise(L)
    oi, ois, osc = oracle.scan_topk(probes, LUT8, B, delta, ix["list_offsets"], ix["codes"], ix["ids"], 5)
    assert np.all(oi == -1) and np.all(ois == np.iinfo(np.int32).min) and np.all(np.isneginf(osc))
    small = int(np.diff(ix["list_offsets"]).argmin())
    probes[:] = 0
    n0 = int(ix["list_offsets"][1] - ix["list_offsets"][0])
    oi, ois, osc = oracle.scan_topk(probes, LUT8, B, delta, ix["list_offsets"], ix["codes"], ix["ids"], n0 + 3)
    assert np.all(oi[:, :n0] >= 0) and np.all(oi[:, n0:] == -1) and np.all(np.isneginf(osc[:, n0:]))
    assert all(sorted(oi[q, :n0].tolist()) == sorted(ix["ids"][:n0].tolist()) for q in range(len(Q)))


# ------------------------------------------------------------------ step 7 / nprobe = nlist: exhaustive ADC
def test_all_lists_probed_equals_exhaustive_adc(trained):
    cfg, ix, Q = trained
    S = oracle.coarse(Q, ix["centroids"])
    probes = oracle.select(S, cfg.nlist)
    L = oracle.lut_f32(Q, ix["centroids"], ix["codebooks"], probes)
    k = 20
    oi, osc = oracle.adc_f32_topk(probes, L, ix["list_offsets"], ix["codes"], ix["ids"], k)
    full = Q.astype(np.float64) @ reconstruct(ix).T                        # [nq][n], independent path
    for q in range(len(Q)):
        rid, rkey = topk_desc(full[q], ix["ids"], k)
        assert np.max(np.abs(osc[q] - rkey)) < 2e-6
        assert len(set(oi[q].tolist()) & set(rid.tolist())) >= k - 1       # fp32 rounding may swap a near-tie
    # the integer path keeps almost all of them and each winner is within the quantisation bound
    LUT8, B, delta = oracle.quantise(L)
    qi, qis, qsc = oracle.scan_topk(probes, LUT8, B, delta, ix["list_offsets"], ix["codes"], ix["ids"], k)
    row_of_id = np.empty(cfg.n, np.int64)
    row_of_id[ix["ids"]] = np.arange(cfg.n)
    overlap = 0
    for q in range(len(Q)):
        overlap += len(set(qi[q].tolist()) & set(oi[q].tolist()))
        assert np.all(full[q][row_of_id[qi[q]]] >= osc[q, k - 1] - delta[q] * (cfg.m + 1))
    assert overlap >= 0.8 * k * len(Q)


def test_single_list_is_plain_pq_scan():
    ix = to_np(synth.random_index(n=400, d=8, m=2, nlist=1, seed=2))
    Q = np.random.default_rng(1).standard_normal((3, 8)).astype(np.float32)
    r = oracle.ivfpq_search(Q, ix, 1, 400)
    assert np.all(r["probes"] == 0)
    assert all(sorted(r["ids"][q].tolist()) == list(range(400)) for q in range(3))
    full = Q.astype(np.float64) @ reconstruct(ix).T
    for q in range(3):                                                     # integer order follows the true order
        top_true = set(np.argsort(-full[q])[:40].tolist())
        assert len(top_true & set(r["ids"][q, :40].tolist())) >= 30


# ------------------------------------------------------------------ recall against exact kNN
def test_recall_monotone_in_nprobe_and_lossless_pq_is_exact():
    # few mixture components split over many lists, so the number of probed lists matters
    cfg = synth.TINY.scaled(n=12000, d=32, m=16, nlist=32, components=3, train_n=6000, pq_train_n=4096,
                            kmeans_iters=5, seed=77)
    ix = to_np(synth.build_index(cfg))
    Q = synth.make_queries(cfg, 16).numpy()
    X = ix["vectors"].astype(np.float64)
    k = 10
    exact = np.argsort(-(Q.astype(np.float64) @ X.T), axis=1, kind="stable")[:, :k]
    rec = []
    for nprobe in (1, 2, 4, 8, 32):
        S = oracle.coarse(Q, ix["centroids"])
        probes = oracle.select(S, nprobe)
        L = oracle.lut_f32(Q, ix["centroids"], ix["codebooks"], probes)
        oi, _ = oracle.adc_f32_topk(probes, L, ix["list_offsets"], ix["codes"], ix["ids"], k)
        rec.append(np.mean([len(set(oi[q].tolist()) & set(exact[q].tolist())) / k for q in range(len(Q))]))
    assert all(b >= a - 1e-9 for a, b in zip(rec, rec[1:])) and rec[-1] > rec[0] + 0.1, rec
    # a database vector used as the query finds its own list first
    own = oracle.select(oracle.coarse(ix["vectors"][:50], ix["centroids"]), 1)[:, 0]
    lst_of_id = np.empty(cfg.n, np.int64)
    lst_of_id[ix["ids"]] = list_of(ix)
    assert np.array_equal(own, lst_of_id[:50])
    # lossless PQ: dsub = 1 and residual coordinates drawn from the 256 codewords themselves
    g = np.random.default_rng(9)
    d, nlist, n = 6, 4, 300
    C = g.standard_normal((nlist, d)).astype(np.float32)
    CB = g.standard_normal((d, 256, 1)).astype(np.float32)
    lst = np.sort(g.integers(0, nlist, n))
    codes = g.integers(0, 256, (n, d)).astype(np.uint8)
    off = np.searchsorted(lst, np.arange(nlist + 1)).astype(np.int64)
    idx = dict(centroids=C, codebooks=CB, list_offsets=off, codes=codes, ids=np.arange(n, dtype=np.int64))
    Xl = reconstruct(idx)                                                  # the database IS its reconstruction
    Ql = g.standard_normal((5, d)).astype(np.float32)
    probes = np.tile(np.arange(nlist, dtype=np.int32), (5, 1))
    oi, osc = oracle.adc_f32_topk(probes, oracle.lut_f32(Ql, C, CB, probes), off, codes, idx["ids"], 7)
    ex = np.argsort(-(Ql.astype(np.float64) @ Xl.T), axis=1, kind="stable")[:, :7]
    assert np.array_equal(oi, ex)


# ------------------------------------------------------------------ whole search = its stages chained
def test_search_equals_stage_chain(trained):
    cfg, ix, Q = trained
    r = oracle.ivfpq_search(Q, ix, 5, 15)
    S = oracle.coarse(Q, ix["centroids"])
    probes = oracle.select(S, 5)
    LUT8, B, delta = oracle.quantise(oracle.lut_f32(Q, ix["centroids"], ix["codebooks"], probes))
    oi, ois, osc = oracle.scan_topk(probes, LUT8, B, delta, ix["list_offsets"], ix["codes"], ix["ids"], 15)
    assert np.array_equal(r["probes"], probes) and np.array_equal(r["delta"], delta)
    assert np.array_equal(r["ids"], oi) and np.array_equal(r["iscores"], ois) and np.array_equal(r["scores"], osc)


# ------------------------------------------------------------------ flat search = matmul + stable argsort
def test_flat_equals_matmul_and_stable_argsort():
    cfg = synth.FLAT
    corpus, queries = synth.make_flat(cfg, requests=2, n=700)
    corpus[1, 5] = corpus[1, 300]                                          # duplicate rows: exact ties
    corpus[1, 301] = corpus[1, 300]
    queries[1, 0] = corpus[1, 300]
    cb = corpus.view(torch.int16).numpy().view(np.uint16)
    qb = queries.view(torch.int16).numpy().view(np.uint16)
    oi, osc = oracle.flat_search(cb, qb, 32)
    ref = torch.einsum("rqd,rnd->rqn", queries.double(), corpus.double()).numpy()
    for r in range(2):
        for q in range(cfg.nq):
            order = np.argsort(-ref[r, q].astype(np.float32), kind="stable")[:32]
            assert np.allclose(osc[r, q], ref[r, q][oi[r, q]], rtol=0, atol=1e-6)
            assert oi[r, q].tolist() == order.tolist()
    assert oi[1, 0, :3].tolist() == [5, 300, 301]
    oi, osc = oracle.flat_search(cb[:, :3], qb, 5)                          # fewer rows than k: padded
    assert np.all(oi[:, :, 3:] == -1) and np.all(np.isneginf(osc[:, :, 3:]))


def test_flat_f16_decodes_every_finite_pattern_as_numpy_does():
    """One-dimensional corpora holding every finite binary16 pattern (subnormals, both zeros), query 1.0: a score is
    the value itself, exactly; equal values (+0 and -0) rank by lower row."""
    bits = np.array([b for b in range(65536) if (b >> 10) & 31 != 31], np.uint16)
    assert bits.size == 63488
    rng = np.random.default_rng(5)
    bits = bits[rng.permutation(bits.size)].reshape(62, 1024, 1)
    one = np.full((62, 1, 1), 0x3C00, np.uint16)
    oi, osc = oracle.flat_search(bits, one, 1024, fmt="f16")
    vals = bits.view(np.float16).astype(np.float32)[:, :, 0]
    for r in range(62):
        order = np.argsort(-vals[r], kind="stable")
        assert oi[r, 0].tolist() == order.tolist()
        assert np.array_equal(osc[r, 0], vals[r][order])
    two = np.full((62, 1, 1), 0xC000, np.uint16)                            # query -2.0: signs and order flip
    oi2, osc2 = oracle.flat_search(bits, two, 5, fmt="f16")
    for r in range(62):
        order = np.argsort(2.0 * vals[r], kind="stable")[:5]
        assert oi2[r, 0].tolist() == order.tolist() and np.array_equal(osc2[r, 0], -2.0 * vals[r][order])


def test_flat_f16_equals_matmul_and_stable_argsort():
    cfg = synth.FLAT
    corpus, queries = synth.make_flat(cfg, requests=2, n=700)
    corpus, queries = corpus.float().half(), queries.float().half()
    corpus[1, 5] = corpus[1, 300]
    corpus[1, 301] = corpus[1, 300]
    queries[1, 0] = corpus[1, 300]
    cb = corpus.view(torch.int16).numpy().view(np.uint16)
    qb = queries.view(torch.int16).numpy().view(np.uint16)
    assert np.any((cb >> 10) & 31 == 0)                                     # the data holds subnormals
    oi, osc = oracle.flat_search(cb, qb, 32, fmt="f16")
    ref = torch.einsum("rqd,rnd->rqn", queries.double(), corpus.double()).numpy()
    for r in range(2):
        for q in range(cfg.nq):
            order = np.argsort(-ref[r, q].astype(np.float32), kind="stable")[:32]
            assert np.allclose(osc[r, q], ref[r, q][oi[r, q]], rtol=0, atol=1e-7)
            assert oi[r, q].tolist() == order.tolist()
    assert oi[1, 0, :3].tolist() == [5, 300, 301]
    bi, _ = oracle.flat_search(cb, qb, 32)                                  # the same bits read as bf16 rank differently
    assert not np.array_equal(bi, oi)


# ------------------------------------------------------------------ Euclidean metric (similarity = minus squared distance)
def test_l2_coarse_equals_numpy_distances(rnd):
    ix, Q = rnd
    S = oracle.coarse(Q, ix["centroids"], metric="l2")
    diff = Q.astype(np.float64)[:, None, :] - ix["centroids"].astype(np.float64)[None, :, :]
    ref = -np.sum(diff * diff, axis=2)
    assert S.dtype == np.float32 and np.all(S <= 0)
    assert np.max(np.abs(S - ref)) <= 2 ** -24 * np.max(np.abs(ref)) * 1.01
    # nearest centroid by distance = the probe of rank 0
    assert np.array_equal(oracle.select(S, 1)[:, 0], np.argmin(-ref, axis=1))
    # a query that IS a centroid is at distance exactly 0 from it
    S0 = oracle.coarse(ix["centroids"][:3], ix["centroids"], metric="l2")
    assert np.all(S0[np.arange(3), np.arange(3)] == 0.0)


def test_l2_lut_sum_identity_zero_entries_and_relation_to_ip(rnd):
    ix, Q = rnd
    nl = len(ix["centroids"])
    probes = np.tile(np.arange(nl, dtype=np.int32), (Q.shape[0], 1))
    L = oracle.lut_f32(Q, ix["centroids"], ix["codebooks"], probes, metric="l2")
    assert np.all(L <= 0)
    xhat, lst, codes = reconstruct(ix), list_of(ix), ix["codes"]
    m = codes.shape[1]
    dsub = Q.shape[1] // m
    for q in range(Q.shape[0]):
        got = sum(L[q, lst, j, codes[:, j]].astype(np.float64) for j in range(m))
        ref = -np.sum((Q[q].astype(np.float64)[None, :] - xhat) ** 2, axis=1)      # independent: reconstruct, subtract
        assert np.max(np.abs(got - ref)) < 1e-5
    # relation to the inner-product tables through the norms: |a - b|^2 = |a|^2 - 2<a,b> + |b|^2
    Lip = oracle.lut_f32(Q, ix["centroids"], ix["codebooks"], probes, metric="ip").astype(np.float64)
    C, CB = ix["centroids"].astype(np.float64), ix["codebooks"].astype(np.float64)
    for q, p, j in ((0, 1, 0), (3, 6, 2), (5, 0, m - 1)):
        qj = Q[q, j * dsub:(j + 1) * dsub].astype(np.float64)
        tgt = C[p, j * dsub:(j + 1) * dsub][None, :] + CB[j]                       # [256][dsub]
        ref = -(qj @ qj - 2.0 * Lip[q, p, j] + np.sum(tgt * tgt, axis=1))
        assert np.max(np.abs(L[q, p, j] - ref)) < 1e-5
    # unlike the inner product, the tables of two lists do NOT differ by a constant in c
    dlt = L[0, 0, 1].astype(np.float64) - L[0, 5, 1].astype(np.float64)
    assert np.ptp(dlt) > 1e-3
    # a query sub-vector that equals centroid + codeword gives an entry of exactly 0, the table's maximum
    Qz = Q.copy()
    Qz[2, 0:dsub] = (ix["centroids"][4, 0:dsub].astype(np.float64) + ix["codebooks"][0, 77].astype(np.float64)).astype(np.float32)
    Lz = oracle.lut_f32(Qz[2:3], ix["centroids"], ix["codebooks"], np.array([[4]], np.int32), metric="l2")
    exact = np.all((ix["centroids"][4, 0:dsub].astype(np.float64) + ix["codebooks"][0, 77].astype(np.float64)).astype(np.float32).astype(np.float64)
                   == ix["centroids"][4, 0:dsub].astype(np.float64) + ix["codebooks"][0, 77].astype(np.float64))
    if exact:
        assert Lz[0, 0, 0, 77] == 0.0
    assert abs(Lz[0, 0, 0, 77]) < 1e-12 and np.argmax(Lz[0, 0, 0]) == 77


def test_l2_all_lists_probed_equals_exhaustive_and_search_chain(trained):
    cfg, ix, Q = trained
    S = oracle.coarse(Q, ix["centroids"], metric="l2")
    probes = oracle.select(S, cfg.nlist)
    L = oracle.lut_f32(Q, ix["centroids"], ix["codebooks"], probes, metric="l2")
    k = 20
    oi, osc = oracle.adc_f32_topk(probes, L, ix["list_offsets"], ix["codes"], ix["ids"], k)
    xhat = reconstruct(ix)
    full = -np.sum((Q.astype(np.float64)[:, None, :] - xhat[None, :, :]) ** 2, axis=2)    # [nq][n], independent path
    for q in range(len(Q)):
        rid, rkey = topk_desc(full[q], ix["ids"], k)
        assert np.max(np.abs(osc[q] - rkey)) < 5e-6
        assert len(set(oi[q].tolist()) & set(rid.tolist())) >= k - 1
    # the whole search = its stages chained, with the quantisation bound on every winner
    nprobe = 6
    r = oracle.ivfpq_search(Q, ix, nprobe, k, metric="l2")
    pr = oracle.select(S, nprobe)
    Lp = oracle.lut_f32(Q, ix["centroids"], ix["codebooks"], pr, metric="l2")
    LUT8, B, delta = oracle.quantise(Lp)
    qi, qis, qsc = oracle.scan_topk(pr, LUT8, B, delta, ix["list_offsets"], ix["codes"], ix["ids"], k)
    assert np.array_equal(r["probes"], pr) and np.array_equal(r["ids"], qi) and np.array_equal(r["iscores"], qis)
    assert np.array_equal(r["scores"], qsc) and np.array_equal(r["delta"], delta)
    row_of_id = np.empty(cfg.n, np.int64)
    row_of_id[ix["ids"]] = np.arange(cfg.n)
    for q in range(len(Q)):
        true = full[q][row_of_id[qi[q]]]
        assert np.all(np.abs(qsc[q].astype(np.float64) - true) <= delta[q] * (cfg.m + 1) / 2 + 1e-5)   # |delta*I - F| bound


def test_l2_and_ip_rank_unit_vectors_alike_on_lossless_codes():
    # dsub = 1, residual coordinates drawn from the codewords: the database IS its reconstruction.
    # Rows are scaled to unit norm by construction of the query only: |q - x|^2 = |q|^2 + |x|^2 - 2<q,x>,
    # so with all |x| equal the two metrics must rank the database identically.
    g = np.random.default_rng(19)
    d, nlist, n = 6, 4, 300
    C = np.zeros((nlist, d), np.float32)
    vals = np.array([-0.5, 0.5], np.float32)                                  # every coordinate is +-0.5: |x|^2 = d/4 for all x
    CB = np.zeros((d, 256, 1), np.float32)
    CB[:, :, 0] = vals[g.integers(0, 2, (d, 256))]
    lst = np.sort(g.integers(0, nlist, n))
    codes = g.integers(0, 256, (n, d)).astype(np.uint8)
    off = np.searchsorted(lst, np.arange(nlist + 1)).astype(np.int64)
    idx = dict(centroids=C, codebooks=CB, list_offsets=off, codes=codes, ids=np.arange(n, dtype=np.int64))
    X = reconstruct(idx)
    assert np.allclose(np.sum(X * X, axis=1), d / 4)
    Ql = g.standard_normal((5, d)).astype(np.float32)
    probes = np.tile(np.arange(nlist, dtype=np.int32), (5, 1))
    k = n                                                                      # full ranking
    i_ip, s_ip = oracle.adc_f32_topk(probes, oracle.lut_f32(Ql, C, CB, probes, metric="ip"), off, codes, idx["ids"], k)
    i_l2, s_l2 = oracle.adc_f32_topk(probes, oracle.lut_f32(Ql, C, CB, probes, metric="l2"), off, codes, idx["ids"], k)
    for q in range(5):
        # same ranking up to exact ties (many rows coincide): compare the score sequences through the identity
        qn = float(np.sum(Ql[q].astype(np.float64) ** 2))
        assert np.max(np.abs(s_l2[q].astype(np.float64) - (-(qn + d / 4 - 2.0 * s_ip[q].astype(np.float64))))) < 1e-5
        ex = np.lexsort((idx["ids"], np.sum((Ql[q].astype(np.float64)[None, :] - X) ** 2, axis=1)))[:10]
        assert set(i_l2[q, :10].tolist()) == set(ex.tolist()) or np.isclose(s_l2[q, 9], s_l2[q, 10])


# ------------------------------------------------------------------ upper level over the lists (two-level coarse search)
def _upper(nlist, nsuper, d, seed, dup=False):
    g = np.random.default_rng(seed)
    owner = g.integers(0, nsuper, nlist)
    owner[:nsuper] = np.arange(nsuper)                     # no empty group ... except when asked for below
    order = np.lexsort((np.arange(nlist), owner))          # by group, ascending list inside a group
    off = np.searchsorted(owner[order], np.arange(nsuper + 1)).astype(np.int64)
    SC = g.standard_normal((nsuper, d)).astype(np.float32)
    if dup:
        SC[1] = SC[0]                                      # exact tie between two groups
    return dict(super_centroids=SC, super_offsets=off, super_lists=order.astype(np.int32)), owner


@pytest.mark.parametrize("metric", ["ip", "l2"])
def test_tree_select_equals_brute_force_and_exhaustive_limit(metric):
    g = np.random.default_rng(3)
    nlist, nsuper, d, nq = 60, 7, 12, 9
    C = g.standard_normal((nlist, d)).astype(np.float32)
    C[11] = C[10]                                          # tie between two lists
    Q = g.standard_normal((nq, d)).astype(np.float32)
    upper, owner = _upper(nlist, nsuper, d, 5, dup=True)

    def score(A, B):                                       # independent numpy formulation
        A, B = A.astype(np.float64), B.astype(np.float64)
        if metric == "ip":
            return (A @ B.T).astype(np.float32).astype(np.float64)
        return (-np.sum((A[:, None, :] - B[None, :, :]) ** 2, axis=2)).astype(np.float32).astype(np.float64)

    Ssup, S = score(Q, upper["super_centroids"]), score(Q, C)
    for nsp, nprobe in ((2, 5), (3, 9), (1, 4), (nsuper, 13)):
        probes, sup = oracle.select_tree(Q, upper, C, nsp, nprobe, metric=metric)
        for q in range(nq):
            keep = np.lexsort((np.arange(nsuper), -Ssup[q]))[:nsp]
            assert sup[q].tolist() == keep.tolist()
            member = np.isin(owner, keep)
            key = np.where(member, S[q], -np.inf)
            ref = np.lexsort((np.arange(nlist), -key))[:nprobe]
            assert probes[q].tolist() == ref.tolist(), (nsp, nprobe, q)
        if nsp == nsuper:                                  # every group kept = the exhaustive coarse search
            assert np.array_equal(probes, oracle.select(oracle.coarse(Q, C, metric=metric), nprobe))
    # duplicated group centroids: the lower group wins the tie (query 0 made to favour them)
    Q2 = np.tile(upper["super_centroids"][0], (1, 1)).astype(np.float32) * (1.0 if metric == "ip" else 1.0)
    _, sup = oracle.select_tree(Q2, upper, C, 1, 1, metric=metric)
    if metric == "l2":
        assert sup[0, 0] == 0                              # distance 0 to groups 0 and 1: lower number


def test_tree_select_fills_up_with_low_lists_when_groups_are_small():
    g = np.random.default_rng(8)
    nlist, d = 20, 6
    C = g.standard_normal((nlist, d)).astype(np.float32)
    # three groups: {17, 19}, {3}, all the rest
    lists = np.array([17, 19, 3] + [l for l in range(nlist) if l not in (3, 17, 19)], np.int32)
    upper = dict(super_centroids=np.stack([C[17], C[3], C[0]]).astype(np.float32),
                 super_offsets=np.array([0, 2, 3, nlist], np.int64), super_lists=lists)
    Q = (C[17:18] * 3.0).astype(np.float32)                # clearly closest (by inner product) to group 0
    probes, sup = oracle.select_tree(Q, upper, C, 1, 5)
    assert sup[0, 0] == 0
    first = sorted(probes[0, :2].tolist())
    assert first == [17, 19] and probes[0, 2:].tolist() == [0, 1, 2]      # -inf elsewhere: lowest list numbers fill up
    with pytest.raises(RuntimeError):
        oracle.select_tree(Q, upper, C, 4, 5)              # more groups than exist


# ------------------------------------------------------------------ 4-bit PQ: two sub-quantisers per code byte
def _reconstruct_pq4(ix):
    """x_hat from nibbles, independent of the byte-codebook expansion."""
    C, CB = ix["centroids"].astype(np.float64), ix["codebooks"].astype(np.float64)      # CB [m][16][dsub]
    codes = ix["codes"]
    m = CB.shape[0]
    parts = []
    for j in range(m):
        nib = (codes[:, j // 2] >> (4 * (j & 1))) & 15
        parts.append(CB[j][nib])
    return C[list_of(ix)] + np.concatenate(parts, axis=1)


@pytest.mark.parametrize("metric", ["ip", "l2"])
def test_pq4_tables_and_search_match_reconstruction_from_nibbles(metric):
    ix = to_np(synth.random_index(n=1200, d=24, m=12, nlist=6, seed=41, ksub=16, dup_codes=30, shuffle_ids=True))
    assert ix["codebooks"].shape == (12, 16, 2) and ix["codes"].shape == (1200, 6)
    CB = oracle.expand_pq4(ix["codebooks"])
    assert CB.shape == (6, 256, 4)
    # word b of byte j = codeword (b & 15) of sub-quantiser 2j, then codeword (b >> 4) of sub-quantiser 2j+1
    assert np.array_equal(CB[2, 0xA7, :2], ix["codebooks"][4, 7]) and np.array_equal(CB[2, 0xA7, 2:], ix["codebooks"][5, 10])
    g = np.random.default_rng(4)
    Q = g.standard_normal((5, 24)).astype(np.float32)
    probes = np.tile(np.arange(6, dtype=np.int32), (5, 1))
    L = oracle.lut_f32(Q, ix["centroids"], CB, probes, metric=metric)
    xhat, lst, codes = _reconstruct_pq4(ix), list_of(ix), ix["codes"]
    ref = Q.astype(np.float64) @ xhat.T if metric == "ip" else -np.sum((Q.astype(np.float64)[:, None, :] - xhat[None]) ** 2, axis=2)
    for q in range(5):
        got = sum(L[q, lst, j, codes[:, j]].astype(np.float64) for j in range(6))
        assert np.max(np.abs(got - ref[q])) < 1e-5
    # every list probed: the unquantised search is the exhaustive ranking of the nibble reconstruction
    k = 15
    oi, osc = oracle.adc_f32_topk(probes, L, ix["list_offsets"], ix["codes"], ix["ids"], k)
    for q in range(5):
        rid, rkey = topk_desc(ref[q], ix["ids"], k)
        assert np.max(np.abs(osc[q] - rkey)) < 5e-6
        assert len(set(oi[q].tolist()) & set(rid.tolist())) >= k - 1
    # the whole search takes the 4-bit index as it is
    r = oracle.ivfpq_search(Q, ix, 3, k, metric=metric)
    ix8 = dict(ix, codebooks=CB)
    r8 = oracle.ivfpq_search(Q, ix8, 3, k, metric=metric)
    assert np.array_equal(r["ids"], r8["ids"]) and np.array_equal(r["iscores"], r8["iscores"])
