"""CPU-only pins of the oracle's rounding conventions: hand-derived worked cases
(tests/golden/rounding_cases.txt) and half-ulp bounds against independent numpy fp64 evaluations.

What they fix: round-half-to-even in the 8-bit entries and in the bias, the IEEE fp32 divide (not a
multiplication by a rounded reciprocal), fp64 accumulation with ONE rounding to fp32 in both kinds of
table, and the fp64 sum of the sub-table minima."""
import os

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "rounding_cases.txt")


def _cases():
    cases, cur = {}, None
    for raw in open(GOLDEN):
        line = raw.split("#", 1)[0].strip()
        if not line:
            continue
        if line.startswith("["):
            cur = cases.setdefault(line.strip("[]"), [])
        else:
            cur.append(line.split())
    return cases


CASES = _cases()


@pytest.mark.parametrize("name", ["ties_to_even", "divide_not_reciprocal", "bias_summed_in_fp64", "bias_divided_in_fp64",
                                  "subtract_and_divide_in_fp32"])
def test_quantise_worked_cases(name):
    rows = CASES[name]
    nprobe, m = next((int(r[1]), int(r[2])) for r in rows if r[0] == "shape")
    L = np.full((1, nprobe, m, 256), np.nan, np.float32)
    for r in rows:
        if r[0] == "fill":
            L[0, int(r[1]), int(r[2]), :] = np.float32(float(r[3]))
    expect = []
    for r in rows:
        if r[0] == "L":
            p, j, c = int(r[1]), int(r[2]), int(r[3])
            assert float(np.float32(float(r[4]))) == float(r[4]), "golden values must be exact in fp32"
            L[0, p, j, c] = np.float32(float(r[4]))
            expect.append((p, j, c, int(r[5])))
    assert not np.isnan(L).any()
    LUT8, B, delta = oracle.quantise(L)
    assert float(delta[0]) == float(next(r[1] for r in rows if r[0] == "delta"))
    for p, j, c, e in expect:
        assert int(LUT8[0, p, j, c]) == e, (name, p, j, c, int(LUT8[0, p, j, c]), e)
    for r in rows:
        if r[0] == "B":
            assert int(B[0, int(r[1])]) == int(r[2]), (name, r, int(B[0, int(r[1])]))


@pytest.mark.parametrize("name", ["ip_table_accumulated_in_fp64", "l2_table_accumulated_in_fp64"])
def test_table_worked_cases(name):
    rows = CASES[name]
    get = lambda key: next(r[1:] for r in rows if r[0] == key)
    metric, d, m = get("metric")[0], int(get("d")[0]), int(get("m")[0])
    dsub = d // m
    Q = np.array([[float(v) for v in get("q")]], np.float32)
    C = np.array([[float(v) for v in get("C")]], np.float32)
    CB = np.zeros((m, 256, dsub), np.float32)
    for r in rows:
        if r[0] == "cbfill":
            CB[int(r[1]), :, :] = [float(v) for v in r[2:]]
    for r in rows:
        if r[0] == "cb":
            CB[int(r[1]), int(r[2]), :] = [float(v) for v in r[3:]]
    probes = np.zeros((1, 1), np.int32)
    L = oracle.lut_f32(Q, C, CB, probes, metric=metric)
    LUT8, B, delta = oracle.quantise(L)
    for r in rows:
        if r[0] == "T":
            j, c = int(r[1]), int(r[2])
            assert float(L[0, 0, j, c]) == float(r[3]), (name, r, float(L[0, 0, j, c]))
            assert int(LUT8[0, 0, j, c]) == int(r[4]), (name, r, int(LUT8[0, 0, j, c]))
    assert float(delta[0]) == float(get("delta")[0])
    assert int(B[0, 0]) == int(get("B")[1])


def _tables_fp64(Q, C, CB, probes, metric):
    """Both kinds of table straight from their definitions in numpy fp64 (no oracle code)."""
    nq, d = Q.shape
    m, _, dsub = CB.shape
    Q64, C64, CB64 = Q.astype(np.float64), C.astype(np.float64), CB.astype(np.float64)
    out = np.empty((nq, probes.shape[1], m, 256))
    for q in range(nq):
        for p, l in enumerate(probes[q]):
            for j in range(m):
                sl = slice(j * dsub, (j + 1) * dsub)
                y = C64[l, sl][None, :] + CB64[j]                   # [256][dsub] reconstruction of the sub-vector
                if metric == "ip":
                    out[q, p, j] = np.einsum("t,ct->c", Q64[q, sl], y)
                else:
                    out[q, p, j] = -np.sum((Q64[q, sl][None, :] - y) ** 2, axis=1)
    return out


@pytest.mark.parametrize("metric", ["ip", "l2"])
def test_tables_are_correctly_rounded_fp64_sums(metric):
    """|L - exact| <= half an fp32 ulp: only an accumulation in (at least) fp64 with one final rounding
    achieves that on 16-term sums with cancellation; an fp32 running sum is off by several ulps."""
    g = np.random.default_rng(23)
    d, m, nlist = 64, 4, 6
    Q = g.standard_normal((5, d)).astype(np.float32)
    C = g.standard_normal((nlist, d)).astype(np.float32) * 3
    CB = g.standard_normal((m, 256, d // m)).astype(np.float32)
    probes = np.stack([g.permutation(nlist)[:4] for _ in range(5)]).astype(np.int32)
    L = oracle.lut_f32(Q, C, CB, probes, metric=metric)
    ref = _tables_fp64(Q, C, CB, probes, metric)
    half_ulp = np.spacing(np.abs(ref).astype(np.float32)).astype(np.float64) / 2      # ulp of the fp32 at or below |ref|
    assert np.all(np.abs(L.astype(np.float64) - ref) <= half_ulp * 1.01 + 1e-30)
    # and the test can tell: the same sums accumulated in fp32 break the bound
    if metric == "ip":
        l0 = probes[0, 0]
        acc = np.zeros(256, np.float32)
        for t in range(d // m):
            acc = (acc + (Q[0, t].astype(np.float64) * (C[l0, t].astype(np.float64) + CB[0, :, t].astype(np.float64)))).astype(np.float32)
        assert np.any(np.abs(acc.astype(np.float64) - ref[0, 0, 0]) > half_ulp[0, 0, 0] * 1.01)


def test_bias_equals_fp64_sum_of_minima_on_random_tables():
    """B = rne(sum_j lo_j / delta) with the sum and the quotient in fp64, on tables whose minima are
    large against delta (so that an fp32 running sum or a truncation shows)."""
    g = np.random.default_rng(29)
    L = (g.standard_normal((4, 5, 24, 256)) * 50 + 4000).astype(np.float32)
    LUT8, B, delta = oracle.quantise(L)
    lo = L.min(axis=3).astype(np.float64).sum(axis=2)                    # [nq][np]
    ref = np.rint(lo / delta.astype(np.float64)[:, None]).astype(np.int64)
    assert np.array_equal(B.astype(np.int64), ref)
    # the 8-bit entries are the rounded fp32 quotient of the fp32 difference
    q = ((L - L.min(axis=3, keepdims=True)) / delta[:, None, None, None]).astype(np.float32)
    assert np.array_equal(LUT8, np.clip(np.rint(q), 0, 255).astype(np.uint8))
