"""GPU parity on seeded random configurations: shapes, code widths, metrics, both scan kernels, ties, empty lists,
magnitudes from 1e-17 to 1e15, against the CPU oracle through the C ABI.  The fixed cases of the other files aim at
known hard spots; this sweep is the net under them."""
import os

import numpy as np
import pytest
import torch

import oracle
import synth
from gpu_common import dev_index
from helpers import to_np

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def rb():
    from paper_2503_14649_amd import binding
    return binding


def _bits(t):
    return t.cpu().view(torch.int16).numpy().view(np.uint16)


# (seed, number of cases, batch sizes): the last line draws batches with as many queries as the chip has compute units and
# more, where the selection, the table kernels and the wave-per-item scan's merge take their large-batch forms
@pytest.mark.parametrize("seed,ncases,batches", [(11, 70, (1, 2, 7, 33, 130)), (12, 70, (1, 2, 7, 33, 130)), (13, 70, (1, 2, 7, 33, 130)),
                                                 (14, 25, (140, 260, 300, 520, 1100))])
def test_ivfpq_random_configurations(rb, seed, ncases, batches):
    rng = np.random.default_rng(seed)
    unproven = 0
    try:
        for case in range(ncases):
            ksub = 16 if rng.random() < 0.25 else 256
            mbytes = int(rng.choice([16, 32, 64, 96, 128]))
            m = mbytes * 2 if ksub == 16 else mbytes
            dsub = int(rng.choice([1, 2, 3, 4, 5, 8, 16] if mbytes <= 32 else [1, 2, 4, 8]))
            if m * dsub > 1536:
                dsub = max(1, 1536 // m)
            d = m * dsub
            nlist = int(rng.choice([1, 2, 5, 17, 64, 300]))
            n = int(rng.choice([0, 1, 63, 64, 65, 1000, 7000, 30000]))
            nq = int(rng.choice(list(batches)))
            nprobe = int(rng.integers(1, nlist + 1))
            k = int(rng.choice([1, 2, 10, 100, 128]))
            metric = "l2" if rng.random() < 0.4 else "ip"
            kernel = str(rng.choice(["wide", "narrow", "wave", ""]))
            kw = {}
            if rng.random() < 0.3 and n > 100:
                kw["dup_codes"] = int(rng.integers(1, 50))
            if rng.random() < 0.3:
                kw["shuffle_ids"] = True
            if rng.random() < 0.2 and nlist > 2:
                kw["empty_lists"] = tuple(int(x) for x in rng.choice(nlist, size=min(2, nlist - 1), replace=False))
            if rng.random() < 0.15:
                kw["cb_scale"] = float(rng.choice([3e-6, 1e-3, 5.0]))
            big = float(rng.choice([1.0, 1.0, 1e-10, 1e-17, 1e8, 1e15]))
            desc = (f"seed {seed} case {case}: n={n} d={d} m={m} ksub={ksub} nlist={nlist} nq={nq} nprobe={nprobe} k={k} "
                    f"metric={metric} kernel={kernel or 'auto'} scale={big} {kw}")
            print(desc, flush=True)
            ix = to_np(synth.random_index(n=n, d=d, m=m, nlist=nlist, seed=int(rng.integers(1 << 30)), ksub=ksub, **kw))
            ix["centroids"] = (ix["centroids"] * big).astype(np.float32)
            ix["codebooks"] = (ix["codebooks"] * big).astype(np.float32)
            g = torch.Generator().manual_seed(int(rng.integers(1 << 30)))
            Q = torch.nn.functional.normalize(torch.randn(nq, d, generator=g), dim=1).numpy()
            Q = (Q * float(rng.choice([1.0, 1.0, 0.01, 30.0])) * big).astype(np.float32)
            rb.rago_debug_force_scan_kernel(kernel or "auto")
            h = rb.rago_index_wrap(dev_index(ix), metric=metric)
            try:
                r = oracle.ivfpq_search(Q, ix, nprobe, k, metric=metric)
                gi, gs, gis = rb.rago_ivfpq_search(h, torch.from_numpy(Q).cuda(), nprobe, k)
                torch.cuda.synchronize()
                unproven += int(rb.rago_debug_counters(h)[3] != 0)    # (probe choice made on exact scores of all lists)
                assert np.array_equal(gi.cpu().numpy(), r["ids"]), desc
                assert np.array_equal(gis.cpu().numpy(), r["iscores"]), desc
                assert np.array_equal(gs.cpu().numpy(), r["scores"], equal_nan=True), desc
            finally:
                rb.rago_index_free(h)
    finally:
        rb.rago_debug_force_scan_kernel("auto")
    print(f"queries' probe choices taken on exact scores in {unproven} cases", flush=True)


def test_flat_random_configurations(rb):
    rng = np.random.default_rng(21)
    for case in range(80):
        R = int(rng.choice([1, 2, 5]))
        n = int(rng.choice([0, 1, 15, 16, 17, 255, 256, 257, 1000, 5000, 40000]))
        d = int(rng.choice([64, 128, 256, 384, 512, 768, 1024]))
        nq = int(rng.integers(1, 17))
        k = int(rng.choice([1, 5, 32, 128]))
        half = rng.random() < 0.5
        scale_c, scale_q = float(rng.choice([1.0, 1.0, 0.05, 4.0])), float(rng.choice([1.0, 1.0, 0.05, 4.0]))
        dup = rng.random() < 0.3 and n > 20
        desc = f"case {case}: R={R} n={n} d={d} nq={nq} k={k} {'f16' if half else 'bf16'} scales {scale_c} {scale_q} dup={dup}"
        print(desc, flush=True)
        g = torch.Generator().manual_seed(int(rng.integers(1 << 30)))
        dt = torch.float16 if half else torch.bfloat16
        c = (torch.nn.functional.normalize(torch.randn(R, max(n, 1), d, generator=g), dim=2)[:, :n] * scale_c).to(dt).contiguous()
        q = (torch.nn.functional.normalize(torch.randn(R, nq, d, generator=g), dim=2) * scale_q).to(dt).contiguous()
        if dup:
            for r in range(R):
                src = int(rng.integers(n))
                for _ in range(int(rng.integers(1, 40))):
                    c[r, int(rng.integers(n))] = c[r, src]
                q[r, 0] = c[r, src]
        fn = rb.rago_flat_search_f16 if half else rb.rago_flat_search
        gi, gs = fn(c.cuda(), q.cuda(), k)
        torch.cuda.synchronize()
        gi, gs = gi.cpu().numpy(), gs.cpu().numpy()
        oi, osc = oracle.flat_search(_bits(c), _bits(q), k, fmt="f16" if half else "bf16")
        kk = min(k, n)
        tol = 1e-4 * max(1.0, scale_c * scale_q)
        assert np.all(gi[:, :, kk:] == -1) and np.all(np.isneginf(gs[:, :, kk:])), desc
        if not kk:
            continue
        assert np.max(np.abs(gs[:, :, :kk] - osc[:, :, :kk])) < tol, desc
        ref = torch.einsum("rqd,rnd->rqn", q.double(), c.double()).numpy()
        for r in range(R):
            for j in range(nq):
                assert np.max(np.abs(ref[r, j][gi[r, j, :kk]] - gs[r, j, :kk])) < tol, desc     # a row's score is its true score
                assert np.all(np.diff(gs[r, j, :kk]) <= 0), desc
                same = np.diff(gs[r, j, :kk]) == 0
                assert np.all(np.diff(gi[r, j, :kk])[same] > 0), desc                            # equal scores: lower row first
                left = np.ones(n, bool)
                left[gi[r, j, :kk]] = False
                if left.any():
                    assert ref[r, j][left].max() <= gs[r, j, kk - 1] + tol, desc                 # nothing better was left out


def test_upper_level_random_configurations(rb):
    rng = np.random.default_rng(31)
    for case in range(60):
        d = int(rng.choice([16, 64, 96, 768]))
        nlist = int(rng.choice([8, 50, 500, 3000]))
        nsuper = int(rng.integers(1, min(nlist, 200) + 1))
        metric = "l2" if rng.random() < 0.5 else "ip"
        nq = int(rng.choice([1, 3, 20]))
        ix = to_np(synth.random_index(n=2000, d=d, m=16, nlist=nlist, seed=int(rng.integers(1 << 30))))
        if rng.random() < 0.3:                                   # duplicate centroids: ties among lists and groups
            for l in range(nlist):
                ix["centroids"][l] = ix["centroids"][l % max(1, nlist // 3)]
        upper = synth.build_upper_level(torch.from_numpy(ix["centroids"]), nsuper, seed=int(rng.integers(1 << 30)), iters=3)
        up = to_np(upper)
        nsuper = len(up["super_offsets"]) - 1
        largest = int(np.diff(up["super_offsets"]).max())
        nsp = int(rng.integers(1, nsuper + 1))
        if nsp * largest > 8192:
            nsp = max(1, 8192 // largest)
        nprobe = int(rng.integers(1, min(nlist, 2016) + 1))
        g = torch.Generator().manual_seed(int(rng.integers(1 << 30)))
        Q = torch.nn.functional.normalize(torch.randn(nq, d, generator=g), dim=1).numpy()
        if rng.random() < 0.2:
            Q[0] = 0.0
        desc = f"case {case}: d={d} nlist={nlist} nsuper={nsuper} nsp={nsp} nprobe={nprobe} nq={nq} metric={metric}"
        print(desc, flush=True)
        h = rb.rago_index_wrap(dev_index(ix), metric=metric)
        try:
            rb.rago_index_set_upper_level(h, {k: v.cuda() for k, v in upper.items()})
            rb.rago_index_set_upper_probe(h, nsp)
            probes, groups = oracle.select_tree(Q, up, ix["centroids"], nsp, nprobe, metric=metric)
            gp, gg = rb.rago_debug_select_tree(h, torch.from_numpy(Q).cuda(), nprobe, nsp)
            assert np.array_equal(gg.cpu().numpy(), groups), desc
            assert np.array_equal(gp.cpu().numpy(), probes), desc
        finally:
            rb.rago_index_free(h)
