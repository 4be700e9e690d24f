"""The seeded input generators: shapes and the packing of 4-bit codes (no method arithmetic lives there)."""
import numpy as np
import torch

import synth


def test_build_index_with_16_word_codebooks_packs_nearest_codewords_into_nibbles():
    cfg = synth.TINY.scaled(n=3000, nlist=8, components=8, train_n=3000, pq_train_n=2000, kmeans_iters=3, m=32, ksub=16)
    ix = synth.build_index(cfg, device="cpu", keep_vectors=True)
    d, m = cfg.d, cfg.m
    assert ix["codebooks"].shape == (m, 16, d // m) and ix["codes"].shape == (cfg.n, m // 2)
    off = ix["list_offsets"].numpy()
    lists = np.repeat(np.arange(cfg.nlist), np.diff(off))
    res = (ix["vectors"][ix["ids"]] - ix["centroids"][lists]).numpy().astype(np.float64)
    cb = ix["codebooks"].numpy().astype(np.float64)
    codes = ix["codes"].numpy()
    nib = np.empty((cfg.n, m), np.int64)
    nib[:, 0::2], nib[:, 1::2] = codes & 15, codes >> 4
    r = res.reshape(cfg.n, m, 1, d // m)
    dist = ((r - cb[None]) ** 2).sum(3)                                  # [n][m][16]
    chosen = np.take_along_axis(dist, nib[:, :, None], 2)[:, :, 0]
    assert np.all(chosen <= dist.min(2) * (1 + 1e-5) + 1e-9)             # each nibble names a nearest codeword


def test_pairs_of_codewords_layout():
    cb = torch.arange(4 * 16 * 2, dtype=torch.float32).view(4, 16, 2)
    P = synth.workloads.pairs_of_codewords(cb)
    assert P.shape == (2, 256, 4)
    for i, b in [(0, 0x00), (0, 0x3a), (1, 0xf1), (1, 0x0f)]:
        assert torch.equal(P[i, b, :2], cb[2 * i, b & 15]) and torch.equal(P[i, b, 2:], cb[2 * i + 1, b >> 4])
