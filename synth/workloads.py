"""Seeded synthetic workloads: Gaussian-mixture embeddings, trained IVF-PQ indexes, queries.

This module only *produces inputs*: database vectors, a trained index (coarse
centroids, PQ codebooks, list-major codes and ids) and query batches.  It holds
none of the search arithmetic; both the CPU oracle and the HIP library consume
the very same bytes it emits.  Everything is written with plain torch ops so it
runs on the host for small cases and on the GPU for the large ones.

Stand-in for the paper's retrieval corpora (a 64-billion-passage store of
768-dimensional embeddings compressed to 96-byte PQ codes, Section 4 "Models
and database"; per-request corpora of 1K-100K 768-d chunk embeddings,
Section 5.2), none of which is public: unit-norm mixture samples with the same
dimensions, code sizes and scan fractions.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Dict, Optional

import torch

KSUB = 256  # codewords per PQ sub-quantiser (8-bit codes)


# --------------------------------------------------------------------------- configs
@dataclasses.dataclass(frozen=True)
class IvfPqConfig:
    """Shape of one IVF-PQ workload (data, index and search parameters)."""

    name: str
    n: int            # database vectors
    d: int            # dimension
    m: int            # PQ sub-quantisers (bytes per code)
    nlist: int        # coarse centroids / inverted lists
    components: int   # mixture components
    var_lo: float     # per-dimension variance range of a component (lo == hi: isotropic)
    var_hi: float
    train_n: int      # vectors in the k-means training sample
    nq: int
    nprobe: int
    k: int
    seed: int
    assign: str = "exact"   # "exact" | "component" (see build_index)
    kmeans_iters: int = 8
    pq_train_n: int = 65536
    ksub: int = 256         # codewords per sub-quantiser; 16 = 4-bit codes, two per byte (m/2 bytes per code)

    def scaled(self, **kw) -> "IvfPqConfig":
        return dataclasses.replace(self, **kw)


# The five workload shapes.  Seeds: 1000 + workload number; every random stream
# (mixture, training sample, database, queries) is a separate generator derived from it.
TINY = IvfPqConfig("tiny", n=1_000_000, d=128, m=16, nlist=1024, components=256,
                   var_lo=1.0, var_hi=1.0, train_n=131072, nq=64, nprobe=16, k=10, seed=1001)
MID = IvfPqConfig("mid", n=10_000_000, d=768, m=96, nlist=16384, components=4096,
                  var_lo=0.1, var_hi=2.0, train_n=1_000_000, nq=256, nprobe=64, k=100, seed=1002,
                  kmeans_iters=6)
HYPER = IvfPqConfig("hyper", n=1_000_000_000, d=768, m=96, nlist=65536, components=16384,
                    var_lo=0.1, var_hi=2.0, train_n=2_000_000, nq=1024, nprobe=128, k=100,
                    seed=1003, assign="component", kmeans_iters=4)
# iterative retrieval runs on the HYPER index: 8 rounds, batches 1/4/16, nprobe 256, k 10
ITER_ROUNDS, ITER_BATCHES, ITER_NPROBE, ITER_K, ITER_DRIFT = 8, (1, 4, 16), 256, 10, 0.05


@dataclasses.dataclass(frozen=True)
class FlatConfig:
    name: str
    requests: int
    n: int
    d: int
    nq: int
    k: int
    components: int
    seed: int


FLAT = FlatConfig("flat", requests=32, n=100_000, d=768, nq=16, k=32, components=64, seed=1005)


# --------------------------------------------------------------------------- mixture
def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


class GaussianMixture:
    """Uniform-weight mixture: means ~ N(0, 4 I); per-component diagonal variance drawn
    log-uniformly from [var_lo, var_hi] per dimension (isotropic unit variance if equal)."""

    def __init__(self, d: int, components: int, var_lo: float, var_hi: float, seed: int, device="cpu"):
        self.d, self.components, self.device = d, components, torch.device(device)
        g = _gen(seed, self.device)
        self.means = 2.0 * torch.randn(components, d, generator=g, device=self.device)
        if var_lo == var_hi:
            self.sigma = torch.full((components, d), math.sqrt(var_lo), device=self.device)
        else:
            u = torch.rand(components, d, generator=g, device=self.device)
            var = torch.exp(math.log(var_lo) + u * (math.log(var_hi) - math.log(var_lo)))
            self.sigma = var.sqrt()

    def raw(self, comp: torch.Tensor, g: torch.Generator) -> torch.Tensor:
        """Un-normalised samples of the given components."""
        z = torch.randn(comp.numel(), self.d, generator=g, device=self.device)
        return self.means[comp] + self.sigma[comp] * z

    def sample(self, n: int, g: torch.Generator):
        comp = torch.randint(0, self.components, (n,), generator=g, device=self.device)
        x = self.raw(comp, g)
        return torch.nn.functional.normalize(x, dim=1), comp


# --------------------------------------------------------------------------- k-means
def _nearest_l2(x: torch.Tensor, c: torch.Tensor, chunk: int = 65536) -> torch.Tensor:
    out = torch.empty(x.shape[0], dtype=torch.int64, device=x.device)
    half = 0.5 * (c * c).sum(1)
    for a in range(0, x.shape[0], chunk):
        out[a:a + chunk] = (x[a:a + chunk] @ c.T - half).argmax(1)
    return out


def kmeans(x: torch.Tensor, kc: int, iters: int, g: torch.Generator) -> torch.Tensor:
    """Plain Lloyd iterations in L2, random-sample initialisation, fixed iteration count.
    Empty clusters are re-seeded from random training points."""
    n = x.shape[0]
    perm = torch.randperm(n, generator=g, device=x.device)
    c = x[perm[:kc]].clone() if n >= kc else x[torch.randint(0, n, (kc,), generator=g, device=x.device)].clone()
    for _ in range(iters):
        a = _nearest_l2(x, c)
        cnt = torch.bincount(a, minlength=kc)
        s = torch.zeros_like(c).index_add_(0, a, x)
        nz = cnt > 0
        c[nz] = s[nz] / cnt[nz].unsqueeze(1).to(c.dtype)
        ne = int((~nz).sum())
        if ne:
            c[~nz] = x[torch.randint(0, n, (ne,), generator=g, device=x.device)]
    return c


def _pq_train(res: torch.Tensor, m: int, iters: int, g: torch.Generator, ksub: int = KSUB) -> torch.Tensor:
    """Per-subspace k-means on residuals: returns codebooks [m][ksub][dsub]."""
    n, d = res.shape
    dsub = d // m
    r = res.view(n, m, dsub).permute(1, 0, 2).contiguous()            # [m][n][dsub]
    idx = torch.randperm(n, generator=g, device=res.device)[:ksub]
    if idx.numel() < ksub:
        idx = torch.randint(0, n, (ksub,), generator=g, device=res.device)
    cb = r[:, idx, :].clone()                                          # [m][ksub][dsub]
    for _ in range(iters):
        a = _pq_assign(r, cb)                                          # [m][n]
        one = torch.ones_like(a, dtype=res.dtype)
        cnt = torch.zeros(m, ksub, device=res.device, dtype=res.dtype).scatter_add_(1, a, one)
        s = torch.zeros_like(cb).scatter_add_(1, a.unsqueeze(2).expand(-1, -1, dsub), r)
        nz = cnt > 0
        cb = torch.where(nz.unsqueeze(2), s / cnt.clamp(min=1).unsqueeze(2), cb)
    return cb


def _pq_assign(r: torch.Tensor, cb: torch.Tensor, chunk: int = 32768) -> torch.Tensor:
    """r [m][n][dsub], cb [m][256][dsub] -> nearest codeword index [m][n] (L2)."""
    m, n, _ = r.shape
    half = 0.5 * (cb * cb).sum(2)                                      # [m][256]
    out = torch.empty(m, n, dtype=torch.int64, device=r.device)
    for a in range(0, n, chunk):
        sc = torch.bmm(r[:, a:a + chunk, :], cb.transpose(1, 2)) - half.unsqueeze(1)
        out[:, a:a + chunk] = sc.argmax(2)
    return out


def pairs_of_codewords(cb16: torch.Tensor) -> torch.Tensor:
    """[m][16][dsub] -> [m/2][256][2 dsub]: entry b of pair i = codeword (b & 15) of sub-quantiser 2i followed by
    codeword (b >> 4) of sub-quantiser 2i+1 (the byte layout of a 4-bit code).  Used to ENCODE the database only."""
    m, ks, dsub = cb16.shape
    assert ks == 16 and m % 2 == 0
    b = torch.arange(256, device=cb16.device)
    lo = cb16[0::2][:, b & 15, :]                                      # [m/2][256][dsub]
    hi = cb16[1::2][:, b >> 4, :]
    return torch.cat([lo, hi], dim=2).contiguous()


def pq_encode(res: torch.Tensor, cb: torch.Tensor) -> torch.Tensor:
    """res [n][d] residuals -> codes uint8 [n][m]."""
    n, d = res.shape
    m = cb.shape[0]
    r = res.view(n, m, d // m).permute(1, 0, 2).contiguous()
    return _pq_assign(r, cb).T.contiguous().to(torch.uint8)


# --------------------------------------------------------------------------- index
def _assign_exact(x: torch.Tensor, c: torch.Tensor, chunk: int = 65536) -> torch.Tensor:
    """List of a vector = the centroid with the largest inner product (the function the
    search ranks lists by), so a database vector used as a query probes its own list first."""
    out = torch.empty(x.shape[0], dtype=torch.int64, device=x.device)
    for a in range(0, x.shape[0], chunk):
        out[a:a + chunk] = (x[a:a + chunk] @ c.T).argmax(1)
    return out


def _native_encode_available() -> bool:
    try:
        from . import native
        return native.available()
    except Exception:
        return False


def build_index(cfg: IvfPqConfig, device="cpu", keep_vectors: Optional[bool] = None,
                chunk: int = 1 << 20, progress=None) -> Dict[str, torch.Tensor]:
    """Generate the database and train/encode an IVF-PQ index for it.

    Returns a dict of tensors on `device`:
      centroids [nlist][d] f32, codebooks [m][ksub][dsub] f32, list_offsets [nlist+1] i64,
      codes [n][m] u8 ([n][m/2] with cfg.ksub = 16; list-major, plain rows), ids [n] i64 (list-major, ascending inside
      a list), and `vectors` [n][d] f32 (id-major) when kept.
    `assign="component"`: the list of a sample is chosen among the 16 centroids with the
    largest inner product to its mixture component's normalised mean instead of among all
    nlist (same argmax rule; used at the billion-vector size where the full assignment
    GEMM alone is ~1e17 flop).
    """
    dev = torch.device(device)
    mix = GaussianMixture(cfg.d, cfg.components, cfg.var_lo, cfg.var_hi, cfg.seed * 10 + 1, dev)
    g_train, g_db = _gen(cfg.seed * 10 + 2, dev), _gen(cfg.seed * 10 + 3, dev)
    if keep_vectors is None:
        keep_vectors = cfg.n * cfg.d * 4 <= (1 << 30)

    xt, _ = mix.sample(min(cfg.train_n, max(cfg.n, cfg.nlist * 4)), g_train)
    centroids = kmeans(xt, cfg.nlist, cfg.kmeans_iters, g_train)
    sub = xt[: cfg.pq_train_n]
    res = sub - centroids[_assign_exact(sub, centroids)]
    codebooks = _pq_train(res, cfg.m, cfg.kmeans_iters, g_train, cfg.ksub)
    del xt, sub, res
    user_codebooks = codebooks
    code_bytes = cfg.m
    if cfg.ksub == 16:
        # the nearest pair of 16-word codewords is the nearest of their 256 concatenations (squared distance
        # adds over the two halves), so encoding against the concatenations yields the packed byte directly
        codebooks = pairs_of_codewords(codebooks)
        code_bytes = cfg.m // 2

    n = cfg.n
    codes_arr = torch.empty(n, code_bytes, dtype=torch.uint8, device=dev)   # arrival (= id) order
    lists_arr = torch.empty(n, dtype=torch.int32, device=dev)
    vectors = torch.empty(n, cfg.d, device=dev) if keep_vectors else None
    use_native = dev.type == "cuda" and _native_encode_available()

    def emit(a, x, li):
        b = a + x.shape[0]
        if use_native:
            from . import native
            native.pq_encode(x.contiguous(), centroids, li.contiguous(), codebooks, codes_arr[a:b])
        else:
            codes_arr[a:b] = pq_encode(x - centroids[li], codebooks)
        lists_arr[a:b] = li.to(torch.int32)
        if vectors is not None:
            vectors[a:b] = x
        if progress:
            progress(b, n)

    if cfg.assign == "exact":
        for a in range(0, n, chunk):
            x, _ = mix.sample(min(n, a + chunk) - a, g_db)
            emit(a, x, _assign_exact(x, centroids))
    elif cfg.assign == "component":
        # component-major stream: every component contributes ceil(n / G) consecutive samples, so
        # the 16 candidate centroids are shared by a whole slab and scored with one batched GEMM
        G = cfg.components
        mu = torch.nn.functional.normalize(mix.means, dim=1)
        cand = (mu @ centroids.T).topk(min(16, cfg.nlist), dim=1).indices          # [G][16]
        per = -(-n // G)
        gc = max(1, chunk // per)
        a = 0
        for g0 in range(0, G, gc):
            if a >= n:
                break
            comps = torch.arange(g0, min(G, g0 + gc), device=dev)
            x = mix.raw(comps.repeat_interleave(per), g_db)
            x = torch.nn.functional.normalize(x, dim=1)
            sc = torch.bmm(x.view(comps.numel(), per, cfg.d), centroids[cand[comps]].transpose(1, 2))   # [gc][per][16]
            li = torch.gather(cand[comps], 1, sc.argmax(2)).reshape(-1)
            take = min(x.shape[0], n - a)
            emit(a, x[:take], li[:take])
            a += take
    else:
        raise ValueError(cfg.assign)

    order = torch.sort(lists_arr, stable=True).indices                 # ids ascend inside a list
    counts = torch.bincount(lists_arr.to(torch.int64), minlength=cfg.nlist)
    del lists_arr
    offsets = torch.zeros(cfg.nlist + 1, dtype=torch.int64, device=dev)
    offsets[1:] = counts.cumsum(0)
    codes = torch.empty_like(codes_arr)
    for a in range(0, n, 1 << 24):
        codes[a:a + (1 << 24)] = codes_arr[order[a:a + (1 << 24)]]
    del codes_arr
    if dev.type == "cuda":
        torch.cuda.empty_cache()
    out = dict(centroids=centroids, codebooks=user_codebooks, list_offsets=offsets, codes=codes,
               ids=order.to(torch.int64))
    if vectors is not None:
        out["vectors"] = vectors
    return out


def build_upper_level(centroids: torch.Tensor, nsuper: int, seed: int, iters: int = 10, spherical: bool = True) -> dict:
    """An upper level over the lists: Lloyd k-means of the list centroids into `nsuper` groups (seeded), every
    list in the group of its nearest group centroid.  `spherical` (for inner-product search over unit-norm
    data): cluster the directions of the centroids and give every group centroid unit norm, so that the
    inner product with a query ranks groups by direction and not by how tight a group happens to be.
    Returns super_centroids [nsuper][d] f32, super_offsets [nsuper+1] i64, super_lists [nlist] i32 (lists
    grouped by group, ascending inside a group)."""
    g = _gen(seed, centroids.device)
    x = centroids.float()
    if spherical:
        x = torch.nn.functional.normalize(x, dim=1)
    sc = kmeans(x, nsuper, iters, g)
    if spherical:
        sc = torch.nn.functional.normalize(sc, dim=1)
    owner = _nearest_l2(x, sc)
    order = torch.argsort(owner * centroids.shape[0] + torch.arange(centroids.shape[0], device=centroids.device))
    off = torch.zeros(nsuper + 1, dtype=torch.int64, device=centroids.device)
    off[1:] = torch.cumsum(torch.bincount(owner, minlength=nsuper), 0)
    return dict(super_centroids=sc.contiguous(), super_offsets=off, super_lists=order.to(torch.int32).contiguous())


def make_queries(cfg: IvfPqConfig, nq: Optional[int] = None, device="cpu", noise: float = 0.1,
                 stream: int = 4) -> torch.Tensor:
    """Queries = un-normalised mixture samples + N(0, noise^2) per coordinate, then L2-normalised."""
    dev = torch.device(device)
    mix = GaussianMixture(cfg.d, cfg.components, cfg.var_lo, cfg.var_hi, cfg.seed * 10 + 1, dev)
    g = _gen(cfg.seed * 10 + stream, dev)
    nq = cfg.nq if nq is None else nq
    comp = torch.randint(0, cfg.components, (nq,), generator=g, device=dev)
    x = mix.raw(comp, g) + noise * torch.randn(nq, cfg.d, generator=g, device=dev)
    return torch.nn.functional.normalize(x, dim=1).contiguous()


def drift_queries(q: torch.Tensor, sigma: float, g: torch.Generator) -> torch.Tensor:
    """Next round of an iterative-retrieval chain: q + N(0, sigma^2) per coordinate, renormalised."""
    return torch.nn.functional.normalize(
        q + sigma * torch.randn(q.shape, generator=g, device=q.device), dim=1).contiguous()


def make_flat(cfg: FlatConfig, requests: Optional[int] = None, n: Optional[int] = None, device="cpu"):
    """Per-request private corpora and queries, bf16: corpus [R][n][d], queries [R][nq][d]."""
    dev = torch.device(device)
    R = cfg.requests if requests is None else requests
    n = cfg.n if n is None else n
    corpus = torch.empty(R, n, cfg.d, dtype=torch.bfloat16, device=dev)
    queries = torch.empty(R, cfg.nq, cfg.d, dtype=torch.bfloat16, device=dev)
    for r in range(R):
        mix = GaussianMixture(cfg.d, cfg.components, 1.0, 1.0, cfg.seed * 1000 + r, dev)
        g = _gen(cfg.seed * 1000 + 500 + r, dev)
        x, _ = mix.sample(n, g)
        corpus[r] = x.to(torch.bfloat16)
        comp = torch.randint(0, cfg.components, (cfg.nq,), generator=g, device=dev)
        qv = mix.raw(comp, g) + 0.1 * torch.randn(cfg.nq, cfg.d, generator=g, device=dev)
        queries[r] = torch.nn.functional.normalize(qv, dim=1).to(torch.bfloat16)
    return corpus, queries


# --------------------------------------------------------------------------- hand-made tiny index
def random_index(n: int, d: int, m: int, nlist: int, seed: int, empty_lists=(), dup_codes: int = 0,
                 shuffle_ids: bool = False, cb_scale: float = 0.3, ksub: int = KSUB) -> Dict[str, torch.Tensor]:
    """Small index with random (untrained) centroids/codebooks/codes for brute-force checks.
    `empty_lists`: list numbers forced empty; `dup_codes`: that many vectors get a copy of
    another vector's code in the same list (forces exact score ties); `shuffle_ids`: ids are a
    random permutation instead of 0..n-1 (still ascending inside each list); `cb_scale`: magnitude of the
    codewords relative to the centroids (tiny values give nearly constant look-up tables); `ksub` = 16: a 4-bit
    PQ index, m sub-quantisers of 16 codewords, two per code byte (even one in the low nibble)."""
    g = _gen(seed, "cpu")
    centroids = torch.randn(nlist, d, generator=g) / math.sqrt(d)
    assert ksub in (16, KSUB)
    codebooks = cb_scale * torch.randn(m, ksub, d // m, generator=g) / math.sqrt(d)
    live = torch.tensor([l for l in range(nlist) if l not in set(empty_lists)])
    li = live[torch.randint(0, live.numel(), (n,), generator=g)]
    order = torch.sort(li, stable=True).indices
    counts = torch.bincount(li, minlength=nlist)
    offsets = torch.zeros(nlist + 1, dtype=torch.int64)
    offsets[1:] = counts.cumsum(0)
    codes = torch.randint(0, KSUB, (n, m if ksub == KSUB else m // 2), generator=g, dtype=torch.int64).to(torch.uint8)
    for _ in range(dup_codes):
        l = int(live[torch.randint(0, live.numel(), (1,), generator=g)])
        a, b = int(offsets[l]), int(offsets[l + 1])
        if b - a >= 2:
            i, j = torch.randint(a, b, (2,), generator=g).tolist()
            codes[i] = codes[j]
    if shuffle_ids:
        perm = torch.randperm(n, generator=g) * 7 + 3       # sparse, non-contiguous ids
        ids = torch.empty(n, dtype=torch.int64)
        for l in range(nlist):
            a, b = int(offsets[l]), int(offsets[l + 1])
            ids[a:b] = torch.sort(perm[a:b]).values
    else:
        ids = order.to(torch.int64)
    return dict(centroids=centroids, codebooks=codebooks, list_offsets=offsets, codes=codes, ids=ids)
