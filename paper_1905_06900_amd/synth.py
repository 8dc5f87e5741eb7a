"""Seeded synthetic inputs for the five benchmark workloads.

This module only manufactures *inputs* (codebooks, code arrays, queries, inverted-list layouts)
as materialised tensors; it holds none of the search arithmetic.  Both the CPU oracle and the GPU
library consume the very same bytes.  Everything is a function of (workload, scale, seed, device);
the CPU and GPU random streams of torch differ, so arrays are generated once per run and shared.

Stand-ins: the paper evaluates on SIFT1M, TINY10M (GIST) and SIFT1B, none of which is available
here.  The generators below produce data with the same dimensionalities, value ranges and code
shapes.  Codebooks are hierarchical so that property P1 of Sec. 3.2 is meaningful: each
sub-quantizer has 2^pbits "parents" and 2^(b-pbits) children per parent, and the centroid index
is (child << pbits) | parent, i.e. the parent sits in the LOW bits, so every group of centroids
that shares its low bbar bits (bbar >= pbits) consists of children of one parent.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import torch


@dataclass(frozen=True)
class Workload:
    name: str
    kind: str            # "flat" | "ivf"
    m: int               # sub-quantizers
    dsub: int            # dims per sub-quantizer
    N: int               # database size
    Q: int               # queries per batch
    r: int               # candidate-set size kept by pass one
    k: int               # result-set size
    data: str            # "zipf_codes" | "sift_gmm" | "deep_random_codes" | "gist_gmm" | "sift_ivf"
    nlist: int = 0
    nprobe: int = 0
    b: int = 16
    bbar: int = 8
    pbits: int = 4
    seed: int = 190506900

    @property
    def D(self) -> int:
        return self.m * self.dsub


WORKLOADS = {
    # Flat PQ 4x16, SIFT1M-shaped 64-bit codes.
    0: Workload("cfg0_flat_pq4x16_d128_n1m", "flat", 4, 32, 1_000_000, 100, 1000, 100, "zipf_codes"),
    # Flat PQ 8x16, SIFT-like 128-d, encoded by nearest centroid.
    1: Workload("cfg1_flat_pq8x16_sift_n10m", "flat", 8, 16, 10_000_000, 1000, 2000, 100, "sift_gmm"),
    # Flat PQ 8x16, Deep-like 96-d, random codes (the headline scan workload).
    2: Workload("cfg2_flat_pq8x16_deep_n100m", "flat", 8, 12, 100_000_000, 4096, 4000, 100, "deep_random_codes"),
    # IVF(65536, nprobe 64) + PQ 8x16 on residuals, SIFT1B-shaped.
    3: Workload("cfg3_ivf_pq8x16_sift_n1b", "ivf", 8, 16, 1_000_000_000, 1024, 1000, 100, "sift_ivf",
                nlist=65536, nprobe=64),
    # Flat PQ 16x16, GIST-like 960-d.
    4: Workload("cfg4_flat_pq16x16_gist_n10m", "flat", 16, 60, 10_000_000, 512, 5000, 100, "gist_gmm"),
}


def scaled(w: Workload, N: int | None = None, Q: int | None = None, r: int | None = None,
           nlist: int | None = None, nprobe: int | None = None) -> Workload:
    """Same recipe at a smaller size (parity cases the CPU oracle finishes in seconds)."""
    kw = {}
    if N is not None: kw["N"] = int(N)
    if Q is not None: kw["Q"] = int(Q)
    if r is not None: kw["r"] = int(r)
    if nlist is not None: kw["nlist"] = int(nlist)
    if nprobe is not None: kw["nprobe"] = int(nprobe)
    return replace(w, **kw)


def _gen(device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


# ------------------------------------------------------------------------------------------------
# codebooks
# ------------------------------------------------------------------------------------------------
def hierarchical_codebooks(m: int, dsub: int, b: int, pbits: int, parent_sampler, sigma_c: float,
                           device, seed: int) -> torch.Tensor:
    """[m][2^b][dsub] fp32; index = (child << pbits) | parent."""
    g = _gen(device, seed)
    npar, nchild = 1 << pbits, 1 << (b - pbits)
    parents = parent_sampler((m, npar, dsub), g)                      # [m][npar][dsub]
    noise = torch.randn((m, nchild, npar, dsub), generator=g, device=device, dtype=torch.float32)
    cb = parents[:, None, :, :] + sigma_c * noise                     # [m][child][parent][dsub]
    return cb.reshape(m, nchild * npar, dsub).contiguous()            # row = child*npar + parent


def _uniform(lo: float, hi: float, device):
    def f(shape, g):
        return lo + (hi - lo) * torch.rand(shape, generator=g, device=device, dtype=torch.float32)
    return f


def _normal(sigma: float, device):
    def f(shape, g):
        return sigma * torch.randn(shape, generator=g, device=device, dtype=torch.float32)
    return f


# ------------------------------------------------------------------------------------------------
# vectors
# ------------------------------------------------------------------------------------------------
def _gmm(n: int, means: torch.Tensor, sigma: float, g: torch.Generator, device) -> torch.Tensor:
    comp = torch.randint(0, means.shape[0], (n,), generator=g, device=device)
    x = means[comp] + sigma * torch.randn((n, means.shape[1]), generator=g, device=device, dtype=torch.float32)
    return x


def sift_like(n: int, device, seed: int, means_seed: int) -> torch.Tensor:
    """1024-component mixture, means ~ U[0,160]^128, sigma 12, clipped to [0,255], rounded."""
    gm = _gen(device, means_seed)
    means = 160.0 * torch.rand((1024, 128), generator=gm, device=device, dtype=torch.float32)
    x = _gmm(n, means, 12.0, _gen(device, seed), device)
    return x.clamp_(0.0, 255.0).round_()


def deep_like(n: int, device, seed: int, means_seed: int) -> torch.Tensor:
    """4096-component mixture around random unit means, sigma 0.05, unit-normalised, 96-d."""
    gm = _gen(device, means_seed)
    means = torch.randn((4096, 96), generator=gm, device=device, dtype=torch.float32)
    means = means / means.norm(dim=1, keepdim=True)
    x = _gmm(n, means, 0.05, _gen(device, seed), device)
    return x / x.norm(dim=1, keepdim=True)


def gist_like(n: int, device, seed: int, means_seed: int) -> torch.Tensor:
    """1024-component mixture, means ~ U[0,0.3]^960, sigma 0.03."""
    gm = _gen(device, means_seed)
    means = 0.3 * torch.rand((1024, 960), generator=gm, device=device, dtype=torch.float32)
    return _gmm(n, means, 0.03, _gen(device, seed), device)


def encode_nearest(x: torch.Tensor, cb: torch.Tensor, chunk: int = 8192) -> torch.Tensor:
    """Offline encoding used only to manufacture code arrays: nearest centroid per sub-space.

    x [n][m*dsub], cb [m][K][dsub] -> codes [n][m] as int16 bit patterns of the unsigned index.
    """
    m, K, dsub = cb.shape
    n = x.shape[0]
    out = torch.empty((n, m), dtype=torch.int32, device=x.device)
    cn = (cb.double() ** 2).sum(-1).float()                             # [m][K]
    for j in range(m):
        cj = cb[j]
        for s in range(0, n, chunk):
            xs = x[s:s + chunk, j * dsub:(j + 1) * dsub]
            d = cn[j][None, :] - 2.0 * (xs @ cj.T)
            out[s:s + chunk, j] = d.argmin(dim=1).to(torch.int32)
    return out.to(torch.int16)        # bit pattern of the unsigned 16-bit index


def random_codes(n: int, m: int, device, seed: int, chunk: int = 1 << 26) -> torch.Tensor:
    """Uniform random 16-bit sub-codes, [n][m] (int16 bit patterns)."""
    g = _gen(device, seed)
    out = torch.empty((n, m), dtype=torch.int16, device=device)
    flat = out.view(-1)
    for s in range(0, flat.numel(), chunk):
        e = min(flat.numel(), s + chunk)
        flat[s:e] = torch.randint(-32768, 32768, (e - s,), generator=g, device=device, dtype=torch.int16)
    return out


def zipf_codes(n: int, m: int, b: int, pbits: int, device, seed: int) -> torch.Tensor:
    """Per sub-code: parent ~ Zipf(1.1) over the 2^pbits parents, child uniform."""
    g = _gen(device, seed)
    npar, nchild = 1 << pbits, 1 << (b - pbits)
    w = 1.0 / torch.arange(1, npar + 1, device=device, dtype=torch.float64) ** 1.1
    parent = torch.multinomial((w / w.sum()).float(), n * m, replacement=True, generator=g).view(n, m)
    child = torch.randint(0, nchild, (n, m), generator=g, device=device)
    code = (child << pbits) | parent
    return code.to(torch.int32).to(torch.int16)


def decode(codes_i16: torch.Tensor, cb: torch.Tensor) -> torch.Tensor:
    """Concatenate the centroids a code names (input manufacture for cfg 0's queries)."""
    m = cb.shape[0]
    idx = codes_i16.to(torch.int32) & 0xFFFF
    return torch.cat([cb[j][idx[:, j].long()] for j in range(m)], dim=1)


# ------------------------------------------------------------------------------------------------
# whole workloads
# ------------------------------------------------------------------------------------------------
def make_flat(w: Workload, device="cpu") -> dict:
    """Returns dict(codebooks [m][2^b][dsub] f32, codes [N][m] u16, queries [Q][D] f32)."""
    assert w.kind == "flat"
    s = w.seed
    if w.data == "zipf_codes":
        cb = hierarchical_codebooks(w.m, w.dsub, w.b, w.pbits, _uniform(0.0, 128.0, device), 4.0, device, s + 1)
        codes = zipf_codes(w.N, w.m, w.b, w.pbits, device, s + 2)
        g = _gen(device, s + 3)
        pick = torch.randint(0, w.N, (w.Q,), generator=g, device=device)
        y = decode(codes[pick], cb)
        y = y + 8.0 * torch.randn(y.shape, generator=g, device=device, dtype=torch.float32)
        queries = y.clamp_(0.0, 255.0)
    elif w.data == "sift_gmm":
        cb = hierarchical_codebooks(w.m, w.dsub, w.b, w.pbits, _uniform(0.0, 160.0, device), 12.0, device, s + 1)
        codes = _encode_chunked(lambda n, sd: sift_like(n, device, sd, s + 7), w.N, cb, s + 2)
        queries = sift_like(w.Q, device, s + 3, s + 7)
    elif w.data == "deep_random_codes":
        cb = hierarchical_codebooks(w.m, w.dsub, w.b, w.pbits, _normal(96 ** -0.5, device), 0.03, device, s + 1)
        codes = random_codes(w.N, w.m, device, s + 2)
        queries = deep_like(w.Q, device, s + 3, s + 7)
    elif w.data == "gist_gmm":
        cb = hierarchical_codebooks(w.m, w.dsub, w.b, w.pbits, _uniform(0.0, 0.3, device), 0.03, device, s + 1)
        codes = _encode_chunked(lambda n, sd: gist_like(n, device, sd, s + 7), w.N, cb, s + 2)
        queries = gist_like(w.Q, device, s + 3, s + 7)
    else:
        raise ValueError(w.data)
    return dict(codebooks=cb.contiguous(), codes=codes.contiguous().view(torch.uint16),
                queries=queries.contiguous())


def _encode_chunked(sampler, n: int, cb: torch.Tensor, seed: int, block: int = 1 << 18) -> torch.Tensor:
    parts = []
    for i, s in enumerate(range(0, n, block)):
        x = sampler(min(block, n - s), seed + 1000 * (i + 1))
        parts.append(encode_nearest(x, cb))
    return torch.cat(parts, dim=0)


def zipf_list_offsets(nlist: int, N: int, device, seed: int) -> torch.Tensor:
    """List sizes ~ 1/rank^0.8 over a seeded permutation of the lists, summing to exactly N;
    returns CSR offsets int64 [nlist+1]."""
    g = _gen("cpu", seed)
    w = 1.0 / torch.arange(1, nlist + 1, dtype=torch.float64) ** 0.8
    sizes = torch.floor(w / w.sum() * N).to(torch.int64)
    sizes[0] += N - int(sizes.sum())
    perm = torch.randperm(nlist, generator=g)
    sizes = sizes[perm]
    off = torch.zeros(nlist + 1, dtype=torch.int64)
    off[1:] = torch.cumsum(sizes, 0)
    return off.to(device)


def make_ivf(w: Workload, device="cpu") -> dict:
    """Returns dict(codebooks, coarse [nlist][D], offsets int64 [nlist+1], codes [N][m], queries)."""
    assert w.kind == "ivf"
    s = w.seed
    coarse = sift_like(w.nlist, device, s + 11, s + 7)
    # residual-scale product quantizer
    cb = hierarchical_codebooks(w.m, w.dsub, w.b, w.pbits, _normal(20.0, device), 6.0, device, s + 1)
    offsets = zipf_list_offsets(w.nlist, w.N, device, s + 12)
    codes = random_codes(w.N, w.m, device, s + 2)
    queries = sift_like(w.Q, device, s + 3, s + 7)
    return dict(codebooks=cb.contiguous(), coarse=coarse.contiguous(), offsets=offsets,
                codes=codes.view(torch.uint16), queries=queries.contiguous())


def to_numpy(t: torch.Tensor):
    """Host numpy view of a tensor (uint16 goes through its int16 bit pattern)."""
    import numpy as np
    if t.dtype == torch.uint16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    if t.dtype == torch.uint32:
        return t.view(torch.int32).cpu().numpy().view(np.uint32)
    return t.cpu().numpy()
