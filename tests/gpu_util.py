"""Helpers of the GPU parity tests: device buffers, a context per configuration, and the
oracle-side conversion of coefficient-form polynomials into the library's evaluation layout
(the oracle's own transform, permuted with the library's published index map)."""
import numpy as np
import torch

from oracle import oracle as O
from paper_2207_04604_amd import binding as B

DEV = torch.device("cuda:0")


def dzeros(n_words, dtype=torch.int64):
    return torch.zeros(n_words, dtype=dtype, device=DEV)


def to_dev(a: np.ndarray):
    if a.dtype == np.uint64:
        return torch.from_numpy(a.view(np.int64).copy()).to(DEV)
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def to_host(t: torch.Tensor, shape=None):
    a = t.cpu().numpy()
    if a.dtype == np.int64:
        a = a.view(np.uint64)
    return a.reshape(shape) if shape is not None else a


def make_ctx(log2_n, q, t, eta=21, f=0, max_group=1, seed=0):
    return B.Context(log2_n, q, t, eta, f, max_group, seed,
                     alloc=lambda n: torch.zeros(n // 8 + 2, dtype=torch.int64, device=DEV))


def make_pair(cfg, max_group=None):
    """(oracle, library context, index map) for a synth.Config."""
    mg = cfg.max_group if max_group is None else max_group
    o = O.Oracle(cfg.log2_n, cfg.q, cfg.t, cfg.eta, cfg.frac_bits, mg, cfg.seed)
    ctx = make_ctx(cfg.log2_n, cfg.q, cfg.t, cfg.eta, cfg.frac_bits, mg, cfg.seed)
    return o, ctx, ctx.index_map()


def to_eval(o, perm, poly):
    """poly [..., L, N] in coefficient form -> evaluation form in the library's layout."""
    out = np.zeros_like(poly)
    fin, fout = poly.reshape(-1, o.L, o.N), out.reshape(-1, o.L, o.N)
    for b in range(fin.shape[0]):
        for i in range(o.L):
            fout[b, i] = O.ntt_forward(fin[b, i], o.q[i], o.psi[i])[perm]
    return out


class Keys:
    """Key shares of parties 0..P-1 on both sides, and per-group public keys."""

    def __init__(self, o, ctx, perm, parties, check=True):
        L, N = o.L, o.N
        self.o, self.ctx = o, ctx
        self.osk, self.opk0, self.sk, self.pk0 = {}, {}, {}, {}
        for k in parties:
            sk, pk0, _, _ = o.keygen_share(k)
            self.osk[k], self.opk0[k] = sk, pk0
            dsk, dpk0 = dzeros(2 * L * N), dzeros(L * N)
            ctx.keygen_share(k, dsk, dpk0)
            self.sk[k], self.pk0[k] = dsk, dpk0
            if check:
                hsk = to_host(dsk, (2, L, N))
                assert np.array_equal(hsk[0], to_eval(o, perm, sk)), f"secret share of party {k}"
                assert np.array_equal(to_host(dpk0, (L, N)), to_eval(o, perm, pk0)), f"pk share of party {k}"
                for i in range(L):           # Shoup quotients, spot-checked with Python integers
                    for j in range(0, N, 257):
                        assert int(hsk[1, i, j]) == (int(hsk[0, i, j]) << 64) // o.q[i]

    def group_pk(self, members, perm=None, check=True):
        o, ctx = self.o, self.ctx
        opk = o.aggregate_pk([self.opk0[k] for k in members])
        dpk = dzeros(4 * o.L * o.N)
        ctx.aggregate_pk([self.pk0[k] for k in members], dpk)
        if check and perm is not None:
            h = to_host(dpk, (2, 2, o.L, o.N))
            assert np.array_equal(h[0, 0], to_eval(o, perm, opk[0])), "p0"
            assert np.array_equal(h[1, 0], to_eval(o, perm, opk[1])), "p1"
        return opk, dpk
