"""ctypes front-end of the CPU oracle (``d2mhe_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by the test-suite, the smoke check and the CPU-baseline
leg of the benchmark.  The HIP library never touches it, and this module never touches the
HIP library.  All arithmetic lives in the C file; this module only marshals numpy arrays.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "libd2mhe_oracle.so")
_SRC = os.path.join(_HERE, "d2mhe_oracle.c")
MAX_LIMBS = 16

DOM_SK, DOM_PK_E, DOM_CRS, DOM_ENC_U, DOM_ENC_E0, DOM_ENC_E1, DOM_DEC_E, DOM_BENCH = range(1, 9)


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP only used by the batch/timing drivers)."""
    hdr = os.path.join(_HERE, "d2mhe_oracle.h")
    stale = (not os.path.exists(_SO)) or any(
        os.path.getmtime(f) > os.path.getmtime(_SO) for f in (_SRC, hdr))
    if force or stale:
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp",
                               "-Wall", "-Wextra", "-o", _SO, _SRC, "-lm"])
    return _SO


class _Params(C.Structure):
    _fields_ = [("log2_n", C.c_uint32), ("num_limbs", C.c_uint32),
                ("q", C.c_uint64 * MAX_LIMBS), ("t", C.c_uint64),
                ("cbd_eta", C.c_uint32), ("frac_bits", C.c_uint32),
                ("max_group", C.c_uint32), ("seed", C.c_uint64)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        # D2MHE_ORACLE_LIBRARY: a build of this oracle from another source file (the test-suite points
        # it at copies with a planted mistake to check that the pins notice)
        _lib = C.CDLL(os.environ.get("D2MHE_ORACLE_LIBRARY") or build())
        u64, u32, i32, vp = C.c_uint64, C.c_uint32, C.c_int, C.c_void_p
        sz = C.c_size_t
        sig = {
            "orc_philox4x32_10": (None, [vp, vp, vp]),
            "orc_sample_ternary": (None, [u64, u32, u32, u32, u32, sz, vp]),
            "orc_sample_cbd": (None, [u64, u32, u32, u32, u32, u32, sz, vp]),
            "orc_sample_uniform": (None, [u64, u32, u32, u32, u32, u32, u64, sz, vp]),
            "orc_mulmod": (u64, [u64, u64, u64]),
            "orc_powmod": (u64, [u64, u64, u64]),
            "orc_is_prime": (i32, [u64]),
            "orc_find_primes": (i32, [u32, u32, i32, vp]),
            "orc_find_psi": (u64, [u64, u32]),
            "orc_negacyclic_schoolbook": (None, [vp, vp, sz, u64, vp]),
            "orc_ntt_definition": (None, [vp, sz, u64, u64, vp]),
            "orc_ntt_forward": (None, [vp, sz, u64, u64]),
            "orc_ntt_inverse": (None, [vp, sz, u64, u64]),
            "orc_ring_mul": (None, [vp, vp, sz, u64, u64, vp]),
            "orc_create": (vp, [vp]),
            "orc_destroy": (None, [vp]),
            "orc_psi": (u64, [vp, u32]),
            "orc_psi_t": (u64, [vp]),
            "orc_lambda_mod_q": (u64, [vp, u32]),
            "orc_q_mod_t": (u64, [vp]),
            "orc_lambda_bits": (u32, [vp]),
            "orc_encode_clamp": (C.c_int64, [vp]),
            "orc_crs": (None, [vp, vp]),
            "orc_keygen_share": (None, [vp, u32, vp, vp, vp, vp]),
            "orc_aggregate_pk": (None, [vp, vp, u32, vp]),
            "orc_encode": (i32, [vp, vp, u64, vp, u32]),
            "orc_encode_coefficients": (i32, [vp, vp, u64, vp, u32]),
            "orc_decode_coefficients": (i32, [vp, vp, u32, u64, vp]),
            "orc_encrypt": (None, [vp, vp, vp, u32, u32, u32, u32, vp]),
            "orc_add": (None, [vp, vp, vp, u32]),
            "orc_partial_decrypt": (None, [vp, vp, vp, u32, u32, u32, u32, vp]),
            "orc_combine": (None, [vp, vp, vp, u32, u32, vp]),
            "orc_decode": (i32, [vp, vp, u32, u64, vp]),
            "orc_decrypt_with_secret": (None, [vp, vp, vp, u32, vp]),
            "orc_receiver_keygen": (None, [vp, u32, vp, vp, vp, vp]),
            "orc_convert_share": (None, [vp, vp, vp, vp, u32, u32, u32, u32, u32, vp]),
            "orc_convert_combine": (None, [vp, vp, vp, u32, u32, vp]),
            "orc_bootstrap_alpha": (None, [vp, u32, u32, vp]),
            "orc_bootstrap_share": (None, [vp, vp, vp, u32, u32, u32, u32, vp]),
            "orc_bootstrap_combine": (None, [vp, vp, vp, u32, u32, u32, u32, vp]),
            "orc_average_update": (None, [vp, u32, vp, C.c_float, u64, vp]),
            "orc_bench_polys": (None, [vp, u32, vp]),
            "orc_ntt_forward_batch": (None, [vp, vp, u32]),
            "orc_ntt_inverse_batch": (None, [vp, vp, u32]),
            "orc_round_group": (i32, [vp, vp, vp, vp, vp, u32, u32, u64, u32, u32, vp]),
        }
        for name, (res, args) in sig.items():
            fn = getattr(_lib, name)
            fn.restype = res
            fn.argtypes = args
    return _lib


def average_update(sum_, K, grad, gamma):
    """Alg. 2 lines 9-10 in float32: sum * (1/K) - gamma * grad."""
    sum_ = np.ascontiguousarray(sum_, dtype=np.float32)
    out = np.zeros_like(sum_)
    g = None if grad is None else np.ascontiguousarray(grad, dtype=np.float32)
    lib().orc_average_update(_p(sum_), K, None if g is None else _p(g), gamma, sum_.size, _p(out))
    return out


def _p(a: np.ndarray):
    return a.ctypes.data_as(C.c_void_p)


def _u64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.uint64)


def _ptr_array(arrays):
    return (C.c_void_p * len(arrays))(*[a.ctypes.data for a in arrays])


# ---- free functions -----------------------------------------------------------------
def philox4x32_10(ctr, key):
    c = np.asarray(ctr, dtype=np.uint32)
    k = np.asarray(key, dtype=np.uint32)
    out = np.zeros(4, dtype=np.uint32)
    lib().orc_philox4x32_10(_p(c), _p(k), _p(out))
    return out


def sample_ternary(seed, domain, party, group, ct, n):
    out = np.zeros(n, dtype=np.int32)
    lib().orc_sample_ternary(seed, domain, party, group, ct, n, _p(out))
    return out


def sample_cbd(seed, domain, party, group, ct, eta, n):
    out = np.zeros(n, dtype=np.int32)
    lib().orc_sample_cbd(seed, domain, party, group, ct, eta, n, _p(out))
    return out


def sample_uniform(seed, domain, limb, party, group, ct, q, n):
    out = np.zeros(n, dtype=np.uint64)
    lib().orc_sample_uniform(seed, domain, limb, party, group, ct, q, n, _p(out))
    return out


def mulmod(a, b, q):
    return int(lib().orc_mulmod(a, b, q))


def powmod(a, e, q):
    return int(lib().orc_powmod(a, e, q))


def is_prime(n):
    return bool(lib().orc_is_prime(n))


def find_primes(bits, log2_n, count):
    out = np.zeros(count, dtype=np.uint64)
    got = lib().orc_find_primes(bits, log2_n, count, _p(out))
    return [int(v) for v in out[:got]]


def find_psi(q, log2_n):
    return int(lib().orc_find_psi(q, log2_n))


def negacyclic_schoolbook(a, b, q):
    a, b = _u64(a), _u64(b)
    out = np.zeros_like(a)
    lib().orc_negacyclic_schoolbook(_p(a), _p(b), a.size, q, _p(out))
    return out


def ntt_definition(x, q, psi):
    x = _u64(x)
    out = np.zeros_like(x)
    lib().orc_ntt_definition(_p(x), x.size, q, psi, _p(out))
    return out


def ntt_forward(x, q, psi):
    x = _u64(x).copy()
    lib().orc_ntt_forward(_p(x), x.size, q, psi)
    return x


def ntt_inverse(x, q, psi):
    x = _u64(x).copy()
    lib().orc_ntt_inverse(_p(x), x.size, q, psi)
    return x


def ring_mul(a, b, q, psi):
    a, b = _u64(a), _u64(b)
    out = np.zeros_like(a)
    lib().orc_ring_mul(_p(a), _p(b), a.size, q, psi, _p(out))
    return out


# ---- scheme -------------------------------------------------------------------------
class Oracle:
    """One parameter set; every method allocates and returns fresh numpy arrays."""

    def __init__(self, log2_n, q, t, cbd_eta=21, frac_bits=0, max_group=1, seed=0):
        q = [int(v) for v in q]
        prm = _Params()
        prm.log2_n, prm.num_limbs = log2_n, len(q)
        for i, v in enumerate(q):
            prm.q[i] = v
        prm.t, prm.cbd_eta, prm.frac_bits = t, cbd_eta, frac_bits
        prm.max_group, prm.seed = max_group, seed
        self._h = lib().orc_create(C.byref(prm))
        if not self._h:
            raise ValueError("oracle rejected the parameters")
        self.log2_n, self.N, self.L, self.q, self.t = log2_n, 1 << log2_n, len(q), q, t
        self.eta, self.frac_bits, self.max_group, self.seed = cbd_eta, frac_bits, max_group, seed
        self.psi = [int(lib().orc_psi(self._h, i)) for i in range(self.L)]
        self.psi_t = int(lib().orc_psi_t(self._h)) if t else 0

    def __del__(self):
        if getattr(self, "_h", None):
            lib().orc_destroy(self._h)
            self._h = None

    def lambda_mod_q(self, limb):
        return int(lib().orc_lambda_mod_q(self._h, limb))

    def q_mod_t(self):
        return int(lib().orc_q_mod_t(self._h))

    def lambda_bits(self):
        return int(lib().orc_lambda_bits(self._h))

    def encode_clamp(self):
        return int(lib().orc_encode_clamp(self._h))

    def crs(self):
        out = np.zeros((self.L, self.N), dtype=np.uint64)
        lib().orc_crs(self._h, _p(out))
        return out

    def keygen_share(self, party):
        sk = np.zeros((self.L, self.N), dtype=np.uint64)
        pk0 = np.zeros((self.L, self.N), dtype=np.uint64)
        s_small = np.zeros(self.N, dtype=np.int32)
        e_small = np.zeros(self.N, dtype=np.int32)
        lib().orc_keygen_share(self._h, party, _p(sk), _p(pk0), _p(s_small), _p(e_small))
        return sk, pk0, s_small, e_small

    def aggregate_pk(self, pk0_shares):
        shares = [_u64(s) for s in pk0_shares]
        pk = np.zeros((2, self.L, self.N), dtype=np.uint64)
        lib().orc_aggregate_pk(self._h, _ptr_array(shares), len(shares), _p(pk))
        return pk

    def num_ct(self, n_values):
        return (n_values + self.N - 1) // self.N

    def encode(self, grad, C_=None):
        grad = np.ascontiguousarray(grad, dtype=np.float32)
        C_ = self.num_ct(grad.size) if C_ is None else C_
        pt = np.zeros((C_, self.N), dtype=np.uint64)
        if lib().orc_encode(self._h, _p(grad), grad.size, _p(pt), C_) != 0:
            raise ValueError("encode: bad sizes")
        return pt

    def encode_coefficients(self, grad, C_=None):
        grad = np.ascontiguousarray(grad, dtype=np.float32)
        C_ = self.num_ct(grad.size) if C_ is None else C_
        pt = np.zeros((C_, self.N), dtype=np.uint64)
        if lib().orc_encode_coefficients(self._h, _p(grad), grad.size, _p(pt), C_) != 0:
            raise ValueError("encode: bad sizes")
        return pt

    def decode_coefficients(self, pt, n_values):
        pt = _u64(pt)
        out = np.zeros(n_values, dtype=np.float32)
        if lib().orc_decode_coefficients(self._h, _p(pt), pt.shape[0], n_values, _p(out)) != 0:
            raise ValueError("decode: bad sizes")
        return out

    def encrypt(self, pk, pt, party, group, ct_base=0):
        pk, pt = _u64(pk), _u64(pt)
        C_ = pt.shape[0]
        ct = np.zeros((C_, 2, self.L, self.N), dtype=np.uint64)
        lib().orc_encrypt(self._h, _p(pk), _p(pt), C_, party, group, ct_base, _p(ct))
        return ct

    def add(self, acc, inp):
        acc = _u64(acc).copy()
        inp = _u64(inp)
        lib().orc_add(self._h, _p(acc), _p(inp), acc.shape[0])
        return acc

    def partial_decrypt(self, sk, ct, party, group, ct_base=0):
        sk, ct = _u64(sk), _u64(ct)
        C_ = ct.shape[0]
        share = np.zeros((C_, self.L, self.N), dtype=np.uint64)
        lib().orc_partial_decrypt(self._h, _p(sk), _p(ct), C_, party, group, ct_base, _p(share))
        return share

    def combine(self, ct, shares):
        ct = _u64(ct)
        shares = [_u64(s) for s in shares]
        C_ = ct.shape[0]
        pt = np.zeros((C_, self.N), dtype=np.uint64)
        lib().orc_combine(self._h, _p(ct), _ptr_array(shares), len(shares), C_, _p(pt))
        return pt

    def decode(self, pt, n_values):
        pt = _u64(pt)
        out = np.zeros(n_values, dtype=np.float32)
        if lib().orc_decode(self._h, _p(pt), pt.shape[0], n_values, _p(out)) != 0:
            raise ValueError("decode: bad sizes")
        return out

    def decrypt_with_secret(self, s, ct):
        s, ct = _u64(s), _u64(ct)
        pt = np.zeros((ct.shape[0], self.N), dtype=np.uint64)
        lib().orc_decrypt_with_secret(self._h, _p(s), _p(ct), ct.shape[0], _p(pt))
        return pt

    # ---- MBFV.Convert (Sec. 4.2 item 3) ----
    def receiver_keygen(self, party):
        sk = np.zeros((self.L, self.N), dtype=np.uint64)
        pk = np.zeros((2, self.L, self.N), dtype=np.uint64)
        s_small = np.zeros(self.N, dtype=np.int32)
        e_small = np.zeros(self.N, dtype=np.int32)
        lib().orc_receiver_keygen(self._h, party, _p(sk), _p(pk), _p(s_small), _p(e_small))
        return sk, pk, s_small, e_small

    def convert_share(self, sk_share, pk_recv, ct, party, receiver, group, ct_base=0):
        sk_share, pk_recv, ct = _u64(sk_share), _u64(pk_recv), _u64(ct)
        C_ = ct.shape[0]
        share = np.zeros((C_, 2, self.L, self.N), dtype=np.uint64)
        lib().orc_convert_share(self._h, _p(sk_share), _p(pk_recv), _p(ct), C_, party, receiver, group,
                                ct_base, _p(share))
        return share

    def convert_combine(self, ct, shares):
        ct = _u64(ct)
        shares = [_u64(s) for s in shares]
        out = np.zeros_like(ct)
        lib().orc_convert_combine(self._h, _p(ct), _ptr_array(shares), len(shares), ct.shape[0], _p(out))
        return out

    # ---- MBFV.Bootstrap (Sec. 4.2 item 4) ----
    def bootstrap_alpha(self, group, ct):
        out = np.zeros((self.L, self.N), dtype=np.uint64)
        lib().orc_bootstrap_alpha(self._h, group, ct, _p(out))
        return out

    def bootstrap_share(self, sk_share, ct, party, group, ct_base=0):
        sk_share, ct = _u64(sk_share), _u64(ct)
        share = np.zeros_like(ct)
        lib().orc_bootstrap_share(self._h, _p(sk_share), _p(ct), ct.shape[0], party, group, ct_base, _p(share))
        return share

    def bootstrap_combine(self, ct, shares, group, ct_base=0):
        ct = _u64(ct)
        shares = [_u64(s) for s in shares]
        out = np.zeros_like(ct)
        lib().orc_bootstrap_combine(self._h, _p(ct), _ptr_array(shares), len(shares), ct.shape[0], group, ct_base,
                                    _p(out))
        return out

    def bench_polys(self, B):
        out = np.zeros((B, self.L, self.N), dtype=np.uint64)
        lib().orc_bench_polys(self._h, B, _p(out))
        return out

    def ntt_forward_batch(self, polys):
        polys = _u64(polys).copy()
        lib().orc_ntt_forward_batch(self._h, _p(polys), polys.shape[0])
        return polys

    def ntt_inverse_batch(self, polys):
        polys = _u64(polys).copy()
        lib().orc_ntt_inverse_batch(self._h, _p(polys), polys.shape[0])
        return polys

    def round_group(self, pk, sks, grads, members, group, ct_begin=0, ct_end=None):
        """Whole round for one group; returns (sum of the members' gradients, threads)."""
        pk = _u64(pk)
        sks = [_u64(s) for s in sks]
        grads = [np.ascontiguousarray(g, dtype=np.float32) for g in grads]
        n_values = grads[0].size
        ct_end = self.num_ct(n_values) if ct_end is None else ct_end
        mem = np.asarray(members, dtype=np.uint32)
        out = np.zeros(n_values, dtype=np.float32)
        thr = lib().orc_round_group(self._h, _p(pk), _ptr_array(sks), _ptr_array(grads), _p(mem),
                                    len(members), group, n_values, ct_begin, ct_end, _p(out))
        return out, thr
