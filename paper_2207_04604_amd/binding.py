"""Thin ctypes front-end of the C-ABI HIP library (``include/d2mhe.h``).

Argument marshalling only: every step of the exchange round runs in the library's kernels.
Buffers are device memory owned by the caller (normally ``torch`` CUDA tensors; anything
with ``data_ptr()`` or a raw integer address is accepted).  There is no CPU fallback: if
the shared library has not been built, importing symbols fails loudly.
"""
from __future__ import annotations

import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("D2MHE_LIBRARY", os.path.join(_HERE, "libd2mhe.so"))

OK = 0
ERR_BAD_PARAMS, ERR_NULL, ERR_ALIGN, ERR_RANGE, ERR_WORKSPACE, ERR_HIP, ERR_UNIMPLEMENTED = range(-1, -8, -1)
STATIC_SCRATCH_BYTES = 64 << 20          # D2MHE_STATIC_SCRATCH_BYTES of the header

SYMBOLS = [
    "d2mhe_workspace_bytes", "d2mhe_create", "d2mhe_destroy", "d2mhe_strerror", "d2mhe_last_hip_error",
    "d2mhe_ntt_index_map", "d2mhe_root", "d2mhe_ntt_forward", "d2mhe_ntt_inverse", "d2mhe_bench_polys",
    "d2mhe_keygen_share", "d2mhe_aggregate_pk", "d2mhe_encode", "d2mhe_encrypt", "d2mhe_add",
    "d2mhe_partial_decrypt", "d2mhe_combine", "d2mhe_decode", "d2mhe_round_scratch_bytes",
    "d2mhe_round", "d2mhe_round_group", "d2mhe_round_group_static",
    "d2mhe_receiver_keygen", "d2mhe_convert_share", "d2mhe_convert_combine", "d2mhe_decrypt",
    "d2mhe_round_convert_scratch_bytes", "d2mhe_round_convert",
    "d2mhe_bootstrap_alpha", "d2mhe_bootstrap_share", "d2mhe_bootstrap_combine",
    "d2mhe_average_update", "d2mhe_encode_coefficients", "d2mhe_decode_coefficients",
]


class Params(C.Structure):
    _fields_ = [("log2_n", C.c_uint32), ("num_limbs", C.c_uint32), ("q", C.POINTER(C.c_uint64)),
                ("t", C.c_uint64), ("cbd_eta", C.c_uint32), ("frac_bits", C.c_uint32),
                ("max_group", C.c_uint32), ("seed", C.c_uint64)]


class RoundDesc(C.Structure):
    _fields_ = [("num_groups", C.c_uint32), ("group_offsets", C.POINTER(C.c_uint32)),
                ("members", C.POINTER(C.c_uint32)), ("group_ids", C.POINTER(C.c_uint32)),
                ("pks", C.POINTER(C.c_void_p)), ("num_parties", C.c_uint32),
                ("sk_shares", C.POINTER(C.c_void_p)), ("grads", C.POINTER(C.c_void_p)),
                ("out_sums", C.POINTER(C.c_void_p)), ("n_values", C.c_uint64), ("packing", C.c_uint32),
                ("ct_base", C.c_uint32)]


class ConvertDesc(C.Structure):
    _fields_ = [("recv_offsets", C.POINTER(C.c_uint32)), ("receivers", C.POINTER(C.c_uint32)),
                ("recv_pks", C.POINTER(C.c_void_p)), ("recv_sks", C.POINTER(C.c_void_p)),
                ("out_recv", C.POINTER(C.c_void_p))]


class D2mheError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__(f"{where}: {strerror(status)} ({status})")


_lib = None


def lib():
    """Load the HIP library (no fallback) and declare the C signatures."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()')")
    L = C.CDLL(LIB_PATH)
    vp, u32, u64, sz, i32 = C.c_void_p, C.c_uint32, C.c_uint64, C.c_size_t, C.c_int32
    PP = C.POINTER(Params)
    sig = {
        "d2mhe_workspace_bytes": (sz, [PP]),
        "d2mhe_create": (i32, [PP, vp, sz, vp, C.POINTER(vp)]),
        "d2mhe_destroy": (None, [vp]),
        "d2mhe_strerror": (C.c_char_p, [i32]),
        "d2mhe_last_hip_error": (C.c_int, [vp]),
        "d2mhe_ntt_index_map": (i32, [vp, vp]),
        "d2mhe_root": (u64, [vp, u32]),
        "d2mhe_ntt_forward": (i32, [vp, vp, u32, vp]),
        "d2mhe_ntt_inverse": (i32, [vp, vp, u32, vp]),
        "d2mhe_bench_polys": (i32, [vp, vp, u32, vp]),
        "d2mhe_keygen_share": (i32, [vp, u32, vp, vp, vp]),
        "d2mhe_aggregate_pk": (i32, [vp, vp, u32, vp, vp]),
        "d2mhe_encode": (i32, [vp, vp, u64, vp, u32, vp]),
        "d2mhe_encrypt": (i32, [vp, vp, vp, u32, u32, u32, u32, vp, vp]),
        "d2mhe_add": (i32, [vp, vp, vp, u32, vp]),
        "d2mhe_partial_decrypt": (i32, [vp, vp, vp, u32, u32, u32, u32, vp, vp]),
        "d2mhe_combine": (i32, [vp, vp, vp, u32, u32, vp, vp]),
        "d2mhe_decode": (i32, [vp, vp, u32, u64, vp, vp]),
        "d2mhe_round_scratch_bytes": (sz, [vp, u32, u32, u64]),
        "d2mhe_round": (i32, [vp, C.POINTER(RoundDesc), vp, sz, vp, vp]),
        "d2mhe_round_group": (i32, [vp, vp, vp, vp, vp, u32, u32, u64, vp, vp, sz, vp]),
        "d2mhe_round_group_static": (i32, [vp, vp, vp, vp, vp, u32, u32, u64, vp, vp]),
        "d2mhe_receiver_keygen": (i32, [vp, u32, vp, vp, vp]),
        "d2mhe_convert_share": (i32, [vp, vp, vp, vp, u32, u32, u32, u32, u32, vp, vp]),
        "d2mhe_convert_combine": (i32, [vp, vp, vp, u32, u32, vp, vp]),
        "d2mhe_decrypt": (i32, [vp, vp, vp, u32, vp, vp]),
        "d2mhe_round_convert_scratch_bytes": (sz, [vp, u32, u32, u32, u64]),
        "d2mhe_round_convert": (i32, [vp, C.POINTER(RoundDesc), C.POINTER(ConvertDesc), vp, sz, vp, vp]),
        "d2mhe_bootstrap_alpha": (i32, [vp, u32, u32, u32, vp, vp]),
        "d2mhe_bootstrap_share": (i32, [vp, vp, vp, vp, u32, u32, u32, u32, vp, vp]),
        "d2mhe_bootstrap_combine": (i32, [vp, vp, vp, vp, u32, u32, vp, vp]),
        "d2mhe_average_update": (i32, [vp, u32, vp, C.c_float, u64, vp, vp]),
        "d2mhe_encode_coefficients": (i32, [vp, vp, u64, vp, u32, vp]),
        "d2mhe_decode_coefficients": (i32, [vp, vp, u32, u64, vp, vp]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(L, name)
        fn.restype, fn.argtypes = res, args
    _lib = L
    return L


def strerror(status: int) -> str:
    return lib().d2mhe_strerror(status).decode()


def _ptr(buf):
    """Device address of a tensor / array / raw integer (None -> NULL)."""
    if buf is None:
        return None
    if isinstance(buf, int):
        return buf
    if hasattr(buf, "data_ptr"):
        return buf.data_ptr()
    return buf.ctypes.data


def _ptr_table(bufs):
    return (C.c_void_p * len(bufs))(*[_ptr(b) for b in bufs])


def make_params(log2_n, q, t, cbd_eta=21, frac_bits=0, max_group=1, seed=0):
    """Returns (Params, keep-alive array of the primes)."""
    arr = (C.c_uint64 * len(q))(*[int(v) for v in q])
    p = Params(log2_n, len(q), C.cast(arr, C.POINTER(C.c_uint64)), t, cbd_eta, frac_bits, max_group, seed)
    return p, arr


def average_update(sum_, K, grad, gamma, n, w, stream=None):
    _check(lib().d2mhe_average_update(_ptr(sum_), K, _ptr(grad), gamma, n, _ptr(w), stream), "d2mhe_average_update")


def workspace_bytes(params: Params) -> int:
    return lib().d2mhe_workspace_bytes(C.byref(params))


def _check(status, where):
    if status != OK:
        raise D2mheError(status, where)


class Context:
    """One parameter set bound to a caller-provided device workspace."""

    def __init__(self, log2_n, q, t, cbd_eta=21, frac_bits=0, max_group=1, seed=0, workspace=None,
                 alloc=None, stream=None):
        """`workspace`: a device buffer of at least workspace_bytes(), or `alloc(nbytes)` makes one."""
        self.params, self._q_keep = make_params(log2_n, q, t, cbd_eta, frac_bits, max_group, seed)
        need = workspace_bytes(self.params)
        if need == 0:
            raise D2mheError(ERR_BAD_PARAMS, "d2mhe_workspace_bytes")
        if workspace is None:
            if alloc is None:
                raise ValueError("pass a device workspace or an allocator")
            workspace = alloc(need)
        self.workspace = workspace
        self.workspace_bytes = need
        handle = C.c_void_p()
        _check(lib().d2mhe_create(C.byref(self.params), _ptr(workspace), need, stream, C.byref(handle)), "d2mhe_create")
        self._h = handle
        self.log2_n, self.N, self.L, self.t = log2_n, 1 << log2_n, len(q), t
        self.q = [int(v) for v in q]

    def close(self):
        if getattr(self, "_h", None) and _lib is not None:
            _lib.d2mhe_destroy(self._h)
        self._h = None

    def __del__(self):
        self.close()

    # -- inspection ----------------------------------------------------------------------
    def index_map(self):
        import numpy as np
        perm = np.zeros(self.N, dtype=np.uint32)
        _check(lib().d2mhe_ntt_index_map(self._h, perm.ctypes.data), "d2mhe_ntt_index_map")
        return perm

    def root(self, limb):
        return int(lib().d2mhe_root(self._h, limb))

    # -- transforms -----------------------------------------------------------------------
    def ntt_forward(self, polys, B, stream=None):
        _check(lib().d2mhe_ntt_forward(self._h, _ptr(polys), B, stream), "d2mhe_ntt_forward")

    def ntt_inverse(self, polys, B, stream=None):
        _check(lib().d2mhe_ntt_inverse(self._h, _ptr(polys), B, stream), "d2mhe_ntt_inverse")

    def bench_polys(self, out, B, stream=None):
        _check(lib().d2mhe_bench_polys(self._h, _ptr(out), B, stream), "d2mhe_bench_polys")

    # -- set-up ---------------------------------------------------------------------------
    def keygen_share(self, party, sk_share, pk0_share, stream=None):
        _check(lib().d2mhe_keygen_share(self._h, party, _ptr(sk_share), _ptr(pk0_share), stream), "d2mhe_keygen_share")

    def aggregate_pk(self, pk0_shares, pk, stream=None):
        _check(lib().d2mhe_aggregate_pk(self._h, _ptr_table(pk0_shares), len(pk0_shares), _ptr(pk), stream),
               "d2mhe_aggregate_pk")

    # -- round ----------------------------------------------------------------------------
    def encode(self, grad, n_values, pt, C_, stream=None):
        _check(lib().d2mhe_encode(self._h, _ptr(grad), n_values, _ptr(pt), C_, stream), "d2mhe_encode")

    def encode_coefficients(self, grad, n_values, pt, C_, stream=None):
        _check(lib().d2mhe_encode_coefficients(self._h, _ptr(grad), n_values, _ptr(pt), C_, stream),
               "d2mhe_encode_coefficients")

    def decode_coefficients(self, pt, C_, n_values, out, stream=None):
        _check(lib().d2mhe_decode_coefficients(self._h, _ptr(pt), C_, n_values, _ptr(out), stream),
               "d2mhe_decode_coefficients")

    def encrypt(self, pk, pt, C_, party, group, ct_base, ct, stream=None):
        _check(lib().d2mhe_encrypt(self._h, _ptr(pk), _ptr(pt), C_, party, group, ct_base, _ptr(ct), stream),
               "d2mhe_encrypt")

    def add(self, ct_acc, ct_in, C_, stream=None):
        _check(lib().d2mhe_add(self._h, _ptr(ct_acc), _ptr(ct_in), C_, stream), "d2mhe_add")

    def partial_decrypt(self, sk_share, ct, C_, party, group, ct_base, share, stream=None):
        _check(lib().d2mhe_partial_decrypt(self._h, _ptr(sk_share), _ptr(ct), C_, party, group, ct_base,
                                           _ptr(share), stream), "d2mhe_partial_decrypt")

    def combine(self, ct, shares, C_, pt, stream=None):
        _check(lib().d2mhe_combine(self._h, _ptr(ct), _ptr_table(shares), len(shares), C_, _ptr(pt), stream),
               "d2mhe_combine")

    def decode(self, pt, C_, n_values, out, stream=None):
        _check(lib().d2mhe_decode(self._h, _ptr(pt), C_, n_values, _ptr(out), stream), "d2mhe_decode")

    def round_scratch_bytes(self, num_jobs, num_groups, n_values):
        return lib().d2mhe_round_scratch_bytes(self._h, num_jobs, num_groups, n_values)

    def make_round(self, groups, pks, sk_shares, grads, out_sums, n_values, group_ids=None, ct_base=0,
                   packing=0):
        """Marshal a whole-round description once (host tables); returns an opaque object for round().
        groups: list of member lists; pks/out_sums: one buffer per group; sk_shares/grads: by party id
        (list, or dict for sparse ids)."""
        flat = [int(m) for g in groups for m in g]
        offs = [0]
        for g in groups:
            offs.append(offs[-1] + len(g))
        P = max(flat) + 1 if flat else 0
        get = (lambda tbl, k: tbl.get(k)) if isinstance(sk_shares, dict) else (lambda tbl, k: tbl[k] if k < len(tbl) else None)
        keep = {
            "offs": (C.c_uint32 * len(offs))(*offs),
            "members": (C.c_uint32 * len(flat))(*flat),
            "gids": (C.c_uint32 * len(groups))(*group_ids) if group_ids is not None else None,
            "pks": _ptr_table(pks),
            "sks": (C.c_void_p * P)(*[_ptr(get(sk_shares, k)) for k in range(P)]),
            "grads": (C.c_void_p * P)(*[_ptr(get(grads, k)) for k in range(P)]),
            "outs": _ptr_table(out_sums),
        }
        d = RoundDesc(len(groups), keep["offs"], keep["members"], keep["gids"],
                      C.cast(keep["pks"], C.POINTER(C.c_void_p)), P,
                      C.cast(keep["sks"], C.POINTER(C.c_void_p)), C.cast(keep["grads"], C.POINTER(C.c_void_p)),
                      C.cast(keep["outs"], C.POINTER(C.c_void_p)), n_values, packing, ct_base)
        d._keep = keep
        d.num_jobs = len(flat)
        return d

    def round(self, desc, scratch, scratch_bytes, phase_events=None, stream=None):
        ev = (C.c_void_p * 5)(*phase_events) if phase_events is not None else None
        _check(lib().d2mhe_round(self._h, C.byref(desc), _ptr(scratch), scratch_bytes, ev, stream), "d2mhe_round")

    # ---- MBFV.Convert ----
    def receiver_keygen(self, party, sk, pk, stream=None):
        _check(lib().d2mhe_receiver_keygen(self._h, party, _ptr(sk), _ptr(pk), stream), "d2mhe_receiver_keygen")

    def convert_share(self, sk_share, pk_recv, ct, C_, party, receiver, group, ct_base, share, stream=None):
        _check(lib().d2mhe_convert_share(self._h, _ptr(sk_share), _ptr(pk_recv), _ptr(ct), C_, party, receiver,
                                         group, ct_base, _ptr(share), stream), "d2mhe_convert_share")

    def convert_combine(self, ct, shares, C_, ct_out, stream=None):
        _check(lib().d2mhe_convert_combine(self._h, _ptr(ct), _ptr_table(shares), len(shares), C_, _ptr(ct_out),
                                           stream), "d2mhe_convert_combine")

    def decrypt(self, sk, ct, C_, pt, stream=None):
        _check(lib().d2mhe_decrypt(self._h, _ptr(sk), _ptr(ct), C_, _ptr(pt), stream), "d2mhe_decrypt")

    def round_convert_scratch_bytes(self, num_jobs, num_groups, num_shares, n_values):
        return lib().d2mhe_round_convert_scratch_bytes(self._h, num_jobs, num_groups, num_shares, n_values)

    def make_convert(self, desc, receivers, recv_pks, recv_sks, out_recv):
        """Receivers of a round made by make_round(): receivers = one list of party ids per group;
        recv_pks / recv_sks by party id (list or dict); out_recv: one buffer per (group, receiver)."""
        flat = [int(r) for g in receivers for r in g]
        offs = [0]
        for g in receivers:
            offs.append(offs[-1] + len(g))
        P = desc.num_parties
        get = (lambda tbl, k: tbl.get(k)) if isinstance(recv_pks, dict) else (lambda tbl, k: tbl[k] if k < len(tbl) else None)
        keep = {
            "offs": (C.c_uint32 * len(offs))(*offs),
            "recv": (C.c_uint32 * len(flat))(*flat),
            "pks": (C.c_void_p * P)(*[_ptr(get(recv_pks, k)) for k in range(P)]),
            "sks": (C.c_void_p * P)(*[_ptr(get(recv_sks, k)) for k in range(P)]),
            "outs": _ptr_table(out_recv),
        }
        cd = ConvertDesc(keep["offs"], keep["recv"], C.cast(keep["pks"], C.POINTER(C.c_void_p)),
                         C.cast(keep["sks"], C.POINTER(C.c_void_p)), C.cast(keep["outs"], C.POINTER(C.c_void_p)))
        cd._keep = keep
        groups = [desc._keep["offs"][g + 1] - desc._keep["offs"][g] for g in range(desc.num_groups)]
        cd.num_shares = sum(k * len(r) for k, r in zip(groups, receivers))
        return cd

    def round_convert(self, desc, conv, scratch, scratch_bytes, phase_events=None, stream=None):
        ev = (C.c_void_p * 5)(*phase_events) if phase_events is not None else None
        _check(lib().d2mhe_round_convert(self._h, C.byref(desc), C.byref(conv), _ptr(scratch), scratch_bytes, ev,
                                         stream), "d2mhe_round_convert")

    # ---- MBFV.Bootstrap ----
    def bootstrap_alpha(self, group, ct_base, C_, alpha, stream=None):
        _check(lib().d2mhe_bootstrap_alpha(self._h, group, ct_base, C_, _ptr(alpha), stream), "d2mhe_bootstrap_alpha")

    def bootstrap_share(self, sk_share, ct, alpha, C_, party, group, ct_base, share, stream=None):
        _check(lib().d2mhe_bootstrap_share(self._h, _ptr(sk_share), _ptr(ct), _ptr(alpha), C_, party, group, ct_base,
                                           _ptr(share), stream), "d2mhe_bootstrap_share")

    def bootstrap_combine(self, ct, alpha, shares, C_, ct_out, stream=None):
        _check(lib().d2mhe_bootstrap_combine(self._h, _ptr(ct), _ptr(alpha), _ptr_table(shares), len(shares), C_,
                                             _ptr(ct_out), stream), "d2mhe_bootstrap_combine")

    def round_group(self, pk, sk_shares, grads, members, group, n_values, out_sum, scratch, scratch_bytes,
                    stream=None):
        ids = (C.c_uint32 * len(members))(*[int(m) for m in members])
        _check(lib().d2mhe_round_group(self._h, _ptr(pk), _ptr_table(sk_shares), _ptr_table(grads), ids,
                                       len(members), group, n_values, _ptr(out_sum), _ptr(scratch),
                                       scratch_bytes, stream), "d2mhe_round_group")

    def round_group_static(self, pk, sk_shares, grads, members, group, n_values, out_sum, stream=None):
        """round_group on the library's own scratch array (nothing is allocated)."""
        ids = (C.c_uint32 * len(members))(*[int(m) for m in members])
        _check(lib().d2mhe_round_group_static(self._h, _ptr(pk), _ptr_table(sk_shares), _ptr_table(grads), ids,
                                              len(members), group, n_values, _ptr(out_sum), stream),
               "d2mhe_round_group_static")
