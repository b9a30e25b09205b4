"""Every (arithmetic back-end, ring degree) pair the library instantiates, against the oracle: the four
back-ends are chosen by the largest prime (< 2^30, < 2^44, < 2^55, < 2^61), the kernel shapes by log2 N.  The five
benchmark configurations cover five of these pairs; this sweep covers the rest with small seeded inputs
(two or three ciphertexts, a ragged tail), every intermediate object compared bit for bit."""
import numpy as np
import pytest

from oracle import oracle as O
from paper_2207_04604_amd.synth import toy_config

from gpu_util import Keys, dzeros, make_ctx, make_pair, to_dev, to_eval, to_host
from test_gpu_parity import fixed_point_sum, run_calls_and_compare, run_fused

pytestmark = pytest.mark.gpu


# (log2 N, prime bits, limbs); primes "of b bits" lie just below 2^b: 30 bits is the widest the 32-bit back-end
# takes, 31 to 44 go to the double-precision one, 45 to 55 to the third, 56 to 61 to the fourth.  Small primes come in pairs so that the
# plaintext modulus leaves room for the noise.
SCHEME_SHAPES = [(10, 30, 2), (10, 31, 2), (11, 30, 2), (12, 30, 2), (12, 27, 3), (14, 30, 2), (10, 44, 2), (10, 45, 1), (10, 55, 2), (10, 56, 1), (10, 61, 2), (11, 36, 3), (11, 44, 1), (11, 61, 2),
                 (12, 45, 2), (12, 55, 1), (12, 61, 2), (13, 30, 2), (13, 44, 2), (13, 56, 1), (13, 61, 2), (14, 36, 2),
                 (14, 44, 1), (14, 61, 2), (14, 45, 2), (14, 55, 1), (13, 54, 2)]


@pytest.mark.parametrize("log2n,bits,L", SCHEME_SHAPES)
def test_round_objects_for_every_backend_and_degree(log2n, bits, L):
    N = 1 << log2n
    t = 12289 if log2n <= 11 else 65537
    q = O.find_primes(bits, log2n, L)
    cfg = toy_config(log2n, q, t, parties=3, n_values=N + 37, frac_bits=5)
    o, ctx, perm = make_pair(cfg, max_group=3)
    rng = np.random.default_rng(1000 * log2n + bits)
    grads = {k: rng.normal(0, 6.0, cfg.n_values).astype(np.float32) for k in range(3)}
    keys = Keys(o, ctx, perm, range(3))
    dpk, opk, _ = run_calls_and_compare(cfg, o, ctx, perm, keys, [0, 1, 2], 4, grads, ct_base=9)
    res, _ = run_fused(ctx, o, dpk, keys, [0, 1, 2], 4, grads, cfg.n_values)
    assert np.array_equal(res, fixed_point_sum([grads[k] for k in range(3)], 5, o.encode_clamp()))
    ctx.close()


@pytest.mark.parametrize("log2n,bits,L,batch", [(15, 36, 2, 3), (15, 55, 1, 2), (15, 61, 2, 2), (16, 44, 1, 3), (16, 45, 2, 2),
                                                (16, 56, 1, 9), (10, 61, 1, 5), (12, 55, 3, 2), (14, 30, 1, 2),
                                                (15, 30, 2, 3), (16, 30, 1, 9), (16, 31, 1, 2), (10, 20, 1, 2), (13, 24, 2, 2)])
def test_transforms_for_every_backend_and_degree(log2n, bits, L, batch):
    """Transform-only contexts (t = 0), including the two-kernel path for N > 16384 with batches that do not
    fill a workgroup's share of polynomials."""
    N = 1 << log2n
    q = O.find_primes(bits, log2n, L)
    o = O.Oracle(log2n, q, 0, 21, 0, 1, 77)
    ctx = make_ctx(log2n, q, 0, seed=77)
    perm = ctx.index_map()
    assert sorted(perm.tolist()) == list(range(N))
    polys = o.bench_polys(batch)
    for i in range(L):
        polys[0, i, :4] = [0, 1, q[i] - 1, q[i] - 2]
    d = to_dev(polys.reshape(-1))
    ctx.ntt_forward(d, batch)
    assert np.array_equal(to_host(d, polys.shape), to_eval(o, perm, polys)), "forward transform"
    ctx.ntt_inverse(d, batch)
    assert np.array_equal(to_host(d, polys.shape), polys), "inverse transform"
    ctx.close()


# every (back-end, ring degree) pair once: 30 bits -> 32-bit words, 44 -> doubles, 55 -> lazy 64-bit, 61 -> Harvey
EXTREME_SHAPES = [(log2n, bits) for log2n in range(10, 17) for bits in (30, 44, 55, 61)]


@pytest.mark.parametrize("log2n,bits", EXTREME_SHAPES)
def test_transforms_of_extreme_polynomials(log2n, bits):
    """Inputs that drive the lazily reduced butterflies to the top of their ranges: every coefficient q - 1, a
    single q - 1 at either end, alternating q - 1 and 0, all ones, and q - 1 on a random half.  Forward: coefficient
    form in, compared with the oracle's transform.  Inverse: the same patterns taken as evaluation-form data in the
    library's layout, compared with the oracle's inverse transform of the values put in natural order."""
    N = 1 << log2n
    (q,) = O.find_primes(bits, log2n, 1)
    o = O.Oracle(log2n, [q], 0, 21, 0, 1, 5)
    ctx = make_ctx(log2n, [q], 0, seed=5)
    perm = ctx.index_map()
    rng = np.random.default_rng(log2n * 100 + bits)
    pats = np.zeros((6, 1, N), dtype=np.uint64)
    pats[0] = q - 1
    pats[1, 0, 0] = q - 1
    pats[2, 0, N - 1] = q - 1
    pats[3, 0, ::2] = q - 1
    pats[4] = 1
    pats[5, 0, rng.random(N) < 0.5] = q - 1
    d = to_dev(pats.reshape(-1))
    ctx.ntt_forward(d, 6)
    assert np.array_equal(to_host(d, pats.shape), to_eval(o, perm, pats)), "forward transform"
    d = to_dev(pats.reshape(-1))
    ctx.ntt_inverse(d, 6)
    got = to_host(d, pats.shape)
    for b in range(6):
        natural = np.zeros(N, dtype=np.uint64)
        natural[perm] = pats[b, 0]                 # position p of the layout holds evaluation perm[p]
        assert np.array_equal(got[b, 0], O.ntt_inverse(natural, q, o.psi[0])), f"inverse transform, pattern {b}"
    ctx.close()


def test_arithmetic_policies_hold_their_contracts_on_the_device():
    """tests/arith_device_check.hip: every operation of every arithmetic policy, as compiled for the GPU (the
    inline-assembly side), on inputs at the ends of the documented ranges, against 128-bit integers."""
    import os
    import subprocess
    from paper_2207_04604_amd import build
    exe = build.DEVICE_CHECK_EXE
    if not os.path.exists(exe):
        build.build_device_check()
    run = subprocess.run([exe], capture_output=True, text=True, timeout=300)
    assert run.returncode == 0, run.stdout[-3000:]
    assert "all arithmetic policies hold their contracts on the device" in run.stdout
