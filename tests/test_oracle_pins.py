"""Pins of the CPU oracle against things other than itself: published known answers,
hand-checked examples, closed forms, invariants from the paper (Sec. 3.2, Sec. 4.2, Eq. (2))
and a structurally different brute-force reference in Python integers (tests/pyref.py)."""
import os
import random

import numpy as np
import pytest

import pyref

GOLD = os.path.join(os.path.dirname(__file__), "golden")
SEED = 0x0123456789ABCDEF


def _rows(name):
    with open(os.path.join(GOLD, name)) as fh:
        return [ln.split() for ln in fh if ln.strip() and not ln.startswith("#")]


# ---------------------------------------------------------------- Philox and samplers
def test_philox_known_answers(orc):
    for row in _rows("philox_kat.txt"):
        w = [int(v, 16) for v in row]
        out = orc.philox4x32_10(w[0:4], w[4:6])
        assert [int(v) for v in out] == w[6:10]
        assert pyref.philox4x32_10(w[0:4], w[4:6]) == w[6:10]


def test_samplers_on_the_all_zero_block(orc):
    # all-zero counter and key -> block 6627e8d5 e169c58d bc57ac4c 9b00dbd8 (published answer);
    # ternary: floor(3w/2^32)-1 = [0,1,1,0]; CBD(21): popcounts of the low 21 bits
    # (0x07e8d5 -> 12, 0x09c58d -> 10, 0x17ac4c -> 11, 0x00dbd8 -> 10) -> [2, 1].
    w = [0x6627e8d5, 0xe169c58d, 0xbc57ac4c, 0x9b00dbd8]
    assert [((x * 3) >> 32) - 1 for x in w] == [0, 1, 1, 0]
    # seed 0, domain 0, everything 0 is exactly that block
    assert list(orc.sample_ternary(0, 0, 0, 0, 0, 4)) == [0, 1, 1, 0]
    assert list(orc.sample_cbd(0, 0, 0, 0, 0, 21, 2)) == [2, 1]
    u = w[0] | (w[1] << 32) | (w[2] << 64) | (w[3] << 96)
    assert int(orc.sample_uniform(0, 0, 0, 0, 0, 0, 1073707009, 1)[0]) == u % 1073707009 == 67482506


def test_sampler_counter_layout_matches_independent_python(orc):
    for (party, group, ct) in [(0, 0, 0), (3, 5, 7), (65535, 65535, 2 ** 32 - 1)]:
        assert list(orc.sample_ternary(SEED, 4, party, group, ct, 37)) == \
            pyref.ternary(SEED, 4, party, group, ct, 37)
        assert list(orc.sample_cbd(SEED, 5, party, group, ct, 21, 37)) == \
            pyref.cbd(SEED, 5, party, group, ct, 21, 37)
        q = 1152921504606584833
        assert [int(v) for v in orc.sample_uniform(SEED, 3, 9, party, group, ct, q, 19)] == \
            pyref.uniform(SEED, 3, 9, party, group, ct, q, 19)


def test_sampler_statistics(orc):
    n = 1 << 16
    s = orc.sample_ternary(SEED, 1, 2, 0, 0, n).astype(np.float64)
    assert set(np.unique(s)) == {-1.0, 0.0, 1.0}
    assert abs(s.mean()) < 0.02 and abs(s.var() - 2.0 / 3.0) < 0.02
    e = orc.sample_cbd(SEED, 2, 2, 0, 0, 21, n).astype(np.float64)
    assert e.min() >= -21 and e.max() <= 21
    assert abs(e.mean()) < 0.06 and abs(e.var() - 10.5) < 0.3    # variance eta/2
    u = orc.sample_uniform(SEED, 3, 0, 0, 0, 0, 1073707009, n).astype(np.float64) / 1073707009
    assert abs(u.mean() - 0.5) < 0.01 and u.max() < 1.0


# ---------------------------------------------------------------- primes and roots
def _python_is_probable_prime(n):
    if n < 2:
        return False
    for p in (2, 3, 5, 7, 11, 13, 17, 19, 23, 29, 31, 37, 41, 43, 47):
        if n % p == 0:
            return n == p
    d, r = n - 1, 0
    while d % 2 == 0:
        d //= 2
        r += 1
    for a in (2, 325, 9375, 28178, 450775, 9780504, 1795265022):   # a second base set
        a %= n
        if a == 0:
            continue
        x = pow(a, d, n)
        if x in (1, n - 1):
            continue
        for _ in range(r - 1):
            x = x * x % n
            if x == n - 1:
                break
        else:
            return False
    return True


def test_stored_expected_values_are_reproduced_by_their_generator():
    """tests/golden/params.txt and toy_round.txt are what tests/golden/regenerate.py writes: plain Python integers
    and the brute-force reference, nothing of the oracle."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(GOLD, "regenerate.py")], capture_output=True, text=True)
    assert r.returncode == 0, r.stdout + r.stderr


def test_prime_search_reproduces_the_pinned_parameter_sets(orc):
    rows = _rows("params.txt")
    sets = {}
    for r in rows:
        if r[0] in ("C1", "C2", "C3", "C4", "C5"):
            sets.setdefault((r[0], int(r[1]), int(r[2])), []).append([int(v) for v in r[3:]])
    counts = {"C1": 1, "C2": 3, "C3": 4, "C4": 8, "C5": 16}
    for (name, bits, log2n), entries in sets.items():
        found = orc.find_primes(bits, log2n, counts[name])
        assert len(found) == counts[name]
        two_n = 2 << log2n
        for q in found:
            assert q % two_n == 1 and _python_is_probable_prime(q) and q < (1 << bits)
        # nothing skipped: every candidate above the smallest found prime is either listed or composite
        k_last = ((1 << bits) + 1 - found[-1]) // two_n
        listed = set(found)
        for k in range(1, k_last + 1):
            cand = (1 << bits) - k * two_n + 1
            assert (cand in listed) == _python_is_probable_prime(cand)
        for (q, k, x, psi) in entries:
            assert q in found and q == (1 << bits) - k * two_n + 1
            assert orc.find_psi(q, log2n) == psi == pow(x, (q - 1) // two_n, q)
            assert pow(psi, 1 << log2n, q) == q - 1
            for y in range(2, x):       # x is the smallest generator candidate that works
                assert pow(pow(y, (q - 1) // two_n, q), 1 << log2n, q) != q - 1
    k5 = [int(v) for r in rows if r[0] == "K5" for v in r[1:]]
    assert orc.find_primes(60, 16, 16) == [(1 << 60) - k * (1 << 17) + 1 for k in k5]
    for r in rows:
        if r[0] == "T":
            log2n = {"C1": 10, "C2": 12, "C3": 13, "C4": 14}[r[1]]
            assert orc.find_psi(int(r[2]), log2n) == int(r[4]) == pow(int(r[3]), (int(r[2]) - 1) >> (log2n + 1), int(r[2]))


def test_is_prime_small_and_carmichael(orc):
    sieve = [True] * 2000
    sieve[0] = sieve[1] = False
    for i in range(2, 2000):
        if sieve[i]:
            for j in range(i * i, 2000, i):
                sieve[j] = False
    for i in range(2000):
        assert orc.is_prime(i) == sieve[i]
    for c in (561, 1105, 1729, 2465, 3215031751, 3825123056546413051, (1 << 61) - 1 - 2):
        assert orc.is_prime(c) == _python_is_probable_prime(c)
    assert orc.is_prime((1 << 61) - 1)


def test_context_constants_match_pinned_values(orc):
    from paper_2207_04604_amd.synth import CONFIGS
    rows = {r[1]: (int(r[2]), int(r[3])) for r in _rows("params.txt") if r[0] == "M"}
    for name in ("C1", "C2", "C3", "C4"):
        cfg = CONFIGS[name]
        o = orc.Oracle(cfg.log2_n, cfg.q, cfg.t, cfg.eta, cfg.frac_bits, cfg.max_group, cfg.seed)
        Q = 1
        for q in cfg.q:
            Q *= q
        assert o.q_mod_t() == Q % cfg.t == rows[name][0]
        assert o.lambda_bits() == (Q // cfg.t).bit_length() == rows[name][1]
        for i, q in enumerate(cfg.q):
            assert o.lambda_mod_q(i) == (Q // cfg.t) % q


# ---------------------------------------------------------------- transforms and ring products
def test_hand_checked_transform_example(orc):
    g = {r[0]: [int(v) for v in r[1:]] for r in _rows("ntt_n4_q17.txt")}
    q, psi = 17, 9
    assert list(orc.ntt_forward(g["x"], q, psi)) == g["xhat"]
    assert list(orc.ntt_definition(g["x"], q, psi)) == g["xhat"]
    assert list(orc.ntt_forward(g["y"], q, psi)) == g["yhat"]
    assert [a * b % q for a, b in zip(g["xhat"], g["yhat"])] == g["had"]
    assert list(orc.ntt_inverse(g["had"], q, psi)) == g["prod"]
    assert list(orc.negacyclic_schoolbook(g["x"], g["y"], q)) == g["prod"]
    assert list(orc.ring_mul(g["x"], g["y"], q, psi)) == g["prod"]
    assert pyref.negacyclic(g["x"], g["y"], q) == g["prod"]


def _all_config_primes():
    from paper_2207_04604_amd.synth import CONFIGS
    out = []
    for cfg in CONFIGS.values():
        out += [(q, cfg.log2_n) for q in cfg.q]
        if cfg.t:
            out.append((cfg.t, cfg.log2_n))
    return out


def test_fast_transform_equals_definition_and_python_pow(orc):
    rnd = random.Random(1)
    for (q, log2n) in _all_config_primes():
        psi_full = orc.find_psi(q, log2n)
        for small in (2, 8, 64):
            psi = pow(psi_full, (1 << log2n) // small, q)     # a primitive 2*small-th root
            assert pow(psi, small, q) == q - 1
            x = [rnd.randrange(q) for _ in range(small)]
            fast = [int(v) for v in orc.ntt_forward(x, q, psi)]
            assert fast == [int(v) for v in orc.ntt_definition(x, q, psi)]
            if small <= 8:
                assert fast == [sum(x[n] * pow(psi, (2 * j + 1) * n, q) for n in range(small)) % q
                                for j in range(small)]
            assert [int(v) for v in orc.ntt_inverse(fast, q, psi)] == x


def test_ring_product_equals_schoolbook_for_every_prime(orc):
    rnd = random.Random(2)
    for (q, log2n) in _all_config_primes():
        psi_full = orc.find_psi(q, log2n)
        for small in (4, 32, 64):
            psi = pow(psi_full, (1 << log2n) // small, q)
            a = [rnd.randrange(q) for _ in range(small)]
            b = [rnd.randrange(q) for _ in range(small)]
            ref = pyref.negacyclic(a, b, q)
            assert [int(v) for v in orc.ring_mul(a, b, q, psi)] == ref
            assert [int(v) for v in orc.negacyclic_schoolbook(a, b, q)] == ref


def test_ring_product_spot_check_n1024(orc):
    q = 1073707009
    psi = orc.find_psi(q, 10)
    rng = np.random.default_rng(3)
    a = rng.integers(0, q, 1024, dtype=np.uint64)
    b = rng.integers(0, q, 1024, dtype=np.uint64)
    assert np.array_equal(orc.ring_mul(a, b, q, psi), orc.negacyclic_schoolbook(a, b, q))
    # X^(N-1) * X = X^N = -1
    xa = np.zeros(1024, dtype=np.uint64); xa[1023] = 1
    xb = np.zeros(1024, dtype=np.uint64); xb[1] = 1
    prod_ = orc.ring_mul(xa, xb, q, psi)
    assert int(prod_[0]) == q - 1 and not prod_[1:].any()


def test_transform_roundtrip_and_linearity_large(orc):
    from paper_2207_04604_amd.synth import CONFIGS
    cfg = CONFIGS["C5"]
    q = cfg.q[-1]
    psi = orc.find_psi(q, 16)
    rng = np.random.default_rng(4)
    a = rng.integers(0, q, 65536, dtype=np.uint64)
    b = rng.integers(0, q, 65536, dtype=np.uint64)
    fa, fb = orc.ntt_forward(a, q, psi), orc.ntt_forward(b, q, psi)
    assert np.array_equal(orc.ntt_inverse(fa, q, psi), a)
    s = ((a.astype(object) + b.astype(object)) % q).astype(np.uint64)
    fs = ((fa.astype(object) + fb.astype(object)) % q).astype(np.uint64)
    assert np.array_equal(orc.ntt_forward(s, q, psi), fs)
    # a delta at position 1 transforms to psi^(2j+1)
    d = np.zeros(65536, dtype=np.uint64); d[1] = 1
    fd = orc.ntt_forward(d, q, psi)
    for j in (0, 1, 2, 12345, 65535):
        assert int(fd[j]) == pow(psi, 2 * j + 1, q)


def test_batched_transforms_and_benchmark_polynomials(orc):
    """The drivers of the transform micro-benchmark: polynomial (b, i) of a batch [B][L][N] is transformed
    with limb i's modulus and root (against the O(N^2) definition and Python's pow), the inverse batch
    undoes it, and the benchmark polynomials are Philox domain 8 with the batch index in the ciphertext
    word and the limb in the tag (against the independent Python generator)."""
    log2n, L, Bn = 5, 2, 3
    n = 1 << log2n
    qs = orc.find_primes(60, log2n, 1) + orc.find_primes(36, log2n, 1)       # two very different limbs
    o = orc.Oracle(log2n, qs, 0, 21, 0, 1, SEED)
    polys = o.bench_polys(Bn)
    assert polys.shape == (Bn, L, n)
    for b in range(Bn):
        for i in range(L):
            assert [int(v) for v in polys[b, i]] == pyref.uniform(SEED, 8, i, 0, 0, b, qs[i], n), (b, i)
    assert len({tuple(polys[b, i]) for b in range(Bn) for i in range(L)}) == Bn * L
    fwd = o.ntt_forward_batch(polys)
    assert fwd.shape == polys.shape and not np.array_equal(fwd, polys)
    for b in range(Bn):
        for i in range(L):
            psi = orc.find_psi(qs[i], log2n)
            assert np.array_equal(fwd[b, i], orc.ntt_definition(polys[b, i], qs[i], psi)), (b, i)
            for j in (0, 1, n - 1):
                assert int(fwd[b, i, j]) == sum(int(polys[b, i, k]) * pow(psi, (2 * j + 1) * k, qs[i])
                                                for k in range(n)) % qs[i]
    assert np.array_equal(o.ntt_inverse_batch(fwd), polys)
    # an inverse from data the forward batch has not made: delta_0 -> all ones, so ones -> delta_0
    ones = np.ones((Bn, L, n), dtype=np.uint64)
    back = o.ntt_inverse_batch(ones)
    assert np.all(back[:, :, 0] == 1) and not back[:, :, 1:].any()


# ---------------------------------------------------------------- scheme vs brute force
def _toy(orc, log2n, bits, L, t, K, f, seed=SEED):
    qs = orc.find_primes(bits, log2n, L)
    o = orc.Oracle(log2n, qs, t, 21, f, K, seed)
    ref = pyref.PyBFV(1 << log2n, qs, t, 21, f, K, seed, orc.find_psi(t, log2n))
    return o, ref, qs


def _residues(poly, qs):
    return np.array([[v % q for v in poly] for q in qs], dtype=np.uint64)


@pytest.mark.parametrize("log2n,bits,L,t,K", [(3, 30, 2, 17, 3), (4, 36, 3, 97, 4), (5, 54, 2, 193, 2),
                                             (4, 60, 4, 65537, 5), (3, 30, 1, 17, 1)])
def test_whole_round_equals_bruteforce_big_integer_bfv(orc, log2n, bits, L, t, K):
    f = 3
    o, ref, qs = _toy(orc, log2n, bits, L, t, K, f)
    n = 1 << log2n
    rng = np.random.default_rng(log2n * 100 + L)
    group = 2
    # keys
    keys = [ref.keygen(k) for k in range(K)]
    p0 = ref.aggregate_pk([k[2] for k in keys])
    okeys = [o.keygen_share(k) for k in range(K)]
    for k in range(K):
        assert list(okeys[k][2]) == keys[k][0] and list(okeys[k][3]) == keys[k][1]
        assert np.array_equal(okeys[k][0], _residues(keys[k][0], qs))
        assert np.array_equal(okeys[k][1], _residues(keys[k][2], qs))
    opk = o.aggregate_pk([k[1] for k in okeys])
    assert np.array_equal(opk[0], _residues(p0, qs)) and np.array_equal(opk[1], _residues(ref.p1, qs))
    assert np.array_equal(o.crs(), _residues(ref.p1, qs))
    # gradients -> plaintexts
    bound = o.encode_clamp()
    grads = [(rng.normal(0, bound / (1 << f) / 2.5 / max(1, K), n)).astype(np.float32) for _ in range(K)]
    fixed = [ref.fixed([float(v) for v in g]) for g in grads]
    ms = [ref.encode_slots([v % t for v in fx]) for fx in fixed]
    opts = [o.encode(g) for g in grads]
    for k in range(K):
        assert [int(v) for v in opts[k][0]] == ms[k]
    # encrypt, aggregate
    cts = [ref.encrypt(p0, ms[k], k, group, 5)[0] for k in range(K)]
    octs = [o.encrypt(opk, opts[k], k, group, ct_base=5) for k in range(K)]
    for k in range(K):
        assert np.array_equal(octs[k][0, 0], _residues(cts[k][0], qs))
        assert np.array_equal(octs[k][0, 1], _residues(cts[k][1], qs))
    agg, oagg = cts[0], octs[0]
    for k in range(1, K):
        agg = ref.add(agg, cts[k])
        oagg = o.add(oagg, octs[k])
    assert np.array_equal(oagg[0, 0], _residues(agg[0], qs)) and np.array_equal(oagg[0, 1], _residues(agg[1], qs))
    # shares, combine, decode
    shares = [ref.share(keys[k][0], agg, k, group, 5)[0] for k in range(K)]
    oshares = [o.partial_decrypt(okeys[k][0], oagg, k, group, ct_base=5) for k in range(K)]
    for k in range(K):
        assert np.array_equal(oshares[k][0], _residues(shares[k], qs))
    m_out = ref.combine(agg, shares)
    opt_out = o.combine(oagg, oshares)
    assert [int(v) for v in opt_out[0]] == m_out
    expect_sum = [sum(fx[j] for fx in fixed) for j in range(n)]
    assert m_out == ref.encode_slots([v % t for v in expect_sum])     # homomorphic sum (Alg. 2, line 6)
    assert ref.decode_slots(m_out) == expect_sum
    dec = o.decode(opt_out, n)
    assert [float(v) for v in dec] == [v / (1 << f) for v in expect_sum]
    # collective decryption == single-key decryption with s = sum s_k  (Eq. (2))
    s_sum = [sum(k[0][j] for k in keys) for j in range(n)]
    assert ref.decrypt(s_sum, agg) == m_out
    assert [int(v) for v in o.decrypt_with_secret(_residues(s_sum, qs), oagg)[0]] == m_out
    # the timing driver walks the same steps
    out, _ = o.round_group(opk, [k[0] for k in okeys], grads, list(range(K)), group)
    # (round_group uses ciphertext index 0.., a different noise stream, same plaintext result)
    assert [float(v) for v in out] == [v / (1 << f) for v in expect_sum]


@pytest.mark.parametrize("log2n,bits,L,t,K,recv", [(3, 30, 2, 17, 3, 1), (4, 36, 3, 97, 4, 0), (4, 60, 4, 65537, 2, 7),
                                                  (3, 30, 1, 17, 1, 0)])
def test_convert_equals_bruteforce_big_integer_bfv(orc, log2n, bits, L, t, K, recv):
    """MBFV.Convert (Sec. 4.2 item 3): receiver key, every share (Eq. (1)), the converted ciphertext
    and its single-key decryption (Eq. (2)) against the big-integer reference; `recv` = 7 is a
    receiver outside the group (the formulas do not need it to be a member)."""
    f = 3
    o, ref, qs = _toy(orc, log2n, bits, L, t, K, f)
    n = 1 << log2n
    rng = np.random.default_rng(log2n * 1000 + L)
    group, cti = 3, 9
    keys = [ref.keygen(k) for k in range(K)]
    p0 = ref.aggregate_pk([k[2] for k in keys])
    okeys = [o.keygen_share(k) for k in range(K)]
    opk = o.aggregate_pk([k[1] for k in okeys])
    # the receiver's own pair
    rs, re_, rpk = ref.receiver_keygen(recv)
    osk, orpk, os_small, oe_small = o.receiver_keygen(recv)
    assert list(os_small) == rs and list(oe_small) == re_
    assert np.array_equal(osk, _residues(rs, qs))
    assert np.array_equal(orpk[0], _residues(rpk[0], qs)) and np.array_equal(orpk[1], _residues(rpk[1], qs))
    # p0_i + p1_i sk_i = -e  (Sec. 3.2 item 2)
    lhs = [(a + b) % ref.Q for a, b in zip(rpk[0], pyref.negacyclic(rpk[1], rs, ref.Q))]
    assert lhs == [(-v) % ref.Q for v in re_]
    # aggregate of K fresh ciphertexts
    ms = [[int(v) for v in rng.integers(0, t, n)] for _ in range(K)]
    cts = [ref.encrypt(p0, ms[k], k, group, cti)[0] for k in range(K)]
    octs = [o.encrypt(opk, np.array([ms[k]], dtype=np.uint64), k, group, ct_base=cti) for k in range(K)]
    agg, oagg = cts[0], octs[0]
    for k in range(1, K):
        agg = ref.add(agg, cts[k])
        oagg = o.add(oagg, octs[k])
    # shares towards the receiver
    shares = [ref.convert_share(keys[k][0], rpk, agg, k, recv, group, cti)[0] for k in range(K)]
    oshares = [o.convert_share(okeys[k][0], orpk, oagg, k, recv, group, ct_base=cti) for k in range(K)]
    for k in range(K):
        assert np.array_equal(oshares[k][0, 0], _residues(shares[k][0], qs))
        assert np.array_equal(oshares[k][0, 1], _residues(shares[k][1], qs))
    new_ct = ref.convert_combine(agg, shares)
    onew = o.convert_combine(oagg, oshares)
    assert np.array_equal(onew[0, 0], _residues(new_ct[0], qs)) and np.array_equal(onew[0, 1], _residues(new_ct[1], qs))
    # the receiver alone decrypts the sum (Eq. (2)); the collective decryption gives the same
    expect = [sum(m[j] for m in ms) % t for j in range(n)]
    assert ref.decrypt(rs, new_ct) == expect
    assert [int(v) for v in o.decrypt_with_secret(osk, onew)[0]] == expect
    plain_shares = [o.partial_decrypt(okeys[k][0], oagg, k, group, ct_base=cti) for k in range(K)]
    assert [int(v) for v in o.combine(oagg, plain_shares)[0]] == expect
    # a share towards another receiver uses other randomness
    other = o.convert_share(okeys[0][0], orpk, oagg, 0, recv + 1, group, ct_base=cti)
    assert not np.array_equal(other, oshares[0])


def test_convert_noise_identity(orc):
    """Eq. (2) expanded: c0' + sk_i c1' - Lambda m = e_ct + e0 + sk_i e1 - mu e_cl exactly, with
    e_ct the noise of the input ciphertext, e_d = sum e_{d,k}, mu = sum mu_k and e_cl the error of
    the receiver's public key (p0_i = -(sk_i p1_i + e_cl)); and it stays below Q/(2t)."""
    o, ref, qs = _toy(orc, 5, 36, 2, 193, 3, 2)
    n, K, recv, group, cti = 32, 3, 2, 1, 4
    keys = [ref.keygen(k) for k in range(K)]
    p0 = ref.aggregate_pk([k[2] for k in keys])
    s = [sum(k[0][j] for k in keys) for j in range(n)]
    rs, e_cl, rpk = ref.receiver_keygen(recv)
    m = [(11 * j + 3) % 193 for j in range(n)]
    ct = ref.encrypt(p0, m, 1, group, cti)[0]
    e_ct = ref.noise(s, ct, m)
    parts = [ref.convert_share(keys[k][0], rpk, ct, k, recv, group, cti) for k in range(K)]
    new_ct = ref.convert_combine(ct, [p[0] for p in parts])
    mu = [sum(p[1][0][j] for p in parts) for j in range(n)]
    e0 = [sum(p[1][1][j] for p in parts) for j in range(n)]
    e1 = [sum(p[1][2][j] for p in parts) for j in range(n)]
    centred = lambda poly: [v - ref.Q if v > ref.Q // 2 else v for v in poly]
    lift = lambda poly: [v % ref.Q for v in poly]
    sk_e1 = centred(pyref.negacyclic(lift(rs), lift(e1), ref.Q))
    mu_ecl = centred(pyref.negacyclic(lift(mu), lift(e_cl), ref.Q))
    noise = ref.noise(rs, new_ct, m)
    assert noise == [e_ct[k] + e0[k] + sk_e1[k] - mu_ecl[k] for k in range(n)]
    assert max(abs(v) for v in noise) < ref.Q // (2 * 193)
    assert ref.decrypt(rs, new_ct) == m


@pytest.mark.parametrize("log2n,bits,L,t,K", [(3, 30, 2, 17, 3), (4, 36, 3, 97, 4), (4, 60, 4, 65537, 2), (3, 30, 1, 17, 1)])
def test_bootstrap_equals_bruteforce_big_integer_bfv(orc, log2n, bits, L, t, K):
    """MBFV.Bootstrap (Sec. 4.2 item 4): alpha, every share (Eq. (3)) and the refreshed ciphertext
    against the big-integer reference; the refreshed ciphertext decrypts to the same plaintext."""
    o, ref, qs = _toy(orc, log2n, bits, L, t, K, 3)
    n = 1 << log2n
    rng = np.random.default_rng(log2n * 77 + L)
    group, cti = 6, 11
    keys = [ref.keygen(k) for k in range(K)]
    p0 = ref.aggregate_pk([k[2] for k in keys])
    okeys = [o.keygen_share(k) for k in range(K)]
    opk = o.aggregate_pk([k[1] for k in okeys])
    ms = [[int(v) for v in rng.integers(0, t, n)] for _ in range(K)]
    cts = [ref.encrypt(p0, ms[k], k, group, cti)[0] for k in range(K)]
    octs = [o.encrypt(opk, np.array([ms[k]], dtype=np.uint64), k, group, ct_base=cti) for k in range(K)]
    agg, oagg = cts[0], octs[0]
    for k in range(1, K):
        agg = ref.add(agg, cts[k])
        oagg = o.add(oagg, octs[k])
    assert np.array_equal(o.bootstrap_alpha(group, cti), _residues(ref.bootstrap_alpha(group, cti), qs))
    shares = [ref.bootstrap_share(keys[k][0], agg, k, group, cti)[0] for k in range(K)]
    oshares = [o.bootstrap_share(okeys[k][0], oagg, k, group, ct_base=cti) for k in range(K)]
    for k in range(K):
        assert np.array_equal(oshares[k][0, 0], _residues(shares[k][0], qs))
        assert np.array_equal(oshares[k][0, 1], _residues(shares[k][1], qs))
    new_ct, _ = ref.bootstrap_combine(agg, shares, group, cti)
    onew = o.bootstrap_combine(oagg, oshares, group, ct_base=cti)
    assert np.array_equal(onew[0, 0], _residues(new_ct[0], qs)) and np.array_equal(onew[0, 1], _residues(new_ct[1], qs))
    expect = [sum(m[j] for m in ms) % t for j in range(n)]
    s_sum = [sum(k[0][j] for k in keys) for j in range(n)]
    assert ref.decrypt(s_sum, new_ct) == expect
    assert [int(v) for v in o.decrypt_with_secret(_residues(s_sum, qs), onew)[0]] == expect
    # the refreshed ciphertext goes through the collective decryption like any other
    plain_shares = [o.partial_decrypt(okeys[k][0], onew, k, group, ct_base=cti) for k in range(K)]
    assert [int(v) for v in o.combine(onew, plain_shares)[0]] == expect


def test_bootstrap_noise_is_reset(orc):
    """Eq. (3) expanded: with M = sum M_k as an integer polynomial and x = (m - M) mod t,
    c0' + s c1' - Lambda m = e1 + j (Q mod t), j = (m - M - x) / t coefficient-wise: the noise of
    the input ciphertext is gone, only e1 = sum e1_k and the wrap term remain."""
    o, ref, qs = _toy(orc, 5, 36, 2, 193, 3, 2)
    n, K, group, cti = 32, 3, 2, 5
    t = 193
    keys = [ref.keygen(k) for k in range(K)]
    p0 = ref.aggregate_pk([k[2] for k in keys])
    s = [sum(k[0][j] for k in keys) for j in range(n)]
    m = [(5 * j + 1) % t for j in range(n)]
    ct = ref.encrypt(p0, m, 0, group, cti)[0]
    for _ in range(3):                       # add the ciphertext to itself: more input noise
        ct = ref.add(ct, ref.encrypt(p0, [0] * n, 1, group, cti)[0])
    e_in = ref.noise(s, ct, m)
    parts = [ref.bootstrap_share(keys[k][0], ct, k, group, cti) for k in range(K)]
    new_ct, x = ref.bootstrap_combine(ct, [p[0] for p in parts], group, cti)
    M = [sum(p[1][0][j] for p in parts) for j in range(n)]
    e1 = [sum(p[1][2][j] for p in parts) for j in range(n)]
    assert x == [(m[j] - M[j]) % t for j in range(n)]
    jwrap = [(m[j] - M[j] - x[j]) // t for j in range(n)]
    assert all((m[j] - M[j] - x[j]) % t == 0 for j in range(n))
    r_t = ref.Q % t
    noise = ref.noise(s, new_ct, m)
    assert noise == [e1[j] + jwrap[j] * r_t for j in range(n)]
    assert max(abs(v) for v in e_in) > max(abs(v) for v in e1)          # the input was noisier
    assert ref.decrypt(s, new_ct) == m


def test_average_update_is_ieee_float32(orc):
    """Alg. 2 lines 9-10: against numpy's float32 arithmetic, plus closed forms."""
    rng = np.random.default_rng(9)
    s = rng.normal(0, 5, 1000).astype(np.float32)
    g = rng.normal(0, 1, 1000).astype(np.float32)
    for K, gamma in ((1, 0.0), (3, 0.1), (5, 0.01), (7, 1.5)):
        inv = np.float32(1.0) / np.float32(K)
        expect = (s * inv).astype(np.float32) - (np.float32(gamma) * g).astype(np.float32)
        assert np.array_equal(orc.average_update(s, K, g, gamma), expect.astype(np.float32))
    assert np.array_equal(orc.average_update(s, 1, None, 0.0), s)
    three = np.array([3.0], dtype=np.float32)
    assert orc.average_update(three, 3, None, 0.0)[0] == np.float32(3.0) * (np.float32(1.0) / np.float32(3.0))


def test_noise_budget_over_many_additions(orc):
    """Homomorphic additions without a refresh (discussion in Sec. 4.3): the noise of a sum of T
    fresh ciphertexts stays below T times the bound of one and, together with the wrap term of
    the plaintext sum (T times Q mod t at most), below Q/(2t); it decrypts.  (With the 30-bit
    modulus of the smallest configuration the wrap term alone allows only a handful of additions,
    which is why its encoding clamps to a sum of K_max values.)"""
    q = orc.find_primes(54, 10, 1)
    t, K, n = 65537, 4, 1024
    o = orc.Oracle(10, q, t, 21, 8, K, SEED)
    keys = [o.keygen_share(k) for k in range(K)]
    pk = o.aggregate_pk([k[1] for k in keys])
    s = np.zeros((1, n), dtype=np.uint64)
    for k in keys:
        s = (s + k[0]) % np.uint64(q[0])
    rng = np.random.default_rng(3)
    T = 40
    acc, msum, worst_one = None, np.zeros(n, dtype=np.int64), 0
    lam = o.lambda_mod_q(0)

    def noise(ct, m):
        y = (orc.ring_mul(ct[0, 1, 0], s[0], q[0], o.psi[0]).astype(object) + ct[0, 0, 0].astype(object)
             - lam * (m % t).astype(object)) % q[0]
        y = np.array([int(v) - q[0] if int(v) > q[0] // 2 else int(v) for v in y])
        # wraps of the plaintext sum add multiples of Q mod t (reading R11): remove them
        r_t = o.q_mod_t()
        return np.array([min((abs(v + w * r_t) for w in range(0, T + 1)), default=0) for v in y])

    for i in range(T):
        m = rng.integers(0, t, n)
        ct = o.encrypt(pk, m.astype(np.uint64)[None, :], i % K, 0, ct_base=i)
        worst_one = max(worst_one, int(noise(ct, m).max()))
        acc = ct if acc is None else o.add(acc, ct)
        msum += m
    total = int(noise(acc, msum).max())
    assert total <= T * worst_one
    assert total + T * o.q_mod_t() < q[0] // (2 * t)
    assert np.array_equal(o.decrypt_with_secret(s, acc)[0], (msum % t).astype(np.uint64))


def test_noise_identity_and_margin(orc):
    """c0 + c1 s - Lambda m = -mu e_pk + e0 + e1 s exactly (Sec. 3.2 item 3 expanded), and it
    stays below Q/(2t) minus the wrap term (correctness condition under Eq. (2))."""
    o, ref, qs = _toy(orc, 5, 36, 2, 193, 3, 2)
    n, K = 32, 3
    keys = [ref.keygen(k) for k in range(K)]
    p0 = ref.aggregate_pk([k[2] for k in keys])
    s = [sum(k[0][j] for k in keys) for j in range(n)]
    e_pk = [sum(k[1][j] for k in keys) for j in range(n)]
    # pk identity: p0 + p1 s = -e_pk
    lhs = [(a + b) % ref.Q for a, b in zip(p0, pyref.negacyclic(ref.p1, s, ref.Q))]
    assert lhs == [(-v) % ref.Q for v in e_pk]
    assert max(abs(v) for v in e_pk) <= 21 * K
    m = [(7 * j) % 193 for j in range(n)]
    (c0, c1), (u, e0, e1) = ref.encrypt(p0, m, 1, 0, 0)
    noise = ref.noise(s, (c0, c1), m)
    centred = lambda poly: [v - ref.Q if v > ref.Q // 2 else v for v in poly]
    ue = centred(pyref.negacyclic(u, [v % ref.Q for v in e_pk], ref.Q))
    e1s = centred(pyref.negacyclic([v % ref.Q for v in e1], [v % ref.Q for v in s], ref.Q))
    assert noise == [-ue[k] + e0[k] + e1s[k] for k in range(n)]
    assert max(abs(v) for v in noise) < ref.Q // (2 * 193)
    # the oracle's ciphertext is the same one
    opk = o.aggregate_pk([o.keygen_share(k)[1] for k in range(K)])
    oct_ = o.encrypt(opk, np.array([m], dtype=np.uint64), 1, 0, 0)
    assert np.array_equal(oct_[0, 0], _residues(c0, qs))


def test_single_key_roundtrip_K1(orc):
    o, ref, qs = _toy(orc, 6, 30, 1, 257, 1, 0)
    sk, pk0, _, _ = o.keygen_share(9)
    pk = o.aggregate_pk([pk0])
    rng = np.random.default_rng(5)
    m = rng.integers(0, 257, (3, 64), dtype=np.uint64)
    ct = o.encrypt(pk, m, 9, 0, 0)
    assert np.array_equal(o.decrypt_with_secret(sk, ct), m)
    share = o.partial_decrypt(sk, ct, 9, 0, 0)
    assert np.array_equal(o.combine(ct, [share]), m)


def test_scale_round_equals_exact_rational_rounding_up_to_8_limbs(orc):
    from fractions import Fraction
    from math import floor
    rnd = random.Random(6)
    for L in (1, 2, 5, 8):
        qs = orc.find_primes(54, 3, L)
        o = orc.Oracle(3, qs, 65537 if L > 1 else 17, 21, 0, 1, 1)
        t = o.t
        Q = 1
        for q in qs:
            Q *= q
        ys = [rnd.randrange(Q) for _ in range(8)]
        ys[0], ys[1], ys[2] = 0, Q - 1, Q // 2
        ct = np.zeros((1, 2, L, 8), dtype=np.uint64)
        ct[0, 0] = _residues(ys, qs)
        zero = np.zeros((1, L, 8), dtype=np.uint64)
        got = [int(v) for v in o.combine(ct, [zero])[0]]
        assert got == [floor(Fraction(t * y, Q) + Fraction(1, 2)) % t for y in ys]


# ---------------------------------------------------------------- encode / decode
def test_encode_decode_fixed_point(orc):
    o, ref, qs = _toy(orc, 4, 36, 2, 65537, 4, 10)
    bound = o.encode_clamp()
    assert bound == ((65537 - 1) // 2) // 4 == 8192
    vals = np.array([0.0, 1.0, -1.0, 0.5 / 1024, 1.5 / 1024, 2.5 / 1024, -0.5 / 1024, -1.5 / 1024,
                     7.9999, -7.9999, 8.0, 1e9, -1e9, np.inf, -np.inf, np.nan], dtype=np.float32)
    dec = o.decode(o.encode(vals), 16)
    # ties to even: 0.5 -> 0, 1.5 -> 2, 2.5 -> 2, -0.5 -> -0, -1.5 -> -2
    expect = [0.0, 1.0, -1.0, 0.0, 2 / 1024, 2 / 1024, 0.0, -2 / 1024,
              8192 / 1024, -8192 / 1024, 8.0, 8.0, -8.0, 8.0, -8.0, 0.0]
    assert [float(v) for v in dec] == expect
    assert [v / 1024 for v in ref.fixed([float(v) for v in vals])] == expect
    # slots: the plaintext polynomial evaluates to the fixed-point values
    pt = o.encode(vals)
    assert [int(v) for v in pt[0]] == ref.encode_slots([v % 65537 for v in ref.fixed([float(v) for v in vals])])
    # ragged tail: 5 values in a 16-slot plaintext, rest is zero
    assert np.array_equal(o.encode(vals[:5]), o.encode(np.concatenate([vals[:5], np.zeros(11, np.float32)])))
    # linearity of the encoding mod t
    a = o.encode(np.full(16, 3 / 1024, np.float32)); b = o.encode(np.arange(16, dtype=np.float32) / 1024)
    s = o.encode((np.arange(16, dtype=np.float32) + 3) / 1024)
    assert np.array_equal((a + b) % 65537, s)


def test_coefficient_packing_cross_check(orc):
    """The two encodings are tied by the slot transform (slot encoding = inverse transform mod t of the
    coefficient encoding), and a whole round decodes to the same sums with either."""
    q = orc.find_primes(36, 6, 2)
    t, K, n_values = 257, 3, 150
    o = orc.Oracle(6, q, t, 21, 2, K, SEED)
    rng = np.random.default_rng(12)
    grads = [rng.normal(0, 4.0, n_values).astype(np.float32) for _ in range(K)]
    grads[0][:4] = [np.nan, np.inf, -np.inf, 0.375]
    for g in grads:
        pc, ps = o.encode_coefficients(g), o.encode(g)
        for c in range(pc.shape[0]):
            assert np.array_equal(orc.ntt_inverse(pc[c], t, o.psi_t), ps[c])
        assert np.array_equal(o.decode_coefficients(pc, n_values), o.decode(ps, n_values))
    keys = [o.keygen_share(k) for k in range(K)]
    pk = o.aggregate_pk([k[1] for k in keys])
    sums = []
    for enc, dec in ((o.encode, o.decode), (o.encode_coefficients, o.decode_coefficients)):
        agg = None
        for k in range(K):
            ct = o.encrypt(pk, enc(grads[k]), k, 0, 0)
            agg = ct if agg is None else o.add(agg, ct)
        shares = [o.partial_decrypt(keys[k][0], agg, k, 0, 0) for k in range(K)]
        sums.append(dec(o.combine(agg, shares), n_values))
    assert np.array_equal(sums[0], sums[1])
    clamp = o.encode_clamp()
    fixed = sum(np.clip(np.where(np.isnan(g), 0, np.rint(g * np.float32(4.0))), -clamp, clamp).astype(np.int64) for g in grads)
    assert np.array_equal(sums[1], (fixed.astype(np.float32) * np.float32(0.25)))


def test_clamp_is_exact_for_a_31_bit_plaintext_modulus(orc):
    """The clamp bound floor(((t-1)/2)/K_max) exceeds 2^24 for t above about 2^25 and then need not be a
    float32: the rounded value is compared with it exactly, so K_max clamped terms still cannot wrap mod t."""
    log2n, n, K = 3, 8, 3
    t = orc.find_primes(31, log2n, 1)[0]
    assert (1 << 30) < t < (1 << 31) and t % (2 * n) == 1
    o = orc.Oracle(log2n, orc.find_primes(36, log2n, 2), t, 21, 0, K, SEED)
    clamp = o.encode_clamp()
    assert clamp == ((t - 1) // 2) // K and 3 * clamp <= (t - 1) // 2
    up = np.float32(clamp)
    if int(up) <= clamp:
        up = np.nextafter(up, np.float32(np.inf))
    assert int(up) > clamp                                  # the next float32 above the bound
    assert int(np.float32(clamp)) != clamp, "pick a modulus whose bound is not a float32"
    v = np.array([up, -up, np.inf, -np.inf, np.nextafter(up, np.float32(0)), 3.0e9, -3.0e9, 12345.0], dtype=np.float32)
    want = [min(max(int(np.rint(x)) if np.isfinite(x) else (1 << 62) * (1 if x > 0 else -1), -clamp), clamp) for x in v]
    assert want[0] == clamp and want[1] == -clamp and want[4] < clamp
    pc = o.encode_coefficients(v)
    assert [int(x) for x in pc[0]] == [w % t for w in want]
    assert np.array_equal(orc.ntt_forward(o.encode(v)[0], t, o.psi_t), pc[0])
    # three clamped terms add up without wrapping
    s3 = ((pc.astype(object) * 3) % t).astype(np.uint64)
    assert np.array_equal(o.decode_coefficients(s3, n), np.array([3 * w for w in want], dtype=np.float32))


def test_decode_centres_at_the_boundary(orc):
    """(t-1)/2 is the largest positive value and (t+1)/2 the most negative one, for slots and for coefficients."""
    t, n = 193, 32
    o = orc.Oracle(5, orc.find_primes(36, 5, 1), t, 21, 2, 1, SEED)
    z = np.zeros(n, dtype=np.uint64)
    z[:6] = [0, 1, (t - 1) // 2, (t + 1) // 2, t - 1, (t - 1) // 2 - 1]
    expect = np.array([0, 1, 96, -96, -1, 95], dtype=np.float32) / np.float32(4)
    assert np.array_equal(o.decode_coefficients(z[None], n)[:6], expect)
    pt = orc.ntt_inverse(z, t, o.psi_t)                  # the polynomial with these slot values (textbook transform)
    assert np.array_equal(o.decode(pt[None], n)[:6], expect)
    assert np.all(o.decode(pt[None], n)[6:] == 0)


def test_ciphertext_index_advances_within_a_call(orc):
    """C ciphertexts in one call are C one-ciphertext calls at ct_base, ct_base + 1, ... (those are pinned against
    the big-integer reference above), for every randomised step; equal plaintexts still give different ciphertexts."""
    o, ref, qs = _toy(orc, 4, 36, 2, 97, 2, 3)
    n, K, group, base, C_ = 16, 2, 3, 9, 3
    keys = [o.keygen_share(k) for k in range(K)]
    pk = o.aggregate_pk([k[1] for k in keys])
    rsk, rpk, _, _ = o.receiver_keygen(1)
    pt = np.tile(np.arange(n, dtype=np.uint64) % 97, (C_, 1))
    ct = o.encrypt(pk, pt, 0, group, ct_base=base)
    sh = o.partial_decrypt(keys[1][0], ct, 1, group, ct_base=base)
    cv = o.convert_share(keys[1][0], rpk, ct, 1, 1, group, ct_base=base)
    bs = [o.bootstrap_share(keys[k][0], ct, k, group, ct_base=base) for k in range(K)]
    fresh = o.bootstrap_combine(ct, bs, group, ct_base=base)
    for c in range(C_):
        one = o.encrypt(pk, pt[c:c + 1], 0, group, ct_base=base + c)
        assert np.array_equal(ct[c], one[0])
        assert np.array_equal(sh[c], o.partial_decrypt(keys[1][0], one, 1, group, ct_base=base + c)[0])
        assert np.array_equal(cv[c], o.convert_share(keys[1][0], rpk, one, 1, 1, group, ct_base=base + c)[0])
        bs1 = [o.bootstrap_share(keys[k][0], one, k, group, ct_base=base + c) for k in range(K)]
        for k in range(K):
            assert np.array_equal(bs[k][c], bs1[k][0])
        assert np.array_equal(fresh[c], o.bootstrap_combine(one, bs1, group, ct_base=base + c)[0])
        assert np.array_equal(fresh[c, 1], o.bootstrap_alpha(group, base + c))
        assert np.array_equal(fresh[c, 1], _residues(ref.bootstrap_alpha(group, base + c), qs))
    for a, b in ((ct[0], ct[1]), (sh[0], sh[1]), (cv[0], cv[1]), (bs[0][0], bs[0][1]), (fresh[0, 1], fresh[1, 1])):
        assert not np.array_equal(a, b)


def test_fixed_point_error_bound(orc):
    o, _, _ = _toy(orc, 6, 36, 2, 65537, 1, 13)
    rng = np.random.default_rng(7)
    v = rng.normal(0, 0.5, 64).astype(np.float32)
    d = o.decode(o.encode(v), 64)
    assert np.max(np.abs(d.astype(np.float64) - v.astype(np.float64))) <= 2.0 ** -14   # half of 2^-d
    assert np.array_equal(d, np.rint(v * np.float32(8192)) / np.float32(8192))


# ---------------------------------------------------------------- the worked toy round
def test_worked_toy_round(orc):
    g = {r[0]: [int(v) for v in r[1:]] for r in _rows("toy_round.txt")}
    qs = orc.find_primes(30, 3, 2)
    assert qs == g["q"]
    o = orc.Oracle(3, qs, 17, 21, 0, 3, SEED)
    assert o.psi == g["psi"] and o.psi_t == g["psi_t"][0]
    assert [o.lambda_mod_q(i) for i in range(2)] == g["lambda_mod_q"] and o.q_mod_t() == g["q_mod_t"][0]
    p1 = o.crs()
    assert list(p1[0]) == g["p1_limb0"] and list(p1[1]) == g["p1_limb1"]
    keys = [o.keygen_share(k) for k in range(3)]
    for k in range(3):
        assert list(keys[k][2]) == g[f"s_{k}"] and list(keys[k][3]) == g[f"e_{k}"]
    assert list(keys[0][1][0]) == g["p0_share_0_limb0"]
    pk = o.aggregate_pk([k[1] for k in keys])
    assert list(pk[0, 0]) == g["pk_p0_limb0"] and list(pk[0, 1]) == g["pk_p0_limb1"]
    vs = [np.array([((j + k) % 5) - 2 for j in range(8)], dtype=np.float32) for k in range(3)]
    pts = [o.encode(v) for v in vs]
    for k in range(3):
        assert list(pts[k][0]) == g[f"m_{k}"]
    assert list(orc.sample_ternary(SEED, 4, 0, 0, 0, 8)) == g["u_0"]
    assert list(orc.sample_cbd(SEED, 5, 0, 0, 0, 21, 8)) == g["e0_0"]
    assert list(orc.sample_cbd(SEED, 6, 0, 0, 0, 21, 8)) == g["e1_0"]
    cts = [o.encrypt(pk, pts[k], k, 0, 0) for k in range(3)]
    assert list(cts[0][0, 0, 0]) == g["ct0_c0_limb0"] and list(cts[0][0, 0, 1]) == g["ct0_c0_limb1"]
    assert list(cts[0][0, 1, 0]) == g["ct0_c1_limb0"]
    agg = o.add(o.add(cts[0], cts[1]), cts[2])
    assert list(agg[0, 0, 0]) == g["agg_c0_limb0"] and list(agg[0, 1, 0]) == g["agg_c1_limb0"]
    assert list(orc.sample_cbd(SEED, 7, 0, 0, 0, 21, 8)) == g["smudge_0"]
    shares = [o.partial_decrypt(keys[k][0], agg, k, 0, 0) for k in range(3)]
    assert list(shares[0][0, 0]) == g["share_0_limb0"]
    out = o.combine(agg, shares)
    assert list(out[0]) == g["combined"]
    assert [int(v) for v in o.decode(out, 8)] == g["decoded"]


# ---------------------------------------------------------------- noise margin of the real configs
def test_noise_margin_C1_single_ciphertext(orc):
    """Measured noise of an aggregated C1 ciphertext (the only tight configuration) against
    the bound q/(2t) of the correctness condition, including the wrap term of summing
    representatives in [0,t)."""
    from paper_2207_04604_amd.synth import CONFIGS
    cfg = CONFIGS["C1"]
    o = orc.Oracle(cfg.log2_n, cfg.q, cfg.t, cfg.eta, cfg.frac_bits, cfg.max_group, cfg.seed)
    q, t, n = cfg.q[0], cfg.t, cfg.N
    keys = [o.keygen_share(k) for k in range(4)]
    pk = o.aggregate_pk([k[1] for k in keys])
    grads = cfg.gradients(n_values=n)
    pts = [o.encode(g) for g in grads]
    agg = None
    for k in range(4):
        ct = o.encrypt(pk, pts[k], k, 0, 0)
        agg = ct if agg is None else o.add(agg, ct)
    s_sum = sum(k[2].astype(np.int64) for k in keys)
    s_res = np.array([[int(v) % q for v in s_sum]], dtype=np.uint64)
    m_sum = sum(p.astype(np.int64) for p in pts)[0] % t
    y = (orc.ring_mul(agg[0, 1, 0], s_res[0], q, o.psi[0]).astype(object) + agg[0, 0, 0].astype(object)) % q
    lam = q // t
    noise = [int((int(v) - lam * int(m)) % q) for v, m in zip(y, m_sum)]
    noise = [v - q if v > q // 2 else v for v in noise]
    assert max(abs(v) for v in noise) < q // (2 * t)
    assert np.array_equal(o.decrypt_with_secret(s_res, agg)[0], m_sum.astype(np.uint64))
