#!/usr/bin/env python3
"""Recomputes tests/golden/params.txt and tests/golden/toy_round.txt from the written rules, in
plain Python integers, and compares them with the stored files (or rewrites them with --write).

These two files are pins FOR the CPU oracle, so nothing here calls the oracle or the HIP library:
primes, roots and constants come from Python's own arithmetic (a Miller-Rabin test of its own,
pow()), and the worked round from the brute-force reference tests/pyref.py (no RNS, no fast
transform, exact rationals).  tests/test_oracle_pins.py runs the comparison, so a stored value that
nobody can reproduce cannot survive.

  python tests/golden/regenerate.py            # compare, exit status 1 on any difference
  python tests/golden/regenerate.py --write    # rewrite both files
"""
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(HERE))
import pyref  # noqa: E402

SEED = 0x0123456789ABCDEF


def is_prime(n):
    """Miller-Rabin with the first 13 primes as bases: deterministic far beyond 2^64."""
    small = (2, 3, 5, 7, 11, 13, 17, 19, 23, 29, 31, 37, 41)
    if n < 2:
        return False
    for p in small:
        if n % p == 0:
            return n == p
    d, r = n - 1, 0
    while d % 2 == 0:
        d, r = d // 2, r + 1
    for a in small:
        y = pow(a, d, n)
        if y in (1, n - 1):
            continue
        for _ in range(r - 1):
            y = y * y % n
            if y == n - 1:
                break
        else:
            return False
    return True


def primes_by_rule(bits, log2n, count):
    """The `count` largest primes 2^bits - k 2N + 1, k = 1, 2, ...; returns [(q, k)]."""
    out, k = [], 0
    while len(out) < count:
        k += 1
        q = (1 << bits) - k * (2 << log2n) + 1
        if is_prime(q):
            out.append((q, k))
    return out


def root_by_rule(q, log2n):
    """(x, psi): psi = x^((q-1)/2N) for the smallest x >= 2 with psi^N = -1."""
    n = 1 << log2n
    for x in range(2, q):
        psi = pow(x, (q - 1) // (2 * n), q)
        if pow(psi, n, q) == q - 1:
            return x, psi
    raise ValueError("no root")


WORKLOADS = [("C1", 30, 10, 1, 12289), ("C2", 36, 12, 3, 65537), ("C3", 54, 13, 4, 65537), ("C4", 54, 14, 8, 65537)]


def params_text():
    lines = ["# Parameter sets of the five workloads.  Primes follow the rule \"the L largest primes of",
             "# the form 2^b - k*2N + 1, k = 1, 2, ...\"; psi = x^((q-1)/2N) for the smallest x >= 2 with",
             "# psi^N = -1.  Written by tests/golden/regenerate.py from these rules in Python integers,",
             "# independently of the oracle; the oracle's own search must reproduce them.",
             "# columns: set b log2N q k x psi"]
    sets = {}
    for name, bits, log2n, count, t in WORKLOADS:
        sets[name] = primes_by_rule(bits, log2n, count)
        for q, k in sets[name]:
            x, psi = root_by_rule(q, log2n)
            lines.append(f"{name} {bits} {log2n} {q} {k} {x} {psi}")
    c5 = primes_by_rule(60, 16, 16)
    for q, k in (c5[0], c5[-1]):
        x, psi = root_by_rule(q, 16)
        lines.append(f"C5 60 16 {q} {k} {x} {psi}")
    lines.append("# slot roots: set t x psi_t")
    for name, bits, log2n, count, t in WORKLOADS:
        x, psi = root_by_rule(t, log2n)
        lines.append(f"T {name} {t} {x} {psi}")
    lines.append("# misc: set (Q mod t) bits(floor(Q/t))")
    for name, bits, log2n, count, t in WORKLOADS:
        Q = 1
        for q, _ in sets[name]:
            Q *= q
        lines.append(f"M {name} {Q % t} {(Q // t).bit_length()}")
    lines.append("# C5 k values in order")
    lines.append("K5 " + " ".join(str(k) for _, k in c5))
    return "\n".join(lines) + "\n"


def toy_round_text():
    log2n, n, t, K = 3, 8, 17, 3
    qs = [q for q, _ in primes_by_rule(30, log2n, 2)]
    psis = [root_by_rule(q, log2n)[1] for q in qs]
    psi_t = root_by_rule(t, log2n)[1]
    ref = pyref.PyBFV(n, qs, t, 21, 0, K, SEED, psi_t)
    limb = lambda poly, i: " ".join(str(v % qs[i]) for v in poly)
    row = lambda vals: " ".join(str(v) for v in vals)
    lines = ["# Worked toy round, written by tests/golden/regenerate.py independently of the oracle, with",
             "# schoolbook products and arbitrary-precision integers (tests/pyref.py).",
             "# N = 8, primes by the rule with b = 30, t = 17, P = 3 parties, complete graph (one group,",
             "# g = 0), one ciphertext (c = 0), f = 0, eta = 21, seed = 0x0123456789ABCDEF,",
             "# values v_k[j] = ((j + k) mod 5) - 2.",
             "q " + row(qs), "psi " + row(psis), f"psi_t {psi_t}",
             "lambda_mod_q " + row(ref.Lam % q for q in qs), f"q_mod_t {ref.Q % t}",
             "p1_limb0 " + limb(ref.p1, 0), "p1_limb1 " + limb(ref.p1, 1)]
    keys = [ref.keygen(k) for k in range(K)]
    for k in range(K):
        lines += [f"s_{k} " + row(keys[k][0]), f"e_{k} " + row(keys[k][1])]
    lines.append("p0_share_0_limb0 " + limb(keys[0][2], 0))
    p0 = ref.aggregate_pk([k[2] for k in keys])
    lines += ["pk_p0_limb0 " + limb(p0, 0), "pk_p0_limb1 " + limb(p0, 1)]
    ms = [ref.encode_slots([z % t for z in ref.fixed([float(((j + k) % 5) - 2) for j in range(n)])]) for k in range(K)]
    for k in range(K):
        lines.append(f"m_{k} " + row(ms[k]))
    cts, rnd = zip(*[ref.encrypt(p0, ms[k], k, 0, 0) for k in range(K)])
    lines += ["u_0 " + row(rnd[0][0]), "e0_0 " + row(rnd[0][1]), "e1_0 " + row(rnd[0][2]),
              "ct0_c0_limb0 " + limb(cts[0][0], 0), "ct0_c0_limb1 " + limb(cts[0][0], 1),
              "ct0_c1_limb0 " + limb(cts[0][1], 0)]
    agg = ref.add(ref.add(cts[0], cts[1]), cts[2])
    lines += ["agg_c0_limb0 " + limb(agg[0], 0), "agg_c1_limb0 " + limb(agg[1], 0)]
    shares, smudge = zip(*[ref.share(keys[k][0], agg, k, 0, 0) for k in range(K)])
    lines += ["smudge_0 " + row(smudge[0]), "share_0_limb0 " + limb(shares[0], 0)]
    combined = ref.combine(agg, shares)
    lines += ["combined " + row(combined), "decoded " + row(ref.decode_slots(combined))]
    return "\n".join(lines) + "\n"


def main(write=False):
    bad = []
    for name, text in (("params.txt", params_text()), ("toy_round.txt", toy_round_text())):
        path = os.path.join(HERE, name)
        if write:
            with open(path, "w") as fh:
                fh.write(text)
        elif open(path).read() != text:
            bad.append(name)
    return bad


if __name__ == "__main__":
    differing = main("--write" in sys.argv[1:])
    if differing:
        print("differs from what the rules give:", ", ".join(differing))
        sys.exit(1)
    print("tests/golden/params.txt and toy_round.txt are reproduced" if "--write" not in sys.argv[1:] else "written")
