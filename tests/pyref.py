"""Brute-force reference for tiny parameters, in pure Python integers.

Deliberately structured differently from the oracle: no RNS, no fast transform.  Ring
elements are lists of Python ints modulo the full Q = prod q_i, products are schoolbook
negacyclic convolutions, the decryption rounding uses exact rational arithmetic and slots
are evaluated/interpolated term by term.  The oracle's RNS results must agree with these
values reduced modulo each q_i.  Only usable for N up to a few hundred.
"""
from fractions import Fraction
from math import floor, prod

M32 = 0xFFFFFFFF


def philox4x32_10(ctr, key):
    c = list(ctr)
    k0, k1 = key
    for _ in range(10):
        p0 = 0xD2511F53 * c[0]
        p1 = 0xCD9E8D57 * c[2]
        c = [((p1 >> 32) ^ c[1] ^ k0) & M32, p1 & M32, ((p0 >> 32) ^ c[3] ^ k1) & M32, p0 & M32]
        k0 = (k0 + 0x9E3779B9) & M32
        k1 = (k1 + 0xBB67AE85) & M32
    return c


def _block(seed, block, ct, party, domain, limb, group):
    return philox4x32_10([block, ct, party, domain | (limb << 8) | (group << 16)],
                         [seed & M32, seed >> 32])


def ternary(seed, domain, party, group, ct, n):
    return [((_block(seed, i >> 2, ct, party, domain, 0, group)[i & 3] * 3) >> 32) - 1
            for i in range(n)]


def cbd(seed, domain, party, group, ct, eta, n):
    mask = (1 << eta) - 1
    out = []
    for i in range(n):
        w = _block(seed, i >> 1, ct, party, domain, 0, group)
        j = 2 * (i & 1)
        out.append(bin(w[j] & mask).count("1") - bin(w[j + 1] & mask).count("1"))
    return out


def uniform(seed, domain, limb, party, group, ct, q, n):
    out = []
    for i in range(n):
        w = _block(seed, i, ct, party, domain, limb, group)
        out.append((w[0] | (w[1] << 32) | (w[2] << 64) | (w[3] << 96)) % q)
    return out


def negacyclic(a, b, mod):
    n = len(a)
    out = [0] * n
    for i, ai in enumerate(a):
        if ai == 0:
            continue
        for j, bj in enumerate(b):
            k = i + j
            if k < n:
                out[k] += ai * bj
            else:
                out[k - n] -= ai * bj
    return [v % mod for v in out]


def crt(residues, qs):
    Q = prod(qs)
    x = 0
    for r, q in zip(residues, qs):
        Qi = Q // q
        x += r * Qi * pow(Qi, -1, q)
    return x % Q


class PyBFV:
    """Multiparty BFV over Z_Q (Q = prod q_i), straight from Sec. 3.2 and Sec. 4.2."""

    DOM = dict(SK=1, PK_E=2, CRS=3, ENC_U=4, ENC_E0=5, ENC_E1=6, DEC_E=7,
               RSK=0x10, RPK_A=0x11, RPK_E=0x12, CVT_U=0x13, CVT_E0=0x14, CVT_E1=0x15,
               BS_M=0x16, BS_E0=0x17, BS_E1=0x18, BS_A=0x19)

    def __init__(self, n, qs, t, eta, frac_bits, max_group, seed, psi_t):
        self.n, self.qs, self.t, self.eta = n, list(qs), t, eta
        self.f, self.kmax, self.seed, self.psi_t = frac_bits, max_group, seed, psi_t
        self.Q = prod(qs)
        self.Lam = self.Q // t
        # CRS: sampled per limb, then glued together by the Chinese remainder theorem
        limbs = [uniform(seed, self.DOM["CRS"], i, 0, 0, 0, q, n) for i, q in enumerate(qs)]
        self.p1 = [crt([limbs[i][k] for i in range(len(qs))], qs) for k in range(n)]

    def keygen(self, party):
        s = ternary(self.seed, self.DOM["SK"], party, 0, 0, self.n)
        e = cbd(self.seed, self.DOM["PK_E"], party, 0, 0, self.eta, self.n)
        prod_ = negacyclic(self.p1, s, self.Q)
        p0 = [(-(prod_[k] + e[k])) % self.Q for k in range(self.n)]
        return s, e, p0

    def aggregate_pk(self, p0s):
        return [sum(col) % self.Q for col in zip(*p0s)]

    def fixed(self, values):
        bound = ((self.t - 1) // 2) // self.kmax
        out = []
        for v in values:
            if v != v:
                r = 0
            elif v in (float("inf"), float("-inf")):
                r = bound if v > 0 else -bound
            else:
                x = Fraction(v) * (1 << self.f)          # exact
                fl = floor(x)
                d = x - fl
                r = fl + (1 if d > Fraction(1, 2) or (d == Fraction(1, 2) and fl % 2 == 1) else 0)
                r = max(-bound, min(bound, r))
            out.append(r)
        return out

    def encode_slots(self, z):
        """m with m(psi_t^(2j+1)) = z[j] (interpolation written out term by term)."""
        n, t = self.n, self.t
        ninv = pow(n, -1, t)
        pinv = pow(self.psi_t, -1, t)
        return [(ninv * sum(z[j] * pow(pinv, (2 * j + 1) * k, t) for j in range(n))) % t
                for k in range(n)]

    def decode_slots(self, m):
        n, t = self.n, self.t
        z = [sum(m[k] * pow(self.psi_t, (2 * j + 1) * k, t) for k in range(n)) % t for j in range(n)]
        return [v - t if v > (t - 1) // 2 else v for v in z]

    def encrypt(self, p0, m, party, group, ct):
        u = ternary(self.seed, self.DOM["ENC_U"], party, group, ct, self.n)
        e0 = cbd(self.seed, self.DOM["ENC_E0"], party, group, ct, self.eta, self.n)
        e1 = cbd(self.seed, self.DOM["ENC_E1"], party, group, ct, self.eta, self.n)
        up0 = negacyclic(p0, u, self.Q)
        up1 = negacyclic(self.p1, u, self.Q)
        c0 = [(self.Lam * m[k] + up0[k] + e0[k]) % self.Q for k in range(self.n)]
        c1 = [(up1[k] + e1[k]) % self.Q for k in range(self.n)]
        return (c0, c1), (u, e0, e1)

    def add(self, a, b):
        return tuple([(x + y) % self.Q for x, y in zip(ca, cb)] for ca, cb in zip(a, b))

    def share(self, s, ct, party, group, cti):
        e = cbd(self.seed, self.DOM["DEC_E"], party, group, cti, self.eta, self.n)
        sc1 = negacyclic(ct[1], s, self.Q)
        return [(sc1[k] + e[k]) % self.Q for k in range(self.n)], e

    def scale_round(self, y):
        out = []
        for v in y:
            x = Fraction(self.t * (v % self.Q), self.Q)
            r = floor(x + Fraction(1, 2))
            out.append(r % self.t)
        return out

    def combine(self, ct, shares):
        y = [(ct[0][k] + sum(h[k] for h in shares)) % self.Q for k in range(self.n)]
        return self.scale_round(y)

    def decrypt(self, s, ct):
        sc1 = negacyclic(ct[1], s, self.Q)
        return self.scale_round([(ct[0][k] + sc1[k]) % self.Q for k in range(self.n)])

    def noise(self, s, ct, m):
        """Centred representative of c0 + c1 s - Lambda m."""
        sc1 = negacyclic(ct[1], s, self.Q)
        out = []
        for k in range(self.n):
            v = (ct[0][k] + sc1[k] - self.Lam * m[k]) % self.Q
            out.append(v - self.Q if v > self.Q // 2 else v)
        return out

    # ---- MBFV.Convert (Sec. 4.2 item 3): key switching to the receiver's own key ----
    def receiver_keygen(self, party):
        """Single-key BFV pair of one node (Sec. 3.2 items 1-2), over Z_Q."""
        s = ternary(self.seed, self.DOM["RSK"], party, 0, 0, self.n)
        e = cbd(self.seed, self.DOM["RPK_E"], party, 0, 0, self.eta, self.n)
        limbs = [uniform(self.seed, self.DOM["RPK_A"], i, party, 0, 0, q, self.n)
                 for i, q in enumerate(self.qs)]
        p1 = [crt([limbs[i][k] for i in range(len(self.qs))], self.qs) for k in range(self.n)]
        sp = negacyclic(p1, s, self.Q)
        p0 = [(-(sp[k] + e[k])) % self.Q for k in range(self.n)]
        return s, e, (p0, p1)

    def convert_share(self, s_k, pk_i, ct, party, receiver, group, cti):
        """Eq. (1): (h0, h1) = (s_k c1 + mu_k p0_i + e0_k, mu_k p1_i + e1_k)."""
        who = party | (receiver << 16)
        mu = ternary(self.seed, self.DOM["CVT_U"], who, group, cti, self.n)
        e0 = cbd(self.seed, self.DOM["CVT_E0"], who, group, cti, self.eta, self.n)
        e1 = cbd(self.seed, self.DOM["CVT_E1"], who, group, cti, self.eta, self.n)
        sc1 = negacyclic(ct[1], s_k, self.Q)
        mp0 = negacyclic(pk_i[0], mu, self.Q)
        mp1 = negacyclic(pk_i[1], mu, self.Q)
        h0 = [(sc1[k] + mp0[k] + e0[k]) % self.Q for k in range(self.n)]
        h1 = [(mp1[k] + e1[k]) % self.Q for k in range(self.n)]
        return (h0, h1), (mu, e0, e1)

    def convert_combine(self, ct, shares):
        """E' = (c0 + sum h0_k, sum h1_k)."""
        c0 = [(ct[0][k] + sum(h[0][k] for h in shares)) % self.Q for k in range(self.n)]
        c1 = [sum(h[1][k] for h in shares) % self.Q for k in range(self.n)]
        return c0, c1

    # ---- MBFV.Bootstrap (Sec. 4.2 item 4): collective refresh ----
    def bootstrap_alpha(self, group, cti):
        limbs = [uniform(self.seed, self.DOM["BS_A"], i, 0, group, cti, q, self.n) for i, q in enumerate(self.qs)]
        return [crt([limbs[i][k] for i in range(len(self.qs))], self.qs) for k in range(self.n)]

    def bootstrap_share(self, s_k, ct, party, group, cti):
        """Eq. (3): (eta0, eta1) = (s_k c1 - Lambda M_k + e0_k, -s_k alpha + Lambda M_k + e1_k)."""
        M = uniform(self.seed, self.DOM["BS_M"], 0, party, group, cti, self.t, self.n)
        e0 = cbd(self.seed, self.DOM["BS_E0"], party, group, cti, self.eta, self.n)
        e1 = cbd(self.seed, self.DOM["BS_E1"], party, group, cti, self.eta, self.n)
        alpha = self.bootstrap_alpha(group, cti)
        sc1 = negacyclic(ct[1], s_k, self.Q)
        sa = negacyclic(alpha, s_k, self.Q)
        eta0 = [(sc1[k] - self.Lam * M[k] + e0[k]) % self.Q for k in range(self.n)]
        eta1 = [(-sa[k] + self.Lam * M[k] + e1[k]) % self.Q for k in range(self.n)]
        return (eta0, eta1), (M, e0, e1)

    def bootstrap_combine(self, ct, shares, group, cti):
        y = [(ct[0][k] + sum(h[0][k] for h in shares)) % self.Q for k in range(self.n)]
        x = self.scale_round(y)
        c0 = [(self.Lam * x[k] + sum(h[1][k] for h in shares)) % self.Q for k in range(self.n)]
        return (c0, self.bootstrap_alpha(group, cti)), x
