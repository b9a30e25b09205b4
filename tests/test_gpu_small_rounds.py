"""Small single-limb rounds through d2mhe_round against the oracle: every fresh ciphertext, aggregate, share and
decoded value the call leaves behind, for every arithmetic back-end, one to eight groups of one to seven members,
overlapping neighbourhoods, ragged tails, both packings, odd group ids and a ciphertext index offset, groups of
different sizes."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from oracle import oracle as O
from paper_2207_04604_amd.synth import toy_config

from gpu_util import DEV, Keys, dzeros, make_pair, to_dev, to_eval, to_host


# (prime bits, log2 N, members per group, groups, packing, all groups of the same size)
@pytest.mark.parametrize("bits,log2n,K,G,packing,uniform", [(30, 10, 4, 1, 0, True), (54, 10, 7, 3, 0, True),
                                                            (44, 11, 3, 8, 1, True), (60, 10, 2, 2, 0, True),
                                                            (55, 10, 1, 5, 0, True), (54, 11, 4, 2, 0, True),
                                                            (54, 10, 3, 2, 0, False)])
def test_round_objects_of_small_single_limb_rounds(bits, log2n, K, G, packing, uniform):
    N = 1 << log2n
    t = 12289
    q = O.find_primes(bits, log2n, 1)
    P = K + G                                            # overlapping neighbourhoods on a ring of P nodes
    cfg = toy_config(log2n, q, t, parties=P, n_values=2 * N + 11, frac_bits=4)
    o, ctx, perm = make_pair(cfg, max_group=K)
    rng = np.random.default_rng(bits * 100 + K)
    grads = [rng.normal(0, 4.0, cfg.n_values).astype(np.float32) for _ in range(P)]
    grads[0][:3] = [np.nan, 1e9, -1e9]
    keys = Keys(o, ctx, perm, range(P), check=False)
    groups = [[(g + m) % P for m in range(K)] for g in range(G)]
    if not uniform:
        groups[-1] = groups[-1][:-1]
    gids = [7 + 3 * g for g in range(G)]
    pks = [keys.group_pk(g, perm, check=False) for g in groups]
    outs = [torch.zeros(cfg.n_values, dtype=torch.float32, device=DEV) for _ in groups]
    J = sum(len(g) for g in groups)
    nbytes = ctx.round_scratch_bytes(J, G, cfg.n_values)
    scratch = dzeros(nbytes // 8)
    ct_base = 5
    desc = ctx.make_round(groups, [p[1] for p in pks], [keys.sk[k] for k in range(P)], [to_dev(g) for g in grads], outs,
                          cfg.n_values, group_ids=gids, ct_base=ct_base, packing=packing)
    for _ in range(2):                                   # the second run overwrites the first one's scratch
        ctx.round(desc, scratch, nbytes)
    torch.cuda.synchronize()
    L, C_ = 1, cfg.C
    LN = L * N
    s = to_host(scratch)
    cts = s[:J * C_ * 2 * LN].reshape(J, C_, 2, L, N)
    agg = s[J * C_ * 2 * LN:(J + G) * C_ * 2 * LN].reshape(G, C_, 2, L, N)
    shares = s[(J + G) * C_ * 2 * LN:(J + G) * C_ * 2 * LN + J * C_ * LN].reshape(J, C_, L, N)
    enc = o.encode_coefficients if packing else o.encode
    dec = o.decode_coefficients if packing else o.decode
    j = 0
    for gi, g in enumerate(groups):
        opk, oagg = pks[gi][0], None
        j0 = j
        for k in g:
            oct_ = o.encrypt(opk, enc(grads[k]), k, gids[gi], ct_base)
            assert np.array_equal(cts[j], to_eval(o, perm, oct_)), f"fresh ciphertexts of party {k} in group {gi}"
            oagg = oct_ if oagg is None else o.add(oagg, oct_)
            j += 1
        assert np.array_equal(agg[gi], to_eval(o, perm, oagg)), f"aggregate of group {gi}"
        oshares = []
        for m, k in enumerate(g):
            osh = o.partial_decrypt(keys.osk[k], oagg, k, gids[gi], ct_base)
            assert np.array_equal(shares[j0 + m], to_eval(o, perm, osh)), f"share of party {k} in group {gi}"
            oshares.append(osh)
        assert np.array_equal(outs[gi].cpu().numpy(), dec(o.combine(oagg, oshares), cfg.n_values)), f"group {gi}"
    ctx.close()
