"""Several iterations of privacy-preserving D-PSGD (Alg. 2) on the GPU against the oracle: every
iteration exchanges the nodes' weight vectors through the encrypted round (collective decryption on
a complete graph, key switching to the receivers on a ring), then every node averages and takes a
local step.  Weights are compared bit for bit after every iteration; the local "gradients" are
seeded synthetic vectors (no dataset is involved)."""
import numpy as np
import pytest
import torch

from oracle import oracle as O
from paper_2207_04604_amd import binding as B
from paper_2207_04604_amd.synth import CONFIGS, toy_config

from gpu_util import DEV, Keys, dzeros, make_pair, to_dev, to_eval, to_host
from test_gpu_convert import RecvKeys

pytestmark = pytest.mark.gpu


def oracle_round(o, opk, osks, weights, members, group, ct_base):
    """One group's round by the oracle's separate calls, ciphertext indices ct_base + c."""
    agg = None
    for k in members:
        ct = o.encrypt(opk, o.encode(weights[k]), k, group, ct_base)
        agg = ct if agg is None else o.add(agg, ct)
    shares = [o.partial_decrypt(osks[k], agg, k, group, ct_base) for k in members]
    return o.decode(o.combine(agg, shares), weights[members[0]].size), agg


@pytest.mark.parametrize("convert", [False, True])
def test_training_iterations_match_the_oracle(convert):
    if convert:     # ring of 5 nodes: five closed neighbourhoods of 3, each with its own receiver
        cfg = toy_config(10, O.find_primes(36, 10, 2), 65537, 5, 1500, frac_bits=8, topology="circulant", offsets=(1,))
    else:           # complete graph of 4 nodes: one group, collective decryption
        cfg = CONFIGS["C1"]
    o, ctx, perm = make_pair(cfg)
    P, n, C_, L, N = cfg.parties, cfg.n_values, cfg.C, cfg.L, cfg.N
    groups, receivers = cfg.groups(), cfg.receivers()
    G, J = len(groups), sum(len(g) for g in groups)
    keys = Keys(o, ctx, perm, range(P), check=False)
    pks = [keys.group_pk(g, perm, check=False) for g in groups]
    rng = np.random.default_rng(77)
    w_host = [rng.normal(0, 0.5, n).astype(np.float32) for _ in range(P)]
    w_dev = [to_dev(w) for w in w_host]
    gamma, T = 0.05, 3
    if convert:
        rkeys = RecvKeys(o, ctx, perm, range(P))
        outs = [torch.zeros(n, dtype=torch.float32, device=DEV) for rs in receivers for _ in rs]
        S = sum(len(g) * len(r) for g, r in zip(groups, receivers))
        nbytes = ctx.round_convert_scratch_bytes(J, G, S, n)
    else:
        outs = [torch.zeros(n, dtype=torch.float32, device=DEV) for _ in groups]
        nbytes = ctx.round_scratch_bytes(J, G, n)
    scratch = dzeros(nbytes // 8)
    owner = {}                                   # node -> (group, index of its output buffer)
    i = 0
    for gi, rs in enumerate(receivers):
        for r in rs:
            owner[r] = (gi, i if convert else gi)
            i += 1
    for it in range(T):
        grads = [rng.normal(0, 0.1, n).astype(np.float32) for _ in range(P)]
        ct_base = it * C_
        desc = ctx.make_round(groups, [p[1] for p in pks], [keys.sk[k] for k in range(P)], w_dev,
                              outs if not convert else [outs[0]] * G, n, ct_base=ct_base)
        if convert:
            conv = ctx.make_convert(desc, receivers, [rkeys.pk[k] for k in range(P)],
                                    [rkeys.sk[k] for k in range(P)], outs)
            ctx.round_convert(desc, conv, scratch, nbytes)
        else:
            ctx.round(desc, scratch, nbytes)
        # oracle: the same round, group by group
        osums, oaggs = [], []
        for gi, g in enumerate(groups):
            s, agg = oracle_round(o, pks[gi][0], keys.osk, w_host, g, gi, ct_base)
            osums.append(s)
            oaggs.append(agg)
        torch.cuda.synchronize()
        # the aggregate in the scratch used this iteration's ciphertext indices
        LN = L * N
        agg0 = to_host(scratch[J * C_ * 2 * LN:(J + 1) * C_ * 2 * LN], (C_, 2, L, N))
        assert np.array_equal(agg0, to_eval(o, perm, oaggs[0])), f"aggregate of group 0, iteration {it}"
        new_dev = []
        for node in range(P):
            gi, oi = owner[node]
            K = len(groups[gi])
            assert np.array_equal(outs[oi].cpu().numpy(), osums[gi]), f"sum for node {node}, iteration {it}"
            w_new = torch.empty(n, dtype=torch.float32, device=DEV)
            B.average_update(outs[oi], K, to_dev(grads[node]), gamma, n, w_new)
            new_dev.append(w_new)
            w_host[node] = O.average_update(osums[gi], K, grads[node], gamma)
        torch.cuda.synchronize()
        w_dev = new_dev
        for node in range(P):
            assert np.array_equal(w_dev[node].cpu().numpy(), w_host[node]), f"weights of node {node}, iteration {it}"
    # the nodes have moved towards each other (averaging) without leaving the fixed-point range
    assert max(float(np.abs(w).max()) for w in w_host) < o.encode_clamp() / 2.0 ** cfg.frac_bits
    ctx.close()


def test_average_update_argument_checks():
    x = torch.zeros(16, dtype=torch.float32, device=DEV)
    with pytest.raises(B.D2mheError) as ei:
        B.average_update(x, 0, x, 0.1, 16, x)
    assert ei.value.status == B.ERR_RANGE
    with pytest.raises(B.D2mheError) as ei:
        B.average_update(x, 2, None, 0.1, 16, x)
    assert ei.value.status == B.ERR_NULL
    B.average_update(x, 2, None, 0.0, 16, x)
    B.average_update(x, 2, x, 0.5, 0, x)
    torch.cuda.synchronize()
