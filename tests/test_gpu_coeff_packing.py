"""Coefficient packing (value j of a ciphertext is coefficient j; the addition-only encoding):
the HIP path against the oracle, bit for bit, per call and through the fused rounds."""
import numpy as np
import pytest
import torch

from oracle import oracle as O
from paper_2207_04604_amd import binding as B
from paper_2207_04604_amd.synth import CONFIGS, toy_config

from gpu_util import DEV, Keys, dzeros, make_pair, to_dev, to_eval, to_host
from test_gpu_parity import fixed_point_sum

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name", ["C1", "C2", "C3"])
def test_encode_decode_coefficients(name):
    cfg = CONFIGS[name]
    o, ctx, perm = make_pair(cfg)
    N = cfg.N
    n = min(cfg.n_values, 6 * N + 123) if cfg.C > 7 else cfg.n_values      # several polynomials and a ragged tail
    C_ = (n + N - 1) // N
    g = cfg.gradients()[1][:n].copy()
    g[:8] = [np.nan, np.inf, -np.inf, 1e9, -1e9, 0.5 / (1 << cfg.frac_bits), 1.5 / (1 << cfg.frac_bits), -0.0]
    dpt = dzeros(C_ * N)
    ctx.encode_coefficients(to_dev(g), n, dpt, C_)
    opt = o.encode_coefficients(g, C_)
    assert np.array_equal(to_host(dpt, opt.shape), opt)
    # decoding any plaintext, not only an encoded one
    rng = np.random.default_rng(3)
    anypt = rng.integers(0, cfg.t, size=(C_, N), dtype=np.uint64)
    anypt[0, :4] = [0, cfg.t - 1, (cfg.t - 1) // 2, (cfg.t - 1) // 2 + 1]
    dres = torch.zeros(n, dtype=torch.float32, device=DEV)
    ctx.decode_coefficients(to_dev(anypt), C_, n, dres)
    assert np.array_equal(dres.cpu().numpy(), o.decode_coefficients(anypt, n))
    # slot decoding of arbitrary plaintexts, and of one whose slots sit at the centring boundary
    ctx.decode(to_dev(anypt), C_, n, dres)
    assert np.array_equal(dres.cpu().numpy(), o.decode(anypt, n))
    z = np.zeros((C_, N), dtype=np.uint64)
    z[0, :5] = [(cfg.t - 1) // 2, (cfg.t + 1) // 2, cfg.t - 1, 1, (cfg.t - 1) // 2 - 1]
    edge = np.stack([O.ntt_inverse(z[c], cfg.t, o.psi_t) for c in range(C_)])
    ctx.decode(to_dev(edge), C_, n, dres)
    got = dres.cpu().numpy()
    assert np.array_equal(got, o.decode(edge, n))
    half = (cfg.t - 1) // 2
    assert list(got[:5] * np.float32(2.0 ** cfg.frac_bits)) == [half, -half, -1, 1, half - 1]
    # the slot encoding of the same values is its inverse transform modulo t
    dslots = dzeros(C_ * N)
    ctx.encode(to_dev(g), n, dslots, C_)
    slots = to_host(dslots, opt.shape)
    assert np.array_equal(slots[0], O.ntt_inverse(opt[0], cfg.t, o.psi_t))
    with pytest.raises(B.D2mheError):
        ctx.encode_coefficients(to_dev(g), C_ * N + 1, dpt, C_)
    ctx.close()


def test_round_with_coefficient_packing_per_call_and_fused():
    cfg = toy_config(11, O.find_primes(36, 11, 2), 65537, 4, 2 * 2048 + 77, frac_bits=8)
    o, ctx, perm = make_pair(cfg)
    L, N, n, C_ = o.L, o.N, cfg.n_values, cfg.C
    grads = cfg.gradients()
    members = cfg.groups()[0]
    keys = Keys(o, ctx, perm, members, check=False)
    opk, dpk = keys.group_pk(members, perm)
    dagg = oagg = None
    for k in members:
        dpt = dzeros(C_ * N)
        ctx.encode_coefficients(to_dev(grads[k]), n, dpt, C_)
        dct = dzeros(C_ * 2 * L * N)
        ctx.encrypt(dpk, dpt, C_, k, 2, 0, dct)
        oct_ = o.encrypt(opk, o.encode_coefficients(grads[k]), k, 2, 0)
        assert np.array_equal(to_host(dct, oct_.shape), to_eval(o, perm, oct_))
        if dagg is None:
            dagg, oagg = dct, oct_
        else:
            ctx.add(dagg, dct, C_)
            oagg = o.add(oagg, oct_)
    dshares, oshares = [], []
    for k in members:
        dsh = dzeros(C_ * L * N)
        ctx.partial_decrypt(keys.sk[k], dagg, C_, k, 2, 0, dsh)
        dshares.append(dsh)
        oshares.append(o.partial_decrypt(keys.osk[k], oagg, k, 2, 0))
    dout = dzeros(C_ * N)
    ctx.combine(dagg, dshares, C_, dout)
    opt = o.combine(oagg, oshares)
    assert np.array_equal(to_host(dout, opt.shape), opt)
    dres = torch.zeros(n, dtype=torch.float32, device=DEV)
    ctx.decode_coefficients(dout, C_, n, dres)
    expect = fixed_point_sum([grads[k] for k in members], cfg.frac_bits, o.encode_clamp())
    assert np.array_equal(o.decode_coefficients(opt, n), expect)
    assert np.array_equal(dres.cpu().numpy(), expect)
    # the fused round with packing = 1: same result, and the same aggregate in its scratch
    K = len(members)
    nbytes = ctx.round_scratch_bytes(K, 1, n)
    scratch = dzeros(nbytes // 8)
    out = torch.zeros(n, dtype=torch.float32, device=DEV)
    desc = ctx.make_round([members], [dpk], [keys.sk[k] for k in members], [to_dev(grads[k]) for k in members], [out], n,
                          group_ids=[2], packing=1)
    ctx.round(desc, scratch, nbytes)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), expect)
    s = to_host(scratch)
    assert np.array_equal(s[K * C_ * 2 * L * N:(K + 1) * C_ * 2 * L * N].reshape(oagg.shape), to_eval(o, perm, oagg))
    bad = ctx.make_round([members], [dpk], [keys.sk[k] for k in members], [to_dev(grads[k]) for k in members], [out], n,
                         group_ids=[2], packing=2)
    with pytest.raises(B.D2mheError) as ei:
        ctx.round(bad, scratch, nbytes)
    assert ei.value.status == B.ERR_RANGE
    ctx.close()


@pytest.mark.parametrize("name", ["C2", "C3"])
def test_whole_round_and_key_switching_round_with_coefficient_packing(name):
    """All groups in one call, in the launch shape the benchmark times, with packing = 1: the decoded sums
    equal the fixed-point sums (which the oracle's coefficient-packed round also gives, checked above and in
    the CPU pins), for the collective decryption and for the key-switching round."""
    from test_gpu_convert import RecvKeys
    cfg = CONFIGS[name]
    o, ctx, perm = make_pair(cfg)
    groups, grads = cfg.groups(), cfg.gradients()
    keys = Keys(o, ctx, perm, range(cfg.parties), check=False)
    pks = [keys.group_pk(g, perm, check=False) for g in groups]
    dgr = [to_dev(g) for g in grads]
    outs = [torch.zeros(cfg.n_values, dtype=torch.float32, device=DEV) for _ in groups]
    J, G = sum(len(g) for g in groups), len(groups)
    sks = [keys.sk[k] for k in range(cfg.parties)]
    desc = ctx.make_round(groups, [p[1] for p in pks], sks, dgr, outs, cfg.n_values, packing=1)
    nbytes = ctx.round_scratch_bytes(J, G, cfg.n_values)
    scratch = dzeros(nbytes // 8)
    ctx.round(desc, scratch, nbytes)
    torch.cuda.synchronize()
    clamp = o.encode_clamp()
    expects = [fixed_point_sum([grads[k] for k in g], cfg.frac_bits, clamp) for g in groups]
    for gi in range(G):
        assert np.array_equal(outs[gi].cpu().numpy(), expects[gi]), f"group {gi}"
    # one sampled fresh ciphertext against the oracle's encryption of the coefficient-packed plaintext
    L, N, C_ = cfg.L, cfg.N, cfg.C
    gi, mi, c = G - 1, 1, C_ - 1
    k = groups[gi][mi]
    off = sum(len(g) for g in groups[:gi]) + mi
    lo, hi = c * N, min((c + 1) * N, cfg.n_values)
    oct_ = o.encrypt(pks[gi][0], o.encode_coefficients(grads[k][lo:hi]), k, gi, c)
    dct = scratch[:J * C_ * 2 * L * N].view(J, C_, 2 * L * N)[off, c]
    assert np.array_equal(to_host(dct, (1, 2, L, N)), to_eval(o, perm, oct_))
    del scratch
    # key switching: every receiver's own decryption gives the same sums
    recvs = cfg.receivers()
    rk = RecvKeys(o, ctx, perm, sorted({r for rs in recvs for r in rs}))
    routs = [torch.zeros(cfg.n_values, dtype=torch.float32, device=DEV) for rs in recvs for _ in rs]
    cd = ctx.make_convert(desc, recvs, rk.pk, rk.sk, routs)
    nbytes = ctx.round_convert_scratch_bytes(J, G, cd.num_shares, cfg.n_values)
    scratch = dzeros(nbytes // 8)
    ctx.round_convert(desc, cd, scratch, nbytes)
    torch.cuda.synchronize()
    i = 0
    for gi, rs in enumerate(recvs):
        for _ in rs:
            assert np.array_equal(routs[i].cpu().numpy(), expects[gi]), f"group {gi} receiver {i}"
            i += 1
    ctx.close()
