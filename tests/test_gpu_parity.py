"""Parity of the HIP library with the CPU oracle, through the C ABI, on a real MI355X.

Bar: bit-exact on every coefficient of every key, ciphertext, share and plaintext, and
0 ulp on the decoded floats (the arithmetic is integer; the float steps are exact)."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from oracle import oracle as O
from paper_2207_04604_amd import binding as B
from paper_2207_04604_amd.synth import CONFIGS, toy_config

from gpu_util import DEV, Keys, dzeros, make_ctx, make_pair, to_dev, to_eval, to_host


def fixed_point_sum(grads, f, clamp):
    """sum_k clamp(rint(v_k 2^f)) 2^-f, in numpy: what every round must decode to."""
    acc = np.zeros(grads[0].shape, dtype=np.int64)
    for g in grads:
        r = np.rint(g.astype(np.float32) * np.float32(2.0 ** f))
        r = np.where(np.isnan(r), 0, r)
        acc += np.clip(r.astype(np.float64), -clamp, clamp).astype(np.int64)     # exact bound, also above 2^24
    return (acc.astype(np.float32) * np.float32(2.0 ** -f)).astype(np.float32)


# ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("name,batch", [("C1", 3), ("C2", 3), ("C3", 2), ("C4", 2), ("C5", 2)])
def test_transforms_on_every_prime_set(name, batch):
    cfg = CONFIGS[name]
    o = O.Oracle(cfg.log2_n, cfg.q, 0, 21, 0, 1, cfg.seed)
    ctx = make_ctx(cfg.log2_n, cfg.q, 0, seed=cfg.seed)
    perm = ctx.index_map()
    assert sorted(perm.tolist()) == list(range(cfg.N))
    for i in range(cfg.L):
        assert ctx.root(i) == o.psi[i]
    polys = o.bench_polys(batch)
    d = dzeros(batch * cfg.L * cfg.N)
    ctx.bench_polys(d, batch)
    assert np.array_equal(to_host(d, polys.shape), polys), "uniform sampling"
    ctx.ntt_forward(d, batch)
    assert np.array_equal(to_host(d, polys.shape), to_eval(o, perm, polys)), "forward transform"
    ctx.ntt_inverse(d, batch)
    assert np.array_equal(to_host(d, polys.shape), polys), "inverse transform"
    # inverse alone, from oracle-made evaluation data with extreme values
    edge = polys.copy()
    for i in range(cfg.L):
        edge[0, i, :4] = [0, 1, cfg.q[i] - 1, cfg.q[i] - 2]
    d = to_dev(to_eval(o, perm, edge).reshape(-1))
    ctx.ntt_inverse(d, batch)
    assert np.array_equal(to_host(d, polys.shape), edge), "inverse of oracle data"
    ctx.close()


def test_transform_full_batch_C5_roundtrip_and_samples():
    """The micro-benchmark configuration at full size (64 x 16 polynomials of 65536): the
    round trip returns the input, and sampled polynomials match the oracle's transform."""
    cfg = CONFIGS["C5"]
    o = O.Oracle(cfg.log2_n, cfg.q, 0, 21, 0, 1, cfg.seed)
    ctx = make_ctx(cfg.log2_n, cfg.q, 0, seed=cfg.seed)
    perm = ctx.index_map()
    Bn = cfg.batch
    d = dzeros(Bn * cfg.L * cfg.N)
    ctx.bench_polys(d, Bn)
    ref = d.clone()
    ctx.ntt_forward(d, Bn)
    fwd = to_host(d, (Bn, cfg.L, cfg.N))
    for (b, i) in [(0, 0), (17, 5), (63, 15)]:
        x = O.sample_uniform(cfg.seed, O.DOM_BENCH, i, 0, 0, b, cfg.q[i], cfg.N)
        assert np.array_equal(to_host(ref, (Bn, cfg.L, cfg.N))[b, i], x)
        assert np.array_equal(fwd[b, i], O.ntt_forward(x, cfg.q[i], o.psi[i])[perm]), (b, i)
    assert not torch.equal(d, ref)
    ctx.ntt_inverse(d, Bn)
    assert torch.equal(d, ref), "round trip"
    ctx.close()


# ------------------------------------------------------------------------------------------
def run_calls_and_compare(cfg, o, ctx, perm, keys, members, group, grads, ct_base=0, check_cts=True):
    """The per-call path for one group; every intermediate object is compared."""
    L, N = o.L, o.N
    n_values = grads[members[0]].size
    C_ = (n_values + N - 1) // N
    opk, dpk = keys.group_pk(members, perm)
    dagg, oagg = None, None
    for k in members:
        dgrad = to_dev(grads[k])
        dpt = dzeros(C_ * N)
        ctx.encode(dgrad, n_values, dpt, C_)
        opt = o.encode(grads[k])
        assert np.array_equal(to_host(dpt, (C_, N)), opt), f"plaintext of party {k}"
        dct = dzeros(C_ * 2 * L * N)
        ctx.encrypt(dpk, dpt, C_, k, group, ct_base, dct)
        oct_ = o.encrypt(opk, opt, k, group, ct_base)
        if check_cts:
            assert np.array_equal(to_host(dct, oct_.shape), to_eval(o, perm, oct_)), f"ciphertexts of party {k}"
        if dagg is None:
            dagg, oagg = dct, oct_
        else:
            ctx.add(dagg, dct, C_)
            oagg = o.add(oagg, oct_)
    assert np.array_equal(to_host(dagg, oagg.shape), to_eval(o, perm, oagg)), "aggregate"
    dshares, oshares = [], []
    for k in members:
        dsh = dzeros(C_ * L * N)
        ctx.partial_decrypt(keys.sk[k], dagg, C_, k, group, ct_base, dsh)
        osh = o.partial_decrypt(keys.osk[k], oagg, k, group, ct_base)
        assert np.array_equal(to_host(dsh, osh.shape), to_eval(o, perm, osh)), f"share of party {k}"
        dshares.append(dsh)
        oshares.append(osh)
    dout = dzeros(C_ * N)
    ctx.combine(dagg, dshares, C_, dout)
    oout = o.combine(oagg, oshares)
    assert np.array_equal(to_host(dout, (C_, N)), oout), "combined plaintext"
    dres = torch.zeros(n_values, dtype=torch.float32, device=DEV)
    ctx.decode(dout, C_, n_values, dres)
    ores = o.decode(oout, n_values)
    assert np.array_equal(dres.cpu().numpy(), ores), "decoded sum"
    expect = fixed_point_sum([grads[k] for k in members], cfg.frac_bits, o.encode_clamp())
    assert np.array_equal(ores, expect), "oracle decodes to the fixed-point sum"
    return dpk, opk, to_host(dagg, oagg.shape)


def run_fused(ctx, o, dpk, keys, members, group, grads, n_values):
    K = len(members)
    nbytes = ctx.round_scratch_bytes(K, 1, n_values)
    scratch = dzeros(nbytes // 8)
    out = torch.zeros(n_values, dtype=torch.float32, device=DEV)
    dgr = [to_dev(grads[k]) for k in members]
    ctx.round_group(dpk, [keys.sk[k] for k in members], dgr, members, group, n_values, out, scratch, nbytes)
    torch.cuda.synchronize()
    return out.cpu().numpy(), scratch


def test_round_C1_every_coefficient():
    cfg = CONFIGS["C1"]
    o, ctx, perm = make_pair(cfg)
    grads = cfg.gradients()
    keys = Keys(o, ctx, perm, range(cfg.parties))
    members = cfg.groups()[0]
    assert members == [0, 1, 2, 3]
    dpk, opk, agg = run_calls_and_compare(cfg, o, ctx, perm, keys, members, 0, grads)
    res, scratch = run_fused(ctx, o, dpk, keys, members, 0, grads, cfg.n_values)
    assert np.array_equal(res, fixed_point_sum(grads, cfg.frac_bits, o.encode_clamp()))
    # the fused path leaves the same aggregate in its scratch as the per-call path built
    K, C_, L, N = 4, cfg.C, cfg.L, cfg.N
    s = to_host(scratch)
    assert np.array_equal(s[K * C_ * 2 * L * N:(K + 1) * C_ * 2 * L * N].reshape(agg.shape), agg)
    ctx.close()


def test_round_C2_two_groups_every_coefficient_and_all_groups_fused():
    cfg = CONFIGS["C2"]
    o, ctx, perm = make_pair(cfg)
    grads = cfg.gradients()
    keys = Keys(o, ctx, perm, range(cfg.parties))
    groups = cfg.groups()
    assert len(groups) == 16 and all(len(g) == 5 for g in groups)
    for g in (0, 9):
        run_calls_and_compare(cfg, o, ctx, perm, keys, groups[g], g, grads)
    for g, members in enumerate(groups):
        opk, dpk = keys.group_pk(members, perm, check=(g % 5 == 0))
        res, _ = run_fused(ctx, o, dpk, keys, members, g, grads, cfg.n_values)
        expect = fixed_point_sum([grads[k] for k in members], cfg.frac_bits, o.encode_clamp())
        assert np.array_equal(res, expect), f"group {g}"
        if g in (3, 15):      # the oracle's whole round for these groups
            ores, _ = o.round_group(opk, [keys.osk[k] for k in members], [grads[k] for k in members], members, g)
            assert np.array_equal(res, ores)
    ctx.close()


@pytest.mark.parametrize("name,group_index,sample", [("C3", 11, (0, 76, 152)), ("C4", 0, (0, 341, 683))])
def test_round_full_size_sampled_against_oracle(name, group_index, sample):
    """One whole group at the configuration's full size in the launch shape the benchmark
    times; the oracle recomputes the sampled ciphertext indices one by one, and the decoded
    result is checked everywhere against the fixed-point sum (holds at any size)."""
    cfg = CONFIGS[name]
    o, ctx, perm = make_pair(cfg)
    groups = cfg.groups()
    members = groups[group_index]
    K, L, N, C_ = len(members), cfg.L, cfg.N, cfg.C
    all_grads = cfg.gradients()
    grads = {k: all_grads[k] for k in members}
    del all_grads
    keys = Keys(o, ctx, perm, members)
    opk, dpk = keys.group_pk(members, perm)
    res, scratch = run_fused(ctx, o, dpk, keys, members, group_index, grads, cfg.n_values)
    expect = fixed_point_sum([grads[k] for k in members], cfg.frac_bits, o.encode_clamp())
    assert np.array_equal(res, expect)
    LN = L * N
    cts = scratch[:K * C_ * 2 * LN].view(K, C_, 2 * LN)
    agg = scratch[K * C_ * 2 * LN:(K + 1) * C_ * 2 * LN].view(C_, 2 * LN)
    shares = scratch[(K + 1) * C_ * 2 * LN:(K + 1) * C_ * 2 * LN + K * C_ * LN].view(K, C_, LN)
    for c in sample:
        lo, hi = c * N, min((c + 1) * N, cfg.n_values)
        oagg = None
        for m, k in enumerate(members):
            oct_ = o.encrypt(opk, o.encode(grads[k][lo:hi]), k, group_index, c)
            assert np.array_equal(to_host(cts[m, c], (1, 2, L, N)), to_eval(o, perm, oct_)), (c, k)
            oagg = oct_ if oagg is None else o.add(oagg, oct_)
        assert np.array_equal(to_host(agg[c], (1, 2, L, N)), to_eval(o, perm, oagg)), c
        oshares = []
        for m, k in enumerate(members):
            osh = o.partial_decrypt(keys.osk[k], oagg, k, group_index, c)
            assert np.array_equal(to_host(shares[m, c], (1, L, N)), to_eval(o, perm, osh)), (c, k)
            oshares.append(osh)
        odec = o.decode(o.combine(oagg, oshares), hi - lo)
        assert np.array_equal(res[lo:hi], odec), c
    ctx.close()


# ------------------------------------------------------------------------------------------
def test_edge_cases_ragged_tail_clamp_and_extreme_ids():
    q = O.find_primes(54, 11, 2)
    cfg = toy_config(11, q, 12289, parties=3, n_values=2 * 2048 + 5, frac_bits=6)
    o, ctx, perm = make_pair(cfg, max_group=3)
    rng = np.random.default_rng(11)
    grads = {k: rng.normal(0, 8.0, cfg.n_values).astype(np.float32) for k in (0, 40000, 65535)}
    grads[0][:10] = [np.nan, np.inf, -np.inf, 1e30, -1e30, 0.5 / 64, 1.5 / 64, -2.5 / 64, 31.99, -0.0]
    members = [0, 40000, 65535]
    keys = Keys(o, ctx, perm, members)
    dpk, opk, _ = run_calls_and_compare(cfg, o, ctx, perm, keys, members, 65535, grads, ct_base=2 ** 32 - 4)
    res, _ = run_fused(ctx, o, dpk, keys, members, 65535, grads, cfg.n_values)
    assert np.array_equal(res, fixed_point_sum([grads[k] for k in members], 6, o.encode_clamp()))
    # a single value, a single party
    one = {0: np.array([0.734], dtype=np.float32)}
    cfg1 = toy_config(11, q, 12289, parties=1, n_values=1, frac_bits=6)
    run_calls_and_compare(cfg1, o, ctx, perm, keys, [0], 0, one)
    # empty requests are accepted and touch nothing
    guard = dzeros(16)
    ctx.encode(None, 0, guard, 0)
    ctx.encrypt(dpk, guard, 0, 0, 0, 0, guard)
    ctx.add(guard, guard, 0)
    ctx.partial_decrypt(keys.sk[0], guard, 0, 0, 0, 0, guard)
    ctx.ntt_forward(guard, 0)
    torch.cuda.synchronize()
    assert int(guard.abs().sum()) == 0
    # requests outside the documented ranges are refused on the host
    for bad in (lambda: ctx.encrypt(dpk, guard, 1, 70000, 0, 0, guard),
                lambda: ctx.encrypt(dpk, guard, 2, 0, 0, 2 ** 32 - 1, guard),
                lambda: ctx.combine(guard, [guard] * 4, 1, guard),
                lambda: ctx.encode(guard, 4097, guard, 2)):
        with pytest.raises(B.D2mheError) as ei:
            bad()
        assert ei.value.status == B.ERR_RANGE
    ctx.close()


@pytest.mark.parametrize("name", ["C1", "C2", "C3"])
def test_coefficient_form_export_equals_the_oracles_objects(name):
    """The library's messages are in evaluation form; d2mhe_ntt_inverse turns them into the coefficient form
    the paper's formulas are written in.  A public key, fresh ciphertexts, their sum and a decryption share go
    through it and are compared with the oracle's coefficient-form objects directly (no oracle transform)."""
    cfg = CONFIGS[name]
    o, ctx, perm = make_pair(cfg)
    L, N = cfg.L, cfg.N
    n_values = 2 * N + 5
    members = cfg.groups()[1 if name != "C1" else 0]
    grads = {k: g[:n_values] for k, g in enumerate(cfg.gradients(n_values=n_values)) if k in members}
    keys = Keys(o, ctx, perm, members, check=False)
    opk, dpk = keys.group_pk(members, perm, check=False)
    C_ = 3
    coeff = lambda t, B: (ctx.ntt_inverse(t, B), to_host(t))[1]
    pkv = dpk.view(2, 2, L * N)[:, 0].contiguous()                 # values of (p0, p1) without the quotients
    assert np.array_equal(coeff(pkv, 2).reshape(2, L, N), opk), "collective public key"
    dagg, oagg = None, None
    for k in members:
        dpt = dzeros(C_ * N)
        ctx.encode(to_dev(grads[k]), n_values, dpt, C_)
        dct = dzeros(C_ * 2 * L * N)
        ctx.encrypt(dpk, dpt, C_, k, 1, 7, dct)
        oct_ = o.encrypt(opk, o.encode(grads[k]), k, 1, 7)
        if dagg is None:
            dagg, oagg = dct.clone(), oct_
        else:
            ctx.add(dagg, dct, C_)
            oagg = o.add(oagg, oct_)
        assert np.array_equal(coeff(dct, 2 * C_).reshape(oct_.shape), oct_), f"fresh ciphertexts of party {k}"
    k = members[-1]
    dsh = dzeros(C_ * L * N)
    ctx.partial_decrypt(keys.sk[k], dagg, C_, k, 1, 7, dsh)
    osh = o.partial_decrypt(keys.osk[k], oagg, k, 1, 7)
    assert np.array_equal(coeff(dsh, C_).reshape(osh.shape), osh), "decryption share"
    assert np.array_equal(coeff(dagg, 2 * C_).reshape(oagg.shape), oagg), "aggregate"
    ctx.close()


def test_clamp_with_a_30_bit_plaintext_modulus():
    """t just below 2^30 (the largest the library takes): the clamp bound is above 2^24 and not a float32;
    values around it, both packings."""
    log2n = 10
    t = O.find_primes(30, log2n, 1)[0]
    cfg = toy_config(log2n, O.find_primes(44, log2n, 2), t, parties=3, n_values=1024 + 9, frac_bits=0)
    o, ctx, perm = make_pair(cfg, max_group=5)        # floor(((t-1)/2)/5) = 107370700 is not a float32
    clamp = o.encode_clamp()
    assert clamp > (1 << 24) and int(np.float32(clamp)) != clamp
    up = np.nextafter(np.float32(clamp), np.float32(np.inf)) if int(np.float32(clamp)) <= clamp else np.float32(clamp)
    rng = np.random.default_rng(31)
    grads = {k: (rng.normal(0, 1.0, cfg.n_values) * clamp).astype(np.float32) for k in range(3)}
    for k in range(3):
        grads[k][:6] = [up, -up, np.inf, -np.inf, np.nextafter(up, np.float32(0)), -3.0e9]
    keys = Keys(o, ctx, perm, range(3))
    run_calls_and_compare(cfg, o, ctx, perm, keys, [0, 1, 2], 1, grads)
    C_ = cfg.C
    for k in range(3):
        dpt = dzeros(C_ * cfg.N)
        ctx.encode_coefficients(to_dev(grads[k]), cfg.n_values, dpt, C_)
        assert np.array_equal(to_host(dpt, (C_, cfg.N)), o.encode_coefficients(grads[k]))
    ctx.close()


def test_eta_and_small_prime_variants():
    """eta = 1 and eta = 32 (full words: the largest samples, |e| <= 32, which the reduction-free first stage of
    the small-input transforms is sized for) on every arithmetic back-end, incl. the longest ring with a prime just
    below 2^55 and the widest double-precision prime."""
    for (eta, bits, L, log2n) in [(1, 30, 1, 10), (32, 60, 2, 10), (7, 36, 4, 12), (32, 55, 1, 14), (32, 54, 2, 13),
                                  (32, 44, 2, 12), (32, 30, 2, 11)]:
        q = O.find_primes(bits, log2n, L)
        cfg = toy_config(log2n, q, 12289 if log2n == 10 else 65537, parties=2, n_values=(1 << log2n) + 3, frac_bits=3)
        cfg.eta = eta
        o, ctx, perm = make_pair(cfg, max_group=2)
        rng = np.random.default_rng(eta)
        grads = {k: rng.normal(0, 1.0, cfg.n_values).astype(np.float32) for k in (0, 1)}
        keys = Keys(o, ctx, perm, [0, 1])
        run_calls_and_compare(cfg, o, ctx, perm, keys, [0, 1], 2, grads)
        ctx.close()


# ------------------------------------------------------------------------------------------
def _setup_whole_round(cfg):
    o, ctx, perm = make_pair(cfg)
    groups = cfg.groups()
    grads = cfg.gradients()
    keys = Keys(o, ctx, perm, range(cfg.parties), check=False)
    pks = [keys.group_pk(g, perm, check=False) for g in groups]
    dgr = [to_dev(g) for g in grads]
    outs = [torch.zeros(cfg.n_values, dtype=torch.float32, device=DEV) for _ in groups]
    J = sum(len(g) for g in groups)
    nbytes = ctx.round_scratch_bytes(J, len(groups), cfg.n_values)
    scratch = dzeros(nbytes // 8)
    desc = ctx.make_round(groups, [p[1] for p in pks], [keys.sk[k] for k in range(cfg.parties)], dgr, outs,
                          cfg.n_values)
    return o, ctx, perm, groups, grads, keys, pks, outs, scratch, nbytes, desc, J


@pytest.mark.parametrize("name,jobs_sample,ct_sample", [("C1", [(0, 0), (0, 3)], (0, 3)),
                                                       ("C2", [(0, 0), (7, 2), (15, 4)], (0, 13, 24)),
                                                       ("C3", [(0, 0), (19, 3), (31, 6)], (0, 152))])
def test_whole_round_in_the_benchmark_launch_shape(name, jobs_sample, ct_sample):
    """All groups of a configuration in one d2mhe_round call (the launch shape bench.py times),
    with phase events.  Every group's decoded result is checked against the fixed-point sum;
    sampled fresh ciphertexts, aggregates and shares are recomputed by the oracle."""
    cfg = CONFIGS[name]
    o, ctx, perm, groups, grads, keys, pks, outs, scratch, nbytes, desc, J = _setup_whole_round(cfg)
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(5)]
    for e in evs:
        e.record()
    for rep in range(2):         # twice: the second run overwrites the scratch of the first
        ctx.round(desc, scratch, nbytes, [e.cuda_event for e in evs], torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    assert all(evs[i].elapsed_time(evs[i + 1]) > 0 for i in range(4))
    clamp = o.encode_clamp()
    for gi, g in enumerate(groups):
        expect = fixed_point_sum([grads[k] for k in g], cfg.frac_bits, clamp)
        assert np.array_equal(outs[gi].cpu().numpy(), expect), f"group {gi}"
    L, N, C_, G = cfg.L, cfg.N, cfg.C, len(groups)
    LN = L * N
    offs = np.cumsum([0] + [len(g) for g in groups])
    cts = scratch[:J * C_ * 2 * LN].view(J, C_, 2 * LN)
    agg = scratch[J * C_ * 2 * LN:(J + G) * C_ * 2 * LN].view(G, C_, 2 * LN)
    shares = scratch[(J + G) * C_ * 2 * LN:(J + G) * C_ * 2 * LN + J * C_ * LN].view(J, C_, LN)
    for (gi, mi) in jobs_sample:
        g = groups[gi]
        opk = pks[gi][0]
        for c in ct_sample:
            lo, hi = c * N, min((c + 1) * N, cfg.n_values)
            oagg = None
            for m, k in enumerate(g):
                oct_ = o.encrypt(opk, o.encode(grads[k][lo:hi]), k, gi, c)
                if m == mi:
                    assert np.array_equal(to_host(cts[offs[gi] + m, c], (1, 2, L, N)), to_eval(o, perm, oct_)), (gi, m, c)
                oagg = oct_ if oagg is None else o.add(oagg, oct_)
            assert np.array_equal(to_host(agg[gi, c], (1, 2, L, N)), to_eval(o, perm, oagg)), (gi, c)
            osh = o.partial_decrypt(keys.osk[g[mi]], oagg, g[mi], gi, c)
            assert np.array_equal(to_host(shares[offs[gi] + mi, c], (1, L, N)), to_eval(o, perm, osh)), (gi, mi, c)
    ctx.close()


def test_whole_round_argument_checks():
    cfg = CONFIGS["C1"]
    o, ctx, perm, groups, grads, keys, pks, outs, scratch, nbytes, desc, J = _setup_whole_round(cfg)
    with pytest.raises(B.D2mheError) as ei:
        ctx.round(desc, scratch, nbytes - 8)
    assert ei.value.status == B.ERR_WORKSPACE
    bad = ctx.make_round([[0, 1, 2, 3, 0]], [pks[0][1]], [keys.sk[k] for k in range(4)], [to_dev(g) for g in grads],
                         outs, cfg.n_values)
    with pytest.raises(B.D2mheError) as ei:           # 5 members > max_group = 4
        ctx.round(bad, scratch, nbytes * 2)
    assert ei.value.status == B.ERR_RANGE
    sks, dgr = [keys.sk[k] for k in range(4)], [to_dev(g) for g in grads]
    for groups_, pks_, outs_, status in (([], [], [], B.ERR_RANGE),                           # no group
                                         ([[]], [pks[0][1]], outs, B.ERR_RANGE),               # an empty group
                                         ([[0, 1, 7]], [pks[0][1]], outs, B.ERR_NULL)):        # a member without key
        with pytest.raises(B.D2mheError) as ei:
            ctx.round(ctx.make_round(groups_, pks_, sks, dgr, outs_, cfg.n_values), scratch, nbytes)
        assert ei.value.status == status
    # ids that would alias Philox streams: a group id beyond 16 bits, two groups with one id, a member twice
    for groups_, gids in (([[0, 1, 2, 3]], [70000]), ([[0, 1], [2, 3]], [5, 5]), ([[0, 1, 1]], None)):
        with pytest.raises(B.D2mheError) as ei:
            ctx.round(ctx.make_round(groups_, [pks[0][1]] * len(groups_), sks, dgr, outs * len(groups_), cfg.n_values,
                                     group_ids=gids), scratch, nbytes)
        assert ei.value.status == B.ERR_RANGE
    with pytest.raises(B.D2mheError) as ei:
        ctx.round_group(pks[0][1], [sks[0], sks[1], sks[0]], [dgr[0], dgr[1], dgr[0]], [0, 1, 0], 0, cfg.n_values, outs[0],
                        scratch, nbytes)
    assert ei.value.status == B.ERR_RANGE
    # a round over zero values is accepted and writes nothing
    before = outs[0].clone()
    ctx.round(ctx.make_round([[0, 1, 2, 3]], [pks[0][1]], sks, dgr, outs, 0), scratch, nbytes)
    torch.cuda.synchronize()
    assert torch.equal(outs[0], before)
    ctx.close()


def test_global_key_variant_through_the_per_call_interface():
    """The other reading of Sec. 4.1 ("all nodes encrypt under the same public key"): one collective
    key over all P nodes, every node encrypts once, node i sums the ciphertexts of its closed
    neighbourhood, and the decryption of that sum takes a share from every one of the P nodes.
    The library is set-generic, so this is expressible with the per-call entry points; every object
    is compared with the oracle's."""
    from oracle import oracle as O
    from paper_2207_04604_amd.synth import toy_config
    cfg = toy_config(10, O.find_primes(36, 10, 2), 65537, 6, 1500, frac_bits=8, topology="circulant", offsets=(1,))
    P = cfg.parties
    o, ctx, perm = make_pair(cfg, max_group=P)
    L, N, n, C_ = o.L, o.N, cfg.n_values, cfg.C
    grads = cfg.gradients()
    keys = Keys(o, ctx, perm, range(P), check=False)
    everyone = list(range(P))
    opk, dpk = keys.group_pk(everyone, perm)
    dcts, octs = [], []
    for k in everyone:                                   # one encryption per node, group id 0
        dpt = dzeros(C_ * N)
        ctx.encode(to_dev(grads[k]), n, dpt, C_)
        dct = dzeros(C_ * 2 * L * N)
        ctx.encrypt(dpk, dpt, C_, k, 0, 0, dct)
        oct_ = o.encrypt(opk, o.encode(grads[k]), k, 0, 0)
        assert np.array_equal(to_host(dct, oct_.shape), to_eval(o, perm, oct_))
        dcts.append(dct)
        octs.append(oct_)
    for i, hood in enumerate(cfg.groups()):              # node i's closed neighbourhood
        dagg, oagg = dcts[hood[0]].clone(), octs[hood[0]]
        for j in hood[1:]:
            ctx.add(dagg, dcts[j], C_)
            oagg = o.add(oagg, octs[j])
        dshares, oshares = [], []
        for k in everyone:                               # shares from all P nodes, indexed by the receiver
            dsh = dzeros(C_ * L * N)
            ctx.partial_decrypt(keys.sk[k], dagg, C_, k, 1 + i, 0, dsh)
            osh = o.partial_decrypt(keys.osk[k], oagg, k, 1 + i, 0)
            assert np.array_equal(to_host(dsh, osh.shape), to_eval(o, perm, osh))
            dshares.append(dsh)
            oshares.append(osh)
        dout = dzeros(C_ * N)
        ctx.combine(dagg, dshares, C_, dout)
        assert np.array_equal(to_host(dout, (C_, N)), o.combine(oagg, oshares))
        dres = torch.zeros(n, dtype=torch.float32, device=DEV)
        ctx.decode(dout, C_, n, dres)
        expect = fixed_point_sum([grads[k] for k in hood], cfg.frac_bits, o.encode_clamp())
        assert np.array_equal(dres.cpu().numpy(), expect), f"node {i}"
    ctx.close()


def test_largest_group_of_64_members():
    """The largest neighbourhood the library accepts (64 members): per-call objects against the oracle, the fused
    round for that group and for two such groups in one call (128 jobs: two launches per phase), and one more
    member refused on the host."""
    q = O.find_primes(36, 10, 2)
    cfg = toy_config(10, q, 65537, parties=64, n_values=1024 + 19, frac_bits=6)
    o, ctx, perm = make_pair(cfg, max_group=64)
    assert o.encode_clamp() == 32768 // 64
    rng = np.random.default_rng(64)
    grads = {k: rng.normal(0, 3.0, cfg.n_values).astype(np.float32) for k in range(64)}
    grads[5][:3] = [1e9, -1e9, np.nan]                  # clamped: 64 such terms still cannot wrap
    members = list(range(64))
    keys = Keys(o, ctx, perm, members, check=False)
    dpk, opk, _ = run_calls_and_compare(cfg, o, ctx, perm, keys, members, 9, grads, check_cts=False)
    res, _ = run_fused(ctx, o, dpk, keys, members, 9, grads, cfg.n_values)
    expect = fixed_point_sum([grads[k] for k in members], 6, o.encode_clamp())
    assert np.array_equal(res, expect)
    # two groups over the same 64 parties (different group ids, hence different randomness), one call
    outs = [torch.zeros(cfg.n_values, dtype=torch.float32, device=DEV) for _ in range(2)]
    nbytes = ctx.round_scratch_bytes(128, 2, cfg.n_values)
    scratch = dzeros(nbytes // 8)
    rev = members[::-1]
    desc = ctx.make_round([members, rev], [dpk, dpk], [keys.sk[k] for k in members], [to_dev(grads[k]) for k in members],
                          outs, cfg.n_values, group_ids=[9, 10])
    ctx.round(desc, scratch, nbytes)
    torch.cuda.synchronize()
    assert np.array_equal(outs[0].cpu().numpy(), expect) and np.array_equal(outs[1].cpu().numpy(), expect)
    L, N, C_ = o.L, o.N, cfg.C
    agg = to_host(scratch[128 * C_ * 2 * L * N:130 * C_ * 2 * L * N], (2, C_, 2, L, N))
    oagg = None
    for k in rev:
        oct_ = o.encrypt(opk, o.encode(grads[k]), k, 10, 0)
        oagg = oct_ if oagg is None else o.add(oagg, oct_)
    assert np.array_equal(agg[1], to_eval(o, perm, oagg))
    guard = dzeros(16)
    with pytest.raises(B.D2mheError) as ei:
        ctx.combine(guard, [guard] * 65, 1, guard)
    assert ei.value.status == B.ERR_RANGE
    ctx.close()
