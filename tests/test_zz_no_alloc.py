"""d2mhe_round_group_static (the entry point that allocates nothing) against d2mhe_round_group,
through the C ABI on a real MI355X: bit-identical decoded sums on two calls in a row, the second
with a smaller input, so that whatever the first call left in the library's scratch array must not
leak into the second."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from oracle import oracle as O
from paper_2207_04604_amd import binding as B
from paper_2207_04604_amd.synth import toy_config

from gpu_util import DEV, Keys, dzeros, make_pair, to_dev


def _both(ctx, dpk, keys, members, group, grads, n_values):
    """(existing entry point's output, new entry point's output) for one group."""
    K = len(members)
    sks = [keys.sk[k] for k in members]
    dgr = [to_dev(grads[k][:n_values]) for k in members]
    nbytes = ctx.round_scratch_bytes(K, 1, n_values)
    assert nbytes <= B.STATIC_SCRATCH_BYTES
    scratch = dzeros(nbytes // 8)
    ref = torch.zeros(n_values, dtype=torch.float32, device=DEV)
    ctx.round_group(dpk, sks, dgr, members, group, n_values, ref, scratch, nbytes)
    got = torch.full((n_values,), float("nan"), dtype=torch.float32, device=DEV)
    ctx.round_group_static(dpk, sks, dgr, members, group, n_values, got)
    torch.cuda.synchronize()
    return ref.cpu().numpy(), got.cpu().numpy()


def test_static_scratch_round_equals_round_group_twice_second_smaller():
    q = O.find_primes(36, 12, 3)
    cfg = toy_config(12, q, 65537, parties=5, n_values=6 * 4096 + 321, frac_bits=10)
    o, ctx, perm = make_pair(cfg, max_group=5)
    rng = np.random.default_rng(2207)
    grads = {k: rng.normal(0, 0.01, cfg.n_values).astype(np.float32) for k in range(5)}
    keys = Keys(o, ctx, perm, range(5), check=False)
    members = [0, 1, 2, 3, 4]
    _, dpk = keys.group_pk(members, perm, check=False)
    # first call: 7 ciphertext indices, 5 members
    ref, got = _both(ctx, dpk, keys, members, 3, grads, cfg.n_values)
    assert np.array_equal(ref, got), "first call"
    clamp = o.encode_clamp()
    acc = sum(np.clip(np.rint(grads[k] * np.float32(1024.0)), -clamp, clamp).astype(np.int64) for k in members)
    assert np.array_equal(got, acc.astype(np.float32) * np.float32(2.0 ** -10)), "first call decodes to the fixed-point sum"
    # second call: smaller input (2 ciphertext indices, ragged tail) and fewer members, other group id
    small = [1, 3, 4]
    _, dpk3 = keys.group_pk(small, perm, check=False)
    ref2, got2 = _both(ctx, dpk3, keys, small, 9, grads, 4096 + 77)
    assert np.array_equal(ref2, got2), "second, smaller call"
    # and the oracle's whole round for the second call
    opk3 = o.aggregate_pk([keys.opk0[k] for k in small])
    ores, _ = o.round_group(opk3, [keys.osk[k] for k in small], [grads[k][:4096 + 77] for k in small], small, 9)
    assert np.array_equal(got2, ores)
    ctx.close()


def test_static_scratch_round_refuses_what_does_not_fit():
    q = O.find_primes(36, 12, 3)
    cfg = toy_config(12, q, 65537, parties=5, n_values=4096, frac_bits=10)
    o, ctx, perm = make_pair(cfg, max_group=5)
    keys = Keys(o, ctx, perm, range(5), check=False)
    members = [0, 1, 2, 3, 4]
    _, dpk = keys.group_pk(members, perm, check=False)
    sks = [keys.sk[k] for k in members]
    # the host checks sizes before it looks at the data: n_values for which the scratch exceeds the array
    n_fit = 1
    while ctx.round_scratch_bytes(5, 1, (n_fit + 1) * 4096) <= B.STATIC_SCRATCH_BYTES:
        n_fit += 1
    # the largest round that fits uses the array up to (nearly) its last word
    rng = np.random.default_rng(64)
    hg = {k: rng.normal(0, 0.01, n_fit * 4096).astype(np.float32) for k in members}
    ref, got = _both(ctx, dpk, keys, members, 1, hg, n_fit * 4096)
    assert np.array_equal(ref, got), "largest round that fits"
    n_big = (n_fit + 1) * 4096
    grads =[dzeros(n_big, dtype=torch.float32) for _ in members]           # full-size buffers, never read
    out = torch.zeros(n_big, dtype=torch.float32, device=DEV)
    with pytest.raises(B.D2mheError) as ei:
        ctx.round_group_static(dpk, sks, grads, members, 0, n_big, out)
    assert ei.value.status == B.ERR_WORKSPACE
    with pytest.raises(B.D2mheError) as ei:
        ctx.round_group_static(dpk, sks, grads, members, 70000, 16, out)
    assert ei.value.status == B.ERR_RANGE
    torch.cuda.synchronize()
    assert float(out.abs().sum()) == 0.0
    ctx.close()
