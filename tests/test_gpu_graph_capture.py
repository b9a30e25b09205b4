"""The fused rounds allocate nothing, synchronise nothing and clear memory with kernels only, so a caller can
capture them into a HIP graph (useful where launch latency dominates, as for the smallest workload).  Replays
are interleaved with eager work and synchronisations, with new inputs written in place before each, and every
replay is checked against the eager call on the same inputs."""
import numpy as np
import pytest
import torch

from paper_2207_04604_amd.synth import CONFIGS

from gpu_util import DEV, Keys, dzeros, make_pair, to_dev
from test_gpu_convert import RecvKeys
from test_gpu_parity import fixed_point_sum

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("convert", [False, True])
def test_round_replayed_from_a_captured_graph(convert):
    cfg = CONFIGS["C1"]
    o, ctx, perm = make_pair(cfg)
    groups, P, n = cfg.groups(), cfg.parties, cfg.n_values
    keys = Keys(o, ctx, perm, range(P), check=False)
    pks = [keys.group_pk(g, perm, check=False) for g in groups]
    grads = cfg.gradients()
    dgr = [to_dev(g) for g in grads]
    J, G = sum(len(g) for g in groups), len(groups)
    sks = [keys.sk[k] for k in range(P)]
    if convert:
        receivers = cfg.receivers()
        rk = RecvKeys(o, ctx, perm, range(P))
        R = sum(len(r) for r in receivers)
        outs = [torch.zeros(n, dtype=torch.float32, device=DEV) for _ in range(R)]
        desc = ctx.make_round(groups, [p[1] for p in pks], sks, dgr, [torch.zeros(1, dtype=torch.float32, device=DEV)] * G, n)
        conv = ctx.make_convert(desc, receivers, rk.pk, rk.sk, outs)
        nbytes = ctx.round_convert_scratch_bytes(J, G, conv.num_shares, n)
        scratch = dzeros(nbytes // 8)
        run = lambda stream: ctx.round_convert(desc, conv, scratch, nbytes, None, stream)
        out_group = [gi for gi, rs in enumerate(receivers) for _ in rs]
    else:
        outs = [torch.zeros(n, dtype=torch.float32, device=DEV) for _ in groups]
        desc = ctx.make_round(groups, [p[1] for p in pks], sks, dgr, outs, n)
        nbytes = ctx.round_scratch_bytes(J, G, n)
        scratch = dzeros(nbytes // 8)
        run = lambda stream: ctx.round(desc, scratch, nbytes, None, stream)
        out_group = list(range(G))
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        run(side.cuda_stream)                                    # warm-up on the capture stream
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=side):
            run(side.cuda_stream)
    torch.cuda.synchronize()
    clamp = o.encode_clamp()
    rng = np.random.default_rng(31)
    for rep in range(4):
        new = [rng.normal(0, 0.05 * (rep + 1), n).astype(np.float32) for _ in range(P)]
        for k in range(P):
            dgr[k].copy_(torch.from_numpy(new[k]))               # eager work between the replays
        for t in outs:
            t.zero_()
        scratch.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        replayed = [t.clone() for t in outs]
        kept = scratch.clone()
        for t in outs:
            t.zero_()
        scratch.zero_()
        run(torch.cuda.current_stream().cuda_stream)             # the same inputs, launched directly
        torch.cuda.synchronize()
        assert torch.equal(kept, scratch), f"replay {rep}: scratch"
        for i, gi in enumerate(out_group):
            expect = fixed_point_sum([new[k] for k in groups[gi]], cfg.frac_bits, clamp)
            assert np.array_equal(replayed[i].cpu().numpy(), expect), f"replay {rep}, output {i}"
            assert torch.equal(replayed[i], outs[i])
    ctx.close()
