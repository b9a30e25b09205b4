#!/usr/bin/env python3
"""Benchmark of the exchange round on one MI355X.

A step is one whole round of the hot path (encode + encrypt, homomorphic sum, decryption
shares, combine + decode) for every group of the workload, with the float32 gradients and
all keys already resident in HBM.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C2] [--no-cpu] [--no-ntt] [--no-convert] [--no-bootstrap] [--no-loop]

Beside the headline round it reports the same round with the paper's own decryption path
(key switching of every aggregate to its receivers, MBFV.Convert), a collective refresh of the
aggregates (MBFV.Bootstrap), the batched transform
micro-benchmark, and the CPU oracle timed on a bounded sample.
"""
import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0                      # MI355X HBM3E
VALU_PEAK_TOPS = 256 * 64 * 2.4e9 / 1e12   # 256 CUs x 64 lanes x 2.4 GHz = 39.3 T lane-ops/s
# VALU instructions of one butterfly in the minimal sequence of each arithmetic back-end
# (csrc/arith.hpp): doubles for moduli < 2^44, 63-bit Shoup with an approximate quotient for
# moduli < 2^55, exact Harvey butterflies for moduli < 2^61.
# HBM bytes of one launch of the dominant kernel, from rocprofv3 FETCH_SIZE / WRITE_SIZE scaled by
# a plain 512 MiB device copy (profiles/k_encrypt_C2_round_and_ntt_C5.txt); only for the
# workload that was profiled.
MEASURED_TRAFFIC_BYTES = {"C2": 73.0e6 + 393.2e6}


def ops_per_butterfly(qmax):
    if qmax < (1 << 44):
        return 8, "f64"
    if qmax < (1 << 55):
        return 16, "u64-lazy"
    return 22, "u64-harvey"


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--workload", default="C2", choices=["C1", "C2", "C3", "C4"])
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--no-ntt", action="store_true", help="skip the transform micro-benchmark")
    ap.add_argument("--no-bootstrap", action="store_true", help="skip the collective refresh (MBFV.Bootstrap)")
    ap.add_argument("--no-loop", action="store_true", help="skip the multi-iteration run (Alg. 2 loop)")
    ap.add_argument("--no-coeff", action="store_true", help="skip the round with coefficient packing")
    ap.add_argument("--no-convert", action="store_true",
                    help="skip the round with key switching to the receivers (MBFV.Convert)")
    ap.add_argument("--ntt-reps", type=int, default=20)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run plain device copies of 512 MiB (reference for the HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (all parties are simulated on one device); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2207_04604_amd import binding
    from paper_2207_04604_amd.synth import CONFIGS

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    dev = torch.device("cuda:0")
    if args.calibrate_copy:
        src = torch.zeros(512 * 1024 * 1024 // 8, dtype=torch.int64, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        ev[0].record()
        for _ in range(10):
            dst.copy_(src)
        ev[1].record()
        torch.cuda.synchronize()
        ms = ev[0].elapsed_time(ev[1]) / 10
        print(json.dumps({"copy_bytes_read": src.numel() * 8, "copy_bytes_written": src.numel() * 8, "ms": ms,
                          "GB_per_s": 2 * src.numel() * 8 / ms / 1e6}))
        return
    stream = torch.cuda.current_stream()
    sptr = stream.cuda_stream

    def dz(n, dtype=torch.int64):
        return torch.zeros(n, dtype=dtype, device=dev)

    cfg = CONFIGS[args.workload]
    N, L, C_, P = cfg.N, cfg.L, cfg.C, cfg.parties
    groups = cfg.groups()
    G, J = len(groups), sum(len(g) for g in groups)
    torch.cuda.synchronize()
    t_create = time.perf_counter()
    ctx = binding.Context(cfg.log2_n, cfg.q, cfg.t, cfg.eta, cfg.frac_bits, cfg.max_group, cfg.seed,
                          alloc=lambda n: dz(n // 8 + 2))
    torch.cuda.synchronize()
    t_create = (time.perf_counter() - t_create) * 1e3
    # ---- set-up (not part of the round: executed once per training run; reported on its own) ----
    grads_host = cfg.gradients()
    grads = [torch.from_numpy(g).to(dev) for g in grads_host]
    sks = [dz(2 * L * N) for _ in range(P)]
    pk0 = [dz(L * N) for _ in range(P)]
    for k in range(P):
        ctx.keygen_share(k, sks[k], pk0[k], sptr)
    pks = []
    for g in groups:
        pk = dz(4 * L * N)
        ctx.aggregate_pk([pk0[k] for k in g], pk, sptr)
        pks.append(pk)
    torch.cuda.synchronize()
    sev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    sev[0].record(stream)                             # the same set-up again, now with the code resident
    for k in range(P):
        ctx.keygen_share(k, sks[k], pk0[k], sptr)
    for gi, g in enumerate(groups):
        ctx.aggregate_pk([pk0[k] for k in g], pks[gi], sptr)
    sev[1].record(stream)
    torch.cuda.synchronize()
    setup_ms = sev[0].elapsed_time(sev[1])
    outs = [torch.zeros(cfg.n_values, dtype=torch.float32, device=dev) for _ in groups]
    nbytes = ctx.round_scratch_bytes(J, G, cfg.n_values)
    scratch = dz(nbytes // 8)
    desc = ctx.make_round(groups, pks, sks, grads, outs, cfg.n_values)
    torch.cuda.synchronize()

    def new_events():
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(5)]
        for e in evs:
            e.record(stream)                      # creates the underlying hipEvent_t
        return evs

    def time_rounds(run, steps):
        """The secondary legs: ms per round from `steps` rounds without events (after a short warm-up),
        and the phase split from up to 20 further rounds with an event after every phase."""
        for _ in range(min(args.warmup, 10)):
            run(None)
        torch.cuda.synchronize()
        t_0 = time.perf_counter()
        for _ in range(steps):
            run(None)
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t_0) * 1e3 / steps
        n_ev = max(1, min(steps, 20))
        evs = [new_events() for _ in range(n_ev)]
        torch.cuda.synchronize()
        for i in range(n_ev):
            run([e.cuda_event for e in evs[i]])
        torch.cuda.synchronize()
        return ms, [sum(e[i].elapsed_time(e[i + 1]) for e in evs) / n_ev for i in range(4)]

    for _ in range(args.warmup):
        ctx.round(desc, scratch, nbytes, None, sptr)
    torch.cuda.synchronize()
    # the timed region records two events around the dominant kernel's launch on every EVENT_EVERY-th
    # step (an event costs a few microseconds of idle GPU); the phase split comes from a few more
    # (untimed) steps with all five events
    EVENT_EVERY = 8
    step_events = {i: new_events()[:2] for i in range(0, args.steps, EVENT_EVERY)}
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        ev = step_events.get(i)
        ctx.round(desc, scratch, nbytes, [ev[0].cuda_event, ev[1].cuda_event, None, None, None] if ev else None, sptr)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    enc_phase_ms = sum(ev[0].elapsed_time(ev[1]) for ev in step_events.values()) / len(step_events)
    nph = max(1, min(args.steps, 20))
    phase_events = [new_events() for _ in range(nph)]
    torch.cuda.synchronize()
    for i in range(nph):
        ctx.round(desc, scratch, nbytes, [e.cuda_event for e in phase_events[i]], sptr)
    torch.cuda.synchronize()
    phase_ms = [sum(ev[i].elapsed_time(ev[i + 1]) for ev in phase_events) / nph for i in range(4)]

    # correctness of what was timed: the decoded sums equal the fixed-point sums
    clamp = ((cfg.t - 1) // 2) // cfg.max_group
    for gi in (0, G - 1):
        acc = np.zeros(cfg.n_values, dtype=np.int64)
        for k in groups[gi]:
            acc += np.clip(np.rint(grads_host[k] * np.float32(2.0 ** cfg.frac_bits)), -clamp, clamp).astype(np.int64)
        expect = acc.astype(np.float32) * np.float32(2.0 ** -cfg.frac_bits)
        if not np.array_equal(outs[gi].cpu().numpy(), expect):
            print("bench.py: decoded result differs from the fixed-point sum", file=sys.stderr)
            sys.exit(4)

    fresh = J * C_
    value = fresh / (ms_per_step * 1e-3)
    S = 16 * L * N                                    # bytes of one ciphertext
    logn = cfg.log2_n
    bf_per_transform = (N // 2) * logn
    # dominant kernel: the fused encode+encrypt kernel (3 L transforms mod q_i + 1 mod t per ciphertext)
    n_enc_launch = math.ceil(J / 112)
    enc_ms = enc_phase_ms / n_enc_launch
    enc_bf = fresh * (3 * L + 1) * bf_per_transform / n_enc_launch
    OPB, arith = ops_per_butterfly(max(cfg.q))
    enc_op_rate = enc_bf * OPB / (enc_ms * 1e-3) / 1e12
    enc_bytes = (fresh * S + fresh * 4 * N) / n_enc_launch
    # whole round, algorithmic: (4K+1) L transforms per aggregated ciphertext + (K+1) mod-t transforms
    round_bf = sum(((4 * len(g) + 1) * L + len(g) + 1) for g in groups) * C_ * bf_per_transform
    round_bytes = sum(S * (3.5 * len(g) + 1.5) for g in groups) * C_
    result = {
        "metric": "BFV gradient ciphertexts/sec (encrypt+aggregate+decrypt-share)",
        "value": value, "unit": "fresh ciphertexts/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u64" if arith != "f64" else "f64",
        "dtype_note": "residues below 2^44 are held as exact integers in doubles, wider ones as 64-bit integers",
        "data": "synthetic",
        "config": {"workload": f"{cfg.name}: N={N}, L={L}, t={cfg.t}, P={P}, G={G}, K={cfg.max_group}, C={C_}, "
                               f"{cfg.n_values} floats/party", "fresh_ciphertexts": fresh,
                   "aggregated_ciphertexts": G * C_},
        "aggregated_ct_per_s": G * C_ / (ms_per_step * 1e-3),
        "setup": {"what": f"once per training run, outside the timed round: tables and context (host + copy), "
                          f"then {P} key shares and {G} collective public keys on the GPU",
                  "create_ms": t_create, "keys_ms": setup_ms},
        "phase_ms": {"encode_encrypt": phase_ms[0], "aggregate": phase_ms[1], "shares": phase_ms[2],
                     "combine_decode": phase_ms[3]},
        "phase_ms_from": f"{nph} further steps with an event after every phase (of the timed steps every {EVENT_EVERY}th "
                         "records two events, around the dominant kernel)",
        "round_algorithmic": {"GB": round_bytes / 1e9, "GB_per_s": round_bytes / 1e9 / (ms_per_step * 1e-3),
                              "frac_hbm_peak": round_bytes / 1e9 / (ms_per_step * 1e-3) / HBM_PEAK_GBS,
                              "butterfly_Tops_per_s": round_bf * OPB / (ms_per_step * 1e-3) / 1e12,
                              "frac_valu_peak": round_bf * OPB / (ms_per_step * 1e-3) / 1e12 / VALU_PEAK_TOPS},
        "roofline": {"kernel": "k_encrypt (fused encode + encrypt)", "bound": "alu", "achieved": enc_op_rate,
                     "peak": VALU_PEAK_TOPS, "unit": f"T lane-ops/s (butterfly instructions, {OPB} per butterfly, {arith})",
                     "frac": enc_op_rate / VALU_PEAK_TOPS,
                     "traffic": MEASURED_TRAFFIC_BYTES.get(cfg.name) if n_enc_launch == 1 else None,
                     "traffic_unit": "bytes per launch (rocprofv3 FETCH_SIZE + WRITE_SIZE, copy-calibrated)",
                     "algorithmic_bytes": enc_bytes, "avg_launch_ms": enc_ms,
                     "hbm_algorithmic_GB_per_s": enc_bytes / 1e9 / (enc_ms * 1e-3),
                     "hbm_frac": enc_bytes / 1e9 / (enc_ms * 1e-3) / HBM_PEAK_GBS},
    }

    # ---- the same round with coefficient packing (value j of a ciphertext is coefficient j): an
    # addition-only workload does not need the slot structure, so both transforms modulo t go away
    if not args.no_coeff:
        pdesc = ctx.make_round(groups, pks, sks, grads, outs, cfg.n_values, packing=1)
        psteps = max(1, min(args.steps, 100))
        for o_ in outs:
            o_.zero_()
        pms, pphase = time_rounds(lambda ev: ctx.round(pdesc, scratch, nbytes, ev, sptr), psteps)
        for gi in (0, G - 1):
            acc = np.zeros(cfg.n_values, dtype=np.int64)
            for k in groups[gi]:
                acc += np.clip(np.rint(grads_host[k] * np.float32(2.0 ** cfg.frac_bits)), -clamp, clamp).astype(np.int64)
            if not np.array_equal(outs[gi].cpu().numpy(), acc.astype(np.float32) * np.float32(2.0 ** -cfg.frac_bits)):
                print("bench.py: coefficient-packed result differs from the fixed-point sum", file=sys.stderr)
                sys.exit(8)
        result["coefficient_packing_round"] = {
            "what": "the whole round with value j of a ciphertext as coefficient j (no transform modulo t in "
                    "encode or decode); same sums",
            "ms_per_step": pms, "steps": psteps, "fresh_ct_per_s": fresh / (pms * 1e-3),
            "phase_ms": {"encode_encrypt": pphase[0], "aggregate": pphase[1], "shares": pphase[2],
                         "combine_decode": pphase[3]}}

    # ---- training iterations (Alg. 2): round with fresh ciphertext indices, then every node's
    # float step (average over its neighbourhood, local gradient step) on its own weights
    if not args.no_loop:
        owner = cfg.receivers()
        node_group = {i: gi for gi, rs in enumerate(owner) for i in rs}
        T_it = 5
        weights = [g.clone() for g in grads]
        descs = [ctx.make_round(groups, pks, sks, weights, outs, cfg.n_values, ct_base=it * C_) for it in range(T_it)]
        le = [torch.cuda.Event(enable_timing=True) for _ in range(2)]

        def iterate():
            for it in range(T_it):
                ctx.round(descs[it], scratch, nbytes, None, sptr)
                for i in range(P):
                    gi = node_group[i]
                    binding.average_update(outs[gi], len(groups[gi]), grads[i], 0.01, cfg.n_values, weights[i], sptr)

        iterate()
        torch.cuda.synchronize()
        le[0].record(stream)
        iterate()
        le[1].record(stream)
        torch.cuda.synchronize()
        result["training_iterations"] = {
            "what": f"{T_it} iterations of Alg. 2 on the workload: encrypted round (collective decryption) with "
                    f"ciphertext indices it*C.., then {P} float steps w = sum/K - gamma*g",
            "ms_per_iteration": le[0].elapsed_time(le[1]) / T_it}
        ctx.round(desc, scratch, nbytes, None, sptr)          # leave the scratch as the headline round left it
        torch.cuda.synchronize()

    # ---- MBFV.Bootstrap: the members of group 0 refresh all G*C aggregates the round left in the
    # scratch (same work for each; the first C are group 0's own and are checked after the refresh)
    if not args.no_bootstrap:
        LN = L * N
        nct = G * C_
        agg = scratch[J * C_ * 2 * LN:(J + G) * C_ * 2 * LN]
        g0 = groups[0]
        alpha = dz(nct * LN)
        bshares = [dz(nct * 2 * LN) for _ in g0]
        fresh_ct = dz(nct * 2 * LN)

        def refresh():
            ctx.bootstrap_alpha(0, 0, nct, alpha, sptr)
            for k, sh in zip(g0, bshares):
                ctx.bootstrap_share(sks[k], agg, alpha, nct, k, 0, 0, sh, sptr)
            ctx.bootstrap_combine(agg, alpha, bshares, nct, fresh_ct, sptr)

        refresh()
        torch.cuda.synchronize()
        bsteps = max(1, min(args.steps, 10))
        be = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        be[0].record(stream)
        for _ in range(bsteps):
            refresh()
        be[1].record(stream)
        torch.cuda.synchronize()
        bms = be[0].elapsed_time(be[1]) / bsteps
        # the refreshed aggregates of group 0 decrypt to the same sums
        psh = [dz(C_ * LN) for _ in g0]
        for k, sh in zip(g0, psh):
            ctx.partial_decrypt(sks[k], fresh_ct, C_, k, 0, 0, sh, sptr)
        bpt = dz(C_ * N)
        ctx.combine(fresh_ct, psh, C_, bpt, sptr)
        bout = torch.zeros(cfg.n_values, dtype=torch.float32, device=dev)
        ctx.decode(bpt, C_, cfg.n_values, bout, sptr)
        torch.cuda.synchronize()
        if not torch.equal(bout, outs[0]):
            print("bench.py: refreshed ciphertexts decrypt to something else", file=sys.stderr)
            sys.exit(7)
        result["bootstrap"] = {"what": f"collective refresh (Eq. (3)) of {nct} ciphertexts by {len(g0)} members: "
                                       "common polynomial, one share per member, refreshed ciphertext",
                               "ms": bms, "refreshed_ct_per_s": nct / (bms * 1e-3)}
        del alpha, bshares, fresh_ct, psh

    # ---- the same round with MBFV.Convert: every node receives the sum of its closed neighbourhood
    # under its own key (three transforms per limb and share instead of one, two polynomials per share)
    if not args.no_convert:
        receivers = cfg.receivers()
        R = sum(len(r) for r in receivers)
        rsk = [dz(2 * L * N) for _ in range(P)]
        rpk = [dz(4 * L * N) for _ in range(P)]
        for k in range(P):
            ctx.receiver_keygen(k, rsk[k], rpk[k], sptr)
        routs = [torch.zeros(cfg.n_values, dtype=torch.float32, device=dev) for _ in range(R)]
        conv = ctx.make_convert(desc, receivers, rpk, rsk, routs)
        cbytes = ctx.round_convert_scratch_bytes(J, G, conv.num_shares, cfg.n_values)
        del scratch
        cscratch = dz(cbytes // 8)
        csteps = max(1, min(args.steps, 100))
        cms, cphase = time_rounds(lambda ev: ctx.round_convert(desc, conv, cscratch, cbytes, ev, sptr), csteps)
        ri = 0
        for gi in range(G):
            for _ in receivers[gi]:
                if gi in (0, G - 1):
                    acc = np.zeros(cfg.n_values, dtype=np.int64)
                    for k in groups[gi]:
                        acc += np.clip(np.rint(grads_host[k] * np.float32(2.0 ** cfg.frac_bits)), -clamp, clamp).astype(np.int64)
                    if not np.array_equal(routs[ri].cpu().numpy(), acc.astype(np.float32) * np.float32(2.0 ** -cfg.frac_bits)):
                        print("bench.py: converted result differs from the fixed-point sum", file=sys.stderr)
                        sys.exit(6)
                ri += 1
        result["convert_round"] = {
            "what": "encode+encrypt, sum, conversion shares towards every receiver (Eq. (1)), "
                    "converted ciphertext + single-key decryption + decode (Eq. (2))",
            "receivers": R, "conversion_shares": conv.num_shares, "ms_per_step": cms, "steps": csteps,
            "fresh_ct_per_s": fresh / (cms * 1e-3),
            "phase_ms": {"encode_encrypt": cphase[0], "aggregate": cphase[1], "convert_shares": cphase[2],
                         "combine_decrypt_decode": cphase[3]}}
        del cscratch

    # ---- transform micro-benchmark: forward + inverse, N = 65536, 16 limbs, batch 64 ------
    if not args.no_ntt:
        c5 = CONFIGS["C5"]
        nctx = binding.Context(c5.log2_n, c5.q, 0, seed=c5.seed, alloc=lambda n: dz(n // 8 + 2))
        polys = dz(c5.batch * c5.L * c5.N)
        nctx.bench_polys(polys, c5.batch, sptr)
        ref = polys.clone()
        for _ in range(3):
            nctx.ntt_forward(polys, c5.batch, sptr)
            nctx.ntt_inverse(polys, c5.batch, sptr)
        reps = args.ntt_reps
        e = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
        tf = ti = 0.0
        for _ in range(reps):
            e[0].record(stream)
            nctx.ntt_forward(polys, c5.batch, sptr)
            e[1].record(stream)
            nctx.ntt_inverse(polys, c5.batch, sptr)
            e[2].record(stream)
            torch.cuda.synchronize()
            tf += e[0].elapsed_time(e[1])
            ti += e[1].elapsed_time(e[2])
        ok = bool(torch.equal(polys, ref))
        tf, ti = tf / reps, ti / reps
        nbytes_alg = 2 * c5.batch * c5.L * c5.N * 16
        bf = 2 * c5.batch * c5.L * (c5.N // 2) * c5.log2_n
        opb5, arith5 = ops_per_butterfly(max(c5.q))
        result["ntt"] = {"workload": "C5: forward+inverse, N=65536, 16 x 60-bit primes, batch 64",
                         "roundtrip_ok": ok, "forward_ms": tf, "inverse_ms": ti,
                         "algorithmic_GB": nbytes_alg / 1e9,
                         "algorithmic_GB_per_s": nbytes_alg / 1e9 / ((tf + ti) * 1e-3),
                         "frac_hbm_peak": nbytes_alg / 1e9 / ((tf + ti) * 1e-3) / HBM_PEAK_GBS,
                         "butterfly_Tops_per_s": bf * opb5 / ((tf + ti) * 1e-3) / 1e12,
                         "frac_valu_peak": bf * opb5 / ((tf + ti) * 1e-3) / 1e12 / VALU_PEAK_TOPS,
                         "arith": arith5, "ops_per_butterfly": opb5}
        nctx.close()

    # ---- CPU baseline: the oracle as it stands, on a bounded sample of the same workload ---
    if not args.no_cpu:
        from oracle import oracle
        orc = oracle.Oracle(cfg.log2_n, cfg.q, cfg.t, cfg.eta, cfg.frac_bits, cfg.max_group, cfg.seed)
        okeys = {}
        sample_groups = list(range(G if cfg.name in ("C1", "C2") else 1))
        for gi in sample_groups:
            for k in groups[gi]:
                if k not in okeys:
                    okeys[k] = orc.keygen_share(k)
        opks = [orc.aggregate_pk([okeys[k][1] for k in groups[gi]]) for gi in sample_groups]
        c_end = min(C_, max(1, int(25 * 4096 * 3 / (N * L))))      # bounds the CPU work to tens of core-seconds
        t0 = time.perf_counter()
        threads = 1
        for gi in sample_groups:
            res, threads = orc.round_group(opks[gi], [okeys[k][0] for k in groups[gi]],
                                           [grads_host[k] for k in groups[gi]], groups[gi], gi, 0, c_end)
            got = outs[gi].cpu().numpy()[: c_end * N]
            if not np.array_equal(res[: c_end * N][: got.size], got[: res.size]):
                print("bench.py: GPU result differs from the oracle", file=sys.stderr)
                sys.exit(5)
        dt = time.perf_counter() - t0
        n_fresh = sum(len(groups[gi]) for gi in sample_groups) * c_end
        result["cpu_baseline"] = {"value": n_fresh / dt, "unit": "fresh ciphertexts/s", "cores": threads,
                                  "kind": "oracle", "seconds": dt,
                                  "sample": f"groups {sample_groups}, ciphertext indices 0..{c_end - 1} of {cfg.name} "
                                            f"({n_fresh} fresh ciphertexts), whole round incl. decode"}
    ctx.close()
    print(json.dumps(result))


if __name__ == "__main__":
    main()
