#!/usr/bin/env python3
"""Benchmark of the exchange round on one MI355X.

A step is one whole round of the hot path (encode + encrypt, homomorphic sum, decryption
shares, combine + decode) for every group of the workload, with the float32 gradients and
all keys already resident in HBM.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C3] [--legs C1,C2,C4]
                  [--no-cpu] [--no-ntt] [--no-coeff] [--no-loop] [--no-bootstrap] [--no-convert]

The headline is the largest configuration (C3: most ciphertexts, bytes and butterflies per round).
The other round configurations are timed as secondary legs with the same fields.  Beside them the
line reports, on the headline workload, the round with coefficient packing, training iterations
(Alg. 2), a collective refresh (MBFV.Bootstrap) and the round with the paper's own decryption path
(MBFV.Convert); the batched transform micro-benchmark (C5); and the CPU oracle timed on bounded
samples of the headline round and of the C5 batch.
"""
import argparse
import glob
import json
import math
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0                      # MI355X HBM3E
VALU_PEAK_TOPS = 256 * 64 * 2.4e9 / 1e12   # 256 CUs x 64 lanes x 2.4 GHz = 39.3 T lane-ops/s
JOBS_PER_LAUNCH = 112                      # (party, group) pairs one launch of a phase takes


def ops_per_butterfly(qmax):
    """VALU instructions of one butterfly in the minimal sequence of each arithmetic back-end
    (csrc/arith.hpp): 32-bit Harvey butterflies for moduli < 2^30, doubles for moduli < 2^44, 63-bit
    Shoup with an approximate quotient for moduli < 2^55, exact Harvey butterflies for moduli < 2^61."""
    if qmax < (1 << 30):
        return 8, "u32-harvey"
    if qmax < (1 << 44):
        return 8, "f64"
    if qmax < (1 << 55):
        return 15, "u64-lazy"
    return 21, "u64-harvey"


def profiled_traffic(workload, kernel):
    """HBM bytes per launch of `kernel` in the round of `workload`, as the committed rocprofv3
    summaries under profiles/ recorded them (FETCH_SIZE and WRITE_SIZE of the launch, each scaled
    by what the same counter reads for a plain 512 MiB copy).  (read, written, file) or None."""
    pat = re.compile(r"^bench-traffic: workload=%s kernel=%s read_bytes=(\d+) written_bytes=(\d+)"
                     % (re.escape(workload), re.escape(kernel)))
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", "*.txt"))):
        with open(path) as fh:
            for line in fh:
                m = pat.match(line)
                if m:
                    return int(m.group(1)), int(m.group(2)), os.path.relpath(path, ROOT)
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="C3", choices=["C1", "C2", "C3", "C4"])
    ap.add_argument("--legs", default="C1,C2,C4", help="round configurations timed as secondary legs ('' = none)")
    ap.add_argument("--leg-steps", type=int, default=0, help="timed steps of a leg (0: sized to about a second)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline legs")
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
    stream = torch.cuda.current_stream()     # every launch and every event below is on this stream
    sptr = stream.cuda_stream

    def dz(n, dtype=torch.int64):
        return torch.zeros(n, dtype=dtype, device=dev)

    def new_events(n=5):
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(n)]
        for e in evs:
            e.record(stream)                      # creates the underlying hipEvent_t
        return evs

    def fixed_point_sum(cfg, grads_host, members):
        clamp = ((cfg.t - 1) // 2) // cfg.max_group
        acc = np.zeros(cfg.n_values, dtype=np.int64)
        for k in members:
            r = np.rint(grads_host[k] * np.float32(2.0 ** cfg.frac_bits)).astype(np.float64)
            acc += np.clip(r, -clamp, clamp).astype(np.int64)
        return acc.astype(np.float32) * np.float32(2.0 ** -cfg.frac_bits)

    class Workload:
        """One round configuration resident on the device: context, keys, gradients, scratch."""

        def __init__(self, name):
            cfg = self.cfg = CONFIGS[name]
            self.N, self.L, self.C, self.P = cfg.N, cfg.L, cfg.C, cfg.parties
            self.groups = cfg.groups()
            self.G, self.J = len(self.groups), sum(len(g) for g in self.groups)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            self.ctx = binding.Context(cfg.log2_n, cfg.q, cfg.t, cfg.eta, cfg.frac_bits, cfg.max_group, cfg.seed,
                                       alloc=lambda n: dz(n // 8 + 2))
            torch.cuda.synchronize()
            self.create_ms = (time.perf_counter() - t0) * 1e3
            # set-up (not part of the round: executed once per training run; reported on its own)
            self.grads_host = cfg.gradients()
            self.grads = [torch.from_numpy(g).to(dev) for g in self.grads_host]
            N, L, P = self.N, self.L, self.P
            self.sks = [dz(2 * L * N) for _ in range(P)]
            self.pk0 = [dz(L * N) for _ in range(P)]
            self.pks = [dz(4 * L * N) for _ in self.groups]
            self.make_keys()
            torch.cuda.synchronize()
            sev = new_events(2)
            sev[0].record(stream)                          # the same set-up again, now with the code resident
            self.make_keys()
            sev[1].record(stream)
            torch.cuda.synchronize()
            self.keys_ms = sev[0].elapsed_time(sev[1])
            self.outs = [torch.zeros(cfg.n_values, dtype=torch.float32, device=dev) for _ in self.groups]
            self.nbytes = self.ctx.round_scratch_bytes(self.J, self.G, cfg.n_values)
            self.scratch = dz(self.nbytes // 8)
            self.desc = self.ctx.make_round(self.groups, self.pks, self.sks, self.grads, self.outs, cfg.n_values)
            self.opb, self.arith = ops_per_butterfly(max(cfg.q))
            self.launches = math.ceil(self.J / JOBS_PER_LAUNCH)          # launches of one phase
            torch.cuda.synchronize()

        def make_keys(self):
            for k in range(self.P):
                self.ctx.keygen_share(k, self.sks[k], self.pk0[k], sptr)
            for gi, g in enumerate(self.groups):
                self.ctx.aggregate_pk([self.pk0[k] for k in g], self.pks[gi], sptr)

        def round(self, events=None, desc=None):
            self.ctx.round(desc or self.desc, self.scratch, self.nbytes, events, sptr)

        def check(self, what, outs=None):
            """What was timed decodes to the fixed-point sums (first and last group)."""
            outs = outs or self.outs
            for gi in sorted({0, self.G - 1}):
                if not np.array_equal(outs[gi].cpu().numpy(), fixed_point_sum(self.cfg, self.grads_host, self.groups[gi])):
                    print(f"bench.py: {what}: decoded result differs from the fixed-point sum", file=sys.stderr)
                    sys.exit(4)

        def describe(self):
            c = self.cfg
            return (f"{c.name}: N={self.N}, L={self.L}, t={c.t}, P={self.P}, G={self.G}, K={c.max_group}, C={self.C}, "
                    f"{c.n_values} floats/party")

        def figures(self, ms, phase_ms, enc_launch_ms):
            """Throughput and roofline figures of a round that took `ms` per step."""
            cfg, N, L, C_ = self.cfg, self.N, self.L, self.C
            fresh = self.J * C_
            S = 16 * L * N                                    # bytes of one ciphertext
            bf_per_transform = (N // 2) * cfg.log2_n
            # whole round, algorithmic: (4K+1) L transforms per aggregated ciphertext + (K+1) mod-t transforms
            round_bf = sum(((4 * len(g) + 1) * L + len(g) + 1) for g in self.groups) * C_ * bf_per_transform
            round_bytes = sum(S * (3.5 * len(g) + 1.5) for g in self.groups) * C_
            # the fused encode+encrypt kernel: 3 L transforms mod q_i + 1 mod t per fresh ciphertext
            enc_bf = fresh * (3 * L + 1) * bf_per_transform / self.launches
            enc_bytes = (fresh * S + fresh * 4 * N) / self.launches
            enc_rate = enc_bf * self.opb / (enc_launch_ms * 1e-3) / 1e12
            sec = ms * 1e-3
            return {
                "workload": self.describe(), "ms_per_step": ms, "fresh_ciphertexts": fresh,
                "aggregated_ciphertexts": self.G * C_, "fresh_ct_per_s": fresh / sec,
                "aggregated_ct_per_s": self.G * C_ / sec,
                "phase_ms": {"encode_encrypt": phase_ms[0], "aggregate": phase_ms[1], "shares": phase_ms[2],
                             "combine_decode": phase_ms[3]},
                "phase_roofline": self.phase_roofline(phase_ms),
                "round_algorithmic": {"GB": round_bytes / 1e9, "GB_per_s": round_bytes / 1e9 / sec,
                                      "frac_hbm_peak": round_bytes / 1e9 / sec / HBM_PEAK_GBS,
                                      "butterfly_Tops_per_s": round_bf * self.opb / sec / 1e12,
                                      "frac_valu_peak": round_bf * self.opb / sec / 1e12 / VALU_PEAK_TOPS},
                "k_encrypt": {"launches_per_round": self.launches, "avg_launch_ms": enc_launch_ms,
                              "butterfly_Tops_per_s": enc_rate, "frac_valu_peak": enc_rate / VALU_PEAK_TOPS,
                              "algorithmic_bytes": enc_bytes,
                              "hbm_algorithmic_GB_per_s": enc_bytes / 1e9 / (enc_launch_ms * 1e-3),
                              "frac_hbm_peak": enc_bytes / 1e9 / (enc_launch_ms * 1e-3) / HBM_PEAK_GBS,
                              "ops_per_butterfly": self.opb, "arith": self.arith},
            }

        def phase_roofline(self, phase_ms):
            """Each phase against both rooflines: algorithmic bytes (every message written once and read once) over
            HBM peak, and butterfly instructions of its transforms over the VALU peak."""
            N, L, C_ = self.N, self.L, self.C
            S = 16 * L * N
            bf = (N // 2) * self.cfg.log2_n
            ks = [len(g) for g in self.groups]
            nbytes = {"encode_encrypt": sum(k * (S + 4 * N) for k in ks) * C_,
                      "aggregate": sum((k + 1) * S for k in ks) * C_,
                      "shares": sum(k * S for k in ks) * C_,                       # c1 read per member, share written
                      "combine_decode": sum((k + 1) * S / 2 + 4 * N for k in ks) * C_}
            # transforms modulo q_i at the context's instruction count, the ones modulo t on 32-bit residues (8)
            ops = {"encode_encrypt": sum(k * (3 * L * self.opb + 8) for k in ks) * C_ * bf,
                   "aggregate": 0,
                   "shares": sum(k * L * self.opb for k in ks) * C_ * bf,
                   "combine_decode": len(ks) * (L * self.opb + 8) * C_ * bf}
            out = {}
            for name, ms in zip(("encode_encrypt", "aggregate", "shares", "combine_decode"), phase_ms):
                sec = ms * 1e-3
                out[name] = {"algorithmic_GB_per_s": nbytes[name] / 1e9 / sec,
                             "frac_hbm_peak": nbytes[name] / 1e9 / sec / HBM_PEAK_GBS,
                             "butterfly_Tops_per_s": ops[name] / sec / 1e12,
                             "frac_valu_peak": ops[name] / sec / 1e12 / VALU_PEAK_TOPS}
            return out

        def close(self):
            self.ctx.close()

    def phase_split(run, n_ev):
        evs = [new_events() for _ in range(n_ev)]
        torch.cuda.synchronize()
        for i in range(n_ev):
            run([e.cuda_event for e in evs[i]])
        torch.cuda.synchronize()
        return [sum(e[i].elapsed_time(e[i + 1]) for e in evs) / n_ev for i in range(4)]

    def time_rounds(run, steps, warmup):
        """A secondary leg: ms per round from `steps` rounds without events (after a warm-up), and the
        phase split from up to 20 further rounds with an event after every phase."""
        for _ in range(warmup):
            run(None)
        torch.cuda.synchronize()
        t_0 = time.perf_counter()
        for _ in range(steps):
            run(None)
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t_0) * 1e3 / steps
        return ms, phase_split(run, max(1, min(steps, 20)))

    # ---------------------------------------------------------------- headline round
    w = Workload(args.workload)
    cfg = w.cfg
    N, L, C_, P, G, J, ctx = w.N, w.L, w.C, w.P, w.G, w.J, w.ctx
    for _ in range(args.warmup):
        w.round()
    torch.cuda.synchronize()
    # Timed region: exactly `steps` rounds.  Two events bracket the dominant kernel's launches (the
    # encrypt phase) on every EVENT_EVERY-th step: an event costs a few microseconds of idle GPU, which
    # matters only for the sub-millisecond rounds.  The phase split comes from further (untimed) steps.
    heavy = w.J * w.C >= 5000
    EVENT_EVERY = 1 if heavy else 8
    step_events = {i: new_events(2) for i in range(0, args.steps, EVENT_EVERY)}
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        ev = step_events.get(i)
        w.round([ev[0].cuda_event, ev[1].cuda_event, None, None, None] if ev else None)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    enc_phase_ms = sum(ev[0].elapsed_time(ev[1]) for ev in step_events.values()) / len(step_events)
    nph = max(1, min(args.steps, 20))
    phase_ms = phase_split(w.round, nph)
    w.check("headline round")

    fig = w.figures(ms_per_step, phase_ms, enc_phase_ms / w.launches)
    ke = fig["k_encrypt"]
    traffic = profiled_traffic(cfg.name, "k_encrypt")
    result = {
        "metric": "BFV gradient ciphertexts/sec (encrypt+aggregate+decrypt-share)",
        "value": fig["fresh_ct_per_s"], "unit": "fresh ciphertexts/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None,
        "dtype": {"f64": "f64", "u32-harvey": "u32"}.get(w.arith, "u64"),
        "dtype_note": "residues below 2^30 are 32-bit integers, below 2^44 exact integers in doubles, wider ones 64-bit integers",
        "data": "synthetic",
        "config": {"workload": fig["workload"], "fresh_ciphertexts": fig["fresh_ciphertexts"],
                   "aggregated_ciphertexts": fig["aggregated_ciphertexts"],
                   "why": "largest round configuration by ciphertexts, bytes and butterflies; the others are the legs below"},
        "aggregated_ct_per_s": fig["aggregated_ct_per_s"],
        "setup": {"what": f"once per training run, outside the timed round: tables and context (host + copy), "
                          f"then {P} key shares and {G} collective public keys on the GPU",
                  "create_ms": w.create_ms, "keys_ms": w.keys_ms},
        "phase_ms": fig["phase_ms"],
        "phase_roofline": fig["phase_roofline"],
        "phase_ms_from": f"{nph} further steps with an event after every phase (of the timed steps every "
                         f"{EVENT_EVERY}th records two events, around the dominant kernel's launches)",
        "round_algorithmic": fig["round_algorithmic"],
        "roofline": {"kernel": f"k_encrypt (fused encode + encrypt), {w.launches} launch(es) per round", "bound": "alu",
                     "achieved": ke["butterfly_Tops_per_s"], "peak": VALU_PEAK_TOPS,
                     "unit": f"T lane-ops/s (butterfly instructions, {w.opb} per butterfly, {w.arith})",
                     "frac": ke["frac_valu_peak"],
                     "traffic": (traffic[0] + traffic[1]) if traffic else None,
                     "traffic_read_written": list(traffic[:2]) if traffic else None,
                     "traffic_from": traffic[2] if traffic else None,
                     "traffic_unit": "bytes per launch (rocprofv3 FETCH_SIZE + WRITE_SIZE, copy-calibrated)",
                     "algorithmic_bytes": ke["algorithmic_bytes"], "avg_launch_ms": ke["avg_launch_ms"],
                     "hbm_algorithmic_GB_per_s": ke["hbm_algorithmic_GB_per_s"], "hbm_frac": ke["frac_hbm_peak"]},
    }

    # ---- the same round with coefficient packing (value j of a ciphertext is coefficient j): an
    # addition-only workload does not need the slot structure, so both transforms modulo t go away
    ex_steps = max(1, min(args.steps, 100 if not heavy else 10))
    ex_warm = max(1, min(args.warmup, 10))
    if not args.no_coeff:
        pdesc = ctx.make_round(w.groups, w.pks, w.sks, w.grads, w.outs, cfg.n_values, packing=1)
        for o_ in w.outs:
            o_.zero_()
        pms, pphase = time_rounds(lambda ev: w.round(ev, pdesc), ex_steps, ex_warm)
        w.check("coefficient-packed round")
        result["coefficient_packing_round"] = {
            "what": "the whole round with value j of a ciphertext as coefficient j (no transform modulo t in "
                    "encode or decode); same sums",
            "ms_per_step": pms, "steps": ex_steps, "fresh_ct_per_s": J * C_ / (pms * 1e-3),
            "phase_ms": {"encode_encrypt": pphase[0], "aggregate": pphase[1], "shares": pphase[2],
                         "combine_decode": pphase[3]}}

    # ---- training iterations (Alg. 2): round with fresh ciphertext indices, then every node's
    # float step (average over its neighbourhood, local gradient step) on its own weights
    if not args.no_loop:
        owner = cfg.receivers()
        node_group = {i: gi for gi, rs in enumerate(owner) for i in rs}
        T_it = 5 if not heavy else 3
        weights = [g.clone() for g in w.grads]
        descs = [ctx.make_round(w.groups, w.pks, w.sks, weights, w.outs, cfg.n_values, ct_base=it * C_) for it in range(T_it)]
        le = new_events(2)

        def iterate():
            for it in range(T_it):
                w.round(None, descs[it])
                for i in range(P):
                    gi = node_group[i]
                    binding.average_update(w.outs[gi], len(w.groups[gi]), w.grads[i], 0.01, cfg.n_values, weights[i], sptr)

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
        del weights, descs
        w.round()          # leave scratch and outputs as the headline round left them
        torch.cuda.synchronize()

    # ---- MBFV.Bootstrap: the members of group 0 refresh aggregates the round left in the scratch
    # (same work for each; the first C are group 0's own and are checked after the refresh)
    if not args.no_bootstrap:
        w.round()          # slot-packed aggregates in the scratch, whatever ran before
        LN = L * N
        nct = min(G * C_, 1024)
        agg = w.scratch[J * C_ * 2 * LN:(J * C_ + nct) * 2 * LN]
        g0 = w.groups[0]
        alpha = dz(nct * LN)
        bshares = [dz(nct * 2 * LN) for _ in g0]
        fresh_ct = dz(nct * 2 * LN)

        def refresh():
            ctx.bootstrap_alpha(0, 0, nct, alpha, sptr)
            for k, sh in zip(g0, bshares):
                ctx.bootstrap_share(w.sks[k], agg, alpha, nct, k, 0, 0, sh, sptr)
            ctx.bootstrap_combine(agg, alpha, bshares, nct, fresh_ct, sptr)

        refresh()
        torch.cuda.synchronize()
        bsteps = max(1, min(args.steps, 10))
        be = new_events(2)
        be[0].record(stream)
        for _ in range(bsteps):
            refresh()
        be[1].record(stream)
        torch.cuda.synchronize()
        bms = be[0].elapsed_time(be[1]) / bsteps
        # the refreshed aggregates of group 0 decrypt to the same sums
        cb = min(C_, nct)
        psh = [dz(cb * LN) for _ in g0]
        for k, sh in zip(g0, psh):
            ctx.partial_decrypt(w.sks[k], fresh_ct, cb, k, 0, 0, sh, sptr)
        bpt = dz(cb * N)
        ctx.combine(fresh_ct, psh, cb, bpt, sptr)
        nb = min(cfg.n_values, cb * N)
        bout = torch.zeros(nb, dtype=torch.float32, device=dev)
        ctx.decode(bpt, cb, nb, bout, sptr)
        torch.cuda.synchronize()
        if not torch.equal(bout, w.outs[0][:nb]):
            print("bench.py: refreshed ciphertexts decrypt to something else", file=sys.stderr)
            sys.exit(7)
        result["bootstrap"] = {"what": f"collective refresh (Eq. (3)) of {nct} ciphertexts by {len(g0)} members: "
                                       "common polynomial, one share per member, refreshed ciphertext",
                               "ms": bms, "refreshed_ct_per_s": nct / (bms * 1e-3)}
        del alpha, bshares, fresh_ct, psh, agg

    # ---- CPU baseline: the oracle as it stands, on a bounded sample of the headline round ------
    # (before the scratch of the collective-decryption round is released)
    if not args.no_cpu:
        from oracle import oracle
        orc = oracle.Oracle(cfg.log2_n, cfg.q, cfg.t, cfg.eta, cfg.frac_bits, cfg.max_group, cfg.seed)
        # about 1.25 us of one (slow) host core per member, limb and coefficient: bound the sample to some
        # 240 such core-seconds -- whole groups if a group's round fits, else the first indices of group 0
        est = cfg.max_group * L * N * 1.25e-6
        whole = int(240.0 / (est * C_))
        sample_groups = list(range(max(1, min(G, whole))))
        c_end = C_ if whole >= 1 else max(1, int(240.0 / est))
        okeys = {}
        for gi in sample_groups:
            for k in w.groups[gi]:
                if k not in okeys:
                    okeys[k] = orc.keygen_share(k)
        opks = [orc.aggregate_pk([okeys[k][1] for k in w.groups[gi]]) for gi in sample_groups]
        t0 = time.perf_counter()
        threads = 1
        for gi in sample_groups:
            res, threads = orc.round_group(opks[gi], [okeys[k][0] for k in w.groups[gi]],
                                           [w.grads_host[k] for k in w.groups[gi]], w.groups[gi], gi, 0, c_end)
            n_cmp = min(cfg.n_values, c_end * N)
            if not np.array_equal(res[:n_cmp], w.outs[gi].cpu().numpy()[:n_cmp]):
                print("bench.py: GPU result differs from the oracle", file=sys.stderr)
                sys.exit(5)
        dt = time.perf_counter() - t0
        n_fresh = sum(len(w.groups[gi]) for gi in sample_groups) * c_end
        result["cpu_baseline"] = {"value": n_fresh / dt, "unit": "fresh ciphertexts/s", "cores": threads,
                                  "kind": "oracle", "seconds": dt,
                                  "sample": f"groups {sample_groups}, ciphertext indices 0..{c_end - 1} of {cfg.name} "
                                            f"({n_fresh} fresh ciphertexts), whole round incl. decode; the GPU's "
                                            "decoded values of the sample equal the oracle's"}
        del orc, okeys, opks

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
        conv = ctx.make_convert(w.desc, receivers, rpk, rsk, routs)
        cbytes = ctx.round_convert_scratch_bytes(J, G, conv.num_shares, cfg.n_values)
        w.scratch = None
        torch.cuda.empty_cache()
        cscratch = dz(cbytes // 8)
        cms, cphase = time_rounds(lambda ev: ctx.round_convert(w.desc, conv, cscratch, cbytes, ev, sptr), ex_steps, ex_warm)
        ri = 0
        for gi in range(G):
            for _ in receivers[gi]:
                if gi in (0, G - 1) and not np.array_equal(routs[ri].cpu().numpy(),
                                                           fixed_point_sum(cfg, w.grads_host, w.groups[gi])):
                    print("bench.py: converted result differs from the fixed-point sum", file=sys.stderr)
                    sys.exit(6)
                ri += 1
        result["convert_round"] = {
            "what": "encode+encrypt, sum, conversion shares towards every receiver (Eq. (1)), "
                    "converted ciphertext + single-key decryption + decode (Eq. (2))",
            "receivers": R, "conversion_shares": conv.num_shares, "ms_per_step": cms, "steps": ex_steps,
            "fresh_ct_per_s": J * C_ / (cms * 1e-3),
            "phase_ms": {"encode_encrypt": cphase[0], "aggregate": cphase[1], "convert_shares": cphase[2],
                         "combine_decrypt_decode": cphase[3]}}
        del cscratch, routs, rsk, rpk, conv
    w.close()
    del w
    torch.cuda.empty_cache()

    # ---------------------------------------------------------------- the other round configurations
    legs = {}
    for name in [s for s in args.legs.split(",") if s and s != args.workload]:
        if name not in ("C1", "C2", "C3", "C4"):
            print(f"bench.py: unknown leg {name}", file=sys.stderr)
            sys.exit(2)
        lw = Workload(name)
        lw.round()
        torch.cuda.synchronize()
        p0 = time.perf_counter()
        lw.round()
        torch.cuda.synchronize()
        probe_ms = (time.perf_counter() - p0) * 1e3
        steps = args.leg_steps or int(max(10, min(200, 1000.0 / probe_ms)))
        ms, ph = time_rounds(lambda ev: lw.round(ev), steps, max(3, min(steps // 2, 50)))
        lw.check(f"leg {name}")
        f = lw.figures(ms, ph, ph[0] / lw.launches)
        f["steps"] = steps
        f["setup"] = {"create_ms": lw.create_ms, "keys_ms": lw.keys_ms}
        tr = profiled_traffic(name, "k_encrypt")
        f["k_encrypt"]["traffic"] = (tr[0] + tr[1]) if tr else None
        f["k_encrypt"]["traffic_from"] = tr[2] if tr else None
        f["k_encrypt"]["avg_launch_ms_from"] = "encrypt phase (events after every phase, untimed steps) / launches"
        legs[name] = f
        lw.close()
        del lw
        torch.cuda.empty_cache()
    if legs:
        result["legs"] = legs

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
        e = new_events(3)
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
        alu_floor_ms = bf * opb5 / (VALU_PEAK_TOPS * 1e12) * 1e3
        tr = [profiled_traffic("C5", k) for k in ("k_head_forward", "k_tail_forward", "k_tail_inverse", "k_head_inverse")]
        result["ntt"] = {"workload": "C5: forward+inverse, N=65536, 16 x 60-bit primes, batch 64",
                         "roundtrip_ok": ok, "forward_ms": tf, "inverse_ms": ti,
                         "algorithmic_GB": nbytes_alg / 1e9,
                         "algorithmic_GB_per_s": nbytes_alg / 1e9 / ((tf + ti) * 1e-3),
                         "frac_hbm_peak": nbytes_alg / 1e9 / ((tf + ti) * 1e-3) / HBM_PEAK_GBS,
                         "butterfly_Tops_per_s": bf * opb5 / ((tf + ti) * 1e-3) / 1e12,
                         "frac_valu_peak": bf * opb5 / ((tf + ti) * 1e-3) / 1e12 / VALU_PEAK_TOPS,
                         "arith": arith5, "ops_per_butterfly": opb5,
                         "alu_floor_ms": alu_floor_ms,
                         "alu_floor_note": f"{bf:.3g} butterflies x {opb5} instructions at {VALU_PEAK_TOPS:.1f} T lane-ops/s; "
                                           "the 60 %-of-HBM-peak target (0.447 ms) lies below this floor",
                         "frac_of_alu_floor": alu_floor_ms / (tf + ti),
                         "traffic": sum(t[0] + t[1] for t in tr) if all(tr) else None,
                         "traffic_from": tr[0][2] if all(tr) else None,
                         "traffic_unit": "HBM bytes of forward + inverse (rocprofv3 FETCH_SIZE + WRITE_SIZE, copy-calibrated)"}
        if not args.no_cpu:
            # the oracle's batched transform on a bounded part of the batch, checked against the GPU's
            from oracle import oracle
            orc5 = oracle.Oracle(c5.log2_n, c5.q, 0, 21, 0, 1, c5.seed)
            Bs = c5.batch          # the whole batch: about a second on 16 cores
            sample = ref[:Bs * c5.L * c5.N].cpu().numpy().view(np.uint64).reshape(Bs, c5.L, c5.N)
            t0 = time.perf_counter()
            fwd = orc5.ntt_forward_batch(sample)
            back = orc5.ntt_inverse_batch(fwd)
            dt = time.perf_counter() - t0
            nctx.ntt_forward(polys, c5.batch, sptr)
            torch.cuda.synchronize()
            got = polys[:Bs * c5.L * c5.N].cpu().numpy().view(np.uint64).reshape(Bs, c5.L, c5.N)
            perm = nctx.index_map()
            if not (np.array_equal(back, sample) and np.array_equal(got, fwd[:, :, perm])):
                print("bench.py: GPU transform differs from the oracle", file=sys.stderr)
                sys.exit(9)
            import ctypes
            cores = int(ctypes.CDLL("libgomp.so.1").omp_get_max_threads())      # the team the batch loops run with
            result["ntt"]["cpu_baseline"] = {
                "value": 2 * Bs * c5.L * c5.N * 16 / 1e9 / dt, "unit": "algorithmic GB/s", "cores": cores, "kind": "oracle",
                "seconds": dt, "sample": f"forward + inverse of all {Bs} batch members ({Bs * c5.L} polynomials of 65536), OpenMP over "
                                         "polynomials; the GPU's forward output equals the oracle's"}
        nctx.close()

    print(json.dumps(result))


if __name__ == "__main__":
    main()
