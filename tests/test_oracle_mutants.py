"""Strength of the oracle's pins: a plausible mistake planted anywhere in the oracle (a dropped term, a wrong
sign or index, a transposed operand) must make the pin suite fail.

Every mutant is a copy of ``oracle/d2mhe_oracle.c`` with one textual change, compiled with gcc and loaded by a
child process that runs ``tests/test_oracle_pins.py``.  CPU only; nothing here touches the HIP library."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "d2mhe_oracle.c")

# (name, text in the source, replacement); every text occurs exactly once
MUTANTS = [
    ("philox_multipliers_swapped", "uint64_t p0 = (uint64_t)0xD2511F53u * c0;", "uint64_t p0 = (uint64_t)0xCD9E8D57u * c0;"),
    ("philox_key_not_bumped", "        k1 += 0xBB67AE85u;\n", ""),
    ("counter_group_shift", "| (group << 16) };", "| (group << 8) };"),
    ("ternary_wrong_word", "(uint64_t)w[i & 3] * 3u", "(uint64_t)w[(i + 1) & 3] * 3u"),
    ("cbd_sign", "popcount32(w[j] & mask) - popcount32(w[j + 1] & mask)", "popcount32(w[j + 1] & mask) - popcount32(w[j] & mask)"),
    ("uniform_word_order", "(u128)w[0] | ((u128)w[1] << 32)", "(u128)w[1] | ((u128)w[0] << 32)"),
    ("prime_search_step", "uint64_t cand = top - k * two_n + 1;", "uint64_t cand = top - k * two_n - 1;"),
    # (starting the search at 3 would be no mistake: 2 is a square modulo every q = 1 mod 8 and never qualifies)
    ("psi_search_skips_3", "for (uint64_t x = 2; x < q; ++x) {\n        uint64_t psi = orc_powmod(x, (q - 1) / (2 * n), q);",
     "for (uint64_t x = 4; x < q; ++x) {\n        uint64_t psi = orc_powmod(x, (q - 1) / (2 * n), q);"),
    ("butterfly_sign", "x[start + k + len / 2] = submod(u, v, q);", "x[start + k + len / 2] = submod(v, u, q);"),
    ("forward_root_not_squared", "cyclic_ntt(x, n, q, orc_mulmod(psi, psi, q));", "cyclic_ntt(x, n, q, psi);"),
    ("inverse_without_scaling", "uint64_t pw = n_inv;", "uint64_t pw = 1;"),
    ("pk_share_not_negated", "pk0_share[(size_t)i * n + k] = submod(0, v, q);       /* negated      */", "pk0_share[(size_t)i * n + k] = v;"),
    ("pk_share_without_error", "uint64_t v = addmod(prod[k], lift_small(e[k], q), q); /* p1 s_k + e_k */", "uint64_t v = prod[k];"),
    ("pk_sum_skips_a_share", "for (uint32_t m = 0; m < K; ++m) acc = addmod(acc, pk0_shares[m][(size_t)i * n + k], q);",
     "for (uint32_t m = 1; m < K; ++m) acc = addmod(acc, pk0_shares[m][(size_t)i * n + k], q);"),
    ("encode_lower_clamp_dropped", "                if (rf < -bound) rf = -bound;\n                r = (int64_t)rf;\n            }\n            z[j] =",
     "                r = (int64_t)rf;\n            }\n            z[j] ="),
    ("encode_transform_direction", "        orc_ntt_inverse(z, n, t, c->psi_t);\n    }\n    return 0;\n}\n\nint orc_decode(",
     "        orc_ntt_forward(z, n, t, c->psi_t);\n    }\n    return 0;\n}\n\nint orc_decode("),
    ("decode_centre_off_by_one", "int64_t v = z[j] > (t - 1) / 2 ? (int64_t)z[j] - (int64_t)t : (int64_t)z[j];\n            out[idx] =",
     "int64_t v = z[j] >= (t - 1) / 2 ? (int64_t)z[j] - (int64_t)t : (int64_t)z[j];\n            out[idx] ="),
    ("coefficient_decode_centre", "int64_t v = pt[idx] > (t - 1) / 2 ?", "int64_t v = pt[idx] > (t + 1) / 2 ?"),
    ("encrypt_without_lambda", "uint64_t lm = orc_mulmod(c->lambda_mod_q[i], m[k] % q, q);\n                c0[", "uint64_t lm = m[k] % q;\n                c0["),
    ("encrypt_c1_uses_e0", "c1[(size_t)i * n + k] = addmod(prod[k], lift_small(e1[k], q), q);", "c1[(size_t)i * n + k] = addmod(prod[k], lift_small(e0[k], q), q);"),
    ("encrypt_c1_uses_p0", "orc_ring_mul(mu_q, p1, n, q, c->psi[i], prod);\n            for (size_t k = 0; k < n; ++k)\n                c1[",
     "orc_ring_mul(mu_q, p0, n, q, c->psi[i], prod);\n            for (size_t k = 0; k < n; ++k)\n                c1["),
    ("add_skips_c1", "for (uint32_t comp = 0; comp < 2; ++comp)", "for (uint32_t comp = 0; comp < 1; ++comp)"),
    ("share_from_c0", "c->p.cbd_eta, n, e);\n        const uint64_t *c1 = ct + ((size_t)ci * 2 + 1) * L * n;",
     "c->p.cbd_eta, n, e);\n        const uint64_t *c1 = ct + ((size_t)ci * 2 + 0) * L * n;"),
    ("share_without_error", "share[((size_t)ci * L + i) * n + k] = addmod(prod[k], lift_small(e[k], q), q);", "share[((size_t)ci * L + i) * n + k] = prod[k];"),
    ("rounding_becomes_floor", "    big_mul_u64(&y, 2 * c->p.t);\n    big_add(&y, &c->Q);\n", "    big_mul_u64(&y, 2 * c->p.t);\n"),
    # (leaving out the reduction of the lifted value modulo Q would be no mistake: it shifts the result by a multiple of t)
    ("crt_without_inverse", "big_mul_u64(&term, orc_mulmod(res[i], c->Q_over_qi_inv[i], c->p.q[i]));", "big_mul_u64(&term, res[i]);"),
    ("combine_skips_a_share", "for (uint32_t m = 0; m < K; ++m)\n                    acc = addmod(acc, shares[m][((size_t)ci * L + i) * n + k], c->p.q[i]);",
     "for (uint32_t m = 1; m < K; ++m)\n                    acc = addmod(acc, shares[m][((size_t)ci * L + i) * n + k], c->p.q[i]);"),
    ("receiver_p1_same_for_all_limbs", "orc_sample_uniform(c->p.seed, ORC_DOM_RPK_A, i, party, 0, 0, q, n, p1);", "orc_sample_uniform(c->p.seed, ORC_DOM_RPK_A, 0, party, 0, 0, q, n, p1);"),
    ("receiver_p0_sign", "p0[k] = submod(0, addmod(prod[k], lift_small(e[k], q), q), q); /* -(p1 sk + e) */", "p0[k] = addmod(prod[k], lift_small(e[k], q), q);"),
    ("convert_counter_transposed", "uint32_t who = party | (receiver << 16);", "uint32_t who = receiver | (party << 16);"),
    ("convert_share_without_s_c1", "h0[(size_t)i * n + k] = addmod(addmod(sc1[k], prod[k], q), lift_small(e0[k], q), q);", "h0[(size_t)i * n + k] = addmod(prod[k], lift_small(e0[k], q), q);"),
    ("convert_keeps_old_c1", "uint64_t a0 = ct[o0 + k], a1 = 0; /* the old c1 is dropped */", "uint64_t a0 = ct[o0 + k], a1 = ct[o1 + k];"),
    ("refresh_mask_sign", "eta0[(size_t)i * n + k] = addmod(submod(sc1[k], lm, q), lift_small(e0[k], q), q);", "eta0[(size_t)i * n + k] = addmod(addmod(sc1[k], lm, q), lift_small(e0[k], q), q);"),
    ("refresh_alpha_sign", "eta1[(size_t)i * n + k] = addmod(submod(lm, sa[k], q), lift_small(e1[k], q), q);", "eta1[(size_t)i * n + k] = addmod(addmod(lm, sa[k], q), lift_small(e1[k], q), q);"),
    ("refresh_sums_eta0_twice", "acc = addmod(acc, shares[m][base + (size_t)(L + i) * n + k], q);", "acc = addmod(acc, shares[m][base + (size_t)i * n + k], q);"),
    ("refresh_alpha_of_wrong_index", "orc_bootstrap_alpha(c, group, ct_base + ci, ct_out + base + (size_t)L * n);", "orc_bootstrap_alpha(c, group, ct_base, ct_out + base + (size_t)L * n);"),
    ("encrypt_index_stuck", "uint32_t index = ct_base + ci;\n        orc_sample_ternary(c->p.seed, ORC_DOM_ENC_U", "uint32_t index = ct_base;\n        orc_sample_ternary(c->p.seed, ORC_DOM_ENC_U"),
    ("share_index_stuck", "ORC_DOM_DEC_E, party, group, ct_base + ci,", "ORC_DOM_DEC_E, party, group, ct_base,"),
    ("convert_index_stuck", "uint32_t index = ct_base + ci;\n        orc_sample_ternary(c->p.seed, ORC_DOM_CVT_U", "uint32_t index = ct_base;\n        orc_sample_ternary(c->p.seed, ORC_DOM_CVT_U"),
    ("refresh_index_stuck", "uint32_t index = ct_base + ci;\n        orc_sample_uniform(c->p.seed, ORC_DOM_BS_M", "uint32_t index = ct_base;\n        orc_sample_uniform(c->p.seed, ORC_DOM_BS_M"),
    ("small_negative_lift", "return v >= 0 ? (uint64_t)v : q - (uint64_t)(-(int64_t)v); }", "return v >= 0 ? (uint64_t)v : q - 1 - (uint64_t)(-(int64_t)v); }"),
    ("lambda_rounded_up", "        big_div_u64(&c->Lambda, p->t);\n", "        big_div_u64(&c->Lambda, p->t);\n        { big_t one_; big_set_u64(&one_, 1); big_add(&c->Lambda, &one_); }\n"),
    ("clamp_ignores_group_size", "c->clamp = (int64_t)(((p->t - 1) / 2) / kmax);", "c->clamp = (int64_t)((p->t - 1) / 2);"),
    ("crt_basis_includes_own_prime", "if (j != i) big_mul_u64(&c->Q_over_qi[i], p->q[j]);", "big_mul_u64(&c->Q_over_qi[i], p->q[j]);"),
    ("encode_truncates", "double rf = isnan(v) ? 0.0 : (double)rintf(v * scale);\n                if (rf > bound) rf = bound;\n                if (rf < -bound) rf = -bound;\n                r = (int64_t)rf;\n            }\n            z[j] =",
     "double rf = isnan(v) ? 0.0 : (double)truncf(v * scale);\n                if (rf > bound) rf = bound;\n                if (rf < -bound) rf = -bound;\n                r = (int64_t)rf;\n            }\n            z[j] ="),
    ("encode_negative_off_by_one", "            z[j] = r >= 0 ? (uint64_t)r : t - (uint64_t)(-r);", "            z[j] = r >= 0 ? (uint64_t)r : t - 1 - (uint64_t)(-r);"),
    ("encode_tail_not_zero", "            int64_t r = 0;\n            if (idx < n_values) {\n                float v = grad[idx];\n                double rf = isnan(v) ? 0.0 : (double)rintf(v * scale);\n                if (rf > bound) rf = bound;\n                if (rf < -bound) rf = -bound;\n                r = (int64_t)rf;\n            }\n            z[j] =",
     "            int64_t r = 1;\n            if (idx < n_values) {\n                float v = grad[idx];\n                double rf = isnan(v) ? 0.0 : (double)rintf(v * scale);\n                if (rf > bound) rf = bound;\n                if (rf < -bound) rf = -bound;\n                r = (int64_t)rf;\n            }\n            z[j] ="),
    ("coefficient_encode_upper_clamp_dropped", "            if (rf > bound) rf = bound;\n            if (rf < -bound) rf = -bound;\n            r = (int64_t)rf;\n        }\n        pt[idx] =",
     "            if (rf < -bound) rf = -bound;\n            r = (int64_t)rf;\n        }\n        pt[idx] ="),
    ("decode_scale_sign", "            out[idx] = ldexpf((float)v, -(int)c->p.frac_bits);\n        }\n    }\n    free(z);", "            out[idx] = ldexpf((float)v, (int)c->p.frac_bits);\n        }\n    }\n    free(z);"),
    ("round_group_shares_of_a_fresh_ciphertext", "orc_partial_decrypt(c, sks[m], agg, 1, members[m], group, (uint32_t)ci,", "orc_partial_decrypt(c, sks[m], ct, 1, members[m], group, (uint32_t)ci,"),
    # (orc_round_group returns decoded sums only, which do not depend on which randomness index it encrypts with)
    ("single_key_decrypt_without_c0", "                y[(size_t)i * n + k] = addmod(y[(size_t)i * n + k], c0[(size_t)i * n + k], q);\n", "                (void)c0;\n"),
    ("is_prime_without_the_squaring_loop", "        if (witness) return 0;\n", "        if (witness && r < 2) return 0;\n"),
    ("batch_forward_uses_limb_0_everywhere", "orc_ntt_forward(polys + (size_t)idx * c->n, c->n, c->p.q[idx % L], c->psi[idx % L]);",
     "orc_ntt_forward(polys + (size_t)idx * c->n, c->n, c->p.q[0], c->psi[0]);"),
    ("batch_inverse_root_of_wrong_limb", "orc_ntt_inverse(polys + (size_t)idx * c->n, c->n, c->p.q[idx % L], c->psi[idx % L]);",
     "orc_ntt_inverse(polys + (size_t)idx * c->n, c->n, c->p.q[idx % L], c->psi[(idx + 1) % L]);"),
    ("bench_polys_batch_and_limb_swapped", "orc_sample_uniform(c->p.seed, ORC_DOM_BENCH, i, 0, 0, b, c->p.q[i], c->n,",
     "orc_sample_uniform(c->p.seed, ORC_DOM_BENCH, b, 0, 0, i, c->p.q[i], c->n,"),
    ("clamp_bound_rounded_to_float32", "    double bound = (double)c->clamp;\n    for (uint32_t ci = 0; ci < C; ++ci) {",
     "    double bound = (double)(float)c->clamp;\n    for (uint32_t ci = 0; ci < C; ++ci) {"),
    ("coefficient_clamp_bound_rounded_to_float32", "double bound = (double)c->clamp;      /* exact comparison, as in orc_encode */",
     "double bound = (double)(float)c->clamp;"),
    ("update_step_sign", "w[j] = avg - step;", "w[j] = avg + step;"),
    ("update_divides_by_k_plus_one", "volatile float inv_k = 1.0f / (float)K;", "volatile float inv_k = 1.0f / (float)(K + 1);"),
]


def _build(args):
    name, old, new, out_dir, source = args
    assert source.count(old) == 1, f"mutant {name}: its text occurs {source.count(old)} times in the oracle"
    c_file = os.path.join(out_dir, name + ".c")
    so_file = os.path.join(out_dir, name + ".so")
    with open(c_file, "w") as f:
        f.write(source.replace(old, new))
    subprocess.check_call(["gcc", "-O1", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-w", "-I", os.path.dirname(SRC),
                           "-o", so_file, c_file, "-lm"])
    return so_file


def _pins_fail(so_file):
    env = dict(os.environ, D2MHE_ORACLE_LIBRARY=so_file, OMP_NUM_THREADS="2")
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q",
                        "-p", "no:cacheprovider"], cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)
    return r.returncode != 0, r.stdout[-400:]


def test_every_planted_mistake_fails_a_pin(tmp_path):
    source = open(SRC).read()
    with ThreadPoolExecutor(max_workers=4) as pool:
        libs = list(pool.map(_build, [(n, o, r, str(tmp_path), source) for n, o, r in MUTANTS]))
        results = list(pool.map(_pins_fail, libs))
    survivors = [name for (name, _, _), (failed, _) in zip(MUTANTS, results) if not failed]
    assert not survivors, f"no pin notices: {survivors}"


def test_the_unchanged_oracle_passes_through_the_same_route(tmp_path):
    """The child-process route itself: the unmodified source, built the same way, passes."""
    source = open(SRC).read()
    so_file = _build(("unchanged", "volatile float inv_k = 1.0f / (float)K;", "volatile float inv_k = 1.0f / (float)K;",
                      str(tmp_path), source))
    failed, tail = _pins_fail(so_file)
    assert not failed, tail
