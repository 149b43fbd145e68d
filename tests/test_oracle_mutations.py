"""Planted mistakes in the CPU oracle must be caught by its pins (CPU only, nothing touches a GPU).

Each mutation is a single-line change of oracle/ckks_oracle.c (swapped operands, a dropped factor, a
wrong index map ...), compiled into a scratch library; the named pin test is then run against it in a
subprocess and must fail.
"""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "ckks_oracle.c")

MUTATIONS = [
    ("x[j + t] = orc_submod(u, v, m);", "x[j + t] = orc_submod(v, u, m);", "test_ntt_equals_bigint_definition"),
    ("uint64_t y = orc_mulmod(x[i * stride + n], hat_inv[i], src[i]);", "uint64_t y = x[i * stride + n];", "test_modup_vs_bigint_crt"),
    ("orc_mulmod(orc_submod(in[(size_t)i * N + n], conv[n], q), Pinv, q)", "orc_mulmod(orc_submod(conv[n], in[(size_t)i * N + n], q), Pinv, q)", "test_moddown_vs_bigint"),
    ("uint64_t e = ((uint64_t)g * (2ull * bitrev(j, logN) + 1)) % (2 * N);", "uint64_t e = ((uint64_t)g * (2ull * j + 1)) % (2 * N);", "test_automorphism_coeff_by_substitution_and_eval_consistency"),
    ("else out[u - N] = (m - in[t]) % m;", "else out[u - N] = in[t];", "test_automorphism_coeff_by_substitution_and_eval_consistency"),
    ("if (i >= j * alpha && i < (j + 1) * alpha) {\n            Pm = 1;", "if (i < L) {\n            Pm = 1;", "test_switch_key_structure"),
    ("orc_keyswitch(rot + (size_t)L * N, rk, out", "orc_keyswitch(ct + (size_t)L * N, rk, out", "test_hrot_decrypts_to_rotated"),
    ("orc_addmod(orc_mulmod(a1[n], b2[n], m), orc_mulmod(a2[n], b1[n], m), m);", "orc_addmod(orc_mulmod(a1[n], b2[n], m), orc_mulmod(a2[n], b2[n], m), m);", "test_hmult_relin_decrypts_to_product"),
    ("if (galois != 1) { orc_automorph_eval(src, perm, p->logN, galois); src = perm; }", "", "test_hoisted_mac_per_rotation_and_linearity"),
    ("limbs_ntt(cp, p, 0, D, 2, D, 1);", "limbs_ntt(cp, p, 0, D, 2, D, 0);", "test_keyswitch_decrypt_and_bound"),
    ("uint64_t n_inv = orc_invmod(N % m, m);", "uint64_t n_inv = 1;", "test_ntt_equals_bigint_definition"),
    ("memcpy(dst, in + (size_t)t * N, N * sizeof(uint64_t));", "memset(dst, 0, N * sizeof(uint64_t));", "test_modup_vs_bigint_crt"),
    ("out[(size_t)i * N + n] = orc_mulmod(orc_submod(in[(size_t)i * N + n], r[n], q), qinv, q);", "out[(size_t)i * N + n] = orc_mulmod(orc_addmod(in[(size_t)i * N + n], r[n], q), qinv, q);", "test_rescale_vs_bigint_floor_division"),
    ("uint64_t qinv = orc_invmod(qlast % q, q);", "uint64_t qinv = orc_invmod(q % qlast, qlast);", "test_rescale_decryption_identity"),
    ("for (size_t n = 0; n < N; n++) r[n] = x[n] % q;", "for (size_t n = 0; n < N; n++) r[n] = (x[n] + qlast / 2) % q;", "test_rescale_vs_bigint_floor_division"),
    ("else orc_conv(in + (size_t)lo * N, N, N, vprimes + lo, hi - lo, vprimes[t], dst);", "else orc_conv(in + (size_t)lo * N, N, N, vprimes + lo, alpha, vprimes[t], dst);", "test_modup_level_vs_bigint_crt"),
    ("        uint32_t src = i < ell ? i : L + (i - ell);\n        v->vprimes[i] = primes[src];", "        uint32_t src = i;\n        v->vprimes[i] = primes[src];", "test_keyswitch_level_decrypt_and_bound"),
    ("key_inner_product(dhat, kc, cp, &v.p, 1);", "key_inner_product(dhat, key, cp, &v.p, 1);", "test_keyswitch_level_decrypt_and_bound"),
    ("orc_keyswitch_level(rot + (size_t)ell * N, rk, out", "orc_keyswitch_level(ct + (size_t)ell * N, rk, out", "test_hmult_hrot_level_decrypt"),
    ("        key_inner_product(dhat, kc, cp, &v.p, galois[r]);", "        key_inner_product(dhat, kc, cp, &v.p, 1);", "test_hoisted_mac_level"),
    ("                const uint64_t* ptr = pt + ((size_t)r * D + i) * N;\n                const uint64_t* src = cp", "                const uint64_t* ptr = pt + ((size_t)r * D + (i % ell)) * N;\n                const uint64_t* src = cp", "test_double_hoisted_mac"),
    ("            orc_automorph_eval(ct + (size_t)i * N, sb, logN, galois[r]);\n            const uint64_t* ptr = pt + ((size_t)r * D + i) * N;", "            orc_automorph_eval(ct + (size_t)i * N, sb, logN, 1);\n            const uint64_t* ptr = pt + ((size_t)r * D + i) * N;", "test_double_hoisted_mac"),
    ("    moddown_eval(C, ks, &v.p);", "    moddown_eval(cp, ks, &v.p);", "test_double_hoisted_mac"),
    ("orc_conv(in + (size_t)T * N, N, N, vprimes + T, ns, q, conv);", "orc_conv(in + (size_t)(T + 1) * N, N, N, vprimes + T + 1, ns - 1, q, conv);", "test_moddown_merged_vs_bigint"),
    ("            C0[n] = orc_addmod(C0[n], orc_mulmod(Pm, d0, m), m);", "            C0[n] = orc_addmod(C0[n], d0, m);", "test_hmult_relin_rescale_merged"),
    ("            C1[n] = orc_addmod(C1[n], orc_mulmod(Pm, d1, m), m);", "            C1[n] = orc_addmod(C1[n], orc_mulmod(Pm, d0, m), m);", "test_hmult_relin_rescale_merged"),
    ("                dst[n] = orc_addmod(dst[n], orc_mulmod(Pm, orc_mulmod(ptr[n], sb[n], m), m), m);", "                dst[n] = orc_addmod(dst[n], orc_mulmod(ptr[n], sb[n], m), m);", "test_double_hoisted_mac_rescale_merged"),
]


@pytest.mark.parametrize("idx", range(len(MUTATIONS)))
def test_planted_mistake_is_caught(idx, tmp_path):
    old, new, victim = MUTATIONS[idx]
    text = open(SRC).read()
    assert text.count(old) >= 1, "mutation target not found: the oracle source changed"
    mutated = tmp_path / "ckks_oracle.c"
    mutated.write_text(text.replace(old, new, 1))
    lib = tmp_path / "libckks_oracle_mut.so"
    subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-w", "-o", str(lib), str(mutated)])
    env = dict(os.environ, CKKS_ORACLE_LIB=str(lib))
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q",
                        "-k", victim, "-p", "no:cacheprovider"], capture_output=True, text=True, env=env, cwd=ROOT)
    assert r.returncode != 0 and "failed" in r.stdout, "the pins did not notice: " + new
