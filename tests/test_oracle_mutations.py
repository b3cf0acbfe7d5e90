"""The pins must catch plausible mistakes in the oracle: each case plants one (a dropped term, a wrong sign or
index, a transposed operand) in a copy of the C source, builds it, and runs the pin files named beside it in a
child process against that build.  The run has to FAIL.  (CPU only: nothing here touches the GPU.)"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRC = os.path.join(ROOT, "oracle", "ckks_oracle.c")

# (name, text in ckks_oracle.c, replacement, pin files that must notice)
MUTANTS = [
    ("ntt_butterfly_swapped",
     "lo[j] = addmod(u, v, q);\n                hi[j] = submod(u, v, q);",
     "lo[j] = submod(u, v, q);\n                hi[j] = addmod(u, v, q);", ["test_oracle_ntt.py"]),
    ("intt_forward_twiddle", "u64 winv = c->pw[limb][2 * N - e];", "u64 winv = c->pw[limb][e];",
     ["test_oracle_ntt.py"]),
    ("intt_without_ninv", "a[j] = mulmod(a[j], ninv, q);", "a[j] = mulmod(a[j], 1, q);", ["test_oracle_ntt.py"]),
    ("automorphism_sign_dropped", "else out[r - N] = in[j] == 0 ? 0 : q - in[j];", "else out[r - N] = in[j];",
     ["test_oracle_galois.py"]),
    ("automorphism_gather_transposed", "out[k] = in[k2];", "out[k2] = in[k];", ["test_oracle_galois.py"]),
    ("rotation_generator", "g = (g * 5) % twoN;", "g = (g * 3) % twoN;", ["test_oracle_galois.py"]),
    ("modup_factor_dropped", "y[a * N + x] = mulmod(in[(u64)i * N + x], inv, qi);",
     "y[a * N + x] = in[(u64)i * N + x];", ["test_oracle_baseconv.py"]),
    ("modup_digit_bounds", "int lo = j * c->alpha, hi = lo + c->alpha;", "int lo = j * c->alpha, hi = lo + c->alpha - 1;",
     ["test_oracle_baseconv.py"]),
    ("moddown_sign", "mulmod(submod(u[(u64)i * N + x], w[x], qi), Pinv, qi);",
     "mulmod(addmod(u[(u64)i * N + x], w[x], qi), Pinv, qi);", ["test_oracle_baseconv.py"]),
    ("moddown_p_not_inverted", "u64 Pinv = invmod(Pmod, qi);", "u64 Pinv = Pmod;", ["test_oracle_baseconv.py"]),
    ("rescale_no_rounding_offset", "r[x] = addmod(r[x], h, ql);", "r[x] = addmod(r[x], 0, ql);",
     ["test_oracle_baseconv.py"]),
    ("rescale_wrong_inverse", "u64 qlinv = invmod(ql % qi, qi);", "u64 qlinv = ql % qi;", ["test_oracle_baseconv.py"]),
    ("key_components_swapped", "const u64 *kk = key + (((u64)j * 2 + comp) * (L + K) + gl) * N;\n"
     "                    u64 *uu = u + ((u64)comp * W + t) * N;\n"
     "                    for (u64 x = 0; x < N; x++) uu[x] = addmod(uu[x], mulmod(perm[x], kk[x], mt), mt);\n"
     "                }\n                free(perm);\n            }\n        orc_moddown(c, level, u, o);",
     "const u64 *kk = key + (((u64)j * 2 + (1 - comp)) * (L + K) + gl) * N;\n"
     "                    u64 *uu = u + ((u64)comp * W + t) * N;\n"
     "                    for (u64 x = 0; x < N; x++) uu[x] = addmod(uu[x], mulmod(perm[x], kk[x], mt), mt);\n"
     "                }\n                free(perm);\n            }\n        orc_moddown(c, level, u, o);",
     ["test_oracle_keyswitch.py"]),
    ("rotated_c0_dropped", "o[(u64)i * N + x] = addmod(o[(u64)i * N + x], tmp[x], c->mod[i]);",
     "o[(u64)i * N + x] = addmod(o[(u64)i * N + x], 0, c->mod[i]);", ["test_oracle_keyswitch.py"]),
    ("key_factor_on_every_digit", "if (t < L && t / c->alpha == j) {", "if (t < L) {", ["test_oracle_keyswitch.py"]),
    ("key_minus_as_sign", "u64 v = submod(en[x], as, mt);", "u64 v = addmod(en[x], as, mt);",
     ["test_oracle_keyswitch.py"]),
    ("negative_coefficients", "return r ? q - r : 0;", "return r;", ["test_oracle_matmul.py"]),
    ("giant_step_amount", "u64 g = orc_galois_elt(c, (i64)p * N1 * m, 0);", "u64 g = orc_galois_elt(c, (i64)p * m, 0);",
     ["test_oracle_matmul.py"]),
    ("diagonal_index_transposed", "((((u64)b * N2 + p) * G + g) * N1 + q) * N;",
     "((((u64)b * N2 + p) * N1 + q) * G + g) * N;", ["test_oracle_matmul.py"]),
    ("merged_c0_dropped", "if (ci < level) v = addmod(v, c0_acc[(u64)ci * N + k], qi);",
     "if (ci < level) v = addmod(v, 0, qi);", ["test_oracle_matmul.py"]),
    ("merged_skips_first_rotation", "for (int p = 1; p < N2; p++)\n                orc_switch_accumulate(",
     "for (int p = 2; p < N2; p++)\n                orc_switch_accumulate(", ["test_oracle_matmul.py"]),
    ("conj_added_twice", "orc_rotate_hoisted(c, y, level, &g, 1, &conj_key, rot);",
     "orc_rotate_hoisted(c, y, level, &g, 1, &conj_key, rot); memcpy(y, rot, sizeof(u64) * 2 * level * N);",
     ["test_oracle_complex.py"]),
    ("conj_per_accumulator_skips_the_first", "for (int p = 0; p < N2; p++) {\n                u64 *a = acc + (u64)p * ctw;",
     "for (int p = 1; p < N2; p++) {\n                u64 *a = acc + (u64)p * ctw;", ["test_oracle_complex.py"]),
    ("bias_without_scale_factor", "u64 bm = bias_mul % qi;", "u64 bm = 1;", ["test_oracle_matmul.py"]),
    ("ctmul_cross_term_dropped",
     "t1[(u64)i * N + x] = addmod(mulmod(a0[x], b1[x], q), mulmod(a1[x], b0[x], q), q);",
     "t1[(u64)i * N + x] = mulmod(a0[x], b1[x], q);", ["test_oracle_ctmul.py"]),
    ("relin_target_is_s", "tg[(u64)t * N + x] = mulmod(sn[(u64)t * N + x], sn[(u64)t * N + x], c->mod[t]);",
     "tg[(u64)t * N + x] = sn[(u64)t * N + x];", ["test_oracle_ctmul.py"]),
    ("ptmul_one_component", "for (int comp = 0; comp < 2; comp++)\n        for (int i = 0; i < level; i++) {\n"
     "            u64 q = c->mod[i];\n            u64 off = ((u64)comp * level + i) * N;",
     "for (int comp = 0; comp < 1; comp++)\n        for (int i = 0; i < level; i++) {\n"
     "            u64 q = c->mod[i];\n            u64 off = ((u64)comp * level + i) * N;", ["test_oracle_primitives.py"]),
    ("shift_bank_masks_swapped", "orc_ptmul(c, rot + (u64)(2 * i) * ctw, level, masks + (u64)(2 * i) * ptw, out + (u64)i * ctw);",
     "orc_ptmul(c, rot + (u64)(2 * i) * ctw, level, masks + (u64)(2 * i + 1) * ptw, out + (u64)i * ctw);",
     ["test_oracle_primitives.py"]),
]


def _run(case, tmp):
    name, old, new, files = case
    src = open(SRC).read()
    if src.count(old) != 1:
        return name, "source text not found exactly once"
    c_path = os.path.join(tmp, name + ".c")
    so_path = os.path.join(tmp, name + ".so")
    with open(c_path, "w") as f:
        f.write(src.replace(old, new))
    subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-w", "-o", so_path, c_path])
    env = dict(os.environ, CKKS_ORACLE_LIB=so_path, OMP_NUM_THREADS="2")
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider"] +
                       [os.path.join(HERE, f) for f in files], cwd=ROOT, env=env, stdout=subprocess.PIPE,
                       stderr=subprocess.STDOUT, timeout=600)
    out = r.stdout.decode(errors="replace")
    if r.returncode == 0:
        return name, "pins passed on the broken oracle"
    if " failed" not in out or "rror while" in out or "ImportError" in out:
        return name, "child run broke without a pin failing:\n" + out[-600:]
    return name, None


def test_unchanged_copy_passes_the_same_way(tmp_path):
    """Control: the same child-process route with an unmodified copy of the source passes, so a failure below
    comes from the planted mistake and not from the route."""
    src = open(SRC).read()
    c_path, so_path = str(tmp_path / "control.c"), str(tmp_path / "control.so")
    with open(c_path, "w") as f:
        f.write(src)
    subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-w", "-o", so_path, c_path])
    files = sorted({f for m in MUTANTS for f in m[3]})
    env = dict(os.environ, CKKS_ORACLE_LIB=so_path)
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider"] +
                       [os.path.join(HERE, f) for f in files], cwd=ROOT, env=env, stdout=subprocess.PIPE,
                       stderr=subprocess.STDOUT, timeout=900)
    assert r.returncode == 0, r.stdout.decode(errors="replace")[-800:]


def test_every_planted_mistake_is_caught(tmp_path):
    with ThreadPoolExecutor(max_workers=4) as pool:
        results = list(pool.map(lambda c: _run(c, str(tmp_path)), MUTANTS))
    missed = [(n, why) for n, why in results if why]
    assert not missed, missed
