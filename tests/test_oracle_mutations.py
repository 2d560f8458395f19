"""The pins must notice a plausible mistake anywhere in the oracle.  Each case below plants one mistake in a copy of
oracle/astra_oracle.c (a dropped term, a wrong sign or index, a transposed operand, a swapped stream), builds it, and
runs the pin file that covers the function against that build in a separate process: the pins have to FAIL.  The
unmodified copy has to pass, which shows the harness itself works.  Everything runs on the CPU."""
import os
import subprocess
import sys
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "astra_oracle.c")

# (pin file, text in the source (must occur exactly once), replacement, what the mistake is)
MUTATIONS = [
    ("test_oracle_vq.py", "if (dist < best) {          /*", "if (dist <= best) {          /*", "ties go to the highest index"),
    ("test_oracle_vq.py", "const double diff = (double)e[j] - (double)z[j];", "const double diff = (double)e[j] + (double)z[j];", "distance to -x"),
    ("test_oracle_vq.py", "const float* z = x + t * (int64_t)D + (int64_t)g * dg;", "const float* z = x + t * (int64_t)D;", "every group reads slice 0"),
    ("test_oracle_vq.py", "const float* e = codebook + ((int64_t)g * K + codes[t * (int64_t)G + g]) * dg;",
     "const float* e = codebook + ((int64_t)codes[t * (int64_t)G + g]) * dg;", "decode ignores the group's codebook"),
    ("test_oracle_attention.py", "const float* wr = w + (int64_t)i * d_out;\n            for (int c = 0; c < d_out; ++c) o[c] += xi * (double)wr[c];",
     "for (int c = 0; c < d_out; ++c) o[c] += xi * (double)w[(int64_t)c * d_in + i];", "linear uses the transposed weight"),
    ("test_oracle_attention.py", "allowed[j] = !causal ? 1 : (is_local ? (jj <= i) : (jj < n_before));",
     "allowed[j] = !causal ? 1 : (is_local ? (jj < i) : (jj < n_before));", "causal mask hides the diagonal"),
    ("test_oracle_attention.py", "allowed[j] = !causal ? 1 : (is_local ? (jj <= i) : (jj < n_before));",
     "allowed[j] = !causal ? 1 : (is_local ? (jj <= i) : 1);", "causal rows see the non-local rows after the chunk"),
    ("test_oracle_attention.py", "const int hk = h / rep;\n            const double* qi", "const int hk = h % n_kv_heads;\n            const double* qi",
     "grouped-query heads interleaved instead of blocked"),
    ("test_oracle_attention.py", "if (scale == 0.0) scale = 1.0 / sqrt((double)head_dim);\n    const int64_t rows",
     "if (scale == 0.0) scale = 1.0 / (double)head_dim;\n    const int64_t rows", "logits scaled by 1/d_k"),
    ("test_oracle_attention.py", "const double* vj = (is_local ? v_loc : v_hat) + ((int64_t)jj * n_kv_heads + hk) * head_dim;",
     "const double* vj = (is_local ? v_loc : v_loc) + ((int64_t)(is_local ? jj : 0) * n_kv_heads + hk) * head_dim;", "non-local values never used"),
    ("test_oracle_lost_codes.py", "if (!is_local && valid_hat && !valid_hat[jj]) allowed[j] = 0;", "if (!is_local && valid_hat && valid_hat[jj]) allowed[j] = 0;",
     "the arrived tokens are dropped instead of the lost ones"),
    ("test_oracle_block.py", "for (int i = 0; i < D; ++i) var += (r[i] - mean) * (r[i] - mean);\n        var /= D;",
     "for (int i = 0; i < D; ++i) var += (r[i] - mean) * (r[i] - mean);\n        var /= (D - 1);", "unbiased variance in the norms"),
    ("test_oracle_block.py", "else r = act_silu(v) * a[t * (int64_t)n1 + d_ff + j];", "else r = v * act_silu(a[t * (int64_t)n1 + d_ff + j]);", "gate and up swapped"),
    ("test_oracle_block.py", "for (int64_t i = 0; i < n; ++i) r[i] = x[i] + y[i];", "for (int64_t i = 0; i < n; ++i) r[i] = h[i] + y[i];",
     "the residual adds the normalised tensor"),
    ("test_oracle_kv_variant.py", "if (!rc) rc = oracle_vq_encode(Vf + (int64_t)n_cls * dkv, n_local, dkv, G, K, codebook_v, codes_v_local, gap_v);",
     "if (!rc) rc = oracle_vq_encode(Vf + (int64_t)n_cls * dkv, n_local, dkv, G, K, codebook_k, codes_v_local, gap_v);", "V rows quantised with the K codebook"),
    ("test_oracle_decode.py", "const float* kr = khf + ((int64_t)(t - n_local) * n_kv_heads + j) * head_dim;",
     "const float* kr = vhf + ((int64_t)(t - n_local) * n_kv_heads + j) * head_dim;", "index-cache scores use the value rows"),
    ("test_oracle_training.py", "s[j] += (double)xs[j];\n                const double d = (double)xs[j] - (double)c[j];",
     "s[j] += (double)xs[j];\n                const double d = (double)xs[j];", "commitment sum without the codeword"),
    ("test_oracle_training.py", "codebook_new[i * dg + j] = n > 0.0 ? m / n : (double)codebook_old[i * dg + j];",
     "codebook_new[i * dg + j] = n > 0.0 ? m / n : 0.0;", "dead codewords are zeroed"),
    ("test_oracle_training.py", "xi += (double)l_factor[(int64_t)i * D + j] * (double)z[t * (int64_t)D + j];",
     "xi += (double)l_factor[(int64_t)j * D + i] * (double)z[t * (int64_t)D + j];", "NAVQ multiplies by the transposed factor"),
    ("test_oracle_rope.py", "x[2 * i + 1] = x0 * sn + x1 * c;", "x[2 * i + 1] = x1 * c - x0 * sn;", "rotation turns the other way in the second component"),
    ("test_oracle_rope.py", "const double theta = pow(base, -2.0 * (double)i / (double)head_dim);",
     "const double theta = pow(base, -(double)i / (double)head_dim);", "angle exponent i/d instead of 2i/d"),
    ("test_oracle_rope.py", "pos[Tq + j] = j < n_before ? j : (int64_t)j + n_local;", "pos[Tq + j] = j;", "non-local rows after the chunk keep their list index as position"),
    ("test_oracle_rope.py", "pos[i] = i < n_cls ? -1 : (int64_t)n_before + (i - n_cls);", "pos[i] = i < n_cls ? -1 : (int64_t)(i - n_cls);",
     "local rows counted from the start of the chunk"),
    ("test_oracle_rope.py", "if (!rc) rc = oracle_rope(Kh, Tn, n_kv_heads, head_dim, pos + Tq, rope_base);", "", "rebuilt keys are not rotated"),
]


def build_and_run(source_text, pin_file, tmp):
    c_path, so_path = os.path.join(tmp, "mutant.c"), os.path.join(tmp, "mutant.so")
    with open(c_path, "w") as f:
        f.write(source_text)
    subprocess.run(["gcc", "-O1", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-fno-fast-math", "-ffp-contract=off", c_path, "-o",
                    so_path, "-lm"], check=True)
    env = dict(os.environ, ASTRA_ORACLE_LIB_OVERRIDE=so_path)
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", os.path.join(ROOT, "tests", pin_file)],
                       cwd=ROOT, env=env, capture_output=True, text=True, timeout=300)
    return r.returncode, r.stdout[-600:]


def test_the_unmodified_source_passes_through_the_same_harness():
    src = open(SRC).read()
    with tempfile.TemporaryDirectory() as tmp:
        for pin_file in sorted({m[0] for m in MUTATIONS}):
            rc, out = build_and_run(src, pin_file, tmp)
            assert rc == 0, f"{pin_file} fails on the unmodified oracle:\n{out}"


@pytest.mark.parametrize("pin_file,old,new,what", MUTATIONS, ids=[m[3] for m in MUTATIONS])
def test_pins_catch_a_planted_mistake(pin_file, old, new, what):
    src = open(SRC).read()
    assert src.count(old) == 1, f"mutation site not unique: {old[:60]}"
    with tempfile.TemporaryDirectory() as tmp:
        rc, out = build_and_run(src.replace(old, new), pin_file, tmp)
    assert rc != 0, f"planted mistake not noticed ({what}); pin output:\n{out}"
