"""Do the pins bite?  Each case plants one plausible mistake in a COPY of the oracle (a dropped term, a
wrong sign, a wrong index, a missing factor, a step left out), on the CPU, and runs the pin tests of
test_oracle_pins.py against that copy in a fresh interpreter: they must fail.  The untouched copy must pass.

The mistakes are textual edits of the copy; the oracle itself carries no test hooks.  None of them makes
the code read outside its arrays.
"""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
INC = "sparse_mlp_oracle_impl.inc"
INIT = "__init__.py"

# (name, file, text as it stands, text with the mistake); the text must occur exactly once
MUTATIONS = [
    ("forward drops the bias", INC,
     "double acc = bias ? (double)bias[i] : 0.0;", "double acc = 0.0 * (bias ? (double)bias[i] : 0.0);"),
    ("forward skips the first entry of a row", INC,
     "for (int32_t p = indptr[i]; p < indptr[i + 1]; ++p) {\n                double t = (double)values[p] * (double)X[",
     "for (int32_t p = indptr[i] + (indptr[i] < indptr[i + 1]); p < indptr[i + 1]; ++p) {\n                double t = (double)values[p] * (double)X["),
    ("ReLU inverted", INC, "if (relu && !(acc > 0.0)) acc = 0.0;", "if (relu && (acc > 0.0)) acc = 0.0;"),
    ("transposed product subtracts", INC, "acc[j * batch + c] += t;", "acc[j * batch + c] -= t;"),
    ("transposed product takes the row's first weight", INC,
     "double t = (double)values[p] * (double)dZ[(int64_t)i * lddz + c];",
     "double t = (double)values[indptr[i]] * (double)dZ[(int64_t)i * lddz + c];"),
    ("ReLU derivative 1 at zero", INC, "> (REAL)0) ? dA[", ">= (REAL)0) ? dA["),
    ("SDDMM reads the row's first column", INC,
     "double t = (double)dZ[(int64_t)i * lddz + c] * (double)X[(int64_t)indices[p] * ldx + c];",
     "double t = (double)dZ[(int64_t)i * lddz + c] * (double)X[(int64_t)indices[indptr[i]] * ldx + c];"),
    ("bias gradient sums absolute values", INC,
     "double t = (double)dZ[(int64_t)i * lddz + c];\n                acc += t;",
     "double t = fabs((double)dZ[(int64_t)i * lddz + c]);\n                acc += t;"),
    ("loss gradient not divided by the batch size", INC,
     "(REAL)((pr - hot) / (double)batch);", "(REAL)(pr - hot);"),
    ("loss adds the target logit", INC, "loss += lse - zt;", "loss += lse + zt;"),
    ("log-sum-exp forgets the maximum", INC, "double lse = m + log(sum);", "double lse = log(sum);"),
    ("momentum step with the wrong sign", INC,
     "double vn = mu * (double)v[p] - lr * (double)g[p];", "double vn = mu * (double)v[p] + lr * (double)g[p];"),
    ("momentum factor dropped", INC,
     "double vn = mu * (double)v[p] - lr * (double)g[p];", "double vn = (double)v[p] - lr * (double)g[p];"),
    ("Nesterov look-ahead without the momentum factor", INC,
     "wn = (double)w[p] + mu * (double)vs - lr * (double)g[p];", "wn = (double)w[p] + (double)vs - lr * (double)g[p];"),
    ("backward pass forgets the ReLU derivative", INIT,
     "dZ[l] = relu_backward(dA[l], A[l], dtype)", "dZ[l] = np.asarray(dA[l], dtype=dtype)"),
    ("weight gradient from the layer's output instead of its input", INIT,
     "inp = X if l == 0 else A[l - 1]", "inp = X if l == 0 else A[l - 1] * 0 + 1"),
    # normalisers (the sums of |terms| that set the parity tolerances)
    ("normaliser of the update drops |lr|", INC,
     "double sg = fabs(lr) * (Sg ? Sg[p] : fabs((double)g[p]));", "double sg = (Sg ? Sg[p] : fabs((double)g[p]));"),
    ("normaliser of the velocity taken from the new velocity", INC,
     "double sv = fabs(mu * (double)v[p]) + sg;", "double sv = fabs(vn) + sg;"),
    ("normaliser of the velocity drops the momentum term", INC,
     "double sv = fabs(mu * (double)v[p]) + sg;", "double sv = sg;"),
    ("Nesterov weight normaliser drops the momentum factor", INC,
     "sw = fabs((double)w[p]) + fabs(mu) * sv + sg;", "sw = fabs((double)w[p]) + sv + sg;"),
    ("weight normaliser drops |w|", INC,
     "sw = fabs((double)w[p]) + sv;", "sw = sv;"),
    ("loss normaliser doubled", INC, "out[1] = sloss / (double)batch;", "out[1] = 2.0 * sloss / (double)batch;"),
    ("loss normaliser not averaged over the batch", INC, "out[1] = sloss / (double)batch;", "out[1] = sloss;"),
    ("loss normaliser is |lse - z_t|", INC, "sloss += fabs(lse) + fabs(zt);", "sloss += fabs(lse - zt);"),
    ("gradient normaliser of dZ_L subtracts the one-hot term", INC,
     "SdZ[(int64_t)i * batch + c] = (pr + hot) / (double)batch;", "SdZ[(int64_t)i * batch + c] = (pr - hot) / (double)batch;"),
    ("step hands the update no gradient normaliser", INIT,
     'momentum(st["values"], st["vel_w"], g[l], lr, mu, Sg[l], dtype, nesterov)',
     'momentum(st["values"], st["vel_w"], g[l], lr, mu, None, dtype, nesterov)'),
    ("biases never updated", INIT,
     'momentum(st["bias"], st["vel_b"], db[l], lr, mu, Sdb[l], dtype, nesterov)',
     'momentum(st["bias"], st["vel_b"], 0 * db[l], lr, mu, Sdb[l], dtype, nesterov)'),
]


def run_pins(oracle_parent):
    env = dict(os.environ, NERVA_ORACLE_DIR=oracle_parent)
    return subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q",
                           "-p", "no:cacheprovider"], cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)


def copy_oracle(tmp_path):
    dst = tmp_path / "oracle"
    shutil.copytree(os.path.join(ROOT, "oracle"), dst, ignore=shutil.ignore_patterns("*.so", "__pycache__"))
    return dst


def test_untouched_copy_passes(tmp_path):
    copy_oracle(tmp_path)
    r = run_pins(str(tmp_path))
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-2000:]


@pytest.mark.parametrize("name,fname,old,new", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_planted_mistake_is_caught(tmp_path, name, fname, old, new):
    dst = copy_oracle(tmp_path)
    path = dst / fname
    text = path.read_text()
    assert text.count(old) == 1, f"{name}: the text to replace occurs {text.count(old)} times in {fname}"
    path.write_text(text.replace(old, new))
    r = run_pins(str(tmp_path))
    assert r.returncode == 1, f"{name}: the pins did not fail\n" + r.stdout[-1500:] + r.stderr[-1500:]
    assert "passed" not in r.stdout.splitlines()[-1] or "failed" in r.stdout.splitlines()[-1]
