"""Do the pins bite?  Each case plants ONE plausible mistake in a copy of the oracle's C source (a dropped
term, a wrong sign or index, a swapped operand, an off-by-one), builds it, and runs the pin tests of that
operator against it in a child process: they must FAIL.  The mistakes live in the oracle, on the CPU; the
unmodified oracle passing the same tests is what the rest of the suite shows.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "lsq_oracle.c")

# (name, text in the oracle, replacement, which occurrence, pin module that must catch it)
MUTANTS = [
    ("philox: nine rounds", "round < 10", "round < 9", 0, "philox"),
    ("philox: multipliers on the wrong words", "uint64_t p0 = M0 * c0;", "uint64_t p0 = M0 * c2;", 0, "philox"),
    ("philox: second key word not bumped", "k0 += W0; k1 += W1;", "k0 += W0;", 0, "philox"),
    ("philox: output words permuted", "c0 = n0; c1 = n1; c2 = n2; c3 = n3;", "c0 = n2; c1 = n1; c2 = n0; c3 = n3;", 0, "philox"),
    ("dropout: halves of a word swapped", "(16 * (lane & 1))", "(16 * (1 - (lane & 1)))", 0, "philox"),
    ("dropout: keeps BELOW the threshold", "dropout_bits(e, seed, offset) >= t16", "dropout_bits(e, seed, offset) < t16", 0, "philox"),
    ("dropout: one call per 4 elements", "uint64_t g = e >> 3;", "uint64_t g = e >> 2;", 0, "philox"),
    ("layernorm: unbiased variance", "double rs = 1.0 / sqrt(q / hidden + eps);", "double rs = 1.0 / sqrt(q / (hidden - 1) + eps);", 0, "layernorm"),
    ("layernorm: eps outside the root", "double rs = 1.0 / sqrt(q / hidden + eps);", "double rs = 1.0 / (sqrt(q / hidden) + eps);", 0, "layernorm"),
    ("layernorm: beta dropped", "* rs) + load(beta, i, dt);", "* rs);", 0, "layernorm"),
    ("layernorm bwd: second row sum dropped", "double v = g / sigma - (s1 + xh * s2) / (hidden * sigma);",
     "double v = g / sigma - (s1) / (hidden * sigma);", 0, "layernorm"),
    ("layernorm bwd: sign of the correction", "double v = g / sigma - (s1 + xh * s2) / (hidden * sigma);",
     "double v = g / sigma + (s1 + xh * s2) / (hidden * sigma);", 0, "layernorm"),
    ("layernorm bwd: gamma missing from the row sums", "double g = load(dy, o + j, dt) * load(gamma, j, dt);",
     "double g = load(dy, o + j, dt);", 0, "layernorm"),
    ("layernorm bwd: dgamma against raw x", "dgamma[i] += g * ((load(x, o + i, dt) - mu) / sigma);",
     "dgamma[i] += g * load(x, o + i, dt);", 0, "layernorm"),
    ("bdr: survivors not rescaled", "? z * scale : 0.0;\n            out[e] = load(residual", "? z : 0.0;\n            out[e] = load(residual", 0, "bdr"),
    ("bdr: bias added after the dropout", "double z = load(x, e, dt) + (bias ? load(bias, i, dt) : 0.0);\n            double d = keep_element(e0 + (uint64_t)e, p, t16, seed, offset) ? z * scale : 0.0;",
     "double z = load(x, e, dt);\n            double d = (keep_element(e0 + (uint64_t)e, p, t16, seed, offset) ? z * scale : 0.0) + (bias ? load(bias, i, dt) : 0.0);", 0, "bdr"),
    ("bdr bwd: gradient not masked", "? load(dy, e, dt) * scale : 0.0;\n        }\n    if (dbias)", "? load(dy, e, dt) * scale : load(dy, e, dt);\n        }\n    if (dbias)", 0, "bdr"),
    ("softmax: causal mask off by one", "if (causal && j > i + (k_len - q_len)) return 0;", "if (causal && j >= i + (k_len - q_len)) return 0;", 0, "softmax"),
    ("softmax: scale applied after the exponential", "v = exp(scale * load(x, o + j, dt) - mx) / Z;", "v = scale * exp(load(x, o + j, dt) - mx) / Z;", 0, "softmax"),
    ("softmax: key length ignored", "if (j >= klen_b) return 0;", "if (j > klen_b) return 0;", 0, "softmax"),
    ("softmax bwd: scale dropped", "v = scale * load(y, o + j, dt) * (g - dot);", "v = load(y, o + j, dt) * (g - dot);", 0, "softmax"),
    ("softmax bwd: dot term dropped", "v = scale * load(y, o + j, dt) * (g - dot);", "v = scale * load(y, o + j, dt) * g;", 0, "softmax"),
    ("xent: smoothing mass spread over the other classes only", "double pi = alpha / vocab + (i == k ? 1.0 - alpha : 0.0);",
     "double pi = (i == k ? 1.0 - alpha : alpha / (vocab - 1));", 0, "xent"),
    ("xent: log-sum-exp without the maximum added back", "double l = mx + log(z);\n        lse[t] = l;", "double l = log(z);\n        lse[t] = l;", 0, "xent"),
    ("xent bwd: smoothing term dropped", "double gr = q - alpha / vocab;", "double gr = q;", 0, "xent"),
    ("xent bwd: sign of the target term", "if (i == k) gr -= 1.0 - alpha;", "if (i == k) gr += 1.0 - alpha;", 0, "xent"),
    ("xent bwd: ignored rows get a gradient", "for (int i = 0; i < vocab; ++i) dlogits[o + i] = 0.0;\n            continue;",
     "for (int i = 0; i < vocab; ++i) dlogits[o + i] = 0.0;", 0, "xent"),
    ("adam: eps inside the root", "double upd = (mi / c1) / (sqrt(vi / c2) + eps);", "double upd = (mi / c1) / sqrt(vi / c2 + eps);", 0, "adam"),
    ("adam: second moment without the square", "(1.0 - beta2) * gh * gh;", "(1.0 - beta2) * gh;", 0, "adam"),
    ("adam: bias corrections swapped", "double upd = (mi / c1) / (sqrt(vi / c2) + eps);", "double upd = (mi / c2) / (sqrt(vi / c1) + eps);", 0, "adam"),
    ("adam: decoupled decay applied to the gradient", "if (adamw) upd += weight_decay * pi;", "if (adamw) gh += weight_decay * pi;", 0, "adam"),
    ("adam: step sign", "p_out[i] = pi - lr * upd;", "p_out[i] = pi + lr * upd;", 0, "adam"),
    ("gelu: erf argument not divided by sqrt 2", "return 0.5 * z * erfc(-z / sqrt(2.0));", "return 0.5 * z * erfc(-z);", 0, "bias_act"),
    ("gelu slope: density term dropped", "return 0.5 * erfc(-z / sqrt(2.0)) + z * exp(-0.5 * z * z) / sqrt(2.0 * PI);",
     "return 0.5 * erfc(-z / sqrt(2.0));", 0, "bias_act"),
    ("gelu-tanh: cubic coefficient", "double u = sqrt(2.0 / PI) * (z + 0.044715 * z * z * z);", "double u = sqrt(2.0 / PI) * (z + 0.44715 * z * z * z);", 0, "bias_act"),
    ("relu slope at negative inputs", "if (act == 0) return z > 0.0 ? 1.0 : 0.0;", "if (act == 0) return 1.0;", 0, "bias_act"),
    ("low-precision Adam: eps inside the root", "double upd = (mi / c1) / (sqrt(vi / c2) + eps);", "double upd = (mi / c1) / sqrt(vi / c2 + eps);", 1, "trainers"),
    ("sgd: nesterov look-ahead dropped", "d = nesterov ? gh + momentum * b : b;", "d = b;", 0, "trainers"),
    ("sgd: step sign", "p_out[i] = pi - lr * d;", "p_out[i] = pi + lr * d;", 0, "trainers"),
    ("heads: heads and positions transposed", "int64_t dst = (((int64_t)b * heads + n) * len + l) * head_dim + d;\n                        outs[part][dst]",
     "int64_t dst = (((int64_t)b * len + l) * heads + n) * head_dim + d;\n                        outs[part][dst]", 0, "heads"),
    ("heads bwd: bias gradient of the wrong column", "if (dbias) dbias[col] += g;", "if (dbias) dbias[(int64_t)n * head_dim + d] += g;", 0, "heads"),
    ("embedding: positions counted over the batch", "const int l = (int)(t % len);", "const int l = (int)(t % (len + 1));", 0, "embedding"),
    ("embedding bwd: table gradient not scaled", "demb[(int64_t)w * hidden + i] += scale * g;", "demb[(int64_t)w * hidden + i] += g;", 0, "embedding"),
    ("padding removal: inclusive prefix sums", "offsets[b] = run;\n        run += clamp_len(key_len, b, max_len);", "run += clamp_len(key_len, b, max_len);\n        offsets[b] = run;", 0, "pad"),
    ("padding removal: restore leaves the padding unset", "i < lb ? load(packed, r * hidden + c, dt) : 0.0;", "load(packed, (i < lb ? r : 0) * hidden + c, dt);", 0, "pad"),
    ("softmax with query lengths: padded query rows computed", "if (query_len && i >= query_len[b]) kl = 0;", "if (query_len && i > query_len[b]) kl = 0;", 0, "pad"),
]


def _nth(hay: str, needle: str, which: int) -> int:
    pos = -1
    for _ in range(which + 1):
        pos = hay.find(needle, pos + 1)
        if pos < 0:
            raise AssertionError(f"the oracle no longer contains {needle!r} (occurrence {which}): update the mutant")
    return pos


def _run(case, tmp):
    idx, (name, old, new, which, module) = case
    src = open(SRC).read()
    at = _nth(src, old, which)
    path = os.path.join(tmp, f"mutant_{idx}.c")
    with open(path, "w") as f:
        f.write(src[:at] + new + src[at + len(old):])
    # the mutant must still be a valid program: a compile error would "fail the tests" for the wrong reason
    c = subprocess.run(["gcc", "-std=c99", "-fsyntax-only", "-fopenmp", path],
                       capture_output=True, text=True)
    if c.returncode != 0:
        return name, module, 99, c.stderr[-400:]
    env = dict(os.environ, LSQ_ORACLE_SRC=path, OMP_NUM_THREADS="1")
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        os.path.join(ROOT, "tests", f"test_oracle_{module}.py")],
                       cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)
    if r.returncode == 1 and "AssertionError" not in r.stdout and "assert " not in r.stdout:
        return name, module, 98, (r.stdout + r.stderr)[-400:]       # failed, but not on an assertion of a pin
    return name, module, r.returncode, (r.stdout + r.stderr)[-400:]


def test_every_planted_mistake_is_caught(tmp_path):
    with ThreadPoolExecutor(max_workers=6) as ex:
        results = list(ex.map(lambda c: _run(c, str(tmp_path)), enumerate(MUTANTS)))
    survivors = [(n, m) for n, m, rc, _ in results if rc == 0]
    broken = [(n, m, tail) for n, m, rc, tail in results if rc not in (0, 1)]     # 1 = tests failed, as they must
    assert not broken, f"could not run: {broken}"
    assert not survivors, f"pins missed these planted mistakes: {survivors}"


def test_the_mutation_harness_itself_passes_the_unmodified_oracle(tmp_path):
    path = os.path.join(str(tmp_path), "copy.c")
    with open(path, "w") as f:
        f.write(open(SRC).read())
    env = dict(os.environ, LSQ_ORACLE_SRC=path, OMP_NUM_THREADS="1")
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        os.path.join(ROOT, "tests", "test_oracle_layernorm.py"), os.path.join(ROOT, "tests", "test_oracle_philox.py")],
                       cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, (r.stdout + r.stderr)[-600:]
