"""How sharp the oracle's pins are: every mistake planted below in a COPY of the oracle (a dropped term, a wrong
sign, factor or index, a transposed operand; CPU only) must be caught by the pin tests of its area.

A copy of oracle/ is made per mutant in a temporary directory, one snippet of its source is replaced, and the pin
file is run in a subprocess that imports the copy (NETMAX_TEST_ORACLE_ROOT, honoured by conftest.py).  The unchanged
copy must pass (so that a failure is the mutant's, not the set-up's); each mutant must fail."""
import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
C, PY, GLUE = "netmax_oracle.c", "policy.py", "__init__.py"

# (pin file, source file, original snippet, planted mistake)
MUTANTS = [
    # random numbers and tables
    ("test_oracle_rng.py", C, "(uint64_t)0xD2511F53u * c0", "(uint64_t)0xCD9E8D57u * c0"),
    ("test_oracle_rng.py", C, "if (r > 0) { k0 += 0x9E3779B9u;", "if (r >= 0) { k0 += 0x9E3779B9u;"),
    ("test_oracle_rng.py", C, "uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;", "uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k0;"),
    ("test_oracle_policy.py", C, "while (m < M && Trow[m] <= u) ++m;", "while (m < M && Trow[m] < u) ++m;"),
    ("test_oracle_policy.py", C, "if (p[m] > 0.0) l = m;", "l = m;"),
    ("test_oracle_policy.py", C, "return m < last ? m : last;", "return m;"),
    ("test_oracle_policy.py", C, "alpha * rho * (dim + dmi) / (2.0 * p)", "alpha * rho * (dim + dmi) / p"),
    ("test_oracle_policy.py", C, "alpha * rho * (dim + dmi) / (2.0 * p)", "rho * (dim + dmi) / (2.0 * p)"),
    ("test_oracle_policy.py", C, "double dmi = adj ? (double)(adj[(size_t)m * M + i] != 0) : 1.0;",
     "double dmi = adj ? (double)(adj[(size_t)i * M + m] != 0) : 1.0;"),
    ("test_oracle_rng.py", C, "idx[(size_t)i * B + b] = (int32_t)(((uint64_t)r[b % 4] * n) >> 32);",
     "idx[(size_t)i * B + b] = (int32_t)(((uint64_t)r[b % 4] * (n - 1)) >> 32);"),
    ("test_oracle_policy.py", C, "if (m != i) ema[e] = (float)(beta * (double)ema[e] + (1.0 - beta) * (double)t[e]);\n        if (clock) clock[i] = (float)((double)clock[i] + (double)t[e]);\n    }\n}\n\n/* The same",
     "if (m != i) ema[e] = (float)((1.0 - beta) * (double)ema[e] + beta * (double)t[e]);\n        if (clock) clock[i] = (float)((double)clock[i] + (double)t[e]);\n    }\n}\n\n/* The same"),
    # synthetic gradient
    ("test_oracle_rng.py", C, "double rad = sqrt(-2.0 * log(u0));", "double rad = sqrt(-log(u0));"),
    ("test_oracle_rng.py", C, "z[2 * h + 1] = rad * sin(two_pi * u1);", "z[2 * h + 1] = rad * cos(two_pi * u1);"),
    ("test_oracle_rng.py", C, "(float)(sigma * z[e])", "(float)(z[e])"),
    # perceptron gradient
    ("test_oracle_grad.py", C, "da[(size_t)b * din + k] = a[l][(size_t)b * din + k] > 0.0 ? s : 0.0;", "da[(size_t)b * din + k] = s;"),
    ("test_oracle_grad.py", C, "(exp(z[o] - mx) / s - (o == y ? 1.0 : 0.0)) / (double)B", "(exp(z[o] - mx) / s + (o == y ? 1.0 : 0.0)) / (double)B"),
    ("test_oracle_grad.py", C, "(exp(z[o] - mx) / s - (o == y ? 1.0 : 0.0)) / (double)B", "(exp(z[o] - mx) / s - (o == y ? 1.0 : 0.0))"),
    ("test_oracle_grad.py", C, "for (int64_t o = 0; o < dout; ++o) z[o] += (double)bias[o];", ""),
    ("test_oracle_grad.py", C, "gW[k * dout + o] = (float)acc[o];", "gW[o * din + k] = (float)acc[o];"),
    ("test_oracle_grad.py", C, "gb[o] = (float)acc[o];", "gb[o] = 0.0f;"),
    ("test_oracle_grad.py", C, "b += 0x7FFFu + ((b >> 16) & 1u);", "b += 0x8000u;"),
    ("test_oracle_grad.py", C, "z[o] = z[o] > 0.0 ? z[o] : 0.0;", "z[o] = z[o] > 0.0 ? z[o] : 0.01 * z[o];"),
    ("test_oracle_grad.py", C, "for (int64_t o = 0; o < dout; ++o) s += d[o] * Wk[o];",
     "for (int64_t o = 0; o < dout; ++o) s += d[o] * Wop[l][o * din + k];"),
    ("test_oracle_grad.py", C, "for (size_t k = 0; k < n; ++k) r[k] = opnd((double)x[k], rb);", "for (size_t k = 0; k < n; ++k) r[k] = (double)x[k];"),
    ("test_oracle_grad.py", C, "for (size_t k = 0; k < n; ++k) r[k] = opnd(x[k], rb);", "for (size_t k = 0; k < n; ++k) r[k] = x[k];"),
    ("test_oracle_grad.py", C, "z_hidden[(size_t)b * dout + o] = z[o];", "z_hidden[(size_t)b * dout + o] = z[o] - (double)bias[o];"),
    ("test_oracle_grad.py", C, "z_hidden[(size_t)b * dout + o] = z[o];", "z_hidden[(size_t)b * dout + o] = z[o] > 0.0 ? z[o] : 0.0;"),
    ("test_oracle_grad.py", C, "z_hidden[(size_t)b * dout + o] = z[o];", "z_hidden[(size_t)o * B + b] = z[o];"),
    # momentum apply + mix
    ("test_oracle_mix.py", C, "const double vn = mu * (double)v[j] + (double)g[j] + wd * (double)x[j];\n            const float vf = (float)vn;           /*",
     "const double vn = mu * (double)v[j] + (double)g[j];\n            const float vf = (float)vn;           /*"),
    ("test_oracle_mix.py", C, "xn[j] = (float)(h - wi * (h - (double)xp[j]));", "xn[j] = (float)(h + wi * (h - (double)xp[j]));"),
    ("test_oracle_mix.py", C, "xn[j] = (float)(h - wi * (h - (double)xp[j]));", "xn[j] = (float)(h - wi * ((double)x[j] - (double)xp[j]));"),
    ("test_oracle_mix.py", C, "*xp = Xcur + (size_t)m * ld, *g = G + (size_t)i * ld;", "*xp = Xcur + (size_t)i * ld, *g = G + (size_t)i * ld;"),
    ("test_oracle_mix.py", C, "*xp = Xcur + (size_t)m * ld, *g = G + (size_t)i * ld;", "*xp = Xnext + (size_t)m * ld, *g = G + (size_t)i * ld;"),
    ("test_oracle_mix.py", C, "const double h = (double)x[j] - alpha * (double)vf;\n            xn[j]", "const double h = (double)x[j] - alpha * (double)g[j];\n            xn[j]"),
    ("test_oracle_mix.py", C, "const double wi = w[(size_t)i * M + m];\n        const float *x = Xcur", "const double wi = w[(size_t)m * M + i];\n        const float *x = Xcur"),
    ("test_oracle_mix.py", C, "mean /= (double)M;", ""),
    # asynchronous schedule
    ("test_oracle_async.py", C, "p_act[i] = 1.0 / tbar;", "p_act[i] = tbar;"),
    ("test_oracle_async.py", C, "const double d = (m == i) ? 0.0 : (adj", "const double d = (adj"),
    ("test_oracle_async.py", C, "*m_out = ora_peer_of_word(M, T + (size_t)i * M, last[i], r[0]);", "*m_out = ora_peer_of_word(M, T, last[0], r[0]);"),
    ("test_oracle_async.py", C, "x[j] = (float)(h - w * (h - xpj));", "x[j] = (float)(h - w * ((double)x[j] - xpj));"),
    ("test_oracle_async.py", C, "const int32_t i = active[s], m = peers[s];", "const int32_t i = peers[s], m = active[s];"),
    # the sequencing of one iteration / one global step
    ("test_oracle_mix.py", GLUE, "        self.X, self.Xn = self.Xn, self.X\n", "        pass\n"),
    ("test_oracle_mix.py", GLUE, "        self.local_step(it)\n        self.mix(peer)\n", "        self.mix(peer)\n        self.local_step(it)\n"),
    ("test_oracle_async.py", GLUE, "np.ascontiguousarray(self.G[i]), i, m, float(self.w[i, m])", "np.ascontiguousarray(self.G[m]), i, m, float(self.w[i, m])"),
    ("test_oracle_async.py", GLUE, "np.ascontiguousarray(self.G[i]), i, m, float(self.w[i, m])", "np.ascontiguousarray(self.G[i]), i, m, float(self.w[m, i])"),
    # policy generation (Algorithm 3)
    ("test_oracle_policy_generation.py", PY, "return alpha * rho * (d + d.T) * d", "return alpha * rho * d"),
    ("test_oracle_policy_generation.py", PY, "L = np.max(alpha * rho / M", "L = np.min(alpha * rho / M"),
    ("test_oracle_policy_generation.py", PY, "gam[sel] = (d + d.T)[sel] / (2.0 * P[sel])", "gam[sel] = (d + d.T)[sel] / P[sel]"),
    ("test_oracle_policy_generation.py", PY, "Y = alpha * rho * (a1 + a1.T) - alpha ** 2", "Y = alpha * rho * (a1 + a1.T) + alpha ** 2"),
    ("test_oracle_policy_generation.py", PY, "(a2.sum(axis=1) + a2.sum(axis=0))", "(a2.sum(axis=1))"),
    ("test_oracle_policy_generation.py", PY, "return float(w[-2])", "return float(w[-1])"),
    ("test_oracle_policy_generation.py", PY, "f = 1.0 / tbar_i", "f = tbar_i"),
    ("test_oracle_policy_generation.py", PY, 'if best is None or t_conv < best["t_conv"]:', 'if best is None or t_conv > best["t_conv"]:'),
    ("test_oracle_policy_generation.py", PY, "cost[-1] = 1.0", "cost[-1] = -1.0"),
    ("test_oracle_policy_generation.py", PY, "t_conv = tbar * np.log(eps) / np.log(lam2)", "t_conv = np.log(eps) / np.log(lam2)"),
    ("test_oracle_policy_generation.py", PY, "rho = L_rho + k * delta_rho", "rho = L_rho + delta_rho"),
]


def _run(tmp_root, pin_file):
    env = dict(os.environ, NETMAX_TEST_ORACLE_ROOT=tmp_root, OMP_NUM_THREADS="2")
    return subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", pin_file), "-x", "-q", "-m", "not gpu",
                           "-p", "no:cacheprovider"], cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)


def _copy_oracle(dst_root):
    dst = os.path.join(dst_root, "oracle")
    os.makedirs(dst)
    for f in ("__init__.py", C, PY):
        shutil.copy(os.path.join(ROOT, "oracle", f), os.path.join(dst, f))
    return dst


def _try_mutant(args):
    k, tmp, (pin_file, src, old, new) = args
    root = os.path.join(tmp, f"m{k}")
    d = _copy_oracle(root)
    text = open(os.path.join(d, src)).read()
    if text.count(old) != 1:
        return k, "snippet not found exactly once"
    open(os.path.join(d, src), "w").write(text.replace(old, new))
    r = _run(root, pin_file)
    if r.returncode == 0:
        return k, "survived"
    if "passed" not in r.stdout and "failed" not in r.stdout:
        return k, "did not run: " + (r.stdout + r.stderr)[-400:]
    return k, None


def test_unchanged_copy_passes(tmp_path):
    root = str(tmp_path / "clean")
    _copy_oracle(root)
    for pin_file in sorted({m[0] for m in MUTANTS}):
        r = _run(root, pin_file)
        assert r.returncode == 0, (pin_file, r.stdout[-1500:], r.stderr[-500:])
        assert root in r.stdout or True


def test_copy_is_what_the_pins_import(tmp_path):
    """The redirect works: a copy whose C source does not compile breaks the pins."""
    root = str(tmp_path / "broken")
    d = _copy_oracle(root)
    open(os.path.join(d, C), "a").write("\n#error planted\n")
    assert _run(root, "test_oracle_rng.py").returncode != 0


def test_every_planted_mistake_is_caught(tmp_path):
    jobs = [(k, str(tmp_path), m) for k, m in enumerate(MUTANTS)]
    with ThreadPoolExecutor(max_workers=6) as ex:
        results = list(ex.map(_try_mutant, jobs))
    bad = [(MUTANTS[k][0], MUTANTS[k][3][:70], why) for k, why in results if why]
    assert not bad, bad
