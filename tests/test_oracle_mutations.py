"""The pins must notice a plausible mistake anywhere in the oracle: every mutant below is
the oracle's source with one such slip planted (CPU only), and tests/test_oracle_pins.py,
run against it in a subprocess, has to fail.  An unmodified copy has to pass."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = open(os.path.join(ROOT, "oracle", "lagkv_oracle.py")).read()

MUTANTS = [
    ("reference is the previous chunk", "ref = slice(a + L, a + 2 * L)", "ref = slice(max(a - L, 0), max(a - L, 0) + L)"),
    ("reference is the chunk itself", "ref = slice(a + L, a + 2 * L)", "ref = slice(a, a + L)"),
    ("min/max over channels instead of tokens", "return Zref.min(axis=0), Zref.max(axis=0)",
     "return (np.broadcast_to(Zref.min(axis=1).min(), Zref.shape[1:]).copy(),\n"
     "            np.broadcast_to(Zref.max(axis=1).max(), Zref.shape[1:]).copy())"),
    ("min and max swapped", "return Zref.min(axis=0), Zref.max(axis=0)", "return Zref.max(axis=0), Zref.min(axis=0)"),
    ("no subtraction of the minimum", "(Zc - mn[None, :]) / safe[None, :]", "Zc / safe[None, :]"),
    ("divide by max instead of the range", "span = mx - mn", "span = mx"),
    ("epsilon in the denominator", "(Zc - mn[None, :]) / safe[None, :]", "(Zc - mn[None, :]) / (safe[None, :] + 1e-6)"),
    ("std over tokens instead of channels", "mu = Zbar.sum(axis=1) / D\n    dev = Zbar - mu[:, None]\n    return np.sqrt((dev * dev).sum(axis=1) / (D - ddof))",
     "mu = Zbar.sum(axis=0) / Zbar.shape[0]\n    dev = Zbar - mu[None, :]\n    return np.sqrt((dev * dev).sum(axis=1) / (D - ddof))"),
    ("variance instead of standard deviation", "return np.sqrt((dev * dev).sum(axis=1) / (D - ddof))", "return (dev * dev).sum(axis=1) / (D - ddof)"),
    ("biased divisor by default", "return np.sqrt((dev * dev).sum(axis=1) / (D - ddof))", "return np.sqrt((dev * dev).sum(axis=1) / D)"),
    ("mean absolute deviation", "return np.sqrt((dev * dev).sum(axis=1) / (D - ddof))", "return np.abs(dev).sum(axis=1) / (D - ddof)"),
    ("no softmax", "return chunk_softmax(token_spread(normalise(Zc, mn, mx), ddof))", "return token_spread(normalise(Zc, mn, mx), ddof)"),
    ("softmax without the exponential", "e = np.exp(sigma - sigma.max())", "e = sigma - sigma.min() + 1e-3"),
    ("keys only", "return tensor_score(Kc, Kref, ddof) + tensor_score(Vc, Vref, ddof)", "return 2.0 * tensor_score(Kc, Kref, ddof)"),
    ("values scored against the key reference", "tensor_score(Vc, Vref, ddof)", "tensor_score(Vc, Kref, ddof)"),
    ("K and V scores multiplied", "return tensor_score(Kc, Kref, ddof) + tensor_score(Vc, Vref, ddof)",
     "return 2.0 * L_ * tensor_score(Kc, Kref, ddof) * tensor_score(Vc, Vref, ddof)".replace("L_", "Kc.shape[0]")),
    ("lowest scores kept", "order = np.lexsort((np.arange(L), -score))", "order = np.lexsort((np.arange(L), score))"),
    ("ties to the later token", "order = np.lexsort((np.arange(L), -score))", "order = np.lexsort((-np.arange(L), -score))"),
    ("kept rows in score order", "return np.sort(order[:k])", "return order[:k]"),
    ("one row too many kept", "return np.sort(order[:k])", "return np.sort(order[:k + 1][:max(k, 1)] if k >= L else order[:k + 1])[:k + 1]"),
    ("k rounded up", "k = int(math.floor(float(r) * int(L)))", "k = int(math.ceil(float(r) * int(L)))"),
    ("last chunk counted as scored", "n_s = n - 1                              # the last chunk has no reference", "n_s = n"),
    ("window starts one chunk late", "window_start = n_static + pl[\"n_scored\"] * L", "window_start = n_static + (pl[\"n_scored\"] + 1) * L"),
    ("sink dropped", "idx = np.concatenate([np.arange(n_static, dtype=np.int64), kept.reshape(-1),", "idx = np.concatenate([np.arange(0, dtype=np.int64), kept.reshape(-1),"),
    ("Eq. 12 without the remainder", "return S + rL * ((Ls - S) // L - 1) + L + (Ls - S) % L", "return S + rL * ((Ls - S) // L - 1) + L"),
    ("Eq. 13 as a retention ratio", "return 1.0 - eq12_length(Ls, S, L, rL) / Ls", "return eq12_length(Ls, S, L, rL) / Ls"),
    ("L2 variant keeps the largest norms", "return -np.sqrt((Kc * Kc).sum(axis=1))", "return np.sqrt((Kc * Kc).sum(axis=1))"),
]


def _run_pins(tmp_path, source):
    pkg = tmp_path / "oracle"
    pkg.mkdir(parents=True, exist_ok=True)
    (pkg / "__init__.py").write_text("")
    (pkg / "lagkv_oracle.py").write_text(source)
    env = dict(os.environ, LAGKV_ORACLE_OVERRIDE=str(tmp_path))
    return subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"),
                           "-x", "-q", "-p", "no:cacheprovider"], capture_output=True, text=True, env=env, cwd=ROOT)


def test_unmodified_copy_passes(tmp_path):
    r = _run_pins(tmp_path, SRC)
    assert r.returncode == 0, r.stdout[-1500:]


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=lambda v: v if isinstance(v, str) and len(v) < 50 else None)
def test_pins_catch_the_planted_mistake(tmp_path, name, old, new):
    assert SRC.count(old) >= 1, f"mutation site of '{name}' not found: the oracle changed, update the mutant"
    r = _run_pins(tmp_path, SRC.replace(old, new, 1))
    # exit status 1 = tests ran and at least one failed (2 and above would be a broken mutant)
    assert r.returncode == 1, f"'{name}': pytest exit status {r.returncode}\n{r.stdout[-800:]}"
    assert "error" not in r.stdout.splitlines()[-1].lower(), r.stdout[-800:]
