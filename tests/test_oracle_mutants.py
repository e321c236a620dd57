"""The pins must notice a plausible mistake in the oracle: each mutant below plants one (a transposed tile index, swapped
plane indices, a wrong sign, a dropped term, a transposed basis) in a COPY of the oracle's sources, and the pin tests, run
against that copy in a sandbox, have to fail -- with the pin that merely compares the oracle's two formulations with each
other switched off, so that every mistake is noticed by a closed form, a textbook special case, a brute-force sum or a
finite difference.  The oracle in the repository is never touched; nothing here uses a GPU."""
import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor
from pathlib import Path

import pytest

ROOT = Path(__file__).resolve().parents[1]

# (file under oracle/, text to find, replacement, which occurrence of the text)
C_TILE_X = "s += E_X[(size_t)p * tt + a * t + b] * TILE_AT(X, k, t, I, L, a, b);"
MUTANTS = [
    # ---- stl_oracle.c, forward (Eq. (2))
    ("stl_oracle.c", C_TILE_X, C_TILE_X.replace("a, b);", "b, a);"), 1),                      # tile of X read transposed
    ("stl_oracle.c", "acc[p] += xh[p] * What[((size_t)p * K + L) * N + J];",
     "acc[p] += xh[p] * What[((size_t)p * K + J) * N + L];", 0),                               # plane of What read transposed
    ("stl_oracle.c", "for (int p = 0; p < r; ++p) s += D[(size_t)p * tt + a * t + b] * acc[p];",
     "for (int p = 0; p < r; ++p) s += D[(size_t)p * tt + b * t + a] * acc[p];", 0),           # output tile written transposed
    ("stl_oracle.c", "for (int64_t L = 0; L < K; ++L) {\n                    /* E_X",
     "for (int64_t L = 0; L < K - 1; ++L) {\n                    /* E_X", 0),                 # last term of the L sum dropped
    ("stl_oracle.c", "for (int p = 0; p < r; ++p) acc[p] = 0.0;\n                for",
     "for (int p = 1; p < r; ++p) acc[p] = 0.0;\n                for", 0),                     # one accumulator never cleared
    # ---- stl_oracle.c, weight and activation encodings
    ("stl_oracle.c", "s += E_W[(size_t)p * tt + a * t + b] * TILE_AT(W, n, t, L, J, a, b);",
     "s += E_W[(size_t)p * tt + a * t + b] * TILE_AT(W, n, t, L, J, b, a);", 0),
    ("stl_oracle.c", C_TILE_X, C_TILE_X.replace("a, b);", "b, a);"), 0),                      # encode_x (used by the backward)
    # ---- stl_oracle.c, backward
    ("stl_oracle.c", "s += dYhat[((size_t)p * M + I) * N + J] * What[((size_t)p * K + L) * N + J];",
     "s += dYhat[((size_t)p * M + I) * N + J] * What[((size_t)p * K + J) * N + L];", 0),       # dXhat with What not transposed
    ("stl_oracle.c", "s += Xhat[((size_t)p * M + I) * K + L] * dYhat[((size_t)p * M + I) * N + J];",
     "s -= Xhat[((size_t)p * M + I) * K + L] * dYhat[((size_t)p * M + I) * N + J];", 0),       # sign of dWhat
    ("stl_oracle.c", "s += Yhat[((size_t)p * M + I) * N + J] * TILE_AT(dC, n, t, I, J, a, b);",
     "s += Yhat[((size_t)p * M + I) * N + J] * TILE_AT(dC, n, t, I, J, b, a);", 0),            # dD against the transposed tile
    ("stl_oracle.c", "s += dXhat[((size_t)p * M + I) * K + L] * TILE_AT(X, k, t, I, L, a, b);",
     "s += dXhat[((size_t)p * M + I) * K + L] * TILE_AT(X, k, t, I, L, b, a);", 0),            # dE_X against the transposed tile
    ("stl_oracle.c", "s += D[(size_t)p * tt + a * t + b] * TILE_AT(dC, n, t, I, J, a, b);",
     "s += D[(size_t)p * tt + b * t + a] * TILE_AT(dC, n, t, I, J, a, b);", 0),                # dYhat with D transposed
    ("stl_oracle.c", "s += E_X[(size_t)p * tt + a * t + b] * dXhat[((size_t)p * M + I) * K + L];",
     "s += E_X[(size_t)p * tt + b * t + a] * dXhat[((size_t)p * M + I) * K + L];", 0),         # dX with E_X transposed
    ("stl_oracle.c", "for (int64_t L = 0; L < K; ++L)\n                    s += Xhat",
     "for (int64_t L = 1; L < K; ++L)\n                    s += Xhat", 0),                     # first term of Yhat dropped (feeds dD)
    # ---- planes.py
    ("planes.py", "return A.reshape(a // t, t, b // t, t).transpose(0, 2, 1, 3).reshape(a // t, b // t, t * t)",
     "return A.reshape(a // t, t, b // t, t).transpose(0, 2, 3, 1).reshape(a // t, b // t, t * t)", 0),   # column-major vec
    ("planes.py", "dYhat = np.ascontiguousarray((dc @ D.T).transpose(2, 0, 1))",
     "dYhat = np.ascontiguousarray((dc @ D.T[::-1]).transpose(2, 0, 1))", 0),                  # tile entries reversed in dYhat
    ("planes.py", "dX = untile(dXhat.transpose(1, 2, 0) @ E_X, t)", "dX = untile(dXhat.transpose(1, 2, 0) @ D, t)", 0),
    ("planes.py", "dE_X = np.tensordot(dXhat, x, axes=([1, 2], [0, 1]))", "dE_X = np.tensordot(dXhat, x, axes=([1, 2], [0, 1])) * 0.5", 0),
    ("planes.py", "return 0.5 * h * (1.0 + erf(h / np.sqrt(2.0)))", "return 0.5 * h * (1.0 + erf(h / 2.0))", 0),
    ("planes.py", "    if activation == \"gelu\":\n        H = gelu(H)", "    if activation == \"gelu\":\n        H = H", 0),
    ("planes.py", "        dE_B += dEb", "        dE_B = dEb", 0),                                # sum over the batch dropped
    ("planes.py", "        dB[b * rb:(b + 1) * rb] = dBb.T if b_transposed else dBb",
     "        dB[b * rb:(b + 1) * rb] = dBb.T if b_transposed else -dBb", 0),
    ("planes.py", "    out[:, body:] = np.einsum(\"ra,iaj->irj\", fold, Y3[:, body:])",
     "    out[:, body:] = np.einsum(\"ra,iaj->irj\", fold[:, ::-1], Y3[:, body:])", 0),         # fold coefficients reversed
    ("planes.py", "        dfold = np.einsum(\"irj,iaj->ra\", dC3[:, body:], Y3[:, body:])",
     "        dfold = np.einsum(\"irj,iaj->ra\", dC3[:, body:], Y3[:, :t])", 0),                  # dfold against the wrong rows
    ("planes.py", "    out[:, :rows] = X.reshape(nimg, rows, -1)", "    out[:, rows_pad - rows:] = X.reshape(nimg, rows, -1)", 0),
    # ---- bases.py
    ("bases.py", "               [-1, 0, 1, 0],\n               [0, 1, 0, -1]], dtype=np.float64)      # coefficients of A",
     "               [-1, 0, 1, 0],\n               [0, 1, 0, 1]], dtype=np.float64)      # coefficients of A", 0),   # a sign of M7
    ("bases.py", "col = 4 * (2 * bi + si) + (2 * bj + sj)", "col = 4 * (2 * bi + bj) + (2 * si + sj)", 0),   # plain Kronecker order
    ("bases.py", "                E_W[p, l * t + b] = 1.0", "                E_W[p, b * t + l] = 1.0", 0),
]


def _nth_replace(text, old, new, which):
    pos = -1
    for _ in range(which + 1):
        pos = text.find(old, pos + 1)
        assert pos >= 0, f"mutation target not found (the oracle changed; update this list): {old[:60]!r}"
    return text[:pos] + new + text[pos + len(old):]


def _sandbox(base: Path, name: str) -> Path:
    box = base / name
    (box / "tests").mkdir(parents=True)
    shutil.copytree(ROOT / "oracle", box / "oracle", ignore=shutil.ignore_patterns("*.so", "*.tmp", "__pycache__"))
    shutil.copy(ROOT / "stl_synth.py", box / "stl_synth.py")
    shutil.copy(ROOT / "tests" / "conftest.py", box / "tests" / "conftest.py")
    shutil.copy(ROOT / "tests" / "test_oracle_pins.py", box / "tests" / "test_oracle_pins.py")
    shutil.copytree(ROOT / "tests" / "golden", box / "tests" / "golden")
    return box


def _run_pins(box: Path) -> subprocess.CompletedProcess:
    env = dict(os.environ, OMP_NUM_THREADS="2", PYTHONDONTWRITEBYTECODE="1")
    env.pop("PYTHONPATH", None)
    return subprocess.run([sys.executable, "-m", "pytest", "tests/test_oracle_pins.py", "-x", "-q", "-p", "no:cacheprovider", "-k", "not two_formulations"],
                          cwd=box, env=env, capture_output=True, text=True, timeout=600)


def test_every_planted_mistake_is_noticed(tmp_path):
    control = _run_pins(_sandbox(tmp_path, "control"))
    assert control.returncode == 0, "the unmodified copy must pass:\n" + control.stdout[-2000:] + control.stderr[-2000:]
    assert "passed" in control.stdout and "oracle" in str(tmp_path / "control" / "oracle")

    def one(idx):
        fname, old, new, which = MUTANTS[idx]
        box = _sandbox(tmp_path, f"mutant{idx}")
        path = box / "oracle" / fname
        path.write_text(_nth_replace(path.read_text(), old, new, which))
        res = _run_pins(box)
        shutil.rmtree(box, ignore_errors=True)
        return idx, res.returncode, res.stdout[-300:]

    with ThreadPoolExecutor(max_workers=4) as pool:
        results = list(pool.map(one, range(len(MUTANTS))))
    survivors = [(i, MUTANTS[i][0], MUTANTS[i][2][:80]) for i, rc, _ in results if rc == 0]
    assert not survivors, f"pins did not notice: {survivors}"
    # a failure must be a failing pin, not a broken sandbox (exit code 1 = tests failed; 2.. = collection or usage error)
    broken = [(i, rc, out) for i, rc, out in results if rc not in (0, 1)]
    assert not broken, broken
