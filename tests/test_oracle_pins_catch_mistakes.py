"""Do the oracle's pins notice a mistake?  Each case below plants one plausible mistake in a *copy* of the oracle's
source (a wrong exponent offset, a tie rounded the other way, a transposed block, swapped nibbles, ...), runs the
CPU pin tests against that copy in a child process, and requires that at least one pin fails.  The unchanged copy
must pass, so a failure really comes from the planted line.  Nothing here touches the GPU or the library."""
import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PIN_FILES = ["test_oracle_mxfp4.py", "test_oracle_rotation_gemm.py", "test_oracle_smoothing.py"]

# (name, file under oracle/, [(text as it stands, text with the mistake), ...])
MISTAKES = [
    ("exponent offset 1 instead of 2 (Eq. 2's b read as the E2M1 bias)", "mxfp4.py",
     [("E2M1_EMAX = 2", "E2M1_EMAX = 1")]),
    ("floor(log2 amax) off by one", "mxfp4.py",
     [("floor_log2 = ex.astype(np.int64) - 1", "floor_log2 = ex.astype(np.int64)")]),
    ("group maximum without the absolute value", "mxfp4.py",
     [("amax = np.max(np.abs(g), axis=-1)", "amax = np.max(g, axis=-1)")]),
    ("tie 1.25 rounded up to 1.5", "mxfp4.py",
     [("code[(v >= 0.75) & (v <= 1.25)] = 2", "code[(v >= 0.75) & (v < 1.25)] = 2"),
      ("code[(v > 1.25) & (v < 1.75)] = 3", "code[(v >= 1.25) & (v < 1.75)] = 3")]),
    ("tie 2.5 rounded up to 3", "mxfp4.py",
     [("code[(v >= 1.75) & (v <= 2.5)] = 4", "code[(v >= 1.75) & (v < 2.5)] = 4"),
      ("code[(v > 2.5) & (v < 3.5)] = 5", "code[(v >= 2.5) & (v < 3.5)] = 5")]),
    ("tie 0.25 rounded up to 0.5", "mxfp4.py",
     [("code[(v > 0.25) & (v < 0.75)] = 1", "code[(v >= 0.25) & (v < 0.75)] = 1")]),
    ("tie 5 rounded up to 6", "mxfp4.py",
     [("code[v > 5.0] = 7", "code[v >= 5.0] = 7")]),
    ("boundary between 2 and 3 at 2.25", "mxfp4.py",
     [("code[(v > 2.5) & (v < 3.5)] = 5", "code[(v > 2.25) & (v < 3.5)] = 5")]),
    ("boundary between 4 and 6 at 4.5", "mxfp4.py",
     [("code[v > 5.0] = 7", "code[v > 4.5] = 7")]),
    ("sign of minus zero dropped", "mxfp4.py",
     [("np.signbit(y32).astype(np.uint8)", "(y32 < 0).astype(np.uint8)")]),
    ("nibbles swapped when packing", "mxfp4.py",
     [("(code[:, 0::2] | (code[:, 1::2] << 4))", "(code[:, 1::2] | (code[:, 0::2] << 4))")]),
    ("nibbles swapped when unpacking", "mxfp4.py",
     [("out[:, 0::2] = codes & 0xF\n    out[:, 1::2] = codes >> 4", "out[:, 1::2] = codes & 0xF\n    out[:, 0::2] = codes >> 4")]),
    ("low clamp of the exponent at -126", "mxfp4.py",
     [("e = np.clip(e, -127, 127)", "e = np.clip(e, -126, 127)")]),
    ("all-zero group given exponent 0", "mxfp4.py",
     [("e = np.where(amax == 0.0, -127, e)", "e = np.where(amax == 0.0, 0, e)")]),
    ("E8M0 bias 128", "mxfp4.py",
     [("E8M0_BIAS = 127", "E8M0_BIAS = 128")]),
    ("largest E2M1 magnitude 5 instead of 6", "mxfp4.py",
     [("2.0, 3.0, 4.0, 6.0]", "2.0, 3.0, 4.0, 5.0]")]),
    ("sign ignored when decoding", "mxfp4.py",
     [("val = np.where((c & 8) != 0, -mag, mag)", "val = mag")]),
    ("rotation block transposed", "rotation.py",
     [("x[:, BLOCK * j:BLOCK * (j + 1)] @ Rj", "x[:, BLOCK * j:BLOCK * (j + 1)] @ Rj.T")]),
    ("rotation block of the neighbouring group", "rotation.py",
     [("Rj = R[j if R.shape[0] == G else 0]", "Rj = R[(j + 1) % G if R.shape[0] == G else 0]")]),
    ("rotation accumulated in fp32", "rotation.py",
     [("x = np.asarray(x, dtype=np.float64)\n    R = np.asarray(R, dtype=np.float64)",
       "x = np.asarray(x, dtype=np.float32)\n    R = np.asarray(R, dtype=np.float32)")]),
    ("product rounded to fp32", "linear.py",
     [("return a @ b.T", "return (a @ b.T).astype(np.float32).astype(np.float64)")]),
    ("product without the transpose of the second operand's scales (scales of A used for B)", "linear.py",
     [("b = mxfp4.dequantize(b_codes, b_scales)", "b = mxfp4.dequantize(b_codes, np.full_like(b_scales, 127))")]),
    ("bf16 rounding half up instead of half to even", "linear.py",
     [("r = u + 0x7FFF + ((u >> 16) & 1)", "r = u + 0x8000")]),
    ("weights divided by Lambda instead of multiplied", "pipeline.py",
     [("w = smoothing.apply(w, lam, inverse=False)", "w = smoothing.apply(w, lam, inverse=True)")]),
    ("group error statistic: squared norms (no square root)", "pipeline.py",
     [("out[ok] = num[ok] / den[ok]", "out[ok] = (num[ok] / den[ok]) ** 2")]),
    ("group error statistic: normalised by the quantised group instead of the group itself", "pipeline.py",
     [("den = np.linalg.norm(y.reshape(y.shape[0], G, 32), axis=-1)",
       "den = np.linalg.norm((d + y).reshape(y.shape[0], G, 32), axis=-1)")]),
    ("group error statistic: ratio of whole-tensor norms instead of the mean of per-group ratios", "pipeline.py",
     [("out[ok] = num[ok] / den[ok]", "out[ok] = np.linalg.norm(num[ok]) / np.linalg.norm(den[ok])")]),
    ("group error statistic: groups without norm counted in the mean", "pipeline.py",
     [("return float(np.mean(r[r >= 0]))", "return float(np.sum(r[r >= 0]) / r.size)")]),
]


def _make_tree(dst, mistake):
    os.makedirs(os.path.join(dst, "tests"))
    shutil.copytree(os.path.join(ROOT, "oracle"), os.path.join(dst, "oracle"), ignore=shutil.ignore_patterns("__pycache__"))
    shutil.copytree(os.path.join(ROOT, "workloads"), os.path.join(dst, "workloads"), ignore=shutil.ignore_patterns("__pycache__"))
    shutil.copytree(os.path.join(ROOT, "tests", "golden"), os.path.join(dst, "tests", "golden"))
    for f in PIN_FILES + ["helpers.py"]:
        shutil.copy(os.path.join(ROOT, "tests", f), os.path.join(dst, "tests", f))
    with open(os.path.join(dst, "tests", "conftest.py"), "w") as fh:
        fh.write("import os, sys\nsys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))\n"
                 "def pytest_configure(config):\n    config.addinivalue_line('markers', 'gpu: needs a GPU')\n")
    if mistake is not None:
        _, fname, edits = mistake
        path = os.path.join(dst, "oracle", fname)
        with open(path) as fh:
            src = fh.read()
        for old, new in edits:
            assert src.count(old) == 1, f"the line to change is not there exactly once: {old!r}"
            src = src.replace(old, new)
        with open(path, "w") as fh:
            fh.write(src)


def _run_pins(tree):
    env = {k: v for k, v in os.environ.items() if k != "PYTHONPATH"}
    env["PYTHONDONTWRITEBYTECODE"] = "1"
    p = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", "-m", "not gpu"]
                       + [os.path.join("tests", f) for f in PIN_FILES],
                       cwd=tree, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=600)
    return p.returncode, p.stdout


def test_every_planted_mistake_fails_a_pin(tmp_path):
    cases = [None] + MISTAKES
    trees = []
    for i, m in enumerate(cases):
        tree = str(tmp_path / f"case{i}")
        _make_tree(tree, m)
        trees.append(tree)
    with ThreadPoolExecutor(max_workers=4) as pool:
        results = list(pool.map(_run_pins, trees))
    rc0, out0 = results[0]
    assert rc0 == 0, "the unchanged copy of the oracle must pass its pins:\n" + out0[-2000:]
    unnoticed = []
    for m, (rc, out) in zip(MISTAKES, results[1:]):
        # 1 = a test failed; anything else (0 = all passed, 2 = could not even be collected) is not a caught mistake
        if rc != 1:
            unnoticed.append(f"{m[0]} (pytest exit {rc}): {out[-300:]}")
    assert not unnoticed, "no pin noticed:\n" + "\n".join(unnoticed)


@pytest.mark.parametrize("fname", sorted({m[1] for m in MISTAKES}))
def test_planted_lines_exist_in_the_oracle(fname):
    """The cases above name lines of the oracle as they stand: a change to the oracle must update them."""
    with open(os.path.join(ROOT, "oracle", fname)) as fh:
        src = fh.read()
    for m in MISTAKES:
        if m[1] == fname:
            for old, _ in m[2]:
                assert src.count(old) == 1, old
