"""Are the oracle's pins tight?  Each entry below plants one plausible mistake (a dropped
term, a wrong sign or index, an off-by-one, swapped operands) in a private copy of an oracle
file; the pins of that file, run against the copy, must then fail.  A mutant that survives
means some line of the oracle is not pinned by anything but itself.  Everything here runs on
the CPU, in temporary directories; the files in the tree are never touched."""
import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

ATTENTION = ("oracle/zz_oracle.py", ["tests/test_oracle_pins.py"], [
    ("return np.asarray(j) <= i", "return np.asarray(j) < i"),
    ("(j <= i) & ((j < sink) | (i - j < window))", "(j <= i) & ((j < sink) | (i - j <= window))"),
    ("(j <= i) & ((j < sink) | (i - j < window))", "(j <= i) & ((j <= sink) | (i - j < window))"),
    ("(j <= i) & ((j < sink) | (i - j < window))", "((j < sink) | (i - j < window))"),
    ("e = np.exp(s - s.max())", "e = np.exp(s)"),
    ("return e / e.sum()", "return e / e.max()"),
    ("p = softmax_weights(scale * (K @ q))", "p = softmax_weights(K @ q)"),
    ("p = softmax_weights(scale * (K @ q))", "p = softmax_weights(-scale * (K @ q))"),
    ("return p @ V", "return p @ K"),
    ("return 1.0 / np.sqrt(float(head_dim))", "return 1.0 / float(head_dim)"),
    ("g = h // G", "g = h % Hkv"),
    ("J = attended_positions(i, bool(kinds[g]), sink, window)", "J = attended_positions(i, not bool(kinds[g]), sink, window)"),
    ("attention_row(Q[b, i, h, :], Kg[J], Vg[J], scale)", "attention_row(Q[b, i, h, :], Vg[J], Kg[J], scale)"),
    ("return sink + window if streaming else max_ctx", "return sink + window + 1 if streaming else max_ctx"),
    ("if r >= window or sink + r > n - 1:", "if r >= window or sink + r > n:"),
    ("return sink + r + window * ((newest - r) // window)", "return sink + r + window * ((newest - r + 1) // window)"),
    ("return sink + r + window * ((newest - r) // window)", "return sink + r + window * (newest // window)"),
    ("return min(n, sink + window) if streaming else n", "return min(n, window) if streaming else n"),
    ("img[:, :, s, :] = X[:, p, :, :]", "img[:, :, s, :] = X[:, s % T, :, :]"),
    ("return slot if slot < n else -1\n    r = slot - sink", "return slot if slot <= n else -1\n    r = slot - sink"),
    ("Qfull[:, i] = q", "Qfull[:, i - 1] = q"),
    ("for qh in np.asarray(q_group)])", "for qh in np.asarray(q_group)[::-1]])"),
])

TRANSPORT = ("oracle/zz_transport_oracle.py", ["tests/test_transport.py", "-k", "test_oracle_"], [
    ("n_stream = int(round(sparsity * L)) * H", "n_stream = int(round(sparsity * L)) * H + 1"),
    ("key=lambda t: (alpha.flat[t], t))", "key=lambda t: (-alpha.flat[t], t))"),
    ("cost = alpha[i, j]                          # o1", "cost = -alpha[i, j]                          # o1"),
    ("cost = -omega * alpha[i, j]", "cost = omega * alpha[i, j]"),
    ("cost = -omega * alpha[i, j]", "cost = -alpha[i, j]"),
    ("if was_streaming == becomes_streaming:", "if was_streaming != becomes_streaming:"),
    ("becomes_streaming = i in chosen", "becomes_streaming = i not in chosen"),
])

ROPE = ("oracle/zz_rope_oracle.py", ["tests/test_rope_oracle_pins.py"], [
    ("out[..., :half] = lo * c - hi * s", "out[..., :half] = lo * c + hi * s"),
    ("out[..., half:] = hi * c + lo * s", "out[..., half:] = hi * c - lo * s"),
    ("out[..., :half] = lo * c - hi * s", "out[..., :half] = lo * s - hi * c"),
    ("out[..., half:] = hi * c + lo * s", "out[..., half:] = lo * c + hi * s"),
    ("lo, hi = x[..., :half], x[..., half:]", "lo, hi = x[..., 0::2], x[..., 1::2]"),
    ("out[..., :half] = lo * c - hi * s", "out[..., :half] = lo * c"),
    ("c = np.asarray(cos, dtype=np.float64)[pos][:, :, None, :]", "c = np.asarray(cos, dtype=np.float64)[pos[:1]][:, :, None, :]"),
    ("s = np.asarray(sin, dtype=np.float64)[pos][:, :, None, :]", "s = np.asarray(sin, dtype=np.float64)[pos + 0 * pos[:, :1]][:, ::-1][:, :, None, :]"),
])

CONFTEST = '''import os, sys
HERE = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, %r)      # the package (library binding) and nothing the copy shadows
sys.path.insert(0, HERE)    # the private copy: oracle/ and zz_inputs.py come from here
def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a GPU")
''' % ROOT


def run_pins(workdir, target, pins, mutation):
    """Copy what the pins need into workdir, plant the mutation (None: none), run them."""
    for rel in ("oracle", "tests/golden"):
        shutil.copytree(os.path.join(ROOT, rel), os.path.join(workdir, rel))
    for rel in ("zz_inputs.py", "tests/test_oracle_pins.py", "tests/test_transport.py", "tests/test_rope_oracle_pins.py"):
        shutil.copy(os.path.join(ROOT, rel), os.path.join(workdir, rel))
    open(os.path.join(workdir, "tests", "conftest.py"), "w").write(CONFTEST)
    if mutation is not None:
        path = os.path.join(workdir, target)
        src = open(path).read()
        old, new = mutation
        assert src.count(old) >= 1, "the mutation's anchor is gone from %s: %r" % (target, old)
        open(path, "w").write(src.replace(old, new, 1))
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", "--rootdir", workdir] + \
          [os.path.join(workdir, p) if p.endswith(".py") else p for p in pins]
    r = subprocess.run(cmd, cwd=workdir, capture_output=True, text=True)
    return r.returncode, r.stdout[-600:] + r.stderr[-300:]


@pytest.mark.parametrize("group", [ATTENTION, TRANSPORT, ROPE], ids=["attention", "transport", "rope"])
def test_every_planted_mistake_fails_a_pin(group, tmp_path):
    target, pins, mutations = group
    rc, out = run_pins(str(tmp_path / "clean"), target, pins, None)
    assert rc == 0, "the pins must pass on an unmodified copy:\n" + out
    assert " passed" in out and "no tests ran" not in out

    def one(k):
        return run_pins(str(tmp_path / ("m%d" % k)), target, pins, mutations[k])
    with ThreadPoolExecutor(max_workers=4) as ex:
        results = list(ex.map(one, range(len(mutations))))
    survivors = [mutations[k] for k, (rc, _) in enumerate(results) if rc == 0]
    assert not survivors, "mistakes no pin notices: %r" % survivors
    # a failing pin, not a broken run (import error, collection error), must be what stopped each mutant
    for k, (rc, out) in enumerate(results):
        summary = [l for l in out.splitlines() if " in " in l and ("passed" in l or "failed" in l or "error" in l)]
        assert summary and " failed" in summary[-1] and " error" not in summary[-1], (mutations[k], out)
