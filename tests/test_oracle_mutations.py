"""The pins of tests/test_oracle_pins.py against planted slips (CPU only).

One plausible mistake at a time (a wrong sign, index, axis, bound, operand or state
transition) is planted in a temporary copy of oracle/cascade_oracle.py, and the pin
suite is run against that copy in a child process: every planted slip must make some
pin fail.  The oracle in the tree is never touched and nothing here uses the GPU.
"""
import os
import shutil
import subprocess
import sys
import tempfile
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
ORACLE = os.path.join(ROOT, "oracle", "cascade_oracle.py")
PINS = os.path.join(ROOT, "tests", "test_oracle_pins.py")

# (text in the oracle, what a slip would have written instead)
SLIPS = [
    ("f = frames_per_block * g + n // (grid_h * grid_w)", "f = frames_per_block * g + n // (grid_h * grid_h)"),
    ("f = frames_per_block * g + n // (grid_h * grid_w)", "f = g + n // (grid_h * grid_w)"),
    ("y = (n % (grid_h * grid_w)) // grid_w", "y = (n % (grid_h * grid_w)) // grid_h"),
    ("x = n % grid_w", "x = n % grid_h"),
    ("return np.stack([f, y, x], axis=1)", "return np.stack([f, x, y], axis=1)"),
    ("-2.0 * j / Da", "-2.0 * j / D"),
    ("-2.0 * j / Da", "-1.0 * j / Da"),
    ("-2.0 * j / Da", "2.0 * j / Da"),
    ("-2.0 * j / Da", "-2.0 * (j + 1) / Da"),
    ("pos[:, a:a + 1]", "pos[:, 0:1]"),
    ("y[..., 0::2] = u * c - v * s", "y[..., 0::2] = u * c + v * s"),
    ("y[..., 1::2] = u * s + v * c", "y[..., 1::2] = u * s - v * c"),
    ("y[..., 1::2] = u * s + v * c", "y[..., 1::2] = v * s + u * c"),
    ("u, v = x[..., 0::2], x[..., 1::2]", "u, v = x[..., :D // 2], x[..., D // 2:]"),
    ("if st in (CLEAN, SINK):", "if st in (CLEAN,):"),
    ("elif st == NOISY and gr in infl:", "elif st == NOISY:"),
    ("gr <= gi", "gr < gi"),
    ("gr <= gi", "gr >= gi"),
    ("mode == BIDIRECTIONAL or", "mode != BIDIRECTIONAL or"),
    ("sc = 1.0 / math.sqrt(D)", "sc = 1.0 / D"),
    ("sc = 1.0 / math.sqrt(D)", "sc = 1.0"),
    ("@ Kh.T) * sc", "@ Kh.T)"),
    ("s -= s.max(axis=1, keepdims=True)", "s -= s.max(axis=0, keepdims=True)"),
    ("p /= p.sum(axis=1, keepdims=True)", "p /= p.max(axis=1, keepdims=True)"),
    ("p /= p.sum(axis=1, keepdims=True)", "pass"),
    ("o[r0:r0 + row_chunk, h, :] = p @ Vh", "o[r0:r0 + row_chunk, h, :] = p @ Kh"),
    ("Vh = np.ascontiguousarray(V[:, h, :])", "Vh = np.ascontiguousarray(V[:, 0, :])"),
    ("Kh = np.ascontiguousarray(K[:, h, :])", "Kh = np.ascontiguousarray(K[:, 0, :])"),
    ("sel = [r for r in range(len(k_blocks)) if vis[i, r]]", "sel = [r for r in range(len(k_blocks)) if vis[0, r]]"),
    ("sel = [r for r in range(len(k_blocks)) if vis[i, r]]", "sel = [r for r in range(len(k_blocks))]"),
    ("q = q[np.asarray(rows[i], dtype=np.int64)]", "q = q[np.asarray(rows[0], dtype=np.int64)]"),
    ("return self.S + ((g - self.S) % (self.W + self.C))", "return self.S + (g % (self.W + self.C))"),
    ("return self.S + ((g - self.S) % (self.W + self.C))", "return self.S + ((g - self.S) % (self.W + self.C - 1))"),
    ("return self.S + ((g - self.S) % (self.W + self.C))", "return ((g - self.S) % (self.W + self.C))"),
    ("return (slot * self.P + page) * self.H + head", "return (slot * self.H + head) * self.P + page"),
    ("return (slot * self.P + page) * self.H + head", "return (slot * self.P + page) * self.H + page"),
    ("if self.state[s] in (CLEAN, SINK):\n            raise CacheError(\"block already finished\")", "pass"),
    ("if self.state[s] != FREE and self.block[s] != g:", "if False:"),
    ("self.state[s] = SINK if g < self.S else CLEAN", "self.state[s] = CLEAN"),
    ("if self.state[s] != NOISY:\n            raise CacheError(\"only", "if False:\n            raise CacheError(\"only"),
    ("if self.state[s] == SINK:\n            raise", "if False:\n            raise"),
    ("if self.state[s] == NOISY:\n                self.epoch[s] = new_epoch", "if True:\n                self.epoch[s] = new_epoch"),
    ("if self.state[s] == NOISY:\n                self.epoch[s] = new_epoch", "if self.state[s] == CLEAN:\n                self.epoch[s] = new_epoch"),
    ("order = sink + self.clean_window() + sorted(inflight_g)", "order = self.clean_window() + sink + sorted(inflight_g)"),
    ("order = sink + self.clean_window() + sorted(inflight_g)", "order = sink + self.clean_window() + list(inflight_g)[::-1]"),
    ("tau = min(step, nT - 1)", "tau = min(step, nT)"),
    ("b = max(0, step - (nT - 1))", "b = max(0, step - nT)"),
    ("batch.append((b + i, timesteps[tau - i]))", "batch.append((b + i, timesteps[i]))"),
    ("for i in range(0, min(tau, width - 1) + 1):", "for i in range(0, min(tau, width - 1)):"),
    ("if batch[0][1] == 0:", "if True:"),
    ("if len(win) > cache.W:", "if len(win) >= cache.W:"),
    ("evicted = win[0]", "evicted = win[-1]"),
    ("batch = [(b + i, tau - i) for i in range(min(d, n_gpus - 1) + 1)]", "batch = [(b + i, tau) for i in range(min(d, n_gpus - 1) + 1)]"),
    ("if b + d >= n_blocks:", "if b + d > n_blocks:"),
    ("if tau - 0 == n_timesteps - 1:", "if tau == n_timesteps:"),
    ("return x @ w.T", "return x @ w"),
    ("return x @ w.T", "return (w @ x.T)"),
    ("for n in range(lag * (n_blocks - 1) + n_timesteps):", "for n in range(lag * n_blocks + n_timesteps):"),
    ("if 0 <= n - lag * j < n_timesteps]", "if 0 <= n - lag * j <= n_timesteps]"),
    ("(j, n - lag * j) for j", "(j, n - j) for j"),
]

CHILD = ("import sys; sys.path.insert(0, {d!r}); import oracle.cascade_oracle as o; "
         "assert o.__file__.startswith({d!r}); import pytest; "
         "sys.exit(pytest.main(['-x', '-q', '-p', 'no:cacheprovider', {pins!r}]))")


def _pins_fail_on(mutant_source: str) -> bool:
    d = tempfile.mkdtemp(prefix="oracle_slip_")
    try:
        os.makedirs(os.path.join(d, "oracle"))
        open(os.path.join(d, "oracle", "__init__.py"), "w").close()
        with open(os.path.join(d, "oracle", "cascade_oracle.py"), "w") as f:
            f.write(mutant_source)
        env = dict(os.environ, PYTHONPATH=d, PYTHONDONTWRITEBYTECODE="1", OMP_NUM_THREADS="1")
        r = subprocess.run([sys.executable, "-c", CHILD.format(d=d, pins=PINS)], cwd=d, env=env,
                           stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL, timeout=300)
        return r.returncode != 0
    finally:
        shutil.rmtree(d, ignore_errors=True)


def test_unchanged_copy_passes_the_pins():
    # the child-process set-up itself must not be what makes a mutant fail
    assert not _pins_fail_on(open(ORACLE).read())


def test_every_planted_slip_fails_a_pin():
    source = open(ORACLE).read()
    missing = [a for a, _ in SLIPS if a not in source]
    assert not missing, f"oracle text changed; update these slips: {missing}"
    mutants = [source.replace(a, b, 1) for a, b in SLIPS]
    with ThreadPoolExecutor(max_workers=4) as pool:
        caught = list(pool.map(_pins_fail_on, mutants))
    survivors = [SLIPS[i] for i, ok in enumerate(caught) if not ok]
    assert not survivors, f"no pin notices: {survivors}"
