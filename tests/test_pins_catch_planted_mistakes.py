"""The pins of the oracle, checked in their turn: one plausible mistake at a time
is planted in a COPY of oracle/okt_oracle.py (a wrong comparison, an off-by-one
rank, a dropped mask, a fused or mis-signed accumulate, a ceiling for a floor, a
wrong region bound, a narrower accumulator, ...) and the pin tests are run
against the copy in a scratch directory.  Every planted mistake must fail at
least one pin.  CPU only; nothing here touches the library or the GPU."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

# (what is planted, text in the oracle, text it is replaced by)
MISTAKES = [
    ("select takes > for >=",
     "selected = np.flatnonzero(magnitude_key(acc) >= th_key)",
     "selected = np.flatnonzero(magnitude_key(acc) > th_key)"),
    ("count_ge takes > for >=",
     "count_ge = int(np.count_nonzero(keys >= th_key))",
     "count_ge = int(np.count_nonzero(keys > th_key))"),
    ("rank k + 1 instead of k (sort)",
     "th_key = descending[k - 1]",
     "th_key = descending[min(k, n - 1)]"),
    ("rank k + 1 instead of k (partition)",
     "th_key = np.partition(keys, n - k)[n - k]",
     "th_key = np.partition(keys, max(n - k - 1, 0))[max(n - k - 1, 0)]"),
    ("keys keep the sign bit",
     "return x.view(np.uint32) & _ABS_MASK",
     "return x.view(np.uint32)"),
    ("accumulate rounded once (fused)",
     "return np.add(residual, scaled, dtype=np.float32)",
     "return (residual.astype(np.float64) + np.float64(np.float32(lr)) * grad.astype(np.float64))"
     ".astype(np.float32)"),
    ("accumulate subtracts",
     "return np.add(residual, scaled, dtype=np.float32)",
     "return np.subtract(residual, scaled, dtype=np.float32)"),
    ("learning rate applied to the residual",
     "scaled = np.multiply(np.float32(lr), grad, dtype=np.float32)\n"
     "    return np.add(residual, scaled, dtype=np.float32)",
     "scaled = np.multiply(np.float32(lr), residual, dtype=np.float32)\n"
     "    return np.add(grad, scaled, dtype=np.float32)"),
    ("quantile position rounded up",
     "b[r] = int(idx[(r * nnz) // R])",
     "b[r] = int(idx[min(-(-(r * nnz) // R), nnz - 1)])"),
    ("region offsets count <= boundary",
     "off[r] = int(np.count_nonzero(idx64 < b[r]))",
     "off[r] = int(np.count_nonzero(idx64 <= b[r]))"),
    ("equal split rounded up",
     "b[r] = (r * n) // R",
     "b[r] = (r * n + R - 1) // R"),
    ("region excludes lo",
     "inside = (i >= lo) & (i < hi)",
     "inside = (i > lo) & (i < hi)"),
    ("region stops one short of hi",
     "inside = (i >= lo) & (i < hi)",
     "inside = (i >= lo) & (i < hi - 1)"),
    ("reduce accumulates in fp32",
     "D = np.zeros(width, dtype=np.float64)",
     "D = np.zeros(width, dtype=np.float32)"),
    ("structural zeros dropped",
     "present = np.flatnonzero(hits > 0)",
     "present = np.flatnonzero((hits > 0) & (D != 0))"),
    ("mean instead of sum",
     "dense = D.astype(np.float32)",
     "dense = (D / max(P, 1)).astype(np.float32)"),
    ("tolerance base sums signed values",
     "A[slot] += np.abs(v[inside])",
     "A[slot] += v[inside]"),
    ("balancing triggers at exactly four times the average",
     "triggered = max(sizes) * P > 4 * T",
     "triggered = max(sizes) * P >= 4 * T"),
    ("balancing triggers at twice the average",
     "triggered = max(sizes) * P > 4 * T",
     "triggered = max(sizes) * P > 2 * T"),
    ("balanced ranges rounded up",
     "new_first = [(j * T) // P for j in range(P + 1)]",
     "new_first = [-(-(j * T) // P) for j in range(P + 1)]"),
    ("global select takes > for >=",
     "keep = np.flatnonzero(magnitude_key(val) >= th_key)",
     "keep = np.flatnonzero(magnitude_key(val) > th_key)"),
    ("global select compares signed values",
     "keep = np.flatnonzero(magnitude_key(val) >= th_key)",
     "keep = np.flatnonzero(val >= np.float32(th))"),
    ("intersection keeps every local index",
     "member = np.isin(local_idx, global_idx)",
     "member = np.ones(local_idx.size, dtype=bool)"),
    ("residual update zeroes the complement",
     "eps[np.asarray(indexes, dtype=np.int64)] = np.float32(0.0)",
     "keep = np.zeros(eps.size, dtype=bool); keep[np.asarray(indexes, dtype=np.int64)] = True; "
     "eps[~keep] = np.float32(0.0)"),
    ("k rounded down",
     "return -(-n * num // den)",
     "return n * num // den"),
    ("entries beyond the capacity zeroed too",
     "    if capacity is not None:\n        selected = selected[:capacity]\n"
     "    idx = selected.astype(np.uint32)\n    val = acc[selected].copy()\n"
     "    residual = acc.copy()\n    residual[selected] = np.float32(0.0)",
     "    residual = acc.copy()\n    residual[selected] = np.float32(0.0)\n"
     "    if capacity is not None:\n        selected = selected[:capacity]\n"
     "    idx = selected.astype(np.uint32)\n    val = acc[selected].copy()"),
    ("carried partial result joined in reverse order",
     'idx_cat = np.concatenate([idx_cat, partial["idx"]])',
     'idx_cat = np.concatenate([idx_cat, partial["idx"][::-1]])'),
]


def run_pins(tmp_path, source):
    """pytest on the pin tests against `source` as oracle/okt_oracle.py; its exit code."""
    work = tmp_path / "copy"
    (work / "oracle").mkdir(parents=True)
    (work / "tests").mkdir()
    for name in os.listdir(os.path.join(ROOT, "oracle")):
        if name.endswith(".py") and name != "okt_oracle.py":
            shutil.copy(os.path.join(ROOT, "oracle", name), work / "oracle" / name)
    (work / "oracle" / "okt_oracle.py").write_text(source)
    for name in ("test_oracle_pins.py", "conftest.py"):
        shutil.copy(os.path.join(ROOT, "tests", name), work / "tests" / name)
    shutil.copytree(os.path.join(ROOT, "tests", "golden"), work / "tests" / "golden")
    env = dict(os.environ, PYTHONPATH=str(work), PYTHONDONTWRITEBYTECODE="1")
    done = subprocess.run([sys.executable, "-m", "pytest", "tests/test_oracle_pins.py", "-x", "-q",
                           "-p", "no:cacheprovider"], cwd=work, env=env, capture_output=True,
                          text=True, timeout=300)
    return done.returncode, done.stdout[-2000:]


def oracle_source():
    with open(os.path.join(ROOT, "oracle", "okt_oracle.py")) as fh:
        return fh.read()


def test_the_unchanged_oracle_passes_in_the_scratch_copy(tmp_path):
    code, out = run_pins(tmp_path, oracle_source())
    assert code == 0, out


@pytest.mark.parametrize("what,old,new", MISTAKES, ids=[m[0] for m in MISTAKES])
def test_a_planted_mistake_fails_a_pin(tmp_path, what, old, new):
    source = oracle_source()
    assert source.count(old) >= 1, f"the oracle no longer contains the text of: {what}"
    code, out = run_pins(tmp_path, source.replace(old, new, 1))
    # 1 = tests ran and some failed; anything else (0 = all passed, 2+ = did not run) is a miss
    assert code == 1, f"{what}: exit code {code}\n{out}"
