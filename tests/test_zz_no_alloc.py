"""okt_threshold_select_noalloc, the entry point that allocates nothing (its scan
state is an array of device memory inside the library), against
okt_threshold_select on the same inputs: indices, values, counts and residual bit
for bit, on two calls in a row that share the array, the second on a shorter
vector; and both against the CPU oracle."""
import numpy as np
import pytest
import torch

import paper_2201_07598_amd as okt
from oracle import okt_oracle as orc
from tests.okt_harness import DEV, bits_equal, to_dev, u32, u64, workspace

pytestmark = pytest.mark.gpu


def run_both(acc, th, capacity):
    n = acc.size
    d_th = to_dev(np.array([th], dtype=np.float32))
    out = []
    for call in ("workspace", "noalloc"):
        d_acc = to_dev(acc)
        idx = torch.full((max(capacity, 1),), -1, dtype=torch.int32, device=DEV)
        val = torch.full((max(capacity, 1),), 7.0, dtype=torch.float32, device=DEV)
        nnz = torch.full((2,), -1, dtype=torch.int64, device=DEV)
        if call == "workspace":
            okt.okt_threshold_select(d_acc, d_th, idx, val, nnz, workspace(okt.okt_workspace_bytes(n, 0)),
                                     capacity=capacity)
        else:
            okt.okt_threshold_select_noalloc(d_acc, d_th, idx, val, nnz, capacity=capacity)
        torch.cuda.synchronize()
        out.append((u32(idx), val.cpu().numpy(), u64(nnz), d_acc.cpu().numpy()))
    return out


def check(acc, th, capacity):
    (i0, v0, c0, r0), (i1, v1, c1, r1) = run_both(acc, th, capacity)
    assert np.array_equal(c0, c1), (c0, c1)
    assert np.array_equal(i0, i1) and bits_equal(v0, v1) and bits_equal(r0, r1)
    ridx, rval, rres, total = orc.threshold_select(acc, th, capacity=capacity)
    e = ridx.size
    assert int(c1[0]) == e and int(c1[1]) == total
    assert np.array_equal(i1[:e], ridx) and bits_equal(v1[:e], rval) and bits_equal(r1, rres)
    assert np.all(i1[e:] == 0xFFFFFFFF)               # nothing written past the count


def test_noalloc_select_matches_the_workspace_call_twice_in_a_row():
    rng = np.random.default_rng(707)
    big = rng.laplace(0, 1e-3, 9_000_017).astype(np.float32)       # several workgroups, ragged end
    th_big = float(np.partition(np.abs(big), big.size - 90_000)[big.size - 90_000])
    check(big, th_big, capacity=4 * 90_000)
    small = rng.laplace(0, 1e-3, 70_003).astype(np.float32)        # the array keeps the first call's state
    th_small = float(np.partition(np.abs(small), small.size - 700)[small.size - 700])
    check(small, th_small, capacity=500)                           # and the output fills up
    check(small[:0], 1.0, capacity=4)                              # empty vector: {0, 0}
