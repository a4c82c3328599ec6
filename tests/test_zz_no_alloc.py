"""The entry point for callers that cannot allocate (ocs_split_act_static) against the entry
point it is a variant of (ocs_split_act with a caller workspace), through the C ABI: two calls in
a row, the second on a smaller input, both grids (per-batch and static), Eq. 3 and Eq. 4 sides;
codes and scales bit for bit, and against the oracle as well."""
import numpy as np
import pytest
import torch

from oracle import ref
from paper_1901_09504_amd import binding as B
from tests import gpu_util as G

pytestmark = pytest.mark.gpu


def _inputs(seed, M, Cn, g, s):
    rng = np.random.Generator(np.random.PCG64(seed))
    X = rng.standard_normal((M, Cn * g)).astype(np.float32)
    X[rng.integers(0, M, 8), rng.integers(0, Cn * g, 8)] *= 9.0
    sel = ref.split_weights(X, Cn, g, s)
    return X, sel["chan_src"].astype(np.int32), sel["chan_depth"].astype(np.int32)


def _both(X, Cn, g, cs, cd, s, bits, threshold, clip):
    M = X.shape[0]
    Xd = G.dev(X)
    ldq = B.ocs_padded_cols((Cn + s) * g)
    csd = G.dev(cs)
    cdd = None if cd is None else G.dev(cd)
    th = None if threshold is None else torch.tensor([threshold], dtype=torch.float32, device="cuda")
    q0 = torch.full((M, ldq), 77, dtype=torch.int8, device="cuda")
    q1 = torch.full((M, ldq), 55, dtype=torch.int8, device="cuda")
    s0 = torch.zeros(2, dtype=torch.float32, device="cuda")
    s1 = torch.zeros(2, dtype=torch.float32, device="cuda")
    ws = B.alloc_workspace(M, Cn * g)
    B.ocs_split_act(Xd, M, Cn, g, Xd.stride(0), csd, cdd, s, bits, th, clip, q0, ldq, s0, ws)
    B.ocs_split_act_static(Xd, M, Cn, g, Xd.stride(0), csd, cdd, s, bits, th, clip, q1, ldq, s1)
    return G.host(q0), G.host(s0), G.host(q1), G.host(s1), ldq


def test_static_scratch_matches_workspace_call_twice_in_a_row():
    G.require_gpu()
    # first a large tensor (many partial maxima left behind in the scratch), then a smaller one
    for seed, (M, Cn, g, s) in enumerate([(3001, 96, 9, 5), (257, 40, 1, 3)]):
        X, cs, cd = _inputs(1000 + seed, M, Cn, g, s)
        assert B.ocs_workspace_bytes(M, Cn * g) <= B.STATIC_SCRATCH_BYTES
        for depth, threshold, clip in [(None, None, 1.0), (cd, None, 0.9), (None, 2.5, 1.0), (cd, 1.75, 1.0)]:
            q0, s0, q1, s1, ldq = _both(X, Cn, g, cs, depth, s, 8, threshold, clip)
            assert np.array_equal(q0, q1) and np.array_equal(s0.view(np.uint32), s1.view(np.uint32))
            qr, sr, _ = ref.split_act(X, Cn, g, cs, depth, s, 8, threshold=threshold, clip_ratio=clip, ldq=ldq)
            assert np.array_equal(q1, qr) and np.array_equal(s1.view(np.uint32), sr.view(np.uint32))


def test_static_scratch_with_the_maxima_folded_by_a_launch_of_their_own():
    """The per-batch grid as tensors from 160 MB on take it (the maxima of the max|X| pass folded into
    one word of the scratch space, the one-shot pass behind it), forced here on small tensors: same
    bits from both entry points and from the oracle, twice in a row, the second input smaller."""
    G.require_gpu()
    B.ocs_tune("max_flat", 2)
    try:
        for seed, (M, Cn, g, s) in enumerate([(3001, 96, 9, 5), (257, 40, 1, 3)]):
            X, cs, _ = _inputs(2000 + seed, M, Cn, g, s)
            q0, s0, q1, s1, ldq = _both(X, Cn, g, cs, None, s, 8, None, 0.8)
            assert np.array_equal(q0, q1) and np.array_equal(s0.view(np.uint32), s1.view(np.uint32))
            qr, sr, _ = ref.split_act(X, Cn, g, cs, None, s, 8, threshold=None, clip_ratio=0.8, ldq=ldq)
            assert np.array_equal(q1, qr) and np.array_equal(s1.view(np.uint32), sr.view(np.uint32))
    finally:
        B.ocs_tune("max_flat", -1)
