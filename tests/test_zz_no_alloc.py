"""The gap entry point that allocates nothing (its partial sums live in a fixed array inside the library)
against chicle_gap, through the C ABI: two calls in a row, the second on a smaller input."""
import numpy as np
import pytest

from harness import cached_problem
from workloads import round_permutations

pytestmark = pytest.mark.gpu


def _round_then_both_gaps(binding, p, K, seed):
    g = binding.ChicleRound.from_problem(p, max_solvers=K)
    g.assign(K, binding.balance(p.chunk_nnz(), K))
    out = []
    for r in range(2):
        g.local_epoch(g.upload_perm(round_permutations(seed, r, g.solver_rows())))
        g.aggregate()
        ref = g.gap()
        got = g.gap_noalloc()
        again = g.gap()
        out.append((ref, got, again))
    g.close()
    return out


def test_gap_noalloc_matches_gap_twice_second_smaller():
    import torch
    assert torch.cuda.is_available(), "this test needs the GPU"
    import paper_1909_04885_amd as binding
    _, big = cached_problem("sparse_zipf", "mini")
    _, small = cached_problem("dense_hinge", "mini")
    for p, K in ((big, 6), (small, 3)):
        print("\ncase gap_noalloc", p.name, "n=%d d=%d chunks=%d" % (p.n, p.d, p.n_chunks), flush=True)
        for ref, got, again in _round_then_both_gaps(binding, p, K, seed=11):
            assert ref[2] > 0
            for a, b in zip(ref, got):        # same kernels, same summation order: the same numbers
                assert abs(a - b) <= 1e-12 * max(abs(a), 1e-300), (ref, got)
            assert again == ref               # and the arena's scratch path is undisturbed
