"""CPU model of how a row that is split over many chunks is summed on the GPU: every chunk adds its fp32
partial to the output with an atomic add, in an order the hardware picks.  The hardest case in the GPU suite
is the closed-form row (10^5 ones against B[k, j] = k (j + 1): integers near 5 * 10^9, where every rounding is
a systematic half-way case).  Summed here in random orders in fp32, it shows why the launch plan keeps chunks
of 512 items for matrices of long rows: the error stays below half the tolerance for every order tried, while
chunks of 64 (what a problem this small would otherwise get) use up nine tenths of it."""
import numpy as np

from paper_2007_03179_amd import gespmm_plan


def worst_ratio_over_orders(chunk, orders=400, seed=0):
    n = 100_000
    k = np.arange(n, dtype=np.float64)
    rng = np.random.default_rng(seed)
    worst = 0.0
    for j in (0, 2, 6):
        b = (k * (j + 1)).astype(np.float32).astype(np.float64)
        # per-chunk partials as the kernel forms them for N = 8: 32 slots add their entries in a chain, then a tree
        parts = []
        for c0 in range(0, n, chunk):
            seg = b[c0:c0 + chunk].astype(np.float32)
            m = np.concatenate([seg, np.zeros((-len(seg)) % 32, np.float32)]).reshape(-1, 32)
            acc = np.zeros(32, np.float32)
            for row in m:
                acc = (acc + row).astype(np.float32)
            while len(acc) > 1:
                acc = (acc[0::2] + acc[1::2]).astype(np.float32)
            parts.append(acc[0])
        parts = np.array(parts, dtype=np.float32)
        perms = np.argsort(rng.random((orders, len(parts))), axis=1)
        total = np.zeros(orders, dtype=np.float32)
        for step in range(len(parts)):
            total = (total + parts[perms[:, step]]).astype(np.float32)
        bound = 1e-5 * np.abs(b).sum() + 1e-6                 # the tolerance of sum, typed out: 1e-5 * Sabs + 1e-6
        worst = max(worst, float((np.abs(total.astype(np.float64) - b.sum()) / bound).max()))
    return worst


def test_long_split_row_stays_below_half_the_tolerance_with_the_planned_chunk_size():
    plan = gespmm_plan(2, 8, 100_000)                         # the shape of the closed-form GPU test
    assert plan["chunk_nnz"] == 512
    assert worst_ratio_over_orders(plan["chunk_nnz"]) <= 0.5


def test_the_same_row_in_chunks_of_64_would_use_up_most_of_the_tolerance():
    assert worst_ratio_over_orders(64, orders=100) > 0.7
