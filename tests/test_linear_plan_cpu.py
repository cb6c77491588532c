"""Host-side check of the projection launch plans (no GPU): every kernel form that a LLaDA-8B-shaped
projection can reach for some number of active rows is one that tests/test_gpu_linear.py launches, with
NaN-filled outputs, on the GPU.  The weight-stream kernel's forms (rows per block, columns per tile,
k-splits) matter most: its operand ring is filled by inline-assembly loads with hand-counted waits, so a
form no test reaches would be a form nobody has seen produce every partial sum."""
import pytest

from paper_2602_06412_amd import binding as B
from tests.test_gpu_linear import CASES

D, HD, DFF, V = 4096, 4096, 12288, 126464
LLADA = {"q|k|v": (3 * HD, D), "out": (D, HD), "gate|up": (2 * DFF, D), "down": (D, DFF), "lm_head": (V, D)}


def _form(plan):
    kernel, splits, rows, cols, tail = plan
    if kernel == 0:                       # weight-stream kernel: (rows per block, columns per tile, trips: splits matter)
        return ("stream", rows, cols, splits)
    if kernel == 1:                       # ring kernel: tile height / tail tile; any split count runs the same loop
        return ("ring", rows, cols, "tail" if tail else "uniform", "split" if splits > 1 else "unsplit")
    return ("lds", rows, cols, "split" if splits > 1 else "unsplit")


def test_every_reachable_launch_form_is_in_the_gpu_test_matrix():
    covered = {_form(B.sl_linear_plan(m_upper, n, k)) for n, k, m_upper, _ in CASES}
    needed = {}
    for name, (n, k) in LLADA.items():
        for mu in list(range(1, 1025)) + list(range(1024, 8193, 37)) + [8192]:
            needed.setdefault(_form(B.sl_linear_plan(mu, n, k)), (name, mu))
    missing = {f: w for f, w in needed.items() if f not in covered}
    assert not missing, f"launch forms no GPU test reaches (form: first projection / row bound that takes it): {missing}"


def test_plan_is_consistent_with_the_split_query_and_its_limits():
    for n, k in LLADA.values():
        for mu in (1, 16, 32, 33, 64, 200, 512, 1000, 4096):
            kernel, splits, rows, cols, tail = B.sl_linear_plan(mu, n, k)
            assert splits == B.sl_linear_splits(mu, n, k) and splits >= 1 and k % (64 * splits) == 0
            assert kernel in (0, 1, 2) and cols in (128, 256) and tail in (0, 1)
            if kernel == 0:
                assert mu <= 64 and rows in (32, 64) and rows >= min(mu, 64)
                assert (k // splits) % (256 if cols == 128 else 128) == 0       # whole trips of the register ring
            if kernel == 1:
                assert rows % 32 == 0 and 64 <= rows <= 256 and k // (32 * splits) >= 8
    with pytest.raises(B.SureLockError):
        B.sl_linear_plan(0, 4096, 4096)
    with pytest.raises(B.SureLockError):
        B.sl_linear_plan(16, 4096, 100)
