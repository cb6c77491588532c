"""GPU parity of the stand-alone M-row projection (sl_linear_pack / sl_linear_forward) against
the plain definition y = x W^T evaluated in fp64 on the CPU (the GEMM terms of Sec. 2.4).

Inputs are bf16, hence exact in fp64; the kernel accumulates in fp32, so every output obeys the
textbook dot-product bound |err| <= gamma_k * sum_j |x_j||w_j| with gamma_k ~ k * 2^-24 (any
summation order), plus half a bf16 spacing when the result is stored as bf16."""
import numpy as np
import pytest
import torch

from paper_2602_06412_amd import binding as B
from tests.gpu_util import DEV, bf16_ulp

pytestmark = pytest.mark.gpu

# (n, k, m_upper, m): thin and thick launches, ragged m < m_upper, n not a multiple of 256
CASES = [
    (4160, 512, 32, 1),
    (1024, 4096, 64, 33),
    (4160, 1024, 128, 100),
    (4160, 512, 96, 70),
    (4160, 1024, 320, 300),       # one full 256-row tile and a ragged one
    (2048, 2048, 384, 200),       # the second row tile lies wholly beyond the device-side row count
    (32768, 512, 300, 290),       # 128 column tiles, two row tiles
    (12288, 1536, 704, 700),
    (8192, 4096, 1024, 1000),
    (4096, 12288, 1024, 1024),
    (4096, 4096, 16, 13),         # thin launches with few column tiles: the 128-column weight-stream tiles
    (4096, 12288, 32, 32),
    (4160, 2048, 24, 20),         # ... with a column tail
    # the ring kernel's fitted tile heights (64 .. 256 rows in steps of 32), ragged row counts
    (4160, 1024, 64, 50),
    (4160, 1024, 96, 90),
    (8192, 2048, 160, 150),
    (8192, 2048, 192, 161),
    (8192, 2048, 224, 224),
    (8192, 2048, 256, 255),
    (12288, 4096, 320, 320),      # two tiles of 160 rows (the LLaDA Q|K|V shape)
    (24576, 4096, 416, 400),
    (4096, 12288, 416, 390),
    (126464, 4096, 160, 131),     # the LM head: 494 column tiles
    (126464, 4096, 224, 224),
    # forms the LLaDA-8B projections reach that the cases above do not (tests/test_linear_plan_cpu.py lists them)
    (12288, 4096, 16, 16),        # weight stream, 128-column tiles, two k-splits
    (126464, 4096, 16, 16),       # weight stream, 256-column tiles, unsplit (the LM head)
    (126464, 4096, 40, 40),       # ring, 64-row tile, unsplit
    (126464, 4096, 96, 80),       # ring, 96-row tile, unsplit
    (12288, 4096, 170, 165),      # ring, 192-row tile, split
    (12288, 4096, 390, 387),      # ring, 224-row tiles, split
    (12288, 4096, 810, 805),      # ring, 192-row tiles, unsplit
    (12288, 4096, 1140, 1140),    # ring, 256-row tiles, unsplit
    (12288, 4096, 2578, 2570),    # ring, eleven row tiles, unsplit
    (24576, 4096, 1140, 1135),    # ring, full-height tiles + half-height tail tile, unsplit (480 workgroups)
    # 16 row tiles and more: an XCD walks its column tiles in bands of four (25 column tiles: one whole band,
    # seven of the eight XCDs with a tile short; 49: a whole band and a ragged one of three)
    (6400, 512, 4200, 4190),
    (12544, 512, 4100, 4099),
]


def _inputs(seed, n, k, m_upper):
    g = torch.Generator().manual_seed(seed)
    w = (torch.randn(n, k, generator=g) * 0.05).bfloat16()
    x = torch.randn(m_upper, k, generator=g).bfloat16()
    return w, x


def _bound(x64, w64, k):
    return 2.0 * k * 2.0 ** -24 * (np.abs(x64) @ np.abs(w64).T) + 1e-30


@pytest.mark.parametrize("n,k,m_upper,m", CASES)
@pytest.mark.parametrize("x_tiled", [0, 1])
def test_linear_fp32_partials(n, k, m_upper, m, x_tiled):
    w, x = _inputs(n + k + m, n, k, m_upper)
    wd, xd = w.to(DEV), x.to(DEV)
    packed = torch.empty_like(wd)
    B.sl_linear_pack(wd, packed)
    S = B.sl_linear_splits(m_upper, n, k)
    assert S >= 1 and k % (16 * S) == 0
    print("plan (kernel, splits, tile_rows, tile_cols, tail):", B.sl_linear_plan(m_upper, n, k), flush=True)
    y = torch.full((S, m_upper, n), float("nan"), device=DEV)
    m_dev = torch.tensor([m], dtype=torch.int32, device=DEV)
    xin = B.tile_activations(xd) if x_tiled else xd
    B.sl_linear_forward(xin, packed, m_dev, m_upper, n, k, S, y_f32=y, x_tiled=x_tiled)
    torch.cuda.synchronize()
    got = y[:, :m].double().sum(0).cpu().numpy()
    x64, w64 = x[:m].double().numpy(), w.double().numpy()
    ref = x64 @ w64.T
    bad = np.argwhere(~np.isfinite(y[:, :m].cpu().numpy()))
    assert len(bad) == 0, f"{len(bad)} non-finite partials, first (plane, row, col): {bad[:8].tolist()}, last {bad[-3:].tolist()}"
    assert np.all(np.abs(got - ref) <= _bound(x64, w64, k))


@pytest.mark.parametrize("n,k,m_upper,m", CASES[1:9] + CASES[13:])
def test_linear_bf16_row_map(n, k, m_upper, m):
    w, x = _inputs(7 * n + k + m, n, k, m_upper)
    wd, xd = w.to(DEV), x.to(DEV)
    packed = torch.empty_like(wd)
    B.sl_linear_pack(wd, packed)
    rows_out = 2 * m_upper
    rng = np.random.default_rng(m)
    row_map = np.sort(rng.choice(rows_out, size=m_upper, replace=False)).astype(np.int32)
    y = torch.full((rows_out, n), -7.0, device=DEV, dtype=torch.bfloat16)
    m_dev = torch.tensor([m], dtype=torch.int32, device=DEV)
    B.sl_linear_forward(B.tile_activations(xd), packed, m_dev, m_upper, n, k, 1, y_bf16=y,
                        row_map=torch.as_tensor(row_map, device=DEV), x_tiled=1)
    torch.cuda.synchronize()
    yh = y.double().cpu().numpy()
    x64, w64 = x[:m].double().numpy(), w.double().numpy()
    ref = x64 @ w64.T
    got = yh[row_map[:m]]
    assert np.all(np.abs(got - ref) <= _bound(x64, w64, k) + 0.5 * bf16_ulp(ref) * (1 + 1e-9))
    untouched = np.ones(rows_out, dtype=bool)
    untouched[row_map[:m]] = False
    assert np.all(yh[untouched] == -7.0), "rows outside row_map[:m] must not be written"


def test_linear_argument_errors():
    wd = torch.zeros(64, 64, device=DEV, dtype=torch.bfloat16)
    packed = torch.empty_like(wd)
    B.sl_linear_pack(wd, packed)
    x = torch.zeros(32, 64, device=DEV, dtype=torch.bfloat16)
    m_dev = torch.tensor([1], dtype=torch.int32, device=DEV)
    y = torch.zeros(1, 32, 64, device=DEV)
    yb = torch.zeros(32, 64, device=DEV, dtype=torch.bfloat16)
    with pytest.raises(B.SureLockError):                      # both outputs given
        B.sl_linear_forward(x, packed, m_dev, 32, 64, 64, 1, y_f32=y, y_bf16=yb)
    with pytest.raises(B.SureLockError):                      # neither
        B.sl_linear_forward(x, packed, m_dev, 32, 64, 64, 1)
    with pytest.raises(B.SureLockError):                      # k not a multiple of 64
        B.sl_linear_forward(x, packed, m_dev, 32, 64, 48, 1, y_f32=y)
    with pytest.raises(B.SureLockError):                      # bf16 output with a k-split
        B.sl_linear_forward(x, packed, m_dev, 32, 64, 64, 2, y_bf16=yb)


@pytest.mark.gpu
def test_clock_probe_matches_plain_launch_and_reports_sane_counters():
    """sl_linear_clock_probe: same bf16 result as sl_linear_forward, counters within physical bounds
    (a 32-deep k-tile cannot take fewer than 1024 cycles: 2 waves x 32 MFMAs x 16 cycles per SIMD)."""
    import torch
    from paper_2602_06412_amd import binding as B
    dev = "cuda:0"
    M, n, k = 300, 1024 + 32, 1024
    g = torch.Generator(device="cpu").manual_seed(5)
    w = (torch.randn(n, k, generator=g) * 0.02).to(torch.bfloat16).to(dev)
    x = torch.randn(M, k, generator=g).to(torch.bfloat16).to(dev)
    packed = torch.empty_like(w)
    B.sl_linear_pack(w, packed)
    m_dev = torch.tensor([M], dtype=torch.int32, device=dev)
    y0 = torch.zeros(M, n, dtype=torch.bfloat16, device=dev)
    y1 = torch.zeros(M, n, dtype=torch.bfloat16, device=dev)
    B.sl_linear_forward(x, packed, m_dev, M, n, k, 1, None, y0)
    counters = torch.zeros(8, dtype=torch.int64, device=dev)
    B.sl_linear_clock_probe(x, packed, m_dev, M, n, k, y1, counters)
    torch.cuda.synchronize()
    assert torch.equal(y0, y1)
    c = [int(v) for v in counters.cpu()]
    assert c[7] == k // 32
    assert c[1] >= 1024 * c[7] and c[1] < 40 * 1024 * c[7]
    assert all(v > 0 for v in c[:6]) and c[6] == 16
    mhz = c[1] / c[4] * 100.0
    assert 500.0 < mhz < 3000.0
    with pytest.raises(B.SureLockError):
        B.sl_linear_clock_probe(x, packed, m_dev, 64, n, k, y1, counters)     # thin launches have no probe


@pytest.mark.parametrize("n,k,m_upper", [(4096, 4096, 16), (4096, 12288, 32), (12288, 4096, 16)])
def test_thin_launch_repeats_bitwise_under_memory_traffic(n, k, m_upper):
    """The weight-stream kernel keeps loads in flight in a register ring with hand-counted waits.  Its result
    must not depend on when those loads land: repeat the launch while a second stream keeps HBM busy and
    compare every repetition bit for bit with the first (every partial written, none left at the NaN fill)."""
    w, x = _inputs(3 * n + k, n, k, m_upper)
    wd = w.to(DEV)
    packed = torch.empty_like(wd)
    B.sl_linear_pack(wd, packed)
    xin = B.tile_activations(x.to(DEV))
    S = B.sl_linear_splits(m_upper, n, k)
    m_dev = torch.tensor([m_upper], dtype=torch.int32, device=DEV)
    src = torch.empty(1 << 26, dtype=torch.float32, device=DEV).normal_()
    dst = torch.empty_like(src)
    side = torch.cuda.Stream()
    first = None
    for rep in range(24):
        y = torch.full((S, m_upper, n), float("nan"), device=DEV)
        torch.cuda.synchronize()
        if rep % 3:
            with torch.cuda.stream(side):
                for _ in range(rep % 3):
                    dst.copy_(src)
        B.sl_linear_forward(xin, packed, m_dev, m_upper, n, k, S, y_f32=y, x_tiled=1)
        torch.cuda.synchronize()
        assert bool(torch.isfinite(y).all()), f"repetition {rep}: partials left unwritten or non-finite"
        if first is None:
            first = y
            ref = x.double().numpy() @ w.double().numpy().T
            assert np.all(np.abs(y.double().sum(0).cpu().numpy() - ref) <= _bound(x.double().numpy(), w.double().numpy(), k))
        else:
            assert torch.equal(y, first), f"repetition {rep} differs from the first"
