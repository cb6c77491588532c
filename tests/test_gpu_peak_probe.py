"""The two peak probes behind bench.py's `achievable` figures really do the work they are priced for:
the MFMA loop's accumulators hold iters x (A B^T) of its operand fragments, the streaming pass reads
(and copies) every 16-byte word exactly once."""
import numpy as np
import pytest
import torch

from paper_2602_06412_amd import binding as B
from tests.gpu_util import DEV

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("wps", [1, 2])
def test_mfma_probe_accumulates_the_products(wps):
    iters = 48
    g = torch.Generator(device="cpu").manual_seed(5)
    ops = torch.randn(8 * 64 * 8, generator=g).to(torch.bfloat16)
    sink = torch.zeros(1 << 19, dtype=torch.float32, device=DEV)
    flops = B.sl_peak_probe_mfma(ops.to(DEV), iters, wps, sink)
    torch.cuda.synchronize()
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    waves = cus * 4 * wps
    assert flops == waves * iters * 16 * 2 * 16 * 16 * 32
    # fragment f, lane l, element e is entry (row l % 16, k = 8 (l / 16) + e) of a 16 x 32 operand; the sum of
    # all entries of A B^T is sum_k colsum_A[k] colsum_B[k]
    frag = ops.double().numpy().reshape(8, 4, 16, 8)               # [f][k-group][row][e]
    colsum = frag.sum(axis=2).reshape(8, 32)
    want = iters * sum(float(colsum[i] @ colsum[4 + j]) for i in range(4) for j in range(4))
    got = sink[:waves * 64].double().cpu().numpy().reshape(waves, 64).sum(axis=1)
    scale = iters * 16 * float(np.abs(frag).sum() / 8)             # loose magnitude of the summed terms
    assert np.all(np.abs(got - want) <= 1e-4 * scale), (got[:4], want)
    assert not torch.any(sink[waves * 64:] != 0)                    # nothing written past the launched threads


def test_stream_probe_reads_and_copies_every_word():
    n_bytes = (1 << 22) + 48                                       # ragged against every stride
    src = torch.randint(-2**31, 2**31 - 1, (n_bytes // 4,), dtype=torch.int32, device=DEV)
    dst = torch.zeros_like(src)
    sink = torch.zeros(1 << 19, dtype=torch.int32, device=DEV)
    B.sl_peak_probe_stream(src, None, sink)
    torch.cuda.synchronize()
    fold = np.bitwise_xor.reduce(sink.cpu().numpy().view(np.uint32))
    assert fold == np.bitwise_xor.reduce(src.cpu().numpy().view(np.uint32))
    assert not torch.any(dst != 0)
    B.sl_peak_probe_stream(src, dst, sink)
    torch.cuda.synchronize()
    assert torch.equal(src, dst)


def test_probes_reject_bad_arguments():
    sink = torch.zeros(1 << 19, dtype=torch.float32, device=DEV)
    buf = torch.zeros(1 << 12, dtype=torch.int32, device=DEV)
    for call in (lambda: B.sl_peak_probe_stream(buf, buf, sink),                      # overlap
                 lambda: B.sl_peak_probe_stream(buf[1:], None, sink),                 # misaligned, ragged size
                 lambda: B.sl_peak_probe_mfma(buf, 0, 1, sink),
                 lambda: B.sl_peak_probe_mfma(buf, 16, 3, sink)):
        with pytest.raises(B.SureLockError) as e:
            call()
        assert e.value.status == B.SL_EINVAL
    for call in (lambda: B.sl_peak_probe_mfma(buf[:64], 16, 1, sink),                 # operands too small
                 lambda: B.sl_peak_probe_mfma(buf, 16, 1, sink[:256]),
                 lambda: B.sl_peak_probe_stream(buf, None, sink[:256])):
        with pytest.raises(B.SureLockError) as e:
            call()
        assert e.value.status == B.SL_ENOSPC
