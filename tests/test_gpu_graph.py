"""The step allocates nothing, synchronises nothing and memsets nothing, so a caller can capture it
in a HIP graph.  Capture one step, replay it several times with eager work and synchronisations in
between, and compare every replay with the eager result (inputs restored before each replay)."""
import numpy as np
import pytest
import torch

from paper_2602_06412_amd import binding as B
from paper_2602_06412_amd import workloads as wl
from tests.gpu_util import DEV, dev, weights_to_device

pytestmark = pytest.mark.gpu


def test_step_replays_from_a_graph():
    shape, Bn, N = wl.S_BF16, 2, 96
    w = weights_to_device(wl.make_weights(shape, seed=4))
    sess = B.Session(shape, w, Bn, N)
    try:
        rng = np.random.default_rng(0)
        tokens0 = dev(np.concatenate([wl.prompt_uniform(b, N, shape.vocab, shape.mask_id) for b in range(Bn)]), torch.int32)
        masked0 = dev((rng.random(Bn * N) < 0.5).astype(np.uint8))
        lock_np = (rng.random(Bn * N) < 0.3).astype(np.uint8) & (1 - masked0.cpu().numpy())
        lock = dev(lock_np)
        eps = dev(np.array([1e-3, 1e-2], dtype=np.float32))
        zero = torch.zeros(Bn * N, dtype=torch.uint8, device=DEV)
        # both posterior buffers and the cache filled for every slot
        for t in (1, 2):
            sess.step(tokens0.clone(), zero.clone(), zero, eps, t, 0, N, 0, new_lock=torch.zeros_like(zero))
        tokens, masked, new_lock = tokens0.clone(), masked0.clone(), torch.zeros_like(lock)

        def outputs():
            torch.cuda.synchronize()
            M = int(sess.cu_active[-1].item())
            return [x.clone() for x in (tokens, masked, new_lock, sess.kl[:M], sess.conf[:M], sess.argmax[:M],
                                        sess.active_idx[:M], sess.logits_view(3))]

        sess.step(tokens, masked, lock, eps, 3, 32, N, 2, new_lock=new_lock)
        eager = outputs()
        g = torch.cuda.CUDAGraph()
        tokens.copy_(tokens0); masked.copy_(masked0)
        s = torch.cuda.Stream()
        s.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(s):
            sess.step(tokens, masked, lock, eps, 3, 32, N, 2, new_lock=new_lock)     # warm-up on the side stream
        torch.cuda.current_stream().wait_stream(s)
        tokens.copy_(tokens0); masked.copy_(masked0)
        with torch.cuda.graph(g):
            sess.step(tokens, masked, lock, eps, 3, 32, N, 2, new_lock=new_lock)
        for rep in range(4):
            tokens.copy_(tokens0); masked.copy_(masked0); new_lock.zero_()
            sess.kl.fill_(-1.0)
            _ = (torch.rand(1 << 16, device=DEV) * 2).sum().item()                   # eager work + a sync between replays
            g.replay()
            got = outputs()
            for a, b in zip(got, eager):
                assert torch.equal(a, b), f"replay {rep} differs from the eager step"
    finally:
        sess.close()
