"""The step allocates nothing, synchronises nothing and memsets nothing, so a caller can capture it
in a HIP graph.  Capture one step, replay it several times with eager work and synchronisations in
between, and compare every replay with the eager result (inputs restored before each replay).  The
same for the step at temperature > 0, the step on a selected subset, and the read-only probe with
the unlock rule."""
import numpy as np
import pytest
import torch

from paper_2602_06412_amd import binding as B
from paper_2602_06412_amd import workloads as wl
from tests.gpu_util import DEV, dev, weights_to_device

pytestmark = pytest.mark.gpu


def replay_against_eager(call, restore, outputs, reps=4):
    """call(): the launches under test; restore(): puts every in/out buffer back to its start state;
    outputs(): clones of everything the launches write."""
    restore()
    call()
    torch.cuda.synchronize()
    eager = outputs()
    s = torch.cuda.Stream()
    restore()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        call()                                                                   # warm-up on the side stream
    torch.cuda.current_stream().wait_stream(s)
    restore()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        call()
    for rep in range(reps):
        restore()
        _ = (torch.rand(1 << 16, device=DEV) * 2).sum().item()                   # eager work + a sync between replays
        g.replay()
        torch.cuda.synchronize()
        for i, (a, b) in enumerate(zip(outputs(), eager)):
            assert torch.equal(a, b), f"replay {rep}: output {i} differs from the eager step"


def bytes_of(x):
    return x.contiguous().view(torch.uint8).clone()


@pytest.mark.parametrize("variant", ["plain", "temperature", "selected", "probe"])
def test_step_replays_from_a_graph(variant):
    shape, Bn, N = wl.S_BF16, 2, 96
    R = Bn * N
    w = weights_to_device(wl.make_weights(shape, seed=4))
    kw = dict(temperature=0.8, seed=77) if variant == "temperature" else {}
    sess = B.Session(shape, w, Bn, N, **kw)
    try:
        rng = np.random.default_rng(0)
        tokens0 = dev(np.concatenate([wl.prompt_uniform(b, N, shape.vocab, shape.mask_id) for b in range(Bn)]), torch.int32)
        masked0 = dev((rng.random(R) < 0.5).astype(np.uint8))
        lock_np = (rng.random(R) < 0.3).astype(np.uint8) & (1 - masked0.cpu().numpy())
        lock0 = dev(lock_np)
        eps = dev(np.array([1e-3, 1e-2], dtype=np.float32))
        zero = torch.zeros(R, dtype=torch.uint8, device=DEV)
        # both posterior buffers and the cache filled for every slot
        for t in (1, 2):
            sess.step(tokens0.clone(), zero.clone(), zero, eps, t, 0, N, 0, new_lock=torch.zeros_like(zero))
        torch.cuda.synchronize()
        post0, kv0 = sess.post.clone(), sess.kv.clone()
        tokens, masked, lock, new_lock = tokens0.clone(), masked0.clone(), lock0.clone(), torch.zeros_like(lock0)

        def restore_common():
            tokens.copy_(tokens0); masked.copy_(masked0); lock.copy_(lock0); new_lock.zero_()
            sess.post.copy_(post0); sess.kv.copy_(kv0)
            sess.kl.fill_(-1.0); sess.conf.fill_(-1.0); sess.argmax.fill_(-1); sess.active_idx.fill_(-1)

        def step_outputs():
            M = int(sess.cu_active[-1].item())
            return [tokens.clone(), masked.clone(), new_lock.clone(), sess.cu_active.clone(), sess.kl[:M].clone(),
                    sess.conf[:M].clone(), sess.argmax[:M].clone(), sess.active_idx[:M].clone(),
                    bytes_of(sess.logits_view(3)), bytes_of(sess.kv)]

        if variant in ("plain", "temperature"):
            replay_against_eager(lambda: sess.step(tokens, masked, lock, eps, 3, 32, N, 2, new_lock=new_lock),
                                 restore_common, step_outputs)
        elif variant == "selected":
            d0 = dev(rng.random(R).astype(np.float32))
            sess.step_selected(tokens0.clone(), zero.clone(), zero.clone(), eps, 2, 0, N, 0, 1.0,
                               new_lock=torch.zeros_like(zero))                  # creates d_last / compute_mask
            torch.cuda.synchronize()
            sess.post.copy_(post0); sess.kv.copy_(kv0)

            def restore():
                restore_common()
                sess.d_last.copy_(d0); sess.compute_mask.zero_()

            replay_against_eager(
                lambda: sess.step_selected(tokens, masked, lock, eps, 3, 32, N, 2, 0.6, new_lock=new_lock), restore,
                lambda: step_outputs() + [sess.d_last.clone(), sess.compute_mask.clone()])
        else:
            sess.unlock_state()
            t_lock0 = dev(np.where(lock_np > 0, rng.integers(1, 3, R), 0), torch.int32)
            sess.step(tokens.clone(), masked0.clone(), lock0, eps, 3, 32, N, 2, new_lock=torch.zeros_like(zero))
            torch.cuda.synchronize()
            post0, kv0 = sess.post.clone(), sess.kv.clone()                       # the probe follows a step: keep its state
            cu0, conf0 = sess.cu_active.clone(), sess.conf.clone()

            def restore():
                tokens.copy_(tokens0); lock.copy_(lock0)
                sess.post.copy_(post0); sess.kv.copy_(kv0); sess.cu_active.copy_(cu0); sess.conf.copy_(conf0)
                sess.t_lock.copy_(t_lock0); sess.relocked.zero_(); sess.cool_until.zero_(); sess.unlocked.zero_()
                sess.probe_kl.fill_(-1.0); sess.probe_conf.fill_(-1.0); sess.probe_argmax.fill_(-1)
                sess.probe_idx.fill_(-1); sess.probe_logits.zero_()

            def outputs():
                P = int(sess.cu_probe[-1].item())
                return [lock.clone(), sess.unlocked.clone(), sess.relocked.clone(), sess.cool_until.clone(),
                        sess.t_lock.clone(), sess.cu_probe.clone(), sess.probe_idx[:P].clone(), sess.probe_kl[:P].clone(),
                        sess.probe_conf[:P].clone(), sess.probe_argmax[:P].clone(), bytes_of(sess.probe_logits[:P]),
                        bytes_of(sess.post), bytes_of(sess.kv)]

            replay_against_eager(lambda: sess.unlock_probe(tokens, lock, 3, 50.0, 1e-6, 0, 2), restore, outputs)
    finally:
        sess.close()
