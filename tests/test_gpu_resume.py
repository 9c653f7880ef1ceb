"""Checkpoint / resume: the library keeps nothing of the training state.  A context holds tables derived from the
registration and the schedule, and a reduction scratch that every call overwrites before reading; parameters, optimizer
state, model copy and the step counter are the caller's.  So a run that is cut after some iterations - its tensors saved,
the context destroyed, a new context registered over restored tensors in other memory - must continue with exactly the
bits of the uninterrupted run."""
import pytest
import torch

from paper_2502_11058_amd import workloads as W

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("fused", [False, True])
def test_resumed_run_equals_the_uninterrupted_one(fused):
    from paper_2502_11058_amd.harness import DeviceReplica
    assert torch.cuda.is_available(), "no GPU visible"
    w = W.small_llama(n_replicas=5, period=3)
    cut, total = 4, 9            # the cut falls inside a period: slot r mod H and AdamW's step r + 1 come from r alone

    def inputs(rep, r):
        rep.fill_grads(r)
        S = rep.sets[r % w.period]
        order_t = [t for l in S for t in range(len(rep.layer_of)) if rep.layer_of[t] == l]
        n = rep.slot_numel[r % w.period]
        if n:
            rep.fill_peers_from(torch.cat([rep.sync[t] for t in order_t]), r, n)

    def advance(rep, r):
        inputs(rep, r)
        (rep.fused_step if fused else rep.step)(r, local_rank=r % w.n_replicas)

    whole = DeviceReplica(w, 0)
    whole.init_params()
    for r in range(cut):
        advance(whole, r)
    torch.cuda.synchronize()
    saved = {k: getattr(whole, k).cpu() for k in ("a_sync", "a_s0", "a_s1", "a_model")}     # the checkpoint: tensors only
    for r in range(cut, total):
        advance(whole, r)
    torch.cuda.synchronize()

    resumed = DeviceReplica(w, 0, arena_offset=2)       # another allocation, another alignment, a new context
    for k, v in saved.items():
        getattr(resumed, k)[2:].copy_(v)                 # arena_offset elements are skipped at the start of every arena
    for r in range(cut, total):
        advance(resumed, r)
    torch.cuda.synchronize()
    for k in ("a_sync", "a_s0", "a_s1", "a_model"):
        a, b = getattr(whole, k), getattr(resumed, k)[2:]
        assert torch.equal(a.view(torch.int16), b.contiguous().view(torch.int16)), k
    # the statistics are fp64 sums whose grouping follows the launch shape, and the other alignment takes other kernels
    assert torch.allclose(whole.stats, resumed.stats, rtol=1e-12, atol=0.0)
    whole.close()
    resumed.close()
