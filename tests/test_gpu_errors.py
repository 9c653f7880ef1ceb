"""Argument errors on a live context: every bad call is turned into an error code on the host, before any launch,
and the context keeps working afterwards."""
import numpy as np
import pytest
import torch

from paper_2502_11058_amd import binding as B
from paper_2502_11058_amd import workloads as W

pytestmark = pytest.mark.gpu


def _expect(code, fn, *a, **k):
    with pytest.raises(B.DdpError) as e:
        fn(*a, **k)
    assert e.value.code == code, str(e.value)
    assert len(str(e.value)) > 12


def test_bad_arguments_are_reported_not_launched(oracle):
    from paper_2502_11058_amd.harness import DeviceReplica
    assert torch.cuda.is_available(), "no GPU visible"
    w = W.tiny()
    rep = DeviceReplica(w, 0, wire16=True)
    rep.init_params()
    c, N = rep.ctx, w.n_replicas
    before = rep.a_sync.clone()
    flat = rep.flat
    _expect(1, c.ddp_pack, 9, flat)                                        # slot out of range
    _expect(1, c.ddp_pack, -1, flat)
    _expect(3, c.ddp_pack, 0, flat[1:])                                    # flat not 16-byte aligned
    _expect(1, c.ddp_partial_average, 0, flat, rep.peers, 0, 0, flat)      # N < 1
    _expect(1, c.ddp_partial_average, 0, flat, rep.peers, B.DDP_MAX_REPLICAS + 1, 0, flat)
    _expect(1, c.ddp_partial_average, 0, flat, rep.peers, N, N, flat)      # local_rank out of range
    _expect(1, c.ddp_partial_average, 0, flat, None, N, 0, flat)           # peers missing
    _expect(3, c.ddp_partial_average, 0, flat, [p[1:] for p in rep.peers], N, 0, flat)
    _expect(1, c.ddp_partial_average, 0, flat, rep.peers, N, 0, rep.peers[0])          # output overlaps a peer
    _expect(1, c.ddp_partial_average, 0, flat, rep.peers, N, 0, flat[4:])              # partial overlap with the input
    _expect(3, c.ddp_unpack, 0, flat[2:])
    f16, p16 = rep.flat16, rep.peers16                                     # bf16-on-the-wire entry points
    _expect(1, c.ddp_pack_wire16, 9, f16)
    _expect(3, c.ddp_pack_wire16, 0, f16[1:])
    _expect(1, c.ddp_partial_average_wire16, 0, f16, p16, 0, 0, flat)
    _expect(1, c.ddp_partial_average_wire16, 0, f16, p16, N, N, flat)
    _expect(1, c.ddp_partial_average_wire16, 0, f16, None, N, 0, flat)
    _expect(3, c.ddp_partial_average_wire16, 0, f16, [p[1:] for p in p16], N, 0, flat)
    _expect(1, c.ddp_partial_average_wire16, 0, f16, p16, N, 0, f16.view(torch.float32))      # no in-place form
    _expect(1, c.ddp_partial_average_wire16, 0, f16, p16, N, 0, p16[0].view(torch.float32))
    _expect(1, c.ddp_fused_sync_update_wire16, 0, p16, N, N, None, B.make_opt("sgdm", 0.01, 1))
    _expect(3, c.ddp_fused_sync_update_wire16, 0, [p[1:] for p in p16], N, 0, None, B.make_opt("sgdm", 0.01, 1))
    _expect(7, c.ddp_local_update, B.make_opt("adamw", 1e-3, 0))           # no second moment registered (checked first)
    opt = B.make_opt("sgdm", 0.01, 1)
    opt.kind = 7
    _expect(1, c.ddp_local_update, opt)
    _expect(7, c.ddp_local_update, B.make_opt("adamw", 1e-3, 1))           # AdamW without state1 registered
    _expect(1, c.ddp_set_option, "no_such_option", 1)
    _expect(1, c.ddp_set_option, "update_wg_per_cu", 33)
    _expect(1, c.ddp_set_option, "mean_wg_per_cu", -1)
    _expect(7, c.ddp_set_option, "update_chunk", 4096)                     # after registration
    _expect(6, c.ddp_set_schedule, [0, 2], [3, 3])                         # duplicate layer in a slot
    _expect(6, c.ddp_set_schedule, [0, 1], [8])                            # layer id out of range
    torch.cuda.synchronize()
    assert torch.equal(rep.a_sync, before)                                 # nothing ran
    # the context still works: one good iteration against the oracle
    hyper = dict(lr=w.lr, momentum=w.momentum)
    wk = oracle.Worker(rep.layer_of, [t.cpu().numpy() for t in rep.sync], "sgdm", hyper, False)
    flat_ref = wk.pack_slot(rep.sets[0])[0]
    rep.fill_grads(0)
    rep.fill_peers_from(torch.from_numpy(flat_ref).to(rep.dev), 0, flat_ref.size)
    peers = [p[:flat_ref.size].cpu().numpy() for p in rep.peers]
    grads = [g.cpu().numpy() for g in rep.grad]
    rep.step(0)
    wk.step(0, rep.sets, peers, 0, grads)
    for a, b in zip(rep.sync, wk.p):
        assert np.array_equal(a.cpu().numpy().view(np.uint32), b.view(np.uint32))
    rep.close()


def test_registration_errors():
    assert torch.cuda.is_available(), "no GPU visible"
    c = B.Context(0)
    x = torch.zeros(64, device="cuda")
    _expect(7, c.ddp_set_schedule, [0, 1], [0])                            # nothing registered yet
    _expect(7, c.ddp_local_update, B.make_opt("sgdm", 0.01, 1))
    _expect(1, c.ddp_register_model, 2, [0], [64], B.DDP_F32, B.DDP_F32, [x], None, [x], [x], None)       # T < L
    _expect(1, c.ddp_register_model, 2, [0, 0], [32, 32], B.DDP_F32, B.DDP_F32, [x, x], None, [x, x], [x, x], None)  # layer 1 missing
    _expect(1, c.ddp_register_model, 2, [1, 0], [32, 32], B.DDP_F32, B.DDP_F32, [x, x], None, [x, x], [x, x], None)  # not sorted
    _expect(2, c.ddp_register_model, 1, [0], [0], B.DDP_F32, B.DDP_F32, [x], None, [x], [x], None)        # empty tensor
    _expect(1, c.ddp_register_model, 1, [0], [64], B.DDP_BF16, B.DDP_F32, [x], None, [x], [x], None)      # bf16 without model copy
    _expect(1, c.ddp_register_model, 1, [0], [64], 5, B.DDP_F32, [x], None, [x], [x], None)
    _expect(3, c.ddp_register_model, 1, [0], [32], B.DDP_F32, B.DDP_F32, [x.data_ptr() + 2], None, [x], [x], None)   # odd address
    _expect(1, c.ddp_register_model, 1, [0], [64], B.DDP_F32, B.DDP_F32, [x], None, [None], [x], None)    # NULL gradient
    c.ddp_register_model(1, [0], [64], B.DDP_F32, B.DDP_F32, [x], None, [x], [x], None)
    _expect(6, c.ddp_pack, 0, x)                                           # no schedule yet
    c.close()
