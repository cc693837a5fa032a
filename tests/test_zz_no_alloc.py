"""The allocation-free dispatch entry point against the ordinary one.

revive_dispatch_static keeps its scratch in a static device array instead of the bound workspace.
Its outputs must be bit-identical to revive_dispatch's on the same input, also on a second call
with a smaller input (the array still holds the first call's histograms), and both must equal the
oracle's stable counting sort."""
import ctypes as C

import numpy as np
import pytest
import torch

import synth
from oracle import revive_oracle as orc
from paper_2602_21140_amd.binding import ReviveLayer, lib

pytestmark = pytest.mark.gpu


def _call(fn, L, x, phys, T, outs, stream):
    x_perm, offs, dst, src = outs
    rc = fn(L._ctx, x.data_ptr(), phys.data_ptr(), T, x_perm.data_ptr(), offs.data_ptr(), dst.data_ptr(), src.data_ptr(),
            stream.cuda_stream)
    assert rc == 0, lib().revive_last_error(L._ctx).decode()


def test_static_scratch_dispatch_matches_the_workspace_one_twice_in_a_row():
    raw = lib()
    cfg = synth.scaled(synth.get_config("c2"), T=5000, H=256, I=64, I_shared=0)     # 30000 routed rows: 30 chunks, ragged tail
    L = ReviveLayer(cfg)
    try:
        dev = L.device
        x = synth.draw_x(cfg, dev)
        rng = np.random.default_rng(5)
        stream = torch.cuda.Stream()
        i32 = torch.int32
        for T in (cfg.T, 1237):                # the second call is smaller and finds the first call's leftovers
            N = T * cfg.k
            phys_h = rng.integers(0, cfg.P, size=(T, cfg.k)).astype(np.int32)
            phys_h[rng.random((T, cfg.k)) < 0.3] = 5          # one crowded slot
            phys = torch.from_numpy(phys_h).to(dev)
            ref = tuple(t.to(dev) for t in (torch.zeros(N, cfg.H, dtype=L.dtype), torch.zeros(cfg.P + 1, dtype=i32),
                                            torch.zeros(N, dtype=i32), torch.zeros(N, dtype=i32)))
            got = tuple(torch.full_like(t, 7) for t in ref)
            torch.cuda.synchronize()
            _call(raw.revive_dispatch, L, x, phys, T, ref, stream)
            _call(raw.revive_dispatch_static, L, x, phys, T, got, stream)
            stream.synchronize()
            for name, a, b in zip(("x_perm", "slot_offsets", "dst_row", "src_of"), ref, got):
                assert torch.equal(a, b), (T, name)
            offs, dst, src = orc.dispatch_indices(phys_h, cfg.P)
            assert np.array_equal(got[1].cpu().numpy(), offs)
            assert np.array_equal(got[2].cpu().numpy(), dst) and np.array_equal(got[3].cpu().numpy(), src)
            assert torch.equal(got[0], x[torch.from_numpy(src // cfg.k).to(dev).long()])
        # beyond the static array's capacity: a clear error, nothing launched
        big = synth.scaled(cfg, T=70000 // cfg.k + 1)
        Lb = ReviveLayer(big)
        try:
            T = big.T
            N = T * big.k
            assert N > 65536
            outs = (Lb.empty(N, big.H), Lb.empty(big.P + 1, dtype=i32), Lb.empty(N, dtype=i32), Lb.empty(N, dtype=i32))
            xb = Lb.empty(T, big.H)
            pb = torch.zeros(T, big.k, dtype=i32, device=dev)
            rc = raw.revive_dispatch_static(Lb._ctx, xb.data_ptr(), pb.data_ptr(), T, outs[0].data_ptr(), outs[1].data_ptr(),
                                            outs[2].data_ptr(), outs[3].data_ptr(), stream.cuda_stream)
            assert rc == -1 and "65536" in raw.revive_last_error(Lb._ctx).decode()
        finally:
            Lb.close()
    finally:
        L.close()


def test_static_scratch_dispatch_needs_no_workspace():
    """A context that never had a workspace bound can still dispatch through the static array."""
    raw = lib()
    cfg = synth.scaled(synth.get_config("c1"), T=300)
    from paper_2602_21140_amd.binding import make_config
    ctx = C.c_void_p()
    cc = make_config(cfg)
    assert raw.revive_create(C.byref(cc), C.byref(ctx)) == 0
    try:
        dev = torch.device("cuda:0")
        x = synth.draw_x(cfg, dev)
        rng = np.random.default_rng(6)
        phys_h = rng.integers(0, cfg.P, size=(cfg.T, cfg.k)).astype(np.int32)
        phys = torch.from_numpy(phys_h).to(dev)
        N = cfg.T * cfg.k
        i32 = torch.int32
        outs = (torch.empty(N, cfg.H, device=dev), torch.empty(cfg.P + 1, dtype=i32, device=dev),
                torch.empty(N, dtype=i32, device=dev), torch.empty(N, dtype=i32, device=dev))
        s = torch.cuda.current_stream().cuda_stream
        rc = raw.revive_dispatch(ctx, x.data_ptr(), phys.data_ptr(), cfg.T, outs[0].data_ptr(), outs[1].data_ptr(),
                                 outs[2].data_ptr(), outs[3].data_ptr(), s)
        assert rc == -3                         # the ordinary call refuses: no workspace bound
        rc = raw.revive_dispatch_static(ctx, x.data_ptr(), phys.data_ptr(), cfg.T, outs[0].data_ptr(), outs[1].data_ptr(),
                                        outs[2].data_ptr(), outs[3].data_ptr(), s)
        assert rc == 0
        torch.cuda.synchronize()
        offs, dst, src = orc.dispatch_indices(phys_h, cfg.P)
        assert np.array_equal(outs[1].cpu().numpy(), offs) and np.array_equal(outs[2].cpu().numpy(), dst)
        assert torch.equal(outs[0], x[torch.from_numpy(src // cfg.k).to(dev).long()])
    finally:
        raw.revive_destroy(ctx)
