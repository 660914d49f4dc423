"""The backward entry point that allocates nothing (bp_embbag_bwd_update_grouped_static: its scratch is a fixed array
inside the library) against bp_embbag_bwd_update_grouped on the same batches: two calls in a row, the second with a
smaller batch, weights and optimizer state bit for bit; and a batch too large for the array is refused."""
import numpy as np
import pytest
import torch

import grouping

pytestmark = pytest.mark.gpu


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def make_batch(rng, bags, C, D, max_len):
    if max_len == 1:
        off = np.arange(bags + 1, dtype=np.int64)
    else:
        off = np.zeros(bags + 1, dtype=np.int64)
        off[1:] = np.cumsum(rng.integers(0, max_len + 1, size=bags))
    n = int(off[-1])
    # Zipf slots: slot 0 takes ~30 % of the lookups (several pieces), a few dozen slots are long rows
    slots = np.minimum(rng.zipf(1.25, size=n) - 1, C - 1).astype(np.int32)
    grad = rng.standard_normal((bags, D)).astype(np.float32)
    return slots, off, grad


@pytest.mark.parametrize("D,dtype,optimizer,max_len", [(48, "f32", "adagrad", 1), (128, "bf16", "adagrad_rowwise", 1),
                                                      (16, "f32", "sgd", 7)])
def test_static_scratch_matches_workspace_variant(D, dtype, optimizer, max_len):
    import paper_2202_12429_amd as bp
    C = 20000
    rng = np.random.default_rng(D)
    cfg = bp.make_config(10 * C, C, D, dtype, optimizer, lr=0.01, eps=1e-8)
    wdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    w0 = torch.from_numpy(rng.uniform(-0.05, 0.05, size=(C, D)).astype(np.float32)).to(wdt)
    s_shape = (C, D) if optimizer == "adagrad" else (C,) if optimizer == "adagrad_rowwise" else None
    s0 = None if s_shape is None else torch.from_numpy(rng.uniform(0, 2, size=s_shape).astype(np.float32))
    wa, wb = w0.cuda(), w0.cuda()
    sa, sb = (None, None) if s0 is None else (s0.cuda(), s0.cuda())
    assert bp.bp_embbag_bwd_update_grouped_static_max_bytes() == 16 << 20
    for bags in (60000, 5003):                       # the second call is the smaller one
        slots, off, grad = make_batch(rng, bags, C, D, max_len)
        n = len(slots)
        gl, rows, roff, pieces, poff = grouping.build_grouping(slots.astype(np.int64), np.array([0, n]), slots)
        assert (pieces.view(np.uint32)[:, 4] > 1).any(), "the batch must hold a row of several pieces"
        gl_d, rows_d, pieces_d, grad_d = dev(gl), dev(rows), dev(pieces), dev(grad)
        off_d = None if max_len == 1 else dev(off)
        ws = torch.empty(bp.bp_embbag_bwd_update_grouped_workspace_bytes(cfg, n, bags, max_len != 1), dtype=torch.uint8,
                         device="cuda")
        bp.bp_embbag_bwd_update_grouped(cfg, wa, sa, gl_d, rows_d, pieces_d, off_d, bags, grad_d, ws, bp.bwd_tickets(n))
        assert bp.bp_embbag_bwd_update_grouped_static_bytes(cfg, n, bags, max_len != 1) <= 16 << 20
        bp.bp_embbag_bwd_update_grouped_static(cfg, wb, sb, gl_d, rows_d, pieces_d, off_d, bags, grad_d)
        torch.cuda.synchronize()
        assert torch.equal(wa.view(torch.int16) if dtype == "bf16" else wa, wb.view(torch.int16) if dtype == "bf16" else wb)
        assert sa is None or torch.equal(sa, sb)
    assert not torch.equal(wa.cpu(), w0)             # the updates did something


def test_static_scratch_refuses_what_does_not_fit():
    import paper_2202_12429_amd as bp
    cfg = bp.make_config(1000, 100, 64, "f32", "sgd")
    n = 3_000_000                                    # bags of several lookups: two 4-byte maps per lookup = 24 MB
    with pytest.raises(bp.BagpipeError) as e:
        bp.bp_embbag_bwd_update_grouped_static_bytes(cfg, 20_000_000, 20_000_000, False)     # more counters than the array has
    assert e.value.status == -6
    assert bp.bp_embbag_bwd_update_grouped_static_bytes(cfg, n, n, True) > 16 << 20
    t = torch.zeros(16, dtype=torch.int32, device="cuda")
    with pytest.raises(bp.BagpipeError) as e:
        lib = bp.load_library()
        import ctypes
        st = lib.bp_embbag_bwd_update_grouped_static(ctypes.byref(cfg), t.data_ptr(), None, t.data_ptr(), t.data_ptr(), 1, None,
                                                    0, t.data_ptr(), n, n, t.data_ptr(), None)
        if st != 0:
            raise bp.BagpipeError(st, bp.bp_last_error_message())
    assert e.value.status == -6
