"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded inputs.

Bars: plans / slot maps / lists bit-exact; pooled outputs relative 1e-5 (bit-exact for one-hot bags); final
table within 1e-4 (helpers.assert_*).  Sizes span several sort and scan tiles and end in ragged tails."""
import sys

import numpy as np
import pytest
import torch

import grouping
import helpers
import oracle
import workloads

pytestmark = pytest.mark.gpu


say = helpers.say


@pytest.fixture(scope="module")
def bp():
    import paper_2202_12429_amd as bp
    bp.load_library()
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return bp


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.cuda()


# ---------------------------------------------------------------------------------------------------
# forward
# ---------------------------------------------------------------------------------------------------
def random_cache(C, D, dtype, seed):
    rng = np.random.default_rng(seed)
    w = torch.from_numpy(rng.uniform(-0.05, 0.05, size=(C, D)).astype(np.float32))
    if dtype == "bf16":
        w = w.to(torch.bfloat16)
    return w


def cache_numpy(w):
    return w.view(torch.int16).numpy().view(np.uint16).copy() if w.dtype == torch.bfloat16 else w.numpy().copy()


def random_bags(rng, bags, max_len, C, allow_empty=True):
    lens = rng.integers(0 if allow_empty else 1, max_len + 1, size=bags)
    off = np.zeros(bags + 1, dtype=np.int64)
    off[1:] = np.cumsum(lens)
    n = int(off[-1])
    slots = np.minimum(rng.zipf(1.3, size=n) - 1, C - 1).astype(np.int32)
    return off, slots


@pytest.mark.parametrize("D,dtype", [(16, "f32"), (48, "f32"), (64, "f32"), (128, "bf16"), (8, "bf16"), (4, "f32"),
                                     (256, "f32")])
@pytest.mark.parametrize("max_len", [1, 50])
def test_forward(bp, D, dtype, max_len):
    say(f"forward D={D} {dtype} max_len={max_len}")
    C, bags = 5000, 3001                                        # ragged: not a multiple of any group count
    rng = np.random.default_rng(D * 7 + max_len)
    w = random_cache(C, D, dtype, D)
    cfg = bp.make_config(10 * C, C, D, dtype)
    out = torch.full((bags, D), float("nan"), device="cuda")
    if max_len == 1:
        slots = rng.integers(0, C, size=bags).astype(np.int32)
        off = np.arange(bags + 1, dtype=np.int64)
        bp.bp_embbag_fwd(cfg, w.cuda(), dev(slots), None, bags, out)
    else:
        off, slots = random_bags(rng, bags, max_len, C)
        bp.bp_embbag_fwd(cfg, w.cuda(), dev(slots), dev(off), bags, out)
    torch.cuda.synchronize()
    want = oracle.train_iter(cache_numpy(w), None, D, oracle.DTYPES[dtype], oracle.SGD, 0.0, 0.0, slots, off, None)
    helpers.assert_outputs_close(out.cpu().numpy(), want, max_len)


def test_forward_edge_cases(bp):
    say("forward edge cases")
    C, D = 64, 16
    w = random_cache(C, D, "f32", 1)
    cfg = bp.make_config(1000, C, D)
    # zero bags: a no-op
    bp.bp_embbag_fwd(cfg, w.cuda(), torch.zeros(0, dtype=torch.int32, device="cuda"), None, 0,
                     torch.zeros((0, D), device="cuda"))
    # all bags empty -> zeros; out-of-range slots contribute nothing
    out = torch.full((5, D), 7.0, device="cuda")
    bp.bp_embbag_fwd(cfg, w.cuda(), torch.zeros(0, dtype=torch.int32, device="cuda"), dev(np.zeros(6, np.int64)), 5, out)
    assert not out.cpu().numpy().any()
    slots = np.array([3, -1, 64, 5, 1 << 30], dtype=np.int32)
    out = torch.full((2, D), 7.0, device="cuda")
    bp.bp_embbag_fwd(cfg, w.cuda(), dev(slots), dev(np.array([0, 3, 5], np.int64)), 2, out)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), np.stack([w[3].numpy(), w[5].numpy()]))
    # n_lookups != bags without offsets is an argument error
    with pytest.raises(bp.BagpipeError) as e:
        bp.bp_embbag_fwd(cfg, w.cuda(), dev(slots), None, 2, out)
    assert e.value.status == -1


def one_hot_grouping(slots, C):
    """Row and piece records of one batch of single-lookup bags whose rows are the slots themselves."""
    off = np.array([0, len(slots)], dtype=np.int64)
    gl, rows, _, pieces, _ = grouping.build_grouping(slots.astype(np.int64), off, slots)
    return gl, rows, pieces


@pytest.mark.parametrize("D,dtype,pad", [(16, "f32", 0), (48, "f32", 0), (48, "f32", 192), (64, "f32", 0), (128, "bf16", 0),
                                         (8, "bf16", 16), (4, "f32", 0), (256, "f32", 0)])
def test_forward_grouped(bp, D, dtype, pad):
    """bp_embbag_fwd_grouped against the oracle's row copies and against bp_embbag_fwd, bit for bit: short rows, rows
    of one piece and of several pieces, a ragged tail; dense and strided cache rows."""
    say(f"forward over row records D={D} {dtype} pad={pad}")
    C, bags = 5000, 30011
    rng = np.random.default_rng(D * 11 + pad)
    w = random_cache(C, D, dtype, D + 1)
    slots = np.minimum(rng.zipf(1.25, size=bags) - 1, C - 1).astype(np.int32)       # slot 0: thousands of lookups
    assert np.bincount(slots).max() > 3 * grouping.PIECE
    gl, rows, pieces = one_hot_grouping(slots, C)
    esz = 2 if dtype == "bf16" else 4
    if pad:
        buf = torch.zeros((C, D * esz + pad), dtype=torch.uint8)
        buf[:, :D * esz] = w.view(torch.uint8).reshape(C, D * esz)
        cfg = bp.make_config(10 * C, C, D, dtype, cache_w_stride=D * esz + pad)
        wd = buf.cuda()
    else:
        cfg = bp.make_config(10 * C, C, D, dtype)
        wd = w.cuda()
    out = torch.full((bags, D), float("nan"), device="cuda")
    bp.bp_embbag_fwd_grouped(cfg, wd, dev(gl), dev(rows), dev(pieces), bags, out)
    ref = torch.full((bags, D), float("nan"), device="cuda")
    bp.bp_embbag_fwd(cfg, wd, dev(slots), None, bags, ref)
    torch.cuda.synchronize()
    off = np.arange(bags + 1, dtype=np.int64)
    want = oracle.train_iter(cache_numpy(w), None, D, oracle.DTYPES[dtype], oracle.SGD, 0.0, 0.0, slots, off, None)
    got = out.cpu().numpy()
    assert np.array_equal(got, want.astype(np.float32))
    assert np.array_equal(got, ref.cpu().numpy())


def test_forward_grouped_edge_cases(bp):
    say("forward over row records: edge cases")
    C, D, bags = 64, 16, 40
    w = random_cache(C, D, "f32", 3)
    cfg = bp.make_config(1000, C, D)
    empty_i32 = torch.zeros(0, dtype=torch.int32, device="cuda")
    bp.bp_embbag_fwd_grouped(cfg, w.cuda(), empty_i32, torch.zeros((0, 4), dtype=torch.int32, device="cuda"), None, 0,
                             torch.zeros((0, D), device="cuda"))
    rng = np.random.default_rng(5)
    slots = rng.integers(0, 8, size=bags).astype(np.int32)
    gl, rows, pieces = one_hot_grouping(slots, C)
    rows = rows.copy()
    u = rows.view(np.uint32)
    # records that name a slot outside the cache, lookups outside the batch or no lookups write nothing
    dead = {0: (2, 1 << 30), 1: (1, bags + 5), 2: (1, 0)}
    skipped = np.zeros(bags, dtype=bool)
    for r, (col, val) in dead.items():
        a, n = int(u[r, 0] & 0x7fffffff), int(u[r, 1])
        skipped[gl[a:a + n]] = True
        u[r, col] = val
    gl2 = gl.copy()
    a5, n5 = int(u[5, 0] & 0x7fffffff), int(u[5, 1])
    assert n5 >= 2
    skipped[gl[a5 + 1]] = True
    gl2[a5 + 1] = bags + 7                                   # a grouped lookup that names no bag of the batch
    skipped[u[3, 3]] = True
    u[3, 3] = bags + 9                                       # nor does this row's first lookup
    out = torch.full((bags, D), 7.0, device="cuda")
    bp.bp_embbag_fwd_grouped(cfg, w.cuda(), dev(gl2), dev(rows), dev(pieces), bags, out)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    assert np.array_equal(got[~skipped], w.numpy()[slots[~skipped]])
    assert (got[skipped] == 7.0).all()
    with pytest.raises(bp.BagpipeError) as e:                # more rows than lookups cannot be a batch's records
        bp.bp_embbag_fwd_grouped(cfg, w.cuda(), dev(gl[:3]), dev(rows), None, 3, out)
    assert e.value.status == -1


# ---------------------------------------------------------------------------------------------------
# backward + update
# ---------------------------------------------------------------------------------------------------
def run_bwd(bp, cfg, w, state, slots, off, bags, grad, onehot):
    wd = w.cuda()
    sd = None if state is None else torch.from_numpy(state).cuda()
    ws = torch.empty(bp.bp_embbag_bwd_update_workspace_bytes(cfg, len(slots), bags), dtype=torch.uint8, device="cuda")
    tk = bp.bwd_tickets(len(slots))
    bp.bp_embbag_bwd_update(cfg, wd, sd, dev(slots), None if onehot else dev(off), bags, dev(grad), ws, tk)
    torch.cuda.synchronize()
    assert not tk.any(), "the call must leave its counters zero"
    return wd.cpu(), None if sd is None else sd.cpu().numpy()


def run_bwd_grouped(bp, cfg, w, state, slots, off, bags, grad, onehot):
    valid = (slots >= 0) & (slots < cfg.capacity)
    assert valid.all()
    gl, rows, roff, pieces, poff = grouping.build_grouping(slots.astype(np.int64), np.array([0, len(slots)]), slots)
    wd = w.cuda()
    sd = None if state is None else torch.from_numpy(state).cuda()
    ws = torch.empty(bp.bp_embbag_bwd_update_grouped_workspace_bytes(cfg, len(slots), bags, not onehot),
                     dtype=torch.uint8, device="cuda")
    tk = bp.bwd_tickets(len(slots))
    bp.bp_embbag_bwd_update_grouped(cfg, wd, sd, dev(gl), dev(rows), dev(pieces) if len(pieces) else None,
                                    None if onehot else dev(off), bags, dev(grad), ws, tk)
    torch.cuda.synchronize()
    assert not tk.any(), "the call must leave its counters zero"
    return wd.cpu(), None if sd is None else sd.cpu().numpy()


@pytest.mark.parametrize("D,dtype,optimizer", [(16, "f32", "sgd"), (48, "f32", "adagrad"), (64, "f32", "sgd"),
                                               (128, "bf16", "adagrad_rowwise"), (32, "bf16", "adagrad"),
                                               (48, "f32", "adagrad_rowwise"), (8, "bf16", "sgd"),
                                               # one lane, 32 and 64 lanes per row (1,024-byte rows are the limit)
                                               (4, "f32", "adagrad"), (128, "f32", "sgd"), (256, "f32", "adagrad"),
                                               (512, "bf16", "adagrad_rowwise"), (160, "f32", "adagrad_rowwise")])
@pytest.mark.parametrize("max_len", [1, 20])
def test_backward_update(bp, D, dtype, optimizer, max_len):
    say(f"backward D={D} {dtype} {optimizer} max_len={max_len}")
    C, bags = 3000, 5003
    rng = np.random.default_rng(D + max_len)
    w = random_cache(C, D, dtype, D + 1)
    op = oracle.OPTIMIZERS[optimizer]
    state = rng.uniform(0.0, 2.0, size=oracle.state_shape(C, D, op)).astype(np.float32) if op != oracle.SGD else None
    cfg = bp.make_config(10 * C, C, D, dtype, optimizer, lr=0.01, eps=1e-8)
    if max_len == 1:
        # Zipf slots: slot 0 is hit by ~30 % of the lookups, so it spans many chunks and tiles
        slots = np.minimum(rng.zipf(1.25, size=bags) - 1, C - 1).astype(np.int32)
        off = np.arange(bags + 1, dtype=np.int64)
    else:
        off, slots = random_bags(rng, bags, max_len, C)
    grad = rng.standard_normal((bags, D)).astype(np.float32)
    got_w, got_s = run_bwd(bp, cfg, w, state, slots, off, bags, grad, max_len == 1)
    again_w, again_s = run_bwd(bp, cfg, w, state, slots, off, bags, grad, max_len == 1)
    # the grouped entry point on the same batch (grouping by slot is a grouping by row) gives the same bits: the
    # fp64 partial sums of a few thousand fp32 values of similar size are exact, so the cuts do not matter
    grp_w, grp_s = run_bwd_grouped(bp, cfg, w, state, slots, off, bags, grad, max_len == 1)
    assert np.array_equal(cache_numpy(grp_w), cache_numpy(got_w)) and (got_s is None or np.array_equal(grp_s, got_s))
    assert torch.equal(got_w.view(torch.int16) if dtype == "bf16" else got_w,
                       again_w.view(torch.int16) if dtype == "bf16" else again_w), "backward is not deterministic"
    want_w = cache_numpy(w)
    want_s = None if state is None else state.copy()
    oracle.train_iter(want_w, want_s, D, oracle.DTYPES[dtype], op, 0.01, 1e-8, slots, off, grad, want_out=False)
    if dtype == "bf16":
        # storage rounding decides a bf16 code, so both sides form the value to be rounded the same way (fp64 sums
        # rounded once, fp32 element-wise steps): the codes and the fp32 state must agree bit for bit
        assert np.array_equal(cache_numpy(got_w), want_w)
        if want_s is not None:
            assert np.array_equal(got_s, want_s)
    else:
        helpers.assert_weights_close(got_w.numpy(), want_w)
        assert np.abs(got_w.numpy() - w.numpy()).max() > 1e-4
    if want_s is not None:
        np.testing.assert_allclose(got_s, want_s, rtol=1e-4, atol=1e-9)     # same bar as the weights
        assert np.array_equal(again_s, got_s)
    # untouched rows keep their bits
    touched = np.zeros(C, bool)
    touched[slots[(slots >= 0) & (slots < C)]] = True
    assert np.array_equal(cache_numpy(got_w)[~touched], cache_numpy(w)[~touched])


def test_backward_degenerate(bp):
    say("backward degenerate: one slot takes every lookup; out-of-range slots; empty input")
    C, D, n = 128, 16, 4099
    w = random_cache(C, D, "f32", 3)
    cfg = bp.make_config(1000, C, D, "f32", "sgd", lr=0.5)
    slots = np.full(n, 7, dtype=np.int32)
    slots[::501] = -5
    slots[1::777] = C + 3
    grad = np.random.default_rng(0).standard_normal((n, D)).astype(np.float32)
    got, _ = run_bwd(bp, cfg, w, None, slots, np.arange(n + 1), n, grad, True)
    valid = slots == 7
    want = w.numpy().copy()
    want[7] = (want[7].astype(np.float64) - np.float64(np.float32(0.5)) * grad[valid].astype(np.float64).sum(0)).astype(np.float32)
    helpers.assert_weights_close(got.numpy(), want)
    assert np.array_equal(np.delete(got.numpy(), 7, axis=0), np.delete(w.numpy(), 7, axis=0))
    # n = 0 is a no-op
    ws = torch.empty(bp.bp_embbag_bwd_update_workspace_bytes(cfg, 0, 0), dtype=torch.uint8, device="cuda")
    tk = bp.bwd_tickets(n)
    bp.bp_embbag_bwd_update(cfg, w.cuda(), None, torch.zeros(0, dtype=torch.int32, device="cuda"), None, 0,
                            torch.zeros((0, D), device="cuda"), ws, tk)
    # workspace too small
    with pytest.raises(bp.BagpipeError) as e:
        bp.bp_embbag_bwd_update(cfg, w.cuda(), None, dev(slots), None, n, dev(grad), ws[:256], tk)
    assert e.value.status == -3


@pytest.mark.parametrize("D,dtype,optimizer,pad", [(48, "f32", "adagrad", 0), (16, "f32", "adagrad", 64),
                                                   (128, "bf16", "adagrad_rowwise", 12), (32, "f32", "sgd", 32)])
def test_strided_cache_equals_dense(bp, D, dtype, optimizer, pad):
    """A cache whose rows carry their optimizer state right behind the weights (one record per slot, bp_config's two
    strides), with and without padding: forward, both backward entry points and every maintenance call give, bit for
    bit, what two dense arrays give."""
    say(f"strided cache D={D} {dtype} {optimizer} pad={pad}")
    C, R, bags = 2000, 5000, 6001
    rng = np.random.default_rng(D + pad)
    eb = 2 if dtype == "bf16" else 4
    rb = D * eb
    sb = D * 4 if optimizer == "adagrad" else 4 if optimizer == "adagrad_rowwise" else 0
    rec = rb + sb + pad                                       # bytes per slot: [weights | state | padding]
    dense = bp.make_config(R, C, D, dtype, optimizer, lr=0.01, eps=1e-8)
    strided = bp.make_config(R, C, D, dtype, optimizer, lr=0.01, eps=1e-8, cache_w_stride=rec,
                             cache_state_stride=rec if sb else 0)
    wdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    w0 = torch.from_numpy(rng.uniform(-0.05, 0.05, size=(C, D)).astype(np.float32)).to(wdt).cuda()
    s0 = None
    if sb:
        s0 = torch.from_numpy(rng.uniform(0, 2, size=(C, D) if optimizer == "adagrad" else (C,)).astype(np.float32)).cuda()
    buf = torch.full((C, rec), 0x5A, dtype=torch.uint8, device="cuda")

    def pack():
        buf[:, :rb] = w0.contiguous().view(torch.uint8).view(C, rb)
        if sb:
            buf[:, rb:rb + sb] = s0.contiguous().view(torch.uint8).view(C, sb)
    def unpack():
        w = buf[:, :rb].contiguous().view(wdt).view(C, D)
        s = buf[:, rb:rb + sb].contiguous().view(torch.float32).view(C, -1).squeeze(-1) if sb else None
        return w, s
    def same(a, b):
        return torch.equal(a.view(torch.int16) if a.dtype == torch.bfloat16 else a, b.view(torch.int16) if b.dtype == torch.bfloat16 else b)
    pw, ps = buf.data_ptr(), (buf.data_ptr() + rb) if sb else None

    slots = np.minimum(rng.zipf(1.25, size=bags) - 1, C - 1).astype(np.int32)
    grad = dev(rng.standard_normal((bags, D)).astype(np.float32))
    # forward
    pack()
    out_d = torch.empty((bags, D), device="cuda")
    out_s = torch.empty((bags, D), device="cuda")
    bp.bp_embbag_fwd(dense, w0, dev(slots), None, bags, out_d)
    bp.bp_embbag_fwd(strided, pw, dev(slots), None, bags, out_s)
    assert torch.equal(out_d, out_s)
    # backward, sorting and grouped
    gl, rows, roff, pieces, poff = grouping.build_grouping(slots.astype(np.int64), np.array([0, bags]), slots)
    for grouped in (False, True):
        pack()
        wd, sd = w0.clone(), None if s0 is None else s0.clone()
        tk = bp.bwd_tickets(bags)
        if grouped:
            ws = torch.empty(bp.bp_embbag_bwd_update_grouped_workspace_bytes(dense, bags, bags, False), dtype=torch.uint8, device="cuda")
            bp.bp_embbag_bwd_update_grouped(dense, wd, sd, dev(gl), dev(rows), dev(pieces), None, bags, grad, ws, tk)
            bp.bp_embbag_bwd_update_grouped(strided, pw, ps, dev(gl), dev(rows), dev(pieces), None, bags, grad, ws, tk)
        else:
            ws = torch.empty(bp.bp_embbag_bwd_update_workspace_bytes(dense, bags, bags), dtype=torch.uint8, device="cuda")
            bp.bp_embbag_bwd_update(dense, wd, sd, dev(slots), None, bags, grad, ws, tk)
            bp.bp_embbag_bwd_update(strided, pw, ps, dev(slots), None, bags, grad, ws, tk)
        torch.cuda.synchronize()
        w, s = unpack()
        assert same(w, wd) and (sd is None or torch.equal(s, sd)), ("grouped" if grouped else "sorting")
        assert not same(wd, w0)
    assert (buf[:, rb + sb:] == 0x5A).all(), "padding was written"
    # maintenance: evict 300 rows to a table, fetch 300 others, through each entry point
    tab_w = torch.from_numpy(rng.uniform(-1, 1, size=(R, D)).astype(np.float32)).to(wdt).cuda()
    tab_s = None if not sb else torch.from_numpy(rng.uniform(0, 2, size=(R, D) if optimizer == "adagrad" else (R,)).astype(np.float32)).cuda()
    perm = rng.permutation(C)[:300].astype(np.int32)
    ids = rng.permutation(R)[:600].astype(np.int64)
    e_ids, p_ids = dev(np.sort(ids[:300])), dev(np.sort(ids[300:]))
    e_slots, p_slots = dev(perm), dev(perm)                  # the fetched rows take the evicted rows' slots, in order
    for call in ("apply", "duplex", "handoff"):
        pack()
        wd, sd = w0.clone(), None if s0 is None else s0.clone()
        td_w, td_s = tab_w.clone(), None if tab_s is None else tab_s.clone()
        ts_w, ts_s = tab_w.clone(), None if tab_s is None else tab_s.clone()
        if call == "apply":
            bp.bp_cache_apply(dense, wd, sd, td_w, td_s, e_ids, e_slots, p_ids, p_slots)
            bp.bp_cache_apply(strided, pw, ps, ts_w, ts_s, e_ids, e_slots, p_ids, p_slots)
        elif call == "duplex":
            st = torch.empty(bp.bp_cache_apply_duplex_workspace_bytes(dense, 300), dtype=torch.uint8, device="cuda")
            bp.bp_cache_apply_duplex(dense, wd, sd, td_w, td_s, e_ids, e_slots, p_ids, p_slots, st)
            bp.bp_cache_apply_duplex(strided, pw, ps, ts_w, ts_s, e_ids, e_slots, p_ids, p_slots, st)
        else:
            flag = torch.zeros(1, dtype=torch.int32, device="cuda")
            bp.bp_cache_apply_handoff(dense, wd, sd, td_w, td_s, e_ids, e_slots, p_ids, p_slots, 0, flag)
            bp.bp_cache_apply_handoff(strided, pw, ps, ts_w, ts_s, e_ids, e_slots, p_ids, p_slots, 0, flag)
            assert int(flag.item()) == 0
        torch.cuda.synchronize()
        w, s = unpack()
        assert same(w, wd) and same(ts_w, td_w), call
        assert sd is None or (torch.equal(s, sd) and torch.equal(ts_s, td_s)), call
        assert not same(wd, w0) and not same(td_w, tab_w)


# ---------------------------------------------------------------------------------------------------
# cache maintenance
# ---------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("D,dtype,optimizer,pinned", [(16, "f32", "sgd", True), (48, "f32", "adagrad", True),
                                                      (128, "bf16", "adagrad_rowwise", True),
                                                      (64, "bf16", "adagrad", False),
                                                      (256, "f32", "adagrad", True), (4, "f32", "sgd", False)])
def test_cache_apply(bp, D, dtype, optimizer, pinned):
    say(f"cache_apply D={D} {dtype} {optimizer} pinned={pinned}")
    R, C = 20011, 1500
    rng = np.random.default_rng(D)
    op = oracle.OPTIMIZERS[optimizer]
    hw = random_cache(R, D, dtype, 11)
    cw = random_cache(C, D, dtype, 12)
    hs = rng.uniform(0, 1, size=oracle.state_shape(R, D, op)).astype(np.float32)
    cs = rng.uniform(1, 2, size=oracle.state_shape(C, D, op)).astype(np.float32)
    # evict 700 rows from distinct slots, then prefetch 900 rows, 400 of them into just-freed slots
    e_slots = rng.permutation(C)[:700].astype(np.int32)
    e_ids = rng.permutation(R)[:700].astype(np.int64)
    p_slots = np.concatenate([e_slots[:400], np.setdiff1d(np.arange(C), e_slots)[:500]]).astype(np.int32)
    p_ids = np.setdiff1d(np.arange(R), e_ids)[:900].astype(np.int64)
    p_ids[:50] = e_ids[:50]                       # re-fetch rows that were just written back
    cfg = bp.make_config(R, C, D, dtype, optimizer)
    mk = (lambda t: t.pin_memory()) if pinned else (lambda t: t.cuda())
    hw_d, cw_d = mk(hw.clone()), cw.cuda()
    hs_d = mk(torch.from_numpy(hs.copy())) if op != oracle.SGD else None
    cs_d = torch.from_numpy(cs.copy()).cuda() if op != oracle.SGD else None
    bp.bp_cache_apply(cfg, cw_d, cs_d, hw_d, hs_d, dev(e_ids), dev(e_slots), dev(p_ids), dev(p_slots))
    torch.cuda.synchronize()
    hw_o, cw_o, hs_o, cs_o = cache_numpy(hw), cache_numpy(cw), hs.copy(), cs.copy()
    oracle.cache_apply(cw_o, cs_o, hw_o, hs_o, D, oracle.DTYPES[dtype], op, e_ids, e_slots, p_ids, p_slots)
    assert np.array_equal(cache_numpy(hw_d.cpu()), hw_o) and np.array_equal(cache_numpy(cw_d.cpu()), cw_o)
    if op != oracle.SGD:
        assert np.array_equal(hs_d.cpu().numpy(), hs_o) and np.array_equal(cs_d.cpu().numpy(), cs_o)
    # empty lists are no-ops
    bp.bp_cache_apply(cfg, cw_d, cs_d, hw_d, hs_d, None, None, None, None)
    # the duplex variant on id-disjoint lists gives the same bytes
    p_ids2 = np.setdiff1d(np.arange(R), e_ids)[:900].astype(np.int64)
    hw_o, cw_o, hs_o, cs_o = cache_numpy(hw), cache_numpy(cw), hs.copy(), cs.copy()
    oracle.cache_apply(cw_o, cs_o, hw_o, hs_o, D, oracle.DTYPES[dtype], op, e_ids, e_slots, p_ids2, p_slots)
    hw_d, cw_d = mk(hw.clone()), cw.cuda()
    hs_d = mk(torch.from_numpy(hs.copy())) if op != oracle.SGD else None
    cs_d = torch.from_numpy(cs.copy()).cuda() if op != oracle.SGD else None
    ws = torch.empty(bp.bp_cache_apply_duplex_workspace_bytes(cfg, len(e_ids)), dtype=torch.uint8, device="cuda")
    bp.bp_cache_apply_duplex(cfg, cw_d, cs_d, hw_d, hs_d, dev(e_ids), dev(e_slots), dev(p_ids2), dev(p_slots), ws)
    bp.bp_cache_apply_duplex(cfg, cw_d, cs_d, hw_d, hs_d, None, None, None, None, None)          # no-op
    torch.cuda.synchronize()
    assert np.array_equal(cache_numpy(hw_d.cpu()), hw_o) and np.array_equal(cache_numpy(cw_d.cpu()), cw_o)
    if op != oracle.SGD:
        assert np.array_equal(hs_d.cpu().numpy(), hs_o) and np.array_equal(cs_d.cpu().numpy(), cs_o)
    # only evictions, only prefetches
    bp.bp_cache_apply_duplex(cfg, cw_d, cs_d, hw_d, hs_d, dev(e_ids), dev(e_slots), None, None, ws)
    bp.bp_cache_apply_duplex(cfg, cw_d, cs_d, hw_d, hs_d, None, None, dev(p_ids2), dev(p_slots), None)
    oracle.cache_apply(cw_o, cs_o, hw_o, hs_o, D, oracle.DTYPES[dtype], op, e_ids, e_slots, np.zeros(0, np.int64), np.zeros(0, np.int32))
    oracle.cache_apply(cw_o, cs_o, hw_o, hs_o, D, oracle.DTYPES[dtype], op, np.zeros(0, np.int64), np.zeros(0, np.int32), p_ids2, p_slots)
    torch.cuda.synchronize()
    assert np.array_equal(cache_numpy(hw_d.cpu()), hw_o) and np.array_equal(cache_numpy(cw_d.cpu()), cw_o)


@pytest.mark.parametrize("D,dtype,optimizer,pinned", [(48, "f32", "adagrad", True), (128, "bf16", "adagrad_rowwise", False),
                                                      (16, "f32", "sgd", True)])
def test_cache_apply_handoff(bp, D, dtype, optimizer, pinned):
    """Maintenance in one launch: 700 evictions, 900 prefetches of which the last 400 take the first 400 evicted
    slots in order (the pairing of a FIFO plan) and 500 go to free slots.  Same bytes as the oracle's two-step rule."""
    say(f"cache_apply_handoff D={D} {dtype} {optimizer} pinned={pinned}")
    R, C = 20011, 1500
    rng = np.random.default_rng(D + 5)
    op = oracle.OPTIMIZERS[optimizer]
    hw, cw = random_cache(R, D, dtype, 41), random_cache(C, D, dtype, 42)
    hs = rng.uniform(0, 1, size=oracle.state_shape(R, D, op)).astype(np.float32)
    cs = rng.uniform(1, 2, size=oracle.state_shape(C, D, op)).astype(np.float32)
    e_slots = rng.permutation(C)[:700].astype(np.int32)
    e_ids = rng.permutation(R)[:700].astype(np.int64)
    free = np.setdiff1d(np.arange(C), e_slots)[:500]
    p_slots = np.concatenate([free, e_slots[:400]]).astype(np.int32)              # early ones first, then the paired ones
    p_ids = rng.permutation(np.setdiff1d(np.arange(R), e_ids))[:900].astype(np.int64)
    cfg = bp.make_config(R, C, D, dtype, optimizer)
    mk = (lambda t: t.pin_memory()) if pinned else (lambda t: t.cuda())

    def run(n_early, ps):
        hw_d, cw_d = mk(hw.clone()), cw.cuda()
        hs_d = mk(torch.from_numpy(hs.copy())) if op != oracle.SGD else None
        cs_d = torch.from_numpy(cs.copy()).cuda() if op != oracle.SGD else None
        flag = torch.zeros(1, dtype=torch.int32, device="cuda")
        bp.bp_cache_apply_handoff(cfg, cw_d, cs_d, hw_d, hs_d, dev(e_ids), dev(e_slots), dev(p_ids), dev(ps), n_early, flag)
        torch.cuda.synchronize()
        return hw_d, cw_d, hs_d, cs_d, int(flag.item())

    hw_d, cw_d, hs_d, cs_d, flag = run(500, p_slots)
    hw_o, cw_o, hs_o, cs_o = cache_numpy(hw), cache_numpy(cw), hs.copy(), cs.copy()
    oracle.cache_apply(cw_o, cs_o, hw_o, hs_o, D, oracle.DTYPES[dtype], op, e_ids, e_slots, p_ids, p_slots)
    assert flag == 0
    assert np.array_equal(cache_numpy(hw_d.cpu()), hw_o) and np.array_equal(cache_numpy(cw_d.cpu()), cw_o)
    if op != oracle.SGD:
        assert np.array_equal(hs_d.cpu().numpy(), hs_o) and np.array_equal(cs_d.cpu().numpy(), cs_o)
    # a pair whose slots differ is reported, its slot is left alone, everything is still written back
    bad = p_slots.copy()
    bad[500 + 7], bad[500 + 8] = bad[500 + 8], bad[500 + 7]
    hw_d, cw_d, hs_d, cs_d, flag = run(500, bad)
    assert flag == 1
    assert np.array_equal(cache_numpy(hw_d.cpu()), hw_o)
    assert np.array_equal(cache_numpy(cw_d.cpu())[e_slots[7]], cache_numpy(cw)[e_slots[7]])
    # argument errors: more late prefetches than evictions
    with pytest.raises(bp.BagpipeError) as e:
        bp.bp_cache_apply_handoff(cfg, cw_d, cs_d, hw_d, hs_d, dev(e_ids[:10]), dev(e_slots[:10]), dev(p_ids),
                                  dev(p_slots), 100, None)
    assert e.value.status == -1
    # no lists: nothing to do
    bp.bp_cache_apply_handoff(cfg, cw_d, cs_d, hw_d, hs_d, None, None, None, None, 0, None)


def test_cache_stage_then_apply_staged(bp):
    """The two halves of the duplex maintenance called on their own, with unrelated work on the cache between them
    (the staged rows' slots are overwritten before the write-back): backing table and cache as the oracle's."""
    say("cache_stage + cache_apply_staged")
    R, C, D = 9001, 800, 48
    rng = np.random.default_rng(21)
    hw, cw = random_cache(R, D, "f32", 31), random_cache(C, D, "f32", 32)
    hs = rng.uniform(0, 1, size=(R, D)).astype(np.float32)
    cs = rng.uniform(1, 2, size=(C, D)).astype(np.float32)
    e_slots = rng.permutation(C)[:300].astype(np.int32)
    e_ids = rng.permutation(R)[:300].astype(np.int64)
    p_slots = np.concatenate([e_slots[:200], np.setdiff1d(np.arange(C), e_slots)[:100]]).astype(np.int32)
    p_ids = np.setdiff1d(np.arange(R), e_ids)[:300].astype(np.int64)
    cfg = bp.make_config(R, C, D, "f32", "adagrad")
    hw_d, cw_d = hw.clone().pin_memory(), cw.cuda()
    hs_d, cs_d = torch.from_numpy(hs.copy()).pin_memory(), torch.from_numpy(cs.copy()).cuda()
    ws = torch.empty(bp.bp_cache_apply_duplex_workspace_bytes(cfg, 300), dtype=torch.uint8, device="cuda")
    bp.bp_cache_stage(cfg, cw_d, cs_d, dev(e_slots), ws)
    cw_d[torch.from_numpy(e_slots[:200].astype(np.int64)).cuda()] = 7.0        # the freed slots are reused at once
    bp.bp_cache_apply_staged(cfg, cw_d, cs_d, hw_d, hs_d, dev(e_ids), dev(e_slots), ws, dev(p_ids), dev(p_slots))
    torch.cuda.synchronize()
    hw_o, cw_o, hs_o, cs_o = hw.numpy().copy(), cw.numpy().copy(), hs.copy(), cs.copy()
    oracle.cache_apply(cw_o, cs_o, hw_o, hs_o, D, oracle.F32, oracle.ADAGRAD, e_ids, e_slots, p_ids, p_slots)
    assert np.array_equal(hw_d.numpy(), hw_o) and np.array_equal(hs_d.numpy(), hs_o)
    assert np.array_equal(cw_d.cpu().numpy(), cw_o) and np.array_equal(cs_d.cpu().numpy(), cs_o)
    # argument errors: staging too small, misaligned
    with pytest.raises(bp.BagpipeError) as e:
        bp.bp_cache_stage(cfg, cw_d, cs_d, dev(e_slots), ws[:256])
    assert e.value.status == -3
    with pytest.raises(bp.BagpipeError) as e:
        bp.bp_cache_apply_staged(cfg, cw_d, cs_d, hw_d, hs_d, dev(e_ids), dev(e_slots), ws[16:], dev(p_ids), dev(p_slots))
    assert e.value.status == -1


# ---------------------------------------------------------------------------------------------------
# planner
# ---------------------------------------------------------------------------------------------------
def assert_plan_equal(got, want, N):
    assert got.L_eff == want.L_eff
    assert np.array_equal(got.occupancy, want.occ) and got.peak_occupancy == want.peak
    for name, oname in (("prefetch_offsets", "prefetch_off"), ("evict_offsets", "evict_off"), ("keep_offsets", "keep_off")):
        assert np.array_equal(getattr(got, name), getattr(want, oname)), name
    for name in ("prefetch_ids", "prefetch_slots", "evict_ids", "evict_slots", "keep_ids", "keep_ttl"):
        assert np.array_equal(getattr(got, name).cpu().numpy(), getattr(want, name)), name
    if got.lookup_slots is not None:
        assert np.array_equal(got.lookup_slots.cpu().numpy(), want.lookup_slots[:N]), "lookup_slots"


def assert_grouping_valid(got, want, ids, off):
    """The plan's optional grouping held to the contract the header gives a caller (tests/grouping.py); the slots
    it must carry are the oracle plan's."""
    grouping.check_grouping(ids, off, want.lookup_slots, got.grouped_lookups.cpu().numpy(), got.row_recs.cpu().numpy(),
                            got.keep_offsets, got.piece_recs.cpu().numpy(), got.piece_offsets)
    assert got.piece_offsets[0] == 0 and got.piece_offsets[-1] == got.piece_recs.shape[0]
    assert got.row_recs.shape[0] == got.keep_offsets[-1]


def plan_both(bp, ids, off, R, L, C):
    cfg = bp.make_config(R, C, 16, lookahead=L)
    got = bp.bp_oracle_plan(cfg, dev(ids), off, grouping=True)
    want = oracle.plan(ids, off, R, L, C)
    assert_plan_equal(got, want, len(ids))
    assert_grouping_valid(got, want, ids, off)
    plain = bp.bp_oracle_plan(cfg, dev(ids), off)                  # without the optional outputs: same plan
    assert_plan_equal(plain, want, len(ids))
    assert plain.grouped_lookups is None
    lean = bp.bp_oracle_plan(cfg, dev(ids), off, grouping=True, slot_map=False)   # grouping without the slot map
    assert lean.lookup_slots is None
    assert_plan_equal(lean, want, len(ids))
    assert_grouping_valid(lean, want, ids, off)
    return got, want


def test_plan_worked_example(bp):
    """Section 3.2's walk-through, on the GPU: lookahead 2, batches {3,9} {3,4} {3,6} {6,1}."""
    say("plan worked example")
    ids = np.array([3, 9, 3, 4, 3, 6, 6, 1], dtype=np.int64)
    off = np.array([0, 2, 4, 6, 8], dtype=np.int64)
    got, _ = plan_both(bp, ids, off, 16, 2, 8)
    assert got.prefetch_ids.cpu().tolist() == [3, 9, 4, 6, 1]
    assert got.prefetch_offsets.tolist() == [0, 2, 3, 4, 5]
    assert got.keep_ttl.cpu().tolist() == [1, 0, 2, 1, 2, 3, 3, 3]      # 0-based: 3->batch 2, then 3->batch 3, 6->batch 4
    assert got.evict_ids.cpu().tolist() == [9, 4, 3, 1, 6]


@pytest.mark.parametrize("seed", range(6))
def test_plan_random_small(bp, seed):
    say(f"plan random small seed={seed}")
    rng = np.random.default_rng(seed)
    R = int(rng.integers(5, 400))
    T = int(rng.integers(1, 40))
    lens = rng.integers(0, 300, size=T)                  # ragged batches, some empty
    lens[rng.integers(0, T)] = 0
    off = np.zeros(T + 1, dtype=np.int64)
    off[1:] = np.cumsum(lens)
    ids = np.minimum(rng.zipf(1.2, size=int(off[-1])) - 1, R - 1).astype(np.int64)
    if len(ids) == 0:
        return
    umax = max(len(np.unique(ids[off[i]:off[i + 1]])) for i in range(T))
    for L, C in ((1, umax), (3, umax), (T + 7, umax + 5), (T, 4 * R), (2, umax + 1), (0, umax + 5), (0, 2 * umax)):
        plan_both(bp, ids, off, R, L, max(1, C))          # L = 0: lookahead from the start-up rule


def test_plan_tiny_config(bp):
    say("plan tiny config, with and without capacity pressure")
    cfg = workloads.CONFIGS[0]
    tr = workloads.make_trace(cfg)
    got, want = plan_both(bp, tr.ids, tr.iter_offsets, cfg.total_rows, cfg.lookahead, cfg.capacity)
    assert got.L_eff == cfg.lookahead
    got, want = plan_both(bp, tr.ids, tr.iter_offsets, cfg.total_rows, cfg.lookahead, 1500)
    assert 1 <= got.L_eff < cfg.lookahead
    # slots wrap around the FIFO ring many times here
    assert len(want.prefetch_ids) > 5 * 1500


def test_plan_medium_multi_tile(bp):
    """~1.3 M lookups: several 4096-key sort tiles per digit, multi-tile scans, ragged tail; capacity binds."""
    say("plan medium")
    cfg = workloads.get_config(1, batch=1000, iterations=50, lookahead=40)
    tr = workloads.make_trace(cfg)
    uniq, uoff = oracle.unique_per_iter(tr.ids, tr.iter_offsets, cfg.total_rows)
    umax = int(np.diff(uoff).max())
    got, want = plan_both(bp, tr.ids, tr.iter_offsets, cfg.total_rows, 40, umax * 2)
    assert 1 < got.L_eff < 40
    plan_both(bp, tr.ids, tr.iter_offsets, cfg.total_rows, 40, umax)            # barely feasible: L_eff = 1
    plan_both(bp, tr.ids, tr.iter_offsets, cfg.total_rows, 60, 10 ** 6)         # lookahead beyond the trace


@pytest.mark.parametrize("largest", [1, 2, 255, 256, 257, 4096, 4097])
def test_plan_word_field_boundaries(bp, largest):
    """The place field of a lookup's word has as many bits as the largest batch needs: sizes at and around powers of
    two (and the sort tile), the largest batch first, last or in the middle, empty batches between, ids up to the
    top of the table."""
    say(f"plan with a largest batch of {largest} lookups")
    rng = np.random.default_rng(largest)
    R = (1 << 22) - 5
    for where in (0, 3, 6):
        lens = rng.integers(0, max(1, largest // 2) + 1, size=7)
        lens[where] = largest
        lens[(where + 2) % 7] = 0
        off = np.zeros(8, dtype=np.int64)
        off[1:] = np.cumsum(lens)
        pool = np.concatenate([rng.integers(0, R, size=40), [R - 1, 0, (1 << 21), (1 << 21) - 1]]).astype(np.int64)
        ids = pool[rng.integers(0, len(pool), size=int(off[-1]))]
        umax = max(len(np.unique(ids[off[i]:off[i + 1]])) for i in range(7))
        plan_both(bp, ids, off, R, 3, umax + 3)
        plan_both(bp, ids, off, R, 1, umax)


def test_plan_degenerate_traces(bp):
    """One id takes every lookup (one pair per batch, one row of many pieces per batch); every lookup has
    an id of its own (no reuse at all: nothing is ever kept); one lookup in the whole trace."""
    say("plan degenerate traces")
    off = np.array([0, 700, 700, 1500, 1501], dtype=np.int64)
    plan_both(bp, np.full(1501, 11, dtype=np.int64), off, 50, 3, 1)
    plan_both(bp, np.full(1501, 11, dtype=np.int64), off, 50, 1, 4)
    distinct = np.random.default_rng(5).permutation(5000)[:1501].astype(np.int64)
    plan_both(bp, distinct, off, 5000, 3, 800)
    plan_both(bp, distinct, off, 5000, 2, 2000)
    plan_both(bp, np.array([4], dtype=np.int64), np.array([0, 0, 1, 1], dtype=np.int64), 9, 2, 1)


def test_plan_many_batches_wide_group_keys(bp):
    """4,100 short batches (13 batch bits) with a capacity of 2^20 (wide slot and batch fields in the lookups' words),
    then with 9 slots: every slot changes hands hundreds of times, so the chains of the free ring are far longer than
    one launch of the chain walk follows."""
    say("plan with many batches: wide words, long slot chains")
    rng = np.random.default_rng(77)
    T, R = 4100, 300
    lens = rng.integers(0, 9, size=T)
    off = np.zeros(T + 1, dtype=np.int64)
    off[1:] = np.cumsum(lens)
    ids = np.minimum(rng.zipf(1.3, size=int(off[-1])) - 1, R - 1).astype(np.int64)
    plan_both(bp, ids, off, R, 50, 1 << 20)
    plan_both(bp, ids, off, R, 7, 9)                       # same trace, narrow keys, capacity binds
    # 300 batches: nine batch bits, which the regrouping sort takes in one pass of 512 digits; several sort tiles
    T = 300
    lens = rng.integers(0, 120, size=T)
    off = np.zeros(T + 1, dtype=np.int64)
    off[1:] = np.cumsum(lens)
    ids = np.minimum(rng.zipf(1.2, size=int(off[-1])) - 1, 4999).astype(np.int64)
    plan_both(bp, ids, off, 5000, 12, 1500)


def test_plan_errors(bp):
    say("plan errors")
    ids = np.array([0, 1, 2, 3, 0, 1], dtype=np.int64)
    off = np.array([0, 4, 6], dtype=np.int64)
    with pytest.raises(bp.BagpipeError) as e:
        bp.bp_oracle_plan(bp.make_config(10, 3, 16, lookahead=2), dev(ids), off)
    assert e.value.status == -2 and e.value.info["min_capacity"] == 4
    with pytest.raises(bp.BagpipeError) as e:
        bp.bp_oracle_plan(bp.make_config(3, 8, 16, lookahead=2), dev(ids), off)
    assert e.value.status == -4
    with pytest.raises(bp.BagpipeError) as e:
        bp.bp_oracle_plan(bp.make_config(10, 8, 16, lookahead=2), dev(ids), off, list_capacity=3)
    assert e.value.status == -3 and e.value.info["n_unique_pairs"] == 6
    # id bits + batch bits + bits of the largest batch beyond one 64-bit word: refused, nothing is launched
    big = np.arange(1 << 17, dtype=np.int64)
    with pytest.raises(bp.BagpipeError) as e:
        bp.bp_oracle_plan(bp.make_config(1 << 44, 1 << 18, 16, lookahead=2), dev(big),
                          np.concatenate([np.zeros(30, np.int64), [1 << 17]]))
    assert e.value.status == -6
    # an all-empty trace plans to nothing
    p = bp.bp_oracle_plan(bp.make_config(10, 8, 16, lookahead=2), torch.zeros(0, dtype=torch.int64, device="cuda"),
                          np.zeros(4, np.int64))
    assert p.L_eff == 2 and p.prefetch_offsets.tolist() == [0, 0, 0, 0]


# ---------------------------------------------------------------------------------------------------
# whole path
# ---------------------------------------------------------------------------------------------------
def run_end_to_end(cfg, trace, pinned=True, capacity=None, grouping=True, overlapped=False, reserve=0, slot_map=True):
    T = trace.iter_offsets.shape[0] - 1
    Wo, So, outs = helpers.oracle_uncached(cfg, trace)
    max_bag = cfg.bag_max

    def check(i, out):
        helpers.assert_outputs_close(out.cpu().numpy(), outs[i], max_bag, same_table=(i == 0))

    tr, plan, W, S = helpers.gpu_cached_training(cfg, trace, pinned=pinned, capacity=capacity, check_outputs=check,
                                                 grouping=grouping, overlapped=overlapped, reserve=reserve,
                                                 slot_map=slot_map)
    assert (plan.lookup_slots is None) == (not slot_map)
    C = cfg.capacity if capacity is None else capacity
    want_plan = oracle.plan(trace.ids, trace.iter_offsets, cfg.total_rows, cfg.lookahead, C, reserve=reserve)
    assert_plan_equal(plan, want_plan, trace.n_lookups)
    got = helpers.table_from_torch(cfg, W)
    if cfg.weight_dtype == "bf16":
        assert np.array_equal(got, Wo), "bf16 codes of the final table must match bit for bit"
    else:
        worst = helpers.assert_weights_close(got, Wo)
        say(f"  worst weight error {worst:.3g} of the 1e-4 bound")
    if So.size:
        np.testing.assert_allclose(S.cpu().numpy(), So, rtol=1e-4, atol=1e-9)
    # the cache drains: every resident row was written back
    assert plan.prefetch_offsets[-1] == plan.evict_offsets[-1]
    tr.close()
    return plan


def test_end_to_end_tiny_config(bp):
    """configs[0] as written: 8 x 10,000 rows, D=16, batch 256, 50 iterations, L=20, cache 4,096, SGD."""
    say("end to end: tiny config")
    cfg = workloads.CONFIGS[0]
    plan = run_end_to_end(cfg, workloads.make_trace(cfg))
    assert plan.L_eff == 20
    plan = run_end_to_end(cfg, workloads.make_trace(cfg), grouping=False)       # backward sorts the slots itself
    assert plan.L_eff == 20
    plan = run_end_to_end(cfg, workloads.make_trace(cfg), slot_map=False)       # no slot per lookup: both passes walk
    assert plan.L_eff == 20                                                     # the row records
    run_end_to_end(cfg, workloads.make_trace(cfg), slot_map=False, overlapped=True, reserve=1200)


@pytest.mark.parametrize("grouping", [True, False])
@pytest.mark.parametrize("optimizer,dtype,bag_max,capacity,pinned", [
    ("adagrad", "f32", 1, 1400, True), ("adagrad_rowwise", "bf16", 1, 4096, True), ("sgd", "f32", 6, 3000, False),
    ("adagrad", "bf16", 4, 2600, True)])
def test_end_to_end_variants(bp, optimizer, dtype, bag_max, capacity, pinned, grouping):
    say(f"end to end: {optimizer} {dtype} bag_max={bag_max} C={capacity} grouping={grouping}")
    cfg = workloads.get_config(0, optimizer=optimizer, weight_dtype=dtype, bag_max=bag_max, capacity=capacity,
                               batch=128 if bag_max > 1 else 256, iterations=30)
    run_end_to_end(cfg, workloads.make_trace(cfg), pinned=pinned, grouping=grouping)


# ---------------------------------------------------------------------------------------------------
# cache maintenance overlapped with training (bp_pipeline_*)
# ---------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("optimizer,dtype,bag_max,capacity,reserve,lookahead,pinned", [
    ("adagrad", "f32", 1, 4096, 1200, 20, True),          # roomy: every prefetch is early
    ("adagrad", "f32", 1, 1400, 0, 20, True),             # capacity binds, no reserve: most prefetches are late
    ("adagrad_rowwise", "bf16", 1, 2400, 700, 20, True),
    ("sgd", "f32", 6, 3000, 600, 20, False),
    ("adagrad", "bf16", 4, 2600, 0, 2, True),             # L_eff == 2: write-back and early fetch take turns
    ("sgd", "f32", 1, 1400, 0, 1, True),                  # L_eff == 1: the synchronous order on the other stream
    # nearly uniform ids, a reserve of ~1.4 batches of misses: no late prefetches, and most early prefetches take the
    # slots of the evictions of two batches before (the one-launch step without staging, with its pairs)
    ("adagrad", "f32", 1, 8000, 2000, 40, True), ("adagrad_rowwise", "bf16", 1, 8000, 2000, 40, False),
    ("sgd", "f32", 1, 9000, 2300, 40, True)])
def test_end_to_end_overlapped(bp, optimizer, dtype, bag_max, capacity, reserve, lookahead, pinned):
    """Same trace, same oracle, maintenance on the library's own stream: outputs and final table as before."""
    say(f"overlapped: {optimizer} {dtype} bag_max={bag_max} C={capacity} reserve={reserve} L={lookahead}")
    uniform = capacity >= 8000
    cfg = workloads.get_config(0, optimizer=optimizer, weight_dtype=dtype, bag_max=bag_max, capacity=capacity,
                               batch=128 if bag_max > 1 else 256, iterations=30, lookahead=lookahead,
                               zipf_s=(0.05 if capacity == 8000 else 0.3) if uniform else 1.2)
    plan = run_end_to_end(cfg, workloads.make_trace(cfg), pinned=pinned, overlapped=True, reserve=reserve)
    early = bp.bp_pipeline_early_counts(plan.prefetch_offsets, plan.evict_offsets, capacity, plan.L_eff)
    misses = np.diff(plan.prefetch_offsets)
    say(f"  L_eff={plan.L_eff} early {int(early[1:].sum())} of {int(misses[1:].sum())} prefetches after batch 0")
    if uniform:     # the case is meant to hand slots over two batches on: make sure it does
        paired = 0
        for i in range(len(misses) - 2):
            if misses[i + 1] == early[i + 1]:
                free = min(max(capacity + int(plan.evict_offsets[i]) - int(plan.prefetch_offsets[i + 2]), 0), int(early[i + 2]))
                paired += int(early[i + 2]) - free
        say(f"  {paired} prefetches take the slot of a row written back in the same launch")
        assert plan.L_eff >= 3 and paired > 500
    if plan.L_eff == 1:
        assert early.sum() == 0
    if reserve >= misses.max():
        assert np.array_equal(early[1:], misses[1:])


def test_plan_without_configured_lookahead(bp):
    """lookahead = 0: the start-up rule of Section 4 (batches prefetched until the cache is full) gives the lookahead,
    the capacity policy may lower it; same plan as the oracle's."""
    say("plan without a configured lookahead")
    cfg = workloads.get_config(0, iterations=40)
    tr = workloads.make_trace(cfg)
    uniq, uoff = oracle.unique_per_iter(tr.ids, tr.iter_offsets, cfg.total_rows)
    for C, reserve in ((1400, 0), (2500, 300), (4096, 0), (200_000, 0)):
        want_L = oracle.auto_lookahead(uniq, uoff, cfg.total_rows, C - reserve)
        want = oracle.plan(tr.ids, tr.iter_offsets, cfg.total_rows, 0, C, reserve=reserve)
        got = bp.bp_oracle_plan(bp.make_config(cfg.total_rows, C, 16, lookahead=0, reserve=reserve), dev(tr.ids),
                                tr.iter_offsets, grouping=True)
        assert got.L_requested == want_L
        assert_plan_equal(got, want, len(tr.ids))
        assert_grouping_valid(got, want, tr.ids, tr.iter_offsets)
        say(f"  C={C} reserve={reserve}: start-up rule {want_L}, L_eff {got.L_eff}")
    with pytest.raises(bp.BagpipeError) as e:            # the first batch alone does not fit
        bp.bp_oracle_plan(bp.make_config(cfg.total_rows, 900, 16, lookahead=0), dev(tr.ids), tr.iter_offsets)
    assert e.value.status == -2


def test_plan_with_reserve(bp):
    """The capacity policy with reserved slots: L_eff as for a cache of capacity - reserve, slots from all of it."""
    say("plan with reserve")
    cfg = workloads.get_config(0, iterations=40)
    tr = workloads.make_trace(cfg)
    for C, reserve in ((4096, 0), (4096, 1500), (2500, 800), (2500, 2499 - 1400)):
        bc = bp.make_config(cfg.total_rows, C, 16, lookahead=cfg.lookahead, reserve=reserve)
        try:
            want = oracle.plan(tr.ids, tr.iter_offsets, cfg.total_rows, cfg.lookahead, C, reserve=reserve)
        except oracle.OracleError:
            with pytest.raises(bp.BagpipeError) as e:
                bp.bp_oracle_plan(bc, dev(tr.ids), tr.iter_offsets)
            assert e.value.status == -2
            continue
        got = bp.bp_oracle_plan(bc, dev(tr.ids), tr.iter_offsets, grouping=True)
        assert_plan_equal(got, want, len(tr.ids))
        assert_grouping_valid(got, want, tr.ids, tr.iter_offsets)
        assert got.peak_occupancy <= C - reserve


@pytest.mark.parametrize("skew", [0.01, 0.4, 0.9])
def test_end_to_end_skew_workload(bp, skew):
    """The skew-sensitivity workload of Section 5.3 (hot 1 % with an exponential law, uniform tail), small."""
    say(f"end to end: skew workload {skew}")
    cfg = workloads.skew_config(0, skew, optimizer="adagrad", capacity=6000, iterations=30)
    run_end_to_end(cfg, workloads.make_trace(cfg))
    run_end_to_end(cfg, workloads.make_trace(cfg), overlapped=True, reserve=1500)


# ---------------------------------------------------------------------------------------------------
# planning a stream chunk by chunk (bp_oracle_plan_chunk)
# ---------------------------------------------------------------------------------------------------
def run_chunked(bp, ids, off, R, L, C, n_emit, reserve=0):
    """Plans the stream n_emit batches at a time through the C ABI, each call seeing L - 1 batches beyond its chunk,
    and compares every emitted batch and every carried state with the oracle's chunk-by-chunk plan."""
    want, L_of = oracle.plan_chunked(ids, off, R, L, C, n_emit, reserve)
    T = len(off) - 1
    cfg = bp.make_config(R, C, 16, lookahead=L, reserve=reserve)
    state = None
    for a in range(0, T, n_emit):
        b = min(T, a + n_emit)
        hi = min(T, b + L - 1)
        sub_off = (off[a:hi + 1] - off[a]).astype(np.int64)
        sub_ids = ids[off[a]:off[hi]]
        got, state = bp.bp_oracle_plan_chunk(cfg, dev(sub_ids), sub_off, b - a, state, grouping=True)
        assert got.L_eff == L_of[a], (a, got.L_eff, L_of[a])
        assert np.array_equal(got.occupancy, want.occ[a:b])
        for k in range(b - a):
            i = a + k
            for name, oname in (("prefetch", "prefetch"), ("evict", "evict")):
                g0, g1 = getattr(got, name + "_offsets")[k], getattr(got, name + "_offsets")[k + 1]
                w0, w1 = getattr(want, oname + "_off")[i], getattr(want, oname + "_off")[i + 1]
                assert np.array_equal(getattr(got, name + "_ids")[g0:g1].cpu().numpy(), getattr(want, oname + "_ids")[w0:w1]), (name, i)
                assert np.array_equal(getattr(got, name + "_slots")[g0:g1].cpu().numpy(), getattr(want, oname + "_slots")[w0:w1]), (name, i)
            g0, g1 = got.keep_offsets[k], got.keep_offsets[k + 1]
            w0, w1 = want.keep_off[i], want.keep_off[i + 1]
            assert np.array_equal(got.keep_ids[g0:g1].cpu().numpy(), want.keep_ids[w0:w1])
            assert np.array_equal(got.keep_ttl[g0:g1].cpu().numpy() + a, want.keep_ttl[w0:w1])
        n_em = int(off[b] - off[a])
        assert np.array_equal(got.lookup_slots[:n_em].cpu().numpy(), want.lookup_slots[off[a]:off[b]])
        if n_em:
            grouping.check_grouping(sub_ids, sub_off, want.lookup_slots[off[a]:off[b]],
                                    got.grouped_lookups[:n_em].cpu().numpy(), got.row_recs.cpu().numpy(),
                                    got.keep_offsets, got.piece_recs.cpu().numpy(), got.piece_offsets, n_batches=b - a)
        # carried state: replay the oracle's lists up to batch b - 1
        held = {}
        free = list(range(C))
        for i in range(b):
            for g, s in zip(want.prefetch_ids[want.prefetch_off[i]:want.prefetch_off[i + 1]].tolist(),
                            want.prefetch_slots[want.prefetch_off[i]:want.prefetch_off[i + 1]].tolist()):
                assert free.pop(0) == s
                held[g] = s
            for g, s in zip(want.evict_ids[want.evict_off[i]:want.evict_off[i + 1]].tolist(),
                            want.evict_slots[want.evict_off[i]:want.evict_off[i + 1]].tolist()):
                assert held.pop(g) == s
                free.append(s)
        n = state.n_resident
        assert n == len(held)
        assert state.resident_ids[:n].cpu().tolist() == sorted(held)
        assert state.ring[:n].cpu().tolist() == [held[g] for g in sorted(held)]
        assert state.ring[n:].cpu().tolist() == free
    return want, L_of


@pytest.mark.parametrize("seed", range(4))
def test_plan_chunked_random(bp, seed):
    say(f"plan chunked random seed={seed}")
    rng = np.random.default_rng(500 + seed)
    R = int(rng.integers(20, 300))
    T = int(rng.integers(4, 30))
    lens = rng.integers(0, 200, size=T)
    lens[rng.integers(0, T)] = 0
    off = np.zeros(T + 1, dtype=np.int64)
    off[1:] = np.cumsum(lens)
    ids = np.minimum(rng.zipf(1.25, size=int(off[-1])) - 1, R - 1).astype(np.int64)
    umax = max(len(np.unique(ids[off[i]:off[i + 1]])) for i in range(T))
    for L, C, n_emit in ((4, 4 * R, 3), (4, 4 * R, 1), (1, 4 * R, 5), (2, 4 * R, 2), (T + 3, 4 * R, 4), (6, 4 * R, T)):
        want, L_of = run_chunked(bp, ids, off, R, L, C, n_emit)
        assert (L_of == L).all()
        # same lookahead everywhere: the chunks together are the whole-trace plan
        whole = oracle.plan(ids, off, R, L, C, L_eff=L)
        assert np.array_equal(want.lookup_slots, whole.lookup_slots) and np.array_equal(want.evict_slots, whole.evict_slots)
    # capacity binds: chunks get different lookaheads; a stream whose batches fit one by one can always be planned
    for L, C, n_emit in ((5, umax, 3), (6, umax + 2, 1), (8, umax + 10, 4), (5, umax + 6, 3)):
        want, L_of = run_chunked(bp, ids, off, R, L, C, n_emit)
        say(f"  L={L} C={C} chunks of {n_emit}: lookaheads {sorted(set(L_of.tolist()))}")
    with pytest.raises(bp.BagpipeError) as e:
        bp.bp_oracle_plan_chunk(bp.make_config(R, umax - 1, 16, lookahead=3), dev(ids), off, T)
    assert e.value.status == -2


def test_plan_chunked_medium(bp):
    """~0.6 M lookups, 50 batches in chunks of 10 with a lookahead of 8: multi-tile sorts and scans in chunk mode."""
    say("plan chunked medium")
    cfg = workloads.get_config(1, batch=500, iterations=50, lookahead=8)
    tr = workloads.make_trace(cfg)
    R = cfg.total_rows
    whole = oracle.plan(tr.ids, tr.iter_offsets, R, 8, 10 ** 6, L_eff=8)
    c = bp.make_config(R, 10 ** 6, 16, lookahead=8)
    state, off = None, tr.iter_offsets
    for a in range(0, 50, 10):
        b, hi = a + 10, min(50, a + 10 + 7)
        got, state = bp.bp_oracle_plan_chunk(c, dev(tr.ids[off[a]:off[hi]]), off[a:hi + 1] - off[a], 10, state, grouping=True)
        assert got.L_eff == 8
        n_em = int(off[b] - off[a])
        assert np.array_equal(got.lookup_slots[:n_em].cpu().numpy(), whole.lookup_slots[off[a]:off[b]])
        g0, g1 = got.prefetch_offsets[0], got.prefetch_offsets[-1]
        assert np.array_equal(got.prefetch_ids[g0:g1].cpu().numpy(), whole.prefetch_ids[whole.prefetch_off[a]:whole.prefetch_off[b]])
        assert np.array_equal(got.prefetch_slots[g0:g1].cpu().numpy(), whole.prefetch_slots[whole.prefetch_off[a]:whole.prefetch_off[b]])
        g0, g1 = got.evict_offsets[0], got.evict_offsets[-1]
        assert np.array_equal(got.evict_slots[g0:g1].cpu().numpy(), whole.evict_slots[whole.evict_off[a]:whole.evict_off[b]])
        assert state.n_resident == whole.prefetch_off[b] - whole.evict_off[b]


@pytest.mark.parametrize("optimizer,dtype,bag_max,capacity,lookahead,n_emit", [
    ("adagrad", "f32", 1, 4096, 6, 7), ("sgd", "f32", 5, 2200, 8, 4), ("adagrad_rowwise", "bf16", 1, 1300, 5, 1),
    ("adagrad", "bf16", 3, 3000, 1, 6),
    ("adagrad", "f32", 1, 1500, 20, 3), ("sgd", "f32", 1, 1450, 20, 1)])      # the capacity binds: lookaheads differ
def test_end_to_end_streaming(bp, optimizer, dtype, bag_max, capacity, lookahead, n_emit):
    """The trace planned chunk by chunk while it is trained on: same outputs and final table as the uncached oracle."""
    say(f"streaming: {optimizer} {dtype} bag_max={bag_max} C={capacity} L={lookahead} chunks of {n_emit}")
    from paper_2202_12429_amd.runner import CachedEmbeddingTrainer
    cfg = workloads.get_config(0, optimizer=optimizer, weight_dtype=dtype, bag_max=bag_max, capacity=capacity,
                               batch=128 if bag_max > 1 else 256, iterations=30, lookahead=lookahead)
    trace = workloads.make_trace(cfg)
    Wo, So, outs = helpers.oracle_uncached(cfg, trace)
    W, S = helpers.make_backing(cfg, True)
    tr = CachedEmbeddingTrainer(helpers.bp_config_of(cfg), W, S)
    T, off, bags = cfg.iterations, trace.iter_offsets, cfg.bags
    seen = []
    for a in range(0, T, n_emit):
        b, hi = min(T, a + n_emit), min(T, a + n_emit + lookahead - 1)
        plan = tr.plan_chunk(dev(trace.ids[off[a]:off[hi]]), off[a:hi + 1] - off[a], b - a)
        seen.append(plan.L_eff)
        for k in range(b - a):
            i = a + k
            bo = None if cfg.one_hot else dev(np.ascontiguousarray(trace.bag_offsets[i]))
            tr.maintain(k)
            out = tr.forward(k, bo, bags)
            helpers.assert_outputs_close(out.cpu().numpy(), outs[i], cfg.bag_max, same_table=(i == 0))
            tr.backward_update(k, bo, bags, workloads.upstream_grad(cfg, i, bags, device="cuda:0"))
    tr.flush()
    torch.cuda.synchronize()
    say(f"  lookaheads of the chunks: {sorted(set(seen))}")
    got = helpers.table_from_torch(cfg, W)
    if dtype == "bf16":
        assert np.array_equal(got, Wo)
    else:
        helpers.assert_weights_close(got, Wo)
    if So.size:
        np.testing.assert_allclose(S.cpu().numpy(), So, rtol=1e-4, atol=1e-9)


# ---------------------------------------------------------------------------------------------------
# HIP graph capture of a step
# ---------------------------------------------------------------------------------------------------
def test_step_captured_in_a_graph(bp):
    """cache maintenance + forward + grouped backward of one batch recorded into a HIP graph (the entry points only
    launch kernels on the given stream: no allocation, no memset, no synchronisation) and replayed three times with
    eager work and synchronisations in between: bit for bit what three eager runs of the same step give."""
    say("one step captured in a HIP graph")
    from paper_2202_12429_amd.runner import CachedEmbeddingTrainer
    cfg = workloads.get_config(0, optimizer="adagrad", iterations=6, capacity=3000)
    trace = workloads.make_trace(cfg)
    bags, k = cfg.bags, 3

    def fresh():
        W, S = helpers.make_backing(cfg, pinned=False)
        tr = CachedEmbeddingTrainer(helpers.bp_config_of(cfg), W, S, max_lookups=bags, max_bags=bags)
        tr.plan(dev(trace.ids), trace.iter_offsets)
        for i in range(k):                                   # bring the cache to the state before batch k
            tr.maintain(i)
            tr.forward(i, None, bags)
            tr.backward_update(i, None, bags, workloads.upstream_grad(cfg, i, bags, device="cuda:0"))
        torch.cuda.synchronize()
        return tr, W, S

    grad = workloads.upstream_grad(cfg, k, bags, device="cuda:0")
    out = torch.empty((bags, cfg.dim), dtype=torch.float32, device="cuda")

    def step(tr):
        tr.maintain(k)
        tr.forward(k, None, bags, out=out)
        tr.backward_update(k, None, bags, grad)

    tr, W, S = fresh()
    outs_eager = []
    for _ in range(3):
        step(tr)
        outs_eager.append(out.clone())
    torch.cuda.synchronize()
    want_w, want_s = tr.cache_w.clone(), tr.cache_state.clone()

    tr, W, S = fresh()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                            # warm-up on the capture stream, then undo it
        pass
    graph = torch.cuda.CUDAGraph()
    w0, s0 = tr.cache_w.clone(), tr.cache_state.clone()
    with torch.cuda.graph(graph):
        step(tr)
    tr.cache_w.copy_(w0)
    tr.cache_state.copy_(s0)
    scratch = torch.zeros(1 << 20, device="cuda")
    for r in range(3):
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, outs_eager[r]), f"replay {r}: pooled output differs from the eager run"
        scratch.add_(1.0)                                    # eager work between the replays
        assert float(scratch.sum()) == (r + 1) * scratch.numel()
    assert torch.equal(tr.cache_w, want_w) and torch.equal(tr.cache_state, want_s)


# ---------------------------------------------------------------------------------------------------
# which logical trainer uses a row
# ---------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("seed", range(3))
def test_plan_trainer_marking(bp, seed):
    """keep_owner of every (id, batch): the single trainer that looks the id up, or -1 / -2 for rows several trainers
    share (deferred / needed by the next batch), for lookups dealt to P trainers by position."""
    say(f"plan trainer marking seed={seed}")
    rng = np.random.default_rng(700 + seed)
    R, T = int(rng.integers(30, 500)), int(rng.integers(2, 25))
    lens = rng.integers(0, 400, size=T)
    off = np.zeros(T + 1, dtype=np.int64)
    off[1:] = np.cumsum(lens)
    ids = np.minimum(rng.zipf(1.2, size=int(off[-1])) - 1, R - 1).astype(np.int64)
    for P in (1, 2, 8, 64):
        even = np.stack([np.floor(np.arange(P + 1) * n / P) for n in lens]).astype(np.int64)        # equal shares
        ragged = np.stack([np.concatenate([[0], np.sort(rng.integers(0, n + 1, size=P - 1)), [n]]) for n in lens]).astype(np.int64)
        for cuts in (even, ragged):
            got = bp.bp_oracle_plan(bp.make_config(R, 4 * R, 16, lookahead=5), dev(ids), off, trainer_cuts=cuts)
            want = oracle.keep_owners(ids, off, R, cuts)
            assert np.array_equal(got.keep_owner.cpu().numpy(), want)
            if P == 1:
                assert (want == 0).all()
    with pytest.raises(bp.BagpipeError):                                # cuts that do not end at the batch's size
        bad = even.copy()
        bad[0, -1] += 1
        bp.bp_oracle_plan(bp.make_config(R, 4 * R, 16, lookahead=5), dev(ids), off, trainer_cuts=bad)


@pytest.mark.parametrize("row_ints,n,u", [(48, 1000, 4), (16, 4097, 1), (4, 3, 8), (256, 77, 2), (64, 999, 8)])
def test_gather_calibration(bp, row_ints, n, u):
    """The row-gather yardstick folds exactly the rows it is given (so it reads them), u rows per lane group."""
    rng = np.random.default_rng(row_ints + n)
    table = rng.integers(-2**31, 2**31, size=(500, row_ints), dtype=np.int64).astype(np.int32)
    rows = rng.integers(0, 500, size=n).astype(np.int32)
    rows[0] = 499
    sink = bp.bp_gather_calibration(torch.from_numpy(table).cuda(), torch.from_numpy(rows).cuda(), rows_in_flight=u)
    torch.cuda.synchronize()
    got = sink.cpu().numpy().reshape(-1, 4)
    for k in range(-(-n // u)):
        sel = table[rows[u * k:u * k + u]].reshape(-1, 4)
        assert np.array_equal(got[k], np.bitwise_xor.reduce(sel, axis=0)), k
    with pytest.raises(bp.BagpipeError):
        bp.bp_gather_calibration(torch.from_numpy(table).cuda(), torch.from_numpy(rows).cuda(), rows_in_flight=3)


@pytest.mark.parametrize("row_ints,n,u", [(48, 1000, 4), (16, 4097, 1), (4, 3, 2), (256, 77, 2), (64, 999, 4)])
def test_scatter_calibration(bp, row_ints, n, u):
    """The row-scatter yardstick writes exactly the rows it is given, every 16-byte piece of them, and nothing else."""
    rng = np.random.default_rng(row_ints * n)
    R = 5000
    rows = rng.permutation(R)[:n].astype(np.int32)
    rows[n // 2] = R + 7                                                 # out of range: skipped
    before = rng.integers(0, 1000, size=(R, row_ints)).astype(np.int32)
    table = torch.from_numpy(before.copy()).cuda()
    bp.bp_scatter_calibration(table, torch.from_numpy(rows).cuda(), rows_in_flight=u)
    torch.cuda.synchronize()
    got = table.cpu().numpy()
    want = before.copy().reshape(R, row_ints // 4, 4)
    for k, r in enumerate(rows):
        if r < R:
            want[r, :, 0] = r
            want[r, :, 1] = np.arange(row_ints // 4)
            want[r, :, 2] = k
            want[r, :, 3] = 0x5ca77e25
    assert np.array_equal(got, want.reshape(R, row_ints))
    with pytest.raises(bp.BagpipeError):
        bp.bp_scatter_calibration(table, torch.from_numpy(rows).cuda(), rows_in_flight=8)


def test_profiler_totals_and_spread(bp):
    """The event profiler: launches are counted per kernel, totals add up, the spread brackets the mean, a selection
    restricts what is recorded, and nothing is recorded once it is switched off."""
    say("profiler")
    a = torch.rand(1 << 20, device="cuda")
    b = torch.empty_like(a)
    bp.bp_profile_select(None)
    bp.bp_profile_enable(True)
    for _ in range(7):
        bp.bp_copy_calibration(b, a)
    bp.bp_profile_collect()
    tot = bp.profile_totals()
    assert tot["copy_calibration"][0] == 7 and tot["copy_calibration"][1] > 0
    lo, med, hi = bp.profile_spread("copy_calibration")
    assert 0 < lo <= med <= hi and lo <= tot["copy_calibration"][1] / 7 <= hi
    bp.bp_profile_enable(True)                       # clears
    bp.bp_profile_select(["embbag_fwd"])
    bp.bp_copy_calibration(b, a)
    bp.bp_profile_collect()
    assert "copy_calibration" not in bp.profile_totals()
    with pytest.raises(bp.BagpipeError):
        bp.profile_spread("copy_calibration")
    bp.bp_profile_select(None)
    bp.bp_profile_enable(False)
    bp.bp_copy_calibration(b, a)
    bp.bp_profile_collect()
    assert "copy_calibration" not in bp.profile_totals()
    assert torch.equal(a, b)
