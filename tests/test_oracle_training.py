"""Pins for the oracle's training arithmetic (oracle parts B and C): torch CPU library routines
(embedding_bag, optim.SGD, optim.Adagrad with sparse gradients), closed forms on one row, the bf16 rounding
rule, and the paper's consistency claim (cached training == uncached synchronous training, bit for bit)."""
import numpy as np
import pytest
import torch

import oracle
import workloads


def rand_problem(seed, rows=50, D=8, bags=40, max_len=5, allow_empty=True):
    rng = np.random.default_rng(seed)
    lens = rng.integers(0 if allow_empty else 1, max_len + 1, size=bags)
    off = np.zeros(bags + 1, dtype=np.int64)
    off[1:] = np.cumsum(lens)
    idx = np.minimum(rng.zipf(1.4, size=int(off[-1])) - 1, rows - 1).astype(np.int64)
    W = rng.uniform(-0.05, 0.05, size=(rows, D)).astype(np.float32)
    return W, idx, off, rng


def torch_bag(W64, idx, off, sparse=True):
    emb = torch.nn.EmbeddingBag.from_pretrained(torch.from_numpy(W64.copy()), mode="sum", sparse=sparse,
                                                freeze=False, include_last_offset=True)
    return emb


def test_forward_matches_torch_embedding_bag():
    W, idx, off, _ = rand_problem(0)
    out = oracle.train_iter(W, None, 8, oracle.F32, oracle.SGD, 0.0, 0.0, idx, off, None)
    ref = torch.nn.functional.embedding_bag(torch.from_numpy(idx), torch.from_numpy(W).double(),
                                            torch.from_numpy(off), mode="sum", include_last_offset=True)
    assert np.array_equal(out, ref.float().numpy())
    # an empty bag gives a zero row
    lens = np.diff(off)
    assert (lens == 0).any() and not out[lens == 0].any()
    # one-hot: the output row is a bit-exact copy of the table row
    assert len(idx) >= 40
    out1 = oracle.train_iter(W, None, 8, oracle.F32, oracle.SGD, 0.0, 0.0, idx[:40], np.arange(41), None)
    assert np.array_equal(out1, W[idx[:40]])


@pytest.mark.parametrize("opt_name", ["sgd", "adagrad"])
def test_update_matches_torch_sparse_optimizers(opt_name):
    """Five iterations with duplicate rows inside and across bags; torch runs in fp64 on the full table, the
    oracle stores fp32 and computes in fp64, so they agree to fp32 rounding of the stored values."""
    D, rows = 8, 50
    W, _, _, rng = rand_problem(1, rows=rows, D=D)
    lr, eps = 0.01, 1e-8
    emb = torch_bag(W.astype(np.float64), None, None)
    if opt_name == "sgd":
        opt = torch.optim.SGD(emb.parameters(), lr=lr)
        S, code = None, oracle.SGD
    else:
        opt = torch.optim.Adagrad(emb.parameters(), lr=lr, eps=eps, initial_accumulator_value=0.0, lr_decay=0.0)
        S, code = np.zeros((rows, D), dtype=np.float32), oracle.ADAGRAD
    Wo = W.copy()
    for it in range(5):
        _, idx, off, r2 = rand_problem(100 + it, rows=rows, D=D)
        g = r2.standard_normal((len(off) - 1, D)).astype(np.float32)
        out = oracle.train_iter(Wo, S, D, oracle.F32, code, lr, eps, idx, off, g)
        opt.zero_grad()
        o = emb(torch.from_numpy(idx), torch.from_numpy(off))
        np.testing.assert_allclose(out, o.detach().numpy(), rtol=2e-6, atol=1e-7)
        o.backward(torch.from_numpy(g).double())
        opt.step()
    np.testing.assert_allclose(Wo, emb.weight.detach().numpy(), rtol=1e-5, atol=1e-7)
    if S is not None:
        st = opt.state[emb.weight]["sum"].numpy()
        np.testing.assert_allclose(S, st, rtol=1e-5, atol=1e-9)
    assert np.abs(Wo - W).max() > 1e-3            # the update did something


def test_sgd_closed_form_one_row_duplicates():
    """w_T = w_0 - lr * sum of all gradients that hit the row (duplicates inside an iteration add up)."""
    D = 4
    W = np.array([[0.01, -0.02, 0.03, 0.04], [1, 1, 1, 1]], dtype=np.float32)
    g = np.array([[1, 2, 3, 4], [10, 20, 30, 40], [0.5, 0.5, 0.5, 0.5]], dtype=np.float32)
    idx = np.array([0, 0, 0], dtype=np.int64)          # bag0 = {0,0}, bag1 = {0}, bag2 = {}
    off = np.array([0, 2, 3, 3], dtype=np.int64)
    out = oracle.train_iter(W, None, D, oracle.F32, oracle.SGD, 0.5, 0.0, idx, off, g)
    assert np.array_equal(out[0], np.float32(2) * np.array([0.01, -0.02, 0.03, 0.04], dtype=np.float32))
    assert not out[2].any()
    G = 2 * g[0].astype(np.float64) + g[1]
    want = (np.array([0.01, -0.02, 0.03, 0.04], dtype=np.float32).astype(np.float64) - 0.5 * G).astype(np.float32)
    assert np.array_equal(W[0], want)
    assert np.array_equal(W[1], np.ones(4, dtype=np.float32))        # untouched row


def test_adagrad_coalesces_before_squaring():
    """Two lookups of one row with gradients a and b: state grows by (a+b)^2, not a^2+b^2."""
    W = np.zeros((1, 1), dtype=np.float32)
    S = np.zeros((1, 1), dtype=np.float32)
    g = np.array([[3.0], [4.0]], dtype=np.float32)
    oracle.train_iter(W, S, 1, oracle.F32, oracle.ADAGRAD, 0.1, 0.0, np.array([0, 0]), np.array([0, 1, 2]), g)
    assert S[0, 0] == 49.0
    assert W[0, 0] == -np.float32(0.1)


def test_rowwise_adagrad_closed_form_and_d1_equivalence():
    D = 4
    W = np.full((2, D), 0.5, dtype=np.float32)
    S = np.zeros(2, dtype=np.float32)
    g = np.array([[1, 2, 3, 4]], dtype=np.float32)
    oracle.train_iter(W, S, D, oracle.F32, oracle.ADAGRAD_ROWWISE, 0.1, 1e-8, np.array([1]), np.array([0, 1]), g)
    assert S[0] == 0 and S[1] == np.float32(30.0 / 4.0)
    lr = np.float64(np.float32(0.1))                       # lr and eps reach the oracle as fp32 values
    want = 0.5 - lr * g[0].astype(np.float64) / (np.sqrt(np.float64(7.5)) + np.float64(np.float32(1e-8)))
    assert np.array_equal(W[1], want.astype(np.float32))
    assert np.array_equal(W[0], np.full(D, 0.5, dtype=np.float32))
    # D = 1: row-wise and element-wise are the same rule
    rng = np.random.default_rng(5)
    Wa = rng.uniform(-1, 1, (20, 1)).astype(np.float32)
    Wb = Wa.copy()
    Sa = np.zeros((20, 1), dtype=np.float32)
    Sb = np.zeros(20, dtype=np.float32)
    for it in range(4):
        idx = rng.integers(0, 20, size=30)
        off = np.arange(31, dtype=np.int64)
        gg = rng.standard_normal((30, 1)).astype(np.float32)
        oracle.train_iter(Wa, Sa, 1, oracle.F32, oracle.ADAGRAD, 0.05, 1e-8, idx, off, gg)
        oracle.train_iter(Wb, Sb, 1, oracle.F32, oracle.ADAGRAD_ROWWISE, 0.05, 1e-8, idx, off, gg)
    assert np.array_equal(Wa, Wb) and np.array_equal(Sa[:, 0], Sb)


def test_rowwise_adagrad_equals_torch_adagrad_on_constant_rows():
    """When every upstream gradient row is constant along the embedding dimension, so is every summed row gradient:
    the mean of its squares is the square of each element, the row's one state value equals every element's state,
    and row-wise Adagrad is torch.optim.Adagrad.  Several iterations, duplicates inside and across bags, multi-hot."""
    D, rows = 8, 40
    W, _, _, rng = rand_problem(7, rows=rows, D=D)
    lr, eps = 0.02, 1e-8
    emb = torch_bag(W.astype(np.float64), None, None)
    opt = torch.optim.Adagrad(emb.parameters(), lr=lr, eps=eps, initial_accumulator_value=0.0, lr_decay=0.0)
    Wo, S = W.copy(), np.zeros(rows, dtype=np.float32)
    for it in range(6):
        _, idx, off, r2 = rand_problem(200 + it, rows=rows, D=D)
        g = np.repeat(r2.standard_normal((len(off) - 1, 1)).astype(np.float32), D, axis=1)
        oracle.train_iter(Wo, S, D, oracle.F32, oracle.ADAGRAD_ROWWISE, lr, eps, idx, off, g)
        opt.zero_grad()
        emb(torch.from_numpy(idx), torch.from_numpy(off)).backward(torch.from_numpy(g).double())
        opt.step()
    np.testing.assert_allclose(Wo, emb.weight.detach().numpy(), rtol=1e-5, atol=1e-7)
    st = opt.state[emb.weight]["sum"].numpy()
    np.testing.assert_allclose(S, st[:, 0], rtol=1e-5, atol=1e-9)
    assert np.allclose(st, st[:, :1])                       # torch's state is indeed constant along a row
    assert np.abs(Wo - W).max() > 1e-3


def test_bf16_storage_rounds_to_nearest_even():
    rng = np.random.default_rng(3)
    w32 = rng.uniform(-0.05, 0.05, size=(64, 8)).astype(np.float32)
    wb = torch.from_numpy(w32).to(torch.bfloat16)
    table = wb.view(torch.int16).numpy().view(np.uint16).copy()
    g = rng.standard_normal((64, 8)).astype(np.float32)
    idx = np.arange(64, dtype=np.int64)
    off = np.arange(65, dtype=np.int64)
    out = oracle.train_iter(table, None, 8, oracle.BF16, oracle.SGD, 0.01, 0.0, idx, off, g)
    assert np.array_equal(out, wb.float().numpy())                   # exact up-conversion
    # bf16 tables: the value that is rounded to bf16 is formed by single fp32 operations (torch CPU float32
    # ops are IEEE single operations): step = lr * g, w - step
    want = (wb.float() - torch.tensor(0.01, dtype=torch.float32) * torch.from_numpy(g)).to(torch.bfloat16)
    assert np.array_equal(table, want.view(torch.int16).numpy().view(np.uint16))
    # Adagrad on a bf16 table, same rule: s += g*g; w -= (lr*g) / (sqrt(s) + eps), every operation in fp32
    table2 = wb.view(torch.int16).numpy().view(np.uint16).copy()
    s0 = rng.uniform(0, 2, size=(64, 8)).astype(np.float32)
    st = s0.copy()
    oracle.train_iter(table2, st, 8, oracle.BF16, oracle.ADAGRAD, 0.01, 1e-8, idx, off, g, want_out=False)
    gt, f = torch.from_numpy(g), (lambda x: torch.tensor(x, dtype=torch.float32))
    s1 = torch.from_numpy(s0) + gt * gt
    want2 = (wb.float() - (f(0.01) * gt) / (torch.sqrt(s1) + f(1e-8))).to(torch.bfloat16)
    assert np.array_equal(st, s1.numpy())
    assert np.array_equal(table2, want2.view(torch.int16).numpy().view(np.uint16))
    # exact ties go to the even mantissa: 1 + 2^-8 is half-way between bf16(1) and the next value
    t2 = torch.tensor([[1.0]], dtype=torch.bfloat16).view(torch.int16).numpy().view(np.uint16).copy()
    oracle.train_iter(t2, None, 1, oracle.BF16, oracle.SGD, 1.0, 0.0, np.array([0]), np.array([0, 1]),
                      np.array([[-(2.0 ** -8)]], dtype=np.float32))
    assert t2[0, 0] == 0x3F80
    oracle.train_iter(t2, None, 1, oracle.BF16, oracle.SGD, 1.0, 0.0, np.array([0]), np.array([0, 1]),
                      np.array([[-3 * (2.0 ** -8)]], dtype=np.float32))
    assert t2[0, 0] == 0x3F82                                       # 1 + 3*2^-8 -> 1 + 2*2^-7 (even)


def run_uncached(cfg, trace, T):
    R, D = cfg.total_rows, cfg.dim
    dt, op = oracle.DTYPES[cfg.weight_dtype], oracle.OPTIMIZERS[cfg.optimizer]
    W = workloads.init_weights(cfg, 0, R)
    W = (W.to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16).copy() if dt == oracle.BF16
         else W.numpy().copy())
    S = np.zeros(oracle.state_shape(R, D, op), dtype=np.float32)
    outs = []
    for i in range(T):
        g = workloads.upstream_grad(cfg, i, trace.bag_offsets.shape[1] - 1).numpy()
        outs.append(oracle.train_iter(W, S, D, dt, op, cfg.lr, cfg.eps, trace.iter_ids(i), trace.bag_offsets[i], g))
    return W, S, outs


def run_cached(cfg, trace, T, plan):
    R, D, C = cfg.total_rows, cfg.dim, cfg.capacity
    dt, op = oracle.DTYPES[cfg.weight_dtype], oracle.OPTIMIZERS[cfg.optimizer]
    W = workloads.init_weights(cfg, 0, R)
    W = (W.to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16).copy() if dt == oracle.BF16
         else W.numpy().copy())
    S = np.zeros(oracle.state_shape(R, D, op), dtype=np.float32)
    cw = np.full((C, D), 0x7FC0 if dt == oracle.BF16 else np.nan, dtype=W.dtype)     # poison: unfetched slots
    cs = np.full(oracle.state_shape(C, D, op), np.nan, dtype=np.float32)
    outs = []
    e_ids = np.zeros(0, np.int64)
    e_slots = np.zeros(0, np.int32)
    for i in range(T):
        a, b = plan.prefetch_off[i], plan.prefetch_off[i + 1]
        oracle.cache_apply(cw, cs, W, S, D, dt, op, e_ids, e_slots, plan.prefetch_ids[a:b], plan.prefetch_slots[a:b])
        g = workloads.upstream_grad(cfg, i, trace.bag_offsets.shape[1] - 1).numpy()
        sl = plan.lookup_slots[trace.iter_offsets[i]:trace.iter_offsets[i + 1]]
        outs.append(oracle.train_iter(cw, cs, D, dt, op, cfg.lr, cfg.eps, sl, trace.bag_offsets[i], g))
        a, b = plan.evict_off[i], plan.evict_off[i + 1]
        e_ids, e_slots = plan.evict_ids[a:b], plan.evict_slots[a:b]
    oracle.cache_apply(cw, cs, W, S, D, dt, op, e_ids, e_slots, np.zeros(0, np.int64), np.zeros(0, np.int32))
    return W, S, outs


@pytest.mark.parametrize("optimizer,dtype,bag_max,capacity", [
    ("sgd", "f32", 1, 4096), ("adagrad", "f32", 1, 1400), ("adagrad_rowwise", "bf16", 1, 4096),
    ("sgd", "f32", 6, 3000), ("adagrad", "bf16", 4, 2600)])
def test_cached_training_equals_uncached(optimizer, dtype, bag_max, capacity):
    """The consistency claim of Section 3.2: training through the plan and the cache gives exactly the result
    of synchronous training on the full table — same pooled outputs every iteration, same final table."""
    cfg = workloads.get_config(0, optimizer=optimizer, weight_dtype=dtype, bag_max=bag_max, capacity=capacity,
                               batch=128 if bag_max > 1 else 256, iterations=30)
    tr = workloads.make_trace(cfg)
    plan = oracle.plan(tr.ids, tr.iter_offsets, cfg.total_rows, cfg.lookahead, cfg.capacity)
    Wu, Su, ou = run_uncached(cfg, tr, cfg.iterations)
    Wc, Sc, oc = run_cached(cfg, tr, cfg.iterations, plan)
    for a, b in zip(ou, oc):
        assert np.array_equal(a, b)
    assert np.array_equal(Wu, Wc) and np.array_equal(Su, Sc)
    # rows never looked up keep their initial value
    W0 = workloads.init_weights(cfg, 0, cfg.total_rows)
    touched = np.zeros(cfg.total_rows, dtype=bool)
    touched[np.unique(tr.ids)] = True
    if dtype == "f32":
        assert np.array_equal(Wu[~touched], W0.numpy()[~touched])
        assert np.abs(Wu[touched] - W0.numpy()[touched]).max() > 0


# ---------------------------------------------------------------------------------------------------
# bf16 rows with row-wise Adagrad (the rule of the largest workload): the value that is rounded to bf16 must be
# formed by single fp32 operations after fp64 sums.  Pinned by hand-computed bit patterns, by the rule written
# with torch tensor operations, and by showing that slips planted in the oracle's source turn these pins red.
# ---------------------------------------------------------------------------------------------------
def bf16_bits(x):
    return torch.as_tensor(x, dtype=torch.float32).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16).copy()


def torch_rowwise_bf16_step(w_bits, s, idx, off, g, lr, eps):
    """One step of the rule on a bf16 table with torch tensor operations only.  w_bits: uint16 [rows, D];
    s: float32 [rows]; returns (new bits, new state).  fp64 sums rounded once to fp32, then one fp32 operation per
    line (torch float32 CPU operations are IEEE single operations), round-to-nearest-even on store."""
    rows, D = w_bits.shape
    w = torch.from_numpy(w_bits.view(np.int16).copy()).view(torch.bfloat16).float()
    bag_of = np.repeat(np.arange(len(off) - 1), np.diff(off))
    G64 = torch.zeros((rows, D), dtype=torch.float64)
    G64.index_add_(0, torch.from_numpy(idx), torch.from_numpy(g[bag_of]).double())
    G = G64.float()                                              # gradient sum: fp64 -> fp32, once
    touched = torch.zeros(rows, dtype=torch.bool)
    touched[torch.from_numpy(idx)] = True
    mean = ((G.double() * G.double()).sum(dim=1) / D).float()    # mean of squares of the rounded sum: fp64 -> fp32
    s_new = torch.from_numpy(s) + mean                           # fp32
    den = torch.sqrt(s_new) + torch.tensor(eps, dtype=torch.float32)
    step = (torch.tensor(lr, dtype=torch.float32) * G) / den[:, None]
    w_new = w - step
    w_out = torch.where(touched[:, None], w_new, w).to(torch.bfloat16)
    s_out = torch.where(touched, s_new, torch.from_numpy(s))
    return w_out.view(torch.int16).numpy().view(np.uint16).copy(), s_out.numpy().copy()


def test_bf16_rowwise_adagrad_hand_computed_row():
    """One row, D = 2, weights (1, 0.5), state 0, lr 0.5, eps 0, two lookups with gradients (1, 1) and (2, 3):
    G = (3, 4); mean of squares 12.5; state 12.5; den = sqrt(12.5) = 3.5355339 (fp32 0x40624621);
    steps 1.5/den = 0.42426407 and 2/den = 0.56568545; new weights 0.57573593 and -0.06568545, which round to
    the bf16 codes 0x3F13 (0.57421875: the fp32 pattern 0x3F136368 drops 0x6368 < 0x8000) and 0xBD87 (the fp32
    pattern 0xBD8685F4 has 0x85F4 > 0x8000 and rounds up to 0xBD87 = -0.065917969)."""
    table = bf16_bits([[1.0, 0.5], [0.25, 0.25]])
    state = np.zeros(2, dtype=np.float32)
    g = np.array([[1, 1], [2, 3]], dtype=np.float32)
    oracle.train_iter(table, state, 2, oracle.BF16, oracle.ADAGRAD_ROWWISE, 0.5, 0.0, np.array([0, 0]),
                      np.array([0, 1, 2]), g, want_out=False)
    assert state[0] == np.float32(12.5) and state[1] == 0
    assert table[0].tolist() == [0x3F13, 0xBD87]
    assert table[1].tolist() == bf16_bits([0.25, 0.25]).tolist()            # untouched row
    # second step on the same row with gradient (-4, 0): mean 8, state 20.5, den = sqrt(20.5) = 4.5276926,
    # step0 = -2/den = -0.44172609 -> w0 = 0.57421875 + 0.44172609 = 1.01594484 -> bf16 0x3F82 (1.015625);
    # step1 = 0 -> w1 stays 0xBD87
    oracle.train_iter(table, state, 2, oracle.BF16, oracle.ADAGRAD_ROWWISE, 0.5, 0.0, np.array([0]),
                      np.array([0, 1]), np.array([[-4, 0]], dtype=np.float32), want_out=False)
    assert state[0] == np.float32(20.5)
    assert table[0].tolist() == [0x3F82, 0xBD87]


def rowwise_bf16_case(seed, rows=37, D=16, steps=6):
    rng = np.random.default_rng(seed)
    w_bits = bf16_bits(rng.uniform(-0.05, 0.05, size=(rows, D)).astype(np.float32))
    batches = []
    for _ in range(steps):
        _, idx, off, r2 = rand_problem(int(rng.integers(1 << 30)), rows=rows, D=D, bags=60, max_len=4)
        # gradients with many significant bits, so that a sum of several of them is not an fp32 number
        g = (r2.standard_normal((len(off) - 1, D)) * r2.uniform(0.01, 30.0, size=(len(off) - 1, 1))).astype(np.float32)
        batches.append((idx, off, g))
    return w_bits, batches


def run_rowwise_bf16(train_iter_fn, w_bits, batches, D, lr, eps):
    table, state = w_bits.copy(), np.zeros(w_bits.shape[0], dtype=np.float32)
    for idx, off, g in batches:
        train_iter_fn(table, state, D, oracle.BF16, oracle.ADAGRAD_ROWWISE, lr, eps, idx, off, g, want_out=False)
    return table, state


@pytest.mark.parametrize("seed", [11, 12, 13])
def test_bf16_rowwise_adagrad_matches_torch_ops(seed):
    """Several rows, several steps, duplicate lookups inside and across bags, gradients that vary along the row:
    weights (bf16 codes) and state (fp32) equal, bit for bit, the rule written with torch tensor operations."""
    D, lr, eps = 16, 0.01, 1e-8
    w_bits, batches = rowwise_bf16_case(seed, D=D)
    table, state = run_rowwise_bf16(oracle.train_iter, w_bits, batches, D, lr, eps)
    wt, st = w_bits.copy(), np.zeros(w_bits.shape[0], dtype=np.float32)
    for idx, off, g in batches:
        wt, st = torch_rowwise_bf16_step(wt, st, idx, off, g, lr, eps)
    assert np.array_equal(state, st)
    assert np.array_equal(table, wt)
    assert (table != w_bits).mean() > 0.5                       # the steps moved most codes


def _mutated_oracle(tmp_path, old, new):
    """The oracle's source with one textual change, compiled with the oracle's own flags into a library of its own."""
    import ctypes
    import os
    import subprocess
    src = open(os.path.join(os.path.dirname(oracle.__file__), "bagpipe_oracle.c")).read()
    assert src.count(old) == 1, f"mutation target not unique: {old!r}"
    c = tmp_path / "mutant.c"
    c.write_text(src.replace(old, new))
    so = tmp_path / "libmutant.so"
    subprocess.run(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off", "-fno-fast-math", "-pthread",
                    "-o", str(so), str(c), "-lm"], check=True)
    lib = ctypes.CDLL(str(so))
    i64, i32, p = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p
    lib.orc_train_iter.restype = i32
    lib.orc_train_iter.argtypes = [p, p, i64, i64, i32, i32, ctypes.c_float, ctypes.c_float, p, i64, p, i64, p, p]

    def train_iter(table, state, D, dtype, optimizer, lr, eps, row_idx, bag_off, grad_out, want_out=False):
        row_idx = np.ascontiguousarray(row_idx, dtype=np.int64)
        bag_off = np.ascontiguousarray(bag_off, dtype=np.int64)
        grad_out = np.ascontiguousarray(grad_out, dtype=np.float32)
        vp = lambda a: ctypes.c_void_p(a.ctypes.data)
        r = lib.orc_train_iter(vp(table), vp(state), table.shape[0], D, dtype, optimizer, lr, eps, vp(row_idx),
                               row_idx.shape[0], vp(bag_off), bag_off.shape[0] - 1, vp(grad_out), None)
        assert r == 0
    return train_iter


@pytest.mark.parametrize("old,new", [
    # the mean of squares divided by D - 1 instead of D
    ("float mean = (float)(ms / (double)D);", "float mean = (float)(ms / (double)(D - 1));"),
    # the squares summed over the unrounded fp64 gradient sum instead of its fp32 value
    ("{ float g = (float)G[d]; ms += (double)g * (double)g; }", "{ ms += G[d] * G[d]; }"),
    # epsilon added under the root
    ("den_row = sqrtf(s) + eps;", "den_row = sqrtf(s + eps);"),
    # the squares added up in fp32 instead of fp64
    ("double ms = 0.0;\n        for (int64_t d = 0; d < D; ++d) { float g = (float)G[d]; ms += (double)g * (double)g; }",
     "float ms = 0.0f;\n        for (int64_t d = 0; d < D; ++d) { float g = (float)G[d]; ms += g * g; }"),
    # the weight stepped by lr * g without the division
    ("step = step / den_row;", "step = step * den_row;"),
    # the state not accumulated
    ("float s = state[row] + mean;\n        state[row] = s;\n        den_row", "float s = mean;\n        state[row] = s;\n        den_row"),
])
def test_bf16_rowwise_pins_catch_planted_slips(tmp_path, old, new):
    """A slip planted in the oracle's bf16 row-wise branch (in a copy of its source, compiled apart) must fail the
    comparison with the torch-operations form of the rule: this is what shows that the pin above can see them."""
    D, lr, eps = 16, 0.01, 1e-3          # an epsilon large enough that its place in the formula shows in fp32
    mutant = _mutated_oracle(tmp_path, old, new)
    caught = False
    for seed in (11, 12, 13):
        w_bits, batches = rowwise_bf16_case(seed, D=D)
        wt, st = w_bits.copy(), np.zeros(w_bits.shape[0], dtype=np.float32)
        for idx, off, g in batches:
            wt, st = torch_rowwise_bf16_step(wt, st, idx, off, g, lr, eps)
        good_t, good_s = run_rowwise_bf16(oracle.train_iter, w_bits, batches, D, lr, eps)
        assert np.array_equal(good_t, wt) and np.array_equal(good_s, st)       # the real oracle passes at this epsilon too
        bad_t, bad_s = run_rowwise_bf16(mutant, w_bits, batches, D, lr, eps)
        caught = caught or not (np.array_equal(bad_t, wt) and np.array_equal(bad_s, st))
    assert caught


# ---------------------------------------------------------------------------------------------------
# the multi-threaded leg is the serial routine, bit for bit
# ---------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("optimizer,dtype", [("sgd", "f32"), ("adagrad", "f32"), ("adagrad_rowwise", "f32"),
                                             ("sgd", "bf16"), ("adagrad", "bf16"), ("adagrad_rowwise", "bf16")])
@pytest.mark.parametrize("threads", [2, 3, 8])
def test_threaded_leg_equals_serial(optimizer, dtype, threads):
    D, rows = 8, 300
    dt, op = oracle.DTYPES[dtype], oracle.OPTIMIZERS[optimizer]
    rng = np.random.default_rng(77)
    w32 = rng.uniform(-0.05, 0.05, size=(rows, D)).astype(np.float32)
    W1 = bf16_bits(w32) if dt == oracle.BF16 else w32.copy()
    W2 = W1.copy()
    S1 = np.zeros(oracle.state_shape(rows, D, op), dtype=np.float32)
    S2 = S1.copy()
    for it in range(5):
        _, idx, off, r2 = rand_problem(500 + it, rows=rows, D=D, bags=700, max_len=6)
        g = r2.standard_normal((len(off) - 1, D)).astype(np.float32)
        o1 = oracle.train_iter(W1, S1, D, dt, op, 0.01, 1e-8, idx, off, g)
        o2 = oracle.train_iter(W2, S2, D, dt, op, 0.01, 1e-8, idx, off, g, threads=threads)
        assert np.array_equal(o1, o2)
        assert np.array_equal(W1, W2) and np.array_equal(S1, S2)
    # forward only / backward only, and more threads than bags
    _, idx, off, r2 = rand_problem(900, rows=rows, D=D, bags=5, max_len=3)
    g = r2.standard_normal((5, D)).astype(np.float32)
    assert np.array_equal(oracle.train_iter(W1, S1, D, dt, op, 0.01, 1e-8, idx, off, None),
                          oracle.train_iter(W2, S2, D, dt, op, 0.01, 1e-8, idx, off, None, threads=threads))
    oracle.train_iter(W1, S1, D, dt, op, 0.01, 1e-8, idx, off, g, want_out=False)
    oracle.train_iter(W2, S2, D, dt, op, 0.01, 1e-8, idx, off, g, want_out=False, threads=threads)
    assert np.array_equal(W1, W2) and np.array_equal(S1, S2)
