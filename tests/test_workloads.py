"""The synthetic input generators: shapes, determinism, skew and value distributions."""
import numpy as np
import torch

import workloads


def test_config_shapes():
    c = workloads.CONFIGS
    assert [x.num_tables for x in c] == [8, 26, 26, 20, 40]
    assert c[0].total_rows == 80_000 and c[3].total_rows == 100_000_000 and c[4].total_rows == 400_000_000
    assert abs(c[1].total_rows - 3_000_000) < 30_000 and min(c[1].table_rows) >= 10 and max(c[1].table_rows) <= 10 ** 6
    assert c[2].total_rows == 33_800_000 and min(c[2].table_rows) == 3 and max(c[2].table_rows) == 10_000_000
    assert c[2].capacity == 676_000 and c[1].capacity == c[1].total_rows // 100
    assert [x.dim for x in c] == [16, 16, 48, 64, 128]
    assert c[2].bags == 425_984                     # 16,384 samples x 26 features (Section 2.3)


def test_zipf_exponents_give_the_papers_skew():
    """Configs 1 and 2: the hottest 1 % of rows carry 92 % +- 0.5 % of the access probability (Section 2.3)."""
    for i in (1, 2):
        m = workloads.top_fraction_mass(workloads.CONFIGS[i].table_rows, workloads.CONFIGS[i].zipf_s)
        assert abs(m - 0.92) < 0.005, (i, m)


def test_trace_is_deterministic_and_well_formed():
    cfg = workloads.CONFIGS[0]
    a, b = workloads.make_trace(cfg), workloads.make_trace(cfg)
    assert np.array_equal(a.ids, b.ids) and a.n_lookups == 50 * 256 * 8
    toff = workloads.table_offsets(cfg)
    ids = a.ids.reshape(50, 256, 8)
    for t in range(8):
        assert ids[:, :, t].min() >= toff[t] and ids[:, :, t].max() < toff[t + 1]
    # skewed: the most frequent row of a table takes a large share (Zipf s=1.2 over 10,000 rows: ~19 %)
    share = np.bincount(ids[:, :, 0].ravel() - toff[0]).max() / (50 * 256)
    assert 0.12 < share < 0.3
    assert not np.array_equal(workloads.make_trace(workloads.get_config(0, seed=1)).ids, a.ids)


def test_multihot_trace_layout():
    cfg = workloads.get_config(3, iterations=3, batch=64)
    tr = workloads.make_trace(cfg)
    toff = workloads.table_offsets(cfg)
    assert tr.bag_offsets.shape == (3, 64 * 20 + 1)
    lens = np.diff(tr.bag_offsets, axis=1)
    assert lens.min() >= 1 and lens.max() <= 50 and 20 < lens.mean() < 31
    for i in range(3):
        ids = tr.iter_ids(i)
        assert len(ids) == tr.bag_offsets[i, -1]
        table_of_lookup = np.repeat(np.arange(64 * 20) % 20, lens[i])
        assert ((ids >= toff[table_of_lookup]) & (ids < toff[table_of_lookup + 1])).all()


def test_drift_changes_hot_set():
    cfg = workloads.get_config(4, iterations=4, batch=512, drift_every=2, table_rows=(100_000,) * 40)
    tr = workloads.make_trace(cfg)
    ids = tr.ids.reshape(4, 512, 40)[:, :, 0]
    hot = [np.bincount(ids[i] - 0, minlength=100_000).argmax() for i in range(4)]
    assert hot[0] == hot[1] and hot[2] == hot[3] and hot[0] != hot[2]


def test_hash_weights_and_grads():
    cfg = workloads.CONFIGS[0]
    W = workloads.init_weights(cfg, 0, 4000)
    assert W.dtype == torch.float32 and W.shape == (4000, 16)
    assert -0.05 < W.min() and W.max() < 0.05 and abs(W.mean()) < 5e-4 and abs(W.std() - 0.1 / 12 ** 0.5) < 3e-4
    assert torch.equal(workloads.init_weights(cfg, 1000, 1010), W[1000:1010])      # pure function of the row
    g = workloads.upstream_grad(cfg, 7, 2048)
    assert abs(g.mean()) < 0.02 and abs(g.std() - 1.0) < 0.02 and g.abs().max() < 6
    assert not torch.equal(g, workloads.upstream_grad(cfg, 8, 2048))
    assert torch.equal(g, workloads.upstream_grad(cfg, 7, 2048))
    # every value is a multiple of 2^-16 (exact in fp32 on any device)
    assert torch.equal((g.double() * 65536).round(), g.double() * 65536)


def test_hot_exp_law_has_the_chosen_skew():
    """Section 5.3's artificial workload: the hottest 1 % of a table's rows carry the chosen share of the accesses
    through a decaying law, the rest is uniform."""
    for n, skew in ((10_000, 0.4), (1_000, 0.9), (50, 0.01), (3, 0.4)):
        cdf = workloads.hot_exp_cdf(n, skew)
        p = np.diff(np.concatenate([[0.0], cdf]))
        h = max(1, int(np.ceil(0.01 * n)))
        assert abs(cdf[-1] - 1.0) < 1e-12 and (p > 0).all()
        assert abs(p[:h].sum() - skew) < 1e-12
        assert np.all(np.diff(p[:h]) < 0)                              # decays over the hot ranks
        if h > 1:
            assert abs(p[0] / p[h - 1] - np.exp(workloads.HOT_EXP_DECAY * (h - 1) / h)) < 1e-6 * p[0] / p[h - 1]
        assert np.allclose(p[h:], (1 - skew) / (n - h), rtol=1e-9)     # uniform tail
    assert abs(workloads.hot_exp_cdf(1, 0.4)[0] - 1.0) < 1e-15       # a one-row table: all of it


def test_skew_config_trace_matches_its_law():
    cfg = workloads.skew_config(0, 0.4, iterations=40, batch=512)
    assert cfg.id_law == "hot_exp" and cfg.name.endswith("skew40")
    tr = workloads.make_trace(cfg)
    tr2 = workloads.make_trace(cfg)
    assert np.array_equal(tr.ids, tr2.ids)
    toff = workloads.table_offsets(cfg)
    # per table: the 1 % most frequent rows of the sample take about 40 % of its draws (20,480 draws per table)
    for t in range(cfg.num_tables):
        col = tr.ids.reshape(-1, cfg.num_tables)[:, t]
        assert col.min() >= toff[t] and col.max() < toff[t + 1]
        counts = np.sort(np.bincount(col - toff[t], minlength=cfg.table_rows[t]))[::-1]
        share = counts[:cfg.table_rows[t] // 100].sum() / counts.sum()
        assert 0.38 < share < 0.44, share                              # top-k of a sample overshoots a little
    # a different skew gives a different trace, and Zipf configs are untouched by the new field
    assert not np.array_equal(tr.ids, workloads.make_trace(workloads.skew_config(0, 0.9, iterations=40, batch=512)).ids)
    assert workloads.CONFIGS[0].id_law == "zipf"
