"""GPU parity at the full sizes of the benchmark configurations, in the launch configuration
bench.py times (device-filled tables, all shards in one batched worker step, coalescing
structure built on the side stream).  The oracle sees the same tables restricted to the rows
the batch touches (ids relabelled in ascending order, which changes no arithmetic), so it
finishes in seconds to minutes."""
import numpy as np
import pytest
import torch

import oracle
import workload as wl
from helpers import BF16_MAX_TOL, assert_close, flat_dense_grad, rel_err

pytestmark = pytest.mark.gpu
TOL32, TOLBF = 1e-5, 2e-2


def compact_problem(cfg, batch):
    """Oracle inputs on the touched rows only: (model, tables, state, relabelled batch, unique ids)."""
    F, D = cfg.num_fields, cfg.dim
    uniq = [np.unique(batch.field_ids(f)) for f in range(F)]
    Rc = max(len(u) for u in uniq)
    ids = batch.ids.copy()
    for f in range(F):
        lo, hi = batch.field_ptr[f], batch.field_ptr[f + 1]
        ids[lo:hi] = np.searchsorted(uniq[f], batch.field_ids(f)).astype(np.int32)
    cb = wl.Batch(ids, batch.field_ptr, batch.offsets, batch.dense, batch.labels)
    tabs = []
    for f in range(F):
        t = np.zeros((Rc, D), np.float32)
        t[:len(uniq[f])] = wl.table_rows_f32(cfg, f, uniq[f])
        tabs.append(t)
    model = oracle.Model(F, Rc, D, cfg.num_dense, tuple(cfg.layer_sizes), cfg.adagrad_state == "rowwise",
                         cfg.table_dtype == "bf16", cfg.gemm_dtype == "bf16", cfg.lr, cfg.eps)
    return model, tabs, cb, uniq


def run_fullsize(cfg, oracle_shards=None, check_rows=200_000):
    import paper_2404_09679_amd as A
    dev = "cuda:0"
    F, R, D = cfg.num_fields, cfg.rows_per_field, cfg.dim
    batch = wl.make_batch(cfg, 0)
    flat = wl.make_mlp_params(cfg)
    tdtype = torch.bfloat16 if cfg.table_dtype == "bf16" else torch.float32
    tables = torch.empty((F * R, D), dtype=tdtype, device=dev)
    A.fill_tables(tables, F, R, D, 0.05)
    state = torch.zeros((F * R, D) if cfg.adagrad_state == "elementwise" else (F * R,), dtype=torch.float32, device=dev)
    params = torch.from_numpy(flat.copy()).to(dev)
    pstate = torch.zeros_like(params)
    ctx = A.Context(A.model_from_config(cfg, max_nnz=int(batch.field_ptr[-1])))
    ctx.bind(tables, state, params, pstate)
    d_ids, d_off = torch.from_numpy(batch.ids).to(dev), torch.from_numpy(batch.offsets).to(dev)
    d_dense = torch.from_numpy(batch.dense).to(dev) if cfg.num_dense else None
    d_labels = torch.from_numpy(batch.labels).to(dev)
    ctx.set_batch(d_ids, batch.field_ptr, d_off, d_dense, d_labels)
    K = cfg.num_shards
    ctx.assign_shard(cfg.batch, K, sizes=cfg.shard_sizes)
    loss = torch.zeros(K, device=dev)
    ctx.worker_step_all(loss)
    ctx.aggregate()
    torch.cuda.synchronize()
    print(f"[{cfg.name}] GPU iteration done; oracle on the touched rows", flush=True)

    # ---- oracle on the touched rows
    model, tabs, cb, uniq = compact_problem(cfg, batch)
    layers = wl.split_params(cfg, flat)
    shards = wl.shard_slices(cfg.shard_sizes)
    which = range(K) if oracle_shards is None else oracle_shards
    res = {k: oracle.worker_step(model, tabs, layers, cb, *shards[k]) for k in which}
    tol = TOLBF if cfg.gemm_dtype == "bf16" else TOL32
    mt = BF16_MAX_TOL if cfg.gemm_dtype == "bf16" else None
    W = cfg.input_width
    gl = loss.cpu().numpy()
    for k, r in res.items():
        x = ctx.view_pooled(k).float().cpu().numpy()
        dense, dx = ctx.view_shard_grads(k)
        assert_close(x[:, :W], r.x, 2.0 ** -8 if cfg.gemm_dtype == "bf16" else TOL32, f"pooled input, shard {k}")
        assert abs(gl[k] - r.loss) <= tol * abs(r.loss)
        assert_close(dense.cpu().numpy(), flat_dense_grad(cfg, r.dW, r.db), tol, f"dense gradient, shard {k}", mt)
        assert_close(dx.cpu().numpy(), r.dx, tol, f"d loss / d pooled, shard {k}", mt)
    print(f"[{cfg.name}] per-shard parity done", flush=True)
    full = oracle_shards is None
    if full:
        agg = oracle.aggregate(model, cb, [res[k] for k in range(K)])
        assert_close(ctx.view_dense_grad().cpu().numpy(), flat_dense_grad(cfg, agg.dW, agg.db), tol,
                     "aggregated dense gradient", mt)
    else:
        sub = oracle.aggregate(model, cb, [res[k] for k in which])
        sub_scale = sum(shards[k][1] for k in which) / cfg.batch
    Gs = []
    for f in range(F):
        u, so, ss, G = ctx.view_coalesced(f)
        u, so = u.cpu().numpy(), so.cpu().numpy()
        # exact structure: the distinct ids ascending and the run starts
        assert np.array_equal(u, uniq[f]), f"unique ids, field {f}"
        counts = np.bincount(cb.field_ids(f), minlength=len(uniq[f]))
        assert np.array_equal(so, np.concatenate([[0], np.cumsum(counts)])), f"segment offsets, field {f}"
        Gs.append(G.cpu().numpy())
        if full:
            assert_close(Gs[-1], agg.G[f], tol, f"coalesced gradient, field {f}", mt)
        else:
            # rows that only the oracle's shards look up: their coalesced gradient is the
            # subset aggregate scaled by (samples of the subset) / B
            su = sub.unique_ids[f]
            only = np.diff(sub.seg_offsets[f]) == counts[su]
            assert only.sum() > 0
            assert_close(Gs[-1][su[only]], sub.G[f][only] * sub_scale, tol,
                         f"coalesced gradient of rows private to the oracle's shards, field {f}", mt)
        if f < 3:  # grouping of the lookups: samples of every run, ascending
            ss = ss.cpu().numpy()
            sample = np.repeat(np.arange(cfg.batch), np.diff(batch.offsets[f]))
            order = np.lexsort((sample, cb.field_ids(f)))
            assert np.array_equal(ss, sample[order]), f"grouping of lookups, field {f}"
    print(f"[{cfg.name}] aggregation parity done", flush=True)
    ctx.apply_update()
    torch.cuda.synchronize()
    # ---- update: the oracle's Adagrad rule applied to the GPU's coalesced gradient, on every
    # touched row; untouched rows (a sample, and both neighbours of touched rows) unchanged
    rule = oracle.adagrad_rowwise if cfg.adagrad_state == "rowwise" else oracle.adagrad_elementwise
    rng = np.random.default_rng(5)
    for f in range(F):
        u = uniq[f]
        rows = torch.from_numpy(f * R + u.astype(np.int64)).to(dev)
        got = tables[rows].float().cpu().numpy()
        got_s = state[rows].cpu().numpy()
        t0 = tabs[f][:len(u)]
        p1, s1 = rule(t0, np.zeros_like(got_s), Gs[f], cfg.lr, cfg.eps)
        if cfg.table_dtype == "f32":
            assert_close(got - t0, p1 - t0, TOL32, f"Adagrad step on the GPU's G, field {f}")
        else:
            # the stored bf16 value is the rounding of the oracle's fp64 result, or its bf16
            # neighbour when the fp32 arithmetic lands on the other side of a rounding
            # boundary (rare); where the step cancels the parameter the slack is absolute
            want = oracle.round_bf16(p1)
            diff = np.abs(got - want)
            ok = (diff <= 2.0 ** -7 * np.maximum(np.abs(want), np.abs(got))) | (diff <= TOL32 * np.abs(t0))
            assert ok.all() and np.mean(got != want) < 0.01, f"bf16 write-back, field {f}"
        assert_close(got_s, s1, TOL32, f"accumulator, field {f}")
        near = np.unique(np.clip(np.concatenate([u - 1, u + 1, rng.integers(0, R, check_rows // F)]), 0, R - 1))
        near = np.setdiff1d(near, u)
        rows = torch.from_numpy(f * R + near.astype(np.int64)).to(dev)
        want = wl.table_rows_f32(cfg, f, near)
        assert np.array_equal(tables[rows].float().cpu().numpy(), want), f"untouched rows changed, field {f}"
        assert float(state[rows].abs().sum()) == 0.0
    # every accumulator outside the touched rows is still zero: the total equals the touched part
    touched_sum = sum(float(state[torch.from_numpy(f * R + uniq[f].astype(np.int64)).to(dev)].double().sum()) for f in range(F))
    assert abs(float(state.double().sum()) - touched_sum) <= 1e-9 * max(touched_sum, 1e-30)
    if full:
        upd_p, upd_s = oracle.adagrad_elementwise(flat, np.zeros_like(flat), ctx_dense_grad_host(agg, cfg), cfg.lr, cfg.eps)
        assert rel_err(params.cpu().numpy() - flat, upd_p - flat)[0] <= tol
    return ctx


def ctx_dense_grad_host(agg, cfg):
    return flat_dense_grad(cfg, agg.dW, agg.db)


def test_config2_full_size():
    run_fullsize(wl.CONFIGS[2])


def test_config3_heterogeneous_shards_full_size():
    run_fullsize(wl.CONFIGS[3])


def test_config4_bf16_tables_rowwise_state_full_size():
    """128 GB of bf16 tables, one Adagrad accumulator per row, 41.8 M lookups per iteration.
    The oracle runs all sixteen shards on the touched rows; rows the batch does not touch are
    checked on a sample of `check_rows` rows and on the neighbours of every touched row."""
    run_fullsize(wl.CONFIGS[4], check_rows=100_000)


def test_config5_dense_adam_full_size_sampled():
    import paper_2404_09679_amd as A
    dc = wl.DENSE_CONFIG
    n, K = dc.n, dc.num_buffers
    gen = torch.Generator(device="cuda")
    gen.manual_seed(dc.seed)
    p = torch.randn(n, device="cuda", generator=gen) * dc.param_std
    grads = [torch.randn(n, device="cuda", generator=gen) * dc.grad_std for _ in range(K)]
    m = torch.randn(n, device="cuda", generator=gen) * 1e-4
    v = torch.rand(n, device="cuda", generator=gen) * 1e-7
    w = np.array([512, 768, 1024, 1536, 2048, 2560, 3072, 4096]) / 15616
    idx = torch.from_numpy(np.concatenate([np.arange(64), n - 1 - np.arange(64),
                                           np.random.default_rng(0).integers(0, n, 1 << 20)])).cuda()
    before = [t[idx].cpu().numpy() for t in (p, m, v)]
    gs = [g[idx].cpu().numpy() for g in grads]
    total_before = float(p.double().sum())
    A.dense_aggregate_adam(p, m, v, grads, w, dc.lr, dc.beta1, dc.beta2, dc.eps, 7)
    torch.cuda.synchronize()
    p1, m1, v1 = oracle.dense_aggregate_adam(*before, gs, w, dc.lr, dc.beta1, dc.beta2, dc.eps, 7)
    assert_close(m[idx].cpu().numpy(), m1, TOL32, "m")
    assert_close(v[idx].cpu().numpy(), v1, TOL32, "v")
    assert rel_err(p[idx].cpu().numpy() - before[0], p1 - before[0])[0] <= TOL32
    # every element moved by at most lr * (bias-corrected ratio bound) and the buffer is finite
    assert torch.isfinite(p).all()
    assert abs(float(p.double().sum()) - total_before) <= n * dc.lr * 10
