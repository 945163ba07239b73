"""Glue shared by the tests: turn a workload configuration into oracle inputs."""
from __future__ import annotations

import numpy as np

import oracle
import workload as wl


def oracle_model(cfg: wl.RankingConfig, bf16_gemm=None) -> oracle.Model:
    return oracle.Model(cfg.num_fields, cfg.rows_per_field, cfg.dim, cfg.num_dense,
                        tuple(cfg.layer_sizes), cfg.adagrad_state == "rowwise",
                        cfg.table_dtype == "bf16",
                        (cfg.gemm_dtype == "bf16") if bf16_gemm is None else bf16_gemm,
                        cfg.lr, cfg.eps, cfg.pooling == "mean")


def tables_as_f32(cfg, tables):
    """[F*R, D] stored tables -> float32 values."""
    return tables if cfg.table_dtype == "f32" else wl.bf16_bits_to_f32(tables)


def per_field(cfg, arr):
    R = cfg.rows_per_field
    return [arr[f * R:(f + 1) * R] for f in range(cfg.num_fields)]


def oracle_iteration(cfg, tables_f32, state, flat_params, flat_state, batch, sizes,
                     mask=None, bf16_gemm=None, want_samples=False, scale=None):
    """Run worker_step for every shard, aggregate and apply_update with the oracle."""
    model = oracle_model(cfg, bf16_gemm)
    tabs = per_field(cfg, tables_f32)
    st = per_field(cfg, state)
    layers = wl.split_params(cfg, flat_params)
    lstate = wl.split_params(cfg, flat_state)
    res = [oracle.worker_step(model, tabs, layers, batch, s, n) for s, n in wl.shard_slices(sizes)]
    agg = oracle.aggregate(model, batch, res, mask, want_samples, scale)
    upd = oracle.apply_update(model, tabs, st, layers, lstate, agg)
    return model, res, agg, upd


def permute_batch(batch: wl.Batch, order) -> wl.Batch:
    """The same samples in another order (bags, dense features and labels move together)."""
    F = batch.offsets.shape[0]
    ids, fp, offs = [], [0], np.zeros_like(batch.offsets)
    for f in range(F):
        fi, o = batch.field_ids(f), batch.offsets[f]
        parts = [fi[o[s]:o[s + 1]] for s in order]
        offs[f, 1:] = np.cumsum([len(p) for p in parts])
        ids.append(np.concatenate(parts) if parts else fi[:0])
        fp.append(fp[-1] + int(offs[f, -1]))
    return wl.Batch(np.concatenate(ids).astype(np.int32), np.array(fp, np.int64), offs,
                    batch.dense[order], batch.labels[order])


def flat_dense_grad(cfg, dW, db):
    out = np.zeros(cfg.num_params, dtype=np.float64)
    for (wo, bo, fi, fo), W, b in zip(wl.param_layout(cfg), dW, db):
        out[wo:bo] = np.asarray(W).reshape(-1)
        out[bo:bo + fo] = np.asarray(b).reshape(-1)
    return out


def flat_layers(cfg, layers):
    return flat_dense_grad(cfg, [W for W, _ in layers], [b for _, b in layers])


def rel_err(a, b):
    """(normwise, maxwise) relative error of a against the reference b."""
    a = np.asarray(a, dtype=np.float64).reshape(-1)
    b = np.asarray(b, dtype=np.float64).reshape(-1)
    if b.size == 0:
        return 0.0, 0.0
    nb = max(float(np.linalg.norm(b)), 1e-300)
    mb = max(float(np.max(np.abs(b))), 1e-300)
    return float(np.linalg.norm(a - b)) / nb, float(np.max(np.abs(a - b))) / mb


def assert_close(a, b, tol, what="", max_tol=None):
    """Both error measures under `tol`; `max_tol` loosens the element-wise one (see BF16_MAX_TOL)."""
    n, m = rel_err(a, b)
    mt = tol if max_tol is None else max_tol
    assert n <= tol and m <= mt, f"{what}: normwise {n:.3e} (<= {tol:.1e}), maxwise {m:.3e} (<= {mt:.1e})"


# Gradients downstream of bf16-rounded activations: where an activation sits within rounding of
# zero, fp32 and float64 accumulation can round it to different sides, the ReLU decision of
# that one unit flips, and the gradient row of that one sample changes by O(1) relative to
# itself.  Such isolated elements are bounded by BF16_MAX_TOL of the tensor's largest entry;
# the normwise error stays under the 2e-2 bound.
BF16_MAX_TOL = 0.25


TINY = wl.RankingConfig("tiny", 2, 7, 3, "f32", "elementwise", 2, (8, 4, 1), "f32", 3, 1.05,
                        (2, 3), wl.SEED0 + 101, min_bag=0)
SMALL = wl.RankingConfig("small", 3, 50, 4, "f32", "elementwise", 3, (15, 8, 6, 1), "f32", 4, 1.05,
                         (5, 1, 0, 6), wl.SEED0 + 102, min_bag=0)


def assert_step_within_bound(step_gpu, step_ref, g_ref, cfg, tol, what):
    """End-to-end bound on an Adagrad step.  step = lr*g/(sqrt(S+g^2)+eps) has
    |d step / d g| <= lr/(|g|+eps), so a gradient that is within delta = tol*max|g| of the
    oracle's moves the step by at most lr*delta/(|g|-delta+eps) (large only where |g| ~ eps),
    on top of the tolerance on the step itself."""
    g = np.abs(np.asarray(g_ref, dtype=np.float64))
    delta = tol * (g.max() if g.size else 0.0)
    bound = cfg.lr * delta / (np.maximum(g - delta, 0.0) + cfg.eps) + tol * cfg.lr
    err = np.abs(np.asarray(step_gpu, np.float64) - np.asarray(step_ref, np.float64))
    worst = float((err / bound).max()) if err.size else 0.0
    assert worst <= 1.0, f"{what}: step error is {worst:.2f}x the bound"
    # and the bulk agrees tightly: all but the |g| ~ eps elements
    big = g > 1e3 * max(delta, cfg.eps)
    if big.any():
        assert rel_err(np.asarray(step_gpu)[big], np.asarray(step_ref)[big])[0] <= 10 * tol, what
