"""CPU-only checks of the library's host side: it loads, exports every symbol the header
declares, validates arguments and call order, and splits batches as Section V-C.1 /
Section VI-A (Eq. 3) require.  No kernel is launched here."""
import ctypes as C
import os
import re
from fractions import Fraction

import numpy as np
import pytest

import oracle
import workload as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
A = pytest.importorskip("paper_2404_09679_amd", reason="build the library first (python paper_2404_09679_amd/build.py)")


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "antdt.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(antdt_[a-z_0-9]+)\s*\(", header))
    assert declared == set(A.binding.EXPORTS)
    for name in declared:
        assert hasattr(A.lib, name), name


def test_model_struct_matches_header_layout():
    # int32, (pad), int64, 4 x int32 ... : the ctypes mirror must have the C layout
    assert C.sizeof(A.Model) == 112 and A.Model.pooling.offset == 104
    assert A.Model.rows_per_field.offset == 8 and A.Model.layer_sizes.offset == 36
    assert A.Model.max_batch.offset == 88 and A.Model.max_nnz.offset == 96


def good_model():
    return A.model_from_config(wl.CONFIGS[1])


def test_shard_scale_arguments():
    ctx = A.Context(good_model())
    ctx.set_shard_scale((1.0, 0.5, 0.0, 2.0))
    ctx.set_shard_scale(None)
    for bad in [(1.0, -0.5), (float("nan"),), (float("inf"), 1.0), (1.0,) * 5]:
        with pytest.raises(A.AntdtError) as e:
            ctx.set_shard_scale(bad)
        assert e.value.code == -1 and "antdt_set_shard_scale" in str(e.value)


@pytest.mark.parametrize("field,value", [("num_fields", 0), ("num_fields", 129), ("rows_per_field", 0),
                                         ("dim", 6), ("dim", 3), ("dim", 512), ("table_dtype", 2), ("num_layers", 0),
                                         ("num_layers", 9), ("max_shards", 65), ("max_batch", 0), ("eps", 0.0),
                                         ("num_dense", 12), ("pooling", 2), ("pooling", -1)])
def test_create_rejects_bad_models(field, value):
    m = good_model()
    setattr(m, field, value)
    with pytest.raises(A.AntdtError) as e:
        A.Context(m)
    assert e.value.code == -1 and "antdt_create" in str(e.value)


def test_create_rejects_bad_layers():
    m = good_model()
    m.layer_sizes[m.num_layers] = 2
    with pytest.raises(A.AntdtError):
        A.Context(m)
    m = A.model_from_config(wl.scaled(wl.CONFIGS[1], layer_sizes=(141, 60, 1), gemm_dtype="bf16"))
    with pytest.raises(A.AntdtError) as e:
        A.Context(m)
    assert "multiples of 8" in str(e.value)


def test_static_binding_checks_its_arguments_before_any_gpu_work():
    """antdt_bind_static: null or misaligned buffers and a model whose workspace exceeds the
    library's static buffer are refused on the host, with both sizes in the message."""
    big = A.Context(A.model_from_config(wl.CONFIGS[2]))
    assert big.workspace_bytes() > 32 << 20
    rc = A.lib.antdt_bind_static(big._h, 256, 256, 256, 256, None)
    msg = A.lib.antdt_last_error(big._h).decode()
    assert rc == -3 and str(big.workspace_bytes()) in msg and str(32 << 20) in msg
    small = A.Context(good_model())
    assert small.workspace_bytes() <= 32 << 20
    assert A.lib.antdt_bind_static(small._h, None, 256, 256, 256, None) == -1
    assert A.lib.antdt_bind_static(small._h, 256, 264, 256, 256, None) == -1
    assert A.lib.antdt_bind_static(None, 256, 256, 256, 256, None) == -1
    header = open(os.path.join(ROOT, "include", "antdt.h")).read()
    assert "#define ANTDT_STATIC_SCRATCH_BYTES (32u << 20)" in header


def test_call_order_is_checked_before_any_gpu_work():
    ctx = A.Context(good_model())
    assert ctx.workspace_bytes() > 0
    fp = (C.c_int64 * 9)()
    rc = A.lib.antdt_set_batch(ctx._h, None, fp, None, None, None, 4, None)
    assert rc == -2 and b"antdt_bind" in A.lib.antdt_last_error(ctx._h)
    assert A.lib.antdt_worker_step(ctx._h, 0, None, None) == -1      # no shards yet
    ctx.assign_shard(256, 4)
    assert A.lib.antdt_worker_step(ctx._h, 0, None, None) == -2      # no batch yet
    assert A.lib.antdt_worker_step(ctx._h, 4, None, None) == -1
    assert A.lib.antdt_aggregate(ctx._h, None, None) == -2
    assert A.lib.antdt_apply_update(ctx._h, None) == -2
    assert A.lib.antdt_bind(ctx._h, None, None, None, None, None, 0, None) == -1
    assert A.lib.antdt_dense_aggregate_adam(None, None, None, None, None, 8, 4, 0.1, 0.9, 0.99, 1e-8, 1, None) == -1


def test_assign_shard_explicit_and_equal():
    ctx = A.Context(A.model_from_config(wl.CONFIGS[3]))
    sizes = wl.CONFIGS[3].shard_sizes
    got = ctx.assign_shard(sum(sizes), len(sizes), sizes=sizes)
    assert got == oracle.explicit_split(sizes)
    assert ctx.assign_shard(10, 4) == oracle.equal_split(10, 4) == [(0, 3), (3, 3), (6, 2), (8, 2)]
    assert ctx.assign_shard(0, 3) == [(0, 0)] * 3
    for bad in ([5, 5, 5], [-1, 11, 0]):
        with pytest.raises(A.AntdtError) as e:
            ctx.assign_shard(10, 3, sizes=bad)
        assert e.value.code == -1
    with pytest.raises(A.AntdtError):
        ctx.assign_shard(10, 9)                     # K > max_shards
    with pytest.raises(A.AntdtError):
        ctx.assign_shard(10, 2, speed=[1.0, 0.0])   # speeds must be positive


@pytest.mark.parametrize("speeds", [(1.0, 1.0, 1.0), (1.0, 2.0, 4.0), (3.0, 1.0), (0.5, 1.5, 1.0, 2.0),
                                    (1.0, 1.0, 3.0, 3.0), (7.0,), (0.3, 0.7, 1.9)])
def test_assign_shard_speed_mode_is_optimal_for_eq3(speeds):
    """ADJUST_BS: the split minimises max_k B_k / v_k over all integer splits (brute force)."""
    ctx = A.Context(A.model_from_config(wl.CONFIGS[1]))
    for B in range(0, 17):
        got = ctx.assign_shard(B, len(speeds), speed=speeds)
        lens = [n for _, n in got]
        assert sum(lens) == B and all(n >= 0 for n in lens)
        assert [s for s, _ in got] == list(np.cumsum([0] + lens[:-1]))
        z, arg = oracle.minmax_split_bruteforce(B, speeds)
        assert oracle.minmax_objective(lens, speeds) == z
        assert tuple(lens) in arg
        assert z >= Fraction(B) / sum(Fraction(v) for v in speeds)


def test_assign_shard_speed_mode_large_batch():
    ctx = A.Context(A.model_from_config(wl.CONFIGS[3]))
    speeds = [1.0, 1.5, 2.0, 3.0, 4.0, 5.0, 6.0, 8.0]
    B = 15616
    lens = [n for _, n in ctx.assign_shard(B, 8, speed=speeds)]
    assert sum(lens) == B
    z = max(n / v for n, v in zip(lens, speeds))
    # within one sample of the continuous optimum on every worker
    assert all(abs(n - B * v / sum(speeds)) <= 1.0 for n, v in zip(lens, speeds))
    # no single move improves the maximum
    for i in range(8):
        for j in range(8):
            if i != j and lens[i] > 0:
                moved = list(lens)
                moved[i] -= 1
                moved[j] += 1
                assert max(n / v for n, v in zip(moved, speeds)) >= z - 1e-12
    # equal speeds reproduce the initial B/n split
    assert [n for _, n in ctx.assign_shard(4096, 8, speed=[2.5] * 8)] == [512] * 8


# ------------------------------------------------------------------ Eq. 4: accumulation plan
def _check_plan(B, counts, speeds, bmin, bmax, cmin, cmax):
    from fractions import Fraction
    want_z, want_plans = oracle.accumulation_plan_bruteforce(B, counts, speeds, bmin, bmax, cmin, cmax)
    got = A.plan_accumulation(B, counts, speeds, bmin, bmax, cmin, cmax)
    if want_z is None:
        assert got is None
        return None
    assert got is not None, "a feasible problem was reported infeasible"
    Bi, Ci, z = got
    assert (tuple(Ci), tuple(Bi)) in want_plans, f"{(Ci, Bi)} is not among the optimal plans {want_plans}"
    assert sum(n * c * b for n, c, b in zip(counts, Ci, Bi)) == B
    assert abs(z - float(want_z)) <= 1e-12 * float(want_z)
    assert max(Fraction(c * b) / Fraction(v) for c, b, v in zip(Ci, Bi, speeds)) == want_z
    return got


def test_accumulation_plan_worked_cases():
    # one fast and one slow device: the fast one accumulates three micro-batches
    Bi, Ci, z = _check_plan(32, (1, 1), (1.0, 3.0), (2, 2), (8, 8), 1, 3)
    assert z == 8.0
    assert _check_plan(5, (2,), (1.0,), (1,), (2,), 1, 1) is None           # 2*C*B = 5 has no solution
    _check_plan(24, (2, 1), (1.0, 2.0), (1, 1), (24, 24), 1, 1)              # no accumulation: Eq. 3 with device counts
    _check_plan(7, (1,), (0.3,), (1,), (7,), 1, 7)                           # one type: any C*B = 7


def test_accumulation_plan_matches_enumeration_on_random_instances():
    rng = np.random.default_rng(11)
    feasible = 0
    for _ in range(60):
        k = int(rng.integers(1, 4))
        counts = tuple(int(x) for x in rng.integers(1, 4, k))
        speeds = tuple(float(x) for x in rng.choice([0.5, 1.0, 1.5, 2.0, 3.0, 0.7, 1.3], k))
        bmin = tuple(int(x) for x in rng.integers(1, 4, k))
        bmax = tuple(int(b + x) for b, x in zip(bmin, rng.integers(0, 6, k)))
        cmin = int(rng.integers(1, 3))
        cmax = cmin + int(rng.integers(0, 3))
        B = int(rng.integers(1, 80))
        if _check_plan(B, counts, speeds, bmin, bmax, cmin, cmax) is not None:
            feasible += 1
    assert feasible >= 10


def test_accumulation_plan_rejects_bad_arguments():
    with pytest.raises(A.AntdtError):
        A.plan_accumulation(0, (1,), (1.0,), (1,), (2,), 1, 1)
    with pytest.raises(A.AntdtError):
        A.plan_accumulation(8, (1,), (-1.0,), (1,), (2,), 1, 1)
    with pytest.raises(A.AntdtError):
        A.plan_accumulation(8, (1,), (1.0,), (3,), (2,), 1, 1)
    with pytest.raises(A.AntdtError):
        A.plan_accumulation(8, (1,), (1.0,), (1,), (2,), 2, 1)


def test_expand_accumulation_lists_micro_batches_device_by_device():
    sizes, dev = A.expand_accumulation((2, 1), (4, 3), (2, 3))
    assert sizes == [4, 4, 4, 4, 3, 3, 3]
    assert dev == [0, 0, 1, 1, 2, 2, 2]
    assert A.expand_accumulation((1,), (5,), (0,)) == ([], [])


# ------------------------------------------------------------------ shard queue (Section V-C)
def test_shard_queue_matches_the_oracle_step_by_step():
    rng = np.random.default_rng(17)
    for N, B, M in [(5003, 7, 13), (100, 10, 10), (1, 4, 100), (0, 3, 2), (999, 1, 1)]:
        lib_q, ref = A.ShardQueue(N, B, M), oracle.ShardQueue(N, B, M)
        K = lib_q.num_shards()
        assert K == len(ref.shards) == oracle.num_data_shards(N, B, M)
        assert [lib_q.shard(k)[:2] for k in range(K)] == list(ref.shards)
        for _ in range(6 * K + 20):
            w, r = int(rng.integers(0, 4)), rng.random()
            if r < 0.5:
                assert lib_q.fetch(w) == ref.fetch(w)
            elif r < 0.85 and K:
                k = int(rng.integers(0, K))
                try:
                    ref.report_done(k, w)
                    ok = True
                except ValueError:
                    ok = False
                if ok:
                    lib_q.report_done(k, w)
                else:
                    with pytest.raises(A.AntdtError) as e:
                        lib_q.report_done(k, w)
                    assert e.value.code == -2
            else:
                assert lib_q.release_worker(w) == ref.release_worker(w)
            assert lib_q.counts() == ref.counts()
            assert all(lib_q.shard(k)[2:] == (ref.state[k], ref.owner[k]) for k in range(K))
    with pytest.raises(A.AntdtError):
        A.ShardQueue(10, 0, 1)
    with pytest.raises(A.AntdtError):
        A.ShardQueue(10, 2, 2).report_done(99, 0)


# ------------------------------------------------------------------ training model
def _same_simulation(**kw):
    ref = oracle.simulate_bsp(oracle.SimConfig(**kw))
    kw = dict(kw)
    got, sizes = A.simulate_bsp(**kw)
    assert (got.iterations, got.processed, got.adjust_actions, got.kills) == \
        (ref.iterations, ref.processed, ref.adjust_actions, ref.kills)
    assert sizes == ref.final_sizes
    # the same operations in the same order on both sides: agreement to the last bits
    for a, b in ((got.jct, ref.jct), (got.max_bpt, ref.max_bpt), (got.sum_bpt, ref.sum_bpt)):
        assert abs(a - b) <= 1e-12 * abs(b)
    return got


def _hand_worked():
    from jct_schedules import SCHEDULES
    return SCHEDULES


@pytest.mark.parametrize("name,cfg,want", _hand_worked(), ids=[s[0] for s in _hand_worked()])
def test_training_model_follows_hand_worked_schedules(name, cfg, want):
    """The library's model against schedules worked out by hand (tests/jct_schedules.py): no
    implementation produced the expected values."""
    kw = dict(cfg)
    r, sizes = A.simulate_bsp(**kw)
    got = dict(jct=r.jct, iterations=r.iterations, processed=r.processed, adjust_actions=r.adjust_actions,
               kills=r.kills, max_bpt=r.max_bpt, sum_bpt=r.sum_bpt, final_sizes=sizes)
    assert got == want


def test_training_model_matches_the_oracle_for_every_policy():
    rng = np.random.default_rng(23)
    for trial in range(24):
        n = int(rng.integers(2, 11))
        B = int(rng.integers(n, 40)) * int(rng.integers(1, 60))
        kw = dict(n=n, B=B, N=B * int(rng.integers(50, 1500)),
                  t0=[float(x) for x in rng.uniform(0.0, 0.2, n)], v=[float(x) for x in rng.uniform(50.0, 500.0, n)],
                  t_server=float(rng.uniform(0.0, 0.1)), period=float(rng.choice([200.0, 1800.0])),
                  duration=float(rng.choice([50.0, 900.0])), prob=float(rng.choice([0.0, 0.3, 0.6])),
                  sleep_duration=1.5, intensity=float(rng.choice([0.1, 0.4, 0.8])), seed=int(rng.integers(1, 1 << 31)),
                  persistent_delay=[float(x) for x in (rng.random(n) < 0.2) * 4.0], policy=trial % 4,
                  backup_b=int(rng.integers(0, max(n // 2, 1))) if trial % 4 == 2 else 0,
                  decide_every=float(rng.choice([20.0, 300.0])), L_trans=float(rng.choice([20.0, 300.0])),
                  L_per=float(rng.choice([40.0, 600.0])), lam=float(rng.choice([1.2, 1.5])),
                  restart_cost=float(rng.choice([0.0, 30.0, 120.0])))
        _same_simulation(**kw)


def test_training_model_with_the_injection_pattern_of_the_evaluation():
    """Ten workers, disturbed with probability 0.3 for 15 of every 30 minutes, sleep 1.5 s times the
    intensity; a persistent straggler adds 4 s (Section VII-A.2).  Batch time: the affine fit of
    a worker that needs 0.45 s for its tenth of the global batch."""
    kw = dict(n=10, B=4096, N=4096 * 6000, t0=[0.05] * 10, v=[4096 / 10 / 0.40] * 10, t_server=0.05,
              prob=0.3, sleep_duration=1.5, decide_every=300.0, L_trans=300.0, L_per=600.0, lam=1.5)
    jct = {}
    for intensity in (0.1, 0.8):
        for pol in range(4):
            r = _same_simulation(policy=pol, intensity=intensity, backup_b=3 if pol == 2 else 0, **kw)
            jct[intensity, pol] = r.jct
    assert jct[0.8, 0] > jct[0.1, 0]                            # stronger disturbance, slower synchronous job
    r = _same_simulation(policy=3, intensity=0.0, prob=0.0, persistent_delay=[0.0] * 9 + [4.0], **{
        k: v for k, v in kw.items() if k != "prob"})
    assert r.kills == 1


def test_training_model_rejects_bad_arguments():
    ok = dict(n=2, B=10, N=100, t0=[0.1, 0.1], v=[10.0, 10.0])
    A.simulate_bsp(**ok)
    for bad in (dict(n=0), dict(B=1), dict(N=0), dict(v=[10.0, 0.0]), dict(t0=[-1.0, 0.1]), dict(policy=4),
                dict(backup_b=2, policy=2), dict(lam=0.5), dict(period=0.0), dict(decide_every=0.0)):
        kw = dict(ok)
        kw.update(bad)
        if "n" in bad:
            kw["t0"], kw["v"] = [], []
        with pytest.raises(A.AntdtError):
            A.simulate_bsp(**kw)
