"""ctypes binding of include/antdt.h.  Argument marshalling only."""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libantdt_hip.so")

MAX_LAYERS, MAX_FIELDS, MAX_SHARDS = 8, 128, 64
F32, BF16 = 0, 1
INFEASIBLE = -6
ELEMENTWISE, ROWWISE = 0, 1
POOL_SUM, POOL_MEAN = 0, 1

EXPORTS = [
    "antdt_create", "antdt_destroy", "antdt_last_error", "antdt_workspace_bytes", "antdt_bind",
    "antdt_set_batch", "antdt_assign_shard", "antdt_worker_step", "antdt_worker_step_all",
    "antdt_aggregate", "antdt_apply_update", "antdt_dense_aggregate_adam", "antdt_fill_tables",
    "antdt_view_pooled", "antdt_view_shard_grads", "antdt_view_dense_grad", "antdt_view_coalesced",
    "antdt_profile", "antdt_profile_read", "antdt_kernel_name",
    "antdt_plan_accumulation", "antdt_expand_accumulation", "antdt_set_lr", "antdt_validate_batch",
    "antdt_set_shard_scale", "antdt_stream_copy", "antdt_profile_overhead", "antdt_bind_static",
    "antdt_set_eager_weight_gradients", "antdt_set_library_streams",
    "antdt_dds_create", "antdt_dds_destroy", "antdt_dds_num_shards", "antdt_dds_fetch", "antdt_dds_report_done",
    "antdt_dds_release_worker", "antdt_dds_shard", "antdt_dds_counts", "antdt_simulate_bsp",
]


class AntdtError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"antdt error {code}: {msg}")
        self.code = code


class Model(C.Structure):
    _fields_ = [
        ("num_fields", C.c_int32), ("rows_per_field", C.c_int64), ("dim", C.c_int32),
        ("table_dtype", C.c_int32), ("adagrad_state", C.c_int32), ("num_dense", C.c_int32),
        ("num_layers", C.c_int32), ("layer_sizes", C.c_int32 * (MAX_LAYERS + 1)),
        ("gemm_dtype", C.c_int32), ("lr", C.c_float), ("eps", C.c_float),
        ("max_shards", C.c_int32), ("max_batch", C.c_int64), ("max_nnz", C.c_int64),
        ("pooling", C.c_int32),
    ]


class SimConfig(C.Structure):
    _fields_ = [("n", C.c_int32), ("B", C.c_int64), ("N", C.c_int64), ("t0", C.POINTER(C.c_double)),
                ("v", C.POINTER(C.c_double)), ("t_server", C.c_double), ("period", C.c_double),
                ("duration", C.c_double), ("prob", C.c_double), ("sleep_duration", C.c_double),
                ("intensity", C.c_double), ("seed", C.c_uint32), ("persistent_delay", C.POINTER(C.c_double)),
                ("policy", C.c_int32), ("backup_b", C.c_int32), ("decide_every", C.c_double),
                ("L_trans", C.c_double), ("L_per", C.c_double), ("lam", C.c_double), ("restart_cost", C.c_double),
                ("max_iterations", C.c_int64)]


class SimResult(C.Structure):
    _fields_ = [("jct", C.c_double), ("iterations", C.c_int64), ("processed", C.c_int64),
                ("adjust_actions", C.c_int32), ("kills", C.c_int32), ("max_bpt", C.c_double), ("sum_bpt", C.c_double)]


def _load():
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is missing: build it with `python paper_2404_09679_amd/build.py` "
                          "(there is no CPU fallback)")
    lib = C.CDLL(_LIB_PATH)
    vp, i32, i64, f32 = C.c_void_p, C.c_int32, C.c_int64, C.c_float
    lib.antdt_create.argtypes = [C.POINTER(Model), C.POINTER(vp)]
    lib.antdt_destroy.argtypes = [vp]
    lib.antdt_last_error.argtypes = [vp]
    lib.antdt_last_error.restype = C.c_char_p
    lib.antdt_workspace_bytes.argtypes = [vp, C.POINTER(C.c_size_t)]
    lib.antdt_bind.argtypes = [vp, vp, vp, vp, vp, vp, C.c_size_t, vp]
    lib.antdt_bind_static.argtypes = [vp, vp, vp, vp, vp, vp]
    lib.antdt_set_batch.argtypes = [vp, vp, C.POINTER(i64), vp, vp, vp, i64, vp]
    lib.antdt_assign_shard.argtypes = [vp, i64, i32, C.POINTER(i64), C.POINTER(C.c_double),
                                       C.POINTER(i64), C.POINTER(i64)]
    lib.antdt_worker_step.argtypes = [vp, i32, vp, vp]
    lib.antdt_worker_step_all.argtypes = [vp, vp, vp]
    lib.antdt_aggregate.argtypes = [vp, C.POINTER(C.c_uint8), vp]
    lib.antdt_apply_update.argtypes = [vp, vp]
    f64 = C.c_double
    lib.antdt_dense_aggregate_adam.argtypes = [vp, vp, vp, C.POINTER(vp), C.POINTER(f32), i32, i64,
                                               f64, f64, f64, f64, i64, vp]
    lib.antdt_fill_tables.argtypes = [vp, i32, i32, i64, i32, f32, vp]
    lib.antdt_view_pooled.argtypes = [vp, i32, C.POINTER(vp), C.POINTER(i64), C.POINTER(i64), C.POINTER(i32)]
    lib.antdt_view_shard_grads.argtypes = [vp, i32, C.POINTER(vp), C.POINTER(vp), C.POINTER(i64)]
    lib.antdt_view_dense_grad.argtypes = [vp, C.POINTER(vp), vp]
    lib.antdt_view_coalesced.argtypes = [vp, i32, C.POINTER(vp), C.POINTER(vp), C.POINTER(vp),
                                         C.POINTER(i64), C.POINTER(i64), C.POINTER(vp), vp]
    lib.antdt_profile.argtypes = [vp, i32, i32]
    lib.antdt_profile_read.argtypes = [vp, i32, C.POINTER(i64), C.POINTER(C.c_double)]
    lib.antdt_kernel_name.argtypes = [i32]
    lib.antdt_kernel_name.restype = C.c_char_p
    lib.antdt_set_lr.argtypes = [vp, f32]
    lib.antdt_set_eager_weight_gradients.argtypes = [vp, i32]
    lib.antdt_set_library_streams.argtypes = [vp, i32]
    lib.antdt_set_shard_scale.argtypes = [vp, C.POINTER(C.c_double), i32]
    lib.antdt_stream_copy.argtypes = [vp, vp, i64, vp]
    lib.antdt_profile_overhead.argtypes = [vp, vp, i32, C.POINTER(C.c_double), C.POINTER(C.c_double)]
    lib.antdt_validate_batch.argtypes = [vp, vp]
    lib.antdt_dds_create.argtypes = [i64, i64, i32, C.POINTER(vp)]
    lib.antdt_dds_destroy.argtypes = [vp]
    lib.antdt_dds_num_shards.argtypes = [vp, C.POINTER(i64)]
    lib.antdt_dds_fetch.argtypes = [vp, i32, C.POINTER(i64), C.POINTER(i64), C.POINTER(i64)]
    lib.antdt_dds_report_done.argtypes = [vp, i64, i32]
    lib.antdt_dds_release_worker.argtypes = [vp, i32, C.POINTER(i64)]
    lib.antdt_dds_shard.argtypes = [vp, i64, C.POINTER(i64), C.POINTER(i64), C.POINTER(i32), C.POINTER(i32)]
    lib.antdt_dds_counts.argtypes = [vp, C.POINTER(i64), C.POINTER(i64), C.POINTER(i64)]
    lib.antdt_simulate_bsp.argtypes = [C.POINTER(SimConfig), C.POINTER(SimResult), C.POINTER(i64)]
    lib.antdt_plan_accumulation.argtypes = [i64, i32, C.POINTER(i32), C.POINTER(C.c_double), C.POINTER(i64),
                                            C.POINTER(i64), i32, i32, C.POINTER(i64), C.POINTER(i32),
                                            C.POINTER(C.c_double)]
    lib.antdt_expand_accumulation.argtypes = [i32, C.POINTER(i32), C.POINTER(i64), C.POINTER(i32), i32,
                                              C.POINTER(i64), C.POINTER(i32), C.POINTER(i32)]
    return lib


lib = _load()


def kernel_names() -> List[str]:
    out, i = [], 0
    while True:
        n = lib.antdt_kernel_name(i)
        if n is None:
            return out
        out.append(n.decode())
        i += 1


def model_from_config(cfg, max_batch: Optional[int] = None, max_nnz: Optional[int] = None,
                      max_shards: Optional[int] = None, gemm_dtype: Optional[str] = None) -> Model:
    """Model descriptor of a workload configuration (any object with its field names)."""
    m = Model()
    m.num_fields, m.rows_per_field, m.dim = cfg.num_fields, cfg.rows_per_field, cfg.dim
    m.table_dtype = BF16 if cfg.table_dtype == "bf16" else F32
    m.adagrad_state = ROWWISE if cfg.adagrad_state == "rowwise" else ELEMENTWISE
    m.num_dense = cfg.num_dense
    m.num_layers = len(cfg.layer_sizes) - 1
    for i, s in enumerate(cfg.layer_sizes):
        m.layer_sizes[i] = s
    m.gemm_dtype = BF16 if (gemm_dtype or cfg.gemm_dtype) == "bf16" else F32
    m.lr, m.eps = cfg.lr, cfg.eps
    m.max_shards = max_shards or max(1, len(cfg.shard_sizes))
    m.max_batch = max_batch or max(1, sum(cfg.shard_sizes))
    m.max_nnz = max_nnz if max_nnz is not None else m.max_batch * cfg.max_bag * cfg.num_fields
    m.pooling = POOL_MEAN if getattr(cfg, "pooling", "sum") == "mean" else POOL_SUM
    return m


_raw_stream = getattr(torch._C, "_cuda_getCurrentRawStream", None)


def _stream() -> int:
    """Handle of torch's current stream on the current device (the raw getter costs about a
    microsecond, torch.cuda.current_stream() about ten)."""
    if _raw_stream is not None:
        return _raw_stream(torch.cuda.current_device())
    return torch.cuda.current_stream().cuda_stream


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


class _RawDeviceBytes:
    """nbytes of device memory at ptr, for torch.as_tensor (no copy, no ownership)."""

    def __init__(self, ptr: int, nbytes: int):
        self.__cuda_array_interface__ = {"shape": (nbytes,), "typestr": "|u1", "data": (ptr, False), "version": 2}


class Context:
    """One model bound to caller-owned device tensors.  Methods mirror the C calls."""

    def __init__(self, model: Model):
        self.model = model
        self._h = C.c_void_p()
        rc = lib.antdt_create(C.byref(model), C.byref(self._h))
        if rc:
            raise AntdtError(rc, lib.antdt_last_error(None).decode())
        self._keep = {}
        self.workspace = None
        self.K = 0

    def close(self):
        if self._h:
            lib.antdt_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, rc: int):
        if rc:
            raise AntdtError(rc, lib.antdt_last_error(self._h).decode())

    def workspace_bytes(self) -> int:
        n = C.c_size_t()
        self._check(lib.antdt_workspace_bytes(self._h, C.byref(n)))
        return n.value

    def bind(self, tables, table_state, mlp_params, mlp_state, workspace=None):
        if workspace is None:
            workspace = torch.empty(self.workspace_bytes() + 256, dtype=torch.uint8, device=tables.device)
            pad = (-workspace.data_ptr()) % 256
            workspace = workspace[pad:pad + self.workspace_bytes()]
        self.workspace = workspace
        self._device = tables.device
        self._keep.update(tables=tables, table_state=table_state, mlp_params=mlp_params,
                          mlp_state=mlp_state, workspace=workspace)
        self._check(lib.antdt_bind(self._h, _ptr(tables), _ptr(table_state), _ptr(mlp_params),
                                   _ptr(mlp_state), _ptr(workspace), workspace.numel(), _stream()))

    def bind_static(self, tables, table_state, mlp_params, mlp_state):
        """antdt_bind_static: the library's static device buffer is the workspace (no allocation)."""
        self.workspace = None
        self._device = tables.device
        self._keep.update(tables=tables, table_state=table_state, mlp_params=mlp_params, mlp_state=mlp_state,
                          workspace=None)
        self._check(lib.antdt_bind_static(self._h, _ptr(tables), _ptr(table_state), _ptr(mlp_params),
                                          _ptr(mlp_state), _stream()))

    def set_batch(self, ids, field_ptr: Sequence[int], offsets, dense, labels):
        F = self.model.num_fields
        fp = (C.c_int64 * (F + 1))(*[int(v) for v in field_ptr])
        B = int(labels.numel())
        self._keep.update(ids=ids, offsets=offsets, dense=dense, labels=labels)
        self._check(lib.antdt_set_batch(self._h, _ptr(ids), fp, _ptr(offsets), _ptr(dense), _ptr(labels),
                                        B, _stream()))
        self.B = B
        self.field_ptr = [int(v) for v in field_ptr]

    def validate_batch(self):
        """Raises AntdtError(INVALID_ARG) when the batch has out-of-range ids or malformed offsets."""
        self._check(lib.antdt_validate_batch(self._h, _stream()))

    def assign_shard(self, B: int, K: int, sizes: Optional[Sequence[int]] = None,
                     speed: Optional[Sequence[float]] = None) -> List[Tuple[int, int]]:
        sz = (C.c_int64 * K)(*[int(v) for v in sizes]) if sizes is not None else None
        sp = (C.c_double * K)(*[float(v) for v in speed]) if speed is not None else None
        start, length = (C.c_int64 * K)(), (C.c_int64 * K)()
        self._check(lib.antdt_assign_shard(self._h, B, K, sz, sp, start, length))
        self.K = K
        self.shards = [(int(start[k]), int(length[k])) for k in range(K)]
        return self.shards

    def worker_step(self, k: int, loss_out: Optional[torch.Tensor] = None):
        self._check(lib.antdt_worker_step(self._h, k, _ptr(loss_out), _stream()))

    def worker_step_all(self, loss_out: Optional[torch.Tensor] = None):
        self._check(lib.antdt_worker_step_all(self._h, _ptr(loss_out), _stream()))

    def aggregate(self, shard_mask: Optional[Sequence[int]] = None):
        mk = (C.c_uint8 * len(shard_mask))(*[1 if v else 0 for v in shard_mask]) if shard_mask is not None else None
        self._check(lib.antdt_aggregate(self._h, mk, _stream()))

    def set_eager_weight_gradients(self, on: bool):
        self._check(lib.antdt_set_eager_weight_gradients(self._h, 1 if on else 0))

    def set_library_streams(self, on: bool):
        self._check(lib.antdt_set_library_streams(self._h, 1 if on else 0))

    def set_lr(self, lr: float):
        self._check(lib.antdt_set_lr(self._h, lr))

    def set_shard_scale(self, scale: Optional[Sequence[float]]):
        if scale is None:
            self._check(lib.antdt_set_shard_scale(self._h, None, 0))
        else:
            arr = (C.c_double * len(scale))(*[float(v) for v in scale])
            self._check(lib.antdt_set_shard_scale(self._h, arr, len(scale)))

    def apply_update(self):
        self._check(lib.antdt_apply_update(self._h, _stream()))

    # ------------------------------------------------------------- views
    def _ws_view(self, ptr: int, nbytes: int, dtype) -> torch.Tensor:
        if self.workspace is None:   # bound to the library's static buffer: wrap the raw device memory
            return torch.as_tensor(_RawDeviceBytes(ptr, nbytes), device=self._device).view(dtype)
        off = ptr - self.workspace.data_ptr()
        assert 0 <= off and off + nbytes <= self.workspace.numel(), "view outside the workspace"
        return self.workspace[off:off + nbytes].view(dtype)

    def view_pooled(self, k: int) -> torch.Tensor:
        x, rows, ld, dt = C.c_void_p(), C.c_int64(), C.c_int64(), C.c_int32()
        self._check(lib.antdt_view_pooled(self._h, k, C.byref(x), C.byref(rows), C.byref(ld), C.byref(dt)))
        if rows.value == 0:
            return torch.empty((0, ld.value), device=self._device)
        dtype, es = (torch.bfloat16, 2) if dt.value == BF16 else (torch.float32, 4)
        return self._ws_view(x.value, rows.value * ld.value * es, dtype).reshape(rows.value, ld.value)

    def view_shard_grads(self, k: int):
        d, dx, ld = C.c_void_p(), C.c_void_p(), C.c_int64()
        self._check(lib.antdt_view_shard_grads(self._h, k, C.byref(d), C.byref(dx), C.byref(ld)))
        P = sum(self.model.layer_sizes[i] * self.model.layer_sizes[i + 1] + self.model.layer_sizes[i + 1]
                for i in range(self.model.num_layers))
        dense = self._ws_view(d.value, P * 4, torch.float32)
        n = self.shards[k][1]
        gx = (self._ws_view(dx.value, n * ld.value * 4, torch.float32).reshape(n, ld.value) if n
              else torch.empty((0, ld.value), device=self._device))
        return dense, gx

    def view_dense_grad(self) -> torch.Tensor:
        g = C.c_void_p()
        self._check(lib.antdt_view_dense_grad(self._h, C.byref(g), _stream()))
        P = sum(self.model.layer_sizes[i] * self.model.layer_sizes[i + 1] + self.model.layer_sizes[i + 1]
                for i in range(self.model.num_layers))
        return self._ws_view(g.value, P * 4, torch.float32)

    def view_coalesced(self, f: int):
        u, so, ss, G = C.c_void_p(), C.c_void_p(), C.c_void_p(), C.c_void_p()
        nu, nnz = C.c_int64(), C.c_int64()
        self._check(lib.antdt_view_coalesced(self._h, f, C.byref(u), C.byref(so), C.byref(ss), C.byref(nu),
                                             C.byref(nnz), C.byref(G), _stream()))
        U, n, D = nu.value, nnz.value, self.model.dim
        dev = self._device
        uniq = self._ws_view(u.value, U * 4, torch.int32) if U else torch.empty(0, dtype=torch.int32, device=dev)
        segoff = self._ws_view(so.value, (U + 1) * 4, torch.int32)
        samples = self._ws_view(ss.value, n * 4, torch.int32) if n else torch.empty(0, dtype=torch.int32, device=dev)
        Gt = (self._ws_view(G.value, U * D * 4, torch.float32).reshape(U, D) if U
              else torch.empty((0, D), device=dev))
        return uniq, segoff, samples, Gt

    # ---------------------------------------------------------- profiling
    def profile(self, mode: int, kernel_id: int = -1):
        self._check(lib.antdt_profile(self._h, mode, kernel_id))

    def profile_overhead(self, n: int = 64) -> Tuple[float, float]:
        """(empty pair, pair around the smallest kernel): mean elapsed milliseconds."""
        e, t = C.c_double(), C.c_double()
        self._check(lib.antdt_profile_overhead(self._h, _stream(), n, C.byref(e), C.byref(t)))
        return e.value, t.value

    def profile_read(self, kernel_id: int) -> Tuple[int, float]:
        n, ms = C.c_int64(), C.c_double()
        self._check(lib.antdt_profile_read(self._h, kernel_id, C.byref(n), C.byref(ms)))
        return n.value, ms.value


def dense_aggregate_adam(p, m, v, grads: Sequence[torch.Tensor], weights: Sequence[float], lr, beta1, beta2,
                         eps, step: int):
    K = len(grads)
    gp = (C.c_void_p * K)(*[g.data_ptr() for g in grads])
    w = (C.c_float * K)(*[float(x) for x in weights])
    rc = lib.antdt_dense_aggregate_adam(_ptr(p), _ptr(m), _ptr(v), gp, w, K, p.numel(), lr, beta1, beta2, eps,
                                        step, _stream())
    if rc:
        raise AntdtError(rc, lib.antdt_last_error(None).decode())


def fill_tables(tables: torch.Tensor, num_fields: int, rows_per_field: int, dim: int, scale: float = 0.05):
    dt = BF16 if tables.dtype == torch.bfloat16 else F32
    rc = lib.antdt_fill_tables(_ptr(tables), dt, num_fields, rows_per_field, dim, scale, _stream())
    if rc:
        raise AntdtError(rc, lib.antdt_last_error(None).decode())


def stream_copy(dst: torch.Tensor, src: torch.Tensor):
    """dst[:] = src with the library's plain copy kernel (fp32, contiguous, same length)."""
    if dst.dtype != torch.float32 or src.dtype != torch.float32 or dst.numel() != src.numel():
        raise ValueError("stream_copy: two float32 tensors of one length")
    if not (dst.is_contiguous() and src.is_contiguous() and dst.is_cuda and src.is_cuda):
        raise ValueError("stream_copy: contiguous device tensors")
    rc = lib.antdt_stream_copy(_ptr(dst), _ptr(src), dst.numel(), _stream())
    if rc:
        raise AntdtError(rc, lib.antdt_last_error(None).decode())


def plan_accumulation(B: int, counts: Sequence[int], speeds: Sequence[float], bmin: Sequence[int],
                      bmax: Sequence[int], cmin: int, cmax: int):
    """Eq. 4 plan: returns (batch sizes B_i, accumulation counts C_i, optimum z), or None when
    no plan satisfies the constraints."""
    k = len(counts)
    Bo, Co, z = (C.c_int64 * k)(), (C.c_int32 * k)(), C.c_double()
    rc = lib.antdt_plan_accumulation(B, k, (C.c_int32 * k)(*counts), (C.c_double * k)(*speeds),
                                     (C.c_int64 * k)(*bmin), (C.c_int64 * k)(*bmax), cmin, cmax, Bo, Co,
                                     C.byref(z))
    if rc == INFEASIBLE:
        return None
    if rc:
        raise AntdtError(rc, lib.antdt_last_error(None).decode())
    return list(Bo), list(Co), z.value


def expand_accumulation(counts: Sequence[int], batch_sizes: Sequence[int], accum: Sequence[int]):
    """Shard sizes (and the device index of each shard) of a plan, for Context.assign_shard."""
    k = len(counts)
    cap = sum(int(n) * int(c) for n, c in zip(counts, accum))
    sizes, dev, cnt = (C.c_int64 * max(cap, 1))(), (C.c_int32 * max(cap, 1))(), C.c_int32()
    rc = lib.antdt_expand_accumulation(k, (C.c_int32 * k)(*counts), (C.c_int64 * k)(*batch_sizes),
                                       (C.c_int32 * k)(*accum), cap, sizes, dev, C.byref(cnt))
    if rc:
        raise AntdtError(rc, lib.antdt_last_error(None).decode())
    return list(sizes)[:cnt.value], list(dev)[:cnt.value]


EMPTY = -7
POLICY_BSP, POLICY_ADJUST_BS, POLICY_BACKUP_WORKERS, POLICY_ANTDT_ND = 0, 1, 2, 3


def _raise(rc: int):
    raise AntdtError(rc, lib.antdt_last_error(None).decode())


class ShardQueue:
    """The shard queue with states of Section V-C (see antdt_dds_* in antdt.h)."""

    def __init__(self, N: int, B: int, M: int):
        h = C.c_void_p()
        rc = lib.antdt_dds_create(N, B, M, C.byref(h))
        if rc:
            _raise(rc)
        self._h = h

    def __del__(self):
        if getattr(self, "_h", None):
            lib.antdt_dds_destroy(self._h)
            self._h = None

    def num_shards(self) -> int:
        k = C.c_int64()
        lib.antdt_dds_num_shards(self._h, C.byref(k))
        return k.value

    def fetch(self, worker: int):
        k, st, ln = C.c_int64(), C.c_int64(), C.c_int64()
        rc = lib.antdt_dds_fetch(self._h, worker, C.byref(k), C.byref(st), C.byref(ln))
        if rc == EMPTY:
            return None
        if rc:
            _raise(rc)
        return k.value, st.value, ln.value

    def report_done(self, shard: int, worker: int):
        rc = lib.antdt_dds_report_done(self._h, shard, worker)
        if rc:
            _raise(rc)

    def release_worker(self, worker: int) -> int:
        n = C.c_int64()
        rc = lib.antdt_dds_release_worker(self._h, worker, C.byref(n))
        if rc:
            _raise(rc)
        return n.value

    def shard(self, k: int):
        st, ln, state, owner = C.c_int64(), C.c_int64(), C.c_int32(), C.c_int32()
        rc = lib.antdt_dds_shard(self._h, k, C.byref(st), C.byref(ln), C.byref(state), C.byref(owner))
        if rc:
            _raise(rc)
        return st.value, ln.value, state.value, owner.value

    def counts(self):
        a, b, c = C.c_int64(), C.c_int64(), C.c_int64()
        lib.antdt_dds_counts(self._h, C.byref(a), C.byref(b), C.byref(c))
        return a.value, b.value, c.value


def simulate_bsp(n, B, N, t0, v, t_server=0.0, period=1800.0, duration=900.0, prob=0.0, sleep_duration=1.5,
                 intensity=0.0, seed=1, persistent_delay=None, policy=POLICY_BSP, backup_b=0, decide_every=300.0,
                 L_trans=300.0, L_per=600.0, lam=1.5, restart_cost=120.0, max_iterations=10_000_000):
    """Job completion time model (see antdt_simulate_bsp in antdt.h).  Returns (SimResult, final sizes)."""
    dbl = C.c_double * n
    cfg = SimConfig(n, B, N, dbl(*t0), dbl(*v), t_server, period, duration, prob, sleep_duration, intensity, seed,
                    dbl(*persistent_delay) if persistent_delay is not None else None, policy, backup_b,
                    decide_every, L_trans, L_per, lam, restart_cost, max_iterations)
    res, sizes = SimResult(), (C.c_int64 * n)()
    rc = lib.antdt_simulate_bsp(C.byref(cfg), C.byref(res), sizes)
    if rc:
        _raise(rc)
    return res, list(sizes)
