"""Helpers for the GPU parity tests: upload a workload, run the library through its
C boundary (via the ctypes binding) and fetch results for comparison with the oracle."""
from __future__ import annotations

import numpy as np
import torch

import paper_2404_09679_amd as A

DEV = "cuda:0"


def upload_tables(cfg, tables_np):
    if cfg.table_dtype == "bf16":
        return torch.from_numpy(tables_np.view(np.int16)).to(DEV).view(torch.bfloat16)
    return torch.from_numpy(tables_np).to(DEV)


def tables_to_f32(cfg, t):
    return t.float().cpu().numpy()


class GpuRun:
    """One model instance on the GPU with the tensors the library is bound to."""

    def __init__(self, cfg, tables_np, flat_params, state_np=None, flat_state=None, gemm_dtype=None,
                 max_batch=None, max_nnz=None, max_shards=None, static=False, eager=False, streams=True):
        self.cfg = cfg
        self.tables = upload_tables(cfg, tables_np)
        n_rows = cfg.num_fields * cfg.rows_per_field
        if state_np is None:
            shape = (n_rows, cfg.dim) if cfg.adagrad_state == "elementwise" else (n_rows,)
            self.state = torch.zeros(shape, dtype=torch.float32, device=DEV)
        else:
            self.state = torch.from_numpy(state_np).to(DEV)
        self.params = torch.from_numpy(flat_params.copy()).to(DEV)
        self.pstate = (torch.zeros_like(self.params) if flat_state is None
                       else torch.from_numpy(flat_state.copy()).to(DEV))
        self.model = A.model_from_config(cfg, max_batch=max_batch, max_nnz=max_nnz, max_shards=max_shards,
                                         gemm_dtype=gemm_dtype)
        self.ctx = A.Context(self.model)
        if not streams:   # every kernel on the caller's stream
            self.ctx.set_library_streams(False)
        if eager:    # every worker step computes its own weight gradients
            self.ctx.set_eager_weight_gradients(True)
        if static:   # the library's static device buffer is the workspace (antdt_bind_static)
            self.ctx.bind_static(self.tables, self.state, self.params, self.pstate)
        else:
            self.ctx.bind(self.tables, self.state, self.params, self.pstate)

    def set_batch(self, batch):
        self.batch = batch
        self.d_ids = torch.from_numpy(batch.ids).to(DEV)
        self.d_off = torch.from_numpy(batch.offsets).to(DEV)
        self.d_dense = torch.from_numpy(batch.dense).to(DEV) if self.cfg.num_dense else None
        self.d_labels = torch.from_numpy(batch.labels).to(DEV)
        self.ctx.set_batch(self.d_ids, batch.field_ptr, self.d_off, self.d_dense, self.d_labels)

    def iteration(self, sizes, batched=False, mask=None, update=True, scale=None, scale_late=False):
        """`scale`: per-worker factors, set before the worker steps or (`scale_late`) after them."""
        K = len(sizes)
        self.ctx.assign_shard(self.batch.batch, K, sizes=sizes)
        if not scale_late:
            self.ctx.set_shard_scale(scale)
        self.loss = torch.zeros(K, dtype=torch.float32, device=DEV)
        if batched:
            self.ctx.worker_step_all(self.loss)
        else:
            for k in range(K):
                if mask is None or mask[k]:
                    self.ctx.worker_step(k, self.loss[k:k + 1])
        torch.cuda.synchronize()
        self.shard_out = []
        for k in range(K):
            x = self.ctx.view_pooled(k).float().cpu().numpy()
            dense, dx = self.ctx.view_shard_grads(k)
            self.shard_out.append((x, dense.cpu().numpy().copy(), dx.cpu().numpy().copy()))
        if scale_late:
            self.ctx.set_shard_scale(scale)
        self.ctx.aggregate(mask)
        torch.cuda.synchronize()
        self.g_dense = self.ctx.view_dense_grad().cpu().numpy().copy()
        self.coalesced = []
        for f in range(self.cfg.num_fields):
            u, so, ss, G = self.ctx.view_coalesced(f)
            self.coalesced.append((u.cpu().numpy().copy(), so.cpu().numpy().copy(), ss.cpu().numpy().copy(),
                                   G.cpu().numpy().copy()))
        if update:
            self.ctx.apply_update()
            torch.cuda.synchronize()
        return self
