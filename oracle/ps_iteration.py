"""Float64 statement of one BSP Parameter-Server iteration of a ranking model.

Test infrastructure: see the package docstring.  All arithmetic is float64;
inputs arrive as the float32 / bf16 values the caller stores and results that
are *stored* (updated parameters and optimizer state) are rounded once to the
storage type.

Worker side (Section II, problem formulation: each worker computes a gradient on
its own local batch B_i and pushes it to the servers): sum-pooled embedding bags, an MLP with ReLU
hidden layers and one logit, mean binary cross-entropy over the shard.
Server side (Section II: the servers combine the gradients pushed by all workers
and then update the parameters): gradients of the included shards are
averaged with weights B_k / sum B_k (the only weights that keep the update
independent of how the fixed global batch is split, cf. the constraint
sum_i B_i = B of Eq. 1), duplicate row ids are coalesced, and Adagrad is
applied to the touched rows and to the dense parameters.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np


@dataclass(frozen=True)
class Model:
    num_fields: int
    rows_per_field: int
    dim: int
    num_dense: int
    layer_sizes: Tuple[int, ...]      # (input, hidden..., 1)
    rowwise_state: bool = False       # one Adagrad accumulator per row instead of per element
    bf16_tables: bool = False         # stored rows are bf16 (write-back rounds to nearest even)
    bf16_gemm: bool = False           # GEMM operands are bf16 values, accumulation exact here
    lr: float = 0.01
    eps: float = 1e-8
    mean_pool: bool = False           # bags are averaged instead of summed (empty bag: zeros)


def round_bf16(x) -> np.ndarray:
    """Nearest-even bfloat16 value of x (via float32, as a float32 producer would), as float64."""
    x32 = np.asarray(x, dtype=np.float64).astype(np.float32)
    b = np.ascontiguousarray(x32).view(np.uint32)
    lsb = (b >> np.uint32(16)) & np.uint32(1)
    with np.errstate(over="ignore"):
        r = (b + np.uint32(0x7FFF) + lsb) & np.uint32(0xFFFF0000)
    return r.view(np.float32).astype(np.float64).reshape(np.shape(x))


# --------------------------------------------------------------------------
# worker side
# --------------------------------------------------------------------------
def embedding_pool(table_f: np.ndarray, ids_f: np.ndarray, offsets_f: np.ndarray,
                   start: int, length: int, mean: bool = False) -> np.ndarray:
    """Pool the bags of samples [start, start+length) of one field.

    out[s, :] = sum over the lookups j of bag s, left to right, of table_f[ids_f[j], :];
    with `mean` the sum is divided by the number of lookups of the bag.
    A duplicate id inside a bag counts twice; an empty bag gives zeros.
    """
    D = table_f.shape[1]
    out = np.zeros((length, D), dtype=np.float64)
    off = np.asarray(offsets_f[start:start + length + 1], dtype=np.int64)
    lens = np.diff(off)
    sample = np.repeat(np.arange(length), lens)
    rows = np.asarray(table_f[np.asarray(ids_f[off[0]:off[-1]], dtype=np.int64)], dtype=np.float64)
    np.add.at(out, sample, rows)
    if mean:
        out = out / np.maximum(lens, 1)[:, None]
    return out


def embedding_pool_loops(table_f, ids_f, offsets_f, start, length, mean=False) -> np.ndarray:
    """The same definition as `embedding_pool`, as explicit loops (tiny inputs only)."""
    D = table_f.shape[1]
    out = np.zeros((length, D), dtype=np.float64)
    for s in range(length):
        lo, hi = int(offsets_f[start + s]), int(offsets_f[start + s + 1])
        for j in range(lo, hi):
            for d in range(D):
                out[s, d] += float(table_f[int(ids_f[j]), d])
        if mean and hi > lo:
            for d in range(D):
                out[s, d] /= (hi - lo)
    return out


def mlp_forward(x: np.ndarray, layers: Sequence[Tuple[np.ndarray, np.ndarray]],
                bf16_gemm: bool = False):
    """h_0 = x; h_l = ReLU(h_{l-1} W_l + b_l) for hidden layers; the last layer is linear.

    With bf16_gemm the operands of every hidden-layer product (the stored
    activation and the weight) are bf16 values; the single-logit last layer
    is a dot product taken on the stored activation with unrounded weights.
    Returns (activations [h_0 .. h_{L-1}] as fed to the next product, logits z).
    """
    rd = round_bf16 if bf16_gemm else (lambda a: np.asarray(a, dtype=np.float64))
    acts = [rd(x)]
    L = len(layers)
    for l, (W, b) in enumerate(layers):
        W64, b64 = np.asarray(W, np.float64), np.asarray(b, np.float64)
        if l < L - 1:
            acts.append(rd(np.maximum(acts[-1] @ rd(W64) + b64, 0.0)))
        else:
            z = acts[-1] @ W64 + b64
    return acts, z[:, 0]


def bce_with_logits(z: np.ndarray, y: np.ndarray) -> np.ndarray:
    """Per-sample -[y log s(z) + (1-y) log(1-s(z))] in its overflow-free form."""
    return np.maximum(z, 0.0) - z * y + np.log1p(np.exp(-np.abs(z)))


@dataclass
class ShardResult:
    start: int
    length: int
    x: np.ndarray                    # [B_k, F*D + num_dense] pooled embeddings then dense features
    z: np.ndarray                    # [B_k] logits
    loss: float                      # mean BCE over the shard (0 for an empty shard)
    dW: List[np.ndarray]             # per layer [in, out]
    db: List[np.ndarray]             # per layer [out]
    dx: np.ndarray                   # [B_k, F*D] gradient w.r.t. the pooled embeddings
    acts: List[np.ndarray] = field(default_factory=list)


def worker_step(model: Model, tables: Sequence[np.ndarray], layers, batch,
                start: int, length: int) -> ShardResult:
    """Local gradient of one worker on its shard = samples [start, start+length).

    tables[f] is the [R, D] table of field f; layers = [(W_l [in,out], b_l)].
    The loss is the *mean* over the shard's B_k samples, so every gradient
    returned is a per-shard mean; the server re-weights by B_k / B.
    """
    F, D, nd = model.num_fields, model.dim, model.num_dense
    x = np.zeros((length, F * D + nd), dtype=np.float64)
    for f in range(F):
        x[:, f * D:(f + 1) * D] = embedding_pool(tables[f], batch.field_ids(f), batch.offsets[f],
                                                 start, length, model.mean_pool)
    if nd:
        x[:, F * D:] = np.asarray(batch.dense[start:start + length], dtype=np.float64)
    y = np.asarray(batch.labels[start:start + length], dtype=np.float64)
    L = len(layers)
    if length == 0:
        return ShardResult(start, 0, x, np.zeros(0), 0.0,
                           [np.zeros(np.shape(W)) for W, _ in layers],
                           [np.zeros(np.shape(b)) for _, b in layers], np.zeros((0, F * D)), [])
    rd = round_bf16 if model.bf16_gemm else (lambda a: np.asarray(a, dtype=np.float64))
    acts, z = mlp_forward(x, layers, model.bf16_gemm)
    loss = float(np.mean(bce_with_logits(z, y)))
    dz = (1.0 / (1.0 + np.exp(-z)) - y) / length              # d(mean loss)/dz
    dW = [None] * L
    db = [None] * L
    W_last = np.asarray(layers[-1][0], np.float64)
    dW[L - 1] = acts[L - 1].T @ dz[:, None]
    db[L - 1] = np.array([dz.sum()])
    dh = dz[:, None] @ W_last.T                               # [B_k, width_{L-1}]
    for l in range(L - 2, -1, -1):
        dh = rd(dh * (acts[l + 1] > 0.0))                     # through the ReLU of layer l
        dW[l] = acts[l].T @ dh
        db[l] = dh.sum(axis=0)
        dh = dh @ rd(np.asarray(layers[l][0], np.float64)).T
    return ShardResult(start, length, x, z, loss, dW, db, dh[:, :F * D], acts)


# --------------------------------------------------------------------------
# server side
# --------------------------------------------------------------------------
def shard_weights(lengths: Sequence[int], mask: Optional[Sequence[bool]] = None,
                  scale: Optional[Sequence[float]] = None) -> np.ndarray:
    """w_k = c_k * B_k / sum of the included B_k (0 for an excluded shard).

    c_k (default 1) is a per-worker factor on that worker's contribution: the per-worker
    learning-rate adjustment of the optimization-based methods of Section III (Table II,
    ADJUST_LR) seen from the server, which applies one update with one learning rate.
    """
    n = np.asarray(lengths, dtype=np.float64)
    inc = np.ones(len(n), bool) if mask is None else np.asarray(mask, dtype=bool)
    tot = float(n[inc].sum())
    w = np.where(inc, n / tot, 0.0) if tot > 0 else np.zeros(len(n))
    if scale is not None:
        w = w * np.asarray(scale, dtype=np.float64)
    return w


@dataclass
class Aggregated:
    weights: np.ndarray
    dW: List[np.ndarray]
    db: List[np.ndarray]
    unique_ids: List[np.ndarray]      # per field, ascending distinct row ids (int64)
    seg_offsets: List[np.ndarray]     # per field, [U_f+1]: #lookups with id < unique_ids[u]; last = nnz_f
    G: List[np.ndarray]               # per field [U_f, D] coalesced weighted gradient rows
    seg_samples: List[List[List[int]]]  # per field, per segment: ascending global sample index of each lookup
    loss: float                       # sum_k w_k loss_k


def aggregate(model: Model, batch, results: Sequence[ShardResult],
              mask: Optional[Sequence[bool]] = None, want_samples: bool = False,
              scale: Optional[Sequence[float]] = None) -> Aggregated:
    """Server-side aggregation of the included shards' pushed gradients.

    Dense: g = sum_k w_k g_k.  Sparse, per field, by direct addressing (no
    sort): count[r] = lookups of row r among the included shards; the rows with
    count > 0 in ascending order are the unique ids, the running sum of their
    counts the segment offsets, and every lookup j of sample s adds
    w_k * dx_k[s, field slice] into its row, walking samples in global order
    (divided by the bag's length when the bags are mean-pooled).
    """
    F, D, R = model.num_fields, model.dim, model.rows_per_field
    K = len(results)
    inc = np.ones(K, bool) if mask is None else np.asarray(mask, dtype=bool)
    w = shard_weights([r.length for r in results], inc, scale)
    L = len(results[0].dW)
    dW = [sum(w[k] * results[k].dW[l] for k in range(K)) for l in range(L)]
    db = [sum(w[k] * results[k].db[l] for k in range(K)) for l in range(L)]
    loss = float(sum(w[k] * results[k].loss for k in range(K)))
    uniq, segs, Gs, samples = [], [], [], []
    for f in range(F):
        ids_f = np.asarray(batch.field_ids(f), dtype=np.int64)
        off = np.asarray(batch.offsets[f], dtype=np.int64)
        count = np.zeros(R, dtype=np.int64)
        for k, r in enumerate(results):
            if inc[k] and r.length:
                np.add.at(count, ids_f[off[r.start]:off[r.start + r.length]], 1)
        u_ids = np.nonzero(count)[0]
        seg = np.zeros(len(u_ids) + 1, dtype=np.int64)
        np.cumsum(count[u_ids], out=seg[1:])
        pos = np.full(R, -1, dtype=np.int64)
        pos[u_ids] = np.arange(len(u_ids))
        G = np.zeros((len(u_ids), D), dtype=np.float64)
        seg_s: List[List[int]] = [[] for _ in range(len(u_ids))] if want_samples else []
        for k, r in enumerate(results):
            if not inc[k] or r.length == 0:
                continue
            lo, hi = off[r.start], off[r.start + r.length]
            lens = np.diff(off[r.start:r.start + r.length + 1])
            local = np.repeat(np.arange(r.length), lens)
            rows = w[k] * r.dx[local, f * D:(f + 1) * D]
            if model.mean_pool:                 # d(mean of the bag)/d(row) = 1 / bag length
                rows = rows / np.repeat(lens, lens)[:, None]
            np.add.at(G, pos[ids_f[lo:hi]], rows)
            if want_samples:
                for j, s in zip(ids_f[lo:hi], local):
                    seg_s[pos[j]].append(int(r.start + s))
        uniq.append(u_ids)
        segs.append(seg)
        Gs.append(G)
        samples.append(seg_s)
    return Aggregated(w, dW, db, uniq, segs, Gs, samples, loss)


def coalesce_loops(ids: Sequence[int], rows: np.ndarray):
    """Brute-force coalescing of (id, row) pairs with an ordered dictionary (tiny inputs)."""
    acc: Dict[int, np.ndarray] = {}
    cnt: Dict[int, int] = {}
    for j, i in enumerate(ids):
        i = int(i)
        if i not in acc:
            acc[i] = np.zeros(rows.shape[1], dtype=np.float64)
            cnt[i] = 0
        acc[i] = acc[i] + np.asarray(rows[j], dtype=np.float64)
        cnt[i] += 1
    keys = sorted(acc)
    seg = [0]
    for k in keys:
        seg.append(seg[-1] + cnt[k])
    G = np.array([acc[k] for k in keys]).reshape(len(keys), rows.shape[1])
    return np.array(keys, dtype=np.int64), np.array(seg, dtype=np.int64), G


def adagrad_elementwise(p, s, g, lr, eps):
    """s' = s + g^2;  p' = p - lr * g / (sqrt(s') + eps), element by element."""
    p, s, g = (np.asarray(a, dtype=np.float64) for a in (p, s, g))
    s1 = s + g * g
    return p - lr * g / (np.sqrt(s1) + eps), s1


def adagrad_rowwise(p, s, g, lr, eps):
    """One accumulator per row: s'[r] = s[r] + mean_d g[r,d]^2;  p' = p - lr*g/(sqrt(s'[r]) + eps)."""
    p, s, g = (np.asarray(a, dtype=np.float64) for a in (p, s, g))
    s1 = s + (g * g).mean(axis=1)
    return p - lr * g / (np.sqrt(s1)[:, None] + eps), s1


@dataclass
class Updated:
    rows: List[np.ndarray]        # per field [U_f, D]: new values of the touched rows, as stored
    row_state: List[np.ndarray]   # per field [U_f, D] or [U_f]: new accumulators (float32 values)
    layers: List[Tuple[np.ndarray, np.ndarray]]        # new MLP parameters (float32 values)
    layer_state: List[Tuple[np.ndarray, np.ndarray]]   # new MLP accumulators (float32 values)


def apply_update(model: Model, tables, table_state, layers, layer_state, agg: Aggregated) -> Updated:
    """Adagrad on the rows listed in agg.unique_ids and on every dense parameter.

    table_state[f] is [R, D] (element-wise) or [R] (row-wise).  Rows that are
    not listed are not read and not returned: they do not change.  Stored
    results are rounded once: parameters to float32 (bf16 tables to the
    nearest-even bf16), accumulators to float32.
    """
    f32 = lambda a: np.asarray(a, dtype=np.float64).astype(np.float32).astype(np.float64)
    rows, rstate = [], []
    for f in range(model.num_fields):
        u = agg.unique_ids[f]
        p0 = np.asarray(tables[f][u], dtype=np.float64)
        s0 = np.asarray(table_state[f][u], dtype=np.float64)
        if model.rowwise_state:
            p1, s1 = adagrad_rowwise(p0, s0, agg.G[f], model.lr, model.eps)
        else:
            p1, s1 = adagrad_elementwise(p0, s0, agg.G[f], model.lr, model.eps)
        rows.append(round_bf16(p1) if model.bf16_tables else f32(p1))
        rstate.append(f32(s1))
    new_layers, new_state = [], []
    for l, (W, b) in enumerate(layers):
        sW, sb = layer_state[l]
        W1, sW1 = adagrad_elementwise(W, sW, agg.dW[l], model.lr, model.eps)
        b1, sb1 = adagrad_elementwise(b, sb, agg.db[l], model.lr, model.eps)
        new_layers.append((f32(W1), f32(b1)))
        new_state.append((f32(sW1), f32(sb1)))
    return Updated(rows, rstate, new_layers, new_state)
