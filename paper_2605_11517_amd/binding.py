"""ctypes binding of ``include/gnnmi.h``: same entry points, argument marshalling only.

``Context`` wraps a ``gnn_ctx*`` and exposes one method per C entry point with the same name
minus the ``gnn_`` prefix.  ``Session`` is a convenience that allocates the device buffers
with torch (torch is used for device memory and streams only) and binds them.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

GNN_GCN, GNN_SAGE_MEAN, GNN_GAT = 0, 1, 2
GNN_F32, GNN_BF16 = 0, 1
GNN_PART_USER, GNN_PART_RANDOM, GNN_PART_LP, GNN_PART_SWITCHING = 0, 1, 2, 3
GNN_PART_SWITCHING_DEVICE = 4
KERNEL_CLASSES = ("gather", "spmm", "gemm_fwd", "loss", "act_bwd", "gemm_dw", "gemm_dz",
                  "spmm_t", "scatter", "other", "spmm_reduce")
STATUS = {0: "GNN_OK", 1: "GNN_EINVAL", 2: "GNN_ENOMEM", 3: "GNN_EHIP", 4: "GNN_ESTATE",
          5: "GNN_EUNSUPPORTED"}
_MODEL = {"gcn": GNN_GCN, "sage": GNN_SAGE_MEAN, "gat": GNN_GAT}
_PART = {"user": GNN_PART_USER, "random": GNN_PART_RANDOM, "lp": GNN_PART_LP,
         "switching": GNN_PART_SWITCHING, "switching_device": GNN_PART_SWITCHING_DEVICE}

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libgnnmi.so")
_lib = None


class GnnError(RuntimeError):
    def __init__(self, status, message):
        super().__init__("%s: %s" % (STATUS.get(status, status), message))
        self.status = status


class _Config(C.Structure):
    _fields_ = [("model", C.c_int32), ("dtype", C.c_int32), ("n_layers", C.c_int32),
                ("dims", C.POINTER(C.c_int32)), ("has_bias", C.c_int32),
                ("hbm_budget_bytes", C.c_int64)]


class _Stats(C.Structure):
    _fields_ = [("n", C.c_int64), ("nnz", C.c_int64), ("k", C.c_int32),
                ("sum_boundary", C.c_int64), ("sum_required", C.c_int64),
                ("max_own", C.c_int64), ("max_boundary", C.c_int64), ("max_nnz", C.c_int64)]


class Optimizer(C.Structure):
    _fields_ = [("kind", C.c_int32), ("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float),
                ("eps", C.c_float), ("weight_decay", C.c_float)]


def make_optimizer(kind="adam", lr=0.01, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0):
    return Optimizer({"sgd": 0, "adam": 1}[kind], lr, beta1, beta2, eps, weight_decay)


class StorageStats(C.Structure):
    _fields_ = [(n_, C.c_int64) for n_ in ("host_pool_bytes", "array_bytes", "loads", "hits", "prefetched",
                                           "evictions", "writebacks", "bytes_read", "bytes_written", "compactions", "dropped", "bypassed", "bypass_bytes")]


class StreamStats(C.Structure):
    _fields_ = [(f, C.c_int64) for f in ("act_loads", "act_hits", "grad_loads", "grad_hits",
                                         "grad_writebacks", "h2d_bytes", "d2h_bytes",
                                         "direct_gathers", "direct_bytes", "direct_scatters",
                                         "direct_scatter_bytes")]


def load_library():
    """Loads ``libgnnmi.so`` from the package directory (build it with
    ``python -m paper_2605_11517_amd.build``).  Raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            "%s not found: build the HIP library first (python -m paper_2605_11517_amd.build)"
            % LIB_PATH)
    lib = C.CDLL(LIB_PATH)
    vp, i32, i64, u64 = C.c_void_p, C.c_int32, C.c_int64, C.c_uint64
    P = C.POINTER
    sig = {
        "gnn_create": [P(_Config), P(vp)],
        "gnn_build_partitions": [vp, i64, P(i64), P(i32), i32, i32, u64, P(i32)],
        "gnn_get_partition": [vp, P(P(i32)), P(i32)],
        "gnn_get_order": [vp, P(P(i32)), P(P(i64))],
        "gnn_get_boundary": [vp, i32, P(P(i32)), P(i64)],
        "gnn_get_stats": [vp, P(_Stats)],
        "gnn_get_schedule": [vp, P(P(i32))],
        "gnn_workspace_bytes": [vp, P(i64), P(i64)],
        "gnn_bind": [vp, vp, P(vp), P(vp), P(vp), P(vp), vp, vp, vp, vp],
        "gnn_permute_rows": [vp, vp, vp, i64, i32, vp],
        "gnn_to_bf16": [vp, vp, vp, i64, vp],
        "gnn_gather_boundary": [vp, i32, i32, vp],
        "gnn_set_gather_fusion": [vp, i32],
        "gnn_gather_is_fused": [vp, P(i32)],
        "gnn_set_masked_backward": [vp, i32],
        "gnn_get_masked_backward_size": [vp, P(i64), P(i64)],
        "gnn_layer_fwd": [vp, i32, i32, vp],
        "gnn_loss": [vp, vp],
        "gnn_loss_static": [vp, vp, vp],
        "gnn_read_loss": [vp, vp, P(C.c_float)],
        "gnn_layer_bwd": [vp, i32, i32, vp],
        "gnn_epoch": [vp, vp, P(C.c_float)],
        "gnn_set_layer_order": [vp, i32],
        "gnn_set_gat_heads": [vp, i32, i32],
        "gnn_set_keep_forward": [vp, i32],
        "gnn_layer_is_transform_first": [vp, i32, P(i32)],
        "gnn_layer_transform_fwd": [vp, i32, i32, vp],
        "gnn_layer_transform_bwd": [vp, i32, i32, vp],
        "gnn_set_dropout": [vp, C.c_float, u64, i64],
        "gnn_bind_optimizer": [vp, P(vp), P(vp)],
        "gnn_bind_master_weights": [vp, P(vp)],
        "gnn_optimizer_step": [vp, P(Optimizer), i64, vp],
        "gnn_train": [vp, P(Optimizer), i32, i64, C.c_float, u64, vp, P(C.c_float)],
        "gnn_set_profiling": [vp, i32],
        "gnn_get_profile": [vp, P(C.c_double), P(i64)],
        "gnn_get_stream_stats": [vp, P(StreamStats)],
        "gnn_storage_open": [vp, C.c_char_p, i64],
        "gnn_storage_close": [vp],
        "gnn_storage_keep_results": [vp, i32],
        "gnn_storage_write": [vp, i32, i32, vp],
        "gnn_storage_read": [vp, i32, i32, vp],
        "gnn_get_storage_stats": [vp, P(StorageStats)],
        "gnn_get_partitioner_history": [vp, P(i32), P(C.c_double), i32],
    }
    for name, args in sig.items():
        fn = getattr(lib, name)
        fn.argtypes = args
        fn.restype = C.c_int
    lib.gnn_destroy.argtypes = [vp]
    lib.gnn_destroy.restype = None
    lib.gnn_last_error.argtypes = [vp]
    lib.gnn_last_error.restype = C.c_char_p
    _lib = lib
    return lib


def _np_ptr(a, t):
    return a.ctypes.data_as(C.POINTER(t))


class Context:
    """Owns one ``gnn_ctx``.  Methods mirror the C entry points and raise ``GnnError``."""

    def __init__(self, model, dims, dtype=GNN_F32, has_bias=True, hbm_budget_bytes=0):
        self.lib = load_library()
        self.model = _MODEL.get(model, model)
        self.dims = [int(d) for d in dims]
        self.L = len(self.dims) - 1
        arr = (C.c_int32 * len(self.dims))(*self.dims)
        cfg = _Config(self.model, dtype, self.L, arr, 1 if has_bias else 0, hbm_budget_bytes)
        h = C.c_void_p()
        st = self.lib.gnn_create(C.byref(cfg), C.byref(h))
        if st != 0:
            raise GnnError(st, self.lib.gnn_last_error(None).decode())
        self.h = h
        self._keep = []

    def _check(self, st):
        if st != 0:
            raise GnnError(st, self.lib.gnn_last_error(self.h).decode())

    def destroy(self):
        if getattr(self, "h", None):
            self.lib.gnn_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    # -- partitions (host) ------------------------------------------------------------------
    def build_partitions(self, rowptr, colidx, k, mode="random", seed=0, user_part=None):
        rowptr = np.ascontiguousarray(rowptr, dtype=np.int64)
        colidx = np.ascontiguousarray(colidx, dtype=np.int32)
        n = len(rowptr) - 1
        up = None
        if user_part is not None:
            up = np.ascontiguousarray(user_part, dtype=np.int32)
        self._check(self.lib.gnn_build_partitions(
            self.h, n, _np_ptr(rowptr, C.c_int64), _np_ptr(colidx, C.c_int32), int(k),
            _PART.get(mode, mode), C.c_uint64(seed & (2 ** 64 - 1)),
            _np_ptr(up, C.c_int32) if up is not None else None))
        self.n = n
        self.k = int(k)

    def get_partition(self):
        p = C.POINTER(C.c_int32)()
        k = C.c_int32()
        self._check(self.lib.gnn_get_partition(self.h, C.byref(p), C.byref(k)))
        return np.ctypeslib.as_array(p, shape=(self.n,)).copy(), int(k.value)

    def get_order(self):
        o = C.POINTER(C.c_int32)()
        off = C.POINTER(C.c_int64)()
        self._check(self.lib.gnn_get_order(self.h, C.byref(o), C.byref(off)))
        return (np.ctypeslib.as_array(o, shape=(self.n,)).copy(),
                np.ctypeslib.as_array(off, shape=(self.k + 1,)).copy())

    def get_boundary(self, p):
        idx = C.POINTER(C.c_int32)()
        cnt = C.c_int64()
        self._check(self.lib.gnn_get_boundary(self.h, int(p), C.byref(idx), C.byref(cnt)))
        if cnt.value == 0:
            return np.zeros(0, dtype=np.int32)
        return np.ctypeslib.as_array(idx, shape=(cnt.value,)).copy()

    def get_stats(self):
        s = _Stats()
        self._check(self.lib.gnn_get_stats(self.h, C.byref(s)))
        return {f: getattr(s, f) for f, _ in _Stats._fields_}

    def get_schedule(self):
        ptr = C.POINTER(C.c_int32)()
        self._check(self.lib.gnn_get_schedule(self.h, C.byref(ptr)))
        _, k = self.get_partition()
        return np.ctypeslib.as_array(ptr, shape=(k,)).copy()

    def get_partitioner_history(self):
        it = C.c_int32()
        obj = (C.c_double * 64)()
        self._check(self.lib.gnn_get_partitioner_history(self.h, C.byref(it), obj, 64))
        return int(it.value), [float(obj[i]) for i in range(min(it.value + 1, 64))]

    def workspace_bytes(self):
        a, b = C.c_int64(), C.c_int64()
        self._check(self.lib.gnn_workspace_bytes(self.h, C.byref(a), C.byref(b)))
        return int(a.value), int(b.value)

    # -- device side (pointers are raw device addresses, stream a raw hipStream_t) ------------
    def bind(self, feat, act, grad_act, weights, grad_w, labels, train_mask, staging, scratch):
        def arr(ptrs):
            a = (C.c_void_p * max(1, len(ptrs)))()
            for i, p in enumerate(ptrs):
                a[i] = p
            return a
        self._check(self.lib.gnn_bind(self.h, feat, arr(act), arr(grad_act), arr(weights),
                                      arr(grad_w), labels, train_mask, staging, scratch))

    def permute_rows(self, src, dst, row_bytes, to_library_order, stream):
        self._check(self.lib.gnn_permute_rows(self.h, src, dst, int(row_bytes),
                                              1 if to_library_order else 0, stream))

    def to_bf16(self, src, dst, count, stream):
        self._check(self.lib.gnn_to_bf16(self.h, src, dst, int(count), stream))

    def gather_boundary(self, layer, p, stream):
        self._check(self.lib.gnn_gather_boundary(self.h, int(layer), int(p), stream))

    def set_gather_fusion(self, on):
        self._check(self.lib.gnn_set_gather_fusion(self.h, 1 if on else 0))

    def set_masked_backward(self, on):
        self._check(self.lib.gnn_set_masked_backward(self.h, 1 if on else 0))

    def masked_backward_size(self):
        """(operator entries, result rows) of the train-vertex operator; (0, 0) when not in use."""
        e, r = C.c_int64(), C.c_int64()
        self._check(self.lib.gnn_get_masked_backward_size(self.h, C.byref(e), C.byref(r)))
        return int(e.value), int(r.value)

    def gather_is_fused(self):
        out = C.c_int32()
        self._check(self.lib.gnn_gather_is_fused(self.h, C.byref(out)))
        return bool(out.value)

    def layer_fwd(self, layer, p, stream):
        self._check(self.lib.gnn_layer_fwd(self.h, int(layer), int(p), stream))

    def loss(self, stream):
        self._check(self.lib.gnn_loss(self.h, stream))

    def loss_static(self, stream, loss_dev):
        self._check(self.lib.gnn_loss_static(self.h, stream, loss_dev))

    def read_loss(self, stream):
        v = C.c_float()
        self._check(self.lib.gnn_read_loss(self.h, stream, C.byref(v)))
        return float(v.value)

    def layer_bwd(self, layer, p, stream):
        self._check(self.lib.gnn_layer_bwd(self.h, int(layer), int(p), stream))

    def epoch(self, stream):
        v = C.c_float()
        self._check(self.lib.gnn_epoch(self.h, stream, C.byref(v)))
        return float(v.value)

    def set_layer_order(self, mode):
        self._check(self.lib.gnn_set_layer_order(self.h, {"aggregate": 0, "auto": 1}[mode]))

    def set_gat_heads(self, layer, heads):
        self._check(self.lib.gnn_set_gat_heads(self.h, int(layer), int(heads)))

    def set_keep_forward(self, on):
        self._check(self.lib.gnn_set_keep_forward(self.h, 1 if on else 0))

    def layer_is_transform_first(self, layer):
        out = C.c_int32()
        self._check(self.lib.gnn_layer_is_transform_first(self.h, layer, C.byref(out)))
        return bool(out.value)

    def layer_transform_fwd(self, layer, p, stream):
        self._check(self.lib.gnn_layer_transform_fwd(self.h, layer, p, stream))

    def layer_transform_bwd(self, layer, p, stream):
        self._check(self.lib.gnn_layer_transform_bwd(self.h, layer, p, stream))

    def set_dropout(self, p, seed, epoch_index):
        self._check(self.lib.gnn_set_dropout(self.h, float(p), int(seed), int(epoch_index)))

    def bind_optimizer(self, m, v):
        def arr(ptrs):
            a = (C.c_void_p * max(1, len(ptrs)))()
            for i, p in enumerate(ptrs):
                a[i] = p
            return a
        self._check(self.lib.gnn_bind_optimizer(self.h, arr(m), arr(v)))

    def bind_master_weights(self, master):
        a = (C.c_void_p * max(1, len(master)))()
        for i, p in enumerate(master):
            a[i] = p
        self._check(self.lib.gnn_bind_master_weights(self.h, a))

    def optimizer_step(self, opt, step, stream):
        self._check(self.lib.gnn_optimizer_step(self.h, C.byref(opt), int(step), stream))

    def train(self, opt, epochs, first_epoch, dropout_p, dropout_seed, stream):
        losses = (C.c_float * max(1, epochs))()
        self._check(self.lib.gnn_train(self.h, C.byref(opt), int(epochs), int(first_epoch),
                                       float(dropout_p), int(dropout_seed), stream, losses))
        return [float(losses[i]) for i in range(epochs)]

    def set_profiling(self, enabled):
        """False/0 off, True/1 every kernel class, 2 the aggregation kernels only."""
        self._check(self.lib.gnn_set_profiling(self.h, int(enabled)))

    def storage_open(self, directory, host_budget_bytes):
        self._check(self.lib.gnn_storage_open(self.h, os.fsencode(directory), int(host_budget_bytes)))

    def storage_keep_results(self, on):
        self._check(self.lib.gnn_storage_keep_results(self.h, 1 if on else 0))

    def storage_close(self):
        self._check(self.lib.gnn_storage_close(self.h))

    def storage_write(self, kind, layer, src_ptr):
        self._check(self.lib.gnn_storage_write(self.h, int(kind), int(layer), src_ptr))

    def storage_read(self, kind, layer, dst_ptr):
        self._check(self.lib.gnn_storage_read(self.h, int(kind), int(layer), dst_ptr))

    def get_storage_stats(self):
        st = StorageStats()
        self._check(self.lib.gnn_get_storage_stats(self.h, C.byref(st)))
        return {name: int(getattr(st, name)) for name, _ in StorageStats._fields_}

    def get_stream_stats(self):
        st = StreamStats()
        self._check(self.lib.gnn_get_stream_stats(self.h, C.byref(st)))
        return {name: int(getattr(st, name)) for name, _ in StreamStats._fields_}

    def get_profile(self):
        ms = (C.c_double * len(KERNEL_CLASSES))()
        ln = (C.c_int64 * len(KERNEL_CLASSES))()
        self._check(self.lib.gnn_get_profile(self.h, ms, ln))
        return {name: (float(ms[i]), int(ln[i])) for i, name in enumerate(KERNEL_CLASSES)}


class Session:
    """Allocates every device buffer of one model on ``cuda:0`` with torch, converts the
    caller's original-order host arrays to library order with ``gnn_permute_rows`` and binds
    them.  Results are read back in original vertex order."""

    def __init__(self, model, dims, rowptr, colidx, k, part_mode, seed, X, weights, labels,
                 train_mask, has_bias=True, user_part=None, device="cuda:0", dtype="f32",
                 hbm_budget_bytes=0, layer_order="aggregate", fuse_gather=False, masked_backward=False,
                 storage_dir=None, host_budget_bytes=0, progress=None, keep_forward=False):
        import torch
        self.torch = torch
        if not torch.cuda.is_available():
            raise RuntimeError("gnnmi needs a GPU: torch.cuda.is_available() is False")
        self.dev = torch.device(device)
        self.bf16 = dtype in ("bf16", GNN_BF16)
        store = torch.bfloat16 if self.bf16 else torch.float32
        # hbm_budget_bytes != 0: streaming schedule; features, activations and their gradients
        # then live in pinned host memory and the library caches partition blocks in HBM
        self.streaming = hbm_budget_bytes != 0
        self.ctx = Context(model, dims, dtype=GNN_BF16 if self.bf16 else GNN_F32, has_bias=has_bias,
                           hbm_budget_bytes=hbm_budget_bytes)
        self.ctx.set_layer_order(layer_order)
        self.ctx.set_gather_fusion(fuse_gather)
        self.ctx.set_masked_backward(masked_backward)
        # keep_forward: True / False, or "auto": kept when the larger workspace fits the device
        # memory that is free once everything else is allocated (decided below)
        self.ctx.set_keep_forward(keep_forward is True)
        if _MODEL.get(model, model) == GNN_GAT:
            # attention heads per layer: weights[l]["heads"] (default 1)
            for l, wl in enumerate(weights):
                if int(wl.get("heads", 1)) != 1:
                    self.ctx.set_gat_heads(l + 1, int(wl["heads"]))
        say = progress or (lambda msg: None)
        self.ctx.build_partitions(rowptr, colidx, k, part_mode, seed, user_part)
        say("partitions built")
        self.model = _MODEL.get(model, model)
        self.dims = list(dims)
        self.L = len(dims) - 1
        self.n = self.ctx.n
        self.has_bias = has_bias
        t = torch
        stream = self.stream
        # inputs: fp32 in original order -> storage type (the library's rounding to bfloat16) ->
        # library order (the library's row permutation); torch only allocates and copies
        self.labels = self._to_library(t.from_numpy(np.ascontiguousarray(labels, dtype=np.int32)).to(self.dev))
        self.mask = self._to_library(t.from_numpy(np.ascontiguousarray(train_mask, dtype=np.uint8)).to(self.dev))
        # storage_dir: the per-vertex arrays live in files there and the library caches whole
        # arrays in a pinned pool of host_budget_bytes (streaming schedule only)
        self.tiered = storage_dir is not None
        if self.tiered:
            if not self.streaming:
                raise ValueError("storage_dir needs a streaming budget (hbm_budget_bytes)")
            self.ctx.storage_open(storage_dir, host_budget_bytes)
            src = self._store(t.from_numpy(np.ascontiguousarray(X, dtype=np.float32)).pin_memory())
            feat = self._to_library(src)
            self.ctx.storage_write(0, 0, feat.data_ptr())
            del src, feat
            self.feat = None
            big = None
        elif self.streaming:
            # pinned (device-mapped) host arrays on both sides: the library's kernels read and
            # write them over the host link
            big = dict(device="cpu", pin_memory=True)
            src = self._store(t.from_numpy(np.ascontiguousarray(X, dtype=np.float32)).pin_memory())
            self.feat = self._to_library(src)
            del src
        else:
            big = dict(device=self.dev)
            self.feat = self._to_library(
                self._store(t.from_numpy(np.ascontiguousarray(X, dtype=np.float32)).to(self.dev)))
        say("features placed")
        self.act, self.gact = [], []
        for l in range(self.L if not self.tiered else 0):
            self.act.append(t.zeros((self.n, dims[l + 1]), dtype=store if l < self.L - 1 else t.float32,
                                    **big))                                  # logits stay fp32
            self.gact.append(t.zeros((self.n, dims[l + 1]), dtype=t.float32, **big))
            say("buffers of layer %d allocated" % (l + 1))
        self.w, self.gw, self.w32 = [], [], []      # w32: fp32 originals of bfloat16 matrices
        for l in range(self.L):
            for key in ("W", "Ws", "b"):
                a = weights[l].get(key)
                if key == "Ws" and self.model == GNN_GAT:
                    # graph attention: the second slot holds the two attention vectors [2, d_out]
                    a = np.stack([weights[l]["a_src"], weights[l]["a_dst"]])
                use = a is not None and (key != "Ws" or self.model in (GNN_SAGE_MEAN, GNN_GAT)) \
                    and (key != "b" or has_bias)
                if use:
                    wt = t.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(self.dev)
                    self.w32.append(wt if key != "b" and self.bf16 else None)
                    if key != "b":
                        wt = self._store(wt)
                    self.w.append(wt)
                    self.gw.append(t.zeros(wt.shape, dtype=t.float32, device=self.dev))
                else:
                    self.w.append(None)
                    self.gw.append(None)
                    self.w32.append(None)
        self.keeps_forward = keep_forward is True
        if keep_forward == "auto" and not self.streaming:
            self.ctx.set_keep_forward(True)
            sb, wb = self.ctx.workspace_bytes()
            free, _ = t.cuda.mem_get_info(self.dev)
            # (bind still allocates index arrays of its own: the second copy of the column
            # indices, 4 bytes per operator entry, and the output layer's operator over train
            # vertices, a fraction of that)
            margin = 4 * 2 ** 30 + 6 * int(rowptr[-1])
            self.keeps_forward = sb + wb + margin <= free
            if not self.keeps_forward:
                self.ctx.set_keep_forward(False)
            say("forward results %s (workspace %.1f GiB, %.1f GiB free)"
                % ("kept" if self.keeps_forward else "recomputed", (sb + wb) / 2 ** 30, free / 2 ** 30))
        ptr = lambda x: x.data_ptr() if x is not None else None

        def allocate_and_bind():
            sb, wb = self.ctx.workspace_bytes()
            self.staging = t.empty(sb, dtype=t.uint8, device=self.dev)
            self.scratch = t.empty(wb, dtype=t.uint8, device=self.dev)
            self.ctx.bind(ptr(self.feat), [ptr(a) for a in self.act], [ptr(g) for g in self.gact],
                          [ptr(w) for w in self.w], [ptr(g) for g in self.gw], ptr(self.labels),
                          ptr(self.mask), ptr(self.staging), ptr(self.scratch))

        try:
            allocate_and_bind()
        except (GnnError, RuntimeError):
            # "auto" misjudged the room: bind again with the smaller workspace
            if not (keep_forward == "auto" and self.keeps_forward):
                raise
            say("not enough device memory with kept forward results: recomputing instead")
            self.staging = self.scratch = None
            t.cuda.empty_cache()
            self.ctx.set_keep_forward(False)
            self.keeps_forward = False
            allocate_and_bind()
        say("bound")
        t.cuda.synchronize()
        del stream

    @property
    def stream(self):
        return self.torch.cuda.current_stream(self.dev).cuda_stream

    def _store(self, f32):
        """fp32 tensor (device, or pinned host) -> the context's storage type, same placement."""
        if not self.bf16:
            return f32
        t = self.torch
        out = t.empty(f32.shape, dtype=t.bfloat16, device=f32.device, pin_memory=not f32.is_cuda)
        self.ctx.to_bf16(f32.data_ptr(), out.data_ptr(), f32.numel(), self.stream)
        t.cuda.synchronize()
        return out

    def _to_library(self, src):
        """Rows in original vertex order -> library order (device tensor, or pinned host tensor)."""
        t = self.torch
        dst = t.empty(src.shape, dtype=src.dtype, device=src.device, pin_memory=not src.is_cuda)
        row_bytes = src.element_size() * (src.shape[1] if src.dim() == 2 else 1)
        self.ctx.permute_rows(src.data_ptr(), dst.data_ptr(), row_bytes, True, self.stream)
        t.cuda.synchronize()
        return dst

    def to_original(self, tensor):
        """Tensor in library order (device or pinned host) -> numpy array in original vertex order."""
        t = self.torch
        dst = t.empty(tensor.shape, dtype=tensor.dtype, device=tensor.device, pin_memory=not tensor.is_cuda)
        row_bytes = tensor.element_size() * (tensor.shape[1] if tensor.dim() == 2 else 1)
        self.ctx.permute_rows(tensor.data_ptr(), dst.data_ptr(), row_bytes, False, self.stream)
        t.cuda.synchronize()
        return dst.float().cpu().numpy()

    def set_layer_order(self, mode):
        """Switches the layer order ("auto" / "aggregate") of a bound session: the workspace sizes
        depend on it, so staging and scratch are allocated anew and everything is bound again."""
        t = self.torch
        t.cuda.synchronize()
        self.ctx.set_layer_order(mode)
        self.staging = self.scratch = None
        t.cuda.empty_cache()
        sb, wb = self.ctx.workspace_bytes()
        self.staging = t.empty(sb, dtype=t.uint8, device=self.dev)
        self.scratch = t.empty(wb, dtype=t.uint8, device=self.dev)
        ptr = lambda x: x.data_ptr() if x is not None else None
        self.ctx.bind(ptr(self.feat), [ptr(a) for a in self.act], [ptr(g) for g in self.gact],
                      [ptr(w) for w in self.w], [ptr(g) for g in self.gw], ptr(self.labels),
                      ptr(self.mask), ptr(self.staging), ptr(self.scratch))
        t.cuda.synchronize()

    def set_keep_forward(self, on):
        """Forward results kept for the backward pass (True) or recomputed there (False): the
        workspace sizes depend on it, so staging and scratch are allocated anew and everything
        is bound again."""
        if bool(on) == self.keeps_forward:
            return
        t = self.torch
        t.cuda.synchronize()
        self.ctx.set_keep_forward(on)
        self.keeps_forward = bool(on)
        self.staging = self.scratch = None
        t.cuda.empty_cache()
        sb, wb = self.ctx.workspace_bytes()
        self.staging = t.empty(sb, dtype=t.uint8, device=self.dev)
        self.scratch = t.empty(wb, dtype=t.uint8, device=self.dev)
        ptr = lambda x: x.data_ptr() if x is not None else None
        self.ctx.bind(ptr(self.feat), [ptr(a) for a in self.act], [ptr(g) for g in self.gact],
                      [ptr(w) for w in self.w], [ptr(g) for g in self.gw], ptr(self.labels),
                      ptr(self.mask), ptr(self.staging), ptr(self.scratch))
        t.cuda.synchronize()

    def set_masked_backward(self, on):
        """Output layer's transposed aggregation over train vertices only (True) or over every entry."""
        self.torch.cuda.synchronize()
        self.ctx.set_masked_backward(on)

    def set_gather_fusion(self, on):
        """Aggregation kernels read the boundary rows themselves (True) or from staging (False)."""
        self.torch.cuda.synchronize()
        self.ctx.set_gather_fusion(on)

    def epoch(self):
        return self.ctx.epoch(self.stream)

    def _from_storage(self, kind, layer):
        """One array of the storage tier as a pinned host tensor in library order."""
        t = self.torch
        d = self.dims[layer]
        dtype = t.float32 if kind == 1 or layer == self.L or not self.bf16 else t.bfloat16
        buf = t.empty((self.n, d), dtype=dtype, device="cpu", pin_memory=True)
        self.ctx.storage_read(kind, layer, buf.data_ptr())
        return buf

    def results(self):
        """Everything the oracle also returns, in original vertex order."""
        if self.tiered:
            acts = [self.to_original(self._from_storage(0, l)) for l in range(1, self.L + 1)]
            gacts = [self.to_original(self._from_storage(1, l)) for l in range(1, self.L + 1)]
        else:
            acts = [self.to_original(a) for a in self.act]
            gacts = [self.to_original(g) for g in self.gact]
        out = {"act": acts, "gact": gacts, "gW": [], "gWs": [], "gb": []}
        for l in range(self.L):
            gW, gWs, gb = self.gw[3 * l:3 * l + 3]
            out["gW"].append(gW.cpu().numpy())
            out["gWs"].append(gWs.cpu().numpy() if gWs is not None else None)
            out["gb"].append(gb.cpu().numpy() if gb is not None else None)
        return out

    # -- training around the epoch -------------------------------------------------------------
    def train(self, epochs, optimizer="adam", lr=0.01, beta1=0.9, beta2=0.999, eps=1e-8,
              weight_decay=0.0, dropout=0.0, seed=0, first_epoch=0):
        """``epochs`` times epoch + optimizer step on the bound weights; returns the losses."""
        t = self.torch
        if optimizer == "adam" and not hasattr(self, "opt_m"):
            self.opt_m = [None if w is None else t.zeros(w.shape, dtype=t.float32, device=self.dev)
                          for w in self.w]
            self.opt_v = [None if w is None else t.zeros(w.shape, dtype=t.float32, device=self.dev)
                          for w in self.w]
            ptr = lambda x: x.data_ptr() if x is not None else None
            self.ctx.bind_optimizer([ptr(x) for x in self.opt_m], [ptr(x) for x in self.opt_v])
        self.bind_master_weights()
        opt = make_optimizer(optimizer, lr, beta1, beta2, eps, weight_decay)
        return self.ctx.train(opt, epochs, first_epoch, dropout, seed, self.stream)

    def bind_master_weights(self):
        """bfloat16 storage: hands the fp32 originals of the weight matrices to the library as the
        copies the optimizer updates (once)."""
        if self.bf16 and not getattr(self, "_masters_bound", False):
            self.ctx.bind_master_weights([x.data_ptr() if x is not None else None for x in self.w32])
            self._masters_bound = True

    def master_weights(self):
        """The fp32 master copies (bfloat16 storage) in the layout of ``weights()``; biases are
        the bound fp32 ones."""
        out = []
        for l in range(self.L):
            W, Ws = self.w32[3 * l], self.w32[3 * l + 1]
            b = self.w[3 * l + 2]
            out.append({"W": W.cpu().numpy() if W is not None else None,
                        "Ws": Ws.cpu().numpy() if Ws is not None else None,
                        "b": b.float().cpu().numpy() if b is not None else None})
        return out

    def weights(self):
        """The bound weights as a list of dicts of numpy arrays (the layout of ``weights``)."""
        out = []
        for l in range(self.L):
            W, Ws, b = self.w[3 * l:3 * l + 3]
            out.append({"W": W.float().cpu().numpy(),
                        "Ws": Ws.float().cpu().numpy() if Ws is not None else None,
                        "b": b.float().cpu().numpy() if b is not None else None})
        return out
