"""ctypes binding of libnerva_sparse.so: argument marshalling only.

Every function below has the name and the argument order of the C entry point it calls
(see include/nerva_sparse.h); tensors are torch CUDA tensors used for their device
pointers, and the stream is torch's current HIP stream unless one is given.  No
arithmetic of the training step happens in Python.  If the compiled library is missing
the import of this module fails: there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("NERVA_SPARSE_LIB") or os.path.join(_PKG, "libnerva_sparse.so")   # (the variable: another build of the same library, for A/B timings)

NERVA_OK = 0
NERVA_ERR_ARGUMENT, NERVA_ERR_SHAPE, NERVA_ERR_CSR, NERVA_ERR_WORKSPACE, NERVA_ERR_HIP = -1, -2, -3, -4, -5
NERVA_ACT_NONE, NERVA_ACT_RELU = 0, 1
NERVA_PACK_MAX_LEN, NERVA_PACK_MIN_ROWS = 128, 2048
NERVA_STAGE_ROWS, NERVA_STAGE_COLS, NERVA_STAGE_MIN_BATCH, NERVA_STAGE_RANGE_ROWS, NERVA_STAGE_QUAD = 512, 64, 128, 512, 1 << 30
NERVA_PARTITION_BALANCED, NERVA_PARTITION_ROW_SPLIT, NERVA_PARTITION_PREFER_STAGED = 0, 1, 2
NERVA_MLP_DEFAULT, NERVA_MLP_UNFUSED, NERVA_MLP_NESTEROV, NERVA_MLP_SEPARATE_HEAD = 0, 1, 2, 4
NERVA_WAVES_PER_BLOCK = 16
NERVA_STATIC_WORKSPACE_BYTES = 32 << 20
NERVA_HUGE_FLAG = 0x40000000

EXPORTS = [
    "nerva_last_error", "nerva_build_info", "nerva_validate_csr_host", "nerva_plan_rows_host", "nerva_plan_short_rows_host", "nerva_plan_staged_host", "nerva_set_partition_mode", "nerva_set_dense_threshold",
    "sparse_linear_create", "sparse_linear_destroy", "sparse_linear_rebind", "sparse_linear_enable_dense", "sparse_linear_sync_values", "sparse_linear_mirror",
    "sparse_linear_forward", "sparse_linear_backward", "sgd_update_values", "sgd_update_values_nesterov",
    "softmax_cross_entropy", "mlp_create", "mlp_destroy", "mlp_rebind_velocity", "mlp_workspace_bytes",
    "mlp_workspace_layout", "mlp_train_step", "mlp_train_step_static", "mlp_forward", "nerva_copy_f32",
    "mlp_profile_enable", "mlp_profile_read", "mlp_profile_slot_name",
]


class NervaError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"nerva_sparse error {code}: {message}")
        self.code = code


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()' "
            "or python paper_2407_17437_amd/build.py). There is no fallback implementation.")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, i64, f32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_float, ctypes.c_size_t
    sig = {
        "nerva_last_error": (ctypes.c_char_p, []),
        "nerva_build_info": (ctypes.c_char_p, []),
        "nerva_validate_csr_host": (ctypes.c_int, [i32, i32, i64, vp, vp]),
        "nerva_plan_rows_host": (ctypes.c_int, [i32, vp, vp, vp, vp, vp, vp]),
        "nerva_plan_short_rows_host": (ctypes.c_int, [i32, vp, vp, vp, vp]),
        "nerva_plan_staged_host": (ctypes.c_int, [i32, i32, vp, vp, i32, i32, vp, vp, vp]),
        "nerva_set_partition_mode": (ctypes.c_int, [i32]),
        "nerva_set_dense_threshold": (ctypes.c_int, [f32]),
        "sparse_linear_create": (ctypes.c_int, [vp, i32, i32, i32, vp, vp, vp, vp, i32, i32, vp]),
        "sparse_linear_destroy": (None, [vp]),
        "sparse_linear_rebind": (ctypes.c_int, [vp, i32, vp, vp, vp, vp]),
        "sparse_linear_enable_dense": (ctypes.c_int, [vp, vp]),
        "sparse_linear_sync_values": (ctypes.c_int, [vp, vp]),
        "mlp_rebind_velocity": (ctypes.c_int, [vp, i32, vp]),
        "sparse_linear_mirror": (ctypes.c_int, [vp, vp, vp, vp, vp]),
        "sparse_linear_forward": (ctypes.c_int, [vp, vp, i32, vp, i32, i32, vp]),
        "sparse_linear_backward": (ctypes.c_int, [vp, vp, i32, vp, i32, vp, i32, vp, i32, vp, vp, i32, vp]),
        "sgd_update_values": (ctypes.c_int, [vp, vp, vp, i64, f32, f32, vp]),
        "sgd_update_values_nesterov": (ctypes.c_int, [vp, vp, vp, i64, f32, f32, vp]),
        "softmax_cross_entropy": (ctypes.c_int, [vp, i32, vp, i32, i32, vp, i32, vp, vp]),
        "mlp_create": (ctypes.c_int, [vp, i32, vp, vp, vp, i32, i32]),
        "mlp_destroy": (None, [vp]),
        "mlp_workspace_bytes": (sz, [vp, i32]),
        "mlp_workspace_layout": (ctypes.c_int, [vp, i32, vp]),
        "mlp_train_step": (ctypes.c_int, [vp, vp, i32, vp, i32, f32, f32, vp, sz, vp, vp]),
        "mlp_train_step_static": (ctypes.c_int, [vp, vp, i32, vp, i32, f32, f32, vp, vp]),
        "mlp_forward": (ctypes.c_int, [vp, vp, i32, i32, vp, sz, vp]),
        "nerva_copy_f32": (ctypes.c_int, [vp, vp, i64, vp]),
        "mlp_profile_enable": (ctypes.c_int, [vp, i32]),
        "mlp_profile_read": (ctypes.c_int, [vp, i32, vp, vp, vp]),
        "mlp_profile_slot_name": (ctypes.c_char_p, [vp, i32]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype = res
        fn.argtypes = args
    return lib


lib = _load()


def last_error() -> str:
    return lib.nerva_last_error().decode()


def build_info() -> str:
    return lib.nerva_build_info().decode()


def _check(rc: int) -> None:
    if rc != NERVA_OK:
        raise NervaError(rc, last_error())


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, torch.cuda.Stream):
        return stream.cuda_stream or None
    return stream or None


def _ld(t: torch.Tensor) -> int:
    assert t.dim() == 2 and t.stride(1) == 1 and t.dtype == torch.float32
    return t.stride(0)


# ---- host-only helpers (no GPU needed) -------------------------------------------------

def nerva_validate_csr_host(rows: int, cols: int, nnz: int, indptr, indices) -> int:
    """indptr / indices: numpy int32 arrays on the host.  Returns the status code."""
    import numpy as np
    indptr = np.ascontiguousarray(indptr, dtype=np.int32)
    indices = np.ascontiguousarray(indices, dtype=np.int32)
    return lib.nerva_validate_csr_host(rows, cols, nnz, indptr.ctypes.data, indices.ctypes.data if indices.size else None)


def nerva_plan_rows_host(rows: int, indptr):
    """Returns (row_order, blocks[nb,4], huge_rows[nh,4], n_huge_blocks, waves[nb,16,4]) as numpy int32 arrays."""
    import numpy as np
    indptr = np.ascontiguousarray(indptr, dtype=np.int32)
    counts = np.zeros(4, dtype=np.int32)
    _check(lib.nerva_plan_rows_host(rows, indptr.ctypes.data, None, None, None, None, counts.ctypes.data))
    order = np.empty(max(1, counts[0]), dtype=np.int32)
    blocks = np.empty((max(1, counts[1]), 4), dtype=np.int32)
    huge = np.empty((max(1, counts[2]), 4), dtype=np.int32)
    waves = np.empty((max(1, counts[1]), NERVA_WAVES_PER_BLOCK, 4), dtype=np.int32)
    _check(lib.nerva_plan_rows_host(rows, indptr.ctypes.data, order.ctypes.data, blocks.ctypes.data, huge.ctypes.data,
                                    waves.ctypes.data, counts.ctypes.data))
    return order[:counts[0]], blocks[:counts[1]], huge[:counts[2]], int(counts[3]), waves[:counts[1]]


def nerva_set_partition_mode(mode: int) -> None:
    _check(lib.nerva_set_partition_mode(mode))


def nerva_set_dense_threshold(density: float) -> None:
    _check(lib.nerva_set_dense_threshold(density))


def nerva_plan_short_rows_host(rows: int, indptr):
    """Returns (short_rows[ns64,4], n_short, long_waves[nl,16,4], n_long_huge_blocks) as numpy int32 arrays."""
    import numpy as np
    indptr = np.ascontiguousarray(indptr, dtype=np.int32)
    counts = np.zeros(3, dtype=np.int32)
    _check(lib.nerva_plan_short_rows_host(rows, indptr.ctypes.data, None, None, counts.ctypes.data))
    ns64 = (int(counts[0]) + 63) // 64 * 64
    short = np.empty((max(1, ns64), 4), dtype=np.int32)
    waves = np.empty((max(1, counts[1]), NERVA_WAVES_PER_BLOCK, 4), dtype=np.int32)
    _check(lib.nerva_plan_short_rows_host(rows, indptr.ctypes.data, short.ctypes.data, waves.ctypes.data, counts.ctypes.data))
    return short[:ns64], int(counts[0]), waves[:counts[1]], int(counts[2])


def nerva_plan_staged_host(rows: int, cols: int, indptr, indices, max_batch: int, min_entries: int = 0):
    """Returns (slot_rows[ranges, 512], ends[ranges, blocks + 1, 512]) as numpy int32 arrays; ranges == 0: not staged."""
    import numpy as np
    indptr = np.ascontiguousarray(indptr, dtype=np.int32)
    indices = np.ascontiguousarray(indices, dtype=np.int32)
    counts = np.zeros(2, dtype=np.int32)
    _check(lib.nerva_plan_staged_host(rows, cols, indptr.ctypes.data, indices.ctypes.data, max_batch, min_entries, None, None, counts.ctypes.data))
    ranges, blocks = int(counts[0]), int(counts[1])
    slot_rows = np.zeros((ranges, NERVA_STAGE_RANGE_ROWS), dtype=np.int32)
    ends = np.zeros((ranges, blocks + 1, NERVA_STAGE_RANGE_ROWS), dtype=np.int32)
    if ranges:
        _check(lib.nerva_plan_staged_host(rows, cols, indptr.ctypes.data, indices.ctypes.data, max_batch, min_entries,
                                          slot_rows.ctypes.data, ends.ctypes.data, counts.ctypes.data))
    return slot_rows, ends


# ---- entry points, same names as the C ABI ------------------------------------------------

def sparse_linear_create(rows, cols, nnz, indptr, indices, values, bias, activation, max_batch, stream=None) -> int:
    h = ctypes.c_void_p()
    _check(lib.sparse_linear_create(ctypes.addressof(h), rows, cols, nnz, _ptr(indptr), _ptr(indices), _ptr(values),
                                    _ptr(bias), activation, max_batch, _stream(stream)))
    return h.value


def sparse_linear_destroy(layer: int) -> None:
    lib.sparse_linear_destroy(layer)


def sparse_linear_rebind(layer: int, nnz, indptr, indices, values, stream=None) -> None:
    _check(lib.sparse_linear_rebind(layer, nnz, _ptr(indptr), _ptr(indices), _ptr(values), _stream(stream)))


def sparse_linear_enable_dense(layer: int, stream=None) -> None:
    _check(lib.sparse_linear_enable_dense(layer, _stream(stream)))


def sparse_linear_sync_values(layer: int, stream=None) -> None:
    _check(lib.sparse_linear_sync_values(layer, _stream(stream)))


def mlp_rebind_velocity(mlp: int, layer_index: int, velocity) -> None:
    _check(lib.mlp_rebind_velocity(mlp, layer_index, _ptr(velocity)))


def sparse_linear_mirror(layer: int):
    """Raw device addresses (indptr_t, indices_t, values_t, perm)."""
    out = [ctypes.c_void_p() for _ in range(4)]
    _check(lib.sparse_linear_mirror(layer, *[ctypes.addressof(o) for o in out]))
    return tuple(o.value for o in out)


def sparse_linear_forward(layer: int, X, Y, batch: int, stream=None) -> None:
    _check(lib.sparse_linear_forward(layer, _ptr(X), _ld(X), _ptr(Y), _ld(Y), batch, _stream(stream)))


def sparse_linear_backward(layer: int, X, Y, dY, dX, dvalues, dbias, batch: int, stream=None) -> None:
    _check(lib.sparse_linear_backward(layer, _ptr(X), _ld(X) if X is not None else 0,
                                      _ptr(Y), _ld(Y) if Y is not None else 0, _ptr(dY), _ld(dY),
                                      _ptr(dX), _ld(dX) if dX is not None else 0, _ptr(dvalues), _ptr(dbias),
                                      batch, _stream(stream)))


def sgd_update_values(values, velocity, grad, n: int, lr: float, momentum: float, stream=None) -> None:
    _check(lib.sgd_update_values(_ptr(values), _ptr(velocity), _ptr(grad), n, lr, momentum, _stream(stream)))


def sgd_update_values_nesterov(values, velocity, grad, n: int, lr: float, momentum: float, stream=None) -> None:
    _check(lib.sgd_update_values_nesterov(_ptr(values), _ptr(velocity), _ptr(grad), n, lr, momentum, _stream(stream)))


def softmax_cross_entropy(Z, labels, classes: int, batch: int, dZ, loss_out, stream=None) -> None:
    _check(lib.softmax_cross_entropy(_ptr(Z), _ld(Z), _ptr(labels), classes, batch, _ptr(dZ), _ld(dZ),
                                     _ptr(loss_out), _stream(stream)))


def mlp_create(layers: Sequence[int], velocities, bias_velocities, max_batch: int, flags: int = NERVA_MLP_DEFAULT) -> int:
    n = len(layers)
    arr_l = (ctypes.c_void_p * n)(*layers)
    arr_v = (ctypes.c_void_p * n)(*[_ptr(v) for v in velocities])
    arr_b = (ctypes.c_void_p * n)(*[_ptr(v) for v in bias_velocities])
    h = ctypes.c_void_p()
    _check(lib.mlp_create(ctypes.addressof(h), n, arr_l, arr_v, arr_b, max_batch, flags))
    return h.value


def mlp_destroy(mlp: int) -> None:
    lib.mlp_destroy(mlp)


def mlp_workspace_bytes(mlp: int, batch: int) -> int:
    return int(lib.mlp_workspace_bytes(mlp, batch))


def mlp_workspace_layout(mlp: int, batch: int, n_layers: int) -> List[int]:
    out = (ctypes.c_int64 * (1 + 4 * n_layers))()
    _check(lib.mlp_workspace_layout(mlp, batch, out))
    return list(out)


def mlp_train_step(mlp: int, X, ldx: int, labels, batch: int, lr: float, momentum: float, workspace,
                   loss_out, stream=None) -> None:
    """X may be a tensor or a raw device address (int); ldx in floats."""
    xp = X if isinstance(X, int) else _ptr(X)
    lp = labels if isinstance(labels, int) else _ptr(labels)
    _check(lib.mlp_train_step(mlp, xp, ldx, lp, batch, lr, momentum, _ptr(workspace),
                              workspace.numel() * workspace.element_size(), _ptr(loss_out), _stream(stream)))


def mlp_train_step_static(mlp: int, X, ldx: int, labels, batch: int, lr: float, momentum: float, loss_out, stream=None) -> None:
    """The same step on the library's own static workspace; X and labels may be tensors or raw device addresses."""
    xp = X if isinstance(X, int) else _ptr(X)
    lp = labels if isinstance(labels, int) else _ptr(labels)
    _check(lib.mlp_train_step_static(mlp, xp, ldx, lp, batch, lr, momentum, _ptr(loss_out), _stream(stream)))


def mlp_forward(mlp: int, X, ldx: int, batch: int, workspace, stream=None) -> None:
    xp = X if isinstance(X, int) else _ptr(X)
    _check(lib.mlp_forward(mlp, xp, ldx, batch, _ptr(workspace), workspace.numel() * workspace.element_size(),
                           _stream(stream)))


def mlp_profile_enable(mlp: int, max_steps: int) -> None:
    _check(lib.mlp_profile_enable(mlp, max_steps))


def mlp_profile_read(mlp: int, max_slots: int = 256):
    """Returns (steps, [(slot name, summed milliseconds), ...])."""
    n = ctypes.c_int32(0); steps = ctypes.c_int32(0)
    ms = (ctypes.c_double * max_slots)()
    _check(lib.mlp_profile_read(mlp, max_slots, ctypes.addressof(n), ms, ctypes.addressof(steps)))
    return steps.value, [(lib.mlp_profile_slot_name(mlp, k).decode(), ms[k]) for k in range(n.value)]


def nerva_copy_f32(dst, src, n: int, stream=None) -> None:
    _check(lib.nerva_copy_f32(_ptr(dst), _ptr(src), n, _stream(stream)))


# ---- owners of device memory and handles (lifetime management only) ------------------------

def padded_ld(batch: int) -> int:
    """Leading dimension the harness uses for a batch: rows start on 128-byte boundaries."""
    return (batch + 31) // 32 * 32


def dense(features: int, batch: int, device="cuda", ld: Optional[int] = None) -> torch.Tensor:
    """(features, batch) fp32 view of a (features, ld) allocation; padding holds NaN so that any
    use of a padding column shows up in the results."""
    ld = padded_ld(batch) if ld is None else ld
    full = torch.full((features, ld), float("nan"), dtype=torch.float32, device=device)
    return full[:, :batch]


def to_dense(array, device="cuda", ld: Optional[int] = None) -> torch.Tensor:
    t = torch.as_tensor(array, dtype=torch.float32)
    out = dense(t.shape[0], t.shape[1], device, ld)
    out.copy_(t)
    return out


class SparseLinear:
    """Device copies of one layer's arrays plus the library handle."""

    def __init__(self, layer_data, max_batch: int = 1024, device="cuda"):
        self.handle = None
        d = layer_data
        self.rows, self.cols, self.nnz = d.rows, d.cols, d.nnz
        self.relu = bool(d.relu)
        self.indptr = torch.as_tensor(d.indptr, dtype=torch.int32).to(device)
        self.indices = torch.as_tensor(d.indices, dtype=torch.int32).to(device)
        self.values = torch.as_tensor(d.values, dtype=torch.float32).to(device)
        self.bias = torch.as_tensor(d.bias, dtype=torch.float32).to(device)
        self.velocity = torch.zeros(max(1, d.nnz), dtype=torch.float32, device=device)[:d.nnz]
        self.bias_velocity = torch.zeros(d.rows, dtype=torch.float32, device=device)
        self.handle = sparse_linear_create(d.rows, d.cols, d.nnz, self.indptr, self.indices, self.values, self.bias,
                                           NERVA_ACT_RELU if d.relu else NERVA_ACT_NONE, max_batch)

    def rebind(self, indptr, indices, values, velocity=None):
        """New pattern for the same rows x cols matrix (numpy arrays; canonical CSR).  The device copies
        replace the old ones once the library has accepted the pattern; velocity defaults to zeros."""
        nnz = int(indptr[-1])
        dev = self.values.device
        new_indptr = torch.as_tensor(indptr, dtype=torch.int32).to(dev)
        new_indices = torch.as_tensor(indices, dtype=torch.int32).to(dev)
        new_values = torch.as_tensor(values, dtype=torch.float32).to(dev)
        sparse_linear_rebind(self.handle, nnz, new_indptr, new_indices, new_values)
        self.indptr, self.indices, self.values, self.nnz = new_indptr, new_indices, new_values, nnz
        if velocity is None:
            self.velocity = torch.zeros(max(1, nnz), dtype=torch.float32, device=dev)[:nnz]
        else:
            self.velocity = torch.as_tensor(velocity, dtype=torch.float32).to(dev)

    def close(self):
        if self.handle:
            sparse_linear_destroy(self.handle)
            self.handle = None

    def __del__(self):
        self.close()


class MLP:
    """A chain of SparseLinear layers, the library's MLP handle and its workspace."""

    def __init__(self, mlp_data, max_batch: int, flags: int = NERVA_MLP_DEFAULT, device="cuda", dense_from_density=None):
        """dense_from_density: layers whose density is at least this take the dense route (None: none)."""
        self.handle = None
        self.layers = []
        self.layers = [SparseLinear(l, max_batch, device) for l in mlp_data.layers]
        if dense_from_density is not None:
            for l in self.layers:
                if l.nnz >= dense_from_density * l.rows * l.cols:
                    sparse_linear_enable_dense(l.handle)
        self.max_batch = max_batch
        self.handle = mlp_create([l.handle for l in self.layers], [l.velocity for l in self.layers],
                                 [l.bias_velocity for l in self.layers], max_batch, flags)
        nbytes = mlp_workspace_bytes(self.handle, max_batch)
        # NaN-filled so that a read of something never written cannot pass unnoticed
        self.workspace = torch.full((nbytes // 4,), float("nan"), dtype=torch.float32, device=device)
        self.loss = torch.zeros(1, dtype=torch.float32, device=device)
        self._layout_batch = None
        self._layout = None

    def layout(self, batch: int):
        if self._layout_batch != batch:
            self._layout = mlp_workspace_layout(self.handle, batch, len(self.layers))
            self._layout_batch = batch
        return self._layout

    def view(self, kind: str, l: int, batch: int) -> torch.Tensor:
        """kind in A / dZ (rows_l x batch views), g (nnz_l), db (rows_l)."""
        lay = self.layout(batch)
        ld = lay[0]
        k = {"A": 0, "dZ": 1, "g": 2, "db": 3}[kind]
        off = lay[1 + 4 * l + k] // 4
        L = self.layers[l]
        if kind in ("A", "dZ"):
            return self.workspace[off: off + L.rows * ld].view(L.rows, ld)[:, :batch]
        n = L.nnz if kind == "g" else L.rows
        return self.workspace[off: off + n]

    def rebind_layer(self, l: int, indptr, indices, values, velocity=None):
        """Topology update of layer l between steps: new pattern, values and (re-mapped) momentum buffer."""
        self.layers[l].rebind(indptr, indices, values, velocity)
        mlp_rebind_velocity(self.handle, l, self.layers[l].velocity)
        # the workspace layout holds one float per stored entry of every layer: it moves with nnz
        self._layout_batch = None
        nbytes = mlp_workspace_bytes(self.handle, self.max_batch)
        if nbytes // 4 > self.workspace.numel():
            self.workspace = torch.full((nbytes // 4,), float("nan"), dtype=torch.float32, device=self.workspace.device)

    def train_step(self, X, labels, batch: int, lr: float, momentum: float, ldx: Optional[int] = None):
        if ldx is None:
            ldx = _ld(X)
        mlp_train_step(self.handle, X, ldx, labels, batch, lr, momentum, self.workspace, self.loss)

    def forward(self, X, batch: int, ldx: Optional[int] = None):
        if ldx is None:
            ldx = _ld(X)
        mlp_forward(self.handle, X, ldx, batch, self.workspace)
        return self.view("A", len(self.layers) - 1, batch)

    def close(self):
        if self.handle:
            mlp_destroy(self.handle)
            self.handle = None
        for l in self.layers:
            l.close()

    def __del__(self):
        self.close()
