"""ctypes binding of libpack.so: the same entry points as include/pack.h, with argument
marshalling only.  Every step of the training path runs inside the library's kernels."""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("PACK_LIB", os.path.join(_HERE, "libpack.so"))

PACK_OK, PACK_EINVAL, PACK_ENOMEM, PACK_EDEVICE, PACK_ESHAPE, PACK_ELABEL, PACK_EINDEX = range(7)
PACK_F32, PACK_BF16 = 0, 1
OPS = {"linear": 0, "conv3x3": 1, "relu": 2, "gap": 3, "res_begin": 4, "res_end": 5,
       "sigmoid": 6, "tanh": 7, "leaky_relu": 8}
OPT_KINDS = {"sgd": 0, "momentum": 1, "adagrad": 2, "adam": 3}
STATUS_NAMES = ["PACK_OK", "PACK_EINVAL", "PACK_ENOMEM", "PACK_EDEVICE", "PACK_ESHAPE", "PACK_ELABEL", "PACK_EINDEX"]

EXPORTS = ["pack_create", "pack_write_weights", "pack_step", "pack_read_loss", "pack_read_weights",
           "pack_read_pred", "pack_read_grads", "pack_read_logits", "pack_num_params",
           "pack_num_classes", "pack_num_launches", "pack_device_bytes", "pack_last_error", "pack_destroy",
           "pack_profile_start", "pack_profile_stop", "pack_launch_name", "pack_launch_flops",
           "pack_set_optimizer", "pack_read_opt_state", "pack_write_opt_state",
           "pack_free", "pack_load", "pack_set_batch", "pack_num_slots", "pack_member_batch",
           "pack_schedule_create", "pack_schedule_next", "pack_schedule_used", "pack_schedule_destroy",
           "pack_gather_batch", "pack_set_input_mode", "pack_config_distance", "pack_opt_knn", "pack_opt_random",
           "pack_opt_batchsize", "pack_hyperband_plan", "pack_halving_keep", "pack_estimate_bytes",
           "pack_keep_grads", "pack_launch_bytes", "pack_measure_ceiling", "pack_launch_tile", "pack_plan_check",
           "pack_step_static", "pack_static_scratch_bytes", "pack_workspace_bytes"]


class pack_opt_spec(C.Structure):
    _fields_ = [("kind", C.c_int32), ("mu", C.c_float), ("acc0", C.c_float), ("beta1", C.c_float),
                ("beta2", C.c_float), ("eps", C.c_float)]


class pack_layer(C.Structure):
    _fields_ = [("op", C.c_int32), ("out", C.c_int32), ("stride", C.c_int32)]


class pack_model_spec(C.Structure):
    _fields_ = [("layers", C.POINTER(pack_layer)), ("n_layers", C.c_int32), ("batch", C.c_int32)]


class pack_input_spec(C.Structure):
    _fields_ = [("B", C.c_int32), ("in_h", C.c_int32), ("in_w", C.c_int32), ("in_c", C.c_int32),
                ("dtype", C.c_int32)]


class PackError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"{STATUS_NAMES[status] if 0 <= status < len(STATUS_NAMES) else status}: {text}")
        self.status = status


_lib = None


def lib() -> C.CDLL:
    """Loads libpack.so (once).  There is no fallback: a missing library is an error."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2002_02885_amd.build`")
        l = C.CDLL(LIB_PATH)
        vp, i32, u64, sz = C.c_void_p, C.c_int32, C.c_uint64, C.c_size_t
        fp = C.POINTER(C.c_float)
        l.pack_create.argtypes = [C.POINTER(pack_input_spec), C.POINTER(pack_model_spec), i32, u64, vp, C.POINTER(vp)]
        l.pack_write_weights.argtypes = [vp, i32, fp, sz]
        l.pack_step.argtypes = [vp, vp, vp, fp]
        l.pack_read_loss.argtypes = [vp, fp]
        l.pack_read_weights.argtypes = [vp, i32, fp, sz]
        l.pack_read_pred.argtypes = [vp, i32, C.POINTER(C.c_int32)]
        l.pack_read_grads.argtypes = [vp, i32, fp, sz]
        l.pack_read_logits.argtypes = [vp, i32, fp, sz]
        l.pack_num_params.argtypes = [vp, i32]
        l.pack_num_params.restype = sz
        l.pack_num_classes.argtypes = [vp, i32]
        l.pack_num_classes.restype = i32
        l.pack_num_launches.argtypes = [vp]
        l.pack_num_launches.restype = i32
        l.pack_device_bytes.argtypes = [vp]
        l.pack_device_bytes.restype = sz
        l.pack_last_error.argtypes = []
        l.pack_last_error.restype = C.c_char_p
        l.pack_destroy.argtypes = [vp]
        l.pack_destroy.restype = None
        l.pack_profile_start.argtypes = [vp, i32, i32]
        l.pack_profile_stop.argtypes = [vp, fp, C.POINTER(C.c_int32)]
        l.pack_launch_name.argtypes = [vp, i32, C.c_char_p, sz]
        l.pack_launch_flops.argtypes = [vp, i32, C.POINTER(C.c_double)]
        l.pack_set_optimizer.argtypes = [vp, i32, C.POINTER(pack_opt_spec)]
        l.pack_read_opt_state.argtypes = [vp, i32, i32, fp, sz, C.POINTER(C.c_int64)]
        l.pack_write_opt_state.argtypes = [vp, i32, i32, fp, sz, C.c_int64]
        i64 = C.c_int64
        l.pack_measure_ceiling.argtypes = [i32, vp, C.POINTER(C.c_double)]
        l.pack_free.argtypes = [vp, i32]
        l.pack_load.argtypes = [vp, C.POINTER(pack_model_spec), u64, C.POINTER(i32)]
        l.pack_set_batch.argtypes = [vp, i32, C.POINTER(i32)]
        l.pack_num_slots.argtypes = [vp]
        l.pack_num_slots.restype = i32
        l.pack_member_batch.argtypes = [vp, i32]
        l.pack_member_batch.restype = i32
        l.pack_schedule_create.argtypes = [i64, C.POINTER(i32), i32, C.POINTER(vp)]
        l.pack_schedule_next.argtypes = [vp, C.POINTER(i64), C.POINTER(i32), C.POINTER(i32), C.POINTER(i32)]
        l.pack_schedule_used.argtypes = [vp, C.POINTER(i64)]
        l.pack_schedule_destroy.argtypes = [vp]
        l.pack_schedule_destroy.restype = None
        l.pack_gather_batch.argtypes = [vp, vp, vp, i64, vp, i32, vp, vp]
        ip, u8p, u64p, dp = C.POINTER(i32), C.POINTER(C.c_uint8), C.POINTER(u64), C.POINTER(C.c_double)
        l.pack_config_distance.argtypes = [ip, ip, u8p, i32]
        l.pack_config_distance.restype = i32
        l.pack_opt_knn.argtypes = [ip, u8p, i32, i32, u64p, u64, i32, dp, ip, ip]
        l.pack_opt_random.argtypes = [i32, i32, ip, ip, ip]
        l.pack_opt_batchsize.argtypes = [ip, i32, u64p, u64, ip, ip]
        l.pack_hyperband_plan.argtypes = [i32, i32, ip, ip, ip, i32, ip]
        l.pack_halving_keep.argtypes = [fp, i32, i32, ip]
        for name in ("pack_opt_knn", "pack_opt_random", "pack_opt_batchsize", "pack_hyperband_plan", "pack_halving_keep"):
            getattr(l, name).restype = C.c_int
        l.pack_estimate_bytes.argtypes = [C.POINTER(pack_input_spec), C.POINTER(pack_model_spec), i32]
        l.pack_estimate_bytes.restype = sz
        l.pack_set_input_mode.argtypes = [vp, i32]
        l.pack_set_input_mode.restype = C.c_int
        l.pack_keep_grads.argtypes = [vp, i32]
        l.pack_keep_grads.restype = C.c_int
        l.pack_launch_bytes.argtypes = [vp, i32, C.POINTER(C.c_double)]
        l.pack_launch_bytes.restype = C.c_int
        l.pack_launch_tile.argtypes = [vp, i32, C.POINTER(i32), C.POINTER(i32), C.POINTER(i32)]
        l.pack_step_static.argtypes = [vp, vp, vp, fp]
        l.pack_step_static.restype = C.c_int
        l.pack_static_scratch_bytes.argtypes = []
        l.pack_static_scratch_bytes.restype = sz
        l.pack_workspace_bytes.argtypes = [vp]
        l.pack_workspace_bytes.restype = sz
        i64p = C.POINTER(C.c_int64)
        l.pack_plan_check.argtypes = [C.POINTER(pack_input_spec), C.POINTER(pack_model_spec), i32, i32, i64p, i64p, i64p]
        l.pack_plan_check.restype = C.c_int
        for name in ("pack_free", "pack_load", "pack_set_batch", "pack_schedule_create", "pack_schedule_next",
                     "pack_schedule_used", "pack_gather_batch"):
            getattr(l, name).restype = C.c_int
        for name in ("pack_create", "pack_write_weights", "pack_step", "pack_read_loss",
                     "pack_read_weights", "pack_read_pred", "pack_read_grads", "pack_read_logits",
                     "pack_profile_start", "pack_profile_stop", "pack_launch_name",
                     "pack_launch_flops", "pack_set_optimizer", "pack_read_opt_state", "pack_write_opt_state"):
            getattr(l, name).restype = C.c_int
        _lib = l
    return _lib


def _check(status: int, allow: Sequence[int] = ()):
    if status != PACK_OK and status not in allow:
        raise PackError(status, lib().pack_last_error().decode())
    return status


def _fptr(a: np.ndarray):
    return a.ctypes.data_as(C.POINTER(C.c_float))


def _layer_array(layers):
    arr = (pack_layer * max(len(layers), 1))()
    for i, op in enumerate(layers):
        arr[i].op = OPS[op[0]] if op[0] in OPS else int(op[0])
        arr[i].out = int(op[1]) if len(op) > 1 else 0
        arr[i].stride = int(op[2]) if len(op) > 2 else 1
    return arr


def _model_specs(B: int, in_shape, dtype: str, models, batch):
    """(input spec, array of member specs, objects to keep alive) for the entry points that take layer lists."""
    K = len(models)
    batch = list(batch) if batch is not None else [B] * K
    keep = []
    specs = (pack_model_spec * max(K, 1))()
    for k, layers in enumerate(models):
        arr = _layer_array(layers)
        keep.append(arr)
        specs[k].layers = arr
        specs[k].n_layers = len(layers)
        specs[k].batch = int(batch[k])
    inp = pack_input_spec(B, in_shape[0], in_shape[1], in_shape[2], PACK_BF16 if dtype == "bf16" else PACK_F32)
    return inp, specs, keep


def static_scratch_bytes() -> int:
    return int(lib().pack_static_scratch_bytes())


def plan_check(B: int, in_shape, dtype: str, models, batch=None, per_member_input: bool = False):
    """pack_plan_check: plans the pack without a GPU and walks the kernels' address rules on the host.
    Returns (launches walked, matrix-product launches without a host model, loads and operand reads checked);
    raises PackError on a violation."""
    inp, specs, keep = _model_specs(B, in_shape, dtype, models, batch)
    walked, skipped, loads = C.c_int64(0), C.c_int64(0), C.c_int64(0)
    _check(lib().pack_plan_check(C.byref(inp), specs, len(models), 1 if per_member_input else 0,
                                 C.byref(walked), C.byref(skipped), C.byref(loads)))
    del keep
    return int(walked.value), int(skipped.value), int(loads.value)


class Pack:
    """One packed model on the current GPU.  `models` is a list of layer lists of tuples
    ("linear", out) / ("conv3x3", out, stride) / ("relu",) / ("sigmoid",) / ("tanh",) /
    ("leaky_relu",) / ("gap",) / ("res_begin",) / ("res_end",); `batch[k]` is the number of leading rows of the shared batch member k uses."""

    def __init__(self, B: int, in_shape: Tuple[int, int, int], dtype: str, models: List[list],
                 batch: Sequence[int] = None, seed: int = 0, stream: int = 0):
        self._h = C.c_void_p()
        self.K = len(models)
        self.B = B
        self.dtype = dtype
        batch = list(batch) if batch is not None else [B] * self.K
        keep = []
        specs = (pack_model_spec * max(self.K, 1))()
        for k, layers in enumerate(models):
            arr = _layer_array(layers)
            keep.append(arr)
            specs[k].layers = arr
            specs[k].n_layers = len(layers)
            specs[k].batch = int(batch[k])
        inp = pack_input_spec(B, in_shape[0], in_shape[1], in_shape[2], PACK_BF16 if dtype == "bf16" else PACK_F32)
        _check(lib().pack_create(C.byref(inp), specs, self.K, seed, C.c_void_p(stream), C.byref(self._h)))
        self.batch = batch

    # -- the ABI, one method per entry point ---------------------------------------------------
    def write_weights(self, k: int, blob: np.ndarray):
        blob = np.ascontiguousarray(blob, dtype=np.float32)
        _check(lib().pack_write_weights(self._h, k, _fptr(blob), blob.size))

    def step(self, x_ptr: int, labels_ptr: int, lr: np.ndarray):
        """x_ptr / labels_ptr are raw device addresses (e.g. torch tensor .data_ptr())."""
        lr = np.ascontiguousarray(lr, dtype=np.float32)
        assert lr.size == self.K
        _check(lib().pack_step(self._h, C.c_void_p(x_ptr), C.c_void_p(labels_ptr), _fptr(lr)))

    def step_static(self, x_ptr: int, labels_ptr: int, lr: np.ndarray):
        """pack_step_static: the same step, allocating nothing; scratch in the library's static array."""
        lr = np.ascontiguousarray(lr, dtype=np.float32)
        assert lr.size == self.K
        _check(lib().pack_step_static(self._h, C.c_void_p(x_ptr), C.c_void_p(labels_ptr), _fptr(lr)))

    def workspace_bytes(self) -> int:
        return int(lib().pack_workspace_bytes(self._h))

    def _refresh_slots(self):
        self.K = int(lib().pack_num_slots(self._h))
        self.batch = [int(lib().pack_member_batch(self._h, k)) for k in range(self.K)]

    def free(self, k: int):
        """Member k leaves the pack (read its checkpoint first); its slot becomes vacant."""
        _check(lib().pack_free(self._h, k))
        self._refresh_slots()

    def load(self, layers: list, batch: int, seed: int = 0) -> int:
        """A new member joins the pack; returns its slot."""
        arr = _layer_array(layers)
        spec = pack_model_spec(arr, len(layers), int(batch))
        k = C.c_int32(-1)
        _check(lib().pack_load(self._h, C.byref(spec), seed, C.byref(k)))
        self._refresh_slots()
        return int(k.value)

    def set_batch(self, B: int, batch: Sequence[int]):
        """The shared batch has B rows from now on; batch[k] per slot (entries of vacant slots ignored)."""
        arr = (C.c_int32 * max(self.K, 1))(*[int(b) for b in batch])
        assert len(batch) == self.K
        _check(lib().pack_set_batch(self._h, int(B), arr))
        self.B = int(B)
        self._refresh_slots()

    def set_input_mode(self, per_member: bool):
        """per_member: step() then takes K stacked batches [K][B, ...] and K stacked label vectors."""
        _check(lib().pack_set_input_mode(self._h, 1 if per_member else 0))

    def gather_batch(self, data_ptr: int, labels_all_ptr: int, n_samples: int, idx_ptr: int, rows: int,
                     x_out_ptr: int, labels_out_ptr: int):
        """All pointers are raw device addresses; idx is int64 [rows]."""
        _check(lib().pack_gather_batch(self._h, C.c_void_p(data_ptr), C.c_void_p(labels_all_ptr), int(n_samples),
                                       C.c_void_p(idx_ptr), int(rows), C.c_void_p(x_out_ptr), C.c_void_p(labels_out_ptr)))

    def set_optimizer(self, k: int, opt: dict):
        """`opt` as in the oracle: {"kind": "sgd" | "momentum" | "adagrad" | "adam", and optionally
        "mu", "acc0", "beta1", "beta2", "eps"}."""
        spec = pack_opt_spec(OPT_KINDS[opt["kind"]], float(opt.get("mu", 0.9)), float(opt.get("acc0", 0.1)),
                             float(opt.get("beta1", 0.9)), float(opt.get("beta2", 0.999)), float(opt.get("eps", 1e-8)))
        _check(lib().pack_set_optimizer(self._h, k, C.byref(spec)))

    def read_opt_state(self, k: int, slot: int):
        """Returns (state array in the blob layout, steps taken)."""
        out = np.empty(self.num_params(k), dtype=np.float32)
        steps = C.c_int64(0)
        _check(lib().pack_read_opt_state(self._h, k, slot, _fptr(out), out.size, C.byref(steps)))
        return out, int(steps.value)

    def write_opt_state(self, k: int, slot: int, state: np.ndarray, steps: int):
        state = np.ascontiguousarray(state, dtype=np.float32)
        _check(lib().pack_write_opt_state(self._h, k, slot, _fptr(state), state.size, steps))

    def read_loss(self, allow_label_error: bool = False) -> np.ndarray:
        out = np.empty(self.K, dtype=np.float32)
        st = _check(lib().pack_read_loss(self._h, _fptr(out)), allow=(PACK_ELABEL, PACK_EINDEX) if allow_label_error else ())
        self.last_status = st
        return out

    def read_weights(self, k: int) -> np.ndarray:
        out = np.empty(self.num_params(k), dtype=np.float32)
        _check(lib().pack_read_weights(self._h, k, _fptr(out), out.size))
        return out

    def read_grads(self, k: int) -> np.ndarray:
        out = np.empty(self.num_params(k), dtype=np.float32)
        _check(lib().pack_read_grads(self._h, k, _fptr(out), out.size))
        return out

    def read_pred(self, k: int) -> np.ndarray:
        out = np.empty(self.batch[k], dtype=np.int32)
        _check(lib().pack_read_pred(self._h, k, out.ctypes.data_as(C.POINTER(C.c_int32))))
        return out

    def read_logits(self, k: int) -> np.ndarray:
        out = np.empty((self.batch[k], self.num_classes(k)), dtype=np.float32)
        _check(lib().pack_read_logits(self._h, k, _fptr(out), out.size))
        return out

    def num_params(self, k: int) -> int:
        return int(lib().pack_num_params(self._h, k))

    def num_classes(self, k: int) -> int:
        return int(lib().pack_num_classes(self._h, k))

    def num_launches(self) -> int:
        return int(lib().pack_num_launches(self._h))

    def device_bytes(self) -> int:
        return int(lib().pack_device_bytes(self._h))

    def profile_start(self, which: int = -1, every: int = 1):
        _check(lib().pack_profile_start(self._h, which, every))

    def profile_stop(self):
        """Returns (summed milliseconds, sample count) per launch index."""
        n = self.num_launches()
        ms = np.zeros(n, dtype=np.float32)
        cnt = np.zeros(n, dtype=np.int32)
        _check(lib().pack_profile_stop(self._h, _fptr(ms), cnt.ctypes.data_as(C.POINTER(C.c_int32))))
        return ms, cnt

    def launch_name(self, i: int) -> str:
        buf = C.create_string_buffer(64)
        _check(lib().pack_launch_name(self._h, i, buf, 64))
        return buf.value.decode()

    def keep_grads(self, on: bool = True):
        """Plain-SGD packs do not store gradients unless asked to (read_grads needs it)."""
        _check(lib().pack_keep_grads(self._h, 1 if on else 0))

    def launch_bytes(self, i: int) -> float:
        out = C.c_double(0.0)
        _check(lib().pack_launch_bytes(self._h, i, C.byref(out)))
        return float(out.value)

    def launch_tile(self, i: int):
        r, c, lean = C.c_int32(0), C.c_int32(0), C.c_int32(0)
        _check(lib().pack_launch_tile(self._h, i, C.byref(r), C.byref(c), C.byref(lean)))
        return r.value, c.value, bool(lean.value)

    def launch_flops(self, i: int) -> float:
        out = C.c_double(0.0)
        _check(lib().pack_launch_flops(self._h, i, C.byref(out)))
        return float(out.value)

    def destroy(self):
        if self._h:
            lib().pack_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


class Schedule:
    """Epoch schedule for members with different batch sizes (host logic of the library)."""

    def __init__(self, n_samples: int, batch: Sequence[int]):
        self._h = C.c_void_p()
        self.K = len(batch)
        self.max_batch = max(batch) if len(batch) else 0
        arr = (C.c_int32 * max(self.K, 1))(*[int(b) for b in batch])
        _check(lib().pack_schedule_create(int(n_samples), arr, self.K, C.byref(self._h)))

    def next(self):
        """Returns (idx int64 [rows], rows_k int32 [K], lead) or None after the last step."""
        idx = np.empty(max(self.max_batch, 1), dtype=np.int64)
        rows_k = np.zeros(self.K, dtype=np.int32)
        rows, lead = C.c_int32(0), C.c_int32(-1)
        _check(lib().pack_schedule_next(self._h, idx.ctypes.data_as(C.POINTER(C.c_int64)), C.byref(rows),
                                        rows_k.ctypes.data_as(C.POINTER(C.c_int32)), C.byref(lead)))
        if rows.value == 0:
            return None
        return idx[:rows.value].copy(), rows_k, int(lead.value)

    def used(self) -> np.ndarray:
        out = np.zeros(self.K, dtype=np.int64)
        _check(lib().pack_schedule_used(self._h, out.ctypes.data_as(C.POINTER(C.c_int64))))
        return out

    def destroy(self):
        if self._h:
            lib().pack_schedule_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


# ---- pack-aware search: host logic of the library -------------------------------------------------
def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _groups_from_ids(ids, n_groups):
    groups = [[] for _ in range(n_groups)]
    for i, g in enumerate(ids):
        groups[int(g)].append(i)
    return groups


def config_distance(a, b, categorical) -> int:
    a, b = _i32(a), _i32(b)
    cat = np.ascontiguousarray(categorical, dtype=np.uint8)
    ip, u8p = C.POINTER(C.c_int32), C.POINTER(C.c_uint8)
    return int(lib().pack_config_distance(a.ctypes.data_as(ip), b.ctypes.data_as(ip), cat.ctypes.data_as(u8p), a.size))


def opt_knn(feats, categorical, need, capacity: int, threshold: int, draws):
    """Groups as lists of indices in list order (the C ABI returns one group number per configuration)."""
    feats = _i32(feats).reshape(len(need), -1)
    cat = np.ascontiguousarray(categorical, dtype=np.uint8)
    need = np.ascontiguousarray(need, dtype=np.uint64)
    draws = np.ascontiguousarray(draws, dtype=np.float64)
    T, D = feats.shape
    assert draws.size >= T
    ids = np.zeros(T, dtype=np.int32)
    n = C.c_int32(0)
    ip = C.POINTER(C.c_int32)
    _check(lib().pack_opt_knn(feats.ctypes.data_as(ip), cat.ctypes.data_as(C.POINTER(C.c_uint8)), T, D,
                              need.ctypes.data_as(C.POINTER(C.c_uint64)), int(capacity), int(threshold),
                              draws.ctypes.data_as(C.POINTER(C.c_double)), ids.ctypes.data_as(ip), C.byref(n)))
    return _groups_from_ids(ids, n.value)


def opt_random(T: int, m: int, perm):
    perm = _i32(perm)
    ids = np.zeros(max(T, 1), dtype=np.int32)
    n = C.c_int32(0)
    ip = C.POINTER(C.c_int32)
    _check(lib().pack_opt_random(T, m, perm.ctypes.data_as(ip), ids.ctypes.data_as(ip), C.byref(n)))
    return _groups_from_ids(ids[:T], n.value)


def opt_batchsize(batch, need, capacity: int):
    batch = _i32(batch)
    need = np.ascontiguousarray(need, dtype=np.uint64)
    ids = np.zeros(max(batch.size, 1), dtype=np.int32)
    n = C.c_int32(0)
    ip = C.POINTER(C.c_int32)
    _check(lib().pack_opt_batchsize(batch.ctypes.data_as(ip), batch.size, need.ctypes.data_as(C.POINTER(C.c_uint64)),
                                    int(capacity), ids.ctypes.data_as(ip), C.byref(n)))
    return _groups_from_ids(ids[:batch.size], n.value)


def hyperband_plan(R: int, eta: int):
    """List of brackets, each a list of (n_i, r_i)."""
    cap = 4096
    n_out, r_out, rungs = np.zeros(cap, np.int32), np.zeros(cap, np.int32), np.zeros(64, np.int32)
    nb = C.c_int32(0)
    ip = C.POINTER(C.c_int32)
    _check(lib().pack_hyperband_plan(R, eta, n_out.ctypes.data_as(ip), r_out.ctypes.data_as(ip), rungs.ctypes.data_as(ip),
                                     cap, C.byref(nb)))
    out, at = [], 0
    for j in range(nb.value):
        out.append([(int(n_out[at + i]), int(r_out[at + i])) for i in range(rungs[j])])
        at += int(rungs[j])
    return out


def halving_keep(loss, keep: int):
    loss = np.ascontiguousarray(loss, dtype=np.float32)
    idx = np.zeros(max(keep, 1), dtype=np.int32)
    _check(lib().pack_halving_keep(_fptr(loss), loss.size, keep, idx.ctypes.data_as(C.POINTER(C.c_int32))))
    return [int(i) for i in idx[:keep]]


def estimate_bytes(B: int, in_shape, dtype: str, layers: list, batch: int, opt_kind: str = "sgd") -> int:
    arr = _layer_array(layers)
    spec = pack_model_spec(arr, len(layers), int(batch))
    inp = pack_input_spec(B, in_shape[0], in_shape[1], in_shape[2], PACK_BF16 if dtype == "bf16" else PACK_F32)
    return int(lib().pack_estimate_bytes(C.byref(inp), C.byref(spec), OPT_KINDS[opt_kind]))


CEILINGS = {"hbm_copy": 0, "mfma_bf16": 1, "mfma_fp32": 2}


def measure_ceiling(what: str, stream: int = 0) -> float:
    """GB/s of a streaming copy ("hbm_copy") or TFLOP/s of a register-resident matrix-instruction
    loop ("mfma_bf16", "mfma_fp32") on the current device."""
    out = C.c_double(0.0)
    _check(lib().pack_measure_ceiling(CEILINGS[what], C.c_void_p(stream), C.byref(out)))
    return out.value
