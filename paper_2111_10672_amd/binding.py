"""ctypes binding of libspb.so.  Same names as the C ABI; no arithmetic happens here."""
from __future__ import annotations

import ctypes as C
import os

HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(HERE, "libspb.so")
_lib = None

SPB_MAX_DIMS, SPB_MAX_STAGES, SPB_NAME_LEN = 64, 8, 48
SPB_OK = 0
ERRORS = {-1: "SPB_ERR_INVALID_ARG", -2: "SPB_ERR_DEPTH_RANGE", -3: "SPB_ERR_STATE",
          -4: "SPB_ERR_WORKSPACE", -5: "SPB_ERR_HIP", -6: "SPB_ERR_UNSUPPORTED"}
FAMILIES = {"mlp": 0, "resnet_basic": 1, "resnet_bottleneck": 2, "encoder": 3}
DTYPES = {"f32": 0, "bf16": 1}


class SpbError(RuntimeError):
    def __init__(self, code, message):
        super().__init__(f"{ERRORS.get(code, code)}: {message}")
        self.code = code


class spb_model_desc(C.Structure):
    _fields_ = [("family", C.c_int32), ("dtype", C.c_int32), ("batch", C.c_int32),
                ("n_dims", C.c_int32), ("dims", C.c_int32 * SPB_MAX_DIMS),
                ("image_h", C.c_int32), ("image_w", C.c_int32), ("image_c", C.c_int32),
                ("stem_kernel", C.c_int32), ("stem_stride", C.c_int32), ("stem_pad", C.c_int32),
                ("stem_pool", C.c_int32), ("stem_width", C.c_int32),
                ("n_stages", C.c_int32), ("stage_blocks", C.c_int32 * SPB_MAX_STAGES),
                ("stage_widths", C.c_int32 * SPB_MAX_STAGES), ("classes", C.c_int32),
                ("seq", C.c_int32), ("layers", C.c_int32), ("hidden", C.c_int32), ("heads", C.c_int32),
                ("ffn", C.c_int32), ("vocab", C.c_int32), ("loss_rows", C.c_int32)]


class spb_tensor_info(C.Structure):
    _fields_ = [("name", C.c_char * SPB_NAME_LEN), ("unit", C.c_int32), ("dtype", C.c_int32),
                ("ndim", C.c_int32), ("shape", C.c_int64 * 4), ("numel", C.c_int64)]


class spb_grad_view(C.Structure):
    _fields_ = [("param_index", C.c_int32), ("unit", C.c_int32), ("data", C.c_void_p), ("numel", C.c_int64)]


class spb_buffer_view(C.Structure):
    _fields_ = [("offset", C.c_int64), ("rows", C.c_int64), ("cols", C.c_int64), ("pitch", C.c_int64),
                ("dtype", C.c_int32), ("relu_applied", C.c_int32)]


class spb_kernel_time(C.Structure):
    _fields_ = [("name", C.c_char * SPB_NAME_LEN), ("launches", C.c_int64), ("total_ms", C.c_double),
                ("flops", C.c_double), ("bytes", C.c_double)]


class spb_sched_job(C.Structure):
    _fields_ = [("arrival", C.c_double), ("model_size", C.c_double), ("iterations", C.c_int32), ("workers", C.c_int32),
                ("durations", C.POINTER(C.c_double)), ("resources", C.POINTER(C.c_double))]


class spb_sched_task(C.Structure):
    _fields_ = [("job", C.c_int32), ("iteration", C.c_int32), ("worker", C.c_int32), ("machine", C.c_int32),
                ("moved", C.c_int32), ("start", C.c_double), ("end", C.c_double), ("held_until", C.c_double)]


EXPORTS = {
    "spb_last_error": (C.c_char_p, []),
    "spb_model_create": (C.c_int, [C.POINTER(spb_model_desc), C.POINTER(C.c_void_p)]),
    "spb_model_destroy": (C.c_int, [C.c_void_p]),
    "spb_num_units": (C.c_int, [C.c_void_p, C.POINTER(C.c_int32)]),
    "spb_param_count": (C.c_int, [C.c_void_p, C.POINTER(C.c_int32)]),
    "spb_param_info": (C.c_int, [C.c_void_p, C.c_int32, C.POINTER(spb_tensor_info)]),
    "spb_bind_params": (C.c_int, [C.c_void_p, C.POINTER(C.c_void_p), C.c_int32]),
    "spb_bind_grads": (C.c_int, [C.c_void_p, C.POINTER(C.c_void_p), C.c_int32]),
    "spb_workspace_size": (C.c_int, [C.c_void_p, C.c_int32, C.POINTER(C.c_size_t)]),
    "spb_forward": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p,
                              C.c_size_t, C.c_void_p, C.c_void_p]),
    "spb_forward_static": (C.c_int, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p]),
    "spb_backward_truncated": (C.c_int, [C.c_void_p, C.c_int32, C.c_void_p]),
    "spb_grad_buffers": (C.c_int, [C.c_void_p, C.c_int32, C.POINTER(spb_grad_view), C.c_int32, C.POINTER(C.c_int32)]),
    "spb_unit_io": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32, C.POINTER(spb_buffer_view), C.POINTER(spb_buffer_view)]),
    "spb_zero_absent_grads": (C.c_int, [C.c_void_p, C.c_int32, C.c_void_p]),
    "spb_worker_depth": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32, C.POINTER(C.c_int32)]),
    "spb_aggregate_update": (C.c_int, [C.c_void_p, C.c_int32, C.POINTER(C.c_int32), C.POINTER(C.c_void_p), C.POINTER(C.c_void_p),
                                       C.c_float, C.c_float, C.c_float, C.c_int32, C.c_void_p]),
    "spb_set_kernel_timing": (C.c_int, [C.c_void_p, C.c_int32]),
    "spb_replay_kernel": (C.c_int, [C.c_void_p, C.c_char_p, C.c_int32, C.c_void_p]),
    "spb_read_kernel_timing": (C.c_int, [C.c_void_p, C.POINTER(spb_kernel_time), C.c_int32, C.POINTER(C.c_int32)]),
    "spb_schedule_tasks": (C.c_int, [C.POINTER(spb_sched_job), C.c_int32, C.c_int32, C.c_double, C.c_double, C.c_int32,
                                     C.POINTER(spb_sched_task), C.c_int64, C.POINTER(C.c_int64), C.POINTER(C.c_double)]),
}


def library_path() -> str:
    return _LIB_PATH


def lib():
    """Load libspb.so; build it first only if it does not exist.  No fallback: raises if it cannot load."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            from .build import build_library
            build_library()
        handle = C.CDLL(_LIB_PATH)
        for name, (res, args) in EXPORTS.items():
            fn = getattr(handle, name)
            fn.restype, fn.argtypes = res, args
        _lib = handle
    return _lib


def spb_last_error() -> str:
    return lib().spb_last_error().decode()


def _check(code):
    if code != SPB_OK:
        raise SpbError(code, spb_last_error())


def desc_from_config(cfg: dict) -> spb_model_desc:
    d = spb_model_desc()
    d.family, d.dtype, d.batch = FAMILIES[cfg["family"]], DTYPES[cfg["dtype"]], cfg["batch"]
    if cfg["family"] == "mlp":
        d.n_dims = len(cfg["dims"])
        for i, w in enumerate(cfg["dims"]):
            d.dims[i] = w
    elif cfg["family"].startswith("resnet"):
        d.image_h, d.image_w, d.image_c = cfg["image"]
        st = cfg["stem"]
        d.stem_kernel, d.stem_stride, d.stem_pad = st["kernel"], st["stride"], st["pad"]
        d.stem_pool, d.stem_width = int(st["pool"]), st["width"]
        d.n_stages = len(cfg["stage_blocks"])
        for i, (b, w) in enumerate(zip(cfg["stage_blocks"], cfg["stage_widths"])):
            d.stage_blocks[i], d.stage_widths[i] = b, w
        d.classes = cfg["classes"]
    else:
        for key in ("seq", "layers", "hidden", "heads", "ffn", "vocab", "loss_rows"):
            setattr(d, key, cfg[key])
    return d


def _ptr(t):
    """Device (or null) pointer of a torch tensor / int / None."""
    if t is None:
        return None
    if isinstance(t, int):
        return C.c_void_p(t)
    return C.c_void_p(t.data_ptr())


def spb_model_create(desc: spb_model_desc) -> C.c_void_p:
    out = C.c_void_p()
    _check(lib().spb_model_create(C.byref(desc), C.byref(out)))
    return out


def spb_model_destroy(m):
    _check(lib().spb_model_destroy(m))


def spb_num_units(m) -> int:
    n = C.c_int32()
    _check(lib().spb_num_units(m, C.byref(n)))
    return n.value


def spb_param_count(m) -> int:
    n = C.c_int32()
    _check(lib().spb_param_count(m, C.byref(n)))
    return n.value


def spb_param_info(m, index: int) -> dict:
    info = spb_tensor_info()
    _check(lib().spb_param_info(m, index, C.byref(info)))
    return {"name": info.name.decode(), "unit": info.unit, "dtype": "f32" if info.dtype == 0 else "bf16",
            "shape": tuple(info.shape[i] for i in range(info.ndim)), "numel": info.numel}


def _ptr_array(tensors):
    arr = (C.c_void_p * len(tensors))()
    for i, t in enumerate(tensors):
        arr[i] = None if t is None else (t if isinstance(t, int) else t.data_ptr())
    return arr


def spb_bind_params(m, tensors):
    _check(lib().spb_bind_params(m, _ptr_array(tensors), len(tensors)))


def spb_bind_grads(m, tensors):
    _check(lib().spb_bind_grads(m, _ptr_array(tensors), len(tensors)))


def spb_workspace_size(m, k: int) -> int:
    n = C.c_size_t()
    _check(lib().spb_workspace_size(m, k, C.byref(n)))
    return n.value


def spb_forward(m, x, labels, loss_rows, k, workspace, workspace_bytes, loss_out, stream):
    _check(lib().spb_forward(m, _ptr(x), _ptr(labels), _ptr(loss_rows), k, _ptr(workspace),
                             workspace_bytes, _ptr(loss_out), C.c_void_p(stream)))


SPB_STATIC_WORKSPACE_BYTES = 8 << 20


def spb_forward_static(m, x, labels, loss_rows, k, loss_out, stream):
    _check(lib().spb_forward_static(m, _ptr(x), _ptr(labels), _ptr(loss_rows), k, _ptr(loss_out), C.c_void_p(stream)))


def spb_backward_truncated(m, k, stream):
    _check(lib().spb_backward_truncated(m, k, C.c_void_p(stream)))


def spb_grad_buffers(m, k, cap=None):
    cap = spb_param_count(m) if cap is None else cap
    views = (spb_grad_view * max(cap, 1))()
    n = C.c_int32()
    _check(lib().spb_grad_buffers(m, k, views, cap, C.byref(n)))
    return [{"param_index": v.param_index, "unit": v.unit, "data": v.data, "numel": v.numel} for v in views[:n.value]]


SPB_VIEW_CALLER_INPUT, SPB_VIEW_NONE = -1, -2


def spb_unit_io(m, k: int, unit: int):
    """(input view, output-gradient view) of a unit as dicts; see spb.h."""
    a, b = spb_buffer_view(), spb_buffer_view()
    _check(lib().spb_unit_io(m, k, unit, C.byref(a), C.byref(b)))
    as_dict = lambda v: {"offset": v.offset, "rows": v.rows, "cols": v.cols, "pitch": v.pitch,
                         "dtype": {0: "f32", 1: "bf16", 2: "i32"}[v.dtype], "relu_applied": bool(v.relu_applied)}
    return as_dict(a), as_dict(b)


def spb_zero_absent_grads(m, k, stream):
    _check(lib().spb_zero_absent_grads(m, k, C.c_void_p(stream)))


def spb_worker_depth(m, j: int, n_workers: int) -> int:
    k = C.c_int32()
    _check(lib().spb_worker_depth(m, j, n_workers, C.byref(k)))
    return k.value


def spb_aggregate_update(m, depths, worker_grads, velocity, lr, momentum, weight_decay, scale_lr, stream):
    """worker_grads: one list per worker, each with one tensor (or None) per parameter; velocity: one tensor per parameter."""
    n = len(depths)
    d = (C.c_int32 * n)(*depths)
    flat = [g for per_worker in worker_grads for g in per_worker]
    _check(lib().spb_aggregate_update(m, n, d, _ptr_array(flat), _ptr_array(velocity), lr, momentum, weight_decay,
                                      int(bool(scale_lr)), C.c_void_p(stream)))


def spb_set_kernel_timing(m, enable: bool):
    _check(lib().spb_set_kernel_timing(m, int(enable)))


def spb_replay_kernel(m, name: str, count: int, stream):
    _check(lib().spb_replay_kernel(m, name.encode(), count, C.c_void_p(stream)))


def spb_read_kernel_timing(m, cap=1024):
    recs = (spb_kernel_time * cap)()
    n = C.c_int32()
    _check(lib().spb_read_kernel_timing(m, recs, cap, C.byref(n)))
    return [{"name": r.name.decode(), "launches": r.launches, "total_ms": r.total_ms, "flops": r.flops,
             "bytes": r.bytes} for r in recs[:n.value]]


def spb_schedule_tasks(jobs, n_machines: int, gamma: float = 0.0, capacity: float = 1.0, gang: bool = False):
    """jobs: list of dict(arrival, iterations, model_size, durations[w], resources[w]) -> (placements, makespan),
    placements as dicts in the order the library placed them (host computation, no GPU)."""
    arr = (spb_sched_job * max(1, len(jobs)))()
    keep = []
    total = 0
    for a, job in zip(arr, jobs):
        w = len(job["durations"])
        if len(job["resources"]) != w:
            raise ValueError("one duration and one resource per worker")
        d = (C.c_double * max(1, w))(*[float(v) for v in job["durations"]])
        r = (C.c_double * max(1, w))(*[float(v) for v in job["resources"]])
        keep += [d, r]
        a.arrival, a.model_size, a.iterations, a.workers = float(job["arrival"]), float(job["model_size"]), int(job["iterations"]), w
        a.durations, a.resources = d, r
        total += w * max(0, int(job["iterations"]))
    out = (spb_sched_task * max(1, total))()
    n, makespan = C.c_int64(), C.c_double()
    _check(lib().spb_schedule_tasks(arr, len(jobs), int(n_machines), float(gamma), float(capacity), int(bool(gang)), out, total,
                                    C.byref(n), C.byref(makespan)))
    return ([dict(job=t.job, iteration=t.iteration, worker=t.worker, machine=t.machine, start=t.start, end=t.end,
                  held_until=t.held_until, moved=bool(t.moved)) for t in out[:n.value]], makespan.value)


class SpbModel:
    """Convenience holder: a model handle plus the torch tensors bound to it (memory and stream plumbing only)."""

    def __init__(self, cfg: dict, params: dict, device="cuda:0"):
        import torch
        self.torch = torch
        self.cfg = cfg
        self.device = torch.device(device)
        if self.device.type != "cuda" or not torch.cuda.is_available():
            raise RuntimeError("the SPB path needs a GPU; there is no host fallback")
        self.handle = spb_model_create(desc_from_config(cfg))
        self.n_units = spb_num_units(self.handle)
        self.infos = [spb_param_info(self.handle, i) for i in range(spb_param_count(self.handle))]
        self.params, self.grads = [], []
        for info in self.infos:
            src = params[info["name"]]
            if tuple(src.shape) != info["shape"]:
                raise ValueError(f"{info['name']}: shape {tuple(src.shape)} != {info['shape']}")
            self.params.append(src.to(self.device).contiguous())
            self.grads.append(torch.empty(info["shape"], dtype=torch.float32, device=self.device))
        spb_bind_params(self.handle, self.params)
        spb_bind_grads(self.handle, self.grads)
        self.loss = torch.zeros(1, dtype=torch.float32, device=self.device)
        self.workspace = None
        self.workspace_bytes = 0

    def reserve(self, k: int):
        need = spb_workspace_size(self.handle, k)
        if need > self.workspace_bytes:
            self.workspace = self.torch.empty(need, dtype=self.torch.uint8, device=self.device)
            self.workspace_bytes = need
        return need

    def stream(self) -> int:
        return self.torch.cuda.current_stream(self.device).cuda_stream

    def forward(self, batch: dict, k: int):
        self.reserve(k)
        spb_forward(self.handle, batch["x"], batch["labels"], batch.get("loss_rows"), k, self.workspace,
                    self.workspace_bytes, self.loss, self.stream())

    def forward_static(self, batch: dict, k: int):
        """The forward pass on the library's own fixed-size workspace (allocates nothing)."""
        spb_forward_static(self.handle, batch["x"], batch["labels"], batch.get("loss_rows"), k, self.loss, self.stream())

    def backward(self, k: int):
        spb_backward_truncated(self.handle, k, self.stream())

    def step(self, batch: dict, k: int):
        self.forward(batch, k)
        self.backward(k)

    def grad_dict(self, k: int) -> dict:
        """name -> float32 tensor view of the buffers spb_grad_buffers lists at depth k."""
        out = {}
        for v in spb_grad_buffers(self.handle, k):
            g = self.grads[v["param_index"]]
            assert g.data_ptr() == v["data"] and g.numel() == v["numel"]
            out[self.infos[v["param_index"]]["name"]] = g
        return out

    def read_view(self, view: dict, batch: dict = None):
        """The tensor a spb_unit_io view describes, copied out of the workspace as a float64 (ids: int64) CPU tensor
        [rows, cols]; None for SPB_VIEW_NONE."""
        torch = self.torch
        if view["offset"] == SPB_VIEW_NONE:
            return None
        if view["offset"] == SPB_VIEW_CALLER_INPUT:
            x = batch["x"].detach().cpu()
            return x.reshape(view["rows"], -1).long() if view["dtype"] == "i32" else x.reshape(view["rows"], -1).double()
        tdtype, size = {"f32": (torch.float32, 4), "bf16": (torch.bfloat16, 2)}[view["dtype"]]
        nbytes = ((view["rows"] - 1) * view["pitch"] + view["cols"]) * size
        raw = self.workspace[view["offset"]:view["offset"] + nbytes].view(tdtype)
        return torch.as_strided(raw, (view["rows"], view["cols"]), (view["pitch"], 1)).double().cpu()

    def close(self):
        if self.handle is not None:
            spb_model_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
