"""ctypes binding of libaccudnn.so: argument marshalling only.

Every step of the training path runs inside the library's kernels and host code.
torch is used here for device memory, pinned host memory and streams, as the C ABI
asks the caller to own them.  There is no fallback: if the library is missing the
import of this module raises.
"""
import ctypes as C
import os
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libaccudnn.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is not built: run `python -m paper_1901_06773_amd.build` "
        "(or __graft_entry__.build()); there is no fallback path")
_lib = C.CDLL(LIB_PATH)

ACC_OK, ACC_EINVAL, ACC_EUNTRAINABLE, ACC_EPOOL, ACC_EHOSTMEM, ACC_EHIP, ACC_ESTATE = 0, -1, -2, -3, -4, -5, -6
PLAN_NONE, PLAN_NAIVE_ALL, PLAN_DYNAMIC = 0, 1, 2
LOC_HOST, LOC_DEVICE = 0, 1
F32, BF16 = 0, 1
DEBUG_POISON = 1
STATUS_NAMES = {0: "ACC_OK", -1: "ACC_EINVAL", -2: "ACC_EUNTRAINABLE", -3: "ACC_EPOOL",
                -4: "ACC_EHOSTMEM", -5: "ACC_EHIP", -6: "ACC_ESTATE"}


class AccError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"{STATUS_NAMES.get(status, status)}: {text}")
        self.status = status


class acc_layer(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("kind", "in0", "in1", "cin", "cout", "r", "s", "stride", "pad")]


class acc_resources(C.Structure):
    _fields_ = [("pool", C.c_void_p), ("pool_bytes", C.c_size_t), ("host", C.c_void_p),
                ("host_bytes", C.c_size_t), ("s_compute", C.c_void_p), ("s_out", C.c_void_p),
                ("s_in", C.c_void_p), ("s_wgrad", C.c_void_p)]


class acc_plan_summary(C.Structure):
    _fields_ = [("n_steps", C.c_int32), ("n_maps", C.c_int32), ("n_swapped", C.c_int32),
                ("n_instr", C.c_int32), ("bytes_swapped", C.c_uint64), ("bytes_maps", C.c_uint64),
                ("static_bytes", C.c_uint64), ("peak_bytes", C.c_uint64),
                ("layer_peak_bytes", C.c_uint64), ("noswap_peak_bytes", C.c_uint64),
                ("host_bytes", C.c_uint64), ("t_compute", C.c_double), ("t_iter", C.c_double),
                ("t_stall", C.c_double), ("plan_ms", C.c_double)]

    def as_dict(self):
        return {n: getattr(self, n) for n, _ in self._fields_}


class acc_tune_result(C.Structure):
    _fields_ = [("k_best", C.c_int32), ("k_trainable_max", C.c_int32), ("k_noswap_max", C.c_int32),
                ("n_evaluated", C.c_int32), ("images_per_s", C.c_double), ("t_iter", C.c_double),
                ("t_stall", C.c_double), ("tune_ms", C.c_double)]

    def as_dict(self):
        return {n: getattr(self, n) for n, _ in self._fields_}


class acc_step_info(C.Structure):
    _fields_ = [("kind", C.c_int32), ("layer", C.c_int32), ("backward", C.c_int32),
                ("reserved", C.c_int32), ("flops", C.c_double), ("t_compute", C.c_double),
                ("t_ready", C.c_double), ("t_start", C.c_double), ("t_end", C.c_double)]


class acc_tensor_info(C.Structure):
    _fields_ = [("kind", C.c_int32), ("producer_step", C.c_int32), ("last_fwd_step", C.c_int32),
                ("first_bwd_step", C.c_int32), ("last_step", C.c_int32), ("is_map", C.c_int32),
                ("swapped", C.c_int32), ("reserved", C.c_int32), ("bytes", C.c_uint64),
                ("offset", C.c_uint64), ("offset2", C.c_uint64), ("host_offset", C.c_uint64)]


class acc_stats(C.Structure):
    _fields_ = [("step_ms", C.c_double), ("host_issue_ms", C.c_double), ("peak_pool_bytes", C.c_uint64),
                ("bytes_out", C.c_uint64), ("bytes_in", C.c_uint64), ("d2h_ms", C.c_double),
                ("h2d_ms", C.c_double), ("steps_run", C.c_uint64), ("touched_pool_bytes", C.c_uint64),
                ("peak_is_measured", C.c_int32), ("reserved", C.c_int32), ("host_wait_ms", C.c_double)]

    def as_dict(self):
        return {n: getattr(self, n) for n, _ in self._fields_}


class acc_instr(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("op", "arg", "wait_step", "wait_d2h", "wait_h2d", "seq", "record",
                                          "reserved")]


class acc_timeline_entry(C.Structure):
    _fields_ = [("op", C.c_int32), ("arg", C.c_int32), ("bytes", C.c_uint64), ("t_start", C.c_double),
                ("t_end", C.c_double)]


class acc_kernel_profile(C.Structure):
    _fields_ = [("name", C.c_char * 48), ("launches", C.c_int32), ("reserved", C.c_int32),
                ("ms", C.c_double), ("flops", C.c_double)]


class acc_launch_profile(C.Structure):
    _fields_ = [("step", C.c_int32), ("layer", C.c_int32), ("role", C.c_int32), ("variant", C.c_int32),
                ("ms", C.c_double), ("flops", C.c_double)]


# every symbol include/accudnn.h declares, with its signature
_VP, _I, _SZ, _F, _D = C.c_void_p, C.c_int, C.c_size_t, C.c_float, C.c_double
_PROTOS = {
    "acc_create": (_I, [C.POINTER(acc_layer), _I, _I, _I, _I, _I, C.POINTER(acc_resources), C.POINTER(_VP)]),
    "acc_destroy": (None, [_VP]),
    "acc_last_error": (C.c_char_p, [_VP]),
    "acc_step_kind_name": (C.c_char_p, [_I]),
    "acc_set_weights": (_I, [_VP, _I, _VP, _SZ]),
    "acc_get_weights": (_I, [_VP, _I, _VP, _SZ]),
    "acc_get_grads": (_I, [_VP, _I, _VP, _SZ]),
    "acc_param_count": (_I, [_VP, _I, C.POINTER(_SZ)]),
    "acc_calibrate": (_I, [_VP, C.POINTER(_I), _I]),
    "acc_set_cost_model": (_I, [_VP, _D, _D, _D, _D, _D, _D]),
    "acc_set_step_times": (_I, [_VP, C.POINTER(_D), _I]),
    "acc_get_calibration": (_I, [_VP, C.POINTER(_I), _I, C.POINTER(_D), _SZ, C.POINTER(_D)]),
    "acc_set_calibration": (_I, [_VP, C.POINTER(_I), _I, C.POINTER(_D), C.POINTER(_D)]),
    "acc_plan_swaps": (_I, [_VP, _I, _SZ, _I, C.POINTER(acc_plan_summary)]),
    "acc_tune_minibatch": (_I, [_VP, _SZ, _I, _I, C.POINTER(acc_tune_result), C.POINTER(acc_plan_summary)]),
    "acc_adaptive_lr": (_D, [_D, _D, _D]),
    "acc_plan_explicit": (_I, [_VP, _I, _SZ, C.POINTER(C.c_uint8), _I, C.POINTER(acc_plan_summary)]),
    "acc_get_step_count": (_I, [_VP]),
    "acc_get_tensor_count": (_I, [_VP]),
    "acc_get_step_info": (_I, [_VP, _I, C.POINTER(acc_step_info)]),
    "acc_get_tensor_info": (_I, [_VP, _I, C.POINTER(acc_tensor_info)]),
    "acc_get_step_io": (_I, [_VP, _I, C.POINTER(C.c_int32), _I, C.POINTER(C.c_int32), _I]),
    "acc_get_instr_count": (_I, [_VP]),
    "acc_get_instr": (_I, [_VP, _I, C.POINTER(acc_instr)]),
    "acc_get_timeline": (_I, [_VP, _I, C.POINTER(acc_timeline_entry), _I]),
    "acc_train_step": (_I, [_VP, _VP, _I, _VP, _F, C.POINTER(_F)]),
    "acc_get_stats": (_I, [_VP, C.POINTER(acc_stats)]),
    "acc_set_profiling": (_I, [_VP, _I]),
    "acc_set_debug": (_I, [_VP, _I]),
    "acc_set_graph": (_I, [_VP, _I]),
    "acc_capture_output": (_I, [_VP, _I, _VP, _SZ]),
    "acc_inject_output": (_I, [_VP, _I, _VP, _SZ]),
    "acc_set_wgrad_overlap": (_I, [_VP, _I]),
    "acc_get_step_times_ms": (_I, [_VP, C.POINTER(_D), _I]),
    "acc_get_kernel_profile": (_I, [_VP, C.POINTER(acc_kernel_profile), _I]),
    "acc_get_launch_profile": (_I, [_VP, C.POINTER(acc_launch_profile), _I]),
    "acc_op_conv_workspace": (_SZ, [_I] * 9),
    "acc_op_conv_fwd": (_I, [_VP, _VP, _VP] + [_I] * 9 + [_I, _VP]),
    "acc_op_conv_dgrad": (_I, [_VP, _VP, _VP] + [_I] * 10 + [_VP, _SZ, _I, _VP]),
    "acc_op_conv_wgrad": (_I, [_VP, _VP, _VP] + [_I] * 9 + [_VP, _SZ, _I, _VP]),
    "acc_op_bn_workspace": (_SZ, [_I]),
    "acc_op_bn_fwd": (_I, [_VP] * 7 + [_I, _I, _I, _F, _VP, _I, _VP]),
    "acc_op_bn_bwd": (_I, [_VP] * 10 + [_I, _I, _VP, _I, _VP]),
    "acc_op_bn_fwd_noalloc": (_I, [_VP] * 7 + [_I, _I, _I, _F, _I, _VP]),
    "acc_op_maxpool_fwd": (_I, [_VP, _VP] + [_I] * 8 + [_VP]),
    "acc_op_maxpool_bwd": (_I, [_VP, _VP, _VP] + [_I] * 9 + [_VP]),
    "acc_op_gap_fwd": (_I, [_VP, _VP, _I, _I, _I, _I, _VP]),
    "acc_op_gap_bwd": (_I, [_VP, _VP, _I, _I, _I, _I, _I, _VP]),
    "acc_op_softmax_ce": (_I, [_VP] * 5 + [_I, _I, _I, _VP]),
}
for _name, (_res, _args) in _PROTOS.items():
    _fn = getattr(_lib, _name)
    _fn.restype = _res
    _fn.argtypes = _args

EXPORTED_SYMBOLS = sorted(_PROTOS)


def lib():
    return _lib


def adaptive_lr(lr_base: float, c: float, q: float) -> float:
    """Eq. 9."""
    return float(_lib.acc_adaptive_lr(float(lr_base), float(c), float(q)))


def _layers_array(spec_array: np.ndarray):
    recs = np.ascontiguousarray(spec_array, np.int32)
    assert recs.ndim == 2 and recs.shape[1] == 9
    arr = (acc_layer * recs.shape[0])()
    C.memmove(arr, recs.ctypes.data, recs.nbytes)
    return arr, recs.shape[0]


class Context:
    """One network on one GPU (or, with pool_bytes=None, a planning-only context)."""

    def __init__(self, spec_array: np.ndarray, in_chw: Sequence[int], pool_bytes: Optional[int] = None,
                 host_bytes: int = 0, device: str = "cuda:0", dtype: int = F32, wgrad_stream: bool = True):
        self._h = _VP()
        self.dtype = int(dtype)
        self._keep = []
        arr, n = _layers_array(spec_array)
        self.n_layers = n
        res_ptr = None
        if pool_bytes is not None:
            import torch
            self.torch = torch
            self.device = torch.device(device)
            torch.cuda.set_device(self.device)
            self.pool = torch.empty(int(pool_bytes), dtype=torch.uint8, device=self.device)
            self.host = torch.empty(max(int(host_bytes), 256), dtype=torch.uint8, pin_memory=True)
            # compute, swap-out, swap-in, weight gradients; all at the default priority
            self.streams = [torch.cuda.Stream(device=self.device) for _ in range(4 if wgrad_stream else 3)]
            res = acc_resources(self.pool.data_ptr(), self.pool.numel(), self.host.data_ptr(), self.host.numel(),
                                self.streams[0].cuda_stream, self.streams[1].cuda_stream,
                                self.streams[2].cuda_stream, self.streams[3].cuda_stream if wgrad_stream else None)
            res_ptr = C.byref(res)
            torch.cuda.synchronize(self.device)
        rc = _lib.acc_create(arr, n, int(in_chw[0]), int(in_chw[1]), int(in_chw[2]), self.dtype, res_ptr, C.byref(self._h))
        if rc != ACC_OK:
            raise AccError(rc, _lib.acc_last_error(None).decode())

    # ---- plumbing
    def _check(self, rc: int):
        if rc < 0:
            raise AccError(rc, _lib.acc_last_error(self._h).decode())
        return rc

    def close(self):
        if self._h:
            _lib.acc_destroy(self._h)
            self._h = _VP()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- weights
    def param_count(self, layer: int) -> int:
        n = _SZ(0)
        self._check(_lib.acc_param_count(self._h, layer, C.byref(n)))
        return n.value

    def set_weights(self, params: List[np.ndarray]):
        for i, p in enumerate(params):
            if p.size:
                p = np.ascontiguousarray(p, np.float32)
                self._check(_lib.acc_set_weights(self._h, i, p.ctypes.data, p.size))

    def _get(self, fn) -> List[np.ndarray]:
        out = []
        for i in range(self.n_layers):
            n = self.param_count(i)
            a = np.zeros(n, np.float32)
            if n:
                self._check(fn(self._h, i, a.ctypes.data, n))
            out.append(a)
        return out

    def get_weights(self) -> List[np.ndarray]:
        return self._get(_lib.acc_get_weights)

    def get_grads(self) -> List[np.ndarray]:
        return self._get(_lib.acc_get_grads)

    # ---- cost model and planning
    def calibrate(self, ks: Sequence[int]):
        arr = (_I * len(ks))(*[int(k) for k in ks])
        self._check(_lib.acc_calibrate(self._h, arr, len(ks)))

    def set_cost_model(self, flops_per_s, bytes_per_s, launch_s, d2h_bps, h2d_bps, copy_latency_s):
        self._check(_lib.acc_set_cost_model(self._h, flops_per_s, bytes_per_s, launch_s, d2h_bps, h2d_bps,
                                            copy_latency_s))

    def set_step_times(self, seconds: Sequence[float]):
        arr = (_D * len(seconds))(*[float(s) for s in seconds])
        self._check(_lib.acc_set_step_times(self._h, arr, len(seconds)))

    def get_calibration(self) -> dict:
        """Measured table of calibrate(): {"ks": [...], "seconds": array [nk, n_steps], "link": (d2h, h2d, latency)}."""
        link = (_D * 3)()
        nk = self._check(_lib.acc_get_calibration(self._h, None, 0, None, 0, link))
        ns = self.step_count()
        ks = (_I * max(nk, 1))()
        sec = (_D * max(nk * ns, 1))()
        self._check(_lib.acc_get_calibration(self._h, ks, nk, sec, nk * ns, link))
        return dict(ks=list(ks[:nk]), seconds=np.array(sec[:nk * ns], dtype=np.float64).reshape(nk, ns),
                    link=tuple(link[:]))

    def set_calibration(self, ks: Sequence[int], seconds, link=None):
        seconds = np.ascontiguousarray(seconds, np.float64)
        assert seconds.shape == (len(ks), self.step_count())
        ka = (_I * len(ks))(*[int(k) for k in ks])
        la = (_D * 3)(*[float(x) for x in link]) if link is not None else None
        self._check(_lib.acc_set_calibration(self._h, ka, len(ks), seconds.ctypes.data_as(C.POINTER(_D)), la))

    def plan_swaps(self, minibatch: int, budget_bytes: int, mode: int = PLAN_DYNAMIC) -> dict:
        s = acc_plan_summary()
        self._check(_lib.acc_plan_swaps(self._h, int(minibatch), int(budget_bytes), int(mode), C.byref(s)))
        self.k = int(minibatch)
        return s.as_dict()

    def tune_minibatch(self, budget_bytes: int, k_lo: int, k_hi: int):
        """Algorithm 2 / Eq. 7: returns (tune result, plan summary); the winner's plan is installed."""
        r, s = acc_tune_result(), acc_plan_summary()
        self._check(_lib.acc_tune_minibatch(self._h, int(budget_bytes), int(k_lo), int(k_hi), C.byref(r), C.byref(s)))
        self.k = int(r.k_best)
        return r.as_dict(), s.as_dict()

    def plan_explicit(self, minibatch: int, budget_bytes: int, swap: Sequence[int]) -> dict:
        s = acc_plan_summary()
        arr = (C.c_uint8 * len(swap))(*[1 if x else 0 for x in swap])
        self._check(_lib.acc_plan_explicit(self._h, int(minibatch), int(budget_bytes), arr, len(swap), C.byref(s)))
        self.k = int(minibatch)
        return s.as_dict()

    def step_count(self) -> int:
        return self._check(_lib.acc_get_step_count(self._h))

    def tensor_count(self) -> int:
        return self._check(_lib.acc_get_tensor_count(self._h))

    def step_info(self, j: int) -> dict:
        s = acc_step_info()
        self._check(_lib.acc_get_step_info(self._h, j, C.byref(s)))
        d = {n: getattr(s, n) for n, _ in s._fields_ if n != "reserved"}
        d["name"] = _lib.acc_step_kind_name(s.kind).decode()
        return d

    def tensor_info(self, t: int) -> dict:
        s = acc_tensor_info()
        self._check(_lib.acc_get_tensor_info(self._h, t, C.byref(s)))
        return {n: getattr(s, n) for n, _ in s._fields_ if n != "reserved"}

    def step_io(self, j: int):
        r = (C.c_int32 * 16)()
        w = (C.c_int32 * 16)()
        rc = self._check(_lib.acc_get_step_io(self._h, j, r, 16, w, 16))
        return list(r[: rc // 256]), list(w[: rc % 256])

    def instructions(self) -> list:
        """The plan's instruction list as dicts (op, arg, wait_step, wait_d2h, wait_h2d, seq, record)."""
        out = []
        ins = acc_instr()
        for i in range(self._check(_lib.acc_get_instr_count(self._h))):
            self._check(_lib.acc_get_instr(self._h, i, C.byref(ins)))
            out.append({n: getattr(ins, n) for n, _ in ins._fields_ if n != "reserved"})
        return out

    def timeline(self, observed: bool = False) -> list:
        """One dict per instruction of the plan (op, arg, bytes, t_start, t_end in seconds after the
        start of the iteration): predicted by the planner's simulation, or observed in the last
        train_step that ran with profiling level 1 or 3."""
        n = self._check(_lib.acc_get_instr_count(self._h))
        arr = (acc_timeline_entry * max(n, 1))()
        n = self._check(_lib.acc_get_timeline(self._h, 1 if observed else 0, arr, n))
        return [dict(op=arr[i].op, arg=arr[i].arg, bytes=arr[i].bytes, t_start=arr[i].t_start, t_end=arr[i].t_end)
                for i in range(n)]

    # ---- execution
    def train_step(self, images, labels: np.ndarray, lr: float) -> float:
        """images: torch tensor fp32 NCHW contiguous, pinned host or device."""
        assert images.dtype == self.torch.float32 and images.is_contiguous()
        loc = LOC_DEVICE if images.is_cuda else LOC_HOST
        labels = np.ascontiguousarray(labels, np.int32)
        loss = _F(0.0)
        self._check(_lib.acc_train_step(self._h, images.data_ptr(), loc, labels.ctypes.data, float(lr), C.byref(loss)))
        return float(loss.value)

    def stats(self) -> dict:
        s = acc_stats()
        self._check(_lib.acc_get_stats(self._h, C.byref(s)))
        return s.as_dict()

    def set_wgrad_overlap(self, on: bool):
        """Weight gradients on their own stream beside the data gradients (default), or on the compute stream."""
        self._check(_lib.acc_set_wgrad_overlap(self._h, 1 if on else 0))

    def set_debug(self, poison: bool):
        """Verification mode: NaN-poison everything the plan has released or not yet brought back,
        and measure the pool's high-water mark after every step."""
        self._check(_lib.acc_set_debug(self._h, DEBUG_POISON if poison else 0))

    def capture_outputs(self, layers: Sequence[int], shapes: dict, k: int) -> dict:
        """Registers pinned buffers for the stored outputs of `layers` (shapes: layer -> (c, h, w));
        returns {layer: torch tensor [k, h, w, c] in the storage type}, filled by every train_step."""
        torch = self.torch
        dt = torch.bfloat16 if self.dtype == BF16 else torch.float32
        out = {}
        for l in layers:
            c, h, w = shapes[l]
            buf = torch.empty((k, h, w, c), dtype=dt, pin_memory=True)
            self._check(_lib.acc_capture_output(self._h, int(l), buf.data_ptr(), buf.numel() * buf.element_size()))
            out[l] = buf
        self._keep.append(out)
        return out

    def inject_outputs(self, values: dict, buffers: Optional[dict] = None):
        """values: layer -> numpy array [k, h, w, c] float32 (device layout); every train_step from now
        on overwrites the stored output of those layers with them right after it is produced.
        buffers: pinned tensors of that shape to stage them in (e.g. those of capture_outputs, once
        the captures are stopped); new ones are allocated otherwise."""
        torch = self.torch
        dt = torch.bfloat16 if self.dtype == BF16 else torch.float32
        keep = {}
        for l, v in values.items():
            src = torch.from_numpy(np.ascontiguousarray(v, np.float32))
            if buffers is not None:
                buf = buffers[l]
                buf.copy_(src.reshape(buf.shape))
            else:
                buf = src.to(dt).pin_memory()
            self._check(_lib.acc_inject_output(self._h, int(l), buf.data_ptr(), buf.numel() * buf.element_size()))
            keep[l] = buf
        self._keep.append(keep)

    def stop_captures(self):
        self._check(_lib.acc_capture_output(self._h, -1, None, 0))
        self._check(_lib.acc_inject_output(self._h, -1, None, 0))

    def set_graph(self, on: bool):
        """Record the compute part of an iteration that swaps nothing into a HIP graph and replay it."""
        self._check(_lib.acc_set_graph(self._h, 1 if on else 0))

    def set_profiling(self, level: int):
        """0 off, 1 per step and copy, 2 per convolution kernel launch, 3 both."""
        self._check(_lib.acc_set_profiling(self._h, int(level)))

    def kernel_profile(self) -> list:
        arr = (acc_kernel_profile * 16)()
        n = self._check(_lib.acc_get_kernel_profile(self._h, arr, 16))
        return [dict(name=arr[i].name.decode(), launches=arr[i].launches, ms=arr[i].ms, flops=arr[i].flops)
                for i in range(n)]

    def launch_profile(self) -> list:
        """One dict per convolution-kernel launch of the last step profiled at level 2 or 3."""
        n = self._check(_lib.acc_get_launch_profile(self._h, None, 0))
        arr = (acc_launch_profile * max(n, 1))()
        n = self._check(_lib.acc_get_launch_profile(self._h, arr, n))
        return [dict(step=arr[i].step, layer=arr[i].layer, role=("fwd", "dgrad", "wgrad")[arr[i].role],
                     variant=arr[i].variant, ms=arr[i].ms, flops=arr[i].flops) for i in range(n)]

    def step_times_ms(self) -> np.ndarray:
        n = self.step_count()
        arr = (_D * n)()
        self._check(_lib.acc_get_step_times_ms(self._h, arr, n))
        return np.array(arr[:], dtype=np.float64)


# ---- single operations on torch device tensors (NHWC activations, O-H-W-I filters)
def _stream_ptr(torch):
    return torch.cuda.current_stream().cuda_stream


def op_conv_workspace(n, h, w, cin, cout, r, stride, pad) -> int:
    return int(_lib.acc_op_conv_workspace(n, h, w, cin, cout, r, r, stride, pad))


def _dtype_of(t) -> int:
    """Storage type of a torch tensor handed to an acc_op_* call."""
    import torch
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"unsupported storage type {t.dtype}")


def op_conv_fwd(x, w, y, stride, pad):
    import torch
    n, h, wd, cin = x.shape
    cout, r, s, _ = w.shape
    rc = _lib.acc_op_conv_fwd(x.data_ptr(), w.data_ptr(), y.data_ptr(), n, h, wd, cin, cout, r, s, stride, pad,
                              _dtype_of(x), _stream_ptr(torch))
    if rc != ACC_OK:
        raise AccError(rc, "acc_op_conv_fwd")


def op_conv_dgrad(dy, w, dx, stride, pad, ws, accumulate=False):
    import torch
    n, h, wd, cin = dx.shape
    cout, r, s, _ = w.shape
    rc = _lib.acc_op_conv_dgrad(dy.data_ptr(), w.data_ptr(), dx.data_ptr(), n, h, wd, cin, cout, r, s, stride, pad,
                                1 if accumulate else 0, ws.data_ptr(), ws.numel() * ws.element_size(),
                                _dtype_of(dy), _stream_ptr(torch))
    if rc != ACC_OK:
        raise AccError(rc, "acc_op_conv_dgrad")


def op_conv_wgrad(x, dy, dw, stride, pad, ws):
    import torch
    n, h, wd, cin = x.shape
    cout, r, s, _ = dw.shape
    rc = _lib.acc_op_conv_wgrad(x.data_ptr(), dy.data_ptr(), dw.data_ptr(), n, h, wd, cin, cout, r, s, stride, pad,
                                ws.data_ptr() if ws is not None else None,
                                ws.numel() * ws.element_size() if ws is not None else 0, _dtype_of(x),
                                _stream_ptr(torch))
    if rc != ACC_OK:
        raise AccError(rc, "acc_op_conv_wgrad")


def op_bn_workspace(c) -> int:
    return int(_lib.acc_op_bn_workspace(c))


def op_bn_fwd(x, gamma, beta, res, y, mean, istd, relu, eps, ws):
    import torch
    c = x.shape[-1]
    rows = x.numel() // c
    rc = _lib.acc_op_bn_fwd(x.data_ptr(), gamma.data_ptr(), beta.data_ptr(),
                            res.data_ptr() if res is not None else None, y.data_ptr(), mean.data_ptr(),
                            istd.data_ptr(), rows, c, 1 if relu else 0, float(eps), ws.data_ptr(), _dtype_of(x),
                            _stream_ptr(torch))
    if rc != ACC_OK:
        raise AccError(rc, "acc_op_bn_fwd")


def op_bn_fwd_noalloc(x, gamma, beta, res, y, mean, istd, relu, eps):
    """acc_op_bn_fwd with the library's built-in workspace (no allocation anywhere)."""
    import torch
    c = x.shape[-1]
    rows = x.numel() // c
    rc = _lib.acc_op_bn_fwd_noalloc(x.data_ptr(), gamma.data_ptr(), beta.data_ptr(),
                                    res.data_ptr() if res is not None else None, y.data_ptr(), mean.data_ptr(),
                                    istd.data_ptr(), rows, c, 1 if relu else 0, float(eps), _dtype_of(x),
                                    _stream_ptr(torch))
    if rc != ACC_OK:
        raise AccError(rc, _lib.acc_last_error(None).decode())


def op_bn_bwd(x, dy, y, gamma, mean, istd, dx, dgamma, dbeta, g_out, ws):
    import torch
    c = x.shape[-1]
    rows = x.numel() // c
    rc = _lib.acc_op_bn_bwd(x.data_ptr(), dy.data_ptr(), y.data_ptr() if y is not None else None, gamma.data_ptr(),
                            mean.data_ptr(), istd.data_ptr(), dx.data_ptr(), dgamma.data_ptr(), dbeta.data_ptr(),
                            g_out.data_ptr() if g_out is not None else None, rows, c, ws.data_ptr(),
                            _dtype_of(x), _stream_ptr(torch))
    if rc != ACC_OK:
        raise AccError(rc, "acc_op_bn_bwd")


def op_maxpool_fwd(x, y, r, stride, pad):
    """x [n, h, w, c] -> y [n, ho, wo, c] (torch device tensors, NHWC)."""
    import torch
    n, h, w, c = x.shape
    rc = _lib.acc_op_maxpool_fwd(x.data_ptr(), y.data_ptr(), n, h, w, c, r, stride, pad, _dtype_of(x), _stream_ptr(torch))
    if rc != ACC_OK:
        raise AccError(rc, "acc_op_maxpool_fwd")


def op_maxpool_bwd(x, dy, dx, r, stride, pad, accumulate=False):
    import torch
    n, h, w, c = x.shape
    rc = _lib.acc_op_maxpool_bwd(x.data_ptr(), dy.data_ptr(), dx.data_ptr(), n, h, w, c, r, stride, pad,
                                 1 if accumulate else 0, _dtype_of(x), _stream_ptr(torch))
    if rc != ACC_OK:
        raise AccError(rc, "acc_op_maxpool_bwd")


def op_gap_fwd(x, y):
    """x [n, h, w, c] -> y [n, c]: the mean over the positions of an image."""
    import torch
    n, h, w, c = x.shape
    rc = _lib.acc_op_gap_fwd(x.data_ptr(), y.data_ptr(), n, h * w, c, _dtype_of(x), _stream_ptr(torch))
    if rc != ACC_OK:
        raise AccError(rc, "acc_op_gap_fwd")


def op_gap_bwd(dy, dx, accumulate=False):
    import torch
    n, h, w, c = dx.shape
    rc = _lib.acc_op_gap_bwd(dy.data_ptr(), dx.data_ptr(), n, h * w, c, 1 if accumulate else 0, _dtype_of(dx),
                             _stream_ptr(torch))
    if rc != ACC_OK:
        raise AccError(rc, "acc_op_gap_bwd")


def op_softmax_ce(z, labels, loss_rows, loss, dz):
    """z [n, classes], labels int32 [n] (device); loss_rows [n] / loss [1] fp32 and dz like z, each optional."""
    import torch
    n, classes = z.shape
    rc = _lib.acc_op_softmax_ce(z.data_ptr(), labels.data_ptr(), loss_rows.data_ptr() if loss_rows is not None else None,
                                loss.data_ptr() if loss is not None else None, dz.data_ptr() if dz is not None else None,
                                n, classes, _dtype_of(z), _stream_ptr(torch))
    if rc != ACC_OK:
        raise AccError(rc, "acc_op_softmax_ce")
