"""Python binding of libee.so, the MI355X early-exit serving library.

Argument marshalling only: every step of the hot path runs inside the library's HIP kernels.
PyTorch supplies device memory (tensors) and the HIP stream; there is no CPU fallback -- if the
shared library is missing the import of this module fails.
"""
import ctypes as C
import os

import numpy as np
import torch  # noqa: F401  -- first: libee.so must bind to the HIP runtime PyTorch has already loaded

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libee.so")

EE_OK, EE_ERR_ARG, EE_ERR_SHAPE, EE_ERR_UNSUPPORTED, EE_ERR_DEVICE, EE_ERR_OVERFLOW = 0, -1, -2, -3, -4, -5
EE_I8, EE_BF16 = 0, 1
K_NAMES = ["conv_mfma", "conv_first", "conv_direct", "depthwise", "maxpool", "pad_input", "gap", "fc", "softmax",
           "compact", "admit", "conv_stream"]

RESULT_DT = np.dtype([("exit_idx", "<i4"), ("label", "<i4"), ("conf", "<f4"), ("pad_", "<i4"),
                      ("score", "<i8"), ("latency_ns", "<i8")])
EVENT_DT = np.dtype([("t_ns", "<i8"), ("kind", "<i4"), ("stage", "<i4"), ("b", "<i4"), ("aux", "<i4")])

SYMBOLS = ["ee_strerror", "ee_blob_check", "ee_create", "ee_destroy", "ee_query", "ee_stage_forward", "ee_exit_head",
           "ee_compact_refill", "ee_serve_stream", "ee_schedule_sim", "ee_measure_lut", "ee_profile_enable",
           "ee_profile_read", "ee_kernel_name", "ee_exp2_table", "ee_tune_conv_tile", "ee_ir_count", "ee_ir_layers", "ee_ir_mode", "ee_ir_table", "ee_ir_set", "ee_last_logits", "ee_profile_reserve", "ee_autotune", "ee_config_table",
           "ee_pair_count", "ee_pair_mode", "ee_pair_table", "ee_config_set", "ee_pair_set", "ee_exit_head_static",
           "ee_static_scratch_bytes", "ee_time_layer", "ee_lanes", "ee_zero_copy_supported"]


class Trace(C.Structure):
    _fields_ = [("n", C.c_int64), ("arrival_ns", C.c_void_p)]


class ServeOpts(C.Structure):
    _fields_ = [("b_max", C.c_int32), ("clock", C.c_int32), ("t_slo_ns", C.c_int64), ("lut_ns", C.c_void_p),
                ("min_incr", C.c_int32), ("refill", C.c_int32), ("t_timeout_ns", C.c_int64), ("lanes", C.c_int32), ("zero_copy", C.c_int32)]


class ServeStats(C.Structure):
    _fields_ = [("rounds", C.c_int64), ("criterion_evals", C.c_int64), ("preemptions", C.c_int64),
                ("end_time_ns", C.c_int64), ("seg_runs", C.c_int64 * 8), ("seg_samples", C.c_int64 * 8),
                ("n_events", C.c_int64)]


class KernelStat(C.Structure):
    _fields_ = [("launches", C.c_int64), ("ms", C.c_double), ("ops", C.c_double), ("bytes", C.c_double)]


if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2209_13443_amd.build` "
                      "(there is no fallback implementation)")
_lib = C.CDLL(LIB_PATH)
_lib.ee_strerror.restype = C.c_char_p
_lib.ee_kernel_name.restype = C.c_char_p
_lib.ee_exp2_table.restype = C.POINTER(C.c_uint32)
_V = C.c_void_p
_lib.ee_blob_check.argtypes = [_V, C.c_size_t]
_lib.ee_create.argtypes = [_V, C.c_size_t, C.c_int, C.c_int, _V, C.POINTER(_V)]
_lib.ee_destroy.argtypes = [_V]
_lib.ee_query.argtypes = [_V, C.POINTER(C.c_int), _V, _V]
_lib.ee_stage_forward.argtypes = [_V, C.c_int, C.c_int, _V, _V]
_lib.ee_exit_head.argtypes = [_V, C.c_int, C.c_int, _V, C.c_float, _V, _V, _V, _V]
_lib.ee_exit_head_static.argtypes = [_V, C.c_int, C.c_int, _V, C.c_float, _V, _V, _V, _V]
_lib.ee_static_scratch_bytes.argtypes = []
_lib.ee_lanes.argtypes = [_V, C.c_int]
_lib.ee_time_layer.argtypes = [_V, C.c_int, C.c_int, C.c_int, C.c_int, _V, _V, _V]
_lib.ee_compact_refill.argtypes = [_V, C.c_int, C.c_int, _V, _V, _V, _V, _V, _V, _V, C.c_int, _V, _V]
_lib.ee_serve_stream.argtypes = [_V, C.POINTER(Trace), _V, C.POINTER(ServeOpts), _V, C.POINTER(ServeStats), _V, C.c_int64]
_lib.ee_schedule_sim.argtypes = [C.c_int, C.POINTER(Trace), _V, C.POINTER(ServeOpts), _V, C.POINTER(ServeStats), _V, C.c_int64]
_lib.ee_measure_lut.argtypes = [_V, C.c_int, _V]
_lib.ee_last_logits.argtypes = [_V, C.c_int, _V]
_lib.ee_autotune.argtypes = [_V, C.c_int]
_lib.ee_config_table.argtypes = [_V, C.c_int, _V, C.c_int]
_lib.ee_pair_count.argtypes = [_V]
_lib.ee_zero_copy_supported.argtypes = [_V]
_lib.ee_pair_mode.argtypes = [_V, C.c_int]
_lib.ee_pair_table.argtypes = [_V, C.c_int, _V, C.c_int]
_lib.ee_config_set.argtypes = [_V, C.c_int, _V, C.c_int]
_lib.ee_pair_set.argtypes = [_V, C.c_int, _V, C.c_int]
_lib.ee_ir_count.argtypes = [_V]
_lib.ee_ir_layers.argtypes = [_V, C.c_int]
_lib.ee_ir_mode.argtypes = [_V, C.c_int]
_lib.ee_ir_table.argtypes = [_V, C.c_int, _V, C.c_int]
_lib.ee_ir_set.argtypes = [_V, C.c_int, _V, C.c_int]
_lib.ee_profile_enable.argtypes = [_V, C.c_int]
_lib.ee_profile_read.argtypes = [_V, _V, _V]
_lib.ee_profile_reserve.argtypes = [_V, C.c_int64]


class EEError(RuntimeError):
    def __init__(self, code):
        super().__init__(f"libee: {_lib.ee_strerror(code).decode()} ({code})")
        self.code = code


def _chk(rc):
    if rc != 0:
        raise EEError(rc)


def raw():
    """The ctypes handle (tests call the C ABI directly through it)."""
    return _lib


def strerror(code):
    return _lib.ee_strerror(code).decode()


def blob_check(blob_bytes):
    buf = np.frombuffer(blob_bytes, np.uint8) if not isinstance(blob_bytes, np.ndarray) else blob_bytes
    return _lib.ee_blob_check(buf.ctypes.data, buf.size)


def tune_conv_tile(tile):
    return _lib.ee_tune_conv_tile(int(tile))


def exp2_table():
    return np.ctypeslib.as_array(_lib.ee_exp2_table(), shape=(256,)).copy()


def _np_ptr(a):
    return None if a is None else a.ctypes.data


def _stats_dict(st, n_stages):
    return dict(rounds=st.rounds, criterion_evals=st.criterion_evals, preemptions=st.preemptions,
                end_time_ns=st.end_time_ns, seg_runs=list(st.seg_runs)[:n_stages],
                seg_samples=list(st.seg_samples)[:n_stages], n_events=st.n_events)


def schedule_sim(n_stages, arrival_ns, forced_exit, b_max, lut_ns, t_slo_ns=-1, min_incr=1, refill=1, max_events=0, t_timeout_ns=0, lanes=1):
    """ee_schedule_sim: Algorithm 1 on the virtual clock with forced exits (host only)."""
    arrival_ns = np.ascontiguousarray(arrival_ns, np.int64)
    forced_exit = np.ascontiguousarray(forced_exit, np.int32)
    lut_ns = np.ascontiguousarray(lut_ns, np.int64)
    n = arrival_ns.size
    tr = Trace(n, arrival_ns.ctypes.data)
    opts = ServeOpts(b_max, 1, t_slo_ns, lut_ns.ctypes.data, min_incr, refill, t_timeout_ns, lanes, 0)
    res = np.zeros(n, RESULT_DT)
    ev = np.zeros(max(max_events, 1), EVENT_DT)
    st = ServeStats()
    _chk(_lib.ee_schedule_sim(n_stages, C.byref(tr), forced_exit.ctypes.data, C.byref(opts), res.ctypes.data,
                              C.byref(st), ev.ctypes.data if max_events else None, max_events))
    return res, _stats_dict(st, n_stages), ev[:min(st.n_events, max_events)]


class Engine:
    """One network resident on the GPU.  Tensors are torch CUDA tensors (int8, or int16 holding bf16 bits)."""

    def __init__(self, blob, b_max, stream=None):
        import torch
        self.torch = torch
        buf = blob.buffer() if hasattr(blob, "buffer") else np.frombuffer(blob, np.uint8)
        self.dtype = int(np.frombuffer(buf[12:16].tobytes(), "<i4")[0])
        self.b_max = b_max
        self.stream = torch.cuda.current_stream() if stream is None else stream
        h = _V()
        _chk(_lib.ee_create(buf.ctypes.data, buf.size, b_max, self.dtype, _V(self.stream.cuda_stream), C.byref(h)))
        self._h = h
        n = C.c_int()
        ib, ob = (C.c_int64 * 8)(), (C.c_int64 * 8)()
        _chk(_lib.ee_query(self._h, C.byref(n), ib, ob))
        self.n_stages = n.value
        self.stage_in_bytes, self.stage_out_bytes = list(ib)[:n.value], list(ob)[:n.value]
        self.tdtype = torch.int8 if self.dtype == EE_I8 else torch.int16
        self.esize = 1 if self.dtype == EE_I8 else 2

    def close(self):
        if getattr(self, "_h", None) and _lib is not None:      # module globals are gone at interpreter exit
            _lib.ee_destroy(self._h)
            self._h = None

    def __del__(self):
        self.close()

    # -- single steps ----------------------------------------------------------------------
    def stage_forward(self, stage, act_in, out_shape):
        t = self.torch
        b = act_in.shape[0]
        out = t.empty((b,) + tuple(out_shape), dtype=self.tdtype, device=act_in.device)
        _chk(_lib.ee_stage_forward(self._h, stage, b, act_in.data_ptr(), out.data_ptr()))
        return out

    def exit_head(self, stage, act, thr):
        t = self.torch
        b, dev = act.shape[0], act.device
        label = t.empty(b, dtype=t.int32, device=dev)
        conf = t.empty(b, dtype=t.float32, device=dev)
        score = t.empty(b, dtype=t.int64, device=dev)
        flag = t.empty(b, dtype=t.uint8, device=dev)
        _chk(_lib.ee_exit_head(self._h, stage, b, act.data_ptr(), thr, label.data_ptr(), conf.data_ptr(),
                               score.data_ptr(), flag.data_ptr()))
        return label, conf, score, flag

    def exit_head_static(self, stage, act, thr, label, conf, score, flag):
        """ee_exit_head_static: the caller brings the four per-slot output tensors; nothing is allocated."""
        _chk(_lib.ee_exit_head_static(self._h, stage, act.shape[0], act.data_ptr(), thr, label.data_ptr(), conf.data_ptr(),
                                      score.data_ptr(), flag.data_ptr()))

    def last_logits(self, b, n_cls):
        out = np.empty((b, n_cls), np.int32 if self.dtype == EE_I8 else np.float32)
        _chk(_lib.ee_last_logits(self._h, b, out.ctypes.data))
        return out

    def compact_refill(self, stage, flags, act_src, ids_src, refill_act=None, refill_ids=None):
        t = self.torch
        b, dev = act_src.shape[0], act_src.device
        b_incr = 0 if refill_act is None else refill_act.shape[0]
        dst = t.zeros((b + b_incr,) + tuple(act_src.shape[1:]), dtype=act_src.dtype, device=dev)
        ids_dst = t.full((b + b_incr,), -1, dtype=t.int32, device=dev)
        counts = t.zeros(2, dtype=t.int32, device=dev)
        _chk(_lib.ee_compact_refill(self._h, stage, b, flags.data_ptr(), act_src.data_ptr(), dst.data_ptr(),
                                    ids_src.data_ptr(), ids_dst.data_ptr(),
                                    None if refill_act is None else refill_act.data_ptr(),
                                    None if refill_ids is None else refill_ids.data_ptr(), b_incr,
                                    counts.data_ptr(), counts.data_ptr() + 4))
        self.stream.synchronize()
        b_rem, b_merged = int(counts[0]), int(counts[1])
        return dst[:b_merged], ids_dst[:b_merged], b_rem, b_merged

    # -- stream serving ----------------------------------------------------------------------
    def serve_stream(self, arrival_ns, pool, lut_ns, b_max=None, clock=0, t_slo_ns=-1, min_incr=1, refill=1, max_events=0, t_timeout_ns=0, lanes=1,
                     zero_copy=0):
        arrival_ns = np.ascontiguousarray(arrival_ns, np.int64)
        lut_ns = np.ascontiguousarray(lut_ns, np.int64)
        b_max = b_max or self.b_max
        assert lut_ns.shape == (self.n_stages, b_max)
        n = arrival_ns.size
        tr = Trace(n, arrival_ns.ctypes.data)
        opts = ServeOpts(b_max, clock, t_slo_ns, lut_ns.ctypes.data, min_incr, refill, t_timeout_ns, lanes, int(zero_copy))
        res = np.zeros(n, RESULT_DT)
        ev = np.zeros(max(max_events, 1), EVENT_DT)
        st = ServeStats()
        _chk(_lib.ee_serve_stream(self._h, C.byref(tr), pool.data_ptr(), C.byref(opts), res.ctypes.data, C.byref(st),
                                  ev.ctypes.data if max_events else None, max_events))
        return res, _stats_dict(st, self.n_stages), ev[:min(st.n_events, max_events)]

    def zero_copy_supported(self):
        return _lib.ee_zero_copy_supported(self._h) == 1

    def set_lanes(self, n):
        """ee_lanes: workspace and streams for n concurrent steps of the stage-pool policy; returns the lane count"""
        rc = _lib.ee_lanes(self._h, int(n))
        if rc < 0:
            _chk(rc)
        return rc

    def measure_lut(self, reps=3):
        lut = np.zeros((self.n_stages, self.b_max), np.int64)
        _chk(_lib.ee_measure_lut(self._h, reps, lut.ctypes.data))
        return lut

    def time_layer(self, layer, b, cfg=0, reps=20):
        """(microseconds per launch, 2 * MACs, algorithmic bytes) of one layer alone; None when the configuration does not exist"""
        us, ops, byt = C.c_double(), C.c_double(), C.c_double()
        rc = _lib.ee_time_layer(self._h, int(layer), int(b), int(cfg), int(reps), C.byref(us), C.byref(ops), C.byref(byt))
        if rc == EE_ERR_DEVICE and cfg:
            return None
        _chk(rc)
        return us.value, ops.value, byt.value

    def autotune(self, reps=5):
        _chk(_lib.ee_autotune(self._h, int(reps)))

    def config_table(self, layer):
        buf = (C.c_int * 16)()
        n = _lib.ee_config_table(self._h, int(layer), buf, 16)
        if n < 0:
            _chk(n)
        return list(buf)[:n]

    def tables(self):
        """The tuned tables as plain data: {"config": {layer: [...]}, "pair": {layer: [...]}} (layers that have one)."""
        out = {"config": {}, "pair": {}, "ir": {}}
        buf = (C.c_int * 16)()
        layer = 0
        while True:
            n = _lib.ee_config_table(self._h, layer, buf, 16)
            if n < 0:                                   # past the last layer
                return out
            if n:
                out["config"][str(layer)] = list(buf)[:n]
            n = _lib.ee_pair_table(self._h, layer, buf, 16)
            if n > 0:
                out["pair"][str(layer)] = list(buf)[:n]
            n = _lib.ee_ir_table(self._h, layer, buf, 16)
            if n > 0:
                out["ir"][str(layer)] = list(buf)[:n]
            layer += 1

    def load_tables(self, tables):
        for key, fn in (("config", _lib.ee_config_set), ("pair", _lib.ee_pair_set), ("ir", _lib.ee_ir_set)):
            for layer, cfg in tables.get(key, {}).items():
                buf = (C.c_int * len(cfg))(*cfg)
                _chk(fn(self._h, int(layer), buf, len(cfg)))

    def pair_count(self):
        n = _lib.ee_pair_count(self._h)
        if n < 0:
            _chk(n)
        return n

    def pair_mode(self, mode):
        _chk(_lib.ee_pair_mode(self._h, int(mode)))

    def ir_count(self):
        n = _lib.ee_ir_count(self._h)
        if n < 0:
            _chk(n)
        return n

    def ir_layers(self, layer):
        """layers of the fused block headed by `layer`, 0 when it heads none"""
        n = _lib.ee_ir_layers(self._h, int(layer))
        if n < 0:
            _chk(n)
        return n

    def ir_mode(self, mode):
        _chk(_lib.ee_ir_mode(self._h, int(mode)))

    def ir_table(self, layer):
        buf = (C.c_int * 16)()
        n = _lib.ee_ir_table(self._h, int(layer), buf, 16)
        return list(buf)[:max(n, 0)]

    def pair_table(self, layer):
        buf = (C.c_int * 16)()
        n = _lib.ee_pair_table(self._h, int(layer), buf, 16)
        if n < 0:
            _chk(n)
        return list(buf)[:n]

    def profile(self, enable):
        _chk(_lib.ee_profile_enable(self._h, int(enable)))

    def profile_reserve(self, n_pairs):
        _chk(_lib.ee_profile_reserve(self._h, int(n_pairs)))

    def profile_read(self, n_layers=0):
        arr = (KernelStat * len(K_NAMES))()
        lay = (KernelStat * n_layers)() if n_layers else None
        _chk(_lib.ee_profile_read(self._h, arr, lay))
        cls = {K_NAMES[i]: dict(launches=arr[i].launches, ms=arr[i].ms, ops=arr[i].ops, bytes=arr[i].bytes)
               for i in range(len(K_NAMES))}
        if not n_layers:
            return cls
        return cls, [dict(launches=x.launches, ms=x.ms, ops=x.ops, bytes=x.bytes) for x in lay]
