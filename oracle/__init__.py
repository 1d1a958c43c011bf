"""ctypes view of the CPU oracle (liborc.so).  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this
package; the GPU library never does.  Build the library with `make -C oracle`.
"""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "liborc.so")

OK, ERR_ARG, ERR_SHAPE, ERR_UNSUPPORTED, ERR_OVERFLOW = 0, -1, -2, -3, -5
EV_ROUND, EV_PROC, EV_PROC_CATCHUP, EV_CRITERION, EV_MERGE = 1, 2, 3, 4, 5

RESULT_DT = np.dtype([("exit_idx", "<i4"), ("label", "<i4"), ("conf", "<f4"), ("pad_", "<i4"),
                      ("score", "<i8"), ("latency_ns", "<i8")])
EVENT_DT = np.dtype([("t_ns", "<i8"), ("kind", "<i4"), ("stage", "<i4"), ("b", "<i4"), ("aux", "<i4")])


class ServeOpts(C.Structure):
    _fields_ = [("b_max", C.c_int32), ("clock", C.c_int32), ("t_slo_ns", C.c_int64), ("lut_ns", C.c_void_p),
                ("min_incr", C.c_int32), ("refill", C.c_int32), ("t_timeout_ns", C.c_int64), ("lanes", C.c_int32), ("pad_", C.c_int32)]


class ServeStats(C.Structure):
    _fields_ = [("rounds", C.c_int64), ("criterion_evals", C.c_int64), ("preemptions", C.c_int64),
                ("end_time_ns", C.c_int64), ("seg_runs", C.c_int64 * 8), ("seg_samples", C.c_int64 * 8),
                ("n_events", C.c_int64)]


def build(force=False):
    if force or not os.path.exists(_LIB_PATH):
        subprocess.check_call(["make", "-C", _HERE, "-B", "liborc.so"], stdout=subprocess.DEVNULL)
    return _LIB_PATH


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(_LIB_PATH)
        _lib.orc_score_threshold.restype = C.c_int64
        _lib.orc_score_threshold.argtypes = [C.c_float]
        _lib.orc_exp2_table.restype = C.POINTER(C.c_uint32)
        _lib.orc_f32_to_bf16.restype = C.c_uint16
        _lib.orc_f32_to_bf16.argtypes = [C.c_float]
    return _lib


class OracleError(RuntimeError):
    def __init__(self, code):
        super().__init__(f"oracle returned {code}")
        self.code = code


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _chk(rc):
    if rc != 0:
        raise OracleError(rc)


def _c(a, dt):
    return np.ascontiguousarray(a, dtype=dt)


def out_hw(h, w, k, stride, pad):
    return (h + 2 * pad - k) // stride + 1, (w + 2 * pad - k) // stride + 1


# ---- int8 primitives ---------------------------------------------------------------
def conv_acc_i8(x, wt, bias, stride, pad, toeplitz=False, pad_w=None):
    """pad: rows of zero padding (top and bottom); pad_w: columns (default: the same)."""
    x, wt = _c(x, np.int8), _c(wt, np.int8)
    n, h, w, ci = x.shape
    co, kh, kw, ci2 = wt.shape
    assert ci == ci2
    pad_w = pad if pad_w is None else pad_w
    bias = None if bias is None else _c(bias, np.int32)
    ho, wo = (h + 2 * pad - kh) // stride + 1, (w + 2 * pad_w - kw) // stride + 1
    acc = np.empty((n, max(ho, 0), max(wo, 0), co), np.int32)
    fn = lib().orc_conv_acc_i8_toeplitz_hw if toeplitz else lib().orc_conv_acc_i8_hw
    _chk(fn(_p(x), n, h, w, ci, _p(wt), _p(bias), co, kh, kw, stride, pad, pad_w, _p(acc)))
    return acc


def dwconv_acc_i8(x, wt, bias, stride, pad):
    x, wt = _c(x, np.int8), _c(wt, np.int8)
    n, h, w, c = x.shape
    c2, kh, kw = wt.shape
    assert c == c2
    bias = None if bias is None else _c(bias, np.int32)
    ho, wo = out_hw(h, w, kh, stride, pad)
    acc = np.empty((n, ho, wo, c), np.int32)
    _chk(lib().orc_dwconv_acc_i8(_p(x), n, h, w, c, _p(wt), _p(bias), kh, kw, stride, pad, _p(acc)))
    return acc


def requant_i8(acc, res, shift, res_shift, lo, hi):
    acc = _c(acc, np.int32)
    res = None if res is None else _c(res, np.int8)
    y = np.empty(acc.shape, np.int8)
    _chk(lib().orc_requant_i8(_p(acc), _p(res), C.c_int64(acc.size), shift, res_shift, lo, hi, _p(y)))
    return y


def maxpool_i8(x, k, stride, pad):
    x = _c(x, np.int8)
    n, h, w, c = x.shape
    ho, wo = out_hw(h, w, k, stride, pad)
    y = np.empty((n, ho, wo, c), np.int8)
    _chk(lib().orc_maxpool_i8(_p(x), n, h, w, c, k, stride, pad, _p(y)))
    return y


def avgpool_i8(x, k, stride, pad):
    x = _c(x, np.int8)
    n, h, w, c = x.shape
    ho, wo = out_hw(h, w, k, stride, pad)
    y = np.empty((n, ho, wo, c), np.int8)
    _chk(lib().orc_avgpool_i8(_p(x), n, h, w, c, k, stride, pad, _p(y)))
    return y


def gap_i8(x, gap_shift):
    x = _c(x, np.int8)
    n, h, w, c = x.shape
    sums, g = np.empty((n, c), np.int32), np.empty((n, c), np.int8)
    _chk(lib().orc_gap_i8(_p(x), n, h, w, c, gap_shift, _p(sums), _p(g)))
    return sums, g


def fc_i8(g, wfc, bfc):
    g, wfc = _c(g, np.int8), _c(wfc, np.int8)
    n, c = g.shape
    n_cls = wfc.shape[0]
    bfc = None if bfc is None else _c(bfc, np.int32)
    a = np.empty((n, n_cls), np.int32)
    _chk(lib().orc_fc_i8(_p(g), n, c, _p(wfc), _p(bfc), n_cls, _p(a)))
    return a


def softmax_top1_i8(a, frac_bits):
    a = _c(a, np.int32)
    n, n_cls = a.shape
    label, score = np.empty(n, np.int32), np.empty(n, np.int64)
    _chk(lib().orc_softmax_top1_i8(_p(a), n, n_cls, frac_bits, _p(label), _p(score)))
    return label, score


def score_threshold(thr):
    return int(lib().orc_score_threshold(C.c_float(thr)))


def exp2_table():
    return np.ctypeslib.as_array(lib().orc_exp2_table(), shape=(256,)).copy()


# ---- bf16 primitives -----------------------------------------------------------------
def conv_bf16(x, wt, bias, stride, pad, res=None, f_lo=-np.inf, f_hi=np.inf, pad_w=None):
    x, wt = _c(x, np.uint16), _c(wt, np.uint16)
    n, h, w, ci = x.shape
    co, kh, kw, _ = wt.shape
    pad_w = pad if pad_w is None else pad_w
    bias = None if bias is None else _c(bias, np.float32)
    res = None if res is None else _c(res, np.uint16)
    ho, wo = (h + 2 * pad - kh) // stride + 1, (w + 2 * pad_w - kw) // stride + 1
    y = np.empty((n, ho, wo, co), np.uint16)
    _chk(lib().orc_conv_bf16_hw(_p(x), n, h, w, ci, _p(wt), _p(bias), co, kh, kw, stride, pad, pad_w, _p(res),
                                C.c_float(f_lo), C.c_float(f_hi), _p(y)))
    return y


def dwconv_bf16(x, wt, bias, stride, pad, f_lo=-np.inf, f_hi=np.inf):
    x, wt = _c(x, np.uint16), _c(wt, np.uint16)
    n, h, w, c = x.shape
    _, kh, kw = wt.shape
    bias = None if bias is None else _c(bias, np.float32)
    ho, wo = out_hw(h, w, kh, stride, pad)
    y = np.empty((n, ho, wo, c), np.uint16)
    _chk(lib().orc_dwconv_bf16(_p(x), n, h, w, c, _p(wt), _p(bias), kh, kw, stride, pad,
                               C.c_float(f_lo), C.c_float(f_hi), _p(y)))
    return y


def maxpool_bf16(x, k, stride, pad):
    x = _c(x, np.uint16)
    n, h, w, c = x.shape
    ho, wo = out_hw(h, w, k, stride, pad)
    y = np.empty((n, ho, wo, c), np.uint16)
    _chk(lib().orc_maxpool_bf16(_p(x), n, h, w, c, k, stride, pad, _p(y)))
    return y


def avgpool_bf16(x, k, stride, pad):
    x = _c(x, np.uint16)
    n, h, w, c = x.shape
    ho, wo = out_hw(h, w, k, stride, pad)
    y = np.empty((n, ho, wo, c), np.uint16)
    _chk(lib().orc_avgpool_bf16(_p(x), n, h, w, c, k, stride, pad, _p(y)))
    return y


def head_bf16(x, wfc, bfc, logit_scale):
    x, wfc = _c(x, np.uint16), _c(wfc, np.uint16)
    n, h, w, c = x.shape
    n_cls = wfc.shape[0]
    bfc = None if bfc is None else _c(bfc, np.float32)
    logits = np.empty((n, n_cls), np.float32)
    label, conf = np.empty(n, np.int32), np.empty(n, np.float32)
    _chk(lib().orc_head_bf16(_p(x), n, h, w, c, _p(wfc), _p(bfc), n_cls, C.c_float(logit_scale), _p(logits), _p(label), _p(conf)))
    return logits, label, conf


# ---- network level ---------------------------------------------------------------------
def _blob_args(blob):
    buf = blob.buffer()
    return _p(buf), C.c_size_t(buf.size)


def blob_check(blob):
    return lib().orc_blob_check(*_blob_args(blob))


def stage_forward(blob, stage, act_in):
    act_in = np.ascontiguousarray(act_in)
    b = act_in.shape[0]
    h, w, c = blob.stage_out_shape(stage)
    out = np.empty((b, h, w, c), act_in.dtype)
    _chk(lib().orc_stage_forward(*_blob_args(blob), stage, b, _p(act_in), _p(out)))
    return out


def exit_head(blob, stage, act, thr, want_logits=False):
    act = np.ascontiguousarray(act)
    b = act.shape[0]
    label, conf = np.empty(b, np.int32), np.empty(b, np.float32)
    score, flag = np.empty(b, np.int64), np.empty(b, np.uint8)
    logits = None
    if want_logits:
        n_cls = int(blob.exits[stage]["n_cls"])
        logits = np.empty((b, n_cls), np.int32 if blob.dtype == 0 else np.float32)
    _chk(lib().orc_exit_head(*_blob_args(blob), stage, b, _p(act), C.c_float(thr), _p(label), _p(conf), _p(score), _p(flag), _p(logits)))
    return (label, conf, score, flag, logits) if want_logits else (label, conf, score, flag)


def compact_refill(flags, act_src, ids_src, refill_act=None, refill_ids=None):
    act_src = np.ascontiguousarray(act_src)
    flags = _c(flags, np.uint8)
    b = act_src.shape[0]
    b_incr = 0 if refill_act is None else refill_act.shape[0]
    per = int(np.prod(act_src.shape[1:])) * act_src.itemsize
    dst = np.zeros((b + b_incr,) + act_src.shape[1:], act_src.dtype)
    ids_src = _c(ids_src, np.int32)
    ids_dst = np.full(b + b_incr, -1, np.int32)
    if refill_act is not None:
        refill_act, refill_ids = np.ascontiguousarray(refill_act, dtype=act_src.dtype), _c(refill_ids, np.int32)
    b_rem, b_merged = C.c_int(), C.c_int()
    _chk(lib().orc_compact_refill(C.c_int64(per), b, _p(flags), _p(act_src), _p(dst), _p(ids_src), _p(ids_dst),
                                  _p(refill_act), _p(refill_ids), b_incr, C.byref(b_rem), C.byref(b_merged)))
    return dst[:b_merged.value], ids_dst[:b_merged.value], b_rem.value, b_merged.value


def forward_alone(blob, inputs, threads=None):
    """every request alone through the segments until it exits; threads: worker threads (None = all cores)"""
    inputs = np.ascontiguousarray(inputs)
    n = inputs.shape[0]
    res = np.zeros(n, RESULT_DT)
    if threads:
        lib().orc_set_threads(int(threads))
    try:
        _chk(lib().orc_forward_alone(*_blob_args(blob), C.c_int64(n), _p(inputs), _p(res)))
    finally:
        if threads:
            lib().orc_set_threads(0)
    return res


def serve_stream(blob, arrival_ns, pool, b_max, lut_ns, t_slo_ns=-1, min_incr=1, refill=1,
                 forced_exit=None, n_stages=None, max_events=0, t_timeout_ns=0, lanes=1):
    """Algorithm 1 on the virtual clock.  Returns (results, stats dict, events)."""
    arrival_ns = _c(arrival_ns, np.int64)
    n = arrival_ns.size
    lut_ns = _c(lut_ns, np.int64)
    opts = ServeOpts(b_max, 1, t_slo_ns, lut_ns.ctypes.data, min_incr, refill, t_timeout_ns, lanes, 0)
    stats = ServeStats()
    res = np.zeros(n, RESULT_DT)
    ev = np.zeros(max_events, EVENT_DT) if max_events else None
    if forced_exit is not None:
        forced_exit = _c(forced_exit, np.int32)
        bp, bl = None, C.c_size_t(0)
        assert lut_ns.shape == (n_stages, b_max)
    else:
        bp, bl = _blob_args(blob)
        pool = np.ascontiguousarray(pool)
        n_stages = blob.n_stages
        assert lut_ns.shape == (n_stages, b_max)
    _chk(lib().orc_serve_stream(bp, bl, C.c_int64(n), _p(arrival_ns), _p(pool), C.byref(opts), _p(forced_exit),
                                n_stages or 0, _p(res), C.byref(stats), _p(ev), C.c_int64(max_events)))
    st = dict(rounds=stats.rounds, criterion_evals=stats.criterion_evals, preemptions=stats.preemptions,
              end_time_ns=stats.end_time_ns, seg_runs=list(stats.seg_runs)[:n_stages],
              seg_samples=list(stats.seg_samples)[:n_stages], n_events=stats.n_events)
    if ev is not None:
        ev = ev[:min(stats.n_events, max_events)]
    return res, st, ev
