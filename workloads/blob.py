"""Binary container ("blob") describing an early-exit network.

Pure data layout, little endian, naturally aligned.  The CPU oracle (C) and
the GPU library (C++) each carry their own parser of this layout.

  header   128 B   HEADER_DT
  stages   n_stages x 32 B   STAGE_DT
  ops      n_ops    x 112 B  OP_DT   (ops of stage s are contiguous)
  exits    n_stages x 64 B   EXIT_DT (exit head s sits on the output of stage s)
  data     weights and biases, each tensor 64-byte aligned

Tensor numbering is local to a stage: id 0 is the stage input, every op
writes a new id (1, 2, ...), except that several ops may each write a channel
slice [c_off, c_off + c_out) of one tensor of c_tot channels (concatenation).
`pad` pads rows (top and bottom), `pad_w` columns.  Activations are NHWC.  Convolution weights are
[C_out][kh][kw][C_in], depthwise weights [C][kh][kw], FC weights [n_cls][C].
int8 networks carry int8 weights / int32 biases; bf16 networks carry bf16
weights (raw uint16) / float32 biases.
"""
import numpy as np

MAGIC = b"EENETv2\0"
DT_I8, DT_BF16 = 0, 1
OP_CONV, OP_DWCONV, OP_MAXPOOL, OP_AVGPOOL = 0, 1, 2, 3

HEADER_DT = np.dtype([
    ("magic", "S8"), ("version", "<i4"), ("dtype", "<i4"), ("n_stages", "<i4"), ("n_ops", "<i4"),
    ("in_h", "<i4"), ("in_w", "<i4"), ("in_c", "<i4"), ("n_classes", "<i4"),
    ("stages_off", "<i8"), ("ops_off", "<i8"), ("exits_off", "<i8"), ("data_off", "<i8"),
    ("total_bytes", "<i8"), ("reserved", "V48"),
])
assert HEADER_DT.itemsize == 128

STAGE_DT = np.dtype([
    ("first_op", "<i4"), ("n_ops", "<i4"), ("n_tensors", "<i4"), ("out_tensor", "<i4"),
    ("out_h", "<i4"), ("out_w", "<i4"), ("out_c", "<i4"), ("reserved", "<i4"),
])
assert STAGE_DT.itemsize == 32

OP_DT = np.dtype([
    ("kind", "<i4"), ("src", "<i4"), ("dst", "<i4"), ("res", "<i4"),
    ("h_in", "<i4"), ("w_in", "<i4"), ("c_in", "<i4"),
    ("h_out", "<i4"), ("w_out", "<i4"), ("c_out", "<i4"),
    ("kh", "<i4"), ("kw", "<i4"), ("stride", "<i4"), ("pad", "<i4"),
    ("shift", "<i4"), ("res_shift", "<i4"), ("lo", "<i4"), ("hi", "<i4"),
    ("f_lo", "<f4"), ("f_hi", "<f4"),
    ("w_off", "<i8"), ("b_off", "<i8"),
    ("pad_w", "<i4"), ("c_off", "<i4"), ("c_tot", "<i4"), ("reserved", "<i4"),
])
assert OP_DT.itemsize == 112

EXIT_DT = np.dtype([
    ("h", "<i4"), ("w", "<i4"), ("c", "<i4"), ("n_cls", "<i4"),
    ("gap_shift", "<i4"), ("frac_bits", "<i4"),
    ("logit_scale", "<f4"), ("thr", "<f4"),
    ("w_off", "<i8"), ("b_off", "<i8"), ("reserved", "V16"),
])
assert EXIT_DT.itemsize == 64


def f32_to_bf16_bits(x):
    """Round float32 to bfloat16 (round to nearest, ties to even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b):
    return (np.asarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


class Blob:
    """A mutable view of a network blob: structured-array views over one byte buffer."""

    def __init__(self, raw):
        self.raw = np.frombuffer(bytearray(raw), dtype=np.uint8)  # private writable copy
        self.header = self.raw[:128].view(HEADER_DT)[0:1]
        h = self.header[0]
        if bytes(h["magic"]).ljust(8, b"\0") != MAGIC:
            raise ValueError("not a network blob")
        ns, no = int(h["n_stages"]), int(h["n_ops"])
        so, oo, eo = int(h["stages_off"]), int(h["ops_off"]), int(h["exits_off"])
        self.stages = self.raw[so:so + 32 * ns].view(STAGE_DT)
        self.ops = self.raw[oo:oo + OP_DT.itemsize * no].view(OP_DT)
        self.exits = self.raw[eo:eo + 64 * ns].view(EXIT_DT)

    # -- convenience -------------------------------------------------------
    @property
    def dtype(self):
        return int(self.header[0]["dtype"])

    @property
    def n_stages(self):
        return int(self.header[0]["n_stages"])

    @property
    def elem_bytes(self):
        return 1 if self.dtype == DT_I8 else 2

    def in_shape(self):
        h = self.header[0]
        return int(h["in_h"]), int(h["in_w"]), int(h["in_c"])

    def stage_in_shape(self, s):
        if s == 0:
            return self.in_shape()
        st = self.stages[s - 1]
        return int(st["out_h"]), int(st["out_w"]), int(st["out_c"])

    def stage_out_shape(self, s):
        st = self.stages[s]
        return int(st["out_h"]), int(st["out_w"]), int(st["out_c"])

    def stage_ops(self, s):
        st = self.stages[s]
        return self.ops[int(st["first_op"]):int(st["first_op"]) + int(st["n_ops"])]

    def op_weights(self, op):
        """Weight and bias arrays (views) of one op record, or (None, None) for max-pool."""
        kind = int(op["kind"])
        if kind in (OP_MAXPOOL, OP_AVGPOOL):
            return None, None
        co, kh, kw, ci = int(op["c_out"]), int(op["kh"]), int(op["kw"]), int(op["c_in"])
        nw = co * kh * kw * (1 if kind == OP_DWCONV else ci)
        return self._tensor(int(op["w_off"]), nw, True), self._tensor(int(op["b_off"]), co, False)

    def exit_weights(self, s):
        e = self.exits[s]
        n = int(e["n_cls"]) * int(e["c"])
        return self._tensor(int(e["w_off"]), n, True), self._tensor(int(e["b_off"]), int(e["n_cls"]), False)

    def _tensor(self, off, count, is_weight):
        if self.dtype == DT_I8:
            return (self.raw[off:off + count].view(np.int8) if is_weight
                    else self.raw[off:off + 4 * count].view("<i4"))
        return (self.raw[off:off + 2 * count].view("<u2") if is_weight
                else self.raw[off:off + 4 * count].view("<f4"))

    def tobytes(self):
        return self.raw.tobytes()

    def buffer(self):
        """The live byte buffer (uint8 numpy array) for passing to C."""
        return self.raw
