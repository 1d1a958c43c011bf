"""Pins for the oracle's network level: segment forward, exit head, compaction, schedule independence."""
import itertools

import numpy as np
import pytest

import workloads as W


@pytest.fixture(scope="module")
def tiny():
    return W.load_net("tiny_i8")


def test_blob_check_accepts_all_configs_and_rejects_broken_chain(orc):
    for name in ("tiny_i8", "tiny_bf16", "resnet50_small_i8", "mobilenetv2_small_i8", "resnet18_small_i8", "inception_small_i8", "inception_small_bf16"):
        assert orc.blob_check(W.build_net(name)) == orc.OK
    b = W.build_net("tiny_i8")
    b.ops[1]["c_in"] = 17
    assert orc.blob_check(b) == orc.ERR_SHAPE
    b = W.build_net("tiny_i8")
    b.ops[0]["h_out"] = 15
    assert orc.blob_check(b) == orc.ERR_SHAPE
    b = W.build_net("tiny_i8")
    b.header[0]["dtype"] = 7
    assert orc.blob_check(b) == orc.ERR_UNSUPPORTED


def test_equidistant_exit_placement(orc):
    """The variant with exits equidistant in work (Sec. IV, "Benchmarks"): same layers as the ResNet-50-style network,
    segment ends at the block ends closest to quarters of the total multiply-accumulates."""
    eq, ref = W.build_net("resnet50_eq_i8"), W.build_net("resnet50_i8")
    assert orc.blob_check(eq) == orc.OK
    keys = ("kind", "h_in", "w_in", "c_in", "h_out", "w_out", "c_out", "kh", "kw", "stride", "pad")
    assert len(eq.ops) == len(ref.ops) and all(int(a[k]) == int(b[k]) for a, b in zip(eq.ops, ref.ops) for k in keys)
    macs = lambda op: int(op["h_out"]) * int(op["w_out"]) * int(op["c_out"]) * int(op["kh"]) * int(op["kw"]) * int(op["c_in"]) * (int(op["kind"]) == 0)
    per = [sum(macs(op) for op in eq.ops[int(st["first_op"]):int(st["first_op"]) + int(st["n_ops"])]) for st in eq.stages]
    cum = np.cumsum(per) / sum(per)
    assert np.all(np.abs(cum - np.array([0.25, 0.5, 0.75, 1.0])) < 0.04)
    assert [eq.stage_out_shape(s) for s in range(4)] == [(28, 28, 512), (14, 14, 1024), (14, 14, 1024), (7, 7, 2048)]


def test_stage_forward_is_the_composition_of_its_layers(orc, tiny):
    x = W.input_pool(tiny, 5)
    ops = tiny.stage_ops(0)
    t = x
    for op in ops:
        w, b = tiny.op_weights(op)
        acc = orc.conv_acc_i8(t, w.reshape(int(op["c_out"]), 3, 3, int(op["c_in"])), b, int(op["stride"]), int(op["pad"]))
        t = orc.requant_i8(acc, None, int(op["shift"]), 0, int(op["lo"]), int(op["hi"]))
    assert np.array_equal(orc.stage_forward(tiny, 0, x), t)


def test_residual_network_segment_against_layerwise(orc):
    net = W.load_net("resnet50_small_i8")
    x = W.input_pool(net, 2)
    tens = {0: x}
    for op in net.stage_ops(0):
        src = tens[int(op["src"])]
        if int(op["kind"]) == W.OP_MAXPOOL:
            y = orc.maxpool_i8(src, int(op["kh"]), int(op["stride"]), int(op["pad"]))
        else:
            w, b = net.op_weights(op)
            acc = orc.conv_acc_i8(src, w.reshape(int(op["c_out"]), int(op["kh"]), int(op["kw"]), int(op["c_in"])), b,
                                  int(op["stride"]), int(op["pad"]))
            res = tens[int(op["res"])] if int(op["res"]) >= 0 else None
            y = orc.requant_i8(acc, res, int(op["shift"]), int(op["res_shift"]), int(op["lo"]), int(op["hi"]))
        tens[int(op["dst"])] = y
    out = orc.stage_forward(net, 0, x)
    assert np.array_equal(out, tens[int(net.stages[0]["out_tensor"])])
    assert 0 < np.count_nonzero(out) < out.size           # calibrated shifts keep the signal alive
    assert any(int(op["res"]) >= 0 for op in net.stage_ops(0))


def test_concatenation_network_segment_against_layerwise(orc):
    """Inception-style segments: every op computed on its own with the primitives (rectangular kernels with their
    per-axis padding, average and max pooling) and written into its channel slice by hand equals the segment."""
    net = W.load_net("inception_small_i8")
    x = W.input_pool(net, 2)
    kinds = set()
    for s in (0, 1):
        tens = {0: x}
        for op in net.stage_ops(s):
            src, kind, k = tens[int(op["src"])], int(op["kind"]), int(op["kh"])
            kinds.add((kind, int(op["kh"]), int(op["kw"])))
            if kind == W.OP_MAXPOOL:
                y = orc.maxpool_i8(src, k, int(op["stride"]), int(op["pad"]))
            elif kind == W.OP_AVGPOOL:
                y = orc.avgpool_i8(src, k, int(op["stride"]), int(op["pad"]))
            else:
                w, b = net.op_weights(op)
                acc = orc.conv_acc_i8(src, w.reshape(int(op["c_out"]), int(op["kh"]), int(op["kw"]), int(op["c_in"])), b,
                                      int(op["stride"]), int(op["pad"]), pad_w=int(op["pad_w"]))
                y = orc.requant_i8(acc, None, int(op["shift"]), 0, int(op["lo"]), int(op["hi"]))
            dst, c_off, c_tot, co = int(op["dst"]), int(op["c_off"]), int(op["c_tot"]), int(op["c_out"])
            if c_tot == co:
                tens[dst] = y
            else:
                tens.setdefault(dst, np.full(y.shape[:3] + (c_tot,), 99, np.int8))[..., c_off:c_off + co] = y
        out = orc.stage_forward(net, s, x)
        assert np.array_equal(out, tens[int(net.stages[s]["out_tensor"])])
        assert 0 < np.count_nonzero(out) < out.size
        x = out
    assert {(0, 1, 7), (0, 7, 1), (0, 5, 5), (0, 3, 3), (0, 1, 1), (2, 3, 3), (3, 3, 3)} <= kinds
    bad = W.load_net("inception_small_i8")
    op = next(o for o in bad.ops if int(o["c_tot"]) != int(o["c_out"]))
    op["c_off"] += 16                                       # a slice that overlaps its neighbour / leaves a gap
    assert orc.blob_check(bad) == orc.ERR_SHAPE


def test_thresholds_zero_and_above_one(orc, tiny):
    x = W.input_pool(tiny, 16)
    for thr, expect_exit in ((0.0, 0), (1.5, tiny.n_stages - 1)):
        b = W.load_net("tiny_i8")
        b.exits["thr"] = thr
        res = orc.forward_alone(b, x)
        assert np.all(res["exit_idx"] == expect_exit)
    # exit head directly: the last exit takes everybody whatever the threshold
    act = orc.stage_forward(tiny, 0, x)
    assert np.all(orc.exit_head(tiny, 0, act, 0.0)[3] == 1)
    assert np.all(orc.exit_head(tiny, 0, act, 1.5)[3] == 0)
    a1 = orc.stage_forward(tiny, 1, act)
    a2 = orc.stage_forward(tiny, 2, a1)
    assert np.all(orc.exit_head(tiny, 2, a2, 1.5)[3] == 1)


def test_exit_head_is_gap_fc_softmax(orc, tiny):
    x = W.input_pool(tiny, 6)
    act = orc.stage_forward(tiny, 0, x)
    e = tiny.exits[0]
    thr = float(e["thr"])
    label, conf, score, flag, logits = orc.exit_head(tiny, 0, act, thr, want_logits=True)
    _, g = orc.gap_i8(act, int(e["gap_shift"]))
    w, b = tiny.exit_weights(0)
    a = orc.fc_i8(g, w.reshape(10, -1), b)
    lab2, s2 = orc.softmax_top1_i8(a, int(e["frac_bits"]))
    assert np.array_equal(logits, a) and np.array_equal(label, lab2) and np.array_equal(score, s2)
    assert np.array_equal(flag, (s2 <= orc.score_threshold(thr)).astype(np.uint8))
    assert np.allclose(conf, 2.0**30 / s2, rtol=1e-6)
    assert np.array_equal(label, a.argmax(axis=1))


def test_compaction_all_flag_patterns(orc):
    act = np.arange(8 * 6, dtype=np.int8).reshape(8, 1, 2, 3)
    ids = np.arange(100, 108, dtype=np.int32)
    refill = -np.arange(1, 2 * 6 + 1, dtype=np.int8).reshape(2, 1, 2, 3)
    rids = np.array([7, 9], np.int32)
    for pattern in itertools.product((0, 1), repeat=8):
        flags = np.array(pattern, np.uint8)
        keep = [k for k in range(8) if not pattern[k]]
        dst, ids_dst, b_rem, b_merged = orc.compact_refill(flags, act, ids, refill, rids)
        assert b_rem == len(keep) and b_merged == len(keep) + 2
        assert np.array_equal(dst[:b_rem], act[keep]) and np.array_equal(dst[b_rem:], refill)
        assert ids_dst.tolist() == [100 + k for k in keep] + [7, 9]
    dst, ids_dst, b_rem, b_merged = orc.compact_refill(np.ones(8, np.uint8), act, ids)
    assert b_rem == 0 and b_merged == 0 and dst.shape[0] == 0


def test_calibrated_split_is_roughly_the_configured_one(orc, tiny):
    x = W.input_pool(tiny, 64)
    res = orc.forward_alone(tiny, x)
    counts = np.bincount(res["exit_idx"], minlength=3)
    assert counts.sum() == 64 and np.all(counts > 6)


@pytest.mark.parametrize("b_max,refill", [(1, 0), (8, 0), (8, 1), (5, 1), (64, 1)])
def test_schedule_independence(orc, tiny, b_max, refill):
    """A sample's exit, label and score do not depend on batch size, slot or refill policy."""
    n = 64
    x = W.input_pool(tiny, n)
    alone = orc.forward_alone(tiny, x)
    lut = np.full((3, b_max), 1000, np.int64) + np.arange(b_max)[None, :] * 10
    arrivals = (np.arange(n) * 137).astype(np.int64)
    res, st, _ = orc.serve_stream(tiny, arrivals, x, b_max, lut, refill=refill)
    for f in ("exit_idx", "label", "score"):
        assert np.array_equal(res[f], alone[f]), f
    assert np.bincount(res["exit_idx"], minlength=3).sum() == n
    assert np.all(res["latency_ns"] > 0)
    assert st["seg_samples"][0] == n


def test_bf16_forward_runs_and_exits_once(orc):
    net = W.load_net("tiny_bf16")
    x = W.input_pool(net, 32)
    res = orc.forward_alone(net, x)
    assert np.all((res["exit_idx"] >= 0) & (res["exit_idx"] < 3))
    assert len(set(res["exit_idx"].tolist())) >= 2
    assert np.all((res["conf"] > 0) & (res["conf"] <= 1.0))
