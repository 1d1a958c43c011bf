"""GPU parity: the HIP path through the C ABI against the CPU oracle, element by element.

int8 networks must match bit for bit (activations, logits, labels, scores, exit flags, compaction
order, and on the virtual clock the whole schedule).  bf16 networks: logits within 2e-2 of the
per-sample max-norm, confidences within 1e-3, exit decisions equal unless the oracle's confidence is
within 1e-3 of the threshold."""
import sys

import numpy as np
import pytest

import workloads as W

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def torch():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    return torch


@pytest.fixture(scope="module")
def ee():
    import paper_2209_13443_amd as ee
    return ee


def dev(torch, a):
    if a.dtype == np.uint16:
        a = a.view(np.int16)
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t, like):
    a = t.cpu().numpy()
    return a.view(np.uint16) if like.dtype == np.uint16 else a


I8_NETS = ["tiny_i8", "zoo_i8", "resnet50_small_i8", "resnet18_small_i8", "mobilenetv2_small_i8", "inception_small_i8"]


@pytest.mark.parametrize("name", I8_NETS)
def test_int8_segments_and_heads_bit_exact(torch, ee, orc, name):
    blob = W.load_net(name)
    eng = ee.Engine(blob, 16)
    x = W.input_pool(blob, 13)
    for b in (1, 13, 6):                                   # ragged batches, smaller after larger
        act = x[:b]
        for s in range(blob.n_stages):
            say(f"[case] {name} segment {s} b={b}")
            ref = orc.stage_forward(blob, s, act)
            got = eng.stage_forward(s, dev(torch, act), ref.shape[1:])
            torch.cuda.synchronize()
            got = host(got, ref)
            assert np.array_equal(got, ref), f"{name} stage {s} b={b}: {np.count_nonzero(got != ref)} of {ref.size} differ"
            thr = float(blob.exits[s]["thr"])
            lab, conf, score, flag, logits = orc.exit_head(blob, s, ref, thr, want_logits=True)
            glab, gconf, gscore, gflag = eng.exit_head(s, dev(torch, ref), thr)
            glog = eng.last_logits(b, logits.shape[1])
            assert np.array_equal(glog, logits)
            assert np.array_equal(glab.cpu().numpy(), lab) and np.array_equal(gscore.cpu().numpy(), score)
            assert np.array_equal(gflag.cpu().numpy(), flag)
            assert np.allclose(gconf.cpu().numpy(), conf, rtol=1e-6, atol=0)
            act = ref
    eng.close()


@pytest.mark.parametrize("seed", range(24))
def test_random_networks_bit_exact(torch, ee, orc, seed):
    """Generated networks (rectangular kernels, per-axis padding, strides, residuals, depthwise, pooling, concatenated
    slices at odd offsets, channel counts that are not multiples of 16): every segment and head against the oracle."""
    blob = W.random_net(seed, W.DT_I8)
    say(f"[case] random int8 network {seed}: {len(blob.ops)} layers")
    eng = ee.Engine(blob, 8)
    x = W.input_pool(blob, 7)
    for b in (7, 2):
        act = x[:b]
        for s in range(blob.n_stages):
            ref = orc.stage_forward(blob, s, act)
            got = host(eng.stage_forward(s, dev(torch, act), ref.shape[1:]), ref)
            assert np.array_equal(got, ref), f"network {seed} segment {s} b={b}: {np.count_nonzero(got != ref)} of {ref.size} differ"
            lab, conf, score, flag = orc.exit_head(blob, s, ref, 0.5)
            glab, gconf, gscore, gflag = eng.exit_head(s, dev(torch, ref), 0.5)
            assert np.array_equal(glab.cpu().numpy(), lab) and np.array_equal(gscore.cpu().numpy(), score) and np.array_equal(gflag.cpu().numpy(), flag)
            act = ref
    assert 0 < np.count_nonzero(ref) < ref.size or blob.n_stages == 1
    eng.close()


EDGE_SHAPES = [(1, 1, 16), (2, 5, 16), (3, 3, 48), (7, 7, 32), (9, 13, 16), (4, 17, 144)]


@pytest.mark.parametrize("kind", ["maxpool", "avgpool", "dw"])
def test_int8_3x3_window_layers_edge_shapes_and_values(torch, ee, orc, kind):
    """The 3x3 pooling and depthwise kernels alone (a segment that is one layer), on shapes around their 4-pixel
    groups and borders, strides 1 and 2, paddings 0..2, with inputs of extreme values: all -128, all 127, a mix of
    -128 / 127 / 0 / -1 (negative half-way cases of the average's rounding) and uniform bytes."""
    r = np.random.default_rng(99)
    for h, w, c in EDGE_SHAPES:
        for stride in (1, 2):
            for pad in (0, 1, 2):
                if min(h, w) + 2 * pad < 3:
                    continue
                blob = W.single_layer_net(kind, h, w, c, 3, stride, pad, W.DT_I8, seed=h * 31 + w)
                say(f"[case] {kind} {h}x{w}x{c} stride {stride} pad {pad}")
                x = np.concatenate([np.full((1, h, w, c), -128, np.int8), np.full((1, h, w, c), 127, np.int8),
                                    r.choice(np.array([-128, 127, 0, -1], np.int8), size=(3, h, w, c)),
                                    r.integers(-128, 128, size=(2, h, w, c), dtype=np.int8)])
                eng = ee.Engine(blob, 8)
                for b in (7, 1):
                    ref = orc.stage_forward(blob, 0, x[:b])
                    got = host(eng.stage_forward(0, dev(torch, x[:b]), ref.shape[1:]), ref)
                    assert np.array_equal(got, ref), f"{kind} {h}x{w}x{c} s{stride} p{pad} b={b}: {np.count_nonzero(got != ref)} of {ref.size} differ"
                eng.close()


IR_CASES = [  # h, w, c_in, expanded, c_out (per block), stride, blocks, samples
    (9, 11, 16, 48, 16, 1, 2, 7), (8, 8, 24, 144, (24, 32), 1, 2, 7), (13, 8, 24, 144, 32, 2, 1, 7), (14, 14, 64, 208, 64, 1, 1, 5),
    (7, 7, 160, 320, 160, 1, 1, 3), (16, 16, 16, 96, (24, 16), 2, 2, 7), (5, 6, 8, 48, (40, 16), 1, 2, 7), (7, 7, 96, 160, 128, 1, 1, 3),
    (20, 18, 32, 64, 96, 1, 1, 3), (1, 1, 16, 32, 16, 1, 1, 2), (3, 2, 32, 96, (8, 16), 2, 2, 2), (28, 28, 32, 192, 32, 1, 1, 40),
    # without expansion (depthwise -> projection): one and several channel groups, both forms of the kernel
    (9, 11, 32, 0, 16, 1, 1, 7), (8, 8, 48, 0, (32, 16), 2, 2, 7), (14, 14, 144, 0, 64, 1, 1, 5), (7, 7, 208, 0, 96, 1, 1, 3), (12, 20, 16, 0, 16, 1, 2, 7),
    (28, 28, 32, 0, 16, 1, 1, 40),
]


@pytest.mark.parametrize("case", IR_CASES, ids=lambda c: "x".join(str(v) if isinstance(v, int) else "_".join(map(str, v)) for v in c))
def test_fused_inverted_residual_blocks_equal_separate_layers_and_oracle(torch, ee, orc, case):
    """Expansion -> depthwise -> projection (+ residual) as one launch: shapes around the kernel's pixel blocks (8, 14 and 7
    columns), channel groups (expanded channels that are and are not multiples of 32), output blocks (8 .. 160 channels, partial
    16-byte stores), strides, one- and two-block segments, extreme inputs; against the oracle and against the three
    separate layers, bit for bit."""
    h, w, ci, ce, co, stride, blocks, n = case
    blob = W.inverted_residual_net(h, w, ci, ce, co, stride, seed=h * 7 + ce, blocks=blocks)
    say(f"[case] inverted residual {h}x{w} {ci} -> {ce if ce else 'no expansion'} -> {co} stride {stride}, {blocks} block(s), {n} samples")
    r = np.random.default_rng(h * 100 + ce)
    x = np.concatenate([np.full((1, h, w, ci), -128, np.int8), np.full((1, h, w, ci), 127, np.int8),
                        r.integers(-128, 128, size=(max(n - 2, 1), h, w, ci), dtype=np.int8)])[:n]
    eng = ee.Engine(blob, max(n, 2))
    assert eng.ir_count() == blocks
    for b in sorted({n, 1}, reverse=True):
        ref = orc.stage_forward(blob, 0, x[:b])
        for mode in (2, 0, 2):
            eng.ir_mode(mode)
            got = host(eng.stage_forward(0, dev(torch, x[:b]), ref.shape[1:]), ref)
            assert np.array_equal(got, ref), f"mode {mode} b={b}: {np.count_nonzero(got != ref)} of {ref.size} differ, first at {np.argwhere(got != ref)[:3].tolist()}"
    assert np.unique(ref).size > 8
    eng.close()


BN_CASES = [  # h, w, c_in, blocks, samples
    (8, 8, 64, 1, 3), (9, 11, 64, 2, 7), (5, 17, 256, 1, 7), (16, 8, 256, 2, 5), (1, 1, 64, 1, 2), (28, 28, 256, 1, 40), (56, 56, 64, 2, 6), (28, 28, 64, 2, 9),
]


@pytest.mark.parametrize("case", BN_CASES, ids=lambda c: "x".join(map(str, c)))
def test_fused_bottleneck_blocks_equal_separate_layers_and_oracle(torch, ee, orc, case):
    """1x1 -> 3x3 -> 1x1 + residual as one launch (64 middle channels, 256 out): images that are and are not whole tiles of
    8 x 8 pixels, a single pixel, 64 and 256 input channels (a convolution or the block's input as residual), more tiles than
    workgroups (a workgroup walks over several), extreme inputs; against the oracle and against the three separate layers,
    bit for bit."""
    h, w, ci, blocks, n = case
    blob = W.bottleneck_net(h, w, ci, seed=h * 7 + w, blocks=blocks)
    say(f"[case] bottleneck {h}x{w} {ci} -> 64 -> 64 -> 256, {blocks} block(s), {n} samples")
    r = np.random.default_rng(h * 100 + w)
    x = np.concatenate([np.full((1, h, w, ci), -128, np.int8), np.full((1, h, w, ci), 127, np.int8),
                        r.integers(-128, 128, size=(max(n - 2, 1), h, w, ci), dtype=np.int8)])[:n]
    eng = ee.Engine(blob, max(n, 2))
    heads = {i: eng.ir_layers(i) for i in range(len(blob.ops)) if eng.ir_layers(i)}
    # with 64 input channels the first block's residual is a convolution of the input: that layer heads a block of four
    assert sorted(heads.values()) == ([3] * blocks + [4] if ci == 64 else [3] * blocks) and eng.ir_count() == len(heads)
    for b in sorted({n, 1}, reverse=True):
        ref = orc.stage_forward(blob, 0, x[:b])
        for mode in (2, 0, 1, 2):
            eng.ir_mode(mode)
            if mode == 1:                                                  # by table: the blocks of three fused, the block of four not
                eng.load_tables({"ir": {str(i): [0 if span == 4 else 1] for i, span in heads.items()}})
            got = host(eng.stage_forward(0, dev(torch, x[:b]), ref.shape[1:]), ref)
            assert np.array_equal(got, ref), f"mode {mode} b={b}: {np.count_nonzero(got != ref)} of {ref.size} differ, first at {np.argwhere(got != ref)[:3].tolist()}"
    assert np.unique(ref).size > 8
    if (h, w) == (28, 28):                                                 # the table ee_autotune writes: an entry per head, results unchanged
        eng.autotune(reps=2)
        tabs = eng.tables()["ir"]
        assert sorted(map(int, tabs)) == sorted(heads) and all(set(v) <= {0, 1} for v in tabs.values())
        eng.ir_mode(1)
        ref = orc.stage_forward(blob, 0, x)
        got = host(eng.stage_forward(0, dev(torch, x), ref.shape[1:]), ref)
        assert np.array_equal(got, ref)
    eng.close()


def test_fused_inverted_residual_blocks_in_a_network(torch, ee, orc):
    """The MobileNetV2-style network with every block fused, with none fused and with the table ee_autotune writes: every
    segment and head against the oracle."""
    blob = W.load_net("mobilenetv2_small_i8")
    eng = ee.Engine(blob, 8)
    assert eng.ir_count() == 16                                            # every block but the last (320 output channels)
    x = W.input_pool(blob, 7)
    for step, mode in enumerate((2, 0, 1)):
        if step == 2:
            eng.autotune(reps=2)
            tabs = eng.tables()["ir"]
            assert len(tabs) == 16 and all(set(v) <= {0, 1} for v in tabs.values())
            eng.load_tables({"ir": tabs})
        eng.ir_mode(mode)
        act = x
        for s in range(blob.n_stages):
            ref = orc.stage_forward(blob, s, act)
            got = host(eng.stage_forward(s, dev(torch, act), ref.shape[1:]), ref)
            assert np.array_equal(got, ref), f"mode {mode} segment {s}: {np.count_nonzero(got != ref)} of {ref.size} differ"
            act = ref
    eng.close()


def test_int8_thin_1x1_layers_bit_exact(torch, ee, orc):
    """1x1 layers with 4..32 input channels (the kernel that feeds one matrix instruction per 32 x 32 outputs straight
    from global memory): every channel count, output widths that are and are not multiples of 32, pixel counts that
    end inside a strip of 32, extreme inputs, relu and linear clamps."""
    r = np.random.default_rng(7)
    for ci in (4, 8, 12, 16, 20, 24, 28, 32):
        for co, act in ((16, "linear"), (48, "relu"), (144, "relu6"), (160, "linear")):
            h, w = (4, 4) if (ci + co) % 3 else (3, 16)
            blob = W.single_layer_net("conv", h, w, ci, 1, 1, 0, W.DT_I8, seed=ci * 7 + co, co=co, act=act)
            say(f"[case] 1x1 conv {ci} -> {co} ({act}) on {h}x{w}")
            x = np.concatenate([np.full((1, h, w, ci), -128, np.int8), np.full((1, h, w, ci), 127, np.int8),
                                r.integers(-128, 128, size=(5, h, w, ci), dtype=np.int8)])
            eng = ee.Engine(blob, 8)
            for b in (7, 3, 1):
                ref = orc.stage_forward(blob, 0, x[:b])
                got = host(eng.stage_forward(0, dev(torch, x[:b]), ref.shape[1:]), ref)
                assert np.array_equal(got, ref), f"1x1 {ci}->{co} b={b}: {np.count_nonzero(got != ref)} of {ref.size} differ"
            assert 0 < np.count_nonzero(ref != ref.flat[0])
            eng.close()


STREAM_CASES = [  # (h, w, c, co, k, stride, pad): layers the streaming kernel covers, on shapes around its 32-pixel strips
    (9, 9, 32, 32, 3, 1, 1), (7, 11, 32, 64, 3, 1, 0), (12, 8, 32, 48, 3, 2, 1), (5, 5, 32, 16, 3, 2, 0), (6, 10, 32, 64, 3, 1, 2),
    (16, 16, 3, 64, 7, 2, 3), (12, 20, 3, 32, 3, 2, 1), (16, 15, 3, 32, 3, 2, 0), (8, 8, 4, 48, 7, 2, 3), (10, 6, 32, 32, (1, 3), 1, (0, 1)),
    (10, 6, 32, 64, (3, 1), 1, (1, 0)),
]


@pytest.mark.parametrize("case", STREAM_CASES)
def test_int8_streaming_kernel_bit_exact(torch, ee, orc, case):
    """The streaming convolution kernel forced on single-layer segments it covers (folded stride-2 first layers, 3 x 3 /
    1 x 3 / 3 x 1 layers over 32 channels), extreme inputs included; and the same segments with the default choice."""
    h, w, c, co, k, stride, pad = case
    r = np.random.default_rng(11)
    if (h * w * c) % 16:
        pytest.skip("a sample must be whole 16-byte chunks")
    blob = W.single_layer_net("conv", h, w, c, k, stride, pad, W.DT_I8, seed=h * 13 + co, co=co, act="relu" if co % 32 else "linear")
    x = np.concatenate([np.full((1, h, w, c), -128, np.int8), np.full((1, h, w, c), 127, np.int8), r.integers(-128, 128, size=(6, h, w, c), dtype=np.int8)])
    for tile in (7, 0):
        old = ee.tune_conv_tile(tile)
        try:
            eng = ee.Engine(blob, 8)
            for b in (8, 5, 1):
                ref = orc.stage_forward(blob, 0, x[:b])
                got = host(eng.stage_forward(0, dev(torch, x[:b]), ref.shape[1:]), ref)
                assert np.array_equal(got, ref), f"{case} tile {tile} b={b}: {np.count_nonzero(got != ref)} of {ref.size} differ"
            eng.close()
        finally:
            ee.tune_conv_tile(old)
    assert 0 < np.count_nonzero(ref != ref.flat[0])


@pytest.mark.parametrize("seed", range(8))
def test_random_networks_bf16_within_tolerance(torch, ee, orc, seed):
    blob = W.random_net(seed, W.DT_BF16)
    say(f"[case] random bf16 network {seed}: {len(blob.ops)} layers")
    eng = ee.Engine(blob, 8)
    act = W.input_pool(blob, 5)
    for s in range(blob.n_stages):
        ref = orc.stage_forward(blob, s, act)
        got = host(eng.stage_forward(s, dev(torch, act), ref.shape[1:]), ref)
        r, g = bf16_to_f32(ref).astype(np.float64), bf16_to_f32(got).astype(np.float64)
        scale = np.abs(r).reshape(r.shape[0], -1).max(axis=1).reshape(-1, 1, 1, 1) + 1e-30
        assert np.all(np.abs(g - r) <= 2e-2 * scale), f"network {seed} segment {s}: {np.max(np.abs(g - r) / scale)}"
        act = ref
    eng.close()


@pytest.mark.parametrize("tile", [1, 2, 3, 4, 7])
@pytest.mark.parametrize("name", ["zoo_i8", "resnet50_small_i8"])
def test_int8_every_conv_tiling_bit_exact(torch, ee, orc, name, tile):
    blob = W.load_net(name)
    eng = ee.Engine(blob, 8)
    x = W.input_pool(blob, 5)
    old = ee.tune_conv_tile(tile)
    try:
        act = x
        for s in range(blob.n_stages):
            say(f"[case] {name} tile {tile} segment {s}")
            ref = orc.stage_forward(blob, s, act)
            got = host(eng.stage_forward(s, dev(torch, act), ref.shape[1:]), ref)
            assert np.array_equal(got, ref), f"tile {tile} stage {s}"
            act = ref
    finally:
        ee.tune_conv_tile(old)
    eng.close()


@pytest.mark.gpu
@pytest.mark.parametrize("cfg", [0x0321, 0x0421, 0x0231, 0x0331, 0x0322, 0x0432, 0x0323, 0x0433, 0x0324, 0x0234,
                                 0x10321, 0x10431, 0x10222, 0x10332, 0x10323, 0x10233, 0x10324, 0x10434])
def test_int8_pipelined_steps_bit_exact(torch, ee, orc, cfg):
    """Reduction steps of 128 and 256 bytes run the pipelined form of the inner loop (fragments read two sub-steps ahead,
    barrier before the end of a step): every tiling of it with rings of 2, 3 and 4 stages, on layers with one, two and
    many steps and a ragged last tile, against the oracle.  Words with bit 16 name the slab kernel (stride-1 layers whose
    output is as large as the input; the other layers keep their default kernel): its four tiles, both weight steps."""
    for name in ("zoo_i8", "resnet50_small_i8") if cfg < 0x10000 else ("resnet50_small_i8", "resnet18_small_i8", "inception_small_i8"):
        blob = W.load_net(name)
        eng = ee.Engine(blob, 8)
        x = W.input_pool(blob, 5)
        old = ee.tune_conv_tile(cfg)
        try:
            act = x
            for s in range(blob.n_stages):
                say(f"[case] {name} cfg {cfg:#x} segment {s}")
                ref = orc.stage_forward(blob, s, act)
                got = host(eng.stage_forward(s, dev(torch, act), ref.shape[1:]), ref)
                assert np.array_equal(got, ref), f"cfg {cfg:#x} stage {s}"
                act = ref
        finally:
            ee.tune_conv_tile(old)
        eng.close()


def test_autotuned_configuration_table_keeps_results(torch, ee, orc):
    """The per-(layer, batch bucket) kernel configuration table only changes speed, never a byte."""
    for name in ("resnet50_small_i8", "zoo_i8"):
        blob = W.load_net(name)
        eng = ee.Engine(blob, 12)
        eng.autotune(reps=2)
        tables = [eng.config_table(k) for k in range(len(blob.ops))]
        assert any(len(t) > 0 for t in tables)
        for t in tables:
            for cfg in t:
                assert cfg == 7 or (1 <= (cfg & 15) <= 4 and 1 <= ((cfg >> 4) & 15) <= 3 and 2 <= ((cfg >> 8) & 15) <= 4 and (cfg >> 12) in (0, 2, 4))
        x = W.input_pool(blob, 11)
        for b in (11, 3, 1):
            act = x[:b]
            for s in range(blob.n_stages):
                say(f"[case] autotuned {name} segment {s} b={b}")
                ref = orc.stage_forward(blob, s, act)
                got = host(eng.stage_forward(s, dev(torch, act), ref.shape[1:]), ref)
                assert np.array_equal(got, ref)
                act = ref
        # the table is plain data: a second engine loads it and runs the same configurations
        stored = eng.tables()
        other = ee.Engine(blob, 12)
        other.load_tables(stored)
        assert other.tables() == stored
        ref = orc.stage_forward(blob, 0, x)
        assert np.array_equal(host(other.stage_forward(0, dev(torch, x), ref.shape[1:]), ref), ref)
        with pytest.raises(ee.EEError):
            other.load_tables({"config": {"0": [0x99]}})                    # tile 9 does not exist
        # the streaming kernel as a stored entry: accepted for the folded first layer it covers (results unchanged),
        # refused for a layer it does not cover (one with a residual)
        if name == "resnet50_small_i8":
            other.load_tables({"config": {"0": [7] * len(stored["config"]["0"])}})
            assert np.array_equal(host(other.stage_forward(0, dev(torch, x), ref.shape[1:]), ref), ref)
            with_res = next(k for k, op in enumerate(blob.ops) if int(op["res"]) >= 0 and str(k) in stored["config"])
            with pytest.raises(ee.EEError):
                other.load_tables({"config": {str(with_res): [7]}})
        other.close()
        eng.close()


def test_thresholds_zero_and_above_one(torch, ee, orc):
    blob = W.load_net("tiny_i8")
    eng = ee.Engine(blob, 8)
    x = W.input_pool(blob, 8)
    a0 = eng.stage_forward(0, dev(torch, x), blob.stage_out_shape(0))
    assert np.all(eng.exit_head(0, a0, 0.0)[3].cpu().numpy() == 1)       # threshold 0: everyone leaves at exit 1
    assert np.all(eng.exit_head(0, a0, 1.5)[3].cpu().numpy() == 0)       # threshold > 1: nobody leaves early
    a1 = eng.stage_forward(1, a0, blob.stage_out_shape(1))
    a2 = eng.stage_forward(2, a1, blob.stage_out_shape(2))
    assert np.all(eng.exit_head(2, a2, 1.5)[3].cpu().numpy() == 1)       # ... and the last exit takes everybody
    eng.close()


def test_edge_arguments_on_device(torch, ee):
    blob = W.load_net("tiny_i8")
    eng = ee.Engine(blob, 4)
    lib = ee.raw()
    x = dev(torch, W.input_pool(blob, 4))
    out = torch.empty((4,) + blob.stage_out_shape(0), dtype=torch.int8, device="cuda")
    assert lib.ee_stage_forward(eng._h, 0, 0, None, None) == ee.EE_OK           # empty batch is a no-op
    assert lib.ee_stage_forward(eng._h, 0, 5, x.data_ptr(), out.data_ptr()) == ee.EE_ERR_ARG   # above b_max
    assert lib.ee_stage_forward(eng._h, 3, 1, x.data_ptr(), out.data_ptr()) == ee.EE_ERR_ARG   # no such segment
    assert lib.ee_stage_forward(eng._h, 0, 1, x.data_ptr() + 1, out.data_ptr()) == ee.EE_ERR_ARG  # misaligned
    assert lib.ee_stage_forward(eng._h, 0, 1, x.data_ptr(), x.data_ptr()) == ee.EE_ERR_ARG     # aliasing
    assert lib.ee_exit_head(eng._h, 0, 0, None, 0.5, None, None, None, None) == ee.EE_OK
    eng.close()


def test_compaction_and_refill(torch, ee, orc):
    blob = W.load_net("zoo_i8")
    b_max = 24
    eng = ee.Engine(blob, b_max)
    rng = np.random.default_rng(7)
    shape = blob.stage_out_shape(0)
    act = rng.integers(-128, 128, size=(16,) + shape).astype(np.int8)
    refill = rng.integers(-128, 128, size=(5,) + shape).astype(np.int8)
    ids = rng.permutation(1000)[:16].astype(np.int32)
    rids = (2000 + np.arange(5)).astype(np.int32)
    patterns = [np.zeros(16, np.uint8), np.ones(16, np.uint8)] + [rng.integers(0, 2, 16).astype(np.uint8) for _ in range(6)]
    for k, flags in enumerate(patterns):
        for with_refill in (False, True):
            say(f"[case] compaction pattern {k} refill={with_refill}")
            r_act, r_ids = (refill, rids) if with_refill else (None, None)
            ref = orc.compact_refill(flags, act, ids, r_act, r_ids)
            got = eng.compact_refill(0, dev(torch, flags), dev(torch, act), dev(torch, ids),
                                     None if r_act is None else dev(torch, r_act), None if r_ids is None else dev(torch, r_ids))
            assert got[2] == ref[2] and got[3] == ref[3]
            assert np.array_equal(got[0].cpu().numpy(), ref[0]) and np.array_equal(got[1].cpu().numpy(), ref[1])
    eng.close()


def synthetic_lut(n_stages, b_max):
    return (np.arange(1, n_stages + 1)[:, None] * 1000 + np.arange(b_max)[None, :] * 37).astype(np.int64)


SERVE_CASES = [  # name, n, b_max, arrival gap ns, slo, min_incr, refill
    ("tiny_i8", 64, 8, 0, -1, 1, 1),            # configuration 1: 64 requests, 8 slots, all at t = 0
    ("tiny_i8", 64, 8, 450, 9000, 1, 1),
    ("tiny_i8", 50, 5, 300, -1, 2, 1),
    ("tiny_i8", 40, 8, 0, -1, 1, 0),
    ("zoo_i8", 48, 8, 700, -1, 1, 1),
    ("resnet50_small_i8", 40, 8, 900, 30000, 1, 1),
    ("mobilenetv2_small_i8", 32, 8, 600, -1, 1, 1),
    ("tiny_i8", 64, 8, 0, -1, 1, 2),            # stage pools: full batches from the pools in front of the segments
    ("tiny_i8", 64, 8, 450, 9000, 1, 2),
    ("tiny_i8", 50, 5, 300, -1, 1, 2),
    ("zoo_i8", 48, 8, 700, 12000, 1, 2),
    ("resnet50_small_i8", 60, 8, 200, -1, 1, 2),
    ("mobilenetv2_small_i8", 40, 8, 100, -1, 1, 2),
    ("inception_small_i8", 40, 8, 300, -1, 1, 2),
    ("inception_small_i8", 32, 8, 0, -1, 1, 1),
]


@pytest.mark.parametrize("case", SERVE_CASES)
def test_serve_stream_virtual_clock_matches_oracle(torch, ee, orc, case):
    name, n, b_max, gap, slo, min_incr, refill = case
    say(f"[case] serve {case}")
    blob = W.load_net(name)
    pool = W.input_pool(blob, n)
    arrivals = (np.arange(n) * gap).astype(np.int64)
    lut = synthetic_lut(blob.n_stages, b_max)
    ref, rst, rev = orc.serve_stream(blob, arrivals, pool, b_max, lut, t_slo_ns=slo, min_incr=min_incr, refill=refill, max_events=5000)
    eng = ee.Engine(blob, b_max)
    got, gst, gev = eng.serve_stream(arrivals, dev(torch, pool), lut, clock=1, t_slo_ns=slo, min_incr=min_incr, refill=refill, max_events=5000)
    for f in ("exit_idx", "label", "score", "latency_ns"):
        assert np.array_equal(got[f], ref[f]), f
    assert np.allclose(got["conf"], ref["conf"], rtol=1e-6)
    assert gst == rst
    assert np.array_equal(gev, rev)
    counts = np.bincount(got["exit_idx"], minlength=blob.n_stages)
    assert counts.sum() == n                                              # everyone leaves exactly once
    eng.close()


def test_serve_stream_wall_clock_invariants(torch, ee, orc):
    blob = W.load_net("tiny_i8")
    n, b_max = 64, 8
    pool = W.input_pool(blob, n)
    alone = orc.forward_alone(blob, pool)
    eng = ee.Engine(blob, b_max)
    lut = eng.measure_lut(reps=2)
    assert lut.shape == (3, b_max) and np.all(lut > 0)
    arrivals = (np.arange(n) * 20000).astype(np.int64)
    got, st, _ = eng.serve_stream(arrivals, dev(torch, pool), lut, clock=0)
    for f in ("exit_idx", "label", "score"):
        assert np.array_equal(got[f], alone[f]), f                       # schedule independence
    assert np.all(got["latency_ns"] > 0)
    assert st["seg_samples"][0] == n
    eng.close()


# ---- several steps in flight, and the baseline policies, on the GPU ---------------------------------------------
LANE_CASES = [  # name, n, b_max, arrival gap ns, slo, refill, lanes, t_timeout
    ("tiny_i8", 64, 8, 0, -1, 2, 2, 0),
    ("tiny_i8", 96, 8, 150, -1, 2, 3, 0),
    ("tiny_i8", 64, 8, 450, 9000, 2, 2, 0),
    ("zoo_i8", 64, 8, 100, -1, 2, 2, 0),
    ("resnet50_small_i8", 96, 8, 60, -1, 2, 2, 0),
    ("resnet50_small_i8", 96, 8, 0, -1, 2, 4, 0),
    ("mobilenetv2_small_i8", 64, 8, 50, -1, 2, 3, 0),
    ("inception_small_i8", 48, 8, 100, -1, 2, 2, 0),
    ("tiny_i8", 40, 8, 900, -1, 0, 1, 3000),       # adaptive batching <8, 3000 ns>
    ("zoo_i8", 40, 8, 400, -1, 0, 1, 100000),      # a window that always fills the batch
    ("tiny_i8", 24, 1, 500, -1, 0, 1, 0),          # SERIAL
]


@pytest.mark.parametrize("case", LANE_CASES)
def test_serve_stream_lanes_and_baselines_match_oracle(torch, ee, orc, case):
    name, n, b_max, gap, slo, refill, lanes, window = case
    say(f"[case] serve {case}")
    blob = W.load_net(name)
    pool = W.input_pool(blob, n)
    arrivals = (np.arange(n) * gap).astype(np.int64)
    lut = synthetic_lut(blob.n_stages, b_max)
    ref, rst, rev = orc.serve_stream(blob, arrivals, pool, b_max, lut, t_slo_ns=slo, refill=refill, lanes=lanes, t_timeout_ns=window, max_events=5000)
    eng = ee.Engine(blob, b_max)
    assert eng.set_lanes(lanes) == lanes
    dpool = dev(torch, pool)
    for rep in range(2):                                                   # the rings and lanes are reused by the second call
        got, gst, gev = eng.serve_stream(arrivals, dpool, lut, clock=1, t_slo_ns=slo, refill=refill, lanes=lanes, t_timeout_ns=window, max_events=5000)
        for f in ("exit_idx", "label", "score", "latency_ns"):
            assert np.array_equal(got[f], ref[f]), (f, rep)
        assert gst == rst and np.array_equal(gev, rev)
    if lanes > 1:
        assert np.any(gev["aux"][gev["kind"] == 2] > 0)                    # the other lanes did run steps
        with pytest.raises(ee.EEError):
            eng.serve_stream(arrivals, dpool, lut, clock=1, refill=2, lanes=lanes + 1)   # more lanes than ee_lanes made
    eng.close()


ZC_CASES = [  # name, n, b_max, arrival gap ns, slo, min_incr, refill, lanes
    ("tiny_i8", 64, 8, 0, -1, 1, 1, 1),              # Algorithm 1: parked survivors, catch-up batches merged behind them
    ("tiny_i8", 64, 8, 450, 9000, 1, 1, 1),
    ("tiny_i8", 50, 5, 300, -1, 2, 1, 1),
    ("tiny_i8", 40, 8, 0, -1, 1, 0, 1),              # model-level batching
    ("resnet50_small_i8", 40, 8, 900, 30000, 1, 1, 1),
    ("resnet50_small_i8", 60, 8, 200, -1, 1, 2, 1),  # stage pools, one lane
    ("resnet50_small_i8", 96, 8, 60, -1, 1, 2, 2),   # stage pools, two steps in flight
    ("resnet18_small_i8", 64, 8, 100, -1, 1, 2, 2),
    ("tiny_i8", 64, 8, 0, -1, 1, 2, 2),
]


@pytest.mark.parametrize("case", ZC_CASES)
def test_serve_stream_zero_copy_matches_oracle_and_copying(torch, ee, orc, case):
    """Zero-copy compaction (survivors stay where the segment wrote them, the next segment gathers them through a slot
    table): results, statistics and the whole event list equal the oracle's on the virtual clock, as with the copying kernel."""
    name, n, b_max, gap, slo, min_incr, refill, lanes = case
    say(f"[case] zero-copy serve {case}")
    blob = W.load_net(name)
    pool = W.input_pool(blob, n)
    arrivals = (np.arange(n) * gap).astype(np.int64)
    lut = synthetic_lut(blob.n_stages, b_max)
    ref, rst, rev = orc.serve_stream(blob, arrivals, pool, b_max, lut, t_slo_ns=slo, min_incr=min_incr, refill=refill, lanes=lanes, max_events=5000)
    eng = ee.Engine(blob, b_max)
    assert eng.zero_copy_supported()
    assert eng.set_lanes(lanes) == lanes
    dpool = dev(torch, pool)
    for zc in (1, 0, 1):                                                   # the slots are reused by later calls
        got, gst, gev = eng.serve_stream(arrivals, dpool, lut, clock=1, t_slo_ns=slo, min_incr=min_incr, refill=refill, lanes=lanes, max_events=5000, zero_copy=zc)
        for f in ("exit_idx", "label", "score", "latency_ns"):
            assert np.array_equal(got[f], ref[f]), (f, zc)
        assert gst == rst and np.array_equal(gev, rev)
    eng.close()


STEM_CASES = [(224, 224, 5), (57, 80, 7), (32, 32, 7), (17, 16, 3), (7, 16, 2), (114, 56, 9), (9, 48, 4)]      # h, w, samples (h * w a multiple of 16: whole 16-byte chunks per input sample)


@pytest.mark.parametrize("case", STEM_CASES, ids=lambda c: "x".join(map(str, c)))
def test_fused_first_convolution_and_pool_equal_separate_layers_and_oracle(torch, ee, orc, case):
    """7x7 / 2 convolution and 3x3 / 2 max-pool as one launch: images whose pooled size is and is not whole tiles of 14 x 4, odd
    sizes (the last pooled row or column sees one convolution row or column only), a pooled image smaller than a tile, extreme
    inputs; against the oracle and against the two separate layers, bit for bit."""
    h, w, n = case
    blob = W.stem_net(h, w, seed=h + w)
    say(f"[case] first convolution + pool on {h}x{w}, {n} samples")
    r = np.random.default_rng(h * 100 + w)
    x = np.concatenate([np.full((1, h, w, 3), -128, np.int8), np.full((1, h, w, 3), 127, np.int8),
                        r.integers(-128, 128, size=(max(n - 2, 1), h, w, 3), dtype=np.int8)])[:n]
    eng = ee.Engine(blob, max(n, 2))
    assert eng.ir_count() == 1 and eng.ir_layers(0) == 2
    for b in sorted({n, 1}, reverse=True):
        ref = orc.stage_forward(blob, 0, x[:b])
        for mode in (2, 0, 2):
            eng.ir_mode(mode)
            got = host(eng.stage_forward(0, dev(torch, x[:b]), ref.shape[1:]), ref)
            assert np.array_equal(got, ref), f"mode {mode} b={b}: {np.count_nonzero(got != ref)} of {ref.size} differ, first at {np.argwhere(got != ref)[:3].tolist()}"
    assert np.unique(ref).size > 8
    eng.close()


BN_SERVE_CASES = [  # h, w, c_in, seed, frac_bits, thresholds of the first two exits, lanes
    (12, 10, 64, 3, 11, (0.782, 0.955), 1), (16, 16, 256, 5, 12, (0.8371, 0.8453), 2),
]


@pytest.mark.parametrize("case", BN_SERVE_CASES, ids=lambda c: "x".join(map(str, c[:4])) + f"_lanes{c[6]}")
def test_serve_stream_with_fused_bottleneck_blocks(torch, ee, orc, case):
    """Three segments of two bottleneck blocks each, served with every block fused: the block that ends a segment also pools
    for the exit head and, with zero-copy compaction, writes its samples to their slots.  Results, statistics and events
    equal the oracle's on the virtual clock with the fused blocks, without them, with and without zero-copy compaction."""
    h, w, ci, seed, fb, thr, lanes = case
    blob = W.bottleneck_net(h, w, ci, seed=seed, blocks=2, stages=3)
    for e, t in zip(blob.exits, thr + (0.0,)):
        e["thr"], e["frac_bits"] = t, fb
    n, b_max = 96, 8
    say(f"[case] serve bottleneck net {case}")
    pool = W.input_pool(blob, n)
    arrivals = (np.arange(n) * 150).astype(np.int64)
    lut = synthetic_lut(blob.n_stages, b_max)
    ref, rst, rev = orc.serve_stream(blob, arrivals, pool, b_max, lut, refill=2, lanes=lanes, max_events=5000)
    assert np.all(np.bincount(ref["exit_idx"], minlength=3) > 0)           # every exit is taken
    eng = ee.Engine(blob, b_max)
    assert eng.ir_count() == (7 if ci == 64 else 6) and eng.zero_copy_supported()   # the first block of a later segment reads slots and stays unfused when served zero-copy
    assert eng.set_lanes(lanes) == lanes
    dpool = dev(torch, pool)
    for mode, zc in ((2, 1), (0, 1), (2, 0), (2, 1)):
        eng.ir_mode(mode)
        got, gst, gev = eng.serve_stream(arrivals, dpool, lut, clock=1, refill=2, lanes=lanes, max_events=5000, zero_copy=zc)
        for f in ("exit_idx", "label", "score", "latency_ns"):
            assert np.array_equal(got[f], ref[f]), (f, mode, zc)
        assert gst == rst and np.array_equal(gev, rev)
    eng.close()


def test_zero_copy_is_refused_where_it_cannot_run(torch, ee, orc):
    blob = W.load_net("mobilenetv2_small_i8")                               # depthwise / thin layers at the segment boundaries
    eng = ee.Engine(blob, 8)
    n = 16
    dpool = dev(torch, W.input_pool(blob, n))
    lut = synthetic_lut(blob.n_stages, 8)
    if not eng.zero_copy_supported():
        with pytest.raises(ee.EEError):
            eng.serve_stream(np.zeros(n, np.int64), dpool, lut, clock=1, zero_copy=1)
    eng.close()
    blob = W.load_net("tiny_i8")
    eng = ee.Engine(blob, 8)
    eng.set_lanes(3)
    dpool = dev(torch, W.input_pool(blob, n))
    lut = synthetic_lut(blob.n_stages, 8)
    with pytest.raises(ee.EEError):
        eng.serve_stream(np.zeros(n, np.int64), dpool, lut, clock=1, refill=2, lanes=3, zero_copy=1)    # the slots cover two steps in flight
    with pytest.raises(ee.EEError):
        eng.serve_stream(np.zeros(n, np.int64), dpool, lut, clock=1, zero_copy=2)
    eng.close()


def test_serve_stream_lanes_wall_clock(torch, ee, orc):
    """On the wall clock the schedule is a measurement; the per-request results are not (schedule independence)."""
    blob = W.load_net("resnet50_small_i8")
    n, b_max = 400, 16
    pool = W.input_pool(blob, n)
    alone = orc.forward_alone(blob, pool)
    eng = ee.Engine(blob, b_max)
    eng.set_lanes(3)
    lut = eng.measure_lut(reps=2)
    dpool = dev(torch, pool)
    for lanes, arrivals in ((3, np.zeros(n, np.int64)), (2, (np.arange(n) * 3000).astype(np.int64)), (1, np.zeros(n, np.int64))):
        say(f"[case] wall clock, lanes {lanes}")
        got, st, ev = eng.serve_stream(arrivals, dpool, lut, clock=0, refill=2, lanes=lanes, max_events=20000)
        for f in ("exit_idx", "label", "score"):
            assert np.array_equal(got[f], alone[f]), (f, lanes)
        assert np.all(got["latency_ns"] > 0) and st["seg_samples"][0] == n
        assert set(ev["aux"][ev["kind"] == 2].tolist()) <= set(range(lanes))
    eng.close()


# ---- full-size configurations, in the launch configuration the benchmark uses ------------------------------------
def golden(name):
    """tests/golden/full_size_<net>.txt, written by tests/golden/make_full_size_golden.py from the oracle alone"""
    import os
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", f"full_size_{name}.txt")
    rows = [line.split() for line in open(path) if not line.startswith("#")]
    return (np.array([int(r[1]) for r in rows]), np.array([int(r[2]) for r in rows]), np.array([int(r[3]) for r in rows], np.int64),
            np.array([float(r[4]) for r in rows], np.float32))


FULL = [("resnet18_i8", 512, 32, [(0, 1, 0)]),                                      # static batches of 32: the configuration as stated
        ("resnet50_i8", 512, 64, [(2, 2, 0), (2, 1, 0), (1, 1, 32), (0, 1, 0)]),    # what the benchmark times, then the other policies
        ("mobilenetv2_i8", 512, 64, [(2, 2, 0), (1, 1, 1)]),
        ("resnet50_eq_i8", 256, 64, [(2, 2, 0)]),                                   # exits equidistant in work
        ("inception_i8", 256, 64, [(2, 2, 0)])]                                     # rectangular kernels, concatenation, average pooling


@pytest.mark.parametrize("case", FULL)
def test_full_size_every_request_against_the_oracle(torch, ee, orc, case):
    """Every request of a prefix of the benchmark's own pool, under the policies the benchmark runs, against what the oracle
    computed for it alone (stored by tests/golden/make_full_size_golden.py): exit, label and score, bit for bit."""
    name, n, b_max, policies = case
    blob = W.load_net(name)
    g_exit, g_label, g_score, _ = golden(name)
    assert len(g_exit) >= n
    pool = W.input_pool(blob, n)
    eng = ee.Engine(blob, b_max)
    eng.set_lanes(2)
    eng.autotune(reps=2)                                   # the launch configuration the benchmark times
    lut = synthetic_lut(blob.n_stages, b_max)
    dpool = dev(torch, pool)
    for refill, lanes, min_incr in policies:
        say(f"[case] full-size {name} n={n} b_max={b_max} refill={refill} lanes={lanes} min_incr={min_incr}")
        got, st, _ = eng.serve_stream(np.zeros(n, np.int64), dpool, lut, clock=1, refill=refill, lanes=lanes, min_incr=max(1, min_incr))
        assert np.array_equal(got["exit_idx"], g_exit[:n]) and np.array_equal(got["label"], g_label[:n]) and np.array_equal(got["score"], g_score[:n])
        say(f"[info] {name} exit counts {np.bincount(got['exit_idx'], minlength=blob.n_stages).tolist()} "
            f"mean batch {[round(a / max(b, 1), 1) for a, b in zip(st['seg_samples'], st['seg_runs'])]}")
    # on the wall clock, as the benchmark runs it; then with zero-copy compaction where the network allows it
    for zc in ((0, 1) if eng.zero_copy_supported() else (0,)):
        say(f"[case] full-size {name} wall clock zero_copy={zc}")
        got, st, _ = eng.serve_stream(np.zeros(n, np.int64), dpool, eng.measure_lut(reps=1), clock=0, refill=policies[0][0], lanes=policies[0][1], zero_copy=zc)
        assert np.array_equal(got["exit_idx"], g_exit[:n]) and np.array_equal(got["label"], g_label[:n]) and np.array_equal(got["score"], g_score[:n])
    eng.close()


@pytest.mark.parametrize("name,b_max", [("resnet18_i8", 32), ("resnet50_i8", 64), ("mobilenetv2_i8", 64), ("inception_i8", 64)])
def test_full_size_every_segment_element_by_element(torch, ee, orc, name, b_max):
    """All segments at the full benchmark batch with the autotuned table, no exits taken: sampled slots (first, middle,
    last, and the one before a tile boundary) of every segment's output against the oracle's chain for those samples."""
    blob = W.load_net(name)
    pool = W.input_pool(blob, b_max)
    slots = sorted({0, b_max // 2 - 1, b_max // 2, b_max - 1})
    eng = ee.Engine(blob, b_max)
    eng.autotune(reps=2)
    act, ref = dev(torch, pool), pool[slots]
    for s in range(blob.n_stages):
        say(f"[case] full-size {name} segment {s} at b={b_max}")
        if eng.ir_count():                                 # every inverted-residual block fused, whatever the tuned table says
            eng.ir_mode(2)
            forced = eng.stage_forward(s, act, blob.stage_out_shape(s))
            eng.ir_mode(1)
        act = eng.stage_forward(s, act, blob.stage_out_shape(s))
        if eng.ir_count():
            assert torch.equal(forced, act), f"{name} segment {s}: fused blocks differ from the tuned mix"
        ref = orc.stage_forward(blob, s, ref)
        got = act.cpu().numpy()[slots]
        assert np.array_equal(got, ref), f"{name} segment {s}: {np.count_nonzero(got != ref)} of {ref.size} differ"
        thr = float(blob.exits[s]["thr"])
        lab, conf, score, flag = orc.exit_head(blob, s, ref, thr)
        glab, gconf, gscore, gflag = eng.exit_head(s, act, thr)
        assert np.array_equal(glab.cpu().numpy()[slots], lab) and np.array_equal(gscore.cpu().numpy()[slots], score)
        assert np.array_equal(gflag.cpu().numpy()[slots], flag)
    eng.close()


# ---- fused layer pairs (conv2 -> conv3 of a bottleneck block in one launch) ------------------------------
@pytest.mark.parametrize("case", [("resnet50_i8", 5), ("resnet50_i8", 64), ("resnet50_bf16", 3), ("resnet50_bf16", 40)])
def test_fused_pairs_equal_separate_layers_and_oracle(torch, ee, orc, case):
    """Every segment of the ResNet-50-style network with all pairs fused against the same segment with none fused
    (same arithmetic, so equal bit for bit in both dtypes), at a batch with ragged tiles and at a full one; the
    fused first segment also against the oracle on sampled slots."""
    name, b = case
    say(f"[case] fused pairs {name} b={b}")
    blob = W.load_net(name)
    eng = ee.Engine(blob, b)
    # conv2 -> conv3 of the 3 + 4 + 6 blocks with up to 256 mid channels; in bf16 the 256-channel pairs do not fit LDS
    assert eng.pair_count() == (13 if blob.dtype == W.DT_I8 else 7)
    pool = W.input_pool(blob, b)
    act = dev(torch, pool)
    for s in range(blob.n_stages):
        say(f"[case] fused pairs {name} b={b} segment {s}")
        eng.pair_mode(0)
        ref = eng.stage_forward(s, act, blob.stage_out_shape(s))
        eng.pair_mode(2)
        got = eng.stage_forward(s, act, blob.stage_out_shape(s))
        assert torch.equal(got, ref), f"segment {s}"
        if s == 0:
            slots = sorted({0, b // 2, b - 1})
            want = orc.stage_forward(blob, 0, pool[slots])
            if blob.dtype == W.DT_I8:
                assert np.array_equal(host(got, want)[slots], want)
            else:
                r, g = bf16_to_f32(want).astype(np.float64), bf16_to_f32(host(got, want)[slots]).astype(np.float64)
                assert np.abs(g - r).max() <= 2e-2 * np.abs(r).max()
        act = ref
    eng.close()


# ---- bf16 ---------------------------------------------------------------------------------------------
def bf16_to_f32(a):
    return W.bf16_bits_to_f32(a)


def test_full_size_bf16_against_the_oracle(torch, ee, orc):
    """The ResNet-50-style bf16 network at its benchmark configuration (256 slots, autotuned kernel table, stage pools on
    two lanes, then Algorithm 1): the first 64 requests against what the oracle computed for each alone (stored by
    tests/golden/make_full_size_golden.py), under the tolerances for bf16; then every segment at the full batch element
    by element on sampled slots."""
    name, n, b_max = "resnet50_bf16", 320, 256
    say(f"[case] full-size {name} n={n} b_max={b_max}")
    blob = W.load_net(name)
    g_exit, g_label, _, g_conf = golden(name)
    m = len(g_exit)
    assert m >= 32
    pool = W.input_pool(blob, n)
    eng = ee.Engine(blob, b_max)
    eng.set_lanes(2)
    eng.autotune(reps=2)
    lut = synthetic_lut(blob.n_stages, b_max)
    thr = np.array([float(e["thr"]) for e in blob.exits], np.float32)
    for refill, lanes in ((2, 2), (1, 1)):
        got, st, _ = eng.serve_stream(np.zeros(n, np.int64), dev(torch, pool), lut, clock=1, refill=refill, lanes=lanes, min_incr=b_max // 2)
        assert np.bincount(got["exit_idx"], minlength=blob.n_stages).sum() == n and np.all(got["exit_idx"] >= 0)
        same = got["exit_idx"][:m] == g_exit
        # where the exits agree the confidences must: both sides computed the same head on the same path
        assert np.all(np.abs(got["conf"][:m][same] - g_conf[same]) <= 1e-3)
        # where they differ the library's confidence at the earlier of the two exits must sit within the tolerance of that
        # exit's threshold (the decision there was a toss-up); request by request through the oracle
        for sid in np.nonzero(~same)[0]:
            act, cleared = pool[sid:sid + 1], False
            for s_ in range(min(int(got["exit_idx"][sid]), int(g_exit[sid])) + 1):
                act = orc.stage_forward(blob, s_, act)
                _, conf, _, _ = orc.exit_head(blob, s_, act, float(thr[s_]))
                cleared = cleared or abs(float(conf[0]) - float(thr[s_])) < 1e-3
            assert cleared, f"request {sid}: exit {got['exit_idx'][sid]} vs oracle {g_exit[sid]} with no confidence near a threshold"
        say(f"[info] bf16 refill={refill}: {int(np.count_nonzero(~same))} of {m} requests sit within 1e-3 of a threshold")
        assert np.count_nonzero(~same) <= m // 8
    # every segment at the full batch, element by element on sampled slots
    slots = [0, 131, b_max - 1]
    act, ref = dev(torch, pool[:b_max]), pool[:b_max][slots]
    for s_ in range(blob.n_stages):
        say(f"[case] full-size bf16 segment {s_} at b=256")
        act = eng.stage_forward(s_, act, blob.stage_out_shape(s_))
        ref_next = orc.stage_forward(blob, s_, ref)
        r, g = bf16_to_f32(ref_next).astype(np.float64), bf16_to_f32(host(act, ref_next)[slots]).astype(np.float64)
        scale = np.abs(r).reshape(r.shape[0], -1).max(axis=1).reshape(-1, 1, 1, 1) + 1e-30
        assert np.all(np.abs(g - r) <= 2e-2 * scale), f"segment {s_}: {np.max(np.abs(g - r) / scale)}"
        ref = ref_next
    eng.close()


@pytest.mark.parametrize("name", ["tiny_bf16", "zoo_bf16", "resnet50_small_bf16", "inception_small_bf16"])
def test_bf16_within_tolerance(torch, ee, orc, name):
    blob = W.load_net(name)
    eng = ee.Engine(blob, 16)
    x = W.input_pool(blob, 12)
    for tile in (0, 1, 2, 3, 4, 0x0321, 0x0432, 0x10321, 0x10332, 0x10423, 0x10234):     # tiles, pipelined steps, the slab kernel
        ee.tune_conv_tile(tile)
        act = x
        for s in range(blob.n_stages):
            say(f"[case] {name} tile {tile:#x} segment {s}")
            ref = orc.stage_forward(blob, s, act)
            got = host(eng.stage_forward(s, dev(torch, act), ref.shape[1:]), ref)
            r, g = bf16_to_f32(ref).astype(np.float64), bf16_to_f32(got).astype(np.float64)
            scale = np.abs(r).reshape(r.shape[0], -1).max(axis=1).reshape(-1, 1, 1, 1) + 1e-30
            assert np.all(np.abs(g - r) <= 2e-2 * scale), f"stage {s}: {np.max(np.abs(g - r) / scale)}"
            thr = float(blob.exits[s]["thr"])
            lab, conf, _, flag, logits = orc.exit_head(blob, s, ref, thr, want_logits=True)
            glab, gconf, _, gflag = eng.exit_head(s, dev(torch, ref), thr)
            glog = eng.last_logits(ref.shape[0], logits.shape[1])
            zmax = np.abs(logits).max(axis=1, keepdims=True)
            assert np.all(np.abs(glog - logits) <= 2e-2 * zmax)
            assert np.all(np.abs(gconf.cpu().numpy() - conf) <= 1e-3)
            clear = np.abs(conf - np.float32(thr)) >= 1e-3
            assert np.array_equal(gflag.cpu().numpy()[clear], flag[clear])
            top2 = np.sort(logits, axis=1)[:, -2:]
            sure = (top2[:, 1] - top2[:, 0]) > 4e-2 * zmax[:, 0]
            assert np.array_equal(glab.cpu().numpy()[sure], lab[sure])
            act = ref
    ee.tune_conv_tile(0)
    eng.close()


def test_bf16_serve_stream_decisions(torch, ee, orc):
    name, n, b_max = "tiny_bf16", 64, 8
    blob = W.load_net(name)
    pool = W.input_pool(blob, n)
    eng = ee.Engine(blob, b_max)
    lut = synthetic_lut(blob.n_stages, b_max)
    got, st, _ = eng.serve_stream(np.zeros(n, np.int64), dev(torch, pool), lut, clock=1)
    # the oracle's view of every sample at every exit it reaches
    act, alive = pool, np.arange(n)
    unclear = np.zeros(n, bool)
    ref_exit = np.full(n, -1)
    for s in range(blob.n_stages):
        act = orc.stage_forward(blob, s, act)
        thr = float(blob.exits[s]["thr"])
        lab, conf, _, flag = orc.exit_head(blob, s, act, thr)
        if s < blob.n_stages - 1:
            unclear[alive[np.abs(conf - np.float32(thr)) < 1e-3]] = True
        ref_exit[alive[flag == 1]] = s
        act, alive = act[flag == 0], alive[flag == 0]
    ok = ~unclear
    assert np.array_equal(got["exit_idx"][ok], ref_exit[ok])
    assert np.bincount(got["exit_idx"], minlength=3).sum() == n
    eng.close()
