"""ee_exit_head_static, the exit head for callers that cannot allocate: its scratch memory is an array
inside the library image.  Called through the C ABI on two calls in a row, the second with a smaller batch
(the array keeps what the first call left), and compared with ee_exit_head on the same inputs: int8 bit for
bit, bf16 bit for bit as well (same kernels, same pooling splits, same order of the float additions)."""
import ctypes as C
import sys

import numpy as np
import pytest

import workloads as W

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def outputs(torch, b):
    return (torch.full((b,), -7, dtype=torch.int32, device="cuda"), torch.full((b,), -7.0, dtype=torch.float32, device="cuda"),
            torch.full((b,), -7, dtype=torch.int64, device="cuda"), torch.full((b,), 9, dtype=torch.uint8, device="cuda"))


@pytest.mark.parametrize("name", ["resnet50_small_i8", "mobilenetv2_small_i8", "resnet50_small_bf16"])
def test_static_scratch_head_equals_workspace_head(name):
    import torch
    import paper_2209_13443_amd as ee
    assert torch.cuda.is_available()
    lib = ee.raw()
    blob = W.load_net(name)
    b_max = 24
    eng = ee.Engine(blob, b_max)
    assert lib.ee_static_scratch_bytes() == 4 * 1024 * 1024
    x = W.input_pool(blob, b_max)
    xd = torch.from_numpy(x.view(np.int16) if x.dtype == np.uint16 else x).cuda()
    acts = []
    act = xd
    for s in range(blob.n_stages):
        act = eng.stage_forward(s, act, blob.stage_out_shape(s))
        acts.append(act)
    torch.cuda.synchronize()
    for s in range(blob.n_stages):
        thr = float(blob.exits[s]["thr"])
        for b in (b_max, 5):                                  # the second call is smaller: stale rows beyond it must not matter
            say(f"[case] {name} exit {s} b={b}")
            a = acts[s][:b].contiguous()
            ref = eng.exit_head(s, a, thr)
            torch.cuda.synchronize()
            got = outputs(torch, b)
            rc = lib.ee_exit_head_static(eng._h, s, b, C.c_void_p(a.data_ptr()), C.c_float(thr), C.c_void_p(got[0].data_ptr()),
                                         C.c_void_p(got[1].data_ptr()), C.c_void_p(got[2].data_ptr()), C.c_void_p(got[3].data_ptr()))
            assert rc == 0, ee.strerror(rc)
            torch.cuda.synchronize()
            for g, r, what in zip(got, ref, ("label", "conf", "score", "flag")):
                assert torch.equal(g, r), f"{name} exit {s} b={b}: {what} differs"
    # and once more after the smaller call, at full size, through the binding
    s = blob.n_stages - 1
    got = outputs(torch, b_max)
    eng.exit_head_static(s, acts[s], 0.5, *got)
    ref = eng.exit_head(s, acts[s], 0.5)
    torch.cuda.synchronize()
    for g, r in zip(got, ref):
        assert torch.equal(g, r)
    eng.close()


def test_static_scratch_head_rejects_what_does_not_fit():
    import torch
    import paper_2209_13443_amd as ee
    lib = ee.raw()
    blob = W.load_net("resnet50_small_i8")
    c, n_cls = int(blob.exits[-1]["c"]), int(blob.exits[-1]["n_cls"])
    per_slot = 4 * (c + n_cls)
    b_big = 4 * 1024 * 1024 // per_slot + 8
    if b_big > 1024:
        pytest.skip("this head fits the array at every batch size the library takes")
    eng = ee.Engine(blob, b_big)
    s = blob.n_stages - 1
    shape = (b_big,) + tuple(blob.stage_out_shape(s))
    a = torch.zeros(shape, dtype=torch.int8, device="cuda")
    got = outputs(torch, b_big)
    rc = lib.ee_exit_head_static(eng._h, s, b_big, C.c_void_p(a.data_ptr()), C.c_float(0.5), C.c_void_p(got[0].data_ptr()),
                                 C.c_void_p(got[1].data_ptr()), C.c_void_p(got[2].data_ptr()), C.c_void_p(got[3].data_ptr()))
    assert rc == ee.EE_ERR_OVERFLOW if hasattr(ee, "EE_ERR_OVERFLOW") else rc == -5
    torch.cuda.synchronize()
    assert int(got[0][0]) == -7                               # nothing was launched
    eng.close()
