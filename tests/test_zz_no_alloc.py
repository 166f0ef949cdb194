"""moe_route_static, the gate for callers that cannot allocate: called through the C ABI (raw ctypes), it must give
what moe_route gives on the same inputs, bit for bit in every output, on two calls in a row, the second on a smaller
problem (the built-in scratch array keeps the first call's contents), and it must refuse shapes whose scratch does
not fit in the array."""
import ctypes as C

import numpy as np
import pytest
import torch

import moe_synth as S
import paper_2501_10714_amd as moe
from moe_harness import Buffers, dev_inputs, make_cfg

pytestmark = pytest.mark.gpu

OUTS = ("logits", "probs", "topk_idx", "topk_w", "pos", "row_of", "count", "offsets", "src_of_row")


def ptr(t):
    return C.c_void_p(0 if t is None else t.data_ptr())


def route_both(w):
    """(outputs of moe_route, outputs of moe_route_static) for workload w, both through raw ctypes."""
    lib = moe.load()
    d = S.draw_all(w)
    cfg = make_cfg(w)
    dd = dev_inputs(d)
    stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    res = []
    for static in (False, True):
        b = Buffers(w, cfg)
        for n in OUTS:                       # poison, so that an output the call does not write shows
            getattr(b, n).fill_(-7)
        args = [C.byref(cfg), ptr(dd["x"]), ptr(dd["w_gate"]), ptr(dd["b_gate"])] + [ptr(getattr(b, n)) for n in OUTS]
        if static:
            st = lib.moe_route_static(*args, stream)
        else:
            st = lib.moe_route(*args, ptr(b.ws), C.c_size_t(b.ws.numel()), stream)
        assert st == 0, moe.moe_last_error()
        torch.cuda.synchronize()
        res.append({n: getattr(b, n).cpu().numpy().copy() for n in OUTS})
    return res


def assert_same(a, b):
    for n in OUTS:
        assert np.array_equal(a[n].view(np.int32), b[n].view(np.int32)), n   # bit patterns, floats included


def test_two_calls_in_a_row_the_second_smaller():
    big = S.scaled(S.WORKLOADS["finegrained"], N=3000, M=256, H=64, E=64, k=6, seed=51)      # drops, bias, 47 token tiles
    small = S.scaled(S.WORKLOADS["mixtral"], N=700, M=192, H=64, E=8, k=2, seed=52)           # fewer tiles, fewer experts
    wide = S.scaled(S.WORKLOADS["gpt2"], N=200, M=9216, H=64, E=12, k=2, f=None, seed=53)     # the kernel that uses the fp64 W_g copy
    ec = S.scaled(S.WORKLOADS["mixtral"], N=500, M=128, H=64, E=8, k=8, f=0.25, renormalize=3, seed=54)  # expert choice
    for w in (big, small, wide, small, ec):
        ref, got = route_both(w)
        assert_same(ref, got)


def test_shapes_beyond_the_scratch_are_refused():
    lib = moe.load()
    # 4 * E * k * ceil(N / 64) bytes of histogram alone exceed 4 MiB
    cfg = moe.MoeConfig.make(1 << 20, 64, 64, 64, 8, 0, moe.DT_BF16, moe.ACT_RELU)
    fake = C.c_void_p(4096)
    st = lib.moe_route_static(C.byref(cfg), *([fake] * 12), C.c_void_p(0))
    assert st == 3 and "scratch" in moe.moe_last_error()
