"""The layer in r chunks (FSMoE Sec. 4.2) through the C ABI: every output and every saved tensor must be
bit-identical to the unchunked layer (which the other GPU tests hold against the oracle)."""
import numpy as np
import pytest
import torch

import moe_synth as S
import paper_2501_10714_amd as moe
from moe_harness import Buffers, dev_inputs, make_cfg, run_layer
from test_gpu_parity import CASES

pytestmark = pytest.mark.gpu

NAMES = ["tiny_full", "f32_ragged", "gpt2_small", "mixtral_small", "fine_small", "switch_small", "erf_odd",
         "k32_pipeline", "sigmoid_glu", "expert_choice_glu"]


def same_bits(a, b):
    return torch.equal(a.contiguous().view(torch.uint8), b.contiguous().view(torch.uint8))


@pytest.mark.parametrize("name", NAMES)
@pytest.mark.parametrize("r,two_streams", [(2, False), (3, True), (16, True)])
def test_chunked_layer_is_bit_identical(name, r, two_streams):
    w = CASES[name]
    d = S.draw_all(w)
    dd = dev_inputs(d)
    cfg, ref = run_layer(w, d, dd=dd)
    b = Buffers(w, cfg)
    # poison what the chunked calls must fill, so that a row they skip shows
    b.saved.fill_(0x7B); b.y.fill_(1); b.dx.fill_(1); b.dw1.fill_(1); b.dw2.fill_(1); b.dw_gate.fill_(1)
    if b.dw3 is not None:
        b.dw3.fill_(1)
    aux = torch.cuda.Stream() if two_streams else None
    moe.moe_layer_fwd_chunked(cfg, dd["x"], dd["w_gate"], dd["b_gate"], dd["w1"], dd["w3"], dd["w2"], b.y, b.saved, b.ws,
                              r, aux)
    moe.moe_layer_bwd_chunked(cfg, dd["dy"], dd["x"], dd["w_gate"], dd["w1"], dd["w3"], dd["w2"], b.saved, b.dx,
                              b.dw_gate, b.db_gate if d["b_gate"] is not None else None, b.dw1, b.dw3, b.dw2, b.ws, r)
    torch.cuda.synchronize()
    A = int(moe.saved_view(cfg, ref.saved, "offsets", torch.int32)[-1])
    el = torch.bfloat16 if w.dtype == S.DT_BF16 else torch.float32
    for nm, dt in [("logits", torch.float32), ("probs", torch.float32), ("topk_idx", torch.int32),
                   ("topk_w", torch.float32), ("pos", torch.int32), ("row_of", torch.int32), ("count", torch.int32),
                   ("offsets", torch.int32)]:
        assert same_bits(moe.saved_view(cfg, b.saved, nm, dt), moe.saved_view(cfg, ref.saved, nm, dt)), nm
    assert same_bits(moe.saved_view(cfg, b.saved, "src_of_row", torch.int32)[:A],
                     moe.saved_view(cfg, ref.saved, "src_of_row", torch.int32)[:A])
    for nm, cols in [("xe", w.M), ("q", w.M), ("a1", w.H), ("hh", w.H)] + ([("a3", w.H)] if w.gated else []):
        got = moe.saved_view(cfg, b.saved, nm, el).view(-1, cols)[:A]
        want = moe.saved_view(cfg, ref.saved, nm, el).view(-1, cols)[:A]
        assert same_bits(got, want), nm
    outs = ["y", "dx", "dw_gate", "dw1", "dw2"] + (["dw3"] if w.gated else []) + (["db_gate"] if d["b_gate"] is not None else [])
    for nm in outs:
        assert same_bits(getattr(b, nm), getattr(ref, nm)), nm


def test_chunk_count_is_validated():
    w = CASES["tiny_full"]
    d = S.draw_all(w)
    dd = dev_inputs(d)
    cfg = make_cfg(w)
    b = Buffers(w, cfg)
    for r in (0, -1, moe.MAX_CHUNKS + 1):
        with pytest.raises(moe.MoeError):
            moe.moe_layer_fwd_chunked(cfg, dd["x"], dd["w_gate"], dd["b_gate"], dd["w1"], dd["w3"], dd["w2"], b.y, b.saved,
                                      b.ws, r)
