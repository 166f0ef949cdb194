"""The layer calls can be captured into a HIP graph (they allocate nothing, never synchronise and record no
memset): a graph of moe_layer_fwd + moe_layer_bwd is replayed several times on changing inputs, with eager work
and synchronisations between the replays, and every replay must equal the eager result bit for bit."""
import pytest
import torch

import moe_synth as S
import paper_2501_10714_amd as moe
from moe_harness import Buffers, dev_inputs, make_cfg
from test_gpu_parity import CASES

pytestmark = pytest.mark.gpu


def same_bits(a, b):
    return torch.equal(a.contiguous().view(torch.uint8), b.contiguous().view(torch.uint8))


def step(cfg, dd, b, has_bias, chunks=0, aux=None):
    if chunks:
        moe.moe_layer_fwd_chunked(cfg, dd["x"], dd["w_gate"], dd["b_gate"], dd["w1"], dd["w3"], dd["w2"], b.y, b.saved, b.ws,
                                  chunks, aux)
        moe.moe_layer_bwd_chunked(cfg, dd["dy"], dd["x"], dd["w_gate"], dd["w1"], dd["w3"], dd["w2"], b.saved, b.dx,
                                  b.dw_gate, b.db_gate if has_bias else None, b.dw1, b.dw3, b.dw2, b.ws, chunks)
    else:
        moe.moe_layer_fwd(cfg, dd["x"], dd["w_gate"], dd["b_gate"], dd["w1"], dd["w3"], dd["w2"], b.y, b.saved, b.ws)
        moe.moe_layer_bwd(cfg, dd["dy"], dd["x"], dd["w_gate"], dd["w1"], dd["w3"], dd["w2"], b.saved, b.dx, b.dw_gate,
                          b.db_gate if has_bias else None, b.dw1, b.dw3, b.dw2, b.ws)


@pytest.mark.parametrize("name,chunks", [("gpt2_small", 0), ("mixtral_small", 0), ("switch_small", 0), ("expert_choice_glu", 0),
                                         ("mixtral_small", 2)])
def test_graph_replays_equal_eager(name, chunks):
    w = CASES[name]
    d = S.draw_all(w)
    dd = dev_inputs(d)                       # the graph's static input buffers
    cfg = make_cfg(w)
    has_bias = d["b_gate"] is not None
    g_buf, e_buf = Buffers(w, cfg), Buffers(w, cfg)
    aux = torch.cuda.Stream() if chunks else None
    step(cfg, dd, g_buf, has_bias, chunks, aux)    # first calls set kernel attributes: not inside a capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step(cfg, dd, g_buf, has_bias, chunks, torch.cuda.current_stream() if chunks else None)
    names = ["y", "dx", "dw1", "dw2", "dw_gate"] + (["dw3"] if w.gated else []) + (["db_gate"] if has_bias else [])
    for rep in range(4):
        # new tokens and upstream gradients every time: the routing changes from replay to replay
        w_rep = S.scaled(w, seed=w.seed + 100 * (rep + 1))
        dd["x"].copy_(dev_inputs({"x": S.draw_x(w_rep)})["x"])
        dd["dy"].copy_(dev_inputs({"dy": S.draw_dy(w_rep)})["dy"])
        for n in names:
            getattr(g_buf, n).fill_(1)
        g_buf.saved.fill_(0x3C)
        graph.replay()
        torch.cuda.synchronize()
        step(cfg, dd, e_buf, has_bias, chunks, aux)    # the program's own eager work between replays
        torch.cuda.synchronize()
        for n in names:
            assert same_bits(getattr(g_buf, n), getattr(e_buf, n)), (rep, n)
        for n, dt in (("topk_idx", torch.int32), ("row_of", torch.int32), ("offsets", torch.int32)):
            assert same_bits(moe.saved_view(cfg, g_buf.saved, n, dt), moe.saved_view(cfg, e_buf.saved, n, dt)), (rep, n)
