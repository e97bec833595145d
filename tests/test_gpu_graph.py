"""The entry points only enqueue kernels (no allocation, no synchronisation, no memset), so a caller can record
a decode step - append, then attention - into a HIP graph and replay it.  Every replay is checked against
the eager result, with eager work and synchronisations between the replays."""
import numpy as np
import pytest
import torch

from gpu_helpers import DevBatch, check_close, gpu_append, make_cache, to_f64
from helpers import fresh_pools, oracle_append
from oracle import oracle as O
from paper_2603_10342_amd import binding as B
from paper_2603_10342_amd import inputs as I

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("entry", ["decode", "merged"])
def test_decode_step_recorded_in_a_graph_replays_to_the_eager_result(entry):
    g = I.Geometry(8, 2, 128, 16, 1024, I.BF16)
    c = I.make_decode(batch=6, lo=200, hi=2500, num_pages=1024, geom=g, seed=55, sigma_qk=1.0, sigma_v=1.0)
    cache = make_cache(g)
    kp, vp = fresh_pools(g)
    fill, step = DevBatch(c.fill), DevBatch(c.step)
    gpu_append(cache, fill)
    for b in (c.fill, c.step):
        oracle_append(kp, vp, b)
    ref = O.decode(kp, vp, g.dtype, c.step.q, c.block_tables, c.ctx_lens, g.num_q_heads, g.scale)
    if entry == "decode":
        nbytes = B.ag_attn_decode_workspace_bytes(6, g.num_q_heads, 128, step.max_ctx)
    else:
        nbytes = B.ag_attn_merged_workspace_bytes(step.total, g.num_q_heads, step.max_ctx)
    ws = torch.empty(nbytes // 4, dtype=torch.float32, device="cuda")
    out = torch.zeros_like(step.q)

    def one_step(stream):
        B.ag_kv_append(cache, step.k_new, step.v_new, step.bt, step.prefix, step.new, step.cu, step.total, stream=stream)
        if entry == "decode":
            B.ag_attn_decode(cache, step.q, out, step.bt, step.ctx, step.max_ctx, g.num_q_heads, g.scale, ws, stream=stream)
        else:
            B.ag_attn_merged(cache, step.q, out, step.bt, step.prefix, step.new, step.cu, step.total, step.max_new,
                             step.max_ctx, g.num_q_heads, g.scale, ws, stream=stream)

    one_step(None)
    torch.cuda.synchronize()
    eager = out.clone()
    check_close(to_f64(eager, g.dtype), ref, g.dtype, "eager")

    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(graph, stream=side):
        one_step(torch.cuda.current_stream())
    torch.cuda.synchronize()
    for r in range(4):
        out.fill_(float("nan"))                      # eager work between replays
        ws.uniform_()                                # the workspace holds nothing a replay relies on
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int16), eager.view(torch.int16)), f"replay {r}"
