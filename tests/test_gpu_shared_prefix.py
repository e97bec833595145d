"""Sessions that share the physical pages of a common prefix (agents started from one system prompt read the
same cached pages; only what follows the prompt is their own), a non-default scale, and a 65k-token context."""
import numpy as np
import pytest
import torch

from gpu_helpers import (DevBatch, check_close, gpu_append, gpu_decode, gpu_merged, gpu_resume, make_cache, to_f64)
from helpers import fresh_pools, make_batch, oracle_append, oracle_attn
from oracle import oracle as O
from paper_2603_10342_amd import inputs as I

pytestmark = pytest.mark.gpu


def test_sessions_sharing_the_pages_of_a_system_prompt():
    g = I.Geometry(8, 2, 128, 16, 512, I.BF16)
    prompt = 1024                                     # a multiple of the page size: the shared part ends on a page
    n_sess = 4
    own = [37, 200, 1, 90]                            # each session's own tokens after the prompt
    # one row of pages for the prompt, shared by all; private pages behind it
    bt_prompt = I.deal_block_tables(I.rng_for(88, 0), [prompt], 16, 64)          # pages 0..63 in some order
    priv = I.deal_block_tables(I.rng_for(88, 1), [n + 1 for n in own], 16, 256) + 64   # private pages start at 64
    width = prompt // 16 + priv.shape[1]
    bt = np.zeros((n_sess, width), np.int32)
    for s in range(n_sess):
        bt[s, :prompt // 16] = bt_prompt[0, :prompt // 16]
        bt[s, prompt // 16:] = priv[s]
    cache = make_cache(g)
    kp, vp = fresh_pools(g)
    # the prompt is written once, through session 0's table
    fill = make_batch(g, [0], [prompt], seed=88, bt=np.ascontiguousarray(bt[:1]), sigma_qk=1.0, sigma_v=1.0)
    gpu_append(cache, DevBatch(fill))
    oracle_append(kp, vp, fill)
    # every session appends its own chunk behind the shared prompt and attends
    chunk = make_batch(g, [prompt] * n_sess, own, seed=88, bt=bt, stream=2, sigma_qk=1.0, sigma_v=1.0)
    d = DevBatch(chunk)
    gpu_append(cache, d)
    oracle_append(kp, vp, chunk)
    ref = oracle_attn(kp, vp, chunk)
    check_close(gpu_resume(cache, d), ref, g.dtype, "resume over a shared prompt")
    check_close(gpu_merged(cache, d), ref, g.dtype, "merged over a shared prompt")
    # one decode token each
    ctx = [prompt + n for n in own]
    step = make_batch(g, ctx, [1] * n_sess, seed=88, bt=bt, stream=3, sigma_qk=1.0, sigma_v=1.0)
    ds = DevBatch(step)
    gpu_append(cache, ds)
    oracle_append(kp, vp, step)
    refd = O.decode(kp, vp, g.dtype, step.q, bt, step.ctx_lens, g.num_q_heads, g.scale)
    check_close(gpu_decode(cache, ds.q, ds.bt, ds.ctx, ds.max_ctx, g), refd, g.dtype, "decode over a shared prompt")


@pytest.mark.parametrize("scale", [0.02, 0.5])
def test_non_default_scale(scale):
    g = I.Geometry(8, 2, 128, 16, 256, I.BF16)
    bt = I.deal_block_tables(I.rng_for(5, 0), [700, 300], 16, g.num_pages)
    fill = make_batch(g, [0, 0], [600, 250], seed=5, bt=bt, sigma_qk=0.5, sigma_v=1.0)
    chunk = make_batch(g, [600, 250], [70, 9], seed=5, bt=bt, stream=2, sigma_qk=0.5, sigma_v=1.0)
    cache = make_cache(g)
    kp, vp = fresh_pools(g)
    for b in (fill, chunk):
        gpu_append(cache, DevBatch(b))
        oracle_append(kp, vp, b)
    d = DevBatch(chunk)
    ref = oracle_attn(kp, vp, chunk, scale=scale)
    check_close(gpu_resume(cache, d, scale), ref, g.dtype, f"resume, scale {scale}")
    check_close(gpu_merged(cache, d, scale), ref, g.dtype, f"merged, scale {scale}")


def test_very_long_context_decode_and_merged():
    g = I.Geometry(8, 2, 128, 16, 4200, I.BF16)
    L = 65000
    bt = I.deal_block_tables(I.rng_for(9, 0), [L + 8], 16, g.num_pages)
    fill = make_batch(g, [0], [L], seed=9, bt=bt)                 # the configs' own distribution: flat logits
    chunk = make_batch(g, [L], [5], seed=9, bt=bt, stream=2)
    cache = make_cache(g)
    kp, vp = fresh_pools(g)
    for b in (fill, chunk):
        gpu_append(cache, DevBatch(b), validate=False)
        oracle_append(kp, vp, b)
    d = DevBatch(chunk)
    ref = oracle_attn(kp, vp, chunk)
    check_close(gpu_merged(cache, d), ref, g.dtype, "merged at 65k")
    check_close(gpu_resume(cache, d), ref, g.dtype, "resume at 65k")
    # the chunk's last row is a decode at context L + 5
    q_last = d.q[-1:].contiguous()
    ctx = torch.tensor([L + 5], dtype=torch.int32, device="cuda")
    check_close(gpu_decode(cache, q_last, d.bt, ctx, L + 5, g), ref[-1:], g.dtype, "decode at 65k")
