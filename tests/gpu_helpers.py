"""Plumbing for the GPU parity tests: move a seeded Batch to the device, call
the library through its C ABI (via the ctypes binding), bring results back as
float64, and compare with the oracle at the stated tolerances."""
import numpy as np
import torch

from helpers import fresh_pools, oracle_append, oracle_attn, rel_fro
from paper_2603_10342_amd import binding as B
from paper_2603_10342_amd import inputs as I

DEV = "cuda"

# Tolerances: the stated bf16 gate (max-abs 2e-2, mean-abs 2e-3) plus stricter relative gates that make it meaningful
# on inputs whose outputs are much smaller than the absolute bound.
BF16_MAX_ABS, BF16_MEAN_ABS, BF16_REL_FRO = 2e-2, 2e-3, 1e-2
F32_MAX_ABS, F32_REL_FRO = 1e-5, 1e-5


def to_dev(a: np.ndarray, dtype: int) -> torch.Tensor:
    """Stored numpy array (float32, or uint16 bf16 bits) -> device tensor of the storage dtype."""
    if dtype == I.F32:
        return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).to(DEV).view(torch.bfloat16)


def to_host_raw(t: torch.Tensor, dtype: int) -> np.ndarray:
    """Device tensor -> numpy in the stored representation (float32 / uint16 bits)."""
    if dtype == I.F32:
        return t.detach().cpu().numpy()
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def to_f64(t: torch.Tensor, dtype: int) -> np.ndarray:
    return I.stored_to_f64(to_host_raw(t, dtype), dtype)


def i32(a) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(DEV)


def make_cache(geom, poison=True) -> B.KVCache:
    return B.KVCache(geom.num_pages, geom.page_size, geom.num_kv_heads, geom.head_dim, geom.dtype, DEV,
                     fill=float("nan") if poison else 0.0)


class DevBatch:
    def __init__(self, b: I.Batch):
        g = b.geom
        self.b, self.geom = b, g
        self.q = to_dev(b.q, g.dtype)
        self.k_new = to_dev(b.k_new, g.dtype)
        self.v_new = to_dev(b.v_new, g.dtype)
        self.bt = i32(b.block_tables)
        self.prefix = i32(b.prefix_lens)
        self.new = i32(b.new_lens)
        self.cu = i32(b.cu_new)
        self.ctx = i32(b.ctx_lens)
        self.total = b.total_new
        self.max_new = int(b.new_lens.max()) if b.batch else 0
        self.max_ctx = int(b.ctx_lens.max()) if b.batch else 0
        self.out = torch.full_like(self.q, float("nan"))


def gpu_append(cache, d: DevBatch, validate=True):
    if validate:
        B.ag_debug_validate(cache, d.bt, d.prefix, d.new, d.cu)
    B.ag_kv_append(cache, d.k_new, d.v_new, d.bt, d.prefix, d.new, d.cu, d.total)


def gpu_prefill(cache, d: DevBatch, scale=None):
    B.ag_attn_prefill(cache, d.q, d.out, d.bt, d.new, d.cu, d.total, d.max_new, d.geom.num_q_heads,
                      d.geom.scale if scale is None else scale)
    torch.cuda.synchronize()
    return to_f64(d.out, d.geom.dtype)


def gpu_resume(cache, d: DevBatch, scale=None):
    B.ag_attn_resume(cache, d.q, d.out, d.bt, d.prefix, d.new, d.cu, d.total, d.max_new, d.max_ctx,
                     d.geom.num_q_heads, d.geom.scale if scale is None else scale)
    torch.cuda.synchronize()
    return to_f64(d.out, d.geom.dtype)


def gpu_decode(cache, q: torch.Tensor, bt: torch.Tensor, ctx: torch.Tensor, max_ctx: int, geom, scale=None):
    nbytes = B.ag_attn_decode_workspace_bytes(q.shape[0], geom.num_q_heads, geom.head_dim, max_ctx)
    ws = torch.empty(max(nbytes, 16) // 4, dtype=torch.float32, device=DEV)
    out = torch.full_like(q, float("nan"))
    B.ag_attn_decode(cache, q, out, bt, ctx, max_ctx, geom.num_q_heads, geom.scale if scale is None else scale, ws)
    torch.cuda.synchronize()
    return to_f64(out, geom.dtype)


def pools_match(cache, kp: np.ndarray, vp: np.ndarray, dtype: int):
    """Bit-exact comparison of the device pools with the oracle's host pools (V viewed token-major)."""
    raw = np.uint32 if dtype == I.F32 else np.uint16
    gk = to_host_raw(cache.k_pool_token_major().contiguous(), dtype)
    gv = to_host_raw(cache.v_pool_token_major().contiguous(), dtype)
    np.testing.assert_array_equal(gk.view(raw), kp.view(raw))
    np.testing.assert_array_equal(gv.view(raw), vp.view(raw))


def check_close(got: np.ndarray, ref: np.ndarray, dtype: int, what: str = ""):
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    assert np.isfinite(got).all(), f"{what}: non-finite values in the GPU output"
    err = np.abs(got - ref)
    rf = rel_fro(got, ref)
    if dtype == I.BF16:
        assert err.max() <= BF16_MAX_ABS, f"{what}: max-abs {err.max():.3e}"
        assert err.mean() <= BF16_MEAN_ABS, f"{what}: mean-abs {err.mean():.3e}"
        assert rf <= BF16_REL_FRO, f"{what}: relative Frobenius error {rf:.3e}"
        rows = ref.reshape(-1, ref.shape[-1])
        erow = err.reshape(rows.shape).max(axis=1)
        bound = 2.0 ** -7 * np.abs(rows).max(axis=1) + 1e-6
        worst = int(np.argmax(erow - bound))
        assert (erow <= bound).all(), f"{what}: row {worst} err {erow[worst]:.3e} > bound {bound[worst]:.3e}"
    else:
        assert err.max() <= F32_MAX_ABS, f"{what}: max-abs {err.max():.3e}"
        assert rf <= F32_REL_FRO, f"{what}: relative Frobenius error {rf:.3e}"
    return float(err.max()), rf


def run_phase(cache, kp, vp, b: I.Batch, kind: str, scale=None):
    """Append + attend on both sides; returns (gpu_f64, oracle_f64).  kind: cold | resume | decode."""
    d = DevBatch(b)
    gpu_append(cache, d)
    oracle_append(kp, vp, b)
    ref = oracle_attn(kp, vp, b, scale=scale)
    if kind == "cold":
        got = gpu_prefill(cache, d, scale)
    elif kind == "resume":
        got = gpu_resume(cache, d, scale)
    else:
        got = gpu_decode(cache, d.q, d.bt, d.ctx, d.max_ctx, d.geom, scale)
    return got, ref


def gpu_merged(cache, d: DevBatch, scale=None):
    nbytes = B.ag_attn_merged_workspace_bytes(d.total, d.geom.num_q_heads, d.max_ctx)
    ws = torch.full((max(nbytes, 16) // 4,), float("nan"), dtype=torch.float32, device=DEV)
    B.ag_attn_merged(cache, d.q, d.out, d.bt, d.prefix, d.new, d.cu, d.total, d.max_new, d.max_ctx,
                     d.geom.num_q_heads, d.geom.scale if scale is None else scale, ws)
    torch.cuda.synchronize()
    return to_f64(d.out, d.geom.dtype)
