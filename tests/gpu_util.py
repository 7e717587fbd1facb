"""Helpers for the GPU parity tests: move seeded cases to the device and call the C ABI binding."""
import numpy as np
import torch

from paper_2601_22438_amd import kvflow

MAX_ABS = 2e-2      # decode tolerance against the fp64 oracle (bf16 inputs, fp32 accumulation)
MEAN_ABS = 2e-3


def bf16_tensor(bits: np.ndarray) -> torch.Tensor:
    """uint16 bit patterns -> bfloat16 CUDA tensor of the same shape."""
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)


def bits_of(t: torch.Tensor) -> np.ndarray:
    """bfloat16 tensor -> uint16 bit patterns on the host."""
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def pool_tensor(bits, k_scale=1.0, v_scale=1.0):
    """Pool bit patterns -> what the binding takes: a bf16 tensor, or an Fp8Pool for uint8 patterns."""
    if bits.dtype == np.uint8:
        return kvflow.Fp8Pool(torch.from_numpy(np.ascontiguousarray(bits)).cuda(), k_scale, v_scale)
    return bf16_tensor(bits)


def pool_bits_of(pool) -> np.ndarray:
    if isinstance(pool, kvflow.Fp8Pool):
        return pool.data.cpu().numpy()
    return bits_of(pool)


class DeviceCase:
    def __init__(self, case, pool_bits=None, k_scale=1.0, v_scale=1.0):
        self.case = case
        g = case.geom
        self.q = bf16_tensor(case.q)
        pool_bits = case.pool if pool_bits is None else pool_bits
        if torch.is_tensor(pool_bits) or isinstance(pool_bits, kvflow.Fp8Pool):
            self.pool = pool_bits
        else:
            self.pool = pool_tensor(pool_bits, k_scale, v_scale)
        self.block_table = torch.from_numpy(case.block_table).cuda()
        self.context_lens = torch.from_numpy(case.context_lens).cuda()
        self.max_len = case.max_context_len
        self.scale = float(g.scale)

    def decode(self, out_dtype=torch.float32, workgroups=0, max_len=None, block_table=None, pool=None):
        c, g = self.case, self.case.geom
        max_len = self.max_len if max_len is None else max_len
        out = torch.full((c.batch, g.num_q_heads, g.head_dim), float("nan"), dtype=out_dtype, device="cuda")
        nbytes = kvflow.kv_decode_workspace_bytes(c.batch, g.num_q_heads, g.num_kv_heads, g.head_dim,
                                                  max_len, workgroups)
        assert nbytes > 0
        # workspace contents on entry must not matter: fill it with NaN
        ws = torch.full((nbytes // 4,), float("nan"), dtype=torch.float32, device="cuda")
        kvflow.kv_decode_attn(out, self.q, self.pool if pool is None else pool,
                              self.block_table if block_table is None else block_table,
                              self.context_lens, max_len, self.scale, workgroups, ws)
        torch.cuda.synchronize()
        return out


def assert_close_to_oracle(got: torch.Tensor, want: np.ndarray, what=""):
    got64 = got.detach().to(torch.float64).cpu().numpy().reshape(want.shape)
    assert np.isfinite(got64).all(), f"{what}: non-finite output"
    err = np.abs(got64 - want)
    assert err.max() <= MAX_ABS, f"{what}: max-abs {err.max():.3e} > {MAX_ABS}"
    assert err.mean() <= MEAN_ABS, f"{what}: mean-abs {err.mean():.3e} > {MEAN_ABS}"
    return err.max(), err.mean()
