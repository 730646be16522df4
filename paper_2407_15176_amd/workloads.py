"""Seeded synthetic inputs for the five benchmark configurations.

This module only draws random tensors (shapes, value distributions, planted
needles).  It holds none of the method's arithmetic and imports neither the HIP
binding nor the CPU oracle, so both sides can be fed the same stored bytes.

Recipe (stands in for Llama-3.1-8B / Llama-3.2-3B layer shapes and for
needle-in-a-haystack caches of 128K..4M tokens; no real model data is used):
  * q, K, V iid N(0,1); seed = 240715000 + 10*cfg + tensor_id with
    tensor_id 0=q, 1=K, 2=V, 3=channel scales, 4=needle positions.
  * configs 2,3,5: K and V of KV head h are multiplied per channel c by
    sigma[h,c] = exp(U(ln 0.5, ln 4)) (outlier channels; the exponential is evaluated with
    correctly rounded elementwise operations only, so that CPU-generated inputs are the same
    bytes on every machine); q is left unscaled.
    config 4: q is scaled too (a query head uses its KV head's sigma).
  * needles (8/32/32/0/64): distinct seeded positions in the middle of the cache,
    shared by all KV heads; K[h,pos,:] = 3*||sigma_h||_2 * qbar_h/||qbar_h||_2
    with qbar_h the sum of the group's stored query rows; V is untouched.
  * everything is cast to the storage dtype once; those bytes are the input.
Layouts: q [M,Hq,D], K and V [Hkv,N,D], contiguous.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import torch

SEED_BASE = 240715000


@dataclass(frozen=True)
class Workload:
    name: str
    cfg: int                 # seed family (1..5)
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    dtype: str               # "f32" | "bf16" | "f16"
    n_ctx: int               # N, current tokens included as the last n_query rows
    n_query: int             # M
    n_sink: int
    n_local: int
    top_k: int
    rope_theta: float
    max_position: int
    channel_scales: bool
    scale_q: bool
    n_needles: int

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def n_sink_eff(self) -> int:
        return min(self.n_sink, self.n_ctx)

    @property
    def n_local_eff(self) -> int:
        return min(self.n_local, self.n_ctx - self.n_sink_eff)

    @property
    def n_mid(self) -> int:
        return self.n_ctx - self.n_sink_eff - self.n_local_eff

    @property
    def k_eff(self) -> int:
        return max(0, min(self.top_k, self.n_mid))

    @property
    def scope(self) -> int:
        """S: sink + selected + local entries attended to."""
        return self.n_sink_eff + self.k_eff + self.n_local_eff

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2

    @property
    def scan_bytes(self) -> int:
        """Algorithmic bytes of the stage-1 key scan (K rows of the middle only)."""
        return self.n_mid * self.n_kv_heads * self.head_dim * self.elem_bytes

    @property
    def score_flops(self) -> int:
        return 2 * self.n_query * self.n_q_heads * self.n_mid * self.head_dim

    def torch_dtype(self):
        return {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}[self.dtype]

    def scaled(self, **kw) -> "Workload":
        """Same recipe at other sizes (parity cases the oracle finishes in seconds)."""
        return replace(self, **kw)


CONFIGS = {
    1: Workload("cfg1_decode_16k_f32", 1, 8, 2, 64, "f32", 16_384, 1, 4, 512, 256,
                10000.0, 772, False, False, 8),
    2: Workload("cfg2_decode_128k_bf16", 2, 32, 8, 128, "bf16", 131_072, 1, 4, 4096, 4096,
                500000.0, 131_072, True, False, 32),
    3: Workload("cfg3_decode_1m_bf16", 3, 32, 8, 128, "bf16", 1_048_576, 1, 4, 4096, 8192,
                500000.0, 131_072, True, False, 32),
    4: Workload("cfg4_prefill_4k_x_256k_bf16", 4, 32, 8, 128, "bf16", 262_144, 4096, 4, 4096, 4096,
                500000.0, 131_072, True, True, 0),
    5: Workload("cfg5_decode_4m_bf16", 5, 24, 8, 128, "bf16", 4_194_304, 1, 4, 4096, 8192,
                500000.0, 131_072, True, False, 64),
}


def _gen(device, cfg: int, tensor_id: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(SEED_BASE + 10 * cfg + tensor_id)
    return g


def channel_sigma(w: Workload) -> torch.Tensor:
    """sigma [Hkv, D] float32 on the CPU (ones when the config has no scales)."""
    if not w.channel_scales:
        return torch.ones(w.n_kv_heads, w.head_dim)
    u = torch.rand(w.n_kv_heads, w.head_dim, generator=_gen("cpu", w.cfg, 3)).double()
    return _exp_portable(_LN_HALF + (_LN_4 - _LN_HALF) * u).float()


_LN_HALF, _LN_4, _LN_2 = -0.6931471805599453, 1.3862943611198906, 0.6931471805599453


def _exp_portable(x: torch.Tensor) -> torch.Tensor:
    """exp(x) for float64 x of moderate size from correctly rounded elementwise operations only
    (round, multiply, add, power-of-two scaling): a library exp differs in the last bit between
    machines, and inputs that stored expected values were computed from must be the same bytes
    everywhere.  Accurate to a few ulp, which is all a random scale needs."""
    n = torch.round(x / _LN_2)
    r = x - n * _LN_2                       # |r| <= 0.35
    acc = torch.ones_like(r)
    for i in range(20, 0, -1):              # Horner form of the Taylor series, degree 20
        acc = acc * r / float(i) + 1.0
    return torch.ldexp(acc, n.to(torch.int32))


def needle_positions(w: Workload) -> torch.Tensor:
    """Distinct absolute positions inside the middle, int64 on the CPU, ascending."""
    n = min(w.n_needles, max(w.n_mid, 0))
    if n == 0:
        return torch.empty(0, dtype=torch.int64)
    perm = torch.randperm(w.n_mid, generator=_gen("cpu", w.cfg, 4))[:n]
    return torch.sort(perm + w.n_sink_eff).values


def generate(w: Workload, device="cpu") -> dict:
    """Returns {"q","k","v"} in the storage dtype on `device`, plus "sigma" and "needles" (CPU)."""
    device = torch.device(device)
    dt = w.torch_dtype()
    Hq, Hkv, D, N, M, G = w.n_q_heads, w.n_kv_heads, w.head_dim, w.n_ctx, w.n_query, w.group
    sigma = channel_sigma(w)
    sig_dev = sigma.to(device)

    q32 = torch.randn(M, Hq, D, generator=_gen(device, w.cfg, 0), device=device)
    if w.scale_q:
        q32 = q32 * sig_dev.repeat_interleave(G, dim=0).unsqueeze(0)
    q = q32.to(dt)

    k = torch.empty(Hkv, N, D, dtype=dt, device=device)
    v = torch.empty(Hkv, N, D, dtype=dt, device=device)
    gk, gv = _gen(device, w.cfg, 1), _gen(device, w.cfg, 2)
    for h in range(Hkv):  # one head at a time bounds the fp32 staging memory
        k[h] = (torch.randn(N, D, generator=gk, device=device) * sig_dev[h]).to(dt)
        v[h] = (torch.randn(N, D, generator=gv, device=device) * sig_dev[h]).to(dt)

    pos = needle_positions(w)
    if pos.numel() and M == 1:
        qbar = q[0].float().reshape(Hkv, G, D).sum(dim=1)                       # [Hkv, D]
        direction = qbar / qbar.norm(dim=1, keepdim=True)
        needle = 3.0 * sig_dev.norm(dim=1, keepdim=True) * direction           # [Hkv, D]
        k[:, pos.to(device), :] = needle.to(dt).unsqueeze(1)
    return {"q": q, "k": k, "v": v, "sigma": sigma, "needles": pos}


def to_numpy_store(t: torch.Tensor):
    """Exact stored bytes as numpy: float32 as is, bfloat16 and float16 as uint16 bit patterns."""
    t = t.detach().contiguous().cpu()
    if t.dtype in (torch.bfloat16, torch.float16):
        return t.view(torch.int16).numpy().view("uint16")
    return t.numpy()
