"""Seeded synthetic inputs for the ProxyKV hot path.

This module only *makes data*: proxy Q/K with planted heavy hitters, a target
KV cache and random-init mapper weights.  It holds none of the method's
arithmetic (no scoring, mapping, selection or compaction) so that both the HIP
library's tests and the CPU oracle's tests can draw the same inputs from it.

The base generator is counter-based and integer-exact: element `i` of tensor
`tensor_id` is (sum of twelve 16-bit fields of three splitmix64 words - 393210)
/ 65536, an Irwin-Hall(12) variate with mean 0 and variance ~1 whose numerator
is below 2^20, hence exact in fp32 on any device.  The same torch integer ops
run on the CPU and on the GPU and give bit-identical tensors.
"""
from __future__ import annotations

import dataclasses
from typing import Dict, Optional, Tuple

import numpy as np
import torch

MASTER_SEED = 20260516
_M64 = (1 << 64) - 1
_GOLDEN = 0x9E3779B97F4A7C15
_MUL1 = 0xBF58476D1CE4E5B9
_MUL2 = 0x94D049BB133111EB

# tensor ids of the generator streams
TID_Q_REC, TID_K_CTX, TID_K_REC, TID_K_T, TID_V_T = 1, 2, 3, 4, 5


def _signed(c: int) -> int:
    c &= _M64
    return c - (1 << 64) if c >= (1 << 63) else c


def _mix_py(z: int) -> int:
    z = (z + _GOLDEN) & _M64
    z = ((z ^ (z >> 30)) * _MUL1) & _M64
    z = ((z ^ (z >> 27)) * _MUL2) & _M64
    return z ^ (z >> 31)


def _lsr(z: torch.Tensor, s: int) -> torch.Tensor:
    """Logical right shift of an int64 tensor holding uint64 bit patterns."""
    return (z >> s) & ((1 << (64 - s)) - 1)


def _mix(z: torch.Tensor) -> torch.Tensor:
    """splitmix64 output function on int64 tensors (arithmetic wraps mod 2^64)."""
    z = z + _signed(_GOLDEN)
    z = (z ^ _lsr(z, 30)) * _signed(_MUL1)
    z = (z ^ _lsr(z, 27)) * _signed(_MUL2)
    return z ^ _lsr(z, 31)


def stream_key(seed: int, tensor_id: int) -> int:
    return _mix_py(((seed * _GOLDEN) + tensor_id) & _M64)


def irwin_hall(seed: int, tensor_id: int, start: int, count: int, device="cpu") -> torch.Tensor:
    """fp32 values of flat elements [start, start+count) of stream (seed, tensor_id)."""
    key = stream_key(seed, tensor_id)
    idx = torch.arange(start, start + count, dtype=torch.int64, device=device)
    total = torch.zeros(count, dtype=torch.int64, device=device)
    for r in range(3):
        ctr = idx * 3 + r
        word = _mix(ctr * _signed(_GOLDEN) + _signed(key))
        for f in range(4):
            total += (word >> (16 * f)) & 0xFFFF
    return (total - 393210).to(torch.float32) / 65536.0


def normal_tensor(shape, seed: int, tensor_id: int, device="cpu", block: int = 1 << 24) -> torch.Tensor:
    """fp32 tensor of `shape` filled from stream (seed, tensor_id), generated in blocks."""
    n = int(np.prod(shape))
    out = torch.empty(n, dtype=torch.float32, device=device)
    for s in range(0, n, block):
        c = min(block, n - s)
        out[s:s + c] = irwin_hall(seed, tensor_id, s, c, device)
    return out.view(*shape)


@dataclasses.dataclass(frozen=True)
class Case:
    """One workload: proxy and target shapes plus the planted structure."""
    name: str
    L_s: int
    H_q: int
    H_kv: int
    d: int
    N: int
    N_q: int
    chunk: int
    L_l: int
    H_l: int
    D: int
    n_planted: int            # heavy-hitter context keys per (layer, KV head)
    plant_scale: float        # planted key = plant_scale * (a random query)
    recency_band: int = 0     # last `recency_band` context keys shifted toward the queries
    band_shift: float = 0.5
    keep_ratios: Tuple[float, ...] = (0.3,)
    fp32_inputs: bool = False  # hand Q/K to the library as fp32 (rounded to bf16 on entry)

    @property
    def G(self) -> int:
        return self.H_q // self.H_kv


# The five workloads: a tiny single-layer case, Llama-3.2-1B -> Llama-3.1-8B shapes at
# 8k and 32k context, Qwen-2.5-0.5B -> 7B shapes at 170k, Qwen-2.5-1.5B -> 32B shapes at 32k.
CASES: Dict[str, Case] = {
    "tiny": Case("tiny", 1, 4, 2, 64, 512, 128, 128, 1, 4, 128, 8, 4.0, fp32_inputs=True),
    "llama_8k": Case("llama_8k", 16, 32, 8, 64, 8192, 8192, 2048, 32, 8, 128, 82, 3.0),
    "llama_32k": Case("llama_32k", 16, 32, 8, 64, 32768, 32768, 2048, 32, 8, 128, 164, 3.0,
                      recency_band=512, keep_ratios=(0.1, 0.3, 0.5)),
    "qwen_170k": Case("qwen_170k", 24, 14, 2, 64, 170000, 170000, 2048, 28, 4, 128, 340, 3.0),
    "qwen32b_32k": Case("qwen32b_32k", 28, 12, 2, 128, 32768, 32768, 4096, 64, 8, 128, 328, 3.0,
                        keep_ratios=(0.1, 0.2, 0.3, 0.5, 0.9)),
}


def scaled_case(base: Case, **overrides) -> Case:
    """A copy of `base` with some fields replaced (reduced sizes for parity tests)."""
    return dataclasses.replace(base, **overrides)


def plant_plan(case: Case, seed: int = MASTER_SEED) -> Dict[str, np.ndarray]:
    """Where the structure is planted: sign vectors u [L, H_kv, d] of the recency band,
    and per (layer, KV head) the planted context positions pos [L, H_kv, P] (distinct) with
    the (group head g, query i) whose scaled copy is written there."""
    c = case
    rng = np.random.default_rng([seed, 77])
    u = rng.integers(0, 2, size=(c.L_s, c.H_kv, c.d)).astype(np.float32) * 2 - 1
    P = c.n_planted
    pos = np.zeros((c.L_s, c.H_kv, P), dtype=np.int64)
    src = np.zeros((c.L_s, c.H_kv, P), dtype=np.int64)
    for l in range(c.L_s):
        for h in range(c.H_kv):
            if P:
                pos[l, h] = rng.choice(c.N, size=P, replace=False)
                src[l, h] = rng.choice(c.G * c.N_q, size=P, replace=False)
    return {"u": u, "pos": pos, "g": src // c.N_q, "i": src % c.N_q}


def make_proxy_qk(case: Case, seed: int = MASTER_SEED, device="cpu",
                  layers: Optional[range] = None):
    """Proxy reconstruction queries and keys.

    Returns (q_rec [L, H_q, N_q, d], k_ctx [L, H_kv, N, d], k_rec [L, H_kv, N_q, d]) as
    bf16 tensors, or fp32 holding unrounded values when case.fp32_inputs.  Structure:
    N(0,1)-like base; optional recency band (a per-(layer, KV head) sign vector u is added,
    times band_shift, to every query of the group and to the last `recency_band` context
    keys); `n_planted` context keys per (layer, KV head) at distinct random positions are
    overwritten by plant_scale times a distinct random query of the group.
    """
    c = case
    L = c.L_s
    q = normal_tensor((L, c.H_q, c.N_q, c.d), seed, TID_Q_REC, device)
    k_ctx = normal_tensor((L, c.H_kv, c.N, c.d), seed, TID_K_CTX, device)
    k_rec = normal_tensor((L, c.H_kv, c.N_q, c.d), seed, TID_K_REC, device)
    plan = plant_plan(c, seed)
    if c.recency_band > 0:
        u = torch.from_numpy(plan["u"]).to(device)
        q += c.band_shift * u.repeat_interleave(c.G, dim=1)[:, :, None, :]
        k_ctx[:, :, c.N - c.recency_band:, :] += c.band_shift * u[:, :, None, :]
    if not c.fp32_inputs:
        q = q.to(torch.bfloat16).to(torch.float32)
    if c.n_planted > 0:
        for l in range(L):
            for h in range(c.H_kv):
                pos = torch.from_numpy(plan["pos"][l, h]).to(device)
                g = torch.from_numpy(plan["g"][l, h]).to(device)
                i = torch.from_numpy(plan["i"][l, h]).to(device)
                k_ctx[l, h, pos] = c.plant_scale * q[l, h * c.G + g, i]
    if c.fp32_inputs:
        return q, k_ctx, k_rec
    return q.to(torch.bfloat16), k_ctx.to(torch.bfloat16), k_rec.to(torch.bfloat16)


def make_target_kv(case: Case, seed: int = MASTER_SEED, device="cpu"):
    """Target KV cache: (k_t, v_t), each bf16 [L_l, H_l, N, D], N(0,1)-like."""
    shape = (case.L_l, case.H_l, case.N, case.D)
    k_t = normal_tensor(shape, seed, TID_K_T, device).to(torch.bfloat16)
    v_t = normal_tensor(shape, seed, TID_V_T, device).to(torch.bfloat16)
    return k_t, v_t


@dataclasses.dataclass(frozen=True)
class MapperDims:
    d_time: int = 512
    c_mid: int = 256
    n_enc_layers: int = 6
    n_enc_heads: int = 8
    d_ffn: int = 2048
    d_head_x: int = 64
    win: int = 2048
    stride: int = 1024


def make_mapper_weights(H_s: int, H_l: int, dims: MapperDims = MapperDims(),
                        seed: int = MASTER_SEED) -> Dict[str, torch.Tensor]:
    """Random-init HybridAxialMapper weights as named fp32 CPU tensors.

    Linear/conv weights and biases ~ U(+-1/sqrt(fan_in)); target queries ~ N(0,1); norm
    scales ~ U(0.5,1.5); norm shifts and running means ~ U(-0.1,0.1); running variances
    ~ U(0.5,1.5).  Names follow the mapper's three stages (stem / enc.<i> / head).
    """
    rng = np.random.default_rng([seed, 4242])
    w: Dict[str, torch.Tensor] = {}

    def uni(name, shape, bound):
        w[name] = torch.from_numpy(rng.uniform(-bound, bound, size=shape).astype(np.float32))

    def rng_range(name, shape, lo, hi):
        w[name] = torch.from_numpy(rng.uniform(lo, hi, size=shape).astype(np.float32))

    def norm(prefix, n, running):
        rng_range(prefix + ".gamma", (n,), 0.5, 1.5)
        rng_range(prefix + ".beta", (n,), -0.1, 0.1)
        if running:
            rng_range(prefix + ".mean", (n,), -0.1, 0.1)
            rng_range(prefix + ".var", (n,), 0.5, 1.5)

    D, C1, F, dh = dims.d_time, dims.c_mid, dims.d_ffn, dims.d_head_x
    b = 1.0 / np.sqrt(3 * H_s)
    uni("stem.conv1.weight", (C1, H_s, 3), b)
    uni("stem.conv1.bias", (C1,), b)
    norm("stem.bn1", C1, True)
    b = 1.0 / np.sqrt(3 * C1)
    uni("stem.conv2.weight", (D, C1, 3), b)
    uni("stem.conv2.bias", (D,), b)
    norm("stem.bn2", D, True)
    for i in range(dims.n_enc_layers):
        p = f"enc.{i}."
        b = 1.0 / np.sqrt(D)
        uni(p + "in_proj.weight", (3 * D, D), b)
        uni(p + "in_proj.bias", (3 * D,), b)
        uni(p + "out_proj.weight", (D, D), b)
        uni(p + "out_proj.bias", (D,), b)
        norm(p + "ln1", D, False)
        uni(p + "ffn1.weight", (F, D), b)
        uni(p + "ffn1.bias", (F,), b)
        b2 = 1.0 / np.sqrt(F)
        uni(p + "ffn2.weight", (D, F), b2)
        uni(p + "ffn2.bias", (D,), b2)
        norm(p + "ln2", D, False)
    b = 1.0 / np.sqrt(D)
    uni("head.k_proj.weight", (H_s * dh, D), b)
    uni("head.k_proj.bias", (H_s * dh,), b)
    uni("head.v_proj.weight", (H_s * dh, D), b)
    uni("head.v_proj.bias", (H_s * dh,), b)
    w["head.queries"] = torch.from_numpy(rng.standard_normal((H_l, dh)).astype(np.float32))
    b = 1.0 / np.sqrt(dh)
    uni("head.out.weight", (dh,), b)
    uni("head.out.bias", (1,), b)
    return w
