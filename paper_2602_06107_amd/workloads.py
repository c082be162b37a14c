"""Seeded synthetic inputs shaped like the paper's Qwen3 workloads.

This module only draws random numbers and lays them out; it contains none of
the OBRS arithmetic and imports neither the HIP binding nor the CPU oracle, so
both sides can be fed the very same bits.

Recipe (all draws from one ``torch.Generator`` seeded ``20260206 + index``,
consumed in row blocks of ``GEN_BLOCK_ROWS`` so the stream does not depend on
free memory):

* ``tiny``        T=64,    V=1024,   fp32: actor ~ N(0, 2^2); policy = actor + N(0, 0.5^2)
* ``rollout``     T=8192,  V=151936, bf16: actor ~ N(0,1) with +8 on 20 random ids per row;
                                           policy = actor + N(0, 1.0^2)
* ``training``    T=65536, V=151936, bf16: as ``rollout`` with policy noise N(0, 2.0^2)
* ``long``        T=32768, V=151936, bf16: policy noise sigma_t ~ U(0.1, 3.0) per row

The policy noise is added in fp32 to the un-rounded actor value and both rows
are then rounded to the storage dtype.  The sampled token is drawn from
softmax(actor) with the Gumbel-max trick (argmax of stored logit + Gumbel
noise), the Bernoulli uniforms are U[0,1) in fp32.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Optional

import numpy as np
import torch

BASE_SEED = 20260206
GEN_BLOCK_ROWS = 512
QWEN3_VOCAB = 151936          # padded Qwen2.5 / Qwen3 vocabulary


@dataclass
class Workload:
    name: str
    actor: torch.Tensor                 # [T, V] rollout-model logits (p_inf)
    policy: torch.Tensor                # [T, V] target-model logits (p_target)
    sampled_ids: torch.Tensor           # [T] int32, < 0 marks a padding row
    uniforms: torch.Tensor              # [T] fp32 in [0, 1)
    lam: float = 1.0
    k: int = 64
    c1: float = 3.0
    c2: float = 3.0
    ref_logprob: Optional[torch.Tensor] = None   # [T] fp32 log p_ref(x) or None
    meta: dict = field(default_factory=dict)

    @property
    def T(self) -> int:
        return self.actor.shape[0]

    @property
    def V(self) -> int:
        return self.actor.shape[1]

    def with_params(self, **kw) -> "Workload":
        return replace(self, **kw)


def _gumbel_argmax(stored: torch.Tensor, gen: torch.Generator) -> torch.Tensor:
    u = torch.rand(stored.shape, generator=gen, device=stored.device, dtype=torch.float32)
    u.clamp_(min=1e-20, max=1.0 - 1e-7)
    g = -torch.log(-torch.log(u))
    return torch.argmax(stored.float() + g, dim=1).to(torch.int32)


def make_logits(T: int, V: int, dtype: torch.dtype, *, seed: int, device="cpu",
                actor_sigma: float = 1.0, spikes: int = 20, spike_height: float = 8.0,
                noise_sigma=1.0, noise_sigma_range=None, pad_every: int = 0,
                name: str = "custom", row_stride: Optional[int] = None) -> Workload:
    """Draw one batch.  ``noise_sigma_range=(lo, hi)`` draws a per-row policy noise scale.

    ``row_stride`` (elements, >= V) leaves unused columns between rows to exercise strided input.
    ``pad_every=n`` marks every n-th row as padding (sampled id -1).
    """
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)
    stride = V if row_stride is None else row_stride
    assert stride >= V
    actor_buf = torch.zeros((T, stride), dtype=dtype, device=dev)
    policy_buf = torch.zeros((T, stride), dtype=dtype, device=dev)
    actor, policy = actor_buf[:, :V], policy_buf[:, :V]
    ids = torch.empty(T, dtype=torch.int32, device=dev)
    uni = torch.empty(T, dtype=torch.float32, device=dev)
    sig_rows = None
    if noise_sigma_range is not None:
        lo, hi = noise_sigma_range
        sig_rows = lo + (hi - lo) * torch.rand(T, generator=gen, device=dev, dtype=torch.float32)
    for r0 in range(0, T, GEN_BLOCK_ROWS):
        r1 = min(T, r0 + GEN_BLOCK_ROWS)
        n = r1 - r0
        a = torch.randn((n, V), generator=gen, device=dev, dtype=torch.float32)
        if actor_sigma != 1.0:
            a.mul_(actor_sigma)
        if spikes > 0 and V > 0:
            sid = torch.randint(0, V, (n, spikes), generator=gen, device=dev)
            a.scatter_(1, sid, a.gather(1, sid) + spike_height)
        z = torch.randn((n, V), generator=gen, device=dev, dtype=torch.float32)
        if sig_rows is not None:
            z.mul_(sig_rows[r0:r1, None])
        else:
            z.mul_(float(noise_sigma))
        z.add_(a)
        actor[r0:r1] = a.to(dtype)
        policy[r0:r1] = z.to(dtype)
        del a, z
        if V > 0:
            ids[r0:r1] = _gumbel_argmax(actor[r0:r1], gen)
        uni[r0:r1] = torch.rand(n, generator=gen, device=dev, dtype=torch.float32)
    if pad_every > 0:
        ids[pad_every - 1::pad_every] = -1
    meta = dict(seed=seed, dtype=str(dtype).replace("torch.", ""), T=T, V=V, row_stride=stride)
    if sig_rows is not None:
        meta["noise_sigma_rows"] = sig_rows
    return Workload(name=name, actor=actor, policy=policy, sampled_ids=ids, uniforms=uni, meta=meta)


def tiny(device="cpu") -> Workload:
    """T=64, V=1024, fp32, lambda=1, k=32, one batch."""
    w = make_logits(64, 1024, torch.float32, seed=BASE_SEED + 0, device=device, actor_sigma=2.0,
                    spikes=0, noise_sigma=0.5, name="tiny")
    return w.with_params(lam=1.0, k=32)


def rollout(device="cuda", T: int = 8192, V: int = QWEN3_VOCAB) -> Workload:
    """Qwen3-1.7B-shaped rollout batch: 16 sequences x 512 tokens, bf16, k=64, lambda in {0.5,1,2}."""
    w = make_logits(T, V, torch.bfloat16, seed=BASE_SEED + 1, device=device, noise_sigma=1.0,
                    name="rollout")
    return w.with_params(lam=1.0, k=64)


def training(device="cuda", T: int = 65536, V: int = QWEN3_VOCAB) -> Workload:
    """Qwen3-8B-shaped training batch: 64 prompts x 8 samples x 128 tokens, bf16, k=128."""
    w = make_logits(T, V, torch.bfloat16, seed=BASE_SEED + 2, device=device, noise_sigma=2.0,
                    name="training")
    return w.with_params(lam=1.0, k=128)


def long_response(device="cuda", T: int = 32768, V: int = QWEN3_VOCAB) -> Workload:
    """4 sequences x 8192 tokens, bf16, per-row noise scale U(0.1, 3.0); k swept over {16,64,256}."""
    w = make_logits(T, V, torch.bfloat16, seed=BASE_SEED + 3, device=device,
                    noise_sigma_range=(0.1, 3.0), name="long")
    return w.with_params(lam=1.0, k=64)


# ---- host views for the CPU side (exact bit copies) --------------------------

def logits_to_numpy(t: torch.Tensor) -> np.ndarray:
    """Stored logits as a numpy array: fp32 as float32, bf16 as its raw bits in uint16."""
    t = t.detach().cpu()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    if t.dtype == torch.float32:
        return t.numpy()
    raise TypeError(t.dtype)


def bf16_bits_to_float64(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def logits_to_float64(t: torch.Tensor) -> np.ndarray:
    a = logits_to_numpy(t)
    return bf16_bits_to_float64(a) if a.dtype == np.uint16 else a.astype(np.float64)


# ---- fused lm_head form: hidden states and vocabulary projections instead of logits --------------

@dataclass
class LmHeadWorkload:
    name: str
    H_actor: torch.Tensor        # [T, d_actor]  bf16
    W_actor: torch.Tensor        # [d_actor, V]  bf16
    H_policy: torch.Tensor       # [T, d_policy] bf16
    W_policy: torch.Tensor       # [d_policy, V] bf16
    sampled_ids: torch.Tensor    # [T] int32
    uniforms: torch.Tensor       # [T] fp32
    lam: float = 1.0
    k: int = 64
    c1: float = 3.0
    c2: float = 3.0
    ref_logprob: Optional[torch.Tensor] = None

    @property
    def T(self) -> int:
        return self.H_actor.shape[0]

    @property
    def V(self) -> int:
        return self.W_actor.shape[1]

    def with_params(self, **kw) -> "LmHeadWorkload":
        return replace(self, **kw)


def lm_head(T: int = 16384, V: int = QWEN3_VOCAB, d_actor: int = 2048, d_policy: int = 4096,
            device="cuda", seed: int = BASE_SEED + 4, k: int = 64, name: str = "lm_head") -> LmHeadWorkload:
    """Hidden states N(0,1), projections N(0, 1/d), all bf16; the sampled token is drawn from
    softmax(H_actor W_actor) by Gumbel-max over vocabulary blocks (fp32 matmul of the harness)."""
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)

    def normal(shape, sigma):
        return (torch.randn(shape, generator=gen, device=dev, dtype=torch.float32) * sigma).to(torch.bfloat16)

    Ha, Wa = normal((T, d_actor), 1.0), normal((d_actor, V), d_actor ** -0.5)
    Hp, Wp = normal((T, d_policy), 1.0), normal((d_policy, V), d_policy ** -0.5)
    best = torch.full((T,), float("-inf"), device=dev)
    ids = torch.zeros(T, dtype=torch.int64, device=dev)
    blk = 8192
    Haf = Ha.float()
    for v0 in range(0, V, blk):
        logits = Haf @ Wa[:, v0:v0 + blk].float()
        u = torch.rand(logits.shape, generator=gen, device=dev, dtype=torch.float32)
        u.clamp_(min=1e-20, max=1.0 - 1e-7)
        logits.add_(-torch.log(-torch.log(u)))
        m, a = logits.max(dim=1)
        upd = m > best
        best = torch.where(upd, m, best)
        ids = torch.where(upd, a + v0, ids)
    uni = torch.rand(T, generator=gen, device=dev, dtype=torch.float32)
    return LmHeadWorkload(name, Ha, Wa, Hp, Wp, ids.to(torch.int32), uni, k=k)
