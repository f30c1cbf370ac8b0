"""Seeded synthetic inputs for the verification step: target logits, draft
distributions and draft tokens shaped like LLM serving workloads.

This module only manufactures inputs.  It holds none of the verification step's own
arithmetic (no accept test, no residual, no sampling of output tokens); both the GPU
library's tests and the CPU oracle's tests read the tensors it returns.

Recipe (one generator for every workload):
  * a seeded permutation `perm` of the vocabulary carries a Zipf(s) popularity bias,
    bias[perm[r]] = -s * ln(r + 1);
  * target logits z = 2 * N(0,1) + bias, independent per row, stored as fp32 or rounded
    to bf16 (round-to-nearest-even);
  * draft distribution Q = softmax((z_stored + sigma * N(0,1)) * inv_temperature) in fp32,
    i.e. the draft model is a noisy copy of the target;
  * draft token x ~ Q (torch.multinomial);
  * optional per-session temperature T ~ U[T_lo, T_hi], applied to both models;
  * optional ragged batch: gamma_b ~ U{g_lo..g_hi}, rows packed with prefix-sum offsets;
  * optional top-k truncation (the paper's experiments sample with k = 10): the target logits
    outside each row's k largest are stored as -inf and each draft row keeps only its own k
    largest entries, renormalised (the draft is drawn from the full target row first);
  * optional session classes: a fraction with Q == P (Q = softmax of the stored target
    logits, so every draft is accepted up to rounding) and a fraction with Q uniform.
"""
from dataclasses import dataclass, replace
from typing import Optional, Tuple

import torch


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    V: int
    gamma: int                                   # uniform gamma (ignored when gamma_range is set)
    dtype: str                                   # "f32" or "bf16" (storage type of the logits)
    zipf_s: float = 1.1
    sigmas: Tuple[float, ...] = (0.5,)           # session b uses sigmas[b * len(sigmas) // B]
    temperature_range: Optional[Tuple[float, float]] = None
    gamma_range: Optional[Tuple[int, int]] = None
    frac_q_equals_p: float = 0.0
    frac_q_uniform: float = 0.0
    top_k: int = 0                               # > 0: both models truncated to their own top-k tokens


# The five workloads of the benchmark definition, by index.
WORKLOADS = (
    Workload("cfg0_B1_g4_V32000_f32", B=1, V=32000, gamma=4, dtype="f32", zipf_s=1.1, sigmas=(0.5,)),
    Workload("cfg1_B64_g4_V32000_f32", B=64, V=32000, gamma=4, dtype="f32", zipf_s=1.1, sigmas=(0.5,)),
    Workload("cfg2_B256_g8_V128256_bf16", B=256, V=128256, gamma=8, dtype="bf16", zipf_s=1.2,
             sigmas=(1.0,)),
    Workload("cfg3_B512_g16_V152064_bf16_temp", B=512, V=152064, gamma=16, dtype="bf16", zipf_s=1.1,
             sigmas=(0.25, 0.5, 1.0, 2.0), temperature_range=(0.5, 1.5)),
    Workload("cfg4_B1024_ragged_g1-16_V256000_bf16", B=1024, V=256000, gamma=0, dtype="bf16",
             zipf_s=1.0, sigmas=(0.5,), gamma_range=(1, 16), frac_q_equals_p=0.10,
             frac_q_uniform=0.10),
)


def scaled(w: Workload, **changes) -> Workload:
    """A copy of a workload with some fields changed (smaller B or V for CPU-sized tests)."""
    return replace(w, **changes)


def generate(w: Workload, seed: int = 0, device="cpu", sessions_per_chunk: int = 32):
    """Build the inputs of one verify step.  Returns a dict of tensors on `device`:

    logits [R_L, V] (float32 or bfloat16), draft_probs [R_Q, V] float32,
    draft_tokens [R_Q] int32, draft_offsets [B+1] int32 (None when gamma is uniform),
    inv_temperature [B] float32 (None when no temperature), session_class [B] int32
    (0 normal, 1 Q == P, 2 Q uniform), plus B, V, gamma, R_L, R_Q as ints.
    """
    dev = torch.device(device)
    g = torch.Generator(device=dev)
    g.manual_seed(int(seed) * 1000003 + 12345)
    B, V = w.B, w.V
    if w.gamma_range is not None:
        lo, hi = w.gamma_range
        gammas = torch.randint(lo, hi + 1, (B,), generator=g, device=dev, dtype=torch.int64)
    else:
        gammas = torch.full((B,), w.gamma, device=dev, dtype=torch.int64)
    offsets = torch.zeros(B + 1, device=dev, dtype=torch.int64)
    offsets[1:] = torch.cumsum(gammas, 0)
    R_Q = int(offsets[-1].item())
    R_L = R_Q + B

    perm = torch.randperm(V, generator=g, device=dev)
    bias = torch.empty(V, device=dev, dtype=torch.float32)
    bias[perm] = -w.zipf_s * torch.log(torch.arange(1, V + 1, device=dev, dtype=torch.float32))

    if w.temperature_range is not None:
        t_lo, t_hi = w.temperature_range
        temperature = t_lo + (t_hi - t_lo) * torch.rand(B, generator=g, device=dev)
        inv_temperature = (1.0 / temperature).to(torch.float32)
    else:
        inv_temperature = None

    sig_table = torch.tensor(w.sigmas, device=dev, dtype=torch.float32)
    sig_idx = (torch.arange(B, device=dev) * len(w.sigmas)) // max(B, 1)
    sigma_b = sig_table[sig_idx]

    cls_draw = torch.rand(B, generator=g, device=dev)
    session_class = torch.zeros(B, device=dev, dtype=torch.int32)
    session_class[cls_draw < w.frac_q_equals_p] = 1
    session_class[(cls_draw >= w.frac_q_equals_p)
                  & (cls_draw < w.frac_q_equals_p + w.frac_q_uniform)] = 2

    store = torch.float32 if w.dtype == "f32" else torch.bfloat16
    logits = torch.empty((R_L, V), device=dev, dtype=store)
    draft_probs = torch.empty((R_Q, V), device=dev, dtype=torch.float32)
    draft_tokens = torch.empty(R_Q, device=dev, dtype=torch.int32)

    for b0 in range(0, B, sessions_per_chunk):
        b1 = min(B, b0 + sessions_per_chunk)
        q0, q1 = int(offsets[b0].item()), int(offsets[b1].item())
        l0, l1 = q0 + b0, q1 + b1
        z = 2.0 * torch.randn((l1 - l0, V), generator=g, device=dev, dtype=torch.float32) + bias
        logits[l0:l1] = z.to(store)
        if q1 == q0:
            if w.top_k > 0:
                kth = torch.topk(z, min(w.top_k, V), dim=1).values[:, -1:]
                logits[l0:l1] = torch.where(z >= kth, z, torch.full_like(z, float("-inf"))).to(store)
            continue
        # session of every draft row in the chunk, and the logits row it is paired with
        sess = torch.repeat_interleave(torch.arange(b0, b1, device=dev), gammas[b0:b1])
        qrow = torch.arange(q0, q1, device=dev)
        lrow = qrow + sess - l0
        zs = logits[l0:l1].to(torch.float32)[lrow]          # what the target model "said"
        noise = torch.randn((q1 - q0, V), generator=g, device=dev, dtype=torch.float32)
        cls = session_class[sess]
        sig = torch.where(cls == 1, torch.zeros_like(sigma_b[sess]), sigma_b[sess])
        y = zs + sig[:, None] * noise
        if inv_temperature is not None:
            y = y * inv_temperature[sess][:, None]
        if w.top_k > 0:
            kth = torch.topk(y, min(w.top_k, V), dim=1).values[:, -1:]
            y = torch.where(y >= kth, y, torch.full_like(y, float("-inf")))
        Q = torch.softmax(y, dim=1)
        Q[cls == 2] = 1.0 / V
        draft_probs[q0:q1] = Q
        draft_tokens[q0:q1] = torch.multinomial(Q, 1, generator=g).squeeze(1).to(torch.int32)
        del z, zs, noise, y, Q
        if w.top_k > 0:
            zf = logits[l0:l1].to(torch.float32)
            kth = torch.topk(zf, min(w.top_k, V), dim=1).values[:, -1:]
            logits[l0:l1] = torch.where(zf >= kth, zf, torch.full_like(zf, float("-inf"))).to(store)

    uniform = w.gamma_range is None
    return dict(
        logits=logits, draft_probs=draft_probs, draft_tokens=draft_tokens,
        draft_offsets=None if uniform else offsets.to(torch.int32),
        inv_temperature=inv_temperature, session_class=session_class,
        B=B, V=V, gamma=w.gamma if uniform else 0, R_L=R_L, R_Q=R_Q, dtype=w.dtype, name=w.name)
