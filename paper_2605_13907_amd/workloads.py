"""Seeded synthetic rollout batches shaped like the paper's GRPO workloads.

This module only *makes inputs*: trainer logits, the tokens a low-precision
rollout engine would have sampled, that engine's log-probabilities, masks and
rewards.  It plays the part of the two systems the method sits between (the FP8
sampler and the BF16 trainer forward, Sec. 3 "Method", first paragraph, and
App. "Low-bit Rollout and AIS") and contains none of the correction itself: no
importance ratio, no diagnostic, no mixing coefficient, no loss, no gradient.
Both the GPU library's tests and the CPU oracle's tests draw their inputs here;
the generated *bits* (not the random generator) are what the two sides share.

Recipe for one batch (all random draws come from seeded torch generators):

1. trainer logits z ~ N(0, sigma^2) in fp32; optionally the row's arg-max gets
   ``boost`` added (a peaked, LLM-like row); the result is cast to the storage
   dtype (bf16 or fp32) and that cast value *is* the trainer logit;
2. rollout logits z_r = s * e4m3(z / s) with a per-row scale s = max|z| / 448,
   e4m3 being the OCP FP8 E4M3 "fn" format (4 exponent bits, 3 mantissa bits,
   bias 7, max 448, round-to-nearest-even) that Sec. 2.1 names; one workload
   adds extra N(0, noise^2) to z_r;
3. the sampled token y ~ Categorical(softmax(z_r)) by the Gumbel-max trick;
4. logp_roll = log_softmax(z_r)[y] stored as fp32;
5. rewards ~ Bernoulli(p) per response; G consecutive responses form a group
   (G = 8 is the paper's "number of generations", App. hyper-parameter table).

Small metadata (lengths, masks, rewards) is always drawn on the CPU so it is
identical whatever device the bulk tensors are generated on.
"""
from __future__ import annotations

import dataclasses
import math
from dataclasses import dataclass
from typing import Optional, Tuple

import torch

E4M3_MAX = 448.0


@dataclass(frozen=True)
class RolloutShape:
    """Shape and value structure of one synthetic rollout batch."""

    name: str
    n_prompts: int
    group_size: int
    vocab: int
    logits_dtype: str            # "bf16" | "f32"
    sigma: float                 # std of the trainer logits
    boost: float                 # added to the row arg-max (0 = none)
    layout: str                  # "padded" | "packed" | "masked"
    max_len: int
    length_dist: Tuple           # ("uniform", lo, hi) | ("lognormal", median, s, lo) | ("fixed",)
    reward_p: float
    rollout_noise: float = 0.0   # extra N(0, noise^2) on the rollout logits
    seed: int = 0

    @property
    def n_resp(self) -> int:
        return self.n_prompts * self.group_size

    def scaled(self, *, vocab: Optional[int] = None, len_div: int = 1,
               n_prompts: Optional[int] = None, seed: Optional[int] = None,
               name: Optional[str] = None) -> "RolloutShape":
        """A smaller batch with the same structure (for tests the oracle can finish)."""
        kind = self.length_dist[0]
        if kind == "uniform":
            ld = ("uniform", max(1, self.length_dist[1] // len_div),
                  max(1, self.length_dist[2] // len_div))
        elif kind == "lognormal":
            ld = ("lognormal", max(1.0, self.length_dist[1] / len_div), self.length_dist[2],
                  max(1, self.length_dist[3] // len_div))
        else:
            ld = self.length_dist
        return dataclasses.replace(
            self,
            name=name or f"{self.name}/scaled",
            vocab=vocab or self.vocab,
            max_len=max(1, self.max_len // len_div),
            length_dist=ld,
            n_prompts=n_prompts or self.n_prompts,
            seed=self.seed if seed is None else seed,
        )


# The five workloads.  Vocabulary sizes are those of the model families the
# paper trains (Sec. 4.1 "Models"); lengths, dtype and reward rates are the
# synthetic stand-ins for its task mix.
CONFIGS = (
    RolloutShape("tiny", n_prompts=2, group_size=4, vocab=1024, logits_dtype="f32",
                 sigma=2.0, boost=0.0, layout="padded", max_len=64,
                 length_dist=("uniform", 16, 64), reward_p=0.5, seed=1001),
    RolloutShape("qwen3-8b", n_prompts=2, group_size=8, vocab=151_936, logits_dtype="bf16",
                 sigma=3.0, boost=8.0, layout="packed", max_len=4096,
                 length_dist=("uniform", 512, 4096), reward_p=0.4, seed=1002),
    RolloutShape("llada-8b", n_prompts=8, group_size=8, vocab=126_464, logits_dtype="bf16",
                 sigma=3.0, boost=0.0, layout="masked", max_len=512,
                 length_dist=("fixed",), reward_p=0.5, seed=1003),
    RolloutShape("qwen3.5-9b", n_prompts=4, group_size=8, vocab=248_320, logits_dtype="bf16",
                 sigma=3.0, boost=8.0, layout="packed", max_len=2048,
                 length_dist=("uniform", 256, 2048), reward_p=0.3, seed=1004),
    RolloutShape("long-horizon", n_prompts=1, group_size=8, vocab=151_936, logits_dtype="bf16",
                 sigma=3.0, boost=0.0, layout="packed", max_len=32_768,
                 length_dist=("lognormal", 8192.0, 0.8, 64), reward_p=0.2,
                 rollout_noise=0.5, seed=1005),
)


def config(k: int) -> RolloutShape:
    """Workload k, numbered from 1 as in the list above."""
    return CONFIGS[k - 1]


@dataclass
class RolloutBatch:
    """Tensors of one batch.  Rows are token positions; response i owns rows
    [cu_rows[i], cu_rows[i+1]); prompt p owns responses [p*G, (p+1)*G)."""

    shape: RolloutShape
    logits: torch.Tensor      # [R, V] bf16 or fp32, row-major
    token_ids: torch.Tensor   # [R] int32; -1 on rows that are not evaluated
    valid: torch.Tensor       # [R] uint8
    cu_rows: torch.Tensor     # [B+1] int64
    logp_roll: torch.Tensor   # [R] fp32; 0 on rows that are not evaluated
    rewards: torch.Tensor     # [B] fp32
    lengths: torch.Tensor     # [B] int64 (CPU): generated tokens per response

    @property
    def n_rows(self) -> int:
        return int(self.logits.shape[0])

    @property
    def n_valid(self) -> int:
        return int(self.valid.sum().item())


def e4m3_round_trip(x: torch.Tensor) -> torch.Tensor:
    """x rounded to the nearest OCP FP8 E4M3 "fn" value (ties to even), saturating at +-448."""
    return x.clamp(-E4M3_MAX, E4M3_MAX).to(torch.float8_e4m3fn).to(torch.float32)


def fp8_rollout_logits(z: torch.Tensor) -> torch.Tensor:
    """Per-row absmax-scaled E4M3 round trip of fp32 logits z [rows, V] (step 2 of the recipe)."""
    amax = z.abs().amax(dim=1, keepdim=True)
    # tensor / tensor is a true fp32 division on every device; tensor / python-scalar is evaluated on the GPU
    # as a multiplication by the rounded reciprocal, which would make the scale depend on the device
    s = amax / torch.full_like(amax, E4M3_MAX)
    s = torch.where(s > 0, s, torch.ones_like(s))
    return e4m3_round_trip(z / s) * s


def _draw_lengths(shape: RolloutShape, gen: torch.Generator) -> torch.Tensor:
    B = shape.n_resp
    kind = shape.length_dist[0]
    if kind == "fixed":
        return torch.full((B,), shape.max_len, dtype=torch.int64)
    if kind == "uniform":
        lo, hi = shape.length_dist[1], shape.length_dist[2]
        return torch.randint(lo, hi + 1, (B,), generator=gen, dtype=torch.int64)
    if kind == "lognormal":
        median, s, lo = shape.length_dist[1], shape.length_dist[2], shape.length_dist[3]
        x = torch.randn(B, generator=gen, dtype=torch.float64) * s + math.log(median)
        return x.exp().floor().to(torch.int64).clamp(min=lo, max=shape.max_len)
    raise ValueError(f"unknown length distribution {kind!r}")


def layout_of(shape: RolloutShape):
    """CPU-side structure of the batch: (lengths[B], valid[R] uint8, cu_rows[B+1], rewards[B])."""
    gen = torch.Generator(device="cpu")
    gen.manual_seed(shape.seed)
    B = shape.n_resp
    lengths = _draw_lengths(shape, gen)
    rewards = (torch.rand(B, generator=gen, dtype=torch.float64) < shape.reward_p).to(torch.float32)
    if shape.layout == "packed":
        cu = torch.zeros(B + 1, dtype=torch.int64)
        cu[1:] = torch.cumsum(lengths, 0)
        valid = torch.ones(int(cu[-1]), dtype=torch.uint8)
    elif shape.layout == "padded":
        cu = torch.arange(B + 1, dtype=torch.int64) * shape.max_len
        pos = torch.arange(shape.max_len).unsqueeze(0)
        valid = (pos < lengths.unsqueeze(1)).to(torch.uint8).reshape(-1)
    elif shape.layout == "masked":
        # diffusion-style: log-probs are evaluated on a random subset of positions,
        # mask ratio t ~ U(0,1) per response, positions i.i.d. Bernoulli(t)
        cu = torch.arange(B + 1, dtype=torch.int64) * shape.max_len
        t = torch.rand(B, generator=gen, dtype=torch.float64)
        u = torch.rand(B, shape.max_len, generator=gen, dtype=torch.float64)
        valid = (u < t.unsqueeze(1)).to(torch.uint8).reshape(-1)
    else:
        raise ValueError(f"unknown layout {shape.layout!r}")
    return lengths, valid, cu, rewards


def generate(shape: RolloutShape, device: str = "cpu", row_chunk: int = 256) -> RolloutBatch:
    """Build one batch on ``device``.  Deterministic for a given (shape, device type, torch build)."""
    lengths, valid_cpu, cu, rewards = layout_of(shape)
    R, V = int(valid_cpu.numel()), shape.vocab
    dt = torch.bfloat16 if shape.logits_dtype == "bf16" else torch.float32
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(shape.seed + 7919)

    logits = torch.empty((R, V), dtype=dt, device=dev)
    token_ids = torch.empty(R, dtype=torch.int32, device=dev)
    logp_roll = torch.empty(R, dtype=torch.float32, device=dev)
    tiny = torch.finfo(torch.float32).tiny
    for r0 in range(0, R, row_chunk):
        r1 = min(R, r0 + row_chunk)
        n = r1 - r0
        z = torch.randn((n, V), generator=gen, device=dev, dtype=torch.float32) * shape.sigma
        if shape.boost != 0.0:
            top = z.argmax(dim=1, keepdim=True)
            z.scatter_add_(1, top, torch.full_like(top, shape.boost, dtype=torch.float32))
        logits[r0:r1] = z.to(dt)
        z = logits[r0:r1].to(torch.float32)            # the trainer's logits, exactly
        zr = fp8_rollout_logits(z)
        if shape.rollout_noise != 0.0:
            zr += torch.randn((n, V), generator=gen, device=dev, dtype=torch.float32) * shape.rollout_noise
        u = torch.rand((n, V), generator=gen, device=dev, dtype=torch.float32).clamp_(min=tiny)
        gumbel = -torch.log(-torch.log(u))
        y = (zr + gumbel).argmax(dim=1, keepdim=True)
        lp = torch.log_softmax(zr, dim=1).gather(1, y)
        token_ids[r0:r1] = y.squeeze(1).to(torch.int32)
        logp_roll[r0:r1] = lp.squeeze(1)
        del z, zr, u, gumbel, y, lp

    valid = valid_cpu.to(dev)
    off = valid == 0
    token_ids[off] = -1           # rows that are not evaluated carry no usable token
    logp_roll[off] = 0.0
    return RolloutBatch(shape=shape, logits=logits, token_ids=token_ids, valid=valid,
                        cu_rows=cu.to(dev), logp_roll=logp_roll, rewards=rewards.to(dev),
                        lengths=lengths)


# ---------------------------------------------------------------------------------------------------------
# Inputs of the hidden-state read-out: final hidden states and an output-embedding matrix instead of logits.

# d_model of the model families whose vocabularies the workloads above use (public model cards).
D_MODEL = {"tiny": 64, "qwen3-8b": 4096, "llada-8b": 4096, "qwen3.5-9b": 4096, "long-horizon": 4096}


@dataclass
class ReadoutBatch:
    """hidden [R, D] and weight [V, D] in bf16, sampled tokens and mask as in RolloutBatch."""

    hidden: torch.Tensor
    weight: torch.Tensor
    token_ids: torch.Tensor   # [R] int32; -1 on rows that are not evaluated
    valid: torch.Tensor       # [R] uint8


def generate_readout(shape: RolloutShape, d_model: Optional[int] = None, device: str = "cpu",
                     n_rows: Optional[int] = None) -> ReadoutBatch:
    """Seeded hidden states and output embeddings whose logits look like a language model's.

    weight rows ~ N(0, I/D) (unit norm on average).  Every row t has a preferred token m_t and a sharpness
    b_t ~ U(0, 12): hidden_t = b_t * weight[m_t] / |weight[m_t]|^2 + xi_t with xi_t ~ N(0, I), so the preferred
    token's logit is b_t + N(0, 1) against a background of roughly N(0, 1 + b_t^2 / D): rows from nearly flat
    to sharply peaked.  The sampled token is m_t with probability 0.7, else uniform over the vocabulary.  Row structure
    (number of rows, mask) is the rollout shape's.  All draws are seeded; bulk tensors are drawn on
    ``device`` and rounded to bf16, and the rounded values are the inputs."""
    _, valid_cpu, _, _ = layout_of(shape)
    R = int(valid_cpu.numel()) if n_rows is None else int(n_rows)
    valid_cpu = valid_cpu[:R]
    V = shape.vocab
    D = int(d_model or D_MODEL.get(shape.name.split("/")[0], 64))
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(shape.seed + 77)
    cgen = torch.Generator(device="cpu")
    cgen.manual_seed(shape.seed + 78)
    weight = (torch.randn(V, D, generator=gen, device=dev, dtype=torch.float32) / math.sqrt(D)).to(torch.bfloat16)
    mode = torch.randint(0, V, (R,), generator=cgen, dtype=torch.int64)
    sharp = torch.rand(R, generator=cgen, dtype=torch.float32) * 12.0
    other = torch.randint(0, V, (R,), generator=cgen, dtype=torch.int64)
    pick = torch.rand(R, generator=cgen, dtype=torch.float32) < 0.7
    y = torch.where(pick, mode, other).to(torch.int32)
    y = torch.where(valid_cpu.bool(), y, torch.full_like(y, -1))
    hidden = torch.empty(R, D, device=dev, dtype=torch.bfloat16)
    step = 4096
    for r0 in range(0, R, step):
        r1 = min(R, r0 + step)
        wm = weight[mode[r0:r1].to(dev)].to(torch.float32)
        nrm = (wm * wm).sum(dim=1, keepdim=True).clamp_min(1e-6)
        noise = torch.randn(r1 - r0, D, generator=gen, device=dev, dtype=torch.float32)
        b = sharp[r0:r1].to(dev).unsqueeze(1)
        hidden[r0:r1] = (b * wm / nrm + noise).to(torch.bfloat16)
    return ReadoutBatch(hidden=hidden, weight=weight, token_ids=y.to(dev), valid=valid_cpu.to(dev))
