"""Synthetic rollout batches and policy-head tensors.

Shapes follow the paper's training setup (Sec. 5.1 and App. D "Implementation
Details"): 7-DoF actions in chunks of L = 8 steps, a fixed number of chunks per
trajectory, K semantic phases per trajectory, groups of G rollouts with a binary
trajectory-level reward.  The simulator, the benchmark suites and the trained
policy are not available, so every array here is drawn from a seeded generator;
the numbers stand in for those rollouts and reproduce none of them.

Nothing in this file evaluates the method: it only draws inputs.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, Optional

import numpy as np


@dataclass(frozen=True)
class RolloutConfig:
    name: str
    n_groups: int
    G: int
    N: int                 # chunks per trajectory
    K: int                 # phases
    B: int                 # kept chunks per trajectory
    d: int                 # trunk hidden size
    ff: int                # gated-MLP inner size
    V: int = 256           # action bins
    L: int = 8             # steps per chunk
    D: int = 7             # action dims per step
    dtype: str = "bf16"    # "f32" or "bf16": storage type of hidden states / weights
    seed: int = 0
    div_lo: int = 1        # number of divergent phases (lo..hi, drawn per group if per_group_div)
    div_hi: int = 1
    per_group_div: bool = False
    success: str = "forced_mixed"   # "forced_mixed" | "group_rate" | "quarter_collapsed"
    phases: str = "uniform_cuts"    # "uniform_cuts" | "dirichlet"
    gap: str = "fixed"              # "fixed" (0.5) | "lognormal" (0.05*exp(1.5 z))
    n_steps: int = 1

    @property
    def T(self) -> int:
        return self.n_groups * self.G

    @property
    def A(self) -> int:
        return self.L * self.D

    def with_(self, **kw) -> "RolloutConfig":
        return replace(self, **kw)


CONFIGS: Dict[str, RolloutConfig] = {
    # tiny fp32 instance
    "cfg1": RolloutConfig("cfg1", n_groups=2, G=8, N=32, K=4, B=6, d=256, ff=1024,
                          dtype="f32", seed=0, div_lo=1, div_hi=1),
    # LIBERO-shaped bf16 instance, 10 consecutive steps of keep-probability updates
    "cfg2": RolloutConfig("cfg2", n_groups=8, G=8, N=64, K=5, B=12, d=4096, ff=11008,
                          dtype="bf16", seed=2, div_lo=2, div_hi=2, n_steps=10),
    # same data, every chunk kept (unmasked GRPO)
    "cfg3": RolloutConfig("cfg3", n_groups=8, G=8, N=64, K=5, B=64, d=4096, ff=11008,
                          dtype="bf16", seed=2, div_lo=2, div_hi=2, n_steps=10),
    # larger batch, divergent set varies per task, per-group success rate
    "cfg4": RolloutConfig("cfg4", n_groups=32, G=8, N=128, K=8, B=16, d=4096, ff=11008,
                          dtype="bf16", seed=4, div_lo=1, div_hi=3, per_group_div=True,
                          success="group_rate"),
    # skewed long-horizon stress
    "cfg5": RolloutConfig("cfg5", n_groups=64, G=8, N=256, K=12, B=24, d=4096, ff=11008,
                          dtype="bf16", seed=5, success="quarter_collapsed",
                          phases="dirichlet", gap="lognormal"),
}


def _rng(*key) -> np.random.Generator:
    return np.random.default_rng(np.random.SeedSequence([int(k) & 0xFFFFFFFF for k in key]))


def _task_structure(cfg: RolloutConfig):
    """Per-task quantities that persist across steps: action means and gaps."""
    r = _rng(cfg.seed, 0xA11CE)
    mean = r.uniform(-0.5, 0.5, size=(cfg.n_groups, cfg.K, cfg.A))
    gap = np.zeros((cfg.n_groups, cfg.K))
    if cfg.gap == "lognormal":
        z = r.standard_normal(cfg.K)
        gap[:] = 0.05 * np.exp(1.5 * z)[None, :]
    else:
        if cfg.per_group_div:
            for g in range(cfg.n_groups):
                n_div = int(r.integers(cfg.div_lo, cfg.div_hi + 1))
                gap[g, r.choice(cfg.K, size=n_div, replace=False)] = 0.5
        else:
            n_div = int(r.integers(cfg.div_lo, cfg.div_hi + 1))
            gap[:, r.choice(cfg.K, size=n_div, replace=False)] = 0.5
    return mean, gap


def _draw_rewards(cfg: RolloutConfig, r: np.random.Generator) -> np.ndarray:
    T, G = cfg.T, cfg.G
    reward = np.zeros(T, dtype=np.uint8)
    if cfg.success == "group_rate":
        for g in range(cfg.n_groups):
            q = r.uniform(0.1, 0.9)
            reward[g * G:(g + 1) * G] = r.random(G) < q
        return reward
    collapsed = np.zeros(cfg.n_groups, dtype=bool)
    if cfg.success == "quarter_collapsed":
        collapsed[r.choice(cfg.n_groups, size=cfg.n_groups // 4, replace=False)] = True
    for g in range(cfg.n_groups):
        if collapsed[g]:
            reward[g * G:(g + 1) * G] = int(r.integers(0, 2))
            continue
        while True:
            draw = r.random(G) < 0.5
            if 0 < draw.sum() < G:
                break
        reward[g * G:(g + 1) * G] = draw
    return reward


def _draw_phases(cfg: RolloutConfig, r: np.random.Generator) -> np.ndarray:
    T, N, K = cfg.T, cfg.N, cfg.K
    phase = np.zeros((T, N), dtype=np.uint8)
    for i in range(T):
        if cfg.phases == "dirichlet":
            w = r.dirichlet(np.full(K, 0.5))
            length = np.floor(w * N).astype(np.int64)
            # hand the remainder to the largest fractional parts so lengths sum to N
            rest = N - int(length.sum())
            order = np.argsort(-(w * N - length), kind="stable")
            length[order[:rest]] += 1
        else:
            cuts = np.sort(r.choice(np.arange(1, N), size=min(K - 1, N - 1), replace=False))
            edges = np.concatenate(([0], cuts, [N]))
            length = np.diff(edges)
            if len(length) < K:
                length = np.concatenate((length, np.zeros(K - len(length), dtype=length.dtype)))
        phase[i] = np.repeat(np.arange(K, dtype=np.uint8), length)
    return phase


def make_rollouts(cfg: RolloutConfig, step: int = 0) -> Dict[str, np.ndarray]:
    """One step's rollout batch.

    Returns reward u8[T], phase u8[T,N], actions f32[T,N,A] in [-1,1],
    tokens u8[T,N,A] (256-bin index of each action value), n_chunks i32[T].
    """
    mean, gap = _task_structure(cfg)
    r = _rng(cfg.seed, 0xB0B, step)
    reward = _draw_rewards(cfg, r)
    phase = _draw_phases(cfg, r)
    T, N, A, G = cfg.T, cfg.N, cfg.A, cfg.G
    group = np.repeat(np.arange(cfg.n_groups), G)
    sign = np.where(reward == 1, 0.5, -0.5)
    centre = mean[group[:, None], phase] + (sign[:, None] * gap[group[:, None], phase])[..., None]
    actions = centre + 0.1 * r.standard_normal((T, N, A))
    actions = np.clip(actions, -1.0, 1.0).astype(np.float32)
    tokens = np.minimum(255, np.floor((actions.astype(np.float64) + 1.0) * 128.0)).astype(np.uint8)
    n_chunks = np.full(T, N, dtype=np.int32)
    return {"reward": reward, "phase": phase, "actions": actions, "tokens": tokens,
            "n_chunks": n_chunks, "divergent": gap}


def make_gripper_actions(cfg: RolloutConfig, step: int = 0) -> np.ndarray:
    """Continuous actions [T, N, L*D] whose last dimension is a gripper command in {-1 (open), +1 (close)}
    with manipulation-like structure: per trajectory zero, one or two grasp cycles (open approach, a few
    chunks in which the command starts to flicker closed, a held grasp with occasional drop-outs, a release
    with flicker, an open tail), plus 3 % random flips of single timesteps.  Other dimensions are noise."""
    r = _rng(cfg.seed, 0x6A1B, step)
    T, N, L, D = cfg.T, cfg.N, cfg.L, cfg.D
    a = r.uniform(-1, 1, size=(T, N, L, D)).astype(np.float32)
    close_prob = np.zeros((T, N))
    for i in range(T):
        cycles = int(r.integers(0, 3))
        pos = int(r.integers(1, max(2, N // 4)))
        for _ in range(cycles):
            ramp = int(r.integers(0, 4))
            hold = int(r.integers(1, max(2, N // 4)))
            release = int(r.integers(0, 4))
            for k in range(ramp):
                if pos + k < N:
                    close_prob[i, pos + k] = r.uniform(0.05, 0.6)
            pos += ramp
            close_prob[i, pos:pos + hold] = r.uniform(0.7, 1.0, size=len(close_prob[i, pos:pos + hold]))
            pos += hold
            for k in range(release):
                if pos + k < N:
                    close_prob[i, pos + k] = r.uniform(0.0, 0.6)
            pos += release + int(r.integers(0, max(1, N // 6)))
            if pos >= N:
                break
    cmd = r.random((T, N, L)) < close_prob[:, :, None]
    cmd ^= r.random((T, N, L)) < 0.03
    a[..., D - 1] = np.where(cmd, 1.0, -1.0)
    return a.reshape(T, N, L * D)


def ragged_n_chunks(cfg: RolloutConfig, salt: int = 0) -> np.ndarray:
    """Per-trajectory valid chunk counts in [0, N], including 0, values below B and N."""
    r = _rng(cfg.seed, 0xC0DE, salt)
    n = r.integers(0, cfg.N + 1, size=cfg.T).astype(np.int32)
    if cfg.T >= 4:
        n[0], n[1], n[2], n[3] = cfg.N, 0, max(1, cfg.B - 1), min(cfg.N, cfg.B)
    return n


# --------------------------------------------------------------------------------------
# policy-head tensors
# --------------------------------------------------------------------------------------

def to_bf16_grid(x: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bf16-representable value (ties to even), as fp32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    bits = x.view(np.uint32).astype(np.uint64)
    bits = (bits + 0x7FFF + ((bits >> 16) & 1)) & 0xFFFF0000
    return bits.astype(np.uint32).view(np.float32).reshape(x.shape)


def make_hidden_numpy(cfg: RolloutConfig, step: int = 0) -> np.ndarray:
    """Trunk hidden states h ~ N(0,1), [T*N*A, d] fp32 (on the bf16 grid for bf16 configs)."""
    r = _rng(cfg.seed, 0xD00D, step)
    h = r.standard_normal((cfg.T * cfg.N * cfg.A, cfg.d), dtype=np.float32)
    return to_bf16_grid(h) if cfg.dtype == "bf16" else h


def make_head_numpy(cfg: RolloutConfig, std: float = 0.02) -> Dict[str, np.ndarray]:
    """Gated-MLP head weights, stored [in, out] row-major: Wg,Wu [d,ff], Wd [ff,d], Wo [d,V]."""
    r = _rng(cfg.seed, 0xFEED)
    w = {
        "Wg": r.standard_normal((cfg.d, cfg.ff), dtype=np.float32) * np.float32(std),
        "Wu": r.standard_normal((cfg.d, cfg.ff), dtype=np.float32) * np.float32(std),
        "Wd": r.standard_normal((cfg.ff, cfg.d), dtype=np.float32) * np.float32(std),
        "Wo": r.standard_normal((cfg.d, cfg.V), dtype=np.float32) * np.float32(std),
    }
    if cfg.dtype == "bf16":
        w = {k: to_bf16_grid(v) for k, v in w.items()}
    return w


def perturb_numpy(cfg: RolloutConfig, w: Dict[str, np.ndarray], std: float = 0.01) -> Dict[str, np.ndarray]:
    """Old-policy weights: current weights plus N(0, std) noise."""
    r = _rng(cfg.seed, 0x01D)
    out = {k: v + r.standard_normal(v.shape, dtype=np.float32) * np.float32(std) for k, v in w.items()}
    if cfg.dtype == "bf16":
        out = {k: to_bf16_grid(v) for k, v in out.items()}
    return out


def _torch_dtype(cfg: RolloutConfig):
    import torch
    return torch.bfloat16 if cfg.dtype == "bf16" else torch.float32


def make_hidden_torch(cfg: RolloutConfig, device, step: int = 0, rows: Optional[int] = None):
    """Device-side hidden states for sizes too large to draw on the host; N(0,1), seeded."""
    import torch
    gen = torch.Generator(device=device)
    gen.manual_seed((cfg.seed << 20) ^ 0xD00D ^ (step << 8))
    n_rows = cfg.T * cfg.N * cfg.A if rows is None else rows
    out = torch.empty((n_rows, cfg.d), dtype=_torch_dtype(cfg), device=device)
    blk = 1 << 15
    for r0 in range(0, n_rows, blk):
        r1 = min(n_rows, r0 + blk)
        out[r0:r1] = torch.randn((r1 - r0, cfg.d), generator=gen, device=device,
                                 dtype=torch.float32).to(out.dtype)
    return out


def make_head_torch(cfg: RolloutConfig, device, std: float = 0.02):
    import torch
    gen = torch.Generator(device=device)
    gen.manual_seed((cfg.seed << 20) ^ 0xFEED)
    dt = _torch_dtype(cfg)
    shapes = {"Wg": (cfg.d, cfg.ff), "Wu": (cfg.d, cfg.ff), "Wd": (cfg.ff, cfg.d), "Wo": (cfg.d, cfg.V)}
    return {k: (torch.randn(s, generator=gen, device=device, dtype=torch.float32) * std).to(dt)
            for k, s in shapes.items()}


def perturb_torch(cfg: RolloutConfig, w, std: float = 0.01):
    import torch
    out = {}
    for k, v in w.items():
        gen = torch.Generator(device=v.device)
        gen.manual_seed((cfg.seed << 20) ^ 0x01D ^ (len(out) << 4))
        noise = torch.randn(v.shape, generator=gen, device=v.device, dtype=torch.float32) * std
        out[k] = (v.float() + noise).to(v.dtype)
    return out
