#!/usr/bin/env python3
"""Throughput of the PCM hot path on one MI355X: kept action tokens per second.

One step = one pass of the whole path over one synthetic rollout batch that is already resident
in HBM: pcm_score_phases -> pcm_update_keep_probs -> pcm_sample_chunks -> grpo_masked_actor_step
(gather, head forward, fused clipped-GRPO loss, full backward), all through the C-ABI library.
Prints one JSON line: metric, value, ms_per_step (mean, median, min), roofline of the dominant GEMM, per-stage
times, the unmasked step for the masking speed-up, timings of the loss variants and the optimizer step, and the
CPU checker timed on the host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np

MFMA_BF16_PEAK_TFLOPS = 2500.0      # MI355X dense bf16 matrix peak
ALU_FP32_PEAK_TFLOPS = 157.3
HBM_PEAK_GBPS = 8000.0              # MI355X HBM3E peak
GEMM_STAGES = ("gemm_gate_up", "gemm_down", "gemm_logits_loss", "gemm_dWo", "gemm_dy", "gemm_dWd", "gemm_da",
               "gemm_dWg_dWu", "gemm_dX")


def stored_traffic(name):
    """HBM-side bytes per launch from the committed counter summary, or None if the kernel changed since."""
    path = os.path.join(ROOT, "profiles", name)
    if not os.path.exists(path):
        return None
    kv = dict(line.strip().split("=", 1) for line in open(path) if "=" in line and not line.startswith("#"))
    from paper_2605_16154_amd.profile_summary import kernel_source_hash
    if kv.get("source_hash") != kernel_source_hash():
        return None
    try:
        return (float(kv["fetch_kib_per_launch"]) * float(kv["scale_fetch"]) +
                float(kv["write_kib_per_launch"]) * float(kv["scale_write"])) * 1024.0
    except (KeyError, ValueError):
        return None


def gemm_flops_per_step(M, d, ff, V, M_bwd=None):
    """Flops per step of each head GEMM stage (all its launches: one per row panel, two for dWg and dWu): the forward
    products over M token rows, the backward products over M_bwd rows (those the library ran them over; M if not
    given).  2 flops per multiply-add."""
    B = M if M_bwd is None else M_bwd
    return {"gemm_gate_up": 2.0 * M * d * 2 * ff, "gemm_down": 2.0 * M * ff * d, "gemm_logits_loss": 2.0 * M * d * V,
            "gemm_dWo": 2.0 * B * d * V, "gemm_dy": 2.0 * B * V * d, "gemm_dWd": 2.0 * B * ff * d,
            "gemm_da": 2.0 * B * d * ff, "gemm_dWg_dWu": 2 * 2.0 * B * d * ff, "gemm_dX": 2.0 * B * 2 * ff * d}


def backward_rows(rows, clip_fractions, dense):
    """Mean number of rows the backward products ran over: the library drops the rows whose gradient the clip
    removes when they are at least one in sixteen (kept chunks of active groups have a non-zero advantage, so in a
    one-panel batch those are all the rows it drops)."""
    if dense or not clip_fractions:
        return float(rows)
    return float(np.mean([rows * (1.0 - c) if c >= 1.0 / 16 else rows for c in clip_fractions]))


class Workload:
    """Device-resident inputs of `n_batches` consecutive training steps plus the head."""

    def __init__(self, cfg, device, n_batches, policy_drift=0.01, dense_backward=False):
        import torch
        from workloads import make_head_torch, make_hidden_torch, make_rollouts, perturb_torch
        import paper_2605_16154_amd as pcm
        self.cfg, self.dev, self.pcm, self.torch = cfg, device, pcm, torch
        t = lambda x: torch.from_numpy(np.ascontiguousarray(x)).to(device)
        self.host = [make_rollouts(cfg, s) for s in range(n_batches)]
        self.batches = [{k: t(ro[k]) for k in ("actions", "phase", "reward", "n_chunks")} for ro in self.host]
        for b, ro in zip(self.batches, self.host):
            b["tokens"] = t(ro["tokens"].reshape(-1))
        self.hidden = make_hidden_torch(cfg, device)
        self.W = make_head_torch(cfg, device)
        self.set_old_policy(policy_drift)
        self.dense_backward = dense_backward
        self.state = pcm.pcm_state_init(cfg.K, device)
        # the forward products' operand layouts of the weights, written once: they change with the weights (once per
        # optimizer step), not with the batch
        self.packed = pcm.pcm_pack_head_weights(self.W["Wg"], self.W["Wu"], self.W["Wd"], self.W["Wo"]) if cfg.dtype == "bf16" else None
        self.sel_out = None
        self.samp_out = None
        self.act_out = {}
        torch.cuda.synchronize()

    def set_old_policy(self, policy_drift):
        """Old-policy log-probabilities of every action token from weights `policy_drift` (noise standard deviation)
        away from the current ones."""
        from workloads import perturb_torch
        cfg, pcm, torch, device = self.cfg, self.pcm, self.torch, self.dev
        W_old = perturb_torch(cfg, self.W, std=policy_drift)
        # old-policy log-probabilities of every action token: forward-only passes with the old weights,
        # T*B chunks at a time (the same launch shape as the timed step)
        per_call = cfg.T * min(cfg.B, cfg.N)
        n_all = cfg.T * cfg.N
        zeros = torch.zeros(n_all * cfg.A, dtype=torch.float32, device=device)
        adv0 = torch.zeros(cfg.T, dtype=torch.float32, device=device)
        for b in self.batches:
            b["logp_old"] = torch.empty(n_all * cfg.A, dtype=torch.float32, device=device)
            for c0 in range(0, n_all, per_call):
                c0 = min(c0, n_all - per_call)          # the last call overlaps the previous one: all calls are full
                n = per_call
                idx = torch.arange(c0, c0 + n, dtype=torch.int32, device=device)
                out = pcm.grpo_masked_actor_step(self.hidden, b["tokens"], zeros, adv0, idx,
                                                 torch.tensor([n], dtype=torch.int32, device=device), cfg.T, cfg.N,
                                                 cfg.A, W_old["Wg"], W_old["Wu"], W_old["Wd"], W_old["Wo"],
                                                 want_grads=False, want_dX=False)
                b["logp_old"][c0 * cfg.A:(c0 + n) * cfg.A] = out["logp"][:n * cfg.A]
        del W_old, zeros
        torch.cuda.synchronize()

    def step(self, t, B=None, **loss_variants):
        cfg, pcm, b = self.cfg, self.pcm, self.batches[t % len(self.batches)]
        B = cfg.B if B is None else B
        self.sel_out = pcm.pcm_score_phases(b["actions"], b["phase"], b["reward"], b["n_chunks"], cfg.n_groups,
                                            cfg.G, cfg.K, 1e-6, out=self.sel_out)
        Cc, valid, adv, active = self.sel_out
        p = pcm.pcm_update_keep_probs(self.state, Cc, valid, 0.1, 5)
        if self.samp_out is not None and self.samp_out[0].shape[0] != cfg.T * min(B, cfg.N):
            self.samp_out, self.act_out = None, {}
        self.samp_out = pcm.pcm_sample_chunks(p, b["phase"], b["n_chunks"], active, B, cfg.seed, t, out=self.samp_out)
        kept, off, nk = self.samp_out
        self.act_out = pcm.grpo_masked_actor_step(self.hidden, b["tokens"], b["logp_old"], adv, kept, nk, cfg.T, cfg.N,
                                                  cfg.A, self.W["Wg"], self.W["Wu"], self.W["Wd"], self.W["Wo"],
                                                  0.2, 0.4, 1.0 / cfg.T, out=self.act_out,
                                                  packed_weights=None if loss_variants.get("composed_head") else self.packed,
                                                  dense_backward=self.dense_backward, **loss_variants)
        return nk


def timed_steps(wl, steps, warmup, B=None, profile=False, **loss_variants):
    torch = wl.torch
    for t in range(warmup):
        wl.step(t, B, **loss_variants)
    torch.cuda.synchronize()
    if profile:
        wl.pcm.pcm_profile_enable(True)
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    clip = torch.zeros(steps, device=wl.dev) if profile else None
    t0 = time.perf_counter()
    marks[0].record()
    for t in range(warmup, warmup + steps):
        nk = wl.step(t, B, **loss_variants)
        if profile:
            clip[t - warmup] = wl.act_out["stats"][0]      # device-side copy, no synchronisation
        marks[t - warmup + 1].record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    wl.clip_fractions = clip.cpu().tolist() if profile else []
    wl.step_ms = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(steps))   # per-step device time
    stages = None
    if profile:
        stages = wl.pcm.pcm_profile_collect()
        wl.pcm.pcm_profile_enable(False)
    return dt, int(nk.item()), stages


def cpu_baseline(wl, kept_host, sample_chunks):
    """The CPU checker, as it stands, on a bounded sample of the same step."""
    from oracle import pcm_oracle as O
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    cfg, ro = wl.cfg, wl.host[0]
    t0 = time.perf_counter()
    adv, active = O.advantages(ro["reward"], cfg.G)
    C, valid = O.phase_scores(ro["actions"], ro["phase"], ro["reward"], ro["n_chunks"], cfg.n_groups, cfg.G, cfg.K)
    p = O.KeepProbState(cfg.K).update(C, valid)
    kept, off, nk = O.sample_chunks(p, ro["phase"], ro["n_chunks"], active, cfg.B, cfg.seed, 0)
    t_sel = time.perf_counter() - t0
    assert np.array_equal(kept, kept_host), "GPU and CPU selection disagree"
    pick = kept[:sample_chunks]
    rows = (pick[:, None].astype(np.int64) * cfg.A + np.arange(cfg.A)[None, :]).reshape(-1)
    torch = wl.torch
    ridx = torch.from_numpy(rows).to(wl.dev)
    hid = wl.hidden[ridx].float().cpu().numpy()
    tok = ro["tokens"].reshape(-1)[rows]
    lp_old = wl.batches[0]["logp_old"][ridx].cpu().numpy()
    W = {k: v.float().cpu().numpy() for k, v in wl.W.items()}
    t0 = time.perf_counter()
    O.actor_step(hid, tok, lp_old, adv[pick // cfg.N], np.arange(len(pick)), 1, cfg.A, W["Wg"], W["Wu"], W["Wd"], W["Wo"],
                 0.2, 0.4, 1.0 / cfg.T)
    t_act = time.perf_counter() - t0
    rows_step = nk * cfg.A
    est_step = t_sel + t_act * rows_step / len(rows)
    return {"value": rows_step / est_step, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"selection stages in full ({t_sel:.2f} s) + fp64 actor step on the first {len(pick)} kept chunks "
                      f"({len(rows)} of {rows_step} rows, {t_act:.2f} s), scaled linearly in rows"}


def selection_only(cfg, dev, steps, warmup):
    """Times the three selection calls alone (any configuration; no hidden states or weights needed), preceded by the
    phase labeler on gripper-structured actions of the same shape."""
    import torch
    import paper_2605_16154_amd as pcm
    from workloads import make_rollouts
    ro = make_rollouts(cfg, 0)
    t = lambda x: torch.from_numpy(np.ascontiguousarray(x)).to(dev)
    actions, phase, reward, n_chunks = t(ro["actions"]), t(ro["phase"]), t(ro["reward"]), t(ro["n_chunks"])
    state = pcm.pcm_state_init(cfg.K, dev)
    sel = samp = None
    from workloads import make_gripper_actions
    grip = t(make_gripper_actions(cfg, 0))
    labels = torch.empty((cfg.T, cfg.N), dtype=torch.uint8, device=dev)

    def one(step):
        nonlocal sel, samp
        pcm.pcm_label_phases(grip, n_chunks, cfg.L, cfg.D, out=labels)
        sel = pcm.pcm_score_phases(actions, phase, reward, n_chunks, cfg.n_groups, cfg.G, cfg.K, 1e-6, out=sel)
        p = pcm.pcm_update_keep_probs(state, sel[0], sel[1], 0.1, 5)
        samp = pcm.pcm_sample_chunks(p, phase, n_chunks, sel[3], cfg.B, cfg.seed, step, out=samp)

    for s in range(warmup):
        one(s)
    copy_dst = torch.empty_like(actions)
    torch.cuda.synchronize()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    ev[0].record()
    for _ in range(steps):
        copy_dst.copy_(actions)
    ev[1].record()
    torch.cuda.synchronize()
    copy_us = ev[0].elapsed_time(ev[1]) * 1e3 / steps
    pcm.pcm_profile_enable(True)
    t0 = time.perf_counter()
    for s in range(warmup, warmup + steps):
        one(s)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    stages = pcm.pcm_profile_collect()
    pcm.pcm_profile_enable(False)
    n_kept = int(samp[2].item())
    chunks = cfg.T * cfg.N
    alg_bytes = {"score_accumulate": chunks * (cfg.A * 4 + 1) + cfg.T, "sample_compact": chunks + 4 * n_kept + 4 * cfg.T,
                 "label_phases": chunks * (cfg.A * 4 + 1)}     # the gripper values sit 4 D bytes apart: whole sectors move
    out = {}
    for name, (ms, n) in stages.items():
        if n == 0:
            continue
        us = ms / n * 1e3
        out[name] = {"us_per_launch": us}
        if name in alg_bytes:
            out[name]["algorithmic_bytes"] = alg_bytes[name]
            out[name]["GB_per_s"] = alg_bytes[name] / us / 1e3
            out[name]["frac_of_8TBps"] = alg_bytes[name] / us / 1e3 / 8000.0
    return {"workload": f"{cfg.name} selection only: T={cfg.T}, N={cfg.N}, K={cfg.K}, B={cfg.B}",
            "us_per_selection_step_wall": dt / steps * 1e6, "kept_chunks": n_kept, "kernels": out,
            "same_size_device_copy": {"bytes_each_way": actions.numel() * 4, "us": copy_us,
                                      "GB_per_s": 2 * actions.numel() * 4 / copy_us / 1e3}}


def board_power_and_clock(work, seconds=2.0):
    """Board power (watts) and shader clock (MHz) read from the driver's hwmon files while `work(deadline)` keeps
    the GPU busy for about `seconds`: shows whether a load runs into the board's power cap, and at what clock.
    Plain file reads from a thread of this process; no child processes."""
    import glob
    import threading
    base = "/sys/class/drm/card*/device/hwmon/hwmon*/"
    first = lambda pat: (sorted(glob.glob(base + pat)) or [None])[0]
    f_power = first("power1_input") or first("power1_average")
    f_clock, f_cap = first("freq1_input"), first("power1_cap")
    watts, mhz, stop = [], [], threading.Event()

    def read(path, scale):
        try:
            return int(open(path).read()) / scale
        except (OSError, ValueError):
            return None

    def sample():
        time.sleep(0.5)                          # let the load settle
        while not stop.is_set():
            w = read(f_power, 1e6) if f_power else None
            c = read(f_clock, 1e6) if f_clock else None
            if w is not None:
                watts.append(w)
            if c is not None:
                mhz.append(c)
            time.sleep(0.02)

    th = threading.Thread(target=sample, daemon=True)
    th.start()
    work(time.perf_counter() + seconds)
    stop.set()
    th.join(timeout=5)
    mean = lambda v: sum(v) / len(v) if v else None
    return {"board_power_w": mean(watts), "shader_clock_mhz": mean(mhz), "samples": len(watts),
            "power_cap_w": read(f_cap, 1e6) if f_cap else None}


def graph_replay_timing(wl, steps):
    """The same steps replayed from HIP graphs (one graph per resident batch, captured once): what is left when the
    launch gaps between the ~30 kernels of a step are gone.  Reported beside `value`, which stays the eager figure."""
    torch, pcm, cfg = wl.torch, wl.pcm, wl.cfg
    n = len(wl.batches)
    wl.state = pcm.pcm_state_init(cfg.K, wl.dev)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graphs = []
    with torch.cuda.stream(side):
        for t in range(n):
            wl.step(t)                              # sizes buffers and workspace on the capture stream
        torch.cuda.synchronize()
        for t in range(n):
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=side):
                wl.step(t)
            graphs.append(g)
    torch.cuda.current_stream().wait_stream(side)
    for t in range(3):
        graphs[t % n].replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for t in range(steps):
        graphs[t % n].replay()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    return {"ms_per_step": dt / steps * 1e3, "graphs": n,
            "note": "each graph replays its batch with the step index it was captured with"}


def vendor_yardstick(wl, rows, iters=20):
    """The vendor BLAS (through torch.matmul) on the gate/up shape with operands of the same distribution: a yardstick
    for what this chip sustains on that shape with a plain bf16 store, never a dependency of the library.  Timed over
    `iters` launches after a warm-up; reported beside `value`, never part of it."""
    torch, cfg = wl.torch, wl.cfg
    x = wl.hidden[:rows].contiguous()
    w = torch.cat([wl.W["Wg"], wl.W["Wu"]], dim=1).t().contiguous()          # [2 ff, d], reduction index contiguous
    out = torch.empty((rows, 2 * cfg.ff), dtype=torch.bfloat16, device=wl.dev)
    for _ in range(5):
        torch.matmul(x, w.t(), out=out)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    ev[0].record()
    for _ in range(iters):
        torch.matmul(x, w.t(), out=out)
    ev[1].record()
    torch.cuda.synchronize()
    ms = ev[0].elapsed_time(ev[1]) / iters
    flops = 2.0 * rows * cfg.d * 2 * cfg.ff
    return {"shape": [rows, 2 * cfg.ff, cfg.d], "ms_per_launch": ms, "tflops": flops / (ms * 1e-3) / 1e12,
            "frac_of_peak": flops / (ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
            "note": "vendor BLAS via torch.matmul, plain bf16 store (no fused activation, one output)"}


def optimizer_step_timing(wl, iters=10):
    """The optimizer step that would follow the actor gradients (App. D: clipping at 2.0 + AdamW), timed on
    the head's real tensors: not part of `value`, reported beside it.  HBM-bound: per parameter the norm pass
    reads 4 B, the update pass reads 16 B (g, m, v, w) and writes 14 B (m, v, w, bf16 copy)."""
    torch, pcm = wl.torch, wl.pcm
    names = ("Wg", "Wu", "Wd", "Wo")
    grads = [wl.act_out["d" + n].reshape(-1) for n in names]
    lowp = [wl.W[n].clone().reshape(-1) for n in names]
    master = [w.float() for w in lowp]
    m = [torch.zeros_like(w) for w in master]
    v = [torch.zeros_like(w) for w in master]
    for t in range(1, 3):
        pcm.pcm_adamw_clip_step(grads, master, m, v, t, weights_bf16=lowp)
    torch.cuda.synchronize()
    pcm.pcm_profile_enable(True)
    for t in range(3, 3 + iters):
        norm = pcm.pcm_adamw_clip_step(grads, master, m, v, t, weights_bf16=lowp)
    torch.cuda.synchronize()
    st = pcm.pcm_profile_collect()
    pcm.pcm_profile_enable(False)
    n_param = sum(w.numel() for w in master)
    ms_norm = st["opt_grad_norm"][0] / iters
    ms_upd = st["opt_adamw"][0] / iters
    # the same with the sum of the squares of the gradients taken from the actor step (it gathers them where it
    # writes the final gradient values): no norm pass; and what asking for that sum costs the actor step
    k = 5
    dt_plain, _, _ = timed_steps(wl, k, 1)
    dt_sq, _, _ = timed_steps(wl, k, 1, grad_sumsq=True)
    sumsq = wl.act_out["grad_sumsq"]
    grads = [wl.act_out["d" + n].reshape(-1) for n in names]
    pcm.pcm_profile_enable(True)
    for t in range(3 + iters, 3 + 2 * iters):
        norm_given = pcm.pcm_adamw_clip_step(grads, master, m, v, t, weights_bf16=lowp, grad_sumsq=sumsq)
    torch.cuda.synchronize()
    st2 = pcm.pcm_profile_collect()
    pcm.pcm_profile_enable(False)
    want = float(torch.stack([(g.double() ** 2).sum() for g in grads]).sum().sqrt().item())
    return {"parameters": n_param, "grad_norm": float(norm.item()), "ms_per_step": ms_norm + ms_upd,
            "grad_norm_pass": {"ms": ms_norm, "bytes": 4 * n_param, "GB_per_s": 4 * n_param / ms_norm / 1e6},
            "adamw_pass": {"ms": ms_upd, "bytes": 30 * n_param, "GB_per_s": 30 * n_param / ms_upd / 1e6,
                           "frac_of_hbm_peak": 30 * n_param / ms_upd / 1e6 / HBM_PEAK_GBPS},
            "with_sum_of_squares_from_actor_step": {
                "ms_per_step": (st2["opt_grad_norm"][0] + st2["opt_adamw"][0]) / iters,
                "norm_stage_ms": st2["opt_grad_norm"][0] / iters,
                "grad_norm": float(norm_given.item()), "grad_norm_recomputed_fp64": want,
                "actor_step_ms_with": dt_sq / k * 1e3, "actor_step_ms_without": dt_plain / k * 1e3}}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="cfg2")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-unmasked", action="store_true")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the legs after the timed steps (stage pass, optimizer step): with --no-unmasked and "
                         "--no-cpu-baseline the timed steps are then the last launches of the process")
    ap.add_argument("--extras", action="store_true",
                    help="also time the loss variants, the composed head evaluation, HIP-graph replay and sample board "
                         "power and clock (none of them enters `value`)")
    ap.add_argument("--yardstick", action="store_true",
                    help="also time the vendor BLAS on the gate/up shape (a yardstick beside the roofline, not part of `value`)")
    ap.add_argument("--cpu-sample-chunks", type=int, default=384)
    ap.add_argument("--dense-backward", action="store_true",
                    help="backward products over all kept rows, also those whose gradient the clip removes")
    ap.add_argument("--policy-drift", type=float, default=0.01,
                    help="standard deviation of the weight noise that separates the old policy (whose log-probabilities "
                         "enter the ratio) from the current one; weights themselves have standard deviation 0.02")
    ap.add_argument("--selection-only", action="store_true",
                    help="time only the three selection calls of --config and print their bytes and GB/s")
    ap.add_argument("--scale-groups", type=int, default=1,
                    help="with --selection-only: multiply the number of groups of --config (same per-trajectory shape), "
                         "to see the bandwidth of the selection kernels on inputs large enough to reach it")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 1 GiB device copy (a known-size reference for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py measures the single-GPU hot path only; run it with --gpus 1 "
              "(sharding over GPUs is a design note, not built)", file=sys.stderr)
        sys.exit(2)

    import torch
    from workloads import CONFIGS
    import paper_2605_16154_amd as pcm
    pcm.lib()                                   # raises if the HIP library has not been built
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    cfg = CONFIGS[args.config]

    if args.selection_only:
        if args.scale_groups > 1:
            cfg = cfg.with_(n_groups=cfg.n_groups * args.scale_groups)
        print(json.dumps(selection_only(cfg, dev, max(args.steps, 50), args.warmup)))
        return
    wl = Workload(cfg, dev, cfg.n_steps, args.policy_drift, args.dense_backward)
    if args.copy_calibration:
        src = torch.zeros(1 << 27, dtype=torch.float64, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.add(src, 1.0, out=dst)      # elementwise kernel on doubles: reads 1 GiB, writes 1 GiB per call
        torch.cuda.synchronize()
        del src, dst
    # step 0 from a fresh state once, to hand its kept set to the CPU baseline for cross-checking
    nk0 = wl.step(0)
    torch.cuda.synchronize()
    kept_host = wl.samp_out[0].cpu().numpy()[:int(nk0.item())]
    wl.state = pcm.pcm_state_init(cfg.K, dev)
    # `value`: the timed steps run with the library's stage timer off (no events, no locks on the call path)
    dt, n_kept, _ = timed_steps(wl, args.steps, args.warmup, profile=False)
    rows = n_kept * cfg.A
    ms_step = dt / args.steps * 1e3
    step_ms = list(wl.step_ms)
    value = rows * args.steps / dt
    # what regime was timed: statistics of the last timed step (fraction of rows whose gradient the clip removes,
    # mean ratio, mean old-minus-new log-probability, rows) and its loss
    st = wl.act_out["stats"].cpu().tolist()
    step_stats = {"clip_fraction": st[0], "mean_ratio": st[1], "mean_logp_old_minus_logp": st[2], "rows": st[3],
                  "loss": float(wl.act_out["loss"].item()), "policy_drift": args.policy_drift}
    # second pass over the same steps with the stage timer on: per-kernel durations (HIP events on the call's stream)
    stage_steps = args.steps if args.no_extras else max(args.steps, 10)
    dt_staged, _, stages = timed_steps(wl, stage_steps, 1, profile=True)

    # what the matrix cores sustain with no memory traffic at all (power-limited; depends on the operand data)
    tf_rand, clk_rand = pcm.pcm_measure_mfma_rate(True, 100)
    tf_zero, clk_zero = pcm.pcm_measure_mfma_rate(False, 100)
    mfma_only = {"random_operands": {"tflops": tf_rand, "clock_ghz": clk_rand},
                 "zero_operands": {"tflops": tf_zero, "clock_ghz": clk_zero}}
    rows_bwd = backward_rows(rows, wl.clip_fractions, args.dense_backward or cfg.dtype != "bf16")
    flops = gemm_flops_per_step(rows, cfg.d, cfg.ff, cfg.V, rows_bwd)
    per_stage = {}
    for name, (ms, launches) in stages.items():
        if launches == 0:
            continue
        per_stage[name] = {"ms_per_launch": ms / launches, "launches_per_step": launches / stage_steps}
        if name in flops:
            per_stage[name]["tflops"] = flops[name] * stage_steps / (ms * 1e-3) / 1e12
    total_flops_step = 3.0 * (6.0 * cfg.d * cfg.ff + 2.0 * cfg.d * cfg.V) * rows           # Eq. 11 over all kept rows
    executed_flops_step = (6.0 * cfg.d * cfg.ff + 2.0 * cfg.d * cfg.V) * (rows + 2.0 * rows_bwd)
    if cfg.dtype == "bf16":
        gemm_ms_step = sum(stages[s][0] for s in GEMM_STAGES) / stage_steps
        dominant = max(GEMM_STAGES, key=lambda s: stages[s][0])
        dom_ms = stages[dominant][0] / stages[dominant][1]
        launches_step = stages[dominant][1] / stage_steps                    # one per row panel
        achieved = flops[dominant] / launches_step / (dom_ms * 1e-3) / 1e12
        roofline = {"bound": "mfma", "kernel": f"gemm_bf16 ({dominant})", "achieved": achieved,
                    "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": achieved / MFMA_BF16_PEAK_TFLOPS,
                    "traffic": stored_traffic("gemm_gate_up_cfg2_traffic.txt") if cfg.name == "cfg2" else None,
                    "flops_per_launch": flops[dominant] / launches_step, "ms_per_launch": dom_ms,
                    "mfma_only_sustained": mfma_only,
                    "frac_of_mfma_only_random": achieved / tf_rand,
                    # executed flops: forward over all kept rows, backward over the rows with a gradient
                    "all_head_gemms": {"tflops": executed_flops_step / (gemm_ms_step * 1e-3) / 1e12,
                                       "frac": executed_flops_step / (gemm_ms_step * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
                                       "ms_per_step": gemm_ms_step, "rows_forward": rows, "rows_backward_mean": rows_bwd,
                                       "tflops_if_all_rows_counted": total_flops_step / (gemm_ms_step * 1e-3) / 1e12}}
    else:
        # fp32 correctness configuration: plain vector-ALU products (forward and backward stages of the fp32 path),
        # against the fp32 vector peak 256 CU x 4 SIMD x 64 lanes x 2 flop x 2.4 GHz
        alu_ms_step = (stages["f32_forward"][0] + stages["f32_backward"][0]) / stage_steps
        achieved = total_flops_step / (alu_ms_step * 1e-3) / 1e12
        roofline = {"bound": "alu", "kernel": "sgemm (fp32 path, forward + backward)", "achieved": achieved,
                    "peak": ALU_FP32_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": achieved / ALU_FP32_PEAK_TFLOPS,
                    "traffic": None, "flops_per_step": total_flops_step, "ms_per_step": alu_ms_step}

    result = {"metric": "kept_action_tokens_per_sec_masked_grpo_actor_step", "value": value, "unit": "tokens/s",
              "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_step,
              "ms_per_step_median": step_ms[len(step_ms) // 2], "ms_per_step_min": step_ms[0],
              "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16" if cfg.dtype == "bf16" else "f32",
              "data": "synthetic",
              "config": {"workload": f"{cfg.name}: {cfg.n_groups} groups x {cfg.G} rollouts, {cfg.N} chunks x {cfg.A} tokens, "
                                     f"K={cfg.K}, B={cfg.B}, head {cfg.d}->{cfg.ff}->{cfg.d}->{cfg.V}",
                         "kept_chunks": n_kept, "kept_rows": rows, "global_batch": cfg.T, "selection_included": True},
              "roofline": roofline, "timed_step_stats": step_stats,
              "stages": per_stage, "stage_pass": {"steps": stage_steps, "ms_per_step": dt_staged / stage_steps * 1e3,
                                                  "note": "stage durations come from a second pass with the stage timer "
                                                          "on; `value` is timed with it off"}}

    if not args.no_unmasked and cfg.B < cfg.N:
        wl.state = pcm.pcm_state_init(cfg.K, dev)
        k_un = max(2, min(4, args.steps))
        dt_un, n_un, _ = timed_steps(wl, k_un, 1, B=cfg.N)
        ms_un = dt_un / k_un * 1e3
        result["unmasked"] = {"ms_per_step": ms_un, "kept_rows": n_un * cfg.A, "tokens_per_s": n_un * cfg.A * k_un / dt_un,
                              "speedup_masked_vs_unmasked": ms_un / ms_step, "ideal": cfg.N / cfg.B,
                              "paper": "4.8x cumulative actor-update time, 2x H100 (Sec. 5.2, Fig. 4c)"}
        # memory of the step beyond its inputs and outputs (the library's workspace: activations of one row panel,
        # operand layouts, row lists), masked against unmasked; the paper's analogue is activation memory (Sec. 5.2)
        code = pcm.PCM_BF16 if cfg.dtype == "bf16" else pcm.PCM_F32
        ws = [pcm.grpo_masked_actor_step_workspace_bytes(cfg.T * b_, cfg.A, cfg.d, cfg.ff, cfg.V, code, True)
              for b_ in (min(cfg.B, cfg.N), cfg.N)]
        result["workspace_bytes"] = {"masked": ws[0], "unmasked": ws[1]}
    if cfg.dtype == "bf16" and args.extras and cfg.B < cfg.N:
        # budget sweep (Sec. 5.3 sweeps B in {8, 12, 16}): step time against kept chunks
        sweep = {}
        for b_ in sorted({max(1, cfg.B * 2 // 3), cfg.B, min(cfg.N, cfg.B * 4 // 3)}):
            wl.state = pcm.pcm_state_init(cfg.K, dev)
            dt_b, n_b, _ = timed_steps(wl, 5, 1, B=b_)
            sweep[str(b_)] = {"ms_per_step": dt_b / 5 * 1e3, "kept_rows": n_b * cfg.A}
        result["budget_sweep"] = sweep
    if cfg.dtype == "bf16" and not args.no_extras:
        # the same step nearer to on-policy: the old policy 20 times closer, so that few ratios leave the clip range
        # and almost no row of the backward products is zero (zero rows cost the matrix cores less power)
        wl.set_old_policy(args.policy_drift / 20)
        wl.state = pcm.pcm_state_init(cfg.K, dev)
        k_n = max(2, min(10, args.steps))
        dt_n, n_n, _ = timed_steps(wl, k_n, 1)
        st_n = wl.act_out["stats"].cpu().tolist()
        result["near_on_policy"] = {"policy_drift": args.policy_drift / 20, "ms_per_step": dt_n / k_n * 1e3,
                                    "tokens_per_s": n_n * cfg.A * k_n / dt_n, "clip_fraction": st_n[0],
                                    "mean_ratio": st_n[1]}
        wl.set_old_policy(args.policy_drift)
        if not args.dense_backward:
            # and in the default regime with every backward product over all kept rows (rows whose gradient the
            # clip removes multiplied through as zeros): what the step costs without that saving
            wl.dense_backward = True
            wl.state = pcm.pcm_state_init(cfg.K, dev)
            dt_d, n_d, _ = timed_steps(wl, k_n, 1)
            wl.dense_backward = False
            result["dense_backward"] = {"ms_per_step": dt_d / k_n * 1e3, "tokens_per_s": n_d * cfg.A * k_n / dt_d}
    if cfg.dtype == "bf16" and args.extras:
        # the same step with the loss of App. D (entropy bonus 1e-3, token-mean normalisation) and with one
        # ratio per chunk: extended entry point, same kernels plus two small ones in the per-chunk case
        wl.state = pcm.pcm_state_init(cfg.K, dev)
        k_v = max(2, min(5, args.steps))
        dt_v, _, _ = timed_steps(wl, k_v, 1, entropy_coef=1e-3, token_mean=True)
        dt_c, _, _ = timed_steps(wl, k_v, 1, entropy_coef=1e-3, token_mean=True, chunk_ratio=True)
        result["loss_variants"] = {"entropy_bonus_token_mean_ms_per_step": dt_v / k_v * 1e3,
                                   "with_per_chunk_ratio_ms_per_step": dt_c / k_v * 1e3}
        # the same step with the down and the logit projection applied as one matrix (PCM_HEAD_COMPOSED): the same
        # loss and gradients, three of the large products replaced by products through the V-wide bottleneck
        wl.state = pcm.pcm_state_init(cfg.K, dev)
        k_h = max(2, min(10, args.steps))
        dt_h, n_h, st_h = timed_steps(wl, k_h, 2, profile=True, composed_head=True)
        rows_h = n_h * cfg.A
        # per row: gate/up, dWg + dWu, dX (4 d ff each) and z, G, da (2 ff V each); per step: W_do, dWd, dWo (2 ff d V each)
        executed = rows_h * (12.0 * cfg.d * cfg.ff + 6.0 * cfg.ff * cfg.V) + 6.0 * cfg.ff * cfg.d * cfg.V
        gemm_ms_h = sum(st_h[s_][0] for s_ in GEMM_STAGES) / k_h
        result["composed_head"] = {
            "ms_per_step": dt_h / k_h * 1e3, "tokens_per_s": rows_h * k_h / dt_h,
            "speedup_vs_as_written": (dt / args.steps) / (dt_h / k_h),
            "executed_flops_per_step": executed, "as_written_flops_per_step": total_flops_step,
            "gemm_ms_per_step": gemm_ms_h, "executed_tflops": executed / (gemm_ms_h * 1e-3) / 1e12,
            "stages_ms_per_step": {n_: st_h[n_][0] / k_h for n_ in st_h if st_h[n_][1]},
            "note": "z = a (Wd Wo); G = a^T dz, dWd = G Wo^T, dWo = Wd^T G, da = dz (Wd Wo)^T; `value` above is the "
                    "evaluation as written"}
        # is the board at its power cap, and at what clock: during the step, and during the matrix-core-only loops
        def steps_until(deadline):
            t = 0
            while time.perf_counter() < deadline:
                for _ in range(5):
                    wl.step(t)
                    t += 1
                torch.cuda.synchronize()
        result["power_and_clock"] = {
            "training_steps": board_power_and_clock(steps_until),
            "mfma_only_random_operands": board_power_and_clock(lambda d: pcm.pcm_measure_mfma_rate(True, 2000)),
            "mfma_only_zero_operands": board_power_and_clock(lambda d: pcm.pcm_measure_mfma_rate(False, 2000))}
        result["hip_graph_replay"] = graph_replay_timing(wl, args.steps)
    if cfg.dtype == "bf16" and not args.no_extras:
        wl.step(0)                                  # leaves fresh gradients of the masked step in wl.act_out
        result["optimizer_step"] = optimizer_step_timing(wl)
    if args.yardstick and cfg.dtype == "bf16":
        result["vendor_blas_yardstick"] = vendor_yardstick(wl, rows)
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(wl, kept_host, args.cpu_sample_chunks)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
