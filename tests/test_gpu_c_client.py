"""The C boundary without PyTorch: tests/c/gpu_client.cpp (HIP runtime for memory, the library's C calls for
everything else) runs one training step on inputs made from a counter hash; the same inputs are rebuilt here in
numpy and go through the Python binding (same kernels: identical results expected) and through the CPU checker."""
import json
import os
import subprocess

import numpy as np
import pytest
import torch

from oracle import pcm_oracle as O

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CLIENT = os.path.join(ROOT, "tests", "c", "gpu_client")


def unit(stream, n):
    """The client's value in [-0.5, 0.5) for indices 0 .. n-1 of a stream (float32)."""
    i = np.arange(n, dtype=np.uint64)
    x = ((i * np.uint64(2654435761)) & np.uint64(0xFFFFFFFF)).astype(np.uint32) ^ np.uint32((stream * 0x9E3779B9) & 0xFFFFFFFF)
    x ^= x >> np.uint32(16)
    x *= np.uint32(0x7FEB352D)
    x ^= x >> np.uint32(15)
    x *= np.uint32(0x846CA68B)
    x ^= x >> np.uint32(16)
    return (x >> np.uint32(8)).astype(np.float32) / np.float32(16777216.0) - np.float32(0.5)


def test_c_client_matches_binding_and_checker():
    import paper_2605_16154_amd as pcm
    if not os.path.exists(CLIENT):                      # normally built beforehand by build()
        from paper_2605_16154_amd.build import build_c_client
        build_c_client()
    r = subprocess.run([CLIENT], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, (r.returncode, r.stdout, r.stderr)
    got = json.loads(r.stdout.strip().splitlines()[-1])

    n_groups, G, N, A, K, B, d, ff, V = 2, 4, 8, 56, 3, 4, 256, 256, 256
    T = n_groups * G
    rows_all = T * N * A
    phase = np.tile((np.arange(N) * K // N).astype(np.uint8), (T, 1))
    reward = np.array([1 if (i % G) < 2 else 0 for i in range(T)], np.uint8)
    actions = (np.float32(2.0) * unit(1, T * N * A)).reshape(T, N, A)
    shift = (reward[:, None] == 1) & (phase == 1)
    actions[shift] += np.float32(0.25)
    tokens = ((unit(2, rows_all) + np.float32(0.5)) * np.float32(256.0)).astype(np.uint8)
    hidden = (np.float32(2.0) * unit(3, rows_all * d)).reshape(rows_all, d)
    W = {k: (np.float32(0.15) * unit(s, a * b)).reshape(a, b)
         for k, s, a, b in (("Wg", 4, d, ff), ("Wu", 5, d, ff), ("Wd", 6, ff, d), ("Wo", 7, d, V))}
    logp_old = np.float32(-5.545) + np.float32(0.6) * unit(8, rows_all)

    # the checker on the same inputs (bf16-rounded where the client rounds)
    dev = torch.device("cuda:0")
    t = lambda x: torch.from_numpy(np.ascontiguousarray(x)).to(dev)
    bf = lambda x: t(x).to(torch.bfloat16)
    rounded = lambda x: bf(x).float().cpu().numpy().astype(np.float64)
    adv_o, active_o = O.advantages(reward, G)
    C_o, valid_o = O.phase_scores(actions, phase, reward, None, n_groups, G, K)
    p_o = O.KeepProbState(K).update(C_o, valid_o)
    kept_o, _, nk_o = O.sample_chunks(p_o, phase, None, active_o, B, seed=77, step=0)
    assert np.array_equal(np.array(got["C"]).view(np.int64), C_o.view(np.int64))
    assert np.array_equal(np.array(got["p"]).view(np.int64), p_o.view(np.int64))
    assert got["n_kept"] == nk_o and got["kept"] == list(kept_o)
    ref = O.actor_step(rounded(hidden), tokens, logp_old.astype(np.float64), adv_o, kept_o, N, A,
                       *(rounded(W[k]) for k in ("Wg", "Wu", "Wd", "Wo")), 0.2, 0.4, 1.0 / T)
    assert 0.05 < ref["stats"][0] < 0.95
    assert abs(got["loss"] - ref["loss"]) <= 3e-2 * max(1.0, abs(ref["loss"])), (got["loss"], ref["loss"])
    assert abs(got["clip_fraction"] - ref["stats"][0]) <= 2e-2 and got["rows"] == nk_o * A
    for name, key in (("dWo", "dWo_sumsq"), ("dWg", "dWg_sumsq")):
        want = float((ref[name] ** 2).sum())
        assert abs(got[key] - want) <= 6e-2 * want, (name, got[key], want)

    # the Python binding on the same inputs: the same library calls, so the same numbers
    Cc, valid, adv, active = pcm.pcm_score_phases(t(actions), t(phase), t(reward), None, n_groups, G, K)
    state = pcm.pcm_state_init(K, dev)
    p = pcm.pcm_update_keep_probs(state, Cc, valid, 0.1, 5)
    kept, _, nk = pcm.pcm_sample_chunks(p, t(phase), None, active, B, 77, 0)
    out = pcm.grpo_masked_actor_step(bf(hidden), t(tokens), t(logp_old), adv, kept, nk, T, N, A,
                                     *(bf(W[k]) for k in ("Wg", "Wu", "Wd", "Wo")), 0.2, 0.4, 1.0 / T)
    torch.cuda.synchronize()
    assert np.float32(got["loss"]) == out["loss"].cpu().numpy()[0]
    assert abs(got["dWo_sumsq"] - float((out["dWo"].double() ** 2).sum().item())) <= 1e-9 * got["dWo_sumsq"]
    assert abs(got["dWg_sumsq"] - float((out["dWg"].double() ** 2).sum().item())) <= 1e-9 * got["dWg_sumsq"]
