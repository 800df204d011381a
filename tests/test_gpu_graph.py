"""The four calls of a training step under HIP graph capture: they only enqueue kernels on the caller's stream
(no allocation, no synchronisation, no memset nodes), so a captured step replays to the same bits as an eager one.
The graph is replayed several times with eager steps and synchronisations in between, every replay checked."""
import numpy as np
import pytest
import torch

from workloads import CONFIGS, make_head_torch, make_hidden_torch, make_rollouts

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def pcm():
    import paper_2605_16154_amd as m
    m.lib()
    return m


@pytest.mark.parametrize("options", [dict(entropy_coef=1e-3, token_mean=True), dict(grad_sumsq=True)],
                         ids=["entropy_bonus_dense_backward", "backward_over_listed_rows_with_gradient_norm"])
def test_captured_step_replays_bit_for_bit(pcm, options):
    cfg = CONFIGS["cfg2"].with_(n_groups=2, G=4, N=16, K=4, B=5, d=256, ff=512, seed=31)
    dev = torch.device("cuda:0")
    ro = make_rollouts(cfg, 0)
    t = lambda x: torch.from_numpy(np.ascontiguousarray(x)).to(dev)
    actions, phase, reward = t(ro["actions"]), t(ro["phase"]), t(ro["reward"])
    tokens = t(ro["tokens"].reshape(-1))
    hidden = make_hidden_torch(cfg, dev)
    W = make_head_torch(cfg, dev, std=0.05)
    logp_old = torch.full((hidden.shape[0],), -5.5, device=dev)
    state0 = pcm.pcm_state_init(cfg.K, dev)
    state = state0.clone()
    bufs = {"sel": None, "p": torch.empty(cfg.K, dtype=torch.float64, device=dev), "samp": None, "act": {}}

    def step(step_index):
        bufs["sel"] = pcm.pcm_score_phases(actions, phase, reward, None, cfg.n_groups, cfg.G, cfg.K, 1e-6, out=bufs["sel"])
        Cc, valid, adv, active = bufs["sel"]
        p = pcm.pcm_update_keep_probs(state, Cc, valid, 0.1, 5, keep_probs_out=bufs["p"])
        bufs["samp"] = pcm.pcm_sample_chunks(p, phase, None, active, cfg.B, cfg.seed, step_index, out=bufs["samp"])
        kept, off, nk = bufs["samp"]
        bufs["act"] = pcm.grpo_masked_actor_step(hidden, tokens, logp_old, adv, kept, nk, cfg.T, cfg.N, cfg.A, W["Wg"],
                                                 W["Wu"], W["Wd"], W["Wo"], 0.2, 0.4, 1.0 / cfg.T, out=bufs["act"],
                                                 **options)

    def snapshot():
        torch.cuda.synchronize()
        out = {k: v.clone() for k, v in bufs["act"].items()}
        out["kept"], out["n_kept"], out["p"], out["state"] = bufs["samp"][0].clone(), bufs["samp"][2].clone(), bufs["p"].clone(), state.clone()
        return out

    def same(a, b):
        for k in a:
            assert torch.equal(a[k], b[k]), k

    # eager reference (also sizes every output buffer and the workspace before capture)
    state.copy_(state0)
    step(3)
    ref = snapshot()
    assert int(ref["n_kept"].item()) > 0 and ref["dWg"].abs().max().item() > 0
    if "grad_sumsq" in options:      # enough clipped rows for the backward products to run over the listed rows
        assert 1 / 8 < ref["stats"][0].item() < 7 / 8

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    state.copy_(state0)
    with torch.cuda.stream(side):
        step(3)                                            # warm-up on the capture stream
        torch.cuda.synchronize()
        state.copy_(state0)
        with torch.cuda.graph(graph, stream=side):
            step(3)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()

    for replay in range(4):
        for k in ("dWg", "dWu", "dWd", "dWo", "dX", "loss", "logp"):
            bufs["act"][k].fill_(float("nan"))            # a replay must rewrite every output
        state.copy_(state0)
        graph.replay()
        same(ref, snapshot())
        # eager work between replays: a different step index, then the reference step again
        step(7 + replay)
        torch.cuda.synchronize()
        state.copy_(state0)
        step(3)
        same(ref, snapshot())


def test_mfma_rate_measurement_aid(pcm):
    """The matrix cores' own sustained rate: positive, below the nominal peak, and lower on random operands than on
    zeros (the chip is power-limited under matrix load)."""
    tf_zero, clk_zero = pcm.pcm_measure_mfma_rate(False, 30)
    tf_rand, clk_rand = pcm.pcm_measure_mfma_rate(True, 30)
    assert 500.0 < tf_rand <= tf_zero * 1.02 and tf_zero < 2600.0
    assert 0.5 < clk_rand <= clk_zero * 1.02 and clk_zero < 2.6
    with pytest.raises(pcm.PcmError):
        pcm.pcm_measure_mfma_rate(True, 0)
