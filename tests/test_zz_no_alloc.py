"""pcm_score_phases_static (the entry point that allocates nothing) against pcm_score_phases.

Both run the same kernels; the static variant keeps its accumulators in an array inside the library instead of
a caller workspace.  Two calls in a row, the second on a smaller batch (the array still holds what the first
call left), each compared bit for bit with the workspace entry point and with the CPU checker; then a shape
whose accumulators exceed the array is refused.
"""
import ctypes

import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import pcm_oracle as O
from workloads import CONFIGS, make_rollouts

pytestmark = pytest.mark.gpu


def dev(x):
    return torch.from_numpy(np.ascontiguousarray(x)).cuda()


def bits(t):
    return np.ascontiguousarray(t.cpu().numpy()).view(np.uint8)


def _outputs(cfg):
    d = torch.device("cuda")
    return (torch.full((cfg.K,), -1.0, dtype=torch.float64, device=d), torch.full((cfg.K,), 7, dtype=torch.uint8, device=d),
            torch.full((cfg.T,), -1.0, dtype=torch.float32, device=d), torch.full((cfg.T,), 7, dtype=torch.uint8, device=d))


def test_static_scratch_entry_point_matches_workspace_entry_point():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2605_16154_amd as pcm
    L = pcm.lib()
    for name in ("cfg5", "cfg2"):                       # a large batch first, then a smaller one
        cfg = CONFIGS[name]
        ro = make_rollouts(cfg, 0)
        actions, phase, reward, n_chunks = dev(ro["actions"]), dev(ro["phase"]), dev(ro["reward"]), dev(ro["n_chunks"])
        want = pcm.pcm_score_phases(actions, phase, reward, n_chunks, cfg.n_groups, cfg.G, cfg.K, 1e-6, out=_outputs(cfg))
        got = _outputs(cfg)
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        pcm.pcm_score_phases(actions, phase, reward, n_chunks, cfg.n_groups, cfg.G, cfg.K, 1e-6, out=got,
                             static_scratch=True)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        for g, w in zip(got, want):
            assert np.array_equal(bits(g), bits(w)), name
        C_o, valid_o = O.phase_scores(ro["actions"], ro["phase"], ro["reward"], ro["n_chunks"], cfg.n_groups, cfg.G, cfg.K)
        assert np.array_equal(got[0].cpu().numpy().view(np.int64), C_o.view(np.int64)), name
        assert np.array_equal(got[1].cpu().numpy(), valid_o), name
    # a shape whose accumulators do not fit the array: refused on the host, nothing launched
    n_groups, G, N, A, K = 4096, 2, 4, 56, 64
    assert L.pcm_score_phases_workspace_bytes(n_groups, G, N, A, K) > (4 << 20)
    one = torch.zeros(16, dtype=torch.float64, device="cuda")
    rc = L.pcm_score_phases_static(one.data_ptr(), one.data_ptr(), one.data_ptr(), None, n_groups, G, N, A, K,
                                   ctypes.c_double(1e-6), one.data_ptr(), one.data_ptr(), None, None, None)
    assert rc == -2
