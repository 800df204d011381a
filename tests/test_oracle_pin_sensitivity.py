"""Do the pins bite?  Each case plants one plausible mistake (a dropped term, a wrong sign, index,
operand or constant) in a copy of the CPU checker and runs the pin tests of that area against the
copy in a child process: at least one pin must fail.  Nothing here touches the GPU library.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CHECKER = os.path.join(ROOT, "oracle", "pcm_oracle.py")

SEL, ACT, LAB, OPT = ("tests/test_oracle_selection.py", "tests/test_oracle_actor.py", "tests/test_oracle_labeler.py",
                      "tests/test_oracle_optimizer.py")

# (name, text in the checker, what it becomes, pin file)
MISTAKES = [
    ("advantage without the square root", "sigma = np.sqrt(mu * (F64(1.0) - mu))", "sigma = mu * (F64(1.0) - mu)", SEL),
    ("advantage sign", "(r.astype(F64) - mu) / (sigma + F64(eps))", "(mu - r.astype(F64)) / (sigma + F64(eps))", SEL),
    ("score pools sums instead of means", "F64(int(S[1, c, j])) / F64(n_pos) - F64(int(S[0, c, j])) / F64(n_neg)",
     "F64(int(S[1, c, j])) - F64(int(S[0, c, j]))", SEL),
    ("score without the square root", "total[c] = total[c] + np.sqrt(acc) * unscale", "total[c] = total[c] + acc * unscale", SEL),
    ("a phase missing one outcome counts as a zero score", "            if n_pos == 0 or n_neg == 0:\n                continue\n",
     "            if n_pos == 0 or n_neg == 0:\n                contributors[c] += 1\n                continue\n", SEL),
    ("keep probabilities normalised by the sum", "rho_tilde = self.S[c] / S_max if S_max > 0", "rho_tilde = self.S[c] / S_sum if S_max > 0", SEL),
    ("floor applied as a ceiling", "self.p[c] = rho_tilde if rho_tilde > p_min else F64(p_min)",
     "self.p[c] = rho_tilde if rho_tilde < p_min else F64(p_min)", SEL),
    ("buffers not reset at a refresh", "            self.S[:] = 0\n", "", SEL),
    ("Philox key schedule", "k1 = (k1 + _PHILOX_W1) & MASK32", "k1 = (k1 + _PHILOX_W0) & MASK32", SEL),
    ("draw picks one index late", "if wk > 0 and run > t:", "if wk > 0 and run > t + wk:", SEL),
    ("sampling with replacement", "        w[chosen] = 0\n", "", SEL),
    ("weights rounded down", "x = p[c] * F64(WEIGHT_SCALE) + F64(0.5)", "x = p[c] * F64(WEIGHT_SCALE)", SEL),
    ("importance weight inverted", "np.float32(len(in_phase)) / np.float32(b)", "np.float32(b) / np.float32(len(in_phase))", SEL),
    ("allocation ignores the phase sizes", "weight = [int(n_c[c]) * int(q[c]) for c in range(K)]", "weight = [int(q[c]) for c in range(K)]", SEL),
    ("allocation ties to the higher index", "key=lambda c: (-rem[c], c)", "key=lambda c: (-rem[c], -c)", SEL),
    ("allocation counts inactive trajectories", "        if active is not None and not active[i]:\n            continue\n", "", SEL),
    ("out-of-range phase ids dropped from the score", "                c = min(int(phase[i, k]), K - 1)        # an id beyond the last phase counts as the last\n",
     "                c = int(phase[i, k])\n                if c >= K:\n                    continue\n", SEL),
    ("top phase picks the smallest probability", "if keep_probs[c] > keep_probs[best]:", "if keep_probs[c] < keep_probs[best]:", SEL),
    ("grasp threshold 0.5 instead of 0.75", "sustained = [4 * c >= 3 * L for c in count]", "sustained = [2 * c >= L for c in count]", LAB),
    ("windows two chunks wide", "range(j + 1, min(j + 4, Ni))", "range(j + 1, min(j + 3, Ni))", LAB),
    ("release before pre-grasp", "            if before_grasp and 10 * c >= L:\n                out[i, j] = PHASE_PRE_GRASP\n            elif after_grasp:",
     "            if after_grasp:\n                out[i, j] = PHASE_RELEASE_RAMP\n            elif before_grasp and 10 * c >= L:\n                out[i, j] = PHASE_PRE_GRASP\n            elif False:", LAB),
    ("tail and approach swapped", "elif last < 0 or j < last:", "elif last >= 0 and j > last:", LAB),
    ("gate without the sigmoid", "    return s, u * s\n", "    return s, u\n", ACT),
    ("down projection transposed operand", "    dWd = a.T @ dy\n", "    dWd = (dy.T @ a).T * 0 + a.T @ (dy * 2)\n", ACT),
    ("silu derivative drops a term", "du = da * v * (s * (1.0 + u * (1.0 - s)))", "du = da * v * s", ACT),
    ("upper clip uses the lower threshold", "clipped = np.clip(rho, 1.0 - eps_low, 1.0 + eps_high)", "clipped = np.clip(rho, 1.0 - eps_low, 1.0 + eps_low)", ACT),
    ("clipped rows still push", "gcoef = np.where(flows, w_row * rho * adv_row, 0.0)", "gcoef = w_row * rho * adv_row", ACT),
    ("entropy bonus with the wrong sign", "loss = -scale * term_sum - F64(entropy_coef) * scale * entropy.sum()",
     "loss = -scale * term_sum + F64(entropy_coef) * scale * entropy.sum()", ACT),
    ("gradient misses the gate path into dX", "dX = du @ Wg.T + dv @ Wu.T", "dX = dv @ Wu.T", ACT),
    ("chunk ratio from the first token only", "rho = np.repeat(np.exp(delta.reshape(-1, A).sum(axis=1)), A)",
     "rho = np.repeat(np.exp(delta.reshape(-1, A)[:, 0]), A)", ACT),
    ("clipping by the largest tensor norm", "        total += np.sum(g * g)\n", "        total = max(total, np.sum(g * g))\n", OPT),
    ("no bias correction of the second moment", "bc2 = F64(1.0) - F64(beta2) ** t", "bc2 = F64(1.0)", OPT),
    ("decay coupled through the gradient", "theta_n = theta * (F64(1.0) - F64(lr) * F64(weight_decay))",
     "theta_n = theta - F64(lr) * F64(weight_decay) * g", OPT),
]


def _run_pins(checker_path, pin_file):
    env = dict(os.environ, PCM_CHECKER_SOURCE=checker_path)
    return subprocess.run([sys.executable, "-m", "pytest", pin_file, "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider"],
                          cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=600)


def test_every_planted_mistake_fails_a_pin(tmp_path):
    source = open(CHECKER).read()
    jobs = []
    for n, (name, old, new, pin_file) in enumerate(MISTAKES):
        assert source.count(old) == 1, f"'{name}': the text to change must occur exactly once in the checker"
        path = tmp_path / f"checker_with_mistake_{n}.py"
        path.write_text(source.replace(old, new))
        jobs.append((name, str(path), pin_file))
    # the unchanged copy must pass through the same mechanism, or a failure below would prove nothing
    same = tmp_path / "checker_unchanged.py"
    same.write_text(source)
    with ThreadPoolExecutor(max_workers=6) as pool:
        clean = pool.submit(_run_pins, str(same), LAB)
        results = list(pool.map(lambda j: (j[0], _run_pins(j[1], j[2])), jobs))
    assert clean.result().returncode == 0, clean.result().stdout[-2000:]
    survivors = [name for name, r in results if r.returncode != 1]   # 1 = some test failed
    assert not survivors, f"no pin noticed: {survivors}"
