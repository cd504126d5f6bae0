"""Draft-length policy (Algorithm 1, Section 3.4.2) and throughput model (Section 3.4.1): pins for the
oracle, and parity of the library's host function against it.  No GPU needed: the call is host
arithmetic behind the same C ABI."""
import os

import numpy as np
import pytest

from oracle import mba_oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _golden():
    rows = []
    for line in open(os.path.join(ROOT, "tests", "golden", "mba_worked_examples.txt")):
        if line.startswith("#") or not line.strip():
            continue
        head, beta, want = line.split("|")
        B_h, B_l, gmax, lam, gstar = head.split()
        rows.append((int(B_h), int(B_l), int(gmax), float(lam), int(gstar), [float(x) for x in beta.split()],
                     tuple(int(x) for x in want.split())))
    return rows


def _step_time_with_argmin(gstar, gmax, alpha):
    """A step-time row whose expected time per token is smallest at gstar (built from the model's own
    closed form only to place the minimum; the value itself is pinned by the simulation test)."""
    tokens = [(1 - alpha ** (g + 1)) / (1 - alpha) for g in range(gmax + 1)]
    return [tokens[g] * (1.0 if g == gstar else 1.3) for g in range(gmax + 1)]


@pytest.mark.parametrize("row", _golden())
def test_oracle_reproduces_the_hand_worked_runs(row):
    B_h, B_l, gmax, lam, gstar, beta, want = row
    alpha = sum(beta[:gmax]) / gmax
    st = _step_time_with_argmin(gstar, gmax, alpha)
    gh, gl, gs = mba_oracle.mba(B_h, B_l, beta, gmax, lam, st)
    assert gs == gstar and (gh, gl) == want


def test_expected_tokens_per_step_against_simulation():
    """(1 - alpha^(gamma+1)) / (1 - alpha): simulate i.i.d. acceptance with probability alpha, stop at the
    first rejection, count accepted + bonus.  Time per token = step time / tokens per step."""
    rng = np.random.default_rng(1)
    for alpha, gamma in ((0.7, 8), (0.5, 3), (0.9, 16), (0.3, 1)):
        acc = rng.random((400000, gamma)) < alpha
        n_acc = np.where(acc.all(axis=1), gamma, np.argmin(acc, axis=1))
        tokens = (n_acc + 1).mean()
        model = 5.0 / mba_oracle.t_sd(alpha, 5.0, gamma)          # tokens per step from the oracle's T_SD
        assert abs(model - tokens) < 5 * (n_acc + 1).std() / np.sqrt(acc.shape[0])
    assert mba_oracle.t_sd(0.6, 2.0, 0) == pytest.approx(2.0)      # gamma = 0 is a plain decode step


def test_optimal_gamma_against_simulated_time_per_token():
    rng = np.random.default_rng(2)
    alpha, gmax = 0.75, 8
    beta = [alpha] * (gmax + 1)
    step = [1.0 + 0.02 * g + 0.012 * g * g for g in range(gmax + 1)]        # verification cost grows with gamma
    sim = []
    for g in range(gmax + 1):
        acc = rng.random((300000, g)) < alpha if g else np.zeros((300000, 0), bool)
        n_acc = np.where(acc.all(axis=1), g, np.argmin(acc, axis=1)) if g else np.zeros(300000, int)
        sim.append(step[g] / (n_acc + 1).mean())
    assert mba_oracle.optimal_gamma(beta, step, gmax) == int(np.argmin(sim))


def test_invariants_of_the_allocation():
    rng = np.random.default_rng(3)
    for _ in range(3000):
        gmax = int(rng.integers(0, 12))
        beta = np.sort(rng.random(gmax + 1 + int(rng.integers(0, 3))))[::-1].tolist()
        B_h, B_l = int(rng.integers(1, 40)), int(rng.integers(0, 300))
        lam = float(1 + 3 * rng.random())
        step = (1 + rng.random(gmax + 1) * np.arange(1, gmax + 2)).tolist()
        gh, gl, gs = mba_oracle.mba(B_h, B_l, beta, gmax, lam, step)
        assert 0 <= gs <= gmax and 0 <= gh <= gmax and 0 <= gl <= gmax
        assert gh * B_h + gl * B_l <= gs * (B_h + B_l)                   # never more than the budget
        if gs * (B_h + B_l) < B_h:
            assert (gh, gl) == (0, 0)
        else:
            assert gh >= 1                                               # every high-priority request drafts
        if B_l == 0 and gs >= 1 and all(beta[i] > beta[i + 1] for i in range(gmax)):
            assert gh == min(gs, gmax)


def test_library_matches_the_oracle():
    from paper_2511_14617_amd import binding
    rng = np.random.default_rng(4)
    for row in _golden():
        B_h, B_l, gmax, lam, gstar, beta, want = row
        st = _step_time_with_argmin(gstar, gmax, sum(beta[:gmax]) / gmax)
        assert binding.seer_mba_draft_lengths(B_h, B_l, beta, gmax, lam, st) == (want[0], want[1], gstar)
    for _ in range(5000):
        gmax = int(rng.integers(0, 20))
        beta = np.sort(rng.random(gmax + 1 + int(rng.integers(0, 3))))[::-1]
        if rng.random() < 0.3:
            beta = np.round(beta, 1)                                     # ties between marginal benefits
        beta = beta.tolist()
        B_h, B_l = int(rng.integers(1, 60)), int(rng.integers(0, 400))
        lam = float(rng.choice([1.0, 2.0, 1 + 3 * rng.random()]))
        step = (1 + rng.random(gmax + 1) * np.arange(1, gmax + 2)).tolist()
        assert binding.seer_mba_draft_lengths(B_h, B_l, beta, gmax, lam, step) == mba_oracle.mba(
            B_h, B_l, beta, gmax, lam, step)


def test_library_argument_errors():
    from paper_2511_14617_amd import binding as b
    ok = dict(B_h=2, B_l=2, beta=[0.9, 0.5, 0.1], gamma_max=2, lam=2.0, step_time=[1.0, 1.1, 1.3])

    def code(**kw):
        a = dict(ok)
        a.update(kw)
        try:
            b.seer_mba_draft_lengths(a["B_h"], a["B_l"], a["beta"], a["gamma_max"], a["lam"], a["step_time"])
        except b.SeerError as e:
            return e.code
        return 0

    assert code() == 0
    assert code(B_h=0) == b.SEER_ESHAPE
    assert code(beta=[0.9, 0.5]) == b.SEER_ESHAPE                    # needs gamma_max + 1 positions
    assert code(beta=[0.9, 1.5, 0.1]) == b.SEER_EINVAL
    assert code(lam=0.5) == b.SEER_EINVAL
    assert code(step_time=[1.0, 0.0, 1.3]) == b.SEER_EINVAL
    assert code(gamma_max=64, beta=[0.5] * 70, step_time=[1.0] * 65) == b.SEER_ESHAPE
