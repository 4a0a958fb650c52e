"""Seeded sweep over random shapes, mask densities, byte budgets (several chunks) and decode modes: whatever the
draw, the HIP path agrees with the oracle (every row for small cases, a thinned sample plus the ragged tail else)
and leaves the entries past the count untouched."""
import numpy as np
import pytest
import torch

from paper_2601_06562_amd import binding, workloads

from gpu_helpers import check_against_oracle, oracle_rows, run_hip
from test_gpu_sampling import check_sample, run_sample

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.mark.parametrize("seed", [11, 12, 13])
def test_random_shapes_against_the_oracle(seed):
    rng = np.random.default_rng(seed)
    for case in range(40):
        d = int(rng.choice([64, 128, 192, 256, 320, 512, 704, 1024]))
        V = int(rng.choice([256, 512, 768, 1000, 1280, 2048, 2304, 4099, 5120, 8192]))
        T = int(rng.integers(1, 6000))
        p = float(rng.choice([0.02, 0.3, 0.7, 1.0]))
        wl = workloads.small_random(T, d, V, p=p, seed=int(rng.integers(1 << 30)), device=DEV)
        M_true = int(wl.mask.sum().item())
        budget = 0
        if rng.random() < 0.4 and M_true > 300:          # a budget of a few partial slots: several chunks
            budget = int(rng.choice([12 * 256 * 1, 12 * 256 * 3, 12 * 512 * 4, 12 * 1024 * 2])) + binding.SYNC_BYTES
        sampling = bool(rng.random() < 0.5)
        tau = float(rng.choice([0.2, 0.7, 1.0, 3.0]))
        draw_seed = int(rng.integers(1 << 62))
        what = f"seed {seed} case {case}: T={T} d={d} V={V} p={p} M={M_true} budget={budget} sampling={sampling} tau={tau}"
        print(what, flush=True)
        w_bits = workloads.bf16_bits(wl.w)
        if sampling:
            out = run_sample(wl, tau, draw_seed, budget_bytes=2 * budget)
        else:
            out = run_hip(wl.hidden, wl.w, wl.mask, budget_bytes=budget)
        M = out["M"]
        assert M == M_true, what
        assert np.all(out["tok"][M:] == -7) and np.all(out["lse"][M:] == -7.0), what
        if M == 0:
            continue
        if budget:
            assert out["op"].plan.workspace_bytes <= (2 * budget if sampling else budget), what
        rows = np.arange(M) if M <= 300 else np.unique(np.concatenate([np.arange(0, M, 7), np.arange(M - 40, M)]))
        if sampling:
            hb = workloads.bf16_bits(wl.hidden[torch.as_tensor(out["idx"][rows].astype(np.int64), device=DEV)])
            check_sample(out, hb, w_bits, rows, tau, draw_seed, what)
        else:
            want, logits = oracle_rows(wl.hidden, w_bits, out["idx"][rows], return_logits=True)
            check_against_oracle(dict(tok=out["tok"][rows], conf=out["conf"][rows], lse=out["lse"][rows]), want, logits,
                                 what=what)
