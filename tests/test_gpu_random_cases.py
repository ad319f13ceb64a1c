"""Seeded random sweep over the argument space of the outer update (table
shapes with empty and tiny segments, every K, hyper-parameter corners, fp32 and
bf16 transport, fused / split form, two-pass / carried norms, with and without
first-step norms), each case checked element by element against the oracle for
three consecutive rounds.  Same tolerance as the other parity tests."""
import gc

import numpy as np
import pytest
import torch

import paper_2401_16265_amd as co2
from harness import HP, OuterStepHarness

pytestmark = pytest.mark.gpu
N_CASES = 48


def make_case(i):
    r = np.random.default_rng(1000 + i)
    n = int(r.choice([1, 3, 64, 255, 256, 257, 1000, 4096, 5000, 12345, 30011]))
    S = int(min(n, r.integers(1, 41))) if r.random() < 0.8 else int(min(n, 300))
    cuts = np.sort(r.integers(0, n + 1, size=S - 1)) if S > 1 else np.array([], dtype=np.int64)
    table = [0] + [int(c) for c in cuts] + [n]
    hp = HP(K=int(r.integers(1, 17)), alpha=float(r.choice([0.1, 0.5, 1.0])),
            beta=float(r.choice([0.0, 0.5, 0.9, 0.99])),
            phi=float(r.choice([1e-3, 1e-2, float("inf")])), c=float(r.choice([0.0, 0.5, 1.0, 2.0])),
            tau=int(r.integers(1, 9)))
    return dict(table=table, hp=hp, bf16=bool(r.random() < 0.4), split=bool(r.random() < 0.3),
                carried=bool(r.random() < 0.5), fsn=bool(r.random() < 0.4),
                drift="student_t" if r.random() < 0.5 else "normal", seed=int(r.integers(0, 1 << 30)))


@pytest.mark.parametrize("i", range(N_CASES))
def test_random_case(i):
    assert torch.cuda.is_available()
    dev = torch.device("cuda:0")
    c = make_case(i)
    split, carried, fsn = c["split"], c["carried"], c["fsn"]
    if split and carried:
        fsn = True            # carried sums of delta_out^2 do not exist in split form
    print(f"  case {i}: n={c['table'][-1]} S={len(c['table']) - 1} {c['hp']} bf16={c['bf16']} "
          f"split={split} carried={carried} fsn={fsn} drift={c['drift']}", flush=True)
    h = OuterStepHarness(c["table"], c["hp"], dev, seed=c["seed"], momentum_std=0.0, truth=True,
                         drift=c["drift"], use_first_step_norm=fsn, bf16=c["bf16"])
    for t in range(3):
        h.step(flags=co2.CO2_FLAG_CARRIED_NORMS if (carried and t >= 1) else 0, split=split)
    del h
    gc.collect()
