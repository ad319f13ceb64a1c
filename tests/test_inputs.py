"""The synthetic workloads have the sizes the task names (CPU only)."""
import numpy as np
import torch

import co2_inputs


def test_workload_tables_match_the_named_sizes():
    want = {"tiny": (1 << 20, 8), "gpt2s": (124_439_808, 148), "1p3b": (1_343_868_928, 292),
            "7b_shard": (421_150_976, None), "350m_overlap": (354_823_168, 292)}
    for name, (n, S) in want.items():
        t = co2_inputs.config_table(co2_inputs.CONFIGS[name])
        assert t[0] == 0 and t[-1] == n and all(b >= a for a, b in zip(t, t[1:]))
        if S is not None:
            assert len(t) - 1 == S
    full = co2_inputs.llama_table(layers=32, d=4096, ffn=11008, vocab=32000)
    assert full[-1] == 6_738_415_616 and len(full) - 1 == 291
    # the 16 shards tile the full table; interior boundaries are kept, ends are cut
    total = 0
    for r in range(16):
        sh = co2_inputs.shard_of_table(full, r, 16)
        assert sh[0] == 0 and sh[-1] == full[-1] // 16
        total += len(sh) - 1
    assert total >= 291
    sh1 = co2_inputs.config_table(co2_inputs.CONFIGS["7b_shard"], rank=1)
    lo = full[-1] // 16
    assert sh1[1] + lo in full and sh1[-2] + lo in full      # first and last pieces are partial tensors
    assert (lo not in full) and (2 * lo not in full)


def test_draws_are_seeded_and_shaped():
    a = co2_inputs.fill_normal_(torch.empty(100000), 0.02, co2_inputs.seed_for(0, 1))
    b = co2_inputs.fill_normal_(torch.empty(100000), 0.02, co2_inputs.seed_for(0, 1))
    c = co2_inputs.fill_normal_(torch.empty(100000), 0.02, co2_inputs.seed_for(0, 2))
    assert torch.equal(a, b) and not torch.equal(a, c)
    assert abs(float(a.std()) - 0.02) < 1e-3
    t = co2_inputs.fill_student_t_(torch.empty(200000), 1e-3, 3, co2_inputs.seed_for(0, 3))
    # Student-t(3): heavy tails (kurtosis far above the normal's 3), scale 1e-3 (variance 3e-6)
    x = t.double().numpy()
    assert 0.97e-3 < np.median(np.abs(x)) / 0.7649 < 1.03e-3     # median |t_3| = 0.7649 * scale
    assert np.mean(np.abs(x) > 5e-3) > 5e-3                       # P(|t_3| > 5) ~ 1.5 %
    g = co2_inputs.fill_bf16_normal_(torch.empty(1000, dtype=torch.bfloat16), 1e-3, 5)
    assert g.dtype == torch.bfloat16 and float(g.float().std()) > 5e-4
