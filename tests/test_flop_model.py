"""The FLOP / speed-up model against the values the paper prints (appendix "Theoretical FLOPs
Reduction", table of theoretical end-to-end speed-ups) and against closed forms."""
import math
import os

import numpy as np
import pytest

from paper_2509_07120_amd import flop_model as F

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "table_a1_theoretical_speedup.txt")


def _table():
    rows = []
    with open(GOLDEN) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            parts = line.split()
            rows.append((int(parts[0]), [float(x) for x in parts[1:]]))
    return rows


def test_printed_table_is_reproduced_by_truncation():
    rhos = [0.25, 0.50, 0.75, 0.90]
    rows = _table()
    assert len(rows) == 4
    for n, printed in rows:
        for rho, want in zip(rhos, printed):
            got = F.theoretical_speedup(n, 1036, rho)
            assert math.floor(got * 10 + 1e-9) / 10 == want, (n, rho, got, want)


def test_table_is_not_reproduced_by_other_readings():
    """Pins the readings: without the L_G factor, or with rho as the fraction KEPT, the printed values fail."""
    no_lg = F.ModelShape(global_blocks=1)
    assert math.floor(F.theoretical_speedup(100, 1036, 0.9, no_lg) * 10) / 10 != 4.0
    kept = F.flop_total(100, 1036, 0.0) / F.flop_total(100, 1036, 1.0 - 0.9)  # rho read as kept fraction
    assert math.floor(kept * 10) / 10 != 4.0


def test_closed_forms():
    d = 1024
    assert F.flop_mlp(d) == 8 * d * d
    assert F.flop_attn(10, d, 0.0) == 4 * 10 * d * d + 2 * 100 * d
    assert F.flop_attn(10, d, 1.0) == 4 * 10 * d * d           # everything skipped: projections only
    assert F.flop_block(7, d) == F.flop_attn(7, d, 0.0) + 7 * 8 * d * d
    assert F.theoretical_speedup(100, 1036, 0.0) == 1.0
    # speed-up grows with rho and with the number of frames
    s = [F.theoretical_speedup(n, 1036, 0.75) for n in (10, 100, 300, 1000)]
    assert all(a < b for a, b in zip(s, s[1:]))
    # the limit for long sequences is 1 / (1 - rho)
    assert abs(F.theoretical_speedup(10 ** 7, 1036, 0.75) - 4.0) < 1e-2
    assert F.attention_only_speedup(0.75) == 4.0


def test_effective_sparsity_counts_tokens():
    n, b = 300, 128  # 3 blocks, tail 44
    cnt = np.array([3, 2, 1])
    last = np.array([True, False, True])
    pairs = F.kept_token_pairs(cnt, last, n, b)
    assert pairs == 128 * 300 + 128 * 256 + 44 * 44
    assert F.effective_sparsity(n * n, n, n) == 0.0
    assert abs(F.effective_sparsity(pairs, n, n) - (1 - pairs / 90000)) < 1e-15
