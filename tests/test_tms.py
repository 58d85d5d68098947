"""The TMS model against the values the paper prints (Sec. 4 tables)."""
import os

import pytest

from paper_2311_09431_amd import tms

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "tms_values.txt")


def _rows():
    with open(GOLDEN) as f:
        for line in f:
            line = line.split("#")[0].split()
            if line:
                yield line[0], int(line[1]), int(line[2]), float(line[3]), float(line[4])


@pytest.mark.parametrize("model,N,n_seq,cost,want", list(_rows()))
def test_printed_tms_values(model, N, n_seq, cost, want):
    assert round(tms.tms(model, n_seq, N, cost), 2) == pytest.approx(want, abs=0.0051)


def test_limits():
    assert tms.attention_only_limit(8) == pytest.approx(1.875)
    assert tms.attention_only_limit(4, c=4) == pytest.approx((10 + 48) / 40)
    # attention dominates at long sequences: TMS tends to the attention-only limit
    assert tms.tms("1B", 10 ** 9, 8, 1) == pytest.approx(1.875, abs=1e-3)
    # and striping cannot pay when attention is negligible
    assert tms.tms("7B", 16, 8, 1) == pytest.approx(1.0, abs=1e-2)
