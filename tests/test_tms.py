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


def test_computed_tiles_match_the_oracle_classifier_and_the_library():
    from oracle import striped_attention as orc
    from paper_2311_09431_amd import binding as sa
    for N, c, tq, tk in [(4, 16, 4, 8), (3, 12, 6, 2), (2, 8, 8, 8)]:
        for layout in (sa.CONTIGUOUS, sa.STRIPED):
            for j in range(N):
                for k in range(N):
                    full, part, _ = orc.classify_tiles(orc.get_mask(j, k, N, c, layout), tq, tk)
                    mine = tms.computed_tiles(j, k, c, layout == sa.STRIPED, tq, tk)
                    assert mine == full + part == sa.sa_step_tiles(j, k, N, layout, c, tq, tk)[0]


def test_tiled_limit_reproduces_the_papers_granularity_remarks():
    # Sec. 3.2: with 4096-token blocks and 2048 x 4096 tiles striping saves nothing ...
    assert tms.tiled_attention_limit(8, 4096, 2048, 4096) == 1.0
    # ... with 2048 x 2048 tiles a quarter of every striped step is skipped:
    # contiguous worst device: 3 tiles in round 0, 4 in the others; striped: 3 in every round
    assert tms.tiled_attention_limit(8, 4096, 2048, 2048) == pytest.approx((3 + 7 * 4) / (8 * 3))
    # element granularity recovers the work ratio
    assert tms.tiled_attention_limit(4, 64, 1, 1) == pytest.approx(tms.attention_only_limit(4, 64))
