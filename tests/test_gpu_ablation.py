"""The ablation module runs and reports what the definitions fix: with the cache emptied
before every step every selected row is fetched (miss rate 1); with the hit/miss cache fewer."""
import io
import re

import pytest

pytestmark = pytest.mark.gpu


def test_no_hit_miss_fetches_every_selected_row():
    from paper_2510_23649_amd import ablation
    buf = io.StringIO()
    ablation.no_hit_miss(steps=4, layers=1, out=buf)
    rows = [ln for ln in buf.getvalue().splitlines() if ln.startswith("| ") and "variant" not in ln]
    default, emptied = (re.split(r"\s*\|\s*", ln.strip("| ")) for ln in rows[-2:])
    assert int(emptied[2]) == 32 * 2048            # B * Hq * k rows of workload 3
    assert 0 < int(default[2]) < int(emptied[2]) // 2
    assert float(emptied[1]) > float(default[1])   # and it costs time
