"""The score-variant comparison tool on workload 1: what must come out follows from the
workload (8 keys planted in the prompt, re-attended every 40-90 steps, budget 128)."""
import pytest

from paper_2506_15969_amd.workload import CONFIGS

pytestmark = pytest.mark.gpu


def test_variants_on_planted_keys(lazyev_lib):
    from paper_2506_15969_amd import ablation
    rows = {r["score_flags"]: r for r in ablation.run(CONFIGS["cfg1"])}
    assert set(rows) == {3, 19, 1, 2, 18, 0}
    for flags in (3, 19, 1):                             # every variant with H1 keeps all of them
        assert rows[flags]["recall"] == 1.0 and rows[flags]["survive"] == 1.0
        assert rows[flags]["err_at_fire"] < 1e-3         # the fired key carries the attention
    # a sliding window has lost every prompt key by the time it fires again
    assert rows[0]["survive"] == 0.0 and rows[0]["recall"] < 0.5 and rows[0]["err_at_fire"] > 0.5
    assert all(r["evictions"] == 28 for r in rows.values())
