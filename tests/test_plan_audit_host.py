"""Host-side checks of the plan audit tool (no GPU): its shape lists and candidate launches."""
import pytest

from paper_2402_00025_amd import binding as b
from paper_2402_00025_amd import plan_audit


def test_shape_lists_are_valid_and_seeded():
    a = plan_audit.random_shapes(25, seed=4)
    assert a == plan_audit.random_shapes(25, seed=4) and a != plan_audit.random_shapes(25, seed=5)
    for (m, n, k) in a + plan_audit.STRUCTURED:
        assert 1 <= m <= 16 and n % 8 == 0 and k % 128 == 0
        assert n * k // 2 <= 160 << 20 or (m, n, k) in plan_audit.STRUCTURED
        assert b.w4a16_check(m, n, k, 128, 0) == 0


@pytest.mark.parametrize("m,n,k,g", [(16, 4096, 4096, 128), (1, 11008, 4096, 128), (6, 2304, 3072, 128), (16, 4096, 4096, 32)])
def test_candidates_are_launches_the_library_accepts(m, n, k, g):
    cands = plan_audit.candidates(b, m, n, k, g)
    assert len(cands) >= 8
    keys = {plan_audit.fmt(c) for c in cands}
    assert len(keys) == len(cands)                      # no launch twice
    for c in cands:
        # asking for exactly this launch gives it back
        again = b.w4a16_plan(m, n, k, g, split_k=c["split_k"], tile_cols=c["tile_cols"], waves=c["waves"], reduce=c["reduce"])
        assert plan_audit.fmt(again) == plan_audit.fmt(c)
        tiles = -(-n // c["tile_cols"])
        assert 96 <= tiles * c["split_k"] <= 1100
    if g == 128:
        assert any(c["tile_cols"] == 256 for c in cands) and any(c["tile_cols"] == 64 for c in cands)
    else:
        assert any(c["waves"] >= 8 for c in cands)      # short groups: larger workgroups among the candidates


@pytest.mark.parametrize("bits", [8, 3, 2])
def test_candidates_of_the_other_field_widths(bits):
    cands = plan_audit.candidates_bits(b, bits, 16, 4096, 4096, 128)
    asks = [c["ask"] for c in cands]
    assert asks == sorted(set(asks)) and set(asks) <= {1, 2, 4, 8, 16, 32}   # 32 groups: the divisors only
    for c in cands:
        assert c["split_k"] == c["ask"] and c["tile_cols"] == 64            # an explicit split: the per-wave kernel
