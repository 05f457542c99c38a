"""Host-only: every lattice-kernel variant the criterion entry points can dispatch to is the
variant of at least one GPU parity case (tests/variant_cases.py).  The set of reachable variants
is found by asking the library's launch-configuration query for every size it accepts."""
import paper_1812_07625_amd as P
from variant_cases import ASG_CASES, CTC_CASES, asg_variant, ctc_variant


def _reachable(query, classes, lmax_max):
    seen = {}
    for C in classes:
        for L in range(1, lmax_max + 1):
            try:
                v = query(P, C, L)
            except P.W2LError:
                continue
            seen.setdefault(v, (C, L))
    return seen


def test_ctc_cases_cover_every_reachable_variant():
    reach = _reachable(ctc_variant, list(range(1, 260)) + [300, 600, 1000, 4096], 3000)
    assert len(reach) == 24, sorted(reach)          # 3 pair counts x 2 block lengths x 4 table depths
    covered = {ctc_variant(P, c, l) for c, l in CTC_CASES}
    missing = {v: eg for v, eg in reach.items() if v not in covered}
    assert not missing, "variants (pairs per lane, table values, block) with no parity case; e.g. (C, Lmax): %r" % missing


def test_asg_cases_cover_every_reachable_variant():
    reach = _reachable(asg_variant, range(1, 65), 3000)
    covered = {asg_variant(P, c, l) for c, l in ASG_CASES}
    missing = {v: eg for v, eg in reach.items() if v not in covered}
    assert not missing, "variants (positions, class lanes, max threads, block, row values) with no parity case: %r" % missing


def test_launch_config_rejects_what_the_entry_points_reject():
    import pytest
    for bad in ((0, 10), (5000, 10), (29, 0), (29, 3001)):
        with pytest.raises(P.W2LError):
            P.w2l_ctc_launch_config(*bad)
    for bad in ((0, 10), (65, 10), (28, 0), (28, 3001)):
        with pytest.raises(P.W2LError):
            P.w2l_asg_launch_config(*bad)
