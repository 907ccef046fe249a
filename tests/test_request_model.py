"""Pins of the access-pattern model against the values the paper prints
(Section 3.2.1 worked example; Section 3.2.2 Little's-law sizing)."""
import itertools

import pytest

from oracle import request_model as rm


def test_worked_example_8_to_5(golden):
    feat = golden["example_row_bytes"] // 4
    idx_list = [golden["example_source_row"]]
    kw = dict(warp_size=golden["example_warp_size"], line_bytes=golden["example_line_bytes"])
    assert rm.count_read_requests(feat, idx_list, shift=False, **kw) == golden["example_requests_naive"]
    assert rm.count_read_requests(feat, idx_list, shift=True, **kw) == golden["example_requests_shifted"]


@pytest.mark.parametrize("feat", [33, 100, 120, 257, 261, 602])
def test_shift_is_a_rotation_and_never_changes_the_result(feat):
    idx_list = [3, 0, 7, 7, 1, 12]
    plain = sorted(rm.copy_pairs(feat, idx_list, shift=False))
    shifted = sorted(rm.copy_pairs(feat, idx_list, shift=True))
    want = sorted((i * feat + o, idx_list[i] * feat + o)
                  for i, o in itertools.product(range(len(idx_list)), range(feat)))
    assert plain == want and shifted == want


@pytest.mark.parametrize("feat", [16, 32, 64, 128, 256])
def test_shift_not_applied_to_short_or_line_multiple_rows(feat):
    idx_list = [5, 2, 9]
    n = len(idx_list) * feat
    assert all(rm.thread_offsets(i, feat, idx_list, True) == rm.thread_offsets(i, feat, idx_list, False)
               for i in range(n))


@pytest.mark.parametrize("feat", [100, 120, 257, 258, 259, 260, 261, 602])
def test_shift_never_needs_more_requests(feat):
    idx_list = [11, 4, 4, 30, 17, 2, 9, 23]
    assert (rm.count_read_requests(feat, idx_list, True)
            <= rm.count_read_requests(feat, idx_list, False))


def test_littles_law_numbers(golden):
    warps_per_sm = golden["threads_per_sm"] // golden["warp_size"]
    assert warps_per_sm == 48
    upper = rm.gpu_share_for_requests(golden["max_outstanding_reads"], warps_per_sm, golden["n_sm"])
    assert round(100 * upper, 1) == golden["share_upper_percent"]
    n_req = rm.outstanding_requests(golden["memcpy_gib_per_s"] * 2 ** 30, golden["request_bytes"],
                                    golden["rtt_us"] * 1e-6)
    assert round(n_req, 1) == golden["requests_in_flight"]
    lower = rm.gpu_share_for_requests(n_req, warps_per_sm, golden["n_sm"])
    assert round(100 * lower, 1) == golden["share_lower_percent"]
