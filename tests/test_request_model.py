"""Pins of the access-pattern model against the values the paper prints
(Section 3.2.1 worked example; Section 3.2.2 Little's-law sizing) and against
what the section says the alignment stage achieves."""
import itertools

import numpy as np
import pytest

from oracle import request_model as rm


def test_worked_example_8_to_5(golden):
    feat = golden["example_row_bytes"] // 4
    idx_list = [golden["example_source_row"]]
    kw = dict(warp_size=golden["example_warp_size"], line_bytes=golden["example_line_bytes"])
    assert rm.count_read_requests(feat, idx_list, shift=False, **kw) == golden["example_requests_naive"]
    assert rm.count_read_requests(feat, idx_list, shift=True, **kw) == golden["example_requests_shifted"]


def test_worked_example_lines_by_hand(golden):
    """The same case without the model: the row is bytes [480, 960) of the table. Unshifted, warp w
    reads bytes [480 + 128 w, 608 + 128 w) cut at 960: each of the 4 warps straddles two lines.
    Shifted, the reads fall on the 5 lines that cover the row and no warp straddles."""
    rb, line = golden["example_row_bytes"], golden["example_line_bytes"]
    start = golden["example_source_row"] * rb
    naive = sum(len({b // line for b in range(start + 128 * w, min(start + 128 * w + 128, start + rb), 4)})
                for w in range(4))
    covering = len({b // line for b in range(start, start + rb, 4)})
    assert (naive, covering) == (golden["example_requests_naive"], golden["example_requests_shifted"])


@pytest.mark.parametrize("feat", [33, 100, 120, 257, 261, 602])
def test_stage_is_a_rotation_and_never_changes_the_result(feat):
    idx_list = [3, 0, 7, 7, 1, 12]
    want = sorted((i * feat + o, idx_list[i] * feat + o)
                  for i, o in itertools.product(range(len(idx_list)), range(feat)))
    for shift in (False, True):
        dst, src = rm.element_map(feat, idx_list, shift)
        assert sorted(zip(dst.tolist(), src.tolist())) == want


@pytest.mark.parametrize("feat", [33, 100, 120, 257, 261, 602])
def test_stage_makes_lane_k_read_elements_congruent_to_k(feat):
    """The section's aim: after the stage a warp's reads start on a line boundary of the source,
    except where a row wraps around its end."""
    idx_list = [3, 0, 7, 7, 1, 12, 5]
    dst, src = rm.element_map(feat, idx_list, True)
    t = np.arange(src.size)
    r, p = np.divmod(t, feat)
    rot = rm.row_rotations(feat, idx_list, True)
    no_wrap = p + rot[r] < feat
    assert np.all((src[no_wrap] - t[no_wrap]) % 32 == 0)
    assert no_wrap.sum() >= src.size - 31 * len(idx_list)


@pytest.mark.parametrize("feat", [16, 32, 64, 128, 256])
def test_stage_not_applied_to_short_or_line_multiple_rows(feat):
    idx_list = [5, 2, 9]
    assert not rm.row_rotations(feat, idx_list, True).any()
    a, b = rm.element_map(feat, idx_list, True), rm.element_map(feat, idx_list, False)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


@pytest.mark.parametrize("feat", [100, 120, 257, 258, 259, 260, 261, 602])
def test_stage_never_needs_more_requests(feat):
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
