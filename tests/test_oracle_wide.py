"""Pins for oracle/kvtc_wide.py: plans over the concatenated features of several layers whose kept coordinates
are stored in sections (paper, Section "Feature decorrelation"; appendices "PCA matrix sizes" and "PCA feature
concat size vs performance").  Every check is against the unsectioned coder, which has pins of its own, against
hand-counted layouts, or against the budget."""
import numpy as np
import pytest

import kvtc_oracle as ko
import kvtc_synth as ks
import kvtc_wide as kw


def test_split_groups_hand_counted():
    assert kw.split_groups([]) == []
    assert kw.split_groups([16]) == [(0, 1)]
    assert kw.split_groups([1024, 16]) == [(0, 1), (1, 2)]
    assert kw.split_groups([256, 256, 256, 256, 64]) == [(0, 4), (4, 5)]            # 1024 fits exactly
    assert kw.split_groups([256, 256, 256, 64, 256]) == [(0, 4), (4, 5)]            # 832 + 256 would not
    assert kw.split_groups([64, 1024, 64]) == [(0, 1), (1, 2), (2, 3)]
    assert kw.split_groups([16] * 70) == [(0, 64), (64, 70)]                        # at most 64 groups a section
    assert kw.split_groups([16] * 5, max_coords=32) == [(0, 2), (2, 4), (4, 5)]


def test_section_offsets_hand_counted():
    # T = 3 tokens, sections of 20 and 8 bytes a token: 60 bytes, then from the next 16-byte boundary 24 more
    assert kw.section_offsets([20, 8], 3) == [0, 64, 88]
    assert kw.section_offsets([16, 4, 4], 4) == [0, 64, 80, 96]
    assert kw.section_offsets([12], 5) == [0, 60]
    assert kw.section_offsets([], 9) == [0]


def _hand_plan(p, group_n, group_bits, seed):
    rng = np.random.default_rng(seed)
    r = int(np.sum(group_n))
    V = np.linalg.qr(rng.standard_normal((p, p)))[0][:, :r]
    mu = rng.normal(0, 0.1, p)
    blocks, j = [], 0
    for n, b in zip(group_n, group_bits):
        blocks.append(ko.Block(j, n, b))
        j += n
    return ko.compile_plan(mu, V, blocks)


@pytest.mark.parametrize("group_n,group_bits", [
    ([256, 64, 256, 256, 256, 64, 16], [6, 5, 4, 3, 2, 2, 1]),        # 1168 coordinates: two sections
    ([1024, 1024, 16], [3, 2, 1]),                                       # three sections, two of them full
    ([64] * 8, [4] * 8),                                                 # 512: a single section = the plain coder
])
def test_sections_hold_the_codes_and_headers_of_the_unsectioned_plan(group_n, group_bits):
    p, T = 2304, 37
    plan = _hand_plan(p, group_n, group_bits, 3)
    x = ko.bf16_round(np.random.default_rng(4).normal(0, 1, (T, p)).astype(np.float32))
    stream = kw.encode_wide(plan, x)
    secs = kw.sections_of(plan)
    offs = kw.section_offsets([s.record_bytes for s in secs], T)
    assert stream.shape == (offs[-1],) and all(o % 16 == 0 for o in offs[:-1])
    assert sum(s.r for s in secs) == plan.r and sum(s.n_groups for s in secs) == plan.n_groups
    assert all(s.r <= 1024 and s.n_groups <= 64 for s in secs)
    # the same quantisation, group by group
    sh0, sc0, co0 = ko.unpack(plan, ko.encode(plan, x))
    sh1, sc1, co1 = kw.unpack_wide(plan, stream, T)
    assert np.array_equal(sh0.view(np.uint16), sh1.view(np.uint16))
    assert np.array_equal(sc0.view(np.uint16), sc1.view(np.uint16))
    assert np.array_equal(co0, co1)
    # and the same reconstruction
    a = ko.decode(plan, ko.encode(plan, x))
    b = kw.decode_wide(plan, stream, T)
    assert np.max(np.abs(a - b)) <= 1e-12 * max(1.0, np.max(np.abs(a)))
    # bytes: the sections' records, nothing else but the alignment gaps
    assert kw.record_bytes(plan) == sum(s.record_bytes for s in secs)
    assert 0 <= kw.record_bytes(plan) - plan.record_bytes <= 4 * (len(secs) - 1)
    if len(secs) == 1:
        assert np.array_equal(stream, ko.encode(plan, x).reshape(-1))


def test_calibration_over_concatenated_layers_respects_budget_and_rank_cap():
    """Two layers side by side (p = 2048) at 8x: the allocation keeps more than 1024 coordinates, all among the first
    rank_cap components, and what is stored per token -- every section's padded record -- fits the budget."""
    L = ks.make_layer(ks.cross_layer_spec(2))
    C = ko.bf16_round(ks.draw_f32(L, 2048 + 512, ks.CALIB_DRAW))
    cap = 1536
    plan, info = kw.calibrate_wide(C, 8.0, cap, n_dp_tokens=512)
    assert plan.p == 2048 and plan.r > 1024
    assert plan.kept.max() < cap
    assert 8 * kw.record_bytes(plan) <= info["budget_bits"] == ko.bit_budget(2048, 8.0) == 4096
    assert info["dp_budget_bits"] <= info["budget_bits"]
    assert len(kw.sections_of(plan)) >= 2
    # a fresh draw reconstructs about as well as the allocation's own error estimate says (same order of magnitude)
    X = ko.bf16_round(ks.draw_f32(L, 64, ks.TEST_DRAW))
    xh = kw.decode_wide(plan, kw.encode_wide(plan, X), 64)
    rel = np.linalg.norm(xh - X) / np.linalg.norm(X - plan.mu32[None, :].astype(np.float64))
    assert rel < 0.5
    # a lower cap can only do worse or equal on the tokens the allocation was optimised for (the basis is orthonormal
    # up to its bf16 rounding, so the error in coordinates is the error in features)
    plan2, _ = kw.calibrate_wide(C, 8.0, 1024, n_dp_tokens=512)
    assert plan2.kept.max() < 1024
    e1 = np.linalg.norm(kw.decode_wide(plan, kw.encode_wide(plan, C[:512]), 512) - C[:512])
    e2 = np.linalg.norm(kw.decode_wide(plan2, kw.encode_wide(plan2, C[:512]), 512) - C[:512])
    assert e1 <= 1.01 * e2
