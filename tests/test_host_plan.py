"""Host logic without a GPU: for any sizes the plan's grid covers every evaluation row and every
sample tile exactly once, stays inside the padded arrays, and the workspace blocks do not overlap
and fit in the size that sdkde_workspace_bytes reports."""
import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

import paper_2602_10378_amd as P

FLAGS = [P.SDKDE_PREC_FP32, P.SDKDE_PREC_FP16X2, P.SDKDE_PREC_FP16X2_ALL, P.SDKDE_PREC_FP16X2_PHI16, P.SDKDE_FLAG_MAX_SHIFT,
         P.SDKDE_FLAG_SYMMETRIC, P.SDKDE_FLAG_SYMMETRIC | P.SDKDE_PREC_FP16X2,
         P.SDKDE_FLAG_SYMMETRIC | P.SDKDE_FLAG_MAX_SHIFT]


def _check(n, m, d, call, flags):
    p = P.sdkde_describe_plan(n, m, d, call, flags)
    rows = n if call == 0 else m
    thin = d <= (3 if call == 2 else 6)      # direct differences: eval up to d = 3, the score kinds up to d = 6
    assert p["thin"] == int(thin)
    assert p["dp"] == (d if thin else -(-d // 16) * 16)
    # rows: the grid's row blocks cover all evaluation rows and stay inside the padded point array
    assert p["row_blocks"] * p["rows_per_block"] >= max(rows, 1)
    assert p["row_blocks"] * p["rows_per_block"] <= p["m_pad"]
    assert p["rows_per_block"] == (256 * p["row_tiles"] if thin else 64 * p["row_tiles"])
    # samples: tiles cover n, stay inside the padded sample array, and the splits cover all tiles
    assert p["tiles"] * 16 >= n and p["tiles"] * 16 <= p["n_pad"]
    assert p["tiles"] % 2 == 0 and p["tiles_per_split"] % 2 == 0
    assert p["splits"] >= 1 and p["splits"] * p["tiles_per_split"] >= p["tiles"]
    assert p["n_pad"] % 1024 == 0 and p["m_pad"] % 1024 == 0 and p["n_pad"] >= n and p["m_pad"] >= rows
    if call == 0:
        assert p["m_pad"] == p["n_pad"]           # one prepared array serves as both operands
        assert p["off_ps"] == p["off_xs"] and p["off_pn"] == p["off_xn"]
    if not thin and call == 0 and p["row_tiles"] >= 2:
        assert p["rows_per_block"] % (16 * p["row_tiles"]) == 0      # own-tile spans are aligned to row tiles
    # workspace: blocks are 256-byte aligned, disjoint, and inside workspace_bytes
    score = call != 2
    blocks = [("xs", p["off_xs"], 4 * p["n_pad"] * p["dp"]), ("xn", p["off_xn"], 4 * p["n_pad"]),
              ("part_d", p["off_part_d"], 4 * p["partial_slots"] * p["m_pad"])]
    if p["off_xt"] >= 0:
        blocks.append(("xt", p["off_xt"], 4 * p["xt_scale"] * p["n_pad"] * p["dp"]))
    if call != 0:
        blocks += [("ps", p["off_ps"], 4 * p["m_pad"] * p["dp"]), ("pn", p["off_pn"], 4 * p["m_pad"])]
    if score:
        blocks.append(("part_t", p["off_part_t"], 4 * p["partial_slots"] * p["m_pad"] * p["dp"]))
        assert (p["off_xt"] >= 0) == (not thin)
    else:
        assert p["off_part_t"] == -1 and p["off_xt"] == -1
    blocks.sort(key=lambda b: b[1])
    for (name, off, size), nxt in zip(blocks, blocks[1:] + [("end", p["workspace_bytes"], 0)]):
        assert off % 256 == 0 and off >= 0, name
        assert off + size <= nxt[1], f"{name} overlaps {nxt[0]}"
    assert p["workspace_bytes"] <= P.sdkde_workspace_bytes(n, m if call else max(m, 1), d, flags)
    _check_symmetric(p, n, d, call, flags)
    # first-contraction MFMAs of the last 16-column block: only the real coordinates (fp32 inputs, d <= 32)
    if not thin and (flags & 15) == 0 and d <= 32:
        assert p["last_block_mfmas"] == -(-(d - (p["dp"] - 16)) // 4)
    else:
        assert p["last_block_mfmas"] == 4
    return p


def _check_symmetric(p, n, d, call, flags):
    """The symmetric mode's decomposition: whole blocks, non-empty groups, LDS within the CU's 160 KiB."""
    wanted = bool(flags & P.SDKDE_FLAG_SYMMETRIC) and call == 0 and 7 <= d <= 32 and (flags & 15) == 0
    if not wanted:
        assert p["symmetric"] == 0
    elif p["symmetric"] == 0:        # declined: too few work items to fill the chip
        assert n < 32768 * 2048 // 1024
    wanted = bool(p["symmetric"])
    if not wanted:
        assert p["sym_block_rows"] == p["sym_blocks_per_group"] == p["sym_groups"] == 0
        return
    rb, per_group, groups = p["sym_block_rows"], p["sym_blocks_per_group"], p["sym_groups"]
    rows_held = 8 * 16 * (8 if p["dp"] == 16 else 4)        # rows a workgroup of the symmetric kernel holds
    assert rb & (rb - 1) == 0 and rb % rows_held == 0 and rb % 256 == 0
    assert p["n_pad"] % rb == 0 and p["n_pad"] - n < max(rb, 1024)
    blocks = p["n_pad"] // rb
    assert 1 <= groups <= 64 and per_group >= 1
    assert groups * per_group >= blocks > (groups - 1) * per_group
    assert p["partial_slots"] == groups + 2      # one per group, one more, and the in-block pass
    assert groups * (groups + 1) // 2 >= 512
    assert 4 * ((p["dp"] // 16) * rb * 16 + rb + 8 * 16 * 20) <= 160 * 1024


@settings(max_examples=300, deadline=None)
@given(n=st.integers(1, 3_000_000), m=st.integers(1, 3_000_000), d=st.integers(1, 128), call=st.integers(0, 2),
       flags=st.sampled_from(FLAGS))
def test_plan_covers_everything_and_fits(n, m, d, call, flags):
    _check(n, m, d, call, flags)


@pytest.mark.parametrize("n,m,d", [(4096, 1024, 16), (32768, 32768, 16), (32768, 65536, 1), (262144, 65536, 64),
                                   (1048576, 131072, 16), (1, 1, 1), (1, 1, 128), (17, 3, 4)])
def test_plan_of_the_benchmark_configs(n, m, d):
    for call in range(3):
        p = _check(n, m, d, call, 0)
        if n >= 32768:
            assert p["row_blocks"] * p["splits"] >= 512      # at least two workgroups per compute unit
        if p["splits"] >= 8:
            assert p["splits"] % 8 == 0                       # one group of splits per XCD
    big = P.sdkde_describe_plan(1048576, 131072, 16, 0)
    assert big["row_tiles"] == 8 and big["splits"] == 8
    sym = P.sdkde_describe_plan(1048576, 131072, 16, 0, P.SDKDE_FLAG_SYMMETRIC)
    assert (sym["sym_block_rows"], sym["sym_blocks_per_group"], sym["sym_groups"]) == (2048, 8, 64)


@pytest.mark.parametrize("n,m,d,call", [(20000, 20000, 16, 0), (12288, 12288, 16, 0), (32768, 4096, 16, 0),
                                        (32768, 4096, 16, 2), (262144, 20000, 16, 2), (1048576, 131072, 16, 2),
                                        (262144, 65536, 64, 0), (262144, 65536, 128, 2), (100000, 100000, 16, 0),
                                        (40000, 40000, 32, 0), (50000, 50000, 128, 0)])
def test_plan_fills_the_last_round_of_workgroups(n, m, d, call):
    """The plan is the (row tiles, splits) pair of least estimated time; with enough samples to choose from, the
    workgroups must come close to a whole number of rounds over the 256 compute units (a count just above a
    multiple of 256 would leave most of the chip idle for a round), without paying for more splits than that takes."""
    p = _check(n, m, d, call, 0)
    groups = p["row_blocks"] * p["splits"]
    rounds = -(-groups // 256)
    assert groups >= 512 and groups / (256 * rounds) >= 0.97
    assert p["splits"] % 8 == 0 and p["tiles_per_split"] >= 16
    if call == 0:
        assert p["splits"] <= 32          # every split costs a slot of partial T and D sums


@settings(max_examples=200, deadline=None)
@given(n=st.integers(1, 3_000_000), m=st.integers(1, 3_000_000), d=st.integers(1, 128),
       other=st.sampled_from([0, P.SDKDE_FLAG_MAX_SHIFT, P.SDKDE_FLAG_SYMMETRIC]))
def test_one_workspace_serves_every_precision_mode(n, m, d, other):
    """The decomposition (and the number of partial-sum slots) depends on the precision mode, and the mode of a
    score at separate points on the max-shift flag, so the buffer the binding makes by default must cover the plan
    of every mode and call, with or without the shift and the symmetric flag."""
    size = max(P.workspace_bytes_any_precision(n, m, d, other), P.workspace_bytes_any_precision(n, m, d, other & ~P.SDKDE_FLAG_SYMMETRIC))
    for prec in (P.SDKDE_PREC_FP32, P.SDKDE_PREC_FP16X2, P.SDKDE_PREC_FP16X2_ALL, P.SDKDE_PREC_FP16X2_PHI16):
        for shift in (0, P.SDKDE_FLAG_MAX_SHIFT):
            for flags in (other | prec | shift, (other & ~P.SDKDE_FLAG_SYMMETRIC) | prec | shift):
                for call in range(3):
                    assert P.sdkde_describe_plan(n, m, d, call, flags)["workspace_bytes"] <= size


def test_describe_plan_rejects_bad_arguments():
    for args in ((0, 1, 16, 0, 0), (10, 10, 16, 3, 0), (10, 10, 200, 0, 0), (10, 10, 16, 0, 100)):
        with pytest.raises(P.SdkdeError):
            P.sdkde_describe_plan(*args)


def test_tuning_overrides_change_the_plan_and_are_validated(tuning):
    """sdkde_set_tuning (a test hook of the C ABI) forces one of the plan's choices; values the kernels are not
    built for are ignored, 0 restores the library's own choice, and the library reads no environment."""
    import os
    base = P.sdkde_describe_plan(65536, 65536, 16, 0)
    tuning(P.SDKDE_TUNE_SCORE_ROW_TILES, 2)
    tuning(P.SDKDE_TUNE_SCORE_SPLITS, 24)
    forced = P.sdkde_describe_plan(65536, 65536, 16, 0)
    assert forced["row_tiles"] == 2 and forced["splits"] == 24
    eval_plan = P.sdkde_describe_plan(65536, 4096, 16, 2)
    tuning(P.SDKDE_TUNE_SCORE_ROW_TILES, 3)            # not a count the kernels are built for: ignored
    assert P.sdkde_describe_plan(65536, 65536, 16, 0)["row_tiles"] in (2, 4, 8)
    tuning(P.SDKDE_TUNE_SCORE_ROW_TILES, 0)
    tuning(P.SDKDE_TUNE_SCORE_SPLITS, 0)
    assert P.sdkde_describe_plan(65536, 4096, 16, 2) == eval_plan      # the score knobs leave eval calls alone
    tuning(P.SDKDE_TUNE_SCORE_ROW_TILES, 0)
    tuning(P.SDKDE_TUNE_SCORE_SPLITS, 0)
    assert P.sdkde_describe_plan(65536, 65536, 16, 0) == base
    os.environ["SDKDE_SCORE_SPLIT"] = "24"
    try:
        assert P.sdkde_describe_plan(65536, 65536, 16, 0) == base
    finally:
        del os.environ["SDKDE_SCORE_SPLIT"]
    for knob, value in ((-1, 1), (P.SDKDE_TUNE_SEPARATE_PREP + 1, 1), (0, -5)):
        with pytest.raises(P.SdkdeError) as e:
            P.sdkde_set_tuning(knob, value)
        assert e.value.status == 1

def test_one_call_pass_folds_the_eval_preparation_where_the_layouts_allow(tuning):
    """sdkde_fit_eval prepares the eval pass's operands inside its score epilogue when both passes are on the matrix
    path with d <= 16 and what that launch writes fits where the score pass no longer reads (the prepared queries must fit inside
    the samples' blocked transpose): reported by sdkde_describe_plan, switched off by its tuning knob."""
    fused = lambda n, m, d, flags=0: P.sdkde_describe_plan(n, m, d, 2, flags)["fit_eval_fused_prep"]
    assert fused(4096, 1024, 16) == 1 and fused(1048576, 131072, 16) == 1 and fused(32768, 4096, 16) == 1
    assert fused(5000, 700, 9) == 1
    assert fused(262144, 65536, 64) == 0 and fused(5000, 700, 20) == 0      # measured: it pays at dp = 16 only
    assert fused(4096, 1024, 16, P.SDKDE_PREC_FP16X2) == 1 and fused(4096, 1024, 16, P.SDKDE_PREC_FP16X2_PHI16) == 1
    assert fused(32768, 32768, 16) == 0                    # as many queries as samples: no room for them
    assert fused(32768, 65536, 1) == 0 and fused(3000, 500, 5) == 0      # thin path (either pass)
    assert fused(4096, 1024, 16, P.SDKDE_FLAG_MAX_SHIFT) == 0 and fused(65536, 1024, 16, P.SDKDE_FLAG_SYMMETRIC) == 0
    assert P.sdkde_describe_plan(4096, 1024, 16, 0)["fit_eval_fused_prep"] == 0     # a property of the eval call's plan
    tuning(P.SDKDE_TUNE_SEPARATE_PREP, 1)
    assert fused(4096, 1024, 16) == 0


def test_library_is_rebuilt_when_a_source_changes(tmp_path, monkeypatch):
    """The binding builds before loading whenever the library was built from other sources than the tree holds
    (compared by content, not by time stamp)."""
    from paper_2602_10378_amd import build
    P.load()
    assert not build.is_stale()
    record = open(build.RECORD).read()
    fake = tmp_path / "extra.h"
    fake.write_text("// an edited header\n")
    monkeypatch.setattr(build, "HEADERS", build.HEADERS + [str(fake)])
    assert build.is_stale()
    monkeypatch.undo()
    assert not build.is_stale() and open(build.RECORD).read() == record
