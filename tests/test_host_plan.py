"""Host logic without a GPU: for any sizes the plan's grid covers every evaluation row and every
sample tile exactly once, stays inside the padded arrays, and the workspace blocks do not overlap
and fit in the size that sdkde_workspace_bytes reports."""
import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

import paper_2602_10378_amd as P

FLAGS = [P.SDKDE_PREC_FP32, P.SDKDE_PREC_FP16X2, P.SDKDE_PREC_FP16X2_ALL, P.SDKDE_FLAG_MAX_SHIFT]


def _check(n, m, d, call, flags):
    p = P.sdkde_describe_plan(n, m, d, call, flags)
    rows = n if call == 0 else m
    thin = d <= 3
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
    assert p["workspace_bytes"] <= P.sdkde_workspace_bytes(n, m if call else max(m, 1), d, flags & 15 | flags & 16)
    return p


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
            assert p["row_blocks"] * p["splits"] >= 1024     # enough workgroups for 256 CUs
        if p["splits"] >= 8:
            assert p["splits"] % 8 == 0                       # one group of splits per XCD
    big = P.sdkde_describe_plan(1048576, 131072, 16, 0)
    assert big["row_tiles"] == 8 and big["splits"] == 8


def test_describe_plan_rejects_bad_arguments():
    for args in ((0, 1, 16, 0, 0), (10, 10, 16, 3, 0), (10, 10, 200, 0, 0), (10, 10, 16, 0, 99)):
        with pytest.raises(P.SdkdeError):
            P.sdkde_describe_plan(*args)
