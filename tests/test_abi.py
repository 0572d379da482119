"""The shared library loads without a GPU and exports every function the headers declare."""
import ctypes
import glob
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    names = set()
    for h in glob.glob(os.path.join(ROOT, "include", "*.h")):
        text = re.sub(r"/\*.*?\*/", "", open(h).read(), flags=re.S)
        names |= set(re.findall(r"\b(rlhf_\w+)\s*\(", text))
    return names


def test_library_exports_every_declared_symbol():
    import paper_2409_13221_amd as R
    if not os.path.exists(R.LIB_PATH):          # nothing built yet: build once, then load
        from paper_2409_13221_amd.build import build_library
        build_library(verbose=False)
    L = R.lib()
    names = _declared()
    assert {"rlhf_generate_step", "rlhf_retire", "rlhf_score", "rlhf_run_stage"} <= names
    for n in sorted(names):
        assert isinstance(getattr(L, n), ctypes._CFuncPtr), n


def test_binding_structs_match_header_sizes():
    """Field-by-field sizes of the ctypes mirrors against the C layout rules (a mismatch here
    would corrupt arguments silently)."""
    import paper_2409_13221_amd.binding as B
    assert ctypes.sizeof(B.rlhf_model_cfg) == 8 * 4 + 2 * 4
    assert ctypes.sizeof(B.rlhf_engine_cfg) == 4 + 4 + 8 + 8 * 4 + 2 * 8 + 8  # padding after page_tokens and at the end
    assert ctypes.sizeof(B.rlhf_weights) == 9 * 8
    assert ctypes.sizeof(B.rlhf_step_info) == 6 * 4
    assert ctypes.sizeof(B.rlhf_stage_opts) == 4 * 4 + 5 * 8 + 8
    assert ctypes.sizeof(B.rlhf_stage_stats) == 8 + 3 * 8 + 3 * 8 + 2 * 8 + 8      # fused_used + padding
    assert ctypes.sizeof(B.rlhf_results) == 9 * 8
    assert ctypes.sizeof(B.rlhf_snapshot) == 10 * 4 + 9 * 8 + 3 * 4 + 4
    assert ctypes.sizeof(B.rlhf_kernel_profile) == 2 * 8 + 5 * 8 + 8 + 8


def test_create_rejects_bad_arguments_without_a_gpu():
    """Argument validation happens before any device call."""
    import paper_2409_13221_amd as R
    from workload import CONFIGS
    mc = R.model_cfg_of(CONFIGS["tiny"].model)
    ec = R.rlhf_engine_cfg(16, 1 << 20, 4, 64, 4, 32, 2, 0, 0, 0, None, None)    # max_batch_tokens < max_ctx
    try:
        R.rlhf_create(mc, ec)
        raise AssertionError("expected RLHF_EINVAL")
    except R.RlhfError as e:
        assert e.code == R.RLHF_EINVAL
    mc.head_dim = 48
    ec.max_batch_tokens = 64
    try:
        R.rlhf_create(mc, ec)
        raise AssertionError("expected RLHF_EINVAL")
    except R.RlhfError as e:
        assert e.code == R.RLHF_EINVAL and "attention shape" in str(e)


def test_tall_gemm_tile_walk_covers_every_tile_once_and_keeps_xcds_on_one_panel():
    """Host copy of the workgroup -> tile mapping of the 256 x 256 launches (no GPU): a bijection
    onto the tile grid for ragged and tiny grids; the workgroups that the 8 XCDs run at the same
    position of their walks sit on the same panel of 8 tile rows; an XCD's columns are its own."""
    import paper_2409_13221_amd as R
    for tiles_m, tiles_n in [(24, 48), (24, 16), (24, 86), (3, 17), (1, 125), (9, 125), (11, 3), (1, 1), (33, 9)]:
        grid = R.rlhf_op_gemm_tall_grid(tiles_m, tiles_n)
        assert grid % 8 == 0
        seen, cols_of = {}, {}
        for bid in range(grid):
            t = R.rlhf_op_gemm_tall_tile(bid, tiles_m, tiles_n)
            if t is None:
                continue
            assert 0 <= t[0] < tiles_m and 0 <= t[1] < tiles_n and t not in seen
            seen[t] = bid
            cols_of.setdefault(bid & 7, set()).add(t[1])
        assert len(seen) == tiles_m * tiles_n
        owners = [x for x, cs in cols_of.items() for _ in cs]
        assert len(owners) == tiles_n                      # every tile column belongs to exactly one XCD
        if tiles_n >= 8:
            for slot in range(0, grid // 8, 5):
                panels = {R.rlhf_op_gemm_tall_tile(slot * 8 + x, tiles_m, tiles_n) for x in range(8)}
                panels = {t[0] // 8 for t in panels if t is not None}
                assert len(panels) <= (1 if tiles_n % 8 == 0 else 2)
