"""Host-side checks of the C ABI: the library loads, exports every symbol that
include/flmoe.h declares, and its host-only entry points validate arguments.
No kernel is launched here."""
import ctypes as C
import os
import re

import pytest

from paper_2510_27656_amd import flmoe

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "flmoe.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fl_moe_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_symbols()
    assert "fl_moe_layout" in names and "fl_moe_combine_reduce" in names and len(names) >= 12
    L = flmoe.lib()
    for n in names:
        assert hasattr(L, n), n
    assert sorted(flmoe.EXPORTS) == names


def cfg(**kw):
    base = dict(n_ranks=32, n_experts=256, max_tokens=128, top_k=8, hidden=7168,
                dispatch_dtype=0, expert_align=1, flags=0, recv_capacity_rows=0,
                expert_capacity_rows=0, spin_limit=0)
    base.update(kw)
    return flmoe.fl_moe_config(**base)


def test_query_sizes_decode_shape():
    s = flmoe.fl_moe_query_sizes(cfg())
    assert s.x_row_bytes == 14336 and s.wire_row_bytes == 14336 and s.combine_row_bytes == 14336
    assert s.recv_capacity_rows == 32 * 128
    assert s.expert_capacity_rows == 32 * 128 * 8
    assert s.send_capacity_rows == 128 * 8
    assert s.workspace_bytes % 256 == 0
    # the two staging buffers dominate: send/combine-receive and receive/combine-send
    assert s.workspace_bytes >= 32 * (1024 * 14336 + 32768 * 14336)
    s8 = flmoe.fl_moe_query_sizes(cfg(dispatch_dtype=1))
    assert s8.wire_row_bytes == 7424 and s8.scales_per_row == 56      # 7168 + 4*56 = 7392, on 128-byte lines
    assert s8.expert_x_row_bytes == 7168


def test_capacities_are_clamped_and_padding_counted():
    s = flmoe.fl_moe_query_sizes(cfg(expert_align=16, expert_capacity_rows=0))
    assert s.expert_capacity_rows == 32 * 128 * 8 + 7 * 15
    s = flmoe.fl_moe_query_sizes(cfg(recv_capacity_rows=10 ** 9, expert_capacity_rows=2000))
    assert s.recv_capacity_rows == 32 * 128 and s.expert_capacity_rows == 2000


def test_private_rows_extend_the_receive_buffer():
    base = flmoe.fl_moe_query_sizes(cfg())
    assert base.private_rows == 0 and base.recv_buffer_rows == base.recv_capacity_rows
    s = flmoe.fl_moe_query_sizes(cfg(max_private_rows=32))
    assert s.private_rows == 32
    assert s.recv_buffer_rows == 32 * 32 + s.recv_capacity_rows
    assert s.workspace_bytes > base.workspace_bytes
    # a source never sends more than T rows to one destination
    s = flmoe.fl_moe_query_sizes(cfg(max_private_rows=10 ** 6))
    assert s.private_rows == 128
    # the shared range can then be configured smaller
    s = flmoe.fl_moe_query_sizes(cfg(max_private_rows=32, recv_capacity_rows=1024))
    assert s.recv_buffer_rows == 32 * 32 + 1024


@pytest.mark.parametrize("bad,code", [
    (dict(n_ranks=0), flmoe.FL_ERR_INVALID_ARG),
    (dict(n_ranks=65, n_experts=65), flmoe.FL_ERR_INVALID_ARG),
    (dict(n_experts=250), flmoe.FL_ERR_INVALID_ARG),
    (dict(top_k=17), flmoe.FL_ERR_INVALID_ARG),
    (dict(top_k=0), flmoe.FL_ERR_INVALID_ARG),
    (dict(hidden=100), flmoe.FL_ERR_ALIGNMENT),
    (dict(hidden=(1 << 20) + 8), flmoe.FL_ERR_INVALID_ARG),
    (dict(hidden=192, dispatch_dtype=1), flmoe.FL_ERR_ALIGNMENT),
    (dict(dispatch_dtype=7), flmoe.FL_ERR_INVALID_ARG),
    (dict(expert_align=0), flmoe.FL_ERR_INVALID_ARG),
    (dict(flags=32), flmoe.FL_ERR_INVALID_ARG),
    (dict(flags=flmoe.FL_FLAG_STREAM_ORDERED | flmoe.FL_FLAG_PROGRESSIVE_RECV), flmoe.FL_ERR_INVALID_ARG),
    (dict(max_tokens=0), flmoe.FL_ERR_INVALID_ARG),
    (dict(max_private_rows=-1), flmoe.FL_ERR_INVALID_ARG),
    (dict(reserved=1), flmoe.FL_ERR_INVALID_ARG),
])
def test_query_sizes_rejects_bad_configs(bad, code):
    with pytest.raises(flmoe.FlMoeError) as ei:
        flmoe.fl_moe_query_sizes(cfg(**bad))
    assert ei.value.code == code


def test_null_arguments_are_errors_not_crashes():
    L = flmoe.lib()
    assert L.fl_moe_query_sizes(None, None) == flmoe.FL_ERR_INVALID_ARG
    assert L.fl_moe_destroy(None) == flmoe.FL_ERR_INVALID_ARG
    assert L.fl_moe_layout(None, 0, 1, None, None, None, None) == flmoe.FL_ERR_INVALID_ARG
    assert L.fl_moe_dispatch_send(None, 0, 1, None, None) == flmoe.FL_ERR_INVALID_ARG
    assert L.fl_moe_status(None, None, None) == flmoe.FL_ERR_INVALID_ARG
    assert L.fl_moe_required_capacities(None, None, None, None) == flmoe.FL_ERR_INVALID_ARG
    assert L.fl_moe_strerror(flmoe.FL_ERR_WORKSPACE) == b"workspace too small"
    names = [L.fl_moe_kernel_name(i).decode() for i in range(flmoe.FL_KERNEL_COUNT)]
    assert all(names) and len(set(names)) == flmoe.FL_KERNEL_COUNT


def test_large_calls_are_cut_into_rank_groups_small_ones_are_not():
    """Host rule behind the launches of a payload call: one launch while the ranks of the
    call move at most three times the per-launch target (860 MiB by default), otherwise
    groups of ranks of about the target size; row = the larger of wire and combine row."""
    groups = flmoe.fl_moe_debug_launch_groups
    dsv3 = dict(n_ranks=32, n_experts=256, top_k=8, hidden=7168)
    per_rank_128 = 128 * 8 * 14336
    assert per_rank_128 * 32 <= 3 * (860 << 20)
    assert groups(cfg(max_tokens=128, **dsv3), 32) == 32          # decode: 470 MB, one launch
    assert groups(cfg(max_tokens=512, **dsv3), 32) == 32          # 1.9 GB: still one launch
    assert groups(cfg(max_tokens=1024, **dsv3), 32) == 7          # 3.8 GB -> 5 launches
    assert groups(cfg(max_tokens=2048, **dsv3), 32) == 4
    assert groups(cfg(max_tokens=4096, **dsv3), 32) == 2          # prefill: 16 launches of 2 ranks
    assert groups(cfg(max_tokens=4096, **dsv3), 1) == 1           # one real rank's call is never cut
    assert groups(cfg(max_tokens=4096, **dsv3), 32, 0) == 32      # knob 0: never cut
    assert groups(cfg(max_tokens=128, **dsv3), 32, 1) == 1        # tiny target: one rank per launch
    assert groups(cfg(max_tokens=1 << 20, **dsv3), 32) == 1       # never below one rank
    assert groups(cfg(max_tokens=4096, flags=flmoe.FL_FLAG_STREAM_ORDERED, **dsv3), 32) == 2
    assert groups(cfg(max_tokens=4096, flags=flmoe.FL_FLAG_PROGRESSIVE_RECV, **dsv3), 32) == 32   # polling receivers: never cut
    # e4m3 dispatch: the combine row (bf16) is the larger one and decides
    assert groups(cfg(max_tokens=4096, dispatch_dtype=flmoe.FL_DTYPE_E4M3_BLOCK128, **dsv3), 32) == 2
    lib = flmoe.lib()
    out = C.c_int(0)
    c = cfg(max_tokens=128, **dsv3)
    assert lib.fl_moe_debug_launch_groups(C.byref(c), 0, -1, C.byref(out)) == flmoe.FL_ERR_INVALID_ARG
    assert lib.fl_moe_debug_launch_groups(C.byref(c), 33, -1, C.byref(out)) == flmoe.FL_ERR_INVALID_ARG
    assert lib.fl_moe_debug_launch_groups(C.byref(c), 32, -1, None) == flmoe.FL_ERR_INVALID_ARG


def test_static_layout_entry_point_checks_its_arguments_before_touching_a_gpu():
    """fl_moe_layout_static validates on the host first: null or misaligned pointers, bad
    configurations and configurations beyond its static scratch array are refused without
    any device call (so this runs without a GPU)."""
    L = flmoe.lib()
    small = cfg(n_ranks=4, n_experts=32, max_tokens=64, top_k=4, hidden=256)
    fake = 0x1000                                   # never dereferenced: every call below fails earlier
    out = flmoe.fl_moe_layout_out(*([fake] * len(flmoe.LAYOUT_OUT_FIELDS)))
    assert L.fl_moe_layout_static(None, fake, fake, C.byref(out), None) == flmoe.FL_ERR_INVALID_ARG
    assert L.fl_moe_layout_static(C.byref(small), None, fake, C.byref(out), None) == flmoe.FL_ERR_INVALID_ARG
    assert L.fl_moe_layout_static(C.byref(small), fake, fake, None, None) == flmoe.FL_ERR_INVALID_ARG
    hole = flmoe.fl_moe_layout_out(*([fake] * (len(flmoe.LAYOUT_OUT_FIELDS) - 1) + [None]))
    assert L.fl_moe_layout_static(C.byref(small), fake, fake, C.byref(hole), None) == flmoe.FL_ERR_INVALID_ARG
    odd = flmoe.fl_moe_layout_out(*([fake + 2] + [fake] * (len(flmoe.LAYOUT_OUT_FIELDS) - 1)))
    assert L.fl_moe_layout_static(C.byref(small), fake, fake, C.byref(odd), None) == flmoe.FL_ERR_ALIGNMENT
    assert L.fl_moe_layout_static(C.byref(small), fake + 1, fake, C.byref(out), None) == flmoe.FL_ERR_ALIGNMENT
    bad = cfg(n_ranks=4, n_experts=30)
    assert L.fl_moe_layout_static(C.byref(bad), fake, fake, C.byref(out), None) == flmoe.FL_ERR_INVALID_ARG
    # the decode shape fits the array, the 4096-token shape does not (per-pair tables of 8 MB)
    big = cfg(max_tokens=4096)
    assert L.fl_moe_layout_static(C.byref(big), fake, fake, C.byref(out), None) == flmoe.FL_ERR_STATIC_LIMIT
    assert b"static" in L.fl_moe_strerror(flmoe.FL_ERR_STATIC_LIMIT)
    assert flmoe.FL_STATIC_SCRATCH_BYTES == 8 << 20


def test_loaded_library_was_built_from_the_sources_in_the_tree():
    from paper_2510_27656_amd import build
    assert flmoe.fl_moe_build_id() == build.source_hash() and len(build.source_hash()) == 16
