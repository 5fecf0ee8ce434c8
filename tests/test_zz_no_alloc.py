"""fl_moe_layout_static, the entry point for callers that cannot allocate: its
tables must equal, bit for bit, those of fl_moe_layout on a context (and the
oracle's), on two calls in a row through the C ABI, the second with a smaller
input of another shape; torch must not see an allocation during the calls."""
import numpy as np
import pytest
import torch

from oracle import oracle as orc
from paper_2510_27656_amd import flmoe, harness
from paper_2510_27656_amd import workloads as wlmod

pytestmark = pytest.mark.gpu


def out_buffers(wl, device="cuda:0"):
    N, E, El, T, K = wl.n_ranks, wl.n_experts, wl.experts_per_rank, wl.tokens, wl.top_k
    shapes = {"counts": (N, E), "dedup_counts": (N, N), "tokens_per_expert": (N, El),
              "send_off": (N, N + 1), "recv_off": (N, N + 1), "expert_off": (N, El + 1),
              "comb_off": (N, N + 1), "comb_pos": (N, T, K), "plan_ok": (N,), "status": (1,)}
    # poisoned, so that an entry the call fails to write is seen
    return {n: torch.full(s, -7, dtype=torch.int32, device=device) for n, s in shapes.items()}


def context_tables(inp, dev, **kw):
    """The same tables from the existing entry point (fl_moe_layout on a context)."""
    sh = harness.make_shuffle(inp, **kw)
    try:
        sh.layout(dev["indices"], dev["num_tokens"])
        torch.cuda.synchronize()
        assert sh.status() == 0
        t = {k: v.cpu().numpy().copy() for k, v in sh.layout_tables().items()}
        cfg = sh.cfg
    finally:
        sh.close()
    return cfg, t


NAMES = {"counts": "C", "dedup_counts": "M", "tokens_per_expert": "G", "send_off": "send_off",
         "recv_off": "recv_off", "expert_off": "expert_off", "comb_off": "comb_off",
         "comb_pos": "comb_pos", "plan_ok": "plan_ok"}


def static_call_and_compare(inp, **kw):
    wl = inp.wl
    dev = harness.to_device(inp)
    cfg, want = context_tables(inp, dev, **kw)
    out = out_buffers(wl)
    torch.cuda.synchronize()
    before = torch.cuda.memory_stats()["allocation.all.allocated"]
    flmoe.fl_moe_layout_static(cfg, dev["indices"], dev["num_tokens"], out)
    after = torch.cuda.memory_stats()["allocation.all.allocated"]
    torch.cuda.synchronize()
    assert after == before, "the call allocated through torch"
    got = {n: t.cpu().numpy() for n, t in out.items()}
    assert got["status"][0] == 0
    for n, m in NAMES.items():
        if n == "comb_pos":          # rows of absent tokens are not written by either entry point
            for s in range(wl.n_ranks):
                k = inp.num_tokens[s]
                assert (got[n][s, :k] == want[m][s, :k]).all(), (n, s)
                assert (got[n][s, k:] == -7).all(), "comb_pos of absent tokens was written"
        else:
            assert (got[n] == want[m]).all(), n
    # and against the oracle directly
    lay = orc.layout(wl.n_ranks, wl.n_experts, wl.top_k, inp.num_tokens, inp.indices,
                     kw.get("expert_align", 1))
    assert (got["counts"] == lay.C).all() and (got["dedup_counts"] == lay.M).all()
    assert (got["tokens_per_expert"] == lay.G).all() and (got["expert_off"] == lay.expert_off).all()
    assert (got["send_off"] == lay.send_off).all() and (got["recv_off"] == lay.recv_off).all()
    assert (got["comb_off"] == lay.comb_off).all()
    ref_pos = orc.comb_pos(wl.n_ranks, wl.n_experts, wl.top_k, inp.num_tokens, inp.indices)
    for s in range(wl.n_ranks):
        k = inp.num_tokens[s]
        assert (got["comb_pos"][s, :k] == ref_pos[s, :k]).all()


def test_two_calls_in_a_row_second_one_smaller():
    big = wlmod.make_inputs(wlmod.custom("static_a", 8, 64, 300, 64, 6, seed=41, ragged=True))
    small = wlmod.make_inputs(wlmod.custom("static_b", 4, 32, 50, 64, 4, seed=42, ragged=True))
    static_call_and_compare(big)
    static_call_and_compare(small)                 # other N: the old counters must not be trusted
    static_call_and_compare(big, expert_align=16)  # and back, with padding between experts


def test_decode_shape_fits_and_matches():
    static_call_and_compare(wlmod.make_inputs(wlmod.WORKLOADS["dsv3_decode"]))


def test_bad_index_and_capacity_are_reported_in_the_callers_status_word():
    inp = wlmod.make_inputs(wlmod.custom("static_c", 4, 32, 50, 64, 4, seed=43))
    dev = harness.to_device(inp)
    cfg, _ = context_tables(inp, dev)
    bad = dev["indices"].clone()
    bad[2, 7, 1] = 32                              # outside [0, E)
    out = out_buffers(inp.wl)
    flmoe.fl_moe_layout_static(cfg, bad, dev["num_tokens"], out)
    torch.cuda.synchronize()
    assert int(out["status"][0]) == flmoe.FL_STATUS_BAD_INDEX
    assert (out["plan_ok"].cpu().numpy() == 0).all()
    # the next call starts from a clean status word and clean counters
    flmoe.fl_moe_layout_static(cfg, dev["indices"], dev["num_tokens"], out)
    torch.cuda.synchronize()
    assert int(out["status"][0]) == 0 and (out["plan_ok"].cpu().numpy() == 1).all()
    tight = flmoe.fl_moe_config.from_buffer_copy(cfg)
    tight.recv_capacity_rows = 3
    flmoe.fl_moe_layout_static(tight, dev["indices"], dev["num_tokens"], out)
    torch.cuda.synchronize()
    assert int(out["status"][0]) == flmoe.FL_STATUS_CAPACITY
    assert (out["plan_ok"].cpu().numpy() == 0).all()


def test_sizes_beyond_the_static_array_are_refused():
    wl = wlmod.WORKLOADS["dsv3_prefill"]           # 4096 tokens per rank: per-pair tables of 8 MB
    cfg = flmoe.fl_moe_config(wl.n_ranks, wl.n_experts, wl.tokens, wl.top_k, wl.hidden, 0, 1, 0,
                              wl.tokens * 9, wl.tokens * 9, 0, 0, 0)
    one = torch.zeros(4, dtype=torch.int32, device="cuda:0")
    out = {n: one for n in flmoe.LAYOUT_OUT_FIELDS}
    with pytest.raises(flmoe.FlMoeError) as e:
        flmoe.fl_moe_layout_static(cfg, one, one, out)
    assert e.value.code == flmoe.FL_ERR_STATIC_LIMIT
    assert "static" in str(e.value)
