"""Parity of the HIP path (through the C ABI) against the CPU oracle, element by
element, on the same seeded inputs.

Bars: bit-exact for counts, offsets, positions and dispatched rows; combined
output within 1 bf16 step of the oracle (fp32 fused multiply-add in k order on
both sides, so bit-equality is expected and its fraction is reported).
"""
import numpy as np
import pytest
import torch

from oracle import oracle as orc
from oracle.reference_step import oracle_step
from paper_2510_27656_amd import flmoe, harness
from paper_2510_27656_amd import workloads as wlmod

pytestmark = pytest.mark.gpu

POISON = 0x7FC1          # a bf16 NaN pattern no computation here produces


def bits(t):
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def ulp_distance(a_bits, b_bits):
    def key(b):
        b = b.astype(np.int32)
        return np.where(b & 0x8000, -(b & 0x7fff), b & 0x7fff)
    return np.abs(key(a_bits) - key(b_bits))


def check_tables(sh, ref, N):
    tabs = {k: v.cpu().numpy() for k, v in sh.layout_tables().items()}
    assert (tabs["plan_ok"] == 1).all()
    assert (tabs["C"] == ref.lay.C).all()
    assert (tabs["M"] == ref.lay.M).all()
    assert (tabs["G"] == ref.lay.G).all()
    assert (tabs["send_off"] == ref.lay.send_off).all()
    assert (tabs["recv_off"] == ref.lay.recv_off).all()
    assert (tabs["expert_off"] == ref.lay.expert_off).all()
    assert (tabs["comb_off"] == ref.lay.comb_off).all()
    return tabs


def run_and_compare(inp, align=1, zero_pad=False, capacity_factor=None, ranks_split=False,
                    ordering="counters", private_rows=0, push=False, partial=False, launch_mb=None,
                    capacities=None):
    """ordering: "counters" = the default mode (the arrival counters are the only ordering:
    announce and gate kernels), "stream" = FL_FLAG_STREAM_ORDERED, "progressive" =
    FL_FLAG_PROGRESSIVE_RECV."""
    wl = inp.wl
    N, T = wl.n_ranks, wl.tokens
    ref = oracle_step(inp, align, zero_pad=True, partial=partial)
    if partial:                      # the combined output follows the partial-sum definition
        ref.out = ref.out_partial
    dev = harness.to_device(inp)
    sh = harness.make_shuffle(inp, expert_align=align, zero_pad=zero_pad, partial_sums=partial,
                              capacity_factor=capacity_factor, capacities=capacities,
                              stream_ordered=ordering == "stream",
                              progressive_recv=ordering == "progressive",
                              max_private_rows=private_rows, peer_push=push)
    try:
        if launch_mb is not None:        # payload per launch above which a call is cut into rank groups
            flmoe.fl_moe_debug_tune(sh.ctx, 6, launch_mb)
        if wl.dispatch_dtype == "bf16":
            sh.expert_x.view(torch.int16).fill_(POISON)
        sh.out.view(torch.int16).fill_(POISON)
        identity = wl.expert == "identity"
        if not ranks_split:
            out = harness.run_step(sh, dev, identity)
        else:
            h = N // 2
            sh.layout(dev["indices"], dev["num_tokens"])
            for rg in [(h, N - h), (0, h)]:
                sh.dispatch_send(dev["x"], rg, weights=harness.send_weights(sh, dev))
            for rg in [(0, h), (h, N - h)]:
                sh.dispatch_recv(rg)
            y = harness.expert_stage(sh, dev["gain"], identity)
            for rg in [(h, N - h), (0, h)]:
                sh.combine_send(y, rg)
            for rg in [(0, h), (h, N - h)]:
                sh.combine_reduce(dev["weights"], rg)
            out = sh.out
        torch.cuda.synchronize()
        assert sh.status() == 0
        tabs = check_tables(sh, ref, N)
        assert (sh.tokens_per_expert.cpu().numpy() == ref.lay.G).all()
        # combine-receive positions of valid tokens
        cp = tabs["comb_pos"]
        for s in range(N):
            n = inp.num_tokens[s]
            assert (cp[s, :n] == ref.comb_pos[s, :n]).all()
        # dispatched rows, bit for bit; padding and unused capacity as specified
        fp8 = wl.dispatch_dtype == "e4m3"
        if fp8:
            ex = sh.expert_x[:, :ref.stride].cpu().numpy()
            exs = sh.expert_scales[:, :ref.stride].cpu().numpy().view(np.uint32)
            for d in range(N):
                n = ref.expert_rows[d].shape[0]
                assert (ex[d, :n] == ref.expert_rows[d]).all(), f"e4m3 bytes, rank {d}"
                assert (exs[d, :n] == ref.expert_scales[d].view(np.uint32)).all(), f"scales, rank {d}"
        else:
            ex = bits(sh.expert_x[:, :ref.stride])
            exi = sh.expert_x.view(torch.int16)
        for d in range(N if not fp8 else 0):
            rows = ref.expert_rows[d]
            n = rows.shape[0]
            if zero_pad:
                assert (ex[d, :n] == rows).all(), f"rank {d}"
            else:
                for j in range(wl.experts_per_rank):
                    lo = ref.lay.expert_off[d, j]
                    hi = lo + ref.lay.G[d, j]
                    assert (ex[d, lo:hi] == rows[lo:hi]).all(), f"rank {d} expert {j}"
                    if j + 1 < wl.experts_per_rank:
                        assert (ex[d, hi:ref.lay.expert_off[d, j + 1]] == POISON).all()
            assert bool((exi[d, n:] == POISON).all()), "rows beyond the layout were written"
        # combined output
        ob = bits(out)
        worst, exact, total = 0, 0, 0
        for s in range(N):
            n = inp.num_tokens[s]
            dist = ulp_distance(ob[s, :n], ref.out[s, :n])
            if dist.size:
                worst = max(worst, int(dist.max()))
                exact += int((dist == 0).sum())
                total += dist.size
            assert (ob[s, n:] == POISON).all(), "rows of absent tokens were written"
        assert worst <= 1, f"max bf16 ulp distance {worst}"
        print(f"[{wl.name}] combine: max ulp {worst}, bit-exact {exact}/{total}")
        assert exact == total          # same arithmetic on both sides: expected identical
        return sh, dev, ob
    except Exception:
        sh.close()
        raise


CASES = {
    "tiny": lambda: wlmod.WORKLOADS["tiny"],
    "ragged_520": lambda: wlmod.custom("ragged_520", 4, 32, 100, 520, 4, seed=11, ragged=True),
    "one_expert_per_rank": lambda: wlmod.custom("el1", 8, 8, 33, 264, 5, seed=12, ragged=True),
    "k_lt_el": lambda: wlmod.custom("el32", 2, 64, 50, 128, 8, seed=13),
    "single_rank": lambda: wlmod.custom("n1", 1, 16, 77, 256, 4, seed=14),
    "top1": lambda: wlmod.custom("k1", 4, 16, 64, 256, 1, seed=15),
    "multi_tile": lambda: wlmod.custom("tiles", 4, 32, 2500, 64, 4, seed=16, ragged=True),
    "k16": lambda: wlmod.custom("k16", 4, 64, 40, 128, 16, seed=17),
}


@pytest.mark.parametrize("name", list(CASES))
def test_parity_small(name):
    inp = wlmod.make_inputs(CASES[name]())
    sh, _, _ = run_and_compare(inp)
    sh.close()


@pytest.mark.parametrize("align,zero_pad", [(16, True), (16, False), (3, True)])
def test_parity_with_padding(align, zero_pad):
    inp = wlmod.make_inputs(CASES["ragged_520"]())
    sh, _, _ = run_and_compare(inp, align=align, zero_pad=zero_pad)
    sh.close()


@pytest.mark.parametrize("form", ["stream", "progressive"])
@pytest.mark.parametrize("name", ["ragged_520", "multi_tile", "k16"])
def test_parity_in_the_other_ordering_modes(name, form):
    """Same results when the caller orders sends before receives itself and the library
    skips the announce and gate kernels (FL_FLAG_STREAM_ORDERED), and with receive
    kernels that poll themselves (FL_FLAG_PROGRESSIVE_RECV)."""
    inp = wlmod.make_inputs(CASES[name]())
    sh, _, _ = run_and_compare(inp, ordering=form)
    sh.close()


def test_rank_subsets_give_the_same_result():
    inp = wlmod.make_inputs(CASES["ragged_520"]())
    sh, _, _ = run_and_compare(inp, ranks_split=True)
    sh.close()


def test_repeated_steps_are_deterministic_and_counters_monotone():
    inp = wlmod.make_inputs(CASES["ragged_520"]())
    sh, dev, first = run_and_compare(inp)
    try:
        for it in range(3):
            out = harness.run_step(sh, dev, identity=False)
            torch.cuda.synchronize()
            assert (bits(out) == first).all()
        dbg = sh.debug()
        assert (dbg["epoch_route"].cpu().numpy() == 4).all()
        assert (dbg["arrive_route"].cpu().numpy() == 4).all()
        # payload counters: delivered == expected, 4 steps x (rows x 16-byte units per row, plus
        # one per transfer, empty ones included)
        units = inp.wl.hidden * 2 // 16
        ref = oracle_step(inp)
        want_disp = 4 * (ref.lay.M.T.astype(np.int64) * units + 1)      # [dst][src]
        pairs = ref.lay.C.reshape(inp.wl.n_ranks, inp.wl.n_ranks, -1).sum(2)   # [src][owner]
        assert (dbg["arrive_disp"].cpu().numpy() == want_disp).all()
        assert (dbg["expect_disp"].cpu().numpy() == want_disp).all()
        assert (dbg["arrive_comb"].cpu().numpy() == 4 * (pairs * units + 1)).all()
        assert (dbg["expect_comb"].cpu().numpy() == 4 * (pairs * units + 1)).all()
        assert sh.status() == 0
    finally:
        sh.close()


@pytest.mark.parametrize("kw", [dict(), dict(stream_ordered=True), dict(peer_push=True, partial_sums=True),
                                dict(progressive_recv=True)])
def test_counters_wrap_around_32_bits(kw):
    """The arrival and expectation counters are monotone 32-bit words compared
    wrap-safely: set just below 2^32 (consistently, as after very many steps), the
    next steps carry them across zero without a time-out or a wrong row."""
    inp = wlmod.make_inputs(CASES["ragged_520"]())
    dev = harness.to_device(inp)
    partial = kw.get("partial_sums", False)
    ref = oracle_step(inp, partial=partial)
    want = ref.out_partial if partial else ref.out
    sh = harness.make_shuffle(inp, **kw)
    try:
        dbg = sh.debug()
        near = 0xFFFFFFFF - 1000                   # a step adds tens of thousands of units
        for name in ("arrive_disp", "expect_disp", "arrive_comb", "expect_comb"):
            dbg[name].view(torch.int32).fill_(near - (1 << 32))
        for name in ("arrive_route", "epoch_route"):
            dbg[name].view(torch.int32).fill_(-2)  # 0xFFFFFFFE: wraps on the second step
        for step in range(4):
            sh.out.view(torch.int16).fill_(POISON)
            out = harness.run_step(sh, dev)
            torch.cuda.synchronize()
            assert sh.status() == 0, step
            ob = bits(out)
            for s in range(inp.wl.n_ranks):
                n = inp.num_tokens[s]
                assert (ob[s, :n] == want[s, :n]).all(), (step, s)
        after = sh.debug()
        assert (after["arrive_disp"] == after["expect_disp"]).all()
        assert (after["arrive_comb"] == after["expect_comb"]).all()
        assert int(after["epoch_route"].view(torch.int32)[0]) == 2         # -2 + 4 steps
        unsigned = after["arrive_disp"].long().cpu().numpy() & 0xFFFFFFFF
        assert (unsigned[ref.lay.M.T > 0] < near).all()                    # they did pass zero
    finally:
        sh.close()


def test_round_trip_identity_returns_input():
    wl = wlmod.custom("rt", 8, 64, 48, 512, 8, seed=21, expert="identity")
    inp = wlmod.make_inputs(wl)
    sh, dev, ob = run_and_compare(inp)
    try:
        assert (ob == inp.x).all()
    finally:
        sh.close()


@pytest.mark.parametrize("name", ["qwen3_skew", "dsv3_decode"])
def test_parity_named_workloads(name):
    inp = wlmod.make_inputs(wlmod.WORKLOADS[name])
    sh, _, _ = run_and_compare(inp)
    sh.close()


FP8_CASES = {
    "fp8_small": lambda: wlmod.custom("fp8_small", 4, 32, 60, 512, 4, seed=31, ragged=True,
                                      dispatch_dtype="e4m3"),
    "fp8_one_block": lambda: wlmod.custom("fp8_one_block", 2, 8, 16, 128, 2, seed=32,
                                          dispatch_dtype="e4m3", expert="identity"),
    "fp8_k16": lambda: wlmod.custom("fp8_k16", 4, 64, 40, 2304, 16, seed=33, dispatch_dtype="e4m3"),
}


@pytest.mark.parametrize("name", list(FP8_CASES))
def test_parity_e4m3_dispatch_small(name):
    inp = wlmod.make_inputs(FP8_CASES[name]())
    sh, _, _ = run_and_compare(inp, zero_pad=True, align=4)
    sh.close()


def test_parity_e4m3_dispatch_edge_values():
    """Blocks of zeros, tiny and huge magnitudes, exact ties: same codes and scales."""
    wl = wlmod.custom("fp8_edges", 2, 8, 32, 256, 2, seed=34, dispatch_dtype="e4m3")
    inp = wlmod.make_inputs(wl)
    x = inp.x.reshape(-1, 128)
    f = lambda v: torch.tensor(v, dtype=torch.float32).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    x[0] = 0                                             # all-zero block: scale 1
    x[1] = f([1e-38] * 128)                               # scale is a subnormal fp32
    x[2] = f([3e38] * 64 + [-3e38] * 64)                  # near the top of the range
    x[3] = f([448.0] + [v * 448.0 / 16 for v in range(1, 128)])   # many exact multiples and ties
    x[4] = f([1.0] + [2.0 ** -e for e in range(1, 128)])  # deep into the subnormal e4m3 range
    x[5] = f([-0.0] * 127 + [5.0])
    sh, _, _ = run_and_compare(inp, zero_pad=True)
    sh.close()


def test_parity_e4m3_dispatch_every_finite_bf16_value():
    """All 65 280 finite bf16 bit patterns, each quantised against several block maxima
    (from its own magnitude up to 2^20 times larger: top codes, low codes, subnormal
    codes, zero) and once in random company: same codes and scales as the oracle."""
    wl = wlmod.custom("fp8_all_values", 2, 8, 64, 3200, 2, seed=35, dispatch_dtype="e4m3")
    inp = wlmod.make_inputs(wl)
    x = inp.x.reshape(-1, 128)
    assert x.shape[0] == 3200
    pats = np.arange(65536, dtype=np.uint32)
    pats = pats[(pats & 0x7f80) != 0x7f80].astype(np.uint16)          # finite values only
    mag = (pats & 0x7fff).astype(np.int32)
    pats = pats[np.argsort(mag, kind="stable")]                        # by magnitude, signs alternate
    chunks = [pats[i:i + 127] for i in range(0, len(pats), 127)]
    as_f32 = lambda b: (b.astype(np.uint32) << 16).view(np.float32)
    to_bf16 = lambda v: torch.tensor(v, dtype=torch.float32).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    row = 0
    for mult in (1.0, 3.0, 37.0, 1000.0, 2.0 ** 20):
        for c in chunks:
            top = float(np.abs(as_f32(c)).max())
            setter = to_bf16([min(top * mult, 3.0e38)])[0]
            x[row, :len(c)] = c
            x[row, len(c):] = setter
            row += 1
    rng = np.random.default_rng(35)
    mixed = rng.permutation(pats)
    for i in range(0, len(mixed), 127):
        c = mixed[i:i + 127]
        x[row, :len(c)] = c
        x[row, len(c):] = 0
        row += 1
    assert row <= 3200
    x[row:] = 0
    sh, _, _ = run_and_compare(inp, zero_pad=True)
    sh.close()


@pytest.mark.parametrize("kw", [dict(), dict(peer_push=True), dict(stream_ordered=True)])
def test_parity_e4m3_dispatch_blocks_with_inf_and_nan(kw):
    """Blocks that hold Inf or NaN (every non-finite bf16 pattern, quiet and signalling,
    both signs): codes and scales equal the oracle's, code for code and scale for scale.
    The rule both sides follow: a NaN is skipped by the block maximum and becomes the NaN
    code with its own sign; an Inf makes the block's scale +Inf, its finite neighbours
    signed zeros and itself the NaN code with its sign.  Only the dispatch is compared:
    what an expert makes of NaN inputs is not the shuffle's business."""
    wl = wlmod.custom("fp8_nonfinite", 2, 8, 32, 512, 2, seed=36, dispatch_dtype="e4m3")
    inp = wlmod.make_inputs(wl)
    x = inp.x.reshape(-1, 128)                     # 256 blocks, four per token
    nonfinite = np.array([p for p in range(65536) if (p & 0x7f80) == 0x7f80], np.uint16)
    assert len(nonfinite) == 256
    rng = np.random.default_rng(36)
    for b in range(0, 128):                        # two non-finite patterns among random finite values
        x[b, rng.integers(0, 128)] = nonfinite[2 * b]
        x[b, rng.integers(0, 128)] = nonfinite[2 * b + 1]
    x[128] = 0x7fc0                                # a block of NaNs only: scale 1
    x[129] = 0x7f80                                # +Inf only
    x[130, ::2] = 0xff80                           # -Inf among finite values, many of them
    x[131, :64] = 0xffc1                           # half NaN, half finite
    x[132, 5] = 0x7f80; x[132, 6] = 0x7fa0         # Inf and a signalling NaN in one block
    x[133, 0] = 0x7f81                             # a signalling NaN as the first element
    x[134, 127] = 0xff81                           # ... and as the last
    x[135, :127] = 0; x[135, 127] = 0x7fc0         # zeros and one NaN: amax 0, scale 1
    ref = oracle_step(inp)
    infs = sum(int(np.isinf(r).sum()) for r in ref.expert_scales)
    nan_codes = sum(int(((r & 0x7f) == 0x7f).sum()) for r in ref.expert_rows)
    assert infs > 0 and nan_codes > 256, "the case does not exercise what it is for"
    dev = harness.to_device(inp)
    sh = harness.make_shuffle(inp, **kw)
    try:
        sh.layout(dev["indices"], dev["num_tokens"])
        sh.dispatch_send(dev["x"])
        sh.dispatch_recv()
        torch.cuda.synchronize()
        assert sh.status() == 0
        ex = sh.expert_x.cpu().numpy()
        exs = sh.expert_scales.cpu().numpy().view(np.uint32)
        for d in range(wl.n_ranks):
            n = ref.expert_rows[d].shape[0]
            assert (ex[d, :n] == ref.expert_rows[d]).all(), f"e4m3 codes, rank {d}"
            assert (exs[d, :n] == ref.expert_scales[d].view(np.uint32)).all(), f"scales, rank {d}"
    finally:
        sh.close()


def test_parity_named_workload_dsv3_fp8():
    inp = wlmod.make_inputs(wlmod.WORKLOADS["dsv3_fp8"])
    sh, _, _ = run_and_compare(inp)
    sh.close()


def test_prefill_full_shape():
    """The 4096-tokens-per-rank workload at its real shape (buffers of 16 GB, byte
    offsets beyond 2^31).  Tables are compared in full; every dispatched row is
    compared on the GPU against the input row at the slot the oracle computed; the
    combined output of all 131 072 tokens is compared with the oracle, rank by rank."""
    wl = wlmod.WORKLOADS["dsv3_prefill"]
    print("drawing inputs ...", flush=True)
    inp = wlmod.make_inputs(wl)
    N, E, K, H, T = wl.n_ranks, wl.n_experts, wl.top_k, wl.hidden, wl.tokens
    El = E // N
    print("oracle layout ...", flush=True)
    lay = orc.layout(N, E, K, inp.num_tokens, inp.indices)
    comb_pos = orc.comb_pos(N, E, K, inp.num_tokens, inp.indices)
    dev = harness.to_device(inp)
    sh = harness.make_shuffle(inp, capacity_factor=1.1)
    try:
        print("gpu step ...", flush=True)
        out = harness.run_step(sh, dev)
        torch.cuda.synchronize()
        assert sh.status() == 0
        tabs = {k: v.cpu().numpy() for k, v in sh.layout_tables().items()}
        for name, want in [("C", lay.C), ("M", lay.M), ("G", lay.G), ("send_off", lay.send_off),
                           ("recv_off", lay.recv_off), ("expert_off", lay.expert_off),
                           ("comb_off", lay.comb_off), ("comb_pos", comb_pos)]:
            assert (tabs[name] == want).all(), name
        assert (sh.tokens_per_expert.cpu().numpy() == lay.G).all()
        print("rows ...", flush=True)
        slot = torch.from_numpy(lay.slot).to("cuda:0").long()
        owner = (dev["indices"] // El).long()
        for s in range(N):
            got = sh.expert_x[owner[s], slot[s]]                    # [T][K][H]
            assert bool((got.view(torch.int16) == dev["x"][s].view(torch.int16)[:, None, :]).all()), s
            del got
        # every row of the layout is one of those pairs: counts already match (G, expert_off)
        # Combined output of every token, source rank by source rank (section Kernel
        # Microbenchmarks: 4096-token prefill chunks; section Combine): the oracle's combine
        # over the rank's 4096 tokens, fed with the expert output of each pair computed
        # from the token's own row (32 768 rows of 14 KB per rank on the host).
        print("combine on every token, rank by rank ...", flush=True)
        ob = bits(out)

        def check_rank(s):
            idx = inp.indices[s]                                     # [T][K]
            y = np.repeat(inp.x[s], K, axis=0)                       # row t*K+k = x of token t
            orc.scale_rows(y, np.ascontiguousarray(inp.expert_gain[idx.reshape(-1)]))
            want = orc.combine_sampled(E, K, idx, inp.weights[s], y)
            dist = ulp_distance(ob[s], want)
            return int(dist.max()), int((dist == 0).sum()), dist.size

        from concurrent.futures import ThreadPoolExecutor
        worst = exact = total = 0
        with ThreadPoolExecutor(4) as pool:                          # the C routines run outside the interpreter lock
            for s, (w, e, n) in enumerate(pool.map(check_rank, range(N))):
                worst, exact, total = max(worst, w), exact + e, total + n
                if s % 8 == 7:
                    print(f"  ranks 0..{s}: max ulp {worst}, bit-exact {exact}/{total}", flush=True)
        assert total == N * T * H
        print(f"[dsv3_prefill] combine, all {N * T} tokens: max ulp {worst}, bit-exact {exact}/{total}")
        assert worst <= 1
        assert exact == total          # same arithmetic on both sides: expected identical
    finally:
        sh.close()


def test_decode_with_practical_capacity():
    """Same decode workload with capacity 1.5x the mean instead of the worst case."""
    inp = wlmod.make_inputs(wlmod.WORKLOADS["dsv3_decode"])
    sh, _, _ = run_and_compare(inp, capacity_factor=1.5)
    sh.close()


# ------------------------------------------------------------------ limits, empty input, graph replay
LIMIT_CASES = {
    "max_ranks_experts_topk": lambda: wlmod.custom("limits", 64, 1024, 9, 64, 16, seed=41, ragged=True),
    "max_experts_per_rank": lambda: wlmod.custom("el256", 4, 1024, 33, 64, 8, seed=42),
    "min_hidden": lambda: wlmod.custom("h8", 4, 16, 40, 8, 2, seed=43, ragged=True),
    "long_row": lambda: wlmod.custom("h32k", 2, 8, 12, 32768, 3, seed=44),
}


@pytest.mark.parametrize("name", list(LIMIT_CASES))
def test_parity_at_the_limits_of_the_interface(name):
    inp = wlmod.make_inputs(LIMIT_CASES[name]())
    sh, _, _ = run_and_compare(inp)
    sh.close()


def test_parity_random_shapes():
    """Forty seeded random shapes: ranks, experts per rank, top-k, hidden size (any
    multiple of 8), ragged token counts, padding, zero fill, fabric mode, capacity."""
    rng = np.random.default_rng(2024)
    for trial in range(40):
        N = int(rng.choice([1, 2, 3, 4, 6, 8, 16]))
        El = int(rng.choice([1, 2, 3, 4, 8, 16]))
        E = N * El
        K = int(rng.integers(1, min(E, 9) + 1))
        T = int(rng.integers(1, 200))
        fp8 = trial % 5 == 4
        H = int(rng.integers(1, 9)) * 128 if fp8 else int(rng.integers(1, 300)) * 8
        wl = wlmod.custom(f"rnd{trial}", N, E, T, H, K, seed=3000 + trial, ragged=bool(trial % 2),
                          dispatch_dtype="e4m3" if fp8 else "bf16",
                          expert="identity" if trial % 7 == 0 else "scale")
        inp = wlmod.make_inputs(wl)
        print(f"trial {trial}: N={N} El={El} K={K} T={T} H={H} fp8={fp8}", flush=True)
        sh, _, _ = run_and_compare(inp, align=int(rng.choice([1, 1, 4, 7])), zero_pad=True,
                                   ordering=["counters", "stream", "progressive"][trial % 3])
        sh.close()


def test_parity_random_shapes_and_mode_combinations():
    """Forty more seeded random shapes, each with a random combination of the optional
    modes: private slots, peer push, partial sums, the three ordering modes, calls split by rank."""
    rng = np.random.default_rng(4242)
    for trial in range(40):
        N = int(rng.choice([1, 2, 3, 4, 8, 16, 32]))
        El = int(rng.choice([1, 2, 4, 8]))
        E = N * El
        K = int(rng.integers(1, min(E, 12) + 1))
        T = int(rng.integers(1, 150))
        fp8 = trial % 4 == 3
        H = int(rng.integers(1, 7)) * 128 if fp8 else int(rng.integers(1, 200)) * 8
        modes = dict(private_rows=int(rng.choice([0, 0, 1, 5, 40, 1000])), push=bool(rng.integers(2)),
                     partial=bool(rng.integers(2)), ordering=["counters", "stream", "progressive"][int(rng.integers(3))],
                     ranks_split=bool(N >= 2 and rng.integers(2)))
        wl = wlmod.custom(f"mix{trial}", N, E, T, H, K, seed=5000 + trial, ragged=bool(trial % 2),
                          dispatch_dtype="e4m3" if fp8 else "bf16")
        inp = wlmod.make_inputs(wl)
        print(f"trial {trial}: N={N} El={El} K={K} T={T} H={H} fp8={fp8} {modes}", flush=True)
        sh, _, _ = run_and_compare(inp, align=int(rng.choice([1, 4])), zero_pad=True, **modes)
        sh.close()


@pytest.mark.parametrize("kw", [dict(), dict(ordering="stream"), dict(push=True), dict(ranks_split=True),
                                dict(partial=True, private_rows=20), dict(fp8=True, align=4),
                                dict(ordering="progressive"),
                                dict(ordering="progressive", push=True, partial=True, fp8=True)])
def test_large_calls_are_issued_as_several_launches_over_rank_groups(kw):
    """A call that moves several times the per-launch target enqueues its kernels once
    per group of ranks; here the target is set to 1 MiB so that a small step is cut into
    one launch per rank (contexts whose receive kernels poll themselves are never cut).
    Same results, and the launch counts show the cut happened."""
    kw = dict(kw)
    fp8 = kw.pop("fp8", False)
    wl = wlmod.custom("groups", 8, 32, 128, 1024, 4, seed=77, ragged=True,
                      dispatch_dtype="e4m3" if fp8 else "bf16")
    inp = wlmod.make_inputs(wl)
    sh, _, _ = run_and_compare(inp, zero_pad=True, launch_mb=1, **kw)
    try:
        dev = harness.to_device(inp)
        before = flmoe.fl_moe_profile_read(sh.ctx)
        flmoe.fl_moe_profile_enable(sh.ctx, 1)
        harness.run_step(sh, dev)
        flmoe.fl_moe_profile_collect(sh.ctx)
        flmoe.fl_moe_profile_enable(sh.ctx, 0)
        after = flmoe.fl_moe_profile_read(sh.ctx)
        assert sh.status() == 0
        launches = {k: after[k][1] - before[k][1] for k in after}
        cut = 1 if kw.get("ordering") == "progressive" else wl.n_ranks
        assert launches["route_layout_kernel"] == 1
        assert launches["dispatch_unpack_kernel"] == cut
        assert launches["combine_reduce_kernel"] == cut
        flmoe.fl_moe_debug_tune(sh.ctx, 6, 0)          # never cut
        before = after
        flmoe.fl_moe_profile_enable(sh.ctx, 1)
        harness.run_step(sh, dev)
        flmoe.fl_moe_profile_collect(sh.ctx)
        flmoe.fl_moe_profile_enable(sh.ctx, 0)
        after = flmoe.fl_moe_profile_read(sh.ctx)
        assert after["dispatch_unpack_kernel"][1] - before["dispatch_unpack_kernel"][1] == 1
    finally:
        sh.close()


@pytest.mark.parametrize("kw", [dict(), dict(push=True), dict(partial=True, private_rows=50),
                                dict(ordering="stream"), dict(ordering="progressive")])
def test_every_token_to_one_rank_is_served_by_the_row_loops(kw):
    """Grids are sized for twice the rows uniform routing would bring; here one rank
    hosts every chosen expert and receives N*T rows and N*T*K pairs, several times
    that, so its kernels loop over their grids."""
    inp = wlmod.make_inputs(wlmod.custom("hot_rank", 8, 64, 300, 256, 4, seed=77, ragged=True))
    rng = np.random.default_rng(77)
    hot = 3
    for s in range(8):
        for t in range(300):
            inp.indices[s, t] = hot * 8 + rng.permutation(8)[:4]
    sh, _, _ = run_and_compare(inp, zero_pad=True, **kw)
    sh.close()


@pytest.mark.parametrize("kw", [dict(), dict(stream_ordered=True), dict(progressive_recv=True), dict(peer_push=True),
                                dict(peer_push=True, stream_ordered=True),
                                dict(peer_push=True, progressive_recv=True),
                                dict(peer_push=True, partial_sums=True, progressive_recv=True)])
def test_no_tokens_anywhere_is_a_clean_no_op(kw):
    inp = wlmod.make_inputs(CASES["ragged_520"]())
    inp.num_tokens[:] = 0
    dev = harness.to_device(inp)
    sh = harness.make_shuffle(inp, **kw)
    try:
        sh.expert_x.view(torch.int16).fill_(POISON)
        sh.out.view(torch.int16).fill_(POISON)
        sh.tokens_per_expert.fill_(-1)
        harness.run_step(sh, dev)
        torch.cuda.synchronize()
        assert sh.status() == 0
        assert (sh.tokens_per_expert.cpu().numpy() == 0).all()
        tabs = sh.layout_tables()
        assert (tabs["C"].cpu().numpy() == 0).all() and (tabs["expert_off"].cpu().numpy() == 0).all()
        assert (bits(sh.expert_x) == POISON).all() and (bits(sh.out) == POISON).all()
        dbg = sh.debug()
        # every transfer was empty, and every one was announced and expected all the same
        for name in ("arrive_disp", "expect_disp", "arrive_comb", "expect_comb"):
            assert (dbg[name].cpu().numpy() == 1).all(), name
    finally:
        sh.close()


def test_hip_graph_replay_with_new_inputs():
    """The five calls only enqueue kernels (no allocation, no reset, no synchronisation):
    captured once, the graph is replayed on new routing and new hidden states written
    into the same tensors, with eager work and synchronisation between replays, and every
    replay matches the oracle."""
    wl0 = wlmod.custom("graph0", 4, 32, 64, 520, 4, seed=51, expert="identity")
    inputs = [wlmod.make_inputs(wlmod.custom(f"graph{i}", 4, 32, 64, 520, 4, seed=51 + i,
                                             ragged=(i % 2 == 1), expert="identity"))
              for i in range(4)]
    dev = harness.to_device(inputs[0])
    sh = harness.make_shuffle(inputs[0])
    try:
        harness.run_hot_path(sh, dev)              # warm-up outside capture
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            harness.run_hot_path(sh, dev)
        for i, inp in enumerate(inputs):
            fresh = harness.to_device(inp)
            for k in ("x", "indices", "weights", "num_tokens"):
                dev[k].copy_(fresh[k])
            sh.out.view(torch.int16).fill_(POISON)
            graph.replay()
            torch.cuda.synchronize()
            assert sh.status() == 0
            ref = oracle_step(inp)
            ob = bits(sh.out)
            ex = bits(sh.expert_x[:, :ref.stride])
            for d in range(4):
                n = ref.expert_rows[d].shape[0]
                assert (ex[d, :n] == ref.expert_rows[d]).all(), (i, d)
            for s in range(4):
                n = inp.num_tokens[s]
                assert (ob[s, :n] == ref.out[s, :n]).all(), (i, s)
                assert (ob[s, n:] == POISON).all()
            # eager work between replays: a full eager step on the same context
            eager = harness.run_hot_path(sh, dev)
            torch.cuda.synchronize()
            assert (bits(eager)[0, :inp.num_tokens[0]] == ref.out[0, :inp.num_tokens[0]]).all()
    finally:
        sh.close()


@pytest.mark.parametrize("form", ["stream", "progressive"])
def test_other_ordering_modes_with_e4m3_dispatch(form):
    inp = wlmod.make_inputs(FP8_CASES["fp8_small"]())
    sh, _, _ = run_and_compare(inp, ordering=form, zero_pad=True, align=4)
    sh.close()


# ------------------------------------------------------------------ senders and receivers overlapping in time
@pytest.mark.parametrize("progressive", [False, True])
@pytest.mark.parametrize("name,shuffled,push", [("ragged_520", False, False), ("ragged_520", True, False),
                                                ("overlap_7168", False, False), ("overlap_7168", True, False),
                                                ("dsv3_decode", False, False),
                                                ("ragged_520", True, True), ("overlap_7168", False, True),
                                                ("dsv3_decode", True, True)])
def test_concurrent_send_and_receive_on_two_streams(name, shuffled, push, progressive):
    if name == "overlap_7168":
        wl = wlmod.custom("overlap_7168", 8, 64, 128, 7168, 8, seed=61)
    elif name == "dsv3_decode":
        wl = wlmod.WORKLOADS[name]
    else:
        wl = CASES[name]()
    inp = wlmod.make_inputs(wl)
    N = wl.n_ranks
    ref = oracle_step(inp)
    dev = harness.to_device(inp)
    sh = harness.make_shuffle(inp, capacity_factor=2.0 if N >= 8 else None,
                              peer_push=push, progressive_recv=progressive)
    try:
        order = None
        if shuffled:      # one launch per sender, in a seeded random order
            perm = np.random.default_rng(5).permutation(N)
            order = [(int(r), 1) for r in perm]
        for rep in range(3):
            flmoe.fl_moe_debug_tune(sh.ctx, 8, rep)    # the fabric takes each sender's destinations in another order
            sh.out.view(torch.int16).fill_(POISON)
            out = harness.run_step_two_streams(sh, dev, wl.expert == "identity", order)
            torch.cuda.synchronize()
            assert sh.status() == 0, "a receiver gave up waiting"
            ex = bits(sh.expert_x[:, :ref.stride])
            ob = bits(out)
            for d in range(N):
                n = ref.expert_rows[d].shape[0]
                assert (ex[d, :n] == ref.expert_rows[d]).all(), (rep, d)
            for s in range(N):
                n = inp.num_tokens[s]
                assert (ob[s, :n] == ref.out[s, :n]).all(), (rep, s)
        dbg = sh.debug()
        assert (dbg["arrive_disp"] == dbg["expect_disp"]).all()
        assert (dbg["arrive_comb"] == dbg["expect_comb"]).all()
    finally:
        sh.close()


@pytest.mark.parametrize("push", [False, True])
def test_one_stream_per_rank_no_cross_rank_events(push):
    """Every simulated rank issues its payload calls (rank_count = 1) on a stream of its
    own, as ranks on separate GPUs would; between the ranks there is no event and no
    common stream, only the arrival counters.  Each rank keeps its own calls in order
    (its stream), which in the default mode is also all the re-use of the staging
    buffers needs: a rank's gate passes only after every peer's announce kernel ran,
    and that kernel runs only after the peer's payload kernels have ended.  Steps
    follow each other without a device synchronisation; each step's results are
    copied aside on the rank's own stream and compared with the oracle at the end.
    (The layout step is one call for all ranks, since its kernels wait for each other
    inside the call.  Host issue order puts all sends of a phase before its receives,
    so that no gate kernel can sit in front of a send in a shared hardware queue.)"""
    inp = wlmod.make_inputs(wlmod.custom("per_rank_streams", 4, 32, 100, 1024, 4, seed=71, ragged=True,
                                         expert="identity"))
    N = inp.wl.n_ranks
    ref = oracle_step(inp)
    dev = harness.to_device(inp)
    sh = harness.make_shuffle(inp, peer_push=push)
    streams = [torch.cuda.Stream() for _ in range(N)]
    lay_stream = torch.cuda.Stream()
    steps, kept = 12, []
    rng = np.random.default_rng(71)
    try:
        torch.cuda.synchronize()
        done = []
        for step in range(steps):
            for e in done:                              # a rank plans its next step after its own reduce
                lay_stream.wait_event(e)
            with torch.cuda.stream(lay_stream):
                sh.expert_x.view(torch.int16).fill_(POISON)
                sh.out.view(torch.int16).fill_(POISON)
                sh.layout(dev["indices"], dev["num_tokens"], stream=lay_stream)
                planned = torch.cuda.Event()
                planned.record(lay_stream)
            order = [int(r) for r in rng.permutation(N)]
            for r in order:
                streams[r].wait_event(planned)
                sh.dispatch_send(dev["x"], (r, 1), stream=streams[r])
            for r in reversed(order):
                sh.dispatch_recv((r, 1), stream=streams[r])
            for r in order:
                sh.combine_send(sh.expert_x, (r, 1), stream=streams[r])      # identity expert
            done, snap = [], []
            for r in reversed(order):
                sh.combine_reduce(dev["weights"], (r, 1), stream=streams[r])
                with torch.cuda.stream(streams[r]):
                    snap.append((r, sh.expert_x[r, :ref.stride].clone(), sh.out[r].clone()))
                    e = torch.cuda.Event()
                    e.record(streams[r])
                    done.append(e)
            kept.append(snap)
        torch.cuda.synchronize()
        assert sh.status() == 0
        for step, snap in enumerate(kept):
            for r, ex, out in snap:
                n = ref.expert_rows[r].shape[0]
                assert (bits(ex)[:n] == ref.expert_rows[r]).all(), (step, r)
                k = inp.num_tokens[r]
                assert (bits(out)[:k] == ref.out[r, :k]).all(), (step, r)
    finally:
        torch.cuda.synchronize()
        sh.close()


@pytest.mark.parametrize("progressive,steps", [(False, 1200), (True, 800)])
def test_soak_two_streams_shuffled_senders_every_step_checked(progressive, steps):
    """Bounded soak of the path where only the arrival counters order senders and
    receivers: the decode workload, receive calls on one stream, one send call per
    sender on another in a freshly shuffled order every step, the fabric kernel taking
    each sender's destinations in a different order from step to step.  The first step
    is compared with the oracle; every later step must reproduce its expert rows and
    its combined output bit for bit (outputs are poisoned before each step, so a
    receiver that ran ahead of its data cannot pass), with a clean status word."""
    import os
    from dataclasses import replace
    steps *= max(1, int(os.environ.get("FLMOE_SOAK_SCALE", "1")))     # a longer run on request
    wl = replace(wlmod.WORKLOADS["dsv3_decode"], name="soak", expert="identity")
    inp = wlmod.make_inputs(wl)
    N = wl.n_ranks
    ref = oracle_step(inp)
    dev = harness.to_device(inp)
    sh = harness.make_shuffle(inp, capacity_factor=1.5, progressive_recv=progressive)
    streams = (torch.cuda.Stream(), torch.cuda.Stream())
    rng = np.random.default_rng(2024)
    try:
        first_x = first_out = None
        for step in range(steps):
            order = [(int(r), 1) for r in rng.permutation(N)]
            flmoe.fl_moe_debug_tune(sh.ctx, 8, step % 3)
            sh.expert_x.view(torch.int16).fill_(POISON)
            sh.out.view(torch.int16).fill_(POISON)
            out = harness.run_step_two_streams(sh, dev, send_order=order, expert_y=sh.expert_x,
                                               streams=streams)
            if step == 0:
                torch.cuda.synchronize()
                assert sh.status() == 0
                ex, ob = bits(sh.expert_x[:, :ref.stride]), bits(out)
                for d in range(N):
                    n = ref.expert_rows[d].shape[0]
                    assert (ex[d, :n] == ref.expert_rows[d]).all(), d
                for r in range(N):
                    assert (ob[r] == ref.out[r]).all(), r
                first_x, first_out = sh.expert_x.clone(), out.clone()
            else:
                same = (torch.equal(sh.expert_x.view(torch.int16), first_x.view(torch.int16))      # as bits:
                        and torch.equal(out.view(torch.int16), first_out.view(torch.int16)))    # the poison is a NaN
                assert same, f"step {step} differs from the oracle-checked first step"
                if step % 100 == 0:
                    assert sh.status() == 0, step
                    print(f"  soak step {step} ok", flush=True)
        assert sh.status() == 0
        dbg = sh.debug()
        assert (dbg["arrive_disp"] == dbg["expect_disp"]).all()
        assert (dbg["arrive_comb"] == dbg["expect_comb"]).all()
    finally:
        sh.close()


# ------------------------------------------------------------------ private slots + shared range
def shared_range_rows(M, P):
    """Rows each destination's shared range must hold: sum over sources of max(M - P, 0)."""
    return np.maximum(M.astype(np.int64) - P, 0).sum(axis=0)


@pytest.mark.parametrize("name,P", [("ragged_520", 1), ("ragged_520", 5), ("ragged_520", 1000),
                                    ("multi_tile", 64), ("k16", 7), ("single_rank", 10)])
def test_parity_with_private_slots(name, P):
    """Section Dispatch: the first P rows per (source, destination) go to private
    slots in a scatter of their own, the rest into the shared range; the receiver
    reads both regions.  Every result of the step is unchanged."""
    inp = wlmod.make_inputs(CASES[name]())
    sh, _, _ = run_and_compare(inp, align=4, zero_pad=True, private_rows=P)
    sh.close()


def test_private_slots_with_e4m3_and_the_other_ordering_modes():
    inp = wlmod.make_inputs(FP8_CASES["fp8_small"]())
    sh, _, _ = run_and_compare(inp, private_rows=9, ordering="stream")
    sh.close()
    inp = wlmod.make_inputs(CASES["multi_tile"]())
    sh, _, _ = run_and_compare(inp, private_rows=300, ordering="progressive", ranks_split=True)
    sh.close()


def test_private_slots_named_decode_workload():
    inp = wlmod.make_inputs(wlmod.WORKLOADS["dsv3_decode"])
    sh, _, _ = run_and_compare(inp, private_rows=32)
    sh.close()


@pytest.mark.parametrize("P", [3, 12, 1000])
def test_receive_buffer_holds_private_slots_then_shared_range(P):
    """Where the scatter put every row, read back from the receive buffers and
    compared with the layout the interface documents: source s's first P rows for
    rank d at rows s*P.., later ones at N*P + (rows of lower sources beyond their
    P) + (i - P); every other row of the buffer untouched."""
    inp = wlmod.make_inputs(CASES["ragged_520"]())
    wl = inp.wl
    N, E, K, H = wl.n_ranks, wl.n_experts, wl.top_k, wl.hidden
    dev = harness.to_device(inp)
    sh = harness.make_shuffle(inp, max_private_rows=P)
    try:
        Pr = int(sh.sizes.private_rows)
        assert Pr == min(P, wl.tokens)
        assert sh.sizes.recv_buffer_rows == N * Pr + sh.sizes.recv_capacity_rows
        buf = sh.debug()["buf_b"]
        buf.fill_(0xA5)
        sh.layout(dev["indices"], dev["num_tokens"])
        sh.dispatch_send(dev["x"])
        torch.cuda.synchronize()
        assert sh.status() == 0
        got = buf.cpu().numpy()
        Bw = 2 * H
        xb = inp.x.view(np.uint8).reshape(N, wl.tokens, Bw)
        M = orc.layout(N, E, K, inp.num_tokens, inp.indices).M
        for d in range(N):
            rows = got[d, :sh.sizes.recv_buffer_rows * Bw].reshape(-1, Bw)
            touched = np.zeros(rows.shape[0], bool)
            sr, st, _ = orc.recv_order(d, N, E, K, inp.num_tokens, inp.indices)
            shared_start = 0
            for s in range(N):
                toks = st[sr == s]
                assert len(toks) == M[s, d]
                for i, t in enumerate(toks):
                    phys = s * Pr + i if i < Pr else N * Pr + shared_start + (i - Pr)
                    assert (rows[phys] == xb[s, t]).all(), (d, s, i)
                    assert not touched[phys]
                    touched[phys] = True
                shared_start += max(len(toks) - Pr, 0)
            assert (rows[~touched] == 0xA5).all(), f"rank {d}: rows outside the layout were written"
    finally:
        sh.close()


def test_private_slots_shrink_the_shared_range_needed():
    """recv_capacity_rows bounds the shared range only: exactly the rows beyond the
    private slots fit, one row less is a capacity error."""
    inp = wlmod.make_inputs(CASES["ragged_520"]())
    wl = inp.wl
    dev = harness.to_device(inp)
    ref = oracle_step(inp)
    P = 6
    need = int(shared_range_rows(ref.lay.M, P).max())
    assert 0 < need < int(ref.lay.M.sum(axis=0).max())
    for cap, ok in [(need, True), (need - 1, False)]:
        sh = flmoe.MoEShuffle(wl.n_ranks, wl.n_experts, wl.tokens, wl.top_k, wl.hidden,
                              recv_capacity_rows=cap, max_private_rows=P)
        try:
            sh.expert_x.view(torch.int16).fill_(POISON)
            out = harness.run_step(sh, dev)
            torch.cuda.synchronize()
            if ok:
                assert sh.status() == 0
                for s in range(wl.n_ranks):
                    n = inp.num_tokens[s]
                    assert (bits(out)[s, :n] == ref.out[s, :n]).all()
            else:
                assert sh.status() == flmoe.FL_STATUS_CAPACITY
                assert (bits(sh.expert_x) == POISON).all()
        finally:
            sh.close()


# ------------------------------------------------------------------ peer push: no send buffer, no scatter
@pytest.mark.parametrize("name", list(CASES))
def test_parity_peer_push_small(name):
    """FL_FLAG_PEER_PUSH: the send kernels store into the peers' receive buffers
    themselves (section Dispatch, pushes within a node).  Same results."""
    inp = wlmod.make_inputs(CASES[name]())
    sh, _, _ = run_and_compare(inp, push=True, align=4, zero_pad=True)
    sh.close()


@pytest.mark.parametrize("kw", [dict(ordering="stream"), dict(private_rows=7), dict(ranks_split=True),
                                dict(ordering="progressive"),
                                dict(ordering="stream", private_rows=1000, ranks_split=True),
                                dict(capacity_factor=2.0)])
def test_parity_peer_push_with_the_other_modes(kw):
    inp = wlmod.make_inputs(CASES["ragged_520"]())
    sh, _, _ = run_and_compare(inp, push=True, **kw)
    sh.close()


@pytest.mark.parametrize("name", list(FP8_CASES))
@pytest.mark.parametrize("ordering", ["counters", "stream", "progressive"])
def test_parity_peer_push_e4m3(name, ordering):
    inp = wlmod.make_inputs(FP8_CASES[name]())
    sh, _, _ = run_and_compare(inp, push=True, ordering=ordering)
    sh.close()


@pytest.mark.parametrize("name", ["dsv3_decode", "qwen3_skew", "dsv3_fp8"])
def test_parity_peer_push_named_workloads(name):
    inp = wlmod.make_inputs(wlmod.WORKLOADS[name])
    sh, _, _ = run_and_compare(inp, push=True)
    sh.close()


@pytest.mark.parametrize("name", ["ragged_520", "fp8_k16"])
def test_peer_push_counters_and_untouched_send_buffer(name):
    """Pushed rows are counted in the same units as scattered ones (arrive ==
    expect == rows x 16-byte units per wire row, also for e4m3 rows whose scale
    tail is not a whole vector), and dispatch_send leaves the send buffer alone."""
    wl = CASES[name]() if name in CASES else FP8_CASES[name]()
    inp = wlmod.make_inputs(wl)
    dev = harness.to_device(inp)
    ref = oracle_step(inp)
    sh = harness.make_shuffle(inp, peer_push=True)
    try:
        buf_a = sh.debug()["buf_a"]
        buf_a.fill_(0x5A)
        sh.layout(dev["indices"], dev["num_tokens"])
        sh.dispatch_send(dev["x"])
        torch.cuda.synchronize()
        assert bool((buf_a == 0x5A).all()), "push mode wrote a send buffer"
        sh.dispatch_recv()
        y = harness.expert_stage(sh, dev["gain"], wl.expert == "identity")
        sh.combine_send(y)
        sh.combine_reduce(dev["weights"])
        torch.cuda.synchronize()
        assert sh.status() == 0
        dbg = sh.debug()
        units = int(sh.sizes.wire_row_bytes) // 16
        assert (dbg["arrive_disp"].cpu().numpy() == ref.lay.M.T.astype(np.int64) * units + 1).all()
        assert (dbg["expect_disp"].cpu().numpy() == ref.lay.M.T.astype(np.int64) * units + 1).all()
        pairs = ref.lay.C.reshape(wl.n_ranks, wl.n_ranks, -1).sum(2)
        cunits = wl.hidden * 2 // 16
        assert (dbg["arrive_comb"].cpu().numpy() == pairs * cunits + 1).all()
        assert (dbg["expect_comb"].cpu().numpy() == pairs * cunits + 1).all()
    finally:
        sh.close()


# ------------------------------------------------------------------ combine with sender-side partial sums
@pytest.mark.parametrize("name", list(CASES))
def test_parity_partial_sums_small(name):
    """FL_FLAG_PARTIAL_SUMS: one bf16 share per (token, expert rank), added in fp32 on
    the token's rank; compared with the oracle's statement of the same definition.
    Dispatch is unchanged (and checked as in every other test)."""
    inp = wlmod.make_inputs(CASES[name]())
    sh, _, _ = run_and_compare(inp, partial=True, align=4, zero_pad=True)
    sh.close()


@pytest.mark.parametrize("kw", [dict(ordering="stream"), dict(private_rows=7), dict(ranks_split=True),
                                dict(ordering="progressive"),
                                dict(push=True), dict(push=True, ordering="stream", private_rows=3),
                                dict(capacity_factor=2.0, ranks_split=True, push=True)])
def test_parity_partial_sums_with_the_other_modes(kw):
    inp = wlmod.make_inputs(CASES["ragged_520"]())
    sh, _, _ = run_and_compare(inp, partial=True, **kw)
    sh.close()


@pytest.mark.parametrize("name", ["fp8_small", "fp8_k16"])
def test_parity_partial_sums_e4m3(name):
    inp = wlmod.make_inputs(FP8_CASES[name]())
    sh, _, _ = run_and_compare(inp, partial=True)
    sh.close()


@pytest.mark.parametrize("name,push", [("dsv3_decode", False), ("dsv3_decode", True), ("qwen3_skew", False)])
def test_parity_partial_sums_named_workloads(name, push):
    inp = wlmod.make_inputs(wlmod.WORKLOADS[name])
    sh, _, _ = run_and_compare(inp, partial=True, push=push)
    sh.close()


def test_partial_sums_differ_from_the_exact_combine_and_need_the_weighted_dispatch():
    """The mode really is another arithmetic (so the parity above has teeth), a step
    moves one reply row per received row, and the plain dispatch call is refused."""
    inp = wlmod.make_inputs(CASES["k16"]())
    wl = inp.wl
    ref = oracle_step(inp, partial=True)
    assert (ref.out != ref.out_partial).any()
    dev = harness.to_device(inp)
    sh = harness.make_shuffle(inp, partial_sums=True)
    try:
        out = harness.run_step(sh, dev)
        torch.cuda.synchronize()
        assert sh.status() == 0
        for s in range(wl.n_ranks):
            n = inp.num_tokens[s]
            assert (bits(out)[s, :n] == ref.out_partial[s, :n]).all()
        dbg = sh.debug()
        units = wl.hidden * 2 // 16
        # one share per de-duplicated row: arrive_comb[s][d] counts M[s][d] rows
        assert (dbg["arrive_comb"].cpu().numpy() == ref.lay.M.astype(np.int64) * units + 1).all()
        assert (dbg["expect_comb"].cpu().numpy() == ref.lay.M.astype(np.int64) * units + 1).all()
        with pytest.raises(flmoe.FlMoeError) as ei:       # refused on the host, nothing enqueued
            sh.dispatch_send(dev["x"])
        assert ei.value.code == flmoe.FL_ERR_INVALID_ARG
    finally:
        sh.close()
    plain = harness.make_shuffle(inp)
    try:
        harness.run_step(plain, dev)
        with pytest.raises(flmoe.FlMoeError) as ei:
            plain.dispatch_send(dev["x"], weights=dev["weights"])
        assert ei.value.code == flmoe.FL_ERR_INVALID_ARG
        torch.cuda.synchronize()
    finally:
        plain.close()


# ------------------------------------------------------------------ chunked prefill
@pytest.mark.parametrize("chunk", [32, 100, 7])
def test_chunked_steps_give_the_same_combined_output(chunk):
    """A context sized for `chunk` tokens per rank stepped over the batch: every chunk
    matches the oracle run on that chunk (tables, dispatched rows, combined rows), and
    the combined rows of all tokens equal those of the one-shot step, since a token's
    sum does not depend on its neighbours.  The staging buffers shrink with the chunk."""
    inp = wlmod.make_inputs(wlmod.custom("chunked", 4, 32, 100, 520, 4, seed=91, ragged=True))
    wl = inp.wl
    N, T = wl.n_ranks, wl.tokens
    whole = oracle_step(inp)
    pieces = [(t0, wlmod.token_chunk(inp, t0, chunk)) for t0 in range(0, T, chunk)]
    one_shot = harness.make_shuffle(inp)
    full_bytes = one_shot.sizes.workspace_bytes
    one_shot.close()
    sh = harness.make_shuffle(pieces[0][1])
    try:
        assert chunk >= T or sh.sizes.workspace_bytes < full_bytes
        out_full = torch.zeros((N, T, wl.hidden), dtype=torch.bfloat16, device="cuda")
        out_full.view(torch.int16).fill_(POISON)
        for t0, piece in pieces:
            harness.run_chunked(sh, [(t0, harness.to_device(piece))], out_full)
            torch.cuda.synchronize()
            assert sh.status() == 0
            ref = oracle_step(piece)
            check_tables(sh, ref, N)
            ex = bits(sh.expert_x[:, :ref.stride])
            for d in range(N):
                n = ref.expert_rows[d].shape[0]
                assert (ex[d, :n] == ref.expert_rows[d]).all(), (t0, d)
            ob = bits(sh.out)
            for s in range(N):
                k = int(piece.num_tokens[s])
                assert (ob[s, :k] == ref.out[s, :k]).all()
        ofb = bits(out_full)
        for s in range(N):
            k = int(inp.num_tokens[s])
            assert (ofb[s, :k] == whole.out[s, :k]).all(), "chunking changed a token's result"
    finally:
        sh.close()


# ------------------------------------------------------------------ tokens the caller quantised itself
@pytest.mark.parametrize("name", list(FP8_CASES))
@pytest.mark.parametrize("kw", [dict(), dict(peer_push=True), dict(stream_ordered=True, peer_push=True),
                                dict(partial_sums=True, max_private_rows=5)])
def test_dispatch_of_ready_made_e4m3_tokens(name, kw):
    """fl_moe_dispatch_send_e4m3 (section Kernel Microbenchmarks: the dispatched token is
    fp8 values plus fp32 scaling factors): codes and scales quantised beforehand, here by
    the oracle, arrive in expert_x / expert_scales byte for byte, and the rest of the step
    is the one of the quantise-on-the-fly path."""
    inp = wlmod.make_inputs(FP8_CASES[name]())
    wl = inp.wl
    N = wl.n_ranks
    partial = kw.get("partial_sums", False)
    ref = oracle_step(inp, partial=partial)
    want = ref.out_partial if partial else ref.out
    q, sc = orc.quant_e4m3_block128(inp.x)
    dev = harness.to_device(inp)
    codes = torch.from_numpy(q).cuda()
    scales = torch.from_numpy(sc).cuda()
    sh = harness.make_shuffle(inp, **kw)
    try:
        sh.out.view(torch.int16).fill_(POISON)
        sh.layout(dev["indices"], dev["num_tokens"])
        sh.dispatch_send(codes, scales=scales, weights=harness.send_weights(sh, dev))
        sh.dispatch_recv()
        y = harness.expert_stage(sh, dev["gain"], wl.expert == "identity")
        sh.combine_send(y)
        out = sh.combine_reduce(dev["weights"])
        torch.cuda.synchronize()
        assert sh.status() == 0
        check_tables(sh, ref, N)
        ex = sh.expert_x[:, :ref.stride].cpu().numpy()
        exs = sh.expert_scales[:, :ref.stride].cpu().numpy().view(np.uint32)
        for d in range(N):
            n = ref.expert_rows[d].shape[0]
            assert (ex[d, :n] == ref.expert_rows[d]).all(), f"e4m3 bytes, rank {d}"
            assert (exs[d, :n] == ref.expert_scales[d].view(np.uint32)).all(), f"scales, rank {d}"
        ob = bits(out)
        for s in range(N):
            k = inp.num_tokens[s]
            assert (ob[s, :k] == want[s, :k]).all()
            assert (ob[s, k:] == POISON).all()
        dbg = sh.debug()
        assert (dbg["arrive_disp"] == dbg["expect_disp"]).all()
    finally:
        sh.close()


def test_ready_made_e4m3_needs_an_e4m3_context():
    inp = wlmod.make_inputs(CASES["tiny"]())
    dev = harness.to_device(inp)
    sh = harness.make_shuffle(inp)
    try:
        harness.run_step(sh, dev, identity=True)
        fake = torch.zeros((2, 16, 256), dtype=torch.uint8, device="cuda")
        fsc = torch.ones((2, 16, 2), dtype=torch.float32, device="cuda")
        with pytest.raises(flmoe.FlMoeError) as ei:
            sh.dispatch_send(fake, scales=fsc)
        assert ei.value.code == flmoe.FL_ERR_INVALID_ARG
        torch.cuda.synchronize()
    finally:
        sh.close()


# ------------------------------------------------------------------ failure handling
def small_shuffle(spin_limit=0, **kw):
    inp = wlmod.make_inputs(CASES["ragged_520"]())
    dev = harness.to_device(inp)
    sh = harness.make_shuffle(inp, spin_limit=spin_limit, **kw)
    return inp, dev, sh


@pytest.mark.parametrize("kw", [dict(), dict(peer_push=True), dict(stream_ordered=True, max_private_rows=4)])
def test_bad_expert_id_skips_the_step_everywhere(kw):
    inp, dev, sh = small_shuffle(**kw)
    try:
        bad = dev["indices"].clone()
        bad[1, 3, 2] = inp.wl.n_experts + 5
        sh.expert_x.view(torch.int16).fill_(POISON)
        sh.out.view(torch.int16).fill_(POISON)
        sh.layout(bad, dev["num_tokens"])
        sh.dispatch_send(dev["x"])
        sh.dispatch_recv()
        sh.combine_send(sh.expert_x)
        sh.combine_reduce(dev["weights"])
        torch.cuda.synchronize()
        assert sh.status() == flmoe.FL_STATUS_BAD_INDEX
        assert (sh.layout_tables()["plan_ok"].cpu().numpy() == 0).all()
        assert (bits(sh.expert_x) == POISON).all() and (bits(sh.out) == POISON).all()
        # duplicate expert inside a token is rejected too
        dup = dev["indices"].clone()
        dup[0, 0, 1] = dup[0, 0, 0]
        sh.layout(dup, dev["num_tokens"])
        sh.dispatch_send(dev["x"])
        torch.cuda.synchronize()
        assert sh.status() == flmoe.FL_STATUS_BAD_INDEX
        sh.dispatch_recv()
        sh.combine_send(sh.expert_x)
        sh.combine_reduce(dev["weights"])
        # the next good step works and the counters are still in step
        ref = oracle_step(inp)
        out = harness.run_step(sh, dev)
        torch.cuda.synchronize()
        assert sh.status() == 0
        for s in range(inp.wl.n_ranks):
            n = inp.num_tokens[s]
            assert (bits(out)[s, :n] == ref.out[s, :n]).all()
    finally:
        sh.close()


@pytest.mark.parametrize("kw", [dict(), dict(peer_push=True), dict(partial_sums=True, max_private_rows=2),
                                dict(stream_ordered=True, peer_push=True)])
def test_capacity_overflow_is_reported_not_written(kw):
    inp = wlmod.make_inputs(CASES["ragged_520"]())
    dev = harness.to_device(inp)
    sh = harness.make_shuffle(inp, capacity_factor=0.25, **kw)
    try:
        sh.expert_x.view(torch.int16).fill_(POISON)
        sh.out.view(torch.int16).fill_(POISON)
        buf_b = sh.debug()["buf_b"]
        buf_b.fill_(0x3C)
        harness.run_hot_path(sh, dev)
        torch.cuda.synchronize()
        assert sh.status() == flmoe.FL_STATUS_CAPACITY
        assert (bits(sh.expert_x) == POISON).all() and (bits(sh.out) == POISON).all()
        assert bool((buf_b == 0x3C).all()), "a skipped step wrote into a receive buffer"
        dbg = sh.debug()
        assert (dbg["arrive_disp"] == dbg["expect_disp"]).all() and (dbg["arrive_comb"] == dbg["expect_comb"]).all()
    finally:
        sh.close()


@pytest.mark.parametrize("align,private_rows", [(1, 0), (16, 0), (1, 4)])
def test_required_capacities_after_an_overflow_size_a_context_that_fits(align, private_rows):
    """A step skipped for capacity tells the caller what it needs: the oracle's per-rank
    maxima.  A context with exactly these capacities runs the step (full parity); one row
    less in either of them is an overflow again."""
    inp = wlmod.make_inputs(CASES["ragged_520"]())
    ref = oracle_step(inp, align, zero_pad=True)
    dev = harness.to_device(inp)
    sh = harness.make_shuffle(inp, expert_align=align, capacities=(4, 4), max_private_rows=private_rows)
    try:
        harness.run_hot_path(sh, dev)
        need = sh.required_capacities()          # synchronises
        assert sh.status() == flmoe.FL_STATUS_CAPACITY
    finally:
        sh.close()
    M = ref.lay.M.astype(np.int64)               # [source][destination]
    want = (max(1, int(np.maximum(M - private_rows, 0).sum(axis=0).max())),
            max(1, int(ref.lay.expert_off[:, -1].max())))
    assert need == want
    sh2, _, _ = run_and_compare(inp, align=align, private_rows=private_rows, capacities=need)
    assert sh2.required_capacities() == want     # the same numbers after a valid step
    sh2.close()
    for short in [(need[0] - 1, need[1]), (need[0], need[1] - 1)]:
        if min(short) < 1:
            continue
        sh3 = harness.make_shuffle(inp, expert_align=align, max_private_rows=private_rows, capacities=short)
        try:
            harness.run_hot_path(sh3, dev)
            torch.cuda.synchronize()
            assert sh3.status() == flmoe.FL_STATUS_CAPACITY, short
        finally:
            sh3.close()


def test_missing_peers_time_out_instead_of_hanging():
    """Only half of the ranks take part: the others' counts never arrive, the
    bounded wait gives up and the step is skipped on the ranks that did run."""
    inp, dev, sh = small_shuffle(spin_limit=200)
    try:
        sh.layout(dev["indices"], dev["num_tokens"], ranks=(0, 2))
        torch.cuda.synchronize()
        assert sh.status() == flmoe.FL_STATUS_TIMEOUT
        assert (sh.layout_tables()["plan_ok"].cpu().numpy()[:2] == 0).all()
    finally:
        sh.close()


def test_reset_brings_a_context_back_in_step_after_a_layout_time_out():
    """A layout call without its peers leaves the ranks' epochs apart (those that ran are
    one step ahead): the next complete step times out as well.  fl_moe_reset zeroes the
    counters; the step after it is correct on every rank."""
    inp, dev, sh = small_shuffle(spin_limit=200)
    try:
        ref = oracle_step(inp)
        sh.layout(dev["indices"], dev["num_tokens"], ranks=(0, 2))
        torch.cuda.synchronize()
        assert sh.status() == flmoe.FL_STATUS_TIMEOUT
        dbg = sh.debug()
        assert dbg["epoch_route"].cpu().tolist() == [1, 1, 0, 0]
        harness.run_step(sh, dev)                     # all ranks, but 0 and 1 now expect a second message
        torch.cuda.synchronize()
        assert sh.status() & flmoe.FL_STATUS_TIMEOUT
        sh.reset()
        dbg = sh.debug()
        for name in ("epoch_route", "arrive_route", "arrive_disp", "expect_disp", "arrive_comb", "expect_comb"):
            assert not bool(dbg[name].any()), name
        sh.out.view(torch.int16).fill_(POISON)
        out = harness.run_step(sh, dev)
        torch.cuda.synchronize()
        assert sh.status() == 0
        check_tables(sh, ref, inp.wl.n_ranks)
        for r in range(inp.wl.n_ranks):
            n = inp.num_tokens[r]
            assert (bits(out)[r, :n] == ref.out[r, :n]).all()
    finally:
        sh.close()


def test_layout_split_over_two_streams_meets_in_the_exchange():
    """Half of the ranks plan on one stream, half on another: each half waits inside
    the call for the other's counts, as ranks on separate GPUs do (bounded wait)."""
    inp, dev, sh = small_shuffle()
    try:
        ref = oracle_step(inp)
        a, b = torch.cuda.Stream(), torch.cuda.Stream()
        torch.cuda.synchronize()
        sh.layout(dev["indices"], dev["num_tokens"], ranks=(0, 2), stream=a)
        sh.layout(dev["indices"], dev["num_tokens"], ranks=(2, 2), stream=b)
        torch.cuda.synchronize()
        sh.dispatch_send(dev["x"])
        sh.dispatch_recv()
        y = harness.expert_stage(sh, dev["gain"])
        sh.combine_send(y)
        out = sh.combine_reduce(dev["weights"])
        torch.cuda.synchronize()
        assert sh.status() == 0
        check_tables(sh, ref, inp.wl.n_ranks)
        for r in range(inp.wl.n_ranks):
            n = inp.num_tokens[r]
            assert (bits(out)[r, :n] == ref.out[r, :n]).all()
    finally:
        sh.close()


@pytest.mark.parametrize("kw", [dict(), dict(stream_ordered=True),
                                dict(progressive_recv=True)])
def test_withheld_arrival_counter_times_out_then_recovers(kw):
    inp, dev, sh = small_shuffle(spin_limit=200, **kw)
    try:
        ref = oracle_step(inp)
        sh.layout(dev["indices"], dev["num_tokens"])
        sh.dispatch_send(dev["x"])
        torch.cuda.synchronize()
        arrive = sh.debug()["arrive_disp"]
        # find a non-empty segment and pretend its notification has not arrived yet
        M = ref.lay.M
        s, d = [(s, d) for s in range(4) for d in range(4) if M[s, d] > 0][0]
        arrive[d, s] -= 1
        sh.expert_x.view(torch.int16).fill_(POISON)
        sh.dispatch_recv()
        torch.cuda.synchronize()
        assert sh.status() == flmoe.FL_STATUS_TIMEOUT
        lo, hi = ref.lay.recv_off[d, s], ref.lay.recv_off[d, s + 1]
        assert hi > lo
        # deliver the notification: the same call now completes
        arrive[d, s] += 1
        sh.dispatch_recv()
        y = harness.expert_stage(sh, dev["gain"])
        sh.combine_send(y)
        out = sh.combine_reduce(dev["weights"])
        torch.cuda.synchronize()
        assert sh.status() == 0
        for r in range(inp.wl.n_ranks):
            n = inp.num_tokens[r]
            assert (bits(out)[r, :n] == ref.out[r, :n]).all()
    finally:
        sh.close()


@pytest.mark.parametrize("nbytes", [16, 4096, 4096 + 16, 65536 - 16, (1 << 20) + 48])
def test_plain_copy_fill_and_read_kernels_stay_inside_their_buffers(nbytes):
    """The three diagnostic kernels (machine ceilings, counter calibration) on sizes that
    end inside a workgroup's share: the copy is exact, the fill writes its constant, and
    neither touches the bytes on either side of the range it was given."""
    guard = 4096
    gen = torch.Generator(device="cuda").manual_seed(nbytes)
    src = torch.randint(0, 256, (nbytes + 2 * guard,), dtype=torch.uint8, device="cuda", generator=gen)
    dst = torch.full((nbytes + 2 * guard,), 0xA5, dtype=torch.uint8, device="cuda")
    flmoe.fl_moe_debug_copy(dst[guard:], src[guard:], nbytes)
    torch.cuda.synchronize()
    assert torch.equal(dst[guard:guard + nbytes], src[guard:guard + nbytes])
    assert bool((dst[:guard] == 0xA5).all()) and bool((dst[guard + nbytes:] == 0xA5).all())
    flmoe.fl_moe_debug_fill(dst[guard:], nbytes)
    torch.cuda.synchronize()
    assert bool((dst[guard:guard + nbytes] == 0x3C).all())
    assert bool((dst[:guard] == 0xA5).all()) and bool((dst[guard + nbytes:] == 0xA5).all())
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    before = src.clone()
    flmoe.fl_moe_debug_read(src[guard:], nbytes, sink)
    torch.cuda.synchronize()
    assert torch.equal(src, before)
    with pytest.raises(flmoe.FlMoeError):
        flmoe.fl_moe_debug_copy(dst[guard:], src[guard:], 24)          # not a multiple of 16


def test_host_visible_argument_errors():
    inp, dev, sh = small_shuffle()
    try:
        with pytest.raises(flmoe.FlMoeError) as ei:
            sh.layout(dev["indices"], dev["num_tokens"], ranks=(3, 2))
        assert ei.value.code == flmoe.FL_ERR_INVALID_ARG
        with pytest.raises(flmoe.FlMoeError):
            flmoe.fl_moe_dispatch_send(sh.ctx, 0, 4, None)
        small = torch.empty(1024, dtype=torch.uint8, device="cuda")
        with pytest.raises(flmoe.FlMoeError) as ei:
            flmoe.fl_moe_create(sh.cfg, small)
        assert ei.value.code == flmoe.FL_ERR_WORKSPACE
    finally:
        sh.close()


def test_c_caller_without_python_or_torch():
    """The library serves a plain C++ host program (hipMalloc'd buffers, no torch):
    expert-major rows checked against their definition, identity round trip bit-exact."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    exe = os.path.join(root, "tests", "c_abi_roundtrip.bin")
    if not os.path.exists(exe):
        sys.path.insert(0, root)
        import __graft_entry__ as entry
        entry.build_c_caller(flmoe.lib()._name)
    run = subprocess.run([exe], capture_output=True, text=True, timeout=100)
    assert run.returncode == 0, run.stdout + run.stderr
    assert "c abi roundtrip ok" in run.stdout
