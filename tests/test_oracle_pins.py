"""Pins for the CPU oracle: every check here compares oracle/ with something that
is NOT the oracle - brute force, a closed form, an invariant of the problem, a
library routine, or a fact the paper states (tests/golden/paper_facts.json).

CPU only.  The paper prints no worked example of a dispatch, so none of the
expected values is a number from the paper; the facts file holds the shapes and
the buffer bound it does state.
"""
import itertools
import json
import math
import os

import numpy as np
import pytest
import torch

from oracle import oracle as orc
from oracle.reference_step import oracle_step
from paper_2510_27656_amd import workloads as wlmod

HERE = os.path.dirname(os.path.abspath(__file__))
FACTS = json.load(open(os.path.join(HERE, "golden", "paper_facts.json")))


# ----------------------------------------------------------------- helpers
def bf16_to_f32(bits):
    return (bits.astype(np.uint32) << 16).view(np.float32)


def f32_to_bf16_torch(a):
    """Library routine for fp32 -> bf16 (round to nearest even)."""
    return torch.from_numpy(np.ascontiguousarray(a, np.float32)).to(torch.bfloat16) \
        .view(torch.int16).numpy().view(np.uint16)


def bf16_ulp_distance(a_bits, b_bits):
    """Distance in representable bf16 steps (finite values)."""
    def key(b):
        b = b.astype(np.int32)
        return np.where(b & 0x8000, -(b & 0x7fff), b & 0x7fff)
    return np.abs(key(a_bits) - key(b_bits))


def brute_force_layout(N, E, K, num_tokens, indices, align=1):
    """Stable sort of all (token, expert) pairs by (expert, source rank, token)."""
    El = E // N
    pairs = []
    for s in range(N):
        for t in range(int(num_tokens[s])):
            for k in range(K):
                pairs.append((int(indices[s, t, k]), s, t, k))
    pairs = sorted(pairs, key=lambda p: (p[0], p[1], p[2]))
    slot = -np.ones(indices.shape, np.int64)
    rows = {d: [] for d in range(N)}          # per rank: list of (s,t) or None (padding)
    for d in range(N):
        for j in range(El):
            e = d * El + j
            for (ee, s, t, k) in pairs:
                if ee == e:
                    slot[s, t, k] = len(rows[d])
                    rows[d].append((s, t))
            if j + 1 < El:
                while len(rows[d]) % align:
                    rows[d].append(None)
    return slot, rows


def small_case(N, E, T, K, H, seed, ragged=False):
    wl = wlmod.custom("case", N, E, T, H, K, seed, ragged=ragged)
    return wlmod.make_inputs(wl)


CASES = [
    dict(N=2, E=8, T=16, K=2, H=8, seed=0),
    dict(N=4, E=32, T=37, K=4, H=8, seed=1, ragged=True),
    dict(N=3, E=6, T=9, K=3, H=8, seed=2, ragged=True),
    dict(N=1, E=4, T=20, K=2, H=8, seed=3),
    dict(N=8, E=8, T=11, K=5, H=8, seed=4),          # one expert per rank
    dict(N=2, E=64, T=13, K=8, H=8, seed=5),         # K < El
]


# ----------------------------------------------------------------- counts / offsets
@pytest.mark.parametrize("case", CASES + [dict(N=32, E=256, T=128, K=8, H=8, seed=2)])
def test_count_invariants(case):
    inp = small_case(**case)
    N, E, K, T = case["N"], case["E"], case["K"], case["T"]
    El = E // N
    nt = inp.num_tokens
    lay = orc.layout(N, E, K, nt, inp.indices)
    # library routine: histogram
    for s in range(N):
        ref = np.bincount(inp.indices[s, :nt[s]].reshape(-1), minlength=E)
        assert (lay.C[s] == ref).all()
    assert (lay.C.sum(1) == nt.astype(np.int64) * K).all()
    assert lay.G.sum() == int(nt.sum()) * K
    assert (lay.G == lay.C.reshape(N, N, El).sum(0)).all()
    Cd = lay.C.reshape(N, N, El)
    assert (Cd.max(2) <= lay.M).all()
    assert (lay.M <= np.minimum(nt[:, None], Cd.sum(2))).all()
    assert (nt <= lay.M.sum(1)).all() or (nt == 0).any()
    assert (lay.M.sum(1) >= nt).all()
    assert (lay.M.sum(1) <= nt * min(K, N)).all()
    # offsets are exclusive scans of the counts
    z = np.zeros((N, 1), np.int64)
    assert (lay.send_off == np.concatenate([z, np.cumsum(lay.M, 1)], 1)).all()
    assert (lay.recv_off == np.concatenate([z, np.cumsum(lay.M.T, 1)], 1)).all()
    assert (lay.expert_off == np.concatenate([z, np.cumsum(lay.G, 1)], 1)).all()
    assert (lay.comb_off == np.concatenate([z, np.cumsum(Cd.sum(2), 1)], 1)).all()
    # the paper's receive-buffer bound (see paper_facts.json: N*T*max(R, E/N))
    bound = N * T * max(K, El)
    assert (lay.recv_off[:, -1] <= bound).all()
    assert (lay.expert_off[:, -1] <= bound).all()
    # tighter bounds used for capacity checks
    assert (lay.recv_off[:, -1] <= N * T).all()
    assert (lay.expert_off[:, -1] <= N * T * min(K, El)).all()


def dedup_counts_by_sets(N, E, num_tokens, indices):
    """M[s][d] as the definition reads: the number of tokens of s with any expert on d."""
    El = E // N
    M = np.zeros((N, N), np.int64)
    for s in range(N):
        for d in range(N):
            M[s, d] = len({t for t in range(int(num_tokens[s]))
                           if any(int(e) // El == d for e in indices[s, t])})
    return M


@pytest.mark.parametrize("case", CASES + [dict(N=4, E=32, T=300, K=8, H=8, seed=6, ragged=True),
                                          dict(N=16, E=16, T=40, K=16, H=8, seed=7)])
def test_dedup_counts_equal_the_set_definition(case):
    """Every entry of M against a Python set per (source, destination rank); the routed
    tokens include ones with several experts on one rank (the case de-duplication is for)."""
    inp = small_case(**case)
    N, E, K = case["N"], case["E"], case["K"]
    lay = orc.layout(N, E, K, inp.num_tokens, inp.indices)
    want = dedup_counts_by_sets(N, E, inp.num_tokens, inp.indices)
    assert (lay.M == want).all()
    if K > 1 and E // N > 1:
        pairs_per_rank = lay.C.reshape(N, N, E // N).sum(2)
        assert (lay.M < pairs_per_rank).any(), "no token had two experts on one rank: weak case"
    # rows of absent tokens never count: the same indices with fewer tokens
    fewer = np.maximum(inp.num_tokens - 3, 0).astype(np.int32)
    lay2 = orc.layout(N, E, K, fewer, inp.indices)
    assert (lay2.M == dedup_counts_by_sets(N, E, fewer, inp.indices)).all()


@pytest.mark.parametrize("name", ["tiny", "dsv3_decode", "dsv3_prefill", "qwen3_skew", "dsv3_fp8"])
def test_workload_description_counts_the_oracles_dedup_rows(name):
    """workloads.describe() feeds the bench's byte counts; its D (counted by sorting owner
    ranks per token) must be the oracle's sum of M, and its pair count the sum of C."""
    inp = wlmod.make_inputs(wlmod.WORKLOADS[name], with_x=False)
    wl = inp.wl
    L = orc.lib()
    M = np.empty((wl.n_ranks, wl.n_ranks), np.int32)
    Cc = np.empty((wl.n_ranks, wl.n_experts), np.int32)
    L.orc_dedup_counts(wl.n_ranks, wl.n_experts, wl.tokens, wl.top_k, orc._p(inp.num_tokens),
                       orc._p(inp.indices), orc._p(M))
    L.orc_counts(wl.n_ranks, wl.n_experts, wl.tokens, wl.top_k, orc._p(inp.num_tokens),
                 orc._p(inp.indices), orc._p(Cc))
    d = wlmod.describe(inp)
    assert d["dedup_rows"] == int(M.astype(np.int64).sum())
    assert d["pairs"] == int(Cc.astype(np.int64).sum())
    assert d["tokens_total"] == int(inp.num_tokens.sum())
    assert d["max_rank_rows"] == int(Cc.astype(np.int64).reshape(wl.n_ranks, wl.n_ranks, -1).sum((0, 2)).max())


@pytest.mark.parametrize("align", [1, 4, 16])
@pytest.mark.parametrize("case", CASES)
def test_layout_matches_brute_force_sort(case, align):
    inp = small_case(**case)
    N, E, K = case["N"], case["E"], case["K"]
    lay = orc.layout(N, E, K, inp.num_tokens, inp.indices, align)
    slot, rows = brute_force_layout(N, E, K, inp.num_tokens, inp.indices, align)
    assert (lay.slot == slot).all()
    for d in range(N):
        got = orc.dispatch_rank(d, N, E, K, inp.num_tokens, inp.indices, inp.x, align,
                                zero_pad=True)
        # strip trailing padding of the brute-force list (last expert is not padded)
        assert got.shape[0] == len(rows[d])
        for r, st in enumerate(rows[d]):
            if st is None:
                assert not got[r].any()
            else:
                assert (got[r] == inp.x[st[0], st[1]]).all()
        # padding offsets: every expert starts on a multiple of align
        assert (lay.expert_off[d, :-1] % align == 0).all()


def test_padding_rows_untouched_without_zero_pad():
    inp = small_case(N=2, E=8, T=16, K=2, H=8, seed=7)
    lay = orc.layout(2, 8, 2, inp.num_tokens, inp.indices, 8)
    for d in range(2):
        got = orc.dispatch_rank(d, 2, 8, 2, inp.num_tokens, inp.indices, inp.x, 8,
                                zero_pad=False, fill=0xAB)
        El = 4
        for j in range(El - 1):
            lo = lay.expert_off[d, j] + lay.G[d, j]
            hi = lay.expert_off[d, j + 1]
            assert (got[lo:hi].view(np.uint8) == 0xAB).all()


def test_exhaustive_two_ranks_two_tokens():
    """Every routing of N=2, E=4, T=2, K=2 (12^4 = 20736 cases)."""
    N, E, T, K = 2, 4, 2, 2
    choices = [p for p in itertools.permutations(range(E), K)]
    assert len(choices) == 12
    nt = np.full((N,), T, np.int32)
    n = 0
    for combo in itertools.product(choices, repeat=N * T):
        idx = np.array(combo, np.int32).reshape(N, T, K)
        lay = orc.layout(N, E, K, nt, idx)
        # de-duplicated counts: a token counts once per rank that hosts any of its experts
        for s in range(N):
            for d in range(N):
                assert lay.M[s, d] == len({t for t in range(T) if d in (idx[s, t, 0] // 2, idx[s, t, 1] // 2)})
        # brute force, written inline: position = number of pairs with a smaller key
        for s in range(N):
            for t in range(T):
                for k in range(K):
                    e = idx[s, t, k]
                    d = e // 2
                    before = 0
                    for s2 in range(N):
                        for t2 in range(T):
                            for k2 in range(K):
                                e2 = idx[s2, t2, k2]
                                if e2 // 2 == d and (e2, s2, t2) < (e, s, t):
                                    before += 1
                    assert lay.slot[s, t, k] == before
        n += 1
    assert n == 20736


def test_all_tokens_to_one_expert():
    N, E, T, K, H = 4, 8, 5, 1, 8
    inp = small_case(N, E, T, K, H, seed=11)
    idx = np.full((N, T, K), 5, np.int32)
    nt = np.array([5, 3, 0, 4], np.int32)
    d = 5 // (E // N)
    got = orc.dispatch_rank(d, N, E, K, nt, idx, inp.x)
    expect = np.concatenate([inp.x[s, :nt[s]] for s in range(N)], 0)
    assert (got == expect).all()
    for other in range(N):
        if other != d:
            assert orc.dispatch_rank(other, N, E, K, nt, idx, inp.x).shape[0] == 0


def test_single_rank_top1_is_stable_argsort():
    N, E, T, K, H = 1, 16, 200, 1, 8
    inp = small_case(N, E, T, K, H, seed=12)
    got = orc.dispatch_rank(0, N, E, K, inp.num_tokens, inp.indices, inp.x)
    order = np.argsort(inp.indices[0, :, 0], kind="stable")
    assert (got == inp.x[0][order]).all()


@pytest.mark.parametrize("case", CASES)
def test_rows_are_a_permutation_of_routed_inputs(case):
    inp = small_case(**case)
    N, E, K = case["N"], case["E"], case["K"]
    nt = inp.num_tokens
    # tag every token with a unique id so that rows can be traced
    tags = np.arange(N * inp.x.shape[1], dtype=np.int64).reshape(N, -1, 1)
    tags = np.ascontiguousarray(tags)
    seen = []
    for d in range(N):
        seen.append(orc.dispatch_rank(d, N, E, K, nt, inp.indices, tags)[:, 0])
    seen = np.sort(np.concatenate(seen))
    expect = np.sort(np.concatenate(
        [np.repeat(tags[s, :nt[s], 0], K) for s in range(N)]))
    assert (seen == expect).all()


def test_dedup_rate_closed_form_uniform_routing():
    """Uniform top-8 of 256 experts on 32 ranks: the expected number of distinct
    destination ranks per token is N * (1 - C(E-El, K) / C(E, K))."""
    wl = wlmod.WORKLOADS["dsv3_decode"]
    inp = wlmod.make_inputs(wl, with_x=False)
    lay = orc.layout(wl.n_ranks, wl.n_experts, wl.top_k, inp.num_tokens, inp.indices)
    N, E, K, El = wl.n_ranks, wl.n_experts, wl.top_k, wl.experts_per_rank
    expect = N * (1 - math.comb(E - El, K) / math.comb(E, K))
    got = lay.M.sum() / inp.num_tokens.sum()
    assert abs(expect - 7.267) < 1e-3
    assert abs(got - expect) < 0.05
    # shape facts the paper states for this workload
    mb = FACTS["microbenchmark_shape"]
    assert wl.hidden == mb["hidden"] and wl.top_k == mb["experts_per_token"]
    assert wl.tokens == mb["decode_tokens_per_rank"]
    assert wl.hidden // 128 == mb["fp8_scales_per_token"]
    assert wlmod.WORKLOADS["dsv3_prefill"].tokens == mb["prefill_tokens_per_rank"]


@pytest.mark.parametrize("case", CASES)
def test_recv_order_and_comb_pos_self_consistent(case):
    """Internal buffer orders (this build's own choice): every (source, token,
    destination) with a route appears once, keys strictly increase, and the
    combine positions are a permutation of 0..T_s*K-1 sorted by (expert, token)."""
    inp = small_case(**case)
    N, E, K = case["N"], case["E"], case["K"]
    El = E // N
    nt = inp.num_tokens
    lay = orc.layout(N, E, K, nt, inp.indices)
    for d in range(N):
        sr, st, mk = orc.recv_order(d, N, E, K, nt, inp.indices)
        assert len(sr) == lay.recv_off[d, -1]
        keys = sr.astype(np.int64) * 100000 + st
        assert (np.diff(keys) > 0).all()
        for r in range(len(sr)):
            want = {int(e) - d * El for e in inp.indices[sr[r], st[r]] if e // El == d}
            have = {j for j in range(El) if (int(mk[r]) >> j) & 1}
            assert want == have and want
        for s in range(N):
            assert (sr == s).sum() == lay.M[s, d]
    cp = orc.comb_pos(N, E, K, nt, inp.indices)
    for s in range(N):
        v = cp[s, :nt[s]].reshape(-1)
        assert sorted(v.tolist()) == list(range(nt[s] * K))
        e = inp.indices[s, :nt[s]].reshape(-1)
        t = np.repeat(np.arange(nt[s]), K)
        order = np.lexsort((t, e))
        assert (v[order] == np.arange(len(v))).all()
        assert (cp[s, nt[s]:] == -1).all()


# ----------------------------------------------------------------- combine
def run_dispatch_all(inp, N, E, K, align=1):
    lay = orc.layout(N, E, K, inp.num_tokens, inp.indices, align)
    stride = int(lay.expert_off[:, -1].max())
    H = inp.x.shape[2]
    Y = np.zeros((N, max(stride, 1), H), np.uint16)
    for d in range(N):
        rows = orc.dispatch_rank(d, N, E, K, inp.num_tokens, inp.indices, inp.x, align,
                                 zero_pad=True)
        Y[d, :rows.shape[0]] = rows
    return lay, Y, max(stride, 1)


@pytest.mark.parametrize("case", [
    dict(N=2, E=8, T=16, K=2, H=256, seed=0),
    dict(N=4, E=32, T=37, K=4, H=64, seed=1, ragged=True),
    dict(N=8, E=64, T=16, K=8, H=64, seed=2),
])
def test_round_trip_identity_is_bit_exact(case):
    """dispatch -> identity experts -> combine returns the input when the weights
    sum to one: the fp32 error (about K * 2^-24) is far below half a bf16 step."""
    inp = small_case(**case)
    N, E, K, H = case["N"], case["E"], case["K"], case["H"]
    lay, Y, stride = run_dispatch_all(inp, N, E, K)
    out = orc.combine(N, E, K, inp.num_tokens, inp.indices, lay.slot, inp.weights, Y,
                      stride, H)
    for s in range(N):
        n = inp.num_tokens[s]
        assert (out[s, :n] == inp.x[s, :n]).all()
        assert not out[s, n:].any()


def emulate_fma_chain(w, y):
    """fp32 fused multiply-add chain evaluated through exact float64 steps.
    w [n][K] fp32, y [n][K][H] fp32 -> (acc fp32 [n][H], exact mask [n][H])."""
    n, K, H = y.shape
    acc = np.zeros((n, H), np.float32)
    exact = np.ones((n, H), bool)
    for k in range(K):
        p = w[:, k, None].astype(np.float64) * y[:, k].astype(np.float64)   # exact: 24 x 8 bits
        a = acc.astype(np.float64)
        s = p + a
        bb = s - p
        err = (p - (s - bb)) + (a - bb)                                     # TwoSum residual
        exact &= (err == 0)
        acc = s.astype(np.float32)                                          # one rounding
    return acc, exact


@pytest.mark.parametrize("K", [1, 2, 8])
def test_combine_matches_exact_fma_chain_and_fp64(K):
    N, E, T, H = 4, 32, 24, 64
    inp = small_case(N, E, T, K, H, seed=20 + K)
    g = (1.0 + np.arange(E, dtype=np.float32) / 256.0).astype(np.float32)
    lay, Y, stride = run_dispatch_all(inp, N, E, K)
    for d in range(N):
        orc.expert_scale_rank(d, N, E, lay, g, H, Y[d])
    out, acc32 = orc.combine(N, E, K, inp.num_tokens, inp.indices, lay.slot, inp.weights, Y,
                             stride, H, return_acc=True)
    El = E // N
    owner = inp.indices // El
    yk = bf16_to_f32(Y[owner, lay.slot])                   # gather [N][T][K][H]
    # (a) expert stage against a library routine
    xk = bf16_to_f32(inp.x)[:, :, None, :] * g[inp.indices][..., None]
    assert (f32_to_bf16_torch(xk) == Y[owner, lay.slot]).all()
    # (b) fixed-order fp32 FMA chain, evaluated exactly
    acc, exact = emulate_fma_chain(inp.weights.reshape(-1, K), yk.reshape(-1, K, H))
    ref = f32_to_bf16_torch(acc).reshape(N, T, H)
    exact = exact.reshape(N, T, H)
    assert exact.mean() > 0.9
    assert (out[exact] == ref[exact]).all()
    # the fp32 accumulator itself, bit for bit (separates a fused multiply-add from
    # a rounded product followed by an add, which the bf16 result rarely shows)
    assert (acc32.view(np.uint32)[exact] == acc.reshape(N, T, H).view(np.uint32)[exact]).all()
    assert (out == f32_to_bf16_torch(acc32)).all()
    # (c) fp64 einsum: the exact sum, rounded once, is within one bf16 step
    ref64 = np.einsum("stk,stkh->sth", inp.weights.astype(np.float64), yk.astype(np.float64))
    ref64_b = f32_to_bf16_torch(ref64.astype(np.float32))
    assert bf16_ulp_distance(out, ref64_b).max() <= 1


def test_combine_order_is_k_order_not_sorted():
    """Reversing the k order of (indices, weights) must be able to change bits:
    guards against an oracle that sums in expert or slot order."""
    N, E, T, K, H = 2, 16, 64, 8, 64
    inp = small_case(N, E, T, K, H, seed=31)
    g = (1.0 + np.arange(E, dtype=np.float32) / 256.0).astype(np.float32)
    lay, Y, stride = run_dispatch_all(inp, N, E, K)
    for d in range(N):
        orc.expert_scale_rank(d, N, E, lay, g, H, Y[d])
    out = orc.combine(N, E, K, inp.num_tokens, inp.indices, lay.slot, inp.weights, Y, stride, H)
    idx_r = np.ascontiguousarray(inp.indices[:, :, ::-1])
    w_r = np.ascontiguousarray(inp.weights[:, :, ::-1])
    lay_r = orc.layout(N, E, K, inp.num_tokens, idx_r)
    out_r, acc_r = orc.combine(N, E, K, inp.num_tokens, idx_r, lay_r.slot, w_r, Y, stride, H,
                               return_acc=True)
    El = E // N
    yk = bf16_to_f32(Y[idx_r // El, lay_r.slot])
    acc, exact = emulate_fma_chain(w_r.reshape(-1, K), yk.reshape(-1, K, H))
    ref = f32_to_bf16_torch(acc).reshape(N, T, H)
    exact = exact.reshape(N, T, H)
    assert (out_r[exact] == ref[exact]).all()
    assert (acc_r.view(np.uint32)[exact] == acc.reshape(N, T, H).view(np.uint32)[exact]).all()
    assert bf16_ulp_distance(out, out_r).max() <= 1
    # the two orders really differ somewhere in fp32, so the check above has teeth
    _, acc_f = orc.combine(N, E, K, inp.num_tokens, inp.indices, lay.slot, inp.weights, Y,
                           stride, H, return_acc=True)
    assert (acc_f != acc_r).any()


# ----------------------------------------------------------------- combine with sender-side partial sums
def partial_reference(indices, weights, yk, El):
    """Independent evaluation of the partial-sum combine for a flat list of tokens:
    indices [n][K], weights [n][K] fp32, yk [n][K][H] fp32.  A rank's share is the fp32
    fused multiply-add chain with the other ranks' weights set to zero (adding 0*y
    leaves an fp32 accumulator unchanged), rounded to bf16; shares are added in fp32
    with numpy's float32 arithmetic in the order of each rank's first k."""
    n, K, H = yk.shape
    owner = indices // El
    total = np.zeros((n, H), np.float32)
    exact = np.ones((n, H), bool)
    for k in range(K):
        first = np.ones(n, bool)
        for k2 in range(k):
            first &= owner[:, k2] != owner[:, k]
        wmask = np.where(owner == owner[:, k:k + 1], weights, np.float32(0)).astype(np.float32)
        part, ex = emulate_fma_chain(wmask, yk)
        part_b = bf16_to_f32(f32_to_bf16_torch(part))
        total = np.where(first[:, None], total + part_b, total).astype(np.float32)
        exact &= ex | ~first[:, None]
    return f32_to_bf16_torch(total), exact


def test_partial_combine_equals_exact_combine_when_one_rank_hosts_everything():
    """With a single rank there is one partial sum per token, the full chain, and
    rounding it twice to bf16 changes nothing."""
    N, E, T, K, H = 1, 16, 40, 6, 64
    inp = small_case(N, E, T, K, H, seed=71)
    g = (1.0 + np.arange(E, dtype=np.float32) / 256.0).astype(np.float32)
    lay, Y, stride = run_dispatch_all(inp, N, E, K)
    orc.expert_scale_rank(0, N, E, lay, g, H, Y[0])
    a = orc.combine(N, E, K, inp.num_tokens, inp.indices, lay.slot, inp.weights, Y, stride, H)
    b = orc.combine_partial(N, E, K, inp.num_tokens, inp.indices, lay.slot, inp.weights, Y, stride, H)
    assert (a == b).all()


def test_partial_combine_with_one_expert_per_rank_is_a_sum_of_rounded_products():
    """E = N: every share is a single product w*y rounded to fp32 and then to bf16,
    and the receiver adds K bf16 numbers in fp32 in k order."""
    N, E, T, K, H = 8, 8, 32, 5, 64
    inp = small_case(N, E, T, K, H, seed=72)
    lay, Y, stride = run_dispatch_all(inp, N, E, K)
    out = orc.combine_partial(N, E, K, inp.num_tokens, inp.indices, lay.slot, inp.weights, Y, stride, H)
    yk = bf16_to_f32(Y[inp.indices, lay.slot]).astype(np.float64)          # owner == expert
    prod = (inp.weights.astype(np.float64)[..., None] * yk).astype(np.float32)   # exact product, one rounding
    shares = bf16_to_f32(f32_to_bf16_torch(prod))
    total = np.zeros((N, T, H), np.float32)
    for k in range(K):
        total = (total + shares[:, :, k]).astype(np.float32)
    assert (out == f32_to_bf16_torch(total)).all()


def test_partial_combine_hand_example_differs_from_exact_combine():
    """Worked by hand.  One token, weights 1, experts 0 and 1 on rank 0 and expert 2
    on rank 1, y = (1, 2^-8, 2^-9); one bf16 step at 1.0 is 2^-7.
    Exact combine: 1 + 2^-8 + 2^-9 = 1 + 0.75 steps -> 1 + 2^-7 (0x3F81).
    Partial sums: rank 0 holds 1 + 2^-8 = 1 + half a step, a tie that rounds to the
    even neighbour 1.0; adding rank 1's 2^-9 gives 1 + a quarter step -> 1.0 (0x3F80)."""
    N, E, T, K, H = 2, 4, 1, 3, 8
    idx = np.array([[[0, 1, 2]], [[0, 1, 2]]], np.int32)
    nt = np.array([1, 0], np.int32)
    w = np.ones((N, T, K), np.float32)
    lay = orc.layout(N, E, K, nt, idx)
    stride = 4
    Y = np.zeros((N, stride, H), np.uint16)
    vals = [1.0, 2.0 ** -8, 2.0 ** -9]
    for k in range(K):
        Y[idx[0, 0, k] // 2, lay.slot[0, 0, k]] = f32_to_bf16_torch(np.full(H, vals[k], np.float32))
    exact = orc.combine(N, E, K, nt, idx, lay.slot, w, Y, stride, H)
    part = orc.combine_partial(N, E, K, nt, idx, lay.slot, w, Y, stride, H)
    assert (exact[0, 0] == 0x3F81).all()
    assert (part[0, 0] == 0x3F80).all()
    # the same three experts listed with rank 1 first: 2^-9 + 1.0 is again a quarter step
    idx2 = np.ascontiguousarray(idx[:, :, [2, 0, 1]])
    lay2 = orc.layout(N, E, K, nt, idx2)
    Y2 = np.zeros_like(Y)
    for k, v in enumerate([vals[2], vals[0], vals[1]]):
        Y2[idx2[0, 0, k] // 2, lay2.slot[0, 0, k]] = f32_to_bf16_torch(np.full(H, v, np.float32))
    part2 = orc.combine_partial(N, E, K, nt, idx2, lay2.slot, w, Y2, stride, H)
    assert (part2[0, 0] == 0x3F80).all()


def test_partial_combine_adds_shares_in_order_of_first_k():
    """Worked by hand.  Three ranks with one expert each, the token lists experts
    (2, 0, 1) with rows 1, 2^-24, -1 and weights 1.  In the order of first k:
    1 + 2^-24 is a tie in fp32 and rounds to 1 (even), then 1 - 1 = +0.  Any order
    that adds 1 and -1 first, or starts from 2^-24 (ascending rank: 2^-24 - 1 + 1),
    ends at 2^-24 instead."""
    N, E, T, K, H = 3, 3, 1, 3, 8
    idx = np.zeros((N, T, K), np.int32)
    idx[:] = [2, 0, 1]
    nt = np.array([1, 0, 0], np.int32)
    w = np.ones((N, T, K), np.float32)
    lay = orc.layout(N, E, K, nt, idx)
    Y = np.zeros((N, 2, H), np.uint16)
    for k, v in enumerate([1.0, 2.0 ** -24, -1.0]):
        Y[idx[0, 0, k], lay.slot[0, 0, k]] = f32_to_bf16_torch(np.full(H, v, np.float32))
    out = orc.combine_partial(N, E, K, nt, idx, lay.slot, w, Y, 2, H)
    assert (out[0, 0] == 0x0000).all()
    # the exact combine adds products in the same k order and agrees here
    assert (orc.combine(N, E, K, nt, idx, lay.slot, w, Y, 2, H)[0, 0] == 0x0000).all()


@pytest.mark.parametrize("N,E,K", [(4, 32, 8), (2, 16, 6), (8, 16, 4)])
def test_partial_combine_matches_grouped_evaluation(N, E, K):
    T, H = 24, 64
    inp = small_case(N, E, T, K, H, seed=80 + N)
    g = (1.0 + np.arange(E, dtype=np.float32) / 256.0).astype(np.float32)
    lay, Y, stride = run_dispatch_all(inp, N, E, K)
    for d in range(N):
        orc.expert_scale_rank(d, N, E, lay, g, H, Y[d])
    out = orc.combine_partial(N, E, K, inp.num_tokens, inp.indices, lay.slot, inp.weights, Y, stride, H)
    El = E // N
    yk = bf16_to_f32(Y[inp.indices // El, lay.slot])
    ref, exact = partial_reference(inp.indices.reshape(-1, K), inp.weights.reshape(-1, K),
                                   yk.reshape(-1, K, H), El)
    ref, exact = ref.reshape(N, T, H), exact.reshape(N, T, H)
    assert exact.mean() > 0.9
    assert (out[exact] == ref[exact]).all()
    # against the exact combine: each share is rounded to bf16 once more, so the two
    # differ by a few bf16 steps at most, and they do differ somewhere
    full = orc.combine(N, E, K, inp.num_tokens, inp.indices, lay.slot, inp.weights, Y, stride, H)
    dist = bf16_ulp_distance(out, full)
    assert dist.max() <= K
    if N > 1:
        assert dist.max() >= 1


def test_unnormalised_weights_scale_the_output():
    N, E, T, K, H = 2, 8, 16, 2, 64
    inp = small_case(N, E, T, K, H, seed=33)
    w = (inp.weights * 3.0).astype(np.float32)
    lay, Y, stride = run_dispatch_all(inp, N, E, K)
    out = orc.combine(N, E, K, inp.num_tokens, inp.indices, lay.slot, w, Y, stride, H)
    x = bf16_to_f32(inp.x)
    got = bf16_to_f32(out)
    want = x * w.sum(-1, keepdims=True)
    assert np.allclose(got, want, rtol=2 ** -7, atol=1e-30)   # no division by the weight sum


# ----------------------------------------------------------------- bf16
def test_bf16_rounding_against_torch_all_interesting_values():
    rng = np.random.default_rng(0)
    a = rng.standard_normal(200000).astype(np.float32)
    # add exact ties, subnormals, large values
    ties = ((np.arange(1, 4000, dtype=np.uint32) << 16) | 0x8000).view(np.float32)
    a = np.concatenate([a, ties, -ties, np.float32([0, -0.0, 1e-40, -1e-40, 3.3e38, -3.3e38])])
    a = np.ascontiguousarray(a, np.float32)
    assert (orc.f32_to_bf16_array(a) == f32_to_bf16_torch(a)).all()


# ----------------------------------------------------------------- fp8 e4m3
def e4m3_table():
    """All 256 codes of the OCP E4M3 finite-only format, from its definition:
    sign, 4-bit exponent (bias 7), 3-bit mantissa; exponent 0 is subnormal
    (mantissa * 2^-9); code 0x7f / 0xff is NaN; no infinities."""
    vals = np.zeros(256, np.float64)
    for c in range(256):
        s, e, m = c >> 7, (c >> 3) & 15, c & 7
        if e == 0:
            v = m * 2.0 ** -9
        elif e == 15 and m == 7:
            v = float("nan")
        else:
            v = (1 + m / 8) * 2.0 ** (e - 7)
        vals[c] = -v if s else v
    return vals


def test_e4m3_decode_table_and_torch():
    tab = e4m3_table()
    codes = np.arange(256, dtype=np.uint8)
    got = orc.e4m3_decode_array(codes)
    ok = ~np.isnan(tab)
    assert (got[ok].astype(np.float64) == tab[ok]).all()
    assert np.isnan(got[~ok]).all()
    assert np.nanmax(tab) == 448.0
    if hasattr(torch, "float8_e4m3fn"):
        tt = torch.from_numpy(codes.copy()).view(torch.float8_e4m3fn).float().numpy()
        assert (tt[ok] == got[ok]).all()


def nearest_code_reference(v):
    """Independent encoder: search all finite codes for the nearest value; ties go
    to the code with an even mantissa; saturate beyond +-448."""
    tab = e4m3_table()
    pos_codes = np.array([c for c in range(127)], np.int64)          # 0x00..0x7e finite
    pos_vals = tab[pos_codes]
    a = np.abs(v.astype(np.float64))
    a = np.minimum(a, 448.0)
    dist = np.abs(a[:, None] - pos_vals[None, :])
    best = dist.min(1)
    cand = dist == best[:, None]
    # at most two candidates (adjacent codes): pick the even one on a tie
    even = (pos_codes % 2 == 0)[None, :]
    pick_even = cand & even
    choice = np.where(cand.sum(1) > 1, np.argmax(pick_even, 1), np.argmax(cand, 1))
    code = pos_codes[choice]
    return (code | np.where(np.signbit(v), 0x80, 0)).astype(np.uint8)


def test_e4m3_encode_exhaustive_against_nearest_code_search():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    x = bf16_to_f32(bits)
    finite = np.isfinite(x)
    x = x[finite]
    for scale in [1.0, 0.0123, 448.0 / 3.0, 2.0 ** -20, 7.7]:
        v = np.ascontiguousarray((x / np.float32(scale)).astype(np.float32))
        v = v[np.isfinite(v)]
        got = orc.e4m3_encode_array(v)
        for lo in range(0, len(v), 8192):
            ref = nearest_code_reference(v[lo:lo + 8192])
            assert (got[lo:lo + 8192] == ref).all(), scale
    # explicit ties: halfway between adjacent codes
    tab = e4m3_table()
    mids = np.array([(tab[c] + tab[c + 1]) / 2 for c in range(0, 126)], np.float32)
    got = orc.e4m3_encode_array(np.ascontiguousarray(mids))
    assert (got == np.array([c if c % 2 == 0 else c + 1 for c in range(0, 126)], np.uint8)).all()
    if hasattr(torch, "float8_e4m3fn"):
        rng = np.random.default_rng(1)
        v = (rng.standard_normal(100000) * 100).astype(np.float32)
        v = v[np.abs(v) <= 448]
        tt = torch.from_numpy(v).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
        assert (orc.e4m3_encode_array(np.ascontiguousarray(v)) == tt).all()


def test_block_quantisation_invariants():
    rng = np.random.default_rng(2)
    H = FACTS["microbenchmark_shape"]["hidden"]
    x = f32_to_bf16_torch(rng.standard_normal((6, H)).astype(np.float32))
    x[1, :128] = 0                         # an all-zero block
    x[2] = f32_to_bf16_torch((bf16_to_f32(x[2]) * 1e-30).astype(np.float32))   # tiny values
    q, sc = orc.quant_e4m3_block128(x)
    assert sc.shape == (6, FACTS["microbenchmark_shape"]["fp8_scales_per_token"])
    xf = bf16_to_f32(x).reshape(6, H // 128, 128)
    amax = np.abs(xf).max(-1)
    want_scale = np.where(amax == 0, np.float32(1), (amax / np.float32(448)).astype(np.float32))
    assert (sc == want_scale).all()
    assert sc[1, 0] == 1.0 and not q[1, :128].any()
    qv = orc.e4m3_decode_array(q).reshape(xf.shape)
    assert (np.abs(qv) <= 448).all()
    # the largest element of every non-zero block maps to +-448
    am = np.abs(xf).argmax(-1)
    top = np.take_along_axis(np.abs(qv), am[..., None], -1)[..., 0]
    assert (top[amax > 0] == 448).all()
    # relative error at most half a step (2^-4) wherever the result is a normal number
    deq = qv * sc[..., None]
    normal = np.abs(qv) >= 2.0 ** -6
    rel = np.abs(deq - xf)[normal] / np.abs(xf)[normal]
    assert rel.max() <= 2.0 ** -4 * (1 + 1e-6)
    # the code is what the independent search gives for x / scale
    v = (xf / sc[..., None]).astype(np.float32).reshape(-1)
    ref = nearest_code_reference(v)
    assert (q.reshape(-1) == ref).all()
    # dequantise: bf16(float(q) * scale) against a library rounding
    y = orc.dequant_e4m3_block128(q, sc)
    assert (y == f32_to_bf16_torch((qv * sc[..., None]).astype(np.float32)).reshape(6, H)).all()


def test_block_quantisation_of_inf_and_nan_follows_the_stated_reading():
    """Expected bytes and scales written out by hand from the reading: NaN is skipped by
    the maximum and becomes 0x7f | its sign; Inf makes the scale +Inf, finite neighbours
    +-0 and itself 0x7f | its sign; the other blocks of the row are untouched."""
    to_bits = f32_to_bf16_torch
    x = np.zeros((1, 128 * 6), np.uint16)
    base = to_bits(np.linspace(-3.0, 4.0, 128).astype(np.float32))     # amax = 4 exactly, at [127]
    for b in range(6):
        x[0, b * 128:(b + 1) * 128] = base
    blk = lambda b: x[0, b * 128:(b + 1) * 128]
    blk(1)[3] = 0x7fc0; blk(1)[100] = 0xffc0; blk(1)[50] = 0x7f81      # +qNaN, -qNaN, +sNaN
    blk(2)[10] = 0x7f80                                                # +Inf
    blk(3)[20] = 0xff80; blk(3)[21] = 0x7fc0                           # -Inf and a NaN
    blk(4)[:] = 0xffc0                                                 # NaNs only
    blk(5)[:] = 0; blk(5)[7] = 0x7fc0                                  # zeros and one NaN
    q, sc = orc.quant_e4m3_block128(x)
    clean_q, clean_sc = orc.quant_e4m3_block128(np.ascontiguousarray(base.reshape(1, 128)))
    assert clean_sc[0, 0] == np.float32(4.0) / np.float32(448.0)
    qb = lambda b: q[0, b * 128:(b + 1) * 128]
    # block 0: no special value
    assert (qb(0) == clean_q[0]).all() and sc[0, 0] == clean_sc[0, 0]
    # block 1: NaNs skipped by the maximum, NaN codes with the element's sign, rest unchanged
    want = clean_q[0].copy(); want[3] = 0x7f; want[100] = 0xff; want[50] = 0x7f
    assert sc[0, 1] == clean_sc[0, 0] and (qb(1) == want).all()
    # block 2: scale +Inf, finite values become zeros with their sign
    signs = (base >> 8) & 0x80
    want = signs.astype(np.uint8); want[10] = 0x7f
    assert np.isposinf(sc[0, 2]) and (qb(2) == want).all()
    want = signs.astype(np.uint8); want[20] = 0xff; want[21] = 0x7f
    assert np.isposinf(sc[0, 3]) and (qb(3) == want).all()
    assert sc[0, 4] == 1.0 and (qb(4) == 0xff).all()
    want = np.zeros(128, np.uint8); want[7] = 0x7f
    assert sc[0, 5] == 1.0 and (qb(5) == want).all()
    # the library's own conversion agrees on what a NaN becomes (code 0x7f with the sign)
    if hasattr(torch, "float8_e4m3fn"):
        t = torch.tensor([float("nan"), -float("nan")]).to(torch.float8_e4m3fn).view(torch.uint8)
        assert (t & 0x7f).tolist() == [0x7f, 0x7f]


def test_named_workloads_match_their_description():
    w = wlmod.WORKLOADS
    assert (w["tiny"].n_ranks, w["tiny"].n_experts, w["tiny"].tokens, w["tiny"].hidden,
            w["tiny"].top_k, w["tiny"].seed) == (2, 8, 16, 256, 2, 0)
    assert (w["qwen3_skew"].n_ranks, w["qwen3_skew"].n_experts, w["qwen3_skew"].tokens,
            w["qwen3_skew"].hidden, w["qwen3_skew"].top_k) == (16, 128, 256, 2048, 8)
    for name in ["qwen3_skew", "dsv3_fp8"]:
        d = wlmod.describe(wlmod.make_inputs(w[name], with_x=False))
        assert 9.0 <= d["hottest_expert_over_mean"] <= 11.0
    inp = wlmod.make_inputs(w["tiny"])
    assert np.allclose(inp.weights.sum(-1), 1.0, atol=1e-6)
    # distinct experts inside every token, listed by descending weight
    assert all(len(set(r)) == len(r) for r in inp.indices.reshape(-1, 2).tolist())
    assert (np.diff(inp.weights, axis=-1) <= 0).all()


def test_oracle_digests_unchanged():
    """Regression guard (not a pin): the oracle's outputs on the tiny workload still
    hash to what tests/golden/make_golden.py recorded."""
    import importlib.util
    spec = importlib.util.spec_from_file_location(
        "make_golden", os.path.join(HERE, "golden", "make_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    stored = json.load(open(os.path.join(HERE, "golden", "oracle_digests.json")))
    assert mod.compute() == stored


def test_sampled_combine_helper_equals_full_path():
    """The helpers used for workloads too large to lay out on the host (explicit rows,
    per-row gain) give what the full dispatch -> expert -> combine path gives."""
    from oracle.reference_step import oracle_step
    wl = wlmod.custom("c", 4, 32, 37, 64, 4, seed=1)
    inp = wlmod.make_inputs(wl)
    ref = oracle_step(inp)
    ss = np.repeat(np.arange(4), 5)
    tt = np.random.default_rng(0).integers(0, 37, ss.size)
    idx = inp.indices[ss, tt]
    y = np.repeat(inp.x[ss, tt], 4, axis=0).copy()
    orc.scale_rows(y, np.ascontiguousarray(inp.expert_gain[idx.reshape(-1)]))
    got = orc.combine_sampled(32, 4, idx, inp.weights[ss, tt], y)
    assert (got == ref.out[ss, tt]).all()


def test_random_shapes_against_brute_force_sort():
    """Many small random shapes (ranks, experts per rank, top-k, ragged token counts,
    alignment): slots and rows equal the brute-force stable sort."""
    rng = np.random.default_rng(123)
    for trial in range(60):
        N = int(rng.choice([1, 2, 3, 4, 5, 8]))
        El = int(rng.choice([1, 2, 3, 4, 8]))
        E = N * El
        K = int(rng.integers(1, min(E, 6) + 1))
        T = int(rng.integers(1, 24))
        align = int(rng.choice([1, 2, 5, 8]))
        inp = small_case(N, E, T, K, 8, seed=1000 + trial, ragged=bool(trial % 2))
        lay = orc.layout(N, E, K, inp.num_tokens, inp.indices, align)
        slot, rows = brute_force_layout(N, E, K, inp.num_tokens, inp.indices, align)
        assert (lay.slot == slot).all(), (trial, N, El, K, T, align)
        for d in range(N):
            got = orc.dispatch_rank(d, N, E, K, inp.num_tokens, inp.indices, inp.x, align, zero_pad=True)
            assert got.shape[0] == len(rows[d])
            for r, st in enumerate(rows[d]):
                assert (got[r] == (0 if st is None else inp.x[st[0], st[1]])).all()


# ----------------------------------------------------------------- chunked prefill (host side)
@pytest.mark.parametrize("chunk", [7, 32, 100, 250])
def test_token_chunks_partition_the_batch_and_keep_every_tokens_result(chunk):
    """workloads.token_chunk cuts tokens [t0, t0 + chunk) out of every rank, pads the last
    chunk with absent tokens, and the oracle run chunk by chunk gives every token the
    combined row of the one-shot run (a token's sum does not depend on its neighbours)."""
    wl = wlmod.custom("chunks", 4, 16, 100, 64, 3, seed=95, ragged=True)
    inp = wlmod.make_inputs(wl)
    whole = oracle_step(inp)
    seen = np.zeros((wl.n_ranks, wl.tokens), bool)
    for t0 in range(0, wl.tokens, chunk):
        piece = wlmod.token_chunk(inp, t0, chunk)
        n = min(chunk, wl.tokens - t0)
        assert piece.x.shape == (wl.n_ranks, chunk, wl.hidden) and piece.wl.tokens == chunk
        assert (piece.x[:, :n] == inp.x[:, t0:t0 + n]).all()
        assert (piece.indices[:, :n] == inp.indices[:, t0:t0 + n]).all()
        assert (piece.weights[:, :n] == inp.weights[:, t0:t0 + n]).all()
        assert (piece.num_tokens == np.clip(inp.num_tokens - t0, 0, n)).all()
        ref = oracle_step(piece)
        for s in range(wl.n_ranks):
            k = int(piece.num_tokens[s])
            assert (ref.out[s, :k] == whole.out[s, t0:t0 + k]).all()
            seen[s, t0:t0 + k] = True
    for s in range(wl.n_ranks):
        assert seen[s, :inp.num_tokens[s]].all() and not seen[s, inp.num_tokens[s]:].any()
