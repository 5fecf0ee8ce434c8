"""One full step through the CPU oracle (test infrastructure)."""
from dataclasses import dataclass

import numpy as np

from . import oracle as orc


@dataclass
class OracleStep:
    lay: orc.Layout
    comb_pos: np.ndarray
    expert_rows: list          # per rank: [rows][H] dispatched payload (uint16 bf16 bits, or uint8 e4m3)
    expert_scales: list        # per rank: [rows][H/128] float32 (e4m3 dispatch only, else None)
    expert_y: np.ndarray       # [N][stride][H] uint16 (after the stand-in expert)
    stride: int
    out: np.ndarray            # [N][T][H] uint16
    out_partial: np.ndarray = None   # same, combine with sender-side partial sums (on request)


def oracle_step(inp, align=1, zero_pad=True, partial=False) -> OracleStep:
    wl = inp.wl
    N, E, K, H = wl.n_ranks, wl.n_experts, wl.top_k, wl.hidden
    nt = inp.num_tokens
    lay = orc.layout(N, E, K, nt, inp.indices, align)
    stride = max(int(lay.expert_off[:, -1].max()), 1)
    rows, scales = [], []
    Y = np.zeros((N, stride, H), np.uint16)
    fp8 = wl.dispatch_dtype == "e4m3"
    if fp8:       # the sender quantises each token once; the quantised record is what travels
        q, sc = orc.quant_e4m3_block128(inp.x)
    for d in range(N):
        if fp8:
            rq = orc.dispatch_rank(d, N, E, K, nt, inp.indices, q, align, zero_pad=zero_pad)
            rs = orc.dispatch_rank(d, N, E, K, nt, inp.indices, sc, align, zero_pad=zero_pad)
            rows.append(rq)
            scales.append(rs)
            # stand-in expert input: bf16(float(q) * scale)
            Y[d, :rq.shape[0]] = orc.dequant_e4m3_block128(rq, rs)
        else:
            r = orc.dispatch_rank(d, N, E, K, nt, inp.indices, inp.x, align, zero_pad=zero_pad)
            rows.append(r)
            scales.append(None)
            Y[d, :r.shape[0]] = r
        if wl.expert != "identity":
            orc.expert_scale_rank(d, N, E, lay, inp.expert_gain, H, Y[d])
    out = orc.combine(N, E, K, nt, inp.indices, lay.slot, inp.weights, Y, stride, H)
    outp = None
    if partial:
        outp = orc.combine_partial(N, E, K, nt, inp.indices, lay.slot, inp.weights, Y, stride, H)
    return OracleStep(lay, orc.comb_pos(N, E, K, nt, inp.indices), rows, scales, Y, stride, out, outp)
