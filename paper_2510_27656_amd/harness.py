"""Driver around the five C calls for tests, smoke and bench: uploads a drawn
workload, runs one step, applies the stand-in expert between dispatch and
combine.  The stand-in expert (a per-expert gain) is harness work done with
torch ops on the GPU; it is not part of the shuffle."""
import numpy as np
import torch

from . import flmoe
from .workloads import Inputs


def to_device(inp: Inputs, device="cuda:0"):
    x = torch.from_numpy(inp.x.view(np.int16)).to(device).view(torch.bfloat16)
    return {
        "x": x,
        "indices": torch.from_numpy(inp.indices).to(device),
        "weights": torch.from_numpy(inp.weights).to(device),
        "num_tokens": torch.from_numpy(inp.num_tokens).to(device),
        "gain": torch.from_numpy(inp.expert_gain).to(device),
    }


def make_shuffle(inp: Inputs, expert_align=1, zero_pad=False, capacity_factor=None,
                 spin_limit=0, stream_ordered=False, max_private_rows=0, peer_push=False,
                 partial_sums=False, progressive_recv=False, capacities=None, device="cuda:0"):
    """capacity_factor None = worst-case capacities, else factor x the mean rows per rank;
    capacities = (recv_capacity_rows, expert_capacity_rows) given outright."""
    wl = inp.wl
    recv_cap = expert_cap = 0
    if capacities is not None:
        recv_cap, expert_cap = capacities
    elif capacity_factor is not None:
        mean_rows = wl.tokens * wl.top_k
        expert_cap = int(mean_rows * capacity_factor) + (wl.experts_per_rank - 1) * (expert_align - 1)
        recv_cap = int(min(mean_rows, wl.n_ranks * wl.tokens) * capacity_factor)
    return flmoe.MoEShuffle(wl.n_ranks, wl.n_experts, wl.tokens, wl.top_k, wl.hidden,
                            dispatch_dtype=wl.dispatch_dtype, expert_align=expert_align,
                            zero_pad=zero_pad, recv_capacity_rows=recv_cap,
                            expert_capacity_rows=expert_cap, spin_limit=spin_limit,
                            stream_ordered=stream_ordered,
                            max_private_rows=max_private_rows, peer_push=peer_push,
                            partial_sums=partial_sums, progressive_recv=progressive_recv, device=device)


def row_gain(sh: flmoe.MoEShuffle, gain: torch.Tensor):
    """Per-row gain [N][cap] of the stand-in expert, from the library's own offsets."""
    tabs = sh.layout_tables()
    off = tabs["expert_off"].long()                       # [N][El+1]
    rows = torch.arange(sh.expert_capacity_rows, device=gain.device)
    j = (torch.searchsorted(off[:, 1:-1].contiguous(), rows.expand(sh.N, -1).contiguous(),
                            right=True))                   # local expert of each row
    e = j + (torch.arange(sh.N, device=gain.device) * sh.El)[:, None]
    return gain[e]


def expert_stage(sh: flmoe.MoEShuffle, gain: torch.Tensor, identity=False):
    """y = bf16(float(x) * gain[e]) on every row; in place on a copy of expert_x."""
    if identity and sh.expert_scales is None:
        return sh.expert_x
    g = row_gain(sh, gain)
    if sh.expert_scales is None:
        if sh.expert_x.numel() < (1 << 31):
            return (sh.expert_x.float() * g[..., None]).to(torch.bfloat16)
        y = torch.empty_like(sh.expert_x)                 # rank by rank to bound the temporaries
        for d in range(sh.N):
            y[d] = (sh.expert_x[d].float() * g[d][:, None]).to(torch.bfloat16)
        return y
    # e4m3 payload: dequantise first, y = bf16(bf16(float(q) * scale) * gain); rank by rank
    # to bound the temporaries; codes are decoded through a 256-entry table
    lut = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).float().to(gain.device)
    y = torch.empty(sh.expert_x.shape, dtype=torch.bfloat16, device=gain.device)
    for d in range(sh.N):
        q = lut[sh.expert_x[d].long()]
        sc = sh.expert_scales[d].repeat_interleave(128, dim=-1)
        xf = (q * sc).to(torch.bfloat16).float()
        y[d] = xf.to(torch.bfloat16) if identity else (xf * g[d][:, None]).to(torch.bfloat16)
    return y


def send_weights(sh: flmoe.MoEShuffle, dev):
    """The routing weights travel with the tokens only in partial-sum mode."""
    return dev["weights"] if sh.partial_sums else None


def run_step(sh: flmoe.MoEShuffle, dev, identity=False, ranks=None):
    sh.layout(dev["indices"], dev["num_tokens"], ranks)
    sh.dispatch_send(dev["x"], ranks, weights=send_weights(sh, dev))
    sh.dispatch_recv(ranks)
    y = expert_stage(sh, dev["gain"], identity)
    sh.combine_send(y, ranks)
    return sh.combine_reduce(dev["weights"], ranks)


def run_hot_path(sh: flmoe.MoEShuffle, dev, expert_y=None, ready=None):
    """The five calls back to back.  bf16 dispatch: identity expert, expert_y aliases
    expert_x.  e4m3 dispatch: the caller passes a resident bf16 expert_y of the layout's
    shape (the stand-in expert is not part of the timed path).  ready: e4m3 codes and
    scales already on the device, dispatched as they are."""
    sh.layout(dev["indices"], dev["num_tokens"])
    if ready is None:
        sh.dispatch_send(dev["x"], weights=send_weights(sh, dev))
    else:                                # (codes, scales) the caller quantised itself
        sh.dispatch_send(ready[0], scales=ready[1], weights=send_weights(sh, dev))
    sh.dispatch_recv()
    sh.combine_send(sh.expert_x if expert_y is None else expert_y)
    return sh.combine_reduce(dev["weights"])


def run_step_two_streams(sh: flmoe.MoEShuffle, dev, identity=False, send_order=None, expert_y=None,
                         streams=None):
    """One step with senders and receivers on different streams (not for a context created
    with stream_ordered=True).  Receive calls are enqueued on stream A right after the
    layout, send calls on stream B: the receivers' gate kernels (or, with
    progressive_recv, the receive kernels themselves) poll the arrival counters while
    the fabric copy is still running or has not started.  Events order only what the
    re-use of the two staging buffers needs.  send_order: list of (rank_begin,
    rank_count) launches for the send calls, default one launch for all ranks."""
    N = sh.N
    a, b = streams or (torch.cuda.Stream(), torch.cuda.Stream())
    cur = torch.cuda.current_stream()
    a.wait_stream(cur)
    b.wait_stream(cur)
    order = send_order or [(0, N)]
    with torch.cuda.stream(a):
        sh.layout(dev["indices"], dev["num_tokens"])
        planned = torch.cuda.Event()
        planned.record(a)
    with torch.cuda.stream(b):
        b.wait_event(planned)
        for rg in order:
            sh.dispatch_send(dev["x"], rg, weights=send_weights(sh, dev))
    with torch.cuda.stream(a):
        sh.dispatch_recv()                       # polls per source while stream B delivers
        y = expert_y if expert_y is not None else expert_stage(sh, dev["gain"], identity)
        unpacked = torch.cuda.Event()
        unpacked.record(a)
    with torch.cuda.stream(b):
        b.wait_event(unpacked)                   # the receive buffer becomes the combine send buffer
        for rg in reversed(order):
            sh.combine_send(y, rg)
    with torch.cuda.stream(a):
        out = sh.combine_reduce(dev["weights"])  # polls while the replies are still arriving
    cur.wait_stream(a)
    cur.wait_stream(b)
    return out


def run_chunked(sh: flmoe.MoEShuffle, chunks, out_full: torch.Tensor, identity=False, with_expert=True):
    """Chunked prefill: one context sized for `sh.T` tokens per rank is stepped over a
    list of (first token, uploaded chunk) pairs, so that the staging buffers hold one
    chunk instead of the whole batch (section Performance, prefill: transfers are not
    chunked there, and buffer memory limits which models can be deployed).  Every
    token's combined row lands in out_full [N][T_total][H]."""
    for t0, dev in chunks:
        n = min(sh.T, out_full.shape[1] - t0)
        sh.layout(dev["indices"], dev["num_tokens"])
        sh.dispatch_send(dev["x"], weights=send_weights(sh, dev))
        sh.dispatch_recv()
        y = expert_stage(sh, dev["gain"], identity) if with_expert else sh.expert_x
        sh.combine_send(y)
        out = sh.combine_reduce(dev["weights"])
        out_full[:, t0:t0 + n].copy_(out[:, :n])
    return out_full
