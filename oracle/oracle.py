"""numpy-facing wrapper around oracle/moe_oracle.c (ctypes, host memory only).

TEST INFRASTRUCTURE.  The product package never imports this module; tests, the
smoke check and the bench's cpu_baseline leg do.  Every function forwards to the
C routine of the same purpose; the arithmetic lives in the C file, which cites
the paper passage each routine follows.
"""
import ctypes as C
from dataclasses import dataclass

import numpy as np

from . import build as _build

_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(_build.build())
        _lib.orc_dispatch_rank.restype = C.c_int64
        _lib.orc_recv_order.restype = C.c_int64
        _lib.orc_e4m3_decode.restype = C.c_float
        _lib.orc_e4m3_decode.argtypes = [C.c_uint8]
        _lib.orc_e4m3_encode.restype = C.c_uint8
        _lib.orc_e4m3_encode.argtypes = [C.c_float]
        _lib.orc_bf16_to_f32.restype = C.c_float
        _lib.orc_bf16_to_f32.argtypes = [C.c_uint16]
        _lib.orc_f32_to_bf16.restype = C.c_uint16
        _lib.orc_f32_to_bf16.argtypes = [C.c_float]
    return _lib


def _p(a):
    return a.ctypes.data_as(C.c_void_p)


def _chk(a, dtype, shape=None):
    assert isinstance(a, np.ndarray) and a.dtype == dtype and a.flags.c_contiguous, (a.dtype, dtype)
    if shape is not None:
        assert tuple(a.shape) == tuple(shape), (a.shape, shape)
    return a


@dataclass
class Layout:
    """Counts and offsets of one step (sections Architecture and Dispatch)."""
    C: np.ndarray           # [N][E]   pairs per (source, expert)
    M: np.ndarray           # [N][N]   deduplicated tokens per (source, destination)
    G: np.ndarray           # [N][El]  tokens per local expert
    send_off: np.ndarray    # [N][N+1]
    recv_off: np.ndarray    # [N][N+1]
    expert_off: np.ndarray  # [N][El+1]
    comb_off: np.ndarray    # [N][N+1]
    slot: np.ndarray        # [N][T][K] row of pair (s,t,k) in its owner's expert-major layout


def layout(N, E, K, num_tokens, indices, align=1):
    Tmax = indices.shape[1]
    _chk(indices, np.int32, (N, Tmax, K))
    _chk(num_tokens, np.int32, (N,))
    El = E // N
    Cc = np.empty((N, E), np.int32)
    M = np.empty((N, N), np.int32)
    G = np.empty((N, El), np.int32)
    send_off = np.empty((N, N + 1), np.int32)
    recv_off = np.empty((N, N + 1), np.int32)
    expert_off = np.empty((N, El + 1), np.int32)
    comb_off = np.empty((N, N + 1), np.int32)
    slot = np.empty((N, Tmax, K), np.int32)
    L = lib()
    L.orc_counts(N, E, Tmax, K, _p(num_tokens), _p(indices), _p(Cc))
    L.orc_dedup_counts(N, E, Tmax, K, _p(num_tokens), _p(indices), _p(M))
    L.orc_offsets(N, E, align, _p(Cc), _p(M), _p(send_off), _p(recv_off), _p(G),
                  _p(expert_off), _p(comb_off))
    L.orc_slots(N, E, Tmax, K, align, _p(num_tokens), _p(indices), _p(slot))
    return Layout(Cc, M, G, send_off, recv_off, expert_off, comb_off, slot)


def dispatch_rank(d, N, E, K, num_tokens, indices, x, align=1, zero_pad=False,
                  out=None, fill=0):
    """Expert-major rows of rank d.  x: [N][T][...] any dtype; each token's record is
    copied whole.  Returns array [rows][...] (padding rows hold `fill` bytes unless
    zero_pad)."""
    Tmax = indices.shape[1]
    _chk(indices, np.int32, (N, Tmax, K))
    assert x.flags.c_contiguous and x.shape[0] == N and x.shape[1] == Tmax
    row_bytes = x.dtype.itemsize * int(np.prod(x.shape[2:], dtype=np.int64))
    lay = layout(N, E, K, num_tokens, indices, align)
    rows = int(lay.expert_off[d, -1])
    if out is None:
        out = np.empty((rows,) + x.shape[2:], x.dtype)
        out.view(np.uint8).fill(fill)
    got = lib().orc_dispatch_rank(d, N, E, Tmax, K, align, int(zero_pad), _p(num_tokens),
                                  _p(indices), _p(x), C.c_int64(row_bytes), _p(out))
    assert got == rows, (got, rows)
    return out


def combine(N, E, K, num_tokens, indices, slot, weights, Y, y_rank_stride_rows, H,
            return_acc=False):
    """Y: uint16 [N * y_rank_stride_rows][H] rank-major expert outputs.  Returns
    out uint16 [N][T][H] (rows of absent tokens are zero)."""
    Tmax = indices.shape[1]
    _chk(indices, np.int32, (N, Tmax, K))
    _chk(slot, np.int32, (N, Tmax, K))
    _chk(weights, np.float32, (N, Tmax, K))
    _chk(Y, np.uint16)
    out = np.zeros((N, Tmax, H), np.uint16)
    acc = np.zeros((N, Tmax, H), np.float32) if return_acc else None
    lib().orc_combine(N, E, Tmax, K, H, _p(num_tokens), _p(indices), _p(slot), _p(weights),
                      _p(Y), C.c_int64(y_rank_stride_rows * H), _p(out),
                      _p(acc) if return_acc else None)
    return (out, acc) if return_acc else out



def combine_partial(N, E, K, num_tokens, indices, slot, weights, Y, y_rank_stride_rows, H):
    """Combine with one bf16 partial sum per (token, expert rank); same arguments as combine."""
    Tmax = indices.shape[1]
    _chk(indices, np.int32, (N, Tmax, K))
    _chk(slot, np.int32, (N, Tmax, K))
    _chk(weights, np.float32, (N, Tmax, K))
    _chk(Y, np.uint16)
    out = np.zeros((N, Tmax, H), np.uint16)
    lib().orc_combine_partial(N, E, Tmax, K, H, _p(num_tokens), _p(indices), _p(slot), _p(weights),
                              _p(Y), C.c_int64(y_rank_stride_rows * H), _p(out))
    return out

def expert_scale_rank(d, N, E, lay, g, H, rows):
    _chk(rows, np.uint16)
    _chk(g, np.float32, (E,))
    lib().orc_expert_scale_rank(d, N, E, _p(lay.expert_off), _p(lay.G), _p(g), H, _p(rows))
    return rows


def recv_order(d, N, E, K, num_tokens, indices):
    Tmax = indices.shape[1]
    sr = np.empty(N * Tmax, np.int32)
    st = np.empty(N * Tmax, np.int32)
    mk = np.empty(N * Tmax, np.uint64)
    n = lib().orc_recv_order(d, N, E, Tmax, K, _p(num_tokens), _p(indices), _p(sr), _p(st), _p(mk))
    return sr[:n].copy(), st[:n].copy(), mk[:n].copy()


def comb_pos(N, E, K, num_tokens, indices):
    Tmax = indices.shape[1]
    out = np.empty((N, Tmax, K), np.int32)
    lib().orc_comb_pos(N, E, Tmax, K, _p(num_tokens), _p(indices), _p(out))
    return out


def quant_e4m3_block128(x):
    """x uint16 [..., H] bf16 bits -> (q uint8 [..., H], scales f32 [..., H/128])."""
    _chk(x, np.uint16)
    H = x.shape[-1]
    rows = x.size // H
    q = np.empty(x.shape, np.uint8)
    sc = np.empty(x.shape[:-1] + (H // 128,), np.float32)
    lib().orc_quant_e4m3_block128(C.c_int64(rows), H, _p(x), _p(q), _p(sc))
    return q, sc


def dequant_e4m3_block128(q, scales):
    _chk(q, np.uint8)
    _chk(scales, np.float32)
    H = q.shape[-1]
    rows = q.size // H
    y = np.empty(q.shape, np.uint16)
    lib().orc_dequant_e4m3_block128(C.c_int64(rows), H, _p(q), _p(scales), _p(y))
    return y


def e4m3_decode(code):
    return float(lib().orc_e4m3_decode(int(code)))


def e4m3_encode(f):
    return int(lib().orc_e4m3_encode(float(f)))


def bf16_to_f32(b):
    return float(lib().orc_bf16_to_f32(int(b)))


def f32_to_bf16(f):
    return int(lib().orc_f32_to_bf16(float(f)))


def e4m3_encode_array(a):
    _chk(a, np.float32)
    out = np.empty(a.shape, np.uint8)
    lib().orc_e4m3_encode_array(C.c_int64(a.size), _p(a), _p(out))
    return out


def e4m3_decode_array(a):
    _chk(a, np.uint8)
    out = np.empty(a.shape, np.float32)
    lib().orc_e4m3_decode_array(C.c_int64(a.size), _p(a), _p(out))
    return out


def f32_to_bf16_array(a):
    _chk(a, np.float32)
    out = np.empty(a.shape, np.uint16)
    lib().orc_f32_to_bf16_array(C.c_int64(a.size), _p(a), _p(out))
    return out


def scale_rows(rows, gains):
    """rows uint16 [n][H] (modified in place): row r *= gains[r], rounded to bf16."""
    _chk(rows, np.uint16)
    _chk(gains, np.float32, (rows.shape[0],))
    lib().orc_scale_rows(C.c_int64(rows.shape[0]), rows.shape[1], _p(gains), _p(rows))
    return rows


def combine_sampled(E, K, indices, weights, y_rows):
    """Combine for an explicit list of n tokens: indices/weights [n][K], y_rows uint16
    [n*K][H] holds the expert output of pair (i, k) at row i*K + k.  Returns [n][H]."""
    n = indices.shape[0]
    H = y_rows.shape[1]
    idx = np.ascontiguousarray(indices.reshape(1, n, K), np.int32)
    w = np.ascontiguousarray(weights.reshape(1, n, K), np.float32)
    slot = np.arange(n * K, dtype=np.int32).reshape(1, n, K)
    nt = np.array([n], np.int32)
    return combine(1, E, K, nt, idx, slot, w, y_rows, 0, H)[0]
