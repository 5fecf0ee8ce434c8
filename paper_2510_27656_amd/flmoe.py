"""ctypes binding of libflmoe.so (the C ABI declared in include/flmoe.h).

Argument marshalling only: every step of the shuffle runs in the library's HIP
kernels.  torch is used for device memory and for the current HIP stream.
There is no CPU fallback: if the shared library is missing, importing the
functions fails with an error that says how to build it.
"""
import ctypes as C
import os

import torch

from . import build as _build

FL_OK = 0
FL_ERR_INVALID_ARG, FL_ERR_ALIGNMENT, FL_ERR_WORKSPACE, FL_ERR_HIP = -1, -2, -3, -4
FL_ERR_STATIC_LIMIT = -5
FL_STATIC_SCRATCH_BYTES = 8 << 20
FL_STATUS_BAD_INDEX, FL_STATUS_CAPACITY, FL_STATUS_TIMEOUT = 1, 2, 4
FL_DTYPE_BF16, FL_DTYPE_E4M3_BLOCK128 = 0, 1
FL_FLAG_ZERO_PAD = 1
FL_FLAG_STREAM_ORDERED = 2
FL_FLAG_PEER_PUSH = 4
FL_FLAG_PARTIAL_SUMS = 8
FL_FLAG_PROGRESSIVE_RECV = 16
FL_KERNEL_COUNT = 14


class fl_moe_config(C.Structure):
    _fields_ = [("n_ranks", C.c_int32), ("n_experts", C.c_int32), ("max_tokens", C.c_int32),
                ("top_k", C.c_int32), ("hidden", C.c_int32), ("dispatch_dtype", C.c_int32),
                ("expert_align", C.c_int32), ("flags", C.c_int32),
                ("recv_capacity_rows", C.c_int64), ("expert_capacity_rows", C.c_int64),
                ("spin_limit", C.c_int64), ("max_private_rows", C.c_int32),
                ("reserved", C.c_int32)]


class fl_moe_sizes(C.Structure):
    _fields_ = [("workspace_bytes", C.c_size_t), ("recv_capacity_rows", C.c_int64),
                ("expert_capacity_rows", C.c_int64), ("send_capacity_rows", C.c_int64),
                ("x_row_bytes", C.c_int64), ("wire_row_bytes", C.c_int64),
                ("expert_x_row_bytes", C.c_int64), ("scales_per_row", C.c_int64),
                ("combine_row_bytes", C.c_int64), ("private_rows", C.c_int64),
                ("recv_buffer_rows", C.c_int64)]


class fl_moe_layout_view(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in
                ("counts", "dedup_counts", "tokens_per_expert", "send_off", "recv_off",
                 "expert_off", "comb_off", "comb_pos", "plan_ok")]


LAYOUT_OUT_FIELDS = ("counts", "dedup_counts", "tokens_per_expert", "send_off", "recv_off",
                     "expert_off", "comb_off", "comb_pos", "plan_ok", "status")


class fl_moe_layout_out(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in LAYOUT_OUT_FIELDS]


class fl_moe_debug_view(C.Structure):
    _fields_ = [("buf_a", C.c_void_p), ("buf_b", C.c_void_p),
                ("buf_a_rank_bytes", C.c_int64), ("buf_b_rank_bytes", C.c_int64),
                ("arrive_route", C.c_void_p), ("epoch_route", C.c_void_p),
                ("arrive_disp", C.c_void_p), ("arrive_comb", C.c_void_p),
                ("expect_disp", C.c_void_p), ("expect_comb", C.c_void_p), ("status", C.c_void_p)]


EXPORTS = ["fl_moe_query_sizes", "fl_moe_create", "fl_moe_destroy", "fl_moe_layout",
           "fl_moe_layout_static",
           "fl_moe_dispatch_send", "fl_moe_dispatch_send_weighted", "fl_moe_dispatch_send_e4m3",
           "fl_moe_dispatch_recv",
           "fl_moe_combine_send",
           "fl_moe_combine_reduce", "fl_moe_status", "fl_moe_reset", "fl_moe_required_capacities",
           "fl_moe_strerror", "fl_moe_debug_views",
           "fl_moe_debug_tune", "fl_moe_debug_launch_groups", "fl_moe_debug_copy", "fl_moe_debug_fill", "fl_moe_debug_read", "fl_moe_profile_enable", "fl_moe_profile_collect", "fl_moe_profile_read",
           "fl_moe_kernel_name", "fl_moe_build_id"]

_lib = None


def lib():
    """The loaded shared library.  Loads what is built; builds only if nothing is.  A
    library built from other sources than the ones beside it is refused: tests and
    benchmarks must never run an older binary than the code they claim to measure."""
    global _lib
    if _lib is None:
        path = _build.lib_path()
        if not os.path.exists(path):
            _build.build()
        L = C.CDLL(path)
        L.fl_moe_build_id.restype = C.c_char_p
        built_from, tree = L.fl_moe_build_id().decode(), _build.source_hash()
        if built_from != tree:
            raise RuntimeError(f"{path} was built from other sources (build id {built_from}, the tree has "
                               f"{tree}): rebuild it with `python -m paper_2510_27656_amd.build`")
        vp, i32, i64 = C.c_void_p, C.c_int, C.c_int64
        L.fl_moe_query_sizes.argtypes = [C.POINTER(fl_moe_config), C.POINTER(fl_moe_sizes)]
        L.fl_moe_create.argtypes = [C.POINTER(fl_moe_config), vp, C.c_size_t, C.POINTER(vp)]
        L.fl_moe_destroy.argtypes = [vp]
        L.fl_moe_layout.argtypes = [vp, i32, i32, vp, vp, C.POINTER(fl_moe_layout_view), vp]
        L.fl_moe_layout_static.argtypes = [C.POINTER(fl_moe_config), vp, vp,
                                           C.POINTER(fl_moe_layout_out), vp]
        L.fl_moe_dispatch_send.argtypes = [vp, i32, i32, vp, vp]
        L.fl_moe_dispatch_send_weighted.argtypes = [vp, i32, i32, vp, vp, vp]
        L.fl_moe_dispatch_send_e4m3.argtypes = [vp, i32, i32, vp, vp, vp, vp]
        L.fl_moe_dispatch_recv.argtypes = [vp, i32, i32, vp, vp, vp, vp]
        L.fl_moe_combine_send.argtypes = [vp, i32, i32, vp, vp]
        L.fl_moe_combine_reduce.argtypes = [vp, i32, i32, vp, vp, vp]
        L.fl_moe_status.argtypes = [vp, C.POINTER(C.c_int32), vp]
        L.fl_moe_reset.argtypes = [vp, vp]
        L.fl_moe_required_capacities.argtypes = [vp, C.POINTER(C.c_int64), C.POINTER(C.c_int64), vp]
        L.fl_moe_strerror.argtypes = [i32]
        L.fl_moe_strerror.restype = C.c_char_p
        L.fl_moe_debug_views.argtypes = [vp, C.POINTER(fl_moe_debug_view)]
        L.fl_moe_debug_tune.argtypes = [vp, i32, i32]
        L.fl_moe_debug_launch_groups.argtypes = [C.POINTER(fl_moe_config), i32, i32, C.POINTER(C.c_int)]
        L.fl_moe_debug_copy.argtypes = [vp, vp, C.c_size_t, vp]
        L.fl_moe_debug_fill.argtypes = [vp, C.c_size_t, vp]
        L.fl_moe_debug_read.argtypes = [vp, C.c_size_t, vp, vp]
        L.fl_moe_profile_enable.argtypes = [vp, i32]
        L.fl_moe_profile_collect.argtypes = [vp, vp]
        L.fl_moe_profile_read.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(i64)]
        L.fl_moe_kernel_name.argtypes = [i32]
        L.fl_moe_kernel_name.restype = C.c_char_p
        L.fl_moe_build_id.argtypes = []
        for name in EXPORTS:
            getattr(L, name)                    # every declared symbol must be exported
        _lib = L
    return _lib


class FlMoeError(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        super().__init__(f"{where}: {lib().fl_moe_strerror(code).decode()} ({code})")


def _check(code, where):
    if code != FL_OK:
        raise FlMoeError(code, where)


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def _ptr(t):
    if t is None:
        return C.c_void_p(0)
    assert t.is_cuda and t.is_contiguous()
    return C.c_void_p(t.data_ptr())


# ------------------------------------------------------------------ the C calls, same names
def fl_moe_query_sizes(cfg: fl_moe_config) -> fl_moe_sizes:
    out = fl_moe_sizes()
    _check(lib().fl_moe_query_sizes(C.byref(cfg), C.byref(out)), "fl_moe_query_sizes")
    return out


def fl_moe_create(cfg: fl_moe_config, workspace: torch.Tensor):
    ctx = C.c_void_p()
    _check(lib().fl_moe_create(C.byref(cfg), _ptr(workspace),
                               workspace.numel() * workspace.element_size(), C.byref(ctx)),
           "fl_moe_create")
    return ctx


def fl_moe_destroy(ctx):
    _check(lib().fl_moe_destroy(ctx), "fl_moe_destroy")


def fl_moe_layout(ctx, rank_begin, rank_count, indices, num_tokens, stream=None):
    view = fl_moe_layout_view()
    _check(lib().fl_moe_layout(ctx, rank_begin, rank_count, _ptr(indices), _ptr(num_tokens),
                               C.byref(view), _stream(stream)), "fl_moe_layout")
    return view


def fl_moe_layout_static(cfg: fl_moe_config, indices, num_tokens, out: dict, stream=None):
    """out: int32 device tensors by the field names of fl_moe_layout_out (caller-owned)."""
    o = fl_moe_layout_out(*[_ptr(out[n]) for n in LAYOUT_OUT_FIELDS])
    _check(lib().fl_moe_layout_static(C.byref(cfg), _ptr(indices), _ptr(num_tokens), C.byref(o),
                                      _stream(stream)), "fl_moe_layout_static")


def fl_moe_dispatch_send(ctx, rank_begin, rank_count, x, stream=None):
    _check(lib().fl_moe_dispatch_send(ctx, rank_begin, rank_count, _ptr(x), _stream(stream)),
           "fl_moe_dispatch_send")


def fl_moe_dispatch_send_e4m3(ctx, rank_begin, rank_count, codes, scales, weights=None, stream=None):
    _check(lib().fl_moe_dispatch_send_e4m3(ctx, rank_begin, rank_count, _ptr(codes), _ptr(scales),
                                           _ptr(weights) if weights is not None else None,
                                           _stream(stream)), "fl_moe_dispatch_send_e4m3")


def fl_moe_dispatch_send_weighted(ctx, rank_begin, rank_count, x, weights, stream=None):
    _check(lib().fl_moe_dispatch_send_weighted(ctx, rank_begin, rank_count, _ptr(x), _ptr(weights),
                                               _stream(stream)), "fl_moe_dispatch_send_weighted")


def fl_moe_dispatch_recv(ctx, rank_begin, rank_count, expert_x, expert_scales, tokens_per_expert,
                         stream=None):
    _check(lib().fl_moe_dispatch_recv(ctx, rank_begin, rank_count, _ptr(expert_x),
                                      _ptr(expert_scales), _ptr(tokens_per_expert),
                                      _stream(stream)), "fl_moe_dispatch_recv")


def fl_moe_combine_send(ctx, rank_begin, rank_count, expert_y, stream=None):
    _check(lib().fl_moe_combine_send(ctx, rank_begin, rank_count, _ptr(expert_y), _stream(stream)),
           "fl_moe_combine_send")


def fl_moe_combine_reduce(ctx, rank_begin, rank_count, weights, out, stream=None):
    _check(lib().fl_moe_combine_reduce(ctx, rank_begin, rank_count, _ptr(weights), _ptr(out),
                                       _stream(stream)), "fl_moe_combine_reduce")


def fl_moe_status(ctx, stream=None) -> int:
    v = C.c_int32(0)
    _check(lib().fl_moe_status(ctx, C.byref(v), _stream(stream)), "fl_moe_status")
    return v.value


def fl_moe_reset(ctx, stream=None):
    _check(lib().fl_moe_reset(ctx, _stream(stream)), "fl_moe_reset")


def fl_moe_required_capacities(ctx, stream=None):
    """(recv_capacity_rows, expert_capacity_rows) the last step needs."""
    recv, expert = C.c_int64(), C.c_int64()
    _check(lib().fl_moe_required_capacities(ctx, C.byref(recv), C.byref(expert), _stream(stream)),
           "fl_moe_required_capacities")
    return recv.value, expert.value


def fl_moe_debug_views(ctx) -> fl_moe_debug_view:
    out = fl_moe_debug_view()
    _check(lib().fl_moe_debug_views(ctx, C.byref(out)), "fl_moe_debug_views")
    return out


def fl_moe_debug_tune(ctx, knob, value):
    _check(lib().fl_moe_debug_tune(ctx, knob, value), "fl_moe_debug_tune")


def fl_moe_debug_launch_groups(cfg: fl_moe_config, rank_count: int, launch_mb: int = -1) -> int:
    out = C.c_int(0)
    _check(lib().fl_moe_debug_launch_groups(C.byref(cfg), rank_count, launch_mb, C.byref(out)),
           "fl_moe_debug_launch_groups")
    return out.value


def fl_moe_debug_copy(dst, src, nbytes, stream=None):
    _check(lib().fl_moe_debug_copy(_ptr(dst), _ptr(src), nbytes, _stream(stream)),
           "fl_moe_debug_copy")


def fl_moe_debug_fill(dst, nbytes, stream=None):
    _check(lib().fl_moe_debug_fill(_ptr(dst), nbytes, _stream(stream)), "fl_moe_debug_fill")


def fl_moe_debug_read(src, nbytes, sink, stream=None):
    _check(lib().fl_moe_debug_read(_ptr(src), nbytes, _ptr(sink), _stream(stream)), "fl_moe_debug_read")


def fl_moe_build_id() -> str:
    return lib().fl_moe_build_id().decode()


def fl_moe_profile_enable(ctx, on):
    _check(lib().fl_moe_profile_enable(ctx, int(on)), "fl_moe_profile_enable")


def fl_moe_profile_collect(ctx, stream=None):
    _check(lib().fl_moe_profile_collect(ctx, _stream(stream)), "fl_moe_profile_collect")


def fl_moe_profile_read(ctx):
    ms = (C.c_double * FL_KERNEL_COUNT)()
    n = (C.c_int64 * FL_KERNEL_COUNT)()
    _check(lib().fl_moe_profile_read(ctx, ms, n), "fl_moe_profile_read")
    return {lib().fl_moe_kernel_name(i).decode(): (ms[i], n[i]) for i in range(FL_KERNEL_COUNT)}


# ------------------------------------------------------------------ convenience wrapper
class MoEShuffle:
    """Owns the device memory of one context (workspace and outputs) and forwards
    to the C calls.  No arithmetic happens here."""

    def __init__(self, n_ranks, n_experts, max_tokens, top_k, hidden, dispatch_dtype="bf16",
                 expert_align=1, zero_pad=False, recv_capacity_rows=0, expert_capacity_rows=0,
                 spin_limit=0, stream_ordered=False, max_private_rows=0, peer_push=False,
                 partial_sums=False, progressive_recv=False, device="cuda:0"):
        self.device = torch.device(device)
        self.cfg = fl_moe_config(
            n_ranks, n_experts, max_tokens, top_k, hidden,
            FL_DTYPE_BF16 if dispatch_dtype == "bf16" else FL_DTYPE_E4M3_BLOCK128,
            expert_align, (FL_FLAG_ZERO_PAD if zero_pad else 0)
            | (FL_FLAG_STREAM_ORDERED if stream_ordered else 0)
            | (FL_FLAG_PEER_PUSH if peer_push else 0)
            | (FL_FLAG_PARTIAL_SUMS if partial_sums else 0)
            | (FL_FLAG_PROGRESSIVE_RECV if progressive_recv else 0),
            recv_capacity_rows, expert_capacity_rows, spin_limit, max_private_rows, 0)
        self.partial_sums = bool(partial_sums)
        self.sizes = fl_moe_query_sizes(self.cfg)
        self.N, self.E, self.T, self.K, self.H = n_ranks, n_experts, max_tokens, top_k, hidden
        self.El = n_experts // n_ranks
        self.workspace = torch.empty(self.sizes.workspace_bytes, dtype=torch.uint8,
                                     device=self.device)
        self.ctx = fl_moe_create(self.cfg, self.workspace)
        cap = self.sizes.expert_capacity_rows
        self.expert_capacity_rows = cap
        if dispatch_dtype == "bf16":
            self.expert_x = torch.empty((n_ranks, cap, hidden), dtype=torch.bfloat16,
                                        device=self.device)
            self.expert_scales = None
        else:
            self.expert_x = torch.empty((n_ranks, cap, hidden), dtype=torch.uint8,
                                        device=self.device)
            self.expert_scales = torch.empty((n_ranks, cap, hidden // 128), dtype=torch.float32,
                                             device=self.device)
        self.tokens_per_expert = torch.zeros((n_ranks, self.El), dtype=torch.int32,
                                             device=self.device)
        self.out = torch.empty((n_ranks, max_tokens, hidden), dtype=torch.bfloat16,
                               device=self.device)
        self.view = None

    def close(self):
        if self.ctx is not None:
            torch.cuda.synchronize(self.device)
            fl_moe_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _ranks(self, ranks):
        return (0, self.N) if ranks is None else ranks

    def layout(self, indices, num_tokens, ranks=None, stream=None):
        self._indices, self._num_tokens = indices, num_tokens      # keep alive for the step
        rb, rc = self._ranks(ranks)
        self.view = fl_moe_layout(self.ctx, rb, rc, indices, num_tokens, stream)
        return self.view

    def dispatch_send(self, x, ranks=None, stream=None, weights=None, scales=None):
        rb, rc = self._ranks(ranks)
        if scales is not None:          # x holds e4m3 codes the caller quantised itself
            fl_moe_dispatch_send_e4m3(self.ctx, rb, rc, x, scales, weights, stream)
        elif weights is None:
            fl_moe_dispatch_send(self.ctx, rb, rc, x, stream)
        else:
            fl_moe_dispatch_send_weighted(self.ctx, rb, rc, x, weights, stream)

    def dispatch_recv(self, ranks=None, stream=None):
        rb, rc = self._ranks(ranks)
        fl_moe_dispatch_recv(self.ctx, rb, rc, self.expert_x, self.expert_scales,
                             self.tokens_per_expert, stream)
        return self.expert_x

    def combine_send(self, expert_y, ranks=None, stream=None):
        rb, rc = self._ranks(ranks)
        fl_moe_combine_send(self.ctx, rb, rc, expert_y, stream)

    def combine_reduce(self, weights, ranks=None, stream=None, out=None):
        rb, rc = self._ranks(ranks)
        fl_moe_combine_reduce(self.ctx, rb, rc, weights, self.out if out is None else out, stream)
        return self.out if out is None else out

    def status(self):
        return fl_moe_status(self.ctx)

    def required_capacities(self):
        return fl_moe_required_capacities(self.ctx)

    def reset(self):
        fl_moe_reset(self.ctx)

    def table(self, ptr, shape, dtype=torch.int32):
        """A tensor view of a table inside the workspace (for parity checks)."""
        off = ptr - self.workspace.data_ptr()
        n = 1
        for s in shape:
            n *= s
        nbytes = n * torch.empty((), dtype=dtype).element_size()
        assert 0 <= off and off + nbytes <= self.workspace.numel()
        return self.workspace[off:off + nbytes].view(dtype).reshape(shape)

    def layout_tables(self):
        v, N, E, El, T, K = self.view, self.N, self.E, self.El, self.T, self.K
        return {
            "C": self.table(v.counts, (N, E)),
            "M": self.table(v.dedup_counts, (N, N)),
            "G": self.table(v.tokens_per_expert, (N, El)),
            "send_off": self.table(v.send_off, (N, N + 1)),
            "recv_off": self.table(v.recv_off, (N, N + 1)),
            "expert_off": self.table(v.expert_off, (N, El + 1)),
            "comb_off": self.table(v.comb_off, (N, N + 1)),
            "comb_pos": self.table(v.comb_pos, (N, T, K)),
            "plan_ok": self.table(v.plan_ok, (N,)),
        }

    def debug(self):
        dv = fl_moe_debug_views(self.ctx)
        N = self.N
        return {
            "arrive_route": self.table(dv.arrive_route, (N, N)),
            "arrive_disp": self.table(dv.arrive_disp, (N, N)),
            "arrive_comb": self.table(dv.arrive_comb, (N, N)),
            "epoch_route": self.table(dv.epoch_route, (N,)),
            "expect_disp": self.table(dv.expect_disp, (N, N)),
            "expect_comb": self.table(dv.expect_comb, (N, N)),
            "buf_a": self.table(dv.buf_a, (N, dv.buf_a_rank_bytes), torch.uint8),
            "buf_b": self.table(dv.buf_b, (N, dv.buf_b_rank_bytes), torch.uint8),
        }
