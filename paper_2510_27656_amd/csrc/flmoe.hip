// Host side of the flmoe C ABI: argument checks, workspace partition, launches.
// Every shuffle call only enqueues kernels on the caller's stream.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <type_traits>

#include "../../include/flmoe.h"
#include "common.h"
#include "kernels_layout.h"
#include "kernels_shuffle.h"

using namespace flmoe;

// Scratch of fl_moe_layout_static, part of the device image: every GPU the library
// is loaded on holds its own copy at its own address.  In host code this name is
// only a handle for hipGetSymbolAddress, never a device address.
static __device__ __align__(256) unsigned char scratch[FL_STATIC_SCRATCH_BYTES];

namespace {

enum KernelId {
    KID_ROUTE_LAYOUT = 0, KID_DISPATCH_PACK, KID_DISPATCH_FABRIC,
    KID_DISPATCH_UNPACK, KID_COMBINE_PACK, KID_COMBINE_FABRIC, KID_COMBINE_REDUCE,
    KID_DISPATCH_PACK_E4M3, KID_DISPATCH_FABRIC_PRIVATE, KID_COMBINE_PARTIAL_PACK, KID_GATE_DISPATCH,
    KID_GATE_COMBINE, KID_ANNOUNCE_DISPATCH, KID_ANNOUNCE_COMBINE
};
const char *kKernelNames[FL_KERNEL_COUNT] = {
    "route_layout_kernel", "dispatch_pack_kernel", "fabric_copy_kernel(dispatch)",
    "dispatch_unpack_kernel", "combine_pack_kernel", "fabric_copy_kernel(combine)",
    "combine_reduce_kernel", "dispatch_pack_e4m3_kernel", "fabric_copy_kernel(dispatch, private slots)",
    "combine_partial_pack_kernel", "arrival_gate_kernel(dispatch)", "arrival_gate_kernel(combine)",
    "announce_kernel(dispatch)", "announce_kernel(combine)"};

constexpr int kEventPool = 512;
constexpr long long kMaxFabricBlocks = 1 << 16;   // waves loop cheaply (no barriers)
constexpr long long kMaxRowBlocks = 1 << 18;      // blocks with barriers: loop only when far oversized
constexpr long long kDefaultSpin = 1 << 20;       // polls about 2 us apart: gives up after about 2 s

constexpr size_t kBigPage = 2u << 20;
constexpr int kLaunchMiB = 860;
size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Walks the workspace; with base == nullptr it only measures.
struct Carver {
    char *base; size_t cur = 0;
    explicit Carver(void *b) : base((char *)b) {}
    template <class T> T *take(size_t count) {
        cur = align_up(cur, 256);
        T *p = base ? (T *)(base + cur) : nullptr;
        cur += count * sizeof(T);
        return p;
    }
};

int resolve(const fl_moe_config *c, Dims *D) {
    if (!c) return FL_ERR_INVALID_ARG;
    if (c->n_ranks < 1 || c->n_ranks > FL_MAX_RANKS) return FL_ERR_INVALID_ARG;
    if (c->n_experts < c->n_ranks || c->n_experts > FL_MAX_EXPERTS ||
        c->n_experts % c->n_ranks != 0) return FL_ERR_INVALID_ARG;
    const int El = c->n_experts / c->n_ranks;
    if (El > FL_MAX_EXPERTS_PER_RANK) return FL_ERR_INVALID_ARG;
    if (c->top_k < 1 || c->top_k > FL_MAX_TOPK || c->top_k > c->n_experts) return FL_ERR_INVALID_ARG;
    if (c->max_tokens < 1 || c->max_tokens >= (1 << 24)) return FL_ERR_INVALID_ARG;
    if (c->hidden < 8 || c->hidden > (1 << 20)) return FL_ERR_INVALID_ARG;
    if ((c->hidden * 2) % 16 != 0) return FL_ERR_ALIGNMENT;
    if (c->dispatch_dtype != FL_DTYPE_BF16 && c->dispatch_dtype != FL_DTYPE_E4M3_BLOCK128)
        return FL_ERR_INVALID_ARG;
    if (c->dispatch_dtype == FL_DTYPE_E4M3_BLOCK128 && c->hidden % 128 != 0) return FL_ERR_ALIGNMENT;
    if (c->expert_align < 1 || c->expert_align > (1 << 16)) return FL_ERR_INVALID_ARG;
    if (c->flags & ~(FL_FLAG_ZERO_PAD | FL_FLAG_STREAM_ORDERED | FL_FLAG_PEER_PUSH | FL_FLAG_PARTIAL_SUMS |
                     FL_FLAG_PROGRESSIVE_RECV))
        return FL_ERR_INVALID_ARG;
    if ((c->flags & FL_FLAG_PROGRESSIVE_RECV) && (c->flags & FL_FLAG_STREAM_ORDERED)) return FL_ERR_INVALID_ARG;
    if (c->recv_capacity_rows < 0 || c->expert_capacity_rows < 0 || c->spin_limit < 0)
        return FL_ERR_INVALID_ARG;
    if (c->max_private_rows < 0 || c->reserved != 0) return FL_ERR_INVALID_ARG;

    D->N = c->n_ranks; D->E = c->n_experts; D->El = El; D->T = c->max_tokens; D->K = c->top_k;
    D->H = c->hidden; D->dtype = c->dispatch_dtype; D->align = c->expert_align; D->flags = c->flags;
    D->route_len = D->E + 2 * D->N + 1;
    D->KM = (D->K + 3) / 4 * 4;
    D->MW = (c->flags & FL_FLAG_PARTIAL_SUMS) ? 2 * D->KM : D->KM;
    const long long NT = (long long)D->N * D->T;
    const long long minKEl = D->K < El ? D->K : El;
    const long long worst_recv = NT;
    const long long worst_expert = NT * minKEl + (long long)(El - 1) * (D->align - 1);
    D->recv_cap = c->recv_capacity_rows ? c->recv_capacity_rows : worst_recv;
    D->expert_cap = c->expert_capacity_rows ? c->expert_capacity_rows : worst_expert;
    if (D->recv_cap > worst_recv) D->recv_cap = worst_recv;
    if (D->expert_cap > worst_expert) D->expert_cap = worst_expert;
    D->P = c->max_private_rows < D->T ? c->max_private_rows : D->T;   // a source sends at most T rows
    D->recv_rows = (long long)D->N * D->P + D->recv_cap;
    if (D->recv_rows >= (1ll << 31) || D->expert_cap >= (1ll << 31)) return FL_ERR_INVALID_ARG;
    D->send_cap = (long long)D->T * (D->K < D->N ? D->K : D->N);
    D->Bx = 2ll * D->H;
    D->Bc = 2ll * D->H;
    if (D->dtype == FL_DTYPE_BF16) {
        D->Bw = D->Bx; D->Be = D->Bx; D->scales_per_row = 0;
    } else {
        D->scales_per_row = D->H / 128;
        D->Be = D->H;
        // wire rows start on 128-byte lines: measured 5-10 % faster pack and unpack than 16-byte packing
        D->Bw = (long long)align_up((size_t)(D->H + 4ll * D->scales_per_row), 128);
    }
    const long long a1 = D->send_cap * D->Bw, a2 = (long long)D->T * D->K * D->Bc;
    const long long b1 = D->recv_rows * D->Bw, b2 = D->expert_cap * D->Bc;
    // Large payload buffers start on 2 MB boundaries of the workspace, rank by rank (the
    // page size the driver maps big allocations with): measured 3 % faster unpack at the
    // decode shape than 256-byte packing.  Small ones stay packed.
    const size_t need_a = (size_t)(a1 > a2 ? a1 : a2), need_b = (size_t)(b1 > b2 ? b1 : b2);
    D->bufA_rank_bytes = (long long)align_up(need_a, need_a >= kBigPage ? kBigPage : 256);
    D->bufB_rank_bytes = (long long)align_up(need_b, need_b >= kBigPage ? kBigPage : 256);
    // arrival counters count 16-byte units in 32 bits with a wrap-safe comparison
    if ((long long)D->T * (D->Bc / 16) >= (1ll << 31)) return FL_ERR_INVALID_ARG;
    D->spin_limit = c->spin_limit ? c->spin_limit : kDefaultSpin;
    // Largest LDS tile of the counting kernel that stays under 60 KB.
    int tt = 32;
    while (tt < 1024 && route_count_lds_bytes(D->E, D->N, tt * 2) <= 60 * 1024) tt *= 2;
    const int need = (D->T + 31) / 32 * 32;
    D->TT = need < tt ? need : tt;
    D->tune_rows = 0;
    D->tune_reduce = 0;
    D->tune_waves = 0;
    D->tune_slices = 0;
    D->tune_stream_mb = 2560;
    D->tune_grid_pct = 200;
    D->tune_cap8 = 3;
    D->tune_order = 0;
    D->tune_parts = 0;
    {   // a token reaches a given rank with probability 1 - (1 - 1/N)^K when experts are drawn uniformly
        double miss = 1.0;
        for (int k = 0; k < D->K; ++k) miss *= 1.0 - 1.0 / D->N;
        D->typ_recv_rows = (long long)(NT * (1.0 - miss)) + 1;
        D->typ_pair_rows = (long long)D->T * D->K;
    }
    return FL_OK;
}

// Returns the number of bytes of the small-table prefix (cleared at create).
size_t carve(const Dims &D, void *base, Tables *W, size_t *total) {
    Carver c(base);
    const size_t N = D.N, E = D.E, El = D.El, T = D.T, K = D.K;
    W->status = c.take<int>(64);
    W->epoch_route = c.take<unsigned>(N);
    W->arrive_route = c.take<unsigned>(N * N);
    W->arrive_disp = c.take<unsigned>(N * N);
    W->arrive_comb = c.take<unsigned>(N * N);
    W->expect_disp = c.take<unsigned>(N * N);
    W->expect_comb = c.take<unsigned>(N * N);
    W->plan_ok = c.take<int>(N);
    W->gate_disp = c.take<int>(N);
    W->gate_comb = c.take<int>(N);
    W->routes = c.take<int>(N * N * D.route_len);
    W->C = c.take<int>(N * E);
    W->M = c.take<int>(N * N);
    W->send_off = c.take<int>(N * (N + 1));
    W->comb_off = c.take<int>(N * (N + 1));
    W->G = c.take<int>(N * El);
    W->expert_off = c.take<int>(N * (El + 1));
    W->recv_off = c.take<int>(N * (N + 1));
    W->recv_shared_off = c.take<int>(N * N);
    W->dst_off = c.take<int>(N * N);
    W->comb_dst_off = c.take<int>(N * N);
    W->ret_off = c.take<int>(N * N);
    W->base_x = c.take<int>(N * El * N);
    W->cs_base = c.take<int>(N * N * El);
    W->cs_off = c.take<int>(N * (N + 1));
    const size_t small = align_up(c.cur, 256);
    W->send_row = c.take<int>(N * T * K);
    W->pair_meta = c.take<unsigned>(N * T * K);
    W->comb_pos = c.take<int>(N * T * K);
    W->send_meta = c.take<unsigned>(N * (size_t)D.send_cap * D.MW);
    W->recv_meta = c.take<unsigned>(N * (size_t)D.recv_rows * D.MW);
    W->fab_dst_disp = c.take<int2>(N * (size_t)D.send_cap);
    W->fab_dst_comb = c.take<int2>(N * (size_t)D.expert_cap);
    if ((size_t)D.bufA_rank_bytes >= kBigPage) c.cur = align_up(c.cur, kBigPage);
    W->bufA = c.take<char>(N * (size_t)D.bufA_rank_bytes);
    if ((size_t)D.bufB_rank_bytes >= kBigPage) c.cur = align_up(c.cur, kBigPage);
    W->bufB = c.take<char>(N * (size_t)D.bufB_rank_bytes);
    *total = align_up(c.cur, 256);
    return small;
}

bool aligned16(const void *p) { return ((uintptr_t)p & 15) == 0; }

// Waves that share one row in the fabric kernel: enough that a lane has at most
// a handful of 16-byte vectors.
int waves_per_row(long long row_bytes, int tune_waves) {
    if (tune_waves >= 1 && tune_waves <= 16) return tune_waves;
    // about 4 KB per wave: one counter update per wave, and those updates serialise in L2
    const long long w = (row_bytes + 4095) / 4096;
    return (int)(w < 1 ? 1 : w > 4 ? 4 : w);
}

// Blocks that share one token in the pack kernel (each takes a slice of the row).
int pack_slices(long long row_bytes, int tune_slices) {
    if (tune_slices > 0) return tune_slices;
    const long long nvec = row_bytes / 16;
    // measured: rows up to 8 KB are fastest with two vectors per thread (4 KB rows: one block,
    // 30 -> 25 us; 7 KB rows of e4m3 codes: two blocks, 61 -> 54 us), longer rows with one
    if (nvec <= 4 * kPackThreads) return (int)((nvec + 2 * kPackThreads - 1) / (2 * kPackThreads));
    long long s = (nvec + kPackThreads - 1) / kPackThreads;   // one vector per thread
    return (int)(s < 1 ? 1 : s > 16 ? 16 : s);
}

// Grids are sized from capacities (the rows really in use are only known on the
// device), so a generous capacity would launch mostly idle blocks; beyond this
// many blocks per launch the kernels loop instead.
unsigned capped_grid(long long blocks_needed, int rank_count, long long max_blocks,
                     int multiple_of = 1) {
    long long limit = max_blocks / rank_count;
    if (limit < 1) limit = 1;
    long long g = blocks_needed < limit ? blocks_needed : limit;
    g = (g + multiple_of - 1) / multiple_of * multiple_of;
    return (unsigned)(g < 1 ? 1 : g);
}

// Rows a row-kernel's grid is sized for: the capacity, or (tune_grid_pct) a percentage of
// what uniform routing would bring; the kernels loop when a rank holds more.
long long grid_rows(const Dims &D, long long capacity, long long typical) {
    if (D.tune_grid_pct <= 0) return capacity;
    const long long want = typical * D.tune_grid_pct / 100 + 1;
    return want < capacity ? want : capacity;
}

int rows_per_block(long long row_bytes, int tune_rows) {
    long long rb = tune_rows > 0 ? tune_rows : 16384 / row_bytes;
    if (rb < 1) rb = 1;
    if (rb > kMaxRowsPerBlock) rb = kMaxRowsPerBlock;
    return (int)rb;
}

}  // namespace

struct fl_moe_ctx {
    fl_moe_config cfg;
    Dims D;
    Tables W;
    size_t workspace_bytes;
    const int32_t *indices = nullptr;
    const int32_t *num_tokens = nullptr;
    int cu_count = 256;
    int launch_mb = kLaunchMiB;   // payload a launch should move per direction, see ranks_per_launch
    // profiling
    int profile = 0;
    hipEvent_t ev_start[kEventPool], ev_stop[kEventPool];
    int ev_kernel[kEventPool];
    int ev_used = 0;
    double total_ms[FL_KERNEL_COUNT];
    int64_t launches[FL_KERNEL_COUNT];
};

namespace {

struct LaunchTimer {
    fl_moe_ctx *ctx; hipStream_t st; int slot = -1;
    LaunchTimer(fl_moe_ctx *c, int kid, hipStream_t s) : ctx(c), st(s) {
        if (c->profile && c->ev_used < kEventPool) {
            slot = c->ev_used++;
            c->ev_kernel[slot] = kid;
            (void)hipEventRecord(c->ev_start[slot], st);
        }
    }
    ~LaunchTimer() { if (slot >= 0) (void)hipEventRecord(ctx->ev_stop[slot], st); }
};

int check_ranks(const fl_moe_ctx *ctx, int rb, int rc) {
    if (!ctx) return FL_ERR_INVALID_ARG;
    if (rb < 0 || rc < 1 || rb + rc > ctx->D.N) return FL_ERR_INVALID_ARG;
    return FL_OK;
}

int launch_status() { return hipGetLastError() == hipSuccess ? FL_OK : FL_ERR_HIP; }

// Ranks one launch of a payload kernel serves.  A launch that walks many GB runs
// measurably slower than the same work cut into launches of somewhat under a GB
// (a plain copy: 6.1 TB/s in 1 GiB launches, 5.7 TB/s as one 12 GiB launch; the
// 4096-token step: 8 % faster in 2-rank launches), while cutting a launch that is
// small already only adds launch tails.  So a call whose ranks move more than three
// times the target is cut into rank groups of about the target size.  Not in
// progressive mode: its receive kernels run on capped grids and its copies write
// through, and there the cut measured 3 % slower.
int ranks_per_launch(const Dims &D, int launch_mb, int rc) {
    if (launch_mb <= 0 || (D.flags & FL_FLAG_PROGRESSIVE_RECV)) return rc;
    const long long row = D.Bw > D.Bc ? D.Bw : D.Bc;
    const long long per_rank = (long long)D.T * D.K * row;
    const long long target = (long long)launch_mb << 20;
    if (per_rank * rc <= 3 * target) return rc;
    long long launches = (per_rank * rc + target - 1) / target;
    if (launches > rc) launches = rc;
    return (int)((rc + launches - 1) / launches);
}

// The whole rank range of a call, and where in it the current launch group sits: the
// gate kernel of a receive call runs once, before the first group, for all its ranks,
// and the announce kernel of a send call once, behind the last group (a receiver needs
// every sender's rows anyway, so announcing group by group would let nobody start earlier).
struct CallSpan {
    int rank_begin, rank_count;
    bool first, last;
};

// Runs f(rank_begin, rank_count, span) over the rank groups of one call.
template <class F>
int for_rank_groups(const fl_moe_ctx *ctx, int rb, int rc, F f) {
    int e = check_ranks(ctx, rb, rc);
    if (e != FL_OK) return e;
    const int g = ranks_per_launch(ctx->D, ctx->launch_mb, rc);
    for (int r = rb; r < rb + rc; r += g) {
        const int n = rb + rc - r < g ? rb + rc - r : g;
        e = f(r, n, CallSpan{rb, rc, r == rb, r + n == rb + rc});
        if (e != FL_OK) return e;
    }
    return FL_OK;
}

// ---------------------------------------------------------------- static scratch
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void *g_scratch_ptr[kMaxDevices];          // device address of `scratch` on each GPU, looked up once

// Address of the current device's copy of `scratch`.
int static_scratch(void **ptr) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return FL_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return FL_ERR_HIP;
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return FL_OK;
}

// What route_layout_kernel keeps outside the caller-visible tables, carved from
// `base` (nullptr: measure only).  The counters come first, in one run of
// *clear_words 32-bit words at `base` that every call clears.  Returns the bytes needed.
size_t carve_static(const Dims &D, void *base, Tables *W, size_t *clear_words) {
    Carver c(base);
    const size_t N = D.N, El = D.El, T = D.T, K = D.K;
    W->epoch_route = c.take<unsigned>(N);
    W->arrive_route = c.take<unsigned>(N * N);
    W->expect_disp = c.take<unsigned>(N * N);
    W->expect_comb = c.take<unsigned>(N * N);
    *clear_words = align_up(c.cur, 256) / sizeof(unsigned);
    W->routes = c.take<int>(N * N * D.route_len);
    W->recv_shared_off = c.take<int>(N * N);
    W->dst_off = c.take<int>(N * N);
    W->comb_dst_off = c.take<int>(N * N);
    W->ret_off = c.take<int>(N * N);
    W->base_x = c.take<int>(N * El * N);
    W->cs_base = c.take<int>(N * N * El);
    W->cs_off = c.take<int>(N * (N + 1));
    W->send_row = c.take<int>(N * T * K);
    W->pair_meta = c.take<unsigned>(N * T * K);
    return align_up(c.cur, 256);
}

// Zeroes the counters of the static scratch and the caller's status word (a kernel,
// not a memset node: the call may be captured in a HIP graph).
__global__ void clear_words_kernel(unsigned *words, size_t n, int *status) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) words[i] = 0u;
    if (i == 0) *status = 0;
}

}  // namespace

extern "C" {

int fl_moe_query_sizes(const fl_moe_config *cfg, fl_moe_sizes *out) {
    if (!out) return FL_ERR_INVALID_ARG;
    Dims D;
    int rc = resolve(cfg, &D);
    if (rc != FL_OK) return rc;
    Tables W;
    size_t total;
    carve(D, nullptr, &W, &total);
    out->workspace_bytes = total;
    out->recv_capacity_rows = D.recv_cap;
    out->expert_capacity_rows = D.expert_cap;
    out->send_capacity_rows = D.send_cap;
    out->x_row_bytes = D.Bx;
    out->wire_row_bytes = D.Bw;
    out->expert_x_row_bytes = D.Be;
    out->scales_per_row = D.scales_per_row;
    out->combine_row_bytes = D.Bc;
    out->private_rows = D.P;
    out->recv_buffer_rows = D.recv_rows;
    return FL_OK;
}

int fl_moe_create(const fl_moe_config *cfg, void *workspace, size_t workspace_bytes,
                  fl_moe_ctx **out) {
    if (!out || !workspace) return FL_ERR_INVALID_ARG;
    if (((uintptr_t)workspace & 255) != 0) return FL_ERR_ALIGNMENT;
    Dims D;
    int rc = resolve(cfg, &D);
    if (rc != FL_OK) return rc;
    Tables W;
    size_t total;
    carve(D, nullptr, &W, &total);
    if (workspace_bytes < total) return FL_ERR_WORKSPACE;
    fl_moe_ctx *ctx = new (std::nothrow) fl_moe_ctx();
    if (!ctx) return FL_ERR_INVALID_ARG;
    ctx->cfg = *cfg;
    ctx->D = D;
    const size_t small = carve(D, workspace, &ctx->W, &total);
    ctx->workspace_bytes = total;
    if (hipMemset(workspace, 0, small) != hipSuccess || hipDeviceSynchronize() != hipSuccess) {
        delete ctx;
        return FL_ERR_HIP;
    }
    {
        int dev = 0, cus = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess &&
            cus > 0)
            ctx->cu_count = cus;
    }
    for (int i = 0; i < kEventPool; ++i) {      // created when profiling is first enabled
        ctx->ev_start[i] = nullptr;
        ctx->ev_stop[i] = nullptr;
    }
    memset(ctx->total_ms, 0, sizeof(ctx->total_ms));
    memset(ctx->launches, 0, sizeof(ctx->launches));
    *out = ctx;
    return FL_OK;
}

int fl_moe_destroy(fl_moe_ctx *ctx) {
    if (!ctx) return FL_ERR_INVALID_ARG;
    for (int i = 0; i < kEventPool; ++i) {
        if (ctx->ev_start[i]) (void)hipEventDestroy(ctx->ev_start[i]);
        if (ctx->ev_stop[i]) (void)hipEventDestroy(ctx->ev_stop[i]);
    }
    delete ctx;
    return FL_OK;
}

int fl_moe_layout(fl_moe_ctx *ctx, int rb, int rc, const int32_t *indices,
                  const int32_t *num_tokens, fl_moe_layout_view *view, void *stream) {
    int e = check_ranks(ctx, rb, rc);
    if (e != FL_OK) return e;
    if (!indices || !num_tokens) return FL_ERR_INVALID_ARG;
    if (((uintptr_t)indices & 3) || ((uintptr_t)num_tokens & 3)) return FL_ERR_ALIGNMENT;
    hipStream_t st = (hipStream_t)stream;
    const Dims &D = ctx->D;
    ctx->indices = indices;
    ctx->num_tokens = num_tokens;
    {
        LaunchTimer t(ctx, KID_ROUTE_LAYOUT, st);
        const size_t lds_count = route_count_lds_bytes(D.E, D.N, D.TT);
        const size_t lds_plan = route_plan_lds_bytes(D.E, D.N, D.El);
        route_layout_kernel<<<dim3(2 * rc), dim3(kRouteThreads), lds_count > lds_plan ? lds_count : lds_plan, st>>>(
            D, ctx->W, rb, rc, indices, num_tokens);
    }
    if (view) {
        const Tables &W = ctx->W;
        view->counts = W.C; view->dedup_counts = W.M; view->tokens_per_expert = W.G;
        view->send_off = W.send_off; view->recv_off = W.recv_off; view->expert_off = W.expert_off;
        view->comb_off = W.comb_off; view->comb_pos = W.comb_pos; view->plan_ok = W.plan_ok;
    }
    return launch_status();
}

int fl_moe_layout_static(const fl_moe_config *cfg, const int32_t *indices, const int32_t *num_tokens,
                         const fl_moe_layout_out *out, void *stream) {
    if (!cfg || !indices || !num_tokens || !out) return FL_ERR_INVALID_ARG;
    int32_t *const outs[] = {out->counts, out->dedup_counts, out->tokens_per_expert, out->send_off,
                             out->recv_off, out->expert_off, out->comb_off, out->comb_pos,
                             out->plan_ok, out->status};
    for (int32_t *p : outs) {
        if (!p) return FL_ERR_INVALID_ARG;
        if ((uintptr_t)p & 3) return FL_ERR_ALIGNMENT;
    }
    if (((uintptr_t)indices & 3) || ((uintptr_t)num_tokens & 3)) return FL_ERR_ALIGNMENT;
    Dims D;
    int e = resolve(cfg, &D);
    if (e != FL_OK) return e;
    Tables W;
    memset(&W, 0, sizeof(W));
    size_t clear_words = 0;
    if (carve_static(D, nullptr, &W, &clear_words) > FL_STATIC_SCRATCH_BYTES) return FL_ERR_STATIC_LIMIT;
    void *ptr = nullptr;
    e = static_scratch(&ptr);
    if (e != FL_OK) return e;
    carve_static(D, ptr, &W, &clear_words);
    W.C = out->counts; W.M = out->dedup_counts; W.G = out->tokens_per_expert;
    W.send_off = out->send_off; W.recv_off = out->recv_off; W.expert_off = out->expert_off;
    W.comb_off = out->comb_off; W.comb_pos = out->comb_pos; W.plan_ok = out->plan_ok;
    W.status = out->status;
    hipStream_t st = (hipStream_t)stream;
    // The array keeps what the last call left (possibly of another shape): the message
    // counters and epochs must start at zero, everything else is written before it is read.
    clear_words_kernel<<<dim3((unsigned)((clear_words + 255) / 256)), dim3(256), 0, st>>>(
        (unsigned *)ptr, clear_words, W.status);
    const size_t lds_count = route_count_lds_bytes(D.E, D.N, D.TT);
    const size_t lds_plan = route_plan_lds_bytes(D.E, D.N, D.El);
    route_layout_kernel<<<dim3(2 * D.N), dim3(kRouteThreads), lds_count > lds_plan ? lds_count : lds_plan, st>>>(
        D, W, 0, D.N, indices, num_tokens);
    return launch_status();
}

static int dispatch_send_range(fl_moe_ctx *ctx, int rb, int rc, CallSpan call, const void *x, const float *weights,
                               const float *ready_scales, bool streaming, void *stream) {
    int e = check_ranks(ctx, rb, rc);
    if (e != FL_OK) return e;
    if (!x || !ctx->indices) return FL_ERR_INVALID_ARG;
    // the weights travel with the tokens exactly when the expert ranks need them
    if (((ctx->D.flags & FL_FLAG_PARTIAL_SUMS) != 0) != (weights != nullptr)) return FL_ERR_INVALID_ARG;
    if (!aligned16(x) || ((uintptr_t)weights & 3) || ((uintptr_t)ready_scales & 3)) return FL_ERR_ALIGNMENT;
    if (ready_scales && ctx->D.dtype != FL_DTYPE_E4M3_BLOCK128) return FL_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    const Dims &D = ctx->D;
    const Tables &W = ctx->W;
    // fenced: every wave reports what it delivered (progressive receivers); in_kernel: the last
    // payload kernel of the call also advances the counters (stream-ordered callers); otherwise
    // a kernel of its own does, behind the payload kernels in this (the sender's) stream
    const bool push = D.flags & FL_FLAG_PEER_PUSH, fenced = D.flags & FL_FLAG_PROGRESSIVE_RECV;
    const bool in_kernel = D.flags & FL_FLAG_STREAM_ORDERED;
    if (D.dtype == FL_DTYPE_E4M3_BLOCK128 && !ready_scales) {
        LaunchTimer t(ctx, KID_DISPATCH_PACK_E4M3, st);
        const char *xp = (const char *)x;
        auto go = [&](auto threads) {
            constexpr int QT = decltype(threads)::value;
            const int per_block = QT / kQuantLanes;              // quantisation blocks per workgroup
            const int slices = (D.scales_per_row + per_block - 1) / per_block;
            const dim3 grid((unsigned)D.T * slices, rc), block(QT);
            if (push && fenced)
                dispatch_pack_e4m3_kernel<true, true, QT><<<grid, block, 0, st>>>(D, W, rb, xp, ctx->indices,
                                                                                  ctx->num_tokens, slices, weights);
            else if (push)
                dispatch_pack_e4m3_kernel<true, false, QT><<<grid, block, 0, st>>>(D, W, rb, xp, ctx->indices,
                                                                                   ctx->num_tokens, slices, weights);
            else
                dispatch_pack_e4m3_kernel<false, false, QT><<<grid, block, 0, st>>>(D, W, rb, xp, ctx->indices,
                                                                                    ctx->num_tokens, slices, weights);
        };
        if (D.scales_per_row > 256 / kQuantLanes) go(std::integral_constant<int, 512>{});
        else go(std::integral_constant<int, 256>{});
    } else {
        LaunchTimer t(ctx, KID_DISPATCH_PACK, st);
        // bf16 rows, or e4m3 codes the caller quantised itself (their scales go along)
        const long long src_row = ready_scales ? D.Be : D.Bx;
        const int slices = pack_slices(src_row, D.tune_slices);
        const dim3 grid((unsigned)D.T * slices, rc), block(kPackThreads);
        const char *xp = (const char *)x;
        if (push && fenced)
            dispatch_pack_kernel<true, true><<<grid, block, 0, st>>>(D, W, rb, xp, ctx->indices,
                                                                     ctx->num_tokens, slices, weights, src_row, ready_scales);
        else if (push)
            dispatch_pack_kernel<true, false><<<grid, block, 0, st>>>(D, W, rb, xp, ctx->indices,
                                                                      ctx->num_tokens, slices, weights, src_row, ready_scales);
        else
            dispatch_pack_kernel<false, false><<<grid, block, 0, st>>>(D, W, rb, xp, ctx->indices,
                                                                       ctx->num_tokens, slices, weights, src_row, ready_scales);
    }
    auto announce = [&]() {                   // counter-ordered mode: the transfers are announced once
        if (fenced || in_kernel || !call.last) return;   // every payload kernel of the call has ended
        LaunchTimer t(ctx, KID_ANNOUNCE_DISPATCH, st);
        announce_kernel<<<dim3(call.rank_count), dim3(kWave), 0, st>>>(D, W, call.rank_begin, W.send_off,
                                                                        W.arrive_disp, (unsigned)(D.Bw / 16));
    };
    if (push) {                               // the rows are already in the peers' receive buffers
        announce();
        return launch_status();
    }
    FabricArgs A;
    A.src_base = W.bufA; A.src_rank_stride = D.bufA_rank_bytes;
    A.dst_base = W.bufB; A.dst_rank_stride = D.bufB_rank_bytes;
    A.seg_off = W.send_off; A.row_dst = W.fab_dst_disp; A.row_cap = D.send_cap;
    A.src_meta = W.send_meta; A.src_meta_rank_stride = D.send_cap * D.MW;
    A.dst_meta = W.recv_meta; A.dst_meta_rank_stride = D.recv_rows * D.MW;
    A.dst_row_lo = 0;
    A.announce = 0;
    A.order = D.tune_order;
    A.arrive = W.arrive_disp;
    A.row_bytes = D.Bw; A.waves_per_row = waves_per_row(D.Bw, D.tune_waves);
    const int wpb = kCopyThreads / kWave;
    // a multiple of waves_per_row blocks keeps every row's waves at a fixed stride
    const unsigned gx = capped_grid((D.send_cap * A.waves_per_row + wpb - 1) / wpb, rc, kMaxFabricBlocks,
                                     A.waves_per_row);
    if (D.P > 0) {
        // First scatter: the rows bound for private slots.  Their targets follow from the
        // sender's own counts alone, so this launch reads nothing a peer produced.
        A.announce = D.P >= D.T ? (in_kernel ? 1 : fenced ? 2 : 0) : 0;   // the call's last copy kernel announces
        LaunchTimer t(ctx, KID_DISPATCH_FABRIC_PRIVATE, st);
        const unsigned g1 = capped_grid(((long long)D.N * D.P * A.waves_per_row + wpb - 1) / wpb, rc,
                                        kMaxFabricBlocks, A.waves_per_row);
        if (fenced)
            fabric_private_kernel<true, true><<<dim3(g1, rc), dim3(kCopyThreads), 0, st>>>(D, W, A, rb);
        else if (streaming)
            fabric_private_kernel<false, true><<<dim3(g1, rc), dim3(kCopyThreads), 0, st>>>(D, W, A, rb);
        else
            fabric_private_kernel<false, false><<<dim3(g1, rc), dim3(kCopyThreads), 0, st>>>(D, W, A, rb);
        A.dst_row_lo = D.N * D.P;             // second scatter: the rest, into the shared range
    }
    if (D.P < D.T) {                          // with P = T every row has a private slot
        A.announce = in_kernel ? 1 : fenced ? 2 : 0;
        LaunchTimer t(ctx, KID_DISPATCH_FABRIC, st);
        if (fenced)
            fabric_copy_kernel<true, 0, true><<<dim3(gx, rc), dim3(kCopyThreads), 0, st>>>(D, W, A, rb);
        else if (streaming)
            fabric_copy_kernel<false, 0, true><<<dim3(gx, rc), dim3(kCopyThreads), 0, st>>>(D, W, A, rb);
        else
            fabric_copy_kernel<false, 0, false><<<dim3(gx, rc), dim3(kCopyThreads), 0, st>>>(D, W, A, rb);
    }
    announce();
    return launch_status();
}

static int dispatch_send_impl(fl_moe_ctx *ctx, int rb, int rc, const void *x, const float *weights,
                              const float *ready_scales, void *stream) {
    if (!ctx) return FL_ERR_INVALID_ARG;
    // cached or streaming stores in the scatter: decided by what the whole call writes
    const bool streaming = (long long)rc * ctx->D.send_cap * ctx->D.Bw > ((long long)ctx->D.tune_stream_mb << 20);
    return for_rank_groups(ctx, rb, rc, [&](int r, int n, CallSpan call) {
        return dispatch_send_range(ctx, r, n, call, x, weights, ready_scales, streaming, stream);
    });
}

int fl_moe_dispatch_send(fl_moe_ctx *ctx, int rb, int rc, const void *x, void *stream) {
    return dispatch_send_impl(ctx, rb, rc, x, nullptr, nullptr, stream);
}

int fl_moe_dispatch_send_weighted(fl_moe_ctx *ctx, int rb, int rc, const void *x, const float *weights,
                                  void *stream) {
    if (!weights) return FL_ERR_INVALID_ARG;
    return dispatch_send_impl(ctx, rb, rc, x, weights, nullptr, stream);
}

int fl_moe_dispatch_send_e4m3(fl_moe_ctx *ctx, int rb, int rc, const void *codes, const float *scales,
                              const float *weights, void *stream) {
    if (!scales) return FL_ERR_INVALID_ARG;
    return dispatch_send_impl(ctx, rb, rc, codes, weights, scales, stream);
}

static int dispatch_recv_range(fl_moe_ctx *ctx, int rb, int rc, CallSpan call, void *expert_x, float *expert_scales,
                               int32_t *tokens_per_expert, void *stream) {
    int e = check_ranks(ctx, rb, rc);
    if (e != FL_OK) return e;
    const Dims &D = ctx->D;
    if (!expert_x || !tokens_per_expert) return FL_ERR_INVALID_ARG;
    if ((D.scales_per_row != 0) != (expert_scales != nullptr)) return FL_ERR_INVALID_ARG;
    if (!aligned16(expert_x) || !aligned16(expert_scales) || ((uintptr_t)tokens_per_expert & 3))
        return FL_ERR_ALIGNMENT;
    hipStream_t st = (hipStream_t)stream;
    const bool gated = !(D.flags & FL_FLAG_STREAM_ORDERED);
    const bool progressive = D.flags & FL_FLAG_PROGRESSIVE_RECV;
    // Default: a gate kernel of one wave per rank polls the rank's arrival counters, and the
    // unpack kernel runs behind it in the stream on a full grid.  Stream-ordered callers need
    // no gate.  Progressive: the unpack kernel polls itself and starts on each
    // source's rows as they land; it may be running while senders still need somewhere to
    // run, so it takes at most three eighths of the resident-block slots (measured best), and
    // to keep the memory system busy with that few waves a block moves 32 KB per turn.
    int rbk = rows_per_block(D.Bw, D.tune_rows);
    if (progressive && D.tune_rows == 0) {
        long long r = (32768 + D.Bw - 1) / D.Bw;
        rbk = (int)(r > kMaxRowsPerBlock ? kMaxRowsPerBlock : r);
    }
    const long long worst_rows = (long long)D.N * D.T;       // received rows in use never exceed this
    const long long max_rows = D.recv_rows < worst_rows ? D.recv_rows : worst_rows;
    unsigned gx = capped_grid((grid_rows(D, max_rows, D.typ_recv_rows) + rbk - 1) / rbk, rc,
                              progressive ? (long long)ctx->cu_count * D.tune_cap8 : kMaxRowBlocks);
    if (gx < (unsigned)D.El) gx = D.El;      // the first El-1 blocks also clear padding rows
    const int *gate = nullptr;
    if (gated && !progressive) {
        if (call.first) {
            LaunchTimer t(ctx, KID_GATE_DISPATCH, st);
            arrival_gate_kernel<<<dim3(call.rank_count), dim3(kWave), 0, st>>>(
                D, ctx->W, call.rank_begin, ctx->W.arrive_disp, ctx->W.expect_disp, ctx->W.gate_disp);
        }
        gate = ctx->W.gate_disp;
    }
    {
        LaunchTimer t(ctx, KID_DISPATCH_UNPACK, st);
        const dim3 grid(gx, rc), block(kCopyThreads);
        char *ex = (char *)expert_x;
        if (progressive && D.P)
            dispatch_unpack_kernel<true, true><<<grid, block, 0, st>>>(D, ctx->W, rb, ex, expert_scales,
                                                                       tokens_per_expert, rbk, gate);
        else if (progressive)
            dispatch_unpack_kernel<true, false><<<grid, block, 0, st>>>(D, ctx->W, rb, ex, expert_scales,
                                                                        tokens_per_expert, rbk, gate);
        else if (D.P)
            dispatch_unpack_kernel<false, true><<<grid, block, 0, st>>>(D, ctx->W, rb, ex, expert_scales,
                                                                        tokens_per_expert, rbk, gate);
        else
            dispatch_unpack_kernel<false, false><<<grid, block, 0, st>>>(D, ctx->W, rb, ex, expert_scales,
                                                                         tokens_per_expert, rbk, gate);
    }
    return launch_status();
}

int fl_moe_dispatch_recv(fl_moe_ctx *ctx, int rb, int rc, void *expert_x, float *expert_scales,
                         int32_t *tokens_per_expert, void *stream) {
    return for_rank_groups(ctx, rb, rc, [&](int r, int n, CallSpan call) {
        return dispatch_recv_range(ctx, r, n, call, expert_x, expert_scales, tokens_per_expert, stream);
    });
}

static int combine_send_range(fl_moe_ctx *ctx, int rb, int rc, CallSpan call, const void *expert_y, void *stream) {
    int e = check_ranks(ctx, rb, rc);
    if (e != FL_OK) return e;
    if (!expert_y) return FL_ERR_INVALID_ARG;
    if (!aligned16(expert_y)) return FL_ERR_ALIGNMENT;
    hipStream_t st = (hipStream_t)stream;
    const Dims &D = ctx->D;
    const Tables &W = ctx->W;
    const int rbk = rows_per_block(D.Bc, D.tune_rows);
    const bool push = D.flags & FL_FLAG_PEER_PUSH, fenced = D.flags & FL_FLAG_PROGRESSIVE_RECV;
    const bool in_kernel = D.flags & FL_FLAG_STREAM_ORDERED;     // as in dispatch_send_range
    const bool partial = D.flags & FL_FLAG_PARTIAL_SUMS;
    // rows a rank sends back: one per pair, or with partial sums one per received row
    const long long worst_recv = (long long)D.N * D.T;
    const long long reply_rows = partial ? (D.recv_rows < worst_recv ? D.recv_rows : worst_recv)
                                         : D.expert_cap;
    const long long reply_grid = grid_rows(D, reply_rows, partial ? D.typ_recv_rows : D.typ_pair_rows);
    const unsigned gx = capped_grid((reply_grid + rbk - 1) / rbk, rc, kMaxRowBlocks);
    {
        const dim3 grid(gx, rc), block(kCopyThreads);
        const char *yp = (const char *)expert_y;
        if (partial) {
            LaunchTimer t(ctx, KID_COMBINE_PARTIAL_PACK, st);
            if (push && fenced) combine_partial_pack_kernel<true, true><<<grid, block, 0, st>>>(D, W, rb, yp, rbk);
            else if (push) combine_partial_pack_kernel<true, false><<<grid, block, 0, st>>>(D, W, rb, yp, rbk);
            else combine_partial_pack_kernel<false, false><<<grid, block, 0, st>>>(D, W, rb, yp, rbk);
        } else {
            LaunchTimer t(ctx, KID_COMBINE_PACK, st);
            if (push && fenced) combine_pack_kernel<true, true><<<grid, block, 0, st>>>(D, W, rb, yp, rbk);
            else if (push) combine_pack_kernel<true, false><<<grid, block, 0, st>>>(D, W, rb, yp, rbk);
            else combine_pack_kernel<false, false><<<grid, block, 0, st>>>(D, W, rb, yp, rbk);
        }
    }
    auto announce = [&]() {
        if (fenced || in_kernel || !call.last) return;
        LaunchTimer t(ctx, KID_ANNOUNCE_COMBINE, st);
        announce_kernel<<<dim3(call.rank_count), dim3(kWave), 0, st>>>(
            D, W, call.rank_begin, partial ? W.recv_off : W.cs_off, W.arrive_comb, (unsigned)(D.Bc / 16));
    };
    if (push) {                               // the rows are already in the sources' receive buffers
        announce();
        return launch_status();
    }
    FabricArgs A;
    A.src_base = W.bufB; A.src_rank_stride = D.bufB_rank_bytes;
    A.dst_base = W.bufA; A.dst_rank_stride = D.bufA_rank_bytes;
    A.seg_off = partial ? W.recv_off : W.cs_off; A.row_dst = W.fab_dst_comb; A.row_cap = D.expert_cap;
    A.src_meta = nullptr; A.src_meta_rank_stride = 0;
    A.dst_meta = nullptr; A.dst_meta_rank_stride = 0;
    A.dst_row_lo = 0;
    A.announce = in_kernel ? 1 : fenced ? 2 : 0;
    A.order = D.tune_order;
    A.arrive = W.arrive_comb;
    A.row_bytes = D.Bc; A.waves_per_row = waves_per_row(D.Bc, D.tune_waves);
    const int wpb = kCopyThreads / kWave;
    const unsigned gxf = capped_grid((reply_grid * A.waves_per_row + wpb - 1) / wpb, rc,
                                      kMaxFabricBlocks, A.waves_per_row);
    {
        LaunchTimer t(ctx, KID_COMBINE_FABRIC, st);
        // what the launch can write: every rank gets back at most T*K rows
        const bool streaming = (long long)D.N * D.T * D.K * D.Bc > ((long long)D.tune_stream_mb << 20);
        if (fenced)
            fabric_copy_kernel<true, 1, true><<<dim3(gxf, rc), dim3(kCopyThreads), 0, st>>>(D, W, A, rb);
        else if (streaming)
            fabric_copy_kernel<false, 1, true><<<dim3(gxf, rc), dim3(kCopyThreads), 0, st>>>(D, W, A, rb);
        else
            fabric_copy_kernel<false, 1, false><<<dim3(gxf, rc), dim3(kCopyThreads), 0, st>>>(D, W, A, rb);
    }
    announce();
    return launch_status();
}

int fl_moe_combine_send(fl_moe_ctx *ctx, int rb, int rc, const void *expert_y, void *stream) {
    return for_rank_groups(ctx, rb, rc, [&](int r, int n, CallSpan call) {
        return combine_send_range(ctx, r, n, call, expert_y, stream);
    });
}

static int combine_reduce_range(fl_moe_ctx *ctx, int rb, int rc, CallSpan call, const float *weights, void *out,
                                void *stream) {
    int e = check_ranks(ctx, rb, rc);
    if (e != FL_OK) return e;
    if (!weights || !out || !ctx->indices) return FL_ERR_INVALID_ARG;
    if (!aligned16(out) || ((uintptr_t)weights & 3)) return FL_ERR_ALIGNMENT;
    hipStream_t st = (hipStream_t)stream;
    const Dims &D = ctx->D;
    const bool gated = !(D.flags & FL_FLAG_STREAM_ORDERED), partial = D.flags & FL_FLAG_PARTIAL_SUMS;
    const bool progressive = D.flags & FL_FLAG_PROGRESSIVE_RECV;
    const int *gate = nullptr;
    if (gated && !progressive) {         // as in dispatch_recv: a gate kernel, then the full grid
        if (call.first) {
            LaunchTimer t(ctx, KID_GATE_COMBINE, st);
            arrival_gate_kernel<<<dim3(call.rank_count), dim3(kWave), 0, st>>>(
                D, ctx->W, call.rank_begin, ctx->W.arrive_comb, ctx->W.expect_comb, ctx->W.gate_comb);
        }
        gate = ctx->W.gate_comb;
    }
    {
        LaunchTimer t(ctx, KID_COMBINE_REDUCE, st);
        // `parts` workgroups share a token, each taking a slice of the row
        const int nvec = (int)(D.Bc / 16);
        // measured: long rows are summed fastest by many small workgroups, one payload wave each
        // (7168-wide rows: 14 workgroups of 2 waves 86 us, 2 of 7 waves 90 us, 1 of 14 waves 92 us);
        // rows of 4 KB and less gain nothing; capped polling grids keep one workgroup per token
        int parts = D.tune_parts > 0 ? D.tune_parts : (nvec >= 512 && !progressive ? (nvec + kWave - 1) / kWave : 1);
        if (parts > nvec) parts = nvec;
        const int per = (nvec + parts - 1) / parts;
        int nt = (per + kWave - 1) / kWave * kWave;
        if (nt > kReduceMaxThreads) nt = kReduceMaxThreads;
        if (nt < 2 * kWave) nt = 2 * kWave;      // wave 0 waits, wave 1 fetches positions and weights
        // progressive (polling) receivers take at most three eighths of the machine's wave slots
        const unsigned gx = progressive ? capped_grid(D.T, rc, (long long)ctx->cu_count * 256 * D.tune_cap8 / nt / parts)
                                        : (unsigned)D.T;
        const dim3 grid(gx * parts, rc);
        char *o = (char *)out;
        if (progressive && partial)
            combine_reduce_kernel<true, true><<<grid, dim3(nt), 0, st>>>(D, ctx->W, rb, weights, o, ctx->num_tokens, gate, parts);
        else if (progressive)
            combine_reduce_kernel<true, false><<<grid, dim3(nt), 0, st>>>(D, ctx->W, rb, weights, o, ctx->num_tokens, gate, parts);
        else if (partial)
            combine_reduce_kernel<false, true><<<grid, dim3(nt), 0, st>>>(D, ctx->W, rb, weights, o, ctx->num_tokens, gate, parts);
        else
            combine_reduce_kernel<false, false><<<grid, dim3(nt), 0, st>>>(D, ctx->W, rb, weights, o, ctx->num_tokens, gate, parts);
    }
    return launch_status();
}

int fl_moe_combine_reduce(fl_moe_ctx *ctx, int rb, int rc, const float *weights, void *out,
                          void *stream) {
    return for_rank_groups(ctx, rb, rc, [&](int r, int n, CallSpan call) {
        return combine_reduce_range(ctx, r, n, call, weights, out, stream);
    });
}

int fl_moe_status(fl_moe_ctx *ctx, int32_t *host_out, void *stream) {
    if (!ctx || !host_out) return FL_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    if (hipMemcpyAsync(host_out, ctx->W.status, sizeof(int32_t), hipMemcpyDeviceToHost, st) !=
        hipSuccess) return FL_ERR_HIP;
    if (hipStreamSynchronize(st) != hipSuccess) return FL_ERR_HIP;
    if (*host_out != 0) {
        if (hipMemsetAsync(ctx->W.status, 0, sizeof(int32_t), st) != hipSuccess) return FL_ERR_HIP;
        if (hipStreamSynchronize(st) != hipSuccess) return FL_ERR_HIP;
    }
    return FL_OK;
}

int fl_moe_reset(fl_moe_ctx *ctx, void *stream) {
    if (!ctx) return FL_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    // status word and every counter: the contiguous head of the workspace up to plan_ok
    const size_t bytes = (size_t)((char *)ctx->W.plan_ok - (char *)ctx->W.status);
    if (hipMemsetAsync(ctx->W.status, 0, bytes, st) != hipSuccess) return FL_ERR_HIP;
    if (hipStreamSynchronize(st) != hipSuccess) return FL_ERR_HIP;
    return FL_OK;
}

int fl_moe_required_capacities(fl_moe_ctx *ctx, int64_t *recv_capacity_rows, int64_t *expert_capacity_rows,
                               void *stream) {
    if (!ctx || !recv_capacity_rows || !expert_capacity_rows) return FL_ERR_INVALID_ARG;
    const Dims &D = ctx->D;
    const size_t nC = (size_t)D.N * D.E, nM = (size_t)D.N * D.N;
    int *host = new (std::nothrow) int[nC + nM];
    if (!host) return FL_ERR_HIP;
    int *C = host, *M = host + nC;          // the sources' own tables: valid whether or not the plan was
    hipError_t e = hipStreamSynchronize((hipStream_t)stream);
    if (e == hipSuccess) e = hipMemcpy(C, ctx->W.C, nC * sizeof(int), hipMemcpyDeviceToHost);
    if (e == hipSuccess) e = hipMemcpy(M, ctx->W.M, nM * sizeof(int), hipMemcpyDeviceToHost);
    if (e != hipSuccess) { delete[] host; return FL_ERR_HIP; }
    long long need_recv = 1, need_expert = 1;   // 0 would read as "worst case" in a configuration
    for (int d = 0; d < D.N; ++d) {
        long long recv = 0, rows = 0;
        for (int s = 0; s < D.N; ++s) recv += std::max(M[(size_t)s * D.N + d] - D.P, 0);
        for (int j = 0; j < D.El; ++j) {
            long long g = 0;
            for (int s = 0; s < D.N; ++s) g += C[(size_t)s * D.E + (size_t)d * D.El + j];
            rows += (j + 1 < D.El) ? (g + D.align - 1) / D.align * D.align : g;   // as the planning block pads
        }
        need_recv = std::max(need_recv, recv);
        need_expert = std::max(need_expert, rows);
    }
    delete[] host;
    *recv_capacity_rows = need_recv;
    *expert_capacity_rows = need_expert;
    return FL_OK;
}

const char *fl_moe_strerror(int code) {
    switch (code) {
        case FL_OK: return "ok";
        case FL_ERR_INVALID_ARG: return "invalid argument";
        case FL_ERR_ALIGNMENT: return "pointer or size not aligned as required";
        case FL_ERR_WORKSPACE: return "workspace too small";
        case FL_ERR_HIP: return "HIP runtime error";
        case FL_ERR_STATIC_LIMIT:
            return "configuration needs more scratch than the library's static array (FL_STATIC_SCRATCH_BYTES)";
        default: return "unknown error";
    }
}

int fl_moe_debug_views(fl_moe_ctx *ctx, fl_moe_debug_view *out) {
    if (!ctx || !out) return FL_ERR_INVALID_ARG;
    const Tables &W = ctx->W;
    out->buf_a = W.bufA; out->buf_b = W.bufB;
    out->buf_a_rank_bytes = ctx->D.bufA_rank_bytes; out->buf_b_rank_bytes = ctx->D.bufB_rank_bytes;
    out->arrive_route = W.arrive_route; out->arrive_disp = W.arrive_disp;
    out->arrive_comb = W.arrive_comb;
    out->epoch_route = W.epoch_route; out->expect_disp = W.expect_disp; out->expect_comb = W.expect_comb;
    out->status = W.status;
    return FL_OK;
}

int fl_moe_debug_tune(fl_moe_ctx *ctx, int knob, int value) {
    if (!ctx || value < -1) return FL_ERR_INVALID_ARG;
    const bool dflt = value == -1;             // -1 = back to the default
    switch (knob) {
        case 0: if (value > kMaxRowsPerBlock) return FL_ERR_INVALID_ARG; ctx->D.tune_rows = dflt ? 0 : value; break;
        case 1: if (value > 8) return FL_ERR_INVALID_ARG; ctx->D.tune_reduce = dflt ? 0 : value; break;
        case 2: ctx->D.tune_waves = dflt ? 0 : value; break;
        case 3: if (value > 16) return FL_ERR_INVALID_ARG; ctx->D.tune_slices = dflt ? 0 : value; break;
        case 4: ctx->D.tune_stream_mb = dflt ? 2560 : value; break;
        case 5: if (value > 1000) return FL_ERR_INVALID_ARG; ctx->D.tune_grid_pct = dflt ? 200 : value; break;
        case 6: ctx->launch_mb = dflt ? kLaunchMiB : value; break;
        case 7: if (value > 8 || value == 0) return FL_ERR_INVALID_ARG; ctx->D.tune_cap8 = dflt ? 3 : value; break;
        case 8: if (value > 2) return FL_ERR_INVALID_ARG; ctx->D.tune_order = dflt ? 0 : value; break;
        case 9: if (value > 64) return FL_ERR_INVALID_ARG; ctx->D.tune_parts = dflt ? 0 : value; break;
        default: return FL_ERR_INVALID_ARG;
    }
    return FL_OK;
}

int fl_moe_debug_launch_groups(const fl_moe_config *cfg, int rank_count, int launch_mb, int *ranks_per_group) {
    if (!ranks_per_group || launch_mb < -1) return FL_ERR_INVALID_ARG;
    Dims D;
    int e = resolve(cfg, &D);
    if (e != FL_OK) return e;
    if (rank_count < 1 || rank_count > D.N) return FL_ERR_INVALID_ARG;
    *ranks_per_group = ranks_per_launch(D, launch_mb < 0 ? kLaunchMiB : launch_mb, rank_count);
    return FL_OK;
}

// launch shapes of the three plain kernels: the fastest measured for each (see the kernels)
constexpr int kPlainCopyThreads = 64, kPlainCopyVecs = 4;
constexpr int kPlainFillThreads = 256, kPlainFillVecs = 1;
constexpr int kPlainReadThreads = 1024, kPlainReadVecs = 1;

int fl_moe_debug_copy(void *dst, const void *src, size_t bytes, void *stream) {
    if (!dst || !src || bytes == 0 || bytes % 16 != 0) return FL_ERR_INVALID_ARG;
    if (!aligned16(dst) || !aligned16(src)) return FL_ERR_ALIGNMENT;
    const size_t nvec = bytes / 16, per = (size_t)kPlainCopyThreads * kPlainCopyVecs;
    const size_t blocks = (nvec + per - 1) / per;
    if (blocks >= (1ull << 31)) return FL_ERR_INVALID_ARG;
    plain_copy_kernel<kPlainCopyThreads, kPlainCopyVecs>
        <<<dim3((unsigned)blocks), dim3(kPlainCopyThreads), 0, (hipStream_t)stream>>>((v4u *)dst, (const v4u *)src, nvec);
    return launch_status();
}

int fl_moe_debug_fill(void *dst, size_t bytes, void *stream) {
    if (!dst || bytes == 0 || bytes % 16 != 0) return FL_ERR_INVALID_ARG;
    if (!aligned16(dst)) return FL_ERR_ALIGNMENT;
    const size_t nvec = bytes / 16, per = (size_t)kPlainFillThreads * kPlainFillVecs;
    const size_t blocks = (nvec + per - 1) / per;
    if (blocks >= (1ull << 31)) return FL_ERR_INVALID_ARG;
    plain_fill_kernel<kPlainFillThreads, kPlainFillVecs>
        <<<dim3((unsigned)blocks), dim3(kPlainFillThreads), 0, (hipStream_t)stream>>>((v4u *)dst, nvec, 0x3C3C3C3Cu);
    return launch_status();
}

int fl_moe_debug_read(const void *src, size_t bytes, void *sink, void *stream) {
    if (!src || !sink || bytes == 0 || bytes % 16 != 0) return FL_ERR_INVALID_ARG;
    if (!aligned16(src) || ((uintptr_t)sink & 3)) return FL_ERR_ALIGNMENT;
    const size_t nvec = bytes / 16, per = (size_t)kPlainReadThreads * kPlainReadVecs;
    const size_t blocks = (nvec + per - 1) / per;
    if (blocks >= (1ull << 31)) return FL_ERR_INVALID_ARG;
    plain_read_kernel<kPlainReadThreads, kPlainReadVecs>
        <<<dim3((unsigned)blocks), dim3(kPlainReadThreads), 0, (hipStream_t)stream>>>((const v4u *)src, nvec,
                                                                                       (unsigned *)sink);
    return launch_status();
}

int fl_moe_profile_enable(fl_moe_ctx *ctx, int on) {
    if (!ctx) return FL_ERR_INVALID_ARG;
    if (on && !ctx->ev_start[kEventPool - 1]) {     // first use: the event pool
        for (int i = 0; i < kEventPool; ++i) {
            if (!ctx->ev_start[i] && hipEventCreate(&ctx->ev_start[i]) != hipSuccess) return FL_ERR_HIP;
            if (!ctx->ev_stop[i] && hipEventCreate(&ctx->ev_stop[i]) != hipSuccess) return FL_ERR_HIP;
        }
    }
    ctx->profile = on ? 1 : 0;
    ctx->ev_used = 0;
    return FL_OK;
}

int fl_moe_profile_collect(fl_moe_ctx *ctx, void *stream) {
    if (!ctx) return FL_ERR_INVALID_ARG;
    if (hipStreamSynchronize((hipStream_t)stream) != hipSuccess) return FL_ERR_HIP;
    for (int i = 0; i < ctx->ev_used; ++i) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, ctx->ev_start[i], ctx->ev_stop[i]) != hipSuccess)
            return FL_ERR_HIP;
        ctx->total_ms[ctx->ev_kernel[i]] += ms;
        ctx->launches[ctx->ev_kernel[i]] += 1;
    }
    ctx->ev_used = 0;
    return FL_OK;
}

int fl_moe_profile_read(fl_moe_ctx *ctx, double *total_ms, int64_t *launches) {
    if (!ctx || !total_ms || !launches) return FL_ERR_INVALID_ARG;
    for (int i = 0; i < FL_KERNEL_COUNT; ++i) {
        total_ms[i] = ctx->total_ms[i];
        launches[i] = ctx->launches[i];
    }
    return FL_OK;
}

#ifndef FLMOE_BUILD_ID
#define FLMOE_BUILD_ID "unknown"
#endif
const char *fl_moe_build_id(void) { return FLMOE_BUILD_ID; }

const char *fl_moe_kernel_name(int kernel_id) {
    if (kernel_id < 0 || kernel_id >= FL_KERNEL_COUNT) return "";
    return kKernelNames[kernel_id];
}

}  // extern "C"
