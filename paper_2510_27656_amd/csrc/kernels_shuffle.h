// The memory-bound half of the shuffle: pack, fabric copy, unpack, reduce.
//
// Paper, section MoE Dispatch/Combine.  Dispatch: input tokens are copied into
// send buffers, a contiguous source per peer, then scattered; the receiver waits
// for all transfers and re-orders tokens into the grouped-GEMM layout.  Combine:
// one scatter per peer re-using the routing information, then a locally computed
// weighted sum.  Every kernel moves whole rows with 16-byte accesses; nothing
// here is a contraction, so there is no MFMA.
#pragma once
#include "common.h"

namespace flmoe {

constexpr int kCopyThreads = 256;
constexpr int kMaxRowsPerBlock = 64;

// ------------------------------------------------------------------ dispatch: pack
// One block per token (s, t): the row is read once and written once per
// distinct destination rank, at send_off[s][d] + (rank of t among s's tokens
// bound for d).  Each copy carries a sidecar of K words naming, for every expert
// of the token that lives on d, the local expert and the token's rank among s's
// tokens of that expert; the receiver turns that into an expert-major row.
__global__ __launch_bounds__(kCopyThreads) void dispatch_pack_kernel(
    Dims D, Tables W, int rank_begin, const char *__restrict__ x,
    const int *__restrict__ indices, const int *__restrict__ num_tokens) {
    const int s = rank_begin + blockIdx.y, t = blockIdx.x, tid = threadIdx.x;
    const int K = D.K, El = D.El;
    if (t == 0 && tid == 0) W.epoch_disp[s] += 1u;
    if (!W.plan_ok[s] || t >= num_tokens[s]) return;
    __shared__ int dst_row[FL_MAX_TOPK];
    __shared__ int ndst;
    const size_t pair0 = ((size_t)s * D.T + t) * K;
    if (tid == 0) {
        int n = 0;
        for (int k = 0; k < K; ++k) {
            const int r = W.send_row[pair0 + k];
            if (r >= 0) dst_row[n++] = r;
        }
        ndst = n;
    }
    if (tid < K) {
        const int r = W.send_row[pair0 + tid];
        if (r >= 0) {
            const int d = indices[pair0 + tid] / El;
            unsigned *meta = W.send_meta + ((size_t)s * D.send_cap + r) * K;
            int m = 0;
            for (int k = 0; k < K; ++k)
                if (indices[pair0 + k] / El == d) meta[m++] = W.pair_meta[pair0 + k];
            for (; m < K; ++m) meta[m] = kNoEntry;
        }
    }
    __syncthreads();
    const int n = ndst;
    const int nvec = (int)(D.Bx / 16);
    const uint4 *src = (const uint4 *)(x + ((size_t)s * D.T + t) * D.Bx);
    char *sendbuf = W.bufA + (size_t)s * D.bufA_rank_bytes;
    for (int v = tid; v < nvec; v += kCopyThreads) {
        const uint4 val = src[v];
        for (int i = 0; i < n; ++i)
            ((uint4 *)(sendbuf + (size_t)dst_row[i] * D.Bw))[v] = val;
    }
}

// ------------------------------------------------------------------ fabric copy
// The stand-in for the NIC scatter: for every (source, destination) pair one
// contiguous segment of the source's send buffer is copied into the range of
// the destination's receive buffer that the exchanged counts reserved for it.
// Blocks copy chunks of rows; a per-segment progress count finds the chunk that
// completes a segment, and only then is arrive[destination][source] bumped
// (release), so the counter says "this payload is fully delivered" and nothing
// is assumed about the order in which chunks or segments land.  Empty segments
// notify too, so every receiver expects exactly one bump per source per step.
struct FabricArgs {
    const char *src_base; long long src_rank_stride;
    char *dst_base;       long long dst_rank_stride;
    const int *seg_off;   // [N][N+1] segment starts in the source buffer
    const int *dst_off;   // [N src][N dst] first row in the destination buffer
    const unsigned *src_meta; long long src_meta_rank_stride;   // in words; may be null
    unsigned *dst_meta;       long long dst_meta_rank_stride;
    unsigned *arrive;     // [N dst][N src]
    unsigned *seg_done;   // [N src][N dst]
    long long row_bytes;
    int rows_per_block;
};

template <bool FENCED>
__global__ __launch_bounds__(kCopyThreads) void fabric_copy_kernel(Dims D, Tables W,
                                                                   FabricArgs A, int rank_begin) {
    const int s = rank_begin + blockIdx.y, tid = threadIdx.x, N = D.N;
    __shared__ int off[FL_MAX_RANKS + 1];
    __shared__ int row_dst[kMaxRowsPerBlock];
    if (!W.plan_ok[s]) {                       // step skipped: keep the counters in step
        if (blockIdx.x == 0 && tid < N) add_counter<FENCED>(A.arrive + (size_t)tid * N + s, 1u);
        return;
    }
    if (tid <= N) off[tid] = A.seg_off[(size_t)s * (N + 1) + tid];
    __syncthreads();
    if (blockIdx.x == 0 && tid < N && off[tid + 1] == off[tid])
        add_counter<FENCED>(A.arrive + (size_t)tid * N + s, 1u);
    const int total = off[N];
    const int i0 = blockIdx.x * A.rows_per_block;
    if (i0 >= total) return;
    const int i1 = min(i0 + A.rows_per_block, total);
    if (tid < i1 - i0) {
        const int i = i0 + tid;
        const int d = seg_of(off, N, i);
        const int dr = A.dst_off[(size_t)s * N + d] + (i - off[d]);
        row_dst[tid] = dr;
        if (A.src_meta) {
            const unsigned *ms = A.src_meta + (size_t)s * A.src_meta_rank_stride + (size_t)i * D.K;
            unsigned *md = A.dst_meta + (size_t)d * A.dst_meta_rank_stride + (size_t)dr * D.K;
            for (int k = 0; k < D.K; ++k) md[k] = ms[k];
        }
    }
    __syncthreads();
    const int nvec = (int)(A.row_bytes / 16);
    const char *src = A.src_base + (size_t)s * A.src_rank_stride;
    int d = seg_of(off, N, i0);
    for (int i = i0; i < i1; ++i) {
        while (off[d + 1] <= i) ++d;
        char *dst = A.dst_base + (size_t)d * A.dst_rank_stride;
        copy_row<kCopyThreads>((uint4 *)(dst + (size_t)row_dst[i - i0] * A.row_bytes),
                               (const uint4 *)(src + (size_t)i * A.row_bytes), nvec, tid);
    }
    stores_done<FENCED>();
    __syncthreads();
    if (tid == 0) {
        for (int dd = seg_of(off, N, i0); dd < N && off[dd] < i1; ++dd) {
            const int lo = max(off[dd], i0), hi = min(off[dd + 1], i1);
            if (hi <= lo) continue;
            const unsigned len = (unsigned)(off[dd + 1] - off[dd]);
            unsigned *done = A.seg_done + (size_t)s * N + dd;
            const unsigned old = add_counter<FENCED>(done, (unsigned)(hi - lo));
            if (old + (unsigned)(hi - lo) == len) {
                __hip_atomic_store(done, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                add_counter<FENCED>(A.arrive + (size_t)dd * N + s, 1u);
            }
        }
    }
}

// ------------------------------------------------------------------ dispatch: unpack
// Receiver half at rank d.  A block takes a chunk of received rows, waits
// (bounded) for the arrival counters of the sources those rows came from, and
// writes every row once per local expert that wants it, at
//   base_x[d][local expert][source] + rank carried in the sidecar,
// which is the (expert, source rank, token) order of the grouped layout.
template <bool FENCED>
__global__ __launch_bounds__(kCopyThreads) void dispatch_unpack_kernel(
    Dims D, Tables W, int rank_begin, char *__restrict__ expert_x,
    float *__restrict__ expert_scales, int *__restrict__ tokens_per_expert, int rows_per_block) {
    const int d = rank_begin + blockIdx.y, tid = threadIdx.x, N = D.N, El = D.El, K = D.K;
    __shared__ int off[FL_MAX_RANKS + 1];
    __shared__ int dst_rows[kMaxRowsPerBlock][FL_MAX_TOPK];
    __shared__ int dst_cnt[kMaxRowsPerBlock];
    __shared__ int timed_out;
    if (!W.plan_ok[d]) return;
    if (blockIdx.x == 0)
        for (int j = tid; j < El; j += kCopyThreads)
            tokens_per_expert[(size_t)d * El + j] = W.G[(size_t)d * El + j];
    char *xd = expert_x + (size_t)d * D.expert_cap * D.Be;
    if ((D.flags & FL_FLAG_ZERO_PAD) && (int)blockIdx.x < El - 1) {
        const int j = blockIdx.x;
        const long long lo = W.expert_off[(size_t)d * (El + 1) + j] + W.G[(size_t)d * El + j];
        const long long hi = W.expert_off[(size_t)d * (El + 1) + j + 1];
        const long long nv = (hi - lo) * (D.Be / 16);
        uint4 *p = (uint4 *)(xd + lo * D.Be);
        for (long long v = tid; v < nv; v += kCopyThreads) p[v] = make_uint4(0, 0, 0, 0);
        if (expert_scales) {
            float *sp = expert_scales + ((size_t)d * D.expert_cap + lo) * D.scales_per_row;
            for (long long v = tid; v < (hi - lo) * D.scales_per_row; v += kCopyThreads) sp[v] = 0.f;
        }
    }
    if (tid <= N) off[tid] = W.recv_off[(size_t)d * (N + 1) + tid];
    if (tid == 0) timed_out = 0;
    __syncthreads();
    const int total = off[N];
    const int r0 = blockIdx.x * rows_per_block;
    if (r0 >= total) return;
    const int r1 = min(r0 + rows_per_block, total);
    const int s0 = seg_of(off, N, r0), s1 = seg_of(off, N, r1 - 1);
    if (tid < kWave) {
        if (!wave_wait_counters(W.arrive_disp + (size_t)d * N + s0, s1 - s0 + 1, W.epoch_disp[d],
                                D.spin_limit)) {
            if (tid == 0) { timed_out = 1; latch_status(W.status, FL_STATUS_TIMEOUT); }
        }
        acquire_payload<FENCED>();
    }
    __syncthreads();
    if (timed_out) return;
    if (tid < r1 - r0) {
        const int r = r0 + tid;
        const int s = seg_of(off, N, r);
        const unsigned *meta = W.recv_meta + ((size_t)d * D.recv_cap + r) * K;
        int n = 0;
        for (int k = 0; k < K; ++k) {
            const unsigned m = meta[k];
            if (m == kNoEntry) break;
            const int j = (int)(m >> 24), i = (int)(m & 0xFFFFFFu);
            dst_rows[tid][n++] = W.base_x[((size_t)d * El + j) * N + s] + i;
        }
        dst_cnt[tid] = n;
    }
    __syncthreads();
    const char *recv = W.bufB + (size_t)d * D.bufB_rank_bytes;
    const int nvec = (int)(D.Be / 16);
    for (int r = r0; r < r1; ++r) {
        const uint4 *src = (const uint4 *)(recv + (size_t)r * D.Bw);
        const int n = dst_cnt[r - r0];
        const int *dr = dst_rows[r - r0];
        for (int v = tid; v < nvec; v += kCopyThreads) {
            const uint4 val = src[v];
            for (int i = 0; i < n; ++i) ((uint4 *)(xd + (size_t)dr[i] * D.Be))[v] = val;
        }
        if (D.scales_per_row) {                // e4m3: the scales follow the bytes on the wire
            const float *ssrc = (const float *)(recv + (size_t)r * D.Bw + D.Be);
            for (int v = tid; v < D.scales_per_row; v += kCopyThreads) {
                const float val = ssrc[v];
                for (int i = 0; i < n; ++i)
                    expert_scales[((size_t)d * D.expert_cap + dr[i]) * D.scales_per_row + v] = val;
            }
        }
    }
}

// ------------------------------------------------------------------ combine: pack
// Rank d gathers, for every source s, the rows of its experts that belong to s
// (contiguous per expert in the grouped layout) into one contiguous reply:
// combine-send row q of source s and local expert j comes from expert-major row
// base_x[d][j][s] + (q - cs_base[d][s][j]).
__global__ __launch_bounds__(kCopyThreads) void combine_pack_kernel(
    Dims D, Tables W, int rank_begin, const char *__restrict__ expert_y, int rows_per_block) {
    const int d = rank_begin + blockIdx.y, tid = threadIdx.x, N = D.N, El = D.El;
    __shared__ int off[FL_MAX_RANKS + 1];
    __shared__ int src_row[kMaxRowsPerBlock];
    if (blockIdx.x == 0 && tid == 0) W.epoch_comb[d] += 1u;
    if (!W.plan_ok[d]) return;
    if (tid <= N) off[tid] = W.cs_off[(size_t)d * (N + 1) + tid];
    __syncthreads();
    const int total = off[N];
    const int q0 = blockIdx.x * rows_per_block;
    if (q0 >= total) return;
    const int q1 = min(q0 + rows_per_block, total);
    if (tid < q1 - q0) {
        const int q = q0 + tid;
        const int s = seg_of(off, N, q);
        const int *csb = W.cs_base + ((size_t)d * N + s) * El;
        const int j = seg_of(csb, El, q);
        src_row[tid] = W.base_x[((size_t)d * El + j) * N + s] + (q - csb[j]);
    }
    __syncthreads();
    const int nvec = (int)(D.Bc / 16);
    const char *yd = expert_y + (size_t)d * D.expert_cap * D.Bc;
    char *out = W.bufB + (size_t)d * D.bufB_rank_bytes;
    for (int q = q0; q < q1; ++q)
        copy_row<kCopyThreads>((uint4 *)(out + (size_t)q * D.Bc),
                               (const uint4 *)(yd + (size_t)src_row[q - q0] * D.Bc), nvec, tid);
}

// ------------------------------------------------------------------ combine: reduce
// One block per token (s, t):
//   out[s][t] = bf16( sum_k w[k] * float(row comb_pos[s][t][k]) ), fp32 fused
// multiply-add, k ascending, one final rounding.
template <int KT>
__device__ inline void reduce_row(const char *__restrict__ recv, const int *pos, const float *w,
                                  int K, long long Bc, int nvec, uint4 *__restrict__ out, int tid) {
    for (int v = tid; v < nvec; v += kCopyThreads) {
        float acc[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = 0.f;
        if (KT > 0) {
            uint4 y[KT > 0 ? KT : 1];
#pragma unroll
            for (int k = 0; k < KT; ++k) y[k] = ((const uint4 *)(recv + (size_t)pos[k] * Bc))[v];
#pragma unroll
            for (int k = 0; k < KT; ++k) {
                const float wk = w[k];
                acc[0] = fmaf(wk, bf16_lo(y[k].x), acc[0]); acc[1] = fmaf(wk, bf16_hi(y[k].x), acc[1]);
                acc[2] = fmaf(wk, bf16_lo(y[k].y), acc[2]); acc[3] = fmaf(wk, bf16_hi(y[k].y), acc[3]);
                acc[4] = fmaf(wk, bf16_lo(y[k].z), acc[4]); acc[5] = fmaf(wk, bf16_hi(y[k].z), acc[5]);
                acc[6] = fmaf(wk, bf16_lo(y[k].w), acc[6]); acc[7] = fmaf(wk, bf16_hi(y[k].w), acc[7]);
            }
        } else {
            for (int k = 0; k < K; ++k) {
                const uint4 y = ((const uint4 *)(recv + (size_t)pos[k] * Bc))[v];
                const float wk = w[k];
                acc[0] = fmaf(wk, bf16_lo(y.x), acc[0]); acc[1] = fmaf(wk, bf16_hi(y.x), acc[1]);
                acc[2] = fmaf(wk, bf16_lo(y.y), acc[2]); acc[3] = fmaf(wk, bf16_hi(y.y), acc[3]);
                acc[4] = fmaf(wk, bf16_lo(y.z), acc[4]); acc[5] = fmaf(wk, bf16_hi(y.z), acc[5]);
                acc[6] = fmaf(wk, bf16_lo(y.w), acc[6]); acc[7] = fmaf(wk, bf16_hi(y.w), acc[7]);
            }
        }
        uint4 o;
        o.x = pack_bf16x2(acc[0], acc[1]); o.y = pack_bf16x2(acc[2], acc[3]);
        o.z = pack_bf16x2(acc[4], acc[5]); o.w = pack_bf16x2(acc[6], acc[7]);
        out[v] = o;
    }
}

template <bool FENCED>
__global__ __launch_bounds__(kCopyThreads) void combine_reduce_kernel(
    Dims D, Tables W, int rank_begin, const float *__restrict__ weights, char *__restrict__ out,
    const int *__restrict__ num_tokens) {
    const int s = rank_begin + blockIdx.y, t = blockIdx.x, tid = threadIdx.x, N = D.N, K = D.K;
    __shared__ int pos[FL_MAX_TOPK];
    __shared__ float w[FL_MAX_TOPK];
    __shared__ int timed_out;
    if (!W.plan_ok[s] || t >= num_tokens[s]) return;
    if (tid == 0) timed_out = 0;
    __syncthreads();
    if (tid < kWave) {
        if (!wave_wait_counters(W.arrive_comb + (size_t)s * N, N, W.epoch_comb[s], D.spin_limit)) {
            if (tid == 0) { timed_out = 1; latch_status(W.status, FL_STATUS_TIMEOUT); }
        }
        acquire_payload<FENCED>();
    } else if (tid < kWave + K) {
        const int k = tid - kWave;
        pos[k] = W.comb_pos[((size_t)s * D.T + t) * K + k];
        w[k] = weights[((size_t)s * D.T + t) * K + k];
    }
    __syncthreads();
    if (timed_out) return;
    const char *recv = W.bufA + (size_t)s * D.bufA_rank_bytes;
    uint4 *o = (uint4 *)(out + ((size_t)s * D.T + t) * D.Bc);
    const int nvec = (int)(D.Bc / 16);
    if (K == 8) reduce_row<8>(recv, pos, w, K, D.Bc, nvec, o, tid);
    else if (K == 4) reduce_row<4>(recv, pos, w, K, D.Bc, nvec, o, tid);
    else if (K == 2) reduce_row<2>(recv, pos, w, K, D.Bc, nvec, o, tid);
    else reduce_row<0>(recv, pos, w, K, D.Bc, nvec, o, tid);
}

// ------------------------------------------------------------------ diagnostic copy
__global__ __launch_bounds__(kCopyThreads) void plain_copy_kernel(uint4 *__restrict__ dst,
                                                                  const uint4 *__restrict__ src,
                                                                  size_t nvec) {
    const size_t stride = (size_t)gridDim.x * kCopyThreads * 4;
    for (size_t v = (size_t)blockIdx.x * kCopyThreads * 4 + threadIdx.x; v < nvec; v += stride) {
        uint4 a, b, c, d;
        const bool f = v + 3 * kCopyThreads < nvec;
        a = src[v];
        if (f) { b = src[v + kCopyThreads]; c = src[v + 2 * kCopyThreads]; d = src[v + 3 * kCopyThreads]; }
        dst[v] = a;
        if (f) { dst[v + kCopyThreads] = b; dst[v + 2 * kCopyThreads] = c; dst[v + 3 * kCopyThreads] = d; }
        else {
            for (size_t u = v + kCopyThreads; u < nvec && u < v + 4 * kCopyThreads; u += kCopyThreads)
                dst[u] = src[u];
        }
    }
}

}  // namespace flmoe
