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
constexpr int kPackThreads = 128;
constexpr int kMaxRowsPerBlock = 64;

// What a completed (sender, receiver) transfer adds to the receiver's counter: its
// payload in 16-byte units plus one for the transfer itself, so that an EMPTY transfer
// is announced too (section TransferEngine: an immediate is delivered even for a
// zero-size write) and a receiver that has seen all its counters complete knows that
// every peer's send call has got as far as announcing - which is what makes the re-use
// of the staging buffers safe without a separate barrier.
//
// Stream-ordered mode: one add per (sender, receiver) announces the whole
// transfer, like the single immediate a NIC delivers after a WRITE (section
// TransferEngine, ImmCounter).  It is issued once per sender inside the kernel of
// the send call that writes into the receivers' buffers (the scatter kernel, or
// with PUSH the pack kernel): receivers are ordered after that kernel by the
// stream, so they find counters and payload complete together, and no extra
// launch is spent.  (Per-wave announcements, as in progressive mode, cost more than
// they give here: adds to one counter from many compute dies serialise at about
// 0.2 us each, which made skewed routing several times slower.)
// off = the sender's row of the segment table ([N + 1] row offsets by receiver);
// threads first, first + step, ... each take one receiver.  only_the_ones: the
// payload units are reported by the waves that deliver them (progressive mode).
__device__ inline void announce_transfers(const int *off, unsigned *arrive, unsigned units_per_row,
                                          int sender, int N, int first, int step, bool only_the_ones = false) {
    for (int p = first; p < N; p += step) {
        const int rows = off[p + 1] - off[p];
        add_counter(arrive + (size_t)p * N + sender, only_the_ones ? 1u : (unsigned)rows * units_per_row + 1u);
    }
}

// ------------------------------------------------------------------ dispatch: pack
// `slices` blocks per token (s, t), each taking a slice of the row (so a thread
// usually has a single vector): the slice is read once and written once per
// distinct destination rank, at send_off[s][d] + (rank of t among s's tokens
// bound for d).  Each copy carries a sidecar of K words naming, for every expert
// of the token that lives on d, the local expert and the token's rank among s's
// tokens of that expert; the receiver turns that into an expert-major row.
//
// PUSH (every peer's receive buffer can be stored to, section Dispatch: within a
// node payloads are pushed from the send kernel): the copies and their sidecars
// go straight into the destinations' receive buffers; no send buffer is filled
// and no scatter follows.  FENCED (progressive mode, PUSH only): device-scope
// stores, and the block adds the 16-byte units it wrote to
// arrive[destination][source] itself once they are acknowledged; stream-ordered
// with PUSH, the sender's first block announces the whole transfers.
template <bool PUSH, bool FENCED>
__global__ __launch_bounds__(kPackThreads) void dispatch_pack_kernel(
    Dims D, Tables W, int rank_begin, const char *__restrict__ x,
    const int *__restrict__ indices, const int *__restrict__ num_tokens, int slices,
    const float *__restrict__ weights /* [N][T][K], only when the sidecar carries them */,
    long long src_row_bytes /* bytes of one row of x: 2*H, or H for ready-made e4m3 codes */,
    const float *__restrict__ src_scales /* [N][T][H/128] with ready-made codes, else null */) {
    const int s = rank_begin + blockIdx.y, t = blockIdx.x / slices, slice = blockIdx.x % slices;
    const int tid = threadIdx.x;
    const int K = D.K, El = D.El;
    // The slice's payload depends on nothing but (s, t): its loads are issued first, so
    // that the validity check and the routing tables are fetched while they are in flight
    // (x has T rows per rank, so the loads are in bounds for absent tokens too).
    const int nvec = (int)(src_row_bytes / 16);
    const int per = (nvec + slices - 1) / slices;          // vectors of this slice: [v0, v1)
    const int v0 = slice * per, v1 = min(v0 + per, nvec);
    const v4u *src = (const v4u *)(x + ((size_t)s * D.T + t) * src_row_bytes);
    v4u r[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
        if (v0 + tid + i * kPackThreads < v1) r[i] = ld_stream(src + v0 + tid + i * kPackThreads);
    const int plan_ok = W.plan_ok[s];
    // with PUSH no scatter kernel follows: the sender's first block announces the transfers (a
    // sender without tokens still announces its empty ones), unless an announce kernel will
    if (PUSH && (FENCED || (D.flags & FL_FLAG_STREAM_ORDERED)) && blockIdx.x == 0 && plan_ok)
        announce_transfers(W.send_off + (size_t)s * (D.N + 1), W.arrive_disp, (unsigned)(D.Bw / 16), s, D.N,
                           tid, kPackThreads, FENCED);
    if (!plan_ok || t >= num_tokens[s]) return;
    __shared__ int s_row[FL_MAX_TOPK];
    __shared__ int s_dst[FL_MAX_TOPK];
    __shared__ unsigned s_meta[FL_MAX_TOPK];
    const size_t pair0 = ((size_t)s * D.T + t) * K;
    int my_row = -1, my_d = 0, target = 0;
    if (tid < K) {                             // independent loads first, then one dependent level
        my_row = W.send_row[pair0 + tid];
        my_d = indices[pair0 + tid] / El;
        s_meta[tid] = W.pair_meta[pair0 + tid];
        s_dst[tid] = my_d;
        if (my_row >= 0)                       // this copy's row in d's receive buffer
            target = recv_buffer_row(D.N, D.P, s, my_row - W.send_off[(size_t)s * (D.N + 1) + my_d],
                                     W.dst_off[(size_t)s * D.N + my_d]);
        s_row[tid] = (PUSH && my_row >= 0) ? target : my_row;
    }
    __syncthreads();
    if (slice == 0 && tid < K && my_row >= 0) {   // sidecar and fabric target of this copy
        unsigned *meta = PUSH ? W.recv_meta + ((size_t)my_d * D.recv_rows + target) * D.MW
                              : W.send_meta + ((size_t)s * D.send_cap + my_row) * D.MW;
        int m = 0;
        for (int k = 0; k < K; ++k)
            if (s_dst[k] == my_d) {
                st_word<PUSH && FENCED>((int *)meta + m, (int)s_meta[k]);
                if (D.MW > D.KM)   // the weight of that expert, for the expert rank's partial sum
                    st_word<PUSH && FENCED>((int *)meta + D.KM + m, __float_as_int(weights[pair0 + k]));
                ++m;
            }
        for (; m < D.KM; ++m) st_word<PUSH && FENCED>((int *)meta + m, (int)kNoEntry);
        if (!PUSH) W.fab_dst_disp[(size_t)s * D.send_cap + my_row] = make_int2(my_d, target);
    }
    char *sendbuf = W.bufA + (size_t)s * D.bufA_rank_bytes;
    for (int b = v0 + tid; b < v1; b += 4 * kPackThreads) {
        if (b != v0 + tid) {                   // later batches (rows beyond 8 KB per slice)
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (b + i * kPackThreads < v1) r[i] = ld_stream(src + b + i * kPackThreads);
        }
        for (int k = 0; k < K; ++k) {
            const int row = s_row[k];          // uniform: one copy per distinct destination
            if (row < 0) continue;
            char *base = PUSH ? W.bufB + (size_t)s_dst[k] * D.bufB_rank_bytes : sendbuf;
            v4u *dst = (v4u *)(base + (size_t)row * D.Bw);
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (b + i * kPackThreads < v1)
                    st_payload<PUSH && FENCED, true>(dst + b + i * kPackThreads, r[i]);
        }
    }
    // Ready-made e4m3 codes (section Kernel Microbenchmarks: the dispatched token is 7168
    // fp8 values and 56 fp32 scaling factors): the scales follow the codes in the wire row.
    const bool with_scales = src_scales != nullptr && slice == 0;
    if (with_scales) {
        const float *sc = src_scales + ((size_t)s * D.T + t) * D.scales_per_row;
        if (D.scales_per_row % 4 == 0) {       // whole 16-byte vectors (rows of scales stay aligned)
            for (int v = tid; v < D.scales_per_row / 4; v += kPackThreads) {
                const v4u val = ld_stream((const v4u *)sc + v);
                for (int k = 0; k < K; ++k) {
                    const int row = s_row[k];
                    if (row < 0) continue;
                    char *base = PUSH ? W.bufB + (size_t)s_dst[k] * D.bufB_rank_bytes : sendbuf;
                    st_payload<PUSH && FENCED, true>((v4u *)(base + (size_t)row * D.Bw + D.Be) + v, val);
                }
            }
        } else {
            for (int v = tid; v < D.scales_per_row; v += kPackThreads) {
                const int val = __float_as_int(sc[v]);
                for (int k = 0; k < K; ++k) {
                    const int row = s_row[k];
                    if (row < 0) continue;
                    char *base = PUSH ? W.bufB + (size_t)s_dst[k] * D.bufB_rank_bytes : sendbuf;
                    st_word<PUSH && FENCED>((int *)(base + (size_t)row * D.Bw + D.Be) + v, val);
                }
            }
        }
    }
    if (PUSH && FENCED) {                      // what this block delivered, per destination
        stores_done<FENCED>();
        __syncthreads();
        const unsigned units = (unsigned)(v1 - v0) + (with_scales ? (unsigned)((D.Bw - D.Be) / 16) : 0u);
        if (tid < K && my_row >= 0 && units > 0)
            add_counter(W.arrive_disp + (size_t)my_d * D.N + s, units);
    }
}

// ------------------------------------------------------------------ dispatch: pack with e4m3 quantisation
// Payload of section Kernel Microbenchmarks: H e4m3 bytes followed by H/128 fp32
// scales per token.  Rule per 128-element block: amax = max |x|, scale =
// amax / 448 (1 when amax is 0), q = e4m3(x / scale) rounded to nearest even and
// saturated at +-448; both divisions are IEEE fp32 divisions.
//
// OCP E4M3, finite-only: 1 sign, 4 exponent bits (bias 7), 3 mantissa bits,
// subnormals m * 2^-9, largest finite 448, no infinities.
//
// Four quotients to four e4m3 bytes with the part's own converter (OCP E4M3 on
// gfx950, round to nearest even, subnormals included; checked against the oracle's
// arithmetic encoder on every finite bf16 input under several block maxima).  A quotient can exceed 448
// by one fp32 step (both divisions round), so magnitudes are held at 448 first.
// The block maximum skips NaN elements (an ordered comparison, as in the rule's plain reading).
__device__ inline float e4m3_hold(float v) {
    return fabsf(v) >= 448.0f ? copysignf(448.0f, v) : v;
}
__device__ inline unsigned e4m3_pack4(float a, float b, float c, float d) {
    int w = __builtin_amdgcn_cvt_pk_fp8_f32(e4m3_hold(a), e4m3_hold(b), 0, false);
    w = __builtin_amdgcn_cvt_pk_fp8_f32(e4m3_hold(c), e4m3_hold(d), w, true);
    return (unsigned)w;
}
// Non-finite inputs (Inf or NaN, exponent bits all ones): the quotient is NaN either
// way (NaN / scale; Inf / Inf, because an Inf makes the block's scale infinite) and the
// code is the NaN code 0x7f with the sign of the INPUT element, which IEEE leaves
// open for Inf / Inf and the converter for NaN.  lo16 / hi16: the two bf16 inputs of
// a packed word; byte positions 2 * i and 2 * i + 1 of the four-code word.
__device__ inline bool bf16x2_nonfinite(unsigned w) {
    return ((w & 0x7f80u) == 0x7f80u) || ((w & 0x7f800000u) == 0x7f800000u);
}
__device__ inline unsigned e4m3_fix_nonfinite(unsigned codes, unsigned w0, unsigned w1) {
    const unsigned in[4] = {w0 & 0xffffu, w0 >> 16, w1 & 0xffffu, w1 >> 16};
#pragma unroll
    for (int i = 0; i < 4; ++i)
        if ((in[i] & 0x7f80u) == 0x7f80u)
            codes = (codes & ~(0xffu << (8 * i))) | ((((in[i] >> 8) & 0x80u) | 0x7fu) << (8 * i));
    return codes;
}

constexpr int kQuantLanes = 8;     // lanes per 128-element block: 16 bf16 values each

// One workgroup of QT threads takes QT / 8 consecutive quantisation blocks of one
// token (QT = 512 covers a 7168-element row whole, 4 us of 64 faster than two
// workgroups of 256; more blocks per lane group measured no gain); every lane loads
// 32 bytes, takes part in an 8-lane max, and stores 16 bytes of e4m3 per destination
// copy; the scales go out as 16-byte vectors from LDS.
template <bool PUSH, bool FENCED, int QT>   // PUSH, FENCED as in dispatch_pack_kernel
__global__ __launch_bounds__(QT) void dispatch_pack_e4m3_kernel(
    Dims D, Tables W, int rank_begin, const char *__restrict__ x,
    const int *__restrict__ indices, const int *__restrict__ num_tokens, int slices,
    const float *__restrict__ weights /* [N][T][K], only when the sidecar carries them */) {
    constexpr int kQuantThreads = QT;
    const int s = rank_begin + blockIdx.y, t = blockIdx.x / slices, slice = blockIdx.x % slices;
    const int tid = threadIdx.x;
    const int K = D.K, El = D.El;
    // as in dispatch_pack_kernel, the payload loads go first
    const int nblk = D.scales_per_row;                          // 128-element blocks in the row
    const int blk = slice * (kQuantThreads / kQuantLanes) + tid / kQuantLanes;
    const int sub = tid % kQuantLanes;
    const bool live = blk < nblk;
    v4u in0 = {0u, 0u, 0u, 0u}, in1 = {0u, 0u, 0u, 0u};
    if (live) {
        const v4u *src = (const v4u *)(x + ((size_t)s * D.T + t) * D.Bx) + (size_t)blk * 16 + sub * 2;
        in0 = ld_stream(src);
        in1 = ld_stream(src + 1);
    }
    const int plan_ok = W.plan_ok[s];
    if (PUSH && (FENCED || (D.flags & FL_FLAG_STREAM_ORDERED)) && blockIdx.x == 0 && plan_ok)   // as in dispatch_pack_kernel
        announce_transfers(W.send_off + (size_t)s * (D.N + 1), W.arrive_disp, (unsigned)(D.Bw / 16), s, D.N,
                           tid, kQuantThreads, FENCED);
    if (!plan_ok || t >= num_tokens[s]) return;
    __shared__ int s_row[FL_MAX_TOPK];
    __shared__ int s_dst[FL_MAX_TOPK];
    __shared__ unsigned s_meta[FL_MAX_TOPK];
    const size_t pair0 = ((size_t)s * D.T + t) * K;
    int my_row = -1, my_d = 0, target = 0;
    if (tid < K) {
        my_row = W.send_row[pair0 + tid];
        my_d = indices[pair0 + tid] / El;
        s_meta[tid] = W.pair_meta[pair0 + tid];
        s_dst[tid] = my_d;
        if (my_row >= 0)
            target = recv_buffer_row(D.N, D.P, s, my_row - W.send_off[(size_t)s * (D.N + 1) + my_d],
                                     W.dst_off[(size_t)s * D.N + my_d]);
        s_row[tid] = (PUSH && my_row >= 0) ? target : my_row;
    }
    __syncthreads();
    if (slice == 0 && tid < K && my_row >= 0) {
        unsigned *meta = PUSH ? W.recv_meta + ((size_t)my_d * D.recv_rows + target) * D.MW
                              : W.send_meta + ((size_t)s * D.send_cap + my_row) * D.MW;
        int m = 0;
        for (int k = 0; k < K; ++k)
            if (s_dst[k] == my_d) {
                st_word<PUSH && FENCED>((int *)meta + m, (int)s_meta[k]);
                if (D.MW > D.KM)   // the weight of that expert, for the expert rank's partial sum
                    st_word<PUSH && FENCED>((int *)meta + D.KM + m, __float_as_int(weights[pair0 + k]));
                ++m;
            }
        for (; m < D.KM; ++m) st_word<PUSH && FENCED>((int *)meta + m, (int)kNoEntry);
        if (!PUSH) W.fab_dst_disp[(size_t)s * D.send_cap + my_row] = make_int2(my_d, target);
    }
    float f[16];
    const unsigned w[8] = {in0.x, in0.y, in0.z, in0.w, in1.x, in1.y, in1.z, in1.w};
#pragma unroll
    for (int i = 0; i < 8; ++i) { f[2 * i] = bf16_lo(w[i]); f[2 * i + 1] = bf16_hi(w[i]); }
    float amax = 0.f;              // a NaN element (quiet or signalling) fails the comparison and is skipped
#pragma unroll
    for (int i = 0; i < 16; ++i) { const float a = fabsf(f[i]); amax = a > amax ? a : amax; }
#pragma unroll
    for (int o = 1; o < kQuantLanes; o <<= 1) amax = fmaxf(amax, __shfl_xor(amax, o));
    const float scale = amax == 0.f ? 1.0f : __fdiv_rn(amax, 448.0f);
    unsigned q[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
        q[i] = e4m3_pack4(__fdiv_rn(f[4 * i], scale), __fdiv_rn(f[4 * i + 1], scale),
                          __fdiv_rn(f[4 * i + 2], scale), __fdiv_rn(f[4 * i + 3], scale));
    bool odd_values = false;       // rare: keep the common path free of the per-byte fix-up
#pragma unroll
    for (int i = 0; i < 8; ++i) odd_values |= bf16x2_nonfinite(w[i]);
    if (odd_values) {
#pragma unroll
        for (int i = 0; i < 4; ++i) q[i] = e4m3_fix_nonfinite(q[i], w[2 * i], w[2 * i + 1]);
    }
    const v4u out = {q[0], q[1], q[2], q[3]};
    // the block's scales are gathered in LDS and stored as 16-byte vectors when the
    // row's scale count allows it (scattered 4-byte stores are partial-line writes)
    __shared__ __align__(16) float s_scale[kQuantThreads / kQuantLanes];
    const bool scale_vectors = nblk % 4 == 0;
    if (scale_vectors) {
        if (live && sub == 0) s_scale[tid / kQuantLanes] = scale;
        __syncthreads();
    }
    const int blk0 = slice * (kQuantThreads / kQuantLanes);
    const int nsv = (min(nblk - blk0, kQuantThreads / kQuantLanes)) / 4;   // scale vectors of this block
    char *sendbuf = W.bufA + (size_t)s * D.bufA_rank_bytes;
    for (int k = 0; k < K; ++k) {
        const int row = s_row[k];
        if (row < 0) continue;
        char *dst = (PUSH ? W.bufB + (size_t)s_dst[k] * D.bufB_rank_bytes : sendbuf) + (size_t)row * D.Bw;
        if (live) st_payload<PUSH && FENCED, true>((v4u *)dst + (size_t)blk * kQuantLanes + sub, out);
        if (scale_vectors) {
            if (tid < nsv)
                st_payload<PUSH && FENCED, true>((v4u *)(dst + D.Be) + blk0 / 4 + tid,
                                                 ((const v4u *)s_scale)[tid]);
        } else if (live && sub == 0) {
            st_word<PUSH && FENCED>((int *)(dst + D.Be) + blk, __float_as_int(scale));
        }
    }
    if (PUSH && FENCED) {
        // Units of the row this block wrote: 8 per quantisation block of codes, and the
        // 16-byte units its scales fall into (blocks start on multiples of 32 scales, so
        // no unit is shared between blocks; the row's last unit may be part padding).
        const int n_live = min(nblk - blk0, kQuantThreads / kQuantLanes);
        stores_done<FENCED>();
        __syncthreads();
        // the padding that brings a wire row to a whole number of 128-byte lines is nobody's
        // to write; the first block claims it so that a row's units add up to Bw / 16
        const int pad_units = (int)(D.Bw / 16) - (nblk * 8 + (nblk + 3) / 4);
        if (tid < K && my_row >= 0 && n_live > 0)
            add_counter(W.arrive_disp + (size_t)my_d * D.N + s,
                        (unsigned)(n_live * 8 + (n_live + 3) / 4 + (slice == 0 ? pad_units : 0)));
    }
}

// ------------------------------------------------------------------ fabric copy
// The stand-in for the NIC scatter: every row of a source's send buffer is
// copied into the row of the destination's receive buffer that the exchanged
// counts reserved for it (the target of each row was recorded when the row was
// packed, so a wave needs one small load before its payload loads; a version
// that searched the offset tables per wave measured 25 % slower).  Waves work on
// their own: a row is shared by `waves_per_row` waves, each copies its slice
// with four loads in flight.  No barrier, no shared memory, no ticket.  In
// progressive mode (FENCED) a wave then adds the number of 16-byte units it
// delivered to arrive[destination][source] with an atomic whose result nobody
// waits for: the counters only ever say "this much of source s's payload has
// landed", in whatever order waves finish.  Otherwise nobody may look before the
// kernel has ended: the whole transfers are announced by the announce kernel
// behind it (default) or, for stream-ordered callers, by one wave per sender
// inside it (announce_transfers).
struct FabricArgs {
    const char *src_base; long long src_rank_stride;
    char *dst_base;       long long dst_rank_stride;
    const int *seg_off;   // [N][N+1] segment starts in the source buffer; [N] = rows in use
    const int2 *row_dst;  // [N][row_cap] (destination rank, row in its buffer) of every source row
    long long row_cap;
    const unsigned *src_meta; long long src_meta_rank_stride;   // in words; may be null
    unsigned *dst_meta;       long long dst_meta_rank_stride;
    unsigned *arrive;     // [N dst][N src]
    long long row_bytes;
    int waves_per_row;    // 1..16
    int dst_row_lo;       // rows whose target row is below this belong to the private-slot scatter
    int announce;         // this launch also advances arrive[.][s] (announce_transfers): 1 = by the whole
                          // transfers (stream-ordered mode), 2 = by the ones only (progressive mode, where
                          // the waves report the payload they deliver)
    int order;            // test switch: order in which a sender's rows (sorted by destination) are
                          // taken: 0 = as stored, 1 = last destination first, 2 = starting with the
                          // sender's right-hand neighbour and wrapping round
};

// One wave's share of one row: slice `sub` of `G` (vectors v with (v / 64) % G ==
// sub), the sidecar when it is slice 0, and in progressive mode the count of
// 16-byte units it delivered, added to arrive[destination][source].
template <bool FENCED, bool STREAMING>
__device__ inline void fabric_send_row(const Dims &D, const FabricArgs &A, int s, int src_row,
                                       int dst_rank, int dst_row, int sub, int lane) {
    const int G = A.waves_per_row, N = D.N;
    const int nvec = (int)(A.row_bytes / 16);
    const int step = G * kWave;
    const v4u *src =
        (const v4u *)(A.src_base + (size_t)s * A.src_rank_stride + (size_t)src_row * A.row_bytes);
    v4u *dst = (v4u *)(A.dst_base + (size_t)dst_rank * A.dst_rank_stride + (size_t)dst_row * A.row_bytes);
    for (int b = sub * kWave + lane; b < nvec; b += 4 * step) {
        v4u v[4];
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (b + j * step < nvec) v[j] = ld_stream(src + b + j * step);
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (b + j * step < nvec) st_payload<FENCED, STREAMING>(dst + b + j * step, v[j]);
    }
    if (A.src_meta && sub == 0) {          // the sidecar travels with the row
        const int mv = D.MW / 4;
        const v4u *ms =
            (const v4u *)(A.src_meta + (size_t)s * A.src_meta_rank_stride) + (size_t)src_row * mv;
        v4u *md = (v4u *)(A.dst_meta + (size_t)dst_rank * A.dst_meta_rank_stride) + (size_t)dst_row * mv;
        if (lane < mv) st_payload<FENCED, STREAMING>(md + lane, ms[lane]);
    }
    if (FENCED) {          // stream-ordered launches announce whole transfers instead (announce_transfers)
        const int full = nvec / step, rem = nvec - full * step;
        const int mine = full * kWave + min(max(rem - sub * kWave, 0), kWave);
        stores_done<FENCED>();
        if (lane == 0 && mine > 0) add_counter(A.arrive + (size_t)dst_rank * N + s, (unsigned)mine);
    }
}

template <bool FENCED, int PHASE, bool STREAMING>   // PHASE only names the launch: 0 dispatch, 1 combine
__global__ __launch_bounds__(kCopyThreads) void fabric_copy_kernel(Dims D, Tables W,
                                                                   FabricArgs A, int rank_begin) {
    const int s = rank_begin + blockIdx.y, N = D.N;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = blockIdx.x * (kCopyThreads / kWave) + threadIdx.x / kWave;   // within rank s
    const int G = A.waves_per_row;
    const int sub = wave % G;
    const int row_stride = (int)(gridDim.x * (kCopyThreads / kWave)) / G;   // grid is a multiple of G waves
    const int ok = W.plan_ok[s];
    const int total = ok ? A.seg_off[(size_t)s * (N + 1) + N] : 0;   // step skipped: nothing sent
    // The first row's target is fetched together with the two loads above; capacities
    // are upper bounds, so the grid may be smaller than the rows in use and a wave loops.
    int i = wave / G;
    if (A.order == 0) {
        int2 t = make_int2(0, 0);
        if (i < A.row_cap) t = A.row_dst[(size_t)s * A.row_cap + i];
        while (i < total) {
            if (t.y >= A.dst_row_lo)       // rows below went out with the private-slot scatter
                fabric_send_row<FENCED, STREAMING>(D, A, s, i, t.x, t.y, sub, lane);
            i += row_stride;
            if (i < total) t = A.row_dst[(size_t)s * A.row_cap + i];
        }
    } else {                               // the same rows, visited in another order of destinations
        const int shift = A.order == 2 ? A.seg_off[(size_t)s * (N + 1) + (s + 1) % N] : 0;
        for (; i < total; i += row_stride) {
            const int row = A.order == 1 ? total - 1 - i : (i + shift) % total;
            const int2 t = A.row_dst[(size_t)s * A.row_cap + row];
            if (t.y >= A.dst_row_lo) fabric_send_row<FENCED, STREAMING>(D, A, s, row, t.x, t.y, sub, lane);
        }
    }
    if (A.announce && wave == 0 && ok)
        announce_transfers(A.seg_off + (size_t)s * (N + 1), A.arrive, (unsigned)(A.row_bytes / 16), s, N, lane, kWave,
                           A.announce == 2);
}

// First scatter of a dispatch with private slots (section Dispatch: tokens up to
// a fixed limit go to private buffers on every peer before the routes are
// known).  Slot q = d * P + i of source s stands for the i-th row s sends to d;
// it exists when i < M[s][d], a number s counted itself, and lands in row
// s * P + i of d's receive buffer.  Nothing here was derived from a peer's counts.
template <bool FENCED, bool STREAMING>
__global__ __launch_bounds__(kCopyThreads) void fabric_private_kernel(Dims D, Tables W,
                                                                      FabricArgs A, int rank_begin) {
    const int s = rank_begin + blockIdx.y, N = D.N, P = D.P;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = blockIdx.x * (kCopyThreads / kWave) + threadIdx.x / kWave;
    const int G = A.waves_per_row;
    const int sub = wave % G;
    const int slot_stride = (int)(gridDim.x * (kCopyThreads / kWave)) / G;
    if (!W.plan_ok[s]) return;
    for (int q = wave / G; q < N * P; q += slot_stride) {
        const int d = q / P, i = q - d * P;
        const int lo = A.seg_off[(size_t)s * (N + 1) + d], hi = A.seg_off[(size_t)s * (N + 1) + d + 1];
        if (i < hi - lo) fabric_send_row<FENCED, STREAMING>(D, A, s, lo + i, d, s * P + i, sub, lane);
    }
    if (A.announce && wave == 0)
        announce_transfers(A.seg_off + (size_t)s * (N + 1), A.arrive, (unsigned)(A.row_bytes / 16), s, N, lane, kWave,
                           A.announce == 2);
}

// ------------------------------------------------------------------ announce
// Counter-ordered mode (the default), sending side: enqueued behind the payload
// kernels of a send call in the sender's own stream, so it starts once they have
// ended and everything they stored has left for memory; one wave per sender then
// adds each whole (sender, receiver) transfer to the receiver's arrival counter
// with release semantics - the single immediate a NIC delivers after a completed
// WRITE (section TransferEngine, ImmCounter).  off: [N][N+1] row offsets of the
// senders' segment tables.
__global__ __launch_bounds__(kWave) void announce_kernel(Dims D, Tables W, int rank_begin, const int *off,
                                                         unsigned *arrive, unsigned units_per_row) {
    const int s = rank_begin + blockIdx.x, N = D.N;
    const int p = threadIdx.x;
    const int plan_ok = W.plan_ok[s];               // one round of loads: the verdict and the segment table
    const int lo = p < N ? off[(size_t)s * (N + 1) + p] : 0, hi = p < N ? off[(size_t)s * (N + 1) + p + 1] : 0;
    if (!plan_ok) return;                           // step skipped: nothing was sent
    if (p < N) {       // payload units plus one per transfer, empty transfers included (announce_transfers)
        const int rows = hi - lo;
        (void)__hip_atomic_fetch_add(arrive + (size_t)p * N + s, (unsigned)rows * units_per_row + 1u,
                                     __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// ------------------------------------------------------------------ arrival gate
// Default mode, receiving side: one wave per rank polls the rank's arrival
// counters (bounded) until every source has delivered what the exchanged counts
// promised.  That is how the paper's receive half begins as well (section
// Dispatch: it first waits until all transfers are complete, the proxy raising a
// flag once the ImmCounter has reached its expectation).  The receive kernel
// proper follows in the same stream: it starts after this kernel has ended, with
// clean caches, so what it reads is what the counters vouched for (the senders'
// payload kernels had ended, their stores written back, before the release adds).
// Waiting costs one wave per rank instead of a grid of pollers, so senders that
// run at the same time keep the machine.
__global__ __launch_bounds__(kWave) void arrival_gate_kernel(Dims D, Tables W, int rank_begin,
                                                             const unsigned *arrive, const unsigned *expect,
                                                             int *gate) {
    const int r = rank_begin + blockIdx.x, N = D.N, lane = threadIdx.x;
    // one round of loads: the verdict, what to expect, and the first look at the counters
    const int plan_ok = W.plan_ok[r];
    const unsigned want = lane < N ? expect[(size_t)r * N + lane] : 0u;
    unsigned have = lane < N ? ld_relaxed(arrive + (size_t)r * N + lane) : 0u;
    if (!plan_ok) return;                           // step skipped: the receive kernel leaves on plan_ok too
    bool ok = true;
    for (long long spins = 0; !__all((int)(have - want) >= 0); ++spins) {      // wrap-safe, bounded
        if (spins >= D.spin_limit) { ok = false; break; }
        __builtin_amdgcn_s_sleep(64);
        if (lane < N) have = ld_relaxed(arrive + (size_t)r * N + lane);
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");     // pairs with the senders' release adds
    if (threadIdx.x == 0) {
        gate[r] = ok ? 1 : 0;
        if (!ok) latch_status(W.status, FL_STATUS_TIMEOUT);
    }
}

// ------------------------------------------------------------------ dispatch: unpack
// Receiver half at rank d.  A block takes a chunk of received rows, waits
// (bounded) for the arrival counters of the sources those rows came from, and
// writes every row once per local expert that wants it, at
//   base_x[d][local expert][source] + rank carried in the sidecar,
// which is the (expert, source rank, token) order of the grouped layout.
//
// FENCED (progressive mode): the kernel may have been started before any payload
// exists, on a grid that is a fraction of the machine, so a block walks many
// chunks.  It keeps the set of sources it has seen complete: a chunk whose
// sources are all in the set costs no poll; otherwise one wave polls the
// counters of ALL sources at once (one load per lane), waits until the chunk's
// own sources are complete, and invalidates the caches once, because it is about
// to rely on arrivals it had not seen before.  That is the whole visibility
// rule: payload and sidecar of a source are read only after its counter was
// seen complete and the caches were invalidated after that observation (a line
// fetched earlier, for a neighbouring row, may hold this source's bytes from
// before they landed; a line fetched later cannot).  The chunk's first payload
// loads are issued before its sidecars are decoded, so a chunk costs one memory
// round trip, not four.
template <bool FENCED, bool PRIVATE>   // PRIVATE: the receive buffer has private slots (P > 0)
__global__ __launch_bounds__(kCopyThreads) void dispatch_unpack_kernel(
    Dims D, Tables W, int rank_begin, char *__restrict__ expert_x,
    float *__restrict__ expert_scales, int *__restrict__ tokens_per_expert, int rows_per_block,
    const int *__restrict__ gate /* [N] or null: a gate kernel's verdict, 0 = its wait gave up */) {
    const int d = rank_begin + blockIdx.y, tid = threadIdx.x, N = D.N, El = D.El, K = D.K;
    __shared__ int off[FL_MAX_RANKS + 1];
    __shared__ int dst_rows[kMaxRowsPerBlock][FL_MAX_TOPK];
    __shared__ int dst_cnt[kMaxRowsPerBlock];
    __shared__ int src_phys[kMaxRowsPerBlock];      // with private slots: buffer row of each received row
    __shared__ int timed_out;
    __shared__ unsigned long long seen_pub;         // FENCED: wave 0 publishes the set of complete sources
    // first round of loads, all independent: the verdicts, the rows in use, the source offsets
    const int plan_ok = W.plan_ok[d], gate_ok = gate ? gate[d] : 1;
    const int total = W.recv_off[(size_t)d * (N + 1) + N];
    const int off_mine = tid <= N ? W.recv_off[(size_t)d * (N + 1) + tid] : 0;
    if (!plan_ok) return;
    if (!gate_ok) return;                           // the arrival wait timed out (status already latched)
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
    // grids are sized from capacities: blocks beyond the rows in use leave at once
    if ((int)blockIdx.x * rows_per_block >= total) return;
    if (tid <= N) off[tid] = off_mine;
    if (tid == 0) timed_out = 0;
    __syncthreads();
    const char *recv = W.bufB + (size_t)d * D.bufB_rank_bytes;
    const int nvec = (int)(D.Be / 16);
    const bool scales_as_vectors = D.scales_per_row > 0 && D.scales_per_row % 4 == 0;
    const int rowvec = nvec + (scales_as_vectors ? D.scales_per_row / 4 : 0);
    unsigned long long seen = 0;                    // FENCED: sources seen complete (same in every thread)
    unsigned my_expect = 0;                         // FENCED, wave 0: lane i holds what source i must deliver
    if (FENCED && tid < N) my_expect = W.expect_disp[(size_t)d * N + tid];
    // capacities are upper bounds, so the grid may be smaller than the rows in use
    for (int r0 = blockIdx.x * rows_per_block; r0 < total; r0 += gridDim.x * rows_per_block) {
        const int r1 = min(r0 + rows_per_block, total);
        const int s0 = seg_of(off, N, r0), s1 = seg_of(off, N, r1 - 1);
        if (FENCED) {
            const unsigned long long range = ((s1 - s0 == 63) ? ~0ull : ((1ull << (s1 - s0 + 1)) - 1)) << s0;
            if (tid < kWave) {
                if (range & ~seen) {                // uniform: every thread holds the same `seen`
                    long long spins = 0;
                    for (;;) {
                        bool ok = false;
                        if (tid < N) ok = (int)(ld_relaxed(W.arrive_disp + (size_t)d * N + tid) - my_expect) >= 0;
                        seen |= __ballot(ok);
                        if (!(range & ~seen)) break;
                        if (++spins > D.spin_limit) {
                            if (tid == 0) { timed_out = 1; latch_status(W.status, FL_STATUS_TIMEOUT); }
                            break;
                        }
                        __builtin_amdgcn_s_sleep(64);
                    }
                    acquire_payload<FENCED>();      // arrivals not relied on before: drop what the caches hold
                }
                if (tid == 0) seen_pub = seen;
            }
        } else if (!gate && tid < kWave) {          // behind a gate kernel the counters were seen complete
            if (!wave_wait_counters(W.arrive_disp + (size_t)d * N + s0,
                                    W.expect_disp + (size_t)d * N + s0, 0u, s1 - s0 + 1,
                                    D.spin_limit)) {
                if (tid == 0) { timed_out = 1; latch_status(W.status, FL_STATUS_TIMEOUT); }
            }
        }
        __syncthreads();
        if (timed_out) return;
        if (FENCED) seen = seen_pub;
        // e4m3: when the scales of a row are a whole number of 16-byte vectors they are
        // moved by the same loop (the vectors after the code bytes go to expert_scales)
        const int chunk = (r1 - r0) * rowvec;
        // U loads per thread in flight.  A full grid keeps the memory system busy with 4; the
        // capped grid of polling receivers has fewer waves per compute unit and needs 8.
        constexpr int U = FENCED ? 8 : 4;
        auto load_batch = [&](int b, v4u *val, int *row, int *col) {
#pragma unroll
            for (int i = 0; i < U; ++i) {
                const int v = b + i * kCopyThreads;
                if (v < chunk) {
                    row[i] = v / rowvec;
                    col[i] = v - row[i] * rowvec;
                    const int pr = PRIVATE ? src_phys[row[i]] : r0 + row[i];
                    val[i] = ld_stream((const v4u *)(recv + (size_t)pr * D.Bw) + col[i]);
                }
            }
        };
        auto plan_rows = [&]() {
            if (tid < r1 - r0) {               // plan of one received row: its expert-major rows
                const int r = r0 + tid;
                const int s = seg_of(off, N, r);
                int phys = r;
                if (PRIVATE) {
                    phys = recv_buffer_row(N, D.P, s, r - off[s], W.recv_shared_off[(size_t)d * N + s]);
                    src_phys[tid] = phys;
                }
                // entry k + 1 is fetched before entry k is looked at, so that it travels together
                // with the base row of entry k (most rows have one entry: two round trips, not three)
                const unsigned *meta = W.recv_meta + ((size_t)d * D.recv_rows + phys) * D.MW;
                int n = 0;
                unsigned m = meta[0];
                for (int k = 0; k < K; ++k) {
                    const unsigned m_next = k + 1 < K ? meta[k + 1] : kNoEntry;
                    if (m == kNoEntry) break;
                    const int j = (int)(m >> 24), i = (int)(m & 0xFFFFFFu);
                    dst_rows[tid][n++] = W.base_x[((size_t)d * El + j) * N + s] + i;
                    m = m_next;
                }
                dst_cnt[tid] = n;
            }
        };
        auto store_batch = [&](int b, const v4u *val, const int *row, const int *col) {
#pragma unroll
            for (int i = 0; i < U; ++i) {
                const int v = b + i * kCopyThreads;
                if (v < chunk) {
                    const int n = dst_cnt[row[i]];
                    for (int j = 0; j < n; ++j) {
                        const size_t dr = (size_t)dst_rows[row[i]][j];
                        if (col[i] < nvec)
                            st_stream((v4u *)(xd + dr * D.Be) + col[i], val[i]);
                        else
                            st_stream((v4u *)(expert_scales + ((size_t)d * D.expert_cap + dr) *
                                                                  D.scales_per_row) + (col[i] - nvec), val[i]);
                    }
                }
            }
        };
        if (FENCED && !PRIVATE) {
            // the first batch's loads go out before the sidecars are decoded: a chunk then
            // costs one memory round trip instead of three in a row (polling receivers run with
            // few waves per compute unit; with a full grid the extra registers cost more occupancy
            // than the shorter chain gains: 156 against 154 us)
            v4u val[U];
            int row[U], col[U];
            load_batch(tid, val, row, col);
            plan_rows();
            __syncthreads();
            store_batch(tid, val, row, col);
            for (int b = tid + U * kCopyThreads; b < chunk; b += U * kCopyThreads) {
                load_batch(b, val, row, col);
                store_batch(b, val, row, col);
            }
        } else {
            plan_rows();
            __syncthreads();
            for (int b = tid; b < chunk; b += U * kCopyThreads) {
                v4u val[U];
                int row[U], col[U];
                load_batch(b, val, row, col);
                store_batch(b, val, row, col);
            }
        }
        if (D.scales_per_row && !scales_as_vectors) {   // odd scale counts: element by element
            for (int r = r0; r < r1; ++r) {
                const int n = dst_cnt[r - r0];
                const int *dr = dst_rows[r - r0];
                const float *ssrc =
                    (const float *)(recv + (size_t)(PRIVATE ? src_phys[r - r0] : r) * D.Bw + D.Be);
                for (int v = tid; v < D.scales_per_row; v += kCopyThreads) {
                    const float val = ssrc[v];
                    for (int i = 0; i < n; ++i)
                        expert_scales[((size_t)d * D.expert_cap + dr[i]) * D.scales_per_row + v] = val;
                }
            }
        }
        __syncthreads();                       // the row plan in LDS is rewritten by the next chunk
    }
}

// ------------------------------------------------------------------ combine: pack
// Rank d gathers, for every source s, the rows of its experts that belong to s
// (contiguous per expert in the grouped layout) into one contiguous reply:
// combine-send row q of source s and local expert j comes from expert-major row
// base_x[d][j][s] + (q - cs_base[d][s][j]).
//
// PUSH: the rows go straight into the sources' combine receive buffers; FENCED as
// in the dispatch pack kernel (the block adds each row's units to
// arrive[source][this rank] itself).
template <bool PUSH, bool FENCED>
__global__ __launch_bounds__(kCopyThreads) void combine_pack_kernel(
    Dims D, Tables W, int rank_begin, const char *__restrict__ expert_y, int rows_per_block) {
    const int d = rank_begin + blockIdx.y, tid = threadIdx.x, N = D.N, El = D.El;
    __shared__ int off[FL_MAX_RANKS + 1];
    __shared__ int src_row[kMaxRowsPerBlock];
    __shared__ int2 push_to[kMaxRowsPerBlock];     // PUSH: (source rank, row of its combine receive buffer)
    if (!W.plan_ok[d]) return;
    const int nvec = (int)(D.Bc / 16);
    // with PUSH the rank's first block announces the replies (a rank without rows its empty ones)
    if (PUSH && (FENCED || (D.flags & FL_FLAG_STREAM_ORDERED)) && blockIdx.x == 0)
        announce_transfers(W.cs_off + (size_t)d * (N + 1), W.arrive_comb, (unsigned)nvec, d, N, tid, kCopyThreads,
                           FENCED);
    // grids are sized from capacities: blocks beyond the rows in use leave at once
    const int total = W.cs_off[(size_t)d * (N + 1) + N];
    if ((int)blockIdx.x * rows_per_block >= total) return;
    if (tid <= N) off[tid] = W.cs_off[(size_t)d * (N + 1) + tid];
    __syncthreads();
    const char *yd = expert_y + (size_t)d * D.expert_cap * D.Bc;
    // capacities are upper bounds, so the grid may be smaller than the rows in use
    for (int q0 = blockIdx.x * rows_per_block; q0 < total; q0 += gridDim.x * rows_per_block) {
        const int q1 = min(q0 + rows_per_block, total);
        if (tid < q1 - q0) {
            const int q = q0 + tid;
            const int s = seg_of(off, N, q);
            int first;                         // first reply row of (source s, local expert j)
            const int j = seg_of_short(W.cs_base + ((size_t)d * N + s) * El, El, q, &first);
            src_row[tid] = W.base_x[((size_t)d * El + j) * N + s] + (q - first);
            const int2 to = make_int2(s, W.comb_dst_off[(size_t)d * N + s] + (q - off[s]));
            if (PUSH) push_to[tid] = to;
            else W.fab_dst_comb[(size_t)d * D.expert_cap + q] = to;
        }
        __syncthreads();
        if (PUSH) {
            copy_rows_flat<kCopyThreads, FENCED>(
                q1 - q0, nvec, tid,
                [&](int r) { return yd + (size_t)src_row[r] * D.Bc; },
                [&](int r) {
                    return W.bufA + (size_t)push_to[r].x * D.bufA_rank_bytes + (size_t)push_to[r].y * D.Bc;
                });
            if (FENCED) {
                stores_done<FENCED>();
                __syncthreads();
                if (tid < q1 - q0)
                    add_counter(W.arrive_comb + (size_t)push_to[tid].x * N + d, (unsigned)nvec);
            }
        } else {
            char *out = W.bufB + (size_t)d * D.bufB_rank_bytes + (size_t)q0 * D.Bc;
            copy_rows_flat<kCopyThreads>(
                q1 - q0, nvec, tid,
                [&](int r) { return yd + (size_t)src_row[r] * D.Bc; },
                [&](int r) { return out + (size_t)r * D.Bc; });
        }
        __syncthreads();                       // the row plan is rewritten by the next chunk
    }
}

// acc[0..7] += wk * (the eight bf16 values of y), fused
__device__ inline void fma8(float *acc, float wk, v4u y) {
    acc[0] = fmaf(wk, bf16_lo(y.x), acc[0]); acc[1] = fmaf(wk, bf16_hi(y.x), acc[1]);
    acc[2] = fmaf(wk, bf16_lo(y.y), acc[2]); acc[3] = fmaf(wk, bf16_hi(y.y), acc[3]);
    acc[4] = fmaf(wk, bf16_lo(y.z), acc[4]); acc[5] = fmaf(wk, bf16_hi(y.z), acc[5]);
    acc[6] = fmaf(wk, bf16_lo(y.w), acc[6]); acc[7] = fmaf(wk, bf16_hi(y.w), acc[7]);
}

// ------------------------------------------------------------------ combine: pack with sender-side partial sums
// Section Comparison with DeepEP: tokens can be pre-accumulated on the sending
// side, which moves fewer rows at the price of a bf16 rounding between the two
// stages.  Rank d answers every row it received with ONE row: the fp32 fused
// multiply-add chain, in the order of the row's sidecar (ascending k), of
// weight * expert output over the token's experts on d, rounded to bf16.  The
// share of received row number i from source s goes back to row
// ret_off[d][s] + i of s's buffer, the row of s's send buffer the token copy
// left from, so s finds it through its own send_row table.
template <bool PUSH, bool FENCED>
__global__ __launch_bounds__(kCopyThreads) void combine_partial_pack_kernel(
    Dims D, Tables W, int rank_begin, const char *__restrict__ expert_y, int rows_per_block) {
    const int d = rank_begin + blockIdx.y, tid = threadIdx.x, N = D.N, El = D.El, K = D.K;
    __shared__ int off[FL_MAX_RANKS + 1];
    __shared__ int src_rows[kMaxRowsPerBlock][FL_MAX_TOPK];
    __shared__ float src_w[kMaxRowsPerBlock][FL_MAX_TOPK];
    __shared__ int src_cnt[kMaxRowsPerBlock];
    __shared__ int2 share_to[kMaxRowsPerBlock];
    if (!W.plan_ok[d]) return;
    const int nvec = (int)(D.Bc / 16);
    if (PUSH && (FENCED || (D.flags & FL_FLAG_STREAM_ORDERED)) && blockIdx.x == 0)   // as in combine_pack_kernel
        announce_transfers(W.recv_off + (size_t)d * (N + 1), W.arrive_comb, (unsigned)nvec, d, N, tid, kCopyThreads,
                           FENCED);
    const int total = W.recv_off[(size_t)d * (N + 1) + N];
    if ((int)blockIdx.x * rows_per_block >= total) return;
    if (tid <= N) off[tid] = W.recv_off[(size_t)d * (N + 1) + tid];
    __syncthreads();
    const char *yd = expert_y + (size_t)d * D.expert_cap * D.Bc;
    for (int r0 = blockIdx.x * rows_per_block; r0 < total; r0 += gridDim.x * rows_per_block) {
        const int r1 = min(r0 + rows_per_block, total);
        if (tid < r1 - r0) {
            const int r = r0 + tid;
            const int s = seg_of(off, N, r);
            const int i = r - off[s];
            const int phys = D.P ? recv_buffer_row(N, D.P, s, i, W.recv_shared_off[(size_t)d * N + s]) : r;
            const unsigned *meta = W.recv_meta + ((size_t)d * D.recv_rows + phys) * D.MW;
            int n = 0;
            for (int k = 0; k < K; ++k) {
                const unsigned m = meta[k];
                if (m == kNoEntry) break;
                src_rows[tid][n] = W.base_x[((size_t)d * El + (int)(m >> 24)) * N + s] + (int)(m & 0xFFFFFFu);
                src_w[tid][n] = __uint_as_float(meta[D.KM + k]);
                ++n;
            }
            src_cnt[tid] = n;
            const int2 to = make_int2(s, W.ret_off[(size_t)d * N + s] + i);
            share_to[tid] = to;
            if (!PUSH) W.fab_dst_comb[(size_t)d * D.expert_cap + r] = to;
        }
        __syncthreads();
        const int chunk = (r1 - r0) * nvec;
        for (int b = tid; b < chunk; b += 4 * kCopyThreads) {
            v4u y0[4];
            int row[4], col[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {          // the first expert row of four items in flight
                const int v = b + u * kCopyThreads;
                if (v < chunk) {
                    row[u] = v / nvec;
                    col[u] = v - row[u] * nvec;
                    y0[u] = ld_stream((const v4u *)(yd + (size_t)src_rows[row[u]][0] * D.Bc) + col[u]);
                }
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int v = b + u * kCopyThreads;
                if (v >= chunk) continue;
                float acc[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[e] = 0.f;
                fma8(acc, src_w[row[u]][0], y0[u]);
                const int n = src_cnt[row[u]];
                for (int k = 1; k < n; ++k)
                    fma8(acc, src_w[row[u]][k],
                         ld_stream((const v4u *)(yd + (size_t)src_rows[row[u]][k] * D.Bc) + col[u]));
                v4u o;
                o.x = pack_bf16x2(acc[0], acc[1]); o.y = pack_bf16x2(acc[2], acc[3]);
                o.z = pack_bf16x2(acc[4], acc[5]); o.w = pack_bf16x2(acc[6], acc[7]);
                char *dst = PUSH ? W.bufA + (size_t)share_to[row[u]].x * D.bufA_rank_bytes +
                                       (size_t)share_to[row[u]].y * D.Bc
                                 : W.bufB + (size_t)d * D.bufB_rank_bytes + (size_t)(r0 + row[u]) * D.Bc;
                st_payload<PUSH && FENCED, true>((v4u *)dst + col[u], o);
            }
        }
        if (PUSH && FENCED) {
            stores_done<FENCED>();
            __syncthreads();
            if (tid < r1 - r0)
                add_counter(W.arrive_comb + (size_t)share_to[tid].x * N + d, (unsigned)nvec);
        }
        __syncthreads();                       // the row plan is rewritten by the next chunk
    }
}

// ------------------------------------------------------------------ combine: reduce
// One block per token (s, t):
//   out[s][t] = bf16( sum_k w[k] * float(row comb_pos[s][t][k]) ), fp32 fused
// multiply-add, k ascending, one final rounding.

// KT = number of row loads issued together (then consumed in k order); the sum
// itself always runs k = 0..K-1.
template <int KT>
__device__ inline void reduce_row(const char *__restrict__ recv, const int *pos, const float *w,
                                  int K, long long Bc, int v0, int nvec, v4u *__restrict__ out, int tid) {
    for (int v = v0 + tid; v < nvec; v += (int)blockDim.x) {
        float acc[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = 0.f;
        int k0 = 0;
        for (; k0 + KT <= K; k0 += KT) {
            v4u y[KT];
#pragma unroll
            for (int k = 0; k < KT; ++k)
                y[k] = ld_stream((const v4u *)(recv + (size_t)pos[k0 + k] * Bc) + v);
#pragma unroll
            for (int k = 0; k < KT; ++k) fma8(acc, w[k0 + k], y[k]);
        }
        for (; k0 < K; ++k0)
            fma8(acc, w[k0], ld_stream((const v4u *)(recv + (size_t)pos[k0] * Bc) + v));
        v4u o;
        o.x = pack_bf16x2(acc[0], acc[1]); o.y = pack_bf16x2(acc[2], acc[3]);
        o.z = pack_bf16x2(acc[4], acc[5]); o.w = pack_bf16x2(acc[6], acc[7]);
        st_stream(out + v, o);
    }
}

// The same sum for a row count only known on the device (partial sums: one row per
// distinct expert rank of the token): batches of up to 8 loads, predicated.
__device__ inline void reduce_row_counted(const char *__restrict__ recv, const int *pos,
                                          const float *w, int n, long long Bc, int v0, int nvec,
                                          v4u *__restrict__ out, int tid) {
    for (int v = v0 + tid; v < nvec; v += (int)blockDim.x) {
        float acc[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = 0.f;
        for (int k0 = 0; k0 < n; k0 += 8) {
            v4u y[8];
#pragma unroll
            for (int k = 0; k < 8; ++k)
                if (k0 + k < n) y[k] = ld_stream((const v4u *)(recv + (size_t)pos[k0 + k] * Bc) + v);
#pragma unroll
            for (int k = 0; k < 8; ++k)
                if (k0 + k < n) fma8(acc, w[k0 + k], y[k]);
        }
        v4u o;
        o.x = pack_bf16x2(acc[0], acc[1]); o.y = pack_bf16x2(acc[2], acc[3]);
        o.z = pack_bf16x2(acc[4], acc[5]); o.w = pack_bf16x2(acc[6], acc[7]);
        st_stream(out + v, o);
    }
}

// The block has min(1024, vectors per row rounded up to a wave) threads, so a
// 7168-wide row is one vector per thread and all K loads of a thread are in
// flight at once.
constexpr int kReduceMaxThreads = 1024;
//
// PARTIAL (sender-side partial sums): the token's rows are the shares of its
// distinct expert ranks, found at send_row[s][t][k] for every k that is the first
// of its rank; they are added in that order in fp32 (a fused multiply-add with
// weight 1 is an exact add), the weights having been applied on the expert ranks.
template <bool FENCED, bool PARTIAL>
__global__ __launch_bounds__(kReduceMaxThreads, 7) void combine_reduce_kernel(
    Dims D, Tables W, int rank_begin, const float *__restrict__ weights, char *__restrict__ out,
    const int *__restrict__ num_tokens, const int *__restrict__ gate /* as in dispatch_unpack_kernel */,
    int parts /* workgroups that share one token, each taking a slice of the row */) {
    const int s = rank_begin + blockIdx.y, tid = threadIdx.x, N = D.N, K = D.K;
    const int t0 = blockIdx.x / parts, part = blockIdx.x - t0 * parts, t_step = gridDim.x / parts;
    // two sets of positions and weights: while the block sums one token, wave 1 already
    // fetches the next one's (a block only walks several tokens when the grid is smaller
    // than the token count, as it is for the polling receivers of progressive mode)
    __shared__ int pos[2][FL_MAX_TOPK];
    __shared__ float w[2][FL_MAX_TOPK];
    __shared__ int n_shares[2];
    __shared__ int timed_out;
    // every load the block needs before its rows go out in ONE round: the verdicts, the token
    // count and (wave 1) the first token's positions and weights, which exist for every t < T
    const int plan_ok = W.plan_ok[s], gate_ok = gate ? gate[s] : 1, Ts = num_tokens[s];
    const bool fetcher = tid >= kWave && tid < 2 * kWave;     // wave 1
    const int k = tid - kWave;
    int pf_pos = -1;
    float pf_w = 1.0f;
    // token t's row positions (and weights): the load, then, once it has landed, the LDS copy
    auto fetch = [&](int t) {
        if (k >= K) { pf_pos = -1; return; }
        const size_t pair = ((size_t)s * D.T + t) * K + k;
        if (PARTIAL) pf_pos = W.send_row[pair];               // share rows: first k of each expert rank
        else { pf_pos = W.comb_pos[pair]; pf_w = weights[pair]; }
    };
    auto publish = [&](int buf) {
        if (PARTIAL) {                                        // compacted in k order, weight 1: an exact add
            const unsigned long long have = __ballot(pf_pos >= 0);
            if (pf_pos >= 0) {
                const int at = __popcll(have & ((1ull << k) - 1));
                pos[buf][at] = pf_pos;
                w[buf][at] = 1.0f;
            }
            if (k == 0) n_shares[buf] = __popcll(have);
        } else if (k < K) {
            pos[buf][k] = pf_pos;
            w[buf][k] = pf_w;
        }
    };
    if (fetcher) fetch(t0);
    if (!plan_ok || !gate_ok || t0 >= Ts) return;
    if (tid == 0) timed_out = 0;               // wave 0 itself is the only one that may raise it
    if (fetcher) publish(0);
    // behind a gate kernel the counters were already seen complete, for every source of this rank
    if (!gate && tid < kWave) {
        if (!wave_wait_counters(W.arrive_comb + (size_t)s * N, W.expect_comb + (size_t)s * N, 0u, N,
                                D.spin_limit)) {
            if (tid == 0) { timed_out = 1; latch_status(W.status, FL_STATUS_TIMEOUT); }
        }
        acquire_payload<FENCED>();
    }
    __syncthreads();
    if (timed_out) return;
    const char *recv = W.bufA + (size_t)s * D.bufA_rank_bytes;
    const int nvec_row = (int)(D.Bc / 16);
    const int per = (nvec_row + parts - 1) / parts;            // this block's slice: [v0, nvec)
    const int v0 = part * per, nvec = min(v0 + per, nvec_row);
    const int kt = D.tune_reduce ? D.tune_reduce : K;
    // one token per block unless the grid was made smaller than the token count
    int cur = 0;
    for (int t = t0; t < Ts; t += t_step) {
        const int next = t + t_step;
        if (fetcher && next < Ts) fetch(next);                // in flight while the rows are summed
        v4u *o = (v4u *)(out + ((size_t)s * D.T + t) * D.Bc);
        if (PARTIAL) reduce_row_counted(recv, pos[cur], w[cur], n_shares[cur], D.Bc, v0, nvec, o, tid);
        else if (kt >= 8) reduce_row<8>(recv, pos[cur], w[cur], K, D.Bc, v0, nvec, o, tid);
        else if (kt >= 4) reduce_row<4>(recv, pos[cur], w[cur], K, D.Bc, v0, nvec, o, tid);
        else if (kt >= 2) reduce_row<2>(recv, pos[cur], w[cur], K, D.Bc, v0, nvec, o, tid);
        else reduce_row<1>(recv, pos[cur], w[cur], K, D.Bc, v0, nvec, o, tid);
        if (next >= Ts) break;
        if (fetcher) publish(cur ^ 1);
        __syncthreads();                       // the other set is complete; this one may be rewritten
        cur ^= 1;
    }
}

// ------------------------------------------------------------------ diagnostic copy
// Plain linear copy, fill and read: the machine's ceilings for a stream of 16-byte
// accesses, each in the launch shape that measured fastest for it on this part (1 GiB,
// non-temporal accesses).  Workgroups that move little and end at once do best:
//   copy  64 threads x 4 vectors (4 KB per workgroup) 6 450 GB/s of read + write traffic;
//         256 x 1: 6 340; 256 x 4 (16 KB): 5 930; 1024 x 4 (64 KB): 5 290
//   fill  256 x 1 (4 KB) 6 790 GB/s; 128 x 2: 6 490; 64 x 4: 6 320; 256 x 4 (16 KB): 6 000;
//         256 x 16 (64 KB): 4 940
//   read  flat at 7 000 - 7 100 GB/s from 2 KB to 32 KB per workgroup, 1024 x 1: 7 200 - 7 500
// THREADS threads take U vectors each, all loads before the stores.
template <int THREADS, int U>
__global__ __launch_bounds__(THREADS) void plain_copy_kernel(v4u *__restrict__ dst, const v4u *__restrict__ src,
                                                             size_t nvec) {
    const size_t base = (size_t)blockIdx.x * THREADS * U + threadIdx.x;
    v4u r[U];
#pragma unroll
    for (int i = 0; i < U; ++i)
        if (base + (size_t)i * THREADS < nvec) r[i] = ld_stream(src + base + (size_t)i * THREADS);
#pragma unroll
    for (int i = 0; i < U; ++i)
        if (base + (size_t)i * THREADS < nvec) st_stream(dst + base + (size_t)i * THREADS, r[i]);
}

// Write-only and read-only companions: the two one-directional ceilings, against which
// kernels that mostly write (dispatch pack) or mostly read (combine reduce) are judged.
template <int THREADS, int U>
__global__ __launch_bounds__(THREADS) void plain_fill_kernel(v4u *__restrict__ dst, size_t nvec, unsigned value) {
    const size_t base = (size_t)blockIdx.x * THREADS * U + threadIdx.x;
    const v4u v = {value, value, value, value};
#pragma unroll
    for (int i = 0; i < U; ++i)
        if (base + (size_t)i * THREADS < nvec) st_stream(dst + base + (size_t)i * THREADS, v);
}

template <int THREADS, int U>
__global__ __launch_bounds__(THREADS) void plain_read_kernel(const v4u *__restrict__ src, size_t nvec,
                                                             unsigned *__restrict__ sink) {
    const size_t base = (size_t)blockIdx.x * THREADS * U + threadIdx.x;
    v4u r[U] = {};
#pragma unroll
    for (int i = 0; i < U; ++i)
        if (base + (size_t)i * THREADS < nvec) r[i] = ld_stream(src + base + (size_t)i * THREADS);
    unsigned x = 0;
#pragma unroll
    for (int i = 0; i < U; ++i) x ^= r[i].x ^ r[i].y ^ r[i].z ^ r[i].w;
    if (x == 0x9E3779B9u) *sink = x;      // keeps the loads alive; practically never taken
}

}  // namespace flmoe
