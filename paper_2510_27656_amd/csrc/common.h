// Shared device-side definitions of the flmoe kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/flmoe.h"

namespace flmoe {

constexpr int kWave = 64;

// Shapes and strides of one context; passed to every kernel by value.
struct Dims {
    int N, E, El, T, K, H;
    int dtype, align, flags;
    int TT;               // tokens per LDS tile of the counting blocks (multiple of 32)
    int route_len;        // ints one rank pushes to every peer: C[E] | M[N] | comb_off[N] | valid
    int scales_per_row;   // 0 or H/128
    long long recv_cap, expert_cap, send_cap;   // rows per rank
    int P;                // private rows per (source, destination) at the head of a receive buffer
    long long recv_rows;  // physical rows of a dispatch receive buffer: N*P private + recv_cap shared
    long long Bx, Bw, Be, Bc;                   // row bytes: input, wire, expert_x, combine
    long long bufA_rank_bytes, bufB_rank_bytes;
    long long spin_limit;
    int KM;               // sidecar entries per row: K rounded up to a multiple of 4
    int MW;               // words per sidecar row: KM, or 2*KM when the routing weights travel too
    int tune_rows;        // rows per block of the copy kernels (0 = by row size)
    int tune_reduce;      // loads in flight per thread in the reduce kernel (0 = all K)
    int tune_waves;       // waves per row in the fabric kernel (0 = by row size)
    int tune_slices;      // blocks per token in the pack kernel (0 = by row size)
    int tune_stream_mb;   // fabric uses streaming stores when a launch may write more than this many MiB
    int tune_grid_pct;    // row-kernel grids cover this percentage of the rows uniform routing would
                          // bring (0 = the whole capacity); kernels loop over whatever is beyond
    long long typ_recv_rows, typ_pair_rows;   // per rank, under uniform routing: received rows, pairs
    int tune_parts;       // workgroups per token in the reduce kernel (0 = by row size)
    int tune_order;       // test switch: order in which the fabric kernel takes a sender's destinations
    int tune_cap8;        // progressive receivers: eighths of the machine's block slots their grids may take
};

// Row of a dispatch receive buffer that holds the i-th row source s sent to this
// rank: the first P rows of every source have fixed private slots at the head of
// the buffer (known without any exchange), later rows are packed into the shared
// range behind them in source order (section MoE Dispatch/Combine, figure
// "Dispatch into private and contiguous buffers").
__host__ __device__ inline int recv_buffer_row(int N, int P, int s, int i, int shared_start) {
    return i < P ? s * P + i : N * P + shared_start + (i - P);
}

// Device pointers into the caller's workspace.
struct Tables {
    int *status;
    unsigned *epoch_route;                                    // [N] layout calls of each rank
    unsigned *arrive_route;                                   // [N dst][N src] route records received
    // Payload counters, monotone: a completed transfer adds its payload in 16-byte units
    // plus one (default: by the announce kernel behind the payload kernels; stream-ordered
    // callers: by one wave of the last payload kernel; progressive mode: the units by every
    // copying wave); expect_* is advanced by the receiver's own planning block from the
    // counts it was sent, so a receiver waits for arrive >= expect per source.
    unsigned *arrive_disp, *arrive_comb;                      // [N dst][N src]
    unsigned *expect_disp, *expect_comb;                      // [N dst][N src]
    int *routes;          // [N receiver][N source][route_len]
    // written by the source side of the layout step
    int *C;               // [N][E]
    int *M;               // [N][N]
    int *send_off;        // [N][N+1]
    int *comb_off;        // [N][N+1]
    int *send_row;        // [N][T][K]  row in the send buffer for the first slot of each destination, else -1
    unsigned *pair_meta;  // [N][T][K]  (local expert << 24) | rank of the token among the source's tokens of that expert
    int *comb_pos;        // [N][T][K]
    // written by the receiving side of the layout step
    int *G;               // [N][El]
    int *expert_off;      // [N][El+1]
    int *recv_off;        // [N][N+1]         received rows of lower sources (the order unpack walks)
    int *recv_shared_off; // [N dst][N src]   shared-range rows of lower sources: sum of max(M - P, 0)
    int *dst_off;         // [N src][N dst]   the same number as seen by the sender: where src's rows
                          //                  beyond its private slots start in dst's shared range
    int *comb_dst_off;    // [N d][N s]       row in s's combine receive buffer where d's reply starts
    int *ret_off;         // [N d][N s]       partial sums: row in s's buffer where d's shares start,
                          //                  = rows s sent to lower ranks, so a share returns to the
                          //                  row of s's send buffer its token copy left from
    int *base_x;          // [N][El][N]       first expert-major row of (local expert, source)
    int *cs_base;         // [N][N][El]       first combine-send row of (source, local expert)
    int *cs_off;          // [N][N+1]         first combine-send row of each source
    int *plan_ok;         // [N]
    int *gate_disp;       // [N] default mode: 1 once the gate kernel saw every source's dispatch payload complete
    int *gate_comb;       // [N] the same for the combine replies
    unsigned *send_meta;  // [N][send_cap][MW]
    unsigned *recv_meta;  // [N][recv_rows][MW]
    int2 *fab_dst_disp;   // [N][send_cap]    (destination rank, row there) of every send row
    int2 *fab_dst_comb;   // [N][expert_cap]  same for the combine send rows
    char *bufA;           // [N][bufA_rank_bytes]  dispatch send / combine receive
    char *bufB;           // [N][bufB_rank_bytes]  dispatch receive / combine send
};

constexpr unsigned kNoEntry = 0xFFFFFFFFu;

// ---------------------------------------------------------------- atomics
// FENCED names the progressive mode, in which senders and receivers overlap in time
// inside their kernels: every sending wave reports the units it delivered and the
// receive kernels poll.  On gfx950 each XCD has its own L2, so a payload only
// becomes visible to a receiver on another XCD once it has left the sender's L2.
// An agent-scope release fence would write back the whole L2 (measured: 5x to 25x
// slower fabric kernel, depending on how many waves fence).  Instead the sender
// writes the payload with device-scope stores (sc1: written through to memory),
// waits until its own stores are acknowledged, and only then updates the counter;
// the receiver polls the counter with device-scope loads and, once it has arrived,
// invalidates its caches (agent-scope acquire) before touching the payload.
// FENCED = false covers the other two modes, where whole kernels order payload and
// counters: the announce kernel behind the payload kernels (default), or the
// caller's stream order (FL_FLAG_STREAM_ORDERED); payload stores are then ordinary
// stores and the in-kernel counter accesses relaxed atomics.
__device__ inline unsigned ld_relaxed(const unsigned *p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// The result is never used, so the hardware atomic does not return a value and
// the wave does not wait for it.
__device__ inline void add_counter(unsigned *p, unsigned v) {
    (void)__hip_atomic_fetch_add(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// After a wave's last payload store and before its add_counter: in progressive mode,
// wait until every store of this wave (including the device-scope ones issued
// from inline assembly, which the compiler does not count) has been acknowledged.
template <bool FENCED>
__device__ inline void stores_done() {
    if (FENCED) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }
}
template <bool FENCED>
__device__ inline void acquire_payload() {
    if (FENCED) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
}
template <bool FENCED>
__device__ inline void st_word(int *p, int v) {        // small table entries pushed to a peer
    if (FENCED) __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    else *p = v;
}
__device__ inline void latch_status(int *status, int bit) {
    __hip_atomic_fetch_or(status, bit, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Bounded wait of one wavefront: lane i (< n) polls ctr[i] until it has reached
// its expectation (wrap-safe comparison; `expect` is either one value for all or,
// with expect_arr, one per counter).  Returns true when all n counters arrived,
// false when the poll budget ran out.  Every lane of the wave must call it.
// SLEEP: pause between polls in units of 64 clocks.  Payload waits may last as long
// as a copy kernel and must not crowd out the senders they wait for (about 2 us);
// the route exchange inside the layout kernel is a few microseconds long (short pause).
template <int SLEEP = 64>
__device__ inline bool wave_wait_counters(const unsigned *ctr, const unsigned *expect_arr,
                                          unsigned expect, int n, long long spin_limit) {
    const int lane = threadIdx.x & (kWave - 1);
    for (int base = 0; base < n; base += kWave) {
        const int i = base + lane;
        long long spins = 0;
        if (expect_arr && i < n) expect = expect_arr[i];
        for (;;) {
            bool ok = true;
            if (i < n) ok = (int)(ld_relaxed(ctr + i) - expect) >= 0;
            if (__all(ok)) break;
            if (++spins > spin_limit) return false;
            __builtin_amdgcn_s_sleep(SLEEP);
        }
    }
    return true;
}

// ---------------------------------------------------------------- scans / search
__device__ inline int wave_incl_scan(int v) {
    const int lane = threadIdx.x & (kWave - 1);
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
        int n = __shfl_up(v, o);
        if (lane >= o) v += n;
    }
    return v;
}

// Exclusive scan over the block (one value per thread, blockDim <= 1024).
// tmp: LDS int[17].  *total receives the block sum.  Contains barriers.
__device__ inline int block_excl_scan(int v, int *tmp, int *total) {
    const int lane = threadIdx.x & (kWave - 1), wid = threadIdx.x / kWave;
    const int nw = (blockDim.x + kWave - 1) / kWave;
    int inc = wave_incl_scan(v);
    __syncthreads();
    if (lane == kWave - 1) tmp[wid] = inc;
    __syncthreads();
    if (threadIdx.x == 0) {
        int acc = 0;
        for (int w = 0; w < nw; ++w) { int t = tmp[w]; tmp[w] = acc; acc += t; }
        tmp[16] = acc;
    }
    __syncthreads();
    *total = tmp[16];
    return inc - v + tmp[wid];
}

// Largest i in [0, n) with off[i] <= x; needs off[0] <= x.  With equal
// neighbours (empty segments) this is the segment that really contains x.
__device__ inline int seg_of(const int *off, int n, int x) {
    int lo = 0, hi = n;
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (off[mid] <= x) lo = mid; else hi = mid;
    }
    return lo;
}

// seg_of for a short table in global memory: all entries are fetched at once (one
// round trip instead of one per halving step); *start receives off[result].
__device__ inline int seg_of_short(const int *off, int n, int x, int *start) {
    if (n > 16) {
        const int j = seg_of(off, n, x);
        *start = off[j];
        return j;
    }
    int c[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) c[i] = i < n ? off[i] : 0x7fffffff;
    int j = 0, cj = c[0];
#pragma unroll
    for (int i = 1; i < 16; ++i)
        if (c[i] <= x) { j = i; cj = c[i]; }
    *start = cj;
    return j;
}

// ---------------------------------------------------------------- row copies
// 16-byte streaming accesses.  The payload of every copy kernel is touched once
// per kernel, so loads and stores carry the non-temporal hint; on this part a
// plain copy with these hints and four independent loads per thread in flight
// measured fastest (more loads in flight per CU than that overruns the L2).
typedef unsigned v4u __attribute__((ext_vector_type(4)));
__device__ inline v4u ld_stream(const v4u *p) { return __builtin_nontemporal_load(p); }
__device__ inline void st_stream(v4u *p, v4u v) { __builtin_nontemporal_store(v, p); }
// Fabric payload store.  Progressive mode: device scope, written through to memory so
// that another XCD can see it without an L2 write-back.  Otherwise: an
// ordinary cached store while the receive buffers are small enough for the caches
// to absorb a good part of them (measured: 17 % faster fabric kernel at the decode
// shape, the kernels after it 4 % slower, the step 5 % faster), a streaming store
// when they are far larger than the caches (at the prefill shape cached stores were
// 4 % slower).
template <bool FENCED, bool STREAMING>
__device__ inline void st_payload(v4u *p, v4u v) {
    if (FENCED) asm volatile("global_store_dwordx4 %0, %1, off sc1" ::"v"(p), "v"(v) : "memory");
    else if (STREAMING) __builtin_nontemporal_store(v, p);
    else *p = v;
}

// A block copies `nrows` rows of `nvec` vectors each; vector v of the chunk lies
// in row v / nvec.  src_of(row) / dst_of(row) return the row's byte address.
// All loads of a batch are issued before its stores.
template <int NT, bool FENCED = false, class SrcFn, class DstFn>
__device__ inline void copy_rows_flat(int nrows, int nvec, int tid, SrcFn src_of, DstFn dst_of) {
    if (nrows == 1) {                          // one row per block: addresses are uniform
        const v4u *s = (const v4u *)src_of(0);
        v4u *d = (v4u *)dst_of(0);
        for (int b = tid; b < nvec; b += 4 * NT) {
            v4u r[4];
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (b + i * NT < nvec) r[i] = ld_stream(s + b + i * NT);
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (b + i * NT < nvec) st_payload<FENCED, true>(d + b + i * NT, r[i]);
        }
        return;
    }
    const int total = nrows * nvec;
    for (int b = tid; b < total; b += 4 * NT) {
        v4u r[4];
        int row[4], col[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int v = b + i * NT;
            if (v < total) {
                row[i] = v / nvec;
                col[i] = v - row[i] * nvec;
                r[i] = ld_stream((const v4u *)src_of(row[i]) + col[i]);
            }
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int v = b + i * NT;
            if (v < total) st_payload<FENCED, true>((v4u *)dst_of(row[i]) + col[i], r[i]);
        }
    }
}

// ---------------------------------------------------------------- bf16
__device__ inline float bf16_lo(unsigned u) { return __uint_as_float(u << 16); }
__device__ inline float bf16_hi(unsigned u) { return __uint_as_float(u & 0xffff0000u); }
__device__ inline unsigned f32_to_bf16_bits(float f) {
    unsigned u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;   // NaN stays a quiet NaN
    u += 0x7fffu + ((u >> 16) & 1u);                                  // ties to even
    return u >> 16;
}
__device__ inline unsigned pack_bf16x2(float lo, float hi) {
    return f32_to_bf16_bits(lo) | (f32_to_bf16_bits(hi) << 16);
}

}  // namespace flmoe
