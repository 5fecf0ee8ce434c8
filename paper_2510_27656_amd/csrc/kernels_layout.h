// Layout step: counting, deterministic ranks, route exchange, offset tables.
//
// Paper, section MoE Dispatch/Combine: the dispatch kernel first counts the
// tokens sent to each expert in shared memory (Dispatch); all peers exchange
// these per-expert counts to determine a unique range in each contiguous receive
// buffer (Architecture).  The paper computes the ranges on a host proxy; here
// both halves run on the device.
#pragma once
#include "common.h"

namespace flmoe {

constexpr int kRouteThreads = 1024;
constexpr int kPlanThreads = 1024;

// Words per row of the LDS bit matrices: the words in use, padded to an odd
// number so that rows do not all start in the same bank.
__host__ __device__ inline int route_row_stride(int TT) { return (TT / 32) | 1; }

__host__ __device__ inline size_t route_count_lds_bytes(int E, int N, int TT) {
    size_t rows = (size_t)E + N;
    return rows * route_row_stride(TT) * 2 * sizeof(unsigned) + rows * 4 * sizeof(int) +
           32 * sizeof(int);
}

// One block per source rank s.
//
// For every tile of TT tokens the block keeps two LDS bit matrices: row e of the
// first has bit t set when token t lists expert e, row d of the second when any
// of token t's experts lives on rank d (OR-ing makes the per-destination
// de-duplication free and the result independent of thread order).  The rank of
// token t among the tokens that hit the same row, in token order, is then
//     rows_before_tile + popcount prefix of the row's words + popcount of the
//     bits below t in its word
// which is the stable counting-sort position the canonical (source rank, token
// index) order needs, with no ticket atomics.
//
// Pass 1 counts (per row totals over all tiles), one block scan over the E + N
// totals turns them into offsets, pass 2 rebuilds each tile's bits (kept from
// pass 1 when there is a single tile) and writes every pair's final positions.
//
// Outputs for rank s: C[s][.], M[s][.], send_off[s][.], comb_off[s][.], per pair
// send_row / pair_meta / comb_pos; the route record (C | M | comb_off | valid) is
// pushed into every peer's routes[peer][s] and arrive_route[peer][s] is bumped.
__device__ __forceinline__ void route_count_block(const Dims &D, const Tables &W, int s,
                                                  const int *__restrict__ indices,
                                                  const int *__restrict__ num_tokens, unsigned *lds) {
    const int tid = threadIdx.x;
    const int E = D.E, N = D.N, El = D.El, K = D.K;
    const int rows = E + N;
    const int Wn = D.TT / 32;                              // words in use per row
    const int Wd = route_row_stride(D.TT);                 // row stride in words
    unsigned *bits = lds;                                  // [rows][Wd]
    unsigned *pre = bits + (size_t)rows * Wd;              // [rows][Wd] popcount prefix inside the tile
    int *count = (int *)(pre + (size_t)rows * Wd);         // [rows] hits over all tiles (C | M)
    int *start = count + rows;                             // [rows] exclusive scan of count
    int *base = start + rows;                              // [rows] hits in the tiles before the current one
    int *total_hits = base + rows;                         // [rows] copy of the totals (pass 2 reuses count)
    int *scan_tmp = total_hits + rows;                     // [32]
    __shared__ int bad;

    int Ts = num_tokens[s];
    if (tid == 0) bad = (Ts < 0 || Ts > D.T) ? 1 : 0;
    Ts = max(0, min(Ts, D.T));
    const int ntiles = (Ts + D.TT - 1) / D.TT;
    for (int r = tid; r < rows; r += kRouteThreads) { count[r] = 0; base[r] = 0; }
    const int *idx_s = indices + (size_t)s * D.T * K;

    // bits and in-tile popcount prefixes of one tile; returns each row's hits in tile_hits
    auto fill_tile = [&](int t0, int nt, int *tile_hits, bool accumulate) {
        for (int i = tid; i < rows * Wd; i += kRouteThreads) bits[i] = 0;
        __syncthreads();
        for (int p = tid; p < nt * K; p += kRouteThreads) {
            const int tl = p / K;
            const int e = idx_s[(size_t)t0 * K + p];
            if (e < 0 || e >= E) { bad = 1; continue; }
            const unsigned bit = 1u << (tl & 31);
            const unsigned old = atomicOr(&bits[(size_t)e * Wd + (tl >> 5)], bit);
            if (old & bit) bad = 1;                        // same expert twice in one token
            atomicOr(&bits[(size_t)(E + e / El) * Wd + (tl >> 5)], bit);
        }
        __syncthreads();
        for (int r = tid; r < rows; r += kRouteThreads) {
            int run = 0;
            for (int w = 0; w < Wn; ++w) {
                pre[(size_t)r * Wd + w] = run;
                run += __popc(bits[(size_t)r * Wd + w]);
            }
            tile_hits[r] = accumulate ? tile_hits[r] + run : run;
        }
        __syncthreads();
    };

    // pass 1: totals over all tiles
    __syncthreads();
    for (int tile = 0; tile < ntiles; ++tile) {
        const int t0 = tile * D.TT;
        fill_tile(t0, min(D.TT, Ts - t0), count, true);
    }

    // one exclusive scan over the E + N totals (two slots per thread)
    {
        const int a = 2 * tid < rows ? count[2 * tid] : 0;
        const int b = 2 * tid + 1 < rows ? count[2 * tid + 1] : 0;
        int total;
        const int ex = block_excl_scan(a + b, scan_tmp, &total);
        if (2 * tid < rows) { start[2 * tid] = ex; total_hits[2 * tid] = a; }
        if (2 * tid + 1 < rows) { start[2 * tid + 1] = ex + a; total_hits[2 * tid + 1] = b; }
    }
    __syncthreads();
    // start[e] = first combine-receive row of expert e; start[E + d] = pairs + send_off[d]
    const int pairs_total = start[E];
    if (tid < E) W.C[(size_t)s * E + tid] = count[tid];
    if (tid < N) {
        W.M[(size_t)s * N + tid] = count[E + tid];
        W.send_off[(size_t)s * (N + 1) + tid] = start[E + tid] - pairs_total;
        W.comb_off[(size_t)s * (N + 1) + tid] = start[tid * El];
    }
    if (tid == 0) {
        W.send_off[(size_t)s * (N + 1) + N] = start[E + N - 1] + count[E + N - 1] - pairs_total;
        W.comb_off[(size_t)s * (N + 1) + N] = pairs_total;
    }

    // Everything a peer needs is known now (pass 1 saw every index, so `bad` is final):
    // the record goes out before pass 2, whose per-pair tables only this rank's later
    // kernels read, so the peers' planning overlaps with it.
    const int valid = bad ? 0 : 1;
    if (bad && tid == 0) latch_status(W.status, FL_STATUS_BAD_INDEX);

    // Route exchange: push this rank's record (C | M | comb_off | valid, all still in
    // LDS) into every peer's table, then notify.
    const int RL = D.route_len;
    for (int i = tid; i < N * RL; i += kRouteThreads) {
        const int peer = i / RL, f = i - peer * RL;
        int v;
        if (f < E + N) v = total_hits[f];
        else if (f < E + 2 * N) v = start[(f - E - N) * El];
        else v = valid;
        st_word<true>(&W.routes[((size_t)peer * N + s) * RL + f], v);
    }
    stores_done<true>();
    __syncthreads();
    if (tid < N) add_counter(W.arrive_route + (size_t)tid * N + s, 1u);

    // pass 2: final position of every pair
    for (int tile = 0; tile < ntiles; ++tile) {
        const int t0 = tile * D.TT, nt = min(D.TT, Ts - t0);
        if (ntiles > 1) fill_tile(t0, nt, count, false);   // count[] now holds this tile's hits
        for (int p = tid; p < nt * K; p += kRouteThreads) {
            const int tl = p / K, k = p - tl * K;
            const size_t g = (size_t)t0 * K + p;
            const int e = idx_s[g];
            if (e < 0 || e >= E) continue;
            const int d = e / El;
            const unsigned below = (1u << (tl & 31)) - 1u;
            const int w = tl >> 5;
            const int re = e, rd = E + d;
            const int rank_e =
                base[re] + pre[(size_t)re * Wd + w] + __popc(bits[(size_t)re * Wd + w] & below);
            const int rank_d =
                base[rd] + pre[(size_t)rd * Wd + w] + __popc(bits[(size_t)rd * Wd + w] & below);
            // first slot of this token bound for rank d?  The token's earlier ids are fetched
            // together (predicated, independent loads) rather than one per loop turn.
            int before[FL_MAX_TOPK];
#pragma unroll
            for (int k2 = 0; k2 < FL_MAX_TOPK; ++k2) before[k2] = k2 < k ? idx_s[g - k + k2] : -1;
            bool first = true;
#pragma unroll
            for (int k2 = 0; k2 < FL_MAX_TOPK; ++k2)
                if (before[k2] >= 0 && before[k2] < E && before[k2] / El == d) first = false;
            const size_t o = (size_t)s * D.T * K + g;
            W.comb_pos[o] = start[re] + rank_e;
            W.pair_meta[o] = ((unsigned)(e - d * El) << 24) | (unsigned)rank_e;
            W.send_row[o] = first ? start[rd] - pairs_total + rank_d : -1;
        }
        if (ntiles > 1) {
            __syncthreads();
            for (int r = tid; r < rows; r += kRouteThreads) base[r] += count[r];
            __syncthreads();
        }
    }
}

__host__ __device__ inline size_t route_plan_lds_bytes(int E, int N, int El) {
    return ((size_t)E /*G_all*/ + (size_t)N * El /*own counts*/ + (size_t)N * N /*M*/ + El + 1 +
            3 * (size_t)N + 8) * sizeof(int);
}

// One block per rank r: waits for the route records of all sources, stages what
// it needs from them in LDS with one wide round of loads, then derives every
// table rank r needs for the step.  All ranks see the same records, so all reach
// the same verdict on validity and capacity: a bad step is skipped by everyone
// without further communication.
__device__ __forceinline__ void route_plan_block(const Dims &D, const Tables &W, int r, unsigned *lds) {
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wid = tid / kWave;
    const int E = D.E, N = D.N, El = D.El, RL = D.route_len;
    int *G_all = (int *)lds;              // [E]      tokens per expert over all sources
    int *Cown = G_all + E;                // [N][El]  counts of rank r's experts per source
    int *Mall = Cown + N * El;            // [N][N]   de-duplicated counts, [source][destination]
    int *eoff = Mall + N * N;             // [El+1]   expert offsets of rank r
    int *csoff = eoff + El + 1;           // [N]      first combine-send row of each source
    __shared__ int flag, invalid, over;
    const int *rt = W.routes + (size_t)r * N * RL;

    if (tid == 0) { flag = 0; invalid = 0; over = 0; }
    for (int e = tid; e < E; e += kPlanThreads) G_all[e] = 0;
    __syncthreads();
    if (wid == 0) {
        // Rank r has planned epoch_route[r] steps so far (only this block touches the
        // word); this step is complete when every source's message count has caught up.
        const unsigned expect = W.epoch_route[r] + 1u;
        if (lane == 0) W.epoch_route[r] = expect;
        if (!wave_wait_counters<2>(W.arrive_route + (size_t)r * N, nullptr, expect, N, D.spin_limit)) {
            if (lane == 0) { flag = 1; latch_status(W.status, FL_STATUS_TIMEOUT); }
        }
        acquire_payload<true>();
    }
    __syncthreads();
    if (flag) {
        if (tid == 0) W.plan_ok[r] = 0;
        return;
    }

    // One wide round of loads.  Expert columns: each thread sums a residue class of
    // the sources for one expert (all its loads are independent), LDS adds the parts.
    {
        const int parts = max(1, kPlanThreads / E);
        for (int i = tid; i < E * parts; i += kPlanThreads) {
            const int e = i % E, part = i / E;
            int acc = 0;
            for (int s = part; s < N; s += parts) acc += rt[(size_t)s * RL + e];
            atomicAdd(&G_all[e], acc);
        }
        for (int i = tid; i < N * El; i += kPlanThreads)
            Cown[i] = rt[(size_t)(i / El) * RL + r * El + (i % El)];
        for (int i = tid; i < N * N; i += kPlanThreads)
            Mall[i] = rt[(size_t)(i / N) * RL + E + (i % N)];
        if (tid < N && rt[(size_t)tid * RL + E + 2 * N] == 0) invalid = 1;
        if (tid < N) W.comb_dst_off[(size_t)r * N + tid] = rt[(size_t)tid * RL + E + N + r];
    }
    __syncthreads();
    if (invalid) {
        if (tid == 0) W.plan_ok[r] = 0;       // the offending source latched BAD_INDEX
        return;
    }

    unsigned exp_units = 0;       // wave 0: lane = source; wave 1: lane = peer answering in combine
    if (wid == 0) {
        // lane = source s: receive offsets and combine-send offsets of rank r
        const int s = lane;
        const int m = s < N ? Mall[s * N + r] : 0;
        // what source s will have added once its transfer to this rank is complete: the
        // payload in 16-byte units, plus one for the transfer itself (an empty one still counts)
        exp_units = (unsigned)m * (unsigned)(D.Bw / 16) + 1u;
        int inc = wave_incl_scan(m);
        if (s < N) W.recv_off[(size_t)r * (N + 1) + s] = inc - m;
        if (s == N - 1) W.recv_off[(size_t)r * (N + 1) + N] = inc;
        const int beyond = max(m - D.P, 0);        // rows of s past its private slots
        inc = wave_incl_scan(beyond);
        if (s < N) W.recv_shared_off[(size_t)r * N + s] = inc - beyond;
        int len = 0;
        if (s < N)
            for (int j = 0; j < El; ++j) len += Cown[s * El + j];
        inc = wave_incl_scan(len);
        if (s < N) { csoff[s] = inc - len; W.cs_off[(size_t)r * (N + 1) + s] = inc - len; }
        if (s == N - 1) W.cs_off[(size_t)r * (N + 1) + N] = inc;
        if ((D.flags & FL_FLAG_PARTIAL_SUMS) && s < N) {   // rows s sent to ranks below r
            int before = 0;
            for (int d2 = 0; d2 < r; ++d2) before += Mall[s * N + d2];
            W.ret_off[(size_t)r * N + s] = before;
        }
    } else if (wid == 1) {
        // lane = rank d: capacity verdict for every rank, start of r's segment at d,
        // size of d's reply to rank r
        const int d = lane;
        if (d < N) {
            long long recv_rows = 0;
            int before_me = 0;
            for (int s = 0; s < N; ++s) {
                const int m = Mall[s * N + d];
                if (s < r) before_me += max(m - D.P, 0);
                recv_rows += max(m - D.P, 0);              // what d's shared range must hold
            }
            W.dst_off[(size_t)r * N + d] = before_me;
            int mine = 0;
            for (int j = 0; j < El; ++j) mine += rt[(size_t)r * RL + d * El + j];
            if (D.flags & FL_FLAG_PARTIAL_SUMS) mine = Mall[r * N + d];   // one share per row r sent to d
            exp_units = (unsigned)mine * (unsigned)(D.Bc / 16) + 1u;
            long long p = 0;
            for (int j = 0; j < El; ++j) {
                const int g = G_all[d * El + j];
                if (d == r) { eoff[j] = (int)p; W.G[(size_t)r * El + j] = g; }
                p += (j + 1 < El) ? ((long long)g + D.align - 1) / D.align * D.align : g;
            }
            if (d == r) eoff[El] = (int)p;
            if (recv_rows > D.recv_cap || p > D.expert_cap) over = 1;
        }
    }
    __syncthreads();
    if (over) {
        if (tid == 0) { W.plan_ok[r] = 0; latch_status(W.status, FL_STATUS_CAPACITY); }
        return;
    }
    for (int j = tid; j <= El; j += kPlanThreads) W.expert_off[(size_t)r * (El + 1) + j] = eoff[j];
    // base_x[j][s] = expert_off[j] + rows of lower sources in expert j;
    // cs_base[s][j] = cs_off[s] + rows of lower experts for source s
    for (int i = tid; i < El * N; i += kPlanThreads) {
        const int j = i / N, s = i - j * N;
        int acc = eoff[j];
        for (int s2 = 0; s2 < s; ++s2) acc += Cown[s2 * El + j];
        W.base_x[(size_t)r * El * N + i] = acc;
        const int s3 = i / El, j3 = i - s3 * El;
        int acc3 = csoff[s3];
        for (int j2 = 0; j2 < j3; ++j2) acc3 += Cown[s3 * El + j2];
        W.cs_base[((size_t)r * N + s3) * El + j3] = acc3;
    }
    if (wid == 0 && lane < N) W.expect_disp[(size_t)r * N + lane] += exp_units;
    if (wid == 1 && lane < N) W.expect_comb[(size_t)r * N + lane] += exp_units;
    if (tid == 0) W.plan_ok[r] = 1;
}

// One launch for both halves of the layout step: blocks [0, rank_count) count for
// their source rank and push its route record, blocks [rank_count, 2 * rank_count)
// plan for their rank as soon as the records of all sources have arrived.  The
// planning blocks poll the message counters (bounded) while the counting blocks
// run: workgroups are dispatched in index order and all of them fit on the
// machine at once (two 1024-thread blocks per compute unit, at most 128 blocks),
// so a poller never keeps a counter from starting.  Records cross compute dies
// inside one kernel, hence device-scope stores and one cache invalidation per
// planning block in every mode.
__global__ __launch_bounds__(kRouteThreads) void route_layout_kernel(
    Dims D, Tables W, int rank_begin, int rank_count, const int *__restrict__ indices,
    const int *__restrict__ num_tokens) {
    extern __shared__ unsigned lds[];
    if ((int)blockIdx.x < rank_count)
        route_count_block(D, W, rank_begin + blockIdx.x, indices, num_tokens, lds);
    else
        route_plan_block(D, W, rank_begin + blockIdx.x - rank_count, lds);
}

}  // namespace flmoe
