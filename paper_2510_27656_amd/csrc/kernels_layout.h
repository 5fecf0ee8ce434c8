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
constexpr int kPlanThreads = 256;

__host__ __device__ inline size_t route_count_lds_bytes(int E, int N, int TT) {
    size_t rows = (size_t)E + N;
    return rows * (TT / 32) * 2 * sizeof(unsigned) + rows * 2 * sizeof(int) + 32 * sizeof(int);
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
// Outputs for rank s: C[s][.], M[s][.], send_off[s][.], comb_off[s][.], per pair
// send_row / pair_meta / comb_pos; the route record (C | M | comb_off | valid) is
// pushed into every peer's routes[peer][s] and arrive_route[peer][s] is bumped.
template <bool FENCED>
__global__ __launch_bounds__(kRouteThreads) void route_count_kernel(
    Dims D, Tables W, int rank_begin, const int *__restrict__ indices,
    const int *__restrict__ num_tokens) {
    extern __shared__ unsigned lds[];
    const int s = rank_begin + blockIdx.x;
    const int tid = threadIdx.x;
    const int E = D.E, N = D.N, El = D.El, K = D.K;
    const int rows = E + N;
    const int Wd = D.TT / 32;
    unsigned *bits = lds;                                  // [rows][Wd]
    unsigned *pre = bits + (size_t)rows * Wd;              // [rows][Wd]
    int *base = (int *)(pre + (size_t)rows * Wd);          // [rows] hits in earlier tiles
    int *tot = base + rows;                                // [rows] hits in this tile
    int *scan_tmp = tot + rows;                            // [32]
    __shared__ int bad;

    int Ts = num_tokens[s];
    if (tid == 0) bad = (Ts < 0 || Ts > D.T) ? 1 : 0;
    Ts = max(0, min(Ts, D.T));
    for (int r = tid; r < rows; r += kRouteThreads) base[r] = 0;
    const int *idx_s = indices + (size_t)s * D.T * K;
    int *rank_se = W.comb_pos + (size_t)s * D.T * K;       // holds the bare rank until the second pass
    int *rank_sd = W.send_row + (size_t)s * D.T * K;
    __syncthreads();

    for (int t0 = 0; t0 < Ts; t0 += D.TT) {
        const int nt = min(D.TT, Ts - t0);
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
            for (int w = 0; w < Wd; ++w) {
                pre[(size_t)r * Wd + w] = run;
                run += __popc(bits[(size_t)r * Wd + w]);
            }
            tot[r] = run;
        }
        __syncthreads();
        for (int p = tid; p < nt * K; p += kRouteThreads) {
            const int tl = p / K;
            const int e = idx_s[(size_t)t0 * K + p];
            if (e < 0 || e >= E) continue;
            const unsigned below = (1u << (tl & 31)) - 1u;
            const int w = tl >> 5;
            const int re = e, rd = E + e / El;
            rank_se[(size_t)t0 * K + p] =
                base[re] + pre[(size_t)re * Wd + w] + __popc(bits[(size_t)re * Wd + w] & below);
            rank_sd[(size_t)t0 * K + p] =
                base[rd] + pre[(size_t)rd * Wd + w] + __popc(bits[(size_t)rd * Wd + w] & below);
        }
        __syncthreads();
        for (int r = tid; r < rows; r += kRouteThreads) base[r] += tot[r];
        __syncthreads();
    }

    // Totals and their exclusive scans.  tot[] is reused: tot[e] = comb_base[e]
    // (first combine-receive row of expert e), tot[E+d] = send_off[d].
    int total;
    {
        const int v = tid < E ? base[tid] : 0;             // E <= kRouteThreads
        const int ex = block_excl_scan(v, scan_tmp, &total);
        if (tid < E) {
            tot[tid] = ex;
            W.C[(size_t)s * E + tid] = v;
        }
    }
    const int pairs_total = total;
    {
        const int v = tid < N ? base[E + tid] : 0;         // N <= 64
        const int ex = block_excl_scan(v, scan_tmp, &total);
        if (tid < N) {
            tot[E + tid] = ex;
            W.M[(size_t)s * N + tid] = v;
            W.send_off[(size_t)s * (N + 1) + tid] = ex;
        }
        if (tid == 0) W.send_off[(size_t)s * (N + 1) + N] = total;
    }
    __syncthreads();
    if (tid < N) W.comb_off[(size_t)s * (N + 1) + tid] = tot[tid * El];
    if (tid == 0) W.comb_off[(size_t)s * (N + 1) + N] = pairs_total;

    // Second pass over the pairs: absolute positions.
    for (int p = tid; p < Ts * K; p += kRouteThreads) {
        const int k = p % K;
        const int e = idx_s[p];
        if (e < 0 || e >= E) continue;
        const int d = e / El;
        const int rse = rank_se[p];
        bool first = true;
        for (int k2 = 0; k2 < k; ++k2) {
            const int e2 = idx_s[p - k + k2];
            if (e2 >= 0 && e2 < E && e2 / El == d) first = false;
        }
        W.comb_pos[(size_t)s * D.T * K + p] = tot[e] + rse;
        W.pair_meta[(size_t)s * D.T * K + p] = ((unsigned)(e - d * El) << 24) | (unsigned)rse;
        rank_sd[p] = first ? tot[E + d] + rank_sd[p] : -1;
    }
    __syncthreads();
    const int valid = bad ? 0 : 1;
    if (bad && tid == 0) latch_status(W.status, FL_STATUS_BAD_INDEX);

    // Route exchange: push this rank's record into every peer's table, then notify.
    const int RL = D.route_len;
    for (int i = tid; i < N * RL; i += kRouteThreads) {
        const int peer = i / RL, f = i % RL;
        int v;
        if (f < E) v = base[f];
        else if (f < E + N) v = base[f];
        else if (f < E + 2 * N) v = tot[(f - E - N) * El];
        else v = valid;
        W.routes[((size_t)peer * N + s) * RL + f] = v;
    }
    stores_done<FENCED>();
    __syncthreads();
    if (tid < N) add_counter<FENCED>(W.arrive_route + (size_t)tid * N + s, 1u);
    if (tid == 0) W.epoch_route[s] += 1u;
}

// One block per rank r: waits for the route records of all sources, then
// derives every table rank r needs for the step from the records it holds.
// All ranks see the same records, so all reach the same verdict on validity and
// capacity: a bad step is skipped by everyone without further communication.
template <bool FENCED>
__global__ __launch_bounds__(kPlanThreads) void route_plan_kernel(Dims D, Tables W,
                                                                  int rank_begin) {
    extern __shared__ unsigned lds[];
    const int r = rank_begin + blockIdx.x;
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wid = tid / kWave;
    const int E = D.E, N = D.N, El = D.El, RL = D.route_len;
    int *G_all = (int *)lds;              // [E]
    int *eoff = G_all + E;                // [El+1] of rank r
    __shared__ int flag;
    const int *rt = W.routes + (size_t)r * N * RL;

    if (tid == 0) flag = 0;
    __syncthreads();
    if (wid == 0) {
        const unsigned expect = W.epoch_route[r];
        if (!wave_wait_counters(W.arrive_route + (size_t)r * N, nullptr, expect, N, D.spin_limit)) {
            if (lane == 0) { flag = 1; latch_status(W.status, FL_STATUS_TIMEOUT); }
        }
        acquire_payload<FENCED>();
    }
    __syncthreads();
    if (flag) {
        if (tid == 0) W.plan_ok[r] = 0;
        return;
    }
    int ok = 1;
    if (tid < N) ok = rt[(size_t)tid * RL + E + 2 * N];
    if (!__syncthreads_and(ok)) {
        if (tid == 0) W.plan_ok[r] = 0;       // the offending source latched BAD_INDEX
        return;
    }

    // Column sums over sources for every expert; running prefixes for own experts.
    for (int e = tid; e < E; e += kPlanThreads) {
        const bool own = e / El == r;
        int acc = 0;
        for (int s = 0; s < N; ++s) {
            if (own) W.base_x[((size_t)r * El + (e - r * El)) * N + s] = acc;
            acc += rt[(size_t)s * RL + e];
        }
        G_all[e] = acc;
    }
    __syncthreads();

    int over = 0;
    unsigned exp_units = 0;       // wave 0: lane = source; wave 1: lane = peer answering in combine
    if (wid == 0) {
        // lane = source s: receive offsets, combine-send offsets of rank r
        const int s = lane;
        const int m = s < N ? rt[(size_t)s * RL + E + r] : 0;
        exp_units = (unsigned)m * (unsigned)(D.Bw / 16);
        int inc = wave_incl_scan(m);
        if (s < N) W.recv_off[(size_t)r * (N + 1) + s] = inc - m;
        if (s == N - 1) W.recv_off[(size_t)r * (N + 1) + N] = inc;
        int len = 0;
        if (s < N)
            for (int j = 0; j < El; ++j) len += rt[(size_t)s * RL + r * El + j];
        inc = wave_incl_scan(len);
        if (s < N) {
            int acc = inc - len;
            W.cs_off[(size_t)r * (N + 1) + s] = acc;
            for (int j = 0; j < El; ++j) {
                W.cs_base[((size_t)r * N + s) * El + j] = acc;
                acc += rt[(size_t)s * RL + r * El + j];
            }
            W.comb_dst_off[(size_t)r * N + s] = rt[(size_t)s * RL + E + N + r];
        }
        if (s == N - 1) W.cs_off[(size_t)r * (N + 1) + N] = inc;
    } else if (wid == 1) {
        // lane = rank d: capacity verdict for every rank, size of d's reply to rank r
        const int d = lane;
        if (d < N) {
            long long recv_rows = 0;
            int before_me = 0;                  // rows of lower ranks ahead of r's segment at d
            for (int s = 0; s < N; ++s) {
                const int m = rt[(size_t)s * RL + E + d];
                if (s < r) before_me += m;
                recv_rows += m;
            }
            W.dst_off[(size_t)r * N + d] = before_me;
            int mine = 0;                       // pairs of rank r served by rank d: its reply
            for (int j = 0; j < El; ++j) mine += rt[(size_t)r * RL + d * El + j];
            exp_units = (unsigned)mine * (unsigned)(D.Bc / 16);
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
    over = __syncthreads_or(over);
    if (over) {
        if (tid == 0) { W.plan_ok[r] = 0; latch_status(W.status, FL_STATUS_CAPACITY); }
        return;
    }
    for (int j = tid; j <= El; j += kPlanThreads) W.expert_off[(size_t)r * (El + 1) + j] = eoff[j];
    for (int i = tid; i < El * N; i += kPlanThreads)
        W.base_x[(size_t)r * El * N + i] += eoff[i / N];
    if (wid == 0 && lane < N) W.expect_disp[(size_t)r * N + lane] += exp_units;
    if (wid == 1 && lane < N) W.expect_comb[(size_t)r * N + lane] += exp_units;
    if (tid == 0) W.plan_ok[r] = 1;
}

}  // namespace flmoe
