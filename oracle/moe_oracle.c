/*
 * CPU oracle for the MoE expert-parallel dispatch/combine token shuffle
 * (paper section "MoE Dispatch/Combine", subsections Architecture, Dispatch,
 * Combine; workload shapes from "Kernel Microbenchmarks").
 *
 * THIS IS TEST INFRASTRUCTURE.  It is a plain, slow, single-threaded statement
 * of what the shuffle computes.  It shares no code with the HIP library, is
 * never linked into it and is never called by it; only tests, the smoke check
 * and the bench's cpu_baseline leg may call it.
 *
 * Problem statement (section Architecture): N ranks host E experts, every rank
 * dispatches up to T tokens to R (= K here) experts each.  Expert e lives on
 * rank e / (E/N).  All arrays are host pointers, dense row-major, owned by the
 * caller.  bf16 values travel as uint16_t bit patterns.
 *
 * Pinned by tests/test_oracle_pins.py (brute-force stable sort, exhaustive tiny
 * enumeration, closed forms, round trip, fp64 bound, independent e4m3 encoder).
 * Parity unpinned (this build's own canonical choices, nothing in the paper or
 * the mathematics fixes them): orc_recv_order and orc_comb_pos (the order of
 * rows inside the internal receive buffers).
 */
#include <math.h>
#include <stdint.h>
#include <string.h>

/* ---------- bf16 <-> fp32, round to nearest even ---------- */

static float bf16_to_f32(uint16_t b) {
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

static uint16_t f32_to_bf16_rne(float f) {
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7fffffffu) > 0x7f800000u)          /* NaN: keep it a quiet NaN */
        return (uint16_t)((u >> 16) | 0x0040u);
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7fffu + lsb;                            /* ties go to the even mantissa */
    return (uint16_t)(u >> 16);
}

static int owner_of(int e, int El) { return e / El; }

/* does token (s,t) list expert e among its K choices?  returns k or -1 */
static int find_k(const int32_t *idx, int K, int e) {
    for (int k = 0; k < K; ++k)
        if (idx[k] == e) return k;
    return -1;
}

/* ---------- O1: per-expert counts (section Dispatch: the kernel first counts
 * the tokens sent to each expert) ----------
 * indices [N][Tmax][K], num_tokens [N]  ->  C [N][E]                         */
void orc_counts(int N, int E, int Tmax, int K, const int32_t *num_tokens,
                const int32_t *indices, int32_t *C) {
    memset(C, 0, sizeof(int32_t) * (size_t)N * E);
    for (int s = 0; s < N; ++s)
        for (int t = 0; t < num_tokens[s]; ++t)
            for (int k = 0; k < K; ++k) {
                int e = indices[((size_t)s * Tmax + t) * K + k];
                C[(size_t)s * E + e] += 1;
            }
}

/* ---------- O2: deduplicated counts.  M[s][d] = number of tokens of rank s
 * that have at least one expert on rank d (one copy per (token, destination
 * rank) is what travels). ---------- */
void orc_dedup_counts(int N, int E, int Tmax, int K, const int32_t *num_tokens,
                      const int32_t *indices, int32_t *M) {
    int El = E / N;
    memset(M, 0, sizeof(int32_t) * (size_t)N * N);
    for (int s = 0; s < N; ++s)
        for (int t = 0; t < num_tokens[s]; ++t) {
            const int32_t *idx = indices + ((size_t)s * Tmax + t) * K;
            for (int d = 0; d < N; ++d) {
                int hit = 0;
                for (int k = 0; k < K; ++k)
                    if (owner_of(idx[k], El) == d) hit = 1;
                M[(size_t)s * N + d] += hit;
            }
        }
}

/* ---------- O3: offsets (section Architecture: the exchanged counts give every
 * source a unique range in the destination's contiguous receive buffer).
 *   send_off  [N][N+1]  exclusive scan of M[s][.] over d
 *   recv_off  [N][N+1]  exclusive scan of M[.][d] over s  (receive buffer of d
 *                        is ordered by source rank)
 *   G         [N][El]   tokens per local expert, G[d][j] = sum_s C[s][d*El+j]
 *   expert_off[N][El+1] exclusive scan over j of G rounded up to a multiple of
 *                        `align` ("optional padding between experts", section
 *                        Dispatch); the last expert is not padded, so entry El
 *                        is the end of its real rows
 *   comb_off  [N][N+1]  comb_off[s][d] = sum of C[s][e] over experts e on ranks
 *                        below d: where the reply of rank d starts at rank s   */
void orc_offsets(int N, int E, int align, const int32_t *C, const int32_t *M,
                 int32_t *send_off, int32_t *recv_off, int32_t *G,
                 int32_t *expert_off, int32_t *comb_off) {
    int El = E / N;
    for (int s = 0; s < N; ++s) {
        int32_t acc = 0;
        for (int d = 0; d < N; ++d) {
            send_off[(size_t)s * (N + 1) + d] = acc;
            acc += M[(size_t)s * N + d];
        }
        send_off[(size_t)s * (N + 1) + N] = acc;
    }
    for (int d = 0; d < N; ++d) {
        int32_t acc = 0;
        for (int s = 0; s < N; ++s) {
            recv_off[(size_t)d * (N + 1) + s] = acc;
            acc += M[(size_t)s * N + d];
        }
        recv_off[(size_t)d * (N + 1) + N] = acc;
    }
    for (int d = 0; d < N; ++d) {
        int32_t acc = 0;
        for (int j = 0; j < El; ++j) {
            int32_t g = 0;
            for (int s = 0; s < N; ++s) g += C[(size_t)s * E + d * El + j];
            G[(size_t)d * El + j] = g;
            expert_off[(size_t)d * (El + 1) + j] = acc;
            if (j + 1 < El)
                acc += (g + align - 1) / align * align;
            else
                acc += g;
        }
        expert_off[(size_t)d * (El + 1) + El] = acc;
    }
    for (int s = 0; s < N; ++s) {
        int32_t acc = 0;
        for (int d = 0; d < N; ++d) {
            comb_off[(size_t)s * (N + 1) + d] = acc;
            for (int j = 0; j < El; ++j) acc += C[(size_t)s * E + d * El + j];
        }
        comb_off[(size_t)s * (N + 1) + N] = acc;
    }
}

/* ---------- O4: the canonical expert-major layout (section Dispatch: tokens
 * from all ranks packed by local expert, optional padding between experts).
 * The rows of rank d are the (source, token, k) triples whose expert lives on
 * d, ordered by expert, then source rank, then token index.
 * slot [N][Tmax][K]: row index of pair (s,t,k) inside its owner rank's layout
 * (entries of tokens t >= num_tokens[s] are set to -1).                        */
void orc_slots(int N, int E, int Tmax, int K, int align,
               const int32_t *num_tokens, const int32_t *indices,
               int32_t *slot) {
    int El = E / N;
    for (size_t i = 0; i < (size_t)N * Tmax * K; ++i) slot[i] = -1;
    for (int d = 0; d < N; ++d) {
        int32_t p = 0;
        for (int j = 0; j < El; ++j) {
            int e = d * El + j;
            for (int s = 0; s < N; ++s)
                for (int t = 0; t < num_tokens[s]; ++t) {
                    size_t base = ((size_t)s * Tmax + t) * K;
                    int k = find_k(indices + base, K, e);
                    if (k >= 0) slot[base + k] = p++;
                }
            if (j + 1 < El) p = (p + align - 1) / align * align;
        }
    }
}

/* Expert-major rows of ONE rank d, written by the same enumeration (it does not
 * use orc_slots).  x [N][Tmax] records of `row_bytes` bytes each is the payload
 * of each token (bf16 hidden state, or any per-token record); out has
 * room for expert_off[d][El] rows.  Padding rows are zero-filled when
 * zero_pad != 0 and left untouched otherwise.  Returns the number of rows of
 * the layout (padding between experts included).                               */
int64_t orc_dispatch_rank(int d, int N, int E, int Tmax, int K, int align,
                          int zero_pad, const int32_t *num_tokens,
                          const int32_t *indices, const void *x,
                          int64_t row_bytes, void *out) {
    int El = E / N;
    const uint8_t *xin = (const uint8_t *)x;
    uint8_t *o = (uint8_t *)out;
    int64_t p = 0;
    for (int j = 0; j < El; ++j) {
        int e = d * El + j;
        for (int s = 0; s < N; ++s)
            for (int t = 0; t < num_tokens[s]; ++t) {
                size_t tok = (size_t)s * Tmax + t;
                if (find_k(indices + tok * K, K, e) >= 0) {
                    memcpy(o + p * row_bytes, xin + tok * row_bytes, (size_t)row_bytes);
                    ++p;
                }
            }
        if (j + 1 < El) {
            int64_t q = (p + align - 1) / align * align;
            if (zero_pad) memset(o + p * row_bytes, 0, (size_t)((q - p) * row_bytes));
            p = q;
        }
    }
    return p;
}

/* ---------- O5: combine (section Combine: the weighted average of the tokens
 * is computed locally on each rank; accumulation entirely in fp32 in a fixed
 * order, section Comparison with DeepEP).
 *   out[s][t] = bf16( sum_{k=0..K-1} w[s][t][k] * float(Y[owner][slot(s,t,k)]) )
 * with an fp32 accumulator that starts at +0 and is updated by a fused
 * multiply-add in the order the caller lists the K experts.  No division by the
 * weight sum.  Y is rank-major: rank d's rows start at Y + d*y_rank_stride
 * elements, each row H bf16.  acc_out (optional, [N][Tmax][H]) receives the
 * fp32 accumulator before the final rounding, so that tests can pin the
 * accumulation order and the fused multiply-add exactly.                       */
void orc_combine(int N, int E, int Tmax, int K, int H,
                 const int32_t *num_tokens, const int32_t *indices,
                 const int32_t *slot, const float *weights, const uint16_t *Y,
                 int64_t y_rank_stride, uint16_t *out, float *acc_out) {
    int El = E / N;
    for (int s = 0; s < N; ++s)
        for (int t = 0; t < num_tokens[s]; ++t) {
            size_t tok = (size_t)s * Tmax + t;
            for (int h = 0; h < H; ++h) {
                float acc = 0.0f;
                for (int k = 0; k < K; ++k) {
                    int e = indices[tok * K + k];
                    int d = owner_of(e, El);
                    const uint16_t *row =
                        Y + (size_t)d * y_rank_stride + (size_t)slot[tok * K + k] * H;
                    acc = fmaf(weights[tok * K + k], bf16_to_f32(row[h]), acc);
                }
                out[tok * H + h] = f32_to_bf16_rne(acc);
                if (acc_out) acc_out[tok * H + h] = acc;   /* fp32 sum before the final rounding */
            }
        }
}

/* ---------- O5b: combine with sender-side partial sums (section Comparison with
 * DeepEP and section Performance, prefill: tokens are pre-accumulated on the
 * sending side, which moves fewer bytes but reduces the accumulation precision
 * to bf16 between the two stages).  The paper names the idea, not the
 * arithmetic; the definition taken here:
 *   group the K experts of token (s,t) by the rank that hosts them;
 *   partial(d) = bf16( fp32 fused multiply-add chain from +0 over the token's
 *                experts on rank d, in ascending k, weight times row )
 *   out[s][t]  = bf16( fp32 sum from +0 of float(partial(d)), ranks taken in
 *                the order of their first k )
 * Weights are applied on the expert's rank, so the receiver only adds.       */
void orc_combine_partial(int N, int E, int Tmax, int K, int H,
                         const int32_t *num_tokens, const int32_t *indices,
                         const int32_t *slot, const float *weights, const uint16_t *Y,
                         int64_t y_rank_stride, uint16_t *out) {
    int El = E / N;
    for (int s = 0; s < N; ++s)
        for (int t = 0; t < num_tokens[s]; ++t) {
            size_t tok = (size_t)s * Tmax + t;
            for (int h = 0; h < H; ++h) {
                float total = 0.0f;
                for (int k = 0; k < K; ++k) {
                    int d = owner_of(indices[tok * K + k], El);
                    int first = 1;              /* is k the first expert of the token on rank d? */
                    for (int k2 = 0; k2 < k; ++k2)
                        if (owner_of(indices[tok * K + k2], El) == d) first = 0;
                    if (!first) continue;
                    float part = 0.0f;          /* rank d's share, accumulated on rank d */
                    for (int k2 = k; k2 < K; ++k2) {
                        if (owner_of(indices[tok * K + k2], El) != d) continue;
                        const uint16_t *row =
                            Y + (size_t)d * y_rank_stride + (size_t)slot[tok * K + k2] * H;
                        part = fmaf(weights[tok * K + k2], bf16_to_f32(row[h]), part);
                    }
                    total = total + bf16_to_f32(f32_to_bf16_rne(part));
                }
                out[tok * H + h] = f32_to_bf16_rne(total);
            }
        }
}

/* Stand-in expert (harness stage between dispatch and combine, not part of the
 * shuffle): every row of expert e is scaled by g[e]; y = bf16(float(x) * g).
 * Applied in place over one rank's layout, padding rows untouched.             */
void orc_expert_scale_rank(int d, int N, int E, const int32_t *expert_off,
                           const int32_t *G, const float *g, int H,
                           uint16_t *rows) {
    int El = E / N;
    for (int j = 0; j < El; ++j) {
        int64_t r0 = expert_off[(size_t)d * (El + 1) + j];
        int64_t n = G[(size_t)d * El + j];
        float ge = g[d * El + j];
        for (int64_t r = r0; r < r0 + n; ++r)
            for (int h = 0; h < H; ++h) {
                uint16_t *p = rows + (size_t)r * H + h;
                *p = f32_to_bf16_rne(bf16_to_f32(*p) * ge);
            }
    }
}

/* ---------- internal buffer orders (parity unpinned: this build's choice) ----
 * Receive order at rank d: the deduplicated (source, token) pairs that reach d,
 * ascending by source rank then token index.  Returns their number; src_rank /
 * src_tok need room for N*Tmax entries.  mask[r] has bit j set when the row is
 * wanted by local expert j.                                                    */
int64_t orc_recv_order(int d, int N, int E, int Tmax, int K,
                       const int32_t *num_tokens, const int32_t *indices,
                       int32_t *src_rank, int32_t *src_tok, uint64_t *mask) {
    int El = E / N;
    int64_t r = 0;
    for (int s = 0; s < N; ++s)
        for (int t = 0; t < num_tokens[s]; ++t) {
            const int32_t *idx = indices + ((size_t)s * Tmax + t) * K;
            uint64_t m = 0;
            for (int k = 0; k < K; ++k)
                if (owner_of(idx[k], El) == d) m |= 1ull << (idx[k] - d * El);
            if (m) {
                src_rank[r] = s;
                src_tok[r] = t;
                if (mask) mask[r] = m;
                ++r;
            }
        }
    return r;
}

/* Position of pair (s,t,k) in rank s's combine receive buffer: replies are laid
 * out by expert id, then token index (so the reply of each peer is one
 * contiguous range).  comb_pos [N][Tmax][K], -1 for absent tokens.             */
void orc_comb_pos(int N, int E, int Tmax, int K, const int32_t *num_tokens,
                  const int32_t *indices, int32_t *comb_pos) {
    for (size_t i = 0; i < (size_t)N * Tmax * K; ++i) comb_pos[i] = -1;
    for (int s = 0; s < N; ++s) {
        int32_t p = 0;
        for (int e = 0; e < E; ++e)
            for (int t = 0; t < num_tokens[s]; ++t) {
                size_t base = ((size_t)s * Tmax + t) * K;
                int k = find_k(indices + base, K, e);
                if (k >= 0) comb_pos[base + k] = p++;
            }
    }
}

/* ---------- fp8 dispatch payload (section Kernel Microbenchmarks: 7168 fp8
 * values with 56 fp32 scaling factors per token, i.e. one scale per 128
 * elements).  Format: OCP E4M3 (finite-only variant): 1 sign, 4 exponent bits
 * with bias 7, 3 mantissa bits, largest finite 448, no infinities, subnormals
 * down to 2^-9.  Rule per 128-element block: amax = max |x|; scale = amax/448
 * (fp32 division; scale = 1 when amax = 0); q = e4m3(x / scale) rounded to
 * nearest, ties to even, saturating at +-448.
 * Non-finite inputs, a reading (the paper dispatches ready-made fp8 and says
 * nothing): a NaN element is skipped by the maximum (a > amax is false) and
 * becomes the NaN code with its own sign, the rest of its block is quantised
 * as if it were absent; an infinite element makes amax and the scale +Inf, so
 * every finite element of that block becomes a signed zero (x / Inf) and every
 * infinite one the NaN code with its sign; a block of NaNs only has scale 1. ---------- */

float orc_e4m3_decode(uint8_t c) {
    int sign = c >> 7, ex = (c >> 3) & 0xf, man = c & 7;
    float v;
    if (ex == 0)
        v = ldexpf((float)man, -9);                /* subnormal: man * 2^-6 / 8 */
    else if (ex == 15 && man == 7)
        v = NAN;
    else
        v = ldexpf(1.0f + (float)man / 8.0f, ex - 7);
    return sign ? -v : v;
}

uint8_t orc_e4m3_encode(float f) {
    uint8_t sign = signbit(f) ? 0x80 : 0;
    float a = fabsf(f);
    if (isnan(a)) return sign | 0x7f;
    if (a >= 448.0f) return sign | 0x7e;           /* saturate (also +-inf) */
    /* quantum of the binade a falls in: 2^(floor(log2 a) - 3), at least 2^-9 */
    int ex;
    (void)frexpf(a, &ex);                          /* a = m * 2^ex, m in [0.5,1) */
    int q = ex - 1 - 3;
    if (q < -9) q = -9;
    /* a / 2^q is exact in fp32 (a has 24 bits, result < 16 needs <= 24+ bits of
     * fraction only when a is tiny, where ldexpf stays exact short of fp32
     * underflow, which cannot happen for q >= -9 and a >= 2^-149)               */
    float steps = ldexpf(a, -q);
    float r = nearbyintf(steps);                   /* default mode: ties to even */
    float v = ldexpf(r, q);
    if (v >= 448.0f) return sign | 0x7e;           /* 432 < a < 448 rounds up to 448 */
    if (v == 0.0f) return sign;
    int ve;
    float vm = frexpf(v, &ve);                     /* v = vm * 2^ve */
    int E = ve - 1 + 7;
    if (E <= 0) {                                  /* subnormal: v = man * 2^-9 */
        int man = (int)ldexpf(v, 9);
        return sign | (uint8_t)man;
    }
    int man = (int)((vm * 2.0f - 1.0f) * 8.0f);
    return sign | (uint8_t)(E << 3) | (uint8_t)man;
}

/* Quantise `rows` rows of H bf16 values.  q [rows][H] bytes, scales
 * [rows][H/128] fp32.  H must be a multiple of 128.                            */
void orc_quant_e4m3_block128(int64_t rows, int H, const uint16_t *x, uint8_t *q,
                             float *scales) {
    int nb = H / 128;
    for (int64_t r = 0; r < rows; ++r)
        for (int b = 0; b < nb; ++b) {
            const uint16_t *xb = x + (size_t)r * H + (size_t)b * 128;
            float amax = 0.0f;
            for (int i = 0; i < 128; ++i) {
                float a = fabsf(bf16_to_f32(xb[i]));
                if (a > amax) amax = a;
            }
            float scale = (amax == 0.0f) ? 1.0f : amax / 448.0f;
            scales[(size_t)r * nb + b] = scale;
            for (int i = 0; i < 128; ++i) {
                float v = bf16_to_f32(xb[i]);
                uint8_t code;
                if (isnan(v) || isinf(v))
                    /* Non-finite input (the paper is silent): the rule above applied in
                     * IEEE arithmetic gives NaN here (NaN / scale, or Inf / Inf since an
                     * Inf makes amax and the scale infinite); the NaN code takes the
                     * sign of the INPUT element, which IEEE leaves open for Inf / Inf. */
                    code = (uint8_t)((xb[i] >> 8) & 0x80) | 0x7f;
                else
                    code = orc_e4m3_encode(v / scale);
                q[(size_t)r * H + (size_t)b * 128 + i] = code;
            }
        }
}

/* Dequantise rows back to bf16: y = bf16(float(q) * scale). */
void orc_dequant_e4m3_block128(int64_t rows, int H, const uint8_t *q,
                               const float *scales, uint16_t *y) {
    int nb = H / 128;
    for (int64_t r = 0; r < rows; ++r)
        for (int h = 0; h < H; ++h)
            y[(size_t)r * H + h] = f32_to_bf16_rne(
                orc_e4m3_decode(q[(size_t)r * H + h]) * scales[(size_t)r * nb + h / 128]);
}

/* bf16 helpers exported for the tests */
float orc_bf16_to_f32(uint16_t b) { return bf16_to_f32(b); }
uint16_t orc_f32_to_bf16(float f) { return f32_to_bf16_rne(f); }

/* array forms for the tests */
void orc_e4m3_encode_array(int64_t n, const float *in, uint8_t *out) {
    for (int64_t i = 0; i < n; ++i) out[i] = orc_e4m3_encode(in[i]);
}
void orc_e4m3_decode_array(int64_t n, const uint8_t *in, float *out) {
    for (int64_t i = 0; i < n; ++i) out[i] = orc_e4m3_decode(in[i]);
}
void orc_f32_to_bf16_array(int64_t n, const float *in, uint16_t *out) {
    for (int64_t i = 0; i < n; ++i) out[i] = f32_to_bf16_rne(in[i]);
}

/* Stand-in expert on explicit rows: row r is scaled by gains[r] (used when a test
 * checks sampled tokens of a workload too large to lay out on the host). */
void orc_scale_rows(int64_t rows, int H, const float *gains, uint16_t *data) {
    for (int64_t r = 0; r < rows; ++r)
        for (int h = 0; h < H; ++h) {
            uint16_t *p = data + (size_t)r * H + h;
            *p = f32_to_bf16_rne(bf16_to_f32(*p) * gains[r]);
        }
}
