/*
 * CPU oracle for the target-side verification step of speculative decoding over a
 * continuous batch with per-request speculative lengths.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the plain definition of what the hot path
 * computes, written from the paper (FASER, arXiv 2604.20503) and the speculative-
 * sampling rule it builds on.  It shares no code with the HIP library, is never
 * loaded by the product path, and is slow on purpose: one obvious loop per sum,
 * fp64 everywhere, no blocking, no fusion.  OpenMP only distributes independent
 * output elements over host threads.
 *
 * Parity pins (tests/test_oracle_*.py) hold every function here against something
 * other than itself: a dense numpy softmax, closed forms, the output-distribution
 * theorem of speculative sampling, brute force on tiny vocabularies, and python-loop
 * definitions of the compaction.
 *
 * What each function follows:
 *   fo_verify_attention  Sec. 2.1 (the target model verifies all drafted tokens of a
 *                        request in one parallel pass) over the paged KV cache of a
 *                        continuous batch (Sec. 2.1, Sec. 3.1: one speculative length
 *                        per request).  Scaled-dot-product softmax attention, causal
 *                        inside the draft suffix.
 *   fo_spec_accept       Sec. 2.1: accept drafted tokens until the first mismatch,
 *                        drop the rejected suffix, resample the first mismatched token
 *                        from the target; Sec. 3.3: "recovery token".  The mismatch
 *                        test and the resampling distribution are those of speculative
 *                        sampling (accept with probability min(1, p/q); recovery token
 *                        from the normalised positive part of p - q; a bonus token from
 *                        the target when every draft is accepted).
 *   fo_kv_append         Sec. 2.1 / Sec. 3.1: the drafted tokens of a request enter the
 *                        target model as new positions behind its cached context; their
 *                        keys and values are stored into the request's pages before the
 *                        attention of the same forward pass reads them.
 *   fo_greedy_accept     the same accept-until-first-mismatch rule at temperature 0: the
 *                        target's choice at a position is its arg-max token, a draft
 *                        matches iff it is that token, and the token "resampled from the
 *                        target" after the accepted run is the arg-max of the next row.
 *   fo_prune_compact     Sec. 3.2: rows predicted/observed to be in the rejected suffix
 *                        are pruned and only the remaining rows proceed; Sec. 3.3: on a
 *                        rejection every speculative token beyond it is discarded.
 *   fo_prune_restore     Sec. 3.2 / Sec. 4: survivors return to their original rows,
 *                        dropped rows get filler and carry no values.
 *   fo_topk_rank_check   Sec. 3.2: intermediate scores predict a rejection when the
 *                        draft is not among their K best tokens; Sec. 4: decided by
 *                        counting the scores above the draft's own.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { FO_F32 = 0, FO_BF16 = 1, FO_F64 = 2 };
enum { FO_PROBS = 0, FO_LOGITS = 1 };

static double load_elem(const void *base, int64_t idx, int dtype)
{
    if (dtype == FO_F32)
        return (double)((const float *)base)[idx];
    if (dtype == FO_F64)
        return ((const double *)base)[idx];
    /* bf16: the upper half of an IEEE fp32 */
    uint32_t bits = (uint32_t)((const uint16_t *)base)[idx] << 16;
    float f;
    memcpy(&f, &bits, 4);
    return (double)f;
}

/*
 * Value of an 8-bit float in the OCP "E4M3" format (1 sign, 4 exponent bits with bias 7, 3
 * mantissa bits; no infinities; exponent 15 with mantissa 7 is NaN; exponent 0 is subnormal,
 * mantissa / 8 * 2^-6).  Used for KV caches stored in 8 bits (a storage variant of the
 * verification attention: the arithmetic is unchanged, the cached values are value * scale).
 */
void fo_decode_e4m3(const uint8_t *codes, double *out, int64_t n)
{
    for (int64_t k = 0; k < n; ++k) {
        const int c = codes[k], e = (c >> 3) & 15, m = c & 7;
        double v;
        if (e == 15 && m == 7)
            v = NAN;
        else if (e == 0)
            v = ldexp((double)m / 8.0, -6);
        else
            v = ldexp(1.0 + (double)m / 8.0, e - 7);
        out[k] = (c & 0x80) ? -v : v;
    }
}

/*
 * The E4M3 byte that stands for x: the finite code whose value is nearest to x, the one with an
 * even code on a tie (round to nearest even), magnitudes beyond the largest finite value (448)
 * giving that value (saturation), NaN giving the NaN code.  Written as a search over the 127
 * non-negative finite codes so that it is the definition and nothing else.
 */
void fo_encode_e4m3(const float *x, uint8_t *out, int64_t n)
{
    double value[127];
    for (int c = 0; c < 127; ++c) {
        const uint8_t code = (uint8_t)c;
        fo_decode_e4m3(&code, &value[c], 1);
    }
    for (int64_t k = 0; k < n; ++k) {
        if (isnan(x[k])) {
            out[k] = 0x7f;
            continue;
        }
        const double mag = fabs((double)x[k]);
        int best = 0;
        for (int c = 1; c < 127; ++c) {
            const double d = fabs(value[c] - mag), db = fabs(value[best] - mag);
            if (d < db || (d == db && (c & 1) == 0))
                best = c;
        }
        out[k] = (uint8_t)(best | (signbit(x[k]) ? 0x80 : 0));
    }
}

/*
 * Attention of every query row over its request's cached keys/values.
 *
 * Request i owns rows cu_q[i] .. cu_q[i+1]-1.  Row j of request i is the query of the
 * token at logical position ctx_lens[i] + j and sees positions 0 .. ctx_lens[i] + j.
 * Logical position t of request i is stored in page block_tables[i*max_pages + t/P],
 * slot t % P; caches are [n_pages, H_kv, P, D].  Query head h reads KV head h / (H_q/H_kv).
 *
 *   s_t = scale * sum_d q[d] * K[t][d];  m = max_t s_t;  w_t = exp(s_t - m)
 *   out[d] = sum_t w_t V[t][d] / sum_t w_t;   lse = m + log(sum_t w_t)
 *
 * out is [N, H_q, D] fp64, lse (nullable) is [N, H_q] fp64.
 */
int fo_verify_attention(const void *q, const void *k_cache, const void *v_cache,
                        const int32_t *block_tables, const int32_t *ctx_lens, const int32_t *cu_q,
                        double *out, double *lse, int B, int H_q, int H_kv, int D, int P,
                        int max_pages, int dtype, double scale)
{
    if (H_kv <= 0 || H_q % H_kv != 0)
        return -1;
    const int G = H_q / H_kv;
    for (int i = 0; i < B; ++i) {
        const int q_len = cu_q[i + 1] - cu_q[i];
        const int c = ctx_lens[i];
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
        for (int j = 0; j < q_len; ++j) {
            for (int h = 0; h < H_q; ++h) {
                const int64_t row = (int64_t)cu_q[i] + j;
                const int g = h / G;
                const int L = c + j + 1; /* visible keys */
                double *s = (double *)malloc(sizeof(double) * (size_t)L);
                double m = -INFINITY;
                for (int t = 0; t < L; ++t) {
                    const int64_t page = block_tables[(int64_t)i * max_pages + t / P];
                    const int64_t kb = ((page * H_kv + g) * P + t % P) * D;
                    double acc = 0.0;
                    for (int d = 0; d < D; ++d)
                        acc += load_elem(q, (row * H_q + h) * D + d, dtype) * load_elem(k_cache, kb + d, dtype);
                    s[t] = scale * acc;
                    if (s[t] > m)
                        m = s[t];
                }
                double denom = 0.0;
                for (int t = 0; t < L; ++t) {
                    s[t] = exp(s[t] - m);
                    denom += s[t];
                }
                for (int d = 0; d < D; ++d) {
                    double acc = 0.0;
                    for (int t = 0; t < L; ++t) {
                        const int64_t page = block_tables[(int64_t)i * max_pages + t / P];
                        const int64_t vb = ((page * H_kv + g) * P + t % P) * D;
                        acc += s[t] * load_elem(v_cache, vb + d, dtype);
                    }
                    out[(row * H_q + h) * D + d] = acc / denom;
                }
                if (lse)
                    lse[row * H_q + h] = m + log(denom);
                free(s);
            }
        }
    }
    return 0;
}

/* Probability vector of one row in fp64: the row itself (PROBS) or softmax(z / T) (LOGITS). */
static void row_probs(const void *rows, int dtype, int64_t r, int V, int mode, double temperature, double *p)
{
    const int64_t base = r * (int64_t)V;
    if (mode == FO_PROBS) {
        for (int v = 0; v < V; ++v)
            p[v] = load_elem(rows, base + v, dtype);
        return;
    }
    double m = -INFINITY;
    for (int v = 0; v < V; ++v) {
        const double z = load_elem(rows, base + v, dtype) / temperature;
        if (z > m)
            m = z;
    }
    double Z = 0.0;
    for (int v = 0; v < V; ++v) {
        p[v] = exp(load_elem(rows, base + v, dtype) / temperature - m);
        Z += p[v];
    }
    for (int v = 0; v < V; ++v)
        p[v] /= Z;
}

/*
 * Inverse CDF over non-negative masses r[0..V): first token whose running sum (index
 * order) is strictly greater than u * R, R = sum r.  Zero-mass tokens are never chosen;
 * if rounding leaves no such token the last positive-mass token is taken.  Returns -1 if
 * R == 0.  cdf_lo/cdf_hi receive the chosen token's interval [F(t-1), F(t)] / R;
 * tok_below/tok_above the nearest tokens of positive mass on either side of it (-1 if
 * there is none): the only other tokens a draw at the very edge of the interval can
 * reach.
 */
static int inverse_cdf(const double *r, int V, double u, double *cdf_lo, double *cdf_hi,
                       int32_t *tok_below, int32_t *tok_above)
{
    double R = 0.0;
    for (int v = 0; v < V; ++v)
        R += r[v];
    if (!(R > 0.0))
        return -1;
    const double thr = u * R;
    double c = 0.0;
    int last_pos = -1, before_last = -1;
    double last_lo = 0.0;
    for (int v = 0; v < V; ++v) {
        const double prev = c;
        c += r[v];
        if (r[v] > 0.0) {
            before_last = last_pos;
            last_pos = v;
            last_lo = prev;
            if (c > thr) {
                if (cdf_lo) *cdf_lo = prev / R;
                if (cdf_hi) *cdf_hi = c / R;
                if (tok_below) *tok_below = before_last;
                if (tok_above) {
                    *tok_above = -1;
                    for (int w = v + 1; w < V; ++w)
                        if (r[w] > 0.0) {
                            *tok_above = w;
                            break;
                        }
                }
                return v;
            }
        }
    }
    if (cdf_lo) *cdf_lo = last_lo / R;
    if (cdf_hi) *cdf_hi = 1.0;
    if (tok_below) *tok_below = before_last;
    if (tok_above) *tok_above = -1;
    return last_pos;
}

/*
 * Accept/reject of every request's drafts, recovery or bonus token.
 *
 * Request i has d_i = cu_d[i+1]-cu_d[i] draft rows and t_i = cu_t[i+1]-cu_t[i] target
 * rows, t_i in {d_i, d_i+1}.  Target row n is the target distribution at the position of
 * draft n; draft row n is the draft distribution that its draft token was drawn from.
 * Call-row r of the target side lives at storage row t_rows[r] of p_target (row r if
 * t_rows is null); call-row r of the draft side lives at storage row d_rows[r] (row r if
 * null) of p_draft, draft_tokens and u_accept alike.
 *
 *   n = 0; while n < d_i and u_accept[n] * q_n(x_n) < p_n(x_n): n++        (x_n = draft n)
 *   rejected (n < d_i): token ~ max(p_n - q_n, 0) normalised (p_n if that is all zero)
 *   all accepted and t_i = d_i+1: token ~ p_{d_i}
 *   all accepted and t_i = d_i: no extra token
 * Tokens are drawn by inverse CDF with the single u_sample[i].
 *
 * emitted is [B, S_max+1] padded with -1.  cdf_lo/cdf_hi (nullable, [B]) give the drawn
 * token's CDF interval (NaN if no token was drawn), tok_below/tok_above (nullable, [B]) the
 * nearest positive-mass tokens on either side of it in the row it was drawn from (-1 if
 * none, or if no token was drawn).  The rows are fp32, or bf16 bit patterns
 * (dtype), a bf16 value being the fp32 value with the same leading bits.
 */
int fo_spec_accept(const void *p_target, const void *p_draft, const int32_t *draft_tokens,
                   const float *u_accept, const float *u_sample, const int32_t *cu_t,
                   const int32_t *cu_d, const int32_t *t_rows, const int32_t *d_rows,
                   int32_t *accepted_len, int32_t *n_emitted, int32_t *emitted, double *cdf_lo,
                   double *cdf_hi, int32_t *tok_below, int32_t *tok_above, int B, int V, int S_max, int mode,
                   double temperature, int dtype)
{
    int status = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int i = 0; i < B; ++i) {
        const int d_i = cu_d[i + 1] - cu_d[i];
        const int t_i = cu_t[i + 1] - cu_t[i];
        int32_t *em = emitted + (int64_t)i * (S_max + 1);
        for (int s = 0; s <= S_max; ++s)
            em[s] = -1;
        if (cdf_lo) cdf_lo[i] = NAN;
        if (cdf_hi) cdf_hi[i] = NAN;
        if (tok_below) tok_below[i] = -1;
        if (tok_above) tok_above[i] = -1;
        accepted_len[i] = 0;
        n_emitted[i] = 0;
        if (d_i > S_max || t_i < d_i || t_i > d_i + 1) {
#pragma omp atomic write
            status = -2;
            continue;
        }
        double *p = (double *)malloc(sizeof(double) * (size_t)V);
        double *qv = (double *)malloc(sizeof(double) * (size_t)V);
        int n = 0;
        while (n < d_i) {
            const int64_t tr = t_rows ? t_rows[cu_t[i] + n] : cu_t[i] + n;
            const int64_t dr = d_rows ? d_rows[cu_d[i] + n] : cu_d[i] + n;
            const int x = draft_tokens[dr];
            double px, qx;
            if (mode == FO_PROBS) {
                px = load_elem(p_target, tr * V + x, dtype);
                qx = load_elem(p_draft, dr * V + x, dtype);
            } else {
                row_probs(p_target, dtype, tr, V, mode, temperature, p);
                row_probs(p_draft, dtype, dr, V, mode, temperature, qv);
                px = p[x];
                qx = qv[x];
            }
            if ((double)u_accept[dr] * qx < px) {
                em[n] = x;
                ++n;
            } else {
                break;
            }
        }
        accepted_len[i] = n;
        int tok = -1;
        if (n < d_i) { /* rejection at position n: recovery token from the residual */
            const int64_t tr = t_rows ? t_rows[cu_t[i] + n] : cu_t[i] + n;
            const int64_t dr = d_rows ? d_rows[cu_d[i] + n] : cu_d[i] + n;
            row_probs(p_target, dtype, tr, V, mode, temperature, p);
            row_probs(p_draft, dtype, dr, V, mode, temperature, qv);
            for (int v = 0; v < V; ++v) {
                const double r = p[v] - qv[v];
                qv[v] = r > 0.0 ? r : 0.0;
            }
            tok = inverse_cdf(qv, V, (double)u_sample[i], cdf_lo ? cdf_lo + i : 0, cdf_hi ? cdf_hi + i : 0,
                              tok_below ? tok_below + i : 0, tok_above ? tok_above + i : 0);
            if (tok < 0)
                tok = inverse_cdf(p, V, (double)u_sample[i], cdf_lo ? cdf_lo + i : 0, cdf_hi ? cdf_hi + i : 0,
                              tok_below ? tok_below + i : 0, tok_above ? tok_above + i : 0);
        } else if (t_i == d_i + 1) { /* everything accepted: bonus token from the extra target row */
            const int64_t tr = t_rows ? t_rows[cu_t[i] + d_i] : cu_t[i] + d_i;
            row_probs(p_target, dtype, tr, V, mode, temperature, p);
            tok = inverse_cdf(p, V, (double)u_sample[i], cdf_lo ? cdf_lo + i : 0, cdf_hi ? cdf_hi + i : 0,
                              tok_below ? tok_below + i : 0, tok_above ? tok_above + i : 0);
        }
        if (tok >= 0) {
            em[n] = tok;
            n_emitted[i] = n + 1;
        } else {
            n_emitted[i] = n;
        }
        free(p);
        free(qv);
    }
    return status;
}

/*
 * Greedy verification (Sec. 2.1 at temperature 0: accept the drafted tokens until the first
 * one that differs from the target's own choice, discard the rest, and take the target's
 * token at the first mismatch; with every draft accepted the extra target row gives the
 * bonus token).
 *
 * `target` is [rows, V] fp32, probabilities or logits alike: only the position of the row
 * maximum matters.  The arg-max of a row is the LOWEST token id holding the row's maximum.
 * A NaN score never wins against a number: it counts as minus infinity (so a row of NaN
 * alone yields token 0).
 * Row layout, t_rows / d_rows maps and outputs as in fo_spec_accept; no uniforms, no draft
 * distributions.
 *
 *   n = 0; while n < d_i and draft n == argmax(target row n): n++
 *   rejected (n < d_i): token = argmax(target row n)
 *   all accepted and t_i = d_i + 1: token = argmax(target row d_i)
 *   all accepted and t_i = d_i: no extra token
 */
static double greedy_score(float x)
{
    return x != x ? -INFINITY : (double)x;
}

static int argmax_row(const float *rows, int64_t r, int V)
{
    int best = 0;
    for (int v = 1; v < V; ++v)
        if (greedy_score(rows[r * V + v]) > greedy_score(rows[r * V + best]))
            best = v;
    return best;
}

int fo_greedy_accept(const float *target, const int32_t *draft_tokens, const int32_t *cu_t,
                     const int32_t *cu_d, const int32_t *t_rows, const int32_t *d_rows,
                     int32_t *accepted_len, int32_t *n_emitted, int32_t *emitted, int B, int V,
                     int S_max)
{
    int status = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int i = 0; i < B; ++i) {
        const int d_i = cu_d[i + 1] - cu_d[i];
        const int t_i = cu_t[i + 1] - cu_t[i];
        int32_t *em = emitted + (int64_t)i * (S_max + 1);
        for (int s = 0; s <= S_max; ++s)
            em[s] = -1;
        accepted_len[i] = 0;
        n_emitted[i] = 0;
        if (d_i > S_max || t_i < d_i || t_i > d_i + 1) {
#pragma omp atomic write
            status = -2;
            continue;
        }
        int n = 0, tok = -1;
        while (n < d_i) {
            const int64_t tr = t_rows ? t_rows[cu_t[i] + n] : cu_t[i] + n;
            const int64_t dr = d_rows ? d_rows[cu_d[i] + n] : cu_d[i] + n;
            const int choice = argmax_row(target, tr, V);
            if (draft_tokens[dr] != choice) {
                tok = choice; /* the target's token at the first mismatch */
                break;
            }
            em[n] = choice;
            ++n;
        }
        accepted_len[i] = n;
        if (n == d_i && t_i == d_i + 1) {
            const int64_t tr = t_rows ? t_rows[cu_t[i] + d_i] : cu_t[i] + d_i;
            tok = argmax_row(target, tr, V);
        }
        if (tok >= 0) {
            em[n] = tok;
            n_emitted[i] = n + 1;
        } else {
            n_emitted[i] = n;
        }
    }
    return status;
}

/*
 * Drop rows and re-pack the ragged batch.
 *
 * suffix_close != 0: request i keeps the leading run of 1s of its keep segment (the first
 * dropped row drops every later row of the request).  suffix_close == 0: it keeps exactly
 * the rows whose mask is non-zero, in order.
 *
 * new_cu_q [B+1], new_q_lens [B], src_row [N] (first new_cu_q[B] entries valid: new row ->
 * old row; the rest -1), dst_row [N] (old row -> new row or -1), active_ids [B] (ascending
 * requests with at least one kept row; the rest -1), *n_active.  If payload_in is given,
 * payload_out[r'] = payload_in[src_row[r']] for row_bytes bytes per row.
 */
int fo_prune_compact(const uint8_t *keep_mask, const int32_t *cu_q, int32_t *new_cu_q,
                     int32_t *new_q_lens, int32_t *src_row, int32_t *dst_row, int32_t *n_active,
                     int32_t *active_ids, const uint8_t *payload_in, uint8_t *payload_out,
                     int64_t row_bytes, int B, int suffix_close)
{
    const int N = cu_q[B];
    int out = 0, act = 0;
    for (int r = 0; r < N; ++r) {
        src_row[r] = -1;
        dst_row[r] = -1;
    }
    new_cu_q[0] = 0;
    for (int i = 0; i < B; ++i) {
        int kept = 0, open = 1;
        for (int r = cu_q[i]; r < cu_q[i + 1]; ++r) {
            const int k = keep_mask[r] != 0;
            if (!k && suffix_close)
                open = 0;
            if (k && open) {
                src_row[out] = r;
                dst_row[r] = out;
                ++out;
                ++kept;
            }
        }
        new_q_lens[i] = kept;
        new_cu_q[i + 1] = out;
        active_ids[i] = -1;
        if (kept > 0)
            active_ids[act++] = i;
    }
    *n_active = act;
    if (payload_in && payload_out)
        for (int r = 0; r < out; ++r)
            memcpy(payload_out + (int64_t)r * row_bytes, payload_in + (int64_t)src_row[r] * row_bytes,
                   (size_t)row_bytes);
    return 0;
}

/*
 * Inverse of the compaction: rows go back to their original positions; pruned rows are
 * filled with the byte `pad` and flagged 0 in has_value (Sec. 3.2 / Sec. 4: a dropped row has
 * no scores of its own; the original shape comes back with filler in its place).
 */
int fo_prune_restore(const uint8_t *compact, const int32_t *dst_row, uint8_t *restored,
                     uint8_t *has_value, int64_t row_bytes, int N, int pad)
{
    for (int r = 0; r < N; ++r) {
        if (dst_row[r] >= 0) {
            memcpy(restored + (int64_t)r * row_bytes, compact + (int64_t)dst_row[r] * row_bytes, (size_t)row_bytes);
            has_value[r] = 1;
        } else {
            memset(restored + (int64_t)r * row_bytes, pad, (size_t)row_bytes);
            has_value[r] = 0;
        }
    }
    return 0;
}

/*
 * Early-exit rank check (Sec. 3.2 token-level decision, Sec. 4 implementation note).
 *
 * Request i owns the logit rows cu_q[i] .. cu_q[i+1]-1 (its active query rows, q_i of them)
 * and the drafts cu_d[i] .. cu_d[i+1]-1 (d_i of them).  Row j holds the model's scores for
 * the token that follows the row's input, which is draft j of the request, so for
 * j < min(q_i, d_i)
 *     rank[cu_d[i] + j] = number of v with z[row j][v] > z[row j][draft j]      (strictly)
 * and the draft passes iff rank < K (it lies inside the Top-K set).  Drafts with no active
 * row get rank -1; a draft id outside [0, V) gets rank V (never passes).
 *
 * keep [N]: keep[cu_q[i]] = 1 (the row of the last committed token is never pruned);
 * keep[cu_q[i] + j + 1] = (rank of draft j < K) for j + 1 < q_i: the row whose input is
 * draft j survives iff draft j passes.  The mask is not suffix-closed here; fo_prune_compact
 * closes it.
 */
int fo_topk_rank_check(const void *logits, const int32_t *draft_tokens, const int32_t *cu_q,
                       const int32_t *cu_d, int32_t *rank, uint8_t *keep, int B, int V, int K,
                       int dtype)
{
    for (int i = 0; i < B; ++i) {
        const int q_i = cu_q[i + 1] - cu_q[i], d_i = cu_d[i + 1] - cu_d[i];
        for (int j = 0; j < d_i; ++j)
            rank[cu_d[i] + j] = -1;
        for (int j = 0; j < q_i; ++j)
            keep[cu_q[i] + j] = 1;
        for (int j = 0; j < q_i && j < d_i; ++j) {
            const int64_t row = cu_q[i] + j;
            const int tok = draft_tokens[cu_d[i] + j];
            int count = V;
            if (tok >= 0 && tok < V) {
                const double mine = load_elem(logits, row * V + tok, dtype);
                count = 0;
                for (int v = 0; v < V; ++v)
                    if (load_elem(logits, row * V + v, dtype) > mine)
                        ++count;
            }
            rank[cu_d[i] + j] = count;
            if (j + 1 < q_i)
                keep[cu_q[i] + j + 1] = count < K ? 1 : 0;
        }
    }
    return 0;
}

/*
 * Store the keys / values of this call's rows into the paged caches.
 *
 * Row j of request i (row cu_q[i] + j of k_new / v_new, each [N, H_kv, D]) is the token at
 * logical position t = ctx_lens[i] + j; it goes to page block_tables[i * max_pages + t / P],
 * slot t % P, of caches laid out [n_pages, H_kv, P, D].  Positions at or beyond max_pages * P
 * are not stored.  elem_bytes is the size of one element (2 for bf16, 4 for fp32); values
 * are copied bit for bit.
 */
int fo_kv_append(const void *k_new, const void *v_new, void *k_cache, void *v_cache,
                 const int32_t *block_tables, const int32_t *ctx_lens, const int32_t *cu_q, int B,
                 int H_kv, int D, int P, int max_pages, int elem_bytes)
{
    const int64_t vec = (int64_t)D * elem_bytes;
    for (int i = 0; i < B; ++i) {
        for (int r = cu_q[i]; r < cu_q[i + 1]; ++r) {
            const int64_t t = (int64_t)ctx_lens[i] + (r - cu_q[i]);
            if (t < 0 || t >= (int64_t)max_pages * P)
                continue;
            const int64_t page = block_tables[(int64_t)i * max_pages + t / P];
            for (int g = 0; g < H_kv; ++g) {
                const int64_t src = ((int64_t)r * H_kv + g) * vec;
                const int64_t dst = ((page * H_kv + g) * P + t % P) * vec;
                memcpy((uint8_t *)k_cache + dst, (const uint8_t *)k_new + src, (size_t)vec);
                memcpy((uint8_t *)v_cache + dst, (const uint8_t *)v_new + src, (size_t)vec);
            }
        }
    }
    return 0;
}
