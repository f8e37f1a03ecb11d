/*
 * CPU oracle for the CachedAttention new-turn prefill path (fp64, plain C).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct statement of
 * what the path computes.  It may be built and called from tests/, from the smoke
 * check and from the benchmark's cpu_baseline leg, and from nowhere else; the
 * product (the HIP library) shares no code, table or constant with it.
 *
 * What it follows (arXiv 2403.19708):
 *   - Section 2.1, attention equation: softmax(Q K^T / sqrt(d_K)) V, causal prefill
 *     (Section 2.2: token i sees tokens 1..i).
 *   - Section 3.1: the new turn's tokens are prefilled against the saved KV of the
 *     history instead of recomputing it; at one attention layer with K/V given this is
 *     the same function as attention over the whole (truncated) context, so the oracle
 *     IS that definition written out, restricted to the new tokens' query rows.
 *   - Section 3.4: keys are saved before the positional encoding; truncation drops the
 *     oldest tokens of the saved cache; on reuse the rotary encoding is embedded again
 *     at the positions the kept tokens have in the truncated context (0..Lk-1).
 *   - Section 3.2: layer-wise loading/saving is pure data movement; its oracle is the
 *     plain page/slot <-> contiguous copy loops below.
 *   - Section 4.2: KV bytes per token (closed form).
 *
 * Readings taken where the paper is silent (listed with reasons in the design notes):
 * rotary pairs are (i, i + D/2) ("rotate_half" convention) unless style = 1 selects
 * interleaved pairs (2i, 2i+1); theta_i = base^(-2i/D); the softmax scale is passed
 * in (1/sqrt(D) by convention); query head h reads KV head h / (Hq/Hkv); the causal
 * mask is index based: key t of the truncated context is visible to new token j iff
 * t <= n + j, n = kept history length.
 *
 * No blocking, no fusion, no reordering: every step is a separate loop in the order
 * the paper states it.  OpenMP only spreads independent query heads over cores.
 *
 * Parity pins (tests/test_oracle_*.py): brute-force recompute of the whole context,
 * rotation identities, shift invariance, softmax row sums, library SDPA on
 * pre-rotated inputs, closed forms printed in the paper.  No function here is
 * unpinned.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define CAO_OK 0
#define CAO_ERR_ARG 1
#define CAO_ERR_NOMEM 2

/* ---- Section 3.4: rotary position embedding of one head vector ------------------- */
/* x, out: [D]; pos may be any real (tests use shifted / negative positions).          */
void cao_rope(const double *x, int D, double pos, double base, int style, double *out)
{
    int half = D / 2;
    for (int i = 0; i < half; ++i) {
        double theta = pow(base, -2.0 * (double)i / (double)D);
        double ang = pos * theta;
        double c = cos(ang), s = sin(ang);
        int ia = (style == 0) ? i : 2 * i;
        int ib = (style == 0) ? i + half : 2 * i + 1;
        double a = x[ia], b = x[ib];
        out[ia] = a * c - b * s;
        out[ib] = b * c + a * s;
    }
}

/* ---- Section 2.1 attention with explicit positions --------------------------------- */
/*
 * K, V : [Lk][Hkv][D]   keys/values of the (already truncated) context, keys WITHOUT
 *                       positional encoding
 * Q    : [Ln][Hq][D]    queries of the new tokens, without positional encoding
 * kpos : [Lk], qpos : [Ln]  positions embedded into keys / queries
 * n    : number of context tokens that precede new token 0 (kept history length);
 *        key t is visible to new token j iff t <= n + j
 * O    : [Ln][Hq][D]    output
 * P    : optional [Hq][Ln][Lk] softmax probabilities (0 where masked), or NULL
 */
int cao_attention_positions(const double *K, const double *V, int Lk,
                            const double *Q, int Ln,
                            const double *kpos, const double *qpos, int n,
                            int Hq, int Hkv, int D, double base, int style, double scale,
                            double *O, double *P)
{
    if (Lk < 0 || Ln < 0 || n < 0 || Hq <= 0 || Hkv <= 0 || D <= 0 || (D & 1) || Hq % Hkv)
        return CAO_ERR_ARG;
    if (n + Ln > Lk && Ln > 0)
        return CAO_ERR_ARG; /* every new token must see at least itself */
    int G = Hq / Hkv;
    size_t nk = (size_t)Lk * Hkv * D, nq = (size_t)Ln * Hq * D;
    double *Rk = (double *)malloc((nk ? nk : 1) * sizeof(double));
    double *Rq = (double *)malloc((nq ? nq : 1) * sizeof(double));
    if (!Rk || !Rq) { free(Rk); free(Rq); return CAO_ERR_NOMEM; }

    /* step: embed positions into every key and every query (V is never rotated) */
    for (int t = 0; t < Lk; ++t)
        for (int g = 0; g < Hkv; ++g)
            cao_rope(K + ((size_t)t * Hkv + g) * D, D, kpos[t], base, style,
                     Rk + ((size_t)t * Hkv + g) * D);
    for (int j = 0; j < Ln; ++j)
        for (int h = 0; h < Hq; ++h)
            cao_rope(Q + ((size_t)j * Hq + h) * D, D, qpos[j], base, style,
                     Rq + ((size_t)j * Hq + h) * D);

    int fail = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int h = 0; h < Hq; ++h) {
        int g = h / G;
        double *z = (double *)malloc(((size_t)Lk + 1) * sizeof(double));
        if (!z) { fail = 1; continue; }
        for (int j = 0; j < Ln; ++j) {
            int vis = n + j + 1; /* keys 0 .. n+j */
            const double *q = Rq + ((size_t)j * Hq + h) * D;
            /* step: scores */
            double m = -INFINITY;
            for (int t = 0; t < vis; ++t) {
                const double *k = Rk + ((size_t)t * Hkv + g) * D;
                double acc = 0.0;
                for (int d = 0; d < D; ++d) acc += q[d] * k[d];
                z[t] = acc * scale;
                if (z[t] > m) m = z[t];
            }
            /* step: softmax over the visible keys */
            double sum = 0.0;
            for (int t = 0; t < vis; ++t) { z[t] = exp(z[t] - m); sum += z[t]; }
            for (int t = 0; t < vis; ++t) z[t] /= sum;
            if (P) {
                double *prow = P + ((size_t)h * Ln + j) * Lk;
                for (int t = 0; t < Lk; ++t) prow[t] = (t < vis) ? z[t] : 0.0;
            }
            /* step: weighted sum of values */
            double *o = O + ((size_t)j * Hq + h) * D;
            for (int d = 0; d < D; ++d) o[d] = 0.0;
            for (int t = 0; t < vis; ++t) {
                const double *v = V + ((size_t)t * Hkv + g) * D;
                for (int d = 0; d < D; ++d) o[d] += z[t] * v[d];
            }
        }
        free(z);
    }
    free(Rk);
    free(Rq);
    return fail ? CAO_ERR_NOMEM : CAO_OK;
}

/* ---- Sections 3.1 + 3.4: the new-turn prefill over a reused, truncated cache ------- */
/*
 * Kh, Vh : [Lh][Hkv][D]  saved history (keys saved before positional encoding)
 * Qn     : [Ln][Hq][D], Kn, Vn : [Ln][Hkv][D]  the new turn
 * keep_start : first history token that survives truncation (0 = none dropped)
 * pos_shift  : constant added to every position (0 in the method itself; non-zero
 *              only to test that the relative encoding does not care)
 */
int cao_cached_attention(const double *Kh, const double *Vh, int Lh,
                         const double *Qn, const double *Kn, const double *Vn, int Ln,
                         int keep_start, int Hq, int Hkv, int D,
                         double base, int style, double scale, double pos_shift,
                         double *O, double *P)
{
    if (Lh < 0 || Ln < 0 || keep_start < 0 || keep_start > Lh) return CAO_ERR_ARG;
    /* step: truncate the saved cache and append the new turn */
    int n = Lh - keep_start;
    int Lk = n + Ln;
    size_t row = (size_t)Hkv * D;
    double *K = (double *)malloc(((size_t)Lk * row + 1) * sizeof(double));
    double *V = (double *)malloc(((size_t)Lk * row + 1) * sizeof(double));
    double *kpos = (double *)malloc(((size_t)Lk + 1) * sizeof(double));
    double *qpos = (double *)malloc(((size_t)Ln + 1) * sizeof(double));
    if (!K || !V || !kpos || !qpos) { free(K); free(V); free(kpos); free(qpos); return CAO_ERR_NOMEM; }
    for (int t = 0; t < n; ++t) {
        memcpy(K + (size_t)t * row, Kh + (size_t)(keep_start + t) * row, row * sizeof(double));
        memcpy(V + (size_t)t * row, Vh + (size_t)(keep_start + t) * row, row * sizeof(double));
    }
    for (int j = 0; j < Ln; ++j) {
        memcpy(K + (size_t)(n + j) * row, Kn + (size_t)j * row, row * sizeof(double));
        memcpy(V + (size_t)(n + j) * row, Vn + (size_t)j * row, row * sizeof(double));
    }
    /* step: positions of the truncated context start again at 0 */
    for (int t = 0; t < Lk; ++t) kpos[t] = (double)t + pos_shift;
    for (int j = 0; j < Ln; ++j) qpos[j] = (double)(n + j) + pos_shift;
    int rc = cao_attention_positions(K, V, Lk, Qn, Ln, kpos, qpos, n, Hq, Hkv, D,
                                     base, style, scale, O, P);
    free(K); free(V); free(kpos); free(qpos);
    return rc;
}

/* ---- Section 3.4 / 4.1: which tokens survive a context-window overflow -------------- */
/*
 * Overflow iff hist + new > W.  The kept tokens are always the most recent ones.
 * policy 0: keep the most recent floor(W*(1-ratio)) tokens of the context
 *           (history + new); the new turn is never dropped.
 * policy 1: drop floor(W*ratio) oldest tokens, again while the context still overflows
 *           (the passage that drops the oldest 2K tokens of a 4K window).
 * policy 2: drop the earliest floor(ratio * context) tokens, again while it still
 *           overflows (the passage that reads ratio 0.5 as dropping the older half of the tokens).
 * keep_start_out[c] = index of the first surviving history token (<= hist).
 */
int cao_truncate_plan(const int32_t *hist_len, const int32_t *new_len, int32_t W, double ratio,
                      int policy, int B, int32_t *keep_start_out)
{
    if (W <= 0 || !(ratio > 0.0) || !(ratio < 1.0) || policy < 0 || policy > 2) return CAO_ERR_ARG;
    for (int c = 0; c < B; ++c) {
        int64_t Lh = hist_len[c], Ln = new_len[c];
        if (Lh < 0 || Ln < 0) return CAO_ERR_ARG;
        int64_t s = 0;
        if (Lh + Ln > W) {
            if (policy == 0) {
                int64_t target = (int64_t)floor((double)W * (1.0 - ratio));
                int64_t n = target - Ln;
                if (n < 0) n = 0;
                if (n > Lh) n = Lh;
                s = Lh - n;
            } else if (policy == 1) {
                int64_t drop = (int64_t)floor((double)W * ratio);
                if (drop < 1) drop = 1;
                while ((Lh - s) + Ln > W && s < Lh) { s += drop; if (s > Lh) s = Lh; }
            } else {
                while ((Lh - s) + Ln > W && s < Lh) {
                    int64_t drop = (int64_t)floor(ratio * (double)((Lh - s) + Ln));
                    if (drop < 1) drop = 1;
                    s += drop; if (s > Lh) s = Lh;
                }
            }
        }
        keep_start_out[c] = (int32_t)s;
    }
    return CAO_OK;
}

/* ---- Section 3.4: integer bookkeeping after truncation ------------------------------ */
/*
 * For a batch: n_keep[c] = hist - keep_start; cu_q/cu_k = exclusive prefix sums of the
 * new-token counts / context lengths (B+1 entries); q_pos[cu_q[c]+j] = n_keep[c]+j;
 * q_seq[cu_q[c]+j] = c; slot_map[cu_k[c]+t] = page*P + t%P with
 * page = block_table[c][t/P] (where context token t lives in the paged pool).
 */
int cao_rebase(int B, const int32_t *hist_len, const int32_t *keep_start, const int32_t *new_len,
               const int32_t *block_table, int max_pages, int P,
               int32_t *n_keep, int32_t *cu_q, int32_t *cu_k,
               int32_t *q_pos, int32_t *q_seq, int32_t *slot_map)
{
    cu_q[0] = 0; cu_k[0] = 0;
    for (int c = 0; c < B; ++c) {
        if (keep_start[c] < 0 || keep_start[c] > hist_len[c] || new_len[c] < 0) return CAO_ERR_ARG;
        n_keep[c] = hist_len[c] - keep_start[c];
        cu_q[c + 1] = cu_q[c] + new_len[c];
        cu_k[c + 1] = cu_k[c] + n_keep[c] + new_len[c];
        if ((n_keep[c] + new_len[c] + P - 1) / P > max_pages) return CAO_ERR_ARG;
    }
    for (int c = 0; c < B; ++c) {
        for (int j = 0; j < new_len[c]; ++j) {
            q_pos[cu_q[c] + j] = n_keep[c] + j;
            q_seq[cu_q[c] + j] = c;
        }
        int Lk = n_keep[c] + new_len[c];
        for (int t = 0; t < Lk; ++t) {
            int32_t page = block_table[(size_t)c * max_pages + t / P];
            slot_map[cu_k[c] + t] = page * P + t % P;
        }
    }
    return CAO_OK;
}

/* ---- Section 3.2: data movement between the paged pool and contiguous token rows ----- */
/*
 * pool   : [num_pages][Hkv][P][D] elements of esize bytes
 * contig : [tokens][Hkv][D]
 * table  : this conversation's row of the block table
 * unpack: contig token (src_tok0 + i) -> context token (dst_tok0 + i), i < count
 * pack  : context token (src_tok0 + i) -> contig token (dst_tok0 + i)
 */
void cao_unpack(const uint8_t *contig, int64_t src_tok0, uint8_t *pool, const int32_t *table,
                int P, int Hkv, int D, int esize, int dst_tok0, int count)
{
    size_t vec = (size_t)D * esize;
    for (int i = 0; i < count; ++i) {
        int t = dst_tok0 + i;
        int32_t page = table[t / P];
        int slot = t % P;
        for (int h = 0; h < Hkv; ++h) {
            const uint8_t *src = contig + ((size_t)(src_tok0 + i) * Hkv + h) * vec;
            uint8_t *dst = pool + (((size_t)page * Hkv + h) * P + slot) * vec;
            for (size_t b = 0; b < vec; ++b) dst[b] = src[b];
        }
    }
}

void cao_pack(const uint8_t *pool, const int32_t *table, int P, int Hkv, int D, int esize,
              int src_tok0, int count, uint8_t *contig, int64_t dst_tok0)
{
    size_t vec = (size_t)D * esize;
    for (int i = 0; i < count; ++i) {
        int t = src_tok0 + i;
        int32_t page = table[t / P];
        int slot = t % P;
        for (int h = 0; h < Hkv; ++h) {
            const uint8_t *src = pool + (((size_t)page * Hkv + h) * P + slot) * vec;
            uint8_t *dst = contig + ((size_t)(dst_tok0 + i) * Hkv + h) * vec;
            for (size_t b = 0; b < vec; ++b) dst[b] = src[b];
        }
    }
}

/* ---- Section 4.2: KV-cache footprint of one token over all layers (K and V) --------- */
int64_t cao_kv_bytes_per_token(int n_layers, int n_kv_heads, int head_dim, int esize)
{
    return (int64_t)2 * n_layers * n_kv_heads * head_dim * esize;
}
