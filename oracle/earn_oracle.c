/*
 * CPU oracle for the EARN register-token attention path.  TEST INFRASTRUCTURE ONLY:
 * it exists to check the HIP library and to be timed as a CPU baseline; nothing in the
 * product path may call it, and it shares no code with the HIP sources.
 *
 * Everything is fp64 and written as the plain definition: materialise one softmax row,
 * then take the weighted sum.  No tiling, no online softmax, no fusion.
 *
 *   Attention            O = Softmax(Q K^T / sqrt(d)) V                  (paper Section 2.2, Eq. 3)
 *   Decode step          append (K_t, V_t) to the cache, then Q_t K_{1:t}^T   (Section 2.2, Eq. 4)
 *   Input layout         X = [R_prefix; Prompt; R_suffix]                (Section 3.2, Eq. 5)
 *   Register compaction  X -> X' = [X_prefix; X_suffix] at the input of layer k
 *                                                                       (Section 3.2, "Inference", item 2)
 *   Cache accounting     N_KV = n_h (k L + (N-k) r), Gamma_cache, Gamma_attn, FLOPs per layer
 *                                                                       (Section 3.3; Appendix A.2)
 *
 * Readings where the paper is silent (each listed in the design notes of the repository):
 * causal mask in every prefill layer; scale 1/sqrt(head_dim); rotary position embedding with
 * half-split pairs (i, i + d/2), theta_i = base^(-2i/d), applied to Q and K at each token's
 * ORIGINAL position (a suffix register keeps position h + L + j after compaction);
 * grouped-query map q head a -> kv head a / (Hq/Hkv) unless an explicit map is given.
 *
 * All tensors are row-major, packed ragged: [tokens, heads, d].
 * Every function returns 0 on success and a negative code on an invalid argument.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_OK 0
#define ORC_BAD_ARG (-1)
#define ORC_NO_MEM (-2)

/* ---- rotary embedding at an absolute position (reading of "RoPE at original positions") ---- */
static void rope_vec(const double *x, int d, double pos, double base, double *y)
{
    int half = d / 2;
    if (base <= 0.0) {
        memcpy(y, x, sizeof(double) * (size_t)d);
        return;
    }
    for (int i = 0; i < half; ++i) {
        double theta = pow(base, -2.0 * (double)i / (double)d);
        double c = cos(pos * theta), s = sin(pos * theta);
        y[i] = x[i] * c - x[i + half] * s;
        y[i + half] = x[i + half] * c + x[i] * s;
    }
}

int oracle_rope(const double *x, const int32_t *pos, int64_t rows, int32_t heads, int32_t d, double base, double *y)
{
    if (!x || !pos || !y || rows < 0 || heads <= 0 || d <= 0 || (d & 1)) return ORC_BAD_ARG;
    for (int64_t r = 0; r < rows; ++r)
        for (int h = 0; h < heads; ++h)
            rope_vec(x + (r * heads + h) * d, d, (double)pos[r], base, y + (r * heads + h) * d);
    return ORC_OK;
}

static int kv_head_of(int a, int hq, int hkv, const int32_t *map) { return map ? map[a] : a / (hq / hkv); }

static int check_heads(int hq, int hkv, int d, const int32_t *map)
{
    if (hq <= 0 || hkv <= 0 || d <= 0 || (d & 1)) return ORC_BAD_ARG;
    if (!map && hq % hkv != 0) return ORC_BAD_ARG;
    if (map)
        for (int a = 0; a < hq; ++a)
            if (map[a] < 0 || map[a] >= hkv) return ORC_BAD_ARG;
    return ORC_OK;
}

/* One softmax row over scores[0..m): p_j = exp(s_j - max) / sum; returns log-sum-exp. */
static double softmax_row(const double *s, int64_t m, double *p)
{
    double mx = s[0];
    for (int64_t j = 1; j < m; ++j) if (s[j] > mx) mx = s[j];
    double sum = 0.0;
    for (int64_t j = 0; j < m; ++j) { p[j] = exp(s[j] - mx); sum += p[j]; }
    for (int64_t j = 0; j < m; ++j) p[j] /= sum;
    return mx + log(sum);
}

/*
 * Causal attention over a packed ragged batch (Eq. 3 per sequence and head).
 *   q [T,Hq,d]; k, v [T,Hkv,d]; cu_seqlens [batch+1]; positions [T] or NULL (= index within the sequence).
 *   row_sel [T] or NULL: only rows with row_sel != 0 are computed (others left untouched).
 *   out [T,Hq,d]; k_rot_out [T,Hkv,d] or NULL (the layer's cache: rotated K);
 *   lse_out [T,Hq] or NULL; rowsum_out [T,Hq] or NULL (sum of the materialised probabilities);
 *   probs_out or NULL: dense [n,n] probabilities of (probs_seq, probs_head), zero above the diagonal.
 */
int oracle_prefill_attn(const double *q, const double *k, const double *v, const int32_t *cu_seqlens,
                        const int32_t *positions, int32_t batch, int32_t hq, int32_t hkv, int32_t d,
                        const int32_t *q_to_kv, double scale, double rope_base, const uint8_t *row_sel, double *out,
                        double *k_rot_out, double *lse_out, double *rowsum_out, double *probs_out, int32_t probs_seq,
                        int32_t probs_head)
{
    if (!q || !k || !v || !cu_seqlens || !out || batch <= 0) return ORC_BAD_ARG;
    int rc = check_heads(hq, hkv, d, q_to_kv);
    if (rc) return rc;
    for (int s = 0; s < batch; ++s) if (cu_seqlens[s + 1] < cu_seqlens[s]) return ORC_BAD_ARG;
    if (cu_seqlens[0] != 0) return ORC_BAD_ARG;
    if (scale <= 0.0) scale = 1.0 / sqrt((double)d);
    int64_t total = cu_seqlens[batch];

    /* rotate every key once (this is what the cache stores) */
    double *kr = (double *)malloc(sizeof(double) * (size_t)(total > 0 ? total : 1) * hkv * d);
    if (!kr) return ORC_NO_MEM;
    for (int s = 0; s < batch; ++s)
        for (int64_t i = cu_seqlens[s]; i < cu_seqlens[s + 1]; ++i) {
            double p = positions ? (double)positions[i] : (double)(i - cu_seqlens[s]);
            for (int c = 0; c < hkv; ++c) rope_vec(k + (i * hkv + c) * d, d, p, rope_base, kr + (i * hkv + c) * d);
        }
    if (k_rot_out) memcpy(k_rot_out, kr, sizeof(double) * (size_t)total * hkv * d);

    int err = 0;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int s = 0; s < batch; ++s)
        for (int a = 0; a < hq; ++a) {
            int64_t b0 = cu_seqlens[s], n = cu_seqlens[s + 1] - b0;
            if (n == 0) continue;
            int c = kv_head_of(a, hq, hkv, q_to_kv);
            double *sc = (double *)malloc(sizeof(double) * (size_t)n * 2);
            double *qr = (double *)malloc(sizeof(double) * (size_t)d);
            if (!sc || !qr) { err = 1; free(sc); free(qr); continue; }
            double *pr = sc + n;
            for (int64_t i = 0; i < n; ++i) {
                int64_t gi = b0 + i;
                if (row_sel && !row_sel[gi]) continue;
                double p = positions ? (double)positions[gi] : (double)i;
                rope_vec(q + (gi * hq + a) * d, d, p, rope_base, qr);
                for (int64_t j = 0; j <= i; ++j) { /* causal: keys 0..i */
                    const double *kj = kr + ((b0 + j) * hkv + c) * d;
                    double acc = 0.0;
                    for (int e = 0; e < d; ++e) acc += qr[e] * kj[e];
                    sc[j] = acc * scale;
                }
                double lse = softmax_row(sc, i + 1, pr);
                double *o = out + (gi * hq + a) * d;
                for (int e = 0; e < d; ++e) o[e] = 0.0;
                double rs = 0.0;
                for (int64_t j = 0; j <= i; ++j) {
                    const double *vj = v + ((b0 + j) * hkv + c) * d;
                    for (int e = 0; e < d; ++e) o[e] += pr[j] * vj[e];
                    rs += pr[j];
                }
                if (lse_out) lse_out[gi * hq + a] = lse;
                if (rowsum_out) rowsum_out[gi * hq + a] = rs;
                if (probs_out && s == probs_seq && a == probs_head) {
                    for (int64_t j = 0; j < n; ++j) probs_out[i * n + j] = j <= i ? pr[j] : 0.0;
                }
            }
            free(sc);
            free(qr);
        }
    free(kr);
    return err ? ORC_NO_MEM : ORC_OK;
}

/*
 * Register compaction (Section 3.2, Inference item 2, prefilling bullet): keep rows [0,h) and [n_s-t, n_s)
 * of every sequence, in order.  Pure byte gather of `src` rows of `row_bytes` bytes.
 *   idx_out[m] = source row in the packed tensor; pos_out[m] = original position within the sequence;
 *   cu_out[s] = s*(h+t).  src/dst may be NULL to compute the index outputs only.
 */
int oracle_compact_registers(const uint8_t *src, int64_t row_bytes, const int32_t *cu_seqlens, int32_t batch,
                             int32_t n_head_reg, int32_t n_tail_reg, uint8_t *dst, int32_t *idx_out,
                             int32_t *pos_out, int32_t *cu_out)
{
    if (!cu_seqlens || batch <= 0 || n_head_reg < 0 || n_tail_reg < 0 || n_head_reg + n_tail_reg == 0)
        return ORC_BAD_ARG;
    if ((src == NULL) != (dst == NULL) || (src && row_bytes <= 0)) return ORC_BAD_ARG;
    int r = n_head_reg + n_tail_reg;
    for (int s = 0; s < batch; ++s)
        if (cu_seqlens[s + 1] - cu_seqlens[s] < r) return ORC_BAD_ARG;
    for (int s = 0; s < batch; ++s) {
        int32_t b0 = cu_seqlens[s], n = cu_seqlens[s + 1] - b0;
        for (int m = 0; m < r; ++m) {
            int32_t p = m < n_head_reg ? m : n - n_tail_reg + (m - n_head_reg);
            int64_t o = (int64_t)s * r + m;
            if (idx_out) idx_out[o] = b0 + p;
            if (pos_out) pos_out[o] = p;
            if (src) memcpy(dst + o * row_bytes, src + (int64_t)(b0 + p) * row_bytes, (size_t)row_bytes);
        }
        if (cu_out) cu_out[s] = s * r;
    }
    if (cu_out) cu_out[batch] = batch * r;
    return ORC_OK;
}

/*
 * One decode step (Eq. 4): for every stream u of sequence s = stream_to_seq[u], rotate q and k_new at position
 * q_pos[u], append (k_new', v_new) at slot gen_len[u] of the stream's generated cache, then attend over the
 * sequence's shared cache rows followed by the stream's gen_len[u]+1 generated rows.  No mask: all keys are past.
 *   shared_k (already rotated), shared_v [sum_len,Hkv,d]; shared_cu [batch+1];
 *   gen_k, gen_v [S,gen_cap,Hkv,d] updated in place; out [S,Hq,d]; lse_out [S,Hq] or NULL.
 */
int oracle_decode_attn(const double *q, const double *k_new, const double *v_new, const int32_t *q_pos,
                       const double *shared_k, const double *shared_v, const int32_t *shared_cu,
                       const int32_t *stream_to_seq, double *gen_k, double *gen_v, const int32_t *gen_len,
                       int32_t gen_cap, int32_t n_streams, int32_t batch, int32_t hq, int32_t hkv, int32_t d,
                       const int32_t *q_to_kv, double scale, double rope_base, double *out, double *lse_out,
                       double *rowsum_out)
{
    if (!q || !k_new || !v_new || !q_pos || !shared_cu || !gen_k || !gen_v || !gen_len || !out) return ORC_BAD_ARG;
    if (n_streams <= 0 || batch <= 0 || gen_cap <= 0) return ORC_BAD_ARG;
    int rc = check_heads(hq, hkv, d, q_to_kv);
    if (rc) return rc;
    if (scale <= 0.0) scale = 1.0 / sqrt((double)d);
    for (int u = 0; u < n_streams; ++u) {
        int s = stream_to_seq ? stream_to_seq[u] : u;
        if (s < 0 || s >= batch || gen_len[u] < 0 || gen_len[u] >= gen_cap) return ORC_BAD_ARG;
    }
    if (shared_cu[batch] > 0 && (!shared_k || !shared_v)) return ORC_BAD_ARG;
    int err = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int u = 0; u < n_streams; ++u) {
        int s = stream_to_seq ? stream_to_seq[u] : u;
        int64_t b0 = shared_cu[s], ns = shared_cu[s + 1] - b0;
        int64_t g = gen_len[u], m = ns + g + 1;
        double *gk = gen_k + (int64_t)u * gen_cap * hkv * d, *gv = gen_v + (int64_t)u * gen_cap * hkv * d;
        for (int c = 0; c < hkv; ++c) { /* cache append, Eq. 4 */
            rope_vec(k_new + ((int64_t)u * hkv + c) * d, d, (double)q_pos[u], rope_base, gk + (g * hkv + c) * d);
            memcpy(gv + (g * hkv + c) * d, v_new + ((int64_t)u * hkv + c) * d, sizeof(double) * (size_t)d);
        }
        double *sc = (double *)malloc(sizeof(double) * (size_t)m * 2);
        double *qr = (double *)malloc(sizeof(double) * (size_t)d);
        if (!sc || !qr) { err = 1; free(sc); free(qr); continue; }
        double *pr = sc + m;
        for (int a = 0; a < hq; ++a) {
            int c = kv_head_of(a, hq, hkv, q_to_kv);
            rope_vec(q + ((int64_t)u * hq + a) * d, d, (double)q_pos[u], rope_base, qr);
            for (int64_t j = 0; j < m; ++j) {
                const double *kj = j < ns ? shared_k + ((b0 + j) * hkv + c) * d : gk + ((j - ns) * hkv + c) * d;
                double acc = 0.0;
                for (int e = 0; e < d; ++e) acc += qr[e] * kj[e];
                sc[j] = acc * scale;
            }
            double lse = softmax_row(sc, m, pr);
            double *o = out + ((int64_t)u * hq + a) * d;
            for (int e = 0; e < d; ++e) o[e] = 0.0;
            double rs = 0.0;
            for (int64_t j = 0; j < m; ++j) {
                const double *vj = j < ns ? shared_v + ((b0 + j) * hkv + c) * d : gv + ((j - ns) * hkv + c) * d;
                for (int e = 0; e < d; ++e) o[e] += pr[j] * vj[e];
                rs += pr[j];
            }
            if (lse_out) lse_out[(int64_t)u * hq + a] = lse;
            if (rowsum_out) rowsum_out[(int64_t)u * hq + a] = rs;
        }
        free(sc);
        free(qr);
    }
    return err ? ORC_NO_MEM : ORC_OK;
}

/* ---- accounting (Section 3.3 and Appendix A.2) ---- */

/* KV entries per attention head kept for one sequence: the first k layers keep all n tokens, the remaining N-k
 * keep the r registers; every layer also keeps the `gen` generated tokens. (N_KV = n_h (k L + (N-k) r).) */
int64_t oracle_cache_entries(int32_t n_layers, int32_t split_k, int64_t n, int32_t r, int64_t gen)
{
    return (int64_t)split_k * n + (int64_t)(n_layers - split_k) * r + (int64_t)n_layers * gen;
}

/* Gamma_cache = 1 - (k L + (N-k) r) / (N L). */
double oracle_gamma_cache(int32_t n_layers, int32_t split_k, double L, double r)
{
    return 1.0 - ((double)split_k * L + (double)(n_layers - split_k) * r) / ((double)n_layers * L);
}

/* FLOPs of one decoder layer at length L: n_h (8 L d_h d_a + 4 L^2 d_a) + 4 L d_h d_f. */
double oracle_flops_layer(double L, double n_h, double d_a, double d_h, double d_f)
{
    return n_h * (8.0 * L * d_h * d_a + 4.0 * L * L * d_a) + 4.0 * L * d_h * d_f;
}

/* Gamma_attn = (k F(L) + (N-k) F(r)) / (N F(L)). */
double oracle_gamma_attn(int32_t n_layers, int32_t split_k, double L, double r, double n_h, double d_a, double d_h,
                         double d_f)
{
    double fl = oracle_flops_layer(L, n_h, d_a, d_h, d_f), fr = oracle_flops_layer(r, n_h, d_a, d_h, d_f);
    return ((double)split_k * fl + (double)(n_layers - split_k) * fr) / ((double)n_layers * fl);
}

/* Causal attention FLOPs actually required for one layer: 4 d Hq sum_s m_s (m_s + 1) / 2
 * (2d for QK^T and 2d for PV per allowed (query, key) pair). */
double oracle_causal_attn_flops(const int32_t *lengths, int32_t batch, int32_t hq, int32_t d)
{
    double pairs = 0.0;
    for (int s = 0; s < batch; ++s) pairs += 0.5 * (double)lengths[s] * ((double)lengths[s] + 1.0);
    return 4.0 * (double)d * (double)hq * pairs;
}

/*
 * Attention-score statistics of chosen query rows (Appendix, "Quantitative Measurements of Attention Score
 * Distributions").  For the causal softmax row p_1..p_n of query row i (n = i + 1 visible keys, Eq. 3):
 *   Sparsity  = (1/n) * #{ j : p_j > epsilon }                      (epsilon = 0.05 in the paper)
 *   Sink_head = sum_{j = 1}^{T_h} p_j                               (T_h = 3)
 *   Sink_tail = sum_{j = T_t}^{n} p_j, T_t = n - tail_back          (tail_back = 3: the LAST FOUR keys, as printed)
 * Rows shorter than the windows sum what exists.  The probabilities are materialised exactly as in
 * oracle_prefill_attn (rotation at the original positions, scale, one softmax row at a time).
 *   q [T,Hq,d], k [T,Hkv,d] (un-rotated), rows: row_sel [T] != 0.  stats_out [T,Hq,3], rows not selected untouched.
 */
int oracle_attn_stats(const double *q, const double *k, const int32_t *cu_seqlens, const int32_t *positions,
                      int32_t batch, int32_t hq, int32_t hkv, int32_t d, const int32_t *q_to_kv, double scale,
                      double rope_base, const uint8_t *row_sel, double epsilon, int32_t t_head, int32_t tail_back,
                      double *stats_out)
{
    if (!q || !k || !cu_seqlens || !stats_out || batch <= 0 || t_head < 0 || tail_back < 0) return ORC_BAD_ARG;
    int rc = check_heads(hq, hkv, d, q_to_kv);
    if (rc) return rc;
    if (scale <= 0.0) scale = 1.0 / sqrt((double)d);
    int err = 0;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int s = 0; s < batch; ++s)
        for (int a = 0; a < hq; ++a) {
            int64_t b0 = cu_seqlens[s], n = cu_seqlens[s + 1] - b0;
            if (n <= 0) continue;
            int c = kv_head_of(a, hq, hkv, q_to_kv);
            double *sc = (double *)malloc(sizeof(double) * (size_t)n * 2);
            double *qr = (double *)malloc(sizeof(double) * (size_t)d * 2);
            if (!sc || !qr) { err = 1; free(sc); free(qr); continue; }
            double *pr = sc + n, *kr = qr + d;
            for (int64_t i = 0; i < n; ++i) {
                int64_t gi = b0 + i;
                if (row_sel && !row_sel[gi]) continue;
                double p = positions ? (double)positions[gi] : (double)i;
                rope_vec(q + (gi * hq + a) * d, d, p, rope_base, qr);
                for (int64_t j = 0; j <= i; ++j) {
                    double pj = positions ? (double)positions[b0 + j] : (double)j;
                    rope_vec(k + ((b0 + j) * hkv + c) * d, d, pj, rope_base, kr);
                    double acc = 0.0;
                    for (int e = 0; e < d; ++e) acc += qr[e] * kr[e];
                    sc[j] = acc * scale;
                }
                softmax_row(sc, i + 1, pr);
                int64_t m = i + 1, count = 0;
                double head = 0.0, tail = 0.0;
                for (int64_t j = 1; j <= m; ++j) { /* 1-based, as the paper writes the sums */
                    double pj = pr[j - 1];
                    if (pj > epsilon) ++count;
                    if (j <= t_head) head += pj;
                    if (j >= m - tail_back) tail += pj;
                }
                double *o = stats_out + (gi * hq + a) * 3;
                o[0] = (double)count / (double)m;
                o[1] = head;
                o[2] = tail;
            }
            free(sc);
            free(qr);
        }
    return err ? ORC_NO_MEM : ORC_OK;
}

/*
 * One selection step of beam search (the paper decodes with beam search, beam size 20: Appendix, implementation
 * details).  For every sequence b with `beams` live beams and `vocab` tokens, candidate (w, t) scores
 * beam_scores[b, w] + token_logprobs[b, w, t]; the `beams` best candidates are kept, best first, equal scores in order
 * of the candidate index w * vocab + t.  The sum is taken in fp32 (the inputs' precision: the comparison that decides
 * an index must see the same numbers on every implementation).  A NaN candidate never wins.
 *   parent_out[b, r] = b * beams + w of pick r (a stream index), token_out[b, r] = t, score_out[b, r] = the score;
 *   -1 / -1 / -inf when a sequence has fewer candidates than beams.
 * Written as the definition: `beams` rounds, each taking the best candidate not taken before.
 */
int oracle_beam_topk(const float *beam_scores, const float *token_logprobs, int32_t batch, int32_t beams, int32_t vocab,
                     int32_t *parent_out, int32_t *token_out, float *score_out)
{
    if (!token_logprobs || !parent_out || !token_out || !score_out || batch <= 0 || beams <= 0 || vocab <= 0)
        return ORC_BAD_ARG;
    int64_t n = (int64_t)beams * vocab;
    uint8_t *taken = (uint8_t *)malloc((size_t)n);
    float *cand = (float *)malloc(sizeof(float) * (size_t)n);
    if (!taken || !cand) { free(taken); free(cand); return ORC_NO_MEM; }
    for (int b = 0; b < batch; ++b) {
        for (int64_t c = 0; c < n; ++c) {
            float bs = beam_scores ? beam_scores[(int64_t)b * beams + c / vocab] : 0.0f;
            volatile float sum = token_logprobs[(int64_t)b * n + c] + bs; /* rounded to fp32 */
            cand[c] = sum == sum ? sum : -INFINITY;
            taken[c] = 0;
        }
        for (int r = 0; r < beams; ++r) {
            int64_t best = -1;
            for (int64_t c = 0; c < n; ++c)
                if (!taken[c] && (best < 0 || cand[c] > cand[best])) best = c; /* first of equals: lowest index */
            int64_t o = (int64_t)b * beams + r;
            if (best < 0) { parent_out[o] = -1; token_out[o] = -1; score_out[o] = -INFINITY; continue; }
            taken[best] = 1;
            parent_out[o] = (int32_t)(b * beams + best / vocab);
            token_out[o] = (int32_t)(best % vocab);
            score_out[o] = cand[best];
        }
    }
    free(taken);
    free(cand);
    return ORC_OK;
}

/*
 * Backward of the causal attention of Eq. 3 (what training, Section 3.2, differentiates through), for queries and keys
 * AS THE ATTENTION SAW THEM (already rotated; this function rotates nothing).  For every sequence, query head a and its
 * kv head c, with P the materialised causal softmax of scale * Q K^T:
 *   dV += P^T dO;   dP = dO V^T;   dS = P o (dP - rowsum(dP o P));   dQ = scale dS K;   dK += scale dS^T Q
 * (dK, dV sum over the query heads that share the kv head).  q, d_out, dq [T,Hq,d]; k, v, dk, dv [T,Hkv,d].
 * The row sum is taken as rowsum(dP o P), the definition of the softmax Jacobian, not as rowsum(dO o O).
 */
int oracle_attn_backward(const double *q, const double *k, const double *v, const double *d_out,
                         const int32_t *cu_seqlens, int32_t batch, int32_t hq, int32_t hkv, int32_t d,
                         const int32_t *q_to_kv, double scale, double *dq, double *dk, double *dv)
{
    if (!q || !k || !v || !d_out || !cu_seqlens || !dq || !dk || !dv || batch <= 0) return ORC_BAD_ARG;
    int rc = check_heads(hq, hkv, d, q_to_kv);
    if (rc) return rc;
    if (scale <= 0.0) scale = 1.0 / sqrt((double)d);
    int64_t total = cu_seqlens[batch];
    memset(dk, 0, sizeof(double) * (size_t)total * hkv * d);
    memset(dv, 0, sizeof(double) * (size_t)total * hkv * d);
    for (int s = 0; s < batch; ++s) {
        int64_t b0 = cu_seqlens[s], n = cu_seqlens[s + 1] - b0;
        if (n <= 0) continue;
        double *sc = (double *)malloc(sizeof(double) * (size_t)n * 3);
        if (!sc) return ORC_NO_MEM;
        double *pr = sc + n, *dp = sc + 2 * n;
        for (int a = 0; a < hq; ++a) {
            int c = kv_head_of(a, hq, hkv, q_to_kv);
            for (int64_t i = 0; i < n; ++i) {
                const double *qi = q + ((b0 + i) * hq + a) * d, *gi = d_out + ((b0 + i) * hq + a) * d;
                for (int64_t j = 0; j <= i; ++j) {
                    const double *kj = k + ((b0 + j) * hkv + c) * d;
                    double acc = 0.0;
                    for (int e = 0; e < d; ++e) acc += qi[e] * kj[e];
                    sc[j] = acc * scale;
                }
                softmax_row(sc, i + 1, pr);
                double rowsum = 0.0;
                for (int64_t j = 0; j <= i; ++j) {
                    const double *vj = v + ((b0 + j) * hkv + c) * d;
                    double acc = 0.0;
                    for (int e = 0; e < d; ++e) acc += gi[e] * vj[e];
                    dp[j] = acc;
                    rowsum += acc * pr[j];
                }
                double *dqi = dq + ((b0 + i) * hq + a) * d;
                for (int e = 0; e < d; ++e) dqi[e] = 0.0;
                for (int64_t j = 0; j <= i; ++j) {
                    double ds = pr[j] * (dp[j] - rowsum);
                    const double *kj = k + ((b0 + j) * hkv + c) * d;
                    double *dkj = dk + ((b0 + j) * hkv + c) * d, *dvj = dv + ((b0 + j) * hkv + c) * d;
                    for (int e = 0; e < d; ++e) {
                        dqi[e] += scale * ds * kj[e];
                        dkj[e] += scale * ds * qi[e];
                        dvj[e] += pr[j] * gi[e];
                    }
                }
            }
        }
        free(sc);
    }
    return ORC_OK;
}
