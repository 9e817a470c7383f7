/*
 * HIPPO hot path -- CPU oracle.  TEST INFRASTRUCTURE, NOT THE PRODUCT.
 *
 * A plain, slow, float64 implementation of what the HIP library computes, written from the
 * paper's equations (Method, "Semantic-aware Token Preservation": Eq. 2-7; Preliminaries,
 * "Speculative Decoding": the draft / verification forward passes whose attention this is).
 * Only tests, the smoke check and the bench's cpu_baseline leg may use it.  It shares no code,
 * header, table or helper with the HIP path.
 *
 * Inputs are float32 arrays whose values are exactly the numbers the GPU sees (bf16 inputs are
 * bf16-representable float32); every value is widened to double on read and all arithmetic,
 * exp, log and sqrt are double.  No tiling, no online softmax, no reordering beyond what the
 * equations state.  `#pragma omp parallel for` over independent (batch, head / frame) items is
 * the only concession to run time; each item is computed serially.
 *
 * Pins (tests/test_oracle_pins.py): closed forms and invariants of Eq. 2-7, brute-force top-k,
 * textbook softmax(QK^T)V through a library routine, truncation / gamma = 0 identities.
 * Pins of the speculative-sampling verification, Eq. 1 (tests/test_oracle_sd_pins.py): the emitted
 * token follows the target distribution for any draft distribution, acceptance rate
 * sum min(p, q), a hand-worked example, inverse-CDF boundaries, greedy limit by brute force.
 * Agreement with the authors' own code is UNPINNED: the paper prints no code and no worked
 * numbers, so the readings listed next to each function are this build's.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int hippo_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------------------------------
 * Eq. 2 -- global semantic relevance.
 *   S^(h) = softmax_j( Q_txt^(h) K_vid^(h)T / sqrt(d_k) )   (softmax over the N_v visual keys)
 *   s_attn[j] = 1/(H L_txt) sum_h sum_i S^(h)[i,j]           (one layer; N_L = 1 per call)
 * Readings: softmax runs over the visual keys only (the matrix is L_txt x N_v as written);
 * H counts query heads, head h reads KV head h / (H / H_kv).
 *
 * q_txt [B, L, H, d]; k_vis points at visual token 0 of KV head 0 of batch 0, element
 * (b, hk, j, c) at k_vis[b*ksb + hk*ksh + j*d + c].  out [B, N_v].
 * ------------------------------------------------------------------------------------------ */
void hippo_oracle_s_attn(const float *q_txt, int B, int L, int H, int Hkv, int d,
                         const float *k_vis, int64_t ksb, int64_t ksh, int Nv, double *out)
{
    const int G = H / Hkv;
    const double inv_sqrt_d = 1.0 / sqrt((double)d);
    for (int b = 0; b < B; ++b) {
        double *acc_h = (double *)calloc((size_t)H * Nv, sizeof(double));
#pragma omp parallel for schedule(dynamic, 1)
        for (int h = 0; h < H; ++h) {
            const float *K = k_vis + b * ksb + (h / G) * ksh;
            double *z = (double *)malloc((size_t)Nv * sizeof(double));
            double *acc = acc_h + (size_t)h * Nv;
            for (int i = 0; i < L; ++i) {
                const float *q = q_txt + (((int64_t)b * L + i) * H + h) * d;
                double zmax = -INFINITY;
                for (int j = 0; j < Nv; ++j) {
                    double dot = 0.0;
                    for (int c = 0; c < d; ++c) dot += (double)q[c] * (double)K[(int64_t)j * d + c];
                    z[j] = dot * inv_sqrt_d;
                    if (z[j] > zmax) zmax = z[j];
                }
                double denom = 0.0;
                for (int j = 0; j < Nv; ++j) { z[j] = exp(z[j] - zmax); denom += z[j]; }
                for (int j = 0; j < Nv; ++j) acc[j] += z[j] / denom;
            }
            free(z);
        }
        for (int j = 0; j < Nv; ++j) {
            double s = 0.0;
            for (int h = 0; h < H; ++h) s += acc_h[(size_t)h * Nv + j];
            out[(int64_t)b * Nv + j] = s / ((double)H * (double)L);
        }
        free(acc_h);
    }
}

/* cosine of two vectors; 0 when either has zero norm (the paper is silent on that case) */
static double cosine(const float *a, const float *b, int n)
{
    double ab = 0.0, aa = 0.0, bb = 0.0;
    for (int c = 0; c < n; ++c) {
        ab += (double)a[c] * (double)b[c];
        aa += (double)a[c] * (double)a[c];
        bb += (double)b[c] * (double)b[c];
    }
    if (aa == 0.0 || bb == 0.0) return 0.0;
    return ab / (sqrt(aa) * sqrt(bb));
}

/* ------------------------------------------------------------------------------------------
 * Eq. 3-4 -- inter-frame temporal redundancy.
 *   s'_temp(v_p^f) = mean over f' in {f-1, f+1} within [0, F) of cos(v_p^f, v_p^f')
 *   s_temp = 1 - s'_temp
 * Reading: a single frame has no neighbour; then s'_temp = 0 and s_temp = 1.
 * emb [B, F*P, de] with row stride `stride_tok` (elements); P = tokens per frame.  out [B, F*P].
 * ------------------------------------------------------------------------------------------ */
void hippo_oracle_s_temp(const float *emb, int B, int F, int P, int de, int64_t stride_b,
                         int64_t stride_tok, double *out)
{
    for (int b = 0; b < B; ++b) {
#pragma omp parallel for schedule(static)
        for (int f = 0; f < F; ++f) {
            for (int p = 0; p < P; ++p) {
                const float *v = emb + b * stride_b + ((int64_t)f * P + p) * stride_tok;
                double sum = 0.0;
                int cnt = 0;
                if (f - 1 >= 0) { sum += cosine(v, v - (int64_t)P * stride_tok, de); ++cnt; }
                if (f + 1 < F)  { sum += cosine(v, v + (int64_t)P * stride_tok, de); ++cnt; }
                double sprime = cnt ? sum / cnt : 0.0;
                out[(int64_t)b * F * P + (int64_t)f * P + p] = 1.0 - sprime;
            }
        }
    }
}

/* ------------------------------------------------------------------------------------------
 * Eq. 5-6 -- intra-frame spatial redundancy.
 *   per crop c with token set C (M_c = |C|):  E = L2-normalised embeddings, S = E E^T,
 *   mu_j = 1/M_c sum_{k in C} S_jk,  s_spa[j] = 1/M_c sum_{k in C} (S_jk - mu_j)^2
 * Readings: crops are non-overlapping crop_h x crop_w tiles of each frame's grid anchored at
 * (0,0); tiles at the right / bottom edge are truncated and use their actual count M_c; the
 * sum runs over all k in the crop including k = j, as the equation is written.
 * ------------------------------------------------------------------------------------------ */
void hippo_oracle_s_spa(const float *emb, int B, int F, int gh, int gw, int ch, int cw, int de,
                        int64_t stride_b, int64_t stride_tok, double *out)
{
    const int P = gh * gw;
    const int ncy = (gh + ch - 1) / ch, ncx = (gw + cw - 1) / cw;
    for (int b = 0; b < B; ++b) {
#pragma omp parallel for schedule(static)
        for (int f = 0; f < F; ++f) {
            int *tok = (int *)malloc((size_t)ch * cw * sizeof(int));
            double *S = (double *)malloc((size_t)ch * cw * ch * cw * sizeof(double));
            for (int cy = 0; cy < ncy; ++cy)
                for (int cx = 0; cx < ncx; ++cx) {
                    int M = 0;
                    for (int y = cy * ch; y < (cy + 1) * ch && y < gh; ++y)
                        for (int x = cx * cw; x < (cx + 1) * cw && x < gw; ++x)
                            tok[M++] = f * P + y * gw + x;
                    for (int j = 0; j < M; ++j)
                        for (int k = 0; k < M; ++k)
                            S[j * M + k] = cosine(emb + b * stride_b + (int64_t)tok[j] * stride_tok,
                                                  emb + b * stride_b + (int64_t)tok[k] * stride_tok, de);
                    for (int j = 0; j < M; ++j) {
                        double mu = 0.0, var = 0.0;
                        for (int k = 0; k < M; ++k) mu += S[j * M + k];
                        mu /= M;
                        for (int k = 0; k < M; ++k) var += (S[j * M + k] - mu) * (S[j * M + k] - mu);
                        out[(int64_t)b * F * P + tok[j]] = var / M;
                    }
                }
            free(tok);
            free(S);
        }
    }
}

/* ------------------------------------------------------------------------------------------
 * Eq. 7 -- holistic fusion.  For each frame and each enabled term: mu_f = mean, sigma_f =
 * population standard deviation over the frame's P tokens, s^ = (s - mu_f) / sigma_f; the
 * score is the sum of the enabled s^.  Reading: sigma_f = 0 gives s^ = 0 for that term/frame.
 * flags: bit0 attn, bit1 temp, bit2 spa.  All arrays [B, F*P].
 * ------------------------------------------------------------------------------------------ */
void hippo_oracle_fuse(const double *s_attn, const double *s_temp, const double *s_spa,
                       unsigned flags, int B, int F, int P, double *score)
{
    const double *terms[3] = { s_attn, s_temp, s_spa };
    for (int64_t i = 0; i < (int64_t)B * F * P; ++i) score[i] = 0.0;
    for (int t = 0; t < 3; ++t) {
        if (!(flags & (1u << t))) continue;
        for (int b = 0; b < B; ++b)
            for (int f = 0; f < F; ++f) {
                const double *s = terms[t] + ((int64_t)b * F + f) * P;
                double *o = score + ((int64_t)b * F + f) * P;
                double mu = 0.0, var = 0.0;
                for (int p = 0; p < P; ++p) mu += s[p];
                mu /= P;
                for (int p = 0; p < P; ++p) var += (s[p] - mu) * (s[p] - mu);
                double sigma = sqrt(var / P);
                if (sigma == 0.0) continue;
                for (int p = 0; p < P; ++p) o[p] += (s[p] - mu) / sigma;
            }
    }
}

/* ------------------------------------------------------------------------------------------
 * Top-k retention ("retain the top-k visual tokens via s(v_j)").  Works on the fp32 scores as
 * given.  Ranking: larger score first; equal scores (-0 == +0) -> lower index first; NaN ranks
 * below every number (ties among NaN by index).  Output: the k winners in ascending index
 * order.  Done by literally ranking every token against every other (O(N^2)): token j is kept
 * iff fewer than k tokens beat it.
 * ------------------------------------------------------------------------------------------ */
static int beats(float a, int ia, float b, int ib) /* does (a, ia) rank before (b, ib)? */
{
    int an = isnan(a), bn = isnan(b);
    if (an != bn) return bn;            /* a number beats a NaN */
    if (!an && a != b) return a > b;
    return ia < ib;
}

void hippo_oracle_topk(const float *scores, int B, int N, int k, int32_t *idx_out)
{
#pragma omp parallel for schedule(static)
    for (int b = 0; b < B; ++b) {
        const float *s = scores + (int64_t)b * N;
        int w = 0;
        for (int j = 0; j < N; ++j) {
            int better = 0;
            for (int i = 0; i < N && better < k; ++i)
                if (i != j && beats(s[i], i, s[j], j)) ++better;
            if (better < k) idx_out[(int64_t)b * k + w++] = j;
        }
    }
}

/* ------------------------------------------------------------------------------------------
 * Draft-cache construction: dst = [src rows before the video | src[vis_off + idx[.]] | src rows
 * after the video], per batch element and KV head, bit copy.  Non-visual tokens are kept whole
 * (App. "Details of Experimental Setups": only the visual part is pruned).
 * src [B, Hkv, src_len, d], dst [B, Hkv, src_len - Nv + k, d], both contiguous.
 * ------------------------------------------------------------------------------------------ */
void hippo_oracle_gather(const float *src, int B, int Hkv, int src_len, int d, int vis_off, int Nv,
                         const int32_t *idx, int k, float *dst)
{
    const int dst_len = src_len - Nv + k;
    for (int b = 0; b < B; ++b)
        for (int h = 0; h < Hkv; ++h) {
            const float *s = src + ((int64_t)b * Hkv + h) * (int64_t)src_len * d;
            float *o = dst + ((int64_t)b * Hkv + h) * (int64_t)dst_len * d;
            for (int n = 0; n < dst_len; ++n) {
                int from;
                if (n < vis_off) from = n;
                else if (n < vis_off + k) from = vis_off + idx[(int64_t)b * k + (n - vis_off)];
                else from = n - k + Nv;
                memcpy(o + (int64_t)n * d, s + (int64_t)from * d, (size_t)d * sizeof(float));
            }
        }
}

/* ------------------------------------------------------------------------------------------
 * Attention of q_len new rows over a cache (Preliminaries, "Speculative Decoding": the target
 * consumes prefix + gamma draft tokens and emits gamma + 1 distributions; the draft consumes
 * one new token per forward).  The cache already holds the new rows' own K/V: it has
 * ctx_len + q_len rows and row i attends to entries [0, ctx_len + i].
 *   z_n = scale * q_i . k_n ;  p = softmax(z) ;  out_i = sum_n p_n v_n ;  lse_i = log sum_n e^{z_n}
 * q, out [B, q_len, H, d]; k, v: element (b, hk, n, c) at base[b*sb + hk*sh + n*d + c];
 * lse [B, H, q_len] (may be NULL).
 * ------------------------------------------------------------------------------------------ */
void hippo_oracle_attention(const float *q, int B, int q_len, int H, int Hkv, int d,
                            const float *k, const float *v, int64_t sb, int64_t sh,
                            int ctx_len, double scale, double *out, double *lse)
{
    const int G = H / Hkv;
#pragma omp parallel for schedule(dynamic, 1) collapse(2)
    for (int b = 0; b < B; ++b)
        for (int h = 0; h < H; ++h) {
            const float *K = k + b * sb + (h / G) * sh;
            const float *V = v + b * sb + (h / G) * sh;
            double *p = (double *)malloc((size_t)(ctx_len + q_len) * sizeof(double));
            for (int i = 0; i < q_len; ++i) {
                const int n_vis = ctx_len + i + 1;
                const float *qi = q + (((int64_t)b * q_len + i) * H + h) * d;
                double *o = out + (((int64_t)b * q_len + i) * H + h) * d;
                double zmax = -INFINITY;
                for (int n = 0; n < n_vis; ++n) {
                    double dot = 0.0;
                    for (int c = 0; c < d; ++c) dot += (double)qi[c] * (double)K[(int64_t)n * d + c];
                    p[n] = dot * scale;
                    if (p[n] > zmax) zmax = p[n];
                }
                double denom = 0.0;
                for (int n = 0; n < n_vis; ++n) { p[n] = exp(p[n] - zmax); denom += p[n]; }
                for (int c = 0; c < d; ++c) o[c] = 0.0;
                for (int n = 0; n < n_vis; ++n) {
                    const double w = p[n] / denom;
                    for (int c = 0; c < d; ++c) o[c] += w * (double)V[(int64_t)n * d + c];
                }
                if (lse) lse[((int64_t)b * H + h) * q_len + i] = zmax + log(denom);
            }
            free(p);
        }
}

/* ------------------------------------------------------------------------------------------
 * Eq. 1 and the resampling rule below it -- speculative-sampling verification of one chain of
 * gamma draft tokens (Preliminaries, "Speculative Decoding").
 *
 *   p_i = softmax(p_logits[i] / T), i = 0..gamma   (target: row i is the distribution of the token
 *                                                   that follows prefix + x_1..x_i)
 *   q_i = softmax(q_logits[i] / T), i = 0..gamma-1 (draft: row i is what x_{i+1} was sampled from)
 * Reading of the paper's indices (it numbers gamma+1 target rows 0..gamma but verifies x_i with
 * "p_i", and conditions q_i on x_i itself): draft token number i (0-based) is verified by row i of
 * both models, and the extra token after a full acceptance comes from the last target row,
 * which is the one the paper names p_gamma.
 *   alpha_i = 1 if p_i[x_i] >= q_i[x_i], else p_i[x_i] / q_i[x_i]               (Eq. 1)
 *   token i is accepted iff u_accept[i] < alpha_i, u in [0, 1); verification stops at the first
 *   rejection j, and the replacement is drawn from r = max(0, p_j - q_j) / sum(max(0, p_j - q_j));
 *   with no rejection the extra token is drawn from p_gamma.
 * Drawing from a distribution r with a uniform u: the first index t whose running sum
 * r_0 + .. + r_t exceeds u * sum(r) (inverse CDF in index order); if rounding leaves none, the last
 * index with r_t > 0.  If sum(max(0, p_j - q_j)) is 0 (p_j == q_j, reachable only through rounding)
 * the replacement is drawn from p_j.
 * T == 0 is greedy decoding, the T -> 0 limit: p_i is one-hot at the first maximum of
 * p_logits[i], q_i is one-hot at x_i (a greedy draft emits its own argmax), and the same rules
 * apply: alpha is 1 or 0 and the replacement / extra token is the target's argmax.
 * alpha is reported for every position, also those after the first rejection.
 */
static void softmax_row(const float *logits, int V, double T, int onehot_at, double *out)
{
    if (T == 0.0) {
        int a = onehot_at;
        if (a < 0) {
            a = 0;
            for (int v = 1; v < V; ++v)
                if ((double)logits[v] > (double)logits[a]) a = v;
        }
        for (int v = 0; v < V; ++v) out[v] = (v == a) ? 1.0 : 0.0;
        return;
    }
    double m = -INFINITY, z = 0.0;
    for (int v = 0; v < V; ++v)
        if ((double)logits[v] / T > m) m = (double)logits[v] / T;
    for (int v = 0; v < V; ++v) z += exp((double)logits[v] / T - m);
    for (int v = 0; v < V; ++v) out[v] = exp((double)logits[v] / T - m) / z;
}

static int draw(const double *r, int V, double u)
{
    double total = 0.0, run = 0.0;
    int last = -1;
    for (int v = 0; v < V; ++v) total += r[v];
    for (int v = 0; v < V; ++v) {
        run += r[v];
        if (r[v] > 0.0) last = v;
        if (run > u * total) return v;
    }
    return last;
}

void hippo_oracle_spec_verify(const float *p_logits, const float *q_logits, const int32_t *tokens,
                              const float *u_accept, const float *u_sample, int B, int gamma, int V,
                              double T, int32_t *n_accept, int32_t *next_token, double *alpha)
{
#pragma omp parallel for schedule(dynamic)
    for (int b = 0; b < B; ++b) {
        double *p = (double *)malloc(sizeof(double) * (size_t)V * 3);
        double *q = p + V, *r = q + V;
        int rejected = -1;
        for (int i = 0; i < gamma; ++i) {
            int x = tokens[(size_t)b * gamma + i];
            softmax_row(p_logits + ((size_t)b * (gamma + 1) + i) * V, V, T, -1, p);
            softmax_row(q_logits ? q_logits + ((size_t)b * gamma + i) * V : NULL, V, T, x, q);
            double a = (p[x] >= q[x]) ? 1.0 : p[x] / q[x];
            alpha[(size_t)b * gamma + i] = a;
            if (rejected < 0 && !((double)u_accept[(size_t)b * gamma + i] < a)) {
                rejected = i;
                double total = 0.0;
                for (int v = 0; v < V; ++v) {
                    r[v] = p[v] - q[v] > 0.0 ? p[v] - q[v] : 0.0;
                    total += r[v];
                }
                next_token[b] = draw(total > 0.0 ? r : p, V, (double)u_sample[b]);
            }
        }
        if (rejected < 0) {
            softmax_row(p_logits + ((size_t)b * (gamma + 1) + gamma) * V, V, T, -1, p);
            next_token[b] = draw(p, V, (double)u_sample[b]);
            n_accept[b] = gamma;
        } else {
            n_accept[b] = rejected;
        }
        free(p);
    }
}
