/*
 * CPU oracle for Temporal Token Fusion (TTF).  TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, double-precision evaluation of what the method defines, written from the
 * paper's equations so that it can be checked against them by eye.  It exists to judge the
 * GPU library: only the test-suite, the smoke check and the benchmark's CPU-baseline leg
 * may build, load or call it.  It shares no code, header, table or helper with the GPU
 * path and must never be used to produce results for a caller.
 *
 * Every clip of the batch is an independent instance of the paper's single-clip problem
 * (own anchor, own matches, own mask, own compressed length); for one clip this is exactly
 * Section 3.  The paper's tied-batch rule (one offset from the batch-mean similarity, keep
 * as a union over the batch) is a different mode: ttf_oracle_compress_tied at the end.
 *
 * Readings taken where the text leaves a choice (all stated with the function they affect):
 *   - search window is (2r+1) x (2r+1)  (Section 3 "Pointwise Matching"; the introduction's
 *     "r x r" is loose wording);
 *   - of several clamped offsets that land on one anchor index, the first in row-major
 *     offset order stays and the others are masked; they have equal similarity and equal
 *     dst, so the choice cannot show in any output;
 *   - arg max ties (anchor frame, or distinct anchor tokens) go to the lowest index;
 *   - cos(u,v) is taken as 0 when either vector has zero norm, and only then: non-finite entries go
 *     through the printed quotient as IEEE arithmetic takes them (a NaN cosine wins no comparison);
 *   - fused means s^ > t strictly (Eq. gating keeps s^ <= t); t is the float32 the caller
 *     passed, widened to double;
 *   - the frame mean in the anchor rule is over raw (un-normalised) tokens, as printed;
 *   - kept source rows follow in ascending flat index k*N+i; position triples are the
 *     original (k, y, x), unshifted.
 *
 * Element types: dtype 0 = bfloat16 bit patterns (uint16), dtype 1 = float32.  Both widen
 * to double exactly.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_BF16 = 0, ORACLE_F32 = 1 };
enum { ORACLE_ANCHOR_AUTO = 0, ORACLE_ANCHOR_FIXED = 1 };

int ttf_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

static inline double elem(const void *x, int dtype, size_t idx)
{
    if (dtype == ORACLE_F32)
        return (double)((const float *)x)[idx];
    uint32_t bits = (uint32_t)((const uint16_t *)x)[idx] << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

/* cos(u, v) = u.v / (|u| |v|)  -- the definition printed under the anchor-selection equation. */
static double cosine_rows(const void *x, int dtype, size_t row_u, size_t row_v, int C)
{
    double uv = 0.0, uu = 0.0, vv = 0.0;
    for (int c = 0; c < C; ++c) {
        double u = elem(x, dtype, row_u * (size_t)C + c);
        double v = elem(x, dtype, row_v * (size_t)C + c);
        uv += u * v;
        uu += u * u;
        vv += v * v;
    }
    double den = sqrt(uu) * sqrt(vv);
    return den == 0.0 ? 0.0 : uv / den;
}

static double cosine_vec(const double *u, const double *v, int C)
{
    double uv = 0.0, uu = 0.0, vv = 0.0;
    for (int c = 0; c < C; ++c) {
        uv += u[c] * v[c];
        uu += u[c] * u[c];
        vv += v[c] * v[c];
    }
    double den = sqrt(uu) * sqrt(vv);
    return den == 0.0 ? 0.0 : uv / den;
}

/* Integer projection onto [lo, hi]  (the clamp defined before the flat-index map). */
static inline int proj(int z, int lo, int hi)
{
    return z < lo ? lo : (z > hi ? hi : z);
}

/*
 * Anchor frame selection, automatic rule:
 *   a* = argmax_k cos( (1/N) sum_i x_{k,i} ,  (1/(F N)) sum_{k'} sum_i x_{k',i} ).
 * x is one clip [F, N, C].  score[k] receives the cosine of every frame.
 */
static int select_anchor(const void *x, int dtype, int F, int N, int C, double *score)
{
    double *mean_k = (double *)calloc((size_t)F * C, sizeof(double));
    double *mean_g = (double *)calloc((size_t)C, sizeof(double));
#pragma omp parallel for schedule(static)
    for (int k = 0; k < F; ++k) {
        double *m = mean_k + (size_t)k * C;
        for (int i = 0; i < N; ++i)
            for (int c = 0; c < C; ++c)
                m[c] += elem(x, dtype, ((size_t)k * N + i) * C + c);
    }
    for (int k = 0; k < F; ++k)
        for (int c = 0; c < C; ++c)
            mean_g[c] += mean_k[(size_t)k * C + c];      /* still plain sums here */
    for (int c = 0; c < C; ++c)
        mean_g[c] /= (double)F * (double)N;
    for (int k = 0; k < F; ++k)
        for (int c = 0; c < C; ++c)
            mean_k[(size_t)k * C + c] /= (double)N;
    int a = 0;
    for (int k = 0; k < F; ++k) {
        score[k] = cosine_vec(mean_k + (size_t)k * C, mean_g, C);
        if (score[k] > score[a])
            a = k;                                        /* strict: lowest k wins a tie */
    }
    free(mean_k);
    free(mean_g);
    return a;
}

/*
 * Local window search for one source token (k, i) of one clip against anchor frame a:
 * offsets Delta_r = {-r..r}^2 in row-major order, clamped flat index pi, duplicates masked,
 * cosine per surviving candidate, arg max (first maximum), s^ and dst.
 * `stamp` is an N-entry scratch array owned by the calling thread; `tag` is unique per call.
 */
static void match_token(const void *x, int dtype, int H, int W, int C, int r,
                        int a, int k, int i, int32_t *stamp, int32_t tag,
                        double *best, double *second, int32_t *dst, int32_t *n_cand)
{
    const int N = H * W;
    const int yi = i / W, xi = i % W;
    double s_hat = -INFINITY, s_2nd = -INFINITY;
    int32_t j_hat = -1, cnt = 0;
    for (int dy = -r; dy <= r; ++dy) {
        for (int dx = -r; dx <= r; ++dx) {
            int j = proj(yi + dy, 0, H - 1) * W + proj(xi + dx, 0, W - 1);
            if (stamp[j] == tag)
                continue;                 /* duplicate of an earlier offset: masked (-inf) */
            stamp[j] = tag;
            ++cnt;
            double s = cosine_rows(x, dtype, (size_t)k * N + i, (size_t)a * N + j, C);
            if (s > s_hat) {
                s_2nd = s_hat;
                s_hat = s;
                j_hat = j;
            } else if (s > s_2nd) {
                s_2nd = s;
            }
        }
    }
    *best = s_hat;
    *second = s_2nd;
    *dst = j_hat;
    *n_cand = cnt;
}

/*
 * Whole pass.  All pointers are host memory owned by the caller.
 *   x             [B,F,H,W,C]  input tokens
 *   anchor_index  [B]          chosen (or given) anchor frame per clip
 *   anchor_score  [B,F]        cosine of every frame mean with the clip mean (0 when FIXED)
 *   best_sim      [B,F,N]      s^ per source token; 1.0 on anchor-frame rows
 *   second_sim    [B,F,N]      runner-up similarity among distinct candidates (-inf if none)
 *   best_idx      [B,F,N]      dst(k,i) for every source token; i on anchor-frame rows
 *   cand_count    [B,F,N]      number of distinct candidates evaluated (0 on anchor rows)
 *   fuse_map      [B,F,N]      dst(k,i) if fused, else -1
 *   kept_count    [B]          L' = N + P
 *   row_offsets   [B+1]        exclusive prefix of kept_count
 *   src_index     [B*F*N]      flat k*N+i of every output row, clip after clip
 *   pos_ids       [3, B*F*N]   planes k, y, x of every output row
 *   tokens_out    [B*F*N, C]   gathered rows in the input element type, or NULL to skip
 * anchor_fixed may be negative (counted from the last frame).  Returns 0, or 1 on bad sizes.
 */
int ttf_oracle_compress(const void *x, int dtype, int B, int F, int H, int W, int C,
                        int r, float t, int anchor_mode, int anchor_fixed,
                        int32_t *anchor_index, double *anchor_score,
                        double *best_sim, double *second_sim, int32_t *best_idx,
                        int32_t *cand_count, int32_t *fuse_map,
                        int32_t *kept_count, int32_t *row_offsets,
                        int32_t *src_index, int32_t *pos_ids, void *tokens_out)
{
    if (B < 1 || F < 1 || H < 1 || W < 1 || C < 1 || r < 0)
        return 1;
    if (dtype != ORACLE_BF16 && dtype != ORACLE_F32)
        return 1;
    if (anchor_mode == ORACLE_ANCHOR_FIXED && (anchor_fixed < -F || anchor_fixed >= F))
        return 1;
    const int N = H * W;
    const size_t esz = dtype == ORACLE_F32 ? 4 : 2;
    const size_t clip_elems = (size_t)F * N * C;
    const size_t cap = (size_t)B * F * N;
    const double thr = (double)t;

    for (int b = 0; b < B; ++b) {
        const void *xb = (const char *)x + (size_t)b * clip_elems * esz;
        double *score = anchor_score + (size_t)b * F;
        int a;
        if (anchor_mode == ORACLE_ANCHOR_FIXED) {
            a = anchor_fixed < 0 ? anchor_fixed + F : anchor_fixed;
            for (int k = 0; k < F; ++k)
                score[k] = 0.0;
        } else {
            a = select_anchor(xb, dtype, F, N, C, score);
        }
        anchor_index[b] = a;

#pragma omp parallel
        {
            int32_t *stamp = (int32_t *)calloc((size_t)N, sizeof(int32_t));
#pragma omp for schedule(dynamic, 16)
            for (int ki = 0; ki < F * N; ++ki) {
                const int k = ki / N, i = ki % N;
                const size_t o = (size_t)b * F * N + ki;
                if (k == a) {                 /* anchor tokens are always retained */
                    best_sim[o] = 1.0;
                    second_sim[o] = -INFINITY;
                    best_idx[o] = i;
                    cand_count[o] = 0;
                    fuse_map[o] = -1;
                    continue;
                }
                match_token(xb, dtype, H, W, C, r, a, k, i, stamp, ki + 1,
                            &best_sim[o], &second_sim[o], &best_idx[o], &cand_count[o]);
                /* gating: keep = 1[s^ <= t]; fused otherwise */
                fuse_map[o] = (best_sim[o] > thr) ? best_idx[o] : -1;
            }
            free(stamp);
        }
    }

    /* Compressed sequence: the N anchor rows, then the preserved source rows in ascending
     * flat order; positions are gathered with the rows. */
    size_t row = 0;
    for (int b = 0; b < B; ++b) {
        const int a = anchor_index[b];
        row_offsets[b] = (int32_t)row;
        for (int pass = 0; pass < 2; ++pass) {
            for (int k = 0; k < F; ++k) {
                if ((pass == 0) != (k == a))
                    continue;
                for (int i = 0; i < N; ++i) {
                    const size_t o = ((size_t)b * F + k) * N + i;
                    if (k != a && fuse_map[o] >= 0)
                        continue;
                    src_index[row] = k * N + i;
                    pos_ids[0 * cap + row] = k;
                    pos_ids[1 * cap + row] = i / W;
                    pos_ids[2 * cap + row] = i % W;
                    if (tokens_out)
                        memcpy((char *)tokens_out + row * (size_t)C * esz,
                               (const char *)x + o * (size_t)C * esz, (size_t)C * esz);
                    ++row;
                }
            }
        }
        kept_count[b] = (int32_t)(row - (size_t)row_offsets[b]);
    }
    row_offsets[B] = (int32_t)row;
    return 0;
}

/*
 * The window search alone, for a list of n tokens given as (b, k, i) triples, with the
 * anchor frame of every clip supplied by the caller.  Used to check samples of a large
 * batch and to re-judge single tokens.  Tokens with k == anchor get the anchor-row values.
 */
int ttf_oracle_match_tokens(const void *x, int dtype, int B, int F, int H, int W, int C, int r,
                            const int32_t *anchor_index, const int32_t *tokens, int n,
                            double *best_sim, double *second_sim, int32_t *best_idx)
{
    if (B < 1 || F < 1 || H < 1 || W < 1 || C < 1 || r < 0 || n < 0)
        return 1;
    const int N = H * W;
    const size_t esz = dtype == ORACLE_F32 ? 4 : 2;
    const size_t clip_elems = (size_t)F * N * C;
#pragma omp parallel
    {
        int32_t *stamp = (int32_t *)calloc((size_t)N, sizeof(int32_t));
#pragma omp for schedule(dynamic, 16)
        for (int q = 0; q < n; ++q) {
            const int b = tokens[3 * q], k = tokens[3 * q + 1], i = tokens[3 * q + 2];
            const void *xb = (const char *)x + (size_t)b * clip_elems * esz;
            if (k == anchor_index[b]) {
                best_sim[q] = 1.0;
                second_sim[q] = -INFINITY;
                best_idx[q] = i;
                continue;
            }
            int32_t cnt;
            memset(stamp, 0, (size_t)N * sizeof(int32_t));
            match_token(xb, dtype, H, W, C, r, anchor_index[b], k, i, stamp, 1,
                        &best_sim[q], &second_sim[q], &best_idx[q], &cnt);
        }
        free(stamp);
    }
    return 0;
}

/*
 * Tied-batch mode (Section 3, the remark after the s^/dst equations and the wording of the
 * gating paragraph): for B > 1 one offset is chosen per source position (k,i) by maximising
 * the MEAN similarity over the batch elements, every element reads its own s^ at that offset,
 * and the position is preserved if ANY element has s^ <= t (the keep masks are united), so all
 * elements keep the same index set and the output is rectangular [B, N+P, C].
 *
 * Readings (the text does not spell these out):
 *   - the anchor frame is shared: with the automatic rule it is the frame whose anchor score,
 *     averaged over the batch elements, is largest (lowest k on ties); a fixed frame otherwise;
 *   - the mean is the plain arithmetic mean of the B cosines of one candidate cell, summed in
 *     ascending b; candidates are the distinct clamped cells in row-major offset order and the
 *     first maximum wins, exactly as in the single-clip search.
 *
 *   anchor_index  [1]         shared anchor frame
 *   anchor_score  [F]         batch-mean anchor score per frame (0 when FIXED)
 *   mean_sim      [F,N]       largest batch-mean similarity; 1.0 on anchor rows
 *   second_mean   [F,N]       runner-up batch-mean similarity (-inf if none)
 *   best_sim      [B,F,N]     s^ of every element at the shared offset; 1.0 on anchor rows
 *   best_idx      [F,N]       shared dst(k,i); i on anchor rows
 *   fuse_map      [F,N]       dst(k,i) if every element has s^ > t, else -1
 *   kept_count    [1]         L' = N + P
 *   src_index     [F*N]       flat k*N+i of every output row
 *   pos_ids       [3, F*N]    planes k, y, x
 *   tokens_out    [B, F*N, C] rows of every element, first L' valid; or NULL
 */
int ttf_oracle_compress_tied(const void *x, int dtype, int B, int F, int H, int W, int C,
                             int r, float t, int anchor_mode, int anchor_fixed,
                             int32_t *anchor_index, double *anchor_score,
                             double *mean_sim, double *second_mean, double *best_sim,
                             int32_t *best_idx, int32_t *fuse_map, int32_t *kept_count,
                             int32_t *src_index, int32_t *pos_ids, void *tokens_out)
{
    if (B < 1 || F < 1 || H < 1 || W < 1 || C < 1 || r < 0)
        return 1;
    if (dtype != ORACLE_BF16 && dtype != ORACLE_F32)
        return 1;
    if (anchor_mode == ORACLE_ANCHOR_FIXED && (anchor_fixed < -F || anchor_fixed >= F))
        return 1;
    const int N = H * W;
    const size_t esz = dtype == ORACLE_F32 ? 4 : 2;
    const size_t clip_elems = (size_t)F * N * C;
    const size_t cap = (size_t)F * N;
    const double thr = (double)t;

    int a;
    for (int k = 0; k < F; ++k)
        anchor_score[k] = 0.0;
    if (anchor_mode == ORACLE_ANCHOR_FIXED) {
        a = anchor_fixed < 0 ? anchor_fixed + F : anchor_fixed;
    } else {
        double *score = (double *)calloc((size_t)F, sizeof(double));
        for (int b = 0; b < B; ++b) {
            select_anchor((const char *)x + (size_t)b * clip_elems * esz, dtype, F, N, C, score);
            for (int k = 0; k < F; ++k)
                anchor_score[k] += score[k];
        }
        free(score);
        a = 0;
        for (int k = 0; k < F; ++k) {
            anchor_score[k] /= (double)B;
            if (anchor_score[k] > anchor_score[a])
                a = k;
        }
    }
    anchor_index[0] = a;

#pragma omp parallel
    {
        int32_t *stamp = (int32_t *)calloc((size_t)N, sizeof(int32_t));
#pragma omp for schedule(dynamic, 16)
        for (int ki = 0; ki < F * N; ++ki) {
            const int k = ki / N, i = ki % N;
            if (k == a) {
                mean_sim[ki] = 1.0;
                second_mean[ki] = -INFINITY;
                best_idx[ki] = i;
                fuse_map[ki] = -1;
                for (int b = 0; b < B; ++b)
                    best_sim[(size_t)b * F * N + ki] = 1.0;
                continue;
            }
            const int yi = i / W, xi = i % W;
            double m_hat = -INFINITY, m_2nd = -INFINITY;
            int32_t j_hat = -1;
            const int32_t tag = ki + 1;
            for (int dy = -r; dy <= r; ++dy) {
                for (int dx = -r; dx <= r; ++dx) {
                    int j = proj(yi + dy, 0, H - 1) * W + proj(xi + dx, 0, W - 1);
                    if (stamp[j] == tag)
                        continue;             /* duplicate of an earlier offset: masked */
                    stamp[j] = tag;
                    double sum = 0.0;
                    for (int b = 0; b < B; ++b)
                        sum += cosine_rows((const char *)x + (size_t)b * clip_elems * esz, dtype,
                                           (size_t)k * N + i, (size_t)a * N + j, C);
                    double m = sum / (double)B;
                    if (m > m_hat) {
                        m_2nd = m_hat;
                        m_hat = m;
                        j_hat = j;
                    } else if (m > m_2nd) {
                        m_2nd = m;
                    }
                }
            }
            mean_sim[ki] = m_hat;
            second_mean[ki] = m_2nd;
            best_idx[ki] = j_hat;
            int all_above = 1;
            for (int b = 0; b < B; ++b) {
                double s = cosine_rows((const char *)x + (size_t)b * clip_elems * esz, dtype,
                                       (size_t)k * N + i, (size_t)a * N + j_hat, C);
                best_sim[(size_t)b * F * N + ki] = s;
                if (!(s > thr))
                    all_above = 0;            /* this element keeps the position: union of keeps */
            }
            fuse_map[ki] = all_above ? j_hat : -1;
        }
        free(stamp);
    }

    size_t row = 0;
    for (int pass = 0; pass < 2; ++pass) {
        for (int k = 0; k < F; ++k) {
            if ((pass == 0) != (k == a))
                continue;
            for (int i = 0; i < N; ++i) {
                const size_t o = (size_t)k * N + i;
                if (k != a && fuse_map[o] >= 0)
                    continue;
                src_index[row] = k * N + i;
                pos_ids[0 * cap + row] = k;
                pos_ids[1 * cap + row] = i / W;
                pos_ids[2 * cap + row] = i % W;
                if (tokens_out)
                    for (int b = 0; b < B; ++b)
                        memcpy((char *)tokens_out + ((size_t)b * cap + row) * (size_t)C * esz,
                               (const char *)x + ((size_t)b * cap + o) * (size_t)C * esz, (size_t)C * esz);
                ++row;
            }
        }
    }
    kept_count[0] = (int32_t)row;
    return 0;
}
