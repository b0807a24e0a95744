/*
 * lcsa_oracle.c -- TEST INFRASTRUCTURE, not product code.
 *
 * A plain, slow, fp64 CPU statement of locality-constrained block-sparse
 * attention (FlashVSR, arXiv 2510.12747): Sec. 3.2 "Stage 2" (block partition,
 * block average pooling, coarse block-to-block map, top-k block pairs, full
 * attention on the kept pairs with the original Q,K,V), Sec. 3.3 and the
 * caption of Fig. 3 (spatial local window; the sparse mask is chosen inside
 * the window), eq. (1) (softmax weights with scale 1/sqrt(d)), and the
 * appendix "Discussion on Stream VSR Pipelines" (keys/values = sliding-window
 * cache of recent latent frames followed by the current chunk).
 *
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may call
 * this file.  It shares no code with the HIP library and never calls it.
 *
 * Conventions
 *   - Tokens are in raster order: token = (frame * H + row) * W + col.
 *   - Inputs are float32 arrays holding the already dtype-rounded values
 *     (a bf16 value widened to float is exact); every sum, product, mean,
 *     exponential and division below is carried out in double.
 *   - x[token][head][c] is addressed as x[token*stride_tok + head*stride_head + c].
 *   - A block is tt consecutive frames x one th x tw spatial tile (Sec. 3.2 uses
 *     (tt,th,tw) = (2,8,8); tt = 1 gives single-frame tiles).  Tiles on the right /
 *     bottom edge of a grid that th / tw do not divide hold fewer tokens.  Frame
 *     counts are multiples of tt.
 *   - Block id = group * nb + by * tx + bx with nb = ty * tx and group = frame / tt,
 *     group 0 = oldest visible frames for keys, first frames of the chunk for queries.
 *
 * Pins (tests/test_oracle_pins.py): brute-force dense softmax attention,
 * windowed dense attention, hand-written window sets, the Q = 0 closed form,
 * constant V, key-shift invariance, duplicated-frame tie-break, convexity.
 * The paper prints no worked numeric example, so agreement with the authors'
 * own implementation is unpinned.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

static int ceil_div(int a, int b) { return (a + b - 1) / b; }

/* ---- Sec. 3.2: block partition -------------------------------------------------- */

/* Rows [r0,r1) and columns [c0,c1) of the grid that tile (by,bx) covers. */
static void tile_extent(int by, int bx, int H, int W, int th, int tw,
                        int *r0, int *r1, int *c0, int *c1)
{
    *r0 = by * th;
    *r1 = (by + 1) * th < H ? (by + 1) * th : H;
    *c0 = bx * tw;
    *c1 = (bx + 1) * tw < W ? (bx + 1) * tw : W;
}

int lcsa_oracle_blocks_per_frame(int H, int W, int th, int tw)
{
    return ceil_div(H, th) * ceil_div(W, tw);
}

/* ---- Sec. 3.2: average pooling inside each block --------------------------------- */

/* pooled[head][group*nb + tile][c] = mean over the block's tokens of x (n_frames = multiple of tt). */
void lcsa_oracle_pool(const float *x, int64_t stride_tok, int64_t stride_head,
                      int heads, int d, int n_frames, int H, int W, int tt, int th, int tw,
                      double *pooled)
{
    const int ty = ceil_div(H, th), tx = ceil_div(W, tw), nb = ty * tx, n_groups = n_frames / tt;
    for (int h = 0; h < heads; ++h)
        for (int g = 0; g < n_groups; ++g)
            for (int by = 0; by < ty; ++by)
                for (int bx = 0; bx < tx; ++bx) {
                    int r0, r1, c0, c1;
                    tile_extent(by, bx, H, W, th, tw, &r0, &r1, &c0, &c1);
                    double *out = pooled + ((int64_t)h * n_groups * nb + (int64_t)g * nb + by * tx + bx) * d;
                    for (int c = 0; c < d; ++c) {
                        double sum = 0.0;
                        for (int f = g * tt; f < (g + 1) * tt; ++f)
                            for (int r = r0; r < r1; ++r)
                                for (int col = c0; col < c1; ++col) {
                                    int64_t tok = ((int64_t)f * H + r) * W + col;
                                    sum += (double)x[tok * stride_tok + h * stride_head + c];
                                }
                        out[c] = sum / (double)(tt * (r1 - r0) * (c1 - c0));
                    }
                }
}

/* ---- Sec. 3.2: coarse block-to-block map ------------------------------------------ */

/* S[head][qb][kb] = <pooled_q[head][qb], pooled_k[head][kb]>, no scale, no softmax. */
void lcsa_oracle_scores(const double *pooled_q, const double *pooled_k,
                        int heads, int n_qb, int n_kb, int d, double *S)
{
    for (int h = 0; h < heads; ++h)
        for (int qb = 0; qb < n_qb; ++qb)
            for (int kb = 0; kb < n_kb; ++kb) {
                const double *a = pooled_q + ((int64_t)h * n_qb + qb) * d;
                const double *b = pooled_k + ((int64_t)h * n_kb + kb) * d;
                double s = 0.0;
                for (int c = 0; c < d; ++c) s += a[c] * b[c];
                S[((int64_t)h * n_qb + qb) * n_kb + kb] = s;
            }
}

/* ---- Sec. 3.3 / Fig. 3: spatial local window -------------------------------------- */

/*
 * Is key tile index b_k admissible for query tile index b_q along one axis?
 * tile = tile extent along the axis, n = number of tiles along it, radius in
 * tokens (< 0: unbounded).
 * mode 0 (boundary-truncated): nominal tile centres (b*tile + tile/2) at most
 *   `radius` apart; the window is simply cut off at the frame border.
 * mode 1 (boundary-preserved): the truncated window of an interior tile spans
 *   2*r+1 tiles with r = floor(radius/tile); near a border the window keeps
 *   that size and slides inward until it fits in the frame.
 */
static int axis_allowed(int b_q, int b_k, int tile, int n, int radius, int mode)
{
    if (radius < 0) return 1;
    if (mode == 0) {
        /* centres doubled so that odd tile sizes stay integral */
        int cq2 = 2 * b_q * tile + tile, ck2 = 2 * b_k * tile + tile;
        int diff = cq2 > ck2 ? cq2 - ck2 : ck2 - cq2;
        return diff <= 2 * radius;
    } else {
        int r = radius / tile, size = 2 * r + 1;
        if (size >= n) return 1;
        int start = b_q - r;
        if (start < 0) start = 0;
        if (start > n - size) start = n - size;
        return b_k >= start && b_k < start + size;
    }
}

/* allowed(qb, kb): spatial only -- the frames of qb and kb play no role. */
int lcsa_oracle_allowed(int qb, int kb, int H, int W, int th, int tw,
                        int radius_h, int radius_w, int window_mode)
{
    const int ty = ceil_div(H, th), tx = ceil_div(W, tw), nb = ty * tx;
    int qt = qb % nb, kt = kb % nb;
    return axis_allowed(qt / tx, kt / tx, th, ty, radius_h, window_mode) &&
           axis_allowed(qt % tx, kt % tx, tw, tx, radius_w, window_mode);
}

/* ---- Sec. 3.2 + Fig. 3: top-k inside the window ------------------------------------ */

typedef struct { double s; int kb; } cand_t;

/* larger score first; equal scores: lower key-block id first */
static int cand_before(const void *pa, const void *pb)
{
    const cand_t *a = (const cand_t *)pa, *b = (const cand_t *)pb;
    if (a->s > b->s) return -1;
    if (a->s < b->s) return 1;
    return (a->kb > b->kb) - (a->kb < b->kb);
}

static int int_ascending(const void *pa, const void *pb)
{
    int a = *(const int *)pa, b = *(const int *)pb;
    return (a > b) - (a < b);
}

/*
 * For every (head, qb): keep the m = min(topk, n_allowed) admissible key blocks
 * that come first in the order above.  sel_idx[head][qb][0..m) = kept ids in
 * ascending order, the remaining topk - m entries are -1; sel_cnt = m;
 * gap = score of the last kept block minus the best score left out
 * (+inf when nothing admissible is left out).
 */
void lcsa_oracle_select(const double *S, int heads, int q_groups, int kv_groups,
                        int H, int W, int th, int tw,
                        int radius_h, int radius_w, int window_mode, int topk,
                        int32_t *sel_idx, int32_t *sel_cnt, double *gap)
{
    const int nb = lcsa_oracle_blocks_per_frame(H, W, th, tw);
    const int n_qb = q_groups * nb, n_kb = kv_groups * nb;   /* groups = frames / tt */
    cand_t *cand = (cand_t *)malloc(sizeof(cand_t) * (size_t)n_kb);
    for (int h = 0; h < heads; ++h)
        for (int qb = 0; qb < n_qb; ++qb) {
            const double *row = S + ((int64_t)h * n_qb + qb) * n_kb;
            int n = 0;
            for (int kb = 0; kb < n_kb; ++kb)
                if (lcsa_oracle_allowed(qb, kb, H, W, th, tw, radius_h, radius_w, window_mode)) {
                    cand[n].s = row[kb];
                    cand[n].kb = kb;
                    ++n;
                }
            qsort(cand, (size_t)n, sizeof(cand_t), cand_before);
            int m = n < topk ? n : topk;
            int32_t *out = sel_idx + ((int64_t)h * n_qb + qb) * topk;
            for (int i = 0; i < topk; ++i) out[i] = i < m ? cand[i].kb : -1;
            qsort(out, (size_t)m, sizeof(int32_t), int_ascending);
            sel_cnt[(int64_t)h * n_qb + qb] = m;
            if (gap) gap[(int64_t)h * n_qb + qb] = (n > m && m > 0) ? cand[m - 1].s - cand[m].s : INFINITY;
        }
    free(cand);
}

/* ---- Sec. 3.2 + eq. (1): exact attention on the kept block pairs ------------------- */

/*
 * Attention of one query token over the tokens of the listed key blocks.
 * Writes o[d]; returns log(sum exp(logit)) in *lse if lse != NULL; if
 * weights != NULL it receives the softmax weight of every key token
 * (length kv_frames*H*W, zero for tokens outside the listed blocks).
 */
static void attend_token(const float *q_tok, const float *k, const float *v,
                         int64_t kv_stride_tok, int d, int H, int W, int tt, int th, int tw,
                         const int32_t *blocks, int n_blocks, double scale,
                         double *logit /* scratch, >= n_blocks*tt*th*tw */,
                         int64_t *tok_of /* scratch, same length */,
                         double *o, double *lse, double *weights)
{
    const int ty = ceil_div(H, th), tx = ceil_div(W, tw), nb = ty * tx;
    int n = 0;
    for (int b = 0; b < n_blocks; ++b) {
        int kb = blocks[b], g = kb / nb, t = kb % nb, r0, r1, c0, c1;
        tile_extent(t / tx, t % tx, H, W, th, tw, &r0, &r1, &c0, &c1);
        for (int f = g * tt; f < (g + 1) * tt; ++f)
            for (int r = r0; r < r1; ++r)
                for (int c = c0; c < c1; ++c) {
                    int64_t tok = ((int64_t)f * H + r) * W + c;
                    const float *kj = k + tok * kv_stride_tok;
                    double dot = 0.0;
                    for (int e = 0; e < d; ++e) dot += (double)q_tok[e] * (double)kj[e];
                    logit[n] = dot * scale;
                    tok_of[n] = tok;
                    ++n;
                }
    }
    for (int e = 0; e < d; ++e) o[e] = 0.0;
    if (n == 0) { if (lse) *lse = -INFINITY; return; }
    double mx = logit[0];
    for (int j = 1; j < n; ++j) if (logit[j] > mx) mx = logit[j];
    double denom = 0.0;
    for (int j = 0; j < n; ++j) { logit[j] = exp(logit[j] - mx); denom += logit[j]; }
    for (int j = 0; j < n; ++j) {
        double p = logit[j] / denom;
        const float *vj = v + tok_of[j] * kv_stride_tok;
        for (int e = 0; e < d; ++e) o[e] += p * (double)vj[e];
        if (weights) weights[tok_of[j]] = p;
    }
    if (lse) *lse = mx + log(denom);
}

/*
 * o[token][head][c] (dense, double) for every token of the query blocks named
 * in rows[] = {head0, qb0, head1, qb1, ...}; n_rows < 0 means every (head, qb).
 * Query tokens are the tokens of q (q_frames frames); keys/values are the
 * tokens of k, v (kv_frames frames, oldest first).  The selection is an input.
 * scale <= 0 selects 1/sqrt(d).  lse (may be NULL) is [token][head].
 * Entries of o / lse that belong to rows not named are left untouched.
 */
void lcsa_oracle_attend(const float *q, int64_t q_stride_tok, int64_t q_stride_head,
                        const float *k, const float *v, int64_t kv_stride_tok, int64_t kv_stride_head,
                        int heads, int d, int q_frames, int kv_frames,
                        int H, int W, int tt, int th, int tw,
                        const int32_t *sel_idx, const int32_t *sel_cnt, int topk,
                        double scale, const int32_t *rows, int n_rows,
                        double *o, double *lse)
{
    const int ty = ceil_div(H, th), tx = ceil_div(W, tw), nb = ty * tx;
    const int n_qb = (q_frames / tt) * nb;
    (void)kv_frames;
    const int total = n_rows < 0 ? heads * n_qb : n_rows;
    if (scale <= 0.0) scale = 1.0 / sqrt((double)d);
#pragma omp parallel
    {
        double *logit = (double *)malloc(sizeof(double) * (size_t)topk * tt * th * tw);
        int64_t *tok_of = (int64_t *)malloc(sizeof(int64_t) * (size_t)topk * tt * th * tw);
#pragma omp for schedule(dynamic, 1)
        for (int it = 0; it < total; ++it) {
            int h = n_rows < 0 ? it / n_qb : rows[2 * it];
            int qb = n_rows < 0 ? it % n_qb : rows[2 * it + 1];
            int g = qb / nb, t = qb % nb, r0, r1, c0, c1;
            tile_extent(t / tx, t % tx, H, W, th, tw, &r0, &r1, &c0, &c1);
            const int32_t *blocks = sel_idx + ((int64_t)h * n_qb + qb) * topk;
            int n_blocks = sel_cnt[(int64_t)h * n_qb + qb];
            for (int f = g * tt; f < (g + 1) * tt; ++f)
                for (int r = r0; r < r1; ++r)
                    for (int c = c0; c < c1; ++c) {
                        int64_t tok = ((int64_t)f * H + r) * W + c;
                        attend_token(q + tok * q_stride_tok + h * q_stride_head,
                                     k + h * kv_stride_head, v + h * kv_stride_head,
                                     kv_stride_tok, d, H, W, tt, th, tw, blocks, n_blocks, scale,
                                     logit, tok_of, o + (tok * heads + h) * d,
                                     lse ? lse + tok * heads + h : NULL, NULL);
                    }
        }
        free(logit);
        free(tok_of);
    }
}

/*
 * Softmax weights of ONE query token (head h, raster token index q_tok of the
 * chunk) over all kv_frames*H*W key tokens, given its block's selection.
 * weights must be zero-filled by the caller's allocation; tokens outside the
 * kept blocks stay zero.  Also returns o[d].
 */
void lcsa_oracle_attend_weights(const float *q, int64_t q_stride_tok, int64_t q_stride_head,
                                const float *k, const float *v, int64_t kv_stride_tok, int64_t kv_stride_head,
                                int d, int kv_frames, int H, int W, int tt, int th, int tw,
                                const int32_t *blocks, int n_blocks, double scale,
                                int h, int64_t q_tok, double *o, double *weights)
{
    (void)kv_frames;
    if (scale <= 0.0) scale = 1.0 / sqrt((double)d);
    int cap = (n_blocks > 0 ? n_blocks : 1) * tt * th * tw;
    double *logit = (double *)malloc(sizeof(double) * (size_t)cap);
    int64_t *tok_of = (int64_t *)malloc(sizeof(int64_t) * (size_t)cap);
    attend_token(q + q_tok * q_stride_tok + h * q_stride_head,
                 k + h * kv_stride_head, v + h * kv_stride_head, kv_stride_tok,
                 d, H, W, tt, th, tw, blocks, n_blocks, scale, logit, tok_of, o, NULL, weights);
    free(logit);
    free(tok_of);
}

/* ---- Sec. 3.2 "Stage 2": gradients of the attention on the kept block pairs --------------------------------- */

/*
 * The model is trained with this sparse attention (Sec. 3.2).  The top-k choice is a discrete decision and carries
 * no gradient, so the backward pass is that of eq. (1) restricted to the kept pairs: with
 *   s_ij = scale q_i.k_j,  p_ij = softmax_j(s_ij) over the tokens j of the blocks kept for i's block,  o_i = sum_j p_ij v_j
 * and an upstream gradient g_i = dL/do_i,
 *   dv_j += p_ij g_i,   t_ij = g_i.v_j,   D_i = sum_j p_ij t_ij (= g_i.o_i),   u_ij = p_ij (t_ij - D_i),
 *   dq_i += scale u_ij k_j,   dk_j += scale u_ij q_i.
 * dq [q tokens][heads][d], dk, dv [kv tokens][heads][d]: dense doubles, written in full (zero where no pair is kept).
 * q, g share strides; k, v share strides.
 */
void lcsa_oracle_attend_bwd(const float *q, const float *g, int64_t q_stride_tok, int64_t q_stride_head,
                            const float *k, const float *v, int64_t kv_stride_tok, int64_t kv_stride_head,
                            int heads, int d, int q_frames, int kv_frames,
                            int H, int W, int tt, int th, int tw,
                            const int32_t *sel_idx, const int32_t *sel_cnt, int topk, double scale,
                            double *dq, double *dk, double *dv)
{
    const int ty = ceil_div(H, th), tx = ceil_div(W, tw), nb = ty * tx;
    const int n_qb = (q_frames / tt) * nb;
    const int64_t n_q = (int64_t)q_frames * H * W, n_kv = (int64_t)kv_frames * H * W;
    if (scale <= 0.0) scale = 1.0 / sqrt((double)d);
    memset(dq, 0, sizeof(double) * (size_t)(n_q * heads * d));
    memset(dk, 0, sizeof(double) * (size_t)(n_kv * heads * d));
    memset(dv, 0, sizeof(double) * (size_t)(n_kv * heads * d));
    /* heads are independent (their slices of dk, dv are disjoint); everything inside a head runs in order */
#pragma omp parallel for schedule(dynamic, 1)
    for (int h = 0; h < heads; ++h) {
        const size_t cap = (size_t)topk * tt * th * tw;
        double *p = (double *)malloc(sizeof(double) * cap);
        int64_t *tok_of = (int64_t *)malloc(sizeof(int64_t) * cap);
        for (int qb = 0; qb < n_qb; ++qb) {
            int grp = qb / nb, t = qb % nb, r0, r1, c0, c1;
            tile_extent(t / tx, t % tx, H, W, th, tw, &r0, &r1, &c0, &c1);
            const int32_t *blocks = sel_idx + ((int64_t)h * n_qb + qb) * topk;
            const int n_blocks = sel_cnt[(int64_t)h * n_qb + qb];
            for (int f = grp * tt; f < (grp + 1) * tt; ++f)
                for (int r = r0; r < r1; ++r)
                    for (int c = c0; c < c1; ++c) {
                        const int64_t i = ((int64_t)f * H + r) * W + c;
                        const float *qi = q + i * q_stride_tok + h * q_stride_head;
                        const float *gi = g + i * q_stride_tok + h * q_stride_head;
                        /* tokens of the kept blocks and their softmax weights */
                        int n = 0;
                        for (int b = 0; b < n_blocks; ++b) {
                            int kb = blocks[b], kg = kb / nb, kt = kb % nb, kr0, kr1, kc0, kc1;
                            tile_extent(kt / tx, kt % tx, H, W, th, tw, &kr0, &kr1, &kc0, &kc1);
                            for (int kf = kg * tt; kf < (kg + 1) * tt; ++kf)
                                for (int kr = kr0; kr < kr1; ++kr)
                                    for (int kc = kc0; kc < kc1; ++kc) {
                                        const int64_t j = ((int64_t)kf * H + kr) * W + kc;
                                        const float *kj = k + j * kv_stride_tok + h * kv_stride_head;
                                        double dot = 0.0;
                                        for (int e = 0; e < d; ++e) dot += (double)qi[e] * (double)kj[e];
                                        p[n] = dot * scale;
                                        tok_of[n] = j;
                                        ++n;
                                    }
                        }
                        if (n == 0) continue;
                        double mx = p[0];
                        for (int a = 1; a < n; ++a) if (p[a] > mx) mx = p[a];
                        double denom = 0.0;
                        for (int a = 0; a < n; ++a) { p[a] = exp(p[a] - mx); denom += p[a]; }
                        for (int a = 0; a < n; ++a) p[a] /= denom;
                        /* D_i = sum_j p_ij (g_i . v_j) */
                        double D = 0.0;
                        for (int a = 0; a < n; ++a) {
                            const float *vj = v + tok_of[a] * kv_stride_tok + h * kv_stride_head;
                            double tij = 0.0;
                            for (int e = 0; e < d; ++e) tij += (double)gi[e] * (double)vj[e];
                            D += p[a] * tij;
                        }
                        double *dqi = dq + (i * heads + h) * d;
                        for (int a = 0; a < n; ++a) {
                            const int64_t j = tok_of[a];
                            const float *kj = k + j * kv_stride_tok + h * kv_stride_head;
                            const float *vj = v + j * kv_stride_tok + h * kv_stride_head;
                            double tij = 0.0;
                            for (int e = 0; e < d; ++e) tij += (double)gi[e] * (double)vj[e];
                            const double u = p[a] * (tij - D);
                            double *dkj = dk + (j * heads + h) * d, *dvj = dv + (j * heads + h) * d;
                            for (int e = 0; e < d; ++e) {
                                dvj[e] += p[a] * (double)gi[e];
                                dqi[e] += scale * u * (double)kj[e];
                                dkj[e] += scale * u * (double)qi[e];
                            }
                        }
                    }
        }
        free(p);
        free(tok_of);
    }
}

/* Number of OpenMP threads lcsa_oracle_attend will use. */
#ifdef _OPENMP
#include <omp.h>
int lcsa_oracle_threads(void) { return omp_get_max_threads(); }
#else
int lcsa_oracle_threads(void) { return 1; }
#endif
