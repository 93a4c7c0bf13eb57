/*
 * ls_oracle.c -- CPU oracle for LoopServe's online-sparsified prefill attention
 * and its decode-time KV retention scorer (arxiv 2507.13681).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the yardstick the HIP path is
 * measured against; nothing in the product path may call, link or import it.
 * It shares no code, header, table or helper with the HIP path.
 *
 * Everything here is deliberately plain: one loop nest per definition, double
 * precision for every sum, exp and dot product, no blocking, no fusion.  The
 * one exception is the greedy walk of Algorithm 2, whose comparisons decide
 * integers (which line is taken next): it is carried out in IEEE binary32,
 * the precision the device kernel uses, so both sides take the same decision
 * when fed the same line weights.  Build with -ffp-contract=off.
 *
 * What each function follows:
 *   lso_score    Alg. 2, steps "compute Q~, K, A = Softmax(Q~ K^T / sqrt(d_k)),
 *                SlashSum, VerticalSum"; line definitions of Sec. 3.1 (Obs. 1):
 *                a vertical line is a key column, a slash line is a diagonal.
 *   lso_walk     Alg. 2, the while-loop (greedy selection with overlap bound).
 *   lso_select   Alg. 2, Desc_Sort of both line lists followed by the walk.
 *   lso_window / lso_select_exact   the window matrix of Alg. 2 itself, and the same loop
 *                with the overlap of a candidate line counted cell by cell.
 *   lso_attend   masked attention Softmax(QK^T/sqrt(d_k) - c(1-M)) V of
 *                Sec. 2.2 with M the union of selected columns and diagonals,
 *                restricted to the rows of the newest turn (Sec. 5, Step 1).
 *   lso_compress Alg. 3, the arg-max-B retention formula of Sec. 5.2.
 *   lso_decode   Alg. 3, the Decoding step: attention of the newest token over the
 *                retained entries plus every token generated since (the two
 *                update lines after the step add each new token to the retained set).
 *
 * Readings of points the paper leaves open (each is restated where used):
 *   - the softmax is causal: window row at absolute position p sees keys <= p;
 *   - slash index o = query position - key position, o = 0 is the main diagonal;
 *   - w^max of a line is its largest single entry among the scored rows;
 *   - the chosen list head is removed; when one list is empty the other is used;
 *   - line lengths are those of the full n_hat x n block, cost clamped to >= 1;
 *   - marginal gains are not clamped at zero (the running sum may decrease);
 *   - the ratio test is evaluated cross-multiplied, ties go to the slash line;
 *   - sort ties: smaller index first;
 *   - masked entries contribute exactly zero (c = +infinity).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------ O1 --- */

/*
 * Window attention and its line sums (Alg. 2, softmax + SlashSum/VerticalSum).
 *
 * q_win [B,Hq,w,d], k [B,Hkv,n,d], row-major floats.  q_pos[w] are the absolute
 * positions of the window rows (NULL: the last w positions n-w..n-1).
 * Outputs, each [B,Hq,n] floats: vert[b] = sum over rows of A[t][b],
 * slash[o] = sum over rows of A[t][p_t - o], vmax / smax the same with max;
 * total [B,Hq] = sum of all entries of A (equals w up to rounding).
 * Query head h reads KV head h / (Hq/Hkv).
 */
int lso_score(int B, int Hq, int Hkv, int d, int64_t n, int w, double scale,
              const float *q_win, const int64_t *q_pos, const float *k,
              float *vert, float *slash, float *vmax, float *smax, float *total)
{
    if (B <= 0 || Hq <= 0 || Hkv <= 0 || Hq % Hkv || d <= 0 || n <= 0 || w <= 0) return -1;
    const int G = Hq / Hkv;
    int rc = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int bh = 0; bh < B * Hq; ++bh) {
        const int b = bh / Hq, h = bh % Hq, kvh = h / G;
        const float *K = k + ((int64_t)b * Hkv + kvh) * n * d;
        const float *Q = q_win + (int64_t)bh * w * d;
        double *cv = calloc(n, sizeof(double)), *cs = calloc(n, sizeof(double));
        double *mv = calloc(n, sizeof(double)), *ms = calloc(n, sizeof(double));
        double *logit = malloc(n * sizeof(double));
        double tot = 0.0;
        if (!cv || !cs || !mv || !ms || !logit) { rc = -2; goto done; }
        for (int t = 0; t < w; ++t) {
            const int64_t p = q_pos ? q_pos[t] : n - w + t;
            if (p < 0 || p >= n) { rc = -3; goto done; }
            double mx = -INFINITY;
            for (int64_t j = 0; j <= p; ++j) {          /* causal: keys 0..p */
                double s = 0.0;
                for (int c = 0; c < d; ++c) s += (double)Q[(int64_t)t * d + c] * (double)K[j * d + c];
                logit[j] = s * scale;
                if (logit[j] > mx) mx = logit[j];
            }
            double den = 0.0;
            for (int64_t j = 0; j <= p; ++j) den += exp(logit[j] - mx);
            for (int64_t j = 0; j <= p; ++j) {
                const double a = exp(logit[j] - mx) / den;   /* A[t][j] */
                const int64_t o = p - j;                     /* its diagonal */
                cv[j] += a; if (a > mv[j]) mv[j] = a;
                cs[o] += a; if (a > ms[o]) ms[o] = a;
                tot += a;
            }
        }
        for (int64_t j = 0; j < n; ++j) {
            vert[(int64_t)bh * n + j] = (float)cv[j];
            slash[(int64_t)bh * n + j] = (float)cs[j];
            vmax[(int64_t)bh * n + j] = (float)mv[j];
            smax[(int64_t)bh * n + j] = (float)ms[j];
        }
        total[bh] = (float)tot;
done:
        free(cv); free(cs); free(mv); free(ms); free(logit);
    }
    return rc;
}

/* ------------------------------------------------------------------ O2 --- */

/*
 * The while-loop of Alg. 2 on two lists that are already in descending order.
 * Entry i of the slash list has weight ws[i], largest entry ms[i], length ls[i];
 * likewise wv, mv, lv for the vertical list.  All arithmetic is binary32.
 *
 *   while sum < alpha * total and a list is non-empty:
 *       ds = w_s - ol_v ;  dv = w_v - ol_s            (marginal-gain bounds)
 *       cost_s = max(1, l_s - |V^|) ; cost_v = max(1, l_v - |S^|)
 *       take the slash iff  ds / cost_s >= dv / cost_v   (cross-multiplied)
 *       slash:    S^ += s ; sum += ds ; ol_s += wmax_s
 *       vertical: V^ += v ; sum += dv ; ol_v += wmax_v
 *
 * Returns the number of list heads taken from each list (the selection is a
 * prefix of each sorted list), the final sum, and the value of the sum before
 * the last pick (for the stop-minimality check).
 */
void lso_walk(int64_t n_s, const float *ws, const float *ms, const float *ls,
              int64_t n_v, const float *wv, const float *mv, const float *lv,
              float alpha, float total,
              int64_t *taken_s, int64_t *taken_v, float *accounted, float *before_last)
{
    volatile float target = alpha * total;
    float ol_s = 0.0f, ol_v = 0.0f, sum = 0.0f, prev = 0.0f;
    int64_t is = 0, iv = 0;
    while (sum < target && (is < n_s || iv < n_v)) {
        int take_s;
        if (iv >= n_v) take_s = 1;
        else if (is >= n_s) take_s = 0;
        else {
            volatile float ds = ws[is] - ol_v;
            volatile float dv = wv[iv] - ol_s;
            float cs = ls[is] - (float)iv; if (cs < 1.0f) cs = 1.0f;
            float cv = lv[iv] - (float)is; if (cv < 1.0f) cv = 1.0f;
            volatile float lhs = ds * cv;
            volatile float rhs = dv * cs;
            take_s = (lhs >= rhs);
        }
        prev = sum;
        if (take_s) {
            volatile float ds = ws[is] - ol_v;
            sum = sum + ds;
            ol_s = ol_s + ms[is];
            ++is;
        } else {
            volatile float dv = wv[iv] - ol_s;
            sum = sum + dv;
            ol_v = ol_v + mv[iv];
            ++iv;
        }
    }
    *taken_s = is; *taken_v = iv; *accounted = sum; *before_last = prev;
}

typedef struct { float w; int32_t idx; } lso_line;

static int lso_cmp_desc(const void *a, const void *b)
{
    const lso_line *x = a, *y = b;
    if (x->w > y->w) return -1;
    if (x->w < y->w) return 1;
    return (x->idx > y->idx) - (x->idx < y->idx);   /* ties: smaller index first */
}

static int lso_cmp_i32(const void *a, const void *b)
{
    const int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

/*
 * Alg. 2 from the Desc_Sort on, for one head.  vert/slash/vmax/smax are that
 * head's n line weights and maxima.  Line lengths are those of the full
 * n_hat x n causal block: column b is crossed by min(n_hat, n-b) of the new
 * rows, diagonal o by min(n_hat, n-o).
 * v_idx / s_idx receive the selected indices in ascending order (at most
 * cap entries are written; *_cnt always holds the full count).
 */
int lso_select(int64_t n, int64_t n_hat, float alpha,
               const float *vert, const float *slash, const float *vmax, const float *smax,
               float total,
               int32_t *v_idx, int32_t *v_cnt, int64_t cap_v,
               int32_t *s_idx, int32_t *s_cnt, int64_t cap_s,
               float *accounted, float *before_last)
{
    if (n <= 0 || n_hat <= 0 || n_hat > n) return -1;
    lso_line *sv = malloc(n * sizeof(lso_line)), *ss = malloc(n * sizeof(lso_line));
    float *buf = malloc(6 * n * sizeof(float));
    if (!sv || !ss || !buf) { free(sv); free(ss); free(buf); return -2; }
    for (int64_t i = 0; i < n; ++i) {
        sv[i].w = vert[i];  sv[i].idx = (int32_t)i;
        ss[i].w = slash[i]; ss[i].idx = (int32_t)i;
    }
    qsort(sv, n, sizeof(lso_line), lso_cmp_desc);
    qsort(ss, n, sizeof(lso_line), lso_cmp_desc);
    float *ws = buf, *ms = buf + n, *ls = buf + 2 * n, *wv = buf + 3 * n, *mv = buf + 4 * n, *lv = buf + 5 * n;
    for (int64_t i = 0; i < n; ++i) {
        const int64_t o = ss[i].idx, b = sv[i].idx;
        ws[i] = ss[i].w; ms[i] = smax[o]; ls[i] = (float)((n - o) < n_hat ? (n - o) : n_hat);
        wv[i] = sv[i].w; mv[i] = vmax[b]; lv[i] = (float)((n - b) < n_hat ? (n - b) : n_hat);
    }
    int64_t ts, tv;
    lso_walk(n, ws, ms, ls, n, wv, mv, lv, alpha, total, &ts, &tv, accounted, before_last);
    int32_t *tmp = malloc((n + 1) * sizeof(int32_t));
    if (!tmp) { free(sv); free(ss); free(buf); return -2; }
    for (int64_t i = 0; i < ts; ++i) tmp[i] = ss[i].idx;
    qsort(tmp, ts, sizeof(int32_t), lso_cmp_i32);
    for (int64_t i = 0; i < ts && i < cap_s; ++i) s_idx[i] = tmp[i];
    for (int64_t i = 0; i < tv; ++i) tmp[i] = sv[i].idx;
    qsort(tmp, tv, sizeof(int32_t), lso_cmp_i32);
    for (int64_t i = 0; i < tv && i < cap_v; ++i) v_idx[i] = tmp[i];
    *s_cnt = (int32_t)ts; *v_cnt = (int32_t)tv;
    free(tmp); free(sv); free(ss); free(buf);
    return 0;
}

/* lso_select over all B*Hq heads; arrays are [B*Hq, n] / [B*Hq, cap] / [B*Hq]. */
int lso_select_all(int64_t heads, int64_t n, int64_t n_hat, float alpha,
                   const float *vert, const float *slash, const float *vmax, const float *smax,
                   const float *total,
                   int32_t *v_idx, int32_t *v_cnt, int64_t cap_v,
                   int32_t *s_idx, int32_t *s_cnt, int64_t cap_s,
                   float *accounted, float *before_last)
{
    int rc = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t h = 0; h < heads; ++h) {
        int r = lso_select(n, n_hat, alpha, vert + h * n, slash + h * n, vmax + h * n, smax + h * n,
                           total[h], v_idx + h * cap_v, v_cnt + h, cap_v,
                           s_idx + h * cap_s, s_cnt + h, cap_s, accounted + h, before_last + h);
        if (r) rc = r;
    }
    return rc;
}

/* ----------------------------------------------------------------- O2x --- */

/*
 * The window attention matrix itself (Alg. 2, the softmax step), kept instead of
 * only its line sums: a_win [B,Hq,w,n] floats, A[t][j] for keys j <= p_t and 0
 * beyond (causal).  Same arguments as lso_score.
 */
int lso_window(int B, int Hq, int Hkv, int d, int64_t n, int w, double scale,
               const float *q_win, const int64_t *q_pos, const float *k, float *a_win)
{
    if (B <= 0 || Hq <= 0 || Hkv <= 0 || Hq % Hkv || d <= 0 || n <= 0 || w <= 0) return -1;
    const int G = Hq / Hkv;
    int rc = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int bh = 0; bh < B * Hq; ++bh) {
        const int b = bh / Hq, h = bh % Hq, kvh = h / G;
        const float *K = k + ((int64_t)b * Hkv + kvh) * n * d;
        const float *Q = q_win + (int64_t)bh * w * d;
        double *logit = malloc(n * sizeof(double));
        if (!logit) { rc = -2; continue; }
        for (int t = 0; t < w; ++t) {
            float *row = a_win + ((int64_t)bh * w + t) * n;
            const int64_t p = q_pos ? q_pos[t] : n - w + t;
            if (p < 0 || p >= n) { rc = -3; break; }
            double mx = -INFINITY, den = 0.0;
            for (int64_t j = 0; j <= p; ++j) {
                double s = 0.0;
                for (int c = 0; c < d; ++c) s += (double)Q[(int64_t)t * d + c] * (double)K[j * d + c];
                logit[j] = s * scale;
                if (logit[j] > mx) mx = logit[j];
            }
            for (int64_t j = 0; j <= p; ++j) den += exp(logit[j] - mx);
            for (int64_t j = 0; j < n; ++j) row[j] = j <= p ? (float)(exp(logit[j] - mx) / den) : 0.0f;
        }
        free(logit);
    }
    return rc;
}

/*
 * Alg. 2 with the marginal contribution of a line taken exactly (Sec. 5.1 describes
 * the quantities compared in the loop as marginal contributions; the listing bounds
 * the part of a line that is already covered by the sum of w^max of the lines taken
 * from the other list).  Here the covered part of a candidate is added up cell by
 * cell: a diagonal o and a column b share the cell of the scored row at position
 * b + o, if there is one, so
 *     overlap(slash o)  = sum over scored rows t with key c = p_t - o >= 0 and c selected     of A[t][c]
 *     overlap(column b) = sum over scored rows t with o = p_t - b >= 0 and o selected         of A[t][b]
 * (added in row order in double precision, rounded once to binary32).  Everything
 * else is the loop of lso_walk: gain = weight - overlap, cost = max(1, length - lines
 * taken from the other list), the slash is taken when gain_s * cost_v >= gain_v * cost_s,
 * the head of the chosen list is removed, the loop ends when the sum reaches
 * alpha * total or both lists are empty.  Gains are never negative here, and the
 * final sum is the weight of the union of the selected lines on the scored rows.
 *
 * a_win [w,n] is the head's window matrix (lso_window), q_pos[w] the rows' positions
 * (NULL: n-w .. n-1), vert / slash [n] the line weights the lists are ordered by.
 */
int lso_select_exact(int64_t n, int64_t n_hat, int w, float alpha,
                     const float *a_win, const int64_t *q_pos,
                     const float *vert, const float *slash, float total,
                     int32_t *v_idx, int32_t *v_cnt, int64_t cap_v,
                     int32_t *s_idx, int32_t *s_cnt, int64_t cap_s,
                     float *accounted, float *before_last)
{
    if (n <= 0 || n_hat <= 0 || n_hat > n || w <= 0) return -1;
    lso_line *sv = malloc(n * sizeof(lso_line)), *ss = malloc(n * sizeof(lso_line));
    char *in_v = calloc(n, 1), *in_s = calloc(n, 1);
    int32_t *tmp = malloc((n + 1) * sizeof(int32_t));
    if (!sv || !ss || !in_v || !in_s || !tmp) { free(sv); free(ss); free(in_v); free(in_s); free(tmp); return -2; }
    for (int64_t i = 0; i < n; ++i) {
        sv[i].w = vert[i];  sv[i].idx = (int32_t)i;
        ss[i].w = slash[i]; ss[i].idx = (int32_t)i;
    }
    qsort(sv, n, sizeof(lso_line), lso_cmp_desc);
    qsort(ss, n, sizeof(lso_line), lso_cmp_desc);
    volatile float target = alpha * total;
    float sum = 0.0f, prev = 0.0f;
    int64_t is = 0, iv = 0;
    while (sum < target && (is < n || iv < n)) {
        volatile float ds = 0.0f, dv = 0.0f;
        if (is < n) {                                   /* the slash at the head of its list */
            const int64_t o = ss[is].idx;
            double ov = 0.0;
            for (int t = 0; t < w; ++t) {
                const int64_t c = (q_pos ? q_pos[t] : n - w + t) - o;
                if (c >= 0 && in_v[c]) ov += (double)a_win[(int64_t)t * n + c];
            }
            ds = ss[is].w - (float)ov;
        }
        if (iv < n) {                                   /* the column at the head of its list */
            const int64_t b = sv[iv].idx;
            double ov = 0.0;
            for (int t = 0; t < w; ++t) {
                const int64_t o = (q_pos ? q_pos[t] : n - w + t) - b;
                if (o >= 0 && in_s[o]) ov += (double)a_win[(int64_t)t * n + b];
            }
            dv = sv[iv].w - (float)ov;
        }
        int take_s;
        if (iv >= n) take_s = 1;
        else if (is >= n) take_s = 0;
        else {
            const int64_t o = ss[is].idx, b = sv[iv].idx;
            float cs = (float)((n - o) < n_hat ? (n - o) : n_hat) - (float)iv; if (cs < 1.0f) cs = 1.0f;
            float cv = (float)((n - b) < n_hat ? (n - b) : n_hat) - (float)is; if (cv < 1.0f) cv = 1.0f;
            volatile float lhs = ds * cv;
            volatile float rhs = dv * cs;
            take_s = (lhs >= rhs);
        }
        prev = sum;
        if (take_s) { sum = sum + ds; in_s[ss[is].idx] = 1; ++is; }
        else        { sum = sum + dv; in_v[sv[iv].idx] = 1; ++iv; }
    }
    for (int64_t i = 0; i < is; ++i) tmp[i] = ss[i].idx;
    qsort(tmp, is, sizeof(int32_t), lso_cmp_i32);
    for (int64_t i = 0; i < is && i < cap_s; ++i) s_idx[i] = tmp[i];
    for (int64_t i = 0; i < iv; ++i) tmp[i] = sv[i].idx;
    qsort(tmp, iv, sizeof(int32_t), lso_cmp_i32);
    for (int64_t i = 0; i < iv && i < cap_v; ++i) v_idx[i] = tmp[i];
    *s_cnt = (int32_t)is; *v_cnt = (int32_t)iv;
    *accounted = sum; *before_last = prev;
    free(sv); free(ss); free(in_v); free(in_s); free(tmp);
    return 0;
}

/* lso_select_exact over all B*Hq heads; a_win is [B*Hq, w, n], the other arrays as in lso_select_all. */
int lso_select_exact_all(int64_t heads, int64_t n, int64_t n_hat, int w, float alpha,
                         const float *a_win, const int64_t *q_pos,
                         const float *vert, const float *slash, const float *total,
                         int32_t *v_idx, int32_t *v_cnt, int64_t cap_v,
                         int32_t *s_idx, int32_t *s_cnt, int64_t cap_s,
                         float *accounted, float *before_last)
{
    int rc = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t h = 0; h < heads; ++h) {
        int r = lso_select_exact(n, n_hat, w, alpha, a_win + h * (int64_t)w * n, q_pos, vert + h * n, slash + h * n,
                                 total[h], v_idx + h * cap_v, v_cnt + h, cap_v,
                                 s_idx + h * cap_s, s_cnt + h, cap_s, accounted + h, before_last + h);
        if (r) rc = r;
    }
    return rc;
}

/* ------------------------------------------------------------------ O3 --- */

/*
 * Masked attention of the newest turn's rows over the selected lines.
 *
 * q [B,Hq,n_hat,d], k, v [B,Hkv,n,d].  Row a of the new turn sits at absolute
 * position p = n - n_hat + a.  Cell (a, b) is allowed iff b <= p and
 * (b is a selected column  or  p - b is a selected diagonal).
 * rows[n_rows] lists flat row ids ((b*Hq + h)*n_hat + a); NULL means every row
 * in order.  out [n_rows, d], lse [n_rows] (log of the softmax denominator,
 * natural log, of the scaled logits; -inf and a zero row when nothing is allowed).
 *
 * mode 0 ("dense-masked"): the literal form -- every causal logit is formed,
 *         disallowed ones are set to -inf, one softmax over the whole row.
 * mode 1 ("row-sparse"):   only allowed cells are visited (a list per row);
 *         used where mode 0 would take hours.  Independent loop structure.
 */
int lso_attend(int B, int Hq, int Hkv, int d, int64_t n, int64_t n_hat, double scale,
               const float *q, const float *k, const float *v,
               const int32_t *v_idx, const int32_t *v_cnt, int64_t cap_v,
               const int32_t *s_idx, const int32_t *s_cnt, int64_t cap_s,
               int64_t n_rows, const int64_t *rows, int mode, float *out, float *lse)
{
    if (Hq % Hkv || n_hat > n || n_hat <= 0) return -1;
    const int G = Hq / Hkv;
    const int64_t all = (int64_t)B * Hq * n_hat;
    if (!rows) n_rows = all;
    int rc = 0;
#pragma omp parallel
    {
        unsigned char *col = malloc(n), *off = malloc(n);
        double *lg = malloc(n * sizeof(double));
        int64_t *lst = malloc(n * sizeof(int64_t));
        double *acc = malloc(d * sizeof(double));
        int64_t cur_head = -1;
#pragma omp for schedule(dynamic, 16)
        for (int64_t r = 0; r < n_rows; ++r) {
            const int64_t id = rows ? rows[r] : r;
            if (id < 0 || id >= all || !col || !off || !lg || !lst || !acc) { rc = -3; continue; }
            const int64_t bh = id / n_hat, a = id % n_hat;
            const int b = (int)(bh / Hq), h = (int)(bh % Hq), kvh = h / G;
            const int64_t p = n - n_hat + a;
            const float *Q = q + id * d;
            const float *K = k + ((int64_t)b * Hkv + kvh) * n * d;
            const float *V = v + ((int64_t)b * Hkv + kvh) * n * d;
            const int32_t *vi = v_idx + bh * cap_v, *si = s_idx + bh * cap_s;
            const int64_t nv = v_cnt[bh], ns = s_cnt[bh];
            if (nv > cap_v || ns > cap_s) { rc = -4; continue; }
            int bad = 0;                                /* every index must name a line of the block */
            for (int64_t i = 0; i < nv; ++i) if (vi[i] < 0 || vi[i] >= n) bad = 1;
            for (int64_t i = 0; i < ns; ++i) if (si[i] < 0 || si[i] >= n) bad = 1;
            if (bad) { rc = -5; continue; }
            if (bh != cur_head) {                       /* membership tables of this head */
                memset(col, 0, n); memset(off, 0, n);
                for (int64_t i = 0; i < nv; ++i) col[vi[i]] = 1;
                for (int64_t i = 0; i < ns; ++i) off[si[i]] = 1;
                cur_head = bh;
            }
            for (int c = 0; c < d; ++c) acc[c] = 0.0;
            double mx = -INFINITY, den = 0.0;
            if (mode == 0) {
                for (int64_t j = 0; j <= p; ++j) {
                    if (col[j] || off[p - j]) {
                        double s = 0.0;
                        for (int c = 0; c < d; ++c) s += (double)Q[c] * (double)K[j * d + c];
                        lg[j] = s * scale;
                    } else lg[j] = -INFINITY;            /* the -c(1-M) term with c = inf */
                    if (lg[j] > mx) mx = lg[j];
                }
                if (mx > -INFINITY) {
                    for (int64_t j = 0; j <= p; ++j) den += exp(lg[j] - mx);
                    for (int64_t j = 0; j <= p; ++j) {
                        const double pr = exp(lg[j] - mx) / den;
                        if (pr != 0.0) for (int c = 0; c < d; ++c) acc[c] += pr * (double)V[j * d + c];
                    }
                }
            } else {
                int64_t m = 0;
                for (int64_t i = 0; i < nv; ++i) if (vi[i] <= p) lst[m++] = vi[i];
                for (int64_t i = 0; i < ns; ++i)
                    if (si[i] <= p && !col[p - si[i]]) lst[m++] = p - si[i];   /* count a crossing once */
                for (int64_t i = 0; i < m; ++i) {
                    double s = 0.0;
                    for (int c = 0; c < d; ++c) s += (double)Q[c] * (double)K[lst[i] * d + c];
                    lg[i] = s * scale;
                    if (lg[i] > mx) mx = lg[i];
                }
                for (int64_t i = 0; i < m; ++i) den += exp(lg[i] - mx);
                for (int64_t i = 0; i < m; ++i) {
                    const double pr = exp(lg[i] - mx) / den;
                    for (int c = 0; c < d; ++c) acc[c] += pr * (double)V[lst[i] * d + c];
                }
            }
            for (int c = 0; c < d; ++c) out[r * d + c] = (float)acc[c];
            if (lse) lse[r] = (mx > -INFINITY) ? (float)(mx + log(den)) : -INFINITY;
        }
        free(col); free(off); free(lg); free(lst); free(acc);
    }
    return rc;
}

/* ------------------------------------------------------------------ O4 --- */

/*
 * Alg. 3 retention step: for each KV head keep the `budget` cache entries with
 * the largest attention received from the last n_obs query rows, summed over
 * the Hq/Hkv query heads that read this KV head.
 *
 * q_obs [B,Hq,n_obs,d] are the queries at positions len-n_obs..len-1;
 * k [B,Hkv,len,d].  score [B,Hkv,len] (optional) receives the summed column
 * weights.  keep_idx [B,Hkv,budget] ascending; keep_cnt = min(budget, len).
 * Ties: smaller index first.
 */
int lso_compress(int B, int Hq, int Hkv, int d, int64_t len, int n_obs, double scale, int64_t budget,
                 const float *q_obs, const float *k,
                 int32_t *keep_idx, int32_t *keep_cnt, float *score)
{
    if (Hq % Hkv || n_obs <= 0 || n_obs > len || budget <= 0) return -1;
    const int G = Hq / Hkv;
    int rc = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int bk = 0; bk < B * Hkv; ++bk) {
        const int b = bk / Hkv, kvh = bk % Hkv;
        const float *K = k + (int64_t)bk * len * d;
        double *sc = calloc(len, sizeof(double)), *lg = malloc(len * sizeof(double));
        lso_line *ln = malloc(len * sizeof(lso_line));
        if (!sc || !lg || !ln) { rc = -2; free(sc); free(lg); free(ln); continue; }
        for (int g = 0; g < G; ++g) {
            const float *Q = q_obs + (((int64_t)b * Hq + kvh * G + g) * n_obs) * d;
            for (int t = 0; t < n_obs; ++t) {
                const int64_t p = len - n_obs + t;
                double mx = -INFINITY, den = 0.0;
                for (int64_t j = 0; j <= p; ++j) {
                    double s = 0.0;
                    for (int c = 0; c < d; ++c) s += (double)Q[(int64_t)t * d + c] * (double)K[j * d + c];
                    lg[j] = s * scale;
                    if (lg[j] > mx) mx = lg[j];
                }
                for (int64_t j = 0; j <= p; ++j) den += exp(lg[j] - mx);
                for (int64_t j = 0; j <= p; ++j) sc[j] += exp(lg[j] - mx) / den;
            }
        }
        for (int64_t j = 0; j < len; ++j) { ln[j].w = (float)sc[j]; ln[j].idx = (int32_t)j; }
        if (score) for (int64_t j = 0; j < len; ++j) score[(int64_t)bk * len + j] = ln[j].w;
        qsort(ln, len, sizeof(lso_line), lso_cmp_desc);
        const int64_t keep = budget < len ? budget : len;
        int32_t *dst = keep_idx + (int64_t)bk * budget;
        for (int64_t i = 0; i < keep; ++i) dst[i] = ln[i].idx;
        qsort(dst, keep, sizeof(int32_t), lso_cmp_i32);
        keep_cnt[bk] = (int32_t)keep;
        free(sc); free(lg); free(ln);
    }
    return rc;
}

/* Top-`budget` of a given score vector (ties: smaller index first), ascending
 * output.  Lets the tests rank a score vector that did not come from lso_compress. */
int lso_topb(int64_t len, int64_t budget, const float *score, int32_t *keep_idx, int32_t *keep_cnt)
{
    lso_line *ln = malloc(len * sizeof(lso_line));
    if (!ln) return -2;
    for (int64_t j = 0; j < len; ++j) { ln[j].w = score[j]; ln[j].idx = (int32_t)j; }
    qsort(ln, len, sizeof(lso_line), lso_cmp_desc);
    const int64_t keep = budget < len ? budget : len;
    for (int64_t i = 0; i < keep; ++i) keep_idx[i] = ln[i].idx;
    qsort(keep_idx, keep, sizeof(int32_t), lso_cmp_i32);
    *keep_cnt = (int32_t)keep;
    free(ln);
    return 0;
}

/* ------------------------------------------------------------------ O5 --- */

/*
 * Alg. 3, the Decoding step seen from one attention layer: the newest token's
 * query attends over the entries its KV head retained at the last retention
 * step, followed by the tokens generated since then (Alg. 3 adds every
 * generated token to the retained set), all of them visible:
 *     out = softmax(scale * q [K_c; K_t]^T) [V_c; V_t].
 *
 * q [B,Hq,d]; kc, vc [B,Hkv,cap,d], of which the first cnt[b][kvh] rows are
 * retained entries (cnt == NULL: all cap rows; rows beyond cnt are never read);
 * kt, vt [B,Hkv,T,d] the tokens since (T may be 0, then kt, vt may be NULL).
 * out [B,Hq,d]; lse [B,Hq] natural-log normaliser (optional).  No key at all:
 * zeros and lse = -inf.
 */
int lso_decode(int B, int Hq, int Hkv, int d, int64_t cap, int64_t T, double scale,
               const float *q, const float *kc, const float *vc, const int32_t *cnt,
               const float *kt, const float *vt, float *out, float *lse)
{
    if (Hq % Hkv || cap < 0 || T < 0) return -1;
    const int G = Hq / Hkv;
    int rc = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int bh = 0; bh < B * Hq; ++bh) {
        const int b = bh / Hq, h = bh % Hq, kvh = h / G;
        const int64_t bk = (int64_t)b * Hkv + kvh;
        const int64_t nc = cnt ? cnt[bk] : cap;
        if (nc < 0 || nc > cap) { rc = -4; continue; }
        const int64_t L = nc + T;
        const float *Q = q + (int64_t)bh * d;
        double *lg = malloc((L > 0 ? L : 1) * sizeof(double)), *acc = malloc(d * sizeof(double));
        if (!lg || !acc) { rc = -2; free(lg); free(acc); continue; }
        double mx = -INFINITY, den = 0.0;
        for (int64_t j = 0; j < L; ++j) {
            const float *K = j < nc ? kc + (bk * cap + j) * d : kt + (bk * T + (j - nc)) * d;
            double s = 0.0;
            for (int c = 0; c < d; ++c) s += (double)Q[c] * (double)K[c];
            lg[j] = s * scale;
            if (lg[j] > mx) mx = lg[j];
        }
        for (int c = 0; c < d; ++c) acc[c] = 0.0;
        for (int64_t j = 0; j < L; ++j) den += exp(lg[j] - mx);
        for (int64_t j = 0; j < L; ++j) {
            const float *V = j < nc ? vc + (bk * cap + j) * d : vt + (bk * T + (j - nc)) * d;
            const double pr = exp(lg[j] - mx) / den;
            for (int c = 0; c < d; ++c) acc[c] += pr * (double)V[c];
        }
        for (int c = 0; c < d; ++c) out[(int64_t)bh * d + c] = (float)acc[c];
        if (lse) lse[bh] = L > 0 ? (float)(mx + log(den)) : -INFINITY;
        free(lg); free(acc);
    }
    return rc;
}
