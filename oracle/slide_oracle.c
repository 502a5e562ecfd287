/*
 * CPU oracle for the Slide Attention operator -- TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, plain, double-precision statement of what the
 * operator computes.  It exists so that the GPU library can be checked
 * against something that can be compared with the paper by eye.  Only the
 * tests, the smoke check and the benchmark's cpu_baseline leg may call it;
 * the product library never links or loads it, and the two share no code.
 *
 * What it follows (paper sections / equations):
 *   - local attention with softmax over the k*k neighbourhood of each
 *     query, per head, scaled by 1/sqrt(d)            (Sec. 3.1, Eq. 2)
 *   - the key/value matrix seen row by row: row (u,v) is the feature map
 *     shifted by (u,v), u,v in [-r, r], r = k/2       (Sec. 4.1, Eq. 8-9)
 *   - a shift is a depthwise convolution with a one-hot k*k kernel, applied
 *     as a cross-correlation with zero padding         (Sec. 4.2, Eq. 10-13,
 *                                                       Fig. 2 caption)
 *   - the deformed shifting module: a second, learned depthwise path in
 *     parallel, summed with the shift path, and the two paths merged into
 *     one kernel for inference                         (Sec. 4.3, Fig. 4)
 *
 * Readings taken where the paper is silent or garbled (all listed in the
 * design notes of the repository):
 *   - i is the row (0..H-1), j the column (0..W-1), flat pixel i*W+j;
 *   - shift index s = (u+r)*k + (v+r); tap index t = p*k+q reads offset
 *     (p-r, q-r); the one-hot kernel of shift s has its 1 at tap t = s;
 *   - padded positions are NOT masked: they stay in the softmax;
 *   - learned kernels have shape [C, k*k, k, k], separate for K and V;
 *   - a per-head bias [heads, k*k] is added to the scaled logit (this
 *     comes from the build's problem statement, not from the paper);
 *   - head m owns channels [m*d, (m+1)*d).
 *
 * Layouts: activations [B, C, H, W] (NCHW), kernels [C, S, k, k] with
 * S = k*k, bias [heads, S], attention [B, heads, S, H, W].  Everything is
 * double.  The backward pass is the chain rule applied to the forward loops
 * (the paper gives none).
 *
 * Parallelism: a plain `omp parallel for` over (batch, head) planes, which
 * are independent.  No blocking, fusion or reordering beyond that.
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define IDX4(b, c, i, j, C, H, W) ((((long)(b) * (C) + (c)) * (H) + (i)) * (W) + (j))

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void oracle_set_num_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* zero-extended read of x[b, c, i, j]  (Fig. 2: zero padding) */
static double padded(const double *x, int b, int c, int i, int j, int C, int H, int W)
{
    if (i < 0 || i >= H || j < 0 || j >= W) return 0.0;
    return x[IDX4(b, c, i, j, C, H, W)];
}

/* Sec. 4.3 / Fig. 4(2): merged kernel = one-hot shift kernel + learned kernel.
 * The one-hot kernel of shift s has a single 1 at tap t = s (Eq. 11 puts the 1
 * of shift (-1,-1) at the top-left tap). */
void oracle_reparam(const double *w_learned, double *w_merged, int C, int ksize)
{
    int S = ksize * ksize;
    for (int c = 0; c < C; ++c)
        for (int s = 0; s < S; ++s)
            for (int t = 0; t < S; ++t) {
                long idx = ((long)c * S + s) * S + t;
                w_merged[idx] = w_learned[idx] + (t == s ? 1.0 : 0.0);
            }
}

/* Eq. 12 generalised: depthwise cross-correlation of channel c with the
 * kernel of shift s, at pixel (i, j).  w is [C, S, k, k]. */
static double dwconv_at(const double *x, const double *w, int b, int c, int s, int i, int j,
                        int C, int H, int W, int ksize)
{
    int r = ksize / 2, S = ksize * ksize;
    double acc = 0.0;
    for (int p = 0; p < ksize; ++p)
        for (int q = 0; q < ksize; ++q)
            acc += w[(((long)c * S + s) * ksize + p) * ksize + q] *
                   padded(x, b, c, i + p - r, j + q - r, C, H, W);
    return acc;
}

/* Eq. 9 / Eq. 10: plain shift by (u, v) of shift index s. */
static double shift_at(const double *x, int b, int c, int s, int i, int j,
                       int C, int H, int W, int ksize)
{
    int r = ksize / 2;
    int u = s / ksize - r, v = s % ksize - r;
    return padded(x, b, c, i + u, j + v, C, H, W);
}

/* The deformed shift of a whole tensor, materialised: out[B, C, S, H, W].
 * two_branch != 0: w is the LEARNED kernel and the shift path is added
 * (training form, Fig. 4(1)); two_branch == 0: w is the MERGED kernel
 * (inference form, Fig. 4(2)). */
void oracle_deformed_shift(const double *x, const double *w, double *out,
                           int B, int H, int W, int C, int ksize, int two_branch)
{
    int S = ksize * ksize;
    for (int b = 0; b < B; ++b)
        for (int c = 0; c < C; ++c)
            for (int s = 0; s < S; ++s)
                for (int i = 0; i < H; ++i)
                    for (int j = 0; j < W; ++j) {
                        double val = dwconv_at(x, w, b, c, s, i, j, C, H, W, ksize);
                        if (two_branch) val += shift_at(x, b, c, s, i, j, C, H, W, ksize);
                        out[((((long)b * C + c) * S + s) * H + i) * W + j] = val;
                    }
}

/* Forward for ONE pixel of ONE head: fills out_px[d] (and attn_px[S], Ks/Vs
 * scratch [d*S]) -- Eq. 2 restricted to the k*k neighbourhood, keys and
 * values taken from the deformed shift.  If lse_px is not NULL it receives the
 * logarithm of the softmax denominator of Eq. 2, log sum_s exp(logit[s]). */
static void forward_pixel(const double *q, const double *k, const double *v,
                          const double *wk, const double *wv, const double *bias,
                          int two_branch, int b, int m, int i, int j,
                          int H, int W, int C, int heads, int ksize,
                          double *Ks, double *Vs, double *attn_px, double *out_px,
                          double *lse_px)
{
    int S = ksize * ksize, d = C / heads;
    double scale = 1.0 / sqrt((double)d);
    for (int cc = 0; cc < d; ++cc) {
        int c = m * d + cc;
        for (int s = 0; s < S; ++s) {
            double ks = dwconv_at(k, wk, b, c, s, i, j, C, H, W, ksize);
            double vs = dwconv_at(v, wv, b, c, s, i, j, C, H, W, ksize);
            if (two_branch) {
                ks += shift_at(k, b, c, s, i, j, C, H, W, ksize);
                vs += shift_at(v, b, c, s, i, j, C, H, W, ksize);
            }
            Ks[cc * S + s] = ks;
            Vs[cc * S + s] = vs;
        }
    }
    /* logits, then softmax over the S shifts */
    double mx = -INFINITY;
    for (int s = 0; s < S; ++s) {
        double dot = 0.0;
        for (int cc = 0; cc < d; ++cc)
            dot += q[IDX4(b, m * d + cc, i, j, C, H, W)] * Ks[cc * S + s];
        attn_px[s] = scale * dot + (bias ? bias[m * S + s] : 0.0);
        if (attn_px[s] > mx) mx = attn_px[s];
    }
    double den = 0.0;
    for (int s = 0; s < S; ++s) { attn_px[s] = exp(attn_px[s] - mx); den += attn_px[s]; }
    for (int s = 0; s < S; ++s) attn_px[s] /= den;
    if (lse_px) *lse_px = mx + log(den);
    for (int cc = 0; cc < d; ++cc) {
        double acc = 0.0;
        for (int s = 0; s < S; ++s) acc += attn_px[s] * Vs[cc * S + s];
        out_px[cc] = acc;
    }
}

/* Whole-tensor forward.  out [B,C,H,W]; attn [B,heads,S,H,W] or NULL; lse
 * [B,heads,H,W] or NULL (log of the softmax denominator per pixel and head).
 * two_branch selects the training form (wk/wv learned) or the merged form. */
void oracle_fwd(const double *q, const double *k, const double *v,
                const double *wk, const double *wv, const double *bias,
                double *out, double *attn, double *lse,
                int B, int H, int W, int C, int heads, int ksize, int two_branch)
{
    int S = ksize * ksize, d = C / heads;
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int b = 0; b < B; ++b)
        for (int m = 0; m < heads; ++m) {
            double *Ks = (double *)malloc(sizeof(double) * d * S);
            double *Vs = (double *)malloc(sizeof(double) * d * S);
            double *a = (double *)malloc(sizeof(double) * S);
            double *o = (double *)malloc(sizeof(double) * d);
            for (int i = 0; i < H; ++i)
                for (int j = 0; j < W; ++j) {
                    forward_pixel(q, k, v, wk, wv, bias, two_branch, b, m, i, j,
                                  H, W, C, heads, ksize, Ks, Vs, a, o,
                                  lse ? lse + (((long)b * heads + m) * H + i) * W + j : NULL);
                    for (int cc = 0; cc < d; ++cc)
                        out[IDX4(b, m * d + cc, i, j, C, H, W)] = o[cc];
                    if (attn)
                        for (int s = 0; s < S; ++s)
                            attn[((((long)b * heads + m) * S + s) * H + i) * W + j] = a[s];
                }
            free(Ks); free(Vs); free(a); free(o);
        }
}

/* Forward at a list of sampled (b, head, i, j) positions (merged or
 * two-branch form): out_samples[n, d].  Lets a test check single outputs of a
 * full-size problem without computing all of it. */
void oracle_fwd_samples(const double *q, const double *k, const double *v,
                        const double *wk, const double *wv, const double *bias,
                        const int *pos, int n_pos, double *out_samples,
                        int B, int H, int W, int C, int heads, int ksize, int two_branch)
{
    (void)B;
    int S = ksize * ksize, d = C / heads;
    double *Ks = (double *)malloc(sizeof(double) * d * S);
    double *Vs = (double *)malloc(sizeof(double) * d * S);
    double *a = (double *)malloc(sizeof(double) * S);
    for (int n = 0; n < n_pos; ++n)
        forward_pixel(q, k, v, wk, wv, bias, two_branch,
                      pos[4 * n], pos[4 * n + 1], pos[4 * n + 2], pos[4 * n + 3],
                      H, W, C, heads, ksize, Ks, Vs, a, out_samples + (long)n * d, NULL);
    free(Ks); free(Vs); free(a);
}

/* Backward of the merged form.  Chain rule through the forward loops:
 *   out[c]  = sum_s a[s] Vs[c,s]            -> da[s] = sum_c dO[c] Vs[c,s],  dVs[c,s] = a[s] dO[c]
 *   a = softmax(l)                          -> dl[s] = a[s] (da[s] - sum_s' a[s'] da[s'])
 *   l[s] = scale sum_c q[c] Ks[c,s] + bias  -> dq[c] = scale sum_s dl[s] Ks[c,s],
 *                                              dKs[c,s] = scale dl[s] q[c],  dbias[s] += dl[s]
 *   Ks[c,s] = sum_t Wk[c,s,t] kpad[c, pix+t] -> dk[c, pix+t] += Wk[c,s,t] dKs[c,s]   (in range only)
 *                                              dWk[c,s,t]   += dKs[c,s] kpad[c, pix+t]
 *   and the same for Vs, Wv, v.
 * The gradient with respect to the learned kernel equals the gradient with
 * respect to the merged kernel (merged = one-hot + learned).
 * dq, dk, dv are [B,C,H,W]; dwk, dwv [C,S,k,k]; dbias [heads,S]; all are
 * overwritten. */
void oracle_bwd(const double *dout, const double *q, const double *k, const double *v,
                const double *wk, const double *wv, const double *bias,
                double *dq, double *dk, double *dv, double *dwk, double *dwv, double *dbias,
                int B, int H, int W, int C, int heads, int ksize)
{
    int S = ksize * ksize, d = C / heads, r = ksize / 2;
    long n_act = (long)B * C * H * W, n_w = (long)C * S * S, n_b = (long)heads * S;
    double scale = 1.0 / sqrt((double)d);
    memset(dq, 0, sizeof(double) * n_act);
    memset(dk, 0, sizeof(double) * n_act);
    memset(dv, 0, sizeof(double) * n_act);
    memset(dwk, 0, sizeof(double) * n_w);
    memset(dwv, 0, sizeof(double) * n_w);
    memset(dbias, 0, sizeof(double) * n_b);

#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int b = 0; b < B; ++b)
        for (int m = 0; m < heads; ++m) {
            /* per-plane private parameter gradients, added to the totals at the end */
            double *Ks = (double *)malloc(sizeof(double) * d * S);
            double *Vs = (double *)malloc(sizeof(double) * d * S);
            double *a = (double *)malloc(sizeof(double) * S);
            double *o = (double *)malloc(sizeof(double) * d);
            double *da = (double *)malloc(sizeof(double) * S);
            double *dl = (double *)malloc(sizeof(double) * S);
            double *pwk = (double *)calloc((size_t)d * S * S, sizeof(double));
            double *pwv = (double *)calloc((size_t)d * S * S, sizeof(double));
            double *pb = (double *)calloc((size_t)S, sizeof(double));
            for (int i = 0; i < H; ++i)
                for (int j = 0; j < W; ++j) {
                    forward_pixel(q, k, v, wk, wv, bias, 0, b, m, i, j,
                                  H, W, C, heads, ksize, Ks, Vs, a, o, NULL);
                    double dsum = 0.0;
                    for (int s = 0; s < S; ++s) {
                        double acc = 0.0;
                        for (int cc = 0; cc < d; ++cc)
                            acc += dout[IDX4(b, m * d + cc, i, j, C, H, W)] * Vs[cc * S + s];
                        da[s] = acc;
                        dsum += a[s] * acc;
                    }
                    for (int s = 0; s < S; ++s) {
                        dl[s] = a[s] * (da[s] - dsum);
                        pb[s] += dl[s];
                    }
                    for (int cc = 0; cc < d; ++cc) {
                        int c = m * d + cc;
                        double qc = q[IDX4(b, c, i, j, C, H, W)];
                        double doc = dout[IDX4(b, c, i, j, C, H, W)];
                        double acc = 0.0;
                        for (int s = 0; s < S; ++s) acc += dl[s] * Ks[cc * S + s];
                        dq[IDX4(b, c, i, j, C, H, W)] = scale * acc;
                        for (int s = 0; s < S; ++s) {
                            double dKs = scale * dl[s] * qc;
                            double dVs = a[s] * doc;
                            for (int p = 0; p < ksize; ++p)
                                for (int qq = 0; qq < ksize; ++qq) {
                                    int y = i + p - r, x = j + qq - r;
                                    if (y < 0 || y >= H || x < 0 || x >= W) continue;
                                    long wi = (((long)c * S + s) * ksize + p) * ksize + qq;
                                    long li = (((long)cc * S + s) * ksize + p) * ksize + qq;
                                    long xi = IDX4(b, c, y, x, C, H, W);
                                    dk[xi] += wk[wi] * dKs;
                                    dv[xi] += wv[wi] * dVs;
                                    pwk[li] += dKs * k[xi];
                                    pwv[li] += dVs * v[xi];
                                }
                        }
                    }
                }
#pragma omp critical
            {
                for (long e = 0; e < (long)d * S * S; ++e) {
                    dwk[(long)m * d * S * S + e] += pwk[e];
                    dwv[(long)m * d * S * S + e] += pwv[e];
                }
                for (int s = 0; s < S; ++s) dbias[m * S + s] += pb[s];
            }
            free(Ks); free(Vs); free(a); free(o); free(da); free(dl);
            free(pwk); free(pwv); free(pb);
        }
}
