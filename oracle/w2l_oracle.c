/*
 * w2l_oracle.c -- TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, fp64 CPU definitions of every operation on the conv-GLU + CTC
 * training path of the wav2letter++ acoustic model (paper Sec. 2.3: a model is a
 * "network" -- here 1-D temporal convolutions with bias and GLU and a per-frame
 * log-softmax -- plus a "criterion", here CTC; Sec. 4.1 uses the 100M-parameter
 * all-convolutional network with CTC).  The paper names these operations but
 * prints no formula; each function below is the textbook definition written out
 * as loops, with the conventions stated next to it.
 *
 * Nothing here is shared with the HIP library: no header, helper, constant or
 * table.  Only tests, the smoke check and the bench's cpu_baseline leg may load
 * this file's shared object.  All tensors are dense, row-major, channels-last:
 * x[b][t][c].  All arithmetic is double; nothing is rounded to a narrower type.
 *
 * Parity pins (tests/test_oracle_*.py): brute-force alignment enumeration,
 * closed forms, finite differences, adjoint identities, invariants.  orc_asg is
 * "parity unpinned" with respect to the paper (which only cites that criterion's
 * source; its definition here is a stated reading, pinned to itself by brute force);
 * no other function in this file is.
 */
#include <math.h>
#include <stddef.h>
#include <stdlib.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define IDX3(a, b, c, nb, nc) (((size_t)(a) * (size_t)(nb) + (size_t)(b)) * (size_t)(nc) + (size_t)(c))

/* ---------------------------------------------------------------------------
 * Temporal convolution (paper Sec. 2.3 "1D convolutions"; Sec. 4.1 "temporal
 * convolution layers").  Cross-correlation, odd width k, symmetric zero padding
 * p=(k-1)/2, stride s, output length T' = ceil(T/s):
 *   y[b,t',co] = bias[co] + sum_{j<k} sum_{ci} w[co,j,ci] * x[b, s*t'+j-p, ci]
 * with x taken as 0 outside 0 <= t < T.   w is [Cout][k][Cin].
 * ------------------------------------------------------------------------- */
static int out_len(int T, int s) { return (T + s - 1) / s; }

static double conv_fwd_elem(const double *x, const double *w, const double *bias,
                            int T, int Cin, int k, int s, int b, int tp, int co)
{
    const int p = (k - 1) / 2;
    double acc = 0.0;
    for (int j = 0; j < k; ++j) {
        const int t = s * tp + j - p;
        if (t < 0 || t >= T) continue;
        const double *xr = x + IDX3(b, t, 0, T, Cin);
        const double *wr = w + IDX3(co, j, 0, k, Cin);
        double part = 0.0;
#pragma omp simd reduction(+ : part)
        for (int ci = 0; ci < Cin; ++ci) part += wr[ci] * xr[ci];
        acc += part;
    }
    return acc + (bias ? bias[co] : 0.0);
}

void orc_conv1d_fwd(const double *x, const double *w, const double *bias, double *y,
                    int B, int T, int Cin, int Cout, int k, int s)
{
    const int Tp = out_len(T, s);
#pragma omp parallel for collapse(2) schedule(static)
    for (int b = 0; b < B; ++b)
        for (int tp = 0; tp < Tp; ++tp)
            for (int co = 0; co < Cout; ++co)
                y[IDX3(b, tp, co, Tp, Cout)] = conv_fwd_elem(x, w, bias, T, Cin, k, s, b, tp, co);
}

/* the same definition evaluated only at the listed flat output indices */
void orc_conv1d_fwd_at(const double *x, const double *w, const double *bias,
                       const long long *idx, int n, double *out,
                       int B, int T, int Cin, int Cout, int k, int s)
{
    const int Tp = out_len(T, s);
    (void)B;
#pragma omp parallel for schedule(dynamic, 16)
    for (int i = 0; i < n; ++i) {
        long long f = idx[i];
        int co = (int)(f % Cout); f /= Cout;
        int tp = (int)(f % Tp);
        int b = (int)(f / Tp);
        out[i] = conv_fwd_elem(x, w, bias, T, Cin, k, s, b, tp, co);
    }
}

/* Gradient with respect to the input: the transpose of the map x -> y.
 *   dx[b,t,ci] = sum_{j} sum_{co} w[co,j,ci] * dy[b,t',co]
 * over those taps j for which t' = (t + p - j)/s is an integer in [0,T').   */
static double conv_dgrad_elem(const double *dy, const double *w,
                              int T, int Cin, int Cout, int k, int s, int b, int t, int ci)
{
    const int p = (k - 1) / 2, Tp = out_len(T, s);
    double acc = 0.0;
    for (int j = 0; j < k; ++j) {
        const int u = t + p - j;
        if (u < 0 || u % s != 0) continue;
        const int tp = u / s;
        if (tp >= Tp) continue;
        const double *dr = dy + IDX3(b, tp, 0, Tp, Cout);
        for (int co = 0; co < Cout; ++co) acc += w[IDX3(co, j, ci, k, Cin)] * dr[co];
    }
    return acc;
}

void orc_conv1d_bwd_data(const double *dy, const double *w, double *dx,
                         int B, int T, int Cin, int Cout, int k, int s)
{
#pragma omp parallel for collapse(2) schedule(static)
    for (int b = 0; b < B; ++b)
        for (int t = 0; t < T; ++t)
            for (int ci = 0; ci < Cin; ++ci)
                dx[IDX3(b, t, ci, T, Cin)] = conv_dgrad_elem(dy, w, T, Cin, Cout, k, s, b, t, ci);
}

void orc_conv1d_bwd_data_at(const double *dy, const double *w, const long long *idx, int n,
                            double *out, int B, int T, int Cin, int Cout, int k, int s)
{
    (void)B;
#pragma omp parallel for schedule(dynamic, 16)
    for (int i = 0; i < n; ++i) {
        long long f = idx[i];
        int ci = (int)(f % Cin); f /= Cin;
        int t = (int)(f % T);
        int b = (int)(f / T);
        out[i] = conv_dgrad_elem(dy, w, T, Cin, Cout, k, s, b, t, ci);
    }
}

/* Gradient with respect to the weights and the bias: the transpose of w -> y.
 *   dw[co,j,ci] = sum_b sum_{t'} dy[b,t',co] * x[b, s*t'+j-p, ci]
 *   dbias[co]   = sum_b sum_{t'} dy[b,t',co]                                  */
static double conv_wgrad_elem(const double *x, const double *dy,
                              int B, int T, int Cin, int Cout, int k, int s, int co, int j, int ci)
{
    const int p = (k - 1) / 2, Tp = out_len(T, s);
    double acc = 0.0;
    for (int b = 0; b < B; ++b)
        for (int tp = 0; tp < Tp; ++tp) {
            const int t = s * tp + j - p;
            if (t < 0 || t >= T) continue;
            acc += dy[IDX3(b, tp, co, Tp, Cout)] * x[IDX3(b, t, ci, T, Cin)];
        }
    return acc;
}

void orc_conv1d_bwd_weight(const double *x, const double *dy, double *dw, double *dbias,
                           int B, int T, int Cin, int Cout, int k, int s)
{
    const int Tp = out_len(T, s);
#pragma omp parallel for collapse(2) schedule(static)
    for (int co = 0; co < Cout; ++co)
        for (int j = 0; j < k; ++j)
            for (int ci = 0; ci < Cin; ++ci)
                dw[IDX3(co, j, ci, k, Cin)] = conv_wgrad_elem(x, dy, B, T, Cin, Cout, k, s, co, j, ci);
    if (dbias) {
#pragma omp parallel for schedule(static)
        for (int co = 0; co < Cout; ++co) {
            double acc = 0.0;
            for (int b = 0; b < B; ++b)
                for (int tp = 0; tp < Tp; ++tp) acc += dy[IDX3(b, tp, co, Tp, Cout)];
            dbias[co] = acc;
        }
    }
}

void orc_conv1d_bwd_weight_at(const double *x, const double *dy, const long long *idx, int n,
                              double *out, int B, int T, int Cin, int Cout, int k, int s)
{
#pragma omp parallel for schedule(dynamic, 4)
    for (int i = 0; i < n; ++i) {
        long long f = idx[i];
        int ci = (int)(f % Cin); f /= Cin;
        int j = (int)(f % k);
        int co = (int)(f / k);
        out[i] = conv_wgrad_elem(x, dy, B, T, Cin, Cout, k, s, co, j, ci);
    }
}

/* ---------------------------------------------------------------------------
 * Gated linear unit (the gated convnet the paper's CNN follows, Sec. 4.1).
 * The channel axis is split in halves: value a = y[..., :C/2], gate
 * g = y[..., C/2:];  h = a * sigmoid(g).
 * ------------------------------------------------------------------------- */
static double sigmoid(double u) { return 1.0 / (1.0 + exp(-u)); }

void orc_glu_fwd(const double *y, double *h, long long rows, int Cout)
{
    const int H = Cout / 2;
#pragma omp parallel for schedule(static)
    for (long long r = 0; r < rows; ++r)
        for (int c = 0; c < H; ++c)
            h[r * H + c] = y[r * Cout + c] * sigmoid(y[r * Cout + H + c]);
}

/*   da = dh * sigmoid(g);   dg = dh * a * sigmoid(g) * (1 - sigmoid(g))     */
void orc_glu_bwd(const double *y, const double *dh, double *dy, long long rows, int Cout)
{
    const int H = Cout / 2;
#pragma omp parallel for schedule(static)
    for (long long r = 0; r < rows; ++r)
        for (int c = 0; c < H; ++c) {
            const double a = y[r * Cout + c], sg = sigmoid(y[r * Cout + H + c]);
            const double d = dh[r * H + c];
            dy[r * Cout + c] = d * sg;
            dy[r * Cout + H + c] = d * a * sg * (1.0 - sg);
        }
}

/* ---------------------------------------------------------------------------
 * Per-frame log-softmax (the normalised per-frame scores CTC consumes,
 * Sec. 2.3):  lp[r,c] = z[r,c] - max_c z - log sum_c exp(z[r,c] - max_c z)
 * ------------------------------------------------------------------------- */
void orc_logsoftmax_fwd(const double *z, double *lp, long long rows, int C)
{
#pragma omp parallel for schedule(static)
    for (long long r = 0; r < rows; ++r) {
        const double *zr = z + r * C;
        double m = zr[0];
        for (int c = 1; c < C; ++c) if (zr[c] > m) m = zr[c];
        double sum = 0.0;
        for (int c = 0; c < C; ++c) sum += exp(zr[c] - m);
        const double lse = m + log(sum);
        for (int c = 0; c < C; ++c) lp[r * C + c] = zr[c] - lse;
    }
}

/*   dz[r,c] = dlp[r,c] - exp(lp[r,c]) * sum_c dlp[r,c]                      */
void orc_logsoftmax_bwd(const double *lp, const double *dlp, double *dz, long long rows, int C)
{
#pragma omp parallel for schedule(static)
    for (long long r = 0; r < rows; ++r) {
        double tot = 0.0;
        for (int c = 0; c < C; ++c) tot += dlp[r * C + c];
        for (int c = 0; c < C; ++c) dz[r * C + c] = dlp[r * C + c] - exp(lp[r * C + c]) * tot;
    }
}

/* ---------------------------------------------------------------------------
 * SGD with momentum (Sec. 4.1: every model in the paper's experiments is trained with
 * it; the update rule itself is not written out there).  Classical (heavy-ball) form,
 * with optional L2 weight decay folded into the gradient:
 *   v' = mu * v + (g + wd * w)
 *   w' = w - lr * v'
 * Elementwise over n values; w and v are updated in place. */
void orc_sgd_momentum(double *w, double *v, const double *g, long long n, double lr, double mu, double wd)
{
#pragma omp parallel for schedule(static)
    for (long long i = 0; i < n; ++i) {
        const double vn = mu * v[i] + (g[i] + wd * w[i]);
        v[i] = vn;
        w[i] = w[i] - lr * vn;
    }
}

/* ---------------------------------------------------------------------------
 * CTC criterion (Sec. 2.3, citing Graves et al. 2006), in log space.
 * For one utterance with T valid frames and target l_1..l_L, the extended
 * sequence l' = (blank, l_1, blank, ..., l_L, blank) has S = 2L+1 states and
 *   alpha_0(0) = lp[0,blank], alpha_0(1) = lp[0,l_1], others -inf
 *   alpha_t(s) = lp[t,l'_s] + lse( alpha_{t-1}(s), alpha_{t-1}(s-1),
 *                                  alpha_{t-1}(s-2) if l'_s != blank and l'_s != l'_{s-2} )
 *   log P      = lse( alpha_{T-1}(S-1), alpha_{T-1}(S-2) );   loss = -log P
 *   beta is the mirror image started from the last frame;
 *   gamma_t(s) = exp( alpha_t(s) + beta_t(s) - lp[t,l'_s] - log P )
 *   G[t,c]     = sum_{s : l'_s = c} gamma_t(s);   dloss/dlp[t,c] = -G[t,c].
 * Frames t >= T get gradient 0.  An utterance with no valid alignment has
 * loss +inf and gradient 0.  T = 0 gives loss 0 when L = 0, +inf otherwise.
 * ------------------------------------------------------------------------- */
static double lse2(double a, double b)
{
    if (a == -INFINITY) return b;
    if (b == -INFINITY) return a;
    const double m = a > b ? a : b;
    return m + log(exp(a - m) + exp(b - m));
}

/* Returns 0, or -1 if a label is the blank or outside [0,C).  alpha_out and
 * beta_out (nullable) are [B][Tp][2*Lmax+1], filled with -inf where unused. */
int orc_ctc(const double *lp, const int *targets, const int *in_len, const int *tgt_len,
            double *loss, double *grad_lp, double *alpha_out, double *beta_out,
            int B, int Tp, int C, int Lmax, int blank)
{
    const int Smax = 2 * Lmax + 1;
    int bad = 0;
    for (int b = 0; b < B; ++b) {
        if (in_len[b] < 0 || in_len[b] > Tp || tgt_len[b] < 0 || tgt_len[b] > Lmax) bad = 1;
        else
            for (int i = 0; i < tgt_len[b]; ++i) {
                const int l = targets[(size_t)b * Lmax + i];
                if (l < 0 || l >= C || l == blank) bad = 1;
            }
    }
    if (bad) return -1;

#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        const int T = in_len[b], L = tgt_len[b], S = 2 * L + 1;
        const double *lpb = lp + IDX3(b, 0, 0, Tp, C);
        const int *lab = targets + (size_t)b * Lmax;
        int *ext = (int *)malloc(sizeof(int) * (size_t)S);
        for (int s = 0; s < S; ++s) ext[s] = (s % 2 == 0) ? blank : lab[(s - 1) / 2];
        double *alpha = (double *)malloc(sizeof(double) * (size_t)(T > 0 ? T : 1) * S);
        double *beta = (double *)malloc(sizeof(double) * (size_t)(T > 0 ? T : 1) * S);

        if (grad_lp)
            for (size_t i = 0; i < (size_t)Tp * C; ++i) grad_lp[IDX3(b, 0, 0, Tp, C) + i] = 0.0;
        if (alpha_out)
            for (size_t i = 0; i < (size_t)Tp * Smax; ++i) alpha_out[IDX3(b, 0, 0, Tp, Smax) + i] = -INFINITY;
        if (beta_out)
            for (size_t i = 0; i < (size_t)Tp * Smax; ++i) beta_out[IDX3(b, 0, 0, Tp, Smax) + i] = -INFINITY;

        double logp;
        if (T == 0) {
            logp = (L == 0) ? 0.0 : -INFINITY;
        } else {
            for (int s = 0; s < S; ++s) alpha[s] = -INFINITY;
            alpha[0] = lpb[ext[0]];
            if (S > 1) alpha[1] = lpb[ext[1]];
            for (int t = 1; t < T; ++t)
                for (int s = 0; s < S; ++s) {
                    double a = alpha[(size_t)(t - 1) * S + s];
                    if (s >= 1) a = lse2(a, alpha[(size_t)(t - 1) * S + s - 1]);
                    if (s >= 2 && ext[s] != blank && ext[s] != ext[s - 2])
                        a = lse2(a, alpha[(size_t)(t - 1) * S + s - 2]);
                    alpha[(size_t)t * S + s] = (a == -INFINITY) ? -INFINITY : a + lpb[(size_t)t * C + ext[s]];
                }
            for (int s = 0; s < S; ++s) beta[(size_t)(T - 1) * S + s] = -INFINITY;
            beta[(size_t)(T - 1) * S + S - 1] = lpb[(size_t)(T - 1) * C + ext[S - 1]];
            if (S > 1) beta[(size_t)(T - 1) * S + S - 2] = lpb[(size_t)(T - 1) * C + ext[S - 2]];
            for (int t = T - 2; t >= 0; --t)
                for (int s = 0; s < S; ++s) {
                    double a = beta[(size_t)(t + 1) * S + s];
                    if (s + 1 < S) a = lse2(a, beta[(size_t)(t + 1) * S + s + 1]);
                    if (s + 2 < S && ext[s] != blank && ext[s] != ext[s + 2])
                        a = lse2(a, beta[(size_t)(t + 1) * S + s + 2]);
                    beta[(size_t)t * S + s] = (a == -INFINITY) ? -INFINITY : a + lpb[(size_t)t * C + ext[s]];
                }
            logp = alpha[(size_t)(T - 1) * S + S - 1];
            if (S > 1) logp = lse2(logp, alpha[(size_t)(T - 1) * S + S - 2]);
        }
        loss[b] = -logp;

        if (T > 0) {
            if (alpha_out)
                for (int t = 0; t < T; ++t)
                    for (int s = 0; s < S; ++s) alpha_out[IDX3(b, t, s, Tp, Smax)] = alpha[(size_t)t * S + s];
            if (beta_out)
                for (int t = 0; t < T; ++t)
                    for (int s = 0; s < S; ++s) beta_out[IDX3(b, t, s, Tp, Smax)] = beta[(size_t)t * S + s];
            if (grad_lp && logp != -INFINITY)
                for (int t = 0; t < T; ++t)
                    for (int s = 0; s < S; ++s) {
                        const double a = alpha[(size_t)t * S + s], bt = beta[(size_t)t * S + s];
                        if (a == -INFINITY || bt == -INFINITY) continue;
                        const double g = exp(a + bt - lpb[(size_t)t * C + ext[s]] - logp);
                        grad_lp[IDX3(b, t, ext[s], Tp, C)] -= g;
                    }
        }
        free(ext);
        free(alpha);
        free(beta);
    }
    return 0;
}

/* ---------------------------------------------------------------------------
 * ASG criterion (AutoSegCriterion; Sec. 2.3 lists it beside CTC and cites Collobert
 * et al. 2016 for it -- the paper itself prints no formula, so the definition below is
 * a stated reading of the cited criterion and is "parity unpinned" with respect to the
 * paper's own text; the tests pin it to this definition by brute-force enumeration,
 * closed forms and finite differences).
 *
 * No blank, no per-frame normalisation.  Inputs per utterance: emissions f[t][c]
 * (unnormalised scores, T valid frames, C classes), a learned transition matrix
 * g[i][j] = score of class j at frame t-1 being followed by class i at frame t, and a
 * target y_0..y_{L-1}.  The score of a frame labelling pi_0..pi_{T-1} is
 *   sc(pi) = sum_{t=0}^{T-1} f[t][pi_t] + sum_{t=1}^{T-1} g[pi_t][pi_{t-1}]
 *   FCC = log sum over all C^T labellings of exp(sc(pi))            ("fully connected")
 *   FAL = log sum over the monotone alignments s_0 = 0, s_{T-1} = L-1,
 *         s_t - s_{t-1} in {0,1}, pi_t = y_{s_t}, of exp(sc(pi))    ("forced alignment")
 *   loss = FCC - FAL   (>= 0: every alignment is one of the labellings)
 * Both by the log-space forward/backward recursions:
 *   A_0[i] = f[0][i];  A_t[i] = f[t][i] + lse_j( A_{t-1}[j] + g[i][j] );  FCC = lse_i A_{T-1}[i]
 *   a_0[0] = f[0][y_0]; a_t[s] = f[t][y_s] + lse( a_{t-1}[s] + g[y_s][y_s], a_{t-1}[s-1] + g[y_s][y_{s-1}] )
 *   FAL = a_{T-1}[L-1]
 * Gradients are differences of posteriors (occupancies of nodes and of edges):
 *   dloss/df[t][c]  = P_fcc(pi_t = c) - P_fal(pi_t = c)
 *   dloss/dg[i][j]  = sum_{t>=1} P_fcc(pi_t = i, pi_{t-1} = j) - the same under FAL
 * grad_trans is the sum over the batch (added in the order b = 0..B-1).  Frames
 * t >= T get gradient 0.  No valid alignment (T < L, or L = 0 with T > 0): loss +inf,
 * zero gradients.  T = 0 and L = 0: loss 0.
 * fcc_out / fal_out (nullable): the two terms per utterance.
 * Returns 0, or -1 for a label outside [0,C) or a length outside its range.
 * ------------------------------------------------------------------------- */
static double lse_n(const double *v, int n)
{
    double m = -INFINITY;
    for (int i = 0; i < n; ++i) if (v[i] > m) m = v[i];
    if (m == -INFINITY) return -INFINITY;
    double sum = 0.0;
    for (int i = 0; i < n; ++i) sum += exp(v[i] - m);
    return m + log(sum);
}

int orc_asg(const double *em, const double *trans, const int *targets, const int *in_len, const int *tgt_len,
            double *loss, double *grad_em, double *grad_trans, double *fcc_out, double *fal_out,
            int B, int Tp, int C, int Lmax)
{
    for (int b = 0; b < B; ++b) {
        if (in_len[b] < 0 || in_len[b] > Tp || tgt_len[b] < 0 || tgt_len[b] > Lmax) return -1;
        for (int i = 0; i < tgt_len[b]; ++i) {
            const int l = targets[(size_t)b * Lmax + i];
            if (l < 0 || l >= C) return -1;
        }
    }
    double *gt_b = (double *)calloc((size_t)B * C * C, sizeof(double)); /* per-utterance d loss_b / d g */

#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        const int T = in_len[b], L = tgt_len[b];
        const double *f = em + IDX3(b, 0, 0, Tp, C);
        const int *y = targets + (size_t)b * Lmax;
        double *ge = grad_em ? grad_em + IDX3(b, 0, 0, Tp, C) : NULL;
        double *gt = gt_b + (size_t)b * C * C;
        if (ge) for (size_t i = 0; i < (size_t)Tp * C; ++i) ge[i] = 0.0;
        if (T == 0) {
            const double fal0 = (L == 0) ? 0.0 : -INFINITY;
            if (fcc_out) fcc_out[b] = 0.0;
            if (fal_out) fal_out[b] = fal0;
            loss[b] = 0.0 - fal0;
            continue;
        }
        double *tmp = (double *)malloc(sizeof(double) * (size_t)C);
        /* fully connected lattice */
        double *A = (double *)malloc(sizeof(double) * (size_t)T * C);
        double *Bt = (double *)malloc(sizeof(double) * (size_t)T * C);
        for (int i = 0; i < C; ++i) A[i] = f[i];
        for (int t = 1; t < T; ++t)
            for (int i = 0; i < C; ++i) {
                for (int j = 0; j < C; ++j) tmp[j] = A[(size_t)(t - 1) * C + j] + trans[(size_t)i * C + j];
                A[(size_t)t * C + i] = f[(size_t)t * C + i] + lse_n(tmp, C);
            }
        const double fcc = lse_n(A + (size_t)(T - 1) * C, C);
        for (int j = 0; j < C; ++j) Bt[(size_t)(T - 1) * C + j] = 0.0;
        for (int t = T - 2; t >= 0; --t)
            for (int j = 0; j < C; ++j) {
                for (int i = 0; i < C; ++i)
                    tmp[i] = trans[(size_t)i * C + j] + f[(size_t)(t + 1) * C + i] + Bt[(size_t)(t + 1) * C + i];
                Bt[(size_t)t * C + j] = lse_n(tmp, C);
            }
        /* forced alignment lattice */
        double fal = -INFINITY;
        double *a = NULL, *bb = NULL;
        const int feasible = (L >= 1 && L <= T);
        if (feasible) {
            a = (double *)malloc(sizeof(double) * (size_t)T * L);
            bb = (double *)malloc(sizeof(double) * (size_t)T * L);
            for (int s = 0; s < L; ++s) a[s] = -INFINITY;
            a[0] = f[y[0]];
            for (int t = 1; t < T; ++t)
                for (int s = 0; s < L; ++s) {
                    double v = a[(size_t)(t - 1) * L + s] + trans[(size_t)y[s] * C + y[s]];
                    if (s >= 1) v = lse2(v, a[(size_t)(t - 1) * L + s - 1] + trans[(size_t)y[s] * C + y[s - 1]]);
                    a[(size_t)t * L + s] = (v == -INFINITY) ? -INFINITY : v + f[(size_t)t * C + y[s]];
                }
            fal = a[(size_t)(T - 1) * L + L - 1];
            for (int s = 0; s < L; ++s) bb[(size_t)(T - 1) * L + s] = -INFINITY;
            bb[(size_t)(T - 1) * L + L - 1] = 0.0;
            for (int t = T - 2; t >= 0; --t)
                for (int s = 0; s < L; ++s) {
                    double v = trans[(size_t)y[s] * C + y[s]] + f[(size_t)(t + 1) * C + y[s]] + bb[(size_t)(t + 1) * L + s];
                    if (s + 1 < L)
                        v = lse2(v, trans[(size_t)y[s + 1] * C + y[s]] + f[(size_t)(t + 1) * C + y[s + 1]] +
                                        bb[(size_t)(t + 1) * L + s + 1]);
                    bb[(size_t)t * L + s] = v;
                }
        }
        if (fcc_out) fcc_out[b] = fcc;
        if (fal_out) fal_out[b] = fal;
        loss[b] = fcc - fal;
        if (feasible && fal != -INFINITY) {
            /* + fully connected occupancies */
            for (int t = 0; t < T; ++t)
                for (int i = 0; i < C; ++i) {
                    if (ge) ge[(size_t)t * C + i] += exp(A[(size_t)t * C + i] + Bt[(size_t)t * C + i] - fcc);
                    if (t >= 1)
                        for (int j = 0; j < C; ++j)
                            gt[(size_t)i * C + j] += exp(A[(size_t)(t - 1) * C + j] + trans[(size_t)i * C + j] +
                                                         f[(size_t)t * C + i] + Bt[(size_t)t * C + i] - fcc);
                }
            /* - forced alignment occupancies */
            for (int t = 0; t < T; ++t)
                for (int s = 0; s < L; ++s) {
                    const double av = a[(size_t)t * L + s], bv = bb[(size_t)t * L + s];
                    if (av != -INFINITY && bv != -INFINITY && ge) ge[(size_t)t * C + y[s]] -= exp(av + bv - fal);
                    if (t >= 1 && bv != -INFINITY) {
                        const double tail = f[(size_t)t * C + y[s]] + bv - fal;
                        const double stay = a[(size_t)(t - 1) * L + s];
                        if (stay != -INFINITY)
                            gt[(size_t)y[s] * C + y[s]] -= exp(stay + trans[(size_t)y[s] * C + y[s]] + tail);
                        if (s >= 1 && a[(size_t)(t - 1) * L + s - 1] != -INFINITY)
                            gt[(size_t)y[s] * C + y[s - 1]] -=
                                exp(a[(size_t)(t - 1) * L + s - 1] + trans[(size_t)y[s] * C + y[s - 1]] + tail);
                    }
                }
        }
        free(tmp); free(A); free(Bt); free(a); free(bb);
    }
    if (grad_trans) {
        for (size_t i = 0; i < (size_t)C * C; ++i) grad_trans[i] = 0.0;
        for (int b = 0; b < B; ++b)
            for (size_t i = 0; i < (size_t)C * C; ++i) grad_trans[i] += gt_b[(size_t)b * C * C + i];
    }
    free(gt_b);
    return 0;
}

int orc_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp single
        n = omp_get_num_threads();
    }
#endif
    return n;
}
