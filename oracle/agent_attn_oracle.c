/*
 * CPU oracle for the agent-attention forward pass (arXiv 2312.08874).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, fp64 statement of
 * what the GPU library must compute.  It shares no code, header, table or
 * helper with the HIP path, and nothing in the product path may call it.
 *
 * Every function works on double arrays that hold the (already rounded)
 * inputs exactly, so the only arithmetic error here is fp64 round-off.
 * Loops follow the paper's definitions term by term; there is no blocking,
 * fusion or reordering.  OpenMP is used only across independent output rows.
 *
 * Layout conventions (all row-major, last index fastest):
 *   tokens live on a grid of gh x gw, token t = y*gw + x;
 *   agents live on a grid of ah x aw, agent a = ay*aw + ax;
 *   a "unit" is one (batch, head) pair, u = b*heads + head.
 *
 * Pins (tests that tie these functions to something other than themselves)
 * are listed in tests/test_oracle_pins.py.  Two choices below are readings of
 * passages the paper leaves open and are "parity unpinned" by the paper
 * itself: the half-pixel bilinear rule in oracle_resize_bilinear() and the
 * zero padding / cross-correlation orientation in oracle_dwc().  Both are
 * pinned only against library routines that implement the same stated rule.
 */
#include <math.h>
#include <stddef.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------------
 * Softmax attention, Sec. 3.1 Eq. (1) with Sim(q,k) = exp(q.k * scale)
 * (Sec. 3.2) and an optional additive bias inside the exponent
 * (Sec. 4.2 Eq. (5)):
 *
 *   out[i,:] = sum_j w[i,j] Vm[j,:],
 *   w[i,j]   = exp(s[i,j]) / sum_j' exp(s[i,j']),
 *   s[i,j]   = scale * <Qm[i,:], Km[j,:]> + bias[i,j].
 *
 * Qm [M,d], Km [L,d], Vm [L,dv], bias [M,L] or NULL, out [M,dv].
 * The row maximum is subtracted before exp (same value, no overflow).
 * If weights != NULL it receives the normalised w [M,L].
 * ---------------------------------------------------------------------- */
void oracle_softmax_attention(const double *Qm, const double *Km,
                              const double *Vm, const double *bias,
                              double scale, int M, int L, int d, int dv,
                              double *out, double *weights)
{
#pragma omp parallel
    {
        double *s = (double *)malloc((size_t)L * sizeof(double));
#pragma omp for schedule(static)
        for (int i = 0; i < M; ++i) {
            double smax = -INFINITY;
            for (int j = 0; j < L; ++j) {
                double dot = 0.0;
                for (int c = 0; c < d; ++c)
                    dot += Qm[(size_t)i * d + c] * Km[(size_t)j * d + c];
                double v = scale * dot;
                if (bias) v += bias[(size_t)i * L + j];
                s[j] = v;
                if (v > smax) smax = v;
            }
            double denom = 0.0;
            for (int j = 0; j < L; ++j) {
                s[j] = exp(s[j] - smax);
                denom += s[j];
            }
            for (int j = 0; j < L; ++j) s[j] /= denom;
            if (weights)
                for (int j = 0; j < L; ++j) weights[(size_t)i * L + j] = s[j];
            for (int c = 0; c < dv; ++c) {
                double acc = 0.0;
                for (int j = 0; j < L; ++j) acc += s[j] * Vm[(size_t)j * dv + c];
                out[(size_t)i * dv + c] = acc;
            }
        }
        free(s);
    }
}

/* ------------------------------------------------------------------------
 * Agent tokens by pooling, Sec. 4.2 ("A = Pooling(Q)", Fig. 3(b)).
 * Average pooling of the gh x gw token grid onto the ah x aw agent grid.
 * Output index i along an axis of length L pooled to La covers
 *   [ floor(i*L/La), ceil((i+1)*L/La) )
 * which is the disjoint equal-window rule whenever La divides L.
 * Q [units, gh*gw, d] -> A [units, ah*aw, d].
 * ---------------------------------------------------------------------- */
static int win_lo(int i, int L, int La) { return (int)(((long long)i * L) / La); }
static int win_hi(int i, int L, int La)
{
    return (int)((((long long)(i + 1)) * L + La - 1) / La);
}

void oracle_pool(const double *Q, int units, int gh, int gw, int ah, int aw,
                 int d, double *A)
{
    const size_t N = (size_t)gh * gw, n = (size_t)ah * aw;
#pragma omp parallel for schedule(static)
    for (int u = 0; u < units; ++u) {
        for (int ay = 0; ay < ah; ++ay)
            for (int ax = 0; ax < aw; ++ax) {
                int y0 = win_lo(ay, gh, ah), y1 = win_hi(ay, gh, ah);
                int x0 = win_lo(ax, gw, aw), x1 = win_hi(ax, gw, aw);
                double cnt = (double)(y1 - y0) * (double)(x1 - x0);
                for (int c = 0; c < d; ++c) {
                    double acc = 0.0;
                    for (int y = y0; y < y1; ++y)
                        for (int x = x0; x < x1; ++x)
                            acc += Q[((size_t)u * N + (size_t)y * gw + x) * d + c];
                    A[((size_t)u * n + (size_t)ay * aw + ax) * d + c] = acc / cnt;
                }
            }
    }
}

/* ------------------------------------------------------------------------
 * Bilinear resize of one h0 x w0 plane to h x w (Appendix B, "resized ... by
 * interpolating"; the paper names no rule, this is the reading taken):
 * half-pixel centres, src = (dst + 0.5) * (L0 / L) - 0.5 clamped below at 0,
 * upper neighbour clamped to L0-1.  Identity when h0 == h and w0 == w.
 * `stride` lets the plane be a strided slice (used for the [h0,w0,n] layout).
 * ---------------------------------------------------------------------- */
static void src_coord(int dst, int L, int L0, int *i0, int *i1, double *frac)
{
    double s = ((double)dst + 0.5) * ((double)L0 / (double)L) - 0.5;
    if (s < 0.0) s = 0.0;
    int lo = (int)floor(s);
    if (lo > L0 - 1) lo = L0 - 1;
    int hi = lo + 1 < L0 ? lo + 1 : L0 - 1;
    *i0 = lo;
    *i1 = hi;
    *frac = s - (double)lo;
}

void oracle_resize_bilinear(const double *src, int h0, int w0, size_t stride,
                            int h, int w, double *dst /* [h*w] dense */)
{
    for (int y = 0; y < h; ++y) {
        int y0, y1;
        double fy;
        src_coord(y, h, h0, &y0, &y1, &fy);
        for (int x = 0; x < w; ++x) {
            int x0, x1;
            double fx;
            src_coord(x, w, w0, &x0, &x1, &fx);
            double v00 = src[((size_t)y0 * w0 + x0) * stride];
            double v01 = src[((size_t)y0 * w0 + x1) * stride];
            double v10 = src[((size_t)y1 * w0 + x0) * stride];
            double v11 = src[((size_t)y1 * w0 + x1) * stride];
            double top = v00 + (v01 - v00) * fx;
            double bot = v10 + (v11 - v10) * fx;
            dst[(size_t)y * w + x] = top + (bot - top) * fy;
        }
    }
}

/* ------------------------------------------------------------------------
 * Agent bias composition, Appendix B, for ONE head.
 *
 *   B1[a, y*w+x] = col1[a,x] + row1[a,y] + resize(blk1[a,:,:])[y,x]
 *     col1 [n,w], row1 [n,h], blk1 [n,h0,w0]            -> B1 [n,N]
 *   B2[y*w+x, a] = col2[x,a] + row2[y,a] + resize(blk2[:,:,a])[y,x]
 *     col2 [w,n], row2 [h,n], blk2 [h0,w0,n]            -> B2 [N,n]
 *
 * Column and row components are repeated along the missing axis, the block
 * component is interpolated.  Any component pointer may be NULL (= zero).
 * ---------------------------------------------------------------------- */
void oracle_bias1_dense(const double *col1, const double *row1,
                        const double *blk1, int n, int h, int w, int h0,
                        int w0, double *B1)
{
    const size_t N = (size_t)h * w;
    double *plane = (double *)malloc(N * sizeof(double));
    for (int a = 0; a < n; ++a) {
        if (blk1)
            oracle_resize_bilinear(blk1 + (size_t)a * h0 * w0, h0, w0, 1, h, w, plane);
        else
            memset(plane, 0, N * sizeof(double));
        for (int y = 0; y < h; ++y)
            for (int x = 0; x < w; ++x) {
                double v = plane[(size_t)y * w + x];
                if (col1) v += col1[(size_t)a * w + x];
                if (row1) v += row1[(size_t)a * h + y];
                B1[(size_t)a * N + (size_t)y * w + x] = v;
            }
    }
    free(plane);
}

void oracle_bias2_dense(const double *col2, const double *row2,
                        const double *blk2, int n, int h, int w, int h0,
                        int w0, double *B2)
{
    const size_t N = (size_t)h * w;
    double *plane = (double *)malloc(N * sizeof(double));
    for (int a = 0; a < n; ++a) {
        if (blk2)
            oracle_resize_bilinear(blk2 + a, h0, w0, (size_t)n, h, w, plane);
        else
            memset(plane, 0, N * sizeof(double));
        for (int y = 0; y < h; ++y)
            for (int x = 0; x < w; ++x) {
                double v = plane[(size_t)y * w + x];
                if (col2) v += col2[(size_t)x * n + a];
                if (row2) v += row2[(size_t)y * n + a];
                B2[((size_t)y * w + x) * n + a] = v;
            }
    }
    free(plane);
}

/* ------------------------------------------------------------------------
 * Diversity-restoration term DWC(V), Sec. 4.2 Eq. (6): depthwise 3x3
 * convolution (k = 3, Eq. (7)) of V viewed as a gh x gw image with d channels.
 * Reading taken where the paper is silent: stride 1, zero padding 1,
 * cross-correlation orientation
 *   out[y,x,c] = b[c] + sum_{u,v in {-1,0,1}} wgt[c,u+1,v+1] * V[y+u,x+v,c].
 * V [gh*gw, d], wgt [d,3,3], b [d] or NULL, out [gh*gw, d].  One unit.
 * ---------------------------------------------------------------------- */
void oracle_dwc(const double *V, const double *wgt, const double *b, int gh,
                int gw, int d, double *out)
{
#pragma omp parallel for schedule(static)
    for (int y = 0; y < gh; ++y)
        for (int x = 0; x < gw; ++x)
            for (int c = 0; c < d; ++c) {
                double acc = b ? b[c] : 0.0;
                for (int u = -1; u <= 1; ++u)
                    for (int v = -1; v <= 1; ++v) {
                        int yy = y + u, xx = x + v;
                        if (yy < 0 || yy >= gh || xx < 0 || xx >= gw) continue;
                        acc += wgt[(size_t)c * 9 + (size_t)(u + 1) * 3 + (v + 1)] *
                               V[((size_t)yy * gw + xx) * d + c];
                    }
                out[((size_t)y * gw + x) * d + c] = acc;
            }
}

/* ------------------------------------------------------------------------
 * Split-N bookkeeping (an implementation device, exact by softmax algebra).
 * oracle_aggregate_partial: un-normalised aggregation of agents over the
 * token range [t0,t1): m[a] = max_j s[a,j], l[a] = sum_j exp(s[a,j]-m[a]),
 * acc[a,:] = sum_j exp(s[a,j]-m[a]) V[j,:].
 * oracle_merge_partials: m = max_s m_s; l = sum_s l_s e^{m_s-m};
 * VA = sum_s acc_s e^{m_s-m} / l.
 * ---------------------------------------------------------------------- */
void oracle_aggregate_partial(const double *A, const double *K, const double *V,
                              const double *B1 /* [n,N] or NULL */, double scale,
                              int n, int N, int d, int t0, int t1, double *m,
                              double *l, double *acc /* [n,d] */)
{
    for (int a = 0; a < n; ++a) {
        double smax = -INFINITY;
        for (int j = t0; j < t1; ++j) {
            double dot = 0.0;
            for (int c = 0; c < d; ++c) dot += A[(size_t)a * d + c] * K[(size_t)j * d + c];
            double v = scale * dot + (B1 ? B1[(size_t)a * N + j] : 0.0);
            if (v > smax) smax = v;
        }
        double denom = 0.0;
        for (int c = 0; c < d; ++c) acc[(size_t)a * d + c] = 0.0;
        for (int j = t0; j < t1; ++j) {
            double dot = 0.0;
            for (int c = 0; c < d; ++c) dot += A[(size_t)a * d + c] * K[(size_t)j * d + c];
            double v = scale * dot + (B1 ? B1[(size_t)a * N + j] : 0.0);
            double p = exp(v - smax);
            denom += p;
            for (int c = 0; c < d; ++c) acc[(size_t)a * d + c] += p * V[(size_t)j * d + c];
        }
        m[a] = smax;
        l[a] = denom;
    }
}

void oracle_merge_partials(const double *m /* [S,n] */, const double *l /* [S,n] */,
                           const double *acc /* [S,n,d] */, int S, int n, int d,
                           double *VA /* [n,d] */)
{
    for (int a = 0; a < n; ++a) {
        double mm = -INFINITY;
        for (int s = 0; s < S; ++s)
            if (m[(size_t)s * n + a] > mm) mm = m[(size_t)s * n + a];
        double ll = 0.0;
        for (int s = 0; s < S; ++s) ll += l[(size_t)s * n + a] * exp(m[(size_t)s * n + a] - mm);
        for (int c = 0; c < d; ++c) {
            double v = 0.0;
            for (int s = 0; s < S; ++s)
                v += acc[((size_t)s * n + a) * d + c] * exp(m[(size_t)s * n + a] - mm);
            VA[(size_t)a * d + c] = v / ll;
        }
    }
}

/* ------------------------------------------------------------------------
 * The whole forward pass over all units.
 *
 *   A   = Pooling(Q)                        (Sec. 4.2)   unless A_in given
 *   VA  = Attn^S(A, K, V)  with bias B1     (Sec. 4.1 Eq. (3), "agent
 *                                            aggregation"; Eq. (5))
 *   O   = Attn^S(Q, A, VA) with bias B2     ("agent broadcast")
 *   O  += DWC(V)                            (Eq. (6))     if dwc_w given
 *   O  += vk * V                            (Appendix C.1) if vk != 0
 *
 * Q,K,V [units,N,d]; A_in [units,n,d] or NULL; B1 [heads,n,N] or NULL;
 * B2 [heads,N,n] or NULL; dwc_w [heads,d,3,3] or NULL; dwc_b [heads,d] or
 * NULL; outputs O [units,N,d], and if non-NULL A_out [units,n,d],
 * VA_out [units,n,d].  Head of unit u is u % heads (bias and DWC parameters
 * are per head and shared across the batch).
 * ---------------------------------------------------------------------- */
void oracle_agent_attn_fwd(const double *Q, const double *K, const double *V,
                           const double *A_in, int units, int heads, int gh,
                           int gw, int ah, int aw, int N, int n, int d,
                           double scale1, double scale2, const double *B1,
                           const double *B2, const double *dwc_w,
                           const double *dwc_b, double vk, double *O,
                           double *A_out, double *VA_out)
{
    double *A = (double *)malloc((size_t)n * d * sizeof(double));
    double *VA = (double *)malloc((size_t)n * d * sizeof(double));
    double *conv = dwc_w ? (double *)malloc((size_t)N * d * sizeof(double)) : NULL;
    for (int u = 0; u < units; ++u) {
        const int hd = u % heads;
        const double *Qu = Q + (size_t)u * N * d;
        const double *Ku = K + (size_t)u * N * d;
        const double *Vu = V + (size_t)u * N * d;
        double *Ou = O + (size_t)u * N * d;
        if (A_in)
            memcpy(A, A_in + (size_t)u * n * d, (size_t)n * d * sizeof(double));
        else
            oracle_pool(Qu, 1, gh, gw, ah, aw, d, A);
        oracle_softmax_attention(A, Ku, Vu, B1 ? B1 + (size_t)hd * n * N : NULL,
                                 scale1, n, N, d, d, VA, NULL);
        oracle_softmax_attention(Qu, A, VA, B2 ? B2 + (size_t)hd * N * n : NULL,
                                 scale2, N, n, d, d, Ou, NULL);
        if (dwc_w) {
            oracle_dwc(Vu, dwc_w + (size_t)hd * d * 9,
                       dwc_b ? dwc_b + (size_t)hd * d : NULL, gh, gw, d, conv);
            for (size_t e = 0; e < (size_t)N * d; ++e) Ou[e] += conv[e];
        }
        if (vk != 0.0)
            for (size_t e = 0; e < (size_t)N * d; ++e) Ou[e] += vk * Vu[e];
        if (A_out) memcpy(A_out + (size_t)u * n * d, A, (size_t)n * d * sizeof(double));
        if (VA_out) memcpy(VA_out + (size_t)u * n * d, VA, (size_t)n * d * sizeof(double));
    }
    free(A);
    free(VA);
    free(conv);
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    return omp_get_max_threads();
#else
    return 1;
#endif
}
