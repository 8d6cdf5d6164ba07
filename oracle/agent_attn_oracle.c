/*
 * CPU oracle for the agent-attention forward pass (arXiv 2312.08874) and its
 * gradients.
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
 * The same holds for the agent-axis interpolation of the bias
 * (oracle_resize_agent_axis(), Appendix D gives no rule).
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
 * Linear projection of the module (Sec. 4.2; the 4NC^2 term of Eq. (7)):
 *   Y[r, o] = sum_k X[r, k] * W[o, k] + b[o]
 * X [rows, K], W [O, K] (one row per output channel), b [O] or NULL, Y [rows, O].
 * ---------------------------------------------------------------------- */
void oracle_linear(const double *X, const double *W, const double *b, int rows,
                   int K, int O, double *Y)
{
#pragma omp parallel for schedule(static)
    for (int r = 0; r < rows; ++r)
        for (int o = 0; o < O; ++o) {
            double acc = 0.0;
            for (int k = 0; k < K; ++k)
                acc += X[(size_t)r * K + k] * W[(size_t)o * K + k];
            if (b) acc += b[o];
            Y[(size_t)r * O + o] = acc;
        }
}

/* ------------------------------------------------------------------------
 * Agent bias adapted to another number of agent tokens (Appendix D.1 / D.2,
 * "Numbers of agent tokens": the bias of a model trained with n agents is
 * bilinearly interpolated to the larger n used on higher-resolution inputs).
 * A bias component is viewed as [outer, ah, aw, inner] with the agents on an
 * ah x aw grid (agent a = ay*aw + ax); every [ah, aw] image (one per outer
 * and inner index) is resized to [ah2, aw2] with the same half-pixel rule as
 * oracle_resize_bilinear().  dst [outer, ah2, aw2, inner].
 * ---------------------------------------------------------------------- */
void oracle_resize_agent_axis(const double *src, int outer, int ah, int aw,
                              int inner, int ah2, int aw2, double *dst)
{
    double *plane = (double *)malloc((size_t)ah2 * aw2 * sizeof(double));
    for (int o = 0; o < outer; ++o)
        for (int i = 0; i < inner; ++i) {
            oracle_resize_bilinear(src + (size_t)o * ah * aw * inner + i, ah, aw,
                                   (size_t)inner, ah2, aw2, plane);
            for (int a = 0; a < ah2 * aw2; ++a)
                dst[((size_t)o * ah2 * aw2 + a) * inner + i] = plane[a];
        }
    free(plane);
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

/* ========================================================================
 * Backward pass.  The paper trains its models end to end (Sec. 5, training
 * set-up), so every operation above needs its gradient; the paper prints none
 * of them, they follow from the definitions by the chain rule and are written
 * out here term by term.  Pins: central finite differences of the forward
 * oracle and an automatic-differentiation library on the same definition
 * (tests/test_oracle_bwd_pins.py).
 * ====================================================================== */

/* ------------------------------------------------------------------------
 * Gradient of oracle_softmax_attention.  With w the normalised weights and
 * g = d(loss)/d(out):
 *   dVm[j,:]  = sum_i w[i,j] g[i,:]
 *   dW[i,j]   = <g[i,:], Vm[j,:]>
 *   dS[i,j]   = w[i,j] (dW[i,j] - sum_j' w[i,j'] dW[i,j'])      (softmax rows)
 *   dBias     = dS
 *   dQm[i,:]  = scale sum_j dS[i,j] Km[j,:]
 *   dKm[j,:]  = scale sum_i dS[i,j] Qm[i,:]
 * dQm [M,d], dKm [L,d], dVm [L,dv] are overwritten; dBias [M,L] (may be NULL)
 * is ACCUMULATED into (bias parameters are shared across the batch).
 * ---------------------------------------------------------------------- */
void oracle_softmax_attention_bwd(const double *Qm, const double *Km,
                                  const double *Vm, const double *bias,
                                  double scale, int M, int L, int d, int dv,
                                  const double *g, double *dQm, double *dKm,
                                  double *dVm, double *dBias)
{
    double *w = (double *)malloc((size_t)M * L * sizeof(double));
    double *dS = (double *)malloc((size_t)M * L * sizeof(double));
    double *out = (double *)malloc((size_t)M * dv * sizeof(double));
    oracle_softmax_attention(Qm, Km, Vm, bias, scale, M, L, d, dv, out, w);
    for (int i = 0; i < M; ++i) {
        double inner = 0.0;
        for (int j = 0; j < L; ++j) {
            double dW = 0.0;
            for (int c = 0; c < dv; ++c)
                dW += g[(size_t)i * dv + c] * Vm[(size_t)j * dv + c];
            dS[(size_t)i * L + j] = dW;
            inner += w[(size_t)i * L + j] * dW;
        }
        for (int j = 0; j < L; ++j)
            dS[(size_t)i * L + j] = w[(size_t)i * L + j] * (dS[(size_t)i * L + j] - inner);
    }
    for (int j = 0; j < L; ++j)
        for (int c = 0; c < dv; ++c) {
            double acc = 0.0;
            for (int i = 0; i < M; ++i)
                acc += w[(size_t)i * L + j] * g[(size_t)i * dv + c];
            dVm[(size_t)j * dv + c] = acc;
        }
    for (int i = 0; i < M; ++i)
        for (int c = 0; c < d; ++c) {
            double acc = 0.0;
            for (int j = 0; j < L; ++j)
                acc += dS[(size_t)i * L + j] * Km[(size_t)j * d + c];
            dQm[(size_t)i * d + c] = scale * acc;
        }
    for (int j = 0; j < L; ++j)
        for (int c = 0; c < d; ++c) {
            double acc = 0.0;
            for (int i = 0; i < M; ++i)
                acc += dS[(size_t)i * L + j] * Qm[(size_t)i * d + c];
            dKm[(size_t)j * d + c] = scale * acc;
        }
    if (dBias)
        for (size_t e = 0; e < (size_t)M * L; ++e) dBias[e] += dS[e];
    free(w);
    free(dS);
    free(out);
}

/* ------------------------------------------------------------------------
 * Gradient of oracle_pool for one unit: every token of agent a's window
 * receives dA[a,:] / |window|.  dA [n,d]; dQ [N,d] is ACCUMULATED into.
 * ---------------------------------------------------------------------- */
void oracle_pool_bwd(const double *dA, int gh, int gw, int ah, int aw, int d,
                     double *dQ)
{
    for (int ay = 0; ay < ah; ++ay)
        for (int ax = 0; ax < aw; ++ax) {
            int y0 = win_lo(ay, gh, ah), y1 = win_hi(ay, gh, ah);
            int x0 = win_lo(ax, gw, aw), x1 = win_hi(ax, gw, aw);
            double cnt = (double)(y1 - y0) * (double)(x1 - x0);
            for (int y = y0; y < y1; ++y)
                for (int x = x0; x < x1; ++x)
                    for (int c = 0; c < d; ++c)
                        dQ[((size_t)y * gw + x) * d + c] +=
                            dA[((size_t)ay * aw + ax) * d + c] / cnt;
        }
}

/* ------------------------------------------------------------------------
 * Gradient of oracle_dwc for one unit, g = d(loss)/d(out) [gh*gw, d]:
 *   dV[y+u,x+v,c]  += wgt[c,u+1,v+1] g[y,x,c]
 *   dwgt[c,u+1,v+1] += V[y+u,x+v,c]  g[y,x,c]
 *   db[c]          += g[y,x,c]
 * All three outputs are ACCUMULATED into; dwgt / db may be NULL.
 * ---------------------------------------------------------------------- */
void oracle_dwc_bwd(const double *V, const double *wgt, const double *g, int gh,
                    int gw, int d, double *dV, double *dwgt, double *db)
{
    for (int y = 0; y < gh; ++y)
        for (int x = 0; x < gw; ++x)
            for (int c = 0; c < d; ++c) {
                double gv = g[((size_t)y * gw + x) * d + c];
                if (db) db[c] += gv;
                for (int u = -1; u <= 1; ++u)
                    for (int v = -1; v <= 1; ++v) {
                        int yy = y + u, xx = x + v;
                        if (yy < 0 || yy >= gh || xx < 0 || xx >= gw) continue;
                        size_t wi = (size_t)c * 9 + (size_t)(u + 1) * 3 + (v + 1);
                        size_t vi = ((size_t)yy * gw + xx) * d + c;
                        dV[vi] += wgt[wi] * gv;
                        if (dwgt) dwgt[wi] += V[vi] * gv;
                    }
            }
}

/* ------------------------------------------------------------------------
 * Gradient of the bias composition (adjoint of oracle_bias1_dense /
 * oracle_bias2_dense) for ONE head: the dense gradient is summed along the
 * axis each component was repeated over, and pushed back through the
 * bilinear weights for the block component.  Outputs are overwritten; any
 * may be NULL.
 * ---------------------------------------------------------------------- */
static void resize_bilinear_bwd(const double *gdst /* [h*w] */, int h0, int w0,
                                size_t stride, int h, int w, double *gsrc)
{
    for (int y = 0; y < h; ++y) {
        int y0, y1;
        double fy;
        src_coord(y, h, h0, &y0, &y1, &fy);
        for (int x = 0; x < w; ++x) {
            int x0, x1;
            double fx;
            src_coord(x, w, w0, &x0, &x1, &fx);
            double gv = gdst[(size_t)y * w + x];
            gsrc[((size_t)y0 * w0 + x0) * stride] += gv * (1.0 - fy) * (1.0 - fx);
            gsrc[((size_t)y0 * w0 + x1) * stride] += gv * (1.0 - fy) * fx;
            gsrc[((size_t)y1 * w0 + x0) * stride] += gv * fy * (1.0 - fx);
            gsrc[((size_t)y1 * w0 + x1) * stride] += gv * fy * fx;
        }
    }
}

void oracle_bias1_components_bwd(const double *dB1 /* [n,N] */, int n, int h,
                                 int w, int h0, int w0, double *dcol1,
                                 double *drow1, double *dblk1)
{
    const size_t N = (size_t)h * w;
    if (dcol1) memset(dcol1, 0, (size_t)n * w * sizeof(double));
    if (drow1) memset(drow1, 0, (size_t)n * h * sizeof(double));
    if (dblk1) memset(dblk1, 0, (size_t)n * h0 * w0 * sizeof(double));
    for (int a = 0; a < n; ++a) {
        for (int y = 0; y < h; ++y)
            for (int x = 0; x < w; ++x) {
                double gv = dB1[(size_t)a * N + (size_t)y * w + x];
                if (dcol1) dcol1[(size_t)a * w + x] += gv;
                if (drow1) drow1[(size_t)a * h + y] += gv;
            }
        if (dblk1)
            resize_bilinear_bwd(dB1 + (size_t)a * N, h0, w0, 1, h, w,
                                dblk1 + (size_t)a * h0 * w0);
    }
}

void oracle_bias2_components_bwd(const double *dB2 /* [N,n] */, int n, int h,
                                 int w, int h0, int w0, double *dcol2,
                                 double *drow2, double *dblk2)
{
    const size_t N = (size_t)h * w;
    double *plane = (double *)malloc(N * sizeof(double));
    if (dcol2) memset(dcol2, 0, (size_t)w * n * sizeof(double));
    if (drow2) memset(drow2, 0, (size_t)h * n * sizeof(double));
    if (dblk2) memset(dblk2, 0, (size_t)h0 * w0 * n * sizeof(double));
    for (int a = 0; a < n; ++a) {
        for (int y = 0; y < h; ++y)
            for (int x = 0; x < w; ++x) {
                double gv = dB2[((size_t)y * w + x) * n + a];
                plane[(size_t)y * w + x] = gv;
                if (dcol2) dcol2[(size_t)x * n + a] += gv;
                if (drow2) drow2[(size_t)y * n + a] += gv;
            }
        if (dblk2) resize_bilinear_bwd(plane, h0, w0, (size_t)n, h, w, dblk2 + a);
    }
    free(plane);
}

/* ------------------------------------------------------------------------
 * Gradient of oracle_agent_attn_fwd.  g = d(loss)/dO [units,N,d].
 *
 *   O = Attn(Q, A, VA; B2) + DWC(V) + vk V,  VA = Attn(A, K, V; B1),
 *   A = Pooling(Q) or given.
 *
 *   broadcast stage  -> dQ, dA (as keys), dVA, dB2
 *   aggregation stage-> dA (as queries), dK, dV, dB1        (fed with dVA)
 *   dV += DWC^T(g) + vk g;   A pooled: dQ += Pooling^T(dA);  A given: dA out.
 *
 * dQ, dK, dV [units,N,d] overwritten; dA_out [units,n,d] overwritten (used
 * only when A_in is given, else ignored / may be NULL); dB1 [heads,n,N],
 * dB2 [heads,N,n], ddwc_w [heads,d,3,3], ddwc_b [heads,d]: overwritten with
 * the sum over the batch, each may be NULL.
 * ---------------------------------------------------------------------- */
void oracle_agent_attn_bwd(const double *Q, const double *K, const double *V,
                           const double *A_in, int units, int heads, int gh,
                           int gw, int ah, int aw, int N, int n, int d,
                           double scale1, double scale2, const double *B1,
                           const double *B2, const double *dwc_w,
                           const double *dwc_b, double vk, const double *g,
                           double *dQ, double *dK, double *dV, double *dA_out,
                           double *dB1, double *dB2, double *ddwc_w,
                           double *ddwc_b)
{
    (void)dwc_b;
    double *A = (double *)malloc((size_t)n * d * sizeof(double));
    double *VA = (double *)malloc((size_t)n * d * sizeof(double));
    double *dVA = (double *)malloc((size_t)n * d * sizeof(double));
    double *dA_keys = (double *)malloc((size_t)n * d * sizeof(double));
    double *dA_queries = (double *)malloc((size_t)n * d * sizeof(double));
    if (dB1) memset(dB1, 0, (size_t)heads * n * N * sizeof(double));
    if (dB2) memset(dB2, 0, (size_t)heads * N * n * sizeof(double));
    if (ddwc_w) memset(ddwc_w, 0, (size_t)heads * d * 9 * sizeof(double));
    if (ddwc_b) memset(ddwc_b, 0, (size_t)heads * d * sizeof(double));
    for (int u = 0; u < units; ++u) {
        const int hd = u % heads;
        const size_t off = (size_t)u * N * d;
        const double *Qu = Q + off, *Ku = K + off, *Vu = V + off, *gu = g + off;
        const double *B1h = B1 ? B1 + (size_t)hd * n * N : NULL;
        const double *B2h = B2 ? B2 + (size_t)hd * N * n : NULL;
        if (A_in)
            memcpy(A, A_in + (size_t)u * n * d, (size_t)n * d * sizeof(double));
        else
            oracle_pool(Qu, 1, gh, gw, ah, aw, d, A);
        oracle_softmax_attention(A, Ku, Vu, B1h, scale1, n, N, d, d, VA, NULL);
        /* broadcast stage: queries Q, keys A, values VA */
        oracle_softmax_attention_bwd(Qu, A, VA, B2h, scale2, N, n, d, d, gu,
                                     dQ + off, dA_keys, dVA,
                                     dB2 ? dB2 + (size_t)hd * N * n : NULL);
        /* aggregation stage: queries A, keys K, values V, upstream dVA */
        oracle_softmax_attention_bwd(A, Ku, Vu, B1h, scale1, n, N, d, d, dVA,
                                     dA_queries, dK + off, dV + off,
                                     dB1 ? dB1 + (size_t)hd * n * N : NULL);
        for (size_t e = 0; e < (size_t)n * d; ++e) dA_keys[e] += dA_queries[e];
        if (A_in) {
            if (dA_out)
                memcpy(dA_out + (size_t)u * n * d, dA_keys, (size_t)n * d * sizeof(double));
        } else {
            oracle_pool_bwd(dA_keys, gh, gw, ah, aw, d, dQ + off);
        }
        if (dwc_w)
            oracle_dwc_bwd(Vu, dwc_w + (size_t)hd * d * 9, gu, gh, gw, d, dV + off,
                           ddwc_w ? ddwc_w + (size_t)hd * d * 9 : NULL,
                           ddwc_b ? ddwc_b + (size_t)hd * d : NULL);
        if (vk != 0.0)
            for (size_t e = 0; e < (size_t)N * d; ++e) dV[off + e] += vk * gu[e];
    }
    free(A);
    free(VA);
    free(dVA);
    free(dA_keys);
    free(dA_queries);
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
