/*
 * xconv_oracle.c -- CPU oracle for the XConv weight-gradient path.
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It is a plain, slow, obviously-correct
 * implementation used to check the GPU library and as the timed CPU baseline.
 * Nothing in the product path may call it.  It shares no code with the HIP
 * kernels: every loop below is written out from the paper's definitions.
 *
 * What it computes (notation of the paper; n = input channel, m = output
 * channel, i = kernel offset, j = probing vector):
 *
 *   exact gradient      dw_i^{n,m} = tr( X^n (dY^m)^T T_{-k(i)} )        Sec. 3, Eq. (2), Eq. (5)
 *   trace estimator     tr(A) ~ (1/r) sum_j z_j^T A z_j, E[z z^T] = I    Sec. 3, Eq. (3)
 *   multi-channel est.  G^{m,n} = (1/r) sum_j z_{n,j}^T (A z_j)_m        Sec. 3, Eq. (6)
 *   block-sparse probes z_{n,j} = 0 with probability 1 - p, scaled by      Sec. 3, Eq. (7), Eq. (8)
 *                       1/nnz(Z_n) instead of 1/r
 *   Algorithm 1         fwd: Xbar = Z[s]^T X, keep (Xbar, s)
 *                       bwd: L = Xbar dY^T,  dw_i = (1/r) tr(L T_{-k(i)} Z[s])
 *
 * Readings taken where the paper is silent (all listed in the design notes):
 *   - the probe acts on the channel axis only: Z is [C_in, r] and the paper's
 *     stacked probe is Z (x) I_N (Kronecker with the pixel identity).  With that
 *     structure Eq. (6) step (i) becomes Xt[b,j,y,x] = sum_n Z[n,j] X[b,n,y,x],
 *     step (ii)/(iii) become the offset-wise correlation of dY with Xt followed
 *     by the left multiplication with Z/r;
 *   - the shift T_k is realised as a zero-padded, strided index offset
 *     (cross-correlation, no kernel flip), not a circular shift;
 *   - dw is laid out [C_out, C_in, kH, kW];
 *   - entries of Z have unit variance and the 1/r factor is applied once at
 *     the end (Eq. (3));
 *   - Xt is rounded once to the storage type (fp32 / bf16 / fp16, round to
 *     nearest even) because it is what Algorithm 1 "computes and saves".
 *
 * All sums are accumulated in double.  Inputs are float arrays holding values
 * that are already exactly representable in the storage type.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------------ */
/* Random probing vectors (Algorithm 1: "draw a seed s and Z[s]", "redraw    */
/* Z[s] from s").  The generator is SplitMix64 (Steele, Lea, Flood 2014):    */
/* state += gamma; output = finalizer(state).  Because the state advances by */
/* a constant it is counter based: the n-th output (1-based) from state s0   */
/* is fin(s0 + n*gamma).                                                     */
/* ------------------------------------------------------------------------ */
#define XO_GAMMA 0x9E3779B97F4A7C15ull

static uint64_t xo_fin(uint64_t z)
{
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

/* One step of the SplitMix64 stream: advances *state, returns the output. */
uint64_t xo_splitmix64(uint64_t *state)
{
    *state += XO_GAMMA;
    return xo_fin(*state);
}

/* Word number `ctr` (0-based) of the stream that belongs to `seed`.  The
 * stream's initial state is the first SplitMix64 output of `seed`, so that
 * nearby seeds do not give shifted copies of one stream. */
uint64_t xo_stream_word(uint64_t seed, uint64_t ctr)
{
    uint64_t key = xo_fin(seed + XO_GAMMA);
    return xo_fin(key + XO_GAMMA * (ctr + 1));
}

/* dist 0: Rademacher (+1/-1 with probability 1/2 each): entry number
 *         i = c*r+j takes bit i mod 64 of word i div 64 of the stream, a set
 *         bit meaning -1 (the 64 bits of a SplitMix64 output are
 *         independent fair bits, so one word serves 64 entries);
 * dist 1: standard normal by the Box-Muller transform on two 53-bit uniforms
 *         (words 2(c*r+j) and 2(c*r+j)+1), evaluated in double and rounded
 *         to float.
 * Both have E[z z^T] = I per column, the one property Eq. (3) needs.
 * Z is [C_in, r] row-major.  Returns 0, or -1 for an unknown dist. */
int xo_probe_matrix(int dist, uint64_t seed, int C_in, int r, float *Z)
{
    for (int c = 0; c < C_in; ++c) {
        for (int j = 0; j < r; ++j) {
            uint64_t idx = (uint64_t)c * (uint64_t)r + (uint64_t)j;
            if (dist == 0) {
                uint64_t word = xo_stream_word(seed, idx / 64);
                Z[idx] = ((word >> (idx % 64)) & 1u) ? -1.0f : 1.0f;
            } else if (dist == 1) {
                uint64_t h1 = xo_stream_word(seed, 2 * idx);
                uint64_t h2 = xo_stream_word(seed, 2 * idx + 1);
                double u1 = ((double)(h1 >> 11) + 1.0) * 0x1.0p-53; /* (0,1] */
                double u2 = (double)(h2 >> 11) * 0x1.0p-53;         /* [0,1) */
                double g = sqrt(-2.0 * log(u1)) * cos(6.283185307179586476925 * u2);
                Z[idx] = (float)g;
            } else {
                return -1;
            }
        }
    }
    return 0;
}

/* Block-sparse probing vectors (Sec. 3, Eq. (7), restricted to the channel
 * axis like the dense probe): entry (n, j) keeps its dense value with
 * probability p and is zero otherwise, independently for every (n, j).  The
 * paper allows a probability p_n per block; one p for all blocks is taken
 * here, p = keep_q15 / 32768 with keep_q15 in 1..32767 (0 means dense).  The
 * keep decision of entry idx = n*r+j is (u < keep_q15) with u the top 15 bits
 * of word idx of the stream of (seed xor XO_MASK_STREAM), a stream of its own
 * so that the kept entries equal those of the dense matrix of the same seed. */
#define XO_MASK_STREAM 0x5851F42D4C957F2Dull

int xo_probe_matrix_sparse(int dist, uint64_t seed, int keep_q15, int C_in, int r, float *Z)
{
    int rc = xo_probe_matrix(dist, seed, C_in, r, Z);
    if (rc != 0 || keep_q15 == 0) return rc;
    for (int c = 0; c < C_in; ++c)
        for (int j = 0; j < r; ++j) {
            uint64_t idx = (uint64_t)c * (uint64_t)r + (uint64_t)j;
            uint64_t u = xo_stream_word(seed ^ XO_MASK_STREAM, idx) >> 49;
            if (u >= (uint64_t)keep_q15) Z[idx] = 0.0f;
        }
    return 0;
}

/* ------------------------------------------------------------------------ */
/* Rounding to the storage type, round-to-nearest-even, with gradual         */
/* underflow and overflow to infinity.  dtype: 0 fp32, 1 bf16, 2 fp16.       */
/* ------------------------------------------------------------------------ */
static double xo_round_format(double v, int mant_bits /* explicit */, int emin, int emax)
{
    if (v == 0.0 || isnan(v) || isinf(v)) return v;
    int e;
    (void)frexp(v, &e);          /* |v| = f * 2^e, f in [0.5, 1) */
    e -= 1;                      /* |v| = f' * 2^e, f' in [1, 2)  */
    if (e < emin) e = emin;      /* subnormal range: fixed quantum */
    double q = ldexp(1.0, e - mant_bits);   /* spacing of the format at v */
    double rounded = nearbyint(v / q) * q;  /* default mode: ties to even */
    double maxv = ldexp(2.0 - ldexp(1.0, -mant_bits), emax);
    if (fabs(rounded) > maxv) return v > 0 ? INFINITY : -INFINITY;
    return rounded;
}

double xo_round_storage(double v, int dtype)
{
    if (dtype == 0) return (double)(float)v;
    if (dtype == 1) return xo_round_format(v, 7, -126, 127);
    if (dtype == 2) return xo_round_format(v, 10, -14, 15);
    return NAN;
}

/* ------------------------------------------------------------------------ */
/* Output extent of the layer: H' = floor((H + 2p - k)/stride) + 1.          */
/* ------------------------------------------------------------------------ */
static int xo_out_extent(int in, int k, int stride, int pad)
{
    int span = in + 2 * pad - k;
    if (span < 0) return 0;
    return span / stride + 1;
}

/* ------------------------------------------------------------------------ */
/* Algorithm 1, forward step 3 / Eq. (6) step (i) restricted to channels:    */
/*   Xt[b,j,y,x] = sum_n Z[n,j] * X[b,n,y,x], then rounded to storage type.  */
/* X  [B,C_in,H,W], Z [C_in,r], Xt [B,r,H,W].                                */
/* ------------------------------------------------------------------------ */
void xo_probe_fwd(const float *X, const float *Z, float *Xt,
                  int B, int C_in, int H, int W, int r, int dtype)
{
    size_t HW = (size_t)H * W;
    double *acc = (double *)malloc(HW * sizeof(double));
    for (int b = 0; b < B; ++b) {
        for (int j = 0; j < r; ++j) {
            for (size_t p = 0; p < HW; ++p) acc[p] = 0.0;
            for (int n = 0; n < C_in; ++n) {
                double z = (double)Z[(size_t)n * r + j];
                const float *xp = X + ((size_t)b * C_in + n) * HW;
                for (size_t p = 0; p < HW; ++p) acc[p] += z * (double)xp[p];
            }
            float *out = Xt + ((size_t)b * r + j) * HW;
            for (size_t p = 0; p < HW; ++p) out[p] = (float)xo_round_storage(acc[p], dtype);
        }
    }
    free(acc);
}

/* ------------------------------------------------------------------------ */
/* Correlation of a residual with an activation-like tensor at every kernel  */
/* offset, summed over batch and output pixels:                              */
/*   G[m,q,ky,kx] = sum_{b,oy,ox} dY[b,m,oy,ox] * A[b,q,oy*sh+ky-ph, ox*sw+kx-pw]
 * with taps outside the image skipped (zero padding).                       */
/* With A = X (Q = C_in) this is the exact gradient of Eq. (2)/(5): the trace */
/* tr(X^n (dY^m)^T T_{-k(i)}) pairs output pixel p of dY with input pixel     */
/* p + k(i) of X.  With A = Xt (Q = r) it is Algorithm 1 backward step 3      */
/* (L = Xbar dY^T) combined with the shift of step 4.                         */
/* dY [B,C_out,Ho,Wo], A [B,Q,H,W], G [C_out,Q,kH,kW] (double).               */
/* ------------------------------------------------------------------------ */
void xo_correlate(const float *dY, const float *A, double *G,
                  int B, int C_out, int Q, int H, int W,
                  int kH, int kW, int sh, int sw, int ph, int pw)
{
    int Ho = xo_out_extent(H, kH, sh, ph);
    int Wo = xo_out_extent(W, kW, sw, pw);
    size_t nG = (size_t)C_out * Q * kH * kW;
    for (size_t i = 0; i < nG; ++i) G[i] = 0.0;
    for (int m = 0; m < C_out; ++m)
      for (int q = 0; q < Q; ++q)
        for (int ky = 0; ky < kH; ++ky)
          for (int kx = 0; kx < kW; ++kx) {
              double s = 0.0;
              for (int b = 0; b < B; ++b) {
                  const float *dy = dY + ((size_t)b * C_out + m) * Ho * Wo;
                  const float *a  = A  + ((size_t)b * Q + q) * H * W;
                  for (int oy = 0; oy < Ho; ++oy) {
                      int iy = oy * sh + ky - ph;
                      if (iy < 0 || iy >= H) continue;
                      for (int ox = 0; ox < Wo; ++ox) {
                          int ix = ox * sw + kx - pw;
                          if (ix < 0 || ix >= W) continue;
                          s += (double)dy[(size_t)oy * Wo + ox] * (double)a[(size_t)iy * W + ix];
                      }
                  }
              }
              G[(((size_t)m * Q + q) * kH + ky) * kW + kx] = s;
          }
}

/* Exact weight gradient, Eq. (2) / Eq. (5).  dW [C_out,C_in,kH,kW]. */
void xo_dw_exact(const float *dY, const float *X, double *dW,
                 int B, int C_in, int C_out, int H, int W,
                 int kH, int kW, int sh, int sw, int ph, int pw)
{
    xo_correlate(dY, X, dW, B, C_out, C_in, H, W, kH, kW, sh, sw, ph, pw);
}

/* ------------------------------------------------------------------------ */
/* Algorithm 1 backward step 4 / Eq. (6) step (iii): probe from the left and */
/* normalise,  dW[m,n,ky,kx] = (1/r) sum_j Z[n,j] * G[m,j,ky,kx].            */
/* ------------------------------------------------------------------------ */
void xo_expand(const double *G, const float *Z, double *dW,
               int C_out, int C_in, int r, int kH, int kW)
{
    int K2 = kH * kW;
    for (int m = 0; m < C_out; ++m)
      for (int n = 0; n < C_in; ++n)
        for (int o = 0; o < K2; ++o) {
            double s = 0.0;
            for (int j = 0; j < r; ++j)
                s += (double)Z[(size_t)n * r + j] * G[((size_t)m * r + j) * K2 + o];
            dW[((size_t)m * C_in + n) * K2 + o] = s / (double)r;
        }
}

/* The same with the scaling of Eq. (8) for block-sparse probing vectors:     */
/*   dW[m,n,ky,kx] = (1/nnz(Z_n)) sum_j Z[n,j] * G[m,j,ky,kx],               */
/* nnz(Z_n) = number of non-zero entries of row n of Z.  A row without any   */
/* (the estimator has nothing to go on for that input channel) gives zeros.  */
void xo_expand_nnz(const double *G, const float *Z, double *dW,
                   int C_out, int C_in, int r, int kH, int kW)
{
    int K2 = kH * kW;
    for (int n = 0; n < C_in; ++n) {
        int nnz = 0;
        for (int j = 0; j < r; ++j)
            if (Z[(size_t)n * r + j] != 0.0f) ++nnz;
        for (int m = 0; m < C_out; ++m)
            for (int o = 0; o < K2; ++o) {
                double s = 0.0;
                for (int j = 0; j < r; ++j)
                    s += (double)Z[(size_t)n * r + j] * G[((size_t)m * r + j) * K2 + o];
                dW[((size_t)m * C_in + n) * K2 + o] = nnz > 0 ? s / (double)nnz : 0.0;
            }
    }
}

/* Backward pass of Algorithm 1 from the stored Xt: steps 3 and 4. */
void xo_dw_from_xt(const float *dY, const float *Xt, const float *Z, double *dW,
                   int B, int C_in, int C_out, int H, int W, int r,
                   int kH, int kW, int sh, int sw, int ph, int pw)
{
    double *G = (double *)malloc((size_t)C_out * r * kH * kW * sizeof(double));
    xo_correlate(dY, Xt, G, B, C_out, r, H, W, kH, kW, sh, sw, ph, pw);
    xo_expand(G, Z, dW, C_out, C_in, r, kH, kW);
    free(G);
}

/* Whole estimator: forward probe (with storage rounding) then backward. */
void xo_dw_estimate(const float *dY, const float *X, const float *Z, double *dW,
                    int B, int C_in, int C_out, int H, int W, int r,
                    int kH, int kW, int sh, int sw, int ph, int pw, int dtype)
{
    float *Xt = (float *)malloc((size_t)B * r * H * W * sizeof(float));
    xo_probe_fwd(X, Z, Xt, B, C_in, H, W, r, dtype);
    xo_dw_from_xt(dY, Xt, Z, dW, B, C_in, C_out, H, W, r, kH, kW, sh, sw, ph, pw);
    free(Xt);
}

/* ------------------------------------------------------------------------- */
/* Volumetric layers: the same definitions with one more spatial axis (the    */
/* paper's implementations cover 2-D and 3-D convolutions; the shift T_{k(i)} */
/* of Eq. (1), (2) then runs over kD*kH*kW offsets).                           */
/*   G[m,q,kz,ky,kx] = sum_{b,oz,oy,ox} dY[b,m,oz,oy,ox]                        */
/*                        * A[b,q,oz*sd+kz-pd, oy*sh+ky-ph, ox*sw+kx-pw]        */
/* dY: [B,C_out,D',H',W'], A: [B,Q,D,H,W], G: [C_out,Q,kD,kH,kW] (double).      */
/* With A = X (Q = C_in) this is the exact gradient, Eq. (2)/(5).              */
/* ------------------------------------------------------------------------- */
void xo_correlate3d(const float *dY, const float *A, double *G,
                    int B, int C_out, int Q, int D, int H, int W,
                    int kD, int kH, int kW, int sd, int sh, int sw, int pd, int ph, int pw)
{
    int Do = xo_out_extent(D, kD, sd, pd);
    int Ho = xo_out_extent(H, kH, sh, ph);
    int Wo = xo_out_extent(W, kW, sw, pw);
    for (int m = 0; m < C_out; ++m)
      for (int q = 0; q < Q; ++q)
        for (int kz = 0; kz < kD; ++kz)
          for (int ky = 0; ky < kH; ++ky)
            for (int kx = 0; kx < kW; ++kx) {
                double s = 0.0;
                for (int b = 0; b < B; ++b)
                  for (int oz = 0; oz < Do; ++oz) {
                      int iz = oz * sd + kz - pd;
                      if (iz < 0 || iz >= D) continue;
                      for (int oy = 0; oy < Ho; ++oy) {
                          int iy = oy * sh + ky - ph;
                          if (iy < 0 || iy >= H) continue;
                          for (int ox = 0; ox < Wo; ++ox) {
                              int ix = ox * sw + kx - pw;
                              if (ix < 0 || ix >= W) continue;
                              double g = dY[((((size_t)b * C_out + m) * Do + oz) * Ho + oy) * Wo + ox];
                              double a = A[((((size_t)b * Q + q) * D + iz) * H + iy) * W + ix];
                              s += g * a;
                          }
                      }
                  }
                G[((((size_t)m * Q + q) * kD + kz) * kH + ky) * kW + kx] = s;
            }
}

/* Entries idx[i] = (m, q, kz, ky, kx) of xo_correlate3d's result, one at a time (for layers too */
/* large to correlate in full on one thread).                                                  */
void xo_correlate3d_at(const float *dY, const float *A, const int *idx, int n, double *out,
                       int B, int C_out, int Q, int D, int H, int W,
                       int kD, int kH, int kW, int sd, int sh, int sw, int pd, int ph, int pw)
{
    int Do = xo_out_extent(D, kD, sd, pd);
    int Ho = xo_out_extent(H, kH, sh, ph);
    int Wo = xo_out_extent(W, kW, sw, pw);
    (void)kD; (void)kH; (void)kW;
    for (int i = 0; i < n; ++i) {
        int m = idx[5 * i], q = idx[5 * i + 1], kz = idx[5 * i + 2], ky = idx[5 * i + 3], kx = idx[5 * i + 4];
        double s = 0.0;
        for (int b = 0; b < B; ++b)
          for (int oz = 0; oz < Do; ++oz) {
              int iz = oz * sd + kz - pd;
              if (iz < 0 || iz >= D) continue;
              for (int oy = 0; oy < Ho; ++oy) {
                  int iy = oy * sh + ky - ph;
                  if (iy < 0 || iy >= H) continue;
                  for (int ox = 0; ox < Wo; ++ox) {
                      int ix = ox * sw + kx - pw;
                      if (ix < 0 || ix >= W) continue;
                      s += (double)dY[((((size_t)b * C_out + m) * Do + oz) * Ho + oy) * Wo + ox] *
                           (double)A[((((size_t)b * Q + q) * D + iz) * H + iy) * W + ix];
                  }
              }
          }
        out[i] = s;
    }
}

/* Keep decisions of block-sparse probing vectors (Eq. (7)): keep[i] = 1 when the top 15 bits of word i of */
/* the mask stream of the seed are below keep_q15 (probability keep_q15 / 32768), else 0; all 1 for 0.     */
void xo_keep_mask(uint64_t seed, int keep_q15, size_t n, float *keep)
{
    for (size_t i = 0; i < n; ++i)
        keep[i] = (keep_q15 == 0 || (xo_stream_word(seed ^ XO_MASK_STREAM, (uint64_t)i) >> 49) < (uint64_t)keep_q15) ? 1.0f : 0.0f;
}

/* v[i] <- v[i] rounded to the storage type (round to nearest even), in place. */
void xo_round_array(float *v, size_t n, int dtype)
{
    for (size_t i = 0; i < n; ++i) v[i] = (float)xo_round_storage((double)v[i], dtype);
}

/* ------------------------------------------------------------------------- */
/* The estimator as the paper states it: probing vectors over the stacked     */
/* pixel x channel space (Sec. 3 multi-channel case, Eq. (6); Algorithm 1).    */
/* Z is [C_in*N, r] with row (n, q) = n*N + q (N = H*W pixels), entries in the */
/* storage type.  Algorithm 1 saves Xbar (and the seed) and nothing else, so   */
/* Xbar is the only rounded quantity: L is a transient of the backward pass    */
/* and stays in double, and the factor 1/r comes once, at the end of step 4.   */
/*   forward   Xbar[b,j] = sum_{n,q} Z[(n,q),j] X[b,n,q]   (saved, fp32)        */
/*   backward  L[j,m,p]  = sum_b Xbar[b,j] dY[b,m,p]             (bwd step 3)  */
/*             dw[m,n,ky,kx] = (1/r) sum_j sum_{oy,ox} L[j,m,oy,ox]             */
/*                                 * Z[(n, (oy*sh+ky-ph, ox*sw+kx-pw)), j]       */
/* which is dw_i = (1/r) tr(L T_{-k(i)} Z) (bwd step 4) with zero padding in   */
/* place of the circular shift.                                                 */
/* ------------------------------------------------------------------------- */
void xo_pixel_probe_fwd(const float *X, const float *Z, float *Xbar, int B, int C_in, int H, int W, int r)
{
    size_t K = (size_t)C_in * H * W;
    for (int b = 0; b < B; ++b)
        for (int j = 0; j < r; ++j) {
            double s = 0.0;
            for (size_t k = 0; k < K; ++k) s += (double)Z[k * r + j] * (double)X[(size_t)b * K + k];
            Xbar[(size_t)b * r + j] = (float)s;
        }
}

void xo_pixel_dw_estimate(const float *dY, const float *Xbar, const float *Z, double *dW,
                          int B, int C_in, int C_out, int H, int W, int r,
                          int kH, int kW, int sh, int sw, int ph, int pw)
{
    int Ho = xo_out_extent(H, kH, sh, ph);
    int Wo = xo_out_extent(W, kW, sw, pw);
    size_t P = (size_t)C_out * Ho * Wo, N = (size_t)H * W;
    double *L = (double *)malloc((size_t)r * P * sizeof(double));
    for (int j = 0; j < r; ++j)
        for (size_t p = 0; p < P; ++p) {
            double s = 0.0;
            for (int b = 0; b < B; ++b) s += (double)Xbar[(size_t)b * r + j] * (double)dY[(size_t)b * P + p];
            L[(size_t)j * P + p] = s;
        }
    for (int m = 0; m < C_out; ++m)
      for (int n = 0; n < C_in; ++n)
        for (int ky = 0; ky < kH; ++ky)
          for (int kx = 0; kx < kW; ++kx) {
              double s = 0.0;
              for (int j = 0; j < r; ++j)
                for (int oy = 0; oy < Ho; ++oy) {
                    int iy = oy * sh + ky - ph;
                    if (iy < 0 || iy >= H) continue;
                    for (int ox = 0; ox < Wo; ++ox) {
                        int ix = ox * sw + kx - pw;
                        if (ix < 0 || ix >= W) continue;
                        double l = L[(size_t)j * P + ((size_t)m * Ho + oy) * Wo + ox];
                        double z = Z[((size_t)n * N + (size_t)iy * W + ix) * r + j];
                        s += l * z;
                    }
                }
              dW[(((size_t)m * C_in + n) * kH + ky) * kW + kx] = s / (double)r;
          }
    free(L);
}

/* ------------------------------------------------------------------------ */
/* Selected entries of the estimate, for layers too large to do in full.     */
/* idx[4*t..4*t+3] = (m, n, ky, kx); out[t] = dW_est[m,n,ky,kx].             */
/* Same arithmetic as xo_correlate + xo_expand, restricted to what the       */
/* requested entry needs.                                                    */
/* ------------------------------------------------------------------------ */
void xo_dw_from_xt_at(const float *dY, const float *Xt, const float *Z,
                      const int32_t *idx, int n_idx, double *out,
                      int B, int C_in, int C_out, int H, int W, int r,
                      int kH, int kW, int sh, int sw, int ph, int pw)
{
    int Ho = xo_out_extent(H, kH, sh, ph);
    int Wo = xo_out_extent(W, kW, sw, pw);
    (void)C_in;
    for (int t = 0; t < n_idx; ++t) {
        int m = idx[4 * t], n = idx[4 * t + 1], ky = idx[4 * t + 2], kx = idx[4 * t + 3];
        double acc = 0.0;
        for (int j = 0; j < r; ++j) {
            double s = 0.0;
            for (int b = 0; b < B; ++b) {
                const float *dy = dY + ((size_t)b * C_out + m) * Ho * Wo;
                const float *a  = Xt + ((size_t)b * r + j) * H * W;
                for (int oy = 0; oy < Ho; ++oy) {
                    int iy = oy * sh + ky - ph;
                    if (iy < 0 || iy >= H) continue;
                    for (int ox = 0; ox < Wo; ++ox) {
                        int ix = ox * sw + kx - pw;
                        if (ix < 0 || ix >= W) continue;
                        s += (double)dy[(size_t)oy * Wo + ox] * (double)a[(size_t)iy * W + ix];
                    }
                }
            }
            acc += (double)Z[(size_t)n * r + j] * s;
        }
        out[t] = acc / (double)r;
    }
}

/* Selected entries of the exact gradient (Eq. (2)/(5)). */
void xo_dw_exact_at(const float *dY, const float *X,
                    const int32_t *idx, int n_idx, double *out,
                    int B, int C_in, int C_out, int H, int W,
                    int kH, int kW, int sh, int sw, int ph, int pw)
{
    int Ho = xo_out_extent(H, kH, sh, ph);
    int Wo = xo_out_extent(W, kW, sw, pw);
    for (int t = 0; t < n_idx; ++t) {
        int m = idx[4 * t], n = idx[4 * t + 1], ky = idx[4 * t + 2], kx = idx[4 * t + 3];
        double s = 0.0;
        for (int b = 0; b < B; ++b) {
            const float *dy = dY + ((size_t)b * C_out + m) * Ho * Wo;
            const float *a  = X  + ((size_t)b * C_in + n) * H * W;
            for (int oy = 0; oy < Ho; ++oy) {
                int iy = oy * sh + ky - ph;
                if (iy < 0 || iy >= H) continue;
                for (int ox = 0; ox < Wo; ++ox) {
                    int ix = ox * sw + kx - pw;
                    if (ix < 0 || ix >= W) continue;
                    s += (double)dy[(size_t)oy * Wo + ox] * (double)a[(size_t)iy * W + ix];
                }
            }
        }
        out[t] = s;
    }
}

/* ------------------------------------------------------------------------ */
/* Forward convolution, Eq. (1)/(5): Y^m = sum_n W^{n,m} X^n with             */
/* W^{n,m} = sum_i w_i^{n,m} T_{k(i)}.  Written as a scatter over input       */
/* pixels so that it does not share its loop structure with xo_correlate;     */
/* it exists only so that tests can pin the gradient through the adjoint      */
/* identity <dY, conv(X,w)> = <dW, w>.                                        */
/* X [B,C_in,H,W], Wt [C_out,C_in,kH,kW] (double), Y [B,C_out,Ho,Wo] (double) */
/* ------------------------------------------------------------------------ */
void xo_conv_fwd(const float *X, const double *Wt, double *Y,
                 int B, int C_in, int C_out, int H, int W,
                 int kH, int kW, int sh, int sw, int ph, int pw)
{
    int Ho = xo_out_extent(H, kH, sh, ph);
    int Wo = xo_out_extent(W, kW, sw, pw);
    size_t nY = (size_t)B * C_out * Ho * Wo;
    for (size_t i = 0; i < nY; ++i) Y[i] = 0.0;
    for (int b = 0; b < B; ++b)
      for (int n = 0; n < C_in; ++n)
        for (int iy = 0; iy < H; ++iy)
          for (int ix = 0; ix < W; ++ix) {
              double x = (double)X[(((size_t)b * C_in + n) * H + iy) * W + ix];
              if (x == 0.0) continue;
              for (int ky = 0; ky < kH; ++ky) {
                  int ty = iy + ph - ky;           /* oy*sh = iy + ph - ky */
                  if (ty < 0 || ty % sh != 0) continue;
                  int oy = ty / sh;
                  if (oy >= Ho) continue;
                  for (int kx = 0; kx < kW; ++kx) {
                      int tx = ix + pw - kx;
                      if (tx < 0 || tx % sw != 0) continue;
                      int ox = tx / sw;
                      if (ox >= Wo) continue;
                      for (int m = 0; m < C_out; ++m)
                          Y[(((size_t)b * C_out + m) * Ho + oy) * Wo + ox] +=
                              Wt[(((size_t)m * C_in + n) * kH + ky) * kW + kx] * x;
                  }
              }
          }
}

/* ------------------------------------------------------------------------ */
/* Input gradient of the layer (Sec. 2: standard backpropagation is kept for  */
/* everything but the weight gradient, so dX is the exact transposed          */
/* convolution):                                                              */
/*   dX[b,n,iy,ix] = sum_{m,ky,kx} dY[b,m,oy,ox] W[m,n,ky,kx]                 */
/* over the (oy, ox) with oy*sh + ky - ph = iy and ox*sw + kx - pw = ix.      */
/* Written as a gather over the outputs of every input pixel, so that it      */
/* shares no loop structure with xo_conv_fwd (a scatter over the inputs); the */
/* two are tied together by <dX, V> = <dY, conv(V, W)> in the tests.           */
/* dY [B,C_out,Ho,Wo], Wt [C_out,C_in,kH,kW] (double), dX [B,C_in,H,W] (double) */
/* ------------------------------------------------------------------------ */
void xo_dx(const float *dY, const double *Wt, double *dX,
           int B, int C_in, int C_out, int H, int W,
           int kH, int kW, int sh, int sw, int ph, int pw)
{
    int Ho = xo_out_extent(H, kH, sh, ph);
    int Wo = xo_out_extent(W, kW, sw, pw);
    for (int b = 0; b < B; ++b)
      for (int n = 0; n < C_in; ++n)
        for (int iy = 0; iy < H; ++iy)
          for (int ix = 0; ix < W; ++ix) {
              double s = 0.0;
              for (int ky = 0; ky < kH; ++ky) {
                  int ty = iy + ph - ky;
                  if (ty < 0 || ty % sh != 0 || ty / sh >= Ho) continue;
                  for (int kx = 0; kx < kW; ++kx) {
                      int tx = ix + pw - kx;
                      if (tx < 0 || tx % sw != 0 || tx / sw >= Wo) continue;
                      for (int m = 0; m < C_out; ++m)
                          s += (double)dY[(((size_t)b * C_out + m) * Ho + ty / sh) * Wo + tx / sw] *
                               Wt[(((size_t)m * C_in + n) * kH + ky) * kW + kx];
                  }
              }
              dX[(((size_t)b * C_in + n) * H + iy) * W + ix] = s;
          }
}

