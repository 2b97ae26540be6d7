/*
 * CPU oracle for multi-step verification through a selective state-space layer.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, fp64 definition of
 * what the GPU library must compute.  It shares no code with the HIP path and
 * may be built, linked or called only by the test-suite, the smoke check and
 * the bench's cpu_baseline leg.
 *
 * What it follows in the paper (arXiv 2408.15237):
 *   - Section 2.1, Eq. 1: the linear-RNN step  h_t = A_t h_{t-1} + B_t x_t,
 *     y_t = C_t^T h_t, with a matrix-valued hidden state.
 *   - Section 2.2: A is diagonal and the discrete parameters are rebuilt every
 *     step from a sampling interval Delta_t.  The paper names the Discretize
 *     function without printing it; the reading used here is the Mamba one,
 *     A_bar = exp(Delta*A) and B_bar = Delta*B, plus the skip term D*x.
 *   - Section 4.2, MultiStep / Algorithm 2 (Verify): from one cached state run
 *     the tokens one after the other; the caller picks the state after the
 *     accepted prefix.  The oracle is eager: it returns the state after every
 *     token, so picking is plain indexing.
 *   - Section 4.3, footnote on the convolution: the conv part of the block sees
 *     the committed raw inputs followed by the new ones; here that is a causal
 *     depthwise cross-correlation of width W over that concatenated sequence.
 *
 * Parity pins (tests/test_oracle_*.py): closed form for scalar A, constant-input
 * geometric series, the linear-attention special case (A=0, Delta=1), the
 * library conv1d, brute force on tiny inputs, and the k-step / from-cache /
 * rollback invariants.  No absolute value printed in the paper exists for this
 * kernel, so a comparison against the paper's own numbers is "parity unpinned".
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { SSMO_F32 = 0, SSMO_BF16 = 1 };
enum { SSMO_A_SCALAR = 0, SSMO_A_DIAG = 1 };
enum { SSMO_ACT_NONE = 0, SSMO_ACT_SILU = 1 };

int ssmo_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Round a double to the nearest bfloat16 value (8 significant bits, fp32
 * exponent range), ties to even, in ONE rounding step. */
double ssmo_round_bf16(double x)
{
    if (x == 0.0 || isnan(x) || isinf(x)) return x;
    int e;
    double m = frexp(x, &e);              /* x = m * 2^e, 0.5 <= |m| < 1 */
    double r;
    if (e - 1 < -126) {
        /* subnormal range of the format: fixed quantum 2^-133 */
        r = ldexp(rint(ldexp(x, 133)), -133);
    } else {
        r = ldexp(rint(ldexp(m, 8)), e - 8);   /* rint: current mode = nearest-even */
    }
    if (fabs(r) > 3.3895313892515355e38) r = copysign(INFINITY, x);   /* above bf16 max */
    return r;
}

double ssmo_round_f32(double x) { return (double)(float)x; }

static double round_io(double x, int io_dtype)
{
    return io_dtype == SSMO_BF16 ? ssmo_round_bf16(x) : ssmo_round_f32(x);
}

void ssmo_round_array(const double *in, double *out, size_t n, int io_dtype)
{
    for (size_t i = 0; i < n; ++i) out[i] = round_io(in[i], io_dtype);
}

/*
 * Causal depthwise convolution (Section 4.3 footnote; cross-correlation with
 * the last tap on the newest token).
 *   raw  [batch][W-1+k][Cx] : the last W-1 committed raw inputs (oldest first)
 *                             followed by the k new tokens
 *   wgt  [Cx][W], bias [Cx] or NULL
 *   xc   [batch][k][Cx]     : act(bias + sum_w wgt[c][w] * raw[t+w][c]), then
 *                             rounded to the I/O storage type (it is an
 *                             activation tensor that the layer stores)
 */
void ssmo_conv(int batch, int k, int Cx, int W, const double *raw, const double *wgt,
               const double *bias, int act, int io_dtype, double *xc)
{
    const int L = W - 1 + k;
    for (int b = 0; b < batch; ++b)
        for (int t = 0; t < k; ++t)
            for (int c = 0; c < Cx; ++c) {
                double s = bias ? bias[c] : 0.0;
                for (int w = 0; w < W; ++w)
                    s += wgt[(size_t)c * W + w] * raw[((size_t)b * L + (t + w)) * Cx + c];
                if (act == SSMO_ACT_SILU) s = s / (1.0 + exp(-s));
                xc[((size_t)b * k + t) * Cx + c] = round_io(s, io_dtype);
            }
}

/*
 * Token-by-token recurrence from a given state (Eq. 1 with the discretization
 * above), keeping the state after every token.
 *   h_in   [batch][H][P][N]
 *   x      [batch][k][H*P]      dt [batch][k][H]
 *   Bm, Cm [batch][k][G][N]     head hd uses group hd*G/H
 *   A      [H] (scalar mode) or [H][N] (diag mode);  D [H]
 *   y      [batch][k][H*P]      (not rounded)
 *   h_snap [k+1][batch][H][P][N]: h_snap[0] = h_in, h_snap[t+1] = state after token t
 */
void ssmo_scan(int a_mode, int batch, int H, int P, int N, int G, int k,
               const double *h_in, const double *x, const double *dt,
               const double *Bm, const double *Cm, const double *A, const double *D,
               double *y, double *h_snap)
{
    const size_t S = (size_t)H * P * N;          /* state elements per sequence */
    const size_t SB = S * (size_t)batch;         /* per snapshot */
    memcpy(h_snap, h_in, SB * sizeof(double));
#pragma omp parallel for collapse(2) schedule(static)
    for (int b = 0; b < batch; ++b)
        for (int hd = 0; hd < H; ++hd) {
            const int g = (int)(((long)hd * G) / H);
            for (int t = 0; t < k; ++t) {
                const double dt_t = dt[((size_t)b * k + t) * H + hd];
                const double *Bt = Bm + (((size_t)b * k + t) * G + g) * N;
                const double *Ct = Cm + (((size_t)b * k + t) * G + g) * N;
                const double *hp = h_snap + (size_t)t * SB + (size_t)b * S + (size_t)hd * P * N;
                double *hn = h_snap + (size_t)(t + 1) * SB + (size_t)b * S + (size_t)hd * P * N;
                for (int p = 0; p < P; ++p) {
                    const double x_t = x[((size_t)b * k + t) * ((size_t)H * P) + (size_t)hd * P + p];
                    double acc = 0.0;
                    for (int n = 0; n < N; ++n) {
                        const double a_coef = (a_mode == SSMO_A_DIAG) ? A[(size_t)hd * N + n] : A[hd];
                        const double decay = exp(dt_t * a_coef);
                        const double h_new = decay * hp[(size_t)p * N + n] + dt_t * Bt[n] * x_t;
                        hn[(size_t)p * N + n] = h_new;
                        acc += Ct[n] * h_new;
                    }
                    y[((size_t)b * k + t) * ((size_t)H * P) + (size_t)hd * P + p] = acc + D[hd] * x_t;
                }
            }
        }
}
