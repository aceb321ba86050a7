/*
 * Plain C oracle of the DEF / DEF-A compression-and-update step with RBGS.
 *
 * TEST INFRASTRUCTURE ONLY.  Scalar loops, no blocking, no fusion beyond what
 * the update rules state; it exists so that full-size parity checks and the
 * CPU baseline do not take minutes.  It shares no code with the HIP library.
 *
 * Follows arXiv 2004.05298: Algorithm 1 (error feedback p = eta*g + e, residual
 * e <- p - C(p), average of the compressed vectors, x <- x - C(p)); Sec. 3.2
 * "Momentum Variant" (m <- mu*m + g, p = eta*m + e); Algorithm 1 "Output"
 * (y = x - mean_k e_k); Sec. 1 for the compressor (one contiguous block of the
 * flat vector, here with circular wrap, start index supplied by the caller).
 *
 * Arithmetic: IEEE binary32, one rounding per multiply and per add.  Build with
 * -ffp-contract=off so the compiler never fuses a multiply with an add.
 *
 * The only concession to speed is an OpenMP "parallel for" over the parameter
 * index; each index is independent, so the result does not depend on threads.
 */
#include <stddef.h>
#include <stdint.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int def_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void def_oracle_set_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* 1 if global index i lies in the circular block of length B starting at s. */
static int kept(int64_t i, int64_t s, int64_t B, int64_t d)
{
    int64_t j = i - s;
    if (j < 0) j += d;
    return j < B;
}

/*
 * One iteration.
 *   x      [n]        parameters for the n columns held (updated in place)
 *   e, m   [W][n]     error memory and momentum buffer, row stride n (in place)
 *   g      [W][ldg]   gradients, row stride ldg >= n
 *   index  [n] or NULL  global index of each column (NULL: column c is index c)
 *   cbar   [n]        out: dense averaged compressed vector C(p_t) (zero off-block)
 * mu == 0 leaves m untouched (Algorithm 1 as printed; m may be NULL); wd == 0 skips the
 * decay term.  Workers are visited in order k = 0..W-1 as in Algorithm 1; the sum of the
 * compressed vectors is accumulated in that order.
 */
void def_oracle_step_f32(int64_t n, int64_t d, int32_t W, int64_t B, int64_t s,
                         float lr, float mu, float wd,
                         float *x, float *e, float *m,
                         const float *g, int64_t ldg,
                         const int64_t *index, float *cbar)
{
    int64_t c;
    int32_t k;
    /* running sum of the compressed vectors starts at +0 */
#pragma omp parallel for schedule(static)
    for (c = 0; c < n; ++c) cbar[c] = 0.0f;

    /* every worker k: momentum, error feedback, compress, residual */
    for (k = 0; k < W; ++k) {
        const float *gk_row = g + (size_t)k * (size_t)ldg;
        float *ek = e + (size_t)k * (size_t)n;
        float *mk_row = m ? m + (size_t)k * (size_t)n : NULL;
#pragma omp parallel for schedule(static)
        for (c = 0; c < n; ++c) {
            const int64_t i = index ? index[c] : c;
            float gk = gk_row[c];
            float mk, p, cp;
            if (wd != 0.0f) {
                float decay = wd * x[c];            /* x is still x_t here */
                gk = gk + decay;
            }
            if (mu != 0.0f) {
                float carried = mu * mk_row[c];
                mk = carried + gk;                  /* m_{k,t+1} = mu*m_{k,t} + g_{k,t} */
                mk_row[c] = mk;
            } else {
                mk = gk;
            }
            {
                float step = lr * mk;
                p = step + ek[c];                   /* p_{k,t} = eta*m_{k,t+1} + e_{k,t} */
            }
            if (kept(i, s, B, d)) {
                cp = p;                             /* C(p_k) keeps the block ...        */
                ek[c] = 0.0f;                       /* ... and the residual there is +0  */
            } else {
                cp = 0.0f;
                ek[c] = p;                          /* e_{k,t+1} = p_k - C(p_k)          */
            }
            cbar[c] = cbar[c] + cp;                 /* sum over workers, k ascending     */
        }
    }

    /* average, then x_{t+1} = x_t - C(p_t) */
#pragma omp parallel for schedule(static)
    for (c = 0; c < n; ++c) {
        cbar[c] = cbar[c] / (float)W;
        x[c] = x[c] - cbar[c];
    }
}

/* w_k = x - lambda*e_k for every worker (Algorithm 1, "detach" line); w is [W][n]. */
void def_oracle_detach_f32(int64_t n, int32_t W, float lambda, const float *x, const float *e,
                           float *w)
{
    int32_t k;
    for (k = 0; k < W; ++k) {
        int64_t c;
#pragma omp parallel for schedule(static)
        for (c = 0; c < n; ++c) {
            float scaled = lambda * e[(size_t)k * (size_t)n + (size_t)c];
            w[(size_t)k * (size_t)n + (size_t)c] = x[c] - scaled;
        }
    }
}

/* y = x - (sum_k e_k) / W, k ascending. */
void def_oracle_y_f32(int64_t n, int32_t W, const float *x, const float *e, float *y)
{
    int64_t c;
#pragma omp parallel for schedule(static)
    for (c = 0; c < n; ++c) {
        float acc = 0.0f;
        int32_t k;
        for (k = 0; k < W; ++k) acc = acc + e[(size_t)k * (size_t)n + (size_t)c];
        y[c] = x[c] - acc / (float)W;
    }
}
