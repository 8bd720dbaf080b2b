/*
 * fp64 CPU oracle for the locally bi-directional selective scan (LBMamba).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, sequential, obviously
 * correct statement of what the GPU library must compute.  It shares no code,
 * header, table or helper with the HIP path and must never be called from the
 * product path; only the tests, the smoke check and the benchmark's
 * cpu_baseline leg load it.
 *
 * What it follows (paper = arXiv 2506.15976):
 *   - discretisation:            Sec. 3.1, Eq. 3 and Algorithm 1 (softplus with
 *                                additive Delta parameter, A-bar, B-bar)
 *   - global forward recurrence: Sec. 3.1, Eq. 1-2
 *   - local backward recurrence: Sec. 3.2, Eq. 7: the state with its own input
 *                                term, restarted at the last step of each window
 *   - combination and output:    Sec. 3.2, Eq. 8: h = f + (h^b - B-bar x), the
 *                                input term counted once; gate: Algorithm 1 (SiLU(z))
 *   - global bi-directional scan (the comparison method): Sec. 3.1, Eq. 4-6
 *   - gradients: the paper gives no formulas (Appendix B reports only
 *     throughput); lbscan_ref_bwd is the reverse-mode derivative of the
 *     forward loop above, derived by hand in the comment at that function and
 *     pinned by finite differences in the tests.
 *
 * Readings taken where the paper is ambiguous:
 *   - Algorithm 1 runs the whole forward loop and then uses "h^f" inside the
 *     backward loop; Eq. 8 is per time step, so the per-step forward state
 *     f_t is used.
 *   - Eq. 7/8 print "B^f x_t" without the bar; Algorithm 1 uses B-bar, and the
 *     text says it is the same term as in Eq. 1, so B-bar_t x_t is meant.
 *   - windows are [kM, kM+M-1] in 0-based time (Eq. 7 counts tokens from 1 and
 *     restarts at t % M = 0; Algorithm 1 counts from 0 and restarts when
 *     (i+1) % M == 0); a ragged last window is an ordinary short window.
 *   - Eq. 4 and Eq. 7 print A-bar without a time index; the backward step
 *     multiplies by A-bar of the step it arrives at (as Algorithm 1 does), which
 *     makes the local backward scan the forward scan run right to left.
 *   - softplus(v) = v for v > 20 (relative effect < 3e-9), else log1p(exp(v)).
 *   - Algorithm 1 starts both states at zero.  The *_state entry points also
 *     accept a forward state h0 entering at the first step and return the
 *     forward state hT after the last one (what a caller needs to process a
 *     long sequence in chunks whose lengths are multiples of the window); the
 *     local backward state stays zero at every window end, as in Eq. 7.
 *
 * Layout (all host, fp64, dense, last index contiguous):
 *   x, delta, z, out, dout, dx, ddelta, dz : (batch, dim, seqlen)
 *   Bm, Cm, dBm, dCm                        : (batch, dstate, seqlen)
 *   A, dA                                   : (dim, dstate)
 *   Dskip, delta_bias, dDskip, ddelta_bias  : (dim)
 *   h0, hT, dh0, dhT                        : (batch, dim, dstate)
 *
 * Parity status: every function here is pinned by tests/test_oracle_pins.py
 * (brute-force sums, IIR-filter library routine, closed forms, impulse
 * responses, finite differences).  The paper prints no worked numerical
 * example, so there is no golden value from the paper itself.
 *
 * Parallelism: OpenMP over independent (batch, channel) rows only.
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct lbref_problem {
    int batch, dim, dstate, seqlen, window;
    int delta_softplus;
    const double *x;          /* (B,D,L) */
    const double *delta;      /* (B,D,L) raw: before bias and softplus */
    const double *A;          /* (D,N)   */
    const double *Bm;         /* (B,N,L) */
    const double *Cm;         /* (B,N,L) */
    const double *Dskip;      /* (D) or NULL => 0 */
    const double *z;          /* (B,D,L) or NULL => no gate */
    const double *delta_bias; /* (D) or NULL => 0 */
} lbref_problem;

static double softplus64(double v) { return v > 20.0 ? v : log1p(exp(v)); }
static double sigmoid64(double v) { return 1.0 / (1.0 + exp(-v)); }

/* Time step delta_t of one row (Eq. 3; Algorithm 1's Delta line). */
static void row_timestep(const lbref_problem *p, int d, const double *draw, double *dt)
{
    double bias = p->delta_bias ? p->delta_bias[d] : 0.0;
    for (int t = 0; t < p->seqlen; ++t) {
        double v = draw[t] + bias;
        dt[t] = p->delta_softplus ? softplus64(v) : v;
    }
}

int lbscan_ref_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void lbscan_ref_set_num_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

static int check_problem(const lbref_problem *p)
{
    if (!p || !p->x || !p->delta || !p->A || !p->Bm || !p->Cm) return -1;
    if (p->batch < 0 || p->dim < 0 || p->dstate < 0 || p->seqlen < 0) return -1;
    if (p->window < 1) return -1;
    return 0;
}

/*
 * Forward: out[b,d,t] = (sum_n Cm[b,n,t] (f_t + g_t) + Dskip[d] x_t) * SiLU(z_t)
 * with f the global forward state (Eq. 1) and g the local backward state
 * without the current input term (Eq. 7-8).
 */
int lbscan_ref_fwd_state(const lbref_problem *p, const double *h0, double *out, double *hT)
{
    if (check_problem(p) || !out) return -1;
    const int Bsz = p->batch, D = p->dim, N = p->dstate, L = p->seqlen, M = p->window;
    if ((long)Bsz * D * L == 0) {
        /* no steps: the state passes through */
        if (hT)
            for (long i = 0; i < (long)Bsz * D * N; ++i) hT[i] = h0 ? h0[i] : 0.0;
        return 0;
    }
    int fail = 0;
#pragma omp parallel for schedule(static)
    for (long row = 0; row < (long)Bsz * D; ++row) {
        const int b = (int)(row / D), d = (int)(row % D);
        const double *xr = p->x + row * L, *draw = p->delta + row * L;
        double *yr = out + row * L;
        double *dt = (double *)malloc(sizeof(double) * L);
        double *F = (double *)malloc(sizeof(double) * L);
        double *HB = (double *)malloc(sizeof(double) * L);
        if (!dt || !F || !HB) { fail = 1; free(dt); free(F); free(HB); continue; }
        row_timestep(p, d, draw, dt);
        const double Dd = p->Dskip ? p->Dskip[d] : 0.0;
        for (int t = 0; t < L; ++t) yr[t] = Dd * xr[t];
        for (int n = 0; n < N; ++n) {
            const double a = p->A[(long)d * N + n];
            const double *Bn = p->Bm + ((long)b * N + n) * L;
            const double *Cn = p->Cm + ((long)b * N + n) * L;
            /* global forward recurrence, Eq. 1 */
            double hf = h0 ? h0[row * N + n] : 0.0;
            for (int t = 0; t < L; ++t) {
                hf = exp(dt[t] * a) * hf + dt[t] * Bn[t] * xr[t];
                F[t] = hf;
            }
            if (hT) hT[row * N + n] = hf;
            /* local backward recurrence, Eq. 7: inside every window [kM, kM+M-1]
               (a ragged last window ends at L-1) the state with its own input
               term is  hb_t = u_t  at the window's last step and
               hb_t = abar_t hb_{t+1} + u_t  before it. */
            for (int t = L - 1; t >= 0; --t) {
                const double ut = dt[t] * Bn[t] * xr[t];
                const int last = ((t + 1) % M == 0) || (t == L - 1);
                HB[t] = last ? ut : exp(dt[t] * a) * HB[t + 1] + ut;
            }
            /* combination, Eq. 8: the input term sits in both states and is
               counted once, h_t = f_t + (hb_t - u_t);  y_t = C_t h_t (+ D x_t above) */
            for (int t = 0; t < L; ++t) {
                const double ut = dt[t] * Bn[t] * xr[t];
                yr[t] += Cn[t] * (F[t] + (HB[t] - ut));
            }
        }
        if (p->z) {
            const double *zr = p->z + row * L;
            for (int t = 0; t < L; ++t) yr[t] *= zr[t] * sigmoid64(zr[t]);
        }
        free(dt); free(F); free(HB);
    }
    return fail ? -2 : 0;
}

int lbscan_ref_fwd(const lbref_problem *p, double *out)
{
    return lbscan_ref_fwd_state(p, NULL, out, NULL);
}

/*
 * Global bi-directional scan of Eq. 4-6: a forward SSM with parameter set pf
 * plus an independent reverse-direction SSM with parameter set pb over the
 * whole sequence; each direction adds its own D x term (Eq. 2 and Eq. 5);
 * the sum is gated once with pf->z.  Window fields are ignored.
 */
int lbscan_ref_bidir_fwd(const lbref_problem *pf, const lbref_problem *pb, double *out)
{
    if (check_problem(pf) || check_problem(pb) || !out) return -1;
    if (pf->batch != pb->batch || pf->dim != pb->dim || pf->dstate != pb->dstate ||
        pf->seqlen != pb->seqlen) return -1;
    const int Bsz = pf->batch, D = pf->dim, N = pf->dstate, L = pf->seqlen;
    if ((long)Bsz * D * L == 0) return 0;
    int fail = 0;
#pragma omp parallel for schedule(static)
    for (long row = 0; row < (long)Bsz * D; ++row) {
        const int b = (int)(row / D), d = (int)(row % D);
        double *yr = out + row * L;
        double *dt = (double *)malloc(sizeof(double) * L);
        if (!dt) { fail = 1; continue; }
        for (int t = 0; t < L; ++t) yr[t] = 0.0;
        for (int dir = 0; dir < 2; ++dir) {
            const lbref_problem *p = dir == 0 ? pf : pb;
            const double *xr = p->x + row * L;
            row_timestep(p, d, p->delta + row * L, dt);
            const double Dd = p->Dskip ? p->Dskip[d] : 0.0;
            for (int t = 0; t < L; ++t) yr[t] += Dd * xr[t];
            for (int n = 0; n < N; ++n) {
                const double a = p->A[(long)d * N + n];
                const double *Bn = p->Bm + ((long)b * N + n) * L;
                const double *Cn = p->Cm + ((long)b * N + n) * L;
                double h = 0.0;
                if (dir == 0) {
                    for (int t = 0; t < L; ++t) {           /* Eq. 1-2 */
                        h = exp(dt[t] * a) * h + dt[t] * Bn[t] * xr[t];
                        yr[t] += Cn[t] * h;
                    }
                } else {
                    for (int t = L - 1; t >= 0; --t) {      /* Eq. 4-5 */
                        h = exp(dt[t] * a) * h + dt[t] * Bn[t] * xr[t];
                        yr[t] += Cn[t] * h;
                    }
                }
            }
        }
        if (pf->z) {
            const double *zr = pf->z + row * L;
            for (int t = 0; t < L; ++t) yr[t] *= zr[t] * sigmoid64(zr[t]);
        }
        free(dt);
    }
    return fail ? -2 : 0;
}

/*
 * Gradient of lbscan_ref_fwd.  With, per (b,d,n),
 *   abar_t = exp(dt_t A),  u_t = dt_t Bm_t x_t,
 *   f_t = abar_t f_{t-1} + u_t,
 *   g_t = 0 at the last step of a window, else abar_t (g_{t+1} + u_{t+1}),
 *   y_t = sum_n Cm_t (f_t + g_t) + Dskip x_t,   out_t = y_t SiLU(z_t),
 * reverse mode gives, with dy_t = dout_t SiLU(z_t) and e_t = dy_t Cm_t:
 *   phi_t   = e_t + abar_{t+1} phi_{t+1}             (adjoint of f_t; phi_L = 0)
 *   gamma_t = e_t + abar_{t-1} gamma_{t-1}  unless t opens a window, then e_t
 *                                                    (adjoint of g_t)
 *   du_t    = phi_t + (gamma_t - e_t)                (u_t feeds f_t and g_{t-1})
 *   q_t     = phi_t (f_t - u_t) + gamma_t g_t        (= abar_t * adjoint of abar_t)
 *   ddt_t   = sum_n q_t A + du_t Bm_t x_t ;  dA += q_t dt_t
 *   dBm_t  += du_t dt_t x_t ;  dx_t += du_t dt_t Bm_t + Dskip dy_t
 *   dCm_t  += dy_t (f_t + g_t) ;  dDskip += dy_t x_t
 *   dz_t    = dout_t y_t sigma(z_t) (1 + z_t (1 - sigma(z_t)))
 *   ddelta_t = ddt_t sigma(delta_t + bias) under softplus, else ddt_t;
 *   ddelta_bias = sum_{b,t} ddelta_t.
 * With a state h0 entering (f_{-1} = h0) and the final state hT = f_{L-1}
 * returned, the loss may also depend on hT: its gradient dhT joins phi at the
 * last step (phi_{L-1} = e_{L-1} + dhT), and dh0 = abar_0 phi_0.
 * Every output is overwritten.  dz may be NULL iff p->z is NULL; h0, dhT and
 * dh0 may be NULL.
 */
int lbscan_ref_bwd_state(const lbref_problem *p, const double *h0, const double *dout,
                         const double *dhT,
                         double *dx, double *ddelta, double *dz,
                         double *dBm, double *dCm,
                         double *dA, double *dDskip, double *ddelta_bias, double *dh0)
{
    if (check_problem(p) || !dout || !dx || !ddelta || !dBm || !dCm || !dA ||
        !dDskip || !ddelta_bias) return -1;
    if (p->z && !dz) return -1;
    const int Bsz = p->batch, D = p->dim, N = p->dstate, L = p->seqlen, M = p->window;
    memset(dBm, 0, sizeof(double) * (size_t)Bsz * N * L);
    memset(dCm, 0, sizeof(double) * (size_t)Bsz * N * L);
    memset(dA, 0, sizeof(double) * (size_t)D * N);
    memset(dDskip, 0, sizeof(double) * (size_t)D);
    memset(ddelta_bias, 0, sizeof(double) * (size_t)D);
    if ((long)Bsz * D * L == 0) {
        if (dh0)
            for (long i = 0; i < (long)Bsz * D * N; ++i) dh0[i] = dhT ? dhT[i] : 0.0;
        return 0;
    }
    int fail = 0;
    /* Rows of one batch entry share dBm/dCm; rows of one channel share
       dA/dDskip/ddelta_bias.  Loop batch entries in order and parallelise over
       channels: channel-owned sums need no synchronisation, and the
       (N,L)-sized sums are merged under a critical section. */
    for (int b = 0; b < Bsz; ++b) {
#pragma omp parallel
        {
            double *dt = (double *)malloc(sizeof(double) * L);
            double *ddt = (double *)malloc(sizeof(double) * L);
            double *yy = (double *)malloc(sizeof(double) * L);
            double *dy = (double *)malloc(sizeof(double) * L);
            double *F = (double *)malloc(sizeof(double) * L);
            double *G = (double *)malloc(sizeof(double) * L);
            double *ab = (double *)malloc(sizeof(double) * L);
            double *u = (double *)malloc(sizeof(double) * L);
            double *gam = (double *)malloc(sizeof(double) * L);
            double *accB = (double *)calloc((size_t)N * L, sizeof(double));
            double *accC = (double *)calloc((size_t)N * L, sizeof(double));
            int ok = dt && ddt && yy && dy && F && G && ab && u && gam && accB && accC;
            if (!ok) {
#pragma omp atomic write
                fail = 1;
            }
#pragma omp for schedule(static)
            for (int d = 0; d < D; ++d) {
                if (!ok) continue;
                const long row = (long)b * D + d;
                const double *xr = p->x + row * L, *draw = p->delta + row * L;
                const double *gr = dout + row * L;
                const double *zr = p->z ? p->z + row * L : NULL;
                const double Dd = p->Dskip ? p->Dskip[d] : 0.0;
                const double bias = p->delta_bias ? p->delta_bias[d] : 0.0;
                row_timestep(p, d, draw, dt);
                for (int t = 0; t < L; ++t) {
                    dy[t] = zr ? gr[t] * zr[t] * sigmoid64(zr[t]) : gr[t];
                    yy[t] = Dd * xr[t];
                    ddt[t] = 0.0;
                    dx[row * L + t] = Dd * dy[t];
                    dDskip[d] += dy[t] * xr[t];
                }
                for (int n = 0; n < N; ++n) {
                    const double a = p->A[(long)d * N + n];
                    const double *Bn = p->Bm + ((long)b * N + n) * L;
                    const double *Cn = p->Cm + ((long)b * N + n) * L;
                    double *aB = accB + (long)n * L, *aC = accC + (long)n * L;
                    /* recompute the forward quantities */
                    const double hin = h0 ? h0[row * N + n] : 0.0;
                    double hf = hin;
                    for (int t = 0; t < L; ++t) {
                        ab[t] = exp(dt[t] * a);
                        u[t] = dt[t] * Bn[t] * xr[t];
                        hf = ab[t] * hf + u[t];
                        F[t] = hf;
                    }
                    for (int t = L - 1; t >= 0; --t) {
                        if ((t + 1) % M == 0 || t == L - 1) G[t] = 0.0;
                        else G[t] = ab[t] * (G[t + 1] + u[t + 1]);
                        yy[t] += Cn[t] * (F[t] + G[t]);
                        aC[t] += dy[t] * (F[t] + G[t]);
                    }
                    /* adjoint of g: forward in time inside each window */
                    for (int t = 0; t < L; ++t) {
                        double e = dy[t] * Cn[t];
                        gam[t] = (t % M == 0) ? e : e + ab[t - 1] * gam[t - 1];
                    }
                    /* adjoint of f: backward in time over the whole row */
                    double phi = 0.0, qsum = 0.0;
                    const double dlast = dhT ? dhT[row * N + n] : 0.0;
                    for (int t = L - 1; t >= 0; --t) {
                        double e = dy[t] * Cn[t];
                        phi = e + (t + 1 < L ? ab[t + 1] * phi : dlast);
                        double du = phi + (gam[t] - e);
                        double q = phi * (F[t] - u[t]) + gam[t] * G[t];
                        ddt[t] += q * a + du * Bn[t] * xr[t];
                        qsum += q * dt[t];
                        aB[t] += du * dt[t] * xr[t];
                        dx[row * L + t] += du * dt[t] * Bn[t];
                    }
                    dA[(long)d * N + n] += qsum;
                    if (dh0) dh0[row * N + n] = ab[0] * phi;
                }
                for (int t = 0; t < L; ++t) {
                    double dd = p->delta_softplus ? ddt[t] * sigmoid64(draw[t] + bias) : ddt[t];
                    /* softplus(v) = v above the threshold: derivative 1 there */
                    if (p->delta_softplus && draw[t] + bias > 20.0) dd = ddt[t];
                    ddelta[row * L + t] = dd;
                    ddelta_bias[d] += dd;
                    if (zr) {
                        double s = sigmoid64(zr[t]);
                        dz[row * L + t] = gr[t] * yy[t] * s * (1.0 + zr[t] * (1.0 - s));
                    }
                }
            }
#pragma omp critical
            {
                if (ok) {
                    double *gB = dBm + (long)b * N * L, *gC = dCm + (long)b * N * L;
                    for (long i = 0; i < (long)N * L; ++i) { gB[i] += accB[i]; gC[i] += accC[i]; }
                }
            }
            free(dt); free(ddt); free(yy); free(dy); free(F); free(G);
            free(ab); free(u); free(gam); free(accB); free(accC);
        }
    }
    return fail ? -2 : 0;
}

int lbscan_ref_bwd(const lbref_problem *p, const double *dout,
                   double *dx, double *ddelta, double *dz,
                   double *dBm, double *dCm,
                   double *dA, double *dDskip, double *ddelta_bias)
{
    return lbscan_ref_bwd_state(p, NULL, dout, NULL, dx, ddelta, dz, dBm, dCm, dA, dDskip,
                                ddelta_bias, NULL);
}
