/*
 * gsa_oracle.c -- fp64 CPU oracle for Gated Slot Attention (GSA).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * GPU library is checked against.  Nothing in the product path may call it:
 * only the tests, the smoke check and the CPU-baseline leg of the benchmark
 * load it.  It shares no code, header, table or helper with the HIP kernels.
 *
 * What it computes (paper, Section 3.2, Eq. (gsa); read-out as in Eq. (memory)
 * of Section 2.1, softmax taken over the m slots):
 *
 *     a_t = exp(g_t),  s_t = 1 - a_t = -expm1(g_t)            (g_t = log alpha_t)
 *     Kt[i,:] <- a_t[i] * Kt[i,:] + s_t[i] * k_t              (slot memories,
 *     Vt[i,:] <- a_t[i] * Vt[i,:] + s_t[i] * v_t               one row per slot)
 *     z_t[i]   = scale * <Kt[i,:], q_t>
 *     p_t      = softmax(z_t)
 *     o_t      = sum_i p_t[i] * Vt[i,:]
 *
 * token by token, per sequence and head, in double precision.  Token t reads
 * the memories after its own write.  The paper has no score scaling; scale is
 * an explicit argument (1.0 = the paper).
 *
 * Variants (Algorithm 1 takes the write intensity I as an input of its own;
 * Section 2.2, Eqs. (abc_recurrent)/(abc_phi); the read-out ablations of the
 * ablation table in Section 4):
 *   - write intensity given: s_t is read from an array `sin` instead of being
 *     1 - exp(g_t).  With g = 0 and s = phi this is ABC, Eq. (abc_recurrent).
 *     The backward then returns dg for the gate alone and ds for the intensity.
 *   - read-out f instead of softmax: p_t = f(z_t) element by element,
 *     f in {identity, Swish z*sigmoid(z), ReLU, ReLU^2}.
 *
 * The backward pass is back-propagation through exactly those lines, walking
 * the tokens in reverse; the states needed on the way back are recomputed from
 * checkpoints taken every GSA_ORACLE_CKPT tokens.
 *
 * Parity pins (tests/test_oracle_pins.py): brute-force quadratic form with
 * explicit cumulative gate products, m = 1 closed form, chunk/segment
 * invariance, g = 0 (frozen memories = softmax attention over fixed slots),
 * g = -inf (o_t = v_t), convexity bounds, slot-permutation symmetry, and
 * central finite differences for every gradient.  No function here is
 * "parity unpinned".
 *
 * Layout: tokens are packed along one axis; sequence s covers tokens
 * cu[s] .. cu[s+1]-1.  q,k are [Ttot,H,dk], v is [Ttot,H,dv], g is [Ttot,H,m],
 * states are [n_seqs,H,m,d]; all dense, last index fastest.  Every input,
 * every output and all arithmetic is double (each bf16 or fp32 value the GPU
 * reads converts to double exactly).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define GSA_ORACLE_CKPT 64

/* read-outs: how the slot scores z become the read weights p */
enum { RO_SOFTMAX = 0, RO_IDENTITY = 1, RO_SWISH = 2, RO_RELU = 3, RO_RELU2 = 4 };

static double sigmoid(double x) { return 1.0 / (1.0 + exp(-x)); }

/* p = f(z) over the m slots */
static void readout_fwd(int ro, int m, const double *z, double *p)
{
    if (ro == RO_SOFTMAX) {
        double zmax = -INFINITY, den = 0.0;
        for (int i = 0; i < m; ++i) if (z[i] > zmax) zmax = z[i];
        for (int i = 0; i < m; ++i) { p[i] = exp(z[i] - zmax); den += p[i]; }
        for (int i = 0; i < m; ++i) p[i] /= den;
        return;
    }
    for (int i = 0; i < m; ++i) {
        double x = z[i];
        if (ro == RO_IDENTITY) p[i] = x;
        else if (ro == RO_SWISH) p[i] = x * sigmoid(x);
        else if (ro == RO_RELU) p[i] = x > 0.0 ? x : 0.0;
        else p[i] = x > 0.0 ? x * x : 0.0;
    }
}

/* dz from dp (p = f(z) as computed by readout_fwd).  ReLU's slope at z = 0 is taken as 0. */
static void readout_bwd(int ro, int m, const double *z, const double *p, const double *dp, double *dz)
{
    if (ro == RO_SOFTMAX) {
        double pdp = 0.0;
        for (int i = 0; i < m; ++i) pdp += p[i] * dp[i];
        for (int i = 0; i < m; ++i) dz[i] = p[i] * (dp[i] - pdp);
        return;
    }
    for (int i = 0; i < m; ++i) {
        double x = z[i], d;
        if (ro == RO_IDENTITY) d = 1.0;
        else if (ro == RO_SWISH) { double sg = sigmoid(x); d = sg + x * sg * (1.0 - sg); }
        else if (ro == RO_RELU) d = x > 0.0 ? 1.0 : 0.0;
        else d = x > 0.0 ? 2.0 * x : 0.0;
        dz[i] = d * dp[i];
    }
}

int gsa_oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* One token of Eq. (gsa): update both memories in place, then read out. */
static void step_token(int dk, int dv, int m, double scale, int ro,
                       const double *q, const double *k, const double *v, const double *g, const double *sin,
                       double *K, double *V, double *z, double *p, double *o)
{
    for (int i = 0; i < m; ++i) {
        double a = exp(g[i]);
        double s = sin ? sin[i] : -expm1(g[i]);
        double *Ki = K + (size_t)i * dk;
        double *Vi = V + (size_t)i * dv;
        for (int c = 0; c < dk; ++c) Ki[c] = a * Ki[c] + s * k[c];
        for (int c = 0; c < dv; ++c) Vi[c] = a * Vi[c] + s * v[c];
    }
    if (!q) return; /* state-only step (used while replaying checkpoints) */
    for (int i = 0; i < m; ++i) {
        const double *Ki = K + (size_t)i * dk;
        double acc = 0.0;
        for (int c = 0; c < dk; ++c) acc += Ki[c] * q[c];
        z[i] = scale * acc;
    }
    readout_fwd(ro, m, z, p);
    if (!o) return;
    for (int c = 0; c < dv; ++c) o[c] = 0.0;
    for (int i = 0; i < m; ++i) {
        const double *Vi = V + (size_t)i * dv;
        for (int c = 0; c < dv; ++c) o[c] += p[i] * Vi[c];
    }
}

/*
 * Forward.  sin [Ttot,H,m] is the write intensity, or NULL for s = 1 - exp(g);
 * readout is one of RO_*.  K0,V0 may be NULL (zero memories, as the paper initialises them).
 * o [Ttot,H,dv]; z_out [Ttot,H,m] (pre-softmax scores), KT,VT [n_seqs,H,m,d]
 * (memories after the last token); each of z_out, KT, VT may be NULL.
 * Returns 0, or -1 if an allocation failed.
 */
int gsa_oracle_fwd(int n_seqs, const int32_t *cu, int H, int dk, int dv, int m, double scale, int readout,
                   const double *q, const double *k, const double *v, const double *g, const double *sin,
                   const double *K0, const double *V0,
                   double *o, double *z_out, double *KT, double *VT)
{
    int fail = 0;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int s = 0; s < n_seqs; ++s) {
        for (int h = 0; h < H; ++h) {
            double *K = (double *)calloc((size_t)m * dk, sizeof(double));
            double *V = (double *)calloc((size_t)m * dv, sizeof(double));
            double *z = (double *)malloc(sizeof(double) * 2 * (size_t)m);
            if (!K || !V || !z) {
#pragma omp atomic write
                fail = 1;
                free(K); free(V); free(z);
                continue;
            }
            double *p = z + m;
            size_t sh = (size_t)s * H + h;
            if (K0) memcpy(K, K0 + sh * m * dk, sizeof(double) * (size_t)m * dk);
            if (V0) memcpy(V, V0 + sh * m * dv, sizeof(double) * (size_t)m * dv);
            for (int64_t t = cu[s]; t < cu[s + 1]; ++t) {
                size_t th = (size_t)t * H + h;
                step_token(dk, dv, m, scale, readout, q + th * dk, k + th * dk, v + th * dv, g + th * m,
                           sin ? sin + th * m : NULL, K, V, z, p, o + th * dv);
                if (z_out) memcpy(z_out + th * m, z, sizeof(double) * (size_t)m);
            }
            if (KT) memcpy(KT + sh * m * dk, K, sizeof(double) * (size_t)m * dk);
            if (VT) memcpy(VT + sh * m * dv, V, sizeof(double) * (size_t)m * dv);
            free(K); free(V); free(z);
        }
    }
    return fail ? -1 : 0;
}

/*
 * Backward of L = sum_t <dO_t, o_t> + <dKT, K_T> + <dVT, V_T>.
 * dO [Ttot,H,dv]; dKT,dVT [n_seqs,H,m,d] (may be NULL = zero).
 * Outputs (double): dq,dk [Ttot,H,dk], dv [Ttot,H,dv], dg [Ttot,H,m] (gradient
 * with respect to the log forget gate g, with s = 1 - exp(g) coupled to it when
 * sin is NULL; with sin given, dg is the gradient through the decay alone and
 * dsin [Ttot,H,m] receives the gradient of the write intensity),
 * dK0,dV0 [n_seqs,H,m,d] (may be NULL); dp_out, dz_out [Ttot,H,m] (may be NULL): the gradients with
 * respect to the read weights p_t and the scores z_t, the two intermediates of the chain.
 */
int gsa_oracle_bwd(int n_seqs, const int32_t *cu, int H, int dk, int dv, int m, double scale, int readout,
                   const double *q, const double *k, const double *v, const double *g, const double *sin,
                   const double *K0, const double *V0, const double *dO,
                   const double *dKT, const double *dVT,
                   double *dq, double *dkk, double *dvv, double *dg, double *dsin,
                   double *dK0, double *dV0, double *dp_out, double *dz_out)
{
    int fail = 0;
    const size_t nK = (size_t)m * dk, nV = (size_t)m * dv;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int s = 0; s < n_seqs; ++s) {
        for (int h = 0; h < H; ++h) {
            const int64_t t0 = cu[s], t1 = cu[s + 1];
            const int64_t L = t1 - t0;
            const int64_t nck = (L + GSA_ORACLE_CKPT - 1) / GSA_ORACLE_CKPT;
            size_t sh = (size_t)s * H + h;
            /* ckK[c] = memories before token t0 + c*CKPT */
            double *ckK = (double *)malloc(sizeof(double) * nK * (size_t)(nck > 0 ? nck : 1));
            double *ckV = (double *)malloc(sizeof(double) * nV * (size_t)(nck > 0 ? nck : 1));
            /* blkK[j] = memories before token j of the current block, j = 0..CKPT */
            double *blkK = (double *)malloc(sizeof(double) * nK * (GSA_ORACLE_CKPT + 1));
            double *blkV = (double *)malloc(sizeof(double) * nV * (GSA_ORACLE_CKPT + 1));
            double *gK = (double *)calloc(nK, sizeof(double));
            double *gV = (double *)calloc(nV, sizeof(double));
            double *tmp = (double *)malloc(sizeof(double) * 4 * (size_t)m);
            if (!ckK || !ckV || !blkK || !blkV || !gK || !gV || !tmp) {
#pragma omp atomic write
                fail = 1;
                free(ckK); free(ckV); free(blkK); free(blkV); free(gK); free(gV); free(tmp);
                continue;
            }
            double *z = tmp, *p = tmp + m, *dp = tmp + 2 * m, *dz = tmp + 3 * m;
            /* forward sweep, keeping a checkpoint at the start of every block */
            {
                double *K = blkK, *V = blkV; /* scratch */
                memset(K, 0, sizeof(double) * nK);
                memset(V, 0, sizeof(double) * nV);
                if (K0) memcpy(K, K0 + sh * nK, sizeof(double) * nK);
                if (V0) memcpy(V, V0 + sh * nV, sizeof(double) * nV);
                for (int64_t j = 0; j < L; ++j) {
                    if (j % GSA_ORACLE_CKPT == 0) {
                        memcpy(ckK + (size_t)(j / GSA_ORACLE_CKPT) * nK, K, sizeof(double) * nK);
                        memcpy(ckV + (size_t)(j / GSA_ORACLE_CKPT) * nV, V, sizeof(double) * nV);
                    }
                    size_t th = (size_t)(t0 + j) * H + h;
                    step_token(dk, dv, m, scale, readout, NULL, k + th * dk, v + th * dv, g + th * m,
                               sin ? sin + th * m : NULL, K, V, NULL, NULL, NULL);
                }
            }
            if (dKT) memcpy(gK, dKT + sh * nK, sizeof(double) * nK);
            if (dVT) memcpy(gV, dVT + sh * nV, sizeof(double) * nV);
            for (int64_t c = nck - 1; c >= 0; --c) {
                const int64_t b0 = c * GSA_ORACLE_CKPT;
                const int64_t bl = (L - b0 < GSA_ORACLE_CKPT) ? (L - b0) : GSA_ORACLE_CKPT;
                memcpy(blkK, ckK + (size_t)c * nK, sizeof(double) * nK);
                memcpy(blkV, ckV + (size_t)c * nV, sizeof(double) * nV);
                for (int64_t j = 0; j < bl; ++j) {
                    size_t th = (size_t)(t0 + b0 + j) * H + h;
                    memcpy(blkK + (size_t)(j + 1) * nK, blkK + (size_t)j * nK, sizeof(double) * nK);
                    memcpy(blkV + (size_t)(j + 1) * nV, blkV + (size_t)j * nV, sizeof(double) * nV);
                    step_token(dk, dv, m, scale, readout, NULL, k + th * dk, v + th * dv, g + th * m,
                               sin ? sin + th * m : NULL,
                               blkK + (size_t)(j + 1) * nK, blkV + (size_t)(j + 1) * nV,
                               NULL, NULL, NULL);
                }
                for (int64_t j = bl - 1; j >= 0; --j) {
                    size_t th = (size_t)(t0 + b0 + j) * H + h;
                    const double *Kt = blkK + (size_t)(j + 1) * nK; /* after token's write */
                    const double *Vt = blkV + (size_t)(j + 1) * nV;
                    const double *Kp = blkK + (size_t)j * nK;       /* before it */
                    const double *Vp = blkV + (size_t)j * nV;
                    const double *qt = q + th * dk, *kt = k + th * dk, *vt = v + th * dv;
                    const double *gt = g + th * m, *dot = dO + th * dv;
                    /* recompute z, p of this token */
                    for (int i = 0; i < m; ++i) {
                        double acc = 0.0;
                        for (int cc = 0; cc < dk; ++cc) acc += Kt[(size_t)i * dk + cc] * qt[cc];
                        z[i] = scale * acc;
                    }
                    readout_fwd(readout, m, z, p);
                    /* o = V^T p  =>  dV += p (x) dO,  dp = V dO */
                    for (int i = 0; i < m; ++i) {
                        double acc = 0.0;
                        for (int cc = 0; cc < dv; ++cc) {
                            gV[(size_t)i * dv + cc] += p[i] * dot[cc];
                            acc += Vt[(size_t)i * dv + cc] * dot[cc];
                        }
                        dp[i] = acc;
                    }
                    /* p = f(z) */
                    readout_bwd(readout, m, z, p, dp, dz);
                    if (dp_out) memcpy(dp_out + th * m, dp, sizeof(double) * (size_t)m);
                    if (dz_out) memcpy(dz_out + th * m, dz, sizeof(double) * (size_t)m);
                    /* z = scale * K q  =>  dq = scale K^T dz,  dK += scale dz (x) q */
                    for (int cc = 0; cc < dk; ++cc) dq[th * dk + cc] = 0.0;
                    for (int i = 0; i < m; ++i) {
                        double w = scale * dz[i];
                        for (int cc = 0; cc < dk; ++cc) {
                            dq[th * dk + cc] += w * Kt[(size_t)i * dk + cc];
                            gK[(size_t)i * dk + cc] += w * qt[cc];
                        }
                    }
                    /* K_t = a K_{t-1} + s k_t  (rows), same for V */
                    for (int cc = 0; cc < dk; ++cc) dkk[th * dk + cc] = 0.0;
                    for (int cc = 0; cc < dv; ++cc) dvv[th * dv + cc] = 0.0;
                    for (int i = 0; i < m; ++i) {
                        double a = exp(gt[i]);
                        double sw = sin ? sin[th * m + i] : -expm1(gt[i]);
                        double ds = 0.0, da = 0.0;
                        for (int cc = 0; cc < dk; ++cc) {
                            double gk = gK[(size_t)i * dk + cc];
                            dkk[th * dk + cc] += sw * gk;
                            ds += gk * kt[cc];
                            da += gk * Kp[(size_t)i * dk + cc];
                            gK[(size_t)i * dk + cc] = a * gk;
                        }
                        for (int cc = 0; cc < dv; ++cc) {
                            double gv = gV[(size_t)i * dv + cc];
                            dvv[th * dv + cc] += sw * gv;
                            ds += gv * vt[cc];
                            da += gv * Vp[(size_t)i * dv + cc];
                            gV[(size_t)i * dv + cc] = a * gv;
                        }
                        if (sin) {   /* a = exp(g): da/dg = a; s is an input of its own */
                            dg[th * m + i] = a * da;
                            dsin[th * m + i] = ds;
                        } else {     /* a = exp(g), s = 1 - exp(g):  da/dg = a, ds/dg = -a */
                            dg[th * m + i] = a * (da - ds);
                        }
                    }
                }
            }
            if (dK0) memcpy(dK0 + sh * nK, gK, sizeof(double) * nK);
            if (dV0) memcpy(dV0 + sh * nV, gV, sizeof(double) * nV);
            free(ckK); free(ckV); free(blkK); free(blkV); free(gK); free(gV); free(tmp);
        }
    }
    return fail ? -1 : 0;
}

/*
 * One recurrent (decode) step of Eq. (gsa) for BH independent memories,
 * updated in place.  q,k [BH,dk], v [BH,dv], g [BH,m]; sin [BH,m] or NULL and readout as in the forward;
 * K [BH,m,dk], V [BH,m,dv], o [BH,dv] double.
 */
int gsa_oracle_decode_step(int BH, int dk, int dv, int m, double scale, int readout,
                           const double *q, const double *k, const double *v, const double *g, const double *sin,
                           double *K, double *V, double *o)
{
    int fail = 0;
#pragma omp parallel for schedule(static)
    for (int b = 0; b < BH; ++b) {
        double *zp = (double *)malloc(sizeof(double) * 2 * (size_t)m);
        if (!zp) {
#pragma omp atomic write
            fail = 1;
            continue;
        }
        step_token(dk, dv, m, scale, readout, q + (size_t)b * dk, k + (size_t)b * dk, v + (size_t)b * dv,
                   g + (size_t)b * m, sin ? sin + (size_t)b * m : NULL, K + (size_t)b * m * dk, V + (size_t)b * m * dv,
                   zp, zp + m, o + (size_t)b * dv);
        free(zp);
    }
    return fail ? -1 : 0;
}
