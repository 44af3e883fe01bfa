/*
 * CPU oracle for optimizer update / update-undo and the state digest.
 *
 * TEST INFRASTRUCTURE ONLY.  Plain scalar loops in IEEE binary64, written to be
 * checked against the paper by eye.  Nothing here is tuned, blocked, fused or
 * vectorised by hand, and nothing here is shared with (or included by) the GPU
 * library.  Only the tests, the smoke check and the benchmark's CPU-baseline leg
 * may call it.
 *
 * Conventions
 *   - one call maps the state at iteration t ("old": x_t, m_{t-1}, v_{t-1}) to the
 *     state at iteration t+1 ("new": x_{t+1}, m_t, v_t), or back;
 *   - every array holds n doubles; outputs never alias inputs;
 *   - `t` is the same integer in a step and in the undo of that step;
 *   - no clamping, no flushing, NaN/Inf propagate as IEEE arithmetic dictates;
 *   - build with -ffp-contract=off so that a*b+c is two roundings, as written.
 *
 * Readings of the paper taken here (the printed algorithms drift in their
 * subscripts and two lines are garbled):
 *   - weight-decay terms always use the pre-update parameter;
 *   - Undo Adam's last line squares g' (the exponent is misprinted);
 *   - Undo AdamW's parameter line has eps inside the denominator, (sqrt(v^)+eps),
 *     the only placement that inverts the AdamW update line;
 *   - AdamW's alpha, never defined in the paper, is 1;
 *   - eps is added after the square root of the bias-corrected second moment;
 *   - bias corrections are 1 - pow(beta, t), evaluated in binary64.
 */
#include <math.h>
#include <stdint.h>
#include <string.h>

/* ------------------------------------------------------------------------- */
/* Alg. 1 (SGD with Momentum): m_t = mu m_{t-1} + (1-tau)(g_t + lambda x_t);    */
/*                             x_{t+1} = x_t - eta_t m_t.                       */
/* With mu = 0 this is App. A's plain SGD with the damped gradient kept in m.   */
void oracle_sgdm_step(int64_t n, const double *x, const double *g, const double *m,
                      double eta, double lambda, double mu, double tau,
                      double *x_new, double *m_new)
{
    for (int64_t i = 0; i < n; ++i) {
        double gp = g[i] + lambda * x[i];
        double mt = mu * m[i] + (1.0 - tau) * gp;
        m_new[i] = mt;
        x_new[i] = x[i] - eta * mt;
    }
}

/* Alg. 2 (Undo SGD with Momentum): x_t = x_{t+1} + eta_t m_t;                  */
/*                                  m_{t-1} = (m_t - (1-tau)(g_t + lambda x_t))/mu. */
/* The recovered x_t (not x_{t+1}) enters the weight-decay term.                 */
/* mu = 0: the second line divides by zero; m_{t-1} carried no information into  */
/* step t (it was multiplied by mu = 0), so the buffer is returned unchanged.    */
void oracle_sgdm_undo(int64_t n, const double *x_new, const double *g, const double *m_new,
                      double eta, double lambda, double mu, double tau,
                      double *x_old, double *m_old)
{
    for (int64_t i = 0; i < n; ++i) {
        double xt = x_new[i] + eta * m_new[i];
        x_old[i] = xt;
        if (mu == 0.0) {
            m_old[i] = m_new[i];
        } else {
            double gp = g[i] + lambda * xt;
            m_old[i] = (m_new[i] - (1.0 - tau) * gp) / mu;
        }
    }
}

/* ------------------------------------------------------------------------- */
/* App. A, Alg. "SGD": x_{t+1} = x_t - eta_t (g_t + lambda x_t).  No optimizer state. */
void oracle_sgd_step(int64_t n, const double *x, const double *g, double eta, double lambda, double *x_new)
{
    for (int64_t i = 0; i < n; ++i) {
        x_new[i] = x[i] - eta * (g[i] + lambda * x[i]);
    }
}

/* App. A, Alg. "Undo SGD": x_t = (x_{t+1} + eta_t g_t) / (1 - eta_t lambda).       */
/* (The printed line drops the subscript of eta in the denominator; it is the same  */
/* eta_t.)  eta_t lambda = 1 divides by zero: the caller refuses that case.         */
void oracle_sgd_undo(int64_t n, const double *x_new, const double *g, double eta, double lambda, double *x_old)
{
    for (int64_t i = 0; i < n; ++i) {
        x_old[i] = (x_new[i] + eta * g[i]) / (1.0 - eta * lambda);
    }
}

/* ------------------------------------------------------------------------- */
/* App. A, Alg. "Adam" (weight decay coupled into the gradient).                */
void oracle_adam_step(int64_t n, const double *x, const double *g, const double *m, const double *v,
                      double eta, double lambda, double beta1, double beta2, double eps, int64_t t,
                      double *x_new, double *m_new, double *v_new)
{
    double bc1 = 1.0 - pow(beta1, (double)t);
    double bc2 = 1.0 - pow(beta2, (double)t);
    for (int64_t i = 0; i < n; ++i) {
        double gp = g[i] + lambda * x[i];
        double mt = beta1 * m[i] + (1.0 - beta1) * gp;
        double vt = beta2 * v[i] + (1.0 - beta2) * (gp * gp);
        double mhat = mt / bc1;
        double vhat = vt / bc2;
        m_new[i] = mt;
        v_new[i] = vt;
        x_new[i] = x[i] - eta * mhat / (sqrt(vhat) + eps);
    }
}

/* App. A, Alg. "Undo Adam": the parameter is recovered first, from the new     */
/* moments; the recovered parameter then rebuilds g'; the two moment recurrences */
/* are solved for their previous values.                                         */
void oracle_adam_undo(int64_t n, const double *x_new, const double *g, const double *m_new, const double *v_new,
                      double eta, double lambda, double beta1, double beta2, double eps, int64_t t,
                      double *x_old, double *m_old, double *v_old)
{
    double bc1 = 1.0 - pow(beta1, (double)t);
    double bc2 = 1.0 - pow(beta2, (double)t);
    for (int64_t i = 0; i < n; ++i) {
        double mhat = m_new[i] / bc1;
        double vhat = v_new[i] / bc2;
        double xt = x_new[i] + eta * mhat / (sqrt(vhat) + eps);
        double gp = g[i] + lambda * xt;
        x_old[i] = xt;
        m_old[i] = (m_new[i] - (1.0 - beta1) * gp) / beta1;
        v_old[i] = (v_new[i] - (1.0 - beta2) * (gp * gp)) / beta2;
    }
}

/* ------------------------------------------------------------------------- */
/* App. A, Alg. "AdamW" (decoupled decay, alpha = 1): moments from the raw      */
/* gradient; x_new = x - eta (u + lambda x), u = m^/(sqrt(v^)+eps).               */
void oracle_adamw_step(int64_t n, const double *x, const double *g, const double *m, const double *v,
                       double eta, double lambda, double beta1, double beta2, double eps, int64_t t,
                       double *x_new, double *m_new, double *v_new)
{
    double bc1 = 1.0 - pow(beta1, (double)t);
    double bc2 = 1.0 - pow(beta2, (double)t);
    for (int64_t i = 0; i < n; ++i) {
        double mt = beta1 * m[i] + (1.0 - beta1) * g[i];
        double vt = beta2 * v[i] + (1.0 - beta2) * (g[i] * g[i]);
        double mhat = mt / bc1;
        double vhat = vt / bc2;
        double u = mhat / (sqrt(vhat) + eps);
        m_new[i] = mt;
        v_new[i] = vt;
        x_new[i] = x[i] - eta * (u + lambda * x[i]);
    }
}

/* App. A, Alg. "Undo AdamW": x_old = (x_new + eta u)/(1 - eta lambda);          */
/* moments as in Undo Adam but with the raw gradient.                            */
void oracle_adamw_undo(int64_t n, const double *x_new, const double *g, const double *m_new, const double *v_new,
                       double eta, double lambda, double beta1, double beta2, double eps, int64_t t,
                       double *x_old, double *m_old, double *v_old)
{
    double bc1 = 1.0 - pow(beta1, (double)t);
    double bc2 = 1.0 - pow(beta2, (double)t);
    for (int64_t i = 0; i < n; ++i) {
        double mhat = m_new[i] / bc1;
        double vhat = v_new[i] / bc2;
        double u = mhat / (sqrt(vhat) + eps);
        x_old[i] = (x_new[i] + eta * u) / (1.0 - eta * lambda);
        m_old[i] = (m_new[i] - (1.0 - beta1) * g[i]) / beta1;
        v_old[i] = (v_new[i] - (1.0 - beta2) * (g[i] * g[i])) / beta2;
    }
}

/* ------------------------------------------------------------------------- */
/* LAMB for ONE tensor (one "layer").  The paper prints no LAMB algorithm; it says   */
/* (section "Update-undo", Table 1) that LAMB adds a sum -- the L2 norms behind its   */
/* trust ratio -- to Adam's elementwise operators, and that saving the norm (a scalar) */
/* at step time makes the step invertible.  The step below is the published LAMB      */
/* update (You et al. 2019, Alg. 2) with phi = identity:                               */
/*   m_t, v_t, m^, v^ as in AdamW;  r = m^/(sqrt(v^)+eps);  u = r + lambda x_t;        */
/*   q = ||x_t|| / ||u||  (q = 1 if either norm is 0);  x_{t+1} = x_t - eta q u.       */
/* norms[0] = ||x_t||, norms[1] = ||u|| are returned: they are what the undo needs.    */
void oracle_lamb_step(int64_t n, const double *x, const double *g, const double *m, const double *v,
                      double eta, double lambda, double beta1, double beta2, double eps, int64_t t,
                      double *x_new, double *m_new, double *v_new, double *norms)
{
    double bc1 = 1.0 - pow(beta1, (double)t);
    double bc2 = 1.0 - pow(beta2, (double)t);
    double sx = 0.0, su = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        double mt = beta1 * m[i] + (1.0 - beta1) * g[i];
        double vt = beta2 * v[i] + (1.0 - beta2) * (g[i] * g[i]);
        double r = (mt / bc1) / (sqrt(vt / bc2) + eps);
        double u = r + lambda * x[i];
        m_new[i] = mt;
        v_new[i] = vt;
        x_new[i] = u;                 /* parked here until the norms are known */
        sx += x[i] * x[i];
        su += u * u;
    }
    double nx = sqrt(sx), nu = sqrt(su);
    double q = (nx > 0.0 && nu > 0.0) ? nx / nu : 1.0;
    for (int64_t i = 0; i < n; ++i)
        x_new[i] = x[i] - eta * q * x_new[i];
    norms[0] = nx;
    norms[1] = nu;
}

/* Undo of the LAMB step with the two saved norms: q is rebuilt from them, r from the */
/* new moments, and x_{t+1} = x_t (1 - eta q lambda) - eta q r is solved for x_t;      */
/* the moments go back as in "Undo AdamW" (App. A).                                    */
void oracle_lamb_undo(int64_t n, const double *x_new, const double *g, const double *m_new, const double *v_new,
                      double eta, double lambda, double beta1, double beta2, double eps, int64_t t,
                      const double *norms, double *x_old, double *m_old, double *v_old)
{
    double bc1 = 1.0 - pow(beta1, (double)t);
    double bc2 = 1.0 - pow(beta2, (double)t);
    double q = (norms[0] > 0.0 && norms[1] > 0.0) ? norms[0] / norms[1] : 1.0;
    for (int64_t i = 0; i < n; ++i) {
        double r = (m_new[i] / bc1) / (sqrt(v_new[i] / bc2) + eps);
        x_old[i] = (x_new[i] + eta * q * r) / (1.0 - eta * q * lambda);
        m_old[i] = (m_new[i] - (1.0 - beta1) * g[i]) / beta1;
        v_old[i] = (v_new[i] - (1.0 - beta2) * (g[i] * g[i])) / beta2;
    }
}

/* ------------------------------------------------------------------------- */
/* Not in the paper: optional clamp of the second moment an undo recovered.     */
/* "Undo Adam" (App. A) solves v_t = beta2 v_{t-1} + (1-beta2) g'^2 for v_{t-1};  */
/* with a rounded v_t the solution can be slightly negative.  The clamp is a     */
/* separate pass over the undo's output: values below zero become +0, NaN stays. */
void oracle_clamp_v(int64_t n, double *v_old)
{
    for (int64_t i = 0; i < n; ++i) {
        if (v_old[i] < 0.0) v_old[i] = 0.0;
    }
}

/* ------------------------------------------------------------------------- */
/* bfloat16 copy of binary32 parameters (mixed-precision training keeps one next to   */
/* the fp32 master weights; not in the paper).  bfloat16 is the upper half of binary32 */
/* (8 exponent bits, 7 fraction bits); the copy is the nearest bfloat16, ties to the   */
/* value whose last fraction bit is 0; overflow rounds to infinity; every NaN becomes   */
/* the quiet NaN 0x7FC0.                                                                */
void oracle_bf16_round(int64_t n, const float *x, uint16_t *out)
{
    for (int64_t i = 0; i < n; ++i) {
        uint32_t u;
        memcpy(&u, &x[i], 4);
        if ((u & 0x7FFFFFFFu) > 0x7F800000u) {          /* NaN */
            out[i] = 0x7FC0u;
            continue;
        }
        uint32_t kept = u >> 16;                        /* truncated candidate */
        uint32_t dropped = u & 0xFFFFu;                 /* the 16 bits that do not fit */
        if (dropped > 0x8000u || (dropped == 0x8000u && (kept & 1u)))
            kept += 1u;                                 /* nearer neighbour is above, or tie and odd */
        out[i] = (uint16_t)kept;                        /* a carry into the exponent is the right value */
    }
}

/* ------------------------------------------------------------------------- */
/* State digest of one shard of n 32-bit words (n < 2^32).                       */
/* Not from the paper (which keeps a per-parameter "updated" flag): it is this   */
/* library's stand-in for that flag.  Each word is tagged with its index inside  */
/* the shard, passed through a 64-bit mixer made of bijective steps, and the      */
/* mixed words are summed modulo 2^64, so the order of summation is immaterial.   */
/*   z = (i << 32) | w_i;  z += K1;  z ^= z >> 32;  z *= K2;  z ^= z >> 29;        */
/*   z *= K3;  z ^= z >> 32;   digest = sum_i z   (empty shard: 0)                 */
uint64_t oracle_digest(const uint32_t *w, int64_t n)
{
    const uint64_t K1 = 0x9E3779B97F4A7C15ull;
    const uint64_t K2 = 0x6A09E667F3BCC909ull;
    const uint64_t K3 = 0xBB67AE8584CAA73Bull;
    uint64_t sum = 0;
    for (int64_t i = 0; i < n; ++i) {
        uint64_t z = ((uint64_t)i << 32) | (uint64_t)w[i];
        z += K1;
        z ^= z >> 32;
        z *= K2;
        z ^= z >> 29;
        z *= K3;
        z ^= z >> 32;
        sum += z;
    }
    return sum;
}
