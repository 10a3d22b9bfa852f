/*
 * po_oracle.c -- CPU reference ("oracle") for PipeOptim's fused optimizer step
 * + optimizer-dependent weight prediction.
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It exists so that the GPU library can be
 * checked against something that is slow, plain and easy to compare with the
 * paper by eye.  It shares no code, header, table or constant with the HIP
 * library, and nothing in the product path may call it.
 *
 * What it computes, per element, in fp64 from fp32 inputs (the paper does not
 * fix a precision; fp32 state is this build's choice, fp64 arithmetic makes the
 * oracle's own rounding negligible):
 *
 *   optimizer state update and update direction dW_t   -- paper Table 1
 *   optimizer step   W_{t+1} = W_t - lr * dW_t         -- paper Eq. 1, first line
 *   prediction       What_{t+s} = W_t - lr * s * dW_t  -- paper Eq. 3 / Eq. 5
 *   version difference s = D - rank - 1                -- paper Eq. 4
 *   prediction from the cached state alone (no new gradient), as Algorithm 1
 *   sequences it ahead of the forward pass             -- po_oracle_predict
 *
 * Readings of the paper taken here, where it is silent or ambiguous:
 *   - dW_t is built from the *updated* state (m_t, v_t), i.e. from the new
 *     gradient g_t and the cached m_{t-1}, v_{t-1}       (Sec. III-A.3 prose).
 *   - The prediction starts from the same W_t the step starts from, so that
 *     s = 1 reproduces the optimizer's own step and s = 0 returns W_t.
 *   - s = 0 is the last pipeline stage, which does no prediction and uses W_t
 *     itself (Algorithm 1, else-branch): What is a copy of W_t.
 *   - Table 1 prints no weight decay.  SGDM / Adam: coupled L2, g~ = g + wd*W
 *     before the state update.  AdamW: decoupled decay; Eq. 1 defines dW_t as
 *     the whole per-step increment over lr, so dW_t = r + wd*W
 *     ("decay_in_prediction" = 1).  With decay_in_prediction = 0 the prediction
 *     uses Table 1's AdamW row exactly as printed (r alone) while the step
 *     still decays.
 *   - eps is added after the square root and after bias correction (Table 1).
 *   - SGDM applies m_t = u*m_{t-1} + (1-tau)*g_t uniformly, no first-step case.
 *   - Outputs are rounded once from fp64 to fp32 (round-to-nearest-even, the C
 *     cast); the bf16 copy of What is the fp32 What rounded to nearest-even.
 *
 * Pins (tests/test_oracle_*.py): the step against torch.optim's fp64 SGD /
 * Adam / AdamW, the prediction law against the s = 0, s = 1 and affine-in-s
 * invariants and the constant-direction case of Eq. 2, Table 1 against hand
 * cases and closed forms, Eq. 4 against the indices of the Fig. 2 discussion,
 * the bf16 rounding against an integer formulation and torch's cast;
 * po_oracle_predict against closed forms, hand cases, and its consistency with
 * the (independently pinned) fused function: predicting s versions ahead from
 * the state a fused call leaves equals the fused call's own s+1 prediction.
 * Parity unpinned by the paper itself: the choice of prediction base (W_t
 * rather than W_{t+1}) and the AdamW decay reading; both are fixed by the
 * invariants above, not by a printed value.
 */
#include <math.h>
#include <stdint.h>
#include <string.h>

/* 0-2: the rows of paper Table 1.  3-5: further optimizers, by the table's own recipe (Sec. III-A.3: dW_t
 * follows from the update rule of the optimizer in use; Eq. 1 makes it the optimizer's increment over lr). */
enum { PO_ORACLE_SGDM = 0, PO_ORACLE_ADAM = 1, PO_ORACLE_ADAMW = 2,
       PO_ORACLE_NESTEROV = 3, PO_ORACLE_RMSPROP = 4, PO_ORACLE_ADAGRAD = 5 };

/* ---- bf16 rounding: nearest representable bf16, ties to the even code ------
 * A bf16 is the upper 16 bits of an fp32.  The two neighbours of x are the
 * truncated pattern `lo` and the next pattern away from zero `hi`; pick the
 * closer one, and on a tie the one whose last kept bit is 0. */
static float f32_from_bits(uint32_t b) { float f; memcpy(&f, &b, 4); return f; }
static uint32_t bits_from_f32(float f) { uint32_t b; memcpy(&b, &f, 4); return b; }

uint16_t po_oracle_bf16_from_f32(float x)
{
    uint32_t b = bits_from_f32(x);
    if (x != x)                                   /* NaN: keep sign, make quiet */
        return (uint16_t)((b >> 16) | 0x0040u);
    if (isinf(x))
        return (uint16_t)(b >> 16);
    uint32_t lo_bits = b & 0xFFFF0000u;           /* toward zero             */
    uint32_t hi_bits = lo_bits + 0x00010000u;     /* next magnitude          */
    double ax = fabs((double)x);
    double lo = fabs((double)f32_from_bits(lo_bits));
    /* hi may be the pattern of infinity; its value as a rounding neighbour is
     * 2^128, the next power of two above the largest finite bf16. */
    double hi = ((hi_bits & 0x7FFFFFFFu) == 0x7F800000u)
                    ? ldexp(1.0, 128)
                    : fabs((double)f32_from_bits(hi_bits));
    double d_lo = ax - lo, d_hi = hi - ax;        /* exact in fp64           */
    uint32_t pick;
    if (d_lo < d_hi)       pick = lo_bits;
    else if (d_hi < d_lo)  pick = hi_bits;
    else                   pick = ((lo_bits >> 16) & 1u) ? hi_bits : lo_bits;
    return (uint16_t)(pick >> 16);
}

void po_oracle_bf16_from_f32_array(const float* x, uint16_t* out, long long n)
{
    for (long long i = 0; i < n; ++i) out[i] = po_oracle_bf16_from_f32(x[i]);
}

/* ---- paper Eq. 4: version difference of stage `rank` in a depth-D pipeline */
int po_oracle_version_difference(int D, int rank) { return D - rank - 1; }

/* ---- one element ----------------------------------------------------------
 * beta1/beta2 double as SGDM's momentum u and dampening tau. */
static void one_element(int opt, double lr, double beta1, double beta2, double eps,
                        double wd, int decay_in_prediction, long long t, int s,
                        double W, double g, double m, double v,
                        double* W_new, double* m_new, double* v_new, double* What)
{
    double dW_step, dW_pred;                      /* dW_t as used by Eq. 1 and by Eq. 5 */
    if (opt == PO_ORACLE_SGDM) {
        double u = beta1, tau = beta2;
        double gt = g + wd * W;                   /* coupled L2                 */
        double mt = u * m + (1.0 - tau) * gt;     /* Table 1, SGDM row          */
        *m_new = mt;
        *v_new = v;                               /* SGDM has no second state   */
        dW_step = dW_pred = mt;
    } else if (opt == PO_ORACLE_NESTEROV) {
        /* momentum SGD with Nesterov's look-ahead: the buffer takes the gradient, the step takes the
         * gradient plus u times the updated buffer */
        double u = beta1;
        double gt = g + wd * W;
        double mt = u * m + gt;
        *m_new = mt;
        *v_new = v;
        dW_step = dW_pred = gt + u * mt;
    } else if (opt == PO_ORACLE_RMSPROP || opt == PO_ORACLE_ADAGRAD) {
        /* RMSprop: running average of squared gradients with smoothing alpha (= beta2), no momentum,
         * not centred.  Adagrad: their plain sum.  The step divides the gradient by the root. */
        double alpha = beta2;
        double gt = g + wd * W;
        double vt = (opt == PO_ORACLE_RMSPROP) ? alpha * v + (1.0 - alpha) * gt * gt : v + gt * gt;
        *m_new = m;
        *v_new = vt;
        dW_step = dW_pred = gt / (sqrt(vt) + eps);
    } else {
        double gt = (opt == PO_ORACLE_ADAM) ? g + wd * W : g;
        double mt = beta1 * m + (1.0 - beta1) * gt;            /* Table 1 */
        double vt = beta2 * v + (1.0 - beta2) * gt * gt;
        double mhat = mt / (1.0 - pow(beta1, (double)t));
        double vhat = vt / (1.0 - pow(beta2, (double)t));
        double r = mhat / (sqrt(vhat) + eps);
        *m_new = mt;
        *v_new = vt;
        if (opt == PO_ORACLE_ADAMW) {
            dW_step = r + wd * W;                 /* decoupled decay            */
            dW_pred = decay_in_prediction ? dW_step : r;
        } else {
            dW_step = dW_pred = r;
        }
    }
    *W_new = W - lr * dW_step;                    /* Eq. 1, first line          */
    if (s == 0) *What = W;                        /* last stage: W_t itself     */
    else        *What = W - lr * (double)s * dW_pred;          /* Eq. 5   */
}

/*
 * Host pointers, n elements each.  v / v_out may be NULL for the optimizers without a second-moment
 * state (SGDM, Nesterov), m / m_out for those without a momentum buffer (RMSprop, Adagrad).  Any of the
 * output pointers may be NULL (that output is skipped).  Outputs may alias the
 * matching inputs (element i is read before element i is written).
 * nthreads > 1 splits the element loop over that many OpenMP threads; it
 * changes no arithmetic.  Returns 0, or -1 on an invalid argument.
 */
int po_oracle_step_predict(int opt, double lr, double beta1, double beta2, double eps,
                           double weight_decay, int decay_in_prediction,
                           long long t, int s, long long n,
                           const float* W, const float* g, const float* m, const float* v,
                           float* W_out, float* m_out, float* v_out,
                           float* What_f32, uint16_t* What_bf16, int nthreads)
{
    if (opt < PO_ORACLE_SGDM || opt > PO_ORACLE_ADAGRAD) return -1;
    if (t < 1 || s < 0 || n < 0) return -1;
    const int uses_m = (opt != PO_ORACLE_RMSPROP && opt != PO_ORACLE_ADAGRAD);
    const int uses_v = (opt != PO_ORACLE_SGDM && opt != PO_ORACLE_NESTEROV);
    if (n > 0 && (!W || !g)) return -1;
    if (n > 0 && uses_m && !m) return -1;
    if (n > 0 && uses_v && !v) return -1;
    if (nthreads < 1) nthreads = 1;

    #pragma omp parallel for num_threads(nthreads) schedule(static) if (nthreads > 1)
    for (long long i = 0; i < n; ++i) {
        double Wn, mn, vn, Wh;
        one_element(opt, lr, beta1, beta2, eps, weight_decay, decay_in_prediction, t, s,
                    (double)W[i], (double)g[i], m ? (double)m[i] : 0.0, v ? (double)v[i] : 0.0,
                    &Wn, &mn, &vn, &Wh);
        float Wh32 = (float)Wh;                   /* one rounding, fp64 -> fp32 */
        if (What_f32)  What_f32[i]  = Wh32;
        if (What_bf16) What_bf16[i] = po_oracle_bf16_from_f32(Wh32);
        if (W_out) W_out[i] = (float)Wn;
        if (m_out && uses_m) m_out[i] = (float)mn;
        if (v_out && uses_v) v_out[i] = (float)vn;
    }
    return 0;
}

/*
 * Prediction alone, from the cached optimizer state (paper Algorithm 1 computes
 * dW_t from Table 1's row for the optimizer in use and applies Eq. 5 ahead of the forward pass; the
 * state was produced by the optimizer step of iteration t).  No gradient is
 * read and nothing but What is written:
 *     SGDM : dW = m
 *     Adam : dW = (m/(1-b1^t)) / (sqrt(v/(1-b2^t)) + eps)      (m, v as stored)
 *     AdamW: dW = that + wd*W   (r alone if !decay_in_prediction)
 *     What = W - lr*s*dW  (Eq. 5);  s == 0: What = W
 * With SGDM and the momentum of the previous step this is also SpecTrain's
 * predictor What = W_t - lr*s*m_{t-1} (paper Eq. 6, first line).
 * Host pointers; v may be NULL for SGDM; either output may be NULL.
 */
int po_oracle_predict(int opt, double lr, double beta1, double beta2, double eps,
                      double weight_decay, int decay_in_prediction,
                      long long t, int s, long long n,
                      const float* W, const float* m, const float* v,
                      float* What_f32, uint16_t* What_bf16, int nthreads)
{
    if (opt < PO_ORACLE_SGDM || opt > PO_ORACLE_ADAMW) return -1;   /* the others need the gradient for dW */
    if (t < 1 || s < 0 || n < 0) return -1;
    if (n > 0 && (!W || !m)) return -1;
    if (n > 0 && opt != PO_ORACLE_SGDM && !v) return -1;
    if (nthreads < 1) nthreads = 1;

    #pragma omp parallel for num_threads(nthreads) schedule(static) if (nthreads > 1)
    for (long long i = 0; i < n; ++i) {
        double Wi = (double)W[i], dW;
        if (opt == PO_ORACLE_SGDM) {
            dW = (double)m[i];
        } else {
            double mhat = (double)m[i] / (1.0 - pow(beta1, (double)t));
            double vhat = (double)v[i] / (1.0 - pow(beta2, (double)t));
            dW = mhat / (sqrt(vhat) + eps);
            if (opt == PO_ORACLE_ADAMW && decay_in_prediction) dW += weight_decay * Wi;
        }
        double Wh = (s == 0) ? Wi : Wi - lr * (double)s * dW;
        float Wh32 = (float)Wh;
        if (What_f32)  What_f32[i]  = Wh32;
        if (What_bf16) What_bf16[i] = po_oracle_bf16_from_f32(Wh32);
    }
    return 0;
}
