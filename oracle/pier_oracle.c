/*
 * CPU oracle for the optimizer arithmetic of Pier's two-level optimizer.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, single-threaded
 * statement of what the GPU library must compute.  It shares no code, header,
 * table or helper with the HIP path, and nothing in the product may call it.
 *
 * Arithmetic: every operation is an IEEE-754 binary32 operation in the order
 * written (the paper keeps optimizer state and arithmetic in FP32, section
 * "Experiments", first paragraph).  Build with
 *     gcc -O2 -ffp-contract=off -fno-fast-math -shared -fPIC
 * so that no product is fused into an FMA and nothing is reassociated.  The
 * only double-precision work is the host-side scalar preparation (bias
 * corrections, schedule ramp), exactly as a caller would do it.
 *
 * Pins (tests/test_oracle_pins.py): step-1 and constant-gradient closed forms,
 * torch.optim.AdamW and torch.optim.SGD(nesterov=True) on CPU as independent
 * library routines, hand-computed Nesterov rounds, warmup telescoping, the
 * schedule constants the paper prints (tests/golden/schedules.txt).
 */
#include <math.h>
#include <stdint.h>
#include <string.h>

/* ------------------------------------------------------------------------
 * Inner optimizer: AdamW with decoupled weight decay and bias correction.
 * The paper names the optimizer (Algorithm 1, "OptimizerUpdate"; section
 * "Implementation": AdamW inside each group; Table I: beta1, beta2, weight
 * decay) without printing its formula, so the textbook rule is used:
 *     m <- b1 m + (1-b1) g          v <- b2 v + (1-b2) g^2
 *     mhat = m / (1-b1^t)           vhat = v / (1-b2^t)
 *     theta <- theta - lr * ( mhat / (sqrt(vhat) + eps) + wd * theta )
 * eps sits outside the root, after bias correction; the decay term uses the
 * parameter value from before the step.
 * ---------------------------------------------------------------------- */
static void adamw_scalars(float beta1, float beta2, int64_t step,
                          float* bc1, float* bc2)
{
    *bc1 = (float)(1.0 - pow((double)beta1, (double)step));
    *bc2 = (float)(1.0 - pow((double)beta2, (double)step));
}

static inline void adamw_one(float* p, float* m, float* v, float g,
                             float lr, float beta1, float beta2, float eps,
                             float wd, float bc1, float bc2, float grad_scale)
{
    float om1 = 1.0f - beta1;
    float om2 = 1.0f - beta2;
    if (grad_scale != 1.0f) g = g * grad_scale;
    float mn = beta1 * (*m) + om1 * g;
    float vn = beta2 * (*v) + (om2 * g) * g;
    float mh = mn / bc1;
    float vh = vn / bc2;
    float u = mh / (sqrtf(vh) + eps) + wd * (*p);
    *p = *p - lr * u;
    *m = mn;
    *v = vn;
}

void pier_oracle_adamw(float* p, float* m, float* v, const float* g, int64_t n,
                       float lr, float beta1, float beta2, float eps, float wd,
                       int64_t step, float grad_scale)
{
    float bc1, bc2;
    adamw_scalars(beta1, beta2, step, &bc1, &bc2);
    for (int64_t i = 0; i < n; ++i)
        adamw_one(&p[i], &m[i], &v[i], g[i], lr, beta1, beta2, eps, wd, bc1, bc2,
                  grad_scale);
}

/* bfloat16 gradients: the 16 stored bits are the top half of a binary32, so
 * widening is exact. */
void pier_oracle_adamw_bf16(float* p, float* m, float* v, const uint16_t* g,
                            int64_t n, float lr, float beta1, float beta2,
                            float eps, float wd, int64_t step, float grad_scale)
{
    float bc1, bc2;
    adamw_scalars(beta1, beta2, step, &bc1, &bc2);
    for (int64_t i = 0; i < n; ++i) {
        uint32_t bits = (uint32_t)g[i] << 16;
        float gf;
        memcpy(&gf, &bits, sizeof gf);
        adamw_one(&p[i], &m[i], &v[i], gf, lr, beta1, beta2, eps, wd, bc1, bc2,
                  grad_scale);
    }
}

/* ------------------------------------------------------------------------
 * Global-norm gradient clipping (Table I: "clip grad 1").  The paper gives the
 * threshold only; the rule is the standard one of the framework it builds on:
 * total L2 norm over every gradient element of the model, coefficient
 * max_norm / (norm + 1e-6), applied only when it is below 1.  The sum of squares
 * is accumulated in double, element by element in list order; the coefficient is
 * formed in double and rounded once to fp32 (it becomes the inner step's
 * grad_scale).
 * ---------------------------------------------------------------------- */
double pier_oracle_sumsq(const float* g, int64_t n, double acc)
{
    for (int64_t i = 0; i < n; ++i) acc = acc + (double)g[i] * (double)g[i];
    return acc;
}

double pier_oracle_sumsq_bf16(const uint16_t* g, int64_t n, double acc)
{
    for (int64_t i = 0; i < n; ++i) {
        uint32_t bits = (uint32_t)g[i] << 16;
        float gf;
        memcpy(&gf, &bits, sizeof gf);
        acc = acc + (double)gf * (double)gf;
    }
    return acc;
}

float pier_oracle_clip_coef(double sumsq, float max_norm)
{
    double coef = (double)max_norm / (sqrt(sumsq) + 1e-6);
    return coef < 1.0 ? (float)coef : 1.0f;
}

/* ------------------------------------------------------------------------
 * BF16 model weights beside the FP32 optimizer copy (section "Experiments": BF16
 * in models, FP32 in optimizers): after an update the working weight is the fp32
 * value rounded to bfloat16, round to nearest, ties to even; NaN becomes the
 * quiet NaN 0x7FC0.
 * ---------------------------------------------------------------------- */
void pier_oracle_to_bf16(const float* x, uint16_t* out, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) {
        uint32_t b;
        memcpy(&b, &x[i], sizeof b);
        if ((b & 0x7FFFFFFFu) > 0x7F800000u) { out[i] = 0x7FC0; continue; }
        uint32_t lsb = (b >> 16) & 1u;
        out[i] = (uint16_t)((b + 0x7FFFu + lsb) >> 16);
    }
}

/* ------------------------------------------------------------------------
 * Outer step (Algorithm 2, the else-branch; Algorithm 1, the t mod r = 0
 * branch).  theta[g] is group g's current model, a the model at the previous
 * synchronisation (theta_{t-r}), M the outer momentum.
 *
 *   delta = mean over groups of (theta_g - a)      [difference, then the
 *                                                   all-reduce, as a mean]
 *   M <- mu M + delta
 *   phase 1 (Pier):   theta <- a + lr (mu M + delta); written to a and to
 *                     every group (all groups hold the same model afterwards)
 *   phase 0 (warmup): momentum only; a <- current model (mean of the
 *                     groups, which are identical in this phase); the groups'
 *                     models are not touched.
 * Summation over groups runs g = 0, 1, ..., G-1.
 * ---------------------------------------------------------------------- */
void pier_oracle_outer(float* const* theta, int G, float* a, float* M, int64_t n,
                       float mu, float lr, int phase)
{
    float invG = 1.0f / (float)G;
    for (int64_t i = 0; i < n; ++i) {
        float s = 0.0f;
        for (int g = 0; g < G; ++g) s = s + (theta[g][i] - a[i]);
        float d = s * invG;
        float Mn = mu * M[i] + d;
        M[i] = Mn;
        if (phase == 1) {
            float x = a[i] + lr * (mu * Mn + d);
            a[i] = x;
            for (int g = 0; g < G; ++g) theta[g][i] = x;
        } else {
            float s2 = 0.0f;
            for (int g = 0; g < G; ++g) s2 = s2 + theta[g][i];
            a[i] = s2 * invG;
        }
    }
}

/* ------------------------------------------------------------------------
 * Schedules.  T = total training iterations, t = current iteration.
 * Breakpoints are compared in integers (10 t vs T, 100 t vs 15 T, ...), so
 * that 0.15 T never goes through a rounded product.
 * ---------------------------------------------------------------------- */

/* Lazy-start phase covers the first 10% (section "Momentum Decay"):
 * iterations 1..0.1T accumulate momentum only (Algorithm 1's loop bound is
 * inclusive); the first applied outer step is the first one after 0.1T. */
int pier_oracle_phase(int64_t t, int64_t T)
{
    return (10 * t <= T) ? 0 : 1;
}

/* Algorithm 2's three-way choice, literally: 0.99 on [0.1T, 0.15T), 0.95 on
 * [0.15T, 0.2T), 0.9 otherwise.  (Below 0.1T that "otherwise" equals the
 * warmup default of 0.9 given with Algorithm 1.) */
float pier_oracle_mu(int64_t t, int64_t T)
{
    if (10 * t >= T && 100 * t < 15 * T) return 0.99f;
    if (100 * t >= 15 * T && 10 * t < 2 * T) return 0.95f;
    return 0.9f;
}

/* Outer learning rate (section "Implementation"): linear from 0 to 1 between
 * 10% and 20% of training, 1.1 from 20% to 80%, 0.9 for the last 20%.
 * Before 10% no outer step is applied; 0 is returned there. */
float pier_oracle_outer_lr(int64_t t, int64_t T)
{
    if (10 * t < T) return 0.0f;
    if (10 * t < 2 * T) return (float)((double)(10 * t - T) / (double)T);
    if (10 * t < 8 * T) return 1.1f;
    return 0.9f;
}

/* Inner learning rate (Table I: cosine decay style, learning rate warmup proportion 2%,
 * a minimum learning rate, decay iterations = training iterations): linear from 0 to
 * lr_max over the first warmup_frac * T iterations (iteration t uses lr_max * t / W,
 * W = warmup_frac * T), then half a cosine from lr_max at t = W down to lr_min at
 * t = T.  Evaluated in double, rounded once to fp32. */
float pier_oracle_inner_lr(int64_t t, int64_t T, float lr_max, float lr_min, double warmup_frac)
{
    const double pi = 3.14159265358979323846;
    double W = warmup_frac * (double)T;
    if (W > 0.0 && (double)t <= W) return (float)((double)lr_max * (double)t / W);
    if (t >= T) return lr_min;
    double ratio = ((double)t - W) / ((double)T - W);
    double coeff = 0.5 * (cos(pi * ratio) + 1.0);
    return (float)((double)lr_min + coeff * ((double)lr_max - (double)lr_min));
}

/* The momentum coefficient and rate one synchronisation at iteration t uses:
 * in the lazy-start phase mu is Algorithm 1's default 0.9 and no rate applies. */
void pier_oracle_outer_scalars(int64_t t, int64_t T, int* phase, float* mu, float* lr)
{
    *phase = pier_oracle_phase(t, T);
    if (*phase == 0) { *mu = 0.9f; *lr = 0.0f; }
    else { *mu = pier_oracle_mu(t, T); *lr = pier_oracle_outer_lr(t, T); }
}
