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
 * library routines, hand-computed Nesterov rounds, the lazy-start synchronisation
 * returning the model bit for bit for every group count, its momentum against the
 * exactly rounded difference and the telescoping sum, the schedule constants the
 * paper prints (tests/golden/schedules.txt).  Every function here has a pin.
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
 * Synchronisation in the lazy-start phase (Algorithm 1, the t mod r = 0 branch).
 * The algorithm is stated for ONE model, trained in ordinary synchronised data
 * parallelism; the sub-groups only come into being afterwards (Algorithm 2,
 * second statement).  With theta_t that model and a = theta_{t-r}:
 *
 *   delta = theta_t - a
 *   M <- mu M + delta
 *   a <- theta_t          (the next synchronisation's theta_{t-r})
 *
 * and the model itself is not touched ("only accumulates the momentum without
 * applying it", section "Momentum Warmup").  A caller that already keeps G
 * copies of the model in this phase keeps them identical, so the model is read
 * from copy 0; nothing is averaged, because no sum of G equal floats followed
 * by a division returns the float itself once G is 3, 5, 6, 7, ...
 * ---------------------------------------------------------------------- */
static void lazy_start_sync(const float* model, float* a, float* M, int64_t n, float mu)
{
    for (int64_t i = 0; i < n; ++i) {
        float delta = model[i] - a[i];
        M[i] = mu * M[i] + delta;
        a[i] = model[i];
    }
}

/* ------------------------------------------------------------------------
 * Outer step of the Pier phase (Algorithm 2, the else-branch).  theta[g] is
 * group g's current model, a the model at the previous synchronisation
 * (theta_{t-r}), M the outer momentum.
 *
 *   delta = mean over groups of (theta_g - a)      [difference, then the
 *                                                   all-reduce, as a mean]
 *   M <- mu M + delta
 *   theta <- a + lr (mu M + delta); written to a and to every group (all
 *   groups hold the same model afterwards)
 *
 * Summation over groups runs g = 0, 1, ..., G-1.
 * ---------------------------------------------------------------------- */
static void pier_sync(float* const* theta, int G, float* a, float* M, int64_t n,
                      float mu, float lr)
{
    float invG = 1.0f / (float)G;
    for (int64_t i = 0; i < n; ++i) {
        float s = 0.0f;
        for (int g = 0; g < G; ++g) s = s + (theta[g][i] - a[i]);
        float d = s * invG;
        float Mn = mu * M[i] + d;
        M[i] = Mn;
        float x = a[i] + lr * (mu * Mn + d);
        a[i] = x;
        for (int g = 0; g < G; ++g) theta[g][i] = x;
    }
}

/* phase 1: Pier's outer step; phase 0: the lazy-start synchronisation (lr unused). */
void pier_oracle_outer(float* const* theta, int G, float* a, float* M, int64_t n,
                       float mu, float lr, int phase)
{
    if (phase == 1) pier_sync(theta, G, a, M, n, mu, lr);
    else lazy_start_sync(theta[0], a, M, n, mu);
}

/* ------------------------------------------------------------------------
 * Schedules.  T = total training iterations, t = current iteration.
 *
 * The paper gives every breakpoint as a share of training: 10 %, 15 %, 20 %,
 * 80 %.  They are kept here as the fractions 1/10, 3/20, 1/5, 4/5, and "t has
 * reached the share num/den of T" is decided exactly, by cross-multiplying
 * integers; 0.15 T is never formed.
 * ---------------------------------------------------------------------- */
typedef struct { int64_t num, den; } share;
static const share k10pct = {1, 10}, k15pct = {3, 20}, k20pct = {1, 5}, k80pct = {4, 5};

/* t/T >= num/den ? */
static int reached(int64_t t, int64_t T, share s)
{
    return t * s.den >= s.num * T;
}

/* t/T > num/den ? */
static int passed(int64_t t, int64_t T, share s)
{
    return t * s.den > s.num * T;
}

/* Lazy-start phase covers the first 10% (section "Momentum Decay"):
 * iterations 1..0.1T accumulate momentum only (Algorithm 1's loop bound is
 * inclusive, so t/T = 1/10 itself still belongs to it); the first applied outer
 * step is the first one after 0.1T. */
int pier_oracle_phase(int64_t t, int64_t T)
{
    return passed(t, T, k10pct) ? 1 : 0;
}

/* Algorithm 2's three-way choice: 0.99 on [10%, 15%), 0.95 on [15%, 20%), 0.9
 * otherwise.  (Below 10% that "otherwise" equals the warmup default of 0.9 given
 * with Algorithm 1.)  Walked from the last band to the first. */
float pier_oracle_mu(int64_t t, int64_t T)
{
    if (reached(t, T, k20pct)) return 0.9f;
    if (reached(t, T, k15pct)) return 0.95f;
    if (reached(t, T, k10pct)) return 0.99f;
    return 0.9f;
}

/* Outer learning rate (section "Implementation"): linear from 0 to 1 between
 * 10% and 20% of training, 1.1 from 20% to 80%, 0.9 for the last 20%.
 * Before 10% no outer step is applied; 0 is returned there.  On the ramp the
 * value is (t - T/10) / (T/5 - T/10) = (10 t - T) / T, an exact ratio of
 * integers rounded once to double and once to fp32. */
float pier_oracle_outer_lr(int64_t t, int64_t T)
{
    if (reached(t, T, k80pct)) return 0.9f;
    if (reached(t, T, k20pct)) return 1.1f;
    if (!reached(t, T, k10pct)) return 0.0f;
    int64_t above = 10 * t - T;            /* ten times the distance from the 10% mark */
    return (float)((double)above / (double)T);
}

/* Inner learning rate (Table I: cosine decay style, learning rate warmup proportion 2%,
 * a minimum learning rate, decay iterations = training iterations).  Two legs:
 *   warmup, t <= W = warmup_frac T:  the share t / W of lr_max (so iteration 1 already
 *                                    moves, and t = W uses lr_max itself);
 *   decay,  W < t < T:               lr_min plus the share (1 + cos(pi x)) / 2 of the span
 *                                    lr_max - lr_min, x = (t - W) / (T - W) the progress
 *                                    through the decay leg; lr_min from T on.
 * Evaluated in double, rounded once to fp32. */
static double cosine_share(double progress)
{
    const double pi = 3.14159265358979323846;
    return 0.5 * (cos(pi * progress) + 1.0);
}

float pier_oracle_inner_lr(int64_t t, int64_t T, float lr_max, float lr_min, double warmup_frac)
{
    double hi = (double)lr_max, lo = (double)lr_min;
    double W = warmup_frac * (double)T;
    int in_warmup = W > 0.0 && (double)t <= W;
    if (in_warmup) return (float)(hi * (double)t / W);
    if (t >= T) return lr_min;
    double progress = ((double)t - W) / ((double)T - W);
    return (float)(lo + cosine_share(progress) * (hi - lo));
}

/* The momentum coefficient and rate one synchronisation at iteration t uses:
 * in the lazy-start phase mu is Algorithm 1's default 0.9 and no rate applies. */
void pier_oracle_outer_scalars(int64_t t, int64_t T, int* phase, float* mu, float* lr)
{
    *phase = pier_oracle_phase(t, T);
    if (*phase == 0) { *mu = 0.9f; *lr = 0.0f; }
    else { *mu = pier_oracle_mu(t, T); *lr = pier_oracle_outer_lr(t, T); }
}
