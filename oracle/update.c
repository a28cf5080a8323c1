/*
 * CPU oracle, part 2: the arithmetic of the update stage.
 *
 * TEST INFRASTRUCTURE ONLY - never linked into, loaded by or called from the
 * product library.  Plain loops, one element at a time, no blocking or fusion
 * beyond what each definition states.  Build: gcc -O2 -fno-fast-math
 * -ffp-contract=off (so no multiply-add is ever fused) -fopenmp.  OpenMP only
 * splits the element range; the operations applied to one element, and their
 * order, do not depend on the thread count.
 *
 * What is computed: the per-rank arithmetic of the Update stage of PaRO-IGG /
 * IIG / NIG (paper Sec. 3.2) - Adam on the rank's own shard from the summed
 * gradients, new parameters out in 16 bits - with the memory model of Sec. 3.1.2
 * (2 bytes/param gradients and parameters, 12 bytes/param of Adam state = fp32
 * master copy + two moments):
 *
 *   fold   g[e]  = sum over the P ranks' contributions, added in the order the
 *                  reduce-scatter ring delivers them (Sec. 3.4), in fp32;
 *   sumsq  S     = sum_e g[e]^2 in fp64;
 *   clip   coef  = min(1, max_norm / (grad_scale * sqrt(S_total) + 1e-6));
 *                  not in the paper - the convention of the usual global-norm
 *                  clipping routine;  PARITY UNPINNED by the paper, pinned to
 *                  torch.nn.utils.clip_grad_norm_ in the tests;
 *   adam   Adam (Kingma & Ba, Algorithm 1) with bias correction, decoupled
 *          weight decay by default, classic L2 as an option;
 *   pack   bf16 round-to-nearest-even of the updated master parameter.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

static inline float bf16_to_f32(uint16_t h) {
    uint32_t u = (uint32_t)h << 16;          /* bf16 is the top half of an fp32: exact */
    float f;
    memcpy(&f, &u, 4);
    return f;
}

/* ---- fold ----------------------------------------------------------------
 * src[k], k = 0..P-1, are the contributions ALREADY LISTED IN FOLD ORDER.
 * Consecutive runs of group_len sources are added left to right into a group
 * partial A; the partials are added left to right into X.  group_len == P is
 * the flat ring.  No add with a zero start value is made (it would turn -0
 * into +0). */
void orc_fold_bf16(const uint16_t *const *src, int P, int group_len, int64_t n, float *out) {
#pragma omp parallel for schedule(static)
    for (int64_t e = 0; e < n; e++) {
        float X = 0.0f;
        for (int k0 = 0; k0 < P; k0 += group_len) {
            float A = bf16_to_f32(src[k0][e]);
            for (int l = 1; l < group_len; l++) A = A + bf16_to_f32(src[k0 + l][e]);
            X = (k0 == 0) ? A : X + A;
        }
        out[e] = X;
    }
}

void orc_fold_f32(const float *const *src, int P, int group_len, int64_t n, float *out) {
#pragma omp parallel for schedule(static)
    for (int64_t e = 0; e < n; e++) {
        float X = 0.0f;
        for (int k0 = 0; k0 < P; k0 += group_len) {
            float A = src[k0][e];
            for (int l = 1; l < group_len; l++) A = A + src[k0 + l][e];
            X = (k0 == 0) ? A : X + A;
        }
        out[e] = X;
    }
}

/* ---- sum of squares --------------------------------------------------------
 * fp64; each square of an fp32 value is exact in fp64.  Elements are summed in
 * index order inside blocks of 65536, block sums in block order. */
#define ORC_BLOCK 65536
double orc_sumsq(const float *g, int64_t n) {
    int64_t nb = (n + ORC_BLOCK - 1) / ORC_BLOCK;
    if (nb <= 0) return 0.0;
    double *part = (double *)malloc((size_t)nb * sizeof(double));
    if (!part) return NAN;
#pragma omp parallel for schedule(static)
    for (int64_t b = 0; b < nb; b++) {
        int64_t lo = b * ORC_BLOCK, hi = lo + ORC_BLOCK < n ? lo + ORC_BLOCK : n;
        double s = 0.0;
        for (int64_t e = lo; e < hi; e++) s += (double)g[e] * (double)g[e];
        part[b] = s;
    }
    double tot = 0.0;
    for (int64_t b = 0; b < nb; b++) tot += part[b];
    free(part);
    return tot;
}

/* ---- clip coefficient ------------------------------------------------------ */
double orc_clip_coef(double total_sumsq, float grad_scale, float max_norm) {
    if (!(max_norm > 0.0f)) return 1.0;
    double norm = (double)grad_scale * sqrt(total_sumsq);
    double c = (double)max_norm / (norm + 1e-6);
    return c < 1.0 ? c : 1.0;
}

/* ---- Adam, reference: fp64 arithmetic on the fp32 inputs, rounded once ------
 * gh = sc*g; [L2: gh += wd*p]; m = b1*m + (1-b1)*gh; v = b2*v + (1-b2)*gh^2;
 * p = p*(1 - lr*wd) - (lr / (1-b1^t)) * m / (sqrt(v)/sqrt(1-b2^t) + eps)
 * sc = grad_scale * coef is passed in as a double. */
void orc_adam64(int64_t n, const float *g, float *p, float *m, float *v, double sc, float lr,
                float beta1, float beta2, float eps, float wd, int step, int adamw) {
    const double b1 = beta1, b2 = beta2, lrd = lr, epsd = eps, wdd = wd;
    const double bc1 = 1.0 - pow(b1, (double)step), bc2 = 1.0 - pow(b2, (double)step);
#pragma omp parallel for schedule(static)
    for (int64_t e = 0; e < n; e++) {
        double gh = sc * (double)g[e], pe = p[e];
        if (!adamw) gh += wdd * pe;
        double me = b1 * (double)m[e] + (1.0 - b1) * gh;
        double ve = b2 * (double)v[e] + (1.0 - b2) * gh * gh;
        double upd = (lrd / bc1) * me / (sqrt(ve) / sqrt(bc2) + epsd);
        pe = adamw ? pe * (1.0 - lrd * wdd) - upd : pe - upd;
        m[e] = (float)me;
        v[e] = (float)ve;
        p[e] = (float)pe;
    }
}

/* ---- Adam, all in fp32: the same formulas with every operation rounded to fp32 ------
 * C evaluates a float expression operation by operation in float (FLT_EVAL_METHOD 0 on this
 * target) and the build forbids fusing a multiply into an add, so each line below is the
 * sequence of IEEE fp32 operations it spells: scale; [L2 term;] the two moving averages;
 * square root, division by sqrt(1 - b2^t), + eps; division; times lr / (1 - b1^t); decay and
 * subtraction.  Scalars that do not depend on the element are formed in fp64 from the fp32
 * hyper-parameters and rounded to fp32 once. */
void orc_adam32(int64_t n, const float *g, float *p, float *m, float *v, double sc_d, float lr,
                float beta1, float beta2, float eps, float wd, int step, int adamw) {
    const float sc = (float)sc_d;
    const float one_minus_b1 = (float)(1.0 - (double)beta1), one_minus_b2 = (float)(1.0 - (double)beta2);
    const float bias1 = (float)(1.0 - pow((double)beta1, (double)step));
    const float bias2 = (float)(1.0 - pow((double)beta2, (double)step));
    const float lr_over_bias1 = (float)((double)lr / (double)bias1);
    const float root_bias2 = (float)sqrt((double)bias2);
    const float keep = (float)(1.0 - (double)lr * (double)wd);
#pragma omp parallel for schedule(static)
    for (int64_t e = 0; e < n; e++) {
        float grad = sc * g[e];
        if (!adamw) grad = grad + wd * p[e];
        const float m_new = beta1 * m[e] + one_minus_b1 * grad;
        const float v_new = beta2 * v[e] + one_minus_b2 * (grad * grad);
        const float step_e = lr_over_bias1 * (m_new / (sqrtf(v_new) / root_bias2 + eps));
        p[e] = adamw ? p[e] * keep - step_e : p[e] - step_e;
        m[e] = m_new;
        v[e] = v_new;
    }
}

/* ---- pack: fp32 -> bf16, round to nearest, ties to even ---------------------
 * NaN stays NaN (quiet bit set, sign kept); infinities are kept. */
void orc_bf16_rne(const float *p, int64_t n, uint16_t *out) {
#pragma omp parallel for schedule(static)
    for (int64_t e = 0; e < n; e++) {
        uint32_t u;
        memcpy(&u, &p[e], 4);
        if ((u & 0x7FFFFFFFu) > 0x7F800000u) {
            out[e] = (uint16_t)((u >> 16) | 0x0040u);
        } else {
            uint32_t keep_lsb = (u >> 16) & 1u;
            out[e] = (uint16_t)((u + 0x7FFFu + keep_lsb) >> 16);
        }
    }
}

/* ---- pack: fp32 -> fp16 (binary16), round to nearest, ties to even ----------
 * The IEEE definition written out on the bit fields: a value is
 * 2^(E-127) * S / 2^23 with the 24-bit significand S (hidden bit included);
 * binary16 keeps 11 significand bits down to exponent -14 and fewer below it
 * (gradual underflow), so S loses 13 bits, or more for a subnormal result; the
 * dropped bits decide the rounding; a carry out of the significand moves into
 * the exponent by plain addition; anything at or beyond 65520 becomes infinity.
 * NaN becomes a quiet NaN of the same sign (its payload is not kept). */
static uint16_t f16_rne_one(uint32_t u) {
    const uint32_t sign = (u >> 16) & 0x8000u, a = u & 0x7FFFFFFFu;
    if (a > 0x7F800000u) return (uint16_t)(sign | 0x7E00u);
    const int E = (int)(a >> 23);
    if (E == 0) return (uint16_t)sign;                 /* fp32 subnormals are far below half of the smallest binary16 */
    const int e = E - 127;
    if (e > 15) return (uint16_t)(sign | 0x7C00u);     /* includes infinity */
    const uint32_t S = (a & 0x7FFFFFu) | 0x800000u;
    int drop = 13;
    if (e < -14) drop += -14 - e;                      /* subnormal result: fewer bits survive */
    if (drop > 25) return (uint16_t)sign;              /* below half of the smallest subnormal */
    uint32_t q = S >> drop;
    const uint32_t rem = S & ((1u << drop) - 1u), half = 1u << (drop - 1);
    if (rem > half || (rem == half && (q & 1u))) q++;
    /* normal: q in [0x400, 0x800]; exponent field e+15 with the hidden bit of q counted once */
    uint32_t h = e < -14 ? q : ((uint32_t)(e + 14) << 10) + q;
    if (h > 0x7C00u) h = 0x7C00u;
    return (uint16_t)(sign | h);
}

void orc_f16_rne(const float *p, int64_t n, uint16_t *out) {
#pragma omp parallel for schedule(static)
    for (int64_t e = 0; e < n; e++) {
        uint32_t u;
        memcpy(&u, &p[e], 4);
        out[e] = f16_rne_one(u);
    }
}

int orc_max_threads(void) {
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void orc_set_threads(int n) {
#ifdef _OPENMP
    extern void omp_set_num_threads(int);
    omp_set_num_threads(n);
#else
    (void)n;
#endif
}
