/*
 * einsum_ref: CPU oracle for one extended Einstein-summation vertex.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the parity reference for the HIP
 * library; it shares no code with it and must never be reached from the
 * product path.
 *
 * It is the general binary EinSum form of the paper (Section 3, "General form
 * of EinSum") written out as a loop nest:
 *
 *     for every l_Z in I(b_Z):
 *         Z[l_Z] = (+)_{l_agg in I(b_XY[l_agg; l_XY])}  (x)( X[l_X], Y[l_Y] )
 *
 * with the unary form (a map, optionally aggregated) of the same section when
 * Y is absent.  l_agg are the labels that occur in an input but not in the
 * output.  Inputs are read in their stored dtype and converted exactly to
 * double; (x) is evaluated in double with libm; (+) accumulates in double in
 * row-major order of l_agg; the result is rounded once to the output dtype.
 *
 * Parity unpinned (covered by tolerance only): last-ulp behaviour of libm
 * exp/log, NaN propagation in max, and bf16 ties that differ between a
 * double-accumulated and an fp32-accumulated sum.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ER_MAX_LABELS 16

enum { ER_F64 = 0, ER_F32 = 1, ER_BF16 = 2 };
enum { ER_AGG_NONE = 0, ER_AGG_SUM = 1, ER_AGG_MAX = 2 };
enum {
    ER_MUL = 0, ER_ADD, ER_SUB, ER_DIV, ER_SQDIFF, ER_ABSDIFF, ER_EXP_SUB, ER_RELU_GRAD, ER_SILU_MUL,
    ER_IDENT = 32, ER_SCALE, ER_RELU, ER_EXP, ER_LOG
};

static inline double load_as_double(const void *p, int dt, int64_t off)
{
    if (dt == ER_F64) return ((const double *)p)[off];
    if (dt == ER_F32) return (double)((const float *)p)[off];
    uint32_t bits = ((uint32_t)((const uint16_t *)p)[off]) << 16;   /* bf16 = top half of an fp32 */
    float f;
    memcpy(&f, &bits, 4);
    return (double)f;
}

/* Round a double to the nearest bf16 value (8 significant bits, fp32 exponent range), ties to even. */
double er_round_bf16(double x)
{
    if (x == 0.0 || isnan(x) || isinf(x)) return x;
    int e;
    double m = frexp(x, &e);                 /* x = m * 2^e, 0.5 <= |m| < 1 */
    int qexp = e - 8;                        /* quantum 2^(e-8) keeps 8 significant bits */
    if (qexp < -133) qexp = -133;            /* bf16 subnormal quantum: 2^-126 * 2^-7 */
    (void)m;
    double q = nearbyint(ldexp(x, -qexp));   /* default rounding mode: nearest-even */
    double r = ldexp(q, qexp);
    if (fabs(r) >= ldexp(1.0, 128)) return x > 0 ? INFINITY : -INFINITY;
    return r;
}

static inline double round_out(double v, int dt)
{
    if (dt == ER_F32) return (double)(float)v;
    if (dt == ER_BF16) return er_round_bf16(v);
    return v;
}

/* The scalar function (x): binary join functions and unary maps (Section 3). */
static inline double otimes_eval(int op, double x, double y, double alpha)
{
    switch (op) {
    case ER_MUL:       return alpha * (x * y);
    case ER_ADD:       return alpha * x + y;
    case ER_SUB:       return alpha * (x - y);
    case ER_DIV:       return x / y;
    case ER_SQDIFF:    return (x - y) * (x - y);
    case ER_ABSDIFF:   return fabs(x - y);
    case ER_EXP_SUB:   return exp(x - y);
    case ER_RELU_GRAD: return y > 0.0 ? x : 0.0;
    case ER_SILU_MUL:  return (x / (1.0 + exp(-x))) * y;
    case ER_IDENT:     return x;
    case ER_SCALE:     return alpha * x;
    case ER_RELU:      return x > 0.0 ? x : 0.0;
    case ER_EXP:       return exp(x);
    case ER_LOG:       return log(x);
    default:           return NAN;
    }
}

/*
 * n_labels : number of unique labels; bound[l] their ranges.
 * labX/labY/labZ : label id of every dimension of X / Y / Z (rankY = 0 and Y = NULL: unary).
 * strideX/strideY : element strides of X / Y per dimension.
 * Z : dense row-major over b_Z (or n_sel values when sel != NULL: only those flat Z indices).
 * Returns 0, or a negative code for a malformed request.
 */
int einsum_ref(int n_labels, const int64_t *bound,
               int rankX, const int *labX, const int64_t *strideX, const void *X, int dtX,
               int rankY, const int *labY, const int64_t *strideY, const void *Y, int dtY,
               int rankZ, const int *labZ,
               int otimes, int oplus, double alpha, int out_dt,
               double *Z, int64_t n_sel, const int64_t *sel)
{
    if (n_labels < 0 || n_labels > ER_MAX_LABELS) return -1;
    int inZ[ER_MAX_LABELS] = {0}, inXY[ER_MAX_LABELS] = {0};
    int64_t sX[ER_MAX_LABELS] = {0}, sY[ER_MAX_LABELS] = {0};
    for (int i = 0; i < rankX; i++) {
        if (labX[i] < 0 || labX[i] >= n_labels || sX[labX[i]] != 0 || (inXY[labX[i]] & 1)) return -2; /* repeated label */
        sX[labX[i]] = strideX[i]; inXY[labX[i]] |= 1;
    }
    for (int i = 0; i < rankY; i++) {
        if (labY[i] < 0 || labY[i] >= n_labels || (inXY[labY[i]] & 2)) return -2;
        sY[labY[i]] = strideY[i]; inXY[labY[i]] |= 2;
    }
    for (int i = 0; i < rankZ; i++) {
        if (labZ[i] < 0 || labZ[i] >= n_labels || inZ[labZ[i]]) return -2;
        if (!inXY[labZ[i]]) return -3;                       /* broadcast label: not handled (Section 3) */
        inZ[labZ[i]] = 1;
    }
    /* l_agg: labels of the inputs that are absent from the output, in label-id order */
    int aggLab[ER_MAX_LABELS], n_agg = 0;
    for (int l = 0; l < n_labels; l++)
        if (inXY[l] && !inZ[l]) aggLab[n_agg++] = l;
    if (n_agg > 0 && oplus == ER_AGG_NONE) return -4;

    int64_t nZ = 1;
    for (int i = 0; i < rankZ; i++) nZ *= bound[labZ[i]];
    int64_t n_aggspace = 1;
    for (int a = 0; a < n_agg; a++) n_aggspace *= bound[aggLab[a]];
    int64_t n_out = sel ? n_sel : nZ;
    int last = n_agg > 0 ? aggLab[n_agg - 1] : -1;
    int64_t last_n = n_agg > 0 ? bound[last] : 1;
    int64_t last_sx = n_agg > 0 ? sX[last] : 0, last_sy = n_agg > 0 ? sY[last] : 0;
    int64_t outer = n_agg > 0 ? n_aggspace / (last_n > 0 ? last_n : 1) : 1;

#pragma omp parallel for schedule(static)
    for (int64_t o = 0; o < n_out; o++) {
        int64_t flat = sel ? sel[o] : o;
        /* bind the output labels */
        int64_t offX = 0, offY = 0, rem = flat;
        for (int i = rankZ - 1; i >= 0; i--) {
            int l = labZ[i];
            int64_t v = rem % bound[l];
            rem /= bound[l];
            offX += v * sX[l];
            offY += v * sY[l];
        }
        double acc = (oplus == ER_AGG_MAX) ? -INFINITY : 0.0;
        if (n_agg == 0) {
            acc = otimes_eval(otimes, load_as_double(X, dtX, offX), rankY ? load_as_double(Y, dtY, offY) : 0.0, alpha);
        } else if (n_aggspace > 0) {
            int64_t idx[ER_MAX_LABELS] = {0};
            for (int64_t it = 0; it < outer; it++) {
                int64_t ox = offX, oy = offY;
                for (int a = 0; a < n_agg - 1; a++) { ox += idx[a] * sX[aggLab[a]]; oy += idx[a] * sY[aggLab[a]]; }
                for (int64_t t = 0; t < last_n; t++) {
                    double x = load_as_double(X, dtX, ox + t * last_sx);
                    double y = rankY ? load_as_double(Y, dtY, oy + t * last_sy) : 0.0;
                    double v = otimes_eval(otimes, x, y, alpha);
                    if (oplus == ER_AGG_MAX) acc = v > acc ? v : acc; else acc += v;
                }
                for (int a = n_agg - 2; a >= 0; a--) {          /* row-major odometer over the outer agg labels */
                    if (++idx[a] < bound[aggLab[a]]) break;
                    idx[a] = 0;
                }
            }
        }
        Z[o] = round_out(acc, out_dt);
    }
    return 0;
}
