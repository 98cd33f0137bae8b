/*
 * sketch_oracle.c -- plain, slow, single-threaded CPU statement of the
 * UltraSketchLLM inference path (multi-row AbsMaxMin sketch + linear layer).
 *
 * THIS IS TEST INFRASTRUCTURE.  It exists so that the GPU library can be
 * checked against something written straight from the paper.  It shares no
 * code, header, table or constant with the GPU library and must never be
 * called from a product path.  Only the test-suite, the smoke check and the
 * benchmark's "cpu_baseline" leg (and its offline sketch generator) use it.
 *
 * What follows the paper and where:
 *   select   Sec. 3.1 "AbsMaxMin Sketch Design", Eq. (3):  I_r = H_r(Addr(w))
 *   update   Sec. 3.1, Eq. (4):  S[r,I_r] <- w  iff |S[r,I_r]| > |w|;
 *            states start at +inf (Sec. 3.1, initial state of the sketch)
 *   query    Sec. 3.1, Eq. (5):  w' = Max_r S[r][H_r(Addr(w))]
 *   groups   Sec. 3.3 "Matrix-based Sketch Operator Mapping": W (d_in x d_out,
 *            row major) is cut into disjoint groups, each with its own sketch
 *            of K states per row; K may differ per group (importance).
 *   linear   Sec. 2.1, Eq. (1)/(2):  y = x W  with W of shape d_in x d_out.
 *
 * Readings taken where the paper is silent (each is listed in the design
 * notes of the repository):
 *   - Hash.  The paper asks for independent hash functions fixed by a
 *     seed and names none.  Here  t_r(a) = (A_r * a + C_r) mod 2^24  and
 *     H_r(a) = floor(t_r(a) * K / 2^24); A_r, C_r are explicit inputs.
 *   - Addr(w) is the offset of the weight inside its group: a group is a tile
 *     of tile_in x tile_out weights, a = j_local * tile_out + o_local.
 *   - "Max" in Eq. (5) is taken by magnitude (the sketch is called AbsMaxMin
 *     and is stated to under-estimate magnitudes); between two candidates of
 *     equal magnitude the one whose sign bit is clear wins.
 *     The literal reading -- Max of the signed values, as Eq. (5) is printed --
 *     is available as query mode 1 (+0 wins over -0).
 *   - Update ties (|S| == |w|) keep the older value (Eq. (4) is strict).
 *   - States that no weight ever reached are written as +0.0 at the end of
 *     the update stream (no query can reach them).
 *   - Low-bit states (Sec. 3.3, last paragraph, and Sec. 4: sketch states
 *     kept in 4-bit / 8-bit types).  The paper names a third-party scalar
 *     quantiser and gives no format.  Here: one binary16 scale per sketch
 *     row of a group, equal to the largest state magnitude of that row;
 *     codes are signed integers q in [-qmax, qmax], qmax = 127 (8 bit) or
 *     7 (4 bit); q = round-half-even(state * qmax / scale); the state a
 *     code stands for is q * scale / qmax rounded once to binary16
 *     (nearest even).  Query and linear layer then run on those states.
 *
 * Precision: weights/states are IEEE binary16 bit patterns and are never
 * rounded here; the linear layer accumulates in binary64 in ascending j.
 *
 * Parity pins (tests/test_oracle_*.py): hand-worked example, identity hash,
 * sort-based brute force of Eq. (4), one-hot matrix forms Eq. (8)/(9),
 * under-estimate / membership / row-order / more-rows invariants, the
 * bucket-minimum survival law behind Eq. (6), numpy fp64 matmul.
 * Low-bit states: exact rational arithmetic (Python fractions), error
 * bound of half a step, end points, symmetry, hand-worked codes.
 * Absolute accuracy or latency figures: parity unpinned (the paper prints
 * no value for this path).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORA_OK 0
#define ORA_BAD_ARG 1
#define ORA_NONFINITE 2

/* ---- binary16 / bfloat16 bit patterns to double (exact) ---------------- */

double ora_half_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1F;
    int m = h & 0x3FF;
    double v;
    if (e == 0)
        v = ldexp((double)m, -24);              /* zero and subnormals */
    else if (e == 31)
        v = m ? NAN : INFINITY;
    else
        v = ldexp((double)(m + 1024), e - 25);  /* (1 + m/1024) * 2^(e-15) */
    return sign ? -v : v;
}

double ora_bf16_to_double(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

static int half_is_finite(uint16_t h) { return ((h >> 10) & 0x1F) != 31; }

/* ---- select: Eq. (3) with the fixed hash family ------------------------ */

uint32_t ora_select(uint32_t A, uint32_t C, uint32_t K, uint32_t a)
{
    uint64_t t = ((uint64_t)A * (uint64_t)a + (uint64_t)C) % (1ull << 24);
    return (uint32_t)((t * (uint64_t)K) >> 24);
}

/* Geometry shared by update and query.  Groups are numbered
 * g = jb * (out / tile_out) + ob; the states array is group-major, then
 * sketch row, then index inside the row. */
typedef struct {
    uint32_t in, out, tj, to, d;
    const uint32_t *A, *C, *width;
    uint32_t n_jb, n_ob;
} geom_t;

static int geom_init(geom_t *g, uint32_t in, uint32_t out, uint32_t tj,
                     uint32_t to, uint32_t d, const uint32_t *A,
                     const uint32_t *C, const uint32_t *width)
{
    if (!A || !C || !width || !in || !out || !tj || !to || !d) return ORA_BAD_ARG;
    if (in % tj || out % to) return ORA_BAD_ARG;
    if ((uint64_t)tj * to > (1ull << 24)) return ORA_BAD_ARG;
    g->in = in; g->out = out; g->tj = tj; g->to = to; g->d = d;
    g->A = A; g->C = C; g->width = width;
    g->n_jb = in / tj; g->n_ob = out / to;
    for (uint32_t r = 0; r < d; ++r)
        if (A[r] >= (1u << 24) || C[r] >= (1u << 24)) return ORA_BAD_ARG;
    for (uint64_t i = 0; i < (uint64_t)g->n_jb * g->n_ob; ++i)
        if (width[i] == 0 || width[i] > 65535) return ORA_BAD_ARG;
    return ORA_OK;
}

uint64_t ora_count_states(uint32_t in, uint32_t out, uint32_t tj, uint32_t to,
                          uint32_t d, const uint32_t *width)
{
    uint64_t n = 0;
    if (!tj || !to || in % tj || out % to) return 0;
    for (uint64_t i = 0; i < (uint64_t)(in / tj) * (out / to); ++i) n += width[i];
    return n * d;
}

/* ---- update: Eq. (4), sequential stream over each group ---------------- */

int ora_update(uint32_t in, uint32_t out, uint32_t tj, uint32_t to, uint32_t d,
               const uint32_t *A, const uint32_t *C, const uint32_t *width,
               const uint16_t *W /* [in][out] binary16 */,
               uint16_t *states, uint64_t n_states)
{
    geom_t g;
    int rc = geom_init(&g, in, out, tj, to, d, A, C, width);
    if (rc) return rc;
    if (!W || !states) return ORA_BAD_ARG;
    if (n_states != ora_count_states(in, out, tj, to, d, width)) return ORA_BAD_ARG;
    for (uint64_t i = 0; i < (uint64_t)in * out; ++i)
        if (!half_is_finite(W[i])) return ORA_NONFINITE;

    for (uint64_t i = 0; i < n_states; ++i) states[i] = 0x7C00; /* +inf */

    uint64_t base = 0;
    for (uint32_t jb = 0; jb < g.n_jb; ++jb)
        for (uint32_t ob = 0; ob < g.n_ob; ++ob) {
            uint32_t K = width[(uint64_t)jb * g.n_ob + ob];
            uint16_t *S = states + base;       /* S[r*K + k] */
            for (uint32_t jl = 0; jl < tj; ++jl)
                for (uint32_t ol = 0; ol < to; ++ol) {
                    uint32_t a = jl * to + ol;  /* Addr(w): offset in the group */
                    uint16_t w = W[(uint64_t)(jb * tj + jl) * out + (ob * to + ol)];
                    double aw = fabs(ora_half_to_double(w));
                    for (uint32_t r = 0; r < d; ++r) {
                        uint32_t k = ora_select(A[r], C[r], K, a);
                        uint16_t *s = &S[(uint64_t)r * K + k];
                        if (fabs(ora_half_to_double(*s)) > aw) *s = w;
                    }
                }
            base += (uint64_t)d * K;
        }
    for (uint64_t i = 0; i < n_states; ++i)
        if (states[i] == 0x7C00) states[i] = 0x0000; /* never reached */
    return ORA_OK;
}

/* ---- query: Eq. (5), magnitude order, clear sign bit wins a tie -------- */

static uint16_t absmax_pick(uint16_t best, uint16_t cand)
{
    uint16_t mb = best & 0x7FFF, mc = cand & 0x7FFF; /* finite binary16:
        magnitude order is the integer order of the low 15 bits */
    if (mc > mb) return cand;
    if (mc == mb && (cand >> 15) == 0) return cand;
    return best;
}

/* Eq. (5) read literally: the printed formula is a plain Max over the d
 * candidates, with no magnitude signs.  The larger signed value wins; the
 * only equal values with different bit patterns are +0 and -0, and there the
 * pattern with the clear sign bit wins (as in the magnitude reading). */
static uint16_t signedmax_pick(uint16_t best, uint16_t cand)
{
    double vb = ora_half_to_double(best), vc = ora_half_to_double(cand);
    if (vc > vb) return cand;
    if (vc == vb && (cand >> 15) == 0) return cand;
    return best;
}

/* mode 0: Max by magnitude (the reading this build takes as default);
 * mode 1: Max of the signed values (Eq. (5) as printed). */
int ora_query_mode(uint32_t in, uint32_t out, uint32_t tj, uint32_t to, uint32_t d,
                   const uint32_t *A, const uint32_t *C, const uint32_t *width,
                   const uint16_t *states, uint64_t n_states, int mode,
                   uint16_t *W_hat /* [in][out] binary16 */)
{
    geom_t g;
    int rc = geom_init(&g, in, out, tj, to, d, A, C, width);
    if (rc) return rc;
    if (!states || !W_hat) return ORA_BAD_ARG;
    if (mode != 0 && mode != 1) return ORA_BAD_ARG;
    if (n_states != ora_count_states(in, out, tj, to, d, width)) return ORA_BAD_ARG;
    for (uint64_t i = 0; i < n_states; ++i)
        if (!half_is_finite(states[i])) return ORA_NONFINITE;

    uint64_t base = 0;
    for (uint32_t jb = 0; jb < g.n_jb; ++jb)
        for (uint32_t ob = 0; ob < g.n_ob; ++ob) {
            uint32_t K = width[(uint64_t)jb * g.n_ob + ob];
            const uint16_t *S = states + base;
            for (uint32_t jl = 0; jl < tj; ++jl)
                for (uint32_t ol = 0; ol < to; ++ol) {
                    uint32_t a = jl * to + ol;
                    uint16_t best = S[ora_select(A[0], C[0], K, a)];
                    for (uint32_t r = 1; r < d; ++r) {
                        uint16_t cand = S[(uint64_t)r * K + ora_select(A[r], C[r], K, a)];
                        best = mode == 1 ? signedmax_pick(best, cand) : absmax_pick(best, cand);
                    }
                    W_hat[(uint64_t)(jb * tj + jl) * out + (ob * to + ol)] = best;
                }
            base += (uint64_t)d * K;
        }
    return ORA_OK;
}

int ora_query(uint32_t in, uint32_t out, uint32_t tj, uint32_t to, uint32_t d,
              const uint32_t *A, const uint32_t *C, const uint32_t *width,
              const uint16_t *states, uint64_t n_states,
              uint16_t *W_hat /* [in][out] binary16 */)
{
    return ora_query_mode(in, out, tj, to, d, A, C, width, states, n_states, 0, W_hat);
}

/* ---- low-bit states (Sec. 3.3 last paragraph; Sec. 4 ablation "sketch
 * states in low-bit types") ---------------------------------------------- */

/* double -> binary16 bit pattern, round to nearest even; |v| must be finite
 * and below the binary16 overflow threshold (callers pass |v| <= 65504). */
static uint16_t double_to_half_rne(double v)
{
    uint16_t sign = signbit(v) ? 0x8000 : 0;
    double a = fabs(v);
    if (a == 0.0) return sign;
    int e;
    (void)frexp(a, &e);                 /* a = f * 2^e, 0.5 <= f < 1 */
    int ex = e - 1;                     /* a = 1.xxx * 2^ex */
    if (ex < -14) ex = -14;             /* subnormal range: fixed step 2^-24 */
    double step = ldexp(1.0, ex - 10);  /* spacing of binary16 around a */
    double q = nearbyint(a / step);     /* default rounding mode: half to even; a/step is exact */
    double r = q * step;                /* may carry into the next binade: still representable */
    int e2;
    double f2 = frexp(r, &e2);
    if (r < ldexp(1.0, -14)) return (uint16_t)(sign | (uint16_t)(r / ldexp(1.0, -24)));
    uint32_t mant = (uint32_t)(f2 * 2048.0) - 1024;   /* f2 in [0.5,1): f2*2048 in [1024,2048) */
    return (uint16_t)(sign | ((uint32_t)(e2 - 1 + 15) << 10) | mant);
}

static int qmax_of(int bits) { return bits == 8 ? 127 : bits == 4 ? 7 : 0; }

/* codes: one int8 per state (also for 4 bit: the packing into nibbles is a
 * storage matter of the caller); scales: binary16, [n_groups][d]. */
int ora_quantize_states(uint32_t in, uint32_t out, uint32_t tj, uint32_t to, uint32_t d,
                        const uint32_t *width, const uint16_t *states, uint64_t n_states,
                        int bits, int8_t *codes, uint16_t *scales)
{
    int qmax = qmax_of(bits);
    if (!qmax || !width || !states || !codes || !scales || !tj || !to || in % tj || out % to) return ORA_BAD_ARG;
    if (n_states != ora_count_states(in, out, tj, to, d, width)) return ORA_BAD_ARG;
    for (uint64_t i = 0; i < n_states; ++i)
        if (!half_is_finite(states[i])) return ORA_NONFINITE;
    uint64_t n_groups = (uint64_t)(in / tj) * (out / to), base = 0;
    for (uint64_t g = 0; g < n_groups; ++g) {
        uint32_t K = width[g];
        for (uint32_t r = 0; r < d; ++r) {
            const uint16_t *S = states + base + (uint64_t)r * K;
            uint16_t top = 0;                               /* largest magnitude: integer order of the low 15 bits */
            for (uint32_t k = 0; k < K; ++k)
                if ((S[k] & 0x7FFF) > top) top = S[k] & 0x7FFF;
            scales[g * d + r] = top;
            double sc = ora_half_to_double(top);
            for (uint32_t k = 0; k < K; ++k) {
                double q = sc > 0.0 ? nearbyint(ora_half_to_double(S[k]) * (double)qmax / sc) : 0.0;
                if (q > qmax) q = qmax;
                if (q < -qmax) q = -qmax;
                codes[base + (uint64_t)r * K + k] = (int8_t)q;
            }
        }
        base += (uint64_t)d * K;
    }
    return ORA_OK;
}

int ora_dequantize_states(uint32_t in, uint32_t out, uint32_t tj, uint32_t to, uint32_t d,
                          const uint32_t *width, int bits, const int8_t *codes,
                          const uint16_t *scales, uint16_t *states, uint64_t n_states)
{
    int qmax = qmax_of(bits);
    if (!qmax || !width || !states || !codes || !scales || !tj || !to || in % tj || out % to) return ORA_BAD_ARG;
    if (n_states != ora_count_states(in, out, tj, to, d, width)) return ORA_BAD_ARG;
    uint64_t n_groups = (uint64_t)(in / tj) * (out / to), base = 0;
    for (uint64_t g = 0; g < n_groups; ++g) {
        uint32_t K = width[g];
        for (uint32_t r = 0; r < d; ++r) {
            if (!half_is_finite(scales[g * d + r]) || (scales[g * d + r] >> 15)) return ORA_BAD_ARG;
            double sc = ora_half_to_double(scales[g * d + r]);
            for (uint32_t k = 0; k < K; ++k) {
                int q = codes[base + (uint64_t)r * K + k];
                if (q > qmax || q < -qmax) return ORA_BAD_ARG;
                /* q * sc is exact in binary64; the quotient is within 2^-53 of the true value, far
                 * closer than any binary16 rounding boundary that the true value does not hit exactly */
                states[base + (uint64_t)r * K + k] = double_to_half_rne((double)q * sc / (double)qmax);
            }
        }
        base += (uint64_t)d * K;
    }
    return ORA_OK;
}

/* ---- linear: y[b][o] = sum_j x[b][j] * W_hat[j][o], binary64, ascending j
 * x_kind: 0 = binary16 bit patterns, 1 = bfloat16 bit patterns.
 * cols == NULL: all `out` columns, y is [batch][out];
 * otherwise y is [batch][n_cols] for the listed output channels. */

int ora_linear(uint32_t in, uint32_t out, const uint16_t *W_hat,
               const uint16_t *x, int x_kind, uint32_t batch, uint64_t ldx,
               const uint32_t *cols, uint32_t n_cols, double *y)
{
    if (!W_hat || !x || !y || !in || !out || ldx < in) return ORA_BAD_ARG;
    if (x_kind != 0 && x_kind != 1) return ORA_BAD_ARG;
    uint32_t nc = cols ? n_cols : out;
    for (uint32_t c = 0; c < nc; ++c)
        if (cols && cols[c] >= out) return ORA_BAD_ARG;
    for (uint32_t b = 0; b < batch; ++b)
        for (uint32_t c = 0; c < nc; ++c) {
            uint32_t o = cols ? cols[c] : c;
            double acc = 0.0;
            for (uint32_t j = 0; j < in; ++j) {
                uint16_t xb = x[(uint64_t)b * ldx + j];
                double xv = x_kind ? ora_bf16_to_double(xb) : ora_half_to_double(xb);
                acc += xv * ora_half_to_double(W_hat[(uint64_t)j * out + o]);
            }
            y[(uint64_t)b * nc + c] = acc;
        }
    return ORA_OK;
}
