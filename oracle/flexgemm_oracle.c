/*
 * CPU oracle for the flexible mixed-precision GEMM and the tensor contraction.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition the GPU
 * library is checked against.  It shares no code with the HIP path, is never
 * linked into or called from the product library, and may be used only by the
 * tests, the smoke check and the CPU-baseline leg of the benchmark.
 *
 * What it computes (paper: Section 2.2 "D = A.B + C"; Section 4.3.2 BLAS-like
 * form "C := alpha.A.B + beta.C"; Section 4.3.1 ReLU form
 * "D_ij = max(sum_k A_ik B_kj + C_ij, 0)"; Section 5.1 N/T = column-/row-major;
 * Section 5.2 diagonal operands; Section 5.3 bias vector; Section 5.4 complex
 * product as four real products; Section 5.5 tensor contraction in Einstein
 * notation):
 *
 *   S_ij = sum_{k=0}^{K-1} opA(i,k) * opB(k,j)          (ascending k, FP64)
 *   Y_ij = alpha*S_ij + beta*C_ij + bias                 (absent terms are 0)
 *   D_ij = act(Y_ij),  act in {identity, max(.,0)}
 *   G_ij = |alpha| * sum_k |opA(i,k)|*|opB(k,j)| + |beta|*|C_ij|
 *
 * A and B are IEEE binary16 bit patterns, widened exactly to double; C and the
 * bias are binary32, widened exactly.  Every sum is a plain loop; there is no
 * blocking, no reordering and no vectorisation by hand.  G is the denominator
 * of the elementwise tolerance the GPU results are held to.
 *
 * Threads only partition the list of output entries; no entry is written by
 * two threads and no partial sums are shared.
 *
 * Parity with the paper's own runs: unpinned (the paper publishes no numeric
 * outputs).  The functions here are pinned by the CPU tests against closed
 * forms, identities and independent library routines.
 */
#include <math.h>
#include <pthread.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { OG_COL = 0, OG_ROW = 1, OG_DIAG = 2 };
enum { OG_ACT_NONE = 0, OG_ACT_RELU = 1 };
enum { OG_OK = 0, OG_BAD_ARG = 1 };

/* ---- binary16 -> double, exact -------------------------------------------------- */

static double half_bits_to_double(uint16_t h) {
    int sign = (h >> 15) & 1;
    int expo = (h >> 10) & 0x1f;
    int frac = h & 0x3ff;
    double v;
    if (expo == 0) {
        v = ldexp((double)frac, -24);            /* zero and subnormals: frac * 2^-24 */
    } else if (expo == 31) {
        v = frac ? NAN : INFINITY;
    } else {
        v = ldexp((double)(1024 + frac), expo - 25); /* (1 + frac/1024) * 2^(expo-15) */
    }
    return sign ? -v : v;
}

/* ---- bfloat16 -> double, exact: the upper 16 bits of a binary32 ---------------------------- */
static double bf16_bits_to_double(uint16_t h) {
    int sign = (h >> 15) & 1;
    int expo = (h >> 7) & 0xff;
    int frac = h & 0x7f;
    double v;
    if (expo == 0) {
        v = ldexp((double)frac, -133);                   /* zero and subnormals: frac * 2^-7 * 2^-126 */
    } else if (expo == 255) {
        v = frac ? NAN : INFINITY;
    } else {
        v = ldexp((double)(128 + frac), expo - 134);     /* (1 + frac/128) * 2^(expo-127) */
    }
    return sign ? -v : v;
}

/* Decode tables for the two 16-bit input types; index 0: binary16, 1: bfloat16. */
static double g_half_table[2][65536];
static pthread_once_t g_half_once = PTHREAD_ONCE_INIT;
static void build_half_table(void) {
    for (int i = 0; i < 65536; ++i) {
        g_half_table[0][i] = half_bits_to_double((uint16_t)i);
        g_half_table[1][i] = bf16_bits_to_double((uint16_t)i);
    }
}
static inline double h2d(uint16_t h) { return g_half_table[0][h]; }

/* Exposed so the tests can pin the decoders against independent conversions. */
double oracle_half_to_double(uint16_t h) { return half_bits_to_double(h); }
double oracle_bf16_to_double(uint16_t h) { return bf16_bits_to_double(h); }

/* Nearest binary16 value (ties to even) of a double, returned as a double.  Used for the
 * element-wise addition on A and B (Section 4.3 "transforms", Section 5.3 fusion table), which
 * the method performs in the element type: the exact sum of two binary16 values, which a double
 * holds exactly, rounded once. */
static double round_to_half(double x) {
    if (isnan(x) || isinf(x) || x == 0.0) return x;
    double ax = fabs(x);
    int e;
    (void)frexp(ax, &e);                    /* ax = m * 2^e with m in [0.5, 1): leading bit 2^(e-1) */
    int lead = e - 1;
    if (lead < -14) lead = -14;             /* subnormals share the quantum of the lowest binade */
    double quantum = ldexp(1.0, lead - 10); /* spacing of binary16 values in that binade */
    double v = nearbyint(ax / quantum) * quantum;   /* round-to-nearest-even is the default mode */
    if (v > 65504.0) v = INFINITY;
    return x < 0.0 ? -v : v;
}
double oracle_round_to_half(double x) { return round_to_half(x); }

/* ---- problem descriptions ------------------------------------------------------- */

typedef struct {
    int64_t M, N, K;
    double alpha, beta;
    const uint16_t *A_re, *A_im;   /* A_im == NULL: real operand                */
    int32_t layoutA;               /* OG_COL / OG_ROW / OG_DIAG                  */
    int64_t lda;                   /* elements; ignored for OG_DIAG              */
    const uint16_t *B_re, *B_im;
    int32_t layoutB;
    int64_t ldb;
    const float *C_re, *C_im;      /* C_re == NULL: no C term                    */
    int32_t layoutC;               /* OG_COL / OG_ROW                            */
    int64_t ldc;
    const float *bias;             /* NULL: none                                 */
    int32_t bias_dim;              /* 0: bias[i] (length M), 1: bias[j] (len N)  */
    int32_t act;
    int32_t ab_dtype;              /* element type of A and B: 0 binary16, 1 bfloat16 */
    int32_t dual;                  /* 1: the second planes are dual parts (eps^2 = 0, Section 5.4)
                                      instead of imaginary parts (i^2 = -1)        */
    /* transforms applied to loaded elements (Section 4.3 "transforms"; last rows of the fusion
       table of Section 5.3); real binary16 COL/ROW operands only */
    int32_t ab_add;                /* 1: A_ik := half(A_ik + a_add), B_kj := half(B_kj + b_add) */
    double a_add, b_add;           /* must be binary16 values                    */
    int32_t c_act;                 /* activation applied to C_ij before beta     */
    /* interleaved complex storage (Section 5.4: the layout of complex matrices in global memory):
       element e of an operand occupies positions 2e (real part) and 2e + 1 (imaginary part) of one
       array.  interleaved_ab / interleaved_c = 1: the *_re pointer is that array, the *_im pointer
       is *_re + 1, and every element index is doubled; leading dimensions count complex elements. */
    int32_t interleaved_ab, interleaved_c;
} og_problem;

/* logical element (r, c) of a stored rows x cols operand */
/* `es`: positions per element, 1 (one array per plane) or 2 (interleaved complex) */
static inline double operand_at(const uint16_t *p, int32_t layout, int64_t ld, int64_t r, int64_t c, const double *decode, int es) {
    if (layout == OG_COL) return decode[p[es * (r + c * ld)]];
    if (layout == OG_ROW) return decode[p[es * (c + r * ld)]];
    /* OG_DIAG: p is the vector of diagonal entries, everything else is zero */
    return (r == c) ? decode[p[es * r]] : 0.0;
}

static inline double c_at(const float *p, int32_t layout, int64_t ld, int64_t i, int64_t j, int es) {
    return (double)((layout == OG_COL) ? p[es * (i + j * ld)] : p[es * (j + i * ld)]);
}

/* One output entry (i, j): the definition written out. */
static void gemm_entry(const og_problem *q, int64_t i, int64_t j,
                       double *d_re, double *d_im, double *g_re, double *g_im) {
    const int is_complex = (q->A_im != NULL) || (q->B_im != NULL);
    const double *dec = g_half_table[q->ab_dtype ? 1 : 0];
    const int es = q->interleaved_ab ? 2 : 1, esc = q->interleaved_c ? 2 : 1;
    double s_re = 0.0, s_im = 0.0, m_re = 0.0, m_im = 0.0;
    for (int64_t k = 0; k < q->K; ++k) {
        double ar = operand_at(q->A_re, q->layoutA, q->lda, i, k, dec, es);
        double br = operand_at(q->B_re, q->layoutB, q->ldb, k, j, dec, es);
        if (q->ab_add) {
            ar = round_to_half(ar + q->a_add);
            br = round_to_half(br + q->b_add);
        }
        if (!is_complex) {
            s_re += ar * br;
            m_re += fabs(ar) * fabs(br);
        } else {
            double ai = q->A_im ? operand_at(q->A_im, q->layoutA, q->lda, i, k, dec, es) : 0.0;
            double bi = q->B_im ? operand_at(q->B_im, q->layoutB, q->ldb, k, j, dec, es) : 0.0;
            if (q->dual) {
                /* (ar + eps ai)(br + eps bi) with eps^2 = 0: the eps.eps product vanishes */
                s_re += ar * br;
                m_re += fabs(ar) * fabs(br);
            } else {
                /* (ar + i ai)(br + i bi): the four real products of Section 5.4 */
                s_re += ar * br - ai * bi;
                m_re += fabs(ar) * fabs(br) + fabs(ai) * fabs(bi);
            }
            s_im += ar * bi + ai * br;
            m_im += fabs(ar) * fabs(bi) + fabs(ai) * fabs(br);
        }
    }
    double y_re = q->alpha * s_re, y_im = q->alpha * s_im;
    double t_re = fabs(q->alpha) * m_re, t_im = fabs(q->alpha) * m_im;
    if (q->C_re) {
        double c = c_at(q->C_re, q->layoutC, q->ldc, i, j, esc);
        if (q->c_act == OG_ACT_RELU) c = (c > 0.0) ? c : 0.0;
        y_re += q->beta * c;
        t_re += fabs(q->beta) * fabs(c);
    }
    if (is_complex && q->C_im) {
        double c = c_at(q->C_im, q->layoutC, q->ldc, i, j, esc);
        y_im += q->beta * c;
        t_im += fabs(q->beta) * fabs(c);
    }
    if (q->bias) y_re += (double)q->bias[q->bias_dim == 0 ? i : j];
    if (q->act == OG_ACT_RELU) y_re = (y_re > 0.0) ? y_re : 0.0;
    *d_re = y_re;
    *g_re = t_re;
    if (d_im) *d_im = y_im;
    if (g_im) *g_im = t_im;
}

static int gemm_problem_ok(const og_problem *q) {
    if (!q || q->M < 0 || q->N < 0 || q->K < 0) return 0;
    if (!q->A_re || !q->B_re) return (q->M == 0 || q->N == 0 || q->K == 0);
    if (q->layoutA < OG_COL || q->layoutA > OG_DIAG) return 0;
    if (q->layoutB < OG_COL || q->layoutB > OG_DIAG) return 0;
    if (q->C_re && q->layoutC != OG_COL && q->layoutC != OG_ROW) return 0;
    if (q->bias && q->bias_dim != 0 && q->bias_dim != 1) return 0;
    if (q->act != OG_ACT_NONE && q->act != OG_ACT_RELU) return 0;
    if (q->ab_dtype != 0 && q->ab_dtype != 1) return 0;
    if (q->c_act != OG_ACT_NONE && q->c_act != OG_ACT_RELU) return 0;
    if (q->interleaved_ab && (!q->A_im || !q->B_im || q->A_im != q->A_re + 1 || q->B_im != q->B_re + 1)) return 0;
    if (q->interleaved_c && q->C_re && q->C_im != q->C_re + 1) return 0;
    /* the activation on C touches only C: any real product; the addition on A and B is defined
       here for stored binary16 matrices only */
    if (q->c_act && (q->A_im || q->B_im)) return 0;
    if (q->ab_add) {
        if (q->A_im || q->B_im || q->ab_dtype != 0 || q->layoutA == OG_DIAG || q->layoutB == OG_DIAG) return 0;
        if (round_to_half(q->a_add) != q->a_add || round_to_half(q->b_add) != q->b_add) return 0;
    }
    const int is_complex = (q->A_im != NULL) || (q->B_im != NULL);
    if (is_complex && (q->bias || q->act != OG_ACT_NONE)) return 0; /* not defined for complex */
    return 1;
}

/* ---- thread plumbing: split [0, total) into contiguous shares ------------------ */

typedef void (*range_fn)(void *ctx, int64_t begin, int64_t end);
typedef struct { range_fn fn; void *ctx; int64_t begin, end; } share_t;
static void *share_main(void *p) { share_t *s = (share_t *)p; s->fn(s->ctx, s->begin, s->end); return NULL; }

static void run_shares(range_fn fn, void *ctx, int64_t total, int nthreads) {
    if (nthreads < 1) nthreads = 1;
    if (nthreads > 256) nthreads = 256;
    if ((int64_t)nthreads > total) nthreads = (int)(total > 0 ? total : 1);
    if (nthreads == 1) { fn(ctx, 0, total); return; }
    pthread_t tid[256];
    share_t sh[256];
    int started[256];
    for (int t = 0; t < nthreads; ++t) {
        sh[t].fn = fn; sh[t].ctx = ctx;
        sh[t].begin = total * t / nthreads;
        sh[t].end = total * (t + 1) / nthreads;
        started[t] = (pthread_create(&tid[t], NULL, share_main, &sh[t]) == 0);
        if (!started[t]) fn(ctx, sh[t].begin, sh[t].end);   /* fall back to this thread */
    }
    for (int t = 0; t < nthreads; ++t) if (started[t]) pthread_join(tid[t], NULL);
}

/* ---- GEMM: every entry, and entries at listed positions ------------------------ */

typedef struct {
    const og_problem *q;
    double *D_re, *D_im, *G_re, *G_im;
    const int64_t *I, *J;          /* NULL in full mode */
} gemm_ctx;

static void gemm_full_range(void *vp, int64_t begin, int64_t end) {
    gemm_ctx *c = (gemm_ctx *)vp;
    const int64_t M = c->q->M;
    /* entry e <-> (i, j) = (e mod M, e div M): output is column-major with ld = M */
    for (int64_t e = begin; e < end; ++e) {
        int64_t i = e % M, j = e / M;
        double dr, di, gr, gi;
        gemm_entry(c->q, i, j, &dr, &di, &gr, &gi);
        c->D_re[e] = dr;
        if (c->D_im) c->D_im[e] = di;
        if (c->G_re) c->G_re[e] = gr;
        if (c->G_im) c->G_im[e] = gi;
    }
}

static void gemm_at_range(void *vp, int64_t begin, int64_t end) {
    gemm_ctx *c = (gemm_ctx *)vp;
    for (int64_t e = begin; e < end; ++e) {
        double dr, di, gr, gi;
        gemm_entry(c->q, c->I[e], c->J[e], &dr, &di, &gr, &gi);
        c->D_re[e] = dr;
        if (c->D_im) c->D_im[e] = di;
        if (c->G_re) c->G_re[e] = gr;
        if (c->G_im) c->G_im[e] = gi;
    }
}

/* D_*, G_*: M*N doubles, column-major, ld = M.  D_im/G_re/G_im may be NULL. */
int oracle_gemm_full(const og_problem *q, double *D_re, double *D_im, double *G_re, double *G_im, int nthreads) {
    pthread_once(&g_half_once, build_half_table);
    if (!gemm_problem_ok(q) || !D_re) return OG_BAD_ARG;
    gemm_ctx c = { q, D_re, D_im, G_re, G_im, NULL, NULL };
    run_shares(gemm_full_range, &c, q->M * q->N, nthreads);
    return OG_OK;
}

/* Entries (I[e], J[e]), e < count; outputs have length count. */
int oracle_gemm_at(const og_problem *q, int64_t count, const int64_t *I, const int64_t *J,
                   double *D_re, double *D_im, double *G_re, double *G_im, int nthreads) {
    pthread_once(&g_half_once, build_half_table);
    if (!gemm_problem_ok(q) || !D_re || count < 0 || (count && (!I || !J))) return OG_BAD_ARG;
    for (int64_t e = 0; e < count; ++e)
        if (I[e] < 0 || I[e] >= q->M || J[e] < 0 || J[e] >= q->N) return OG_BAD_ARG;
    gemm_ctx c = { q, D_re, D_im, G_re, G_im, I, J };
    run_shares(gemm_at_range, &c, count, nthreads);
    return OG_OK;
}

/* ---- tensor contraction --------------------------------------------------------- *
 * C[free modes] = alpha * sum over contracted modes A[...] * B[...] + beta * Cin[...]
 * (Section 4.1 and Section 5.5).  A mode is identified by an integer label; the free
 * modes are those of C, the contracted modes are the modes of A or B that C lacks.
 * Element offsets are sum_m index_m * stride_m, strides in elements.               */

#define OC_MAX_MODES 16

typedef struct {
    int32_t n_modes;
    const int32_t *labels;         /* n_modes distinct labels     */
    const int64_t *extents;        /* extent of each label        */
    int32_t nA; const int32_t *modesA; const int64_t *stridesA; const uint16_t *A;
    int32_t nB; const int32_t *modesB; const int64_t *stridesB; const uint16_t *B;
    int32_t nC; const int32_t *modesC; const int64_t *stridesC; const float *Cin; /* Cin may be NULL */
    double alpha, beta;
} oc_problem;

typedef struct {
    int n_free, n_sum;
    int64_t ext_free[OC_MAX_MODES], ext_sum[OC_MAX_MODES];
    /* stride of each free / contracted mode inside A, B and C (0 where the tensor lacks it) */
    int64_t a_free[OC_MAX_MODES], b_free[OC_MAX_MODES], c_free[OC_MAX_MODES];
    int64_t a_sum[OC_MAX_MODES], b_sum[OC_MAX_MODES];
} oc_plan;

static int find_label(const oc_problem *q, int32_t label) {
    for (int m = 0; m < q->n_modes; ++m) if (q->labels[m] == label) return m;
    return -1;
}
static int64_t stride_in(int32_t n, const int32_t *modes, const int64_t *strides, int32_t label) {
    for (int t = 0; t < n; ++t) if (modes[t] == label) return strides[t];
    return 0;
}
static int has_mode(int32_t n, const int32_t *modes, int32_t label) {
    for (int t = 0; t < n; ++t) if (modes[t] == label) return 1;
    return 0;
}
static int distinct(int32_t n, const int32_t *modes) {
    for (int a = 0; a < n; ++a) for (int b = a + 1; b < n; ++b) if (modes[a] == modes[b]) return 0;
    return 1;
}

static int make_plan(const oc_problem *q, oc_plan *pl) {
    if (!q || q->n_modes < 0 || q->n_modes > OC_MAX_MODES) return 0;
    if (q->nA < 0 || q->nB < 0 || q->nC < 0) return 0;
    if (q->nA > OC_MAX_MODES || q->nB > OC_MAX_MODES || q->nC > OC_MAX_MODES) return 0;
    if (!distinct(q->n_modes, q->labels)) return 0;
    if (!distinct(q->nA, q->modesA) || !distinct(q->nB, q->modesB) || !distinct(q->nC, q->modesC)) return 0;
    for (int t = 0; t < q->nA; ++t) if (find_label(q, q->modesA[t]) < 0) return 0;
    for (int t = 0; t < q->nB; ++t) if (find_label(q, q->modesB[t]) < 0) return 0;
    for (int m = 0; m < q->n_modes; ++m) if (q->extents[m] < 0) return 0;
    memset(pl, 0, sizeof *pl);
    /* free modes in the order C lists them; each must come from A or B */
    for (int t = 0; t < q->nC; ++t) {
        int32_t lab = q->modesC[t];
        int m = find_label(q, lab);
        if (m < 0) return 0;
        if (!has_mode(q->nA, q->modesA, lab) && !has_mode(q->nB, q->modesB, lab)) return 0;
        int f = pl->n_free++;
        pl->ext_free[f] = q->extents[m];
        pl->a_free[f] = stride_in(q->nA, q->modesA, q->stridesA, lab);
        pl->b_free[f] = stride_in(q->nB, q->modesB, q->stridesB, lab);
        pl->c_free[f] = q->stridesC[t];
    }
    /* contracted modes in label order */
    for (int m = 0; m < q->n_modes; ++m) {
        int32_t lab = q->labels[m];
        if (has_mode(q->nC, q->modesC, lab)) continue;
        int inA = has_mode(q->nA, q->modesA, lab), inB = has_mode(q->nB, q->modesB, lab);
        if (!inA && !inB) continue;              /* label not used by this contraction */
        int s = pl->n_sum++;
        pl->ext_sum[s] = q->extents[m];
        pl->a_sum[s] = stride_in(q->nA, q->modesA, q->stridesA, lab);
        pl->b_sum[s] = stride_in(q->nB, q->modesB, q->stridesB, lab);
    }
    return 1;
}

/* One output entry, given the index of every free mode. */
static void contract_entry(const oc_problem *q, const oc_plan *pl, const int64_t *free_idx,
                           double *out, double *g, int64_t *c_offset) {
    int64_t offA = 0, offB = 0, offC = 0;
    for (int f = 0; f < pl->n_free; ++f) {
        offA += free_idx[f] * pl->a_free[f];
        offB += free_idx[f] * pl->b_free[f];
        offC += free_idx[f] * pl->c_free[f];
    }
    int64_t total = 1;
    for (int s = 0; s < pl->n_sum; ++s) total *= pl->ext_sum[s];
    double acc = 0.0, mag = 0.0;
    int64_t idx[OC_MAX_MODES] = {0};
    for (int64_t t = 0; t < total; ++t) {
        int64_t pa = offA, pb = offB;
        for (int s = 0; s < pl->n_sum; ++s) { pa += idx[s] * pl->a_sum[s]; pb += idx[s] * pl->b_sum[s]; }
        double a = h2d(q->A[pa]), b = h2d(q->B[pb]);
        acc += a * b;
        mag += fabs(a) * fabs(b);
        /* odometer over the contracted modes, first mode fastest */
        for (int s = 0; s < pl->n_sum; ++s) { if (++idx[s] < pl->ext_sum[s]) break; idx[s] = 0; }
    }
    double y = q->alpha * acc, t = fabs(q->alpha) * mag;
    if (q->Cin) { double c = (double)q->Cin[offC]; y += q->beta * c; t += fabs(q->beta) * fabs(c); }
    *out = y; *g = t; *c_offset = offC;
}

typedef struct {
    const oc_problem *q; const oc_plan *pl;
    double *out, *g;
    const int64_t *at;            /* NULL in full mode; else count x nC indices */
} contract_ctx;

static void contract_full_range(void *vp, int64_t begin, int64_t end) {
    contract_ctx *c = (contract_ctx *)vp;
    const oc_plan *pl = c->pl;
    for (int64_t e = begin; e < end; ++e) {
        /* e enumerates the free multi-index with C's first listed mode fastest */
        int64_t idx[OC_MAX_MODES], r = e;
        for (int f = 0; f < pl->n_free; ++f) { idx[f] = r % pl->ext_free[f]; r /= pl->ext_free[f]; }
        double y, t; int64_t offC;
        contract_entry(c->q, pl, idx, &y, &t, &offC);
        c->out[offC] = y;
        if (c->g) c->g[offC] = t;
    }
}
static void contract_at_range(void *vp, int64_t begin, int64_t end) {
    contract_ctx *c = (contract_ctx *)vp;
    for (int64_t e = begin; e < end; ++e) {
        double y, t; int64_t offC;
        contract_entry(c->q, c->pl, c->at + e * c->pl->n_free, &y, &t, &offC);
        c->out[e] = y;
        if (c->g) c->g[e] = t;
    }
}

/* out, g: indexed by C's own element offsets (sum idx*strideC); g may be NULL.
 * Entries of out that no free multi-index reaches are left untouched.            */
int oracle_contract_full(const oc_problem *q, double *out, double *g, int nthreads) {
    pthread_once(&g_half_once, build_half_table);
    oc_plan pl;
    if (!make_plan(q, &pl) || !out || !q->A || !q->B) return OG_BAD_ARG;
    int64_t total = 1;
    for (int f = 0; f < pl.n_free; ++f) total *= pl.ext_free[f];
    contract_ctx c = { q, &pl, out, g, NULL };
    run_shares(contract_full_range, &c, total, nthreads);
    return OG_OK;
}

/* at: count x nC free-mode indices, in the order C lists its modes; out, g: length count. */
int oracle_contract_at(const oc_problem *q, int64_t count, const int64_t *at, double *out, double *g, int nthreads) {
    pthread_once(&g_half_once, build_half_table);
    oc_plan pl;
    if (!make_plan(q, &pl) || !out || !q->A || !q->B || count < 0 || (count && !at)) return OG_BAD_ARG;
    for (int64_t e = 0; e < count; ++e)
        for (int f = 0; f < pl.n_free; ++f)
            if (at[e * pl.n_free + f] < 0 || at[e * pl.n_free + f] >= pl.ext_free[f]) return OG_BAD_ARG;
    contract_ctx c = { q, &pl, out, g, at };
    run_shares(contract_at_range, &c, count, nthreads);
    return OG_OK;
}
