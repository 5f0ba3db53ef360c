/*
 * CPU oracle for the MOM prefill hot path.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the plain, slow, obviously-correct statement of what the GPU
 * library must compute.  It is used by tests, by the smoke check and by the
 * benchmark's "cpu_baseline" leg; the product (the HIP library and its Python
 * binding) never includes, links or calls it, and it shares no code, header,
 * table or helper with the HIP sources.
 *
 * What it follows (paper: "MOM: Memory-efficient Offloaded Mini-sequence
 * Inference", arXiv 2504.12526):
 *   - Section 3.3, paragraph "Llama MLP Layer": the SwiGLU block
 *         MLP(X) = ( Swish(X W_gate) .* (X W_up) ) W_down ,
 *     Swish taken with beta = 1 (SiLU), no biases.
 *   - Algorithm 1, else-branch, and Section 3 / Eq. 3: the rows of A are cut
 *     into M = ceil(S/C) mini-sequences, O_i = MLP(A_i), O = concat(O_i);
 *     only a C x I intermediate is alive at a time.
 *   - Algorithm 1, if-branch (last MLP layer): A_last = A[-1],
 *     O_last = MLP(A_last), L = LM_Head(O_last).
 *   - Section 3.2 / Algorithm 1 "offload": the KV offload is a move of bytes;
 *     its definition is byte equality and needs no arithmetic here.
 *
 * Data layout (a reading of the paper, which gives only d->I / I->d shapes):
 *   x      [S, H]  row-major, bf16 bit patterns (uint16_t)
 *   W_gate [I, H], W_up [I, H], W_down [H, I], W_lm [V, H]   row-major bf16
 *   i.e. every weight is stored "output features x input features".
 *
 * Arithmetic: inputs are bf16 values widened exactly; every sum runs in index
 * order k = 0,1,2,... in the accumulator type chosen by `acc64` (0: float,
 * 1: double); products are rounded to the accumulator type before the add (no
 * fused multiply-add; build with -ffp-contract=off).  SiLU and the gate*up
 * product are evaluated in the accumulator type.  Nothing is rounded to bf16
 * unless `round_h` asks for the intermediate h to be rounded once
 * (round-to-nearest-even), which mirrors a bf16 workspace and is offered as a
 * diagnostic only.  Outputs are float.
 *
 * Threads: OpenMP over output rows only (each row is an independent job), so
 * the thread count never changes a result.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ---- bf16 <-> f32 (own implementation; IEEE binary32 upper half) -------- */

float oracle_bf16_to_f32(uint16_t b)
{
    uint32_t u = ((uint32_t)b) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

/* round-to-nearest, ties-to-even; NaN stays NaN (quiet), Inf stays Inf */
uint16_t oracle_f32_to_bf16(float f)
{
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    if ((u & 0x7fffffffu) > 0x7f800000u)          /* NaN */
        return (uint16_t)((u >> 16) | 0x0040u);
    uint32_t lower = u & 0xffffu;
    uint32_t upper = u >> 16;
    if (lower > 0x8000u || (lower == 0x8000u && (upper & 1u)))
        upper += 1u;                              /* carries into exponent correctly */
    return (uint16_t)upper;
}

/* ---- SiLU = Swish with beta = 1 :  s(g) = g / (1 + e^{-g}) --------------- */

float oracle_silu_f32(float g)
{
    return g / (1.0f + expf(-g));
}

double oracle_silu_f64(double g)
{
    return g / (1.0 + exp(-g));
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void oracle_set_num_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* widen a bf16 array to float (exact) */
static float *widen(const uint16_t *src, size_t n)
{
    float *dst = (float *)malloc(n * sizeof(float) + 16);
    if (!dst) return NULL;
    for (size_t i = 0; i < n; ++i) dst[i] = oracle_bf16_to_f32(src[i]);
    return dst;
}

/*
 * One token row through the SwiGLU MLP (Section 3.3 formula), float sums.
 *   xr [H] float, wg/wu [I,H] float, wd [H,I] float, h [I] scratch, o [H] out
 */
static void mlp_row_f32(const float *xr, const float *wg, const float *wu,
                        const float *wd, int64_t H, int64_t I, int round_h,
                        float *h, float *o)
{
    for (int64_t j = 0; j < I; ++j) {
        const float *g_row = wg + j * H;
        const float *u_row = wu + j * H;
        float g = 0.0f, u = 0.0f;
        for (int64_t k = 0; k < H; ++k) {
            g += xr[k] * g_row[k];
            u += xr[k] * u_row[k];
        }
        float hv = oracle_silu_f32(g) * u;
        if (round_h) hv = oracle_bf16_to_f32(oracle_f32_to_bf16(hv));
        h[j] = hv;
    }
    for (int64_t i = 0; i < H; ++i) {
        const float *d_row = wd + i * I;
        float s = 0.0f;
        for (int64_t j = 0; j < I; ++j) s += h[j] * d_row[j];
        o[i] = s;
    }
}

/* the same with double sums and double SiLU; result rounded to float once */
static void mlp_row_f64(const float *xr, const float *wg, const float *wu,
                        const float *wd, int64_t H, int64_t I, int round_h,
                        double *h, float *o)
{
    for (int64_t j = 0; j < I; ++j) {
        const float *g_row = wg + j * H;
        const float *u_row = wu + j * H;
        double g = 0.0, u = 0.0;
        for (int64_t k = 0; k < H; ++k) {
            g += (double)xr[k] * (double)g_row[k];
            u += (double)xr[k] * (double)u_row[k];
        }
        double hv = oracle_silu_f64(g) * u;
        if (round_h) hv = (double)oracle_bf16_to_f32(oracle_f32_to_bf16((float)hv));
        h[j] = hv;
    }
    for (int64_t i = 0; i < H; ++i) {
        const float *d_row = wd + i * I;
        double s = 0.0;
        for (int64_t j = 0; j < I; ++j) s += h[j] * (double)d_row[j];
        o[i] = (float)s;
    }
}

/*
 * Unchunked definition on a list of rows.
 *   rows == NULL : rows 0 .. n_rows-1 of x (n_rows <= S)
 *   rows != NULL : the n_rows row indices given (each in [0,S))
 *   out [n_rows, H] float, row r of out belongs to rows[r].
 * Rows are independent (Algorithm 1: O_i depends on A_i only), so evaluating
 * a subset is exact, not an approximation.
 * Returns 0, or -1 on a bad argument / allocation failure.
 */
int oracle_mlp_rows(const uint16_t *x, const uint16_t *W_gate, const uint16_t *W_up,
                    const uint16_t *W_down, int64_t S, int64_t H, int64_t I,
                    const int64_t *rows, int64_t n_rows, int acc64, int round_h,
                    float *out)
{
    if (!x || !W_gate || !W_up || !W_down || !out) return -1;
    if (S < 0 || H <= 0 || I <= 0 || n_rows < 0) return -1;
    if (!rows && n_rows > S) return -1;
    if (rows)
        for (int64_t r = 0; r < n_rows; ++r)
            if (rows[r] < 0 || rows[r] >= S) return -1;
    if (n_rows == 0) return 0;

    float *wg = widen(W_gate, (size_t)I * H);
    float *wu = widen(W_up, (size_t)I * H);
    float *wd = widen(W_down, (size_t)H * I);
    int fail = (!wg || !wu || !wd);

    if (!fail) {
#pragma omp parallel
        {
            float *xr = (float *)malloc((size_t)H * sizeof(float));
            void *h = malloc((size_t)I * sizeof(double));
            int ok = (xr && h);
            /* every thread meets the loop; a thread without scratch marks failure */
#pragma omp for schedule(dynamic, 1)
            for (int64_t r = 0; r < n_rows; ++r) {
                if (!ok) {
#pragma omp atomic write
                    fail = 1;
                    continue;
                }
                int64_t m = rows ? rows[r] : r;
                for (int64_t k = 0; k < H; ++k)
                    xr[k] = oracle_bf16_to_f32(x[m * H + k]);
                if (acc64)
                    mlp_row_f64(xr, wg, wu, wd, H, I, round_h, (double *)h, out + r * H);
                else
                    mlp_row_f32(xr, wg, wu, wd, H, I, round_h, (float *)h, out + r * H);
            }
            free(xr);
            free(h);
        }
    }
    free(wg); free(wu); free(wd);
    return fail ? -1 : 0;
}

/*
 * Algorithm 1, else-branch, written as the algorithm states it: cut the S rows
 * into n = ceil(S/C) mini-sequences of C rows (the last one shorter), run the
 * three projections of each mini-sequence with a C x I intermediate that is
 * reused, and place O_i at its rows of O (the concat).  float sums only.
 * C <= 0 or C > S means one mini-sequence of S rows.
 * `peak_intermediate_elems`, if not NULL, receives the element count of the
 * largest intermediate allocated (Eq. 3: C*I, against S*I for Eq. 1).
 */
int oracle_mlp_miniseq(const uint16_t *x, const uint16_t *W_gate, const uint16_t *W_up,
                       const uint16_t *W_down, int64_t S, int64_t H, int64_t I,
                       int64_t C, float *out, int64_t *peak_intermediate_elems)
{
    if (!x || !W_gate || !W_up || !W_down || !out) return -1;
    if (S < 0 || H <= 0 || I <= 0) return -1;
    if (C <= 0 || C > S) C = S;
    if (peak_intermediate_elems) *peak_intermediate_elems = C * I;
    if (S == 0) return 0;

    float *wg = widen(W_gate, (size_t)I * H);
    float *wu = widen(W_up, (size_t)I * H);
    float *wd = widen(W_down, (size_t)H * I);
    float *xf = widen(x, (size_t)S * H);
    float *inter = (float *)malloc((size_t)C * I * sizeof(float));   /* the one reused buffer */
    if (!wg || !wu || !wd || !xf || !inter) {
        free(wg); free(wu); free(wd); free(xf); free(inter);
        return -1;
    }
    int64_t n = (S + C - 1) / C;
    for (int64_t i = 0; i < n; ++i) {
        int64_t r0 = i * C;
        int64_t rows = (r0 + C <= S) ? C : (S - r0);
        /* gate and up projections, Swish, element-wise product -> intermediate */
#pragma omp parallel for schedule(static)
        for (int64_t m = 0; m < rows; ++m) {
            const float *xr = xf + (r0 + m) * H;
            for (int64_t j = 0; j < I; ++j) {
                float g = 0.0f, u = 0.0f;
                for (int64_t k = 0; k < H; ++k) {
                    g += xr[k] * wg[j * H + k];
                    u += xr[k] * wu[j * H + k];
                }
                inter[m * I + j] = oracle_silu_f32(g) * u;
            }
        }
        /* down projection, written straight to rows r0.. of O */
#pragma omp parallel for schedule(static)
        for (int64_t m = 0; m < rows; ++m) {
            for (int64_t c = 0; c < H; ++c) {
                float s = 0.0f;
                for (int64_t j = 0; j < I; ++j) s += inter[m * I + j] * wd[c * I + j];
                out[(r0 + m) * H + c] = s;
            }
        }
    }
    free(wg); free(wu); free(wd); free(xf); free(inter);
    return 0;
}

/*
 * LM head on one token (Algorithm 1 if-branch; Section 3.3: the head needs
 * only V outputs when one token is projected):
 *     logits[v] = sum_k x_last[k] * W_lm[v,k]
 */
int oracle_lmhead(const uint16_t *x_last, const uint16_t *W_lm, int64_t V, int64_t H,
                  int acc64, float *logits)
{
    if (!x_last || !W_lm || !logits || V < 0 || H <= 0) return -1;
    float *xf = widen(x_last, (size_t)H);
    if (!xf) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t v = 0; v < V; ++v) {
        const uint16_t *w = W_lm + v * H;
        if (acc64) {
            double s = 0.0;
            for (int64_t k = 0; k < H; ++k)
                s += (double)xf[k] * (double)oracle_bf16_to_f32(w[k]);
            logits[v] = (float)s;
        } else {
            float s = 0.0f;
            for (int64_t k = 0; k < H; ++k) s += xf[k] * oracle_bf16_to_f32(w[k]);
            logits[v] = s;
        }
    }
    free(xf);
    return 0;
}

/*
 * Algorithm 1 if-branch end to end: take the last row of A, run the MLP on
 * it, round O_last to bf16 (the activation dtype the next operator receives),
 * and project through the LM head.  o_last [H] float (unrounded), logits [V].
 */
int oracle_last_token(const uint16_t *A, const uint16_t *W_gate, const uint16_t *W_up,
                      const uint16_t *W_down, const uint16_t *W_lm, int64_t S, int64_t H,
                      int64_t I, int64_t V, int acc64, float *o_last, float *logits)
{
    if (S < 1) return -1;
    int64_t last = S - 1;
    int rc = oracle_mlp_rows(A, W_gate, W_up, W_down, S, H, I, &last, 1, acc64, 0, o_last);
    if (rc) return rc;
    uint16_t *ob = (uint16_t *)malloc((size_t)H * sizeof(uint16_t));
    if (!ob) return -1;
    for (int64_t k = 0; k < H; ++k) ob[k] = oracle_f32_to_bf16(o_last[k]);
    rc = oracle_lmhead(ob, W_lm, V, H, acc64, logits);
    free(ob);
    return rc;
}
