/*
 * CPU oracle for incremental GNN inference on streaming graphs -- TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, plain definition that the HIP library is checked against.  It is
 * used by tests, by the smoke check and by the benchmark's "cpu_baseline" leg; the product
 * path never calls it and shares no code with it.
 *
 * What it computes is the paper's "classic method": ordinary k-layer inference on the
 * latest graph snapshot (Sec. 1, Fig. "Inference on a streaming graph" (a); the "Full"
 * baseline of Sec. 4.1).  The incremental method is specified to give the identical result
 * for min/max aggregation (Abstract; Sec. 1 "No Accuracy Loss"), so the oracle is that plain
 * definition and contains no events, caches or resets.
 *
 * Layout: all matrices row-major, float32 unless stated.  Graph = in-neighbour CSR: row v
 * lists the sources u of edges u -> v (Sec. 2.1: alpha_{l,v} = A(m_{l,u} : u in N(v))).
 * The only parallelism is an OpenMP "parallel for" over destination rows.
 *
 * Pins: tests/test_oracle_pins.py (brute force, dense-matrix closed forms, hand-computed
 * star/path graphs under tests/golden/, duality and invariants).  The paper prints no numeric
 * worked example (its illustrative figures carry the numbers), so no printed value is pinned.
 */
#include <math.h>
#include <stdint.h>
#include <stddef.h>

/* Sec. 2.1 / Sec. 2.2 item 1: alpha = A(m_u : u in N(v)), A = max (is_min = 0) or min.
 * arg[v][i] = the lowest neighbour id attaining the selected value.  A node without
 * in-neighbours gets alpha = 0 and arg = -1 (reading: Sec. 2.4.1 names +-inf only as the
 * intermediate reset value, so the stored result of an empty selection is taken as zero). */
void orc_agg_select(int64_t n, const int64_t *rowptr, const int32_t *col, const float *m,
                    int32_t d, int32_t is_min, float *alpha, int32_t *arg)
{
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t v = 0; v < n; v++) {
        for (int32_t i = 0; i < d; i++) {
            float best = 0.0f;
            int32_t who = -1;
            for (int64_t e = rowptr[v]; e < rowptr[v + 1]; e++) {
                int32_t u = col[e];
                float x = m[(int64_t)u * d + i];
                int better;
                if (who < 0) better = 1;
                else if (is_min) better = (x < best) || (x == best && u < who);
                else better = (x > best) || (x == best && u < who);
                if (better) { best = x; who = u; }
            }
            alpha[v * d + i] = best;
            arg[v * d + i] = who;
        }
    }
}

/* Plain sum aggregation (GIN, eq. (5) with A = sum): fp64 accumulation over neighbours in CSR
 * order, rounded once to float.  mean = 1: divide by max(deg, 1) before rounding. */
void orc_agg_sum(int64_t n, const int64_t *rowptr, const int32_t *col, const float *m,
                 int32_t d, int32_t mean, float *alpha)
{
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t v = 0; v < n; v++) {
        int64_t deg = rowptr[v + 1] - rowptr[v];
        for (int32_t i = 0; i < d; i++) {
            double acc = 0.0;
            for (int64_t e = rowptr[v]; e < rowptr[v + 1]; e++)
                acc += (double)m[(int64_t)col[e] * d + i];
            if (mean) acc /= (double)(deg > 0 ? deg : 1);
            alpha[v * d + i] = (float)acc;
        }
    }
}

/* Symmetric degree-normalised sum with self loop (GCN, eq. (1) with the normalised aggregator):
 * a_v = sum over u in N(v) + {v} of h_u / sqrt(dhat_u * dhat_v), dhat_x = indeg(x) + 1. */
void orc_agg_gcn_sym(int64_t n, const int64_t *rowptr, const int32_t *col, const float *h,
                     int32_t d, float *alpha)
{
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t v = 0; v < n; v++) {
        double dv = (double)(rowptr[v + 1] - rowptr[v] + 1);
        for (int32_t i = 0; i < d; i++) {
            double acc = (double)h[v * d + i] / sqrt(dv * dv);
            for (int64_t e = rowptr[v]; e < rowptr[v + 1]; e++) {
                int32_t u = col[e];
                double du = (double)(rowptr[u + 1] - rowptr[u] + 1);
                acc += (double)h[(int64_t)u * d + i] / sqrt(du * dv);
            }
            alpha[v * d + i] = (float)acc;
        }
    }
}

/* Dense combination y = act(x W + b) for `rows` rows (eqs. (2), (4), (6)); W is [din][dout].
 * mode 0: fp64 accumulation, k ascending, one rounding to float (the definition).
 * mode 1: float accumulator starting at +0, one fused multiply-add per k in ascending order,
 *         then a float add of the bias: the fp32 evaluation order used when an integer decision
 *         (changed set, argmax) downstream must be taken in the same precision as fp32 hardware.
 *         The loop over the outputs j is the inner one here (each y[r][j] is its own accumulator
 *         and still receives k = 0, 1, 2, ... in that order), so that the compiler may work on
 *         several outputs at once: the full-size parity runs push 10^10 such chains through it.
 * relu: x > 0 ? x : +0. */
void orc_linear(int64_t rows, int32_t din, int32_t dout, const float *x, const float *W,
                const float *bias, int32_t relu, int32_t mode, float *y)
{
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; r++) {
        if (mode == 0) {
            for (int32_t j = 0; j < dout; j++) {
                double acc = 0.0;
                for (int32_t k = 0; k < din; k++)
                    acc += (double)x[r * din + k] * (double)W[(int64_t)k * dout + j];
                if (bias) acc += (double)bias[j];
                y[r * dout + j] = (float)acc;
            }
        } else {
            float *acc = y + r * dout;
            for (int32_t j = 0; j < dout; j++) acc[j] = 0.0f;
            for (int32_t k = 0; k < din; k++) {
                const float xv = x[r * din + k];
                const float *w = W + (int64_t)k * dout;
                for (int32_t j = 0; j < dout; j++) acc[j] = fmaf(xv, w[j], acc[j]);
            }
            if (bias)
                for (int32_t j = 0; j < dout; j++) acc[j] = acc[j] + bias[j];
        }
        if (relu)
            for (int32_t j = 0; j < dout; j++)
                y[r * dout + j] = y[r * dout + j] > 0.0f ? y[r * dout + j] : 0.0f;
    }
}
