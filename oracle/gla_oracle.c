/*
 * CPU fp64 oracle for the forward pass of the gated-linear-attention (GLA)
 * token mixer of DiG.  TEST INFRASTRUCTURE ONLY: nothing in the product path
 * may call, link or load this file; it exists so that the GPU kernels can be
 * checked against something that is obviously the definition.
 *
 * What it computes (the recurrence of Sec. 3.1, "Gated Linear Attention
 * Transformer", Eq. (attn_gla), first three rows, with the gate restricted to
 * its key-side factor alpha_t, i.e. beta_t = 1):
 *
 *     S'_{t-1} = diag(alpha_t) S_{t-1}           (row c of S scaled by alpha_t[c])
 *     S_t      = S'_{t-1} + k_t^T v_t            (outer product, dk x dv)
 *     o_t      = q_t S_t                         (row vector times matrix)
 *
 * taken token by token, S_0 = 0 unless an initial state is handed in, in fp64,
 * along one of the four scan orders that the DiG block produces by alternating
 * transpose and flip of the token grid (Sec. 3.3, Algorithm 1; the flattening /
 * transposing / flipping operators of the supplementary Algorithms 2-4).
 * The gate arrives as log_alpha = log(alpha) <= 0; alpha = exp(log_alpha).
 *
 * Readings of the paper taken here:
 *   - the printed "Q_t^T S_t" cannot be a 1 x dv row unless it means q_t S_t;
 *   - o_t reads S_t, the state that already contains token t, and alpha_t
 *     decays only what came before token t;
 *   - "flip" reverses the flattened 1-D sequence; "transpose" swaps grid rows
 *     and columns before flattening, so a column scan walks down a column of
 *     grid_h tokens and then moves to the next column.
 *
 * There is no blocking, no chunking and no reordering in here.
 *
 * Layouts (row-major, canonical row-major grid order for every scan order):
 *   q, k, log_alpha : [B, H, T, dk]     v, out : [B, H, T, dv]
 *   init_state (may be NULL), final_state (may be NULL) : [B, H, dk, dv]
 * Inputs are doubles: the caller up-casts bf16 / fp32 values exactly.
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

enum { SCAN_ROW_FWD = 0, SCAN_ROW_REV = 1, SCAN_COL_FWD = 2, SCAN_COL_REV = 3 };

/* Scan step s (0-based) -> canonical token index n = r * grid_w + c.
 * Row-major order visits n = s.  Column-major order is the row-major order of
 * the transposed grid: step s sits at column s / grid_h, row s % grid_h.
 * The reversed orders visit the same sequence from its last step backwards. */
long gla_oracle_scan_index(int scan_dir, long s, int grid_h, int grid_w)
{
    long T = (long)grid_h * (long)grid_w;
    if (scan_dir == SCAN_ROW_REV || scan_dir == SCAN_COL_REV)
        s = T - 1 - s;
    if (scan_dir == SCAN_ROW_FWD || scan_dir == SCAN_ROW_REV)
        return s;
    long c = s / grid_h;
    long r = s % grid_h;
    return r * (long)grid_w + c;
}

int gla_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Returns 0 on success, 1 on a bad argument. nthreads <= 0 means "all". */
int gla_oracle_fwd(const double *q, const double *k, const double *v,
                   const double *log_alpha, const double *init_state,
                   int B, int H, int T, int dk, int dv,
                   int grid_h, int grid_w, int scan_dir,
                   double *out, double *final_state, int nthreads)
{
    if (!q || !k || !v || !log_alpha || !out) return 1;
    if (B <= 0 || H <= 0 || T <= 0 || dk <= 0 || dv <= 0) return 1;
    if (grid_h <= 0 || grid_w <= 0 || (long)grid_h * grid_w != (long)T) return 1;
    if (scan_dir < 0 || scan_dir > 3) return 1;

    long BH = (long)B * H;
    int failed = 0;
#ifdef _OPENMP
    if (nthreads <= 0) nthreads = omp_get_max_threads();
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads)
#endif
    for (long bh = 0; bh < BH; ++bh) {
        double *S = (double *)malloc(sizeof(double) * (size_t)dk * dv);
        if (!S) { failed = 1; continue; }
        if (init_state)
            memcpy(S, init_state + bh * dk * dv, sizeof(double) * (size_t)dk * dv);
        else
            memset(S, 0, sizeof(double) * (size_t)dk * dv);

        const double *qs = q + bh * (long)T * dk;
        const double *ks = k + bh * (long)T * dk;
        const double *gs = log_alpha + bh * (long)T * dk;
        const double *vs = v + bh * (long)T * dv;
        double *os = out + bh * (long)T * dv;

        for (long s = 0; s < T; ++s) {
            long n = gla_oracle_scan_index(scan_dir, s, grid_h, grid_w);
            const double *qn = qs + n * dk, *kn = ks + n * dk, *gn = gs + n * dk;
            const double *vn = vs + n * dv;
            double *on = os + n * dv;
            /* decay the old state by the current token's gate, then add k^T v */
            for (int c = 0; c < dk; ++c) {
                double a = exp(gn[c]);
                double *Sc = S + (long)c * dv;
                for (int j = 0; j < dv; ++j)
                    Sc[j] = a * Sc[j] + kn[c] * vn[j];
            }
            /* read the updated state with the query */
            for (int j = 0; j < dv; ++j) {
                double acc = 0.0;
                for (int c = 0; c < dk; ++c)
                    acc += qn[c] * S[(long)c * dv + j];
                on[j] = acc;
            }
        }
        if (final_state)
            memcpy(final_state + bh * dk * dv, S, sizeof(double) * (size_t)dk * dv);
        free(S);
    }
    return failed;
}
