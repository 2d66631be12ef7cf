/*
 * CPU fp64 oracle for the backward pass of the GLA token mixer of DiG.
 * TEST INFRASTRUCTURE ONLY (see gla_oracle.c): nothing in the product path may
 * call, link or load this file.
 *
 * The forward recurrence (Sec. 3.1, Eq. (attn_gla), rows 1-3, beta = 1), along
 * scan step s = 0 .. T-1 visiting token n = pi(s), from S_{-1} = 0:
 *
 *     A_s = exp(log_alpha_n)      S_s = diag(A_s) S_{s-1} + k_n^T v_n      o_n = q_n S_s
 *
 * Given dO = dL/d out for a scalar L that depends on `out` only, this file
 * differentiates those three assignments one scan step at a time, last step
 * first (reverse-mode differentiation written out; the paper does not print
 * the backward pass, it only states that training uses it).  With
 * G = dL/dS_s, accumulated from the later steps:
 *
 *     G      += q_n^T dO_n                      (o_n = q_n S_s)
 *     dq_n[c] = sum_j S_s[c,j] dO_n[j]
 *     dk_n[c] = sum_j G[c,j] v_n[j]             (S_s contains k_n^T v_n)
 *     dv_n[j] = sum_c k_n[c] G[c,j]
 *     dlog_alpha_n[c] = A_s[c] * sum_j G[c,j] S_{s-1}[c,j]     (S_s contains diag(A_s) S_{s-1})
 *     G       = diag(A_s) G                     (now dL/dS_{s-1})
 *
 * The states S_s are needed again in reverse order; they are recomputed from
 * checkpoints kept every kBlock steps by the same forward assignment, so that
 * nothing is reordered or approximated.
 *
 * Layouts as in gla_oracle.c: q, k, log_alpha, dq, dk, dlog_alpha : [B,H,T,dk];
 * v, d_out, dv : [B,H,T,dv]; all doubles.
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

long gla_oracle_scan_index(int scan_dir, long s, int grid_h, int grid_w);

enum { kBlock = 128 };

static void step_forward(double *S, const double *kn, const double *vn, const double *gn, int dk, int dv)
{
    for (int c = 0; c < dk; ++c) {
        double a = exp(gn[c]);
        double *Sc = S + (long)c * dv;
        for (int j = 0; j < dv; ++j)
            Sc[j] = a * Sc[j] + kn[c] * vn[j];
    }
}

/* Returns 0 on success, 1 on a bad argument or failed allocation. nthreads <= 0 means "all". */
int gla_oracle_bwd(const double *q, const double *k, const double *v,
                   const double *log_alpha, const double *d_out,
                   int B, int H, int T, int dk, int dv,
                   int grid_h, int grid_w, int scan_dir,
                   double *dq, double *dk_out, double *dv_out, double *dlog_alpha, int nthreads)
{
    if (!q || !k || !v || !log_alpha || !d_out || !dq || !dk_out || !dv_out || !dlog_alpha) return 1;
    if (B <= 0 || H <= 0 || T <= 0 || dk <= 0 || dv <= 0) return 1;
    if (grid_h <= 0 || grid_w <= 0 || (long)grid_h * grid_w != (long)T) return 1;
    if (scan_dir < 0 || scan_dir > 3) return 1;

    const long BH = (long)B * H;
    const long ne = (long)dk * dv;
    const long nblocks = ((long)T + kBlock - 1) / kBlock;
    int failed = 0;
#ifdef _OPENMP
    if (nthreads <= 0) nthreads = omp_get_max_threads();
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads)
#endif
    for (long bh = 0; bh < BH; ++bh) {
        /* check[b] = state before the first step of block b; blk[i] = state after step i-1 of the current block */
        double *check = (double *)malloc(sizeof(double) * (size_t)(nblocks * ne));
        double *blk = (double *)malloc(sizeof(double) * (size_t)((kBlock + 1) * ne));
        double *G = (double *)calloc((size_t)ne, sizeof(double));
        if (!check || !blk || !G) { failed = 1; free(check); free(blk); free(G); continue; }

        const double *qs = q + bh * (long)T * dk, *ks = k + bh * (long)T * dk;
        const double *gs = log_alpha + bh * (long)T * dk;
        const double *vs = v + bh * (long)T * dv, *dos = d_out + bh * (long)T * dv;
        double *dqs = dq + bh * (long)T * dk, *dks = dk_out + bh * (long)T * dk;
        double *dgs = dlog_alpha + bh * (long)T * dk, *dvs = dv_out + bh * (long)T * dv;

        /* forward sweep: checkpoints only */
        memset(blk, 0, sizeof(double) * (size_t)ne);
        for (long s = 0; s < T; ++s) {
            if (s % kBlock == 0) memcpy(check + (s / kBlock) * ne, blk, sizeof(double) * (size_t)ne);
            long n = gla_oracle_scan_index(scan_dir, s, grid_h, grid_w);
            step_forward(blk, ks + n * dk, vs + n * dv, gs + n * dk, dk, dv);
        }

        /* reverse sweep, block by block */
        for (long b = nblocks - 1; b >= 0; --b) {
            const long s0 = b * kBlock;
            const long s1 = (s0 + kBlock < T) ? s0 + kBlock : T;
            memcpy(blk, check + b * ne, sizeof(double) * (size_t)ne);
            for (long s = s0; s < s1; ++s) {
                double *next = blk + (s - s0 + 1) * ne;
                memcpy(next, blk + (s - s0) * ne, sizeof(double) * (size_t)ne);
                long n = gla_oracle_scan_index(scan_dir, s, grid_h, grid_w);
                step_forward(next, ks + n * dk, vs + n * dv, gs + n * dk, dk, dv);
            }
            for (long s = s1 - 1; s >= s0; --s) {
                const long n = gla_oracle_scan_index(scan_dir, s, grid_h, grid_w);
                const double *S_prev = blk + (s - s0) * ne, *S_cur = blk + (s - s0 + 1) * ne;
                const double *qn = qs + n * dk, *kn = ks + n * dk, *gn = gs + n * dk;
                const double *vn = vs + n * dv, *don = dos + n * dv;
                for (int c = 0; c < dk; ++c)
                    for (int j = 0; j < dv; ++j)
                        G[(long)c * dv + j] += qn[c] * don[j];
                for (int c = 0; c < dk; ++c) {
                    const double a = exp(gn[c]);
                    double sq = 0.0, sk = 0.0, sa = 0.0;
                    for (int j = 0; j < dv; ++j) {
                        sq += S_cur[(long)c * dv + j] * don[j];
                        sk += G[(long)c * dv + j] * vn[j];
                        sa += G[(long)c * dv + j] * S_prev[(long)c * dv + j];
                    }
                    dqs[n * dk + c] = sq;
                    dks[n * dk + c] = sk;
                    dgs[n * dk + c] = a * sa;
                }
                for (int j = 0; j < dv; ++j) {
                    double sv = 0.0;
                    for (int c = 0; c < dk; ++c)
                        sv += kn[c] * G[(long)c * dv + j];
                    dvs[n * dv + j] = sv;
                }
                for (int c = 0; c < dk; ++c) {
                    const double a = exp(gn[c]);
                    for (int j = 0; j < dv; ++j)
                        G[(long)c * dv + j] *= a;
                }
            }
        }
        free(check); free(blk); free(G);
    }
    return failed;
}
