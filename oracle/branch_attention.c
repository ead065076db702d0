/*
 * CPU ORACLE -- test infrastructure only.  Nothing in the product path may call this.
 *
 * What it computes: the *baseline* the paper starts from (Section "Derivation", Eq. 1 and the
 * forward-equivalence requirement Eq. 6): every root-to-leaf branch of the trajectory tree is
 * treated as its own linear sequence and run through plain causal softmax attention, row by row,
 * with no tiling, no tree mask and no sharing between branches.  Gradients of the per-branch runs
 * are scatter-summed back onto the unique tokens (Eq. 5: the tree gradient is the sum of the
 * per-branch gradients).  The upstream gradient dO of a token that lies on g branches is split
 * evenly, dO/g per branch, so that the g branch copies together carry exactly dO (Eq. 2-4: a token
 * with g paths through it is counted g times in the per-branch sum).
 *
 * Arithmetic type: ORACLE_REAL (double unless overridden at compile time).
 * Layouts: q, d_o, o, dq: [n_tokens][hq][d]; k, v, dk, dv: [n_tokens][hkv][d]; lse: [hq][n_tokens].
 * Query head h uses key/value head h / (hq / hkv).
 *
 * Pure C99 + OpenMP.  No code is shared with the GPU library.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#else
static int omp_get_max_threads(void) { return 1; }
static int omp_get_thread_num(void) { return 0; }
#endif

#ifndef ORACLE_REAL
#define ORACLE_REAL double
#endif
typedef ORACLE_REAL real;

int oracle_real_bytes(void) { return (int)sizeof(real); }
int oracle_max_threads(void) { return omp_get_max_threads(); }

/* One query row of plain causal attention on a linear sequence given by token indices idx[0..r].
 * Forward: s_c = scale * <q, K[idx[c]]>, softmax over c = 0..r, o = sum_c p_c V[idx[c]],
 *          lse = log sum_c exp(s_c)   (natural log).
 * s_buf must hold r+1 reals.  k/v point at the head's first element; tok_stride_kv is the
 * distance between consecutive tokens. */
static void row_forward(int r, const int32_t *idx, int d, real scale,
                        const real *q_row, const float *k, const float *v, int64_t tok_stride_kv,
                        real *s_buf, real *o_row, real *lse_out)
{
    real m = -INFINITY;
    for (int c = 0; c <= r; c++) {
        const float *kc = k + (int64_t)idx[c] * tok_stride_kv;
        real acc = 0;
#pragma omp simd reduction(+ : acc)
        for (int e = 0; e < d; e++) acc += q_row[e] * (real)kc[e];
        acc *= scale;
        s_buf[c] = acc;
        if (acc > m) m = acc;
    }
    real l = 0;
    for (int c = 0; c <= r; c++) l += exp((double)(s_buf[c] - m));
    for (int e = 0; e < d; e++) o_row[e] = 0;
    for (int c = 0; c <= r; c++) {
        real p = (real)exp((double)(s_buf[c] - m)) / l;
        const float *vc = v + (int64_t)idx[c] * tok_stride_kv;
#pragma omp simd
        for (int e = 0; e < d; e++) o_row[e] += p * (real)vc[e];
    }
    *lse_out = m + (real)log((double)l);
}

/* Backward of the same row.  With P_c = exp(s_c - lse), D = <dO, O>, dP_c = <dO, V_c>,
 * dS_c = P_c (dP_c - D):   dq += scale * dS_c K_c;  dk_c += scale * dS_c q;  dv_c += P_c dO.
 * dk_loc / dv_loc are indexed by position c on the branch ([r+1][d]). */
static void row_backward(int r, const int32_t *idx, int d, real scale,
                         const real *q_row, const real *do_row, const real *o_row, real lse,
                         const float *k, const float *v, int64_t tok_stride_kv,
                         const real *s_buf, real *dq_row, real *dk_loc, real *dv_loc)
{
    real D = 0;
    for (int e = 0; e < d; e++) D += do_row[e] * o_row[e];
    for (int e = 0; e < d; e++) dq_row[e] = 0;
    for (int c = 0; c <= r; c++) {
        const float *kc = k + (int64_t)idx[c] * tok_stride_kv;
        const float *vc = v + (int64_t)idx[c] * tok_stride_kv;
        real p = (real)exp((double)(s_buf[c] - lse));
        real dp = 0;
#pragma omp simd reduction(+ : dp)
        for (int e = 0; e < d; e++) dp += do_row[e] * (real)vc[e];
        real ds = p * (dp - D);
        real sds = scale * ds;
        real *dkc = dk_loc + (int64_t)c * d;
        real *dvc = dv_loc + (int64_t)c * d;
#pragma omp simd
        for (int e = 0; e < d; e++) {
            dq_row[e] += sds * (real)kc[e];
            dkc[e] += sds * q_row[e];
            dvc[e] += p * do_row[e];
        }
    }
}

/*
 * Full per-branch oracle.
 *   paths: path_ptr[n_paths+1], path_idx[] = DFS token indices of each branch, root first.
 *   g_tok[t] = number of branches through token t (used only to split d_o).
 *   kvh_lo..kvh_hi: key/value head groups to process (all their query heads are processed, so every
 *   output that is written is complete); other heads' outputs are left untouched.
 *   d_o == NULL: forward only (dq, dk, dv ignored).
 * Outputs must be zero-initialised by the caller (dq, dk, dv are accumulated).
 * n_mismatch: number of (token, head) forward results that differed bitwise between two branches
 *   sharing the token -- the forward-equivalence self check (Eq. 6); must come out 0.
 * Returns 0, or -1 on allocation failure / bad arguments.
 */
int oracle_attn_branches(int64_t n_tokens, int hq, int hkv, int d, double scale_in,
                         const float *q, const float *k, const float *v, const float *d_o,
                         int n_paths, const int64_t *path_ptr, const int32_t *path_idx,
                         const int32_t *g_tok, int kvh_lo, int kvh_hi,
                         real *o, real *lse, real *dq, real *dk, real *dv,
                         int64_t *n_mismatch)
{
    if (hq % hkv != 0 || kvh_lo < 0 || kvh_hi > hkv) return -1;
    const int G = hq / hkv;
    const real scale = (real)scale_in;
    const int64_t sq = (int64_t)hq * d, skv = (int64_t)hkv * d;
    unsigned char *seen = (unsigned char *)calloc((size_t)(n_tokens * hq), 1);
    if (!seen) return -1;
    int64_t mismatch = 0;
    int failed = 0;
    const int n_tasks = (kvh_hi - kvh_lo) * n_paths;

#pragma omp parallel for ordered schedule(dynamic, 1)
    for (int task = 0; task < n_tasks; task++) {
        const int kvh = kvh_lo + task / n_paths;
        const int p = task % n_paths;
        const int32_t *idx = path_idx + path_ptr[p];
        const int L = (int)(path_ptr[p + 1] - path_ptr[p]);
        const int bwd = d_o != NULL;
        /* branch-local results for the G query heads of this group */
        real *o_loc = (real *)malloc(sizeof(real) * (size_t)G * L * d + 8);
        real *lse_loc = (real *)malloc(sizeof(real) * (size_t)G * L + 8);
        real *dq_loc = bwd ? (real *)malloc(sizeof(real) * (size_t)G * L * d + 8) : NULL;
        real *dk_loc = bwd ? (real *)calloc((size_t)L * d + 1, sizeof(real)) : NULL;
        real *dv_loc = bwd ? (real *)calloc((size_t)L * d + 1, sizeof(real)) : NULL;
        real *s_buf = (real *)malloc(sizeof(real) * (size_t)(L + 1));
        real *q_row = (real *)malloc(sizeof(real) * (size_t)d * 2);
        real *do_row = q_row + d;
        int ok = o_loc && lse_loc && s_buf && q_row && (!bwd || (dq_loc && dk_loc && dv_loc));
        if (ok) {
            for (int gq = 0; gq < G; gq++) {
                const int h = kvh * G + gq;
                const float *kh = k + (int64_t)kvh * d;
                const float *vh = v + (int64_t)kvh * d;
                for (int r = 0; r < L; r++) {
                    const int64_t t = idx[r];
                    for (int e = 0; e < d; e++) q_row[e] = (real)q[t * sq + (int64_t)h * d + e];
                    real *o_row = o_loc + ((int64_t)gq * L + r) * d;
                    row_forward(r, idx, d, scale, q_row, kh, vh, skv, s_buf, o_row,
                                &lse_loc[(int64_t)gq * L + r]);
                    if (bwd) {
                        const real inv_g = (real)1 / (real)g_tok[t];
                        for (int e = 0; e < d; e++)
                            do_row[e] = (real)d_o[t * sq + (int64_t)h * d + e] * inv_g;
                        row_backward(r, idx, d, scale, q_row, do_row, o_row,
                                     lse_loc[(int64_t)gq * L + r], kh, vh, skv, s_buf,
                                     dq_loc + ((int64_t)gq * L + r) * d, dk_loc, dv_loc);
                    }
                }
            }
        }
#pragma omp ordered
        {
            if (!ok) {
                failed = 1;
            } else {
                for (int gq = 0; gq < G; gq++) {
                    const int h = kvh * G + gq;
                    for (int r = 0; r < L; r++) {
                        const int64_t t = idx[r];
                        real *og = o + t * sq + (int64_t)h * d;
                        const real *ol = o_loc + ((int64_t)gq * L + r) * d;
                        real *lg = lse + (int64_t)h * n_tokens + t;
                        if (!seen[t * hq + h]) {
                            seen[t * hq + h] = 1;
                            memcpy(og, ol, sizeof(real) * (size_t)d);
                            *lg = lse_loc[(int64_t)gq * L + r];
                        } else if (memcmp(og, ol, sizeof(real) * (size_t)d) != 0 ||
                                   memcmp(lg, &lse_loc[(int64_t)gq * L + r], sizeof(real)) != 0) {
                            mismatch++;
                        }
                        if (bwd) {
                            real *dqg = dq + t * sq + (int64_t)h * d;
                            const real *dql = dq_loc + ((int64_t)gq * L + r) * d;
                            for (int e = 0; e < d; e++) dqg[e] += dql[e];
                        }
                    }
                }
                if (bwd) {
                    for (int r = 0; r < L; r++) {
                        const int64_t t = idx[r];
                        real *dkg = dk + t * skv + (int64_t)kvh * d;
                        real *dvg = dv + t * skv + (int64_t)kvh * d;
                        for (int e = 0; e < d; e++) {
                            dkg[e] += dk_loc[(int64_t)r * d + e];
                            dvg[e] += dv_loc[(int64_t)r * d + e];
                        }
                    }
                }
            }
        }
        free(o_loc); free(lse_loc); free(dq_loc); free(dk_loc); free(dv_loc); free(s_buf); free(q_row);
    }
    free(seen);
    if (n_mismatch) *n_mismatch = mismatch;
    return failed ? -1 : 0;
}

/*
 * Sampled oracle for sizes where the full per-branch run is too slow: the same per-row arithmetic,
 * evaluated only for the rows that the requested outputs depend on.
 *
 * Every query row t is run on its own branch prefix row_idx[row_ptr[i] .. row_ptr[i+1]) (the DFS
 * token indices of its root-to-t sequence, t last); which leaf the branch continues to does not
 * matter for row t, which is the content of Eq. 6.  Because the g branch copies of a row carry
 * dO/g each and are otherwise identical, their summed contribution equals one run with the full
 * dO; that is what is evaluated here (Eq. 2-5).
 *
 *   rows[n_rows]: query tokens to evaluate, for the G query heads of key/value head kvh.
 *   o_out [n_rows][G][d], lse_out [n_rows][G], dq_out [n_rows][G][d].
 *   key_tok[n_keys]: key tokens whose dk/dv are wanted; dk_out/dv_out [n_keys][d] accumulate
 *     the contributions of the evaluated rows only -- the caller must pass *every* row that can
 *     see a wanted key (all tokens of the key's subtree range from the key onwards).
 */
int oracle_attn_rows(int64_t n_tokens, int hq, int hkv, int d, double scale_in,
                     const float *q, const float *k, const float *v, const float *d_o,
                     int kvh, int n_rows, const int32_t *rows,
                     const int64_t *row_ptr, const int32_t *row_idx,
                     int n_keys, const int32_t *key_tok,
                     real *o_out, real *lse_out, real *dq_out, real *dk_out, real *dv_out)
{
    if (hq % hkv != 0 || kvh < 0 || kvh >= hkv) return -1;
    (void)n_tokens;
    const int G = hq / hkv;
    const real scale = (real)scale_in;
    const int64_t sq = (int64_t)hq * d, skv = (int64_t)hkv * d;
    const float *kh = k + (int64_t)kvh * d;
    const float *vh = v + (int64_t)kvh * d;
    int failed = 0;
    /* per-thread partial dk/dv for the wanted keys, reduced in thread order afterwards */
    int max_threads = omp_get_max_threads();
    real *part = (real *)calloc((size_t)max_threads * (size_t)(n_keys > 0 ? n_keys : 1) * d * 2, sizeof(real));
    if (!part) return -1;

#pragma omp parallel
    {
        const int tid = omp_get_thread_num();
        real *dk_part = part + (size_t)tid * (size_t)(n_keys > 0 ? n_keys : 1) * d * 2;
        real *dv_part = dk_part + (size_t)(n_keys > 0 ? n_keys : 1) * d;
#pragma omp for schedule(static)
        for (int i = 0; i < n_rows; i++) {
            const int32_t *idx = row_idx + row_ptr[i];
            const int L = (int)(row_ptr[i + 1] - row_ptr[i]);
            const int r = L - 1;
            const int64_t t = rows[i];
            real *s_buf = (real *)malloc(sizeof(real) * (size_t)(L + 1));
            real *q_row = (real *)malloc(sizeof(real) * (size_t)d * 4);
            real *dk_loc = d_o ? (real *)malloc(sizeof(real) * (size_t)L * d + 8) : NULL;
            real *dv_loc = d_o ? (real *)malloc(sizeof(real) * (size_t)L * d + 8) : NULL;
            if (!s_buf || !q_row || (d_o && (!dk_loc || !dv_loc)) || idx[r] != t) {
#pragma omp atomic write
                failed = 1;
            } else {
                real *do_row = q_row + d, *o_row = q_row + 2 * d, *dq_row = q_row + 3 * d;
                for (int gq = 0; gq < G; gq++) {
                    const int h = kvh * G + gq;
                    for (int e = 0; e < d; e++) q_row[e] = (real)q[t * sq + (int64_t)h * d + e];
                    real lse_v;
                    row_forward(r, idx, d, scale, q_row, kh, vh, skv, s_buf, o_row, &lse_v);
                    if (o_out) memcpy(o_out + ((int64_t)i * G + gq) * d, o_row, sizeof(real) * (size_t)d);
                    if (lse_out) lse_out[(int64_t)i * G + gq] = lse_v;
                    if (d_o) {
                        for (int e = 0; e < d; e++) do_row[e] = (real)d_o[t * sq + (int64_t)h * d + e];
                        memset(dk_loc, 0, sizeof(real) * (size_t)L * d);
                        memset(dv_loc, 0, sizeof(real) * (size_t)L * d);
                        row_backward(r, idx, d, scale, q_row, do_row, o_row, lse_v, kh, vh, skv, s_buf,
                                     dq_row, dk_loc, dv_loc);
                        if (dq_out) memcpy(dq_out + ((int64_t)i * G + gq) * d, dq_row, sizeof(real) * (size_t)d);
                        for (int kk = 0; kk < n_keys; kk++) {
                            /* position of the wanted key on this row's branch, if it is there */
                            for (int c = 0; c <= r; c++) {
                                if (idx[c] == key_tok[kk]) {
                                    for (int e = 0; e < d; e++) {
                                        dk_part[(int64_t)kk * d + e] += dk_loc[(int64_t)c * d + e];
                                        dv_part[(int64_t)kk * d + e] += dv_loc[(int64_t)c * d + e];
                                    }
                                    break;
                                }
                            }
                        }
                    }
                }
            }
            free(s_buf); free(q_row); free(dk_loc); free(dv_loc);
        }
    }
    if (dk_out && dv_out) {
        for (int tid = 0; tid < max_threads; tid++) {
            const real *dk_part = part + (size_t)tid * (size_t)(n_keys > 0 ? n_keys : 1) * d * 2;
            const real *dv_part = dk_part + (size_t)(n_keys > 0 ? n_keys : 1) * d;
            for (int64_t x = 0; x < (int64_t)n_keys * d; x++) {
                dk_out[x] += dk_part[x];
                dv_out[x] += dv_part[x];
            }
        }
    }
    free(part);
    return failed ? -1 : 0;
}
