/*
 * CPU oracle for CSB-RNN inference.  TEST INFRASTRUCTURE ONLY: nothing in the product
 * path may call this file; only the tests, the smoke check and the benchmark's
 * cpu_baseline leg do.  It shares no code with the HIP library.
 *
 * What it computes, and where the paper defines it:
 *   - the CSB encoding of a block-structured pruned matrix and its inverse
 *     (Sec. 3.1.1: per block the kernel-matrix row and column counts, the indices of the
 *     surviving rows and columns, and the kernel values of successive blocks, blocks in
 *     row-major order, concatenated);
 *   - y = A x and Y = A X on the DECOMPRESSED dense matrix, float64 accumulation
 *     (CSB is a lossless encoding, so CSB-MVM of Sec. 4.3.1 equals the plain product); beside
 *     it CSB-MVM on the encoded arrays in float32, a timed baseline that is itself checked
 *     against the float64 product;
 *   - LSTM and GRU inference over a sequence (Sec. 2.1: mat-vec of the weight matrices
 *     with input and hidden vectors, then sigmoid / tanh / element-wise products and
 *     sums, with c_{t-1}, h_{t-1} carried to the next step), float64 throughout; also the
 *     LSTM with a recurrent projection layer (LSTMP) that the paper's speech model SR1 uses
 *     (Table 1);
 *
 * Readings where the paper is silent (its cell equations sit in a figure):
 *   - LSTM without peepholes, gate rows stacked i,f,g,o; W = [W_x | W_h], one bias;
 *   - GRU in the "reset after the recurrent product" form, rows stacked r,z,n;
 *   - inside a block the kernel is stored row-major; indices ascend;
 *   - "non-zero" means v != 0.0f (so -0.0 is zero and NaN is kept);
 *   - edge blocks of a ragged matrix are truncated.
 *
 *   - the projection of a dense matrix onto the CSB pattern at a given pruning rate (the
 *     pruning step inside Algorithm 1, described in Sec. 3.2.2: partition into blocks; in
 *     every block-column rank the in-block row segments by the sum of their squares and zero
 *     the weakest share 1 - sqrt(1 - PruneRate); then the same for the in-block column
 *     segments of every block-row, on the row-pruned matrix).
 *
 * Readings for the projection (the paper gives the procedure in words only):
 *   - "PruneRate" is the pruned fraction 1 - 1/rate for a rate given as "rate x";
 *   - the ranking runs over ALL row segments of a block-column (all column segments of a
 *     block-row), so the kept count varies from block to block, as Sec. 3.1.2 says it does;
 *   - the number zeroed among n segments is floor(n * (1 - rate^-1/2) + 1/2);
 *   - ties and the decision itself: the sum of squares is accumulated in float32, left to
 *     right (top to bottom), one fused multiply-add per element -- the arithmetic of the
 *     device kernel, because the decision must be taken in one precision on both sides;
 *     equal sums are ranked by position (the earlier segment is the weaker); a NaN sum
 *     ranks above everything (its segment is kept);
 *   - surviving entries keep their bits, pruned entries become +0.0.
 *
 * Parity pins (tests/test_oracle_*.py): a hand-worked two-block example, brute force on
 * tiny matrices, numpy's float64 product, torch.nn.LSTM / torch.nn.GRU in float64 on the
 * CPU (LSTMP: torch.nn.LSTM with proj_size), closed forms for zero weights, encode/decode
 * invariants; for the projection a
 * hand-worked example, exact integer brute force on tiny matrices, kept-count and
 * pattern invariants.  No function here is "parity unpinned".
 *
 * Plain loops on purpose: no blocking, no fusion, no reordering.  The only concession to
 * run time is an OpenMP "parallel for" over output rows, which does not change any sum.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int orc_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void orc_set_threads(int n) {
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

static int64_t imin64(int64_t a, int64_t b) { return a < b ? a : b; }

/*
 * CSB encoding (Sec. 3.1.1).  Blocks are visited in row-major order.  In block b the kept
 * rows are those with any non-zero inside the block, likewise the kept columns; the
 * kernel is the sub-matrix at their cross-points (zeros at cross-points stay, as values).
 *
 * Outputs may be NULL to only count.  nrows/ncols have one entry per block.  rowidx /
 * colidx / val are filled up to the given capacities; the totals are returned in tot[3] =
 * {sum of kernel sizes, sum of kept rows, sum of kept cols}.  Returns 0, or -1 if a
 * capacity was too small or an argument invalid.
 */
int orc_csb_encode(const float *A, int64_t R, int64_t C, int64_t ld, int32_t BR, int32_t BC,
                   int32_t *nrows, int32_t *ncols,
                   uint16_t *rowidx, int64_t cap_row, uint16_t *colidx, int64_t cap_col,
                   float *val, int64_t cap_val, int64_t tot[3]) {
    if (!A || R <= 0 || C <= 0 || ld < C || BR <= 0 || BC <= 0 || !tot) return -1;
    int64_t nbr = (R + BR - 1) / BR, nbc = (C + BC - 1) / BC;
    int64_t nv = 0, nr = 0, nc = 0;
    int *keep_r = (int *)malloc(sizeof(int) * (size_t)BR);
    int *keep_c = (int *)malloc(sizeof(int) * (size_t)BC);
    int status = 0;
    for (int64_t bi = 0; bi < nbr; ++bi) {
        for (int64_t bj = 0; bj < nbc; ++bj) {
            int64_t r0 = bi * BR, c0 = bj * BC;
            int64_t h = imin64(BR, R - r0), w = imin64(BC, C - c0);
            for (int64_t i = 0; i < h; ++i) keep_r[i] = 0;
            for (int64_t j = 0; j < w; ++j) keep_c[j] = 0;
            for (int64_t i = 0; i < h; ++i)
                for (int64_t j = 0; j < w; ++j)
                    if (A[(r0 + i) * ld + (c0 + j)] != 0.0f) { keep_r[i] = 1; keep_c[j] = 1; }
            int32_t rb = 0, cb = 0;
            for (int64_t i = 0; i < h; ++i) rb += keep_r[i];
            for (int64_t j = 0; j < w; ++j) cb += keep_c[j];
            int64_t b = bi * nbc + bj;
            if (nrows) nrows[b] = rb;
            if (ncols) ncols[b] = cb;
            for (int64_t i = 0; i < h; ++i) {
                if (!keep_r[i]) continue;
                if (rowidx) { if (nr < cap_row) rowidx[nr] = (uint16_t)i; else status = -1; }
                ++nr;
            }
            for (int64_t j = 0; j < w; ++j) {
                if (!keep_c[j]) continue;
                if (colidx) { if (nc < cap_col) colidx[nc] = (uint16_t)j; else status = -1; }
                ++nc;
            }
            for (int64_t i = 0; i < h; ++i) {
                if (!keep_r[i]) continue;
                for (int64_t j = 0; j < w; ++j) {
                    if (!keep_c[j]) continue;
                    if (val) { if (nv < cap_val) val[nv] = A[(r0 + i) * ld + (c0 + j)]; else status = -1; }
                    ++nv;
                }
            }
        }
    }
    free(keep_r);
    free(keep_c);
    tot[0] = nv; tot[1] = nr; tot[2] = nc;
    return status;
}

/* Inverse of the encoding: writes the full R x C matrix (zeros elsewhere).  The arrays are
 * consumed strictly sequentially, as the format intends (it stores no offsets). */
int orc_csb_decode(int64_t R, int64_t C, int32_t BR, int32_t BC,
                   const int32_t *nrows, const int32_t *ncols,
                   const uint16_t *rowidx, const uint16_t *colidx, const float *val,
                   float *A, int64_t ld) {
    if (!A || R <= 0 || C <= 0 || ld < C || BR <= 0 || BC <= 0) return -1;
    int64_t nbr = (R + BR - 1) / BR, nbc = (C + BC - 1) / BC;
    for (int64_t i = 0; i < R; ++i)
        for (int64_t j = 0; j < C; ++j) A[i * ld + j] = 0.0f;
    int64_t pv = 0, pr = 0, pc = 0;
    for (int64_t bi = 0; bi < nbr; ++bi) {
        for (int64_t bj = 0; bj < nbc; ++bj) {
            int64_t b = bi * nbc + bj;
            int32_t rb = nrows[b], cb = ncols[b];
            for (int32_t i = 0; i < rb; ++i) {
                int64_t gi = bi * BR + rowidx[pr + i];
                if (gi >= R) return -1;
                for (int32_t j = 0; j < cb; ++j) {
                    int64_t gj = bj * BC + colidx[pc + j];
                    if (gj >= C) return -1;
                    A[gi * ld + gj] = val[pv + (int64_t)i * cb + j];
                }
            }
            pv += (int64_t)rb * cb; pr += rb; pc += cb;
        }
    }
    return 0;
}

/* y = A x; A float32 widened, float64 accumulation in column order. */
void orc_matvec(const float *A, int64_t R, int64_t C, int64_t ld, const float *x, double *y) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < R; ++i) {
        double s = 0.0;
        for (int64_t j = 0; j < C; ++j) s += (double)A[i * ld + j] * (double)x[j];
        y[i] = s;
    }
}

/*
 * CSB-MVM straight on the encoded arrays, in float32 (Sec. 4.3.1: for every block the kernel
 * matrix times the inputs that its column indices select, added to the outputs that its row
 * indices name; the blocks of a block-row accumulate one after another).  The like-for-like
 * CPU baseline of the device kernels, timed by the benchmark; NOT the parity reference, which
 * is orc_matvec on the decompressed matrix in float64 (this function is itself checked
 * against it).  val_off / row_off / col_off are the exclusive prefix sums of the counts.
 */
void orc_csb_matvec_f32(int64_t R, int64_t C, int32_t BR, int32_t BC,
                        const int32_t *nrows, const int32_t *ncols,
                        const uint16_t *rowidx, const uint16_t *colidx, const float *val,
                        const int64_t *val_off, const int64_t *row_off, const int64_t *col_off,
                        const float *x, float *y) {
    int64_t nbr = (R + BR - 1) / BR, nbc = (C + BC - 1) / BC;
#pragma omp parallel for schedule(static)
    for (int64_t bi = 0; bi < nbr; ++bi) {
        int64_t r0 = bi * BR, h = imin64(BR, R - r0);
        for (int64_t i = 0; i < h; ++i) y[r0 + i] = 0.0f;
        for (int64_t bj = 0; bj < nbc; ++bj) {
            int64_t b = bi * nbc + bj;
            int32_t rb = nrows[b], cb = ncols[b];
            const float *k = val + val_off[b];
            const uint16_t *ri = rowidx + row_off[b], *ci = colidx + col_off[b];
            for (int32_t i = 0; i < rb; ++i) {
                float s = 0.0f;
                for (int32_t j = 0; j < cb; ++j) s += k[(int64_t)i * cb + j] * x[bj * BC + ci[j]];
                y[r0 + ri[i]] += s;
            }
        }
    }
}

/* Per-row sum of |a_ij x_j| (the scale of the textbook dot-product rounding bound). */
void orc_matvec_abs(const float *A, int64_t R, int64_t C, int64_t ld, const float *x, double *y) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < R; ++i) {
        double s = 0.0;
        for (int64_t j = 0; j < C; ++j) s += fabs((double)A[i * ld + j] * (double)x[j]);
        y[i] = s;
    }
}

/* Y = A X; X is [C][ldx] (column k = right-hand side k), Y is [R][ldy], nb columns. */
void orc_matmat(const float *A, int64_t R, int64_t C, int64_t ld,
                const float *X, int64_t ldx, double *Y, int64_t ldy, int64_t nb) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < R; ++i) {
        for (int64_t k = 0; k < nb; ++k) {
            double s = 0.0;
            for (int64_t j = 0; j < C; ++j) s += (double)A[i * ld + j] * (double)X[j * ldx + k];
            Y[i * ldy + k] = s;
        }
    }
}

/* Selected rows of Y = A X (for sampled checks at full size): rows[k], k < nsel. */
void orc_matmat_rows(const float *A, int64_t C, int64_t ld, const int64_t *rows, int64_t nsel,
                     const float *X, int64_t ldx, double *Y, int64_t ldy, int64_t nb) {
#pragma omp parallel for schedule(static)
    for (int64_t q = 0; q < nsel; ++q) {
        int64_t i = rows[q];
        for (int64_t k = 0; k < nb; ++k) {
            double s = 0.0;
            for (int64_t j = 0; j < C; ++j) s += (double)A[i * ld + j] * (double)X[j * ldx + k];
            Y[q * ldy + k] = s;
        }
    }
}

static double sigmoid(double v) { return 1.0 / (1.0 + exp(-v)); }

/*
 * One layer, one time step, one sequence of the batch (Sec. 2.1; cell arithmetic after
 * the works the paper cites for LSTM and GRU).
 *   cell 0, LSTM: a = W [u; h] + b, rows i,f,g,o;
 *                 c' = sig(a_f) c + sig(a_i) tanh(a_g);  h' = sig(a_o) tanh(c')
 *   cell 1, GRU : ax = W[:, :n_in] u, ah = W[:, n_in:] h, rows r,z,n;
 *                 r = sig(ax_r + ah_r + b_r), z = sig(ax_z + ah_z + b_z),
 *                 n = tanh(ax_n + b_n + r ah_n);  h' = (1 - z) n + z h
 *   cell 3, Li-GRU (the cell of the paper's SR3 model, Table 1; as published by its authors,
 *                 with the batch normalisation of the input part folded into W and b, which
 *                 is what it is at inference): rows z, c;
 *                 z = sig(a_z), cand = max(a_c, 0);  h' = z h + (1 - z) cand
 *   cell 4, GRU with the reset gate applied BEFORE the recurrent product (the form of the
 *                 work the paper cites for GRU): r, z as in cell 1, then
 *                 n = tanh(ax_n + b_n + W[n rows, n_in:] (r * h));  h' = (1 - z) n + z h
 * W is (G*H) x (n_in + H) dense float32 with leading dimension n_in + H.
 */
static void cell_step(int cell, int64_t n_in, int64_t H, const float *W, const float *bias,
                      const double *u, double *h, double *c, double *ax, double *ah) {
    int64_t G = cell == 0 ? 4 : (cell == 3 ? 2 : 3), ld = n_in + H;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < G * H; ++i) {
        double sx = 0.0, sh = 0.0;
        for (int64_t j = 0; j < n_in; ++j) sx += (double)W[i * ld + j] * u[j];
        for (int64_t j = 0; j < H; ++j) sh += (double)W[i * ld + n_in + j] * h[j];
        ax[i] = sx; ah[i] = sh;
    }
    if (cell == 0) {
        for (int64_t k = 0; k < H; ++k) {
            double ai = ax[k] + ah[k] + (bias ? (double)bias[k] : 0.0);
            double af = ax[H + k] + ah[H + k] + (bias ? (double)bias[H + k] : 0.0);
            double ag = ax[2 * H + k] + ah[2 * H + k] + (bias ? (double)bias[2 * H + k] : 0.0);
            double ao = ax[3 * H + k] + ah[3 * H + k] + (bias ? (double)bias[3 * H + k] : 0.0);
            double cn = sigmoid(af) * c[k] + sigmoid(ai) * tanh(ag);
            c[k] = cn;
            h[k] = sigmoid(ao) * tanh(cn);
        }
    } else if (cell == 1) {
        for (int64_t k = 0; k < H; ++k) {
            double br = bias ? (double)bias[k] : 0.0;
            double bz = bias ? (double)bias[H + k] : 0.0;
            double bn = bias ? (double)bias[2 * H + k] : 0.0;
            double r = sigmoid(ax[k] + ah[k] + br);
            double z = sigmoid(ax[H + k] + ah[H + k] + bz);
            double n = tanh(ax[2 * H + k] + bn + r * ah[2 * H + k]);
            /* all ah were formed from the old h before any h[k] is replaced */
            h[k] = (1.0 - z) * n + z * h[k];
        }
    } else if (cell == 3) {
        for (int64_t k = 0; k < H; ++k) {
            double bz = bias ? (double)bias[k] : 0.0;
            double bc = bias ? (double)bias[H + k] : 0.0;
            double z = sigmoid(ax[k] + ah[k] + bz);
            double pre = ax[H + k] + ah[H + k] + bc;
            double cand = pre > 0.0 ? pre : 0.0;
            h[k] = z * h[k] + (1.0 - z) * cand;
        }
    } else {
        /* reset-before: the candidate's recurrent product is taken of q = r * h, so it can
           only be formed once every r is known (ah's n rows, formed from h, are not used) */
        double *q = (double *)malloc(sizeof(double) * (size_t)H);
        for (int64_t k = 0; k < H; ++k) {
            double br = bias ? (double)bias[k] : 0.0;
            q[k] = sigmoid(ax[k] + ah[k] + br) * h[k];
        }
        for (int64_t k = 0; k < H; ++k) {
            double s = 0.0;
            for (int64_t j = 0; j < H; ++j) s += (double)W[(2 * H + k) * ld + n_in + j] * q[j];
            ah[2 * H + k] = s;
        }
        for (int64_t k = 0; k < H; ++k) {
            double bz = bias ? (double)bias[H + k] : 0.0;
            double bn = bias ? (double)bias[2 * H + k] : 0.0;
            double z = sigmoid(ax[H + k] + ah[H + k] + bz);
            double n = tanh(ax[2 * H + k] + bn + ah[2 * H + k]);
            h[k] = (1.0 - z) * n + z * h[k];
        }
        free(q);
    }
}

/*
 * Stacked RNN over a sequence.  Layer l at time t reads the layer below at the same t.
 *   x    [T][B][I] float32        h0,c0 [L][B][H] float64 or NULL (zeros)
 *   hseq [T][B][H] float64 of the last layer, or NULL
 *   hT,cT [L][B][H] float64 (cT may be NULL; only the LSTM has a c)
 * W[l] dense (G*H) x (in_l + H), in_0 = I, in_l = H; bias[l] of G*H or NULL;
 * G = 4 (LSTM), 3 (both GRU forms), 2 (Li-GRU).
 */
int orc_rnn_forward(int cell, int32_t L, int64_t I, int64_t H,
                    const float *const *W, const float *const *bias,
                    const float *x, const double *h0, const double *c0,
                    double *hseq, double *hT, double *cT, int64_t T, int64_t B) {
    if ((cell != 0 && cell != 1 && cell != 3 && cell != 4) || L <= 0 || I <= 0 || H <= 0 || T < 0 || B <= 0 || !W || !hT) return -1;
    int64_t G = cell == 0 ? 4 : (cell == 3 ? 2 : 3);
    int64_t maxin = I > H ? I : H;
    double *h = (double *)calloc((size_t)(L * B * H), sizeof(double));
    double *c = (double *)calloc((size_t)(L * B * H), sizeof(double));
    double *u = (double *)malloc(sizeof(double) * (size_t)maxin);
    double *ax = (double *)malloc(sizeof(double) * (size_t)(G * H));
    double *ah = (double *)malloc(sizeof(double) * (size_t)(G * H));
    if (h0) memcpy(h, h0, sizeof(double) * (size_t)(L * B * H));
    if (c0) memcpy(c, c0, sizeof(double) * (size_t)(L * B * H));
    for (int64_t t = 0; t < T; ++t) {
        for (int64_t s = 0; s < B; ++s) {
            for (int32_t l = 0; l < L; ++l) {
                int64_t n_in = l == 0 ? I : H;
                if (l == 0) for (int64_t j = 0; j < I; ++j) u[j] = (double)x[(t * B + s) * I + j];
                else        for (int64_t j = 0; j < H; ++j) u[j] = h[((l - 1) * B + s) * H + j];
                cell_step(cell, n_in, H, W[l], bias ? bias[l] : NULL, u,
                          h + (l * B + s) * H, c + (l * B + s) * H, ax, ah);
            }
            if (hseq) for (int64_t k = 0; k < H; ++k) hseq[(t * B + s) * H + k] = h[((L - 1) * B + s) * H + k];
        }
    }
    memcpy(hT, h, sizeof(double) * (size_t)(L * B * H));
    if (cT) memcpy(cT, c, sizeof(double) * (size_t)(L * B * H));
    free(h); free(c); free(u); free(ax); free(ah);
    return 0;
}


/* ------------------------------------------------------------------ LSTM with a recurrent projection */

/*
 * LSTMP (the cell of the paper's speech model SR1, Table 1; the paper cites it and gives no
 * equations, so this is the cell as published by its authors): an LSTM whose output
 * m_t = o * tanh(c_t) (H wide) is projected to r_t = Wp m_t (P wide, no bias, no
 * non-linearity); r_t is what recurs and what the next layer reads.
 *   W[l]  dense (4H) x (in_l + P), rows i,f,g,o, in_0 = I, in_l = P; bias[l] of 4H or NULL
 *   Wp[l] dense P x H
 *   x [T][B][I] float32;  h0 [L][B][P], c0 [L][B][H] float64 or NULL (zeros)
 *   hseq [T][B][P] of the last layer or NULL;  hT [L][B][P];  cT [L][B][H] or NULL
 */
int orc_lstmp_forward(int32_t L, int64_t I, int64_t H, int64_t P,
                      const float *const *W, const float *const *Wp, const float *const *bias,
                      const float *x, const double *h0, const double *c0,
                      double *hseq, double *hT, double *cT, int64_t T, int64_t B) {
    if (L <= 0 || I <= 0 || H <= 0 || P <= 0 || T < 0 || B <= 0 || !W || !Wp || !hT) return -1;
    int64_t maxin = I > P ? I : P;
    double *r = (double *)calloc((size_t)(L * B * P), sizeof(double));
    double *c = (double *)calloc((size_t)(L * B * H), sizeof(double));
    double *u = (double *)malloc(sizeof(double) * (size_t)maxin);
    double *a = (double *)malloc(sizeof(double) * (size_t)(4 * H));
    double *m = (double *)malloc(sizeof(double) * (size_t)H);
    double *rn = (double *)malloc(sizeof(double) * (size_t)P);
    if (h0) memcpy(r, h0, sizeof(double) * (size_t)(L * B * P));
    if (c0) memcpy(c, c0, sizeof(double) * (size_t)(L * B * H));
    for (int64_t t = 0; t < T; ++t) {
        for (int64_t s = 0; s < B; ++s) {
            for (int32_t l = 0; l < L; ++l) {
                const int64_t n_in = l == 0 ? I : P, ld = n_in + P;
                if (l == 0) for (int64_t j = 0; j < I; ++j) u[j] = (double)x[(t * B + s) * I + j];
                else        for (int64_t j = 0; j < P; ++j) u[j] = r[((l - 1) * B + s) * P + j];
                double *rl = r + (l * B + s) * P, *cl = c + (l * B + s) * H;
                const float *Wl = W[l], *bl = bias ? bias[l] : NULL;
#pragma omp parallel for schedule(static)
                for (int64_t i = 0; i < 4 * H; ++i) {
                    double sum = bl ? (double)bl[i] : 0.0;
                    for (int64_t j = 0; j < n_in; ++j) sum += (double)Wl[i * ld + j] * u[j];
                    for (int64_t j = 0; j < P; ++j) sum += (double)Wl[i * ld + n_in + j] * rl[j];
                    a[i] = sum;
                }
                for (int64_t k = 0; k < H; ++k) {
                    double cn = sigmoid(a[H + k]) * cl[k] + sigmoid(a[k]) * tanh(a[2 * H + k]);
                    cl[k] = cn;
                    m[k] = sigmoid(a[3 * H + k]) * tanh(cn);
                }
                const float *Pl = Wp[l];
#pragma omp parallel for schedule(static)
                for (int64_t i = 0; i < P; ++i) {
                    double sum = 0.0;
                    for (int64_t k = 0; k < H; ++k) sum += (double)Pl[i * H + k] * m[k];
                    rn[i] = sum;
                }
                memcpy(rl, rn, sizeof(double) * (size_t)P);
            }
            if (hseq) for (int64_t k = 0; k < P; ++k) hseq[(t * B + s) * P + k] = r[((L - 1) * B + s) * P + k];
        }
    }
    memcpy(hT, r, sizeof(double) * (size_t)(L * B * P));
    if (cT) memcpy(cT, c, sizeof(double) * (size_t)(L * B * H));
    free(r); free(c); free(u); free(a); free(m); free(rn);
    return 0;
}


/* ------------------------------------------------------------------ CSB projection */

typedef struct { uint32_t key; int64_t idx; } orc_rank;

static int orc_rank_cmp(const void *a, const void *b) {
    const orc_rank *x = (const orc_rank *)a, *y = (const orc_rank *)b;
    if (x->key != y->key) return x->key < y->key ? -1 : 1;
    return x->idx < y->idx ? -1 : (x->idx > y->idx ? 1 : 0);
}

/* Ranking key of a float32 sum of squares: its bit pattern (sums are >= 0 or NaN, so the
 * unsigned order of the bits is the numeric order, with NaN on top). */
static uint32_t orc_key(float s) {
    uint32_t u;
    memcpy(&u, &s, 4);
    if (s != s) u = 0xffffffffu;          /* every NaN alike */
    return u & 0x7fffffffu ? u : 0u;      /* -0.0 cannot occur, but +0.0 == 0 */
}

static int64_t orc_prune_count(int64_t n, double rate) {
    const double q = 1.0 - 1.0 / sqrt(rate);
    int64_t k = (int64_t)floor((double)n * q + 0.5);
    if (k < 0) k = 0;
    if (k > n) k = n;
    return k;
}

/*
 * Z = projection of W (R x C, leading dimension ld) onto the CSB pattern with blocks
 * BR x BC at pruning rate `rate` (>= 1; "rate x").  Z has leading dimension ldz and may not
 * alias W.  Returns 0, or -1 on a bad argument.
 */
int orc_csb_project(const float *W, int64_t R, int64_t C, int64_t ld, int32_t BR, int32_t BC,
                    double rate, float *Z, int64_t ldz) {
    if (!W || !Z || R <= 0 || C <= 0 || ld < C || ldz < C || BR < 1 || BC < 1 || !(rate >= 1.0)) return -1;
    const int64_t nbr = (R + BR - 1) / BR, nbc = (C + BC - 1) / BC;
    for (int64_t i = 0; i < R; ++i) memcpy(Z + i * ldz, W + i * ld, sizeof(float) * (size_t)C);
    orc_rank *rk = (orc_rank *)malloc(sizeof(orc_rank) * (size_t)(R > C ? R : C));
    if (!rk) return -1;
    /* RowPrune, block-column by block-column */
    for (int64_t bj = 0; bj < nbc; ++bj) {
        const int64_t c0 = bj * BC, c1 = imin64(C, c0 + BC);
        for (int64_t i = 0; i < R; ++i) {
            float s = 0.0f;
            for (int64_t c = c0; c < c1; ++c) s = fmaf(Z[i * ldz + c], Z[i * ldz + c], s);
            rk[i].key = orc_key(s);
            rk[i].idx = i;
        }
        qsort(rk, (size_t)R, sizeof(orc_rank), orc_rank_cmp);
        const int64_t k = orc_prune_count(R, rate);
        for (int64_t t = 0; t < k; ++t)
            for (int64_t c = c0; c < c1; ++c) Z[rk[t].idx * ldz + c] = 0.0f;
    }
    /* ColumnPrune, block-row by block-row, on the row-pruned matrix */
    for (int64_t bi = 0; bi < nbr; ++bi) {
        const int64_t r0 = bi * BR, r1 = imin64(R, r0 + BR);
        for (int64_t c = 0; c < C; ++c) {
            float s = 0.0f;
            for (int64_t i = r0; i < r1; ++i) s = fmaf(Z[i * ldz + c], Z[i * ldz + c], s);
            rk[c].key = orc_key(s);
            rk[c].idx = c;
        }
        qsort(rk, (size_t)C, sizeof(orc_rank), orc_rank_cmp);
        const int64_t k = orc_prune_count(C, rate);
        for (int64_t t = 0; t < k; ++t)
            for (int64_t i = r0; i < r1; ++i) Z[i * ldz + rk[t].idx] = 0.0f;
    }
    free(rk);
    return 0;
}

/*
 * The same projection with the decision taken in float64: sums of squares accumulated in
 * double, in the same order, ranked by value and then by position (NaN on top).  This is the
 * plain definition of Sec. 3.2.2 without the reading "the decision is taken in float32"; it
 * exists to measure how often that reading matters (tests count the entries on which the two
 * differ) and to check the device result against wherever no two sums at a cut are nearly equal.
 */
typedef struct { double key; int nan; int64_t idx; } orc_rank64;

static int orc_rank64_cmp(const void *a, const void *b) {
    const orc_rank64 *x = (const orc_rank64 *)a, *y = (const orc_rank64 *)b;
    if (x->nan != y->nan) return x->nan < y->nan ? -1 : 1;
    if (!x->nan && x->key != y->key) return x->key < y->key ? -1 : 1;
    return x->idx < y->idx ? -1 : (x->idx > y->idx ? 1 : 0);
}

int orc_csb_project_f64(const float *W, int64_t R, int64_t C, int64_t ld, int32_t BR, int32_t BC,
                        double rate, float *Z, int64_t ldz) {
    if (!W || !Z || R <= 0 || C <= 0 || ld < C || ldz < C || BR < 1 || BC < 1 || !(rate >= 1.0)) return -1;
    const int64_t nbr = (R + BR - 1) / BR, nbc = (C + BC - 1) / BC;
    for (int64_t i = 0; i < R; ++i) memcpy(Z + i * ldz, W + i * ld, sizeof(float) * (size_t)C);
    orc_rank64 *rk = (orc_rank64 *)malloc(sizeof(orc_rank64) * (size_t)(R > C ? R : C));
    if (!rk) return -1;
    for (int64_t bj = 0; bj < nbc; ++bj) {
        const int64_t c0 = bj * BC, c1 = imin64(C, c0 + BC);
        for (int64_t i = 0; i < R; ++i) {
            double s = 0.0;
            for (int64_t c = c0; c < c1; ++c) s += (double)Z[i * ldz + c] * (double)Z[i * ldz + c];
            rk[i].nan = s != s; rk[i].key = s; rk[i].idx = i;
        }
        qsort(rk, (size_t)R, sizeof(orc_rank64), orc_rank64_cmp);
        const int64_t k = orc_prune_count(R, rate);
        for (int64_t t = 0; t < k; ++t)
            for (int64_t c = c0; c < c1; ++c) Z[rk[t].idx * ldz + c] = 0.0f;
    }
    for (int64_t bi = 0; bi < nbr; ++bi) {
        const int64_t r0 = bi * BR, r1 = imin64(R, r0 + BR);
        for (int64_t c = 0; c < C; ++c) {
            double s = 0.0;
            for (int64_t i = r0; i < r1; ++i) s += (double)Z[i * ldz + c] * (double)Z[i * ldz + c];
            rk[c].nan = s != s; rk[c].key = s; rk[c].idx = c;
        }
        qsort(rk, (size_t)C, sizeof(orc_rank64), orc_rank64_cmp);
        const int64_t k = orc_prune_count(C, rate);
        for (int64_t t = 0; t < k; ++t)
            for (int64_t i = r0; i < r1; ++i) Z[i * ldz + rk[t].idx] = 0.0f;
    }
    free(rk);
    return 0;
}
