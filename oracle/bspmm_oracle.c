/*
 * CPU oracle for Batched SpMM.  TEST INFRASTRUCTURE ONLY: nothing on the product path may
 * call, link or import this file; it shares no code with the HIP library.
 *
 * What it computes is the plain definition that all three pseudo-codes of the paper reach
 * (Fig. 2, Fig. 3 and Fig. 4: "set C to O", then for every stored entry (r, c, v) of A and
 * every column j:  C[r][j] += v * B[c][j]), once per operation of the batch (Sec. IV-C):
 *
 *   forward     C_i[r][j] = sum_{p = rpt_i[r]}^{rpt_i[r+1]-1} values_i[p] * B_i[colids_i[p]][j]
 *   transposed  G_i[c][j] = sum_{r} sum_{p in row r, colids_i[p] == c} values_i[p] * dY_i[r][j]
 *
 * Several operations may name the SAME output block (the graph-convolution layer adds up the
 * products of a graph's channels, Fig. 6 / Fig. 7 "ElementWiseAdd"): the block then holds the sum
 * of their products.  Blocks are zeroed first, then every operation adds into its block.
 *
 * The loops are the four nested loops of that definition (operation, row, stored entry,
 * column), in that order, with no blocking, fusion or reordering.  fp32 inputs are promoted
 * to fp64 and accumulated in fp64; the result stays fp64.  Beside the result the oracle
 * returns S[r][j] = sum |v| * |B[c][j]|, the scale of the per-element tolerance.
 * The transposed product is a scatter over the ORIGINAL row-major entries (it never builds
 * a transposed matrix), so it has no structure in common with a gather over a transposed CSR.
 *
 * Layout (the paper's problem statement: CSR arrays rpt/colids/values of Sec. II-B and
 * Fig. 4, 0-based; dense operands row-major, packed for the whole batch as in Sec. IV-D):
 *   rpt      per-operation LOCAL row pointers (first 0, last nnz_i), op i at rpt + rpt_off[i]
 *   colids   column indices, op i at colids + nz_off[i]
 *   values   fp32 values,    op i at values + nz_off[i]
 *   dense input  row-major fp32, leading dimension ld_in ; output/scale row-major fp64, ld_out
 * Output rows that belong to no operation are left untouched.
 *
 * Pins (tests/test_oracle_pins.py): dense brute force, a library CSR product, A = I,
 * empty rows, linearity, node relabelling, the eigenvector of the symmetric normalisation,
 * row sums of the row normalisation, the adjoint identity <AB, dY> = <B, A^T dY>; for the COO
 * functions a dense matrix assembled entry by entry, a library COO product, invariance under
 * shuffling the entries, repeated pairs, and a library stable sort for the conversion.
 *
 * Returns 0, or a negative number naming the first malformed operation (-(i+1)).
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>

static int check_op(int32_t rows, int32_t cols, int32_t nnz, const int32_t* rp,
                    const int32_t* ci)
{
    if (rows < 0 || cols < 0 || nnz < 0) return 0;
    if (rows == 0) return nnz == 0;
    if (rp[0] != 0 || rp[rows] != nnz) return 0;
    for (int32_t r = 0; r < rows; ++r)
        if (rp[r + 1] < rp[r]) return 0;
    for (int32_t p = 0; p < nnz; ++p)
        if (ci[p] < 0 || ci[p] >= cols) return 0;
    return 1;
}

/* 1 when two operations name overlapping row ranges (then they are summed, one at a time). */
static int shares_a_block(int32_t batch, const int64_t* off, const int32_t* len)
{
    for (int32_t i = 0; i < batch; ++i)
        for (int32_t k = 0; k < i; ++k)
            if (len[i] > 0 && len[k] > 0 && off[i] < off[k] + len[k] && off[k] < off[i] + len[i])
                return 1;
    return 0;
}

/* Forward product of every operation; C and S are fully overwritten on the operations' rows
 * (operations that name the same block are added up). */
int oracle_bspmm_forward(int32_t batch, const int32_t* rows, const int32_t* cols,
                         const int32_t* nnz, const int64_t* rpt_off, const int64_t* nz_off,
                         const int64_t* b_row_off, const int64_t* c_row_off,
                         const int32_t* rpt, const int32_t* colids, const float* values,
                         const float* B, int64_t ldb, int32_t F,
                         double* C, double* S, int64_t ldc)
{
    for (int32_t i = 0; i < batch; ++i)
        if (!check_op(rows[i], cols[i], nnz[i], rpt + rpt_off[i], colids + nz_off[i]))
            return -(i + 1);
    for (int32_t i = 0; i < batch; ++i)
        for (int32_t r = 0; r < rows[i]; ++r)
            for (int32_t j = 0; j < F; ++j) {
                C[(c_row_off[i] + r) * ldc + j] = 0.0;
                if (S) S[(c_row_off[i] + r) * ldc + j] = 0.0;
            }
    const int shared = shares_a_block(batch, c_row_off, rows);
#pragma omp parallel for schedule(dynamic, 1) if (!shared)
    for (int32_t i = 0; i < batch; ++i) {
        const int32_t* rp = rpt + rpt_off[i];
        const int32_t* ci = colids + nz_off[i];
        const float* va = values + nz_off[i];
        for (int32_t r = 0; r < rows[i]; ++r) {
            double* c = C + (c_row_off[i] + r) * ldc;
            double* s = S ? S + (c_row_off[i] + r) * ldc : NULL;
            for (int32_t p = rp[r]; p < rp[r + 1]; ++p) {
                const double v = (double)va[p];
                const float* b = B + (b_row_off[i] + ci[p]) * ldb;
                for (int32_t j = 0; j < F; ++j) {
                    c[j] += v * (double)b[j];
                    if (s) s[j] += fabs(v) * fabs((double)b[j]);
                }
            }
        }
    }
    return 0;
}

/*
 * The same forward product with an fp64 dense input (no scale output): the last step of the
 * batched graph-convolution layer (Fig. 7: U = MatMul(Xr, W[ch]); B = Add(bias[ch], U);
 * C[ch] = BatchedSpMM(A_list, B)), whose B the oracle keeps in fp64 instead of rounding it to
 * fp32 between the steps.  `accumulate` != 0 adds to C instead of overwriting it (the
 * ElementWiseAdd over channels taken one channel at a time).
 */
int oracle_bspmm_forward_f64(int32_t batch, const int32_t* rows, const int32_t* cols,
                             const int32_t* nnz, const int64_t* rpt_off, const int64_t* nz_off,
                             const int64_t* b_row_off, const int64_t* c_row_off,
                             const int32_t* rpt, const int32_t* colids, const float* values,
                             const double* B, int64_t ldb, int32_t F, int32_t accumulate,
                             double* C, int64_t ldc)
{
    for (int32_t i = 0; i < batch; ++i)
        if (!check_op(rows[i], cols[i], nnz[i], rpt + rpt_off[i], colids + nz_off[i]))
            return -(i + 1);
    if (!accumulate)
        for (int32_t i = 0; i < batch; ++i)
            for (int32_t r = 0; r < rows[i]; ++r)
                for (int32_t j = 0; j < F; ++j) C[(c_row_off[i] + r) * ldc + j] = 0.0;
    for (int32_t i = 0; i < batch; ++i) {
        const int32_t* rp = rpt + rpt_off[i];
        const int32_t* ci = colids + nz_off[i];
        const float* va = values + nz_off[i];
        for (int32_t r = 0; r < rows[i]; ++r) {
            double* c = C + (c_row_off[i] + r) * ldc;
            for (int32_t p = rp[r]; p < rp[r + 1]; ++p) {
                const double v = (double)va[p];
                const double* b = B + (b_row_off[i] + ci[p]) * ldb;
                for (int32_t j = 0; j < F; ++j) c[j] += v * b[j];
            }
        }
    }
    return 0;
}

/*
 * Transposed product G_i = A_i^T dY_i.  dY_i has rows[i] rows at dY + c_row_off[i]*ldy,
 * G_i has cols[i] rows at G + b_row_off[i]*ldg.  Operations that name the same output block
 * (channels reading one dense input in the forward direction) are added up.
 */
int oracle_bspmm_transposed(int32_t batch, const int32_t* rows, const int32_t* cols,
                            const int32_t* nnz, const int64_t* rpt_off, const int64_t* nz_off,
                            const int64_t* b_row_off, const int64_t* c_row_off,
                            const int32_t* rpt, const int32_t* colids, const float* values,
                            const float* dY, int64_t ldy, int32_t F,
                            double* G, double* S, int64_t ldg)
{
    for (int32_t i = 0; i < batch; ++i)
        if (!check_op(rows[i], cols[i], nnz[i], rpt + rpt_off[i], colids + nz_off[i]))
            return -(i + 1);
    for (int32_t i = 0; i < batch; ++i)
        for (int32_t c = 0; c < cols[i]; ++c)
            for (int32_t j = 0; j < F; ++j) {
                G[(b_row_off[i] + c) * ldg + j] = 0.0;
                if (S) S[(b_row_off[i] + c) * ldg + j] = 0.0;
            }
    const int shared = shares_a_block(batch, b_row_off, cols);
#pragma omp parallel for schedule(dynamic, 1) if (!shared)
    for (int32_t i = 0; i < batch; ++i) {
        const int32_t* rp = rpt + rpt_off[i];
        const int32_t* ci = colids + nz_off[i];
        const float* va = values + nz_off[i];
        for (int32_t r = 0; r < rows[i]; ++r) {
            const float* y = dY + (c_row_off[i] + r) * ldy;
            for (int32_t p = rp[r]; p < rp[r + 1]; ++p) {
                const double v = (double)va[p];
                double* g = G + (b_row_off[i] + ci[p]) * ldg;
                double* s = S ? S + (b_row_off[i] + ci[p]) * ldg : NULL;
                for (int32_t j = 0; j < F; ++j) {
                    g[j] += v * (double)y[j];
                    if (s) s[j] += fabs(v) * fabs((double)y[j]);
                }
            }
        }
    }
    return 0;
}

/*
 * Transposed CSR of every operation, by the textbook counting sort over columns: count the
 * entries of each column, prefix-sum the counts into row pointers of A^T, then walk the
 * entries in stored order (row by row) and append each to its column's list.  Because the
 * walk is in stored order the result is the unique STABLE transpose: inside row c of A^T the
 * entries are ordered by original row, ties (duplicate (r,c) entries) by stored position.
 * Op i of the result has cols[i] rows: rpt_t at rpt_t_off[i] (cols[i]+1 entries, local),
 * entries at nz_off[i] (same packing of the non-zeros as the input).
 */
int oracle_csr_transpose(int32_t batch, const int32_t* rows, const int32_t* cols,
                         const int32_t* nnz, const int64_t* rpt_off, const int64_t* nz_off,
                         const int32_t* rpt, const int32_t* colids, const float* values,
                         const int64_t* rpt_t_off, int32_t* rpt_t, int32_t* colids_t,
                         float* values_t, int32_t* cursor_scratch /* >= max cols */)
{
    for (int32_t i = 0; i < batch; ++i)
        if (!check_op(rows[i], cols[i], nnz[i], rpt + rpt_off[i], colids + nz_off[i]))
            return -(i + 1);
    for (int32_t i = 0; i < batch; ++i) {
        const int32_t* rp = rpt + rpt_off[i];
        const int32_t* ci = colids + nz_off[i];
        const float* va = values + nz_off[i];
        int32_t* rt = rpt_t + rpt_t_off[i];
        int32_t* ct = colids_t + nz_off[i];
        float* vt = values_t + nz_off[i];
        for (int32_t c = 0; c <= cols[i]; ++c) rt[c] = 0;
        for (int32_t p = 0; p < nnz[i]; ++p) rt[ci[p] + 1] += 1;
        for (int32_t c = 0; c < cols[i]; ++c) rt[c + 1] += rt[c];
        for (int32_t c = 0; c < cols[i]; ++c) cursor_scratch[c] = rt[c];
        for (int32_t r = 0; r < rows[i]; ++r)
            for (int32_t p = rp[r]; p < rp[r + 1]; ++p) {
                const int32_t q = cursor_scratch[ci[p]]++;
                ct[q] = r;
                vt[q] = va[p];
            }
    }
    return 0;
}

/*
 * COO / SparseTensor operands (Sec. II-B, Fig. 1: an entry is a (row, column) index pair and a
 * value; Sec. IV: the entries are NOT sorted by row or column).  Op i holds nnz[i] entries:
 * pair p at ids[2*(nz_off[i]+p)] = row, ids[2*(nz_off[i]+p)+1] = column, value at
 * values[nz_off[i]+p].  The product is the loop nest of Fig. 2: set C to O, then for every
 * stored entry in stored order and every column j, C[rid][j] += val * B[cid][j]; with
 * `transposed` != 0 the roles of the two indices are swapped (G[cid][j] += val * dY[rid][j],
 * dY at c_row_off with rows[i] rows, G at b_row_off with cols[i] rows).  Repeated (row, column)
 * pairs are added up, as the loop nest does.  Operations naming one output block are summed.
 */
static int check_coo(int32_t rows, int32_t cols, int32_t nnz, const int32_t* id)
{
    if (rows < 0 || cols < 0 || nnz < 0) return 0;
    for (int32_t p = 0; p < nnz; ++p)
        if (id[2 * p] < 0 || id[2 * p] >= rows || id[2 * p + 1] < 0 || id[2 * p + 1] >= cols)
            return 0;
    return 1;
}

int oracle_coo_product(int32_t batch, int32_t transposed, const int32_t* rows,
                       const int32_t* cols, const int32_t* nnz, const int64_t* nz_off,
                       const int64_t* b_row_off, const int64_t* c_row_off, const int32_t* ids,
                       const float* values, const float* X, int64_t ldx, int32_t F,
                       double* Y, double* S, int64_t ldy)
{
    for (int32_t i = 0; i < batch; ++i)
        if (!check_coo(rows[i], cols[i], nnz[i], ids + 2 * nz_off[i])) return -(i + 1);
    const int64_t* in_off = transposed ? c_row_off : b_row_off;
    const int64_t* out_off = transposed ? b_row_off : c_row_off;
    const int32_t* out_rows = transposed ? cols : rows;
    for (int32_t i = 0; i < batch; ++i)
        for (int32_t r = 0; r < out_rows[i]; ++r)
            for (int32_t j = 0; j < F; ++j) {
                Y[(out_off[i] + r) * ldy + j] = 0.0;
                if (S) S[(out_off[i] + r) * ldy + j] = 0.0;
            }
    for (int32_t i = 0; i < batch; ++i) {
        const int32_t* id = ids + 2 * nz_off[i];
        const float* va = values + nz_off[i];
        for (int32_t p = 0; p < nnz[i]; ++p) {
            const int32_t rid = transposed ? id[2 * p + 1] : id[2 * p];
            const int32_t cid = transposed ? id[2 * p] : id[2 * p + 1];
            const double val = (double)va[p];
            const float* x = X + (in_off[i] + cid) * ldx;
            double* y = Y + (out_off[i] + rid) * ldy;
            double* s = S ? S + (out_off[i] + rid) * ldy : NULL;
            for (int32_t j = 0; j < F; ++j) {
                y[j] += val * (double)x[j];
                if (s) s[j] += fabs(val) * fabs((double)x[j]);
            }
        }
    }
    return 0;
}

/*
 * CSR of every COO operation by the textbook stable counting sort over rows: count the
 * entries of each row, prefix-sum into row pointers, then walk the entries in stored order and
 * append each to its row's list.  Inside a row the entries keep their stored order (repeated
 * pairs stay separate entries).  Op i of the result has rows[i]+1 local row pointers at
 * rpt_off[i]; its entries sit at nz_off[i] like the input's.
 */
int oracle_coo_to_csr(int32_t batch, const int32_t* rows, const int32_t* cols,
                      const int32_t* nnz, const int64_t* nz_off, const int32_t* ids,
                      const float* values, const int64_t* rpt_off, int32_t* rpt,
                      int32_t* colids, float* csr_values, int32_t* cursor_scratch /* >= max rows */)
{
    for (int32_t i = 0; i < batch; ++i)
        if (!check_coo(rows[i], cols[i], nnz[i], ids + 2 * nz_off[i])) return -(i + 1);
    for (int32_t i = 0; i < batch; ++i) {
        const int32_t* id = ids + 2 * nz_off[i];
        const float* va = values + nz_off[i];
        int32_t* rp = rpt + rpt_off[i];
        for (int32_t r = 0; r <= rows[i]; ++r) rp[r] = 0;
        for (int32_t p = 0; p < nnz[i]; ++p) rp[id[2 * p] + 1] += 1;
        for (int32_t r = 0; r < rows[i]; ++r) rp[r + 1] += rp[r];
        for (int32_t r = 0; r < rows[i]; ++r) cursor_scratch[r] = rp[r];
        for (int32_t p = 0; p < nnz[i]; ++p) {
            const int32_t q = cursor_scratch[id[2 * p]]++;
            colids[nz_off[i] + q] = id[2 * p + 1];
            csr_values[nz_off[i] + q] = va[p];
        }
    }
    return 0;
}

/* Threads the forward/transposed loops will use (for reporting beside timings). */
#ifdef _OPENMP
#include <omp.h>
int oracle_num_threads(void) { return omp_get_max_threads(); }
void oracle_set_num_threads(int n) { if (n > 0) omp_set_num_threads(n); }
#else
int oracle_num_threads(void) { return 1; }
void oracle_set_num_threads(int n) { (void)n; }
#endif
