// Host-side CSB packer (Sec. 3.1.1) and the handle's housekeeping.
#include <algorithm>
#include <cstring>
#include <mutex>
#include <new>

#include "csb_internal.hpp"

namespace csb {
static thread_local std::string g_err;
void set_error(const std::string &msg) { g_err = msg; }
}  // namespace csb

namespace csb {
// Tags of the 64-bit (tag, value) words that kernels exchange through global memory: unique
// across the process, never 0, `count` consecutive ones inside one 2^32 generation.
uint32_t reserve_tags(uint32_t count, uint32_t *generation) {
    static std::mutex mu;
    static uint64_t next = 1;
    std::lock_guard<std::mutex> lock(mu);
    uint64_t n0 = next;
    if ((uint32_t)n0 == 0) ++n0;
    if (((n0 + count) >> 32) != (n0 >> 32)) n0 = (((n0 >> 32) + 1) << 32) | 1u;
    next = n0 + count;
    *generation = (uint32_t)(n0 >> 32);
    return (uint32_t)n0;
}
}  // namespace csb

extern "C" const char *csb_last_error(void) { return csb::g_err.c_str(); }

// Sec. 3.1.1: blocks in row-major order; per block the surviving rows/columns (those
// holding at least one non-zero of the block), then the kernel at their cross-points.
extern "C" int csb_pack(const float *dense, int64_t rows, int64_t cols, int64_t ld,
                        int32_t br, int32_t bc, csb_matrix **out) {
    if (!dense || !out) { csb::set_error("csb_pack: NULL pointer"); return CSB_EINVAL; }
    *out = nullptr;
    if (rows <= 0 || cols <= 0) { csb::set_error("csb_pack: rows and cols must be positive"); return CSB_EINVAL; }
    if (br < 1 || br > CSB_MAX_BLOCK || bc < 1 || bc > CSB_MAX_BLOCK) {
        csb::set_error("csb_pack: block size outside [1, 256]");
        return CSB_EINVAL;
    }
    if (ld < cols) { csb::set_error("csb_pack: ld < cols"); return CSB_EINVAL; }
    try {
        auto *m = new csb_matrix();
        m->rows = rows; m->cols = cols; m->br = br; m->bc = bc;
        m->nbr = (int32_t)((rows + br - 1) / br);
        m->nbc = (int32_t)((cols + bc - 1) / bc);
        const size_t nb = (size_t)m->nbr * (size_t)m->nbc;
        m->nrows.assign(nb, 0);
        m->ncols.assign(nb, 0);
        m->val_off.assign(nb + 1, 0);
        m->row_off.assign(nb + 1, 0);
        m->col_off.assign(nb + 1, 0);
        uint64_t colmask[4];              // bc <= 256 columns of the block
        uint16_t rows_kept[CSB_MAX_BLOCK], cols_kept[CSB_MAX_BLOCK];
        for (int32_t bi = 0; bi < m->nbr; ++bi) {
            const int64_t r0 = (int64_t)bi * br;
            const int h = (int)std::min<int64_t>(br, rows - r0);
            for (int32_t bj = 0; bj < m->nbc; ++bj) {
                const int64_t c0 = (int64_t)bj * bc;
                const int w = (int)std::min<int64_t>(bc, cols - c0);
                colmask[0] = colmask[1] = colmask[2] = colmask[3] = 0;
                int nr = 0;
                for (int i = 0; i < h; ++i) {
                    const float *p = dense + (r0 + i) * ld + c0;
                    bool any = false;
                    for (int j = 0; j < w; ++j)
                        if (p[j] != 0.0f) { any = true; colmask[j >> 6] |= 1ull << (j & 63); }
                    if (any) rows_kept[nr++] = (uint16_t)i;
                }
                int nc = 0;
                for (int j = 0; j < w; ++j)
                    if (colmask[j >> 6] >> (j & 63) & 1) cols_kept[nc++] = (uint16_t)j;
                const size_t b = (size_t)bi * m->nbc + bj;
                m->nrows[b] = nr;
                m->ncols[b] = nc;
                m->rowidx.insert(m->rowidx.end(), rows_kept, rows_kept + nr);
                m->colidx.insert(m->colidx.end(), cols_kept, cols_kept + nc);
                for (int a = 0; a < nr; ++a) {
                    const float *p = dense + (r0 + rows_kept[a]) * ld + c0;
                    for (int q = 0; q < nc; ++q) m->val.push_back(p[cols_kept[q]]);
                }
                m->val_off[b + 1] = (int64_t)m->val.size();
                m->row_off[b + 1] = (int64_t)m->rowidx.size();
                m->col_off[b + 1] = (int64_t)m->colidx.size();
            }
        }
        *out = m;
        return CSB_OK;
    } catch (const std::bad_alloc &) {
        csb::set_error("csb_pack: out of host memory");
        return CSB_ENOMEM;
    }
}

extern "C" int csb_view_get(const csb_matrix *m, csb_view *out) {
    if (!m || !out) { csb::set_error("csb_view_get: NULL pointer"); return CSB_EINVAL; }
    out->rows = m->rows; out->cols = m->cols;
    out->br = m->br; out->bc = m->bc; out->nbr = m->nbr; out->nbc = m->nbc;
    out->nnz = (int64_t)m->val.size();
    out->n_rowidx = (int64_t)m->rowidx.size();
    out->n_colidx = (int64_t)m->colidx.size();
    out->nrows = m->nrows.data(); out->ncols = m->ncols.data();
    out->rowidx = m->rowidx.data(); out->colidx = m->colidx.data();
    out->val = m->val.data();
    out->val_off = m->val_off.data(); out->row_off = m->row_off.data(); out->col_off = m->col_off.data();
    return CSB_OK;
}

extern "C" int csb_unpack(const csb_matrix *m, float *dense, int64_t ld) {
    if (!m || !dense) { csb::set_error("csb_unpack: NULL pointer"); return CSB_EINVAL; }
    if (ld < m->cols) { csb::set_error("csb_unpack: ld < cols"); return CSB_EINVAL; }
    for (int64_t i = 0; i < m->rows; ++i) std::memset(dense + i * ld, 0, sizeof(float) * (size_t)m->cols);
    for (int32_t bi = 0; bi < m->nbr; ++bi)
        for (int32_t bj = 0; bj < m->nbc; ++bj) {
            const size_t b = (size_t)bi * m->nbc + bj;
            const int nr = m->nrows[b], nc = m->ncols[b];
            const uint16_t *ri = m->rowidx.data() + m->row_off[b];
            const uint16_t *ci = m->colidx.data() + m->col_off[b];
            const float *v = m->val.data() + m->val_off[b];
            for (int a = 0; a < nr; ++a) {
                float *row = dense + ((int64_t)bi * m->br + ri[a]) * ld + (int64_t)bj * m->bc;
                for (int q = 0; q < nc; ++q) row[ci[q]] = v[(size_t)a * nc + q];
            }
        }
    return CSB_OK;
}

extern "C" void csb_free(csb_matrix *m) { delete m; }
