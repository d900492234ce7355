// Host-side CSB packer (Sec. 3.1.1) and the handle's housekeeping.
#include <algorithm>
#include <cstring>
#include <mutex>
#include <new>
#include <unordered_map>

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

bool workspace_changed_hands(const void *ws, const void *user) {
    static std::mutex mu;
    static std::unordered_map<const void *, const void *> last_user;
    std::lock_guard<std::mutex> lock(mu);
    auto it = last_user.find(ws);
    if (it == last_user.end()) { last_user.emplace(ws, user); return true; }
    const bool changed = it->second != user;
    it->second = user;
    return changed;
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

namespace csb {

// binary32 -> binary16, round to nearest even; overflow to infinity, gradual underflow.
uint16_t f32_to_f16_bits(float f) {
    uint32_t x;
    std::memcpy(&x, &f, 4);
    const uint16_t sign = (uint16_t)((x >> 16) & 0x8000u);
    x &= 0x7fffffffu;
    if (x > 0x7f800000u) return (uint16_t)(sign | 0x7e00u | ((x >> 13) & 0x3ffu));      // NaN stays NaN (quiet)
    if (x >= 0x477ff000u) return (uint16_t)(sign | 0x7c00u);                            // >= 65520 (or inf): infinity
    if (x < 0x38800000u) {                                                              // below 2^-14: subnormal or zero
        const uint32_t e = x >> 23;
        if (e < 102u) return sign;                                                      // below 2^-25: zero (2^-25 itself ties to zero)
        const uint32_t mant = (x & 0x7fffffu) | 0x800000u, shift = 126u - e;            // value = mant 2^(e-150); unit 2^-24
        uint32_t q = mant >> shift;
        const uint32_t rem = mant & ((1u << shift) - 1u), half = 1u << (shift - 1u);
        if (rem > half || (rem == half && (q & 1u))) ++q;
        return (uint16_t)(sign | q);
    }
    uint32_t q = (x - 0x38000000u) >> 13;                                               // rebias 127 -> 15, keep 10 bits
    const uint32_t rem = x & 0x1fffu;
    if (rem > 0x1000u || (rem == 0x1000u && (q & 1u))) ++q;
    return (uint16_t)(sign | q);
}

float f16_bits_to_f32(uint16_t h) {
    const uint32_t sign = (uint32_t)(h & 0x8000u) << 16, e = (h >> 10) & 0x1fu, mant = h & 0x3ffu;
    uint32_t x;
    if (e == 0x1fu) x = sign | 0x7f800000u | (mant << 13);
    else if (e != 0) x = sign | ((e + 112u) << 23) | (mant << 13);
    else if (mant == 0) x = sign;
    else {                                                                              // subnormal: mant 2^-24
        float v = (float)mant * 5.9604644775390625e-8f;
        std::memcpy(&x, &v, 4);
        x |= sign;
    }
    float f;
    std::memcpy(&f, &x, 4);
    return f;
}

uint16_t f32_to_bf16_bits(float f) {
    uint32_t x;
    std::memcpy(&x, &f, 4);
    if ((x & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((x >> 16) | 0x40u);          // NaN stays NaN
    return (uint16_t)((x + 0x7fffu + ((x >> 16) & 1u)) >> 16);
}

}  // namespace csb

extern "C" int csb_set_value_format(csb_matrix *m, int32_t format) {
    using namespace csb;
    if (!m) { set_error("csb_set_value_format: NULL handle"); return CSB_EINVAL; }
    if (format != CSB_VAL_F32 && format != CSB_VAL_F16 && format != CSB_VAL_BF16) {
        set_error("csb_set_value_format: unknown format");
        return CSB_EINVAL;
    }
    if (format == CSB_VAL_F16)
        for (float &v : m->val) v = f16_bits_to_f32(f32_to_f16_bits(v));
    else if (format == CSB_VAL_BF16)
        for (float &v : m->val) v = bf16_bits_to_f32(f32_to_bf16_bits(v));
    m->val_fmt = format;
    m->plan.valid = false;
    m->uploaded = false;
    return CSB_OK;
}

extern "C" int csb_value_format(const csb_matrix *m) { return m ? m->val_fmt : -1; }

extern "C" void csb_free(csb_matrix *m) { delete m; }
