// Batched CSB-MVM for gfx950: Y = A X with fp32 MFMA.
//
// With B right-hand sides a kernel matrix K_b (r x c) meets a gathered c x B slab of X: a
// real dense product, so it goes to the matrix cores (v_mfma_f32_16x16x4_f32).  One
// workgroup owns one output row tile and one batch tile; its wavefronts take the tile's
// virtual blocks round-robin, each as 16-row slices: per 4 columns one A operand (16 x 4
// of the kernel) feeds one MFMA per 16 batch columns.  The 16 x 16 results are added at
// the block's row indices into a per-wavefront accumulator tile in LDS (the role of
// NeuronAccumBuffer, Sec. 4.3.1); the wavefronts' tiles are summed in wavefront order, so
// the result does not depend on timing.  The paper's engine is batch 1 only; this is the
// batched extension the matrix cores make worthwhile.
#include <hip/hip_runtime.h>

#include "csb_internal.hpp"
#include "csb_kernels.hpp"

namespace csb {

typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int kSpmmWaves = 8;
constexpr int kSpmmThreads = kSpmmWaves * 64;

__device__ __forceinline__ uint32_t uni_(uint32_t v) { return __builtin_amdgcn_readfirstlane(v); }

// Element (column j of A, right-hand side n) of the input, from one of two sources.
struct XSrc {
    const float *p0;
    uint32_t n0;          // columns j < n0 come from p0, the rest from p1
    int64_t sj0, sn0;     // strides over j and over n
    const float *p1;
    int64_t sj1, sn1;
};

template <int NT>
__global__ __launch_bounds__(kSpmmThreads) void spmm_kernel(const DevMat m, const XSrc X, float *__restrict__ Y,
                                                             const int64_t ldy, const uint32_t batch) {
    extern __shared__ float smem_f[];
    constexpr int NB = 16 * NT;                    // batch columns per workgroup
    const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = uni_(tid >> 6);
    const uint32_t bt0 = blockIdx.y * NB;
    const uint32_t br = m.br;
    if (blockIdx.x >= m.n_nz_tiles) {              // a row tile without work: zeros
        const uint32_t tile = m.zero_tiles[blockIdx.x - m.n_nz_tiles];
        for (uint32_t e = tid; e < br * NB; e += kSpmmThreads) {
            const uint32_t row = tile * br + e / NB, n = bt0 + e % NB;
            if (row < m.rows_out && n < batch) Y[(size_t)row * ldy + n] = 0.0f;
        }
        return;
    }
    float *acc = smem_f;                                           // [waves][br][NB]
    float *myacc = acc + (size_t)wave * br * NB;
    for (uint32_t e = lane; e < br * NB; e += 64) myacc[e] = 0.0f;
    const uint32_t rank = blockIdx.x, tile = m.nz_tiles[rank];
    const uint32_t g0 = m.tile_g0[rank], g1 = m.tile_g0[rank + 1];
    const uint32_t mrow = lane & 15u, kq = lane >> 4;              // A: row, column-in-4; B: column n, row-in-4
    uint32_t task = 0;
    for (uint32_t g = g0; g < g1; ++g) {
        const GroupRec *gp = m.groups + g;
        const uint32_t nvb = uni_(gp->nvb), nlanes = uni_(gp->nlanes);
        const uint32_t idx_off = uni_(gp->idx_off), vb_off = uni_(gp->vb_off);
        const float *gv = m.vals + uni_(gp->val_off);
        // does this wavefront have a slice in the group?
        uint32_t ntask = 0;
        for (uint32_t k = 0; k < nvb; ++k) ntask += ((uint32_t)m.vbs[vb_off + k].r + 15u) >> 4;
        const uint32_t first_mine = (wave + kSpmmWaves - task % kSpmmWaves) % kSpmmWaves;
        if (first_mine >= ntask) { task += ntask; continue; }
        const uint8_t *colbase = m.idx + idx_off + ((4 * nlanes + 7) & ~7u);
        for (uint32_t k = 0; k < nvb; ++k) {
            const VbRec v = m.vbs[vb_off + k];
            const uint32_t r = uni_(v.r), c = uni_(v.c), lane0 = uni_(v.lane0);
            const uint16_t *colp = (const uint16_t *)(colbase + 4u * uni_(v.coloff4));   // byte offsets of the inputs
            for (uint32_t m0 = 0; m0 < r; m0 += 16, ++task) {
                if (task % kSpmmWaves != wave) continue;
                floatx4 D[NT];
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) D[nt] = floatx4{0.0f, 0.0f, 0.0f, 0.0f};
                const bool row_ok = m0 + mrow < r;
                const uint32_t arow = lane0 + m0 + (row_ok ? mrow : 0u);
                // 32 columns (8 MFMA k-steps) per pass: all kernel values and column indices
                // first, then all gathered inputs, then the MFMAs -- the loads of a pass
                // are independent, so their latencies overlap.  Out-of-range lanes load
                // from clamped addresses and their operands are zeroed.
                for (uint32_t kc = 0; kc < c; kc += 32) {
                    float av[8];
                    uint32_t gc[8];
                    bool ok[8];
#pragma unroll
                    for (int s8 = 0; s8 < 8; ++s8) {
                        const uint32_t jj = kc + 4u * s8 + kq;
                        ok[s8] = jj < c;
                        const uint32_t jc = ok[s8] ? jj : 0u;
                        const float t = gv[jc * (uint32_t)kWave + arow];
                        av[s8] = ok[s8] && row_ok ? t : 0.0f;
                        gc[s8] = (uint32_t)colp[jc] >> 2;
                    }
                    float bv[8][NT];
#pragma unroll
                    for (int s8 = 0; s8 < 8; ++s8)
#pragma unroll
                        for (int nt = 0; nt < NT; ++nt) {
                            const uint32_t n = bt0 + 16u * nt + mrow;
                            const uint32_t nc = n < batch ? n : 0u;
                            const float t = gc[s8] < X.n0 ? X.p0[(int64_t)gc[s8] * X.sj0 + (int64_t)nc * X.sn0]
                                                          : X.p1[(int64_t)(gc[s8] - X.n0) * X.sj1 + (int64_t)nc * X.sn1];
                            bv[s8][nt] = ok[s8] && n < batch ? t : 0.0f;
                        }
#pragma unroll
                    for (int s8 = 0; s8 < 8; ++s8) {
                        if (kc + 4u * s8 >= c) break;          // uniform
#pragma unroll
                        for (int nt = 0; nt < NT; ++nt)
                            D[nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[s8], bv[s8][nt], D[nt], 0, 0, 0);
                    }
                }
                // lane holds rows 4*(lane/16)+i, column lane%16 of each 16 x 16 result
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const uint32_t mr = m0 + 4u * kq + i;
                    if (mr < r) {
                        const uint32_t slot = m.idx[idx_off + 4u * (lane0 + mr)];
#pragma unroll
                        for (int nt = 0; nt < NT; ++nt)
                            myacc[slot * NB + 16u * nt + mrow] += D[nt][i];   // rows of a slice are distinct: no two lanes meet
                    }
                }
            }
        }
    }
    __syncthreads();
    for (uint32_t e = tid; e < br * NB; e += kSpmmThreads) {
        float s = 0.0f;
#pragma unroll
        for (int w = 0; w < kSpmmWaves; ++w) s += acc[(size_t)w * br * NB + e];
        const uint32_t row = tile * br + e / NB, n = bt0 + e % NB;
        if (row < m.rows_out && n < batch) Y[(size_t)row * ldy + n] = s;
    }
}

int spmm_strided(const csb_matrix *mat, const float *p0, uint32_t n0, int64_t sj0, int64_t sn0, const float *p1,
                 int64_t sj1, int64_t sn1, float *d_Y, int64_t ldy, int32_t batch, void *stream) {
    if (!mat->plan.valid || !mat->uploaded || !mat->d_buf) { set_error("csb_spmm: matrix not planned and uploaded"); return CSB_ESTATE; }
    const DevHeader &h = mat->plan.hdr;
    const DevMat dm = dev_mat(mat);
    XSrc X{p0, n0, sj0, sn0, p1, sj1, sn1};
    const int nt = h.br <= 128 ? 2 : 1;
    const size_t lds = (size_t)kSpmmWaves * h.br * 16 * nt * sizeof(float);
    const dim3 grid(h.n_nz_tiles + h.n_zero_tiles, (unsigned)((batch + 16 * nt - 1) / (16 * nt)));
    hipError_t e;
    if (nt == 2) {
        e = hipFuncSetAttribute((const void *)spmm_kernel<2>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e == hipSuccess) hipLaunchKernelGGL(spmm_kernel<2>, grid, dim3(kSpmmThreads), lds, (hipStream_t)stream, dm, X, d_Y, ldy, (uint32_t)batch);
    } else {
        e = hipFuncSetAttribute((const void *)spmm_kernel<1>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e == hipSuccess) hipLaunchKernelGGL(spmm_kernel<1>, grid, dim3(kSpmmThreads), lds, (hipStream_t)stream, dm, X, d_Y, ldy, (uint32_t)batch);
    }
    if (e == hipSuccess) e = hipGetLastError();
    if (e != hipSuccess) { set_error(std::string("csb_spmm: ") + hipGetErrorString(e)); return CSB_EDEVICE; }
    return CSB_OK;
}

}  // namespace csb

extern "C" int csb_spmm(const csb_matrix *m, const float *d_X, int64_t ldx, float *d_Y, int64_t ldy,
                        int32_t batch, void *d_ws, void *stream) {
    (void)d_ws;
    if (!m || !d_X || !d_Y) { csb::set_error("csb_spmm: NULL pointer"); return CSB_EINVAL; }
    if (batch <= 0 || ldx < batch || ldy < batch) { csb::set_error("csb_spmm: batch <= 0 or a leading dimension below batch"); return CSB_EINVAL; }
    if (m->plan.valid && m->plan.split.active()) { csb::set_error("csb_spmm: matrix is planned for a GRU step"); return CSB_ESTATE; }
    return csb::spmm_strided(m, d_X, (uint32_t)m->cols, ldx, 1, d_X, ldx, 1, d_Y, ldy, batch, stream);
}
