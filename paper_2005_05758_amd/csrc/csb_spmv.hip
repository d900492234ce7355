// CSB-MVM (Sec. 4.3.1) for gfx950: y = A x from the planned device image.
//
// One workgroup per chunk, one contiguous range of group steps per wavefront.  Inside a
// group, lane l owns one kernel-matrix row of one virtual block (inner-block parallelism
// over rows, inter-block parallelism over the lanes' different blocks, as the two
// hierarchy levels of Sec. 4.3.1) and walks that block's columns; a step reads the active
// lanes' values as one contiguous run of the value stream.  Row results go to a
// per-wavefront accumulator in LDS (the role of NeuronAccumBuffer) and are summed over
// wavefronts in a fixed order; row tiles shared by several workgroups are merged by the
// last workgroup to arrive, again in a fixed order, so results are bitwise reproducible.
#include <hip/hip_runtime.h>

#include "csb_internal.hpp"
#include "csb_kernels.hpp"

namespace csb {

DevMat dev_mat(const csb_matrix *m) {
    const DevHeader &h = m->plan.hdr;
    uint8_t *b = (uint8_t *)m->d_buf;
    DevMat d{};
    d.chunks = (const ChunkRec *)(b + h.off_chunks);
    d.waves = (const WaveRec *)(b + h.off_waves);
    d.groups = (const GroupRec *)(b + h.off_groups);
    d.vbs = (const VbRec *)(b + h.off_vbs);
    d.idx = b + h.off_idx;
    d.vals = (const float *)(b + h.off_vals);
    d.nz_tiles = (const uint32_t *)(b + h.off_nz_tiles);
    d.zero_tiles = (const uint32_t *)(b + h.off_zero_tiles);
    d.shared = (const SharedRec *)(b + h.off_shared);
    d.counters = (uint32_t *)(b + h.off_counters);
    d.n_chunks = h.n_chunks; d.waves_per_chunk = h.waves_per_chunk;
    d.n_zero_tiles = h.n_zero_tiles; d.n_shared = h.n_shared;
    d.br = h.br; d.bc = h.bc;
    d.rows_out = (uint32_t)h.rows_out; d.cols = (uint32_t)h.cols;
    d.n_groups = h.n_groups;
    return d;
}

__device__ __forceinline__ uint32_t uni(uint32_t v) { return __builtin_amdgcn_readfirstlane(v); }

// The wavefront's share of the mat-vec: accumulates into myacc[(tile slot) * br + row slot].
__device__ __forceinline__ void wave_groups(const DevMat &m, const WaveRec wr, const uint32_t nzrank0,
                                            const float *z, float *myacc, const int lane) {
    const uint32_t g_begin = uni(wr.g_begin), g_end = uni(wr.g_end);
    for (uint32_t g = g_begin; g <= g_end && g < m.n_groups; ++g) {
        const GroupRec *gp = m.groups + g;
        const uint32_t cmax = uni(gp->cmax), nvb = uni(gp->nvb), nlanes = uni(gp->nlanes);
        const uint32_t jlo = g == g_begin ? uni(wr.j_begin) : 0u;
        const uint32_t jhi = g == g_end ? uni(wr.j_end) : cmax;
        if (jhi <= jlo) continue;
        const uint32_t idx_off = uni(gp->idx_off), vb_off = uni(gp->vb_off);
        const float *gv = m.vals + uni(gp->val_off) + (g == g_begin ? uni(wr.val_begin) : 0u);
        const bool act = (uint32_t)lane < nlanes;
        uint32_t slot = 0, k = 0xffffffffu, c_lane = 0, zb = 0;
        const uint8_t *colp = m.idx;
        if (act) {
            const uint32_t d = *(const uint16_t *)(m.idx + idx_off + 2 * lane);
            slot = d & 0xffu;
            k = d >> 8;
            const VbRec v = m.vbs[vb_off + k];
            c_lane = v.c;
            zb = (uint32_t)v.bj * m.bc;
            colp = m.idx + idx_off + ((2 * nlanes + 3) & ~3u) + 4u * v.coloff4;
        }
        float a = 0.0f;
        uint32_t off = 0;
        for (uint32_t j = jlo; j < jhi; ++j) {
            const bool on = j < c_lane;
            if (on) {
                const float w = gv[off + lane];
                const uint32_t col = colp[j];
                a = fmaf(w, z[zb + col], a);
            }
            off += (uint32_t)__popcll(__ballot(on));
        }
        // Row results into the wavefront's accumulator.  Lanes of different virtual blocks
        // may target the same row, so the blocks go one after another; a wavefront's LDS
        // operations execute in program order, which fixes the order of the sum.
        const uint32_t rs = (uni(gp->nzrank) - nzrank0) * m.br + slot;
        for (uint32_t kk = 0; kk < nvb; ++kk) {
            if (k == kk) __hip_atomic_fetch_add(&myacc[rs], a, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
        }
    }
}

template <int NW>
__global__ __launch_bounds__(NW * 64) void spmv_kernel(const DevMat m, const float *__restrict__ x0,
                                                        const uint32_t n0, const float *__restrict__ x1,
                                                        float *__restrict__ y, float *__restrict__ partials,
                                                        const uint32_t zpad) {
    extern __shared__ float smem[];
    __shared__ uint32_t s_last;
    float *z = smem;            // [zpad] input vector
    float *acc = smem + zpad;   // [NW][ntiles * br]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t c = blockIdx.x;
    constexpr int NT = NW * 64;

    for (uint32_t i = tid; i < m.cols; i += NT) z[i] = i < n0 ? x0[i] : x1[i - n0];
    const ChunkRec cr = m.chunks[c];
    const uint32_t arows = cr.ntiles * m.br;
    for (uint32_t i = tid; i < NW * arows; i += NT) acc[i] = 0.0f;
    // output tiles nobody has work for
    for (uint32_t q = c; q < m.n_zero_tiles; q += m.n_chunks) {
        const uint32_t r0 = m.zero_tiles[q] * m.br;
        for (uint32_t i = tid; i < m.br; i += NT)
            if (r0 + i < m.rows_out) y[r0 + i] = 0.0f;
    }
    __syncthreads();

    wave_groups(m, m.waves[(size_t)c * NW + wave], cr.nzrank0, z, acc + wave * arows, lane);
    __syncthreads();

    // sum over wavefronts in wavefront order; store or hand over as a partial
    for (uint32_t i = tid; i < arows; i += NT) {
        float s = 0.0f;
#pragma unroll
        for (int w = 0; w < NW; ++w) s += acc[w * arows + i];
        const uint32_t ts = i / m.br, ri = i - ts * m.br;
        const uint32_t row = m.nz_tiles[cr.nzrank0 + ts] * m.br + ri;
        if (ts == 0 && cr.sid_first >= 0)
            partials[(size_t)(m.shared[cr.sid_first].partial_off + cr.part_first) * m.br + ri] = s;
        else if (ts == cr.ntiles - 1 && cr.sid_last >= 0)
            partials[(size_t)(m.shared[cr.sid_last].partial_off + cr.part_last) * m.br + ri] = s;
        else if (row < m.rows_out)
            y[row] = s;
    }
    // shared tiles: the last workgroup to arrive adds the parts in part order
#pragma unroll
    for (int e = 0; e < 2; ++e) {
        const int32_t sid = e == 0 ? cr.sid_first : cr.sid_last;
        if (sid < 0) continue;               // uniform over the workgroup
        __threadfence();
        __syncthreads();
        const SharedRec sr = m.shared[sid];
        if (tid == 0) {
            const uint32_t t = __hip_atomic_fetch_add(&m.counters[sid], 1u, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
            s_last = t == sr.nparts - 1 ? 1u : 0u;
        }
        __syncthreads();
        if (s_last) {
            __threadfence();
            for (uint32_t i = tid; i < m.br; i += NT) {
                const uint32_t row = sr.tile * m.br + i;
                if (row >= m.rows_out) continue;
                float s = 0.0f;
                for (uint32_t p = 0; p < sr.nparts; ++p)
                    s += __builtin_nontemporal_load(&partials[(size_t)(sr.partial_off + p) * m.br + i]);
                y[row] = s;
            }
            if (tid == 0) __hip_atomic_store(&m.counters[sid], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        __syncthreads();
    }
}

static hipError_t launch_spmv(const csb_matrix *mat, const float *x0, uint32_t n0, const float *x1, float *y,
                              float *partials, hipStream_t stream) {
    const DevHeader &h = mat->plan.hdr;
    const DevMat dm = dev_mat(mat);
    const uint32_t zpad = ((uint32_t)h.cols + 63u) & ~63u;
    const size_t lds = ((size_t)zpad + (size_t)h.waves_per_chunk * h.max_chunk_tiles * h.br) * sizeof(float);
    auto go = [&](auto kern, int nw) -> hipError_t {
        if (lds > 48 * 1024) {
            hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
        }
        hipLaunchKernelGGL(kern, dim3(h.n_chunks), dim3(nw * 64), lds, stream, dm, x0, n0, x1, y, partials, zpad);
        return hipGetLastError();
    };
    switch (h.waves_per_chunk) {
        case 4: return go(spmv_kernel<4>, 4);
        case 8: return go(spmv_kernel<8>, 8);
        default: return go(spmv_kernel<16>, 16);
    }
}

int spmv_segments(const csb_matrix *m, const float *d_x0, uint32_t n0, const float *d_x1, float *d_y,
                  void *d_ws, void *stream) {
    if (!m->plan.valid || !m->uploaded || !m->d_buf) { set_error("csb_spmv: matrix not planned and uploaded"); return CSB_ESTATE; }
    if (m->plan.hdr.cols > (uint64_t)kMaxStageCols) { set_error("csb_spmv: more columns than the LDS staging covers"); return CSB_EUNSUPPORTED; }
    if (m->plan.hdr.n_partial_slots && !d_ws) { set_error("csb_spmv: workspace is NULL"); return CSB_EINVAL; }
    hipError_t e = launch_spmv(m, d_x0, n0, d_x1, d_y, (float *)d_ws, (hipStream_t)stream);
    if (e != hipSuccess) { set_error(std::string("csb_spmv: ") + hipGetErrorString(e)); return CSB_EDEVICE; }
    return CSB_OK;
}

}  // namespace csb

extern "C" int csb_upload(csb_matrix *m, void *d_buf, size_t bytes, void *stream) {
    if (!m || !d_buf) { csb::set_error("csb_upload: NULL pointer"); return CSB_EINVAL; }
    if (!m->plan.valid) { csb::set_error("csb_upload: matrix not planned"); return CSB_ESTATE; }
    if (bytes < m->plan.image.size()) { csb::set_error("csb_upload: device buffer too small"); return CSB_ENOMEM; }
    if ((uintptr_t)d_buf % 256) { csb::set_error("csb_upload: device buffer not 256-byte aligned"); return CSB_EINVAL; }
    hipError_t e = hipMemcpyAsync(d_buf, m->plan.image.data(), m->plan.image.size(), hipMemcpyHostToDevice,
                                  (hipStream_t)stream);
    if (e != hipSuccess) { csb::set_error(std::string("csb_upload: ") + hipGetErrorString(e)); return CSB_EDEVICE; }
    m->d_buf = d_buf;
    m->uploaded = true;
    return CSB_OK;
}

extern "C" int csb_spmv(const csb_matrix *m, const float *d_x, float *d_y, void *d_ws, void *stream) {
    if (!m || !d_x || !d_y) { csb::set_error("csb_spmv: NULL pointer"); return CSB_EINVAL; }
    if (m->plan.valid && m->plan.split.active()) { csb::set_error("csb_spmv: matrix is planned for a GRU step"); return CSB_ESTATE; }
    return csb::spmv_segments(m, d_x, (uint32_t)m->cols, d_x, d_y, d_ws, stream);
}
