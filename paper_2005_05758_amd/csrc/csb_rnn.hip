// LSTM / GRU inference over a sequence (Sec. 2.1) on top of the CSB mat-vec.
#include <hip/hip_runtime.h>

#include <new>
#include <vector>

#include "csb_internal.hpp"
#include "csb_kernels.hpp"

struct csb_rnn {
    int32_t cell = 0, n_layers = 0, input = 0, hidden = 0;
    std::vector<csb_matrix *> W;
    std::vector<const float *> d_bias;
};

namespace csb {

__device__ __forceinline__ float sigmoidf_(float v) { return 1.0f / (1.0f + expf(-v)); }

// Element-wise part of the LSTM cell: a = W [u; h] (+ bias), rows i,f,g,o.
__global__ void lstm_gates_kernel(const float *__restrict__ a, const float *__restrict__ bias,
                                  float *__restrict__ c, float *__restrict__ h, float *__restrict__ hseq,
                                  const int H) {
    const int k = blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= H) return;
    float ai = a[k], af = a[H + k], ag = a[2 * H + k], ao = a[3 * H + k];
    if (bias) { ai += bias[k]; af += bias[H + k]; ag += bias[2 * H + k]; ao += bias[3 * H + k]; }
    const float cn = sigmoidf_(af) * c[k] + sigmoidf_(ai) * tanhf(ag);
    const float hn = sigmoidf_(ao) * tanhf(cn);
    c[k] = cn;
    h[k] = hn;
    if (hseq) hseq[k] = hn;
}

// Element-wise part of the GRU cell.  a has 4H rows: r, z (input + recurrent sums),
// then the n rows' input-side sum, then the n rows' recurrent-side sum.
__global__ void gru_gates_kernel(const float *__restrict__ a, const float *__restrict__ bias,
                                 float *__restrict__ h, float *__restrict__ hseq, const int H) {
    const int k = blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= H) return;
    float ar = a[k], az = a[H + k], anx = a[2 * H + k];
    const float anh = a[3 * H + k];
    if (bias) { ar += bias[k]; az += bias[H + k]; anx += bias[2 * H + k]; }
    const float r = sigmoidf_(ar), z = sigmoidf_(az);
    const float n = tanhf(anx + r * anh);
    const float hn = (1.0f - z) * n + z * h[k];
    h[k] = hn;
    if (hseq) hseq[k] = hn;
}

__global__ void fill_kernel(float *p, size_t n, float v) {
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = v;
}

__global__ void copy_kernel(float *__restrict__ d, const float *__restrict__ s, size_t n) {
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) d[i] = s[i];
}

static void init_state(float *dst, const float *src, size_t n, hipStream_t st) {
    const int blocks = (int)std::min<size_t>((n + 255) / 256, 1024);
    if (src) hipLaunchKernelGGL(copy_kernel, dim3(blocks), dim3(256), 0, st, dst, src, n);
    else hipLaunchKernelGGL(fill_kernel, dim3(blocks), dim3(256), 0, st, dst, n, 0.0f);
}

static size_t align256(size_t v) { return (v + 255) / 256 * 256; }

struct RnnWs {
    size_t off_a, off_c, off_part, total;
};

static RnnWs ws_layout(const csb_rnn *r, int32_t batch) {
    RnnWs w{};
    size_t off = 0;
    size_t rows_out = 0, part = 0;
    for (auto *m : r->W) {
        rows_out = std::max<size_t>(rows_out, (size_t)m->plan.hdr.rows_out);
        part = std::max<size_t>(part, (size_t)m->plan.hdr.n_partial_slots * m->plan.hdr.br * sizeof(float));
    }
    w.off_a = off; off = align256(off + rows_out * sizeof(float));
    w.off_c = off; off = align256(off + (size_t)r->n_layers * batch * r->hidden * sizeof(float));
    w.off_part = off; off = align256(off + part);
    w.total = off;
    return w;
}

}  // namespace csb

extern "C" int csb_rnn_create(int32_t cell, int32_t n_layers, int32_t input, int32_t hidden,
                              csb_matrix *const *W, const float *const *d_bias, csb_rnn **out) {
    using namespace csb;
    if (!W || !out) { set_error("csb_rnn_create: NULL pointer"); return CSB_EINVAL; }
    *out = nullptr;
    if (cell != CSB_CELL_LSTM && cell != CSB_CELL_GRU) { set_error("csb_rnn_create: unknown cell"); return CSB_EINVAL; }
    if (n_layers <= 0 || input <= 0 || hidden <= 0) { set_error("csb_rnn_create: non-positive size"); return CSB_EINVAL; }
    const int G = cell == CSB_CELL_LSTM ? 4 : 3;
    for (int l = 0; l < n_layers; ++l) {
        if (!W[l]) { set_error("csb_rnn_create: NULL weight matrix"); return CSB_EINVAL; }
        const int64_t n_in = l == 0 ? input : hidden;
        if (W[l]->rows != (int64_t)G * hidden || W[l]->cols != n_in + hidden) {
            set_error("csb_rnn_create: weight matrix shape does not match (G*hidden) x (in + hidden)");
            return CSB_EINVAL;
        }
    }
    try {
        auto *r = new csb_rnn();
        r->cell = cell; r->n_layers = n_layers; r->input = input; r->hidden = hidden;
        for (int l = 0; l < n_layers; ++l) {
            SplitSpec sp{};
            if (cell == CSB_CELL_GRU) { sp.split_row = 2 * (int64_t)hidden; sp.split_col = l == 0 ? input : hidden; sp.shift = hidden; }
            if (!W[l]->plan.valid || !(W[l]->plan.split == sp)) {
                int rc = plan_matrix(W[l], 0, 16, sp, nullptr, 0);
                if (rc != CSB_OK) { delete r; return rc; }
            }
            r->W.push_back(W[l]);
            r->d_bias.push_back(d_bias ? d_bias[l] : nullptr);
        }
        *out = r;
        return CSB_OK;
    } catch (const std::bad_alloc &) {
        set_error("csb_rnn_create: out of host memory");
        return CSB_ENOMEM;
    }
}

extern "C" size_t csb_rnn_workspace_bytes(const csb_rnn *r, int32_t batch, int32_t T) {
    (void)T;
    if (!r || batch <= 0) return 0;
    return csb::ws_layout(r, batch).total;
}

extern "C" int csb_rnn_forward(const csb_rnn *r, const float *d_x, const float *d_h0, const float *d_c0,
                               float *d_hseq, float *d_hT, float *d_cT, int32_t T, int32_t batch,
                               void *d_ws, void *stream) {
    using namespace csb;
    if (!r || !d_hT || !d_ws) { set_error("csb_rnn_forward: NULL pointer"); return CSB_EINVAL; }
    if (batch <= 0 || T < 0) { set_error("csb_rnn_forward: batch <= 0 or T < 0"); return CSB_EINVAL; }
    if (T > 0 && !d_x) { set_error("csb_rnn_forward: NULL input sequence"); return CSB_EINVAL; }
    for (auto *m : r->W)
        if (!m->plan.valid || !m->uploaded) { set_error("csb_rnn_forward: a weight matrix is not uploaded"); return CSB_ESTATE; }
    hipStream_t st = (hipStream_t)stream;
    const int L = r->n_layers, H = r->hidden, I = r->input;
    const bool lstm = r->cell == CSB_CELL_LSTM;
    const RnnWs wl = ws_layout(r, batch);
    float *a = (float *)((uint8_t *)d_ws + wl.off_a);
    float *c = (lstm && d_cT) ? d_cT : (float *)((uint8_t *)d_ws + wl.off_c);
    void *part = (uint8_t *)d_ws + wl.off_part;
    const size_t nstate = (size_t)L * batch * H;
    // the outputs double as the running state
    init_state(d_hT, d_h0, nstate, st);
    if (lstm) init_state(c, d_c0, nstate, st);
    const int gblocks = (H + 255) / 256;
    for (int t = 0; t < T; ++t)
        for (int s = 0; s < batch; ++s)
            for (int l = 0; l < L; ++l) {
                const float *u = l == 0 ? d_x + ((size_t)t * batch + s) * I : d_hT + ((size_t)(l - 1) * batch + s) * H;
                const uint32_t n_in = l == 0 ? (uint32_t)I : (uint32_t)H;
                float *h = d_hT + ((size_t)l * batch + s) * H;
                int rc = spmv_segments(r->W[l], u, n_in, h, a, part, st);
                if (rc != CSB_OK) return rc;
                float *hs = (d_hseq && l == L - 1) ? d_hseq + ((size_t)t * batch + s) * H : nullptr;
                if (lstm)
                    hipLaunchKernelGGL(lstm_gates_kernel, dim3(gblocks), dim3(256), 0, st, a, r->d_bias[l],
                                       c + ((size_t)l * batch + s) * H, h, hs, H);
                else
                    hipLaunchKernelGGL(gru_gates_kernel, dim3(gblocks), dim3(256), 0, st, a, r->d_bias[l], h, hs, H);
            }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) { set_error(std::string("csb_rnn_forward: ") + hipGetErrorString(e)); return CSB_EDEVICE; }
    return CSB_OK;
}

extern "C" void csb_rnn_free(csb_rnn *r) { delete r; }

extern "C" int csb_spmm(const csb_matrix *m, const float *d_X, int64_t ldx, float *d_Y, int64_t ldy,
                        int32_t batch, void *d_ws, void *stream) {
    (void)m; (void)d_X; (void)ldx; (void)d_Y; (void)ldy; (void)batch; (void)d_ws; (void)stream;
    csb::set_error("csb_spmm: not built yet");
    return CSB_EUNSUPPORTED;
}
