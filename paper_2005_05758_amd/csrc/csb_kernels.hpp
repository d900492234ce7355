// Internal entry points between the translation units of the library.
#pragma once

#include <hip/hip_runtime.h>

#include "csb_internal.hpp"

namespace csb {

constexpr int kMaxJobsPerLaunch = 4;   // independent products that may share one launch

// A segment of the mat-vec's input that is not in memory yet: the output h_t of a recurrent
// cell whose gate sums `a` an earlier launch on the same stream has produced.  The mat-vec
// kernel applies the cell's element-wise part (Sec. 2.1) while it stages its input, so a
// timestep of the streaming path is one launch per layer instead of two; every workgroup
// recomputes the (cheap) gates, workgroup 0 also stores the new state where the next step
// reads it.  kind 0: a plain vector at `a`.
struct GateSrc {
    const float *a;        // kind 0: the vector itself; else the sums, rows stacked as the cell stacks them
    const float *a2;       // reset-before GRU, gate part: the candidate's recurrent sums Un (r h_(t-1))
    const float *bias;     // may be null
    const float *c_in;     // LSTM: c_(t-1)
    const float *h_in;     // GRU, Li-GRU: h_(t-1)
    float *c_out, *h_out;  // where c_t (LSTM) and h_t go; distinct from c_in / h_in
    float *hseq;           // also h_t, or null
    uint32_t kind;         // 0 plain, else 1 + CSB_CELL_LSTM / _GRU / _LIGRU, or one of the two below
    uint32_t H;
};
constexpr uint32_t kGateRbReset = 6;   // reset-before GRU: q = sigmoid(a_r) h_(t-1), the operand of the second product
constexpr uint32_t kGateRbGate = 7;    // reset-before GRU: h_t from the z and n rows of a, and a2
__device__ __host__ inline GateSrc plain_src(const float *v) {
    GateSrc g{};
    g.a = v;
    return g;
}

#ifdef __HIPCC__
// Gate non-linearities of every path, built on the hardware exp2 and reciprocal
// (each within 1 ulp): sigmoid(v) = 1 / (1 + 2^(-v log2 e)); tanh(v) = 2 sigmoid(2v) - 1 for
// |v| >= 0.1 and its odd Taylor polynomial up to v^5 below (truncation 17 v^7 / 315 < 6e-9
// there), which keeps the relative error near zero small.  Absolute error below 5e-7 for any v
// (the argument scaling adds |v| 2^-24 relative error to the exponential, which only matters
// while the exponential is not negligible against 1).  A few instructions each: the kernels
// that stage a cell's output on their way in run for microseconds and pay for their code size.
__device__ __forceinline__ float fast_sigmoid(float v) {
    const float e = __builtin_amdgcn_exp2f(-1.44269504088896341f * v);
    return __builtin_amdgcn_rcpf(1.0f + e);
}
__device__ __forceinline__ float tanh_small(float v) {
    const float v2 = v * v;
    return v * fmaf(v2, fmaf(v2, 2.0f / 15.0f, -1.0f / 3.0f), 1.0f);
}
__device__ __forceinline__ float fast_tanh(float v) {
    const float big = fmaf(2.0f, fast_sigmoid(2.0f * v), -1.0f);
    return fabsf(v) < 0.1f ? tanh_small(v) : big;
}

// h_t of unit u of the cell whose gate sums are s.a (Sec. 2.1; LSTM rows i,f,g,o; GRU rows r,z,
// input side of n, recurrent side of n; Li-GRU rows z, candidate), the same arithmetic as the
// stand-alone gate kernels.  `store`: also write the new state (and the output sequence).
__device__ __forceinline__ float gate_value(const GateSrc &s, uint32_t u, bool store) {
    const uint32_t H = s.H;
    const float *a = s.a, *b = s.bias;
    float hn, cn = 0.0f;
    if (s.kind == 1u + CSB_CELL_LSTM) {
        float ai = a[u], af = a[H + u], ag = a[2 * H + u], ao = a[3 * H + u];
        if (b) { ai += b[u]; af += b[H + u]; ag += b[2 * H + u]; ao += b[3 * H + u]; }
        cn = fast_sigmoid(af) * s.c_in[u] + fast_sigmoid(ai) * fast_tanh(ag);
        hn = fast_sigmoid(ao) * fast_tanh(cn);
    } else if (s.kind == 1u + CSB_CELL_GRU) {
        float ar = a[u], az = a[H + u], anx = a[2 * H + u];
        const float anh = a[3 * H + u];
        if (b) { ar += b[u]; az += b[H + u]; anx += b[2 * H + u]; }
        const float r = fast_sigmoid(ar), z = fast_sigmoid(az);
        hn = (1.0f - z) * fast_tanh(anx + r * anh) + z * s.h_in[u];
    } else if (s.kind == kGateRbReset) {                       // rows r,z,n; only r is needed here
        float ar = a[u];
        if (b) ar += b[u];
        hn = fast_sigmoid(ar) * s.h_in[u];
    } else if (s.kind == kGateRbGate) {
        float az = a[H + u], an = a[2 * H + u] + s.a2[u];
        if (b) { az += b[H + u]; an += b[2 * H + u]; }
        const float z = fast_sigmoid(az);
        hn = (1.0f - z) * fast_tanh(an) + z * s.h_in[u];
    } else {                                                   // Li-GRU
        float az = a[u], ac = a[H + u];
        if (b) { az += b[u]; ac += b[H + u]; }
        const float z = fast_sigmoid(az);
        hn = z * s.h_in[u] + (1.0f - z) * fmaxf(ac, 0.0f);
    }
    if (store) {
        if (s.c_out) s.c_out[u] = cn;
        if (s.h_out) s.h_out[u] = hn;
        if (s.hseq) s.hseq[u] = hn;
    }
    return hn;
}

// One segment of the input vector into LDS: a plain copy, or the cell outputs computed on the way.
__device__ __forceinline__ void stage_segment(float *z, const GateSrc &s, uint32_t n, uint32_t tid, uint32_t nthreads, bool store) {
    if (s.kind == 0u) {                                        // uniform
        for (uint32_t u = tid; u < n; u += nthreads) z[u] = s.a[u];
    } else {
        for (uint32_t u = tid; u < n; u += nthreads) z[u] = gate_value(s, u, store);
    }
}
#endif

// y = A [x0[0..n0) ; x1[0..cols-n0)] on `stream`; y has the image's rows_out entries.
int spmv_segments(const csb_matrix *m, const float *d_x0, uint32_t n0, const float *d_x1, float *d_y,
                  void *d_ws, void *stream, unsigned long long *d_stamps = nullptr);
// y = A x from the row-owned stream section of the image (plan.stream.valid) on `stream`.
int spmv_rows(const csb_matrix *m, const float *d_x, float *d_y, void *stream, unsigned long long *d_stamps = nullptr);
// The same with the input vector in two segments, either one possibly a cell output still to be
// computed (see GateSrc); several independent such products in one launch (at most kMaxJobsPerLaunch).
int spmv_rows_gated(const csb_matrix *m, const GateSrc &s0, uint32_t n0, const GateSrc &s1, float *d_y, void *stream);
struct SpmvGatedCall;
int spmv_rows_gated_multi(const SpmvGatedCall *calls, int n, void *stream);
// One step of a recurrent layer (LSTM, GRU, Li-GRU; Sec. 2.1) in one launch: the product
// W [x0[0..n0) ; h_prev] from a row-owned plan whose workgroups own whole units
// (StreamPlan::cell_gates), then the element-wise part, by the workgroup that has a unit's sums:
// c_t (LSTM: c_in -> c_out) and h_t -> h_out (and hseq).  h_out is not h_prev.  The second segment
// has the matrix's other columns; for the LSTM it need not be the cell's own output (LSTMP: it is
// the projected state, and h_out receives m_t).
// The reset-before GRU takes two such launches per step: kCellRbReset on its first matrix (rows r, z,
// n over [input ; h_(t-1)]) writes q = sigmoid(a_r) h_(t-1) to h_out, z = sigmoid(a_z) to c_out and
// the n row's sum (with its bias) to hseq; kCellRbGate on the second (Un, one row per unit, input q:
// n0 = all columns) reads z from c_in, that sum from aux and h_(t-1) from h_state, and writes
// h_t = (1 - z) tanh(sum + Un q) + z h_(t-1) to h_out (and hseq).
constexpr int32_t kCellRbReset = 100, kCellRbGate = 101;
struct SpmvCellCall {
    const csb_matrix *mat;
    const float *x0;
    uint32_t n0;
    const float *h_prev;       // the second input segment (any valid pointer if there is none); null: zeros
                               // (LSTM, GRU, Li-GRU; c_in null likewise: the state of a sequence that starts at zero)
    int32_t cell;              // CSB_CELL_LSTM, CSB_CELL_GRU, CSB_CELL_LIGRU, kCellRbReset or kCellRbGate
    const float *bias;         // as the cell stacks them, or null
    const float *c_in;
    float *c_out, *h_out, *hseq;
    const float *h_state = nullptr;   // h_(t-1) where it is not the second input segment
    const float *aux = nullptr;
};
// ... for up to kMaxJobsPerLaunch layers at once (one value format for all).
int spmv_rows_cell_multi(const SpmvCellCall *calls, int n, void *stream);
// Up to kMaxJobsPerLaunch independent plain products y = A x from row-owned plans in one launch.
struct SpmvPlainCall {
    const csb_matrix *mat;
    const float *x;
    float *y;
};
int spmv_rows_multi(const SpmvPlainCall *calls, int n, void *stream);
// ... with either segment possibly a cell output still to be computed (see GateSrc).
int spmv_gated(const csb_matrix *m, const GateSrc &s0, uint32_t n0, const GateSrc &s1, float *d_y, void *d_ws, void *stream);
// The element-wise part alone, one thread per unit: stores c_t, h_t (and hseq) of `s`.
int commit_gates(const GateSrc &s, void *stream);
// One product of spmv_gated_multi (the arguments of spmv_gated).
struct SpmvGatedCall {
    const csb_matrix *mat;
    GateSrc s0;
    uint32_t n0;
    GateSrc s1;
    float *y;
    void *ws;
};
// Several independent gated mat-vecs on `stream`: one launch when there are two to four of one
// value format (the layers of a stacked model on one diagonal), else a launch each.
int spmv_gated_multi(const SpmvGatedCall *calls, int n, void *stream);

// Y = A Z for `batch` right-hand sides.  Element (column j, right-hand side n) of Z is
// p0[j*sj0 + n*sn0] for j < n0 and p1[(j-n0)*sj1 + n*sn1] otherwise; Y is [rows_out][ldy].
int spmm_strided(const csb_matrix *mat, const float *p0, uint32_t n0, int64_t sj0, int64_t sn0, const float *p1,
                 int64_t sj1, int64_t sn1, float *d_Y, int64_t ldy, int32_t batch, void *stream);

// Raises a kernel's limit of dynamic LDS on the current device to `bytes` if it is below it.
// (The limit sticks to the kernel; setting it is a runtime call of its own, too slow to repeat
// before every launch of a path that launches a kernel per timestep.)
hipError_t ensure_dynamic_lds(const void *kernel, size_t bytes);

// One product of spmm_strided_multi (the arguments of spmm_strided).
struct SpmmCall {
    const csb_matrix *mat;
    const float *p0;
    uint32_t n0;
    int64_t sj0, sn0;
    const float *p1;
    int64_t sj1, sn1;
    float *Y;
    int64_t ldy;
};
// Several independent products of the same batch on `stream`: one launch when their launch
// shapes agree (the layers of a stacked model), else one launch each.
int spmm_strided_multi(const SpmmCall *calls, int n, int32_t batch, void *stream);

}  // namespace csb
