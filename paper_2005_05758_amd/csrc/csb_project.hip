// Projection of a dense matrix onto the CSB pattern (the pruning step inside Algorithm 1,
// Sec. 3.2.2) for gfx950: RowPrune in every block-column, then ColumnPrune in every
// block-row on the row-pruned matrix, each zeroing the share 1 - sqrt(1 - PruneRate) of the
// segments with the smallest sums of squares.
//
// Five launches on one stream: sums of squares of the in-block row segments, selection per
// block-column, sums of squares of the in-block column segments of the row-pruned matrix,
// selection per block-row, and the masked copy.  The decisions are integers taken from
// float32 sums, so the sums use one fixed order (left to right / top to bottom, one fused
// multiply-add per element) and ties go by position: the result is the same bits on every
// run and on every machine that does the arithmetic this way.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>

#include "csb_internal.hpp"

namespace csb {

constexpr int kProjectMaxDim = 16384;     // segments ranked by one workgroup in LDS

// Ranking key of a sum of squares: its bit pattern (sums are >= +0 or NaN, so the unsigned
// order of the bits is the numeric order); every NaN ranks on top.
__device__ __forceinline__ uint32_t rank_key(float s) {
    const uint32_t u = __float_as_uint(s);
    return s != s ? 0xffffffffu : u;
}

// keys[bj * R + i] for row segment (i, bj).  A workgroup takes TR rows x TS segments: it
// reads their columns coalesced into LDS (segment stride BC | 1 words, so that the lanes of
// the next phase hit different banks), then thread (r, sj) adds up its own segment from left
// to right.  DIV_SHIFT >= 0: BC is 1 << DIV_SHIFT.
template <int DIV_SHIFT>
__global__ __launch_bounds__(256) void row_segment_keys_kernel(const float *__restrict__ W, const int64_t ld,
                                                                 const uint32_t R, const uint32_t C, const uint32_t BC,
                                                                 const uint32_t NBC, const uint32_t TR, const uint32_t TS,
                                                                 uint32_t *__restrict__ keys) {
    extern __shared__ float tile[];
    const uint32_t tid = threadIdx.x;
    const uint32_t bj0 = blockIdx.x * TS, i0 = blockIdx.y * TR;
    const uint32_t c0 = bj0 * BC, c1 = min(C, (bj0 + TS) * BC), ncols = c1 - c0;
    const uint32_t BCp = BC | 1u;
    for (uint32_t r = 0; r < TR && i0 + r < R; ++r) {
        const float *p = W + (size_t)(i0 + r) * ld + c0;
        float *row = tile + (size_t)r * TS * BCp;
        for (uint32_t cb = tid; cb < ncols; cb += 1024) {           // four independent loads per pass
            float v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) v[u] = cb + 256u * u < ncols ? p[cb + 256u * u] : 0.0f;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const uint32_t cc = cb + 256u * u;
                if (cc < ncols) {
                    const uint32_t seg = DIV_SHIFT >= 0 ? cc >> (DIV_SHIFT >= 0 ? DIV_SHIFT : 0) : cc / BC;
                    row[seg * BCp + (cc - seg * BC)] = v[u];
                }
            }
        }
    }
    __syncthreads();
    const uint32_t r = tid / TS, sj = tid - r * TS;
    if (r < TR && i0 + r < R && bj0 + sj < NBC) {
        const uint32_t w = min(BC, C - (bj0 + sj) * BC);
        const float *q = tile + ((size_t)r * TS + sj) * BCp;
        float s = 0.0f;
        for (uint32_t c = 0; c < w; ++c) s = fmaf(q[c], q[c], s);
        keys[(size_t)(bj0 + sj) * R + i0 + r] = rank_key(s);
    }
}

// keys[bi * C + c] for column segment (bi, c) of the row-pruned matrix: thread per segment,
// c fastest (every row of the segment is read coalesced).
__global__ __launch_bounds__(256) void col_segment_keys_kernel(const float *__restrict__ W, const int64_t ld,
                                                                 const uint32_t R, const uint32_t C, const uint32_t BR,
                                                                 const uint32_t BC, const uint8_t *__restrict__ keep_r,
                                                                 uint32_t *__restrict__ keys) {
    const uint32_t c = blockIdx.x * blockDim.x + threadIdx.x, bi = blockIdx.y;
    if (c >= C) return;
    const uint32_t r0 = bi * BR, r1 = min(R, r0 + BR);
    const uint8_t *kr = keep_r + (size_t)(c / BC) * R;
    float s = 0.0f;
    for (uint32_t i = r0; i < r1; ++i) {
        const float v = kr[i] ? W[(size_t)i * ld + c] : 0.0f;
        s = fmaf(v, v, s);
    }
    keys[(size_t)bi * C + c] = rank_key(s);
}

// One workgroup ranks the n segments of one block-column (block-row): bitonic sort of
// (key, position) words in LDS; the first k of the ascending order are the pruned ones.
__global__ __launch_bounds__(1024) void select_kernel(const uint32_t *__restrict__ keys, uint8_t *__restrict__ keep,
                                                       const uint32_t n, const uint32_t P, const uint32_t k) {
    extern __shared__ unsigned long long sk[];
    const uint32_t tid = threadIdx.x;
    const size_t base = (size_t)blockIdx.x * n;
    for (uint32_t i = tid; i < P; i += 1024)
        sk[i] = i < n ? ((unsigned long long)keys[base + i] << 32) | i : ~0ull;
    __syncthreads();
    for (uint32_t size = 2; size <= P; size <<= 1)
        for (uint32_t stride = size >> 1; stride > 0; stride >>= 1) {
            for (uint32_t t = tid; t < P / 2; t += 1024) {
                const uint32_t i = (t / stride) * 2 * stride + (t & (stride - 1)), j = i + stride;
                const bool ascending = (i & size) == 0;
                const unsigned long long a = sk[i], b = sk[j];
                if ((a > b) == ascending) { sk[i] = b; sk[j] = a; }
            }
            __syncthreads();
        }
    for (uint32_t i = tid; i < n; i += 1024) keep[base + (uint32_t)sk[i]] = i >= k ? 1 : 0;
}

// Z = W where both its row segment and its column segment survive, else +0.  A thread takes
// four consecutive columns of one row (kMaskedCopyRows rows per workgroup).
constexpr int kMaskedCopyRows = 4;
__global__ __launch_bounds__(256) void masked_copy_kernel(const float *W, const int64_t ld, float *Z,
                                                            const int64_t ldz, const uint32_t R, const uint32_t C,
                                                            const uint32_t BR, const uint32_t BC,
                                                            const uint8_t *__restrict__ keep_r, const uint8_t *__restrict__ keep_c,
                                                            const bool vec4) {
    const uint32_t c = (blockIdx.x * 64u + (threadIdx.x & 63u)) * 4u;
    const uint32_t i = blockIdx.y * kMaskedCopyRows + (threadIdx.x >> 6);
    if (c >= C || i >= R) return;
    const uint8_t *kc = keep_c + (size_t)(i / BR) * C;
    if (vec4 && c + 3 < C) {
        const float4 w = *(const float4 *)(W + (size_t)i * ld + c);
        const uint32_t kc4 = *(const uint32_t *)(kc + c);           // four keep flags (C is a multiple of 4 here)
        float4 z;
        z.x = keep_r[(size_t)(c / BC) * R + i] && (kc4 & 0xffu) ? w.x : 0.0f;
        z.y = keep_r[(size_t)((c + 1) / BC) * R + i] && (kc4 & 0xff00u) ? w.y : 0.0f;
        z.z = keep_r[(size_t)((c + 2) / BC) * R + i] && (kc4 & 0xff0000u) ? w.z : 0.0f;
        z.w = keep_r[(size_t)((c + 3) / BC) * R + i] && (kc4 & 0xff000000u) ? w.w : 0.0f;
        *(float4 *)(Z + (size_t)i * ldz + c) = z;
    } else {
        for (uint32_t cc = c; cc < min(C, c + 4u); ++cc) {
            const bool on = keep_r[(size_t)(cc / BC) * R + i] && kc[cc];
            Z[(size_t)i * ldz + cc] = on ? W[(size_t)i * ld + cc] : 0.0f;
        }
    }
}

static size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

struct ProjectLayout {
    size_t keys_r, keep_r, keys_c, keep_c, total;
};

static ProjectLayout project_layout(int64_t R, int64_t C, int32_t br, int32_t bc) {
    const size_t nbr = (size_t)((R + br - 1) / br), nbc = (size_t)((C + bc - 1) / bc);
    ProjectLayout L{};
    size_t off = 0;
    L.keys_r = off; off = align256(off + nbc * (size_t)R * 4);
    L.keep_r = off; off = align256(off + nbc * (size_t)R);
    L.keys_c = off; off = align256(off + nbr * (size_t)C * 4);
    L.keep_c = off; off = align256(off + nbr * (size_t)C);
    L.total = off;
    return L;
}

// Segments zeroed among n at pruning rate `rate` x: floor(n (1 - rate^-1/2) + 1/2).
static uint32_t prune_count(int64_t n, double rate) {
    const double q = 1.0 - 1.0 / std::sqrt(rate);
    int64_t k = (int64_t)std::floor((double)n * q + 0.5);
    if (k < 0) k = 0;
    if (k > n) k = n;
    return (uint32_t)k;
}

static uint32_t pow2_at_least(uint32_t n) {
    uint32_t p = 2;
    while (p < n) p <<= 1;
    return p;
}

}  // namespace csb

extern "C" size_t csb_project_workspace_bytes(int64_t rows, int64_t cols, int32_t br, int32_t bc) {
    if (rows <= 0 || cols <= 0 || br < 1 || bc < 1) return 0;
    return csb::project_layout(rows, cols, br, bc).total;
}

extern "C" int csb_project(const float *d_W, int64_t rows, int64_t cols, int64_t ld, int32_t br, int32_t bc,
                           double rate, float *d_Z, int64_t ldz, void *d_ws, void *stream) {
    using namespace csb;
    if (!d_W || !d_Z || !d_ws) { set_error("csb_project: NULL pointer"); return CSB_EINVAL; }
    if (rows <= 0 || cols <= 0 || ld < cols || ldz < cols) { set_error("csb_project: bad shape or leading dimension"); return CSB_EINVAL; }
    if (br < 1 || br > CSB_MAX_BLOCK || bc < 1 || bc > CSB_MAX_BLOCK) { set_error("csb_project: block size outside [1, 256]"); return CSB_EINVAL; }
    if (!(rate >= 1.0) || !std::isfinite(rate)) { set_error("csb_project: pruning rate must be a finite number >= 1"); return CSB_EINVAL; }
    if (rows > kProjectMaxDim || cols > kProjectMaxDim) {
        set_error("csb_project: more than 16384 rows or columns (one workgroup ranks a block-column in LDS)");
        return CSB_EUNSUPPORTED;
    }
    const uint32_t R = (uint32_t)rows, C = (uint32_t)cols, BR = (uint32_t)br, BC = (uint32_t)bc;
    const uint32_t NBR = (R + BR - 1) / BR, NBC = (C + BC - 1) / BC;
    const ProjectLayout L = project_layout(rows, cols, br, bc);
    uint8_t *ws = (uint8_t *)d_ws;
    uint32_t *keys_r = (uint32_t *)(ws + L.keys_r), *keys_c = (uint32_t *)(ws + L.keys_c);
    uint8_t *keep_r = ws + L.keep_r, *keep_c = ws + L.keep_c;
    hipStream_t st = (hipStream_t)stream;
    const uint32_t Pr = pow2_at_least(R), Pc = pow2_at_least(C);
    hipError_t e = hipFuncSetAttribute((const void *)select_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)(std::max(Pr, Pc) * sizeof(unsigned long long)));
    if (e == hipSuccess) {
        // tile of the row-sum kernel: TS segments x TR rows, at most 256 threads and 48 KB of LDS
        const uint32_t BCp = BC | 1u;
        const uint32_t TS = std::max(1u, std::min({NBC, 256u, 12288u / BCp}));
        const uint32_t TR = std::max(1u, std::min({256u / TS, 12288u / (TS * BCp), R}));
        const size_t lds_rows = (size_t)TR * TS * BCp * sizeof(float);
        const dim3 grid_r((NBC + TS - 1) / TS, (R + TR - 1) / TR);
        int shift = -1;
        for (int b = 0; b < 9; ++b) if (BC == (1u << b)) shift = b;
        switch (shift) {
            case 4: hipLaunchKernelGGL(row_segment_keys_kernel<4>, grid_r, dim3(256), lds_rows, st, d_W, ld, R, C, BC, NBC, TR, TS, keys_r); break;
            case 5: hipLaunchKernelGGL(row_segment_keys_kernel<5>, grid_r, dim3(256), lds_rows, st, d_W, ld, R, C, BC, NBC, TR, TS, keys_r); break;
            case 6: hipLaunchKernelGGL(row_segment_keys_kernel<6>, grid_r, dim3(256), lds_rows, st, d_W, ld, R, C, BC, NBC, TR, TS, keys_r); break;
            default: hipLaunchKernelGGL(row_segment_keys_kernel<-1>, grid_r, dim3(256), lds_rows, st, d_W, ld, R, C, BC, NBC, TR, TS, keys_r); break;
        }
        hipLaunchKernelGGL(select_kernel, dim3(NBC), dim3(1024), Pr * sizeof(unsigned long long), st, keys_r, keep_r, R, Pr,
                           prune_count(rows, rate));
        hipLaunchKernelGGL(col_segment_keys_kernel, dim3((C + 255) / 256, NBR), dim3(256), 0, st, d_W, ld, R, C, BR, BC, keep_r, keys_c);
        hipLaunchKernelGGL(select_kernel, dim3(NBR), dim3(1024), Pc * sizeof(unsigned long long), st, keys_c, keep_c, C, Pc,
                           prune_count(cols, rate));
        // float4 accesses need 16-byte aligned rows on both sides (and flag words at multiples of 4)
        const bool vec4 = C % 4 == 0 && ld % 4 == 0 && ldz % 4 == 0 && (uintptr_t)d_W % 16 == 0 && (uintptr_t)d_Z % 16 == 0;
        hipLaunchKernelGGL(masked_copy_kernel, dim3((C + 255) / 256, (R + kMaskedCopyRows - 1) / kMaskedCopyRows), dim3(256), 0, st,
                           d_W, ld, d_Z, ldz, R, C, BR, BC, keep_r, keep_c, vec4);
        e = hipGetLastError();
    }
    if (e != hipSuccess) { set_error(std::string("csb_project: ") + hipGetErrorString(e)); return CSB_EDEVICE; }
    return CSB_OK;
}
