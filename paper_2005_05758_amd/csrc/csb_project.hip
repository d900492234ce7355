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

constexpr int kProjectMaxDim = 16384;     // segments ranked by one workgroup: 16 keys in each of 1024 threads

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

// One workgroup ranks the n <= 16384 segments of one block-column (block-row) and marks the k
// weakest as pruned, "weaker" being the order of (key, position).  No sort: every thread keeps
// 16 consecutive keys in registers; the key T of the k-th weakest is found bit by bit from the
// top (per bit: how many of the still possible keys have a 0 there -- wavefront counts by
// ballot, workgroup count through LDS); then a segment is pruned if its key is below T, or
// equal to T and fewer than (k - #below) equal keys lie at earlier positions.
constexpr int kSelPer = 16;          // keys per thread
__global__ __launch_bounds__(1024) void select_kernel(const uint32_t *__restrict__ keys, uint8_t *__restrict__ keep,
                                                       const uint32_t n, const uint32_t k) {
    __shared__ uint32_t wsum[3][16];
    __shared__ uint32_t cand[1024];              // the keys still possible once they are few (first: scratch)
    const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
    const size_t base = (size_t)blockIdx.x * n;
    const uint32_t i0 = tid * kSelPer;
    if (k == 0 || k >= n) {                      // nothing / everything pruned
        for (uint32_t q = 0; q < kSelPer; ++q)
            if (i0 + q < n) keep[base + i0 + q] = k == 0 ? 1 : 0;
        return;
    }
    uint32_t key[kSelPer];
    bool valid[kSelPer];
    const bool vec = (n & 15u) == 0;             // 16-byte accesses: every thread's run is whole and aligned
#pragma unroll
    for (int q = 0; q < kSelPer; ++q) valid[q] = i0 + q < n;
    if (vec) {
        if (valid[0]) {
            const uint4 *src = (const uint4 *)(keys + base + i0);
#pragma unroll
            for (int v = 0; v < kSelPer / 4; ++v) {
                const uint4 w = src[v];
                key[4 * v] = w.x; key[4 * v + 1] = w.y; key[4 * v + 2] = w.z; key[4 * v + 3] = w.w;
            }
        } else {
#pragma unroll
            for (int q = 0; q < kSelPer; ++q) key[q] = 0u;
        }
    } else {
#pragma unroll
        for (int q = 0; q < kSelPer; ++q) key[q] = valid[q] ? keys[base + i0 + q] : 0u;
    }
    // workgroup sum of a per-wavefront count (uniform in the wavefront)
    auto wg_sum = [&](uint32_t wave_count, int buf) {
        if (lane == 0) wsum[buf][wave] = wave_count;
        __syncthreads();
        uint32_t s = 0;
#pragma unroll
        for (int w = 0; w < 16; ++w) s += wsum[buf][w];
        return s;
    };
    // bits on which every key agrees need no counting
    uint32_t all_and = 0xffffffffu, all_or = 0u;
#pragma unroll
    for (int q = 0; q < kSelPer; ++q)
        if (valid[q]) { all_and &= key[q]; all_or |= key[q]; }
    for (int d = 32; d > 0; d >>= 1) {
        all_and &= (uint32_t)__shfl_xor((int)all_and, d, 64);
        all_or |= (uint32_t)__shfl_xor((int)all_or, d, 64);
    }
    if (lane == 0) { cand[wave] = all_and; cand[16 + wave] = all_or; }
    __syncthreads();
    for (int w = 0; w < 16; ++w) { all_and &= cand[w]; all_or |= cand[16 + w]; }
    __syncthreads();                             // cand is reused below
    const uint32_t varying = all_and ^ all_or;
    uint32_t prefix = 0, mask = 0, kk = k;       // the kk-th weakest of the keys that match prefix on mask
    uint32_t act = n;                            // keys still matching
    bool compact = false;                        // the matching keys have been gathered, one per thread
    uint32_t ckey = 0, ncand = 0;
    int par = 0;
    for (int b = 31; b >= 0; --b) {
        const uint32_t bit = 1u << b;
        if (!(varying & bit)) { prefix |= all_and & bit; mask |= bit; continue; }
        if (!compact && act <= 1024u) {
            // gather the matching keys into LDS, one per thread from here on (16 times fewer
            // ballots per bit); their order does not matter for counting
            uint32_t mine = 0;
#pragma unroll
            for (int q = 0; q < kSelPer; ++q) mine += (valid[q] && (key[q] & mask) == prefix) ? 1u : 0u;
            uint32_t incl = mine;                // inclusive scan over the wavefront's lanes
            for (int d = 1; d < 64; d <<= 1) {
                const uint32_t up = (uint32_t)__shfl_up((int)incl, d, 64);
                if (lane >= (uint32_t)d) incl += up;
            }
            if (lane == 63) wsum[0][wave] = incl;
            __syncthreads();
            uint32_t slot = incl - mine;
            for (uint32_t w = 0; w < wave; ++w) slot += wsum[0][w];
#pragma unroll
            for (int q = 0; q < kSelPer; ++q)
                if (valid[q] && (key[q] & mask) == prefix) cand[slot++] = key[q];
            __syncthreads();
            ncand = act;
            ckey = tid < ncand ? cand[tid] : 0u;
            compact = true;
        }
        uint32_t c0 = 0;
        if (compact) {
            c0 = (uint32_t)__popcll(__ballot(tid < ncand && !(ckey & bit) && (ckey & mask) == prefix));
        } else {
#pragma unroll
            for (int q = 0; q < kSelPer; ++q)
                c0 += (uint32_t)__popcll(__ballot(valid[q] && (key[q] & mask) == prefix && !(key[q] & bit)));
        }
        const uint32_t zeros = wg_sum(c0, 1 + (par ^= 1));   // two buffers in turn: one barrier per counted bit
        if (kk > zeros) { prefix |= bit; kk -= zeros; act -= zeros; } else act = zeros;
        mask |= bit;
    }
    // prefix is T; kk of the keys equal to T are pruned: the first ones by position
    uint32_t eq_wave = 0, eq_lower = 0;          // equal keys in the wavefront / in its lower lanes
#pragma unroll
    for (int q = 0; q < kSelPer; ++q) {
        const unsigned long long m = __ballot(valid[q] && key[q] == prefix);
        eq_wave += (uint32_t)__popcll(m);
        eq_lower += __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
    }
    __syncthreads();                             // the last wg_sum's readers are done with wsum[0]
    if (lane == 0) wsum[0][wave] = eq_wave;
    __syncthreads();
    uint32_t rank = eq_lower;
    for (uint32_t w = 0; w < wave; ++w) rank += wsum[0][w];
    uint32_t flags[kSelPer / 4] = {};            // keep flags, one byte each
#pragma unroll
    for (int q = 0; q < kSelPer; ++q) {
        const bool eq = valid[q] && key[q] == prefix;
        const bool pruned = key[q] < prefix || (eq && rank < kk);
        rank += eq ? 1u : 0u;
        flags[q >> 2] |= (pruned ? 0u : 1u) << (8 * (q & 3));
        if (!vec && valid[q]) keep[base + i0 + q] = pruned ? 0 : 1;
    }
    if (vec && valid[0]) *(uint4 *)(keep + base + i0) = make_uint4(flags[0], flags[1], flags[2], flags[3]);
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
    static const char project_user = 0;                    // this entry point as a user of workspaces
    workspace_changed_hands(d_ws, &project_user);
    const uint32_t R = (uint32_t)rows, C = (uint32_t)cols, BR = (uint32_t)br, BC = (uint32_t)bc;
    const uint32_t NBR = (R + BR - 1) / BR, NBC = (C + BC - 1) / BC;
    const ProjectLayout L = project_layout(rows, cols, br, bc);
    uint8_t *ws = (uint8_t *)d_ws;
    uint32_t *keys_r = (uint32_t *)(ws + L.keys_r), *keys_c = (uint32_t *)(ws + L.keys_c);
    uint8_t *keep_r = ws + L.keep_r, *keep_c = ws + L.keep_c;
    hipStream_t st = (hipStream_t)stream;
    hipError_t e = hipSuccess;
    {
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
        hipLaunchKernelGGL(select_kernel, dim3(NBC), dim3(1024), 0, st, keys_r, keep_r, R, prune_count(rows, rate));
        hipLaunchKernelGGL(col_segment_keys_kernel, dim3((C + 255) / 256, NBR), dim3(256), 0, st, d_W, ld, R, C, BR, BC, keep_r, keys_c);
        hipLaunchKernelGGL(select_kernel, dim3(NBR), dim3(1024), 0, st, keys_c, keep_c, C, prune_count(cols, rate));
        // float4 accesses need 16-byte aligned rows on both sides (and flag words at multiples of 4)
        const bool vec4 = C % 4 == 0 && ld % 4 == 0 && ldz % 4 == 0 && (uintptr_t)d_W % 16 == 0 && (uintptr_t)d_Z % 16 == 0;
        hipLaunchKernelGGL(masked_copy_kernel, dim3((C + 255) / 256, (R + kMaskedCopyRows - 1) / kMaskedCopyRows), dim3(256), 0, st,
                           d_W, ld, d_Z, ldz, R, C, BR, BC, keep_r, keep_c, vec4);
        e = hipGetLastError();
    }
    if (e != hipSuccess) { set_error(std::string("csb_project: ") + hipGetErrorString(e)); return CSB_EDEVICE; }
    return CSB_OK;
}
